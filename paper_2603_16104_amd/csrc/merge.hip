// Log-sum-exp combine of partial attention results (one wavefront per output row).
//   lse = ln sum_n exp(lse_n),  out = sum_n exp(lse_n - lse) * o_n
// A partial with lse = -inf is skipped without reading its o (which may hold anything); a row
// without finite partials gives out = 0, lse = -inf.
#include "hkv_device.h"

namespace hkv {

namespace {

constexpr int kRowsPerBlock = 4;

template <int OUT_DT>
__global__ __launch_bounds__(64 * kRowsPerBlock) void lse_merge_kernel(const float *__restrict__ o_parts,
                                                                        const float *__restrict__ lse_parts,
                                                                        const int32_t *__restrict__ row_indptr,
                                                                        const int32_t *__restrict__ part_idx,
                                                                        int32_t n_rows, void *__restrict__ out,
                                                                        float *__restrict__ lse_out) {
    const int row = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (row >= n_rows) return;
    const int beg = row_indptr[row], end = row_indptr[row + 1];
    float M = -INFINITY;
    for (int k = beg; k < end; ++k) M = fmaxf(M, lse_parts[part_idx[k]]);
    float acc0 = 0.f, acc1 = 0.f, z = 0.f;
    if (M != -INFINITY) {
        for (int k = beg; k < end; ++k) {
            const int n = part_idx[k];
            const float ls = lse_parts[n];
            if (ls == -INFINITY) continue;
            const float w = fast_exp2((ls - M) * kLog2e);
            const float2 o = *reinterpret_cast<const float2 *>(o_parts + (size_t)n * kHeadDim + 2 * lane);
            z += w;
            acc0 = __builtin_fmaf(w, o.x, acc0);
            acc1 = __builtin_fmaf(w, o.y, acc1);
        }
        const float inv = 1.0f / z;
        acc0 *= inv;
        acc1 *= inv;
    }
    if (OUT_DT == 0) {
        reinterpret_cast<uint32_t *>(out)[(size_t)row * (kHeadDim / 2) + lane] = pack_bf16(acc0, acc1);
    } else {
        reinterpret_cast<float2 *>(out)[(size_t)row * (kHeadDim / 2) + lane] = make_float2(acc0, acc1);
    }
    if (lse_out && lane == 0) lse_out[row] = (M == -INFINITY) ? -INFINITY : M + fast_log2(z) * kLn2;
}

}  // namespace

hipError_t launch_lse_merge(const float *o_parts, const float *lse_parts, const int32_t *row_indptr,
                            const int32_t *part_idx, int32_t n_rows, void *out, int32_t out_dtype, float *lse_out,
                            hipStream_t s) {
    if (n_rows <= 0) return hipSuccess;
    dim3 grid((n_rows + kRowsPerBlock - 1) / kRowsPerBlock), block(64 * kRowsPerBlock);
    if (out_dtype == 0)
        hipLaunchKernelGGL(lse_merge_kernel<0>, grid, block, 0, s, o_parts, lse_parts, row_indptr, part_idx, n_rows,
                           out, lse_out);
    else
        hipLaunchKernelGGL(lse_merge_kernel<2>, grid, block, 0, s, o_parts, lse_parts, row_indptr, part_idx, n_rows,
                           out, lse_out);
    return hipGetLastError();
}

}  // namespace hkv
