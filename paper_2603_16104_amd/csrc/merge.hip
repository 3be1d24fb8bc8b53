// Log-sum-exp combine of partial attention results (one wavefront per output row).
//   lse = ln sum_n exp(lse_n),  out = sum_n exp(lse_n - lse) * o_n
// A partial with lse = -inf is skipped without reading its o (which may hold anything); a row
// without finite partials gives out = 0, lse = -inf.
#include <hip/hip_ext.h>

#include <type_traits>

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

// Dense variant: row i owns partials i*max_parts + k, k < part_count[i / rows_per_count].  Half a
// wavefront per row (32 lanes x 4 dims); the first kUnroll partials and their lse values are
// requested together, so a row costs one memory round trip after its count (kUnroll is 8, or 16 for
// forests whose paths collect more than 8 partials).
constexpr int kDenseRowsPerBlock = 8;
constexpr int kManyRows = 16384;  // from here on a half wavefront merges four rows

// four consecutive values of a partial, as floats
template <bool PB16>
__device__ __forceinline__ f32x4 load_part4(const void *o_parts, size_t elem) {
    if constexpr (PB16) {  // fp16; the caller applies the partial's factor
        const u32x2 w = *reinterpret_cast<const u32x2 *>(static_cast<const uint16_t *>(o_parts) + elem);
        const uint32_t w0 = w[0], w1 = w[1];  // (a bit cast straight from a vector element reads element 0 for both)
        const f16x2 a = __builtin_bit_cast(f16x2, w0), b = __builtin_bit_cast(f16x2, w1);
        return f32x4{(float)a[0], (float)a[1], (float)b[0], (float)b[1]};
    } else {
        return *reinterpret_cast<const f32x4 *>(static_cast<const float *>(o_parts) + elem);
    }
}

template <int OUT_DT, int kUnroll, bool PB16>
__device__ __forceinline__ void merge_dense_row(const void *__restrict__ o_parts, const float *__restrict__ lse_parts,
                                                const int32_t *__restrict__ part_count, int32_t rows_per_count,
                                                int32_t max_parts, int row, int l, void *__restrict__ out,
                                                float *__restrict__ lse_out, const int32_t *__restrict__ out_rows,
                                                const float *__restrict__ down_parts) {
    const int cnt = min(part_count[row / rows_per_count], max_parts);
    const size_t base = (size_t)row * max_parts;
    const float *lp = lse_parts + base;
    const float *dp = PB16 ? down_parts + base : nullptr;  // fp16 partials: the factor each one is to be multiplied by
    const size_t o0 = base * kHeadDim + 4 * l;  // element index of this lane's four dims in slot 0
    // With few slots per row all of them are requested before the count is known (slots k < max_parts
    // exist for every row; what an unused one holds is never looked at), so the count, the lse values
    // and the partials travel in one round trip instead of two.  With many slots only the used ones
    // are read.
    float ls[kUnroll], ds[kUnroll];
    f32x4 ov[kUnroll];
    if (max_parts <= kUnroll) {
#pragma unroll
        for (int k = 0; k < kUnroll; ++k) {
            const int kc = min(k, max_parts - 1);
            ls[k] = lp[kc];
            ds[k] = PB16 ? dp[kc] : 1.0f;
            ov[k] = load_part4<PB16>(o_parts, o0 + (size_t)kc * kHeadDim);
        }
#pragma unroll
        for (int k = 0; k < kUnroll; ++k)
            if (k >= cnt) ls[k] = -INFINITY;
    } else {
#pragma unroll
        for (int k = 0; k < kUnroll; ++k) {
            ls[k] = -INFINITY;
            ds[k] = 1.0f;
            ov[k] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (k < cnt) {
                ls[k] = lp[k];
                if (PB16) ds[k] = dp[k];
                ov[k] = load_part4<PB16>(o_parts, o0 + (size_t)k * kHeadDim);
            }
        }
    }
    float M = -INFINITY;
#pragma unroll
    for (int k = 0; k < kUnroll; ++k) M = fmaxf(M, ls[k]);
    for (int k = kUnroll; k < cnt; ++k) M = fmaxf(M, lp[k]);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    float z = 0.f;
    if (M != -INFINITY) {
#pragma unroll
        for (int k = 0; k < kUnroll; ++k) {
            if (ls[k] != -INFINITY) {  // an empty partial may hold anything in o
                const float w = fast_exp2((ls[k] - M) * kLog2e);
                z += w;
                acc += ov[k] * (w * ds[k]);
            }
        }
        for (int k = kUnroll; k < cnt; ++k) {
            const float lk = lp[k];
            if (lk == -INFINITY) continue;
            const float w = fast_exp2((lk - M) * kLog2e);
            z += w;
            acc += load_part4<PB16>(o_parts, o0 + (size_t)k * kHeadDim) * (PB16 ? w * dp[k] : w);
        }
        acc *= 1.0f / z;
    }
    const size_t dst = out_rows ? (size_t)out_rows[row / rows_per_count] * rows_per_count + row % rows_per_count : (size_t)row;
    if (OUT_DT == 0) {
        u32x2 w;
        w[0] = pack_bf16(acc[0], acc[1]);
        w[1] = pack_bf16(acc[2], acc[3]);
        reinterpret_cast<u32x2 *>(out)[dst * (kHeadDim / 4) + l] = w;
    } else {
        reinterpret_cast<f32x4 *>(out)[dst * (kHeadDim / 4) + l] = acc;
    }
    if (lse_out && l == 0) lse_out[dst] = (M == -INFINITY) ? -INFINITY : M + fast_log2(z) * kLn2;
}

// kRowsPerLane rows per half wavefront (rows row0, row0 + stride, ...): large batches run four, whose loads the
// compiler issues together, on a quarter of the workgroups.
template <int OUT_DT, int kUnroll, bool PB16, int kRowsPerLane>
__global__ __launch_bounds__(32 * kDenseRowsPerBlock) void lse_merge_dense_kernel(
    const void *__restrict__ o_parts, const float *__restrict__ lse_parts, const int32_t *__restrict__ part_count,
    int32_t rows_per_count, int32_t max_parts, int32_t n_rows, void *__restrict__ out, float *__restrict__ lse_out,
    const int32_t *__restrict__ out_rows, const float *__restrict__ down_parts) {
    const int row0 = (blockIdx.x * kRowsPerLane) * kDenseRowsPerBlock + (threadIdx.x >> 5);
    const int l = threadIdx.x & 31;
#pragma unroll
    for (int r = 0; r < kRowsPerLane; ++r) {
        const int row = row0 + r * kDenseRowsPerBlock;
        if (row < n_rows)
            merge_dense_row<OUT_DT, kUnroll, PB16>(o_parts, lse_parts, part_count, rows_per_count, max_parts, row, l, out,
                                                   lse_out, out_rows, down_parts);
    }
}

}  // namespace

hipError_t launch_lse_merge_dense(const void *o_parts, const float *lse_parts, const int32_t *part_count,
                                  int32_t rows_per_count, int32_t max_parts, int32_t n_rows, void *out,
                                  int32_t out_dtype, float *lse_out, hipStream_t s, hipEvent_t ev_begin,
                                  hipEvent_t ev_end, const int32_t *out_rows, const float *down_parts) {
    if (n_rows <= 0) return hipSuccess;
    const bool many = n_rows >= kManyRows && max_parts <= 8;
    const int per_block = kDenseRowsPerBlock * (many ? 4 : 1);
    dim3 grid((n_rows + per_block - 1) / per_block), block(32 * kDenseRowsPerBlock);
    auto go = [&](auto kernel) {
        hipExtLaunchKernelGGL(kernel, grid, block, 0, s, ev_begin, ev_end, 0, o_parts, lse_parts, part_count,
                              rows_per_count, max_parts, n_rows, out, lse_out, out_rows, down_parts);
    };
    auto pick = [&](auto pb16) {
        constexpr bool PB = decltype(pb16)::value;
        if (many && max_parts <= 2) {
            if (out_dtype == 0)
                go(lse_merge_dense_kernel<0, 2, PB, 4>);
            else
                go(lse_merge_dense_kernel<2, 2, PB, 4>);
        } else if (many) {
            if (out_dtype == 0)
                go(lse_merge_dense_kernel<0, 8, PB, 4>);
            else
                go(lse_merge_dense_kernel<2, 8, PB, 4>);
        } else if (max_parts <= 8) {
            if (out_dtype == 0)
                go(lse_merge_dense_kernel<0, 8, PB, 1>);
            else
                go(lse_merge_dense_kernel<2, 8, PB, 1>);
        } else {
            if (out_dtype == 0)
                go(lse_merge_dense_kernel<0, 16, PB, 1>);
            else
                go(lse_merge_dense_kernel<2, 16, PB, 1>);
        }
    };
    if (down_parts)
        pick(std::true_type{});
    else
        pick(std::false_type{});
    return hipGetLastError();
}

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
