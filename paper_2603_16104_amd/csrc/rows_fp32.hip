// Full-precision path for fp32 pools: plain softmax attention of every query row over its request's
// block table, all arithmetic in fp32 on the vector ALUs (no matrix cores, no bf16 rounding anywhere),
// so that fp32 inputs meet the 1e-4 bound.  One wavefront per (query token, query head); nothing is
// shared between requests here: this path is for checking and for callers that need the precision,
// not a throughput path.  (Same definition as everywhere: Section 2, "Scope": the result equals plain
// attention over the request's whole key/value sequence.)
//
// fp32 block format: K in 64-byte dimension chunks of 16 floats, chunk-major then slot
// ((d / 16) * 256 + slot * 16 + d % 16); V dimension-major (d * 16 + slot).
#include "hkv_device.h"

namespace hkv {

namespace {

constexpr int kRowWaves = 4;

__device__ __forceinline__ float wave_max_f(float v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum_f(float v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

__global__ __launch_bounds__(64 * kRowWaves) void rows_fp32_kernel(RowsLaunch a) {
    __shared__ float sQ[kRowWaves][kHeadDim];
    __shared__ float sP[kRowWaves][64];
    __shared__ int sPage[kRowWaves][4];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const long row = (long)blockIdx.x * kRowWaves + wave;
    const bool live = row < (long)a.n_q_tokens * a.num_q_heads;
    const int tq = live ? (int)(row / a.num_q_heads) : 0, h = live ? (int)(row % a.num_q_heads) : 0;
    const int G = a.num_q_heads / a.pool.num_kv_heads, kvh = h / G;
    const int req = a.row_req[tq];
    const int len = live ? a.row_len[tq] : 0;  // keys this query token sees
    const int32_t *bt = a.block_table + (size_t)req * a.max_pages;
    const float *K = static_cast<const float *>(a.pool.k_pages), *V = static_cast<const float *>(a.pool.v_pages);
    const float *qp = a.q + ((size_t)tq * a.num_q_heads + h) * kHeadDim;
    sQ[wave][lane] = live ? qp[lane] : 0.f;
    sQ[wave][64 + lane] = live ? qp[64 + lane] : 0.f;
    __syncthreads();
    float m = -INFINITY, l = 0.f, acc0 = 0.f, acc1 = 0.f;  // this lane owns dims 2*lane, 2*lane + 1
    // The trip count differs between the wavefronts of a workgroup, so nothing below synchronises across
    // them: sP and sPage are per wavefront, and LDS operations of one wavefront execute in order.
    for (int t0 = 0; t0 < len; t0 += 64) {
        const int t = t0 + lane;
        const bool valid = t < len;
        float s = -INFINITY;
        if (valid) {
            const size_t blk = ((size_t)bt[t >> 4] * a.pool.num_kv_heads + kvh) * kBlockElems;
            const float *kp = K + blk + (t & 15) * 16;
            float dot = 0.f;
#pragma unroll
            for (int c = 0; c < 8; ++c) {
#pragma unroll
                for (int j4 = 0; j4 < 4; ++j4) {
                    const f32x4 kv = *reinterpret_cast<const f32x4 *>(kp + c * 256 + 4 * j4);
#pragma unroll
                    for (int j = 0; j < 4; ++j) dot = __builtin_fmaf(sQ[wave][c * 16 + 4 * j4 + j], kv[j], dot);
                }
            }
            s = dot * a.scale;
        }
        const float m_new = fmaxf(m, wave_max_f(s));  // finite: the step holds at least one valid key
        const float p = valid ? __expf(s - m_new) : 0.f;
        const float alpha = __expf(m - m_new);         // 0 on the first step (m = -inf)
        l = l * alpha + wave_sum_f(p);
        acc0 *= alpha;
        acc1 *= alpha;
        m = m_new;
        sP[wave][lane] = p;
        if (lane < 4) sPage[wave][lane] = (t0 + 16 * lane < len) ? bt[(t0 >> 4) + lane] : -1;
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int pg = 0; pg < 4; ++pg) {
            const int page = sPage[wave][pg];
            if (page < 0) continue;  // uniform
            const float *vp = V + ((size_t)page * a.pool.num_kv_heads + kvh) * kBlockElems + (2 * lane) * 16;
#pragma unroll
            for (int j4 = 0; j4 < 4; ++j4) {
                const f32x4 v0 = *reinterpret_cast<const f32x4 *>(vp + 4 * j4);
                const f32x4 v1 = *reinterpret_cast<const f32x4 *>(vp + 16 + 4 * j4);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float pj = sP[wave][pg * 16 + 4 * j4 + j];
                    if (pj != 0.f) {  // slots past the sequence end may hold anything (NaN included)
                        acc0 = __builtin_fmaf(pj, v0[j], acc0);
                        acc1 = __builtin_fmaf(pj, v1[j], acc1);
                    }
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
    if (!live) return;
    float *op = a.out + ((size_t)tq * a.num_q_heads + h) * kHeadDim;
    const float inv = l > 0.f ? 1.0f / l : 0.f;  // a row without keys gives out = 0, lse = -inf
    op[2 * lane] = acc0 * inv;
    op[2 * lane + 1] = acc1 * inv;
    if (a.lse_out && lane == 0) a.lse_out[(size_t)tq * a.num_q_heads + h] = l > 0.f ? m + __logf(l) : -INFINITY;
}

// fp32 source tokens -> fp32 block format, one thread per element
__global__ __launch_bounds__(256) void pool_write_fp32_kernel(PoolWriteLaunch a) {
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    const long n = (long)a.n_tokens * a.num_kv_heads * kHeadDim;
    if (i >= n) return;
    const int d = (int)(i % kHeadDim), h = (int)((i / kHeadDim) % a.num_kv_heads), t = (int)(i / ((long)kHeadDim * a.num_kv_heads));
    const int pos = a.first_slot + t, page = a.page_ids[pos >> 4], slot = pos & 15;
    const size_t blk = ((size_t)page * a.num_kv_heads + h) * kBlockElems;
    static_cast<float *>(a.k_pages)[blk + (d >> 4) * 256 + slot * 16 + (d & 15)] = static_cast<const float *>(a.k_src)[i];
    static_cast<float *>(a.v_pages)[blk + d * 16 + slot] = static_cast<const float *>(a.v_src)[i];
}

}  // namespace

hipError_t launch_rows_fp32(const RowsLaunch &a, hipStream_t s) {
    const long rows = (long)a.n_q_tokens * a.num_q_heads;
    if (rows <= 0) return hipSuccess;
    hipLaunchKernelGGL(rows_fp32_kernel, dim3((unsigned)((rows + kRowWaves - 1) / kRowWaves)), dim3(64 * kRowWaves), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_pool_write_fp32(const PoolWriteLaunch &a, hipStream_t s) {
    const long n = (long)a.n_tokens * a.num_kv_heads * kHeadDim;
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(pool_write_fp32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace hkv
