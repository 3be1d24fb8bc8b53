// Scatter of new tokens' K/V into the pool's block format (one workgroup per touched page and KV
// head).  bf16 pools: plain re-ordering.  fp8 pools: per-block amax, scale = amax/448, codes =
// round-to-nearest-even(x / scale) saturated to +-448 (OCP e4m3), all in float.  A block that is
// continued (the call starts at first_slot > 0 of its first page) keeps a running scale:
// scale' = max(scale, amax_new/448); when the scale grows, the codes already in the slots below
// first_slot are re-encoded as RNE(value(code) * scale / scale'); the scale never shrinks.
// (The "compute a prefix's KV once and keep it in GPU memory" step of Section 5, "Proactive Cache
// Management", seen from the pool.)
// Also here, all small: the one-token-per-sequence form of the writer for decode steps, whole-page
// copies (copy-on-write), the fp8 -> bf16 pre-pass of prefill over fp8 pools, the copy kernel that
// replaces small host-to-device DMA copies, and the in-place update of a growing decode plan.
#include <algorithm>

#include "hkv_device.h"

namespace hkv {

namespace {

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}

__device__ __forceinline__ uint32_t quant4(float a, float b, float c, float d, float scale) {
    auto q = [scale](float x) { return fminf(fmaxf(x / scale, -448.0f), 448.0f); };
    int p = 0;
    p = __builtin_amdgcn_cvt_pk_fp8_f32(q(a), q(b), p, false);
    p = __builtin_amdgcn_cvt_pk_fp8_f32(q(c), q(d), p, true);
    return (uint32_t)p;
}

// One workgroup's work.  single: one token per block (source row pi goes to slot one_slot of block
// `page`) instead of a run of tokens over consecutive blocks.
template <int DT>
__device__ __forceinline__ void pool_write_block(const PoolWriteLaunch &a, const int page, const bool single,
                                                 const int one_slot) {
    __shared__ uint16_t sV[kPage][kHeadDim + 8];
    __shared__ float sRed[2][4];
    __shared__ float sScale[2], sOld[2];

    const int pi = blockIdx.x, h = blockIdx.y;
    const int tid = threadIdx.x;
    const int slot = tid >> 4, d0 = (tid & 15) * 8;
    const int tok = single ? pi : pi * kPage + slot - a.first_slot;  // source row of this thread's slot
    const bool valid = single ? slot == one_slot : (tok >= 0 && tok < a.n_tokens);
    const size_t blk = ((size_t)page * a.num_kv_heads + h) * kBlockElems;

    u32x4 kw = {0u, 0u, 0u, 0u}, vw = {0u, 0u, 0u, 0u};
    if (valid) {
        const size_t src = (((size_t)tok * a.num_kv_heads + h) * kHeadDim + d0) * 2;
        kw = ld16(static_cast<const char *>(a.k_src) + src);
        vw = ld16(static_cast<const char *>(a.v_src) + src);
    }
    *reinterpret_cast<u32x4 *>(&sV[slot][d0]) = vw;

    // which slots of this page does the call write?  (contiguous range)
    const int s_lo = single ? one_slot : max(0, a.first_slot - pi * kPage);
    const int s_hi = single ? one_slot + 1 : min(kPage, a.first_slot + a.n_tokens - pi * kPage);  // exclusive

    if (DT == 0) {
        if (valid) {
            uint16_t *kdst = static_cast<uint16_t *>(a.k_pages) + blk + (d0 >> 5) * (kPage * 32) + slot * 32 + (d0 & 31);
            *reinterpret_cast<u32x4 *>(kdst) = kw;
        }
        __syncthreads();
        const int d = tid >> 1, half = tid & 1;
        uint16_t *vdst = static_cast<uint16_t *>(a.v_pages) + blk + d * kPage + half * 8;
        if (s_lo <= half * 8 && s_hi >= half * 8 + 8) {
            u32x4 w;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                w[j] = (uint32_t)sV[half * 8 + 2 * j][d] | ((uint32_t)sV[half * 8 + 2 * j + 1][d] << 16);
            *reinterpret_cast<u32x4 *>(vdst) = w;
        } else {
            for (int j = 0; j < 8; ++j) {
                const int sl = half * 8 + j;
                if (sl >= s_lo && sl < s_hi) vdst[j] = sV[sl][d];
            }
        }
    } else {
        float kf[8], vf[8];
        float ka = 0.f, va = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            kf[2 * j] = __uint_as_float(kw[j] << 16);
            kf[2 * j + 1] = __uint_as_float(kw[j] & 0xFFFF0000u);
            vf[2 * j] = __uint_as_float(vw[j] << 16);
            vf[2 * j + 1] = __uint_as_float(vw[j] & 0xFFFF0000u);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            ka = fmaxf(ka, fabsf(kf[j]));
            va = fmaxf(va, fabsf(vf[j]));
        }
        ka = wave_max(ka);
        va = wave_max(va);
        if ((tid & 63) == 0) {
            sRed[0][tid >> 6] = ka;
            sRed[1][tid >> 6] = va;
        }
        __syncthreads();
        const bool append = s_lo > 0;  // slots below s_lo of this block hold codes of an earlier call
        if (tid < 2) {
            const float am = fmaxf(fmaxf(sRed[tid][0], sRed[tid][1]), fmaxf(sRed[tid][2], sRed[tid][3]));
            float *scales = tid ? a.v_scale : a.k_scale;
            float sc, old = 0.f;
            if (!append) {
                sc = am > 0.f ? am / 448.0f : 1.0f;
            } else {
                old = scales[(size_t)page * a.num_kv_heads + h];
                const float cand = am > 0.f ? am / 448.0f : 0.f;
                sc = old >= cand ? old : cand;  // an unset (NaN) old scale gives cand
                if (!(sc > 0.f)) sc = 1.0f;
            }
            sScale[tid] = sc;
            sOld[tid] = old;
            scales[(size_t)page * a.num_kv_heads + h] = sc;
        }
        __syncthreads();
        const float ksc = sScale[0], vsc = sScale[1];
        const bool k_grew = append && ksc > sOld[0], v_grew = append && vsc > sOld[1];
        auto reencode4 = [](uint32_t w, float old, float sc) {  // four codes: value * old / sc, rounded again
            const auto lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false), hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true);
            return quant4(lo[0] * old, lo[1] * old, hi[0] * old, hi[1] * old, sc);
        };
        if (k_grew && slot < s_lo) {
            uint8_t *kdst = static_cast<uint8_t *>(a.k_pages) + blk + (d0 >> 6) * (kPage * 64) + slot * 64 + (d0 & 63);
            u32x2 c = *reinterpret_cast<u32x2 *>(kdst);
            c[0] = reencode4(c[0], sOld[0], ksc);
            c[1] = reencode4(c[1], sOld[0], ksc);
            *reinterpret_cast<u32x2 *>(kdst) = c;
        }
        if (valid) {
            u32x2 c;
            c[0] = quant4(kf[0], kf[1], kf[2], kf[3], ksc);
            c[1] = quant4(kf[4], kf[5], kf[6], kf[7], ksc);
            uint8_t *kdst = static_cast<uint8_t *>(a.k_pages) + blk + (d0 >> 6) * (kPage * 64) + slot * 64 + (d0 & 63);
            *reinterpret_cast<u32x2 *>(kdst) = c;
        }
        const int d = tid >> 1, half = tid & 1;
        float x[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = bf16_bits_to_float(sV[half * 8 + j][d]);
        u32x2 c;
        c[0] = quant4(x[0], x[1], x[2], x[3], vsc);
        c[1] = quant4(x[4], x[5], x[6], x[7], vsc);
        uint8_t *vdst = static_cast<uint8_t *>(a.v_pages) + blk + d * kPage + half * 8;
        if (s_lo <= half * 8 && s_hi >= half * 8 + 8) {
            *reinterpret_cast<u32x2 *>(vdst) = c;
        } else {
            u32x2 r = {0u, 0u};  // the earlier codes of these eight slots, re-encoded if the scale grew
            if (v_grew && half * 8 < s_lo) {
                r = *reinterpret_cast<u32x2 *>(vdst);
                r[0] = reencode4(r[0], sOld[1], vsc);
                r[1] = reencode4(r[1], sOld[1], vsc);
            }
            for (int j = 0; j < 8; ++j) {
                const int sl = half * 8 + j;
                if (sl >= s_lo && sl < s_hi)
                    vdst[j] = (uint8_t)(c[j >> 2] >> (8 * (j & 3)));
                else if (v_grew && sl < s_lo)
                    vdst[j] = (uint8_t)(r[j >> 2] >> (8 * (j & 3)));
            }
        }
    }
}

template <int DT>
__global__ __launch_bounds__(256) void pool_write_kernel(PoolWriteLaunch a) {
    const int pi = blockIdx.x;
    pool_write_block<DT>(a, a.page_ids[pi], a.slots != nullptr, a.slots ? a.slots[pi] : 0);
}

// The decode step's append for up to kMaxInlineAppend sequences: block ids and slots travel in the kernel
// arguments, so the call needs no staging buffer, no copy and no event.
template <int DT>
__global__ __launch_bounds__(256) void pool_append_inline_kernel(PoolAppendInline a) {
    const int pi = blockIdx.x;
    pool_write_block<DT>(a.base, a.block[pi], true, a.slot[pi]);
}

// One workgroup per (pair, K or V): copies the page's blocks of all KV heads, 16 bytes per thread and
// step, and (fp8 pools) the page's scales.  Source and destination pages are distinct.
__global__ __launch_bounds__(256) void pool_copy_kernel(PoolCopyLaunch a) {
    const int pair = blockIdx.x, which = blockIdx.y;
    const int elem = a.pool.dtype == 0 ? 2 : a.pool.dtype == 1 ? 1 : 4;
    const size_t page_bytes = (size_t)a.blocks_per_page * a.pool.num_kv_heads * kBlockElems * elem;
    const char *base = static_cast<const char *>(which ? a.pool.v_pages : a.pool.k_pages);
    const uint4 *src = reinterpret_cast<const uint4 *>(base + (size_t)a.src[pair] * page_bytes);
    uint4 *dst = reinterpret_cast<uint4 *>(const_cast<char *>(base) + (size_t)a.dst[pair] * page_bytes);
    for (size_t i = threadIdx.x; i < page_bytes / 16; i += 256) dst[i] = src[i];
    if (a.pool.dtype == 1) {
        float *sc = const_cast<float *>(which ? a.pool.v_scale : a.pool.k_scale);
        const int per_page = a.blocks_per_page * a.pool.num_kv_heads;  // one scale per 16-token block and head
        for (int h = threadIdx.x; h < per_page; h += 256)
            sc[(size_t)a.dst[pair] * per_page + h] = sc[(size_t)a.src[pair] * per_page + h];
    }
}

// One workgroup per (scratch page, KV head): value = code * scale, rounded to bf16 (RNE), written in the
// bf16 block format.  A thread converts 8 consecutive codes of K and of V: in both formats they are 8
// consecutive elements (K: 8 dimensions of one slot inside a 64-byte chunk; V: 8 slots of one dimension).
__global__ __launch_bounds__(256) void pool_dequant_kernel(PoolDequantLaunch a) {
    const int i = blockIdx.x, h = blockIdx.y, tid = threadIdx.x;
    const int page = a.src_pages[i];
    const size_t src_blk = ((size_t)page * a.pool.num_kv_heads + h) * kBlockElems;
    const size_t dst_blk = ((size_t)i * a.pool.num_kv_heads + h) * kBlockElems;
    const float ks = a.pool.k_scale[(size_t)page * a.pool.num_kv_heads + h];
    const float vs = a.pool.v_scale[(size_t)page * a.pool.num_kv_heads + h];
    typedef __attribute__((ext_vector_type(2))) float f32x2;
    auto convert = [](u32x2 w, float sc) {
        u32x4 o;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[j], false), hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[j], true);
            o[2 * j] = pack_bf16(lo[0] * sc, lo[1] * sc);
            o[2 * j + 1] = pack_bf16(hi[0] * sc, hi[1] * sc);
        }
        return o;
    };
    {   // K: fp8 element (slot t, dim d) at (d / 64) * 1024 + t * 64 + d % 64, bf16 at (d / 32) * 512 + t * 32 + d % 32
        const int e = 8 * tid, c = e >> 10, t = (e >> 6) & 15, d = 64 * c + (e & 63);
        const u32x2 w = *reinterpret_cast<const u32x2 *>(static_cast<const uint8_t *>(a.pool.k_pages) + src_blk + e);
        *reinterpret_cast<u32x4 *>(static_cast<uint16_t *>(a.k_dst) + dst_blk + (d >> 5) * 512 + t * 32 + (d & 31)) = convert(w, ks);
    }
    {   // V: element (slot t, dim d) at d * 16 + t in both formats
        const int e = 8 * tid;
        const u32x2 w = *reinterpret_cast<const u32x2 *>(static_cast<const uint8_t *>(a.pool.v_pages) + src_blk + e);
        *reinterpret_cast<u32x4 *>(static_cast<uint16_t *>(a.v_dst) + dst_blk + e) = convert(w, vs);
    }
}

// Plain copy of n16 16-byte pieces; the source may be pinned host memory (read over the host link).
__global__ __launch_bounds__(256) void upload_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void plan_grow_inline_kernel(PlanGrowInline a) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t < a.n_grow) a.items[a.grow_items[t]].n_tokens += 1;
    if (t < a.n_req && a.new_block[t] >= 0) a.pages[a.block_pos[t]] = a.new_block[t];
}

// A decode step's append in one launch: workgroup (r, head) stores request r's new token and lengthens the
// item of that head in the request's leaf (grow_items is [request][head]); head 0 enters a new block id.
template <int DT>
__global__ __launch_bounds__(256) void decode_step_append_kernel(PoolAppendInline w, PlanGrowInline g) {
    const int r = blockIdx.x, h = blockIdx.y;
    pool_write_block<DT>(w.base, w.block[r], true, w.slot[r]);
    if (threadIdx.x == 0) g.items[g.grow_items[r * w.base.num_kv_heads + h]].n_tokens += 1;
    if (threadIdx.x == 1 && h == 0 && g.new_block[r] >= 0) g.pages[g.block_pos[r]] = g.new_block[r];
}

}  // namespace

hipError_t launch_decode_step_append(const PoolAppendInline &w, const PlanGrowInline &g, hipStream_t s) {
    if (w.base.n_pages <= 0) return hipSuccess;
    dim3 grid(w.base.n_pages, w.base.num_kv_heads), block(256);
    if (w.base.dtype == 0)
        hipLaunchKernelGGL(decode_step_append_kernel<0>, grid, block, 0, s, w, g);
    else
        hipLaunchKernelGGL(decode_step_append_kernel<1>, grid, block, 0, s, w, g);
    return hipGetLastError();
}

hipError_t launch_plan_grow_inline(const PlanGrowInline &a, hipStream_t s) {
    const int n = a.n_grow > a.n_req ? a.n_grow : a.n_req;
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(plan_grow_inline_kernel, dim3((n + 255) / 256), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_pool_dequant(const PoolDequantLaunch &a, hipStream_t s) {
    if (a.n_pages <= 0) return hipSuccess;
    hipLaunchKernelGGL(pool_dequant_kernel, dim3(a.n_pages, a.pool.num_kv_heads), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_upload(const void *src, void *dst, size_t bytes, hipStream_t s) {
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    const unsigned blocks = (unsigned)std::min<size_t>((n16 + 255) / 256, 256);
    hipLaunchKernelGGL(upload_kernel, dim3(blocks), dim3(256), 0, s, static_cast<const uint4 *>(src),
                       static_cast<uint4 *>(dst), n16);
    return hipGetLastError();
}

hipError_t launch_pool_copy(const PoolCopyLaunch &a, hipStream_t s) {
    if (a.n <= 0) return hipSuccess;
    hipLaunchKernelGGL(pool_copy_kernel, dim3(a.n, 2), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_pool_append_inline(const PoolAppendInline &a, hipStream_t s) {
    if (a.base.n_pages <= 0) return hipSuccess;
    dim3 grid(a.base.n_pages, a.base.num_kv_heads), block(256);
    if (a.base.dtype == 0)
        hipLaunchKernelGGL(pool_append_inline_kernel<0>, grid, block, 0, s, a);
    else
        hipLaunchKernelGGL(pool_append_inline_kernel<1>, grid, block, 0, s, a);
    return hipGetLastError();
}

hipError_t launch_pool_write(const PoolWriteLaunch &a, hipStream_t s) {
    if (a.n_pages <= 0) return hipSuccess;
    dim3 grid(a.n_pages, a.num_kv_heads), block(256);
    if (a.dtype == 0)
        hipLaunchKernelGGL(pool_write_kernel<0>, grid, block, 0, s, a);
    else
        hipLaunchKernelGGL(pool_write_kernel<1>, grid, block, 0, s, a);
    return hipGetLastError();
}

}  // namespace hkv
