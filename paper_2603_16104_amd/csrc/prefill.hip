// Suffix-only prefill attention for gfx950: the new tokens of a request attend to the cached
// prefix pages plus the causal part of their own suffix, all read through the block table.
// (Section 5, "Token usage": a call processes only the tokens that are not already cached.)
//
// One workgroup (4 wavefronts) owns 256 query rows = 256/G consecutive new tokens x the G query
// heads of one KV head, so every K/V tile staged in LDS is used by all G heads.  Each wavefront
// owns 64 rows (two 32-row tiles) and keeps Q^T and the O^T accumulators in registers; K/V
// stream through LDS in 64-token blocks, double buffered.
//
// Matrix-core mapping (v_mfma_f32_32x32x16_bf16):
//   S^T = K * Q^T   A = 32 tokens x 16 dims (LDS), B = 16 dims x 32 rows (registers)
//   O^T = V^T * P^T A = 32 dims x 16 tokens (LDS), B = 16 tokens x 32 rows (registers)
// The token order of the score tile's M index is permuted (groups of four: 0,2,1,3) so that a lane
// of the result holds eight consecutive tokens of a page per half, i.e. a ready B operand for the
// second product and a 16-byte read of the dimension-major V page for its A operand.
#include "hkv_device.h"

namespace hkv {

namespace {

constexpr int kThreads = 256;
constexpr int kRowsPerGroup = 256;
constexpr int KB = 64;                    // tokens per LDS stage (4 pages)
constexpr int kTileBytes = KB * kHeadDim * 2;  // 16 KiB for K, same for V

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ float half_swap_max(float v) { return fmaxf(v, __shfl_xor(v, 32)); }

__global__ __launch_bounds__(kThreads, 1) void prefill_kernel(PrefillLaunch a) {
    __shared__ __attribute__((aligned(16))) char sK[2][kTileBytes];
    __shared__ __attribute__((aligned(16))) char sV[2][kTileBytes];

    const PrefillTile tl = a.tiles[blockIdx.x];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, h = lane >> 5;
    const int Hq = a.num_q_heads, Hkv = a.pool.num_kv_heads;
    const int G = Hq / Hkv;
    const int tbh = 8 / G;  // 32-token blocks per head inside the workgroup's rows
    const float c = a.scale * kLog2e;

    // the two 32-row tiles of this wavefront
    int head[2], tok[2];  // query head; token index of this lane's row within the tile's new tokens
    bf16x8 qf[2][8];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        const int T = 2 * wave + nt;
        head[nt] = tl.kv_head * G + T / tbh;
        tok[nt] = 32 * (T % tbh) + n;
        const int qrow = tl.q_row0 + min(tok[nt], tl.n_q - 1);
        const char *qp = static_cast<const char *>(a.q) + ((size_t)qrow * Hq + head[nt]) * (kHeadDim * 2);
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) qf[nt][kk] = as_bf16x8(ld16(qp + (16 * kk + 8 * h) * 2));
    }
    // wavefront-uniform: smallest absolute position among this wavefront's rows
    const int wave_min_pos = tl.prefix_len + tl.q_begin + 32 * ((2 * wave) % tbh);

    f32x16 o[2][4];
    float m_run[2], l_run[2];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
#pragma unroll
        for (int dm = 0; dm < 4; ++dm)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[nt][dm][i] = 0.f;
        m_run[nt] = -INFINITY;
        l_run[nt] = 0.f;
    }

    const int kv_end = tl.prefix_len + tl.q_begin + tl.n_q;  // keys any row of the tile can see
    const int n_blk = (kv_end + KB - 1) / KB;
    const int last_page = (tl.kv_len - 1) >> 4;
    const char *kbase = static_cast<const char *>(a.pool.k_pages) + (size_t)tl.kv_head * (kBlockElems * 2);
    const char *vbase = static_cast<const char *>(a.pool.v_pages) + (size_t)tl.kv_head * (kBlockElems * 2);
    const size_t page_stride = (size_t)Hkv * (kBlockElems * 2);
    const int32_t *bt = a.block_table + tl.bt_off;

    // LDS offsets of this thread's 16-byte pieces within a page (bank-conflict swizzles):
    //   K page: [chunk][slot][4 units of 16 B], unit ^= (slot / 4) % 4
    //   V page: [d][2 units of 16 B],            unit ^= (d / 8) % 2
    const int k_slot = (tid & 63) >> 2, k_unit = tid & 3;
    const int k_lds = (tid >> 6) * 1024 + k_slot * 64 + ((k_unit ^ ((k_slot >> 2) & 3)) << 4);
    const int v_d = tid >> 1, v_unit = tid & 1;
    const int v_lds = v_d * 32 + ((v_unit ^ ((v_d >> 3) & 1)) << 4);

    u32x4 kreg[4], vreg[4];
    auto load_global = [&](int blk) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int id = bt[min(blk * 4 + i, last_page)];
            kreg[i] = ld16(kbase + (size_t)id * page_stride + tid * 16);
            vreg[i] = ld16(vbase + (size_t)id * page_stride + tid * 16);
        }
    };
    auto store_lds = [&](int blk, int buf) {
        const bool tail = blk * KB + KB > tl.kv_len;  // block holds slots past the sequence end
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            u32x4 vv = vreg[i];
            if (tail) {  // V of slots past the end may be anything (NaN included): store zeros
                const int t0 = blk * KB + i * 16 + v_unit * 8;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t keep = (t0 + 2 * j + 1 < tl.kv_len) ? 0xFFFFFFFFu
                                          : (t0 + 2 * j < tl.kv_len)   ? 0x0000FFFFu
                                                                       : 0u;
                    vv[j] &= keep;
                }
            }
            *reinterpret_cast<u32x4 *>(&sK[buf][i * 4096 + k_lds]) = kreg[i];
            *reinterpret_cast<u32x4 *>(&sV[buf][i * 4096 + v_lds]) = vv;
        }
    };

    // A-operand LDS offsets of this lane.
    //   K: M index n -> token sigma(n) of the 32-token tile (groups of four permuted 0,2,1,3)
    const int grp = n >> 2;
    const int grp_p = ((grp & 3) == 1) ? grp + 1 : ((grp & 3) == 2) ? grp - 1 : grp;
    const int tau = 4 * grp_p + (n & 3);
    const int ka_page = tau >> 4, ka_slot = tau & 15;
    const int ka_swz = (ka_slot >> 2) & 3;
    const int ka_base = ka_page * 4096 + ka_slot * 64;
    //   V: M index n -> dim 32*dm + n; unit h (slots 8h..8h+7), swizzled by (d/8)%2
    const int va_base = n * 32 + ((h ^ ((n >> 3) & 1)) << 4);

    load_global(0);
    store_lds(0, 0);
    __syncthreads();

    for (int blk = 0; blk < n_blk; ++blk) {
        const int buf = blk & 1;
        const bool more = blk + 1 < n_blk;
        if (more) load_global(blk + 1);

        // ---- S^T = K Q^T for 64 tokens x 64 rows
        f32x16 s[2][2];
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int i = 0; i < 16; ++i) s[nt][mt][i] = 0.f;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                const int unit = 2 * (kk & 1) + h;
                const bf16x8 ka = as_bf16x8(*reinterpret_cast<const u32x4 *>(
                    &sK[buf][mt * 8192 + ka_base + (kk >> 1) * 1024 + ((unit ^ ka_swz) << 4)]));
#pragma unroll
                for (int nt = 0; nt < 2; ++nt) s[nt][mt] = mfma32(ka, qf[nt][kk], s[nt][mt]);
            }

        // ---- online softmax per row; lane-local score (mt, i) is token blk*64 + mt*32 + (i/8)*16 + 8h + i%8
        const bool need_mask = blk * KB + KB - 1 > wave_min_pos;
        bf16x8 pb[2][4];
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            if (need_mask) {
                const int pos = tl.prefix_len + tl.q_begin + tok[nt];  // absolute position of this lane's row
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int t = blk * KB + mt * 32 + (i >> 3) * 16 + 8 * h + (i & 7);
                        if (t > pos) s[nt][mt][i] = -INFINITY;
                    }
            }
            float mx = s[nt][0][0];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[nt][mt][i]);
            mx = half_swap_max(mx);
            const float m_new = fmaxf(m_run[nt], mx);
            const float mc = m_new * c;
            const float alpha = fast_exp2(m_run[nt] * c - mc);
            float sum = 0.f;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                float p[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    p[i] = fast_exp2(__builtin_fmaf(s[nt][mt][i], c, -mc));
                    sum += p[i];
                }
#pragma unroll
                for (int hf = 0; hf < 2; ++hf) {
                    u32x4 w;
#pragma unroll
                    for (int j = 0; j < 4; ++j) w[j] = pack_bf16(p[hf * 8 + 2 * j], p[hf * 8 + 2 * j + 1]);
                    pb[nt][mt * 2 + hf] = as_bf16x8(w);
                }
            }
            l_run[nt] = l_run[nt] * alpha + sum;
            m_run[nt] = m_new;
            if (__builtin_amdgcn_ballot_w64(alpha != 1.0f)) {
#pragma unroll
                for (int dm = 0; dm < 4; ++dm)
#pragma unroll
                    for (int i = 0; i < 16; ++i) o[nt][dm][i] *= alpha;
            }
        }

        // ---- O^T += V^T P^T
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int dm = 0; dm < 4; ++dm) {
                const bf16x8 va = as_bf16x8(
                    *reinterpret_cast<const u32x4 *>(&sV[buf][u * 4096 + dm * 1024 + va_base]));
#pragma unroll
                for (int nt = 0; nt < 2; ++nt) o[nt][dm] = mfma32(va, pb[nt][u], o[nt][dm]);
            }

        if (more) store_lds(blk + 1, buf ^ 1);
        __syncthreads();
    }

    // ---- normalise and store; lane (n, h) holds dims 32*dm + 8*(i/4) + 4*h + i%4 of its row
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        const float l_tot = l_run[nt] + __shfl_xor(l_run[nt], 32);
        if (tok[nt] >= tl.n_q) continue;
        const float inv = 1.0f / l_tot;
        const size_t row = (size_t)(tl.q_row0 + tok[nt]) * Hq + head[nt];
        uint16_t *op = static_cast<uint16_t *>(a.out) + row * kHeadDim;
#pragma unroll
        for (int dm = 0; dm < 4; ++dm)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                u32x2 w;
                w[0] = pack_bf16(o[nt][dm][4 * q4] * inv, o[nt][dm][4 * q4 + 1] * inv);
                w[1] = pack_bf16(o[nt][dm][4 * q4 + 2] * inv, o[nt][dm][4 * q4 + 3] * inv);
                *reinterpret_cast<u32x2 *>(op + 32 * dm + 8 * q4 + 4 * h) = w;
            }
        if (a.lse_out && h == 0) a.lse_out[row] = (m_run[nt] * c + fast_log2(l_tot)) * kLn2;
    }
}

}  // namespace

int prefill_tile_tokens(int group) { return kRowsPerGroup / group; }

hipError_t launch_prefill(const PrefillLaunch &a, hipStream_t s) {
    if (a.n_tiles <= 0) return hipSuccess;
    hipLaunchKernelGGL(prefill_kernel, dim3(a.n_tiles), dim3(kThreads), 0, s, a);
    return hipGetLastError();
}

}  // namespace hkv
