// Per-node decode attention for gfx950: each workgroup streams the K/V pages of one chunk of one
// prefix-tree node and one KV head from HBM exactly once and applies them to every request below
// the node (all G query heads of the KV head), writing one partial result (o, lse) per query row.
// The partials of a request's path are combined afterwards by the log-sum-exp merge kernel.
// (Shared prefix KV computed/kept once and reused by every call below it: Section 5, "Proactive
// Cache Management"; results must equal unshared attention: Section 2, "Scope".)
//
// Matrix-core mapping (v_mfma_f32_16x16x32_bf16, one wavefront):
//   S^T = K * Q^T   A = 16 tokens x 32 dims of K, B = 32 dims x 16 query rows, D[token][row]
//   O^T = V^T * P^T A = 16 dims x 32 tokens of V^T, B = 32 tokens x 16 query rows, D[dim][row]
// A lane of D holds four consecutive M indices of one query row, which is exactly the shape a B
// operand wants (eight consecutive K indices of one column) once the token order of the two score
// tiles is interleaved, so probabilities go from the first product to the second in registers.
// The pool's block format (K in 64-byte dimension chunks, V dimension-major) makes every operand
// a 16-byte load and every wavefront load a run of whole cache lines.
#include "hkv_device.h"

namespace hkv {

namespace {

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kORow = kHeadDim + 4;  // padded LDS row: 16 rows x 132 floats do not collide in banks

template <int DT>
struct Traits;
template <>
struct Traits<0> {  // bf16 pool
    static constexpr int kTokBlock = 32;  // tokens per wavefront step
    static constexpr int kBlockBytes = kBlockElems * 2;
};
template <>
struct Traits<1> {  // fp8 e4m3 pool
    static constexpr int kTokBlock = 64;
    static constexpr int kBlockBytes = kBlockElems;
};

struct Frags {
    u32x4 k[8];
    u32x4 v[8];
    float ksc, vsc;  // fp8 only
};

struct WaveState {
    f32x4 o[8];  // O^T accumulators: d = 16*dt + 4*g + i, row = lane % 16
    float m;     // running row maximum of the raw (unscaled by log2e) scores
    float l;     // this lane's share of the row sum
};

template <int DT>
__device__ __forceinline__ void load_block(Frags &f, const DecodeLaunch &a, const DecodeItem &it, int blk, int lane) {
    constexpr int kPagesPerBlock = Traits<DT>::kTokBlock / kPage;
    const int m = lane & 15, g = lane >> 4;
    const int last_page = (it.n_tokens - 1) >> 4;
    const char *kb = static_cast<const char *>(a.pool.k_pages);
    const char *vb = static_cast<const char *>(a.pool.v_pages);
    const size_t head_off = (size_t)it.kv_head * Traits<DT>::kBlockBytes;
    const size_t page_stride = (size_t)a.pool.num_kv_heads * Traits<DT>::kBlockBytes;
    if constexpr (DT == 0) {
        // score tile a holds tokens 8*(m/4) + m%4, tile b the same + 4 (of the 32-token block)
        const int pk = min(blk * kPagesPerBlock + (m >> 3), last_page);
        const int pv = min(blk * kPagesPerBlock + (g >> 1), last_page);
        const int idk = a.pages[it.page_off + pk];
        const int idv = a.pages[it.page_off + pv];
        const int slot_a = ((m >> 2) & 1) * 8 + (m & 3);
        const char *kp = kb + (size_t)idk * page_stride + head_off + slot_a * 64 + g * 16;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            f.k[ks] = ld16(kp + ks * 1024);
            f.k[4 + ks] = ld16(kp + ks * 1024 + 4 * 64);
        }
        const char *vp = vb + (size_t)idv * page_stride + head_off + m * 32 + (g & 1) * 16;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) f.v[dt] = ld16(vp + dt * 16 * 32);
    } else {
        // score tile (s, h) holds tokens 16*(m/4) + 8*s + 4*h + m%4 (of the 64-token block)
        const int pk = min(blk * kPagesPerBlock + (m >> 2), last_page);
        const int pv = min(blk * kPagesPerBlock + g, last_page);
        const int idk = a.pages[it.page_off + pk];
        const int idv = a.pages[it.page_off + pv];
        const char *kp = kb + (size_t)idk * page_stride + head_off + (m & 3) * 64 + g * 16;
#pragma unroll
        for (int t4 = 0; t4 < 4; ++t4)
#pragma unroll
            for (int ks2 = 0; ks2 < 2; ++ks2) f.k[t4 * 2 + ks2] = ld16(kp + ks2 * 1024 + t4 * 4 * 64);
        const char *vp = vb + (size_t)idv * page_stride + head_off + m * 16;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) f.v[dt] = ld16(vp + dt * 16 * 16);
        f.ksc = a.pool.k_scale[(size_t)idv * a.pool.num_kv_heads + it.kv_head];
        f.vsc = a.pool.v_scale[(size_t)idv * a.pool.num_kv_heads + it.kv_head];
    }
}

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16x8 zero_bf16_from(bf16x8 v, int first_bad) {
    u32x4 w = __builtin_bit_cast(u32x4, v);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        uint32_t keep = (2 * j + 1 < first_bad) ? 0xFFFFFFFFu : (2 * j < first_bad) ? 0x0000FFFFu : 0u;
        w[j] &= keep;
    }
    return as_bf16x8(w);
}

// One wavefront step over kTokBlock tokens.  qf: the wavefront's Q^T operands.  c = scale*log2(e).
template <int DT>
__device__ __forceinline__ void step(WaveState &st, const Frags &f, const bf16x8 (&qf)[4], int blk, int n_tokens,
                                     float c, int lane) {
    constexpr int TB = Traits<DT>::kTokBlock;
    constexpr int NS = TB / 4;  // scores per lane (16 query rows x TB tokens over 64 lanes)
    const int g = lane >> 4;
    float s[NS];
    bf16x8 vfr[NS / 8][8];  // [k-step][dt]
    if constexpr (DT == 0) {
        f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            sa = mfma16(as_bf16x8(f.k[ks]), qf[ks], sa);
            sb = mfma16(as_bf16x8(f.k[4 + ks]), qf[ks], sb);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            s[i] = sa[i];
            s[4 + i] = sb[i];
        }
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) vfr[0][dt] = as_bf16x8(f.v[dt]);
    } else {
#pragma unroll
        for (int t4 = 0; t4 < 4; ++t4) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks2 = 0; ks2 < 2; ++ks2) {
                u32x4 w = f.k[t4 * 2 + ks2];
                acc = mfma16(fp8x8_to_bf16x8(w[0], w[1]), qf[ks2 * 2], acc);
                acc = mfma16(fp8x8_to_bf16x8(w[2], w[3]), qf[ks2 * 2 + 1], acc);
            }
            // tile t4 = 2*s + h: tokens 16*g + 8*s + 4*h + i  ->  lane-local index 4*t4 + i
#pragma unroll
            for (int i = 0; i < 4; ++i) s[t4 * 4 + i] = acc[i] * f.ksc;
        }
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            vfr[0][dt] = fp8x8_to_bf16x8(f.v[dt][0], f.v[dt][1]);
            vfr[1][dt] = fp8x8_to_bf16x8(f.v[dt][2], f.v[dt][3]);
        }
    }
    // lane-local score j belongs to token tok0 + j of the item
    const int tok0 = blk * TB + g * NS;
    if (blk * TB + TB > n_tokens) {  // block reaches past the item's end: hide garbage slots
        const int first_bad = n_tokens - tok0;  // lane-local index of the first invalid token
#pragma unroll
        for (int j = 0; j < NS; ++j)
            if (j >= first_bad) s[j] = -INFINITY;
#pragma unroll
        for (int ks = 0; ks < NS / 8; ++ks)
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) vfr[ks][dt] = zero_bf16_from(vfr[ks][dt], first_bad - 8 * ks);
    }
    float mx = s[0];
#pragma unroll
    for (int j = 1; j < NS; ++j) mx = fmaxf(mx, s[j]);
    mx = rows_max(mx);
    const float m_new = fmaxf(st.m, mx);
    const float mc = m_new * c;
    const float alpha = fast_exp2(st.m * c - mc);
    float p[NS];
    float sum = 0.f;
#pragma unroll
    for (int j = 0; j < NS; ++j) {
        p[j] = fast_exp2(__builtin_fmaf(s[j], c, -mc));
        sum += p[j];
    }
    st.l = st.l * alpha + sum;
    st.m = m_new;
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f)) {
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) st.o[dt] *= alpha;
    }
    const float vs = (DT == 0) ? 1.0f : f.vsc;
#pragma unroll
    for (int ks = 0; ks < NS / 8; ++ks) {
        u32x4 pw;
#pragma unroll
        for (int j = 0; j < 4; ++j) pw[j] = pack_bf16(p[ks * 8 + 2 * j] * vs, p[ks * 8 + 2 * j + 1] * vs);
        const bf16x8 pb = as_bf16x8(pw);
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) st.o[dt] = mfma16(vfr[ks][dt], pb, st.o[dt]);
    }
}

template <int DT>
__global__ __launch_bounds__(kThreads, 2) void decode_node_kernel(DecodeLaunch a) {
    __shared__ float sO[kWaves][16][kORow];
    __shared__ float sM[kWaves][16];
    __shared__ float sL[kWaves][16];

    const DecodeItem it = a.items[blockIdx.x];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 15, g = lane >> 4;
    const int G = a.num_q_heads / a.pool.num_kv_heads;
    const int rows = it.n_req * G;
    const int n_rt = rows <= 16 ? 1 : rows <= 32 ? 2 : 4;  // 16-row tiles, one or more wavefronts each
    const int n_ts = kWaves / n_rt;                         // wavefronts sharing a row tile split the tokens
    const int rt = wave % n_rt, ts = wave / n_rt;
    const float c = a.scale * kLog2e;

    // Q^T operands of this wavefront's 16 rows; rows past the item's end are zero
    bf16x8 qf[4];
    {
        const int row = rt * 16 + col;
        u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < 4; ++i) qf[i] = as_bf16x8(z);
        if (row < rows) {
            const int req = a.node_req_idx[it.req_off + row / G];
            const int head = it.kv_head * G + row % G;
            const char *qp = static_cast<const char *>(a.q) + ((size_t)req * a.num_q_heads + head) * (kHeadDim * 2);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                // bf16 pool: k-step i covers dims 32*i + 8*g ..; fp8 pool: k-step (i/2, i%2) covers 64*(i/2) + 16*g + 8*(i%2) ..
                const int d0 = (DT == 0) ? 32 * i + 8 * g : 64 * (i >> 1) + 16 * g + 8 * (i & 1);
                qf[i] = as_bf16x8(ld16(qp + d0 * 2));
            }
        }
    }

    WaveState st;
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) st.o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    st.m = -INFINITY;
    st.l = 0.f;

    constexpr int TB = Traits<DT>::kTokBlock;
    const int n_blk = (it.n_tokens + TB - 1) / TB;
    int b = ts;
    if (b < n_blk) {
        Frags fa, fb;
        load_block<DT>(fa, a, it, b, lane);
        for (;;) {
            if (b + n_ts < n_blk) load_block<DT>(fb, a, it, b + n_ts, lane);
            step<DT>(st, fa, qf, b, it.n_tokens, c, lane);
            b += n_ts;
            if (b >= n_blk) break;
            if (b + n_ts < n_blk) load_block<DT>(fa, a, it, b + n_ts, lane);
            step<DT>(st, fb, qf, b, it.n_tokens, c, lane);
            b += n_ts;
            if (b >= n_blk) break;
        }
    }

    // combine the wavefronts that split the tokens of a row tile, normalise, write the partials
    const float l_row = rows_sum(st.l);
#pragma unroll
    for (int dt = 0; dt < 8; ++dt)
        *reinterpret_cast<f32x4 *>(&sO[wave][col][16 * dt + 4 * g]) = st.o[dt];
    if (g == 0) {
        sM[wave][col] = st.m;
        sL[wave][col] = l_row;
    }
    __syncthreads();
    for (int idx = tid; idx < rows * kHeadDim; idx += kThreads) {
        const int row = idx >> 7, d = idx & 127;
        const int r_t = row >> 4, r_c = row & 15;
        float M = -INFINITY;
        for (int t = 0; t < n_ts; ++t) M = fmaxf(M, sM[t * n_rt + r_t][r_c]);
        float L = 0.f, acc = 0.f;
        for (int t = 0; t < n_ts; ++t) {
            const int w = t * n_rt + r_t;
            const float wgt = fast_exp2((sM[w][r_c] - M) * c);
            L += sL[w][r_c] * wgt;
            acc += sO[w][r_c][d] * wgt;
        }
        a.o_parts[(size_t)(it.part_base + row) * kHeadDim + d] = acc / L;
        if (d == 0) a.lse_parts[it.part_base + row] = (M * c + fast_log2(L)) * kLn2;
    }
}

}  // namespace

hipError_t launch_decode(const DecodeLaunch &a, hipStream_t s) {
    if (a.n_items <= 0) return hipSuccess;
    if (a.pool.dtype == 0)
        hipLaunchKernelGGL(decode_node_kernel<0>, dim3(a.n_items), dim3(kThreads), 0, s, a);
    else
        hipLaunchKernelGGL(decode_node_kernel<1>, dim3(a.n_items), dim3(kThreads), 0, s, a);
    return hipGetLastError();
}

}  // namespace hkv
