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
//
// The kernel is bound by HBM reads, so the loop is organised around keeping loads in flight:
// page ids come through scalar loads one step ahead, K of step b+1 is requested as soon as the
// first product of step b has consumed the K registers, V of step b+1 as soon as the second
// product has consumed the V registers; nothing in the loop waits for all outstanding loads.
#include <type_traits>

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

// Page ids (and fp8 scales) of one step, wavefront-uniform so that they travel in scalar registers.
template <int DT>
struct StepPages {
    static constexpr int N = Traits<DT>::kTokBlock / kPage;
    int id[N];
    float ksc[N], vsc[N];
};

template <int DT>
__device__ __forceinline__ void load_step_pages(StepPages<DT> &sp, const DecodeLaunch &a, const DecodeItem &it,
                                                int blk, int last_page) {
#pragma unroll
    for (int i = 0; i < StepPages<DT>::N; ++i) {
        sp.id[i] = a.pages[it.page_off + min(blk * StepPages<DT>::N + i, last_page)];
        if constexpr (DT == 1) {
            sp.ksc[i] = a.pool.k_scale[(size_t)sp.id[i] * a.pool.num_kv_heads + it.kv_head];
            sp.vsc[i] = a.pool.v_scale[(size_t)sp.id[i] * a.pool.num_kv_heads + it.kv_head];
        }
    }
}

template <int N>
__device__ __forceinline__ int pick(const int (&v)[N], int sel) {
    int r = v[0];
#pragma unroll
    for (int i = 1; i < N; ++i) r = (sel == i) ? v[i] : r;
    return r;
}
template <int N>
__device__ __forceinline__ float pickf(const float (&v)[N], int sel) {
    float r = v[0];
#pragma unroll
    for (int i = 1; i < N; ++i) r = (sel == i) ? v[i] : r;
    return r;
}

template <int DT>
__global__ __launch_bounds__(kThreads, 2) void decode_node_kernel(DecodeLaunch a) {
    __shared__ float sO[kWaves][16][kORow];
    __shared__ float sM[kWaves][16];
    __shared__ float sL[kWaves][16];

    constexpr int TB = Traits<DT>::kTokBlock;
    constexpr int NS = TB / 4;  // scores per lane (16 query rows x TB tokens over 64 lanes)
    constexpr int BB = Traits<DT>::kBlockBytes;

    const DecodeItem it = a.items[blockIdx.x];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m = lane & 15, g = lane >> 4;
    const int Hkv = a.pool.num_kv_heads;
    const int G = a.num_q_heads / Hkv;
    const int rows = it.n_req * G;
    const int n_rt = rows <= 16 ? 1 : rows <= 32 ? 2 : 4;  // 16-row tiles, one or more wavefronts each
    const int n_ts = kWaves / n_rt;                         // wavefronts sharing a row tile split the tokens
    const int rt = wave % n_rt, ts = wave / n_rt;
    const float c = a.scale * kLog2e;

    // Q^T operands of this wavefront's 16 rows; rows past the item's end are zero
    bf16x8 qf[4];
    {
        const int row = rt * 16 + m;
        u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < 4; ++i) qf[i] = as_bf16x8(z);
        if (row < rows) {
            const int req = a.node_req_idx[it.req_off + row / G];
            const int head = it.kv_head * G + row % G;
            const char *qp = static_cast<const char *>(a.q) + ((size_t)req * a.num_q_heads + head) * (kHeadDim * 2);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                // bf16 pool: k-step i covers dims 32*i + 8*g ..; fp8 pool: k-step (i/2, i%2) covers
                // dims 64*(i/2) + 16*g + 8*(i%2) ..
                const int d0 = (DT == 0) ? 32 * i + 8 * g : 64 * (i >> 1) + 16 * g + 8 * (i & 1);
                qf[i] = as_bf16x8(ld16(qp + d0 * 2));
            }
        }
    }

    // Loop-invariant byte offsets of this lane inside a (page, head) block and the page of the step
    // it reads.  bf16: score tile a holds tokens 8*(m/4) + m%4 of the 32-token step, tile b those + 4;
    // the V operand holds tokens 8g..8g+7.  fp8: score tile t4 holds tokens 16*(m/4) + 4*t4 + m%4 of
    // the 64-token step; the V operand holds the 16 tokens of page g.
    const int k_sel = (DT == 0) ? (m >> 3) : (m >> 2);
    const int v_sel = (DT == 0) ? (g >> 1) : g;
    const uint32_t k_off = (uint32_t)it.kv_head * BB +
                           ((DT == 0) ? (((m >> 2) & 1) * 8 + (m & 3)) * 64 + g * 16 : (m & 3) * 64 + g * 16);
    const uint32_t v_off = (uint32_t)it.kv_head * BB + ((DT == 0) ? m * 32 + (g & 1) * 16 : m * 16);
    const size_t page_stride = (size_t)Hkv * BB;
    const char *kb = static_cast<const char *>(a.pool.k_pages) + k_off;
    const char *vb = static_cast<const char *>(a.pool.v_pages) + v_off;

    f32x4 o[8];  // O^T accumulators: d = 16*dt + 4*g + i, row = lane % 16
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY;  // running maximum of the raw scores of this lane's row
    float l_run = 0.f;        // this lane's share of the row sum

    const int n_blk = (it.n_tokens + TB - 1) / TB;
    const int last_page = (it.n_tokens - 1) >> 4;

    u32x4 kf[8], vf[8];
    auto issue_k = [&](const StepPages<DT> &sp) {
        const char *p = kb + (size_t)pick(sp.id, k_sel) * page_stride;
        if constexpr (DT == 0) {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                kf[ks] = ld16(p + ks * 1024);
                kf[4 + ks] = ld16(p + ks * 1024 + 256);
            }
        } else {
#pragma unroll
            for (int t4 = 0; t4 < 4; ++t4)
#pragma unroll
                for (int ks2 = 0; ks2 < 2; ++ks2) kf[t4 * 2 + ks2] = ld16(p + ks2 * 1024 + t4 * 256);
        }
    };
    auto issue_v = [&](const StepPages<DT> &sp) {
        const char *p = vb + (size_t)pick(sp.id, v_sel) * page_stride;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) vf[dt] = ld16(p + dt * ((DT == 0) ? 512 : 256));
    };

    // One step over TB tokens.  MORE: another step follows, so its K and V are requested as soon as
    // the registers are free; the last step (and only it) may reach past the item's end.
    auto step = [&](auto more_tag, int b, const StepPages<DT> &cur, const StepPages<DT> &nxt) {
        constexpr bool MORE = decltype(more_tag)::value;
        // ---- S^T = K Q^T
        float s[NS];
        if constexpr (DT == 0) {
            f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                sa = mfma16(as_bf16x8(kf[ks]), qf[ks], sa);
                sb = mfma16(as_bf16x8(kf[4 + ks]), qf[ks], sb);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                s[i] = sa[i];
                s[4 + i] = sb[i];
            }
        } else {
            const float ksc = pickf(cur.ksc, g);
#pragma unroll
            for (int t4 = 0; t4 < 4; ++t4) {
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks2 = 0; ks2 < 2; ++ks2) {
                    const u32x4 w = kf[t4 * 2 + ks2];
                    acc = mfma16(fp8x8_to_bf16x8(w[0], w[1]), qf[ks2 * 2], acc);
                    acc = mfma16(fp8x8_to_bf16x8(w[2], w[3]), qf[ks2 * 2 + 1], acc);
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) s[t4 * 4 + i] = acc[i] * ksc;
            }
        }
        if constexpr (MORE) issue_k(nxt);  // the K registers are free again

        // ---- online softmax; lane-local score j belongs to token tok0 + j of the item
        const int tok0 = b * TB + g * NS;
        const bool tail = !MORE && b * TB + TB > it.n_tokens;  // step reaches past the item's end
        const int first_bad = it.n_tokens - tok0;               // lane-local index of the first invalid token
        if (tail) {
#pragma unroll
            for (int j = 0; j < NS; ++j)
                if (j >= first_bad) s[j] = -INFINITY;
        }
        float mx = s[0];
#pragma unroll
        for (int j = 1; j < NS; ++j) mx = fmaxf(mx, s[j]);
        mx = rows_max(mx);
        const float m_new = fmaxf(m_run, mx);
        const float mc = m_new * c;
        const float alpha = fast_exp2(m_run * c - mc);
        float p[NS];
        float sum = 0.f;
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            p[j] = fast_exp2(__builtin_fmaf(s[j], c, -mc));
            sum += p[j];
        }
        l_run = l_run * alpha + sum;
        m_run = m_new;
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f)) {
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) o[dt] *= alpha;
        }

        // ---- O^T += V^T P^T
        const float vs = (DT == 0) ? 1.0f : pickf(cur.vsc, g);
#pragma unroll
        for (int ks = 0; ks < NS / 8; ++ks) {
            u32x4 pw;
#pragma unroll
            for (int j = 0; j < 4; ++j) pw[j] = pack_bf16(p[ks * 8 + 2 * j] * vs, p[ks * 8 + 2 * j + 1] * vs);
            const bf16x8 pb = as_bf16x8(pw);
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) {
                bf16x8 va;
                if constexpr (DT == 0)
                    va = as_bf16x8(vf[dt]);
                else
                    va = fp8x8_to_bf16x8(vf[dt][2 * ks], vf[dt][2 * ks + 1]);
                if (tail) va = zero_bf16_from(va, first_bad - 8 * ks);  // garbage slots may hold NaN
                o[dt] = mfma16(va, pb, o[dt]);
            }
        }
        if constexpr (MORE) issue_v(nxt);  // the V registers are free again
    };

    int b = ts;
    if (b < n_blk) {
        StepPages<DT> cur, nxt;
        load_step_pages<DT>(cur, a, it, b, last_page);
        issue_k(cur);
        issue_v(cur);
        load_step_pages<DT>(nxt, a, it, b + n_ts, last_page);  // clamped: always in bounds
        while (b + n_ts < n_blk) {
            step(std::true_type{}, b, cur, nxt);
            b += n_ts;
            cur = nxt;
            load_step_pages<DT>(nxt, a, it, b + n_ts, last_page);
        }
        step(std::false_type{}, b, cur, nxt);
    }

    // combine the wavefronts that split the tokens of a row tile, normalise, write the partials
    const float l_row = rows_sum(l_run);
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) *reinterpret_cast<f32x4 *>(&sO[wave][m][16 * dt + 4 * g]) = o[dt];
    if (g == 0) {
        sM[wave][m] = m_run;
        sL[wave][m] = l_row;
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
