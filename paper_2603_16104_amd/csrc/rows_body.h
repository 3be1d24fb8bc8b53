// Per-node decode attention for gfx950 (device code shared by the kernels that run it): each workgroup streams the K/V pages of one chunk of one
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
#pragma once
#include <type_traits>

#include <hip/hip_ext.h>

#include "hkv_device.h"

namespace hkv {

namespace rows {

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kORow = kHeadDim + 4;  // padded LDS row: 16 rows x 132 floats do not collide in banks
constexpr int kStageBytes = 16 * 1024;  // one step's 16 operand fragments x 64 lanes x 16 bytes
constexpr int kMinStages = 3, kMaxStages = 5;  // the launch picks how many stages a workgroup owns
constexpr int kIdRegs = 2;  // LDS-staged items hold their page ids in registers: at most 64*kIdRegs pages
static_assert(kMaxSharedItemTokens <= 64 * kIdRegs * kPage, "planner limit exceeds what the kernel can index");

#ifndef HKV_LDS_PTR
#define HKV_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#endif
#ifndef HKV_GLOBAL_PTR
#define HKV_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void *)(p))
#endif

// s_waitcnt immediate that waits for vmcnt <= n only (gfx9 encoding: vmcnt in bits 3:0 and 15:14,
// expcnt 6:4 and lgkmcnt 11:8 left at their maxima)
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

template <int DT>
struct Traits;
template <>
struct Traits<0> {  // bf16 pool
    static constexpr int kTokBlock = 32;  // tokens per wavefront step
    static constexpr int kBlockBytes = kBlockElems * 2;
};
template <>
struct Traits<1> {  // fp8 e4m3 pool, codes widened to bf16 in registers (exact)
    static constexpr int kTokBlock = 64;
    static constexpr int kBlockBytes = kBlockElems;
};
template <>
struct Traits<2> : Traits<1> {};  // fp8 e4m3 pool, codes fed to the fp8 matrix instruction as they are

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// fp8 matrix instruction: A and B hold 8 e4m3 codes each (k = 8 * (lane / 16) + byte), the lane
// layout of the operands and of the result is that of the bf16 instruction above.
__device__ __forceinline__ f32x4 mfma16_fp8(uint32_t a_lo, uint32_t a_hi, long b, f32x4 c) {
    const long a = (long)(((unsigned long)a_hi << 32) | a_lo);
    return __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(a, b, c, 0, 0, 0);
}

// Two-term e4m3 representation of eight floats x[0..7] (|x| <= 448): hi = fp8(x), lo = fp8(x - hi).
// With 4 significant bits per term the pair carries 8, as many as a bf16 value.
__device__ __forceinline__ void split_fp8x8(const float (&x)[8], long &hi, long &lo) {
    typedef __attribute__((ext_vector_type(2))) float f32x2;
    uint32_t h[2] = {0u, 0u}, l[2] = {0u, 0u};
#pragma unroll
    for (int j = 0; j < 2; ++j) {  // dword j holds elements 4j .. 4j+3: two in the lower half, two in the upper
        h[j] = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(x[4 * j], x[4 * j + 1], (int)h[j], false);
        h[j] = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(x[4 * j + 2], x[4 * j + 3], (int)h[j], true);
        const f32x2 b0 = __builtin_amdgcn_cvt_pk_f32_fp8((int)h[j], false), b1 = __builtin_amdgcn_cvt_pk_f32_fp8((int)h[j], true);
        l[j] = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(x[4 * j] - b0[0], x[4 * j + 1] - b0[1], (int)l[j], false);
        l[j] = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(x[4 * j + 2] - b1[0], x[4 * j + 3] - b1[1], (int)l[j], true);
    }
    hi = (long)(((unsigned long)h[1] << 32) | h[0]);
    lo = (long)(((unsigned long)l[1] << 32) | l[0]);
}

// Keeps the first n (of 8) codes of an operand, zeroes the rest (garbage slots may hold NaN codes).
__device__ __forceinline__ void zero_fp8_from(uint32_t &w0, uint32_t &w1, int n) {
    const unsigned long keep = n >= 8 ? ~0ul : n <= 0 ? 0ul : ((1ul << (8 * n)) - 1ul);
    w0 &= (uint32_t)keep;
    w1 &= (uint32_t)(keep >> 32);
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
        if constexpr (DT != 0) {
            sp.ksc[i] = a.pool.k_scale[(size_t)sp.id[i] * a.pool.num_kv_heads + it.kv_head];
            sp.vsc[i] = a.pool.v_scale[(size_t)sp.id[i] * a.pool.num_kv_heads + it.kv_head];
        }
    }
}

// Per-lane choice among a step's wavefront-uniform values (scalars in, one v_cndmask tree out).
template <typename T>
__device__ __forceinline__ T pick(const T (&v)[2], int sel) {
    const T v0 = v[0], v1 = v[1];
    return (sel & 1) ? v1 : v0;
}
template <typename T>
__device__ __forceinline__ T pick(const T (&v)[4], int sel) {
    const T v0 = v[0], v1 = v[1], v2 = v[2], v3 = v[3];
    const T lo = (sel & 1) ? v1 : v0, hi = (sel & 1) ? v3 : v2;
    return (sel & 2) ? hi : lo;
}

// One workgroup's (FUSED: one half-workgroup's) share of the launch: virtual block `vblock` of the grid of
// n_single + ceil((n_items - n_single) / 4) blocks, run by the 256 threads `tid` = 0..255 with `smem` as their LDS.
// FUSED: the 256 threads are one half of a 512-thread workgroup whose other half runs another block (or
// none: vblock beyond the grid); every half executes exactly one workgroup barrier, so the launch must hold
// no item shared by more than 16 query rows (those synchronise once per step).
constexpr int kCombineBytes = (int)sizeof(float) * (kWaves * 16 * kORow + 2 * kWaves * 16 + 16);

template <int DT, bool FUSED>
__device__ __forceinline__ void body(const DecodeLaunch &a, char *smem, int vblock, int tid) {
    // LDS: a ring of a.n_stages K/V stages for items shared by many query rows; items with at most 16
    // rows use the same bytes for the cross-wavefront combine instead.
    float(*sO)[16][kORow] = reinterpret_cast<float(*)[16][kORow]>(smem);
    float(*sM)[16] = reinterpret_cast<float(*)[16]>(smem + sizeof(float) * kWaves * 16 * kORow);
    float(*sL)[16] = sM + kWaves;
    int *sPart = reinterpret_cast<int *>(sL + kWaves);  // partial index of each of the 16 rows
    static_assert(kCombineBytes <= kMinStages * kStageBytes, "LDS overlay");

    constexpr int TB = Traits<DT>::kTokBlock;
    constexpr int NS = TB / 4;  // scores per lane (16 query rows x TB tokens over 64 lanes)
    constexpr int BB = Traits<DT>::kBlockBytes;

    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Blocks [0, n_single) run one item each.  The blocks behind them run four short items
    // of at most 16 rows each, one per wavefront (no LDS, no barrier: the wavefronts are independent),
    // so that a forest of many short nodes does not pay a workgroup's start-up per 64 tokens.
    const bool packed = vblock >= a.n_single;
    const int item_idx = packed ? a.n_single + kWaves * (vblock - a.n_single) + wave : vblock;
    if (item_idx >= a.n_items) {  // wavefront-uniform (FUSED: also the half without a block)
        if constexpr (FUSED) __syncthreads();
        return;
    }
    const DecodeItem it = a.items[item_idx];
    const int m = lane & 15, g = lane >> 4;
    const int Hkv = a.pool.num_kv_heads;
    const int G = a.num_q_heads / Hkv;
    const int rows = it.n_req * G;
    // Up to 16 rows: the four wavefronts split the tokens and read K/V straight into registers.
    // More rows: each wavefront owns a 16-row tile, all tokens, and K/V are staged once in LDS.
    const bool shared = !FUSED && !packed && rows > 16;
    const int n_rt = shared ? kWaves : 1;
    const int n_ts = packed ? 1 : kWaves / n_rt;
    const int rt = packed ? 0 : wave % n_rt, ts = packed ? 0 : wave / n_rt;
    const float c = a.scale * kLog2e;

    // Q^T operands of this wavefront's 16 rows; rows past the item's end are zero.  The loads are
    // unconditional (row clamped) so that they can stay in flight next to the first K/V requests.
    const int row = rt * 16 + m;
    const int rowc = min(row, rows - 1);
    auto load_req = [&]() {
        int req = a.node_req_idx[it.req_off];  // wavefront-uniform: scalar load
        if (it.n_req > 1) req = a.node_req_idx[it.req_off + rowc / G];
        return req;
    };
    auto load_q = [&](bf16x8 (&qf)[4], int req) {
        const int head = it.kv_head * G + rowc % G;
        const int q_row = a.q_rows ? a.q_rows[req] : req;
        const char *qp = static_cast<const char *>(a.q) + ((size_t)q_row * a.num_q_heads + head) * (kHeadDim * 2);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            // bf16 pool: k-step i covers dims 32*i + 8*g ..; fp8 pool: k-step (i/2, i%2) covers
            // dims 64*(i/2) + 16*g + 8*(i%2) ..
            const int d0 = (DT == 0) ? 32 * i + 8 * g : 64 * (i >> 1) + 16 * g + 8 * (i & 1);
            u32x4 w = ld16(qp + d0 * 2);
            if (row >= rows) w = u32x4{0u, 0u, 0u, 0u};
            qf[i] = as_bf16x8(w);
        }
    };
    bf16x8 qf[4];
    // DT == 2: the query row as two e4m3 terms per element, q * 2^e = hi + lo with the row's largest
    // magnitude brought into [128, 256) by the power of two 2^e (exact for every element down to 2^-10
    // of the largest; below that the second term is rounded to a multiple of 2^-9); q_unscale = 2^-e.
    long qh[4], ql[4];
    float q_unscale = 1.0f;
    auto split_q = [&]() {
        if constexpr (DT == 2) {
            float qx[4][8];
            float amax = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    qx[i][j] = (float)qf[i][j];
                    amax = fmaxf(amax, fabsf(qx[i][j]));
                }
            amax = rows_max(amax);
            // exponent field of the largest magnitude, kept where both 2^e and 2^-e are normal floats
            const int ex = min(max((int)(__float_as_uint(amax) >> 23), 8), 254);
            const float up = __uint_as_float((uint32_t)(261 - ex) << 23);  // 2^(7 - (ex - 127))
            q_unscale = __uint_as_float((uint32_t)(ex - 7) << 23);        // its reciprocal
#pragma unroll
            for (int i = 0; i < 4; ++i) {
#pragma unroll
                for (int j = 0; j < 8; ++j) qx[i][j] *= up;
                split_fp8x8(qx[i], qh[i], ql[i]);
            }
        }
    };
    // Tokens of this item that this lane's query row may see (all of them unless the row is one of
    // several query tokens of a request and this is the node that holds the request's newest tokens).
    int lim = it.n_tokens;
    unsigned long long vis = 0;  // visibility of the tokens from lim on, one bit each
    auto load_limit = [&](int req) {
        if (a.row_leaf && a.row_leaf[req] == it.node) {
            lim = a.row_limit[req] - it.tok_begin;
            vis = a.row_mask[req];
        }
    };

    // Loop-invariant byte offsets of this lane inside a (page, head) block and the page of the step
    // it reads.  bf16: score tile a holds tokens 8*(m/4) + m%4 of the 32-token step, tile b those + 4;
    // the V operand holds tokens 8g..8g+7.  fp8: score tile t4 holds tokens 16*(m/4) + 4*t4 + m%4 of
    // the 64-token step; the V operand holds the 16 tokens of page g.
    const int k_sel = (DT == 0) ? (m >> 3) : (m >> 2);
    const int v_sel = (DT == 0) ? (g >> 1) : g;
    const uint32_t k_off = (uint32_t)it.kv_head * BB +
                           ((DT == 0) ? (((m >> 2) & 1) * 8 + (m & 3)) * 64 + g * 16 : (m & 3) * 64 + g * 16);
    const uint32_t v_off = (uint32_t)it.kv_head * BB + ((DT == 0) ? m * 32 + (g & 1) * 16 : m * 16);
    const uint32_t page_stride = (uint32_t)Hkv * BB;  // 32-bit factors: id * stride is one 32 x 32 -> 64 bit multiply-add
    const char *kb = static_cast<const char *>(a.pool.k_pages) + k_off;
    const char *vb = static_cast<const char *>(a.pool.v_pages) + v_off;

    f32x4 o[8];  // O^T accumulators: d = 16*dt + 4*g + i, row = lane % 16
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY;  // running maximum of the raw scores of this lane's row
    float l_run = 0.f;        // this lane's share of the row sum
    uint32_t v_ref_bits = 0;  // DT == 2: bit pattern of the last step's v_ref (wavefront-uniform), 0 before the first

    const int n_blk = (it.n_tokens + TB - 1) / TB;
    const int last_page = (it.n_tokens - 1) >> 4;

    u32x4 kf[8], vf[8];
    auto issue_k = [&](const StepPages<DT> &sp) {
        const char *p = kb + (uint64_t)(uint32_t)pick(sp.id, k_sel) * page_stride;
        if constexpr (DT == 0) {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                kf[ks] = ld16_stream(p + ks * 1024);
                kf[4 + ks] = ld16_stream(p + ks * 1024 + 256);
            }
        } else {
#pragma unroll
            for (int t4 = 0; t4 < 4; ++t4)
#pragma unroll
                for (int ks2 = 0; ks2 < 2; ++ks2) kf[t4 * 2 + ks2] = ld16_stream(p + ks2 * 1024 + t4 * 256);
        }
    };
    auto issue_v = [&](const StepPages<DT> &sp) {
        const char *p = vb + (uint64_t)(uint32_t)pick(sp.id, v_sel) * page_stride;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) vf[dt] = ld16_stream(p + dt * ((DT == 0) ? 512 : 256));
    };

    // One step over TB tokens.  LAST: the item's last step, the only one that may reach past the item's
    // end (every other instance carries no end-of-item masking at all).  MORE: another step follows, so its K and V are requested as soon as
    // the registers are free; the last step (and only it) may reach past the item's end.
    auto step = [&](auto more_tag, auto last_tag, int b, const StepPages<DT> &cur, const StepPages<DT> &nxt) {
        constexpr bool MORE = decltype(more_tag)::value;
        constexpr bool LAST = decltype(last_tag)::value;
        static_assert(!(MORE && LAST), "the last step has no successor");
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
        } else if constexpr (DT == 1) {
            const float ksc = pick(cur.ksc, g);
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
        } else {
            // codes of K against the two terms of Q; the block scale and the row's 2^-e come afterwards
            const float kq = pick(cur.ksc, g) * q_unscale;
#pragma unroll
            for (int t4 = 0; t4 < 4; ++t4) {
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks2 = 0; ks2 < 2; ++ks2) {
                    const u32x4 w = kf[t4 * 2 + ks2];
                    acc = mfma16_fp8(w[0], w[1], qh[ks2 * 2], acc);
                    acc = mfma16_fp8(w[0], w[1], ql[ks2 * 2], acc);
                    acc = mfma16_fp8(w[2], w[3], qh[ks2 * 2 + 1], acc);
                    acc = mfma16_fp8(w[2], w[3], ql[ks2 * 2 + 1], acc);
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) s[t4 * 4 + i] = acc[i] * kq;
            }
        }
        if constexpr (MORE) {  // the K registers are free again; keep the request exactly here
            __builtin_amdgcn_sched_barrier(0);
            issue_k(nxt);
            __builtin_amdgcn_sched_barrier(0);
        }

        // ---- online softmax; lane-local score j belongs to token tok0 + j of the item
        const int tok0 = b * TB + g * NS;
        const bool tail = LAST && b * TB + TB > it.n_tokens;  // step reaches past the item's end
        const int first_bad = it.n_tokens - tok0;               // lane-local index of the first invalid token
        if (tail) {
#pragma unroll
            for (int j = 0; j < NS; ++j)
                if (j >= first_bad) s[j] = -INFINITY;
        }
        if (__builtin_amdgcn_ballot_w64(tok0 + NS > lim)) {  // some row of the tile does not see the whole step
#pragma unroll
            for (int j = 0; j < NS; ++j)
            {
                const int d = tok0 + j - lim;  // index among the request's newest tokens
                if (d >= 0 && !(d < 64 && ((vis >> d) & 1ull))) s[j] = -INFINITY;
            }
        }
        float mx = s[0];
#pragma unroll
        for (int j = 1; j < NS; ++j) mx = fmaxf(mx, s[j]);
        mx = rows_max(mx);
        const float m_new = fmaxf(m_run, mx);
        // a row that has seen nothing so far keeps m = -inf; its exponentials use 0 as the reference
        // (they are all exp2(-inf) = 0), so that no inf - inf arises
        const float mc = (m_new == -INFINITY) ? 0.f : m_new * c;
        const float alpha = fast_exp2(m_run * c - mc);
        float p[NS];
        float sum = 0.f;
        if constexpr (DT != 2) {
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
        } else {
            // The second product runs on codes of V, so a token's weight carries its block's V scale:
            // x = p * vs / v_ref * 2^8 <= 256, with v_ref the largest V scale of this step's four blocks
            // rounded up to a power of two (o is kept in units of v_ref * 2^-8 and is rescaled whenever
            // v_ref changes from one step to the next, in either direction).
            uint32_t top = 0;  // largest V scale of the step; positive floats order like their bit patterns
#pragma unroll
            for (int i = 0; i < StepPages<DT>::N; ++i) top = max(top, __float_as_uint(cur.vsc[i]));
            const uint32_t ref_new = max((top + 0x007FFFFFu) & 0x7F800000u, 0x00800000u);  // power of two, normal
            const float grow = __uint_as_float(v_ref_bits) * __uint_as_float(0x7F000000u - ref_new);  // v_ref_old / v_ref_new
            v_ref_bits = ref_new;
            const float lv = fast_log2(pick(cur.vsc, g) * __uint_as_float(0x7F000000u - ref_new)) + 8.0f;
#pragma unroll
            for (int j = 0; j < NS; ++j) {
                p[j] = fast_exp2(__builtin_fmaf(s[j], c, lv - mc));
                sum += p[j];
            }
            l_run = l_run * alpha + sum * fast_exp2(-lv);
            m_run = m_new;
            const float alpha_o = alpha * grow;
            if (__builtin_amdgcn_ballot_w64(alpha_o != 1.0f)) {
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) o[dt] *= alpha_o;
            }
        }

        // ---- O^T += V^T P^T
        if constexpr (DT != 2) {
            const float vs = (DT == 0) ? 1.0f : pick(cur.vsc, g);
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
        } else {
#pragma unroll
            for (int ks = 0; ks < NS / 8; ++ks) {
                float x[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) x[j] = p[ks * 8 + j];
                long ph, pl;
                split_fp8x8(x, ph, pl);
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) {
                    uint32_t v0 = vf[dt][2 * ks], v1 = vf[dt][2 * ks + 1];
                    if (tail) zero_fp8_from(v0, v1, first_bad - 8 * ks);  // garbage slots may hold NaN codes
                    o[dt] = mfma16_fp8(v0, v1, ph, o[dt]);
                    o[dt] = mfma16_fp8(v0, v1, pl, o[dt]);
                }
            }
        }
        if constexpr (MORE) {  // the V registers are free again
            __builtin_amdgcn_sched_barrier(0);
            issue_v(nxt);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // Partials of a wavefront that has seen all tokens of its rows: normalise and store from registers.
    auto write_rows = [&](int req) {
        const float l_row = rows_sum(l_run);
        // a row that saw no token of this item delivers the empty partial (o = 0, lse = -inf)
        float inv = l_row > 0.f ? 1.0f / l_row : 0.f;
        if constexpr (DT == 2) inv *= __uint_as_float(v_ref_bits) * 0.00390625f;  // o is in units of v_ref * 2^-8
        float amax = 0.f;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            o[dt] *= inv;
#pragma unroll
            for (int i = 0; i < 4; ++i) amax = fmaxf(amax, fabsf(o[dt][i]));
        }
        amax = rows_max(amax);  // the row's 128 values sit in the four lanes m, m + 16, m + 32, m + 48 (all lanes take part)
        float up, down;
        part_factors(amax, up, down);
        if (row < rows) {
            const size_t part = (size_t)(req * a.num_q_heads + it.kv_head * G + row % G) * a.max_parts + it.part_slot;
            uint16_t *op = a.o_parts + part * kHeadDim + 4 * g;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) {
                u32x2 w;
                w[0] = pack_f16(o[dt][0] * up, o[dt][1] * up);
                w[1] = pack_f16(o[dt][2] * up, o[dt][3] * up);
                *reinterpret_cast<u32x2 *>(op + 16 * dt) = w;
            }
            if (g == 0) a.down_parts[part] = down;
            if (g == 0) a.lse_parts[part] = l_row > 0.f ? (m_run * c + fast_log2(l_row)) * kLn2 : -INFINITY;
        }
    };

    if (shared) {
        // ---- K/V staged in LDS, fetched once for all row tiles of the item (LDS-direct loads: the
        // data in flight occupies no registers, so n_stages - 1 steps are kept in flight: a step of
        // such an item takes about a memory round trip divided by that number).  A stage
        // holds the 16 operand fragments of a step in lane order; wavefront w fetches fragments
        // w, 4+w (K) and 8+w, 12+w (V) with exactly the addresses the register path uses.
        const bool active = rt * 16 < rows;
        // page ids (and fp8 scales) of the whole item, kIdRegs pages per lane (the planner keeps such
        // items at 64*kIdRegs pages or fewer); a step's entries are then read across lanes, so no
        // global load sits between the LDS-direct loads
        int id_lane[kIdRegs];
        float ksc_lane[kIdRegs], vsc_lane[kIdRegs];
#pragma unroll
        for (int r = 0; r < kIdRegs; ++r) {
            id_lane[r] = a.pages[it.page_off + min(lane + 64 * r, last_page)];
            if constexpr (DT != 0) {
                ksc_lane[r] = a.pool.k_scale[(size_t)id_lane[r] * Hkv + it.kv_head];
                vsc_lane[r] = a.pool.v_scale[(size_t)id_lane[r] * Hkv + it.kv_head];
            }
        }
        auto step_pages = [&](StepPages<DT> &sp, int blk) {
#pragma unroll
            for (int i = 0; i < StepPages<DT>::N; ++i) {
                const int pg = min(blk * StepPages<DT>::N + i, last_page);
                const int hi = pg >> 6, lo = pg & 63;  // wavefront-uniform
                int idv = id_lane[0];
                float kv = ksc_lane[0], vv = vsc_lane[0];
#pragma unroll
                for (int r = 1; r < kIdRegs; ++r)
                    if (hi == r) {
                        idv = id_lane[r];
                        kv = ksc_lane[r];
                        vv = vsc_lane[r];
                    }
                sp.id[i] = __builtin_amdgcn_readlane(idv, lo);
                if constexpr (DT != 0) {
                    sp.ksc[i] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, kv), lo));
                    sp.vsc[i] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, vv), lo));
                }
            }
        };
        const int n_stages = a.n_stages, n_ahead = n_stages - 1;
        int issue_slot = 0, read_slot = 0;  // stage of the next step to request / to consume (step % n_stages)
        auto issue_stage = [&](int blk) {
            StepPages<DT> sp;
            step_pages(sp, blk);
            char *stage = smem + issue_slot * kStageBytes;
            issue_slot = issue_slot + 1 == n_stages ? 0 : issue_slot + 1;
            const char *pk = kb + (uint64_t)(uint32_t)pick(sp.id, k_sel) * page_stride;
            const char *pv = vb + (uint64_t)(uint32_t)pick(sp.id, v_sel) * page_stride;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int f = 4 * j + wave;
                const int koff = (DT == 0) ? (f & 3) * 1024 + (f >> 2) * 256 : (f & 1) * 1024 + (f >> 1) * 256;
                __builtin_amdgcn_global_load_lds(HKV_GLOBAL_PTR(pk + koff), HKV_LDS_PTR(stage + f * 1024), 16, 0, 0);
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int dt = 4 * j + wave;
                __builtin_amdgcn_global_load_lds(HKV_GLOBAL_PTR(pv + dt * ((DT == 0) ? 512 : 256)),
                                                 HKV_LDS_PTR(stage + (8 + dt) * 1024), 16, 0, 0);
            }
        };
        const int req = load_req();
        load_q(qf, req);
        load_limit(req);
        for (int i = 0; i < n_ahead && i < n_blk; ++i) issue_stage(i);
        split_q();
        // one step of the item; the last one is peeled off the loop: it alone waits for every load and
        // carries the end-of-item masking
        auto staged_step = [&](auto last_tag, int b) {
            constexpr bool LAST = decltype(last_tag)::value;
            StepPages<DT> cur;
            step_pages(cur, b);  // fp8 scales of this step
            // this wavefront's share of step b has landed once at most the 4 loads of each later step
            // requested so far are pending (loads complete in order)
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (LAST) {
                __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
            } else {
                const int later = min(n_ahead - 1, n_blk - 1 - b);  // >= 1 here; wavefront-uniform
                if (later >= 3)
                    __builtin_amdgcn_s_waitcnt(vmcnt_imm(12));
                else if (later == 2)
                    __builtin_amdgcn_s_waitcnt(vmcnt_imm(8));
                else
                    __builtin_amdgcn_s_waitcnt(vmcnt_imm(4));
            }
            __builtin_amdgcn_s_barrier();  // everyone's share landed; everyone is done with step b-1
            __builtin_amdgcn_sched_barrier(0);
            if (b + n_ahead < n_blk) issue_stage(b + n_ahead);  // overwrites the stage of step b-1
            __builtin_amdgcn_sched_barrier(0);
            const char *stage = smem + read_slot * kStageBytes + lane * 16;
            read_slot = read_slot + 1 == n_stages ? 0 : read_slot + 1;
            if (active) {
#pragma unroll
                for (int f = 0; f < 8; ++f) {
                    kf[f] = *reinterpret_cast<const u32x4 *>(stage + f * 1024);
                    vf[f] = *reinterpret_cast<const u32x4 *>(stage + (8 + f) * 1024);
                }
                step(std::false_type{}, last_tag, b, cur, cur);
            }
        };
        for (int b = 0; b + 1 < n_blk; ++b) staged_step(std::false_type{}, b);
        staged_step(std::true_type{}, n_blk - 1);
        if (active) write_rows(req);
        return;
    }

    int b = ts;
    int req = 0;
    if (b < n_blk) {
        StepPages<DT> cur, nxt;
        load_step_pages<DT>(cur, a, it, b, last_page);
        req = load_req();  // requested before K/V so that waiting for it does not wait for them
        issue_k(cur);
        issue_v(cur);
        load_q(qf, req);
        load_limit(req);
        load_step_pages<DT>(nxt, a, it, b + n_ts, last_page);  // clamped: always in bounds
        split_q();
        while (b + n_ts < n_blk) {
            step(std::true_type{}, std::false_type{}, b, cur, nxt);
            b += n_ts;
            cur = nxt;
            load_step_pages<DT>(nxt, a, it, b + n_ts, last_page);
        }
        step(std::false_type{}, std::true_type{}, b, cur, nxt);
    }
    if (packed) {  // this wavefront did the whole item (it holds at least one token, so req is loaded)
        write_rows(req);
        if constexpr (FUSED) __syncthreads();
        return;
    }

    // combine the wavefronts that split the tokens of a row tile, normalise, write the partials
    const float l_row = rows_sum(l_run);
    if constexpr (DT == 2) {  // o leaves the units of this wavefront's v_ref * 2^-8
        const float unit = __uint_as_float(v_ref_bits) * 0.00390625f;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) o[dt] *= unit;
    }
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) *reinterpret_cast<f32x4 *>(&sO[wave][m][16 * dt + 4 * g]) = o[dt];
    if (g == 0) {
        sM[wave][m] = m_run;
        sL[wave][m] = l_row;
        // wavefront 0 always has a step (the item holds at least one token), so its req is loaded
        if (wave == 0 && row < rows) sPart[m] = (req * a.num_q_heads + it.kv_head * G + row % G) * a.max_parts + it.part_slot;
    }
    __syncthreads();
    // a row's 64 pairs of neighbouring dims are one wavefront's 64 lanes: wavefront w takes rows w, w + 4, ...
    for (int row = wave; row < rows; row += kWaves) {
        const int d = lane * 2;
        const int r_t = row >> 4, r_c = row & 15;
        float M = -INFINITY;
        for (int t = 0; t < n_ts; ++t) M = fmaxf(M, sM[t * n_rt + r_t][r_c]);
        float L = 0.f, acc0 = 0.f, acc1 = 0.f;
        if (M != -INFINITY) {
            for (int t = 0; t < n_ts; ++t) {
                const int w = t * n_rt + r_t;
                const float mw = sM[w][r_c];
                if (mw == -INFINITY) continue;  // that wavefront's tokens were all invisible to the row
                const float wgt = fast_exp2((mw - M) * c);
                L += sL[w][r_c] * wgt;
                acc0 += sO[w][r_c][d] * wgt;
                acc1 += sO[w][r_c][d + 1] * wgt;
            }
        }
        const size_t part = (size_t)sPart[row];
        // a row that saw no token of this item delivers the empty partial (o = 0, lse = -inf)
        const float inv = L > 0.f ? 1.0f / L : 0.f;
        acc0 *= inv;
        acc1 *= inv;
        float amax = fmaxf(fabsf(acc0), fabsf(acc1));
#pragma unroll
        for (int sh = 1; sh < 64; sh <<= 1) amax = fmaxf(amax, __shfl_xor(amax, sh));
        float up, down;
        part_factors(amax, up, down);
        *reinterpret_cast<uint32_t *>(a.o_parts + part * kHeadDim + d) = pack_f16(acc0 * up, acc1 * up);
        if (lane == 0) {
            a.down_parts[part] = down;
            a.lse_parts[part] = L > 0.f ? (M * c + fast_log2(L)) * kLn2 : -INFINITY;
        }
    }
}

}  // namespace rows

}  // namespace hkv
