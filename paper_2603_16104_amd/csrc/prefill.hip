// Suffix-only prefill attention for gfx950: the new tokens of a request attend to the cached
// prefix pages plus the causal part of their own suffix, all read through the block table.
// (Section 5, "Token usage": a call processes only the tokens that are not already cached.)
//
// One workgroup (8 wavefronts, two per SIMD) owns up to 256 query rows = floor(256 / G) consecutive
// new tokens x the G query heads of one KV head, so every K/V tile staged in LDS is used by all G
// heads.  Rows are numbered token-major (row = token * G + head), so any head ratio fills the
// eight 32-row tiles except for at most G - 1 rows.  Each wavefront owns one
// 32-row tile and keeps Q^T and the O^T accumulators in registers; K/V stream
// through LDS in 64-token blocks, four stages each, fetched by LDS-direct loads
// (global_load_lds_dwordx4) two blocks ahead so that the data in flight occupies no registers.
//
// Matrix-core mapping (v_mfma_f32_32x32x16_bf16):
//   S^T = K * Q^T   A = 32 tokens x 16 dims (LDS), B = 16 dims x 32 rows (registers)
//   O^T = V^T * P^T A = 32 dims x 16 tokens (LDS), B = 16 tokens x 32 rows (registers)
// The token order of the score tile's M index is permuted (groups of four: 0,2,1,3) so that a lane
// of the result holds eight consecutive tokens of a page per half, i.e. a ready B operand for the
// second product and a 16-byte read of the dimension-major V page for its A operand.
//
// Softmax.  The exponentials of a block cost about as many VALU cycles as its two products cost
// matrix-core cycles, so the main loop does as little else as possible and overlaps the two:
//   - every row keeps ONE reference value m_ref, the maximum of its first 32 scores, for the whole
//     key range: p = exp2((s - m_ref) * scale * log2 e).  Softmax is invariant to the reference, and
//     fp32 / bf16 carry 8 exponent bits, so p may range over 2^-126 .. 2^90 without loss; there is
//     no running maximum, no cross-lane traffic and no rescaling of O^T in the loop.  Should a row
//     sum pass 2^90 (a later score more than ~60 above the first 32 ones), the workgroup abandons
//     the result and recomputes its tile with the classic running-maximum loop further down.
//   - the loop is software-pipelined inside each wavefront at 32-token steps.  Phase t issues three
//     mutually independent instruction streams, interleaved one to one:
//         S^T(t+1) = K(t+1) Q^T      8 matrix instructions
//         P(t)     = exp2(...S(t))    VALU
//         O^T     += V^T(t-1) P^T(t-1) 8 matrix instructions
//     so every matrix instruction has about three VALU instructions in its shadow and neither of
//     the two wavefronts of a SIMD ever runs a VALU-only or matrix-only stretch.
#include "hkv_device.h"

namespace hkv {

namespace {

constexpr int kWaves = 8;                      // one 32-row tile each
constexpr int kThreads = 64 * kWaves;
constexpr int KB = 64;                         // tokens per LDS stage (4 pages)
constexpr int kTileBytes = KB * kHeadDim * 2;  // 16 KiB for K, same for V
constexpr float kSumLimit = 1.2379400392853803e27f;  // 2^90
constexpr int kIdSlots = 2048;                 // page ids kept in LDS at a time (32768 tokens)
constexpr int kStages = 4;                     // K blocks and V blocks resident in LDS (4 x 16 KiB each)
constexpr int kParts = 16 / kWaves;            // (page, quarter) pairs of a block per wavefront
constexpr int kLoadsPerBlock = 2 * kParts;     // LDS-direct loads each wavefront issues per iteration

#define HKV_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
// s_waitcnt immediate that waits for vmcnt <= n only (gfx9 encoding)
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

// LDS-direct load of 16 bytes per lane: lane l's piece lands at LDS byte lds_base + 16*l.  Issued as
// inline assembly on purpose: the compiler makes every LDS read wait for ALL outstanding loads of
// this kind that it knows of (it cannot tell the stages apart), which would drain the prefetch queue
// at the top of every iteration.  Completion is tracked by hand (vmcnt waits + barriers) instead.
__device__ __forceinline__ void load_to_lds16(const void *gptr, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_base) : "memory");
}
__device__ __forceinline__ uint32_t lds_address(const void *p) { return (uint32_t)(size_t)HKV_LDS_PTR(p); }

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ f32x16 zero16() {
    f32x16 z;
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] = 0.f;
    return z;
}

__global__ __launch_bounds__(kThreads, 2) void prefill_kernel(PrefillLaunch a) {
    __shared__ __attribute__((aligned(16))) char sK[kStages][kTileBytes];
    __shared__ __attribute__((aligned(16))) char sV[kStages][kTileBytes];
    __shared__ int sIds[kIdSlots];  // page ids of the keys in use (a window of the block table row)
    __shared__ int sBail;

    const PrefillTile tl = a.tiles[blockIdx.x];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, h = lane >> 5;
    const int Hq = a.num_q_heads, Hkv = a.pool.num_kv_heads;
    const int G = Hq / Hkv;
    const float c = a.scale * kLog2e;

    // the 32-row tile of this wavefront
    const int r_tile = 32 * wave + n;            // this lane's row within the workgroup's rows
    const int tok = r_tile / G;                  // token index within the tile's new tokens (>= n_q: no such row)
    const int head = tl.kv_head * G + r_tile % G;  // query head
    bf16x8 qf[8];
    {
        const int qrow = tl.q_row0 + min(tok, tl.n_q - 1);
        const char *qp = static_cast<const char *>(a.q) + ((size_t)qrow * Hq + head) * (kHeadDim * 2);
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) qf[kk] = as_bf16x8(ld16(qp + (16 * kk + 8 * h) * 2));
    }
    // wavefront-uniform: smallest absolute position among this wavefront's rows
    const int wave_min_pos = tl.prefix_len + tl.q_begin + min((32 * wave) / G, tl.n_q - 1);

    const int kv_end = tl.prefix_len + tl.q_begin + tl.n_q;  // keys any row of the tile can see
    const int n_blk = (kv_end + KB - 1) / KB;
    const int last_page = (tl.kv_len - 1) >> 4;
    const char *kbase = static_cast<const char *>(a.pool.k_pages) + (size_t)tl.kv_head * (kBlockElems * 2);
    const char *vbase = static_cast<const char *>(a.pool.v_pages) + (size_t)tl.kv_head * (kBlockElems * 2);
    const uint32_t page_stride = (uint32_t)Hkv * (kBlockElems * 2);  // 32-bit factors: one multiply-add per address
    const int32_t *bt = a.block_table + tl.bt_off;

    // LDS-direct loads: a wavefront-level load writes 1 KiB, lane l at byte 16*l.  The LDS image of a
    // page carries bank-conflict swizzles, so each lane fetches the 16-byte piece that belongs at
    // its LDS position:
    //   K page: [chunk = 1 KiB quarter][slot][4 units of 16 B], unit ^= (slot / 4) % 4
    //   V page: [d][2 units of 16 B],                            unit ^= (d / 8) % 2
    // A block is 16 (page i, quarter cq) pairs for K and 16 for V; wavefront w takes the pairs
    // 4*i + cq = u * kWaves + w, u < kParts.
    const int k_slot = lane >> 2, k_unit = lane & 3;
    const int k_in_quarter = k_slot * 64 + ((k_unit ^ ((k_slot >> 2) & 3)) << 4);  // + cq*1024
    const int v_unit = lane & 1;
    int id_base = 0;  // first page held in sIds
    auto fill_ids = [&](int first_page) {  // all threads; the caller separates it from readers by barriers
        for (int i = tid; i < kIdSlots; i += kThreads) sIds[i] = bt[min(first_page + i, last_page)];
    };
    auto k_source = [&](int id, int cq) { return kbase + ((uint64_t)(uint32_t)id * page_stride + (uint32_t)(cq * 1024 + k_in_quarter)); };
    auto v_source = [&](int id, int cq) {
        const int v_d = cq * 32 + (lane >> 1);
        return vbase + ((uint64_t)(uint32_t)id * page_stride + (uint32_t)(v_d * 32 + ((v_unit ^ ((v_d >> 3) & 1)) << 4)));
    };
    // Main path: lane l of a window register holds the id of page 64 * (blk / 16) + l (pages past the
    // sequence are clamped: in bounds), so a request costs a lane read instead of a memory access.
    auto window = [&](int blk) { return sIds[min((blk & ~15) * 4 + lane, last_page) - id_base]; };
    int kwin = 0, vwin = 0;
    auto issue_k_part = [&](int blk, int u) {  // K of block blk -> stage blk % kStages
        const int pc = u * kWaves + wave, i = pc >> 2, cq = pc & 3;
        const int id = __builtin_amdgcn_readlane(kwin, (blk * 4 + i) & 63);
        load_to_lds16(k_source(id, cq), lds_address(sK[blk % kStages] + i * 4096 + cq * 1024));
    };
    auto issue_v_part = [&](int blk, int u) {  // V of block blk -> stage blk % kStages
        const int pc = u * kWaves + wave, i = pc >> 2, cq = pc & 3;
        const int id = __builtin_amdgcn_readlane(vwin, (blk * 4 + i) & 63);
        load_to_lds16(v_source(id, cq), lds_address(sV[blk % kStages] + i * 4096 + cq * 1024));
    };
    // Fallback path: K and V of block blk -> stage st, ids straight from LDS
    auto issue_block = [&](int blk, int st) {
#pragma unroll
        for (int u = 0; u < kParts; ++u) {
            const int pc = u * kWaves + wave, i = pc >> 2, cq = pc & 3;
            const int id = __builtin_amdgcn_readfirstlane(sIds[min(blk * 4 + i, last_page) - id_base]);
            load_to_lds16(k_source(id, cq), lds_address(sK[st] + i * 4096 + cq * 1024));
            load_to_lds16(v_source(id, cq), lds_address(sV[st] + i * 4096 + cq * 1024));
        }
    };
    // V of slots past the sequence end may be anything (NaN included): overwrite with zeros.  Called
    // by all threads between two barriers, only for the block that holds the sequence end.
    auto zero_tail = [&](int blk, int st) {
#pragma unroll
        for (int u = 0; u < kParts; ++u) {
            const int pc = u * kWaves + wave;
            const int i = pc >> 2, cq = pc & 3;
            const int v_d = cq * 32 + (lane >> 1);
            u32x4 *pv = reinterpret_cast<u32x4 *>(sV[st] + i * 4096 + cq * 1024 + lane * 16);
            u32x4 vv = *pv;
            // the piece at this LDS position holds slots 8*u .. 8*u+7 of dim v_d, u = the un-swizzled unit
            const int t0 = blk * KB + i * 16 + (v_unit ^ ((v_d >> 3) & 1)) * 8;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t keep = (t0 + 2 * j + 1 < tl.kv_len) ? 0xFFFFFFFFu : (t0 + 2 * j < tl.kv_len) ? 0x0000FFFFu : 0u;
                vv[j] &= keep;
            }
            *pv = vv;
        }
    };

    // A-operand LDS offsets of this lane.
    //   K: M index n -> token sigma(n) of the 32-token tile (groups of four permuted 0,2,1,3)
    const int grp = n >> 2;
    const int grp_p = ((grp & 3) == 1) ? grp + 1 : ((grp & 3) == 2) ? grp - 1 : grp;
    const int tau = 4 * grp_p + (n & 3);
    const int ka_slot = tau & 15;
    const int ka_swz = (ka_slot >> 2) & 3;
    const int ka_base = (tau >> 4) * 4096 + ka_slot * 64;
    //   V: M index n -> dim 32*dm + n; unit h (slots 8h..8h+7), swizzled by (d/8)%2
    const int va_base = n * 32 + ((h ^ ((n >> 3) & 1)) << 4);
    // operand kk (dims 16kk .. 16kk+15) of the 32-token K tile at ktile
    auto lds_k = [&](const char *ktile, int kk) {
        const int unit = 2 * (kk & 1) + h;
        return as_bf16x8(*reinterpret_cast<const u32x4 *>(ktile + ka_base + (kk >> 1) * 1024 + ((unit ^ ka_swz) << 4)));
    };
    // operand i (page i / 4 of the tile, dims 32 * (i % 4) ..) of the 32-token V tile at vtile
    auto lds_v = [&](const char *vtile, int i) {
        return as_bf16x8(*reinterpret_cast<const u32x4 *>(vtile + (i >> 2) * 4096 + (i & 3) * 1024 + va_base));
    };
    // tiles of step s (32 tokens): block s / 2, half s % 2
    auto k_tile = [&](int s) { return sK[(s >> 1) % kStages] + (s & 1) * 8192; };
    auto v_tile = [&](int s) { return sV[(s >> 1) % kStages] + (s & 1) * 8192; };

    // S^T = K Q^T for one 32-token step, straight from LDS (prologue and fallback)
    auto scores = [&](f32x16 &s, const char *ktile) {
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) s = mfma32(lds_k(ktile, kk), qf[kk], kk == 0 ? zero16() : s);
    };
    // lane-local score i of step st is token st*32 + (i/8)*16 + 8h + i%8.  Rows past the tile's end
    // behave like its last row, so they never see the garbage slots behind the sequence.
    const int pos = tl.prefix_len + tl.q_begin + min(tok, tl.n_q - 1);
    auto mask_scores = [&](f32x16 &s, int st) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int t = st * 32 + (i >> 3) * 16 + 8 * h + (i & 7);
            if (t > pos) s[i] = -INFINITY;
        }
    };

    f32x16 o[4];
    float l_run = 0.f;
    auto pack_probs = [&](u32x4 (&w)[2], const float (&p)[16]) {
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int j = 0; j < 4; ++j) w[hf][j] = pack_bf16(p[hf * 8 + 2 * j], p[hf * 8 + 2 * j + 1]);
    };

    // =========================================================================================
    // main path: one reference value per row, pipelined steps
    // =========================================================================================
#pragma unroll
    for (int dm = 0; dm < 4; ++dm) o[dm] = zero16();
    if (tid == 0) sBail = 0;
    fill_ids(0);
    __syncthreads();
    // Request schedule: K runs one block ahead of V (phase t multiplies K(t+1) but V(t-1)).  The
    // prologue requests K(0); {K(1), V(0)}; {K(2), V(1)}; iteration j requests {K(j+3), V(j+2)}.
    kwin = window(0);
    vwin = kwin;
#pragma unroll
    for (int u = 0; u < kParts; ++u) issue_k_part(0, u);
#pragma unroll
    for (int u = 0; u < kParts; ++u) {
        issue_k_part(1, u);
        issue_v_part(0, u);
    }
#pragma unroll
    for (int u = 0; u < kParts; ++u) {
        issue_k_part(2, u);
        issue_v_part(1, u);
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(kLoadsPerBlock));  // all but the last group: K(0), K(1), V(0) are here
    __builtin_amdgcn_s_barrier();
    if (KB > tl.kv_len) {  // the sequence ends inside block 0
        zero_tail(0, 0);
        __syncthreads();
    }
    f32x16 sa, sb;  // scores of even and odd steps
    scores(sa, k_tile(0));
    if (31 > wave_min_pos) mask_scores(sa, 0);
    float m_ref;  // reference = maximum of the row's first 32 scores (token 0 is visible)
    {
        float mx = sa[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) mx = fmaxf(mx, sa[i]);
        m_ref = fmaxf(mx, __shfl_xor(mx, 32));
    }
    const float mc = m_ref * c;

    // One phase, written in issue order and fenced so that the compiler keeps it.  Operands live in
    // two rings of four registers sets: each set is reloaded right after the matrix instruction
    // that read it, four slots (eight matrix instructions) before its next use.
    //   on entry  kf = operands 0-3 of K(t+1),  vf = operands 0-3 of V(t-1)
    //   on exit   kf = operands 0-3 of K(t+2),  vf = operands 0-3 of V(t)
    // dma_u >= 0: this wavefront's part dma_u of the requests {K(dma_k), V(dma_v)} goes out in slot 2.
    bf16x8 kf[4], vf[4];
    auto phase = [&](const f32x16 &sp, f32x16 &sn, const u32x4 (&wp)[2], u32x4 (&wn)[2], const char *k1,
                     const char *k2, const char *v0, const char *v1, int dma_k, int dma_v, int dma_u) {
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            // The empty asm statements are ordered like the fences; they pin each VALU group between
            // the two matrix instructions it is meant to follow (its inputs become available at the
            // first, its results are consumed at the second).
            float x0 = sp[2 * i], x1 = sp[2 * i + 1];
            sn = mfma32(kf[i & 3], qf[i], i == 0 ? zero16() : sn);
            kf[i & 3] = i < 4 ? lds_k(k1, i + 4) : lds_k(k2, i - 4);
            asm volatile("" : "+v"(x0));
            float p0 = fast_exp2(__builtin_fmaf(x0, c, -mc));
            asm volatile("" : "+v"(p0));
            __builtin_amdgcn_sched_barrier(0);
            o[i & 3] = mfma32(vf[i & 3], as_bf16x8(wp[i >> 2]), o[i & 3]);
            vf[i & 3] = i < 4 ? lds_v(v0, i + 4) : lds_v(v1, i - 4);
            asm volatile("" : "+v"(x1));
            const float p1 = fast_exp2(__builtin_fmaf(x1, c, -mc));
            sum += p0 + p1;
            uint32_t pk = pack_bf16(p0, p1);
            asm volatile("" : "+v"(pk), "+v"(sum));
            wn[i >> 2][i & 3] = pk;
            if (i == 2 && dma_u >= 0) {
                issue_k_part(dma_k, dma_u);
                issue_v_part(dma_v, dma_u);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        l_run += sum;
    };

    u32x4 wa[2], wb[2];  // probabilities (packed bf16) of even and odd steps
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) wb[hf] = u32x4{0u, 0u, 0u, 0u};  // "P(-1)" = 0: phase 0 adds nothing to O^T
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        kf[i] = lds_k(k_tile(1), i);
        vf[i] = lds_v(v_tile(0), i);  // stands in for V(-1): finite data, multiplied by zeros
    }
    // Iteration j = phases 2j and 2j+1: reads K of blocks j, j+1, j+2 and V of blocks j-1, j.  The
    // wait at its end allows only its own requests to be outstanding, so K(j+2) and V(j+1) are
    // complete before iteration j+1 and a request has two iterations to land; K stage (j-1) % 4 and
    // V stage (j-2) % 4 are free from the barrier at the end of iteration j-1 on, which is where
    // iteration j's requests go.  One barrier per iteration.
    for (int j = 0; j < n_blk; ++j) {
        if (((j + 3) & 15) == 0) {
            if ((j + 3) * 4 - id_base >= kIdSlots && (j + 3) * 4 <= last_page) {  // id slots exhausted (rare)
                __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
                __syncthreads();
                id_base = (j + 3) * 4;  // a multiple of 64: the windows stay aligned
                fill_ids(id_base);
                __syncthreads();
            }
            kwin = window(j + 3);
        }
        if (((j + 2) & 15) == 0) vwin = window(j + 2);
        const int t = 2 * j;
        if (j > 0 && j * KB + 31 > wave_min_pos) mask_scores(sa, t);
        phase(sa, sb, wb, wa, k_tile(t + 1), k_tile(t + 2), v_tile(t > 0 ? t - 1 : 0), v_tile(t), j + 3, j + 2, 0);
        if (j * KB + 63 > wave_min_pos) mask_scores(sb, t + 1);
        phase(sb, sa, wa, wb, k_tile(t + 2), k_tile(t + 3), v_tile(t), v_tile(t + 1), j + 3, j + 2, kParts - 1);
        // (after the last block the K operands come from stale stages: in bounds, never used)
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(kLoadsPerBlock));
        __syncthreads();
        if ((j + 1) * KB + KB > tl.kv_len && (j + 1) * KB < tl.kv_len) {  // V(j+1) holds the sequence end
            zero_tail(j + 1, (j + 1) % kStages);
            __syncthreads();
        }
    }
    // drain: O^T += V^T P^T of the last step (vf holds its operands 0-3, wb its probabilities)
    {
        const char *vl = v_tile(2 * n_blk - 1);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            o[i & 3] = mfma32(vf[i & 3], as_bf16x8(wb[i >> 2]), o[i & 3]);
            if (i < 4) vf[i & 3] = lds_v(vl, i + 4);
        }
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // nothing of this path is in flight any more
    // A row sum beyond 2^90, inf or NaN (all of them sticky) means that the reference was far too low
    // for some row: the whole workgroup then repeats its tile with the running-maximum loop.
    if (__builtin_amdgcn_ballot_w64(!(l_run < kSumLimit))) sBail = 1;
    __syncthreads();
    const bool bail = sBail != 0;
    float m_fin = m_ref;

    // =========================================================================================
    // fallback: classic online softmax with a running maximum, one 64-token block at a time.
    // Only taken when a row's later scores exceed its first ones by more than the exponent range
    // allows; always correct, not tuned.
    // =========================================================================================
    if (bail) {
        float m_run = -INFINITY;
#pragma unroll
        for (int dm = 0; dm < 4; ++dm) o[dm] = zero16();
        l_run = 0.f;
        __syncthreads();
        id_base = 0;
        fill_ids(0);
        __syncthreads();
        for (int j = 0; j < n_blk; ++j) {
            if (j * 4 + 3 - id_base >= kIdSlots) {
                id_base = j * 4;
                fill_ids(id_base);
                __syncthreads();
            }
            issue_block(j, 0);
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
            __syncthreads();
            if (j * KB + KB > tl.kv_len) {
                zero_tail(j, 0);
                __syncthreads();
            }
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                f32x16 s;
                scores(s, sK[0] + mt * 8192);
                if (j * KB + mt * 32 + 31 > wave_min_pos) mask_scores(s, 2 * j + mt);
                float mx = s[0];
#pragma unroll
                for (int i = 1; i < 16; ++i) mx = fmaxf(mx, s[i]);
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_new = fmaxf(m_run, mx);
                const float mcn = m_new * c;
                const float alpha = fast_exp2(m_run * c - mcn);
                float p[16];
                float sum = 0.f;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    p[i] = fast_exp2(__builtin_fmaf(s[i], c, -mcn));
                    sum += p[i];
                }
                u32x4 w[2];
                pack_probs(w, p);
                l_run = l_run * alpha + sum;
                m_run = m_new;
#pragma unroll
                for (int dm = 0; dm < 4; ++dm)
#pragma unroll
                    for (int i = 0; i < 16; ++i) o[dm][i] *= alpha;
#pragma unroll
                for (int i = 0; i < 8; ++i) o[i & 3] = mfma32(lds_v(sV[0] + mt * 8192, i), as_bf16x8(w[i >> 2]), o[i & 3]);
            }
            __syncthreads();
        }
        m_fin = m_run;
    }

    // ---- normalise and store; lane (n, h) holds dims 32*dm + 8*(i/4) + 4*h + i%4 of its row
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (tok < tl.n_q) {
        const float inv = 1.0f / l_tot;
        const size_t row = (size_t)(tl.q_row0 + tok) * Hq + head;
        uint16_t *op = static_cast<uint16_t *>(a.out) + row * kHeadDim;
#pragma unroll
        for (int dm = 0; dm < 4; ++dm)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                u32x2 w;
                w[0] = pack_bf16(o[dm][4 * q4] * inv, o[dm][4 * q4 + 1] * inv);
                w[1] = pack_bf16(o[dm][4 * q4 + 2] * inv, o[dm][4 * q4 + 3] * inv);
                *reinterpret_cast<u32x2 *>(op + 32 * dm + 8 * q4 + 4 * h) = w;
            }
        if (a.lse_out && h == 0) a.lse_out[row] = (m_fin * c + fast_log2(l_tot)) * kLn2;
    }
}

}  // namespace

int prefill_tile_tokens(int group) { return 256 / group; }

hipError_t launch_prefill(const PrefillLaunch &a, hipStream_t s) {
    if (a.n_tiles <= 0) return hipSuccess;
    hipLaunchKernelGGL(prefill_kernel, dim3(a.n_tiles), dim3(kThreads), 0, s, a);
    return hipGetLastError();
}

}  // namespace hkv
