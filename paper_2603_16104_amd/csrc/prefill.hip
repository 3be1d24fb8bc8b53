// Suffix-only prefill attention for gfx950: the new tokens of a request attend to the cached
// prefix pages plus the causal part of their own suffix, all read through the block table.
// (Section 5, "Token usage": a call processes only the tokens that are not already cached.)
//
// One workgroup (4 wavefronts) owns 256 query rows = 256/G consecutive new tokens x the G query
// heads of one KV head, so every K/V tile staged in LDS is used by all G heads.  Each wavefront
// owns 64 rows (two 32-row tiles) and keeps Q^T and the O^T accumulators in registers; K/V
// stream through LDS in 64-token blocks, triple buffered, fetched by LDS-direct loads
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
//   - the loop is software-pipelined inside each wavefront at 32-token steps: while the VALU turns
//     the scores of step t into probabilities, the matrix core computes the scores of step t+1 into
//     a second set of registers; the two instruction streams are interleaved explicitly.
#include "hkv_device.h"

namespace hkv {

namespace {

constexpr int kRowsPerGroup = 256;
#ifndef HKV_PREFILL_NT
#define HKV_PREFILL_NT 1
#endif
constexpr int NT = HKV_PREFILL_NT;            // 32-row tiles per wavefront
constexpr int kWaves = 8 / NT;                // 8 row tiles per workgroup
constexpr int kThreads = 64 * kWaves;
constexpr int KB = 64;                         // tokens per LDS stage (4 pages)
constexpr int kTileBytes = KB * kHeadDim * 2;  // 16 KiB for K, same for V
constexpr float kSumLimit = 1.2379400392853803e27f;  // 2^90
constexpr int kIdSlots = 2048;                 // page ids kept in LDS at a time (32768 tokens)
constexpr int kStages = 4;                     // K/V blocks resident in LDS (4 x 32 KiB)
constexpr int kLoadsPerBlock = 32 / kWaves;    // LDS-direct loads each wavefront issues per block

#define HKV_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#define HKV_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void *)(p))
// s_waitcnt immediate that waits for vmcnt <= n only (gfx9 encoding)
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

// LDS-direct load of 16 bytes per lane: lane l's piece lands at LDS byte lds_base + 16*l.  Issued as
// inline assembly on purpose: the compiler makes every LDS read wait for ALL outstanding loads of
// this kind that it knows of (it cannot tell the stages apart), which would drain the prefetch queue
// at the top of every iteration.  Completion is tracked by hand (vmcnt waits + barriers) instead.
__device__ __forceinline__ void load_to_lds16(const void *gptr, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_base) : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_address(const void *p) {
    return (uint32_t)(size_t)HKV_LDS_PTR(p);
}

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ f32x16 zero16() {
    f32x16 z;
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] = 0.f;
    return z;
}

struct Step {
    f32x16 t[NT];  // scores of one 32-token step: [row tile nt]
};

__global__ __launch_bounds__(kThreads, 2 / NT) void prefill_kernel(PrefillLaunch a) {
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
    const int tbh = 8 / G;  // 32-token blocks per head inside the workgroup's rows
    const float c = a.scale * kLog2e;

    // the two 32-row tiles of this wavefront
    int head[NT], tok[NT];  // query head; token index of this lane's row within the tile's new tokens
    bf16x8 qf[NT][8];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int T = NT * wave + nt;
        head[nt] = tl.kv_head * G + T / tbh;
        tok[nt] = 32 * (T % tbh) + n;
        const int qrow = tl.q_row0 + min(tok[nt], tl.n_q - 1);
        const char *qp = static_cast<const char *>(a.q) + ((size_t)qrow * Hq + head[nt]) * (kHeadDim * 2);
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            u32x4 w = ld16(qp + (16 * kk + 8 * h) * 2);
#if HKV_PREFILL_NT == 2
            asm volatile("" : "+a"(w));  // Q^T is only read by matrix instructions: park it in the accumulation file
#endif
            qf[nt][kk] = as_bf16x8(w);
        }
    }
    // wavefront-uniform: smallest absolute position among this wavefront's rows
    const int wave_min_pos = tl.prefix_len + tl.q_begin + 32 * ((NT * wave) % tbh);

    const int kv_end = tl.prefix_len + tl.q_begin + tl.n_q;  // keys any row of the tile can see
    const int n_blk = (kv_end + KB - 1) / KB;
    const int last_page = (tl.kv_len - 1) >> 4;
    const char *kbase = static_cast<const char *>(a.pool.k_pages) + (size_t)tl.kv_head * (kBlockElems * 2);
    const char *vbase = static_cast<const char *>(a.pool.v_pages) + (size_t)tl.kv_head * (kBlockElems * 2);
    const size_t page_stride = (size_t)Hkv * (kBlockElems * 2);
    const int32_t *bt = a.block_table + tl.bt_off;

    // LDS-direct loads: a wavefront-level load writes 1 KiB, lane l at byte 16*l.  The LDS image of a
    // page carries bank-conflict swizzles, so each lane fetches the 16-byte piece that belongs at
    // its LDS position:
    //   K page: [chunk = wavefront][slot][4 units of 16 B], unit ^= (slot / 4) % 4
    //   V page: [d][2 units of 16 B],                        unit ^= (d / 8) % 2
    // Per block 32 wavefront-level loads: (page i, 1 KiB quarter c) for K and for V; wavefront w takes
    // the pairs with (4*i + c) % kWaves == w.
    const int k_slot = lane >> 2, k_unit = lane & 3;
    const int k_in_quarter = k_slot * 64 + ((k_unit ^ ((k_slot >> 2) & 3)) << 4);  // + c*1024
    const int v_unit = lane & 1;
    int id_base = 0;  // first page held in sIds
    auto fill_ids = [&](int first_page) {  // all threads; the caller separates it from readers by barriers
        for (int i = tid; i < kIdSlots; i += kThreads) sIds[i] = bt[min(first_page + i, last_page)];
    };
    // queue the 8 loads of block blk into stage `st` (pages past the sequence are clamped: in bounds)
    auto issue_block = [&](int blk, int st) {
#pragma unroll
        for (int u = 0; u < 16 / kWaves; ++u) {
            const int pc = u * kWaves + wave;  // 4*page + quarter
            const int i = pc >> 2, cq = pc & 3;
            const int id = __builtin_amdgcn_readfirstlane(sIds[min(blk * 4 + i, last_page) - id_base]);
            const size_t page = (size_t)id * page_stride;
            const int v_d = cq * 32 + (lane >> 1);
            const int v_src = v_d * 32 + ((v_unit ^ ((v_d >> 3) & 1)) << 4);
            load_to_lds16(kbase + page + cq * 1024 + k_in_quarter, lds_address(sK[st] + i * 4096 + cq * 1024));
            load_to_lds16(vbase + page + v_src, lds_address(sV[st] + i * 4096 + cq * 1024));
        }
    };
    // V of slots past the sequence end may be anything (NaN included): overwrite with zeros.  Called
    // by all threads between two barriers, only for the block that holds the sequence end.
    auto zero_tail = [&](int blk, int st) {
#pragma unroll
        for (int u = 0; u < 16 / kWaves; ++u) {
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
    // everything queued by this wavefront has landed; then everyone's has
    auto land = [&]() {
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        __builtin_amdgcn_s_barrier();
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

    // S^T = K Q^T for one 32-token step (token tile mt of the block in kbuf) x this wavefront's 64 rows
    auto scores = [&](Step &s, const char *kbuf, int mt) {
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            const int unit = 2 * (kk & 1) + h;
            const bf16x8 ka = as_bf16x8(*reinterpret_cast<const u32x4 *>(
                kbuf + mt * 8192 + ka_base + (kk >> 1) * 1024 + ((unit ^ ka_swz) << 4)));
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) s.t[nt] = mfma32(ka, qf[nt][kk], kk == 0 ? zero16() : s.t[nt]);
        }
    };
    // lane-local score i of step st is token st*32 + (i/8)*16 + 8h + i%8
    auto mask_scores = [&](Step &s, int st) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            // absolute position of this lane's row; rows past the tile's end behave like its last row,
            // so they never see the garbage slots behind the sequence
            const int pos = tl.prefix_len + tl.q_begin + min(tok[nt], tl.n_q - 1);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int t = st * 32 + (i >> 3) * 16 + 8 * h + (i & 7);
                if (t > pos) s.t[nt][i] = -INFINITY;
            }
        }
    };

    f32x16 o[NT][4];
    float m_ref[NT], l_run[NT];
    bf16x8 pb[NT][2];
    // The O^T tiles are only ever touched by matrix instructions inside the loop.  Telling the
    // register allocator that they belong in the accumulation registers (an empty asm with an "a"
    // constraint) keeps it from parking them in the VALU registers and shuffling them back and
    // forth around every softmax.
    auto pin_accumulators = [&]() {
#if HKV_PREFILL_NT == 2
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int dm = 0; dm < 4; ++dm) asm volatile("" : "+a"(o[nt][dm]));
#endif
    };
    // O^T += V^T P^T for one step: pages 2*mt and 2*mt + 1 of the block in vbuf
    auto accumulate = [&](const char *vbuf, int mt) {
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int dm = 0; dm < 4; ++dm) {
                const bf16x8 va = as_bf16x8(
                    *reinterpret_cast<const u32x4 *>(vbuf + (2 * mt + hf) * 4096 + dm * 1024 + va_base));
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) o[nt][dm] = mfma32(va, pb[nt][hf], o[nt][dm]);
            }
    };
    auto pack_probs = [&](int nt, const float (&p)[16]) {
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
            u32x4 w;
#pragma unroll
            for (int j = 0; j < 4; ++j) w[j] = pack_bf16(p[hf * 8 + 2 * j], p[hf * 8 + 2 * j + 1]);
            pb[nt][hf] = as_bf16x8(w);
        }
    };

    // =========================================================================================
    // main path: one reference value per row, pipelined steps
    // =========================================================================================
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
        for (int dm = 0; dm < 4; ++dm) o[nt][dm] = zero16();
        l_run[nt] = 0.f;
    }
    if (tid == 0) sBail = 0;
    fill_ids(0);
    __syncthreads();
    issue_block(0, 0);
    issue_block(1, 1);
    issue_block(2, 2);
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(kLoadsPerBlock));  // blocks 0 and 1 are complete, block 2 may fly on
    __builtin_amdgcn_s_barrier();
    if (2 * KB > tl.kv_len) {  // the sequence ends inside block 0 or 1
        if (KB > tl.kv_len) zero_tail(0, 0);
        zero_tail(1, 1);
        __syncthreads();
    }
    Step sa, sb;  // even and odd steps
    scores(sa, sK[0], 0);
    if (31 > wave_min_pos) mask_scores(sa, 0);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {  // reference = maximum of the row's first 32 scores (token 0 is visible)
        float mx = sa.t[nt][0];
#pragma unroll
        for (int i = 1; i < 16; ++i) mx = fmaxf(mx, sa.t[nt][i]);
        m_ref[nt] = fmaxf(mx, __shfl_xor(mx, 32));
    }
    float mc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) mc[nt] = m_ref[nt] * c;

    // One pipeline phase = one 32-token step t, written in issue order and fenced so that the
    // compiler keeps it:
    //   1. request the eight V^T operands of step t from LDS;
    //   2. eight matrix instructions S^T(t+1) = K(t+1) Q^T on the K operands already in registers,
    //      each followed by the VALU work that turns two scores of step t into probabilities
    //      (they run in the shadow of the matrix instruction; the V^T reads land meanwhile);
    //   3. request the eight K operands of step t+2;
    //   4. eight matrix instructions O^T += V^T(t) P^T(t) (the K reads land meanwhile).
    static_assert(NT == 1, "the pipelined path is written for one row tile per wavefront");
    bf16x8 kf[8];
    auto load_k = [&](const char *ktile) {
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            const int unit = 2 * (kk & 1) + h;
            kf[kk] = as_bf16x8(*reinterpret_cast<const u32x4 *>(ktile + ka_base + (kk >> 1) * 1024 + ((unit ^ ka_swz) << 4)));
        }
    };
    auto phase = [&](const f32x16 &sp, f32x16 &sn, const char *vtile, const char *knext) {
        bf16x8 vf[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
            vf[i] = as_bf16x8(*reinterpret_cast<const u32x4 *>(vtile + (i >> 2) * 4096 + (i & 3) * 1024 + va_base));
        __builtin_amdgcn_sched_barrier(0);
        u32x4 w[2];
        float sum = 0.f;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            sn = mfma32(kf[kk], qf[0][kk], kk == 0 ? zero16() : sn);
            const float p0 = fast_exp2(__builtin_fmaf(sp[2 * kk], c, -mc[0]));
            const float p1 = fast_exp2(__builtin_fmaf(sp[2 * kk + 1], c, -mc[0]));
            sum += p0 + p1;
            w[kk >> 2][kk & 3] = pack_bf16(p0, p1);
            __builtin_amdgcn_sched_barrier(0);
        }
        l_run[0] += sum;
        load_k(knext);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 8; ++i) o[0][i & 3] = mfma32(vf[i], as_bf16x8(w[i >> 2]), o[0][i & 3]);
        __builtin_amdgcn_sched_barrier(0);
    };

    // Block j = steps 2j and 2j+1, held in stage j % kStages.  At the top of iteration j block j+3
    // is requested into the stage that block j-1 has just left; blocks j and j+1 are complete (the
    // wait at the end of iteration j-1 allows only the youngest request to be outstanding), so a
    // request has two iterations to land and one barrier per iteration suffices.
    load_k(sK[0] + 8192);  // step 1
    bool bail = false;
    for (int j = 0; j < n_blk; ++j) {
        const char *knext = sK[(j + 1) % kStages], *vcur = sV[j % kStages];
        if ((j + 3) * 4 + 3 - id_base >= kIdSlots && (j + 3) * 4 <= last_page) {  // id window exhausted (rare)
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
            __syncthreads();
            id_base = (j + 2) * 4;
            fill_ids(id_base);
            __syncthreads();
        }
        issue_block(j + 3, (j + 3) % kStages);
        if (j > 0 && j * KB + 31 > wave_min_pos) mask_scores(sa, 2 * j);
        phase(sa.t[0], sb.t[0], vcur, knext);  // step 2j; scores of 2j+1; K of 2j+2
        if (j * KB + 63 > wave_min_pos) mask_scores(sb, 2 * j + 1);
        phase(sb.t[0], sa.t[0], vcur + 8192, knext + 8192);  // step 2j+1; scores of 2j+2; K of 2j+3
        // (after the last block these read stale stages: in bounds, never used)
        // a row sum beyond 2^90 (or inf/NaN) means the reference was far too low: give up this path
        const bool over = !(l_run[0] < kSumLimit);
        if (__builtin_amdgcn_ballot_w64(over)) sBail = 1;
        // blocks up to j+2 are complete (only the request of this iteration may be outstanding);
        // stage j % kStages is no longer read; the flag is visible
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(kLoadsPerBlock));
        __syncthreads();
        if (sBail) {
            bail = true;
            break;
        }
        if ((j + 2) * KB + KB > tl.kv_len && (j + 2) * KB < tl.kv_len) {  // block j+2 holds the sequence end
            zero_tail(j + 2, (j + 2) % kStages);
            __syncthreads();
        }
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // nothing of this path is in flight any more
    __syncthreads();
    float m_fin[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) m_fin[nt] = m_ref[nt];

    // =========================================================================================
    // fallback: classic online softmax with a running maximum, one 64-token block at a time.
    // Only taken when a row's later scores exceed its first ones by more than the exponent range
    // allows; always correct, not tuned.
    // =========================================================================================
    if (bail) {
        float m_run[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
            for (int dm = 0; dm < 4; ++dm) o[nt][dm] = zero16();
            m_run[nt] = -INFINITY;
            l_run[nt] = 0.f;
        }
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
            land();
            if (j * KB + KB > tl.kv_len) {
                zero_tail(j, 0);
                __syncthreads();
            }
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                Step s;
                scores(s, sK[0], mt);
                if (j * KB + mt * 32 + 31 > wave_min_pos) mask_scores(s, 2 * j + mt);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    float mx = s.t[nt][0];
#pragma unroll
                    for (int i = 1; i < 16; ++i) mx = fmaxf(mx, s.t[nt][i]);
                    mx = fmaxf(mx, __shfl_xor(mx, 32));
                    const float m_new = fmaxf(m_run[nt], mx);
                    const float mcn = m_new * c;
                    const float alpha = fast_exp2(m_run[nt] * c - mcn);
                    float p[16];
                    float sum = 0.f;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        p[i] = fast_exp2(__builtin_fmaf(s.t[nt][i], c, -mcn));
                        sum += p[i];
                    }
                    pack_probs(nt, p);
                    l_run[nt] = l_run[nt] * alpha + sum;
                    m_run[nt] = m_new;
#pragma unroll
                    for (int dm = 0; dm < 4; ++dm)
#pragma unroll
                        for (int i = 0; i < 16; ++i) o[nt][dm][i] *= alpha;
                }
                accumulate(sV[0], mt);
            }
            __syncthreads();
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) m_fin[nt] = m_run[nt];
    }

    // ---- normalise and store; lane (n, h) holds dims 32*dm + 8*(i/4) + 4*h + i%4 of its row
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
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
        if (a.lse_out && h == 0) a.lse_out[row] = (m_fin[nt] * c + fast_log2(l_tot)) * kLn2;
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
