// The 256-row attention tile of gfx950 (device code shared by the kernels that run it), in two roles:
//
//  - suffix-only prefill: the new tokens of a request attend to the cached prefix pages plus the
//    causal part of their own suffix, all read through the block table (Section 5, "Token usage": a
//    call processes only the tokens that are not already cached);
//  - decode work items shared by many query rows: a chunk of a prefix-tree node applied to up to
//    256 / G requests below it at once, one partial result (o, lse) per query row (the prefix KV
//    computed once and reused by every call below it: Section 5, "Proactive Cache Management").
//    Here a workgroup is persistent: workgroup w runs items w, w + grid, ..., so that the launch
//    holds a chosen number of compute units and leaves the others to the kernel that streams the
//    nodes few rows share, which runs next to it on another stream.
//
// One workgroup (8 wavefronts, two per SIMD) owns up to 256 query rows = floor(256 / G) consecutive
// new tokens (resp. requests) x the G query heads of one KV head, so every K/V tile staged in LDS is
// used by all G heads.  Rows are numbered token-major (row = token * G + head), so any head ratio
// fills the eight 32-row tiles except for at most G - 1 rows.  Each wavefront owns one 32-row tile
// and keeps Q^T and the O^T accumulators in registers; K/V stream through LDS in 64-token blocks,
// four stages each, as a swizzled bf16 image:
//   bf16 pools: LDS-direct loads (global_load_lds_dwordx4) two blocks ahead, so that the data in
//               flight occupies no registers;
//   fp8 pools (decode items): 16-byte loads into a two-deep register queue, the codes widened to
//               bf16 (exact) once per workgroup on their way into LDS; the block scales stay out of
//               the operands: the K scale multiplies the score inside the exponential's argument, the
//               V scale enters as an exponent offset, and the row sum is taken per 16-token block
//               and divided by that block's V scale again.
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
//   - every row keeps ONE reference value, the maximum of its first 32 scores, for the whole key
//     range: p = exp2(s * scale * log2 e - reference).  Softmax is invariant to the reference, and
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
#pragma once
#include <hip/hip_ext.h>

#include <type_traits>

#include "hkv_device.h"

namespace hkv {

namespace tile {

constexpr int kWaves = 8;                      // one 32-row tile each
constexpr int kThreads = 64 * kWaves;
constexpr int KB = 64;                         // tokens per LDS stage (4 pages)
constexpr int kTileBytes = KB * kHeadDim * 2;  // 16 KiB for K, same for V
constexpr float kSumLimit = 1.2379400392853803e27f;  // 2^90
constexpr int kIdSlots = 2048;                 // page ids kept in LDS at a time (32768 tokens)
constexpr int kStages = 4;                     // K blocks and V blocks resident in LDS (4 x 16 KiB each)
constexpr int kParts = 16 / kWaves;            // (page, quarter) pairs of a block per wavefront
constexpr int kLoadsPerBlock = 2 * kParts;     // LDS-direct loads each wavefront issues per iteration
static_assert(kMaxTileItemTokens <= kScaleSlots * kPage && kMaxTileItemTokens <= kIdSlots * kPage, "decode item limit");

#ifndef HKV_LDS_PTR
#define HKV_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#endif
// s_waitcnt immediate that waits for vmcnt <= n only (gfx9 encoding)
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

// LDS-direct load of 16 bytes per lane: lane l's piece lands at LDS byte lds_base + 16*l.  Issued as
// inline assembly on purpose: the compiler makes every LDS read wait for ALL outstanding loads of
// this kind that it knows of (it cannot tell the stages apart), which would drain the prefetch queue
// at the top of every iteration.  Completion is tracked by hand (vmcnt waits + barriers) instead.
__device__ __forceinline__ void load_to_lds16(const void *gptr, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_base) : "memory");
}
// The same from a wavefront-uniform base plus a 32-bit offset per lane: the address arithmetic of the uniform
// part stays on the scalar unit.
__device__ __forceinline__ void load_to_lds16(const void *uniform_base, uint32_t lane_offset, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 ::"v"(lane_offset), "s"(uniform_base), "s"(lds_base)
                 : "memory");
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

// What the two roles hand the kernel.
struct TileArgs {
    PoolView pool;
    const void *q;
    const void *tiles;           // device: PrefillTile[] (prefill) or DecodeItem[] (decode items)
    const int32_t *ids;          // device: block table (prefill) or the plan's block list (decode items)
    int32_t n_tiles;
    int32_t num_q_heads;
    float scale;
    void *out;                   // prefill: [tokens][Hq][128] bf16
    float *lse_out;              // prefill: may be null
    const int32_t *node_req_idx; // decode items: node->request CSR values
    uint16_t *o_parts;           // decode items: partial results (o in fp16 times a power of two per partial,
    float *lse_parts;            // lse and the reciprocal of that power in fp32)
    float *down_parts;
    int32_t max_parts;
    const int32_t *q_rows;       // decode items, may be null: row r of the plan reads row q_rows[r] of q
    unsigned int *fallback_tiles;  // may be null: incremented once per tile that takes the running-maximum path
};

// DECODE: decode work items (persistent workgroups, partial results) instead of prefill tiles.
// FP8: the pool holds e4m3 codes with a scale per 16-token block and head (decode items only).
// lds: kLdsBytes of the workgroup's LDS, 16-byte aligned.  The workgroup (kThreads threads, thread index
// threadIdx.x) runs tiles first, first + stride, ... (prefill runs one: stride is not used).
constexpr int kLdsBytes = 2 * kStages * kTileBytes + kIdSlots * 4 + kScaleSlots * 16 + 16;

template <bool DECODE, bool FP8>
__device__ __forceinline__ void body(const TileArgs &a, char *lds, int first, int stride) {
    static_assert(DECODE || !FP8, "prefill reads fp8 pools through the dequantising pre-pass");
    char(*sK)[kTileBytes] = reinterpret_cast<char(*)[kTileBytes]>(lds);
    char(*sV)[kTileBytes] = reinterpret_cast<char(*)[kTileBytes]>(lds + kStages * kTileBytes);
    int *sIds = reinterpret_cast<int *>(lds + 2 * kStages * kTileBytes);  // page ids of the keys in use (a window of the block table row)
    // fp8: per page of the item {c * K scale, log2(V scale), 1 / V scale, -}: one 16-byte read per page, and the
    // two pages of a 32-token step sit side by side (entries behind the item's last page repeat it, so a step
    // needs no clamp)
    f32x4 *sScale = reinterpret_cast<f32x4 *>(sIds + kIdSlots);
    int &sBail = *reinterpret_cast<int *>(sScale + kScaleSlots);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, h = lane >> 5;
    const int Hq = a.num_q_heads, Hkv = a.pool.num_kv_heads;
    const int G = Hq / Hkv;
    const float c = a.scale * kLog2e;
    constexpr int BB = FP8 ? kBlockElems : kBlockElems * 2;  // bytes of a (page, head) block of the pool
    const uint32_t page_stride = (uint32_t)Hkv * BB;  // 32-bit factors: one multiply-add per address

    // loop-invariant lane geometry
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
    // fp8: thread (page i = tid / 128 of the block, piece q = tid % 128) moves 16 bytes of K (16 dims of
    // one slot) and 16 bytes of V (the 16 slots of one dim) of every block, widened into two 16-byte units
    const int f_i = tid >> 7, f_q = tid & 127;
    const int fk_slot = (f_q >> 2) & 15, fk_p = f_q & 3;
    const int fk_swz = (fk_slot >> 2) & 3;
    const uint32_t fk_dst0 = (uint32_t)(f_i * 4096 + (2 * (f_q >> 6) + (fk_p >> 1)) * 1024 + fk_slot * 64 + (((2 * (fk_p & 1)) ^ fk_swz) << 4));
    const uint32_t fk_dst1 = (uint32_t)(f_i * 4096 + (2 * (f_q >> 6) + (fk_p >> 1)) * 1024 + fk_slot * 64 + (((2 * (fk_p & 1) + 1) ^ fk_swz) << 4));
    const int fv_swz = (f_q >> 3) & 1;
    const uint32_t fv_dst0 = (uint32_t)(f_i * 4096 + (f_q >> 5) * 1024 + (f_q & 31) * 32 + ((0 ^ fv_swz) << 4));
    const uint32_t fv_dst1 = (uint32_t)(f_i * 4096 + (f_q >> 5) * 1024 + (f_q & 31) * 32 + ((1 ^ fv_swz) << 4));
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

    // prefill: one tile per workgroup; decode items: workgroup w runs items w, w + grid, ...
    for (int ti = first; ti < a.n_tiles; ti += stride) {
    if (DECODE && ti != first) __syncthreads();  // everyone has left the last item's LDS

    // ---- the tile: kv_head, n_slots tokens (requests) x G heads, keys 0 .. kv_end-1 of the page list bt
    int kv_head, n_slots, kv_len, kv_end, pos_first;
    const int32_t *bt;
    PrefillTile tl{};
    DecodeItem it{};
    if constexpr (DECODE) {
        it = static_cast<const DecodeItem *>(a.tiles)[ti];
        kv_head = it.kv_head;
        n_slots = it.n_req;
        kv_len = kv_end = it.n_tokens;
        pos_first = it.n_tokens - 1;  // every row sees every token of the item
        bt = a.ids + it.page_off;
    } else {
        tl = static_cast<const PrefillTile *>(a.tiles)[ti];
        kv_head = tl.kv_head;
        n_slots = tl.n_q;
        kv_len = tl.kv_len;
        kv_end = tl.prefix_len + tl.q_begin + tl.n_q;  // keys any row of the tile can see
        pos_first = tl.prefix_len + tl.q_begin;
        bt = a.ids + tl.bt_off;
    }

    // the 32-row tile of this wavefront
    const int r_tile = 32 * wave + n;            // this lane's row within the workgroup's rows
    const int tok = r_tile / G;                  // token (request) index within the tile (>= n_slots: no such row)
    const int head = kv_head * G + r_tile % G;   // query head
    const int slot_c = min(tok, n_slots - 1);
    uint32_t io_row;                             // row of out (prefill) / of the partials' owner (decode items)
    uint32_t q_row;                              // row of q
    if constexpr (DECODE) {
        const uint32_t r = (uint32_t)a.node_req_idx[it.req_off + slot_c];
        io_row = r * Hq + head;
        q_row = (a.q_rows ? (uint32_t)a.q_rows[r] : r) * Hq + head;
    } else {
        q_row = io_row = (uint32_t)(tl.q_row0 + slot_c) * Hq + head;
    }
    bf16x8 qf[8];
    {
        const char *qp = static_cast<const char *>(a.q) + (size_t)q_row * (kHeadDim * 2);
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) qf[kk] = as_bf16x8(ld16(qp + (16 * kk + 8 * h) * 2));
    }
    // wavefront-uniform: smallest absolute position among this wavefront's rows
    const int wave_min_pos = DECODE ? pos_first : pos_first + min((32 * wave) / G, n_slots - 1);
    // Rows past the tile's end behave like its last row, so they never see the garbage slots behind the sequence.
    const int pos = DECODE ? pos_first : pos_first + slot_c;

    const int n_blk = (kv_end + KB - 1) / KB;
    const int last_page = (kv_len - 1) >> 4;
    const char *kbase = static_cast<const char *>(a.pool.k_pages) + (size_t)kv_head * BB;
    const char *vbase = static_cast<const char *>(a.pool.v_pages) + (size_t)kv_head * BB;

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
    // (page and quarter are wavefront-uniform: only the lane's place inside the quarter is a vector operand)
    const uint32_t v_in_quarter = (uint32_t)((lane >> 1) * 32 + ((v_unit ^ ((lane >> 4) & 1)) << 4));
    auto issue_k_part = [&](int blk, int u, int st) {  // K of block blk -> stage st = blk % kStages
        const int pc = u * kWaves + wave, i = pc >> 2, cq = pc & 3;
        const int id = __builtin_amdgcn_readlane(kwin, (blk * 4 + i) & 63);
        load_to_lds16(kbase + ((uint64_t)(uint32_t)id * page_stride + (uint32_t)(cq * 1024)), (uint32_t)k_in_quarter,
                      lds_address(sK[st] + i * 4096 + cq * 1024));
    };
    auto issue_v_part = [&](int blk, int u, int st) {  // V of block blk -> stage st = blk % kStages
        const int pc = u * kWaves + wave, i = pc >> 2, cq = pc & 3;
        const int id = __builtin_amdgcn_readlane(vwin, (blk * 4 + i) & 63);
        load_to_lds16(vbase + ((uint64_t)(uint32_t)id * page_stride + (uint32_t)(cq * 1024)), v_in_quarter,
                      lds_address(sV[st] + i * 4096 + cq * 1024));
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
                const uint32_t keep = (t0 + 2 * j + 1 < kv_len) ? 0xFFFFFFFFu : (t0 + 2 * j < kv_len) ? 0x0000FFFFu : 0u;
                vv[j] &= keep;
            }
            *pv = vv;
        }
    };
    // fp8: this thread's 16 bytes of K resp. V of block blk (page clamped: in bounds), and their way into
    // the bf16 image of stage st (V codes of slots past the item's end, which may be NaN, are cleared first)
    auto fetch_fp8 = [&](const char *base, int blk) {
        const int id = __builtin_amdgcn_readfirstlane(sIds[min(blk * 4 + f_i, last_page)]);  // (items never refill the window)
        return ld16_stream(base + ((uint64_t)(uint32_t)id * page_stride + (uint32_t)(f_q * 16)));
    };
    auto store_k_fp8 = [&](u32x4 w, int st) {
        *reinterpret_cast<u32x4 *>(sK[st] + fk_dst0) = __builtin_bit_cast(u32x4, fp8x8_to_bf16x8(w[0], w[1]));
        *reinterpret_cast<u32x4 *>(sK[st] + fk_dst1) = __builtin_bit_cast(u32x4, fp8x8_to_bf16x8(w[2], w[3]));
    };
    auto store_v_fp8 = [&](u32x4 w, int blk, int st) {
        const int valid = kv_len - (blk * KB + f_i * 16);
        if (valid < 16) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int left = valid - 4 * j;  // bytes of word j to keep
                w[j] &= left >= 4 ? 0xFFFFFFFFu : left <= 0 ? 0u : ((1u << (8 * left)) - 1u);
            }
        }
        *reinterpret_cast<u32x4 *>(sV[st] + fv_dst0) = __builtin_bit_cast(u32x4, fp8x8_to_bf16x8(w[0], w[1]));
        *reinterpret_cast<u32x4 *>(sV[st] + fv_dst1) = __builtin_bit_cast(u32x4, fp8x8_to_bf16x8(w[2], w[3]));
    };

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
    // lane-local score i of step st is token st*32 + (i/8)*16 + 8h + i%8
    auto mask_scores = [&](f32x16 &s, int st) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int t = st * 32 + (i >> 3) * 16 + 8 * h + (i & 7);
            if (t > pos) s[i] = -INFINITY;
        }
    };
    // Factors of the two 16-token blocks of step st.  bf16 pools: the same for every block.  fp8 pools: the
    // K scale multiplies the score inside the exponential's argument, log2 of the V scale is added to it
    // (so that p carries the V scale into the second product), and the row sum divides it out again.
    struct StepScale {
        float ck[2], lv[2], iv[2];
    };
    auto step_scale = [&](int st) {
        StepScale r;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            if constexpr (FP8) {
                const f32x4 e = sScale[2 * st + i];
                r.ck[i] = e[0];
                r.lv[i] = e[1];
                r.iv[i] = e[2];
            } else {
                r.ck[i] = c;
                r.lv[i] = 0.f;
                r.iv[i] = 1.f;
            }
        }
        return r;
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
    if constexpr (FP8) {
        for (int p = tid; p < min(4 * n_blk, kScaleSlots); p += kThreads) {  // every page of every 64-token block
            const size_t id = (size_t)bt[min(p, last_page)];
            const float vs = a.pool.v_scale[id * Hkv + kv_head];
            sScale[p] = f32x4{c * a.pool.k_scale[id * Hkv + kv_head], fast_log2(vs), 1.0f / vs, 0.f};
        }
    }
    __syncthreads();
    // Request schedule: K runs one block ahead of V (phase t multiplies K(t+1) but V(t-1)).  The
    // prologue requests K(0); {K(1), V(0)}; {K(2), V(1)}; iteration j requests {K(j+3), V(j+2)}.
    // fp8: K(0), K(1), V(0) are widened into LDS here; {K(2), V(1)} and {K(3), V(2)} wait in the register
    // queue; iteration j widens {K(j+2), V(j+1)} and requests {K(j+4), V(j+3)} in their place.
    u32x4 kq[2], vq[2];
    if constexpr (FP8) {
        const u32x4 k0 = fetch_fp8(kbase, 0), k1 = fetch_fp8(kbase, 1), v0 = fetch_fp8(vbase, 0);
        kq[0] = fetch_fp8(kbase, 2);
        vq[0] = fetch_fp8(vbase, 1);
        kq[1] = fetch_fp8(kbase, 3);
        vq[1] = fetch_fp8(vbase, 2);
        store_k_fp8(k0, 0);
        store_k_fp8(k1, 1);
        store_v_fp8(v0, 0, 0);
        __syncthreads();
    } else {
        kwin = window(0);
        vwin = kwin;
#pragma unroll
        for (int u = 0; u < kParts; ++u) issue_k_part(0, u, 0);
#pragma unroll
        for (int u = 0; u < kParts; ++u) {
            issue_k_part(1, u, 1);
            issue_v_part(0, u, 0);
        }
#pragma unroll
        for (int u = 0; u < kParts; ++u) {
            issue_k_part(2, u, 2);
            issue_v_part(1, u, 1);
        }
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(kLoadsPerBlock));  // all but the last group: K(0), K(1), V(0) are here
        __builtin_amdgcn_s_barrier();
        if (KB > kv_len) {  // the sequence ends inside block 0
            zero_tail(0, 0);
            __syncthreads();
        }
    }
    f32x16 sa, sb;  // scores of even and odd steps
    scores(sa, k_tile(0));
    if (31 > wave_min_pos) mask_scores(sa, 0);
    float mc;  // reference = maximum of the row's first 32 scores (token 0 is visible), times scale * log2 e
    {
        const StepScale s0 = step_scale(0);
        float mx = sa[0] * s0.ck[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) mx = fmaxf(mx, sa[i] * s0.ck[i >> 3]);
        mc = fmaxf(mx, __shfl_xor(mx, 32));
    }

    // One phase, written in issue order and fenced so that the compiler keeps it.  Operands live in
    // two rings of four registers sets: each set is reloaded right after the matrix instruction
    // that read it, four slots (eight matrix instructions) before its next use.
    //   on entry  kf = operands 0-3 of K(t+1),  vf = operands 0-3 of V(t-1)
    //   on exit   kf = operands 0-3 of K(t+2),  vf = operands 0-3 of V(t)
    // `front` (called once, early in the phase) moves this wavefront's share of the K/V stream.
    bf16x8 kf[4], vf[4];
    auto phase = [&](const f32x16 &sp, f32x16 &sn, const u32x4 (&wp)[2], u32x4 (&wn)[2], int t, const char *k1,
                     const char *k2, const char *v0, const char *v1, auto &&front) {
        const StepScale sc = step_scale(t);
        const float bias0 = FP8 ? sc.lv[0] - mc : -mc, bias1 = FP8 ? sc.lv[1] - mc : -mc;
        float sum0 = 0.f, sum1 = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            // The empty asm statements are ordered like the fences; they pin each VALU group between
            // the two matrix instructions it is meant to follow (its inputs become available at the
            // first, its results are consumed at the second).
            const float ck = i < 4 ? sc.ck[0] : sc.ck[1], bias = i < 4 ? bias0 : bias1;
            float x0 = sp[2 * i], x1 = sp[2 * i + 1];
            sn = mfma32(kf[i & 3], qf[i], i == 0 ? zero16() : sn);
            kf[i & 3] = i < 4 ? lds_k(k1, i + 4) : lds_k(k2, i - 4);
            asm volatile("" : "+v"(x0));
            float p0 = fast_exp2(__builtin_fmaf(x0, ck, bias));
            asm volatile("" : "+v"(p0));
            __builtin_amdgcn_sched_barrier(0);
            o[i & 3] = mfma32(vf[i & 3], as_bf16x8(wp[i >> 2]), o[i & 3]);
            vf[i & 3] = i < 4 ? lds_v(v0, i + 4) : lds_v(v1, i - 4);
            asm volatile("" : "+v"(x1));
            const float p1 = fast_exp2(__builtin_fmaf(x1, ck, bias));
            if (FP8 && i >= 4)
                sum1 += p0 + p1;
            else
                sum0 += p0 + p1;
            uint32_t pk = pack_bf16(p0, p1);
            if constexpr (FP8)
                asm volatile("" : "+v"(pk), "+v"(sum0), "+v"(sum1));
            else
                asm volatile("" : "+v"(pk), "+v"(sum0));
            wn[i >> 2][i & 3] = pk;
            if (i == 2) front();
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (FP8)
            l_run += sum0 * sc.iv[0] + sum1 * sc.iv[1];
        else
            l_run += sum0;
    };

    u32x4 wa[2], wb[2];  // probabilities (packed bf16) of even and odd steps
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) wb[hf] = u32x4{0u, 0u, 0u, 0u};  // "P(-1)" = 0: phase 0 adds nothing to O^T
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        kf[i] = lds_k(k_tile(1), i);
        vf[i] = lds_v(v_tile(0), i);  // stands in for V(-1): finite data, multiplied by zeros
    }
    // Iteration j = phases 2j and 2j+1: reads K of blocks j, j+1 and V of blocks j-1, j.  The
    // wait at its end allows only its own requests to be outstanding, so K(j+2) and V(j+1) are
    // complete before iteration j+1 and a request has two iterations to land; K stage (j-1) % 4 and
    // V stage (j-2) % 4 are free from the barrier at the end of iteration j-1 on, which is where
    // iteration j's requests go.  One barrier per iteration.
    // fp8: kq_now / vq_now hold {K(j+2), V(j+1)} on entry and {K(j+4), V(j+3)} on exit; the other pair of
    // the register queue holds {K(j+3), V(j+2)} throughout (the two pairs swap roles every iteration).
    // The loop body exists four times, once per value of j % kStages, so that every LDS stage it touches is a
    // compile-time offset of its reads and writes instead of an address computed per access.
    auto iteration = [&](auto stage_tag, int j, u32x4 &kq_now, u32x4 &vq_now) {
        constexpr int S = decltype(stage_tag)::value;  // j % kStages
        // K resp. V tile of step 2j + c (c >= -1): block j + c / 2, half c % 2
        auto kt = [&](int c) { return sK[(S + kStages + (c >> 1)) % kStages] + (c & 1) * 8192; };
        auto vt = [&](int c) { return sV[(S + kStages + (c >> 1)) % kStages] + (c & 1) * 8192; };
        if constexpr (!FP8) {
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
        }
        const int t = 2 * j;
        if (j > 0 && j * KB + 31 > wave_min_pos) mask_scores(sa, t);
        phase(sa, sb, wb, wa, t, kt(1), kt(2), (S != 0 || j > 0) ? vt(-1) : vt(0), vt(0), [&]() {
            if constexpr (FP8) {  // widen {K(j+2), V(j+1)}: visible to everyone after this iteration's barrier
                store_k_fp8(kq_now, (S + 2) % kStages);
                store_v_fp8(vq_now, j + 1, (S + 1) % kStages);
            } else {
                issue_k_part(j + 3, 0, (S + 3) % kStages);
                issue_v_part(j + 2, 0, (S + 2) % kStages);
            }
        });
        if (j * KB + 63 > wave_min_pos) mask_scores(sb, t + 1);
        phase(sb, sa, wa, wb, t + 1, kt(2), kt(3), vt(0), vt(1), [&]() {
            if constexpr (FP8) {  // the request that takes the free place has two iterations to land
                kq_now = fetch_fp8(kbase, j + 4);
                vq_now = fetch_fp8(vbase, j + 3);
            } else {
                issue_k_part(j + 3, kParts - 1, (S + 3) % kStages);
                issue_v_part(j + 2, kParts - 1, (S + 2) % kStages);
            }
        });
        // (after the last block the K operands come from stale stages: in bounds, never used)
        if constexpr (FP8) {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        } else {
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(kLoadsPerBlock));
            __syncthreads();
            if ((j + 1) * KB + KB > kv_len && (j + 1) * KB < kv_len) {  // V(j+1) holds the sequence end
                zero_tail(j + 1, (S + 1) % kStages);
                __syncthreads();
            }
        }
    };
    for (int j = 0; j < n_blk; j += kStages) {
        iteration(std::integral_constant<int, 0>{}, j, kq[0], vq[0]);
        if (j + 1 >= n_blk) break;
        iteration(std::integral_constant<int, 1>{}, j + 1, kq[1], vq[1]);
        if (j + 2 >= n_blk) break;
        iteration(std::integral_constant<int, 2>{}, j + 2, kq[0], vq[0]);
        if (j + 3 >= n_blk) break;
        iteration(std::integral_constant<int, 3>{}, j + 3, kq[1], vq[1]);
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
    if (bail && tid == 0 && a.fallback_tiles) atomicAdd(a.fallback_tiles, 1u);
    float m_fin = mc;

    // =========================================================================================
    // fallback: classic online softmax with a running maximum, one 64-token block at a time.
    // Only taken when a row's later scores exceed its first ones by more than the exponent range
    // allows; always correct, not tuned.
    // =========================================================================================
    if (bail) {
        float m_run = -INFINITY;  // in units of scale * log2 e, like mc
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
            if constexpr (FP8) {
                store_k_fp8(fetch_fp8(kbase, j), 0);
                store_v_fp8(fetch_fp8(vbase, j), j, 0);
                __syncthreads();
            } else {
                issue_block(j, 0);
                __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
                __syncthreads();
                if (j * KB + KB > kv_len) {
                    zero_tail(j, 0);
                    __syncthreads();
                }
            }
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                f32x16 s;
                scores(s, sK[0] + mt * 8192);
                if (j * KB + mt * 32 + 31 > wave_min_pos) mask_scores(s, 2 * j + mt);
                const StepScale sc = step_scale(2 * j + mt);
                float mx = s[0] * sc.ck[0];
#pragma unroll
                for (int i = 1; i < 16; ++i) mx = fmaxf(mx, s[i] * sc.ck[i >> 3]);
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_new = fmaxf(m_run, mx);
                const float alpha = fast_exp2(m_run - m_new);
                float p[16];
                float sum0 = 0.f, sum1 = 0.f;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    p[i] = fast_exp2(__builtin_fmaf(s[i], sc.ck[i >> 3], sc.lv[i >> 3] - m_new));
                    if (i < 8)
                        sum0 += p[i];
                    else
                        sum1 += p[i];
                }
                u32x4 w[2];
                pack_probs(w, p);
                l_run = l_run * alpha + sum0 * sc.iv[0] + sum1 * sc.iv[1];
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
    float up = 1.f, down = 1.f;
    if constexpr (DECODE) {  // the partial goes out as fp16 times a power of two that puts the row's largest value near 2^14
        float amax = 0.f;
#pragma unroll
        for (int dm = 0; dm < 4; ++dm)
#pragma unroll
            for (int i = 0; i < 16; ++i) amax = fmaxf(amax, fabsf(o[dm][i]));
        amax = fmaxf(amax, __shfl_xor(amax, 32)) * (1.0f / l_tot);
        part_factors(amax, up, down);
        up *= 1.0f / l_tot;
    }
    if (tok < n_slots) {
        const float inv = 1.0f / l_tot;
        if constexpr (DECODE) {  // the row's partial for this chunk of the node
            const size_t part = (size_t)io_row * a.max_parts + it.part_slot;
            uint16_t *op = a.o_parts + part * kHeadDim + 4 * h;
#pragma unroll
            for (int dm = 0; dm < 4; ++dm)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    u32x2 w;
                    w[0] = pack_f16(o[dm][4 * q4] * up, o[dm][4 * q4 + 1] * up);
                    w[1] = pack_f16(o[dm][4 * q4 + 2] * up, o[dm][4 * q4 + 3] * up);
                    *reinterpret_cast<u32x2 *>(op + 32 * dm + 8 * q4) = w;
                }
            if (h == 0) a.down_parts[part] = down;
            if (h == 0) a.lse_parts[part] = (m_fin + fast_log2(l_tot)) * kLn2;
        } else {
            uint16_t *op = static_cast<uint16_t *>(a.out) + (size_t)io_row * kHeadDim;
#pragma unroll
            for (int dm = 0; dm < 4; ++dm)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    u32x2 w;
                    w[0] = pack_bf16(o[dm][4 * q4] * inv, o[dm][4 * q4 + 1] * inv);
                    w[1] = pack_bf16(o[dm][4 * q4 + 2] * inv, o[dm][4 * q4 + 3] * inv);
                    *reinterpret_cast<u32x2 *>(op + 32 * dm + 8 * q4 + 4 * h) = w;
                }
            if (a.lse_out && h == 0) a.lse_out[io_row] = (m_fin + fast_log2(l_tot)) * kLn2;
        }
    }
    if constexpr (!DECODE) break;
    }  // tiles of this workgroup
}

}  // namespace tile

}  // namespace hkv
