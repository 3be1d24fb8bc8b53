// Kernels of the 256-row attention tile (tile_body.h): suffix-only prefill (Section 5, "Token usage") and the
// decode work items shared by many query rows as a kernel of their own, for plans that run them next to
// the kernel of the other items on a second stream.
#include <hip/hip_ext.h>

#include "tile_body.h"

namespace hkv {

namespace {

using namespace tile;

template <bool DECODE, bool FP8>
__global__ __launch_bounds__(kThreads, 2) void attn_tile_kernel(TileArgs a) {
    __shared__ __attribute__((aligned(16))) char lds[kLdsBytes];
    body<DECODE, FP8>(a, lds, (int)blockIdx.x, (int)gridDim.x);
}

}  // namespace

int prefill_tile_tokens(int group) { return 256 / group; }

hipError_t launch_prefill(const PrefillLaunch &p, hipStream_t s) {
    if (p.n_tiles <= 0) return hipSuccess;
    TileArgs a{};
    a.pool = p.pool;
    a.q = p.q;
    a.tiles = p.tiles;
    a.ids = p.block_table;
    a.n_tiles = p.n_tiles;
    a.num_q_heads = p.num_q_heads;
    a.scale = p.scale;
    a.out = p.out;
    a.lse_out = p.lse_out;
    a.fallback_tiles = p.fallback_tiles;
    hipLaunchKernelGGL((attn_tile_kernel<false, false>), dim3(p.n_tiles), dim3(kThreads), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_decode_tiles(const DecodeTilesLaunch &d, hipStream_t s, hipEvent_t ev_begin, hipEvent_t ev_end) {
    if (d.n_items <= 0) return hipSuccess;
    if (d.n_workgroups <= 0 || (d.pool.dtype != 0 && d.pool.dtype != 1)) return hipErrorInvalidValue;
    TileArgs a{};
    a.pool = d.pool;
    a.q = d.q;
    a.tiles = d.items;
    a.ids = d.pages;
    a.n_tiles = d.n_items;
    a.num_q_heads = d.num_q_heads;
    a.scale = d.scale;
    a.node_req_idx = d.node_req_idx;
    a.o_parts = d.o_parts;
    a.lse_parts = d.lse_parts;
    a.max_parts = d.max_parts;
    a.down_parts = d.down_parts;
    a.q_rows = d.q_rows;
    const dim3 grid(d.n_workgroups < d.n_items ? d.n_workgroups : d.n_items);
    if (d.pool.dtype == 0)
        hipExtLaunchKernelGGL((attn_tile_kernel<true, false>), grid, dim3(kThreads), 0, s, ev_begin, ev_end, 0, a);
    else
        hipExtLaunchKernelGGL((attn_tile_kernel<true, true>), grid, dim3(kThreads), 0, s, ev_begin, ev_end, 0, a);
    return hipGetLastError();
}

}  // namespace hkv
