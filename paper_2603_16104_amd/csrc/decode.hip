// Kernels of the decode plans: the per-node kernel over the items few query rows share (rows_body.h), and
// the launch that runs those items and the items of the 256-row tile (tile_body.h) as ONE kernel, so that
// a step needs neither a second stream nor events between streams (Section 5, "Proactive Cache Management":
// the shared prefix is computed once per node, the private branches beside it).
#include <mutex>

#include <hip/hip_ext.h>

#include "rows_body.h"
#include "tile_body.h"

namespace hkv {

namespace {

using rows::kMaxStages;
using rows::kMinStages;
using rows::kStageBytes;

template <int DT>
__global__ __launch_bounds__(rows::kThreads, DT == 0 ? 3 : 2) void decode_node_kernel(DecodeLaunch a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];  // a.n_stages * kStageBytes
    rows::body<DT, false>(a, smem, (int)blockIdx.x, (int)threadIdx.x);
}

// Workgroups [0, n_tile_wgs) are the persistent workgroups of the tile items (all 512 threads); each
// workgroup behind them runs two blocks of the other items, one per half.  Dispatch follows the workgroup
// index, so the tile workgroups, which need a whole compute unit each, are placed first.
constexpr int kFusedLds = tile::kLdsBytes > 2 * rows::kCombineBytes ? tile::kLdsBytes : 2 * rows::kCombineBytes;
template <bool FP8>
__global__ __launch_bounds__(tile::kThreads, 2) void decode_fused_kernel(DecodeLaunch r, tile::TileArgs t, int n_tile_wgs) {
    extern __shared__ __attribute__((aligned(16))) char smem[];  // kFusedLds
    if ((int)blockIdx.x < n_tile_wgs) {
        tile::body<true, FP8>(t, smem, (int)blockIdx.x, n_tile_wgs);
    } else {
        const int half = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 8);  // wavefront-uniform: keeps the item in scalar registers
        rows::body<FP8 ? 1 : 0, true>(r, smem + half * rows::kCombineBytes, 2 * ((int)blockIdx.x - n_tile_wgs) + half,
                                      (int)threadIdx.x & 255);
    }
}

}  // namespace

// Per-device set-up of the decode path, done once per device with that device current (at plan creation,
// i.e. outside any graph capture): more than 64 KiB of LDS per workgroup has to be allowed once per kernel
// variant (0 bf16 pool, 1 fp8 pool with codes widened to bf16, 2 fp8 pool on the fp8 matrix instruction),
// and the device's own copy of the static workspace below is looked up.
namespace {
constexpr int kMaxDevices = 64;
struct DeviceSetup {
    std::once_flag once;
    hipError_t err = hipSuccess;
    void *static_ws = nullptr;  // this device's address of `scratch`
};
DeviceSetup g_setup[kMaxDevices];
}  // namespace
}  // namespace hkv

// Workspace of attn_decode_plan_run_static, for callers that cannot allocate device memory: the partial
// results (o, lse) of one decode step.  Every GPU the library runs on holds its own copy at its own
// address until the process ends.  In host code the name below is only a handle for hipGetSymbolAddress:
// kernels, copies and fills get the looked-up device address, never the name.
static __device__ __align__(256) unsigned char scratch[hkv::kStaticWorkspaceBytes];

namespace hkv {

static hipError_t setup_device(DeviceSetup &st) {
    const void *fns[3] = {reinterpret_cast<const void *>(decode_node_kernel<0>),
                          reinterpret_cast<const void *>(decode_node_kernel<1>),
                          reinterpret_cast<const void *>(decode_node_kernel<2>)};
    for (const void *fn : fns)
        if (hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxStages * kStageBytes);
            e != hipSuccess)
            return e;
    const void *fused[2] = {reinterpret_cast<const void *>(decode_fused_kernel<false>),
                            reinterpret_cast<const void *>(decode_fused_kernel<true>)};
    for (const void *fn : fused)
        if (hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kFusedLds); e != hipSuccess)
            return e;
    return hipGetSymbolAddress(&st.static_ws, HIP_SYMBOL(scratch));
}

hipError_t prepare_decode_device(void **static_ws) {
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    DeviceSetup &st = g_setup[dev];
    std::call_once(st.once, [&st] { st.err = setup_device(st); });
    if (st.err != hipSuccess) return st.err;
    if (static_ws) *static_ws = st.static_ws;
    return hipSuccess;
}

// With events, they are bound to the dispatch itself (begin and end of the kernel on the device), so
// their difference is the kernel's duration without the gap to its neighbours in the queue.
hipError_t launch_decode(const DecodeLaunch &a, hipStream_t s, hipEvent_t ev_begin, hipEvent_t ev_end) {
    if (a.n_items <= 0) return hipSuccess;
    if (a.n_stages < kMinStages || a.n_stages > kMaxStages) return hipErrorInvalidValue;
    const int variant = a.pool.dtype == 0 ? 0 : a.fp8_matrix ? 2 : 1;
    if (hipError_t e = prepare_decode_device(nullptr); e != hipSuccess) return e;
    const dim3 grid(a.n_single + (a.n_items - a.n_single + rows::kWaves - 1) / rows::kWaves);
    const unsigned lds = (unsigned)a.n_stages * kStageBytes;
    if (variant == 0)
        hipExtLaunchKernelGGL(decode_node_kernel<0>, grid, dim3(rows::kThreads), lds, s, ev_begin, ev_end, 0, a);
    else if (variant == 1)
        hipExtLaunchKernelGGL(decode_node_kernel<1>, grid, dim3(rows::kThreads), lds, s, ev_begin, ev_end, 0, a);
    else
        hipExtLaunchKernelGGL(decode_node_kernel<2>, grid, dim3(rows::kThreads), lds, s, ev_begin, ev_end, 0, a);
    return hipGetLastError();
}

// Both kinds of items in one launch.  The caller guarantees that no item of `a` is shared by more than 16
// query rows (such items synchronise their workgroup once per step, which two halves cannot do apart).
hipError_t launch_decode_fused(const DecodeLaunch &a, const DecodeTilesLaunch &d, hipStream_t s, hipEvent_t ev_begin,
                               hipEvent_t ev_end) {
    if (a.n_items <= 0 || d.n_items <= 0 || d.n_workgroups <= 0) return hipErrorInvalidValue;
    if ((a.pool.dtype != 0 && a.pool.dtype != 1) || a.fp8_matrix) return hipErrorInvalidValue;
    if (hipError_t e = prepare_decode_device(nullptr); e != hipSuccess) return e;
    tile::TileArgs t{};
    t.pool = d.pool;
    t.q = d.q;
    t.tiles = d.items;
    t.ids = d.pages;
    t.n_tiles = d.n_items;
    t.num_q_heads = d.num_q_heads;
    t.scale = d.scale;
    t.node_req_idx = d.node_req_idx;
    t.o_parts = d.o_parts;
    t.lse_parts = d.lse_parts;
    t.down_parts = d.down_parts;
    t.max_parts = d.max_parts;
    t.q_rows = d.q_rows;
    const int n_tile_wgs = d.n_workgroups < d.n_items ? d.n_workgroups : d.n_items;
    const int n_blocks = a.n_single + (a.n_items - a.n_single + rows::kWaves - 1) / rows::kWaves;
    const dim3 grid(n_tile_wgs + (n_blocks + 1) / 2);
    if (a.pool.dtype == 0)
        hipExtLaunchKernelGGL(decode_fused_kernel<false>, grid, dim3(tile::kThreads), kFusedLds, s, ev_begin, ev_end, 0, a, t, n_tile_wgs);
    else
        hipExtLaunchKernelGGL(decode_fused_kernel<true>, grid, dim3(tile::kThreads), kFusedLds, s, ev_begin, ev_end, 0, a, t, n_tile_wgs);
    return hipGetLastError();
}

}  // namespace hkv
