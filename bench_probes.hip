// Ceiling probes for bench.py (measurement aids, no part of the attention library): what this chip
// sustains when a kernel does nothing but read HBM, or nothing but issue bf16 matrix instructions.
// Built into libbench_probes.so beside bench.py; plain C entry points, called through ctypes.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// Register-only stream of v_mfma_f32_32x32x16_bf16 (the instruction the prefill kernel is built on),
// four independent accumulators per wavefront, all-zero operands (little switching activity) or
// random ones (the realistic case: the clock drops under the power limit).
__global__ __launch_bounds__(512) void mfma_probe_kernel(float *sink, unsigned long long *ticks, int iters, int random_operands) {
    bf16x8 a, b;
    uint32_t x = (blockIdx.x * 1024u + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        x ^= x << 13; x ^= x >> 17; x ^= x << 5;
        a[i] = random_operands ? (__bf16)(((int)(x & 0xFFFF) - 32768) * (1.0f / 32768)) : (__bf16)0.f;
        x ^= x << 13; x ^= x >> 17; x ^= x << 5;
        b[i] = random_operands ? (__bf16)(((int)(x & 0xFFFF) - 32768) * (1.0f / 32768)) : (__bf16)0.f;
    }
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
    const unsigned long long c0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[j][i];
    const unsigned long long c1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
    sink[blockIdx.x * blockDim.x + threadIdx.x] = s;
    if (threadIdx.x == 0) {
        ticks[2 * blockIdx.x] = c1 - c0;      // core clock cycles
        ticks[2 * blockIdx.x + 1] = r1 - r0;  // 100 MHz reference
    }
}

// Plain streaming read.  Every lane fetches 16 bytes at a time, IN_FLIGHT loads outstanding per lane;
// a workgroup walks a contiguous slab of the buffer (CONTIG) or the whole grid strides over it.  The
// xor of what was read goes to one word per workgroup so that the loads cannot be dropped.
template <int IN_FLIGHT, bool NONTEMPORAL>
__global__ __launch_bounds__(1024) void read_probe_kernel(const u32x4 *__restrict__ src, size_t n_vec, int contiguous,
                                                           uint32_t *sink) {
    size_t i, end, stride;
    if (contiguous) {  // workgroup b reads vectors [b * per, (b + 1) * per)
        const size_t per = (n_vec + gridDim.x - 1) / gridDim.x;
        i = (size_t)blockIdx.x * per + threadIdx.x;
        end = per * (blockIdx.x + 1) < n_vec ? per * (blockIdx.x + 1) : n_vec;
        stride = blockDim.x;
    } else {
        i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
        end = n_vec;
        stride = (size_t)gridDim.x * blockDim.x;
    }
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (; i + (IN_FLIGHT - 1) * stride < end; i += IN_FLIGHT * stride) {
        u32x4 v[IN_FLIGHT];
#pragma unroll
        for (int j = 0; j < IN_FLIGHT; ++j)
            v[j] = NONTEMPORAL ? __builtin_nontemporal_load(src + i + j * stride) : src[i + j * stride];
#pragma unroll
        for (int j = 0; j < IN_FLIGHT; ++j) acc ^= v[j];
    }
    for (; i < end; i += stride) acc ^= src[i];
    uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
#pragma unroll
    for (int o = 32; o; o >>= 1) x ^= __shfl_xor(x, o);
    if ((threadIdx.x & 63) == 0) atomicXor(&sink[blockIdx.x], x);
}

// Paged read: the buffer is cut into blocks of BLOCK_VEC 16-byte vectors (a (page, head) block of a KV pool:
// 2 KiB for fp8, 4 KiB for bf16); wavefront w of the grid reads the blocks order[w], order[w + n_waves], ...
// whole, all of a block's loads (BLOCK_VEC / 64 per lane) issued together and `depth` blocks requested
// before the first is consumed.  This is the access pattern of a decode step over randomly placed pages.
template <int BLOCK_VEC, int DEPTH, bool NONTEMPORAL>
__global__ __launch_bounds__(1024) void paged_read_kernel(const u32x4 *__restrict__ src, const int32_t *__restrict__ order,
                                                           int n_blocks, uint32_t *sink) {
    constexpr int PER_LANE = BLOCK_VEC / 64;
    const int lane = threadIdx.x & 63;
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int n_waves = (gridDim.x * blockDim.x) >> 6;
    u32x4 acc = {0u, 0u, 0u, 0u};
    u32x4 v[DEPTH][PER_LANE];
    int b = wave;
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
        const int bb = b + d * n_waves;
        const int id = order[bb < n_blocks ? bb : n_blocks - 1];
        const u32x4 *p = src + (size_t)id * BLOCK_VEC + lane;
#pragma unroll
        for (int j = 0; j < PER_LANE; ++j) v[d][j] = NONTEMPORAL ? __builtin_nontemporal_load(p + 64 * j) : p[64 * j];
    }
    for (; b < n_blocks; b += DEPTH * n_waves) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            if (b + d * n_waves < n_blocks) {
#pragma unroll
                for (int j = 0; j < PER_LANE; ++j) acc ^= v[d][j];
            }
            const int bb = b + (d + DEPTH) * n_waves;
            const int id = order[bb < n_blocks ? bb : n_blocks - 1];
            const u32x4 *p = src + (size_t)id * BLOCK_VEC + lane;
#pragma unroll
            for (int j = 0; j < PER_LANE; ++j) v[d][j] = NONTEMPORAL ? __builtin_nontemporal_load(p + 64 * j) : p[64 * j];
        }
    }
    uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
#pragma unroll
    for (int o = 32; o; o >>= 1) x ^= __shfl_xor(x, o);
    if (lane == 0) atomicXor(&sink[blockIdx.x], x);
}

template <int BLOCK_VEC, bool NT>
hipError_t launch_paged(int depth, int grid, int threads, const u32x4 *src, const int32_t *order, int n_blocks, uint32_t *sink,
                        hipStream_t s) {
    switch (depth) {
        case 1: hipLaunchKernelGGL((paged_read_kernel<BLOCK_VEC, 1, NT>), dim3(grid), dim3(threads), 0, s, src, order, n_blocks, sink); break;
        case 2: hipLaunchKernelGGL((paged_read_kernel<BLOCK_VEC, 2, NT>), dim3(grid), dim3(threads), 0, s, src, order, n_blocks, sink); break;
        case 4: hipLaunchKernelGGL((paged_read_kernel<BLOCK_VEC, 4, NT>), dim3(grid), dim3(threads), 0, s, src, order, n_blocks, sink); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <bool NT>
hipError_t launch_read(int in_flight, int grid, int threads, const u32x4 *src, size_t n_vec, int contiguous, uint32_t *sink,
                       hipStream_t s) {
    switch (in_flight) {
        case 1: hipLaunchKernelGGL((read_probe_kernel<1, NT>), dim3(grid), dim3(threads), 0, s, src, n_vec, contiguous, sink); break;
        case 2: hipLaunchKernelGGL((read_probe_kernel<2, NT>), dim3(grid), dim3(threads), 0, s, src, n_vec, contiguous, sink); break;
        case 4: hipLaunchKernelGGL((read_probe_kernel<4, NT>), dim3(grid), dim3(threads), 0, s, src, n_vec, contiguous, sink); break;
        case 8: hipLaunchKernelGGL((read_probe_kernel<8, NT>), dim3(grid), dim3(threads), 0, s, src, n_vec, contiguous, sink); break;
        case 16: hipLaunchKernelGGL((read_probe_kernel<16, NT>), dim3(grid), dim3(threads), 0, s, src, n_vec, contiguous, sink); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

extern "C" {

// Launches the read kernel `reps` times back to back, launch i over bufs[i % n_buf] (`bytes` each, a
// multiple of 16, 16-byte aligned device buffers owned by the caller), after one untimed pass over
// every buffer; with buffers larger in sum than the last-level cache every launch reads HBM.
//   wgs_per_cu x (compute units) workgroups of `threads` (64..1024, multiple of 64) threads,
//   in_flight in {1, 2, 4, 8, 16} 16-byte loads outstanding per lane, contiguous: slab per workgroup (1)
//   or grid-strided (0), nontemporal: loads carry the streaming hint (1) or not (0).
// gbps (host): bytes * reps / time between two HIP events around the timed launches (launch gaps
// included, as in a real step).  Blocks until done.  Returns a hipError_t value (0 = success).
int probe_hbm_read(const void *const *bufs, int n_buf, size_t bytes, int reps, int wgs_per_cu, int threads,
                   int in_flight, int contiguous, int nontemporal, float *gbps, void *stream) {
    if (!bufs || !gbps || n_buf < 1 || reps < 1 || bytes < 16 || bytes % 16 || wgs_per_cu < 1 || threads < 64 ||
        threads > 1024 || threads % 64)
        return (int)hipErrorInvalidValue;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int dev = 0, n_cu = 0;
    hipError_t rc = hipGetDevice(&dev);
    if (rc == hipSuccess) rc = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
    if (rc != hipSuccess) return (int)rc;
    const int grid = n_cu * wgs_per_cu;
    uint32_t *sink = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    rc = hipMalloc(&sink, sizeof(uint32_t) * grid);
    if (rc == hipSuccess) rc = hipMemsetAsync(sink, 0, sizeof(uint32_t) * grid, s);
    if (rc == hipSuccess) rc = hipEventCreate(&e0);
    if (rc == hipSuccess) rc = hipEventCreate(&e1);
    const size_t n_vec = bytes / 16;
    auto go = [&](const void *buf) {
        const u32x4 *p = static_cast<const u32x4 *>(buf);
        return nontemporal ? launch_read<true>(in_flight, grid, threads, p, n_vec, contiguous, sink, s)
                           : launch_read<false>(in_flight, grid, threads, p, n_vec, contiguous, sink, s);
    };
    for (int i = 0; i < n_buf && rc == hipSuccess; ++i) rc = go(bufs[i]);
    if (rc == hipSuccess) rc = hipEventRecord(e0, s);
    for (int i = 0; i < reps && rc == hipSuccess; ++i) rc = go(bufs[i % n_buf]);
    if (rc == hipSuccess) rc = hipEventRecord(e1, s);
    if (rc == hipSuccess) rc = hipEventSynchronize(e1);
    float ms = 0.f;
    if (rc == hipSuccess) rc = hipEventElapsedTime(&ms, e0, e1);
    if (rc == hipSuccess) *gbps = (float)((double)n_vec * 16.0 * reps / (ms * 1e-3) / 1e9);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (sink) (void)hipFree(sink);
    return (int)rc;
}

// The paged variant: every buffer is read as n_blocks blocks of block_bytes (2048 or 4096) in the order
// given by `order` (device, int32 [n_blocks], a permutation), one block per wavefront at a time, `depth`
// (1, 2 or 4) blocks requested ahead per wavefront.  Other arguments and the result as probe_hbm_read.
int probe_hbm_paged_read(const void *const *bufs, int n_buf, const int32_t *order, int n_blocks, int block_bytes, int reps,
                         int wgs_per_cu, int threads, int depth, int nontemporal, float *gbps, void *stream) {
    if (!bufs || !order || !gbps || n_buf < 1 || reps < 1 || n_blocks < 1 || (block_bytes != 2048 && block_bytes != 4096) ||
        wgs_per_cu < 1 || threads < 64 || threads > 1024 || threads % 64)
        return (int)hipErrorInvalidValue;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int dev = 0, n_cu = 0;
    hipError_t rc = hipGetDevice(&dev);
    if (rc == hipSuccess) rc = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
    if (rc != hipSuccess) return (int)rc;
    const int grid = n_cu * wgs_per_cu;
    uint32_t *sink = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    rc = hipMalloc(&sink, sizeof(uint32_t) * grid);
    if (rc == hipSuccess) rc = hipMemsetAsync(sink, 0, sizeof(uint32_t) * grid, s);
    if (rc == hipSuccess) rc = hipEventCreate(&e0);
    if (rc == hipSuccess) rc = hipEventCreate(&e1);
    auto go = [&](const void *buf) {
        const u32x4 *p = static_cast<const u32x4 *>(buf);
        if (block_bytes == 2048)
            return nontemporal ? launch_paged<128, true>(depth, grid, threads, p, order, n_blocks, sink, s)
                               : launch_paged<128, false>(depth, grid, threads, p, order, n_blocks, sink, s);
        return nontemporal ? launch_paged<256, true>(depth, grid, threads, p, order, n_blocks, sink, s)
                           : launch_paged<256, false>(depth, grid, threads, p, order, n_blocks, sink, s);
    };
    for (int i = 0; i < n_buf && rc == hipSuccess; ++i) rc = go(bufs[i]);
    if (rc == hipSuccess) rc = hipEventRecord(e0, s);
    for (int i = 0; i < reps && rc == hipSuccess; ++i) rc = go(bufs[i % n_buf]);
    if (rc == hipSuccess) rc = hipEventRecord(e1, s);
    if (rc == hipSuccess) rc = hipEventSynchronize(e1);
    float ms = 0.f;
    if (rc == hipSuccess) rc = hipEventElapsedTime(&ms, e0, e1);
    if (rc == hipSuccess) *gbps = (float)((double)n_blocks * block_bytes * reps / (ms * 1e-3) / 1e9);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (sink) (void)hipFree(sink);
    return (int)rc;
}

// Runs the matrix-core stream on one workgroup per compute unit, waves_per_simd in {1, 2} wavefronts
// per SIMD, iters x 4 instructions per wavefront.  tflops (host): dense bf16 TFLOP/s by HIP event
// time; clock_ghz (host): core clock during the run, from the core-cycle and 100 MHz counters read
// inside the kernel.  Blocks until done.  Returns a hipError_t value.
int probe_mfma_bf16(int iters, int random_operands, int waves_per_simd, float *tflops, float *clock_ghz, void *stream) {
    if (!tflops || !clock_ghz || iters < 1 || (waves_per_simd != 1 && waves_per_simd != 2)) return (int)hipErrorInvalidValue;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int dev = 0, n_cu = 0;
    hipError_t rc = hipGetDevice(&dev);
    if (rc == hipSuccess) rc = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
    if (rc != hipSuccess) return (int)rc;
    const int waves = 4 * waves_per_simd;
    float *sink = nullptr;
    unsigned long long *ticks = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    rc = hipMalloc(&sink, sizeof(float) * n_cu * 64 * waves);
    if (rc == hipSuccess) rc = hipMalloc(&ticks, sizeof(unsigned long long) * 2 * n_cu);
    if (rc == hipSuccess) rc = hipEventCreate(&e0);
    if (rc == hipSuccess) rc = hipEventCreate(&e1);
    if (rc == hipSuccess) {
        hipLaunchKernelGGL(mfma_probe_kernel, dim3(n_cu), dim3(64 * waves), 0, s, sink, ticks, iters / 10 + 1, random_operands);
        rc = hipEventRecord(e0, s);
    }
    if (rc == hipSuccess) {
        hipLaunchKernelGGL(mfma_probe_kernel, dim3(n_cu), dim3(64 * waves), 0, s, sink, ticks, iters, random_operands);
        rc = hipGetLastError();
    }
    if (rc == hipSuccess) rc = hipEventRecord(e1, s);
    if (rc == hipSuccess) rc = hipEventSynchronize(e1);
    float ms = 0.f;
    if (rc == hipSuccess) rc = hipEventElapsedTime(&ms, e0, e1);
    if (rc == hipSuccess) {
        unsigned long long *h = new unsigned long long[2 * n_cu];
        rc = hipMemcpy(h, ticks, sizeof(unsigned long long) * 2 * n_cu, hipMemcpyDeviceToHost);
        if (rc == hipSuccess) {
            // the middle workgroup's ratio; all of them run the same stream for the same time
            const unsigned long long c = h[2 * (n_cu / 2)], r = h[2 * (n_cu / 2) + 1];
            *clock_ghz = r ? 0.1f * (float)c / (float)r : 0.f;
            *tflops = (float)((double)n_cu * waves * iters * 4.0 * 32768.0 / (ms * 1e-3) / 1e12);
        }
        delete[] h;
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (sink) (void)hipFree(sink);
    if (ticks) (void)hipFree(ticks);
    return (int)rc;
}

}  // extern "C"
