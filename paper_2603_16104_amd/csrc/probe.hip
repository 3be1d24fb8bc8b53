// Matrix-core ceiling probe: a register-only stream of v_mfma_f32_32x32x16_bf16 on every SIMD,
// timed with HIP events and with the core-clock and 100 MHz counters inside the kernel.  It answers
// "what can this chip sustain when nothing but the matrix cores is busy", with all-zero operands
// (little switching activity) or with random ones (the realistic case: the clock drops under the
// power limit), so that the fraction a real kernel reaches can be set against that figure as well
// as against the data-sheet peak.
#include <hip/hip_runtime.h>

#include "hkv_device.h"

namespace hkv {

namespace {

typedef __attribute__((ext_vector_type(16))) float probe_f32x16;

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
    probe_f32x16 acc[4];
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

// Plain streaming read: every lane fetches 16 bytes at a time, four loads in flight per lane, the
// grid walks the buffer once; the xor of what was read goes to one word per workgroup so that the
// loads cannot be dropped.
__global__ __launch_bounds__(256) void read_probe_kernel(const u32x4 *__restrict__ src, size_t n_vec, uint32_t *sink) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (; i + 3 * stride < n_vec; i += 4 * stride) {
        const u32x4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        acc ^= a ^ b ^ c ^ d;
    }
    for (; i < n_vec; i += stride) acc ^= src[i];
    uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
#pragma unroll
    for (int o = 32; o; o >>= 1) x ^= __shfl_xor(x, o);
    if ((threadIdx.x & 63) == 0) atomicXor(&sink[blockIdx.x], x);
}

}  // namespace

// Reads each of the n_buf buffers (bytes each) in turn, `reps` launches in total, one event pair
// around all of them; returns bytes * reps / time.
hipError_t run_read_probe(const void *const *bufs, int n_buf, size_t bytes, int reps, int n_cu, float *gbps,
                          hipStream_t s) {
    const int grid = n_cu * 8;
    uint32_t *sink = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t rc = hipMalloc(&sink, sizeof(uint32_t) * grid);
    if (rc == hipSuccess) rc = hipMemsetAsync(sink, 0, sizeof(uint32_t) * grid, s);
    if (rc == hipSuccess) rc = hipEventCreate(&e0);
    if (rc == hipSuccess) rc = hipEventCreate(&e1);
    const size_t n_vec = bytes / 16;
    for (int i = 0; i < n_buf && rc == hipSuccess; ++i) {  // warm-up: one pass over every buffer
        hipLaunchKernelGGL(read_probe_kernel, dim3(grid), dim3(256), 0, s, static_cast<const u32x4 *>(bufs[i]), n_vec, sink);
        rc = hipGetLastError();
    }
    if (rc == hipSuccess) rc = hipEventRecord(e0, s);
    for (int i = 0; i < reps && rc == hipSuccess; ++i) {
        hipLaunchKernelGGL(read_probe_kernel, dim3(grid), dim3(256), 0, s, static_cast<const u32x4 *>(bufs[i % n_buf]), n_vec, sink);
        rc = hipGetLastError();
    }
    if (rc == hipSuccess) rc = hipEventRecord(e1, s);
    if (rc == hipSuccess) rc = hipEventSynchronize(e1);
    float ms = 0.f;
    if (rc == hipSuccess) rc = hipEventElapsedTime(&ms, e0, e1);
    if (rc == hipSuccess) *gbps = (float)((double)n_vec * 16.0 * reps / (ms * 1e-3) / 1e9);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (sink) (void)hipFree(sink);
    return rc;
}

// Runs the probe on `n_cu` workgroups of 64*waves threads.  Returns TFLOP/s by event time and the
// core clock in GHz (median over workgroups of core ticks / reference ticks).
hipError_t run_mfma_probe(int n_cu, int waves, int iters, int random_operands, float *tflops, float *clock_ghz,
                          hipStream_t s) {
    float *sink = nullptr;
    unsigned long long *ticks = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t rc = hipMalloc(&sink, sizeof(float) * n_cu * 64 * waves);
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
    return rc;
}

}  // namespace hkv
