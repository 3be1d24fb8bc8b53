// Device-side helpers shared by the gfx950 kernels: matrix-core operand types, bf16/fp8
// conversions and cross-lane reductions for 64-wide wavefronts.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hkv_internal.h"

namespace hkv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// 16-byte global load of matrix-core operand data (8 bf16 or 16 fp8).
__device__ __forceinline__ u32x4 ld16(const void *p) { return *reinterpret_cast<const u32x4 *>(p); }
// The same with the streaming hint: for bytes that are read once per launch (K/V of a node that few query
// rows share), so that they do not displace what other workgroups will read again.
__device__ __forceinline__ u32x4 ld16_stream(const void *p) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
}

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// float -> bf16 bits, round to nearest even (inputs here are finite or +-inf, never NaN payloads
// that matter).  The compiler turns the pair form into the packed convert of gfx950.
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    bf16x2 v;
    v[0] = (__bf16)lo;
    v[1] = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, v);
}

// Partial results of the decode plans travel as fp16 with one power-of-two factor per partial (a row of 128
// values): 11 significant bits relative to the row's largest magnitude, so that what the merge reads carries
// more precision than the bf16 output it produces, at half the bytes of fp32.
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
__device__ __forceinline__ uint32_t pack_f16(float lo, float hi) {
    f16x2 v;
    v[0] = (_Float16)lo;
    v[1] = (_Float16)hi;
    return __builtin_bit_cast(uint32_t, v);
}
// For a row whose largest magnitude is amax: `up` = power of two with amax * up in [2^14, 2^15) (fp16 holds
// up to 65504), `down` = 1 / up.  amax = 0 or tiny: up = 2^114; inf / NaN rows stay inf / NaN.
__device__ __forceinline__ void part_factors(float amax, float &up, float &down) {
    const uint32_t e = max((__float_as_uint(amax) >> 23) & 0xFFu, 27u);
    up = __uint_as_float((268u - e) << 23);
    down = __uint_as_float((e - 14u) << 23);
}

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// Eight e4m3 codes (two dwords) -> eight bf16 (exact: every e4m3 value is a bf16 value), one
// instruction per pair (v_cvt_scalef32_pk_bf16_fp8 with scale 1; its results equal the two-step
// conversion through float bit for bit on all 256 codes).
__device__ __forceinline__ bf16x8 fp8x8_to_bf16x8(uint32_t w0, uint32_t w1) {
    u32x4 r;
    r[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w0, 1.0f, false));
    r[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w0, 1.0f, true));
    r[2] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w1, 1.0f, false));
    r[3] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w1, 1.0f, true));
    return as_bf16x8(r);
}

// Reductions across the four 16-lane rows of a wavefront (lanes l, l^16, l^32, l^48 hold the
// same matrix column): after the call every lane holds the result.  v_permlane16_swap exchanges the
// odd rows of its first operand with the even rows of its second, v_permlane32_swap the upper half of
// the first with the lower half of the second; fed the same value twice they return (even rows twice,
// odd rows twice) resp. (lower half twice, upper half twice), all in the vector ALU, where a shuffle
// through ds_bpermute would be an LDS round trip in the middle of every softmax step.
__device__ __forceinline__ float rows_max(float v) {
    uint32_t x = __float_as_uint(v);
    const auto a = __builtin_amdgcn_permlane16_swap(x, x, false, false);
    x = __float_as_uint(fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1])));
    const auto b = __builtin_amdgcn_permlane32_swap(x, x, false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float rows_sum(float v) {
    uint32_t x = __float_as_uint(v);
    const auto a = __builtin_amdgcn_permlane16_swap(x, x, false, false);
    x = __float_as_uint(__uint_as_float(a[0]) + __uint_as_float(a[1]));
    const auto b = __builtin_amdgcn_permlane32_swap(x, x, false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

}  // namespace hkv
