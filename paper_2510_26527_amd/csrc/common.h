// Shared device helpers for the gfx950 kernels: bf16 conversion, wavefront (64-lane)
// reductions, MFMA operand types.  Host code includes it only for the typedefs.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace psd {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;   // one MFMA A/B operand (8 k-values)
typedef __attribute__((ext_vector_type(4))) float f32x4;     // 16x16 MFMA accumulator
typedef __attribute__((ext_vector_type(16))) float f32x16;   // 32x32 MFMA accumulator
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;  // a 16-byte load

typedef __attribute__((ext_vector_type(8))) float f32x8;

constexpr int kWave = 64;

// An fp32 activation as a pair of bf16 values hi + lo (hi = RNE(x), lo = RNE(x - hi)): fed to
// two MFMAs it carries ~16 mantissa bits through the bf16 matrix cores.
__device__ __forceinline__ void split_bf16(const f32x8 &x, bf16x8 *hi, bf16x8 *lo) {
    const bf16x8 h = __builtin_convertvector(x, bf16x8);
    *hi = h;
    *lo = __builtin_convertvector(x - __builtin_convertvector(h, f32x8), bf16x8);
}
__device__ __forceinline__ f32x8 load_f32x8(const float *p) {
    const f32x4 a = *reinterpret_cast<const f32x4 *>(p);
    const f32x4 b = *reinterpret_cast<const f32x4 *>(p + 4);
    return f32x8{a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// round-to-nearest-even fp32 -> bf16 bit pattern (NaN stays NaN)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

// round-to-nearest-even fp32 -> fp16 bit pattern
__device__ __forceinline__ uint16_t f32_to_f16_bits(float f) {
    const _Float16 h = (_Float16)f;
    return __builtin_bit_cast(uint16_t, h);
}

// element loads / stores by storage type
__device__ __forceinline__ float load_elem(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_elem(const uint16_t *p, size_t i) { return bf16_bits_to_f32(p[i]); }
__device__ __forceinline__ void store_elem(float *p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void store_elem(uint16_t *p, size_t i, float v) { p[i] = (uint16_t)f32_to_bf16_bits(v); }

typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;

// 8 bf16 (as stored) -> 8 fp16, exact for every value the fp16 grid holds
__device__ __forceinline__ u32x4 bf16x8_to_f16x8(u32x4 w) {
    u32x4 r;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const auto h = __builtin_amdgcn_cvt_pkrtz(__uint_as_float(w[e] << 16), __uint_as_float(w[e] & 0xffff0000u));
        r[e] = __builtin_bit_cast(uint32_t, h);
    }
    return r;
}
// 8 fp32 -> 8 fp16, round to nearest even
__device__ __forceinline__ u32x4 f32x8_to_f16x8(const f32x8 &x) {
    const f16x8 h = __builtin_convertvector(x, f16x8);
    return __builtin_bit_cast(u32x4, h);
}

template <typename T>
__device__ __forceinline__ T wave_max(T v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        T other = __shfl_xor(v, o, kWave);
        v = other > v ? other : v;
    }
    return v;
}
// butterfly sum: every lane ends with the same value, summed in a fixed tree order
template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

}  // namespace psd
