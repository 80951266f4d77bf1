// Shared device/host helpers of the ADPSGD library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace adpsgd {

typedef uint16_t bf16_t;   // raw bfloat16 bits
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

// fp32 -> bf16, round to nearest even, on the gfx950 conversion unit (v_cvt_pk_bf16_f32).
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
__device__ inline bf16_t f32_to_bf16(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }
// two values into one register: lo in bits 0..15, hi in bits 16..31
__device__ inline uint32_t pack_bf16(float lo, float hi) {
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__host__ __device__ inline float bf16_to_f32(bf16_t h) {
    return __builtin_bit_cast(float, (uint32_t)h << 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    __device__ static float from(float v) { return v; }
    __device__ static float to(float v) { return v; }
};
template <> struct Elem<bf16_t> {
    __device__ static bf16_t from(float v) { return f32_to_bf16(v); }
    __device__ static float to(bf16_t v) { return bf16_to_f32(v); }
};

// Gate non-linearities on the hardware exp2 and reciprocal units (about 1 ulp each; the absolute
// error of the result stays below 3e-7, far inside the parity tolerance).  They saturate correctly:
// exp2 overflows to +inf, whose reciprocal is 0.
__device__ inline float exp_fast_(float a) { return __builtin_amdgcn_exp2f(a * 1.4426950408889634f); }
__device__ inline float sigmoidf_(float a) { return __builtin_amdgcn_rcpf(1.0f + exp_fast_(-a)); }
__device__ inline float tanhf_(float a) { return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + exp_fast_(2.0f * a)); }

inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }

}  // namespace adpsgd
