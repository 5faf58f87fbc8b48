// Device-side helpers shared by the exat kernels: vector types, the counter-based noise
// function of the synthetic input, bf16 conversion.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

namespace exat {

// ---- synthetic noise g(seed; i,j,k) (definition in include/exat.h, exat_gen_t) ----
// mix_a / mix_b: two published public-domain 32-bit multiply-xorshift hash finalisers ("lowbias32" and a second
// constant set from the same hash-prospector search); only the constants are taken, the keying is this library's.
__host__ __device__ __forceinline__ uint32_t mix_a(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}
__host__ __device__ __forceinline__ uint32_t mix_b(uint32_t x)
{
    x ^= x >> 16; x *= 0x21f0aaadu; x ^= x >> 15; x *= 0x735a2d97u; x ^= x >> 15;
    return x;
}
// host: 64-bit seed -> 32-bit stream key
__host__ __device__ __forceinline__ uint32_t seed_key(uint64_t seed)
{
    return mix_a(mix_a((uint32_t)seed ^ 0x243f6a88u) ^ (uint32_t)(seed >> 32));
}
// key of the fibre (:, j, k)
__device__ __forceinline__ uint32_t fibre_key(uint32_t skey, uint32_t j, uint32_t k)
{
    return mix_a(mix_a(skey ^ k) ^ j);
}
// Box-Muller on the two 16-bit halves of w: returns amp*sqrt(-2 ln u1)*(cos, sin)(2 pi u2).
// v_log_f32 is log2, v_sin/v_cos take their argument in revolutions.
__device__ __forceinline__ void box_muller(uint32_t w, float amp2_ln2, float &zc, float &zs)
{
    const float u1 = __builtin_fmaf((float)(w >> 16), 0x1p-16f, 0x1p-17f);
    const float u2 = __builtin_fmaf((float)(w & 0xffffu), 0x1p-16f, 0x1p-17f);
    // amp2_ln2 = -2 * ln(2) * amp^2  (>= 0 times a non-positive log2)
    const float rad = __builtin_amdgcn_sqrtf(amp2_ln2 * __builtin_amdgcn_logf(u1));
    zc = rad * __builtin_amdgcn_cosf(u2);
    zs = rad * __builtin_amdgcn_sinf(u2);
}
// the four noise values of the aligned quad iq = i>>2 of fibre key ck, scaled by amp
__device__ __forceinline__ void noise_quad(uint32_t ck, uint32_t iq, float amp2_ln2, float z[4])
{
    const uint32_t x = ck ^ iq;
    box_muller(mix_a(x), amp2_ln2, z[0], z[1]);
    box_muller(mix_b(x), amp2_ln2, z[2], z[3]);
}

// ---- element conversion ----
template <typename T> struct elem;
template <> struct elem<float> {
    static constexpr int per16 = 4;  // elements per 16-byte fragment
    __device__ static __forceinline__ float from_f32(float v) { return v; }
};
template <> struct elem<__bf16> {
    static constexpr int per16 = 8;
    __device__ static __forceinline__ __bf16 from_f32(float v) { return (__bf16)v; }  // RNE
};

}  // namespace exat
