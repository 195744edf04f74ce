// Shared device/host helpers of libqgalore (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qgalore.h"

namespace qg {

constexpr int kGroup = 256;  // quantization block size (Sec. 3.1)
constexpr int kWave = 64;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// ---- host-side error plumbing (defined in qg_api.hip) ----
void set_hip_error(hipError_t e);
int check_launch();

// ---- stochastic-rounding generator (Sec. 3.4 leaves the random source open) ----
// mix32: xorshift 16, * 0x7FEB352D, xorshift 15, * 0x846CA68B, xorshift 16.
__host__ __device__ inline uint32_t mix32(uint32_t x) {
    x ^= x >> 16;
    x *= 0x7FEB352Du;
    x ^= x >> 15;
    x *= 0x846CA68Bu;
    x ^= x >> 16;
    return x;
}

// Fold (seed_lo, seed_hi, step_lo, step_hi, idx_hi) into a 32-bit key.
__host__ __device__ inline uint32_t sr_key(uint64_t seed, uint64_t step, uint32_t idx_hi) {
    uint32_t key = 0x9E3779B9u;
    const uint32_t w[5] = {(uint32_t)seed, (uint32_t)(seed >> 32), (uint32_t)step, (uint32_t)(step >> 32), idx_hi};
    for (int i = 0; i < 5; ++i) key = mix32((key ^ w[i]) + 0x9E3779B9u);
    return key;
}

// u in [0,1): top 24 bits of the hash of (key, low word of the element index).
__device__ inline float sr_uniform(uint32_t key, uint32_t idx_lo) {
    return (float)(mix32(key ^ idx_lo) >> 8) * 0x1p-24f;
}

// ---- bf16 packing (round to nearest even, hardware v_cvt_pk_bf16_f32) ----
__device__ inline uint32_t pack_bf16x2(float a, float b) {
    f32x2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ inline uint16_t to_bf16(float a) { return (uint16_t)(pack_bf16x2(a, 0.0f) & 0xFFFFu); }

// Dequantize the 8 INT4 codes of one 32-bit word (flat elements 8w..8w+7, low
// nibble first, stored nibble = code + 8) with one block scale to 8 bf16:
// fl32((nib - 8) * s) through one fma, then one rounding to bf16.
__device__ inline u32x4 dequant8_bf16(uint32_t w, float s) {
    const float ms = -8.0f * s;
    // even and odd nibbles spread to one byte each, so that each conversion is a single byte-to-float instruction
    uint32_t lo = w & 0x0F0F0F0Fu, hi = (w >> 4) & 0x0F0F0F0Fu;
    // (opaque to the optimizer, which would otherwise fold the masks back into eight 4-bit field extracts)
    asm("" : "+v"(lo));
    asm("" : "+v"(hi));
    float e[8];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        e[2 * j] = __builtin_fmaf((float)((lo >> (8 * j)) & 0xFFu), s, ms);
        e[2 * j + 1] = __builtin_fmaf((float)((hi >> (8 * j)) & 0xFFu), s, ms);
    }
    const u32x4 o = {pack_bf16x2(e[0], e[1]), pack_bf16x2(e[2], e[3]), pack_bf16x2(e[4], e[5]),
                     pack_bf16x2(e[6], e[7])};
    return o;
}

__device__ inline float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// ---- Adam on one element (Sec. 3.5; Adam as cited in Sec. 4.1) ----
struct AdamCoef {
    float b1, b2, omb1, omb2, rc1, rc2, eps;  // rc = 1/(1 - beta^t)
    float sqrt_rc2;                           // sqrt(rc2): sqrt(V rc2) = sqrt(V) sqrt(rc2)
};

__device__ inline float adam_one(float r, float& m, float& v, const AdamCoef& c) {
    m = __builtin_fmaf(c.b1, m, c.omb1 * r);
    v = __builtin_fmaf(c.b2, v, c.omb2 * (r * r));
    const float mhat = m * c.rc1;
    // N is stored as bf16 (8 significant bits): the hardware square root and reciprocal (1 ulp of fp32 each) are
    // exact enough, and a correctly rounded sqrt and divide would cost about 15 more instructions per element in
    // the projection's epilogue.  M and V above are exact fp32 recurrences.
    return mhat * __builtin_amdgcn_rcpf(__builtin_fmaf(__builtin_amdgcn_sqrtf(v), c.sqrt_rc2, c.eps));
}

AdamCoef make_adam_coef(const qg_hparams* hp, int64_t step);   // host, qg_adam.hip

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace qg
