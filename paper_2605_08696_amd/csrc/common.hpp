// Shared device helpers for the SRM kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

typedef _Float16 f16;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4_t;

constexpr int kWave = 64;

// ---- activation-type load / store of 4 consecutive channels -----------------
__device__ __forceinline__ float4 load4(const float *p) { return *reinterpret_cast<const float4 *>(p); }
__device__ __forceinline__ float4 load4(const bf16 *p)
{
    bf16x4_t v = *reinterpret_cast<const bf16x4_t *>(p);
    return make_float4((float)v[0], (float)v[1], (float)v[2], (float)v[3]);
}
__device__ __forceinline__ void store4(float *p, float4 v) { *reinterpret_cast<float4 *>(p) = v; }
__device__ __forceinline__ void store4(bf16 *p, float4 v)
{
    // round to nearest even; converted in pairs so that each pair is one packed conversion
    const bf16x2_t lo = __builtin_convertvector(f32x2_t{v.x, v.y}, bf16x2_t);
    const bf16x2_t hi = __builtin_convertvector(f32x2_t{v.z, v.w}, bf16x2_t);
    *reinterpret_cast<bf16x4_t *>(p) = __builtin_shufflevector(lo, hi, 0, 1, 2, 3);
}
__device__ __forceinline__ void store1(float *p, float v) { *p = v; }
__device__ __forceinline__ void store1(bf16 *p, float v) { *p = (bf16)v; }

// ---- recurrent state: fp32, or binary16 when the model keeps a half-precision cache --------
// Vector j = channels 4j .. 4j+3 of the slab.  The state is touched once per step:
// streaming (nontemporal) accesses (with ordinary ones the C4 step measured 1.9 % slower).  to_state() is
// the value as the cache keeps it.
__device__ __forceinline__ float4 load_state4(const float *S, int64_t j)
{
    const f32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t *>(S) + j);
    return make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ float4 load_state4(const f16 *S, int64_t j)
{
    const f16x4_t v = __builtin_nontemporal_load(reinterpret_cast<const f16x4_t *>(S) + j);
    return make_float4((float)v[0], (float)v[1], (float)v[2], (float)v[3]);
}
__device__ __forceinline__ void store_state4(float *S, int64_t j, float4 v)
{
    f32x4_t o;
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
    __builtin_nontemporal_store(o, reinterpret_cast<f32x4_t *>(S) + j);
}
__device__ __forceinline__ void store_state4(f16 *S, int64_t j, float4 v)
{
    f16x4_t o;
    o[0] = (f16)v.x; o[1] = (f16)v.y; o[2] = (f16)v.z; o[3] = (f16)v.w;   // already binary16 values
    __builtin_nontemporal_store(o, reinterpret_cast<f16x4_t *>(S) + j);
}
__device__ __forceinline__ float to_state(float v, const float *) { return v; }
__device__ __forceinline__ float to_state(float v, const f16 *)
{
    // The update is formed in fp32 first and then rounded to binary16 (nearest, ties to even).  The empty
    // statement pins that: left alone, the compiler folds the conversion into a mixed-precision FMA with a
    // binary16 result for some elements of a kernel and not for others (one rounding against two), so the
    // same update could differ in the last bit from kernel to kernel.
    asm volatile("" : "+v"(v));
    return (float)(f16)v;
}

// ---- wavefront reductions ------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// Sum over each group of 16 consecutive lanes (a DPP row), result in every lane of the group.
__device__ __forceinline__ float row16_sum(float v)
{
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));  // row_half_mirror
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));  // row_mirror
    return v;
}

// (value, index) pair ordered by larger value, then smaller index.
__device__ __forceinline__ bool arg_better(float v, int i, float bv, int bi)
{
    return v > bv || (v == bv && i < bi);
}

// exact GELU: x * Phi(x)
__device__ __forceinline__ float gelu_erf(float x)
{
    return 0.5f * x * (1.0f + erff(x * 0.70710678118654752440f));
}

// ---- counter-based random numbers for sampling ------------------------------------
// Gumbel noise for (seed, position, sample b, vocabulary index v), a pure function
// of its arguments (specified in include/srm.h):
//   hash(x): x ^= x>>16; x *= 0x7feb352d; x ^= x>>15; x *= 0x846ca68b; x ^= x>>16
//   rowkey  = hash(b ^ hash(pos + 0x9E3779B9 * (seed + 1)))          (mod 2^32)
//   h       = hash(rowkey + v * 0x9E3779B9)
//   w       = ((h >> 9) + 0.5) * 2^-23            uniform in (0, 1), exact in fp32
//   E       = -log(1 - w)                          exponential variate
//   g       = -log(E)                              standard Gumbel variate
__device__ __forceinline__ uint32_t srm_hash32(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}
__device__ __forceinline__ uint32_t srm_rowkey(uint32_t seed, uint32_t pos, uint32_t b)
{
    return srm_hash32(b ^ srm_hash32(pos + 0x9E3779B9u * (seed + 1u)));
}
__device__ __forceinline__ float srm_gumbel(uint32_t rowkey, uint32_t v)
{
    const uint32_t h = srm_hash32(rowkey + v * 0x9E3779B9u);
    const float w = ((float)(h >> 9) + 0.5f) * (1.0f / 8388608.0f);
    // -log(1 - w): series where 1 - w is too close to 1 for a fast logarithm
    const float e_small = w * (1.0f + w * (0.5f + w * (1.0f / 3.0f)));
    const float e_big = -0.69314718055994530942f * __builtin_amdgcn_logf(1.0f - w);
    const float e = w < (1.0f / 64.0f) ? e_small : e_big;
    return -0.69314718055994530942f * __builtin_amdgcn_logf(e);
}
