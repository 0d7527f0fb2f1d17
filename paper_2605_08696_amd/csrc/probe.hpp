// Two measuring kernels that give the chip's achievable rates beside its published peaks: a plain
// streaming copy (HBM read + write) and a register-resident chain of bf16 matrix-core instructions.
// Neither is part of the model's path; the benchmark reports the hot kernels against both.
#pragma once
#include "common.hpp"

// dst[i] = src[i] over n16 16-byte words; every lane moves `UNROLL` words per trip, all loads issued
// before the first store, and the grid covers the array once.  NT selects streaming (non-temporal)
// loads and stores.
template <int UNROLL, bool NT>
__global__ __launch_bounds__(256) void probe_copy_kernel(const u32x4_t *__restrict__ src, u32x4_t *__restrict__ dst,
                                                         int64_t n16)
{
    const int64_t base = ((int64_t)blockIdx.x * UNROLL) * 256 + threadIdx.x;
    u32x4_t v[UNROLL];
#pragma unroll
    for (int i = 0; i < UNROLL; ++i) {
        const int64_t j = base + (int64_t)i * 256;
        if (j < n16) v[i] = NT ? __builtin_nontemporal_load(src + j) : src[j];
    }
#pragma unroll
    for (int i = 0; i < UNROLL; ++i) {
        const int64_t j = base + (int64_t)i * 256;
        if (j < n16) {
            if (NT) __builtin_nontemporal_store(v[i], dst + j);
            else dst[j] = v[i];
        }
    }
}

// Every wavefront issues `iters` rounds of four independent 32x32x16 bf16 products into four fp32
// accumulator tiles held in registers (no memory traffic inside the loop), then writes one sum per
// lane.  With A = 1 and B = 1 every accumulator element ends at 16 * iters, so the written value is
// 4 * 16 * 16 * iters per lane (16 accumulator registers per tile): checkable on the host.  With
// random_operands the operand elements are pseudo-random values in (-1, 1), different per lane and
// element: the matrix cores draw more power on such data than on constants, and the clock the chip
// holds (hence the rate) is lower; the sums are then only finite, not predictable.
__global__ __launch_bounds__(256) void probe_mfma_kernel(float *__restrict__ out, int iters, float a_val,
                                                         int random_operands)
{
    bf16x8_t a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (bf16)a_val;
        b[i] = (bf16)1.0f;
        if (random_operands) {
            uint32_t h = (threadIdx.x * 2654435761u) ^ (uint32_t)(i * 40503 + 12345);
            h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
            a[i] = (bf16)((float)(int32_t)h * (1.0f / 2147483648.0f));
            h *= 3266489917u; h ^= h >> 16;
            b[i] = (bf16)((float)(int32_t)h * (1.0f / 2147483648.0f));
        }
    }
    f32x16_t c0 = {}, c1 = {}, c2 = {}, c3 = {};
    for (int it = 0; it < iters; ++it) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
    out[(int64_t)blockIdx.x * 256 + threadIdx.x] = s;
}
