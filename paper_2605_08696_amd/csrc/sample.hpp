// Nucleus (top-p) sampling on materialised logits ("Reasoning Experiments
// details": rollouts are drawn with top-p 0.9 at temperature 0.7).
//
// With p_v = softmax(logits / T), the nucleus is the smallest set of most
// probable tokens whose probability reaches top_p (equal logits kept or dropped
// together); the token is drawn from the renormalised nucleus with the
// Gumbel-max rule and the same counter-based noise as plain sampling,
// argmax_{v in nucleus} (logit_v + T * g_v).
//
// One block per row.  The unrestricted Gumbel-max winner w0 (from the LM-head
// epilogue, or found here) is the answer whenever it lies inside the nucleus,
// which one streaming pass decides: w0 is inside iff the probability mass of
// the strictly larger logits is below top_p.  That holds for about top_p of the
// rows.  Otherwise the cut is located by bisection over the order-preserving
// integer image of the logits (at most 32 passes over the row, which stays in
// cache), each pass a deterministic block reduction, then the Gumbel-max is
// repeated over the kept tokens only.
//
// Re-reading rows from memory is what those passes cost, so the decode step
// splits the work: nucleus_kernel<.., DEFER> makes the streaming pass for every
// row and appends the rows that need the search to a list, and
// nucleus_slow_kernel takes the listed rows one at a time with the row held in
// registers (persistent blocks of 512 threads, 64 elements per thread), so each
// row is read from memory twice in total.  Larger vocabularies use the
// one-kernel form.
#pragma once
#include "common.hpp"

// Unsigned integers ordered as the floats are; -0 and +0 share a key.
__device__ __forceinline__ uint32_t order_key(float f)
{
    const uint32_t u = __float_as_uint(f + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

template <int NW>
__device__ __forceinline__ float block_sum(float v, float *red)
{
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = 0.0f;
#pragma unroll
    for (int i = 0; i < NW; ++i) t += red[i];
    __syncthreads();
    return t;
}

template <int NW>
__device__ __forceinline__ float block_max(float v, float *red)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = -INFINITY;
#pragma unroll
    for (int i = 0; i < NW; ++i) t = fmaxf(t, red[i]);
    __syncthreads();
    return t;
}

// (value, index) maximum, lowest index on equal values; every thread gets the result.
template <int NW>
__device__ __forceinline__ int block_argmax(float bv, int bi, float *red, int *redi)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float ov = __shfl_xor(bv, off, kWave);
        const int oi = __shfl_xor(bi, off, kWave);
        if (arg_better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
    if ((threadIdx.x & 63) == 0) { red[threadIdx.x >> 6] = bv; redi[threadIdx.x >> 6] = bi; }
    __syncthreads();
    float tv = -INFINITY;
    int ti = 0x7fffffff;
#pragma unroll
    for (int i = 0; i < NW; ++i)
        if (arg_better(red[i], redi[i], tv, ti)) { tv = red[i]; ti = redi[i]; }
    __syncthreads();
    return ti;
}

// Calls fn(value, index) for this thread's share of one row.  Rows that allow it
// are read as 16-byte vectors, four independent loads in flight per thread, so a
// pass over a cache-resident row costs a few memory latencies, not one per element.
template <int NT, typename F>
__device__ __forceinline__ void row_foreach(const float *__restrict__ L, int V, F &&fn)
{
    const int tid = threadIdx.x;
    if ((V & 3) == 0 && (reinterpret_cast<uintptr_t>(L) & 15) == 0) {
        const f32x4_t *L4 = reinterpret_cast<const f32x4_t *>(L);
        const int n4 = V >> 2;
        int i = tid;
        for (; i + 3 * NT < n4; i += 4 * NT) {
            const f32x4_t a = L4[i], b = L4[i + NT], c = L4[i + 2 * NT], d = L4[i + 3 * NT];
#pragma unroll
            for (int k = 0; k < 4; ++k) fn(a[k], 4 * i + k);
#pragma unroll
            for (int k = 0; k < 4; ++k) fn(b[k], 4 * (i + NT) + k);
#pragma unroll
            for (int k = 0; k < 4; ++k) fn(c[k], 4 * (i + 2 * NT) + k);
#pragma unroll
            for (int k = 0; k < 4; ++k) fn(d[k], 4 * (i + 3 * NT) + k);
        }
        for (; i < n4; i += NT) {
            const f32x4_t a = L4[i];
#pragma unroll
            for (int k = 0; k < 4; ++k) fn(a[k], 4 * i + k);
        }
    } else {
        int v = tid;
        for (; v + 3 * NT < V; v += 4 * NT) {
            const float a = L[v], b = L[v + NT], c = L[v + 2 * NT], d = L[v + 3 * NT];
            fn(a, v); fn(b, v + NT); fn(c, v + 2 * NT); fn(d, v + 3 * NT);
        }
        for (; v < V; v += NT) fn(L[v], v);
    }
}

// logits: [rows][ld] fp32, V <= ld.  tok[rows]: with FIND_W0 = false it holds the
// unrestricted Gumbel-max winner on entry (a negative value marks an idle row,
// which is skipped) and the nucleus sample on exit; with FIND_W0 = true it is
// output only.  Position of the random counter: pos_rows[row], else *pos_dev,
// else pos.  If store is not null the token also goes to
// store[*step_dev * store_stride + row].  If pos_advance is not null the
// position of every non-idle row is incremented at the end (pos_advance may be
// the same array as pos_rows), or set to -1 (idle) if the row's token is
// eos_plus1 - 1 (eos_plus1 = 0: no such token).
// With DEFER, a row that needs the search is appended to slow_list (its count in
// *slow_count, which must be zero at launch) and left to nucleus_slow_kernel,
// which also does that row's store / pos_advance.
template <int NT, bool FIND_W0, bool DEFER = false>
__global__ void __launch_bounds__(NT)
nucleus_kernel(const float *__restrict__ logits, int64_t ld, int V, float temp, float top_p, uint32_t seed, int pos,
               const int *__restrict__ pos_dev, const int *pos_rows, int32_t *__restrict__ tok,
               int32_t *__restrict__ store, const int *__restrict__ step_dev, int64_t store_stride,
               int32_t *pos_advance, int *__restrict__ slow_count = nullptr, int *__restrict__ slow_list = nullptr,
               uint32_t row_base = 0, int eos_plus1 = 0)
{
    constexpr int NW = NT / 64;
    __shared__ float red[NW];
    __shared__ int redi[NW];
    const int64_t row = blockIdx.x;
    const int tid = threadIdx.x;
    const float *__restrict__ L = logits + row * ld;
    int w0 = FIND_W0 ? 0 : tok[row];
    if (!FIND_W0 && w0 < 0) return;                       // idle row (the whole block leaves)
    const uint32_t p = (uint32_t)(pos_rows ? pos_rows[row] : (pos_dev ? *pos_dev : pos));
    const uint32_t rk = srm_rowkey(seed, p, (uint32_t)row + row_base);     // the counter is keyed on the sample index
    const float inv = 1.4426950408889634f / temp;

    if constexpr (FIND_W0) {
        float bv = -INFINITY;
        int bi = 0x7fffffff;
        row_foreach<NT>(L, V, [&](float x, int v) {
            const float s = x + temp * srm_gumbel(rk, (uint32_t)v);
            if (arg_better(s, v, bv, bi)) { bv = s; bi = v; }
        });
        w0 = block_argmax<NW>(bv, bi, red, redi);
    }
    w0 = min(max(w0, 0), V - 1);
    const uint32_t kw = order_key(L[w0]);

    // one pass: row maximum, normaliser Z and the mass above w0, rescaled on the fly
    float mt = -INFINITY, z = 0.0f, fa = 0.0f;
    row_foreach<NT>(L, V, [&](float x, int) {
        const float above = order_key(x) > kw ? 1.0f : 0.0f;
        if (x > mt) {
            const float sc = __builtin_amdgcn_exp2f((mt - x) * inv);
            z = fmaf(z, sc, 1.0f);
            fa = fmaf(fa, sc, above);
            mt = x;
        } else {
            const float e = __builtin_amdgcn_exp2f((x - mt) * inv);
            z += e;
            fa = fmaf(above, e, fa);
        }
    });
    const float M = block_max<NW>(mt, red);
    const float sc = mt == -INFINITY ? 0.0f : __builtin_amdgcn_exp2f((mt - M) * inv);
    const float Z = block_sum<NW>(z * sc, red);
    const float FA = block_sum<NW>(fa * sc, red);
    const float target = top_p * Z;

    int result = w0;
    uint32_t lo = kw, hi = order_key(M);
    if (DEFER && !(FA < target) && hi > lo) {
        if (tid == 0) slow_list[atomicAdd(slow_count, 1)] = (int)row;
        return;
    }
    if (!(FA < target) && hi > lo) {
        // invariant: mass{key > lo} >= target, mass{key > hi} < target; kept = {key >= hi} at the end
        while (hi - lo > 1u) {
            const uint32_t mid = lo + ((hi - lo) >> 1);
            float f = 0.0f;
            row_foreach<NT>(L, V, [&](float x, int) {
                if (order_key(x) > mid) f += __builtin_amdgcn_exp2f((x - M) * inv);
            });
            f = block_sum<NW>(f, red);
            if (f < target) hi = mid; else lo = mid;
        }
        float bv = -INFINITY;
        int bi = 0x7fffffff;
        row_foreach<NT>(L, V, [&](float x, int v) {
            if (order_key(x) >= hi) {
                const float s = x + temp * srm_gumbel(rk, (uint32_t)v);
                if (arg_better(s, v, bv, bi)) { bv = s; bi = v; }
            }
        });
        result = block_argmax<NW>(bv, bi, red, redi);
        if (result < 0 || result >= V) result = w0;
    }
    if (tid == 0) {
        tok[row] = result;
        if (store) store[(int64_t)(*step_dev) * store_stride + row] = result;
        if (pos_advance) pos_advance[row] = (eos_plus1 && result == eos_plus1 - 1) ? -1 : (int32_t)p + 1;
    }
}

// The rows nucleus_kernel<.., DEFER> listed, each held in registers for the whole
// search: a thread keeps the keys and the exp() values of its EPT elements
// (V <= NT * EPT), so a bisection pass is a compare and an add per element.
// Persistent: block i takes list entries i, i + gridDim, ...  Arguments as
// nucleus_kernel; tok[row] holds the unrestricted winner on entry.
template <int NT, int EPT>
__global__ void __launch_bounds__(NT)
nucleus_slow_kernel(const float *__restrict__ logits, int64_t ld, int V, float temp, float top_p, uint32_t seed, int pos,
                    const int *__restrict__ pos_dev, const int *pos_rows, int32_t *__restrict__ tok,
                    int32_t *__restrict__ store, const int *__restrict__ step_dev, int64_t store_stride,
                    int32_t *pos_advance, const int *__restrict__ slow_count, const int *__restrict__ slow_list,
                    uint32_t row_base, int eos_plus1)
{
    static_assert(EPT % 4 == 0, "EPT must be a multiple of 4");
    constexpr int NW = NT / 64;
    __shared__ float red[NW];
    __shared__ int redi[NW];
    const int tid = threadIdx.x;
    const int n = *slow_count;
    const float inv = 1.4426950408889634f / temp;
    for (int i = blockIdx.x; i < n; i += gridDim.x) {
        const int64_t row = slow_list[i];
        const float *__restrict__ L = logits + row * ld;
        const bool vec = (V & 3) == 0 && (reinterpret_cast<uintptr_t>(L) & 15) == 0;
        // absent elements are -inf: key below every logit's, exp() = 0
        uint32_t key[EPT];
        float e[EPT];
        float mt = -INFINITY;
        if (vec) {
            const f32x4_t *L4 = reinterpret_cast<const f32x4_t *>(L);
            const int n4 = V >> 2;
#pragma unroll
            for (int k = 0; k < EPT / 4; ++k) {
                const int j = tid + k * NT;
                f32x4_t a;
                if (j < n4) a = L4[j];
                else a[0] = a[1] = a[2] = a[3] = -INFINITY;
#pragma unroll
                for (int c = 0; c < 4; ++c) { e[4 * k + c] = a[c]; mt = fmaxf(mt, a[c]); }
            }
        } else {
#pragma unroll
            for (int k = 0; k < EPT; ++k) {
                const int v = tid + k * NT;
                e[k] = v < V ? L[v] : -INFINITY;
                mt = fmaxf(mt, e[k]);
            }
        }
        const int w0 = min(max(tok[row], 0), V - 1);
        const uint32_t kw = order_key(L[w0]);
        const uint32_t p = (uint32_t)(pos_rows ? pos_rows[row] : (pos_dev ? *pos_dev : pos));
        const uint32_t rk = srm_rowkey(seed, p, (uint32_t)row + row_base);
        const float M = block_max<NW>(mt, red);
        float z = 0.0f, fa = 0.0f;
#pragma unroll
        for (int k = 0; k < EPT; ++k) {
            key[k] = order_key(e[k]);
            e[k] = __builtin_amdgcn_exp2f((e[k] - M) * inv);          // exp2(-inf) = 0 for absent elements
            z += e[k];
            if (key[k] > kw) fa += e[k];
        }
        const float Z = block_sum<NW>(z, red);
        const float FA = block_sum<NW>(fa, red);
        const float target = top_p * Z;
        int result = w0;
        uint32_t lo = kw, hi = order_key(M);
        if (!(FA < target) && hi > lo) {
            while (hi - lo > 1u) {
                const uint32_t mid = lo + ((hi - lo) >> 1);
                float f = 0.0f;
#pragma unroll
                for (int k = 0; k < EPT; ++k) f += key[k] > mid ? e[k] : 0.0f;
                f = block_sum<NW>(f, red);
                if (f < target) hi = mid; else lo = mid;
            }
            float bv = -INFINITY;
            int bi = 0x7fffffff;
            // the kept tokens' scores, from the row as it lies in memory (one more cached read)
            row_foreach<NT>(L, V, [&](float x, int v) {
                if (order_key(x) >= hi) {
                    const float s = x + temp * srm_gumbel(rk, (uint32_t)v);
                    if (arg_better(s, v, bv, bi)) { bv = s; bi = v; }
                }
            });
            result = block_argmax<NW>(bv, bi, red, redi);
            if (result < 0 || result >= V) result = w0;
        }
        if (tid == 0) {
            tok[row] = result;
            if (store) store[(int64_t)(*step_dev) * store_stride + row] = result;
            if (pos_advance) pos_advance[row] = (eos_plus1 && result == eos_plus1 - 1) ? -1 : (int32_t)p + 1;
        }
    }
}
