// The structured token mixer in its three evaluation orders.
//
//   state_update_kernel   one position for every sample (decode): Eq. 2 / Eq. 3
//   mixer_scan_kernel     all prompt positions in sequence (prefill), state kept
//                         in registers, same arithmetic as state_update_kernel
//   scan_chunk_*_kernel   the same scan cut into chunks that run side by side
//                         (prefill of few sequences)
//   np_token_mix_kernel   decode of a non-projected layer: both LayerNorms, the
//                         update and the residual add in one pass
//   mixer_parallel_kernel the explicit triangular product Y = U M + beta with M
//                         built on the fly from alpha and lambda (Eq. 1, Eq. 3)
//
// Both head types share one update, S' = lam*S + p*u ; m = q*S' + beta, with
// (p, q) = (alpha, 1) for row-repeat heads and (1, alpha) for column-repeat
// heads; multiplying by the constant 1 is exact, so this is Eq. 2 / Eq. 3 as
// written.  alpha, beta: [H][n_ctx] of this layer; lam: [H].  Heads 0..hrow-1
// are row-repeat, heads hrow..H-1 column-repeat (hrow = H/2: the mixed layout;
// H or 0: one kind only).  H and d are the mixer's: a model with combined heads
// runs as 2H heads over a row of width 2d (see srm_init_weights).
#pragma once
#include "common.hpp"

constexpr int kMaxHeads = 64;

// Streams u [B][d] (TAct), S [B][d] (fp32, in place) and m [B][d] (TAct), four
// channels per thread.  The launch makes gridDim.x * 256 a multiple of d/4, so a
// thread keeps one channel group, hence one head, for its whole loop; the per
// head coefficients of this position are staged in LDS once per block.  If
// pos_dev is not null the position is read from device memory, so that a captured
// graph of the step can be replayed as is; a position outside [0, n_ctx) there
// makes the whole batch inactive, as in the fused in-projection epilogue: the
// state is left alone and m is written as zeros.
template <typename TAct, int UNROLL, typename TState = float>
__global__ void __launch_bounds__(256)
state_update_kernel(const TAct *__restrict__ u, TState *__restrict__ S, TAct *__restrict__ m,
                    const float *__restrict__ alpha, const float *__restrict__ beta,
                    const float *__restrict__ lam, int pos, const int *__restrict__ pos_dev, int n_ctx, int H, int hrow,
                    int d, int64_t nvec)
{
    __shared__ float4 coef[kMaxHeads];      // (lam, p, q, beta) per head
    bool active = true;
    if (pos_dev) {
        const int pd = *pos_dev;
        active = pd >= 0 && pd < n_ctx;
        pos = active ? pd : 0;
    }
    if (threadIdx.x < H) {
        const int h = threadIdx.x;
        const float a = alpha[(size_t)h * n_ctx + pos];
        const bool row_repeat = h < hrow;
        coef[h] = make_float4(lam[h], row_repeat ? a : 1.0f, row_repeat ? 1.0f : a,
                              beta[(size_t)h * n_ctx + pos]);
    }
    __syncthreads();
    const int dv = d >> 2, dhv = (d / H) >> 2;
    const int64_t nthreads = (int64_t)gridDim.x * 256;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const float4 cf = coef[(int)(gid % dv) / dhv];
    const float l = cf.x, p = cf.y, q = cf.z, be = cf.w;

    if (!active) {
        for (int64_t i = gid; i < nvec; i += nthreads) store4(m + i * 4, make_float4(0.f, 0.f, 0.f, 0.f));
        return;
    }
    for (int64_t i = gid; i < nvec; i += nthreads * UNROLL) {
        float4 s[UNROLL], x[UNROLL];
#pragma unroll
        for (int k = 0; k < UNROLL; ++k) {
            const int64_t j = i + k * nthreads;
            if (j < nvec) {
                s[k] = load_state4(S, j);
                x[k] = load4(u + j * 4);
            }
        }
#pragma unroll
        for (int k = 0; k < UNROLL; ++k) {
            const int64_t j = i + k * nthreads;
            if (j < nvec) {
                float4 n, o;
                n.x = to_state(fmaf(l, s[k].x, p * x[k].x), S); o.x = fmaf(q, n.x, be);
                n.y = to_state(fmaf(l, s[k].y, p * x[k].y), S); o.y = fmaf(q, n.y, be);
                n.z = to_state(fmaf(l, s[k].z, p * x[k].z), S); o.z = fmaf(q, n.z, be);
                n.w = to_state(fmaf(l, s[k].w, p * x[k].w), S); o.w = fmaf(q, n.w, be);
                store_state4(S, j, n);
                store4(m + j * 4, o);
            }
        }
    }
}

// Prefill: u, m are [nseq][P][d]; thread = (sequence, 4 channels), sequential in
// t from a zero state (positions 0..P-1).  The final state is written to `rep`
// consecutive samples: S[((seq0 + seq) * rep + r)][d] of this layer's slab.
// Dynamic LDS: 2 * H * P floats (alpha then beta of the P positions).
template <typename TAct, typename TState = float>
__global__ void __launch_bounds__(256)
mixer_scan_kernel(const TAct *__restrict__ u, TAct *__restrict__ m, TState *__restrict__ S,
                  const float *__restrict__ alpha, const float *__restrict__ beta,
                  const float *__restrict__ lam, int n_ctx, int H, int hrow, int d, int nseq, int P,
                  int64_t seq0, int rep)
{
    extern __shared__ float sc[];
    float *sa = sc, *sb = sc + H * P;
    for (int i = threadIdx.x; i < H * P; i += 256) {
        const int h = i / P, t = i - h * P;
        sa[i] = alpha[(size_t)h * n_ctx + t];
        sb[i] = beta[(size_t)h * n_ctx + t];
    }
    __syncthreads();
    const int dv = d >> 2, dhv = (d / H) >> 2;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t seq = gid / dv;
    if (seq >= nseq) return;
    const int cv = (int)(gid - seq * dv);
    const int h = cv / dhv;
    const bool row_repeat = h < hrow;
    const float l = lam[h];
    const TAct *up = u + (seq * P) * (int64_t)d + cv * 4;
    TAct *mp = m + (seq * P) * (int64_t)d + cv * 4;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int t = 0; t < P; ++t) {
        const float4 x = load4(up + (int64_t)t * d);
        const float a = sa[h * P + t], be = sb[h * P + t];
        const float p = row_repeat ? a : 1.0f, q = row_repeat ? 1.0f : a;
        float4 o;
        s.x = to_state(fmaf(l, s.x, p * x.x), S); o.x = fmaf(q, s.x, be);
        s.y = to_state(fmaf(l, s.y, p * x.y), S); o.y = fmaf(q, s.y, be);
        s.z = to_state(fmaf(l, s.z, p * x.z), S); o.z = fmaf(q, s.z, be);
        s.w = to_state(fmaf(l, s.w, p * x.w), S); o.w = fmaf(q, s.w, be);
        store4(mp + (int64_t)t * d, o);
    }
    const int64_t dst = (((seq0 + seq) * rep) * (int64_t)d + cv * 4) >> 2;       // vector index
    for (int r = 0; r < rep; ++r) store_state4(S, dst + (int64_t)r * (d >> 2), s);
}

// Token mixing of a non-projected layer in one pass over the row (decode): LayerNorm1,
// the state update on its output (head h = channels h*d_h ..), the residual add
// and LayerNorm2, one wavefront per sample, the row held in registers:
//   u = LN1(x) ; S <- lam*S + p*u ; m = q*S + beta ; x <- x + m ; out = LN2(x)
// u and m pass through the activation type TAct exactly where the separate
// kernels (ln_kernel, state_update_kernel, ln_kernel with add_act) store them, so
// the results are bit-identical to that sequence.  Reads x and S, writes S, x and
// out: 16d + 2d bytes per sample for bf16 activations.  VPL = float4 vectors per
// lane (d <= 256 * VPL).  Position: pos_rows[row], else *pos_dev, else pos; a
// position outside [0, n_ctx) leaves S alone and adds nothing.
template <typename TAct, int VPL, typename TState = float>
__global__ void __launch_bounds__(256)
np_token_mix_kernel(float *x, TState *__restrict__ S, TAct *__restrict__ out, const float *__restrict__ g1,
                    const float *__restrict__ b1, const float *__restrict__ g2, const float *__restrict__ b2,
                    const float *__restrict__ alpha, const float *__restrict__ beta,
                    const float *__restrict__ lam, int pos, const int *__restrict__ pos_dev,
                    const int *__restrict__ pos_rows, int n_ctx, int H, int hrow, int d, int64_t rows, float eps)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int p = pos_rows ? pos_rows[row] : (pos_dev ? *pos_dev : pos);
    const bool active = p >= 0 && p < n_ctx;
    const int dh = d / H;

    float4 v[VPL];
    float sum = 0.0f;
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
        const int c = (i * 64 + lane) * 4;
        if (c < d) {
            v[i] = load4(x + row * d + c);
            sum += (v[i].x + v[i].y) + (v[i].z + v[i].w);
        } else {
            v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    float mean = wave_sum(sum) / (float)d;
    float sq = 0.0f;
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
        const int c = (i * 64 + lane) * 4;
        if (c < d) {
            const float a = v[i].x - mean, bb = v[i].y - mean, cc = v[i].z - mean, dd = v[i].w - mean;
            sq += (a * a + bb * bb) + (cc * cc + dd * dd);
        }
    }
    float rstd = 1.0f / sqrtf(wave_sum(sq) / (float)d + eps);
    sum = 0.0f;
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
        const int c = (i * 64 + lane) * 4;
        if (c < d) {
            if (active) {
                const float4 gg = load4(g1 + c), bb = load4(b1 + c);
                // LN1 output as the activation type holds it
                const float u0 = (float)(TAct)((v[i].x - mean) * rstd * gg.x + bb.x);
                const float u1 = (float)(TAct)((v[i].y - mean) * rstd * gg.y + bb.y);
                const float u2 = (float)(TAct)((v[i].z - mean) * rstd * gg.z + bb.z);
                const float u3 = (float)(TAct)((v[i].w - mean) * rstd * gg.w + bb.w);
                const int h = c / dh;
                const float a = alpha[(size_t)h * n_ctx + p], be = beta[(size_t)h * n_ctx + p], l = lam[h];
                const bool row_repeat = h < hrow;
                const float pp = row_repeat ? a : 1.0f, q = row_repeat ? 1.0f : a;
                const int64_t sj = (row * d + c) >> 2;
                const float4 sv = load_state4(S, sj);
                float4 nv;
                nv.x = to_state(fmaf(l, sv.x, pp * u0), S);
                nv.y = to_state(fmaf(l, sv.y, pp * u1), S);
                nv.z = to_state(fmaf(l, sv.z, pp * u2), S);
                nv.w = to_state(fmaf(l, sv.w, pp * u3), S);
                store_state4(S, sj, nv);
                v[i].x += (float)(TAct)fmaf(q, nv.x, be);
                v[i].y += (float)(TAct)fmaf(q, nv.y, be);
                v[i].z += (float)(TAct)fmaf(q, nv.z, be);
                v[i].w += (float)(TAct)fmaf(q, nv.w, be);
                store4(x + row * d + c, v[i]);
            }
            sum += (v[i].x + v[i].y) + (v[i].z + v[i].w);
        }
    }
    mean = wave_sum(sum) / (float)d;
    sq = 0.0f;
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
        const int c = (i * 64 + lane) * 4;
        if (c < d) {
            const float a = v[i].x - mean, bb = v[i].y - mean, cc = v[i].z - mean, dd = v[i].w - mean;
            sq += (a * a + bb * bb) + (cc * cc + dd * dd);
        }
    }
    rstd = 1.0f / sqrtf(wave_sum(sq) / (float)d + eps);
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
        const int c = (i * 64 + lane) * 4;
        if (c < d) {
            const float4 gg = load4(g2 + c), bb = load4(b2 + c);
            float4 o;
            o.x = (v[i].x - mean) * rstd * gg.x + bb.x;
            o.y = (v[i].y - mean) * rstd * gg.y + bb.y;
            o.z = (v[i].z - mean) * rstd * gg.z + bb.z;
            o.w = (v[i].w - mean) * rstd * gg.w + bb.w;
            store4(out + row * d + c, o);
        }
    }
}

// Decode with one position per sample (ragged batches, continuous batching):
// pos_rows[b] is sample b's position; a sample whose position is outside
// [0, n_ctx) is inactive: its state is left as it is and its m row is zero.
// Thread = (sample, 4 channels); alpha and beta come straight from the tables
// (a few KB, cache resident).
template <typename TAct, typename TState = float>
__global__ void __launch_bounds__(256)
state_update_ragged_kernel(const TAct *__restrict__ u, TState *__restrict__ S, TAct *__restrict__ m,
                           const float *__restrict__ alpha, const float *__restrict__ beta,
                           const float *__restrict__ lam, const int *__restrict__ pos_rows, int n_ctx, int H, int hrow,
                           int d, int64_t nvec)
{
    const int dv = d >> 2, dhv = (d / H) >> 2;
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= nvec) return;
    const int64_t b = j / dv;
    const int h = (int)(j - b * dv) / dhv;
    const int pos = pos_rows[b];
    if (pos < 0 || pos >= n_ctx) {
        store4(m + j * 4, make_float4(0.f, 0.f, 0.f, 0.f));
        return;
    }
    const float a = alpha[(size_t)h * n_ctx + pos], be = beta[(size_t)h * n_ctx + pos], l = lam[h];
    const bool row_repeat = h < hrow;
    const float p = row_repeat ? a : 1.0f, q = row_repeat ? 1.0f : a;
    const float4 sv = load_state4(S, j);
    const float4 x = load4(u + j * 4);
    float4 o, nv;
    nv.x = to_state(fmaf(l, sv.x, p * x.x), S); o.x = fmaf(q, nv.x, be);
    nv.y = to_state(fmaf(l, sv.y, p * x.y), S); o.y = fmaf(q, nv.y, be);
    nv.z = to_state(fmaf(l, sv.z, p * x.z), S); o.z = fmaf(q, nv.z, be);
    nv.w = to_state(fmaf(l, sv.w, p * x.w), S); o.w = fmaf(q, nv.w, be);
    store_state4(S, j, nv);
    store4(m + j * 4, o);
}

// Prefill of packed sequences of different lengths: u, m are [rows][d] holding
// the sequences back to back; sequence s (0 <= s < nseq) occupies rows
// offsets[seq0 + s] - base .. offsets[seq0 + s + 1] - base - 1 (clamped to
// [0, rows), so that no access depends on the array being well formed) and is
// scanned from a zero state, positions 0.. (at most Pmax, the longest length of
// the launch).  Its final state goes to sample slot[seq0 + s] if slot is given
// (skipped when outside [0, nslots)), else to the `rep` samples
// (seq0 + s) * rep + r.  Dynamic LDS: 2 * H * Pmax floats.
template <typename TAct, typename TState = float>
__global__ void __launch_bounds__(256)
mixer_scan_ragged_kernel(const TAct *__restrict__ u, TAct *__restrict__ m, TState *__restrict__ S,
                         const float *__restrict__ alpha, const float *__restrict__ beta,
                         const float *__restrict__ lam, int n_ctx, int H, int hrow, int d, int nseq, int Pmax,
                         const int32_t *__restrict__ offsets, int64_t base, int64_t rows, int64_t seq0, int rep,
                         const int32_t *__restrict__ slot, int64_t nslots)
{
    extern __shared__ float sc[];
    float *sa = sc, *sb = sc + H * Pmax;
    for (int i = threadIdx.x; i < H * Pmax; i += 256) {
        const int h = i / Pmax, t = i - h * Pmax;
        sa[i] = alpha[(size_t)h * n_ctx + t];
        sb[i] = beta[(size_t)h * n_ctx + t];
    }
    __syncthreads();
    const int dv = d >> 2, dhv = (d / H) >> 2;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t seq = gid / dv;
    if (seq >= nseq) return;
    const int cv = (int)(gid - seq * dv);
    const int h = cv / dhv;
    const bool row_repeat = h < hrow;
    const float l = lam[h];
    const int64_t r0 = min(max((int64_t)offsets[seq0 + seq] - base, (int64_t)0), rows);
    const int64_t r1 = min(max((int64_t)offsets[seq0 + seq + 1] - base, r0), rows);
    const int len = (int)min(r1 - r0, (int64_t)Pmax);
    const TAct *up = u + r0 * (int64_t)d + cv * 4;
    TAct *mp = m + r0 * (int64_t)d + cv * 4;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int t = 0; t < len; ++t) {
        const float4 x = load4(up + (int64_t)t * d);
        const float a = sa[h * Pmax + t], be = sb[h * Pmax + t];
        const float p = row_repeat ? a : 1.0f, q = row_repeat ? 1.0f : a;
        float4 o;
        s.x = to_state(fmaf(l, s.x, p * x.x), S); o.x = fmaf(q, s.x, be);
        s.y = to_state(fmaf(l, s.y, p * x.y), S); o.y = fmaf(q, s.y, be);
        s.z = to_state(fmaf(l, s.z, p * x.z), S); o.z = fmaf(q, s.z, be);
        s.w = to_state(fmaf(l, s.w, p * x.w), S); o.w = fmaf(q, s.w, be);
        store4(mp + (int64_t)t * d, o);
    }
    const int dq = d >> 2;
    if (slot) {
        const int64_t dst = slot[seq0 + seq];
        if (dst >= 0 && dst < nslots) store_state4(S, dst * dq + cv, s);
    } else {
        const int64_t dst = ((seq0 + seq) * rep) * (int64_t)dq + cv;
        for (int r = 0; r < rep; ++r) store_state4(S, dst + (int64_t)r * dq, s);
    }
}

// Chunked scan for prefill with few sequences, where the sequential kernels leave
// most of the chip idle (the "parallel scan for recurrent prefill" the paper's
// "MAX model details" name as unexplored).  The recurrence S_t = lam S_{t-1} + p_t u_t
// is linear, so the state entering chunk j (positions j*c ..) is
//   C_j = lam^c C_{j-1} + F_{j-1},   C_0 = 0,
// with F_j the state chunk j reaches from zero.  Two launches:
//   scan_chunk_partials_kernel  F_j for every chunk but the last  (thread = sequence x chunk x 4 channels)
//   scan_chunk_apply_kernel     each thread folds the F_i, i < j, into C_j (a short loop), then
//                               scans its chunk from C_j, writing m; the last chunk writes the state
// The sums are the sequential ones in another association: results agree with
// mixer_scan_kernel to fp32 rounding, not bit for bit.  u, m: [rows][d];
// sequence s occupies rows s*P .. s*P+P-1, or, with offsets, rows
// offsets[seq0+s]-base .. offsets[seq0+s+1]-base-1 (clamped as in
// mixer_scan_ragged_kernel).  F: [nseq][nchunks][d] fp32 scratch.
template <typename TAct>
__device__ __forceinline__ void scan_chunk_range(int64_t seq, int P, const int32_t *offsets, int64_t base,
                                                 int64_t rows, int64_t seq0, int n_ctx, int64_t &r0, int &len)
{
    if (offsets) {
        r0 = min(max((int64_t)offsets[seq0 + seq] - base, (int64_t)0), rows);
        const int64_t r1 = min(max((int64_t)offsets[seq0 + seq + 1] - base, r0), rows);
        len = (int)min(r1 - r0, (int64_t)n_ctx);
    } else {
        r0 = seq * P;
        len = P;
    }
}

template <typename TAct>
__global__ void __launch_bounds__(256)
scan_chunk_partials_kernel(const TAct *__restrict__ u, float *__restrict__ F, const float *__restrict__ alpha,
                           const float *__restrict__ lam, int n_ctx, int H, int hrow, int d, int nseq, int P, int c,
                           int nchunks, const int32_t *__restrict__ offsets, int64_t base, int64_t rows,
                           int64_t seq0)
{
    const int dv = d >> 2, dhv = (d / H) >> 2;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int cv = (int)(gid % dv);
    const int64_t sj = gid / dv;
    const int j = (int)(sj % nchunks);
    const int64_t seq = sj / nchunks;
    if (seq >= nseq || j >= nchunks - 1) return;
    int64_t r0;
    int len;
    scan_chunk_range<TAct>(seq, P, offsets, base, rows, seq0, n_ctx, r0, len);
    const int t0 = j * c, t1 = min(t0 + c, len);
    if (t0 >= len) return;
    const int h = cv / dhv;
    const bool row_repeat = h < hrow;
    const float l = lam[h];
    const TAct *up = u + r0 * (int64_t)d + cv * 4;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int t = t0; t < t1; ++t) {
        const float4 x = load4(up + (int64_t)t * d);
        const float p = row_repeat ? alpha[(size_t)h * n_ctx + t] : 1.0f;
        s.x = fmaf(l, s.x, p * x.x);
        s.y = fmaf(l, s.y, p * x.y);
        s.z = fmaf(l, s.z, p * x.z);
        s.w = fmaf(l, s.w, p * x.w);
    }
    store4(F + (seq * nchunks + j) * (int64_t)d + cv * 4, s);
}

template <typename TAct>
__global__ void __launch_bounds__(256)
scan_chunk_apply_kernel(const TAct *__restrict__ u, TAct *__restrict__ m, float *__restrict__ S,
                        const float *__restrict__ F, const float *__restrict__ alpha,
                        const float *__restrict__ beta, const float *__restrict__ lam, int n_ctx, int H, int hrow, int d,
                        int nseq, int P, int c, int nchunks, const int32_t *__restrict__ offsets, int64_t base,
                        int64_t rows, int64_t seq0, int rep, const int32_t *__restrict__ slot, int64_t nslots)
{
    const int dv = d >> 2, dhv = (d / H) >> 2;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int cv = (int)(gid % dv);
    const int64_t sj = gid / dv;
    const int j = (int)(sj % nchunks);
    const int64_t seq = sj / nchunks;
    if (seq >= nseq) return;
    int64_t r0;
    int len;
    scan_chunk_range<TAct>(seq, P, offsets, base, rows, seq0, n_ctx, r0, len);
    const int t0 = j * c, t1 = min(t0 + c, len);
    if (t0 >= len) return;
    const int h = cv / dhv;
    const bool row_repeat = h < hrow;
    const float l = lam[h];
    float lc = 1.0f;                               // lam^c
    for (int i = 0; i < c; ++i) lc *= l;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    const float *Fp = F + (seq * nchunks) * (int64_t)d + cv * 4;
    for (int i = 0; i < j; ++i) {
        const float4 f = load4(Fp + (int64_t)i * d);
        s.x = fmaf(lc, s.x, f.x);
        s.y = fmaf(lc, s.y, f.y);
        s.z = fmaf(lc, s.z, f.z);
        s.w = fmaf(lc, s.w, f.w);
    }
    const TAct *up = u + r0 * (int64_t)d + cv * 4;
    TAct *mp = m + r0 * (int64_t)d + cv * 4;
    for (int t = t0; t < t1; ++t) {
        const float4 x = load4(up + (int64_t)t * d);
        const float a = alpha[(size_t)h * n_ctx + t], be = beta[(size_t)h * n_ctx + t];
        const float p = row_repeat ? a : 1.0f, q = row_repeat ? 1.0f : a;
        float4 o;
        s.x = fmaf(l, s.x, p * x.x); o.x = fmaf(q, s.x, be);
        s.y = fmaf(l, s.y, p * x.y); o.y = fmaf(q, s.y, be);
        s.z = fmaf(l, s.z, p * x.z); o.z = fmaf(q, s.z, be);
        s.w = fmaf(l, s.w, p * x.w); o.w = fmaf(q, s.w, be);
        store4(mp + (int64_t)t * d, o);
    }
    if (t1 == len) {                               // this chunk ends the sequence: its state is the result
        if (slot) {
            const int64_t dst = slot[seq0 + seq];
            if (dst >= 0 && dst < nslots) store4(S + dst * (int64_t)d + cv * 4, s);
        } else {
            float *dst = S + ((seq0 + seq) * rep) * (int64_t)d + cv * 4;
            for (int r = 0; r < rep; ++r) store4(dst + (int64_t)r * d, s);
        }
    }
}

// Parallel form.  U, Y: [B][T][d].  grid = (ceil(T/64), H * ceil(d_h/64), B);
// a block owns 64 output positions j x up to 64 channels c of one head and sums
// over source positions i <= j in tiles of 64:
//   Y[j][c] = sum_i U[i][c] * M[i][j] + beta_j,
//   M[i][j] = lam^(j-i) * alpha_i (row-repeat) | lam^(j-i) * alpha_j (column-repeat), 0 for i > j.
// lam^k comes from a per-block table computed with pow() in double, not from
// running products, so this path shares no rounding with the recurrence.
// Dynamic LDS: T floats (the power table).
template <typename TAct>
__global__ void __launch_bounds__(256)
mixer_parallel_kernel(const TAct *__restrict__ U, TAct *__restrict__ Y,
                      const float *__restrict__ alpha, const float *__restrict__ beta,
                      const float *__restrict__ lam, int n_ctx, int H, int hrow, int d, int T)
{
    extern __shared__ float pw[];            // [T]
    __shared__ float Ms[64][64 + 4];         // [i][j]
    __shared__ float Us[64][64 + 4];         // [i][c]
    const int dh = d / H;
    const int ctiles = (dh + 63) / 64;
    const int h = blockIdx.y / ctiles, ct = blockIdx.y % ctiles;
    const int jt = blockIdx.x, b = blockIdx.z;
    const int tid = threadIdx.x;
    const bool row_repeat = h < hrow;
    const float *al = alpha + (size_t)h * n_ctx;
    const double lh = (double)lam[h];
    for (int k = tid; k < T; k += 256) pw[k] = (float)pow(lh, (double)k);

    const int j0 = jt * 64, c0 = h * dh + ct * 64, cw = min(64, dh - ct * 64);
    const int tj = tid >> 4, tc = tid & 15;
    const TAct *Ub = U + (size_t)b * T * d;
    float acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[a][c] = 0.0f;

    for (int it = 0; it <= jt; ++it) {
        const int i0 = it * 64;
        __syncthreads();                     // previous tile consumed; pw ready on the first pass
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            const int e = tid + s * 256, ii = e >> 6, x = e & 63;
            const int i = i0 + ii, j = j0 + x;
            Ms[ii][x] = (i <= j && j < T) ? pw[j - i] * (row_repeat ? al[i] : al[j]) : 0.0f;
            Us[ii][x] = (i < T && x < cw) ? (float)Ub[(size_t)i * d + c0 + x] : 0.0f;
        }
        __syncthreads();
#pragma unroll 8
        for (int ii = 0; ii < 64; ++ii) {
            float mj[4], uc[4];
#pragma unroll
            for (int a = 0; a < 4; ++a) mj[a] = Ms[ii][tj * 4 + a];
#pragma unroll
            for (int c = 0; c < 4; ++c) uc[c] = Us[ii][tc * 4 + c];
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[a][c] = fmaf(uc[c], mj[a], acc[a][c]);
        }
    }
    TAct *Yb = Y + (size_t)b * T * d;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const int j = j0 + tj * 4 + a;
        if (j >= T) continue;
        const float be = beta[(size_t)h * n_ctx + j];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int x = tc * 4 + c;
            if (x < cw) store1(Yb + (size_t)j * d + c0 + x, acc[a][c] + be);
        }
    }
}

// Step counters of a multi-step generate call, kept in device memory so that the
// captured step needs no host-side update: ctr[0] = position, ctr[1] = step.  (Every step after the
// first advances them in its first kernel, the embedding LayerNorm.)
__global__ void counters_set_kernel(int *ctr, int pos, int step) { ctr[0] = pos; ctr[1] = step; }
