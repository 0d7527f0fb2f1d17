// Generation with a handful of samples in ONE persistent kernel (fp32 models, at most
// kMegaMaxB samples).  With so few rows every kernel of the ordinary step costs its fixed
// launch-to-completion time (about 4 us on this chip) whatever it computes, and a step is
// 6L + 7 such kernels.  Here a small grid of co-resident work-groups walks through all G steps:
// each work-group owns a fixed slice of the output columns of every matrix, the phases of a
// step are separated by a grid barrier, and LayerNorm is recomputed by every work-group instead
// of being a phase of its own: 4L + 1 barriers per step.  Measured on MI355X: a barrier costs
// about 1.4 us + 65 ns per work-group (device-scope atomics and the cache write-back / invalidate
// of the fences), which is why the grid is small (16 work-groups); a phase then costs one more
// memory latency for the activations the other work-groups have just written, plus its
// arithmetic on 16 CUs.  C1's model: 93 us per step at B = 1 and 128 us at B = 8, against 135 and
// 148 us for the step kernels under graph replay.
//
// Phases of one step (position pos), rows b < B, x = residual stream [B][d] in global memory:
//   layer l:  IN    a = LN1(x) (layer 0: x = embedding rows of the current tokens)
//                   u = a W_in^T + b_in ; S <- lam S + p u ; mbuf = q S + beta     (Eq. 2 / Eq. 3)
//             OUT   x <- x + mbuf W_out^T + b_out
//             UP    a = LN2(x) ; gbuf = GELU(a W_up^T + b_up)
//             DOWN  x <- x + gbuf W_down^T + b_down
//   HEAD      a = LNf(x) ; every work-group: best (score, index) of its vocabulary slice per row
//   next step: every work-group reduces the partial winners itself (same result everywhere)
// The launch must be cooperative (all work-groups resident); every barrier wait is bounded, and
// a work-group that gives up marks the tokens -1 and leaves.
#pragma once
#include "common.hpp"

constexpr int kMegaMaxB = 8;
constexpr int kMegaThreads = 256;      // one wavefront per SIMD: the whole register file (VGPRs and AGPRs) per lane
constexpr int kMegaWaves = kMegaThreads / 64;

struct MegaLayer {
    const float *ln1_g, *ln1_b, *w_in, *b_in, *alpha, *beta, *lam, *w_out, *b_out, *ln2_g, *ln2_b, *w_up, *b_up,
        *w_down, *b_down;
};

struct MegaArgs {
    const MegaLayer *layers;     // [L], device
    const float *embed, *head, *lnf_g, *lnf_b;
    int V, d, dm, ff, L, Hs, hrow, n_ctx;
    float eps;
    int B, pos0, G;
    int32_t *tok;                // [B]: in = tokens at pos0, out = the last generated tokens
    float *state;                // [L][B][dm]
    int32_t *store;              // [G][B] generated tokens
    float temp;                  // > 0: Gumbel-max sampling
    uint32_t seed;
    float *x, *mbuf, *gbuf;      // [B][d], [B][dm], [B][ff]
    float *pv;                   // [gridDim.x][kMegaMaxB] partial winners
    int32_t *pi;
    unsigned *bar;               // barrier slots and give-up flag (see mega_barrier), all zero at the start
};


// Grid barrier without read-modify-write traffic: work-group i publishes the number of the barrier it
// has reached in its own 64-byte slot, and the first wavefront of every work-group polls all slots at
// once (lane i reads slot i) until none is behind.  bar[i * 16] = slot of work-group i (all start at 0),
// bar[kMegaMaxBlocks * 16] = give-up flag.  The wait is bounded: a work-group that gives up raises the
// flag, which ends every other wait.
constexpr int kMegaMaxBlocks = 64;
__device__ __forceinline__ bool mega_barrier(unsigned *bar, unsigned &epoch, int *ok_lds)
{
    __syncthreads();
    if (threadIdx.x < 64) {
        ++epoch;
        if (threadIdx.x == 0) {
            __threadfence();                   // this work-group's writes first
            __hip_atomic_store(bar + blockIdx.x * 16, epoch, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        }
        unsigned *flag = bar + kMegaMaxBlocks * 16;
        const unsigned *slot = bar + (threadIdx.x < gridDim.x ? threadIdx.x : 0) * 16;
        bool ok = true;
        unsigned spins = 0;
        for (;;) {
            const unsigned seen = __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            // unsigned distance, so that the comparison survives a wrap of the counter
            if (__all((int)(seen - epoch) >= 0)) break;
            if (++spins > (1u << 22) || __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
                __hip_atomic_store(flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ok = false;
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        __threadfence();                       // acquire: drop what the caches hold of the others' data
        if (threadIdx.x == 0) *ok_lds = ok;
    }
    __syncthreads();
    return *ok_lds != 0;
}

constexpr int kMegaMaxLayers = 32;   // the layers' pointer tables are kept in LDS
constexpr int kMegaPF = 8;       // float4 values per lane in one weight batch

__device__ __forceinline__ float wave64_sum(float v)
{
    v = row16_sum(v);
    v += __shfl_xor(v, 16, kWave);
    v += __shfl_xor(v, 32, kWave);
    return v;
}

// What one phase does (uniform over the grid); one generic body serves all of them, so that the
// kernel holds one copy of the product loop and the compiler has few loop invariants to keep.
enum { MEGA_IN = 0, MEGA_OUT = 1, MEGA_UP = 2, MEGA_DOWN = 3, MEGA_HEAD = 4 };

struct MegaPhase {
    int kind;
    const float *W;          // [N][K]
    const float *bias;       // [N] or null (head)
    int K, n0, n1;           // this work-group's columns
    // activation rows: LayerNorm of ln_src rows (stride ln_stride; per-row base ln_rows[b] if not null) or a copy of `stage`
    const float *ln_g, *ln_b, *ln_src;
    const float *stage;
    // MEGA_IN: state slab and coefficient tables; MEGA_OUT / MEGA_DOWN: residual source (x, or embedding rows in layer 0)
    float *S;
    const float *alpha, *beta, *lam;
    bool resid_from_embed;
};

// One phase for this work-group: activations into lds_a [MB][K], products of the columns
// [n0, n1) with all rows, epilogue by `kind`.  16 lanes share CPG columns (4 such groups per
// wavefront), each lane covering every 16th float4 of a row; lane (l16 == b) of a group owns
// row b of the group's columns.  All global loads whose addresses are known at the start (first
// weight batch, epilogue operands, activation rows) are issued before anything waits.
template <int MB, int CPG>
__device__ __forceinline__ void mega_phase(const MegaArgs &p, const MegaPhase &ph, float *lds_a, const int *tokb, int pos,
                                           float (&best_v)[CPG], int (&best_i)[CPG])
{
    constexpr int JB = kMegaPF / CPG;
    const int B = p.B, d = p.d;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, l16 = lane & 15;
    const int grp = wave * 4 + (lane >> 4);
    const int K = ph.K, K4 = K >> 2, nch = (K4 + 15) >> 4;
    const int n0 = ph.n0, n1 = ph.n1;
    const bool any = n0 < n1;
    const float4 *W4 = reinterpret_cast<const float4 *>(ph.W);
    const bool owner = l16 < B;
    const int dh = p.dm / p.Hs;

    // ---- first weight batch of round 0 (clamped addresses, zeroed by a select: no control flow between loads)
    float4 w[CPG][JB];
    int n[CPG];
#pragma unroll
    for (int c = 0; c < CPG; ++c) {
        n[c] = n0 + grp * CPG + c;
        const float4 *wr = W4 + (size_t)min(n[c], max(n1 - 1, 0)) * K4;
#pragma unroll
        for (int j = 0; j < JB; ++j) {
            const int k4 = j * 16 + l16;
            const float4 v = wr[min(k4, K4 - 1)];
            w[c][j] = (any && n[c] < n1 && k4 < K4) ? v : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    // ---- epilogue operands of round 0
    float e0[CPG], e1[CPG], e2[CPG], e3[CPG], e4[CPG];
    auto pre = [&](int c, int col) {
        e0[c] = ph.bias ? ph.bias[col] : 0.f;
        e1[c] = e2[c] = e3[c] = e4[c] = 0.f;
        if (ph.kind == MEGA_IN) {
            const int h = col / dh;
            e1[c] = ph.S[(size_t)l16 * p.dm + col];
            e2[c] = ph.alpha[(size_t)h * p.n_ctx + pos];
            e3[c] = ph.beta[(size_t)h * p.n_ctx + pos];
            e4[c] = ph.lam[h];
        } else if (ph.kind == MEGA_OUT || ph.kind == MEGA_DOWN) {
            e1[c] = ph.resid_from_embed ? p.embed[(size_t)tokb[l16] * d + col] : p.x[(size_t)l16 * d + col];
        }
    };
#pragma unroll
    for (int c = 0; c < CPG; ++c) {
        e0[c] = e1[c] = e2[c] = e3[c] = e4[c] = 0.f;
        if (owner && any && n[c] < n1) pre(c, n[c]);
    }
    // ---- activation rows into LDS
    if (ph.stage) {
        for (int i = threadIdx.x * 4; i < B * K; i += kMegaThreads * 4)
            *reinterpret_cast<float4 *>(lds_a + i) = *reinterpret_cast<const float4 *>(ph.stage + i);
    } else {
        // LayerNorm, one wavefront per row (biased variance), two rows in flight per wavefront; K == d here,
        // d <= 1024: at most 4 float4 per lane and row
        for (int b0 = wave; b0 < B; b0 += 2 * kMegaWaves) {
            float4 v[2][4], gg[4], bb[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int k = min((i * 64 + lane) * 4, d - 4);
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const int b = min(b0 + t * kMegaWaves, B - 1);
                    const float *row = ph.ln_src ? ph.ln_src + (size_t)b * d : p.embed + (size_t)tokb[b] * d;
                    v[t][i] = *reinterpret_cast<const float4 *>(row + k);
                }
                gg[i] = *reinterpret_cast<const float4 *>(ph.ln_g + k);
                bb[i] = *reinterpret_cast<const float4 *>(ph.ln_b + k);
            }
            float s[2] = {0.f, 0.f};
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if ((i * 64 + lane) * 4 < d) {
#pragma unroll
                    for (int t = 0; t < 2; ++t) s[t] += v[t][i].x + v[t][i].y + v[t][i].z + v[t][i].w;
                }
            float mean[2], rstd[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) mean[t] = wave64_sum(s[t]) * (1.0f / (float)d);
            float q[2] = {0.f, 0.f};
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if ((i * 64 + lane) * 4 < d) {
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        const float a = v[t][i].x - mean[t], b2 = v[t][i].y - mean[t], c2 = v[t][i].z - mean[t],
                                    e = v[t][i].w - mean[t];
                        q[t] += a * a + b2 * b2 + c2 * c2 + e * e;
                    }
                }
#pragma unroll
            for (int t = 0; t < 2; ++t) rstd[t] = rsqrtf(wave64_sum(q[t]) * (1.0f / (float)d) + p.eps);
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int b = b0 + t * kMegaWaves;
                if (b < B) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int k = (i * 64 + lane) * 4;
                        if (k < d) {
                            float4 o;
                            o.x = (v[t][i].x - mean[t]) * rstd[t] * gg[i].x + bb[i].x;
                            o.y = (v[t][i].y - mean[t]) * rstd[t] * gg[i].y + bb[i].y;
                            o.z = (v[t][i].z - mean[t]) * rstd[t] * gg[i].z + bb[i].z;
                            o.w = (v[t][i].w - mean[t]) * rstd[t] * gg[i].w + bb[i].w;
                            *reinterpret_cast<float4 *>(lds_a + (size_t)b * d + k) = o;
                        }
                    }
                }
            }
        }
    }
    __syncthreads();
    if (!any) return;

    // ---- rounds over the slice, each a sequence of weight batches; the next batch (of this round or of the
    // next one) is requested before the current one is used.  All loop bounds are wave-uniform.
    const float4 *a4 = reinterpret_cast<const float4 *>(lds_a);
    const int first = n0 + wave * 4 * CPG, stride = kMegaWaves * 4 * CPG;
    const int rounds = first < n1 ? (n1 - first + stride - 1) / stride : 0;
    const int nbatch = (nch + JB - 1) / JB;
    const int total = rounds * nbatch;
    float acc[CPG][MB];
    int r = 0, jb = 0;
#pragma unroll 1
    for (int t = 0; t < total; ++t) {
        float4 wn[CPG][JB];
        int r2 = r, jb2 = jb + 1;
        if (jb2 == nbatch) { jb2 = 0; ++r2; }
        if (t + 1 < total) {
#pragma unroll
            for (int c = 0; c < CPG; ++c) {
                const int col = n0 + (r2 * kMegaWaves * 4 + grp) * CPG + c;
                const float4 *wr = W4 + (size_t)min(col, n1 - 1) * K4;
#pragma unroll
                for (int j = 0; j < JB; ++j) {
                    const int k4 = (jb2 * JB + j) * 16 + l16;
                    const float4 v = wr[min(k4, K4 - 1)];
                    wn[c][j] = (col < n1 && k4 < K4) ? v : make_float4(0.f, 0.f, 0.f, 0.f);
                }
            }
        }
        if (jb == 0) {
            if (r > 0) {
#pragma unroll
                for (int c = 0; c < CPG; ++c) {
                    n[c] = n0 + (r * kMegaWaves * 4 + grp) * CPG + c;
                    e0[c] = e1[c] = e2[c] = e3[c] = e4[c] = 0.f;
                    if (owner && n[c] < n1) pre(c, n[c]);
                }
            }
#pragma unroll
            for (int c = 0; c < CPG; ++c)
#pragma unroll
                for (int b = 0; b < MB; ++b) acc[c][b] = 0.f;
        }
        // all MB rows are read whatever B is (rows >= B hold finite filler) and a k-chunk past the end reads a
        // clamped address against zero weights: straight-line code, reads issued in batches
#pragma unroll
        for (int j = 0; j < JB; ++j) {
            const int k4 = min((jb * JB + j) * 16 + l16, K4 - 1);
            float4 a[MB];
#pragma unroll
            for (int b = 0; b < MB; ++b) a[b] = a4[b * K4 + k4];
#pragma unroll
            for (int b = 0; b < MB; ++b)
#pragma unroll
                for (int c = 0; c < CPG; ++c) {
                    acc[c][b] = fmaf(w[c][j].x, a[b].x, acc[c][b]);
                    acc[c][b] = fmaf(w[c][j].y, a[b].y, acc[c][b]);
                    acc[c][b] = fmaf(w[c][j].z, a[b].z, acc[c][b]);
                    acc[c][b] = fmaf(w[c][j].w, a[b].w, acc[c][b]);
                }
        }
        if (jb == nbatch - 1) {
#pragma unroll
            for (int c = 0; c < CPG; ++c) {
                float mine = 0.f;
#pragma unroll
                for (int b = 0; b < MB; ++b) {
                    const float v = row16_sum(acc[c][b]);
                    if (l16 == b) mine = v;
                }
                const int col = n[c];
                if (owner && col < n1) {
                    const float tt = mine + e0[c];
                    if (ph.kind == MEGA_IN) {                       // Eq. 2 / Eq. 3
                        const bool row_repeat = col / dh < p.hrow;
                        const float pp = row_repeat ? e2[c] : 1.0f, qq = row_repeat ? 1.0f : e2[c];
                        const float s_new = fmaf(e4[c], e1[c], pp * tt);
                        ph.S[(size_t)l16 * p.dm + col] = s_new;
                        p.mbuf[(size_t)l16 * p.dm + col] = fmaf(qq, s_new, e3[c]);
                    } else if (ph.kind == MEGA_UP) {
                        p.gbuf[(size_t)l16 * p.ff + col] = gelu_erf(tt);
                    } else if (ph.kind == MEGA_HEAD) {
                        float score = mine;
                        if (p.temp > 0.0f)
                            score = mine + p.temp * srm_gumbel(srm_rowkey(p.seed, (uint32_t)pos, (uint32_t)l16), (uint32_t)col);
                        if (arg_better(score, col, best_v[c], best_i[c])) { best_v[c] = score; best_i[c] = col; }
                    } else {                                        // MEGA_OUT, MEGA_DOWN
                        p.x[(size_t)l16 * d + col] = e1[c] + tt;
                    }
                }
            }
        }
#pragma unroll
        for (int c = 0; c < CPG; ++c)
#pragma unroll
            for (int j = 0; j < JB; ++j) w[c][j] = wn[c][j];
        r = r2;
        jb = jb2;
    }
}

// MB = number of rows the arithmetic is unrolled for (B <= MB <= kMegaMaxB).
template <int MB>
__global__ void __launch_bounds__(kMegaThreads) mega_generate_kernel(MegaArgs p)
{
    extern __shared__ __align__(16) float mega_lds[];       // [MB][max(d, dm, ff)]
    __shared__ int tokb[kMegaMaxB];
    __shared__ MegaLayer lay[kMegaMaxLayers];                // a global (or scalar-cache) read per phase would cost a memory latency
    __shared__ int bar_ok;
    __shared__ float red_v[kMegaWaves * 4][kMegaMaxB];
    __shared__ int red_i[kMegaWaves * 4][kMegaMaxB];
    float *lds_a = mega_lds;
    const int B = p.B, d = p.d, dm = p.dm, ff = p.ff, V = p.V;
    const int nblk = gridDim.x, blk = blockIdx.x;
    unsigned epoch = 0;
    // this work-group's column slices (whole columns; the last work-groups may get none)
    auto slice = [&](int N, int &n0, int &n1) {
        const int per = (N + nblk - 1) / nblk;
        n0 = min(N, blk * per);
        n1 = min(N, n0 + per);
    };
    if (threadIdx.x < B) tokb[threadIdx.x] = p.tok[threadIdx.x];
    for (int i = threadIdx.x; i < p.L * (int)(sizeof(MegaLayer) / sizeof(float *)); i += kMegaThreads)
        reinterpret_cast<const float **>(lay)[i] = reinterpret_cast<const float *const *>(p.layers)[i];
    {   // the products read MB rows of the activation stage whatever B is: start from zeros
        const int widest = max(max(d, dm), ff);
        for (int i = threadIdx.x; i < MB * widest; i += kMegaThreads) lds_a[i] = 0.f;
    }
    __syncthreads();
    constexpr int CW = 4;                                   // columns per lane group where the slice is wide
    const int nphase = 4 * p.L + 1;

    for (int g = 0; g < p.G; ++g) {
        const int pos = p.pos0 + g;
        float best_v[CW];
        int best_i[CW];
#pragma unroll
        for (int c = 0; c < CW; ++c) { best_v[c] = -INFINITY; best_i[c] = 0x7fffffff; }
#pragma unroll 1
        for (int ip = 0; ip < nphase; ++ip) {
            const int l = ip >> 2;
            MegaPhase ph;
            ph.kind = ip == nphase - 1 ? MEGA_HEAD : (ip & 3);
            const MegaLayer &y = lay[ph.kind == MEGA_HEAD ? 0 : l];
            ph.ln_g = ph.ln_b = ph.ln_src = ph.stage = nullptr;
            ph.S = nullptr;
            ph.alpha = ph.beta = ph.lam = nullptr;
            ph.resid_from_embed = false;
            int N;
            switch (ph.kind) {
            case MEGA_IN:
                ph.W = y.w_in; ph.bias = y.b_in; ph.K = d; N = dm;
                ph.ln_g = y.ln1_g; ph.ln_b = y.ln1_b; ph.ln_src = l == 0 ? nullptr : p.x;
                ph.S = p.state + (size_t)l * B * dm; ph.alpha = y.alpha; ph.beta = y.beta; ph.lam = y.lam;
                break;
            case MEGA_OUT:
                ph.W = y.w_out; ph.bias = y.b_out; ph.K = dm; N = d;
                ph.stage = p.mbuf; ph.resid_from_embed = l == 0;
                break;
            case MEGA_UP:
                ph.W = y.w_up; ph.bias = y.b_up; ph.K = d; N = ff;
                ph.ln_g = y.ln2_g; ph.ln_b = y.ln2_b; ph.ln_src = p.x;
                break;
            case MEGA_DOWN:
                ph.W = y.w_down; ph.bias = y.b_down; ph.K = ff; N = d;
                ph.stage = p.gbuf;
                break;
            default:
                ph.W = p.head; ph.bias = nullptr; ph.K = d; N = V;
                ph.ln_g = p.lnf_g; ph.ln_b = p.lnf_b; ph.ln_src = p.x;
                break;
            }
            slice(N, ph.n0, ph.n1);
            // narrow slices: one column per lane group keeps all wavefronts busy; wide ones: CW columns share
            // every activation value read from LDS
            if (ph.n1 - ph.n0 > kMegaWaves * 4) {
                mega_phase<MB, CW>(p, ph, lds_a, tokb, pos, best_v, best_i);
            } else {
                float bv1[1] = {-INFINITY};
                int bi1[1] = {0x7fffffff};
                mega_phase<MB, 1>(p, ph, lds_a, tokb, pos, bv1, bi1);
                if (ph.kind == MEGA_HEAD) { best_v[0] = bv1[0]; best_i[0] = bi1[0]; }
            }
            if (ph.kind == MEGA_HEAD) {
                // best (score, index) of this work-group's vocabulary slice, per row
                const int lane = threadIdx.x & 63, l16 = lane & 15;
                float bv = best_v[0];
                int bi = best_i[0];
#pragma unroll
                for (int c = 1; c < CW; ++c)
                    if (arg_better(best_v[c], best_i[c], bv, bi)) { bv = best_v[c]; bi = best_i[c]; }
                if (l16 < B) {
                    red_v[(threadIdx.x >> 6) * 4 + (lane >> 4)][l16] = bv;
                    red_i[(threadIdx.x >> 6) * 4 + (lane >> 4)][l16] = bi;
                }
                __syncthreads();
                if (threadIdx.x < B) {
                    bv = red_v[0][threadIdx.x];
                    bi = red_i[0][threadIdx.x];
                    for (int r = 1; r < kMegaWaves * 4; ++r)
                        if (arg_better(red_v[r][threadIdx.x], red_i[r][threadIdx.x], bv, bi)) {
                            bv = red_v[r][threadIdx.x];
                            bi = red_i[r][threadIdx.x];
                        }
                    p.pv[blk * kMegaMaxB + threadIdx.x] = bv;
                    p.pi[blk * kMegaMaxB + threadIdx.x] = bi;
                }
            }
            if (!mega_barrier(p.bar, epoch, &bar_ok)) goto give_up;
        }
        // ---- every work-group picks the winners from all partials (identical everywhere)
        if (threadIdx.x < B) {
            float bv = p.pv[threadIdx.x];
            int bi = p.pi[threadIdx.x];
            for (int r = 1; r < nblk; ++r) {
                const float ov = p.pv[r * kMegaMaxB + threadIdx.x];
                const int oi = p.pi[r * kMegaMaxB + threadIdx.x];
                if (arg_better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
            }
            tokb[threadIdx.x] = bi;
            if (blk == 0) {
                p.store[(size_t)g * B + threadIdx.x] = bi;
                p.tok[threadIdx.x] = bi;
            }
        }
        __syncthreads();
    }
    return;
give_up:
    if (threadIdx.x < B) p.tok[threadIdx.x] = -1;
}

// The barrier slots and the give-up flag start at zero; the token store starts at -1, so that the rows of
// the steps a kernel that gave up never reached are recognisable.
__global__ void mega_reset_kernel(unsigned *bar, int32_t *store, int n_store)
{
    for (int i = threadIdx.x; i <= kMegaMaxBlocks * 16; i += blockDim.x) bar[i] = 0u;
    for (int i = threadIdx.x; i < n_store; i += blockDim.x) store[i] = -1;
}
