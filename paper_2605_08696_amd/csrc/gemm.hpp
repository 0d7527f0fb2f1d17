// GEMMs of the SRM block: out = epilogue(A W^T + bias), A [M][K], W [N][K]
// (both K-contiguous), for the head projections (Eq. 10), the channel-mixing
// MLP and the LM head.
//
//   gemm_bf16_kernel: bf16 operands on the gfx950 matrix cores
//     (v_mfma_f32_32x32x16_bf16, fp32 accumulate); tiles go global -> LDS with
//     buffer_load ... lds into a 16-byte XOR-swizzled layout, two LDS stages,
//     operands read from LDS two k-substeps ahead of the MFMAs that use them.
//   gemm_f32_kernel: plain fp32 FMA tiles for the fp32 configurations.
//
// Epilogues are fused: bias, exact GELU, residual add into the fp32 stream,
// and for the LM head a per-tile (max, index) partial so that logits need not
// be written at all.
#pragma once
#include "common.hpp"
#include <type_traits>

enum { EPI_STORE = 0, EPI_GELU = 1, EPI_RESID = 2, EPI_ARGMAX = 3, EPI_F32 = 4, EPI_MIX = 5 };

struct GemmEpi {
    const float *bias;   // [N] or nullptr
    void *out;           // EPI_STORE/GELU: TAct [M][ldo]; EPI_RESID: float [M][ldo] (+=);
                         // EPI_F32: float [M][ldo]; EPI_ARGMAX: float [M][ldo] or nullptr
    int64_t ldo;
    float *part_val;     // EPI_ARGMAX: [nparts][M] (part-major: the rows of a tile write consecutive words)
    int32_t *part_idx;   // EPI_ARGMAX: [nparts][M]
    int32_t nparts;      // number of column tiles
    // EPI_ARGMAX with temp > 0: the decision is argmax_v(logit_v + temp * gumbel(seed, pos, row, v)),
    // i.e. a sample from softmax(logits / temp); stored logits stay the raw ones.
    float temp;
    uint32_t seed;
    int32_t pos;         // position of the counter, unless pos_dev or pos_rows is set
    const int *pos_dev;  // one position for all rows, in device memory
    const int *pos_rows; // [M] one position per row, in device memory
    uint32_t row_base;   // sample index of row 0 (the random counter is keyed on the sample, not on the GEMM row)
    // EPI_MIX: the recurrent state update (Eq. 2 / Eq. 3) applied to the product, which is the
    // stacked head projection u: S <- lam*S + p*u, out = q*S + beta at the row's position
    // (pos / pos_dev / pos_rows as above; a position outside [0, n_ctx) leaves S alone and
    // writes zeros).  state: [M][ldo], fp32 or (state_half) binary16; alpha, beta: [H][n_ctx];
    // lam: [H]; dh = ldo / H.
    void *state;
    const float *alpha, *beta, *lam;
    int32_t n_ctx, hrow, dh, state_half;   // heads 0..hrow-1 row-repeat, the rest column-repeat
    // EPI_RESID: add_nsplit slabs [M][ldo] (slab stride add_stride floats) are added to the old value first, in
    // slab order: the pending result of a K-sliced projection, which no kernel has folded into the stream yet.
    const float *add_part;
    int32_t add_nsplit;
    int64_t add_stride;
    // LNA kernels (A operand = LayerNorm of ln_x rows, computed by the block): ln_x [M][K] fp32 (+ ln_nsplit slabs
    // of a K-sliced projection, added first in slab order, stride ln_stride floats), gain, bias, epsilon.
    const float *ln_x, *ln_g, *ln_b, *ln_part;
    int32_t ln_nsplit;
    int64_t ln_stride;
    float ln_eps;
    // Measuring hook (srm_linear_timeline_probe): if not null, every work-group b < clk_blocks of
    // gemm_bf16_kernel writes eight words at clk + 8 b: the 100 MHz wall clock at its start, at the start
    // of its k loop, at the end of the k loop and after its last store has completed; the shader cycle
    // counter at the k loop's start and end; HW_ID | XCC_ID << 32 (which CU it ran on); the cycle
    // counter at its start.  (gemm_bf16_persist_kernel: one record per output tile.)
    unsigned long long *clk;
    int64_t clk_blocks;
};

// The position all rows share: ep.pos, or *ep.pos_dev if that is set.  (Written as a conditional load with a
// scalar result: from `pos_dev ? *pos_dev : pos` the compiler made a load through a selected pointer, which
// needs ep.pos in scratch memory and a flat load per use.)
__device__ __forceinline__ uint32_t epi_shared_pos(const GemmEpi &ep)
{
    int p = ep.pos;
    if (ep.pos_dev) p = __builtin_amdgcn_readfirstlane(*ep.pos_dev);
    return (uint32_t)p;
}
// Position that keys the random numbers of output row `row` (rows >= M read nothing).
__device__ __forceinline__ uint32_t epi_pos(const GemmEpi &ep, int64_t row, int M)
{
    if (ep.pos_rows) return row < M ? (uint32_t)ep.pos_rows[row] : 0u;
    return epi_shared_pos(ep);
}

// Block -> tile mapping.  Workgroups are dealt round-robin to the 8 XCDs, each
// with its own L2: give every XCD one contiguous run of tiles, and inside a run
// walk groups of GM row-tiles column by column so the A rows of a group and the
// W tile being shared stay L2-resident.
__device__ __forceinline__ void tile_of_pid(int pid, int nbm, int nbn, int &bm, int &bn)
{
    constexpr int GM = 8;
    const int nblk = nbm * nbn;
    if ((nblk & 7) == 0) pid = (pid & 7) * (nblk >> 3) + (pid >> 3);
    const int gsz = GM * nbn;
    const int g = pid / gsz;
    const int first_m = g * GM;
    const int gm = min(nbm - first_m, GM);
    const int in_g = pid - g * gsz;
    bm = first_m + in_g % gm;
    bn = in_g / gm;
}
__device__ __forceinline__ void tile_of_block(int nbm, int nbn, int &bm, int &bn)
{
    tile_of_pid(blockIdx.x, nbm, nbn, bm, bn);
}

template <int EPI, typename TAct>
__device__ __forceinline__ void epi_store(const GemmEpi &ep, int64_t row, int col, float v)
{
    if constexpr (EPI == EPI_STORE) {
        store1(reinterpret_cast<TAct *>(ep.out) + row * ep.ldo + col, v);
    } else if constexpr (EPI == EPI_GELU) {
        store1(reinterpret_cast<TAct *>(ep.out) + row * ep.ldo + col, gelu_erf(v));
    } else if constexpr (EPI == EPI_RESID) {
        float *p = reinterpret_cast<float *>(ep.out) + row * ep.ldo + col;
        float o = *p;
        for (int s_ = 0; s_ < ep.add_nsplit; ++s_) o += ep.add_part[(int64_t)s_ * ep.add_stride + row * ep.ldo + col];
        *p = o + v;
    } else if constexpr (EPI == EPI_F32) {
        reinterpret_cast<float *>(ep.out)[row * ep.ldo + col] = v;
    } else if constexpr (EPI == EPI_MIX) {
        const int pos = (int)(ep.pos_rows ? (uint32_t)ep.pos_rows[row] : epi_shared_pos(ep));
        TAct *o = reinterpret_cast<TAct *>(ep.out) + row * ep.ldo + col;
        if (pos < 0 || pos >= ep.n_ctx) { store1(o, 0.0f); return; }
        const int h = col / ep.dh;
        const float a = ep.alpha[(size_t)h * ep.n_ctx + pos], be = ep.beta[(size_t)h * ep.n_ctx + pos], l = ep.lam[h];
        const bool row_repeat = h < ep.hrow;
        const float p = row_repeat ? a : 1.0f, q = row_repeat ? 1.0f : a;
        const float u = (float)(TAct)v;                 // u in the activation type, as the unfused path stores it
        float n;
        if (ep.state_half) {
            f16 *sp = static_cast<f16 *>(ep.state) + row * ep.ldo + col;
            n = to_state(fmaf(l, (float)*sp, p * u), sp);
            *sp = (f16)n;
        } else {
            float *sp = static_cast<float *>(ep.state) + row * ep.ldo + col;
            n = fmaf(l, *sp, p * u);
            *sp = n;
        }
        store1(o, fmaf(q, n, be));
    } else {
        if (ep.out) reinterpret_cast<float *>(ep.out)[row * ep.ldo + col] = v;
    }
}

// ------------------------------------------------------------------ bf16 MFMA
// Block tile BM x BN x 64 split over WM x WN waves, each wave holding a
// (BM/WM) x (BN/WN) accumulator tile of 32x32x16 MFMAs.  Built to keep the matrix
// pipe fed:
//  (1) the MFMA operands of k-substep kk+1 are read from LDS before the MFMAs of
//      kk issue (two register sets, order pinned with scheduling barriers);
//  (2) tiles travel global -> LDS directly (buffer_load ... lds), two tiles ahead
//      of the MFMAs, and the barrier sits one substep before the end of a tile
//      (see the pipeline table in the kernel); writing the tiles with ds_write
//      from registers instead cost ~30% of the main loop;
//  (3) the product is formed transposed (W fragment as the first MFMA operand),
//      so a lane holds four consecutive output columns of ONE row per register
//      quad: the LM-head argmax reduces in-lane and needs a single cross-lane
//      exchange, and the epilogue passes 32-row slices through a wave-private
//      LDS stage with 16-byte writes and reads, so that global stores and the
//      residual read-modify-write are 16-byte vectors over whole cache lines.
// LDS chunk swizzle: 16-byte chunk c of row r sits at chunk c ^ ((r >> 1) & 7);
// with 64 banks this makes both the tile writes and the fragment reads
// conflict-free (measured: SQ_LDS_BANK_CONFLICT ~1% of SQ_LDS_IDX_ACTIVE).
__device__ __forceinline__ int swz_of_row(int r) { return (r >> 1) & 7; }

// f(integral_constant<int, I>) for I = FIRST .. LAST-1, unrolled by construction
template <int FIRST, int LAST, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (FIRST < LAST) {
        f(std::integral_constant<int, FIRST>{});
        static_for<FIRST + 1, LAST>(f);
    }
}

// Exact (erf) GELU for bf16 outputs: x * Phi(x) with erfc(|x| / sqrt(2)) / 2 = 2^-P(|x|), |x| clamped to
// 4.3 * sqrt(2) (beyond it Phi is 0 or 1 to 1e-9), P a degree-6 polynomial fitted to
// -log2(erfc(z) / 2), z = |x| / sqrt(2) (minimax in the absolute error of erfc: 2.2e-7; |error| of the
// GELU value <= 6.5e-7 in fp32 evaluation; the 1 / sqrt(2) is folded into the coefficients), so one exp2
// and six FMAs, no reciprocal.  With q = 2^-P: x * (1 - q) for x >= 0 and x * q for x < 0 are both
// max(x, 0) - |x| * q, one max and one FMA instead of a subtraction, a compare, a select and a
// product.  The result is rounded to bf16 (relative 2^-9) right after, so the approximation error is
// invisible there.
__device__ __forceinline__ float gelu_bf16out(float x)
{
    // Eleven instructions, written out: from the C form the compiler made 14 to 18 per element (a
    // NaN-quieting max in front of each min / max, whose inputs come straight from LDS, and a move per
    // constant in every other Horner chain), and this epilogue is bound by its instruction count.
    //   w = min(|x|, 6.0811183)                       P(w) by Horner, coefficients high to low:
    //   -1.917465077776602e-05, 0.0006586045579087176, -0.00775440879176911, 0.05296539231773387,
    //   0.4590602540550674, 1.1511220519383694, 0.9999996936263803
    //   q = 2^-P ;  result = max(x, 0) - |x| * q
    float w, p, q, r;
    const float c5 = 0.0006586045579087176f;
    asm("v_and_b32 %0, 0x7fffffff, %4\n\t"
        "v_min_f32 %0, 0x40c29885, %0\n\t"
        "v_fmamk_f32 %1, %0, 0xb7a0d940, %5\n\t"
        "v_fmaak_f32 %1, %0, %1, 0xbbfe18b2\n\t"
        "v_fmaak_f32 %1, %0, %1, 0x3d58f23d\n\t"
        "v_fmaak_f32 %1, %0, %1, 0x3eeb09f2\n\t"
        "v_fmaak_f32 %1, %0, %1, 0x3f9357f8\n\t"
        "v_fmaak_f32 %1, %0, %1, 0x3f7ffffb\n\t"
        "v_exp_f32_e64 %2, -%1\n\t"
        "v_max_f32 %3, 0, %4\n\t"
        "v_fma_f32 %3, -|%4|, %2, %3"
        : "=&v"(w), "=&v"(p), "=&v"(q), "=&v"(r)
        : "v"(x), "v"(c5));
    return r;
}

// GELU in the precision of the output type: the fitted form for bf16 outputs, erf for fp32 ones.
__device__ __forceinline__ float gelu_for(const bf16 *, float x) { return gelu_bf16out(x); }
__device__ __forceinline__ float gelu_for(const float *, float x) { return gelu_erf(x); }

template <int EPI, typename TAct>
__device__ __forceinline__ void epi_store4(const GemmEpi &ep, int64_t row, int col, float4 v)
{
    if constexpr (EPI == EPI_STORE) {
        store4(reinterpret_cast<TAct *>(ep.out) + row * ep.ldo + col, v);
    } else if constexpr (EPI == EPI_GELU) {
        TAct *o = reinterpret_cast<TAct *>(ep.out) + row * ep.ldo + col;
        store4(o, make_float4(gelu_for(o, v.x), gelu_for(o, v.y), gelu_for(o, v.z), gelu_for(o, v.w)));
    } else if constexpr (EPI == EPI_RESID) {
        float *p = reinterpret_cast<float *>(ep.out) + row * ep.ldo + col;
        float4 o = load4(p);
        for (int s_ = 0; s_ < ep.add_nsplit; ++s_) {
            const float4 t = load4(ep.add_part + (int64_t)s_ * ep.add_stride + row * ep.ldo + col);
            o.x += t.x; o.y += t.y; o.z += t.z; o.w += t.w;
        }
        store4(p, make_float4(o.x + v.x, o.y + v.y, o.z + v.z, o.w + v.w));
    } else if constexpr (EPI == EPI_F32) {
        store4(reinterpret_cast<float *>(ep.out) + row * ep.ldo + col, v);
    } else if constexpr (EPI == EPI_MIX) {
        // four consecutive channels lie in one head (dh is a multiple of 4)
        const int pos = (int)(ep.pos_rows ? (uint32_t)ep.pos_rows[row] : epi_shared_pos(ep));
        TAct *o = reinterpret_cast<TAct *>(ep.out) + row * ep.ldo + col;
        if (pos < 0 || pos >= ep.n_ctx) { store4(o, make_float4(0.f, 0.f, 0.f, 0.f)); return; }
        const int h = col / ep.dh;
        const float a = ep.alpha[(size_t)h * ep.n_ctx + pos], be = ep.beta[(size_t)h * ep.n_ctx + pos], l = ep.lam[h];
        const bool row_repeat = h < ep.hrow;
        const float p = row_repeat ? a : 1.0f, q = row_repeat ? 1.0f : a;
        const int64_t sj = (row * ep.ldo + col) >> 2;
        float4 n, m;
        if (ep.state_half) {
            f16 *sp = static_cast<f16 *>(ep.state);
            const float4 s0 = load_state4(sp, sj);
            n.x = to_state(fmaf(l, s0.x, p * (float)(TAct)v.x), sp);
            n.y = to_state(fmaf(l, s0.y, p * (float)(TAct)v.y), sp);
            n.z = to_state(fmaf(l, s0.z, p * (float)(TAct)v.z), sp);
            n.w = to_state(fmaf(l, s0.w, p * (float)(TAct)v.w), sp);
            store_state4(sp, sj, n);
        } else {
            float *sp = static_cast<float *>(ep.state);
            const float4 s0 = load_state4(sp, sj);
            n.x = fmaf(l, s0.x, p * (float)(TAct)v.x);
            n.y = fmaf(l, s0.y, p * (float)(TAct)v.y);
            n.z = fmaf(l, s0.z, p * (float)(TAct)v.z);
            n.w = fmaf(l, s0.w, p * (float)(TAct)v.w);
            store_state4(sp, sj, n);
        }
        m.x = fmaf(q, n.x, be);
        m.y = fmaf(q, n.y, be);
        m.z = fmaf(q, n.z, be);
        m.w = fmaf(q, n.w, be);
        store4(o, m);
    } else {
        if (ep.out) store4(reinterpret_cast<float *>(ep.out) + row * ep.ldo + col, v);
    }
}

template <int EPI, typename TAct>
__device__ __forceinline__ void epi_store1p(const GemmEpi &ep, int64_t row, int col, float v)
{
    if constexpr (EPI == EPI_GELU) {
        TAct *o = reinterpret_cast<TAct *>(ep.out) + row * ep.ldo + col;
        store1(o, gelu_for(o, v));
    } else {
        epi_store<EPI, TAct>(ep, row, col, v);
    }
}

// Epilogue shared by the bf16 kernels.  Accumulator register r of lane (lk, lr)
// of tile (i, j) is output row i*32 + lr, column j*32 + 8*(r/4) + 4*lk + r%4 of
// the wave tile.  smem_raw: the block's LDS, free for reuse (all tile reads and
// loads have completed and a barrier has been passed); lds_bytes its size.
template <int BM, int BN, int WM, int WN, int EPI, typename TAct>
__device__ __forceinline__ void gemm_epilogue(f32x16_t (&acc)[BM / WM / 32][BN / WN / 32], unsigned char *smem_raw,
                                              const GemmEpi &ep, int M, int N, int m0, int n0, int bn,
                                              const int tid = threadIdx.x)
{
    constexpr int NW = WM * WN, NTHR = NW * 64;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int STG = WTN + 4;                     // stage row stride in floats: 16 B * odd
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int lr = lane & 31, lk = lane >> 5;
    float *stage = reinterpret_cast<float *>(smem_raw) + wave * 32 * STG;        // wave-private [32][STG]
    float *red_val = reinterpret_cast<float *>(smem_raw) + NW * 32 * STG;        // [BM][WN]
    int *red_idx = reinterpret_cast<int *>(red_val + BM * WN);                   // [BM][WN]
    const bool vec_ok = (N & 3) == 0;
    constexpr int LPR = WTN / 4;                      // lanes per staged row
    constexpr int RPI = 64 / LPR;                     // rows per read instruction
    const int s_row = lane / LPR, s_col = (lane % LPR) * 4;
    const int wcol0 = n0 + wn * WTN;                  // first column of this wave's tile
    const int gcol = wcol0 + s_col;
    const bool want_store = EPI != EPI_ARGMAX || ep.out != nullptr;
    const bool n_edge = wcol0 + WTN > N;              // wave-uniform
    const bool cols_inside = vec_ok && n0 + BN <= N;                   // block-uniform
    const bool rows_inside = m0 + BM <= M;                             // block-uniform

    // (a compile-time loop: with the largest epilogue the compiler kept `#pragma unroll` rolled, which indexes
    // the accumulators with a variable and so moves all of them, main loop included, to scratch memory)
    static_for<0, TM>([&](auto ic_) {
        constexpr int i = decltype(ic_)::value;
        if constexpr (EPI == EPI_ARGMAX) {
            // in-lane over this lane's TN*16 columns in ascending order (strict >
            // keeps the lowest index), then one exchange with the lane holding
            // the other half of the row's columns
            float bv = -INFINITY;
            int brel = 0;
            if (ep.temp > 0.0f) {
                const int srow = m0 + wm * WTM + i * 32 + lr;
                const uint32_t rk = srm_rowkey(ep.seed, epi_pos(ep, srow, M), (uint32_t)srow + ep.row_base);
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int rel = j * 32 + 8 * (r >> 2) + (r & 3);
                        const int col = wcol0 + 4 * lk + rel;
                        const float v = acc[i][j][r] + ep.temp * srm_gumbel(rk, (uint32_t)col);
                        if (col < N && v > bv) { bv = v; brel = rel; }
                    }
            } else if (!n_edge) {
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float v = acc[i][j][r];
                        if (v > bv) { bv = v; brel = j * 32 + 8 * (r >> 2) + (r & 3); }
                    }
            } else {
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int rel = j * 32 + 8 * (r >> 2) + (r & 3);
                        const int col = wcol0 + 4 * lk + rel;
                        const float v = acc[i][j][r];
                        if (col < N && v > bv) { bv = v; brel = rel; }
                    }
            }
            int bi = bv == -INFINITY ? 0x7fffffff : wcol0 + 4 * lk + brel;
            const float ov = __shfl_xor(bv, 32, kWave);
            const int oi = __shfl_xor(bi, 32, kWave);
            if (arg_better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
            if (lk == 0) {
                const int lrow = wm * WTM + i * 32 + lr;
                red_val[lrow * WN + wn] = bv;
                red_idx[lrow * WN + wn] = bi;
            }
        }
        if (want_store) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    *reinterpret_cast<float4 *>(stage + lr * STG + j * 32 + 8 * g + 4 * lk) =
                        make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
            // All columns of the tile inside the matrix: no column tests, all staged reads (and, for the
            // residual add and the state update, all loads of the old values) issued before the first use,
            // so their latencies overlap instead of adding up once per 128-byte row segment.  Compiled
            // twice: for tiles with all rows inside too (no tests at all; the hot path of large batches),
            // and for the last row tile (a handful of rows), where rows past M load from row M - 1
            // instead and store nothing.
            auto whole_columns = [&](auto rows_inside_c) {
                constexpr bool RI = decltype(rows_inside_c)::value;
                constexpr int NIT = 32 / RPI;
                const int64_t row0 = m0 + wm * WTM + i * 32 + s_row;
                auto row_of = [&](int it) {
                    if constexpr (RI) return row0 + it * RPI;
                    else return min(row0 + it * RPI, (int64_t)M - 1);
                };
                auto exists = [&](int it) {
                    if constexpr (RI) return true;
                    else return row0 + it * RPI < M;
                };
                float4 v[NIT];
#pragma unroll
                for (int it = 0; it < NIT; ++it)
                    v[it] = *reinterpret_cast<const float4 *>(stage + (it * RPI + s_row) * STG + s_col);
                if constexpr (EPI == EPI_RESID) {
                    float *p = reinterpret_cast<float *>(ep.out) + gcol;
                    float4 o[NIT];
#pragma unroll
                    for (int it = 0; it < NIT; ++it) o[it] = load4(p + row_of(it) * ep.ldo);
                    for (int s_ = 0; s_ < ep.add_nsplit; ++s_) {
                        const float *q = ep.add_part + (int64_t)s_ * ep.add_stride + gcol;
#pragma unroll
                        for (int it = 0; it < NIT; ++it) {
                            const float4 t = load4(q + row_of(it) * ep.ldo);
                            o[it].x += t.x; o[it].y += t.y; o[it].z += t.z; o[it].w += t.w;
                        }
                    }
#pragma unroll
                    for (int it = 0; it < NIT; ++it)
                        if (exists(it))
                            store4(p + row_of(it) * ep.ldo,
                                   make_float4(o[it].x + v[it].x, o[it].y + v[it].y, o[it].z + v[it].z, o[it].w + v[it].w));
                } else if constexpr (EPI == EPI_MIX) {
                    // the state update of NIT rows: positions, coefficients and old states are all
                    // requested before the first is used
                    const int h = gcol / ep.dh;
                    const bool row_repeat = h < ep.hrow;
                    const float l = ep.lam[h];
                    int ps[NIT];
                    float al[NIT], be[NIT];
                    float4 s0[NIT];
#pragma unroll
                    for (int it = 0; it < NIT; ++it) {
                        const int64_t row = row_of(it);
                        ps[it] = (int)(ep.pos_rows ? (uint32_t)ep.pos_rows[row] : epi_shared_pos(ep));
                    }
#pragma unroll
                    for (int it = 0; it < NIT; ++it) {
                        const int64_t sj = (row_of(it) * ep.ldo + gcol) >> 2;
                        const bool act = ps[it] >= 0 && ps[it] < ep.n_ctx;
                        const int pc = act ? ps[it] : 0;
                        al[it] = ep.alpha[(size_t)h * ep.n_ctx + pc];
                        be[it] = ep.beta[(size_t)h * ep.n_ctx + pc];
                        s0[it] = ep.state_half ? load_state4(static_cast<const f16 *>(ep.state), sj)
                                               : load_state4(static_cast<const float *>(ep.state), sj);
                    }
#pragma unroll
                    for (int it = 0; it < NIT; ++it) {
                        if (!exists(it)) continue;
                        const int64_t row = row0 + it * RPI;
                        const int64_t sj = (row * ep.ldo + gcol) >> 2;
                        TAct *o = reinterpret_cast<TAct *>(ep.out) + row * ep.ldo + gcol;
                        if (!(ps[it] >= 0 && ps[it] < ep.n_ctx)) { store4(o, make_float4(0.f, 0.f, 0.f, 0.f)); continue; }
                        const float p = row_repeat ? al[it] : 1.0f, q = row_repeat ? 1.0f : al[it];
                        float4 n;
                        n.x = fmaf(l, s0[it].x, p * (float)(TAct)v[it].x);
                        n.y = fmaf(l, s0[it].y, p * (float)(TAct)v[it].y);
                        n.z = fmaf(l, s0[it].z, p * (float)(TAct)v[it].z);
                        n.w = fmaf(l, s0[it].w, p * (float)(TAct)v[it].w);
                        if (ep.state_half) {
                            f16 *sp = static_cast<f16 *>(ep.state);
                            n = make_float4(to_state(n.x, sp), to_state(n.y, sp), to_state(n.z, sp), to_state(n.w, sp));
                            store_state4(sp, sj, n);
                        } else {
                            store_state4(static_cast<float *>(ep.state), sj, n);
                        }
                        store4(o, make_float4(fmaf(q, n.x, be[it]), fmaf(q, n.y, be[it]), fmaf(q, n.z, be[it]),
                                              fmaf(q, n.w, be[it])));
                    }
                } else {
#pragma unroll
                    for (int it = 0; it < NIT; ++it) {
                        if (exists(it)) epi_store4<EPI, TAct>(ep, row0 + it * RPI, gcol, v[it]);
                    }
                }
            };
            if (cols_inside) {
                if (rows_inside) whole_columns(std::true_type{});
                else if (m0 + wm * WTM + i * 32 < M) whole_columns(std::false_type{});   // else: nothing of this slice exists
                return;
            }
#pragma unroll
            for (int it = 0; it < 32 / RPI; ++it) {
                const int lrow = it * RPI + s_row;
                const int64_t row = m0 + wm * WTM + i * 32 + lrow;
                const float4 v = *reinterpret_cast<const float4 *>(stage + lrow * STG + s_col);
                if (row < M) {
                    if (vec_ok && gcol + 3 < N) {
                        epi_store4<EPI, TAct>(ep, row, gcol, v);
                    } else {
                        if (gcol < N) epi_store1p<EPI, TAct>(ep, row, gcol, v.x);
                        if (gcol + 1 < N) epi_store1p<EPI, TAct>(ep, row, gcol + 1, v.y);
                        if (gcol + 2 < N) epi_store1p<EPI, TAct>(ep, row, gcol + 2, v.z);
                        if (gcol + 3 < N) epi_store1p<EPI, TAct>(ep, row, gcol + 3, v.w);
                    }
                }
            }
        }
    });
    if constexpr (EPI == EPI_ARGMAX) {
        __syncthreads();
        for (int lrow = tid; lrow < BM; lrow += NTHR) {
            const int row = m0 + lrow;
            if (row >= M) continue;
            float bv = red_val[lrow * WN];
            int bi = red_idx[lrow * WN];
#pragma unroll
            for (int w = 1; w < WN; ++w) {
                const float ov = red_val[lrow * WN + w];
                const int oi = red_idx[lrow * WN + w];
                if (arg_better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
            }
            ep.part_val[(int64_t)bn * M + row] = bv;
            ep.part_idx[(int64_t)bn * M + row] = bi;
        }
    }
}

// LNA (a handful of rows, M <= kLnaRows, one row tile, K <= 1024, no split): the A operand is not read
// from memory but made by the block itself, A = LayerNorm(ep.ln_x rows [+ slabs]) in the arithmetic of
// ln_kernel, written once as a panel [K / 64][32 rows][64] into LDS in the layout the tile loads would have
// produced; only W then travels through the ring.  Every column block normalises the few rows again,
// which is cheaper than the LayerNorm launch it replaces.  Rows >= M of the panel are never written: they
// feed accumulator rows that no epilogue stores.
constexpr int kLnaRows = 8;
template <int BM, int BN, int WM, int WN, int EPI, typename TAct, int NS = 2, bool LNA = false>
__global__ void __launch_bounds__(WM *WN * 64)
gemm_bf16_kernel(const bf16 *__restrict__ A, const bf16 *__restrict__ W, int M, int N, int K, GemmEpi ep)
{
    constexpr int BK = 64;
    constexpr int PANEL_ROWS = 32;                   // rows per k tile of the LNA panel
    static_assert(!LNA || (BM == 64 && WM == 2 && WN == 2), "the LNA panel is laid out for the 64x64 tile");
    static_assert(NS >= 2 && (NS & (NS - 1)) == 0, "the LDS ring holds a power-of-two number of k tiles");
    constexpr int NW = WM * WN, NTHR = NW * 64;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int A_IT = BM * BK / 8 / NTHR, B_IT = BN * BK / 8 / NTHR;
    constexpr int STG = WTN + 4;                     // stage row stride in floats: 16 B * odd
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of 32x32");
    static_assert((BM * BK / 8) % NTHR == 0 && (BN * BK / 8) % NTHR == 0, "tile/threads mismatch");
    static_assert(NW * 32 * STG * 4 + BM * WN * 8 <= NS * (BM + BN) * BK * 2, "epilogue stage exceeds the tile LDS");

    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int64_t probe_id = (int64_t)blockIdx.y * gridDim.x + blockIdx.x;
    const bool probe = ep.clk != nullptr && probe_id < ep.clk_blocks;
    unsigned long long clk_c0 = 0, clk_t0 = 0, clk_c1 = 0, clk_t1 = 0, clk_c2 = 0, clk_t2 = 0;
    if (probe) { clk_c0 = clock64(); clk_t0 = wall_clock64(); }
    bf16 *As = reinterpret_cast<bf16 *>(smem_raw);   // [NS][BM*BK]; LNA: [K / BK][PANEL_ROWS*BK]
    bf16 *Bs = As + (LNA ? (K / BK) * PANEL_ROWS * BK : NS * BM * BK);   // [NS][BN*BK]
    constexpr int A_TILE = LNA ? PANEL_ROWS * BK : BM * BK;            // elements between k tiles of A in LDS
    constexpr int A_LD = LNA ? 0 : A_IT;                               // tile loads of A per thread and k tile

    // Split K (gridDim.y > 1, EPI_F32 only): block row y of the grid contracts k in
    // [y * K / gridDim.y, (y + 1) * K / gridDim.y) and writes its own output slab
    // out + y * M * ldo; slab 0 carries the bias.  The consumer adds the slabs in
    // a fixed order, so the result does not depend on scheduling.
    const int ksplit = gridDim.y;
    const int kbeg = blockIdx.y * (K / ksplit);
    if (ksplit > 1) {
        ep.out = reinterpret_cast<float *>(ep.out) + (int64_t)blockIdx.y * M * ep.ldo;
        if (blockIdx.y) ep.bias = nullptr;
    }

    const int nbm = (M + BM - 1) / BM, nbn = (N + BN - 1) / BN;
    int bm, bn;
    tile_of_block(nbm, nbn, bm, bn);
    const int m0 = bm * BM, n0 = bn * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: LDS targets of the tile loads
    const int wm = wave / WN, wn = wave % WN;
    const int lr = lane & 31, lk = lane >> 5;

    // global -> LDS: buffer loads that write LDS directly (no VGPR staging, no
    // ds_write).  One wave instruction moves 8 rows x 128 bytes; the hardware puts
    // lane l's 16 bytes at M0-base + 16*l, so lane (r = l>>3, slot = l&7) fetches the
    // global chunk slot ^ swz(r) of its row, which lands the row swizzled in LDS.
    // The descriptors cover exactly this block's rows of A and W: rows past M or
    // N and k past K arrive as zeros (hardware range check).
    constexpr int ROWS_PER_IT = NTHR / 8;            // multiple of 16: the swizzle term repeats
    const int ld_r = tid >> 3, ld_c = tid & 7;
    const __amdgpu_buffer_rsrc_t rs_a = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16 *>(A + (size_t)m0 * K), 0, min(BM, M - m0) * K * 2, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16 *>(W + (size_t)n0 * K), 0, min(BN, N - n0) * K * 2, 0x00020000);
    const int ld_voff = (ld_r * K + ((ld_c ^ swz_of_row(ld_r)) << 3)) * 2;       // bytes
    typedef __attribute__((address_space(3))) void lds_void;
    // tile load number i of a k tile: the first A_LD fetch A, the rest W
#define SRM_DMA_ONE(i, k0, buf)                                                                  \
    if ((i) < A_LD)                                                                              \
        __builtin_amdgcn_raw_ptr_buffer_load_lds(                                                \
            rs_a, (lds_void *)(As + (buf) * BM * BK + ((i) * ROWS_PER_IT + wave * 8) * BK), 16,  \
            ld_voff, ((i) * ROWS_PER_IT * K + kbeg + (k0)) * 2, 0, 0);                           \
    else                                                                                         \
        __builtin_amdgcn_raw_ptr_buffer_load_lds(                                                \
            rs_w, (lds_void *)(Bs + (buf) * BN * BK + (((i) - A_LD) * ROWS_PER_IT + wave * 8) * BK), 16, \
            ld_voff, (((i) - A_LD) * ROWS_PER_IT * K + kbeg + (k0)) * 2, 0, 0);
#define SRM_DMA_TILE(k0, buf)                                                                    \
    _Pragma("unroll") for (int i = 0; i < A_LD + B_IT; ++i) { SRM_DMA_ONE(i, k0, buf) }
    // s_waitcnt immediate: vmcnt = n, expcnt and lgkmcnt unconstrained
#define SRM_WAIT_VM(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))

    // The accumulators start at the bias of their column (bias + sum: the epilogues add nothing).  Register
    // quad g of tile (i, j) holds columns j*32 + 8g + 4lk .. +3 of the wave tile (see gemm_epilogue).  The
    // bias is requested here, in front of the first tile loads, and moved into the accumulators once the
    // first tile has landed (loads return in order): its latency hides under the first tile's.
    float4 bq[TN][4];
    if (ep.bias && (N & 3) == 0 && n0 + BN <= N) {       // block-uniform: all of the tile's columns exist
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) bq[j][g] = load4(ep.bias + n0 + wn * WTN + j * 32 + 8 * g + 4 * lk);
    } else {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int col = n0 + wn * WTN + j * 32 + 8 * g + 4 * lk;
                bq[j][g] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (ep.bias) {
                    bq[j][g].x = col < N ? ep.bias[col] : 0.f;
                    bq[j][g].y = col + 1 < N ? ep.bias[col + 1] : 0.f;
                    bq[j][g].z = col + 2 < N ? ep.bias[col + 2] : 0.f;
                    bq[j][g].w = col + 3 < N ? ep.bias[col + 3] : 0.f;
                }
            }
    }
    f32x16_t acc[TM][TN];

    const int sw = swz_of_row(lr);                   // wave-tile rows are multiples of 32 apart
    const int a_row_off = (wm * WTM + lr) * BK;
    const int b_row_off = (wn * WTN + lr) * BK;
    bf16x8_t fa[4][TM], fb[4][TN];                   // one operand set per k-substep
    // abuf: the k tile's place in the A area (its ring slot; LNA: the k tile's own number), bbuf: its ring slot
#define SRM_READ_FRAGS(abuf, bbuf, kk, set)                                                      \
    {                                                                                            \
        const int ch_ = ((((kk) * 2 + lk) ^ sw) << 3);                                           \
        const bf16 *as_ = As + (abuf) * A_TILE + a_row_off + ch_;                                \
        const bf16 *bs_ = Bs + (bbuf) * BN * BK + b_row_off + ch_;                               \
        _Pragma("unroll") for (int i = 0; i < TM; ++i)                                           \
            fa[set][i] = *reinterpret_cast<const bf16x8_t *>(as_ + i * 32 * BK);                 \
        _Pragma("unroll") for (int j = 0; j < TN; ++j)                                           \
            fb[set][j] = *reinterpret_cast<const bf16x8_t *>(bs_ + j * 32 * BK);                 \
    }

#define SRM_MFMA_STEP(set)                                                                       \
    _Pragma("unroll") for (int i = 0; i < TM; ++i)                                               \
        _Pragma("unroll") for (int j = 0; j < TN; ++j) /* transposed: MFMA rows run over N */    \
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[set][j], fa[set][i], acc[i][j], 0, 0, 0);
    // Issue order inside the k-substeps that only read operands (0, 1 and 3): one LDS read behind
    // each MFMA, so that the reads issue while the matrix pipe works instead of in a burst in front
    // of it.  (Substep 2, which also issues the tile loads, is written out in issue order below.)
#define SRM_INTERLEAVE()                                                                         \
    _Pragma("unroll") for (int q = 0; q < TM * TN; ++q) {                                        \
        constexpr int S_ = TM * TN;                                                              \
        constexpr int R_ = (TM + TN + S_ - 1) / S_;                                              \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                       \
        if (q * R_ < TM + TN) __builtin_amdgcn_sched_group_barrier(0x100, R_, 0);                \
    }                                                                                            \
    __builtin_amdgcn_sched_barrier(0);

    // Software pipeline over K tiles (four k-substeps of 16 each), a ring of NS LDS
    // buffers (NS = 2 below; with few blocks on the chip a k loop is bound by the
    // latency of its tile loads, and a deeper ring keeps NS - 1 tiles in flight),
    // MFMA operands read two substeps ahead (four register sets):
    //   substep 0: read operands of substep 2                  | MFMAs of substep 0
    //   substep 1: read operands of substep 3                  | MFMAs of substep 1
    //              wait for tile kt+1's loads, barrier: buffer `cur` is now free
    //   substep 2: read substep-0 operands of tile kt+1,       | MFMAs of substep 2
    //              start tile kt+2's loads into `cur`
    //   substep 3: read substep-1 operands of tile kt+1        | MFMAs of substep 3
    // A tile's loads have a full tile period to land and every operand read has
    // two substeps, which absorbs the queueing of reads behind the tile writes in
    // the LDS pipe.  Loads for tiles past the end are issued like any other
    // (range check: zeros nobody reads), which keeps the loop branch-free.
    const int KT = K / ksplit / BK;
    static_assert((NS - 1) * (A_IT + B_IT) <= 63, "more tile loads in flight than the counter holds");
    constexpr int LD_IT = A_LD + B_IT;
    if constexpr (LNA) {
        // Two rows per wavefront.  Their values (and the first four slabs) are requested before the ring's tile
        // loads, so that they return first and the normalisation runs while the W tiles travel.
        constexpr int RW = kLnaRows / NW, VPL = 4;
        const int d = K;
        float4 v[RW][VPL], t[RW][VPL][4], pg[VPL], pb[VPL];
        const int ns0 = ep.ln_part ? ep.ln_nsplit : 0;
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const int c = (i * 64 + lane) * 4;
            pg[i] = pb[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (c < d) { pg[i] = load4(ep.ln_g + c); pb[i] = load4(ep.ln_b + c); }
#pragma unroll
            for (int j = 0; j < RW; ++j) {
                const int r = wave * RW + j;
                v[j][i] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (r < M && c < d) {
                    v[j][i] = load4(ep.ln_x + (int64_t)r * d + c);
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (ns0 > 0) t[j][i][q] = load4(ep.ln_part + (int64_t)min(q, ns0 - 1) * ep.ln_stride + (int64_t)r * d + c);
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int stage = 0; stage < NS; ++stage) { SRM_DMA_TILE(stage * BK, stage) }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < RW; ++j) {
            const int r = wave * RW + j;
            if (r >= M) continue;                    // wave-uniform
            float sum = 0.0f;
#pragma unroll
            for (int i = 0; i < VPL; ++i) {
                const int c = (i * 64 + lane) * 4;
                if (c < d) {
                    // the slabs, in slab order (the first four were requested above)
                    for (int s0 = 0; s0 < ns0; s0 += 4) {
                        if (s0 > 0) {
#pragma unroll
                            for (int q = 0; q < 4; ++q)
                                t[j][i][q] = load4(ep.ln_part + (int64_t)min(s0 + q, ns0 - 1) * ep.ln_stride + (int64_t)r * d + c);
                        }
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            if (s0 + q < ns0) {
                                v[j][i].x += t[j][i][q].x; v[j][i].y += t[j][i][q].y;
                                v[j][i].z += t[j][i][q].z; v[j][i].w += t[j][i][q].w;
                            }
                    }
                    sum += (v[j][i].x + v[j][i].y) + (v[j][i].z + v[j][i].w);
                }
            }
            const float mean = wave_sum(sum) / (float)d;
            float sq = 0.0f;
#pragma unroll
            for (int i = 0; i < VPL; ++i) {
                const int c = (i * 64 + lane) * 4;
                if (c < d) {
                    const float a = v[j][i].x - mean, bb = v[j][i].y - mean, cc = v[j][i].z - mean, dd = v[j][i].w - mean;
                    sq += (a * a + bb * bb) + (cc * cc + dd * dd);
                }
            }
            const float var = wave_sum(sq) / (float)d;
            const float rstd = 1.0f / sqrtf(var + ep.ln_eps);
#pragma unroll
            for (int i = 0; i < VPL; ++i) {
                const int c = (i * 64 + lane) * 4;
                if (c < d) {
                    float4 o;
                    o.x = (v[j][i].x - mean) * rstd * pg[i].x + pb[i].x;
                    o.y = (v[j][i].y - mean) * rstd * pg[i].y + pb[i].y;
                    o.z = (v[j][i].z - mean) * rstd * pg[i].z + pb[i].z;
                    o.w = (v[j][i].w - mean) * rstd * pg[i].w + pb[i].w;
                    store4(As + (c >> 6) * A_TILE + r * BK + ((((c & 63) >> 3) ^ swz_of_row(r)) << 3) + (c & 7), o);
                }
            }
        }
    } else {
#pragma unroll
        for (int stage = 0; stage < NS; ++stage) { SRM_DMA_TILE(stage * BK, stage) }   // (the macro's own loops use `i`)
    }
    SRM_WAIT_VM((NS - 1) * LD_IT);
    __syncthreads();
    SRM_READ_FRAGS(0, 0, 0, 0)
    SRM_READ_FRAGS(0, 0, 1, 1)
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                acc[i][j][4 * g] = bq[j][g].x; acc[i][j][4 * g + 1] = bq[j][g].y;
                acc[i][j][4 * g + 2] = bq[j][g].z; acc[i][j][4 * g + 3] = bq[j][g].w;
            }
    __builtin_amdgcn_sched_barrier(0);
    if (probe) { clk_c1 = clock64(); clk_t1 = wall_clock64(); }

    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & (NS - 1), nxt = (kt + 1) & (NS - 1);
        const int acur = LNA ? kt : cur, anxt = LNA ? kt + 1 : nxt;
        SRM_READ_FRAGS(acur, cur, 2, 2)
        SRM_MFMA_STEP(0)
        SRM_INTERLEAVE()
        SRM_READ_FRAGS(acur, cur, 3, 3)
        SRM_MFMA_STEP(1)
        SRM_INTERLEAVE()
        SRM_WAIT_VM((NS - 2) * LD_IT);                   // tile kt+1 has landed; later tiles may still be in flight
        __syncthreads();
        // substep 2 in issue order, pinned: behind each MFMA its share of the operand reads of the next
        // tile's substep 0 and of the tile loads (left to the scheduler, the reads and loads all went in
        // front of the second MFMA in one burst)
        {
            const int ch_ = ((lk ^ sw) << 3);
            const bf16 *as_ = As + anxt * A_TILE + a_row_off + ch_;
            const bf16 *bs_ = Bs + nxt * BN * BK + b_row_off + ch_;
            constexpr int S_ = TM * TN;
            constexpr int RPM = (TM + TN + S_ - 1) / S_, LPM = (LD_IT + S_ - 1) / S_;
#pragma unroll
            for (int q = 0; q < S_; ++q) {
                acc[q / TN][q % TN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[2][q % TN], fa[2][q / TN],
                                                                              acc[q / TN][q % TN], 0, 0, 0);
#pragma unroll
                for (int r = q * RPM; r < (q + 1) * RPM && r < TM + TN; ++r) {
                    if (r < TM) fa[0][r] = *reinterpret_cast<const bf16x8_t *>(as_ + r * 32 * BK);
                    else fb[0][r - TM] = *reinterpret_cast<const bf16x8_t *>(bs_ + (r - TM) * 32 * BK);
                }
#pragma unroll
                for (int l = q * LPM; l < (q + 1) * LPM && l < LD_IT; ++l) { SRM_DMA_ONE(l, (kt + NS) * BK, cur) }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        SRM_READ_FRAGS(anxt, nxt, 1, 1)
        SRM_MFMA_STEP(3)
        SRM_INTERLEAVE()
    }
    SRM_WAIT_VM(0);
    __syncthreads();                                  // LDS is reused by the epilogue
    if (probe) { clk_c2 = clock64(); clk_t2 = wall_clock64(); }
#undef SRM_MFMA_STEP
#undef SRM_INTERLEAVE
#undef SRM_DMA_TILE
#undef SRM_DMA_ONE
#undef SRM_WAIT_VM
#undef SRM_READ_FRAGS

    gemm_epilogue<BM, BN, WM, WN, EPI, TAct>(acc, smem_raw, ep, M, N, m0, n0, bn);
    if (probe) {
        __builtin_amdgcn_s_waitcnt(0);                // this wave's stores have completed
        if (tid == 0) {
            unsigned long long *p = ep.clk + 8 * probe_id;
            p[0] = clk_t0; p[1] = clk_t1; p[2] = clk_t2; p[3] = wall_clock64(); p[4] = clk_c1; p[5] = clk_c2;
            p[6] = (unsigned long long)__builtin_amdgcn_s_getreg((31 << 11) | 4) |        // HW_ID
                   ((unsigned long long)__builtin_amdgcn_s_getreg((3 << 11) | 20) << 32);  // XCC_ID
            p[7] = clk_c0;
        }
    }
}

// ------------------------------------------------------------------ fp32 FMA
// 64x64x16 tiles, 256 threads, 4x4 outputs per thread, k ascending.
template <int EPI>
__global__ void __launch_bounds__(256)
gemm_f32_kernel(const float *__restrict__ A, const float *__restrict__ W, int M, int N, int K, GemmEpi ep)
{
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ float As[BK][BM + 4];
    __shared__ float Bs[BK][BN + 4];
    const int nbn = (N + BN - 1) / BN;
    const int bm = blockIdx.x / nbn, bn = blockIdx.x % nbn;
    const int m0 = bm * BM, n0 = bn * BN;
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;

    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.0f;

    for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int e = tid + s * 256, r = e >> 4, k = e & 15;
            const bool kin = k0 + k < K;
            As[k][r] = (kin && m0 + r < M) ? A[(size_t)(m0 + r) * K + k0 + k] : 0.0f;
            Bs[k][r] = (kin && n0 + r < N) ? W[(size_t)(n0 + r) * K + k0 + k] : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < BK; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }

#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int lrow = ty * 4 + i, row = m0 + lrow;
        float bv = -INFINITY;
        int bi = 0x7fffffff;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int col = n0 + tx * 4 + j;
            if (col >= N) continue;
            const float v = acc[i][j] + (ep.bias ? ep.bias[col] : 0.0f);
            if (row < M) epi_store<EPI, float>(ep, row, col, v);
            if constexpr (EPI == EPI_ARGMAX) {
                const float vs = ep.temp > 0.0f
                                     ? v + ep.temp * srm_gumbel(srm_rowkey(ep.seed, epi_pos(ep, row, M), (uint32_t)row + ep.row_base), (uint32_t)col)
                                     : v;
                if (arg_better(vs, col, bv, bi)) { bv = vs; bi = col; }
            }
        }
        if constexpr (EPI == EPI_ARGMAX) {
            // the 16 threads of a row are 16 consecutive lanes
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) {
                const float ov = __shfl_xor(bv, off, kWave);
                const int oi = __shfl_xor(bi, off, kWave);
                if (arg_better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
            }
            if (tx == 0 && row < M) {
                ep.part_val[(int64_t)bn * M + row] = bv;
                ep.part_idx[(int64_t)bn * M + row] = bi;
            }
        }
    }
}

// ------------------------------------------------------------------ few rows: streaming GEMV
// out = epilogue(A W^T + bias) for at most a few dozen rows (fp32 models; with bf16 weights the 64x64
// MFMA tile is faster even for one row: measured 2.7 us + 3.4 us per 1024 k against 5.5 + 6.9 for this
// kernel reading bf16, whose eight rows of activations per weight vector make it LDS-bound).  The
// product is bound by streaming W once, so the grid is made of
// many small column slices (16 * CPG columns per block) and the loads are coalesced: 16 lanes
// share CPG columns (4 such groups per wavefront), lane l16 reading every 16th 16-byte vector of
// a weight row; MB rows of A sit in LDS as fp32 and are read by every column; after the 16-lane
// reduction lane l16 == b owns row b of the group's columns.  Weight vectors are requested one
// batch ahead, the first batch before A is staged.  Rows are processed MB at a time (W is streamed
// again per group of MB rows).  Split K as in gemm_bf16_kernel (gridDim.y slabs, EPI_F32 only).
// Dynamic LDS: MB * (K / gridDim.y) floats.
template <typename TW> struct GemvVec;
template <> struct GemvVec<float> {
    static constexpr int VW = 4;
    __device__ static void unpack(const u32x4_t &r, float (&f)[4])
    {
        const f32x4_t t = __builtin_bit_cast(f32x4_t, r);
        f[0] = t[0]; f[1] = t[1]; f[2] = t[2]; f[3] = t[3];
    }
};
template <typename TW, typename TAct, int EPI, int MB, int CPG>
__global__ void __launch_bounds__(256)
gemv_rows_kernel(const TAct *__restrict__ A, const TW *__restrict__ W, int M, int N, int K, GemmEpi ep)
{
    extern __shared__ __align__(16) float gr_sm[];      // [MB][Kp]
    __shared__ float red_v[16][MB];
    __shared__ int red_i[16][MB];
    constexpr int VW = GemvVec<TW>::VW;
    constexpr int JB = 8 / CPG;                          // 16-byte vectors per lane, column and batch
    static_assert(MB <= 16 && CPG * JB == 8, "one owner lane per row; eight vectors per lane and batch");
    const int Kp = K / (int)gridDim.y, kb = blockIdx.y * Kp;
    if (gridDim.y > 1) {
        ep.out = reinterpret_cast<float *>(ep.out) + (int64_t)blockIdx.y * M * ep.ldo;
        if (blockIdx.y) ep.bias = nullptr;
    }
    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15;
    const int grp = (tid >> 6) * 4 + (lane >> 4);        // 0..15
    const int KV = Kp / VW;                              // 16-byte vectors per row slice
    const int nbatch = (KV + 16 * JB - 1) / (16 * JB);
    int n[CPG];
    const u32x4_t *wr[CPG];
#pragma unroll
    for (int c = 0; c < CPG; ++c) {
        n[c] = (blockIdx.x * 16 + grp) * CPG + c;
        wr[c] = reinterpret_cast<const u32x4_t *>(W + (size_t)min(n[c], N - 1) * K + kb);
    }
    auto load_batch = [&](u32x4_t (&w)[CPG][JB], int jb) {
#pragma unroll
        for (int c = 0; c < CPG; ++c)
#pragma unroll
            for (int j = 0; j < JB; ++j) {
                const int kv = (jb * JB + j) * 16 + l16;
                const u32x4_t v = wr[c][min(kv, KV - 1)];          // clamped address, zeroed by a mask: no branches between loads
                const uint32_t keep = (n[c] < N && kv < KV) ? 0xffffffffu : 0u;
                w[c][j] = v & keep;
            }
    };
    u32x4_t w[CPG][JB];
    load_batch(w, 0);
    float bias[CPG];
#pragma unroll
    for (int c = 0; c < CPG; ++c) bias[c] = (ep.bias && n[c] < N) ? ep.bias[n[c]] : 0.0f;

    for (int mg = 0; mg < M; mg += MB) {
        __syncthreads();                                 // the previous group's products are done with the stage
        // stage the group's rows as fp32: a thread takes the same four k of every row, all MB loads in flight
        const int rows_here = min(MB, M - mg);
        for (int k = tid * 4; k < Kp; k += 256 * 4) {
            float4 v[MB];
#pragma unroll
            for (int m = 0; m < MB; ++m) {
                v[m] = load4(A + (size_t)(mg + min(m, rows_here - 1)) * K + kb + k);
                if (m >= rows_here) v[m] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int m = 0; m < MB; ++m) *reinterpret_cast<float4 *>(gr_sm + m * Kp + k) = v[m];
        }
        __syncthreads();
        if (mg > 0) load_batch(w, 0);
        float acc[CPG][MB];
#pragma unroll
        for (int c = 0; c < CPG; ++c)
#pragma unroll
            for (int b = 0; b < MB; ++b) acc[c][b] = 0.0f;
#pragma unroll 1
        for (int jb = 0; jb < nbatch; ++jb) {
            u32x4_t wn[CPG][JB];
            if (jb + 1 < nbatch) load_batch(wn, jb + 1);
#pragma unroll
            for (int j = 0; j < JB; ++j) {
                const int kv = min((jb * JB + j) * 16 + l16, KV - 1);
                float wf[CPG][VW];
#pragma unroll
                for (int c = 0; c < CPG; ++c) GemvVec<TW>::unpack(w[c][j], wf[c]);
                // all rows' activations for this k position first (one batch of LDS reads), then the products
                float4 av[MB][VW / 4];
#pragma unroll
                for (int b = 0; b < MB; ++b)
#pragma unroll
                    for (int q = 0; q < VW / 4; ++q)
                        av[b][q] = *reinterpret_cast<const float4 *>(gr_sm + b * Kp + kv * VW + q * 4);
#pragma unroll
                for (int b = 0; b < MB; ++b)
#pragma unroll
                    for (int q = 0; q < VW / 4; ++q)
#pragma unroll
                        for (int c = 0; c < CPG; ++c) {
                            acc[c][b] = fmaf(wf[c][q * 4], av[b][q].x, acc[c][b]);
                            acc[c][b] = fmaf(wf[c][q * 4 + 1], av[b][q].y, acc[c][b]);
                            acc[c][b] = fmaf(wf[c][q * 4 + 2], av[b][q].z, acc[c][b]);
                            acc[c][b] = fmaf(wf[c][q * 4 + 3], av[b][q].w, acc[c][b]);
                        }
            }
#pragma unroll
            for (int c = 0; c < CPG; ++c)
#pragma unroll
                for (int j = 0; j < JB; ++j) w[c][j] = wn[c][j];
        }
        float bv = -INFINITY;
        int bi = 0x7fffffff;
#pragma unroll
        for (int c = 0; c < CPG; ++c) {
            float mine = 0.0f;
#pragma unroll
            for (int b = 0; b < MB; ++b) {
                const float v = row16_sum(acc[c][b]);
                if (l16 == b) mine = v;
            }
            const int row = mg + l16;
            if (l16 < MB && row < M && n[c] < N) {
                float v = mine + bias[c];
                epi_store1p<EPI, TAct>(ep, row, n[c], v);
                if constexpr (EPI == EPI_ARGMAX) {
                    if (ep.temp > 0.0f)
                        v += ep.temp * srm_gumbel(srm_rowkey(ep.seed, epi_pos(ep, row, M), (uint32_t)row + ep.row_base), (uint32_t)n[c]);
                    if (arg_better(v, n[c], bv, bi)) { bv = v; bi = n[c]; }
                }
            }
        }
        if constexpr (EPI == EPI_ARGMAX) {
            // best (score, index) of this block's columns per row: 16 lane groups -> one partial
            if (l16 < MB) { red_v[grp][l16] = bv; red_i[grp][l16] = bi; }
            __syncthreads();
            if (tid < MB && mg + tid < M) {
                float v = red_v[0][tid];
                int i = red_i[0][tid];
                for (int g = 1; g < 16; ++g)
                    if (arg_better(red_v[g][tid], red_i[g][tid], v, i)) { v = red_v[g][tid]; i = red_i[g][tid]; }
                ep.part_val[(int64_t)blockIdx.x * M + mg + tid] = v;
                ep.part_idx[(int64_t)blockIdx.x * M + mg + tid] = i;
            }
        }
    }
}

// Optional behaviour of argmax_finalize_kernel for ragged batches.
struct FinalizeRagged {
    const int32_t *slot;      // destination index of sequence row0 + row (replaces the (row0 + row) * rep rule)
    int64_t nslots;           // destinations outside [0, nslots) are skipped
    int32_t *pos_rows;        // decode: position of each row; a row outside [0, n_ctx) is inactive -> token -1
    int32_t advance;          // decode: add 1 to the position of every active row
    int32_t n_ctx;
    const int32_t *offsets;   // prefill: sequence boundaries, offsets[row0 + row + 1] - offsets[row0 + row] = length
    int32_t *pos_set;         // prefill: pos_set[destination] = length of the sequence
    int32_t *zero_counter;    // set to 0 (the row list of the nucleus pass that follows)
    int32_t eos_plus1;        // decode with advance: eos token + 1 (0: none); a row that emits it goes idle (position -1)
};

// Reduce the per-tile partials [nparts][rows] of each row to one token; writes `rep`
// consecutive copies starting at out[(row0 + row) * rep].  One work-group per 16
// rows: thread (r = tid & 15, q = tid >> 4) scans parts q, q + 16, ... of row r
// (16 consecutive lanes read 16 consecutive rows; the loads of eight parts are in
// flight together), the sixteen scans of a row meet in LDS.
// A row without any ordered value (all NaN) yields token 0, so that the id is
// always a valid embedding row.  If store is not null the token also goes to
// store[step * store_stride + (row0 + row) * rep + r] with step = *step_dev.
constexpr int kFinalRows = 16;
__global__ void __launch_bounds__(256)
argmax_finalize_kernel(const float *__restrict__ part_val, const int32_t *__restrict__ part_idx,
                       int64_t rows, int nparts, int32_t *__restrict__ out, int64_t row0, int rep,
                       int vocab, int32_t *__restrict__ store, const int *__restrict__ step_dev,
                       int64_t store_stride, FinalizeRagged rg)
{
    constexpr int NQ = 256 / kFinalRows, U = 8;
    __shared__ float sv[NQ][kFinalRows];
    __shared__ int si[NQ][kFinalRows];
    const int r = threadIdx.x % kFinalRows, q = threadIdx.x / kFinalRows;
    const int64_t blk0 = (int64_t)blockIdx.x * kFinalRows;
    const int64_t row = blk0 + r;
    if (rg.zero_counter && blockIdx.x == 0 && threadIdx.x == 0) *rg.zero_counter = 0;
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    if (row < rows)
        for (int p0 = q; p0 < nparts; p0 += NQ * U) {
            float v[U];
            int i[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int p = min(p0 + u * NQ, nparts - 1);          // clamped address, masked below
                v[u] = part_val[(int64_t)p * rows + row];
                i[u] = part_idx[(int64_t)p * rows + row];
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (p0 + u * NQ < nparts && arg_better(v[u], i[u], bv, bi)) { bv = v[u]; bi = i[u]; }
        }
    sv[q][r] = bv;
    si[q][r] = bi;
    __syncthreads();
    if (q == 0 && row < rows) {
        for (int k = 1; k < NQ; ++k)
            if (arg_better(sv[k][r], si[k][r], bv, bi)) { bv = sv[k][r]; bi = si[k][r]; }
        if (bi < 0 || bi >= vocab) bi = 0;
        if (rg.pos_rows) {
            const int p = rg.pos_rows[row0 + row];
            const bool active = p >= 0 && p < rg.n_ctx;
            if (!active) bi = -1;
            else if (rg.advance) rg.pos_rows[row0 + row] = (rg.eos_plus1 && bi == rg.eos_plus1 - 1) ? -1 : p + 1;
        }
        if (rg.slot) {
            const int64_t dst = rg.slot[row0 + row];
            if (dst >= 0 && dst < rg.nslots) {
                out[dst] = bi;
                if (rg.pos_set) rg.pos_set[dst] = rg.offsets[row0 + row + 1] - rg.offsets[row0 + row];
            }
        }
        si[0][r] = bi;
    }
    if (rg.slot) return;
    __syncthreads();
    // the rep copies of the block's tokens, consecutive threads writing consecutive words
    const int64_t nrow = min((int64_t)kFinalRows, rows - blk0);
    int32_t *dst2 = store ? store + (int64_t)(*step_dev) * store_stride : nullptr;
    for (int64_t e = threadIdx.x; e < nrow * rep; e += 256) {
        const int rl = (int)(e / rep);
        const int64_t o = (row0 + blk0) * rep + e;
        out[o] = si[0][rl];
        if (rg.pos_set) rg.pos_set[o] = rg.offsets[row0 + blk0 + rl + 1] - rg.offsets[row0 + blk0 + rl];
        if (dst2) dst2[o] = si[0][rl];
    }
}
