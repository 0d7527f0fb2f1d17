// GEMMs of the SRM block: out = epilogue(A W^T + bias), A [M][K], W [N][K]
// (both K-contiguous), for the head projections (Eq. 10), the channel-mixing
// MLP and the LM head.
//
//   gemm_bf16_kernel: bf16 operands on the gfx950 matrix cores
//     (v_mfma_f32_32x32x16_bf16, fp32 accumulate), tiles staged through LDS
//     with a 16-byte XOR swizzle, two LDS stages, global loads of tile k+1 in
//     flight while tile k is multiplied.
//   gemm_f32_kernel: plain fp32 FMA tiles for the fp32 configurations.
//
// Epilogues are fused: bias, exact GELU, residual add into the fp32 stream,
// and for the LM head a per-tile (max, index) partial so that logits need not
// be written at all.
#pragma once
#include "common.hpp"

enum { EPI_STORE = 0, EPI_GELU = 1, EPI_RESID = 2, EPI_ARGMAX = 3, EPI_F32 = 4 };

struct GemmEpi {
    const float *bias;   // [N] or nullptr
    void *out;           // EPI_STORE/GELU: TAct [M][ldo]; EPI_RESID: float [M][ldo] (+=);
                         // EPI_F32: float [M][ldo]; EPI_ARGMAX: float [M][ldo] or nullptr
    int64_t ldo;
    float *part_val;     // EPI_ARGMAX: [M][nparts]
    int32_t *part_idx;   // EPI_ARGMAX: [M][nparts]
    int32_t nparts;      // number of column tiles
};

// Block -> tile mapping.  Workgroups are dealt round-robin to the 8 XCDs, each
// with its own L2: give every XCD one contiguous run of tiles, and inside a run
// walk groups of GM row-tiles column by column so the A rows of a group and the
// W tile being shared stay L2-resident.
__device__ __forceinline__ void tile_of_block(int nbm, int nbn, int &bm, int &bn)
{
    constexpr int GM = 8;
    int pid = blockIdx.x;
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

template <int EPI, typename TAct>
__device__ __forceinline__ void epi_store(const GemmEpi &ep, int64_t row, int col, float v)
{
    if constexpr (EPI == EPI_STORE) {
        store1(reinterpret_cast<TAct *>(ep.out) + row * ep.ldo + col, v);
    } else if constexpr (EPI == EPI_GELU) {
        store1(reinterpret_cast<TAct *>(ep.out) + row * ep.ldo + col, gelu_erf(v));
    } else if constexpr (EPI == EPI_RESID) {
        float *p = reinterpret_cast<float *>(ep.out) + row * ep.ldo + col;
        *p += v;
    } else if constexpr (EPI == EPI_F32) {
        reinterpret_cast<float *>(ep.out)[row * ep.ldo + col] = v;
    } else {
        if (ep.out) reinterpret_cast<float *>(ep.out)[row * ep.ldo + col] = v;
    }
}

// ------------------------------------------------------------------ bf16 MFMA
template <int BM, int BN, int WM, int WN, int EPI, typename TAct>
__global__ void __launch_bounds__(WM *WN * 64)
gemm_bf16_kernel(const bf16 *__restrict__ A, const bf16 *__restrict__ W, int M, int N, int K, GemmEpi ep)
{
    constexpr int BK = 64;
    constexpr int NTHR = WM * WN * 64;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int A_IT = BM * BK / 8 / NTHR, B_IT = BN * BK / 8 / NTHR;
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of 32x32");
    static_assert((BM * BK / 8) % NTHR == 0 && (BN * BK / 8) % NTHR == 0, "tile/threads mismatch");

    extern __shared__ __align__(16) unsigned char smem_raw[];
    bf16 *As = reinterpret_cast<bf16 *>(smem_raw);   // [2][BM*BK]
    bf16 *Bs = As + 2 * BM * BK;                     // [2][BN*BK]

    const int nbm = (M + BM - 1) / BM, nbn = (N + BN - 1) / BN;
    int bm, bn;
    tile_of_block(nbm, nbn, bm, bn);
    const int m0 = bm * BM, n0 = bn * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int lr = lane & 31, lk = lane >> 5;

    // global -> LDS assignment: 16-byte chunks, 8 consecutive threads cover one
    // 128-byte row segment.  Rows past the edge are clamped (never stored).
    const bf16 *a_src[A_IT];
    const bf16 *b_src[B_IT];
    int a_dst[A_IT], b_dst[B_IT];
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
        const int q = i * NTHR + tid, r = q >> 3, c = q & 7;
        const int gr = min(m0 + r, M - 1);
        a_src[i] = A + (size_t)gr * K + c * 8;
        a_dst[i] = r * BK + ((c ^ ((r >> 1) & 7)) << 3);
    }
#pragma unroll
    for (int i = 0; i < B_IT; ++i) {
        const int q = i * NTHR + tid, r = q >> 3, c = q & 7;
        const int gr = min(n0 + r, N - 1);
        b_src[i] = W + (size_t)gr * K + c * 8;
        b_dst[i] = r * BK + ((c ^ ((r >> 1) & 7)) << 3);
    }

    u32x4_t ra[A_IT], rb[B_IT];
#define SRM_LOAD_GLOBAL(k0)                                                                      \
    _Pragma("unroll") for (int i = 0; i < A_IT; ++i)                                             \
        ra[i] = *reinterpret_cast<const u32x4_t *>(a_src[i] + (k0));                             \
    _Pragma("unroll") for (int i = 0; i < B_IT; ++i)                                             \
        rb[i] = *reinterpret_cast<const u32x4_t *>(b_src[i] + (k0));
#define SRM_STORE_LDS(buf)                                                                       \
    _Pragma("unroll") for (int i = 0; i < A_IT; ++i)                                             \
        *reinterpret_cast<u32x4_t *>(As + (buf) * BM * BK + a_dst[i]) = ra[i];                   \
    _Pragma("unroll") for (int i = 0; i < B_IT; ++i)                                             \
        *reinterpret_cast<u32x4_t *>(Bs + (buf) * BN * BK + b_dst[i]) = rb[i];

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // operand fetch offsets (row within the wave tile is lr; swizzle uses row>>1)
    const int sw = (lr >> 1) & 7;
    const int a_row_off = (wm * WTM + lr) * BK;
    const int b_row_off = (wn * WTN + lr) * BK;

    const int KT = K / BK;
    SRM_LOAD_GLOBAL(0)
    SRM_STORE_LDS(0)
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < KT) { SRM_LOAD_GLOBAL((kt + 1) * BK) }
        const bf16 *as = As + cur * BM * BK + a_row_off;
        const bf16 *bs = Bs + cur * BN * BK + b_row_off;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            const int ch = ((kk * 2 + lk) ^ sw) << 3;
            bf16x8_t af[TM], bf[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) af[i] = *reinterpret_cast<const bf16x8_t *>(as + i * 32 * BK + ch);
#pragma unroll
            for (int j = 0; j < TN; ++j) bf[j] = *reinterpret_cast<const bf16x8_t *>(bs + j * 32 * BK + ch);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) { SRM_STORE_LDS(cur ^ 1) }
        __syncthreads();
    }

#undef SRM_LOAD_GLOBAL
#undef SRM_STORE_LDS

    // ---- epilogue.  Accumulator register r of lane (lk, lr) is element
    // (row 8*(r/4) + 4*lk + r%4, column lr) of its 32x32 tile.
    float bias_v[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = n0 + wn * WTN + j * 32 + lr;
        bias_v[j] = (ep.bias && col < N) ? ep.bias[col] : 0.0f;
    }

    if constexpr (EPI != EPI_ARGMAX) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm * WTM + i * 32 + 8 * (r >> 2) + 4 * lk + (r & 3);
                if (row >= M) continue;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int col = n0 + wn * WTN + j * 32 + lr;
                    if (col < N) epi_store<EPI, TAct>(ep, row, col, acc[i][j][r] + bias_v[j]);
                }
            }
    } else {
        // LM head: optional logits store plus per-row (max, index) over this
        // block's BN columns.  In-lane over the TN column tiles, across the 32
        // lanes that share a row, then across the WN waves through LDS.
        float *red_val = reinterpret_cast<float *>(smem_raw);               // [BM][WN]
        int *red_idx = reinterpret_cast<int *>(smem_raw + BM * WN * 4);     // [BM][WN]
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int lrow = wm * WTM + i * 32 + 8 * (r >> 2) + 4 * lk + (r & 3);
                const int row = m0 + lrow;
                float bv = -INFINITY;
                int bi = 0x7fffffff;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int col = n0 + wn * WTN + j * 32 + lr;
                    const float v = acc[i][j][r] + bias_v[j];
                    if (col < N) {
                        if (row < M) epi_store<EPI, TAct>(ep, row, col, v);
                        if (arg_better(v, col, bv, bi)) { bv = v; bi = col; }
                    }
                }
#pragma unroll
                for (int off = 16; off >= 1; off >>= 1) {
                    const float ov = __shfl_xor(bv, off, kWave);
                    const int oi = __shfl_xor(bi, off, kWave);
                    if (arg_better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
                }
                if (lr == 0) { red_val[lrow * WN + wn] = bv; red_idx[lrow * WN + wn] = bi; }
            }
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
            ep.part_val[(int64_t)row * ep.nparts + bn] = bv;
            ep.part_idx[(int64_t)row * ep.nparts + bn] = bi;
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
            if constexpr (EPI == EPI_ARGMAX)
                if (arg_better(v, col, bv, bi)) { bv = v; bi = col; }
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
                ep.part_val[(int64_t)row * ep.nparts + bn] = bv;
                ep.part_idx[(int64_t)row * ep.nparts + bn] = bi;
            }
        }
    }
}

// Reduce the per-tile partials of each row to one token; writes `rep`
// consecutive copies starting at out[(row0 + row) * rep].  One wave per row.
// A row without any ordered value (all NaN) yields token 0, so that the id is
// always a valid embedding row.
__global__ void __launch_bounds__(256)
argmax_finalize_kernel(const float *__restrict__ part_val, const int32_t *__restrict__ part_idx,
                       int64_t rows, int nparts, int32_t *__restrict__ out, int64_t row0, int rep,
                       int vocab)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int p = lane; p < nparts; p += kWave) {
        const float v = part_val[row * nparts + p];
        const int i = part_idx[row * nparts + p];
        if (arg_better(v, i, bv, bi)) { bv = v; bi = i; }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float ov = __shfl_xor(bv, off, kWave);
        const int oi = __shfl_xor(bi, off, kWave);
        if (arg_better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
    if (bi < 0 || bi >= vocab) bi = 0;
    for (int r = lane; r < rep; r += kWave) out[(row0 + row) * rep + r] = bi;
}
