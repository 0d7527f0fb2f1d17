// Token mixing of an SRM block for decode steps of a dozen to about a thousand rows of a bf16 model
// (Eq. 2 / Eq. 3 with the head projections of Eq. 10, behind the block's first LayerNorm), as ONE kernel:
//
//   a = LN1(x + pending slabs);  u = a W_in^T + b_in;  S, m = state update(S, u);  slab_q = m_q W_out[:, q]^T
//
// followed by the LayerNorm kernel that adds the slabs to x and normalises (ln_kernel).  As separate launches
// (LayerNorm, in-projection + update, out-projection) these are three dependent kernels of 5 - 8 us each at such
// sizes, none of which comes near filling the chip.
//
// A work-group owns 16 rows x 128 columns of u (block q of the d / 128 column blocks): it normalises its 16 rows
// (every column block does that again: 32 KB of x per work-group, from L2), forms its 128 columns of u and
// updates its 16 x 128 piece of the state.  Its 128 columns of m are a K slice of the out-projection, so it can
// go on to form that slice's contribution to all d output columns, which it writes as fp32 slab q; the slabs
// are added in slab order by the next kernel, so the sum does not depend on scheduling.  u and m never
// leave the CU, and the d / 128 work-groups of a row group run on different CUs, each reading only 1 / (d / 128)
// of both weight matrices (256 d bytes of each), each requested whole, in one go - no k loop waits for memory.
// The share of W_in is requested at the start and goes global -> LDS (buffer_load ... lds, whole 128-byte row
// segments per request, into the swizzled layout of gemm_bf16_kernel; each wavefront loads and reads only its
// own rows, so no barrier guards them).  The share of W_out is as large and follows into the same LDS once the
// in-projection has read W_in: a second trip to memory, under the state update.  (Loaded straight into registers
// as MFMA operand fragments instead, every lane's 16 bytes are a request of their own: 8.6 us until both shares
// had arrived that way, and 2.5 us of stalled issue for W_out's alone.)
//
// Work-group: 4 wavefronts; the products are 16x16x32 bf16 MFMAs formed transposed (W rows as first operand), so
// a lane holds 4 consecutive output columns of one row: lane l works on row l & 15, column quad l >> 4 of a
// 16-column tile.  Wavefront w forms u columns 128 q + 32 w .. + 31 (2 tiles) and output columns
// w d / 4 .. + d / 4 - 1 of the slab (d / 64 tiles); the second operands (LN1 rows: 16 x d; m: 16 x 128, bf16)
// are panels in LDS shared by the four wavefronts.
#pragma once
#include "gemm.hpp"

struct TokMixArgs {
    const float *x;            // [rows][d] residual stream
    const float *pend;         // npend slabs [rows][d] (slab stride pend_stride floats) that a K-sliced projection
    int32_t npend;             // left to be added to x: LN1 sees x + slabs (summed in slab order); or nullptr
    int64_t pend_stride;
    const float *ln1_g, *ln1_b;
    float eps;
    const bf16 *w_in, *w_out;  // [d][d]
    const float *b_in, *b_out; // [d]
    void *state;               // [rows][d] fp32 or binary16 (template)
    const float *alpha, *beta, *lam;   // [H][n_ctx], [H][n_ctx], [H]
    int32_t n_ctx, hrow, dh;
    int32_t pos;               // the position, unless pos_dev or pos_rows is set; a position outside [0, n_ctx)
    const int *pos_dev;        // leaves the row's state alone and mixes zeros (as EPI_MIX does)
    const int *pos_rows;
    float *slabs;              // [d / 128][rows][d] written: slab q = m[:, 128 q ..] W_out[:, 128 q ..]^T (+ b_out in slab 0)
    int64_t rows;
    // Measuring hook (srm_linear_timeline_probe): if not null, work-group b < clk_blocks writes eight words at
    // clk + 8 b: the 100 MHz wall clock at its start, when its first batch of loads has arrived, after
    // LayerNorm1, after the in-projection, after the state update, after the out-projection's products, and
    // after its stores have completed; HW_ID | XCC_ID << 32.
    unsigned long long *clk;
    int64_t clk_blocks;
};

constexpr int kTokMixCols = 128;                     // columns of u per work-group

template <int D>
constexpr int tokmix_lds_bytes()
{
    // the work-group's rows of W_in: 128 x D bf16; panel of LN1 rows: 16 x (D + 8) bf16; panel of m: 16 x (128 + 8) bf16
    return kTokMixCols * D * 2 + 16 * (D + 8) * 2 + 16 * (kTokMixCols + 8) * 2;
}

template <int D, typename TState>
__global__ void __launch_bounds__(256)
token_mix_kernel(TokMixArgs a)
{
    constexpr int RB = 16, NW = 4, QC = kTokMixCols, Q = D / QC;
    constexpr int NL = D / 64;                       // 16-column tiles of the slab per wavefront
    constexpr int NU = QC / NW / 16;                 // 16-column tiles of u per wavefront (2)
    constexpr int HK1 = D / 32, HK2 = QC / 32;       // 32-wide k steps of the two projections
    constexpr int PLD = D + 8, MLD = QC + 8;         // panel row strides: 16 bytes of padding, conflict-free reads
    static_assert(D % 256 == 0 && D % QC == 0, "whole LayerNorm vectors per lane, whole column blocks");

    extern __shared__ __align__(16) unsigned char smem_raw[];
    constexpr int BK = 64, KT = D / BK, WR = QC / NW;                       // k tiles of W_in; its rows per wavefront
    constexpr int STAGE = WR * BK;                                         // elements of one k tile of a wavefront
    static_assert(KT * WR / 8 <= 63, "more tile loads in flight than the counter holds");
    bf16 *wring = reinterpret_cast<bf16 *>(smem_raw);                      // [NW][KT][WR rows][BK], rows swizzled
    bf16 *panel = wring + NW * KT * STAGE;                                 // [RB][PLD]
    bf16 *mpanel = panel + RB * PLD;                                       // [RB][MLD]

    // work-group barrier that orders LDS traffic only: it does not wait for the weight loads still in flight
#define SRM_LDS_BARRIER()                                                                        \
    {                                                                                            \
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");                          \
        __builtin_amdgcn_s_barrier();                                                            \
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");                          \
    }
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int j = lane & 15, g = lane >> 4;
    const int q = blockIdx.x % Q;
    const int64_t row = (int64_t)(blockIdx.x / Q) * RB + j;
    const bool valid = row < a.rows;
    const int64_t rl = valid ? row : a.rows - 1;     // rows past the end load the last row and store nothing
    const int ucol0 = q * QC + wave * (QC / NW);     // this wavefront's columns of u
    const int ocol0 = wave * (D / NW);               // ... and of the slab

    const bool probe = a.clk != nullptr && (int64_t)blockIdx.x < a.clk_blocks;
    unsigned long long ck[7] = {0, 0, 0, 0, 0, 0, 0};
    if (probe) ck[0] = wall_clock64();

    // ---- everything the first phases need from memory is requested up front: the wavefront's rows of W_in, the
    // position, the rows of x with the waiting slabs, the parameters, the old state - LayerNorm1 starts when these
    // have arrived, one round trip into the kernel.  The coefficients at the position follow (they need the
    // position) and arrive under LayerNorm1.
    // ---- tile loads (buffer_load ... lds): one instruction moves rows 8 i .. 8 i + 7 x 128 bytes of a k tile of this
    // wavefront's rows; lane (r = l >> 3, slot = l & 7) fetches chunk slot ^ swz(8 i + r) of its row, swz(8 i + r) =
    // (4 (i & 1) + (r >> 1)) & 7.  Issued from an asm statement (see gemm_persist.hpp); all waits are explicit.
    typedef __attribute__((address_space(3))) unsigned char lds_byte;
    const int wv = __builtin_amdgcn_readfirstlane(wave);
    const unsigned dst0 = __builtin_amdgcn_readfirstlane(
        (unsigned)reinterpret_cast<unsigned long long>((lds_byte *)smem_raw)) + wv * KT * STAGE * 2;
    auto descriptor = [](const void *base, int bytes) {
        u32x4_t rs;
        const unsigned long long p = reinterpret_cast<unsigned long long>(base);
        rs[0] = __builtin_amdgcn_readfirstlane((unsigned)p);
        rs[1] = __builtin_amdgcn_readfirstlane((unsigned)(p >> 32));
        rs[2] = __builtin_amdgcn_readfirstlane((unsigned)bytes);
        rs[3] = 0x00020000u;
        return rs;
    };
    const int ld_r = lane >> 3, ld_c = lane & 7;
    const int voff_even = (ld_r * D + ((ld_c ^ (ld_r >> 1)) << 3)) * 2;
    const int voff_odd = (ld_r * D + ((ld_c ^ ((4 + (ld_r >> 1)) & 7)) << 3)) * 2;
    auto dma = [&](const u32x4_t &rs, unsigned lds_dst, int voff, int soff) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                     :
                     : "s"(lds_dst), "v"(voff), "s"(rs), "s"(soff)
                     : "memory");
    };
    {
        // W_in rows ucol0 .. ucol0 + 31, all k, as KT k tiles of 32 rows x 64.  They are the oldest loads of the
        // wavefront, so the wait for x (LayerNorm1) also waits for them.
        const u32x4_t rs = descriptor(a.w_in + (size_t)(q * QC + wv * WR) * D, WR * D * 2);
        static_for<0, KT * (WR / 8)>([&](auto n_) {
            constexpr int kt = decltype(n_)::value / (WR / 8), i = decltype(n_)::value % (WR / 8);
            dma(rs, dst0 + (kt * STAGE + i * 8 * BK) * 2, (i & 1) ? voff_odd : voff_even, (i * 8 * D + kt * BK) * 2);
        });
    }
    int p_dev = 0, p_row = 0;
    if (a.pos_dev) p_dev = *a.pos_dev;
    if (a.pos_rows) p_row = a.pos_rows[rl];
    // LayerNorm1's rows in the layout of ln_kernel: wavefront w normalises rows 4 w .. 4 w + 3, lane l holds
    // columns 256 i + 4 l .. + 3 of each (whole-kilobyte requests; as fragments, 16 bytes per lane and row, the
    // same rows cost 3 us more)
    constexpr int VPL = D / 256, RPW = RB / NW;
    float4 xr[RPW][VPL], lg[VPL], lb[VPL];
    int64_t xrow[RPW];
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        xrow[r] = min((int64_t)(blockIdx.x / Q) * RB + wave * RPW + r, a.rows - 1);
#pragma unroll
        for (int i = 0; i < VPL; ++i) xr[r][i] = load4(a.x + xrow[r] * D + i * 256 + lane * 4);
    }
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
        lg[i] = load4(a.ln1_g + i * 256 + lane * 4);
        lb[i] = load4(a.ln1_b + i * 256 + lane * 4);
    }
    const TState *sp = static_cast<const TState *>(a.state);
    float4 bo[NL], sv[NU], bi[NU];
#pragma unroll
    for (int t = 0; t < NL; ++t) bo[t] = load4(a.b_out + ocol0 + t * 16 + 4 * g);     // (only slab 0 carries the bias)
#pragma unroll
    for (int t = 0; t < NU; ++t) {
        const int c = ucol0 + t * 16 + 4 * g;
        sv[t] = load_state4(sp, (rl * D + c) >> 2);
        bi[t] = load4(a.b_in + c);
    }
    // the slabs still to be added to x, four requested at a time (one at a time would serialise their latencies),
    // summed in slab order
    for (int s0 = 0; s0 < a.npend; s0 += 4) {
        float4 p[4][RPW][VPL];
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int r = 0; r < RPW; ++r)
#pragma unroll
                for (int i = 0; i < VPL; ++i)
                    p[s][r][i] = load4(a.pend + (int64_t)min(s0 + s, a.npend - 1) * a.pend_stride + xrow[r] * D + i * 256 + lane * 4);
#pragma unroll
        for (int s = 0; s < 4; ++s)
            if (s0 + s < a.npend) {
#pragma unroll
                for (int r = 0; r < RPW; ++r)
#pragma unroll
                    for (int i = 0; i < VPL; ++i) {
                        xr[r][i].x += p[s][r][i].x; xr[r][i].y += p[s][r][i].y;
                        xr[r][i].z += p[s][r][i].z; xr[r][i].w += p[s][r][i].w;
                    }
            }
    }
    const int ps = a.pos_rows ? p_row : a.pos_dev ? __builtin_amdgcn_readfirstlane(p_dev) : a.pos;
    const bool act = ps >= 0 && ps < a.n_ctx;
    const int pc = act ? ps : 0;
    float al[NU], be[NU], la[NU];
#pragma unroll
    for (int t = 0; t < NU; ++t) {
        const int h = (ucol0 + t * 16 + 4 * g) / a.dh;
        al[t] = a.alpha[(size_t)h * a.n_ctx + pc];
        be[t] = a.beta[(size_t)h * a.n_ctx + pc];
        la[t] = a.lam[h];
    }
    constexpr int kSecond = 3 * NU;                  // loads that may still be in flight: the coefficients
    if (probe) { __builtin_amdgcn_s_waitcnt(0x0F70 | (kSecond & 15) | ((kSecond >> 4) << 14)); ck[1] = wall_clock64(); }

    // ---- LayerNorm1 (the arithmetic of ln_kernel, in its order), normalised rows to the panel as bf16
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        float sum = 0.0f;
#pragma unroll
        for (int i = 0; i < VPL; ++i) sum += (xr[r][i].x + xr[r][i].y) + (xr[r][i].z + xr[r][i].w);
        const float mean = wave_sum(sum) / (float)D;
        float sq = 0.0f;
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const float p = xr[r][i].x - mean, t = xr[r][i].y - mean, s = xr[r][i].z - mean, u = xr[r][i].w - mean;
            sq += (p * p + t * t) + (s * s + u * u);
        }
        const float var = wave_sum(sq) / (float)D;
        const float rstd = 1.0f / sqrtf(var + a.eps);
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            float4 o;
            o.x = (xr[r][i].x - mean) * rstd * lg[i].x + lb[i].x;
            o.y = (xr[r][i].y - mean) * rstd * lg[i].y + lb[i].y;
            o.z = (xr[r][i].z - mean) * rstd * lg[i].z + lb[i].z;
            o.w = (xr[r][i].w - mean) * rstd * lg[i].w + lb[i].w;
            store4(panel + (wave * RPW + r) * PLD + i * 256 + lane * 4, o);
        }
    }
    SRM_LDS_BARRIER()                                // the panel is complete
    if (probe) ck[2] = wall_clock64();

    // ---- u = LN1 rows x W_in^T + b_in on this wavefront's 32 columns
    f32x4_t accu[NU];
#pragma unroll
    for (int t = 0; t < NU; ++t) { accu[t][0] = bi[t].x; accu[t][1] = bi[t].y; accu[t][2] = bi[t].z; accu[t][3] = bi[t].w; }
    // (the wavefront's W_in rows have landed long ago: the tile loads are older than x, which LayerNorm1 waited
    // for.  Waiting for everything here, the coefficients included, leaves the compiler no later wait that would
    // also wait for the tile loads issued below.)
    __builtin_amdgcn_s_waitcnt(0x0F70);
    {
        const bf16 *ws = wring + wave * KT * STAGE + j * BK;
        const int swz = (j >> 1) & 7;
#pragma unroll
        for (int hk = 0; hk < HK1; ++hk) {
            const bf16x8_t fa = *reinterpret_cast<const bf16x8_t *>(panel + j * PLD + hk * 32 + 8 * g);
#pragma unroll
            for (int t = 0; t < NU; ++t) {
                const bf16x8_t fw = *reinterpret_cast<const bf16x8_t *>(ws + (hk >> 1) * STAGE + t * 16 * BK +
                                                                        ((((hk & 1) * 4 + g) ^ swz) << 3));
                accu[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fw, fa, accu[t], 0, 0, 0);
            }
        }
    }

    if (probe) { __builtin_amdgcn_sched_barrier(0); asm volatile("s_nop 0" :: "v"(accu[NU - 1][0])); ck[3] = wall_clock64(); }

    // ---- the wavefront's share of W_out takes the place of its W_in rows in LDS (rows ocol0 .. + d / 4 - 1,
    // k = 128 q .. + 127, as two k tiles of d / 4 rows x 64), requested now and travelling under the state update.
    // Nothing else is issued to memory between here and the products that wait for it (the state is stored at
    // the end), so the two waits below can count tile loads.
    constexpr int WRO = D / NW, OSTAGE = WRO * BK, O_IT = WRO / 8;
    static_assert(2 * OSTAGE == KT * STAGE && 2 * O_IT <= 63, "the share of W_out fits the ring and the counter");
    __builtin_amdgcn_s_waitcnt(0xC07F);              // lgkmcnt(0): the W_in rows have been read
    {
        const u32x4_t rs = descriptor(a.w_out + (size_t)(wv * WRO) * D + q * QC, (WRO * D - q * QC) * 2);
        static_for<0, 2 * O_IT>([&](auto n_) {
            constexpr int kt = decltype(n_)::value / O_IT, i = decltype(n_)::value % O_IT;
            dma(rs, dst0 + (kt * OSTAGE + i * 8 * BK) * 2, (i & 1) ? voff_odd : voff_even, (i * 8 * D + kt * BK) * 2);
        });
    }

    // ---- state update (u in the activation type, as the unfused path stores it); m goes to its panel
    TState *sq_ = static_cast<TState *>(a.state);
    float4 nv[NU];
#pragma unroll
    for (int t = 0; t < NU; ++t) {
        const int c = ucol0 + t * 16 + 4 * g;
        const bool row_repeat = c / a.dh < a.hrow;
        const float p = row_repeat ? al[t] : 1.0f, r = row_repeat ? 1.0f : al[t];
        float4 n = make_float4(0.f, 0.f, 0.f, 0.f), m = n;
        if (act) {
            n.x = fmaf(la[t], sv[t].x, p * (float)(bf16)accu[t][0]);
            n.y = fmaf(la[t], sv[t].y, p * (float)(bf16)accu[t][1]);
            n.z = fmaf(la[t], sv[t].z, p * (float)(bf16)accu[t][2]);
            n.w = fmaf(la[t], sv[t].w, p * (float)(bf16)accu[t][3]);
            n = make_float4(to_state(n.x, sq_), to_state(n.y, sq_), to_state(n.z, sq_), to_state(n.w, sq_));
            m = make_float4(fmaf(r, n.x, be[t]), fmaf(r, n.y, be[t]), fmaf(r, n.z, be[t]), fmaf(r, n.w, be[t]));
        }
        nv[t] = n;
        store4(mpanel + j * MLD + (c - q * QC), m);
    }
    SRM_LDS_BARRIER()                                // the panel of m is complete
    if (probe) ck[4] = wall_clock64();

    // ---- slab q = m (16 x 128) x W_out[:, 128 q ..]^T on this wavefront's d / 4 output columns (+ b_out in slab 0)
    f32x4_t acco[NL];
#pragma unroll
    for (int t = 0; t < NL; ++t) {
        const float on = q == 0 ? 1.0f : 0.0f;
        acco[t][0] = on * bo[t].x; acco[t][1] = on * bo[t].y; acco[t][2] = on * bo[t].z; acco[t][3] = on * bo[t].w;
    }
    {
        const bf16 *ws = wring + wave * KT * STAGE + j * BK;
        const int swz = (j >> 1) & 7;
#pragma unroll
        for (int hk = 0; hk < HK2; ++hk) {
            if (hk == 0) __builtin_amdgcn_s_waitcnt(0x0F70 | (O_IT & 15) | ((O_IT >> 4) << 14));   // k tile 0 has landed
            if (hk == 2) __builtin_amdgcn_s_waitcnt(0x0F70);                                        // vmcnt(0): k tile 1
            const bf16x8_t fa = *reinterpret_cast<const bf16x8_t *>(mpanel + j * MLD + hk * 32 + 8 * g);
#pragma unroll
            for (int t = 0; t < NL; ++t) {
                const bf16x8_t fw = *reinterpret_cast<const bf16x8_t *>(ws + (hk >> 1) * OSTAGE + t * 16 * BK +
                                                                        ((((hk & 1) * 4 + g) ^ swz) << 3));
                acco[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fw, fa, acco[t], 0, 0, 0);
            }
        }
    }
    if (probe) { __builtin_amdgcn_sched_barrier(0); asm volatile("s_nop 0" :: "v"(acco[NL - 1][0])); ck[5] = wall_clock64(); }
    if (valid && act) {
#pragma unroll
        for (int t = 0; t < NU; ++t) store_state4(sq_, (row * D + ucol0 + t * 16 + 4 * g) >> 2, nv[t]);
    }
    if (valid) {
        float *dst = a.slabs + ((int64_t)q * a.rows + row) * D + ocol0 + 4 * g;
#pragma unroll
        for (int t = 0; t < NL; ++t) store4(dst + t * 16, make_float4(acco[t][0], acco[t][1], acco[t][2], acco[t][3]));
    }
    if (probe) {
        __builtin_amdgcn_s_waitcnt(0);               // this wave's stores have completed
        if (tid == 0) {
            unsigned long long *p = a.clk + 8 * (int64_t)blockIdx.x;
            for (int i = 0; i < 6; ++i) p[i] = ck[i];
            p[6] = wall_clock64();
            p[7] = (unsigned long long)__builtin_amdgcn_s_getreg((31 << 11) | 4) |
                   ((unsigned long long)__builtin_amdgcn_s_getreg((3 << 11) | 20) << 32);
        }
    }
#undef SRM_LDS_BARRIER
}
