// Persistent form of the 256x256 bf16 MFMA GEMM (same contract and epilogues as gemm_bf16_kernel in
// gemm.hpp: out = epilogue(A W^T + bias)), for launches with more output tiles than CUs.
//
// One work-group per CU walks its tiles v = blockIdx.x, blockIdx.x + gridDim.x, ... and keeps the LDS ring
// running from one output tile into the next: the first k tile of the next output tile (and its 256 bias
// values) is requested two k tiles before the current k loop ends, so it has landed before the epilogue
// starts.  A tile that is not a CU's first therefore starts its MFMAs at once instead of after a work-group
// launch and a cold round trip to memory.
//
// LDS (160 KB): ring slot 0 | ring slot 1 | 32 KB; a slot holds a 256x64 A tile, then a 256x64 W tile, in
// the swizzled layout of gemm_bf16_kernel; the last 1 KB holds the tile's bias.
//   RING = false: the epilogue stages its stores through slot 1 and the 32 KB behind it (78 KB), so only
//     slot 0 is filled under it, and the next tile's second k tile is requested right after the epilogue.
//   RING = true (the LM head's argmax without stored logits, whose epilogue needs 8 KB only, which lie behind
//     the ring): both slots keep filling, the k loop of the next tile continues as if it were the same one.
#pragma once
#include "gemm.hpp"

constexpr int kPersistLds = 160 * 1024;

template <int EPI, typename TAct, bool RING = false>
__global__ void __launch_bounds__(512)
gemm_bf16_persist_kernel(const bf16 *__restrict__ A, const bf16 *__restrict__ W, int M, int N, int K, GemmEpi ep)
{
    constexpr int BM = 256, BN = 256, WM = 2, WN = 4, BK = 64;
    constexpr int NW = WM * WN, NTHR = NW * 64;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int A_IT = BM * BK / 8 / NTHR, B_IT = BN * BK / 8 / NTHR, LD_IT = A_IT + B_IT;
    constexpr int SLOT = (BM + BN) * BK;             // elements per ring slot
    constexpr int STG = WTN + 4;
    static_assert(!RING || EPI == EPI_ARGMAX, "only the argmax epilogue can do without a stage");
    // bytes: the epilogue's stage starts at slot 1; RING: placed so that the argmax partials lie behind the ring
    constexpr int kStageOff = RING ? 2 * SLOT * 2 - NW * 32 * STG * 4 : SLOT * 2;
    constexpr int kBiasOff = kPersistLds - BN * 4;
    static_assert(kStageOff + NW * 32 * STG * 4 + BM * WN * 8 <= kBiasOff, "epilogue stage runs into the bias");

    extern __shared__ __align__(16) unsigned char smem_raw[];
    bf16 *ring = reinterpret_cast<bf16 *>(smem_raw);
    const float *bias_lds = reinterpret_cast<const float *>(smem_raw + kBiasOff);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int lr = lane & 31, lk = lane >> 5;

    const int nbm = (M + BM - 1) / BM, nbn = (N + BN - 1) / BN, nblk = nbm * nbn;
    const int KT = K / BK;                           // even and >= 4 (the launcher checks)

    // Tile loads: buffer_load ... lds, one wave instruction = 8 rows x 128 bytes, lane (r = l >> 3, slot = l & 7)
    // fetches chunk slot ^ swz(r) of its row.  A descriptor covers exactly one tile's rows of A or W (rows past
    // M or N, and everything of a descriptor of zero bytes, arrive as zeros).  They are issued from an asm
    // statement: a load that the compiler knows to write LDS makes it wait for all outstanding loads in front
    // of the next LDS read it cannot prove disjoint.  The waits are the explicit ones below.
    constexpr int ROWS_PER_IT = NTHR / 8;
    const int ld_r = tid >> 3, ld_c = tid & 7;
    const int ld_voff = (ld_r * K + ((ld_c ^ swz_of_row(ld_r)) << 3)) * 2;       // bytes
    typedef __attribute__((address_space(3))) unsigned char lds_byte;
    const unsigned ring_lds = __builtin_amdgcn_readfirstlane(
        (unsigned)reinterpret_cast<unsigned long long>((lds_byte *)smem_raw));
    auto descriptor = [](const void *base, int bytes) {
        u32x4_t rs;
        const unsigned long long a = reinterpret_cast<unsigned long long>(base);
        rs[0] = __builtin_amdgcn_readfirstlane((unsigned)a);
        rs[1] = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32));             // stride 0: raw buffer
        rs[2] = __builtin_amdgcn_readfirstlane((unsigned)bytes);
        rs[3] = 0x00020000u;
        return rs;
    };
    auto dma = [&](const u32x4_t &rs, unsigned lds_dst, int voff, int soff) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                     :
                     : "s"(lds_dst), "v"(voff), "s"(rs), "s"(soff)
                     : "memory");
    };
    // tile load number i of k tile kq (the first A_IT fetch A, the rest W) into ring slot `slot`
    auto dma_one = [&](int i, const u32x4_t &ra, const u32x4_t &rw, int kq, int slot) {
        if (i < A_IT)
            dma(ra, ring_lds + (slot * SLOT + (i * ROWS_PER_IT + wave * 8) * BK) * 2, ld_voff,
                (i * ROWS_PER_IT * K + kq * BK) * 2);
        else
            dma(rw, ring_lds + (slot * SLOT + BM * BK + ((i - A_IT) * ROWS_PER_IT + wave * 8) * BK) * 2, ld_voff,
                ((i - A_IT) * ROWS_PER_IT * K + kq * BK) * 2);
    };
    auto dma_tile = [&](const u32x4_t &ra, const u32x4_t &rw, int kq, int slot) {
        static_for<0, LD_IT>([&](auto i_) { dma_one(decltype(i_)::value, ra, rw, kq, slot); });
    };
    // the 256 bias values of a tile: one instruction of wavefront 0 (zeros for columns past N)
    auto dma_bias = [&](const u32x4_t &rb) {
        if (ep.bias && wave == 0) dma(rb, ring_lds + kBiasOff, lane * 16, 0);
    };
    struct Tile {
        int m0, n0, bn;
        u32x4_t ra, rw, rb;
    };
    auto tile_at = [&](int v) {
        Tile t;
        const bool exists = v < nblk;
        int bm;
        tile_of_pid(exists ? v : 0, nbm, nbn, bm, t.bn);
        t.m0 = bm * BM;
        t.n0 = t.bn * BN;
        t.ra = descriptor(A + (size_t)t.m0 * K, exists ? min(BM, M - t.m0) * K * 2 : 0);
        t.rw = descriptor(W + (size_t)t.n0 * K, exists ? min(BN, N - t.n0) * K * 2 : 0);
        t.rb = descriptor(ep.bias ? ep.bias + t.n0 : nullptr, exists && ep.bias ? min(BN, N - t.n0) * 4 : 0);
        return t;
    };
#define SRM_WAIT_VM(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))

    const int sw = swz_of_row(lr);
    const int a_row_off = (wm * WTM + lr) * BK;
    const int b_row_off = BM * BK + (wn * WTN + lr) * BK;
    bf16x8_t fa[4][TM], fb[4][TN];                   // one operand set per k-substep
    f32x16_t acc[TM][TN];
#define SRM_READ_FRAGS(slot, kk, set)                                                            \
    {                                                                                            \
        const int ch_ = ((((kk) * 2 + lk) ^ sw) << 3);                                           \
        const bf16 *as_ = ring + (slot) * SLOT + a_row_off + ch_;                                \
        const bf16 *bs_ = ring + (slot) * SLOT + b_row_off + ch_;                                \
        _Pragma("unroll") for (int i = 0; i < TM; ++i)                                           \
            fa[set][i] = *reinterpret_cast<const bf16x8_t *>(as_ + i * 32 * BK);                 \
        _Pragma("unroll") for (int j = 0; j < TN; ++j)                                           \
            fb[set][j] = *reinterpret_cast<const bf16x8_t *>(bs_ + j * 32 * BK);                 \
    }
#define SRM_MFMA_STEP(set)                                                                       \
    _Pragma("unroll") for (int i = 0; i < TM; ++i)                                               \
        _Pragma("unroll") for (int j = 0; j < TN; ++j) /* transposed: MFMA rows run over N */    \
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[set][j], fa[set][i], acc[i][j], 0, 0, 0);
    // one LDS read behind each MFMA (see gemm_bf16_kernel)
#define SRM_INTERLEAVE()                                                                         \
    _Pragma("unroll") for (int q = 0; q < TM * TN; ++q) {                                        \
        constexpr int S_ = TM * TN;                                                              \
        constexpr int R_ = (TM + TN + S_ - 1) / S_;                                              \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                       \
        if (q * R_ < TM + TN) __builtin_amdgcn_sched_group_barrier(0x100, R_, 0);                \
    }                                                                                            \
    __builtin_amdgcn_sched_barrier(0);

    int v = blockIdx.x;                              // gridDim.x <= nblk: every work-group has a first tile
    Tile cur = tile_at(v);
    unsigned long long clk_c0 = 0, clk_t0 = 0, clk_c1 = 0, clk_t1 = 0, clk_c2 = 0, clk_t2 = 0;
    if (ep.clk) { clk_c0 = clock64(); clk_t0 = wall_clock64(); }
    dma_bias(cur.rb);
    dma_tile(cur.ra, cur.rw, 0, 0);
    dma_tile(cur.ra, cur.rw, 1, 1);
    SRM_WAIT_VM(LD_IT);                              // loads return in order: the bias and k tile 0 are there
    __syncthreads();
    SRM_READ_FRAGS(0, 0, 0)
    SRM_READ_FRAGS(0, 1, 1)

    for (;;) {
        const bool probe = ep.clk != nullptr && v < ep.clk_blocks;
        const int vn = v + (int)gridDim.x;
        const Tile nxt = tile_at(vn);                // of zero size behind the last tile
        // the accumulators start at the bias of their column: register quad g of tile (i, j) holds columns
        // j*32 + 8g + 4lk .. +3 of the wave tile
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                float4 b = make_float4(0.f, 0.f, 0.f, 0.f);
                if (ep.bias) b = *reinterpret_cast<const float4 *>(bias_lds + wn * WTN + j * 32 + 8 * g + 4 * lk);
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    acc[i][j][4 * g] = b.x; acc[i][j][4 * g + 1] = b.y;
                    acc[i][j][4 * g + 2] = b.z; acc[i][j][4 * g + 3] = b.w;
                }
            }
        __builtin_amdgcn_sched_barrier(0);
        if (probe) { clk_c1 = clock64(); clk_t1 = wall_clock64(); }

        // The schedule of gemm_bf16_kernel.  The loads issued in k tile kt fill the slot it frees with k tile
        // kt+2 of this output tile or, from k tile KT-2 on, with k tile kt+2-KT of the next one; the operands
        // it reads ahead in its second half are those of k tile kt+1, in k tile KT-1 (RING only) the next
        // output tile's first.
        const int kt_end = RING ? KT : KT - 1;
        for (int kt = 0; kt < kt_end; ++kt) {
            const int s_cur = kt & 1, s_nxt = s_cur ^ 1;
            const bool ahead = kt + 2 >= KT;
            const u32x4_t ra = ahead ? nxt.ra : cur.ra, rw = ahead ? nxt.rw : cur.rw;
            const int kq = ahead ? kt + 2 - KT : kt + 2;
            SRM_READ_FRAGS(s_cur, 2, 2)
            SRM_MFMA_STEP(0)
            SRM_INTERLEAVE()
            SRM_READ_FRAGS(s_cur, 3, 3)
            SRM_MFMA_STEP(1)
            SRM_INTERLEAVE()
            SRM_WAIT_VM(0);                          // k tile kt+1 has landed
            __syncthreads();                         // ... for everyone, and slot s_cur is free
            {
                const int ch_ = ((lk ^ sw) << 3);
                const bf16 *as_ = ring + s_nxt * SLOT + a_row_off + ch_;
                const bf16 *bs_ = ring + s_nxt * SLOT + b_row_off + ch_;
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
                    for (int l = q * LPM; l < (q + 1) * LPM && l < LD_IT; ++l) dma_one(l, ra, rw, kq, s_cur);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (kt == KT - 2) dma_bias(nxt.rb);      // (read by nobody before the next output tile starts)
            SRM_READ_FRAGS(s_nxt, 1, 1)
            SRM_MFMA_STEP(3)
            SRM_INTERLEAVE()
        }
        if constexpr (!RING) {
            // k tile KT-1, from slot 1: nothing to read ahead, nothing to load (slot 1 becomes the epilogue's stage)
            SRM_READ_FRAGS(1, 2, 2)
            SRM_MFMA_STEP(0)
            SRM_INTERLEAVE()
            SRM_READ_FRAGS(1, 3, 3)
            SRM_MFMA_STEP(1)
            SRM_INTERLEAVE()
            SRM_MFMA_STEP(2)
            SRM_MFMA_STEP(3)
            SRM_WAIT_VM(0);                          // the next output tile's k tile 0 and bias have landed
            __syncthreads();                         // ... for everyone, and slot 1 is free
        }
        if (probe) { clk_c2 = clock64(); clk_t2 = wall_clock64(); }

        // (the thread index through an opaque copy: what the epilogue derives from it is computed here, per
        // tile, and not once in front of the tile loop, where it would be held in registers across every k loop)
        int tid_e = threadIdx.x;
        asm volatile("" : "+v"(tid_e));
        gemm_epilogue<BM, BN, WM, WN, EPI, TAct>(acc, smem_raw + kStageOff, ep, M, N, cur.m0, cur.n0, cur.bn, tid_e);
        if (probe) {
            __builtin_amdgcn_s_waitcnt(0);           // this wave's stores have completed
            if (tid == 0) {
                unsigned long long *p = ep.clk + 8 * (int64_t)v;
                p[0] = clk_t0; p[1] = clk_t1; p[2] = clk_t2; p[3] = wall_clock64(); p[4] = clk_c1; p[5] = clk_c2;
                p[6] = (unsigned long long)__builtin_amdgcn_s_getreg((31 << 11) | 4) |        // HW_ID
                       ((unsigned long long)__builtin_amdgcn_s_getreg((3 << 11) | 20) << 32);  // XCC_ID
                p[7] = clk_c0;
            }
            clk_c0 = clock64();
            clk_t0 = wall_clock64();
        }
        if (vn >= nblk) break;                       // (block-uniform)
        v = vn;
        cur = nxt;
        if constexpr (!RING) {
            // every wave has read its stage back (the stores themselves may still be on their way): slot 1 can
            // take the new output tile's k tile 1
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
            dma_tile(cur.ra, cur.rw, 1, 1);
            SRM_READ_FRAGS(0, 0, 0)
            SRM_READ_FRAGS(0, 1, 1)
        }
    }
    SRM_WAIT_VM(0);                                  // (RING: the loads behind the last tile, of zero size)
#undef SRM_MFMA_STEP
#undef SRM_INTERLEAVE
#undef SRM_WAIT_VM
#undef SRM_READ_FRAGS
}
