// Embedding gather and LayerNorm (one wavefront per token row).
//
// The residual stream is fp32; the normalised row is written in the type the
// next GEMM consumes (bf16 or fp32).  Statistics are two-pass (mean, then the
// biased variance of the centred values) over values held in registers, summed
// with wavefront shuffles.
#pragma once
#include "common.hpp"
#include <type_traits>

// VPL = float4 vectors per lane: covers d <= 256 * VPL.
//   GATHER: x = embed[tok[row]] is fetched, stored to x_out (fp32) and normalised.
//   else:   x is read from x_in + row * in_stride, or, if seq_end is given, from
//           the last row of packed sequence `row`: source row seq_end[row + 1] - 1 - base,
//           clamped to [0, src_rows).
//   part:   nsplit slabs [rows][d] (slab stride part_stride floats) of a split-K
//           GEMM are added to x first, in slab order, and the updated x is written
//           back to x_out: the residual add of that GEMM, done here.
//   add_act: [rows][d] in the activation type, added to x first (x_out gets the
//           sum): the residual add of a non-projected mixer layer.
//   advance_ctr (GATHER only): the two step counters of a multi-step generate call
//           (position, step), advanced by one here, in the first kernel of a step,
//           instead of by a launch of their own behind the previous step; no block
//           of this kernel reads them.
template <typename TW, typename TAct, int VPL, bool GATHER>
__global__ void __launch_bounds__(256)
ln_kernel(const float *x_in, int64_t in_stride, const int32_t *__restrict__ tok,
          const TW *__restrict__ embed, int vocab, float *x_out,
          const float *__restrict__ g, const float *__restrict__ b, TAct *__restrict__ out,
          int64_t rows, int d, float eps, const int32_t *__restrict__ seq_end = nullptr, int64_t base = 0,
          int64_t src_rows = 0, const float *__restrict__ part = nullptr, int nsplit = 0, int64_t part_stride = 0,
          const TAct *__restrict__ add_act = nullptr, int *advance_ctr = nullptr)
{
    if (GATHER && advance_ctr && blockIdx.x == 0 && threadIdx.x == 0) {
        advance_ctr[0] += 1;
        advance_ctr[1] += 1;
    }
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;

    float4 v[VPL];
    // up to 4 vectors per lane the gain and bias are requested together with the row, so that their latency
    // does not follow the two reductions (wider rows would need too many registers for that)
    constexpr bool kEarlyParams = VPL <= 4;
    float4 pg[kEarlyParams ? VPL : 1], pb[kEarlyParams ? VPL : 1];
    float sum = 0.0f;
    const TW *erow = nullptr;
    int64_t src = row;
    if (!GATHER && seq_end) src = min(max((int64_t)seq_end[row + 1] - 1 - base, (int64_t)0), src_rows - 1);
    if constexpr (GATHER) {
        int t = tok[row];
        t = min(max(t, 0), vocab - 1);          // never read outside the table
        erow = embed + (size_t)t * d;
    }
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
        const int c = (i * 64 + lane) * 4;
        if (c < d) {
            if constexpr (kEarlyParams) {
                pg[i] = load4(g + c);
                pb[i] = load4(b + c);
            }
            if constexpr (GATHER) {
                v[i] = load4(erow + c);
                store4(x_out + row * d + c, v[i]);
            } else {
                v[i] = load4(x_in + src * in_stride + c);
                if (part) {
                    // four slabs requested at a time (a load per iteration would serialise their latencies), eight
                    // when there are more than four (the slabs of two projections: a second round trip saved);
                    // the sums are still formed in slab order
                    auto add_slabs = [&](auto width) {
                        constexpr int W = decltype(width)::value;
                        for (int s0 = 0; s0 < nsplit; s0 += W) {
                            float4 t[W];
#pragma unroll
                            for (int j = 0; j < W; ++j)
                                t[j] = load4(part + (int64_t)min(s0 + j, nsplit - 1) * part_stride + row * d + c);
#pragma unroll
                            for (int j = 0; j < W; ++j)
                                if (s0 + j < nsplit) { v[i].x += t[j].x; v[i].y += t[j].y; v[i].z += t[j].z; v[i].w += t[j].w; }
                        }
                    };
                    if (nsplit > 4) add_slabs(std::integral_constant<int, 8>{});
                    else add_slabs(std::integral_constant<int, 4>{});
                    store4(x_out + row * d + c, v[i]);
                }
                if (add_act) {
                    const float4 t = load4(add_act + row * d + c);
                    v[i].x += t.x; v[i].y += t.y; v[i].z += t.z; v[i].w += t.w;
                    store4(x_out + row * d + c, v[i]);
                }
            }
            sum += (v[i].x + v[i].y) + (v[i].z + v[i].w);
        } else {
            v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    const float mean = wave_sum(sum) / (float)d;
    float sq = 0.0f;
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
        const int c = (i * 64 + lane) * 4;
        if (c < d) {
            const float a = v[i].x - mean, bb = v[i].y - mean, cc = v[i].z - mean, dd = v[i].w - mean;
            sq += (a * a + bb * bb) + (cc * cc + dd * dd);
        }
    }
    const float var = wave_sum(sq) / (float)d;
    const float rstd = 1.0f / sqrtf(var + eps);
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
        const int c = (i * 64 + lane) * 4;
        if (c < d) {
            float4 gg, bb;
            if constexpr (kEarlyParams) { gg = pg[i]; bb = pb[i]; }
            else { gg = load4(g + c); bb = load4(b + c); }
            float4 o;
            o.x = (v[i].x - mean) * rstd * gg.x + bb.x;
            o.y = (v[i].y - mean) * rstd * gg.y + bb.y;
            o.z = (v[i].z - mean) * rstd * gg.z + bb.z;
            o.w = (v[i].w - mean) * rstd * gg.w + bb.w;
            store4(out + row * d + c, o);
        }
    }
}

// Plain LayerNorm (x -> out in the activation type) for large row counts: one
// wavefront normalises RPW rows, with the loads of all of them issued before the
// first reduction, so more bytes are in flight per wavefront (measured at 16384
// rows of 1024: 21.6 us per launch with one row per wavefront, 18.2 with two,
// 20.1 with four).  Same arithmetic, in the same order per row, as ln_kernel.
template <typename TAct, int VPL, int RPW>
__global__ void __launch_bounds__(256)
ln_rows_kernel(const float *__restrict__ x, const float *__restrict__ g, const float *__restrict__ b,
               TAct *__restrict__ out, int64_t rows, int d, float eps)
{
    const int lane = threadIdx.x & 63;
    const int64_t row0 = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * RPW;
    if (row0 >= rows) return;
    float4 v[RPW][VPL];
#pragma unroll
    for (int r = 0; r < RPW; ++r)
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const int c = (i * 64 + lane) * 4;
            if (c < d && row0 + r < rows) {
                // (ordinary loads: x was written by the kernel just before and is still in the caches; with the
                // streaming hint the C4 step measured 1 % slower)
                const f32x4_t t4 = *reinterpret_cast<const f32x4_t *>(x + (row0 + r) * d + c);
                v[r][i] = make_float4(t4[0], t4[1], t4[2], t4[3]);
            } else {
                v[r][i] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        if (row0 + r >= rows) break;
        float sum = 0.0f;
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const int c = (i * 64 + lane) * 4;
            if (c < d) sum += (v[r][i].x + v[r][i].y) + (v[r][i].z + v[r][i].w);
        }
        const float mean = wave_sum(sum) / (float)d;
        float sq = 0.0f;
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const int c = (i * 64 + lane) * 4;
            if (c < d) {
                const float a = v[r][i].x - mean, bb = v[r][i].y - mean, cc = v[r][i].z - mean, dd = v[r][i].w - mean;
                sq += (a * a + bb * bb) + (cc * cc + dd * dd);
            }
        }
        const float rstd = 1.0f / sqrtf(wave_sum(sq) / (float)d + eps);
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const int c = (i * 64 + lane) * 4;
            if (c < d) {
                const float4 gg = load4(g + c), bb = load4(b + c);
                float4 o;
                o.x = (v[r][i].x - mean) * rstd * gg.x + bb.x;
                o.y = (v[r][i].y - mean) * rstd * gg.y + bb.y;
                o.z = (v[r][i].z - mean) * rstd * gg.z + bb.z;
                o.w = (v[r][i].w - mean) * rstd * gg.w + bb.w;
                store4(out + (row0 + r) * d + c, o);
            }
        }
    }
}
