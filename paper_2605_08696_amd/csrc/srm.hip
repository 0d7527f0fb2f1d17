// libsrm: C ABI and step scheduler for SRM generation on gfx950.
// The exported calls are declared and documented in include/srm.h.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "srm.h"
#include "gemm.hpp"
#include "gemm_persist.hpp"
#include "mega.hpp"
#include "mixer.hpp"
#include "norm.hpp"
#include "probe.hpp"
#include "sample.hpp"
#include "tokmix.hpp"

// ------------------------------------------------------------------ errors
static thread_local std::string g_err;

static int fail(int code, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

#define HIP_TRY(expr)                                                                       \
    do {                                                                                    \
        hipError_t e_ = (expr);                                                             \
        if (e_ != hipSuccess)                                                               \
            return fail(SRM_EHIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_),    \
                        __FILE__, __LINE__);                                                \
    } while (0)

#define SRM_TRY(expr)                 \
    do {                              \
        int rc_ = (expr);             \
        if (rc_ != SRM_OK) return rc_; \
    } while (0)

static inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ------------------------------------------------------------------ model
struct LayerDev {
    const float *ln1_g, *ln1_b, *b_in, *alpha, *beta, *lam, *b_out, *ln2_g, *ln2_b, *b_up, *b_down;
    const void *w_in, *w_out, *w_up, *w_down;
};

struct srm_model {
    srm_config cfg;
    int device;
    int d, ff, V, L, H;
    // The mixer's own geometry: row width dm, Hs heads of which the first hrow are row-repeat.
    // Mixed, row-only and column-only layouts: dm = d, Hs = H.  Combined heads (one row-repeat
    // and one column-repeat matrix per head, outputs added) run as a mixer of width 2d with 2H
    // heads, the H row-repeat ones first: the in-projection's rows and the out-projection's
    // columns are stored twice, so that both halves see the same input and the out-projection
    // adds their outputs.  A mixer with k filters along the hidden dimension (Eq. 11) runs the
    // same way with k copies, all column-repeat, copy i of the in-projection shifted by i rows.
    int dm, Hs, hrow;
    bool noproj;           // non-projected mixer layers
    bool shalf;            // recurrent state (and lambda) in binary16
    size_t ssize;          // bytes per state element
    size_t wsize;          // bytes per matrix element
    void *slab;
    MegaLayer *mega_layers;   // device copy of the layers' pointers for the one-kernel small-batch path, or null
    const void *embed, *head;
    const float *lnf_g, *lnf_b;
    std::vector<LayerDev> layers;
    // cached graph of one decode step for srm_generate (see there)
    hipGraphExec_t gexec;
    struct { int64_t B; const void *tok, *state, *store, *ws; float temp; uint32_t seed; float top_p; const void *logits; size_t ws_bytes; const void *pos; int eos_plus1; } gkey;
};

static uint16_t host_f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);   // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

namespace {
struct SlabBuilder {
    std::vector<unsigned char> host;
    size_t add(const float *src, size_t n, bool as_bf16)
    {
        size_t off = align_up(host.size(), 256);
        size_t bytes = n * (as_bf16 ? 2 : 4);
        host.resize(off + bytes);
        if (as_bf16) {
            uint16_t *dst = reinterpret_cast<uint16_t *>(host.data() + off);
            for (size_t i = 0; i < n; ++i) dst[i] = host_f32_to_bf16(src[i]);
        } else {
            memcpy(host.data() + off, src, bytes);
        }
        return off;
    }
};
}  // namespace

extern "C" const char *srm_last_error(void) { return g_err.c_str(); }

// Checks a configuration and fills the sizes derived from it (no device work): what srm_init_weights
// starts with, and all that the host-side planning queries need of a model.
static int model_geometry(const char *who, const srm_config *cfg, srm_model *m)
{
    if (cfg->vocab <= 0 || cfg->d_model <= 0 || cfg->n_layers <= 0 || cfg->n_heads <= 0 ||
        cfg->mlp_expansion <= 0 || cfg->n_ctx <= 0)
        return fail(SRM_EINVAL, "%s: sizes must be positive", who);
    const int layout = cfg->head_layout;
    if (layout < SRM_HEADS_MIXED || layout > SRM_HEADS_COMBINED)
        return fail(SRM_EINVAL, "%s: unknown head_layout %d", who, layout);
    const int kmix = cfg->mixer_kernel > 1 ? cfg->mixer_kernel : 1;
    if (cfg->mixer_kernel < 0 || kmix > cfg->d_model)
        return fail(SRM_EINVAL, "%s: mixer_kernel %d outside [0, d_model]", who, cfg->mixer_kernel);
    if (kmix > 1 && (layout != SRM_HEADS_COLUMN || cfg->no_projections))
        return fail(SRM_EINVAL, "%s: mixer_kernel > 1 needs column-repeat heads and the head projections", who);
    const int slots = cfg->n_heads * (kmix > 1 ? kmix : layout == SRM_HEADS_COMBINED ? 2 : 1);
    if ((layout == SRM_HEADS_MIXED && cfg->n_heads % 2) || slots > kMaxHeads)
        return fail(SRM_EINVAL, "%s: n_heads must be even for mixed heads, and at most %d "
                                "coefficient rows per layer", who, kMaxHeads);
    if (layout == SRM_HEADS_COMBINED && cfg->no_projections)
        return fail(SRM_EINVAL, "%s: combined heads need the head projections", who);
    if (cfg->d_model % (4 * cfg->n_heads))
        return fail(SRM_EINVAL, "%s: d_model must be a multiple of 4*n_heads", who);
    if (cfg->d_model > 4096) return fail(SRM_EINVAL, "%s: d_model > 4096 unsupported", who);
    if (cfg->weight_dtype != SRM_FP32 && cfg->weight_dtype != SRM_BF16)
        return fail(SRM_EINVAL, "%s: unknown weight_dtype %d", who, cfg->weight_dtype);
    if (cfg->weight_dtype == SRM_BF16 && cfg->d_model % 64)
        return fail(SRM_EINVAL, "%s: bf16 needs d_model %% 64 == 0", who);
    if (!(cfg->ln_eps > 0.0f)) return fail(SRM_EINVAL, "%s: ln_eps must be > 0", who);
    if (cfg->state_dtype != SRM_FP32 && cfg->state_dtype != SRM_FP16)
        return fail(SRM_EINVAL, "%s: unknown state_dtype %d", who, cfg->state_dtype);
    m->cfg = *cfg;
    m->device = -1;
    m->d = cfg->d_model; m->ff = cfg->mlp_expansion * cfg->d_model; m->V = cfg->vocab; m->L = cfg->n_layers;
    m->H = cfg->n_heads;
    const int copies = kmix > 1 ? kmix : layout == SRM_HEADS_COMBINED ? 2 : 1;   // times the mixer row repeats the head input
    m->dm = copies * m->d;
    m->Hs = slots;
    m->hrow = layout == SRM_HEADS_MIXED ? m->H / 2 : layout == SRM_HEADS_COLUMN ? 0 : m->H;
    m->noproj = cfg->no_projections != 0;
    m->shalf = cfg->state_dtype == SRM_FP16;
    m->ssize = m->shalf ? 2 : 4;
    m->wsize = cfg->weight_dtype == SRM_BF16 ? 2 : 4;
    m->slab = nullptr;
    m->mega_layers = nullptr;
    m->gexec = nullptr;
    m->gkey = {0, nullptr, nullptr, nullptr, nullptr, 0.0f, 0, 1.0f, nullptr, 0, nullptr, 0};
    return SRM_OK;
}

extern "C" int srm_init_weights(const srm_config *cfg, const srm_host_weights *w, srm_model **out)
{
    if (!cfg || !w || !out) return fail(SRM_EINVAL, "srm_init_weights: null argument");
    *out = nullptr;
    srm_model *m = new (std::nothrow) srm_model();
    if (!m) return fail(SRM_ENOMEM, "srm_init_weights: host allocation failed");
    const int grc = model_geometry("srm_init_weights", cfg, m);
    if (grc != SRM_OK) { delete m; return grc; }
    if (!w->embed || !w->head || !w->lnf_g || !w->lnf_b || !w->layers) {
        delete m;
        return fail(SRM_EINVAL, "srm_init_weights: null weight pointer");
    }
    const int d = m->d, L = m->L, H = m->H, V = m->V;
    const int layout = cfg->head_layout;
    const int kmix = cfg->mixer_kernel > 1 ? cfg->mixer_kernel : 1;
    const int slots = m->Hs, copies = m->dm / d;
    const bool comb = layout == SRM_HEADS_COMBINED;
    (void)comb;
    const bool bf = cfg->weight_dtype == SRM_BF16;
    const size_t ff = (size_t)m->ff, nc = cfg->n_ctx;
    for (int l = 0; l < L; ++l) {
        const srm_host_layer &y = w->layers[l];
        const float *ptrs[] = {y.ln1_g, y.ln1_b, y.alpha, y.beta, y.lambda, y.ln2_g, y.ln2_b, y.w_up, y.b_up,
                               y.w_down, y.b_down};
        for (const float *p : ptrs)
            if (!p) { delete m; return fail(SRM_EINVAL, "srm_init_weights: null weight pointer in layer %d", l); }
        if (!cfg->no_projections && (!y.w_in || !y.b_in || !y.w_out || !y.b_out)) {
            delete m;
            return fail(SRM_EINVAL, "srm_init_weights: null projection weights in layer %d", l);
        }
        for (int h = 0; h < slots; ++h)
            if (!(y.lambda[h] > 0.0f && y.lambda[h] <= 1.0f)) {
                delete m;
                return fail(SRM_EINVAL, "srm_init_weights: lambda[%d][%d] = %g outside (0, 1]", l, h,
                            (double)y.lambda[h]);
            }
    }

    struct Offs { size_t v[15]; };
    std::vector<Offs> lo(L);
    size_t o_embed, o_head, o_lnfg, o_lnfb;
    SlabBuilder sb;
    try {
        o_embed = sb.add(w->embed, (size_t)V * d, bf);
        o_head = sb.add(w->head, (size_t)V * d, bf);
        o_lnfg = sb.add(w->lnf_g, d, false);
        o_lnfb = sb.add(w->lnf_b, d, false);
        for (int l = 0; l < L; ++l) {
            const srm_host_layer &y = w->layers[l];
            size_t *o = lo[l].v;
            o[0] = sb.add(y.ln1_g, d, false);          o[1] = sb.add(y.ln1_b, d, false);
            const bool pj = !m->noproj;
            if (copies > 1) {
                // W_in [d][d] -> [copies*d][d], W_out [d][d] -> [d][copies*d] (columns repeated).  Copy i of
                // W_in / b_in holds rows i .. d-1 followed by i zero rows (combined heads: no shift), so that
                // mixer channel i*d + c receives head input c + i, or zero past the last channel (Eq. 11).
                std::vector<float> t((size_t)copies * d * d, 0.0f), tb((size_t)copies * d, 0.0f);
                for (int i = 0; i < copies; ++i) {
                    const int sh = kmix > 1 ? i : 0;
                    memcpy(t.data() + (size_t)i * d * d, y.w_in + (size_t)sh * d, (size_t)(d - sh) * d * 4);
                    memcpy(tb.data() + (size_t)i * d, y.b_in + sh, (size_t)(d - sh) * 4);
                }
                o[2] = sb.add(t.data(), t.size(), bf);
                o[3] = sb.add(tb.data(), tb.size(), false);
            } else {
                o[2] = pj ? sb.add(y.w_in, (size_t)d * d, bf) : 0;   o[3] = pj ? sb.add(y.b_in, d, false) : 0;
            }
            o[4] = sb.add(y.alpha, slots * nc, false);
            if (kmix > 1) {                              // beta [H][n_ctx] is added once: rows of filter 0, zeros after
                std::vector<float> t((size_t)slots * nc, 0.0f);
                memcpy(t.data(), y.beta, (size_t)H * nc * 4);
                o[5] = sb.add(t.data(), t.size(), false);
            } else {
                o[5] = sb.add(y.beta, slots * nc, false);
            }
            if (m->shalf) {                              // decay constants as binary16 values
                float lh[kMaxHeads];
                for (int h = 0; h < slots; ++h) lh[h] = (float)(_Float16)y.lambda[h];
                o[6] = sb.add(lh, slots, false);
            } else {
                o[6] = sb.add(y.lambda, slots, false);
            }
            if (copies > 1) {
                std::vector<float> t((size_t)copies * d * d);
                for (int i = 0; i < d; ++i)
                    for (int c = 0; c < copies; ++c)
                        memcpy(t.data() + ((size_t)i * copies + c) * d, y.w_out + (size_t)i * d, (size_t)d * 4);
                o[7] = sb.add(t.data(), t.size(), bf);
                o[8] = sb.add(y.b_out, d, false);
            } else {
                o[7] = pj ? sb.add(y.w_out, (size_t)d * d, bf) : 0;  o[8] = pj ? sb.add(y.b_out, d, false) : 0;
            }
            o[9] = sb.add(y.ln2_g, d, false);           o[10] = sb.add(y.ln2_b, d, false);
            o[11] = sb.add(y.w_up, ff * d, bf);         o[12] = sb.add(y.b_up, ff, false);
            o[13] = sb.add(y.w_down, (size_t)d * ff, bf); o[14] = sb.add(y.b_down, d, false);
        }
    } catch (const std::bad_alloc &) {
        delete m;
        return fail(SRM_ENOMEM, "srm_init_weights: host staging allocation failed");
    }
    hipError_t e = hipGetDevice(&m->device);
    if (e == hipSuccess) e = hipMalloc(&m->slab, align_up(sb.host.size(), 256));
    if (e != hipSuccess) {
        delete m;
        return fail(e == hipErrorOutOfMemory ? SRM_ENOMEM : SRM_EHIP, "srm_init_weights: hipMalloc(%zu): %s",
                    sb.host.size(), hipGetErrorString(e));
    }
    e = hipMemcpy(m->slab, sb.host.data(), sb.host.size(), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        (void)hipFree(m->slab);
        delete m;
        return fail(SRM_EHIP, "srm_init_weights: hipMemcpy: %s", hipGetErrorString(e));
    }
    const unsigned char *base = static_cast<const unsigned char *>(m->slab);
    auto F = [&](size_t off) { return reinterpret_cast<const float *>(base + off); };
    m->embed = base + o_embed; m->head = base + o_head;
    m->lnf_g = F(o_lnfg); m->lnf_b = F(o_lnfb);
    m->layers.resize(L);
    for (int l = 0; l < L; ++l) {
        const size_t *o = lo[l].v;
        LayerDev &y = m->layers[l];
        y.ln1_g = F(o[0]); y.ln1_b = F(o[1]); y.w_in = base + o[2]; y.b_in = F(o[3]);
        y.alpha = F(o[4]); y.beta = F(o[5]); y.lam = F(o[6]); y.w_out = base + o[7];
        y.b_out = F(o[8]); y.ln2_g = F(o[9]); y.ln2_b = F(o[10]); y.w_up = base + o[11];
        y.b_up = F(o[12]); y.w_down = base + o[13]; y.b_down = F(o[14]);
    }
    if (!bf && !m->noproj) {
        std::vector<MegaLayer> ml(L);
        for (int l = 0; l < L; ++l) {
            const LayerDev &y = m->layers[l];
            ml[l] = MegaLayer{y.ln1_g, y.ln1_b, static_cast<const float *>(y.w_in), y.b_in, y.alpha, y.beta, y.lam,
                              static_cast<const float *>(y.w_out), y.b_out, y.ln2_g, y.ln2_b,
                              static_cast<const float *>(y.w_up), y.b_up, static_cast<const float *>(y.w_down), y.b_down};
        }
        e = hipMalloc(reinterpret_cast<void **>(&m->mega_layers), sizeof(MegaLayer) * L);
        if (e == hipSuccess) e = hipMemcpy(m->mega_layers, ml.data(), sizeof(MegaLayer) * L, hipMemcpyHostToDevice);
        if (e != hipSuccess) {
            if (m->mega_layers) (void)hipFree(m->mega_layers);
            (void)hipFree(m->slab);
            delete m;
            return fail(SRM_EHIP, "srm_init_weights: layer table: %s", hipGetErrorString(e));
        }
    }
    *out = m;
    return SRM_OK;
}

extern "C" void srm_free(srm_model *m)
{
    if (!m) return;
    if (m->gexec) (void)hipGraphExecDestroy(m->gexec);
    if (m->mega_layers) (void)hipFree(m->mega_layers);
    if (m->slab) (void)hipFree(m->slab);
    delete m;
}

extern "C" size_t srm_state_bytes(const srm_model *m, int64_t batch)
{
    if (!m || batch <= 0) return 0;
    return (size_t)m->L * (size_t)batch * (size_t)m->dm * m->ssize;
}

// Layer l's [B][dm] slab of a state array.
static void *layer_state(const srm_model *m, void *state, int l, int64_t B)
{
    return static_cast<unsigned char *>(state) + (size_t)l * (size_t)B * (size_t)m->dm * m->ssize;
}

// ------------------------------------------------------------------ workspace
// Column-tile width that bounds the number of argmax partials per row.
static int head_min_bn(const srm_model *m) { return m->cfg.weight_dtype == SRM_BF16 ? 128 : 64; }

struct Workspace {
    float *x;          // [rows][d]  residual stream
    void *a;           // [rows][d]  activation type
    void *u, *mx;      // [rows][dm] activation type: mixer input and output
    void *g;           // [rows][ff] activation type
    float *pv;         // [rows][nparts]
    int32_t *pi;       // [rows][nparts]
    int *ctr;          // [2] position and step counters of srm_generate
    int *slow;         // [64 + rows] nucleus pass: count, then (from slow + 64) the rows that need the search
    unsigned char *mega;  // [kMegaScratch] one-kernel small-batch path: partial winners and the barrier words
    float *part;       // [slices][rows][d] split-K slabs of a residual projection (rows <= kSplitMaxRows), else null
    size_t bytes;
};

// Split-K of the MLP down projection for small batches: with few token rows the
// GEMM has too few tiles to fill the chip and a long serial k loop, so K is cut
// into kSplitK slices whose fp32 slabs the following LayerNorm kernel adds to the
// residual stream (in slab order: deterministic).
constexpr int kSplitK = 4;
constexpr int64_t kSplitMaxRows = 2048;
// fp32 models with at most kGemvRows rows run their projections as GEMVs, whose grid is only
// N / 64 blocks: the two residual projections are cut into up to kGemvSplitMax K slices the same way.
constexpr int kGemvSplitMax = 8;
constexpr int64_t kGemvRows = 32;

// Scratch of the one-kernel path: [kMegaMaxBlocks][kMegaMaxB] floats, the same of ints, then the barrier's
// 64-byte slots (one per work-group) and its give-up flag.
constexpr size_t kMegaScratch = (size_t)kMegaMaxBlocks * kMegaMaxB * 8 + (size_t)kMegaMaxBlocks * 64 + 256;

static Workspace carve(const srm_model *m, void *base, int64_t rows)
{
    Workspace w;
    unsigned char *p = static_cast<unsigned char *>(base);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        unsigned char *r = p ? p + off : nullptr;
        off += align_up(bytes, 256);
        return r;
    };
    const size_t r = (size_t)rows, d = m->d, dm = m->dm, s = m->wsize;
    const size_t nparts = cdiv(m->V, head_min_bn(m));
    w.x = reinterpret_cast<float *>(take(r * d * 4));
    w.a = take(r * d * s);
    w.u = m->noproj ? w.a : take(r * dm * s);     // without projections the mixer reads the LayerNorm output
    w.mx = take(r * dm * s);
    w.g = take(r * (size_t)m->ff * s);
    w.pv = reinterpret_cast<float *>(take(r * nparts * 4));
    w.pi = reinterpret_cast<int32_t *>(take(r * nparts * 4));
    w.slow = reinterpret_cast<int *>(take(256 + r * 4));
    // sized so that the workspace grows monotonically with the row count
    // (twice kSplitK slabs: the one-kernel token mixing writes its out-projection slabs behind the MLP's)
    const size_t part_rows = std::max<size_t>((size_t)2 * kSplitK * std::min<int64_t>(rows, kSplitMaxRows),
                                              (size_t)kGemvSplitMax * std::min<int64_t>(rows, kGemvRows));
    float *part = reinterpret_cast<float *>(take(part_rows * d * 4));
    w.part = rows <= kSplitMaxRows ? part : nullptr;
    w.mega = take(kMegaScratch);
    w.ctr = reinterpret_cast<int *>(take(256));
    w.bytes = off;
    return w;
}

extern "C" size_t srm_workspace_bytes(const srm_model *m, int64_t rows)
{
    if (!m || rows <= 0) return 0;
    return carve(m, nullptr, rows).bytes;
}

// ------------------------------------------------------------------ launchers
template <int BM, int BN, int WM, int WN, int EPI, typename TAct, int NS = 2>
static int launch_bf16_tile(const bf16 *A, const bf16 *W, int M, int N, int K, const GemmEpi &ep, hipStream_t st,
                            int ksplit = 1)
{
    constexpr size_t smem = (size_t)NS * (BM + BN) * 64 * sizeof(bf16);
    auto kern = gemm_bf16_kernel<BM, BN, WM, WN, EPI, TAct, NS>;
    static bool attr_set = false;
    if (!attr_set) {
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
        attr_set = true;
    }
    const int64_t nb = cdiv(M, BM) * cdiv(N, BN);
    hipLaunchKernelGGL(kern, dim3((unsigned)nb, (unsigned)ksplit), dim3(WM * WN * 64), smem, st, A, W, M, N, K, ep);
    HIP_TRY(hipGetLastError());
    return SRM_OK;
}

// The 256x256 tile as a persistent kernel (gemm_persist.hpp): one work-group per CU, for launches of more
// tiles than CUs.  It needs an even number >= 4 of k tiles and whole float4 groups of bias per column tile.
static bool persist_ok(int64_t M, int N, int K)
{
    return K % 128 == 0 && K >= 256 && (N & 3) == 0 && cdiv(M, 256) * cdiv(N, 256) < (1 << 30);
}
static int device_cus()
{
    static thread_local int dev_of = -1, cus_of = 0;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (dev != dev_of) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        dev_of = dev;
        cus_of = cus;
    }
    return cus_of;
}
template <int EPI, typename TAct, bool RING = false>
static int launch_bf16_persist(const bf16 *A, const bf16 *W, int M, int N, int K, const GemmEpi &ep, hipStream_t st)
{
    // (the argmax epilogue that stores no logits needs no stage in LDS: the ring runs through)
    if constexpr (EPI == EPI_ARGMAX && !RING)
        if (!ep.out) return launch_bf16_persist<EPI, TAct, true>(A, W, M, N, K, ep, st);
    auto kern = gemm_bf16_persist_kernel<EPI, TAct, RING>;
    static bool attr_set = false;
    if (!attr_set) {
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kPersistLds));
        attr_set = true;
    }
    const int cus = device_cus();
    if (cus <= 0) return fail(SRM_EHIP, "cannot read the number of compute units");
    const int64_t nb = cdiv(M, 256) * cdiv(N, 256);
    hipLaunchKernelGGL(kern, dim3((unsigned)std::min<int64_t>(nb, cus)), dim3(512), kPersistLds, st, A, W, M, N, K, ep);
    HIP_TRY(hipGetLastError());
    return SRM_OK;
}

// A handful of rows, LayerNorm made by the GEMM itself (see the LNA note in gemm.hpp): one row tile of 64x64
// blocks, the normalised rows as a [K / 64][32][64] bf16 panel in LDS next to an eight-tile ring for W.
template <int EPI>
static int launch_bf16_lna(const bf16 *W, int M, int N, int K, const GemmEpi &ep, hipStream_t st)
{
    constexpr int NS = 8;
    const size_t smem = (size_t)K * 64 + (size_t)NS * 64 * 64 * sizeof(bf16);
    auto kern = gemm_bf16_kernel<64, 64, 2, 2, EPI, bf16, NS, true>;
    static bool attr_set = false;
    if (!attr_set) {
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    1024 * 64 + NS * 64 * 64 * (int)sizeof(bf16)));
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)cdiv(N, 64), 1), dim3(256), smem, st, W /*A: unused*/, W, M, N, K, ep);
    HIP_TRY(hipGetLastError());
    return SRM_OK;
}
static bool lna_ok(int64_t M, int K) { return M <= kLnaRows && K <= 1024 && K % 64 == 0; }

// Few rows: the streaming GEMV (gemv_rows_kernel), 16 * CPG columns per block.
constexpr int kGemvMB = 8;                 // rows per pass over W
constexpr size_t kGemvMaxLds = 128 * 1024;
template <typename TW, typename TAct, int EPI, int CPG>
static int launch_gemv_rows(const TAct *A, const TW *W, int M, int N, int K, GemmEpi ep, hipStream_t st, int ksplit,
                            int *nparts_out)
{
    const size_t lds = (size_t)kGemvMB * (K / ksplit) * sizeof(float);
    auto kern = gemv_rows_kernel<TW, TAct, EPI, kGemvMB, CPG>;
    static bool attr_set = false;
    if (!attr_set) {
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)kGemvMaxLds));
        attr_set = true;
    }
    ep.nparts = (int)cdiv(N, 16 * CPG);
    if (nparts_out) *nparts_out = ep.nparts;
    hipLaunchKernelGGL(kern, dim3((unsigned)ep.nparts, (unsigned)ksplit), dim3(256), lds, st, A, W, M, N, K, ep);
    HIP_TRY(hipGetLastError());
    return SRM_OK;
}
// whether the streaming GEMV applies: few rows, whole 16-byte weight vectors per K slice, the rows' stage within LDS
template <typename TW>
static bool gemv_rows_ok(int64_t M, int K, int ksplit, int64_t max_rows)
{
    const int vw = 16 / (int)sizeof(TW);
    return M <= max_rows && K % (vw * ksplit) == 0 && (size_t)kGemvMB * (K / ksplit) * sizeof(float) <= kGemvMaxLds;
}

// The 64x64 tile with few blocks on the chip: its k loop is bound by the latency of the tile loads, so
// the LDS ring is deepened as far as the blocks per CU allow (8 stages = 128 KB: one block per CU;
// 4 stages = 64 KB: two).
template <int EPI, typename TAct>
static int launch_bf16_small(const bf16 *A, const bf16 *W, int M, int N, int K, const GemmEpi &ep, hipStream_t st,
                             int ksplit)
{
    const int64_t blocks = cdiv(M, 64) * cdiv(N, 64) * ksplit;
    const int kt = K / ksplit / 64;
    if (blocks <= 256 && kt > 4) return launch_bf16_tile<64, 64, 2, 2, EPI, TAct, 8>(A, W, M, N, K, ep, st, ksplit);
    if (blocks <= 512 && kt > 2) return launch_bf16_tile<64, 64, 2, 2, EPI, TAct, 4>(A, W, M, N, K, ep, st, ksplit);
    return launch_bf16_tile<64, 64, 2, 2, EPI, TAct>(A, W, M, N, K, ep, st, ksplit);
}

// Tile codes of the bf16 GEMM: 0 = 256x256 (8 waves), 1 = 128x128 (4 waves),
// 2 = 64x64 (4 waves), 3 = 128x128 (8 waves), 4 = 256x128 (8 waves); 5 .. 8 pin the
// ring depth of a tile for sweeps, 9 / 10 pin the persistent / one-tile-per-work-group form of 256x256.  min_bn > 64 rules out the 64-wide tile (the LM
// head's partial buffers are sized for column tiles >= 128).  Measured on C4's
// shapes over 512 .. 16384 rows: the big tile wins once it fills most of the chip in
// whole rounds (one block per CU: 384 tiles are two rounds at 75 %, and lose to 1536
// tiles of 128x128); 128x128 wins over 64x64 from about 144 blocks on.
constexpr int kNumTiles = 11;
static int choose_tile(int64_t M, int N, int K, int min_bn)
{
    const int64_t t256 = cdiv(M, 256) * cdiv(N, 256), t128 = cdiv(M, 128) * cdiv(N, 128);
    int tile;
    // (a long k loop makes up for CUs left idle: with K >= 2048 the big tile wins from 160 tiles on)
    const int64_t t256_min = K >= 2048 ? 160 : 200;
    if (t256 >= t256_min && (t256 >= 1024 || t256 < 256 || (double)t256 / (double)(cdiv(t256, 256) * 256) >= 0.8)) tile = 0;
    else if (t128 >= 144) tile = 1;
    else tile = 2;
    if (tile == 2 && min_bn > 64) tile = 1;
    return tile;
}
static int tile_bn(int tile) { return tile == 0 || tile >= 9 ? 256 : (tile == 2 || tile >= 6) ? 64 : 128; }

static thread_local int g_force_tile = -1;   // test/bench hook of srm_linear only
static thread_local unsigned long long *g_clock_probe = nullptr;   // measuring hook of srm_linear only
static thread_local int64_t g_clock_blocks = 0;

template <int EPI, typename TAct>
static int launch_bf16(const bf16 *A, const bf16 *W, int64_t M, int N, int K, GemmEpi ep, hipStream_t st,
                       int min_bn, int *nparts_out, int ksplit = 1)
{
    if (K % 64) return fail(SRM_EINVAL, "bf16 GEMM needs K %% 64 == 0 (K = %d)", K);
    if (ksplit > 1) {
        // slices of whole 64-wide k tiles, fp32 slabs, small tiles (the point is to fill the chip)
        if (EPI != EPI_F32 || K % (64 * ksplit)) return fail(SRM_EINVAL, "bf16 GEMM: bad split of K = %d", K);
        if (M <= 0 || M >= (1 << 30) || N <= 0) return fail(SRM_EINVAL, "GEMM shape out of range");
        ep.nparts = 0;
        return launch_bf16_small<EPI, TAct>(A, W, (int)M, N, K, ep, st, ksplit);
    }
    if (M <= 0 || M >= (1 << 30) || N <= 0) return fail(SRM_EINVAL, "GEMM shape out of range");
    if ((int64_t)K * 256 * 2 >= (1LL << 31)) return fail(SRM_EINVAL, "bf16 GEMM: K = %d too large", K);
    const int tile = g_force_tile >= 0 ? g_force_tile : choose_tile(M, N, K, min_bn);
    ep.nparts = (int)cdiv(N, tile_bn(tile));
    if (nparts_out) *nparts_out = ep.nparts;
    const int m = (int)M;
    switch (tile) {
    case 0:
        // more tiles than CUs: the persistent form, whose tiles after a CU's first start without a launch and
        // a cold first load (measured on C4's shapes: MLP-up -1 .. -4 %, LM head -2 %)
        if (persist_ok(M, N, K) && cdiv(M, 256) * cdiv(N, 256) > device_cus())
            return launch_bf16_persist<EPI, TAct>(A, W, m, N, K, ep, st);
        return launch_bf16_tile<256, 256, 2, 4, EPI, TAct>(A, W, m, N, K, ep, st);
    case 1:
        // at most one block per CU: the k loop is bound by the latency of its tile loads (a 128x128x64 tile is
        // 0.27 us of MFMAs, a load about 1 us), so the LDS ring is deepened to keep three tiles in flight
        if (cdiv(M, 128) * cdiv(N, 128) <= 256 && K / 64 > 4)
            return launch_bf16_tile<128, 128, 2, 2, EPI, TAct, 4>(A, W, m, N, K, ep, st);
        return launch_bf16_tile<128, 128, 2, 2, EPI, TAct>(A, W, m, N, K, ep, st);
    case 2: return launch_bf16_small<EPI, TAct>(A, W, m, N, K, ep, st, 1);
    case 3: return launch_bf16_tile<128, 128, 2, 4, EPI, TAct>(A, W, m, N, K, ep, st);
    case 4: return launch_bf16_tile<256, 128, 4, 2, EPI, TAct>(A, W, m, N, K, ep, st);
    // sweeps only: a fixed ring depth
    case 5: return launch_bf16_tile<128, 128, 2, 2, EPI, TAct, 4>(A, W, m, N, K, ep, st);
    case 6: return launch_bf16_tile<64, 64, 2, 2, EPI, TAct, 2>(A, W, m, N, K, ep, st);
    case 7: return launch_bf16_tile<64, 64, 2, 2, EPI, TAct, 4>(A, W, m, N, K, ep, st);
    case 8: return launch_bf16_tile<64, 64, 2, 2, EPI, TAct, 8>(A, W, m, N, K, ep, st);
    case 9:
        if (!persist_ok(M, N, K)) return fail(SRM_EINVAL, "the persistent GEMM does not take this shape");
        return launch_bf16_persist<EPI, TAct>(A, W, m, N, K, ep, st);
    case 10: return launch_bf16_tile<256, 256, 2, 4, EPI, TAct>(A, W, m, N, K, ep, st);
    default: return fail(SRM_EINVAL, "unknown GEMM tile code %d", tile);
    }
}

template <int EPI>
static int launch_f32(const float *A, const float *W, int64_t M, int N, int K, GemmEpi ep, hipStream_t st,
                      int *nparts_out, int ksplit = 1)
{
    if (M <= 0 || M >= (1 << 30) || N <= 0 || K <= 0) return fail(SRM_EINVAL, "GEMM shape out of range");
    ep.nparts = (int)cdiv(N, 64);
    if (nparts_out) *nparts_out = ep.nparts;
    const bool rows_ok = gemv_rows_ok<float>(M, K, ksplit, 32);
    if (ksplit > 1 && !(EPI == EPI_F32 && rows_ok)) return fail(SRM_EINVAL, "fp32 GEMM: bad split of K = %d", K);
    if (rows_ok) {
        // few rows: stream W once per group of kGemvMB rows (64 columns per block where the partial winners of the
        // LM head are counted per 64 columns, or where 16 would make too many blocks)
        if (EPI == EPI_ARGMAX || N >= 16384) return launch_gemv_rows<float, float, EPI, 4>(A, W, (int)M, N, K, ep, st, ksplit, nparts_out);
        return launch_gemv_rows<float, float, EPI, 1>(A, W, (int)M, N, K, ep, st, ksplit, nparts_out);
    } else {
        const int64_t nb = cdiv(M, 64) * cdiv(N, 64);
        hipLaunchKernelGGL(gemm_f32_kernel<EPI>, dim3((unsigned)nb), dim3(256), 0, st, A, W, (int)M, N, K, ep);
    }
    HIP_TRY(hipGetLastError());
    return SRM_OK;
}

struct Sampling {          // temp == 0: greedy
    float temp = 0.0f;
    uint32_t seed = 0;
    int pos = 0;
    const int *pos_dev = nullptr;
    const int *pos_rows = nullptr;
    float top_p = 1.0f;    // < 1 (with temp > 0): nucleus truncation, needs the logits in memory
    uint32_t row_base = 0; // sample index of the first row
    int eos_plus1 = 0;     // ragged decode with advance: end-of-sequence token + 1 (0: none)
};

// Nucleus pass over the logits the LM head has just written; tok holds the
// unrestricted Gumbel-max winners and *slow (the row-list counter) is zero.
static int nucleus(const float *logits, int64_t rows, int V, const Sampling &sm, int32_t *tok, int32_t *store,
                   const int *step_dev, int64_t store_stride, int32_t *pos_advance, int *slow, hipStream_t st)
{
    constexpr int NT = 512, EPT = 64;
    if (V > NT * EPT) {
        // vocabulary too large for the register-resident search: one kernel, searching from memory
        hipLaunchKernelGGL((nucleus_kernel<256, false, false>), dim3((unsigned)rows), dim3(256), 0, st, logits,
                           (int64_t)V, V, sm.temp, sm.top_p, sm.seed, sm.pos, sm.pos_dev, sm.pos_rows, tok, store,
                           step_dev, store_stride, pos_advance, nullptr, nullptr, sm.row_base, sm.eos_plus1);
        HIP_TRY(hipGetLastError());
        return SRM_OK;
    }
    hipLaunchKernelGGL((nucleus_kernel<256, false, true>), dim3((unsigned)rows), dim3(256), 0, st, logits, (int64_t)V,
                       V, sm.temp, sm.top_p, sm.seed, sm.pos, sm.pos_dev, sm.pos_rows, tok, store, step_dev,
                       store_stride, pos_advance, slow, slow + 64, sm.row_base, sm.eos_plus1);
    HIP_TRY(hipGetLastError());
    const unsigned nb = (unsigned)std::min<int64_t>(rows, 256);
    hipLaunchKernelGGL((nucleus_slow_kernel<NT, EPT>), dim3(nb), dim3(NT), 0, st, logits, (int64_t)V, V, sm.temp,
                       sm.top_p, sm.seed, sm.pos, sm.pos_dev, sm.pos_rows, tok, store, step_dev, store_stride,
                       pos_advance, slow, slow + 64, sm.row_base, sm.eos_plus1);
    HIP_TRY(hipGetLastError());
    return SRM_OK;
}

struct MixArgs {           // EPI_MIX: state slab of the layer and its coefficient tables
    void *state = nullptr;
    const float *alpha = nullptr, *beta = nullptr, *lam = nullptr;
    int n_ctx = 0, hrow = 0, dh = 0, state_half = 0;
};

struct SlabArgs {          // slabs of a K-sliced projection that no kernel has added to the residual stream yet
    const float *part = nullptr;
    int nsplit = 0;
    int64_t stride = 0;
};
struct LnArgs {            // A = LayerNorm(x [+ slabs]) made by the GEMM itself (bf16, a handful of rows)
    const float *x = nullptr, *g = nullptr, *b = nullptr;
    SlabArgs slabs;
    float eps = 0.0f;
};

// out = epilogue(A W^T + bias) with operands of type T (float or bf16)
template <int EPI, typename T>
static int linear(const void *A, const void *W, const float *bias, int64_t M, int N, int K, void *out,
                  hipStream_t st, float *pv = nullptr, int32_t *pi = nullptr, int min_bn = 64,
                  int *nparts_out = nullptr, Sampling sm = Sampling(), int ksplit = 1, MixArgs mx = MixArgs(),
                  SlabArgs add = SlabArgs(), LnArgs ln = LnArgs())
{
    GemmEpi ep{bias, out, (int64_t)N, pv, pi, 0, sm.temp, sm.seed, sm.pos, sm.pos_dev, sm.pos_rows, sm.row_base,
               mx.state, mx.alpha, mx.beta, mx.lam, mx.n_ctx, mx.hrow, mx.dh, mx.state_half};
    ep.add_part = add.part; ep.add_nsplit = add.part ? add.nsplit : 0; ep.add_stride = add.stride;
    ep.clk = g_clock_probe; ep.clk_blocks = g_clock_blocks;
    if (add.part && EPI != EPI_RESID) return fail(SRM_EINVAL, "linear: pending slabs need the residual epilogue");
    if (ln.x) {
        if constexpr (sizeof(T) == 2 && (EPI == EPI_STORE || EPI == EPI_GELU || EPI == EPI_MIX)) {
            if (!lna_ok(M, K) || ksplit != 1) return fail(SRM_EINVAL, "linear: LayerNorm-on-load needs M <= %d, K <= 1024", kLnaRows);
            ep.ln_x = ln.x; ep.ln_g = ln.g; ep.ln_b = ln.b; ep.ln_eps = ln.eps;
            ep.ln_part = ln.slabs.part; ep.ln_nsplit = ln.slabs.part ? ln.slabs.nsplit : 0; ep.ln_stride = ln.slabs.stride;
            ep.nparts = 0;
            return launch_bf16_lna<EPI>(static_cast<const bf16 *>(W), (int)M, N, K, ep, st);
        } else {
            return fail(SRM_EINVAL, "linear: LayerNorm-on-load exists for bf16 store / GELU / mixer epilogues only");
        }
    }
    if constexpr (sizeof(T) == 2)
        return launch_bf16<EPI, bf16>(static_cast<const bf16 *>(A), static_cast<const bf16 *>(W), M, N, K, ep,
                                      st, min_bn, nparts_out, ksplit);
    else
        return launch_f32<EPI>(static_cast<const float *>(A), static_cast<const float *>(W), M, N, K, ep, st,
                               nparts_out, ksplit);
}

struct TokenStore {        // optional second destination of the greedy tokens (srm_generate)
    int32_t *store = nullptr;
    const int *step_dev = nullptr;
    int64_t stride = 0;
};

static int argmax_finalize(const float *pv, const int32_t *pi, int64_t rows, int nparts, int32_t *out,
                           int64_t row0, int rep, int vocab, hipStream_t st, TokenStore ts = TokenStore(),
                           FinalizeRagged rg = FinalizeRagged{})
{
    hipLaunchKernelGGL(argmax_finalize_kernel, dim3((unsigned)cdiv(rows, kFinalRows)), dim3(256), 0, st, pv, pi, rows,
                       nparts, out, row0, rep, vocab, ts.store, ts.step_dev, ts.stride, rg);
    HIP_TRY(hipGetLastError());
    return SRM_OK;
}

template <typename T, bool GATHER>
static int layernorm(const srm_model *m, const float *x_in, int64_t in_stride, const int32_t *tok,
                     float *x_out, const float *g, const float *b, void *out, int64_t rows, hipStream_t st,
                     const int32_t *seq_end = nullptr, int64_t base = 0, int64_t src_rows = 0,
                     const float *part = nullptr, int nsplit = 0, const void *add_act = nullptr,
                     int *advance_ctr = nullptr)
{
    const int d = m->d;
    T *o = static_cast<T *>(out);
    if (!GATHER && !seq_end && !part && !add_act && in_stride == d && rows >= 4096 && d <= 1024 && d % 256 == 0) {
        // plain, many rows: several rows per wavefront
        constexpr int RPW = 2;
        const unsigned nb2 = (unsigned)cdiv(rows, 4 * RPW);
        if (d == 256) hipLaunchKernelGGL((ln_rows_kernel<T, 1, RPW>), dim3(nb2), dim3(256), 0, st, x_in, g, b, o, rows, d, m->cfg.ln_eps);
        else if (d == 512) hipLaunchKernelGGL((ln_rows_kernel<T, 2, RPW>), dim3(nb2), dim3(256), 0, st, x_in, g, b, o, rows, d, m->cfg.ln_eps);
        else if (d == 768) hipLaunchKernelGGL((ln_rows_kernel<T, 3, RPW>), dim3(nb2), dim3(256), 0, st, x_in, g, b, o, rows, d, m->cfg.ln_eps);
        else hipLaunchKernelGGL((ln_rows_kernel<T, 4, RPW>), dim3(nb2), dim3(256), 0, st, x_in, g, b, o, rows, d, m->cfg.ln_eps);
        HIP_TRY(hipGetLastError());
        return SRM_OK;
    }
    const unsigned nb = (unsigned)cdiv(rows, 4);
    const T *emb = static_cast<const T *>(m->embed);
#define LN_CASE(VPL)                                                                                     \
    hipLaunchKernelGGL((ln_kernel<T, T, VPL, GATHER>), dim3(nb), dim3(256), 0, st, x_in, in_stride, tok, \
                       emb, m->V, x_out, g, b, o, rows, d, m->cfg.ln_eps, seq_end, base, src_rows, part, nsplit,       \
                       (int64_t)rows * d, static_cast<const T *>(add_act), advance_ctr)
    if (d <= 256) LN_CASE(1);
    else if (d <= 512) LN_CASE(2);
    else if (d <= 1024) LN_CASE(4);
    else if (d <= 2048) LN_CASE(8);
    else LN_CASE(16);
#undef LN_CASE
    HIP_TRY(hipGetLastError());
    return SRM_OK;
}

template <typename T>
static int state_update(const srm_model *m, int layer, int pos, int64_t B, const void *u, void *S, void *mx,
                        hipStream_t st, const int *pos_dev = nullptr)
{
    // Two 16-byte state vectors per thread and one pass over the slab (measured
    // best on MI355X: 6.15 TB/s at B = 16384, against 5.55 TB/s with four vectors
    // per thread and a capped grid).  The block count is rounded up so that
    // gridDim * 256 is a multiple of d/4: the kernel relies on a thread keeping
    // one channel group.
    constexpr int UNROLL = 2;
    const LayerDev &y = m->layers[layer];
    const int dv = m->dm / 4;
    const int64_t nvec = B * dv;
    int a = dv, b = 256;
    while (b) { int t = a % b; a = b; b = t; }
    const int step = dv / a;
    const int64_t nb = cdiv(cdiv(nvec, 256 * UNROLL), step) * step;
    if (m->shalf)
        hipLaunchKernelGGL((state_update_kernel<T, UNROLL, f16>), dim3((unsigned)nb), dim3(256), 0, st,
                           static_cast<const T *>(u), static_cast<f16 *>(S), static_cast<T *>(mx), y.alpha, y.beta,
                           y.lam, pos, pos_dev, m->cfg.n_ctx, m->Hs, m->hrow, m->dm, nvec);
    else
        hipLaunchKernelGGL((state_update_kernel<T, UNROLL>), dim3((unsigned)nb), dim3(256), 0, st,
                           static_cast<const T *>(u), static_cast<float *>(S), static_cast<T *>(mx), y.alpha, y.beta,
                           y.lam, pos, pos_dev, m->cfg.n_ctx, m->Hs, m->hrow, m->dm, nvec);
    HIP_TRY(hipGetLastError());
    return SRM_OK;
}

static hipStream_t as_stream(void *s) { return static_cast<hipStream_t>(s); }

static int check_device(const srm_model *m)
{
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev != m->device)
        return fail(SRM_EINVAL, "model lives on device %d but device %d is current", m->device, dev);
    return SRM_OK;
}

// Whether the state update rides in the in-projection's epilogue (EPI_MIX) instead of running as a
// kernel of its own.  bf16 models: always (few rows: one dependent kernel less per layer; many rows: the
// head input u is never written to memory and read back, 66 MB per layer at 16384 x 1024, measured
// 7.35 -> 7.15 ms per step there).  fp32 models: below 2^20 state elements per layer, where the step is
// bound by its number of kernels; the fp32 tile kernel has not been measured beyond.
// SRM_FUSE_MIXER=0 in the environment keeps the two kernels apart (tests, measurements).
static bool fuse_mixer(const srm_model *m, int64_t rows)
{
    if (m->noproj) return false;
    const char *e = getenv("SRM_FUSE_MIXER");
    if (e && e[0] == '0') return false;
    return m->wsize == 2 || rows * m->dm <= (1 << 20);
}

// A handful of samples of a bf16 model: every LayerNorm between two GEMMs of the step is made by the GEMM
// that consumes it (gemm_bf16_kernel's LNA form) instead of a launch of its own - with one row the
// LayerNorm launches are a quarter of the step's time.  SRM_LN_ON_LOAD=0 in the environment keeps the
// separate kernels.
static bool ln_on_load(const srm_model *m, int64_t rows)
{
    if (m->wsize != 2 || m->noproj || !lna_ok(rows, m->d)) return false;
    const char *e = getenv("SRM_LN_ON_LOAD");
    return !(e && e[0] == '0');
}

// A dozen to about a thousand rows of a bf16 model with head projections: LayerNorm1, in-projection, state
// update and out-projection of a layer are one kernel (tokmix.hpp), which leaves the out-projection as d / 128
// slabs behind the slabs that the previous layer's K-sliced MLP-down projection may have left; the LayerNorm2
// kernel adds all of them to x.  Taken while its work-groups (16 rows x 128 columns each) fit the chip in one
// round: measured on C3's model (d 512, L 8) per step 0.280 -> 0.248 ms at 16 rows, 0.298 -> 0.260 at 64,
// 0.318 -> 0.285 at 256, 0.353 -> 0.310 at 512, 0.378 -> 0.361 at 1024, and 0.473 -> 0.512 at 2048 (two rounds).
// SRM_TOKEN_MIX=0 in the environment keeps the separate kernels, =1 takes the one kernel wherever it can run.
constexpr int64_t kTokMixMinRows = 9;
static bool token_mix_shape_ok(const srm_model *m)
{
    return m->wsize == 2 && !m->noproj && m->dm == m->d && (m->d == 256 || m->d == 512);
}
static bool token_mix_one_kernel(const srm_model *m, int64_t rows)
{
    if (!token_mix_shape_ok(m) || ln_on_load(m, rows) || rows > kSplitMaxRows) return false;   // (w.part: see carve)
    if (!fuse_mixer(m, rows)) return false;          // (SRM_FUSE_MIXER=0 asks for the state update as a kernel of its own)
    const char *e = getenv("SRM_TOKEN_MIX");
    if (e && e[0] == '0') return false;
    if (e && e[0] == '1') return true;
    return rows >= kTokMixMinRows && cdiv(rows, 16) * (m->d / kTokMixCols) <= device_cus();
}
struct TokMixCall {
    const float *x;
    SlabArgs pending;
    void *state;
    Sampling where;
    float *slabs;          // [d / 128][rows][d]
};
static int token_mix(const srm_model *m, int l, const TokMixCall &c, int64_t rows, hipStream_t st)
{
    const LayerDev &y = m->layers[l];
    TokMixArgs a{};
    a.x = c.x;
    a.pend = c.pending.nsplit > 0 ? c.pending.part : nullptr;
    a.npend = c.pending.nsplit > 0 ? c.pending.nsplit : 0;
    a.pend_stride = c.pending.stride;
    a.ln1_g = y.ln1_g; a.ln1_b = y.ln1_b;
    a.eps = m->cfg.ln_eps;
    a.w_in = static_cast<const bf16 *>(y.w_in); a.w_out = static_cast<const bf16 *>(y.w_out);
    a.b_in = y.b_in; a.b_out = y.b_out;
    a.state = c.state;
    a.alpha = y.alpha; a.beta = y.beta; a.lam = y.lam;
    a.n_ctx = m->cfg.n_ctx; a.hrow = m->hrow; a.dh = m->dm / m->Hs;
    a.pos = c.where.pos; a.pos_dev = c.where.pos_dev; a.pos_rows = c.where.pos_rows;
    a.slabs = c.slabs;
    a.rows = rows;
    a.clk = g_clock_probe;
    a.clk_blocks = g_clock_blocks;
    const unsigned nb = (unsigned)(cdiv(rows, 16) * (m->d / kTokMixCols));
#define TOKMIX_LAUNCH(D, TS)                                                                                   \
    do {                                                                                                       \
        auto kern = token_mix_kernel<D, TS>;                                                                   \
        static bool attr_set = false;                                                                          \
        if (!attr_set) {                                                                                       \
            HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),                                  \
                                        hipFuncAttributeMaxDynamicSharedMemorySize, tokmix_lds_bytes<D>()));   \
            attr_set = true;                                                                                   \
        }                                                                                                      \
        hipLaunchKernelGGL(kern, dim3(nb), dim3(256), tokmix_lds_bytes<D>(), st, a);                           \
    } while (0)
    if (m->d == 256) { if (m->shalf) TOKMIX_LAUNCH(256, f16); else TOKMIX_LAUNCH(256, float); }
    else if (m->d == 512) { if (m->shalf) TOKMIX_LAUNCH(512, f16); else TOKMIX_LAUNCH(512, float); }
    else return fail(SRM_EINVAL, "token_mix: d = %d has no one-kernel form", m->d);
#undef TOKMIX_LAUNCH
    HIP_TRY(hipGetLastError());
    return SRM_OK;
}

// One block (token mixing + channel mixing) on `rows` token rows.  On entry
// w.a holds LayerNorm1(x) of this layer; mix(l) turns w.u into w.mx.  With
// norm_next, w.a leaves holding the next layer's LayerNorm1(x), or the final
// LayerNorm after the last layer.
// With pend (decode of a handful of rows, see ln_on_load): no LayerNorm kernels between the GEMMs.  From
// layer 1 on w.a is not used: the in- and up-projection normalise the rows of w.x themselves, *pend says how
// many slabs of the previous layer's K-sliced MLP-down projection still wait in w.part (the in-projection
// adds them for its LayerNorm, the out-projection's residual epilogue adds them to w.x), and on return it
// holds this layer's count.  Layer 0 enters with w.a from the embedding kernel as usual.
template <typename T, typename MIX>
static int block(const srm_model *m, int l, const Workspace &w, int64_t rows, hipStream_t st, MIX &&mix,
                 bool norm_next, bool allow_split = false, void *fuse_state = nullptr, Sampling fuse_pos = Sampling(),
                 void *np_state = nullptr, int *pend = nullptr, int *tm_pend = nullptr)
{
    const LayerDev &y = m->layers[l];
    const int d = m->d, dm = m->dm, ff = m->ff;
    const bool lnf = pend != nullptr;
    const SlabArgs waiting = lnf && *pend > 0 ? SlabArgs{w.part, *pend, (int64_t)rows * d} : SlabArgs();
    const LnArgs ln1 = lnf && l > 0 ? LnArgs{w.x, y.ln1_g, y.ln1_b, waiting, m->cfg.ln_eps} : LnArgs();
    const LnArgs ln2 = lnf ? LnArgs{w.x, y.ln2_g, y.ln2_b, SlabArgs(), m->cfg.ln_eps} : LnArgs();
    // K slices of a residual projection (decode with few rows; see kSplitK).  bf16: the MLP down projection in
    // kSplitK slices while the 64x64 tiles number at most 192 (measured: more slices, or slicing the
    // out-projection too, costs more in the LayerNorm that adds the slabs than the shorter k loops save;
    // since the unsplit tile runs on a deep LDS ring the two arrangements time the same at 192 tiles and
    // the unsplit one is 5 % faster per step at 256, for d = 512 and for d = 1024).
    // fp32 with at most kGemvRows rows (GEMVs): both projections, slices of at least 64 k.
    auto resid_split = [&](int K, bool down) {
        if (!allow_split || !w.part) return 1;
        if (sizeof(T) == 4) {
            if (rows > kGemvRows) return 1;
            int sp = kGemvSplitMax;
            while (sp > 1 && (K % (16 * sp) || K / sp < 64)) sp >>= 1;
            return sp;
        }
        return down && K >= 1024 && K % (64 * kSplitK) == 0 && cdiv(rows, 64) * cdiv(d, 64) <= 192 ? kSplitK : 1;
    };
    if constexpr (sizeof(T) == 2) {
        if (tm_pend) {
            // Token mixing in one kernel (see token_mix_one_kernel).  w.part holds 2 * kSplitK slabs: the first
            // kSplitK are the MLP-down projection's (*tm_pend of them wait from the previous layer), the rest
            // take this layer's out-projection.  w.a on entry is not used (the kernel normalises w.x + waiting
            // slabs itself); LayerNorm2 adds everything to w.x.  On return *tm_pend is this layer's count.
            const int64_t stride = (int64_t)rows * d;
            const int nq = d / kTokMixCols;
            float *mine = w.part + (size_t)*tm_pend * stride;      // directly behind the waiting slabs
            const SlabArgs waiting_tm = *tm_pend > 0 ? SlabArgs{w.part, *tm_pend, stride} : SlabArgs();
            SRM_TRY(token_mix(m, l, TokMixCall{w.x, waiting_tm, np_state, fuse_pos, mine}, rows, st));
            SRM_TRY((layernorm<T, false>(m, w.x, d, nullptr, w.x, y.ln2_g, y.ln2_b, w.a, rows, st, nullptr, 0, 0, w.part,
                                         *tm_pend + nq)));
            SRM_TRY((linear<EPI_GELU, T>(w.a, y.w_up, y.b_up, rows, ff, d, w.g, st)));
            const int spd = resid_split(ff, true);
            if (spd > 1)
                SRM_TRY((linear<EPI_F32, T>(w.g, y.w_down, y.b_down, rows, d, ff, w.part, st, nullptr, nullptr, 64,
                                            nullptr, Sampling(), spd)));
            else
                SRM_TRY((linear<EPI_RESID, T>(w.g, y.w_down, y.b_down, rows, d, ff, w.x, st)));
            *tm_pend = spd > 1 ? spd : 0;
            if (l + 1 < m->L) return SRM_OK;                       // the next layer's kernels add the slabs
            if (spd > 1)
                return layernorm<T, false>(m, w.x, d, nullptr, w.x, m->lnf_g, m->lnf_b, w.a, rows, st, nullptr, 0, 0,
                                           w.part, spd);
            return layernorm<T, false>(m, w.x, d, nullptr, nullptr, m->lnf_g, m->lnf_b, w.a, rows, st);
        }
    }
    if (m->noproj && np_state) {
        // non-projected layer, decode: LayerNorm1, state update, residual add and LayerNorm2 in one kernel
        const unsigned nb = (unsigned)cdiv(rows, 4);
#define NP_LAUNCH(VPL, TS)                                                                                    \
    hipLaunchKernelGGL((np_token_mix_kernel<T, VPL, TS>), dim3(nb), dim3(256), 0, st, w.x,                     \
                       static_cast<TS *>(np_state), static_cast<T *>(w.a), y.ln1_g, y.ln1_b, y.ln2_g, y.ln2_b, \
                       y.alpha, y.beta, y.lam, fuse_pos.pos, fuse_pos.pos_dev, fuse_pos.pos_rows, m->cfg.n_ctx, \
                       m->Hs, m->hrow, d, rows, m->cfg.ln_eps)
#define NP_CASE(VPL)                                                                                          \
    do {                                                                                                      \
        if (m->shalf) NP_LAUNCH(VPL, f16);                                                                    \
        else NP_LAUNCH(VPL, float);                                                                           \
    } while (0)
        if (d <= 256) NP_CASE(1);
        else if (d <= 512) NP_CASE(2);
        else if (d <= 1024) NP_CASE(4);
        else if (d <= 2048) NP_CASE(8);
        else NP_CASE(16);
#undef NP_CASE
#undef NP_LAUNCH
        HIP_TRY(hipGetLastError());
    } else if (m->noproj) {
        // non-projected layer: mixer on the LayerNorm output, its result added to x by the LayerNorm kernel
        SRM_TRY(mix(l));
        SRM_TRY((layernorm<T, false>(m, w.x, d, nullptr, w.x, y.ln2_g, y.ln2_b, w.a, rows, st, nullptr, 0, 0, nullptr,
                                     0, w.mx)));
    } else if (fuse_state) {
        // few rows: the state update rides in the in-projection's epilogue (one kernel less per layer)
        const MixArgs mx{fuse_state, y.alpha, y.beta, y.lam, m->cfg.n_ctx, m->hrow, dm / m->Hs, m->shalf ? 1 : 0};
        SRM_TRY((linear<EPI_MIX, T>(w.a, y.w_in, y.b_in, rows, dm, d, w.mx, st, nullptr, nullptr, 64, nullptr, fuse_pos,
                                    1, mx, SlabArgs(), ln1)));
    } else {
        SRM_TRY((linear<EPI_STORE, T>(w.a, y.w_in, y.b_in, rows, dm, d, w.u, st, nullptr, nullptr, 64, nullptr, Sampling(),
                                      1, MixArgs(), SlabArgs(), ln1)));
        SRM_TRY(mix(l));
    }
    if (!m->noproj) {
        const int sp = resid_split(dm, false);
        if (sp > 1) {
            SRM_TRY((linear<EPI_F32, T>(w.mx, y.w_out, y.b_out, rows, d, dm, w.part, st, nullptr, nullptr, 64, nullptr,
                                        Sampling(), sp)));
            SRM_TRY((layernorm<T, false>(m, w.x, d, nullptr, w.x, y.ln2_g, y.ln2_b, w.a, rows, st, nullptr, 0, 0, w.part,
                                         sp)));
        } else {
            SRM_TRY((linear<EPI_RESID, T>(w.mx, y.w_out, y.b_out, rows, d, dm, w.x, st, nullptr, nullptr, 64, nullptr,
                                          Sampling(), 1, MixArgs(), l > 0 ? waiting : SlabArgs())));
            if (!lnf) SRM_TRY((layernorm<T, false>(m, w.x, d, nullptr, nullptr, y.ln2_g, y.ln2_b, w.a, rows, st)));
        }
    }
    SRM_TRY((linear<EPI_GELU, T>(w.a, y.w_up, y.b_up, rows, ff, d, w.g, st, nullptr, nullptr, 64, nullptr, Sampling(), 1,
                                 MixArgs(), SlabArgs(), ln2)));
    // (not with the fused non-projected layer: no LayerNorm kernel follows there to add the slabs)
    const int spd = (norm_next && !(m->noproj && np_state)) ? resid_split(ff, true) : 1;
    if (spd > 1)
        SRM_TRY((linear<EPI_F32, T>(w.g, y.w_down, y.b_down, rows, d, ff, w.part, st, nullptr, nullptr, 64, nullptr,
                                    Sampling(), spd)));
    else
        SRM_TRY((linear<EPI_RESID, T>(w.g, y.w_down, y.b_down, rows, d, ff, w.x, st)));
    if (lnf) *pend = spd > 1 ? spd : 0;
    if (lnf && l + 1 < m->L) return SRM_OK;                        // the next layer's in-projection normalises
    if (norm_next && !(m->noproj && np_state && l + 1 < m->L)) {   // the fused kernel does its own LayerNorm1
        const float *g = l + 1 < m->L ? m->layers[l + 1].ln1_g : m->lnf_g;
        const float *b = l + 1 < m->L ? m->layers[l + 1].ln1_b : m->lnf_b;
        if (spd > 1)               // x += slabs, then normalise
            SRM_TRY((layernorm<T, false>(m, w.x, d, nullptr, w.x, g, b, w.a, rows, st, nullptr, 0, 0, w.part, spd)));
        else
            SRM_TRY((layernorm<T, false>(m, w.x, d, nullptr, nullptr, g, b, w.a, rows, st)));
    }
    return SRM_OK;
}

// LM head on M normalised rows `a`: optional fp32 logits, greedy token written
// `rep` times at d_tok[(row0 + row) * rep + r].
template <typename T>
static int head_argmax(const srm_model *m, const Workspace &w, const void *a, int64_t M, float *logits,
                       int32_t *d_tok, int64_t row0, int rep, hipStream_t st, TokenStore ts = TokenStore(),
                       Sampling sm = Sampling(), FinalizeRagged rg = FinalizeRagged{})
{
    int nparts = 0;
    SRM_TRY((linear<EPI_ARGMAX, T>(a, m->head, nullptr, M, m->V, m->d, logits, st, w.pv, w.pi, head_min_bn(m),
                                   &nparts, sm)));
    return argmax_finalize(w.pv, w.pi, M, nparts, d_tok, row0, rep, m->V, st, ts, rg);
}

// ------------------------------------------------------------------ decode
// One decode step for the rows b0 .. b0+nb-1 of a batch of B samples; uniform position
// (pos / pos_dev) or one position per sample (pos_rows, base pointer of the batch).
struct DecodeArgs {
    int64_t B;
    int pos;
    const int *pos_dev;
    int32_t *pos_rows;
    int advance;
    const int32_t *tok_in;
    void *state;
    int32_t *tok_out;
    float *logits, *hidden;
    TokenStore ts;
    float temperature;
    uint32_t seed;
    float top_p;
    int eos_plus1 = 0;
    int *advance_ctr = nullptr;     // step counters of srm_generate, advanced by the first kernel of the step
};

template <typename T>
static int decode_rows(srm_model *m, const DecodeArgs &a, int64_t b0, int64_t nb, void *ws, hipStream_t st)
{
    const Workspace w = carve(m, ws, nb);
    const int d = m->d, dm = m->dm;
    int32_t *pos_rows = a.pos_rows ? a.pos_rows + b0 : nullptr;
    auto slab = [&](int l) {       // rows b0.. of layer l's state
        return static_cast<void *>(static_cast<unsigned char *>(layer_state(m, a.state, l, a.B)) +
                                   (size_t)b0 * dm * m->ssize);
    };
    SRM_TRY((layernorm<T, true>(m, nullptr, 0, a.tok_in + b0, w.x, m->layers[0].ln1_g, m->layers[0].ln1_b, w.a, nb,
                                st, nullptr, 0, 0, nullptr, 0, nullptr, b0 == 0 ? a.advance_ctr : nullptr)));
    auto mix = [&](int l) {
        if (!pos_rows) return state_update<T>(m, l, a.pos, nb, w.u, slab(l), w.mx, st, a.pos_dev);
        const LayerDev &y = m->layers[l];
        const int64_t nvec = nb * (dm / 4);
        if (m->shalf)
            hipLaunchKernelGGL((state_update_ragged_kernel<T, f16>), dim3((unsigned)cdiv(nvec, 256)), dim3(256), 0, st,
                               static_cast<const T *>(w.u), static_cast<f16 *>(slab(l)), static_cast<T *>(w.mx),
                               y.alpha, y.beta, y.lam, pos_rows, m->cfg.n_ctx, m->Hs, m->hrow, dm, nvec);
        else
            hipLaunchKernelGGL((state_update_ragged_kernel<T>), dim3((unsigned)cdiv(nvec, 256)), dim3(256), 0, st,
                               static_cast<const T *>(w.u), static_cast<float *>(slab(l)), static_cast<T *>(w.mx),
                               y.alpha, y.beta, y.lam, pos_rows, m->cfg.n_ctx, m->Hs, m->hrow, dm, nvec);
        HIP_TRY(hipGetLastError());
        return (int)SRM_OK;
    };
    const bool fuse = fuse_mixer(m, nb);
    const Sampling where{0.0f, 0, a.pos, a.pos_dev, pos_rows, 1.0f, 0};
    int pend = 0, tm_pend = 0;
    const bool lnf = ln_on_load(m, nb);
    const bool tm = token_mix_one_kernel(m, nb);
    for (int l = 0; l < m->L; ++l)
        SRM_TRY((block<T>(m, l, w, nb, st, mix, true, true, fuse ? slab(l) : nullptr, where, slab(l),
                          lnf ? &pend : nullptr, tm ? &tm_pend : nullptr)));
    if (a.hidden)
        HIP_TRY(hipMemcpyAsync(a.hidden + (size_t)b0 * d, w.x, (size_t)nb * d * 4, hipMemcpyDeviceToDevice, st));
    const Sampling sm{a.temperature, a.seed, a.pos, a.pos_dev, pos_rows, a.top_p, (uint32_t)b0, a.eos_plus1};
    const bool topp = a.temperature > 0.0f && a.top_p < 1.0f;
    FinalizeRagged rg{};
    if (a.pos_rows) {
        rg.pos_rows = a.pos_rows;             // indexed with row0 + row
        rg.advance = a.advance && !topp;      // with a nucleus pass the positions move after it
        rg.n_ctx = m->cfg.n_ctx;
        rg.eos_plus1 = a.eos_plus1;
    }
    if (topp) rg.zero_counter = w.slow;
    float *lg = a.logits ? a.logits + (size_t)b0 * m->V : nullptr;
    SRM_TRY((head_argmax<T>(m, w, w.a, nb, lg, a.tok_out, b0, 1, st, a.ts, sm, rg)));
    if (topp)
        SRM_TRY(nucleus(lg, nb, m->V, sm, a.tok_out + b0, a.ts.store ? a.ts.store + b0 : nullptr, a.ts.step_dev,
                        a.ts.stride, (pos_rows && a.advance) ? pos_rows : nullptr, w.slow, st));
    return SRM_OK;
}

// Rows per pass of a decode call: the whole batch if the workspace holds it, else as many
// rows as it holds (the samples are independent, so a step can be taken in slices; this lets
// a caller keep far more sequences resident than one workspace covers).  0: too small.
// srm_workspace_bytes(rows) = the row arrays + 256 bytes that srm_generate uses for its step
// counters at the very end of the caller's buffer, so the row arrays get workspace_bytes - 256.
static int64_t decode_rows_per_pass(const srm_model *m, int64_t B, size_t workspace_bytes)
{
    if (srm_workspace_bytes(m, B) <= workspace_bytes) return B;
    int64_t lo = 0, hi = B;
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) / 2;
        if (srm_workspace_bytes(m, mid) <= workspace_bytes) lo = mid; else hi = mid - 1;
    }
    if (lo >= 256) lo = lo / 256 * 256;       // whole GEMM tiles per pass
    return lo < std::min<int64_t>(B, 256) ? 0 : lo;
}

static int decode_batch(srm_model *m, const DecodeArgs &a, void *ws, size_t workspace_bytes, hipStream_t st)
{
    const int64_t rpp = decode_rows_per_pass(m, a.B, workspace_bytes);
    if (rpp <= 0) return fail(SRM_ENOMEM, "workspace %zu bytes holds fewer than %lld rows", workspace_bytes,
                              (long long)std::min<int64_t>(a.B, 256));
    for (int64_t b0 = 0; b0 < a.B; b0 += rpp) {
        const int64_t nb = std::min<int64_t>(rpp, a.B - b0);
        SRM_TRY(m->wsize == 2 ? decode_rows<bf16>(m, a, b0, nb, ws, st) : decode_rows<float>(m, a, b0, nb, ws, st));
    }
    return SRM_OK;
}

static int decode_step_common(const char *who, srm_model *m, int64_t B, int32_t pos, const int32_t *d_tok_in,
                              void *d_state, int32_t *d_tok_out, float *d_logits, float *d_hidden,
                              void *d_workspace, size_t workspace_bytes, void *hip_stream, float temperature,
                              uint32_t seed, float top_p = 1.0f)
{
    if (!m || !d_tok_in || !d_state || !d_tok_out || !d_workspace) return fail(SRM_EINVAL, "%s: null argument", who);
    if (B <= 0 || B >= (1 << 30)) return fail(SRM_EINVAL, "%s: batch %lld out of range", who, (long long)B);
    if (pos < 0 || pos >= m->cfg.n_ctx) return fail(SRM_EINVAL, "%s: pos %d outside [0, %d)", who, pos, m->cfg.n_ctx);
    if (!(temperature >= 0.0f)) return fail(SRM_EINVAL, "%s: temperature must be >= 0", who);
    if (!(top_p > 0.0f)) return fail(SRM_EINVAL, "%s: top_p must be > 0", who);
    if (temperature > 0.0f && top_p < 1.0f && !d_logits)
        return fail(SRM_EINVAL, "%s: top_p < 1 needs a logits buffer", who);
    SRM_TRY(check_device(m));
    const DecodeArgs a{B, pos, nullptr, nullptr, 0, d_tok_in, d_state, d_tok_out, d_logits, d_hidden, TokenStore(),
                       temperature, seed, top_p};
    return decode_batch(m, a, d_workspace, workspace_bytes, as_stream(hip_stream));
}

extern "C" int srm_decode_step(srm_model *m, int64_t B, int32_t pos, const int32_t *d_tok_in, void *d_state,
                               int32_t *d_tok_out, float *d_logits, float *d_hidden, void *d_workspace,
                               size_t workspace_bytes, void *hip_stream)
{
    return decode_step_common("srm_decode_step", m, B, pos, d_tok_in, d_state, d_tok_out, d_logits, d_hidden,
                              d_workspace, workspace_bytes, hip_stream, 0.0f, 0);
}

extern "C" int srm_decode_step_sampled(srm_model *m, int64_t B, int32_t pos, const int32_t *d_tok_in, void *d_state,
                                       int32_t *d_tok_out, float temperature, uint32_t seed, float *d_logits,
                                       float *d_hidden, void *d_workspace, size_t workspace_bytes, void *hip_stream)
{
    return decode_step_common("srm_decode_step_sampled", m, B, pos, d_tok_in, d_state, d_tok_out, d_logits, d_hidden,
                              d_workspace, workspace_bytes, hip_stream, temperature, seed);
}

extern "C" int srm_decode_step_topp(srm_model *m, int64_t B, int32_t pos, const int32_t *d_tok_in, void *d_state,
                                    int32_t *d_tok_out, float temperature, float top_p, uint32_t seed,
                                    float *d_logits, float *d_hidden, void *d_workspace, size_t workspace_bytes,
                                    void *hip_stream)
{
    return decode_step_common("srm_decode_step_topp", m, B, pos, d_tok_in, d_state, d_tok_out, d_logits, d_hidden,
                              d_workspace, workspace_bytes, hip_stream, temperature, seed, top_p);
}

// ------------------------------------------------------------------ decode, one position per sample
template <typename T>
static int decode_ragged_impl(srm_model *m, int64_t B, int32_t *pos_rows, int advance, const int32_t *tok_in,
                              void *state, int32_t *tok_out, float *logits, void *ws, hipStream_t st,
                              float temperature, uint32_t seed, float top_p)
{
    const Workspace w = carve(m, ws, B);
    const int dm = m->dm;
    SRM_TRY((layernorm<T, true>(m, nullptr, 0, tok_in, w.x, m->layers[0].ln1_g, m->layers[0].ln1_b, w.a, B, st)));
    auto mix = [&](int l) {
        const LayerDev &y = m->layers[l];
        const int64_t nvec = B * (dm / 4);
        if (m->shalf)
            hipLaunchKernelGGL((state_update_ragged_kernel<T, f16>), dim3((unsigned)cdiv(nvec, 256)), dim3(256), 0, st,
                               static_cast<const T *>(w.u), static_cast<f16 *>(layer_state(m, state, l, B)),
                               static_cast<T *>(w.mx), y.alpha, y.beta, y.lam, pos_rows, m->cfg.n_ctx, m->Hs, m->hrow, dm, nvec);
        else
            hipLaunchKernelGGL((state_update_ragged_kernel<T>), dim3((unsigned)cdiv(nvec, 256)), dim3(256), 0, st,
                               static_cast<const T *>(w.u), static_cast<float *>(layer_state(m, state, l, B)),
                               static_cast<T *>(w.mx), y.alpha, y.beta, y.lam, pos_rows, m->cfg.n_ctx, m->Hs, m->hrow, dm, nvec);
        HIP_TRY(hipGetLastError());
        return (int)SRM_OK;
    };
    const bool fuse = fuse_mixer(m, B);
    const Sampling where{0.0f, 0, 0, nullptr, pos_rows, 1.0f};
    int pend = 0, tm_pend = 0;
    const bool lnf = ln_on_load(m, B);
    const bool tm = token_mix_one_kernel(m, B);
    for (int l = 0; l < m->L; ++l)
        SRM_TRY((block<T>(m, l, w, B, st, mix, true, true, fuse ? layer_state(m, state, l, B) : nullptr, where,
                          layer_state(m, state, l, B), lnf ? &pend : nullptr, tm ? &tm_pend : nullptr)));
    const bool topp = temperature > 0.0f && top_p < 1.0f;
    FinalizeRagged rg{};
    rg.pos_rows = pos_rows;
    rg.advance = advance && !topp;        // with a nucleus pass the positions move after it
    rg.n_ctx = m->cfg.n_ctx;
    if (topp) rg.zero_counter = w.slow;
    const Sampling sm{temperature, seed, 0, nullptr, pos_rows, top_p};
    SRM_TRY((head_argmax<T>(m, w, w.a, B, logits, tok_out, 0, 1, st, TokenStore(), sm, rg)));
    if (topp)
        SRM_TRY(nucleus(logits, B, m->V, sm, tok_out, nullptr, nullptr, 0, advance ? pos_rows : nullptr, w.slow, st));
    return SRM_OK;
}

extern "C" int srm_decode_step_ragged(srm_model *m, int64_t B, int32_t *d_pos, int32_t advance,
                                      const int32_t *d_tok_in, void *d_state, int32_t *d_tok_out,
                                      float temperature, float top_p, uint32_t seed, float *d_logits,
                                      void *d_workspace, size_t workspace_bytes, void *hip_stream)
{
    const char *who = "srm_decode_step_ragged";
    if (!m || !d_pos || !d_tok_in || !d_state || !d_tok_out || !d_workspace)
        return fail(SRM_EINVAL, "%s: null argument", who);
    if (B <= 0 || B >= (1 << 30)) return fail(SRM_EINVAL, "%s: batch %lld out of range", who, (long long)B);
    if (!(temperature >= 0.0f)) return fail(SRM_EINVAL, "%s: temperature must be >= 0", who);
    if (!(top_p > 0.0f)) return fail(SRM_EINVAL, "%s: top_p must be > 0", who);
    if (temperature > 0.0f && top_p < 1.0f && !d_logits)
        return fail(SRM_EINVAL, "%s: top_p < 1 needs a logits buffer", who);
    SRM_TRY(check_device(m));
    const DecodeArgs a{B, 0, nullptr, d_pos, advance != 0, d_tok_in, d_state, d_tok_out, d_logits, nullptr, TokenStore(),
                       temperature, seed, top_p};
    return decode_batch(m, a, d_workspace, workspace_bytes, as_stream(hip_stream));
}

// ------------------------------------------------------------------ generate, few samples: one persistent kernel
// Number of work-groups for the one-kernel path (see mega.hpp), or 0 if the call does not
// qualify: fp32 weights and state, head projections, at most kMegaMaxB samples, d <= 1024,
// the widest activation row of all samples within 128 KB of LDS, cooperative launches
// supported, and a model small enough for the small grid to win (see below).  SRM_MEGAKERNEL=0
// in the environment switches the path off, =2 takes it whatever the model's size,
// SRM_MEGA_BLOCKS=n sets the grid (default 16: a grid barrier costs about 1.4 us + 65 ns per
// work-group).
static int mega_rows(int64_t B) { return B <= 1 ? 1 : B <= 2 ? 2 : B <= 4 ? 4 : kMegaMaxB; }   // rows the kernel is unrolled for

static int mega_blocks(const srm_model *m, int64_t B)
{
    if (!m->mega_layers || m->shalf || B > kMegaMaxB || m->L > kMegaMaxLayers) return 0;
    const int widest = std::max(std::max(m->d, m->dm), m->ff);
    if (m->d > 1024 || m->d % 4 || m->dm % 4 || m->ff % 4 || (size_t)mega_rows(B) * widest * 4 > 128 * 1024) return 0;
    // The small grid has a fraction of the chip's arithmetic and cache bandwidth: measured against the step
    // kernels, the path wins while rows x matrix elements stay below about 16 M (C1's model: 93 against 132 us
    // per step at B = 1, 112 against 132 at B = 4, 130 against 126 at B = 8; a 25 M-element model loses at B = 1).
    const char *sw = getenv("SRM_MEGAKERNEL");
    if (sw && sw[0] == '0') return 0;
    const double elems = (double)m->L * ((double)2 * m->d * m->dm + (double)2 * m->d * m->ff) + (double)m->V * m->d;
    if (elems * mega_rows(B) > 16e6 && !(sw && sw[0] == '2')) return 0;      // SRM_MEGAKERNEL=2: whatever the size
    int coop = 0;
    if (hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, m->device) != hipSuccess || !coop) return 0;
    int nblk = 16;
    if (const char *nb = getenv("SRM_MEGA_BLOCKS")) nblk = atoi(nb);
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, m->device) != hipSuccess) return 0;
    return std::max(1, std::min(std::min(nblk, kMegaMaxBlocks), cus));
}

extern "C" int32_t srm_generate_one_kernel_blocks(const srm_model *m, int64_t B)
{
    return m && B > 0 ? mega_blocks(m, B) : 0;
}

static int mega_generate(srm_model *m, int B, int pos0, int G, int32_t *tok, void *state, int32_t *store,
                         float temperature, uint32_t seed, void *ws, int nblk, hipStream_t st)
{
    const Workspace w = carve(m, ws, B);
    MegaArgs a;
    a.layers = m->mega_layers;
    a.embed = static_cast<const float *>(m->embed);
    a.head = static_cast<const float *>(m->head);
    a.lnf_g = m->lnf_g; a.lnf_b = m->lnf_b;
    a.V = m->V; a.d = m->d; a.dm = m->dm; a.ff = m->ff; a.L = m->L; a.Hs = m->Hs; a.hrow = m->hrow;
    a.n_ctx = m->cfg.n_ctx; a.eps = m->cfg.ln_eps;
    a.B = B; a.pos0 = pos0; a.G = G;
    a.tok = tok; a.state = static_cast<float *>(state); a.store = store;
    a.temp = temperature; a.seed = seed;
    a.x = w.x; a.mbuf = static_cast<float *>(w.mx); a.gbuf = static_cast<float *>(w.g);
    a.pv = reinterpret_cast<float *>(w.mega);
    a.pi = reinterpret_cast<int32_t *>(w.mega + (size_t)kMegaMaxBlocks * kMegaMaxB * 4);
    a.bar = reinterpret_cast<unsigned *>(w.mega + (size_t)kMegaMaxBlocks * kMegaMaxB * 8);
    const int mb = mega_rows(B);
    const size_t lds = (size_t)mb * std::max(std::max(m->d, m->dm), m->ff) * 4;
    const void *kern = mb == 1 ? reinterpret_cast<const void *>(mega_generate_kernel<1>)
                       : mb == 2 ? reinterpret_cast<const void *>(mega_generate_kernel<2>)
                       : mb == 4 ? reinterpret_cast<const void *>(mega_generate_kernel<4>)
                                 : reinterpret_cast<const void *>(mega_generate_kernel<kMegaMaxB>);
    static bool attr_set[4] = {false, false, false, false};
    const int slot = mb == 1 ? 0 : mb == 2 ? 1 : mb == 4 ? 2 : 3;
    if (!attr_set[slot]) {
        HIP_TRY(hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024));
        attr_set[slot] = true;
    }
    hipLaunchKernelGGL(mega_reset_kernel, dim3(1), dim3(256), 0, st, a.bar, store, G * B);
    HIP_TRY(hipGetLastError());
    void *args[] = {&a};
    HIP_TRY(hipLaunchCooperativeKernel(kern, dim3((unsigned)nblk), dim3(kMegaThreads), args, (unsigned)lds, st));
    return SRM_OK;
}

// ------------------------------------------------------------------ generate (G steps in one call)
static int generate_step(srm_model *m, int64_t B, int32_t *tok, void *state, void *ws, size_t ws_bytes, int *ctr,
                         TokenStore ts, hipStream_t st, float temperature, uint32_t seed, float top_p, float *logits,
                         int32_t *pos_rows, int eos_plus1, bool advance_first)
{
    // uniform position: read from the device counter; ragged: one position per sample, advanced on the device.
    // Every step but the first of a call advances the counters in its first kernel.
    const DecodeArgs a{B, 0, pos_rows ? nullptr : ctr, pos_rows, pos_rows ? 1 : 0, tok, state, tok, logits, nullptr, ts,
                       temperature, seed, top_p, eos_plus1, advance_first ? ctr : nullptr};
    return decode_batch(m, a, ws, ws_bytes, st);
}

static int generate_common(srm_model *m, int64_t B, int32_t pos0, int32_t G, int32_t *d_tok, void *d_state,
                           int32_t *d_tokens_out, float temperature, uint32_t seed, float top_p, float *d_logits,
                           void *d_workspace, size_t workspace_bytes, void *hip_stream, int32_t *d_pos = nullptr,
                           int eos_plus1 = 0)
{
    if (!m || !d_tok || !d_state || !d_tokens_out || !d_workspace) return fail(SRM_EINVAL, "srm_generate: null argument");
    if (!(top_p > 0.0f)) return fail(SRM_EINVAL, "srm_generate: top_p must be > 0");
    const bool topp = temperature > 0.0f && top_p < 1.0f;
    if (topp && !d_logits) return fail(SRM_EINVAL, "srm_generate: top_p < 1 needs a logits buffer");
    if (!topp) { d_logits = nullptr; top_p = 1.0f; }
    if (B <= 0 || B >= (1 << 30)) return fail(SRM_EINVAL, "srm_generate: batch %lld out of range", (long long)B);
    if (G <= 0) return fail(SRM_EINVAL, "srm_generate: G must be positive");
    if (!(temperature >= 0.0f)) return fail(SRM_EINVAL, "srm_generate: temperature must be >= 0");
    if (!d_pos && (pos0 < 0 || (int64_t)pos0 + G > m->cfg.n_ctx))
        return fail(SRM_EINVAL, "srm_generate: positions %d..%lld outside [0, %d)", pos0, (long long)pos0 + G - 1,
                    m->cfg.n_ctx);
    // the step counters live in the last 256 bytes of the workspace, whatever rows the rest is cut into
    if (workspace_bytes < 512) return fail(SRM_ENOMEM, "srm_generate: workspace too small");
    const size_t ws_bytes = workspace_bytes / 256 * 256;          // counters in its last 256 bytes
    if (decode_rows_per_pass(m, B, ws_bytes) <= 0)
        return fail(SRM_ENOMEM, "srm_generate: workspace %zu bytes holds fewer than %lld rows", workspace_bytes,
                    (long long)std::min<int64_t>(B, 256));
    SRM_TRY(check_device(m));
    hipStream_t st = as_stream(hip_stream);
    if (!topp && !d_pos && !eos_plus1 && srm_workspace_bytes(m, B) <= ws_bytes) {
        const int nblk = mega_blocks(m, B);
        if (nblk > 0)
            return mega_generate(m, (int)B, pos0, G, d_tok, d_state, d_tokens_out, temperature, seed, d_workspace, nblk, st);
    }
    int *ctr = reinterpret_cast<int *>(static_cast<unsigned char *>(d_workspace) + ws_bytes - 256);
    const TokenStore ts{d_tokens_out, ctr + 1, B};
    hipLaunchKernelGGL(counters_set_kernel, dim3(1), dim3(1), 0, st, ctr, pos0, 0);
    HIP_TRY(hipGetLastError());
    // first step eagerly (it also performs every one-time kernel attribute set-up)
    SRM_TRY(generate_step(m, B, d_tok, d_state, d_workspace, ws_bytes, ctr, ts, st, temperature, seed, top_p, d_logits,
                          d_pos, eos_plus1, false));
    if (G == 1) return SRM_OK;
    // The legacy default stream cannot be captured: loop eagerly there.
    if (st == nullptr) {
        for (int g = 1; g < G; ++g)
            SRM_TRY(generate_step(m, B, d_tok, d_state, d_workspace, ws_bytes, ctr, ts, st, temperature, seed, top_p,
                                  d_logits, d_pos, eos_plus1, true));
        return SRM_OK;
    }
    const bool hit = m->gexec && m->gkey.B == B && m->gkey.tok == d_tok && m->gkey.state == d_state &&
                     m->gkey.store == d_tokens_out && m->gkey.ws == d_workspace && m->gkey.temp == temperature &&
                     m->gkey.seed == seed && m->gkey.top_p == top_p && m->gkey.logits == d_logits &&
                     m->gkey.ws_bytes == workspace_bytes && m->gkey.pos == d_pos && m->gkey.eos_plus1 == eos_plus1;
    if (!hit) {
        if (m->gexec) { (void)hipGraphExecDestroy(m->gexec); m->gexec = nullptr; }
        hipGraph_t graph = nullptr;
        HIP_TRY(hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal));
        const int rc = generate_step(m, B, d_tok, d_state, d_workspace, ws_bytes, ctr, ts, st, temperature, seed, top_p,
                                     d_logits, d_pos, eos_plus1, true);
        const hipError_t e = hipStreamEndCapture(st, &graph);
        if (rc != SRM_OK) { if (graph) (void)hipGraphDestroy(graph); return rc; }
        if (e != hipSuccess) return fail(SRM_EHIP, "srm_generate: stream capture failed: %s", hipGetErrorString(e));
        const hipError_t e2 = hipGraphInstantiate(&m->gexec, graph, nullptr, nullptr, 0);
        (void)hipGraphDestroy(graph);
        if (e2 != hipSuccess) { m->gexec = nullptr; return fail(SRM_EHIP, "srm_generate: hipGraphInstantiate: %s", hipGetErrorString(e2)); }
        m->gkey = {B, d_tok, d_state, d_tokens_out, d_workspace, temperature, seed, top_p, d_logits, workspace_bytes,
                   d_pos, eos_plus1};
        // the captured step was recorded, not run: replay it G - 1 times below
    }
    for (int g = 1; g < G; ++g) HIP_TRY(hipGraphLaunch(m->gexec, st));
    return SRM_OK;
}

extern "C" int srm_generate(srm_model *m, int64_t B, int32_t pos0, int32_t G, int32_t *d_tok, void *d_state,
                            int32_t *d_tokens_out, float temperature, uint32_t seed, void *d_workspace,
                            size_t workspace_bytes, void *hip_stream)
{
    return generate_common(m, B, pos0, G, d_tok, d_state, d_tokens_out, temperature, seed, 1.0f, nullptr, d_workspace,
                           workspace_bytes, hip_stream);
}

extern "C" int srm_generate_topp(srm_model *m, int64_t B, int32_t pos0, int32_t G, int32_t *d_tok, void *d_state,
                                 int32_t *d_tokens_out, float temperature, float top_p, uint32_t seed,
                                 float *d_logits, void *d_workspace, size_t workspace_bytes, void *hip_stream)
{
    return generate_common(m, B, pos0, G, d_tok, d_state, d_tokens_out, temperature, seed, top_p, d_logits,
                           d_workspace, workspace_bytes, hip_stream);
}

extern "C" int srm_generate_ragged(srm_model *m, int64_t B, int32_t G, int32_t *d_pos, int32_t *d_tok, void *d_state,
                                   int32_t *d_tokens_out, int32_t eos_id, float temperature, float top_p,
                                   uint32_t seed, float *d_logits, void *d_workspace, size_t workspace_bytes,
                                   void *hip_stream)
{
    if (!d_pos) return fail(SRM_EINVAL, "srm_generate_ragged: null argument");
    if (m && eos_id >= m->V) return fail(SRM_EINVAL, "srm_generate_ragged: eos_id %d outside the vocabulary", eos_id);
    return generate_common(m, B, 0, G, d_tok, d_state, d_tokens_out, temperature, seed, top_p, d_logits, d_workspace,
                           workspace_bytes, hip_stream, d_pos, eos_id >= 0 ? eos_id + 1 : 0);
}

// ------------------------------------------------------------------ prefill
// Whole sequences per pass that fit the workspace (0 if not even one does).
static int64_t seqs_per_pass(const srm_model *m, size_t workspace_bytes, int T, int64_t nseq)
{
    if (srm_workspace_bytes(m, T) > workspace_bytes) return 0;
    int64_t lo = 1, hi = nseq;       // largest n with bytes(n*T) <= workspace_bytes
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) / 2;
        if (srm_workspace_bytes(m, mid * T) <= workspace_bytes) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// Chunk length of the chunked scan for a call with nseq sequences of up to P
// positions, or 0 for the sequential kernel.  Chunks are used only while the
// sequential kernel (one thread per sequence and 4 channels) would leave the
// chip mostly idle; the choice depends on the whole call, not on how the
// workspace cuts it into passes, so results do not depend on the workspace size.
static int scan_chunk_len(const srm_model *m, int64_t nseq, int P)
{
    const int64_t dv = m->dm / 4;
    if (P < 64 || nseq * dv >= 65536 || m->shalf) return 0;   // a half-precision cache is rounded at every step
    for (int c : {16, 32, 64, 128}) {
        const int64_t nch = cdiv(P, c);
        if (nch < 2) break;
        if (nseq * dv * nch <= 262144) return c;
    }
    return 0;
}

// The chunked scan keeps its per-chunk partial states F [nc][nchunks][dm] fp32 in the pass's MLP buffer
// w.g ([rows][ff] activation elements, free until the layer's MLP): whether they fit there.
static bool scan_scratch_fits(const srm_model *m, int64_t nc, int nchunks, int64_t rows)
{
    return (size_t)nc * (size_t)nchunks * (size_t)m->dm * sizeof(float) <= (size_t)rows * (size_t)m->ff * m->wsize;
}

// How srm_prefill_ragged cuts packed prompts into passes of whole prompts that fit max_rows workspace rows,
// and which mixer scan the call takes: the chunked one only if its partial states fit the MLP buffer in
// EVERY pass (many short prompts next to a long one do not: the chunk count follows the longest prompt of
// the call, the buffer the rows of the pass), so that one call uses one kind of scan whatever the workspace.
struct RaggedPlan {
    std::vector<int> first;        // first prompt of each pass, then N
    int chunk = 0, nchunks = 1;    // the scan taken (chunk 0: sequential)
    int chunk_by_shape = 0;        // what (N, longest prompt) alone would choose
    size_t need = 0, room = 0;     // tightest pass under chunk_by_shape: bytes of F, bytes of w.g
};
static RaggedPlan plan_ragged(const srm_model *m, const int32_t *h_off, int N, int64_t max_rows, int pmax_call)
{
    RaggedPlan pl;
    pl.chunk_by_shape = scan_chunk_len(m, N, pmax_call);
    const int nch = pl.chunk_by_shape ? (int)cdiv(pmax_call, pl.chunk_by_shape) : 1;
    bool fits = true;
    int n0 = 0;
    while (n0 < N) {
        int n1 = n0;
        while (n1 < N && (int64_t)h_off[n1 + 1] - h_off[n0] <= max_rows) ++n1;
        if (n1 == n0) break;                          // a prompt longer than the workspace: rejected by the caller
        pl.first.push_back(n0);
        if (pl.chunk_by_shape) {
            const int64_t nc = n1 - n0, rows = (int64_t)h_off[n1] - h_off[n0];
            const size_t need = (size_t)nc * nch * m->dm * sizeof(float), room = (size_t)rows * m->ff * m->wsize;
            if (!scan_scratch_fits(m, nc, nch, rows)) fits = false;
            if (pl.room == 0 || (double)need * (double)pl.room > (double)pl.need * (double)room) { pl.need = need; pl.room = room; }
        }
        n0 = n1;
    }
    pl.first.push_back(N);
    if (pl.chunk_by_shape && fits) { pl.chunk = pl.chunk_by_shape; pl.nchunks = nch; }
    return pl;
}

// The mixer of one prefill pass: nc sequences in rows of w.u -> w.mx, final states to S_layer.
template <typename T>
static int prefill_mixer(const srm_model *m, int l, const Workspace &w, void *S_layer, int nc, int P, int chunk,
                         int nchunks, const int32_t *offsets, int64_t base, int64_t rows, int64_t seq0, int rep,
                         const int32_t *slot, int64_t nslots, hipStream_t st)
{
    const LayerDev &y = m->layers[l];
    const int d = m->dm;           // the mixer's row width
    if (chunk > 0) {
        float *F = static_cast<float *>(w.g);       // free until the MLP of this layer
        const unsigned nb = (unsigned)cdiv((int64_t)nc * nchunks * (d / 4), 256);
        hipLaunchKernelGGL((scan_chunk_partials_kernel<T>), dim3(nb), dim3(256), 0, st, static_cast<const T *>(w.u), F,
                           y.alpha, y.lam, m->cfg.n_ctx, m->Hs, m->hrow, d, nc, P, chunk, nchunks, offsets, base, rows, seq0);
        HIP_TRY(hipGetLastError());
        hipLaunchKernelGGL((scan_chunk_apply_kernel<T>), dim3(nb), dim3(256), 0, st, static_cast<const T *>(w.u),
                           static_cast<T *>(w.mx), static_cast<float *>(S_layer), F, y.alpha, y.beta, y.lam,
                           m->cfg.n_ctx, m->Hs, m->hrow, d, nc, P, chunk, nchunks, offsets, base, rows, seq0, rep, slot, nslots);
        HIP_TRY(hipGetLastError());
        return SRM_OK;
    }
    const unsigned nb = (unsigned)cdiv((int64_t)nc * (d / 4), 256);
    const size_t scan_lds = (size_t)2 * m->Hs * P * sizeof(float);
#define SCAN_LAUNCH(TS)                                                                                        \
    do {                                                                                                       \
        if (offsets)                                                                                           \
            hipLaunchKernelGGL((mixer_scan_ragged_kernel<T, TS>), dim3(nb), dim3(256), scan_lds, st,           \
                               static_cast<const T *>(w.u), static_cast<T *>(w.mx), static_cast<TS *>(S_layer), \
                               y.alpha, y.beta, y.lam, m->cfg.n_ctx, m->Hs, m->hrow, d, nc, P, offsets, base, rows, seq0, \
                               rep, slot, nslots);                                                             \
        else                                                                                                   \
            hipLaunchKernelGGL((mixer_scan_kernel<T, TS>), dim3(nb), dim3(256), scan_lds, st,                  \
                               static_cast<const T *>(w.u), static_cast<T *>(w.mx), static_cast<TS *>(S_layer), \
                               y.alpha, y.beta, y.lam, m->cfg.n_ctx, m->Hs, m->hrow, d, nc, P, seq0, rep);     \
    } while (0)
    if (m->shalf) SCAN_LAUNCH(f16);
    else SCAN_LAUNCH(float);
#undef SCAN_LAUNCH
    HIP_TRY(hipGetLastError());
    return SRM_OK;
}

template <typename T>
static int prefill_impl(srm_model *m, const int32_t *prompts, int N, int P, int k, void *state,
                        int32_t *next_tok, float *logits, void *ws, int64_t per_pass, int chunk, hipStream_t st)
{
    const int d = m->d;
    const int64_t Btot = (int64_t)N * k;
    const int nchunks = chunk ? (int)cdiv(P, chunk) : 1;
    for (int64_t n0 = 0; n0 < N; n0 += per_pass) {
        const int64_t nc = std::min<int64_t>(per_pass, N - n0);
        const int64_t rows = nc * P;
        const Workspace w = carve(m, ws, rows);
        SRM_TRY((layernorm<T, true>(m, nullptr, 0, prompts + n0 * P, w.x, m->layers[0].ln1_g,
                                    m->layers[0].ln1_b, w.a, rows, st)));
        auto mix = [&](int l) {
            return prefill_mixer<T>(m, l, w, layer_state(m, state, l, Btot), (int)nc, P, chunk, nchunks, nullptr, 0, rows,
                                    n0, k, nullptr, 0, st);
        };
        for (int l = 0; l < m->L; ++l) SRM_TRY((block<T>(m, l, w, rows, st, mix, l + 1 < m->L)));
        // final LayerNorm of each prompt's last position only, packed [nc][d] into w.a
        SRM_TRY((layernorm<T, false>(m, w.x + (size_t)(P - 1) * d, (int64_t)P * d, nullptr, nullptr, m->lnf_g,
                                     m->lnf_b, w.a, nc, st)));
        SRM_TRY((head_argmax<T>(m, w, w.a, nc, logits ? logits + (size_t)n0 * m->V : nullptr, next_tok, n0, k, st)));
    }
    return SRM_OK;
}

extern "C" int srm_prefill(srm_model *m, const int32_t *d_prompts, int32_t N, int32_t P, int32_t fanout_k,
                           void *d_state, int32_t *d_next_tok, float *d_logits, void *d_workspace,
                           size_t workspace_bytes, void *hip_stream)
{
    if (!m || !d_prompts || !d_state || !d_next_tok || !d_workspace)
        return fail(SRM_EINVAL, "srm_prefill: null argument");
    if (N <= 0 || P <= 0 || fanout_k <= 0) return fail(SRM_EINVAL, "srm_prefill: N, P and fanout_k must be positive");
    if (P > m->cfg.n_ctx) return fail(SRM_EINVAL, "srm_prefill: P = %d exceeds n_ctx = %d", P, m->cfg.n_ctx);
    if ((int64_t)N * fanout_k >= (1 << 30)) return fail(SRM_EINVAL, "srm_prefill: N * fanout_k too large");
    // the chunked scan where the call's shape asks for it and its partial states fit the MLP buffer of a pass
    // (rows = prompts x P there, so the test does not depend on how many prompts a pass holds)
    int chunk = scan_chunk_len(m, N, P);
    if (chunk && !scan_scratch_fits(m, 1, (int)cdiv(P, chunk), P)) chunk = 0;
    if (!chunk && (size_t)2 * m->Hs * P * sizeof(float) > 64 * 1024)   // the sequential scan stages its coefficients in LDS
        return fail(SRM_EINVAL, "srm_prefill: n_heads * P too large for the coefficient stage");
    const int64_t max_seqs = std::max<int64_t>(1, ((1 << 30) - 1) / P);
    int64_t per_pass = seqs_per_pass(m, workspace_bytes, P, std::min<int64_t>(N, max_seqs));
    if (per_pass < 1)
        return fail(SRM_ENOMEM, "srm_prefill: workspace %zu < %zu bytes (one prompt)", workspace_bytes,
                    srm_workspace_bytes(m, P));
    SRM_TRY(check_device(m));
    hipStream_t st = as_stream(hip_stream);
    return m->wsize == 2 ? prefill_impl<bf16>(m, d_prompts, N, P, fanout_k, d_state, d_next_tok, d_logits,
                                              d_workspace, per_pass, chunk, st)
                         : prefill_impl<float>(m, d_prompts, N, P, fanout_k, d_state, d_next_tok, d_logits,
                                               d_workspace, per_pass, chunk, st);
}

// ------------------------------------------------------------------ prefill of packed ragged prompts
template <typename T>
static int prefill_ragged_impl(srm_model *m, const int32_t *tokens, const int32_t *h_off, const int32_t *d_off, int N,
                               int k, const int32_t *slot, int64_t state_batch, void *state, int32_t *next_tok,
                               int32_t *pos_out, float *logits, void *ws, const RaggedPlan &plan, int pmax_call,
                               hipStream_t st)
{
    const int d = m->d;
    const int chunk = plan.chunk, nchunks = plan.nchunks;
    for (size_t pass = 0; pass + 1 < plan.first.size(); ++pass) {
        // as many whole prompts as the workspace holds
        const int n0 = plan.first[pass], n1 = plan.first[pass + 1];
        int pmax = 0;
        for (int n = n0; n < n1; ++n) pmax = std::max(pmax, h_off[n + 1] - h_off[n]);
        const int nc = n1 - n0;
        const int64_t base = h_off[n0], rows = (int64_t)h_off[n1] - base;
        const Workspace w = carve(m, ws, rows);
        SRM_TRY((layernorm<T, true>(m, nullptr, 0, tokens + base, w.x, m->layers[0].ln1_g, m->layers[0].ln1_b, w.a,
                                    rows, st)));
        auto mix = [&](int l) {
            return prefill_mixer<T>(m, l, w, layer_state(m, state, l, state_batch), nc, chunk ? pmax_call : pmax, chunk,
                                    nchunks, d_off, base, rows, (int64_t)n0, k, slot, state_batch, st);
        };
        for (int l = 0; l < m->L; ++l) SRM_TRY((block<T>(m, l, w, rows, st, mix, l + 1 < m->L)));
        // final LayerNorm of each prompt's last row, packed [nc][d] into w.a
        SRM_TRY((layernorm<T, false>(m, w.x, d, nullptr, nullptr, m->lnf_g, m->lnf_b, w.a, nc, st, d_off + n0, base,
                                     rows)));
        FinalizeRagged rg{};
        rg.slot = slot;
        rg.nslots = state_batch;
        rg.offsets = d_off;
        rg.pos_set = pos_out;
        SRM_TRY((head_argmax<T>(m, w, w.a, nc, logits ? logits + (size_t)n0 * m->V : nullptr, next_tok, n0, k, st,
                                TokenStore(), Sampling(), rg)));
    }
    return SRM_OK;
}

// Host-side checks of a packed prompt list against a model and a workspace size: every length within
// [1, n_ctx] and within the rows the workspace holds; returns those rows and the longest prompt.
static int ragged_lengths(const char *who, const srm_model *m, const int32_t *h_offsets, int N, size_t workspace_bytes,
                          int64_t &max_rows, int &pmax)
{
    if (h_offsets[0] < 0) return fail(SRM_EINVAL, "%s: offsets[0] is negative", who);
    // rows the workspace holds (largest r with srm_workspace_bytes(r) <= workspace_bytes)
    int64_t lo = 0, hi = (1 << 30) - 1;
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) / 2;
        if (srm_workspace_bytes(m, mid) <= workspace_bytes) lo = mid; else hi = mid - 1;
    }
    max_rows = lo;
    pmax = 0;
    for (int n = 0; n < N; ++n) {
        const int64_t len = (int64_t)h_offsets[n + 1] - h_offsets[n];
        if (len < 1 || len > m->cfg.n_ctx)
            return fail(SRM_EINVAL, "%s: prompt %d has length %lld outside [1, n_ctx = %d]", who, n, (long long)len,
                        m->cfg.n_ctx);
        if (len > max_rows)
            return fail(SRM_ENOMEM, "%s: workspace %zu < %zu bytes (prompt %d of %lld tokens)", who, workspace_bytes,
                        srm_workspace_bytes(m, len), n, (long long)len);
        pmax = std::max(pmax, (int)len);
    }
    return SRM_OK;
}

extern "C" int srm_prefill_ragged(srm_model *m, const int32_t *d_tokens, const int32_t *h_offsets,
                                  const int32_t *d_offsets, int32_t N, int32_t fanout_k, const int32_t *d_slot,
                                  int64_t state_batch, void *d_state, int32_t *d_next_tok, int32_t *d_pos,
                                  float *d_logits, void *d_workspace, size_t workspace_bytes, void *hip_stream)
{
    const char *who = "srm_prefill_ragged";
    if (!m || !d_tokens || !h_offsets || !d_offsets || !d_state || !d_next_tok || !d_workspace)
        return fail(SRM_EINVAL, "%s: null argument", who);
    if (N <= 0 || fanout_k <= 0) return fail(SRM_EINVAL, "%s: N and fanout_k must be positive", who);
    if (d_slot && fanout_k != 1) return fail(SRM_EINVAL, "%s: a slot list needs fanout_k = 1", who);
    if (state_batch <= 0 || state_batch >= (1 << 30)) return fail(SRM_EINVAL, "%s: state_batch out of range", who);
    if (!d_slot && (int64_t)N * fanout_k > state_batch)
        return fail(SRM_EINVAL, "%s: N * fanout_k = %lld exceeds state_batch = %lld", who, (long long)N * fanout_k,
                    (long long)state_batch);
    int64_t max_rows = 0;
    int pmax = 0;
    SRM_TRY(ragged_lengths(who, m, h_offsets, N, workspace_bytes, max_rows, pmax));
    const RaggedPlan plan = plan_ragged(m, h_offsets, N, max_rows, pmax);
    if (!plan.chunk && (size_t)2 * m->Hs * pmax * sizeof(float) > 64 * 1024)   // the sequential scan's coefficient stage
        return fail(SRM_EINVAL, "%s: n_heads * longest prompt too large for the coefficient stage", who);
    SRM_TRY(check_device(m));
    hipStream_t st = as_stream(hip_stream);
    return m->wsize == 2 ? prefill_ragged_impl<bf16>(m, d_tokens, h_offsets, d_offsets, N, fanout_k, d_slot,
                                                     state_batch, d_state, d_next_tok, d_pos, d_logits, d_workspace,
                                                     plan, pmax, st)
                         : prefill_ragged_impl<float>(m, d_tokens, h_offsets, d_offsets, N, fanout_k, d_slot,
                                                      state_batch, d_state, d_next_tok, d_pos, d_logits, d_workspace,
                                                      plan, pmax, st);
}

extern "C" size_t srm_workspace_bytes_config(const srm_config *cfg, int64_t rows)
{
    if (!cfg || rows <= 0) return 0;
    srm_model m;
    if (model_geometry("srm_workspace_bytes_config", cfg, &m) != SRM_OK) return 0;
    return carve(&m, nullptr, rows).bytes;
}

extern "C" int srm_prefill_ragged_plan(const srm_config *cfg, const int32_t *h_offsets, int32_t N,
                                       size_t workspace_bytes, srm_prefill_plan *out)
{
    const char *who = "srm_prefill_ragged_plan";
    if (!cfg || !h_offsets || !out) return fail(SRM_EINVAL, "%s: null argument", who);
    if (N <= 0) return fail(SRM_EINVAL, "%s: N must be positive", who);
    srm_model m;
    SRM_TRY(model_geometry(who, cfg, &m));
    int64_t max_rows = 0;
    int pmax = 0;
    SRM_TRY(ragged_lengths(who, &m, h_offsets, N, workspace_bytes, max_rows, pmax));
    const RaggedPlan plan = plan_ragged(&m, h_offsets, N, max_rows, pmax);
    out->passes = (int32_t)plan.first.size() - 1;
    out->chunk_len = plan.chunk;
    out->chunk_len_by_shape = plan.chunk_by_shape;
    out->n_chunks = plan.chunk_by_shape ? (int32_t)cdiv(pmax, plan.chunk_by_shape) : 1;
    out->scratch_need = plan.need;
    out->scratch_room = plan.room;
    return SRM_OK;
}

// ------------------------------------------------------------------ parallel form
template <typename T>
static int parallel_impl(srm_model *m, const int32_t *tok, int B, int T_, float *hidden, float *logits, void *ws,
                         int64_t per_pass, hipStream_t st)
{
    const int d = m->d, dm = m->dm, dh = dm / m->Hs;
    for (int64_t b0 = 0; b0 < B; b0 += per_pass) {
        const int64_t nc = std::min<int64_t>(per_pass, B - b0);
        const int64_t rows = nc * T_;
        const Workspace w = carve(m, ws, rows);
        SRM_TRY((layernorm<T, true>(m, nullptr, 0, tok + b0 * T_, w.x, m->layers[0].ln1_g, m->layers[0].ln1_b,
                                    w.a, rows, st)));
        auto mix = [&](int l) {
            const LayerDev &y = m->layers[l];
            const dim3 grid((unsigned)cdiv(T_, 64), (unsigned)(m->Hs * cdiv(dh, 64)), (unsigned)nc);
            hipLaunchKernelGGL((mixer_parallel_kernel<T>), grid, dim3(256), (size_t)T_ * sizeof(float), st,
                               static_cast<const T *>(w.u), static_cast<T *>(w.mx), y.alpha, y.beta, y.lam,
                               m->cfg.n_ctx, m->Hs, m->hrow, dm, T_);
            HIP_TRY(hipGetLastError());
            return (int)SRM_OK;
        };
        for (int l = 0; l < m->L; ++l) SRM_TRY((block<T>(m, l, w, rows, st, mix, true)));
        HIP_TRY(hipMemcpyAsync(hidden + (size_t)b0 * T_ * d, w.x, (size_t)rows * d * 4, hipMemcpyDeviceToDevice, st));
        if (logits)
            SRM_TRY((linear<EPI_F32, T>(w.a, m->head, nullptr, rows, m->V, d, logits + (size_t)b0 * T_ * m->V, st)));
    }
    return SRM_OK;
}

extern "C" int srm_parallel_forward(srm_model *m, const int32_t *d_tok, int32_t B, int32_t T, float *d_hidden,
                                    float *d_logits, void *d_workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!m || !d_tok || !d_hidden || !d_workspace) return fail(SRM_EINVAL, "srm_parallel_forward: null argument");
    if (B <= 0 || T <= 0) return fail(SRM_EINVAL, "srm_parallel_forward: B and T must be positive");
    if (T > m->cfg.n_ctx) return fail(SRM_EINVAL, "srm_parallel_forward: T = %d exceeds n_ctx = %d", T, m->cfg.n_ctx);
    if ((size_t)T * sizeof(float) > 32 * 1024) return fail(SRM_EINVAL, "srm_parallel_forward: T too large");
    if (B > 65535) return fail(SRM_EINVAL, "srm_parallel_forward: B > 65535");
    const int64_t max_seqs = std::max<int64_t>(1, ((1 << 30) - 1) / T);
    int64_t per_pass = seqs_per_pass(m, workspace_bytes, T, std::min<int64_t>(B, max_seqs));
    if (per_pass < 1)
        return fail(SRM_ENOMEM, "srm_parallel_forward: workspace %zu < %zu bytes (one sequence)", workspace_bytes,
                    srm_workspace_bytes(m, T));
    SRM_TRY(check_device(m));
    hipStream_t st = as_stream(hip_stream);
    return m->wsize == 2
               ? parallel_impl<bf16>(m, d_tok, B, T, d_hidden, d_logits, d_workspace, per_pass, st)
               : parallel_impl<float>(m, d_tok, B, T, d_hidden, d_logits, d_workspace, per_pass, st);
}

// ------------------------------------------------------------------ kernel-level entry points
extern "C" int srm_mixer_update(srm_model *m, int32_t layer, int32_t pos, int64_t B, const void *d_u,
                                void *d_state_layer, void *d_m, void *hip_stream)
{
    if (!m || !d_u || !d_state_layer || !d_m) return fail(SRM_EINVAL, "srm_mixer_update: null argument");
    if (layer < 0 || layer >= m->L) return fail(SRM_EINVAL, "srm_mixer_update: layer %d outside [0, %d)", layer, m->L);
    if (pos < 0 || pos >= m->cfg.n_ctx) return fail(SRM_EINVAL, "srm_mixer_update: pos %d outside [0, %d)", pos, m->cfg.n_ctx);
    if (B <= 0 || B >= (1 << 30)) return fail(SRM_EINVAL, "srm_mixer_update: batch out of range");
    SRM_TRY(check_device(m));
    hipStream_t st = as_stream(hip_stream);
    return m->wsize == 2 ? state_update<bf16>(m, layer, pos, B, d_u, d_state_layer, d_m, st)
                         : state_update<float>(m, layer, pos, B, d_u, d_state_layer, d_m, st);
}

extern "C" int srm_mixer_project_update(srm_model *m, int32_t layer, int32_t pos, int64_t B, const void *d_a,
                                        void *d_state_layer, void *d_m, void *hip_stream)
{
    if (!m || !d_a || !d_state_layer || !d_m) return fail(SRM_EINVAL, "srm_mixer_project_update: null argument");
    if (m->noproj) return fail(SRM_EINVAL, "srm_mixer_project_update: the model has no head projections");
    if (layer < 0 || layer >= m->L)
        return fail(SRM_EINVAL, "srm_mixer_project_update: layer %d outside [0, %d)", layer, m->L);
    if (pos < 0 || pos >= m->cfg.n_ctx)
        return fail(SRM_EINVAL, "srm_mixer_project_update: pos %d outside [0, %d)", pos, m->cfg.n_ctx);
    if (B <= 0 || B >= (1 << 30)) return fail(SRM_EINVAL, "srm_mixer_project_update: batch out of range");
    SRM_TRY(check_device(m));
    hipStream_t st = as_stream(hip_stream);
    const LayerDev &y = m->layers[layer];
    const MixArgs mx{d_state_layer, y.alpha, y.beta, y.lam, m->cfg.n_ctx, m->hrow, m->dm / m->Hs, m->shalf ? 1 : 0};
    Sampling where;
    where.pos = pos;
    return m->wsize == 2 ? linear<EPI_MIX, bf16>(d_a, y.w_in, y.b_in, B, m->dm, m->d, d_m, st, nullptr, nullptr, 64,
                                                 nullptr, where, 1, mx)
                         : linear<EPI_MIX, float>(d_a, y.w_in, y.b_in, B, m->dm, m->d, d_m, st, nullptr, nullptr, 64,
                                                  nullptr, where, 1, mx);
}

extern "C" int srm_mixer_block(srm_model *m, int32_t layer, int32_t pos, const int32_t *d_pos_rows, int64_t B,
                               float *d_x, void *d_state_layer, void *d_norm_out, float *d_slabs, void *hip_stream)
{
    if (!m || !d_x || !d_state_layer || !d_norm_out || !d_slabs) return fail(SRM_EINVAL, "srm_mixer_block: null argument");
    if (!token_mix_shape_ok(m))
        return fail(SRM_EINVAL, "srm_mixer_block: needs bf16 weights, head projections of width d and d = 256 or 512");
    if (layer < 0 || layer >= m->L) return fail(SRM_EINVAL, "srm_mixer_block: layer %d outside [0, %d)", layer, m->L);
    if (!d_pos_rows && (pos < 0 || pos >= m->cfg.n_ctx))
        return fail(SRM_EINVAL, "srm_mixer_block: pos %d outside [0, %d)", pos, m->cfg.n_ctx);
    if (B <= 0 || B >= (1 << 26)) return fail(SRM_EINVAL, "srm_mixer_block: batch out of range");
    SRM_TRY(check_device(m));
    hipStream_t st = as_stream(hip_stream);
    Sampling where;
    where.pos = pos;
    where.pos_rows = d_pos_rows;
    SRM_TRY(token_mix(m, layer, TokMixCall{d_x, SlabArgs(), d_state_layer, where, d_slabs}, B, st));
    const LayerDev &y = m->layers[layer];
    return layernorm<bf16, false>(m, d_x, m->d, nullptr, d_x, y.ln2_g, y.ln2_b, d_norm_out, B, st, nullptr, 0, 0, d_slabs,
                                  m->d / kTokMixCols);
}

extern "C" int srm_sample_logits(const float *d_logits, int64_t rows, int32_t vocab, float temperature, float top_p,
                                 uint32_t seed, int32_t pos, int32_t *d_tok_out, void *hip_stream)
{
    if (!d_logits || !d_tok_out) return fail(SRM_EINVAL, "srm_sample_logits: null argument");
    if (rows <= 0 || rows >= (1 << 30) || vocab <= 0) return fail(SRM_EINVAL, "srm_sample_logits: sizes out of range");
    if (!(temperature > 0.0f)) return fail(SRM_EINVAL, "srm_sample_logits: temperature must be > 0");
    if (!(top_p > 0.0f)) return fail(SRM_EINVAL, "srm_sample_logits: top_p must be > 0");
    hipLaunchKernelGGL((nucleus_kernel<256, true, false>), dim3((unsigned)rows), dim3(256), 0, as_stream(hip_stream),
                       d_logits, (int64_t)vocab, vocab, temperature, top_p, seed, pos, nullptr, nullptr, d_tok_out,
                       nullptr, nullptr, (int64_t)0, nullptr, nullptr, nullptr, 0u);
    HIP_TRY(hipGetLastError());
    return SRM_OK;
}

extern "C" int srm_probe_copy(void *d_dst, const void *d_src, size_t bytes, int32_t streaming, void *hip_stream)
{
    if (!d_dst || !d_src) return fail(SRM_EINVAL, "srm_probe_copy: null argument");
    if (bytes == 0 || bytes % 16 || ((uintptr_t)d_dst | (uintptr_t)d_src) % 16)
        return fail(SRM_EINVAL, "srm_probe_copy: size and pointers must be multiples of 16 bytes");
    constexpr int U = 4;
    const int64_t n16 = (int64_t)(bytes / 16);
    const int64_t blocks = cdiv(n16, 256 * U);
    if (blocks >= (1ll << 31)) return fail(SRM_EINVAL, "srm_probe_copy: at most 32 TiB per call");
    if (streaming)
        hipLaunchKernelGGL((probe_copy_kernel<U, true>), dim3((unsigned)blocks), dim3(256), 0, as_stream(hip_stream),
                           (const u32x4_t *)d_src, (u32x4_t *)d_dst, n16);
    else
        hipLaunchKernelGGL((probe_copy_kernel<U, false>), dim3((unsigned)blocks), dim3(256), 0, as_stream(hip_stream),
                           (const u32x4_t *)d_src, (u32x4_t *)d_dst, n16);
    HIP_TRY(hipGetLastError());
    return SRM_OK;
}

extern "C" int srm_probe_mfma(float *d_out, int32_t blocks, int32_t iters, int32_t random_operands, double *flop,
                              void *hip_stream)
{
    if (!d_out) return fail(SRM_EINVAL, "srm_probe_mfma: null argument");
    if (blocks <= 0 || blocks > (1 << 20) || iters <= 0 || iters > (1 << 20))
        return fail(SRM_EINVAL, "srm_probe_mfma: blocks and iters must lie in [1, 2^20]");
    hipLaunchKernelGGL(probe_mfma_kernel, dim3((unsigned)blocks), dim3(256), 0, as_stream(hip_stream), d_out, iters, 1.0f,
                       random_operands ? 1 : 0);
    HIP_TRY(hipGetLastError());
    if (flop) *flop = (double)blocks * 4 /*wavefronts*/ * iters * 4 /*tiles*/ * (2.0 * 32 * 32 * 16);
    return SRM_OK;
}

extern "C" void srm_linear_timeline_probe(void *d_u64, int64_t blocks)
{
    g_clock_probe = blocks > 0 ? static_cast<unsigned long long *>(d_u64) : nullptr;
    g_clock_blocks = g_clock_probe ? blocks : 0;
}

extern "C" size_t srm_linear_scratch_bytes(int64_t M, int32_t N)
{
    if (M <= 0 || N <= 0) return 0;
    return align_up((size_t)M * cdiv(N, 64) * 4, 256) * 2;
}

template <typename T>
static int linear_entry(int epilogue, const void *A, const void *W, const float *bias, int64_t M, int N, int K,
                        void *out, int32_t *amax, void *scratch, hipStream_t st)
{
    switch (epilogue) {
    case 0: return linear<EPI_STORE, T>(A, W, bias, M, N, K, out, st);
    case 1: return linear<EPI_GELU, T>(A, W, bias, M, N, K, out, st);
    case 2: return linear<EPI_RESID, T>(A, W, bias, M, N, K, out, st);
    case 3: {
        float *pv = static_cast<float *>(scratch);
        int32_t *pi = reinterpret_cast<int32_t *>(static_cast<unsigned char *>(scratch) +
                                                  align_up((size_t)M * cdiv(N, 64) * 4, 256));
        int nparts = 0;
        SRM_TRY((linear<EPI_ARGMAX, T>(A, W, bias, M, N, K, out, st, pv, pi, 64, &nparts)));
        return argmax_finalize(pv, pi, M, nparts, amax, 0, 1, N, st);
    }
    case 4: return linear<EPI_F32, T>(A, W, bias, M, N, K, out, st);
    default: return fail(SRM_EINVAL, "srm_linear: unknown epilogue %d", epilogue);
    }
}

// ------------------------------------------------------------------ entry point that allocates nothing
// Scratch of srm_linear_argmax_noalloc: the per-column-tile (max, index) partials of the LM-head form,
// [M][ceil(N / 64)] fp32 then the same of int32, in a file-scope device array instead of a caller's
// workspace.  Every GPU the library runs on holds its own copy until the process ends.  In host code the
// array's name is only a handle: its device address is looked up once per device and used from then on.
constexpr size_t kNoallocScratch = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kNoallocScratch];
constexpr int kNoallocMaxDevices = 64;
static void *g_noalloc_ptr[kNoallocMaxDevices];
static std::mutex g_noalloc_mutex;

static int noalloc_scratch(void **out)
{
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kNoallocMaxDevices) return fail(SRM_EINVAL, "srm_linear_argmax_noalloc: device %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_noalloc_mutex);
    if (!g_noalloc_ptr[dev]) {
        void *ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return fail(SRM_EHIP, "srm_linear_argmax_noalloc: no address for the scratch array on device %d", dev);
        g_noalloc_ptr[dev] = ptr;
    }
    *out = g_noalloc_ptr[dev];
    return SRM_OK;
}

extern "C" size_t srm_linear_argmax_noalloc_max_bytes(void) { return kNoallocScratch; }

extern "C" int srm_linear_argmax_noalloc(int32_t dtype, const void *d_A, const void *d_W, const float *d_bias,
                                         int64_t M, int32_t N, int32_t K, int32_t *d_argmax, void *hip_stream)
{
    const char *who = "srm_linear_argmax_noalloc";
    if (!d_A || !d_W || !d_argmax) return fail(SRM_EINVAL, "%s: null argument", who);
    if (M <= 0 || N <= 0 || K <= 0) return fail(SRM_EINVAL, "%s: sizes must be positive", who);
    const size_t need = srm_linear_scratch_bytes(M, N);
    if (need > kNoallocScratch)
        return fail(SRM_EINVAL, "%s: M = %lld rows x N = %d columns need %zu bytes of partial results, the built-in "
                                "scratch holds %zu (use srm_linear with a workspace)", who, (long long)M, N, need,
                    kNoallocScratch);
    void *ptr = nullptr;
    SRM_TRY(noalloc_scratch(&ptr));
    hipStream_t st = as_stream(hip_stream);
    if (dtype == SRM_BF16) return linear_entry<bf16>(3, d_A, d_W, d_bias, M, N, K, nullptr, d_argmax, ptr, st);
    if (dtype == SRM_FP32) return linear_entry<float>(3, d_A, d_W, d_bias, M, N, K, nullptr, d_argmax, ptr, st);
    return fail(SRM_EINVAL, "%s: unknown dtype %d", who, dtype);
}

extern "C" int srm_linear(int32_t dtype, int32_t epilogue, const void *d_A, const void *d_W, const float *d_bias,
                          int64_t M, int32_t N, int32_t K, void *d_out, int32_t *d_argmax, void *d_scratch,
                          void *hip_stream)
{
    if (!d_A || !d_W) return fail(SRM_EINVAL, "srm_linear: null operand");
    // epilogue codes >= 100 pin a bf16 tile, (tile + 1) * 100 + epilogue, for tile sweeps
    int forced = -1;
    if (epilogue >= 100) {
        forced = epilogue / 100 - 1;
        epilogue %= 100;
        if (forced >= kNumTiles || dtype != SRM_BF16) return fail(SRM_EINVAL, "srm_linear: unknown tile code");
    }
    if (epilogue == 3 ? (!d_argmax || !d_scratch) : !d_out) return fail(SRM_EINVAL, "srm_linear: null output");
    if (M <= 0 || N <= 0 || K <= 0) return fail(SRM_EINVAL, "srm_linear: sizes must be positive");
    hipStream_t st = as_stream(hip_stream);
    g_force_tile = forced;
    int rc;
    if (dtype == SRM_BF16) rc = linear_entry<bf16>(epilogue, d_A, d_W, d_bias, M, N, K, d_out, d_argmax, d_scratch, st);
    else if (dtype == SRM_FP32) rc = linear_entry<float>(epilogue, d_A, d_W, d_bias, M, N, K, d_out, d_argmax, d_scratch, st);
    else rc = fail(SRM_EINVAL, "srm_linear: unknown dtype %d", dtype);
    g_force_tile = -1;
    return rc;
}
