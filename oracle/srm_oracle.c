/*
 * srm_oracle.c -- plain CPU oracle for the Structured Recurrent Mixer (SRM).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct
 * statement of what the SRM decode path computes.  Only the tests, the smoke
 * check and the benchmark's cpu_baseline leg may call it; the HIP library
 * shares no code, header, table or helper with it.
 *
 * Compiled twice from this one source: -DREAL=double (the truth build that
 * parity tests compare against) and -DREAL=float (the plain fp32 build that
 * is timed as the CPU baseline).  Every arithmetic step is carried in REAL;
 * libm calls (sqrt, erf, pow) are evaluated in double and rounded to REAL.
 * The only parallelism is OpenMP over independent samples ("Recurrent
 * Throughput and Concurrency": samples are independent).
 *
 * What follows the paper, and where:
 *   - token mixing as Y = X M + B with a triangular, data-independent M
 *     ("Masked Mixer Parameterization");
 *   - row-repeat M (Eq. 1) and its recurrence (Eq. 2); column-repeat M and
 *     its recurrence (Eq. 3); trainable decay lambda in (0.9, 1] per diagonal
 *     ("Architecture");
 *   - "mixed" heads: half the heads row-repeat, half column-repeat, each of
 *     width d/h, concatenated before the out projection; per-head input
 *     projections I_h stacked into one d x d matrix and P_out (Eq. 10);
 *   - cache of d values per layer per sample ("SRM architecture optimization").
 *
 * What the paper leaves open and this oracle therefore DEFINES (each reading
 * is listed in the design notes of this repository):
 *   pre-LN residual blocks with affine LayerNorm (biased variance, eps given
 *   by the caller), exact erf GELU, MLP expansion e, biased linears, untied
 *   embedding / head with no head bias, a final LayerNorm before the head,
 *   alpha and beta scalar per (layer, head, position), one lambda per
 *   (layer, head), heads 0..H/2-1 row-repeat and H/2..H-1 column-repeat,
 *   argmax ties resolved to the lowest index.  The structural part of that
 *   reading (2 affine LNs per layer, biased linears, scalar alpha/beta,
 *   expansion 4, untied embeddings) is pinned by the parameter counts printed
 *   in Tables S1, S3 and S5; see orc_count_params.
 *
 * Pins (tests/test_oracle_pins.py): Eq. 1 worked example for n = 3; literal
 * Eq. 2 / Eq. 3 closed forms; parallel == recurrent on brute-force inputs;
 * cumsum / first-order IIR special cases checked against library routines;
 * rank-1 generator; causality; constant state size; printed parameter counts;
 * the other head layouts (row-only, column-only, combined) against matrices
 * written out entry by entry, running sums and the sum of a row-only and a
 * column-only model; the k-filter mixer (Eq. 11) against the equation written
 * out in the paper's orientation and against a running sum of a library
 * correlation along the hidden dimension.
 * The numerical value of a whole-model logit has no printed example in the
 * paper: for whole-model outputs "parity unpinned" beyond those structural
 * pins and the cross-form identity.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

#ifndef REAL
#define REAL double
#endif
typedef REAL real;

typedef struct {
    real *ln1_g, *ln1_b, *w_in, *b_in, *alpha, *beta, *lam;
    real *w_out, *b_out, *ln2_g, *ln2_b, *w_up, *b_up, *w_down, *b_down;
} orc_layer;

typedef struct {
    int vocab, d, L, H, e, n_ctx;
    int no_proj;        /* 1: non-projected ("head-parallel") mixer layers, see orc_set_projections */
    int half_state;     /* 1: cache and decay constants in half precision, see orc_set_state_half */
    int layout;         /* ORC_MIXED, ORC_ROW, ORC_COLUMN or ORC_COMBINED, see orc_create_layout */
    int kmix;           /* > 1: mixer with that many filters along the hidden dimension, see orc_create_kernel */
    double eps;
    real *embed, *head, *lnf_g, *lnf_b;
    orc_layer *layers;
} orc_model;

/*
 * Head layouts ("Method", the paragraph after Eq. 2 on combining row- and
 * column-repeat outputs; the rows of Table S0):
 *   ORC_MIXED     heads 0..H/2-1 row-repeat, H/2..H-1 column-repeat (H even);
 *   ORC_ROW       every head row-repeat;  ORC_COLUMN  every head column-repeat
 *                 (any H dividing d; H = 1 is the non-headed model);
 *   ORC_COMBINED  every head owns one row-repeat and one column-repeat matrix,
 *                 each with its own alpha, beta, lambda, applied to the same
 *                 input, and the two outputs are added.  Any other fixed linear
 *                 combination is this one with the weights folded into alpha and
 *                 beta.  The cache is twice as large: per layer S[0..d) belongs
 *                 to the row-repeat matrices, S[d..2d) to the column-repeat ones.
 * alpha, beta have one row (lam one entry) per "slot": H slots, or 2H for
 * ORC_COMBINED with slot h = head h's row-repeat matrix and slot H + h its
 * column-repeat matrix.
 */
enum { ORC_MIXED = 0, ORC_ROW = 1, ORC_COLUMN = 2, ORC_COMBINED = 3 };

#define ORC_LAYER_TENSORS 15
#define ORC_GLOBAL_TENSORS 4

int orc_real_bytes(void) { return (int)sizeof(real); }

static real *orc_copy(const float *src, size_t n)
{
    real *dst = (real *)malloc(n * sizeof(real));
    for (size_t i = 0; i < n; ++i) dst[i] = (real)src[i];
    return dst;
}

/*
 * tensors: embed[V][d], head[V][d], lnf_g[d], lnf_b[d], then for each layer
 * ln1_g[d] ln1_b[d] w_in[d][d] b_in[d] alpha[slots][n_ctx] beta[slots][n_ctx] lam[slots]
 * w_out[d][d] b_out[d] ln2_g[d] ln2_b[d] w_up[e*d][d] b_up[e*d]
 * w_down[d][e*d] b_down[d].  All float32, row-major [out][in]; copied.
 */
static orc_model *orc_create_any(int vocab, int d, int L, int H, int e, int n_ctx, double eps, int layout,
                                 int k, const float *const *tensors)
{
    if (vocab <= 0 || d <= 0 || L <= 0 || H <= 0 || (d % H) || e <= 0 || n_ctx <= 0) return NULL;
    if (layout < ORC_MIXED || layout > ORC_COMBINED || (layout == ORC_MIXED && (H % 2))) return NULL;
    orc_model *m = (orc_model *)calloc(1, sizeof(orc_model));
    m->vocab = vocab; m->d = d; m->L = L; m->H = H; m->e = e; m->n_ctx = n_ctx; m->eps = eps;
    m->layout = layout;
    m->kmix = k;
    const int slots = k > 1 ? k * H : layout == ORC_COMBINED ? 2 * H : H;    /* rows of alpha, entries of lam */
    const int bslots = k > 1 ? H : slots;                                    /* rows of beta */
    size_t dd = (size_t)d * d, ff = (size_t)e * d;
    m->embed = orc_copy(tensors[0], (size_t)vocab * d);
    m->head  = orc_copy(tensors[1], (size_t)vocab * d);
    m->lnf_g = orc_copy(tensors[2], d);
    m->lnf_b = orc_copy(tensors[3], d);
    m->layers = (orc_layer *)calloc(L, sizeof(orc_layer));
    for (int l = 0; l < L; ++l) {
        const float *const *t = tensors + ORC_GLOBAL_TENSORS + (size_t)l * ORC_LAYER_TENSORS;
        orc_layer *y = &m->layers[l];
        y->ln1_g = orc_copy(t[0], d);            y->ln1_b = orc_copy(t[1], d);
        y->w_in  = orc_copy(t[2], dd);           y->b_in  = orc_copy(t[3], d);
        y->alpha = orc_copy(t[4], (size_t)slots * n_ctx);
        y->beta  = orc_copy(t[5], (size_t)bslots * n_ctx);
        y->lam   = orc_copy(t[6], slots);
        y->w_out = orc_copy(t[7], dd);           y->b_out = orc_copy(t[8], d);
        y->ln2_g = orc_copy(t[9], d);            y->ln2_b = orc_copy(t[10], d);
        y->w_up  = orc_copy(t[11], ff * d);      y->b_up  = orc_copy(t[12], ff);
        y->w_down = orc_copy(t[13], (size_t)d * ff); y->b_down = orc_copy(t[14], d);
    }
    return m;
}

orc_model *orc_create_layout(int vocab, int d, int L, int H, int e, int n_ctx, double eps, int layout,
                             const float *const *tensors)
{
    return orc_create_any(vocab, d, L, H, e, n_ctx, eps, layout, 1, tensors);
}

/*
 * Mixer with k filters along the hidden dimension (Eq. 11 and the paragraph
 * above it): Y = sum_i X_(i:d+i, :) W_i + beta, X zero-padded in the hidden
 * dimension, every W_i a column-repeat matrix (Eq. 3).  Reading defined here
 * (the text leaves these open): k filters i = 0..k-1; the padding follows the
 * last hidden element, so filter i sees channel c + i of the mixer input, or
 * zero past the end; every filter has its own alpha and lambda; beta is added
 * once.  With H heads the filters' coefficients are per head of the OUTPUT
 * channel (alpha, lam row i*H + h for filter i, head h; beta row h), while the
 * shift runs over the whole hidden vector.  Recurrent form: one cache per
 * filter, T_i <- lam_i T_i + x shifted by i, y = sum_i alpha_i T_i + beta, so
 * the cache is k*d values per layer: S[i*d + c].
 * tensors as for orc_create except alpha [k*H][n_ctx], beta [H][n_ctx], lam [k*H].
 */
orc_model *orc_create_kernel(int vocab, int d, int L, int H, int e, int n_ctx, double eps, int k,
                             const float *const *tensors)
{
    if (k < 1 || k > d) return NULL;
    return orc_create_any(vocab, d, L, H, e, n_ctx, eps, ORC_COLUMN, k, tensors);
}

/* The mixed-head model (the paper's default); alpha, beta [H][n_ctx], lam [H]. */
orc_model *orc_create(int vocab, int d, int L, int H, int e, int n_ctx, double eps,
                      const float *const *tensors)
{
    return orc_create_layout(vocab, d, L, H, e, n_ctx, eps, ORC_MIXED, tensors);
}

/* Cache values per layer per sample: d; 2d for ORC_COMBINED ("Method": combined layers need twice the
 * cache); k*d with k filters (orc_create_kernel). */
int orc_state_width(const orc_model *m)
{
    return m->kmix > 1 ? m->kmix * m->d : m->layout == ORC_COMBINED ? 2 * m->d : m->d;
}

/*
 * Non-projected SRM ("Method": the input projection "may or may not be applied,
 * heads are sliced ... and outputs concatenated and optionally projected back";
 * "SRM architecture optimization" and Tables S2-S4 call these parallel heads /
 * non-projected models).  With on = 0 the mixer of every layer reads the
 * LayerNorm output directly, head h being channels h*d_h .. (h+1)*d_h - 1, and
 * its output is added to the residual stream as it is; w_in, b_in, w_out, b_out
 * are unused.  orc_count_params(..., with_projections = 0) is this model's size
 * (pinned to Table S3).
 */
void orc_set_projections(orc_model *m, int on) { m->no_proj = !on; }

/*
 * Round to the nearest IEEE binary16 value (ties to even), result kept in `real`:
 * 11 significant bits, normal exponents -14..15, subnormals in steps of 2^-24,
 * overflow to infinity from 65520 on.
 */
real orc_round_half(real v)
{
    double a = fabs((double)v);
    if (!(a == a) || a == 0.0) return v;
    if (a >= 65520.0) return (real)(v < 0 ? -INFINITY : INFINITY);
    int e;
    (void)frexp(a, &e);                 /* a = f * 2^e, f in [0.5, 1): exponent of the leading bit is e - 1 */
    int lead = e - 1;
    if (lead < -14) lead = -14;         /* subnormal range: fixed step */
    double q = ldexp(1.0, lead - 10);   /* spacing of binary16 values in this binade */
    double r = rint(a / q) * q;         /* rint: ties to even in the default rounding mode */
    return (real)(v < 0 ? -r : r);
}

/*
 * Half-precision cache ("SRM architecture optimization": the recurrent form stays
 * stable with cache values and decay constants in half precision).  With on = 1
 * the stored sum S and lambda are binary16 values: each update computes
 * lam_h * S + p * u in the build's precision from the stored S, rounds the
 * result to binary16, stores it, and forms the layer output from the stored
 * value, so that the output is a function of the cache as it is kept.
 */
void orc_set_state_half(orc_model *m, int on) { m->half_state = on != 0; }

void orc_mixer_step_half(real *S, const real *u, const real *alpha_t, const real *beta_t,
                         const real *lam, int H, int d, real *m);

void orc_destroy(orc_model *m)
{
    if (!m) return;
    for (int l = 0; l < m->L; ++l) {
        orc_layer *y = &m->layers[l];
        free(y->ln1_g); free(y->ln1_b); free(y->w_in); free(y->b_in); free(y->alpha);
        free(y->beta); free(y->lam); free(y->w_out); free(y->b_out); free(y->ln2_g);
        free(y->ln2_b); free(y->w_up); free(y->b_up); free(y->w_down); free(y->b_down);
    }
    free(m->layers); free(m->embed); free(m->head); free(m->lnf_g); free(m->lnf_b);
    free(m);
}

/*
 * Number of trainable scalars of the block structure above, obtained by adding
 * up tensor shapes one by one (not from a closed formula).  with_projections=0
 * drops the in/out projections (the "non-projected" variant of Table S3).
 */
long long orc_count_params(int vocab, int d, int L, int H, int e, int n_ctx, int with_projections)
{
    long long n = 0, ff = (long long)e * d;
    n += (long long)vocab * d;           /* embedding              */
    n += (long long)vocab * d;           /* head (untied, no bias) */
    n += 2LL * d;                        /* final LayerNorm        */
    for (int l = 0; l < L; ++l) {
        n += 2LL * d;                    /* LN1 gain + bias        */
        if (with_projections) {
            n += (long long)d * d + d;   /* stacked I_h + bias     */
            n += (long long)d * d + d;   /* P_out + bias           */
        }
        n += (long long)H * n_ctx;       /* alpha: scalar per head per position */
        n += (long long)H * n_ctx;       /* beta                                */
        n += H;                          /* lambda per head                     */
        n += 2LL * d;                    /* LN2                    */
        n += ff * d + ff;                /* MLP up                 */
        n += (long long)d * ff + d;      /* MLP down               */
    }
    return n;
}

/* ---- per-token pieces ------------------------------------------------- */

/* LayerNorm over d: biased variance, affine. */
void orc_layernorm(const real *x, const real *g, const real *b, int d, double eps, real *out)
{
    real mean = 0;
    for (int i = 0; i < d; ++i) mean += x[i];
    mean /= (real)d;
    real var = 0;
    for (int i = 0; i < d; ++i) { real c = x[i] - mean; var += c * c; }
    var /= (real)d;
    real rstd = (real)(1.0 / sqrt((double)var + eps));
    for (int i = 0; i < d; ++i) out[i] = (x[i] - mean) * rstd * g[i] + b[i];
}

/* y = W a (+ bias), W row-major [n_out][n_in]. */
void orc_linear(const real *W, const real *bias, const real *a, int n_out, int n_in, real *y)
{
    for (int o = 0; o < n_out; ++o) {
        const real *w = W + (size_t)o * n_in;
        real acc = 0;
        for (int k = 0; k < n_in; ++k) acc += w[k] * a[k];
        y[o] = bias ? acc + bias[o] : acc;
    }
}

/* exact GELU: x * Phi(x). */
real orc_gelu(real x)
{
    return (real)(0.5 * (double)x * (1.0 + erf((double)x * 0.70710678118654752440)));
}

/* lowest index among maxima */
int orc_argmax(const real *v, int n)
{
    int best = 0;
    for (int i = 1; i < n; ++i) if (v[i] > v[best]) best = i;
    return best;
}

/*
 * One recurrent mixer update for one sample at one position (Eq. 2, Eq. 3).
 * S[d] is the cache; it holds the running sum INCLUDING the current token:
 *   row-repeat head:    S <- lam*S + alpha_t*u ;  m = S + beta_t
 *   column-repeat head: S <- lam*S + u         ;  m = alpha_t*S + beta_t
 * (the paper's cache C_n, the sum over m < n, equals lam*S_{n-1}; same size,
 * same outputs).  alpha_t, beta_t, lam: [H] values for this position.
 */
void orc_mixer_step(real *S, const real *u, const real *alpha_t, const real *beta_t,
                    const real *lam, int H, int d, real *m)
{
    int dh = d / H;
    for (int h = 0; h < H; ++h) {
        int row_repeat = h < H / 2;
        for (int c = h * dh; c < (h + 1) * dh; ++c) {
            if (row_repeat) {
                S[c] = lam[h] * S[c] + alpha_t[h] * u[c];
                m[c] = S[c] + beta_t[h];
            } else {
                S[c] = lam[h] * S[c] + u[c];
                m[c] = alpha_t[h] * S[c] + beta_t[h];
            }
        }
    }
}

/* orc_mixer_step with the cache and lambda held as binary16 values (see orc_set_state_half). */
void orc_mixer_step_half(real *S, const real *u, const real *alpha_t, const real *beta_t,
                         const real *lam, int H, int d, real *m)
{
    int dh = d / H;
    for (int h = 0; h < H; ++h) {
        int row_repeat = h < H / 2;
        real lh = orc_round_half(lam[h]);
        for (int c = h * dh; c < (h + 1) * dh; ++c) {
            if (row_repeat) {
                S[c] = orc_round_half(lh * S[c] + alpha_t[h] * u[c]);
                m[c] = S[c] + beta_t[h];
            } else {
                S[c] = orc_round_half(lh * S[c] + u[c]);
                m[c] = alpha_t[h] * S[c] + beta_t[h];
            }
        }
    }
}

/*
 * The mixer update for any head layout (see the enum): S[d], or S[2d] for
 * ORC_COMBINED.  alpha_t, beta_t, lam: one value per slot for this position.
 * half != 0 keeps the cache and lambda as binary16 values (orc_set_state_half).
 *   row-repeat (Eq. 2):     S <- lam*S + alpha_t*u ;  y = S + beta_t
 *   column-repeat (Eq. 3):  S <- lam*S + u         ;  y = alpha_t*S + beta_t
 *   combined: both, on separate caches, m = y_row + y_column.
 */
void orc_mixer_step_layout(real *S, const real *u, const real *alpha_t, const real *beta_t, const real *lam,
                           int H, int d, int layout, int half, real *m)
{
    int dh = d / H;
    for (int h = 0; h < H; ++h) {
        int row = layout == ORC_ROW || layout == ORC_COMBINED || (layout == ORC_MIXED && h < H / 2);
        int col = layout == ORC_COLUMN || layout == ORC_COMBINED || (layout == ORC_MIXED && h >= H / 2);
        int cs = layout == ORC_COMBINED ? H + h : h;              /* slot of the column-repeat matrix */
        real *Sc = layout == ORC_COMBINED ? S + d : S;            /* its cache */
        real lr = half ? orc_round_half(lam[h]) : lam[h];
        real lc = half ? orc_round_half(lam[cs]) : lam[cs];
        for (int c = h * dh; c < (h + 1) * dh; ++c) {
            real y = 0;
            if (row) {
                real v = lr * S[c] + alpha_t[h] * u[c];
                S[c] = half ? orc_round_half(v) : v;
                y += S[c] + beta_t[h];
            }
            if (col) {
                real v = lc * Sc[c] + u[c];
                Sc[c] = half ? orc_round_half(v) : v;
                y += alpha_t[cs] * Sc[c] + beta_t[cs];
            }
            m[c] = y;
        }
    }
}

/*
 * Parallel mixer for one sample: the T x T matrix of each head is written out
 * in full (Eq. 1 for row-repeat, Eq. 3 for column-repeat heads), each entry
 * with pow(), and applied as a dense product.  Tokens are rows here
 * (U[T][d]), i.e. the paper's Y = X M + B transposed: Y[j] = sum_i U[i] M[i][j].
 * alpha, beta: [H][n_ctx]; pos0 is the absolute position of row 0.
 */
void orc_mixer_parallel(const real *U, const real *alpha, const real *beta, const real *lam,
                        int H, int d, int T, int n_ctx, int pos0, real *Y)
{
    int dh = d / H;
    real *M = (real *)malloc((size_t)T * T * sizeof(real));
    for (int h = 0; h < H; ++h) {
        int row_repeat = h < H / 2;
        const real *a = alpha + (size_t)h * n_ctx + pos0;
        const real *b = beta + (size_t)h * n_ctx + pos0;
        for (int i = 0; i < T; ++i)
            for (int j = 0; j < T; ++j) {
                if (i > j) { M[(size_t)i * T + j] = 0; continue; }
                real decay = (real)pow((double)lam[h], (double)(j - i));
                M[(size_t)i * T + j] = decay * (row_repeat ? a[i] : a[j]);
            }
        for (int j = 0; j < T; ++j)
            for (int c = h * dh; c < (h + 1) * dh; ++c) {
                real acc = 0;
                for (int i = 0; i < T; ++i) acc += U[(size_t)i * d + c] * M[(size_t)i * T + j];
                Y[(size_t)j * d + c] = acc + b[j];
            }
    }
    free(M);
}

/*
 * orc_mixer_parallel for any head layout: the T x T matrix of a head is Eq. 1
 * (row-repeat), Eq. 3 (column-repeat) or, for ORC_COMBINED, the sum of the
 * head's two matrices, with the two bias rows added.
 */
void orc_mixer_parallel_layout(const real *U, const real *alpha, const real *beta, const real *lam,
                               int H, int d, int T, int n_ctx, int pos0, int layout, real *Y)
{
    int dh = d / H;
    real *M = (real *)malloc((size_t)T * T * sizeof(real));
    real *bias = (real *)malloc((size_t)T * sizeof(real));
    for (int h = 0; h < H; ++h) {
        int row = layout == ORC_ROW || layout == ORC_COMBINED || (layout == ORC_MIXED && h < H / 2);
        int col = layout == ORC_COLUMN || layout == ORC_COMBINED || (layout == ORC_MIXED && h >= H / 2);
        int cs = layout == ORC_COMBINED ? H + h : h;
        const real *ar = alpha + (size_t)h * n_ctx + pos0, *br = beta + (size_t)h * n_ctx + pos0;
        const real *ac = alpha + (size_t)cs * n_ctx + pos0, *bc = beta + (size_t)cs * n_ctx + pos0;
        for (int j = 0; j < T; ++j) bias[j] = (row ? br[j] : 0) + (col ? bc[j] : 0);
        for (int i = 0; i < T; ++i)
            for (int j = 0; j < T; ++j) {
                real v = 0;
                if (i <= j) {
                    if (row) v += (real)pow((double)lam[h], (double)(j - i)) * ar[i];
                    if (col) v += (real)pow((double)lam[cs], (double)(j - i)) * ac[j];
                }
                M[(size_t)i * T + j] = v;
            }
        for (int j = 0; j < T; ++j)
            for (int c = h * dh; c < (h + 1) * dh; ++c) {
                real acc = 0;
                for (int i = 0; i < T; ++i) acc += U[(size_t)i * d + c] * M[(size_t)i * T + j];
                Y[(size_t)j * d + c] = acc + bias[j];
            }
    }
    free(bias);
    free(M);
}

/*
 * One recurrent update of the k-filter mixer (orc_create_kernel) for one
 * sample: S[k*d], alpha_t and lam [k*H], beta_t [H], values of this position.
 */
void orc_mixer_step_kernel(real *S, const real *u, const real *alpha_t, const real *beta_t, const real *lam,
                           int H, int d, int k, int half, real *m)
{
    int dh = d / H;
    for (int c = 0; c < d; ++c) {
        int h = c / dh;
        real y = beta_t[h];
        for (int i = 0; i < k; ++i) {
            real x = c + i < d ? u[c + i] : 0;                  /* zero padding past the last channel */
            real l = half ? orc_round_half(lam[i * H + h]) : lam[i * H + h];
            real v = l * S[(size_t)i * d + c] + x;
            S[(size_t)i * d + c] = half ? orc_round_half(v) : v;
            y += alpha_t[i * H + h] * S[(size_t)i * d + c];
        }
        m[c] = y;
    }
}

/*
 * The same mixer over a whole sequence, Eq. 11 as printed: for every filter the
 * T x T column-repeat matrix (Eq. 3) is written out and applied to the input
 * shifted by i channels.  U, Y: [T][d] (tokens are rows); alpha [k*H][n_ctx],
 * beta [H][n_ctx]; pos0 = absolute position of row 0.
 */
void orc_mixer_parallel_kernel(const real *U, const real *alpha, const real *beta, const real *lam,
                               int H, int d, int k, int T, int n_ctx, int pos0, real *Y)
{
    int dh = d / H;
    real *M = (real *)malloc((size_t)T * T * sizeof(real));
    for (int j = 0; j < T; ++j)
        for (int c = 0; c < d; ++c) Y[(size_t)j * d + c] = beta[(size_t)(c / dh) * n_ctx + pos0 + j];
    for (int i = 0; i < k; ++i)
        for (int h = 0; h < H; ++h) {
            const real *a = alpha + (size_t)(i * H + h) * n_ctx + pos0;
            for (int r = 0; r < T; ++r)
                for (int j = 0; j < T; ++j)
                    M[(size_t)r * T + j] = r <= j ? (real)pow((double)lam[i * H + h], (double)(j - r)) * a[j] : 0;
            for (int j = 0; j < T; ++j)
                for (int c = h * dh; c < (h + 1) * dh; ++c) {
                    if (c + i >= d) continue;                   /* padded rows of X are zero */
                    real acc = 0;
                    for (int r = 0; r < T; ++r) acc += U[(size_t)r * d + c + i] * M[(size_t)r * T + j];
                    Y[(size_t)j * d + c] += acc;
                }
        }
    free(M);
}

/*
 * The closed forms on the right of Eq. 2 and Eq. 3, evaluated literally for
 * every position n (a third, independent statement used only as a pin):
 *   row:    Y_n = alpha_n X_n + beta_n + sum_{m<n} lam^{n-m} alpha_m X_m
 *   column: Y_n = alpha_n X_n + beta_n + alpha_n sum_{m<n} lam^{n-m} X_m
 */
void orc_mixer_closed_form(const real *U, const real *alpha, const real *beta, const real *lam,
                           int H, int d, int T, int n_ctx, real *Y)
{
    int dh = d / H;
    for (int h = 0; h < H; ++h) {
        int row_repeat = h < H / 2;
        const real *a = alpha + (size_t)h * n_ctx, *b = beta + (size_t)h * n_ctx;
        for (int n = 0; n < T; ++n)
            for (int c = h * dh; c < (h + 1) * dh; ++c) {
                real sum = 0;
                for (int m = 0; m < n; ++m) {
                    real p = (real)pow((double)lam[h], (double)(n - m));
                    sum += row_repeat ? p * a[m] * U[(size_t)m * d + c] : p * U[(size_t)m * d + c];
                }
                real y = a[n] * U[(size_t)n * d + c] + b[n];
                Y[(size_t)n * d + c] = row_repeat ? y + sum : y + a[n] * sum;
            }
    }
}

/* ---- sampling ------------------------------------------------------------ */

/*
 * Counter-based Gumbel noise, a pure function of (seed, position, sample index b,
 * vocabulary index v).  The paper only says that rollouts are sampled with a
 * temperature ("Training Details"); the generator is this build's definition and
 * is stated in full in the library's header so that both sides can implement it:
 *   hash(x): x ^= x>>16; x *= 0x7feb352d; x ^= x>>15; x *= 0x846ca68b; x ^= x>>16  (uint32)
 *   rowkey = hash(b ^ hash(pos + 0x9E3779B9 * (seed + 1)))
 *   h      = hash(rowkey + v * 0x9E3779B9)
 *   w      = ((h >> 9) + 0.5) * 2^-23        uniform in (0, 1)
 *   g      = -log(-log(1 - w))               standard Gumbel
 * Everything after the integer hash is evaluated in double here.
 */
#include <stdint.h>
static uint32_t orc_hash32(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}

double orc_uniform(uint32_t seed, uint32_t pos, uint32_t b, uint32_t v)
{
    uint32_t rowkey = orc_hash32(b ^ orc_hash32(pos + 0x9E3779B9U * (seed + 1U)));
    uint32_t h = orc_hash32(rowkey + v * 0x9E3779B9U);
    return ((double)(h >> 9) + 0.5) / 8388608.0;
}

double orc_gumbel(uint32_t seed, uint32_t pos, uint32_t b, uint32_t v)
{
    double w = orc_uniform(seed, pos, b, v);
    return -log(-log1p(-w));
}

/*
 * Next token from logits[V]: greedy for temperature == 0, otherwise the
 * Gumbel-max rule argmax_v(logit_v + temperature * g_v), which draws from
 * softmax(logits / temperature).  Lowest index on ties.  If margin is not NULL
 * it receives best minus second-best of the scores the decision was taken on.
 */
int orc_pick(const real *logits, int V, double temperature, uint32_t seed, int pos, int b, real *margin)
{
    int best = -1;
    real bs = -INFINITY, second = -INFINITY;
    for (int v = 0; v < V; ++v) {
        real sc = logits[v];
        if (temperature > 0) sc += (real)(temperature * orc_gumbel(seed, (uint32_t)pos, (uint32_t)b, (uint32_t)v));
        if (sc > bs) { second = bs; bs = sc; best = v; }
        else if (sc > second) second = sc;
    }
    if (margin) *margin = bs - second;
    return best < 0 ? 0 : best;
}

/*
 * Nucleus (top-p) truncation, the sampling rule of the paper's rollouts
 * ("Reasoning Experiments details": top-p 0.9 at temperature 0.7; the method is
 * the nucleus sampling the "Reinforcement Learning" paragraph cites).  With
 * p_v = softmax(logits / temperature): order the tokens by descending
 * probability (equal values by ascending index), take the shortest prefix whose
 * cumulative probability reaches top_p, and keep every token whose logit is at
 * least the last prefix element's (so equal values are kept or dropped
 * together).  keep[V] receives 0/1.  top_p >= 1 keeps everything.  Returns the
 * number kept.  mass_margin (may be NULL): distance of the deciding cumulative
 * sums from top_p, min(cum_k - top_p, top_p - cum_{k-1}), as a probability.
 */
typedef struct { double l; int v; } orc_lv;
static int orc_lv_desc(const void *a, const void *b)
{
    const orc_lv *x = (const orc_lv *)a, *y = (const orc_lv *)b;
    if (x->l > y->l) return -1;
    if (x->l < y->l) return 1;
    return x->v < y->v ? -1 : (x->v > y->v ? 1 : 0);
}

int orc_nucleus(const real *logits, int V, double temperature, double top_p, unsigned char *keep,
                double *mass_margin)
{
    if (mass_margin) *mass_margin = 1.0;
    if (!(top_p < 1.0) || !(temperature > 0)) {
        for (int v = 0; v < V; ++v) keep[v] = 1;
        return V;
    }
    orc_lv *o = (orc_lv *)malloc(sizeof(orc_lv) * (size_t)V);
    double mx = -INFINITY, Z = 0;
    for (int v = 0; v < V; ++v) { o[v].l = (double)logits[v]; o[v].v = v; if (o[v].l > mx) mx = o[v].l; }
    qsort(o, (size_t)V, sizeof(orc_lv), orc_lv_desc);
    for (int v = 0; v < V; ++v) Z += exp((o[v].l - mx) / temperature);
    double cum = 0, prev = 0;
    int k = 0;
    for (; k < V; ++k) {
        prev = cum;
        cum += exp((o[k].l - mx) / temperature) / Z;
        if (cum >= top_p) break;
    }
    if (k == V) k = V - 1;                       /* rounding left the total just below top_p */
    if (mass_margin) {
        double a = cum - top_p, b = top_p - prev;
        *mass_margin = a < b ? a : b;
    }
    const double cut = o[k].l;
    int n = 0;
    for (int v = 0; v < V; ++v) { keep[v] = (double)logits[v] >= cut; n += keep[v]; }
    free(o);
    return n;
}

/*
 * orc_pick restricted to the nucleus: argmax over the kept tokens of
 * logit_v + temperature * g_v, the Gumbel-max draw from the renormalised
 * truncated distribution, with the same counter as orc_pick (so for top_p >= 1
 * the two agree).  temperature == 0 is greedy whatever top_p.
 */
int orc_pick_topp(const real *logits, int V, double temperature, double top_p, uint32_t seed, int pos, int b,
                  real *margin, double *mass_margin)
{
    if (!(temperature > 0) || !(top_p < 1.0)) {
        if (mass_margin) *mass_margin = 1.0;
        return orc_pick(logits, V, temperature, seed, pos, b, margin);
    }
    unsigned char *keep = (unsigned char *)malloc((size_t)V);
    orc_nucleus(logits, V, temperature, top_p, keep, mass_margin);
    int best = -1;
    real bs = -INFINITY, second = -INFINITY;
    for (int v = 0; v < V; ++v) {
        if (!keep[v]) continue;
        real sc = logits[v] + (real)(temperature * orc_gumbel(seed, (uint32_t)pos, (uint32_t)b, (uint32_t)v));
        if (sc > bs) { second = bs; bs = sc; best = v; }
        else if (sc > second) second = sc;
    }
    free(keep);
    if (margin) *margin = bs - second;
    return best < 0 ? 0 : best;
}

/* ---- whole model, recurrent form --------------------------------------- */

/*
 * One token of one sample through the whole model in recurrent form.
 * S: [L][orc_state_width] cache, updated in place.  hidden (may be NULL): residual stream
 * after the last block [d].  logits (may be NULL): [V].
 */
void orc_step(const orc_model *m, int tok, int pos, real *S, real *hidden, real *logits)
{
    int d = m->d, ff = m->e * m->d, H = m->H;
    const int slots = m->kmix > 1 ? m->kmix * H : m->layout == ORC_COMBINED ? 2 * H : H, sd = orc_state_width(m);
    real *x = (real *)malloc(sizeof(real) * (size_t)(4 * d + 2 * ff + 2 * slots));
    real *a = x + d, *u = a + d, *mix = u + d, *g = mix + d, *t = g + ff;
    real *al = t + ff, *be = al + slots;
    for (int i = 0; i < d; ++i) x[i] = m->embed[(size_t)tok * d + i];
    for (int l = 0; l < m->L; ++l) {
        const orc_layer *y = &m->layers[l];
        orc_layernorm(x, y->ln1_g, y->ln1_b, d, m->eps, a);
        if (m->no_proj) memcpy(u, a, sizeof(real) * d);
        else orc_linear(y->w_in, y->b_in, a, d, d, u);
        for (int h = 0; h < slots; ++h) {
            al[h] = y->alpha[(size_t)h * m->n_ctx + pos];
            if (m->kmix <= 1 || h < H) be[h] = y->beta[(size_t)h * m->n_ctx + pos];
        }
        if (m->kmix > 1)
            orc_mixer_step_kernel(S + (size_t)l * sd, u, al, be, y->lam, H, d, m->kmix, m->half_state, mix);
        else if (m->layout != ORC_MIXED)
            orc_mixer_step_layout(S + (size_t)l * sd, u, al, be, y->lam, H, d, m->layout, m->half_state, mix);
        else if (m->half_state) orc_mixer_step_half(S + (size_t)l * d, u, al, be, y->lam, H, d, mix);
        else orc_mixer_step(S + (size_t)l * d, u, al, be, y->lam, H, d, mix);
        if (m->no_proj) memcpy(t, mix, sizeof(real) * d);
        else orc_linear(y->w_out, y->b_out, mix, d, d, t);
        for (int i = 0; i < d; ++i) x[i] += t[i];
        orc_layernorm(x, y->ln2_g, y->ln2_b, d, m->eps, a);
        orc_linear(y->w_up, y->b_up, a, ff, d, g);
        for (int i = 0; i < ff; ++i) g[i] = orc_gelu(g[i]);
        orc_linear(y->w_down, y->b_down, g, d, ff, t);
        for (int i = 0; i < d; ++i) x[i] += t[i];
    }
    if (hidden) memcpy(hidden, x, sizeof(real) * d);
    if (logits) {
        orc_layernorm(x, m->lnf_g, m->lnf_b, d, m->eps, a);
        orc_linear(m->head, NULL, a, m->vocab, d, logits);
    }
    free(x);
}

/*
 * Teacher-forced recurrent pass: tokens[B][T] at absolute positions
 * pos0..pos0+T-1, starting from state[B][L][orc_state_width] (updated in place; zero it for
 * pos0 = 0).  Optional outputs: hidden[B][T][d], logits[B][T][V],
 * greedy[B][T] (argmax of each position's logits).  Returns 0, or -1 on a
 * bad argument.
 */
int orc_recurrent_forward(const orc_model *m, int B, int T, const int *tokens, int pos0,
                          real *state, real *hidden, real *logits, int *greedy)
{
    if (pos0 < 0 || pos0 + T > m->n_ctx) return -1;
    for (long long i = 0; i < (long long)B * T; ++i)
        if (tokens[i] < 0 || tokens[i] >= m->vocab) return -1;
    int d = m->d, V = m->vocab;
    size_t Ld = (size_t)m->L * orc_state_width(m);
    int need_logits = logits || greedy;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        real *lg = need_logits && !logits ? (real *)malloc(sizeof(real) * V) : NULL;
        for (int t = 0; t < T; ++t) {
            size_t bt = (size_t)b * T + t;
            real *lrow = logits ? logits + bt * V : lg;
            orc_step(m, tokens[bt], pos0 + t, state + b * Ld,
                     hidden ? hidden + bt * d : NULL, lrow);
            if (greedy) greedy[bt] = orc_argmax(lrow, V);
        }
        free(lg);
    }
    return 0;
}

/*
 * Generation: consume prompts[B][P] from a zero state, then generate G tokens;
 * out_tokens[b][0] is chosen from the logits at the last prompt position and each
 * generated token is fed back.  temperature == 0: greedy; otherwise sampled with
 * orc_pick_topp (nucleus truncation when top_p < 1), the counter being (seed,
 * position of the token just consumed, b0 + b).
 * state[B][L][orc_state_width] is overwritten.  Optional: logits[B][G][V] (the raw logits each
 * generated token was chosen from) and margin[B][G] (top-1 minus top-2 of the
 * scores the choice was made on).
 */
int orc_generate_topp(const orc_model *m, int B, int P, int G, const int *prompts, real *state,
                      int *out_tokens, real *logits, real *margin, double temperature, uint32_t seed, int b0,
                      double top_p, double *mass_margin)
{
    if (P < 1 || G < 1 || P + G - 1 > m->n_ctx || temperature < 0 || !(top_p > 0)) return -1;
    for (long long i = 0; i < (long long)B * P; ++i)
        if (prompts[i] < 0 || prompts[i] >= m->vocab) return -1;
    int V = m->vocab;
    size_t Ld = (size_t)m->L * orc_state_width(m);
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        real *S = state + b * Ld;
        real *lg = (real *)malloc(sizeof(real) * V);
        for (size_t i = 0; i < Ld; ++i) S[i] = 0;
        int tok = 0;
        for (int t = 0; t < P + G - 1; ++t) {
            int in = t < P ? prompts[(size_t)b * P + t] : tok;
            int want = t >= P - 1;
            orc_step(m, in, t, S, NULL, want ? lg : NULL);
            if (!want) continue;
            int g = t - (P - 1);
            real mg;
            double mm;
            tok = orc_pick_topp(lg, V, temperature, top_p, seed, t, b0 + b, &mg, &mm);
            out_tokens[(size_t)b * G + g] = tok;
            if (logits) memcpy(logits + ((size_t)b * G + g) * V, lg, sizeof(real) * V);
            if (margin) margin[(size_t)b * G + g] = mg;
            if (mass_margin) mass_margin[(size_t)b * G + g] = mm;
        }
        free(lg);
    }
    return 0;
}

int orc_generate(const orc_model *m, int B, int P, int G, const int *prompts, real *state,
                 int *out_tokens, real *logits, real *margin, double temperature, uint32_t seed, int b0)
{
    return orc_generate_topp(m, B, P, G, prompts, state, out_tokens, logits, margin, temperature, seed, b0, 1.0,
                             NULL);
}

int orc_greedy(const orc_model *m, int B, int P, int G, const int *prompts, real *state,
               int *out_tokens, real *logits, real *margin)
{
    return orc_generate(m, B, P, G, prompts, state, out_tokens, logits, margin, 0.0, 0, 0);
}

/* ---- whole model, parallel (sequence) form ------------------------------ */

/*
 * The same model applied to whole sequences tokens[B][T] (positions 0..T-1),
 * layer by layer, with the token mixer as the explicit structured triangular
 * product (orc_mixer_parallel).  Outputs hidden[B][T][d] and, if not NULL,
 * logits[B][T][V].  No cache is read or written.
 */
int orc_parallel_forward(const orc_model *m, int B, int T, const int *tokens,
                         real *hidden, real *logits)
{
    if (T < 1 || T > m->n_ctx) return -1;
    for (long long i = 0; i < (long long)B * T; ++i)
        if (tokens[i] < 0 || tokens[i] >= m->vocab) return -1;
    int d = m->d, ff = m->e * m->d, V = m->vocab;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        size_t Td = (size_t)T * d;
        real *X = hidden + (size_t)b * Td;
        real *A = (real *)malloc(sizeof(real) * (3 * Td + (size_t)ff + d));
        real *U = A + Td, *Y = U + Td, *g = Y + Td, *tmp = g + ff;   /* g[ff], tmp[d] */
        for (int s = 0; s < T; ++s)
            for (int i = 0; i < d; ++i)
                X[(size_t)s * d + i] = m->embed[(size_t)tokens[(size_t)b * T + s] * d + i];
        for (int l = 0; l < m->L; ++l) {
            const orc_layer *y = &m->layers[l];
            for (int s = 0; s < T; ++s) {
                orc_layernorm(X + (size_t)s * d, y->ln1_g, y->ln1_b, d, m->eps, A + (size_t)s * d);
                if (m->no_proj) memcpy(U + (size_t)s * d, A + (size_t)s * d, sizeof(real) * d);
                else orc_linear(y->w_in, y->b_in, A + (size_t)s * d, d, d, U + (size_t)s * d);
            }
            if (m->kmix > 1)
                orc_mixer_parallel_kernel(U, y->alpha, y->beta, y->lam, m->H, d, m->kmix, T, m->n_ctx, 0, Y);
            else if (m->layout != ORC_MIXED)
                orc_mixer_parallel_layout(U, y->alpha, y->beta, y->lam, m->H, d, T, m->n_ctx, 0, m->layout, Y);
            else orc_mixer_parallel(U, y->alpha, y->beta, y->lam, m->H, d, T, m->n_ctx, 0, Y);
            for (int s = 0; s < T; ++s) {
                real *x = X + (size_t)s * d;
                if (m->no_proj) memcpy(tmp, Y + (size_t)s * d, sizeof(real) * d);
                else orc_linear(y->w_out, y->b_out, Y + (size_t)s * d, d, d, tmp);
                for (int i = 0; i < d; ++i) x[i] += tmp[i];
                orc_layernorm(x, y->ln2_g, y->ln2_b, d, m->eps, A + (size_t)s * d);
                orc_linear(y->w_up, y->b_up, A + (size_t)s * d, ff, d, g);
                for (int i = 0; i < ff; ++i) g[i] = orc_gelu(g[i]);
                orc_linear(y->w_down, y->b_down, g, d, ff, tmp);
                for (int i = 0; i < d; ++i) x[i] += tmp[i];
            }
        }
        if (logits)
            for (int s = 0; s < T; ++s) {
                orc_layernorm(X + (size_t)s * d, m->lnf_g, m->lnf_b, d, m->eps, A);
                orc_linear(m->head, NULL, A, V, d, logits + ((size_t)b * T + s) * V);
            }
        free(A);
    }
    return 0;
}
