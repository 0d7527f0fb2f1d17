/*
 * srm.h -- C ABI of libsrm: batched autoregressive generation with the
 * Structured Recurrent Mixer (SRM) in its recurrent form, plus the parallel
 * (sequence) form of the same model, on one AMD MI355X (gfx950).
 *
 * Model (paper section "Method"): token embedding, then n_layers blocks of
 *   [ LayerNorm -> per-head input projections I_h (stacked, d x d) ->
 *     structured token mixer -> output projection P_out -> residual ]      (Eq. 10)
 *   [ LayerNorm -> channel-mixing MLP (expansion e, exact GELU) -> residual ]
 * then a final LayerNorm and an untied LM head; greedy next token = argmax,
 * lowest index on ties.  The token mixer is the paper's causal mixing matrix
 * restricted to row-repeat (Eq. 1) or column-repeat (Eq. 3) form with one
 * decay factor lambda per diagonal; heads 0..H/2-1 are row-repeat, heads
 * H/2..H-1 column-repeat ("mixed" heads).  Its recurrent form (Eq. 2, Eq. 3)
 * keeps one fp32 value per channel per layer per sample (the cache):
 *   row head:    S <- lambda_h S + alpha_{h,t} u ;  m = S + beta_{h,t}
 *   column head: S <- lambda_h S + u             ;  m = alpha_{h,t} S + beta_{h,t}
 * with u the projected input at absolute position t.  alpha and beta are
 * scalars per (layer, head, position); positions are bounded by n_ctx.
 *
 * Conventions
 *   - "d_" arguments are DEVICE pointers on the model's GPU; all other pointers
 *     are HOST pointers.  The library owns only srm_model (device copies of the
 *     weights).  State, workspace, token and output buffers belong to the caller.
 *   - Matrices are row-major [out][in].  Tokens are int32.  The state is fp32,
 *     laid out [n_layers][batch][d_model]; the caller zeroes it before position 0.
 *   - Compute calls are asynchronous on the given hipStream_t (passed as void*,
 *     NULL = the default stream); they never synchronise and never copy to host.
 *   - Every call returns SRM_OK (0) or a negative srm_status; after a failure
 *     srm_last_error() returns a message for the calling thread.  Arguments are
 *     validated on the host before any kernel is launched.  Token ids outside
 *     [0, vocab) are not checked on the device: the caller must not pass them.
 *   - weight_dtype SRM_BF16: matrices (embed, head, w_in, w_out, w_up, w_down)
 *     are stored in bf16 (host values are rounded to nearest-even), activations
 *     entering a GEMM are bf16, accumulation, residual stream, LayerNorm,
 *     mixer state and logits are fp32.  Requires d_model % 64 == 0.
 *     weight_dtype SRM_FP32: everything fp32.  Both need d_model % (4*n_heads) == 0
 *     and d_model <= 4096.
 *   - Environment switches (read at each call; they select between arrangements
 *     of the same arithmetic and exist for tests and measurements):
 *     SRM_FUSE_MIXER=0   the recurrent state update as a kernel of its own instead
 *                        of inside the in-projection's epilogue (same bits);
 *     SRM_LN_ON_LOAD=0   bf16 models, at most 8 samples: LayerNorm launches
 *                        between the GEMMs instead of LayerNorm made by the
 *                        consuming GEMM (same bits);
 *     SRM_MEGAKERNEL, SRM_MEGA_BLOCKS   see srm_generate_one_kernel_blocks.
 */
#ifndef SRM_H
#define SRM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct srm_model srm_model;

typedef enum {
    SRM_OK = 0,
    SRM_EINVAL = -1,   /* bad argument (message says which)            */
    SRM_ENOMEM = -2,   /* device or host allocation failed, or the workspace is too small */
    SRM_EHIP = -3      /* a HIP runtime call failed (message has the HIP error) */
} srm_status;

enum { SRM_FP32 = 0, SRM_BF16 = 1, SRM_FP16 = 2 };
/* Head layouts ("Method", the paragraph after Eq. 2 on combining row- and column-repeat outputs; Table S0). */
enum { SRM_HEADS_MIXED = 0, SRM_HEADS_ROW = 1, SRM_HEADS_COLUMN = 2, SRM_HEADS_COMBINED = 3 };

typedef struct {
    int32_t vocab;
    int32_t d_model;
    int32_t n_layers;
    int32_t n_heads;        /* H; see head_layout (mixed heads: even, first half row-repeat, second half
                               column-repeat) */
    int32_t mlp_expansion;
    int32_t n_ctx;          /* number of positions alpha/beta are defined for */
    int32_t weight_dtype;   /* SRM_FP32 | SRM_BF16 */
    float ln_eps;
    int32_t state_dtype;    /* SRM_FP32 (default, 0): fp32 recurrent state; SRM_FP16: the cache and the decay
                               constants as IEEE binary16 values ("SRM architecture optimization": the
                               recurrent form stays stable with both in half precision).  Each update
                               computes lam*S + p*u in fp32 from the stored S, rounds it to binary16
                               (nearest, ties to even), stores it and forms the output from the stored
                               value; d_state arrays then hold binary16 elements. */
    int32_t no_projections; /* 0: in/out head projections (the default model); 1: non-projected mixer
                               layers ("Method", last paragraph; Tables S2-S4): head h is channels
                               h*d_h .. of the LayerNorm output, the mixer output joins the residual
                               stream directly; w_in, b_in, w_out, b_out are ignored and may be NULL */
    int32_t head_layout;    /* SRM_HEADS_MIXED (default, 0): "mixed" heads, the model the paper settles on.
                               SRM_HEADS_ROW / SRM_HEADS_COLUMN: every head row-repeat (Eq. 2) / column-
                               repeat (Eq. 3); n_heads may be odd, 1 is the non-headed model.
                               SRM_HEADS_COMBINED: every head owns one row-repeat and one column-repeat
                               matrix, each with its own alpha, beta, lambda, applied to the same head
                               input; the two outputs are added (any fixed linear combination is this one
                               with the weights folded into alpha and beta).  alpha, beta then have 2H
                               rows and lambda 2H entries: row h = head h's row-repeat matrix, row H + h
                               its column-repeat matrix.  The cache doubles ("Method": combined layers
                               need twice the cache): every state row is [2d], first the d values of the
                               row-repeat matrices, then the d values of the column-repeat ones, and
                               srm_state_bytes counts 2d.  Needs the head projections. */
    int32_t mixer_kernel;   /* 0 or 1: none.  k > 1: every mixer layer has k filters along the hidden
                               dimension (Eq. 11): Y = sum_i X_(i:d+i, :) W_i + beta with X zero-padded and
                               each W_i a column-repeat matrix.  Reading: filters i = 0..k-1; the padding
                               follows the last hidden element, so filter i sees channel c + i of the head
                               input (zero past the end); own alpha and lambda per filter and head of the
                               output channel, one beta.  alpha is [k*H][n_ctx] and lambda [k*H] (row
                               i*H + h: filter i, head h), beta [H][n_ctx].  One cache per filter: every
                               state row is [k*d], filter-major, and srm_state_bytes counts k*d.  Needs
                               head_layout = SRM_HEADS_COLUMN and the head projections; k*H <= 64. */
} srm_config;

/* HOST pointers, fp32, caller-owned, not retained after srm_init_weights. */
typedef struct {
    const float *ln1_g, *ln1_b;        /* [d], [d]                                  */
    const float *w_in, *b_in;          /* [d][d] (rows h*d_h.. are I_h), [d]         */
    const float *alpha, *beta;         /* [H][n_ctx], [H][n_ctx] ([2H] rows: combined; alpha [k*H] rows: mixer_kernel k) */
    const float *lambda;               /* [H] ([2H]: combined; [k*H]: mixer_kernel k), each in (0, 1] */
    const float *w_out, *b_out;        /* [d][d] (P_out), [d]                        */
    const float *ln2_g, *ln2_b;        /* [d], [d]                                   */
    const float *w_up, *b_up;          /* [e*d][d], [e*d]                            */
    const float *w_down, *b_down;      /* [d][e*d], [d]                              */
} srm_host_layer;

typedef struct {
    const float *embed;                /* [vocab][d]                                 */
    const float *head;                 /* [vocab][d], no bias                        */
    const float *lnf_g, *lnf_b;        /* [d], [d]                                   */
    const srm_host_layer *layers;      /* [n_layers]                                 */
} srm_host_weights;

/*
 * Copy the weights to the current HIP device (casting matrices to bf16 when
 * configured) and return an opaque model.  ("Method": one parameter set serves
 * both the recurrent and the parallel form.)
 * Errors: SRM_EINVAL for a null pointer, non-positive size, odd n_heads with
 * mixed heads, more than 64 coefficient rows per layer, an unknown head_layout,
 * combined heads or mixer_kernel > 1 without projections, mixer_kernel > 1 with
 * another head layout than column, d_model not divisible by 4*n_heads, d_model > 4096, bf16 with d_model % 64,
 * or a lambda outside (0, 1]; SRM_ENOMEM; SRM_EHIP.
 */
int srm_init_weights(const srm_config *cfg, const srm_host_weights *w, srm_model **out);
void srm_free(srm_model *m);

/*
 * Bytes of recurrent state for `batch` samples: n_layers * batch * d_model * 4
 * (2 with a binary16 state; times 2 with combined heads, times k with mixer_kernel = k), whatever the position ("Computational Complexity": O(d) space per sample).
 * Returns 0 for a null model or batch <= 0.
 */
size_t srm_state_bytes(const srm_model *m, int64_t batch);

/*
 * Bytes of scratch a call needs for `rows` token rows processed at once
 * (decode calls: rows = B takes the step in one pass; srm_prefill /
 * srm_parallel_forward: any multiple of the sequence length, at least one
 * sequence; more rows = fewer passes).  The decode calls (srm_decode_step*,
 * srm_generate*) accept a smaller workspace and then take the step in slices of
 * as many samples as it holds, at least min(B, 256) - the samples are
 * independent - so the number of resident sequences is bounded by the state,
 * not by the workspace.  Results do not depend on the slicing in fp32 models;
 * in bf16 models a different slice size may select another GEMM tile shape.
 */
size_t srm_workspace_bytes(const srm_model *m, int64_t rows);
/* The same number from a configuration alone (host only, no GPU call), for sizing buffers before a model
 * exists; 0 for a null or invalid configuration or rows <= 0. */
size_t srm_workspace_bytes_config(const srm_config *cfg, int64_t rows);

/*
 * One decode step for B samples that all sit at absolute position `pos`
 * ("Recurrent Throughput and Concurrency": one token per sample per step,
 * parallel over the batch).  Reads d_tok_in[B], updates d_state[L][B][d] in
 * place (Eq. 2 / Eq. 3), writes the greedy next token d_tok_out[B].
 * Optional outputs (NULL to skip): d_logits[B][vocab] fp32, d_hidden[B][d]
 * fp32 (residual stream after the last block, before the final LayerNorm).
 * d_tok_out may alias d_tok_in.  Errors: SRM_EINVAL (null pointer, B <= 0,
 * pos outside [0, n_ctx)), SRM_ENOMEM (workspace smaller than
 * srm_workspace_bytes(m, min(B, 256))).
 */
int srm_decode_step(srm_model *m, int64_t B, int32_t pos, const int32_t *d_tok_in,
                    void *d_state, int32_t *d_tok_out, float *d_logits, float *d_hidden,
                    void *d_workspace, size_t workspace_bytes, void *hip_stream);

/*
 * srm_decode_step with the next token SAMPLED from softmax(logits / temperature)
 * instead of taken greedily (the paper's rollouts use temperature 0.7, "Training
 * Details"; top-p truncation is not applied).  The sample is exact and needs no
 * normalisation pass: tok = argmax_v(logit_v + temperature * g_v) with g_v
 * independent standard Gumbel variates (the Gumbel-max rule), fused into the LM
 * head like the greedy argmax.  g is a pure function of (seed, pos, sample index
 * b, vocabulary index v), so a call can be reproduced exactly anywhere:
 *   hash(x): x ^= x>>16; x *= 0x7feb352d; x ^= x>>15; x *= 0x846ca68b; x ^= x>>16   (uint32)
 *   rowkey = hash(b ^ hash(pos + 0x9E3779B9 * (seed + 1)))
 *   h      = hash(rowkey + v * 0x9E3779B9)
 *   w      = ((h >> 9) + 0.5) * 2^-23 ;   g_v = -log(-log(1 - w))
 * temperature = 0 gives srm_decode_step.  d_logits, if requested, are the raw
 * logits.  Ties as in the greedy case.  Errors as srm_decode_step, plus
 * SRM_EINVAL for a negative or NaN temperature.
 */
int srm_decode_step_sampled(srm_model *m, int64_t B, int32_t pos, const int32_t *d_tok_in,
                            void *d_state, int32_t *d_tok_out, float temperature, uint32_t seed,
                            float *d_logits, float *d_hidden, void *d_workspace,
                            size_t workspace_bytes, void *hip_stream);

/*
 * G decode steps in one call, for callers that only want the tokens
 * ("MAX model details": looping forward passes and cache updates inside the
 * compiled code instead of calling it once per token removed a per-call delay
 * that dominated the paper's measurements).  Step g (0-based) consumes d_tok[B]
 * at absolute position pos0 + g, updates d_state in place, overwrites d_tok with
 * the greedy tokens and also stores them at d_tokens_out[g][B].  The position
 * lives in device memory (the last 256 bytes of the workspace), so one step is
 * captured into a HIP graph on the first call and replayed G - 1 times; the
 * graph is cached in the model and reused while B and the four device pointers
 * stay the same.  On the legacy default stream (NULL), which cannot be
 * captured, the steps are launched one by one instead.  temperature = 0 is
 * greedy; temperature > 0 samples as srm_decode_step_sampled does.  Results are
 * identical to G srm_decode_step(_sampled) calls, except that a call which
 * qualifies for the one-kernel path (see srm_generate_one_kernel_blocks) runs
 * all G steps in one cooperative launch, with fp32 sums in another order: equal
 * to the step calls up to fp32 rounding, token-exact unless two scores tie
 * within that rounding.  Such a call must not be made under stream capture.
 * The one-kernel path synchronises its work-groups with bounded waits; should a
 * wait ever give up (a work-group that is not resident: never observed), the
 * kernel ends early, d_tok and the rows of d_tokens_out from that step on hold
 * -1, the state is undefined and the call has already returned SRM_OK (it is
 * asynchronous): a caller that cannot rule this out checks d_tokens_out for -1
 * after synchronising.  Not thread-safe per model.
 * Errors: SRM_EINVAL (null pointer, B or G <= 0, pos0 + G > n_ctx), SRM_ENOMEM
 * (workspace smaller than srm_workspace_bytes(m, B)), SRM_EHIP.
 */
int srm_generate(srm_model *m, int64_t B, int32_t pos0, int32_t G, int32_t *d_tok, void *d_state,
                 int32_t *d_tokens_out, float temperature, uint32_t seed, void *d_workspace,
                 size_t workspace_bytes, void *hip_stream);

/*
 * Consume N prompts of P tokens (positions 0..P-1) from a zero state, layer by
 * layer over all positions, with the mixer evaluated as the sequential
 * recurrence (the result equals P decode steps), then replicate each prompt's
 * state and first generated token to fanout_k consecutive samples:
 * sample n*fanout_k + r takes prompt n.  Writes d_state[L][N*k][d] (every
 * element), d_next_tok[N*k], and, if not NULL, d_logits[N][vocab] (last
 * position).  Processes as many whole prompts per pass as the workspace holds.
 * Errors: SRM_EINVAL (null pointer, N, P or fanout_k <= 0, P > n_ctx),
 * SRM_ENOMEM (workspace smaller than srm_workspace_bytes(m, P)).
 */
int srm_prefill(srm_model *m, const int32_t *d_prompts, int32_t N, int32_t P, int32_t fanout_k,
                void *d_state, int32_t *d_next_tok, float *d_logits,
                void *d_workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Decode step with nucleus (top-p) sampling, the rule of the paper's rollouts
 * ("Reasoning Experiments details": top-p 0.9, temperature 0.7).  With
 * p = softmax(logits / temperature), the nucleus is the smallest set of most
 * probable tokens whose probability reaches top_p (tokens with equal logits are
 * kept or dropped together); the token is drawn from the renormalised nucleus
 * by the Gumbel-max rule with the noise of srm_decode_step_sampled, restricted
 * to the nucleus: whenever the unrestricted draw lies inside the nucleus the two
 * calls return the same token.  The truncation needs the whole row, so
 * d_logits[B][vocab] is required when top_p < 1 and temperature > 0 (it is left
 * holding the raw logits); top_p >= 1 or temperature = 0 behave as
 * srm_decode_step_sampled.  Sums of probabilities are formed in fp32 by a fixed
 * reduction tree, so results are reproducible from run to run.
 * Errors: as srm_decode_step_sampled, plus SRM_EINVAL for top_p <= 0 or a
 * missing logits buffer.
 */
int srm_decode_step_topp(srm_model *m, int64_t B, int32_t pos, const int32_t *d_tok_in, void *d_state,
                         int32_t *d_tok_out, float temperature, float top_p, uint32_t seed,
                         float *d_logits, float *d_hidden,
                         void *d_workspace, size_t workspace_bytes, void *hip_stream);

/* srm_generate with nucleus sampling; d_logits[B][vocab] is scratch for the truncation
 * (required when top_p < 1 and temperature > 0).  Otherwise as srm_generate. */
int srm_generate_topp(srm_model *m, int64_t B, int32_t pos0, int32_t G, int32_t *d_tok, void *d_state,
                      int32_t *d_tokens_out, float temperature, float top_p, uint32_t seed,
                      float *d_logits, void *d_workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The sampler alone, on logits that are already in device memory:
 * d_logits[rows][vocab] fp32 -> d_tok_out[rows], drawn from
 * softmax(logits / temperature) truncated to the top_p nucleus (top_p >= 1: no
 * truncation), with the counter (seed, pos, row).  Same kernel as in
 * srm_decode_step_topp.  Needs no model.
 * Errors: SRM_EINVAL (null pointer, sizes <= 0, temperature <= 0, top_p <= 0).
 */
int srm_sample_logits(const float *d_logits, int64_t rows, int32_t vocab, float temperature, float top_p,
                      uint32_t seed, int32_t pos, int32_t *d_tok_out, void *hip_stream);

/*
 * Decode step with one position per sample, for batches whose samples are at
 * different positions (prompts of different lengths, slots that join and leave
 * a running batch).  The recurrent form makes this free: a sample's cache has
 * the same size at every position (Eq. 2, Eq. 3), so samples at different
 * positions share one batch without padding; only alpha and beta are looked up
 * per sample.  d_pos[B] (device, int32) holds each sample's absolute position.
 * A sample whose position is outside [0, n_ctx) is inactive: its state is left
 * untouched and d_tok_out gets -1 for it (its d_tok_in is still read and may be
 * any value).  With advance != 0 the position of every active sample is
 * incremented on the device at the end of the step, so a loop of calls needs no
 * host-side update.  temperature = 0 is greedy; temperature > 0 samples as
 * srm_decode_step_topp does (top_p >= 1: no truncation), keyed on the sample's
 * own position.  For active samples the result equals the uniform-position call
 * at that position.  d_logits: [B][vocab], optional unless top_p < 1.
 * Errors: SRM_EINVAL (null pointer, B out of range, negative temperature,
 * top_p <= 0, top_p < 1 without d_logits), SRM_ENOMEM (workspace smaller than
 * srm_workspace_bytes(m, B)), SRM_EHIP.
 */
int srm_decode_step_ragged(srm_model *m, int64_t B, int32_t *d_pos, int32_t advance,
                           const int32_t *d_tok_in, void *d_state, int32_t *d_tok_out,
                           float temperature, float top_p, uint32_t seed, float *d_logits,
                           void *d_workspace, size_t workspace_bytes, void *hip_stream);

/*
 * G ragged decode steps in one call: a serving loop that runs on the device.
 * Step g feeds d_tok[B] back at each sample's own position d_pos[b], advances
 * the positions of the active samples and stores the tokens at
 * d_tokens_out[g][B] (-1 for idle samples).  A sample that emits eos_id
 * (eos_id < 0: no such token) or runs out of positions goes idle - position -1
 * respectively >= n_ctx - and stays idle, its state untouched, until the caller
 * admits a new prompt into the slot (srm_prefill_ragged with d_slot).  As in
 * srm_generate, one step is captured into a HIP graph and replayed; the
 * positions are device data, so the graph needs no update between steps or
 * calls.  Sampling as in srm_decode_step_ragged.
 * Errors: as srm_generate and srm_decode_step_ragged; SRM_EINVAL for eos_id >= vocab.
 */
int srm_generate_ragged(srm_model *m, int64_t B, int32_t G, int32_t *d_pos, int32_t *d_tok, void *d_state,
                        int32_t *d_tokens_out, int32_t eos_id, float temperature, float top_p, uint32_t seed,
                        float *d_logits, void *d_workspace, size_t workspace_bytes, void *hip_stream);

/*
 * srm_prefill for N prompts of different lengths, packed back to back in
 * d_tokens: prompt n is d_tokens[offsets[n] .. offsets[n+1]-1], positions
 * 0 .. length-1, from a zero state.  The offsets (N + 1 values, int32) are
 * passed twice: h_offsets in host memory, which the call validates (every
 * length in [1, n_ctx]) and uses to cut the work into passes of whole prompts
 * that fit the workspace, and d_offsets, the same values in device memory, which
 * the kernels read (clamped, so a mismatch cannot cause an access outside the
 * workspace; results are then unspecified).
 * Destination of prompt n in d_state[L][state_batch][d] (only the destination
 * samples are written), d_next_tok[state_batch] and, if not NULL,
 * d_pos[state_batch] (set to the prompt's length, the position of the next
 * token): with d_slot == NULL the fanout_k consecutive samples
 * n*fanout_k + r; with d_slot (device, int32 [N], fanout_k must be 1) sample
 * d_slot[n], skipped if outside [0, state_batch) - this admits new prompts
 * into free slots of a running batch.  d_logits: optional [N][vocab], last
 * position of each prompt.  The first token is greedy.
 * Errors: SRM_EINVAL (null pointer, N or fanout_k <= 0, a length outside
 * [1, n_ctx], N*fanout_k > state_batch, slots with fanout_k != 1), SRM_ENOMEM
 * (workspace smaller than srm_workspace_bytes(m, longest prompt)), SRM_EHIP.
 */
int srm_prefill_ragged(srm_model *m, const int32_t *d_tokens, const int32_t *h_offsets,
                       const int32_t *d_offsets, int32_t N, int32_t fanout_k, const int32_t *d_slot,
                       int64_t state_batch, void *d_state, int32_t *d_next_tok, int32_t *d_pos,
                       float *d_logits, void *d_workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Host-only planning query (no GPU call, no model): how srm_prefill_ragged would
 * take the packed prompts h_offsets[N + 1] of a model with configuration cfg
 * through a workspace of workspace_bytes.  The mixer of a prefill pass is either
 * one sequential scan per prompt or a chunked scan ("MAX model details" names a
 * parallel scan for recurrent prefill as unexplored; the recurrence of Eq. 2 /
 * Eq. 3 is linear, so the state entering chunk j is lambda^c times the state
 * entering chunk j-1 plus what chunk j-1 reaches from zero).  The chunked scan
 * keeps one fp32 partial state per (prompt, chunk, channel) in the MLP buffer of
 * the pass; it is taken when the call's shape (N, longest prompt) asks for it AND
 * those partial states fit that buffer in every pass - many short prompts next
 * to one long prompt do not fit, and the whole call then takes the sequential
 * scan.  Reports the passes, the chunk length taken (0: sequential) and the one
 * the shape alone would choose, and for the tightest pass under that choice the
 * bytes of partial states and the bytes of the buffer they would live in.
 * Errors: as srm_prefill_ragged for cfg, the lengths and the workspace size.
 */
typedef struct {
    int32_t passes;              /* passes of whole prompts                                */
    int32_t chunk_len;           /* chunk length of the scan taken, 0 = sequential scan     */
    int32_t chunk_len_by_shape;  /* what (N, longest prompt) alone would choose             */
    int32_t n_chunks;            /* chunks per prompt under chunk_len_by_shape              */
    size_t scratch_need;         /* tightest pass under chunk_len_by_shape: partial states  */
    size_t scratch_room;         /* ... and the room of that pass's MLP buffer, in bytes    */
} srm_prefill_plan;
int srm_prefill_ragged_plan(const srm_config *cfg, const int32_t *h_offsets, int32_t N,
                            size_t workspace_bytes, srm_prefill_plan *out);

/*
 * Parallel (sequence) form over d_tok[B][T], positions 0..T-1: identical model,
 * but the mixer is the explicit structured triangular product Y = U M + beta
 * with M built from alpha and lambda as in Eq. 1 (row-repeat heads) and Eq. 3
 * (column-repeat heads).  Reads and writes no state.  Writes d_hidden[B][T][d]
 * fp32 and, if not NULL, d_logits[B][T][vocab] fp32.
 * Errors: SRM_EINVAL (null pointer, B or T <= 0, T > n_ctx), SRM_ENOMEM
 * (workspace smaller than srm_workspace_bytes(m, T)).
 */
int srm_parallel_forward(srm_model *m, const int32_t *d_tok, int32_t B, int32_t T,
                         float *d_hidden, float *d_logits,
                         void *d_workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Kernel-level entry points (the pieces of srm_decode_step, callable alone so
 * each can be checked and timed by itself).
 *
 * srm_mixer_update: the recurrent state update of one layer (Eq. 2 / Eq. 3)
 * for B samples at position pos.  d_u and d_m are [B][d] in the model's
 * activation type (bf16 for SRM_BF16 models, fp32 otherwise); d_state_layer is
 * that layer's [B][d] slab (fp32, or binary16 with a half-precision state),
 * updated in place.  d_m may alias d_u.  With combined heads all three rows are
 * [2d]: the row-repeat half then the column-repeat half, d_u holding the head
 * input twice; the model adds the two halves of d_m in its out-projection
 * (mixer_kernel = k: rows [k*d], copy i holding the head input shifted by i).
 */
int srm_mixer_update(srm_model *m, int32_t layer, int32_t pos, int64_t B, const void *d_u,
                     void *d_state_layer, void *d_m, void *hip_stream);

/*
 * srm_mixer_project_update: the stacked head in-projection of one layer (Eq. 10:
 * u = a W_in^T + b_in) and the recurrent state update (Eq. 2 / Eq. 3) of its
 * result in ONE launch, the form a decode step uses: u stays in registers, the
 * state slab is read and written once, d_m [B][state width] receives the mixer
 * output.  d_a is the layer's LayerNorm1 output [B][d_model] in the activation
 * type; d_state_layer and d_m as for srm_mixer_update.  Same values as
 * srm_linear(epilogue 0) with the layer's W_in followed by srm_mixer_update
 * (u is rounded to the activation type before the update, as the two-launch
 * form stores it).  Models without head projections: SRM_EINVAL.
 */
int srm_mixer_project_update(srm_model *m, int32_t layer, int32_t pos, int64_t B, const void *d_a,
                             void *d_state_layer, void *d_m, void *hip_stream);

/*
 * The token-mixing half of block `layer` in the form a decode step takes for a few dozen
 * to a couple of thousand rows of a bf16 model (the block of Fig. 1: the mixer of
 * Eq. 2 / Eq. 3 with the head projections of Eq. 10, between its LayerNorms):
 *   a = LayerNorm1(x); u = a W_in^T + b_in; (S, m) = state update of Eq. 2 / 3 at `pos`;
 *   x += m W_out^T + b_out; norm_out = LayerNorm2(x)
 * as two kernels: one from LayerNorm1 to the out-projection, which it leaves as d / 128
 * K slices in d_slabs, and the LayerNorm kernel that adds them to x.
 * d_x [B][d] fp32 (device, read and written), d_state_layer [B][d] in the model's
 * state type (device, updated in place), d_norm_out [B][d] bf16 (device, written),
 * d_slabs (device, scratch, (d / 128) * B * d floats).
 * d_pos_rows (device, [B], may be NULL) gives one position per row instead of `pos`;
 * a row whose position is outside [0, n_ctx) keeps its state and mixes zeros.
 * The caller owns all buffers.  Needs bf16 weights, use_projections with projection
 * width d, and d = 256 or 512: SRM_EINVAL otherwise, and for a null pointer, a layer
 * or (without d_pos_rows) a position out of range, B <= 0.  SRM_EHIP.
 */
int srm_mixer_block(srm_model *m, int32_t layer, int32_t pos, const int32_t *d_pos_rows, int64_t B,
                    float *d_x, void *d_state_layer, void *d_norm_out, float *d_slabs, void *hip_stream);

/*
 * srm_linear: out = epilogue(A W^T + bias) with A [M][K] and W [N][K] device
 * arrays of type `dtype` (SRM_BF16: bf16 operands on the matrix cores with fp32
 * accumulation, K % 64 == 0; SRM_FP32: fp32).  d_bias [N] fp32 or NULL.
 * epilogue: 0 = store (type `dtype`), 1 = exact GELU then store (type `dtype`),
 * 2 = add into fp32 d_out (residual), 3 = store fp32 and also write the
 * row-wise argmax (lowest index on ties) to d_argmax[M] (needs d_scratch of
 * srm_linear_scratch_bytes(M, N) bytes); d_out may be NULL for epilogue 3;
 * 4 = store fp32 (the form the parallel pass uses for its logits).
 * Test and measurement hook: with SRM_BF16, epilogue = (tile + 1) * 100 + e runs
 * epilogue e on a pinned tile shape instead of the one the library would choose:
 * tile 0 = 256x256 (8 wavefronts), 1 = 128x128 (4), 2 = 64x64 (4), 3 = 128x128 (8),
 * 4 = 256x128 (8), 5 = 128x128 on a four-stage LDS ring, 6 / 7 / 8 = 64x64 on a
 * ring of 2 / 4 / 8 stages, 9 / 10 = 256x256 as a persistent kernel (one work-group
 * per compute unit walks several tiles; needs K % 128 == 0, K >= 256, N % 4 == 0) /
 * as one work-group per tile (tile 0 takes the first form when there are more tiles
 * than compute units and the shape allows it).  Same values for every tile up to the fp32 summation
 * order inside a k tile (none: all tiles accumulate k in the same order).
 * Errors: SRM_EINVAL (null operand or output, sizes <= 0, K % 64 with SRM_BF16,
 * unknown dtype, epilogue or tile code).
 */
int srm_linear(int32_t dtype, int32_t epilogue, const void *d_A, const void *d_W,
               const float *d_bias, int64_t M, int32_t N, int32_t K, void *d_out,
               int32_t *d_argmax, void *d_scratch, void *hip_stream);
size_t srm_linear_scratch_bytes(int64_t M, int32_t N);

/*
 * srm_linear's epilogue 3 without logits and without a workspace, for callers
 * that cannot allocate device memory or pass a scratch buffer along: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * d_argmax[M] = row-wise argmax of A W^T + bias (lowest index on ties), same
 * kernels and same values as srm_linear(dtype, 3, ..., d_out = NULL, ...).  The
 * per-column-tile partial results live in a device array built into the
 * library (srm_linear_argmax_noalloc_max_bytes() = 8 MiB per GPU, held until
 * the process ends); the call allocates and frees nothing.  A shape whose
 * partials need more (srm_linear_scratch_bytes(M, N) > the maximum, e.g. more
 * than 2097 rows at N = 32000) is rejected with SRM_EINVAL.  All calls on one
 * GPU share that array: calls that overlap in time on one GPU (two streams, two
 * threads) race; calls on one stream do not.  Nothing in the array needs
 * clearing between calls (every partial a call reads, it has written).  The
 * first call on a device looks up the array's address and must not be made
 * under stream capture; later calls may be.
 * Errors: SRM_EINVAL (null pointer, sizes <= 0, K % 64 with SRM_BF16, unknown
 * dtype, shape beyond the built-in scratch), SRM_EHIP.
 */
int srm_linear_argmax_noalloc(int32_t dtype, const void *d_A, const void *d_W, const float *d_bias,
                              int64_t M, int32_t N, int32_t K, int32_t *d_argmax, void *hip_stream);
size_t srm_linear_argmax_noalloc_max_bytes(void);

/*
 * Work-groups of the one-kernel path that srm_generate / srm_generate_topp take
 * for a batch of B samples, or 0 if such a call runs the ordinary step kernels.
 * The one-kernel path ("MAX model details": per-call overhead dominates small
 * batches) serves greedy and temperature sampling (no top-p) for fp32 models
 * with fp32 state and head projections, B <= 8, d_model <= 1024, at most
 * 128 KB for the widest activation row of all samples, and rows x matrix
 * elements below about 16 M (beyond, the step kernels are faster): a small cooperative grid
 * walks through all G steps, its phases separated by grid barriers, so a step
 * costs 4L + 1 barriers instead of 6L + 7 kernel launches.  Same results up to
 * the fp32 summation order.  Environment: SRM_MEGAKERNEL=0 switches it off,
 * SRM_MEGAKERNEL=2 takes it whatever the model's size, SRM_MEGA_BLOCKS=n sets
 * the grid (default 16, at most 64).
 */
int32_t srm_generate_one_kernel_blocks(const srm_model *m, int64_t B);

/*
 * Measuring tools (not part of the model's path): the chip's achievable rates,
 * which the benchmark reports beside the published peaks.
 *
 * srm_probe_copy: d_dst[0..bytes) = d_src[0..bytes) with one plain kernel (device
 * pointers, 16-byte aligned, bytes % 16 == 0, no overlap); streaming != 0 uses
 * non-temporal loads and stores.  HBM traffic = 2 * bytes.
 *
 * srm_probe_mfma: `blocks` work-groups of four wavefronts each issue `iters`
 * rounds of four independent 32x32x16 bf16 matrix-core products on register
 * operands and write one fp32 sum per lane to d_out[blocks * 256].
 * random_operands == 0: A = B = 1, every sum is 1024 * iters (checkable).
 * random_operands != 0: operand elements pseudo-random in (-1, 1), which costs
 * the matrix cores more power than constants do and so shows the rate at the
 * clock the chip holds on real data; the sums are finite, not predictable.
 * *flop (host pointer, may be NULL) receives the floating-point operations of
 * the launch.
 *
 * srm_linear_timeline_probe: sets (d_u64 = NULL or blocks = 0: clears), for the calling thread, a device
 * buffer of 8 * blocks uint64.  While set, every work-group b < blocks of a bf16 srm_linear launch of this
 * thread stores at d_u64 + 8 b: the 100 MHz wall clock at its start, at the start of its k loop, at the end
 * of its k loop and after its last store has completed; the shader cycle counter at the k loop's start and
 * end; HW_ID | XCC_ID << 32 (the CU it ran on); the cycle counter at its start.  (cycles / wall ticks) x
 * 100 MHz is the clock the chip held: the matrix-core peak is quoted at the maximum clock, and under the
 * power of a GEMM on real data the chip holds a lower one.  The work-groups of one CU, ordered by start
 * time, give that CU's timeline: prologue, k loop, epilogue and the turnaround to the next work-group.
 * The persistent form of the 256x256 tile writes one such record per output tile (tile number in place of b;
 * "start" is the end of the work-group's previous tile), and waits for its stores once per tile to do so,
 * which costs it more than it costs the one-tile work-groups: time the two forms with the probe cleared.
 * While it is set, every bf16 tile-GEMM launch of the calling thread writes such records (the model's own
 * launches included, each overwriting the last), and srm_mixer_block's first kernel writes, per work-group:
 * the wall clock at its start, when its first batch of loads has arrived, after LayerNorm1, after the
 * in-projection, after the state update, after the out-projection's products and after its stores have
 * completed; HW_ID | XCC_ID << 32.  Clear it before running a model.
 */
void srm_linear_timeline_probe(void *d_u64, int64_t blocks);
int srm_probe_copy(void *d_dst, const void *d_src, size_t bytes, int32_t streaming, void *hip_stream);
int srm_probe_mfma(float *d_out, int32_t blocks, int32_t iters, int32_t random_operands, double *flop,
                   void *hip_stream);

/* Message for the last failure on the calling thread ("" if none). */
const char *srm_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SRM_H */
