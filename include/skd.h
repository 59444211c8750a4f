/*
 * skd.h -- C ABI of the SkipDecode decode path for AMD MI355X (gfx950).
 *
 * SkipDecode (arXiv 2307.02628) is a token-level early-exit policy for
 * autoregressive decoders that keeps batching and KV caching intact:
 *   - all sequences of a batch compute the same number of layers n(t) at
 *     sequence position t (one exit point per batch column, Section 2.1);
 *   - n(t) never increases with t (Section 2.2), so a layer that runs at
 *     position t already holds the keys/values of every earlier position and
 *     nothing is ever recomputed;
 *   - n(t) decays linearly from n_max to n_min over the generated positions
 *     and the prompt uses all layers (Section 2.3, the token_idx equation);
 *   - the budget is spent on the TOP layers; lower layers are bypassed, i.e.
 *     the hidden state passes through unchanged and no key/value is stored
 *     (Section 2.4), optionally after `warmup` bottom layers.
 * The model is an OPT-style decoder (Section 3): learned positions,
 * pre-LayerNorm blocks with multi-head causal attention and a ReLU FFN, a
 * final LayerNorm and an LM head tied to the token embedding.
 *
 * Conventions
 *   t, i        0-based sequence position (column) of the token being processed
 *   P, N        prompt_size, sequence_length; T = N - P decode steps
 *   B           batch rows; every call works on one column of B tokens
 *   All functions return 0 (SKD_OK) or a positive count on success and a
 *   negative skd_err on failure; nothing aborts or throws across this boundary.
 *   Unless a parameter says "device", pointers are host memory owned by the
 *   caller and only read/written during the call.
 */
#ifndef SKD_H
#define SKD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SKD_OK = 0,
  SKD_ERR_NULL = -1,     /* a required pointer is NULL */
  SKD_ERR_SHAPE = -2,    /* inconsistent configuration (see skd_create) */
  SKD_ERR_RANGE = -3,    /* position, layer, token id or size out of range */
  SKD_ERR_ORDER = -4,    /* call out of sequence (prefill missing, wrong t, ...) */
  SKD_ERR_SCHEDULE = -5, /* layer set not monotone / not ascending */
  SKD_ERR_NOMEM = -6,    /* host or device allocation failed, page pool exhausted */
  SKD_ERR_HIP = -7       /* a HIP runtime call failed (skd_last_hip_error) */
} skd_err;

enum { SKD_BF16 = 0, SKD_FP32 = 1 }; /* skd_config.dtype                 */
enum { SKD_HOST = 0, SKD_DEVICE = 1 }; /* skd_weights.location            */
enum { SKD_W_FP32 = 0, SKD_W_BF16 = 1 }; /* skd_weights.elem              */

typedef struct skd_state skd_state; /* opaque: device weights, KV pages, workspaces */

typedef struct {
  /* model shape */
  int32_t L;        /* num_decoder_layers                                   */
  int32_t d_model;  /* multiple of n_heads; bf16 path: head_dim 64 or 128, d_model <= 16384 */
  int32_t n_heads;
  int32_t ffn;      /* FFN width; bf16 path: d_model and ffn multiples of 32 */
  int32_t vocab;
  int32_t max_pos;  /* rows of the position table, >= sequence_length       */
  /* workload: the hyper-parameters of the Section 2.3 schedule */
  int32_t batch;            /* B >= 1                                        */
  int32_t prompt_size;      /* P >= 1, the padded prompt length             */
  int32_t sequence_length;  /* N > P                                        */
  int32_t n_min, n_max;     /* 1 <= n_min <= n_max <= L                     */
  int32_t warmup;           /* bottom layers always run, 0 <= warmup <= n_min;
                               they count inside n(t) (Section 2.4)         */
  /* implementation knobs */
  int32_t page_tokens;  /* tokens per KV page, multiple of 32; 0 = 64       */
  int32_t dtype;        /* SKD_BF16: bf16 weights/KV/activations, fp32 residual
                           stream and accumulation (the production path);
                           SKD_FP32: everything fp32, simple kernels (debug)  */
  int32_t io_on_device; /* 0: token / logit buffers of prefill, decode_step and
                           logits_argmax are host memory and the calls
                           synchronise; 1: they are device memory and the calls
                           only enqueue work on the stream                    */
} skd_config;

/* Model parameters.  Matrices are [out_features][in_features] row-major.
 * `location` and `elem` apply to every tensor; the per-layer members are HOST
 * arrays of L pointers to tensors at `location`.  skd_create copies what it
 * needs (re-laid-out for the kernels); the caller may free everything after
 * it returns.  With dtype SKD_BF16, matrices and embedding tables are rounded
 * to bf16 (nearest even) if given as fp32; vectors (biases, LayerNorm gain and
 * bias) are kept in fp32 with the values given. */
typedef struct {
  int32_t location;    /* SKD_HOST or SKD_DEVICE */
  int32_t elem;        /* SKD_W_FP32 or SKD_W_BF16 (raw bf16 bit patterns)  */
  const void *tok_emb; /* [vocab][d]   */
  const void *pos_emb; /* [max_pos][d] */
  const void *lnf_g, *lnf_b; /* final LayerNorm [d] */
  const void *lm_head; /* [vocab][d] or NULL = tied to tok_emb */
  const void *const *ln1_g, *const *ln1_b;
  const void *const *wqkv, *const *bqkv; /* [3d][d], [3d]: rows q | k | v, head h = rows h*dh.. within each */
  const void *const *wo, *const *bo;     /* [d][d], [d] */
  const void *const *ln2_g, *const *ln2_b;
  const void *const *w1, *const *b1;     /* [ffn][d], [ffn] */
  const void *const *w2, *const *b2;     /* [d][ffn], [d]   */
} skd_weights;

/* n(t): number of layers computed at position t (Section 2.3, token_idx).
 * t < P gives L.  For P <= t <= N the linear interpolation between n_max (at
 * t = P) and n_min (at t = N) is rounded to the nearest integer, halves up,
 * in exact integer arithmetic.  Host only, no device needed.
 * Errors: SKD_ERR_SHAPE if L < 1, n_min < 1, n_min > n_max, n_max > L, P < 0
 * or N <= P;  SKD_ERR_RANGE if t < 0 or t > N. */
int skd_schedule(int32_t t, int32_t prompt_size, int32_t sequence_length, int32_t n_min, int32_t n_max, int32_t L);

/* Active layers at position t (Section 2.4), ascending, into layers_out[0..L):
 * all L layers on the prompt; afterwards the `warmup` bottom layers plus the
 * top n(t) - warmup layers.  Returns their number.  Uses only the schedule
 * fields and L of cfg.  Errors as skd_schedule, plus SKD_ERR_SHAPE if warmup
 * is outside [0, n_min]. */
int skd_active_layers(int32_t t, const skd_config *cfg, int32_t *layers_out);

/* Build a decoding state on the current HIP device: validates cfg, uploads and
 * re-lays-out the weights, reserves the KV page pool.  The pool holds exactly
 * the entries the static schedule will ever write (P*L + sum of n(t) per row,
 * rounded up to pages per layer), not N*L.  `hip_stream` is a hipStream_t (NULL =
 * the default stream) on which every later call of this state enqueues its
 * work.  Errors: SKD_ERR_NULL; SKD_ERR_SHAPE (d % heads, N <= P, P < 1,
 * max_pos < N, schedule fields, page_tokens % 32, bf16-path shape limits
 * above, unknown enum); SKD_ERR_NOMEM; SKD_ERR_HIP. */
int skd_create(const skd_config *cfg, const skd_weights *w, void *hip_stream, skd_state **out);

/* As skd_create, with the layer count of EVERY position supplied by the caller
 * instead of the linear decay: n_table[i], i = 0..N-1 (the paper leaves the
 * decay function open: power law, Section 2.3 / Section 5; decay that already
 * starts inside the prompt, Section 5).  The table must be non-increasing
 * (SKD_ERR_SCHEDULE otherwise: a layer that re-enters would miss keys, Section
 * 2.2), with 1 <= n_table[i] <= L (SKD_ERR_RANGE) and n_table[i] >= warmup
 * (SKD_ERR_SHAPE).  n_min / n_max of cfg must still be valid but are not used;
 * prefill processes prompt column i with n_table[i] layers.  The active set
 * keeps its shape: `warmup` bottom layers plus the top n - warmup. */
int skd_create_with_schedule(const skd_config *cfg, const skd_weights *w, void *hip_stream,
                             const int32_t *n_table, skd_state **out);

/* Active layers of this state at position t (0 <= t < N), ascending, into
 * layers_out[0..L); returns their number.  Equals skd_active_layers for states
 * made by skd_create. */
int skd_state_active_layers(const skd_state *st, int32_t t, int32_t *layers_out);

/* Process the prompt: columns 0..P-1, every one through all L layers
 * (Section 2.3: the prompt uses the full network), filling every layer's KV
 * cache.  tokens [B][P] int32 row-major.  attn_mask [B][P] uint8, 1 = real
 * token, NULL = all real; only LEFT padding is accepted (each row is zeros
 * followed by at least one 1), anything else is SKD_ERR_SHAPE.  Position ids
 * count real tokens; padded entries are never attended to.  Restarts the
 * generation if one was in progress.  With io_on_device = 1, `tokens` is a
 * device pointer laid out [P][B] (column-major) and attn_mask stays a host
 * pointer.  Errors: SKD_ERR_NULL, SKD_ERR_RANGE (host token outside
 * [0, vocab)), SKD_ERR_SHAPE, SKD_ERR_HIP.  Device-resident token ids are
 * not validated; the kernels clamp them into [0, vocab). */
int skd_prefill(skd_state *st, const int32_t *tokens, const uint8_t *attn_mask);

/* One decode step: process column t for all B rows with the layer set of
 * skd_active_layers(t).  Layers outside the set are not launched: the hidden
 * state passes through them and they store no key/value (Section 2.4).
 * tokens_in [B] is the column's input (the tokens generated for position t);
 * NULL = use the tokens the last skd_logits_argmax produced (greedy
 * free-running).  t must equal P + (decode steps done so far) and be < N:
 * the whole batch shares one position (Sections 2.1 and 5).
 * Errors: SKD_ERR_NULL, SKD_ERR_ORDER (no prefill, wrong t, NULL tokens_in
 * with no argmax since the last step), SKD_ERR_RANGE (t >= N, host token id),
 * SKD_ERR_HIP. */
int skd_decode_step(skd_state *st, int32_t t, const int32_t *tokens_in);

/* Final LayerNorm + LM head + greedy argmax on the hidden state of the last
 * processed column: every column emits a token for the whole batch, whatever
 * number of layers it ran (Section 2.1: one exit point per batch column; the
 * hidden state that leaves the last active layer goes straight to the head,
 * Section 2.4).  The paper leaves the head itself to the base model: the final
 * LayerNorm and the LM head always run and the head is tied to the token
 * embedding unless skd_weights.lm_head is given; the contract path is greedy
 * (beam 1), with the LOWEST index winning ties, and Section 3.2's sampling
 * setting is skd_logits_sample below.  tokens_out [B] (may be NULL) receives, per row, the
 * lowest index attaining the maximum logit; logits_out [B][vocab] fp32 (may be
 * NULL) receives the logits.  The tokens are also kept inside the state for
 * skd_decode_step(.., NULL).  Errors: SKD_ERR_NULL, SKD_ERR_ORDER (nothing
 * processed yet), SKD_ERR_HIP. */
int skd_logits_argmax(skd_state *st, int32_t *tokens_out, float *logits_out);

/* skd_logits_argmax for callers that cannot allocate device memory: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same kernels and the same results, but the LM head's per-workgroup
 * (max, argmax) partials live in a file-scope static device array of 2 MiB
 * (every GPU the library runs on holds its own copy until the process ends)
 * instead of buffers of the state, and the call itself calls no hipMalloc,
 * hipFree or other allocating routine.  Only for states with dtype SKD_BF16
 * and io_on_device = 1 (SKD_ERR_SHAPE otherwise): tokens_out [B] and
 * logits_out [B][vocab] (either may be NULL) are device memory and the call
 * only enqueues work on the state's stream.  Limit:
 * ceil(vocab / (16 R)) * B_pad <= 262144 partials, R = LM-head tile rows per
 * workgroup (2 below batch 32, else 4; SKD_R_HEAD), B_pad = batch padded to
 * 16/32/64/128, i.e. vocabularies up to 131072 at batch 128 and larger ones
 * at smaller batches; beyond the limit SKD_ERR_RANGE and nothing is launched.  All calls on one GPU, from whatever
 * state, share that GPU's array: calls that may overlap there (different
 * streams, different threads) race; calls on one stream are safe.  The array
 * keeps the previous call's contents; nothing in it needs clearing, since the
 * projection of a call writes every partial its final reduction reads.
 * Errors otherwise as skd_logits_argmax. */
int skd_logits_argmax_noalloc(skd_state *st, int32_t *tokens_out, float *logits_out);

/* Sampling head (the paper's generation setting: temperature 0.3, top-p 0.7,
 * Section 3.2) in place of the greedy argmax: final LayerNorm + LM head, then
 * per row, with p_i = exp((z_i - max z) / temperature): the nucleus is the
 * smallest set of most likely tokens whose mass reaches top_p (tokens tied with
 * the last admitted one are admitted too), and the token is the first index of
 * the nucleus, in ascending index order, whose running mass exceeds
 * u[b] * mass(nucleus).  u [B] are uniform numbers in [0,1) supplied by the
 * caller (host memory, or device memory with io_on_device = 1): the library
 * draws no random numbers.  Deterministic for given (state, u).  tokens_out [B]
 * and logits_out [B][vocab] may be NULL; the tokens are kept for
 * skd_decode_step(.., NULL).  vocab <= 65536.  Errors: SKD_ERR_NULL,
 * SKD_ERR_ORDER, SKD_ERR_RANGE (temperature <= 0, top_p outside (0,1], host u
 * outside [0,1)), SKD_ERR_SHAPE, SKD_ERR_HIP. */
int skd_logits_sample(skd_state *st, const float *u, float temperature, float top_p, int32_t *tokens_out,
                      float *logits_out);

/* Move the generation back to position t (P <= t <= current position): the
 * next skd_decode_step must be for column t; cache entries at columns >= t are
 * forgotten (they are overwritten when those columns are processed again).
 * The static schedule makes this exact: which layers hold which columns only
 * depends on t.  Used to regenerate from a point and to time a run after a
 * warm-up without repeating the prompt.  Errors: SKD_ERR_NULL, SKD_ERR_ORDER
 * (no prefill), SKD_ERR_RANGE. */
int skd_rewind(skd_state *st, int32_t t);

/* Number of columns layer `layer`'s KV cache holds (host bookkeeping).  For a
 * layer active at t this equals t before the step and t + 1 after it. */
int skd_kv_len(const skd_state *st, int32_t layer);

/* KV pages reserved for the whole state and pages that would be needed
 * without layer-sparse reservation (N tokens in every layer). */
int64_t skd_kv_pages_reserved(const skd_state *st);
int64_t skd_kv_pages_dense(const skd_state *st);

/* Wait until everything enqueued by this state has finished. */
int skd_synchronize(skd_state *st);

/* Test / measurement hooks ------------------------------------------------ */

/* Copy the fp32 residual stream of the last processed column to host x_out [B][d]. */
int skd_debug_read_hidden(skd_state *st, float *x_out);

/* Declare columns 0..cols-1 processed (P <= cols < N), as if a prompt of that
 * length had run, and set layer caches from host arrays: for each layer l with
 * Kin[l] != NULL, Kin[l] and Vin[l] are [B][cols][d] fp32 and become that
 * layer's cache (rounded to the path's KV precision); layers with NULL entries
 * hold zeros.  Layers that leave the active window before column `cols` keep
 * only what they reserved.  start [B] (may be NULL = no padding) gives each
 * row's number of left-padding columns, 0 <= start[b] < cols; the entries of
 * Kin / Vin at those columns are ignored.  Used to set up
 * single decode steps at long contexts without running a long prompt.  Kin /
 * Vin are host arrays of L host pointers.  Errors: SKD_ERR_NULL,
 * SKD_ERR_RANGE, SKD_ERR_NOMEM, SKD_ERR_HIP. */
int skd_debug_kv_load(skd_state *st, int32_t cols, const float *const *Kin, const float *const *Vin,
                      const int32_t *start);

/* Read back row b of layer l's cache: k_out, v_out [len][d] fp32 with
 * len = skd_kv_len(l), indexed by column.  Left-padding columns of the row are
 * never attended to; what is returned for them is unspecified (the bf16 path
 * stores nothing for them and returns zeros). */
int skd_debug_kv_read(skd_state *st, int32_t layer, int32_t b, float *k_out, float *v_out);

/* Per-kernel timing.  skd_profile_enable(st, 1): every kernel launch of this
 * state is given its own pair of HIP events that receive the begin and end time
 * stamps of that kernel (what a kernel trace reports as its duration); mode 2
 * instead records one event before and one after the launches of each class
 * on the state's stream, which adds the cost of the two markers to every
 * measurement; 0 switches timing off.  Neither mode serialises anything, but
 * both cost host time per launch, so time whole runs with timing off.
 * skd_profile_read waits for the stream and adds the elapsed milliseconds and
 * launch counts per kernel class into ms[SKD_PROF_CLASSES] and
 * launches[SKD_PROF_CLASSES] (either may be NULL), then clears the internal
 * accumulators.  Classes: see skd_prof_class.  Errors: SKD_ERR_NULL,
 * SKD_ERR_RANGE (mode), SKD_ERR_HIP. */
typedef enum {
  SKD_PROF_EMBED_LN = 0, /* embedding gather + first LayerNorm */
  SKD_PROF_GEMM_QKV = 1, /* q,k,v projection + KV page write  */
  SKD_PROF_ATTENTION = 2,/* decode attention over the paged KV (incl. split merge) */
  SKD_PROF_GEMM_OUT = 3, /* attention output projection        */
  SKD_PROF_REDUCE_LN = 4,/* split-K reduce + bias + residual + LayerNorm */
  SKD_PROF_GEMM_FFN1 = 5,
  SKD_PROF_GEMM_FFN2 = 6,
  SKD_PROF_LM_HEAD = 7,  /* LM head projection with per-workgroup argmax */
  SKD_PROF_ARGMAX = 8,   /* final argmax reduction             */
  SKD_PROF_OTHER = 9,    /* fp32 debug path kernels            */
  SKD_PROF_CLASSES = 10
} skd_prof_class;
int skd_profile_enable(skd_state *st, int32_t on);
int skd_profile_read(skd_state *st, double *ms, int64_t *launches);

void skd_destroy(skd_state *st);
const char *skd_strerror(int err);
/* hipError_t (as int) of the most recent failing HIP call on this thread, 0 if none. */
int skd_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SKD_H */
