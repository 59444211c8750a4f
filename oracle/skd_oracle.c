/*
 * SkipDecode CPU oracle  --  TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct CPU implementation of what the SkipDecode
 * decode path computes, written from the paper so that the HIP library can be
 * checked against it.  Only the test-suite, the smoke check and the benchmark's
 * "cpu_baseline" leg may call it; the product never does.  It shares no code,
 * header, table or helper with the HIP path.
 *
 * Arithmetic type: `real` (ORA_REAL, double by default; a float build of the
 * same file gives the fp32 variant).  Weights arrive as float arrays and are
 * promoted on use.  Plain loops, sequential accumulation, no blocking, no
 * fusion; OpenMP only over independent outputs (batch rows / output features).
 *
 * What follows the paper, passage by passage:
 *   ora_schedule        Section 2.3, the piecewise token_idx equation (linear
 *                       decay between max_exit_layer and min_exit_layer over
 *                       the generated positions, num_decoder_layers on the
 *                       prompt), rounded half-up in exact integer arithmetic.
 *   ora_active_layers   Section 2.4: the budget is spent on the TOP layers
 *                       (skipping, not early termination), optionally after
 *                       `warmup` bottom layers.
 *   ora_column          Sections 2.1-2.2: one column of the batch (all rows at
 *                       one position) runs the same layer set; each active
 *                       layer appends its key/value to that layer's cache and
 *                       attends to the cache of the same layer; inactive
 *                       layers are the identity and store nothing.
 *   ora_recompute       the same function without any cache: every position
 *                       is recomputed, layer by layer (brute-force check of
 *                       the Section 2.2 claim that monotone exits never need
 *                       a key/value that was not stored).
 * The decoder block is the OPT one (Section 3: OPT decoder-only models):
 * pre-LayerNorm, learned positions, multi-head causal attention, ReLU FFN,
 * final LayerNorm, LM head tied to the token embedding unless one is given.
 *
 * Pins (tests/test_oracle_*.py): the worked example of Fig. 3 and the means
 * of Table 2 for the schedule; an independent composition of library ops for
 * the full-depth decoder and for the prefix form of skipping; cached ==
 * non-cached; batch / padding invariance; skipped-layer weights are dead.
 * Output *quality* of SkipDecode (Table 4) is not reproduced: parity unpinned
 * for that, it needs the paper's trained weights and datasets.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef ORA_REAL
#define ORA_REAL double
#endif
typedef ORA_REAL real;

enum {
  ORA_OK = 0,
  ORA_ERR_NULL = -1,
  ORA_ERR_SHAPE = -2,
  ORA_ERR_RANGE = -3,
  ORA_ERR_ORDER = -4,
  ORA_ERR_SCHEDULE = -5,
  ORA_ERR_NOMEM = -6
};

typedef struct {
  int32_t L, d, H, f, V, max_pos;
} ora_shape;

/* All matrices are [out_features][in_features], row-major, float. */
typedef struct {
  const float *tok_emb; /* [V][d] */
  const float *pos_emb; /* [max_pos][d] */
  const float *lnf_g, *lnf_b;
  const float *lm_head; /* [V][d]; NULL = tied to tok_emb */
  const float *const *ln1_g, *const *ln1_b;
  const float *const *wqkv, *const *bqkv; /* [3d][d]: rows q | k | v */
  const float *const *wo, *const *bo;     /* [d][d] */
  const float *const *ln2_g, *const *ln2_b;
  const float *const *w1, *const *b1;     /* [f][d] */
  const float *const *w2, *const *b2;     /* [d][f] */
} ora_weights;

int ora_real_bytes(void) { return (int)sizeof(real); }

#ifdef _OPENMP
#include <omp.h>
int ora_threads(void) { return omp_get_max_threads(); }
#else
int ora_threads(void) { return 1; }
#endif

/* ------------------------------------------------------------------ */
/* Schedule (Section 2.3)                                              */
/* ------------------------------------------------------------------ */

/* Number of layers computed at 0-based position i.
 * Prompt positions (i < P) use all L layers.  For P <= i <= N the paper's
 * real value is (1 - t) * n_max + t * n_min with t = (i - P) / (N - P); it is
 * rounded to the nearest integer, halves up, without any floating point:
 * floor(r + 1/2) = floor((2 * (n_max (T - k) + n_min k) + T) / (2 T)). */
int ora_schedule(int32_t i, int32_t P, int32_t N, int32_t n_min, int32_t n_max, int32_t L) {
  if (L < 1 || n_min < 1 || n_min > n_max || n_max > L || P < 0 || N <= P) return ORA_ERR_SHAPE;
  if (i < 0 || i > N) return ORA_ERR_RANGE;
  if (i < P) return L;
  int64_t T = (int64_t)N - P, k = (int64_t)i - P;
  int64_t twice_r_times_T = 2 * ((int64_t)n_max * (T - k) + (int64_t)n_min * k);
  return (int)((twice_r_times_T + T) / (2 * T));
}

/* Active layer set at position i, ascending, written to out[0..count).
 * `warmup` bottom layers run first, the rest of the budget n(i) goes to the
 * top of the stack (Section 2.4).  warmup = 0 is the plain top window. */
int ora_active_layers(int32_t i, int32_t P, int32_t N, int32_t n_min, int32_t n_max,
                      int32_t warmup, int32_t L, int32_t *out) {
  if (!out) return ORA_ERR_NULL;
  int n = ora_schedule(i, P, N, n_min, n_max, L);
  if (n < 0) return n;
  if (warmup < 0 || warmup > n_min) return ORA_ERR_SHAPE;
  int c = 0;
  if (i < P) {
    for (int l = 0; l < L; ++l) out[c++] = l;
    return c;
  }
  for (int l = 0; l < warmup; ++l) out[c++] = l;
  int top = n - warmup;
  for (int l = L - top; l < L; ++l) out[c++] = l;
  return c;
}

/* ------------------------------------------------------------------ */
/* Elementary operations                                               */
/* ------------------------------------------------------------------ */

/* LayerNorm over the last dimension: mean and biased variance, eps 1e-5. */
static void layernorm(const real *x, const float *g, const float *b, int d, real *out) {
  real mean = 0;
  for (int k = 0; k < d; ++k) mean += x[k];
  mean /= (real)d;
  real var = 0;
  for (int k = 0; k < d; ++k) var += (x[k] - mean) * (x[k] - mean);
  var /= (real)d;
  real rstd = (real)1 / (real)sqrt((double)(var + (real)1e-5));
  for (int k = 0; k < d; ++k) out[k] = (x[k] - mean) * rstd * (real)g[k] + (real)b[k];
}

/* out[r][o] = bias[o] + sum_k W[o][k] * in[r][k]      (rows r independent) */
static void linear(const float *W, const float *bias, const real *in, int rows, int K, int N,
                   real *out) {
#pragma omp parallel for collapse(2) schedule(static)
  for (int r = 0; r < rows; ++r)
    for (int o = 0; o < N; ++o) {
      const float *w = W + (size_t)o * K;
      const real *a = in + (size_t)r * K;
      real acc = 0;
      for (int k = 0; k < K; ++k) acc += (real)w[k] * a[k];
      out[(size_t)r * N + o] = acc + (bias ? (real)bias[o] : (real)0);
    }
}

/* One query against `len` cached keys/values of one sequence, all heads.
 * Kc, Vc: [len][d] (head h owns columns h*dh .. h*dh+dh-1); valid[j] = 0
 * removes key j from the softmax.  scores = q.k / sqrt(dh), softmax with the
 * maximum subtracted, out = sum_j p_j v_j.  No valid key => out = 0. */
static void attention(const real *q, const real *Kc, const real *Vc, const uint8_t *valid, int len,
                      int H, int dh, real *out, real *scratch /* [len] */) {
  int d = H * dh;
  real inv = (real)1 / (real)sqrt((double)dh);
  for (int h = 0; h < H; ++h) {
    real mx = 0;
    int any = 0;
    for (int j = 0; j < len; ++j) {
      if (!valid[j]) continue;
      real s = 0;
      for (int e = 0; e < dh; ++e) s += q[h * dh + e] * Kc[(size_t)j * d + h * dh + e];
      s *= inv;
      scratch[j] = s;
      if (!any || s > mx) mx = s;
      any = 1;
    }
    for (int e = 0; e < dh; ++e) out[h * dh + e] = 0;
    if (!any) continue;
    real den = 0;
    for (int j = 0; j < len; ++j) {
      if (!valid[j]) continue;
      scratch[j] = (real)exp((double)(scratch[j] - mx));
      den += scratch[j];
    }
    for (int j = 0; j < len; ++j) {
      if (!valid[j]) continue;
      real p = scratch[j] / den;
      for (int e = 0; e < dh; ++e) out[h * dh + e] += p * Vc[(size_t)j * d + h * dh + e];
    }
  }
}

static int check_shape(const ora_shape *s) {
  if (!s) return ORA_ERR_NULL;
  if (s->L < 1 || s->d < 1 || s->H < 1 || s->f < 1 || s->V < 1 || s->max_pos < 1) return ORA_ERR_SHAPE;
  if (s->d % s->H) return ORA_ERR_SHAPE;
  return ORA_OK;
}

/* ------------------------------------------------------------------ */
/* Cached column-by-column decoder (Sections 2.1, 2.2, 2.4)            */
/* ------------------------------------------------------------------ */

typedef struct {
  ora_shape s;
  ora_weights w;
  int B, N;
  real **K, **V;  /* [L] -> [B][N][d], allocated when the layer first runs */
  int *len;       /* [L] number of columns the layer's cache holds */
  uint8_t *valid; /* [B][N] 1 where row b holds a real (non-pad) token */
  int *n_real;    /* [B] real tokens seen so far = next position id */
  int next_col;
} ora_state;

void ora_free(ora_state *st) {
  if (!st) return;
  if (st->K)
    for (int l = 0; l < st->s.L; ++l) free(st->K[l]);
  if (st->V)
    for (int l = 0; l < st->s.L; ++l) free(st->V[l]);
  free(st->K);
  free(st->V);
  free(st->len);
  free(st->valid);
  free(st->n_real);
  free(st);
}

int ora_new(const ora_shape *s, const ora_weights *w, int32_t B, int32_t N, ora_state **out) {
  if (!s || !w || !out) return ORA_ERR_NULL;
  int rc = check_shape(s);
  if (rc) return rc;
  if (B < 1 || N < 1 || N > s->max_pos) return ORA_ERR_SHAPE;
  ora_state *st = (ora_state *)calloc(1, sizeof(*st));
  if (!st) return ORA_ERR_NOMEM;
  st->s = *s;
  st->w = *w;
  st->B = B;
  st->N = N;
  st->K = (real **)calloc(s->L, sizeof(real *));
  st->V = (real **)calloc(s->L, sizeof(real *));
  st->len = (int *)calloc(s->L, sizeof(int));
  st->valid = (uint8_t *)calloc((size_t)B * N, 1);
  st->n_real = (int *)calloc(B, sizeof(int));
  if (!st->K || !st->V || !st->len || !st->valid || !st->n_real) {
    ora_free(st);
    return ORA_ERR_NOMEM;
  }
  *out = st;
  return ORA_OK;
}

int ora_kv_len(const ora_state *st, int32_t layer) {
  if (!st) return ORA_ERR_NULL;
  if (layer < 0 || layer >= st->s.L) return ORA_ERR_RANGE;
  return st->len[layer];
}

static int ensure_layer_cache(ora_state *st, int l) {
  if (st->K[l]) return ORA_OK;
  size_t n = (size_t)st->B * st->N * st->s.d;
  st->K[l] = (real *)calloc(n, sizeof(real));
  st->V[l] = (real *)calloc(n, sizeof(real));
  return (st->K[l] && st->V[l]) ? ORA_OK : ORA_ERR_NOMEM;
}

/* Test / timing hook: place `cols` columns of given keys and values
 * ([B][cols][d] float each) into layer l's cache, as if the layer had been
 * active at columns 0..cols-1 with every token real.  Only used to set up
 * single-step checks and the bounded CPU timing sample at long contexts. */
int ora_kv_load(ora_state *st, int32_t l, int32_t cols, const float *Kin, const float *Vin) {
  if (!st || !Kin || !Vin) return ORA_ERR_NULL;
  if (l < 0 || l >= st->s.L || cols < 0 || cols > st->N) return ORA_ERR_RANGE;
  int rc = ensure_layer_cache(st, l);
  if (rc) return rc;
  int d = st->s.d;
  for (int b = 0; b < st->B; ++b)
    for (int j = 0; j < cols; ++j)
      for (int e = 0; e < d; ++e) {
        st->K[l][((size_t)b * st->N + j) * d + e] = (real)Kin[((size_t)b * cols + j) * d + e];
        st->V[l][((size_t)b * st->N + j) * d + e] = (real)Vin[((size_t)b * cols + j) * d + e];
      }
  st->len[l] = cols;
  return ORA_OK;
}

/* Test hook: copy the keys and values layer l holds for row b ([len][d] double
 * each) out of the cache.  Returns the number of columns copied. */
int ora_kv_read(const ora_state *st, int32_t l, int32_t b, double *Kout, double *Vout) {
  if (!st || !Kout || !Vout) return ORA_ERR_NULL;
  if (l < 0 || l >= st->s.L || b < 0 || b >= st->B) return ORA_ERR_RANGE;
  int d = st->s.d, len = st->len[l];
  if (!st->K[l]) return 0;
  for (int j = 0; j < len; ++j)
    for (int e = 0; e < d; ++e) {
      Kout[(size_t)j * d + e] = (double)st->K[l][((size_t)b * st->N + j) * d + e];
      Vout[(size_t)j * d + e] = (double)st->V[l][((size_t)b * st->N + j) * d + e];
    }
  return len;
}

/* Companion of ora_kv_load: declare columns 0..cols-1 real for every row and
 * move the column cursor there. */
int ora_seek(ora_state *st, int32_t cols) {
  if (!st) return ORA_ERR_NULL;
  if (cols < 0 || cols > st->N) return ORA_ERR_RANGE;
  for (int b = 0; b < st->B; ++b) {
    for (int j = 0; j < cols; ++j) st->valid[(size_t)b * st->N + j] = 1;
    st->n_real[b] = cols;
  }
  st->next_col = cols;
  return ORA_OK;
}

/* As ora_seek, with left padding: row b's columns 0..start[b]-1 are padding
 * (never attended to, no position id). */
int ora_seek_ragged(ora_state *st, int32_t cols, const int32_t *start) {
  if (!st || !start) return ORA_ERR_NULL;
  if (cols < 0 || cols > st->N) return ORA_ERR_RANGE;
  for (int b = 0; b < st->B; ++b) {
    if (start[b] < 0 || start[b] >= cols) return ORA_ERR_RANGE;
    for (int j = 0; j < cols; ++j) st->valid[(size_t)b * st->N + j] = (uint8_t)(j >= start[b]);
    st->n_real[b] = cols - start[b];
  }
  st->next_col = cols;
  return ORA_OK;
}

/* Process column i for all B rows with the given ascending layer list.
 *   tokens[B]      input token of each row at column i
 *   real_tok[B]    1 = real token, 0 = padding (NULL = all real).  A padded
 *                  entry is never read by any later softmax and does not
 *                  advance the row's position id.
 *   logits[B][V]   (double, may be NULL) output after the final LayerNorm and
 *                  the LM head;  argmax[B] (may be NULL) lowest index of the
 *                  maximum.
 * Columns must come in order (i == number of columns processed so far), and a
 * layer that runs at column i must already hold columns 0..i-1 in its cache:
 * that is the property Section 2.2 derives from monotonically decreasing exit
 * points; a layer set that violates it is refused (ORA_ERR_ORDER). */
int ora_column(ora_state *st, int32_t i, const int32_t *tokens, const uint8_t *real_tok,
               const int32_t *layers, int32_t n_layers, double *logits, int32_t *argmax) {
  if (!st || !tokens || (!layers && n_layers > 0)) return ORA_ERR_NULL;
  const ora_shape *s = &st->s;
  const ora_weights *w = &st->w;
  const int B = st->B, d = s->d, f = s->f, H = s->H, dh = d / H, V = s->V, N = st->N;
  if (i != st->next_col) return ORA_ERR_ORDER;
  if (i < 0 || i >= N) return ORA_ERR_RANGE;
  if (n_layers < 0 || n_layers > s->L) return ORA_ERR_RANGE;
  for (int a = 0; a < n_layers; ++a) {
    if (layers[a] < 0 || layers[a] >= s->L) return ORA_ERR_RANGE;
    if (a && layers[a] <= layers[a - 1]) return ORA_ERR_SCHEDULE;
    if (st->len[layers[a]] != i) return ORA_ERR_ORDER; /* a key/value would be missing */
  }
  for (int b = 0; b < B; ++b) {
    if (tokens[b] < 0 || tokens[b] >= V) return ORA_ERR_RANGE;
    if (st->n_real[b] >= s->max_pos) return ORA_ERR_RANGE;
  }

  real *x = (real *)malloc(sizeof(real) * (size_t)B * d);
  real *a1 = (real *)malloc(sizeof(real) * (size_t)B * d);
  real *qkv = (real *)malloc(sizeof(real) * (size_t)B * 3 * d);
  real *o = (real *)malloc(sizeof(real) * (size_t)B * d);
  real *t1 = (real *)malloc(sizeof(real) * (size_t)B * d);
  real *u = (real *)malloc(sizeof(real) * (size_t)B * f);
  real *sc = (real *)malloc(sizeof(real) * (size_t)B * (i + 1));
  real *z = (real *)malloc(sizeof(real) * (size_t)B * V);
  int rc = ORA_OK;
  if (!x || !a1 || !qkv || !o || !t1 || !u || !sc || !z) {
    rc = ORA_ERR_NOMEM;
    goto done;
  }

  /* token + learned position embedding; position id = real tokens before */
  for (int b = 0; b < B; ++b) {
    int is_real = real_tok ? (real_tok[b] != 0) : 1;
    st->valid[(size_t)b * N + i] = (uint8_t)is_real;
    int pos = st->n_real[b];
    for (int k = 0; k < d; ++k)
      x[(size_t)b * d + k] = (real)w->tok_emb[(size_t)tokens[b] * d + k] + (real)w->pos_emb[(size_t)pos * d + k];
    if (is_real) st->n_real[b] += 1;
  }

  for (int a = 0; a < n_layers; ++a) {
    const int l = layers[a];
    rc = ensure_layer_cache(st, l);
    if (rc) goto done;
    /* self-attention sub-block: x += Wo . attn(LN1(x)) + bo */
    for (int b = 0; b < B; ++b) layernorm(x + (size_t)b * d, w->ln1_g[l], w->ln1_b[l], d, a1 + (size_t)b * d);
    linear(w->wqkv[l], w->bqkv[l], a1, B, d, 3 * d, qkv);
    for (int b = 0; b < B; ++b) {
      real *Kd = st->K[l] + ((size_t)b * N + i) * d;
      real *Vd = st->V[l] + ((size_t)b * N + i) * d;
      for (int k = 0; k < d; ++k) {
        Kd[k] = qkv[(size_t)b * 3 * d + d + k];
        Vd[k] = qkv[(size_t)b * 3 * d + 2 * d + k];
      }
    }
    st->len[l] = i + 1;
#pragma omp parallel for schedule(static)
    for (int b = 0; b < B; ++b)
      attention(qkv + (size_t)b * 3 * d, st->K[l] + (size_t)b * N * d, st->V[l] + (size_t)b * N * d,
                st->valid + (size_t)b * N, i + 1, H, dh, o + (size_t)b * d, sc + (size_t)b * (i + 1));
    linear(w->wo[l], w->bo[l], o, B, d, d, t1);
    for (size_t k = 0; k < (size_t)B * d; ++k) x[k] += t1[k];
    /* feed-forward sub-block: x += W2 . relu(W1 . LN2(x) + b1) + b2 */
    for (int b = 0; b < B; ++b) layernorm(x + (size_t)b * d, w->ln2_g[l], w->ln2_b[l], d, a1 + (size_t)b * d);
    linear(w->w1[l], w->b1[l], a1, B, d, f, u);
    for (size_t k = 0; k < (size_t)B * f; ++k) u[k] = u[k] > 0 ? u[k] : 0;
    linear(w->w2[l], w->b2[l], u, B, f, d, t1);
    for (size_t k = 0; k < (size_t)B * d; ++k) x[k] += t1[k];
  }
  /* layers not in the list: nothing happens, nothing is stored */

  st->next_col = i + 1;
  if (logits || argmax) {
    for (int b = 0; b < B; ++b) layernorm(x + (size_t)b * d, w->lnf_g, w->lnf_b, d, a1 + (size_t)b * d);
    linear(w->lm_head ? w->lm_head : w->tok_emb, NULL, a1, B, d, V, z);
    for (int b = 0; b < B; ++b) {
      int best = 0;
      for (int v = 0; v < V; ++v) {
        if (logits) logits[(size_t)b * V + v] = (double)z[(size_t)b * V + v];
        if (z[(size_t)b * V + v] > z[(size_t)b * V + best]) best = v;
      }
      if (argmax) argmax[b] = best;
    }
  }
done:
  free(x); free(a1); free(qkv); free(o); free(t1); free(u); free(sc); free(z);
  return rc;
}

/* ------------------------------------------------------------------ */
/* Non-cached recomputation (brute force)                              */
/* ------------------------------------------------------------------ */

/* Recompute columns 0..C-1 from nothing and return the logits of the last
 * one.  layer_on[j][l] (uint8, [C][L]) says whether layer l runs at column j.
 * The loop nest is layer-major (all columns through layer 0, then layer 1,
 * ...), i.e. the transpose of ora_column's column-major order; nothing is
 * kept between calls.  Layer l's keys/values exist only at the columns where
 * it ran; if it runs at column j but did not run at some j' < j, the key the
 * attention needs was never produced and the set is refused
 * (ORA_ERR_SCHEDULE) -- with monotonically decreasing exits this cannot
 * happen (Section 2.2). */
int ora_recompute(const ora_shape *s, const ora_weights *w, int32_t B, int32_t C,
                  const int32_t *tokens /* [B][C] */, const uint8_t *real_tok /* [B][C] or NULL */,
                  const uint8_t *layer_on /* [C][L] */, double *logits /* [B][V] */) {
  if (!s || !w || !tokens || !layer_on || !logits) return ORA_ERR_NULL;
  int rc = check_shape(s);
  if (rc) return rc;
  if (B < 1 || C < 1 || C > s->max_pos) return ORA_ERR_SHAPE;
  const int d = s->d, f = s->f, H = s->H, dh = d / H, V = s->V, L = s->L;
  for (int l = 0; l < L; ++l) {
    int seen_off = 0;
    for (int j = 0; j < C; ++j) {
      if (!layer_on[(size_t)j * L + l]) seen_off = 1;
      else if (seen_off) return ORA_ERR_SCHEDULE;
    }
  }
  size_t BC = (size_t)B * C;
  real *h = (real *)malloc(sizeof(real) * BC * d);
  real *a1 = (real *)malloc(sizeof(real) * BC * d);
  real *qkv = (real *)malloc(sizeof(real) * BC * 3 * d);
  real *Kc = (real *)malloc(sizeof(real) * BC * d);
  real *Vc = (real *)malloc(sizeof(real) * BC * d);
  real *o = (real *)malloc(sizeof(real) * BC * d);
  real *t1 = (real *)malloc(sizeof(real) * BC * d);
  real *u = (real *)malloc(sizeof(real) * BC * f);
  real *sc = (real *)malloc(sizeof(real) * (size_t)C);
  real *z = (real *)malloc(sizeof(real) * (size_t)V);
  uint8_t *valid = (uint8_t *)malloc(BC);
  if (!h || !a1 || !qkv || !Kc || !Vc || !o || !t1 || !u || !sc || !z || !valid) {
    rc = ORA_ERR_NOMEM;
    goto done;
  }
  for (int b = 0; b < B; ++b) {
    int pos = 0;
    for (int j = 0; j < C; ++j) {
      int tok = tokens[(size_t)b * C + j];
      int is_real = real_tok ? (real_tok[(size_t)b * C + j] != 0) : 1;
      if (tok < 0 || tok >= V || pos >= s->max_pos) { rc = ORA_ERR_RANGE; goto done; }
      valid[(size_t)b * C + j] = (uint8_t)is_real;
      for (int k = 0; k < d; ++k)
        h[((size_t)b * C + j) * d + k] = (real)w->tok_emb[(size_t)tok * d + k] + (real)w->pos_emb[(size_t)pos * d + k];
      if (is_real) pos += 1;
    }
  }
  for (int l = 0; l < L; ++l) {
    /* columns where layer l runs form a prefix 0..cl-1 (checked above) */
    int cl = 0;
    while (cl < C && layer_on[(size_t)cl * L + l]) ++cl;
    if (cl == 0) continue;
    for (int b = 0; b < B; ++b) {
      real *hb = h + (size_t)b * C * d;
      real *ab = a1 + (size_t)b * C * d;
      real *qb = qkv + (size_t)b * C * 3 * d;
      real *Kb = Kc + (size_t)b * C * d, *Vb = Vc + (size_t)b * C * d;
      real *ob = o + (size_t)b * C * d, *tb = t1 + (size_t)b * C * d, *ub = u + (size_t)b * C * f;
      for (int j = 0; j < cl; ++j) layernorm(hb + (size_t)j * d, w->ln1_g[l], w->ln1_b[l], d, ab + (size_t)j * d);
      linear(w->wqkv[l], w->bqkv[l], ab, cl, d, 3 * d, qb);
      for (int j = 0; j < cl; ++j)
        for (int k = 0; k < d; ++k) {
          Kb[(size_t)j * d + k] = qb[(size_t)j * 3 * d + d + k];
          Vb[(size_t)j * d + k] = qb[(size_t)j * 3 * d + 2 * d + k];
        }
      for (int j = 0; j < cl; ++j) /* causal: column j sees columns 0..j */
        attention(qb + (size_t)j * 3 * d, Kb, Vb, valid + (size_t)b * C, j + 1, H, dh, ob + (size_t)j * d, sc);
      linear(w->wo[l], w->bo[l], ob, cl, d, d, tb);
      for (size_t k = 0; k < (size_t)cl * d; ++k) hb[k] += tb[k];
      for (int j = 0; j < cl; ++j) layernorm(hb + (size_t)j * d, w->ln2_g[l], w->ln2_b[l], d, ab + (size_t)j * d);
      linear(w->w1[l], w->b1[l], ab, cl, d, f, ub);
      for (size_t k = 0; k < (size_t)cl * f; ++k) ub[k] = ub[k] > 0 ? ub[k] : 0;
      linear(w->w2[l], w->b2[l], ub, cl, f, d, tb);
      for (size_t k = 0; k < (size_t)cl * d; ++k) hb[k] += tb[k];
    }
  }
  for (int b = 0; b < B; ++b) {
    layernorm(h + ((size_t)b * C + (C - 1)) * d, w->lnf_g, w->lnf_b, d, a1);
    linear(w->lm_head ? w->lm_head : w->tok_emb, NULL, a1, 1, d, V, z);
    for (int v = 0; v < V; ++v) logits[(size_t)b * V + v] = (double)z[v];
  }
done:
  free(h); free(a1); free(qkv); free(Kc); free(Vc); free(o); free(t1); free(u); free(sc); free(z); free(valid);
  return rc;
}

/* ------------------------------------------------------------------ */
/* Single operations with double I/O (per-kernel checks)               */
/* ------------------------------------------------------------------ */

int ora_op_layernorm(const double *x, const float *g, const float *b, int32_t rows, int32_t d, double *out) {
  if (!x || !g || !b || !out) return ORA_ERR_NULL;
  real *xi = (real *)malloc(sizeof(real) * d), *oo = (real *)malloc(sizeof(real) * d);
  if (!xi || !oo) { free(xi); free(oo); return ORA_ERR_NOMEM; }
  for (int r = 0; r < rows; ++r) {
    for (int k = 0; k < d; ++k) xi[k] = (real)x[(size_t)r * d + k];
    layernorm(xi, g, b, d, oo);
    for (int k = 0; k < d; ++k) out[(size_t)r * d + k] = (double)oo[k];
  }
  free(xi); free(oo);
  return ORA_OK;
}

int ora_op_linear(const float *W, const float *bias, const double *in, int32_t rows, int32_t K, int32_t N,
                  double *out) {
  if (!W || !in || !out) return ORA_ERR_NULL;
  real *ii = (real *)malloc(sizeof(real) * (size_t)rows * K), *oo = (real *)malloc(sizeof(real) * (size_t)rows * N);
  if (!ii || !oo) { free(ii); free(oo); return ORA_ERR_NOMEM; }
  for (size_t k = 0; k < (size_t)rows * K; ++k) ii[k] = (real)in[k];
  linear(W, bias, ii, rows, K, N, oo);
  for (size_t k = 0; k < (size_t)rows * N; ++k) out[k] = (double)oo[k];
  free(ii); free(oo);
  return ORA_OK;
}

/* q [d]; Kc, Vc [len][d]; valid [len] (NULL = all) -> out [d] */
int ora_op_attention(const double *q, const double *Kc, const double *Vc, const uint8_t *valid, int32_t len,
                     int32_t H, int32_t dh, double *out) {
  if (!q || !Kc || !Vc || !out) return ORA_ERR_NULL;
  if (len < 0 || H < 1 || dh < 1) return ORA_ERR_SHAPE;
  int d = H * dh;
  real *qq = (real *)malloc(sizeof(real) * d), *kk = (real *)malloc(sizeof(real) * ((size_t)len * d + 1));
  real *vv = (real *)malloc(sizeof(real) * ((size_t)len * d + 1)), *oo = (real *)malloc(sizeof(real) * d);
  real *sc = (real *)malloc(sizeof(real) * (len + 1));
  uint8_t *va = (uint8_t *)malloc(len + 1);
  int rc = ORA_OK;
  if (!qq || !kk || !vv || !oo || !sc || !va) { rc = ORA_ERR_NOMEM; goto done; }
  for (int k = 0; k < d; ++k) qq[k] = (real)q[k];
  for (size_t k = 0; k < (size_t)len * d; ++k) { kk[k] = (real)Kc[k]; vv[k] = (real)Vc[k]; }
  for (int j = 0; j < len; ++j) va[j] = valid ? valid[j] : 1;
  attention(qq, kk, vv, va, len, H, dh, oo, sc);
  for (int k = 0; k < d; ++k) out[k] = (double)oo[k];
done:
  free(qq); free(kk); free(vv); free(oo); free(sc); free(va);
  return rc;
}

/* ------------------------------------------------------------------ */
/* Sampling head (the paper's generation setting, Section 3.2)         */
/* ------------------------------------------------------------------ */

static int cmp_desc(const void *a, const void *b) {
  const double x = *(const double *)a, y = *(const double *)b;
  return (x < y) - (x > y);
}

/* Temperature + nucleus (top-p) sampling of one token from logits[V] with one
 * uniform number u in [0,1):
 *   p_i = exp((z_i - max z) / temperature),  Z = sum p_i;
 *   tau = the largest probability value such that the mass of {p_i >= tau} is at
 *         least top_p * Z  (the smallest set of most likely tokens reaching
 *         top_p, tokens tied with the last one included);
 *   the token is the first index i (ascending) of that set whose running mass
 *   over the set exceeds u * (mass of the set).
 * margins[0] = distance of top_p * Z from the two candidate masses around the
 * boundary (relative to Z), margins[1] = distance of u * mass from the nearest
 * running-sum boundary (relative to the mass): a checker in lower precision can
 * only be expected to agree when both are well above its rounding error. */
int ora_op_sample(const double *logits, int32_t V, double temperature, double top_p, double u, double *margins) {
  if (!logits) return ORA_ERR_NULL;
  if (V < 1 || !(temperature > 0) || !(top_p > 0) || top_p > 1 || u < 0 || u >= 1) return ORA_ERR_RANGE;
  double *p = (double *)malloc(sizeof(double) * V), *srt = (double *)malloc(sizeof(double) * V);
  if (!p || !srt) { free(p); free(srt); return ORA_ERR_NOMEM; }
  double mx = logits[0];
  for (int i = 1; i < V; ++i) if (logits[i] > mx) mx = logits[i];
  double Z = 0;
  for (int i = 0; i < V; ++i) { p[i] = exp((logits[i] - mx) / temperature); Z += p[i]; srt[i] = p[i]; }
  qsort(srt, V, sizeof(double), cmp_desc);
  const double target = top_p * Z;
  double cum = 0, tau = srt[V - 1], before = 0;
  for (int i = 0; i < V; ++i) {
    cum += srt[i];
    if (cum >= target) { tau = srt[i]; break; }
  }
  double mass = 0, above = 0;
  for (int i = 0; i < V; ++i) { if (p[i] >= tau) mass += p[i]; if (p[i] > tau) above += p[i]; }
  before = above; /* mass of the strictly larger values: must be below the target */
  const double goal = u * mass;
  double run = 0, m1 = 1e300;
  int tok = -1;
  for (int i = 0; i < V; ++i) {
    if (p[i] < tau) continue;
    if (tok < 0 && run + p[i] > goal) tok = i;
    run += p[i];
    if (fabs(run - goal) < m1) m1 = fabs(run - goal);
  }
  if (tok < 0)
    for (int i = V - 1; i >= 0; --i) if (p[i] >= tau) { tok = i; break; }
  if (margins) {
    double a = fabs(mass - target), b = fabs(target - before);
    margins[0] = top_p >= 1.0 ? 1.0 : (a < b ? a : b) / Z; /* top_p = 1: everything is in, nothing to decide */
    margins[1] = m1 / mass;
  }
  free(p); free(srt);
  return tok;
}
