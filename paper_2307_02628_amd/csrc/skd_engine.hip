// Host engine behind the C ABI of include/skd.h: configuration checks, weight
// upload, the layer-sparse paged KV cache and the skip-aware layer loop that
// launches kernels for the active layers only (Sections 2.1-2.4).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/skd.h"
#include "skd_kernels.h"

using namespace skd;

static thread_local int g_last_hip = 0;
extern "C" int skd_last_hip_error(void) { return g_last_hip; }

#define HIPCHECK(expr)                         \
  do {                                         \
    hipError_t e_ = (expr);                    \
    if (e_ != hipSuccess) {                    \
      g_last_hip = (int)e_;                    \
      return e_ == hipErrorOutOfMemory ? SKD_ERR_NOMEM : SKD_ERR_HIP; \
    }                                          \
  } while (0)
#define SKDCHECK(expr)       \
  do {                       \
    int r_ = (expr);         \
    if (r_ < 0) return r_;   \
  } while (0)

// Scratch of skd_logits_argmax_noalloc: the per-workgroup (max, argmax) partials of the LM head, fp32 maxima in
// the first half and int32 indices in the second.  Every GPU the library runs on holds its own copy of this
// array at its own address until the process ends.  In host code the name below is only a handle for
// hipGetSymbolAddress; kernels are given the resolved device address.
#define SKD_NOALLOC_MAX_PARTIALS (1 << 18) /* workgroups of the LM head x padded batch rows */
static __device__ __align__(256) unsigned char scratch[2 * 4 * SKD_NOALLOC_MAX_PARTIALS];  // 2 MiB

namespace {

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each device, resolved once per device

// Called with `device` current (skd_create): looks the array's address up on that device.
int resolve_scratch(int device) {
  if (device < 0 || device >= kMaxDevices) return SKD_ERR_RANGE;
  if (g_scratch_ptr[device]) return SKD_OK;
  void *ptr = nullptr;
  HIPCHECK(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)));
  if (!ptr) return SKD_ERR_HIP;
  g_scratch_ptr[device] = ptr;
  return SKD_OK;
}

struct LayerW {
  // matrices: fp32 row-major (debug path) or bf16 fragment-major (production path)
  void *wqkv = nullptr, *wo = nullptr, *w1 = nullptr, *w2 = nullptr;
  float *ln1_g = nullptr, *ln1_b = nullptr, *bqkv = nullptr, *bo = nullptr;
  float *ln2_g = nullptr, *ln2_b = nullptr, *b1 = nullptr, *b2 = nullptr;
};

struct GemmPlan {
  int R = 1, split = 1, U = 1, waves = 8;
  bool ws = false;  // 128 batch rows: the wave-specialised kernel (weight-streaming waves + activation-loading waves)
  int ws_rot = 0;   // workgroups start their K range at different stages
};

}  // namespace

namespace skd {
thread_local LaunchTimer *g_launch_timer = nullptr;
}

// hands the launches of one kernel class their event pairs (skd_profile_enable mode 1)
struct StateTimer final : LaunchTimer {
  skd_state *st = nullptr;
  int cls = 0;
  void next(hipEvent_t *start, hipEvent_t *stop) override;
};

struct skd_state {
  skd_config cfg{};
  hipStream_t stream = nullptr;
  int B_pad = 0, dh = 0;
  bool bf16 = true;
  std::vector<void *> allocs;
  // weights
  std::vector<LayerW> lw;
  void *tok_emb = nullptr;  // row-major (gather)
  void *pos_emb = nullptr;  // row-major
  void *head = nullptr;     // LM head: fp32 row-major or bf16 fragment-major
  float *lnf_g = nullptr, *lnf_b = nullptr;
  // KV cache
  KvGeom geom{};
  void *pool = nullptr;
  int32_t *bt_dev = nullptr;       // [L][B][max_pages]
  std::vector<int32_t> bt_host;
  std::vector<int> kv_len, kv_cap; // columns held / columns reserved, per layer
  int64_t pages_reserved = 0, pages_dense = 0;
  // per-step device buffers
  int32_t *tok_dev = nullptr;      // [B] input column
  int32_t *prompt_dev = nullptr;   // [P][B]
  int32_t *order_dev = nullptr;    // [B] rows by descending real length (attention dispatch order)
  bool ragged = false;             // rows differ in length: use order_dev
  int32_t *start_dev = nullptr;    // [B] first real column
  std::vector<int32_t> start_host;
  int32_t *argmax_dev = nullptr;   // [B]
  float *u_dev = nullptr;          // [B] uniform numbers of the sampling head
  float *x = nullptr;              // residual stream fp32 [B_pad][d]
  void *a = nullptr;               // LayerNorm output
  void *q = nullptr;               // bf16: q [B_pad][d]; fp32: qkv [B][3d]
  void *o = nullptr;               // attention output
  void *u = nullptr;               // FFN hidden
  float *partial = nullptr;        // bf16: split-K partials
  bf16_t *kv_new = nullptr;        // bf16: k and v of the column being processed, [B][k | v][d]
  float *attn_part = nullptr;      // bf16: split-KV partials; fp32: score scratch
  float *logits_dev = nullptr;     // [B][V] (fp32 path always; bf16 path when asked)
  float *pmax = nullptr;
  int32_t *pidx = nullptr;
  // plans (bf16)
  GemmPlan p_qkv, p_out, p_ffn1, p_ffn2, p_head;
  int max_split = 1, attn_splits = 1, attn_waves = 4;
  // batched prompt workspace (allocated by the first batched skd_prefill)
  float *pf_x = nullptr;
  bf16_t *pf_a = nullptr, *pf_q = nullptr, *pf_o = nullptr, *pf_u = nullptr;
  int32_t *pf_seq = nullptr, *pf_first = nullptr;  // row map of the prompt pass (sequence of each row, first row of each sequence)
  int prefill_mode = 1;            // 1 = whole prompt per layer (bf16 path), 0 = column by column
  int prefill_tiles = 1;           // 1 = prompt projections on 256 x 256 tiles where the shape allows
  int device = 0;                  // HIP device the state lives on
  // sequencing
  bool prefilled = false, have_hidden = false, have_argmax = false;
  int steps_done = 0;
  std::vector<int32_t> layers_tmp;
  std::vector<int32_t> n_table;    // caller-supplied layer counts per position (empty = the linear schedule)
  // per-kernel timing (off by default): 1 = each kernel's own begin/end time stamps, 2 = event brackets
  int profiling = 0;
  StateTimer timer;
  struct ProfRec { int cls; hipEvent_t a, b; };
  std::vector<ProfRec> prof_pending;
  std::vector<hipEvent_t> prof_free;
  double prof_ms[SKD_PROF_CLASSES] = {};
  int64_t prof_n[SKD_PROF_CLASSES] = {};
};

namespace {

template <typename T>
int dev_alloc(skd_state *st, T **out, size_t count) {
  void *p = nullptr;
  HIPCHECK(hipMalloc(&p, std::max<size_t>(count * sizeof(T), 256)));
  st->allocs.push_back(p);
  *out = (T *)p;
  return SKD_OK;
}

int env_int(const char *name, int dflt) {
  const char *v = getenv(name);
  return v && *v ? atoi(v) : dflt;
}

int check_config(const skd_config &c) {
  if (c.L < 1 || c.d_model < 1 || c.n_heads < 1 || c.ffn < 1 || c.vocab < 1 || c.max_pos < 1) return SKD_ERR_SHAPE;
  if (c.d_model % c.n_heads) return SKD_ERR_SHAPE;
  if (c.batch < 1 || c.prompt_size < 1 || c.sequence_length <= c.prompt_size) return SKD_ERR_SHAPE;
  if (c.max_pos < c.sequence_length) return SKD_ERR_SHAPE;
  if (c.n_min < 1 || c.n_min > c.n_max || c.n_max > c.L) return SKD_ERR_SHAPE;
  if (c.warmup < 0 || c.warmup > c.n_min) return SKD_ERR_SHAPE;
  if (c.page_tokens < 0 || c.page_tokens % 32) return SKD_ERR_SHAPE;
  if (c.dtype != SKD_BF16 && c.dtype != SKD_FP32) return SKD_ERR_SHAPE;
  if (c.io_on_device != 0 && c.io_on_device != 1) return SKD_ERR_SHAPE;
  if (c.dtype == SKD_BF16) {
    const int dh = c.d_model / c.n_heads;
    if (dh != 64 && dh != 128) return SKD_ERR_SHAPE;
    if (c.d_model % 32 || c.ffn % 32 || c.d_model > 16384) return SKD_ERR_SHAPE;
    if (c.batch > 128) return SKD_ERR_SHAPE;
  }
  return SKD_OK;
}

// Upload one tensor (host or device, fp32 or bf16) into a device staging area.
int stage(skd_state *st, const skd_weights &w, const void *src, size_t n, void *staging, const void **dev_src) {
  if (!src) return SKD_ERR_NULL;
  if (w.location == SKD_DEVICE) {
    *dev_src = src;
    return SKD_OK;
  }
  const size_t bytes = n * (w.elem == SKD_W_BF16 ? 2 : 4);
  HIPCHECK(hipMemcpyAsync(staging, src, bytes, hipMemcpyHostToDevice, st->stream));
  HIPCHECK(hipStreamSynchronize(st->stream));  // the staging area is reused by the next tensor
  *dev_src = staging;
  return SKD_OK;
}

int upload_vec(skd_state *st, const skd_weights &w, const void *src, size_t n, void *staging, float **out) {
  const void *dsrc = nullptr;
  SKDCHECK(stage(st, w, src, n, staging, &dsrc));
  SKDCHECK(dev_alloc(st, out, n));
  prep_to_f32(st->stream, dsrc, w.elem == SKD_W_BF16, *out, (long)n);
  HIPCHECK(hipStreamSynchronize(st->stream));
  return SKD_OK;
}

// matrix [N][K]: fp32 path -> fp32 row-major; bf16 path -> fragment-major (frag > 0) or row-major bf16
// (frag = tile-group size of the fragment-major layout, 0 = row-major)
int upload_mat(skd_state *st, const skd_weights &w, const void *src, long N, long K, void *staging, int frag,
               void **out) {
  const void *dsrc = nullptr;
  SKDCHECK(stage(st, w, src, (size_t)N * K, staging, &dsrc));
  if (!st->bf16) {
    float *p = nullptr;
    SKDCHECK(dev_alloc(st, &p, (size_t)N * K));
    prep_to_f32(st->stream, dsrc, w.elem == SKD_W_BF16, p, N * K);
    *out = p;
  } else if (frag) {
    const long N_pad = (N + 191) / 192 * 192;  // whole groups of 1..4 tiles: no wave tile ever leaves the buffer
    bf16_t *p = nullptr;
    SKDCHECK(dev_alloc(st, &p, (size_t)N_pad * K));
    prep_matrix_frag(st->stream, dsrc, w.elem == SKD_W_BF16, p, N, K, N_pad, frag);
    *out = p;
  } else {
    bf16_t *p = nullptr;
    SKDCHECK(dev_alloc(st, &p, (size_t)N * K));
    prep_matrix_rm_bf16(st->stream, dsrc, w.elem == SKD_W_BF16, p, N * K);
    *out = p;
  }
  HIPCHECK(hipStreamSynchronize(st->stream));
  return SKD_OK;
}

// Launch shapes.  Measured on MI355X at the OPT-6.7B widths: up to batch 64, 8
// waves per workgroup interleaving k-steps with 48-64 weight rows per workgroup
// and one k-step per register buffer stream best; at batch 128 the 4 x 8 tile
// accumulators need the whole register file, so workgroups have 4 waves.
// Every CU should get a workgroup; when K is split across workgroups a wave
// should still see at least 2 k-steps.
int plan_waves(int B_pad) { return B_pad >= 128 ? 4 : 8; }
GemmPlan plan_direct(int N, int B_pad) {  // whole K inside the workgroup
  GemmPlan p;
  p.waves = plan_waves(B_pad);
  p.split = 1;
  // several rounds of workgroups (the LM head): tile rows that keep the activation re-reads at half the weight
  // stream; with one batch tile, 2 rows do that and leave twice the workgroups to even out the last round
  p.R = B_pad >= 32 ? 4 : 2;
  if (bf16_gemm_groups(N, p.R) >= 512) return p;
  // one or two rounds: the R that keeps the largest share of the 256 CUs busy over whole rounds; ties go to the
  // larger R (measured: 768 tiles -> R = 3, 256 workgroups; 384 tiles -> R = 2, 192 workgroups beats 384)
  double best = -1.0;
  for (int R = 1; R <= 4; ++R) {
    const int g = bf16_gemm_groups(N, R);
    const double e = (double)g / (256.0 * ((g + 255) / 256));
    if (e >= best) { best = e; p.R = R; }
  }
  return p;
}
GemmPlan plan_split(int N, int K, int B_pad) {  // partial sums, reduced by the LayerNorm kernel
  GemmPlan p;
  p.waves = plan_waves(B_pad);
  const int Kf = K / 32;
  // tile rows per workgroup: enough that the activation re-reads (B_pad / (16 R) of the weight bytes) stay at
  // half the weight stream; more rows than that only force a deeper split, whose partials the reducer pays for
  p.R = B_pad >= 32 ? 4 : 2;
  while (p.R > 1 && N % (16 * p.R)) --p.R;
  for (;;) {
    int S = 1;
    while (S < 16 && bf16_gemm_groups(N, p.R) * S < 256 && Kf % (2 * S) == 0 && Kf / (2 * S) >= 2 * p.waves) S *= 2;
    p.split = S;
    if (bf16_gemm_groups(N, p.R) * S >= 256 || p.R == 1) break;
    --p.R;
    while (p.R > 1 && N % (16 * p.R)) --p.R;
  }
  return p;
}

// Active layers at position t for this state: the linear schedule of the
// configuration, or the caller's table (same shape of the set: warm-up layers
// at the bottom, the rest of the budget at the top).
int state_active_layers(const skd_state *st, int t, int32_t *out) {
  const skd_config &c = st->cfg;
  if (st->n_table.empty()) return skd_active_layers(t, &c, out);
  if (t < 0 || t >= c.sequence_length) return SKD_ERR_RANGE;
  const int n = st->n_table[t];
  int k = 0;
  for (int l = 0; l < c.warmup; ++l) out[k++] = l;
  for (int l = c.L - (n - c.warmup); l < c.L; ++l) out[k++] = l;
  return k;
}

int build_kv(skd_state *st) {
  const skd_config &c = st->cfg;
  const int pt = c.page_tokens ? c.page_tokens : 64;
  KvGeom &g = st->geom;
  g.page_tokens = pt;
  g.max_pages = (c.sequence_length + pt - 1) / pt;
  g.H = c.n_heads;
  g.dh = st->dh;
  g.page_elems = 2L * pt * c.d_model;
  // Static policy: the columns at which each layer runs are known before
  // generation starts, so each layer reserves exactly what it will hold.
  st->kv_cap.assign(c.L, 0);
  std::vector<int32_t> act(c.L);
  for (int t = 0; t < c.sequence_length; ++t) {
    const int n = state_active_layers(st, t, act.data());
    if (n < 0) return n;
    for (int i = 0; i < n; ++i) {
      if (st->kv_cap[act[i]] != t) return SKD_ERR_SCHEDULE;  // a layer re-entered: its cache would have a hole
      st->kv_cap[act[i]] = t + 1;
    }
  }
  st->bt_host.assign((size_t)c.L * c.batch * g.max_pages, -1);
  int64_t next = 0;
  // Page order inside a layer is position-major (all rows' page 0, then all
  // rows' page 1, ...): the B*H workgroups of the attention kernel advance
  // through their keys in step, so at any moment the chip reads one dense
  // B-MiB-scale window instead of B windows a fixed large stride apart
  // (measured: up to 13 % faster attention when a row holds 12 pages).
  for (int l = 0; l < c.L; ++l) {
    const int np = (st->kv_cap[l] + pt - 1) / pt;
    for (int p = 0; p < np; ++p)
      for (int b = 0; b < c.batch; ++b) st->bt_host[((size_t)l * c.batch + b) * g.max_pages + p] = (int32_t)next++;
  }
  if (next > 0x7fffffffLL) return SKD_ERR_NOMEM;
  st->pages_reserved = next;
  st->pages_dense = (int64_t)c.L * c.batch * g.max_pages;
  const size_t esz = st->bf16 ? 2 : 4;
  const size_t bytes = (size_t)next * g.page_elems * esz;
  void *pool = nullptr;
  HIPCHECK(hipMalloc(&pool, std::max<size_t>(bytes, 256)));
  st->allocs.push_back(pool);
  st->pool = pool;
  // unwritten slots must hold finite values: a masked key still meets its V in the MFMA
  HIPCHECK(hipMemsetAsync(pool, 0, bytes, st->stream));
  SKDCHECK(dev_alloc(st, &st->bt_dev, st->bt_host.size()));
  HIPCHECK(hipMemcpyAsync(st->bt_dev, st->bt_host.data(), st->bt_host.size() * sizeof(int32_t), hipMemcpyHostToDevice,
                          st->stream));
  HIPCHECK(hipStreamSynchronize(st->stream));
  st->kv_len.assign(c.L, 0);
  return SKD_OK;
}

hipEvent_t prof_event(skd_state *st) {
  if (!st->prof_free.empty()) {
    hipEvent_t e = st->prof_free.back();
    st->prof_free.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  (void)hipEventCreate(&e);
  return e;
}
// Times the launches issued inside its scope when profiling is on: mode 1 gives every launch its own event
// pair, stamped with the kernel's begin and end; mode 2 records one event before and one after the launches.
struct ProfScope {
  skd_state *st;
  int cls;
  hipEvent_t a = nullptr;
  ProfScope(skd_state *s, int c) : st(s), cls(c) {
    if (st->profiling == 1) {
      st->timer.st = st;
      st->timer.cls = cls;
      skd::g_launch_timer = &st->timer;
    } else if (st->profiling == 2) {
      a = prof_event(st);
      if (a) (void)hipEventRecord(a, st->stream);
    }
  }
  ~ProfScope() {
    skd::g_launch_timer = nullptr;
    if (a) {
      hipEvent_t b = prof_event(st);
      if (b) (void)hipEventRecord(b, st->stream);
      st->prof_pending.push_back({cls, a, b});
    }
  }
};
}  // namespace
void StateTimer::next(hipEvent_t *start, hipEvent_t *stop) {
  *start = prof_event(st);
  *stop = prof_event(st);
  st->prof_pending.push_back({cls, *start, *stop});
}
namespace {
int prof_drain(skd_state *st) {
  HIPCHECK(hipStreamSynchronize(st->stream));
  for (auto &r : st->prof_pending) {
    float ms = 0.f;
    if (r.a && r.b && hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) {
      st->prof_ms[r.cls] += ms;
      st->prof_n[r.cls] += 1;
    }
    if (r.a) st->prof_free.push_back(r.a);
    if (r.b) st->prof_free.push_back(r.b);
  }
  st->prof_pending.clear();
  return SKD_OK;
}

const int32_t *bt_layer(const skd_state *st, int l) {
  return st->bt_dev + (size_t)l * st->cfg.batch * st->geom.max_pages;
}

// a decode projection on the kernel its plan names; returns the row groups launched or -1
int launch_gemm(hipStream_t s, GemmArgs &ga, int epi, const GemmPlan &p) {
  ga.ws_rot = p.ws_rot;
  return p.ws ? bf16_gemm_ws(s, ga, epi, p.R) : bf16_gemm(s, ga, epi, p.R, p.U, p.waves);
}
int check_gemm(const GemmArgs &ga, int epi, const GemmPlan &p) {
  return p.ws ? bf16_gemm_ws_check(ga, epi, p.R) : bf16_gemm_check(ga, epi, p.R, p.U, p.waves);
}

// The projections of a layer (the same shapes in every layer) and the LM head against what the kernels can launch.
bool decode_shapes_ok(const skd_state *st) {
  const skd_config &c = st->cfg;
  const int d = c.d_model, f = c.ffn;
  GemmArgs ga{};
  ga.B = c.batch; ga.B_pad = st->B_pad;
  auto ok = [&](int N, int K, const GemmPlan &p, int epi) {
    ga.N = N; ga.K = K; ga.G = p.R; ga.split = p.split;
    return check_gemm(ga, epi, p) > 0;
  };
  return ok(3 * d, d, st->p_qkv, EPI_QKV) && ok(d, d, st->p_out, EPI_PARTIAL) && ok(f, d, st->p_ffn1, EPI_RELU) &&
         ok(d, f, st->p_ffn2, EPI_PARTIAL) && ok(c.vocab, d, st->p_head, EPI_LOGITS);
}

// One column (all B rows at position t) through the given ascending layer list.  Everything that can refuse
// the column (layer list, cache lengths, launch shapes) is checked before the first launch, so an error leaves
// the caches as they were.
int run_column(skd_state *st, int t, const int32_t *tokens_dev, const int32_t *layers, int n) {
  const skd_config &c = st->cfg;
  const int B = c.batch, d = c.d_model, f = c.ffn;
  hipStream_t s = st->stream;
  for (int i = 0; i < n; ++i) {
    const int l = layers[i];
    if (l < 0 || l >= c.L || (i && layers[i - 1] >= l)) return SKD_ERR_SCHEDULE;
    if (st->kv_len[l] != t) return SKD_ERR_ORDER;  // every earlier key of an active layer must exist
    if (t >= st->kv_cap[l]) return SKD_ERR_NOMEM;
  }
  if (st->bf16 && !decode_shapes_ok(st)) return SKD_ERR_SHAPE;  // before the first launch: nothing is half done
  if (!st->bf16) {
    float *a = (float *)st->a, *qkv = (float *)st->q, *o = (float *)st->o, *u = (float *)st->u;
    { ProfScope ps_(st, SKD_PROF_OTHER); f32_embed(s, st->x, (const float *)st->tok_emb, (const float *)st->pos_emb, tokens_dev, st->start_dev, t, B, d, c.vocab); }
    for (int i = 0; i < n; ++i) {
      const LayerW &w = st->lw[layers[i]];
      { ProfScope ps_(st, SKD_PROF_OTHER); f32_layernorm(s, st->x, w.ln1_g, w.ln1_b, a, B, d); }
      { ProfScope ps_(st, SKD_PROF_OTHER); f32_linear(s, (const float *)w.wqkv, w.bqkv, a, qkv, B, d, 3 * d, 0, 0); }
      { ProfScope ps_(st, SKD_PROF_OTHER); f32_kv_write(s, qkv, (float *)st->pool, bt_layer(st, layers[i]), t, B, st->geom); }
      { ProfScope ps_(st, SKD_PROF_OTHER); f32_attention(s, qkv, (const float *)st->pool, bt_layer(st, layers[i]), st->start_dev, t, o, st->attn_part, c.sequence_length, B, st->geom); }
      { ProfScope ps_(st, SKD_PROF_OTHER); f32_linear(s, (const float *)w.wo, w.bo, o, st->x, B, d, d, 0, 1); }
      { ProfScope ps_(st, SKD_PROF_OTHER); f32_layernorm(s, st->x, w.ln2_g, w.ln2_b, a, B, d); }
      { ProfScope ps_(st, SKD_PROF_OTHER); f32_linear(s, (const float *)w.w1, w.b1, a, u, B, d, f, 1, 0); }
      { ProfScope ps_(st, SKD_PROF_OTHER); f32_linear(s, (const float *)w.w2, w.b2, u, st->x, B, f, d, 0, 1); }
      st->kv_len[layers[i]] = t + 1;
    }
  } else {
    bf16_t *a = (bf16_t *)st->a, *q = (bf16_t *)st->q, *o = (bf16_t *)st->o, *u = (bf16_t *)st->u;
    const LayerW &w0 = st->lw[layers[0]];
    { ProfScope ps_(st, SKD_PROF_EMBED_LN); bf16_embed_ln(s, tokens_dev, st->start_dev, t, (const bf16_t *)st->tok_emb, (const bf16_t *)st->pos_emb, w0.ln1_g, w0.ln1_b, st->x, a, B, d, c.vocab); }
    int grc = 0;
    for (int i = 0; i < n; ++i) {
      const int l = layers[i];
      const LayerW &w = st->lw[l];
      GemmArgs ga{};
      ga.B = B; ga.B_pad = st->B_pad; ga.kv = st->geom; ga.d = d;
      // q, k, v projection; the attention kernel files k and v into this layer's page slot for column t
      ga.W = (const bf16_t *)w.wqkv; ga.G = st->p_qkv.R; ga.A = a; ga.bias = w.bqkv; ga.N = 3 * d; ga.K = d; ga.split = 1;
      ga.q_out = q; ga.kv_new = st->kv_new;
      { ProfScope ps_(st, SKD_PROF_GEMM_QKV); grc = launch_gemm(s, ga, EPI_QKV, st->p_qkv); }
      if (grc < 0) return SKD_ERR_SHAPE;
      AttnArgs aa{};
      aa.q = q; aa.kv_new = st->kv_new; aa.pool = (bf16_t *)st->pool; aa.bt_layer = bt_layer(st, l); aa.start = st->start_dev; aa.order = st->ragged ? st->order_dev : nullptr;
      aa.t = t; aa.B = B; aa.splits = st->attn_splits; aa.waves = st->attn_waves; aa.kv = st->geom; aa.o = o; aa.part = st->attn_part;
      { ProfScope ps_(st, SKD_PROF_ATTENTION); bf16_attention(s, aa); }
      // output projection -> partials; bias + residual + LayerNorm 2 in the reducer
      ga.W = (const bf16_t *)w.wo; ga.G = st->p_out.R; ga.A = o; ga.N = d; ga.K = d; ga.split = st->p_out.split; ga.partial = st->partial;
      { ProfScope ps_(st, SKD_PROF_GEMM_OUT); grc = launch_gemm(s, ga, EPI_PARTIAL, st->p_out); }
      if (grc < 0) return SKD_ERR_SHAPE;
      { ProfScope ps_(st, SKD_PROF_REDUCE_LN); bf16_reduce_ln(s, st->partial, st->p_out.split, st->B_pad, w.bo, st->x, w.ln2_g, w.ln2_b, a, B, d); }
      ga.W = (const bf16_t *)w.w1; ga.G = st->p_ffn1.R; ga.A = a; ga.bias = w.b1; ga.N = f; ga.K = d; ga.split = 1; ga.act_out = u;
      { ProfScope ps_(st, SKD_PROF_GEMM_FFN1); grc = launch_gemm(s, ga, EPI_RELU, st->p_ffn1); }
      if (grc < 0) return SKD_ERR_SHAPE;
      ga.W = (const bf16_t *)w.w2; ga.G = st->p_ffn2.R; ga.A = u; ga.N = d; ga.K = f; ga.split = st->p_ffn2.split;
      { ProfScope ps_(st, SKD_PROF_GEMM_FFN2); grc = launch_gemm(s, ga, EPI_PARTIAL, st->p_ffn2); }
      if (grc < 0) return SKD_ERR_SHAPE;
      // the reducer of the last sub-block already applies the next LayerNorm:
      // LayerNorm 1 of the next ACTIVE layer, or the final LayerNorm
      const float *ng = (i + 1 < n) ? st->lw[layers[i + 1]].ln1_g : st->lnf_g;
      const float *nb = (i + 1 < n) ? st->lw[layers[i + 1]].ln1_b : st->lnf_b;
      { ProfScope ps_(st, SKD_PROF_REDUCE_LN); bf16_reduce_ln(s, st->partial, st->p_ffn2.split, st->B_pad, w.b2, st->x, ng, nb, a, B, d); }
      st->kv_len[l] = t + 1;
    }
  }
  HIPCHECK(hipGetLastError());
  st->have_hidden = true;
  st->have_argmax = false;
  return SKD_OK;
}

}  // namespace

static int create_impl(const skd_config *cfg, const skd_weights *w, void *hip_stream, const int32_t *n_table,
                       skd_state **out) {
  if (!cfg || !w || !out) return SKD_ERR_NULL;
  *out = nullptr;
  SKDCHECK(check_config(*cfg));
  if (n_table) {  // monotone, within [max(1, warmup), L]
    for (int i = 0; i < cfg->sequence_length; ++i) {
      if (n_table[i] < 1 || n_table[i] > cfg->L) return SKD_ERR_RANGE;
      if (n_table[i] < cfg->warmup) return SKD_ERR_SHAPE;
      if (i && n_table[i] > n_table[i - 1]) return SKD_ERR_SCHEDULE;
    }
  }
  if ((w->location != SKD_HOST && w->location != SKD_DEVICE) || (w->elem != SKD_W_FP32 && w->elem != SKD_W_BF16))
    return SKD_ERR_SHAPE;
  if (!w->tok_emb || !w->pos_emb || !w->lnf_g || !w->lnf_b || !w->ln1_g || !w->ln1_b || !w->wqkv || !w->bqkv ||
      !w->wo || !w->bo || !w->ln2_g || !w->ln2_b || !w->w1 || !w->b1 || !w->w2 || !w->b2)
    return SKD_ERR_NULL;
  skd_state *st = new (std::nothrow) skd_state();
  if (!st) return SKD_ERR_NOMEM;
  auto fail = [&](int rc) {
    skd_destroy(st);
    return rc;
  };
  st->cfg = *cfg;
  if (n_table) st->n_table.assign(n_table, n_table + cfg->sequence_length);
  if (!st->cfg.page_tokens) st->cfg.page_tokens = 64;
  st->stream = (hipStream_t)hip_stream;
  st->bf16 = cfg->dtype == SKD_BF16;
  st->dh = cfg->d_model / cfg->n_heads;
  const skd_config &c = st->cfg;
  const int B = c.batch, d = c.d_model, f = c.ffn, V = c.vocab, L = c.L;
  st->B_pad = 16;
  while (st->B_pad < B) st->B_pad *= 2;
  st->layers_tmp.resize(L);

  // ---- launch shapes (the weight layout below depends on them)
  auto ov = [&](const char *name, int &v, int lo, int hi) { const int e = env_int(name, 0); if (e >= lo && e <= hi) v = e; };
  if (st->bf16) {
    const int Bp = st->B_pad;
    st->p_qkv = plan_direct(3 * d, Bp);
    st->p_ffn1 = plan_direct(f, Bp);
    st->p_head = plan_direct(V, Bp);
    st->p_out = plan_split(d, d, Bp);
    st->p_ffn2 = plan_split(d, f, Bp);
    ov("SKD_R_QKV", st->p_qkv.R, 1, 4); ov("SKD_R_FFN1", st->p_ffn1.R, 1, 4); ov("SKD_R_HEAD", st->p_head.R, 1, 4);
    ov("SKD_R_OUT", st->p_out.R, 1, 4); ov("SKD_R_FFN2", st->p_ffn2.R, 1, 4);
    ov("SKD_S_OUT", st->p_out.split, 1, 32); ov("SKD_S_FFN2", st->p_ffn2.split, 1, 32);
    ov("SKD_U_QKV", st->p_qkv.U, 1, 4); ov("SKD_U_FFN1", st->p_ffn1.U, 1, 4); ov("SKD_U_HEAD", st->p_head.U, 1, 4);
    ov("SKD_U_OUT", st->p_out.U, 1, 4); ov("SKD_U_FFN2", st->p_ffn2.U, 1, 4);
    ov("SKD_W_QKV", st->p_qkv.waves, 4, 8); ov("SKD_W_FFN1", st->p_ffn1.waves, 4, 8); ov("SKD_W_HEAD", st->p_head.waves, 4, 8);
    ov("SKD_W_OUT", st->p_out.waves, 4, 8); ov("SKD_W_FFN2", st->p_ffn2.waves, 4, 8);
  }

  if (st->bf16 && st->B_pad == 128 && env_int("SKD_GEMM_WS", 1) != 0) {
    // 128 batch rows: every projection whose K range divides into stages of 4 k-steps per workgroup
    GemmArgs ga{};
    ga.B = B; ga.B_pad = st->B_pad;
    auto pick = [&](int N, int K, GemmPlan &p, int epi) {
      ga.N = N; ga.K = K; ga.G = p.R; ga.split = p.split;
      p.ws = bf16_gemm_ws_check(ga, epi, p.R) > 0;
      // rotated K start: pays while the XCD's L2 (4 MiB) holds the activation matrix beside the weight stream
      // (measured at 128 x 4096: FFN1 35.5 -> 33.7 us; at 128 x 16384, 4 MiB, FFN2 36.3 -> 38.8 us)
      // Not for the LM head: there every vocabulary row keeps the same summation order, so that identical rows give
      // identical logits at every batch size (ties are then broken by index, as documented), and it gains nothing.
      p.ws_rot = epi != EPI_LOGITS && (long)st->B_pad * K * 2 <= (2L << 20);
      const int e = env_int("SKD_WS_ROT", -1);
      if (e == 0 || (e == 1 && epi != EPI_LOGITS)) p.ws_rot = e;
    };
    pick(3 * d, d, st->p_qkv, EPI_QKV); pick(d, d, st->p_out, EPI_PARTIAL); pick(f, d, st->p_ffn1, EPI_RELU);
    pick(d, f, st->p_ffn2, EPI_PARTIAL); pick(V, d, st->p_head, EPI_LOGITS);
  }
  if (st->bf16 && !decode_shapes_ok(st)) return fail(SKD_ERR_SHAPE);  // an override the kernels cannot launch
  {  // the device this state lives on, and that device's copy of the static scratch array
    hipError_t e = hipGetDevice(&st->device);
    if (e != hipSuccess) { g_last_hip = (int)e; return fail(SKD_ERR_HIP); }
    const int src = resolve_scratch(st->device);
    if (src != SKD_OK) return fail(src);
  }

  // ---- weights
  const size_t esz = w->elem == SKD_W_BF16 ? 2 : 4;
  size_t biggest = std::max({(size_t)V * d, (size_t)c.max_pos * d, (size_t)3 * d * d, (size_t)f * d});
  void *staging = nullptr;
  if (w->location == SKD_HOST) {
    hipError_t e = hipMalloc(&staging, biggest * esz);
    if (e != hipSuccess) { g_last_hip = (int)e; return fail(SKD_ERR_NOMEM); }
  }
  int rc = SKD_OK;
  auto vec = [&](const void *src, size_t n, float **o) { if (rc == SKD_OK) rc = upload_vec(st, *w, src, n, staging, o); };
  auto mat = [&](const void *src, long N, long K, int frag, void **o) { if (rc == SKD_OK) rc = upload_mat(st, *w, src, N, K, staging, frag, o); };
  mat(w->tok_emb, V, d, 0, &st->tok_emb);
  mat(w->pos_emb, c.max_pos, d, 0, &st->pos_emb);
  if (st->bf16 || w->lm_head) mat(w->lm_head ? w->lm_head : w->tok_emb, V, d, st->bf16 ? st->p_head.R : 1, &st->head);
  else st->head = st->tok_emb;
  vec(w->lnf_g, d, &st->lnf_g);
  vec(w->lnf_b, d, &st->lnf_b);
  st->lw.resize(L);
  for (int l = 0; l < L && rc == SKD_OK; ++l) {
    LayerW &lw = st->lw[l];
    vec(w->ln1_g[l], d, &lw.ln1_g); vec(w->ln1_b[l], d, &lw.ln1_b);
    mat(w->wqkv[l], 3L * d, d, st->p_qkv.R, &lw.wqkv); vec(w->bqkv[l], 3 * (size_t)d, &lw.bqkv);
    mat(w->wo[l], d, d, st->p_out.R, &lw.wo); vec(w->bo[l], d, &lw.bo);
    vec(w->ln2_g[l], d, &lw.ln2_g); vec(w->ln2_b[l], d, &lw.ln2_b);
    mat(w->w1[l], f, d, st->p_ffn1.R, &lw.w1); vec(w->b1[l], f, &lw.b1);
    mat(w->w2[l], d, f, st->p_ffn2.R, &lw.w2); vec(w->b2[l], d, &lw.b2);
  }
  if (staging) (void)hipFree(staging);
  if (rc != SKD_OK) return fail(rc);

  // ---- KV cache
  rc = build_kv(st);
  if (rc != SKD_OK) return fail(rc);

  // ---- workspaces
  const int Bp = st->B_pad;
  auto A = [&](auto **p, size_t n) { if (rc == SKD_OK) rc = dev_alloc(st, p, n); };
  A(&st->tok_dev, B); A(&st->prompt_dev, (size_t)c.prompt_size * B); A(&st->start_dev, B); A(&st->order_dev, B); A(&st->argmax_dev, B); A(&st->u_dev, B);
  A(&st->x, (size_t)Bp * d);
  if (st->bf16) {
    st->prefill_mode = env_int("SKD_PREFILL_BATCHED", 1) != 0 ? 1 : 0;
    st->prefill_tiles = env_int("SKD_PREFILL_TILES", 1) != 0 ? 1 : 0;
    st->max_split = std::max(st->p_out.split, st->p_ffn2.split);
    // split the key range of one head over several workgroups only when rows*heads alone cannot fill the chip
    // decode attention wants 16 waves on every CU: few (row, head) pairs get wider workgroups first (merged in
    // LDS), then splits of the key range (merged by a second kernel)
    // (one wave per pair streams 4 % faster with the arithmetic removed, but not with it: measured 128.7 vs 127.2 us
    // at 128 rows x 32 heads, so the planner starts at two; SKD_ATTN_WAVES=1 forces it)
    int waves = 2, splits = 1;
    while (B * c.n_heads * waves < 4096 && waves < 16) waves *= 2;
    while (B * c.n_heads * waves * splits < 4096 && splits < 8) splits *= 2;
    ov("SKD_ATTN_WAVES", waves, 1, 16);
    ov("SKD_ATTN_SPLITS", splits, 1, 16);
    st->attn_waves = waves;
    st->attn_splits = splits;
    bf16_t *t16 = nullptr;
    A(&t16, (size_t)Bp * d); st->a = t16; if (rc == SKD_OK) rc = hipMemsetAsync(st->a, 0, (size_t)Bp * d * 2, st->stream) == hipSuccess ? SKD_OK : SKD_ERR_HIP;
    A(&t16, (size_t)Bp * d); st->q = t16;
    A(&t16, (size_t)Bp * d); st->o = t16; if (rc == SKD_OK) rc = hipMemsetAsync(st->o, 0, (size_t)Bp * d * 2, st->stream) == hipSuccess ? SKD_OK : SKD_ERR_HIP;
    A(&t16, (size_t)Bp * f); st->u = t16;
    A(&st->kv_new, (size_t)B * 2 * d);
    A(&st->partial, (size_t)st->max_split * Bp * d);
    A(&st->attn_part, (size_t)st->attn_splits * B * c.n_heads * (st->dh + 2));
    const int groups = bf16_gemm_groups(V, st->p_head.R);
    A(&st->pmax, (size_t)groups * Bp); A(&st->pidx, (size_t)groups * Bp);
    A(&st->logits_dev, (size_t)B * V);
  } else {
    float *t32 = nullptr;
    A(&t32, (size_t)B * d); st->a = t32;
    A(&t32, (size_t)B * 3 * d); st->q = t32;
    A(&t32, (size_t)B * d); st->o = t32;
    A(&t32, (size_t)B * f); st->u = t32;
    A(&st->attn_part, (size_t)B * c.n_heads * c.sequence_length);
    A(&st->logits_dev, (size_t)B * V);
  }
  if (rc != SKD_OK) return fail(rc);
  if (hipStreamSynchronize(st->stream) != hipSuccess) return fail(SKD_ERR_HIP);
  *out = st;
  return SKD_OK;
}

extern "C" int skd_create(const skd_config *cfg, const skd_weights *w, void *hip_stream, skd_state **out) {
  return create_impl(cfg, w, hip_stream, nullptr, out);
}

extern "C" int skd_create_with_schedule(const skd_config *cfg, const skd_weights *w, void *hip_stream,
                                        const int32_t *n_table, skd_state **out) {
  if (!n_table) return SKD_ERR_NULL;
  return create_impl(cfg, w, hip_stream, n_table, out);
}

extern "C" int skd_state_active_layers(const skd_state *st, int32_t t, int32_t *layers_out) {
  if (!st || !layers_out) return SKD_ERR_NULL;
  return state_active_layers(st, t, layers_out);
}

extern "C" void skd_destroy(skd_state *st) {
  if (!st) return;
  (void)hipStreamSynchronize(st->stream);
  for (auto &r : st->prof_pending) { if (r.a) (void)hipEventDestroy(r.a); if (r.b) (void)hipEventDestroy(r.b); }
  for (hipEvent_t e : st->prof_free) (void)hipEventDestroy(e);
  for (void *p : st->allocs) (void)hipFree(p);
  delete st;
}

// per-row padding offsets and the dispatch order of the attention workgroups (longest rows first)
static int upload_start(skd_state *st, const std::vector<int32_t> &start) {
  const int B = st->cfg.batch;
  std::vector<int32_t> order(B);
  for (int b = 0; b < B; ++b) order[b] = b;
  std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return start[x] < start[y]; });
  st->ragged = *std::max_element(start.begin(), start.end()) != *std::min_element(start.begin(), start.end());
  st->start_host = start;
  HIPCHECK(hipMemcpyAsync(st->start_dev, start.data(), B * sizeof(int32_t), hipMemcpyHostToDevice, st->stream));
  HIPCHECK(hipMemcpyAsync(st->order_dev, order.data(), B * sizeof(int32_t), hipMemcpyHostToDevice, st->stream));
  HIPCHECK(hipStreamSynchronize(st->stream));
  return SKD_OK;
}

// Whole prompt at once, layer by layer (Section 2.3: the prompt needs no generation, so it can be batched over
// positions): activation rows are the real (sequence, position) pairs (left padding gets no rows), the projections
// run on 256 x 256 tiles, attention is causal over the pages the QKV projection has just filled.
static int prefill_batched(skd_state *st, const int32_t *cols) {
  const skd_config &c = st->cfg;
  const int B = c.batch, P = c.prompt_size, d = c.d_model, f = c.ffn, L = c.L;
  const int P_pad = (P + 15) / 16 * 16;
  const long cap = ((long)B * P_pad + 255) / 256 * 256;  // workspace rows: every position of every sequence
  hipStream_t s = st->stream;
  if (!st->pf_x) {
    SKDCHECK(dev_alloc(st, &st->pf_x, (size_t)cap * d));
    SKDCHECK(dev_alloc(st, &st->pf_a, (size_t)cap * d));
    SKDCHECK(dev_alloc(st, &st->pf_q, (size_t)cap * d));
    SKDCHECK(dev_alloc(st, &st->pf_o, (size_t)cap * d));
    SKDCHECK(dev_alloc(st, &st->pf_u, (size_t)cap * f));
    SKDCHECK(dev_alloc(st, &st->pf_seq, (size_t)cap));
    SKDCHECK(dev_alloc(st, &st->pf_first, (size_t)B));
  }
  // only real tokens get rows: sequence b owns its P - start[b] positions, padded to whole 16-row tiles
  std::vector<int32_t> first(B), seq((size_t)cap, -1);
  long rows = 0;
  for (int b = 0; b < B; ++b) {
    const int len = P - st->start_host[b], lp = (len + 15) / 16 * 16;
    first[b] = (int32_t)rows;
    std::fill(seq.begin() + rows, seq.begin() + rows + lp, b);
    rows += lp;
  }
  const long rows_pad = (rows + 255) / 256 * 256;
  HIPCHECK(hipMemcpyAsync(st->pf_seq, seq.data(), (size_t)rows_pad * sizeof(int32_t), hipMemcpyHostToDevice, s));
  HIPCHECK(hipMemcpyAsync(st->pf_first, first.data(), (size_t)B * sizeof(int32_t), hipMemcpyHostToDevice, s));
  HIPCHECK(hipStreamSynchronize(s));  // the host vectors go out of scope
  RowMap rm{st->pf_seq, st->pf_first, st->start_dev, P};
  // padding rows are read by the projections: keep them finite
  HIPCHECK(hipMemsetAsync(st->pf_x, 0, (size_t)rows_pad * d * sizeof(float), s));
  HIPCHECK(hipMemsetAsync(st->pf_a, 0, (size_t)rows_pad * d * sizeof(bf16_t), s));
  HIPCHECK(hipMemsetAsync(st->pf_q, 0, (size_t)rows_pad * d * sizeof(bf16_t), s));
  HIPCHECK(hipMemsetAsync(st->pf_o, 0, (size_t)rows_pad * d * sizeof(bf16_t), s));
  bf16_embed_ln_rows(s, cols, rm, (int)rows, (const bf16_t *)st->tok_emb, (const bf16_t *)st->pos_emb, st->lw[0].ln1_g,
                     st->lw[0].ln1_b, st->pf_x, st->pf_a, B, d, c.vocab);
  // 256 x 256 tiles where the shape allows, else 128-row chunks through the skinny kernel
  auto proj = [&](const GemmArgs &g, int epi) {
    if (st->prefill_tiles && bf16_gemm_tile(s, g, epi) == 0) return 0;
    return bf16_gemm(s, g, epi, g.N % 64 ? 1 : 4, 1, 4);
  };
  for (int l = 0; l < L; ++l) {
    const LayerW &w = st->lw[l];
    GemmArgs ga{};
    ga.B = B; ga.B_pad = 128; ga.rows = (int)rows_pad; ga.rm = rm; ga.kv = st->geom; ga.d = d; ga.split = 1;
    ga.W = (const bf16_t *)w.wqkv; ga.G = st->p_qkv.R; ga.A = st->pf_a; ga.bias = w.bqkv; ga.N = 3 * d; ga.K = d;
    ga.q_out = st->pf_q; ga.kv_pool = (bf16_t *)st->pool; ga.bt_layer = bt_layer(st, l);
    if (proj(ga, EPI_QKV_ROWS) < 0) return SKD_ERR_SHAPE;
    AttnRowsArgs aa{};
    aa.q = st->pf_q; aa.pool = (const bf16_t *)st->pool; aa.bt_layer = bt_layer(st, l); aa.rm = rm;
    aa.rows = (int)rows; aa.kv = st->geom; aa.o = st->pf_o;
    bf16_attention_rows(s, aa);
    ga.W = (const bf16_t *)w.wo; ga.G = st->p_out.R; ga.A = st->pf_o; ga.bias = w.bo; ga.N = d; ga.K = d; ga.x = st->pf_x;
    if (proj(ga, EPI_RESID) < 0) return SKD_ERR_SHAPE;
    bf16_ln_rows(s, st->pf_x, w.ln2_g, w.ln2_b, st->pf_a, (int)rows, d);
    ga.W = (const bf16_t *)w.w1; ga.G = st->p_ffn1.R; ga.A = st->pf_a; ga.bias = w.b1; ga.N = f; ga.K = d; ga.act_out = st->pf_u;
    if (proj(ga, EPI_RELU) < 0) return SKD_ERR_SHAPE;
    ga.W = (const bf16_t *)w.w2; ga.G = st->p_ffn2.R; ga.A = st->pf_u; ga.bias = w.b2; ga.N = d; ga.K = f; ga.x = st->pf_x;
    if (proj(ga, EPI_RESID) < 0) return SKD_ERR_SHAPE;
    if (l + 1 < L) bf16_ln_rows(s, st->pf_x, st->lw[l + 1].ln1_g, st->lw[l + 1].ln1_b, st->pf_a, (int)rows, d);
    st->kv_len[l] = P;
  }
  // hidden state of the last prompt column, and its final LayerNorm, where the heads expect them
  bf16_gather_rows(s, st->pf_x, st->x, rm, B, d);
  bf16_ln_rows(s, st->x, st->lnf_g, st->lnf_b, (bf16_t *)st->a, B, d);
  HIPCHECK(hipGetLastError());
  st->have_hidden = true;
  st->have_argmax = false;
  return SKD_OK;
}

extern "C" int skd_prefill(skd_state *st, const int32_t *tokens, const uint8_t *attn_mask) {
  if (!st || !tokens) return SKD_ERR_NULL;
  const skd_config &c = st->cfg;
  const int B = c.batch, P = c.prompt_size;
  std::vector<int32_t> start(B, 0);
  if (attn_mask) {
    for (int b = 0; b < B; ++b) {
      int j = 0;
      while (j < P && attn_mask[(size_t)b * P + j] == 0) ++j;
      if (j == P) return SKD_ERR_SHAPE;  // a row needs at least one real token
      start[b] = j;
      for (; j < P; ++j)
        if (attn_mask[(size_t)b * P + j] == 0) return SKD_ERR_SHAPE;  // only left padding
    }
  }
  const int32_t *cols = nullptr;
  if (c.io_on_device) {
    cols = tokens;
  } else {
    std::vector<int32_t> tr((size_t)P * B);
    for (int b = 0; b < B; ++b)
      for (int j = 0; j < P; ++j) {
        const int32_t tok = tokens[(size_t)b * P + j];
        if (tok < 0 || tok >= c.vocab) return SKD_ERR_RANGE;
        tr[(size_t)j * B + b] = tok;
      }
    HIPCHECK(hipMemcpyAsync(st->prompt_dev, tr.data(), tr.size() * sizeof(int32_t), hipMemcpyHostToDevice, st->stream));
    HIPCHECK(hipStreamSynchronize(st->stream));
    cols = st->prompt_dev;
  }
  SKDCHECK(upload_start(st, start));
  std::fill(st->kv_len.begin(), st->kv_len.end(), 0);
  st->prefilled = false;
  st->steps_done = 0;
  bool full_depth_prompt = true;  // a caller's table may decay inside the prompt: then columns differ in depth
  for (int i = 0; i < P && full_depth_prompt; ++i)
    if (!st->n_table.empty() && st->n_table[i] != c.L) full_depth_prompt = false;
  if (st->bf16 && st->prefill_mode == 1 && full_depth_prompt) {
    SKDCHECK(prefill_batched(st, cols));
  } else {
    for (int i = 0; i < P; ++i) {  // column by column
      const int n = state_active_layers(st, i, st->layers_tmp.data());
      if (n < 0) return n;
      SKDCHECK(run_column(st, i, cols + (size_t)i * B, st->layers_tmp.data(), n));
    }
  }
  st->prefilled = true;
  if (!c.io_on_device) HIPCHECK(hipStreamSynchronize(st->stream));
  return SKD_OK;
}

extern "C" int skd_decode_step(skd_state *st, int32_t t, const int32_t *tokens_in) {
  if (!st) return SKD_ERR_NULL;
  const skd_config &c = st->cfg;
  if (!st->prefilled) return SKD_ERR_ORDER;
  if (t < 0 || t >= c.sequence_length) return SKD_ERR_RANGE;
  if (t != c.prompt_size + st->steps_done) return SKD_ERR_ORDER;
  const int32_t *tok = nullptr;
  if (!tokens_in) {
    if (!st->have_argmax) return SKD_ERR_ORDER;
    tok = st->argmax_dev;
  } else if (c.io_on_device) {
    tok = tokens_in;
  } else {
    for (int b = 0; b < c.batch; ++b)
      if (tokens_in[b] < 0 || tokens_in[b] >= c.vocab) return SKD_ERR_RANGE;
    HIPCHECK(hipMemcpyAsync(st->tok_dev, tokens_in, c.batch * sizeof(int32_t), hipMemcpyHostToDevice, st->stream));
    HIPCHECK(hipStreamSynchronize(st->stream));
    tok = st->tok_dev;
  }
  const int n = state_active_layers(st, t, st->layers_tmp.data());
  if (n < 0) return n;
  SKDCHECK(run_column(st, t, tok, st->layers_tmp.data(), n));
  st->steps_done += 1;
  if (!c.io_on_device) HIPCHECK(hipStreamSynchronize(st->stream));
  return SKD_OK;
}

// Final LayerNorm + LM head (+ greedy argmax into argmax_dev).  logits_target: device buffer [B][V] or null.
// final LayerNorm output -> logits (optional) and, unless the caller picks the token itself, the greedy token
static int head_logits(skd_state *st, float *logits_target, bool want_argmax = true) {
  const skd_config &c = st->cfg;
  const int B = c.batch, d = c.d_model, V = c.vocab;
  hipStream_t s = st->stream;
  if (!st->bf16) {
    float *lg = logits_target ? logits_target : st->logits_dev;
    { ProfScope ps_(st, SKD_PROF_OTHER); f32_layernorm(s, st->x, st->lnf_g, st->lnf_b, (float *)st->a, B, d); }
    { ProfScope ps_(st, SKD_PROF_OTHER); f32_linear(s, (const float *)st->head, nullptr, (const float *)st->a, lg, B, d, V, 0, 0); }
    if (want_argmax) { ProfScope ps_(st, SKD_PROF_OTHER); f32_argmax(s, lg, st->argmax_dev, B, V); }
  } else {
    GemmArgs ga{};
    ga.B = B; ga.B_pad = st->B_pad; ga.W = (const bf16_t *)st->head; ga.G = st->p_head.R; ga.A = (const bf16_t *)st->a;  // a = final LayerNorm output
    ga.N = V; ga.K = d; ga.split = 1; ga.logits = logits_target; ga.pmax = st->pmax; ga.pidx = st->pidx;
    int groups = 0;
    { ProfScope ps_(st, SKD_PROF_LM_HEAD); groups = launch_gemm(s, ga, EPI_LOGITS, st->p_head); }
    if (groups < 0) return SKD_ERR_SHAPE;
    if (want_argmax) { ProfScope ps_(st, SKD_PROF_ARGMAX); bf16_argmax_final(s, st->pmax, st->pidx, groups, st->B_pad, st->argmax_dev, B); }
  }
  HIPCHECK(hipGetLastError());
  return SKD_OK;
}

extern "C" int skd_logits_argmax(skd_state *st, int32_t *tokens_out, float *logits_out) {
  if (!st) return SKD_ERR_NULL;
  if (!st->have_hidden) return SKD_ERR_ORDER;
  const skd_config &c = st->cfg;
  const int B = c.batch, V = c.vocab;
  hipStream_t s = st->stream;
  float *logits_target = nullptr;  // where the kernels write logits, if anywhere
  if (logits_out) logits_target = c.io_on_device ? logits_out : st->logits_dev;
  SKDCHECK(head_logits(st, logits_target));
  st->have_argmax = true;
  if (c.io_on_device) {
    if (tokens_out)
      HIPCHECK(hipMemcpyAsync(tokens_out, st->argmax_dev, B * sizeof(int32_t), hipMemcpyDeviceToDevice, s));
    return SKD_OK;
  }
  if (tokens_out) HIPCHECK(hipMemcpyAsync(tokens_out, st->argmax_dev, B * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  if (logits_out)
    HIPCHECK(hipMemcpyAsync(logits_out, st->logits_dev, (size_t)B * V * sizeof(float), hipMemcpyDeviceToHost, s));
  HIPCHECK(hipStreamSynchronize(s));
  return SKD_OK;
}

// skd_logits_argmax for callers that cannot allocate: same kernels, with the LM head's per-workgroup partials in
// the static device array instead of the buffers skd_create reserved.  No hipMalloc / hipFree, no event creation,
// no host-side staging: outputs are device memory and the call only enqueues work on the state's stream.
extern "C" int skd_logits_argmax_noalloc(skd_state *st, int32_t *tokens_out, float *logits_out) {
  if (!st) return SKD_ERR_NULL;
  if (!st->have_hidden) return SKD_ERR_ORDER;
  const skd_config &c = st->cfg;
  if (!st->bf16 || !c.io_on_device) return SKD_ERR_SHAPE;
  const int groups = bf16_gemm_groups(c.vocab, st->p_head.R);
  if ((int64_t)groups * st->B_pad > SKD_NOALLOC_MAX_PARTIALS) return SKD_ERR_RANGE;  // beyond the static scratch
  void *base = (st->device >= 0 && st->device < kMaxDevices) ? g_scratch_ptr[st->device] : nullptr;
  if (!base) return SKD_ERR_ORDER;  // resolved by skd_create on the state's device
  float *pmax = (float *)base;
  int32_t *pidx = (int32_t *)((unsigned char *)base + 4 * (size_t)SKD_NOALLOC_MAX_PARTIALS);
  hipStream_t s = st->stream;
  GemmArgs ga{};
  ga.B = c.batch; ga.B_pad = st->B_pad; ga.W = (const bf16_t *)st->head; ga.G = st->p_head.R; ga.A = (const bf16_t *)st->a;
  ga.N = c.vocab; ga.K = c.d_model; ga.split = 1; ga.logits = logits_out; ga.pmax = pmax; ga.pidx = pidx;
  if (check_gemm(ga, EPI_LOGITS, st->p_head) != groups) return SKD_ERR_SHAPE;
  // every partial the final reduction reads is written by the projection of this same call: nothing to clear
  (void)launch_gemm(s, ga, EPI_LOGITS, st->p_head);
  bf16_argmax_final(s, pmax, pidx, groups, st->B_pad, st->argmax_dev, c.batch);
  HIPCHECK(hipGetLastError());
  st->have_argmax = true;
  if (tokens_out)
    HIPCHECK(hipMemcpyAsync(tokens_out, st->argmax_dev, c.batch * sizeof(int32_t), hipMemcpyDeviceToDevice, s));
  return SKD_OK;
}

extern "C" int skd_logits_sample(skd_state *st, const float *u, float temperature, float top_p, int32_t *tokens_out,
                                 float *logits_out) {
  if (!st || !u) return SKD_ERR_NULL;
  if (!st->have_hidden) return SKD_ERR_ORDER;
  if (!(temperature > 0.f) || !(top_p > 0.f) || top_p > 1.f) return SKD_ERR_RANGE;
  const skd_config &c = st->cfg;
  const int B = c.batch, V = c.vocab;
  if (V > 65536) return SKD_ERR_SHAPE;
  hipStream_t s = st->stream;
  const float *u_dev = u;
  if (!c.io_on_device) {
    for (int b = 0; b < B; ++b)
      if (!(u[b] >= 0.f) || u[b] >= 1.f) return SKD_ERR_RANGE;
    HIPCHECK(hipMemcpyAsync(st->u_dev, u, B * sizeof(float), hipMemcpyHostToDevice, s));
    HIPCHECK(hipStreamSynchronize(s));
    u_dev = st->u_dev;
  }
  float *lg = (logits_out && c.io_on_device) ? logits_out : st->logits_dev;
  SKDCHECK(head_logits(st, lg, false));
  { ProfScope ps_(st, SKD_PROF_ARGMAX); if (sample_top_p(s, lg, B, V, temperature, top_p, u_dev, st->argmax_dev) < 0) return SKD_ERR_SHAPE; }
  HIPCHECK(hipGetLastError());
  st->have_argmax = true;  // skd_decode_step(.., NULL) continues from the sampled tokens
  if (c.io_on_device) {
    if (tokens_out)
      HIPCHECK(hipMemcpyAsync(tokens_out, st->argmax_dev, B * sizeof(int32_t), hipMemcpyDeviceToDevice, s));
    return SKD_OK;
  }
  if (tokens_out) HIPCHECK(hipMemcpyAsync(tokens_out, st->argmax_dev, B * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  if (logits_out)
    HIPCHECK(hipMemcpyAsync(logits_out, st->logits_dev, (size_t)B * V * sizeof(float), hipMemcpyDeviceToHost, s));
  HIPCHECK(hipStreamSynchronize(s));
  return SKD_OK;
}

extern "C" int skd_rewind(skd_state *st, int32_t t) {
  if (!st) return SKD_ERR_NULL;
  if (!st->prefilled) return SKD_ERR_ORDER;
  const skd_config &c = st->cfg;
  if (t < c.prompt_size || t > c.prompt_size + st->steps_done) return SKD_ERR_RANGE;
  for (int l = 0; l < c.L; ++l) st->kv_len[l] = std::min(st->kv_len[l], (int)t);
  st->steps_done = t - c.prompt_size;
  st->have_hidden = false;  // the residual stream on the device belongs to a later column
  st->have_argmax = false;
  return SKD_OK;
}

extern "C" int skd_profile_enable(skd_state *st, int32_t on) {
  if (!st) return SKD_ERR_NULL;
  if (on < 0 || on > 2) return SKD_ERR_RANGE;
  SKDCHECK(prof_drain(st));
  st->profiling = on;
  return SKD_OK;
}

extern "C" int skd_profile_read(skd_state *st, double *ms, int64_t *launches) {
  if (!st) return SKD_ERR_NULL;
  SKDCHECK(prof_drain(st));
  for (int i = 0; i < SKD_PROF_CLASSES; ++i) {
    if (ms) ms[i] = st->prof_ms[i];
    if (launches) launches[i] = st->prof_n[i];
    st->prof_ms[i] = 0;
    st->prof_n[i] = 0;
  }
  return SKD_OK;
}

extern "C" int skd_kv_len(const skd_state *st, int32_t layer) {
  if (!st) return SKD_ERR_NULL;
  if (layer < 0 || layer >= st->cfg.L) return SKD_ERR_RANGE;
  return st->kv_len[layer];
}
extern "C" int64_t skd_kv_pages_reserved(const skd_state *st) { return st ? st->pages_reserved : SKD_ERR_NULL; }
extern "C" int64_t skd_kv_pages_dense(const skd_state *st) { return st ? st->pages_dense : SKD_ERR_NULL; }

extern "C" int skd_synchronize(skd_state *st) {
  if (!st) return SKD_ERR_NULL;
  HIPCHECK(hipStreamSynchronize(st->stream));
  return SKD_OK;
}

extern "C" int skd_debug_read_hidden(skd_state *st, float *x_out) {
  if (!st || !x_out) return SKD_ERR_NULL;
  if (!st->have_hidden) return SKD_ERR_ORDER;
  HIPCHECK(hipMemcpyAsync(x_out, st->x, (size_t)st->cfg.batch * st->cfg.d_model * sizeof(float), hipMemcpyDeviceToHost,
                          st->stream));
  HIPCHECK(hipStreamSynchronize(st->stream));
  return SKD_OK;
}

extern "C" int skd_debug_kv_load(skd_state *st, int32_t cols, const float *const *Kin, const float *const *Vin,
                                 const int32_t *start_in) {
  if (!st) return SKD_ERR_NULL;
  const skd_config &c = st->cfg;
  if (cols < c.prompt_size || cols >= c.sequence_length) return SKD_ERR_RANGE;
  const int B = c.batch, d = c.d_model;
  if (start_in)
    for (int b = 0; b < B; ++b)
      if (start_in[b] < 0 || start_in[b] >= cols) return SKD_ERR_RANGE;
  {
    std::vector<int32_t> start(B, 0);
    if (start_in) start.assign(start_in, start_in + B);
    SKDCHECK(upload_start(st, start));  // the bf16 pages are addressed by real position
  }
  const size_t n = (size_t)B * cols * d;
  float *kd = nullptr, *vd = nullptr;
  HIPCHECK(hipMalloc((void **)&kd, n * sizeof(float)));
  if (hipMalloc((void **)&vd, n * sizeof(float)) != hipSuccess) { (void)hipFree(kd); return SKD_ERR_NOMEM; }
  int rc = SKD_OK;
  for (int l = 0; l < c.L && rc == SKD_OK; ++l) {
    if (st->kv_cap[l] < cols) {  // the layer left the window before column `cols`: it never runs again
      st->kv_len[l] = st->kv_cap[l];
      continue;
    }
    const float *ks = Kin ? Kin[l] : nullptr, *vs = Vin ? Vin[l] : nullptr;
    const bool have = ks && vs;
    if (have && (hipMemcpyAsync(kd, ks, n * sizeof(float), hipMemcpyHostToDevice, st->stream) != hipSuccess ||
                 hipMemcpyAsync(vd, vs, n * sizeof(float), hipMemcpyHostToDevice, st->stream) != hipSuccess)) {
      rc = SKD_ERR_HIP;
      break;
    }
    if (st->bf16)
      kv_load_bf16(st->stream, have ? kd : nullptr, have ? vd : nullptr, (bf16_t *)st->pool, bt_layer(st, l), st->start_dev, cols, B, st->geom);
    else
      kv_load_f32(st->stream, have ? kd : nullptr, have ? vd : nullptr, (float *)st->pool, bt_layer(st, l), cols, B, st->geom);
    if (hipStreamSynchronize(st->stream) != hipSuccess) { rc = SKD_ERR_HIP; break; }
    st->kv_len[l] = cols;
  }
  (void)hipFree(kd);
  (void)hipFree(vd);
  if (rc != SKD_OK) return rc;
  st->prefilled = true;
  st->steps_done = cols - c.prompt_size;
  st->have_hidden = false;
  st->have_argmax = false;
  return SKD_OK;
}

extern "C" int skd_debug_kv_read(skd_state *st, int32_t layer, int32_t b, float *k_out, float *v_out) {
  if (!st || !k_out || !v_out) return SKD_ERR_NULL;
  const skd_config &c = st->cfg;
  if (layer < 0 || layer >= c.L || b < 0 || b >= c.batch) return SKD_ERR_RANGE;
  const int len = st->kv_len[layer], d = c.d_model;
  if (len == 0) return SKD_OK;
  float *kd = nullptr, *vd = nullptr;
  HIPCHECK(hipMalloc((void **)&kd, (size_t)len * d * sizeof(float)));
  if (hipMalloc((void **)&vd, (size_t)len * d * sizeof(float)) != hipSuccess) { (void)hipFree(kd); return SKD_ERR_NOMEM; }
  const int32_t *row = bt_layer(st, layer) + (size_t)b * st->geom.max_pages;
  if (st->bf16) kv_read_bf16(st->stream, (const bf16_t *)st->pool, row, st->start_host.empty() ? 0 : st->start_host[b], len, kd, vd, st->geom);
  else kv_read_f32(st->stream, (const float *)st->pool, row, len, kd, vd, st->geom);
  int rc = SKD_OK;
  if (hipMemcpyAsync(k_out, kd, (size_t)len * d * sizeof(float), hipMemcpyDeviceToHost, st->stream) != hipSuccess ||
      hipMemcpyAsync(v_out, vd, (size_t)len * d * sizeof(float), hipMemcpyDeviceToHost, st->stream) != hipSuccess ||
      hipStreamSynchronize(st->stream) != hipSuccess)
    rc = SKD_ERR_HIP;
  (void)hipFree(kd);
  (void)hipFree(vd);
  return rc;
}
