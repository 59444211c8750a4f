// Internal launch interface between the host engine and the gfx950 kernels.
// Not part of the public ABI (include/skd.h is).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

namespace skd {

typedef uint16_t bf16_t;  // raw bfloat16 bit pattern in host-visible signatures

// Per-launch timing.  While a thread has a LaunchTimer installed, every kernel launch it makes through
// SKD_LAUNCH takes a (start, stop) event pair from the timer and goes through hipExtLaunchKernelGGL, which
// stamps the two events with the begin and end of that kernel itself (the dispatch's own time stamps, what a
// kernel trace reports), not with the time of extra marker packets around it.
struct LaunchTimer {
  virtual void next(hipEvent_t *start, hipEvent_t *stop) = 0;

 protected:
  ~LaunchTimer() = default;
};
extern thread_local LaunchTimer *g_launch_timer;

#define SKD_LAUNCH(kernel, grid, blk, lds, stream, ...)                                        \
  do {                                                                                         \
    if (skd::g_launch_timer) {                                                                 \
      hipEvent_t e0_ = nullptr, e1_ = nullptr;                                                 \
      skd::g_launch_timer->next(&e0_, &e1_);                                                   \
      hipExtLaunchKernelGGL(kernel, grid, blk, lds, stream, e0_, e1_, 0, __VA_ARGS__);         \
    } else {                                                                                   \
      hipLaunchKernelGGL(kernel, grid, blk, lds, stream, __VA_ARGS__);                         \
    }                                                                                          \
  } while (0)

// Geometry of the paged KV cache.  A page holds `page_tokens` consecutive
// positions of ONE batch row in ONE layer, all heads.  On the bf16 path a row's
// keys are stored by real position (column j of a row that starts at column
// start[b] sits in slot j - start[b]; padding columns store nothing), so that a
// left-padded row reads no padding; the fp32 path stores by column.
struct KvGeom {
  int page_tokens;
  int max_pages;      // block-table entries per (layer, row)
  int H, dh;
  long page_elems;    // elements (fp32 or bf16) per page = 2 * page_tokens * H * dh
};

// ---------------------------------------------------------------- fp32 debug path
// Everything row-major fp32.  KV page layout: [K|V][page_tokens][H*dh].
void f32_embed(hipStream_t s, float *x, const float *tok_emb, const float *pos_emb, const int32_t *tokens,
               const int32_t *start, int t, int B, int d, int V);
void f32_layernorm(hipStream_t s, const float *x, const float *g, const float *b, float *out, int B, int d);
// out[b][n] = (accumulate ? out[b][n] : 0) + bias[n] + sum_k W[n][k] * in[b][k]; optional ReLU
void f32_linear(hipStream_t s, const float *W, const float *bias, const float *in, float *out, int B, int K, int N,
                int relu, int accumulate);
void f32_kv_write(hipStream_t s, const float *qkv, float *pool, const int32_t *bt_layer, int t, int B, KvGeom g);
void f32_attention(hipStream_t s, const float *qkv, const float *pool, const int32_t *bt_layer, const int32_t *start,
                   int t, float *o, float *scores, int score_stride, int B, KvGeom g);
void f32_argmax(hipStream_t s, const float *logits, int32_t *tokens, int B, int V);
// temperature + top-p sampling from fp32 logits [B][V] with one uniform number per row; -1 if V > 65536
int sample_top_p(hipStream_t s, const float *logits, int B, int V, float temperature, float top_p, const float *u,
                 int32_t *tokens);

// ---------------------------------------------------------------- bf16 production path
// Weights [N][K] are "fragment-major": 16-row x 32-column fragments stored as
// 64 lanes x 8 elements, lane = (row % 16) + 16 * ((col % 32) / 8), element =
// col % 8: one lane-wide 16-byte load is exactly one A operand of
// v_mfma_f32_16x16x32_bf16.  The 16-row tiles are bundled in groups of G
// (1..4, chosen per matrix as the tile rows one workgroup owns) and stored
// [tile / G][col / 32][tile % G], so that the G fragments a wave needs for one
// k-step are G KiB of consecutive addresses.
// Activations [rows][K] (rows padded to 16) use the same 16 x 32 tiles in the
// order [row / 16][col / 32], but row-major inside a tile (16 rows of 64
// bytes): one tile is still one 1 KiB B-operand load (lane l reads 16-byte
// slot (l % 16) * 4 + l / 16), while a producer that owns a row stores 64-byte
// runs instead of scattered 8- or 16-byte pieces.
// Rows of the batched prompt pass.  Only real tokens get rows: sequence b owns P - start[b] rows (its real
// positions, in order), padded to a multiple of 16, starting at first_row[b].
struct RowMap {
  const int32_t *seq;        // [rows] sequence of each row (rows past the last sequence: -1)
  const int32_t *first_row;  // [B] multiple of 16
  const int32_t *start;      // [B] first real column of each sequence
  int P;                     // prompt columns
};

enum GemmEpilogue {
  EPI_PARTIAL = 0,  // fp32 partial sums [split][B_pad][N], no bias
  EPI_QKV = 1,      // + bias; q -> row-major bf16, k/v -> row-major staging rows (filed into the page by bf16_attention)
  EPI_RELU = 2,     // + bias, ReLU -> activation tiles bf16 [B_pad][N]
  EPI_LOGITS = 3,   // optional fp32 logits [B][N] + per-workgroup (max, argmax) partials
  EPI_QKV_ROWS = 4, // batched prompt: + bias; q -> activation tiles [rows][d]; k/v -> KV page slot of (sequence, position)
  EPI_RESID = 5     // batched prompt: x[row][n] += value + bias (fp32 residual stream)
};

struct GemmArgs {
  const bf16_t *W;     // fragment-major [Nt_pad*16][K], tiles in groups of G
  int G;               // tile-group size of W's layout (Nt_pad is a multiple of 12, so of every G)
  const bf16_t *A;     // activation tiles [B_pad][K]
  const float *bias;   // [N] or null
  int N, K, B, B_pad;
  int split;           // workgroups along K (grid.y)
  int ws_rot;          // bf16_gemm_ws: workgroups start their K range at different stages
  // batched prompt processing: activation rows are the real (sequence, position) pairs of `rm`, handled in
  // 256 x 256 tiles or in chunks of B_pad rows along grid.z.  rows = 0: one chunk whose rows are the batch (decode).
  int rows;            // rows of the prompt pass, padded to 256
  RowMap rm;           // EPI_QKV_ROWS
  float *x;            // EPI_RESID: [rows][N] fp32
  // outputs (by epilogue)
  float *partial;      // EPI_PARTIAL
  bf16_t *q_out;       // EPI_QKV: [B_pad][d] row-major
  bf16_t *kv_new;      // EPI_QKV: [B][k | v][d] row-major
  bf16_t *kv_pool;     // EPI_QKV_ROWS
  const int32_t *bt_layer;  // EPI_QKV_ROWS: [B][max_pages]
  int d;               // EPI_QKV, EPI_QKV_ROWS: d_model (N = 3d)
  KvGeom kv;           // EPI_QKV_ROWS
  bf16_t *act_out;     // EPI_RELU
  float *logits;       // EPI_LOGITS (nullable)
  float *pmax;         // EPI_LOGITS: [groups][B_pad]
  int32_t *pidx;       // EPI_LOGITS
};
// R in 1..4: 16-row weight tiles per workgroup (each wave accumulates all of them over its share of K); U in {1,2,4}: k-steps per register buffer (prefetch depth);
// waves in {4,8}: waves per workgroup.  K/32 must be a multiple of a.split.
// Returns the number of row groups launched (grid.x), or -1 for an unsupported shape.
int bf16_gemm(hipStream_t s, const GemmArgs &a, int epilogue, int R, int U, int waves);
// The same shape checks without a launch (only N, K, B_pad, G, split and rows of `a` are read): groups or -1.
int bf16_gemm_check(const GemmArgs &a, int epilogue, int R, int U, int waves);
int bf16_gemm_groups(int N, int R);
// Decode projections with B_pad = 128 on the wave-specialised kernel (weight-streaming waves + activation-loading
// waves); (K / 32 / split) must be a multiple of 4.  Returns the row groups launched, or -1 (nothing launched) for
// shapes it does not handle; bf16_gemm_ws_check answers the same without launching.
int bf16_gemm_ws(hipStream_t s, const GemmArgs &a, int epilogue, int R);
int bf16_gemm_ws_check(const GemmArgs &a, int epilogue, int R);
// Batched prompt only (a.rows > 0; EPI_QKV_ROWS, EPI_RESID or EPI_RELU): 256 x 256 output tiles with LDS-staged
// operands.  Needs rows % 256 == 0 and N % 256 == 0 (K % 32 == 0 as everywhere); returns -1 otherwise (nothing launched).
int bf16_gemm_tile(hipStream_t s, const GemmArgs &a, int epilogue);

void bf16_embed_ln(hipStream_t s, const int32_t *tokens, const int32_t *start, int t, const bf16_t *tok_emb,
                   const bf16_t *pos_emb, const float *g, const float *b, float *x, bf16_t *a_out, int B, int d,
                   int V);
// x[b][:] += bias + sum_s partial[s][b][:]; a_out = LayerNorm(x; g, b) as bf16 activation tiles
void bf16_reduce_ln(hipStream_t s, const float *partial, int split, int B_pad, const float *bias, float *x,
                    const float *g, const float *b, bf16_t *a_out, int B, int d);
// Decode attention at position t.  Keys of columns start[b] .. t-1 (slots 0 .. t-start[b]-1) come from the pages; k and v of position t itself come
// from kv_new (written by the EPI_QKV projection) and are stored into the page slot of t by this kernel.
struct AttnArgs {
  const bf16_t *q;          // [B_pad][d] row-major
  const bf16_t *kv_new;     // [B][k | v][d] row-major
  bf16_t *pool;
  const int32_t *bt_layer;  // [B][max_pages]
  const int32_t *start;     // [B] first real column of each row
  const int32_t *order;     // [B] rows sorted by descending length: workgroup x/H handles row order[x/H] (null = identity)
  int t;                    // position being processed: cached keys start[b] .. t-1, plus t itself from kv_new
  int B, splits;
  int waves;                // waves per workgroup: 2, 4, 8 or 16
  KvGeom kv;
  bf16_t *o;                // activation tiles [B_pad][d]
  float *part;              // splits > 1: [splits][B*H][dh + 2]
};
void bf16_attention(hipStream_t s, const AttnArgs &a);
// Causal attention of a whole prompt: query rows (b, pos), 64 positions per workgroup, keys of columns start[b] .. pos.
struct AttnRowsArgs {
  const bf16_t *q;          // activation tiles [rows][d]
  const bf16_t *pool;
  const int32_t *bt_layer;  // [B][max_pages]
  RowMap rm;
  int rows;                 // multiple of 16
  KvGeom kv;
  bf16_t *o;                // activation tiles [rows][d]
};
void bf16_attention_rows(hipStream_t s, const AttnRowsArgs &a);
// Batched prompt row kernels; tokens laid out [P][B].
void bf16_embed_ln_rows(hipStream_t s, const int32_t *tokens, RowMap rm, int rows, const bf16_t *tok_emb,
                        const bf16_t *pos_emb, const float *g, const float *b, float *x, bf16_t *a_out, int B, int d,
                        int V);
void bf16_ln_rows(hipStream_t s, const float *x, const float *g, const float *b, bf16_t *a_out, int rows, int d);
// x_out[b][:] = row of sequence b's last prompt position
void bf16_gather_rows(hipStream_t s, const float *x_rows, float *x_out, RowMap rm, int B, int d);
void bf16_argmax_final(hipStream_t s, const float *pmax, const int32_t *pidx, int groups, int B_pad, int32_t *tokens,
                       int B);

// weight preparation (source fp32 or bf16 row-major, on device)
void prep_matrix_frag(hipStream_t s, const void *src, int src_is_bf16, bf16_t *dst, long N, long K, long N_pad,
                      int G);
void prep_matrix_rm_bf16(hipStream_t s, const void *src, int src_is_bf16, bf16_t *dst, long n);
void prep_to_f32(hipStream_t s, const void *src, int src_is_bf16, float *dst, long n);
// KV debug hooks: [B][cols][d] fp32 <-> pages
void kv_load_f32(hipStream_t s, const float *K, const float *V, float *pool, const int32_t *bt_layer, int cols, int B,
                 KvGeom g);
void kv_load_bf16(hipStream_t s, const float *K, const float *V, bf16_t *pool, const int32_t *bt_layer,
                  const int32_t *start, int cols, int B, KvGeom g);
void kv_read_f32(hipStream_t s, const float *pool, const int32_t *bt_row, int len, float *K, float *V, KvGeom g);
void kv_read_bf16(hipStream_t s, const bf16_t *pool, const int32_t *bt_row, int start, int len, float *K, float *V,
                  KvGeom g);

}  // namespace skd
