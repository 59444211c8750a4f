// fp32 debug path: small, straightforward kernels (no MFMA, no tiling) whose
// only job is to be an easily-audited GPU implementation of the decode step
// for the tight-tolerance parity build.  Not tuned.
#include "skd_kernels.h"

namespace skd {

__device__ inline float wave_sum(float v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
__device__ inline float wave_max(float v) {
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
// sum over a 256-thread workgroup; `sh` holds >= 4 floats; result to all threads
__device__ inline float block_sum(float v, float *sh) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = 0;
  for (unsigned w = 0; w < (blockDim.x >> 6); ++w) r += sh[w];
  return r;
}

__global__ void k_f32_embed(float *x, const float *tok_emb, const float *pos_emb, const int32_t *tokens,
                            const int32_t *start, int t, int d, int V) {
  const int b = blockIdx.x;
  int tok = tokens[b];
  tok = tok < 0 ? 0 : (tok >= V ? V - 1 : tok);
  int pos = t - start[b];  // real tokens before this column
  if (pos < 0) pos = 0;    // padding column: never read later
  for (int k = threadIdx.x; k < d; k += blockDim.x) x[(long)b * d + k] = tok_emb[(long)tok * d + k] + pos_emb[(long)pos * d + k];
}

__global__ void k_f32_layernorm(const float *x, const float *g, const float *bt, float *out, int d) {
  __shared__ float sh[4];
  const float *xr = x + (long)blockIdx.x * d;
  float s = 0;
  for (int k = threadIdx.x; k < d; k += blockDim.x) s += xr[k];
  const float mean = block_sum(s, sh) / d;
  float v = 0;
  for (int k = threadIdx.x; k < d; k += blockDim.x) v += (xr[k] - mean) * (xr[k] - mean);
  const float rstd = 1.0f / sqrtf(block_sum(v, sh) / d + 1e-5f);
  for (int k = threadIdx.x; k < d; k += blockDim.x) out[(long)blockIdx.x * d + k] = (xr[k] - mean) * rstd * g[k] + bt[k];
}

// one wave per output element (b, n): lanes stride over k
__global__ void k_f32_linear(const float *W, const float *bias, const float *in, float *out, int K, int N, int relu,
                             int accumulate) {
  const int n = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  const int b = blockIdx.y;
  if (n >= N) return;
  const float *w = W + (long)n * K, *a = in + (long)b * K;
  float acc = 0;
  for (int k = threadIdx.x & 63; k < K; k += 64) acc += w[k] * a[k];
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) {
    float v = acc + (bias ? bias[n] : 0.f);
    if (relu) v = fmaxf(v, 0.f);
    float *o = out + (long)b * N + n;
    *o = accumulate ? *o + v : v;
  }
}

__device__ inline long f32_kv_off(const int32_t *bt_row, int pos, int which, const KvGeom &g) {
  const int page = bt_row[pos / g.page_tokens];
  return (long)page * g.page_elems + ((long)which * g.page_tokens + pos % g.page_tokens) * (g.H * g.dh);
}

__global__ void k_f32_kv_write(const float *qkv, float *pool, const int32_t *bt_layer, int t, KvGeom g) {
  const int b = blockIdx.x, d = g.H * g.dh;
  const int32_t *bt_row = bt_layer + (long)b * g.max_pages;
  float *Kd = pool + f32_kv_off(bt_row, t, 0, g), *Vd = pool + f32_kv_off(bt_row, t, 1, g);
  for (int k = threadIdx.x; k < d; k += blockDim.x) {
    Kd[k] = qkv[(long)b * 3 * d + d + k];
    Vd[k] = qkv[(long)b * 3 * d + 2 * d + k];
  }
}

// one 64-lane workgroup per (b, h); scores kept in a global scratch row
__global__ void k_f32_attention(const float *qkv, const float *pool, const int32_t *bt_layer, const int32_t *start,
                                int t, float *o, float *scores, int score_stride, KvGeom g) {
  const int b = blockIdx.x / g.H, h = blockIdx.x % g.H, d = g.H * g.dh, lane = threadIdx.x;
  const int32_t *bt_row = bt_layer + (long)b * g.max_pages;
  const float *q = qkv + (long)b * 3 * d + h * g.dh;
  float *sc = scores + (long)blockIdx.x * score_stride;
  const int j0 = start[b];
  const float inv = 1.0f / sqrtf((float)g.dh);
  float mx = -3.0e38f;
  for (int j = j0 + lane; j <= t; j += 64) {
    const float *kr = pool + f32_kv_off(bt_row, j, 0, g) + h * g.dh;
    float s = 0;
    for (int e = 0; e < g.dh; ++e) s += q[e] * kr[e];
    s *= inv;
    sc[j] = s;
    mx = fmaxf(mx, s);
  }
  mx = wave_max(mx);
  float den = 0;
  for (int j = j0 + lane; j <= t; j += 64) {
    const float p = expf(sc[j] - mx);
    sc[j] = p;
    den += p;
  }
  den = wave_sum(den);
  __syncthreads();  // scores written by other lanes are read below
  for (int e = lane; e < g.dh; e += 64) {
    float acc = 0;
    for (int j = j0; j <= t; ++j) acc += sc[j] * pool[f32_kv_off(bt_row, j, 1, g) + h * g.dh + e];
    o[(long)b * d + h * g.dh + e] = (j0 <= t) ? acc / den : 0.f;
  }
}

__global__ void k_f32_argmax(const float *logits, int32_t *tokens, int V) {
  __shared__ float sv[256];
  __shared__ int si[256];
  const float *z = logits + (long)blockIdx.x * V;
  float best = -3.0e38f;
  int bi = 0x7fffffff;
  for (int v = threadIdx.x; v < V; v += blockDim.x)
    if (z[v] > best) { best = z[v]; bi = v; }  // ascending v per thread: first maximum kept
  sv[threadIdx.x] = best;
  si[threadIdx.x] = bi;
  __syncthreads();
  for (int s = blockDim.x / 2; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) {
      const float ov = sv[threadIdx.x + s];
      const int oi = si[threadIdx.x + s];
      if (ov > sv[threadIdx.x] || (ov == sv[threadIdx.x] && oi < si[threadIdx.x])) { sv[threadIdx.x] = ov; si[threadIdx.x] = oi; }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) tokens[blockIdx.x] = si[0];
}

// ------------------------------------------------------------------ sampling head (both paths; fp32 logits)
// Temperature + nucleus (top-p) sampling, one 1024-thread workgroup per row.
// Wave w keeps the contiguous index range [w*R*64, (w+1)*R*64) in registers, R = ceil(V / 1024) <= 64 rows of 64
// tokens, lane l holding token w*R*64 + 64 i + l of row i (coalesced 256-byte loads).
//   p_i = exp((z_i - max z) / T);  nucleus = {p_i >= tau}, tau = the largest value whose upper set has mass
//   >= top_p * sum p  (found bit by bit on the float bit pattern, 31 block sums; tokens tied with tau are in);
//   token = first index of the nucleus whose running mass (ascending index) exceeds u * mass(nucleus).
// Every sum is taken in a fixed order, so a given (logits, u) always yields the same token.
constexpr int SAMPLE_C = 64;
constexpr int SAMPLE_CAND = 1024;  // candidates one wave finishes alone (16 per lane; 32 per lane spills registers)

// RC: rows compiled in (>= R); 52 rows cover vocabularies up to 53248 without register spills
template <int RC>
__global__ __launch_bounds__(1024) void k_sample_top_p(const float *logits, int V, float inv_temp, float top_p,
                                                       const float *u, int32_t *tokens) {
  __shared__ float sh[16], wmass[16];
  __shared__ int wcount[16];
  __shared__ float cand_p[SAMPLE_CAND];  // candidates of the short cut, ascending token index
  __shared__ int cand_i[SAMPLE_CAND];
  __shared__ float rows[RC * 64];  // the rows of the one wave that walks its range
  __shared__ int last_in, hit_tok;
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int R = (V + 1023) / 1024, base = wave * R * 64 + lane;
  const float *z = logits + (long)b * V;
  float p[RC];
  float mx = -3.0e38f;
#pragma unroll
  for (int i = 0; i < RC; ++i) {
    p[i] = (i < R && base + 64 * i < V) ? z[base + 64 * i] * inv_temp : -3.0e38f;  // sentinel: no such token
    mx = fmaxf(mx, p[i]);
  }
  mx = wave_max(mx);
  if (lane == 0) sh[wave] = mx;
  if (tid == 0) { last_in = -1; hit_tok = -1; }
  __syncthreads();
  mx = sh[0];
  for (int w = 1; w < 16; ++w) mx = fmaxf(mx, sh[w]);
  float loc = 0;
#pragma unroll
  for (int i = 0; i < RC; ++i) {
    p[i] = p[i] > -1.0e38f ? expf(p[i] - mx) : 0.f;
    loc += p[i];
  }
  const float total = block_sum(loc, sh);
  const float target = top_p * total;

  // The threshold is found bit by bit on the float bit pattern, from the top.  The first 8 rounds (sign excluded:
  // the exponent bits) are taken by the whole workgroup; they fix the threshold to within a factor of two, and every
  // token below that lower bound is out of the nucleus whatever the remaining bits turn out to be.  If the tokens at
  // or above it are few (<= SAMPLE_CAND: nearly always at the paper's temperature 0.3, where the nucleus is a few
  // hundred tokens), they are compacted in index order into LDS and one wave finishes the row alone with wave-level
  // sums: no workgroup barrier in the remaining 23 rounds.  For every trial threshold at or above the lower bound
  // the sums run over the same tokens as in the whole-workgroup search, so the threshold is the same up to the
  // order of the fp32 additions.
  unsigned T = 0;
  for (int bit = 30; bit >= 23; --bit) {
    const unsigned cand = T | (1u << bit);
    float m = 0;
#pragma unroll
    for (int i = 0; i < RC; ++i) m += (__float_as_uint(p[i]) >= cand) ? p[i] : 0.f;  // absent tokens hold zeros
    if (block_sum(m, sh) >= target) T = cand;  // uniform decision: every thread sees the same sum
  }
  {
    const unsigned lower = max(T, 1u);  // bit pattern 0 = an absent token or an underflowed probability: never a candidate
    int cnt = 0;  // per lane first (a ballot per row here would be kept for the compaction below: 2 SGPRs per row)
    const unsigned below = lower - 1u;  // lower >= 1
#pragma unroll
    for (int i = 0; i < RC; ++i) cnt += (__float_as_uint(p[i]) > below) ? 1 : 0;  // non-negative floats order like their bits
    for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o);
    __syncthreads();  // sh (read by block_sum above) is free
    if (lane == 0) wcount[wave] = cnt;
    __syncthreads();
    int C = 0, wbase = 0;
    for (int w = 0; w < 16; ++w) {
      if (w < wave) wbase += wcount[w];
      C += wcount[w];
    }
    // uniform over the workgroup, and said so: as a divergent branch it would keep the 52-64 probabilities of the
    // other path alive in registers next to this path's candidates
    C = __builtin_amdgcn_readfirstlane(C);
    wbase = __builtin_amdgcn_readfirstlane(wbase);
    if (C <= SAMPLE_CAND) {
      int pos = wbase;
#pragma unroll
      for (int i = 0; i < RC; ++i) {
        // (the counting loop tests "> lower - 1", this one ">= lower": the same test, but the compiler recomputes it
        // here instead of keeping one lane mask per row from there)
        const bool c = __float_as_uint(p[i]) >= lower;
        const unsigned long long m = __ballot(c);
        if (c) {
          const int k = pos + __popcll(m & ((1ull << lane) - 1ull));
          cand_p[k] = p[i];
          cand_i[k] = base + 64 * i;
        }
        pos += __popcll(m);
        __builtin_amdgcn_sched_barrier(0);  // row by row: hoisted, the rows' lane masks would need 2 SGPRs each
      }
      __syncthreads();
      if (__builtin_amdgcn_readfirstlane(wave) == 0) {
        constexpr int PER = SAMPLE_CAND / 64;  // lane l owns candidates l * PER .. l * PER + PER - 1 (index order)
        float v[PER];
#pragma unroll
        for (int j = 0; j < PER; ++j) v[j] = lane * PER + j < C ? cand_p[lane * PER + j] : 0.f;
        for (int bit = 22; bit >= 0; --bit) {
          const unsigned cand = T | (1u << bit);
          float m = 0;
#pragma unroll
          for (int j = 0; j < PER; ++j) m += (__float_as_uint(v[j]) >= cand) ? v[j] : 0.f;
          if (wave_sum(m) >= target) T = cand;
        }
        float lm = 0;
        int last = -1;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
          if (__float_as_uint(v[j]) < T) v[j] = 0.f;
          lm += v[j];
          if (v[j] > 0.f) last = lane * PER + j;
        }
        float inc = lm;  // inclusive prefix of the lanes' masses = prefix in index order
        for (int off = 1; off < 64; off <<= 1) {
          const float t = __shfl_up(inc, off);
          if (lane >= off) inc += t;
        }
        const float goal = u[b] * __shfl(inc, 63);
        const unsigned long long over = __ballot(inc > goal);
        int k = -1;
        if (over) {
          const int L = (int)__builtin_ctzll(over);
          if (lane == L) {
            float run = inc - lm;
#pragma unroll
            for (int j = 0; j < PER; ++j) {
              run += v[j];
              if (k < 0 && v[j] > 0.f && run > goal) k = lane * PER + j;
            }
            if (k < 0) k = last;  // rounding between the lane's two summation orders: its last member
          }
          k = __shfl(k, L);
        } else {  // rounding at the very end: the last member of the nucleus
          for (int o = 32; o > 0; o >>= 1) last = max(last, __shfl_xor(last, o));
          k = last;
        }
        if (lane == 0) tokens[b] = k >= 0 ? cand_i[k] : 0;
      }
      return;
    }
  }
  for (int bit = 22; bit >= 0; --bit) {
    const unsigned cand = T | (1u << bit);
    float m = 0;
#pragma unroll
    for (int i = 0; i < RC; ++i) m += (__float_as_uint(p[i]) >= cand) ? p[i] : 0.f;  // absent tokens hold zeros
    if (block_sum(m, sh) >= target) T = cand;  // uniform decision: every thread sees the same sum
  }
  // nucleus: zero everything else; mass per wave (each wave owns a contiguous index range)
  loc = 0;
  int last = -1;
#pragma unroll
  for (int i = 0; i < RC; ++i) {
    if (__float_as_uint(p[i]) < T) p[i] = 0.f;
    loc += p[i];
    if (p[i] > 0.f) last = base + 64 * i;
  }
  loc = wave_sum(loc);
  __syncthreads();  // sh is free again
  if (lane == 0) wmass[wave] = loc;
  if (last >= 0) atomicMax(&last_in, last);
  __syncthreads();
  float mass = 0, before = 0;
  for (int w = 0; w < 16; ++w) {
    if (w < wave) before += wmass[w];
    mass += wmass[w];
  }
  const float goal = u[b] * mass;
  // the wave whose range contains the crossing walks its rows in index order
  const bool mine = before <= goal && before + wmass[wave] > goal;  // at most one wave: the prefix sums are monotone
  if (mine) {
#pragma unroll
    for (int i = 0; i < RC; ++i) rows[i * 64 + lane] = p[i];  // own lane's column: no barrier needed
    float run = before;
    int tok = -1;
    for (int i = 0; i < R && tok < 0; ++i) {
      {
        const float pi = rows[i * 64 + lane];
        float inc = pi;  // inclusive prefix over the lanes of this row
        for (int off = 1; off < 64; off <<= 1) {
          const float t = __shfl_up(inc, off);
          if (lane >= off) inc += t;
        }
        const float row = __shfl(inc, 63);
        if (run + row > goal) {
          const unsigned long long over = __ballot(pi > 0.f && run + inc > goal);
          if (over) tok = wave * R * 64 + 64 * i + (int)__builtin_ctzll(over);
        }
        run += row;
      }
    }
    if (tok < 0) {  // rounding between the two summation orders: the last member of this wave's range
      int wl = last;
      for (int o = 32; o > 0; o >>= 1) wl = max(wl, __shfl_xor(wl, o));
      tok = wl;
    }
    if (lane == 0) hit_tok = tok;
  }
  __syncthreads();
  if (tid == 0) tokens[b] = hit_tok >= 0 ? hit_tok : last_in;  // rounding at the very end: last member
}

int sample_top_p(hipStream_t s, const float *logits, int B, int V, float temperature, float top_p, const float *u,
                 int32_t *tokens) {
  if (V > 1024 * SAMPLE_C) return -1;
  const int R = (V + 1023) / 1024;
  const float it = 1.0f / temperature;
  if (R <= 16) SKD_LAUNCH(k_sample_top_p<16>, dim3(B), dim3(1024), 0, s, logits, V, it, top_p, u, tokens);
  else if (R <= 32) SKD_LAUNCH(k_sample_top_p<32>, dim3(B), dim3(1024), 0, s, logits, V, it, top_p, u, tokens);
  else if (R <= 52) SKD_LAUNCH(k_sample_top_p<52>, dim3(B), dim3(1024), 0, s, logits, V, it, top_p, u, tokens);
  else SKD_LAUNCH(k_sample_top_p<SAMPLE_C>, dim3(B), dim3(1024), 0, s, logits, V, it, top_p, u, tokens);
  return 0;
}

void f32_embed(hipStream_t s, float *x, const float *tok_emb, const float *pos_emb, const int32_t *tokens,
               const int32_t *start, int t, int B, int d, int V) {
  SKD_LAUNCH(k_f32_embed, dim3(B), dim3(256), 0, s, x, tok_emb, pos_emb, tokens, start, t, d, V);
}
void f32_layernorm(hipStream_t s, const float *x, const float *g, const float *b, float *out, int B, int d) {
  SKD_LAUNCH(k_f32_layernorm, dim3(B), dim3(256), 0, s, x, g, b, out, d);
}
void f32_linear(hipStream_t s, const float *W, const float *bias, const float *in, float *out, int B, int K, int N,
                int relu, int accumulate) {
  SKD_LAUNCH(k_f32_linear, dim3((N + 3) / 4, B), dim3(256), 0, s, W, bias, in, out, K, N, relu, accumulate);
}
void f32_kv_write(hipStream_t s, const float *qkv, float *pool, const int32_t *bt_layer, int t, int B, KvGeom g) {
  SKD_LAUNCH(k_f32_kv_write, dim3(B), dim3(256), 0, s, qkv, pool, bt_layer, t, g);
}
void f32_attention(hipStream_t s, const float *qkv, const float *pool, const int32_t *bt_layer, const int32_t *start,
                   int t, float *o, float *scores, int score_stride, int B, KvGeom g) {
  SKD_LAUNCH(k_f32_attention, dim3(B * g.H), dim3(64), 0, s, qkv, pool, bt_layer, start, t, o, scores,
                     score_stride, g);
}
void f32_argmax(hipStream_t s, const float *logits, int32_t *tokens, int B, int V) {
  SKD_LAUNCH(k_f32_argmax, dim3(B), dim3(256), 0, s, logits, tokens, V);
}

// ------------------------------------------------------------------ KV debug hooks (fp32 pages)
__global__ void k_kv_load_f32(const float *K, const float *V, float *pool, const int32_t *bt_layer, int cols,
                              KvGeom g) {
  const int b = blockIdx.y, j = blockIdx.x, d = g.H * g.dh;
  const int32_t *bt_row = bt_layer + (long)b * g.max_pages;
  float *Kd = pool + f32_kv_off(bt_row, j, 0, g), *Vd = pool + f32_kv_off(bt_row, j, 1, g);
  for (int k = threadIdx.x; k < d; k += blockDim.x) {
    Kd[k] = K ? K[((long)b * cols + j) * d + k] : 0.f;
    Vd[k] = V ? V[((long)b * cols + j) * d + k] : 0.f;
  }
}
__global__ void k_kv_read_f32(const float *pool, const int32_t *bt_row, float *K, float *V, KvGeom g) {
  const int j = blockIdx.x, d = g.H * g.dh;
  for (int k = threadIdx.x; k < d; k += blockDim.x) {
    K[(long)j * d + k] = pool[f32_kv_off(bt_row, j, 0, g) + k];
    V[(long)j * d + k] = pool[f32_kv_off(bt_row, j, 1, g) + k];
  }
}
void kv_load_f32(hipStream_t s, const float *K, const float *V, float *pool, const int32_t *bt_layer, int cols, int B,
                 KvGeom g) {
  if (cols > 0) SKD_LAUNCH(k_kv_load_f32, dim3(cols, B), dim3(256), 0, s, K, V, pool, bt_layer, cols, g);
}
void kv_read_f32(hipStream_t s, const float *pool, const int32_t *bt_row, int len, float *K, float *V, KvGeom g) {
  if (len > 0) SKD_LAUNCH(k_kv_read_f32, dim3(len), dim3(256), 0, s, pool, bt_row, K, V, g);
}

}  // namespace skd
