// bf16 production kernels for gfx950 (CDNA4, wave64).
//
// Decode at batch sizes 8..128 is a weight- and KV-streaming problem: every
// projection reads its whole weight matrix once per step and every attention
// head reads its whole KV history once per step, with O(batch) flops per byte.
// The kernels are therefore organised around 16-byte-per-lane, fully coalesced
// streams that land directly in the register layout of
// v_mfma_f32_16x16x32_bf16 (no LDS round trip for streamed data):
//   * weights are stored "fragment-major" (see skd_kernels.h) so one
//     wave-wide load = one 16x32 MFMA A-operand;
//   * activations are kept in 16-row x 32-column tiles, row-major inside the
//     tile: one tile is one 1 KiB B-operand load, and a producer that owns a
//     row stores whole 32-byte sectors;
//   * K is stored per 16-key tile as A-operand fragments (keys x head_dim),
//     V per 32-key block as A-operand fragments of V^T (head_dim x keys) with
//     the key order inside a block chosen so that the softmax weights leave
//     the QK^T accumulator already in B-operand position.
#include "skd_kernels.h"

namespace skd {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t uint32x4;

// fp32 -> bf16, round to nearest even: the conversion instruction of gfx950 (v_cvt_pk_bf16_f32), which the compiler
// emits for these casts; the same rounding in integer arithmetic takes five instructions per value.
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float floatx2;
__device__ inline uint32_t f2bf(float f) { return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)f); }
__device__ inline float bf2f(uint32_t h) { return __uint_as_float(h << 16); }
__device__ inline uint32_t pack2(float lo, float hi) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(floatx2{lo, hi}, bf16x2));
}

__device__ inline float wave_sum_f(float v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
// one barrier: `sh` (16 floats) must not have been read since the last barrier of the block
__device__ inline float block_sum_once(float v, float *sh) {
  v = wave_sum_f(v);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = 0;
  for (unsigned w = 0; w < (blockDim.x >> 6); ++w) r += sh[w];
  return r;
}

// Activations [rows][K]: 16-row x 32-column tiles in the order [row / 16][col / 32], each tile 16 rows of 64
// contiguous bytes.  A producer that owns one row writes 64-byte runs (whole 32-byte sectors); a consumer reads a
// tile as one MFMA B-operand fragment, lane l taking the 16 bytes at row l % 16, columns 8 * (l / 16) .. + 7,
// i.e. 16-byte slot act_lane(l) of the 1 KiB tile.
__device__ inline long d_act_index(long row, long col, long K) {
  return ((row >> 4) * (K >> 5) + (col >> 5)) * 512 + (row & 15) * 32 + (col & 31);
}
__device__ inline int act_lane(int lane) { return (lane & 15) * 4 + (lane >> 4); }

// ------------------------------------------------------------------ KV page addressing
// Page (one batch row, one layer): [head][32-key block][K block | V block],
// K block = [tile 0..1][chunk 0..dh/32-1][lane][8], V block = [dh/16][lane][8].
__device__ inline long kv_block_base(int h, int tt, const KvGeom &g) {
  return (long)h * (g.page_tokens * g.dh * 2) + (long)(tt >> 5) * (64 * g.dh);
}
__device__ inline long kv_k_off(int h, int tt, int e, const KvGeom &g) {
  const int kk = tt & 31;
  return kv_block_base(h, tt, g) +
         ((long)((kk >> 4) * (g.dh >> 5) + (e >> 5)) * 64 + (kk & 15) + 16 * ((e & 31) >> 3)) * 8 + (e & 7);
}
__device__ inline long kv_v_off(int h, int tt, int e, const KvGeom &g) {
  const int kk = tt & 31;
  return kv_block_base(h, tt, g) + 32 * g.dh +
         ((long)(e >> 4) * 64 + 16 * ((kk & 15) >> 2) + (e & 15)) * 8 + 4 * (kk >> 4) + (kk & 3);
}

// ------------------------------------------------------------------ skinny GEMM
// C[b][n] = sum_k A[b][k] * W[n][k], batch on the MFMA column side.
// Workgroup = 4 or 8 waves that share the same 16*R weight rows and interleave
// the workgroup's K range among themselves; grid.y splits K further across
// workgroups.  Each wave streams R weight-fragment rows and MB activation
// fragments per 32-wide k-step through two register buffers of U k-steps.
// What an epilogue reads from global memory (bias, residual, page index) is
// fetched ahead of the cross-wave reduction, so the end of the kernel is not a
// chain of dependent round trips.
struct EpiPre {
  floatx4 bias, x;
  int page, slot;
};
template <int EPI>
__device__ inline EpiPre epi_prefetch(const GemmArgs &a, int row, int n0) {
  EpiPre p;
  p.bias = p.x = floatx4{0.f, 0.f, 0.f, 0.f};
  p.page = 0;
  p.slot = 0;
  if constexpr (EPI == EPI_QKV || EPI == EPI_RELU || EPI == EPI_QKV_ROWS || EPI == EPI_RESID) {
    if (n0 + 3 < a.N) p.bias = *(const floatx4 *)&a.bias[n0];  // N is a multiple of 4 for these
  }
  if constexpr (EPI == EPI_QKV_ROWS) {
    p.page = -1;
    if (n0 >= a.d && n0 < a.N && row < a.rows) {
      const int b = a.rm.seq[row];
      if (b >= 0) {
        const int slot = row - a.rm.first_row[b];  // = real position: keys are stored by real position
        if (slot < a.rm.P - a.rm.start[b]) {       // else padding of the sequence's last 16-row tile
          p.page = a.bt_layer[(long)b * a.kv.max_pages + slot / a.kv.page_tokens];
          p.slot = slot;
        }
      }
    }
  }
  if constexpr (EPI == EPI_RESID) {
    if (n0 + 3 < a.N && row < a.rows) p.x = *(const floatx4 *)&a.x[(long)row * a.N + n0];
  }
  return p;
}

template <int EPI>
__device__ inline void gemm_epilogue(const GemmArgs &a, int b, int n0, floatx4 v, const EpiPre &pre);

template <>
__device__ inline void gemm_epilogue<EPI_PARTIAL>(const GemmArgs &a, int b, int n0, floatx4 v, const EpiPre &) {
  if (n0 + 3 < a.N) {
    *(floatx4 *)&a.partial[((long)blockIdx.y * a.B_pad + b) * a.N + n0] = v;
  }
}

template <>
__device__ inline void gemm_epilogue<EPI_QKV>(const GemmArgs &a, int b, int n0, floatx4 v, const EpiPre &pre) {
  if (n0 >= a.N) return;
  v += pre.bias;
  const int which = n0 / a.d, within = n0 - which * a.d;
  if (which == 0) {
    uint2 pk = make_uint2(pack2(v[0], v[1]), pack2(v[2], v[3]));
    *(uint2 *)&a.q_out[(long)b * a.d + within] = pk;
    return;
  }
  // k and v of the new position: row-major staging [B][k | v][d]; the attention kernel that follows
  // files them into the KV page while it streams the cache (scattered 2- and 8-byte stores at the end of this
  // kernel cost 3 us per layer)
  if (b >= a.B) return;
  uint2 pk = make_uint2(pack2(v[0], v[1]), pack2(v[2], v[3]));
  *(uint2 *)&a.kv_new[((long)b * 2 + (which - 1)) * a.d + within] = pk;
}

template <>
__device__ inline void gemm_epilogue<EPI_RELU>(const GemmArgs &a, int b, int n0, floatx4 v, const EpiPre &pre) {
  if (n0 >= a.N) return;
  for (int i = 0; i < 4; ++i) v[i] = fmaxf(v[i] + pre.bias[i], 0.f);
  uint2 pk = make_uint2(pack2(v[0], v[1]), pack2(v[2], v[3]));
  *(uint2 *)&a.act_out[d_act_index(b, n0, a.N)] = pk;
}

// tile rows that fit the 64 KiB cross-wave reduction buffer at once (each tile row = WAVES * MB KiB)
constexpr int gemm_stage_rows(int waves, int R, int MB) {
  const int fit = 64 / (waves * MB);
  return fit >= R ? R : (fit > 0 ? fit : 1);
}

template <>
__device__ inline void gemm_epilogue<EPI_QKV_ROWS>(const GemmArgs &a, int row, int n0, floatx4 v, const EpiPre &pre) {
  if (n0 >= a.N || row >= a.rows) return;
  v += pre.bias;
  const int which = n0 / a.d, within = n0 - which * a.d;
  const uint2 pk = make_uint2(pack2(v[0], v[1]), pack2(v[2], v[3]));
  if (which == 0) {
    *(uint2 *)&a.q_out[d_act_index(row, within, a.d)] = pk;
    return;
  }
  if (pre.page < 0) return;  // padding row
  const int h = within / a.kv.dh, e = within - h * a.kv.dh;
  bf16_t *pg = a.kv_pool + (long)pre.page * a.kv.page_elems;
  const int tt = pre.slot % a.kv.page_tokens;
  if (which == 1) {
    *(uint2 *)&pg[kv_k_off(h, tt, e, a.kv)] = pk;
  } else {
    for (int i = 0; i < 4; ++i) pg[kv_v_off(h, tt, e + i, a.kv)] = (bf16_t)f2bf(v[i]);
  }
}

template <>
__device__ inline void gemm_epilogue<EPI_RESID>(const GemmArgs &a, int row, int n0, floatx4 v, const EpiPre &pre) {
  if (n0 + 3 >= a.N || row >= a.rows) return;
  *(floatx4 *)&a.x[(long)row * a.N + n0] = pre.x + (v + pre.bias);
}

template <int MB, int R, int EPI, int U, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void k_gemm(GemmArgs a) {
  constexpr int RM = R * MB;
  extern __shared__ floatx4 red[];  // [WAVES][RM][64 lanes]
  // The wave index is the same in all lanes.  Saying so makes the loop conditions that depend on it scalar: as
  // (formally) divergent exits they make the compiler shuttle every accumulator between register files in each
  // iteration to keep the values of lanes that might have left the loop.
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int Kf = a.K >> 5;
  // K range of this workgroup, cut into buffers of U k-steps that are dealt
  // round-robin to the waves: at any moment the workgroup reads WAVES * U KiB
  // of consecutive addresses from each of its R weight-row streams.
  const int kw0 = (int)((long)Kf * blockIdx.y / a.split), kw1 = (int)((long)Kf * (blockIdx.y + 1) / a.split);
  const int nbuf = (kw1 - kw0) / U;  // the launcher picks U so that this is exact
  // weight tile T lives in tile group T / G at slot T % G; the G tiles of a group alternate per k-step
  const bf16x8 *Wl = (const bf16x8 *)a.W + lane;
  const long kstride = (long)a.G * 64;
  long woff[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int T = blockIdx.x * R + r;
    woff[r] = (((long)(T / a.G) * Kf + kw0) * a.G + T % a.G) * 64;
  }
  const int row0 = blockIdx.z * (MB * 16);  // chunk of activation rows (0 when decoding)
  const bf16x8 *Ab = (const bf16x8 *)a.A + ((long)blockIdx.z * MB * Kf + kw0) * 64 + act_lane(lane);

  floatx4 acc[R][MB];
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int m = 0; m < MB; ++m) acc[r][m] = floatx4{0.f, 0.f, 0.f, 0.f};

  bf16x8 w0[U][R], x0[U][MB], w1[U][R], x1[U][MB];
  auto load = [&](int j, bf16x8(&w)[U][R], bf16x8(&x)[U][MB]) {  // j-th buffer of the workgroup
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int r = 0; r < R; ++r) w[u][r] = __builtin_nontemporal_load(&Wl[woff[r] + (long)(j * U + u) * kstride]);
#pragma unroll
      for (int m = 0; m < MB; ++m) x[u][m] = Ab[((long)m * Kf + j * U + u) * 64];
    }
  };
  auto fma = [&](bf16x8(&w)[U][R], bf16x8(&x)[U][MB]) {
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int m = 0; m < MB; ++m)
          acc[r][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[u][r], x[u][m], acc[r][m], 0, 0, 0);
  };

  // epilogue operands of the (tile row, batch tile) pairs this wave will finish: fetched now when they are few,
  // else at the start of each reduction stage
  constexpr int RS = gemm_stage_rows(WAVES, R, MB);
  constexpr int NP = (RS * MB + WAVES - 1) / WAVES;
  constexpr bool EARLY = RS == R && NP <= 2;
  EpiPre pre[NP];
  auto fetch_pre = [&](int r0) {
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int p = wave + i * WAVES;
      const int r = r0 + p / MB, m = p % MB;
      if (p < RS * MB && r < R)
        pre[i] = epi_prefetch<EPI>(a, row0 + m * 16 + (lane & 15), (blockIdx.x * R + r) * 16 + 4 * (lane >> 4));
    }
  };
  if constexpr (EARLY) fetch_pre(0);

  // two register buffers: the loads of one are in flight while the MFMAs of the other issue
  // A wave beyond the last buffer (short K) streams buffer 0 with its weights zeroed, once: guarding the loop instead
  // makes the compiler keep two copies of the accumulators and move all of them between the copies every iteration.
  const bool idle = wave >= nbuf;
  int j = idle ? 0 : wave;
  load(j, w0, x0);
  if (idle) {
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int r = 0; r < R; ++r) w0[u][r] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
  }
  // Behind the conditional prefetch the compiler cannot count the loads in flight and makes the first MFMA of a
  // buffer wait for the prefetch as well, so a wave alone does not overlap its loads with its MFMAs: the other
  // waves of the CU do.  Measured with the prefetch made unconditional (exact wait counts, twice the bytes in
  // flight per wave): 2 % slower at 32 rows (8 waves per workgroup), faster only at 128 rows (4 waves).
  while (true) {
    const int j1 = j + WAVES, j2 = j + 2 * WAVES;
    if (j1 < nbuf) load(j1, w1, x1);
    fma(w0, x0);
    if (j1 >= nbuf) break;
    if (j2 < nbuf) load(j2, w0, x0);
    fma(w1, x1);
    if (j2 >= nbuf) break;
    j = j2;
  }

  // sum the waves' partial tiles in a fixed order (deterministic).  The LDS buffer holds RS of the R tile rows
  // at a time (64 KiB at most), so wide batches reduce in stages.
  constexpr int NST = (R + RS - 1) / RS;
  float cand_v[NST * NP];  // LM head: lanes 0..15 keep the best logit of each (tile row, batch row) they reduced
  int cand_i[NST * NP];
#pragma unroll
  for (int r0 = 0; r0 < R; r0 += RS) {
    if (r0) __syncthreads();  // the previous stage has been consumed
    if constexpr (!EARLY) fetch_pre(r0);
#pragma unroll
    for (int rr = 0; rr < RS; ++rr)
#pragma unroll
      for (int m = 0; m < MB; ++m)
        if (r0 + rr < R) red[(wave * (RS * MB) + rr * MB + m) * 64 + lane] = acc[r0 + rr < R ? r0 + rr : 0][m];
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int p = wave + i * WAVES;
      const int r = r0 + p / MB, m = p % MB;
      if (p < RS * MB && r < R) {
        floatx4 v = red[p * 64 + lane];
        for (int w = 1; w < WAVES; ++w) v += red[(w * (RS * MB) + p) * 64 + lane];
        const int n0 = (blockIdx.x * R + r) * 16 + 4 * (lane >> 4);
        if constexpr (EPI != EPI_LOGITS) {
          gemm_epilogue<EPI>(a, row0 + m * 16 + (lane & 15), n0, v, pre[i]);
        } else {
          // optional fp32 logits, and the largest of this tile row per batch row (lowest index on ties)
          const int b = m * 16 + (lane & 15);
          float best = -3.0e38f;
          int bi = 0x7fffffff;
          for (int j = 0; j < 4; ++j) {
            if (n0 + j < a.N) {
              if (a.logits && b < a.B) a.logits[(long)b * a.N + n0 + j] = v[j];
              if (v[j] > best) { best = v[j]; bi = n0 + j; }
            }
          }
          for (int o = 16; o < 64; o <<= 1) {  // across the four 4-row groups of this column
            const float ov = __shfl_xor(best, o);
            const int oi = __shfl_xor(bi, o);
            if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
          }
          cand_v[(r0 / RS) * NP + i] = best;
          cand_i[(r0 / RS) * NP + i] = bi;
        }
      }
    }
  }
  if constexpr (EPI == EPI_LOGITS) {
    __syncthreads();  // the reduction buffer is free: it now collects the candidates, [R * MB][16] values and indices
    float *cv = (float *)red;
    int *ci = (int *)red + RM * 16;
#pragma unroll
    for (int st = 0; st < NST; ++st)
#pragma unroll
      for (int i = 0; i < NP; ++i) {
        const int p = wave + i * WAVES;
        const int r = st * RS + p / MB, m = p % MB;
        if (p < RS * MB && r < R && lane < 16) {
          cv[(r * MB + m) * 16 + lane] = cand_v[st * NP + i];
          ci[(r * MB + m) * 16 + lane] = cand_i[st * NP + i];
        }
      }
    __syncthreads();
    if (threadIdx.x < MB * 16) {
      const int m = threadIdx.x >> 4, c = threadIdx.x & 15;
      float best = cv[m * 16 + c];
      int bi = ci[m * 16 + c];
      for (int r = 1; r < R; ++r) {
        const float ov = cv[(r * MB + m) * 16 + c];
        const int oi = ci[(r * MB + m) * 16 + c];
        if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
      }
      a.pmax[(long)blockIdx.x * a.B_pad + m * 16 + c] = best;
      a.pidx[(long)blockIdx.x * a.B_pad + m * 16 + c] = bi;
    }
  }
}

int bf16_gemm_groups(int N, int R) { return (N + 16 * R - 1) / (16 * R); }

template <int MB, int R, int U, int WAVES>
static void launch_gemm_epi(hipStream_t s, const GemmArgs &a, int epi, dim3 grid) {
  const size_t lds = (size_t)WAVES * gemm_stage_rows(WAVES, R, MB) * MB * 64 * sizeof(floatx4);
  const dim3 blk(WAVES * 64);
  switch (epi) {
    case EPI_PARTIAL: SKD_LAUNCH((k_gemm<MB, R, EPI_PARTIAL, U, WAVES>), grid, blk, lds, s, a); break;
    case EPI_QKV: SKD_LAUNCH((k_gemm<MB, R, EPI_QKV, U, WAVES>), grid, blk, lds, s, a); break;
    case EPI_RELU: SKD_LAUNCH((k_gemm<MB, R, EPI_RELU, U, WAVES>), grid, blk, lds, s, a); break;
    case EPI_QKV_ROWS:
      if constexpr (MB == 8) SKD_LAUNCH((k_gemm<MB, R, EPI_QKV_ROWS, U, WAVES>), grid, blk, lds, s, a);
      break;
    case EPI_RESID:
      if constexpr (MB == 8) SKD_LAUNCH((k_gemm<MB, R, EPI_RESID, U, WAVES>), grid, blk, lds, s, a);
      break;
    default: SKD_LAUNCH((k_gemm<MB, R, EPI_LOGITS, U, WAVES>), grid, blk, lds, s, a); break;
  }
}
template <int MB, int R, int U>
static void launch_gemm_w(hipStream_t s, const GemmArgs &a, int epi, int waves, dim3 grid) {
  // 8 batch tiles need 4-wave workgroups: with 8 waves (2 per SIMD, 256 registers each) the accumulators spill
  if constexpr (MB < 8) {
    if (waves >= 8) { launch_gemm_epi<MB, R, U, 8>(s, a, epi, grid); return; }
  }
  launch_gemm_epi<MB, R, U, 4>(s, a, epi, grid);
}
template <int MB, int R>
static void launch_gemm_u(hipStream_t s, const GemmArgs &a, int epi, int U, int waves, dim3 grid) {
  // register budget: R * MB accumulators plus two buffers of U * (R + MB) fragments, 4 VGPRs each (beyond 44
  // units the 8-wave instantiations spill)
  if constexpr (R * MB + 2 * 4 * (R + MB) <= 44) {
    if (U >= 4) { launch_gemm_w<MB, R, 4>(s, a, epi, waves, grid); return; }
  }
  if constexpr (R * MB + 2 * 2 * (R + MB) <= 44) {
    if (U >= 2) { launch_gemm_w<MB, R, 2>(s, a, epi, waves, grid); return; }
  }
  launch_gemm_w<MB, R, 1>(s, a, epi, waves, grid);
}
template <int MB>
static void launch_gemm_r(hipStream_t s, const GemmArgs &a, int epi, int R, int U, int waves, dim3 grid) {
  if (R == 1) launch_gemm_u<MB, 1>(s, a, epi, U, waves, grid);
  else if (R == 2) launch_gemm_u<MB, 2>(s, a, epi, U, waves, grid);
  else if (R == 3) launch_gemm_u<MB, 3>(s, a, epi, U, waves, grid);
  else launch_gemm_u<MB, 4>(s, a, epi, U, waves, grid);
}

// Batch tiles of 16 rows are compiled for B_pad in {16, 32, 64, 128}.
// Launch shape of a skinny GEMM, or false if the kernel cannot run it: nothing is launched here.
static bool gemm_shape(const GemmArgs &a, int epi, int R, int &U, int waves, dim3 &grid, int &groups) {
  const int MB = a.B_pad / 16;
  if (R < 1 || R > 4 || a.G < 1 || a.G > 4 || (waves != 4 && waves != 8)) return false;
  if (a.B_pad % 16 || (MB != 1 && MB != 2 && MB != 4 && MB != 8)) return false;
  if (a.K < 32 || a.K % 32 || a.N < 1) return false;
  const int split = epi == EPI_LOGITS ? 1 : a.split;
  const int Kf = a.K / 32;
  if (split < 1 || Kf % split) return false;  // equal K ranges per workgroup
  while (U > 1 && (Kf / split) % U) U >>= 1;  // whole buffers only
  if (U < 1) return false;
  groups = bf16_gemm_groups(a.N, R);
  const bool by_rows = epi == EPI_QKV_ROWS || epi == EPI_RESID || (epi == EPI_RELU && a.rows > 0);
  if ((epi == EPI_QKV_ROWS || epi == EPI_RESID) && (MB != 8 || a.rows <= 0)) return false;
  if (by_rows && (a.rows % a.B_pad || split != 1)) return false;
  grid = dim3(groups, split, by_rows ? a.rows / a.B_pad : 1);
  return true;
}

int bf16_gemm_check(const GemmArgs &a, int epi, int R, int U, int waves) {
  dim3 grid;
  int groups = 0;
  return gemm_shape(a, epi, R, U, waves, grid, groups) ? groups : -1;
}

int bf16_gemm(hipStream_t s, const GemmArgs &a, int epi, int R, int U, int waves) {
  dim3 grid;
  int groups = 0;
  if (!gemm_shape(a, epi, R, U, waves, grid, groups)) return -1;
  switch (a.B_pad / 16) {
    case 1: launch_gemm_r<1>(s, a, epi, R, U, waves, grid); break;
    case 2: launch_gemm_r<2>(s, a, epi, R, U, waves, grid); break;
    case 4: launch_gemm_r<4>(s, a, epi, R, U, waves, grid); break;
    default: launch_gemm_r<8>(s, a, epi, R, U, waves, grid); break;
  }
  return groups;
}

// ------------------------------------------------------------------ skinny GEMM for 128 batch rows
// With 8 batch tiles a workgroup pulls two bytes of activations out of L2 for every byte of weights it streams
// from HBM, and on this part a CU's vector memory path serves the two kinds of request largely one after the
// other: measured per CU with plain streaming waves, 512 KiB of HBM misses take 19.9 us and every further MiB of
// L2 hits adds 7.5 us when separate waves fetch it (12.7 us when the same four waves fetch both in turn, as the
// general kernel above does).  So the work is split by wave role:
//   waves 0..3 (one per SIMD) stream the weights into registers, three k-steps deep, and issue the MFMAs;
//   waves 4..7 fetch the activations with LDS-direct loads (no registers in flight) into a ring of four
//   stages; a stage holds the 8 activation fragments of 4 consecutive k-steps; wave 4 + w fetches the k-step
//   that wave w multiplies.  One bare s_barrier per stage orders the ring (as in the tiled prompt GEMM below).
// With a.ws_rot the workgroups start their K range at different stages (and wrap), so that at any moment the
// CUs of an XCD ask its L2 for different lines; the sum over k is then taken in that rotated order: fixed for a
// given launch shape, hence run-to-run deterministic, but not the same order in every workgroup (the caller leaves
// it off for the LM head, where identical vocabulary rows are to give identical logits).
constexpr int WS_NS = 4;  // ring stages
constexpr int WS_CW = 4;  // MFMA waves = loader waves = k-steps per stage
constexpr int WS_MB = 8;  // batch tiles

template <int R, int EPI>
__global__ __launch_bounds__(512) void k_gemm_ws(GemmArgs a) {
  constexpr int MB = WS_MB, NS = WS_NS;
  constexpr int STAGE = WS_CW * MB * 64;     // bf16x8 units per stage (32 KiB)
  extern __shared__ bf16x8 ws_lds[];         // ring [NS][WS_CW][MB][64 lanes]; later the reduction buffer
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int Kf = a.K >> 5;
  const int kw0 = (int)((long)Kf * blockIdx.y / a.split), kw1 = (int)((long)Kf * (blockIdx.y + 1) / a.split);
  const int nchunk = (kw1 - kw0) / WS_CW;  // the launcher makes this exact and >= 1
  const int rot = a.ws_rot ? (int)((blockIdx.x >> 3) * 5u + blockIdx.y * 3u) % nchunk : 0;
  floatx4 *red = (floatx4 *)ws_lds;        // [WS_CW][R * MB][64 lanes] after the main loop
  auto bar = [&]() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };

  if (wave >= WS_CW) {
    // ---- loader of k-step kw0 + 4 * chunk + l of every stage
    const int l = wave - WS_CW;
    const bf16x8 *Ab = (const bf16x8 *)a.A + act_lane(lane);  // fetched in MFMA lane order: LDS holds ready-made fragments
    auto issue = [&](int ci) {
      int c = ci + rot;
      if (c >= nchunk) c -= nchunk;
      const long kf = kw0 + c * WS_CW + l;
      bf16x8 *dst = ws_lds + (ci % NS) * STAGE + l * (MB * 64);
#pragma unroll
      for (int m = 0; m < MB; ++m)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(Ab + ((long)m * Kf + kf) * 64),
                                         (__attribute__((address_space(3))) void *)(dst + m * 64), 16, 0, 0);
    };
#pragma unroll
    for (int i = 0; i < NS - 1; ++i)
      if (i < nchunk) issue(i);
    for (int ci = 0; ci < nchunk; ++ci) {
      // this wave's 8 loads of stage ci have landed once only those of the (up to two) later stages in flight
      // are outstanding (vector-memory operations of a wave complete in order)
      const int later = min(nchunk - 1 - ci, NS - 2);
      if (later == 0) __builtin_amdgcn_s_waitcnt(0x0F70);       // vmcnt = 0
      else if (later == 1) __builtin_amdgcn_s_waitcnt(0x0F78);  // vmcnt <= 8
      else __builtin_amdgcn_s_waitcnt(0x4F70);                  // vmcnt <= 16
      bar();  // stage ci is complete; every wave has finished reading stage ci - 1
      if (ci + NS - 1 < nchunk) issue(ci + NS - 1);  // into the slot of stage ci - 1
    }
    bar();  // every stage has been read: the ring becomes the reduction buffer
  } else {
    // ---- weight streamer + MFMA: k-step kw0 + 4 * chunk + wave of every stage
    floatx4 acc[R][MB];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int m = 0; m < MB; ++m) acc[r][m] = floatx4{0.f, 0.f, 0.f, 0.f};
    // addresses = wave-uniform base (scalar registers) + the lane's 32-bit offset: no 64-bit vector address
    // arithmetic, no address registers shared with the fragments in flight
    const bf16x8 *Wu = (const bf16x8 *)a.W;
    long wbase[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int T = blockIdx.x * R + r;
      wbase[r] = (((long)(T / a.G) * Kf + kw0 + wave) * a.G + T % a.G) * 64;
    }
    const long cstride = (long)a.G * 64 * WS_CW;  // one stage further along K
    const unsigned ulane = (unsigned)lane;
    auto loadw = [&](int ci, bf16x8(&w)[R]) {
      int c = ci + rot;
      if (c >= nchunk) c -= nchunk;
#pragma unroll
      for (int r = 0; r < R; ++r) w[r] = __builtin_nontemporal_load(&(Wu + (wbase[r] + c * cstride))[ulane]);
    };
    auto step = [&](int ci, bf16x8(&w)[R]) {
      bar();
      const bf16x8 *fs = ws_lds + (ci % NS) * STAGE + wave * (MB * 64) + lane;
      bf16x8 x[MB];
#pragma unroll
      for (int m = 0; m < MB; ++m) x[m] = fs[m * 64];
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int m = 0; m < MB; ++m) acc[r][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[r], x[m], acc[r][m], 0, 0, 0);
    };
    // three k-steps of weights in flight; the prefetches are unconditional (index clamped to the last stage,
    // which is then fetched again and not used), so that the compiler can count the loads in flight, and fenced
    // so that they stay ahead of the MFMAs they overlap with
    bf16x8 w0[R], w1[R], w2[R];
    const int cl = nchunk - 1;
    loadw(0, w0);
    loadw(min(1, cl), w1);
    // One stage: prefetch the weights two stages ahead into the buffer that came free, then multiply.  Twelve stages
    // per trip of the loop (the three buffers rotate four times): at the loop's head the compiler waits for every
    // load in flight, which costs the prefetch once per trip (measured effect of 12 instead of 3 stages per trip:
    // under 1 %).
#define SKD_WS_STAGE(k, wuse, wload)                     \
  loadw(min(ci + (k) + 2, cl), wload);                   \
  __builtin_amdgcn_sched_barrier(0);                     \
  step(ci + (k), wuse);                                  \
  __builtin_amdgcn_sched_barrier(0);                     \
  if (ci + (k) + 1 >= nchunk) break;
    int ci = 0;
    while (true) {
      SKD_WS_STAGE(0, w0, w2) SKD_WS_STAGE(1, w1, w0) SKD_WS_STAGE(2, w2, w1)
      SKD_WS_STAGE(3, w0, w2) SKD_WS_STAGE(4, w1, w0) SKD_WS_STAGE(5, w2, w1)
      SKD_WS_STAGE(6, w0, w2) SKD_WS_STAGE(7, w1, w0) SKD_WS_STAGE(8, w2, w1)
      SKD_WS_STAGE(9, w0, w2) SKD_WS_STAGE(10, w1, w0) SKD_WS_STAGE(11, w2, w1)
      ci += 12;
    }
#undef SKD_WS_STAGE
    bar();  // all waves are done with the ring
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int m = 0; m < MB; ++m) red[(wave * (R * MB) + r * MB + m) * 64 + lane] = acc[r][m];
  }

  // ---- sum the four MFMA waves' tiles in a fixed order; all eight waves share the epilogue work
  constexpr int NW = 2 * WS_CW;
  constexpr int NP = (R * MB + NW - 1) / NW;
  EpiPre pre[NP];
#pragma unroll
  for (int i = 0; i < NP; ++i) {
    const int p = wave + i * NW;
    if (p < R * MB) pre[i] = epi_prefetch<EPI>(a, (p % MB) * 16 + (lane & 15), (blockIdx.x * R + p / MB) * 16 + 4 * (lane >> 4));
  }
  __syncthreads();
  float cand_v[NP];
  int cand_i[NP];
#pragma unroll
  for (int i = 0; i < NP; ++i) {
    const int p = wave + i * NW;
    const int r = p / MB, m = p % MB;
    if (p < R * MB) {
      floatx4 v = red[p * 64 + lane];
      for (int w = 1; w < WS_CW; ++w) v += red[(w * (R * MB) + p) * 64 + lane];
      const int n0 = (blockIdx.x * R + r) * 16 + 4 * (lane >> 4);
      if constexpr (EPI != EPI_LOGITS) {
        gemm_epilogue<EPI>(a, m * 16 + (lane & 15), n0, v, pre[i]);
      } else {
        const int b = m * 16 + (lane & 15);
        float best = -3.0e38f;
        int bi = 0x7fffffff;
        for (int j = 0; j < 4; ++j) {
          if (n0 + j < a.N) {
            if (a.logits && b < a.B) a.logits[(long)b * a.N + n0 + j] = v[j];
            if (v[j] > best) { best = v[j]; bi = n0 + j; }
          }
        }
        for (int o = 16; o < 64; o <<= 1) {
          const float ov = __shfl_xor(best, o);
          const int oi = __shfl_xor(bi, o);
          if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
        }
        cand_v[i] = best;
        cand_i[i] = bi;
      }
    }
  }
  if constexpr (EPI == EPI_LOGITS) {
    __syncthreads();  // the reduction buffer is free: it now collects the candidates, [R * MB][16] values and indices
    float *cv = (float *)ws_lds;
    int *ci = (int *)ws_lds + R * MB * 16;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int p = wave + i * NW;
      if (p < R * MB && lane < 16) {
        cv[p * 16 + lane] = cand_v[i];
        ci[p * 16 + lane] = cand_i[i];
      }
    }
    __syncthreads();
    if (threadIdx.x < MB * 16) {
      const int m = threadIdx.x >> 4, c = threadIdx.x & 15;
      float best = cv[m * 16 + c];
      int bi = ci[m * 16 + c];
      for (int r = 1; r < R; ++r) {
        const float ov = cv[(r * MB + m) * 16 + c];
        const int oi = ci[(r * MB + m) * 16 + c];
        if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
      }
      a.pmax[(long)blockIdx.x * a.B_pad + m * 16 + c] = best;
      a.pidx[(long)blockIdx.x * a.B_pad + m * 16 + c] = bi;
    }
  }
}

// Decode projections at 128 (padded) batch rows on the wave-specialised kernel.  Returns the number of row groups,
// or -1 when the shape is not one it handles (the caller then uses bf16_gemm); nothing is launched in that case.
static bool gemm_ws_shape(const GemmArgs &a, int epi, int R, dim3 &grid, int &groups) {
  if (a.B_pad != 128 || a.rows != 0 || R < 1 || R > 4 || a.G < 1 || a.G > 4 || a.K < 32 || a.K % 32 || a.N < 1) return false;
  if (epi != EPI_PARTIAL && epi != EPI_QKV && epi != EPI_RELU && epi != EPI_LOGITS) return false;
  const int split = epi == EPI_LOGITS ? 1 : a.split;
  const int Kf = a.K / 32;
  if (split < 1 || Kf % split || (Kf / split) % WS_CW || Kf / split < WS_CW) return false;
  groups = bf16_gemm_groups(a.N, R);
  grid = dim3(groups, split, 1);
  return true;
}
int bf16_gemm_ws_check(const GemmArgs &a, int epi, int R) {
  dim3 grid;
  int groups = 0;
  return gemm_ws_shape(a, epi, R, grid, groups) ? groups : -1;
}
template <int R>
static int launch_gemm_ws(hipStream_t s, const GemmArgs &a, int epi, dim3 grid) {
  // the activation ring (4 stages of 32 KiB), reused for the cross-wave reduction (4 waves x R x 8 KiB): 128 KiB
  constexpr size_t ring = (size_t)WS_NS * WS_CW * WS_MB * 64 * sizeof(bf16x8);
  constexpr size_t redb = (size_t)WS_CW * R * WS_MB * 64 * sizeof(floatx4);
  constexpr size_t lds = ring > redb ? ring : redb;
  static bool configured = false;
  if (!configured) {
    if (hipFuncSetAttribute((const void *)k_gemm_ws<R, EPI_PARTIAL>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess ||
        hipFuncSetAttribute((const void *)k_gemm_ws<R, EPI_QKV>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess ||
        hipFuncSetAttribute((const void *)k_gemm_ws<R, EPI_RELU>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess ||
        hipFuncSetAttribute((const void *)k_gemm_ws<R, EPI_LOGITS>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return -1;
    configured = true;
  }
  const dim3 blk(512);
  switch (epi) {
    case EPI_PARTIAL: SKD_LAUNCH((k_gemm_ws<R, EPI_PARTIAL>), grid, blk, lds, s, a); break;
    case EPI_QKV: SKD_LAUNCH((k_gemm_ws<R, EPI_QKV>), grid, blk, lds, s, a); break;
    case EPI_RELU: SKD_LAUNCH((k_gemm_ws<R, EPI_RELU>), grid, blk, lds, s, a); break;
    default: SKD_LAUNCH((k_gemm_ws<R, EPI_LOGITS>), grid, blk, lds, s, a); break;
  }
  return 0;
}
int bf16_gemm_ws(hipStream_t s, const GemmArgs &a, int epi, int R) {
  dim3 grid;
  int groups = 0;
  if (!gemm_ws_shape(a, epi, R, grid, groups)) return -1;
  int rc;
  if (R == 1) rc = launch_gemm_ws<1>(s, a, epi, grid);
  else if (R == 2) rc = launch_gemm_ws<2>(s, a, epi, grid);
  else if (R == 3) rc = launch_gemm_ws<3>(s, a, epi, grid);
  else rc = launch_gemm_ws<4>(s, a, epi, grid);
  return rc < 0 ? -1 : groups;
}

// ------------------------------------------------------------------ tiled GEMM for the batched prompt
// With thousands of activation rows the projections are compute-bound, and the
// skinny kernel above (every wave fetching its own operands) is limited by
// L2-to-CU traffic.  Here a workgroup of 8 waves owns a 256 x 256 output tile
// (16 weight tiles x 16 activation-row tiles).  The operand fragments of one
// k-step (32 KiB) form a stage; a ring of 4 stages lives in LDS and is filled by
// LDS-direct global loads (each lane supplies a global address, its 16 bytes
// land at the wave's LDS base + 16 * lane: fragments arrive ready-made and no
// register holds data in flight), three stages ahead of the one being
// multiplied.  Each wave accumulates a 64 x 128 sub-tile (4 x 8 MFMA tiles, 128
// accumulator registers), reading 12 fragments from LDS per 32 MFMAs, one
// k-step ahead of the MFMAs that use them.
constexpr int TILE_NS = 4;   // ring stages
constexpr int TILE_FR = 32;  // fragments per stage: 16 weight tiles, then 16 activation-row tiles

// wait until at most n of this wave's vector-memory operations are outstanding (they complete in order)
__device__ inline void wait_vmcnt_le(int n) {
  switch (n) {  // s_waitcnt immediate: vmcnt in bits 3:0 (and 15:14), no wait on the export and LDS counters
    case 0: __builtin_amdgcn_s_waitcnt(0x0F70); break;
    case 4: __builtin_amdgcn_s_waitcnt(0x0F74); break;
    default: __builtin_amdgcn_s_waitcnt(0x0F78); break;  // 8
  }
}

template <int EPI>
__global__ __launch_bounds__(512) void k_gemm_tile(GemmArgs a) {
  extern __shared__ bf16x8 tile_lds[];  // [TILE_NS stages][TILE_FR][64 lanes]
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int wr = wave >> 1, wc = wave & 1;  // sub-tile: weight tiles 4wr .. 4wr+3, activation tiles 8wc .. 8wc+7
  const int Kf = a.K >> 5;

  // workgroup -> output tile.  Workgroups are dealt to the 8 XCDs round-robin; the ones that share an XCD (and
  // its L2) at any moment should share operands, so each XCD walks its own contiguous range of tiles in bands
  // of 4 activation tiles x all weight tiles, weight tile fastest in groups of 4 rows (the last band has the
  // gy % 4 activation tiles that are left; XCD x owns the workgroups with id % 8 == x, one more than the others
  // when x < total % 8).
  int tn, tm;
  {
    const int gx = gridDim.x, gy = gridDim.y, total = gx * gy;
    const int id = blockIdx.x + gx * blockIdx.y;
    const int xcd = id & 7, per = total >> 3, rem = total & 7;
    const int logical = xcd * per + min(xcd, rem) + (id >> 3);
    const int full = gy >> 2, tail0 = full * 4 * gx;
    if (logical < tail0) {
      const int band = logical / (4 * gx), within = logical - band * 4 * gx;
      tn = within >> 2;
      tm = band * 4 + (within & 3);
    } else {
      const int hb = gy & 3, within = logical - tail0;  // hb > 0 here
      tn = within / hb;
      tm = full * 4 + within % hb;
    }
  }

  // this wave's share of a stage: 4 fragments; waves 0..3 fetch the weight tiles, waves 4..7 the activation tiles.
  // Fragment bases are wave-uniform (scalar registers); the only per-lane part of an address is the lane's place
  // in the fragment, one 32-bit register.
  const int ld_is_a = wave >> 2, ld_t0 = (wave & 3) * 4;
  const bf16x8 *src[4];
  long sstride;
  unsigned vlane;
  if (!ld_is_a) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int T = tn * 16 + ld_t0 + i;
      src[i] = (const bf16x8 *)a.W + (((long)(T / a.G) * Kf) * a.G + T % a.G) * 64;
    }
    sstride = (long)a.G * 64;
    vlane = lane;
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) src[i] = (const bf16x8 *)a.A + ((long)(tm * 16 + ld_t0 + i) * Kf) * 64;
    sstride = 64;
    vlane = act_lane(lane);  // fetched in MFMA lane order, so that LDS holds ready-made fragments
  }
  const int dfrag = ld_is_a * 16 + ld_t0;

  floatx4 acc[4][8];
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int m = 0; m < 8; ++m) acc[r][m] = floatx4{0.f, 0.f, 0.f, 0.f};

  auto issue = [&](int st) {  // 4 vector-memory operations per wave and stage
    bf16x8 *dst = tile_lds + ((st % TILE_NS) * TILE_FR + dfrag) * 64;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)&(src[i] + (long)st * sstride)[vlane],
                                       (__attribute__((address_space(3))) void *)(dst + i * 64), 16, 0, 0);
  };
  auto read = [&](int buf, bf16x8(&wf)[4], bf16x8(&xf)[8]) {  // 12 fragments of a stage into registers
    const bf16x8 *base = tile_lds + buf * (TILE_FR * 64) + lane;
#pragma unroll
    for (int r = 0; r < 4; ++r) wf[r] = base[(wr * 4 + r) * 64];
#pragma unroll
    for (int m = 0; m < 8; ++m) xf[m] = base[(16 + wc * 8 + m) * 64];
  };
  auto mma = [&](const bf16x8(&wf)[4], const bf16x8(&xf)[8]) {
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int m = 0; m < 8; ++m) acc[r][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[r], xf[m], acc[r][m], 0, 0, 0);
  };
  // Stage st becomes readable.  This wave's loads of it have landed once at most the loads of the (up to two)
  // later stages in flight are outstanding, and its own LDS reads (of stage st - 1) have completed; the barrier
  // then says both of every wave, so stage st may be read and the ring slot of stage st - 1 refilled.  It is a
  // bare s_barrier between compiler fences: __syncthreads() would also wait for the loads of the later stages.
  auto open_stage = [&](int st) {
    const int later = min(Kf - 1 - st, TILE_NS - 2);
    wait_vmcnt_le(4 * later);
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (st + TILE_NS - 1 < Kf) issue(st + TILE_NS - 1);
  };

#pragma unroll
  for (int i = 0; i < TILE_NS - 1; ++i)
    if (i < Kf) issue(i);
  // Two register sets of fragments: while the matrix cores work on stage st out of one, the LDS reads of stage
  // st + 1 fill the other.  With one set, every k-step began with all 8 waves waiting for 96 KiB of LDS reads
  // (the barrier puts them in phase) while the matrix cores sat idle.
  bf16x8 wfA[4], xfA[8], wfB[4], xfB[8];
  open_stage(0);
  read(0, wfA, xfA);
  // Steady state (three later stages still to be requested): one straight-line block per k-step, in which the
  // scheduler is told to deal the 12 LDS reads of the next stage out among the 32 MFMAs of the current one, so
  // that a wave does not sit on a full LDS queue with MFMAs ready behind it (instructions issue in order).
  auto steady = [&](int nx, bf16x8(&wn)[4], bf16x8(&xn)[8], const bf16x8(&wc_)[4], const bf16x8(&xc)[8]) {
    wait_vmcnt_le(8);
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    issue(nx + TILE_NS - 1);
    read(nx % TILE_NS, wn, xn);
    mma(wc_, xc);
    __builtin_amdgcn_sched_group_barrier(0x020, 4, 0);  // the 4 LDS-direct loads first
#pragma unroll
    for (int i = 0; i < 4; ++i) {  // the reads early: (MFMA, read) x 4, (MFMA x 2, read) x 8, then 12 MFMAs, so that
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // no read is still in flight when the wave reaches the
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // next barrier
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 12, 0);
  };
  int st = 0;
  for (; st + 5 < Kf; st += 2) {
    steady(st + 1, wfB, xfB, wfA, xfA);
    steady(st + 2, wfA, xfA, wfB, xfB);
  }
  for (; st < Kf; st += 2) {  // the last stages, where waits and requests depend on what is left
    if (st + 1 < Kf) {
      open_stage(st + 1);
      read((st + 1) % TILE_NS, wfB, xfB);
    }
    __builtin_amdgcn_sched_barrier(0);
    mma(wfA, xfA);
    if (st + 1 < Kf) {
      if (st + 2 < Kf) {
        open_stage(st + 2);
        read((st + 2) % TILE_NS, wfA, xfA);
      }
      __builtin_amdgcn_sched_barrier(0);
      mma(wfB, xfB);
    }
  }

  // ---- epilogue.  acc[r][m]: lane l holds output rows (weight rows) n0 .. n0 + 3 of activation row
  // row0(m) + (l & 15), n0 = 16 * (weight tile) + 4 * (l >> 4).
  const int grp = lane >> 4, j = lane & 15;
  auto n0_of = [&](int r) { return ((tn * 16 + wr * 4 + r) << 4) + 4 * grp; };
  auto row0_of = [&](int m) { return (tm * 16 + wc * 8 + m) << 4; };
  if constexpr (EPI == EPI_RELU) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int n0 = n0_of(r);
      EpiPre pre;
      pre.bias = *(const floatx4 *)&a.bias[n0];
#pragma unroll
      for (int m = 0; m < 8; ++m) gemm_epilogue<EPI>(a, row0_of(m) + j, n0, acc[r][m], pre);
    }
  } else if constexpr (EPI == EPI_RESID) {
    // the residual values of the next weight tile are requested before the current one is stored: one exposed
    // round trip per workgroup instead of four
    floatx4 xv[2][8];
    auto fetch = [&](int r, floatx4(&x)[8]) {
#pragma unroll
      for (int m = 0; m < 8; ++m) x[m] = *(const floatx4 *)&a.x[(long)(row0_of(m) + j) * a.N + n0_of(r)];
    };
    auto store = [&](int r, const floatx4(&x)[8]) {
      const floatx4 bias = *(const floatx4 *)&a.bias[n0_of(r)];
#pragma unroll
      for (int m = 0; m < 8; ++m) *(floatx4 *)&a.x[(long)(row0_of(m) + j) * a.N + n0_of(r)] = x[m] + (acc[r][m] + bias);
    };
    fetch(0, xv[0]);
    fetch(1, xv[1]);
    store(0, xv[0]);
    fetch(2, xv[0]);
    store(1, xv[1]);
    fetch(3, xv[1]);
    store(2, xv[0]);
    store(3, xv[1]);
  } else {  // EPI_QKV_ROWS
    // The 256 output rows of a workgroup lie inside one of q | k | v (d is a multiple of 256 when 3 d is), and the
    // 16 activation rows of a tile belong to one sequence and one page: what the stores need to know about a tile
    // is wave-uniform and is looked up once, with scalar loads, not once per weight tile and lane.
    const int which = (tn * 256) / a.d;
    int t_page[8], t_slot0[8], t_len[8];
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      t_page[m] = -1;
      t_slot0[m] = 0;
      t_len[m] = 0;
      const int row0 = row0_of(m);
      if (which != 0 && row0 < a.rows) {
        const int b = a.rm.seq[row0];
        if (b >= 0) {
          t_slot0[m] = row0 - a.rm.first_row[b];  // = real position of the tile's first row
          t_len[m] = a.rm.P - a.rm.start[b];      // positions of the sequence; the rest of its last tile is padding
          if (t_slot0[m] < t_len[m]) t_page[m] = a.bt_layer[(long)b * a.kv.max_pages + t_slot0[m] / a.kv.page_tokens];
        }
      }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int n0 = n0_of(r), within = n0 - which * a.d;
      const floatx4 bias = *(const floatx4 *)&a.bias[n0];
      const int h = within / a.kv.dh, e = within - h * a.kv.dh;
#pragma unroll
      for (int m = 0; m < 8; ++m) {
        floatx4 v = acc[r][m] + bias;
        if (which == 0) {
          if (row0_of(m) < a.rows)
            *(uint2 *)&a.q_out[d_act_index(row0_of(m) + j, within, a.d)] = make_uint2(pack2(v[0], v[1]), pack2(v[2], v[3]));
          continue;
        }
        if (t_page[m] < 0) continue;
        bf16_t *pg = a.kv_pool + (long)t_page[m] * a.kv.page_elems;
        const int tt = (t_slot0[m] + j) % a.kv.page_tokens;
        if (which == 1) {
          if (t_slot0[m] + j < t_len[m])
            *(uint2 *)&pg[kv_k_off(h, tt, e, a.kv)] = make_uint2(pack2(v[0], v[1]), pack2(v[2], v[3]));
          continue;
        }
        // v: a page holds, for one element e, four consecutive positions side by side.  The four lanes of a quad
        // hold positions 4q .. 4q + 3 for elements e .. e + 3 each: transposed inside the quad (two exchanges,
        // with the lane 1 and the lane 2 away), lane t ends up with element e + t of all four positions and
        // stores them as one 8-byte word.
        const int t = j & 3;
        {
          const float s0 = (t & 1) ? v[0] : v[1], s1 = (t & 1) ? v[2] : v[3];
          const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, s0), 0xB1, 0xF, 0xF, true));
          const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, s1), 0xB1, 0xF, 0xF, true));
          if (t & 1) { v[0] = r0; v[2] = r1; } else { v[1] = r0; v[3] = r1; }
        }
        {
          const float s0 = (t & 2) ? v[0] : v[2], s1 = (t & 2) ? v[1] : v[3];
          const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, s0), 0x4E, 0xF, 0xF, true));
          const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, s1), 0x4E, 0xF, 0xF, true));
          if (t & 2) { v[0] = r0; v[1] = r1; } else { v[2] = r0; v[3] = r1; }
        }
        // now v[s] = element e + t of position 4 * (j / 4) + s
        const int pos0 = t_slot0[m] + (j & ~3), nvalid = t_len[m] - pos0;
        bf16_t *dst = &pg[kv_v_off(h, pos0 % a.kv.page_tokens, e + t, a.kv)];
        if (nvalid >= 4) {
          *(uint2 *)dst = make_uint2(pack2(v[0], v[1]), pack2(v[2], v[3]));
        } else {
          for (int s_ = 0; s_ < 4; ++s_)
            if (s_ < nvalid) dst[s_] = (bf16_t)f2bf(v[s_]);
        }
        (void)tt;
      }
    }
  }
}

// Batched-prompt projections on 256 x 256 tiles.  Returns 0, or -1 when the shape does not tile (the caller then
// uses bf16_gemm on row chunks).
int bf16_gemm_tile(hipStream_t s, const GemmArgs &a, int epi) {
  if (a.rows <= 0 || a.rows % 256 || a.N % 256 || a.K % 32 || a.G < 1 || a.G > 4) return -1;
  const dim3 grid(a.N / 256, a.rows / 256), blk(512);
  const size_t lds = (size_t)TILE_NS * TILE_FR * 64 * sizeof(bf16x8);  // 128 KiB of the CU's 160
  static bool configured = false;
  if (!configured) {
    if (hipFuncSetAttribute((const void *)k_gemm_tile<EPI_QKV_ROWS>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess ||
        hipFuncSetAttribute((const void *)k_gemm_tile<EPI_RESID>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess ||
        hipFuncSetAttribute((const void *)k_gemm_tile<EPI_RELU>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return -1;
    configured = true;
  }
  switch (epi) {
    case EPI_QKV_ROWS: SKD_LAUNCH(k_gemm_tile<EPI_QKV_ROWS>, grid, blk, lds, s, a); break;
    case EPI_RESID: SKD_LAUNCH(k_gemm_tile<EPI_RESID>, grid, blk, lds, s, a); break;
    case EPI_RELU: SKD_LAUNCH(k_gemm_tile<EPI_RELU>, grid, blk, lds, s, a); break;
    default: return -1;
  }
  return 0;
}

// ------------------------------------------------------------------ row kernels: embedding / split-K reduce, + LayerNorm
// One workgroup per batch row, one thread per float4 chunk up to 1024 threads.  These kernels move < 5 MB and are
// pure latency chains, so each thread keeps its share of the row in registers
// (float4 chunk c = threadIdx.x + blockDim.x * i, rows up to 16384 wide), issues
// every global load it will ever need up front, and the row never touches LDS.
constexpr int LN_NC = 4;

// v[i] = elements 4c .. 4c+3 of row b.  LayerNorm (mean, biased variance, eps 1e-5) -> bf16 row of the activation tiles.
__device__ inline void ln_finish_row(const floatx4 (&v)[LN_NC], const floatx4 (&gv)[LN_NC], const floatx4 (&bv)[LN_NC],
                                     int d, int b, bf16_t *a_out, float *sh) {
  const int d4 = d >> 2;
  float s = 0;
#pragma unroll
  for (int i = 0; i < LN_NC; ++i)
    if ((int)(threadIdx.x + blockDim.x * i) < d4) s += (v[i][0] + v[i][1]) + (v[i][2] + v[i][3]);
  const float mean = block_sum_once(s, sh) / d;  // sh: 32 floats, one half per reduction, so two barriers in all
  float q = 0;
#pragma unroll
  for (int i = 0; i < LN_NC; ++i)
    if ((int)(threadIdx.x + blockDim.x * i) < d4) {
      const floatx4 t = v[i] - mean;
      q += (t[0] * t[0] + t[1] * t[1]) + (t[2] * t[2] + t[3] * t[3]);
    }
  const float rstd = 1.0f / sqrtf(block_sum_once(q, sh + 16) / d + 1e-5f);
#pragma unroll
  for (int i = 0; i < LN_NC; ++i) {
    const int c = (int)(threadIdx.x + blockDim.x * i);
    if (c < d4) {
      const floatx4 y = (v[i] - mean) * rstd * gv[i] + bv[i];
      *(uint2 *)&a_out[d_act_index(b, 4 * c, d)] = make_uint2(pack2(y[0], y[1]), pack2(y[2], y[3]));
    }
  }
}

// threads of a row workgroup: one per float4 chunk, whole waves, at most 1024 (narrow rows: fewer waves at the barriers)
static int row_threads(int d) { return d / 4 >= 1024 ? 1024 : (d / 4 + 63) / 64 * 64; }

__global__ __launch_bounds__(1024) void k_embed_ln(const int32_t *tokens, const int32_t *start, int t,
                                                   const bf16_t *tok_emb, const bf16_t *pos_emb, const float *g,
                                                   const float *bt, float *x, bf16_t *a_out, int d, int V) {
  __shared__ float sh[32];
  const int b = blockIdx.x, d4 = d >> 2;
  int tok = tokens[b];
  tok = tok < 0 ? 0 : (tok >= V ? V - 1 : tok);
  int pos = t - start[b];  // number of real tokens before this column
  if (pos < 0) pos = 0;    // padding column, never attended to
  const uint2 *te = (const uint2 *)(tok_emb + (long)tok * d), *pe = (const uint2 *)(pos_emb + (long)pos * d);
  floatx4 v[LN_NC], gv[LN_NC], bv[LN_NC];
#pragma unroll
  for (int i = 0; i < LN_NC; ++i) {
    const int c = (int)(threadIdx.x + blockDim.x * i);
    if (c < d4) {
      const uint2 a = te[c], p = pe[c];
      gv[i] = ((const floatx4 *)g)[c];
      bv[i] = ((const floatx4 *)bt)[c];
      v[i] = floatx4{bf2f(a.x & 0xffffu) + bf2f(p.x & 0xffffu), bf2f(a.x >> 16) + bf2f(p.x >> 16),
                     bf2f(a.y & 0xffffu) + bf2f(p.y & 0xffffu), bf2f(a.y >> 16) + bf2f(p.y >> 16)};
      ((floatx4 *)x)[(long)b * d4 + c] = v[i];
    }
  }
  ln_finish_row(v, gv, bv, d, b, a_out, sh);
}

void bf16_embed_ln(hipStream_t s, const int32_t *tokens, const int32_t *start, int t, const bf16_t *tok_emb,
                   const bf16_t *pos_emb, const float *g, const float *b, float *x, bf16_t *a_out, int B, int d,
                   int V) {
  SKD_LAUNCH(k_embed_ln, dim3(B), dim3(row_threads(d)), 0, s, tokens, start, t, tok_emb, pos_emb, g, b, x, a_out, d, V);
}

// x[b][:] += bias + sum_s partial[s][b][:] (fixed order), then LayerNorm
__global__ __launch_bounds__(1024) void k_reduce_ln(const float *partial, int split, int B_pad, const float *bias,
                                                    float *x, const float *g, const float *bt, bf16_t *a_out, int d) {
  __shared__ float sh[32];
  const int b = blockIdx.x, d4 = d >> 2;
  const floatx4 *p4 = (const floatx4 *)partial;
  floatx4 *x4 = (floatx4 *)x + (long)b * d4;
  floatx4 v[LN_NC], gv[LN_NC], bv[LN_NC];
#pragma unroll
  for (int i = 0; i < LN_NC; ++i) {
    const int c = (int)(threadIdx.x + blockDim.x * i);
    if (c < d4) {
      const floatx4 xv = x4[c], bias4 = ((const floatx4 *)bias)[c];
      gv[i] = ((const floatx4 *)g)[c];
      bv[i] = ((const floatx4 *)bt)[c];
      floatx4 acc = p4[(long)b * d4 + c];
#pragma unroll 8
      for (int sp = 1; sp < split; ++sp) acc += p4[((long)sp * B_pad + b) * d4 + c];
      v[i] = xv + (acc + bias4);
      x4[c] = v[i];
    }
  }
  ln_finish_row(v, gv, bv, d, b, a_out, sh);
}

void bf16_reduce_ln(hipStream_t s, const float *partial, int split, int B_pad, const float *bias, float *x,
                    const float *g, const float *b, bf16_t *a_out, int B, int d) {
  SKD_LAUNCH(k_reduce_ln, dim3(B), dim3(row_threads(d)), 0, s, partial, split, B_pad, bias, x, g, b, a_out, d);
}

// ------------------------------------------------------------------ decode attention over the paged KV cache
// One workgroup of NW waves (1, 2, 4, 8 or 16) per (row, head, split).  Wave w takes
// 32-key blocks first + w, first + w + NW, ...; each block is 2 K tiles (QK^T:
// 2 * DH/32 MFMAs, q replicated over the 16 MFMA columns) and one V block
// (DH/16 MFMAs).  Online softmax per wave in fp32; the waves (and, with
// splits > 1, the workgroups of one head) are merged with the usual max / sum
// rescaling.  Batches with few (row, head) pairs get their 16 waves per CU from
// wider workgroups rather than from splits, which need a second kernel.
// Four waves per SIMD are required: with three the kernel is 13 % slower.
template <int DH, int NW>
__global__ __launch_bounds__(NW * 64, 4) void k_attention(AttnArgs a) {  // 4 waves per SIMD whatever the workgroup width
  constexpr int QC = DH / 32, VM = DH / 16;
  __shared__ float sm_m[NW], sm_l[NW], sm_dot[NW];
  __shared__ float sm_o[NW][DH];
  // uniform wave index: block numbers, page lookups and block addresses become scalar work
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, grp = lane >> 4;
  const int H = a.kv.H, h = blockIdx.x % H, d = H * DH;
  // longest rows are dispatched first, so that the last workgroups to start are the short ones
  const int b = a.order ? a.order[blockIdx.x / H] : (int)(blockIdx.x / H);
  const int j0 = a.start[b], t = a.t;
  // a row's keys are stored by real position: column j sits in slot j - j0, so neither end of the row's first
  // block is padding.  Slots 0 .. len-1 are cached; slot len (column t) arrives in kv_new.
  const int len = t - j0;  // cached keys of this row (negative: column t is still padding for it)
  const int blk_lo = 0, blk_hi = (len + 31) >> 5;
  const int nblk = blk_hi - blk_lo;
  const int per = (nblk + a.splits - 1) / a.splits;
  const int my_lo = blk_lo + (int)blockIdx.y * per;
  const int my_hi = min(my_lo + per, blk_hi);
  const int bpp = a.kv.page_tokens >> 5;  // blocks per page
  const int32_t *bt_row = a.bt_layer + (long)b * a.kv.max_pages;
  const float scale = 1.0f / sqrtf((float)DH);

  bf16x8 qf[QC];
#pragma unroll
  for (int c = 0; c < QC; ++c)
    qf[c] = *(const bf16x8 *)&a.q[(long)b * d + h * DH + 32 * c + 8 * grp];

  // Position t itself is not in the cache yet: its k and v arrive in the projection's staging rows.  Thread e
  // takes element e of q, k_t and v_t; the token joins the softmax as one more partial state when the waves
  // are merged, and is filed into its page slot at the very end, when the lines around it have just been read
  // and are resident in L2 (the same stores from the projection's epilogue or from a later kernel cost about
  // 3 us per layer).  When len is not a multiple of 32 the 32-key block that contains slot len IS loaded above,
  // with several splits possibly by another workgroup while this one stores: the result does not depend on
  // what that load sees, because keys >= len get weight 0 and every slot of the pool holds finite bits at all
  // times (the pool is zeroed when it is created and only finite k and v are ever filed), so 0 x slot = 0.
  // (a one-wave workgroup has 64 threads for 128 elements: EPT elements per thread, e = threadIdx.x + i * NW * 64)
  constexpr int EPT = (DH + NW * 64 - 1) / (NW * 64);
  const bool with_new = blockIdx.y == gridDim.y - 1 && len >= 0;
  float q_e[EPT], k_e[EPT], v_e[EPT];
  bf16_t k_bits[EPT], v_bits[EPT];
  int page_t = 0;
#pragma unroll
  for (int i = 0; i < EPT; ++i) {
    q_e[i] = k_e[i] = v_e[i] = 0.f;
    k_bits[i] = v_bits[i] = 0;
    const int e = (int)threadIdx.x + i * NW * 64;
    if (with_new && e < DH) {
      const bf16_t *kr = a.kv_new + ((long)b * 2) * d + h * DH;
      k_bits[i] = kr[e];
      v_bits[i] = kr[d + e];
      q_e[i] = bf2f(a.q[(long)b * d + h * DH + e]);
      k_e[i] = bf2f(k_bits[i]);
      v_e[i] = bf2f(v_bits[i]);
      page_t = bt_row[len / a.kv.page_tokens];
    }
  }

  floatx4 O[VM];
#pragma unroll
  for (int m = 0; m < VM; ++m) O[m] = floatx4{0.f, 0.f, 0.f, 0.f};
  float m_run = -1.0e30f, l_run = 0.f;  // l_run: this lane group's share of the denominator

  auto load_blk = [&](int blk, bf16x8(&kf)[2][QC], bf16x8(&vf)[VM]) {
    const int page = bt_row[blk / bpp];
    const bf16x8 *kp = (const bf16x8 *)(a.pool + (long)page * a.kv.page_elems + (long)h * (a.kv.page_tokens * DH * 2) +
                                        (long)(blk % bpp) * (64 * DH)) + lane;
#pragma unroll
    for (int tl = 0; tl < 2; ++tl)
#pragma unroll
      for (int c = 0; c < QC; ++c) kf[tl][c] = __builtin_nontemporal_load(&kp[(tl * QC + c) * 64]);
#pragma unroll
    for (int m = 0; m < VM; ++m) vf[m] = __builtin_nontemporal_load(&kp[4 * DH + m * 64]);
  };
  auto use_blk = [&](int blk, bf16x8(&kf)[2][QC], bf16x8(&vf)[VM]) {
    floatx4 S[2];
#pragma unroll
    for (int tl = 0; tl < 2; ++tl) {
      S[tl] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int c = 0; c < QC; ++c) S[tl] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[tl][c], qf[c], S[tl], 0, 0, 0);
    }
    // S[tl][i] = q . k of key  blk*32 + 16*tl + 4*grp + i
    float sv[8];
    bool ok[8];
    float bm = -1.0e30f;
#pragma unroll
    for (int tl = 0; tl < 2; ++tl)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int key = blk * 32 + 16 * tl + 4 * grp + i;
        ok[tl * 4 + i] = key < len;
        sv[tl * 4 + i] = S[tl][i] * scale;
        if (ok[tl * 4 + i]) bm = fmaxf(bm, sv[tl * 4 + i]);
      }
    bm = fmaxf(bm, __shfl_xor(bm, 16));
    bm = fmaxf(bm, __shfl_xor(bm, 32));
    const float m_new = fmaxf(m_run, bm);
    const float alpha = __expf(m_run - m_new);
    float p[8], ps = 0.f;
    uint32_t pk[4];
#pragma unroll
    for (int j = 0; j < 8; ++j) p[j] = ok[j] ? __expf(sv[j] - m_new) : 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      pk[j] = pack2(p[2 * j], p[2 * j + 1]);
      ps += bf2f(pk[j] & 0xffffu) + bf2f(pk[j] >> 16);  // the denominator uses the rounded weights
    }
    l_run = l_run * alpha + ps;
    m_run = m_new;
    const uint32x4 pku = uint32x4{pk[0], pk[1], pk[2], pk[3]};
    const bf16x8 pv = __builtin_bit_cast(bf16x8, pku);
#pragma unroll
    for (int m = 0; m < VM; ++m) {
      O[m] *= alpha;
      O[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[m], pv, O[m], 0, 0, 0);
    }
  };
  // With 64-wide heads a second block fits in the registers (four waves per SIMD leave 128), so the next block's
  // loads are in flight while this one is used: rows of a few blocks per wave are otherwise one full memory
  // latency per block.  128-wide heads would need 64 more registers than four waves per SIMD allow.
  if constexpr (DH == 64) {
    bf16x8 kf0[2][QC], vf0[VM], kf1[2][QC], vf1[VM];
    int blk = my_lo + wave;
    if (blk < my_hi) {
      load_blk(blk, kf0, vf0);
      while (true) {
        if (blk + NW < my_hi) load_blk(blk + NW, kf1, vf1);
        use_blk(blk, kf0, vf0);
        if (blk + NW >= my_hi) break;
        if (blk + 2 * NW < my_hi) load_blk(blk + 2 * NW, kf0, vf0);
        use_blk(blk + NW, kf1, vf1);
        if (blk + 2 * NW >= my_hi) break;
        blk += 2 * NW;
      }
    }
  } else {
    for (int blk = my_lo + wave; blk < my_hi; blk += NW) {
      bf16x8 kf[2][QC], vf[VM];
      load_blk(blk, kf, vf);
      use_blk(blk, kf, vf);
    }
  }
  // O[m][i] = sum_key p * v[key][16*m + 4*grp + i]   (same in all 16 columns)
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  if (lane == 0) { sm_m[wave] = m_run; sm_l[wave] = l_run; }
  if ((lane & 15) == 0) {
#pragma unroll
    for (int m = 0; m < VM; ++m)
#pragma unroll
      for (int i = 0; i < 4; ++i) sm_o[wave][16 * m + 4 * grp + i] = O[m][i];
  }
  {  // q . k_t: the first waves (the threads below DH) hold the products
    float dot = 0.f;
#pragma unroll
    for (int i = 0; i < EPT; ++i) dot += q_e[i] * k_e[i];
    for (int o = 32; o > 0; o >>= 1) dot += __shfl_xor(dot, o);
    if (lane == 0) sm_dot[wave] = dot;
  }
  __syncthreads();
  constexpr int NDW = NW < DH / 64 ? NW : DH / 64;  // waves whose sm_dot holds products
#pragma unroll
  for (int i = 0; i < EPT; ++i) {
    const int e = (int)threadIdx.x + i * NW * 64;
    if (e >= DH) continue;
    float M = sm_m[0];
    for (int w = 1; w < NW; ++w) M = fmaxf(M, sm_m[w]);
    float s_t = 0.f;
    if (with_new) {
      for (int w = 0; w < NDW; ++w) s_t += sm_dot[w];
      s_t *= scale;
      M = fmaxf(M, s_t);
    }
    float num = 0.f, den = 0.f;
    for (int w = 0; w < NW; ++w) {
      const float f = __expf(sm_m[w] - M);
      num += f * sm_o[w][e];
      den += f * sm_l[w];
    }
    if (with_new) {
      const float f = __expf(s_t - M);
      num += f * v_e[i];
      den += f;
    }
    if (a.splits == 1) {
      const float r = den > 0.f ? num / den : 0.f;
      a.o[d_act_index(b, h * DH + e, d)] = (bf16_t)f2bf(r);
    } else {
      float *pp = a.part + ((long)blockIdx.y * gridDim.x + (long)b * H + h) * (DH + 2);
      pp[e] = num;
      if (e == 0) { pp[DH] = M; pp[DH + 1] = den; }
    }
    if (with_new) {
      bf16_t *pg = a.pool + (long)page_t * a.kv.page_elems;
      const int tt = len % a.kv.page_tokens;
      pg[kv_k_off(h, tt, e, a.kv)] = k_bits[i];
      pg[kv_v_off(h, tt, e, a.kv)] = v_bits[i];
    }
  }
}

template <int DH>
__global__ void k_attn_merge(AttnArgs a) {
  const int H = a.kv.H, b = blockIdx.x / H, h = blockIdx.x % H, d = H * DH, e = threadIdx.x;
  float M = -1.0e30f;
  for (int s = 0; s < a.splits; ++s) M = fmaxf(M, a.part[((long)s * gridDim.x + blockIdx.x) * (DH + 2) + DH]);
  float num = 0.f, den = 0.f;
  for (int s = 0; s < a.splits; ++s) {
    const float *pp = a.part + ((long)s * gridDim.x + blockIdx.x) * (DH + 2);
    const float f = __expf(pp[DH] - M);
    num += f * pp[e];
    den += f * pp[DH + 1];
  }
  a.o[d_act_index(b, h * DH + e, d)] = (bf16_t)f2bf(den > 0.f ? num / den : 0.f);
}

void bf16_attention(hipStream_t s, const AttnArgs &a) {
  const dim3 grid(a.B * a.kv.H, a.splits);
  const int nw = a.waves >= 16 ? 16 : a.waves >= 8 ? 8 : a.waves >= 4 ? 4 : a.waves >= 2 ? 2 : 1;
  if (a.kv.dh == 64) {
    if (nw == 1) SKD_LAUNCH((k_attention<64, 1>), grid, dim3(64), 0, s, a);
    else if (nw == 16) SKD_LAUNCH((k_attention<64, 16>), grid, dim3(1024), 0, s, a);
    else if (nw == 8) SKD_LAUNCH((k_attention<64, 8>), grid, dim3(512), 0, s, a);
    else if (nw == 2) SKD_LAUNCH((k_attention<64, 2>), grid, dim3(128), 0, s, a);
    else SKD_LAUNCH((k_attention<64, 4>), grid, dim3(256), 0, s, a);
    if (a.splits > 1) SKD_LAUNCH(k_attn_merge<64>, dim3(a.B * a.kv.H), dim3(64), 0, s, a);
  } else {
    if (nw == 1) SKD_LAUNCH((k_attention<128, 1>), grid, dim3(64), 0, s, a);
    else if (nw == 16) SKD_LAUNCH((k_attention<128, 16>), grid, dim3(1024), 0, s, a);
    else if (nw == 8) SKD_LAUNCH((k_attention<128, 8>), grid, dim3(512), 0, s, a);
    else if (nw == 2) SKD_LAUNCH((k_attention<128, 2>), grid, dim3(128), 0, s, a);
    else SKD_LAUNCH((k_attention<128, 4>), grid, dim3(256), 0, s, a);
    if (a.splits > 1) SKD_LAUNCH(k_attn_merge<128>, dim3(a.B * a.kv.H), dim3(128), 0, s, a);
  }
}

// ------------------------------------------------------------------ causal attention over a whole prompt
// Same block arithmetic as k_attention, but the 16 MFMA columns now carry 16
// different queries (consecutive positions of one sequence) instead of one
// replicated query.  A wave owns NT = 2 consecutive 16-position tiles of one
// sequence and one head when both exist (every K and V fragment it loads then
// serves 32 queries: the kernel is bound by what the vector memory path delivers
// to registers, 64 bytes per clock and CU, so bytes per query are what counts),
// else one tile; it walks all key blocks of its tiles itself (no merge; softmax
// state per column), loading the keys of block i + 1 while it works on block i.  A workgroup
// is 4 waves on 128 consecutive rows: they read almost the same keys at almost
// the same time, so all but the first of those loads are cache hits (L2 at
// worst).  Keys of a query: real positions 0 .. own.
template <int DH, int NT>
__device__ inline void attention_rows_tiles(const AttnRowsArgs &a, int h, long row0, int b) {
  constexpr int QC = DH / 32, VM = DH / 16;
  const int lane = threadIdx.x & 63, grp = lane >> 4, col = lane & 15;
  const int d = a.kv.H * DH;
  const int p0 = (int)(row0 - a.rm.first_row[b]);        // real position of the first query
  const int len = a.rm.P - a.rm.start[b];                // real positions of this sequence
  const int last = min(p0 + 16 * NT - 1, len - 1);       // last real position of the tiles
  const int nblk = (last >> 5) + 1;
  const int bpp = a.kv.page_tokens >> 5;
  const int32_t *bt_row = a.bt_layer + (long)b * a.kv.max_pages;
  const float scale = 1.0f / sqrtf((float)DH);

  bf16x8 qf[NT][QC];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int c = 0; c < QC; ++c)
      qf[t][c] = ((const bf16x8 *)a.q)[(((row0 >> 4) + t) * (d >> 5) + ((h * DH) >> 5) + c) * 64 + act_lane(lane)];

  floatx4 O[NT][VM];
  float m_run[NT], l_run[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    m_run[t] = -1.0e30f;
    l_run[t] = 0.f;
#pragma unroll
    for (int m = 0; m < VM; ++m) O[t][m] = floatx4{0.f, 0.f, 0.f, 0.f};
  }

  auto blk_ptr = [&](int blk) {
    const int page = bt_row[blk / bpp];
    return (const bf16x8 *)(a.pool + (long)page * a.kv.page_elems + (long)h * (a.kv.page_tokens * DH * 2) +
                            (long)(blk % bpp) * (64 * DH)) + lane;
  };
  auto load_k = [&](int blk, bf16x8(&kf)[2][QC]) {
    const bf16x8 *kp = blk_ptr(blk);
#pragma unroll
    for (int tl = 0; tl < 2; ++tl)
#pragma unroll
      for (int c = 0; c < QC; ++c) kf[tl][c] = kp[(tl * QC + c) * 64];
  };
  auto load_v = [&](int blk, bf16x8(&vf)[VM]) {
    const bf16x8 *kp = blk_ptr(blk);
#pragma unroll
    for (int m = 0; m < VM; ++m) vf[m] = kp[4 * DH + m * 64];
  };
  auto use_blk = [&](int blk, const bf16x8(&kf)[2][QC], const bf16x8(&vf)[VM]) {
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int my_len = p0 + 16 * t + col + 1;  // keys of this column's query: real positions 0 .. own
      if (NT > 1 && t == 0 && blk * 32 > p0 + 15) continue;  // (uniform) the block lies past the first tile's keys
      floatx4 S[2];
#pragma unroll
      for (int tl = 0; tl < 2; ++tl) {
        S[tl] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < QC; ++c) S[tl] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[tl][c], qf[t][c], S[tl], 0, 0, 0);
      }
      float sv[8];
      bool ok[8];
      float bm = -1.0e30f;
#pragma unroll
      for (int tl = 0; tl < 2; ++tl)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int key = blk * 32 + 16 * tl + 4 * grp + i;
          ok[tl * 4 + i] = key < my_len;
          sv[tl * 4 + i] = S[tl][i] * scale;
          if (ok[tl * 4 + i]) bm = fmaxf(bm, sv[tl * 4 + i]);
        }
      bm = fmaxf(bm, __shfl_xor(bm, 16));  // lanes 16 and 32 apart hold the same query column
      bm = fmaxf(bm, __shfl_xor(bm, 32));
      const float m_new = fmaxf(m_run[t], bm);
      const float alpha = __expf(m_run[t] - m_new);
      float ps = 0.f;
      uint32_t pk[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float p_lo = ok[2 * j] ? __expf(sv[2 * j] - m_new) : 0.f;
        const float p_hi = ok[2 * j + 1] ? __expf(sv[2 * j + 1] - m_new) : 0.f;
        pk[j] = pack2(p_lo, p_hi);
        ps += bf2f(pk[j] & 0xffffu) + bf2f(pk[j] >> 16);
      }
      l_run[t] = l_run[t] * alpha + ps;
      m_run[t] = m_new;
      const uint32x4 pku = uint32x4{pk[0], pk[1], pk[2], pk[3]};
      const bf16x8 pv = __builtin_bit_cast(bf16x8, pku);
#pragma unroll
      for (int m = 0; m < VM; ++m) {
        O[t][m] *= alpha;
        O[t][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[m], pv, O[t][m], 0, 0, 0);
      }
    }
  };

  // keys one block ahead (two register sets), values requested at the top of their block: they are not needed
  // before the scores and the softmax of the first tile are done
  bf16x8 kA[2][QC], kB[2][QC], vf[VM];
  load_k(0, kA);
  for (int blk = 0; blk < nblk; blk += 2) {
    load_v(blk, vf);
    if (blk + 1 < nblk) load_k(blk + 1, kB);
    use_blk(blk, kA, vf);
    if (blk + 1 < nblk) {
      load_v(blk + 1, vf);
      if (blk + 2 < nblk) load_k(blk + 2, kA);
      use_blk(blk + 1, kB, vf);
    }
  }
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    float l = l_run[t];
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    // O[t][m][i] = numerator of query `col` of tile t, head-dim element 16m + 4grp + i
    const float inv = l > 0.f ? 1.0f / l : 0.f;
#pragma unroll
    for (int m = 0; m < VM; ++m) {
      const uint2 pk = make_uint2(pack2(O[t][m][0] * inv, O[t][m][1] * inv), pack2(O[t][m][2] * inv, O[t][m][3] * inv));
      *(uint2 *)&a.o[d_act_index(row0 + 16 * t + col, h * DH + 16 * m + 4 * grp, d)] = pk;
    }
  }
}

template <int DH>
__global__ __launch_bounds__(256, 2) void k_attention_rows(AttnRowsArgs a) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int h = blockIdx.x;
  const long row0 = ((long)blockIdx.y * 4 + wave) * 32;  // first row of this wave's pair of tiles (no barriers below)
  // rows past the last sequence carry -1; a sequence's rows are whole 16-row tiles, so the second tile of a pair may
  // belong to the next sequence
  const int b0 = row0 < a.rows ? a.rm.seq[row0] : -1;
  const int b1 = row0 + 16 < a.rows ? a.rm.seq[row0 + 16] : -1;
  if (b0 >= 0 && b1 == b0) {
    attention_rows_tiles<DH, 2>(a, h, row0, b0);
    return;
  }
  if (b0 >= 0) attention_rows_tiles<DH, 1>(a, h, row0, b0);
  if (b1 >= 0) attention_rows_tiles<DH, 1>(a, h, row0 + 16, b1);
}

void bf16_attention_rows(hipStream_t s, const AttnRowsArgs &a) {
  const dim3 grid(a.kv.H, (a.rows + 127) / 128);
  if (a.kv.dh == 64) SKD_LAUNCH(k_attention_rows<64>, grid, dim3(256), 0, s, a);
  else SKD_LAUNCH(k_attention_rows<128>, grid, dim3(256), 0, s, a);
}

// ------------------------------------------------------------------ row kernels of the batched prompt
__global__ __launch_bounds__(1024) void k_embed_ln_rows(const int32_t *tokens, RowMap rm, const bf16_t *tok_emb,
                                                        const bf16_t *pos_emb, const float *g, const float *bt, float *x,
                                                        bf16_t *a_out, int B, int d, int V) {
  __shared__ float sh[32];
  const int row = blockIdx.x, d4 = d >> 2;
  const int b = rm.seq[row];
  if (b < 0) return;  // rows past the last sequence stay zero
  const int pos = row - rm.first_row[b];  // real position = position id
  if (pos >= rm.P - rm.start[b]) return;  // padding of the sequence's last 16-row tile: stays zero
  int tok = tokens[(long)(rm.start[b] + pos) * B + b];
  tok = tok < 0 ? 0 : (tok >= V ? V - 1 : tok);
  const uint2 *te = (const uint2 *)(tok_emb + (long)tok * d), *pe = (const uint2 *)(pos_emb + (long)pos * d);
  floatx4 v[LN_NC], gv[LN_NC], bv[LN_NC];
#pragma unroll
  for (int i = 0; i < LN_NC; ++i) {
    const int c = (int)threadIdx.x + 1024 * i;
    if (c < d4) {
      const uint2 aa = te[c], p = pe[c];
      gv[i] = ((const floatx4 *)g)[c];
      bv[i] = ((const floatx4 *)bt)[c];
      v[i] = floatx4{bf2f(aa.x & 0xffffu) + bf2f(p.x & 0xffffu), bf2f(aa.x >> 16) + bf2f(p.x >> 16),
                     bf2f(aa.y & 0xffffu) + bf2f(p.y & 0xffffu), bf2f(aa.y >> 16) + bf2f(p.y >> 16)};
      ((floatx4 *)x)[(long)row * d4 + c] = v[i];
    }
  }
  ln_finish_row(v, gv, bv, d, row, a_out, sh);
}

__global__ __launch_bounds__(1024) void k_ln_rows(const float *x, const float *g, const float *bt, bf16_t *a_out, int d) {
  __shared__ float sh[32];
  const int row = blockIdx.x, d4 = d >> 2;
  floatx4 v[LN_NC], gv[LN_NC], bv[LN_NC];
#pragma unroll
  for (int i = 0; i < LN_NC; ++i) {
    const int c = (int)threadIdx.x + 1024 * i;
    if (c < d4) {
      v[i] = ((const floatx4 *)x)[(long)row * d4 + c];
      gv[i] = ((const floatx4 *)g)[c];
      bv[i] = ((const floatx4 *)bt)[c];
    }
  }
  ln_finish_row(v, gv, bv, d, row, a_out, sh);
}

// LayerNorm of 16 consecutive rows (one activation row tile) per workgroup: wave w keeps row 16 * tile + w in
// registers (rows up to 4096 wide) and needs no barrier for its statistics; the normalised values go through an
// 8 KiB LDS buffer per 256 columns so that the tile leaves the workgroup as whole, contiguous 8 KiB runs.
constexpr int LNW_NC = 16;
__global__ __launch_bounds__(1024) void k_ln_rows16(const float *x, const float *g, const float *bt, bf16_t *a_out, int d) {
  __shared__ uint2 stage[2][1024];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const long row = (long)blockIdx.x * 16 + wave;
  const int nc = d >> 8;  // 256-column chunks
  const floatx4 *xr = (const floatx4 *)x + row * (d >> 2);
  floatx4 v[LNW_NC];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < LNW_NC; ++i)
    if (i < nc) {
      v[i] = xr[lane + 64 * i];
      s += (v[i][0] + v[i][1]) + (v[i][2] + v[i][3]);
    }
  const float mean = wave_sum_f(s) / d;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < LNW_NC; ++i)
    if (i < nc) {
      const floatx4 t = v[i] - mean;
      q += (t[0] * t[0] + t[1] * t[1]) + (t[2] * t[2] + t[3] * t[3]);
    }
  const float rstd = 1.0f / sqrtf(wave_sum_f(q) / d + 1e-5f);
  uint2 *out = (uint2 *)(a_out + (long)blockIdx.x * 16 * d);  // the row tile: d / 32 tiles of 1 KiB, back to back
#pragma unroll
  for (int i = 0; i < LNW_NC; ++i)
    if (i < nc) {
      const floatx4 gv = ((const floatx4 *)g)[lane + 64 * i], bv = ((const floatx4 *)bt)[lane + 64 * i];
      const floatx4 y = (v[i] - mean) * rstd * gv + bv;
      // columns 256 i + 4 lane .. + 3 of row `wave`: tile lane / 8 of this chunk, byte wave * 64 + (lane % 8) * 8
      stage[i & 1][(lane >> 3) * 128 + wave * 8 + (lane & 7)] = make_uint2(pack2(y[0], y[1]), pack2(y[2], y[3]));
      __syncthreads();
      out[(long)i * 1024 + threadIdx.x] = stage[i & 1][threadIdx.x];
    }
}

__global__ void k_gather_rows(const float *x_rows, float *x_out, RowMap rm, int d) {
  const int b = blockIdx.x;
  const long src = ((long)rm.first_row[b] + (rm.P - rm.start[b]) - 1) * d;  // the sequence's last prompt position
  for (int k = threadIdx.x; k < d; k += blockDim.x) x_out[(long)blockIdx.x * d + k] = x_rows[src + k];
}

void bf16_embed_ln_rows(hipStream_t s, const int32_t *tokens, RowMap rm, int rows, const bf16_t *tok_emb,
                        const bf16_t *pos_emb, const float *g, const float *b, float *x, bf16_t *a_out, int B, int d,
                        int V) {
  SKD_LAUNCH(k_embed_ln_rows, dim3(rows), dim3(1024), 0, s, tokens, rm, tok_emb, pos_emb, g, b, x, a_out, B, d, V);
}
void bf16_ln_rows(hipStream_t s, const float *x, const float *g, const float *b, bf16_t *a_out, int rows, int d) {
  if (rows % 16 == 0 && d % 256 == 0 && d <= 256 * LNW_NC) {
    SKD_LAUNCH(k_ln_rows16, dim3(rows / 16), dim3(1024), 0, s, x, g, b, a_out, d);
    return;
  }
  SKD_LAUNCH(k_ln_rows, dim3(rows), dim3(1024), 0, s, x, g, b, a_out, d);
}
void bf16_gather_rows(hipStream_t s, const float *x_rows, float *x_out, RowMap rm, int B, int d) {
  SKD_LAUNCH(k_gather_rows, dim3(B), dim3(256), 0, s, x_rows, x_out, rm, d);
}

// ------------------------------------------------------------------ argmax over workgroup partials
__global__ void k_argmax_final(const float *pmax, const int32_t *pidx, int groups, int B_pad, int32_t *tokens) {
  __shared__ float sv[256];
  __shared__ int si[256];
  const int b = blockIdx.x;
  float best = -3.0e38f;
  int bi = 0x7fffffff;
  for (int g = threadIdx.x; g < groups; g += 256) {
    const float v = pmax[(long)g * B_pad + b];
    const int i = pidx[(long)g * B_pad + b];
    if (v > best || (v == best && i < bi)) { best = v; bi = i; }
  }
  sv[threadIdx.x] = best;
  si[threadIdx.x] = bi;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) {
      const float ov = sv[threadIdx.x + s];
      const int oi = si[threadIdx.x + s];
      if (ov > sv[threadIdx.x] || (ov == sv[threadIdx.x] && oi < si[threadIdx.x])) { sv[threadIdx.x] = ov; si[threadIdx.x] = oi; }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) tokens[b] = si[0];
}
void bf16_argmax_final(hipStream_t s, const float *pmax, const int32_t *pidx, int groups, int B_pad, int32_t *tokens,
                       int B) {
  SKD_LAUNCH(k_argmax_final, dim3(B), dim3(256), 0, s, pmax, pidx, groups, B_pad, tokens);
}

// ------------------------------------------------------------------ weight preparation
template <typename T>
__device__ inline float src_to_f(const T *p, long i);
template <>
__device__ inline float src_to_f<float>(const float *p, long i) { return p[i]; }
template <>
__device__ inline float src_to_f<bf16_t>(const bf16_t *p, long i) { return bf2f(p[i]); }

// one thread per 8-element lane slot of the destination
template <typename T>
__global__ void k_prep_frag(const T *src, bf16_t *dst, long N, long K, long N_pad, int G) {
  const long slot = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const long Kf = K >> 5;
  if (slot >= (N_pad >> 4) * Kf * 64) return;
  const int lane = slot & 63;
  const long frag = slot >> 6, kf = (frag / G) % Kf, nt = frag / (G * Kf) * G + frag % G;
  const long row = nt * 16 + (lane & 15), col = kf * 32 + (lane >> 4) * 8;
  uint32_t pk[4] = {0, 0, 0, 0};
  if (row < N)
    for (int j = 0; j < 4; ++j) pk[j] = pack2(src_to_f<T>(src, row * K + col + 2 * j), src_to_f<T>(src, row * K + col + 2 * j + 1));
  *(uint32x4 *)&dst[slot * 8] = uint32x4{pk[0], pk[1], pk[2], pk[3]};
}
template <typename T>
__global__ void k_prep_rm(const T *src, bf16_t *dst, long n) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = (bf16_t)f2bf(src_to_f<T>(src, i));
}
template <typename T>
__global__ void k_prep_f32(const T *src, float *dst, long n) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src_to_f<T>(src, i);
}
void prep_matrix_frag(hipStream_t s, const void *src, int src_is_bf16, bf16_t *dst, long N, long K, long N_pad,
                      int G) {
  const long slots = (N_pad / 16) * (K / 32) * 64;
  const dim3 grid((unsigned)((slots + 255) / 256));
  if (src_is_bf16) SKD_LAUNCH(k_prep_frag<bf16_t>, grid, dim3(256), 0, s, (const bf16_t *)src, dst, N, K, N_pad, G);
  else SKD_LAUNCH(k_prep_frag<float>, grid, dim3(256), 0, s, (const float *)src, dst, N, K, N_pad, G);
}
void prep_matrix_rm_bf16(hipStream_t s, const void *src, int src_is_bf16, bf16_t *dst, long n) {
  const dim3 grid((unsigned)((n + 255) / 256));
  if (src_is_bf16) SKD_LAUNCH(k_prep_rm<bf16_t>, grid, dim3(256), 0, s, (const bf16_t *)src, dst, n);
  else SKD_LAUNCH(k_prep_rm<float>, grid, dim3(256), 0, s, (const float *)src, dst, n);
}
void prep_to_f32(hipStream_t s, const void *src, int src_is_bf16, float *dst, long n) {
  const dim3 grid((unsigned)((n + 255) / 256));
  if (src_is_bf16) SKD_LAUNCH(k_prep_f32<bf16_t>, grid, dim3(256), 0, s, (const bf16_t *)src, dst, n);
  else SKD_LAUNCH(k_prep_f32<float>, grid, dim3(256), 0, s, (const float *)src, dst, n);
}

// ------------------------------------------------------------------ KV debug hooks (bf16 pages)
__global__ void k_kv_load_bf16(const float *K, const float *V, bf16_t *pool, const int32_t *bt_layer,
                               const int32_t *start, int cols, KvGeom g) {
  const int b = blockIdx.y, j = blockIdx.x, d = g.H * g.dh;
  const int slot = j - start[b];  // stored by real position
  if (slot < 0) return;
  const int page = bt_layer[(long)b * g.max_pages + slot / g.page_tokens];
  bf16_t *pg = pool + (long)page * g.page_elems;
  const int tt = slot % g.page_tokens;
  for (int k = threadIdx.x; k < d; k += blockDim.x) {
    const int h = k / g.dh, e = k % g.dh;
    pg[kv_k_off(h, tt, e, g)] = (bf16_t)f2bf(K ? K[((long)b * cols + j) * d + k] : 0.f);
    pg[kv_v_off(h, tt, e, g)] = (bf16_t)f2bf(V ? V[((long)b * cols + j) * d + k] : 0.f);
  }
}
__global__ void k_kv_read_bf16(const bf16_t *pool, const int32_t *bt_row, int start, float *K, float *V, KvGeom g) {
  const int j = blockIdx.x, d = g.H * g.dh, slot = j - start;
  if (slot < 0) {  // padding column: nothing is stored for it
    for (int k = threadIdx.x; k < d; k += blockDim.x) K[(long)j * d + k] = V[(long)j * d + k] = 0.f;
    return;
  }
  const bf16_t *pg = pool + (long)bt_row[slot / g.page_tokens] * g.page_elems;
  const int tt = slot % g.page_tokens;
  for (int k = threadIdx.x; k < d; k += blockDim.x) {
    const int h = k / g.dh, e = k % g.dh;
    K[(long)j * d + k] = bf2f(pg[kv_k_off(h, tt, e, g)]);
    V[(long)j * d + k] = bf2f(pg[kv_v_off(h, tt, e, g)]);
  }
}
void kv_load_bf16(hipStream_t s, const float *K, const float *V, bf16_t *pool, const int32_t *bt_layer,
                  const int32_t *start, int cols, int B, KvGeom g) {
  if (cols > 0) SKD_LAUNCH(k_kv_load_bf16, dim3(cols, B), dim3(256), 0, s, K, V, pool, bt_layer, start, cols, g);
}
void kv_read_bf16(hipStream_t s, const bf16_t *pool, const int32_t *bt_row, int start, int len, float *K, float *V,
                  KvGeom g) {
  if (len > 0) SKD_LAUNCH(k_kv_read_bf16, dim3(len), dim3(256), 0, s, pool, bt_row, start, K, V, g);
}

}  // namespace skd
