/* Host-only checks meant to run under AddressSanitizer + UndefinedBehaviorSanitizer:
 * the oracle (plain C, included as source) and the library's integer schedule
 * (skd_schedule.cpp, linked) are driven through their pins on tiny inputs and
 * on the extreme int32 arguments, so that an out-of-bounds access, a signed
 * overflow or a use after free in either shows up as a sanitizer report.
 * No device code, no GPU. */
#include <stdio.h>

#include "../../oracle/skd_oracle.c"

/* the library's side (C ABI, host only) */
int skd_schedule(int32_t t, int32_t P, int32_t N, int32_t n_min, int32_t n_max, int32_t L);

static uint32_t lcg_state = 12345u;
static float lcg(void) { /* uniform in [-0.5, 0.5) */
  lcg_state = lcg_state * 1664525u + 1013904223u;
  return (float)(lcg_state >> 8) / 16777216.0f - 0.5f;
}
static float *vec(size_t n, float scale, float mean) {
  float *p = (float *)malloc(n * sizeof(float));
  for (size_t i = 0; i < n; ++i) p[i] = mean + scale * lcg();
  return p;
}

static int fails = 0;
#define EXPECT(cond)                                                     \
  do {                                                                   \
    if (!(cond)) { printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); ++fails; } \
  } while (0)

static void schedules(void) {
  const int32_t big = INT32_MAX;
  const int32_t Ps[] = {0, 1, 7, 512, big - 1000}, Ts[] = {1, 2, 3, 100, 256, 999};
  const int32_t Ls[] = {1, 2, 12, 32, 1 << 20, big};
  for (unsigned a = 0; a < sizeof Ps / sizeof *Ps; ++a)
    for (unsigned b = 0; b < sizeof Ts / sizeof *Ts; ++b)
      for (unsigned c = 0; c < sizeof Ls / sizeof *Ls; ++c) {
        const int32_t P = Ps[a], N = P + Ts[b], L = Ls[c];
        const int32_t lo[] = {1, L / 3 + 1, L}, hi[] = {L, L - L / 4, L};
        for (int m = 0; m < 3; ++m) {
          if (lo[m] > hi[m]) continue;
          int prev = L;
          for (int64_t t = P > 2 ? P - 2 : 0; t <= N; ++t) {
            const int n1 = ora_schedule((int32_t)t, P, N, lo[m], hi[m], L);
            const int n2 = skd_schedule((int32_t)t, P, N, lo[m], hi[m], L);
            EXPECT(n1 == n2);
            EXPECT(n1 >= lo[m] && n1 <= L && n1 <= prev);
            if (t >= P) EXPECT(n1 <= hi[m]);
            prev = n1;
          }
          EXPECT(ora_schedule(N, P, N, lo[m], hi[m], L) == lo[m]);
          EXPECT(ora_schedule(P, P, N, lo[m], hi[m], L) == hi[m]);
        }
      }
  /* widest arguments an int32 interface can carry */
  for (int64_t t = 0; t <= big; t += big / 7) {
    EXPECT(ora_schedule((int32_t)t, 0, big, 1, big, big) == skd_schedule((int32_t)t, 0, big, 1, big, big));
  }
  EXPECT(ora_schedule(big, 0, big, 1, big, big) == 1);
  /* refused arguments: same codes on both sides */
  const int32_t bad[][6] = {{0, 4, 4, 1, 2, 2}, {-1, 4, 8, 1, 2, 2}, {9, 4, 8, 1, 2, 2}, {5, 4, 8, 0, 2, 2},
                            {5, 4, 8, 2, 1, 2}, {5, 4, 8, 1, 3, 2}, {5, -1, 8, 1, 2, 2}, {5, 4, 8, 1, 2, 0}};
  for (unsigned i = 0; i < sizeof bad / sizeof *bad; ++i) {
    const int r1 = ora_schedule(bad[i][0], bad[i][1], bad[i][2], bad[i][3], bad[i][4], bad[i][5]);
    const int r2 = skd_schedule(bad[i][0], bad[i][1], bad[i][2], bad[i][3], bad[i][4], bad[i][5]);
    EXPECT(r1 < 0 && r1 == r2);
  }
  int32_t out[8];
  EXPECT(ora_active_layers(7, 4, 8, 2, 6, 1, 8, out) == ora_schedule(7, 4, 8, 2, 6, 8));
  EXPECT(out[0] == 0 && out[1] > 1);
}

/* cached column-by-column decoding == brute-force recomputation, with skipping, warm-up and left padding */
static void tiny_decoder(void) {
  enum { L = 3, d = 16, H = 2, f = 32, V = 11, MP = 12, B = 2, C = 7 };
  ora_shape s = {L, d, H, f, V, MP};
  ora_weights w;
  memset(&w, 0, sizeof w);
  const float *ptr[12][L];
  w.tok_emb = vec((size_t)V * d, 0.5f, 0.f);
  w.pos_emb = vec((size_t)MP * d, 0.5f, 0.f);
  w.lnf_g = vec(d, 0.2f, 1.f);
  w.lnf_b = vec(d, 0.2f, 0.f);
  for (int l = 0; l < L; ++l) {
    ptr[0][l] = vec(d, 0.2f, 1.f); ptr[1][l] = vec(d, 0.2f, 0.f);
    ptr[2][l] = vec((size_t)3 * d * d, 0.6f, 0.f); ptr[3][l] = vec(3 * d, 0.2f, 0.f);
    ptr[4][l] = vec((size_t)d * d, 0.6f, 0.f); ptr[5][l] = vec(d, 0.2f, 0.f);
    ptr[6][l] = vec(d, 0.2f, 1.f); ptr[7][l] = vec(d, 0.2f, 0.f);
    ptr[8][l] = vec((size_t)f * d, 0.6f, 0.f); ptr[9][l] = vec(f, 0.2f, 0.f);
    ptr[10][l] = vec((size_t)d * f, 0.6f, 0.f); ptr[11][l] = vec(d, 0.2f, 0.f);
  }
  w.ln1_g = ptr[0]; w.ln1_b = ptr[1]; w.wqkv = ptr[2]; w.bqkv = ptr[3]; w.wo = ptr[4]; w.bo = ptr[5];
  w.ln2_g = ptr[6]; w.ln2_b = ptr[7]; w.w1 = ptr[8]; w.b1 = ptr[9]; w.w2 = ptr[10]; w.b2 = ptr[11];

  const int n_of[C] = {3, 3, 3, 3, 2, 2, 1};   /* layers per column, non-increasing */
  for (int warm = 0; warm <= 1; ++warm) {
    int32_t tokens[B][C];
    uint8_t realtok[B][C], layer_on[C][L];
    for (int b = 0; b < B; ++b)
      for (int j = 0; j < C; ++j) {
        tokens[b][j] = (int32_t)((b * 5 + j * 3 + warm) % V);
        realtok[b][j] = (uint8_t)(b == 0 || j >= 2);   /* row 1 is left-padded by two columns */
      }
    memset(layer_on, 0, sizeof layer_on);
    ora_state *st = NULL;
    EXPECT(ora_new(&s, &w, B, C, &st) == ORA_OK);
    double logits[B][V], brute[B][V];
    int32_t am[B];
    for (int j = 0; j < C && st; ++j) {
      int32_t lay[L], col_tok[B];
      uint8_t col_real[B];
      int c = 0;
      for (int l = 0; l < warm && c < n_of[j]; ++l) lay[c++] = l;
      for (int l = L - (n_of[j] - c); l < L; ++l) lay[c++] = l;
      for (int a = 0; a < c; ++a) layer_on[j][lay[a]] = 1;
      for (int b = 0; b < B; ++b) { col_tok[b] = tokens[b][j]; col_real[b] = realtok[b][j]; }
      EXPECT(ora_column(st, j, col_tok, col_real, lay, c, &logits[0][0], am) == ORA_OK);
    }
    EXPECT(ora_recompute(&s, &w, B, C, &tokens[0][0], &realtok[0][0], &layer_on[0][0], &brute[0][0]) == ORA_OK);
    for (int b = 0; b < B; ++b)
      for (int v = 0; v < V; ++v) EXPECT(fabs(logits[b][v] - brute[b][v]) <= 1e-9 * (1.0 + fabs(brute[b][v])));
    if (st) {
      double K[C][d], Vv[C][d];
      const int top_len = warm ? C - 1 : C;   /* with a warm-up layer the last column's single layer is layer 0 */
      EXPECT(ora_kv_len(st, L - 1) == top_len);
      EXPECT(ora_kv_read(st, L - 1, 1, &K[0][0], &Vv[0][0]) == top_len);
      EXPECT(ora_kv_len(st, 0) == (warm ? C : 4));
      /* a layer that left the window may not come back */
      if (!warm) {
        int32_t lay0[1] = {0}, tk[B] = {1, 2};
        EXPECT(ora_column(st, C, tk, NULL, lay0, 1, NULL, NULL) < 0);
      }
      ora_free(st);
    }
  }
  /* sampling head on a small distribution */
  {
    double z[5] = {0.1, 2.0, -1.0, 1.9, 0.0}, m[2];
    const int tok = ora_op_sample(z, 5, 0.3, 0.7, 0.25, m);
    EXPECT(tok == 1 || tok == 3);
    EXPECT(ora_op_sample(z, 5, 0.0, 0.7, 0.25, m) < 0);
  }
  free((void *)w.tok_emb); free((void *)w.pos_emb); free((void *)w.lnf_g); free((void *)w.lnf_b);
  for (int k = 0; k < 12; ++k)
    for (int l = 0; l < L; ++l) free((void *)ptr[k][l]);
}

int main(void) {
  schedules();
  tiny_decoder();
  if (fails) { printf("%d checks failed\n", fails); return 1; }
  printf("sanitize driver: all checks passed\n");
  return 0;
}
