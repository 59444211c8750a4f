// Host-only part of the C ABI: the SkipDecode schedule (Section 2.3) and the
// active-layer set (Section 2.4).  Pure integer arithmetic, no device.
#include "../../include/skd.h"

extern "C" int skd_schedule(int32_t t, int32_t P, int32_t N, int32_t n_min, int32_t n_max, int32_t L) {
  if (L < 1 || n_min < 1 || n_max < n_min || L < n_max || P < 0 || N <= P) return SKD_ERR_SHAPE;
  if (t < 0 || t > N) return SKD_ERR_RANGE;
  if (t < P) return L;  // the prompt runs the whole network
  // Linear decay over k = t - P in [0, T], T = N - P: the real value is
  // r = n_max - span * k / T with span = n_max - n_min.  Nearest integer,
  // halves up:  floor(r + 1/2) = n_max - ceil((2 * span * k - T) / (2 T)),
  // evaluated exactly (the numerator is >= -T, so it can be negative).
  const int64_t T = (int64_t)N - P, k = (int64_t)t - P, span = (int64_t)n_max - n_min;
  const int64_t a = 2 * span * k - T, b = 2 * T;
  int64_t q = a / b;       // truncates toward zero = ceiling for negative a
  if (a % b > 0) ++q;      // positive non-multiple: round up
  return (int)(n_max - q);
}

extern "C" int skd_active_layers(int32_t t, const skd_config *cfg, int32_t *layers_out) {
  if (!cfg || !layers_out) return SKD_ERR_NULL;
  const int n = skd_schedule(t, cfg->prompt_size, cfg->sequence_length, cfg->n_min, cfg->n_max, cfg->L);
  if (n < 0) return n;
  if (cfg->warmup < 0 || cfg->warmup > cfg->n_min) return SKD_ERR_SHAPE;
  int c = 0;
  if (t < cfg->prompt_size) {
    for (int l = 0; l < cfg->L; ++l) layers_out[c++] = l;
    return c;
  }
  for (int l = 0; l < cfg->warmup; ++l) layers_out[c++] = l;       // warm-up layers at the bottom
  for (int l = cfg->L - (n - cfg->warmup); l < cfg->L; ++l) layers_out[c++] = l;  // the rest at the top
  return c;
}

extern "C" const char *skd_strerror(int err) {
  switch (err) {
    case SKD_OK: return "ok";
    case SKD_ERR_NULL: return "null pointer";
    case SKD_ERR_SHAPE: return "inconsistent shape or configuration";
    case SKD_ERR_RANGE: return "value out of range";
    case SKD_ERR_ORDER: return "call out of sequence";
    case SKD_ERR_SCHEDULE: return "layer set is not monotone";
    case SKD_ERR_NOMEM: return "out of memory";
    case SKD_ERR_HIP: return "HIP runtime error";
    default: return err > 0 ? "ok (count)" : "unknown error";
  }
}
