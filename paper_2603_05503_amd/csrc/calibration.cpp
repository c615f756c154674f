// Host-side calibration steps (paper, Section 3.2): block selection by energy
// (Eq. 6), threshold schedule (Eq. 7), cross-prompt vote (Eq. 8-9).
#include <stdint.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <limits>
#include <new>
#include <numeric>
#include <vector>

#include "calibatt.h"

namespace {
// Ascending in this key = descending in value, for all finite values and infinities; -0 equals +0.
inline uint32_t sort_key(float x) {
  uint32_t u;
  std::memcpy(&u, &x, 4);
  if (u == 0x80000000u) u = 0;
  const uint32_t ascending = (u & 0x80000000u) ? ~u : (u | 0x80000000u);  // ascending in value
  return ~ascending;
}
}  // namespace

extern "C" int calibatt_select_blocks(const float *energy, int64_t n_rows, int nbk, double eps, uint8_t *mask) {
  if (!energy || !mask) return CALIBATT_ERR_NULL;
  if (n_rows < 0 || nbk <= 0 || std::isnan(eps)) return CALIBATT_ERR_SHAPE;
  std::vector<int32_t> order;
  try {
    order.resize((size_t)nbk);
  } catch (const std::bad_alloc &) {
    return CALIBATT_ERR_NOMEM;
  }
  for (int64_t row = 0; row < n_rows; ++row) {
    const float *e = energy + row * nbk;
    uint8_t *m = mask + row * nbk;
    std::iota(order.begin(), order.end(), 0);
    // descending energy; among equals the lower column first (stable sort of ascending columns).
    // Compared through the order-reversing integer key the device routine sorts by (-0 as +0): a total
    // order whatever the values, NaN included.
    std::stable_sort(order.begin(), order.end(), [e](int32_t a, int32_t b) { return sort_key(e[a]) < sort_key(e[b]); });
    std::fill(m, m + nbk, (uint8_t)0);
    double total = 0.0;
    for (int i = 0; i < nbk; ++i) {
      m[order[i]] = 1;
      total += (double)e[order[i]];
      if (total >= eps) break;
    }
  }
  return CALIBATT_OK;
}

extern "C" int calibatt_vote_masks(const uint8_t *masks, int n_prompts, int64_t n, double rho, uint8_t *out) {
  if (!masks || !out) return CALIBATT_ERR_NULL;
  if (n_prompts <= 0 || n < 0 || std::isnan(rho)) return CALIBATT_ERR_SHAPE;
  for (int64_t i = 0; i < n; ++i) {
    int count = 0;
    for (int p = 0; p < n_prompts; ++p) count += masks[(int64_t)p * n + i] != 0;
    out[i] = ((double)count / (double)n_prompts >= rho) ? 1 : 0;
  }
  return CALIBATT_OK;
}

extern "C" int calibatt_vote_accumulate(const uint8_t *mask, int64_t n, uint16_t *counts) {
  if (!mask || !counts) return CALIBATT_ERR_NULL;
  if (n < 0) return CALIBATT_ERR_SHAPE;
  for (int64_t i = 0; i < n; ++i)
    if (mask[i] != 0 && counts[i] == 65535) return CALIBATT_ERR_SHAPE;  // checked before anything is changed
  for (int64_t i = 0; i < n; ++i) counts[i] = (uint16_t)(counts[i] + (mask[i] != 0));
  return CALIBATT_OK;
}

extern "C" int calibatt_vote_finish(const uint16_t *counts, int n_prompts, int64_t n, double rho, uint8_t *out) {
  if (!counts || !out) return CALIBATT_ERR_NULL;
  if (n_prompts <= 0 || n_prompts > 65535 || n < 0 || std::isnan(rho)) return CALIBATT_ERR_SHAPE;
  for (int64_t i = 0; i < n; ++i)
    if (counts[i] > n_prompts) return CALIBATT_ERR_SHAPE;
  for (int64_t i = 0; i < n; ++i) out[i] = ((double)counts[i] / (double)n_prompts >= rho) ? 1 : 0;
  return CALIBATT_OK;
}

extern "C" double calibatt_epsilon_schedule(int t, int T, double A, double C, double k) {
  if (T <= 0) return std::numeric_limits<double>::quiet_NaN();
  return A + (C - A) * std::exp(-k * (double)t / (double)T);
}

extern "C" double calibatt_schedule_base_level(int N) { return 0.796 + 1.41e-6 * (double)N; }

extern "C" int calibatt_schedule_constants(int regime, int N, double *A, double *C, double *k) {
  if (!A || !C || !k) return CALIBATT_ERR_NULL;
  if (N <= 0) return CALIBATT_ERR_SHAPE;
  if (regime == CALIBATT_REGIME_MANY_STEP) {
    *A = calibatt_schedule_base_level(N);
    *C = 0.99;
    *k = 16.0;
  } else if (regime == CALIBATT_REGIME_DISTILLED) {
    *A = 0.763;
    *C = 0.863;
    *k = 5.64;
  } else {
    return CALIBATT_ERR_UNSUPPORTED;
  }
  return CALIBATT_OK;
}

extern "C" int calibatt_flag_heads(const float *scores, int n_prompts, int H, double gamma, uint8_t *flags,
                                   double *mean) {
  if (!scores || !flags) return CALIBATT_ERR_NULL;
  if (n_prompts <= 0 || H <= 0 || std::isnan(gamma)) return CALIBATT_ERR_SHAPE;
  for (int h = 0; h < H; ++h) {
    double total = 0.0;
    for (int p = 0; p < n_prompts; ++p) total += (double)scores[(int64_t)p * H + h];
    const double m = total / (double)n_prompts;
    if (mean) mean[h] = m;
    flags[h] = m > gamma ? 1 : 0;
  }
  return CALIBATT_OK;
}
