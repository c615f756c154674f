// Host side of the spatial-row anchor scheme (paper, Section 3.3): which query
// tokens are computed and which tokens receive each result.
#include <stdint.h>

#include "calibatt.h"

extern "C" int calibatt_anchor_map(int N, int F, int Hs, int Ws, int k, int32_t *q_index, int32_t *dst_ptr,
                                   int32_t *dst_idx, int32_t *n_q) {
  if (!n_q) return CALIBATT_ERR_NULL;
  if (N <= 0 || F <= 0 || Hs <= 0 || Ws <= 0 || k <= 0 || k > Hs) return CALIBATT_ERR_SHAPE;
  const int64_t n_video = (int64_t)F * Hs * Ws;
  if (n_video > N) return CALIBATT_ERR_SHAPE;
  const int n_free = N - (int)n_video;  // tokens without a spatial position
  *n_q = F * k * Ws + n_free;
  if (!q_index || !dst_ptr || !dst_idx) return CALIBATT_OK;

  // Anchor j sits under the centre of the j-th of k equal segments of [0, Hs).
  auto anchor_row = [&](int j) { return (int)(((int64_t)(2 * j + 1) * Hs) / (2 * k)); };

  int32_t i = 0;    // computed query
  int32_t pos = 0;  // fill position in dst_idx
  for (int f = 0; f < F; ++f) {
    const int32_t frame0 = f * Hs * Ws;
    int y_lo = 0;  // first row served by anchor j
    for (int j = 0; j < k; ++j) {
      // Rows served by anchor j end where the next anchor is strictly nearer.
      int y_hi = Hs;  // one past the last row served
      if (j + 1 < k) {
        const int a = anchor_row(j), a_next = anchor_row(j + 1);
        y_hi = (a + a_next) / 2 + 1;  // y - a <= a_next - y  <=>  y <= (a + a_next) / 2
      }
      for (int x = 0; x < Ws; ++x, ++i) {
        q_index[i] = frame0 + anchor_row(j) * Ws + x;
        dst_ptr[i] = pos;
        for (int y = y_lo; y < y_hi; ++y) dst_idx[pos++] = frame0 + y * Ws + x;
      }
      y_lo = y_hi;
    }
  }
  for (int t = (int)n_video; t < N; ++t, ++i) {
    q_index[i] = t;
    dst_ptr[i] = pos;
    dst_idx[pos++] = t;
  }
  dst_ptr[i] = pos;
  return CALIBATT_OK;
}

extern "C" int calibatt_anchor_partner(int F, int Hs, int Ws, int k, int32_t *partner) {
  if (!partner) return CALIBATT_ERR_NULL;
  if (F <= 0 || Hs <= 0 || Ws <= 0 || k <= 0 || k > Hs) return CALIBATT_ERR_SHAPE;
  for (int f = 0; f < F; ++f) {
    int j = 0;  // nearest anchor of row y; moves up once the next anchor is strictly nearer
    for (int y = 0; y < Hs; ++y) {
      auto anchor_row = [&](int jj) { return (int)(((int64_t)(2 * jj + 1) * Hs) / (2 * k)); };
      while (j + 1 < k && anchor_row(j + 1) - y < y - anchor_row(j)) ++j;
      const int a = anchor_row(j);
      for (int x = 0; x < Ws; ++x) partner[(f * Hs + y) * Ws + x] = (f * Hs + a) * Ws + x;
    }
  }
  return CALIBATT_OK;
}
