// Host-side skip-list tools (paper, supplement Sections A.2 and A.3): flat
// interval layout of a compiled pattern, interval merging by percentile,
// timestep sharing by IoU cliques.
#include <stdint.h>

#include <algorithm>
#include <cmath>
#include <new>
#include <vector>

#include "calibatt.h"

extern "C" int calibatt_encode_intervals(const int32_t *row_ptr, const int32_t *col_idx, int64_t n_rows,
                                         int32_t *iv_ptr, uint32_t *iv, int64_t iv_cap, int64_t *n_words) {
  if (!row_ptr || (!col_idx && n_rows > 0 && row_ptr[n_rows] > row_ptr[0])) return CALIBATT_ERR_NULL;
  if (n_rows < 0) return CALIBATT_ERR_SHAPE;
  // pass 1: validate and count
  int64_t words = 0;
  for (int64_t r = 0; r < n_rows; ++r) {
    const int32_t b = row_ptr[r], e = row_ptr[r + 1];
    if (e < b || e - b > 65535) return CALIBATT_ERR_SHAPE;
    for (int32_t i = b; i < e; ++i) {
      if (col_idx[i] < 0 || col_idx[i] > 65535) return CALIBATT_ERR_SHAPE;
      if (i > b && col_idx[i] <= col_idx[i - 1]) return CALIBATT_ERR_SHAPE;
      if (i == b || col_idx[i] != col_idx[i - 1] + 1) ++words;
    }
    ++words;  // terminating word
  }
  if (n_words) *n_words = words;
  if (!iv_ptr || !iv) return CALIBATT_OK;
  if (iv_cap < words || words > 0x7fffffffLL) return CALIBATT_ERR_BUFFER_TOO_SMALL;
  int64_t w = 0;
  for (int64_t r = 0; r < n_rows; ++r) {
    const int32_t b = row_ptr[r], e = row_ptr[r + 1];
    iv_ptr[r] = (int32_t)w;
    for (int32_t i = b; i < e; ++i)
      if (i == b || col_idx[i] != col_idx[i - 1] + 1) iv[w++] = (uint32_t)col_idx[i] | ((uint32_t)(i - b) << 16);
    iv[w++] = (uint32_t)(e - b) << 16;
  }
  iv_ptr[n_rows] = (int32_t)w;
  return CALIBATT_OK;
}

namespace {

// [start, end) runs of non-zero bytes
void runs_of(const uint8_t *row, int nbk, std::vector<std::pair<int, int>> &out) {
  out.clear();
  int start = -1;
  for (int c = 0; c <= nbk; ++c) {
    const bool kept = c < nbk && row[c] != 0;
    if (kept && start < 0) start = c;
    if (!kept && start >= 0) {
      out.emplace_back(start, c);
      start = -1;
    }
  }
}

}  // namespace

extern "C" int calibatt_merge_intervals(const uint8_t *mask, int64_t n_rows, int nbk, double pct, uint8_t *out,
                                        int32_t *width) {
  if (!mask || !out) return CALIBATT_ERR_NULL;
  if (n_rows < 0 || nbk <= 0 || !(pct > 0.0) || !(pct <= 100.0)) return CALIBATT_ERR_SHAPE;
  try {
    std::vector<std::pair<int, int>> runs;
    std::vector<int32_t> counts((size_t)n_rows);
    for (int64_t r = 0; r < n_rows; ++r) {
      runs_of(mask + r * nbk, nbk, runs);
      counts[(size_t)r] = (int32_t)runs.size();
    }
    int32_t w = 0;
    if (n_rows > 0) {
      std::vector<int32_t> sorted(counts);
      std::sort(sorted.begin(), sorted.end());
      int64_t rank = (int64_t)std::ceil(pct / 100.0 * (double)n_rows);
      rank = std::min<int64_t>(std::max<int64_t>(rank, 1), n_rows);
      w = sorted[(size_t)(rank - 1)];
    }
    if (width) *width = w;
    const int32_t limit = std::max(w, 1);
    std::vector<std::pair<int, int>> gaps;  // (gap length, index of the run on its left)
    for (int64_t r = 0; r < n_rows; ++r) {
      const uint8_t *src = mask + r * nbk;
      uint8_t *dst = out + r * nbk;
      runs_of(src, nbk, runs);  // before writing: out may alias mask
      for (int c = 0; c < nbk; ++c) dst[c] = src[c] != 0;
      const int excess = (int)runs.size() - limit;
      if (excess <= 0) continue;
      // Filling a gap never changes another gap, so "smallest gap first, leftmost among equals,
      // until the count fits" selects the `excess` first gaps in (length, position) order.
      gaps.clear();
      for (size_t i = 0; i + 1 < runs.size(); ++i) gaps.emplace_back(runs[i + 1].first - runs[i].second, (int)i);
      std::sort(gaps.begin(), gaps.end());
      for (int g = 0; g < excess; ++g) {
        const int i = gaps[(size_t)g].second;
        for (int c = runs[(size_t)i].second; c < runs[(size_t)i + 1].first; ++c) dst[c] = 1;
      }
    }
  } catch (const std::bad_alloc &) {
    return CALIBATT_ERR_NOMEM;
  }
  return CALIBATT_OK;
}

extern "C" int calibatt_share_timesteps(const uint8_t *masks, int T, int64_t n, double tau, int32_t *cluster,
                                        uint8_t *shared, int32_t *n_clusters) {
  if (!masks || !cluster || !shared || !n_clusters) return CALIBATT_ERR_NULL;
  if (T <= 0 || n < 0 || std::isnan(tau)) return CALIBATT_ERR_SHAPE;
  try {
    std::vector<std::vector<int>> members;
    auto iou_ok = [&](int a, int b) {
      const uint8_t *ma = masks + (int64_t)a * n, *mb = masks + (int64_t)b * n;
      int64_t inter = 0, uni = 0;
      for (int64_t i = 0; i < n; ++i) {
        const bool sa = ma[i] == 0, sb = mb[i] == 0;
        inter += sa && sb;
        uni += sa || sb;
      }
      const double iou = uni == 0 ? 1.0 : (double)inter / (double)uni;
      return iou >= tau;
    };
    for (int t = 0; t < T; ++t) {
      int found = -1;
      for (size_t c = 0; c < members.size() && found < 0; ++c) {
        bool all = true;
        for (int u : members[c])
          if (!iou_ok(t, u)) {
            all = false;
            break;
          }
        if (all) found = (int)c;
      }
      if (found < 0) {
        members.emplace_back();
        found = (int)members.size() - 1;
      }
      members[(size_t)found].push_back(t);
      cluster[t] = found;
    }
    *n_clusters = (int32_t)members.size();
    for (size_t c = 0; c < members.size(); ++c) {
      uint8_t *dst = shared + (int64_t)c * n;
      for (int64_t i = 0; i < n; ++i) dst[i] = 0;
      for (int u : members[c]) {
        const uint8_t *m = masks + (int64_t)u * n;
        for (int64_t i = 0; i < n; ++i) dst[i] |= (uint8_t)(m[i] != 0);
      }
    }
  } catch (const std::bad_alloc &) {
    return CALIBATT_ERR_NOMEM;
  }
  return CALIBATT_OK;
}
