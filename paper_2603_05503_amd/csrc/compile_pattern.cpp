// Host-side pattern compilation: block mask + repeat map -> CSR lists of kept
// key/value block columns, repeat sources, fan-out lists and a work schedule.
//
// Paper, Section 3.4: every calibrated block mask is encoded once, per query
// block-row, as the key block-columns to compute, and stays read-only on the
// GPU.  Supplement A.2 describes a padding-free flat layout with per-row
// offsets; this file builds that layout with single block indices as entries.
//
// Pure integer code, no device calls.  Ordering uses counting sorts, so one
// pattern costs O(H*nbq*nbk) byte reads plus O(H*nbq + nbk) bookkeeping.
#include "calibatt.h"

#include <algorithm>
#include <cstring>
#include <new>
#include <numeric>
#include <vector>

namespace {

struct Dims {
  int nbq, nbk;
  int64_t rows;
  bool last_partial;
};

int make_dims(int H, int N, int bq, int bk, Dims &d) {
  if (H <= 0 || N <= 0 || bq <= 0 || bk <= 0) return CALIBATT_ERR_SHAPE;
  d.nbq = (N + bq - 1) / bq;
  d.nbk = (N + bk - 1) / bk;
  d.rows = (int64_t)H * d.nbq;
  if (d.rows > 0x7ffffff0LL) return CALIBATT_ERR_SHAPE;
  d.last_partial = (N % bq) != 0;
  return CALIBATT_OK;
}

int check_repeat(const int32_t *repeat, int H, const Dims &d) {
  if (!repeat) return CALIBATT_OK;
  for (int h = 0; h < H; ++h) {
    const int32_t *rep = repeat + (int64_t)h * d.nbq;
    for (int r = 0; r < d.nbq; ++r) {
      const int32_t s = rep[r];
      if (s == -1) continue;
      if (s < -1 || s >= d.nbq || s == r) return CALIBATT_ERR_REPEAT_RANGE;
      if (rep[s] != -1) return CALIBATT_ERR_REPEAT_CHAIN;
      if (d.last_partial && s == d.nbq - 1 && r != d.nbq - 1) return CALIBATT_ERR_REPEAT_TAIL;
    }
  }
  return CALIBATT_OK;
}

inline int32_t count_row(const uint8_t *row, int n) {
  int32_t c = 0;
  for (int i = 0; i < n; ++i) c += row[i] != 0;
  return c;
}

}  // namespace

extern "C" int calibatt_pattern_sizes(const uint8_t *mask, const int32_t *repeat, int H, int N,
                                      int block_q, int block_k, int64_t *nnz, int32_t *n_work,
                                      int32_t *n_repeat) {
  if (!mask) return CALIBATT_ERR_NULL;
  Dims d;
  int st = make_dims(H, N, block_q, block_k, d);
  if (st) return st;
  st = check_repeat(repeat, H, d);
  if (st) return st;
  int64_t total = 0;
  int32_t reps = 0;
  for (int64_t i = 0; i < d.rows; ++i) {
    if (repeat && repeat[i] >= 0) {
      ++reps;
      continue;
    }
    total += count_row(mask + i * d.nbk, d.nbk);
  }
  if (nnz) *nnz = total;
  if (n_work) *n_work = (int32_t)(d.rows - reps);
  if (n_repeat) *n_repeat = reps;
  return CALIBATT_OK;
}

extern "C" int calibatt_compile_pattern(const uint8_t *mask, const int32_t *repeat, int H, int N,
                                        int block_q, int block_k, int order, int32_t *row_ptr,
                                        int32_t *col_idx, int64_t col_cap, int32_t *repeat_src,
                                        int32_t *work, int32_t *fan_ptr, int32_t *fan_dst,
                                        calibatt_pattern *out) {
  if (!mask || !row_ptr || !col_idx || !repeat_src || !work || !fan_ptr || !fan_dst || !out)
    return CALIBATT_ERR_NULL;
  if (order < CALIBATT_ORDER_NATURAL || order > CALIBATT_ORDER_XCD_HEADS_TAIL)
    return CALIBATT_ERR_UNSUPPORTED;
  const bool xcd_groups = order == CALIBATT_ORDER_XCD_HEADS || order == CALIBATT_ORDER_XCD_HEADS_TAIL;
  Dims d;
  int st = make_dims(H, N, block_q, block_k, d);
  if (st) return st;
  st = check_repeat(repeat, H, d);
  if (st) return st;

  // CSR of kept columns, (h, r) order; repeated rows stay empty.
  int64_t nnz = 0;
  int32_t n_rep = 0, max_row = 0;
  row_ptr[0] = 0;
  for (int64_t i = 0; i < d.rows; ++i) {
    const int32_t src = repeat ? repeat[i] : -1;
    repeat_src[i] = src;
    if (src >= 0) {
      ++n_rep;
    } else {
      const uint8_t *row = mask + i * d.nbk;
      const int64_t begin = nnz;
      for (int c = 0; c < d.nbk; ++c) {
        if (row[c]) {
          if (nnz >= col_cap) return CALIBATT_ERR_BUFFER_TOO_SMALL;
          col_idx[nnz++] = c;
        }
      }
      if (nnz > 0x7fffffffLL) return CALIBATT_ERR_SHAPE;
      if (nnz - begin > max_row) max_row = (int32_t)(nnz - begin);
    }
    row_ptr[i + 1] = (int32_t)nnz;
  }
  const int32_t n_work = (int32_t)(d.rows - n_rep);

  // Schedule.  A stable counting sort on (nbk - count) keeps (h, r) ascending
  // inside one count; per head for order 2, over all rows for order 1.
  int32_t group_ptr[CALIBATT_GROUPS + 1];
  group_ptr[0] = 0;
  for (int g = 1; g <= CALIBATT_GROUPS; ++g) group_ptr[g] = n_work;
  try {
    if (order == CALIBATT_ORDER_NATURAL) {
      int32_t w = 0;
      for (int64_t i = 0; i < d.rows; ++i)
        if (repeat_src[i] < 0) work[w++] = (int32_t)i;
    } else if (xcd_groups) {
      // Deal heads, heaviest first, to the currently lightest group.
      std::vector<int64_t> weight((size_t)H);
      for (int h = 0; h < H; ++h)
        weight[(size_t)h] = (int64_t)row_ptr[(int64_t)(h + 1) * d.nbq] - row_ptr[(int64_t)h * d.nbq];
      std::vector<int> heads((size_t)H);
      std::iota(heads.begin(), heads.end(), 0);
      std::stable_sort(heads.begin(), heads.end(),
                       [&](int a, int b) { return weight[(size_t)a] > weight[(size_t)b]; });
      int64_t load[CALIBATT_GROUPS] = {0};
      std::vector<int> members[CALIBATT_GROUPS];
      for (int h : heads) {
        int best = 0;
        for (int g = 1; g < CALIBATT_GROUPS; ++g)
          if (load[g] < load[best]) best = g;
        members[best].push_back(h);
        load[best] += weight[(size_t)h];
      }
      // Per group: long rows first (longest first), then head by head.
      int32_t w = 0;
      std::vector<int32_t> longs;
      auto is_long = [&](int64_t i) {
        return 2 * (int64_t)(row_ptr[i + 1] - row_ptr[i]) * n_work > 3 * nnz;
      };
      for (int g = 0; g < CALIBATT_GROUPS; ++g) {
        group_ptr[g] = w;
        longs.clear();
        for (int h : members[g])
          for (int64_t i = (int64_t)h * d.nbq; i < (int64_t)(h + 1) * d.nbq; ++i)
            if (repeat_src[i] < 0 && is_long(i)) longs.push_back((int32_t)i);
        // longs is in (dealing order, r) order; a stable sort by count keeps that for ties
        std::stable_sort(longs.begin(), longs.end(), [&](int32_t a, int32_t b) {
          return row_ptr[a + 1] - row_ptr[a] > row_ptr[b + 1] - row_ptr[b];
        });
        if (order == CALIBATT_ORDER_XCD_HEADS) {
          for (int32_t i : longs) work[w++] = i;
          for (int h : members[g])
            for (int64_t i = (int64_t)h * d.nbq; i < (int64_t)(h + 1) * d.nbq; ++i)
              if (repeat_src[i] < 0 && !is_long(i)) work[w++] = (int32_t)i;
        } else {
          // head by head, each head's blocks longest first (stable: r ascending among equal counts):
          // every head, and with it the group's queue, ends with its shortest blocks
          for (int h : members[g]) {
            const int32_t head_begin = w;
            for (int64_t i = (int64_t)h * d.nbq; i < (int64_t)(h + 1) * d.nbq; ++i)
              if (repeat_src[i] < 0) work[w++] = (int32_t)i;
            std::stable_sort(work + head_begin, work + w, [&](int32_t a, int32_t b) {
              return row_ptr[a + 1] - row_ptr[a] > row_ptr[b + 1] - row_ptr[b];
            });
          }
        }
      }
      group_ptr[CALIBATT_GROUPS] = w;
    } else {
      std::vector<int32_t> bucket((size_t)d.nbk + 2);
      const int64_t span = order == CALIBATT_ORDER_LONGEST ? d.rows : d.nbq;
      int32_t base = 0;
      for (int64_t lo = 0; lo < d.rows; lo += span) {
        std::fill(bucket.begin(), bucket.end(), 0);
        for (int64_t i = lo; i < lo + span; ++i)
          if (repeat_src[i] < 0) ++bucket[(size_t)(d.nbk - (row_ptr[i + 1] - row_ptr[i])) + 1];
        for (size_t b = 1; b < bucket.size(); ++b) bucket[b] += bucket[b - 1];
        const int32_t placed = bucket.back();
        for (int64_t i = lo; i < lo + span; ++i)
          if (repeat_src[i] < 0)
            work[base + bucket[(size_t)(d.nbk - (row_ptr[i + 1] - row_ptr[i]))]++] = (int32_t)i;
        base += placed;
      }
    }

    // Fan-out lists: for work item i, the blocks that copy it, ascending.
    std::vector<int32_t> slot((size_t)d.rows, -1);
    for (int32_t i = 0; i < n_work; ++i) slot[(size_t)work[i]] = i;
    std::memset(fan_ptr, 0, sizeof(int32_t) * ((size_t)n_work + 1));
    for (int64_t i = 0; i < d.rows; ++i) {
      if (repeat_src[i] < 0) continue;
      const int64_t src_id = (i / d.nbq) * d.nbq + repeat_src[i];
      ++fan_ptr[slot[(size_t)src_id] + 1];
    }
    for (int32_t i = 0; i < n_work; ++i) fan_ptr[i + 1] += fan_ptr[i];
    std::vector<int32_t> cursor(fan_ptr, fan_ptr + n_work);
    for (int64_t i = 0; i < d.rows; ++i) {
      if (repeat_src[i] < 0) continue;
      const int64_t src_id = (i / d.nbq) * d.nbq + repeat_src[i];
      fan_dst[cursor[(size_t)slot[(size_t)src_id]]++] = (int32_t)(i % d.nbq);
    }
  } catch (const std::bad_alloc &) {
    return CALIBATT_ERR_NOMEM;
  }

  out->H = H;
  out->N = N;
  out->block_q = block_q;
  out->block_k = block_k;
  out->nbq = d.nbq;
  out->nbk = d.nbk;
  out->n_work = n_work;
  out->n_repeat = n_rep;
  out->order = order;
  out->max_row = max_row;
  out->nnz = nnz;
  out->row_ptr = row_ptr;
  out->col_idx = col_idx;
  out->repeat_src = repeat_src;
  out->work = work;
  out->fan_ptr = fan_ptr;
  out->fan_dst = fan_dst;
  out->work_counter = nullptr;
  out->iv_ptr = nullptr;
  out->iv = nullptr;
  out->head_map = nullptr;
  out->n_groups = xcd_groups ? CALIBATT_GROUPS : 1;
  for (int g = 0; g <= CALIBATT_GROUPS; ++g) out->group_ptr[g] = group_ptr[g];
  return CALIBATT_OK;
}

extern "C" const char *calibatt_strerror(int status) {
  switch (status) {
    case CALIBATT_OK: return "success";
    case CALIBATT_ERR_NULL: return "a required pointer is NULL";
    case CALIBATT_ERR_SHAPE: return "non-positive or inconsistent dimension";
    case CALIBATT_ERR_UNSUPPORTED: return "unsupported head dimension, block size or schedule order";
    case CALIBATT_ERR_REPEAT_RANGE: return "repeat map entry out of range or block repeats itself";
    case CALIBATT_ERR_REPEAT_CHAIN: return "source of a repeated block is itself repeated";
    case CALIBATT_ERR_REPEAT_TAIL: return "short last query block used as source of a full block";
    case CALIBATT_ERR_BUFFER_TOO_SMALL: return "a caller-provided or built-in buffer is smaller than the call needs";
    case CALIBATT_ERR_PATTERN_MISMATCH: return "pattern was compiled for different H, N or block sizes";
    case CALIBATT_ERR_LAUNCH: return "HIP runtime refused the kernel launch";
    case CALIBATT_ERR_NOMEM: return "host scratch allocation failed";
    default: return "unknown calibatt status";
  }
}

extern "C" int calibatt_version(void) { return 200; }
