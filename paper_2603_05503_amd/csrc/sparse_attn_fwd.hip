// Host launcher and C entry point of the block-sparse attention forward
// (paper, Section 3.4 "Inference stage").  The kernels live in attn_kernel_*.h.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <atomic>

#include "attn_kernel_2wg.h"
#include "attn_kernel_anchor.h"
#include "attn_kernel_energy.h"
#include "attn_kernel_similarity.h"
#include "calibration_kernels.h"
#include "attn_kernel_il.h"
#include "calibatt.h"

namespace {
using namespace calibatt_dev;

struct FwdPtrs {
  const uint16_t *q, *k, *v;
  uint16_t *out;
  const int32_t *row_ptr, *col_idx, *work, *fan_ptr, *fan_dst;
  int32_t *counter;
  const int32_t *iv_ptr;  // interval form of the kept-block lists, or NULL
  const uint32_t *iv;
  const int32_t *head_map;  // tensor head of each pattern head, or NULL
  float *lse;               // log-sum-exp output, or NULL
  int dtype;                // CALIBATT_BF16 or CALIBATT_F16
};

// Per-device launch facts of one kernel: how many workgroups the whole device holds at a time.
// Looked up on the first call per device.  Concurrent first calls all compute the same figure, so
// the slot is a plain atomic (0 = not known yet) and no lock is taken.
struct DevInfo {
  std::atomic<int> slots[64];
};

template <typename Kernel>
int prepare(Kernel kernel, int threads, int smem, DevInfo &info, int &slots) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return CALIBATT_ERR_LAUNCH;
  slots = info.slots[dev].load(std::memory_order_acquire);
  if (slots > 0) return CALIBATT_OK;
  int cus = 0, per_cu = 0;
  if (hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
      hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void *)kernel, threads, smem) != hipSuccess ||
      cus <= 0 || per_cu <= 0)
    return CALIBATT_ERR_LAUNCH;
  slots = cus * per_cu;
  info.slots[dev].store(slots, std::memory_order_release);
  return CALIBATT_OK;
}

// Registers a kernel's dynamic LDS ceiling once per device (same scheme as above).
struct DevReady {
  std::atomic<int> ready[64];
};
template <typename Kernel>
int register_lds(Kernel kernel, int smem, DevReady &state, int &dev) {
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return CALIBATT_ERR_LAUNCH;
  if (state.ready[dev].load(std::memory_order_acquire)) return CALIBATT_OK;
  if (hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
    return CALIBATT_ERR_LAUNCH;
  state.ready[dev].store(1, std::memory_order_release);
  return CALIBATT_OK;
}

// Launches through the call that reports its own status: the runtime's "last error" may still hold
// an unrelated error left by earlier calls of the host program.
template <typename Kernel, typename... Args>
int launch_kernel(Kernel kernel, unsigned grid, int threads, int smem, hipStream_t stream, Args... args) {
  void *argv[] = {(void *)&args...};
  return hipLaunchKernel((const void *)kernel, dim3(grid), dim3(threads), argv, smem, stream) == hipSuccess
             ? CALIBATT_OK
             : CALIBATT_ERR_LAUNCH;
}

// Grid of the two-workgroup kernel: persistent workgroups popping from the counters when there are
// more items than the device holds workgroups, one workgroup per item otherwise.
template <typename Kernel>
int enqueue(Kernel kernel, int threads, int smem, int slots, const FwdPtrs &a, const FwdDims &p, hipStream_t stream) {
  const long long items = (long long)p.n_work * p.B;
  long long grid = items;
  int32_t *counter = a.counter;
  if (counter && items > slots) grid = slots; else counter = nullptr;
  return launch_kernel(kernel, (unsigned)grid, threads, smem, stream, a.q, a.k, a.v, a.out, a.row_ptr, a.col_idx,
                       a.work, a.fan_ptr, a.fan_dst, counter, p, a.iv_ptr, a.iv, a.head_map, a.lse);
}

// IV: the pattern comes as intervals.  `which` (CALIBATT_KERNEL_*) picks the schedule of the tile
// loop: the interleaved kernel (attn_kernel_il.h) or the two-workgroup kernel (attn_kernel_2wg.h).
template <int D, int BQ, int BK, bool IV, typename T>
int launch_typed(const FwdPtrs &a, const FwdDims &p, int which, hipStream_t stream) {
  int slots = 0;
  if (which != CALIBATT_KERNEL_TWO_WORKGROUPS) {
    static DevInfo info;
    constexpr int SMEM = IlRow<D, BQ, BK, T>::LDS_BYTES + 64 + (IV ? IV_COLS * 4 : 0);
    auto kernel = sparse_attn_fwd_il_kernel<D, BQ, BK, IV, T>;
    if (int st = prepare(kernel, BQ * 2, SMEM, info, slots)) return st;
    return enqueue(kernel, BQ * 2, SMEM, slots, a, p, stream);
  }
  if constexpr (BK == 64 || BK == 128) {
    static DevInfo info;
    constexpr int SMEM = RowBlock<D, BQ, BK>::LDS_BYTES + 64 + (IV ? IV_COLS * 4 : 0);
    auto kernel = sparse_attn_fwd_kernel<D, BQ, BK, IV, T>;
    if (int st = prepare(kernel, BQ * 2, SMEM, info, slots)) return st;
    return enqueue(kernel, BQ * 2, SMEM, slots, a, p, stream);
  } else {
    return CALIBATT_ERR_UNSUPPORTED;  // the two-workgroup kernel is built for key blocks of 64 and 128 only
  }
}

template <int D, int BQ, int BK>
int launch(const FwdPtrs &a, const FwdDims &p, int which, hipStream_t stream) {
  const long long items = (long long)p.n_work * p.B;
  if (items <= 0) return CALIBATT_OK;
  if (items > 0x7fffffffLL) return CALIBATT_ERR_SHAPE;
  if (a.dtype == CALIBATT_F16)
    return a.iv ? launch_typed<D, BQ, BK, true, F16>(a, p, which, stream)
                : launch_typed<D, BQ, BK, false, F16>(a, p, which, stream);
  return a.iv ? launch_typed<D, BQ, BK, true, Bf16>(a, p, which, stream)
              : launch_typed<D, BQ, BK, false, Bf16>(a, p, which, stream);
}

bool strides_ok(const calibatt_strides &t, int B, int H, int N, int D) {
  if (t.n < D || t.b < 0 || t.h < 0 || (t.n % 8) || (t.h % 8) || (t.b % 8)) return false;
  // the kernels address one head's rows with 32-bit byte offsets
  if ((unsigned long long)(N - 1) * (unsigned long long)t.n * 2 + (unsigned long long)D * 2 > 0xffffffffULL) return false;
  (void)B;
  (void)H;
  return true;
}

// Key-range split of the anchor path: S in [1, ANCHOR_MAX_SPLIT] minimising the length of the last
// round of work units on an XCD, ceil(rem * S / slots) / S, with a small charge per part for the
// merge; 1 when every XCD's range is a whole number of rounds or nothing is gained.
void plan_anchor_split(AnchorDims &p, int slots_per_xcd) {
  p.slots = slots_per_xcd;
  p.n_split = 1;
  p.rem_max = 0;
  if (slots_per_xcd <= 0) return;
  int rem_max = 0;
  for (int x = 0; x < ANCHOR_XCDS; ++x) {
    const AnchorRange range(p, x, ANCHOR_XCDS);
    rem_max = std::max(rem_max, range.n % slots_per_xcd);
  }
  if (rem_max == 0) return;
  int best = 1;
  double best_cost = 1.0;
  for (int s = 2; s <= ANCHOR_MAX_SPLIT && s <= p.nbk; ++s) {
    const double cost = (double)((rem_max * s + slots_per_xcd - 1) / slots_per_xcd) / s + 0.01 * s;
    if (cost < best_cost - 1e-9) {
      best_cost = cost;
      best = s;
    }
  }
  if (best_cost > 0.9) return;  // less than a tenth of a round to gain
  p.n_split = best;
  p.rem_max = rem_max;
}

template <int D>
long long anchor_workspace_bytes(const AnchorDims &p) {
  return p.n_split > 1 ? (long long)ANCHOR_XCDS * p.rem_max * p.n_split * AnchorLds<D>::PART_FLOATS * 4 : 0;
}

// slots of one XCD for the anchor kernel on the current device
template <int D>
int anchor_slots(int &slots_per_xcd) {
  static DevInfo info;
  int slots = 0;
  if (int st = prepare(anchor_attn_fwd_kernel<D>, ANCHOR_BQ * 2, AnchorLds<D>::BYTES, info, slots)) return st;
  slots_per_xcd = slots / ANCHOR_XCDS;
  return CALIBATT_OK;
}

// workspace == nullptr: every unit whole.  Otherwise the split is planned for the current device and
// the workspace must hold anchor_workspace_bytes().
template <int D>
int launch_anchor(const FwdPtrs &a, const int32_t *head_ids, const int32_t *q_index, const int32_t *dst_ptr,
                  const int32_t *dst_idx, AnchorDims p, float *workspace, long long workspace_bytes,
                  hipStream_t stream) {
  const long long units = (long long)p.B * p.n_heads * p.nbq;
  if (units <= 0) return CALIBATT_OK;
  int slots_per_xcd = 0;
  if (int st = anchor_slots<D>(slots_per_xcd)) return st;
  p.slots = slots_per_xcd;
  p.n_split = 1;
  p.rem_max = 0;
  if (workspace) {
    plan_anchor_split(p, slots_per_xcd);
    if (anchor_workspace_bytes<D>(p) > workspace_bytes) return CALIBATT_ERR_BUFFER_TOO_SMALL;
  }
  long long per_xcd = 0;
  for (int x = 0; x < ANCHOR_XCDS; ++x) {
    const AnchorRange range(p, x, ANCHOR_XCDS);
    per_xcd = std::max(per_xcd, (long long)range.whole + (long long)(range.n - range.whole) * p.n_split);
  }
  const long long grid = ANCHOR_XCDS * per_xcd;
  if (grid > 0x7fffffffLL) return CALIBATT_ERR_SHAPE;
  if (int st = launch_kernel(anchor_attn_fwd_kernel<D>, (unsigned)grid, ANCHOR_BQ * 2, AnchorLds<D>::BYTES, stream, a.q,
                             a.k, a.v, a.out, head_ids, q_index, dst_ptr, dst_idx, workspace, p))
    return st;
  if (p.n_split == 1) return CALIBATT_OK;
  static DevInfo merge_info;
  int unused = 0;
  if (int st = prepare(anchor_merge_kernel<D>, ANCHOR_BQ * 2, AnchorLds<D>::MERGE_BYTES, merge_info, unused)) return st;
  return launch_kernel(anchor_merge_kernel<D>, (unsigned)(ANCHOR_XCDS * p.rem_max), ANCHOR_BQ * 2,
                       AnchorLds<D>::MERGE_BYTES, stream, a.out, head_ids, dst_ptr, dst_idx, (const float *)workspace, p);
}

// Dynamic LDS of the energy kernel grows with the number of key blocks; one generous ceiling is
// registered per kernel and device, launches above it are refused.
constexpr int ENERGY_MAX_LDS = 128 * 1024;

template <int D, int BQ, int BK>
int launch_energy(const uint16_t *q, const uint16_t *k, float *energy, const EnergyDims &p, hipStream_t stream) {
  const long long units = (long long)p.B * p.H * p.nbq;
  const long long grid = ENERGY_XCDS * ((units + ENERGY_XCDS - 1) / ENERGY_XCDS);
  if (grid > 0x7fffffffLL) return CALIBATT_ERR_SHAPE;
  const long long smem = EnergyLds<D, BQ, BK>::bytes(p.nbk);
  if (smem > ENERGY_MAX_LDS) return CALIBATT_ERR_UNSUPPORTED;
  auto kernel = block_energy_kernel<D, BQ, BK>;
  static DevReady state;
  int dev = 0;
  if (int st = register_lds(kernel, ENERGY_MAX_LDS, state, dev)) return st;
  return launch_kernel(kernel, (unsigned)grid, BQ * 2, (int)smem, stream, q, k, energy, p);
}

// One-pass energy kernel: as many persistent workgroups as the device holds at a time, the
// workspace has slices for, and there are units.
template <int D, int BQ, int BK>
int launch_energy_onepass(const uint16_t *q, const uint16_t *k, float *energy, const EnergyDims &p, float *workspace,
                          long long workspace_bytes, hipStream_t stream) {
  const long long units = (long long)p.B * p.H * p.nbq;
  const long long smem = EnergyLds<D, BQ, BK>::bytes(p.nbk);
  if (smem > ENERGY_MAX_LDS) return CALIBATT_ERR_UNSUPPORTED;
  const long long slice = (long long)p.nbk * BQ * 4;
  if (workspace_bytes < slice) return CALIBATT_ERR_BUFFER_TOO_SMALL;
  auto kernel = block_energy_onepass_kernel<D, BQ, BK>;
  static DevReady state;
  int dev = 0, cus = 0, per_cu = 0;
  if (int st = register_lds(kernel, ENERGY_MAX_LDS, state, dev)) return st;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
      hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void *)kernel, BQ * 2, (size_t)smem) != hipSuccess ||
      cus <= 0 || per_cu <= 0)
    return CALIBATT_ERR_LAUNCH;
  EnergyOnePassDims pp;
  pp.e = p;
  pp.n_wg = (int)std::min<long long>({units, (long long)cus * per_cu, workspace_bytes / slice, 1 << 20});
  pp.xcds = pp.n_wg >= ENERGY_XCDS ? ENERGY_XCDS : 1;
  return launch_kernel(kernel, (unsigned)pp.n_wg, BQ * 2, (int)smem, stream, q, k, energy, workspace, pp);
}

template <int D>
int launch_similarity(const uint16_t *q, const uint16_t *k, const int32_t *partner, float *triples, float *score,
                      const SimilarityDims &p, hipStream_t stream) {
  const long long units = (long long)p.B * p.H * p.nbq;
  const long long grid = SIM_XCDS * ((units + SIM_XCDS - 1) / SIM_XCDS);
  if (grid > 0x7fffffffLL) return CALIBATT_ERR_SHAPE;
  constexpr int SMEM = 2 * RowBlock<D, SIM_BQ, SIM_BK>::TILE_BYTES;
  auto kernel = pair_similarity_kernel<D>;
  static DevInfo info;
  int slots = 0;
  if (int st = prepare(kernel, SIM_BQ * 2, SMEM, info, slots)) return st;
  if (int st = launch_kernel(kernel, (unsigned)grid, SIM_BQ * 2, SMEM, stream, q, k, partner, triples, p)) return st;
  return launch_kernel(similarity_reduce_kernel, (unsigned)(p.B * p.H), 64, 0, stream, (const float *)triples, score,
                       p.n_tok, p.row_len);
}

}  // namespace

extern "C" int calibatt_select_blocks_device(const float *energy, int64_t n_rows, int nbk, double eps, uint8_t *mask,
                                             void *stream) {
  if (!energy || !mask) return CALIBATT_ERR_NULL;
  if (n_rows < 0 || nbk <= 0 || eps != eps) return CALIBATT_ERR_SHAPE;
  if (nbk > SELECT_MAX_COLS) return CALIBATT_ERR_UNSUPPORTED;
  if ((uintptr_t)energy & 3) return CALIBATT_ERR_SHAPE;
  if (n_rows == 0) return CALIBATT_OK;
  int P = 2;
  while (P < nbk) P <<= 1;
  const unsigned grid = (unsigned)std::min<long long>(n_rows, 1 << 16);
  return launch_kernel(select_blocks_kernel, grid, SELECT_THREADS, P * 8, (hipStream_t)stream, energy,
                       (long long)n_rows, nbk, P, eps, mask);
}

extern "C" int calibatt_vote_accumulate_device(const uint8_t *mask, int64_t n, uint16_t *counts, void *stream) {
  if (!mask || !counts) return CALIBATT_ERR_NULL;
  if (n < 0 || ((uintptr_t)counts & 1)) return CALIBATT_ERR_SHAPE;
  if (n == 0) return CALIBATT_OK;
  const unsigned grid = (unsigned)std::min<long long>((n + 255) / 256, 1 << 16);
  return launch_kernel(vote_accumulate_kernel, grid, 256, 0, (hipStream_t)stream, mask, (long long)n, counts);
}

extern "C" int calibatt_spatial_similarity(const void *q, const void *k, int B, int H, int N, int D,
                                           const int32_t *partner, int n_tok, int row_len, float scale,
                                           float *workspace, float *score, void *stream) {
  if (!q || !k || !partner || !workspace || !score) return CALIBATT_ERR_NULL;
  if (B <= 0 || H <= 0 || N <= 0 || D <= 0 || n_tok <= 0 || row_len <= 0 || n_tok > N || n_tok % row_len)
    return CALIBATT_ERR_SHAPE;
  if (!(D == 64 || D == 128)) return CALIBATT_ERR_UNSUPPORTED;
  if ((size_t)B * H * N * D > 0x7fffffff00ULL) return CALIBATT_ERR_SHAPE;
  SimilarityDims p;
  p.B = B;
  p.H = H;
  p.N = N;
  p.n_tok = n_tok;
  p.nbq = (n_tok + SIM_BQ - 1) / SIM_BQ;
  p.nbk = (N + SIM_BK - 1) / SIM_BK;
  p.row_len = row_len;
  p.scale_log2e = scale * 1.4426950408889634f;
  hipStream_t s = (hipStream_t)stream;
  if (D == 128)
    return launch_similarity<128>((const uint16_t *)q, (const uint16_t *)k, partner, workspace, score, p, s);
  return launch_similarity<64>((const uint16_t *)q, (const uint16_t *)k, partner, workspace, score, p, s);
}

// Scratch of calibatt_spatial_similarity_static: one copy per GPU the library runs on, held until
// the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the
// device address it yields (per device) is what kernels and copies get.
constexpr long long SIMILARITY_SCRATCH_BYTES = CALIBATT_SIMILARITY_STATIC_MAX_BYTES;
static __device__ __align__(256) unsigned char scratch[SIMILARITY_SCRATCH_BYTES];

namespace {
std::atomic<void *> scratch_address[64];  // device address of `scratch` on each device, looked up once

int similarity_scratch(void *&ptr) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return CALIBATT_ERR_LAUNCH;
  ptr = scratch_address[dev].load(std::memory_order_acquire);
  if (ptr) return CALIBATT_OK;
  void *found = nullptr;
  if (hipGetSymbolAddress(&found, HIP_SYMBOL(scratch)) != hipSuccess || !found) return CALIBATT_ERR_LAUNCH;
  scratch_address[dev].store(found, std::memory_order_release);  // concurrent first calls store the same address
  ptr = found;
  return CALIBATT_OK;
}
}  // namespace

extern "C" int calibatt_spatial_similarity_static(const void *q, const void *k, int B, int H, int N, int D,
                                                  const int32_t *partner, int n_tok, int row_len, float scale,
                                                  float *score, void *stream) {
  if (!q || !k || !partner || !score) return CALIBATT_ERR_NULL;
  if (B <= 0 || H <= 0 || N <= 0 || D <= 0 || n_tok <= 0 || row_len <= 0 || n_tok > N || n_tok % row_len)
    return CALIBATT_ERR_SHAPE;
  if ((long long)B * H * n_tok * 3 * 4 > SIMILARITY_SCRATCH_BYTES) return CALIBATT_ERR_BUFFER_TOO_SMALL;
  void *workspace = nullptr;
  if (int st = similarity_scratch(workspace)) return st;
  return calibatt_spatial_similarity(q, k, B, H, N, D, partner, n_tok, row_len, scale, (float *)workspace, score,
                                     stream);
}

extern "C" int calibatt_block_energy(const void *q, const void *k, float *energy, int B, int H, int N, int D,
                                     int block_q, int block_k, float scale, void *stream) {
  if (!q || !k || !energy) return CALIBATT_ERR_NULL;
  if (B <= 0 || H <= 0 || N <= 0 || D <= 0 || block_q <= 0 || block_k <= 0) return CALIBATT_ERR_SHAPE;
  if (!(D == 64 || D == 128) || !(block_q == 64 || block_q == 128) || !(block_k == 64 || block_k == 128))
    return CALIBATT_ERR_UNSUPPORTED;
  if ((size_t)B * H * N * D > 0x7fffffff00ULL) return CALIBATT_ERR_SHAPE;
  EnergyDims p;
  p.B = B;
  p.H = H;
  p.N = N;
  p.nbq = (N + block_q - 1) / block_q;
  p.nbk = (N + block_k - 1) / block_k;
  p.scale_log2e = scale * 1.4426950408889634f;
  const uint16_t *qq = (const uint16_t *)q, *kk = (const uint16_t *)k;
  hipStream_t s = (hipStream_t)stream;
#define CALIBATT_CASE(d, bq, bk) \
  if (D == d && block_q == bq && block_k == bk) return launch_energy<d, bq, bk>(qq, kk, energy, p, s);
  CALIBATT_CASE(128, 128, 128)
  CALIBATT_CASE(128, 128, 64)
  CALIBATT_CASE(128, 128, 96)
  CALIBATT_CASE(128, 128, 160)
  CALIBATT_CASE(128, 128, 192)
  CALIBATT_CASE(128, 64, 128)
  CALIBATT_CASE(128, 64, 64)
  CALIBATT_CASE(64, 128, 128)
  CALIBATT_CASE(64, 128, 64)
  CALIBATT_CASE(64, 64, 128)
  CALIBATT_CASE(64, 64, 64)
#undef CALIBATT_CASE
  return CALIBATT_ERR_UNSUPPORTED;
}

extern "C" int calibatt_block_energy_workspace_bytes(int N, int block_q, int block_k, int64_t *bytes) {
  if (!bytes) return CALIBATT_ERR_NULL;
  if (N <= 0 || block_q <= 0 || block_k <= 0) return CALIBATT_ERR_SHAPE;
  if (!(block_q == 64 || block_q == 128) || !(block_k == 64 || block_k == 128)) return CALIBATT_ERR_UNSUPPORTED;
  *bytes = 1024LL * ((N + block_k - 1) / block_k) * block_q * 4;
  return CALIBATT_OK;
}

extern "C" int calibatt_block_energy_onepass(const void *q, const void *k, float *energy, int B, int H, int N, int D,
                                             int block_q, int block_k, float scale, void *workspace,
                                             int64_t workspace_bytes, void *stream) {
  if (!q || !k || !energy || !workspace) return CALIBATT_ERR_NULL;
  if (B <= 0 || H <= 0 || N <= 0 || D <= 0 || block_q <= 0 || block_k <= 0 || workspace_bytes < 0)
    return CALIBATT_ERR_SHAPE;
  if (!(D == 64 || D == 128) || !(block_q == 64 || block_q == 128) || !(block_k == 64 || block_k == 128))
    return CALIBATT_ERR_UNSUPPORTED;
  if ((size_t)B * H * N * D > 0x7fffffff00ULL || ((uintptr_t)workspace & 3)) return CALIBATT_ERR_SHAPE;
  EnergyDims p;
  p.B = B;
  p.H = H;
  p.N = N;
  p.nbq = (N + block_q - 1) / block_q;
  p.nbk = (N + block_k - 1) / block_k;
  p.scale_log2e = scale * 1.4426950408889634f;
  const uint16_t *qq = (const uint16_t *)q, *kk = (const uint16_t *)k;
  hipStream_t s = (hipStream_t)stream;
#define CALIBATT_CASE(d, bq, bk)                        \
  if (D == d && block_q == bq && block_k == bk)         \
    return launch_energy_onepass<d, bq, bk>(qq, kk, energy, p, (float *)workspace, workspace_bytes, s);
  CALIBATT_CASE(128, 128, 128)
  CALIBATT_CASE(128, 128, 64)
  CALIBATT_CASE(128, 128, 96)
  CALIBATT_CASE(128, 128, 160)
  CALIBATT_CASE(128, 128, 192)
  CALIBATT_CASE(128, 64, 128)
  CALIBATT_CASE(128, 64, 64)
  CALIBATT_CASE(64, 128, 128)
  CALIBATT_CASE(64, 128, 64)
  CALIBATT_CASE(64, 64, 128)
  CALIBATT_CASE(64, 64, 64)
#undef CALIBATT_CASE
  return CALIBATT_ERR_UNSUPPORTED;
}

extern "C" int calibatt_anchor_attn_fwd(const void *q, const void *k, const void *v, void *out, int B, int H,
                                        int N, int D, const int32_t *head_ids, int n_heads,
                                        const int32_t *q_index, const int32_t *dst_ptr,
                                        const int32_t *dst_idx, int n_q, float scale, void *stream) {
  if (B <= 0 || H <= 0 || N <= 0 || D <= 0) return q && k && v && out ? CALIBATT_ERR_SHAPE : CALIBATT_ERR_NULL;
  if ((size_t)B * H * N * D > 0x7fffffff00ULL) return CALIBATT_ERR_SHAPE;
  const calibatt_strides packed = {(int64_t)H * N * D, (int64_t)N * D, (int64_t)D};
  return calibatt_anchor_attn_fwd_strided(q, k, v, out, B, H, N, D, head_ids, n_heads, q_index, dst_ptr, dst_idx, n_q,
                                          scale, &packed, &packed, stream);
}

namespace {
int fill_anchor_dims(AnchorDims &p, int B, int H, int N, int D, int n_heads, int n_q, float scale,
                     const calibatt_strides *in_strides, const calibatt_strides *out_strides) {
  if (B <= 0 || H <= 0 || N <= 0 || D <= 0 || n_heads < 0 || n_q < 0) return CALIBATT_ERR_SHAPE;
  if (!(D == 64 || D == 128)) return CALIBATT_ERR_UNSUPPORTED;
  p.B = B;
  p.H = H;
  p.N = N;
  p.n_heads = n_heads;
  p.n_q = n_q;
  p.nbq = (n_q + ANCHOR_BQ - 1) / ANCHOR_BQ;
  p.nbk = (N + ANCHOR_BK - 1) / ANCHOR_BK;
  p.scale_log2e = scale * 1.4426950408889634f;
  if (in_strides) p.in = Strides{in_strides->b, in_strides->h, in_strides->n};
  if (out_strides) p.out = Strides{out_strides->b, out_strides->h, out_strides->n};
  p.n_split = 1;
  p.slots = 0;
  p.rem_max = 0;
  return CALIBATT_OK;
}
}  // namespace

extern "C" int calibatt_anchor_attn_fwd_strided(const void *q, const void *k, const void *v, void *out, int B,
                                                int H, int N, int D, const int32_t *head_ids, int n_heads,
                                                const int32_t *q_index, const int32_t *dst_ptr,
                                                const int32_t *dst_idx, int n_q, float scale,
                                                const calibatt_strides *in_strides,
                                                const calibatt_strides *out_strides, void *stream) {
  return calibatt_anchor_attn_fwd_split(q, k, v, out, B, H, N, D, head_ids, n_heads, q_index, dst_ptr, dst_idx, n_q,
                                        scale, in_strides, out_strides, nullptr, 0, stream);
}

extern "C" int calibatt_anchor_split_plan(int B, int N, int D, int n_heads, int n_q, int32_t *n_split,
                                          int64_t *workspace_bytes) {
  if (!n_split || !workspace_bytes) return CALIBATT_ERR_NULL;
  AnchorDims p{};
  if (int st = fill_anchor_dims(p, B, 1, N, D, n_heads, n_q, 1.0f, nullptr, nullptr)) return st;
  *n_split = 1;
  *workspace_bytes = 0;
  if (n_heads == 0 || n_q == 0) return CALIBATT_OK;
  int slots_per_xcd = 0;
  if (int st = D == 128 ? anchor_slots<128>(slots_per_xcd) : anchor_slots<64>(slots_per_xcd)) return st;
  plan_anchor_split(p, slots_per_xcd);
  *n_split = p.n_split;
  *workspace_bytes = D == 128 ? anchor_workspace_bytes<128>(p) : anchor_workspace_bytes<64>(p);
  return CALIBATT_OK;
}

extern "C" int calibatt_anchor_attn_fwd_split(const void *q, const void *k, const void *v, void *out, int B, int H,
                                              int N, int D, const int32_t *head_ids, int n_heads,
                                              const int32_t *q_index, const int32_t *dst_ptr,
                                              const int32_t *dst_idx, int n_q, float scale,
                                              const calibatt_strides *in_strides,
                                              const calibatt_strides *out_strides, void *workspace,
                                              int64_t workspace_bytes, void *stream) {
  if (!q || !k || !v || !out || !in_strides || !out_strides) return CALIBATT_ERR_NULL;
  AnchorDims p{};
  if (int st = fill_anchor_dims(p, B, H, N, D, n_heads, n_q, scale, in_strides, out_strides)) return st;
  if (out == q || out == k || out == v) return CALIBATT_ERR_SHAPE;
  if (!strides_ok(*in_strides, B, H, N, D) || !strides_ok(*out_strides, B, H, N, D)) return CALIBATT_ERR_SHAPE;
  if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)out | (uintptr_t)workspace) & 15) return CALIBATT_ERR_SHAPE;
  if (workspace_bytes < 0) return CALIBATT_ERR_SHAPE;
  if (n_heads == 0 || n_q == 0) return CALIBATT_OK;
  if (!head_ids || !q_index || !dst_ptr || !dst_idx) return CALIBATT_ERR_NULL;
  FwdPtrs a{};
  a.q = (const uint16_t *)q;
  a.k = (const uint16_t *)k;
  a.v = (const uint16_t *)v;
  a.out = (uint16_t *)out;
  hipStream_t s = (hipStream_t)stream;
  if (D == 128)
    return launch_anchor<128>(a, head_ids, q_index, dst_ptr, dst_idx, p, (float *)workspace, workspace_bytes, s);
  return launch_anchor<64>(a, head_ids, q_index, dst_ptr, dst_idx, p, (float *)workspace, workspace_bytes, s);
}

extern "C" int calibatt_sparse_attn_fwd(const void *q, const void *k, const void *v, void *out, int B,
                                        int H, int N, int D, int block_q, int block_k,
                                        const calibatt_pattern *pattern, float scale, void *stream) {
  if (B <= 0 || H <= 0 || N <= 0 || D <= 0) return q && k && v && out && pattern ? CALIBATT_ERR_SHAPE : CALIBATT_ERR_NULL;
  const calibatt_strides packed = {(int64_t)H * N * D, (int64_t)N * D, (int64_t)D};
  if ((size_t)B * H * N * D > 0x7fffffff00ULL) return CALIBATT_ERR_SHAPE;
  return calibatt_sparse_attn_fwd_strided(q, k, v, out, B, H, N, D, block_q, block_k, pattern, scale, &packed, &packed,
                                          stream);
}

extern "C" int calibatt_sparse_attn_fwd_strided(const void *q, const void *k, const void *v, void *out, int B,
                                                int H, int N, int D, int block_q, int block_k,
                                                const calibatt_pattern *pattern, float scale,
                                                const calibatt_strides *in_strides,
                                                const calibatt_strides *out_strides, void *stream) {
  if (!in_strides || !out_strides) return CALIBATT_ERR_NULL;
  calibatt_fwd_options opt;
  opt.in_strides = in_strides;
  opt.out_strides = out_strides;
  opt.dtype = CALIBATT_BF16;
  opt.lse = nullptr;
  opt.kernel = CALIBATT_KERNEL_AUTO;
  return calibatt_sparse_attn_fwd_ex(q, k, v, out, B, H, N, D, block_q, block_k, pattern, scale, &opt, stream);
}

extern "C" int calibatt_sparse_attn_fwd_ex(const void *q, const void *k, const void *v, void *out, int B, int H,
                                           int N, int D, int block_q, int block_k,
                                           const calibatt_pattern *pattern, float scale,
                                           const calibatt_fwd_options *options, void *stream) {
  if (!options) return CALIBATT_ERR_NULL;
  if (options->dtype != CALIBATT_BF16 && options->dtype != CALIBATT_F16) return CALIBATT_ERR_UNSUPPORTED;
  if (options->kernel != CALIBATT_KERNEL_AUTO && options->kernel != CALIBATT_KERNEL_TWO_WORKGROUPS &&
      options->kernel != CALIBATT_KERNEL_INTERLEAVED)
    return CALIBATT_ERR_UNSUPPORTED;
  if (B <= 0 || H <= 0 || N <= 0 || D <= 0) return q && k && v && out && pattern ? CALIBATT_ERR_SHAPE : CALIBATT_ERR_NULL;
  const calibatt_strides packed_strides = {(int64_t)H * N * D, (int64_t)N * D, (int64_t)D};
  const calibatt_strides *in_strides = options->in_strides ? options->in_strides : &packed_strides;
  const calibatt_strides *out_strides = options->out_strides ? options->out_strides : &packed_strides;
  if (options->lse && ((uintptr_t)options->lse & 3)) return CALIBATT_ERR_SHAPE;
  if (!q || !k || !v || !out || !pattern) return CALIBATT_ERR_NULL;
  if (B <= 0 || H <= 0 || N <= 0 || D <= 0 || block_q <= 0 || block_k <= 0) return CALIBATT_ERR_SHAPE;
  const bool wide_keys = D == 128 && block_q == 128 && (block_k == 96 || block_k == 160 || block_k == 192);
  if (!(D == 64 || D == 128) || !(block_q == 64 || block_q == 128) || !(block_k == 64 || block_k == 128 || wide_keys))
    return CALIBATT_ERR_UNSUPPORTED;
  if (out == q || out == k || out == v) return CALIBATT_ERR_SHAPE;
  const int nbq = (N + block_q - 1) / block_q, nbk = (N + block_k - 1) / block_k;
  if ((pattern->head_map ? pattern->H <= 0 : pattern->H != H) || pattern->N != N || pattern->block_q != block_q || pattern->block_k != block_k ||
      pattern->nbq != nbq || pattern->nbk != nbk || pattern->n_work < 0 || pattern->n_repeat < 0 ||
      (int64_t)pattern->n_work + pattern->n_repeat != (int64_t)pattern->H * nbq)
    return CALIBATT_ERR_PATTERN_MISMATCH;
  if (pattern->n_groups != 1 && pattern->n_groups != CALIBATT_GROUPS) return CALIBATT_ERR_PATTERN_MISMATCH;
  if (pattern->group_ptr[0] != 0 || pattern->group_ptr[pattern->n_groups] != pattern->n_work)
    return CALIBATT_ERR_PATTERN_MISMATCH;
  for (int g = 0; g < pattern->n_groups; ++g)
    if (pattern->group_ptr[g] > pattern->group_ptr[g + 1]) return CALIBATT_ERR_PATTERN_MISMATCH;
  const bool intervals = pattern->iv_ptr && pattern->iv;
  if ((pattern->iv_ptr != nullptr) != (pattern->iv != nullptr)) return CALIBATT_ERR_NULL;
  if (!pattern->row_ptr || !pattern->work || !pattern->fan_ptr ||
      (pattern->nnz > 0 && !pattern->col_idx && !intervals) || (pattern->n_repeat > 0 && !pattern->fan_dst))
    return CALIBATT_ERR_NULL;
  if (intervals && nbk > 65535) return CALIBATT_ERR_UNSUPPORTED;
  if (!strides_ok(*in_strides, B, H, N, D) || !strides_ok(*out_strides, B, H, N, D)) return CALIBATT_ERR_SHAPE;
  if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)out) & 15) return CALIBATT_ERR_SHAPE;

  FwdPtrs a;
  a.q = (const uint16_t *)q;
  a.k = (const uint16_t *)k;
  a.v = (const uint16_t *)v;
  a.out = (uint16_t *)out;
  a.row_ptr = pattern->row_ptr;
  a.col_idx = pattern->col_idx;
  a.work = pattern->work;
  a.fan_ptr = pattern->fan_ptr;
  a.fan_dst = pattern->fan_dst;
  a.counter = pattern->work_counter;
  a.iv_ptr = intervals ? pattern->iv_ptr : nullptr;
  a.iv = intervals ? pattern->iv : nullptr;
  a.head_map = pattern->head_map;
  a.lse = options->lse;
  a.dtype = options->dtype;
  FwdDims p;
  p.B = B;
  p.H = H;
  p.N = N;
  p.nbq = nbq;
  p.nbk = nbk;
  p.n_work = pattern->n_work;
  p.scale_log2e = scale * 1.4426950408889634f;
  p.n_groups = pattern->n_groups;
  for (int g = 0; g <= CALIBATT_GROUPS; ++g) p.group_ptr[g] = pattern->group_ptr[g];
  p.in = Strides{in_strides->b, in_strides->h, in_strides->n};
  p.out = Strides{out_strides->b, out_strides->h, out_strides->n};
  hipStream_t s = (hipStream_t)stream;
#define CALIBATT_CASE(d, bq, bk) \
  if (D == d && block_q == bq && block_k == bk) return launch<d, bq, bk>(a, p, options->kernel, s);
  CALIBATT_CASE(128, 128, 128)
  CALIBATT_CASE(128, 128, 64)
  CALIBATT_CASE(128, 128, 96)
  CALIBATT_CASE(128, 128, 160)
  CALIBATT_CASE(128, 128, 192)
  CALIBATT_CASE(128, 64, 128)
  CALIBATT_CASE(128, 64, 64)
  CALIBATT_CASE(64, 128, 128)
  CALIBATT_CASE(64, 128, 64)
  CALIBATT_CASE(64, 64, 128)
  CALIBATT_CASE(64, 64, 64)
#undef CALIBATT_CASE
  return CALIBATT_ERR_UNSUPPORTED;
}
