// Dense attention on a reduced query set with broadcast of the results, for
// gfx950 (MI355X): the spatial-row anchor scheme of the paper's Section 3.3 as
// run at inference (Section 3.4).
//
// The computed queries are given by a gather list (q_index), the receivers of
// each result by a CSR list (dst_ptr / dst_idx).  A workgroup takes 128
// consecutive computed queries of one (batch, head), gathers their rows of Q,
// runs them against ALL key/value tiles with the same tile engine as the
// block-sparse kernel (RowBlock: transposed MFMA contractions, online softmax,
// direct-to-LDS K/V tiles), stages the normalised bf16 rows in LDS and writes
// each row to all of its receivers with 16-byte stores.
//
// Placement: workgroups are dispatched to the 8 XCDs in turn (workgroup i runs
// on XCD i mod 8), and every XCD has its own L2.  All workgroups of one head
// walk the same K/V tiles in the same order at the same pace, so the work
// units (batch, head, query block) are laid out as one sequence, cut into 8
// equal contiguous ranges, one per XCD: the workgroups resident on an XCD at
// one time then belong to one or two heads and share their K/V tiles in L2.
//
// Key-range split.  All work units take the same time, so they finish in rounds
// of `slots` units per XCD and the last round may be mostly empty (with k = 5
// anchors at the Wan-480p shape 23 of 64 slots).  When n_split = S > 1 the
// units of every XCD's range beyond its last full round are cut into S parts
// of the key tiles each; a part leaves its rows normalised by its own sum and
// their log-sum-exp in a workspace, and anchor_merge_kernel combines the parts
// of a unit (weights exp(lse_s - max lse)) and does the broadcast.  Units of
// full rounds are untouched.
#pragma once
#include "attn_kernel_2wg.h"

namespace calibatt_dev {

struct AnchorDims {
  int B, H, N, n_heads, n_q, nbq, nbk;
  float scale_log2e;
  Strides in, out;  // element strides of q, k, v (shared) and of out
  int n_split;      // 1: every unit whole; S > 1: see "Key-range split" above (S <= nbk)
  int slots;        // workgroups resident on one XCD at a time
  int rem_max;      // largest number of split units of any XCD (workspace indexing)
};

constexpr int ANCHOR_MAX_SPLIT = 8;

// Range of work units of XCD `xcd` and how many of them stay whole.
struct AnchorRange {
  long long lo;
  int n, whole;
  __host__ __device__ AnchorRange(const AnchorDims &p, int xcd, int xcds) {
    const long long units = (long long)p.B * p.n_heads * p.nbq;
    lo = units * xcd / xcds;
    n = (int)(units * (xcd + 1) / xcds - lo);
    whole = p.n_split > 1 ? n / p.slots * p.slots : n;
  }
};

constexpr int ANCHOR_BQ = 128;
constexpr int ANCHOR_BK = 128;
constexpr int ANCHOR_XCDS = 8;
constexpr int ANCHOR_EC = 2048;  // receiver entries staged in LDS at a time

template <int D>
struct AnchorLds {
  using RB = RowBlock<D, ANCHOR_BQ, ANCHOR_BK>;
  static constexpr int PTR_OFF = ANCHOR_BQ * RB::OST;          // int32[BQ + 1] receiver offsets of the block's rows
  static constexpr int ENT_OFF = PTR_OFF + 1024;               // int32[EC] receiver tokens
  static constexpr int ROW_OFF = ENT_OFF + ANCHOR_EC * 4;      // uint8[EC] row of the block each entry belongs to
  static constexpr int EPILOGUE_BYTES = ROW_OFF + ANCHOR_EC;
  static constexpr int BYTES = RB::LDS_BYTES > EPILOGUE_BYTES ? RB::LDS_BYTES : EPILOGUE_BYTES;
  static constexpr int MERGE_W_OFF = EPILOGUE_BYTES;           // float[BQ][MAX_SPLIT] merge weights
  static constexpr int MERGE_BYTES = MERGE_W_OFF + ANCHOR_BQ * ANCHOR_MAX_SPLIT * 4;
  static constexpr int PART_FLOATS = ANCHOR_BQ * D + ANCHOR_BQ;  // one part in the workspace: rows, then their lse
  static_assert((ANCHOR_BQ + 1) * 4 <= 1024, "offset table does not fit its slot");
};

// Every one of the `rows_valid` rows staged in LDS (row i at i * OST) goes to all of its receivers.
template <int D>
__device__ __forceinline__ void anchor_broadcast(char *lds, int tid, int r, int b, int h, uint16_t *__restrict__ gout,
                                                 const int32_t *__restrict__ dst_ptr,
                                                 const int32_t *__restrict__ dst_idx, const AnchorDims &p) {
  constexpr int BQ = ANCHOR_BQ, EC = ANCHOR_EC;
  using RB = RowBlock<D, ANCHOR_BQ, ANCHOR_BK>;
  using L = AnchorLds<D>;
  constexpr int NT = RB::NT, CH = RB::CH, OST = RB::OST;
  const int N = p.N;
  const int rows_valid = min(BQ, p.n_q - r * BQ);
  int *const s_ptr = reinterpret_cast<int *>(lds + L::PTR_OFF);
  int *const s_ent = reinterpret_cast<int *>(lds + L::ENT_OFF);
  uint8_t *const s_row = reinterpret_cast<uint8_t *>(lds + L::ROW_OFF);
  if (tid <= rows_valid) s_ptr[tid] = dst_ptr[r * BQ + tid];
  __syncthreads();
  const int e_begin = s_ptr[0];
  const int e_end = s_ptr[rows_valid];
  uint16_t *const out_head = gout + (size_t)b * p.out.b + (size_t)h * p.out.h;
  for (int base = e_begin; base < e_end; base += EC) {
    const int n = min(EC, e_end - base);
    for (int j = tid; j < n; j += NT) s_ent[j] = dst_idx[base + j];
    for (int row = tid; row < rows_valid; row += NT) {
      const int e0 = max(s_ptr[row], base), e1 = min(s_ptr[row + 1], base + n);
      for (int e = e0; e < e1; ++e) s_row[e - base] = (uint8_t)row;
    }
    __syncthreads();
#pragma unroll 4
    for (int w = tid; w < n * CH; w += NT) {
      const int j = w / CH;
      const int cc = w % CH;
      const int tok = s_ent[j];
      if ((unsigned)tok < (unsigned)N) {
        const u32x4 val = *reinterpret_cast<const u32x4 *>(lds + (int)s_row[j] * OST + cc * 16);
        *reinterpret_cast<u32x4 *>(out_head + (size_t)tok * p.out.n + cc * 8) = val;
      }
    }
    __syncthreads();
  }
}

template <int D>
__global__ __launch_bounds__(ANCHOR_BQ * 2, 2) void anchor_attn_fwd_kernel(
    const uint16_t *__restrict__ gq, const uint16_t *__restrict__ gk, const uint16_t *__restrict__ gv,
    uint16_t *__restrict__ gout, const int32_t *__restrict__ head_ids, const int32_t *__restrict__ q_index,
    const int32_t *__restrict__ dst_ptr, const int32_t *__restrict__ dst_idx, float *__restrict__ workspace,
    const AnchorDims p) {
  constexpr int BQ = ANCHOR_BQ, BK = ANCHOR_BK;
  using RB = RowBlock<D, BQ, BK>;
  using L = AnchorLds<D>;
  constexpr int NT = RB::NT, ROWB = RB::ROWB;
  static_assert(NT >= BQ + 1, "one thread per offset-table entry");

  extern __shared__ __attribute__((aligned(1024))) char lds[];  // AnchorLds<D>::BYTES

  // Work of this workgroup: position `slot` of the range of its XCD.  The whole
  // units come first; behind them the parts of the split units, part-major, so
  // that workgroups running side by side walk the same key tiles.
  const int xcd = blockIdx.x % ANCHOR_XCDS;
  const int slot = blockIdx.x / ANCHOR_XCDS;
  const AnchorRange range(p, xcd, ANCHOR_XCDS);
  const int n_rem = range.n - range.whole;
  int unit, c0 = 0, c1 = p.nbk;
  float *part_out = nullptr;
  if (slot < range.whole) {
    unit = (int)(range.lo + slot);
  } else {
    const int j = slot - range.whole;
    if (j >= n_rem * p.n_split) return;
    const int part = j / n_rem, u = j - part * n_rem;
    unit = (int)(range.lo + range.whole + u);
    c0 = (int)((long long)p.nbk * part / p.n_split);
    c1 = (int)((long long)p.nbk * (part + 1) / p.n_split);
    part_out = workspace + ((size_t)(xcd * p.rem_max + u) * p.n_split + part) * L::PART_FLOATS;
  }
  const int r = unit % p.nbq;
  const int bh = unit / p.nbq;
  const int b = bh / p.n_heads;
  const int h = head_ids[bh - b * p.n_heads];
  if ((unsigned)h >= (unsigned)p.H) return;

  RB rb(lds, (uint32_t)p.in.n * 2);
  const int tid = rb.tid;
  const int N = p.N;
  const size_t head_off = (size_t)b * p.in.b + (size_t)h * p.in.h;
  const uint32_t head_bytes = (uint32_t)(N - 1) * rb.kv_row_bytes + ROWB;  // first byte after the last row
  const u32x4 Kres = head_rsrc(gk + head_off, head_bytes);
  const u32x4 Vres = head_rsrc(gv + head_off, head_bytes);
  rb.issue_k(Kres, c0);
  rb.issue_v(Vres, c0);
  {
    int qi = r * BQ + rb.row_in_block();
    qi = qi < p.n_q ? qi : p.n_q - 1;
    int tok = q_index[qi];
    tok = tok < 0 ? 0 : (tok < N ? tok : N - 1);
    rb.begin(gq + head_off + (size_t)tok * p.in.n);
  }
  const float sc = p.scale_log2e;
  for (int c = c0; c < c1; ++c) rb.tile(Kres, Vres, c, c + 1 < c1, c + 1, N, p.nbk, sc);
  if (part_out) {
    rb.store_partial(part_out, part_out + BQ * D);
    return;
  }
  rb.stage_result();
  anchor_broadcast<D>(lds, tid, r, b, h, gout, dst_ptr, dst_idx, p);
}

// Combines the parts of every split unit and broadcasts the rows: workgroup
// (xcd, u) takes split unit u of XCD xcd's range.  With lse_s the log-sum-exp
// of part s and m their maximum, a row is sum_s e^(lse_s - m) rows_s divided by
// sum_s e^(lse_s - m): exactly the softmax over all keys of the parts.
template <int D>
__global__ __launch_bounds__(ANCHOR_BQ * 2) void anchor_merge_kernel(
    uint16_t *__restrict__ gout, const int32_t *__restrict__ head_ids, const int32_t *__restrict__ dst_ptr,
    const int32_t *__restrict__ dst_idx, const float *__restrict__ workspace, const AnchorDims p) {
  constexpr int BQ = ANCHOR_BQ, S_MAX = ANCHOR_MAX_SPLIT;
  using RB = RowBlock<D, ANCHOR_BQ, ANCHOR_BK>;
  using L = AnchorLds<D>;
  constexpr int NT = RB::NT, OST = RB::OST;
  extern __shared__ __attribute__((aligned(1024))) char lds[];  // AnchorLds<D>::MERGE_BYTES

  const int xcd = blockIdx.x % ANCHOR_XCDS;
  const int u = blockIdx.x / ANCHOR_XCDS;
  const AnchorRange range(p, xcd, ANCHOR_XCDS);
  if (u >= range.n - range.whole) return;
  const int unit = (int)(range.lo + range.whole + u);
  const int r = unit % p.nbq;
  const int bh = unit / p.nbq;
  const int b = bh / p.n_heads;
  const int h = head_ids[bh - b * p.n_heads];
  if ((unsigned)h >= (unsigned)p.H) return;
  const int tid = threadIdx.x;
  const int S = p.n_split;
  const float *const parts = workspace + (size_t)(xcd * p.rem_max + u) * S * L::PART_FLOATS;
  float *const wgt = reinterpret_cast<float *>(lds + L::MERGE_W_OFF);

  if (tid < BQ) {
    float lse[S_MAX], m = -INFINITY, total = 0.f;
#pragma unroll
    for (int s = 0; s < S_MAX; ++s) {
      lse[s] = s < S ? parts[(size_t)s * L::PART_FLOATS + BQ * D + tid] : -INFINITY;
      m = fmaxf(m, lse[s]);
    }
#pragma unroll
    for (int s = 0; s < S_MAX; ++s) {
      lse[s] = lse[s] > -INFINITY ? __expf(lse[s] - m) : 0.f;
      total += lse[s];
    }
    const float inv = total > 0.f ? 1.0f / total : 0.f;
#pragma unroll
    for (int s = 0; s < S_MAX; ++s) wgt[tid * S_MAX + s] = lse[s] * inv;
  }
  __syncthreads();
  for (int i = tid; i < BQ * (D / 4); i += NT) {
    const int row = i / (D / 4), c4 = i % (D / 4);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < S; ++s) {
      const f32x4 x = *reinterpret_cast<const f32x4 *>(parts + (size_t)s * L::PART_FLOATS + row * D + c4 * 4);
      const float w = wgt[row * S_MAX + s];
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] += w * x[j];
    }
    u32x2 pk;
    pk[0] = Bf16::pack(acc[0], acc[1]);
    pk[1] = Bf16::pack(acc[2], acc[3]);
    *reinterpret_cast<u32x2 *>(lds + row * OST + c4 * 8) = pk;
  }
  __syncthreads();
  anchor_broadcast<D>(lds, tid, r, b, h, gout, dst_ptr, dst_idx, p);
}

}  // namespace calibatt_dev
