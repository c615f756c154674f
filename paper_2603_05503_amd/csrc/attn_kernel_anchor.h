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
#pragma once
#include "attn_kernel_2wg.h"

namespace calibatt_dev {

struct AnchorDims {
  int B, H, N, n_heads, n_q, nbq, nbk;
  float scale_log2e;
  Strides in, out;  // element strides of q, k, v (shared) and of out
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
  static_assert((ANCHOR_BQ + 1) * 4 <= 1024, "offset table does not fit its slot");
};

template <int D>
__global__ __launch_bounds__(ANCHOR_BQ * 2, 2) void anchor_attn_fwd_kernel(
    const uint16_t *__restrict__ gq, const uint16_t *__restrict__ gk, const uint16_t *__restrict__ gv,
    uint16_t *__restrict__ gout, const int32_t *__restrict__ head_ids, const int32_t *__restrict__ q_index,
    const int32_t *__restrict__ dst_ptr, const int32_t *__restrict__ dst_idx, const AnchorDims p) {
  constexpr int BQ = ANCHOR_BQ, BK = ANCHOR_BK, EC = ANCHOR_EC;
  using RB = RowBlock<D, BQ, BK>;
  using L = AnchorLds<D>;
  constexpr int NT = RB::NT, CH = RB::CH, ROWB = RB::ROWB, OST = RB::OST;
  static_assert(NT >= BQ + 1, "one thread per offset-table entry");

  extern __shared__ __attribute__((aligned(1024))) char lds[];  // AnchorLds<D>::BYTES

  // work unit of this workgroup: position `slot` of the range of its XCD
  const int xcd = blockIdx.x % ANCHOR_XCDS;
  const int slot = blockIdx.x / ANCHOR_XCDS;
  const long long units = (long long)p.B * p.n_heads * p.nbq;
  const long long lo = units * xcd / ANCHOR_XCDS;
  const long long hi = units * (xcd + 1) / ANCHOR_XCDS;
  if (slot >= hi - lo) return;
  const int unit = (int)(lo + slot);
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
  rb.issue_k(Kres, 0);
  rb.issue_v(Vres, 0);
  {
    int qi = r * BQ + rb.row_in_block();
    qi = qi < p.n_q ? qi : p.n_q - 1;
    int tok = q_index[qi];
    tok = tok < 0 ? 0 : (tok < N ? tok : N - 1);
    rb.begin(gq + head_off + (size_t)tok * p.in.n);
  }
  const float sc = p.scale_log2e;
  for (int c = 0; c < p.nbk; ++c) rb.tile(Kres, Vres, c, c + 1 < p.nbk, c + 1, N, p.nbk, sc);
  rb.stage_result();

  // ---- broadcast: every staged row goes to all of its receivers ---------------
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

}  // namespace calibatt_dev
