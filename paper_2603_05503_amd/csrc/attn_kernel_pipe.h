// Block-sparse attention forward for gfx950, software-pipelined variant for
// 128-row query blocks, 128-row kv blocks and head dimension 128: one workgroup
// per CU, one wavefront per SIMD, and the softmax of one kv tile overlapped,
// inside every wavefront, with the matrix products of its neighbours.
//
// What it computes is the same as the two-workgroup kernel (paper, Section 2
// Eq. 1-4 restricted to the kept blocks of Section 3.2, run as in Section 3.4;
// repeated query blocks of Section 3.3 written by the owner of their source).
//
// Schedule of one query block with kept tiles 0..n-1 (S_t = K_t Q^T, P_t =
// exp2(sc S_t - m), O += V_t^T P_t):
//
//   phase A(i) : MFMA  S_{i+1} = K_{i+1} Q^T         | VALU  later part of P_i   | DMA V_{i+1}
//   phase B1(i): MFMA  O += V_i^T P_i, slabs 0-1     | VALU  row maximum of S_{i+1}
//   phase B2(i): MFMA  O += V_i^T P_i, slabs 2-7     | VALU  first part of P_{i+1} | DMA K_{i+3}
//
// The compiler neither interleaves MFMA and VALU streams by itself nor keeps
// 250 live vector registers where they are, so S, P, O, Q and the MFMA
// operands live in registers the compiler never allocates (the kernel is built
// with a cap of 64 vector registers; v64-v255 and a64-a223 are addressed by
// name), and every instruction touching them comes from attn_pipe_asm.h, which
// a script in this directory writes.  What is left to the compiler is the
// control flow, addresses, and the per-row scalars m, l, alpha.
//
// The reference maximum m only moves when a tile's row maximum exceeds it by
// more than 8 in the log2 domain (probabilities then stay below 2^8: no
// overflow, same relative precision in bf16), so the rescale of O and of the
// row sum is a rare, wave-uniform branch instead of 64 multiplies per tile; O
// is rescaled after the product that was still formed with the old reference.
// A negative softmax scale is folded into the sign of Q, so only maxima are
// ever needed.
//
// K and V tiles are double-buffered in LDS (4 x 32 KB) and arrive by
// buffer_load ... lds issued from inside the phases, three phases ahead of
// their first use; there are two barriers per tile.  The kv-block list of the
// row is copied to LDS once per query block.
#pragma once
#include <type_traits>

#include "attn_common.h"
#include "attn_pipe_asm.h"

namespace calibatt_dev {

constexpr int PIPE_COL_CAP = 4096;  // kv-block list entries held in LDS per query block

template <int D, int BQ, int BK>
struct PipeLds {
  static constexpr int TILE = BK * D * 2;
  static constexpr int MAILBOX = 4 * TILE;
  static constexpr int COLS = MAILBOX + 64;
  static constexpr int BYTES = COLS + PIPE_COL_CAP * 4;
};

__device__ __forceinline__ void pipe_barrier() { asm volatile("s_barrier"); }

template <int D, int BQ, int BK>
__global__ __launch_bounds__(BQ * 2, 1) __attribute__((amdgpu_num_vgpr(64))) void sparse_attn_fwd_pipe_kernel(
    const uint16_t *__restrict__ gq, const uint16_t *__restrict__ gk, const uint16_t *__restrict__ gv,
    uint16_t *__restrict__ gout, const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx,
    const int32_t *__restrict__ work, const int32_t *__restrict__ fan_ptr, const int32_t *__restrict__ fan_dst,
    int32_t *counter, const FwdDims p) {
  static_assert(D == 128 && BQ == 128 && BK == 128, "the instruction streams are written for 128 x 128 x 128 tiles");
  constexpr int NT = 256;
  constexpr int CH = D / 8;
  constexpr int DS = 8;   // k-slabs of S = K Q^T
  constexpr int DB = 4;   // 32-wide d blocks of O^T
  constexpr int ROWB = D * 2;
  constexpr int TILE = BK * ROWB;
  constexpr int OST = ROWB + 16;
  using Lds = PipeLds<D, BQ, BK>;
  using LoadK = TileLoader<D, BK, NT, false>;
  using LoadV = TileLoader<D, BK, NT, true>;
  constexpr int LPW = LoadK::ITERS;  // DMA instructions per wave and tile
  static_assert(LPW == 8 && LoadK::INVARIANT && LoadV::INVARIANT, "shape not covered by this kernel");
  static_assert(BQ * OST <= 2 * TILE, "output staging must fit into the K buffers");
  static_assert(TILE == 32768, "LDS offsets in the instruction streams assume 32 KB tiles");
  constexpr float RESCALE_STEP = 8.0f;

  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int l32 = lane & 31;
  const int g = lane >> 5;

  const uint32_t k_lane_off = LoadK::lane_offset(tid, 0);
  const uint32_t v_lane_off = LoadV::lane_offset(tid, 0);
  const uint32_t lds_base = (uint32_t)(uintptr_t)(LDS_PTR(char))lds;
  const uint32_t wave_u = __builtin_amdgcn_readfirstlane(wave);
  const uint32_t lds_wave = lds_base + wave_u * 1024;  // + buffer offset
  const int N = p.N;
  const int n_items = p.n_work * p.B;
  volatile int *const mailbox = reinterpret_cast<volatile int *>(lds + Lds::MAILBOX);
  int *const colbuf = reinterpret_cast<int *>(lds + Lds::COLS);

  // MFMA operand addresses (see the two-workgroup kernel for the derivation); the
  // XOR swizzle makes the K address of k-slab s equal to k_addr[0] ^ (s << 5).
  // Buffer and sub-block offsets are immediates in the instruction streams.
  const int krow_in_kb = (l32 & 0x13) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);
  uint32_t k_addr[DS];
#pragma unroll
  for (int s = 0; s < DS; ++s)
    k_addr[s] = lds_base + ((krow_in_kb * ROWB + ((g ^ k_swz<D>(krow_in_kb)) << 4)) ^ (s << 5));
  const int L16 = lane & 15;
  const int blk = lane >> 4;
  const int v_row_off = 8 * (blk >> 1) + (L16 >> 2);
  uint32_t v_addr[DB];  // V buffer 0
#pragma unroll
  for (int db = 0; db < DB; ++db)
    v_addr[db] = lds_base + 2 * TILE + v_row_off * ROWB +
                 (((4 * db + 2 * (blk & 1) + ((L16 & 3) >> 1)) ^ v_swz<D>(v_row_off)) << 4) + (L16 & 1) * 8;
  const uint32_t o_addr = lds_base + (wave * 32 + l32) * OST + 8 * g;  // output staging row of this lane
  // softmax scale in the log2 domain; its sign moves into Q
  const bool neg_scale = p.scale_log2e < 0.f;
  const float sc = fabsf(p.scale_log2e);
  const uint32_t q_flip = neg_scale ? 0x80008000u : 0u;

  int cur_group = 0, groups_left = p.n_groups;
  if (counter && p.n_groups > 1)
    cur_group = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) % p.n_groups;  // HW_REG_XCC_ID[3:0]

  for (int wg_item = blockIdx.x;;) {
    if (counter) {
      if (tid == 0) {
        int found = -1;
        while (groups_left > 0) {
          const int it = atomicAdd(counter + cur_group, 1);
          if (it < (p.group_ptr[cur_group + 1] - p.group_ptr[cur_group]) * p.B) {
            found = p.group_ptr[cur_group] * p.B + it;
            break;
          }
          cur_group = cur_group + 1 == p.n_groups ? 0 : cur_group + 1;
          --groups_left;
        }
        *mailbox = found;
      }
      __syncthreads();
      wg_item = __builtin_amdgcn_readfirstlane(*mailbox);
      if (wg_item < 0) break;
    }
    if (wg_item >= n_items) break;
    const int item = wg_item / p.B;
    const int b = wg_item - item * p.B;
    const int id = work[item];
    const int h = id / p.nbq;
    const int r = id - h * p.nbq;
    const size_t head_off = ((size_t)b * p.H + h) * (size_t)N * D;
    const u32x4 Kres = head_rsrc(gk + head_off, (uint32_t)N * ROWB);
    const u32x4 Vres = head_rsrc(gv + head_off, (uint32_t)N * ROWB);
    const int cbeg = row_ptr[id];
    const int n = row_ptr[id + 1] - cbeg;

    // kv-block list of this row -> LDS (read back as wave-uniform values)
    for (int t = tid; t < n; t += NT) colbuf[t] = col_idx[cbeg + t];
    __syncthreads();
    auto col = [&](int t) { return __builtin_amdgcn_readfirstlane(colbuf[t]); };
    auto issue_k = [&](int t) { LoadK::issue(Kres, col(t) * BK, lds_wave + (t & 1) * TILE, tid, k_lane_off); };
    auto issue_v = [&](int t) { LoadV::issue(Vres, col(t) * BK, lds_wave + (2 + (t & 1)) * TILE, tid, v_lane_off); };

    if (n > 0) {
      issue_k(0);
      issue_v(0);
      if (n > 1) issue_k(1);
    }
    // Q^T as MFMA B operand: lane (query l32, half g) holds d = 16 s + 8 g + [0,8) of k-slab s
    {
      int qrow = r * BQ + wave * 32 + l32;
      qrow = qrow < N ? qrow : N - 1;
      const u32x4 *qp = reinterpret_cast<const u32x4 *>(gq + head_off + (size_t)qrow * D + 8 * g);
      u32x4 qa[4], qb[4];
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        qa[s] = qp[2 * s];
        qb[s] = qp[2 * (s + 4)];
      }
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        qa[s] ^= q_flip;
        qb[s] ^= q_flip;
      }
      pipe_load_q<0>(qa[0], qa[1], qa[2], qa[3]);
      pipe_load_q<1>(qb[0], qb[1], qb[2], qb[3]);
    }
    pipe_zero_o();

    float m_ref = -INFINITY;    // reference maximum (log2 domain), same in lane and lane^32
    float l0 = 0.f, l1 = 0.f;   // this lane's share of the row sum (two partial sums), relative to m_ref
    float alpha_o = 1.f;        // factor O still has to be multiplied with
    float sc_t[2] = {sc, sc};   // multiplier of S of even / odd tiles (1 once a ragged tile was scaled and masked)

    // ragged last kv block: scale and mask S of tile parity T now, continue with multiplier 1
    auto mask_if_tail = [&](auto tpar, int c) {
      constexpr int T = decltype(tpar)::value;
      sc_t[T] = sc;
      if (c == p.nbk - 1 && (N % BK) != 0) {
        pipe_mask_tail<T>(sc, N - c * BK - 8 * g, -INFINITY);
        sc_t[T] = 1.0f;
      }
    };
    // the (rare) move of the reference maximum, given this lane's maximum of the raw logits
    auto new_tile_max = [&](float mx, float s_mul) {
      const float m_loc = max_with_other_half(mx * s_mul);
      const bool up = m_loc > m_ref + RESCALE_STEP;
      if (__any(up)) {
        const float a = up ? __builtin_amdgcn_exp2f(m_ref - m_loc) : 1.0f;  // 0 while m_ref is still -inf
        l0 *= a;
        l1 *= a;
        alpha_o *= a;
        m_ref = up ? m_loc : m_ref;
      }
    };
    auto wait_tiles = [&](int tiles_in_flight) {  // DMA of older tiles has landed
      if (tiles_in_flight >= 2) wait_vmem<2 * LPW>();
      else if (tiles_in_flight == 1) wait_vmem<LPW>();
      else wait_vmem<0>();
    };
    auto rescale_o_if_pending = [&]() {
      if (__any(alpha_o != 1.0f)) {
        pipe_rescale_o(alpha_o);
        alpha_o = 1.0f;
      }
    };

    // One tile step with a successor (i + 1 < n), PAR = i & 1: tile i uses the S / P registers and
    // the V buffer of parity PAR, tile i+1 the other ones and K buffer 1 - PAR.
    // c1 / c3 = kv block of tile i+1 / i+3.
    auto stage_full = [&](auto par, int i, int c1, int c3) {
      constexpr int PAR = decltype(par)::value;
      using Y = std::integral_constant<int, 1 - PAR>;
      rescale_o_if_pending();
      pipe_phase_a<PAR>(k_addr, sc_t[PAR], m_ref, l0, l1, Vres, v_lane_off, (uint32_t)c1 * (BK * ROWB),
                        lds_wave + (2 + (1 - PAR)) * TILE);
      wait_tiles((i + 2 < n ? 1 : 0) + 1);  // V_i landed; K_{i+2}, V_{i+1} may be in flight
      pipe_barrier();
      mask_if_tail(Y{}, c1);
      float mx;
      pipe_phase_b1<PAR>(v_addr, mx);
      new_tile_max(mx, sc_t[1 - PAR]);
#ifdef PIPE_DEBUG_NO_B2K
      if (i + 3 < n) {
        issue_k(i + 3);
        pipe_phase_b2<PAR>(v_addr, sc_t[1 - PAR], m_ref, l0, l1);
        wait_tiles(2);
      } else
#endif
      if (i + 3 < n) {
        pipe_phase_b2_k<PAR>(v_addr, sc_t[1 - PAR], m_ref, l0, l1, Kres, k_lane_off, (uint32_t)c3 * (BK * ROWB),
                             lds_wave + (1 - PAR) * TILE);
        wait_tiles(2);  // K_{i+2} landed; V_{i+1}, K_{i+3} may be in flight
      } else {
        pipe_phase_b2<PAR>(v_addr, sc_t[1 - PAR], m_ref, l0, l1);
        wait_tiles(1);  // K_{i+2} landed (if any); V_{i+1} may be in flight
      }
      pipe_barrier();
    };
    // The last tile: nothing left to overlap with.
    auto stage_last = [&](auto par) {
      constexpr int PAR = decltype(par)::value;
      rescale_o_if_pending();
      pipe_softmax_part1<PAR>(sc_t[PAR], m_ref, l0, l1);
      wait_vmem<0>();
      pipe_barrier();
      pipe_pv_plain<PAR>(v_addr);
    };

    using T0 = std::integral_constant<int, 0>;
    using T1 = std::integral_constant<int, 1>;
    if (n > 0) {
      // ---- prologue: S_0, its maximum, first part of P_0
      wait_vmem<0>();
      pipe_barrier();  // every wave's share of K_0, V_0, K_1 has landed
      pipe_qk_first(k_addr);
      pipe_barrier();  // K buffer 0 is free again
      if (n > 2) issue_k(2);
      mask_if_tail(T0{}, col(0));
      float mx;
      pipe_max_plain<0>(mx);
      new_tile_max(mx, sc_t[0]);
      alpha_o = 1.0f;  // O is still zero: nothing to rescale for the first maximum
      pipe_softmax_part0<0>(sc_t[0], m_ref, l0, l1);
      // kv blocks of the next tiles, kept in scalar registers; the LDS read of the entry
      // needed two steps later is issued one step ahead of its use
      auto colc = [&](int t) { return colbuf[t < n ? t : n - 1]; };
      int c1 = __builtin_amdgcn_readfirstlane(colc(1)), c2 = __builtin_amdgcn_readfirstlane(colc(2));
      int c3 = __builtin_amdgcn_readfirstlane(colc(3));
      int pend = colc(4);
      auto advance = [&](int i) {
        c1 = c2;
        c2 = c3;
        c3 = __builtin_amdgcn_readfirstlane(pend);
        pend = colc(i + 5);
      };
      int i = 0;
      for (; i + 2 < n; i += 2) {
        stage_full(T0{}, i, c1, c3);
        advance(i);
        stage_full(T1{}, i + 1, c1, c3);
        advance(i + 1);
      }
      if (n - i == 2) {
        stage_full(T0{}, i, c1, c3);
        stage_last(T1{});
      } else {
        stage_last(T0{});
      }
    }

    // ---- normalise, stage in LDS (K buffers), store to the block and its repeat targets
    const float l_tot = sum_with_other_half(l0 + l1);
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    pipe_store_o(inv, o_addr);
    __syncthreads();
    const int fbeg = fan_ptr[item];
    const int fend = fan_ptr[item + 1];
    uint16_t *const out_head = gout + head_off;
    for (int f = fbeg - 1; f < fend; ++f) {
      const int rd = f < fbeg ? r : fan_dst[f];
      const int rows_valid = min(BQ, N - rd * BQ);
      uint16_t *dst = out_head + (size_t)rd * BQ * D;
#pragma unroll 4
      for (int L = tid; L < BQ * CH; L += NT) {
        const int row = L / CH;
        const int cc = L % CH;
        if (row < rows_valid) {
          const u32x4 val = *reinterpret_cast<const u32x4 *>(lds + row * OST + cc * 16);
          *reinterpret_cast<u32x4 *>(dst + (size_t)row * D + cc * 8) = val;
        }
      }
    }
    if (!counter) break;
    __syncthreads();  // staging tile fully read before the next item's loads overwrite it
  }

  if (counter && tid == 0) {
    __threadfence();
    if (atomicAdd(counter + CALIBATT_GROUPS, 1) == (int)gridDim.x - 1) {
      for (int i = 0; i <= CALIBATT_GROUPS; ++i) counter[i] = 0;
      __threadfence();
    }
  }
}

}  // namespace calibatt_dev
