// Block-sparse attention forward for gfx950, software-pipelined variant for
// 128-row query blocks, 128-row kv blocks and head dimension 128.
//
// What it computes is the same as the two-workgroup kernel (paper, Section 2
// Eq. 1-4 restricted to the kept blocks of Section 3.2, run as in Section 3.4;
// repeated query blocks of Section 3.3 written by the owner of their source).
//
// Shape of the work: a workgroup of TWO wavefronts owns one query block, each
// wavefront 64 queries (two groups of 32), two workgroups per CU so that every
// SIMD hosts one wavefront with the whole register file.  An MFMA operand read
// from LDS then feeds two MFMAs (one per query group): with 32 queries per
// wavefront the LDS reads of the four wavefronts take as long as the MFMAs
// themselves and cannot be hidden.  Every kept 128-key block is processed as
// two sub-tiles of 64 keys.
//
// Schedule of one query block with sub-tiles 0..T-1 (S_t = K_t Q^T, P_t =
// exp2(sc S_t - m), O += V_t^T P_t), inside every wavefront:
//
//   phase A(i) : MFMA  S_{i+1} = K_{i+1} Q^T         | VALU  middle part of P_i            | DMA V_{i+1}
//   phase B1(i): MFMA  O += V_i^T P_i, slabs 0-1     | VALU  last part of P_i, row maxima of S_{i+1}
//   phase B2(i): MFMA  O += V_i^T P_i, slabs 2-3     | VALU  first part of P_{i+1}         | DMA K_{i+3}
//
// Measured on this hardware, per MFMA of 8 passes: one transcendental and up to
// four or five plain VALU instructions of the same wavefront cost a few cycles
// each; a second transcendental or a dot instruction stalls the matrix pipeline
// for about 20 cycles.  Hence exactly one v_exp_f32 behind every MFMA, and row
// sums by plain additions.  The two workgroup barriers of a sub-tile sit inside
// the streams, in front of the last slab of phases A and B2, and the first LDS
// operand reads of the following phase are issued right behind them, so that
// their latency is covered by that slab's MFMAs.
//
// The compiler neither interleaves MFMA and VALU streams by itself nor keeps
// 400 live registers where they are, so S, P, O, Q and the MFMA operands live
// in registers the compiler never allocates (the kernel is built with a cap of
// 64 vector registers; v64-v255 and a16-a255 are addressed by name; the build
// verifies that the compiler stayed out of them), and every instruction
// touching them comes from attn_pipe_asm.h, which a script in this directory
// writes.  What is left to the compiler is the control flow, addresses, and
// the per-row scalars m, l, alpha.
//
// The reference maximum m only moves when a sub-tile's row maximum exceeds it
// by more than 8 in the log2 domain (probabilities then stay below 2^8: no
// overflow, same relative precision in bf16), so the rescale of O and of the
// row sum is a rare, wave-uniform branch instead of 128 multiplies per
// sub-tile; O is rescaled after the product that was still formed with the old
// reference.  A negative softmax scale is folded into the sign of Q, so only
// maxima are ever needed.
//
// K and V sub-tiles are double-buffered in LDS (4 x 16 KB) and arrive by
// buffer_load ... lds issued from inside the phases, three phases ahead of
// their first use.
// The first keys of the row's sub-tiles are written to LDS once per query block.
#pragma once
#include <type_traits>

#include "attn_common.h"
#include "attn_pipe_asm.h"

namespace calibatt_dev {

constexpr int PIPE_COL_CAP = 1000;  // longest kv-block list of a query block this kernel takes
constexpr int PIPE_THREADS = 128;   // two wavefronts of 64 queries

template <int D, int BQ, int BK>
struct PipeLds {
  static constexpr int SUB = BK / 2;           // keys per sub-tile
  static constexpr int TILE = SUB * D * 2;     // bytes of one K or V sub-tile
  static constexpr int MAILBOX = 4 * TILE;
  static constexpr int COLS = MAILBOX + 64;
  static constexpr int BYTES = COLS + (2 * PIPE_COL_CAP + 8) * 4;  // first key of every sub-tile
};

__device__ __forceinline__ void pipe_barrier() {
  asm volatile("s_barrier");
}

template <int D, int BQ, int BK>
__global__ __launch_bounds__(PIPE_THREADS, 1) __attribute__((amdgpu_num_vgpr(64))) void sparse_attn_fwd_pipe_kernel(
    const uint16_t *__restrict__ gq, const uint16_t *__restrict__ gk, const uint16_t *__restrict__ gv,
    uint16_t *__restrict__ gout, const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx,
    const int32_t *__restrict__ work, const int32_t *__restrict__ fan_ptr, const int32_t *__restrict__ fan_dst,
    int32_t *counter, const FwdDims p) {
  static_assert(D == 128 && BQ == 128 && BK == 128, "the instruction streams are written for 128 x 128 x 128 blocks");
  constexpr int NT = PIPE_THREADS;
  constexpr int CH = D / 8;
  constexpr int DS = 8;   // k-slabs of S = K Q^T
  constexpr int DB = 4;   // 32-wide d blocks of O^T
  constexpr int ROWB = D * 2;
  using Lds = PipeLds<D, BQ, BK>;
  constexpr int SUB = Lds::SUB;
  constexpr int TILE = Lds::TILE;
  constexpr int OST = ROWB + 16;
  using LoadK = TileLoader<D, SUB, NT, false>;
  using LoadV = TileLoader<D, SUB, NT, true>;
  constexpr int LPW = LoadK::ITERS;  // DMA instructions per wave and sub-tile
  static_assert(LPW == 8 && LoadV::INVARIANT, "shape not covered by this kernel");
  static_assert(BQ * OST <= 4 * TILE, "output staging must fit into the K and V buffers");
  static_assert(TILE == 16384, "LDS offsets in the instruction streams assume 16 KB sub-tiles");
  constexpr float RESCALE_STEP = 8.0f;

  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int l32 = lane & 31;
  const int g = lane >> 5;

  // lane offsets of the direct-to-LDS loads; the K swizzle differs between even and odd instructions
  const uint32_t k_lane_off0 = LoadK::lane_offset(tid, 0), k_lane_off1 = LoadK::lane_offset(tid, 1);
  const uint32_t v_lane_off = LoadV::lane_offset(tid, 0);
  const uint32_t lds_base = (uint32_t)(uintptr_t)(LDS_PTR(char))lds;
  const uint32_t wave_u = __builtin_amdgcn_readfirstlane(wave);
  const uint32_t lds_wave = lds_base + wave_u * 1024;  // + buffer offset
  const int N = p.N;
  const int n_items = p.n_work * p.B;
  volatile int *const mailbox = reinterpret_cast<volatile int *>(lds + Lds::MAILBOX);
  int *const keybuf = reinterpret_cast<int *>(lds + Lds::COLS);

  // MFMA operand addresses (see the two-workgroup kernel for the derivation); the
  // XOR swizzle makes the K address of k-slab s equal to k_addr[0] ^ (s << 5).
  // Buffer, sub-block and slab offsets are immediates in the instruction streams.
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
  // output staging rows of this lane's two queries (query group qg: row 64 wave + 32 qg + l32)
  const uint32_t o_addr0 = lds_base + (wave * 64 + l32) * OST + 8 * g;
  const uint32_t o_addr1 = o_addr0 + 32 * OST;
  // softmax scale in the log2 domain; its sign moves into Q
  const float sc = fabsf(p.scale_log2e);
  const uint32_t q_flip = p.scale_log2e < 0.f ? 0x80008000u : 0u;

  int cur_group = 0, groups_left = p.n_groups;
  if (counter && p.n_groups > 1)
    cur_group = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) % p.n_groups;  // HW_REG_XCC_ID[3:0]
  ResidencyClock residency;
  residency.start();

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

    // First key of every sub-tile of this row -> LDS.  Sub-tile t = half (t & 1) of kept kv block
    // t >> 1; T of them (the second half of a ragged last block is dropped when it holds no key).
    // Entry j holds sub-tile j + 1 (so that the pairs read in the loop are 8-byte aligned); entries
    // past the end repeat the last sub-tile, which is what the loads issued past the end fetch.
    int T = 2 * n;
    if (n > 0 && N - col_idx[cbeg + n - 1] * BK <= SUB) --T;
    for (int j = tid; j < T + 8; j += NT) {
      const int t = j + 1 < T ? j + 1 : T - 1;
      keybuf[j] = T > 0 ? col_idx[cbeg + (t >> 1)] * BK + (t & 1) * SUB : 0;
    }
    const int key_first = n > 0 ? col_idx[cbeg] * BK : 0;  // sub-tile 0
    __syncthreads();
    auto key_of = [&](int t) { return __builtin_amdgcn_readfirstlane(keybuf[t - 1]); };  // t >= 1
    auto issue_k = [&](int t, int key) { LoadK::issue(Kres, key, lds_wave + (t & 1) * TILE, tid, k_lane_off0); };
    auto issue_v = [&](int t, int key) { LoadV::issue(Vres, key, lds_wave + (2 + (t & 1)) * TILE, tid, v_lane_off); };

    if (T > 0) {
      issue_k(0, key_first);
      issue_v(0, key_first);
      issue_k(1, key_of(1));
    }
    // Q^T as MFMA B operand: lane (query l32 of group qg, half g) holds d = 16 s + 8 g + [0,8) of k-slab s
    {
      const int q0 = r * BQ + wave * 64 + l32;
      const int qrow0 = q0 < N ? q0 : N - 1, qrow1 = q0 + 32 < N ? q0 + 32 : N - 1;
      const u32x4 *qp0 = reinterpret_cast<const u32x4 *>(gq + head_off + (size_t)qrow0 * D + 8 * g);
      const u32x4 *qp1 = reinterpret_cast<const u32x4 *>(gq + head_off + (size_t)qrow1 * D + 8 * g);
      auto load_part = [&](auto part) {
        constexpr int PART = decltype(part)::value;
        u32x4 a0 = qp0[2 * (2 * PART)], a1 = qp1[2 * (2 * PART)];
        u32x4 b0 = qp0[2 * (2 * PART + 1)], b1 = qp1[2 * (2 * PART + 1)];
        a0 ^= q_flip; a1 ^= q_flip; b0 ^= q_flip; b1 ^= q_flip;
        pipe_load_q<PART>(a0, a1, b0, b1);
      };
      load_part(std::integral_constant<int, 0>{});
      load_part(std::integral_constant<int, 1>{});
      load_part(std::integral_constant<int, 2>{});
      load_part(std::integral_constant<int, 3>{});
    }
    pipe_zero_o();

    // per query group of this lane:
    float m_ref[2] = {-INFINITY, -INFINITY};  // reference maximum (log2 domain), same in lane and lane^32
    float l[2][2] = {{0.f, 0.f}, {0.f, 0.f}}; // this lane's share of the row sum (two partial sums), relative to m_ref
    float alpha_o[2] = {1.f, 1.f};            // factor O still has to be multiplied with
    float sc_t[2] = {sc, sc};  // multiplier of S of even / odd sub-tiles (1 once a ragged one was scaled and masked)

    // ragged end of the key sequence: scale and mask S of sub-tile parity TP now, continue with multiplier 1
    auto mask_if_tail = [&](auto tpar, int key0) {
      constexpr int TP = decltype(tpar)::value;
      sc_t[TP] = sc;
      if (key0 + SUB > N) {
        pipe_mask_tail<TP>(sc, N - key0 - 8 * g, -INFINITY);
        sc_t[TP] = 1.0f;
      }
    };
    // the (rare) move of the reference maxima, given the row maxima of the new sub-tile
    auto new_tile_max = [&](const float (&mx)[2]) {
      const bool up0 = mx[0] > m_ref[0] + RESCALE_STEP, up1 = mx[1] > m_ref[1] + RESCALE_STEP;
      if (__any(up0 || up1)) {
        const float a0 = up0 ? __builtin_amdgcn_exp2f(m_ref[0] - mx[0]) : 1.0f;  // 0 while m_ref is still -inf
        const float a1 = up1 ? __builtin_amdgcn_exp2f(m_ref[1] - mx[1]) : 1.0f;
        l[0][0] *= a0;
        l[0][1] *= a0;
        l[1][0] *= a1;
        l[1][1] *= a1;
        alpha_o[0] *= a0;
        alpha_o[1] *= a1;
        m_ref[0] = up0 ? mx[0] : m_ref[0];
        m_ref[1] = up1 ? mx[1] : m_ref[1];
      }
    };
    auto rescale_o_if_pending = [&]() {
      if (__any(alpha_o[0] != 1.0f || alpha_o[1] != 1.0f)) {
        pipe_rescale_o<0>(alpha_o[0]);
        pipe_rescale_o<1>(alpha_o[1]);
        alpha_o[0] = alpha_o[1] = 1.0f;
      }
    };

    // One sub-tile step with a successor (i + 1 < T), PAR = i & 1: sub-tile i uses the S / P registers
    // and the V buffer of parity PAR, sub-tile i+1 the other ones and K buffer 1 - PAR.
    // k1 / k3 = first key of sub-tile i+1 / i+3 (the last sub-tile again where there is none: the
    // load then lands in a buffer nobody reads, and the count of loads in flight stays the same).
    auto stage_full = [&](auto par, int k1, int k3) {
      constexpr int PAR = decltype(par)::value;
      using Y = std::integral_constant<int, 1 - PAR>;
      rescale_o_if_pending();
      // (barrier inside, in front of the last k-slab: V_i has landed; K_{i+2}, V_{i+1} may be in flight)
      pipe_phase_a<PAR>(k_addr, v_addr, sc_t[PAR], m_ref, l, Vres, v_lane_off, v_lane_off, (uint32_t)k1 * ROWB,
                        lds_wave + (2 + (1 - PAR)) * TILE);
      mask_if_tail(Y{}, k1);
      float mx[2];
      pipe_phase_b1<PAR>(v_addr, sc_t[PAR], m_ref, l, sc_t[1 - PAR], mx);
      new_tile_max(mx);
      // (barrier inside, in front of the last slab: K_{i+2} has landed; V_{i+1}, K_{i+3} may be in flight)
      pipe_phase_b2<PAR>(v_addr, k_addr, sc_t[1 - PAR], m_ref, l, Kres, k_lane_off0, k_lane_off1, (uint32_t)k3 * ROWB,
                         lds_wave + (1 - PAR) * TILE);
    };
    // The last sub-tile: nothing left to overlap with.
    auto stage_last = [&](auto par) {
      constexpr int PAR = decltype(par)::value;
      rescale_o_if_pending();
      pipe_softmax_part1<PAR>(sc_t[PAR], m_ref, l);
      wait_vmem<0>();
      pipe_barrier();
      pipe_pv_plain<PAR>(v_addr);
      pipe_barrier();  // the other wavefront has read its last V operands: the buffers may be reused
    };

    using T0 = std::integral_constant<int, 0>;
    using T1 = std::integral_constant<int, 1>;
    if (T > 0) {
      // ---- prologue: S_0, its maxima, first part of P_0
      wait_vmem<0>();
      pipe_barrier();  // every wave's share of K_0, V_0, K_1 has landed
      pipe_qk_first(k_addr);
      pipe_barrier();  // K buffer 0 is free again
      issue_k(2, key_of(2));
      mask_if_tail(T0{}, key_first);
      float mx[2];
      pipe_max_plain<0>(sc_t[0], mx);
      new_tile_max(mx);
      alpha_o[0] = alpha_o[1] = 1.0f;  // O is still zero: nothing to rescale for the first maxima
      pipe_softmax_part0<0>(sc_t[0], m_ref, l);
      pipe_k_preread<1>(k_addr);  // what a phase B2 does for the phase A behind it
      // first keys of the next four sub-tiles, kept in scalar registers; the next two are read from
      // LDS one loop iteration ahead of their use
      int k1 = key_of(1), k2 = key_of(2), k3 = key_of(3), k4 = key_of(4);
      int i = 0;
      for (; i + 2 < T; i += 2) {
        const u32x2 next = *reinterpret_cast<const u32x2 *>(keybuf + i + 4);  // sub-tiles i+5, i+6
        stage_full(T0{}, k1, k3);
        stage_full(T1{}, k2, k4);
        k1 = k3;
        k2 = k4;
        k3 = __builtin_amdgcn_readfirstlane(next[0]);
        k4 = __builtin_amdgcn_readfirstlane(next[1]);
      }
      if (T - i == 2) {
        stage_full(T0{}, k1, k3);
        stage_last(T1{});
      } else {
        stage_last(T0{});
      }
    }

    // ---- normalise, stage in LDS (K and V buffers), store to the block and its repeat targets
    const float l_tot0 = sum_with_other_half(l[0][0] + l[0][1]), l_tot1 = sum_with_other_half(l[1][0] + l[1][1]);
    pipe_store_o<0>(l_tot0 > 0.f ? 1.0f / l_tot0 : 0.f, o_addr0);
    pipe_store_o<1>(l_tot1 > 0.f ? 1.0f / l_tot1 : 0.f, o_addr1);
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

  if (counter && blockIdx.x == 0 && tid == 0) residency.store(counter);
  if (counter && tid == 0) {
    __threadfence();
    if (atomicAdd(counter + CALIBATT_GROUPS, 1) == (int)gridDim.x - 1) {
      for (int i = 0; i <= CALIBATT_GROUPS; ++i) counter[i] = 0;
      __threadfence();
    }
  }
}

}  // namespace calibatt_dev
