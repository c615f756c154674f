// Block-sparse attention forward for gfx950, "ping-pong" variant: one workgroup
// of TWO wavefront groups per CU, two wavefronts per SIMD, which alternate
// between a matrix phase and a softmax phase.
//
// What it computes is the same as the two-workgroup kernel (paper, Section 2
// Eq. 1-4 restricted to the kept blocks of Section 3.2, run as in Section 3.4;
// repeated query blocks of Section 3.3 written by the owner of their source).
//
// Why: measured on this hardware, VALU work (also transcendental and dot
// instructions) of one wavefront runs at full rate beside the MFMAs of ANOTHER
// wavefront of the same SIMD without slowing them down, while VALU work woven
// between the MFMAs of the SAME wavefront is not hidden.  So the softmax of one
// wavefront is placed, by construction, beside the MFMAs of its SIMD partner:
//
//   both groups own the same BQ queries (wavefront w of either group: queries
//   32 w .. 32 w + 31) and split every kept kv block: group 0 takes its first
//   BK/2 keys, group 1 the other half (a "tile" below is such a half block).
//   Each keeps its own running maximum, row sum and O; the two partial results
//   are merged at the end (the usual split-softmax merge), in a fixed order, so
//   results are the same on every run, and both groups always have the same
//   amount of work.
//
//   Time is cut into intervals by workgroup barriers.  In an interval one group
//   runs a matrix phase - O += V^T P of its previous tile, then S = K Q^T of
//   its next tile, 32 MFMAs per wavefront at 128 x 128 x 128 - while the other
//   runs the softmax of its current tile (row maximum, exp2, rounding to bf16,
//   row sum, rescale of O) and issues direct-to-LDS loads.  At the barrier they
//   swap.  There is no other barrier.  K and V tiles are double-buffered per
//   group: the loads issued in the softmax phase of tile j are the K tile j+2
//   and the V tile j+1, first needed three intervals later.
//
// LDS: per group two K and two V tiles (8 x BK/2 x D x 2 bytes in all), then the
// merge area for the row statistics of group 1, then the work-item mailbox.
// Group 1's partial O goes through its own (then free) tiles; the output staging
// tile overlays group 0's.
#pragma once
#include "attn_common.h"

namespace calibatt_dev {

template <int D, int BQ, int BK>
struct PpLds {
  static constexpr int SUB = BK / 2;                     // keys per tile (half a kv block)
  static constexpr int TILE = SUB * D * 2;
  static constexpr int STATS = 8 * TILE;                 // float2 {m, l} per thread of a group
  static constexpr int MAILBOX = STATS + BQ * 2 * 8;
  static constexpr int BYTES = MAILBOX + 64;
};

template <int D, int BQ, int BK>
__global__ __launch_bounds__(BQ * 4, 1) void sparse_attn_fwd_pp_kernel(
    const uint16_t *__restrict__ gq, const uint16_t *__restrict__ gk, const uint16_t *__restrict__ gv,
    uint16_t *__restrict__ gout, const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx,
    const int32_t *__restrict__ work, const int32_t *__restrict__ fan_ptr, const int32_t *__restrict__ fan_dst,
    int32_t *counter, const FwdDims p) {
  static_assert(BQ <= BK, "group 1's partial O must fit into its K and V tiles");
  constexpr int GT = BQ * 2;      // threads per group (BQ / 32 wavefronts)
  constexpr int NT = 2 * GT;      // threads per workgroup
  constexpr int CH = D / 8;       // 16-byte chunks per row
  using Lds = PpLds<D, BQ, BK>;
  constexpr int SUB = Lds::SUB;   // keys per tile
  constexpr int KB = SUB / 32;    // 32-key sub-blocks per tile
  constexpr int DS = D / 16;      // k-slabs of the QK^T contraction
  constexpr int DB = D / 32;      // 32-wide d blocks of O^T
  constexpr int ROWB = D * 2;     // bytes per LDS row
  constexpr int TILE_BYTES = Lds::TILE;
  constexpr int OST = ROWB + 16;  // padded row stride of the output staging tile
  static_assert(BQ * OST <= 4 * TILE_BYTES, "output staging must fit into group 0's tiles");
  static_assert(SUB % 32 == 0, "a tile is made of 32-key sub-blocks");
  using LoadK = TileLoader<D, SUB, GT, false>;
  using LoadV = TileLoader<D, SUB, GT, true>;
  constexpr int LPW = LoadK::ITERS;  // direct-to-LDS instructions per wave and tile
  static_assert(2 * LPW == 2 || 2 * LPW == 4 || 2 * LPW == 8 || 2 * LPW == 16, "no s_waitcnt immediate for this shape");

  extern __shared__ __attribute__((aligned(1024))) char lds[];

  const int tid = threadIdx.x;
  const int grp = __builtin_amdgcn_readfirstlane(tid / GT);  // wavefront group 0 / 1 (wave-uniform)
  const int tg = tid % GT;         // thread within the group
  const int lane = tid & 63;
  const int wave = tg >> 6;        // wavefront within the group: queries 32 wave .. 32 wave + 31
  const int l32 = lane & 31;
  const int g = lane >> 5;

  char *const ldsK = lds + grp * 4 * TILE_BYTES;  // K buffers 0, 1
  char *const ldsV = ldsK + 2 * TILE_BYTES;       // V buffers 0, 1
  const uint32_t k_lane_off = LoadK::lane_offset(tg, 0);
  const uint32_t v_lane_off = LoadV::lane_offset(tg, 0);
  const uint32_t lds_base = (uint32_t)(uintptr_t)(LDS_PTR(char))lds;
  const uint32_t wave_u = __builtin_amdgcn_readfirstlane(tid >> 6);  // wavefront within the workgroup
  const uint32_t ldsK_wave = lds_base + (wave_u / (GT / 64)) * 4 * TILE_BYTES + (wave_u % (GT / 64)) * 1024;
  const uint32_t ldsV_wave = ldsK_wave + 2 * TILE_BYTES;
  const int N = p.N;
  const int n_items = p.n_work * p.B;
  volatile int *const mailbox = reinterpret_cast<volatile int *>(lds + Lds::MAILBOX);

  int cur_group = 0, groups_left = p.n_groups;
  if (counter && p.n_groups > 1)
    cur_group = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) % p.n_groups;  // HW_REG_XCC_ID[3:0]
  ResidencyClock residency;
  residency.start();

  // MFMA operand addresses inside a tile (see the two-workgroup kernel for the derivation)
  const int krow_in_kb = (l32 & 0x13) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);
  const uint32_t k_addr0 = krow_in_kb * ROWB + ((g ^ k_swz<D>(krow_in_kb)) << 4);
  const int L16 = lane & 15;
  const int blk = lane >> 4;
  const int v_row_off = 8 * (blk >> 1) + (L16 >> 2);
  // address of d block 0; the XOR swizzle makes the one of d block db equal to v_addr0 ^ (db << 6)
  // (4 db lands on the chunk-index bits that the swizzle flips; registers are scarce here)
  const uint32_t v_addr0 = v_row_off * ROWB + (((2 * (blk & 1) + ((L16 & 3) >> 1)) ^ v_swz<D>(v_row_off)) << 4) +
                           (L16 & 1) * 8;
  const float sc = p.scale_log2e;

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
    const int n_tiles = row_ptr[id + 1] - cbeg;  // kept blocks = tiles of either group

    // The row's kv blocks, 64 entries at a time in one VGPR (lane j = entry j), read back with
    // v_readlane: no memory operation per tile.  Tile j of this group = keys [first_key(j), + SUB).
    int win = 0;  // the VGPR window holds entries win .. win + 63
    auto load_cols = [&](int j0) { return col_idx[cbeg + min(j0 + lane, n_tiles - 1)]; };
    int col_cache = n_tiles > 0 ? load_cols(0) : 0;
    auto first_key = [&](int j) { return __builtin_amdgcn_readlane(col_cache, j - win) * BK + grp * SUB; };
    auto issue_k = [&](int j, int key) { LoadK::issue(Kres, key, ldsK_wave + (j & 1) * TILE_BYTES, tg, k_lane_off); };
    auto issue_v = [&](int j, int key) { LoadV::issue(Vres, key, ldsV_wave + (j & 1) * TILE_BYTES, tg, v_lane_off); };
    if (n_tiles > 0) {
      issue_k(0, first_key(0));
      issue_v(0, first_key(0));
      if (n_tiles > 1) issue_k(1, first_key(1));
    }

    // Q^T as MFMA B operand: lane (query l32, half g) holds d = 16 s + 8 g + [0,8)
    bf16x8 qreg[DS];
    {
      int qrow = r * BQ + wave * 32 + l32;
      qrow = qrow < N ? qrow : N - 1;
      const uint16_t *qp = gq + head_off + (size_t)qrow * D + 8 * g;
#pragma unroll
      for (int s = 0; s < DS; ++s) qreg[s] = *reinterpret_cast<const bf16x8 *>(qp + 16 * s);
#pragma unroll
      // wait for Q (and the first tiles) here
      for (int s = 0; s < DS; ++s) asm volatile("" : "+v"(qreg[s]));
    }

    f32x16 o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
    float m_run = -INFINITY;  // running max of scaled (log2-domain) logits, shared by lane and lane^32
    float l_run = 0.f;        // this lane's share of the running row sum
    f32x16 s_acc[KB];         // S^T of the current tile
    uint32_t pb[KB][8];       // its probabilities as bf16 pairs: pb[kb][4*s2 + j] = keys (2j, 2j+1) of 16-key slab s2

    // ---- the two halves of a matrix phase ------------------------------------------------------
    auto pv_product = [&](int buf) {  // O^T += V^T P^T with the tile in V buffer buf
      const char *const tile = ldsV + buf * TILE_BYTES;
      u32x4 va[2][DB];
      auto v_read = [&](int j, int st) {
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const char *a = tile + (v_addr0 ^ (db << 6)) + 16 * j * ROWB;
          const u32x2 lo = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_PTR(bf16x4))(a)));
          const u32x2 hi =
              __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_PTR(bf16x4))(a + 4 * ROWB)));
          va[st][db] = u32x4{lo[0], lo[1], hi[0], hi[1]};
        }
      };
      v_read(0, 0);
#pragma unroll
      for (int j = 0; j < 2 * KB; ++j) {
        if (j + 1 < 2 * KB) v_read(j + 1, (j + 1) & 1);
        const int kb = j >> 1, s2 = j & 1;
        const u32x4 pw = {pb[kb][4 * s2 + 0], pb[kb][4 * s2 + 1], pb[kb][4 * s2 + 2], pb[kb][4 * s2 + 3]};
        const bf16x8 pB = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
        for (int db = 0; db < DB; ++db)
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, va[j & 1][db]), pB, o[db], 0, 0, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x100, 2 * DB, 0);
#pragma unroll
      for (int j = 0; j < 2 * KB; ++j) {
        if (j + 1 < 2 * KB) __builtin_amdgcn_sched_group_barrier(0x100, 2 * DB, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, DB, 0);
      }
    };
    auto qk_product = [&](int buf) {  // S^T = K Q^T with the tile in K buffer buf
      const char *const tile = ldsK + buf * TILE_BYTES;
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) s_acc[kb][v] = 0.f;
      bf16x8 ka[2][KB];
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
        ka[0][kb] = *reinterpret_cast<const bf16x8 *>(tile + (k_addr0 + kb * 32 * ROWB));
#pragma unroll
      for (int s = 0; s < DS; ++s) {
        if (s + 1 < DS) {
#pragma unroll
          for (int kb = 0; kb < KB; ++kb)
            ka[(s + 1) & 1][kb] =
                *reinterpret_cast<const bf16x8 *>(tile + ((k_addr0 ^ ((s + 1) << 5)) + kb * 32 * ROWB));
        }
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
          s_acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[s & 1][kb], qreg[s], s_acc[kb], 0, 0, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x100, KB, 0);
#pragma unroll
      for (int s = 0; s < DS; ++s) {
        if (s + 1 < DS) __builtin_amdgcn_sched_group_barrier(0x100, KB, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, KB, 0);
      }
    };
    // ---- the softmax phase of this group's tile j (first key key0) --------------------------------
    auto softmax_phase = [&](int j, int key0) {
      // loads first: K buffer j & 1 was read by the product just finished, V buffer (j+1) & 1 by the
      // one before
      if (j + 2 < n_tiles) issue_k(j + 2, first_key(j + 2));
      if (j + 1 < n_tiles) issue_v(j + 1, first_key(j + 1));
      float sc_t = sc;  // multiplier still to be applied to s_acc
      if (key0 + SUB > N) {
        // ragged end of the sequence: scale now, put keys >= N at -inf, continue with multiplier 1
        const int k0 = key0 + 8 * g;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int key = k0 + 32 * kb + 16 * (v >> 3) + (v & 7);
            s_acc[kb][v] = key < N ? s_acc[kb][v] * sc : -INFINITY;
          }
        sc_t = 1.0f;
      }
      float m_loc;
      if (sc_t >= 0.f) {
        m_loc = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) m_loc = fmaxf(m_loc, s_acc[kb][v]);
      } else {
        m_loc = INFINITY;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) m_loc = fminf(m_loc, s_acc[kb][v]);
      }
      m_loc = max_with_other_half(m_loc * sc_t);
      // The reference maximum only moves when the tile's row maximum exceeds it by more than 8 in
      // the log2 domain (probabilities then stay below 2^8: no overflow, same relative precision in
      // bf16), which makes the rescale of O and of the row sum below a rare, wave-uniform branch.
      // (A tile wholly past the end of the sequence has m_loc = -inf and changes nothing.)
      const bool up = m_loc > m_run + 8.0f;
      const float m_new = up ? m_loc : m_run;
      const float alpha = up ? __builtin_amdgcn_exp2f(m_run - m_new) : 1.0f;  // 0 on the first tile
      const float m_sub = m_new == -INFINITY ? 0.f : m_new;
      m_run = m_new;
      // P = exp2(sc * S - m) rounded to bf16 pairs; the row sum is taken over the rounded values
      // (two per v_dot2c with a vector of ones), so numerator and denominator of the final
      // division see the same probabilities.
      float psum = 0.f;
      const bf16x2 ones = __builtin_bit_cast(bf16x2, 0x3f803f80u);
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int v = 0; v < 16; v += 2) {
          const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[kb][v], sc_t, -m_sub));
          const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[kb][v + 1], sc_t, -m_sub));
          const uint32_t pk = pack_bf16(p0, p1);
          pb[kb][v >> 1] = pk;
          psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk), ones, psum, false);
        }
      l_run = l_run * alpha + psum;
      if (__any(alpha != 1.0f)) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int v = 0; v < 16; ++v) o[db][v] *= alpha;
      }
      // what the next matrix phase reads (V tile j, K tile j+1) was issued one softmax phase ago:
      // all but the loads just issued must have landed
      if (j + 2 < n_tiles) wait_vmem<2 * LPW>();
      else if (j + 1 < n_tiles) wait_vmem<LPW>();
      else wait_vmem<0>();
    };

    // ---- intervals: group 0 runs its matrix phases in the even ones, group 1 in the odd ones; both
    //      pass 2 n_tiles + 2 barriers.  Written out per group so that each loop body is straight-line.
    wait_vmem<0>();
    __syncthreads();  // the first tiles have landed
    auto softmax_of = [&](int j) {
      if (j + 2 >= win + 64) {  // the phase looks two tiles ahead: slide the window of kv blocks
        win = j;
        col_cache = load_cols(win);
      }
      softmax_phase(j, first_key(j));
    };
    auto matrix_phase = [&](int j) {  // O += V^T P of tile j-1, then S = K Q^T of tile j
      __builtin_amdgcn_s_setprio(2);
      pv_product((j - 1) & 1);
      qk_product(j & 1);
      __builtin_amdgcn_s_setprio(0);
    };
    if (n_tiles > 0) {
      if (grp == 0) {
        qk_product(0);
        __syncthreads();
        for (int j = 0; j + 1 < n_tiles; ++j) {
          softmax_of(j);
          __syncthreads();
          matrix_phase(j + 1);
          __syncthreads();
        }
        softmax_of(n_tiles - 1);
        __syncthreads();
        pv_product((n_tiles - 1) & 1);
        __syncthreads();
        __syncthreads();
      } else {
        __syncthreads();
        qk_product(0);
        __syncthreads();
        softmax_of(0);
        __syncthreads();
        for (int j = 1; j < n_tiles; ++j) {
          matrix_phase(j);
          __syncthreads();
          softmax_of(j);
          __syncthreads();
        }
        pv_product((n_tiles - 1) & 1);
        __syncthreads();
      }
    }

    // ---- merge the two groups' partial results, normalise, stage, store ---------------------------
    float2 *const stats = reinterpret_cast<float2 *>(lds + Lds::STATS);
    float *const o_part = reinterpret_cast<float *>(lds + 4 * TILE_BYTES);  // group 1's tiles
    if (grp == 1) {
      stats[tg] = make_float2(m_run, l_run);
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o_part[(db * 16 + v) * GT + tg] = o[db][v];
    }
    __syncthreads();
    if (grp == 0) {
      const float2 other = stats[tg];
      const float m_tot = fmaxf(m_run, other.x);
      // a group without tiles has m = -inf, l = 0, O = 0: its factor is irrelevant but must not be NaN
      const float fa = m_run == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_run - m_tot);
      const float fb = other.x == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(other.x - m_tot);
      const float l_tot = sum_with_other_half(l_run * fa + other.y * fb);
      const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
      char *orow = lds + (wave * 32 + l32) * OST;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
          float e[4];
#pragma unroll
          for (int u = 0; u < 4; ++u)
            e[u] = (o[db][4 * a + u] * fa + o_part[(db * 16 + 4 * a + u) * GT + tg] * fb) * inv;
          u32x2 w;
          w[0] = pack_bf16(e[0], e[1]);
          w[1] = pack_bf16(e[2], e[3]);
          *reinterpret_cast<u32x2 *>(orow + (32 * db + 8 * a + 4 * g) * 2) = w;
        }
    }
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
  // Last workgroup out re-arms the counters for the next launch.
  if (counter && tid == 0) {
    __threadfence();
    if (atomicAdd(counter + CALIBATT_GROUPS, 1) == (int)gridDim.x - 1) {
      for (int i = 0; i <= CALIBATT_GROUPS; ++i) counter[i] = 0;
      __threadfence();
    }
  }
}

}  // namespace calibatt_dev
