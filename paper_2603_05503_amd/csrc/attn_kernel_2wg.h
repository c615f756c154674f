// Block-sparse attention forward for gfx950 (MI355X), bf16 in / fp32 accumulate.
//
// What it computes (paper, Section 2 Eq. 1-4 restricted by the block mask of
// Section 3.2, run as in Section 3.4): for every computed query block r of a
// head, loop over the kept key/value blocks listed in the CSR pattern, form
// S = scale * Q_r K_c^T, fold it into a running row max / row sum (online
// softmax), accumulate O += P V_c, and finally write O / rowsum.  Skipped
// blocks are never loaded.  Query blocks marked as repeats (Section 3.3 at
// block granularity) are not computed: the workgroup that owns their source
// block writes its result to the source and to every block that copies it.
//
// Mapping to CDNA4:
//  * one workgroup per (work item, batch index); BQ/32 wavefronts, each owning
//    32 query rows;
//  * both contractions use v_mfma_f32_32x32x16_bf16 in the "transposed" form
//    S^T = K Q^T and O^T = V^T P^T, so that a lane owns ONE query column: the
//    row max / row sum are in-lane reductions plus one exchange with lane^32,
//    the rescale factor is a per-lane scalar, and the fp32 S^T accumulators
//    are, after conversion to bf16, exactly the B operand of the second MFMA
//    (no trip through LDS for P);
//  * K and V tiles go global -> LDS with global_load_lds_dwordx4 (no staging
//    registers).  K is read back with ds_read_b128 as the A operand; V stays
//    row-major and is read with the transposing ds_read_b64_tr_b16;
//  * both tiles are XOR-swizzled at 16-byte granularity (applied on the global
//    side of the direct load) so the MFMA operand reads are bank-conflict free;
//  * K and V have one LDS buffer each: K[i+1] streams in during softmax + PV of
//    tile i, V[i+1] during QK^T + softmax of tile i+1; two workgroups per CU
//    (64 KB LDS each at 128x128x128) let one workgroup's MFMAs overlap the
//    other's softmax VALU work;
//  * the epilogue stages the normalised bf16 tile in LDS and stores whole rows
//    with 16-byte accesses to the block itself and to all its repeat targets.
#pragma once
#include "attn_common.h"

namespace calibatt_dev {

// One workgroup's share of the forward: BQ query rows against a sequence of
// BK-key tiles.  Holds the per-lane state (Q^T operand, O^T accumulators,
// running max / sum) and the LDS addressing; the kernels decide which rows,
// which tiles, and where the result goes.
template <int D, int BQ, int BK, typename T = Bf16>
struct RowBlock {
  using Operand = u32x4;  // eight 16-bit elements of an MFMA operand, as raw bits
  static constexpr int NW = BQ / 32;     // wavefronts per workgroup
  static constexpr int NT = NW * 64;     // threads
  static constexpr int CH = D / 8;       // 16-byte chunks per row
  static constexpr int KB = BK / 32;     // 32-key sub-blocks per tile
  static constexpr int DS = D / 16;      // k-slabs of the QK^T contraction
  static constexpr int DB = D / 32;      // 32-wide d blocks of O^T
  static constexpr int ROWB = D * 2;     // bytes per LDS row
  static constexpr int TILE_BYTES = BK * ROWB;
  static constexpr int OST = ROWB + 16;  // padded row stride of the output staging tile
  static constexpr int LDS_BYTES = (2 * TILE_BYTES > BQ * OST) ? 2 * TILE_BYTES : BQ * OST;
  using LoadK = TileLoader<D, BK, NT, false>;
  using LoadV = TileLoader<D, BK, NT, true>;
  static constexpr int LOADS_PER_WAVE = LoadK::ITERS;  // direct-to-LDS instructions per wave and tile

  char *lds, *ldsK, *ldsV;
  int tid, lane, wave, l32, g;
  uint32_t k_lane_off, v_lane_off, ldsK_wave, ldsV_wave;
  uint32_t kv_row_bytes;  // distance between consecutive K (and V) rows in memory
  uint32_t k_addr0, v_addr[DB];
  Operand qreg[DS];  // Q^T as MFMA B operand: lane (query l32, half g) holds d = 16 s + 8 g + [0,8)
  f32x16 o[DB];
  float m_run;  // running max of scaled (log2-domain) logits, shared by lane and lane^32
  float l_run;  // this lane's share of the running row sum

  // tid_: index of the thread among the NT threads that share this row block
  __device__ __forceinline__ explicit RowBlock(char *lds_, uint32_t kv_row_bytes_ = ROWB, int tid_ = threadIdx.x)
      : lds(lds_), ldsK(lds_), ldsV(lds_ + TILE_BYTES), kv_row_bytes(kv_row_bytes_) {
    tid = tid_;
    lane = tid & 63;
    wave = tid >> 6;
    l32 = lane & 31;
    g = lane >> 5;
    k_lane_off = LoadK::lane_offset(tid, 0, kv_row_bytes);
    v_lane_off = LoadV::lane_offset(tid, 0, kv_row_bytes);
    const uint32_t lds_base = (uint32_t)(uintptr_t)(LDS_PTR(char))lds;
    const uint32_t wave_u = __builtin_amdgcn_readfirstlane(wave);
    ldsK_wave = lds_base + wave_u * 1024;
    ldsV_wave = ldsK_wave + TILE_BYTES;
    // K operand row for MFMA row i = l32: swap bits 2 and 3 so that the 8 S^T
    // values a lane holds per 16-key slab belong to 8 consecutive keys.  With the
    // XOR swizzle the address of k-slab s is k_addr0 ^ (s << 5).
    const int krow_in_kb = (l32 & 0x13) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);
    k_addr0 = krow_in_kb * ROWB + ((g ^ k_swz<D>(krow_in_kb)) << 4);
    // transposing V read: 16-lane block -> (d sub-block, key half); lane L16 in block
    const int L16 = lane & 15;
    const int blk = lane >> 4;
    const int v_row_off = 8 * (blk >> 1) + (L16 >> 2);  // + 32 kb + 16 s2 + 4 t
#pragma unroll
    for (int db = 0; db < DB; ++db)
      v_addr[db] = v_row_off * ROWB + (((4 * db + 2 * (blk & 1) + ((L16 & 3) >> 1)) ^ v_swz<D>(v_row_off)) << 4) +
                   (L16 & 1) * 8;
  }

  // Query row this lane owns within the block.
  __device__ __forceinline__ int row_in_block() const { return wave * 32 + l32; }

  __device__ __forceinline__ void issue_k(const u32x4 &Kres, int c) const {
    LoadK::issue(Kres, c * BK, ldsK_wave, tid, k_lane_off, kv_row_bytes);
  }
  // K tile c into the LDS window at byte offset `buf_off` (a multiple of TILE_BYTES)
  __device__ __forceinline__ void issue_k_at(const u32x4 &Kres, int c, uint32_t buf_off) const {
    LoadK::issue(Kres, c * BK, ldsK_wave + buf_off, tid, k_lane_off, kv_row_bytes);
  }
  __device__ __forceinline__ void issue_v(const u32x4 &Vres, int c) const {
    LoadV::issue(Vres, c * BK, ldsV_wave, tid, v_lane_off, kv_row_bytes);
  }

  // A query row as MFMA B operand: `qrow_ptr` points at the D bf16 of this lane's row.
  __device__ __forceinline__ void load_q(const uint16_t *qrow_ptr, Operand (&dst)[DS]) const {
    const uint16_t *qp = qrow_ptr + 8 * g;
#pragma unroll
    for (int s = 0; s < DS; ++s) dst[s] = *reinterpret_cast<const Operand *>(qp + 16 * s);
    // touch the registers here so that the compiler's wait for these loads sits
    // in front of the tile loop and not inside it
#pragma unroll
    for (int s = 0; s < DS; ++s) asm volatile("" : "+v"(dst[s]));
  }

  // Start a row block: `qrow_ptr` points at the D bf16 of this lane's query row.
  __device__ __forceinline__ void begin(const uint16_t *qrow_ptr) {
    load_q(qrow_ptr, qreg);
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
    m_run = -INFINITY;
    l_run = 0.f;
  }

  // S^T = K Q^T for the K tile at byte offset `buf_off` of the LDS window:
  // s_acc[kb][v] = dot(key 32 kb + 16 (v >> 3) + 8 g + (v & 7), query l32), unscaled.
  __device__ __forceinline__ void scores(uint32_t buf_off, f32x16 (&s_acc)[KB]) const { scores(buf_off, s_acc, qreg); }
  // The same against an explicit query operand (see load_q).
  __device__ __forceinline__ void scores(uint32_t buf_off, f32x16 (&s_acc)[KB], const Operand (&q)[DS]) const {
    const char *const kbuf = ldsK + buf_off;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) s_acc[kb][v] = 0.f;
    // k-slab outer, key sub-block inner: consecutive MFMAs hit different
    // accumulators; the A operands of slab s+1 are read while slab s multiplies.
    Operand ka[2][KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
      ka[0][kb] = *reinterpret_cast<const Operand *>(kbuf + (k_addr0 + kb * 32 * ROWB));
#pragma unroll
    for (int s = 0; s < DS; ++s) {
      if (s + 1 < DS) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
          ka[(s + 1) & 1][kb] =
              *reinterpret_cast<const Operand *>(kbuf + ((k_addr0 ^ ((s + 1) << 5)) + kb * 32 * ROWB));
      }
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
        s_acc[kb] = T::mfma(ka[s & 1][kb], q[s], s_acc[kb]);
    }
    __builtin_amdgcn_sched_group_barrier(0x100, KB, 0);  // LDS reads of slab 0
#pragma unroll
    for (int s = 0; s < DS; ++s) {
      if (s + 1 < DS) __builtin_amdgcn_sched_group_barrier(0x100, KB, 0);  // LDS reads of slab s+1
      __builtin_amdgcn_sched_group_barrier(0x008, KB, 0);                  // MFMAs of slab s
    }
  }

  // Fold key/value tile c into the running result.  On entry the K and V loads
  // of tile c are in flight (K issued first); if has_next, the loads of tile
  // c_next are issued as soon as the K resp. V buffer is free.  `sc` is
  // scale * log2(e); keys >= N (last, ragged tile: c == nbk - 1) get zero weight.
  __device__ __forceinline__ void tile(const u32x4 &Kres, const u32x4 &Vres, int c, bool has_next, int c_next, int N, int nbk,
                       float sc) {
    // ---- S^T = K Q^T --------------------------------------------------------
    // K[c] was issued before V[c]: V's loads may stay in flight.
    wait_vmem<LOADS_PER_WAVE>();
    __syncthreads();
    f32x16 s_acc[KB];
    // The matrix phases run at raised priority: when the SIMD's other wavefront (of the co-resident
    // workgroup) is in its softmax, the matrix pipe's issue slots go to this one first.
    __builtin_amdgcn_s_setprio(2);
    scores(0, s_acc);
    __builtin_amdgcn_s_setprio(0);
    __syncthreads();  // every wave is done with the K tile
    if (has_next) issue_k(Kres, c_next);

    // ---- online softmax (log2 domain) ----------------------------------------
    float sc_t = sc;  // multiplier still to be applied to s_acc
    if (c == nbk - 1 && (N % BK) != 0) {
      // ragged last block: scale now, put keys >= N at -inf, continue with multiplier 1
      int limit = N - c * BK - 8 * g;  // this lane's key offsets below `limit` exist
      // Opaque to the optimiser: hoisted out of the tile loop, the 64 comparisons below would be
      // evaluated for every row block and their masks would hold 128 scalar registers throughout.
      asm volatile("" : "+v"(limit));
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          s_acc[kb][v] = 32 * kb + 16 * (v >> 3) + (v & 7) < limit ? s_acc[kb][v] * sc : -INFINITY;
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
    const float m_new = fmaxf(m_run, m_loc);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);  // 0 on the first tile
    m_run = m_new;
    // P = exp2(sc * S - m) rounded to bf16 pairs; the row sum is taken over the
    // rounded values (two per v_dot2c with a vector of ones), so numerator and
    // denominator of the final division see the same probabilities.
    float psum = 0.f;
    uint32_t pb[KB][8];  // bf16 pairs: pb[kb][4*s2 + j] = keys (2j, 2j+1) of 16-key slab s2
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int v = 0; v < 16; v += 2) {
        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[kb][v], sc_t, -m_new));
        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[kb][v + 1], sc_t, -m_new));
        const uint32_t pk = T::pack(p0, p1);
        pb[kb][v >> 1] = pk;
        psum = T::add_pair(pk, psum);
      }
    l_run = l_run * alpha + psum;
    if (__any(alpha != 1.0f)) {
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[db][v] *= alpha;
    }

    // ---- O^T += V^T P^T -----------------------------------------------------
    if (has_next) wait_vmem<LOADS_PER_WAVE>(); else wait_vmem<0>();
    __syncthreads();
    __builtin_amdgcn_s_setprio(2);
    {
      // 16-key slab j = 2 kb + s2: V^T operands of slab j+1 are read while slab j multiplies
      u32x4 va[2][DB];
      auto v_read = [&](int j, int st) {
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const char *a = ldsV + v_addr[db] + 16 * j * ROWB;
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

#pragma unroll
        for (int db = 0; db < DB; ++db)
          o[db] = T::mfma(va[j & 1][db], pw, o[db]);
      }
      __builtin_amdgcn_sched_group_barrier(0x100, 2 * DB, 0);
#pragma unroll
      for (int j = 0; j < 2 * KB; ++j) {
        if (j + 1 < 2 * KB) __builtin_amdgcn_sched_group_barrier(0x100, 2 * DB, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, DB, 0);
      }
    }
    __builtin_amdgcn_s_setprio(0);
    __syncthreads();  // every wave is done with the V tile
    if (has_next) issue_v(Vres, c_next);
  }

  // Normalise and stage the BQ x D result in LDS: row i at lds + i * OST.
  // A row that saw no key is all zero.  Ends with a barrier: the tile is
  // complete for every thread on return.  Returns the natural logarithm of the
  // sum of exp(scaled logit) over the keys this lane's row saw (-inf for none).
  __device__ __forceinline__ float stage_result() {
    const float l_tot = sum_with_other_half(l_run);
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    __syncthreads();
    char *orow = lds + (wave * 32 + l32) * OST;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        u32x2 w;
        w[0] = T::pack(o[db][4 * a + 0] * inv, o[db][4 * a + 1] * inv);
        w[1] = T::pack(o[db][4 * a + 2] * inv, o[db][4 * a + 3] * inv);
        *reinterpret_cast<u32x2 *>(orow + (32 * db + 8 * a + 4 * g) * 2) = w;
      }
    __syncthreads();
    // m_run is the maximum of the logits times log2(e), l_tot the sum of 2^(logit - m_run)
    return l_tot > 0.f ? (m_run + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f : -INFINITY;
  }

  // Result over a PART of the keys, for a later merge with the other parts: the
  // rows normalised by their own sum as fp32 (rows[row_in_block][D]) and the
  // natural logarithm of that sum (row_lse[row_in_block], -inf and a zero row
  // when no key was seen), straight from the accumulators to global memory.
  __device__ __forceinline__ void store_partial(float *rows, float *row_lse) const {
    const float l_tot = sum_with_other_half(l_run);
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    float *orow = rows + (size_t)(wave * 32 + l32) * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        f32x4 w;
#pragma unroll
        for (int j = 0; j < 4; ++j) w[j] = o[db][4 * a + j] * inv;
        *reinterpret_cast<f32x4 *>(orow + 32 * db + 8 * a + 4 * g) = w;
      }
    if (g == 0)
      row_lse[wave * 32 + l32] = l_tot > 0.f ? (m_run + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f : -INFINITY;
  }
};

// Kept-block columns of a row held in LDS when the pattern comes as intervals
// (IV = true): this many at a time, behind the work-item mailbox.
constexpr int IV_COLS = 2048;

// IV = false: the kept key blocks of a row are read from col_idx (row_ptr gives
// the slice).  IV = true: col_idx is not touched; `iv_ptr` / `iv` hold every
// row as runs of consecutive key blocks, one word per run (low half = first
// block, high half = kept blocks of the row before the run) plus a terminating
// word per row, and the workgroup expands them into LDS.
// T: element type of q, k, v, out (Bf16 or F16).  lse: NULL, or fp32 [B][H][N] (tensor heads)
// receiving per query the natural log of the sum of exp(scaled logit) over its kept keys.
template <int D, int BQ, int BK, bool IV = false, typename T = Bf16>
__global__ __launch_bounds__(BQ * 2, (BQ >= 128 ? 2 : 1)) void sparse_attn_fwd_kernel(
    const uint16_t *__restrict__ gq, const uint16_t *__restrict__ gk, const uint16_t *__restrict__ gv,
    uint16_t *__restrict__ gout, const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx,
    const int32_t *__restrict__ work, const int32_t *__restrict__ fan_ptr, const int32_t *__restrict__ fan_dst,
    int32_t *counter, const FwdDims p, const int32_t *__restrict__ iv_ptr, const uint32_t *__restrict__ iv,
    const int32_t *__restrict__ head_map, float *__restrict__ lse) {
  using RB = RowBlock<D, BQ, BK, T>;
  constexpr int NT = RB::NT, CH = RB::CH, ROWB = RB::ROWB, OST = RB::OST, LDS_BYTES = RB::LDS_BYTES;

  // LDS_BYTES + 64 (work-item mailbox) [+ IV_COLS * 4 (column list) if IV]
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  int *const cols = reinterpret_cast<int *>(lds + LDS_BYTES + 64);
  RB rb(lds, (uint32_t)p.in.n * 2);
  const int tid = rb.tid;
  const int lane = rb.lane;
  const int N = p.N;
  const int n_items = p.n_work * p.B;
  volatile int *const mailbox = reinterpret_cast<volatile int *>(lds + LDS_BYTES);
  // Persistent workgroups (counter != nullptr): every workgroup pops (work item,
  // batch index) pairs from per-group counters until all groups are drained, so
  // uneven rows balance dynamically.  With one group per XCD a workgroup starts
  // on the group of the XCD it runs on (the heads of a group then share that
  // XCD's L2) and moves on to the next group, for good, once one is empty.
  // Otherwise: one workgroup per pair.
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
  // h is the head of the pattern; the tensors' head may differ (pattern over a subset of heads).
  // An entry outside the tensor's heads is treated as head 0 for the reads and writes nothing.
  const int h_raw = head_map ? head_map[h] : h;
  const bool head_ok = (unsigned)h_raw < (unsigned)p.H;
  const int ht = head_ok ? h_raw : 0;
  // q, k, v: element (b, h, n, d) at b * in.b + h * in.h + n * in.n + d; out likewise with `out`
  const size_t head_off = (size_t)b * p.in.b + (size_t)ht * p.in.h;
  const uint32_t head_bytes = (uint32_t)(N - 1) * rb.kv_row_bytes + ROWB;  // first byte after the last row
  const u32x4 Kres = head_rsrc(gk + head_off, head_bytes);
  const u32x4 Vres = head_rsrc(gv + head_off, head_bytes);

  const int cbeg = row_ptr[id];
  const int cend = row_ptr[id + 1];

  // The row's kv-block list is held 64 entries at a time in one VGPR (lane j =
  // entry j) and read back with v_readlane: no memory operation per tile.
  const int n_tiles = cend - cbeg;
  // IV: entries [chunk_lo, chunk_lo + IV_COLS) of the list are expanded from the
  // row's runs into LDS; every thread takes runs tid, tid + NT, ...
  int chunk_lo = 0;
  auto expand_runs = [&]() {
    const int ib = iv_ptr[id], ie = iv_ptr[id + 1] - 1;  // the last word only terminates the row
    for (int i = ib + tid; i < ie; i += NT) {
      const uint32_t w = iv[i], w_next = iv[i + 1];
      const int start = (int)(w & 0xffffu), before = (int)(w >> 16), len = (int)(w_next >> 16) - before;
      const int j0 = max(0, chunk_lo - before), j1 = min(len, chunk_lo + IV_COLS - before);
      for (int j = j0; j < j1; ++j) cols[before + j - chunk_lo] = start + j;
    }
    __syncthreads();
  };
  auto col_at = [&](int entry) { return IV ? cols[entry - chunk_lo] : col_idx[cbeg + entry]; };
  if constexpr (IV) expand_runs();  // the previous item's readers are behind the barrier that ended it
  int col_cache = n_tiles > 0 ? col_at(min(lane, n_tiles - 1)) : 0;
  // first K and V tiles
  int c_next = 0;
  if (n_tiles > 0) {
    c_next = __builtin_amdgcn_readlane(col_cache, 0);
    rb.issue_k(Kres, c_next);
    rb.issue_v(Vres, c_next);
  }
  {
    int qrow = r * BQ + rb.row_in_block();
    qrow = qrow < N ? qrow : N - 1;
    rb.begin(gq + head_off + (size_t)qrow * p.in.n);
  }
  const float sc = p.scale_log2e;

  for (int ti = 0; ti < n_tiles; ++ti) {
    const int c = c_next;
    const bool has_next = ti + 1 < n_tiles;
    if (has_next) {
      if (((ti + 1) & 63) == 0) {
        if constexpr (IV) {
          if ((ti + 1) % IV_COLS == 0) {
            __syncthreads();  // every wave has taken its entries of the chunk that is replaced
            chunk_lo = ti + 1;
            expand_runs();
          }
        }
        col_cache = col_at(min(ti + 1 + lane, n_tiles - 1));
      }
      c_next = __builtin_amdgcn_readlane(col_cache, (ti + 1) & 63);
    }

    rb.tile(Kres, Vres, c, has_next, c_next, N, p.nbk, sc);
  }

  // ---- normalise, stage in LDS, store to the block and its repeat targets ----
  const float row_lse = rb.stage_result();
  const int fbeg = fan_ptr[item];
  const int fend = fan_ptr[item + 1];
  if (lse && head_ok && rb.g == 0) {  // one lane per query row; repeated blocks copy the value as well
    float *const lse_head = lse + ((size_t)b * p.H + ht) * (size_t)N;
    for (int f = fbeg - 1; f < fend; ++f) {
      const int row = (f < fbeg ? r : fan_dst[f]) * BQ + rb.row_in_block();
      if (row < N) lse_head[row] = row_lse;
    }
  }
  uint16_t *const out_head = gout + (size_t)b * p.out.b + (size_t)ht * p.out.h;
  for (int f = fbeg - 1; head_ok && f < fend; ++f) {
    const int rd = f < fbeg ? r : fan_dst[f];
    const int rows_valid = min(BQ, N - rd * BQ);
    uint16_t *dst = out_head + (size_t)rd * BQ * p.out.n;
#pragma unroll 4
    for (int L = tid; L < BQ * CH; L += NT) {
      const int row = L / CH;
      const int cc = L % CH;
      if (row < rows_valid) {
        const u32x4 val = *reinterpret_cast<const u32x4 *>(lds + row * OST + cc * 16);
        *reinterpret_cast<u32x4 *>(dst + (size_t)row * p.out.n + cc * 8) = val;
      }
    }
  }
  if (!counter) break;
  __syncthreads();  // staging tile fully read before the next item's loads overwrite it
  }  // work-item loop

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
