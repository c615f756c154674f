// Block-sparse attention forward, interleaved schedule: every wavefront runs
// its MFMAs and its softmax as ONE instruction stream.
//
// Same computation per query block as attn_kernel_2wg.h (paper, Section 2
// Eq. 1-4 under the block mask of Section 3.2, repeated query blocks written
// as copies, Section 3.3 / 3.4); the online softmax moves the reference of
// its exponentials lazily (see IlRow::softmax_op), which changes roundings but
// not what is computed.
//
// Why.  On this hardware a wavefront issues a vector-ALU instruction only
// every 5-8 cycles, and the softmax of a 128-key tile is ~225 of them: with
// the three phases of a tile (S = K Q^T, softmax, O += P V) run one after the
// other, a wavefront spends more time in its softmax than in its MFMAs, and
// two wavefronts per SIMD keep the matrix pipe only about 60 % busy however
// their phases happen to fall.  But an MFMA occupies the pipe for 32 cycles
// and its wavefront can issue a few other instructions meanwhile.  So here a
// kept key block is cut into sub-tiles of 64 keys (32 where the block is not
// a multiple of 64 or is 64 keys itself), a row's kept blocks become one
// stream of sub-tiles, and in every STAGE a wavefront issues, interleaved
// instruction by instruction,
//     the MFMAs of  O += P V  of the sub-tile before the previous one,
//     the MFMAs of  S = K Q^T of the next sub-tile,
//     the vector instructions of the softmax of the previous sub-tile
// (about four vector instructions behind every MFMA).  The chain of one
// wavefront per tile is then little longer than its MFMAs alone, and the two
// wavefronts per SIMD (two workgroups per CU, as in attn_kernel_2wg.h)
// together keep the matrix pipe fed.  One workgroup barrier per stage.
//
// Registers (256 per wavefront).  The compiler gets 72 arch VGPRs (addresses,
// softmax temporaries); the rest is addressed BY NAME from inline assembly
// (attn_named_regs.h):
//   v[72 .. 72 + 2 * 16 KBS)  S^T of two sub-tiles (16 per 32-key sub-block);
//                             the softmax overwrites elements 0..7 of each
//                             sub-block with its probabilities as packed
//                             pairs, the B operand of the second contraction
//   a[0 .. 16 DB)             O^T accumulators
//   a[A_ST .. A_ST + 24)      six 4-register slots for MFMA A operands read
//                             from LDS four instructions ahead of their use
//   a[A_Q .. A_Q + 4 DS)      Q^T of the row block (B operand of S = K Q^T)
// Hazards the assembler does not police, kept by construction: an MFMA result
// is read by the vector ALU only in a later stage, behind s_nops and the
// barrier; an LDS read is consumed behind an s_waitcnt counting the reads
// issued after it; a staging slot is refilled two MFMAs after the one that
// read it was issued; a transcendental's result is read at least four vector
// instructions later; a dot product's result is read by another kind of
// instruction only behind an s_nop.
#pragma once
#include "attn_kernel_2wg.h"
#include "attn_named_regs.h"

namespace calibatt_dev {

// The reference of the exponentials moves only when a logit exceeds it by more
// than this (log2 domain): probabilities stay below 2^8, far inside the bf16 /
// fp16 range, and keep their full relative precision.
constexpr float IL_REF_SLACK = 8.0f;
constexpr int IL_VGPRS = 72;  // arch VGPRs left to the compiler; the named ones follow
constexpr int IL_STAGES = 6;  // operand staging slots
constexpr int IL_AHEAD = 4;   // MFMAs between the issue of an operand's LDS reads and its use

// Keys per sub-tile for a key block of BK keys: the block is a whole number of sub-tiles (two for
// the power-of-two widths; three or five for 96, 160 and 192).
constexpr __host__ __device__ int il_sub(int bk) { return bk >= 128 && bk % 64 == 0 ? 64 : 32; }

// The base class lays out LDS and lanes for a window of two sub-tiles of K and of V.
template <int D, int BQ, int BK, typename T = Bf16>
struct IlRow : RowBlock<D, BQ, 2 * il_sub(BK), T> {
  using RB = RowBlock<D, BQ, 2 * il_sub(BK), T>;
  using RB::DB;
  using RB::DS;
  using RB::ROWB;
  static constexpr int SUB = il_sub(BK);         // keys per sub-tile
  static constexpr int SPB = BK / SUB;           // sub-tiles per key block
  static_assert(BK % SUB == 0 && SPB >= 2, "a key block is a whole number of sub-tiles");
  static constexpr int KBS = SUB / 32;           // 32-key sub-blocks per sub-tile
  static_assert(KBS >= 1, "sub-tiles of at least 32 keys");
  static constexpr int EL = 16 * KBS;            // S^T elements per lane and sub-tile
  static constexpr int SUB_BYTES = SUB * ROWB;   // LDS bytes of a K or V sub-tile
  static constexpr int V_S = IL_VGPRS;           // S^T buffer p at v[V_S + p * EL ...)
  static constexpr int A_O = 0, A_ST = 16 * DB, A_Q = A_ST + 4 * IL_STAGES, N_AGPR = A_Q + 4 * DS;
  static_assert(V_S + 2 * EL + N_AGPR <= 256, "register map does not fit");
  static constexpr int N_PV = 2 * KBS * DB, N_QK = DS * KBS;  // MFMAs of the two contractions of a sub-tile
  using LoadKs = TileLoader<D, SUB, RB::NT, false>;
  using LoadVs = TileLoader<D, SUB, RB::NT, true>;
  static constexpr int LOADS_PER_WAVE = LoadKs::ITERS;

  uint32_t k_base, v_base[DB];  // LDS byte addresses of this lane's operand pieces in K / V slot 0
  // softmax state of the row (per lane; lanes l and l^32 share a query)
  float sc;          // |scale| * log2(e) (a negative scale is folded into the sign of Q)
  float alpha;       // factor by which O and the row sum shrink at the end of the current stage
  float psum[2];     // row sum of the sub-tile being exponentiated
  float part[4], rm, neg_ref;
  float x[8];

  __device__ __forceinline__ IlRow(char *lds_, uint32_t kv_row_bytes_) : RB(lds_, kv_row_bytes_) {
    const uint32_t lds_base = (uint32_t)(uintptr_t)(LDS_PTR(char))lds_;  // a multiple of 1024
    k_base = lds_base + this->k_addr0;
#pragma unroll
    for (int db = 0; db < DB; ++db) v_base[db] = lds_base + RB::TILE_BYTES + this->v_addr[db];
  }

  // K / V rows [row0, row0 + SUB) of the head into slot `slot` (0 or 1) of the K / V window
  __device__ __forceinline__ void issue_k_sub(const u32x4 &Kres, int row0, int slot) const {
    LoadKs::issue(Kres, row0, this->ldsK_wave + slot * SUB_BYTES, this->tid, this->k_lane_off, this->kv_row_bytes);
  }
  __device__ __forceinline__ void issue_v_sub(const u32x4 &Vres, int row0, int slot) const {
    LoadVs::issue(Vres, row0, this->ldsV_wave + slot * SUB_BYTES, this->tid, this->v_lane_off, this->kv_row_bytes);
  }

  // ---- the MFMA side of a stage -------------------------------------------------------------
  // Instruction I of a stage working on buffers of parity PAR: I < N_PV: O^T += V^T P^T of the
  // sub-tile whose V sits in V slot PAR and whose P sits in S buffer PAR (16-key slab I / DB outer,
  // d block I % DB inner); then S^T = K Q^T of the sub-tile whose K sits in K slot PAR, into S buffer
  // PAR (k-slab outer, key sub-block inner).
  static constexpr __device__ int lds_reads_of(int i) { return i < N_PV ? 2 : 1; }
  template <int PAR, int I>
  __device__ __forceinline__ void issue_operand_reads() const {
    constexpr int slot = A_ST + 4 * (I % IL_STAGES);
    if constexpr (I < N_PV) {
      constexpr int j = I / DB, db = I % DB;
      lds_to_acc_tr_b64<slot, PAR * SUB_BYTES + 16 * j * ROWB>(v_base[db]);
      lds_to_acc_tr_b64<slot + 2, PAR * SUB_BYTES + 16 * j * ROWB + 4 * ROWB>(v_base[db]);
    } else {
      constexpr int s = (I - N_PV) / KBS, kb = (I - N_PV) % KBS;
      lds_to_acc_b128<slot, PAR * SUB_BYTES + kb * 32 * ROWB>(k_base ^ (uint32_t)(s << 5));
    }
  }
  template <int PAR, int I>
  __device__ __forceinline__ void issue_mfma() const {
    constexpr int slot = A_ST + 4 * (I % IL_STAGES);
    if constexpr (I < N_PV) {
      constexpr int j = I / DB, db = I % DB;
      mfma_named<T, false, A_O + 16 * db, slot, true, V_S + PAR * EL + 16 * (j >> 1) + 4 * (j & 1), false>();
    } else {
      constexpr int s = (I - N_PV) / KBS, kb = (I - N_PV) % KBS;
      mfma_named<T, true, V_S + PAR * EL + 16 * kb, slot, false, A_Q + 4 * s, s == 0>();
    }
  }
  template <int I, int LAST>
  static constexpr __device__ int reads_behind() {
    int n = 0;
    for (int k = I + 1; k <= I + IL_AHEAD && k < LAST; ++k) n += lds_reads_of(k);
    return n;
  }

  // ---- the vector side of a stage: softmax of the sub-tile in S buffer PAR, as a list of N_OPS steps
  // Steps [0, EL/2): running maxima of the logits (four chains).  Step EL/2: the row's largest logit
  // of this sub-tile and the decision about the reference: m_run is the value subtracted in the
  // exponent; any value works as long as the exponentials stay in range, since numerator and
  // denominator carry the same factor.  It moves up to the running maximum only when that exceeds
  // it by more than IL_REF_SLACK (always on a row's first sub-tile, whose reference is -inf); then
  // alpha = 2^(old - new) < 1 and O and the row sum are rescaled at the end of the stage, else
  // alpha = 1 and they are left alone (O sits in AGPRs, where rescaling costs three instructions
  // per element).  Then, per group of 8 keys: 8 x (sc * s - m_run), 8 x exp2, 4 x round-and-pack
  // into the named registers over the logits plus add the packed pair to the row sum.
  static constexpr int N_GROUPS = EL / 8;
  static constexpr int OPS_MAX = EL / 2, OPS_GROUP = 8 + 8 + 4;
  static constexpr int N_OPS = OPS_MAX + 1 + N_GROUPS * OPS_GROUP;
  template <int PAR, int J>
  __device__ __forceinline__ void softmax_op() {
    constexpr int B = V_S + PAR * EL;
    if constexpr (J < OPS_MAX) {
      if constexpr (J < 4) part[J] = -INFINITY;
      named_max3<B + 2 * J, B + 2 * J + 1>(part[J & 3]);
    } else if constexpr (J == OPS_MAX) {
      // (plain asm maxima: the compiler would first canonicalise every operand that came out of an asm)
      asm volatile("v_max3_f32 %0, %0, %1, %2" : "+v"(part[0]) : "v"(part[1]), "v"(part[2]));
      asm volatile("v_max_f32 %0, %0, %1" : "+v"(part[0]) : "v"(part[3]));
      float other;
      halves_of(part[0], rm, other);
      asm volatile("v_max_f32 %0, %0, %1" : "+v"(rm) : "v"(other));
      rm *= sc;
      const float m_old = this->m_run;
      const float m_new = rm - m_old > IL_REF_SLACK ? rm : m_old;  // rm > m_old where it is taken
      alpha = __builtin_amdgcn_exp2f(m_old - m_new);  // 0 on the first sub-tile; 1 when nothing moves
      this->m_run = m_new;
      neg_ref = -m_new;
      psum[0] = 0.f;
      psum[1] = 0.f;
    } else {
      constexpr int g = (J - OPS_MAX - 1) / OPS_GROUP, o = (J - OPS_MAX - 1) % OPS_GROUP;
      if constexpr (o < 8) {
        x[o] = named_fma<B + 8 * g + o>(sc, neg_ref);
      } else if constexpr (o < 16) {
        x[o - 8] = ordered_exp2(x[o - 8]);
      } else {
        // pairs 4 (g % 2) + [0,4) of sub-block g / 2 land on logits consumed above (this group or the one before)
        constexpr int i = o - 16;
        named_pack_and_sum<T, B + 16 * (g / 2) + 4 * (g % 2) + i>(x[2 * i], x[2 * i + 1], psum[i & 1]);
      }
    }
  }

  // One stage.  HAS_PV / HAS_QK: which contractions run (on buffers of parity PAR); HAS_SM: the
  // softmax of the sub-tile in S buffer 1 - PAR runs beside them.  Ends with the row-sum update
  // and, when some row's reference moved, the rescale of O; the caller waits for its tile loads
  // and passes the workgroup barrier.
  // LOADS: the tile loads of the next stages are issued from inside the stream, one instruction
  // behind each (or every second) of the first MFMAs: V rows [v_row0, v_row0 + SUB) into V slot
  // 1 - PAR, then K rows [k_row0, k_row0 + SUB) into K slot 1 - PAR (both slots were released by the
  // stage before).
  template <int PAR, bool HAS_PV, bool HAS_QK, bool HAS_SM, bool LOADS = false>
  __device__ __forceinline__ void stage(const u32x4 &Vres = u32x4{0, 0, 0, 0}, int v_row0 = 0,
                                        const u32x4 &Kres = u32x4{0, 0, 0, 0}, int k_row0 = 0) {
    constexpr int FIRST = HAS_PV ? 0 : N_PV, LAST = HAS_QK ? N_PV + N_QK : N_PV, M = LAST - FIRST;
    constexpr int OPS = HAS_SM ? N_OPS : 0;
    static_assert(!LOADS || 2 * LOADS_PER_WAVE <= M, "more load instructions than MFMAs");
    __builtin_amdgcn_s_setprio(1);
    static_unroll<(IL_AHEAD < M ? IL_AHEAD : M)>([&](auto k) { issue_operand_reads<PAR, FIRST + k>(); });
    static_unroll<M>([&](auto k) {
      constexpr int I = FIRST + k;
      if constexpr (I + IL_AHEAD < LAST) issue_operand_reads<PAR, I + IL_AHEAD>();
      wait_lds<reads_behind<I, LAST>()>();
      issue_mfma<PAR, I>();
      // a load instruction behind every second MFMA where the stage is long enough for that, else behind
      // every MFMA (all at once at the start of the stage measures 3 % slower, every second one 0.5 % faster)
      constexpr int STEP = 4 * LOADS_PER_WAVE <= M ? 2 : 1;
      constexpr int li = k / STEP;
      if constexpr (!LOADS || k % STEP != 0) {
      } else if constexpr (li < LOADS_PER_WAVE)
        LoadVs::issue_one(li, Vres, v_row0, this->ldsV_wave + (1 - PAR) * SUB_BYTES, this->tid, this->v_lane_off,
                          this->kv_row_bytes);
      else if constexpr (li < 2 * LOADS_PER_WAVE)
        LoadKs::issue_one(li - LOADS_PER_WAVE, Kres, k_row0, this->ldsK_wave + (1 - PAR) * SUB_BYTES, this->tid,
                          this->k_lane_off, this->kv_row_bytes);
      // the softmax steps are spread evenly over the MFMAs: step J follows MFMA floor(J * M / OPS)
      constexpr int J0 = (k * OPS + M - 1) / M, J1 = ((k + 1) * OPS + M - 1) / M;
      static_unroll<J1 - J0>([&](auto q) { softmax_op<1 - PAR, J0 + q>(); });
    });
    __builtin_amdgcn_s_setprio(0);
    // MFMA results are read by vector instructions only behind this (S in the next stage, O below
    // and in the epilogue): the last MFMA's write has to land first
    asm volatile("s_nop 15\n\ts_nop 7");
    if constexpr (HAS_SM) {
      this->l_run = this->l_run * alpha + (psum[0] + psum[1]);
      if (__any(alpha != 1.0f)) {
        static_unroll<2 * DB>([&](auto h) {
          float o8[8];
          static_unroll<8>([&](auto i) { o8[i] = acc_read<A_O + 8 * h + i>(); });
          static_unroll<8>([&](auto i) { acc_write<A_O + 8 * h + i>(o8[i] * alpha); });
        });
      }
    }
  }

  // Keys of the sub-tile in S buffer PAR at offsets >= limit (within the sub-tile, for this lane:
  // limit already has 8 g subtracted) lie beyond the sequence: their logits become -inf.
  template <int PAR>
  __device__ __forceinline__ void mask_tail(int limit) {
    static_unroll<EL>([&](auto e) {
      constexpr int key = 32 * (e / 16) + 16 * ((e % 16) >> 3) + (e & 7);
      float s;
      asm volatile("v_mov_b32 %0, v[%1]" : "=v"(s) : "n"(V_S + PAR * EL + e));
      s = key < limit ? s : -INFINITY;
      named_write<V_S + PAR * EL + e>(__builtin_bit_cast(uint32_t, s));
    });
  }

  // Start a row: Q^T operand into the AGPRs (lane (query l32, half g) holds d = 16 s + 8 g + [0,8) of
  // k-slab s), negated when the scale is negative; zero accumulators; empty running state.
  __device__ __forceinline__ void begin_row(const uint16_t *qrow_ptr, float scale_log2e) {
    const uint32_t flip = scale_log2e < 0.f ? 0x80008000u : 0u;
    const uint16_t *qp = qrow_ptr + 8 * this->g;
    static_unroll<DS / 2>([&](auto pair) {  // two k-slabs at a time: few registers in flight
      const typename RB::Operand q0 = *reinterpret_cast<const typename RB::Operand *>(qp + 32 * pair);
      const typename RB::Operand q1 = *reinterpret_cast<const typename RB::Operand *>(qp + 32 * pair + 16);
      static_unroll<4>([&](auto i) { acc_write<A_Q + 8 * pair + i>(__builtin_bit_cast(float, q0[(int)i] ^ flip)); });
      static_unroll<4>([&](auto i) { acc_write<A_Q + 8 * pair + 4 + i>(__builtin_bit_cast(float, q1[(int)i] ^ flip)); });
    });
    static_unroll<16 * DB>([&](auto i) { acc_write<A_O + i>(0.f); });
    // a scale of exactly zero would turn the -inf of masked keys into NaN
    sc = fmaxf(fabsf(scale_log2e), 1e-30f);
    this->m_run = -INFINITY;
    this->l_run = 0.f;
    alpha = 1.f;
  }

  // Normalised rows as packed element pairs into the staging tile (row i at tile + i * OST).
  // Returns the natural logarithm of the row's sum of exp(scaled logit) (-inf for a row without keys).
  __device__ __forceinline__ float stage_rows(char *tile) const {
    const float l_tot = sum_with_other_half(this->l_run);
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    char *orow = tile + (this->wave * 32 + this->l32) * RB::OST;
    static_unroll<4 * DB>([&](auto q4) {
      constexpr int db = q4 / 4, a = q4 % 4, base = A_O + 16 * db + 4 * a;
      u32x2 w;
      w[0] = T::pack(acc_read<base + 0>() * inv, acc_read<base + 1>() * inv);
      w[1] = T::pack(acc_read<base + 2>() * inv, acc_read<base + 3>() * inv);
      *reinterpret_cast<u32x2 *>(orow + (32 * db + 8 * a + 4 * this->g) * 2) = w;
    });
    return l_tot > 0.f ? (this->m_run + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f : -INFINITY;
  }
};

// Marks the named registers as used by the kernel (they only ever appear inside asm text):
// v72 .. v135 and a0 .. a119.
__device__ __forceinline__ void il_claim_registers() {
  static_assert(IL_VGPRS == 72, "the clobber list below names the registers");
#define CALIBATT_R10(p, n) p #n "0", p #n "1", p #n "2", p #n "3", p #n "4", p #n "5", p #n "6", p #n "7", p #n "8", p #n "9"
  asm volatile("" : : : "a0", "a1", "a2", "a3", "a4", "a5", "a6", "a7", "a8", "a9", CALIBATT_R10("a", 1),
               CALIBATT_R10("a", 2), CALIBATT_R10("a", 3), CALIBATT_R10("a", 4), CALIBATT_R10("a", 5), CALIBATT_R10("a", 6),
               CALIBATT_R10("a", 7), CALIBATT_R10("a", 8), CALIBATT_R10("a", 9), CALIBATT_R10("a", 10), CALIBATT_R10("a", 11));
  asm volatile("" : : : "v72", "v73", "v74", "v75", "v76", "v77", "v78", "v79", CALIBATT_R10("v", 8), CALIBATT_R10("v", 9),
               CALIBATT_R10("v", 10), CALIBATT_R10("v", 11), CALIBATT_R10("v", 12), "v130", "v131", "v132", "v133", "v134",
               "v135");
#undef CALIBATT_R10
}

// Arguments and work distribution exactly as sparse_attn_fwd_kernel (attn_kernel_2wg.h).
template <int D, int BQ, int BK, bool IV = false, typename T = Bf16>
__global__ __launch_bounds__(BQ * 2, (BQ >= 128 ? 2 : 1)) __attribute__((amdgpu_num_vgpr(IL_VGPRS))) void sparse_attn_fwd_il_kernel(
    const uint16_t *__restrict__ gq, const uint16_t *__restrict__ gk, const uint16_t *__restrict__ gv,
    uint16_t *__restrict__ gout, const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx,
    const int32_t *__restrict__ work, const int32_t *__restrict__ fan_ptr, const int32_t *__restrict__ fan_dst,
    int32_t *counter, const FwdDims p, const int32_t *__restrict__ iv_ptr, const uint32_t *__restrict__ iv,
    const int32_t *__restrict__ head_map, float *__restrict__ lse) {
  using Row = IlRow<D, BQ, BK, T>;
  constexpr int NT = Row::NT, CH = Row::CH, ROWB = Row::ROWB, OST = Row::OST, LDS_BYTES = Row::LDS_BYTES, SUB = Row::SUB;
  il_claim_registers();

  // [K window: 2 sub-tiles][V window: 2 sub-tiles] (reused as the output staging tile), work-item mailbox,
  // [IV: column list]
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  int *const cols = reinterpret_cast<int *>(lds + LDS_BYTES + 64);
  Row rb(lds, (uint32_t)p.in.n * 2);
  const int tid = rb.tid;
  const int lane = rb.lane;
  const int N = p.N;
  const int n_items = p.n_work * p.B;
  volatile int *const mailbox = reinterpret_cast<volatile int *>(lds + LDS_BYTES);
  int cur_group = 0, groups_left = p.n_groups;
  if (counter && p.n_groups > 1)
    cur_group = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) % p.n_groups;  // HW_REG_XCC_ID[3:0]
  ResidencyClock residency;
  residency.start();
#ifdef IL_PROFILE
  // cycles of one wavefront in: full stages, waits for the tile loads, barriers, everything else
  unsigned long long prof[4] = {0, 0, 0, 0};
  unsigned long long prof_t = __builtin_amdgcn_s_memtime();
#define IL_PROF(i)                                                \
  {                                                               \
    const unsigned long long now_ = __builtin_amdgcn_s_memtime(); \
    prof[i] += now_ - prof_t;                                     \
    prof_t = now_;                                                \
  }
#else
#define IL_PROF(i)
#endif
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
    const int h_raw = head_map ? head_map[h] : h;
    const bool head_ok = (unsigned)h_raw < (unsigned)p.H;
    const int ht = head_ok ? h_raw : 0;
    const size_t head_off = (size_t)b * p.in.b + (size_t)ht * p.in.h;
    const uint32_t head_bytes = (uint32_t)(N - 1) * rb.kv_row_bytes + ROWB;
    const u32x4 Kres = head_rsrc(gk + head_off, head_bytes);
    const u32x4 Vres = head_rsrc(gv + head_off, head_bytes);

    const int cbeg = row_ptr[id];
    int n_tiles = row_ptr[id + 1] - cbeg;
    // IV: entries [chunk_lo, chunk_lo + IV_COLS) of the row's list are expanded from its runs of
    // consecutive key blocks into LDS; every thread takes runs tid, tid + NT, ...
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
    if constexpr (IV) {
      n_tiles = (int)(iv[iv_ptr[id + 1] - 1] >> 16);
      expand_runs();  // the previous item's readers are behind the barrier that ended it
    }
    auto col_at = [&](int entry) { return IV ? cols[entry - chunk_lo] : col_idx[cbeg + entry]; };
    // kept key blocks of the row, 64 at a time in one VGPR (lane j = entry j of the current 64)
    int col_cache = n_tiles > 0 ? col_at(min(lane, n_tiles - 1)) : 0;
    auto col_of = [&](int t) {  // t inside the cached 64
      return __builtin_amdgcn_readlane(col_cache, t & 63);
    };
    {
      int qrow = r * BQ + rb.row_in_block();
      qrow = qrow < N ? qrow : N - 1;
      rb.begin_row(gq + head_off + (size_t)qrow * p.in.n, p.scale_log2e);
    }

    if (n_tiles > 0) {
      // The row's kept blocks as a stream of sub-tiles u_0, u_1, ... (SPB per block, an odd total is
      // padded with one sub-tile beyond the sequence, all of whose keys are masked).  Stage k:
      // O += P V of u_(k-2), S = K Q^T of u_k, softmax of u_(k-1); at its start the loads of V of u_(k-1)
      // and K of u_(k+1) are issued into the slots the stage before has finished with, and they land by
      // its end.  Stages alternate between the two slots of the windows and the two S buffers.
      constexpr int SPB = Row::SPB;
      const int n_sub = n_tiles * SPB;
      const int n_stream = (n_sub + 1) & ~1;
      // First key row of the next sub-tile of the stream (N beyond its end: rows there read as zeros
      // and the keys are masked); called once per sub-tile, in order.
      int nx_entry = 0, nx_part = 0, nx_col = col_of(0);
      auto next_rows = [&]() {
        if (nx_entry >= n_tiles) return N;
        const int row0 = nx_col * BK + nx_part * SUB;
        if (++nx_part == SPB) {
          nx_part = 0;
          ++nx_entry;
          if ((nx_entry & 63) == 0 && nx_entry < n_tiles) {
            if constexpr (IV) {
              if (nx_entry % IV_COLS == 0) {  // every wave has taken its entries of the chunk that is replaced
                chunk_lo = nx_entry;
                expand_runs();
              }
            }
            col_cache = col_at(min(nx_entry + lane, n_tiles - 1));
          }
          if (nx_entry < n_tiles) nx_col = col_of(nx_entry);
        }
        return row0;
      };
      // keys of a sub-tile that starts at key row row0 and lie beyond the sequence get -inf
#define CALIBATT_IL_MASK(PAR, row0) \
  if ((row0) + SUB > N) rb.template mask_tail<PAR>(N - (row0) - 8 * rb.g);
      const int r0 = next_rows();
      rb.issue_k_sub(Kres, r0, 0);
      wait_vmem<0>();
      __syncthreads();
      // stage 0: K of u_1 streams in; S of u_0
      const int r1 = next_rows();
      rb.issue_k_sub(Kres, r1, 1);
      rb.template stage<0, false, true, false>();
      CALIBATT_IL_MASK(0, r0)
      wait_vmem<0>();
      __syncthreads();
      // stage 1: V of u_0, K of u_2; S of u_1, softmax of u_0
      rb.issue_v_sub(Vres, r0, 0);
      int row_a = r1;            // of u_(k-1) at the start of stage k (k even below)
      int row_b = next_rows();   // of u_k
      rb.issue_k_sub(Kres, row_b, 0);
      rb.template stage<1, false, true, true>();
      CALIBATT_IL_MASK(1, r1)
      wait_vmem<0>();
      __syncthreads();
      for (int k = 2; k < n_stream; k += 2) {
        // stage k: loads inside the stream: V of u_(k-1), K of u_(k+1)
        const int row_c = next_rows();
        IL_PROF(3);
        rb.template stage<0, true, true, true, true>(Vres, row_a, Kres, row_c);
        IL_PROF(0);
        CALIBATT_IL_MASK(0, row_b)
        wait_vmem<0>();
        IL_PROF(1);
        __syncthreads();
        IL_PROF(2);
        // stage k + 1: V of u_k, K of u_(k+2) (beyond the stream: zeros into a slot nobody reads)
        const int row_d = next_rows();
        IL_PROF(3);
        rb.template stage<1, true, true, true, true>(Vres, row_b, Kres, row_d);
        IL_PROF(0);
        CALIBATT_IL_MASK(1, row_c)
        wait_vmem<0>();
        IL_PROF(1);
        __syncthreads();
        IL_PROF(2);
        row_a = row_c;
        row_b = row_d;
      }
#undef CALIBATT_IL_MASK
      // stage n_stream: V of the last sub-tile; O += P V of u_(n_stream-2), softmax of u_(n_stream-1)
      rb.issue_v_sub(Vres, row_a, 1);
      rb.template stage<0, true, false, true>();
      wait_vmem<0>();
      __syncthreads();
      // stage n_stream + 1: O += P V of u_(n_stream-1)
      rb.template stage<1, true, false, false>();
    }

    // ---- normalise, stage in LDS, store to the block and its repeat targets ----
    __syncthreads();  // every wave is done with the tile windows
    const float row_lse = rb.stage_rows(lds);
    __syncthreads();
    const int fbeg = fan_ptr[item];
    const int fend = fan_ptr[item + 1];
    if (lse && head_ok && rb.g == 0) {
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
#pragma unroll 2
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
#ifdef IL_PROFILE
  if (counter && blockIdx.x == 2 && tid == 0)
    for (int i = 0; i < 4; ++i) counter[12 + i] = (int32_t)(prof[i] >> 6);
#endif
#undef IL_PROF
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
