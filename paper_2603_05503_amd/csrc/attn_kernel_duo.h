// Block-sparse attention forward, "duo" schedule: one workgroup per CU made of
// two independent halves that run in opposite phases.
//
// Same computation per query block as attn_kernel_2wg.h (paper, Section 2
// Eq. 1-4 under the block mask of Section 3.2, repeated query blocks written
// as copies, Section 3.3 / 3.4) with one difference in the online softmax: the
// reference subtracted inside the exponentials is moved lazily (see
// DuoRow::softmax), which changes roundings but not what is computed.
//
// Why: a SIMD overlaps one wavefront's MFMAs with ANOTHER wavefront's vector
// ALU work at no cost, but hardly with the same wavefront's.  Two co-resident
// workgroups (attn_kernel_2wg.h) overlap only as far as they happen to drift
// apart.  Here the 2 * BQ/32 wavefronts of a workgroup form two halves, A and
// B, each with its own query block, its own K/V tile buffers and its own work
// items; wavefront w of A and wavefront w of B share a SIMD.  Time is cut into
// phases by workgroup barriers.  In every phase one half is in its MATRIX slot
// (O += P V of its previous tile, then S = K Q^T of its next tile: 2*BK*D/256
// MFMAs back to back at raised priority, nothing else but their LDS operand
// reads) and the other half is in its VECTOR slot (issue the next K and V
// tile loads, softmax of the tile just multiplied, wait for the loads).  At
// the barrier they swap.  Row changes (normalise, store, next work item) take
// vector and matrix slots of one half while the other half keeps going.
//
// Registers.  With two wavefronts per SIMD a wavefront has 256 registers.  The
// kernel is compiled for 64 arch VGPRs (addresses and temporaries: the
// compiler's) and addresses the rest BY NAME from inline assembly:
//   v[64 .. 64 + 16 KB)      S^T of the tile, 16 per 32-key sub-block; the
//                            vector slot overwrites elements 0..7 of each
//                            sub-block with its probabilities as packed pairs
//                            (the B operand of the second contraction).  Arch
//                            VGPRs, because the vector ALU reads and writes
//                            them in place: a single wavefront issues a vector
//                            instruction only every 5-8 cycles, so the slot's
//                            length is its instruction count, and copies to
//                            and from AGPRs would double that count.
//   a[0 .. 16 DB)            O^T accumulators, 16 per 32-wide d block (an MFMA
//                            whose accumulator is an AGPR issues faster when a
//                            single wavefront feeds the matrix pipe)
//   a[A_ST .. A_ST + 24)     six 4-register slots for MFMA A operands read
//                            from LDS a few instructions ahead of their use
//   a[A_Q .. A_Q + 4 DS)     Q^T of the row block, the B operand of the first
//                            contraction, loaded from memory straight into AGPRs
// Every instruction that touches a named register is a volatile asm statement,
// so they execute in program order; the hazards the assembler does not police
// are kept by construction: an MFMA result is read by the vector ALU (or an
// operand register rewritten) only in a later slot, behind a barrier and an
// explicit s_nop; an LDS read is consumed only behind an s_waitcnt that counts
// the reads issued after it; a staging slot is refilled two MFMAs after the
// one that read it was issued; a transcendental's result is read no earlier
// than four instructions later and a dot product's by another kind of
// instruction only behind an s_nop.
#pragma once
#include <limits.h>

#include <utility>

#include "attn_kernel_2wg.h"

namespace calibatt_dev {

// The reference of the exponentials moves only when a logit exceeds it by more
// than this (log2 domain): probabilities stay below 2^8, far inside the bf16 /
// fp16 range, and keep their full relative precision.
constexpr float DUO_REF_SLACK = 8.0f;
constexpr int DUO_VGPRS = 64;   // arch VGPRs left to the compiler; the named ones follow
constexpr int DUO_AGPRS = 120;  // AGPRs addressed by name
constexpr int DUO_STAGES = 6;   // operand staging slots
#ifndef DUO_PRIO_MATRIX
#define DUO_PRIO_MATRIX 2
#endif
constexpr int DUO_AHEAD = 4;    // MFMAs between the issue of an operand's LDS reads and its use

template <typename F, int... I>
__device__ __forceinline__ void duo_unroll_impl(F &&f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), indices usable as template arguments
template <int N, typename F>
__device__ __forceinline__ void duo_unroll(F &&f) {
  duo_unroll_impl(f, std::make_integer_sequence<int, N>{});
}

template <int R>
__device__ __forceinline__ float acc_read() {
  float x;
  asm volatile("v_accvgpr_read_b32 %0, a[%1]" : "=v"(x) : "n"(R));
  return x;
}
template <int R>
__device__ __forceinline__ void acc_write(float x) {
  asm volatile("v_accvgpr_write_b32 a[%1], %0" : : "v"(x), "n"(R));
}
// LDS -> AGPR operand reads; addr is an LDS byte address, OFF a 16-bit immediate added to it
template <int DST, int OFF>
__device__ __forceinline__ void lds_to_acc_b128(uint32_t addr) {
  asm volatile("ds_read_b128 a[%1:%2], %0 offset:%3" : : "v"(addr), "n"(DST), "n"(DST + 3), "n"(OFF));
}
template <int DST, int OFF>
__device__ __forceinline__ void lds_to_acc_tr_b64(uint32_t addr) {
  asm volatile("ds_read_b64_tr_b16 a[%1:%2], %0 offset:%3" : : "v"(addr), "n"(DST), "n"(DST + 1), "n"(OFF));
}
template <int N>
__device__ __forceinline__ void wait_lds() {
  static_assert(N >= 0 && N <= 15, "lgkmcnt is a 4-bit counter");
  asm volatile("s_waitcnt lgkmcnt(%0)" : : "n"(N));
}
// MFMA on named registers.  CV: the accumulator is v[C..C+16) (else a[C..C+16)); BV: the B operand is
// v[B..B+4) (else a[B..B+4)); the A operand is a[A..A+4); ZERO: the accumulator starts from 0.
template <typename T, bool CV, int C, int A, bool BV, int B, bool ZERO>
__device__ __forceinline__ void mfma_named() {
#define CALIBATT_MFMA(op, c, bsrc, cin)                                                                              \
  asm volatile(op " " c "[%0:%1], a[%2:%3], " bsrc "[%4:%5], " cin : : "n"(C), "n"(C + 15), "n"(A), "n"(A + 3), "n"(B), \
               "n"(B + 3))
#define CALIBATT_MFMA_T(op)                                              \
  if constexpr (CV && BV) {                                              \
    if constexpr (ZERO) CALIBATT_MFMA(op, "v", "v", "0");                \
    else CALIBATT_MFMA(op, "v", "v", "v[%0:%1]");                        \
  } else if constexpr (CV) {                                             \
    if constexpr (ZERO) CALIBATT_MFMA(op, "v", "a", "0");                \
    else CALIBATT_MFMA(op, "v", "a", "v[%0:%1]");                        \
  } else if constexpr (BV) {                                             \
    if constexpr (ZERO) CALIBATT_MFMA(op, "a", "v", "0");                \
    else CALIBATT_MFMA(op, "a", "v", "a[%0:%1]");                        \
  } else {                                                               \
    if constexpr (ZERO) CALIBATT_MFMA(op, "a", "a", "0");                \
    else CALIBATT_MFMA(op, "a", "a", "a[%0:%1]");                        \
  }
  if constexpr (std::is_same<T, Bf16>::value) {
    CALIBATT_MFMA_T("v_mfma_f32_32x32x16_bf16")
  } else {
    CALIBATT_MFMA_T("v_mfma_f32_32x32x16_f16")
  }
#undef CALIBATT_MFMA_T
#undef CALIBATT_MFMA
}
// Vector ALU on named arch VGPRs (volatile: executed in the order written).
template <int R0, int R1>
__device__ __forceinline__ void named_max3(float &m) {
  asm volatile("v_max3_f32 %0, %0, v[%1], v[%2]" : "+v"(m) : "n"(R0), "n"(R1));
}
template <int R0, int R1>
__device__ __forceinline__ void named_min3(float &m) {
  asm volatile("v_min3_f32 %0, %0, v[%1], v[%2]" : "+v"(m) : "n"(R0), "n"(R1));
}
template <int R>
__device__ __forceinline__ float named_mul(float c) {
  float x;
  asm volatile("v_mul_f32 %0, %1, v[%2]" : "=v"(x) : "v"(c), "n"(R));
  return x;
}
template <int R>
__device__ __forceinline__ float named_fma(float c, float d) {  // v[R] * c + d
  float x;
  asm volatile("v_fma_f32 %0, v[%1], %2, %3" : "=v"(x) : "n"(R), "v"(c), "v"(d));
  return x;
}
__device__ __forceinline__ float ordered_exp2(float x) {
  float y;
  asm volatile("v_exp_f32 %0, %1" : "=v"(y) : "v"(x));
  return y;
}
template <int R>
__device__ __forceinline__ void named_write(uint32_t x) {
  asm volatile("v_mov_b32 v[%1], %0" : : "v"(x), "n"(R));
}
// v[R] = (lo, hi) rounded to nearest-even and packed; the packed pair's two values are added to acc
template <typename T, int R>
__device__ __forceinline__ void named_pack_and_sum(float lo, float hi, float &acc) {
  if constexpr (std::is_same<T, Bf16>::value) {
    asm volatile("v_cvt_pk_bf16_f32 v[%2], %0, %1" : : "v"(lo), "v"(hi), "n"(R));
    asm volatile("v_dot2c_f32_bf16 %0, 0x3f803f80, v[%1]" : "+v"(acc) : "n"(R));
  } else {
    asm volatile("v_cvt_pk_f16_f32 v[%2], %0, %1" : : "v"(lo), "v"(hi), "n"(R));
    asm volatile("v_dot2c_f32_f16 %0, 0x3c003c00, v[%1]" : "+v"(acc) : "n"(R));
  }
}
// 16 bytes of global memory at ptr + OFF straight into AGPRs DST..DST+3
template <int DST, int OFF>
__device__ __forceinline__ void global_to_acc_b128(const void *ptr) {
  asm volatile("global_load_dwordx4 a[%1:%2], %0, off offset:%3" : : "v"(ptr), "n"(DST), "n"(DST + 3), "n"(OFF));
}

template <int D, int BQ, int BK, typename T = Bf16>
struct DuoRow : RowBlock<D, BQ, BK, T> {
  using RB = RowBlock<D, BQ, BK, T>;
  using RB::DB;
  using RB::DS;
  using RB::KB;
  using RB::ROWB;
  static constexpr int V_SP = DUO_VGPRS;  // first named arch VGPR
  static constexpr int A_O = 0, A_ST = 16 * DB, A_Q = A_ST + 4 * DUO_STAGES;
  static_assert(A_Q + 4 * DS <= DUO_AGPRS && V_SP + 16 * KB + DUO_AGPRS <= 256, "register map does not fit");
  static constexpr int N_PV = 2 * KB * DB, N_QK = DS * KB;  // MFMAs of the two contractions
  uint32_t k_base, v_base[DB];  // LDS byte addresses of this lane's operand pieces in the K and V tile

  __device__ __forceinline__ DuoRow(char *lds_, uint32_t kv_row_bytes_, int tid_) : RB(lds_, kv_row_bytes_, tid_) {
    const uint32_t lds_base = (uint32_t)(uintptr_t)(LDS_PTR(char))lds_;  // a multiple of 1024
    k_base = lds_base + this->k_addr0;
#pragma unroll
    for (int db = 0; db < DB; ++db) v_base[db] = lds_base + RB::TILE_BYTES + this->v_addr[db];
  }

  // Instruction i of a matrix slot: first the N_PV MFMAs of O^T += V^T P^T (16-key slab j = i / DB
  // outer, d block i % DB inner), then the N_QK MFMAs of S^T = K Q^T (k-slab outer, key sub-block
  // inner).
  static constexpr __device__ int lds_reads_of(int i) { return i < N_PV ? 2 : 1; }
  template <int I>
  __device__ __forceinline__ void issue_operand_reads() const {
    constexpr int slot = A_ST + 4 * (I % DUO_STAGES);
    if constexpr (I < N_PV) {
      constexpr int j = I / DB, db = I % DB;
      lds_to_acc_tr_b64<slot, 16 * j * ROWB>(v_base[db]);
      lds_to_acc_tr_b64<slot + 2, 16 * j * ROWB + 4 * ROWB>(v_base[db]);
    } else {
      constexpr int s = (I - N_PV) / KB, kb = (I - N_PV) % KB;
      // (volatile: computed here, per use, instead of being kept in eight more registers)
      uint32_t addr;
      asm volatile("v_xor_b32 %0, %1, %2" : "=v"(addr) : "n"(s << 5), "v"(k_base));
      lds_to_acc_b128<slot, kb * 32 * ROWB>(addr);
    }
  }
  template <int I>
  __device__ __forceinline__ void issue_mfma() const {
    constexpr int slot = A_ST + 4 * (I % DUO_STAGES);
    if constexpr (I < N_PV) {
      constexpr int j = I / DB, db = I % DB;
      mfma_named<T, false, A_O + 16 * db, slot, true, V_SP + 16 * (j >> 1) + 4 * (j & 1), false>();
    } else {
      constexpr int s = (I - N_PV) / KB, kb = (I - N_PV) % KB;
      mfma_named<T, true, V_SP + 16 * kb, slot, false, A_Q + 4 * s, s == 0>();
    }
  }
  // LDS reads in flight behind those of instruction I when its MFMA is about to issue
  template <int I, int LAST>
  static constexpr __device__ int reads_behind() {
    int n = 0;
    for (int k = I + 1; k <= I + DUO_AHEAD && k < LAST; ++k) n += lds_reads_of(k);
    return n;
  }
  // The matrix slot: instructions [FIRST, LAST) as one software pipeline.
  template <int FIRST, int LAST>
  __device__ __forceinline__ void matrix_slot() const {
    duo_unroll<(DUO_AHEAD < LAST - FIRST ? DUO_AHEAD : LAST - FIRST)>([&](auto k) { issue_operand_reads<FIRST + k>(); });
    duo_unroll<LAST - FIRST>([&](auto k) {
      constexpr int I = FIRST + k;
      if constexpr (I + DUO_AHEAD < LAST) issue_operand_reads<I + DUO_AHEAD>();
      wait_lds<reads_behind<I, LAST>()>();
      issue_mfma<I>();
    });
    // results are read by vector instructions in the next slot: cover the MFMA write latency
    asm volatile("s_nop 15\n\ts_nop 7");
  }

  // Start a row: Q^T operand (lane (query l32, half g) holds d = 16 s + 8 g + [0,8) of k-slab s; the
  // caller waits for the loads), zero accumulators, empty running state.
  __device__ __forceinline__ void begin_row(const uint16_t *qrow_ptr) {
    const uint16_t *qp = qrow_ptr + 8 * this->g;
    duo_unroll<DS>([&](auto s) { global_to_acc_b128<A_Q + 4 * s, 32 * s>(qp); });
    duo_unroll<16 * DB>([&](auto i) { acc_write<A_O + i>(0.f); });
    this->m_run = -INFINITY;
    this->l_run = 0.f;
  }

  // Online softmax of the tile whose S^T sits in the AGPRs (log2 domain, sc = scale * log2(e)).
  // m_run is the reference subtracted in the exponent: any value works as long as the
  // exponentials stay in range, since numerator and denominator carry the same factor 2^-m_run.
  // A first pass finds the tile's largest logit per row.  Only when some row of the wavefront has
  // one more than DUO_REF_SLACK above its reference (always on a row's first tile, whose
  // reference is -inf) the references move up to the running maxima and the row sums and O are
  // rescaled - O sits in AGPRs, where a rescale costs three instructions per element, so it is
  // kept rare.  The second pass forms p = 2^(sc * s - m_run), rounds to the element type, adds the
  // rounded values to the row sum and writes the packed pairs over the logits.
  // TAIL: this lane's key offsets >= limit lie beyond the sequence.
  template <bool TAIL>
  __device__ __forceinline__ void softmax(float sc, int limit) {
    constexpr int NG = 2 * KB;  // groups of 8 consecutive keys of a lane (element e = 8 G + i of S^T)
    // ---- pass 1: the tile's largest logit of this lane's row (four independent chains)
    float part[4];
    const bool flip = !TAIL && sc < 0.f;  // a negative scale turns the smallest product into the largest logit
#pragma unroll
    for (int i = 0; i < 4; ++i) part[i] = flip ? INFINITY : -INFINITY;
    if constexpr (TAIL) {
      duo_unroll<8 * KB>([&](auto pr) {
        constexpr int e = 2 * pr, key = 32 * (e / 16) + 16 * ((e % 16) >> 3) + (e & 7);
        const float y0 = named_mul<V_SP + e>(sc), y1 = named_mul<V_SP + e + 1>(sc);
        part[pr & 3] = fmaxf(part[pr & 3], fmaxf(key < limit ? y0 : -INFINITY, key + 1 < limit ? y1 : -INFINITY));
      });
    } else if (flip) {
      duo_unroll<8 * KB>([&](auto pr) { named_min3<V_SP + 2 * pr, V_SP + 2 * pr + 1>(part[pr & 3]); });
    } else {
      duo_unroll<8 * KB>([&](auto pr) { named_max3<V_SP + 2 * pr, V_SP + 2 * pr + 1>(part[pr & 3]); });
    }
    float rm = flip ? fminf(fminf(part[0], part[1]), fminf(part[2], part[3]))
                    : fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
    if constexpr (!TAIL) rm *= sc;
    rm = max_with_other_half(rm);
    if (__any(!(rm - this->m_run <= DUO_REF_SLACK))) {
      const float m_new = fmaxf(this->m_run, rm);
      const float alpha = __builtin_amdgcn_exp2f(this->m_run - m_new);  // 0 on the first tile
      this->m_run = m_new;
      this->l_run *= alpha;
      duo_unroll<2 * DB>([&](auto h) {
        float o8[8];
        duo_unroll<8>([&](auto i) { o8[i] = acc_read<A_O + 8 * h + i>(); });
        duo_unroll<8>([&](auto i) { acc_write<A_O + 8 * h + i>(o8[i] * alpha); });
      });
    }
    // ---- pass 2: probabilities, written over the logits.  Per group of 8 keys: 8 x (sc * s - ref),
    // 8 x exp2, 4 x round-and-pack into the named registers, 4 x add the packed pair to the row sum.
    if constexpr (TAIL) asm volatile("" : "+v"(limit));
    const float neg_ref = -this->m_run;
    float psum[2] = {0.f, 0.f};
    duo_unroll<NG>([&](auto G) {
      float x[8];
      duo_unroll<8>([&](auto i) {
        x[i] = named_fma<V_SP + 8 * G + i>(sc, neg_ref);
        if constexpr (TAIL) {
          constexpr int key = 32 * (G / 2) + 16 * (G % 2) + i;
          x[i] = key < limit ? x[i] : -INFINITY;
        }
      });
      duo_unroll<8>([&](auto i) { x[i] = ordered_exp2(x[i]); });
      // pairs 4 (G % 2) + [0,4) of sub-block G / 2 land on logits consumed above (this group or G - 1)
      duo_unroll<4>([&](auto i) {
        named_pack_and_sum<T, V_SP + 16 * (G / 2) + 4 * (G % 2) + i>(x[2 * i], x[2 * i + 1], psum[i & 1]);
      });
    });
    asm volatile("s_nop 4");  // dot-product results are read by an add next
    this->l_run += psum[0] + psum[1];
  }

  // Normalised rows as packed element pairs into this half's staging tile (row i at tile + i * OST).
  // Returns the natural logarithm of the row's sum of exp(scaled logit) (-inf for a row without keys).
  __device__ __forceinline__ float stage_rows(char *tile) const {
    const float l_tot = sum_with_other_half(this->l_run);
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    char *orow = tile + (this->wave * 32 + this->l32) * RB::OST;
    duo_unroll<4 * DB>([&](auto q4) {
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
// v64 .. v127 and a0 .. a119.
__device__ __forceinline__ void duo_claim_registers() {
#define CALIBATT_R10(p, n) p #n "0", p #n "1", p #n "2", p #n "3", p #n "4", p #n "5", p #n "6", p #n "7", p #n "8", p #n "9"
  asm volatile("" : : : "a0", "a1", "a2", "a3", "a4", "a5", "a6", "a7", "a8", "a9", CALIBATT_R10("a", 1),
               CALIBATT_R10("a", 2), CALIBATT_R10("a", 3), CALIBATT_R10("a", 4), CALIBATT_R10("a", 5), CALIBATT_R10("a", 6),
               CALIBATT_R10("a", 7), CALIBATT_R10("a", 8), CALIBATT_R10("a", 9), CALIBATT_R10("a", 10), CALIBATT_R10("a", 11));
  asm volatile("" : : : "v64", "v65", "v66", "v67", "v68", "v69", CALIBATT_R10("v", 7), CALIBATT_R10("v", 8),
               CALIBATT_R10("v", 9), CALIBATT_R10("v", 10), CALIBATT_R10("v", 11), "v120", "v121", "v122", "v123", "v124",
               "v125", "v126", "v127");
#undef CALIBATT_R10
}

// Stages of one half's walk through its work items.  A half alternates vector and matrix slots:
// PROLOGUE and FINISH run in vector slots, STORE in a matrix slot, TILES in both.
enum DuoStage { DUO_PROLOGUE, DUO_TILES, DUO_FINISH, DUO_STORE, DUO_DONE };

template <int D, int BQ, int BK, bool IV = false, typename T = Bf16>
__global__ __launch_bounds__(BQ * 4, 1) __attribute__((amdgpu_num_vgpr(DUO_VGPRS))) void sparse_attn_fwd_duo_kernel(
    const uint16_t *__restrict__ gq, const uint16_t *__restrict__ gk, const uint16_t *__restrict__ gv,
    uint16_t *__restrict__ gout, const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx,
    const int32_t *__restrict__ work, const int32_t *__restrict__ fan_ptr, const int32_t *__restrict__ fan_dst,
    int32_t *counter, const FwdDims p, const int32_t *__restrict__ iv_ptr, const uint32_t *__restrict__ iv,
    const int32_t *__restrict__ head_map, float *__restrict__ lse) {
  using Row = DuoRow<D, BQ, BK, T>;
  constexpr int NT = Row::NT, CH = Row::CH, ROWB = Row::ROWB, OST = Row::OST, HALF_LDS = Row::LDS_BYTES;
  constexpr int N_PV = Row::N_PV, N_ALL = Row::N_PV + Row::N_QK;
  duo_claim_registers();

  // [half A: K tile, V tile][half B: K tile, V tile][shared words][IV: column lists of A and B]
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int half = __builtin_amdgcn_readfirstlane((int)threadIdx.x / NT);
  const int tid = (int)threadIdx.x - half * NT;
  char *const hlds = lds + half * HALF_LDS;
  // words 0,1: next work item of half A, B; words 2,3: loop iteration in which half A, B stores its last rows
  volatile int *const shared = reinterpret_cast<volatile int *>(lds + 2 * HALF_LDS);
  int *const cols = reinterpret_cast<int *>(lds + 2 * HALF_LDS + 64) + half * IV_COLS;
  Row rb(hlds, (uint32_t)p.in.n * 2, tid);
  const int lane = rb.lane;
  const int N = p.N;

  // Work items come from the per-group counters exactly as in the two-workgroup kernel; each half
  // pops for itself.
  int cur_group = 0, groups_left = p.n_groups;
  if (p.n_groups > 1) cur_group = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) % p.n_groups;  // HW_REG_XCC_ID
  auto pop = [&]() {
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
    return found;
  };
  ResidencyClock residency;
  residency.start();

  // state of this half's current work item (wave-uniform)
  int stage = DUO_DONE;
  int r = 0, b = 0, ht = 0, cbeg = 0, n_tiles = 0, fbeg = 0, fend = 0, k_slot = 0, c_cur = 0, c_next = 0;
  bool head_ok = false;
  size_t head_off = 0;
  u32x4 Kres = {0, 0, 0, 0}, Vres = {0, 0, 0, 0};
  int col_cache = 0;
  const float sc = p.scale_log2e;

  // Reads the mailbox and the lists' entries of the item.
  auto fetch_item = [&]() {
    const int wg_item = __builtin_amdgcn_readfirstlane(shared[half]);
    if (wg_item < 0) {
      stage = DUO_DONE;
      return;
    }
    const int item = wg_item / p.B;
    b = wg_item - item * p.B;
    const int id = work[item];
    const int h = id / p.nbq;
    r = id - h * p.nbq;
    const int h_raw = head_map ? head_map[h] : h;
    head_ok = (unsigned)h_raw < (unsigned)p.H;
    ht = head_ok ? h_raw : 0;
    head_off = (size_t)b * p.in.b + (size_t)ht * p.in.h;
    const uint32_t head_bytes = (uint32_t)(N - 1) * rb.kv_row_bytes + ROWB;
    Kres = head_rsrc(gk + head_off, head_bytes);
    Vres = head_rsrc(gv + head_off, head_bytes);
    cbeg = row_ptr[id];
    n_tiles = row_ptr[id + 1] - cbeg;
    fbeg = fan_ptr[item];
    fend = fan_ptr[item + 1];
    if constexpr (IV) {
      // the row's runs expanded into this half's column list (rows of at most IV_COLS kept blocks)
      const int ib = iv_ptr[id], ie = iv_ptr[id + 1] - 1;
      n_tiles = (int)(iv[ie] >> 16);
      for (int i = ib + tid; i < ie; i += NT) {
        const uint32_t w = iv[i], w_next = iv[i + 1];
        const int start = (int)(w & 0xffffu), before = (int)(w >> 16), len = (int)(w_next >> 16) - before;
        for (int j = 0; j < len; ++j) cols[before + j] = start + j;
      }
    }
    stage = DUO_PROLOGUE;
  };
  auto col_at = [&](int entry) { return IV ? cols[entry] : col_idx[cbeg + entry]; };

  if (tid == 0) {
    const int first = pop();
    shared[half] = first;
    shared[2 + half] = first < 0 ? -1 : INT_MAX;
  }
  __syncthreads();
  fetch_item();
  __syncthreads();

  // Half B runs one phase behind half A: while one half is in its vector slot the other is in
  // its matrix slot.  (s_barrier counts arrivals; it does not matter where in the code a
  // wavefront arrives from.)
  if (half == 1) __syncthreads();
#ifdef DUO_PROFILE
  unsigned long long prof[4] = {0, 0, 0, 0};
  unsigned long long prof_t = __builtin_amdgcn_s_memtime();
  auto prof_mark = [&](int which) {
    const unsigned long long now = __builtin_amdgcn_s_memtime();
    prof[which] += now - prof_t;
    prof_t = now;
  };
#else
  auto prof_mark = [](int) {};
#endif
  for (int it = 0;; ++it) {
    // ------------------------------ vector slot ------------------------------
    if (stage == DUO_PROLOGUE) {
      col_cache = n_tiles > 0 ? col_at(min(lane, n_tiles - 1)) : 0;
      c_next = __builtin_amdgcn_readlane(col_cache, 0);
      if (n_tiles > 0) rb.issue_k(Kres, c_next);
      int qrow = r * BQ + rb.row_in_block();
      qrow = qrow < N ? qrow : N - 1;
      rb.begin_row(gq + head_off + (size_t)qrow * p.in.n);
      wait_vmem<0>();
      k_slot = 0;
      stage = DUO_TILES;
    } else if (stage == DUO_TILES) {
      // tile t was multiplied by Q in the matrix slot before this one
      const int t = k_slot - 1;
      c_cur = c_next;
      const bool has_next = t + 1 < n_tiles;
      if (has_next) {
        if (((t + 1) & 63) == 0) col_cache = col_at(min(t + 1 + lane, n_tiles - 1));
        c_next = __builtin_amdgcn_readlane(col_cache, (t + 1) & 63);
      }
      rb.issue_v(Vres, c_cur);
      if (has_next) rb.issue_k(Kres, c_next);
      if (c_cur == p.nbk - 1 && (N % BK) != 0) {
        int limit = N - c_cur * BK - 8 * rb.g;
        asm volatile("" : "+v"(limit));
        rb.template softmax<true>(sc, limit);
      } else {
        rb.template softmax<false>(sc, 0);
      }
      prof_mark(0);
      wait_vmem<0>();
      prof_mark(1);
    } else if (stage == DUO_FINISH) {
      // normalise and stage the rows in this half's (now free) tile buffers; pop the next item
      if (tid == 0) {
        const int next = pop();
        shared[half] = next;
        if (next < 0) shared[2 + half] = it;  // this iteration's matrix slot stores the half's last rows
      }
      const float row_lse = rb.stage_rows(hlds);
      if (lse && head_ok && rb.g == 0) {
        float *const lse_head = lse + ((size_t)b * p.H + ht) * (size_t)N;
        for (int f = fbeg - 1; f < fend; ++f) {
          const int row = (f < fbeg ? r : fan_dst[f]) * BQ + rb.row_in_block();
          if (row < N) lse_head[row] = row_lse;
        }
      }
      stage = DUO_STORE;
    }
    prof_mark(0);
    __syncthreads();
    prof_mark(3);
    // ------------------------------ matrix slot ------------------------------
    if (stage == DUO_TILES) {
      __builtin_amdgcn_s_setprio(DUO_PRIO_MATRIX);
      if (k_slot == 0) {
        if (n_tiles > 0) rb.template matrix_slot<N_PV, N_ALL>();
      } else if (k_slot < n_tiles) {
        rb.template matrix_slot<0, N_ALL>();
      } else {
        rb.template matrix_slot<0, N_PV>();
      }
      __builtin_amdgcn_s_setprio(0);
      ++k_slot;
      if (k_slot > n_tiles) stage = DUO_FINISH;
    } else if (stage == DUO_STORE) {
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
            const u32x4 val = *reinterpret_cast<const u32x4 *>(hlds + row * OST + cc * 16);
            *reinterpret_cast<u32x4 *>(dst + (size_t)row * p.out.n + cc * 8) = val;
          }
        }
      }
      fetch_item();
    }
    prof_mark(2);
    __syncthreads();
    prof_mark(3);
    // Both halves take the same decision: a half's entry only ever changes from INT_MAX to the
    // iteration in which it was written, and it is written before the barrier that ends that
    // iteration's vector slot.
    if (shared[2] <= it && shared[3] <= it) break;
  }
  if (half == 0) __syncthreads();

  if (blockIdx.x == 0 && threadIdx.x == 0) residency.store(counter);
#ifdef DUO_PROFILE
  // cycles of workgroup 1's half A, wavefront 0 (x 1/64): vector slots up to the wait for the tile loads, that wait,
  // matrix slots, barrier waits
  if (blockIdx.x == 1 && threadIdx.x == 0)
    for (int i = 0; i < 4; ++i) counter[12 + i] = (int32_t)(prof[i] >> 6);
#endif
  // Last workgroup out re-arms the counters for the next launch.
  if (threadIdx.x == 0) {
    __threadfence();
    if (atomicAdd(counter + CALIBATT_GROUPS, 1) == (int)gridDim.x - 1) {
      for (int i = 0; i <= CALIBATT_GROUPS; ++i) counter[i] = 0;
      __threadfence();
    }
  }
}

}  // namespace calibatt_dev
