// Device-side building blocks shared by the attention kernels of this library:
// vector types, LDS swizzles, the direct-to-LDS tile loader, bf16 packing and
// the lane^32 exchange.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "calibatt.h"

namespace calibatt_dev {


typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
#define LDS_PTR(T) __attribute__((address_space(3))) T *

// Element strides of a [B][H][N][D] tensor whose D axis is contiguous.
struct Strides {
  long long b, h, n;
};

struct FwdDims {
  int B, H, N, nbq, nbk, n_work;
  float scale_log2e;
  int n_groups;                         // segments of the work list (1, or one per XCD)
  int group_ptr[CALIBATT_GROUPS + 1];   // segment g = work[group_ptr[g] .. group_ptr[g+1])
  Strides in, out;                      // q, k, v share `in`; only the two-workgroup kernel reads these
};

template <int N_OUTSTANDING>
__device__ __forceinline__ void wait_vmem() {
  // waits until at most N_OUTSTANDING vector-memory operations of this wave are in flight
  static_assert(N_OUTSTANDING == 0 || N_OUTSTANDING == 2 || N_OUTSTANDING == 4 || N_OUTSTANDING == 8 ||
                N_OUTSTANDING == 16, "add the immediate below");
  if constexpr (N_OUTSTANDING == 0) asm volatile("s_waitcnt vmcnt(0)");
  else if constexpr (N_OUTSTANDING == 2) asm volatile("s_waitcnt vmcnt(2)");
  else if constexpr (N_OUTSTANDING == 4) asm volatile("s_waitcnt vmcnt(4)");
  else if constexpr (N_OUTSTANDING == 8) asm volatile("s_waitcnt vmcnt(8)");
  else asm volatile("s_waitcnt vmcnt(16)");
}

// 16-byte-chunk XOR swizzles of the LDS tiles.  CH = chunks per row (D/8); one
// 256-byte LDS line (all 64 banks) holds 16/CH rows.
//  K: 16 lanes reading 16 consecutive rows at one chunk column hit 16 distinct chunks.
//  V: a transposing read touches 4 consecutive rows x 4 consecutive chunks; they
//     land on 16 distinct chunks.
template <int D>
__device__ __forceinline__ int k_swz(int row) {
  constexpr int CH = D / 8;
  return (row / (16 / CH)) % CH;
}
template <int D>
__device__ __forceinline__ int v_swz(int row) {
  constexpr int CH = D / 8;
  return 4 * ((row / (16 / CH)) % (CH / 4));
}

// Raw buffer descriptor (V#) over one head's [N][D] bf16 matrix: loads past the
// end return zero instead of faulting, which is how ragged tails are handled.
__device__ __forceinline__ u32x4 head_rsrc(const uint16_t *base, uint32_t bytes) {
  const uint64_t a = reinterpret_cast<uint64_t>(base);
  u32x4 r;
  r[0] = __builtin_amdgcn_readfirstlane((uint32_t)a);
  r[1] = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32) & 0xffffu);  // stride 0, no swizzle
  r[2] = bytes;
  r[3] = 0x00020000u;
  return r;
}

// One direct-to-LDS load: every lane fetches 16 bytes at rsrc.base + voff + soff
// and the wave's 1 KB lands at LDS byte address lds_off + 16 * lane.  Issued as
// inline asm so that the compiler keeps no record of LDS being written by an
// in-flight vector-memory operation (it would otherwise drain vmcnt before
// every LDS read); completion is tracked by hand with wait_vmem<>().
__device__ __forceinline__ void dma_16B_per_lane(const u32x4 rsrc, uint32_t voff, uint32_t soff, uint32_t lds_off) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"  // one wait state between the M0 write and the LDS-DMA that reads it
      "buffer_load_dwordx4 %1, %2, %3 offen lds"
      :
      : "s"(lds_off), "v"(voff), "s"(rsrc), "s"(soff)
      : "m0");
}

// Stream one ROWS x D bf16 tile global -> LDS.  Each instruction fills 1 KB of
// LDS; LDS chunk (row, c') receives global chunk (row, c' ^ swz(row)).
template <int D, int ROWS, int NT, bool FOR_V>
struct TileLoader {
  static constexpr int CH = D / 8;
  static constexpr int RPI = NT / CH;            // rows filled per instruction slab
  static constexpr int ITERS = ROWS / RPI;
  // lane offsets are the same for every instruction when the swizzle period (16 rows for K, 4 for V) divides RPI
  static constexpr bool INVARIANT = (RPI % (FOR_V ? 4 : 16)) == 0;
  static_assert(ROWS % RPI == 0, "tile must split evenly over the workgroup");

  // row_bytes: distance between consecutive rows of the matrix in memory (D * 2 when rows are packed)
  static __device__ __forceinline__ uint32_t lane_offset(int tid, int it, uint32_t row_bytes = D * 2) {
    const int row = it * RPI + tid / CH;
    const int cs = tid % CH;
    const int c = cs ^ (FOR_V ? v_swz<D>(row) : k_swz<D>(row));
    return (tid / CH) * row_bytes + c * 16;
  }

  // Instruction `it` of the ITERS that fill the tile.
  // lds_wave_off: LDS byte address of the tile + 1024 * wave index (wave-uniform)
  static __device__ __forceinline__ void issue_one(int it, const u32x4 rsrc, int row0, uint32_t lds_wave_off, int tid,
                                                   uint32_t lane_off0, uint32_t row_bytes = D * 2) {
    const uint32_t voff = INVARIANT ? lane_off0 : lane_offset(tid, it, row_bytes);
    const uint32_t soff = (uint32_t)(row0 + it * RPI) * row_bytes;
    dma_16B_per_lane(rsrc, voff, soff, lds_wave_off + it * NT * 16);
  }
  static __device__ __forceinline__ void issue(const u32x4 rsrc, int row0, uint32_t lds_wave_off, int tid,
                                               uint32_t lane_off0, uint32_t row_bytes = D * 2) {
#pragma unroll
    for (int it = 0; it < ITERS; ++it) issue_one(it, rsrc, row0, lds_wave_off, tid, lane_off0, row_bytes);
  }
};

// Diagnostic kept in the caller's workspace: how long workgroup 0 was resident, in shader-clock
// cycles (word 10) and in ticks of the constant 100 MHz counter (word 11).  Their ratio is the
// clock the GPU sustained during the launch.
struct ResidencyClock {
  uint64_t cycles0, ticks0;
  __device__ __forceinline__ void start() {
    cycles0 = __builtin_amdgcn_s_memtime();
    ticks0 = __builtin_amdgcn_s_memrealtime();
  }
  __device__ __forceinline__ void store(int32_t *workspace) const {
    workspace[10] = (int32_t)(__builtin_amdgcn_s_memtime() - cycles0);
    workspace[11] = (int32_t)(__builtin_amdgcn_s_memrealtime() - ticks0);
  }
};

typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;

// Element type of q, k, v, out (and of the probabilities fed to the second
// contraction).  Operands travel as raw 16-byte words; the traits supply the
// MFMA, the round-to-nearest-even packing of two fp32 values, and the sum of a
// packed pair accumulated into fp32 (a dot product with a vector of ones).
struct Bf16 {
  static __device__ __forceinline__ f32x16 mfma(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack(float lo, float hi) {
    bf16x2 t;
    t[0] = (__bf16)lo;
    t[1] = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, t);
  }
  static __device__ __forceinline__ float add_pair(uint32_t pk, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk), __builtin_bit_cast(bf16x2, 0x3f803f80u), acc, false);
  }
};
struct F16 {
  static __device__ __forceinline__ f32x16 mfma(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack(float lo, float hi) {
    f16x2 t;
    t[0] = (_Float16)lo;
    t[1] = (_Float16)hi;
    return __builtin_bit_cast(uint32_t, t);
  }
  static __device__ __forceinline__ float add_pair(uint32_t pk, float acc) {
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, pk), __builtin_bit_cast(f16x2, 0x3c003c00u), acc, false);
  }
};

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  bf16x2 t;
  t[0] = (__bf16)lo;
  t[1] = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, t);
}

// After the swap, a holds {x[0..31], x[0..31]} and b holds {x[32..63], x[32..63]}:
// every lane sees its own value and the one of lane ^ 32.  (Inline asm: the
// two-result builtin folds both results into one when fed the same operand
// twice.)  The leading s_nop covers the VALU-write -> permlane-read hazard.
__device__ __forceinline__ void halves_of(float x, float &a, float &b) {
  a = x;
  b = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ float max_with_other_half(float x) {
  float a, b;
  halves_of(x, a, b);
  return fmaxf(a, b);
}
__device__ __forceinline__ float sum_with_other_half(float x) {
  float a, b;
  halves_of(x, a, b);
  return a + b;
}

// Sum of x over the 32 lanes of this lane's half of the wave (half_wave_sum) or
// over all 64 lanes (wave_sum), delivered to every lane, as a fixed butterfly
// (the same order of additions in every run): xor 1, 2 (quad permutes), 4
// (half-row mirror), 8 (row mirror) inside rows of 16 lanes, then the 16-lane
// and, for the whole wave, the 32-lane swap across rows.
__device__ __forceinline__ float half_wave_sum(float x) {
  auto dpp = [](float v, auto ctrl) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), decltype(ctrl)::value,
                                                                 0xf, 0xf, false));
  };
  x += dpp(x, std::integral_constant<int, 0xB1>{});   // quad_perm [1,0,3,2]
  x += dpp(x, std::integral_constant<int, 0x4E>{});   // quad_perm [2,3,0,1]
  x += dpp(x, std::integral_constant<int, 0x141>{});  // row_half_mirror
  x += dpp(x, std::integral_constant<int, 0x140>{});  // row_mirror
  float a = x, b = x;
  asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(a), "+v"(b));
  return a + b;
}
__device__ __forceinline__ float wave_sum(float x) { return sum_with_other_half(half_wave_sum(x)); }

}  // namespace calibatt_dev
