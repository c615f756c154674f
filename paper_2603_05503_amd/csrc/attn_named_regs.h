// Inline-assembly building blocks for kernels that address part of the register
// file BY NAME: MFMAs, LDS / global reads and vector ALU instructions whose
// operands are physical registers given as template arguments.  Every helper is
// one volatile asm statement, so statements execute in the order written and
// the compiler neither moves nor merges them.  The compiler does not know what
// these registers hold: a kernel using them is compiled for a reduced number
// of arch VGPRs (amdgpu_num_vgpr), names only registers above that number
// (and AGPRs), and lists them in a clobber so that they count as used.
#pragma once
#include <utility>

#include "attn_common.h"

namespace calibatt_dev {

template <typename F, int... I>
__device__ __forceinline__ void unroll_impl(F &&f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), indices usable as template arguments
template <int N, typename F>
__device__ __forceinline__ void static_unroll(F &&f) {
  unroll_impl(f, std::make_integer_sequence<int, N>{});
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

}  // namespace calibatt_dev
