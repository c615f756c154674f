// Device side of the mask calibration that follows the block-energy kernel
// (paper, Section 3.2): Eq. 6, the smallest set of key blocks of a block-row
// whose energies sum to at least eps, and the per-block vote counters behind
// Eq. 8-9.  Small kernels next to the energy kernel's 20 ms; they exist so
// that a calibration step never leaves the GPU (the same selection on the host
// costs five times the energy kernel in sorting alone).
//
// The selection is an integer decision taken on floating-point data, so it is
// defined exactly and matches the host routine bit for bit: order the row by
// (energy descending, column ascending) - a total order, so any correct sort
// gives the same permutation - then add the energies in that order, one by
// one, in fp64, and stop at the first prefix whose sum is >= eps.
#pragma once
#include <stdint.h>

namespace calibatt_dev {

constexpr int SELECT_THREADS = 256;
constexpr int SELECT_MAX_COLS = 4096;  // key blocks per row (keys of the sort held in LDS)

// 32-bit key that grows as the value falls (-0 counts as +0).
__device__ __forceinline__ uint32_t falling_key(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u << 1) == 0) u = 0;
  u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);  // now ascending with the value
  return ~u;
}
__device__ __forceinline__ float key_to_value(uint32_t key) {
  const uint32_t u = ~key;
  return __uint_as_float((u & 0x80000000u) ? (u & 0x7fffffffu) : ~u);
}

// One workgroup per row at a time.  P: power of two >= nbk, >= 2 (entries of the sort).
__global__ __launch_bounds__(SELECT_THREADS) void select_blocks_kernel(const float *__restrict__ energy,
                                                                       long long n_rows, int nbk, int P, double eps,
                                                                       uint8_t *__restrict__ mask) {
  extern __shared__ __attribute__((aligned(16))) unsigned long long sort_keys[];  // [P]
  __shared__ int cut_shared;
  const int tid = threadIdx.x;
  for (long long row = blockIdx.x; row < n_rows; row += gridDim.x) {
    const float *e = energy + row * nbk;
    for (int i = tid; i < P; i += SELECT_THREADS)
      sort_keys[i] = i < nbk ? ((unsigned long long)falling_key(e[i]) << 32) | (unsigned)i : ~0ull;
    __syncthreads();
    // bitonic network, ascending: the keys are distinct (the column is part of them)
    for (int k = 2; k <= P; k <<= 1)
      for (int j = k >> 1; j > 0; j >>= 1) {
        for (int i = tid; i < P; i += SELECT_THREADS) {
          const int partner = i ^ j;
          if (partner > i) {
            const unsigned long long a = sort_keys[i], b = sort_keys[partner];
            if ((a > b) == ((i & k) == 0)) {
              sort_keys[i] = b;
              sort_keys[partner] = a;
            }
          }
        }
        __syncthreads();
      }
    if (tid == 0) {
      double total = 0.0;
      int cut = nbk - 1;
      for (int i = 0; i < nbk; ++i) {
        total += (double)key_to_value((uint32_t)(sort_keys[i] >> 32));
        if (total >= eps) {
          cut = i;
          break;
        }
      }
      cut_shared = cut;
    }
    __syncthreads();
    const int cut = cut_shared;
    uint8_t *m = mask + row * nbk;
    for (int i = tid; i < nbk; i += SELECT_THREADS) m[(uint32_t)sort_keys[i]] = i <= cut ? 1 : 0;
    __syncthreads();
  }
}

// counts[i] += mask[i] != 0, stopping at 65535.
__global__ __launch_bounds__(256) void vote_accumulate_kernel(const uint8_t *__restrict__ mask, long long n,
                                                              uint16_t *__restrict__ counts) {
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x) {
    const uint16_t c = counts[i];
    if (mask[i] != 0 && c != 65535) counts[i] = (uint16_t)(c + 1);
  }
}

}  // namespace calibatt_dev
