// Block energy of an attention map without materialising it (paper, Section
// 3.2, Eq. 5): E[r][c] = mean over the queries of block r of the softmax mass
// they put on the keys of block c.  gfx950 (MI355X), bf16 in, fp32 out.
//
// One workgroup per (batch, head, query block), two passes over all key tiles
// with the QK^T engine of the attention kernels (RowBlock::scores; a lane owns
// one query and half of the tile's keys):
//   pass 1  running row max and row sum (online softmax statistics);
//   pass 2  p = exp2(s - max) / sum per entry, summed over the lane's keys,
//           then over the wave's 32 queries with a fixed butterfly, one fp32
//           partial per (wave, key block) in LDS; at the end the partials of
//           the workgroup's waves are added in wave order and divided by the
//           number of rows the block has.
// No V, so both LDS tile buffers hold K: tile c+1 streams in while tile c is
// multiplied, one barrier per tile.  Work units are placed like those of the
// anchor kernel (contiguous ranges per XCD) since all query blocks of a head
// walk the same K tiles in step.  Every addition order is fixed: the result is
// the same bits on every run.
#pragma once
#include "attn_kernel_2wg.h"

namespace calibatt_dev {

struct EnergyDims {
  int B, H, N, nbq, nbk;
  float scale_log2e;
};

constexpr int ENERGY_XCDS = 8;

template <int D, int BQ, int BK>
struct EnergyLds {
  using RB = RowBlock<D, BQ, BK>;
  static constexpr int PART_OFF = 2 * RB::TILE_BYTES;  // float[NW][nbk] partial sums behind the two K buffers
  static __host__ __device__ constexpr long long bytes(int nbk) { return PART_OFF + (long long)RB::NW * nbk * 4; }
};

template <int D, int BQ, int BK>
__global__ __launch_bounds__(BQ * 2, (BQ >= 128 ? 2 : 1)) void block_energy_kernel(
    const uint16_t *__restrict__ gq, const uint16_t *__restrict__ gk, float *__restrict__ gE, const EnergyDims p) {
  using RB = RowBlock<D, BQ, BK>;
  constexpr int NT = RB::NT, NW = RB::NW, KB = RB::KB, ROWB = RB::ROWB, TILE_BYTES = RB::TILE_BYTES;

  extern __shared__ __attribute__((aligned(1024))) char lds[];  // EnergyLds::bytes(nbk)

  const int xcd = blockIdx.x % ENERGY_XCDS;
  const int slot = blockIdx.x / ENERGY_XCDS;
  const long long units = (long long)p.B * p.H * p.nbq;
  const long long lo = units * xcd / ENERGY_XCDS;
  const long long hi = units * (xcd + 1) / ENERGY_XCDS;
  if (slot >= hi - lo) return;
  const int unit = (int)(lo + slot);
  const int r = unit % p.nbq;
  const int bh = unit / p.nbq;  // b * H + h

  RB rb(lds);
  const int tid = rb.tid;
  const int N = p.N;
  const size_t head_off = (size_t)bh * (size_t)N * D;
  const u32x4 Kres = head_rsrc(gk + head_off, (uint32_t)N * ROWB);
  float *const part = reinterpret_cast<float *>(lds + EnergyLds<D, BQ, BK>::PART_OFF);
  const int rows_valid = min(BQ, N - r * BQ);

  rb.issue_k_at(Kres, 0, 0);
  const bool row_valid = rb.row_in_block() < rows_valid;
  rb.begin(gq + head_off + (size_t)(r * BQ + (row_valid ? rb.row_in_block() : 0)) * D);
  const float sc = p.scale_log2e;
  const bool ragged = (N % BK) != 0;

  float m_run = -INFINITY, l_run = 0.f, weight = 0.f;
  // Tiles of both passes form one sequence t = pass * nbk + c; tile t sits in buffer t & 1.
  const int n_steps = 2 * p.nbk;
  for (int t = 0; t < n_steps; ++t) {
    const bool second = t >= p.nbk;
    const int c = second ? t - p.nbk : t;
    wait_vmem<0>();
    __syncthreads();  // tile t has landed for every wave; everyone is done with the other buffer
    if (t + 1 < n_steps) rb.issue_k_at(Kres, c + 1 < p.nbk ? c + 1 : 0, ((t + 1) & 1) * TILE_BYTES);
    f32x16 s[KB];
    rb.scores((t & 1) * TILE_BYTES, s);
    // Work on the raw products with the scale folded into the exponent's FMA; only the ragged last
    // tile is scaled up front so that its keys >= N can sit at -inf (multiplier 1 from then on).
    float sc_t = sc;
    if (ragged && c == p.nbk - 1) {
      int limit = N - c * BK - 8 * rb.g;  // this lane's key offsets below `limit` exist
      asm volatile("" : "+v"(limit));      // keeps the comparisons (and their 64 masks) inside this branch
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          s[kb][v] = 32 * kb + 16 * (v >> 3) + (v & 7) < limit ? s[kb][v] * sc : -INFINITY;
      sc_t = 1.0f;
    }
    if (!second) {
      // largest scaled logit of the tile: the largest product, or the smallest under a negative scale
      float m_loc;
      if (sc_t >= 0.f) {
        m_loc = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) m_loc = fmaxf(m_loc, s[kb][v]);
      } else {
        m_loc = INFINITY;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) m_loc = fminf(m_loc, s[kb][v]);
      }
      const float m_new = fmaxf(m_run, max_with_other_half(m_loc * sc_t));
      float psum = 0.f;
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) psum += __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][v], sc_t, -m_new));
      l_run = l_run * __builtin_amdgcn_exp2f(m_run - m_new) + psum;
      m_run = m_new;
      if (c == p.nbk - 1) weight = row_valid ? 1.0f / sum_with_other_half(l_run) : 0.f;
    } else {
      float e = 0.f;
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) e += __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][v], sc_t, -m_run));
      e = wave_sum(e * weight);
      if (rb.lane == 0) part[rb.wave * p.nbk + c] = e;
    }
  }
  __syncthreads();
  const float inv_rows = 1.0f / (float)rows_valid;
  float *const out = gE + ((size_t)bh * p.nbq + r) * (size_t)p.nbk;
  for (int c = tid; c < p.nbk; c += NT) {
    float e = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) e += part[w * p.nbk + c];
    out[c] = e * inv_rows;
  }
}

// The same energies in ONE pass over the key tiles, for callers that bring a
// workspace.  While the online-softmax statistics of a row are still running,
// the mass it puts on key block c is only known relative to the running
// maximum of that moment; its logarithm, t[c][row] = m + log2(sum over the
// block's keys of 2^(s - m)), needs no reference.  A workgroup keeps these
// nbk x BQ values in its slice of the workspace (one 128-byte store per wave
// and tile), and once the row's log-sum-exp L is known reads its own values
// back: E[r][c] = mean over the rows of 2^(t[c][row] - L[row]).  Every lane
// reads only what it wrote itself (the two lanes of a row take the even and the
// odd key blocks).  Half the matrix work of the two-pass
// kernel; 2 x nbk x BQ x 4 bytes of extra traffic per query block.
//
// Persistent workgroups, no counters: workgroup i serves XCD i mod xcds and
// takes every (workgroups of that XCD)-th unit of the XCD's contiguous range;
// all units cost the same.  The workspace slice belongs to the workgroup, not
// to the unit.
struct EnergyOnePassDims {
  EnergyDims e;
  int n_wg;  // workgroups launched
  int xcds;  // 8, or 1 when fewer than 8 workgroups run
};

template <int D, int BQ, int BK>
__global__ __launch_bounds__(BQ * 2, (BQ >= 128 ? 2 : 1)) void block_energy_onepass_kernel(
    const uint16_t *__restrict__ gq, const uint16_t *__restrict__ gk, float *__restrict__ gE,
    float *__restrict__ workspace, const EnergyOnePassDims pp) {
  using RB = RowBlock<D, BQ, BK>;
  constexpr int NT = RB::NT, NW = RB::NW, KB = RB::KB, ROWB = RB::ROWB, TILE_BYTES = RB::TILE_BYTES;
  const EnergyDims &p = pp.e;

  extern __shared__ __attribute__((aligned(1024))) char lds[];  // EnergyLds::bytes(nbk)

  const int xcd = blockIdx.x % pp.xcds;
  const int slot = blockIdx.x / pp.xcds;
  const int wgs_here = (pp.n_wg - xcd + pp.xcds - 1) / pp.xcds;  // workgroups serving this XCD's range
  const long long units = (long long)p.B * p.H * p.nbq;
  const long long lo = units * xcd / pp.xcds;
  const long long hi = units * (xcd + 1) / pp.xcds;

  RB rb(lds);
  const int tid = rb.tid;
  const int N = p.N;
  float *const part = reinterpret_cast<float *>(lds + EnergyLds<D, BQ, BK>::PART_OFF);
  float *const mine = workspace + (size_t)blockIdx.x * p.nbk * BQ + rb.row_in_block();  // + c * BQ
  const float sc = p.scale_log2e;
  const bool ragged = (N % BK) != 0;

  for (long long unit = lo + slot; unit < hi; unit += wgs_here) {
    const int r = (int)(unit % p.nbq);
    const long long bh = unit / p.nbq;  // b * H + h
    const size_t head_off = (size_t)bh * (size_t)N * D;
    const u32x4 Kres = head_rsrc(gk + head_off, (uint32_t)N * ROWB);
    const int rows_valid = min(BQ, N - r * BQ);
    const bool row_valid = rb.row_in_block() < rows_valid;

    // both K buffers are free: every wave is behind the barrier that followed the last tile of the previous unit
    rb.issue_k_at(Kres, 0, 0);
    rb.begin(gq + head_off + (size_t)(r * BQ + (row_valid ? rb.row_in_block() : 0)) * D);

    float m_run = -INFINITY, l_run = 0.f, t_prev = 0.f;
    for (int c = 0; c < p.nbk; ++c) {
      wait_vmem<0>();
      __syncthreads();  // tile c has landed for every wave; everyone is done with the other buffer
      // the value of the previous tile goes out here, a whole tile ahead of the next wait for memory
      if (c > 0 && ((c - 1) & 1) == rb.g) mine[(size_t)(c - 1) * BQ] = t_prev;
      if (c + 1 < p.nbk) rb.issue_k_at(Kres, c + 1, ((c + 1) & 1) * TILE_BYTES);
      f32x16 s[KB];
      rb.scores((c & 1) * TILE_BYTES, s);
      float sc_t = sc;
      if (ragged && c == p.nbk - 1) {  // keys >= N sit at -inf; the tile is scaled up front, multiplier 1 from then on
        int limit = N - c * BK - 8 * rb.g;  // this lane's key offsets below `limit` exist
        asm volatile("" : "+v"(limit));      // keeps the comparisons (and their 64 masks) inside this branch
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            s[kb][v] = 32 * kb + 16 * (v >> 3) + (v & 7) < limit ? s[kb][v] * sc : -INFINITY;
        sc_t = 1.0f;
      }
      // The reference m_run of the exponentials only has to keep them in range, it need not be the
      // maximum: the tile is first summed against the reference as it stands, and only if some
      // lane's sum leaves the safe range (always on the first tile, where the reference is -inf)
      // does the wave look for the tile's maximum, move the reference and sum again.  The sums
      // stay below 2^100 per tile, so the row sum cannot overflow.
      float psum = 0.f;
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) psum += __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][v], sc_t, -m_run));
      if (__any(!(psum < 0x1p100f))) {
        float m_loc;
        if (sc_t >= 0.f) {
          m_loc = -INFINITY;
#pragma unroll
          for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) m_loc = fmaxf(m_loc, s[kb][v]);
        } else {
          m_loc = INFINITY;
#pragma unroll
          for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) m_loc = fminf(m_loc, s[kb][v]);
        }
        const float m_new = fmaxf(m_run, max_with_other_half(m_loc * sc_t));
        psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) psum += __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][v], sc_t, -m_new));
        l_run *= __builtin_amdgcn_exp2f(m_run - m_new);  // 0 on the first tile
        m_run = m_new;
      }
      l_run += psum;
      // log2 of the row's mass on this block (-inf when it underflowed: the block then counts as 0)
      t_prev = m_run + __builtin_amdgcn_logf(sum_with_other_half(psum));
    }
    if (((p.nbk - 1) & 1) == rb.g) mine[(size_t)(p.nbk - 1) * BQ] = t_prev;
    const float lse2 = m_run + __builtin_amdgcn_logf(sum_with_other_half(l_run));
    wait_vmem<0>();
    __syncthreads();  // K buffers free for the next unit; `part` of the previous unit fully consumed
    // this lane's own values back (blocks c = 2 j + g), 16 loads in flight at a time; each half of
    // the wave sums its 32 rows
    for (int c0 = 0; c0 < p.nbk; c0 += 32) {
      float t[16];
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int c = c0 + 2 * j + rb.g;
        t[j] = c < p.nbk ? __hip_atomic_load(mine + (size_t)c * BQ, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                         : -INFINITY;  // read at L2, where the stores went
      }
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int c = c0 + 2 * j + rb.g;
        const float e = half_wave_sum(row_valid ? __builtin_amdgcn_exp2f(t[j] - lse2) : 0.f);
        if (rb.l32 == 0 && c < p.nbk) part[rb.wave * p.nbk + c] = e;
      }
    }
    __syncthreads();
    const float inv_rows = 1.0f / (float)rows_valid;
    float *const out = gE + ((size_t)bh * p.nbq + r) * (size_t)p.nbk;
    for (int c = tid; c < p.nbk; c += NT) {
      float e = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) e += part[w * p.nbk + c];
      out[c] = e * inv_rows;
    }
  }
}

}  // namespace calibatt_dev
