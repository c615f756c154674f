// Spatial similarity score of attention heads (paper, Section 3.3, detection of
// spatially repetitive heads) without materialising the attention map.
// gfx950 (MI355X), bf16 in, fp32 out.
//
// The score of a head is the mean, over spatial rows, of the cosine similarity
// between the attention rows of the row's tokens and those of the matching
// tokens of its anchor row (same frame, same column), both flattened over
// (column, key).  Per token t with partner a:
//     dot[t] = sum_j P[t][j] P[a][j],  nt[t] = sum_j P[t][j]^2,  na[t] = sum_j P[a][j]^2
// and per spatial row  cos = sum_x dot / sqrt(sum_x nt * sum_x na).
//
// Kernel 1: one workgroup per (batch, head, 128 tokens).  A lane owns a token
// AND its partner: two query operands, two score tiles per key tile
// (RowBlock::scores twice), ONE pass over all keys: the row sums of both and
// the three sums of products are kept relative to the running maxima of the
// two queries and rescaled when a maximum moves (the sums of products by the
// product of the two factors), exactly as an online softmax keeps its row sum;
// the normalisers divide out at the end.  Writes the normalised triple of
// every token.
// Kernel 2: one wavefront per (batch, head) adds the triples of each spatial
// row, forms the cosine and averages over rows in a fixed order.
#pragma once
#include "attn_kernel_2wg.h"

namespace calibatt_dev {

struct SimilarityDims {
  int B, H, N, n_tok, nbq, nbk, row_len;
  float scale_log2e;
};

constexpr int SIM_BQ = 128;
constexpr int SIM_BK = 128;
constexpr int SIM_XCDS = 8;

template <int D>
__global__ __launch_bounds__(SIM_BQ * 2, 2) void pair_similarity_kernel(
    const uint16_t *__restrict__ gq, const uint16_t *__restrict__ gk, const int32_t *__restrict__ partner,
    float *__restrict__ triples, const SimilarityDims p) {
  constexpr int BQ = SIM_BQ, BK = SIM_BK;
  using RB = RowBlock<D, BQ, BK>;
  constexpr int KB = RB::KB, DS = RB::DS, ROWB = RB::ROWB, TILE_BYTES = RB::TILE_BYTES;

  extern __shared__ __attribute__((aligned(1024))) char lds[];  // two K tiles

  const int xcd = blockIdx.x % SIM_XCDS;
  const int slot = blockIdx.x / SIM_XCDS;
  const long long units = (long long)p.B * p.H * p.nbq;
  const long long lo = units * xcd / SIM_XCDS;
  const long long hi = units * (xcd + 1) / SIM_XCDS;
  if (slot >= hi - lo) return;
  const int unit = (int)(lo + slot);
  const int r = unit % p.nbq;
  const int bh = unit / p.nbq;

  RB rb(lds);
  const int N = p.N;
  const size_t head_off = (size_t)bh * (size_t)N * D;
  const u32x4 Kres = head_rsrc(gk + head_off, (uint32_t)N * ROWB);
  rb.issue_k_at(Kres, 0, 0);

  const int tok_raw = r * BQ + rb.row_in_block();
  const bool valid = tok_raw < p.n_tok;
  const int tok = valid ? tok_raw : p.n_tok - 1;
  int par = partner[tok];
  par = par < 0 ? 0 : (par < N ? par : N - 1);
  typename RB::Operand q_t[DS], q_a[DS];
  rb.load_q(gq + head_off + (size_t)tok * D, q_t);
  rb.load_q(gq + head_off + (size_t)par * D, q_a);

  const float sc = p.scale_log2e;
  const bool ragged = (N % BK) != 0;
  float m_t = -INFINITY, l_t = 0.f, m_a = -INFINITY, l_a = 0.f;
  float dot = 0.f, nt = 0.f, na = 0.f;

  // largest scaled logit of one query over one tile of raw products (multiplier sc_t still to apply),
  // folded into the running maximum; returns the factor 2^(old max - new max) for what was summed so far
  auto fold_max = [&](const f32x16 (&s)[KB], float sc_t, float &m_run) {
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
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);  // 0 on the first tile
    m_run = m_new;
    return alpha;
  };
  // keys >= N of the ragged last tile to -inf; scales the tile up front
  auto mask_tail = [&](f32x16 (&s)[KB], int c) {
    int limit = N - c * BK - 8 * rb.g;  // this lane's key offsets below `limit` exist
    asm volatile("" : "+v"(limit));      // keeps the comparisons (and their 64 masks) out of the tile loop's prologue
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        s[kb][v] = 32 * kb + 16 * (v >> 3) + (v & 7) < limit ? s[kb][v] * sc : -INFINITY;
  };

  // One pass: all five sums are kept relative to the running maxima of the two queries and
  // rescaled when a maximum moves, like the row sum of an online softmax.  Tile c sits in buffer c & 1.
  for (int c = 0; c < p.nbk; ++c) {
    wait_vmem<0>();
    __syncthreads();  // tile c has landed for every wave; everyone is done with the other buffer
    if (c + 1 < p.nbk) rb.issue_k_at(Kres, c + 1, ((c + 1) & 1) * TILE_BYTES);
    f32x16 s_t[KB], s_a[KB];
    rb.scores((c & 1) * TILE_BYTES, s_t, q_t);
    rb.scores((c & 1) * TILE_BYTES, s_a, q_a);
    float sc_t = sc;
    if (ragged && c == p.nbk - 1) {
      mask_tail(s_t, c);
      mask_tail(s_a, c);
      sc_t = 1.0f;
    }
    const float alpha_t = fold_max(s_t, sc_t, m_t);
    const float alpha_a = fold_max(s_a, sc_t, m_a);
    float sum_t = 0.f, sum_a = 0.f, sum_ta = 0.f, sum_tt = 0.f, sum_aa = 0.f;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float et = __builtin_amdgcn_exp2f(__builtin_fmaf(s_t[kb][v], sc_t, -m_t));
        const float ea = __builtin_amdgcn_exp2f(__builtin_fmaf(s_a[kb][v], sc_t, -m_a));
        sum_t += et;
        sum_a += ea;
        sum_ta = __builtin_fmaf(et, ea, sum_ta);
        sum_tt = __builtin_fmaf(et, et, sum_tt);
        sum_aa = __builtin_fmaf(ea, ea, sum_aa);
      }
    l_t = __builtin_fmaf(l_t, alpha_t, sum_t);
    l_a = __builtin_fmaf(l_a, alpha_a, sum_a);
    dot = __builtin_fmaf(dot, alpha_t * alpha_a, sum_ta);
    nt = __builtin_fmaf(nt, alpha_t * alpha_t, sum_tt);
    na = __builtin_fmaf(na, alpha_a * alpha_a, sum_aa);
  }
  const float wt = 1.0f / sum_with_other_half(l_t);
  const float wa = 1.0f / sum_with_other_half(l_a);
  dot = sum_with_other_half(dot) * wt * wa;
  nt = sum_with_other_half(nt) * wt * wt;
  na = sum_with_other_half(na) * wa * wa;
  if (valid && rb.g == 0) {
    float *o = triples + ((size_t)bh * p.n_tok + tok) * 3;
    o[0] = dot;
    o[1] = nt;
    o[2] = na;
  }
}

// score[b*H + h] = mean over the n_tok / row_len spatial rows of the row's cosine.
__global__ __launch_bounds__(64) void similarity_reduce_kernel(const float *__restrict__ triples,
                                                               float *__restrict__ score, int n_tok, int row_len) {
  const int bh = blockIdx.x;
  const int n_rows = n_tok / row_len;
  const float *base = triples + (size_t)bh * n_tok * 3;
  float acc = 0.f;
  for (int row = threadIdx.x; row < n_rows; row += 64) {
    float dot = 0.f, nt = 0.f, na = 0.f;
    for (int x = 0; x < row_len; ++x) {
      const float *t = base + ((size_t)row * row_len + x) * 3;
      dot += t[0];
      nt += t[1];
      na += t[2];
    }
    acc += dot / (sqrtf(nt) * sqrtf(na));
  }
  acc = wave_sum(acc);
  if (threadIdx.x == 0) score[bh] = acc / (float)n_rows;
}

}  // namespace calibatt_dev
