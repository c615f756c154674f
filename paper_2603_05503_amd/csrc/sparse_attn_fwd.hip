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
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "calibatt.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
#define LDS_PTR(T) __attribute__((address_space(3))) T *

struct FwdParams {
  const uint16_t *q, *k, *v;
  uint16_t *out;
  const int32_t *row_ptr, *col_idx, *work, *fan_ptr, *fan_dst;
  int B, H, N, nbq, nbk, n_work;
  float scale_log2e;
};

template <int N_OUTSTANDING>
__device__ __forceinline__ void wait_vmem() {
  // waits until at most N_OUTSTANDING vector-memory loads of this wave are in flight
  if constexpr (N_OUTSTANDING == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  else if constexpr (N_OUTSTANDING == 1) asm volatile("s_waitcnt vmcnt(1)" ::: "memory");
  else if constexpr (N_OUTSTANDING == 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
  else if constexpr (N_OUTSTANDING == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
  else if constexpr (N_OUTSTANDING == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
  else if constexpr (N_OUTSTANDING == 16) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
  else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// 16-byte-chunk swizzles.  CH = chunks per row (D/8).  A 256-byte LDS line
// (all 64 banks) holds 16/CH rows.
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

// Stream one ROWS x D bf16 tile global -> LDS.  Rows >= N are clamped to N-1
// (their logits are masked later).  LDS chunk (row, c') receives global chunk
// (row, c' ^ swz(row)).
template <int D, int ROWS, int NT, bool FOR_V>
__device__ __forceinline__ void load_tile(const uint16_t *__restrict__ head_base, int row0, int N,
                                          char *lds_tile, int tid) {
  constexpr int CH = D / 8;
  constexpr int CHUNKS = ROWS * CH;
  constexpr int ITERS = CHUNKS / NT;
  static_assert(CHUNKS % NT == 0, "tile must split evenly over the workgroup");
  const int wave_base = (tid / 64) * 64;
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int L = it * NT + tid;
    const int row = L / CH;
    const int cs = L % CH;
    const int c = cs ^ (FOR_V ? v_swz<D>(row) : k_swz<D>(row));
    int grow = row0 + row;
    grow = grow < N ? grow : N - 1;
    const uint16_t *src = head_base + (size_t)grow * D + c * 8;
    char *dst = lds_tile + (size_t)(it * NT + wave_base) * 16;  // wave-uniform; lane*16 is implicit
    __builtin_amdgcn_global_load_lds(src, (LDS_PTR(void))dst, 16, 0, 0);
  }
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  bf16x2 t;
  t[0] = (__bf16)lo;
  t[1] = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, t);
}

template <int D, int BQ, int BK>
__global__ __launch_bounds__(BQ * 2, (BQ >= 128 ? 2 : 1)) void sparse_attn_fwd_kernel(const FwdParams p) {
  constexpr int NW = BQ / 32;     // wavefronts per workgroup
  constexpr int NT = NW * 64;     // threads
  constexpr int CH = D / 8;       // 16-byte chunks per row
  constexpr int KB = BK / 32;     // 32-key sub-blocks per tile
  constexpr int DS = D / 16;      // k-slabs of the QK^T contraction
  constexpr int DB = D / 32;      // 32-wide d blocks of O^T
  constexpr int ROWB = D * 2;     // bytes per LDS row
  constexpr int TILE_BYTES = BK * ROWB;
  constexpr int LOADS_PER_WAVE = (BK * CH) / NT;  // direct-to-LDS instructions per wave and tile
  constexpr int OST = ROWB + 16;  // padded row stride of the output staging tile
  constexpr int LDS_BYTES = (2 * TILE_BYTES > BQ * OST) ? 2 * TILE_BYTES : BQ * OST;

  __shared__ __attribute__((aligned(1024))) char lds[LDS_BYTES];
  char *const ldsK = lds;
  char *const ldsV = lds + TILE_BYTES;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int l32 = lane & 31;
  const int g = lane >> 5;

  const int item = blockIdx.x / p.B;
  const int b = blockIdx.x - item * p.B;
  const int id = p.work[item];
  const int h = id / p.nbq;
  const int r = id - h * p.nbq;
  const int N = p.N;
  const size_t head_off = ((size_t)b * p.H + h) * (size_t)N * D;
  const uint16_t *__restrict__ Kh = p.k + head_off;
  const uint16_t *__restrict__ Vh = p.v + head_off;

  const int cbeg = p.row_ptr[id];
  const int cend = p.row_ptr[id + 1];

  // Q^T as MFMA B operand: lane (query l32, half g) holds d = 16 s + 8 g + [0,8)
  bf16x8 qreg[DS];
  {
    int qrow = r * BQ + wave * 32 + l32;
    qrow = qrow < N ? qrow : N - 1;
    const uint16_t *qp = p.q + head_off + (size_t)qrow * D + 8 * g;
#pragma unroll
    for (int s = 0; s < DS; ++s) qreg[s] = *reinterpret_cast<const bf16x8 *>(qp + 16 * s);
  }
  // first K and V tiles (issued after the Q loads: vmem loads retire in order)
  if (cbeg < cend) {
    const int c0 = p.col_idx[cbeg];
    load_tile<D, BK, NT, false>(Kh, c0 * BK, N, ldsK, tid);
    load_tile<D, BK, NT, true>(Vh, c0 * BK, N, ldsV, tid);
  }

  f32x16 o[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
  float m_run = -INFINITY;  // running max of scaled (log2-domain) logits, shared by lane and lane^32
  float l_run = 0.f;        // this lane's share of the running row sum

  // K operand row for MFMA row i = l32: swap bits 2 and 3 so that the 8 S^T
  // values a lane holds per 16-key slab belong to 8 consecutive keys.
  const int krow_in_kb = (l32 & 0x13) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);
  // transposing V read: 16-lane block -> (d sub-block, key half); lane L in block
  const int L16 = lane & 15;
  const int blk = lane >> 4;
  const int v_row_off = 8 * (blk >> 1) + (L16 >> 2);                 // + 32 kb + 16 s2 + 4 t
  const int v_chunk_off = 2 * (blk & 1) + ((L16 & 3) >> 1);          // + 4 db
  const int v_byte_off = (L16 & 1) * 8;

  for (int ci = cbeg; ci < cend; ++ci) {
    const int c = p.col_idx[ci];
    const bool has_next = ci + 1 < cend;
    const int c_next = has_next ? p.col_idx[ci + 1] : 0;

    // ---- S^T = K Q^T --------------------------------------------------------
    // K[ci] was issued before V[ci]: allow V's loads to stay in flight.
    wait_vmem<LOADS_PER_WAVE>();
    __syncthreads();
    f32x16 s_acc[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
      for (int v = 0; v < 16; ++v) s_acc[kb][v] = 0.f;
      const int krow = 32 * kb + krow_in_kb;
      const char *kbase = ldsK + krow * ROWB;
      const int sw = k_swz<D>(krow);
#pragma unroll
      for (int s = 0; s < DS; ++s) {
        const int cs = (2 * s + g) ^ sw;
        const bf16x8 a = *reinterpret_cast<const bf16x8 *>(kbase + cs * 16);
        s_acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[s], s_acc[kb], 0, 0, 0);
      }
    }
    __syncthreads();  // every wave is done with the K tile
    if (has_next) load_tile<D, BK, NT, false>(Kh, c_next * BK, N, ldsK, tid);

    // ---- online softmax -----------------------------------------------------
    const float sc = p.scale_log2e;
    float m_loc = -INFINITY;
    if (c == p.nbk - 1 && (N % BK) != 0) {
      const int key0 = c * BK + 8 * g;
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = key0 + 32 * kb + 16 * (v >> 3) + (v & 7);
          const float t = s_acc[kb][v] * sc;
          s_acc[kb][v] = key < N ? t : -INFINITY;
        }
    } else {
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) s_acc[kb][v] *= sc;
    }
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) m_loc = fmaxf(m_loc, s_acc[kb][v]);
    m_loc = fmaxf(m_loc, __shfl_xor(m_loc, 32));
    const float m_new = fmaxf(m_run, m_loc);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);  // 0 on the first tile
    m_run = m_new;
    float psum = 0.f;
    uint32_t pb[KB][8];  // bf16 pairs: pb[kb][4*s2 + j] = keys (2j, 2j+1) of slab s2
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int v = 0; v < 16; v += 2) {
        const float p0 = __builtin_amdgcn_exp2f(s_acc[kb][v] - m_new);
        const float p1 = __builtin_amdgcn_exp2f(s_acc[kb][v + 1] - m_new);
        psum += p0 + p1;
        pb[kb][v >> 1] = pack_bf16(p0, p1);
      }
    l_run = l_run * alpha + psum;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[db][v] *= alpha;

    // ---- O^T += V^T P^T -----------------------------------------------------
    if (has_next) wait_vmem<LOADS_PER_WAVE>(); else wait_vmem<0>();
    __syncthreads();
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        u32x4 pw = {pb[kb][4 * s2 + 0], pb[kb][4 * s2 + 1], pb[kb][4 * s2 + 2], pb[kb][4 * s2 + 3]};
        const bf16x8 pB = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          u32x2 lo, hi;
          {
            const int row = 32 * kb + 16 * s2 + v_row_off;
            const int cs = (4 * db + v_chunk_off) ^ v_swz<D>(row);
            lo = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                                               (LDS_PTR(bf16x4))(ldsV + row * ROWB + cs * 16 + v_byte_off)));
          }
          {
            const int row = 32 * kb + 16 * s2 + 4 + v_row_off;
            const int cs = (4 * db + v_chunk_off) ^ v_swz<D>(row);
            hi = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                                               (LDS_PTR(bf16x4))(ldsV + row * ROWB + cs * 16 + v_byte_off)));
          }
          u32x4 aw = {lo[0], lo[1], hi[0], hi[1]};
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, aw), pB, o[db], 0, 0, 0);
        }
      }
    __syncthreads();  // every wave is done with the V tile
    if (has_next) load_tile<D, BK, NT, true>(Vh, c_next * BK, N, ldsV, tid);
  }

  // ---- normalise, stage in LDS, store to the block and its repeat targets ----
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
  __syncthreads();
  {
    char *orow = lds + (wave * 32 + l32) * OST;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        u32x2 w;
        w[0] = pack_bf16(o[db][4 * a + 0] * inv, o[db][4 * a + 1] * inv);
        w[1] = pack_bf16(o[db][4 * a + 2] * inv, o[db][4 * a + 3] * inv);
        *reinterpret_cast<u32x2 *>(orow + (32 * db + 8 * a + 4 * g) * 2) = w;
      }
  }
  __syncthreads();
  const int fbeg = p.fan_ptr[item];
  const int fend = p.fan_ptr[item + 1];
  uint16_t *const out_head = p.out + head_off;
  for (int f = fbeg - 1; f < fend; ++f) {
    const int rd = f < fbeg ? r : p.fan_dst[f];
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
}

template <int D, int BQ, int BK>
int launch(const FwdParams &p, hipStream_t stream) {
  const long long grid = (long long)p.n_work * p.B;
  if (grid <= 0) return CALIBATT_OK;
  if (grid > 0x7fffffffLL) return CALIBATT_ERR_SHAPE;
  hipLaunchKernelGGL((sparse_attn_fwd_kernel<D, BQ, BK>), dim3((unsigned)grid), dim3(BQ * 2), 0, stream, p);
  return hipGetLastError() == hipSuccess ? CALIBATT_OK : CALIBATT_ERR_LAUNCH;
}

}  // namespace

extern "C" int calibatt_sparse_attn_fwd(const void *q, const void *k, const void *v, void *out, int B,
                                        int H, int N, int D, int block_q, int block_k,
                                        const calibatt_pattern *pattern, float scale, void *stream) {
  if (!q || !k || !v || !out || !pattern) return CALIBATT_ERR_NULL;
  if (B <= 0 || H <= 0 || N <= 0 || D <= 0 || block_q <= 0 || block_k <= 0) return CALIBATT_ERR_SHAPE;
  if (!(D == 64 || D == 128) || !(block_q == 64 || block_q == 128) || !(block_k == 64 || block_k == 128))
    return CALIBATT_ERR_UNSUPPORTED;
  if (out == q || out == k || out == v) return CALIBATT_ERR_SHAPE;
  const int nbq = (N + block_q - 1) / block_q, nbk = (N + block_k - 1) / block_k;
  if (pattern->H != H || pattern->N != N || pattern->block_q != block_q || pattern->block_k != block_k ||
      pattern->nbq != nbq || pattern->nbk != nbk || pattern->n_work < 0 || pattern->n_repeat < 0 ||
      (int64_t)pattern->n_work + pattern->n_repeat != (int64_t)H * nbq)
    return CALIBATT_ERR_PATTERN_MISMATCH;
  if (!pattern->row_ptr || !pattern->work || !pattern->fan_ptr ||
      (pattern->nnz > 0 && !pattern->col_idx) || (pattern->n_repeat > 0 && !pattern->fan_dst))
    return CALIBATT_ERR_NULL;
  if ((size_t)B * H * N * D > 0x7fffffff00ULL) return CALIBATT_ERR_SHAPE;

  FwdParams p;
  p.q = (const uint16_t *)q;
  p.k = (const uint16_t *)k;
  p.v = (const uint16_t *)v;
  p.out = (uint16_t *)out;
  p.row_ptr = pattern->row_ptr;
  p.col_idx = pattern->col_idx;
  p.work = pattern->work;
  p.fan_ptr = pattern->fan_ptr;
  p.fan_dst = pattern->fan_dst;
  p.B = B;
  p.H = H;
  p.N = N;
  p.nbq = nbq;
  p.nbk = nbk;
  p.n_work = pattern->n_work;
  p.scale_log2e = scale * 1.4426950408889634f;
  hipStream_t s = (hipStream_t)stream;
#define CALIBATT_CASE(d, bq, bk) \
  if (D == d && block_q == bq && block_k == bk) return launch<d, bq, bk>(p, s);
  CALIBATT_CASE(128, 128, 128)
  CALIBATT_CASE(128, 128, 64)
  CALIBATT_CASE(128, 64, 128)
  CALIBATT_CASE(128, 64, 64)
  CALIBATT_CASE(64, 128, 128)
  CALIBATT_CASE(64, 128, 64)
  CALIBATT_CASE(64, 64, 128)
  CALIBATT_CASE(64, 64, 64)
#undef CALIBATT_CASE
  return CALIBATT_ERR_UNSUPPORTED;
}
