/*
 * calibatt.h - C ABI of the block-sparse attention forward with repeated
 * query blocks (inference hot path of calibrated sparse attention for video
 * diffusion transformers), MI355X / gfx950.
 *
 * Two stages, as in the paper's Section 3.4 ("Inference stage"):
 *   1. once per calibrated (timestep, layer) pattern, on the host:
 *      calibatt_compile_pattern() turns the binary block mask M (Section 3.2:
 *      entry 1 = block computed, 0 = skipped) and the map of repeated query
 *      blocks (block-level form of Section 3.3) into read-only index lists;
 *   2. at every attention call: calibatt_sparse_attn_fwd() runs the tiled
 *      forward (Section 2, Eq. 3-4: per query block, loop over key/value
 *      blocks with an online softmax) over the kept blocks only.
 * Heads flagged as spatially repetitive (Section 3.3 at token-row granularity)
 * go through calibatt_anchor_map() / calibatt_anchor_attn_fwd() instead.
 * Both forwards have a *_strided variant for tensors that are not packed.
 *
 * The calibration stage (Section 3.2-3.3) that produces the masks and the
 * flags: calibatt_block_energy() / calibatt_block_energy_onepass() and
 * calibatt_spatial_similarity() on the GPU; calibatt_select_blocks() and the
 * vote counters on the host or, as *_device, on the GPU;
 * calibatt_epsilon_schedule() on the host.  Skip-list tools of the supplement (Sections A.2, A.3):
 * calibatt_encode_intervals() (a compact form of the index lists that the
 * forward reads directly), calibatt_merge_intervals(),
 * calibatt_share_timesteps().
 *
 * Plain C, no exceptions cross the boundary, every buffer is owned by the
 * caller, and the library allocates no device memory (scratch comes in through
 * workspace arguments).  Nothing in the environment changes what a call does.
 * The only state kept between calls is a per-device cache of launch facts (how
 * many workgroups of a kernel the device holds), filled on first use through
 * atomics: calls may come from any number of host threads at once, as long as
 * calls that overlap on the GPU use separate workspaces.  All functions return a
 * calibatt_status (0 = success, negative = error) unless stated otherwise.
 */
#ifndef CALIBATT_H
#define CALIBATT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Element strides of a [B][H][N][D] tensor whose D axis is contiguous (see
 * calibatt_sparse_attn_fwd_strided). */
typedef struct calibatt_strides {
  int64_t b, h, n; /* in elements */
} calibatt_strides;

typedef enum calibatt_status {
  CALIBATT_OK = 0,
  CALIBATT_ERR_NULL = -1,             /* a required pointer is NULL */
  CALIBATT_ERR_SHAPE = -2,            /* non-positive or inconsistent dimension */
  CALIBATT_ERR_UNSUPPORTED = -3,      /* head dim / block size / order not built */
  CALIBATT_ERR_REPEAT_RANGE = -4,     /* repeat value outside {-1} U [0, nbq) or self */
  CALIBATT_ERR_REPEAT_CHAIN = -5,     /* source of a repeated block is itself repeated */
  CALIBATT_ERR_REPEAT_TAIL = -6,      /* short last block used as source of a full block */
  CALIBATT_ERR_BUFFER_TOO_SMALL = -7, /* a buffer (col_cap, a workspace, the built-in scratch) is too small */
  CALIBATT_ERR_PATTERN_MISMATCH = -8, /* pattern was compiled for another H/N/block */
  CALIBATT_ERR_LAUNCH = -9,           /* the HIP runtime refused the launch */
  CALIBATT_ERR_NOMEM = -10            /* host scratch allocation failed in compile */
} calibatt_status;

/* Schedule orders for calibatt_compile_pattern (ids are h*nbq + r). */
enum {
  CALIBATT_ORDER_NATURAL = 0,   /* (h, r) ascending */
  CALIBATT_ORDER_LONGEST = 1,   /* kept count descending, then h, then r */
  CALIBATT_ORDER_HEAD_LONGEST = 2, /* h ascending, then kept count descending, then r */
  CALIBATT_ORDER_XCD_HEADS = 3 /* heads dealt to CALIBATT_GROUPS groups (one per XCD, each XCD has its
                                  own L2): heads by total kept blocks descending (then h), each to the
                                  group with the smallest load so far (then lowest group).  A group's
                                  segment of work lists first its long blocks (2*count*n_work > 3*nnz)
                                  by count descending, then dealing order of the head, then r; then the
                                  other blocks head by head in dealing order, r ascending.  Segments
                                  follow each other in group order. */
  ,
  CALIBATT_ORDER_XCD_HEADS_TAIL = 4 /* heads dealt to groups as for CALIBATT_ORDER_XCD_HEADS; a group's
                                  segment lists its heads in dealing order and, within a head, the
                                  blocks by count descending, then r.  Every head, and with it the
                                  group's queue, ends with its shortest blocks: heads change over
                                  sharply (few heads live at a time) and the persistent workgroups'
                                  idle tail is short. */
};
#define CALIBATT_GROUPS 8

/*
 * Compiled pattern: plain data, all pointers BORROWED (never freed by the
 * library).  calibatt_compile_pattern() fills it with the HOST buffers the
 * caller passed in; before calibatt_sparse_attn_fwd() the caller copies the
 * six arrays to the GPU and stores the DEVICE pointers in a copy of the struct
 * (the struct itself stays in host memory).
 *
 * nbq = ceil(N/block_q), nbk = ceil(N/block_k).  A "row" is one query block of
 * one head, id = h*nbq + r.
 */
typedef struct calibatt_pattern {
  int32_t H, N, block_q, block_k;
  int32_t nbq, nbk;
  int32_t n_work;    /* rows that are computed (not repeated) */
  int32_t n_repeat;  /* rows that are copies; n_work + n_repeat == H*nbq */
  int32_t order;     /* schedule order used for `work` */
  int32_t max_row;   /* largest kept count of any computed row */
  int64_t nnz;       /* kept blocks over computed rows */
  const int32_t *row_ptr;    /* [H*nbq + 1] offsets into col_idx; repeated rows are empty */
  const int32_t *col_idx;    /* [nnz] kept key/value block columns, ascending within a row */
  const int32_t *repeat_src; /* [H*nbq] -1, or the source query block of the same head */
  const int32_t *work;       /* [n_work] row ids in schedule order */
  const int32_t *fan_ptr;    /* [n_work + 1] offsets into fan_dst, per work item */
  const int32_t *fan_dst;    /* [n_repeat] query blocks that copy work item i, ascending */
  int32_t *work_counter;     /* NULL, or DEVICE int32[16] workspace, see calibatt_sparse_attn_fwd */
  int32_t n_groups;          /* 1, or CALIBATT_GROUPS for the two CALIBATT_ORDER_XCD_HEADS* orders */
  int32_t group_ptr[CALIBATT_GROUPS + 1]; /* segment g of `work` is [group_ptr[g], group_ptr[g+1]) */
  /* Optional interval form of the kept-block lists (calibatt_encode_intervals): when both are
   * non-NULL the forward reads them and never touches col_idx, which may then be NULL. */
  const int32_t *iv_ptr;     /* [H*nbq + 1] offsets into iv */
  const uint32_t *iv;        /* interval words, see calibatt_encode_intervals */
  /* Optional: the pattern covers a subset of the tensor's heads.  NULL = pattern head h is tensor
   * head h (and pattern H must equal the tensor's H); else DEVICE int32 [H of the pattern], the
   * tensor head each pattern head reads and writes (entries outside the tensor's heads are
   * skipped; heads no entry names are left untouched).  calibatt_compile_pattern sets NULL. */
  const int32_t *head_map;
} calibatt_pattern;

/*
 * Validate a mask / repeat map and count what compile will produce.
 *
 * mask   HOST, uint8 [H][nbq][nbk] row-major; any non-zero byte = block kept
 *        (Section 3.2).  The mask row of a repeated block is ignored.
 * repeat HOST, int32 [H][nbq]; -1 = computed, s >= 0 = copy of query block s
 *        of the same head (Section 3.3 at block granularity); NULL = none.
 * nnz, n_work, n_repeat  HOST outputs, each may be NULL.
 * Errors: NULL, SHAPE, REPEAT_RANGE / REPEAT_CHAIN / REPEAT_TAIL.
 */
int calibatt_pattern_sizes(const uint8_t *mask, const int32_t *repeat, int H, int N, int block_q,
                           int block_k, int64_t *nnz, int32_t *n_work, int32_t *n_repeat);

/*
 * Compile a pattern into caller-provided HOST buffers (Section 3.4: the
 * per-row list of key block-columns to compute, precomputed once; supplement
 * A.2: padding-free flat layout).  The result is a pure function of the
 * inputs:
 *   row_ptr    [H*nbq + 1]  exclusive prefix sum of kept counts in (h, r) order
 *   col_idx    [col_cap]    first nnz entries written; needs col_cap >= nnz
 *   repeat_src [H*nbq]
 *   work       [H*nbq]      first n_work entries written, order per `order`
 *                           (out->n_groups / out->group_ptr describe its segments)
 *   fan_ptr    [H*nbq + 1]  first n_work + 1 entries written
 *   fan_dst    [H*nbq]      first n_repeat entries written
 * `out` receives the dimensions, counts and the six host pointers.
 * Errors: as calibatt_pattern_sizes, plus UNSUPPORTED (order),
 * BUFFER_TOO_SMALL, NOMEM.  On error the output buffers hold garbage.
 */
int calibatt_compile_pattern(const uint8_t *mask, const int32_t *repeat, int H, int N, int block_q,
                             int block_k, int order, int32_t *row_ptr, int32_t *col_idx,
                             int64_t col_cap, int32_t *repeat_src, int32_t *work, int32_t *fan_ptr,
                             int32_t *fan_dst, calibatt_pattern *out);

/*
 * Block-sparse attention forward (Section 2, Eq. 1-4 restricted to kept
 * blocks; Section 3.4).
 *
 * q, k, v  DEVICE, bf16, contiguous [B][H][N][D]; read only.
 * out      DEVICE, bf16, contiguous [B][H][N][D]; must not alias the inputs.
 *          Every row < N is written exactly once: a computed row holds
 *          softmax(scale * q K_kept^T) V_kept with fp32 accumulation, rounded
 *          to bf16; a row whose block keeps nothing holds zeros; a repeated
 *          block holds a bitwise copy of the leading rows of its source block.
 * pattern  HOST struct holding DEVICE pointers (see above).  The same pattern
 *          serves every batch index (supplement Section A: one mask for the
 *          conditional and unconditional branch).  Index contents cannot be
 *          validated on the device: build them with calibatt_compile_pattern
 *          (and calibatt_encode_intervals for the optional interval form,
 *          which replaces col_idx: pattern bytes shrink from 4 per kept block
 *          to 4 per run of consecutive kept blocks).
 *          pattern->work_counter selects how work items reach the GPU:
 *          NULL  - one workgroup per (computed query block, batch index), in
 *                  schedule order;
 *          else  - DEVICE int32[16] owned by the caller, all zero before the
 *                  first call.  A device-filling set of persistent workgroups
 *                  pops work items from one counter per group (uneven rows
 *                  then balance dynamically).  With n_groups ==
 *                  CALIBATT_GROUPS a workgroup first drains the group of the
 *                  XCD it runs on - the heads of one group then share that
 *                  XCD's L2 - and steals from the other groups afterwards.
 *                  The last workgroup to finish sets words 0..8 back to zero,
 *                  so consecutive calls on one stream may share the workspace.
 *                  Words 10 and 11 hold a diagnostic after every launch:
 *                  shader-clock cycles and ticks of the constant 100 MHz
 *                  counter during which workgroup 0 was resident (ratio x 100
 *                  MHz = the clock the GPU sustained); the other words are
 *                  reserved.
 *                  Calls that overlap in time (different streams) need
 *                  separate workspaces.  calibatt_compile_pattern sets NULL.
 * scale    multiplies the logits before the softmax (1/sqrt(D) in Eq. 1).
 * stream   hipStream_t (NULL = default stream).  The call only enqueues work.
 *
 * Supported: D in {64, 128}, block_q and block_k in {64, 128}; with D = 128 and
 * block_q = 128 also block_k in {96, 160, 192} (the key-block widths of the
 * supplement's block-size ablation).
 * Errors: NULL, SHAPE, UNSUPPORTED, PATTERN_MISMATCH (pattern compiled for a
 * different H, N, block_q or block_k), LAUNCH.
 */
int calibatt_sparse_attn_fwd(const void *q, const void *k, const void *v, void *out, int B, int H,
                             int N, int D, int block_q, int block_k,
                             const calibatt_pattern *pattern, float scale, void *stream);

/*
 * The same forward on tensors that are not packed [B][H][N][D]: element
 * (b, h, n, d) of q, k and v sits at b*in->b + h*in->h + n*in->n + d from the
 * respective pointer, element (b, h, n, d) of out at the same expression with
 * `out_strides`.  The D axis stays contiguous.  This covers the layouts
 * attention layers produce without a transpose: [B][N][H][D] (b = N*H*D, h = D,
 * n = H*D) and q, k, v as slices of one fused projection output
 * [B][N][3][H][D] (b = 3*N*H*D, h = D, n = 3*H*D, three base pointers).
 * Requirements: every stride a multiple of 8 elements, n >= D, pointers
 * 16-byte aligned, (N-1)*n*2 + D*2 < 2^32 bytes; the caller guarantees that
 * distinct (b, h, n) rows of out do not overlap.  Everything else as in
 * calibatt_sparse_attn_fwd, which is this call with packed strides.
 * Errors: as calibatt_sparse_attn_fwd; SHAPE also for strides or alignment
 * that break the requirements.
 */
int calibatt_sparse_attn_fwd_strided(const void *q, const void *k, const void *v, void *out, int B,
                                     int H, int N, int D, int block_q, int block_k,
                                     const calibatt_pattern *pattern, float scale,
                                     const calibatt_strides *in_strides,
                                     const calibatt_strides *out_strides, void *stream);

/*
 * The forward with every option.  `options` (HOST, required):
 *   in_strides, out_strides  NULL = packed [B][H][N][D], else as in the _strided call
 *   dtype   CALIBATT_BF16 (the models of the paper) or CALIBATT_F16: element
 *           type of q, k, v, out; accumulation is fp32 either way and the
 *           probabilities are rounded to that type for the second contraction
 *   lse     NULL, or DEVICE fp32 packed [B][H][N] (tensor heads): receives for
 *           every query the natural logarithm of the sum over its kept keys
 *           of exp(scale * q.k), -inf for a query that keeps no key; queries of
 *           a repeated block receive the value of their source row.  With it,
 *           results over disjoint key sets can be merged exactly.
 *   kernel  which of the two schedules of the same tile loop (Section 2,
 *           Eq. 3-4) runs.  CALIBATT_KERNEL_AUTO (0, what the other entry
 *           points use) and CALIBATT_KERNEL_INTERLEAVED: every wavefront
 *           issues the MFMAs of two contractions and the softmax of a third
 *           sub-tile as one instruction stream.
 *           CALIBATT_KERNEL_TWO_WORKGROUPS: the three phases of a tile run
 *           one after the other, two workgroups per CU overlap as they
 *           happen to fall; kept as the reference schedule (key blocks of
 *           64 and 128 keys only, UNSUPPORTED otherwise).  Both meet the
 *           same tolerance; their outputs differ in the last bits (the
 *           interleaved schedule moves the reference of its exponentials
 *           lazily).
 * Everything else as in calibatt_sparse_attn_fwd.
 * Errors: as calibatt_sparse_attn_fwd_strided; NULL (options), UNSUPPORTED
 * (dtype, kernel), SHAPE (lse not 4-byte aligned).
 */
enum { CALIBATT_BF16 = 0, CALIBATT_F16 = 1 };
enum { CALIBATT_KERNEL_AUTO = 0, CALIBATT_KERNEL_TWO_WORKGROUPS = 1, CALIBATT_KERNEL_INTERLEAVED = 2 };
typedef struct calibatt_fwd_options {
  const calibatt_strides *in_strides;
  const calibatt_strides *out_strides;
  int32_t dtype;
  float *lse;
  int32_t kernel;
} calibatt_fwd_options;
int calibatt_sparse_attn_fwd_ex(const void *q, const void *k, const void *v, void *out, int B, int H,
                                int N, int D, int block_q, int block_k,
                                const calibatt_pattern *pattern, float scale,
                                const calibatt_fwd_options *options, void *stream);

/*
 * Spatial-row anchor scheme (Section 3.3; "Inference stage" of Section 3.4:
 * heads flagged as spatially repetitive run dense attention on a reduced query
 * set and broadcast the result).
 *
 * Geometry: the first F*Hs*Ws tokens of a head are a video latent, token
 * (frame f, spatial row y, column x) at index (f*Hs + y)*Ws + x; the remaining
 * N - F*Hs*Ws tokens (text tokens of joint-attention models) have no position.
 * Per frame, k anchor rows a_j = floor((2j+1)*Hs / (2k)), j = 0..k-1 (the rows
 * under the centres of k equal segments).  Row y takes the result of the
 * anchor nearest to it, the lower one on a tie.  Tokens without a position are
 * computed themselves.
 *
 * calibatt_anchor_map writes, into caller-provided HOST buffers,
 *   q_index [n_q]      token whose query is the i-th computed one: frames
 *                      ascending, then anchors ascending, then columns; then
 *                      the tokens without a position
 *   dst_ptr [n_q + 1]  exclusive prefix sum of the receiver counts
 *   dst_idx [N]        receivers of computed query i: dst_idx[dst_ptr[i] ..
 *                      dst_ptr[i+1]), ascending; every token is listed once
 *   *n_q               F*k*Ws + (N - F*Hs*Ws)
 * Any of the three arrays may be NULL (then none is written): use that to
 * learn n_q.  Errors: NULL (n_q), SHAPE (a non-positive dimension, F*Hs*Ws > N,
 * k > Hs).
 */
int calibatt_anchor_map(int N, int F, int Hs, int Ws, int k, int32_t *q_index, int32_t *dst_ptr,
                        int32_t *dst_idx, int32_t *n_q);

/*
 * Dense attention on a reduced query set with broadcast of the results
 * (Section 3.3; Section 2, Eq. 1-4 for the attention itself).
 *
 * q, k, v  DEVICE, bf16, contiguous [B][H][N][D]; read only.
 * out      DEVICE, bf16, contiguous [B][H][N][D]; must not alias the inputs.
 *          Only the heads listed in head_ids are touched.  In those, for every
 *          i < n_q, softmax(scale * q[q_index[i]] K^T) V over all N keys (fp32
 *          accumulation, rounded to bf16) is written to each row
 *          dst_idx[dst_ptr[i] .. dst_ptr[i+1]); all receivers of one i hold
 *          the same bits.  Rows that no list names keep their contents.
 * head_ids DEVICE int32 [n_heads]: the heads to process, each in [0, H); an
 *          entry outside that range is skipped.  The other heads of `out` are
 *          left to calibatt_sparse_attn_fwd (give these heads an empty mask
 *          there and enqueue this call after it on the same stream, or run the
 *          two on disjoint tensors).
 * q_index, dst_ptr, dst_idx  DEVICE copies of what calibatt_anchor_map wrote,
 *          or any other lists of that form (q_index entries are clamped to
 *          [0, N), dst_idx entries outside [0, N) are skipped; dst_ptr must be
 *          non-decreasing with dst_ptr[0] >= 0 and is not checked).  The same
 *          lists serve every listed head and every batch index.
 * stream   hipStream_t (NULL = default stream).  The call only enqueues work.
 *
 * Supported: D in {64, 128}.  n_heads == 0 or n_q == 0 is a no-op.
 * Errors: NULL, SHAPE (non-positive B/H/N/D, negative n_heads or n_q, out
 * aliasing an input), UNSUPPORTED (D), LAUNCH.
 */
int calibatt_anchor_attn_fwd(const void *q, const void *k, const void *v, void *out, int B, int H,
                             int N, int D, const int32_t *head_ids, int n_heads,
                             const int32_t *q_index, const int32_t *dst_ptr, const int32_t *dst_idx,
                             int n_q, float scale, void *stream);

/* The same on strided tensors; strides, requirements and errors as in
 * calibatt_sparse_attn_fwd_strided. */
int calibatt_anchor_attn_fwd_strided(const void *q, const void *k, const void *v, void *out, int B,
                                     int H, int N, int D, const int32_t *head_ids, int n_heads,
                                     const int32_t *q_index, const int32_t *dst_ptr,
                                     const int32_t *dst_idx, int n_q, float scale,
                                     const calibatt_strides *in_strides,
                                     const calibatt_strides *out_strides, void *stream);

/*
 * The anchor forward with the tail of its work evened out (Section 3.3 / 3.4,
 * anchor benchmark of the supplement: few anchors mean few computed queries).
 * Every unit of work (128 computed queries of one head against all keys) takes
 * the same time, so the units run in rounds of as many as the GPU holds at a
 * time and the last round may be mostly empty.  This call cuts the units of
 * that last round into n_split parts of the keys each, runs the parts side by
 * side, and merges them: with lse_s the log-sum-exp of the scaled logits of
 * part s and A_s its softmax-weighted values, the result is
 * sum_s e^(lse_s - m) A_s / sum_s e^(lse_s - m), m = max_s lse_s, which is the
 * softmax over all keys of Eq. 1-2.  Same outputs as
 * calibatt_anchor_attn_fwd_strided up to fp32 rounding of the merge (compare
 * with the tolerance of the forward, not bitwise); receivers of one computed
 * query still hold the same bits.
 *
 * calibatt_anchor_split_plan (needs a current HIP device; no GPU work): for the
 * shape (B, N, D, n_heads, n_q) writes n_split in [1, 8] (1 = splitting gains
 * nothing: the forward then ignores the workspace) and the bytes of workspace
 * the forward needs on this device (0 for n_split 1).  Errors: NULL, SHAPE,
 * UNSUPPORTED, LAUNCH.
 *
 * calibatt_anchor_attn_fwd_split: arguments as calibatt_anchor_attn_fwd_strided,
 * plus
 * workspace        DEVICE, 16-byte aligned, workspace_bytes long, owned by the
 *                  caller, contents irrelevant before and undefined after; it
 *                  is written and read by the call's kernels only, so one
 *                  buffer may serve successive calls on one stream, never
 *                  calls that may overlap.  NULL: every unit is computed whole
 *                  (the plain call).
 * workspace_bytes  at least what calibatt_anchor_split_plan returns for the
 *                  shape, else BUFFER_TOO_SMALL.
 */
int calibatt_anchor_split_plan(int B, int N, int D, int n_heads, int n_q, int32_t *n_split,
                               int64_t *workspace_bytes);
int calibatt_anchor_attn_fwd_split(const void *q, const void *k, const void *v, void *out, int B, int H,
                                   int N, int D, const int32_t *head_ids, int n_heads,
                                   const int32_t *q_index, const int32_t *dst_ptr,
                                   const int32_t *dst_idx, int n_q, float scale,
                                   const calibatt_strides *in_strides,
                                   const calibatt_strides *out_strides, void *workspace,
                                   int64_t workspace_bytes, void *stream);

/*
 * Detection of spatially repetitive heads (Section 3.3): the spatial
 * similarity score of a head is the cosine similarity between the attention
 * rows of a spatial row of tokens and those of its nearest anchor row (same
 * frame; both flattened over column and key), averaged over frames and spatial
 * rows - every row counts, anchors included (their similarity is 1).  A head
 * is flagged when the score, averaged over calibration prompts by the caller,
 * exceeds the threshold gamma (0.87 in the paper, with k = 5).
 *
 * calibatt_anchor_partner (host): partner[t] = the token of t's nearest anchor
 * row at the same frame and column, for the F*Hs*Ws video tokens (anchor
 * positions and ties as in calibatt_anchor_map).  Errors: NULL, SHAPE.
 *
 * calibatt_spatial_similarity: score[b][h] for every head, the N x N attention
 * map never stored.
 *   q, k       DEVICE, bf16, contiguous [B][H][N][D]; read only.
 *   partner    DEVICE int32 [n_tok]: token compared with token t (clamped to
 *              [0, N)); tokens t < n_tok are the ones that have a spatial
 *              position, in rows of row_len consecutive tokens.
 *   workspace  DEVICE fp32 [B][H][n_tok][3]: per token the three sums of
 *              products of probabilities (with the partner, with itself, the
 *              partner with itself); overwritten.
 *   score      DEVICE fp32 [B][H].  Same bits on every run.
 *   stream     hipStream_t (NULL = default stream).  The call only enqueues work.
 * Supported: D in {64, 128}.  Errors: NULL, SHAPE (a non-positive dimension,
 * n_tok > N, n_tok not a multiple of row_len), UNSUPPORTED, LAUNCH.
 */
int calibatt_anchor_partner(int F, int Hs, int Ws, int k, int32_t *partner);
int calibatt_spatial_similarity(const void *q, const void *k, int B, int H, int N, int D,
                                const int32_t *partner, int n_tok, int row_len, float scale,
                                float *workspace, float *score, void *stream);

/*
 * calibatt_spatial_similarity for callers that cannot allocate device memory
 * or hand a workspace over (code under HIP graph capture, serving loops that
 * forbid hipMalloc): the per-token sums live in a buffer inside the library,
 * CALIBATT_SIMILARITY_STATIC_MAX_BYTES of device memory per GPU that the
 * library runs on, held until the process ends.  The call allocates nothing.
 * Arguments and result as calibatt_spatial_similarity without `workspace`.
 * The buffer keeps the last call's contents (the kernels overwrite every entry
 * they read, nothing has to be cleared), and every call on a GPU shares it:
 * calls on one GPU that may overlap (different streams, different host
 * threads) race on it - serialise them, or use the workspace form.
 * Errors: as calibatt_spatial_similarity; BUFFER_TOO_SMALL when
 * B * H * n_tok * 12 bytes exceed the buffer (16 MiB: 40 heads of 34 952
 * tokens).
 */
#define CALIBATT_SIMILARITY_STATIC_MAX_BYTES (16 * 1024 * 1024)
int calibatt_spatial_similarity_static(const void *q, const void *k, int B, int H, int N, int D,
                                       const int32_t *partner, int n_tok, int row_len, float scale,
                                       float *score, void *stream);

/*
 * Calibration steps that turn attention maps into a block mask (Section 3.2).
 * They run offline, once per (timestep, layer, head) and calibration prompt;
 * the energy kernel is the one part that touches N x N work.
 *
 * calibatt_block_energy (Eq. 5): energy[b][h][r][c] = the softmax mass
 * (Section 2, Eq. 1, logits scale * q k^T over all N keys) that the queries of
 * block r put on the keys of block c, averaged over the queries of the block
 * (a short last block averages over the rows it has, so every block-row sums
 * to 1).  The N x N map is never stored.
 *   q, k    DEVICE, bf16, contiguous [B][H][N][D]; read only.
 *   energy  DEVICE, fp32, contiguous [B][H][ceil(N/block_q)][ceil(N/block_k)];
 *           every entry is written.  Same bits on every run.
 *   stream  hipStream_t (NULL = default stream).  The call only enqueues work.
 * Supported: D in {64, 128}, block_q and block_k in {64, 128}, and
 * ceil(N/block_k) small enough for the per-workgroup partial sums to fit in
 * LDS next to two K tiles (N up to 262144 at least).
 * Errors: NULL, SHAPE, UNSUPPORTED, LAUNCH.
 */
int calibatt_block_energy(const void *q, const void *k, float *energy, int B, int H, int N, int D,
                          int block_q, int block_k, float scale, void *stream);

/*
 * The same energies (Eq. 5) in one pass over the keys instead of two, for
 * callers that bring a workspace: while a row's softmax statistics are still
 * running, the logarithm of the mass it puts on each key block is parked in
 * the workspace (it needs no reference maximum), and turned into the block's
 * share once the row's log-sum-exp is known.  Half the matrix work; results
 * agree with calibatt_block_energy within the energies' tolerance (not bit for
 * bit), same bits on every run.
 *   workspace        DEVICE, 4-byte aligned, owned by the caller, contents
 *                    irrelevant before and undefined after; used by this call's
 *                    kernel only (successive calls on one stream may share it,
 *                    calls that may overlap may not).
 *   workspace_bytes  any size from one slice (ceil(N/block_k) * block_q * 4
 *                    bytes) up: the kernel runs as many workgroups as there
 *                    are slices, the GPU holds at a time, and there are query
 *                    blocks.  calibatt_block_energy_workspace_bytes (host, no
 *                    GPU needed) returns 1024 slices, enough for every
 *                    supported shape on a 256-CU part.
 * Other arguments, supported shapes and errors as calibatt_block_energy, plus
 * BUFFER_TOO_SMALL (less than one slice).
 */
int calibatt_block_energy_workspace_bytes(int N, int block_q, int block_k, int64_t *bytes);
int calibatt_block_energy_onepass(const void *q, const void *k, float *energy, int B, int H, int N, int D,
                                  int block_q, int block_k, float scale, void *workspace,
                                  int64_t workspace_bytes, void *stream);

/*
 * calibatt_select_blocks (Eq. 6): for each of n_rows block-rows of nbk
 * energies, keep the smallest set of blocks whose energies sum to at least
 * eps: sort descending (equal energies: lower column first), take the shortest
 * prefix whose running sum, accumulated in double in that order, reaches eps;
 * a row whose total stays below eps keeps every block.
 *   energy  HOST, fp32 [n_rows][nbk]       mask  HOST, uint8 [n_rows][nbk], 1 = kept
 * Errors: NULL, SHAPE (n_rows < 0, nbk <= 0, eps not a number), NOMEM.
 */
int calibatt_select_blocks(const float *energy, int64_t n_rows, int nbk, double eps, uint8_t *mask);

/*
 * calibatt_vote_masks (Eq. 8-9): masks of n_prompts calibration prompts, each
 * n entries (any non-zero byte = kept) -> out[i] = 1 where count_i / n_prompts
 * >= rho (compared in double), else 0.  HOST buffers; out may alias masks[0..n).
 * Errors: NULL, SHAPE (n_prompts <= 0, n < 0, rho not a number).
 */
int calibatt_vote_masks(const uint8_t *masks, int n_prompts, int64_t n, double rho, uint8_t *out);

/*
 * The same vote without keeping every prompt's mask: calibatt_vote_accumulate
 * adds one prompt's mask (n entries, non-zero = kept) to per-block counters
 * (uint16, zeroed by the caller before the first prompt; at most 65535
 * prompts), calibatt_vote_finish thresholds them exactly like
 * calibatt_vote_masks: out[i] = counts[i] / n_prompts >= rho.  HOST buffers.
 * Errors: NULL, SHAPE (n < 0, n_prompts outside [1, 65535], rho not a number, a
 * counter that would overflow or exceeds n_prompts).
 */
int calibatt_vote_accumulate(const uint8_t *mask, int64_t n, uint16_t *counts);
int calibatt_vote_finish(const uint16_t *counts, int n_prompts, int64_t n, double rho, uint8_t *out);

/*
 * The two per-prompt steps on the GPU, so that a calibration step (block
 * energy, Eq. 6, one more vote for Eq. 8-9) never leaves it; only the counters
 * come back, once, for calibatt_vote_finish.
 *
 * calibatt_select_blocks_device: Eq. 6 exactly as calibatt_select_blocks defines
 * it (same order, same fp64 running sum in that order), bit for bit the same
 * mask; energies must not be NaN (the order is then unspecified; nothing
 * faults).
 *   energy  DEVICE, fp32 [n_rows][nbk], 4-byte aligned, e.g. the output of
 *           calibatt_block_energy        mask  DEVICE, uint8 [n_rows][nbk]
 * Supported: nbk <= 4096.  Errors: NULL, SHAPE, UNSUPPORTED, LAUNCH.
 *
 * calibatt_vote_accumulate_device: counts[i] += (mask[i] != 0) on DEVICE
 * buffers (counts 2-byte aligned, zeroed by the caller before the first
 * prompt).  A counter at 65535 stays there (the host routine refuses instead).
 * Errors: NULL, SHAPE, LAUNCH.
 *
 * Both only enqueue work on `stream` (hipStream_t, NULL = default stream).
 */
int calibatt_select_blocks_device(const float *energy, int64_t n_rows, int nbk, double eps, uint8_t *mask,
                                  void *stream);
int calibatt_vote_accumulate_device(const uint8_t *mask, int64_t n, uint16_t *counts, void *stream);

/*
 * Energy threshold of diffusion step t of T (Eq. 7): A + (C - A) exp(-k t / T),
 * t = 0 the highest-noise step.  Returns NaN when T <= 0.
 * calibatt_schedule_base_level: the base level A the paper uses in the
 * many-step regime for sequence length N, 0.796 + 1.41e-6 N (with C = 0.99,
 * k = 16; supplement, "Hyperparameter search for energy threshold schedule").
 */
double calibatt_epsilon_schedule(int t, int T, double A, double C, double k);
double calibatt_schedule_base_level(int N);

/*
 * The parameters (A, C, k) of Eq. 7 the paper settles on (supplement,
 * "Hyperparameter search for energy threshold schedule"), written to *A, *C,
 * *k.  CALIBATT_REGIME_MANY_STEP: the 50-step models, A =
 * calibatt_schedule_base_level(N), C = 0.99, k = 16.  CALIBATT_REGIME_DISTILLED:
 * the few-step (distilled) models, one schedule for every resolution,
 * A = 0.763, C = 0.863, k = 5.64.  Errors: NULL, SHAPE (N <= 0), UNSUPPORTED
 * (regime).
 */
enum { CALIBATT_REGIME_MANY_STEP = 0, CALIBATT_REGIME_DISTILLED = 1 };
int calibatt_schedule_constants(int regime, int N, double *A, double *C, double *k);

/*
 * Which heads are spatially repetitive (Section 3.3): scores (HOST, fp32
 * [n_prompts][H]) holds the spatial similarity score of every head on every
 * calibration prompt; the scores of a head are averaged over the prompts (in
 * double, prompts in order) and flags[h] (HOST, uint8 [H]) is 1 when the
 * average EXCEEDS gamma (0.87 in the paper), else 0.  mean (HOST, double [H])
 * receives the averages when not NULL.  Errors: NULL, SHAPE (n_prompts <= 0,
 * H <= 0, gamma NaN).
 */
int calibatt_flag_heads(const float *scores, int n_prompts, int H, double gamma, uint8_t *flags, double *mean);

/*
 * Skip-list tools of the supplement (Section A.2 "Skip-List Memory
 * Optimization", Section A.3 "Timestep Mask Sharing").  All HOST buffers.
 *
 * calibatt_encode_intervals: the flat ("1D") interval layout of the kept-block
 * lists of a compiled pattern - every row as its maximal runs of consecutive
 * key blocks.  One 32-bit word per interval: low 16 bits = first key block of
 * the run, high 16 bits = number of kept blocks of the row before the run; each
 * row ends with one more word carrying (0, kept blocks of the row), so a row of
 * n runs takes n + 1 words and a run's length is the difference of two
 * neighbouring high halves.  Needs nbk <= 65535.
 *   row_ptr [n_rows + 1], col_idx: as written by calibatt_compile_pattern
 *   iv_ptr  [n_rows + 1]  offsets into iv          iv [iv_cap]  words
 *   n_words               number of words needed (always written when non-NULL)
 * iv_ptr or iv may be NULL to learn n_words only.
 * Errors: NULL, SHAPE (n_rows < 0, a column >= 65536, a row longer than 65535,
 * columns of a row not strictly ascending), BUFFER_TOO_SMALL (iv_cap < n_words).
 */
int calibatt_encode_intervals(const int32_t *row_ptr, const int32_t *col_idx, int64_t n_rows,
                              int32_t *iv_ptr, uint32_t *iv, int64_t iv_cap, int64_t *n_words);

/*
 * calibatt_merge_intervals: interval merging by percentile.  width = the
 * nearest-rank pct-th percentile of the interval counts of the n_rows rows
 * (the smallest count w such that at least pct percent of the rows have <= w
 * intervals; at least 1).  Rows with more intervals get their smallest gaps
 * between neighbouring intervals filled with kept blocks (the leftmost among
 * equal gaps first) until they have `width` intervals; other rows are copied.
 *   mask [n_rows][nbk] uint8, non-zero = kept     out [n_rows][nbk], 0 / 1;
 *   may alias mask.                                width: may be NULL.
 * Errors: NULL, SHAPE (n_rows < 0, nbk <= 0, pct outside (0, 100]), NOMEM.
 */
int calibatt_merge_intervals(const uint8_t *mask, int64_t n_rows, int nbk, double pct, uint8_t *out,
                             int32_t *width);

/*
 * calibatt_share_timesteps: masks[T][n] of one (layer, head), one per diffusion
 * step.  Steps are visited in ascending order; a step joins the first cluster
 * (in order of creation) in which the IoU of its skipped-block set with that of
 * every member is >= tau (two masks that skip nothing: IoU 1), else it founds
 * a new cluster.  cluster[t] receives the cluster of step t, shared[c][n] the
 * OR of the kept blocks of the members of cluster c (first *n_clusters rows
 * written; the buffer holds T rows), 0 / 1.
 * Errors: NULL, SHAPE (T <= 0, n < 0, tau not a number), NOMEM.
 */
int calibatt_share_timesteps(const uint8_t *masks, int T, int64_t n, double tau, int32_t *cluster,
                             uint8_t *shared, int32_t *n_clusters);

/* Static, NUL-terminated description of a status code. */
const char *calibatt_strerror(int status);

/* Library version: major*10000 + minor*100 + patch. */
int calibatt_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CALIBATT_H */
