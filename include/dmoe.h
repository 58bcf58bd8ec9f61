/*
 * dmoe.h -- C ABI of the MI355X (gfx950) dropless-MoE expert layer.
 *
 * The layer is the dMoE of "MegaBlocks: Efficient Sparse Training with Mixture-of-Experts" (arXiv 2211.15841),
 * Figure 6:   router -> make_topology -> padded_gather -> sdd -> dsd -> padded_scatter -> scale,
 * with the backward products of Section 5.1 (SDD^T, DS^TD, DSD^T, DD^TS).
 *
 * Problem statement (Figure 6, Section 2.1):
 *   x        [T, d]      tokens, row-major bf16                      T = num_tokens, d = d_model (hidden_size)
 *   w_router [d, E]      router projection, row-major bf16           E = num_experts
 *   w1       [d, E*h]    first expert layer, row-major bf16          h = ffn_hidden; expert e owns columns [e*h,(e+1)*h)
 *   w2       [E*h, d]    second expert layer, row-major bf16         expert e owns rows [e*h,(e+1)*h)
 *   y        [T, d]      layer output, row-major bf16
 * All matrix products accumulate in fp32.  "bf16" means the upper 16 bits of an IEEE binary32.
 *
 * Conventions
 *   - Every pointer named below is a DEVICE pointer into caller-owned memory unless it says "host".
 *     The library allocates no device memory, frees none, and keeps no device state between calls.
 *   - Every device buffer must be 256-byte aligned.  Outputs are overwritten (never accumulated into), except
 *     the three accumulators of dmoe_backward_accumulate.
 *   - dmoe_topology / dmoe_forward / dmoe_backward only enqueue work on `stream` (a hipStream_t passed as
 *     void*; NULL = the null stream).  They never synchronise and never copy to the host: the padded row
 *     count P and the number of nonzero blocks live in device memory (dmoe_topology_t.counts) and the
 *     kernels read them there, so buffers are sized for the upper bounds reported by dmoe_sizes().
 *   - Return value: DMOE_OK (0) or a negative error code; dmoe_last_error() gives a message.  Arguments are
 *     validated on the host before anything is launched; on error nothing has been enqueued.
 *   - Inputs holding NaN or infinity give undefined routing.
 */
#ifndef DMOE_H_
#define DMOE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
#define DMOE_API __attribute__((visibility("default")))
#else
#define DMOE_API
#endif

#define DMOE_OK        0
#define DMOE_EINVAL   (-1)   /* null pointer, misaligned pointer, or a configuration outside the supported set */
#define DMOE_ENOMEM   (-2)   /* a caller-provided buffer is smaller than dmoe_sizes() asks for                  */
#define DMOE_ELAUNCH  (-3)   /* the HIP runtime reported an error while enqueueing                              */

#define DMOE_BLOCK 128       /* side of a sparse block (Section 5.1.2: 128x128 blocks)                          */

/* Layer hyper-parameters.  Supported: block == 128; d_model and ffn_hidden multiples of 128;
 * 1 <= top_k <= min(num_experts, 8); 1 <= num_experts <= 256; num_tokens >= 1; num_tokens*top_k < 2^24. */
typedef struct {
  int32_t num_tokens;      /* T */
  int32_t d_model;         /* d  (hidden_size)     */
  int32_t ffn_hidden;      /* h  (ffn_hidden_size) */
  int32_t num_experts;     /* E */
  int32_t top_k;           /* k  experts per token (Section 2.1) */
  int32_t block;           /* must be 128 */
  int32_t activation;      /* between the two expert layers: 0 exact GELU v*Phi(v); 1 its tanh form
                              0.5 v (1 + tanh(sqrt(2/pi) (v + 0.044715 v^3))) */
  int32_t normalize_topk;  /* 0: confidence = softmax probability of the chosen expert (Section 2.1);
                              1: that, divided by the sum over the token's k chosen experts */
  int32_t expert_capacity; /* 0: dropless (the dMoE of Section 4: every assignment is computed).  > 0: the
                              token-dropping MoE of Section 2.2 on the same kernels: an expert keeps the first
                              expert_capacity assignments routed to it, in ascending flat index f; the others are
                              dropped (row_of[f] = -1, no contribution to y, no gradient through them).  The caller
                              computes it, e.g. as num_tokens*top_k/num_experts * capacity_factor (Section 2.2) */
  int32_t pad_to_capacity; /* with expert_capacity > 0 only.  0: a group is padded to the next multiple of 128 rows
                              as in the dropless layer; 1: every expert owns ceil(expert_capacity/128)*128 rows,
                              unused capacity being zero rows (the fixed shape of Section 2.2 and Figure 2)  */
} dmoe_config;

/* Routing result + block-sparse topology, all in device memory (views into one caller-owned allocation,
 * laid out by dmoe_topology_bind).  f = t*top_k + s is the flat index of token t's s-th choice.
 * Index arrays are block-wise int32 (Figure 5).  With R = P/128 block-rows, hb = h/128, nnz = R*hb:           */
typedef struct {
  int32_t *expert_idx;         /* [T*k]     chosen expert of f; slots in descending score, ties -> lower expert */
  float   *weights;            /* [T*k]     confidence of f (fp32)                                               */
  float   *logits;             /* [T*E]     router scores (fp32, bias included), kept for the backward pass      */
  int32_t *tokens_per_expert;  /* [E]       n_e                                                                  */
  int32_t *padded_offsets;     /* [E+1]     first padded row of each expert; rows per expert = ceil(n_e/128)*128 */
  int32_t *row_of;             /* [T*k]     padded row holding f (stable: ascending f inside an expert)          */
  int32_t *token_of;           /* [P_max]   f held by a padded row, -1 on padding rows (valid for rows < P)      */
  int32_t *row_offsets;        /* [R_max+1] blocked CSR: first block of each block-row            (Sec. 5.1.3)   */
  int32_t *column_indices;     /* [nnz_max] blocked CSR: block-column of each block, row-wise order              */
  int32_t *row_indices;        /* [nnz_max] block-row of each block (the COO half of the hybrid encoding)        */
  int32_t *column_offsets_t;   /* [E*hb+1]  transposed matrix: first entry of each block-column   (Sec. 5.1.4)   */
  int32_t *row_indices_t;      /* [nnz_max] transposed order: block-row of each entry, ascending in a column     */
  int32_t *block_offsets_t;    /* [nnz_max] transposed order: number of that block in the primary order          */
  int32_t *counts;             /* [4]       P, R, nnz, 0                                                         */
  /* Scheduling aids of this implementation (not part of the paper's encoding):                                  */
  int32_t *expert_order;       /* [E]       experts by descending n_e (ties -> lower expert); the weight-gradient
                                            products visit the heaviest experts first                            */
  int32_t *group_offsets;      /* [E+1]     block-rows of an expert are taken two at a time ("row groups");
                                            first group of each expert, group_offsets[E] = number of groups      */
  int32_t *row_group;          /* [G_max]   2*(first block-row of the group) + (1 if the group has a second row) */
  int32_t *sched;              /* [4]       sched[0] = 1 if the weight-gradient products should use 128x128 tiles
                                            (one expert holds so many rows that its 256x256 tiles alone would
                                            outlast a balanced schedule), else 0; sched[1] = tiles per XCD patch
                                            for those products (16 when no expert is large against an XCD's
                                            share of the rows, else 1); sched[2] = 1 if DSD / DSD^T, when launched
                                            in both tile shapes, should take the single 128x128 blocks (their
                                            rounds of 512 come to less time than the macro tiles' rounds of 256);
                                            sched[3] reserved                                                    */
} dmoe_topology_t;

/* Buffer sizes in bytes for `cfg` (host pointers; any may be NULL).  P_max = upper bound on padded rows,
 * nnz_max = (P_max/128)*(h/128).  topology: the arrays of dmoe_topology_t; saved: what forward keeps for
 * backward (permuted tokens, the sparse activation and the activation's derivative, permuted expert output); scratch: the larger of what
 * the three calls need (contents are dead after each call returns... after its work completes).             */
DMOE_API int dmoe_sizes(const dmoe_config *cfg, size_t *topology_bytes, size_t *saved_bytes, size_t *scratch_bytes,
               int32_t *P_max, int32_t *nnz_max);

/* Carve `topology_mem` (device, `bytes` >= topology_bytes) into the arrays of *out (host struct).  No GPU work. */
DMOE_API int dmoe_topology_bind(const dmoe_config *cfg, void *topology_mem, size_t bytes, dmoe_topology_t *out);

/* Steps (1)-(2) of Figure 6: route every token (Section 2.1), group the assignments by expert with each
 * group padded to a multiple of 128 rows (Section 5.2), and build the blocked-CSR-COO topology with its
 * transpose indices (Sections 5.1.3, 5.1.4).  router_bias: fp32 [E] added to the scores, or NULL.
 * Router scores are accumulated in fp32 in ascending hidden index, so expert_idx is reproducible bit for bit. */
DMOE_API int dmoe_topology(const dmoe_config *cfg, const void *x, const void *w_router, const float *router_bias,
                  dmoe_topology_t *topo, void *scratch, size_t scratch_bytes, void *stream);

/* dmoe_topology for callers that cannot allocate device memory or carry a workspace around: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs, same results in *topo (bit for bit),
 * but the scratch of the call (the per-chunk expert counts, ceil(T*k/256)*E int32) lives in a 1 MiB device array
 * built into the library instead of a caller buffer; each GPU the library runs on holds that array until the process
 * ends.  The call allocates and frees nothing.  The device that `stream` belongs to must be the current device.
 * Limit: ceil(T*k/256) * E * 4 <= 1 048 576 bytes, else DMOE_ENOMEM and nothing is enqueued.  All calls on one GPU
 * share the one array: calls that overlap in time on the same GPU (different streams, different threads) race; calls
 * on one stream are ordered and safe (every call rewrites the part of the array it reads).  Other errors as
 * dmoe_topology, plus DMOE_ELAUNCH if the array's device address cannot be obtained.                            */
DMOE_API int dmoe_topology_static(const dmoe_config *cfg, const void *x, const void *w_router,
                                  const float *router_bias, dmoe_topology_t *topo, void *stream);

/* Steps (3)-(5) of Figure 6: padded gather, SDD (+GELU), DSD, padded scatter scaled by the confidences and
 * summed over the k slots (Section 2.4).  Writes y [T,d] bf16 and `saved` (>= saved_bytes).                    */
DMOE_API int dmoe_forward(const dmoe_config *cfg, const void *x, const void *w1, const void *w2,
                 const dmoe_topology_t *topo, void *y, void *saved, size_t saved_bytes,
                 void *scratch, size_t scratch_bytes, void *stream);

/* Backward of the layer for upstream gradient dy [T,d] bf16 (Section 5.1: SDD^T and DS^TD for the second
 * layer, DSD^T and DD^TS for the first), plus the router's gradient with the assignments held constant.
 * Writes dx [T,d] bf16, dw_router [d,E] fp32, dw1 [d,E*h] bf16, dw2 [E*h,d] bf16; the slices of dw1/dw2 that
 * belong to experts with no tokens are written as zeros.                                                      */
DMOE_API int dmoe_backward(const dmoe_config *cfg, const void *x, const void *w_router, const void *w1, const void *w2,
                  const dmoe_topology_t *topo, const void *saved, size_t saved_bytes, const void *dy,
                  void *dx, void *dw_router, void *dw1, void *dw2,
                  void *scratch, size_t scratch_bytes, void *stream);

/* The same backward pass for training with gradient accumulation over micro-batches (Section 6.2 trains every
 * model that way): the three weight gradients are ADDED, in fp32, to caller-owned fp32 accumulators
 * dw_router_acc [d,E], dw1_acc [d,E*h] and dw2_acc [E*h,d] (the products' fp32 sums are added without being
 * rounded to bf16 first; the caller zeroes the accumulators before the first micro-batch).  dx is written as in
 * dmoe_backward.  Slices of experts with no tokens are left as they are.  Same errors as dmoe_backward.        */
DMOE_API int dmoe_backward_accumulate(const dmoe_config *cfg, const void *x, const void *w_router, const void *w1,
                             const void *w2, const dmoe_topology_t *topo, const void *saved, size_t saved_bytes,
                             const void *dy, void *dx, float *dw_router_acc, float *dw1_acc, float *dw2_acc,
                             void *scratch, size_t scratch_bytes, void *stream);

/* Test helper: waits for `stream` and copies counts[4] (P, R, nnz, 0) to host memory `out4`. */
DMOE_API int dmoe_topology_counts_host(const dmoe_topology_t *topo, int32_t *out4, void *stream);

/* Test helper: byte offset, inside the `scratch` buffer of `cfg`, of one of the intermediates that dmoe_backward leaves
 * there ("dyp": permuted, confidence-scaled upstream gradient [P_max,d] bf16; "dh": gradient of the hidden blocks;
 * "dxp": permuted input gradient [P_max,d] bf16; "dweights": [T*k] fp32; "dlogits": gradient of the router scores
 * [T,E] fp32; "partials"; "chunk_counts").  Host pointers; no GPU work.  Errors: DMOE_EINVAL (unknown name).       */
DMOE_API int dmoe_debug_scratch_offset(const dmoe_config *cfg, const char *region, size_t *offset);

/* Measurement aid: while `buffer` (device, 256-byte aligned, zero-filled by the caller) is non-NULL, the block-sparse
 * product of stage `stage` (DMOE_STAGE_SDD ... DMOE_STAGE_DDTS) launched by this thread's next calls records, per work
 * item w < bytes/40, five int64 at buffer[5w...]: the 100 MHz wall counter when the item starts, when its first
 * operands are in LDS, when its K loop ends, when its epilogue ends, and its number of K tiles (64 of K each).
 * Items are numbered as the launch numbers them (workgroup index plus multiples of the grid for persistent launches).
 * NULL switches it off.  Errors: DMOE_EINVAL.                                                                    */
DMOE_API int dmoe_debug_trace(void *buffer, size_t bytes, int stage);

/* Timing helper for benchmarks: when `events` (host array of 2*DMOE_NUM_STAGES hipEvent_t, created by the
 * caller) is non-NULL, the next calls on this thread record an event before and after each stage's kernels
 * on the stream they are launched on.  Pass NULL to switch it off.  Stage numbers are DMOE_STAGE_*.           */
#define DMOE_STAGE_ROUTER        0   /* scores, top-k, softmax                        (dmoe_topology) */
#define DMOE_STAGE_SORT          1   /* histogram, offsets, stable ranks              (dmoe_topology) */
#define DMOE_STAGE_TOPOLOGY      2   /* blocked-CSR-COO arrays and transpose indices  (dmoe_topology) */
#define DMOE_STAGE_GATHER        3   /* padded gather                                 (dmoe_forward)  */
#define DMOE_STAGE_SDD           4   /* H = Xp W1, A = gelu(H), G = gelu'(H)          (dmoe_forward)  */
#define DMOE_STAGE_DSD           5   /* Yp = A W2                                     (dmoe_forward)  */
#define DMOE_STAGE_SCATTER       6   /* weighted un-permute                           (dmoe_forward)  */
#define DMOE_STAGE_BWD_GATHER    7   /* dYp = w dY permuted, dweights                 (dmoe_backward) */
#define DMOE_STAGE_SDDT          8   /* dA = dYp W2^T, dH = dA G                      (dmoe_backward) */
#define DMOE_STAGE_DSTD          9   /* dW2 = A^T dYp                                 (dmoe_backward) */
#define DMOE_STAGE_DSDT         10   /* dXp = dH W1^T                                 (dmoe_backward) */
#define DMOE_STAGE_DDTS         11   /* dW1 = Xp^T dH                                 (dmoe_backward) */
#define DMOE_STAGE_ROUTER_BWD   12   /* dlogits, dW_r, un-permute of dXp + router term (dmoe_backward) */
#define DMOE_NUM_STAGES         13
DMOE_API int dmoe_set_stage_events(void *events);

/* Tile shape of the block-sparse products: 0 = chosen from the configuration (default), 1 = one 128x128 block per
 * workgroup, 2 = 256x256 macro tiles (2x2 blocks), 3 = 256x256 macro tiles whose token-row products run on two LDS
 * stages instead of the five-stage slab ring (kept so that the two loops can be measured against each other).
 * Process-wide; results are identical, only speed differs.  Meant for tests and tuning.                        */
DMOE_API int dmoe_set_tile_mode(int mode);

/* ---- General block-sparse products (Sections 4.2, 5.1) ---------------------------------------------------------
 * The six products of the layer (and the other six that Section 5.1.1 counts, which the layer does not need) are general primitives on a 128x128 block-sparse matrix S of block_rows x block_cols
 * blocks with ANY mask; the dMoE topology is the block-diagonal instance.  These entry points expose them for a
 * caller-supplied mask, without the fused dMoE epilogues, one 128x128 block per workgroup.  Values of S: block b of
 * the row-wise order (ascending row, ascending column inside a row) is a contiguous row-major 128x128 bf16 tile at
 * element offset b*16384.  M = 128*block_rows, N = 128*block_cols, D = `dense` (a positive multiple of 128); dense
 * matrices are row-major bf16, accumulation is fp32.  All data pointers are DEVICE pointers, 256-byte aligned,
 * caller-owned; nothing is allocated.
 *
 *   DMOE_OP_SDD   a = X [M,D]   b = W [D,N]   out = S    S = (X W)   sampled on the mask     (Figure 3A)
 *   DMOE_OP_DSD   a = S         b = W [N,D]   out [M,D]  = S W                                (Figure 3B)
 *   DMOE_OP_SDDT  a = X [M,D]   b = W [N,D]   out = S    S = (X W^T) sampled on the mask
 *   DMOE_OP_DSTD  a = S         b = X [M,D]   out [N,D]  = S^T X      (through the transpose indices, Section 5.1.4)
 *   DMOE_OP_DSDT  a = S         b = W [D,N]   out [M,D]  = S W^T
 *   DMOE_OP_DDTS  a = X [M,D]   b = S         out [D,N]  = X^T S      (through the transpose indices)
 *   DMOE_OP_DDS   a = X [D,M]   b = S         out [D,N]  = X S        (through the transpose indices; Section 5.1.1)
 *
 * The remaining combinations of transposed and non-transposed inputs (Section 5.1.1: every product with every
 * combination), named like the paper's superscripts with the T after the operand's letter:
 *   DMOE_OP_SDTD  a = X [D,M]   b = W [D,N]   out = S    S = (X^T W)   sampled on the mask
 *   DMOE_OP_SDTDT a = X [D,M]   b = W [N,D]   out = S    S = (X^T W^T) sampled on the mask
 *   DMOE_OP_DSTDT a = S         b = X [D,M]   out [N,D]  = S^T X^T     (through the transpose indices)
 *   DMOE_OP_DDST  a = X [D,N]   b = S         out [D,M]  = X S^T       (block rows of S walked in the primary order)
 *   DMOE_OP_DDTST a = X [N,D]   b = S         out [D,M]  = X^T S^T
 */
enum { DMOE_OP_SDD = 0, DMOE_OP_DSD = 1, DMOE_OP_SDDT = 2, DMOE_OP_DSTD = 3, DMOE_OP_DSDT = 4, DMOE_OP_DDTS = 5,
       DMOE_OP_DDS = 6, DMOE_OP_SDTD = 7, DMOE_OP_SDTDT = 8, DMOE_OP_DSTDT = 9, DMOE_OP_DDST = 10, DMOE_OP_DDTST = 11 };

/* Bytes of device memory that the topology of a mask with `nnz` nonzero blocks needs (host pointer out).
 * Errors: DMOE_EINVAL (dimensions < 1, 128*dimension >= 2^24, nnz out of range).                               */
DMOE_API int dmoe_bsmm_sizes(int block_rows, int block_cols, int nnz, size_t *topology_bytes);

/* Encode `mask` (HOST pointer, row-major [block_rows][block_cols] bytes, nonzero = block present) as row_offsets,
 * column_indices, row_indices and the transpose indices (Sections 5.1.3-5.1.4) and copy them into `topology_mem`
 * (device, `bytes` >= dmoe_bsmm_sizes).  Fills `out` (host struct; the arrays a mask does not have point at zeros) and
 * `nnz_out` (host, may be NULL).  A set-up call: the encoding runs on the host and the copy is synchronous.
 * Errors: DMOE_EINVAL, DMOE_ENOMEM (buffer too small), DMOE_ELAUNCH (copy failed).                              */
DMOE_API int dmoe_bsmm_topology(const uint8_t *mask, int block_rows, int block_cols, void *topology_mem, size_t bytes,
                                dmoe_topology_t *out, int32_t *nnz_out);

/* Enqueue one product (table above) on `stream`; asynchronous.  `topo` must come from dmoe_bsmm_topology with the same
 * block_rows and block_cols, and `nnz` is the number of nonzero blocks it reported: SDD and SDD^T launch one workgroup
 * per nonzero block and find its row through the per-block row indices (Section 5.1.3), so their cost follows nnz and
 * not block_rows * block_cols.  Rows of S without blocks give zero rows of the DSD / DSD^T output, columns without
 * blocks zero rows of the DS^TD output and zero columns of the DD^TS / DDS output.
 * Errors: DMOE_EINVAL (unknown op, NULL or misaligned pointer, dense not a multiple of 128), DMOE_ELAUNCH.       */
DMOE_API int dmoe_bsmm(int op, const dmoe_topology_t *topo, int block_rows, int block_cols, int nnz, int dense,
                       const void *a, const void *b, void *out, void *stream);

/* Measurement aid: runs a register-only loop of v_mfma_f32_32x32x16_bf16 (four waves per SIMD on 256 CUs, no memory
 * traffic) on `stream`, waits for it (this call SYNCHRONISES) and returns the rate in TFLOP/s: the matrix-pipe peak
 * this device delivers at the clock it sustains, to set beside the published 2.5 PFLOP/s.  `scratch4`: device, >= 4
 * bytes, 256-byte aligned (never written).  Errors: DMOE_EINVAL, DMOE_ELAUNCH.                                  */
DMOE_API int dmoe_probe_mfma_tflops(float *tflops, void *scratch4, void *stream);

/* Measurement aid: the rate the matrix pipes SUSTAIN.  Runs the same instruction shaped like a wave of the 256x256 tile
 * (4 x 2 fragments, eight accumulators, two waves per SIMD on 256 CUs, no memory traffic) on pseudo-random operands
 * whose mantissa bits change every iteration, launch after launch for about `seconds` (0 < seconds <= 5), and reports
 * the rate of the last five launches in TFLOP/s together with the shader clock observed inside the kernel (shader-clock
 * counter against the 100 MHz wall counter) in GHz.  The published peak assumes 2.4 GHz; under sustained matrix load
 * the device runs slower, and this is the ceiling the block-sparse products can be set against.  This call SYNCHRONISES.
 * `scratch64`: device, >= 64 bytes, 256-byte aligned (overwritten).  Errors: DMOE_EINVAL, DMOE_ELAUNCH.            */
DMOE_API int dmoe_probe_mfma_sustained(float *tflops, float *shader_ghz, float seconds, void *scratch64, void *stream);

/* Message for the last error returned on this thread (host pointer to static thread-local storage). */
DMOE_API const char *dmoe_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DMOE_H_ */
