/*
 * salad.h - C ABI of the MI355X (gfx950) library for the SALAD attention-layer forward:
 * block-sparse softmax attention in parallel with ReLU linear attention, combined through
 * static (per-layer, per-head) and dynamic (input-dependent) scaling.
 *
 * Conventions for every entry point
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are
 *     ordinary host memory read during the call only.  The library allocates no device memory
 *     and keeps no pointer after a call returns.
 *   - Work is enqueued on the given HIP stream (a hipStream_t passed as void*, NULL = the
 *     default stream); no entry point synchronises with the host.
 *   - All argument checks happen on the host before the first HIP call and return
 *     SALAD_EINVAL / SALAD_ENOTSUP / SALAD_ENOSPC without touching the GPU.  HIP failures are
 *     returned as SALAD_EHIP.  Nothing throws across this boundary.  salad_last_error() gives
 *     the text for the calling thread's last non-OK status.
 *   - Tensors are contiguous.  Q, K, V and the output are [B, H, N, d] with N = T*Hh*W tokens
 *     stored time-slowest: n = t*Hh*W + y*W + x (the default flattening of App. A.1.1).
 *   - block is 64 tokens; d is 64 or 128; H <= 64.
 */
#ifndef SALAD_H
#define SALAD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SALAD_OK = 0,
    SALAD_EINVAL = 1,  /* bad argument (null pointer, shape mismatch, out of range)            */
    SALAD_ENOTSUP = 2, /* well-formed request outside the supported envelope                   */
    SALAD_ENOSPC = 3,  /* a caller-provided buffer (col_idx, workspace) is too small           */
    SALAD_EHIP = 4     /* a HIP runtime call failed                                            */
} salad_status;

typedef enum { SALAD_F32 = 0, SALAD_BF16 = 1 } salad_dtype;

/* Token order of a head (App. A.1.1).  SPATIAL: the stored order, position p = n.
 * TEMPORAL: tokens regrouped by spatial location so that the frames of one location are
 * consecutive, p = (y*W + x)*T + t. */
typedef enum { SALAD_HEAD_SPATIAL = 0, SALAD_HEAD_TEMPORAL = 1 } salad_head_kind;

/* Feature map phi of the linear branch (Sec. 3, Linear Attention; Eq. (3) uses ReLU). */
typedef enum { SALAD_PHI_RELU = 0 } salad_feature_map;

/* Thread-local text describing the last non-OK status returned on this thread ("" if none). */
const char *salad_last_error(void);

/* ---- mask ---------------------------------------------------------------------------------- */

/* Kept KV blocks per query block for a sparsity ("proportion of computations reduced by sparse
 * attention", Sec. 5.1), counted in block pairs: clamp(floor((1-sparsity)*nb + 0.5), 1, nb).
 * Pure host arithmetic.  Returns 0 if nb < 1. */
int32_t salad_kept_from_sparsity(int32_t nb, double sparsity);

/* Number of col_idx entries salad_block_mask will write: sum_h nb*kept[h].  -1 on bad input. */
int64_t salad_block_mask_nnz(int32_t T, int32_t Hh, int32_t W, int32_t block, int32_t H,
                             const int32_t *kept_host);

/* Spatial-temporal sliding-window block mask (Sec. 3 "Sliding-window attention", App. A.1.1)
 * as CSR over 64-token blocks of each head's own token order.  Row h*nb + i lists, ascending,
 * the KV blocks query block i of head h keeps: kept[h] consecutive blocks centred on i (the
 * extra one on the left for even counts), shifted inward at both sequence ends so that every
 * row has exactly kept[h] entries.  The mask is static (it depends on no activation), so it is
 * built once per (grid, kept) and reused by every layer and timestep.
 *   T, Hh, W        latent grid, N = T*Hh*W, nb = ceil(N/block)
 *   kept_host       host [H], each in 1..nb
 *   row_ptr_dev     device int32 [H*nb + 1]  (written)
 *   col_idx_dev     device int32 [col_capacity] (first nnz entries written)
 * SALAD_ENOSPC if col_capacity < nnz. */
salad_status salad_block_mask(int32_t T, int32_t Hh, int32_t W, int32_t block, int32_t H,
                              const int32_t *kept_host,
                              int32_t *row_ptr_dev, int32_t *col_idx_dev, int64_t col_capacity,
                              void *hip_stream);

/* The same mask with the other plain reading of the window at the sequence ends (the paper gives no formula, Sec. 3
 * "Sliding-window attention", App. A.1.1): SALAD_WINDOW_SHIFTED is salad_block_mask above (every row has exactly
 * kept[h] entries); SALAD_WINDOW_TRUNCATED keeps the blocks of [i - kept[h]/2, i - kept[h]/2 + kept[h]) that exist, so
 * the first kept[h]/2 and the last kept[h] - 1 - kept[h]/2 rows of a head are shorter and
 * nnz = sum_h (nb*kept[h] - l(l+1)/2 - r(r+1)/2), l = kept[h]/2, r = kept[h] - 1 - l.  The layer call takes either CSR.
 * Arguments, ownership and errors as for salad_block_mask / salad_block_mask_nnz; an unknown window_mode is
 * SALAD_EINVAL (-1 from the nnz function). */
typedef enum { SALAD_WINDOW_SHIFTED = 0, SALAD_WINDOW_TRUNCATED = 1 } salad_window_mode;
int64_t salad_block_mask_nnz_mode(int32_t T, int32_t Hh, int32_t W, int32_t block, int32_t H,
                                  const int32_t *kept_host, int32_t window_mode);
salad_status salad_block_mask_mode(int32_t T, int32_t Hh, int32_t W, int32_t block, int32_t H,
                                   const int32_t *kept_host, int32_t window_mode,
                                   int32_t *row_ptr_dev, int32_t *col_idx_dev, int64_t col_capacity,
                                   void *hip_stream);

/* Visit lists of the large-tile attention kernel (bf16, d = 128) for a CSR: for every head and every tile of 4
 * consecutive query blocks the union of the 4 rows' kept KV blocks, each entry tagged with the rows that keep it.  Like
 * the mask they depend on no activation (App. A.1.1: the sliding-window mask is static), so they can be built once per
 * CSR and passed to every layer call as salad_fwd_params.tile_lists; without them the layer call rebuilds them in its
 * workspace each time (a few microseconds).  Works for any CSR with ascending unique block ids per row.
 *   salad_tile_lists_bytes   size of the buffer for H heads and nb = ceil(N/64) blocks; 0 if the shape is invalid or the
 *                            lists of this nb do not fit the kernel (nb > 6144: the layer call then uses another kernel
 *                            and ignores tile_lists)
 *   lists_dev                device, 256-byte aligned, >= salad_tile_lists_bytes (written); SALAD_ENOSPC if smaller */
size_t salad_tile_lists_bytes(int32_t H, int32_t nb);
salad_status salad_tile_lists(const int32_t *row_ptr_dev, const int32_t *col_idx_dev, int32_t H, int32_t nb,
                              void *lists_dev, size_t lists_bytes, void *hip_stream);

/* W_p of the full Level-1 projection (Alg. 1 "Proj"; see salad_fwd_params.w_proj) rearranged once into the order the
 * projection GEMM reads it in (MFMA operand fragments of its [H x H] blocks of d x d).  The weights are static per layer,
 * so this runs once per layer, not per call; pass the result as salad_fwd_params.w_proj_packed.
 *   salad_proj_pack_bytes   size of the packed buffer (2 (H d)^2 bytes); 0 unless 1 <= H <= 64 and d == 128
 *   w_proj_dev              device bf16 [H*d, H*d], row-major (read)
 *   packed_dev              device, 256-byte aligned, >= salad_proj_pack_bytes (written); SALAD_ENOSPC if smaller */
size_t salad_proj_pack_bytes(int32_t H, int32_t d);
salad_status salad_proj_pack(const void *w_proj_dev, int32_t H, int32_t d, void *packed_dev, size_t packed_bytes,
                             void *hip_stream);

/* ---- whole layer --------------------------------------------------------------------------- */

typedef struct salad_fwd_params {
    int32_t B, H, N, d;
    int32_t dtype;            /* salad_dtype of q, k, v, out and x_t                              */
    int32_t T, Hh, W, block;  /* latent grid (N == T*Hh*W) and block size (64)                    */
    const void *q, *k, *v;    /* device [B,H,N,d]                                                 */
    void *out;                /* device [B,H,N,d]; must not alias an input                        */
    const int32_t *row_ptr;   /* device CSR from salad_block_mask, or any CSR with ascending      */
    const int32_t *col_idx;   /*   unique block ids per row (rows h*nb + i, shared by all b)      */
    const uint8_t *head_kind_host; /* host [H] salad_head_kind; NULL = all spatial               */
    float softmax_scale;      /* 0 selects 1/sqrt(d) (Eq. (1))                                    */
    int32_t phi;              /* salad_feature_map                                                */
    float eps;                /* added to the linear branch's denominator phi(Q_i).Z              */
    float lambda;             /* static per-layer scalar (Sec. 4.2, the lambda equation)          */
    const float *head_scale;  /* device [H] static per-head scale a_h; NULL = 1                   */
    const float *s_dev;       /* device [B] precomputed dynamic scale s, or NULL                  */
    const void *x_t;          /* device [B,N,H*d], used when s_dev == NULL (Alg. 1 Level 2)       */
    const float *w_gate;      /* device [H*d] gate weights, used when s_dev == NULL               */
    float b_gate;             /* scalar added before the sigmoid (0 in the paper's layer)         */
    float *s_out;             /* optional device [B]: the dynamic scale that was applied          */
    float *o_sparse_dbg;      /* optional device fp32 [B,H,N,d]: sparse branch alone              */
    float *o_linear_dbg;      /* optional device fp32 [B,H,N,d]: unscaled linear branch alone     */
    void *workspace;          /* device, >= salad_fwd_workspace_bytes(), 256-byte aligned; always needed */
    size_t workspace_bytes;
    int32_t flags;            /* SALAD_FLAG_* */
    void *hip_stream;
    float drop_threshold;     /* post-tuning branch dropping (Sec. 4.3): tau_t; <= 0 disables         */
    int32_t *dropped_out;     /* optional device int32 [B]: 1 where the linear branch was pruned, else 0;
                                 written only when dropping is active (lambda != 0, drop_threshold > 0)  */
    const void *w_proj;       /* optional device bf16 [H*d, H*d], row-major, row = input channel h_in*d + a,
                                 column = output channel h_out*d + c: the full Level-1 projection (Alg. 1
                                 "Proj").  Needs dtype bf16, d = 128 and head_scale == NULL                */
    int32_t topk;             /* > 0: Top-K dynamic block mask (Sec. 3 "Top-K attention", App. A.1.2) instead of the
                                 CSR: every query token keeps the topk (<= 8) key blocks whose mean key has the
                                 largest dot product with it; row_ptr / col_idx are ignored (may be NULL).  Needs
                                 dtype bf16, d = 128.  Key blocks are runs of the head's own token order           */
    int32_t topk_key_block;   /* tokens (positions of the head's order) per key block: a multiple of 64 with
                                 ceil(N / topk_key_block) <= 64                                                       */
    uint64_t *topk_mask_out;  /* optional device uint64 [B,H,N]: bit J set = the query keeps key block J            */
    const float *rope_cos;    /* optional device fp32 [N, d/2] (shared by all samples and heads), with rope_sin: rotary  */
    const float *rope_sin;    /*   position embedding inside the linear branch (Sec. 4.1): cosine and sine of the angle
                                   of channel pair (2p, 2p+1) of token n at [n*d/2 + p].  Needs dtype bf16, d = 128;
                                   may be combined with w_proj (the rotated O_l is what gets projected)             */
    const void *tile_lists;   /* optional device buffer filled by salad_tile_lists for exactly this row_ptr / col_idx (same H, N):
                                 the bf16 d = 128 kernel then skips its per-call list pre-pass.  NULL: the lists are built
                                 in the workspace on every call.  Ignored with topk > 0 and by the other kernels            */
    const void *w_proj_packed; /* optional device buffer filled by salad_proj_pack from the layer's W_p (static per layer): the
                                 full projection then skips its per-call rearrangement of w_proj, which may be NULL.
                                 Same conditions as w_proj (dtype bf16, d = 128, head_scale == NULL)                          */
} salad_fwd_params;

/* Run the linear apply and the scale-and-sum as a separate streaming kernel after the sparse
 * kernel instead of inside its epilogue (same result up to rounding; bf16 only). */
#define SALAD_FLAG_UNFUSED_EPILOGUE 1

/* Device scratch the forward needs for these shapes (partial states, partial gate sums, the
 * reduced state, per-tile block lists; with w_proj also O_l and the rearranged W_p; with topk the key-block means,
 * the masks and per-sample lists).  Reads only B, H, N, d, dtype, topk and whether w_proj and rope_cos are NULL.
 * 0 on invalid shapes. */
size_t salad_fwd_workspace_bytes(const salad_fwd_params *p);

/* Alg. 1 from SparseAttn to the residual sum:
 *   O_s = softmax over the kept KV blocks of (Q K^T * softmax_scale) V          (Eq. (2))
 *   O_l = phi(Q) Hs / (phi(Q).Z + eps), Hs = sum_j phi(K_j)^T V_j, Z = sum_j phi(K_j)  (Eq. (3))
 *   s_b = mean_n sigmoid(x_t[b,n,:].w_gate + b_gate)                             (Level 2)
 *   out = O_s + lambda * a_h * s_b * O_l                (Level 1 in per-head form + residual)
 * With lambda == 0 the linear branch is skipped and out is the sparse branch alone.
 * With w_proj the static scaling is the paper's full projection across heads instead of per-head scalars:
 *   out[b,n,:] = O_s[b,n,:] + lambda * s_b * (O_l[b,n,:] W_p),  O_l[b,n,:] the heads' outputs concatenated
 * (per-head form: W_p = blockdiag(a_h I)).  It runs as separate kernels after the sparse kernel: O_l is written
 * to the workspace (bf16), W_p is rearranged into MFMA fragment order, and one bf16 MFMA GEMM adds lambda s_b O_l W_p
 * to O_s (fp32 accumulation, one rounding of the sum).  o_linear_dbg is not written in this mode.
 * With topk > 0 the sparse branch uses the Top-K block mask of App. A.1.2 in place of the CSR: the keys are cut into
 * blocks of topk_key_block consecutive tokens of the head's own order (App. A.1.1: the stored order for a SPATIAL head,
 * tokens grouped by location for a TEMPORAL one; the token-mask variant of salad_tune("topk_variant", 1) takes SPATIAL
 * heads only), each block is reduced to its mean key, every query token
 * keeps the topk blocks with the largest q.mean and attends to exactly their tokens.  The selection runs on the
 * device in a fixed float32 order (block sums token by token, scores channel by channel with fused multiply-adds,
 * ties to the lower block index), so that it can be reproduced bit for bit.  The default Top-K path computes one
 * partial result per kept key block and query (normalised, rounded to bf16, with its log-sum-exp in fp32) and merges
 * them; with topk <= 4, lambda != 0 and none of w_proj, rope_*, o_sparse_dbg, o_linear_dbg the merge happens inside
 * the linear-apply pass in fp32 (one rounding of the sum), otherwise a merge kernel writes O_s in bf16 first.
 * With rope_cos / rope_sin the linear branch carries a rotary position embedding (the paper states that it does and
 * gives no formula; the reading implemented): phi(Q), phi(K) are rotated pairwise by the given angles in the numerator,
 * the normaliser keeps the unrotated features:
 *   O_l[i] = sum_j (R_i phi(Q_i)).(R_j phi(K_j)) V_j / (phi(Q_i).Z + eps) = (R_i phi(Q_i)) Hr / (phi(Q_i).Z + eps),
 *   Hr = sum_j (R_j phi(K_j))^T V_j.  The caller owns the split of the pairs over the t, y, x axes and the frequencies
 * (they are in the tables; the kernels read them as fp16 pairs packed once per call).  The rotation of phi(Q) happens
 * in the attention kernel's epilogue (bf16 d = 128 large-tile kernel) or in the separate linear-apply kernel (unfused
 * epilogue, Top-K, w_proj: there the rotated O_l is what the projection multiplies).
 * Post-tuning branch dropping (Sec. 4.3, App. A.3): with drop_threshold = tau > 0, a sample whose dynamic
 * scale s_b < tau (strict, compared in fp32) loses its linear branch: out[b] = O_s[b], exactly as with
 * lambda == 0.  The decision is taken on the device (no host synchronisation): the gate is reduced first,
 * and the state, reduce and apply kernels skip the pruned samples, so their K, V are not read again.
 * bf16: MFMA kernels, fp32 accumulation, one round-to-nearest-even of the sum to bf16.
 * fp32: plain fp32 kernels intended for small shapes. */
salad_status salad_sparse_linear_attn_fwd(const salad_fwd_params *p);

/* ---- single steps (the same kernels the layer call launches) -------------------------------- */

/* Eq. (3) sums: Hs [B,H,d,d] (Hs[a][c] = sum_j relu(K[j][a]) V[j][c]) and Z [B,H,d], fp32.
 * workspace as for the layer call with the same B, H, N, d, dtype. */
salad_status salad_linear_state_fwd(const void *k, const void *v, int32_t B, int32_t H, int32_t N,
                                    int32_t d, int32_t dtype, float *Hs_out, float *Z_out,
                                    void *workspace, size_t workspace_bytes, void *hip_stream);

/* Alg. 1 Level 2: s[b] = mean_n sigmoid(x_t[b,n,:].w_gate + b_gate); x_t [B,N,D], s fp32 [B].  D a multiple of 8 up to
 * 8192 (the widest row of the layer: 64 heads of 128 channels).  workspace: 256-byte aligned, at least
 * 4 * B * min(ceil(N/16), 512) + 4 * B bytes with each of the two parts rounded up to 256 bytes. */
salad_status salad_gate_fwd(const void *x_t, const float *w_gate, float b_gate, int32_t B, int32_t N,
                            int32_t D, int32_t dtype, float *s_out,
                            void *workspace, size_t workspace_bytes, void *hip_stream);

/* salad_gate_fwd for callers that cannot allocate or bring a workspace (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): same kernels and same result, with the partial sums in a static device
 * buffer of SALAD_STATIC_SCRATCH_BYTES that is part of the library (one copy per GPU, held until the process ends).
 * Calls no hipMalloc / hipFree or any allocating routine.  SALAD_ENOSPC when B is too large for the buffer
 * (B * min(ceil(N/16), 512) partial sums + B results, each group rounded up to 256 bytes).  All calls on one GPU share
 * the buffer: calls that may overlap on one GPU (different streams or threads) race; calls on one stream do not. */
#define SALAD_STATIC_SCRATCH_BYTES 65536
salad_status salad_gate_fwd_static(const void *x_t, const float *w_gate, float b_gate, int32_t B, int32_t N,
                                   int32_t D, int32_t dtype, float *s_out, void *hip_stream);

/* ---- per-kernel timing ----------------------------------------------------------------------- */

typedef struct salad_kernel_times {
    float gate_ms, state_ms, finalize_ms, attn_ms, epilogue_ms; /* summed over calls            */
    int32_t calls;
    float proj_ms;            /* full Level-1 projection: W_p rearrangement + GEMM (0 without w_proj)   */
    float topk_ms;            /* Top-K mask: key-block means, selection, visit lists (0 without topk);
                                 attn_ms is then the attention kernel alone                             */
} salad_kernel_times;

/* on = 1: the layer call brackets each of its stages with HIP events on its stream (eight records per call; every
 * record is a dependency between two kernels that would otherwise start back to back, so the call itself gets some
 * 5 % slower).  on = 2: only the attention stage (pre-pass + attention kernel, Top-K: + the merge kernel when the
 * linear-apply pass does not merge) is bracketed, two
 * records per call; salad_timing_read then fills attn_ms and calls only.  on = 0: no events.  Other values:
 * SALAD_EINVAL. */
salad_status salad_timing_enable(int32_t on);
/* Waits for the recorded events, adds up the elapsed times since the last reset into *out and
 * (if reset != 0) clears the record.  This one call does synchronise with the host. */
salad_status salad_timing_read(salad_kernel_times *out, int32_t reset);

/* ---- tuning ----------------------------------------------------------------------------------- */

/* Launch-shape knobs for experiments; results do not depend on them beyond rounding order.  These are all the keys
 * (any other key, or a value out of range: SALAD_EINVAL).  The values are process-wide atomics; an entry point reads
 * each once at its start, so a concurrent salad_tune cannot change a call half way through.  A thread that changes
 * "state_wgs" between salad_fwd_workspace_bytes and the call gets SALAD_ENOSPC from the call's own size check.
 *   "state_wgs"     1..65536 (default 256): target workgroup count of the linear-state kernel (changes the workspace
 *                   size: query salad_fwd_workspace_bytes again after setting it).
 *   "attn_variant"  0 (default): the bf16 attention kernel is chosen by shape (256-query tiles for d = 128 and
 *                   d = 64, falling back to 128-query tiles at d = 128, to the first-generation kernel at d = 64,
 *                   when the block list does not fit); 1: never 256-query tiles; 2: the first-generation kernel.
 *                   Same results within the parity bar.
 *   "topk_variant"  0 (default): Top-K attention regrouped by key block (queries that keep a block are gathered,
 *                   partial results merged); 1: token mask applied on ordinary query tiles. */
salad_status salad_tune(const char *key, int32_t value);

#ifdef __cplusplus
}
#endif
#endif /* SALAD_H */
