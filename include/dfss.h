/*
 * dfss.h -- C ABI of the DFSS attention forward library for AMD MI355X (gfx950).
 *
 * DFSS = dynamic N:M fine-grained structured sparse attention, arXiv 2203.00091.
 * The forward pass of one attention head is (Sec. 3.1, stages of the attention):
 *
 *   stage 1  S = scale * Q K^T, and inside the same kernel every aligned run of M
 *            consecutive keys of a row is pruned to its N largest scores; only the
 *            kept scores ("non-zeros") and their position codes ("metadata") are
 *            written (Sec. 3.4, App. A.1.1, A.1.2);
 *   stage 2  softmax over the kept scores of each row (Sec. 3.1, App. A.1.3);
 *   stage 3  O = A_sparse V with the compressed weights (Sec. 3.1).
 *
 * Supported: bfloat16 inputs, N:M = 2:4 (the paper's bfloat16 mode, Sec. 2.3) and
 * 1:2 on the same 2-byte data; float inputs with 1:2 (the paper's 4-byte mode, see
 * "the 4-byte mode" below); d in {64, 128}; Lq a multiple of 64, Lk a multiple
 * of 128 and at most 8192.  With bfloat16 data the stage calls (stage 1, 2, 3, the staged forward
 * pass, the three-kernel baseline), the *_ragged one-kernel calls and the one-kernel *_mask calls also take any Lq >= 1 and any
 * Lk % 4 == 0 ("lengths that are not tile multiples" below).  Selection rule: larger signed score wins, equal scores -> lower key
 * index wins; comparisons are made on the fp32 value scale*dot, which is then
 * rounded to bfloat16 (nearest-even) for storage (kept as it is in the 4-byte mode).
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers to contiguous row-major arrays owned by
 *     the caller; the library allocates, frees and retains nothing.
 *   - Q is [B*H, Lq, d], K and V are [B*H, Lk, d], O is [B*H, Lq, d]  (bfloat16).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is
 *     enqueued asynchronously; no call synchronises the host with the device.
 *   - Return value is a dfss_status; nothing throws, aborts or prints.  Arguments
 *     are validated before any launch, so an error return means no work was queued
 *     (except DFSS_ERR_HIP, which reports a failed launch).
 *   - Results are deterministic: no atomics, fixed reduction order.
 */
#ifndef DFSS_H
#define DFSS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DFSS_OK = 0,
    DFSS_ERR_NULL = 1,        /* a required pointer is NULL                             */
    DFSS_ERR_SHAPE = 2,       /* non-positive size, or a size that breaks alignment      */
    DFSS_ERR_UNSUPPORTED = 3, /* N:M, dtype, d or scale outside what is implemented      */
    DFSS_ERR_WORKSPACE = 4,   /* workspace smaller than *_workspace_bytes() reports      */
    DFSS_ERR_HIP = 5          /* the HIP runtime refused a launch                        */
} dfss_status;

typedef enum { DFSS_BF16 = 0, DFSS_F32 = 1, DFSS_F32_BF16X3 = 2 } dfss_dtype;

typedef struct {
    int32_t B, H;   /* batch and heads; only the product B*H matters, except that a     */
                    /* key bias is indexed by the batch element b = (b*H + h) / H       */
    int32_t Lq, Lk; /* number of queries (rows of S) and keys (columns of S)            */
    int32_t d;      /* head dimension                                                   */
    int32_t N, M;   /* keep N of every M consecutive keys: (2,4) or (1,2)               */
    int32_t dtype;  /* dfss_dtype                                                       */
} dfss_shape;

/* ---- sizes (host only, no GPU needed); 0 if the shape is invalid ---------------- */

/* Kept scores / weights: bfloat16 [B*H, Lq, Lk*N/M], row-major, key order (Sec. 2.3). */
size_t dfss_vals_bytes(const dfss_shape *s);
/* Metadata: one 4-bit code per run of 4 keys, four codes per uint16 (Sec. 2.3: 1/16 of
 * the dense matrix in bits; App. A.1.2: code k of a word at bits [4k,4k+3]).  The words
 * are held in the library's own order (see dfss_meta_to_canonical). */
size_t dfss_meta_bytes(const dfss_shape *s);
/* Workspace of dfss_attention_staged (and of dfss_attention with DFSS_F32): vals, then meta. */
size_t dfss_workspace_bytes(const dfss_shape *s);
/* Workspace of dense_attention: the dense bfloat16 score/weight matrix [B*H, Lq, Lk]. */
size_t dense_workspace_bytes(const dfss_shape *s);

/* ---- stage 1: SDDMM with the pruning epilogue (Sec. 3.4, App. A.1.2) ------------- */
/* Q, K: device, bfloat16.  scale: finite and > 0 (1/sqrt(d) in Eq. 1).
 * vals: device out, dfss_vals_bytes().  meta: device out, dfss_meta_bytes(). */
dfss_status dfss_sddmm_prune(const void *Q, const void *K, const dfss_shape *s, float scale,
                             void *vals, void *meta, void *stream);

/* ---- stage 2: softmax over the kept entries of each row, in place (App. A.1.3) --- */
/* vals: device in/out, bfloat16 [B*H, Lq, Lk*N/M]; fp32 arithmetic inside. */
dfss_status dfss_sparse_softmax(void *vals, const dfss_shape *s, void *stream);

/* ---- stage 3: O = A_sparse V (Sec. 3.1) ------------------------------------------ */
/* vals, meta: device in, as written by stage 1 (vals after stage 2).  V: device in.
 * O: device out, bfloat16 [B*H, Lq, d]; fp32 accumulation. */
dfss_status dfss_spmm(const void *vals, const void *meta, const void *V, const dfss_shape *s,
                      void *O, void *stream);

/* ---- whole forward pass (Eq. 1 with the pruned score matrix) ---------------------- */
/* Computes the same function as stage 1 -> 2 -> 3 in ONE kernel that keeps the pruned scores in
 * registers (the pruning epilogue of Sec. 3.4 taken to its end: nothing of the score matrix is
 * written).  ws / ws_bytes: used only with dtype DFSS_F32, which has no one-kernel path and runs the
 * three stage kernels through ws (then at least dfss_workspace_bytes(), 256-byte aligned); with every
 * other dtype they are ignored and ws may be NULL.  Which kernel runs depends on the arguments only
 * (no environment variables, no global state). */
dfss_status dfss_attention(const void *Q, const void *K, const void *V, const dfss_shape *s,
                           float scale, void *O, void *ws, size_t ws_bytes, void *stream);

/* The same function through the workspace, the structure whose latency the paper reports (Sec. 5.2).
 * 2-byte dtype: TWO kernels.  Stage 1 writes the kept scores and the metadata into ws; the second kernel
 * is the stage-3 product with the softmax of stage 2 applied to the scores as it reads them (running row
 * maximum, sums divided out at the end), which saves the separate pass of App. A.1.3 over all kept values
 * (one read and one write of them).  Afterwards ws holds the kept SCORES (at offset 0) and the metadata
 * (at offset dfss_vals_bytes() rounded up to 256) of this forward pass.  The weights that
 * dfss_attention_backward needs are not formed: run the three stage calls for them.  The result differs
 * from the three stage calls by roundings only (same kept keys; the weights are rounded to bfloat16 before
 * instead of after the normalisation).
 * 4-byte dtypes: the three stage kernels one after the other; ws then holds the weights and the metadata.
 * ws: device scratch of at least dfss_workspace_bytes(), 256-byte aligned.  key_bias (may be NULL) as
 * described below. */
dfss_status dfss_attention_staged(const void *Q, const void *K, const void *V, const dfss_shape *s,
                                  float scale, void *O, void *ws, size_t ws_bytes, void *stream);
dfss_status dfss_attention_staged_bias(const void *Q, const void *K, const void *V, const void *key_bias,
                                       const dfss_shape *s, float scale, void *O, void *ws, size_t ws_bytes,
                                       void *stream);

/* ---- full attention on the same GPU (Eq. 1), the denominator of every speedup ---- */
/* Same three-stage structure with the dense score matrix stored in bfloat16 in ws
 * (at least dense_workspace_bytes()).  s->N, s->M are ignored. */
dfss_status dense_attention(const void *Q, const void *K, const void *V, const dfss_shape *s,
                            float scale, void *O, void *ws, size_t ws_bytes, void *stream);

/* Eq. 1 in one kernel (scores, softmax and P V fused; nothing of the score matrix is
 * written): the stronger full-attention baseline, reported next to dense_attention. */
dfss_status dense_attention_fused(const void *Q, const void *K, const void *V, const dfss_shape *s,
                                  float scale, void *O, void *stream);

/* ---- the staged forward pass without a workspace argument ------------------------------------ */
/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): dfss_attention_staged_bias with the workspace taken from a fixed
 * array inside the library instead of from the caller.  key_bias may be NULL.  Same kernels, same
 * results bit for bit, same validation.  The call allocates and frees nothing; the array
 * (dfss_static_scratch_bytes() = 32 MiB of device memory per GPU the library runs on, held until the
 * process ends) bounds the shape: dfss_workspace_bytes(s) must not exceed it, else DFSS_ERR_WORKSPACE
 * and nothing is launched.  The array's address is looked up on the first call on each device (a
 * symbol lookup, no allocation), with that device current: make the first call on a device outside
 * any stream capture, and pass a stream of the current device.  Every call on a GPU uses that GPU's
 * one array: calls that overlap in time on the same GPU (different streams, or a graph replayed while
 * another call runs) race on it and give undefined results; calls ordered on one stream are safe.
 * Nothing in the array needs to be cleared between calls: stage 1 writes every byte that the kernels after
 * it read.  Afterwards the array holds what ws of dfss_attention_staged holds, for the last call. */
size_t dfss_static_scratch_bytes(void);
dfss_status dfss_attention_staged_static(const void *Q, const void *K, const void *V, const void *key_bias,
                                         const dfss_shape *s, float scale, void *O, void *stream);

/* ---- additive key bias (padding mask) ---------------------------------------------- */
/* The paper has no mask; padded batches need one.  Reading taken: key_bias[b][j] (float32,
 * device, [B, Lk] row-major, 16-byte aligned, shared by the H heads and all queries of batch
 * element b) is ADDED to the scaled score in fp32 BEFORE the N:M comparison of stage 1, so a
 * masked key (bias = -inf) loses against any unmasked key of its group; a run of M keys that is
 * entirely masked still emits N entries, whose softmax weight is exactly 0.  Sequences whose
 * length is not a multiple of the tile sizes need no padding of Q, K, V (see "lengths that are not
 * tile multiples" below); where a caller pads all the same, the padded keys are masked this way.
 * Precondition: every batch element has at least one key with a finite bias.
 * key_bias == NULL means no bias: each call then equals the call without the suffix.  All other
 * arguments, layouts and error behaviour are those of the call without the suffix.
 * Arithmetic: when scale is a power of two the bias is the initial value of the fp32 accumulator
 * (identical to a separate addition whenever the bias is 0 or -inf, else equal up to the
 * rounding order); otherwise it is added by a separate fp32 addition after the scaling. */
dfss_status dfss_sddmm_prune_bias(const void *Q, const void *K, const void *key_bias, const dfss_shape *s,
                                  float scale, void *vals, void *meta, void *stream);
dfss_status dfss_attention_bias(const void *Q, const void *K, const void *V, const void *key_bias,
                                const dfss_shape *s, float scale, void *O, void *ws, size_t ws_bytes,
                                void *stream);
dfss_status dense_attention_bias(const void *Q, const void *K, const void *V, const void *key_bias,
                                 const dfss_shape *s, float scale, void *O, void *ws, size_t ws_bytes,
                                 void *stream);
dfss_status dense_attention_fused_bias(const void *Q, const void *K, const void *V, const void *key_bias,
                                       const dfss_shape *s, float scale, void *O, void *stream);

/* A padding mask given by its lengths: key_len, device, int32 [B], 4-byte aligned; keys
 * key_len[b] .. Lk - 1 of batch element b are padding (as if key_bias[b][j] were -inf there and 0
 * before; 1 <= key_len[b] <= Lk, values outside are clamped).  The arrays keep the padded shape
 * [B*H, Lk, d]; precondition: the padding rows of K and V hold finite numbers (a kept padding key
 * has weight exactly 0, and 0 x infinity is not 0).  One kernel; every block before the one a
 * sequence ends in costs what it costs without padding, the blocks after it are not visited and no
 * bias array is read -- the fast call for padded batches.  2-byte dtype, tile shapes (Lq % 64 == 0,
 * Lk % 128 == 0).  The baseline on a padded batch is dense_attention_fused_bias with the equivalent
 * bias (the library's fastest full attention on such input). */
dfss_status dfss_attention_varlen(const void *Q, const void *K, const void *V, const void *key_len,
                                  const dfss_shape *s, float scale, void *O, void *stream);

/* ---- causal mask ---------------------------------------------------------------------- */
/* The paper evaluates encoders only (Sec. 5.1) and has no mask; a decoder needs one.  Reading taken:
 * the queries are the LAST Lq of the Lk positions (Lk >= Lq, else DFSS_ERR_SHAPE), so query i sits at
 * position i + (Lk - Lq) and sees keys 0 .. i + (Lk - Lq); the score of a hidden key counts as -inf
 * BEFORE the N:M comparison of stage 1 (the same place as the key bias), so a hidden key loses against
 * any visible key of its run of M, and a run that is entirely hidden still emits N entries, whose
 * softmax weight is exactly 0.  Every query sees at least key 0.  No mask array: the kernels derive
 * the hidden entries from the indices.  key_bias (may be NULL) is added as in the *_bias calls.
 * 2-byte dtype only (DFSS_ERR_UNSUPPORTED otherwise).
 *   dfss_sddmm_prune_causal       stage 1; the hidden entries are part of vals / meta (stages 2 and 3 are
 *                                 the plain calls)
 *   dfss_attention_causal         the whole forward pass in one kernel; blocks of 64 keys past the last
 *                                 visible key of a workgroup's queries are skipped (neither read nor
 *                                 computed)
 *   dfss_attention_staged_causal  the same through the workspace (as dfss_attention_staged)
 *   dense_attention_causal, dense_attention_fused_causal   Eq. 1 with the same mask (the baselines)
 * All other arguments, layouts and error behaviour are those of the calls without the suffix. */
dfss_status dfss_sddmm_prune_causal(const void *Q, const void *K, const void *key_bias, const dfss_shape *s,
                                    float scale, void *vals, void *meta, void *stream);
dfss_status dfss_attention_causal(const void *Q, const void *K, const void *V, const void *key_bias,
                                  const dfss_shape *s, float scale, void *O, void *stream);
dfss_status dfss_attention_staged_causal(const void *Q, const void *K, const void *V, const void *key_bias,
                                         const dfss_shape *s, float scale, void *O, void *ws, size_t ws_bytes,
                                         void *stream);
dfss_status dense_attention_causal(const void *Q, const void *K, const void *V, const void *key_bias,
                                   const dfss_shape *s, float scale, void *O, void *ws, size_t ws_bytes,
                                   void *stream);
dfss_status dense_attention_fused_causal(const void *Q, const void *K, const void *V, const void *key_bias,
                                         const dfss_shape *s, float scale, void *O, void *stream);

/* ---- general additive mask ---------------------------------------------------------------- */
/* mask: device, float32 [Lq, Lk] row-major, 16-byte aligned, shared by all B*H heads (relative
 * position terms, arbitrary visibility patterns; -inf hides a key from a query).  mask[i][j] is ADDED
 * to the scaled score of query i and key j in fp32 BEFORE the N:M comparison of stage 1 -- the reading
 * of the key bias and of the causal mask, which are its special cases (a mask of 0 / -inf along the
 * diagonal gives the causal calls' results bit for bit); a run of M keys that is entirely hidden from
 * a query still emits N entries of weight exactly 0.  Precondition: every query sees at least one
 * key.  Arithmetic and rounding: those of the key bias.  2-byte dtype only (DFSS_ERR_UNSUPPORTED
 * otherwise); lengths as in the stage calls (tile multiples, or any Lq and Lk % 4 == 0 with the
 * compressed arrays in the padded layout).  No block is skipped and the mask costs 4 bytes of reads
 * per score: where a mask is causal or a padding mask, the dedicated calls are the fast ones.
 *   dfss_sddmm_prune_mask        stage 1 (stages 2 and 3 are the plain calls)
 *   dfss_attention_staged_mask   the forward pass through the workspace (as dfss_attention_staged)
 *   dense_attention_mask         Eq. 1 with the same mask, three kernels (the baseline)
 * All other arguments, layouts and error behaviour are those of the calls without the suffix. */
dfss_status dfss_sddmm_prune_mask(const void *Q, const void *K, const void *mask, const dfss_shape *s,
                                  float scale, void *vals, void *meta, void *stream);
dfss_status dfss_attention_staged_mask(const void *Q, const void *K, const void *V, const void *mask,
                                       const dfss_shape *s, float scale, void *O, void *ws, size_t ws_bytes,
                                       void *stream);
dfss_status dense_attention_mask(const void *Q, const void *K, const void *V, const void *mask,
                                 const dfss_shape *s, float scale, void *O, void *ws, size_t ws_bytes,
                                 void *stream);

/* The same mask in the one-kernel forward pass (nothing but O is written; Sec. 3.1 as dfss_attention
 * computes it).  mask as above; mask[i][j] joins the scaled score before the selection -- when scale is
 * a power of two as the initial value of the fp32 accumulation (one rounding less than in the stage
 * calls), so the two families agree to the tolerance of the one-kernel calls, not bit for bit.  Lengths
 * as in the _ragged calls: any Lq, Lk % 4 == 0, arrays unpadded (Q, O [B*H, Lq, d]; K, V [B*H, Lk, d]).
 * Every 64-key block is visited.  2-byte dtype only.  dense_attention_fused_mask is Eq. 1 with the same
 * mask in one kernel (the baseline). */
dfss_status dfss_attention_mask(const void *Q, const void *K, const void *V, const void *mask, const dfss_shape *s,
                                float scale, void *O, void *stream);
dfss_status dense_attention_fused_mask(const void *Q, const void *K, const void *V, const void *mask,
                                       const dfss_shape *s, float scale, void *O, void *stream);

/* ---- hybrid block sparsity x N:M (App. A.1.2, "Blocked-ELL Sparsity") ---------------- */
/* block_mask: device, uint8 [Lq/64, Lk/64] row-major, shared by all B*H heads.  A 64 x 64 block
 * of the score matrix whose entry is zero is not part of the attention: it is skipped (neither
 * its K/V blocks are read nor its scores formed), which as a function means that all its scores
 * are -inf.  Within the kept blocks the N:M pruning, softmax and product with V are those of
 * dfss_attention.  The block size equals the workgroup tile (64 queries x 64 keys), as the paper
 * prescribes.  key_bias (may be NULL) as in dfss_attention_bias.  Precondition: every row of
 * blocks keeps at least one block that holds an unmasked key.  Runs as one fused kernel; no
 * workspace.  dense_attention_fused_blocked is the same block pattern without N:M pruning
 * (block-sparse full attention), the baseline for this mode. */
dfss_status dfss_attention_blocked(const void *Q, const void *K, const void *V, const void *key_bias,
                                   const void *block_mask, const dfss_shape *s, float scale, void *O,
                                   void *stream);
dfss_status dense_attention_fused_blocked(const void *Q, const void *K, const void *V, const void *key_bias,
                                          const void *block_mask, const dfss_shape *s, float scale, void *O,
                                          void *stream);

/* The same two functions with a workspace, for patterns whose row blocks differ widely in length (a
 * few "global" row blocks that see every key next to rows that see a window: the pattern family of
 * the block-sparse long-sequence models the paper combines with).  The first four row blocks of the
 * pattern that keep more than 16 blocks are each shared between four workgroups, which take every
 * fourth kept block; their partial results (running reference, row sums, unnormalised O; fp32) pass
 * through ws and a second kernel merges them in a fixed order, so results are deterministic.  Every
 * other row block is computed as in the calls above.  Which row blocks are shared depends on
 * block_mask alone.  Results equal those of the calls above up to the rounding of the merge.
 * Pays where the long row blocks set the time of the call above: d = 64 and 2048 keys or more
 * (elsewhere it costs the second launch and gains nothing).
 * ws: device, 16-byte aligned, at least dfss_blocked_split_workspace_bytes(s) bytes (0 = unsupported
 * shape or dtype; 2-byte dtype only), caller-owned, contents undefined before and after; no
 * initialisation needed.  Errors as above, plus DFSS_ERR_WORKSPACE. */
size_t dfss_blocked_split_workspace_bytes(const dfss_shape *s);
dfss_status dfss_attention_blocked_split(const void *Q, const void *K, const void *V, const void *key_bias,
                                         const void *block_mask, const dfss_shape *s, float scale, void *O,
                                         void *ws, size_t ws_bytes, void *stream);
dfss_status dense_attention_fused_blocked_split(const void *Q, const void *K, const void *V,
                                                const void *key_bias, const void *block_mask,
                                                const dfss_shape *s, float scale, void *O, void *ws,
                                                size_t ws_bytes, void *stream);

/* ---- lengths that are not tile multiples ------------------------------------------------ */
/* The stage calls, bfloat16 data.  dfss_sddmm_prune(_bias), dfss_sparse_softmax, dfss_spmm,
 * dfss_attention_staged(_bias), dfss_attention_staged_static, dense_attention(_bias), dfss_spmm_t,
 * dfss_attention_backward, the size functions and the metadata conversions take ANY Lq >= 1 and any
 * Lk <= 8192 that is a multiple of 4 (whole runs of M keys).  Q and O are [B*H, Lq, d], K and V [B*H, Lk, d], key_bias [B, Lk], as
 * always; only the arrays the library defines -- vals, meta (both word orders), the workspaces --
 * are laid out for the PADDED lengths LqP = Lq rounded up to a multiple of 64 and LkP = Lk rounded up
 * to a multiple of 128: vals [B*H, LqP, LkP*N/M], canonical meta [B*H, LqP, LkP/16]
 * (dfss_vals_bytes etc. report these sizes; tile multiples are their own padded lengths, so nothing
 * changes for them).  The keys Lk .. LkP-1 do not exist: their scores count as -inf before the
 * comparison (as under a key bias of -inf), so a run of M keys that is entirely absent emits N
 * entries of weight exactly 0.  The rows Lq .. LqP-1 of vals and meta hold valid but meaningless
 * entries, and no such row of O is written; nothing is read or written past the caller's arrays.
 * The backward calls take P, meta (and dS in the workspace) in the same padded layout, whatever the
 * rows past Lq hold: those rows take no part in dK and dV, the absent keys (weight 0) none in dQ,
 * and dQ [B*H, Lq, d], dK, dV [B*H, Lk, d] are written for the real rows only.
 * The causal calls and the block-pattern calls take tile multiples only (DFSS_ERR_UNSUPPORTED /
 * DFSS_ERR_SHAPE otherwise), and so do the 4-byte dtypes.
 *
 * The one-kernel calls: */
/* The paper's long-sequence tasks have lengths such as 4000 (Sec. 5.1, the retrieval task).  These two
 * calls take the arrays as they are: Q, O [B*H, Lq, d] and K, V [B*H, Lk, d] with ANY Lq >= 1 and any
 * Lk <= 8192 that is a multiple of 4 (whole runs of M keys; the key_bias rows [B, Lk] stay 16-byte
 * aligned); key_bias may be NULL.  dtype: DFSS_BF16 or DFSS_F32_BF16X3.  The function is that of
 * dfss_attention_bias / dense_attention_fused_bias on those lengths (Eq. 1 over the Lk keys, pruned
 * per aligned run of M): inside the kernel the absent keys of the last 64-key block count as masked
 * keys and the absent queries of the last tile are not stored; nothing is read or written past the
 * arrays.  One kernel, no workspace.  Lengths that are tile multiples give the result of the calls
 * above bit for bit. */
dfss_status dfss_attention_ragged(const void *Q, const void *K, const void *V, const void *key_bias,
                                  const dfss_shape *s, float scale, void *O, void *stream);
dfss_status dense_attention_fused_ragged(const void *Q, const void *K, const void *V, const void *key_bias,
                                         const dfss_shape *s, float scale, void *O, void *stream);

/* ---- backward pass through the fixed selection (finetuning, Sec. 5.1) ---------------- */
/* Transposed sparse product: out[B*H, Lk, d] = A^T X with A given in compressed form (vals,
 * meta as written by stage 1 / stage 2) and X bfloat16 [B*H, Lq, d]; fp32 accumulation, bfloat16
 * output.  With A = softmax weights P and X = dO this is dV; with A = dS and X = Q it is dK. */
dfss_status dfss_spmm_t(const void *vals, const void *meta, const void *X, const dfss_shape *s, void *out,
                        void *stream);

/* Gradients of O = dfss attention(Q, K, V) with respect to Q, K, V, the N:M selection of the forward
 * pass held fixed (the paper finetunes with this attention but gives no backward kernel; a pruning
 * decision has no gradient, so gradients flow through the kept entries only).  With P the softmax
 * weights of the kept entries:
 *     dV = P^T dO,  dP = dO V^T at the kept positions,  delta_i = dO_i . O_i,
 *     dS = P .* (dP - delta),  dQ = scale dS K,  dK = scale dS^T Q.
 * Inputs (device, bfloat16 unless noted): dO [B*H, Lq, d]; Q, K, V, O as in the forward pass; P, meta =
 * the vals buffer after dfss_sparse_softmax and the metadata of dfss_sddmm_prune of the SAME forward pass
 * (run the three stage calls to keep them; they compose to dfss_attention).  Outputs: dQ [B*H, Lq, d],
 * dK, dV [B*H, Lk, d], bfloat16.  ws: device scratch of at least dfss_backward_workspace_bytes(),
 * 256-byte aligned (holds dS).  A key bias of the forward pass needs no extra argument: masked
 * entries have weight 0 and so receive and pass on no gradient.  Kernels: the stage-1 mainloop with the stored
 * position codes in the place of the selection (dS; at d = 64 it forms dQ in the same pass, at d = 128 the
 * stage-3 SpMM does), and the transposed sparse product twice (dV, dK). */
size_t dfss_backward_workspace_bytes(const dfss_shape *s);
dfss_status dfss_attention_backward(const void *dO, const void *Q, const void *K, const void *V, const void *O,
                                    const void *P, const void *meta, const dfss_shape *s, float scale, void *dQ,
                                    void *dK, void *dV, void *ws, size_t ws_bytes, void *stream);

/* ---- the 4-byte mode (Sec. 2.3: 1:2 on float data; App. A.1.1) ------------------------ */
/* With dfss_shape.dtype = DFSS_F32 the arrays Q, K, V, O, vals (kept scores / weights) and the dense
 * workspace hold float32 instead of bfloat16, and N:M must be 1:2 (2:4 is DFSS_ERR_UNSUPPORTED).
 * Calls that take this dtype: the size functions, dfss_sddmm_prune(_bias), dfss_sparse_softmax,
 * dfss_spmm, dfss_attention(_bias) and dfss_attention_staged(_bias) (always the three stage kernels
 * through the workspace), dense_attention(_bias) and the two metadata conversions; the remaining
 * calls return DFSS_ERR_UNSUPPORTED.  With DFSS_F32_BF16X3 (see below) every call of the library
 * is available: also the one-kernel forms, the *_blocked calls, dfss_spmm_t and
 * dfss_attention_backward (all arrays float32 there, dS in the workspace included).
 * (In both, the key bias is added by a separate fp32 addition after the scaling, whatever the scale.)
 * Arithmetic: fp32 products and fp32 accumulation on the fp32 matrix instruction (the paper rounds
 * the float inputs to a shorter mantissa for its tensor cores; this GPU has no such format, so the
 * scores are at least that accurate); the kept scores are stored unrounded.
 * Metadata: a float fills two consecutive 2-byte slots of a run of four, so a run is one aligned
 * pair of keys and only two codes occur, the ones App. A.1.1 prints: 0x4 = the first float of the
 * pair is kept, 0xE = the second.  uint16 [B*H, Lq, Lk/8], word w of a row = codes of pairs
 * 4w..4w+3, pair 4w+k at bits [4k, 4k+3] -- again 1/16 of the dense matrix in bits.  That is the
 * canonical order; the library holds the words pairwise as 32-bit words (word v of a row = keys
 * 16v..16v+15), rows in blocks of 16, keys in blocks of 64:
 *   lib32[bh][r/16][v/4][r%16][v%4] = canon32[bh][r][v]
 * (the blocking of the 2-byte modes without their slot permutation); dfss_meta_to_canonical and
 * dfss_meta_from_canonical convert.
 * DFSS_F32_BF16X3 is the same mode (same arrays, layouts, calls and restrictions) with the products
 * formed on the bfloat16 matrix pipe, the analogue of the paper's reduced-mantissa multiplication
 * (App. A.1.2): each fp32 operand is split as x = hi + lo with hi = bf16(x), lo = bf16(x - hi), and
 * a*b is taken as a_hi*b_hi + a_hi*b_lo + a_lo*b_hi, accumulated in fp32.  The dropped terms are at
 * most 3 * 2^-18 |a*b| per product (the paper's format drops about 2^-10); operands that are exact
 * in bfloat16 (e.g. small integers) give exactly the DFSS_F32 result.  The softmax stage is the same
 * fp32 kernel.  Several times faster than DFSS_F32, whose matrix instruction is 16x slower.
 * With this dtype dfss_attention runs as ONE kernel that keeps the pruned scores and the weights in
 * registers (same function as the three stages, softmax kept up to date block by block;
 * dfss_attention_staged runs the stage kernels), and dense_attention_fused is available as
 * the matching full-attention kernel. */

/* ---- metadata order ---------------------------------------------------------------- */
/* Canonical order: uint16 [B*H, Lq, Lk/16], word w of a row = codes of key runs
 * 4w..4w+3, code = p_lo | p_hi << 2 with p the kept key index mod 4 (the 2-bit
 * position rule that yields the two codes App. A.1.1 prints, 0x4 and 0xe).
 * Library order: the canonical words are taken in pairs as 32-bit words (the earlier one in
 * the low half; word v covers keys 32v..32v+31), rows in blocks of 16, keys in blocks of 128:
 *   lib32[bh][r/16][v/4][r%16][slot(v%4)] = canon32[bh][r][v],  slot(c) = 2*(c%2) + c/2,
 * i.e. the four words of a row for one 128-key block are adjacent (chunk order 0, 2, 1, 3).
 * Both calls take device pointers; `meta` and `canon` must not overlap. */
dfss_status dfss_meta_to_canonical(const void *meta, const dfss_shape *s, uint16_t *canon, void *stream);
dfss_status dfss_meta_from_canonical(const uint16_t *canon, const dfss_shape *s, void *meta, void *stream);

const char *dfss_status_string(dfss_status st);

#ifdef __cplusplus
}
#endif
#endif /* DFSS_H */
