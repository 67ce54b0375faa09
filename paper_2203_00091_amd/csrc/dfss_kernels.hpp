// Host-side launchers of the DFSS kernels (internal to the library; the public
// interface is include/dfss.h).  Every launcher assumes validated arguments.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dfss {

// key_bias (where present): fp32 [BH / H][Lk] added to the scaled scores before the selection, or
// nullptr for none (then H is ignored).
// LqR, LkR (where present): the real lengths of the caller's arrays (Q, K, V, key_bias, O) when they differ from the
// layout lengths Lq (a multiple of 64) and Lk (of 128) of the compressed arrays; else equal to Lq, Lk.
// Stage 1 (Sec. 3.4, App. A.1.2): scores + N:M pruning epilogue.  mode: 0 = 2:4, 1 = 1:2.
hipError_t launch_sddmm_prune(const void *Q, const void *K, const float *key_bias, int H, int causal, int BH, int Lq, int Lk,
                              int LqR, int LkR, int d, int mode, float scale, void *vals, void *meta, hipStream_t st);
// Dense scores S = scale * Q K^T stored as bfloat16 [BH, Lq, Lk] (Eq. 1), same mainloop.
hipError_t launch_dense_scores(const void *Q, const void *K, const float *key_bias, int H, int causal, int BH, int Lq, int Lk,
                               int LqR, int LkR, int d, float scale, void *S, hipStream_t st);
// The same two with an additive mask fp32 [LqR][LkR] shared by all heads (added like the key bias; -inf hides a key
// from a query) in the place of the per-key bias.
hipError_t launch_sddmm_prune_mask(const void *Q, const void *K, const float *mask, int BH, int Lq, int Lk, int LqR,
                                   int LkR, int d, int mode, float scale, void *vals, void *meta, hipStream_t st);
hipError_t launch_dense_scores_mask(const void *Q, const void *K, const float *mask, int BH, int Lq, int Lk, int LqR,
                                    int LkR, int d, float scale, void *S, hipStream_t st);
// Row softmax in place over bfloat16 rows (App. A.1.3); rows of `cols` elements.
hipError_t launch_row_softmax(void *x, long rows, int cols, hipStream_t st);
// Stage 3 (Sec. 3.1): O = A_sparse V from compressed weights + metadata.
hipError_t launch_spmm(const void *vals, const void *meta, const void *V, int BH, int Lq, int Lk, int LqR, int LkR, int d,
                       void *O, hipStream_t st);
// The same product on the kept SCORES of stage 1, with the softmax over them applied on the way.
hipError_t launch_softmax_spmm(const void *scores, const void *meta, const void *V, int BH, int Lq, int Lk, int LqR,
                               int LkR, int d, void *O, hipStream_t st);
// Dense O = P V with P bfloat16 [BH, Lq, Lk].
hipError_t launch_dense_av(const void *P, const void *V, int BH, int Lq, int Lk, int LqR, int LkR, int d, void *O,
                           hipStream_t st);
// Whole forward pass in one kernel.  mode: 0 = 2:4, 1 = 1:2, 2 = dense (full attention, Eq. 1).
// block_mask: uint8 [Lq/64][Lk/64] shared by all heads (zero = block not part of the attention), or nullptr.
// variant: a DFSS_VARIANT_* tiling (dfss_internal.h), 0 = chosen from the shape.
// The same for a padded batch given by its lengths: key_len int32 [BH / H] on the device (keys key_len[b] .. Lk - 1 of batch
// element b are padding); Lq a multiple of 64, Lk of 64; mode 0 or 1.
hipError_t launch_fused_attention_varlen(const void *Q, const void *K, const void *V, const int *key_len, int H, int BH,
                                         int Lq, int Lk, int d, int mode, float scale, void *O, hipStream_t st);
// The same with an additive mask fp32 [Lq][Lk] shared by all heads (any Lq; Lk a multiple of 4); mode 2 = full attention.
hipError_t launch_fused_attention_mask(const void *Q, const void *K, const void *V, const float *mask, int BH, int Lq,
                                       int Lk, int d, int mode, float scale, void *O, hipStream_t st);
hipError_t launch_fused_attention(const void *Q, const void *K, const void *V, const float *key_bias, int H,
                                  const uint8_t *block_mask, int causal, int BH, int Lq, int Lk, int d, int mode, float scale,
                                  void *O, int variant, hipStream_t st);
// The same with a block pattern (block_mask not null) and a workspace of fused_attention_split_workspace_bytes: row
// blocks that visit many blocks are shared between several workgroups and merged by a second kernel.
size_t fused_attention_split_workspace_bytes(int BH, int Lq, int d);
hipError_t launch_fused_attention_split_rows(const void *Q, const void *K, const void *V, const float *key_bias, int H,
                                             const uint8_t *block_mask, int BH, int Lq, int Lk, int d, int mode,
                                             float scale, void *O, void *part, hipStream_t st);
// Transposed sparse product out[BH, Lk, d] = A^T X for compressed A (vals + metadata) and X bf16 [BH, Lq, d]:
// dV = P^T dO and dK = dS^T Q of the backward pass.
hipError_t launch_spmm_t(const void *vals, const void *meta, const void *X, int BH, int Lq, int Lk, int LqR, int LkR,
                         int d, void *out, hipStream_t st);
// dS' = scale * P .* (dO V^T - delta) at the kept positions (delta_q = dO_q . O_q), compressed like P.
// K, dQ: both null, or (d = 64 only) the keys and the output of dQ = dS' K, formed in the same pass.
hipError_t launch_masked_sddmm_ds(const void *dO, const void *V, const void *O, const void *P, const void *meta,
                                  const void *K, int BH, int Lq, int Lk, int LqR, int LkR, int d, float scale, void *dS,
                                  void *dQ, hipStream_t st);
// The 4-byte mode (Sec. 2.3: float data, 1:2): fp32 Q, K, V, kept scores, weights and O; metadata = one
// 4-bit code per kept float, 32-bit words in the blocked order [BH, Lq/16, Lk/64, 16, 4].
hipError_t launch_sddmm_prune_f32(const void *Q, const void *K, const float *key_bias, int H, int BH, int Lq, int Lk,
                                  int d, float scale, void *vals, void *meta, hipStream_t st);
hipError_t launch_dense_scores_f32(const void *Q, const void *K, const float *key_bias, int H, int BH, int Lq, int Lk,
                                   int d, float scale, void *S, hipStream_t st);
hipError_t launch_row_softmax_f32(void *x, long rows, int cols, hipStream_t st);
hipError_t launch_spmm_f32(const void *vals, const void *meta, const void *V, int BH, int Lq, int Lk, int d, void *O,
                           hipStream_t st);
hipError_t launch_dense_av_f32(const void *P, const void *V, int BH, int Lq, int Lk, int d, void *O, hipStream_t st);
// The same four operations with every fp32 product formed from bfloat16 pieces on the bf16 matrix pipe
// (x = hi + lo; a.b ~ a_hi b_hi + a_hi b_lo + a_lo b_hi, fp32 accumulation); same layouts.
hipError_t launch_sddmm_prune_split(const void *Q, const void *K, const float *key_bias, int H, int BH, int Lq, int Lk,
                                    int d, float scale, void *vals, void *meta, hipStream_t st);
hipError_t launch_dense_scores_split(const void *Q, const void *K, const float *key_bias, int H, int BH, int Lq,
                                     int Lk, int d, float scale, void *S, hipStream_t st);
hipError_t launch_spmm_split(const void *vals, const void *meta, const void *V, int BH, int Lq, int Lk, int d,
                             void *O, hipStream_t st);
hipError_t launch_dense_av_split(const void *P, const void *V, int BH, int Lq, int Lk, int d, void *O,
                                 hipStream_t st);
// dS' = scale * P .* (dO V^T - delta) at the kept positions of the 4-byte mode (split products), compressed like P.
hipError_t launch_masked_sddmm_ds_split(const void *dO, const void *V, const void *O, const void *P, const void *meta,
                                        int BH, int Lq, int Lk, int d, float scale, void *dS, hipStream_t st);
// out[BH, Lk, d] = A^T X for A in the compressed form of the 4-byte mode, X fp32 [BH, Lq, d] (split products).
hipError_t launch_spmm_t_split(const void *vals, const void *meta, const void *X, int BH, int Lq, int Lk, int d,
                               void *out, hipStream_t st);
// Whole forward pass of the 4-byte mode in one kernel (split products).  prune = false: full attention.
// key_bias and block_mask (both may be null) as in launch_fused_attention.
hipError_t launch_fused_attention_split(const void *Q, const void *K, const void *V, const float *key_bias, int H,
                                        const uint8_t *block_mask, int BH, int Lq, int Lk, int d, bool prune,
                                        float scale, void *O, hipStream_t st);
// Metadata word order: library <-> canonical.  W = 32-bit words per row; permute: the 2-byte modes' order of
// the four words of a (row, block), false for the 4-byte mode.
hipError_t launch_meta_reorder(const void *src, void *dst, int BH, int Lq, int W, bool to_canonical, bool permute,
                               hipStream_t st);

}  // namespace dfss
