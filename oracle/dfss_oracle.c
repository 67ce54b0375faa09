/*
 * dfss_oracle.c -- CPU oracle for the DFSS attention forward pass.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It is a plain, slow,
 * obviously-correct restatement of what the method computes, used only by the
 * test-suite, the smoke check and the CPU-baseline leg of the benchmark.  It
 * shares no code, header, table or helper with the HIP library and the HIP
 * library never calls it.
 *
 * What it follows (arXiv 2203.00091):
 *   - full attention  O = softmax(Q K^T / sqrt(d)) V          Sec. 2.1, Eq. 1
 *   - dynamic N:M pruning of the *score* matrix, after Q K^T and before the
 *     softmax: in every aligned run of M consecutive keys of a row the N
 *     largest scores survive                                   Sec. 2.3, Sec. 3.1, App. A.1.1
 *   - compressed form = kept values in key order + per-selection 4-bit
 *     position code, four codes per 16-bit word, code k of a word at bits
 *     [4k, 4k+3]                                               Sec. 2.3, App. A.1.1, App. A.1.2
 *   - softmax over the kept entries only, max-subtracted      Sec. 3.1, App. A.1.3 (stable softmax)
 *   - compressed weights times V                               Sec. 3.1
 *   - L^p quality of a mask                                    Sec. 4.2, Def. 4.1
 *
 * Readings taken where the paper is silent (all listed in the design notes):
 *   - "larger" means larger signed value (softmax is monotone, Sec. 3.1);
 *   - equal scores: the lower key index wins;
 *   - the scale factor multiplies the fp32 dot product once, before any
 *     comparison, so the comparison sees exactly the value that is stored;
 *   - accumulation of the dot product is fp32, sequential in k (the paper
 *     accumulates in float regardless of input type, App. A.1.2);
 *   - masks are not in the paper: an optional per-key bias, and an optional
 *     per-(query, key) mask, are added to the scaled score in fp32 before
 *     the comparison (-inf masks an entry); the causal mask is the
 *     per-(query, key) mask that hides the keys after the query's own
 *     position, the queries being the LAST Lq positions of the Lk keys;
 *   - a block of the score matrix pruned by the block pattern (blocked-ELL,
 *     App. A.1.2) acts as if all its scores were -inf;
 *   - position code = lower kept position in bits [1:0], higher in bits [3:2];
 *     this is the unique 2-bit-per-position rule that reproduces the two
 *     codes the paper prints (0x4 for "first float", 0xe for "second float").
 *
 * Every function works on ONE head; oracle_attention_batched() loops heads.
 * Pinning of every function against something other than itself is in
 * tests/test_oracle_*.py.  No function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ */
/* Stage 1a: scores.  S[i][j] = scale * sum_k Q[i][k] * K[j][k]        */
/* Eq. 1 (the argument of the softmax); fp32, k ascending.             */
/* Q is [Lq][d], K is [Lk][d], S is [Lq][Lk], all row-major.           */
/* ------------------------------------------------------------------ */
void oracle_scores(const float *Q, const float *K, int Lq, int Lk, int d,
                   float scale, float *S)
{
    for (int i = 0; i < Lq; ++i) {
        for (int j = 0; j < Lk; ++j) {
            float acc = 0.0f;
            for (int k = 0; k < d; ++k)
                acc = acc + Q[(size_t)i * d + k] * K[(size_t)j * d + k];
            S[(size_t)i * Lk + j] = acc * scale;
        }
    }
}

/* ------------------------------------------------------------------ */
/* Stage 1a': additive key bias (padding mask).                        */
/* The paper never mentions masks; real inputs (padded batches) need   */
/* one, so the reading taken is the usual one for Eq. 1: a per-key     */
/* term is ADDED to the scaled score in fp32, BEFORE the N:M           */
/* comparison (so that a masked key loses against any unmasked one of  */
/* its group), S[i][j] <- S[i][j] + bias[j].  bias[j] = -inf masks key */
/* j; a group whose keys are all masked still emits N entries, which   */
/* the softmax then weights with exactly 0.  bias is [Lk].             */
/* ------------------------------------------------------------------ */
void oracle_add_key_bias(float *S, int Lq, int Lk, const float *bias)
{
    for (int i = 0; i < Lq; ++i)
        for (int j = 0; j < Lk; ++j)
            S[(size_t)i * Lk + j] = S[(size_t)i * Lk + j] + bias[j];
}

/* ------------------------------------------------------------------ */
/* Stage 1a': general additive mask, one term per (query, key):        */
/* S[i][j] <- S[i][j] + mask[i][j], fp32, BEFORE the N:M comparison    */
/* (same reading as the key bias: what the comparison sees is what the */
/* softmax sees).  mask is [Lq][Lk], shared by all heads; -inf hides   */
/* key j from query i.                                                 */
/* ------------------------------------------------------------------ */
void oracle_add_mask(float *S, int Lq, int Lk, const float *mask)
{
    for (int i = 0; i < Lq; ++i)
        for (int j = 0; j < Lk; ++j)
            S[(size_t)i * Lk + j] = S[(size_t)i * Lk + j] + mask[(size_t)i * Lk + j];
}

/* The causal mask (decoder self-attention: the paper finetunes and    */
/* evaluates encoders only, Sec. 5.1; a position must not see later    */
/* ones) written out as such a mask.  Reading taken for Lq != Lk: the  */
/* queries are the last Lq of the Lk positions, so query i sits at     */
/* position i + (Lk - Lq) and sees keys 0 .. i + (Lk - Lq).  Needs     */
/* Lk >= Lq (every query then sees at least one key).  mask[i][j] = 0  */
/* for a visible key, -inf for a hidden one.                           */
int oracle_causal_mask(int Lq, int Lk, float *mask)
{
    if (Lq <= 0 || Lk < Lq) return -1;
    const int off = Lk - Lq;
    for (int i = 0; i < Lq; ++i)
        for (int j = 0; j < Lk; ++j)
            mask[(size_t)i * Lk + j] = j <= i + off ? 0.0f : -INFINITY;
    return 0;
}

/* ------------------------------------------------------------------ */
/* Stage 1a'': block mask (hybrid blocked-ELL x N:M sparsity,          */
/* App. A.1.2 "Blocked-ELL Sparsity": blocks of the score matrix that  */
/* the block pattern prunes are simply not computed).  As a function:  */
/* every score of a pruned block is -inf, i.e. it loses every          */
/* comparison and gets softmax weight 0.  block_mask is                */
/* [Lq/bs][Lk/bs], non-zero = the block is kept.                       */
/* ------------------------------------------------------------------ */
int oracle_apply_block_mask(float *S, int Lq, int Lk, const uint8_t *block_mask, int bs)
{
    if (bs <= 0 || Lq % bs != 0 || Lk % bs != 0) return -1;
    const int nbk = Lk / bs;
    for (int i = 0; i < Lq; ++i)
        for (int j = 0; j < Lk; ++j)
            if (!block_mask[(size_t)(i / bs) * nbk + j / bs]) S[(size_t)i * Lk + j] = -INFINITY;
    return 0;
}

/* ------------------------------------------------------------------ */
/* Stage 1b: N:M selection (Sec. 2.3, App. A.1.1).                     */
/* Groups are aligned runs of M consecutive keys starting at key 0.    */
/* rank(t) = #{u : S_u > S_t} + #{u < t : S_u == S_t}; keep iff        */
/* rank(t) < N.  Outputs, per row i:                                   */
/*   mask[i][j]           1 if score (i,j) is kept, else 0             */
/*   vals[i][g*N + r]     r-th kept score of group g, key ascending    */
/*   kidx[i][g*N + r]     its key index j                              */
/* Lk must be a multiple of M.  Returns 0, or -1 on bad arguments.     */
/* ------------------------------------------------------------------ */
int oracle_prune(const float *S, int Lq, int Lk, int N, int M,
                 uint8_t *mask, float *vals, int32_t *kidx)
{
    if (M <= 0 || N <= 0 || N > M || Lk % M != 0) return -1;
    const int G = Lk / M;
    const int Lc = G * N;
    for (int i = 0; i < Lq; ++i) {
        const float *row = S + (size_t)i * Lk;
        for (int g = 0; g < G; ++g) {
            int r = 0;
            for (int t = 0; t < M; ++t) {
                const float st = row[g * M + t];
                int rank = 0;
                for (int u = 0; u < M; ++u) {
                    const float su = row[g * M + u];
                    if (su > st) rank++;
                    else if (u < t && su == st) rank++;
                }
                const int keep = rank < N;
                mask[(size_t)i * Lk + g * M + t] = (uint8_t)keep;
                if (keep) {
                    vals[(size_t)i * Lc + g * N + r] = st;
                    kidx[(size_t)i * Lc + g * N + r] = g * M + t;
                    r++;
                }
            }
            /* a total order always yields exactly N survivors */
            if (r != N) return -2;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Metadata (Sec. 2.3: 4 bits per 1:2 / 2:4 selection; App. A.1.1;     */
/* packing of four codes into a 16-bit word: App. A.1.2).              */
/* One code describes one run of 4 keys, of which exactly 2 survive:   */
/*   2:4 -> the run is one group;  1:2 -> the run is two groups.       */
/* code = p_lo | (p_hi << 2), p = key index mod 4, p_lo < p_hi.        */
/* Word w of a row holds the codes of runs 4w..4w+3, run 4w+k at bits  */
/* [4k, 4k+3].  meta is [Lq][Lk/16] uint16.  Lk % 16 == 0 required.    */
/* ------------------------------------------------------------------ */
int oracle_encode_meta(const int32_t *kidx, int Lq, int Lk, uint16_t *meta)
{
    if (Lk % 16 != 0) return -1;
    const int Lc = Lk / 2;
    const int W = Lk / 16;
    for (int i = 0; i < Lq; ++i) {
        for (int w = 0; w < W; ++w) {
            unsigned word = 0;
            for (int k = 0; k < 4; ++k) {
                const int run = 4 * w + k;          /* keys 4run .. 4run+3 */
                const int j0 = kidx[(size_t)i * Lc + 2 * run + 0];
                const int j1 = kidx[(size_t)i * Lc + 2 * run + 1];
                if (j0 / 4 != run || j1 / 4 != run || j0 >= j1) return -2;
                const unsigned code = (unsigned)(j0 % 4) | ((unsigned)(j1 % 4) << 2);
                word |= code << (4 * k);
            }
            meta[(size_t)i * W + w] = (uint16_t)word;
        }
    }
    return 0;
}

int oracle_decode_meta(const uint16_t *meta, int Lq, int Lk, int32_t *kidx)
{
    if (Lk % 16 != 0) return -1;
    const int Lc = Lk / 2;
    const int W = Lk / 16;
    for (int i = 0; i < Lq; ++i) {
        for (int w = 0; w < W; ++w) {
            const unsigned word = meta[(size_t)i * W + w];
            for (int k = 0; k < 4; ++k) {
                const unsigned code = (word >> (4 * k)) & 0xFu;
                const int run = 4 * w + k;
                kidx[(size_t)i * Lc + 2 * run + 0] = 4 * run + (int)(code & 3u);
                kidx[(size_t)i * Lc + 2 * run + 1] = 4 * run + (int)((code >> 2) & 3u);
            }
        }
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Metadata of the 4-byte mode (1:2 on float data, Sec. 2.3; App.      */
/* A.1.1).  A code still describes a run of four 2-byte slots, two of  */
/* which survive; a 4-byte element fills two consecutive slots, so a   */
/* run is one aligned pair of keys and element e of the pair covers    */
/* slots 2e and 2e+1.  code = p_lo | (p_hi << 2) over slot positions,  */
/* exactly as in the 2-byte mode.  Word w of a row holds the codes of  */
/* pairs 4w..4w+3, pair 4w+k at bits [4k, 4k+3] (App. A.1.2).          */
/* kidx is [Lq][Lk/2] (one kept key per pair), meta [Lq][Lk/8] uint16. */
/* Lk % 8 == 0 required.                                               */
/* ------------------------------------------------------------------ */
int oracle_encode_meta_f32(const int32_t *kidx, int Lq, int Lk, uint16_t *meta)
{
    if (Lk % 8 != 0) return -1;
    const int Lc = Lk / 2;
    const int W = Lk / 8;
    for (int i = 0; i < Lq; ++i) {
        for (int w = 0; w < W; ++w) {
            unsigned word = 0;
            for (int k = 0; k < 4; ++k) {
                const int pair = 4 * w + k;         /* keys 2pair, 2pair+1 */
                const int j = kidx[(size_t)i * Lc + pair];
                if (j / 2 != pair) return -2;
                const unsigned e = (unsigned)(j % 2);
                const unsigned slot_lo = 2u * e, slot_hi = 2u * e + 1u;
                const unsigned code = slot_lo | (slot_hi << 2);
                word |= code << (4 * k);
            }
            meta[(size_t)i * W + w] = (uint16_t)word;
        }
    }
    return 0;
}

/* Inverse; returns -2 if a code does not name two consecutive slots of one element. */
int oracle_decode_meta_f32(const uint16_t *meta, int Lq, int Lk, int32_t *kidx)
{
    if (Lk % 8 != 0) return -1;
    const int Lc = Lk / 2;
    const int W = Lk / 8;
    for (int i = 0; i < Lq; ++i) {
        for (int w = 0; w < W; ++w) {
            const unsigned word = meta[(size_t)i * W + w];
            for (int k = 0; k < 4; ++k) {
                const unsigned code = (word >> (4 * k)) & 0xFu;
                const unsigned slot_lo = code & 3u, slot_hi = (code >> 2) & 3u;
                if ((slot_lo & 1u) != 0u || slot_hi != slot_lo + 1u) return -2;
                const int pair = 4 * w + k;
                kidx[(size_t)i * Lc + pair] = 2 * pair + (int)(slot_lo >> 1);
            }
        }
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Stage 2: softmax over the kept entries of each row                  */
/* (Sec. 3.1; max-subtracted form of App. A.1.3).                      */
/* x, P are [Lq][Lc].  The sum is carried in double so the oracle's    */
/* own rounding stays far below any tolerance used against it.         */
/* ------------------------------------------------------------------ */
void oracle_softmax_kept(const float *x, int Lq, int Lc, float *P)
{
    for (int i = 0; i < Lq; ++i) {
        const float *xi = x + (size_t)i * Lc;
        float *pi = P + (size_t)i * Lc;
        float c = xi[0];
        for (int j = 1; j < Lc; ++j)
            if (xi[j] > c) c = xi[j];
        double s = 0.0;
        for (int j = 0; j < Lc; ++j)
            s += exp((double)xi[j] - (double)c);
        for (int j = 0; j < Lc; ++j)
            pi[j] = (float)(exp((double)xi[j] - (double)c) / s);
    }
}

/* ------------------------------------------------------------------ */
/* Stage 3: compressed weights times V (Sec. 3.1).                     */
/* O[i][:] = sum over kept entries c (ascending) P[i][c] * V[kidx[i][c]][:]. */
/* V is [Lk][d]; O is [Lq][d]; double accumulation.                    */
/* ------------------------------------------------------------------ */
void oracle_spmm(const float *P, const int32_t *kidx, const float *V,
                 int Lq, int Lc, int d, float *O)
{
    double *acc = (double *)malloc(sizeof(double) * (size_t)d);
    for (int i = 0; i < Lq; ++i) {
        for (int k = 0; k < d; ++k) acc[k] = 0.0;
        for (int c = 0; c < Lc; ++c) {
            const double p = (double)P[(size_t)i * Lc + c];
            const float *v = V + (size_t)kidx[(size_t)i * Lc + c] * d;
            for (int k = 0; k < d; ++k) acc[k] += p * (double)v[k];
        }
        for (int k = 0; k < d; ++k) O[(size_t)i * d + k] = (float)acc[k];
    }
    free(acc);
}

/* ------------------------------------------------------------------ */
/* bfloat16 storage rounding: round-to-nearest-even of the top 16 bits */
/* of an IEEE binary32 (finite inputs).  Used only to model the 2-byte */
/* storage of the compressed scores / weights (App. A.1.1: 2-byte      */
/* non-zeros in bfloat16 mode).                                        */
/* ------------------------------------------------------------------ */
float oracle_round_bf16(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    if ((u & 0x7F800000u) == 0x7F800000u) return x; /* inf / nan untouched */
    const uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    u &= 0xFFFF0000u;
    float y;
    memcpy(&y, &u, 4);
    return y;
}

void oracle_round_bf16_array(const float *x, size_t n, float *y)
{
    for (size_t i = 0; i < n; ++i) y[i] = oracle_round_bf16(x[i]);
}

/* ------------------------------------------------------------------ */
/* Whole forward pass for one head.                                    */
/*   store_bf16 = 0 : everything stays fp32 between stages (the pure   */
/*                    mathematical function);                          */
/*   store_bf16 = 1 : the kept scores and the weights are rounded to   */
/*                    bfloat16 where the method stores them in 2 bytes. */
/* Optional outputs (may be NULL): mask, vals (after optional rounding,*/
/* before softmax), kidx, P.                                           */
/* ------------------------------------------------------------------ */
int oracle_attention_masked(const float *Q, const float *K, const float *V, const float *key_bias,
                            const float *mask2d, const uint8_t *block_mask, int block_size,
                            int Lq, int Lk, int d, int N, int M, float scale,
                            int store_bf16, float *O,
                            uint8_t *mask_out, float *vals_out, int32_t *kidx_out, float *P_out)
{
    if (M <= 0 || N <= 0 || N > M || Lk % M != 0) return -1;
    const int Lc = Lk / M * N;
    float *S = (float *)malloc(sizeof(float) * (size_t)Lq * Lk);
    uint8_t *mask = (uint8_t *)malloc((size_t)Lq * Lk);
    float *vals = (float *)malloc(sizeof(float) * (size_t)Lq * Lc);
    int32_t *kidx = (int32_t *)malloc(sizeof(int32_t) * (size_t)Lq * Lc);
    float *P = (float *)malloc(sizeof(float) * (size_t)Lq * Lc);
    int rc = -3;
    if (S && mask && vals && kidx && P) {
        oracle_scores(Q, K, Lq, Lk, d, scale, S);
        if (key_bias) oracle_add_key_bias(S, Lq, Lk, key_bias);   /* NULL = no mask (the paper's case) */
        if (mask2d) oracle_add_mask(S, Lq, Lk, mask2d);
        rc = block_mask ? oracle_apply_block_mask(S, Lq, Lk, block_mask, block_size) : 0;
        if (rc == 0) rc = oracle_prune(S, Lq, Lk, N, M, mask, vals, kidx);
        if (rc == 0) {
            if (store_bf16) oracle_round_bf16_array(vals, (size_t)Lq * Lc, vals);
            oracle_softmax_kept(vals, Lq, Lc, P);
            if (store_bf16) oracle_round_bf16_array(P, (size_t)Lq * Lc, P);
            oracle_spmm(P, kidx, V, Lq, Lc, d, O);
            if (mask_out) memcpy(mask_out, mask, (size_t)Lq * Lk);
            if (vals_out) memcpy(vals_out, vals, sizeof(float) * (size_t)Lq * Lc);
            if (kidx_out) memcpy(kidx_out, kidx, sizeof(int32_t) * (size_t)Lq * Lc);
            if (P_out) memcpy(P_out, P, sizeof(float) * (size_t)Lq * Lc);
        }
    }
    free(S); free(mask); free(vals); free(kidx); free(P);
    return rc;
}

int oracle_attention_bias(const float *Q, const float *K, const float *V, const float *key_bias,
                          int Lq, int Lk, int d, int N, int M, float scale,
                          int store_bf16, float *O,
                          uint8_t *mask_out, float *vals_out, int32_t *kidx_out, float *P_out)
{
    return oracle_attention_masked(Q, K, V, key_bias, NULL, NULL, 0, Lq, Lk, d, N, M, scale, store_bf16, O,
                                   mask_out, vals_out, kidx_out, P_out);
}

int oracle_attention(const float *Q, const float *K, const float *V,
                     int Lq, int Lk, int d, int N, int M, float scale,
                     int store_bf16, float *O,
                     uint8_t *mask_out, float *vals_out, int32_t *kidx_out, float *P_out)
{
    return oracle_attention_masked(Q, K, V, NULL, NULL, NULL, 0, Lq, Lk, d, N, M, scale, store_bf16, O,
                                   mask_out, vals_out, kidx_out, P_out);
}

/* Heads are independent (App. A.1.2, batched kernel): loop them, in parallel
 * over host threads when built with OpenMP.  Q,K,V,O are [BH][L][d]. */
/* key_bias (may be NULL) is [BH / heads_per_batch][Lk]: the heads of one batch element share
 * one bias vector (a padding mask belongs to the sequence, not to the head).  mask2d (may be NULL) is
 * [Lq][Lk], shared by all heads. */
int oracle_attention_masked_batched(const float *Q, const float *K, const float *V, const float *key_bias,
                                    int heads_per_batch, const float *mask2d,
                                    const uint8_t *block_mask, int block_size,
                                    int BH, int Lq, int Lk, int d, int N, int M,
                                    float scale, int store_bf16, float *O)
{
    int bad = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1)
#endif
    for (int h = 0; h < BH; ++h) {
        const float *bias = key_bias ? key_bias + (size_t)(h / heads_per_batch) * Lk : NULL;
        int rc = oracle_attention_masked(Q + (size_t)h * Lq * d, K + (size_t)h * Lk * d,
                                         V + (size_t)h * Lk * d, bias, mask2d, block_mask, block_size,
                                         Lq, Lk, d, N, M, scale,
                                         store_bf16, O + (size_t)h * Lq * d,
                                         NULL, NULL, NULL, NULL);
        if (rc != 0) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            bad = rc;
        }
    }
    return bad;
}

int oracle_attention_bias_batched(const float *Q, const float *K, const float *V, const float *key_bias,
                                  int heads_per_batch, int BH, int Lq, int Lk, int d, int N, int M,
                                  float scale, int store_bf16, float *O)
{
    return oracle_attention_masked_batched(Q, K, V, key_bias, heads_per_batch, NULL, NULL, 0, BH, Lq, Lk, d, N, M,
                                           scale, store_bf16, O);
}

int oracle_attention_batched(const float *Q, const float *K, const float *V,
                             int BH, int Lq, int Lk, int d, int N, int M,
                             float scale, int store_bf16, float *O)
{
    return oracle_attention_masked_batched(Q, K, V, NULL, 1, NULL, NULL, 0, BH, Lq, Lk, d, N, M, scale, store_bf16, O);
}

/* ------------------------------------------------------------------ */
/* Backward pass of one head through the FIXED selection of the        */
/* forward pass (the paper finetunes with DFSS attention, Sec. 5.1,    */
/* but does not describe a backward kernel; the reading taken is the   */
/* usual one for pruning masks: the selection is a constant of the     */
/* step, gradients flow through the kept entries only).  With          */
/*   S = scale Q K^T (+ bias), kept set and P = softmax over the kept  */
/*   entries, O = P V   (Sec. 3.1)                                     */
/* the chain rule gives, for an upstream gradient dO:                  */
/*   dV[j]   = sum_i P[i][j] dO[i]                                      */
/*   dP[i][j] = dO[i] . V[j]                  (kept j only)             */
/*   delta_i = sum_j P[i][j] dP[i][j]                                   */
/*   dS[i][j] = P[i][j] (dP[i][j] - delta_i)                            */
/*   dQ[i]   = scale sum_j dS[i][j] K[j],  dK[j] = scale sum_i dS[i][j] Q[i] */
/* All sums in double.  P (the weights, [Lq][Lc]) and kidx come from   */
/* the forward pass; dS_out (may be NULL) receives dS, [Lq][Lc].       */
/* ------------------------------------------------------------------ */
void oracle_attention_backward(const float *Q, const float *K, const float *V, const float *dO,
                               const float *P, const int32_t *kidx,
                               int Lq, int Lk, int Lc, int d, float scale,
                               float *dQ, float *dK, float *dV, float *dS_out)
{
    double *aQ = (double *)calloc((size_t)Lq * d, sizeof(double));
    double *aK = (double *)calloc((size_t)Lk * d, sizeof(double));
    double *aV = (double *)calloc((size_t)Lk * d, sizeof(double));
    double *dP = (double *)malloc(sizeof(double) * (size_t)Lc);
    for (int i = 0; i < Lq; ++i) {
        const float *doi = dO + (size_t)i * d;
        double delta = 0.0;
        for (int c = 0; c < Lc; ++c) {
            const float *v = V + (size_t)kidx[(size_t)i * Lc + c] * d;
            double acc = 0.0;
            for (int k = 0; k < d; ++k) acc += (double)doi[k] * (double)v[k];
            dP[c] = acc;
            delta += (double)P[(size_t)i * Lc + c] * acc;
        }
        for (int c = 0; c < Lc; ++c) {
            const int j = kidx[(size_t)i * Lc + c];
            const double p = (double)P[(size_t)i * Lc + c];
            const double ds = p * (dP[c] - delta);
            if (dS_out) dS_out[(size_t)i * Lc + c] = (float)ds;
            for (int k = 0; k < d; ++k) {
                aV[(size_t)j * d + k] += p * (double)doi[k];
                aQ[(size_t)i * d + k] += (double)scale * ds * (double)K[(size_t)j * d + k];
                aK[(size_t)j * d + k] += (double)scale * ds * (double)Q[(size_t)i * d + k];
            }
        }
    }
    for (size_t t = 0; t < (size_t)Lq * d; ++t) dQ[t] = (float)aQ[t];
    for (size_t t = 0; t < (size_t)Lk * d; ++t) { dK[t] = (float)aK[t]; dV[t] = (float)aV[t]; }
    free(aQ); free(aK); free(aV); free(dP);
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* L^p quality of a mask (Sec. 4.2, Def. 4.1):                         */
/*   Q^p = (1/n) sum_rows [ sum_i (m .* A)^p / sum_i A^p ],            */
/* A = row softmax of the score matrix S.  Since A_ji is proportional  */
/* to exp(S_ji) within a row, the row term equals                      */
/*   sum_kept exp(p (S - max)) / sum_all exp(p (S - max)).             */
/* ------------------------------------------------------------------ */
double oracle_quality_p(const float *S, const uint8_t *mask, int Lq, int Lk, double p)
{
    double total = 0.0;
    for (int i = 0; i < Lq; ++i) {
        const float *row = S + (size_t)i * Lk;
        float c = row[0];
        for (int j = 1; j < Lk; ++j)
            if (row[j] > c) c = row[j];
        double num = 0.0, den = 0.0;
        for (int j = 0; j < Lk; ++j) {
            const double e = exp(p * ((double)row[j] - (double)c));
            den += e;
            if (mask[(size_t)i * Lk + j]) num += e;
        }
        total += num / den;
    }
    return total / (double)Lq;
}
