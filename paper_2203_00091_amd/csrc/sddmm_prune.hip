// Stage 1 of the DFSS forward pass: S = scale * Q K^T on bf16 MFMA with the N:M pruning
// done on the accumulators, so the dense score matrix never reaches memory
// (arXiv 2203.00091, Sec. 3.4 and App. A.1.2).  The same mainloop with a plain
// bfloat16 store is the first stage of the dense baseline (Eq. 1).
//
// Orientation.  The product is formed transposed (keys on the MFMA rows, queries on its
// columns) because a lane owns four consecutive ROWS of one column of the 16x16 result:
// with keys on the rows a lane owns runs of four consecutive keys of one query, which is
// what the selection needs -- no cross-lane traffic.  (App. A.1.2 reaches the same end on
// its hardware by interleaving the columns of one operand.)
//
// Streaming.  A workgroup (4 waves) owns 64*NQ queries; each wave keeps the Q operand of
// its 16*NQ queries in registers for the whole kernel and walks over blocks of 128 keys.
// K blocks are copied global -> LDS by the direct-to-LDS load (no register round trip),
// double buffered, XOR-swizzled so the 16-byte operand reads are conflict free.
//
// Key order inside a 128-key block.  LDS row slot 16*t + i (tile t = 0..7, MFMA row i)
// holds key 32*(i/4) + 4*t + i%4.  After tiles 0..3 lane (column c, row group g) holds the
// 16 consecutive keys 32g .. 32g+15 of query c, after tiles 4..7 the next 16: per
// 128-key block a lane emits 32 contiguous bytes of kept values and one 32-bit word of
// metadata (two canonical 16-bit words), and a row receives 128 contiguous bytes.
#include <stdlib.h>

#include "dfss_device.hpp"
#include "dfss_kernels.hpp"

namespace dfss {

namespace {

constexpr int NT = 256;   // threads per workgroup
constexpr int KB = 128;   // keys per block

enum { MODE_2TO4 = 0, MODE_1TO2 = 1, MODE_DENSE = 2 };

// PRESCALE: the scale is a power of two and is applied (exactly) to the Q operand once,
// instead of to every accumulator.
// BIAS: an additive per-key term (fp32 [B][Lk], shared by the H heads of a batch element; -inf masks a
// key) joins the scaled score before the selection: as the initial value of the accumulators when the
// scale is folded into Q, else added (as a separate fp32 addition) after the multiplication by scale.
// CAUSAL: query i sees keys 0 .. i + (Lk - Lq); the scores of the hidden keys are overwritten with
// -inf before the selection, by index, in the blocks that reach past the diagonal of the wave's first query
// (every block is still computed and written: the hidden entries are part of the compressed matrix).
template <int D, int MODE, int NQ, bool PRESCALE, bool BIAS, bool CAUSAL>
__global__ __launch_bounds__(NT, 2) void k_sddmm(const __bf16 *__restrict__ Q, const __bf16 *__restrict__ K,
                                                 const float *__restrict__ key_bias, int H,
                                                 int Lq, int Lk, float scale, int ksplit, int blocks_per_wg,
                                                 uint32_t *__restrict__ out, uint32_t *__restrict__ meta) {
    constexpr int CPR = D / 8;           // 16-byte chunks per row
    constexpr int TILE = KB * CPR;       // chunks per K block
    constexpr int LPT = TILE / NT;       // direct-to-LDS loads per thread per block
    constexpr int STEPS = D / 32;        // MFMA k-steps
    constexpr int TQ = 64 * NQ;          // queries per workgroup
    __shared__ u32x4 Ks[2][TILE];
    __shared__ f32x4 Bs[BIAS ? 2 : 1][KB / 4];   // bias of the block's 128 keys, copied along with K

    const int tid = threadIdx.x;
    const int w = tid >> 6, l = tid & 63, li = l & 15, kb = l >> 4;

    // work item -> (head, query tile, key range)
    const unsigned qtiles = Lq / TQ;
    const unsigned item = xcd_contiguous(blockIdx.x, gridDim.x);
    const int ks_id = item % ksplit;
    const int qt = (item / ksplit) % qtiles;
    const int bh = item / (ksplit * qtiles);
    const int jb0 = ks_id * blocks_per_wg;
    const int q0 = qt * TQ + w * 16 * NQ;

    const __bf16 *Kh = K + (size_t)bh * Lk * D;

    // per-thread source offsets of the direct-to-LDS copies: LDS position p (16-byte units)
    // = slot * CPR + (c ^ (slot & 7)) holds chunk c of the key stored in row slot `slot`
    int src_off[LPT];
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
        const int p = i * NT + tid;
        const int slot = p / CPR, c = (p % CPR) ^ (slot & 7);
        const int key = (slot & 3) | (((slot >> 4) & 7) << 2) | (((slot >> 2) & 3) << 5);
        src_off[i] = key * D + c * 8;
    }
    const uint32_t lds_k = lds_address(&Ks[0][w * 64]);   // this wave's 1 KB slice of copy 0, buffer 0
    const float *bias_b = BIAS ? key_bias + (size_t)(bh / H) * Lk : nullptr;
    const uint32_t lds_b = lds_address(&Bs[0][0]);
    auto issue_block = [&](int jb, int buf) {
        const __bf16 *src = Kh + (size_t)jb * KB * D;
#pragma unroll
        for (int i = 0; i < LPT; ++i) async_copy16(src, 2u * src_off[i], lds_k + 16u * (buf * TILE + i * NT));
        if constexpr (BIAS) {   // 512 bytes: lanes 0..31 of wave 0 (the copy lands through the same counter as K)
            if (tid < KB / 4) async_copy16(bias_b + (size_t)jb * KB, 16u * tid, lds_b + (uint32_t)(buf * KB * 4));
        }
    };

    // Order of the blocks: workgroup g starts g blocks into its range and wraps around (the blocks of stage 1 do not
    // depend on one another).  Rows of the compressed matrix are a power of two apart for the usual lengths: workgroups
    // marching from their first block in step would all write the same few memory channels at a time.
    const int rot = __builtin_amdgcn_readfirstlane((int)(item % (unsigned)blocks_per_wg));
    auto blk = [&](int it) { return jb0 + (it + rot < blocks_per_wg ? it + rot : it + rot - blocks_per_wg); };
    issue_block(blk(0), 0);

    // Q operand: lane (column li, chunk kb) of MFMA step s holds Q[q][32 s + 8 kb .. +7]
    bf16x8 bq[NQ][STEPS];
#pragma unroll
    for (int qs = 0; qs < NQ; ++qs)
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            const u32x4 raw = *reinterpret_cast<const u32x4 *>(Q + ((size_t)bh * Lq + q0 + 16 * qs + li) * D +
                                                               32 * s + 8 * kb);
            if constexpr (PRESCALE) {
                u32x4 sc;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    sc[e] = pack_bf16x2(bf16_lo_to_f32(raw[e]) * scale, bf16_hi_to_f32(raw[e]) * scale);
                bq[qs][s] = __builtin_bit_cast(bf16x8, sc);
            } else {
                bq[qs][s] = __builtin_bit_cast(bf16x8, raw);
            }
        }

    const int rb0 = q0 >> 4;                 // first 16-row block of this wave

    for (int it = 0; it < blocks_per_wg; ++it) {
        const int jb = blk(it);
        const int buf = it & 1;
        // this block's copies (issued one iteration ago) have landed for every wave; the stores of
        // the previous iteration, issued after those copies, stay in flight
        constexpr int kStoresPerBlock = MODE == MODE_DENSE ? 4 * NQ : 3 * NQ;
        if (it == 0) wait_async_copies();
        else wait_async_copies_keep<kStoresPerBlock>();
        __syncthreads();
        // every wave has also finished reading the other buffer: refill it
        if (it + 1 < blocks_per_wg) issue_block(blk(it + 1), buf ^ 1);

        uint32_t mword[NQ];
#pragma unroll
        for (int qs = 0; qs < NQ; ++qs) mword[qs] = 0;

        u32x4 kept_out[2][NQ];   // kept values of both halves: a lane's 32 contiguous bytes, stored together
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            f32x4 acc[NQ][4];
            f32x4 kb4[4];    // bias of keys 128 jb + 32 kb + 16 half + 4 t + r
            if constexpr (BIAS) {
#pragma unroll
                for (int t = 0; t < 4; ++t) kb4[t] = Bs[buf][8 * kb + 4 * half + t];
            }
#pragma unroll
            for (int qs = 0; qs < NQ; ++qs)
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    if constexpr (BIAS && PRESCALE) acc[qs][t] = kb4[t];
                    else acc[qs][t] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                bf16x8 ak[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int slot = 16 * (4 * half + t) + li;
                    ak[t] = __builtin_bit_cast(bf16x8, Ks[buf][slot * CPR + ((4 * s + kb) ^ (li & 7))]);
                }
#pragma unroll
                for (int qs = 0; qs < NQ; ++qs)
#pragma unroll
                    for (int t = 0; t < 4; ++t) acc[qs][t] = mfma16(ak[t], bq[qs][s], acc[qs][t]);
            }
            // acc[qs][t][r] = score of query q0 + 16 qs + li and key 128 jb + 32 kb + 16 half + 4 t + r
            const int kbase = KB * jb + 32 * kb + 16 * half;
            // causal: hidden scores become -inf on the raw accumulators (the scaling and the bias leave -inf as it is).
            // q0 is the same in every lane of the wave; as a scalar, the test is one branch around the masking.
            if (CAUSAL && KB * jb + KB - 1 > __builtin_amdgcn_readfirstlane(q0) + Lk - Lq) {
                asm volatile("" ::: "memory");   // (not to be turned into selects that every block would execute)
#pragma unroll
                for (int qs = 0; qs < NQ; ++qs) {
                    const int lim = q0 + 16 * qs + li + Lk - Lq - kbase;   // key offsets above it are hidden
#pragma unroll
                    for (int t = 0; t < 4; ++t)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            if (4 * t + r > lim) acc[qs][t][r] = -INFINITY;
                }
            }
#pragma unroll
            for (int qs = 0; qs < NQ; ++qs) {
                const size_t row = (size_t)bh * Lq + q0 + 16 * qs + li;
                if constexpr (MODE == MODE_DENSE) {
                    uint32_t p[8];
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        f32x4 a = acc[qs][t];
                        if constexpr (!PRESCALE) {
                            a = a * scale;
                            if constexpr (BIAS) {
#pragma unroll
                                for (int r = 0; r < 4; ++r) a[r] = add_unfused(a[r], kb4[t][r]);
                            }
                        }
                        p[2 * t] = pack_bf16x2(a[0], a[1]);
                        p[2 * t + 1] = pack_bf16x2(a[2], a[3]);
                    }
                    u32x4 *dst = reinterpret_cast<u32x4 *>(out + (row * Lk + kbase) / 2);
                    dst[0] = u32x4{p[0], p[1], p[2], p[3]};
                    dst[1] = u32x4{p[4], p[5], p[6], p[7]};
                } else {
                    u32x4 pk;
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        f32x4 a = acc[qs][t];
                        if constexpr (!PRESCALE) {
                            a = a * scale;
                            if constexpr (BIAS) {
#pragma unroll
                                for (int r = 0; r < 4; ++r) a[r] = add_unfused(a[r], kb4[t][r]);
                            }
                        }
                        float lo, hi;
                        uint32_t code;
                        if constexpr (MODE == MODE_2TO4)
                            select_2of4(a[0], a[1], a[2], a[3], 16 * half + 4 * t, lo, hi, code);
                        else
                            select_1of2(a[0], a[1], a[2], a[3], 16 * half + 4 * t, lo, hi, code);
                        pk[t] = pack_bf16x2(lo, hi);
                        mword[qs] |= code;
                    }
                    kept_out[half][qs] = pk;
                }
            }
        }
        if constexpr (MODE != MODE_DENSE) {
            // the two halves of a lane are adjacent in memory (keys 32 kb .. +31 of the row): issued back to back,
            // the four lanes of a row complete a whole 128-byte line
#pragma unroll
            for (int qs = 0; qs < NQ; ++qs) {
                const size_t row = (size_t)bh * Lq + q0 + 16 * qs + li;
                u32x4 *dst = reinterpret_cast<u32x4 *>(out + (row * (size_t)(Lk / 2) + (KB * jb + 32 * kb) / 2) / 2);
                dst[0] = kept_out[0][qs];
                dst[1] = kept_out[1][qs];
            }
#pragma unroll
            for (int qs = 0; qs < NQ; ++qs)
                meta[((((size_t)bh * (Lq / 16) + rb0 + qs) * (Lk / KB) + jb) * 16 + li) * 4 + (((kb & 1) << 1) | (kb >> 1))] =
                    mword[qs];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// 32-query variant.  Same method, but the scores are formed with v_mfma_f32_32x32x16_bf16, which
// on gfx950 has twice the flops per cycle of the 16x16x32 form (both take 32 cycles per SIMD).
// A wave owns 32 queries; lane l holds query l%32 and, per 32-key tile, the 16 registers
// 4g + x are MFMA rows 8g + 4h + x (h = l/32).  LDS row slot 32 t + i (tile t of a 128-key block,
// MFMA row i = 8g + 4h' + x) holds key 64 (t/2) + 32 h' + 16 (t%2) + 4 g + x, so that over a PAIR
// of tiles lane (query, h) owns the 32 consecutive keys 64 p + 32 h .. +31: 32 contiguous bytes of
// kept values and one 32-bit metadata word, exactly the units of the 16-query kernel.
// ---------------------------------------------------------------------------------------------
typedef float f32x16 __attribute__((ext_vector_type(16)));

// KMASK: 0 = none; 1 = causal (as above); 2 = unpadded lengths: Q holds LqR <= Lq rows per head and K (and key_bias)
// LkR <= Lk keys, while the outputs keep the layout of the padded lengths Lq (a multiple of 64) and Lk (of 128).
// The keys LkR .. Lk - 1 do not exist: their scores count as -inf, overwritten by index like the causal ones; their
// places in a partial last block are filled with the block's last real key, and rows past LqR are computed on a copy
// of the last query (never read past the arrays).  Waves whose 32 rows lie past Lq store nothing.
enum { KMASK_NONE = 0, KMASK_CAUSAL = 1, KMASK_UNPADDED = 2 };
// MASK2D (with BIAS): key_bias is an additive mask [LqR][LkR] (fp32, shared by all heads; -inf hides a key from a
// query) instead of a per-key bias: every lane reads the 16 values of its own query's row from global memory at the
// top of a block (the path of the per-key bias at d = 128); H is ignored.
template <int D, int MODE, bool PRESCALE, bool BIAS, int KMASK, bool MASK2D = false>
__global__ __launch_bounds__(NT, 2) void k_sddmm32(const __bf16 *__restrict__ Q, const __bf16 *__restrict__ K,
                                                   const float *__restrict__ key_bias, int H,
                                                   int Lq, int Lk, int LqR, int LkR, float scale, int ksplit,
                                                   int blocks_per_wg, uint32_t *__restrict__ out,
                                                   uint32_t *__restrict__ meta) {
    constexpr bool CAUSAL = KMASK == KMASK_CAUSAL, UNPADDED = KMASK == KMASK_UNPADDED;
    constexpr int CPR = D / 8;           // 16-byte chunks per row
    constexpr int TILE = KB * CPR;       // chunks per K block
    constexpr int LPT = TILE / NT;       // asynchronous copies per thread per block
    constexpr int STEPS = D / 16;        // k-steps of the 32x32x16 MFMA
    constexpr int TQ = 128;              // queries per workgroup (4 waves x 32)
    // One LDS array, so that d = 128 fits two workgroups per compute unit (2 x 80 KiB):
    //   Ks     double buffer of K blocks: the copy of block it+1 runs under the work on block it
    //   Stage  per-wave staging of the kept values of one 128-key block (32 rows x 128 bytes), so that they
    //          leave as whole 128-byte lines from consecutive lanes instead of 16-byte pieces scattered over
    //          32 rows
    //   Bs     bias of the block's 128 keys (double buffer), copied along with K
    constexpr int STAGE = MODE == MODE_DENSE ? 0 : 32 * 8;   // 16-byte units per wave
    // (d = 128: K and the staging fill the 80 KiB that let two workgroups share a compute unit, so there the bias
    // is read from global memory into registers at the top of every block instead)
    static_assert(!MASK2D || BIAS, "the 2-D mask travels the bias path");
    constexpr bool BIAS_LDS = BIAS && D == 64 && !MASK2D;
    __shared__ u32x4 Smem[2 * TILE + 4 * STAGE + (BIAS_LDS ? 2 * (KB / 4) : 0)];
    u32x4(*const Ks)[TILE] = reinterpret_cast<u32x4(*)[TILE]>(Smem);
    f32x4(*const Bs)[KB / 4] = reinterpret_cast<f32x4(*)[KB / 4]>(Smem + 2 * TILE + 4 * STAGE);

    const int tid = threadIdx.x;
    const int w = tid >> 6, l = tid & 63, lj = l & 31, h = l >> 5;

    const unsigned qtiles = (Lq + TQ - 1) / TQ;   // (Lq % 128 == 64 only with unpadded lengths)
    const unsigned item = xcd_contiguous(blockIdx.x, gridDim.x);
    const int ks_id = item % ksplit;
    const int qt = (item / ksplit) % qtiles;
    const int bh = item / (ksplit * qtiles);
    const int jb0 = ks_id * blocks_per_wg;
    const int q0 = qt * TQ + w * 32;
    const bool wave_stores = !UNPADDED || __builtin_amdgcn_readfirstlane(q0) < Lq;

    const __bf16 *Kh = K + (size_t)bh * LkR * D;

    // LDS position p (16-byte units) = slot * CPR + (c ^ (slot & 7)) holds chunk c of the key of row slot `slot`
    int src_off[LPT];
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
        const int p = i * NT + tid;
        const int slot = p / CPR, c = (p % CPR) ^ (slot & 7);
        const int t = slot >> 5, r = slot & 31;          // tile, MFMA row = 8 g + 4 h' + x
        const int key = 64 * (t >> 1) + 32 * ((r >> 2) & 1) + 16 * (t & 1) + 4 * (r >> 3) + (r & 3);
        src_off[i] = key * D + c * 8;
    }
    const uint32_t lds_k = lds_address(&Ks[0][w * 64]);
    const float *bias_b = !BIAS ? nullptr
                          : MASK2D ? key_bias + (size_t)(UNPADDED && q0 + lj >= LqR ? LqR - 1 : q0 + lj) * LkR
                                   : key_bias + (size_t)(bh / H) * LkR;
    const uint32_t lds_b = lds_address(&Bs[0][0]);
    auto issue_block = [&](int jb, int buf) {
        const __bf16 *src = Kh + (size_t)jb * KB * D;
        const int real = LkR - jb * KB;   // real keys from this block's first one on
        if (UNPADDED && real < KB) {
            // partial last block: the places of the absent keys take the block's last real key
#pragma unroll
            for (int i = 0; i < LPT; ++i) {
                const int p = i * NT + tid;
                const int slot = p / CPR, c = (p % CPR) ^ (slot & 7);
                const int t = slot >> 5, r = slot & 31;
                const int key = 64 * (t >> 1) + 32 * ((r >> 2) & 1) + 16 * (t & 1) + 4 * (r >> 3) + (r & 3);
                async_copy16(src, 2u * ((key < real ? key : real - 1) * D + c * 8), lds_k + 16u * (buf * TILE + i * NT));
            }
            if constexpr (BIAS_LDS) {   // (LkR is a multiple of 4: the last float4 of the row stands in for the absent ones)
                if (tid < KB / 4)
                    async_copy16(bias_b + (size_t)jb * KB, 16u * (4 * tid < real ? tid : real / 4 - 1),
                                 lds_b + (uint32_t)(buf * KB * 4));
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < LPT; ++i) async_copy16(src, 2u * src_off[i], lds_k + 16u * (buf * TILE + i * NT));
        if constexpr (BIAS_LDS) {   // 512 bytes: lanes 0..31 of wave 0 (the copy lands through the same counter as K)
            if (tid < KB / 4) async_copy16(bias_b + (size_t)jb * KB, 16u * tid, lds_b + (uint32_t)(buf * KB * 4));
        }
    };

    // Order of the blocks: workgroup g starts g blocks into its range and wraps around (the blocks of stage 1 do not
    // depend on one another).  Rows of the compressed matrix are a power of two apart for the usual lengths: workgroups
    // marching from their first block in step would all write the same few memory channels at a time.
    const int rot = __builtin_amdgcn_readfirstlane((int)(item % (unsigned)blocks_per_wg));
    auto blk = [&](int it) { return jb0 + (it + rot < blocks_per_wg ? it + rot : it + rot - blocks_per_wg); };
    issue_block(blk(0), 0);

    // Q operand: lane (column lj, half h) of step s holds Q[q][16 s + 8 h .. +7]
    bf16x8 bq[STEPS];
#pragma unroll
    for (int s = 0; s < STEPS; ++s) {
        const int qrow = UNPADDED && q0 + lj >= LqR ? LqR - 1 : q0 + lj;
        const u32x4 raw = *reinterpret_cast<const u32x4 *>(Q + ((size_t)bh * LqR + qrow) * D + 16 * s + 8 * h);
        if constexpr (PRESCALE) {
            u32x4 sc;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                sc[e] = pack_bf16x2(bf16_lo_to_f32(raw[e]) * scale, bf16_hi_to_f32(raw[e]) * scale);
            bq[s] = __builtin_bit_cast(bf16x8, sc);
        } else {
            bq[s] = __builtin_bit_cast(bf16x8, raw);
        }
    }

    const size_t row = (size_t)bh * Lq + q0 + lj;
    // read-back role of this lane when the staged block is written out: store i (0..3) covers rows
    // 8 i + l/8, 16-byte chunk l%8 of the row's 128 bytes; chunks are XOR-swizzled by row % 8, which keeps
    // the 8 lanes of one LDS pass on 8 different chunk columns for the writes (8 rows, one chunk) and for
    // the reads (one row, 8 chunks)
    const int sb_row = l >> 3, sb_chunk = l & 7;
    uint32_t *const out_sb = out + (((size_t)bh * Lq + q0 + sb_row) * (size_t)(Lk / 2)) / 2 + sb_chunk * 4;
    const size_t sb_step = (size_t)8 * (Lk / 4);   // 8 rows further, in dwords
    // metadata of (row, block jb): 16 bytes at ((row block * blocks + jb) * 16 + row % 16) * 4 words;
    // a lane computes the words of chunks (p = 0, h) and (p = 1, h) = slots 2 h and 2 h + 1 of its row
    u32x4 *const meta_row4 = reinterpret_cast<u32x4 *>(
        meta + (((size_t)bh * (Lq / 16) + ((q0 + lj) >> 4)) * (Lk / KB) * 16 + (lj & 15)) * 4);

    for (int it = 0; it < blocks_per_wg; ++it) {
        const int jb = blk(it);
        const int buf = it & 1;
        // Block `it` must have landed.  The stores of the previous iteration were issued after its
        // copy and may stay in flight (waiting for them would expose the store latency every block).
        constexpr int kStores = MODE == MODE_DENSE ? 8 : 5;   // stores per iteration, exactly (or lower): 4 of values + 1 of metadata
        if (it == 0 || !wave_stores) wait_async_copies();   // (a wave that stores nothing has nothing younger in flight)
        else wait_async_copies_keep<kStores>();
        __syncthreads();       // ... for every wave, and everybody is done with the block before
        f32x4 kbg[2][2][4];    // (BIAS without LDS) bias of keys 128 jb + 64 p + 32 h + 16 u + 4 g + x, loaded before the
                               // next block's copies are issued so that waiting for it does not wait for them
        if constexpr (BIAS && !BIAS_LDS) {
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int g = 0; g < 4; ++g)
                    {
                        int key = jb * KB + 64 * p + 32 * h + 16 * u + 4 * g;
                        if (UNPADDED && key >= LkR) key = LkR - 4;   // (an absent key: masked below, whatever its bias)
                        kbg[p][u][g] = *reinterpret_cast<const f32x4 *>(bias_b + key);
                    }
        }
        if (it + 1 < blocks_per_wg) issue_block(blk(it + 1), buf ^ 1);

        u32x2 mwords = {0u, 0u};
#pragma unroll
        for (int p = 0; p < 2; ++p) {                 // pair of key tiles = 64 keys
            f32x16 acc[2];
            f32x4 kb4[2][4];   // bias of keys 128 jb + 64 p + 32 h + 16 u + 4 g + x
            if constexpr (BIAS) {
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int g = 0; g < 4; ++g) kb4[u][g] = BIAS_LDS ? Bs[buf][16 * p + 8 * h + 4 * u + g] : kbg[p][u][g];
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int t = 2 * p + u;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    if constexpr (BIAS && PRESCALE) acc[u][r] = kb4[u][r >> 2][r & 3];
                    else acc[u][r] = 0.f;
                }
#pragma unroll
                for (int s = 0; s < STEPS; ++s) {
                    const bf16x8 ak =
                        __builtin_bit_cast(bf16x8, Ks[buf][(32 * t + lj) * CPR + ((2 * s + h) ^ (lj & 7))]);
                    acc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak, bq[s], acc[u], 0, 0, 0);
                }
            }
            // acc[u][4g + x] = score of query q0 + lj and key 128 jb + 64 p + 32 h + 16 u + 4 g + x
            const int kbase = KB * jb + 64 * p + 32 * h;
            // causal: hidden scores become -inf on the raw accumulators (the scaling and the bias leave -inf as it is).
            // q0 is the same in every lane of the wave; as a scalar, the test is one branch around the masking.
            if (KMASK != KMASK_NONE &&
                KB * jb + 64 * p + 63 > (CAUSAL ? __builtin_amdgcn_readfirstlane(q0) + Lk - Lq : LkR - 1)) {
                asm volatile("" ::: "memory");   // (not to be turned into selects that every block would execute)
                const int lim = (CAUSAL ? q0 + lj + Lk - Lq : LkR - 1) - kbase;   // key offsets above it are hidden
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (16 * u + r > lim) acc[u][r] = -INFINITY;
            }
            if constexpr (MODE == MODE_DENSE) {
                uint32_t pk[16];
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        float a0 = acc[u][2 * e], a1 = acc[u][2 * e + 1];
                        if constexpr (!PRESCALE) {
                            a0 *= scale; a1 *= scale;
                            if constexpr (BIAS) {
                                a0 = add_unfused(a0, kb4[u][e >> 1][2 * (e & 1)]);
                                a1 = add_unfused(a1, kb4[u][e >> 1][2 * (e & 1) + 1]);
                            }
                        }
                        pk[8 * u + e] = pack_bf16x2(a0, a1);
                    }
                u32x4 *dst = reinterpret_cast<u32x4 *>(out + (row * Lk + kbase) / 2);
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (wave_stores) dst[c] = u32x4{pk[4 * c], pk[4 * c + 1], pk[4 * c + 2], pk[4 * c + 3]};
            } else {
                uint32_t word = 0;
                u32x4 pk[2];
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        float a0 = acc[u][4 * g], a1 = acc[u][4 * g + 1], a2 = acc[u][4 * g + 2], a3 = acc[u][4 * g + 3];
                        if constexpr (!PRESCALE) {
                            a0 *= scale; a1 *= scale; a2 *= scale; a3 *= scale;
                            if constexpr (BIAS) {
                                a0 = add_unfused(a0, kb4[u][g][0]); a1 = add_unfused(a1, kb4[u][g][1]);
                                a2 = add_unfused(a2, kb4[u][g][2]); a3 = add_unfused(a3, kb4[u][g][3]);
                            }
                        }
                        float lo, hi;
                        uint32_t code;
                        if constexpr (MODE == MODE_2TO4) select_2of4(a0, a1, a2, a3, 16 * u + 4 * g, lo, hi, code);
                        else select_1of2(a0, a1, a2, a3, 16 * u + 4 * g, lo, hi, code);
                        pk[u][g] = pack_bf16x2(lo, hi);
                        word |= code;
                    }
                // stage: this lane's 32 bytes are chunks 4p + 2h, 4p + 2h + 1 of row lj
                u32x4 *const st = Smem + 2 * TILE + w * STAGE;
                st[lj * 8 + ((4 * p + 2 * h) ^ (lj & 7))] = pk[0];
                st[lj * 8 + ((4 * p + 2 * h + 1) ^ (lj & 7))] = pk[1];
                mwords[p] = word;
            }
        }
        if constexpr (MODE != MODE_DENSE) {
            u32x4 *const st = Smem + 2 * TILE + w * STAGE;
            wave_lds_sync();
            u32x4 v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = st[(8 * i + sb_row) * 8 + (sb_chunk ^ sb_row)];
            wave_lds_sync();   // the staging rows are free for the next block
            // the two lanes (lj, h = 0/1) of a row hold 8 bytes of metadata each: lane (lj, 0) takes the other
            // half from lane (lj, 1), so that lanes 0..31 store the 16 bytes of rows 0..31 (two contiguous
            // 256-byte runs)
            const u32x4 m4 = {mwords[0], mwords[1], (uint32_t)__shfl_xor((int)mwords[0], 32),
                              (uint32_t)__shfl_xor((int)mwords[1], 32)};
            // four stores of 8 rows x 128 contiguous bytes: one whole line per row
            uint32_t *const dst = out_sb + (size_t)(KB * jb) / 4;
            if (wave_stores) {
#pragma unroll
                for (int i = 0; i < 4; ++i) __builtin_nontemporal_store(v[i], reinterpret_cast<u32x4 *>(dst + i * sb_step));
                if (h == 0) __builtin_nontemporal_store(m4, &meta_row4[(size_t)jb * 16]);
            }
        }
    }
}

inline bool is_pow2(float x) {
    int e;
    return frexpf(x, &e) == 0.5f;
}

template <int MODE, int NQ, bool BIAS, bool CAUSAL>
hipError_t launch_nq(const void *Q, const void *K, const float *key_bias, int H, int BH, int Lq, int Lk,
                     int d, float scale, void *out, void *meta, hipStream_t st) {
    const int qtiles = Lq / (64 * NQ);
    const int kblocks = Lk / KB;
    // split the key range until the grid has a few workgroups per compute unit
    int ksplit = 1;
    while ((long)BH * qtiles * ksplit < 1024 && kblocks % (ksplit * 2) == 0) ksplit *= 2;
    if ((long)BH * qtiles * ksplit < 1024 && kblocks % 3 == 0 && ksplit == 1) ksplit = 3;
    const int per_wg = kblocks / ksplit;
    const unsigned grid = (unsigned)((long)BH * qtiles * ksplit);
    const bool pre = is_pow2(scale);
#define DFSS_LAUNCH(DD, PRE)                                                                              \
    hipLaunchKernelGGL((k_sddmm<DD, MODE, NQ, PRE, BIAS, CAUSAL>), dim3(grid), dim3(NT), 0, st,               \
                       (const __bf16 *)Q, (const __bf16 *)K, key_bias, H, Lq, Lk, scale, ksplit, per_wg,       \
                       (uint32_t *)out, (uint32_t *)meta)
    if (d == 64) {
        if (pre) DFSS_LAUNCH(64, true); else DFSS_LAUNCH(64, false);
    } else {
        if (pre) DFSS_LAUNCH(128, true); else DFSS_LAUNCH(128, false);
    }
#undef DFSS_LAUNCH
    return hipGetLastError();
}

template <int MODE, bool BIAS, int KMASK, bool MASK2D = false>
hipError_t launch32(const void *Q, const void *K, const float *key_bias, int H, int BH, int Lq, int Lk, int LqR, int LkR,
                    int d, float scale, void *out, void *meta, hipStream_t st) {
    const int qtiles = (Lq + 127) / 128;
    const int kblocks = Lk / KB;
    int ksplit = 1;
    while ((long)BH * qtiles * ksplit < 1024 && kblocks % (ksplit * 2) == 0) ksplit *= 2;
    if ((long)BH * qtiles * ksplit < 1024 && kblocks % 3 == 0 && ksplit == 1) ksplit = 3;
    const int per_wg = kblocks / ksplit;
    const unsigned grid = (unsigned)((long)BH * qtiles * ksplit);
    const bool pre = is_pow2(scale);
#define DFSS_LAUNCH(DD, PRE)                                                                             \
    hipLaunchKernelGGL((k_sddmm32<DD, MODE, PRE, BIAS, KMASK, MASK2D>), dim3(grid), dim3(NT), 0, st,         \
                       (const __bf16 *)Q, (const __bf16 *)K, key_bias, H, Lq, Lk, LqR, LkR, scale, ksplit, per_wg, \
                       (uint32_t *)out, (uint32_t *)meta)
    if (d == 64) {
        if (pre) DFSS_LAUNCH(64, true); else DFSS_LAUNCH(64, false);
    } else {
        if (pre) DFSS_LAUNCH(128, true); else DFSS_LAUNCH(128, false);
    }
#undef DFSS_LAUNCH
    return hipGetLastError();
}

template <int MODE, bool BIAS, bool CAUSAL>
hipError_t launch_b(const void *Q, const void *K, const float *key_bias, int H, int BH, int Lq, int Lk,
                    int d, float scale, void *out, void *meta, hipStream_t st) {
    // 32 queries per wave (32x32x16 MFMA) when the query count allows it, else 16 (16x16x32 MFMA)
    if (Lq % 128 == 0)
        return launch32<MODE, BIAS, CAUSAL ? KMASK_CAUSAL : KMASK_NONE>(Q, K, key_bias, H, BH, Lq, Lk, Lq, Lk, d, scale, out,
                                                                         meta, st);
    // Lq = 64 (mod 128): the same kernel with the upper half of the last workgroup idle (its waves store nothing; the
    // mechanism of the unpadded lengths) is faster than 16 queries per wave; the causal mask keeps the latter
    if constexpr (!CAUSAL)
        return launch32<MODE, BIAS, KMASK_UNPADDED>(Q, K, key_bias, H, BH, Lq, Lk, Lq, Lk, d, scale, out, meta, st);
    return launch_nq<MODE, 1, BIAS, CAUSAL>(Q, K, key_bias, H, BH, Lq, Lk, d, scale, out, meta, st);
}

template <int MODE>
hipError_t launch(const void *Q, const void *K, const float *key_bias, int H, int causal, int BH, int Lq, int Lk,
                  int LqR, int LkR, int d, float scale, void *out, void *meta, hipStream_t st) {
    if (LqR != Lq || LkR != Lk) {   // unpadded lengths (never with the causal mask)
        if (key_bias)
            return launch32<MODE, true, KMASK_UNPADDED>(Q, K, key_bias, H, BH, Lq, Lk, LqR, LkR, d, scale, out, meta, st);
        return launch32<MODE, false, KMASK_UNPADDED>(Q, K, nullptr, 1, BH, Lq, Lk, LqR, LkR, d, scale, out, meta, st);
    }
    if (causal) {
        if (key_bias) return launch_b<MODE, true, true>(Q, K, key_bias, H, BH, Lq, Lk, d, scale, out, meta, st);
        return launch_b<MODE, false, true>(Q, K, nullptr, 1, BH, Lq, Lk, d, scale, out, meta, st);
    }
    if (key_bias) return launch_b<MODE, true, false>(Q, K, key_bias, H, BH, Lq, Lk, d, scale, out, meta, st);
    return launch_b<MODE, false, false>(Q, K, nullptr, 1, BH, Lq, Lk, d, scale, out, meta, st);
}

}  // namespace

hipError_t launch_sddmm_prune(const void *Q, const void *K, const float *key_bias, int H, int causal, int BH, int Lq,
                              int Lk, int LqR, int LkR, int d, int mode, float scale, void *vals, void *meta,
                              hipStream_t st) {
    return mode == 0 ? launch<MODE_2TO4>(Q, K, key_bias, H, causal, BH, Lq, Lk, LqR, LkR, d, scale, vals, meta, st)
                     : launch<MODE_1TO2>(Q, K, key_bias, H, causal, BH, Lq, Lk, LqR, LkR, d, scale, vals, meta, st);
}

hipError_t launch_dense_scores(const void *Q, const void *K, const float *key_bias, int H, int causal, int BH, int Lq,
                               int Lk, int LqR, int LkR, int d, float scale, void *S, hipStream_t st) {
    return launch<MODE_DENSE>(Q, K, key_bias, H, causal, BH, Lq, Lk, LqR, LkR, d, scale, S, nullptr, st);
}

namespace {
template <int MODE>
hipError_t launch_mask2d(const void *Q, const void *K, const float *mask, int BH, int Lq, int Lk, int LqR, int LkR, int d,
                         float scale, void *out, void *meta, hipStream_t st) {
    if (LqR != Lq || LkR != Lk || Lq % 128 != 0)
        return launch32<MODE, true, KMASK_UNPADDED, true>(Q, K, mask, 1, BH, Lq, Lk, LqR, LkR, d, scale, out, meta, st);
    return launch32<MODE, true, KMASK_NONE, true>(Q, K, mask, 1, BH, Lq, Lk, LqR, LkR, d, scale, out, meta, st);
}
}  // namespace

hipError_t launch_sddmm_prune_mask(const void *Q, const void *K, const float *mask, int BH, int Lq, int Lk, int LqR,
                                   int LkR, int d, int mode, float scale, void *vals, void *meta, hipStream_t st) {
    return mode == 0 ? launch_mask2d<MODE_2TO4>(Q, K, mask, BH, Lq, Lk, LqR, LkR, d, scale, vals, meta, st)
                     : launch_mask2d<MODE_1TO2>(Q, K, mask, BH, Lq, Lk, LqR, LkR, d, scale, vals, meta, st);
}

hipError_t launch_dense_scores_mask(const void *Q, const void *K, const float *mask, int BH, int Lq, int Lk, int LqR,
                                    int LkR, int d, float scale, void *S, hipStream_t st) {
    return launch_mask2d<MODE_DENSE>(Q, K, mask, BH, Lq, Lk, LqR, LkR, d, scale, S, nullptr, st);
}

}  // namespace dfss
