// Whole DFSS forward pass in one kernel, 32 queries per wave (see fused_attention.hip for the
// method: arXiv 2203.00091, Sec. 3.1 stages, Sec. 3.4 pruning on the accumulators,
// App. A.1.3 softmax).  Scores come from v_mfma_f32_32x32x16_bf16 (twice the flops per cycle of
// the 16x16x32 form on gfx950), the product with V from v_smfmac_f32_32x32x32_bf16.
//
// What keeps the vector ALU work per score low (the unit this kernel is bound by):
//
//  * Scores are formed RELATIVE TO THE SOFTMAX REFERENCE on the matrix unit.  The accumulator operand
//    of the first matrix instruction of a tile is a register tuple that holds -c for the lane's query
//    (c = reference value, in units of the raw dot product; a bfloat16 number, so integer-valued
//    inputs keep exact scores), so the scores arrive as s' = q.k - c.  Softmax does not depend on c
//    (App. A.1.3 subtracts the row maximum for the same reason), the weight is
//    exp2(s' * scale * log2 e): one multiply, no subtraction, and the scale needs no instruction of
//    its own.  c is set from the first block (row maximum + kTau) and raised only when a later score
//    reaches it (rare; then the partial results are rescaled), so every s' the selection sees is
//    negative.  kTau is small on purpose: the scores are rounded at the magnitude of s', and a large
//    offset would cost comparison precision.
//
//  * The 2:4 selection carries the key position inside the value.  The two low mantissa bits
//    of each of the four scores of a run are replaced by the position 0..3 (a relative change
//    of 2^-22).  For negative numbers a smaller bit pattern is a larger value, so among equal
//    scores the lower position wins -- the tie rule of the method.  The two largest of the four
//    are then max3 / med3 / max / med3 (4 instructions), and their positions are read off the
//    low bits (2 instructions) straight into the index operand of the sparse matrix
//    instruction, which takes the two positions of a run in either order.
//    Selection on the raw dot product is selection on scale * dot: scale > 0.
//
// Register layouts (lane l, lj = l % 32, h = l / 32):
//   scores of one 32-key tile: lane holds query lj and, thanks to the key order of the
//   LDS rows (row 8g + 4h' + x holds key 16h' + 4g + x), the 16 consecutive keys
//   16h .. 16h+15 of the tile in registers 4g + x: four runs of four keys.
//   The 8 kept weights + 16 position bits of the lane are the A operand / index of the sparse
//   instruction for row lj, contraction chunk h.
//   O and the row sums: column lj of a 32-column tile, rows (queries) 8(r/4) + 4h + r%4.
#include <type_traits>

#include "block_list.hpp"
#include "dfss_device.hpp"
#include "dfss_kernels.hpp"


namespace dfss {

namespace {

constexpr int KB = 64;    // keys per block (two 32-key tiles)
constexpr float kTau = 4.0f;    // distance of the reference above the row maximum it was set from (score units)
constexpr float kLog2e = 1.4426950408889634f;

enum { MODE_2TO4 = 0, MODE_1TO2 = 1, MODE_DENSE = 2 };

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ float with_position(float v, uint32_t pos) {
    return __uint_as_float((__float_as_uint(v) & 0xFFFFFFFCu) | pos);
}
// smallest bfloat16 number >= v, as a float (v finite, far from overflow)
__device__ __forceinline__ float bf16_ceil(float v) {
    const uint32_t u = __float_as_uint(v);
    return __uint_as_float(((u >> 31) ? u : u + 0xFFFFu) & 0xFFFF0000u);
}
// idx = (idx >> 2) | (low two bits of v) << 30: sixteen of these fill idx with sixteen positions, first one lowest
__device__ __forceinline__ uint32_t push_position(uint32_t idx, float v) {
    return __builtin_amdgcn_alignbit(__float_as_uint(v), idx, 2);
}

// NW waves per workgroup = NW / KS query tiles of 32 queries x KS waves per tile.  With KS = 2 the two
// waves of a query tile share its keys: of every 64-key block, wave ks takes the 32-key tile ks (its own
// reference value, row sums and partial O, merged at the end through LDS).  Smaller work items, more
// waves per SIMD: what short sequences and small batches need to fill the chip.
// MASKED: the call carries a key bias, a block mask and / or the causal flag (KS = 1 only):
//   key_bias   additive per-key term (fp32 [B][Lk], shared by the H heads of a batch element; -inf masks a key).
//              The scores here are raw dot products relative to the reference, so the bias joins them as
//              bias / scale in the accumulator the score tile starts from (exact for 0, -inf and, with a scale that
//              is a power of two, for every finite bias).  -inf becomes -1e30: the position bits need a finite number,
//              and exp2 of it is exactly 0 all the same.
//   block_mask uint8 [Lq/64][Lk/64] shared by all heads (needs 64-query workgroups, NW = 2: the launchers below do
//              not instantiate that form, the 16-query kernel measured faster for block patterns); causal: query i
//              sees keys 0 .. i + (Lk - Lq).  Blocks that hold nothing for the workgroup are skipped (block_list.hpp); hidden
//              scores of the blocks that the diagonal cuts are overwritten with -1e30 by index.
// VARLEN (unmasked kernels with KS = 1): key_len[b] keys of batch element b = head / H are real (1 <= key_len[b] <= Lk; the
//   arrays are padded to Lk).  A head's workgroups walk only the blocks that hold real keys, and in the block a
//   sequence ends in the scores of the keys past its end are overwritten by index -- no bias array is read, and every
//   other block costs what it costs without padding.  (Block 0 always holds key 0, so the first block sets a finite
//   reference.)
// CAUSAL_ONLY (the same kernels): the causal mask and nothing else (query i sees keys 0 .. i + Lk - Lq), by the same two
//   means: a workgroup walks the blocks up to the last key its last query sees, and in the blocks that the diagonal of
//   a wave's queries cuts the hidden scores are overwritten by index.  Launch order: last row block of every head first.
// RAGGED (the same kernels): lengths that are no tile multiples (any Lq; Lk a multiple of 4), arrays unpadded.  Absent
//   queries of the last tile read the last query and are not stored; the places of absent keys in the last block are
//   copied from the block's last key (never past the arrays) and their scores overwritten like padding keys.
template <int D, int MODE, int NW, int KS, int OCC, bool MASKED, bool VARLEN = false, bool CAUSAL_ONLY = false,
          bool RAGGED = false>
__global__ __launch_bounds__(64 * NW, OCC * 4 / NW) void k_fused32(const __bf16 *__restrict__ Q, const __bf16 *__restrict__ K,
                                                        const __bf16 *__restrict__ V, const float *__restrict__ key_bias,
                                                        int H, const uint8_t *__restrict__ block_mask, int causal,
                                                        int Lq, int Lk, float scale, uint16_t *__restrict__ O,
                                                        const int *__restrict__ key_len) {
    static_assert(!MASKED || KS == 1, "the masked variants do not split the keys of a block over waves");
    static_assert(!VARLEN || (KS == 1 && !MASKED), "key lengths: whole blocks per wave, no other mask");
    static_assert(!CAUSAL_ONLY || (KS == 1 && !MASKED && !VARLEN), "causal alone: whole blocks per wave, no other mask");
    static_assert(!RAGGED || (KS == 1 && !MASKED && !VARLEN && !CAUSAL_ONLY), "ragged lengths: whole blocks per wave, no mask");
    constexpr int NT = 64 * NW;
    constexpr int CPR = D / 8;          // 16-byte chunks per row
    constexpr int TILE = KB * CPR;      // chunks per K (or V) block
    constexpr int LPT = TILE / NT;      // direct-to-LDS loads per thread per block and operand
    constexpr int STEPS = D / 16;       // k-steps of the 32x32x16 MFMA
    constexpr int DT = D / 32;          // 32-column tiles of O
    constexpr int TQ = 32 * NW / KS;    // queries per workgroup
    constexpr int KT = 2 / KS;          // 32-key tiles of a block that this wave works on
    constexpr bool SPARSE = MODE != MODE_DENSE;
    constexpr int NP = SPARSE ? 4 : 8;  // packed weight dwords per lane per key tile
    static_assert(KS == 1 || KS == 2, "a 64-key block has two 32-key tiles");
    static_assert(TILE % NT == 0, "every thread copies the same number of chunks");
    __shared__ u32x4 Smem[4 * TILE];                       // K double buffer, then V double buffer
    u32x4 (*const Ks)[TILE] = reinterpret_cast<u32x4 (*)[TILE]>(&Smem[0]);
    u32x4 (*const Vs)[TILE] = reinterpret_cast<u32x4 (*)[TILE]>(&Smem[2 * TILE]);

    const int tid = threadIdx.x;
    const int w = tid >> 6, l = tid & 63, lj = l & 31, h = l >> 5;
    const int qw = w / KS, ks = w % KS;   // query tile of the workgroup, key tile of the block

    const unsigned qtiles = RAGGED ? (Lq + TQ - 1) / TQ : Lq / TQ;
    int qt, bh;
    if (CAUSAL_ONLY || (MASKED && (block_mask || causal))) {
        // row blocks differ widely in work: hand them out across heads in launch order, heavy ones first (with a
        // block pattern the global rows come first; under the causal mask the work grows with the row block)
        const unsigned heads = gridDim.x / qtiles;
        qt = blockIdx.x / heads;
        if (CAUSAL_ONLY || (causal && !block_mask)) qt = qtiles - 1 - qt;
        bh = blockIdx.x % heads;
    } else {
        const unsigned item = xcd_contiguous(blockIdx.x, gridDim.x);
        qt = item % qtiles;
        bh = item / qtiles;
        if constexpr (VARLEN) {
            // neighbours in launch order come from different batch elements, so that every XCD (and compute unit)
            // gets long and short sequences alike
            const unsigned nb = gridDim.x / qtiles / (unsigned)H;
            bh = (bh % nb) * H + bh / nb;
        }
    }
    const int q0 = qt * TQ + qw * 32;
    int lk_eff = Lk;   // VARLEN: real keys of this head
    if constexpr (VARLEN) {
        const int n = __builtin_amdgcn_readfirstlane(key_len[bh / H]);
        lk_eff = n < 1 ? 1 : n > Lk ? Lk : n;
    }
    const int coff = Lk - Lq;           // causal: query i sits at position i + coff
    const int nblocks = VARLEN || RAGGED ? (lk_eff + KB - 1) / KB
                        : CAUSAL_ONLY    ? (__builtin_amdgcn_readfirstlane(qt) * TQ + TQ - 1 + coff) / KB + 1
                                         : Lk / KB;
    [[maybe_unused]] const int tail_keys = Lk - (nblocks - 1) * KB;   // RAGGED: keys of the last block

    // K block in LDS: row slot 32 kt + i (key tile kt, MFMA row i = 8g + 4h' + x) holds key
    // 32 kt + 16 h' + 4 g + x; chunk c sits at slot * CPR + (c ^ (slot & 7)).
    // V block: row = key, chunk c at row * CPR + (c ^ ((row & 3) << 1)).
    // Copy i of a thread handles LDS position p = i * NT + tid: NT / CPR row slots further on, which moves
    // neither the swizzle (low slot bits) nor the low key bits: source = that of copy 0 + a constant.
    constexpr int SPC = NT / CPR;       // row slots between consecutive copies of a thread
    static_assert(SPC % 8 == 0, "the slot bits that a thread's copies differ in are bits 3, 4 and 5");
    const int slot0 = tid / CPR;
    const int key0 = (slot0 & 32) | (((slot0 >> 2) & 1) << 4) | (((slot0 >> 3) & 3) << 2) | (slot0 & 3);
    const int k_chunk = ((tid % CPR) ^ (slot0 & 7)) * 8, v_chunk = ((tid % CPR) ^ ((slot0 & 3) << 1)) * 8;
    const uint32_t k_off = 2u * (key0 * D + k_chunk);
    const uint32_t v_off = 2u * (slot0 * D + v_chunk);
    const uint32_t lds_k = lds_address(&Ks[0][w * 64]), lds_v = lds_address(&Vs[0][w * 64]);
    const uint64_t k_base = uniform_address(K + (size_t)bh * Lk * D), v_base = uniform_address(V + (size_t)bh * Lk * D);
    // Q operand (B side of Q K^T): lane (column lj, half h) of step s holds Q[q][16 s + 8 h .. +7]
    bf16x8 bq[STEPS];
    const int qrow = RAGGED && q0 + lj >= Lq ? Lq - 1 : q0 + lj;
#pragma unroll
    for (int s = 0; s < STEPS; ++s)
        bq[s] = __builtin_bit_cast(
            bf16x8, *reinterpret_cast<const u32x4 *>(Q + ((size_t)bh * Lq + qrow) * D + 16 * s + 8 * h));

    const float k2 = scale * kLog2e;       // weight = exp2(s' * k2)
    const float tau = kTau / scale;        // kTau in units of the raw dot product
    float cref = 0.f;                      // reference value of query lj (raw dot product units; a bfloat16 number)
    f32x16 cneg;                           // -cref in every register: the accumulator the score tiles start from
#pragma unroll
    for (int r = 0; r < 16; ++r) cneg[r] = 0.f;
    f32x16 acc_o[DT], acc_l;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        acc_l[r] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) acc_o[dt][r] = 0.f;
    }
    const uint32_t one2 = 0x3F803F80u;  // two bfloat16 ones
    const bf16x8 ones8 = __builtin_bit_cast(bf16x8, u32x4{one2, one2, one2, one2});

    // transposing LDS read (per group of 16 lanes): lane s addresses V[key0 + s/4][col0 + 4 (s%4)]
    const int s16 = l & 15;
    const int tr_row = s16 >> 2, tr_sub = (s16 >> 1) & 1, tr_byte = 8 * (s16 & 1), tr_xor = tr_row << 1;
    const int tr_colgrp = (l >> 4) & 1;   // which 16 of the 32 columns of a tile this lane group reads
    const int kt0 = KS == 2 ? ks : 0;     // first (only, if KS = 2) key tile of this wave

    auto issue_block = [&](int jb, int buf) {
        const uint64_t ks_ = k_base + (uint64_t)jb * (KB * D * 2);
        const uint64_t vs_ = v_base + (uint64_t)jb * (KB * D * 2);
        if (RAGGED && jb == nblocks - 1 && tail_keys < KB) {   // partial last block: absent keys -> the block's last key
#pragma unroll
            for (int i = 0; i < LPT; ++i) {
                const int key = key0 + (((i * SPC) >> 3) & 1) * 4 + (((i * SPC) >> 4) & 1) * 8 + ((i * SPC) & 32);
                const int row = slot0 + i * SPC;
                async_copy16(ks_, 2u * ((key < tail_keys ? key : tail_keys - 1) * D + k_chunk), lds_k + 16u * (buf * TILE + i * NT));
                async_copy16(vs_, 2u * ((row < tail_keys ? row : tail_keys - 1) * D + v_chunk), lds_v + 16u * (buf * TILE + i * NT));
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < LPT; ++i)
            async_copy16(ks_ + (uint64_t)((((i * SPC) >> 3) & 1) * 4 + (((i * SPC) >> 4) & 1) * 8 + ((i * SPC) & 32)) * D * 2, k_off,
                         lds_k + 16u * (buf * TILE + i * NT));
#pragma unroll
        for (int i = 0; i < LPT; ++i)
            async_copy16(vs_ + (uint64_t)(i * SPC) * D * 2, v_off, lds_v + 16u * (buf * TILE + i * NT));
    };
    issue_block(0, 0);   // block 0 is copied before anything else (with masks: speculatively)

    const float *brow = nullptr;        // bias row of this head's batch element
    const float inv_scale = 1.0f / scale;
    BlockList<MASKED, false> blocks;
    if constexpr (MASKED) {
        if (key_bias) brow = key_bias + (size_t)(bh / H) * Lk;
        blocks.init(key_bias != nullptr, brow, block_mask != nullptr, block_mask + (size_t)(qt * TQ / 64) * nblocks,
                    causal, qt * TQ, TQ, coff, Lq, Lk, nblocks, l);
    }

    // one key block; the buffer index is a compile-time constant so that every LDS access names its buffer.
    // jn: the block after this one (>= nblocks: none); first: this is the first block the workgroup visits
    auto block = [&](auto parity, int jb, int jn, bool first) {
        constexpr int buf = decltype(parity)::value;
        wait_async_copies();  // vmcnt(0): this block's copies have landed
        __syncthreads();
        if (jn < nblocks) issue_block(jn, buf ^ 1);

        // ---- scores relative to the reference: acc[t][4g + x] = q . k - cref for query q0 + lj,
        //      key 64 jb + 32 (kt0 + t) + 16 h + 4 g + x ----
        f32x16 acc[KT];
        bool with_bias = false;
        if constexpr (MASKED) with_bias = brow != nullptr && blocks.has_bias(jb);
        if (MASKED && with_bias) {
            // the score tiles start from -c + bias / scale: keys 64 jb + 32 t + 16 h + r of this lane
#pragma unroll
            for (int t = 0; t < KT; ++t) {
                f32x16 cb;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 b = *reinterpret_cast<const f32x4 *>(brow + KB * jb + 32 * t + 16 * h + 4 * g);
#pragma unroll
                    for (int x = 0; x < 4; ++x) cb[4 * g + x] = cneg[4 * g + x] + fmaxf(b[x] * inv_scale, -1.0e30f);
                }
#pragma unroll
                for (int s = 0; s < STEPS; ++s) {
                    const bf16x8 ak =
                        __builtin_bit_cast(bf16x8, Ks[buf][(32 * t + lj) * CPR + ((2 * s + h) ^ (lj & 7))]);
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak, bq[s], s == 0 ? cb : acc[t], 0, 0, 0);
                }
            }
        } else {
#pragma unroll
            for (int t = 0; t < KT; ++t) {
#pragma unroll
                for (int s = 0; s < STEPS; ++s) {
                    const bf16x8 ak =
                        __builtin_bit_cast(bf16x8, Ks[buf][(32 * (kt0 + t) + lj) * CPR + ((2 * s + h) ^ (lj & 7))]);
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak, bq[s], s == 0 ? cneg : acc[t], 0, 0, 0);
                }
            }
        }
        if constexpr (VARLEN || RAGGED) {
            if (KB * jb + KB > lk_eff) {   // the block the sequence ends in: keys from lk_eff on count as masked
                asm volatile("" ::: "memory");   // (a branch, not selects that every block would execute)
                const int lim = lk_eff - 1 - (KB * jb + 16 * h);   // key offsets above it are padding
#pragma unroll
                for (int t = 0; t < KT; ++t)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (32 * t + r > lim) acc[t][r] = -1.0e30f;
            }
        }
        if constexpr (CAUSAL_ONLY) {
            if (KB * jb + KB - 1 > __builtin_amdgcn_readfirstlane(q0) + coff) {   // the wave's first query has hidden keys here
                asm volatile("" ::: "memory");   // (a branch, not selects that every block would execute)
                const int lim = q0 + lj + coff - (KB * jb + 16 * h);   // key offsets above it are hidden
#pragma unroll
                for (int t = 0; t < KT; ++t)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (32 * t + r > lim) acc[t][r] = -1.0e30f;
            }
        }
        if constexpr (MASKED) {
            // causal: the scores of keys after the query's own position count as masked (q0 is the same in every
            // lane of the wave; as a scalar, the test is one branch around the masking)
            if (causal && KB * jb + KB - 1 > __builtin_amdgcn_readfirstlane(q0) + coff) {
                asm volatile("" ::: "memory");   // (not to be turned into selects that every block would execute)
                const int lim = q0 + lj + coff - (KB * jb + 16 * h);   // key offsets above it are hidden
#pragma unroll
                for (int t = 0; t < KT; ++t)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (32 * t + r > lim) acc[t][r] = -1.0e30f;
            }
        }

        // ---- prune; arguments of the weights ----
        float kept[KT][2 * NP];
        uint32_t idx = 0;       // positions: tile t in bits [32 - 16 (KT - t), +16)
        bool force = first;     // the first block sets the reference
        for (;;) {
            float m_blk = -3.0e38f;
#pragma unroll
            for (int t = 0; t < KT; ++t) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const float a0 = acc[t][4 * g], a1 = acc[t][4 * g + 1], a2 = acc[t][4 * g + 2],
                                a3 = acc[t][4 * g + 3];
                    if constexpr (MODE == MODE_2TO4) {
                        const float e0 = with_position(a0, 0), e1 = with_position(a1, 1), e2 = with_position(a2, 2),
                                    e3 = with_position(a3, 3);
                        const float hi3 = fmaxf(fmaxf(e0, e1), e2);                 // v_max3_f32
                        const float md3 = __builtin_amdgcn_fmed3f(e0, e1, e2);
                        const float x = fmaxf(hi3, e3);                            // largest of the four
                        const float y = __builtin_amdgcn_fmed3f(hi3, md3, e3);     // second largest
                        kept[t][2 * g] = x;
                        kept[t][2 * g + 1] = y;
                        idx = push_position(push_position(idx, x), y);
                        m_blk = fmaxf(m_blk, x);
                    } else if constexpr (MODE == MODE_1TO2) {
                        const float x = fmaxf(with_position(a0, 0), with_position(a1, 1));   // larger of each pair
                        const float y = fmaxf(with_position(a2, 2), with_position(a3, 3));
                        kept[t][2 * g] = x;
                        kept[t][2 * g + 1] = y;
                        idx = push_position(push_position(idx, x), y);
                        m_blk = fmaxf(fmaxf(m_blk, x), y);
                    } else {
                        kept[t][4 * g] = a0; kept[t][4 * g + 1] = a1; kept[t][4 * g + 2] = a2; kept[t][4 * g + 3] = a3;
                        m_blk = fmaxf(m_blk, fmaxf(fmaxf(a0, a1), fmaxf(a2, a3)));
                    }
                }
            }
            // a score at or above the reference (not negative): raise the reference, redo the block
            if (!__any(force || m_blk >= 0.f)) break;
            // lanes lj and lj + 32 hold different keys of the same query
            const float mq = fmaxf(m_blk, __shfl_xor(m_blk, 32, 64));
            const bool up = force || mq >= 0.f;
            // the new reference, rounded UP to bfloat16 (so that it stays above the row maximum + tau and this
            // loop ends: after this pass every score of the block is negative); the scores of this block and
            // the reference move by delta (a difference of two bfloat16 numbers: exact)
            const float c_new = up ? bf16_ceil(cref + mq + tau) : cref;
            const float delta = c_new - cref;
            const float alpha = (up && !first) ? __builtin_amdgcn_exp2f(-delta * k2) : 1.f;
            cref = c_new;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                cneg[r] = -cref;
#pragma unroll
                for (int t = 0; t < KT; ++t) acc[t][r] -= delta;
            }
            if (!first) {
                // accumulator rows are queries 8 (r/4) + 4 h + r%4: fetch their factors from those columns' lanes
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float a_r = __shfl(alpha, 8 * (r >> 2) + 4 * h + (r & 3), 64);
                    acc_l[r] *= a_r;
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) acc_o[dt][r] *= a_r;
                }
            }
            force = false;
            idx = 0;
        }

        // ---- weights exp2(s' k2), packed as the A operand of the second product ----
        uint32_t pk[KT][NP];
#pragma unroll
        for (int t = 0; t < KT; ++t)
#pragma unroll
            for (int e = 0; e < NP; ++e) {
                const float p0 = __builtin_amdgcn_exp2f(kept[t][2 * e] * k2);
                const float p1 = __builtin_amdgcn_exp2f(kept[t][2 * e + 1] * k2);
                pk[t][e] = pack_bf16x2(p0, p1);
            }

        // ---- O += P V ; row sums += P 1 ----
        const char *vbase = reinterpret_cast<const char *>(&Vs[buf][0]);
        auto tr = [&](int key0, int dt) {
            const int row = key0 + tr_row;
            const int chunk = (4 * dt + 2 * tr_colgrp + tr_sub) ^ tr_xor;
            return lds_read_tr16(vbase + (row * CPR + chunk) * 16 + tr_byte);
        };
#pragma unroll
        for (int t = 0; t < KT; ++t) {
            const int kt = kt0 + t;
            if constexpr (SPARSE) {
                // contraction index of the sparse instruction = key of the tile; B lane (column, h)
                // holds keys 8 h .. +7 and 16 + 8 h .. +7.  The positions of the wave's last tile are the
                // high half of idx, those of the one before it (if any) the low half.
                const bf16x8 a = __builtin_bit_cast(bf16x8, u32x4{pk[t][0], pk[t][1], pk[t][2], pk[t][3]});
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    const int k0 = 32 * kt + 8 * h;
                    const s16x4 t0 = tr(k0, dt), t1 = tr(k0 + 4, dt), t2 = tr(k0 + 16, dt), t3 = tr(k0 + 20, dt);
                    const s16x8 lo = __builtin_shufflevector(t0, t1, 0, 1, 2, 3, 4, 5, 6, 7);
                    const s16x8 hi = __builtin_shufflevector(t2, t3, 0, 1, 2, 3, 4, 5, 6, 7);
                    const bf16x16 b = __builtin_bit_cast(
                        bf16x16, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15));
                    if (t + 1 < KT) acc_o[dt] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(a, b, acc_o[dt], (int)idx, 0, 0);
                    else acc_o[dt] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(a, b, acc_o[dt], (int)idx, 0, 1);
                }
                // row sums: against ones the positions do not matter, so the kept weights go through the dense
                // instruction as 16 "keys" per row (32 cycles against 43 for the sparse one)
                acc_l = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, ones8, acc_l, 0, 0, 0);
            } else {
                // dense: MFMA m (0/1) contracts the lanes' keys 16 h' + 8 m .. +7 (h' = 0, 1)
#pragma unroll
                for (int m = 0; m < 2; ++m) {
                    const bf16x8 a = __builtin_bit_cast(
                        bf16x8, u32x4{pk[t][4 * m], pk[t][4 * m + 1], pk[t][4 * m + 2], pk[t][4 * m + 3]});
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) {
                        const int k0 = 32 * kt + 16 * h + 8 * m;
                        const s16x4 t0 = tr(k0, dt), t1 = tr(k0 + 4, dt);
                        const bf16x8 b =
                            __builtin_bit_cast(bf16x8, __builtin_shufflevector(t0, t1, 0, 1, 2, 3, 4, 5, 6, 7));
                        acc_o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc_o[dt], 0, 0, 0);
                    }
                    acc_l = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, ones8, acc_l, 0, 0, 0);
                }
            }
        }
    };
    if constexpr (!MASKED) {
        for (int jb = 0; jb < nblocks; jb += 2) {
            block(std::integral_constant<int, 0>{}, jb, jb + 1, jb == 0);
            if (jb + 1 < nblocks) block(std::integral_constant<int, 1>{}, jb + 1, jb + 2, false);
        }
    } else {
        int jb = blocks.take();
        int jn = blocks.take();   // the block after this one
        // block 0 (copied speculatively at the top) turned out to hold nothing: overwrite the buffer with the first
        // live block (the two copies of a wave complete in issue order)
        if (jb != 0 && jb < nblocks) issue_block(jb, 0);
        for (bool first = true; jb < nblocks; first = false) {
            block(std::integral_constant<int, 0>{}, jb, jn, first);
            jb = jn;
            jn = blocks.take();
            if (jb >= nblocks) break;
            block(std::integral_constant<int, 1>{}, jb, jn, false);
            jb = jn;
            jn = blocks.take();
        }
    }

    if constexpr (KS == 2) {
        // ---- merge the two key halves of a query tile: wave ks = 1 hands its reference values, row sums
        //      and partial O to wave ks = 0 through LDS (the K and V buffers are free now) ----
        constexpr int SLOT = ((DT + 1) * 16 + 1) * 64;   // floats per wave pair: register-major, lane-minor
        static_assert((NW / 2) * SLOT * 4 <= 4 * TILE * 16, "the merge area fits into the K and V buffers");
        float *const area = reinterpret_cast<float *>(&Smem[0]) + qw * SLOT;
        __syncthreads();   // every wave is done with the last block
        if (ks == 1) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) area[(dt * 16 + r) * 64 + l] = acc_o[dt][r];
                area[(DT * 16 + r) * 64 + l] = acc_l[r];
            }
            area[(DT + 1) * 16 * 64 + l] = cref;
        }
        __syncthreads();
        if (ks == 1) return;
        // weights were formed as exp2((q.k - c) k2) with c = cref of the wave: bring both halves to the larger c
        const float c_b = area[(DT + 1) * 16 * 64 + l];
        const float c = fmaxf(cref, c_b);
        const float f_a = __builtin_amdgcn_exp2f((cref - c) * k2), f_b = __builtin_amdgcn_exp2f((c_b - c) * k2);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int src = 8 * (r >> 2) + 4 * h + (r & 3);   // lane that holds the factors of this row's query
            const float fa = __shfl(f_a, src, 64), fb = __shfl(f_b, src, 64);
            acc_l[r] = acc_l[r] * fa + area[(DT * 16 + r) * 64 + l] * fb;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) acc_o[dt][r] = acc_o[dt][r] * fa + area[(dt * 16 + r) * 64 + l] * fb;
        }
    }

    // ---- O[q][32 dt + lj] = acc_o / row sum, q = q0 + 8 (r/4) + 4 h + r%4 ----
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const float inv = __builtin_amdgcn_rcpf(acc_l[r]);
        if (RAGGED && q0 + 8 * (r >> 2) + 4 * h + (r & 3) >= Lq) continue;   // an absent query
        const size_t q = (size_t)bh * Lq + q0 + 8 * (r >> 2) + 4 * h + (r & 3);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
            O[q * D + 32 * dt + lj] = (uint16_t)(pack_bf16x2(acc_o[dt][r] * inv, 0.f) & 0xFFFFu);
    }
}

// waves per SIMD the kernels are compiled for (registers per lane <= 512 / OCC)
#define DFSS_OCC(DD) ((DD) == 128 || MASKED ? 2 : MODE == MODE_DENSE ? (KS == 2 ? 3 : 2) : 3)

template <int MODE, int NW, int KS, bool MASKED, bool VARLEN = false, bool CAUSAL_ONLY = false, bool RAGGED = false>
hipError_t launch_nw(const void *Q, const void *K, const void *V, const float *key_bias, int H,
                     const uint8_t *block_mask, int causal, int BH, int Lq, int Lk, int d, float scale, void *O,
                     hipStream_t st, const int *key_len = nullptr) {
    const unsigned grid = (unsigned)((long)BH * ((Lq + (RAGGED ? 32 * NW / KS - 1 : 0)) / (32 * NW / KS)));
#define DFSS_LAUNCH(DD)                                                                                       \
    hipLaunchKernelGGL((k_fused32<DD, MODE, NW, KS, DFSS_OCC(DD), MASKED, VARLEN, CAUSAL_ONLY, RAGGED>), dim3(grid), dim3(64 * NW), 0, st, \
                       (const __bf16 *)Q, (const __bf16 *)K, (const __bf16 *)V, key_bias, H, block_mask,      \
                       causal, Lq, Lk, scale, (uint16_t *)O, key_len)
    if (d == 64) DFSS_LAUNCH(64);
    else DFSS_LAUNCH(128);
#undef DFSS_LAUNCH
    return hipGetLastError();
}

template <int MODE>
hipError_t launch_mode(const void *Q, const void *K, const void *V, const float *key_bias, int H,
                       const uint8_t *block_mask, int causal, int BH, int Lq, int Lk, int d, int nw, int ks,
                       float scale, void *O, hipStream_t st) {
    if (key_bias || block_mask || causal) {   // masked calls: 128-query workgroups (block patterns need 64: not here)
        if (block_mask || nw != 4 || Lq % 128 != 0) return hipErrorInvalidValue;
        if constexpr (MODE != MODE_DENSE) {
            if (!key_bias)   // the causal mask alone: the kernel without the masking machinery
                return launch_nw<MODE, 4, 1, false, false, true>(Q, K, V, nullptr, H, nullptr, 1, BH, Lq, Lk, d, scale, O, st);
        }
        return launch_nw<MODE, 4, 1, true>(Q, K, V, key_bias, H, nullptr, causal, BH, Lq, Lk, d, scale, O, st);
    }
    if (ks == 2) return launch_nw<MODE, 4, 2, false>(Q, K, V, nullptr, 1, nullptr, 0, BH, Lq, Lk, d, scale, O, st);
    if (nw == 4) return launch_nw<MODE, 4, 1, false>(Q, K, V, nullptr, 1, nullptr, 0, BH, Lq, Lk, d, scale, O, st);
    return launch_nw<MODE, 2, 1, false>(Q, K, V, nullptr, 1, nullptr, 0, BH, Lq, Lk, d, scale, O, st);
}

template <int MODE>
hipError_t launch_varlen(const void *Q, const void *K, const void *V, const int *key_len, int H, int BH, int Lq, int Lk,
                         int d, float scale, void *O, hipStream_t st) {
    if (Lq % 128 == 0)
        return launch_nw<MODE, 4, 1, false, true>(Q, K, V, nullptr, H, nullptr, 0, BH, Lq, Lk, d, scale, O, st, key_len);
    return launch_nw<MODE, 2, 1, false, true>(Q, K, V, nullptr, H, nullptr, 0, BH, Lq, Lk, d, scale, O, st, key_len);
}

}  // namespace

// Padded batches given by their lengths: key_len int32 [BH / H] (device), Lq a multiple of 64, Lk (the padded length) of 64;
// mode 0 or 1 (full attention on padded batches stays with the key-bias path: this kernel's full-attention form is the
// slower one at most shapes).
hipError_t launch_fused_attention_varlen(const void *Q, const void *K, const void *V, const int *key_len, int H, int BH,
                                         int Lq, int Lk, int d, int mode, float scale, void *O, hipStream_t st) {
    if (mode == 0) return launch_varlen<MODE_2TO4>(Q, K, V, key_len, H, BH, Lq, Lk, d, scale, O, st);
    if (mode == 1) return launch_varlen<MODE_1TO2>(Q, K, V, key_len, H, BH, Lq, Lk, d, scale, O, st);
    return hipErrorInvalidValue;
}

// Lengths that are no tile multiples (any Lq, Lk a multiple of 4), arrays unpadded, no mask; mode 0 or 1; 128-query
// workgroups.
hipError_t launch_fused_attention32_ragged(const void *Q, const void *K, const void *V, int BH, int Lq, int Lk, int d,
                                           int mode, float scale, void *O, hipStream_t st) {
    if (mode == 0)
        return launch_nw<MODE_2TO4, 4, 1, false, false, false, true>(Q, K, V, nullptr, 1, nullptr, 0, BH, Lq, Lk, d, scale, O, st);
    if (mode == 1)
        return launch_nw<MODE_1TO2, 4, 1, false, false, false, true>(Q, K, V, nullptr, 1, nullptr, 0, BH, Lq, Lk, d, scale, O, st);
    return hipErrorInvalidValue;
}

// nw: waves per workgroup (2 or 4); ks: waves that share the keys of one 32-query tile (1, or 2 with nw = 4).
// Lq must be a multiple of 32 * nw / ks, Lk of 64.  key_bias and causal as in launch_fused_attention; with either of
// them nw must be 4 and ks is taken as 1; a block_mask is refused.
hipError_t launch_fused_attention32(const void *Q, const void *K, const void *V, const float *key_bias, int H,
                                    const uint8_t *block_mask, int causal, int BH, int Lq, int Lk, int d, int mode,
                                    int nw, int ks, float scale, void *O, hipStream_t st) {
    if (mode == 0)
        return launch_mode<MODE_2TO4>(Q, K, V, key_bias, H, block_mask, causal, BH, Lq, Lk, d, nw, ks, scale, O, st);
    if (mode == 1)
        return launch_mode<MODE_1TO2>(Q, K, V, key_bias, H, block_mask, causal, BH, Lq, Lk, d, nw, ks, scale, O, st);
    return launch_mode<MODE_DENSE>(Q, K, V, key_bias, H, block_mask, causal, BH, Lq, Lk, d, nw, ks, scale, O, st);
}

}  // namespace dfss
