// Whole DFSS forward pass in one kernel: scores on bf16 MFMA, N:M pruning on the
// accumulators (arXiv 2203.00091, Sec. 3.4), softmax over the kept scores (Sec. 3.1,
// App. A.1.3) and the product with V on the structured-sparse MFMA -- without writing the
// compressed score matrix to memory at all.  It computes the same function as the three
// stage kernels; what differs is only where the intermediate lives.
//
// Why no data movement is needed between the stages: the score tile is formed transposed
// (keys on MFMA rows), so lane (column c, row group g) ends up with the kept values of
// query c for the 16 keys 16g .. 16g+15 of a 64-key block -- which is exactly the A
// operand of v_smfmac_f32_16x16x64_bf16 for row c, contraction chunk g, and the four
// 4-bit position codes are its index operand.
//
// Softmax is done online over key blocks with a lazily updated reference value m per
// query: weights are exp(s - m); m is only raised (and the partial results rescaled) when
// a block's maximum exceeds it by more than kTau, which keeps every weight below e^kTau
// and makes rescaling rare.  softmax(x) does not depend on the reference value, so the
// result is the max-subtracted softmax of App. A.1.3 up to rounding.  The row sums come
// out of the matrix unit as well (an extra all-ones column of V), in the same register
// layout as O, so the final division needs no cross-lane traffic.
//
// The dense variant of the same kernel (no pruning, dense MFMA for P V) is a fused
// full-attention baseline (Eq. 1).
#include <stdlib.h>

#include <type_traits>
#include "block_list.hpp"
#include "dfss_device.hpp"
#include "dfss_internal.h"
#include "dfss_kernels.hpp"

namespace dfss {

namespace {

constexpr int NT = 256;   // threads per workgroup (4 waves)
constexpr int KB = 64;    // keys per block
constexpr float kTau = 8.0f;
constexpr float kLog2e = 1.4426950408889634f;

enum { MODE_2TO4 = 0, MODE_1TO2 = 1, MODE_DENSE = 2 };

// Row blocks of a block pattern that visit more blocks than this are shared between the workgroups of a split launch.
constexpr int kSplitFromBlocks = 16;
constexpr int kSplit = 4;        // workgroups per shared row block in a split launch
constexpr int kSplitSlots = 4;   // row blocks that can be shared

// Split launches: which row blocks are shared is a function of the pattern alone, so every workgroup works it out for
// itself (a key bias may mask some of the blocks; it does not enter).  The first kSplitSlots row blocks that keep more
// than kSplitFromBlocks blocks get the slots 0, 1, ... in row order.
// Blocks kept by row block `row` (one lane per row; 16 bytes at a time where the rows allow).
__device__ __forceinline__ int kept_blocks(const uint8_t *__restrict__ block_mask, int row, int nblocks) {
    const uint8_t *const p = block_mask + (size_t)row * nblocks;
    int kept = 0;
    if (nblocks % 16 == 0 && (reinterpret_cast<uintptr_t>(block_mask) & 15u) == 0) {
        for (int j = 0; j < nblocks; j += 16) {
            const u32x4 v = *reinterpret_cast<const u32x4 *>(p + j);
#pragma unroll
            for (int e = 0; e < 4; ++e) {   // bit 0 of every byte := OR of its bits
                uint32_t t = v[e] | (v[e] >> 4);
                t |= t >> 2;
                t |= t >> 1;
                kept += __builtin_popcount(t & 0x01010101u);
            }
        }
    } else {
        for (int j = 0; j < nblocks; ++j) kept += p[j] != 0;
    }
    return kept;
}
// Lane mask of the long row blocks among rows c .. c + 63 (the whole wave calls).
__device__ __forceinline__ uint64_t long_rows(const uint8_t *__restrict__ block_mask, int c, int nrows, int nblocks, int l) {
    const int kept = c + l < nrows ? kept_blocks(block_mask, c + l, nblocks) : 0;
    return __ballot(kept > kSplitFromBlocks);
}
// Row block that holds slot `slot`, or -1 (the whole wave calls; the result is the same in every lane).
__device__ __forceinline__ int row_of_slot(const uint8_t *__restrict__ block_mask, int slot, int nrows, int nblocks, int l) {
    int given = 0;
    for (int c = 0; c < nrows; c += kWave) {
        uint64_t m = long_rows(block_mask, c, nrows, nblocks, l);
        const int n = __builtin_popcountll(m);
        if (slot < given + n) {
            for (int i = given; i < slot; ++i) m &= m - 1ull;
            return c + __builtin_ctzll(m);
        }
        given += n;
    }
    return -1;
}
// Slot of row block `row` (which is a long one), or -1 if the slots ran out before it.
__device__ __forceinline__ int slot_of_row(const uint8_t *__restrict__ block_mask, int row, int nrows, int nblocks, int l) {
    int before = 0;
    for (int c = 0; c < row; c += kWave) {
        uint64_t m = long_rows(block_mask, c, nrows, nblocks, l);
        if (row - c < kWave) m &= (1ull << (row - c)) - 1ull;
        before += __builtin_popcountll(m);
    }
    return before < kSplitSlots ? before : -1;
}

// Launch order of the general-mask kernel: tiles of th heads x tr row blocks (at most 8 x 8, the workgroups that an XCD
// runs at a time), hts x rts of them, sized evenly so that few places of the last tiles stay empty.
struct MaskTiling {
    unsigned hts, rts, th, tr;
    __host__ __device__ MaskTiling(unsigned heads, unsigned qtiles) {
        hts = (heads + 7) / 8, rts = (qtiles + 7) / 8;
        th = (heads + hts - 1) / hts, tr = (qtiles + rts - 1) / rts;
    }
    __host__ __device__ unsigned workgroups() const { return hts * rts * th * tr; }
};

// MASKED: the call carries a key bias and/or a block mask (either pointer may be null).
// RAGGED (implies MASKED; no block mask): the lengths are not multiples of the tiles.  Q, O hold Lq rows and K, V,
//   key_bias Lk keys (Lk a multiple of 4); the absent keys of the last block count as masked keys and the absent
//   queries of the last tile are computed on a copy of the last query and not stored.
//   key_bias   additive per-key term (fp32, [B][Lk], shared by the H heads of a batch element; -inf masks
//              a key), joined to the scaled score before the selection: as the initial value of the
//              accumulators when the scale is folded into Q, else added after the multiplication by scale.
//   block_mask uint8 [Lq/64][Lk/64], shared by all heads: 64 x 64 blocks of the score matrix with a zero
//              entry are not part of the attention (hybrid blocked-ELL x N:M sparsity, App. A.1.2: the
//              block equals the workgroup tile and pruned blocks are skipped).  Needs 64-query workgroups.
//   causal     (MASKED kernels only) non-zero: query i sees keys 0 .. i + (Lk - Lq) (the queries are the last Lq
//              positions; Lk >= Lq).  The hidden scores count as -inf before the selection.  No array: blocks
//              past the last visible key of the workgroup's queries are skipped like pruned blocks, and in
//              the blocks that the diagonal of some query of the workgroup cuts the hidden scores are
//              overwritten by index.
//   G          key groups (block patterns only).  The workgroup has G x 4 waves: group g takes every G-th block that the
//              64 queries visit (the g-th, G + g-th, ... of the list), through K/V buffers of its own; the G partial
//              results of a query tile are merged through LDS at the end (as the key halves of a split are).
//              A row block that sees every key then costs 1/G of the time, and the rows of a pattern differ widely.
//   SPLIT      (block patterns only) long row blocks are shared between SPLIT workgroups.  The first kSplitSlots row
//              blocks of the pattern that keep more than kSplitFromBlocks blocks have a slot each (row_of_slot,
//              slot_of_row).  The launch holds, first, SPLIT - 1 helper workgroups per head and slot (those of an
//              unused slot leave at once), then one workgroup per head and row block.  The SPLIT workgroups of a
//              shared row block take every SPLIT-th block of its list and write their partial results (reference,
//              row sums, unnormalised O; fp32) to `part` [head][slot][SPLIT][64 x (D + 2)]; k_merge_split forms O.
//              Every other row block is the work of its one workgroup, as in a launch without SPLIT.
//   MASK2D     `key_bias` is an additive mask fp32 [Lq][Lk] shared by all heads (H = the number of heads): entry (i, j) joins
//              the scaled score of query i and key j where the key bias would.  Every block is visited and every
//              block takes the arithmetic with bias; a lane reads the 16 entries of its query and its keys one
//              block ahead.  No block mask, no causal flag.
template <int D, int MODE, int NQ, bool PRESCALE, bool MASKED, bool RAGGED = false, int G = 1, int SPLIT = 1,
          bool MASK2D = false>
__global__ __launch_bounds__(NT * G, 2) void k_fused(const __bf16 *__restrict__ Q, const __bf16 *__restrict__ K,
                                                 const __bf16 *__restrict__ V, const float *__restrict__ key_bias,
                                                 int H, const uint8_t *__restrict__ block_mask, int causal, int Lq,
                                                 int Lk, float scale, uint16_t *__restrict__ O,
                                                 float *__restrict__ part) {
    constexpr int CPR = D / 8;          // 16-byte chunks per row
    constexpr int TILE = KB * CPR;      // chunks per K (or V) block
    constexpr int LPT = TILE / NT;      // direct-to-LDS loads per thread per block and operand
    constexpr int STEPS = D / 32;       // MFMA k-steps of Q K^T
    constexpr int DS = D / 16;          // 16-column tiles of O
    constexpr int TQ = 64 * NQ;         // queries per workgroup
    constexpr bool SPARSE = MODE != MODE_DENSE;
    static_assert(!RAGGED || MASKED, "ragged lengths use the masking machinery");
    static_assert(G == 1 || (MASKED && !RAGGED && NQ == 1), "key groups: block patterns on 64-query workgroups");
    static_assert(SPLIT == 1 || (MASKED && !RAGGED && NQ == 1 && G == 1), "split rows: block patterns, 64-query workgroups");
    static_assert(!MASK2D || (MASKED && NQ == 1 && G == 1 && SPLIT == 1), "general mask: 64-query workgroups, no groups");
    // per key group: two K buffers, then two V buffers; MASK_LDS: then 16 rows x 64 entries of the mask per wave
    constexpr bool MASK_LDS = MASK2D && D == 64;
    __shared__ u32x4 Smem[G * 4 * TILE + (MASK_LDS ? 4 * 256 : 0)];

    const int tid = threadIdx.x & (NT - 1);   // within the key group
    const int w = tid >> 6, l = tid & 63, li = l & 15, kb = l >> 4;
    const int g = G > 1 ? __builtin_amdgcn_readfirstlane((int)threadIdx.x / NT) : 0;
    u32x4 *const Ks = Smem + g * (4 * TILE), *const Vs = Ks + 2 * TILE;

    const unsigned qtiles = (Lq + TQ - 1) / TQ;
    int qt, bh;
    int sp = 0, stride = 1, slot = -1;   // SPLIT: place among the workgroups that share the row block; their number; the slot
    [[maybe_unused]] int first_blk = 0, visits = 0;   // MASK2D: the block this workgroup starts at; blocks taken so far
    if constexpr (SPLIT > 1) {
        const int nblk = Lk / KB, lane = threadIdx.x & 63;
        const unsigned heads = gridDim.x / (kSplitSlots * (SPLIT - 1) + qtiles);
        const unsigned helpers = heads * kSplitSlots * (SPLIT - 1);
        if (blockIdx.x < helpers) {   // (the helpers come first in launch order: they belong to the longest row blocks)
            slot = blockIdx.x / (heads * (SPLIT - 1));
            const unsigned rest = blockIdx.x % (heads * (SPLIT - 1));
            sp = 1 + rest / heads;
            bh = rest % heads;
            qt = __builtin_amdgcn_readfirstlane(row_of_slot(block_mask, slot, qtiles, nblk, lane));
            if (qt < 0) return;   // unused slot
            stride = SPLIT;
        } else {
            const unsigned row = blockIdx.x - helpers;   // row block 0 of every head, then row block 1, ...
            qt = row / heads;
            bh = row % heads;
            const uint8_t *const mine = block_mask + (size_t)qt * nblk;
            const int kept = __builtin_popcountll(__ballot(lane < nblk && mine[lane < nblk ? lane : 0] != 0)) +
                             __builtin_popcountll(__ballot(64 + lane < nblk && mine[64 + lane < nblk ? 64 + lane : 0] != 0));
            if (kept > kSplitFromBlocks) {
                slot = __builtin_amdgcn_readfirstlane(slot_of_row(block_mask, qt, qtiles, nblk, lane));
                if (slot >= 0) stride = SPLIT;
            }
        }
    } else if (MASKED && !MASK2D && (block_mask || causal)) {
        // Row blocks of a block pattern differ widely in work (rows that see every key next to rows
        // that see a window), and the heavy ones usually come first: hand out row block 0 of every
        // head, then row block 1, ... in launch order, so that the long workgroups start at once.
        // Under the causal mask the work grows with the row block: the last one of every head goes first.
        const unsigned heads = gridDim.x / qtiles;
        qt = blockIdx.x / heads;
        if (causal && !block_mask) qt = qtiles - 1 - qt;
        bh = blockIdx.x % heads;
    } else if (MASK2D) {
        // Workgroups that run side by side on an XCD form a tile of heads x row blocks (MaskTiling): the heads of a
        // row block read the same rows of the mask and the row blocks of a head the same K and V, so that both come
        // out of that XCD's L2 most of the time.  H carries the number of heads (B * H of the call).
        const MaskTiling T(H, qtiles);
        const unsigned item = xcd_contiguous(blockIdx.x, gridDim.x);
        const unsigned tile = item / (T.th * T.tr), in = item % (T.th * T.tr);
        bh = (tile % T.hts) * T.th + in % T.th;
        qt = (tile / T.hts) * T.tr + in / T.th;
        if (bh >= H || qt >= (int)qtiles) return;   // the tiles overhang the grid of heads x row blocks
        // Row block qt starts at key block qt (mod their number) and wraps around -- the order of the blocks does not
        // matter to Sec. 3.1's softmax.  The heads of a row block stay in step (they share its mask rows through the
        // L2); the row blocks, whose mask rows are a power of two apart for the usual lengths, no longer read the same
        // few memory channels at the same time.
        first_blk = __builtin_amdgcn_readfirstlane(qt % ((Lk + KB - 1) / KB));
    } else {
        const unsigned item = xcd_contiguous(blockIdx.x, gridDim.x);
        qt = item % qtiles;
        bh = item / qtiles;
    }
    const int q0 = qt * TQ + w * 16 * NQ;
    const int nblocks = (Lk + KB - 1) / KB;
    const int tail_keys = Lk - (nblocks - 1) * KB;   // keys of the last block (KB unless the lengths are ragged)
    const int coff = Lk - Lq;                        // causal: query i sits at position i + coff

    const __bf16 *Kh = K + (size_t)bh * Lk * D;
    const __bf16 *Vh = V + (size_t)bh * Lk * D;

    // K block in LDS: row slot 16 t + i holds key 16 (i/4) + 4 t + i%4 (tile t, MFMA row i), chunk c
    // at position slot * CPR + (c ^ (slot & 7)).  V block: row = key, chunk c at row * CPR + (c ^ tr_row_swizzle(row)).
    int k_off[LPT], v_off[LPT];
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
        const int p = i * NT + tid;
        const int slot = p / CPR;
        const int key = (slot & 3) | (((slot >> 4) & 3) << 2) | (((slot >> 2) & 3) << 4);
        k_off[i] = key * D + ((p % CPR) ^ (slot & 7)) * 8;
        v_off[i] = slot * D + ((p % CPR) ^ tr_row_swizzle<CPR>(slot)) * 8;
    }
    const uint32_t lds_k = lds_address(&Ks[w * 64]), lds_v = lds_address(&Vs[w * 64]);
    const uint64_t k_base = uniform_address(Kh), v_base = uniform_address(Vh);
    auto issue_block = [&](int jb, int buf) {
        const uint64_t ks = k_base + (uint64_t)jb * (KB * D * 2);
        const uint64_t vs = v_base + (uint64_t)jb * (KB * D * 2);
        if (RAGGED && jb == nblocks - 1 && tail_keys < KB) {
            // partial last block: the places of the absent keys are filled with the block's last key (never
            // read past the arrays); those keys are masked below, so what is copied there is never used
#pragma unroll
            for (int i = 0; i < LPT; ++i) {
                const int p = i * NT + tid, slot = p / CPR;
                const int key = (slot & 3) | (((slot >> 4) & 3) << 2) | (((slot >> 2) & 3) << 4);
                const int kc = key < tail_keys ? key : tail_keys - 1, vc = slot < tail_keys ? slot : tail_keys - 1;
                async_copy16(ks, 2u * (kc * D + ((p % CPR) ^ (slot & 7)) * 8), lds_k + 16u * (buf * TILE + i * NT));
                async_copy16(vs, 2u * (vc * D + ((p % CPR) ^ tr_row_swizzle<CPR>(slot)) * 8), lds_v + 16u * (buf * TILE + i * NT));
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < LPT; ++i) async_copy16(ks, 2u * k_off[i], lds_k + 16u * (buf * TILE + i * NT));
#pragma unroll
        for (int i = 0; i < LPT; ++i) async_copy16(vs, 2u * v_off[i], lds_v + 16u * (buf * TILE + i * NT));
    };

    // Blocks to visit (block_list.hpp): pruned, fully masked and causally hidden blocks are skipped.
    const float *brow = nullptr;    // bias row of this head's batch element
    f32x4 kb4[4];                   // bias of this lane's 16 keys of a block: keys 64 jb + 16 kb + 4 t + r
    BlockList<MASKED, RAGGED> blocks;
    auto init_blocks = [&]() {
        if constexpr (MASK2D) {
            blocks.init(false, nullptr, false, nullptr, 0, qt * TQ, TQ, 0, Lq, Lk, nblocks, l);
        } else if constexpr (MASKED) {
            if (key_bias) brow = key_bias + (size_t)(bh / H) * Lk;
            blocks.init(key_bias != nullptr, brow, block_mask != nullptr, block_mask + (size_t)(qt * TQ / 64) * nblocks,
                        causal, qt * TQ, TQ, coff, Lq, Lk, nblocks, l);
        } else {
            blocks.init(false, nullptr, false, nullptr, 0, 0, TQ, 0, Lq, Lk, nblocks, l);
        }
    };

    if (!MASK2D && g == 0 && stride == 1) issue_block(0, 0);   // block 0 is copied before anything else (with a key bias or a pattern: speculatively)

    // Q operand (B side of Q K^T): lane (column li, chunk kb) of step s holds Q[q][32 s + 8 kb .. +7]
    bf16x8 bq[NQ][STEPS];
#pragma unroll
    for (int qs = 0; qs < NQ; ++qs)
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            int qrow = q0 + 16 * qs + li;
            if (RAGGED && qrow >= Lq) qrow = Lq - 1;   // absent query of a ragged last tile: computed, not stored
            const u32x4 raw = *reinterpret_cast<const u32x4 *>(Q + ((size_t)bh * Lq + qrow) * D + 32 * s + 8 * kb);
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

    // running state.  m: reference value of the query in column li (same in the four lanes
    // that share the column).  acc_o / acc_l: O and row sums, rows 4 kb + r of the 16-query tile.
    float m_ref[NQ];
    f32x4 acc_o[NQ][DS], acc_l[NQ];
#pragma unroll
    for (int qs = 0; qs < NQ; ++qs) {
        m_ref[qs] = -1.0e30f;   // below any real score, and small enough that exp2((-inf) - m_ref) is 0, not NaN
        acc_l[qs] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ds = 0; ds < DS; ++ds) acc_o[qs][ds] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const uint32_t one2 = 0x3F803F80u;  // two bfloat16 ones
    const bf16x8 ones8 = __builtin_bit_cast(bf16x8, u32x4{one2, one2, one2, one2});

    const int tr_row = li >> 2, tr_sub = (li >> 1) & 1, tr_byte = 8 * (li & 1);

    init_blocks();
    // The next block of this wave's key group: G blocks come off the list, one per group.  `lead` is group 0's,
    // the first of the G: while it exists the round exists, and every group passes the round's barrier.
    int lead_n = 0;
    auto take_live = [&]() -> int {
        if constexpr (MASK2D) {
            const int j = first_blk + visits;
            lead_n = visits < nblocks ? (j < nblocks ? j : j - nblocks) : nblocks;
            ++visits;
            return lead_n;
        } else if constexpr (G == 1 && SPLIT == 1) {
            return lead_n = blocks.take();
        } else if constexpr (SPLIT > 1) {
            int mine = nblocks;
            for (int i = 0; i < stride; ++i) {
                const int j = blocks.take();
                if (i == sp) mine = j;
            }
            return lead_n = __builtin_amdgcn_readfirstlane(mine);   // (the same in every lane; said to the compiler)
        } else {
            int mine = nblocks;
#pragma unroll
            for (int i = 0; i < G; ++i) {
                const int j = blocks.take();
                if (i == 0) lead_n = j;
                if (i == g) mine = j;
            }
            return mine;
        }
    };
    int jb = take_live();
    int lead = lead_n;
    int jn = take_live();   // the block after this one
    // block 0 (copied speculatively at the top) turned out to be fully masked: overwrite the buffer
    // with the first live block (the two copies of a wave complete in issue order)
    if (MASKED && (MASK2D || g != 0 || stride > 1 || jb != 0) && jb < nblocks) issue_block(jb, 0);

    // General mask.  d = 64 (MASK_LDS): the 16 x 64 entries of a wave's queries and a block's keys are read as whole
    // rows -- load i of lane l: row 4 i + l / 16, 16-byte piece l % 16, so that a load covers four runs of 256
    // contiguous bytes and every line is fetched once -- one block ahead, into registers; at the top of the block they
    // pass through the wave's own LDS rows (piece c of row r at place c ^ r: no bank conflicts either way) to the
    // lanes that own the scores (measured at 4096 keys: 239 against 252 us; at 4000: 208 against 230).  d = 128: the
    // lane reads the 16 entries of its own query and keys (four 16-byte pieces; with the LDS passage 8 % slower
    // there).  An absent query of a ragged last tile reads the last row; the absent keys of a partial last block are
    // masked.
    [[maybe_unused]] const float *mrow[4] = {nullptr, nullptr, nullptr, nullptr};
    [[maybe_unused]] f32x4 kbn[4];
    [[maybe_unused]] u32x4 *const Ms = Smem + G * 4 * TILE + w * 256;
    [[maybe_unused]] auto load_mask = [&](int blk) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int key = KB * blk + (MASK_LDS ? 4 * (l & 15) : 16 * kb + 4 * i);
            kbn[i] = f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
            if (!RAGGED || key < Lk) kbn[i] = *reinterpret_cast<const f32x4 *>(mrow[MASK_LDS ? i : 0] + key);
        }
    };
    if constexpr (MASK2D) {
#pragma unroll
        for (int i = 0; i < (MASK_LDS ? 4 : 1); ++i) {
            int qrow = q0 + (MASK_LDS ? 4 * i + (l >> 4) : li);
            if (RAGGED && qrow >= Lq) qrow = Lq - 1;
            mrow[i] = key_bias + (size_t)qrow * Lk;
        }
        if (jb < nblocks) load_mask(jb);
    }

    for (int it = 0; lead < nblocks; ++it) {
        const int buf = it & 1;
        wait_async_copies();  // vmcnt(0): this block's copies have landed
        __syncthreads();
        if (jn < nblocks) issue_block(jn, buf ^ 1);
        if (G > 1 && jb >= nblocks) {   // this group has no block in the last round
            jb = jn, lead = lead_n;
            jn = take_live();
            continue;
        }

        // ---- scores: acc[qs][t][r] = s(query q0 + 16 qs + li, key 64 jb + 16 kb + 4 t + r) ----
        bool with_bias = false;   // does this block hold a non-zero bias?
        if constexpr (MASK2D) with_bias = true;
        else if constexpr (MASKED) with_bias = blocks.has_bias(jb);
        f32x4 acc[NQ][4];
        auto scores = [&](auto init_from_bias) {
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                bf16x8 ak[4];
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    ak[t] = __builtin_bit_cast(bf16x8, Ks[buf * TILE + (16 * t + li) * CPR + ((4 * s + kb) ^ (li & 7))]);
#pragma unroll
                for (int qs = 0; qs < NQ; ++qs)
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        f32x4 c = acc[qs][t];
                        if (s == 0) c = decltype(init_from_bias)::value ? kb4[t] : f32x4{0.f, 0.f, 0.f, 0.f};
                        acc[qs][t] = mfma16(ak[t], bq[qs][s], c);
                    }
            }
        };
        if (MASKED && with_bias) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int key = KB * jb + 16 * kb + 4 * t;
                if constexpr (MASK2D) {
                    // (filled below)
                } else if constexpr (RAGGED) {
                    if (key >= Lk) kb4[t] = f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
                    else if (brow) kb4[t] = *reinterpret_cast<const f32x4 *>(brow + key);
                    else kb4[t] = f32x4{0.f, 0.f, 0.f, 0.f};
                } else {
                    kb4[t] = brow ? *reinterpret_cast<const f32x4 *>(brow + key) : f32x4{0.f, 0.f, 0.f, 0.f};
                }
            }
            if constexpr (MASK2D) {
                if constexpr (MASK_LDS) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int row = 4 * i + (l >> 4);
                        Ms[row * 16 + ((l & 15) ^ row)] = __builtin_bit_cast(u32x4, kbn[i]);
                    }
                    wave_lds_sync();
#pragma unroll
                    for (int t = 0; t < 4; ++t) kb4[t] = __builtin_bit_cast(f32x4, Ms[li * 16 + ((4 * kb + t) ^ li)]);
                } else {
#pragma unroll
                    for (int t = 0; t < 4; ++t) kb4[t] = kbn[t];
                }
                if (jn < nblocks) load_mask(jn);   // the next block's entries travel under this block's arithmetic
            }
            if constexpr (PRESCALE) {
                scores(std::true_type{});    // bias = initial value of the accumulators
            } else {
                scores(std::false_type{});   // two roundings (product, then sum), never a fused multiply-add
#pragma unroll
                for (int qs = 0; qs < NQ; ++qs)
#pragma unroll
                    for (int t = 0; t < 4; ++t)
#pragma unroll
                        for (int r = 0; r < 4; ++r) acc[qs][t][r] = add_unfused(acc[qs][t][r] * scale, kb4[t][r]);
            }
        } else {
            scores(std::false_type{});
            if constexpr (!PRESCALE) {
#pragma unroll
                for (int qs = 0; qs < NQ; ++qs)
#pragma unroll
                    for (int t = 0; t < 4; ++t) acc[qs][t] = acc[qs][t] * scale;
            }
        }

        if constexpr (MASKED) {
            // causal: the scores of keys after the query's own position count as -inf
            // (q0 is the same in every lane of the wave; as a scalar, the test is a branch around the masking)
            if (causal && KB * jb + KB - 1 > __builtin_amdgcn_readfirstlane(q0) + coff) {   // the wave's first query has hidden keys here
                asm volatile("" ::: "memory");   // (not to be turned into selects that every block would execute)
#pragma unroll
                for (int qs = 0; qs < NQ; ++qs) {
                    const int lim = q0 + 16 * qs + li + coff - (KB * jb + 16 * kb);   // key offsets above it are hidden
#pragma unroll
                    for (int t = 0; t < 4; ++t)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            if (4 * t + r > lim) acc[qs][t][r] = -INFINITY;
                }
            }
        }

        // ---- prune, block maximum ----
        float kept[NQ][SPARSE ? 8 : 16];
        uint32_t idx[NQ];
        float m_blk[NQ];
#pragma unroll
        for (int qs = 0; qs < NQ; ++qs) {
            idx[qs] = 0;
            m_blk[qs] = -3.0e38f;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const f32x4 a = acc[qs][t];   // scaled (and biased) above, outside any per-block condition
                if constexpr (SPARSE) {
                    float lo, hi;
                    uint32_t code;
                    if constexpr (MODE == MODE_2TO4) select_2of4(a[0], a[1], a[2], a[3], 4 * t, lo, hi, code);
                    else select_1of2(a[0], a[1], a[2], a[3], 4 * t, lo, hi, code);
                    kept[qs][2 * t] = lo;
                    kept[qs][2 * t + 1] = hi;
                    idx[qs] |= code;
                    m_blk[qs] = fmaxf(fmaxf(m_blk[qs], lo), hi);   // one v_max3_f32
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r) kept[qs][4 * t + r] = a[r];
                    m_blk[qs] = fmaxf(m_blk[qs], fmaxf(fmaxf(a[0], a[1]), fmaxf(a[2], a[3])));
                }
            }
        }

        // ---- raise the reference value where a block outgrew it (rare after the first block) ----
        // Every lane tests its own 16 keys; only when some lane of the wave sees a score above
        // reference + tau are the maxima of the four lanes kb = 0..3 of a column (different keys of the
        // same query) combined, so that the common path has no cross-lane traffic.
        bool raise = false;
#pragma unroll
        for (int qs = 0; qs < NQ; ++qs) raise |= m_blk[qs] > m_ref[qs] + kTau;
        if (__any(raise)) {
#pragma unroll
            for (int qs = 0; qs < NQ; ++qs) {
                float mb = m_blk[qs];
                mb = fmaxf(mb, __shfl_xor(mb, 16, 64));
                mb = fmaxf(mb, __shfl_xor(mb, 32, 64));
                const bool up = mb > m_ref[qs] + kTau;
                const float m_new = up ? mb : m_ref[qs];
                const float alpha = __builtin_amdgcn_exp2f((m_ref[qs] - m_new) * kLog2e);  // 1 where unchanged
                m_ref[qs] = m_new;
                // rows of acc_o/acc_l are queries 4 kb + r: fetch their factors from the lanes of that column
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float a_r = __shfl(alpha, 4 * kb + r, 64);
                    acc_l[qs][r] *= a_r;
#pragma unroll
                    for (int ds = 0; ds < DS; ++ds) acc_o[qs][ds][r] *= a_r;
                }
            }
        }

        // ---- weights exp(s - m), packed as the A operand of the second product ----
        uint32_t pk[NQ][SPARSE ? 4 : 8];
#pragma unroll
        for (int qs = 0; qs < NQ; ++qs) {
            const float mb = m_ref[qs] * kLog2e;
#pragma unroll
            for (int e = 0; e < (SPARSE ? 4 : 8); ++e) {
                const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(kept[qs][2 * e], kLog2e, -mb));
                const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(kept[qs][2 * e + 1], kLog2e, -mb));
                pk[qs][e] = pack_bf16x2(p0, p1);
            }
        }

        // ---- O += P V ; row sums += P 1 ----
        const char *vbase = reinterpret_cast<const char *>(&Vs[buf * TILE]);
        auto tr = [&](int key0, int ds) {
            const int row = key0 + tr_row;
            const int chunk = (2 * ds + tr_sub) ^ tr_row_swizzle<CPR>(row);
            return lds_read_tr16(vbase + (row * CPR + chunk) * 16 + tr_byte);
        };
        if constexpr (SPARSE) {
            // contraction index k of the sparse instruction = key of the block; B lane (column, kb)
            // holds keys 8 kb .. +7 and 32 + 8 kb .. +7
#pragma unroll
            for (int ds = 0; ds < DS; ++ds) {
                const s16x4 t0 = tr(8 * kb, ds), t1 = tr(8 * kb + 4, ds), t2 = tr(32 + 8 * kb, ds),
                            t3 = tr(36 + 8 * kb, ds);
                const s16x8 lo = __builtin_shufflevector(t0, t1, 0, 1, 2, 3, 4, 5, 6, 7);
                const s16x8 hi = __builtin_shufflevector(t2, t3, 0, 1, 2, 3, 4, 5, 6, 7);
                const bf16x16 b = __builtin_bit_cast(
                    bf16x16, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15));
#pragma unroll
                for (int qs = 0; qs < NQ; ++qs) {
                    const bf16x8 a = __builtin_bit_cast(bf16x8, u32x4{pk[qs][0], pk[qs][1], pk[qs][2], pk[qs][3]});
                    acc_o[qs][ds] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(a, b, acc_o[qs][ds], (int)idx[qs], 0, 0);
                }
            }
#pragma unroll
            for (int qs = 0; qs < NQ; ++qs) {
                const bf16x8 a = __builtin_bit_cast(bf16x8, u32x4{pk[qs][0], pk[qs][1], pk[qs][2], pk[qs][3]});
                acc_l[qs] = mfma16(a, ones8, acc_l[qs]);   // (against ones the positions do not matter: dense instruction)
            }
        } else {
            // dense: MFMA m (0/1) contracts the lane's keys 16 kb + 8 m .. +7
#pragma unroll
            for (int m = 0; m < 2; ++m) {
#pragma unroll
                for (int ds = 0; ds < DS; ++ds) {
                    const s16x4 t0 = tr(16 * kb + 8 * m, ds), t1 = tr(16 * kb + 8 * m + 4, ds);
                    const bf16x8 b = __builtin_bit_cast(bf16x8, __builtin_shufflevector(t0, t1, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
                    for (int qs = 0; qs < NQ; ++qs) {
                        const bf16x8 a = __builtin_bit_cast(
                            bf16x8, u32x4{pk[qs][4 * m], pk[qs][4 * m + 1], pk[qs][4 * m + 2], pk[qs][4 * m + 3]});
                        acc_o[qs][ds] = mfma16(a, b, acc_o[qs][ds]);
                    }
                }
#pragma unroll
                for (int qs = 0; qs < NQ; ++qs) {
                    const bf16x8 a = __builtin_bit_cast(
                        bf16x8, u32x4{pk[qs][4 * m], pk[qs][4 * m + 1], pk[qs][4 * m + 2], pk[qs][4 * m + 3]});
                    acc_l[qs] = mfma16(a, ones8, acc_l[qs]);
                }
            }
        }
        jb = jn, lead = lead_n;
        jn = take_live();
    }
    if constexpr (MASKED) wait_async_copies();   // (only matters if no block was live: the speculative copy)

    if constexpr (SPLIT > 1) {
        if (stride > 1) {
            // ---- shared row block: this workgroup's partial result goes to `part` (k_merge_split forms O) ----
            // per (row block, sp): reference of the 64 queries, their row sums, then O [64][D], all fp32 and relative
            // to the workgroup's own reference
            float *const P = part + ((size_t)(bh * kSplitSlots + slot) * SPLIT + sp) * (64 * (D + 2));
            if (kb == 0) P[16 * w + li] = m_ref[0];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int q = 16 * w + 4 * kb + r;
                if (li == 0) P[64 + q] = acc_l[0][r];
#pragma unroll
                for (int ds = 0; ds < DS; ++ds) P[128 + q * D + 16 * ds + li] = acc_o[0][ds][r];
            }
            return;
        }
    }

    if constexpr (G > 1) {
        // ---- merge the key groups: groups 1 .. G-1 hand (reference, row sums, O) to group 0 through LDS ----
        // Lane for lane (wave w of every group holds the same queries in the same places): value f of a lane at
        // float f * 64 + l of the wave's slot.  The slots lie behind the rows that the store of O stages.
        constexpr int NF = 4 * DS + 5;   // floats per lane
        __syncthreads();   // every wave is done with the K/V buffers
        float *const slots = reinterpret_cast<float *>(Smem + 2 * TILE);
        static_assert((size_t)2 * TILE * 16 + (size_t)(G - 1) * 4 * NF * 64 * 4 <= (size_t)G * 4 * TILE * 16, "the slots fit");
        if (g != 0) {
            float *const mine = slots + ((g - 1) * 4 + w) * (NF * 64) + l;
            mine[0] = m_ref[0];
#pragma unroll
            for (int r = 0; r < 4; ++r) mine[(1 + r) * 64] = acc_l[0][r];
#pragma unroll
            for (int ds = 0; ds < DS; ++ds)
#pragma unroll
                for (int r = 0; r < 4; ++r) mine[(5 + 4 * ds + r) * 64] = acc_o[0][ds][r];
        }
        __syncthreads();
        if (g != 0) return;
#pragma unroll
        for (int h = 1; h < G; ++h) {
            const float *const theirs = slots + ((h - 1) * 4 + w) * (NF * 64) + l;
            const float m_b = theirs[0];
            const float m_new = fmaxf(m_ref[0], m_b);
            const float fa = __builtin_amdgcn_exp2f((m_ref[0] - m_new) * kLog2e);
            const float fb = __builtin_amdgcn_exp2f((m_b - m_new) * kLog2e);
            m_ref[0] = m_new;
            // rows of acc_o/acc_l are queries 4 kb + r: their factors sit in the lanes of that column
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float a_r = __shfl(fa, 4 * kb + r, 64), b_r = __shfl(fb, 4 * kb + r, 64);
                acc_l[0][r] = acc_l[0][r] * a_r + theirs[(1 + r) * 64] * b_r;
#pragma unroll
                for (int ds = 0; ds < DS; ++ds)
                    acc_o[0][ds][r] = acc_o[0][ds][r] * a_r + theirs[(5 + 4 * ds + r) * 64] * b_r;
            }
        }
    }

    // ---- O[q][16 ds + li] = acc_o / row sum, q = q0 + 16 qs + 4 kb + r ----
    // A lane holds single elements of 4 rows; they pass through LDS (the K buffers, free now) so that
    // every lane stores 16 contiguous bytes and a row leaves as one 2 D-byte run.
    if constexpr (G == 1) __syncthreads();   // every wave is done reading K
    constexpr int ROWB = 2 * D + 16;   // padded row: the four lane groups of a column fall into different banks
    char *const stage = reinterpret_cast<char *>(Smem) + w * (16 * ROWB);
    static_assert(4 * 16 * ROWB <= 2 * TILE * 16, "the staging rows fit into the K buffers");
    constexpr int RPP = kWave / CPR;   // rows per read-back pass (CPR lanes x 16 bytes cover a row)
#pragma unroll
    for (int qs = 0; qs < NQ; ++qs) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float inv = __builtin_amdgcn_rcpf(acc_l[qs][r]);   // 1 ulp; the row sum is >= ~1: the reference never exceeds the row maximum
#pragma unroll
            for (int ds = 0; ds < DS; ++ds)
                *reinterpret_cast<uint16_t *>(stage + (4 * kb + r) * ROWB + (16 * ds + li) * 2) =
                    (uint16_t)(pack_bf16x2(acc_o[qs][ds][r] * inv, 0.f) & 0xFFFFu);
        }
        wave_lds_sync();
#pragma unroll
        for (int pass = 0; pass < 16 / RPP; ++pass) {
            const int row = pass * RPP + l / CPR, c = l % CPR;
            const u32x4 v = *reinterpret_cast<const u32x4 *>(stage + row * ROWB + c * 16);
            if (!RAGGED || q0 + 16 * qs + row < Lq)
                *reinterpret_cast<u32x4 *>(O + ((size_t)bh * Lq + q0 + 16 * qs + row) * D + c * 8) = v;
        }
        wave_lds_sync();   // the staging rows are free for the next tile
    }
}

// Block patterns at d = 64: rows of at least this many keys run with two key groups (measured on window + global +
// random patterns: 13.0 against 15.5 us at 1024 keys, 21 against 28 at 2048, 40 against 51 at 4096, where the row
// blocks that see every key set the kernel time; a pattern with no such rows loses about a fifth, 26 against 21 us
// at 4096).  Four groups, or two at d = 128, need the LDS of a whole compute unit: one workgroup per unit, which
// measured slower than no groups at all.
constexpr int kGroupsFromKeys = 1024;

// O of the row blocks that k_fused<..., SPLIT> shared between workgroups: the SPLIT partial results are brought to the
// largest of their references and summed (Sec. 3.1's softmax does not depend on the reference), in a fixed order.
// One workgroup per head and slot.  Thread t: query t / 4, a quarter of the columns.
template <int D, int SPLIT>
__global__ __launch_bounds__(NT) void k_merge_split(const float *__restrict__ part, const uint8_t *__restrict__ block_mask,
                                                    uint16_t *__restrict__ O, int Lq, int Lk) {
    const unsigned qtiles = Lq / 64, heads = gridDim.x / kSplitSlots;
    const unsigned slot = blockIdx.x / heads, bh = blockIdx.x % heads;
    const int qt = row_of_slot(block_mask, slot, qtiles, Lk / KB, threadIdx.x & 63);
    if (qt < 0) return;
    const float *const P = part + (size_t)(bh * kSplitSlots + slot) * SPLIT * (64 * (D + 2));
    const int q = threadIdx.x >> 2, c0 = (threadIdx.x & 3) * (D / 4);
    float m = -3.0e38f;
#pragma unroll
    for (int sp = 0; sp < SPLIT; ++sp) m = fmaxf(m, P[sp * (64 * (D + 2)) + q]);
    float f[SPLIT], sum = 0.f;
#pragma unroll
    for (int sp = 0; sp < SPLIT; ++sp) {
        f[sp] = __builtin_amdgcn_exp2f((P[sp * (64 * (D + 2)) + q] - m) * kLog2e);
        sum += P[sp * (64 * (D + 2)) + 64 + q] * f[sp];
    }
    const float inv = 1.f / sum;
    uint16_t *const out = O + ((size_t)bh * Lq + qt * 64 + q) * D + c0;
#pragma unroll
    for (int c = 0; c < D / 4; c += 8) {
        f32x4 a0 = {0.f, 0.f, 0.f, 0.f}, a1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int sp = 0; sp < SPLIT; ++sp) {
            const f32x4 *const src = reinterpret_cast<const f32x4 *>(P + sp * (64 * (D + 2)) + 128 + q * D + c0 + c);
            a0 += src[0] * f[sp];
            a1 += src[1] * f[sp];
        }
        a0 *= inv, a1 *= inv;
        *reinterpret_cast<u32x4 *>(out + c) = u32x4{pack_bf16x2(a0[0], a0[1]), pack_bf16x2(a0[2], a0[3]),
                                                    pack_bf16x2(a1[0], a1[1]), pack_bf16x2(a1[2], a1[3])};
    }
}

inline bool is_pow2(float x) {
    int e;
    return frexpf(x, &e) == 0.5f;
}

template <int MODE, int NQ, bool MASKED, bool RAGGED = false>
hipError_t launch_nq(const void *Q, const void *K, const void *V, const float *key_bias, int H,
                     const uint8_t *block_mask, int causal, int BH, int Lq, int Lk, int d, float scale, void *O,
                     hipStream_t st) {
    const unsigned grid = (unsigned)((long)BH * ((Lq + 64 * NQ - 1) / (64 * NQ)));
    const bool pre = is_pow2(scale);
#define DFSS_LAUNCH(DD, PRE)                                                                                    \
    hipLaunchKernelGGL((k_fused<DD, MODE, NQ, PRE, MASKED, RAGGED>), dim3(grid), dim3(NT), 0, st,               \
                       (const __bf16 *)Q, (const __bf16 *)K, (const __bf16 *)V, key_bias, H, block_mask, causal, \
                       Lq, Lk, scale, (uint16_t *)O, (float *)nullptr)
    if (d == 64) {
        if (pre) DFSS_LAUNCH(64, true); else DFSS_LAUNCH(64, false);
    } else {
        if (pre) DFSS_LAUNCH(128, true); else DFSS_LAUNCH(128, false);
    }
#undef DFSS_LAUNCH
    return hipGetLastError();
}

// General mask [Lq][Lk]: 64-query workgroups of the kernel for lengths of any kind (whole tiles are a special case).
template <int MODE>
hipError_t launch_mask2d(const void *Q, const void *K, const void *V, const float *mask, int BH, int Lq, int Lk, int d,
                         float scale, void *O, hipStream_t st) {
    const unsigned grid = MaskTiling((unsigned)BH, (unsigned)((Lq + 63) / 64)).workgroups();
    const bool pre = is_pow2(scale);
#define DFSS_LAUNCH(DD, PRE)                                                                                      \
    hipLaunchKernelGGL((k_fused<DD, MODE, 1, PRE, true, true, 1, 1, true>), dim3(grid), dim3(NT), 0, st,          \
                       (const __bf16 *)Q, (const __bf16 *)K, (const __bf16 *)V, mask, BH, (const uint8_t *)nullptr, 0, \
                       Lq, Lk, scale, (uint16_t *)O, (float *)nullptr)
    if (d == 64) {
        if (pre) DFSS_LAUNCH(64, true); else DFSS_LAUNCH(64, false);
    } else {
        if (pre) DFSS_LAUNCH(128, true); else DFSS_LAUNCH(128, false);
    }
#undef DFSS_LAUNCH
    return hipGetLastError();
}

// Block patterns on long rows at d = 64: two key groups.
template <int MODE>
hipError_t launch_groups(const void *Q, const void *K, const void *V, const float *key_bias, int H,
                         const uint8_t *block_mask, int causal, int BH, int Lq, int Lk, int d, float scale, void *O,
                         hipStream_t st) {
    const unsigned grid = (unsigned)((long)BH * (Lq / 64));
    const bool pre = is_pow2(scale);
#define DFSS_LAUNCH(DD, PRE, GG)                                                                                \
    hipLaunchKernelGGL((k_fused<DD, MODE, 1, PRE, true, false, GG>), dim3(grid), dim3(NT * GG), 0, st,          \
                       (const __bf16 *)Q, (const __bf16 *)K, (const __bf16 *)V, key_bias, H, block_mask, causal, \
                       Lq, Lk, scale, (uint16_t *)O, (float *)nullptr)
    if (d != 64) return hipErrorInvalidValue;
    if (pre) DFSS_LAUNCH(64, true, 2); else DFSS_LAUNCH(64, false, 2);
#undef DFSS_LAUNCH
    return hipGetLastError();
}

// Block patterns with a workspace: kSplit workgroups per row block, then the merge of the shared row blocks.
template <int MODE>
hipError_t launch_split(const void *Q, const void *K, const void *V, const float *key_bias, int H,
                        const uint8_t *block_mask, int BH, int Lq, int Lk, int d, float scale, void *O, float *part,
                        hipStream_t st) {
    const unsigned qtiles = Lq / 64;
    const unsigned grid = (unsigned)BH * (kSplitSlots * (kSplit - 1) + qtiles);
    const bool pre = is_pow2(scale);
#define DFSS_LAUNCH(DD, PRE)                                                                                      \
    hipLaunchKernelGGL((k_fused<DD, MODE, 1, PRE, true, false, 1, kSplit>), dim3(grid), dim3(NT), 0, st,          \
                       (const __bf16 *)Q, (const __bf16 *)K, (const __bf16 *)V, key_bias, H, block_mask, 0, Lq, Lk, \
                       scale, (uint16_t *)O, part)
    if (d == 64) {
        if (pre) DFSS_LAUNCH(64, true); else DFSS_LAUNCH(64, false);
        hipLaunchKernelGGL((k_merge_split<64, kSplit>), dim3(BH * kSplitSlots), dim3(NT), 0, st, part, block_mask,
                           (uint16_t *)O, Lq, Lk);
    } else {
        if (pre) DFSS_LAUNCH(128, true); else DFSS_LAUNCH(128, false);
        hipLaunchKernelGGL((k_merge_split<128, kSplit>), dim3(BH * kSplitSlots), dim3(NT), 0, st, part, block_mask,
                           (uint16_t *)O, Lq, Lk);
    }
#undef DFSS_LAUNCH
    return hipGetLastError();
}

}  // namespace

hipError_t launch_fused_attention32(const void *Q, const void *K, const void *V, const float *key_bias, int H,
                                    const uint8_t *block_mask, int causal, int BH, int Lq, int Lk, int d, int mode,
                                    int nw, int ks, float scale, void *O, hipStream_t st);
hipError_t launch_fused_attention32_ragged(const void *Q, const void *K, const void *V, int BH, int Lq, int Lk, int d,
                                           int mode, float scale, void *O, hipStream_t st);

namespace {

template <int MODE>
hipError_t launch(const void *Q, const void *K, const void *V, const float *key_bias, int H,
                  const uint8_t *block_mask, int causal, int BH, int Lq, int Lk, int d, float scale, void *O,
                  int variant, hipStream_t st) {
    // 32 queries per wave when that still leaves at least ~2 workgroups per compute unit
    bool two = Lq % 128 == 0 && (long)BH * (Lq / 128) >= 768;   // at least 3 workgroups per compute unit
    if (variant == DFSS_VARIANT_Q16) two = false;
    if (variant == DFSS_VARIANT_Q16X2) two = Lq % 128 == 0;
    if (block_mask) two = false;   // the block of the mask is the 64-query workgroup tile
    if (Lq % 64 != 0 || Lk % 64 != 0) {   // (never together with a block mask)
        // no mask at all and at least half as many 128-query workgroups as compute units: the 32-query kernel (103
        // against 119 us at 4000 x 4000 with 24 heads, 51 against 61 us with 8; 64 against 96 us at d = 128, 32 heads x
        // 2000).  Rows of fewer than 256 keys stay with the kernel below, which compares full fp32 scores: that
        // kernel's comparison gives up the two lowest mantissa bits, and in a short row the weight that a near-tie
        // decided the other way is large.
        if constexpr (MODE != MODE_DENSE) {
            if (!key_bias && !causal && variant == DFSS_VARIANT_AUTO && Lk >= 256 &&
                (long)BH * ((Lq + 127) / 128) >= 128)
                return launch_fused_attention32_ragged(Q, K, V, BH, Lq, Lk, d, MODE == MODE_2TO4 ? 0 : 1, scale, O, st);
        }
        if ((long)BH * ((Lq + 127) / 128) >= 768)
            return launch_nq<MODE, 2, true, true>(Q, K, V, key_bias, H, nullptr, causal, BH, Lq, Lk, d, scale, O, st);
        return launch_nq<MODE, 1, true, true>(Q, K, V, key_bias, H, nullptr, causal, BH, Lq, Lk, d, scale, O, st);
    }
    if (block_mask && d == 64 && Lk >= kGroupsFromKeys && variant == DFSS_VARIANT_AUTO)
        return launch_groups<MODE>(Q, K, V, key_bias, H, block_mask, causal, BH, Lq, Lk, d, scale, O, st);
    if (key_bias || block_mask || causal) {
        if (two)
            return launch_nq<MODE, 2, true>(Q, K, V, key_bias, H, block_mask, causal, BH, Lq, Lk, d, scale, O, st);
        return launch_nq<MODE, 1, true>(Q, K, V, key_bias, H, block_mask, causal, BH, Lq, Lk, d, scale, O, st);
    }
    if (two) return launch_nq<MODE, 2, false>(Q, K, V, nullptr, 1, nullptr, 0, BH, Lq, Lk, d, scale, O, st);
    return launch_nq<MODE, 1, false>(Q, K, V, nullptr, 1, nullptr, 0, BH, Lq, Lk, d, scale, O, st);
}

}  // namespace

size_t fused_attention_split_workspace_bytes(int BH, int Lq, int d) {
    return (size_t)BH * kSplitSlots * kSplit * 64 * (d + 2) * sizeof(float);
}

hipError_t launch_fused_attention_split_rows(const void *Q, const void *K, const void *V, const float *key_bias, int H,
                                             const uint8_t *block_mask, int BH, int Lq, int Lk, int d, int mode,
                                             float scale, void *O, void *part, hipStream_t st) {
    if (mode == 0) return launch_split<MODE_2TO4>(Q, K, V, key_bias, H, block_mask, BH, Lq, Lk, d, scale, O, (float *)part, st);
    if (mode == 1) return launch_split<MODE_1TO2>(Q, K, V, key_bias, H, block_mask, BH, Lq, Lk, d, scale, O, (float *)part, st);
    return launch_split<MODE_DENSE>(Q, K, V, key_bias, H, block_mask, BH, Lq, Lk, d, scale, O, (float *)part, st);
}

hipError_t launch_fused_attention_mask(const void *Q, const void *K, const void *V, const float *mask, int BH, int Lq,
                                       int Lk, int d, int mode, float scale, void *O, hipStream_t st) {
    if (mode == 0) return launch_mask2d<MODE_2TO4>(Q, K, V, mask, BH, Lq, Lk, d, scale, O, st);
    if (mode == 1) return launch_mask2d<MODE_1TO2>(Q, K, V, mask, BH, Lq, Lk, d, scale, O, st);
    return launch_mask2d<MODE_DENSE>(Q, K, V, mask, BH, Lq, Lk, d, scale, O, st);
}

hipError_t launch_fused_attention(const void *Q, const void *K, const void *V, const float *key_bias, int H,
                                  const uint8_t *block_mask, int causal, int BH, int Lq, int Lk, int d, int mode,
                                  float scale, void *O, int variant, hipStream_t st) {
    // Calls without bias or block pattern on whole tiles take the 32-queries-per-wave kernel, and so do causal calls
    // (callers that name a 16-query tiling get the kernel above).  Its tilings, chosen from the number of 128-query
    // workgroups and the key length (measured): four waves x 32 queries as a rule; two waves per 32-query tile
    // (64-query workgroups, twice as many, each wave half the keys) where the grid is at most one and a half
    // workgroups per compute unit and the keys number 1024 or more (2048 where the grid already gives nearly
    // every compute unit a workgroup of its own); d = 128 always the former (the merge of the
    // two key halves costs more than it gains there).  Full attention
    // (the baseline) runs the 16-query kernel below: the faster of the two at every shape measured (96 heads x 384,
    // 24 heads x 1024 .. 4096, 192 heads x 512, d = 128), the 32-query form being reachable through the test hook.
    const bool masked = key_bias || block_mask || causal;
    // masked calls: the 32-query kernel where it measured faster -- the causal mask on 128-query workgroups (alone: its
    // form without the masking machinery, d = 64 and 128; with a key bias: the masked form, d = 64); a key bias alone
    // and block patterns stay with the kernel above
    const bool masked32 = causal && !block_mask && (d == 64 || !key_bias) && Lq % 128 == 0 && mode != 2;
    const bool tiles = Lq % 64 == 0 && Lk % 64 == 0;
    if (tiles && (!masked || masked32) && variant != DFSS_VARIANT_Q16 && variant != DFSS_VARIANT_Q16X2) {
        const long wg128 = (long)BH * (Lq / 128);
        int nw = Lq % 128 == 0 ? 4 : 2, ks = 1;
        if (variant == DFSS_VARIANT_AUTO && !masked) {
            // the key split doubles the workgroups: it pays while all of them still fit the chip at once (3 x 256
            // four-wave workgroups) and the sequence is long enough to carry the merge of the two halves
            if (mode != 2 && d == 64 && wg128 <= 384 && Lk >= (wg128 > 160 && wg128 <= 256 ? 2048 : 1024)) nw = 4, ks = 2;
            if (mode != 2 && Lq % 128 != 0 && d == 64) nw = 4, ks = 2;   // 64-query workgroups either way
            // ... unless the grid is large: then 128-query workgroups, the last one of a head half empty (the kernel
            // of the unpadded lengths), beat 64-query ones (38.6 against 46.7 us at 24 heads x 2112, 19.3 against
            // 22.8 at 192 x 448, 157 against 199 at d = 128, 64 x 2112; at 216 .. 384 workgroups level or 3-10 % behind)
            if (mode != 2 && Lq % 128 != 0 && (long)BH * (Lq / 128 + 1) > 384)
                return launch_fused_attention32_ragged(Q, K, V, BH, Lq, Lk, d, mode, scale, O, st);
            if (mode == 2) nw = 0;   // full attention: the 16-query kernel measured faster at every shape tried
            if (mode != 2 && d == 128 && Lq % 128 != 0) nw = 0;       // (two-wave workgroups at d = 128: too many registers)
        }
        if (!masked) {
            if (variant == DFSS_VARIANT_Q32W2) nw = 2;
            if (variant == DFSS_VARIANT_Q32W4 && Lq % 128 == 0) nw = 4;
            if (variant == DFSS_VARIANT_Q32K2) nw = 4, ks = 2;
        }
        if (nw != 0)
            return launch_fused_attention32(Q, K, V, key_bias, H, nullptr, causal, BH, Lq, Lk, d, mode, nw, ks, scale, O,
                                            st);
    }
    if (mode == 0)
        return launch<MODE_2TO4>(Q, K, V, key_bias, H, block_mask, causal, BH, Lq, Lk, d, scale, O, variant, st);
    if (mode == 1)
        return launch<MODE_1TO2>(Q, K, V, key_bias, H, block_mask, causal, BH, Lq, Lk, d, scale, O, variant, st);
    return launch<MODE_DENSE>(Q, K, V, key_bias, H, block_mask, causal, BH, Lq, Lk, d, scale, O, variant, st);
}

}  // namespace dfss
