// The 64-key blocks that a workgroup of the one-kernel forward pass visits, and which of them need the
// bias arithmetic (arXiv 2203.00091 has no masks; App. A.1.2 "Blocked-ELL Sparsity" skips pruned blocks).
//
// Blocks that the block mask prunes, blocks whose 64 keys are all masked by the key bias (-inf) and, under the
// causal mask, blocks past the last visible key of the workgroup's queries contribute exactly nothing and are
// skipped, copies included; blocks whose biases are all zero (with a padding mask: every block but the one
// the sequence ends in) take the arithmetic of the call without bias.  Every wave derives the bitmaps by
// itself (Lk <= 8192, so at most 128 blocks: two 64-bit masks each, in scalar registers; no LDS, no barrier).
#pragma once
#include "dfss_device.hpp"

namespace dfss {

// Bit b of the result = some bit of nibble b of m is set (b = 0 .. 15).
__device__ __forceinline__ uint64_t any_of_4(uint64_t m) {
    m |= m >> 1;
    m |= m >> 2;
    m &= 0x1111111111111111ull;                       // bit 4 b
    m = (m | (m >> 3)) & 0x0303030303030303ull;       // two per byte
    m = (m | (m >> 6)) & 0x000F000F000F000Full;       // four per 16 bits
    m = (m | (m >> 12)) & 0x000000FF000000FFull;      // eight per 32 bits
    return (m | (m >> 24)) & 0xFFFFull;
}

// MASKED = false: every block, in order (a plain counter).
template <bool MASKED, bool RAGGED>
struct BlockList {
    static constexpr int KB = 64;
    uint64_t live_lo = ~0ull, live_hi = ~0ull;   // block is visited
    uint64_t bias_lo = 0ull, bias_hi = 0ull;     // block holds a non-zero bias (or is cut by the causal diagonal)
    int next_plain = 0;
    int nblocks = 0;

    // brow: bias row of the head's batch element (fp32 [Lk]), read if with_bias.  mask_row: the workgroup's row of
    // the block mask (uint8 [nblocks]), read if with_mask.  (The two flags are kernel arguments, the same in every
    // lane; the pointers come out of per-head arithmetic on the vector unit, and a branch on them would make the
    // bitmaps lane-dependent in the compiler's eyes.)  causal: non-zero = query i sees keys 0 .. i + coff.
    // q_first, tq: first query and number of queries of the workgroup.  l: lane.
    __device__ __forceinline__ void init(bool with_bias, const float *brow, bool with_mask, const uint8_t *mask_row,
                                         int causal, int q_first, int tq, int coff, int Lq, int Lk, int nblocks_,
                                         int l) {
        nblocks = nblocks_;
        if constexpr (MASKED) {
        if (with_mask) {   // row of the block mask that belongs to this workgroup's 64 queries
            const uint8_t *row = mask_row;
            live_lo = __ballot(l < nblocks && row[l < nblocks ? l : 0] != 0);
            live_hi = __ballot(64 + l < nblocks && row[64 + l < nblocks ? 64 + l : 0] != 0);
        }
        if (with_bias) {
            // Lane l looks at block l (then 64 + l): 16 float4 loads per lane, all in flight at once, a running
            // maximum (is any key of the block unmasked?) and the OR of the bit patterns (is any bias non-zero?);
            // one ballot each turns the lanes' answers into the block bitmaps.  In a partial last block the loads
            // past the row's end re-read its last float4 (the absent keys are accounted for below).
            uint64_t real_lo = 0ull, real_hi = 0ull;
            if (nblocks <= 16) {
                // Short rows (the usual padded batch): four lanes per block, four loads each -- a quarter of the
                // instructions, which every wave of every workgroup spends before its first block.  The ballots
                // then hold four bits per block; any_of_4 folds them to one.
                const int blk = l >> 2;
                float mx = -INFINITY;
                uint32_t bits = 0u;
                if (blk < nblocks) {
                    const float *bp = brow + KB * blk;
                    const int last = Lk - 4 - KB * blk;
#pragma unroll
                    for (int c = 0; c < KB / 16; ++c) {
                        const int cc = 4 * (KB / 16 * (l & 3) + c);
                        const f32x4 b = *reinterpret_cast<const f32x4 *>(bp + (RAGGED && cc > last ? last : cc));
                        mx = fmaxf(fmaxf(mx, b[0]), b[1]);
                        mx = fmaxf(fmaxf(mx, b[2]), b[3]);
                        bits |= __float_as_uint(b[0]) | __float_as_uint(b[1]);
                        bits |= __float_as_uint(b[2]) | __float_as_uint(b[3]);
                    }
                }
                real_lo = any_of_4(__ballot(__float_as_uint(mx) != 0xFF800000u));
                bias_lo = any_of_4(__ballot((bits & 0x7FFFFFFFu) != 0u));
            } else
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                if (64 * half >= nblocks) break;
                const int blk = 64 * half + l;
                float mx = -INFINITY;
                uint32_t bits = 0u;
                if (blk < nblocks) {
                    const float *bp = brow + KB * blk;
                    const int last = Lk - 4 - KB * blk;   // offset of the row's last float4 from the block's start
#pragma unroll
                    for (int c = 0; c < KB / 4; ++c) {
                        const f32x4 b = *reinterpret_cast<const f32x4 *>(bp + (RAGGED && 4 * c > last ? last : 4 * c));
                        mx = fmaxf(fmaxf(mx, b[0]), b[1]);
                        mx = fmaxf(fmaxf(mx, b[2]), b[3]);
                        bits |= __float_as_uint(b[0]) | __float_as_uint(b[1]);
                        bits |= __float_as_uint(b[2]) | __float_as_uint(b[3]);
                    }
                }
                const uint64_t real = __ballot(__float_as_uint(mx) != 0xFF800000u);   // some key above -inf
                const uint64_t nonzero = __ballot((bits & 0x7FFFFFFFu) != 0u);         // some bias other than +-0
                if (half == 0) real_lo = real, bias_lo = nonzero;
                else real_hi = real, bias_hi = nonzero;
            }
            live_lo &= real_lo, live_hi &= real_hi;
        }
        if (RAGGED && Lk - (nblocks - 1) * KB < KB) {   // the absent keys of a partial last block are masked keys
            if (nblocks <= 64) bias_lo |= 1ull << (nblocks - 1);
            else bias_hi |= 1ull << (nblocks - 65);
        }
        if (causal) {
            // the workgroup's queries q_first .. q_first + tq - 1 see keys up to (their index) + coff: blocks past the last query's
            // diagonal hold nothing; blocks from the first query's diagonal on are cut for some query
            // (the query index comes out of an integer division, which runs on the vector unit: back to a scalar,
            // so that the block list stays in scalar registers)
            const int qt0 = __builtin_amdgcn_readfirstlane(q_first);
            const int q_hi = (qt0 + tq - 1 < Lq ? qt0 + tq - 1 : Lq - 1) + coff;
            const int last_blk = q_hi / KB, first_cut = (qt0 + coff + 1) / KB;   // block of the first hidden key
            if (last_blk < 63) live_lo &= (2ull << last_blk) - 1ull, live_hi = 0ull;
            else if (last_blk == 63) live_hi = 0ull;
            else if (last_blk < 127) live_hi &= (2ull << (last_blk - 64)) - 1ull;
            if (first_cut < 64) bias_lo |= ~0ull << first_cut, bias_hi = ~0ull;
            else if (first_cut < 128) bias_hi |= ~0ull << (first_cut - 64);
        }
            if (nblocks < 64) live_lo &= (1ull << nblocks) - 1ull, live_hi = 0ull;   // only blocks that exist
            else if (nblocks < 128) live_hi &= (1ull << (nblocks - 64)) - 1ull;
        }
    }

    // The blocks still to visit, as a list that is consumed: takes the smallest one off (or returns nblocks).
    __device__ __forceinline__ int take() {
        if constexpr (!MASKED) {
            return next_plain++;
        } else {
            if (live_lo) {
                const int j = __builtin_ctzll(live_lo);
                live_lo &= live_lo - 1ull;
                return j;
            }
            if (live_hi) {
                const int j = __builtin_ctzll(live_hi);
                live_hi &= live_hi - 1ull;
                return 64 + j;
            }
            return nblocks;
        }
    }

    __device__ __forceinline__ bool has_bias(int jb) const {
        if constexpr (!MASKED) return false;
        return ((jb < 64 ? bias_lo >> jb : bias_hi >> (jb - 64)) & 1ull) != 0;
    }
};

}  // namespace dfss
