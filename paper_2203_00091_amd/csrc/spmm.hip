// Stage 3 of the DFSS forward pass: O = A_sparse V with the 2:4-compressed attention
// weights (arXiv 2203.00091, Sec. 3.1), on the gfx950 structured-sparse matrix
// instruction v_smfmac_f32_16x16x64_bf16.  Per 128-key block a lane loads the 32 bytes of
// kept weights and the 32-bit metadata word that the same lane of stage 1 stored; the two
// halves of the word are the index operands of two instructions (selected with ABID), so
// nothing is decoded or shuffled.  1:2 pruning is stored with the same codes and runs
// through the same kernel.  The dense variant (P V of Eq. 1, for the baseline) shares the
// V staging and uses v_mfma_f32_16x16x32_bf16.
//
// The SOFTMAX variant takes the kept SCORES of stage 1 instead of weights and applies the softmax
// on the way (Sec. 3.1; the max-subtracted form of App. A.1.3 with a running reference m in the place of the
// maximum): the scores of a block become exp(s - m) in registers before they enter the matrix instruction,
// the accumulators are rescaled when a block exceeds m by more than a threshold, the row sums come from the
// matrix unit too (an all-ones operand), and the result is divided by the sum at the end.  It replaces the separate softmax kernel (one read and one write of all kept values)
// in the two-kernel forward pass.
//
// V blocks (128 keys x d) are copied global -> LDS by the direct-to-LDS load, double
// buffered, row-major with an XOR swizzle of the 16-byte chunks; the B operand (keys along
// the contraction, one d-column per lane) comes from the transposing LDS read.
//
// Which keys an instruction contracts over is free as long as A and B agree.  Sparse
// instruction h (0/1) of a block takes, for its 16-wide contraction chunk c, the keys
// 32c + 16h .. +15 of the block -- the 16 keys whose kept weights lane group c holds in
// half h of its 32 bytes.
#include <cstdlib>
#include "dfss_device.hpp"
#include "dfss_kernels.hpp"

namespace dfss {

namespace {

constexpr int NT = 256;   // 4 waves
constexpr int KB = 128;   // keys per block

// UNPADDED: V holds LkR <= Lk keys per head and O LqR <= Lq rows, while P and meta have the layout of the padded
// lengths Lq (a multiple of 64) and Lk (of 128).  The weights of the absent keys are 0 (their scores were -inf); their
// places in a partial last block of V are filled with the block's last real key, and rows past LqR are not stored.
template <int D, bool SPARSE, int RB, bool SOFTMAX, bool UNPADDED = false>
__global__ __launch_bounds__(NT, 2) void k_av(const uint32_t *__restrict__ P, const uint32_t *__restrict__ meta,
                                              const __bf16 *__restrict__ V, int Lq, int Lk, int LqR, int LkR,
                                              uint16_t *__restrict__ O) {
    constexpr int CPR = D / 8;          // 16-byte chunks per V row
    constexpr int TILE = KB * CPR;      // chunks per V block
    constexpr int LPT = TILE / NT;      // direct-to-LDS loads per thread per block
    constexpr int DS = D / 16;          // 16-column output tiles
    constexpr int TQ = 64 * RB;         // queries per workgroup
    __shared__ u32x4 Vs[2][TILE];

    const int tid = threadIdx.x;
    const int w = tid >> 6, l = tid & 63, li = l & 15, kb = l >> 4;

    const unsigned qtiles = Lq / TQ;
    const unsigned item = xcd_contiguous(blockIdx.x, gridDim.x);
    const int qt = item % qtiles;
    const int bh = item / qtiles;
    const int rb0 = (qt * TQ >> 4) + w * RB;   // first 16-row block of this wave
    const int nblocks = Lk / KB;
    const int meta_slot = ((kb & 1) << 1) | (kb >> 1);   // where the word of 32-key chunk kb sits in a row's 16 bytes

    // LDS position p (16-byte units) = row * CPR + (c ^ ((row & 3) << 1)) holds chunk c of key `row`
    const __bf16 *Vh = V + (size_t)bh * LkR * D;
    int src_off[LPT];
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
        const int p = i * NT + tid;
        const int row = p / CPR, c = (p % CPR) ^ ((row & 3) << 1);
        src_off[i] = row * D + c * 8;
    }
    const uint32_t lds_v = lds_address(&Vs[0][w * 64]);   // this wave's 1 KB slice of copy 0, buffer 0
    auto issue_block = [&](int jb, int buf) {
        const __bf16 *src = Vh + (size_t)jb * KB * D;
        const int real = LkR - jb * KB;   // real keys from this block's first one on
        if (UNPADDED && real < KB) {
#pragma unroll
            for (int i = 0; i < LPT; ++i) {
                const int p = i * NT + tid;
                const int row = p / CPR, c = (p % CPR) ^ ((row & 3) << 1);
                async_copy16(src, 2u * ((row < real ? row : real - 1) * D + c * 8), lds_v + 16u * (buf * TILE + i * NT));
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < LPT; ++i) async_copy16(src, 2u * src_off[i], lds_v + 16u * (buf * TILE + i * NT));
    };

    // A operand of one block
    struct AFrag {
        u32x4 v[SPARSE ? 2 : 4];
        uint32_t idx;
    };
    auto load_a = [&](int jb, AFrag (&a)[RB]) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const size_t row = (size_t)bh * Lq + (size_t)(rb0 + rb) * 16 + li;
            if constexpr (SPARSE) {
                // kept weights of keys 128 jb + 32 kb .. +31: 16 of them, 32 bytes
                const u32x4 *pr = reinterpret_cast<const u32x4 *>(P + row * (size_t)(Lk / 4)) + jb * 8 + kb * 2;
                a[rb].v[0] = pr[0];
                a[rb].v[1] = pr[1];
                a[rb].idx = meta[((((size_t)bh * (Lq / 16) + rb0 + rb) * nblocks + jb) * 16 + li) * 4 + meta_slot];
            } else {
                // dense weights: MFMA m takes keys 128 jb + 32 m + 8 kb .. +7
                const u32x4 *pr = reinterpret_cast<const u32x4 *>(P + row * (size_t)(Lk / 2)) + jb * 16 + kb;
#pragma unroll
                for (int m = 0; m < 4; ++m) a[rb].v[m] = pr[4 * m];
                a[rb].idx = 0;
            }
        }
    };

    f32x4 acc[RB][DS];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int ds = 0; ds < DS; ++ds) acc[rb][ds] = f32x4{0.f, 0.f, 0.f, 0.f};

    // transposing read: lane li of a 16-lane group addresses V[key0 + li/4][col0 + 4*(li%4)]
    const int tr_row = li >> 2;
    const int tr_sub = (li >> 1) & 1;      // which 16-byte chunk of the 32-byte column group
    const int tr_byte = 8 * (li & 1);
    const int tr_xor = tr_row << 1;        // (row & 3) << 1, key0 is a multiple of 4

    // SOFTMAX: reference value of row li of each row block (the same in the four lane groups kb of a row)
    static_assert(!SOFTMAX || SPARSE, "the softmax is folded into the sparse product only");
    constexpr float kLog2e = 1.4426950408889634f;
    constexpr float kTau = 8.0f;   // the running reference of a row is raised when a score exceeds it by more than this
    float m_run[RB];
    f32x4 acc_l[RB];               // row sums, rows 4 kb + r (from the matrix unit: an all-ones B operand)
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) m_run[rb] = -INFINITY, acc_l[rb] = f32x4{0.f, 0.f, 0.f, 0.f};
    const uint32_t one2 = 0x3F803F80u;   // two bfloat16 ones
    const bf16x8 ones8 = __builtin_bit_cast(bf16x8, u32x4{one2, one2, one2, one2});

    // SOFTMAX: turns the kept scores of one block into exp(s - m) in place, m = the row's reference value: the largest
    // score seen when it was last set.  It is raised (and the accumulators, which hold the blocks before, rescaled)
    // only when a score exceeds it by more than kTau, so weights stay below e^kTau and the common block needs no
    // cross-lane traffic; softmax does not depend on m (App. A.1.3 subtracts the row maximum for the same reason).
    auto softmax_block = [&](AFrag (&a)[RB]) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            float x[16];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                x[2 * e] = bf16_lo_to_f32(a[rb].v[0][e]);
                x[2 * e + 1] = bf16_hi_to_f32(a[rb].v[0][e]);
                x[8 + 2 * e] = bf16_lo_to_f32(a[rb].v[1][e]);
                x[8 + 2 * e + 1] = bf16_hi_to_f32(a[rb].v[1][e]);
            }
            float bm = fmaxf(x[0], x[1]);
#pragma unroll
            for (int e = 2; e < 16; e += 2) bm = fmaxf(fmaxf(x[e], x[e + 1]), bm);   // this lane's 16 scores
            // (m_run = -inf, the start: any finite score is above -inf + kTau = -inf)
            if (__builtin_amdgcn_ballot_w64(bm > m_run[rb] + kTau) != 0) {   // rare after the first blocks
                bm = fmaxf(bm, __shfl_xor(bm, 16, kWave));
                bm = fmaxf(bm, __shfl_xor(bm, 32, kWave));   // maximum of row li over the block's 64 kept scores
                const bool up = bm > m_run[rb] + kTau;       // (the same in the four lanes of a row)
                // (a row still at -inf gets the factor 0: its sums are 0 anyway)
                const float f = up ? __builtin_amdgcn_exp2f((m_run[rb] - bm) * kLog2e) : 1.f;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float fr = __shfl(f, 4 * kb + r, kWave);   // accumulator row 4 kb + r
                    acc_l[rb][r] *= fr;
#pragma unroll
                    for (int ds = 0; ds < DS; ++ds) acc[rb][ds][r] *= fr;
                }
                if (up) m_run[rb] = bm;
            }
            // a row whose keys so far are all masked (-inf): subtract 0, its weights are exp(-inf) = 0
            const float mb = m_run[rb] == -INFINITY ? 0.f : m_run[rb] * kLog2e;
#pragma unroll
            for (int e = 0; e < 16; ++e) x[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(x[e], kLog2e, -mb));
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                a[rb].v[0][e] = pack_bf16x2(x[2 * e], x[2 * e + 1]);
                a[rb].v[1][e] = pack_bf16x2(x[8 + 2 * e], x[8 + 2 * e + 1]);
            }
        }
    };

    // The A operand is loaded two blocks ahead: block jb + 1 is in registers while block jb is multiplied, so that the
    // softmax of block jb + 1 runs on the vector unit under the matrix instructions of block jb.
    // Order of the blocks: workgroup g starts at block g mod nblocks and wraps around (neither the product nor the
    // softmax with its running reference depends on the order).  The rows of P are a power of two apart for the usual
    // lengths, so that workgroups marching from block 0 in step would all read the same few memory channels at a time.
    const int rot = __builtin_amdgcn_readfirstlane((int)(item % (unsigned)nblocks));
    auto blk = [&](int it) { return it + rot < nblocks ? it + rot : it + rot - nblocks; };
    issue_block(blk(0), 0);
    AFrag a_cur[RB], a_nxt[RB], a_far[RB];
    load_a(blk(0), a_cur);
    if (nblocks > 1) load_a(blk(1), a_nxt);
    if constexpr (SOFTMAX) softmax_block(a_cur);

    for (int jb = 0; jb < nblocks; ++jb) {   // jb: place in the order
        const int buf = jb & 1;
        wait_async_copies();  // vmcnt(0): this block's V copies and the A loads of the next block are in
        __syncthreads();
        if (jb + 1 < nblocks) issue_block(blk(jb + 1), buf ^ 1);
        if (jb + 2 < nblocks) load_a(blk(jb + 2), a_far);
        const char *vbase = reinterpret_cast<const char *>(&Vs[buf][0]);
        auto tr = [&](int key0, int ds) {
            const int row = key0 + tr_row;
            const int chunk = (2 * ds + tr_sub) ^ tr_xor;
            return lds_read_tr16(vbase + (row * CPR + chunk) * 16 + tr_byte);
        };
        if constexpr (SPARSE) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int k0 = 32 * (kb >> 1) + 16 * h + 8 * (kb & 1);
#pragma unroll
                for (int ds = 0; ds < DS; ++ds) {
                    const s16x4 t0 = tr(k0, ds), t1 = tr(k0 + 4, ds), t2 = tr(64 + k0, ds), t3 = tr(64 + k0 + 4, ds);
                    const s16x8 lo = __builtin_shufflevector(t0, t1, 0, 1, 2, 3, 4, 5, 6, 7);
                    const s16x8 hi = __builtin_shufflevector(t2, t3, 0, 1, 2, 3, 4, 5, 6, 7);
                    const bf16x16 b = __builtin_bit_cast(
                        bf16x16, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15));
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb) {
                        const bf16x8 a = __builtin_bit_cast(bf16x8, a_cur[rb].v[h]);
                        if (h == 0)
                            acc[rb][ds] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(a, b, acc[rb][ds],
                                                                                    (int)a_cur[rb].idx, 0, 0);
                        else
                            acc[rb][ds] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(a, b, acc[rb][ds],
                                                                                    (int)a_cur[rb].idx, 0, 1);
                    }
                }
                if constexpr (SOFTMAX) {   // row sums of the (rounded) weights
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb) {
                        const bf16x8 a = __builtin_bit_cast(bf16x8, a_cur[rb].v[h]);
                        // (against ones the positions do not matter: the dense instruction, 32 "keys" per row)
                        acc_l[rb] = mfma16(a, ones8, acc_l[rb]);
                    }
                }
            }
        } else {
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const int k0 = 32 * m + 8 * kb;
#pragma unroll
                for (int ds = 0; ds < DS; ++ds) {
                    const s16x4 t0 = tr(k0, ds), t1 = tr(k0 + 4, ds);
                    const bf16x8 b = __builtin_bit_cast(bf16x8, __builtin_shufflevector(t0, t1, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
                        acc[rb][ds] = mfma16(__builtin_bit_cast(bf16x8, a_cur[rb].v[m]), b, acc[rb][ds]);
                }
            }
        }
        if (jb + 1 < nblocks) {
            if constexpr (SOFTMAX) softmax_block(a_nxt);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) a_cur[rb] = a_nxt[rb], a_nxt[rb] = a_far[rb];
        }
    }

    // acc[rb][ds][r] = O[q][16 ds + li], q = 16 (rb0 + rb) + 4 kb + r
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int qrow = (rb0 + rb) * 16 + 4 * kb + r;
            if (UNPADDED && qrow >= LqR) continue;
            const size_t q = (size_t)bh * LqR + qrow;
            const float ir = SOFTMAX ? 1.0f / acc_l[rb][r] : 1.f;   // (the sum of row 4 kb + r, in every column)
#pragma unroll
            for (int ds = 0; ds < DS; ++ds)
                O[q * D + 16 * ds + li] = (uint16_t)(pack_bf16x2(SOFTMAX ? acc[rb][ds][r] * ir : acc[rb][ds][r], 0.f) & 0xFFFFu);
        }
    }
}

template <bool SPARSE, bool SOFTMAX = false>
hipError_t launch(const void *P, const void *meta, const void *V, int BH, int Lq, int Lk, int LqR, int LkR, int d,
                  void *O, hipStream_t st) {
    if (LqR != Lq || LkR != Lk) {   // unpadded lengths: 64-query workgroups (Lq is a multiple of 64)
        const unsigned grid = (unsigned)((long)BH * (Lq / 64));
#define DFSS_LAUNCH(DD)                                                                                             \
    hipLaunchKernelGGL((k_av<DD, SPARSE, 1, SOFTMAX, true>), dim3(grid), dim3(NT), 0, st, (const uint32_t *)P,     \
                       (const uint32_t *)meta, (const __bf16 *)V, Lq, Lk, LqR, LkR, (uint16_t *)O)
        if (d == 64) DFSS_LAUNCH(64); else DFSS_LAUNCH(128);
#undef DFSS_LAUNCH
        return hipGetLastError();
    }
    // two row blocks per wave when that still leaves two workgroups per compute unit (measured:
    // from there on the larger tile wins, below it the finer grid does)
    bool rb2 = (Lq % 128 == 0) && ((long)BH * (Lq / 128) >= 512);
    const unsigned grid = (unsigned)((long)BH * (Lq / (rb2 ? 128 : 64)));
#define DFSS_LAUNCH(DD, RR)                                                                                   \
    hipLaunchKernelGGL((k_av<DD, SPARSE, RR, SOFTMAX>), dim3(grid), dim3(NT), 0, st, (const uint32_t *)P,              \
                       (const uint32_t *)meta, (const __bf16 *)V, Lq, Lk, Lq, Lk, (uint16_t *)O)
    if (d == 64) {
        if (rb2) DFSS_LAUNCH(64, 2); else DFSS_LAUNCH(64, 1);
    } else {
        if (rb2) DFSS_LAUNCH(128, 2); else DFSS_LAUNCH(128, 1);
    }
#undef DFSS_LAUNCH
    return hipGetLastError();
}

}  // namespace

hipError_t launch_spmm(const void *vals, const void *meta, const void *V, int BH, int Lq, int Lk, int LqR, int LkR, int d,
                       void *O, hipStream_t st) {
    return launch<true>(vals, meta, V, BH, Lq, Lk, LqR, LkR, d, O, st);
}

hipError_t launch_softmax_spmm(const void *scores, const void *meta, const void *V, int BH, int Lq, int Lk, int LqR,
                               int LkR, int d, void *O, hipStream_t st) {
    return launch<true, true>(scores, meta, V, BH, Lq, Lk, LqR, LkR, d, O, st);
}

hipError_t launch_dense_av(const void *P, const void *V, int BH, int Lq, int Lk, int LqR, int LkR, int d, void *O,
                           hipStream_t st) {
    return launch<false>(P, nullptr, V, BH, Lq, Lk, LqR, LkR, d, O, st);
}

}  // namespace dfss
