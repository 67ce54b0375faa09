// Backward pass of DFSS attention through the fixed selection of the forward pass.
//
// The paper finetunes with DFSS attention (arXiv 2203.00091, Sec. 5.1) but describes no backward
// kernel; the selection is treated as a constant of the step, so with P the softmax weights of the
// kept entries (Sec. 3.1) and dO the upstream gradient:
//     dV = P^T dO,   dP = (dO V^T) at the kept positions,   delta_i = dO_i . O_i,
//     dS = P .* (dP - delta),   dQ = scale dS K,   dK = scale dS^T Q.
// Two kernels live here; dQ comes out of the first one at d = 64 and reuses the forward SpMM (stage 3) with K in the
// place of V at d = 128.
//
//   k_masked_sddmm_ds  dS' = scale * P .* (dO V^T - delta) at the kept positions, written in the
//                      compressed layout of the forward pass.  It is the stage-1 mainloop with V in
//                      the place of K and dO in the place of Q; the epilogue picks the kept entries
//                      with the stored position codes instead of selecting them.
//   k_spmm_t           out = A^T X for a compressed A (dV = P^T dO, dK = dS'^T Q).  The contraction
//                      runs over queries, across which the N:M structure does not run, so the tile
//                      of A is expanded to dense bfloat16 in LDS and both operands are read with the
//                      transposing LDS read.
#include <cstdlib>

#include "dfss_device.hpp"
#include "dfss_kernels.hpp"

namespace dfss {

namespace {

constexpr int NT = 256;   // 4 waves
constexpr int KB = 128;   // keys per block

// ------------------------------------------------------------------------------------------------
// out[bh][key][c] = sum_q A[bh][q][key] X[bh][q][c]
// A: kept values bf16 [BH, Lq, Lk/2] + metadata in the library's order; X: bf16 [BH, Lq, D].
// One workgroup owns 128 keys of one head (wave w: keys 32 w .. 32 w + 31, all D columns) and walks
// over the queries 64 at a time.
// ------------------------------------------------------------------------------------------------
// UNP: X holds LqR <= Lq rows per head and out LkR <= Lk rows, while A and meta have the layout of the padded lengths
// Lq (a multiple of 64) and Lk (of 128).  The rows LqR .. Lq - 1 of A hold meaningless entries: they are expanded to
// zeros; the places of the absent rows of a partial last X tile take its last real row; keys past LkR are not stored.
template <int D, bool UNP>
__global__ __launch_bounds__(NT, 2) void k_spmm_t(const uint32_t *__restrict__ A, const uint32_t *__restrict__ meta,
                                                  const __bf16 *__restrict__ X, int Lq, int Lk, int LqR, int LkR,
                                                  uint16_t *__restrict__ out) {
    constexpr int QB = 64;              // queries per step
    constexpr int CPR = D / 8;          // 16-byte chunks per X row
    constexpr int XT = QB * CPR;        // chunks per X tile
    constexpr int LPT = XT / NT;        // asynchronous copies per thread per tile
    constexpr int DS = D / 16;          // 16-column output tiles
    constexpr int AROW = 2 * KB + 16;   // bytes per row of the expanded A tile (padded; three workgroups fit a CU at D = 64)
    __shared__ u32x4 Xs[2][XT];
    __shared__ __attribute__((aligned(16))) char Ad[2][QB * AROW];

    const int tid = threadIdx.x;
    const int w = tid >> 6, l = tid & 63, li = l & 15, g = l >> 4;

    const unsigned kblocks = Lk / KB;
    const unsigned item = xcd_contiguous(blockIdx.x, gridDim.x);
    const int jblk = item % kblocks;
    const int bh = item / kblocks;
    const int nq = Lq / QB;

    // X tile in LDS: row = query, chunk c at row * CPR + (c ^ ((row & 3) << 1))
    const __bf16 *Xh = X + (size_t)bh * LqR * D;
    int src_off[LPT];
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
        const int p = i * NT + tid;
        const int row = p / CPR, c = (p % CPR) ^ ((row & 3) << 1);
        src_off[i] = row * D + c * 8;
    }
    const uint32_t lds_x = lds_address(&Xs[0][w * 64]);
    auto issue_x = [&](int qb, int buf) {
        const __bf16 *src = Xh + (size_t)qb * QB * D;
        const int real = LqR - qb * QB;   // real rows from this tile's first one on
        if (UNP && real < QB) {
#pragma unroll
            for (int i = 0; i < LPT; ++i) {
                const int p = i * NT + tid;
                const int row = p / CPR, c = (p % CPR) ^ ((row & 3) << 1);
                async_copy16(src, 2u * ((row < real ? row : real - 1) * D + c * 8), lds_x + 16u * (buf * XT + i * NT));
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < LPT; ++i) async_copy16(src, 2u * src_off[i], lds_x + 16u * (buf * XT + i * NT));
    };

    // A tile: thread (query aq, chunk ac) expands the 32 keys 128 jblk + 32 ac .. +31 of its query
    const int aq = tid >> 2, ac = tid & 3;
    const int meta_slot = ((ac & 1) << 1) | (ac >> 1);
    struct ARaw {
        u32x4 v0, v1;      // 16 kept values
        uint32_t word;     // their 8 position codes
    };
    auto load_a = [&](int qb) {
        ARaw r;
        const int q = qb * QB + aq;
        const u32x4 *pr = reinterpret_cast<const u32x4 *>(A + ((size_t)bh * Lq + q) * (size_t)(Lk / 4)) + jblk * 8 + ac * 2;
        r.v0 = pr[0];
        r.v1 = pr[1];
        r.word = meta[((((size_t)bh * (Lq / 16) + (q >> 4)) * kblocks + jblk) * 16 + (q & 15)) * 4 + meta_slot];
        return r;
    };
    auto expand_a = [&](const ARaw &r, int buf, int qb) {
        u32x4 *dst = reinterpret_cast<u32x4 *>(&Ad[buf][aq * AROW + ac * 64]);
        if (UNP && qb * QB + aq >= LqR) {   // a row past the end: it takes no part in the sums
#pragma unroll
            for (int i = 0; i < 4; ++i) dst[i] = u32x4{0u, 0u, 0u, 0u};
            return;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {       // 8 keys = 2 groups per 16 bytes
            u32x4 o;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int grp = 2 * i + h;
                const uint32_t kept = grp < 4 ? r.v0[grp] : r.v1[grp - 4];
                const uint32_t lo = kept & 0xFFFFu, hi = kept >> 16;
                const uint32_t code = (r.word >> (4 * grp)) & 0xFu;
                const uint32_t plo = code & 3u, phi = code >> 2;
                const uint32_t k0 = plo == 0 ? lo : 0u;
                const uint32_t k1 = plo == 1 ? lo : (phi == 1 ? hi : 0u);
                const uint32_t k2 = plo == 2 ? lo : (phi == 2 ? hi : 0u);
                const uint32_t k3 = phi == 3 ? hi : 0u;
                o[2 * h] = k0 | (k1 << 16);
                o[2 * h + 1] = k2 | (k3 << 16);
            }
            dst[i] = o;
        }
    };

    f32x4 acc[2][DS];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < DS; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    // transposing reads: lane li of a 16-lane group addresses element [row0 + li/4][col0 + 4 (li%4)]
    const int tr_row = li >> 2;
    const int tr_sub = (li >> 1) & 1, tr_byte = 8 * (li & 1), tr_xor = tr_row << 1;

    // One step = 64 queries.  The compressed operand is loaded two steps ahead into registers (r0 for
    // even steps, r1 for odd ones: fixed names, so no register is copied while its load is in flight),
    // the X tile one step ahead into the other LDS buffer.
    auto step = [&](int qb, ARaw &r) {
        const int buf = qb & 1;
        expand_a(r, buf, qb);
        // X(qb) must have landed; the three loads of A(qb + 1), issued after its copy, may stay in flight
        if (qb >= 1 && qb + 1 < nq) wait_async_copies_keep<3>();
        else wait_async_copies();
        __syncthreads();       // both tiles are complete; the other buffers are free
        if (qb + 1 < nq) issue_x(qb + 1, buf ^ 1);
        if (qb + 2 < nq) r = load_a(qb + 2);
        const char *abase = &Ad[buf][0];
        const char *xbase = reinterpret_cast<const char *>(&Xs[buf][0]);
        auto tr_a = [&](int q0, int col0) {
            return lds_read_tr16(abase + (q0 + tr_row) * AROW + (col0 + 4 * (li & 3)) * 2);
        };
        auto tr_x = [&](int q0, int nt) {
            const int row = q0 + tr_row;
            const int chunk = (2 * nt + tr_sub) ^ tr_xor;   // (row & 3) == tr_row: q0 is a multiple of 4
            return lds_read_tr16(xbase + (row * CPR + chunk) * 16 + tr_byte);
        };
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {     // 32 queries per MFMA step; lane group g takes queries 8 g .. 8 g + 7
            const int q0 = 32 * ks + 8 * g;
            bf16x8 a[2];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                const s16x4 t0 = tr_a(q0, 32 * w + 16 * mt), t1 = tr_a(q0 + 4, 32 * w + 16 * mt);
                a[mt] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(t0, t1, 0, 1, 2, 3, 4, 5, 6, 7));
            }
#pragma unroll
            for (int nt = 0; nt < DS; ++nt) {
                const s16x4 t0 = tr_x(q0, nt), t1 = tr_x(q0 + 4, nt);
                const bf16x8 b = __builtin_bit_cast(bf16x8, __builtin_shufflevector(t0, t1, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) acc[mt][nt] = mfma16(a[mt], b, acc[mt][nt]);
            }
        }
    };

    issue_x(0, 0);
    ARaw r0 = load_a(0), r1 = r0;
    if (nq > 1) r1 = load_a(1);
    for (int qb = 0; qb < nq; qb += 2) {
        step(qb, r0);
        if (qb + 1 < nq) step(qb + 1, r1);
    }

    // acc[mt][nt][r] = out[key 128 jblk + 32 w + 16 mt + 4 g + r][16 nt + li]
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int krow = jblk * KB + 32 * w + 16 * mt + 4 * g + r;
            if (UNP && krow >= LkR) continue;
            const size_t key = (size_t)bh * LkR + krow;
#pragma unroll
            for (int nt = 0; nt < DS; ++nt)
                out[key * D + 16 * nt + li] = (uint16_t)(pack_bf16x2(acc[mt][nt][r], 0.f) & 0xFFFFu);
        }
}

// ------------------------------------------------------------------------------------------------
// dS'[q][c] = scale * P[q][c] * (dO[q] . V[key(q, c)] - delta_q),  delta_q = dO[q] . O[q]
// for the kept entries c of every row, in the compressed layout (same addresses as the weights P).
// Mainloop and data layout of the 16-query stage-1 kernel: keys on the MFMA rows, so lane
// (column li, row group kb) of a 128-key block holds, per half, the 16 consecutive keys
// 32 kb + 16 half .. +15 of query li: four runs of four, of which the position codes name the two
// kept ones.
// ------------------------------------------------------------------------------------------------
// DQ: the same pass also forms dQ = dS' K (the dS' values a lane has just computed ARE the compressed operand of the
// structured-sparse matrix instruction for its query, and the stored position codes its index operand, exactly as
// in the forward SpMM), so dS' is not read back for it.  Needs the whole key range in one workgroup (ksplit = 1) and
// a second LDS tile per block (K in row order for the transposing read): d = 64 only.
// UNP: dO, O, dQ hold LqR <= Lq rows per head and V, K LkR <= Lk keys, while P, meta and dS have the layout of the
// padded lengths.  Rows past LqR are computed on a copy of the last row (their dS' is meaningless and the transposed
// products skip it), the places of absent keys in a partial last block take the block's last key (their weights are
// 0, so their dS' is 0), and rows of dQ past LqR are not stored.
template <int D, int NQ, bool DQ, bool UNP>
__global__ __launch_bounds__(NT, 2) void k_masked_sddmm_ds(const __bf16 *__restrict__ dO, const __bf16 *__restrict__ V,
                                                           const __bf16 *__restrict__ O,
                                                           const uint32_t *__restrict__ P,
                                                           const uint32_t *__restrict__ meta,
                                                           const __bf16 *__restrict__ K, int Lq, int Lk, int LqR,
                                                           int LkR, float scale, int ksplit, int blocks_per_wg,
                                                           uint32_t *__restrict__ dS, uint16_t *__restrict__ dQ) {
    constexpr int CPR = D / 8;           // 16-byte chunks per row
    constexpr int TILE = KB * CPR;       // chunks per V block
    constexpr int LPT = TILE / NT;       // asynchronous copies per thread per block
    constexpr int STEPS = D / 32;        // MFMA k-steps
    constexpr int DS = D / 16;           // 16-column tiles of dQ
    constexpr int TQ = 64 * NQ;          // queries per workgroup
    static_assert(!DQ || D == 64, "the fused dQ needs two LDS tiles per block");
    __shared__ u32x4 Vs[2][TILE];
    __shared__ u32x4 Kr[DQ ? 2 : 1][DQ ? TILE : 1];   // K block, row = key, chunk c at row * CPR + (c ^ ((row & 3) << 1))

    const int tid = threadIdx.x;
    const int w = tid >> 6, l = tid & 63, li = l & 15, kb = l >> 4;

    const unsigned qtiles = Lq / TQ;
    const unsigned item = xcd_contiguous(blockIdx.x, gridDim.x);
    const int ks_id = item % ksplit;
    const int qt = (item / ksplit) % qtiles;
    const int bh = item / (ksplit * qtiles);
    const int jb0 = ks_id * blocks_per_wg;
    const int q0 = qt * TQ + w * 16 * NQ;

    // LDS position p (16-byte units) = slot * CPR + (c ^ (slot & 7)) holds chunk c of the key stored in row
    // slot `slot`; slot 16 t' + i (MFMA tile t', row i) holds key 32 (i/4) + 4 t' + i%4 ... in the order that
    // gives a lane 16 consecutive keys per half
    const __bf16 *Vh = V + (size_t)bh * LkR * D;
    int src_off[LPT];
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
        const int p = i * NT + tid;
        const int slot = p / CPR, c = (p % CPR) ^ (slot & 7);
        const int key = (slot & 3) | (((slot >> 4) & 7) << 2) | (((slot >> 2) & 3) << 5);
        src_off[i] = key * D + c * 8;
    }
    const uint32_t lds_v = lds_address(&Vs[0][w * 64]);
    int k_off[LPT];
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
        const int p = i * NT + tid;
        const int row = p / CPR, c = (p % CPR) ^ ((row & 3) << 1);
        k_off[i] = row * D + c * 8;
    }
    const uint32_t lds_k = lds_address(&Kr[0][DQ ? w * 64 : 0]);
    const __bf16 *Kh = DQ ? K + (size_t)bh * LkR * D : nullptr;
    auto issue_block = [&](int jb, int buf) {
        const __bf16 *src = Vh + (size_t)jb * KB * D;
        const int real = LkR - jb * KB;   // real keys from this block's first one on
        if (UNP && real < KB) {
#pragma unroll
            for (int i = 0; i < LPT; ++i) {
                const int p = i * NT + tid;
                const int slot = p / CPR, c = (p % CPR) ^ (slot & 7);
                const int key = (slot & 3) | (((slot >> 4) & 7) << 2) | (((slot >> 2) & 3) << 5);
                async_copy16(src, 2u * ((key < real ? key : real - 1) * D + c * 8), lds_v + 16u * (buf * TILE + i * NT));
            }
            if constexpr (DQ) {
                const __bf16 *ksrc = Kh + (size_t)jb * KB * D;
#pragma unroll
                for (int i = 0; i < LPT; ++i) {
                    const int p = i * NT + tid;
                    const int row = p / CPR, c = (p % CPR) ^ ((row & 3) << 1);
                    async_copy16(ksrc, 2u * ((row < real ? row : real - 1) * D + c * 8), lds_k + 16u * (buf * TILE + i * NT));
                }
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < LPT; ++i) async_copy16(src, 2u * src_off[i], lds_v + 16u * (buf * TILE + i * NT));
        if constexpr (DQ) {
            const __bf16 *ksrc = Kh + (size_t)jb * KB * D;
#pragma unroll
            for (int i = 0; i < LPT; ++i) async_copy16(ksrc, 2u * k_off[i], lds_k + 16u * (buf * TILE + i * NT));
        }
    };

    issue_block(jb0, 0);

    // dO operand: lane (column li, chunk kb) of MFMA step s holds dO[q][32 s + 8 kb .. +7]; the same
    // elements of O give this lane's share of delta_q
    bf16x8 bq[NQ][STEPS];
    float delta[NQ];
#pragma unroll
    for (int qs = 0; qs < NQ; ++qs) {
        float part = 0.f;
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            const int qrow = UNP && q0 + 16 * qs + li >= LqR ? LqR - 1 : q0 + 16 * qs + li;
            const size_t off = ((size_t)bh * LqR + qrow) * D + 32 * s + 8 * kb;
            const u32x4 g = *reinterpret_cast<const u32x4 *>(dO + off);
            const u32x4 o = *reinterpret_cast<const u32x4 *>(O + off);
            bq[qs][s] = __builtin_bit_cast(bf16x8, g);
#pragma unroll
            for (int e = 0; e < 4; ++e)
                part += bf16_lo_to_f32(g[e]) * bf16_lo_to_f32(o[e]) + bf16_hi_to_f32(g[e]) * bf16_hi_to_f32(o[e]);
        }
        part += __shfl_xor(part, 16, 64);
        part += __shfl_xor(part, 32, 64);
        delta[qs] = part;
    }

    const int rb0 = q0 >> 4;                 // first 16-row block of this wave
    const int meta_slot = ((kb & 1) << 1) | (kb >> 1);

    // DQ: accumulators of dQ (rows 4 kb + r of the 16-query tile, column 16 ds + li) and the lane's role in the
    // transposing read of K (as in the forward SpMM)
    f32x4 acc_dq[NQ][DS];
#pragma unroll
    for (int qs = 0; qs < NQ; ++qs)
#pragma unroll
        for (int ds = 0; ds < DS; ++ds) acc_dq[qs][ds] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int tr_row = li >> 2, tr_sub = (li >> 1) & 1, tr_byte = 8 * (li & 1), tr_xor = tr_row << 1;

    for (int it = 0; it < blocks_per_wg; ++it) {
        const int jb = jb0 + it;
        const int buf = it & 1;
        // this block's copy has landed; the 2 NQ stores of the previous iteration may stay in flight
        if (it == 0) wait_async_copies();
        else wait_async_copies_keep<2 * NQ>();
        __syncthreads();
        if (it + 1 < blocks_per_wg) issue_block(jb + 1, buf ^ 1);

        uint32_t mword[NQ];
#pragma unroll
        for (int qs = 0; qs < NQ; ++qs)
            mword[qs] = meta[((((size_t)bh * (Lq / 16) + rb0 + qs) * (Lk / KB) + jb) * 16 + li) * 4 + meta_slot];

        u32x4 ds_out[2][NQ];   // dS' of both halves: a lane's 32 contiguous bytes, stored together
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int kbase = KB * jb + 32 * kb + 16 * half;
            u32x4 pw[NQ];   // the weights of this lane's 8 kept entries
#pragma unroll
            for (int qs = 0; qs < NQ; ++qs) {
                const size_t row = (size_t)bh * Lq + q0 + 16 * qs + li;
                pw[qs] = *reinterpret_cast<const u32x4 *>(P + (row * (size_t)(Lk / 2) + kbase / 2) / 2);
            }
            f32x4 acc[NQ][4];
#pragma unroll
            for (int qs = 0; qs < NQ; ++qs)
#pragma unroll
                for (int t = 0; t < 4; ++t) acc[qs][t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                bf16x8 av[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int slot = 16 * (4 * half + t) + li;
                    av[t] = __builtin_bit_cast(bf16x8, Vs[buf][slot * CPR + ((4 * s + kb) ^ (li & 7))]);
                }
#pragma unroll
                for (int qs = 0; qs < NQ; ++qs)
#pragma unroll
                    for (int t = 0; t < 4; ++t) acc[qs][t] = mfma16(av[t], bq[qs][s], acc[qs][t]);
            }
            // acc[qs][t][r] = dO[q] . V[key], key = 128 jb + 32 kb + 16 half + 4 t + r
#pragma unroll
            for (int qs = 0; qs < NQ; ++qs) {
                const size_t row = (size_t)bh * Lq + q0 + 16 * qs + li;
                u32x4 o;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const uint32_t code = (mword[qs] >> (16 * half + 4 * t)) & 0xFu;
                    const uint32_t plo = code & 3u, phi = code >> 2;     // plo in {0,1,2}, phi in {1,2,3}
                    const f32x4 a = acc[qs][t];
                    const float dp_lo = plo == 0 ? a[0] : (plo == 1 ? a[1] : a[2]);
                    const float dp_hi = phi == 3 ? a[3] : (phi == 2 ? a[2] : a[1]);
                    const float ds_lo = bf16_lo_to_f32(pw[qs][t]) * (dp_lo - delta[qs]) * scale;
                    const float ds_hi = bf16_hi_to_f32(pw[qs][t]) * (dp_hi - delta[qs]) * scale;
                    o[t] = pack_bf16x2(ds_lo, ds_hi);
                }
                ds_out[half][qs] = o;
                if constexpr (DQ) {
                    // dQ += dS' K over the block's keys 32 c + 16 half .. +15 (c = lane group): instruction `half`
                    const char *kbase_lds = reinterpret_cast<const char *>(&Kr[buf][0]);
                    auto tr = [&](int key0, int ds) {
                        const int krow = key0 + tr_row;
                        const int chunk = (2 * ds + tr_sub) ^ tr_xor;
                        return lds_read_tr16(kbase_lds + (krow * CPR + chunk) * 16 + tr_byte);
                    };
                    const int k0 = 32 * (kb >> 1) + 16 * half + 8 * (kb & 1);
                    const bf16x8 a = __builtin_bit_cast(bf16x8, o);
#pragma unroll
                    for (int ds = 0; ds < DS; ++ds) {
                        const s16x4 t0 = tr(k0, ds), t1 = tr(k0 + 4, ds), t2 = tr(64 + k0, ds), t3 = tr(64 + k0 + 4, ds);
                        const s16x8 lo = __builtin_shufflevector(t0, t1, 0, 1, 2, 3, 4, 5, 6, 7);
                        const s16x8 hi = __builtin_shufflevector(t2, t3, 0, 1, 2, 3, 4, 5, 6, 7);
                        const bf16x16 b = __builtin_bit_cast(
                            bf16x16, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15));
                        if (half == 0)
                            acc_dq[qs][ds] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(a, b, acc_dq[qs][ds],
                                                                                       (int)mword[qs], 0, 0);
                        else
                            acc_dq[qs][ds] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(a, b, acc_dq[qs][ds],
                                                                                       (int)mword[qs], 0, 1);
                    }
                }
            }
        }
        // the two halves of a lane are adjacent in memory (keys 32 kb .. +31 of the row): issued back to back, the
        // four lanes of a row complete a whole 128-byte line
#pragma unroll
        for (int qs = 0; qs < NQ; ++qs) {
            const size_t row = (size_t)bh * Lq + q0 + 16 * qs + li;
            u32x4 *dst = reinterpret_cast<u32x4 *>(dS + (row * (size_t)(Lk / 2) + (KB * jb + 32 * kb) / 2) / 2);
            __builtin_nontemporal_store(ds_out[0][qs], dst);
            __builtin_nontemporal_store(ds_out[1][qs], dst + 1);
        }
    }
    if constexpr (DQ) {
        // acc_dq[qs][ds][r] = dQ[q][16 ds + li], q = q0 + 16 qs + 4 kb + r
#pragma unroll
        for (int qs = 0; qs < NQ; ++qs)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int qrow = q0 + 16 * qs + 4 * kb + r;
                if (UNP && qrow >= LqR) continue;
                const size_t q = (size_t)bh * LqR + qrow;
#pragma unroll
                for (int ds = 0; ds < DS; ++ds)
                    dQ[q * D + 16 * ds + li] = (uint16_t)(pack_bf16x2(acc_dq[qs][ds][r], 0.f) & 0xFFFFu);
            }
    }
}

}  // namespace

hipError_t launch_spmm_t(const void *vals, const void *meta, const void *X, int BH, int Lq, int Lk, int LqR, int LkR,
                         int d, void *out, hipStream_t st) {
    const unsigned grid = (unsigned)((long)BH * (Lk / KB));
    const bool unp = LqR != Lq || LkR != Lk;
#define DFSS_LAUNCH(DD, UU)                                                                                        \
    hipLaunchKernelGGL((k_spmm_t<DD, UU>), dim3(grid), dim3(NT), 0, st, (const uint32_t *)vals, (const uint32_t *)meta, \
                       (const __bf16 *)X, Lq, Lk, LqR, LkR, (uint16_t *)out)
    if (d == 64) {
        if (unp) DFSS_LAUNCH(64, true); else DFSS_LAUNCH(64, false);
    } else {
        if (unp) DFSS_LAUNCH(128, true); else DFSS_LAUNCH(128, false);
    }
#undef DFSS_LAUNCH
    return hipGetLastError();
}

}  // namespace dfss

namespace dfss {

namespace {
template <int NQ, bool UNP>
hipError_t launch_ds_nq(const void *dO, const void *V, const void *O, const void *P, const void *meta, const void *K,
                        int BH, int Lq, int Lk, int LqR, int LkR, int d, float scale, void *dS, void *dQ,
                        hipStream_t st) {
    const int qtiles = Lq / (64 * NQ);
    const int kblocks = Lk / KB;
    const bool with_dq = dQ != nullptr;   // (d = 64: checked by the caller)
    // split the key range until the grid has a few workgroups per compute unit (not with the fused dQ, whose sums
    // run over all keys of a query)
    int ksplit = 1;
    if (!with_dq) {
        while ((long)BH * qtiles * ksplit < 1024 && kblocks % (ksplit * 2) == 0) ksplit *= 2;
        if ((long)BH * qtiles * ksplit < 1024 && kblocks % 3 == 0 && ksplit == 1) ksplit = 3;
    }
    const int per_wg = kblocks / ksplit;
    const unsigned grid = (unsigned)((long)BH * qtiles * ksplit);
#define DFSS_LAUNCH(DD, WITH)                                                                                      \
    hipLaunchKernelGGL((k_masked_sddmm_ds<DD, NQ, WITH, UNP>), dim3(grid), dim3(NT), 0, st, (const __bf16 *)dO,    \
                       (const __bf16 *)V, (const __bf16 *)O, (const uint32_t *)P, (const uint32_t *)meta,         \
                       (const __bf16 *)K, Lq, Lk, LqR, LkR, scale, ksplit, per_wg, (uint32_t *)dS, (uint16_t *)dQ)
    if (d == 64) {
        if (with_dq) DFSS_LAUNCH(64, true); else DFSS_LAUNCH(64, false);
    } else {
        DFSS_LAUNCH(128, false);
    }
#undef DFSS_LAUNCH
    return hipGetLastError();
}
}  // namespace

// K, dQ: both null, or (d = 64 only) the keys and the output of dQ = dS' K, formed in the same pass.
hipError_t launch_masked_sddmm_ds(const void *dO, const void *V, const void *O, const void *P, const void *meta,
                                  const void *K, int BH, int Lq, int Lk, int LqR, int LkR, int d, float scale, void *dS,
                                  void *dQ, hipStream_t st) {
    if (dQ && d != 64) return hipErrorInvalidValue;
    if (LqR != Lq || LkR != Lk) {
        if (Lq % 128 == 0)
            return launch_ds_nq<2, true>(dO, V, O, P, meta, K, BH, Lq, Lk, LqR, LkR, d, scale, dS, dQ, st);
        return launch_ds_nq<1, true>(dO, V, O, P, meta, K, BH, Lq, Lk, LqR, LkR, d, scale, dS, dQ, st);
    }
    if (Lq % 128 == 0) return launch_ds_nq<2, false>(dO, V, O, P, meta, K, BH, Lq, Lk, Lq, Lk, d, scale, dS, dQ, st);
    return launch_ds_nq<1, false>(dO, V, O, P, meta, K, BH, Lq, Lk, Lq, Lk, d, scale, dS, dQ, st);
}

}  // namespace dfss
