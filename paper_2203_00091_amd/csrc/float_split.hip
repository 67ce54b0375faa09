// The 4-byte mode with products formed on the bf16 matrix pipe (arXiv 2203.00091, Sec. 2.3: 1:2 on
// float data; App. A.1.2: float inputs are multiplied on the tensor cores in a shorter-mantissa format
// and accumulated in fp32).  gfx950 has no such format, and its fp32 matrix instruction is sixteen times
// slower than the bf16 one.  Here every fp32 operand x is split into two bfloat16 pieces,
//     hi = bf16(x),  lo = bf16(x - hi),      |x - hi - lo| <= 2^-18 |x|,
// and a product is formed as  a.b ~ a_hi b_hi + a_hi b_lo + a_lo b_hi  (each bf16 x bf16 product is exact
// in fp32; accumulation in fp32).  The dropped terms are bounded by 3 * 2^-18 |a b|: about five more
// mantissa bits than the paper's own multiplication format keeps.  Integer-valued inputs up to 256 have
// lo = 0 and give exactly the fp32 result.
//
// The workgroup converts each 64-row block of K (or V) once: every thread loads its 32-byte pieces of the
// fp32 block into registers one block ahead, splits them, and writes the two bf16 images into LDS, which the
// waves then read as ordinary bf16 matrix operands.  The stage kernels double-buffer the images (one barrier
// per block, the conversion of block j+1 next to the matrix instructions of block j); the one-kernel path
// holds four images per block and keeps a single copy.  The layouts, the 1:2
// epilogue and the metadata are those of the exact fp32 kernels (float_mode.hip).
#include <cstdlib>

#include "dfss_device.hpp"
#include "dfss_kernels.hpp"

namespace dfss {

namespace {

constexpr int NT = 256;   // 4 waves
constexpr int QT = 64;    // queries per workgroup (the score kernel takes 64 NQ)
constexpr int KB = 64;    // keys per block

// x[0..7] -> bf16 images (hi, lo), element e in the low/high half of dword e/2
__device__ __forceinline__ void split8(const f32x4 &x0, const f32x4 &x1, u32x4 &hi, u32x4 &lo) {
    const float x[8] = {x0[0], x0[1], x0[2], x0[3], x1[0], x1[1], x1[2], x1[3]};
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const uint32_t h = pack_bf16x2(x[2 * p], x[2 * p + 1]);
        hi[p] = h;
        // x - bf16(x) is exact in fp32 (it is the discarded low part of the mantissa)
        lo[p] = pack_bf16x2(x[2 * p] - bf16_lo_to_f32(h), x[2 * p + 1] - bf16_hi_to_f32(h));
    }
}

__device__ __forceinline__ bf16x8 as_bf16x8(const u32x4 &v) { return __builtin_bit_cast(bf16x8, v); }

// scale * dot (+ key bias): two separately rounded fp32 operations, the order the scores are defined in
template <bool BIAS>
__device__ __forceinline__ float scaled_score(float dot, float scale, float bias) {
    const float s = __fmul_rn(dot, scale);
    return BIAS ? add_unfused(s, bias) : s;
}

// acc += a . b with a = ah + al, b = bh + bl (small terms first)
__device__ __forceinline__ f32x4 mfma_split(const u32x4 &ah, const u32x4 &al, const u32x4 &bh, const u32x4 &bl,
                                            f32x4 acc) {
    acc = mfma16(as_bf16x8(al), as_bf16x8(bh), acc);
    acc = mfma16(as_bf16x8(ah), as_bf16x8(bl), acc);
    return mfma16(as_bf16x8(ah), as_bf16x8(bh), acc);
}

// One thread's share of a 64-row fp32 block (rows of D floats, contiguous in memory): NCONV pieces of 8
// floats, piece i = the 8 floats at float offset 8 * (i * THREADS + tid) of the block.
template <int NCONV, int THREADS = NT>
struct RawBlock {
    f32x4 v[NCONV][2];
    __device__ __forceinline__ void load(const float *block, int tid) {
#pragma unroll
        for (int i = 0; i < NCONV; ++i) {
            const f32x4 *p = reinterpret_cast<const f32x4 *>(block + 8 * (i * THREADS + tid));
            v[i][0] = p[0];
            v[i][1] = p[1];
        }
    }
    // the same for a block that holds only `rows` rows of CPR 8-float chunks: the places of the absent rows are
    // filled with the last row (nothing is read past the array)
    template <int CPR>
    __device__ __forceinline__ void load_partial(const float *block, int tid, int rows) {
#pragma unroll
        for (int i = 0; i < NCONV; ++i) {
            const int idx = i * THREADS + tid, row = idx / CPR < rows ? idx / CPR : rows - 1;
            const f32x4 *p = reinterpret_cast<const f32x4 *>(block + 8 * (row * CPR + idx % CPR));
            v[i][0] = p[0];
            v[i][1] = p[1];
        }
    }
};

// ---------------------------------------------------------------------------------------------
// Scores.  PRUNE: 1:2 selection, kept fp32 scores [BH, Lq, Lk/2] + metadata words; else S fp32.
// Per 64-key block j, after the barrier: every thread converts its share of block j+1 (loaded during block
// j-1) to the two bf16 images, stored at the permuted row (so that a lane ends up with 16 consecutive
// keys, as in the fp32 kernel) with the 16-byte chunks XOR-swizzled by row; loads its share of block j+2;
// then the waves run 3 matrix instructions per 16 x 16 x 32 product piece of block j, and the epilogue.
// A wave owns NQ groups of 16 queries: the conversion of a block and the reads of its images are
// shared by NQ times as many matrix instructions.
// ---------------------------------------------------------------------------------------------
// BIAS: key_bias[b][j] (b = head / H) is added to the scaled score before the selection (-inf masks a key).
// NW waves per workgroup (4 or 8): with 8 the conversion of a block is spread over twice the threads and shared by
// twice the queries.
template <int D, bool PRUNE, int NQ, bool BIAS, int NW>
__global__ __launch_bounds__(NW * 64, 2) void k_scores_split(const float *__restrict__ Q, const float *__restrict__ K,
                                                        const float *__restrict__ key_bias, int H, int Lq, int Lk,
                                                        float scale, float *__restrict__ out,
                                                        uint32_t *__restrict__ meta) {
    constexpr int CPR = D / 8;                   // 16-byte chunks per bf16 row
    constexpr int KS = D / 32;                   // contraction steps of 32
    constexpr int NT = NW * 64;                  // threads per workgroup
    constexpr int NCONV = KB * CPR / NT;         // bf16 chunks each thread converts per block
    constexpr int QT = 16 * NW * NQ;             // queries per workgroup
    __shared__ u32x4 Kh[2][KB * CPR], Kl[2][KB * CPR];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    const unsigned nqt = Lq / QT;
    const unsigned item = xcd_contiguous(blockIdx.x, gridDim.x);
    const unsigned bh = item / nqt, qt = item % nqt;
    const int nkb = Lk / KB;
    const int q = qt * QT + wave * (16 * NQ) + n;     // first of this lane's NQ queries (16 apart)

    // B operand: query q + 16 j, k = 32 s + 8 g + e
    u32x4 qh[NQ][KS], ql[NQ][KS];
#pragma unroll
    for (int j = 0; j < NQ; ++j) {
        const f32x4 *qp = reinterpret_cast<const f32x4 *>(Q + ((size_t)bh * Lq + q + 16 * j) * D + 8 * g);
#pragma unroll
        for (int s = 0; s < KS; ++s) split8(qp[8 * s], qp[8 * s + 1], qh[j][s], ql[j][s]);
    }

    const float *kblocks = K + (size_t)bh * Lk * D;
    const float *bias_b = BIAS ? key_bias + (size_t)(bh / H) * Lk + 16 * g : nullptr;   // this lane's 16 keys of block 0
    // where this thread's pieces go: piece idx = (key, c); row of the matrix tile that holds this key:
    // tile (key/4)%4, row 4*(key/16) + key%4
    int dst[NCONV];
#pragma unroll
    for (int i = 0; i < NCONV; ++i) {
        const int idx = i * NT + tid;
        const int key = idx / CPR, c = idx % CPR;
        const int slot = 16 * ((key >> 2) & 3) + 4 * (key >> 4) + (key & 3);
        dst[i] = slot * CPR + (c ^ (slot & 7));
    }
    auto convert = [&](const RawBlock<NCONV, NT> &raw, int buf) {
#pragma unroll
        for (int i = 0; i < NCONV; ++i) {
            u32x4 h, l;
            split8(raw.v[i][0], raw.v[i][1], h, l);
            Kh[buf][dst[i]] = h;
            Kl[buf][dst[i]] = l;
        }
    };

    const size_t ostride = PRUNE ? Lk / 2 : Lk;       // floats per output row
    float *orow = out + ((size_t)bh * Lq + q) * ostride;
    // metadata word of (row group, block jb, row n, lane group g); the next 16 queries are the next row group
    uint32_t *mrow = PRUNE ? meta + ((size_t)bh * (Lq / 16) + (q >> 4)) * nkb * 64 + n * 4 + g : nullptr;

    RawBlock<NCONV, NT> raw;
    raw.load(kblocks, tid);
    convert(raw, 0);
    if (nkb > 1) raw.load(kblocks + (size_t)KB * D, tid);
    for (int jb = 0; jb < nkb; ++jb) {
        const int buf = jb & 1;
        __syncthreads();            // images of block jb complete; every wave is done with those of block jb-1
        if (jb + 1 < nkb) convert(raw, buf ^ 1);
        if (jb + 2 < nkb) raw.load(kblocks + (size_t)(jb + 2) * KB * D, tid);
        f32x4 kb[4];                // bias of keys 16g + 4t + r of this block
#pragma unroll
        for (int t = 0; t < 4; ++t)
            kb[t] = BIAS ? *reinterpret_cast<const f32x4 *>(bias_b + jb * KB + 4 * t) : f32x4{0.f, 0.f, 0.f, 0.f};

        f32x4 acc[NQ][4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
#pragma unroll
            for (int j = 0; j < NQ; ++j) acc[j][t] = f32x4{0.f, 0.f, 0.f, 0.f};
            const int slot = 16 * t + n;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const int pos = slot * CPR + ((4 * s + g) ^ (n & 7));
                const u32x4 ah = Kh[buf][pos], al = Kl[buf][pos];
#pragma unroll
                for (int j = 0; j < NQ; ++j) acc[j][t] = mfma_split(ah, al, qh[j][s], ql[j][s], acc[j][t]);
            }
        }

#pragma unroll
        for (int j = 0; j < NQ; ++j) {
            if constexpr (PRUNE) {
                f32x4 kept[2];
                uint32_t word = 0;
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const float s0 = scaled_score<BIAS>(acc[j][t][2 * h], scale, kb[t][2 * h]);
                        const float s1 = scaled_score<BIAS>(acc[j][t][2 * h + 1], scale, kb[t][2 * h + 1]);
                        const bool second = s1 > s0;
                        const int p = 2 * t + h;
                        kept[p >> 2][p & 3] = second ? s1 : s0;
                        word |= (second ? 0xEu : 0x4u) << (4 * p);
                    }
                f32x4 *vp = reinterpret_cast<f32x4 *>(orow + (size_t)(16 * j) * ostride + jb * (KB / 2) + 8 * g);
                vp[0] = kept[0];
                vp[1] = kept[1];
                mrow[((size_t)j * nkb + jb) * 64] = word;
            } else {
                f32x4 *sp = reinterpret_cast<f32x4 *>(orow + (size_t)(16 * j) * ostride + jb * KB + 16 * g);
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    f32x4 v;
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[r] = scaled_score<BIAS>(acc[j][t][r], scale, kb[t][r]);
                    sp[t] = v;
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// O = A V.  SPARSE: A = kept weights [BH, Lq, Lk/2] fp32 + metadata of the 4-byte mode, expanded and
// split in registers; else A dense [BH, Lq, Lk] fp32.  SPARSE: the lane's 8 kept weights of keys
// 16g .. 16g+15 are the compressed operand of the structured-sparse matrix instruction
// (v_smfmac_f32_16x16x64_bf16; one kept value per aligned pair is a valid 2-of-4 pattern), with position
// codes 2 (i%2) + [code of pair i is 0xE]; one instruction covers the 64-key block.  Dense: matrix step
// m (0, 1) takes, in lane group g, the keys 32 m + 8 g .. +7 on the dense instruction.  V blocks are
// converted like K blocks (one block ahead, double-buffered images), into row-major bf16 images whose
// 16-byte chunk c of key k sits at chunk c ^ tr_row_swizzle(k); the B operand (keys along the contraction) comes
// from the transposing LDS read.
// ---------------------------------------------------------------------------------------------
template <int D, bool SPARSE, int NW>
__global__ __launch_bounds__(NW * 64, 2) void k_av_split(const float *__restrict__ A, const uint16_t *__restrict__ meta,
                                                    const float *__restrict__ V, int Lq, int Lk,
                                                    float *__restrict__ O) {
    constexpr int CPR = D / 8;
    constexpr int NT = NW * 64, QT = NW * 16;    // threads and queries per workgroup
    constexpr int NCONV = KB * CPR / NT;
    constexpr int DS = D / 16;
    __shared__ u32x4 Vh[2][KB * CPR], Vl[2][KB * CPR];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, g = lane >> 4;
    const unsigned nqt = Lq / QT;
    const unsigned item = xcd_contiguous(blockIdx.x, gridDim.x);
    const unsigned bh = item / nqt, qt = item % nqt;
    const int nkb = Lk / KB;
    const int q = qt * QT + wave * 16 + li;      // A operand row of this lane

    const float *vblocks = V + (size_t)bh * Lk * D;
    int dst[NCONV];
#pragma unroll
    for (int i = 0; i < NCONV; ++i) {
        const int idx = i * NT + tid;
        const int key = idx / CPR, c = idx % CPR;
        dst[i] = key * CPR + (c ^ tr_row_swizzle<CPR>(key));
    }
    auto convert = [&](const RawBlock<NCONV, NT> &raw, int buf) {
#pragma unroll
        for (int i = 0; i < NCONV; ++i) {
            u32x4 h, l;
            split8(raw.v[i][0], raw.v[i][1], h, l);
            Vh[buf][dst[i]] = h;
            Vl[buf][dst[i]] = l;
        }
    };

    // weights of this lane for one block
    struct AFrag {
        f32x4 v[SPARSE ? 2 : 4];
        uint32_t word;          // the metadata word of keys 16g .. 16g+15 (8 codes)
    };
    const float *arow = A + ((size_t)bh * Lq + q) * (SPARSE ? Lk / 2 : Lk);
    const uint32_t *mrow = SPARSE ? reinterpret_cast<const uint32_t *>(meta) +
                                        ((size_t)bh * (Lq / 16) + (q >> 4)) * nkb * 64 + li * 4 + g
                                  : nullptr;
    auto load_a = [&](int jb, AFrag &a) {
        if constexpr (SPARSE) {
            const f32x4 *p = reinterpret_cast<const f32x4 *>(arow + jb * (KB / 2) + 8 * g);
            a.v[0] = p[0];
            a.v[1] = p[1];
            a.word = mrow[jb * 64];
        } else {
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                const f32x4 *p = reinterpret_cast<const f32x4 *>(arow + jb * KB + 32 * m + 8 * g);
                a.v[2 * m] = p[0];
                a.v[2 * m + 1] = p[1];
            }
            a.word = 0;
        }
    };

    f32x4 acc[DS];
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) acc[ds] = f32x4{0.f, 0.f, 0.f, 0.f};

    // transposing read: lane li of a 16-lane group addresses V[key0 + li/4][col0 + 4*(li%4)]
    const int tr_row = li >> 2;
    const int tr_sub = (li >> 1) & 1;
    const int tr_byte = 8 * (li & 1);
    auto tr8 = [&](const u32x4 *img, int key0, int ds) {
        const char *base = reinterpret_cast<const char *>(img);
        // key0 is a multiple of 8: the rows key0 + tr_row and key0 + 4 + tr_row share the pattern
        const int chunk = (2 * ds + tr_sub) ^ tr_row_swizzle<CPR>(key0 + tr_row);
        const s16x4 t0 = lds_read_tr16(base + ((key0 + tr_row) * CPR + chunk) * 16 + tr_byte);
        const s16x4 t1 = lds_read_tr16(base + ((key0 + 4 + tr_row) * CPR + chunk) * 16 + tr_byte);
        return __builtin_bit_cast(u32x4, __builtin_shufflevector(t0, t1, 0, 1, 2, 3, 4, 5, 6, 7));
    };

    AFrag a_cur, a_nxt;
    load_a(0, a_cur);
    RawBlock<NCONV, NT> raw;
    raw.load(vblocks, tid);
    convert(raw, 0);
    if (nkb > 1) raw.load(vblocks + (size_t)KB * D, tid);
    for (int jb = 0; jb < nkb; ++jb) {
        const int buf = jb & 1;
        __syncthreads();            // images of block jb complete; every wave is done with those of block jb-1
        if (jb + 1 < nkb) {
            convert(raw, buf ^ 1);
            load_a(jb + 1, a_nxt);
        }
        if (jb + 2 < nkb) raw.load(vblocks + (size_t)(jb + 2) * KB * D, tid);

        if constexpr (SPARSE) {
            // bit 1 of code i (0x4 / 0xE) -> bit 2i of the instruction's index operand; bits 2i+1 = i%2
            uint32_t x = (a_cur.word >> 1) & 0x11111111u;
            x = (x | (x >> 2)) & 0x05050505u;
            x = (x | (x >> 4)) & 0x00FF00FFu;
            x = (x | (x >> 8)) & 0xFFFFu;
            const int idx = (int)(0x8888u | x);
            u32x4 ah, al;
            split8(a_cur.v[0], a_cur.v[1], ah, al);
#pragma unroll
            for (int ds = 0; ds < DS; ++ds) {
                const u32x4 h0 = tr8(Vh[buf], 8 * g, ds), h1 = tr8(Vh[buf], 32 + 8 * g, ds);
                const u32x4 l0 = tr8(Vl[buf], 8 * g, ds), l1 = tr8(Vl[buf], 32 + 8 * g, ds);
                const bf16x16 bh16 = __builtin_bit_cast(bf16x16, __builtin_shufflevector(h0, h1, 0, 1, 2, 3, 4, 5, 6, 7));
                const bf16x16 bl16 = __builtin_bit_cast(bf16x16, __builtin_shufflevector(l0, l1, 0, 1, 2, 3, 4, 5, 6, 7));
                acc[ds] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(as_bf16x8(al), bh16, acc[ds], idx, 0, 0);
                acc[ds] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(as_bf16x8(ah), bl16, acc[ds], idx, 0, 0);
                acc[ds] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(as_bf16x8(ah), bh16, acc[ds], idx, 0, 0);
            }
        } else {
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                u32x4 ah, al;
                split8(a_cur.v[2 * m], a_cur.v[2 * m + 1], ah, al);
                const int key0 = 32 * m + 8 * g;
#pragma unroll
                for (int ds = 0; ds < DS; ++ds)
                    acc[ds] = mfma_split(ah, al, tr8(Vh[buf], key0, ds), tr8(Vl[buf], key0, ds), acc[ds]);
            }
        }
        if (jb + 1 < nkb) a_cur = a_nxt;
    }

    // acc[ds][r] = O[query 4 g + r of this wave][16 ds + li]
    float *op = O + ((size_t)bh * Lq + qt * QT + wave * 16 + 4 * g) * D + li;
#pragma unroll
    for (int ds = 0; ds < DS; ++ds)
#pragma unroll
        for (int r = 0; r < 4; ++r) op[(size_t)r * D + ds * 16] = acc[ds][r];
}

// ---------------------------------------------------------------------------------------------
// Backward pass, first step: dS' = scale * P .* (dO V^T - delta) at the kept positions, delta_q = dO_q . O_q,
// written in the compressed layout of P.  The mainloop is k_scores_split's with V in the place of K and dO
// in the place of Q; the epilogue reads the stored position codes instead of selecting.  delta comes from the
// slices of dO and O the lane holds anyway (its share of d) and two cross-lane additions.
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(NT, 2) void k_ds_split(const float *__restrict__ dO, const float *__restrict__ V,
                                                    const float *__restrict__ O, const float *__restrict__ P,
                                                    const uint32_t *__restrict__ meta, int Lq, int Lk, float scale,
                                                    float *__restrict__ dS) {
    constexpr int CPR = D / 8;
    constexpr int KS = D / 32;
    constexpr int NCONV = KB * CPR / NT;
    __shared__ u32x4 Vh[2][KB * CPR], Vl[2][KB * CPR];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    const unsigned nqt = Lq / QT;
    const unsigned item = xcd_contiguous(blockIdx.x, gridDim.x);
    const unsigned bh = item / nqt, qt = item % nqt;
    const int nkb = Lk / KB;
    const int q = qt * QT + wave * 16 + n;

    // B operand: dO of query q, k = 32 s + 8 g + e; delta from the same slices of dO and O
    u32x4 gh[KS], gl[KS];
    float delta = 0.f;
    {
        const f32x4 *gp = reinterpret_cast<const f32x4 *>(dO + ((size_t)bh * Lq + q) * D + 8 * g);
        const f32x4 *op = reinterpret_cast<const f32x4 *>(O + ((size_t)bh * Lq + q) * D + 8 * g);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const f32x4 g0 = gp[8 * s], g1 = gp[8 * s + 1], o0 = op[8 * s], o1 = op[8 * s + 1];
#pragma unroll
            for (int e = 0; e < 4; ++e) delta += g0[e] * o0[e] + g1[e] * o1[e];
            split8(g0, g1, gh[s], gl[s]);
        }
        delta += __shfl_xor(delta, 16, kWave);
        delta += __shfl_xor(delta, 32, kWave);
    }

    const float *vblocks = V + (size_t)bh * Lk * D;
    int dst[NCONV];
#pragma unroll
    for (int i = 0; i < NCONV; ++i) {
        const int idx = i * NT + tid;
        const int key = idx / CPR, c = idx % CPR;
        const int slot = 16 * ((key >> 2) & 3) + 4 * (key >> 4) + (key & 3);     // as in k_scores_split
        dst[i] = slot * CPR + (c ^ (slot & 7));
    }
    auto convert = [&](const RawBlock<NCONV> &raw, int buf) {
#pragma unroll
        for (int i = 0; i < NCONV; ++i) {
            u32x4 h, l;
            split8(raw.v[i][0], raw.v[i][1], h, l);
            Vh[buf][dst[i]] = h;
            Vl[buf][dst[i]] = l;
        }
    };

    const size_t row = (size_t)bh * Lq + q;
    const float *prow = P + row * (Lk / 2) + 8 * g;
    float *srow = dS + row * (Lk / 2) + 8 * g;
    const uint32_t *mrow = meta + ((size_t)bh * (Lq / 16) + (q >> 4)) * nkb * 64 + n * 4 + g;

    RawBlock<NCONV> raw;
    raw.load(vblocks, tid);
    convert(raw, 0);
    if (nkb > 1) raw.load(vblocks + (size_t)KB * D, tid);
    for (int jb = 0; jb < nkb; ++jb) {
        const int buf = jb & 1;
        __syncthreads();
        if (jb + 1 < nkb) convert(raw, buf ^ 1);
        if (jb + 2 < nkb) raw.load(vblocks + (size_t)(jb + 2) * KB * D, tid);
        const f32x4 p0 = *reinterpret_cast<const f32x4 *>(prow + jb * (KB / 2));
        const f32x4 p1 = *reinterpret_cast<const f32x4 *>(prow + jb * (KB / 2) + 4);
        const uint32_t word = mrow[jb * 64];

        f32x4 acc[4];       // dP of keys 16g + 4t + r of query n
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
            const int slot = 16 * t + n;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const int pos = slot * CPR + ((4 * s + g) ^ (n & 7));
                acc[t] = mfma_split(Vh[buf][pos], Vl[buf][pos], gh[s], gl[s], acc[t]);
            }
        }

        f32x4 ds[2];
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int i = 2 * t + h;                               // pair i: keys 16g + 2i, +1
                const bool second = (word >> (4 * i + 1)) & 1u;        // code 0xE
                const float dp = second ? acc[t][2 * h + 1] : acc[t][2 * h];
                const float p = i < 4 ? p0[i & 3] : p1[i & 3];
                ds[i >> 2][i & 3] = scale * p * (dp - delta);
            }
        f32x4 *sp = reinterpret_cast<f32x4 *>(srow + jb * (KB / 2));
        sp[0] = ds[0];
        sp[1] = ds[1];
    }
}

// ---------------------------------------------------------------------------------------------
// Transposed sparse product out[BH, Lk, D] = A^T X for A given as kept fp32 values + metadata of the 4-byte
// mode and X fp32 [BH, Lq, D] (dV = P^T dO and dK = dS^T Q of the backward pass).  The contraction runs over
// the queries, across which the 1:2 structure does not run, so a workgroup (64 keys of one head) walks the
// queries in blocks of 64: every thread expands its share of the 64 x 64 tile of A to dense values (8 kept
// values + one metadata word -> 16 keys of one query), splits it and X's tile into bf16 images in LDS, and
// both matrix operands come from the transposing LDS read (the images hold queries along their rows):
// output rows = keys (wave w owns keys 16w .. 16w+15 of the block), contraction step m = queries 32m + 8g ..+7.
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(NT, 2) void k_spmm_t_split(const float *__restrict__ A, const uint32_t *__restrict__ meta,
                                                        const float *__restrict__ X, int Lq, int Lk,
                                                        float *__restrict__ out) {
    constexpr int CPRA = KB / 8;                 // 16-byte chunks per row of the A images (64 keys)
    constexpr int CPRX = D / 8;
    constexpr int NCX = KB * CPRX / NT;          // pieces of X each thread converts per block
    constexpr int DS = D / 16;
    __shared__ u32x4 Ah[KB * CPRA], Al[KB * CPRA], Xh[KB * CPRX], Xl[KB * CPRX];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, g = lane >> 4;
    const int nkb = Lk / KB, nqb = Lq / KB;
    const unsigned item = xcd_contiguous(blockIdx.x, gridDim.x);
    const unsigned bh = item / nkb, kb = item % nkb;

    // this thread's share of a tile of A: query row aq of the block, keys 16 ag .. 16 ag + 15
    const int aq = tid >> 2, ag = tid & 3;
    const float *arow = A + ((size_t)bh * Lq + aq) * (Lk / 2) + kb * (KB / 2) + 8 * ag;
    const uint32_t *mrow = meta + ((size_t)bh * (Lq / 16) + (aq >> 4)) * nkb * 64 + kb * 64 + (aq & 15) * 4 + ag;
    // chunk c of image row r sits at chunk c ^ 2 (r % 4), the layout the transposing read expects
    const int a_dst0 = aq * CPRA + ((2 * ag) ^ ((aq & 3) << 1)), a_dst1 = aq * CPRA + ((2 * ag + 1) ^ ((aq & 3) << 1));
    const float *xblocks = X + (size_t)bh * Lq * D;
    int x_dst[NCX];
#pragma unroll
    for (int i = 0; i < NCX; ++i) {
        const int idx = i * NT + tid;
        const int row = idx / CPRX, c = idx % CPRX;
        x_dst[i] = row * CPRX + (c ^ ((row & 3) << 1));
    }

    struct ATile {
        f32x4 v[2];
        uint32_t word;
    };
    auto load_a = [&](int qb, ATile &t) {
        const f32x4 *p = reinterpret_cast<const f32x4 *>(arow + (size_t)qb * KB * (Lk / 2));
        t.v[0] = p[0];
        t.v[1] = p[1];
        t.word = mrow[(size_t)qb * 4 * nkb * 64];     // 64 queries = 4 row groups further
    };

    const int tr_row = li >> 2;
    const int tr_sub = (li >> 1) & 1;
    const int tr_byte = 8 * (li & 1);
    const int tr_xor = tr_row << 1;
    // rows row0 .. row0+7 (queries) of column tile `ct` (16 columns) of an image with CPR chunks per row
    auto tr8 = [&](const u32x4 *img, int cpr, int row0, int ct) {
        const char *base = reinterpret_cast<const char *>(img);
        const int chunk = (2 * ct + tr_sub) ^ tr_xor;
        const s16x4 t0 = lds_read_tr16(base + ((row0 + tr_row) * cpr + chunk) * 16 + tr_byte);
        const s16x4 t1 = lds_read_tr16(base + ((row0 + 4 + tr_row) * cpr + chunk) * 16 + tr_byte);
        return __builtin_bit_cast(u32x4, __builtin_shufflevector(t0, t1, 0, 1, 2, 3, 4, 5, 6, 7));
    };

    f32x4 acc[DS];
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) acc[ds] = f32x4{0.f, 0.f, 0.f, 0.f};

    ATile at;
    RawBlock<NCX> rx;
    load_a(0, at);
    rx.load(xblocks, tid);
    for (int qb = 0; qb < nqb; ++qb) {
        __syncthreads();            // every wave is done with the images of the previous block of queries
        {
            // expand: pair i keeps its second key iff code i is 0xE (bit 1 of the nibble)
            float dlo[8], dhi[8];   // keys 16 ag + 0..7 and + 8..15
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bool s0 = (at.word >> (4 * i + 1)) & 1u, s1 = (at.word >> (4 * (i + 4) + 1)) & 1u;
                dlo[2 * i] = s0 ? 0.f : at.v[0][i];
                dlo[2 * i + 1] = s0 ? at.v[0][i] : 0.f;
                dhi[2 * i] = s1 ? 0.f : at.v[1][i];
                dhi[2 * i + 1] = s1 ? at.v[1][i] : 0.f;
            }
            u32x4 h, l;
            split8(f32x4{dlo[0], dlo[1], dlo[2], dlo[3]}, f32x4{dlo[4], dlo[5], dlo[6], dlo[7]}, h, l);
            Ah[a_dst0] = h;
            Al[a_dst0] = l;
            split8(f32x4{dhi[0], dhi[1], dhi[2], dhi[3]}, f32x4{dhi[4], dhi[5], dhi[6], dhi[7]}, h, l);
            Ah[a_dst1] = h;
            Al[a_dst1] = l;
#pragma unroll
            for (int i = 0; i < NCX; ++i) {
                split8(rx.v[i][0], rx.v[i][1], h, l);
                Xh[x_dst[i]] = h;
                Xl[x_dst[i]] = l;
            }
        }
        if (qb + 1 < nqb) {
            load_a(qb + 1, at);
            rx.load(xblocks + (size_t)(qb + 1) * KB * D, tid);
        }
        __syncthreads();            // images complete

#pragma unroll
        for (int m = 0; m < 2; ++m) {
            const int q0 = 32 * m + 8 * g;
            const u32x4 ah = tr8(Ah, CPRA, q0, wave), al = tr8(Al, CPRA, q0, wave);   // A^T: rows = keys 16 wave + li
#pragma unroll
            for (int ds = 0; ds < DS; ++ds)
                acc[ds] = mfma_split(ah, al, tr8(Xh, CPRX, q0, ds), tr8(Xl, CPRX, q0, ds), acc[ds]);
        }
    }

    // acc[ds][r] = out[key 64 kb + 16 wave + 4 g + r][16 ds + li]
    float *op = out + ((size_t)bh * Lk + kb * KB + wave * 16 + 4 * g) * D + li;
#pragma unroll
    for (int ds = 0; ds < DS; ++ds)
#pragma unroll
        for (int r = 0; r < 4; ++r) op[(size_t)r * D + ds * 16] = acc[ds][r];
}

// ---------------------------------------------------------------------------------------------
// The whole forward pass of the 4-byte mode in one kernel: scores on split products, 1:2 selection on
// the accumulators, softmax over the kept scores kept up to date block by block (running maximum and
// sum per query, the output accumulators rescaled when a maximum rises), and A V on split products,
// with the weights never leaving registers.  Nothing of the score matrix is written.
//
// Per 64-key block a lane (query n = l%16, lane group g) holds the scores of keys 16g .. 16g+15 of its
// query (keys on the rows of the score tiles, as in k_scores_split).  For the second product the lane's
// weights ARE the A operand.  With pruning it is the compressed operand of the structured-sparse matrix
// instruction (v_smfmac_f32_16x16x64_bf16: 8 kept values per lane out of 16, one from each aligned pair
// is a valid 2-of-4 pattern), whose 2-bit position codes are 2 (i%2) + [the later key of pair i was
// kept]; one instruction covers the whole 64-key block, with B = the V rows 8g .. 8g+7 and
// 32+8g .. 32+8g+7 read (transposed) from the images.  Without pruning matrix step m (0, 1) contracts, in
// lane group g, the keys 16g + 8m .. +7 on the dense instruction.  The softmax statistics of
// query n live in the lanes with l%16 = n; the output tiles hold queries 4g + r, so the factors they need
// are fetched from lanes 4g + r.
// PRUNE = false is full attention (Eq. 1) in the same structure, the baseline of this mode.
// ---------------------------------------------------------------------------------------------
// BIAS: additive key bias as in k_scores_split; a masked key gets weight exactly 0.
// block_mask (may be null): uint8 [Lq/64][Lk/64] shared by all heads; the 64 x 64 blocks of the score matrix with a
// zero entry are skipped (the workgroup's 64 queries are one row of blocks), as if all their scores were -inf.
// RAGGED (implies BIAS; key_bias may then be null): Lq and Lk are not multiples of 64.  Q, O hold Lq rows and K, V,
// key_bias Lk keys (Lk a multiple of 4); the absent keys of the last block count as masked keys, the absent queries of
// the last tile are computed on a copy of the last query and not stored.
// NW waves of 16 queries per workgroup: with 8 waves (Lq a multiple of 128, no block pattern) the conversion
// of a block is spread over twice the threads and shared by twice the queries (at d = 64 the register budget
// is then held to 128 so that two such workgroups share a CU).
template <int D, bool PRUNE, bool BIAS, int NW, bool RAGGED = false>
__global__ __launch_bounds__(NW * 64, (D == 64 && NW == 8) ? 4 : 2) void k_fused_split(const float *__restrict__ Q, const float *__restrict__ K,
                                                       const float *__restrict__ V, const float *__restrict__ key_bias,
                                                       int H, const uint8_t *__restrict__ block_mask, int Lq, int Lk,
                                                       float scale, float *__restrict__ O) {
    constexpr int CPR = D / 8;
    constexpr int KS = D / 32;
    constexpr int NT = NW * 64, QT = NW * 16;    // threads and queries per workgroup
    constexpr int NCONV = KB * CPR / NT;
    constexpr int DS = D / 16;
    constexpr int NV = PRUNE ? 8 : 16;           // weights per lane per block
    constexpr float kLog2e = 1.4426950408889634f;
    // The four images are single buffered (two barriers per block: before the conversion, and between conversion
    // and use): for d = 128 they fill the 64 KB a workgroup may declare, and for d = 64 the halved footprint lets a
    // third workgroup share the CU, which gains more than overlapping the conversion with the arithmetic does.
    __shared__ u32x4 Kh[KB * CPR], Kl[KB * CPR], Vh[KB * CPR], Vl[KB * CPR];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    static_assert(!RAGGED || BIAS, "ragged lengths use the arithmetic of the biased variant");
    const unsigned nqt = (Lq + QT - 1) / QT;
    const unsigned item = xcd_contiguous(blockIdx.x, gridDim.x);
    const unsigned bh = item / nqt, qt = item % nqt;
    const int nkb = (Lk + KB - 1) / KB;
    const int tail_keys = Lk - (nkb - 1) * KB;     // keys of the last block
    int q = qt * QT + wave * 16 + n;
    if (RAGGED && q >= Lq) q = Lq - 1;

    u32x4 qh[KS], ql[KS];
    {
        const f32x4 *qp = reinterpret_cast<const f32x4 *>(Q + ((size_t)bh * Lq + q) * D + 8 * g);
#pragma unroll
        for (int s = 0; s < KS; ++s) split8(qp[8 * s], qp[8 * s + 1], qh[s], ql[s]);
    }

    const float *kblocks = K + (size_t)bh * Lk * D;
    const float *vblocks = V + (size_t)bh * Lk * D;
    const float *bias_b = BIAS && key_bias ? key_bias + (size_t)(bh / H) * Lk + 16 * g : nullptr;
    int dst_k[NCONV], dst_v[NCONV];
#pragma unroll
    for (int i = 0; i < NCONV; ++i) {
        const int idx = i * NT + tid;
        const int key = idx / CPR, c = idx % CPR;
        const int slot = 16 * ((key >> 2) & 3) + 4 * (key >> 4) + (key & 3);
        dst_k[i] = slot * CPR + (c ^ (slot & 7));
        dst_v[i] = key * CPR + (c ^ tr_row_swizzle<CPR>(key));
    }
    auto convert = [&](const RawBlock<NCONV, NT> &rk, const RawBlock<NCONV, NT> &rv) {
#pragma unroll
        for (int i = 0; i < NCONV; ++i) {
            u32x4 h, l;
            split8(rk.v[i][0], rk.v[i][1], h, l);
            Kh[dst_k[i]] = h;
            Kl[dst_k[i]] = l;
            split8(rv.v[i][0], rv.v[i][1], h, l);
            Vh[dst_v[i]] = h;
            Vl[dst_v[i]] = l;
        }
    };

    // transposing read of the V images (see k_av_split)
    const int tr_row = n >> 2;
    const int tr_sub = (n >> 1) & 1;
    const int tr_byte = 8 * (n & 1);
    auto tr8 = [&](const u32x4 *img, int key0, int ds) {
        const char *base = reinterpret_cast<const char *>(img);
        const int chunk = (2 * ds + tr_sub) ^ tr_row_swizzle<CPR>(key0 + tr_row);   // key0 is a multiple of 8
        const s16x4 t0 = lds_read_tr16(base + ((key0 + tr_row) * CPR + chunk) * 16 + tr_byte);
        const s16x4 t1 = lds_read_tr16(base + ((key0 + 4 + tr_row) * CPR + chunk) * 16 + tr_byte);
        return __builtin_bit_cast(u32x4, __builtin_shufflevector(t0, t1, 0, 1, 2, 3, 4, 5, 6, 7));
    };

    f32x4 acc_o[DS];
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) acc_o[ds] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -1e30f;      // running maximum of query n (the same in its four lanes)
    float l_run = 0.f;         // this lane's share of the running sum of query n

    // the blocks of this row of blocks that take part, in order (all of them without a block pattern)
    const uint8_t *live = block_mask ? block_mask + (size_t)qt * nkb : nullptr;
    auto next_block = [&](int j) {
        if (live)
            while (j < nkb && live[j] == 0) ++j;
        return j;
    };

    RawBlock<NCONV, NT> rk, rv;
    auto load_block = [&](int j) {
        if (RAGGED && j == nkb - 1 && tail_keys < KB) {
            rk.template load_partial<CPR>(kblocks + (size_t)j * KB * D, tid, tail_keys);
            rv.template load_partial<CPR>(vblocks + (size_t)j * KB * D, tid, tail_keys);
        } else {
            rk.load(kblocks + (size_t)j * KB * D, tid);
            rv.load(vblocks + (size_t)j * KB * D, tid);
        }
    };
    int jb = next_block(0);
    if (jb < nkb) load_block(jb);
    while (jb < nkb) {
        const int jnext = next_block(jb + 1);
        __syncthreads();            // every wave is done with the images of the previous block
        convert(rk, rv);
        if (jnext < nkb) load_block(jnext);   // the next block travels while this one is used
        __syncthreads();            // images of block jb complete
        f32x4 kb[4];                // bias of keys 16g + 4t + r of this block
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            if constexpr (RAGGED) {
                if (jb * KB + 16 * g + 4 * t >= Lk) kb[t] = f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
                else if (bias_b) kb[t] = *reinterpret_cast<const f32x4 *>(bias_b + jb * KB + 4 * t);
                else kb[t] = f32x4{0.f, 0.f, 0.f, 0.f};
            } else {
                kb[t] = BIAS ? *reinterpret_cast<const f32x4 *>(bias_b + jb * KB + 4 * t) : f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }

        // scores of keys 16g + 4t + r (tile t, register r) of query n
        f32x4 acc[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
            const int slot = 16 * t + n;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const int pos = slot * CPR + ((4 * s + g) ^ (n & 7));
                acc[t] = mfma_split(Kh[pos], Kl[pos], qh[s], ql[s], acc[t]);
            }
        }

        // selection: w[i] = kept score of pair i (keys 16g + 2i, +1), bit i of `second` = the later one was kept
        float w[NV];
        uint32_t second = 0;
        float m_loc;
        if constexpr (PRUNE) {
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const float s0 = scaled_score<BIAS>(acc[t][2 * h], scale, kb[t][2 * h]);
                    const float s1 = scaled_score<BIAS>(acc[t][2 * h + 1], scale, kb[t][2 * h + 1]);
                    const bool sec = s1 > s0;
                    w[2 * t + h] = sec ? s1 : s0;
                    second |= (sec ? 1u : 0u) << (2 * (2 * t + h));     // bit 2i: position code of pair i
                }
        } else {
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r) w[4 * t + r] = scaled_score<BIAS>(acc[t][r], scale, kb[t][r]);
        }
        m_loc = w[0];
#pragma unroll
        for (int i = 1; i < NV; ++i) m_loc = fmaxf(m_loc, w[i]);
        m_loc = fmaxf(m_loc, __shfl_xor(m_loc, 16, kWave));
        m_loc = fmaxf(m_loc, __shfl_xor(m_loc, 32, kWave));
        const float m_new = fmaxf(m_run, m_loc);
        if (__ballot(m_new > m_run) != 0) {     // some query of this wave has a new maximum: rescale
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * kLog2e);   // 1 where unchanged
            l_run *= alpha;
            m_run = m_new;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float a_r = __shfl(alpha, 4 * g + r, kWave);
#pragma unroll
                for (int ds = 0; ds < DS; ++ds) acc_o[ds][r] *= a_r;
            }
        }
        const float mb = m_run * kLog2e;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            w[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(w[i], kLog2e, -mb));   // the bare instruction: tiny results flush to 0
            l_run += w[i];
        }

        if constexpr (PRUNE) {
            // weights x V on the structured-sparse instruction: kept value i sits at dense position
            // 4 (i/2) + 2 (i%2) + second_i of this lane's 16 keys
            u32x4 ah, al;
            split8(f32x4{w[0], w[1], w[2], w[3]}, f32x4{w[4], w[5], w[6], w[7]}, ah, al);
            const int idx = (int)(0x8888u | second);
#pragma unroll
            for (int ds = 0; ds < DS; ++ds) {
                const u32x4 h0 = tr8(Vh, 8 * g, ds), h1 = tr8(Vh, 32 + 8 * g, ds);
                const u32x4 l0 = tr8(Vl, 8 * g, ds), l1 = tr8(Vl, 32 + 8 * g, ds);
                const bf16x16 bh16 = __builtin_bit_cast(bf16x16, __builtin_shufflevector(h0, h1, 0, 1, 2, 3, 4, 5, 6, 7));
                const bf16x16 bl16 = __builtin_bit_cast(bf16x16, __builtin_shufflevector(l0, l1, 0, 1, 2, 3, 4, 5, 6, 7));
                acc_o[ds] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(as_bf16x8(al), bh16, acc_o[ds], idx, 0, 0);
                acc_o[ds] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(as_bf16x8(ah), bl16, acc_o[ds], idx, 0, 0);
                acc_o[ds] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(as_bf16x8(ah), bh16, acc_o[ds], idx, 0, 0);
            }
        } else {
            // weights x V: matrix step m takes keys 16g + 8m .. +7 in lane group g
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                u32x4 ah, al;
                split8(f32x4{w[8 * m], w[8 * m + 1], w[8 * m + 2], w[8 * m + 3]},
                       f32x4{w[8 * m + 4], w[8 * m + 5], w[8 * m + 6], w[8 * m + 7]}, ah, al);
                const int key0 = 16 * g + 8 * m;
#pragma unroll
                for (int ds = 0; ds < DS; ++ds)
                    acc_o[ds] = mfma_split(ah, al, tr8(Vh, key0, ds), tr8(Vl, key0, ds), acc_o[ds]);
            }
        }
        jb = jnext;
    }

    // row sums: the four lanes of a query add up; then the factor of query 4g + r comes from lane 4g + r
    l_run += __shfl_xor(l_run, 16, kWave);
    l_run += __shfl_xor(l_run, 32, kWave);
    const float inv = 1.0f / l_run;
    float *op = O + ((size_t)bh * Lq + qt * QT + wave * 16 + 4 * g) * D + n;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const float inv_r = __shfl(inv, 4 * g + r, kWave);
        if (RAGGED && (int)(qt * QT) + wave * 16 + 4 * g + r >= Lq) continue;
#pragma unroll
        for (int ds = 0; ds < DS; ++ds) op[(size_t)r * D + ds * 16] = acc_o[ds][r] * inv_r;
    }
}

template <int D, bool PRUNE, int NQ, int NW>
hipError_t launch_scores_nq(const void *Q, const void *K, const float *key_bias, int H, int BH, int Lq, int Lk,
                            float scale, void *out, void *meta, hipStream_t st) {
    const unsigned grid = (unsigned)BH * (unsigned)(Lq / (16 * NW * NQ));
    if (key_bias)
        hipLaunchKernelGGL((k_scores_split<D, PRUNE, NQ, true, NW>), dim3(grid), dim3(NW * 64), 0, st,
                           (const float *)Q, (const float *)K, key_bias, H, Lq, Lk, scale, (float *)out,
                           (uint32_t *)meta);
    else
        hipLaunchKernelGGL((k_scores_split<D, PRUNE, NQ, false, NW>), dim3(grid), dim3(NW * 64), 0, st,
                           (const float *)Q, (const float *)K, key_bias, H, Lq, Lk, scale, (float *)out,
                           (uint32_t *)meta);
    return hipGetLastError();
}

template <bool PRUNE>
hipError_t launch_scores(const void *Q, const void *K, const float *key_bias, int H, int BH, int Lq, int Lk, int d,
                         float scale, void *out, void *meta, hipStream_t st) {
    // 128 queries per workgroup (4 waves x 32 queries) where Lq allows and the grid still fills the chip
    int nw = 4, nq = (Lq % 128 == 0 && (long)BH * (Lq / 128) >= 512) ? 2 : 1;
    if (Lq % (16 * nw * nq) != 0) nw = 4, nq = 1;
#define DFSS_LAUNCH_SCORES(DD)                                                                                   \
    do {                                                                                                         \
        if (nw == 8 && nq == 2) return launch_scores_nq<DD, PRUNE, 2, 8>(Q, K, key_bias, H, BH, Lq, Lk, scale, out, meta, st); \
        if (nw == 8) return launch_scores_nq<DD, PRUNE, 1, 8>(Q, K, key_bias, H, BH, Lq, Lk, scale, out, meta, st);            \
        if (nq == 2) return launch_scores_nq<DD, PRUNE, 2, 4>(Q, K, key_bias, H, BH, Lq, Lk, scale, out, meta, st);            \
        return launch_scores_nq<DD, PRUNE, 1, 4>(Q, K, key_bias, H, BH, Lq, Lk, scale, out, meta, st);                         \
    } while (0)
    if (d == 64) DFSS_LAUNCH_SCORES(64);
    if (d == 128) DFSS_LAUNCH_SCORES(128);
#undef DFSS_LAUNCH_SCORES
    return hipErrorInvalidValue;
}

template <int D, bool SPARSE, int NW>
hipError_t launch_av_nw(const void *A, const void *meta, const void *V, int BH, int Lq, int Lk, void *O,
                        hipStream_t st) {
    const unsigned grid = (unsigned)BH * (unsigned)(Lq / (16 * NW));
    hipLaunchKernelGGL((k_av_split<D, SPARSE, NW>), dim3(grid), dim3(NW * 64), 0, st, (const float *)A,
                       (const uint16_t *)meta, (const float *)V, Lq, Lk, (float *)O);
    return hipGetLastError();
}

template <bool SPARSE>
hipError_t launch_av(const void *A, const void *meta, const void *V, int BH, int Lq, int Lk, int d, void *O,
                     hipStream_t st) {
    // 8 waves per workgroup where the 128-query tile divides Lq and the grid still fills the chip
    int nw = (Lq % 128 == 0 && (long)BH * (Lq / 128) >= 512) ? 8 : 4, nq = 1;
    if (Lq % (16 * nw) != 0) nw = 4;
    if (d == 64)
        return nw == 8 ? launch_av_nw<64, SPARSE, 8>(A, meta, V, BH, Lq, Lk, O, st)
                       : launch_av_nw<64, SPARSE, 4>(A, meta, V, BH, Lq, Lk, O, st);
    if (d == 128)
        return nw == 8 ? launch_av_nw<128, SPARSE, 8>(A, meta, V, BH, Lq, Lk, O, st)
                       : launch_av_nw<128, SPARSE, 4>(A, meta, V, BH, Lq, Lk, O, st);
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_fused_attention_split(const void *Q, const void *K, const void *V, const float *key_bias, int H,
                                        const uint8_t *block_mask, int BH, int Lq, int Lk, int d, bool prune,
                                        float scale, void *O, hipStream_t st) {
    // 8 waves per workgroup where the 128-query tile divides Lq, is not cut by a 64 x 64 block pattern, and still
    // leaves at least two workgroups per compute unit
    const bool ragged = Lq % 64 != 0 || Lk % 64 != 0;   // (never together with a block pattern)
    const bool wide = (ragged || Lq % 128 == 0) && !block_mask && (long)BH * ((Lq + 127) / 128) >= 512;
    const unsigned grid = (unsigned)BH * (unsigned)((Lq + (wide ? 127 : 63)) / (wide ? 128 : 64));
#define DFSS_LAUNCH_FUSED_SPLIT(DD, PP, BB, WW)                                                                   \
    hipLaunchKernelGGL((k_fused_split<DD, PP, BB, WW>), dim3(grid), dim3(WW * 64), 0, st, (const float *)Q,       \
                       (const float *)K, (const float *)V, key_bias, H, block_mask, Lq, Lk, scale, (float *)O)
#define DFSS_LAUNCH_FUSED_SPLIT_B(DD, PP)                                 \
    do {                                                                  \
        if (ragged && wide)                                               \
            hipLaunchKernelGGL((k_fused_split<DD, PP, true, 8, true>), dim3(grid), dim3(512), 0, st, (const float *)Q,  \
                               (const float *)K, (const float *)V, key_bias, H, block_mask, Lq, Lk, scale, (float *)O); \
        else if (ragged)                                                  \
            hipLaunchKernelGGL((k_fused_split<DD, PP, true, 4, true>), dim3(grid), dim3(256), 0, st, (const float *)Q,  \
                               (const float *)K, (const float *)V, key_bias, H, block_mask, Lq, Lk, scale, (float *)O); \
        else if (key_bias && wide) DFSS_LAUNCH_FUSED_SPLIT(DD, PP, true, 8);   \
        else if (key_bias) DFSS_LAUNCH_FUSED_SPLIT(DD, PP, true, 4);      \
        else if (wide) DFSS_LAUNCH_FUSED_SPLIT(DD, PP, false, 8);         \
        else DFSS_LAUNCH_FUSED_SPLIT(DD, PP, false, 4);                   \
    } while (0)
    if (d == 64 && prune) DFSS_LAUNCH_FUSED_SPLIT_B(64, true);
    else if (d == 64) DFSS_LAUNCH_FUSED_SPLIT_B(64, false);
    else if (d == 128 && prune) DFSS_LAUNCH_FUSED_SPLIT_B(128, true);
    else if (d == 128) DFSS_LAUNCH_FUSED_SPLIT_B(128, false);
    else return hipErrorInvalidValue;
#undef DFSS_LAUNCH_FUSED_SPLIT_B
#undef DFSS_LAUNCH_FUSED_SPLIT
    return hipGetLastError();
}

hipError_t launch_sddmm_prune_split(const void *Q, const void *K, const float *key_bias, int H, int BH, int Lq, int Lk,
                                    int d, float scale, void *vals, void *meta, hipStream_t st) {
    return launch_scores<true>(Q, K, key_bias, H, BH, Lq, Lk, d, scale, vals, meta, st);
}
hipError_t launch_dense_scores_split(const void *Q, const void *K, const float *key_bias, int H, int BH, int Lq,
                                     int Lk, int d, float scale, void *S, hipStream_t st) {
    return launch_scores<false>(Q, K, key_bias, H, BH, Lq, Lk, d, scale, S, nullptr, st);
}
hipError_t launch_masked_sddmm_ds_split(const void *dO, const void *V, const void *O, const void *P, const void *meta,
                                        int BH, int Lq, int Lk, int d, float scale, void *dS, hipStream_t st) {
    const unsigned grid = (unsigned)BH * (unsigned)(Lq / QT);
    if (d == 64)
        hipLaunchKernelGGL((k_ds_split<64>), dim3(grid), dim3(NT), 0, st, (const float *)dO, (const float *)V,
                           (const float *)O, (const float *)P, (const uint32_t *)meta, Lq, Lk, scale, (float *)dS);
    else if (d == 128)
        hipLaunchKernelGGL((k_ds_split<128>), dim3(grid), dim3(NT), 0, st, (const float *)dO, (const float *)V,
                           (const float *)O, (const float *)P, (const uint32_t *)meta, Lq, Lk, scale, (float *)dS);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_spmm_t_split(const void *vals, const void *meta, const void *X, int BH, int Lq, int Lk, int d,
                               void *out, hipStream_t st) {
    const unsigned grid = (unsigned)BH * (unsigned)(Lk / KB);
    if (d == 64)
        hipLaunchKernelGGL((k_spmm_t_split<64>), dim3(grid), dim3(NT), 0, st, (const float *)vals,
                           (const uint32_t *)meta, (const float *)X, Lq, Lk, (float *)out);
    else if (d == 128)
        hipLaunchKernelGGL((k_spmm_t_split<128>), dim3(grid), dim3(NT), 0, st, (const float *)vals,
                           (const uint32_t *)meta, (const float *)X, Lq, Lk, (float *)out);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_spmm_split(const void *vals, const void *meta, const void *V, int BH, int Lq, int Lk, int d,
                             void *O, hipStream_t st) {
    return launch_av<true>(vals, meta, V, BH, Lq, Lk, d, O, st);
}
hipError_t launch_dense_av_split(const void *P, const void *V, int BH, int Lq, int Lk, int d, void *O,
                                 hipStream_t st) {
    return launch_av<false>(P, nullptr, V, BH, Lq, Lk, d, O, st);
}

}  // namespace dfss
