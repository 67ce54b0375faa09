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
// Blocks of K (or V) arrive in LDS as fp32 by asynchronous copies; the workgroup converts each block
// once into its two bf16 images, which the waves then read as ordinary bf16 matrix operands.  The
// layouts, the 1:2 epilogue and the metadata are those of the exact fp32 kernels (float_mode.hip).
#include "dfss_device.hpp"
#include "dfss_kernels.hpp"

namespace dfss {

namespace {

constexpr int NT = 256;   // 4 waves, 16 queries each
constexpr int QT = 64;    // queries per workgroup
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

// acc += a . b with a = ah + al, b = bh + bl (small terms first)
__device__ __forceinline__ f32x4 mfma_split(const u32x4 &ah, const u32x4 &al, const u32x4 &bh, const u32x4 &bl,
                                            f32x4 acc) {
    acc = mfma16(as_bf16x8(al), as_bf16x8(bh), acc);
    acc = mfma16(as_bf16x8(ah), as_bf16x8(bl), acc);
    return mfma16(as_bf16x8(ah), as_bf16x8(bh), acc);
}

// Asynchronous copy of one 64-row fp32 block (rows of D floats, contiguous in memory) into LDS, in
// memory order: 16 D bytes per wave instruction.
template <int D>
struct BlockCopy {
    static constexpr int NCOPY = KB * D * 4 / (NT * 16);
    uint64_t base;
    uint32_t lds, lane_off;
    int wave;
    __device__ void issue(int jb) const {
        const uint64_t b = base + (uint64_t)jb * (KB * D * 4);
#pragma unroll
        for (int c = 0; c < NCOPY; ++c) {
            const uint32_t piece = (uint32_t)(c * 4 + wave) * 1024u;
            async_copy16(b, piece + lane_off, lds + piece);
        }
    }
};

// ---------------------------------------------------------------------------------------------
// Scores.  PRUNE: 1:2 selection, kept fp32 scores [BH, Lq, Lk/2] + metadata words; else S fp32.
// Per 64-key block: (1) wait for the fp32 copy, barrier; (2) every thread converts its share of the
// block to the two bf16 images, stored at the permuted row (so that a lane ends up with 16 consecutive
// keys, as in the fp32 kernel) with the 16-byte chunks XOR-swizzled by row; barrier; (3) the copy of the
// next block is issued (the fp32 buffer is free again) and the waves run 3 matrix instructions per
// 16 x 16 x 32 product piece, then the epilogue.
// ---------------------------------------------------------------------------------------------
template <int D, bool PRUNE>
__global__ __launch_bounds__(NT, 2) void k_scores_split(const float *__restrict__ Q, const float *__restrict__ K,
                                                        int Lq, int Lk, float scale, float *__restrict__ out,
                                                        uint32_t *__restrict__ meta) {
    constexpr int CPR = D / 8;                   // 16-byte chunks per bf16 row
    constexpr int KS = D / 32;                   // contraction steps of 32
    constexpr int NCONV = KB * CPR / NT;         // bf16 chunks each thread converts per block
    constexpr int NSTORE = PRUNE ? 3 : 4;        // vector stores per lane per block
    __shared__ __attribute__((aligned(16))) float Kf[KB * D];
    __shared__ u32x4 Kh[KB * CPR], Kl[KB * CPR];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    const unsigned nqt = Lq / QT;
    const unsigned item = xcd_contiguous(blockIdx.x, gridDim.x);
    const unsigned bh = item / nqt, qt = item % nqt;
    const int nkb = Lk / KB;
    const int q = qt * QT + wave * 16 + n;

    // B operand: query q, k = 32 s + 8 g + e
    u32x4 qh[KS], ql[KS];
    {
        const f32x4 *qp = reinterpret_cast<const f32x4 *>(Q + ((size_t)bh * Lq + q) * D + 8 * g);
#pragma unroll
        for (int s = 0; s < KS; ++s) split8(qp[8 * s], qp[8 * s + 1], qh[s], ql[s]);
    }

    const BlockCopy<D> copy{uniform_address(K + (size_t)bh * Lk * D), lds_address(&Kf[0]), (uint32_t)lane * 16u, wave};

    float *orow = out + ((size_t)bh * Lq + q) * (PRUNE ? Lk / 2 : Lk);
    uint32_t *mrow = PRUNE ? meta + ((size_t)bh * Lq + q) * (Lk / 16) : nullptr;

    copy.issue(0);
    for (int jb = 0; jb < nkb; ++jb) {
        // the copy of block jb is older than the stores of block jb-1: leave those in flight
        if (jb == 0) wait_async_copies();
        else wait_async_copies_keep<NSTORE>();
        __syncthreads();            // fp32 block landed; every wave is done with the bf16 images of block jb-1
#pragma unroll
        for (int i = 0; i < NCONV; ++i) {
            const int idx = i * NT + tid;
            const int key = idx / CPR, c = idx % CPR;
            const f32x4 *src = reinterpret_cast<const f32x4 *>(&Kf[key * D + 8 * c]);
            u32x4 h, l;
            split8(src[0], src[1], h, l);
            // row of the matrix tile that holds this key: tile (key/4)%4, row 4*(key/16) + key%4
            const int slot = 16 * ((key >> 2) & 3) + 4 * (key >> 4) + (key & 3);
            const int pos = slot * CPR + (c ^ (slot & 7));
            Kh[pos] = h;
            Kl[pos] = l;
        }
        __syncthreads();            // images complete; the fp32 buffer may be overwritten
        if (jb + 1 < nkb) copy.issue(jb + 1);

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

        if constexpr (PRUNE) {
            f32x4 kept[2];
            uint32_t word = 0;
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const float s0 = acc[t][2 * h] * scale, s1 = acc[t][2 * h + 1] * scale;
                    const bool second = s1 > s0;
                    const int p = 2 * t + h;
                    kept[p >> 2][p & 3] = second ? s1 : s0;
                    word |= (second ? 0xEu : 0x4u) << (4 * p);
                }
            f32x4 *vp = reinterpret_cast<f32x4 *>(orow + jb * (KB / 2) + 8 * g);
            vp[0] = kept[0];
            vp[1] = kept[1];
            mrow[jb * 4 + g] = word;
        } else {
            f32x4 *sp = reinterpret_cast<f32x4 *>(orow + jb * KB + 16 * g);
#pragma unroll
            for (int t = 0; t < 4; ++t) sp[t] = acc[t] * scale;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// O = A V.  SPARSE: A = kept weights [BH, Lq, Lk/2] fp32 + metadata of the 4-byte mode, expanded and
// split in registers; else A dense [BH, Lq, Lk] fp32.  Matrix step m (0, 1) of a 64-key block takes, in
// lane group g, the keys 32 m + 8 g .. +7: four kept weights and one 16-bit metadata word.  V blocks are
// converted like K blocks, into row-major bf16 images whose 16-byte chunk c of key k sits at chunk
// c ^ 2 (k % 4); the B operand (keys along the contraction) comes from the transposing LDS read.
// ---------------------------------------------------------------------------------------------
template <int D, bool SPARSE>
__global__ __launch_bounds__(NT, 2) void k_av_split(const float *__restrict__ A, const uint16_t *__restrict__ meta,
                                                    const float *__restrict__ V, int Lq, int Lk,
                                                    float *__restrict__ O) {
    constexpr int CPR = D / 8;
    constexpr int NCONV = KB * CPR / NT;
    constexpr int DS = D / 16;
    __shared__ __attribute__((aligned(16))) float Vf[KB * D];
    __shared__ u32x4 Vh[KB * CPR], Vl[KB * CPR];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, g = lane >> 4;
    const unsigned nqt = Lq / QT;
    const unsigned item = xcd_contiguous(blockIdx.x, gridDim.x);
    const unsigned bh = item / nqt, qt = item % nqt;
    const int nkb = Lk / KB;
    const int q = qt * QT + wave * 16 + li;      // A operand row of this lane

    const BlockCopy<D> copy{uniform_address(V + (size_t)bh * Lk * D), lds_address(&Vf[0]), (uint32_t)lane * 16u, wave};

    // weights of this lane for one block: two runs of 8 keys
    struct AFrag {
        f32x4 v[SPARSE ? 2 : 4];
        uint32_t code[2];
    };
    const float *arow = A + ((size_t)bh * Lq + q) * (SPARSE ? Lk / 2 : Lk);
    const uint16_t *mrow = SPARSE ? meta + ((size_t)bh * Lq + q) * (Lk / 8) : nullptr;
    auto load_a = [&](int jb, AFrag &a) {
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            if constexpr (SPARSE) {
                a.v[m] = *reinterpret_cast<const f32x4 *>(arow + jb * (KB / 2) + 16 * m + 4 * g);
                a.code[m] = mrow[jb * (KB / 8) + 4 * m + g];
            } else {
                const f32x4 *p = reinterpret_cast<const f32x4 *>(arow + jb * KB + 32 * m + 8 * g);
                a.v[2 * m] = p[0];
                a.v[2 * m + 1] = p[1];
                a.code[m] = 0;
            }
        }
    };

    f32x4 acc[DS];
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) acc[ds] = f32x4{0.f, 0.f, 0.f, 0.f};

    // transposing read: lane li of a 16-lane group addresses V[key0 + li/4][col0 + 4*(li%4)]
    const int tr_row = li >> 2;
    const int tr_sub = (li >> 1) & 1;
    const int tr_byte = 8 * (li & 1);
    const int tr_xor = tr_row << 1;
    auto tr8 = [&](const u32x4 *img, int key0, int ds) {
        const char *base = reinterpret_cast<const char *>(img);
        const int chunk = (2 * ds + tr_sub) ^ tr_xor;      // key0 is a multiple of 4: (row & 3) == tr_row
        const s16x4 t0 = lds_read_tr16(base + ((key0 + tr_row) * CPR + chunk) * 16 + tr_byte);
        const s16x4 t1 = lds_read_tr16(base + ((key0 + 4 + tr_row) * CPR + chunk) * 16 + tr_byte);
        return __builtin_bit_cast(u32x4, __builtin_shufflevector(t0, t1, 0, 1, 2, 3, 4, 5, 6, 7));
    };

    AFrag a_cur, a_nxt;
    load_a(0, a_cur);
    copy.issue(0);
    for (int jb = 0; jb < nkb; ++jb) {
        wait_async_copies();        // this block's V copy and weights
        __syncthreads();
#pragma unroll
        for (int i = 0; i < NCONV; ++i) {
            const int idx = i * NT + tid;
            const int key = idx / CPR, c = idx % CPR;
            const f32x4 *src = reinterpret_cast<const f32x4 *>(&Vf[key * D + 8 * c]);
            u32x4 h, l;
            split8(src[0], src[1], h, l);
            const int pos = key * CPR + (c ^ ((key & 3) << 1));
            Vh[pos] = h;
            Vl[pos] = l;
        }
        __syncthreads();
        if (jb + 1 < nkb) {
            copy.issue(jb + 1);
            load_a(jb + 1, a_nxt);
        }

#pragma unroll
        for (int m = 0; m < 2; ++m) {
            f32x4 a0, a1;       // the 8 dense weights of keys 32 m + 8 g .. +7
            if constexpr (SPARSE) {
                // pair p: code 0x4 keeps element 0, 0xE element 1 (they differ in bit 1)
                float d[8];
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const bool second = (a_cur.code[m] >> (4 * p + 1)) & 1u;
                    d[2 * p] = second ? 0.f : a_cur.v[m][p];
                    d[2 * p + 1] = second ? a_cur.v[m][p] : 0.f;
                }
                a0 = f32x4{d[0], d[1], d[2], d[3]};
                a1 = f32x4{d[4], d[5], d[6], d[7]};
            } else {
                a0 = a_cur.v[2 * m];
                a1 = a_cur.v[2 * m + 1];
            }
            u32x4 ah, al;
            split8(a0, a1, ah, al);
            const int key0 = 32 * m + 8 * g;
#pragma unroll
            for (int ds = 0; ds < DS; ++ds)
                acc[ds] = mfma_split(ah, al, tr8(Vh, key0, ds), tr8(Vl, key0, ds), acc[ds]);
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

template <bool PRUNE>
hipError_t launch_scores(const void *Q, const void *K, int BH, int Lq, int Lk, int d, float scale, void *out,
                         void *meta, hipStream_t st) {
    const unsigned grid = (unsigned)BH * (unsigned)(Lq / QT);
    if (d == 64)
        hipLaunchKernelGGL((k_scores_split<64, PRUNE>), dim3(grid), dim3(NT), 0, st, (const float *)Q,
                           (const float *)K, Lq, Lk, scale, (float *)out, (uint32_t *)meta);
    else if (d == 128)
        hipLaunchKernelGGL((k_scores_split<128, PRUNE>), dim3(grid), dim3(NT), 0, st, (const float *)Q,
                           (const float *)K, Lq, Lk, scale, (float *)out, (uint32_t *)meta);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

template <bool SPARSE>
hipError_t launch_av(const void *A, const void *meta, const void *V, int BH, int Lq, int Lk, int d, void *O,
                     hipStream_t st) {
    const unsigned grid = (unsigned)BH * (unsigned)(Lq / QT);
    if (d == 64)
        hipLaunchKernelGGL((k_av_split<64, SPARSE>), dim3(grid), dim3(NT), 0, st, (const float *)A,
                           (const uint16_t *)meta, (const float *)V, Lq, Lk, (float *)O);
    else if (d == 128)
        hipLaunchKernelGGL((k_av_split<128, SPARSE>), dim3(grid), dim3(NT), 0, st, (const float *)A,
                           (const uint16_t *)meta, (const float *)V, Lq, Lk, (float *)O);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace

hipError_t launch_sddmm_prune_split(const void *Q, const void *K, int BH, int Lq, int Lk, int d, float scale,
                                    void *vals, void *meta, hipStream_t st) {
    return launch_scores<true>(Q, K, BH, Lq, Lk, d, scale, vals, meta, st);
}
hipError_t launch_dense_scores_split(const void *Q, const void *K, int BH, int Lq, int Lk, int d, float scale,
                                     void *S, hipStream_t st) {
    return launch_scores<false>(Q, K, BH, Lq, Lk, d, scale, S, nullptr, st);
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
