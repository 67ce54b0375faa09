// The 4-byte mode of the DFSS forward pass (arXiv 2203.00091, Sec. 2.3: 1:2 selection on float
// data; App. A.1.1: the metadata codes of that mode; App. A.1.2: scores with fp32 accumulation).
// The paper multiplies float inputs on the tensor cores in a reduced-mantissa format; gfx950 has no
// such format, so the products here are formed by the plain fp32 matrix instruction
// v_mfma_f32_16x16x4_f32 (fp32 products, fp32 accumulation: at least the paper's precision).
//
// Register layout of v_mfma_f32_16x16x4_f32 (wave64, lane l; one value per lane for A and B):
//   A: row i = l%16, k = l/16        B: col j = l%16, k = l/16
//   D: col j = l%16, rows i = 4*(l/16)+r (r = 0..3)
// As in the 2-byte kernels the KEYS sit on the output rows, so the two scores of an aligned pair of
// keys of one query are adjacent registers of one lane and the 1:2 choice is one compare and one
// select, with no cross-lane traffic.  The rows of a 64-key block are permuted on their way into
// LDS such that a lane ends up with 16 CONSECUTIVE keys (its four output tiles are keys
// 16g+4t .. 16g+4t+3, g = l/16): it then writes 32 contiguous bytes of kept scores and one whole
// 32-bit metadata word per block, or 64 contiguous bytes of the dense row.
//
// Metadata of this mode: one 4-bit code per kept float (0x4 = first of the pair, 0xE = second),
// the code of pair p of a row at bits [4(p%4), 4(p%4)+3] of uint16 word p/4.  A lane's 8 codes are
// one aligned pair of words = one 32-bit word; the 32-bit words are stored blocked,
// [BH, Lq/16, Lk/64, 16 rows, 4 words], so that the 16 rows x 16 bytes a wave produces per block are
// 256 contiguous bytes (16-byte pieces of 16 rows cost a partial-line write each).
#include "dfss_device.hpp"
#include "dfss_kernels.hpp"

namespace dfss {

namespace {

constexpr int NT = 256;   // 4 waves, 16 queries each
constexpr int QT = 64;    // queries per workgroup
constexpr int KB = 64;    // keys per block

__device__ __forceinline__ f32x4 mfma4(float a, float b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// LDS slot (row of the staged block) -> key of the block, for the score kernel: tile t = slot/16
// holds, in its row i, key 16*(i/4) + 4t + i%4.
__device__ __forceinline__ int key_of_slot(int slot) {
    const int t = slot >> 4, i = slot & 15;
    return 16 * (i >> 2) + 4 * t + (i & 3);
}

// ---------------------------------------------------------------------------------------------
// Scores of the 4-byte mode.  PRUNE: keep the larger of each aligned pair (equal: the first),
// write kept scores [BH, Lq, Lk/2] fp32 and the metadata words; else write S [BH, Lq, Lk] fp32.
// One workgroup: 64 queries of one head, all keys in blocks of 64, K double-buffered in LDS by
// asynchronous copies.  A 16-byte chunk c of the row in LDS slot s is stored at chunk c ^ (s%16),
// which spreads the 16 rows that one 128-bit read touches over all banks.
// ---------------------------------------------------------------------------------------------
// BIAS: key_bias [B][Lk] (fp32, shared by the H heads of a batch element; -inf masks a key) is added to the scaled
// score before the comparison: score = fl(fl(scale * q.k) + bias), two roundings.
template <int D, bool PRUNE, bool BIAS>
__global__ __launch_bounds__(NT, 2) void k_scores_f32(const float *__restrict__ Q, const float *__restrict__ K,
                                                      const float *__restrict__ key_bias, int H,
                                                      int Lq, int Lk, float scale, float *__restrict__ out,
                                                      uint32_t *__restrict__ meta) {
    constexpr int CPR = D / 4;                   // 16-byte chunks per row
    constexpr int NCOPY = KB * CPR / NT;         // copy instructions per thread per block
    constexpr int KS = D / 4;                    // matrix instructions per tile (k = 4 each)
    constexpr int NSTORE = PRUNE ? 3 : 4;        // vector stores per lane per block
    __shared__ __attribute__((aligned(16))) float Ks[2][KB * D];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    const unsigned nqt = Lq / QT;
    const unsigned item = xcd_contiguous(blockIdx.x, gridDim.x);
    const unsigned bh = item / nqt, qt = item % nqt;
    const int nkb = Lk / KB;

    // this lane's share of Q: query q, k = g*KS + s  (one B operand per matrix instruction)
    const int q = qt * QT + wave * 16 + n;
    float qv[KS];
    {
        const f32x4 *qp = reinterpret_cast<const f32x4 *>(Q + ((size_t)bh * Lq + q) * D + g * KS);
#pragma unroll
        for (int c = 0; c < KS / 4; ++c) {
            const f32x4 v = qp[c];
#pragma unroll
            for (int e = 0; e < 4; ++e) qv[4 * c + e] = v[e];
        }
    }

    // source byte offsets (within a block of K) of the chunks this lane copies
    uint32_t src[NCOPY];
#pragma unroll
    for (int c = 0; c < NCOPY; ++c) {
        const int p = (c * 4 + wave) * 64 + lane;           // chunk position in the LDS buffer
        const int slot = p / CPR, cl = p % CPR;
        src[c] = (uint32_t)(key_of_slot(slot) * D * 4 + ((cl ^ (slot & 15)) * 16));
    }
    const uint64_t kbase = uniform_address(K + (size_t)bh * Lk * D);
    const uint32_t lds0 = lds_address(&Ks[0][0]);
    auto issue_block = [&](int jb) {
        const uint64_t base = kbase + (uint64_t)jb * (KB * D * 4);
        const uint32_t lds = lds0 + (uint32_t)(jb & 1) * (KB * D * 4);
#pragma unroll
        for (int c = 0; c < NCOPY; ++c) async_copy16(base, src[c], lds + (uint32_t)((c * 4 + wave) * 1024));
    };

    const float *const brow = BIAS ? key_bias + (size_t)(bh / H) * Lk : nullptr;
    float *orow = out + ((size_t)bh * Lq + q) * (PRUNE ? Lk / 2 : Lk);
    // metadata word of (row group, block jb, row n, lane group g)
    uint32_t *mrow = PRUNE ? meta + ((size_t)bh * (Lq / 16) + (q >> 4)) * nkb * 64 + n * 4 + g : nullptr;

    issue_block(0);
    for (int jb = 0; jb < nkb; ++jb) {
        // the copies of block jb are older than the stores of block jb-1: leave those in flight
        if (jb == 0) wait_async_copies();
        else wait_async_copies_keep<NSTORE>();
        __syncthreads();            // block jb landed for all waves; all waves are done with block jb-1
        // bias of this lane's keys 64 jb + 16 g + 4 t + e, loaded before the next block's copies are issued (the
        // memory counter retires in order: waiting for these loads must not mean waiting for those copies)
        f32x4 b4[4];
        if constexpr (BIAS) {
#pragma unroll
            for (int t = 0; t < 4; ++t) b4[t] = *reinterpret_cast<const f32x4 *>(brow + jb * KB + 16 * g + 4 * t);
        }
        if (jb + 1 < nkb) issue_block(jb + 1);

        const float *kb = &Ks[jb & 1][0];
        f32x4 acc[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
            const int slot = 16 * t + n;
            const f32x4 *row = reinterpret_cast<const f32x4 *>(kb + slot * D);
            float kv[KS];
#pragma unroll
            for (int c = 0; c < KS / 4; ++c) {
                const f32x4 v = row[(g * (KS / 4) + c) ^ n];
#pragma unroll
                for (int e = 0; e < 4; ++e) kv[4 * c + e] = v[e];
            }
#pragma unroll
            for (int s = 0; s < KS; ++s) acc[t] = mfma4(kv[s], qv[s], acc[t]);
        }

        if constexpr (PRUNE) {
            f32x4 kept[2];
            uint32_t word = 0;
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    float s0 = acc[t][2 * h] * scale, s1 = acc[t][2 * h + 1] * scale;
                    if constexpr (BIAS) s0 = add_unfused(s0, b4[t][2 * h]), s1 = add_unfused(s1, b4[t][2 * h + 1]);
                    const bool second = s1 > s0;
                    const int p = 2 * t + h;
                    kept[p >> 2][p & 3] = second ? s1 : s0;
                    word |= (second ? 0xEu : 0x4u) << (4 * p);
                }
            f32x4 *vp = reinterpret_cast<f32x4 *>(orow + jb * (KB / 2) + 8 * g);
            vp[0] = kept[0];
            vp[1] = kept[1];
            mrow[jb * 64] = word;
        } else {
            f32x4 *sp = reinterpret_cast<f32x4 *>(orow + jb * KB + 16 * g);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                f32x4 v = acc[t] * scale;
                if constexpr (BIAS) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = add_unfused(v[e], b4[t][e]);
                }
                sp[t] = v;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// O = A V for fp32 weights.  SPARSE: A is given as kept weights [BH, Lq, Lk/2] fp32 plus the
// metadata words of the 4-byte mode, and is expanded in registers (the matrix units of gfx950
// have no structured-sparse fp32 form, so the saving is the halved read of A, not the
// arithmetic); else A is dense [BH, Lq, Lk] fp32.
// Matrix instruction step t of a 64-key block contracts the four keys 16g + t (g = 0..3), so a lane
// needs exactly the 16 consecutive keys 16g .. 16g+15 of its query row: 8 kept weights + one
// 32-bit metadata word (or 16 dense weights), all contiguous in memory.
// V is staged in LDS by asynchronous copies with chunk c of key k stored at chunk c ^ 4*((k/16)%4):
// the four 16-lane groups of one 32-bit read then fall into different banks.
// ---------------------------------------------------------------------------------------------
template <int D, bool SPARSE>
__global__ __launch_bounds__(NT, 2) void k_av_f32(const float *__restrict__ A, const uint32_t *__restrict__ meta,
                                                  const float *__restrict__ V, int Lq, int Lk,
                                                  float *__restrict__ O) {
    constexpr int CPR = D / 4;
    constexpr int NCOPY = KB * CPR / NT;
    constexpr int DS = D / 16;                   // 16-column tiles of O
    constexpr int NA = SPARSE ? 2 : 4;           // 16-byte loads of A per lane per block
    __shared__ __attribute__((aligned(16))) float Vs[2][KB * D];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    const unsigned nqt = Lq / QT;
    const unsigned item = xcd_contiguous(blockIdx.x, gridDim.x);
    const unsigned bh = item / nqt, qt = item % nqt;
    const int nkb = Lk / KB;
    const int q = qt * QT + wave * 16 + n;       // the query whose weights this lane feeds (A operand row)

    uint32_t src[NCOPY];
#pragma unroll
    for (int c = 0; c < NCOPY; ++c) {
        const int p = (c * 4 + wave) * 64 + lane;
        const int key = p / CPR, cl = p % CPR;
        src[c] = (uint32_t)(key * D * 4 + ((cl ^ (4 * ((key >> 4) & 3))) * 16));
    }
    const uint64_t vbase = uniform_address(V + (size_t)bh * Lk * D);
    const uint32_t lds0 = lds_address(&Vs[0][0]);
    auto issue_block = [&](int jb) {
        const uint64_t base = vbase + (uint64_t)jb * (KB * D * 4);
        const uint32_t lds = lds0 + (uint32_t)(jb & 1) * (KB * D * 4);
#pragma unroll
        for (int c = 0; c < NCOPY; ++c) async_copy16(base, src[c], lds + (uint32_t)((c * 4 + wave) * 1024));
    };

    const float *arow = A + ((size_t)bh * Lq + q) * (SPARSE ? Lk / 2 : Lk) + (SPARSE ? 8 : 16) * g;
    const uint32_t *mrow = SPARSE ? meta + ((size_t)bh * (Lq / 16) + (q >> 4)) * nkb * 64 + n * 4 + g : nullptr;
    auto load_a = [&](int jb, f32x4 (&a)[NA], uint32_t &w) {
        const f32x4 *ap = reinterpret_cast<const f32x4 *>(arow + jb * (SPARSE ? KB / 2 : KB));
#pragma unroll
        for (int c = 0; c < NA; ++c) a[c] = ap[c];
        if constexpr (SPARSE) w = mrow[jb * 64];
    };

    f32x4 acc[DS];
#pragma unroll
    for (int nt = 0; nt < DS; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    f32x4 a_cur[NA];
    uint32_t w_cur = 0;
    load_a(0, a_cur, w_cur);
    issue_block(0);
    for (int jb = 0; jb < nkb; ++jb) {
        wait_async_copies();        // also completes the (older) loads of this block's weights
        __syncthreads();
        f32x4 a_nxt[NA];
        uint32_t w_nxt = 0;
        if (jb + 1 < nkb) {
            issue_block(jb + 1);
            load_a(jb + 1, a_nxt, w_nxt);
        }

        const float *vb = &Vs[jb & 1][0];
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            float a;
            if constexpr (SPARSE) {
                // pair t/2 of this lane's 8 pairs: code 0x4 keeps element 0, 0xE element 1 (they differ in bit 1)
                const uint32_t second = (w_cur >> (4 * (t >> 1) + 1)) & 1u;
                a = second == (uint32_t)(t & 1) ? a_cur[t >> 3][(t >> 1) & 3] : 0.f;
            } else {
                a = a_cur[t >> 2][t & 3];
            }
            const float *vrow = vb + (16 * g + t) * D + n;
#pragma unroll
            for (int nt = 0; nt < DS; ++nt) acc[nt] = mfma4(a, vrow[(nt ^ g) * 16], acc[nt]);
        }
        if (jb + 1 < nkb) {
#pragma unroll
            for (int c = 0; c < NA; ++c) a_cur[c] = a_nxt[c];
            w_cur = w_nxt;
        }
    }

    // D layout: column n of tile nt, rows (queries) 4g + r
    float *op = O + ((size_t)bh * Lq + qt * QT + wave * 16 + 4 * g) * D + n;
#pragma unroll
    for (int nt = 0; nt < DS; ++nt)
#pragma unroll
        for (int r = 0; r < 4; ++r) op[(size_t)r * D + nt * 16] = acc[nt][r];
}

template <bool PRUNE>
hipError_t launch_scores(const void *Q, const void *K, const float *key_bias, int H, int BH, int Lq, int Lk, int d,
                         float scale, void *out, void *meta, hipStream_t st) {
    const unsigned grid = (unsigned)BH * (unsigned)(Lq / QT);
    if (d != 64 && d != 128) return hipErrorInvalidValue;
#define DFSS_LAUNCH(DD, BB)                                                                                         \
    hipLaunchKernelGGL((k_scores_f32<DD, PRUNE, BB>), dim3(grid), dim3(NT), 0, st, (const float *)Q, (const float *)K, \
                       key_bias, H, Lq, Lk, scale, (float *)out, (uint32_t *)meta)
    if (d == 64) {
        if (key_bias) DFSS_LAUNCH(64, true); else DFSS_LAUNCH(64, false);
    } else {
        if (key_bias) DFSS_LAUNCH(128, true); else DFSS_LAUNCH(128, false);
    }
#undef DFSS_LAUNCH
    return hipGetLastError();
}

template <bool SPARSE>
hipError_t launch_av(const void *A, const void *meta, const void *V, int BH, int Lq, int Lk, int d, void *O,
                     hipStream_t st) {
    const unsigned grid = (unsigned)BH * (unsigned)(Lq / QT);
    if (d == 64)
        hipLaunchKernelGGL((k_av_f32<64, SPARSE>), dim3(grid), dim3(NT), 0, st, (const float *)A,
                           (const uint32_t *)meta, (const float *)V, Lq, Lk, (float *)O);
    else if (d == 128)
        hipLaunchKernelGGL((k_av_f32<128, SPARSE>), dim3(grid), dim3(NT), 0, st, (const float *)A,
                           (const uint32_t *)meta, (const float *)V, Lq, Lk, (float *)O);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace

hipError_t launch_sddmm_prune_f32(const void *Q, const void *K, const float *key_bias, int H, int BH, int Lq, int Lk,
                                  int d, float scale, void *vals, void *meta, hipStream_t st) {
    return launch_scores<true>(Q, K, key_bias, H, BH, Lq, Lk, d, scale, vals, meta, st);
}
hipError_t launch_dense_scores_f32(const void *Q, const void *K, const float *key_bias, int H, int BH, int Lq, int Lk,
                                   int d, float scale, void *S, hipStream_t st) {
    return launch_scores<false>(Q, K, key_bias, H, BH, Lq, Lk, d, scale, S, nullptr, st);
}
hipError_t launch_spmm_f32(const void *vals, const void *meta, const void *V, int BH, int Lq, int Lk, int d, void *O,
                           hipStream_t st) {
    return launch_av<true>(vals, meta, V, BH, Lq, Lk, d, O, st);
}
hipError_t launch_dense_av_f32(const void *P, const void *V, int BH, int Lq, int Lk, int d, void *O, hipStream_t st) {
    return launch_av<false>(P, nullptr, V, BH, Lq, Lk, d, O, st);
}

}  // namespace dfss
