// Stage 1 of the DFSS forward pass: S = scale * Q K^T on bf16 MFMA with the N:M pruning
// done on the accumulators, so the dense score matrix never reaches memory
// (arXiv 2203.00091, Sec. 3.4 and App. A.1.2).  The same mainloop with a plain
// bfloat16 store is the first stage of the dense baseline (Eq. 1).
//
// Tiling.  One workgroup (4 waves) computes 64 queries x 128 keys; each wave owns
// 32 queries x 64 keys as 2 x 4 MFMA tiles of 16 x 16.  The product is formed transposed
// (keys on the MFMA rows, queries on its columns) because a lane owns four consecutive
// ROWS of one column: with that orientation a lane owns runs of four consecutive keys of
// one query, which is what the selection needs.  Within a 64-key block the key that
// feeds MFMA row i of tile t is 16*(i/4) + 4*t + i%4, so that after the four tiles lane
// (column c, row group g) holds the 16 consecutive keys 16g .. 16g+15 of query c: eight
// kept values (16 bytes, one store) and four 4-bit codes (one 16-bit word).  This plays
// the role of the column interleaving of App. A.1.2, chosen here for the MFMA layout.
#include "dfss_device.hpp"
#include "dfss_kernels.hpp"

namespace dfss {

namespace {

constexpr int TQ = 64;    // queries per workgroup
constexpr int TK = 128;   // keys per workgroup
constexpr int NT = 256;   // threads per workgroup

enum { MODE_2TO4 = 0, MODE_1TO2 = 1, MODE_DENSE = 2 };

// Position of key row `r` (0..127) inside the LDS tile: within each block of 64 keys the
// two 2-bit fields (r/4)%4 and (r/16)%4 are swapped, which makes the 16 rows a wave reads
// for one MFMA tile adjacent in LDS (conflict-free 16-byte reads).
__device__ __forceinline__ int lds_key_slot(int r) {
    return (r & 64) | ((r & 0xC) << 2) | ((r & 0x30) >> 2) | (r & 3);
}

// The six comparisons of a run of four scores are taken as 64-bit lane masks (one bit per
// lane of the wave) so that the rank logic runs on the scalar unit, off the vector ALU
// that the MFMA epilogue is short of; the vector unit only does the final selects.
typedef uint64_t lanemask;
__device__ __forceinline__ lanemask gt(float a, float b) { return __builtin_amdgcn_fcmpf(a, b, 2 /* ordered > */); }
__device__ __forceinline__ bool lane_bit(lanemask m) { return __builtin_amdgcn_inverse_ballot_w64(m); }

// Keep the two largest of four scores; equal scores: the lower index wins
// (rank(t) = #{u: s_u > s_t} + #{u < t: s_u == s_t}; keep iff rank < 2).
// Returns the kept values in key order and the position code (p_lo | p_hi << 2) << SHIFT
// (SHIFT is a constant after unrolling: the code lands directly in its slot of the word).
__device__ __forceinline__ void select_2of4(float s0, float s1, float s2, float s3, const int SHIFT, float &lo,
                                            float &hi, uint32_t &code) {
    // cXY: the later element Y is strictly larger than X, i.e. Y outranks X;
    // otherwise X outranks Y (ties go to the lower index).
    const lanemask c01 = gt(s1, s0), c02 = gt(s2, s0), c03 = gt(s3, s0);
    const lanemask c12 = gt(s2, s1), c13 = gt(s3, s1), c23 = gt(s3, s2);
    // element t survives unless at least two others outrank it
    const lanemask k0 = ~((c01 & (c02 | c03)) | (c02 & c03));
    const lanemask k1 = ~((~c01 & (c12 | c13)) | (c12 & c13));
    const lanemask k2 = ~((~c02 & (~c12 | c23)) | (~c12 & c23));
    const lanemask k3 = ~((~c03 & (~c13 | ~c23)) | (~c13 & ~c23));
    const bool b0 = lane_bit(k0), b1 = lane_bit(k1), b2 = lane_bit(k2), b3 = lane_bit(k3);
    lo = b0 ? s0 : (b1 ? s1 : s2);
    hi = b3 ? s3 : (b2 ? s2 : s1);
    const uint32_t plo = b0 ? 0u : (b1 ? (1u << SHIFT) : (2u << SHIFT));
    const uint32_t phi = b3 ? (12u << SHIFT) : (b2 ? (8u << SHIFT) : (4u << SHIFT));
    code = plo | phi;
}

// Keep the larger of each aligned pair; equal scores: the lower index wins.
__device__ __forceinline__ void select_1of2(float s0, float s1, float s2, float s3, const int SHIFT, float &lo,
                                            float &hi, uint32_t &code) {
    const bool c01 = lane_bit(gt(s1, s0)), c23 = lane_bit(gt(s3, s2));
    lo = c01 ? s1 : s0;
    hi = c23 ? s3 : s2;
    code = (c01 ? (1u << SHIFT) : 0u) | (c23 ? (12u << SHIFT) : (8u << SHIFT));
}

template <int D, int MODE>
__global__ __launch_bounds__(NT, 2) void k_sddmm(const __bf16 *__restrict__ Q, const __bf16 *__restrict__ K,
                                              int Lq, int Lk, float scale, uint32_t *__restrict__ out,
                                              uint16_t *__restrict__ meta) {
    constexpr int KC = D / 8;       // 16-byte chunks per row
    constexpr int KROWS = TK + 1;   // +1 row of padding: conflict-free LDS writes
    constexpr int QROWS = TQ + 1;
    __shared__ u32x4 Ks[KC * KROWS];
    __shared__ u32x4 Qs[KC * QROWS];

    const int tid = threadIdx.x;
    const int bh = blockIdx.z;
    const int q0 = blockIdx.y * TQ;
    const int k0 = blockIdx.x * TK;

    {
        const u32x4 *Kg = reinterpret_cast<const u32x4 *>(K + ((size_t)bh * Lk + k0) * D);
        for (int c = tid; c < TK * KC; c += NT) {
            const int row = c / KC, kc = c % KC;
            Ks[kc * KROWS + lds_key_slot(row)] = Kg[c];
        }
        const u32x4 *Qg = reinterpret_cast<const u32x4 *>(Q + ((size_t)bh * Lq + q0) * D);
        for (int c = tid; c < TQ * KC; c += NT) {
            const int row = c / KC, kc = c % KC;
            Qs[kc * QROWS + row] = Qg[c];
        }
    }
    __syncthreads();

    const int w = tid >> 6, l = tid & 63, li = l & 15, kb = l >> 4;
    const int wq = w & 1, wk = w >> 1;

    f32x4 acc[2][4];
#pragma unroll
    for (int qs = 0; qs < 2; ++qs)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) acc[qs][ks] = f32x4{0.f, 0.f, 0.f, 0.f};

#pragma unroll
    for (int step = 0; step < D / 32; ++step) {
        bf16x8 bq[2], ak[4];
        const int kc = 4 * step + kb;
#pragma unroll
        for (int qs = 0; qs < 2; ++qs)
            bq[qs] = __builtin_bit_cast(bf16x8, Qs[kc * QROWS + 32 * wq + 16 * qs + li]);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            ak[ks] = __builtin_bit_cast(bf16x8, Ks[kc * KROWS + 64 * wk + 16 * ks + li]);
#pragma unroll
        for (int qs = 0; qs < 2; ++qs)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) acc[qs][ks] = mfma16(ak[ks], bq[qs], acc[qs][ks]);
    }

    // acc[qs][ks][r] = dot(Q[q], K[key]) with q = q0 + 32 wq + 16 qs + li,
    // key = k0 + 64 wk + 16 kb + 4 ks + r.
    const int kbase = k0 + 64 * wk + 16 * kb;
#pragma unroll
    for (int qs = 0; qs < 2; ++qs) {
        const int q = q0 + 32 * wq + 16 * qs + li;
        const size_t row = (size_t)bh * Lq + q;
        if constexpr (MODE == MODE_DENSE) {
            uint32_t p[8];
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                p[2 * ks] = pack_bf16x2(acc[qs][ks][0] * scale, acc[qs][ks][1] * scale);
                p[2 * ks + 1] = pack_bf16x2(acc[qs][ks][2] * scale, acc[qs][ks][3] * scale);
            }
            u32x4 *dst = reinterpret_cast<u32x4 *>(out + (row * Lk + kbase) / 2);
            dst[0] = u32x4{p[0], p[1], p[2], p[3]};
            dst[1] = u32x4{p[4], p[5], p[6], p[7]};
        } else {
            u32x4 pk;
            uint32_t word = 0;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const float s0 = acc[qs][ks][0] * scale, s1 = acc[qs][ks][1] * scale;
                const float s2 = acc[qs][ks][2] * scale, s3 = acc[qs][ks][3] * scale;
                float lo, hi;
                uint32_t code;
                if constexpr (MODE == MODE_2TO4) select_2of4(s0, s1, s2, s3, 4 * ks, lo, hi, code);
                else select_1of2(s0, s1, s2, s3, 4 * ks, lo, hi, code);
                pk[ks] = pack_bf16x2(lo, hi);
                word |= code;
            }
            *reinterpret_cast<u32x4 *>(out + (row * (size_t)(Lk / 2) + kbase / 2) / 2) = pk;
            const int W = Lk / 16;
            meta[(((size_t)bh * (Lq / 16) + q / 16) * W + kbase / 16) * 16 + li] = (uint16_t)word;
        }
    }
}

template <int MODE>
hipError_t launch(const void *Q, const void *K, int BH, int Lq, int Lk, int d, float scale, void *out,
                  void *meta, hipStream_t st) {
    dim3 grid(Lk / TK, Lq / TQ, BH), block(NT);
    if (d == 64)
        hipLaunchKernelGGL((k_sddmm<64, MODE>), grid, block, 0, st, (const __bf16 *)Q, (const __bf16 *)K, Lq, Lk,
                           scale, (uint32_t *)out, (uint16_t *)meta);
    else
        hipLaunchKernelGGL((k_sddmm<128, MODE>), grid, block, 0, st, (const __bf16 *)Q, (const __bf16 *)K, Lq, Lk,
                           scale, (uint32_t *)out, (uint16_t *)meta);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_sddmm_prune(const void *Q, const void *K, int BH, int Lq, int Lk, int d, int mode, float scale,
                              void *vals, void *meta, hipStream_t st) {
    return mode == 0 ? launch<MODE_2TO4>(Q, K, BH, Lq, Lk, d, scale, vals, meta, st)
                     : launch<MODE_1TO2>(Q, K, BH, Lq, Lk, d, scale, vals, meta, st);
}

hipError_t launch_dense_scores(const void *Q, const void *K, int BH, int Lq, int Lk, int d, float scale, void *S,
                               hipStream_t st) {
    return launch<MODE_DENSE>(Q, K, BH, Lq, Lk, d, scale, S, nullptr, st);
}

}  // namespace dfss
