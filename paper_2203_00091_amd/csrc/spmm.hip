// Stage 3 of the DFSS forward pass: O = A_sparse V with the 2:4-compressed attention
// weights (arXiv 2203.00091, Sec. 3.1), on the gfx950 structured-sparse matrix
// instruction v_smfmac_f32_16x16x64_bf16: per lane eight kept weights (one 16-byte load,
// exactly what stage 1 stored) plus the lane's 16-bit metadata word as the index operand.
// Because 1:2 pruning is stored with the same 4-bit codes it runs through the same kernel.
// The dense variant (full P V of Eq. 1, for the baseline) shares the V staging and uses
// two v_mfma_f32_16x16x32_bf16 per 64 keys.
//
// V tiles (64 keys x d) are staged row-major in LDS; the B operand (keys along the
// contraction, one d-column per lane) is produced by the transposing LDS read.
#include "dfss_device.hpp"
#include "dfss_kernels.hpp"

namespace dfss {

namespace {

constexpr int NT = 256;        // 4 waves
constexpr int RB = 1;          // 16-row blocks per wave
constexpr int TQ = 4 * 16 * RB;  // queries per workgroup
constexpr int KT = 64;         // keys per step

template <int D, bool SPARSE>
__global__ __launch_bounds__(NT, 2) void k_av(const uint32_t *__restrict__ P, const uint16_t *__restrict__ meta,
                                           const __bf16 *__restrict__ V, int Lq, int Lk,
                                           uint16_t *__restrict__ O) {
    constexpr int VSTRIDE = D + 16;  // bf16 elements per LDS row (+32 bytes of padding)
    constexpr int DS = D / 16;       // 16-column output tiles
    __shared__ __attribute__((aligned(16))) __bf16 Vs[KT * VSTRIDE];

    const int tid = threadIdx.x;
    const int bh = blockIdx.y;
    const int q0 = blockIdx.x * TQ;
    const int w = tid >> 6, l = tid & 63, li = l & 15, kb = l >> 4;
    const int W = Lk / 16;

    f32x4 acc[RB][DS];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int ds = 0; ds < DS; ++ds) acc[rb][ds] = f32x4{0.f, 0.f, 0.f, 0.f};

    // row of P this lane feeds (A operand row = li)
    const int rowblk0 = (q0 >> 4) + w * RB;
    const int nsteps = Lk / KT;

    // per-lane offsets of the four transposing reads of one 16-column tile:
    // source lane s = li reads 4 elements at V[key0 + s/4][col0 + 4*(s%4)]
    const int tr_row = li >> 2, tr_col = 4 * (li & 3);

    for (int step = 0; step < nsteps; ++step) {
        __syncthreads();  // previous step's LDS reads are done
        {
            const u32x4 *Vg = reinterpret_cast<const u32x4 *>(V + ((size_t)bh * Lk + (size_t)step * KT) * D);
            for (int c = tid; c < KT * (D / 8); c += NT) {
                const int row = c / (D / 8), kc = c % (D / 8);
                *reinterpret_cast<u32x4 *>(&Vs[row * VSTRIDE + kc * 8]) = Vg[c];
            }
        }
        // A operands for this step (global loads overlap the LDS fill)
        bf16x8 a_sp[RB];
        int idx[RB];
        bf16x8 a_d0[RB], a_d1[RB];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const size_t row = (size_t)bh * Lq + (size_t)(rowblk0 + rb) * 16 + li;
            if constexpr (SPARSE) {
                const u32x4 *pr = reinterpret_cast<const u32x4 *>(P + row * (size_t)(Lk / 4));
                a_sp[rb] = __builtin_bit_cast(bf16x8, pr[step * 4 + kb]);
                idx[rb] = meta[(((size_t)bh * (Lq / 16) + rowblk0 + rb) * W + step * 4 + kb) * 16 + li];
            } else {
                const u32x4 *pr = reinterpret_cast<const u32x4 *>(P + row * (size_t)(Lk / 2));
                a_d0[rb] = __builtin_bit_cast(bf16x8, pr[step * 8 + kb]);
                a_d1[rb] = __builtin_bit_cast(bf16x8, pr[step * 8 + 4 + kb]);
            }
        }
        __syncthreads();
#pragma unroll
        for (int ds = 0; ds < DS; ++ds) {
            const __bf16 *base = &Vs[tr_row * VSTRIDE + 16 * ds + tr_col];
            const s16x4 t0 = lds_read_tr16(base + (8 * kb) * VSTRIDE);
            const s16x4 t1 = lds_read_tr16(base + (8 * kb + 4) * VSTRIDE);
            const s16x4 t2 = lds_read_tr16(base + (32 + 8 * kb) * VSTRIDE);
            const s16x4 t3 = lds_read_tr16(base + (32 + 8 * kb + 4) * VSTRIDE);
            const s16x8 lo = __builtin_shufflevector(t0, t1, 0, 1, 2, 3, 4, 5, 6, 7);
            const s16x8 hi = __builtin_shufflevector(t2, t3, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                if constexpr (SPARSE) {
                    const s16x16 b = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13,
                                                             14, 15);
                    acc[rb][ds] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(
                        a_sp[rb], __builtin_bit_cast(bf16x16, b), acc[rb][ds], idx[rb], 0, 0);
                } else {
                    acc[rb][ds] = mfma16(a_d0[rb], __builtin_bit_cast(bf16x8, lo), acc[rb][ds]);
                    acc[rb][ds] = mfma16(a_d1[rb], __builtin_bit_cast(bf16x8, hi), acc[rb][ds]);
                }
            }
        }
    }

    // acc[rb][ds][r] = O[q][16 ds + li], q = 16 (rowblk0 + rb) + 4 kb + r
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const size_t q = (size_t)bh * Lq + (size_t)(rowblk0 + rb) * 16 + 4 * kb + r;
#pragma unroll
            for (int ds = 0; ds < DS; ++ds)
                O[q * D + 16 * ds + li] = (uint16_t)(pack_bf16x2(acc[rb][ds][r], 0.f) & 0xFFFFu);
        }
}

template <bool SPARSE>
hipError_t launch(const void *P, const void *meta, const void *V, int BH, int Lq, int Lk, int d, void *O,
                  hipStream_t st) {
    dim3 grid(Lq / TQ, BH), block(NT);
    if (d == 64)
        hipLaunchKernelGGL((k_av<64, SPARSE>), grid, block, 0, st, (const uint32_t *)P, (const uint16_t *)meta,
                           (const __bf16 *)V, Lq, Lk, (uint16_t *)O);
    else
        hipLaunchKernelGGL((k_av<128, SPARSE>), grid, block, 0, st, (const uint32_t *)P, (const uint16_t *)meta,
                           (const __bf16 *)V, Lq, Lk, (uint16_t *)O);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_spmm(const void *vals, const void *meta, const void *V, int BH, int Lq, int Lk, int d, void *O,
                       hipStream_t st) {
    return launch<true>(vals, meta, V, BH, Lq, Lk, d, O, st);
}

hipError_t launch_dense_av(const void *P, const void *V, int BH, int Lq, int Lk, int d, void *O, hipStream_t st) {
    return launch<false>(P, nullptr, V, BH, Lq, Lk, d, O, st);
}

}  // namespace dfss
