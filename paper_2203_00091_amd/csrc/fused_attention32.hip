// Whole DFSS forward pass in one kernel, 32-query tiles (see fused_attention.hip for the
// method: arXiv 2203.00091, Sec. 3.1 stages, Sec. 3.4 pruning on the accumulators,
// App. A.1.3 softmax).  This variant forms the scores with v_mfma_f32_32x32x16_bf16, which
// on gfx950 delivers twice the flops per cycle of the 16x16x32 form, and multiplies by V
// with v_smfmac_f32_32x32x32_bf16.  It needs 32 queries per wave, so it is used when the
// problem has enough 32-query tiles to fill the chip; smaller problems use the 16-query
// kernel.
//
// Register layouts (lane l, h = l/32):
//   scores of one 32-key tile: lane holds query l%32 and, thanks to the key order of the
//   LDS rows (row 8g + 4h' + x holds key 16h' + 4g + x), the 16 consecutive keys
//   16h .. 16h+15 of the tile in registers 4g + x: four runs of four keys.
//   The 8 kept weights + 16 code bits of the lane are the A operand / index of the sparse
//   instruction for row l%32, contraction chunk h.
//   O and the row sums: column l%32 of a 32-column tile, rows (queries) 8(r/4) + 4h + r%4.
#include <type_traits>

#include "dfss_device.hpp"
#include "dfss_kernels.hpp"

namespace dfss {

namespace {

constexpr int KB = 64;    // keys per block (two 32-key tiles)
constexpr float kTau = 8.0f;
constexpr float kLog2e = 1.4426950408889634f;

enum { MODE_2TO4 = 0, MODE_1TO2 = 1, MODE_DENSE = 2 };

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));
template <int D, int MODE, int NW, bool PRESCALE>
__global__ __launch_bounds__(64 * NW, 2) void k_fused32(const __bf16 *__restrict__ Q, const __bf16 *__restrict__ K,
                                                        const __bf16 *__restrict__ V, int Lq, int Lk, float scale,
                                                        uint16_t *__restrict__ O) {
    constexpr int NT = 64 * NW;
    constexpr int CPR = D / 8;          // 16-byte chunks per row
    constexpr int TILE = KB * CPR;      // chunks per K (or V) block
    constexpr int LPT = TILE / NT;      // direct-to-LDS loads per thread per block and operand
    constexpr int STEPS = D / 16;       // k-steps of the 32x32x16 MFMA
    constexpr int DT = D / 32;          // 32-column tiles of O
    constexpr int TQ = 32 * NW;         // queries per workgroup
    constexpr bool SPARSE = MODE != MODE_DENSE;
    constexpr int NP = SPARSE ? 4 : 8;  // packed weight dwords per lane per key tile
    // two named buffers per operand (not one indexed array): the compiler can then see that the
    // buffer being filled by the direct-to-LDS copies is not the one being read
    __shared__ u32x4 Ks0[TILE], Ks1[TILE];
    __shared__ u32x4 Vs0[TILE], Vs1[TILE];

    const int tid = threadIdx.x;
    const int w = tid >> 6, l = tid & 63, lj = l & 31, h = l >> 5;

    const unsigned qtiles = Lq / TQ;
    const unsigned item = xcd_contiguous(blockIdx.x, gridDim.x);
    const int qt = item % qtiles;
    const int bh = item / qtiles;
    const int q0 = qt * TQ + w * 32;
    const int nblocks = Lk / KB;

    const __bf16 *Kh = K + (size_t)bh * Lk * D;
    const __bf16 *Vh = V + (size_t)bh * Lk * D;

    // K block in LDS: row slot 32 kt + i (key tile kt, MFMA row i = 8g + 4h' + x) holds key
    // 32 kt + 16 h' + 4 g + x; chunk c sits at slot * CPR + (c ^ (slot & 7)).
    // V block: row = key, chunk c at row * CPR + (c ^ ((row & 3) << 1)).
    int k_off[LPT], v_off[LPT];
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
        const int p = i * NT + tid;
        const int slot = p / CPR;
        const int key = (slot & 32) | (((slot >> 2) & 1) << 4) | (((slot >> 3) & 3) << 2) | (slot & 3);
        k_off[i] = key * D + ((p % CPR) ^ (slot & 7)) * 8;
        v_off[i] = slot * D + ((p % CPR) ^ ((slot & 3) << 1)) * 8;
    }
    auto issue_k = [&](int jb, u32x4 *dst) {
        const __bf16 *ks = Kh + (size_t)jb * KB * D;
        const uint32_t lds = lds_address(&dst[w * 64]);
#pragma unroll
        for (int i = 0; i < LPT; ++i) async_copy16(ks, 2u * k_off[i], lds + 16u * (i * NT));
    };
    auto issue_v = [&](int jb, u32x4 *dst) {
        const __bf16 *vs = Vh + (size_t)jb * KB * D;
        const uint32_t lds = lds_address(&dst[w * 64]);
#pragma unroll
        for (int i = 0; i < LPT; ++i) async_copy16(vs, 2u * v_off[i], lds + 16u * (i * NT));
    };

    issue_k(0, Ks0);
    // V buffer 1 is read (with all-zero weights) before it is first filled: clear it
    for (int i = tid; i < TILE; i += NT) Vs1[i] = u32x4{0u, 0u, 0u, 0u};

    // Q operand (B side of Q K^T): lane (column lj, half h) of step s holds Q[q][16 s + 8 h .. +7]
    bf16x8 bq[STEPS];
#pragma unroll
    for (int s = 0; s < STEPS; ++s) {
        const u32x4 raw =
            *reinterpret_cast<const u32x4 *>(Q + ((size_t)bh * Lq + q0 + lj) * D + 16 * s + 8 * h);
        if constexpr (PRESCALE) {
            u32x4 sc;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                sc[e] = pack_bf16x2(bf16_lo_to_f32(raw[e]) * scale, bf16_hi_to_f32(raw[e]) * scale);
            bq[s] = __builtin_bit_cast(bf16x8, sc);
        } else {
            bq[s] = __builtin_bit_cast(bf16x8, raw);
        }
    }

    float m_ref = 0.f;   // reference value of query lj (set from the first block)
    f32x16 acc_o[DT], acc_l;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        acc_l[r] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) acc_o[dt][r] = 0.f;
    }
    const uint32_t one2 = 0x3F803F80u;  // two bfloat16 ones
    const bf16x16 ones16 =
        __builtin_bit_cast(bf16x16, u32x8{one2, one2, one2, one2, one2, one2, one2, one2});
    const bf16x8 ones8 = __builtin_bit_cast(bf16x8, u32x4{one2, one2, one2, one2});

    // transposing LDS read (per group of 16 lanes): lane s addresses V[key0 + s/4][col0 + 4 (s%4)]
    const int s16 = l & 15;
    const int tr_row = s16 >> 2, tr_sub = (s16 >> 1) & 1, tr_byte = 8 * (s16 & 1), tr_xor = tr_row << 1;
    const int tr_colgrp = (l >> 4) & 1;   // which 16 of the 32 columns of a tile this lane group reads

    // scores of one block: acc[kt][4g + x] = s(query q0 + lj, key 64 jb + 32 kt + 16 h + 4 g + x)
    auto scores = [&](const u32x4 *Kbuf, f32x16 (&acc)[2]) {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[kt][r] = 0.f;
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                const bf16x8 ak =
                    __builtin_bit_cast(bf16x8, Kbuf[(32 * kt + lj) * CPR + ((2 * s + h) ^ (lj & 7))]);
                acc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak, bq[s], acc[kt], 0, 0, 0);
            }
        }
    };
    // O += P V and row sums += P 1 for one block whose weights are pk / idx
    auto weighted_sum = [&](const u32x4 *Vbuf, const uint32_t (&pk)[2][NP], const uint32_t (&idx)[2]) {
        const char *vbase = reinterpret_cast<const char *>(Vbuf);
        auto tr = [&](int key0, int dt) {
            const int row = key0 + tr_row;
            const int chunk = (4 * dt + 2 * tr_colgrp + tr_sub) ^ tr_xor;
            return lds_read_tr16(vbase + (row * CPR + chunk) * 16 + tr_byte);
        };
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            if constexpr (SPARSE) {
                // contraction index of the sparse instruction = key of the tile; B lane (column, h)
                // holds keys 8 h .. +7 and 16 + 8 h .. +7
                const bf16x8 a = __builtin_bit_cast(bf16x8, u32x4{pk[kt][0], pk[kt][1], pk[kt][2], pk[kt][3]});
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    const int k0 = 32 * kt + 8 * h;
                    const s16x4 t0 = tr(k0, dt), t1 = tr(k0 + 4, dt), t2 = tr(k0 + 16, dt), t3 = tr(k0 + 20, dt);
                    const s16x8 lo = __builtin_shufflevector(t0, t1, 0, 1, 2, 3, 4, 5, 6, 7);
                    const s16x8 hi = __builtin_shufflevector(t2, t3, 0, 1, 2, 3, 4, 5, 6, 7);
                    const bf16x16 b = __builtin_bit_cast(
                        bf16x16, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15));
                    acc_o[dt] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(a, b, acc_o[dt], (int)idx[kt], 0, 0);
                }
                acc_l = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(a, ones16, acc_l, (int)idx[kt], 0, 0);
            } else {
                // dense: MFMA m (0/1) contracts the lanes' keys 16 h' + 8 m .. +7 (h' = 0, 1)
#pragma unroll
                for (int m = 0; m < 2; ++m) {
                    const bf16x8 a = __builtin_bit_cast(
                        bf16x8, u32x4{pk[kt][4 * m], pk[kt][4 * m + 1], pk[kt][4 * m + 2], pk[kt][4 * m + 3]});
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

    // Software pipeline.  Iteration jb issues, for the matrix unit, the scores of block jb+1 and
    // the weighted sum of block jb-1, both independent of the vector-ALU work of the iteration
    // (prune + softmax of block jb), so the two units run side by side.
    //   K ring: K(jb+1) is read from buffer (jb+1)%2 while K(jb+2) is copied into buffer jb%2.
    //   V ring: V(jb-1) is read from buffer (jb-1)%2 while V(jb) is copied into buffer jb%2.
    // The first iteration multiplies all-zero weights with the cleared V buffer; the last one
    // computes scores of a stale K buffer that nobody uses: both keep the loop body branch-free.
    if (nblocks > 1) issue_k(1, Ks1);
    wait_async_copies();
    __syncthreads();
    f32x16 acc_cur[2], acc_nxt[2];
    scores(Ks0, acc_cur);
    uint32_t pk_prev[2][NP], idx_prev[2];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
        idx_prev[kt] = 0x4444u;
#pragma unroll
        for (int e = 0; e < NP; ++e) pk_prev[kt][e] = 0;
    }

    // one iteration; B = jb % 2 is a compile-time constant so that every LDS access names its buffer
    auto iteration = [&](auto parity, int jb) {
        constexpr int B = decltype(parity)::value;
        u32x4 *const Kfill = B ? Ks1 : Ks0;        // K(jb+2) goes where K(jb) was
        const u32x4 *const Kread = B ? Ks0 : Ks1;  // K(jb+1)
        u32x4 *const Vfill = B ? Vs1 : Vs0;        // V(jb)
        const u32x4 *const Vread = B ? Vs0 : Vs1;  // V(jb-1)

        wait_async_copies();  // vmcnt(0): K(jb+1) and V(jb-1) have landed
        __syncthreads();                     // ... for every wave, and iteration jb-1 is over everywhere
        if (jb + 2 < nblocks) issue_k(jb + 2, Kfill);
        issue_v(jb, Vfill);

        // ---- matrix unit: scores of the next block, weighted sum of the previous one ----
        scores(Kread, acc_nxt);
        weighted_sum(Vread, pk_prev, idx_prev);

        // ---- vector unit: prune block jb, block maximum ----
        float kept[2][2 * NP];
        uint32_t idx[2];
        float m_blk = -3.0e38f;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            idx[kt] = 0;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                float a0 = acc_cur[kt][4 * g], a1 = acc_cur[kt][4 * g + 1], a2 = acc_cur[kt][4 * g + 2],
                      a3 = acc_cur[kt][4 * g + 3];
                if constexpr (!PRESCALE) {
                    a0 *= scale; a1 *= scale; a2 *= scale; a3 *= scale;
                }
                if constexpr (SPARSE) {
                    float lo, hi;
                    uint32_t code;
                    if constexpr (MODE == MODE_2TO4) select_2of4(a0, a1, a2, a3, 4 * g, lo, hi, code);
                    else select_1of2(a0, a1, a2, a3, 4 * g, lo, hi, code);
                    kept[kt][2 * g] = lo;
                    kept[kt][2 * g + 1] = hi;
                    idx[kt] |= code;
                    m_blk = fmaxf(m_blk, fmaxf(lo, hi));
                } else {
                    kept[kt][4 * g] = a0; kept[kt][4 * g + 1] = a1; kept[kt][4 * g + 2] = a2; kept[kt][4 * g + 3] = a3;
                    m_blk = fmaxf(m_blk, fmaxf(fmaxf(a0, a1), fmaxf(a2, a3)));
                }
            }
        }
        // lanes lj and lj + 32 hold different keys of the same query
        m_blk = fmaxf(m_blk, __shfl_xor(m_blk, 32, 64));

        // ---- reference value: taken from the first block, raised when a later block outgrows it ----
        if (jb == 0) {
            m_ref = m_blk;
        } else if (__any(m_blk > m_ref + kTau)) {
            const bool up = m_blk > m_ref + kTau;
            const float m_new = up ? m_blk : m_ref;
            const float alpha = __builtin_amdgcn_exp2f((m_ref - m_new) * kLog2e);  // 1 where unchanged
            m_ref = m_new;
            // accumulator rows are queries 8 (r/4) + 4 h + r%4: fetch their factors from those columns' lanes
            // (acc_o already holds every block before jb, all weighted with the old reference value)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float a_r = __shfl(alpha, 8 * (r >> 2) + 4 * h + (r & 3), 64);
                acc_l[r] *= a_r;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) acc_o[dt][r] *= a_r;
            }
        }

        // ---- weights exp(s - m) of block jb, packed as the A operand of the second product ----
        const float mb = m_ref * kLog2e;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            idx_prev[kt] = idx[kt];
#pragma unroll
            for (int e = 0; e < NP; ++e) {
                const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(kept[kt][2 * e], kLog2e, -mb));
                const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(kept[kt][2 * e + 1], kLog2e, -mb));
                pk_prev[kt][e] = pack_bf16x2(p0, p1);
            }
        }
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) acc_cur[kt] = acc_nxt[kt];
    };

    for (int jb = 0; jb < nblocks; jb += 2) {
        iteration(std::integral_constant<int, 0>{}, jb);
        if (jb + 1 < nblocks) iteration(std::integral_constant<int, 1>{}, jb + 1);
    }
    // drain: weighted sum of the last block
    wait_async_copies();
    __syncthreads();
    if ((nblocks - 1) & 1) weighted_sum(Vs1, pk_prev, idx_prev);
    else weighted_sum(Vs0, pk_prev, idx_prev);

    // ---- O[q][32 dt + lj] = acc_o / row sum, q = q0 + 8 (r/4) + 4 h + r%4 ----
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const float inv = 1.0f / acc_l[r];
        const size_t q = (size_t)bh * Lq + q0 + 8 * (r >> 2) + 4 * h + (r & 3);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
            O[q * D + 32 * dt + lj] = (uint16_t)(pack_bf16x2(acc_o[dt][r] * inv, 0.f) & 0xFFFFu);
    }
}

inline bool is_pow2(float x) {
    int e;
    return frexpf(x, &e) == 0.5f;
}

template <int MODE, int NW>
hipError_t launch_nw(const void *Q, const void *K, const void *V, int BH, int Lq, int Lk, int d, float scale,
                     void *O, hipStream_t st) {
    const unsigned grid = (unsigned)((long)BH * (Lq / (32 * NW)));
    const bool pre = is_pow2(scale);
#define DFSS_LAUNCH(DD, PRE)                                                                                 \
    hipLaunchKernelGGL((k_fused32<DD, MODE, NW, PRE>), dim3(grid), dim3(64 * NW), 0, st, (const __bf16 *)Q, \
                       (const __bf16 *)K, (const __bf16 *)V, Lq, Lk, scale, (uint16_t *)O)
    if (d == 64) {
        if (pre) DFSS_LAUNCH(64, true); else DFSS_LAUNCH(64, false);
    } else if constexpr (NW == 4) {   // (two-wave workgroups are built for d = 64 only: at d = 128 they need the
                                      // registers of a whole SIMD and are never asked for)
        if (pre) DFSS_LAUNCH(128, true); else DFSS_LAUNCH(128, false);
    } else {
        return hipErrorInvalidValue;
    }
#undef DFSS_LAUNCH
    return hipGetLastError();
}

}  // namespace

// nw: waves (32-query tiles) per workgroup, 2 or 4; Lq must be a multiple of 32 * nw.
hipError_t launch_fused_attention32(const void *Q, const void *K, const void *V, int BH, int Lq, int Lk, int d,
                                    int mode, int nw, float scale, void *O, hipStream_t st) {
    if (nw == 4) {
        if (mode == 0) return launch_nw<MODE_2TO4, 4>(Q, K, V, BH, Lq, Lk, d, scale, O, st);
        if (mode == 1) return launch_nw<MODE_1TO2, 4>(Q, K, V, BH, Lq, Lk, d, scale, O, st);
        return launch_nw<MODE_DENSE, 4>(Q, K, V, BH, Lq, Lk, d, scale, O, st);
    }
    if (mode == 0) return launch_nw<MODE_2TO4, 2>(Q, K, V, BH, Lq, Lk, d, scale, O, st);
    if (mode == 1) return launch_nw<MODE_1TO2, 2>(Q, K, V, BH, Lq, Lk, d, scale, O, st);
    return launch_nw<MODE_DENSE, 2>(Q, K, V, BH, Lq, Lk, d, scale, O, st);
}

}  // namespace dfss
