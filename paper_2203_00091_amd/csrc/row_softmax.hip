// Stage 2 of the DFSS forward pass: softmax over the kept scores of each row, in place
// (arXiv 2203.00091, Sec. 3.1; max-subtracted form of App. A.1.3).  The row is read
// once into registers, reduced with cross-lane shuffles, and written once -- the
// register-cached variant App. A.1.3 describes.  The dense baseline runs the same kernel
// on full rows.
#include "dfss_device.hpp"
#include "dfss_kernels.hpp"

namespace dfss {

namespace {

constexpr int NT = 256;

// A team of TPR lanes owns one row; lane t holds the 16-byte chunks t, t+TPR, ... (NCH of them).
// F32: the row holds fp32 values (the 4-byte mode), else bfloat16.
template <int TPR, int NCH, bool F32>
__global__ __launch_bounds__(NT) void k_row_softmax(uint32_t *__restrict__ x, long rows, int cols) {
    constexpr int EPC = F32 ? 4 : 8;    // elements per 16-byte chunk
    const int tid = threadIdx.x;
    const long row = (long)blockIdx.x * (NT / TPR) + tid / TPR;
    const int t = tid % TPR;
    const int chunks = cols / EPC;
    const bool live = row < rows;
    u32x4 *p = reinterpret_cast<u32x4 *>(x) + (live ? row : 0) * (long)chunks;

    float v[NCH][EPC];
    float m = -INFINITY;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int c = t + i * TPR;
        if (live && c < chunks) {
            const u32x4 u = p[c];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if constexpr (F32) {
                    v[i][e] = __uint_as_float(u[e]);   // (by value: a bit cast applied to the element lvalue itself reads element 0)
                } else {
                    v[i][2 * e] = bf16_lo_to_f32(u[e]);
                    v[i][2 * e + 1] = bf16_hi_to_f32(u[e]);
                }
            }
        } else {
#pragma unroll
            for (int e = 0; e < EPC; ++e) v[i][e] = -INFINITY;
        }
#pragma unroll
        for (int e = 0; e < EPC; ++e) m = fmaxf(m, v[i][e]);
    }
    m = wave_xor_max(m, TPR);
    if (!live) m = 0.f;

    constexpr float kLog2e = 1.4426950408889634f;
    const float mb = m * kLog2e;
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NCH; ++i)
#pragma unroll
        for (int e = 0; e < EPC; ++e) {
            v[i][e] = __builtin_amdgcn_exp2f(v[i][e] * kLog2e - mb);  // exp(x - max); padding lanes give exp2(-inf) = 0
            s += v[i][e];
        }
    s = wave_xor_sum(s, TPR);
    const float inv = 1.0f / s;

#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int c = t + i * TPR;
        if (live && c < chunks) {
            u32x4 u;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if constexpr (F32) u[e] = __float_as_uint(v[i][e] * inv);
                else u[e] = pack_bf16x2(v[i][2 * e] * inv, v[i][2 * e + 1] * inv);
            }
            p[c] = u;
        }
    }
}

template <int TPR, int NCH, bool F32>
hipError_t launch(void *x, long rows, int cols, hipStream_t st) {
    const int rpw = NT / TPR;
    const unsigned grid = (unsigned)((rows + rpw - 1) / rpw);
    hipLaunchKernelGGL((k_row_softmax<TPR, NCH, F32>), dim3(grid), dim3(NT), 0, st, (uint32_t *)x, rows, cols);
    return hipGetLastError();
}

template <bool F32>
hipError_t dispatch(void *x, long rows, int cols, hipStream_t st) {
    const int chunks = cols / (F32 ? 4 : 8);
    if (chunks <= 8) return launch<8, 1, F32>(x, rows, cols, st);
    if (chunks <= 16) return launch<16, 1, F32>(x, rows, cols, st);
    if (chunks <= 32) return launch<32, 1, F32>(x, rows, cols, st);
    if (chunks <= 64) return launch<64, 1, F32>(x, rows, cols, st);
    if (chunks <= 128) return launch<64, 2, F32>(x, rows, cols, st);
    if (chunks <= 256) return launch<64, 4, F32>(x, rows, cols, st);
    if (chunks <= 512) return launch<64, 8, F32>(x, rows, cols, st);
    if (chunks <= 1024) return launch<64, 16, F32>(x, rows, cols, st);
    if constexpr (F32)
        if (chunks <= 2048) return launch<64, 32, F32>(x, rows, cols, st);
    return hipErrorInvalidValue;  // rows longer than 8192 elements: rejected by the caller
}

}  // namespace

hipError_t launch_row_softmax(void *x, long rows, int cols, hipStream_t st) {
    return dispatch<false>(x, rows, cols, st);
}
hipError_t launch_row_softmax_f32(void *x, long rows, int cols, hipStream_t st) {
    return dispatch<true>(x, rows, cols, st);
}

}  // namespace dfss
