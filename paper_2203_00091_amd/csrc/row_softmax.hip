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
template <int TPR, int NCH>
__global__ __launch_bounds__(NT) void k_row_softmax(uint32_t *__restrict__ x, long rows, int cols) {
    const int tid = threadIdx.x;
    const long row = (long)blockIdx.x * (NT / TPR) + tid / TPR;
    const int t = tid % TPR;
    const int chunks = cols / 8;
    const bool live = row < rows;
    u32x4 *p = reinterpret_cast<u32x4 *>(x) + (live ? row : 0) * (long)chunks;

    float v[NCH][8];
    float m = -INFINITY;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int c = t + i * TPR;
        if (live && c < chunks) {
            const u32x4 u = p[c];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                v[i][2 * e] = bf16_lo_to_f32(u[e]);
                v[i][2 * e + 1] = bf16_hi_to_f32(u[e]);
            }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[i][e] = -INFINITY;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) m = fmaxf(m, v[i][e]);
    }
    m = wave_xor_max(m, TPR);
    if (!live) m = 0.f;

    constexpr float kLog2e = 1.4426950408889634f;
    const float mb = m * kLog2e;
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NCH; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            v[i][e] = exp2f(v[i][e] * kLog2e - mb);  // exp(x - max); padding lanes give exp2(-inf) = 0
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
            for (int e = 0; e < 4; ++e) u[e] = pack_bf16x2(v[i][2 * e] * inv, v[i][2 * e + 1] * inv);
            p[c] = u;
        }
    }
}

template <int TPR, int NCH>
hipError_t launch(void *x, long rows, int cols, hipStream_t st) {
    const int rpw = NT / TPR;
    const unsigned grid = (unsigned)((rows + rpw - 1) / rpw);
    hipLaunchKernelGGL((k_row_softmax<TPR, NCH>), dim3(grid), dim3(NT), 0, st, (uint32_t *)x, rows, cols);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_row_softmax(void *x, long rows, int cols, hipStream_t st) {
    const int chunks = cols / 8;
    if (chunks <= 8) return launch<8, 1>(x, rows, cols, st);
    if (chunks <= 16) return launch<16, 1>(x, rows, cols, st);
    if (chunks <= 32) return launch<32, 1>(x, rows, cols, st);
    if (chunks <= 64) return launch<64, 1>(x, rows, cols, st);
    if (chunks <= 128) return launch<64, 2>(x, rows, cols, st);
    if (chunks <= 256) return launch<64, 4>(x, rows, cols, st);
    if (chunks <= 512) return launch<64, 8>(x, rows, cols, st);
    if (chunks <= 1024) return launch<64, 16>(x, rows, cols, st);
    return hipErrorInvalidValue;  // rows longer than 8192 elements: rejected by the caller
}

}  // namespace dfss
