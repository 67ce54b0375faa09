// Metadata word order (arXiv 2203.00091, Sec. 2.3 and App. A.1.1-A.1.2 define the 4-bit
// codes and their packing into 16-bit words; the ORDER of the words in memory is free).
// Canonical: uint16 [BH, Lq, Lk/16], taken here as 32-bit words [BH, Lq, W], W = Lk/32 (two
// consecutive 16-bit words, the earlier one in the low half).  Library: [BH, Lq/16, Lk/128, 16, 4]:
// per block of 128 keys the four words of a row are adjacent (in the order c = 0, 2, 1, 3 of
// their 32-key chunks) and the 16 rows of a row block follow each other.  That is the order in
// which the pruning epilogue holds them (a lane owns the chunks c and c + 2 of one row and
// writes them with one 8-byte store) and in which the SpMM reads them.
// The 4-byte mode (one code per kept float, uint16 [BH, Lq, Lk/8] = 32-bit words [BH, Lq, W], W = Lk/16)
// uses the same blocking with 64-key blocks and no permutation inside a row's four words:
// [BH, Lq/16, Lk/64, 16, 4] -- a wave of its score kernel writes the 256 bytes of 16 rows x 64 keys as
// whole lines instead of 16-byte pieces of 16 different rows.
#include "dfss_device.hpp"
#include "dfss_kernels.hpp"

namespace dfss {

namespace {

__global__ __launch_bounds__(256) void k_meta_reorder(const uint32_t *__restrict__ src, uint32_t *__restrict__ dst,
                                                      long total, int Lq, int W, bool to_canonical, bool permute) {
    const long i = (long)blockIdx.x * 256 + threadIdx.x;  // index in canonical order
    if (i >= total) return;
    const int w = (int)(i % W);
    const long r = i / W;  // bh * Lq + row
    const int row = (int)(r % Lq);
    const long bh = r / Lq;
    // word w = 4 jb + c of a row; 2-byte data: c = 2 p + h (p: 64-key pair, h: 32-key half) is stored at slot 2 h + p
    const int jb = w >> 2, c = w & 3, slot = permute ? ((c & 1) << 1) | (c >> 1) : c;
    const long lib = (((bh * (Lq / 16) + row / 16) * (W / 4) + jb) * 16 + row % 16) * 4 + slot;
    if (to_canonical) dst[i] = src[lib];
    else dst[lib] = src[i];
}

}  // namespace

hipError_t launch_meta_reorder(const void *src, void *dst, int BH, int Lq, int W, bool to_canonical, bool permute,
                               hipStream_t st) {
    const long total = (long)BH * Lq * W;
    const unsigned grid = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL(k_meta_reorder, dim3(grid), dim3(256), 0, st, (const uint32_t *)src, (uint32_t *)dst, total,
                       Lq, W, to_canonical, permute);
    return hipGetLastError();
}

}  // namespace dfss
