// Device-side helpers shared by the HIP kernels of the DFSS library (gfx950 only).
//
// Register layouts of the matrix instructions used here (wave64, lane l):
//   v_mfma_f32_16x16x32_bf16   A: row i = l%16, k = 8*(l/16)+e (e = 0..7)
//                              B: col j = l%16, k = 8*(l/16)+e
//                              D: col j = l%16, rows i = 4*(l/16)+r (r = 0..3)
//   v_smfmac_f32_16x16x64_bf16 A (2:4 compressed, 8 kept values per lane): row i = l%16,
//                              kept value e belongs to dense k = 16*(l/16) + 4*(e/2) + idx_e,
//                              idx_e = bits [2e, 2e+1] of the low half of the index register
//                              B (16 values per lane): col j = l%16,
//                              k = 8*(l/16)+e for e < 8 and k = 32 + 8*(l/16)+(e-8) for e >= 8
//                              D: as the dense 16x16 instruction.
// Each lane therefore owns four consecutive output rows of one column.  The kernels put
// KEYS on the output rows, so that a whole run of four consecutive keys of one query
// sits in one lane and the N:M selection needs no cross-lane traffic.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dfss {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef short s16x16 __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;

// Two fp32 -> two bfloat16 (round to nearest even) packed in one dword, `lo` in bits 15:0.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    f32x2 v = {lo, hi};
    bf16x2 b = __builtin_convertvector(v, bf16x2);
    return __builtin_bit_cast(uint32_t, b);
}

__device__ __forceinline__ float bf16_lo_to_f32(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi_to_f32(uint32_t w) { return __builtin_bit_cast(float, w & 0xFFFF0000u); }

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// Transposing LDS read: within each group of 16 lanes, lane s supplies the address of
// four consecutive 16-bit elements; lane t receives element t%4 of source lanes
// t/4, 4 + t/4, 8 + t/4, 12 + t/4.
__device__ __forceinline__ s16x4 lds_read_tr16(const void *p) {
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)p);
}

// Asynchronous 16-byte-per-lane copy global -> LDS (no register round trip): lane i of the
// wave reads 16 bytes at gbase + lane_off and writes LDS bytes [lds_wave_addr + 16 i, +16).
// `gbase` and `lds_wave_addr` are wave-uniform (scalar registers); `lane_off` is the per-lane
// byte offset.  Completion is tracked by the vector-memory counter: the caller waits with
// s_waitcnt vmcnt(..) and a workgroup barrier before other waves read the data.  Written as
// inline assembly so that the compiler does not serialise later LDS reads of OTHER buffers
// against copies that are still in flight, and so that no vector ALU work is spent on addresses.
// A global address known to be the same in every lane, moved into scalar registers once (so that
// address arithmetic derived from it stays on the scalar unit).
__device__ __forceinline__ uint64_t uniform_address(const void *p) {
    const uint64_t g = (uint64_t)(uintptr_t)p;
    // (readfirstlane returns a signed int: widen through uint32_t, or the low half sign-extends)
    const uint32_t g_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(g >> 32));
    const uint32_t g_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)g);
    return ((uint64_t)g_hi << 32) | (uint64_t)g_lo;
}
__device__ __forceinline__ void async_copy16(uint64_t uniform_base, uint32_t lane_off, uint32_t lds_wave_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_wave_addr), "v"(lane_off), "s"(uniform_base)
                 : "memory", "m0");
}
__device__ __forceinline__ void async_copy16(const void *gbase, uint32_t lane_off, uint32_t lds_wave_addr) {
    async_copy16(uniform_address(gbase), lane_off, lds_wave_addr);
}
// LDS byte address of a __shared__ object, as a wave-uniform scalar.
__device__ __forceinline__ uint32_t lds_address(const void *shared_ptr) {
    typedef __attribute__((address_space(3))) const void lds_cvoid;
    return __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_cvoid *)shared_ptr);
}
__device__ __forceinline__ void wait_async_copies() { __builtin_amdgcn_s_waitcnt(0x0F70); /* vmcnt(0) */ }
// Wait until at most YOUNGER vector-memory operations of this wave are outstanding.  The counter
// retires in issue order, so this waits for the copies while leaving the YOUNGER stores that were
// issued after them in flight (waiting for those would expose the full store latency every block).
template <int YOUNGER>
__device__ __forceinline__ void wait_async_copies_keep() {
    static_assert(YOUNGER >= 0 && YOUNGER < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (YOUNGER & 15) | ((YOUNGER >> 4) << 14));
}

// XOR pattern for the 16-byte chunks of row `row` of a tile that is read with the transposing 8-byte LDS read
// (lane (li, g): row = row0(g) + li / 4, chunk 2 x + (li / 2) % 2, half li % 2, where row0 differs between the lane
// groups g by a multiple of 8): the 32 lanes served together (two groups) then fall into 32 different pairs of banks.
// Bits used: row bit 1 (bit 0 alternates the bank halves of 128-byte rows by itself), and bit 3 ^ bit 4 -- whichever
// of the two tells the lane groups of one instruction apart (row0 = 8 g for the sparse product, 16 g + 8 m for the
// dense one).
template <int CPR>
__device__ __forceinline__ int tr_row_swizzle(int row) {
    static_assert(CPR == 8 || CPR == 16, "rows of 128 or 256 bytes");
    const int g = ((row >> 3) ^ (row >> 4)) & 1;
    return CPR == 8 ? (((row >> 1) & 1) << 1) | (g << 2) : ((row & 3) << 1) | (g << 3);
}

// Orders this wave's own LDS traffic: writes issued before the call are visible to reads of any
// lane of the same wave issued after it.  The hardware executes a wave's LDS operations in order;
// the fences (wavefront scope, no instructions) only keep the compiler from moving them across.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// product + c in two roundings, whatever the compiler's contraction rules: the (already rounded) product passes through
// an empty assembly statement, so that it cannot be folded into a fused multiply-add with the addition (a plain
// addition -- also __fadd_rn -- was seen fused in one instantiation and not in another).  The bias and mask additions
// are specified with two roundings (they must give the oracle's kept values and positions bit for bit).
__device__ __forceinline__ float add_unfused(float product, float c) {
    asm("" : "+v"(product));
    return product + c;
}

// N:M selection on the fp32 accumulators (arXiv 2203.00091, Sec. 2.3, App. A.1.1).  The comparisons of
// a run of four scores are taken as 64-bit lane masks (one bit per lane of the wave) so that the
// boolean logic runs on the scalar unit, off the vector ALU that the MFMA epilogue is short of; the
// vector unit only does the compares, min/max and the final selects.
typedef uint64_t lanemask;
__device__ __forceinline__ lanemask gt(float a, float b) { return __builtin_amdgcn_fcmpf(a, b, 2 /* ordered > */); }
__device__ __forceinline__ bool lane_bit(lanemask m) { return __builtin_amdgcn_inverse_ballot_w64(m); }

// Two largest of four scores, equal scores: the lower index wins (the order "larger value
// first, then lower index" is total, so the result is the one of the rank rule
// rank(t) = #{u: s_u > s_t} + #{u < t: s_u == s_t}, keep iff rank < 2).
// Evaluated as a tournament: A = {s0, s1}, B = {s2, s3}.  Both survivors come from A iff the
// weaker of A still outranks the stronger of B (ties favour A, the lower indices); both come
// from B iff the weaker of B strictly beats the stronger of A; otherwise each pair sends its
// stronger element.  Four comparisons land in lane masks, four min/max and eight selects on
// the vector unit, almost nothing on the scalar unit.
// Returns the kept values in key order and the position code (p_lo | p_hi << 2) << SHIFT.
__device__ __forceinline__ void select_2of4(float s0, float s1, float s2, float s3, const int SHIFT, float &lo,
                                            float &hi, uint32_t &code) {
    const lanemask c01 = gt(s1, s0), c23 = gt(s3, s2);      // stronger element of each pair is the later one
    const float amax = fmaxf(s0, s1), amin = fminf(s0, s1);
    const float bmax = fmaxf(s2, s3), bmin = fminf(s2, s3);
    const lanemask not_a = gt(bmax, amin);                   // B's best strictly beats A's worst
    const lanemask both_b = gt(bmin, amax);                  // B's worst strictly beats A's best
    const bool na = lane_bit(not_a), bb = lane_bit(both_b);
    const float lo_m = bb ? s2 : amax, hi_m = na ? bmax : s1;
    lo = na ? lo_m : s0;
    hi = bb ? s3 : hi_m;
    // p_lo: 0 if both from A, 2 if both from B, else index of A's stronger element
    // p_hi: 1 if both from A, 3 if both from B, else index of B's stronger element
    const bool lo1 = lane_bit(not_a & c01), hi3 = lane_bit(both_b | c23);
    const uint32_t plo_m = lo1 ? (1u << SHIFT) : 0u;
    const uint32_t plo = bb ? (2u << SHIFT) : plo_m;
    const uint32_t phi_m = hi3 ? (12u << SHIFT) : (8u << SHIFT);
    const uint32_t phi = na ? phi_m : (4u << SHIFT);
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

// Workgroups are handed to the 8 XCDs round-robin by linear id; each XCD has its own L2.
// Give every XCD one contiguous range of work items so that the workgroups sharing one
// head's K meet in one L2.
__device__ __forceinline__ unsigned xcd_contiguous(unsigned id, unsigned total) {
    const unsigned per = total / 8;
    return id < per * 8 ? (id % 8) * per + id / 8 : id;
}

template <typename T>
__device__ __forceinline__ T wave_xor_max(T v, int width) {
    for (int o = width >> 1; o > 0; o >>= 1) {
        T u = __shfl_xor(v, o, kWave);
        v = v > u ? v : u;
    }
    return v;
}
template <typename T>
__device__ __forceinline__ T wave_xor_sum(T v, int width) {
    for (int o = width >> 1; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

}  // namespace dfss
