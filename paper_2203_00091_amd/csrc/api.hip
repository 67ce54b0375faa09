// C ABI of the DFSS library: argument validation and kernel sequencing.
// The public contract is documented in include/dfss.h.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include "../../include/dfss.h"
#include "dfss_internal.h"
#include "dfss_kernels.hpp"

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Dims {
    int BH, H, Lq, Lk, d, mode;
    bool f32;      // the 4-byte mode: fp32 data, 1:2 only, staged kernels only
    bool split;    // ... with products formed from bfloat16 pieces on the bf16 matrix pipe
    // The stage calls with unpadded lengths (check_shape_stage): Lq, Lk above are the lengths of the compressed arrays'
    // layout (Lq rounded up to a multiple of 64, Lk to one of 128) and these the lengths of Q, K, V, key_bias and O.
    // Everywhere else they equal Lq, Lk.
    int LqR = 0, LkR = 0;
    bool unpadded() const { return LqR != Lq || LkR != Lk; }
    size_t elem() const { return f32 ? 4 : 2; }
};

// Shape rules common to every entry point.  need_nm: also check N:M.
dfss_status check_shape(const dfss_shape *s, bool need_nm, Dims *out) {
    if (!s) return DFSS_ERR_NULL;
    if (s->B <= 0 || s->H <= 0 || s->Lq <= 0 || s->Lk <= 0 || s->d <= 0) return DFSS_ERR_SHAPE;
    const long long bh = (long long)s->B * s->H;
    if (bh > 65535) return DFSS_ERR_SHAPE;
    if (s->Lq % 64 != 0 || s->Lk % 128 != 0) return DFSS_ERR_SHAPE;
    if (s->Lk > 8192 || s->Lq > (1 << 20)) return DFSS_ERR_SHAPE;
    if (s->dtype != DFSS_BF16 && s->dtype != DFSS_F32 && s->dtype != DFSS_F32_BF16X3) return DFSS_ERR_UNSUPPORTED;
    const bool f32 = s->dtype != DFSS_BF16, split = s->dtype == DFSS_F32_BF16X3;
    if (s->d != 64 && s->d != 128) return DFSS_ERR_UNSUPPORTED;
    int mode = -1;
    if (need_nm) {
        if (s->N == 2 && s->M == 4 && !f32) mode = 0;   // 2:4 belongs to 2-byte data (Sec. 2.3)
        else if (s->N == 1 && s->M == 2) mode = 1;
        else return DFSS_ERR_UNSUPPORTED;
    }
    if (out) *out = Dims{(int)bh, s->H, s->Lq, s->Lk, s->d, mode, f32, split, s->Lq, s->Lk};
    return DFSS_OK;
}

// Shape rules of the calls that take unpadded lengths (one-kernel paths only): any Lq, Lk a multiple of 4.
dfss_status check_shape_ragged(const dfss_shape *s, bool need_nm, Dims *out) {
    if (!s) return DFSS_ERR_NULL;
    if (s->B <= 0 || s->H <= 0 || s->Lq <= 0 || s->Lk <= 0 || s->d <= 0) return DFSS_ERR_SHAPE;
    const long long bh = (long long)s->B * s->H;
    if (bh > 65535) return DFSS_ERR_SHAPE;
    if (s->Lk % 4 != 0) return DFSS_ERR_SHAPE;
    if (s->Lk > 8192 || s->Lq > (1 << 20)) return DFSS_ERR_SHAPE;
    if (s->dtype != DFSS_BF16 && s->dtype != DFSS_F32_BF16X3) return DFSS_ERR_UNSUPPORTED;
    const bool split = s->dtype == DFSS_F32_BF16X3;
    if (s->d != 64 && s->d != 128) return DFSS_ERR_UNSUPPORTED;
    int mode = -1;
    if (need_nm) {
        if (s->N == 2 && s->M == 4 && !split) mode = 0;
        else if (s->N == 1 && s->M == 2) mode = 1;
        else return DFSS_ERR_UNSUPPORTED;
    }
    *out = Dims{(int)bh, s->H, s->Lq, s->Lk, s->d, mode, split, split, s->Lq, s->Lk};
    return DFSS_OK;
}

// Shape rules of the stage calls (stage 1, 2, 3, the staged forward pass, the three-kernel dense baseline and the size
// functions): the tile multiples of check_shape, or -- 2-byte dtype -- the unpadded lengths of check_shape_ragged, for
// which the compressed arrays take the layout of the lengths rounded up to the tiles.
dfss_status check_shape_stage(const dfss_shape *s, bool need_nm, Dims *out) {
    const dfss_status tiles = check_shape(s, need_nm, out);
    if (tiles != DFSS_ERR_SHAPE || !s || s->dtype != DFSS_BF16) return tiles;
    if (s->Lq % 64 == 0 && s->Lk % 128 == 0) return tiles;   // (refused for another reason)
    Dims R;
    if (const dfss_status st = check_shape_ragged(s, need_nm, &R)) return st;
    R.Lq = (R.LqR + 63) / 64 * 64;
    R.Lk = (R.LkR + 127) / 128 * 128;
    *out = R;
    return DFSS_OK;
}

inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }
// scale must be finite and > 0.  Tested on the bit pattern: the library is built with finite-math
// flags, under which a floating-point comparison may not be relied on to reject NaN.
inline bool bad_scale(float x) {
    uint32_t u;
    memcpy(&u, &x, sizeof(u));
    const bool negative = (u >> 31) != 0, zero = (u & 0x7FFFFFFFu) == 0, inf_or_nan = (u & 0x7F800000u) == 0x7F800000u;
    return negative || zero || inf_or_nan;
}
inline dfss_status hip_status(hipError_t e) { return e == hipSuccess ? DFSS_OK : DFSS_ERR_HIP; }

// stage 1 and stage 3 of the 4-byte mode, by the way the products are formed
inline hipError_t sddmm_prune_f32(const Dims &D, const void *Q, const void *K, const float *bias, float scale,
                                  void *vals, void *meta, hipStream_t st) {
    return D.split ? dfss::launch_sddmm_prune_split(Q, K, bias, D.H, D.BH, D.Lq, D.Lk, D.d, scale, vals, meta, st)
                   : dfss::launch_sddmm_prune_f32(Q, K, bias, D.H, D.BH, D.Lq, D.Lk, D.d, scale, vals, meta, st);
}
inline hipError_t spmm_f32(const Dims &D, const void *vals, const void *meta, const void *V, void *O, hipStream_t st) {
    return D.split ? dfss::launch_spmm_split(vals, meta, V, D.BH, D.Lq, D.Lk, D.d, O, st)
                   : dfss::launch_spmm_f32(vals, meta, V, D.BH, D.Lq, D.Lk, D.d, O, st);
}

}  // namespace

extern "C" {

size_t dfss_vals_bytes(const dfss_shape *s) {
    Dims D;
    if (check_shape_stage(s, true, &D) != DFSS_OK) return 0;
    return (size_t)D.BH * D.Lq * (D.Lk / 2) * D.elem();
}

size_t dfss_meta_bytes(const dfss_shape *s) {
    Dims D;
    if (check_shape_stage(s, true, &D) != DFSS_OK) return 0;
    return (size_t)D.BH * D.Lq * (D.Lk / (D.f32 ? 8 : 16)) * 2;   // one code per 8 bytes of dense data
}

size_t dfss_workspace_bytes(const dfss_shape *s) {
    const size_t v = dfss_vals_bytes(s), m = dfss_meta_bytes(s);
    if (!v || !m) return 0;
    return align_up(v) + align_up(m);
}

size_t dense_workspace_bytes(const dfss_shape *s) {
    Dims D;
    if (check_shape_stage(s, false, &D) != DFSS_OK) return 0;
    return align_up((size_t)D.BH * D.Lq * D.Lk * D.elem());
}

// causal: query i sees keys 0 .. i + (Lk - Lq); needs Lk >= Lq and a 2-byte dtype
static dfss_status bad_causal(const Dims &D) {
    if (D.f32) return DFSS_ERR_UNSUPPORTED;
    return D.Lk >= D.Lq ? DFSS_OK : DFSS_ERR_SHAPE;
}

static dfss_status sddmm_prune(const void *Q, const void *K, const void *key_bias, const dfss_shape *s, float scale,
                               void *vals, void *meta, void *stream, bool causal) {
    Dims D;
    if (!Q || !K || !vals || !meta) return DFSS_ERR_NULL;
    if (dfss_status st = check_shape_stage(s, true, &D)) return st;
    if (bad_scale(scale)) return DFSS_ERR_UNSUPPORTED;
    if (misaligned(Q) || misaligned(K) || misaligned(vals) || misaligned(meta) || misaligned(key_bias))
        return DFSS_ERR_SHAPE;
    if (causal) {
        if (D.unpadded()) return DFSS_ERR_UNSUPPORTED;
        if (dfss_status st = bad_causal(D)) return st;
    }
    if (D.f32)
        return hip_status(sddmm_prune_f32(D, Q, K, (const float *)key_bias, scale, vals, meta, (hipStream_t)stream));
    return hip_status(dfss::launch_sddmm_prune(Q, K, (const float *)key_bias, D.H, causal, D.BH, D.Lq, D.Lk, D.LqR, D.LkR,
                                               D.d, D.mode, scale, vals, meta, (hipStream_t)stream));
}

dfss_status dfss_sddmm_prune_bias(const void *Q, const void *K, const void *key_bias, const dfss_shape *s,
                                  float scale, void *vals, void *meta, void *stream) {
    return sddmm_prune(Q, K, key_bias, s, scale, vals, meta, stream, false);
}

dfss_status dfss_sddmm_prune_causal(const void *Q, const void *K, const void *key_bias, const dfss_shape *s,
                                    float scale, void *vals, void *meta, void *stream) {
    return sddmm_prune(Q, K, key_bias, s, scale, vals, meta, stream, true);
}

dfss_status dfss_sddmm_prune(const void *Q, const void *K, const dfss_shape *s, float scale, void *vals,
                             void *meta, void *stream) {
    return dfss_sddmm_prune_bias(Q, K, nullptr, s, scale, vals, meta, stream);
}

dfss_status dfss_sparse_softmax(void *vals, const dfss_shape *s, void *stream) {
    Dims D;
    if (!vals) return DFSS_ERR_NULL;
    if (dfss_status st = check_shape_stage(s, true, &D)) return st;
    if (misaligned(vals)) return DFSS_ERR_SHAPE;
    if (D.f32) return hip_status(dfss::launch_row_softmax_f32(vals, (long)D.BH * D.Lq, D.Lk / 2, (hipStream_t)stream));
    return hip_status(dfss::launch_row_softmax(vals, (long)D.BH * D.Lq, D.Lk / 2, (hipStream_t)stream));
}

dfss_status dfss_spmm(const void *vals, const void *meta, const void *V, const dfss_shape *s, void *O,
                      void *stream) {
    Dims D;
    if (!vals || !meta || !V || !O) return DFSS_ERR_NULL;
    if (dfss_status st = check_shape_stage(s, true, &D)) return st;
    if (misaligned(vals) || misaligned(meta) || misaligned(V) || misaligned(O)) return DFSS_ERR_SHAPE;
    if (D.f32) return hip_status(spmm_f32(D, vals, meta, V, O, (hipStream_t)stream));
    return hip_status(dfss::launch_spmm(vals, meta, V, D.BH, D.Lq, D.Lk, D.LqR, D.LkR, D.d, O, (hipStream_t)stream));
}

// The whole forward pass.  staged: the three stage kernels through the workspace; otherwise one kernel
// (the exact-product float mode has no one-kernel path and always takes the stages).
static dfss_status attention_forward(const void *Q, const void *K, const void *V, const void *key_bias,
                                     const dfss_shape *s, float scale, void *O, void *ws, size_t ws_bytes, void *stream,
                                     bool staged, int variant, bool causal = false) {
    Dims D;
    if (!Q || !K || !V || !O) return DFSS_ERR_NULL;
    // (unpadded lengths: the staged calls only; the one-kernel calls for them are the *_ragged ones)
    if (dfss_status st = staged ? check_shape_stage(s, true, &D) : check_shape(s, true, &D)) return st;
    if (bad_scale(scale)) return DFSS_ERR_UNSUPPORTED;
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O) || misaligned(key_bias))
        return DFSS_ERR_SHAPE;
    if (causal) {
        if (D.unpadded()) return DFSS_ERR_UNSUPPORTED;
        if (dfss_status cs = bad_causal(D)) return cs;
    }
    if (D.f32 && !D.split) staged = true;   // (fp32 matrix instructions: the stage kernels only)
    hipStream_t st = (hipStream_t)stream;
    const float *bias = (const float *)key_bias;
    if (!staged) {   // the workspace is not touched (and may be NULL)
        if (D.f32)
            return hip_status(dfss::launch_fused_attention_split(Q, K, V, bias, D.H, nullptr, D.BH, D.Lq, D.Lk, D.d, true,
                                                                 scale, O, st));
        return hip_status(dfss::launch_fused_attention(Q, K, V, bias, D.H, nullptr, causal, D.BH, D.Lq, D.Lk, D.d, D.mode,
                                                       scale, O, variant, st));
    }
    if (!ws) return DFSS_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(ws) & (kAlign - 1)) != 0) return DFSS_ERR_SHAPE;
    if (ws_bytes < dfss_workspace_bytes(s)) return DFSS_ERR_WORKSPACE;
    char *vals = static_cast<char *>(ws);
    char *meta = vals + align_up(dfss_vals_bytes(s));
    if (D.f32) {
        hipError_t e = sddmm_prune_f32(D, Q, K, bias, scale, vals, meta, st);
        if (e == hipSuccess) e = dfss::launch_row_softmax_f32(vals, (long)D.BH * D.Lq, D.Lk / 2, st);
        if (e == hipSuccess) e = spmm_f32(D, vals, meta, V, O, st);
        return hip_status(e);
    }
    // two kernels: the kept scores go to the workspace once and the product applies the softmax as it reads them
    hipError_t e =
        dfss::launch_sddmm_prune(Q, K, bias, D.H, causal, D.BH, D.Lq, D.Lk, D.LqR, D.LkR, D.d, D.mode, scale, vals, meta, st);
    if (e == hipSuccess) e = dfss::launch_softmax_spmm(vals, meta, V, D.BH, D.Lq, D.Lk, D.LqR, D.LkR, D.d, O, st);
    return hip_status(e);
}

dfss_status dfss_attention_bias(const void *Q, const void *K, const void *V, const void *key_bias,
                                const dfss_shape *s, float scale, void *O, void *ws, size_t ws_bytes, void *stream) {
    return attention_forward(Q, K, V, key_bias, s, scale, O, ws, ws_bytes, stream, false, 0);
}

dfss_status dfss_attention(const void *Q, const void *K, const void *V, const dfss_shape *s, float scale, void *O,
                           void *ws, size_t ws_bytes, void *stream) {
    return attention_forward(Q, K, V, nullptr, s, scale, O, ws, ws_bytes, stream, false, 0);
}

dfss_status dfss_attention_staged_bias(const void *Q, const void *K, const void *V, const void *key_bias,
                                       const dfss_shape *s, float scale, void *O, void *ws, size_t ws_bytes,
                                       void *stream) {
    return attention_forward(Q, K, V, key_bias, s, scale, O, ws, ws_bytes, stream, true, 0);
}

dfss_status dfss_attention_staged(const void *Q, const void *K, const void *V, const dfss_shape *s, float scale,
                                  void *O, void *ws, size_t ws_bytes, void *stream) {
    return attention_forward(Q, K, V, nullptr, s, scale, O, ws, ws_bytes, stream, true, 0);
}

dfss_status dfss_attention_causal(const void *Q, const void *K, const void *V, const void *key_bias,
                                  const dfss_shape *s, float scale, void *O, void *stream) {
    return attention_forward(Q, K, V, key_bias, s, scale, O, nullptr, 0, stream, false, 0, true);
}

dfss_status dfss_attention_staged_causal(const void *Q, const void *K, const void *V, const void *key_bias,
                                         const dfss_shape *s, float scale, void *O, void *ws, size_t ws_bytes,
                                         void *stream) {
    return attention_forward(Q, K, V, key_bias, s, scale, O, ws, ws_bytes, stream, true, 0, true);
}

// ---- the staged forward pass for callers that cannot allocate ------------------------------------
// Scratch of the variant below: vals, then meta, as in a caller's workspace.  One array per GPU for the
// lifetime of the process; host code reaches it only through the address looked up per device.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU (null = not looked up yet)

// Device address of the current device's copy of `scratch` (looked up once per device).
static dfss_status static_scratch_address(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return DFSS_ERR_HIP;
    void *p = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return DFSS_ERR_HIP;
        __atomic_store_n(&g_scratch_ptr[dev], p, __ATOMIC_RELEASE);   // (racing first calls store the same address)
    }
    *out = p;
    return DFSS_OK;
}

size_t dfss_static_scratch_bytes(void) { return kStaticScratchBytes; }

dfss_status dfss_attention_staged_static(const void *Q, const void *K, const void *V, const void *key_bias,
                                         const dfss_shape *s, float scale, void *O, void *stream) {
    // validate first (the size check needs a valid shape), then fetch the scratch address
    Dims D;
    if (!Q || !K || !V || !O) return DFSS_ERR_NULL;
    if (dfss_status st = check_shape(s, true, &D)) return st;
    const size_t need = dfss_workspace_bytes(s);
    if (need == 0 || need > kStaticScratchBytes) return DFSS_ERR_WORKSPACE;
    void *ws = nullptr;
    if (dfss_status st = static_scratch_address(&ws)) return st;
    return attention_forward(Q, K, V, key_bias, s, scale, O, ws, kStaticScratchBytes, stream, true, 0);
}

// Test hook (csrc/dfss_internal.h): the one-kernel path with the tiling named by the caller.
dfss_status dfss_internal_attention_variant(const void *Q, const void *K, const void *V, const void *key_bias,
                                            const dfss_shape *s, float scale, void *O, int variant, int dense,
                                            void *stream) {
    if (variant < 0 || variant > DFSS_VARIANT_LAST) return DFSS_ERR_UNSUPPORTED;
    if (!dense) return attention_forward(Q, K, V, key_bias, s, scale, O, nullptr, 0, stream, false, variant);
    Dims D;
    if (!Q || !K || !V || !O) return DFSS_ERR_NULL;
    if (dfss_status st = check_shape(s, false, &D)) return st;
    if (bad_scale(scale)) return DFSS_ERR_UNSUPPORTED;
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O) || misaligned(key_bias)) return DFSS_ERR_SHAPE;
    if (D.f32) return DFSS_ERR_UNSUPPORTED;
    return hip_status(dfss::launch_fused_attention(Q, K, V, (const float *)key_bias, D.H, nullptr, 0, D.BH, D.Lq, D.Lk,
                                                   D.d, 2, scale, O, variant, (hipStream_t)stream));
}

static dfss_status dense_fused(const void *Q, const void *K, const void *V, const void *key_bias, const dfss_shape *s,
                               float scale, void *O, void *stream, bool causal) {
    Dims D;
    if (!Q || !K || !V || !O) return DFSS_ERR_NULL;
    if (dfss_status st = check_shape(s, false, &D)) return st;
    if (bad_scale(scale)) return DFSS_ERR_UNSUPPORTED;
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O) || misaligned(key_bias))
        return DFSS_ERR_SHAPE;
    if (causal)
        if (dfss_status st = bad_causal(D)) return st;
    if (D.f32) {
        if (!D.split) return DFSS_ERR_UNSUPPORTED;
        return hip_status(dfss::launch_fused_attention_split(Q, K, V, (const float *)key_bias, D.H, nullptr, D.BH, D.Lq,
                                                             D.Lk, D.d, false, scale, O, (hipStream_t)stream));
    }
    return hip_status(dfss::launch_fused_attention(Q, K, V, (const float *)key_bias, D.H, nullptr, causal, D.BH, D.Lq,
                                                   D.Lk, D.d, 2, scale, O, 0, (hipStream_t)stream));
}

dfss_status dense_attention_fused_bias(const void *Q, const void *K, const void *V, const void *key_bias,
                                       const dfss_shape *s, float scale, void *O, void *stream) {
    return dense_fused(Q, K, V, key_bias, s, scale, O, stream, false);
}

dfss_status dense_attention_fused_causal(const void *Q, const void *K, const void *V, const void *key_bias,
                                         const dfss_shape *s, float scale, void *O, void *stream) {
    return dense_fused(Q, K, V, key_bias, s, scale, O, stream, true);
}

dfss_status dense_attention_fused(const void *Q, const void *K, const void *V, const dfss_shape *s, float scale,
                                  void *O, void *stream) {
    return dense_attention_fused_bias(Q, K, V, nullptr, s, scale, O, stream);
}

static dfss_status dense_staged(const void *Q, const void *K, const void *V, const void *key_bias, const dfss_shape *s,
                                float scale, void *O, void *ws, size_t ws_bytes, void *stream, bool causal) {
    Dims D;
    if (!Q || !K || !V || !O || !ws) return DFSS_ERR_NULL;
    if (dfss_status st = check_shape_stage(s, false, &D)) return st;
    if (bad_scale(scale)) return DFSS_ERR_UNSUPPORTED;
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O) || misaligned(key_bias))
        return DFSS_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(ws) & (kAlign - 1)) != 0) return DFSS_ERR_SHAPE;
    if (ws_bytes < dense_workspace_bytes(s)) return DFSS_ERR_WORKSPACE;
    if (causal) {
        if (D.unpadded()) return DFSS_ERR_UNSUPPORTED;
        if (dfss_status cs = bad_causal(D)) return cs;
    }
    hipStream_t st = (hipStream_t)stream;
    if (D.f32) {
        hipError_t e = D.split ? dfss::launch_dense_scores_split(Q, K, (const float *)key_bias, D.H, D.BH, D.Lq, D.Lk, D.d,
                                                                 scale, ws, st)
                               : dfss::launch_dense_scores_f32(Q, K, (const float *)key_bias, D.H, D.BH, D.Lq, D.Lk, D.d,
                                                               scale, ws, st);
        if (e == hipSuccess) e = dfss::launch_row_softmax_f32(ws, (long)D.BH * D.Lq, D.Lk, st);
        if (e == hipSuccess)
            e = D.split ? dfss::launch_dense_av_split(ws, V, D.BH, D.Lq, D.Lk, D.d, O, st)
                        : dfss::launch_dense_av_f32(ws, V, D.BH, D.Lq, D.Lk, D.d, O, st);
        return hip_status(e);
    }
    hipError_t e =
        dfss::launch_dense_scores(Q, K, (const float *)key_bias, D.H, causal, D.BH, D.Lq, D.Lk, D.LqR, D.LkR, D.d, scale, ws, st);
    if (e == hipSuccess) e = dfss::launch_row_softmax(ws, (long)D.BH * D.Lq, D.Lk, st);
    if (e == hipSuccess) e = dfss::launch_dense_av(ws, V, D.BH, D.Lq, D.Lk, D.LqR, D.LkR, D.d, O, st);
    return hip_status(e);
}

dfss_status dense_attention_bias(const void *Q, const void *K, const void *V, const void *key_bias,
                                 const dfss_shape *s, float scale, void *O, void *ws, size_t ws_bytes, void *stream) {
    return dense_staged(Q, K, V, key_bias, s, scale, O, ws, ws_bytes, stream, false);
}

dfss_status dense_attention_causal(const void *Q, const void *K, const void *V, const void *key_bias,
                                   const dfss_shape *s, float scale, void *O, void *ws, size_t ws_bytes, void *stream) {
    return dense_staged(Q, K, V, key_bias, s, scale, O, ws, ws_bytes, stream, true);
}

dfss_status dense_attention(const void *Q, const void *K, const void *V, const dfss_shape *s, float scale, void *O,
                            void *ws, size_t ws_bytes, void *stream) {
    return dense_attention_bias(Q, K, V, nullptr, s, scale, O, ws, ws_bytes, stream);
}

// mode: the N:M of the shape, or dense (N, M ignored)
static dfss_status attention_blocked(const void *Q, const void *K, const void *V, const void *key_bias,
                                     const void *block_mask, const dfss_shape *s, bool dense, float scale, void *O,
                                     void *stream) {
    Dims D;
    if (!Q || !K || !V || !O || !block_mask) return DFSS_ERR_NULL;
    if (dfss_status st = check_shape(s, !dense, &D)) return st;
    if (bad_scale(scale)) return DFSS_ERR_UNSUPPORTED;
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O) || misaligned(key_bias))
        return DFSS_ERR_SHAPE;
    if (D.f32) {
        if (!D.split) return DFSS_ERR_UNSUPPORTED;
        return hip_status(dfss::launch_fused_attention_split(Q, K, V, (const float *)key_bias, D.H,
                                                             (const uint8_t *)block_mask, D.BH, D.Lq, D.Lk, D.d, !dense,
                                                             scale, O, (hipStream_t)stream));
    }
    return hip_status(dfss::launch_fused_attention(Q, K, V, (const float *)key_bias, D.H, (const uint8_t *)block_mask,
                                                   0, D.BH, D.Lq, D.Lk, D.d, dense ? 2 : D.mode, scale, O, 0,
                                                   (hipStream_t)stream));
}

dfss_status dfss_attention_blocked(const void *Q, const void *K, const void *V, const void *key_bias,
                                   const void *block_mask, const dfss_shape *s, float scale, void *O, void *stream) {
    return attention_blocked(Q, K, V, key_bias, block_mask, s, false, scale, O, stream);
}

dfss_status dense_attention_fused_blocked(const void *Q, const void *K, const void *V, const void *key_bias,
                                          const void *block_mask, const dfss_shape *s, float scale, void *O,
                                          void *stream) {
    return attention_blocked(Q, K, V, key_bias, block_mask, s, true, scale, O, stream);
}

size_t dfss_blocked_split_workspace_bytes(const dfss_shape *s) {
    Dims D;
    if (check_shape(s, false, &D) != DFSS_OK || D.f32) return 0;
    return align_up(dfss::fused_attention_split_workspace_bytes(D.BH, D.Lq, D.d));
}

static dfss_status attention_blocked_split(const void *Q, const void *K, const void *V, const void *key_bias,
                                           const void *block_mask, const dfss_shape *s, bool dense, float scale, void *O,
                                           void *ws, size_t ws_bytes, void *stream) {
    Dims D;
    if (!Q || !K || !V || !O || !block_mask || !ws) return DFSS_ERR_NULL;
    if (dfss_status st = check_shape(s, !dense, &D)) return st;
    if (bad_scale(scale)) return DFSS_ERR_UNSUPPORTED;
    if (D.f32) return DFSS_ERR_UNSUPPORTED;
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O) || misaligned(key_bias) || misaligned(ws))
        return DFSS_ERR_SHAPE;
    if (ws_bytes < dfss_blocked_split_workspace_bytes(s)) return DFSS_ERR_WORKSPACE;
    return hip_status(dfss::launch_fused_attention_split_rows(Q, K, V, (const float *)key_bias, D.H,
                                                              (const uint8_t *)block_mask, D.BH, D.Lq, D.Lk, D.d,
                                                              dense ? 2 : D.mode, scale, O, ws, (hipStream_t)stream));
}

dfss_status dfss_attention_blocked_split(const void *Q, const void *K, const void *V, const void *key_bias,
                                         const void *block_mask, const dfss_shape *s, float scale, void *O, void *ws,
                                         size_t ws_bytes, void *stream) {
    return attention_blocked_split(Q, K, V, key_bias, block_mask, s, false, scale, O, ws, ws_bytes, stream);
}

dfss_status dense_attention_fused_blocked_split(const void *Q, const void *K, const void *V, const void *key_bias,
                                                const void *block_mask, const dfss_shape *s, float scale, void *O,
                                                void *ws, size_t ws_bytes, void *stream) {
    return attention_blocked_split(Q, K, V, key_bias, block_mask, s, true, scale, O, ws, ws_bytes, stream);
}

// ---- additive mask [Lq, Lk] shared by all heads (stage calls, 2-byte dtype) ----
// what: 0 = stage 1 only (out0 = vals, out1 = meta), 1 = the staged forward pass, 2 = the three-kernel dense baseline
static dfss_status with_mask(int what, const void *Q, const void *K, const void *V, const void *mask, const dfss_shape *s,
                             float scale, void *out0, void *out1, void *ws, size_t ws_bytes, void *stream) {
    Dims D;
    if (!Q || !K || !mask || !out0) return DFSS_ERR_NULL;
    if (what == 0 ? !out1 : (!V || !ws)) return DFSS_ERR_NULL;
    if (dfss_status st = check_shape_stage(s, what != 2, &D)) return st;
    if (bad_scale(scale)) return DFSS_ERR_UNSUPPORTED;
    if (D.f32) return DFSS_ERR_UNSUPPORTED;
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(mask) || misaligned(out0) || misaligned(out1))
        return DFSS_ERR_SHAPE;
    hipStream_t st = (hipStream_t)stream;
    const float *m = (const float *)mask;
    if (what == 0)
        return hip_status(dfss::launch_sddmm_prune_mask(Q, K, m, D.BH, D.Lq, D.Lk, D.LqR, D.LkR, D.d, D.mode, scale, out0,
                                                        out1, st));
    if ((reinterpret_cast<uintptr_t>(ws) & (kAlign - 1)) != 0) return DFSS_ERR_SHAPE;
    if (ws_bytes < (what == 1 ? dfss_workspace_bytes(s) : dense_workspace_bytes(s))) return DFSS_ERR_WORKSPACE;
    if (what == 1) {
        char *vals = static_cast<char *>(ws);
        char *meta = vals + align_up(dfss_vals_bytes(s));
        hipError_t e = dfss::launch_sddmm_prune_mask(Q, K, m, D.BH, D.Lq, D.Lk, D.LqR, D.LkR, D.d, D.mode, scale, vals, meta, st);
        if (e == hipSuccess) e = dfss::launch_softmax_spmm(vals, meta, V, D.BH, D.Lq, D.Lk, D.LqR, D.LkR, D.d, out0, st);
        return hip_status(e);
    }
    hipError_t e = dfss::launch_dense_scores_mask(Q, K, m, D.BH, D.Lq, D.Lk, D.LqR, D.LkR, D.d, scale, ws, st);
    if (e == hipSuccess) e = dfss::launch_row_softmax(ws, (long)D.BH * D.Lq, D.Lk, st);
    if (e == hipSuccess) e = dfss::launch_dense_av(ws, V, D.BH, D.Lq, D.Lk, D.LqR, D.LkR, D.d, out0, st);
    return hip_status(e);
}

dfss_status dfss_sddmm_prune_mask(const void *Q, const void *K, const void *mask, const dfss_shape *s, float scale,
                                  void *vals, void *meta, void *stream) {
    return with_mask(0, Q, K, nullptr, mask, s, scale, vals, meta, nullptr, 0, stream);
}

dfss_status dfss_attention_staged_mask(const void *Q, const void *K, const void *V, const void *mask,
                                       const dfss_shape *s, float scale, void *O, void *ws, size_t ws_bytes,
                                       void *stream) {
    return with_mask(1, Q, K, V, mask, s, scale, O, nullptr, ws, ws_bytes, stream);
}

dfss_status dense_attention_mask(const void *Q, const void *K, const void *V, const void *mask, const dfss_shape *s,
                                 float scale, void *O, void *ws, size_t ws_bytes, void *stream) {
    return with_mask(2, Q, K, V, mask, s, scale, O, nullptr, ws, ws_bytes, stream);
}

// One kernel, padded batch given by its key lengths.
dfss_status dfss_attention_varlen(const void *Q, const void *K, const void *V, const void *key_len, const dfss_shape *s,
                                  float scale, void *O, void *stream) {
    Dims D;
    if (!Q || !K || !V || !key_len || !O) return DFSS_ERR_NULL;
    if (dfss_status st = check_shape(s, true, &D)) return st;
    if (bad_scale(scale)) return DFSS_ERR_UNSUPPORTED;
    if (D.f32) return DFSS_ERR_UNSUPPORTED;
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O)) return DFSS_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(key_len) & 3u) != 0) return DFSS_ERR_SHAPE;
    return hip_status(dfss::launch_fused_attention_varlen(Q, K, V, (const int *)key_len, D.H, D.BH, D.Lq, D.Lk, D.d,
                                                          D.mode, scale, O, (hipStream_t)stream));
}

// One kernel, general mask; lengths as in the _ragged calls.  dense: full attention (N, M ignored)
static dfss_status attention_mask_fused(const void *Q, const void *K, const void *V, const void *mask,
                                        const dfss_shape *s, bool dense, float scale, void *O, void *stream) {
    Dims D;
    if (!Q || !K || !V || !mask || !O) return DFSS_ERR_NULL;
    if (dfss_status st = check_shape_ragged(s, !dense, &D)) return st;
    if (bad_scale(scale)) return DFSS_ERR_UNSUPPORTED;
    if (D.f32) return DFSS_ERR_UNSUPPORTED;
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O) || misaligned(mask)) return DFSS_ERR_SHAPE;
    return hip_status(dfss::launch_fused_attention_mask(Q, K, V, (const float *)mask, D.BH, D.Lq, D.Lk, D.d,
                                                        dense ? 2 : D.mode, scale, O, (hipStream_t)stream));
}

dfss_status dfss_attention_mask(const void *Q, const void *K, const void *V, const void *mask, const dfss_shape *s,
                                float scale, void *O, void *stream) {
    return attention_mask_fused(Q, K, V, mask, s, false, scale, O, stream);
}

dfss_status dense_attention_fused_mask(const void *Q, const void *K, const void *V, const void *mask,
                                       const dfss_shape *s, float scale, void *O, void *stream) {
    return attention_mask_fused(Q, K, V, mask, s, true, scale, O, stream);
}

// dense: full attention (N, M ignored)
static dfss_status attention_ragged(const void *Q, const void *K, const void *V, const void *key_bias,
                                    const dfss_shape *s, bool dense, float scale, void *O, void *stream) {
    Dims D;
    if (!Q || !K || !V || !O) return DFSS_ERR_NULL;
    if (dfss_status st = check_shape_ragged(s, !dense, &D)) return st;
    if (bad_scale(scale)) return DFSS_ERR_UNSUPPORTED;
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O) || misaligned(key_bias))
        return DFSS_ERR_SHAPE;
    if (D.split)
        return hip_status(dfss::launch_fused_attention_split(Q, K, V, (const float *)key_bias, D.H, nullptr, D.BH, D.Lq,
                                                             D.Lk, D.d, !dense, scale, O, (hipStream_t)stream));
    return hip_status(dfss::launch_fused_attention(Q, K, V, (const float *)key_bias, D.H, nullptr, 0, D.BH, D.Lq, D.Lk,
                                                   D.d, dense ? 2 : D.mode, scale, O, 0, (hipStream_t)stream));
}

dfss_status dfss_attention_ragged(const void *Q, const void *K, const void *V, const void *key_bias,
                                  const dfss_shape *s, float scale, void *O, void *stream) {
    return attention_ragged(Q, K, V, key_bias, s, false, scale, O, stream);
}

dfss_status dense_attention_fused_ragged(const void *Q, const void *K, const void *V, const void *key_bias,
                                         const dfss_shape *s, float scale, void *O, void *stream) {
    return attention_ragged(Q, K, V, key_bias, s, true, scale, O, stream);
}

dfss_status dfss_spmm_t(const void *vals, const void *meta, const void *X, const dfss_shape *s, void *out,
                        void *stream) {
    Dims D;
    if (!vals || !meta || !X || !out) return DFSS_ERR_NULL;
    if (dfss_status st = check_shape_stage(s, true, &D)) return st;
    if (misaligned(vals) || misaligned(meta) || misaligned(X) || misaligned(out)) return DFSS_ERR_SHAPE;
    if (D.f32) {
        if (!D.split) return DFSS_ERR_UNSUPPORTED;
        return hip_status(dfss::launch_spmm_t_split(vals, meta, X, D.BH, D.Lq, D.Lk, D.d, out, (hipStream_t)stream));
    }
    return hip_status(dfss::launch_spmm_t(vals, meta, X, D.BH, D.Lq, D.Lk, D.LqR, D.LkR, D.d, out, (hipStream_t)stream));
}

dfss_status dfss_attention_backward(const void *dO, const void *Q, const void *K, const void *V, const void *O,
                                    const void *P, const void *meta, const dfss_shape *s, float scale, void *dQ,
                                    void *dK, void *dV, void *ws, size_t ws_bytes, void *stream) {
    Dims D;
    if (!dO || !Q || !K || !V || !O || !P || !meta || !dQ || !dK || !dV || !ws) return DFSS_ERR_NULL;
    if (dfss_status st = check_shape_stage(s, true, &D)) return st;
    if (bad_scale(scale)) return DFSS_ERR_UNSUPPORTED;
    if (misaligned(dO) || misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O) || misaligned(P) ||
        misaligned(meta) || misaligned(dQ) || misaligned(dK) || misaligned(dV))
        return DFSS_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(ws) & (kAlign - 1)) != 0) return DFSS_ERR_SHAPE;
    if (D.f32 && !D.split) return DFSS_ERR_UNSUPPORTED;
    if (ws_bytes < align_up(dfss_vals_bytes(s))) return DFSS_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    void *dS = ws;   // scale * dS in the compressed layout of P
    if (D.f32) {
        hipError_t e = dfss::launch_masked_sddmm_ds_split(dO, V, O, P, meta, D.BH, D.Lq, D.Lk, D.d, scale, dS, st);
        if (e == hipSuccess) e = dfss::launch_spmm_split(dS, meta, K, D.BH, D.Lq, D.Lk, D.d, dQ, st);       // dQ = dS' K
        if (e == hipSuccess) e = dfss::launch_spmm_t_split(P, meta, dO, D.BH, D.Lq, D.Lk, D.d, dV, st);     // dV = P^T dO
        if (e == hipSuccess) e = dfss::launch_spmm_t_split(dS, meta, Q, D.BH, D.Lq, D.Lk, D.d, dK, st);     // dK = dS'^T Q
        return hip_status(e);
    }
    hipError_t e;
    if (D.d == 64) {   // dS' and dQ = dS' K in one pass over the compressed rows
        e = dfss::launch_masked_sddmm_ds(dO, V, O, P, meta, K, D.BH, D.Lq, D.Lk, D.LqR, D.LkR, D.d, scale, dS, dQ, st);
    } else {
        e = dfss::launch_masked_sddmm_ds(dO, V, O, P, meta, nullptr, D.BH, D.Lq, D.Lk, D.LqR, D.LkR, D.d, scale, dS,
                                         nullptr, st);
        if (e == hipSuccess) e = dfss::launch_spmm(dS, meta, K, D.BH, D.Lq, D.Lk, D.LqR, D.LkR, D.d, dQ, st);   // dQ = dS' K
    }
    if (e == hipSuccess) e = dfss::launch_spmm_t(P, meta, dO, D.BH, D.Lq, D.Lk, D.LqR, D.LkR, D.d, dV, st);    // dV = P^T dO
    if (e == hipSuccess) e = dfss::launch_spmm_t(dS, meta, Q, D.BH, D.Lq, D.Lk, D.LqR, D.LkR, D.d, dK, st);    // dK = dS'^T Q
    return hip_status(e);
}

size_t dfss_backward_workspace_bytes(const dfss_shape *s) {
    if (s && s->dtype == DFSS_F32) return 0;     // the backward pass of the float mode takes split products only
    const size_t v = dfss_vals_bytes(s);
    return v ? align_up(v) : 0;
}

dfss_status dfss_meta_to_canonical(const void *meta, const dfss_shape *s, uint16_t *canon, void *stream) {
    Dims D;
    if (!meta || !canon) return DFSS_ERR_NULL;
    if (dfss_status st = check_shape_stage(s, true, &D)) return st;
    if (misaligned(meta) || misaligned(canon)) return DFSS_ERR_SHAPE;
    return hip_status(dfss::launch_meta_reorder(meta, canon, D.BH, D.Lq, D.Lk / (D.f32 ? 16 : 32), true, !D.f32,
                                                (hipStream_t)stream));
}

dfss_status dfss_meta_from_canonical(const uint16_t *canon, const dfss_shape *s, void *meta, void *stream) {
    Dims D;
    if (!meta || !canon) return DFSS_ERR_NULL;
    if (dfss_status st = check_shape_stage(s, true, &D)) return st;
    if (misaligned(meta) || misaligned(canon)) return DFSS_ERR_SHAPE;
    return hip_status(dfss::launch_meta_reorder(canon, meta, D.BH, D.Lq, D.Lk / (D.f32 ? 16 : 32), false, !D.f32,
                                                (hipStream_t)stream));
}

const char *dfss_status_string(dfss_status st) {
    switch (st) {
        case DFSS_OK: return "ok";
        case DFSS_ERR_NULL: return "null pointer";
        case DFSS_ERR_SHAPE: return "invalid shape or alignment";
        case DFSS_ERR_UNSUPPORTED: return "unsupported N:M, dtype, head size or scale";
        case DFSS_ERR_WORKSPACE: return "workspace too small";
        case DFSS_ERR_HIP: return "HIP launch failed";
    }
    return "unknown status";
}

}  // extern "C"
