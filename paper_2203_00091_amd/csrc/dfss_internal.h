/*
 * dfss_internal.h -- symbols that libdfss.so exports for its own tests and measurements only.
 * Not part of the public interface (include/dfss.h); may change without notice.
 */
#ifndef DFSS_INTERNAL_H
#define DFSS_INTERNAL_H

#include "../../include/dfss.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Tilings of the one-kernel forward pass (bfloat16 data).  The public calls pick one from the shape
 * (DFSS_VARIANT_AUTO); the test hook below runs the one it is told to, so that every tiling is
 * checked against the oracle whatever the heuristics would choose. */
enum {
    DFSS_VARIANT_AUTO = 0,
    DFSS_VARIANT_Q16 = 1,    /* 16 queries per wave, 16x16x32 matrix instruction, 64-query workgroups   */
    DFSS_VARIANT_Q16X2 = 2,  /* two such query tiles per wave, 128-query workgroups (Lq % 128 == 0)     */
    DFSS_VARIANT_Q32W2 = 3,  /* 32 queries per wave, 32x32x16 matrix instruction, 2 waves              */
    DFSS_VARIANT_Q32W4 = 4,  /* ... 4 waves, 128-query workgroups (Lq % 128 == 0)                       */
    DFSS_VARIANT_Q32K2 = 5,  /* 32 queries per pair of waves that split the keys, 4 waves, 64 queries  */
    DFSS_VARIANT_LAST = 5
};

/* dfss_attention_bias (dense == 0) or dense_attention_fused_bias (dense != 0) on bfloat16 data with the
 * named tiling; key_bias may be NULL.  A tiling that does not fit the shape falls back to the automatic
 * choice.  Same validation and error behaviour as the public calls. */
dfss_status dfss_internal_attention_variant(const void *Q, const void *K, const void *V, const void *key_bias,
                                            const dfss_shape *s, float scale, void *O, int variant, int dense,
                                            void *stream);

#ifdef __cplusplus
}
#endif
#endif /* DFSS_INTERNAL_H */
