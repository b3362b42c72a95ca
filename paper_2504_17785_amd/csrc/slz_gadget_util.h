// Host helpers shared by the gadget sources: workspace rounding, the launch shape of the element-wise kernels on
// ciphertext vectors, and the chunked table lookup (programmable bootstrapping + keyswitch).
#ifndef SLZ_GADGET_UTIL_H
#define SLZ_GADGET_UTIL_H
#include "slz_internal.h"

#define MR_THREADS 256

static inline size_t up256(size_t x) { return (x + 255) / 256 * 256; }

static inline dim3 ew_grid(size_t total) {
    size_t blocks = (total + MR_THREADS - 1) / MR_THREADS;
    return dim3((unsigned)(blocks < 65536 ? (blocks ? blocks : 1) : 65536));
}

// one table lookup per ciphertext (table idx[c], or table 0 without idx), in chunks the context can hold;
// in/out: count x n1 words under the small key, big: room for one chunk of bootstrapping outputs
static inline int lookup_n(slz_ctx *ctx, size_t chunk, size_t n1, const uint64_t *in, const uint64_t *luts, const uint32_t *idx,
                           uint32_t n_luts, const void *bskp, const uint64_t *ksk, uint64_t *big, uint64_t *out, size_t count, void *stream) {
    for (size_t c0 = 0; c0 < count; c0 += chunk) {
        const uint32_t nb = (uint32_t)(count - c0 < chunk ? count - c0 : chunk);
        int rc = slz_pbs_batch(ctx, in + c0 * n1, luts, idx ? idx + c0 : nullptr, n_luts, bskp, big, nb, stream);
        if (rc != SLZ_OK) return rc;
        rc = slz_keyswitch_batch(ctx, big, ksk, out + c0 * n1, nb, stream);
        if (rc != SLZ_OK) return rc;
    }
    return SLZ_OK;
}
#endif
