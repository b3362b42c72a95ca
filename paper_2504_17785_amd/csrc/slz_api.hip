// C-ABI entry points of libsilenzio_pbs: argument checks, path selection, scratch ownership.
#include "slz_internal.h"
#include <new>
#include <cstring>

static bool is_pow2(uint32_t v) { return v && !(v & (v - 1)); }

static int check_params(const slz_params *p) {
    if (!p) return SLZ_E_INVALID_ARG;
    if (p->n == 0 || p->k == 0 || !is_pow2(p->N) || p->N < 2) return SLZ_E_INVALID_ARG;
    if (p->pbs_base_log == 0 || p->pbs_level == 0 || p->pbs_base_log * p->pbs_level > 64) return SLZ_E_INVALID_ARG;
    if (p->ks_base_log == 0 || p->ks_level == 0 || p->ks_base_log * p->ks_level > 64) return SLZ_E_INVALID_ARG;
    if (p->msg_bits == 0 || p->msg_bits > 62) return SLZ_E_INVALID_ARG;
    return SLZ_OK;
}

static bool misaligned(const void *p) { return ((uintptr_t)p & 15u) != 0; }
// ciphertext arrays: rows are n+1 (or kN+1) words, so only word alignment can hold for every row and every sub-batch
static bool misaligned8(const void *p) { return ((uintptr_t)p & 7u) != 0; }

// hipMalloc behind a counter that a test can arm: the SLZ_OPT_FAIL_ALLOC_AFTER-th scratch allocation from now fails (the way
// an exhausted device would) without touching the device.
static int g_fail_alloc_after = -1;
int slz_scratch_alloc(void **out, size_t bytes) {
    *out = nullptr;
    if (g_fail_alloc_after == 0) { g_fail_alloc_after = -1; return SLZ_E_NOMEM; }
    if (g_fail_alloc_after > 0) g_fail_alloc_after--;
    if (hipMalloc(out, bytes) != hipSuccess) { (void)hipGetLastError(); *out = nullptr; return SLZ_E_NOMEM; }
    return SLZ_OK;
}

extern "C" int slz_ctx_create(const slz_params *params, uint32_t max_batch, slz_ctx **out) {
    if (!out) return SLZ_E_INVALID_ARG;
    *out = nullptr;
    int rc = check_params(params);
    if (rc != SLZ_OK) return rc;
    if (max_batch == 0) return SLZ_E_INVALID_ARG;
    uint32_t logN = 0;
    while ((1u << logN) < params->N) logN++;
    if (logN > SLZ_MAX_LOGN) return SLZ_E_UNSUPPORTED;
    if (params->pbs_base_log > 30) return SLZ_E_UNSUPPORTED;
    // Exactness: the integer sum of (k+1) l N products digit * key word is below
    // (k+1) l N 2^(beta-1) 2^63; it must stay below p1 p2 / 4 (about 2^97.99) for the CRT lift.
    {
        long double bound = (long double)(params->k + 1) * params->pbs_level * params->N;
        bound *= (long double)(1ull << (params->pbs_base_log - 1));
        bound *= 9223372036854775808.0L;                          // 2^63
        long double M = (long double)SLZ_P1 * (long double)SLZ_P2;
        if (4.0L * bound > M) return SLZ_E_UNSUPPORTED;
    }
    slz_ctx *ctx = new (std::nothrow) slz_ctx;
    if (!ctx) return SLZ_E_NOMEM;
    std::memset(ctx, 0, sizeof(*ctx));
    ctx->prm = *params;
    ctx->max_batch = max_batch;
    ctx->logN = logN;
    if (hipGetDevice(&ctx->device) != hipSuccess) { delete ctx; return SLZ_E_HIP; }
    rc = slz_build_tables(ctx);
    // specialised paths are optional: a shape they decline (SLZ_E_UNSUPPORTED) runs on the generic path
    if (rc == SLZ_OK && slz_fused_supported(params)) {
        rc = slz_fused_init(ctx);
        ctx->has_fused = (rc == SLZ_OK);
        ctx->fused_pacing = 1;
        if (rc == SLZ_E_UNSUPPORTED) rc = SLZ_OK;
    }
    if (rc == SLZ_OK && slz_fused4096_supported(params)) {
        rc = slz_fused4096_init(ctx);
        ctx->has_fused4096 = (rc == SLZ_OK);
        if (rc == SLZ_E_UNSUPPORTED) rc = SLZ_OK;
    }
    if (rc == SLZ_OK && slz_fused512_supported(params)) {
        rc = slz_fused512_init(ctx);
        ctx->has_fused512 = (rc == SLZ_OK);
        if (rc == SLZ_E_UNSUPPORTED) rc = SLZ_OK;
    }
    if (rc == SLZ_OK && slz_fused1024_supported(params)) {
        rc = slz_fused1024_init(ctx);
        ctx->has_fused1024 = (rc == SLZ_OK);
        if (rc == SLZ_E_UNSUPPORTED) rc = SLZ_OK;
    }
    if (rc == SLZ_OK && slz_bign_supported(params)) {
        rc = slz_bign_init(ctx);
        ctx->has_bign = (rc == SLZ_OK);
        if (rc == SLZ_E_UNSUPPORTED) rc = SLZ_OK;
    }
    if (rc != SLZ_OK) { slz_ctx_destroy(ctx); return rc; }
    *out = ctx;
    return SLZ_OK;
}

extern "C" int slz_ctx_destroy(slz_ctx *ctx) {
    if (!ctx) return SLZ_E_INVALID_ARG;
    slz_fused_destroy(ctx);
    slz_fused1024_destroy(ctx);
    slz_fused512_destroy(ctx);
    slz_fused4096_destroy(ctx);
    slz_bign_destroy(ctx);
    slz_ksm_destroy(ctx);
    slz_lcm_destroy(ctx);
    slz_free_tables(ctx);
    if (ctx->acc) (void)hipFree(ctx->acc);
    if (ctx->dig) (void)hipFree(ctx->dig);
    if (ctx->xhat) (void)hipFree(ctx->xhat);
    if (ctx->outhat) (void)hipFree(ctx->outhat);
    if (ctx->ks_first_small) (void)hipFree(ctx->ks_first_small);
    delete ctx;
    return SLZ_OK;
}

extern "C" int slz_ctx_set_option(slz_ctx *ctx, int option, int value) {
    if (!ctx) return SLZ_E_INVALID_ARG;
    if (option == SLZ_OPT_FORCE_GENERIC) { ctx->force_generic = value != 0; return SLZ_OK; }
    if (option == SLZ_OPT_FAIL_ALLOC_AFTER) { g_fail_alloc_after = value < 0 ? -1 : value; return SLZ_OK; }
    if (option == SLZ_OPT_LARGE_N_BLOCK) {
        if (!ctx->has_bign) return SLZ_E_INVALID_ARG;
        if (value == 1024 && ctx->has_bign16) { ctx->bign_block = 1024; return SLZ_OK; }
        if (value == 2048 && ctx->bign_rowA) { ctx->bign_block = 2048; return SLZ_OK; }
        return SLZ_E_INVALID_ARG;
    }
    if (option == SLZ_OPT_FUSED_PACING) {
        if (!ctx->has_fused || value < 0 || value > 2) return SLZ_E_INVALID_ARG;
        ctx->fused_pacing = value;
        return SLZ_OK;
    }
    if (option == SLZ_OPT_LARGE_N_LATENCY) {
        if (!ctx->has_bign || (value != 0 && value != 1)) return SLZ_E_INVALID_ARG;
        ctx->bign_latency = value;
        return SLZ_OK;
    }
    if (option == SLZ_OPT_LARGE_N_LANES) {
        if (!ctx->has_bign || (value != 1 && value != 2)) return SLZ_E_INVALID_ARG;
        ctx->bign_lanes = value;
        return SLZ_OK;
    }
    return SLZ_E_INVALID_ARG;
}

extern "C" const char *slz_pbs_path(const slz_ctx *ctx) {
    if (!ctx) return "none";
    if (ctx->force_generic) return "generic";
    if (ctx->has_fused1024) return "fused_n1024";
    if (ctx->has_fused512) return "fused_n512";
    if (ctx->has_fused4096) return "fused_n4096";
    return ctx->has_fused ? "fused_n2048" : (ctx->has_bign ? "three_pass_large_n" : "generic");
}

extern "C" int slz_lut_encode(const slz_params *p, const uint64_t *table, uint32_t n_tables, uint64_t *lut_out) {
    int rc = check_params(p);
    if (rc != SLZ_OK) return rc;
    if (!table || !lut_out || n_tables == 0) return SLZ_E_INVALID_ARG;
    if (p->msg_bits >= 31) return SLZ_E_INVALID_ARG;
    const uint64_t t = 1ull << p->msg_bits;
    if ((uint64_t)p->N < 2 * t) return SLZ_E_INVALID_ARG;
    const uint64_t delta = 1ull << (63 - p->msg_bits);
    const uint32_t box = (uint32_t)(p->N / t), half = box / 2;
    for (uint32_t q = 0; q < n_tables; q++) {
        const uint64_t *f = table + (size_t)q * t;
        for (uint64_t m = 0; m < t; m++) if (f[m] >= t) return SLZ_E_INVALID_ARG;
        uint64_t *V = lut_out + (size_t)q * p->N;
        // box m covers coefficients [m*box - half, (m+1)*box - half); the part of box 0 below zero wraps
        // negacyclically to the top of the polynomial with its sign flipped.
        for (uint64_t m = 0; m < t; m++) {
            uint64_t val = delta * f[m];
            int64_t lo = (int64_t)(m * box) - (int64_t)half, hi = (int64_t)((m + 1) * box) - (int64_t)half;
            for (int64_t j = lo; j < hi; j++) {
                if (j >= 0) V[j] = val;
                else V[j + (int64_t)p->N] = (uint64_t)0 - val;
            }
        }
    }
    return SLZ_OK;
}

static size_t prepared_bytes(const slz_params &p) {
    return (size_t)p.n * 2 * (p.k + 1) * p.pbs_level * (p.k + 1) * p.N * sizeof(double);
}

extern "C" int slz_bsk_prepare(slz_ctx *ctx, const uint64_t *bsk_dev, void *dst_dev, size_t *dst_bytes, void *hip_stream) {
    if (!ctx || !dst_bytes) return SLZ_E_INVALID_ARG;
    const size_t need = prepared_bytes(ctx->prm);
    if (!dst_dev) { *dst_bytes = need; return SLZ_OK; }
    if (!bsk_dev || *dst_bytes < need || misaligned(bsk_dev) || misaligned(dst_dev)) return SLZ_E_INVALID_ARG;
    return slz_generic_bsk_prepare(ctx, bsk_dev, (double *)dst_dev, (hipStream_t)hip_stream);
}

// Scratch of the generic and the large-N path, sized for max_batch.  All or nothing: a buffer is committed to the context
// only when every allocation of the call has succeeded, so a call after SLZ_E_NOMEM starts from a clean state and no kernel
// ever sees a null scratch pointer.  The digit buffer is only used by the generic per-step kernels.
static int ensure_generic_scratch(slz_ctx *ctx) {
    const bool need_dig = !(ctx->has_bign && !ctx->force_generic);
    if (ctx->acc && ctx->xhat && ctx->outhat && (ctx->dig || !need_dig)) return SLZ_OK;
    const slz_params &p = ctx->prm;
    const size_t R = (size_t)(p.k + 1) * p.pbs_level, C = p.k + 1, B = ctx->max_batch, N = p.N;
    void *fresh[4] = {nullptr, nullptr, nullptr, nullptr};
    void *const have[4] = {ctx->acc, ctx->dig, ctx->xhat, ctx->outhat};
    const size_t bytes[4] = {B * C * N * 8, B * R * N * 8, B * 2 * R * N * 8, B * 2 * C * N * 8};
    const bool want[4] = {true, need_dig, true, true};
    for (int q = 0; q < 4; q++) {
        if (have[q] || !want[q]) continue;
        if (slz_scratch_alloc(&fresh[q], bytes[q]) != SLZ_OK) {
            for (int r = 0; r < q; r++)
                if (fresh[r]) (void)hipFree(fresh[r]);
            return SLZ_E_NOMEM;
        }
    }
    if (fresh[0]) ctx->acc = (uint64_t *)fresh[0];
    if (fresh[1]) ctx->dig = (double *)fresh[1];
    if (fresh[2]) ctx->xhat = (double *)fresh[2];
    if (fresh[3]) ctx->outhat = (double *)fresh[3];
    return SLZ_OK;
}

static int blind_rotate_common(slz_ctx *ctx, const uint64_t *lwe_in, const uint64_t *luts, const uint32_t *lut_idx,
                               uint32_t n_luts, const void *bskp, uint32_t n_steps, uint64_t *acc_out, uint64_t *lwe_out,
                               uint32_t batch, void *hip_stream) {
    if (!ctx || !lwe_in || !luts || !bskp || n_luts == 0 || batch == 0) return SLZ_E_INVALID_ARG;
    if (!acc_out && !lwe_out) return SLZ_E_INVALID_ARG;
    if (batch > ctx->max_batch) return SLZ_E_TOO_LARGE;
    if (n_steps > ctx->prm.n) return SLZ_E_INVALID_ARG;
    if (misaligned8(lwe_in) || misaligned(luts) || misaligned(bskp) || misaligned(acc_out) || misaligned8(lwe_out) ||
        ((uintptr_t)lut_idx & 3u))
        return SLZ_E_INVALID_ARG;
    hipStream_t s = (hipStream_t)hip_stream;
    if (ctx->has_fused && !ctx->force_generic)
        return slz_fused_blind_rotate(ctx, lwe_in, luts, lut_idx, (const double *)bskp, n_steps, acc_out, lwe_out, batch, s);
    if (ctx->has_fused4096 && !ctx->force_generic)
        return slz_fused4096_blind_rotate(ctx, lwe_in, luts, lut_idx, (const double *)bskp, n_steps, acc_out, lwe_out, batch, s);
    if (ctx->has_fused512 && !ctx->force_generic)
        return slz_fused512_blind_rotate(ctx, lwe_in, luts, lut_idx, (const double *)bskp, n_steps, acc_out, lwe_out, batch, s);
    if (ctx->has_fused1024 && !ctx->force_generic)
        return slz_fused1024_blind_rotate(ctx, lwe_in, luts, lut_idx, (const double *)bskp, n_steps, acc_out, lwe_out, batch, s);
    int rc = ensure_generic_scratch(ctx);
    if (rc != SLZ_OK) return rc;
    return slz_generic_blind_rotate(ctx, lwe_in, luts, lut_idx, (const double *)bskp, n_steps, acc_out, lwe_out, batch, s);
}

extern "C" int slz_pbs_batch(slz_ctx *ctx, const uint64_t *lwe_in_dev, const uint64_t *luts_dev, const uint32_t *lut_idx_dev,
                             uint32_t n_luts, const void *bsk_prepared_dev, uint64_t *lwe_out_dev, uint32_t batch,
                             void *hip_stream) {
    if (!lwe_out_dev) return SLZ_E_INVALID_ARG;
    return blind_rotate_common(ctx, lwe_in_dev, luts_dev, lut_idx_dev, n_luts, bsk_prepared_dev, ctx ? ctx->prm.n : 0, nullptr,
                               lwe_out_dev, batch, hip_stream);
}

extern "C" int slz_blind_rotate_batch(slz_ctx *ctx, const uint64_t *lwe_in_dev, const uint64_t *luts_dev,
                                      const uint32_t *lut_idx_dev, uint32_t n_luts, const void *bsk_prepared_dev, uint32_t n_steps,
                                      uint64_t *acc_out_dev, uint32_t batch, void *hip_stream) {
    if (!acc_out_dev) return SLZ_E_INVALID_ARG;
    return blind_rotate_common(ctx, lwe_in_dev, luts_dev, lut_idx_dev, n_luts, bsk_prepared_dev, n_steps, acc_out_dev, nullptr,
                               batch, hip_stream);
}

extern "C" int slz_keyswitch_batch(slz_ctx *ctx, const uint64_t *lwe_in_dev, const uint64_t *ksk_dev, uint64_t *lwe_out_dev,
                                   uint32_t batch, void *hip_stream) {
    if (!ctx || !lwe_in_dev || !ksk_dev || !lwe_out_dev || batch == 0) return SLZ_E_INVALID_ARG;
    if (misaligned8(lwe_in_dev) || misaligned(ksk_dev) || misaligned8(lwe_out_dev)) return SLZ_E_INVALID_ARG;
    return slz_keyswitch_launch(ctx, lwe_in_dev, ksk_dev, lwe_out_dev, batch, (hipStream_t)hip_stream);
}

extern "C" int slz_ksk_prepare(slz_ctx *ctx, const uint64_t *ksk_dev, void *dst_dev, size_t *dst_bytes, void *hip_stream) {
    if (!ctx || !dst_bytes) return SLZ_E_INVALID_ARG;
    const size_t need = slz_ksm_prepared_bytes(&ctx->prm);
    if (need == 0) return SLZ_E_UNSUPPORTED;
    if (!dst_dev) { *dst_bytes = need; return SLZ_OK; }
    if (!ksk_dev || *dst_bytes < need || misaligned(ksk_dev) || misaligned(dst_dev)) return SLZ_E_INVALID_ARG;
    return slz_ksm_prepare(ctx, ksk_dev, dst_dev, (hipStream_t)hip_stream);
}

extern "C" int slz_keyswitch_batch_prepared(slz_ctx *ctx, const uint64_t *lwe_in_dev, const void *ksk_prepared_dev,
                                            uint64_t *lwe_out_dev, uint32_t batch, void *hip_stream) {
    if (!ctx || !lwe_in_dev || !ksk_prepared_dev || !lwe_out_dev || batch == 0) return SLZ_E_INVALID_ARG;
    if (misaligned8(lwe_in_dev) || misaligned(ksk_prepared_dev) || misaligned8(lwe_out_dev)) return SLZ_E_INVALID_ARG;
    const slz_params &p = ctx->prm;
    if (slz_ksm_prepared_bytes(&p) == 0) return SLZ_E_UNSUPPORTED;
    return slz_ksm_launch(ctx, lwe_in_dev, nullptr, ksk_prepared_dev, lwe_out_dev, batch, (hipStream_t)hip_stream);
}

// Keyswitch first, then bootstrapping, on ciphertexts under the big key.  The small ciphertexts between the two live in a
// scratch buffer of the context (max_batch rows, allocated on first use); everything is ordered on the one stream.
extern "C" int slz_ks_pbs_batch(slz_ctx *ctx, const uint64_t *lwe_in_dev, const uint64_t *ksk_dev, const uint64_t *luts_dev,
                                const uint32_t *lut_idx_dev, uint32_t n_luts, const void *bsk_prepared_dev, uint64_t *lwe_out_dev,
                                uint32_t batch, void *hip_stream) {
    if (!ctx || !lwe_in_dev || !ksk_dev || !luts_dev || !bsk_prepared_dev || !lwe_out_dev || batch == 0 || n_luts == 0)
        return SLZ_E_INVALID_ARG;
    if (batch > ctx->max_batch) return SLZ_E_TOO_LARGE;
    if (misaligned8(lwe_in_dev) || misaligned(ksk_dev) || misaligned(luts_dev) || misaligned(bsk_prepared_dev) ||
        misaligned8(lwe_out_dev) || ((uintptr_t)lut_idx_dev & 3u))
        return SLZ_E_INVALID_ARG;
    if (!ctx->ks_first_small) {
        void *buf = nullptr;
        if (slz_scratch_alloc(&buf, (size_t)ctx->max_batch * (ctx->prm.n + 1) * 8) != SLZ_OK) return SLZ_E_NOMEM;
        ctx->ks_first_small = (uint64_t *)buf;
    }
    int rc = slz_keyswitch_launch(ctx, lwe_in_dev, ksk_dev, ctx->ks_first_small, batch, (hipStream_t)hip_stream);
    if (rc != SLZ_OK) return rc;
    return blind_rotate_common(ctx, ctx->ks_first_small, luts_dev, lut_idx_dev, n_luts, bsk_prepared_dev, ctx->prm.n, nullptr,
                               lwe_out_dev, batch, hip_stream);
}

extern "C" int slz_lwe_lincomb_batch(slz_ctx *ctx, const uint64_t *cts_dev, const int32_t *w_dev, uint64_t *out_dev, uint32_t G,
                                     uint32_t J, uint32_t O, void *hip_stream) {
    if (!ctx || !cts_dev || !w_dev || !out_dev || G == 0 || J == 0 || O == 0) return SLZ_E_INVALID_ARG;
    if (G > 65535) return SLZ_E_UNSUPPORTED;
    if (misaligned8(cts_dev) || misaligned8(out_dev) || ((uintptr_t)w_dev & 3u)) return SLZ_E_INVALID_ARG;
    return slz_lincomb_launch(ctx, cts_dev, w_dev, out_dev, G, J, O, (hipStream_t)hip_stream);
}

extern "C" const char *slz_strerror(int code) {
    switch (code) {
        case SLZ_OK: return "success";
        case SLZ_E_INVALID_ARG: return "invalid argument";
        case SLZ_E_UNSUPPORTED: return "parameter set not supported by this build";
        case SLZ_E_HIP: return "HIP runtime error";
        case SLZ_E_NOMEM: return "out of device memory";
        case SLZ_E_TOO_LARGE: return "batch larger than the context's max_batch or than the fixed scratch of a _static entry point";
        default: return "unknown error code";
    }
}
