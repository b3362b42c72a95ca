// Host-side pieces shared by the fused blind-rotation kernels (N = 512, 1024, 2048, 4096): the argument fields every one
// of them takes, the worst-case bound check of their fixed reduction schedules, and the launch shape.
#pragma once
#include "slz_internal.h"

// What every fused kernel is given: the call's buffers and sizes, the per-prime tables every schedule uses, the CRT
// constant.  Each kernel's argument struct derives from this and adds its own tables.
struct slz_fused_io {
    const uint64_t *lwe_in;
    const uint64_t *luts;
    const uint32_t *lut_idx;
    const double *bskp;
    uint64_t *acc_out;
    uint64_t *lwe_out;
    uint32_t n, n_steps, batch, beta;
    const double *inv[2];     // [N]  inv[t + j]: cyclic inverse twiddles
    const double *post[2];    // [N]  psi^-j / N
    slz_mod mod[2];
    double p1inv_mod_p2;
};

static inline void slz_fused_fill_io(slz_fused_io &A, const slz_ctx *ctx, const uint64_t *lwe_in, const uint64_t *luts,
                                     const uint32_t *lut_idx, const double *bskp, uint32_t n_steps, uint64_t *acc_out,
                                     uint64_t *lwe_out, uint32_t batch) {
    A.lwe_in = lwe_in; A.luts = luts; A.lut_idx = lut_idx; A.bskp = bskp; A.acc_out = acc_out; A.lwe_out = lwe_out;
    A.n = ctx->prm.n; A.n_steps = n_steps; A.batch = batch; A.beta = ctx->prm.pbs_base_log;
    for (int q = 0; q < 2; q++) {
        A.inv[q] = ctx->tab[q].inv;
        A.post[q] = ctx->tab[q].post;
        A.mod[q] = ctx->mod[q];
    }
    A.p1inv_mod_p2 = ctx->p1inv_mod_p2;
}

// The reduction schedule all fused kernels share, as stage counts (bounds in units of p; every value must stay below
// 2^53 = 8 p, taken as 7.5 p):
//   forward: `pre` stages across blocks on the digits (N = 4096: 1), `fwd_a` stages, one full reduction, `fwd_b` stages;
//   products: `summed` products of a forward output with a key word are added before the next reduction;
//   inverse: two multiply-free stages (each doubles the bound), `inv_a` stages, one full reduction, `inv_b` stages, then
//   `post_mul` further multiplies (twist; N = 4096: reduction, stage across the blocks, twist), after which the CRT lift
//   needs |r| < 1.95 p.
static inline bool slz_fused_schedule_ok(int pre, int fwd_a, int fwd_b, int summed, int inv_a, int inv_b, bool reduce_before_post,
                                         int post_mul) {
    double a = 1e-6;
    for (int s = 0; s < pre + fwd_a; s++) a += slz_mulmod_bound(a);
    if (a > 7.5) return false;
    a = 0.5 + 1e-9;
    for (int s = 0; s < fwd_b; s++) a += slz_mulmod_bound(a);
    if (a > 7.5 || summed * slz_mulmod_bound(a) > 7.5) return false;
    a = 2.0 * (0.5 + 1e-9) * 2.0;
    for (int s = 0; s < inv_a; s++) a += slz_mulmod_bound(a);
    if (a > 7.5) return false;
    a = 0.5 + 1e-9;
    for (int s = 0; s < inv_b; s++) a += slz_mulmod_bound(a);
    if (a > 7.5) return false;
    if (reduce_before_post) a = 0.5 + 1e-9;
    for (int s = 0; s + 1 < post_mul; s++) a += slz_mulmod_bound(a);
    return slz_mulmod_bound(a) <= 1.95;
}

// Persistent grid: one workgroup per ciphertext up to what is resident at `per_cu` workgroups per compute unit.
static inline uint32_t slz_fused_grid(uint32_t batch, uint32_t per_cu) {
    const uint32_t resident = per_cu * 256u;
    return batch < resident ? batch : resident;
}

// host copy of the lane-uniform inverse twiddles inv[t + j], t + j < 32, of both primes (kernel-argument scalars)
static inline int slz_fused_load_inv_scalars(slz_ctx *ctx) {
    for (int q = 0; q < 2; q++)
        SLZ_HIP(hipMemcpy(ctx->fused_scalars[q][1], ctx->tab[q].inv, 32 * sizeof(double), hipMemcpyDeviceToHost));
    return SLZ_OK;
}
