// Host side: transform tables for the two primes and the worst-case bound bookkeeping.
#include "slz_internal.h"
#include <vector>
#include <cmath>

typedef unsigned __int128 u128;

static uint64_t mulmod_u64(uint64_t a, uint64_t b, uint64_t p) { return (uint64_t)((u128)a * b % p); }
static uint64_t powmod_u64(uint64_t a, uint64_t e, uint64_t p) {
    uint64_t r = 1;
    while (e) { if (e & 1) r = mulmod_u64(r, a, p); a = mulmod_u64(a, a, p); e >>= 1; }
    return r;
}
static double centred(uint64_t v, uint64_t p) { return v > p / 2 ? -(double)(p - v) : (double)v; }
static uint32_t bitrev(uint32_t x, uint32_t bits) {
    uint32_t r = 0;
    for (uint32_t i = 0; i < bits; i++) r |= ((x >> i) & 1u) << (bits - 1 - i);
    return r;
}

// A primitive 2N-th root of unity mod p: 3 is a quadratic non-residue for both primes, so
// 3^((p-1)/2^18) has order exactly 2^18; raise it to 2^18/(2N).
static uint64_t root_2N(uint64_t p, uint32_t logN) {
    uint64_t g = powmod_u64(3, (p - 1) >> 18, p);
    return powmod_u64(g, 1ull << (18 - (logN + 1)), p);
}

// Worst-case bound (in units of p) of slz_mulmod's result for an input |x| <= in_bound * p, |w| <= p/2:
// 1/2 from the rounding to the nearest multiple plus the error of the quotient estimate,
// |x w / p| * 3 * 2^-53 <= in_bound * (p/2) * 3 * 2^-53 < in_bound * 0.1875 for p < 2^50.
double slz_mulmod_bound(double in_bound) { return 0.5 + 0.1875 * in_bound + 1e-9; }

int slz_build_tables(slz_ctx *ctx) {
    const uint32_t N = ctx->prm.N, logN = ctx->logN;
    const uint64_t primes[2] = {SLZ_P1_U64, SLZ_P2_U64};
    for (int q = 0; q < 2; q++) {
        const uint64_t p = primes[q];
        ctx->mod[q].p = (double)p;
        ctx->mod[q].pinv = 1.0 / (double)p;
        ctx->two32[q] = centred((1ull << 32) % p, p);
        const uint64_t psi = root_2N(p, logN);
        if (powmod_u64(psi, N, p) != p - 1) return SLZ_E_UNSUPPORTED;      // psi^N must be -1
        const uint64_t psi_inv = powmod_u64(psi, p - 2, p);
        const uint64_t n_inv = powmod_u64(N, p - 2, p);
        std::vector<double> fwd(N), inv(N), post(N);
        std::vector<uint64_t> pw(N), pwi(N);
        pw[0] = 1; pwi[0] = 1;
        for (uint32_t j = 1; j < N; j++) { pw[j] = mulmod_u64(pw[j - 1], psi, p); pwi[j] = mulmod_u64(pwi[j - 1], psi_inv, p); }
        fwd[0] = 1.0;
        for (uint32_t x = 1; x < N; x++) fwd[x] = centred(pw[bitrev(x, logN)], p);
        inv[0] = 1.0;
        for (uint32_t t = 1; t < N; t <<= 1)
            for (uint32_t j = 0; j < t; j++) {
                // psi^(-(N/t) j): exponent below 2N since j < t... (N/t)*j < N
                inv[t + j] = centred(pwi[(size_t)(N / t) * j], p);
            }
        for (uint32_t j = 0; j < N; j++) post[j] = centred(mulmod_u64(pwi[j], n_inv, p), p);
        double **dst[3] = {&ctx->tab[q].fwd, &ctx->tab[q].inv, &ctx->tab[q].post};
        std::vector<double> *src[3] = {&fwd, &inv, &post};
        for (int a = 0; a < 3; a++) {
            if (hipMalloc((void **)dst[a], (size_t)N * sizeof(double)) != hipSuccess) return SLZ_E_NOMEM;
            SLZ_HIP(hipMemcpy(*dst[a], src[a]->data(), (size_t)N * sizeof(double), hipMemcpyHostToDevice));
        }
    }
    ctx->p1inv_mod_p2 = centred(powmod_u64(SLZ_P1_U64 % SLZ_P2_U64, SLZ_P2_U64 - 2, SLZ_P2_U64), SLZ_P2_U64);

    // Where the generic path must fully reduce its values so that nothing reaches 2^53 (= 8 p):
    // simulate the worst-case growth |U +- V| <= |U| + mulmod_bound(|V|) stage by stage.
    const double limit = 7.0;
    const double rows = (double)((ctx->prm.k + 1) * ctx->prm.pbs_level);
    double a = 0.5 + 1e-9;                             // reduced key residues; digits are far smaller
    ctx->fwd_reduce_mask = 0;
    for (uint32_t s = 0; s < logN; s++) {
        if (a + slz_mulmod_bound(a) > limit) { ctx->fwd_reduce_mask |= 1u << s; a = 0.5 + 1e-9; }
        a = a + slz_mulmod_bound(a);
    }
    ctx->fwd_out_bound = a;
    a = 0.5 + 1e-9;                                    // the pointwise sums are reduced before the inverse
    ctx->inv_reduce_mask = 0;
    for (uint32_t s = 0; s < logN; s++) {
        if (a + slz_mulmod_bound(a) > limit) { ctx->inv_reduce_mask |= 1u << s; a = 0.5 + 1e-9; }
        a = a + slz_mulmod_bound(a);
    }
    (void)rows;
    return SLZ_OK;
}

void slz_free_tables(slz_ctx *ctx) {
    for (int q = 0; q < 2; q++) {
        if (ctx->tab[q].fwd) (void)hipFree(ctx->tab[q].fwd);
        if (ctx->tab[q].inv) (void)hipFree(ctx->tab[q].inv);
        if (ctx->tab[q].post) (void)hipFree(ctx->tab[q].post);
        ctx->tab[q].fwd = ctx->tab[q].inv = ctx->tab[q].post = nullptr;
    }
}
