// Lookup with two encrypted inputs, IntCELossDeriv (the paper's Algorithm of that name) and the clipped weight update (last
// step of the paper's Algorithm "End-to-End Training") on LWE ciphertexts: table lookups joined by element-wise kernels.
#include "slz_gadget_util.h"
#include "../../include/silenzio_gadgets.h"
#include <cmath>
#include <vector>

// out[c][.] = mult * x[c][.] + y[c][.], plus add_body on the body word (all modulo 2^64)
__global__ void __launch_bounds__(MR_THREADS)
k_pack2(const uint64_t *__restrict__ x, const uint64_t *__restrict__ y, uint64_t *__restrict__ out, uint64_t mult, uint64_t add_body,
        size_t count, uint32_t n1) {
    const size_t total = count * n1;
    for (size_t gid = (size_t)blockIdx.x * MR_THREADS + threadIdx.x; gid < total; gid += (size_t)gridDim.x * MR_THREADS) {
        uint64_t v = mult * x[gid] + y[gid];
        if (gid % n1 == n1 - 1) v += add_body;
        out[gid] = v;
    }
}

// out[r][j][.] = mult * x[r][j][.] + sum_j' e[r][j'][.]
__global__ void __launch_bounds__(MR_THREADS)
k_pack_rowsum(const uint64_t *__restrict__ x, const uint64_t *__restrict__ e, uint64_t *__restrict__ out, uint64_t mult, uint32_t a,
              uint32_t b, uint32_t n1) {
    const size_t total = (size_t)a * b * n1;
    for (size_t gid = (size_t)blockIdx.x * MR_THREADS + threadIdx.x; gid < total; gid += (size_t)gridDim.x * MR_THREADS) {
        const uint32_t word = (uint32_t)(gid % n1);
        const size_t r = gid / ((size_t)b * n1);
        const uint64_t *row = e + r * b * n1 + word;
        uint64_t sum = 0;
        for (uint32_t j = 0; j < b; j++) sum += row[(size_t)j * n1];
        out[gid] = mult * x[gid] + sum;
    }
}

static uint32_t bits_of(uint64_t v) { uint32_t n = 0; while (v) { n++; v >>= 1; } return n; }

// round(num / den), ties to even, on non-negative integers
static uint64_t div_round_even(uint64_t num, uint64_t den) {
    const uint64_t q = num / den, r = num % den;
    return q + ((2 * r > den || (2 * r == den && (q & 1))) ? 1 : 0);
}

// ---- two-input lookup ------------------------------------------------------------------------------------------------
struct bv_plan { size_t n1, N1, chunk, o_big, o_packed, total; };

static bv_plan make_bv_plan(const slz_ctx *ctx, size_t count) {
    bv_plan P;
    P.n1 = ctx->prm.n + 1;
    P.N1 = (size_t)ctx->prm.k * ctx->prm.N + 1;
    P.chunk = count < ctx->max_batch ? count : ctx->max_batch;
    size_t o = 0;
    P.o_big = o;    o += up256(P.chunk * P.N1 * 8);
    P.o_packed = o; o += up256(count * P.n1 * 8);
    P.total = o;
    return P;
}

extern "C" int slz_bivariate_workspace(const slz_ctx *ctx, uint32_t count, size_t *bytes) {
    if (!ctx || !bytes || count == 0) return SLZ_E_INVALID_ARG;
    *bytes = make_bv_plan(ctx, count).total;
    return SLZ_OK;
}

static bool ct_ptrs_ok(const void *a, const void *b, const void *c, const void *luts, const void *ws) {
    return a && b && c && luts && ws && !(((uintptr_t)a | (uintptr_t)b | (uintptr_t)c) & 7u) && !((uintptr_t)luts & 15u) &&
           !((uintptr_t)ws & 255u);
}

// the packed ciphertexts mult x + y (+ add on the body), then one lookup each
static int packed_lookup(slz_ctx *ctx, const uint64_t *x, const uint64_t *y, uint64_t mult, uint64_t add, const uint64_t *luts,
                         const uint32_t *idx, uint32_t n_luts, const void *bskp, const uint64_t *ksk, uint64_t *out, uint32_t count,
                         void *workspace, size_t workspace_bytes, void *hip_stream) {
    const bv_plan P = make_bv_plan(ctx, count);
    if (workspace_bytes < P.total) return SLZ_E_INVALID_ARG;
    char *ws = (char *)workspace;
    uint64_t *big = (uint64_t *)(ws + P.o_big), *packed = (uint64_t *)(ws + P.o_packed);
    const uint64_t add_body = add << (63 - ctx->prm.msg_bits);
    hipLaunchKernelGGL(k_pack2, ew_grid((size_t)count * P.n1), dim3(MR_THREADS), 0, (hipStream_t)hip_stream, x, y, packed, mult, add_body,
                       (size_t)count, (uint32_t)P.n1);
    int rc = lookup_n(ctx, P.chunk, P.n1, packed, luts, idx, n_luts, bskp, ksk, big, out, count, hip_stream);
    if (rc != SLZ_OK) return rc;
    SLZ_HIP(hipGetLastError());
    return SLZ_OK;
}

extern "C" int slz_bivariate_lookup(slz_ctx *ctx, const uint64_t *x, const uint64_t *y, uint32_t y_bits, const uint64_t *luts,
                                    const uint32_t *lut_index, uint32_t n_luts, const void *bskp, const uint64_t *ksk, uint64_t *out,
                                    uint32_t count, void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!ctx || !bskp || !ksk || count == 0 || n_luts == 0 || !ct_ptrs_ok(x, y, out, luts, workspace)) return SLZ_E_INVALID_ARG;
    if (y_bits >= ctx->prm.msg_bits || ((uintptr_t)lut_index & 3u)) return SLZ_E_INVALID_ARG;
    return packed_lookup(ctx, x, y, 1ull << y_bits, 0, luts, lut_index, n_luts, bskp, ksk, out, count, workspace, workspace_bytes,
                         hip_stream);
}

// ---- clipped weight update --------------------------------------------------------------------------------------------
extern "C" int slz_weight_update_luts(const slz_params *p, uint32_t alpha, uint64_t *luts_out) {
    if (!p || !luts_out || alpha < 2 || alpha + 2 > p->msg_bits) return SLZ_E_INVALID_ARG;
    const uint64_t t = 1ull << p->msg_bits;
    const int64_t half = 1ll << (alpha - 1);
    std::vector<uint64_t> tab(t, 0);
    for (uint64_t u = 0; u < (1ull << (alpha + 2)); u++) {
        const int64_t w = (int64_t)(u >> 2) - half;
        const int64_t code = (int64_t)(u & 3);
        int64_t r = w - ((code > 2 ? 2 : code) - 1);
        r = r < -half ? -half : (r > half - 1 ? half - 1 : r);
        tab[u] = (uint64_t)((r + (int64_t)t) % (int64_t)t);
    }
    return slz_lut_encode(p, tab.data(), 1, luts_out);
}

extern "C" int slz_weight_update(slz_ctx *ctx, uint32_t alpha, const uint64_t *w, const uint64_t *gcode, const uint64_t *luts,
                                 const void *bskp, const uint64_t *ksk, uint64_t *w_out, uint32_t count, void *workspace,
                                 size_t workspace_bytes, void *hip_stream) {
    if (!ctx || !bskp || !ksk || count == 0 || !ct_ptrs_ok(w, gcode, w_out, luts, workspace)) return SLZ_E_INVALID_ARG;
    if (alpha < 2 || alpha + 2 > ctx->prm.msg_bits) return SLZ_E_INVALID_ARG;
    return packed_lookup(ctx, w, gcode, 4, 4ull << (alpha - 1), luts, nullptr, 1, bskp, ksk, w_out, count, workspace, workspace_bytes,
                         hip_stream);
}

// ---- IntCELossDeriv --------------------------------------------------------------------------------------------------------
static bool loss_shape_ok(const slz_params *p, const slz_loss_shape *sh, uint32_t *eb, uint32_t *sb) {
    if (!p || !sh || sh->a == 0 || sh->b == 0 || sh->b > 16 || sh->kappa == 0 || sh->kappa > 16) return false;
    if (sh->big_gamma < 2 || sh->big_gamma > p->msg_bits) return false;
    *eb = bits_of(1ull << sh->kappa);
    *sb = bits_of((uint64_t)sh->b << sh->kappa);
    return *eb + *sb <= p->msg_bits && (uint64_t)sh->a * sh->b < (1ull << 31);
}

extern "C" int slz_loss_luts(const slz_params *p, const slz_loss_shape *sh, uint64_t *luts_out) {
    uint32_t eb, sb;
    if (!luts_out || !loss_shape_ok(p, sh, &eb, &sb)) return SLZ_E_INVALID_ARG;
    const uint64_t t = 1ull << p->msg_bits;
    std::vector<uint64_t> tab((size_t)5 * t, 0);
    uint64_t *relu = tab.data(), *ex = relu + t, *share = ex + t, *prod = share + t, *sgn = prod + t;
    const uint64_t top = (1ull << (sh->big_gamma - 1)) - 1;      // the largest logit
    for (uint64_t v = 0; v < t; v++) {
        relu[v] = v < t / 2 ? v : 0;
        if (v <= top) ex[v] = (uint64_t)std::nearbyint(std::exp((double)v - (double)top) * (double)(1ull << sh->kappa));
        sgn[v] = v > t / 2 ? 1 : (v < t / 2 ? t - 1 : 0);
    }
    for (uint64_t e = 0; e < (1ull << eb); e++)
        for (uint64_t s = 0; s < (1ull << sb); s++)
            share[(e << sb) + s] = div_round_even((e << sh->kappa) + 1, s + 1) % t;
    for (uint64_t s = 0; s < (1ull << sb); s++) prod[(1ull << sb) + s] = s;
    return slz_lut_encode(p, tab.data(), 5, luts_out);
}

struct loss_plan { size_t n1, N1, cts, chunk, o_big, o_e, o_q, o_packed, total; };

static loss_plan make_loss_plan(const slz_ctx *ctx, const slz_loss_shape *sh) {
    loss_plan P;
    P.n1 = ctx->prm.n + 1;
    P.N1 = (size_t)ctx->prm.k * ctx->prm.N + 1;
    P.cts = (size_t)sh->a * sh->b;
    P.chunk = P.cts < ctx->max_batch ? P.cts : ctx->max_batch;
    size_t o = 0;
    P.o_big = o;    o += up256(P.chunk * P.N1 * 8);
    P.o_e = o;      o += up256(P.cts * P.n1 * 8);       // exponentials, later the label products
    P.o_q = o;      o += up256(P.cts * P.n1 * 8);       // shares
    P.o_packed = o; o += up256(P.cts * P.n1 * 8);       // input of the current lookup
    P.total = o;
    return P;
}

extern "C" int slz_loss_workspace(const slz_ctx *ctx, const slz_loss_shape *sh, size_t *bytes) {
    uint32_t eb, sb;
    if (!ctx || !bytes || !loss_shape_ok(&ctx->prm, sh, &eb, &sb)) return SLZ_E_INVALID_ARG;
    *bytes = make_loss_plan(ctx, sh).total;
    return SLZ_OK;
}

extern "C" int slz_int_ce_loss_deriv(slz_ctx *ctx, const slz_loss_shape *sh, const uint64_t *logits, const uint64_t *labels,
                                     const uint64_t *luts, const void *bskp, const uint64_t *ksk, uint64_t *e_out, void *workspace,
                                     size_t workspace_bytes, void *hip_stream) {
    uint32_t eb, sb;
    if (!ctx || !bskp || !ksk || !loss_shape_ok(&ctx->prm, sh, &eb, &sb) || !ct_ptrs_ok(logits, labels, e_out, luts, workspace))
        return SLZ_E_INVALID_ARG;
    const loss_plan P = make_loss_plan(ctx, sh);
    if (workspace_bytes < P.total) return SLZ_E_INVALID_ARG;
    hipStream_t s = (hipStream_t)hip_stream;
    char *ws = (char *)workspace;
    uint64_t *big = (uint64_t *)(ws + P.o_big), *e = (uint64_t *)(ws + P.o_e), *q = (uint64_t *)(ws + P.o_q);
    uint64_t *packed = (uint64_t *)(ws + P.o_packed);
    const size_t N = ctx->prm.N;
    const uint32_t n1 = (uint32_t)P.n1;
    auto look = [&](const uint64_t *in, uint32_t table, uint64_t *out) {
        return lookup_n(ctx, P.chunk, P.n1, in, luts + (size_t)table * N, nullptr, 1, bskp, ksk, big, out, P.cts, hip_stream);
    };
    // E = ReLU(logits), then the approximated exponential
    int rc = look(logits, 0, packed);
    if (rc != SLZ_OK) return rc;
    rc = look(packed, 1, e);
    if (rc != SLZ_OK) return rc;
    // share of the row sum: lookup on 2^sb E + S
    hipLaunchKernelGGL(k_pack_rowsum, ew_grid(P.cts * n1), dim3(MR_THREADS), 0, s, e, e, packed, 1ull << sb, sh->a, sh->b, n1);
    rc = look(packed, 2, q);
    if (rc != SLZ_OK) return rc;
    // label times the row sum of the shares: lookup on 2^sb label + T
    hipLaunchKernelGGL(k_pack_rowsum, ew_grid(P.cts * n1), dim3(MR_THREADS), 0, s, labels, q, packed, 1ull << sb, sh->a, sh->b, n1);
    rc = look(packed, 3, e);
    if (rc != SLZ_OK) return rc;
    // error = share - product, moved up by t / 2; then its sign
    hipLaunchKernelGGL(k_pack2, ew_grid(P.cts * n1), dim3(MR_THREADS), 0, s, e, q, packed, ~0ull, 1ull << 62, P.cts, n1);
    rc = look(packed, 4, e_out);
    if (rc != SLZ_OK) return rc;
    SLZ_HIP(hipGetLastError());
    return SLZ_OK;
}
