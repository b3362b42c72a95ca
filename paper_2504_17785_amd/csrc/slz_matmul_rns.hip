// Matmul^RNS (the paper's Algorithm "Matmul^RNS") on LWE ciphertexts: three rounds of table lookups
// (slz_pbs_batch + slz_keyswitch_batch) joined by element-wise kernels on ciphertext vectors.
#include "slz_internal.h"
#include "../../include/silenzio_gadgets.h"
#include <vector>

#define MR_THREADS 256

static bool shape_ok(const slz_params *p, const slz_matmul_rns_shape *sh) {
    if (!p || !sh || sh->k == 0 || sh->k > SLZ_MATMUL_RNS_MAX_K || sh->a == 0 || sh->b == 0 || sh->c == 0) return false;
    if (p->msg_bits < 8) return false;
    for (uint32_t i = 0; i < sh->k; i++)
        if (sh->m[i] < 2 || sh->m[i] > 16) return false;
    const uint64_t prods = (uint64_t)sh->k * sh->a * sh->b * sh->c;
    return prods < (1ull << 31) && (uint64_t)sh->k * ((uint64_t)sh->a * sh->b + (uint64_t)sh->b * sh->c) < (1ull << 31);
}

extern "C" int slz_matmul_rns_luts(const slz_params *p, const slz_matmul_rns_shape *sh, uint64_t *luts_out) {
    if (!luts_out || !shape_ok(p, sh)) return SLZ_E_INVALID_ARG;
    const uint64_t t = 1ull << p->msg_bits;
    std::vector<uint64_t> tab((size_t)3 * sh->k * t);
    for (uint32_t i = 0; i < sh->k; i++) {
        const int64_t q = sh->m[i];
        uint64_t *rs = tab.data() + (size_t)i * t, *pr = tab.data() + (size_t)(sh->k + i) * t, *rd = tab.data() + (size_t)(2 * sh->k + i) * t;
        for (uint64_t v = 0; v < t; v++) {
            const int64_t sv = v < t / 2 ? (int64_t)v : (int64_t)v - (int64_t)t;
            rs[v] = (uint64_t)(((sv % q) + q) % q);
            pr[v] = v < 256 ? ((v >> 4) * (v & 15)) % (uint64_t)q : 0;
            rd[v] = v % (uint64_t)q;
        }
    }
    return slz_lut_encode(p, tab.data(), 3 * sh->k, luts_out);
}

// ---- workspace -----------------------------------------------------------------------------------------------------
struct mr_plan {
    size_t n1, N1;
    size_t n_in, n_prod, n_out, nblk, chunk;
    // offsets in bytes
    size_t o_rep, o_idx, o_big, o_res, o_packed, o_ys, o_sums, o_wts, o_tmp, total;
};

static size_t up256(size_t x) { return (x + 255) / 256 * 256; }

static mr_plan make_plan(const slz_ctx *ctx, const slz_matmul_rns_shape *sh) {
    mr_plan P;
    P.n1 = ctx->prm.n + 1;
    P.N1 = (size_t)ctx->prm.k * ctx->prm.N + 1;
    P.n_in = (size_t)sh->k * ((size_t)sh->a * sh->b + (size_t)sh->b * sh->c);
    P.n_prod = (size_t)sh->k * sh->a * sh->b * sh->c;
    P.n_out = (size_t)sh->k * sh->a * sh->c;
    P.nblk = (sh->b + SLZ_MATMUL_RNS_BLOCK - 1) / SLZ_MATMUL_RNS_BLOCK;
    const size_t biggest = P.n_in > P.n_prod ? P.n_in : P.n_prod;
    P.chunk = biggest < ctx->max_batch ? biggest : ctx->max_batch;
    size_t o = 0;
    P.o_rep = o;    o += up256(P.n_in * P.n1 * 8);            // step 1 inputs, one copy per modulus
    P.o_idx = o;    o += up256(biggest * 4);                  // table index per ciphertext of the current lookup
    P.o_big = o;    o += up256(P.chunk * P.N1 * 8);           // PBS outputs of one chunk (big key)
    P.o_res = o;    o += up256(P.n_in * P.n1 * 8);            // X', W'
    P.o_packed = o; o += up256(P.n_prod * P.n1 * 8);          // 16 x' + w', laid out [k][a][c][b]
    P.o_ys = o;     o += up256(P.n_prod * P.n1 * 8);          // Y*, same layout
    P.o_sums = o;   o += up256(P.n_out * P.nblk * P.n1 * 8);  // block sums [k a c][nblk]
    P.o_wts = o;    o += up256((size_t)sh->b * P.nblk * 4);   // block-indicator weights [b][nblk]
    P.o_tmp = o;    o += up256(P.n_out * P.n1 * 8);           // Y + Y'
    P.total = o;
    return P;
}

extern "C" int slz_matmul_rns_workspace(const slz_ctx *ctx, const slz_matmul_rns_shape *sh, size_t *bytes) {
    if (!ctx || !bytes || !shape_ok(&ctx->prm, sh)) return SLZ_E_INVALID_ARG;
    *bytes = make_plan(ctx, sh).total;
    return SLZ_OK;
}

// ---- element-wise kernels on ciphertext vectors --------------------------------------------------------------------
// rep[i][j][.] = (j < ab ? X[j] : W[j - ab]) for every modulus i; idx[i][j] = i
__global__ void __launch_bounds__(MR_THREADS)
k_mr_replicate(const uint64_t *__restrict__ x, const uint64_t *__restrict__ w, uint64_t *__restrict__ rep, uint32_t *__restrict__ idx,
               uint32_t k, size_t ab, size_t bc, uint32_t n1) {
    const size_t per = ab + bc;
    const size_t total = (size_t)k * per * n1;
    for (size_t gid = (size_t)blockIdx.x * MR_THREADS + threadIdx.x; gid < total; gid += (size_t)gridDim.x * MR_THREADS) {
        const uint32_t word = (uint32_t)(gid % n1);
        const size_t ct = gid / n1;
        const size_t j = ct % per;
        rep[gid] = j < ab ? x[j * n1 + word] : w[(j - ab) * n1 + word];
        if (word == 0) idx[ct] = (uint32_t)(ct / per);
    }
}

// packed[i][r][s][j][.] = 16 X'[i][r][j][.] + W'[i][j][s][.];  idx[...] = i.   res = [k][ab + bc][n1]
__global__ void __launch_bounds__(MR_THREADS)
k_mr_pack(const uint64_t *__restrict__ res, uint64_t *__restrict__ packed, uint32_t *__restrict__ idx, uint32_t k, uint32_t a,
          uint32_t b, uint32_t c, uint32_t n1) {
    const size_t per = (size_t)a * b + (size_t)b * c;
    const size_t total = (size_t)k * a * c * b * n1;
    for (size_t gid = (size_t)blockIdx.x * MR_THREADS + threadIdx.x; gid < total; gid += (size_t)gridDim.x * MR_THREADS) {
        const uint32_t word = (uint32_t)(gid % n1);
        size_t ct = gid / n1;
        const uint32_t j = (uint32_t)(ct % b);
        const uint32_t s = (uint32_t)((ct / b) % c);
        const uint32_t r = (uint32_t)((ct / ((size_t)b * c)) % a);
        const uint32_t i = (uint32_t)(ct / ((size_t)a * b * c));
        const uint64_t *base = res + (size_t)i * per * n1;
        const uint64_t xv = base[((size_t)r * b + j) * n1 + word];
        const uint64_t wv = base[((size_t)a * b + (size_t)j * c + s) * n1 + word];
        packed[gid] = 16ull * xv + wv;
        if (word == 0) idx[ct] = i;
    }
}

// wts[j][o] = 1 if input j belongs to block o
__global__ void k_mr_weights(int32_t *wts, uint32_t b, uint32_t nblk) {
    const uint32_t gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (gid < b * nblk) wts[gid] = (gid / nblk) / SLZ_MATMUL_RNS_BLOCK == gid % nblk ? 1 : 0;
}

// tmp[g][.] = (t > 0 ? y[g][.] : 0) + sums[g][t][.];  idx[g] = g / (a c)
__global__ void __launch_bounds__(MR_THREADS)
k_mr_accumulate(const uint64_t *__restrict__ y, const uint64_t *__restrict__ sums, uint64_t *__restrict__ tmp, uint32_t *__restrict__ idx,
                size_t n_out, uint32_t ac, uint32_t nblk, uint32_t t, uint32_t n1) {
    const size_t total = n_out * n1;
    for (size_t gid = (size_t)blockIdx.x * MR_THREADS + threadIdx.x; gid < total; gid += (size_t)gridDim.x * MR_THREADS) {
        const uint32_t word = (uint32_t)(gid % n1);
        const size_t g = gid / n1;
        const uint64_t sv = sums[(g * nblk + t) * n1 + word];
        tmp[gid] = t > 0 ? y[gid] + sv : sv;
        if (word == 0) idx[g] = (uint32_t)(g / ac);
    }
}

static dim3 ew_grid(size_t total) {
    size_t blocks = (total + MR_THREADS - 1) / MR_THREADS;
    return dim3((unsigned)(blocks < 65536 ? (blocks ? blocks : 1) : 65536));
}

// one table lookup per ciphertext, in chunks the context can hold
static int lookup(slz_ctx *ctx, const mr_plan &P, const uint64_t *in, const uint64_t *luts, const uint32_t *idx, uint32_t n_luts,
                  const void *bskp, const uint64_t *ksk, uint64_t *big, uint64_t *out, size_t count, void *stream) {
    for (size_t c0 = 0; c0 < count; c0 += P.chunk) {
        const uint32_t nb = (uint32_t)(count - c0 < P.chunk ? count - c0 : P.chunk);
        int rc = slz_pbs_batch(ctx, in + c0 * P.n1, luts, idx + c0, n_luts, bskp, big, nb, stream);
        if (rc != SLZ_OK) return rc;
        rc = slz_keyswitch_batch(ctx, big, ksk, out + c0 * P.n1, nb, stream);
        if (rc != SLZ_OK) return rc;
    }
    return SLZ_OK;
}

extern "C" int slz_matmul_rns(slz_ctx *ctx, const slz_matmul_rns_shape *sh, const uint64_t *x, const uint64_t *w, const uint64_t *luts,
                              const void *bskp, const uint64_t *ksk, uint64_t *y, void *workspace, size_t workspace_bytes,
                              void *hip_stream) {
    if (!ctx || !x || !w || !luts || !bskp || !ksk || !y || !workspace || !shape_ok(&ctx->prm, sh)) return SLZ_E_INVALID_ARG;
    if (((uintptr_t)workspace & 255u) || ((uintptr_t)x & 7u) || ((uintptr_t)w & 7u) || ((uintptr_t)y & 7u) || ((uintptr_t)luts & 15u))
        return SLZ_E_INVALID_ARG;
    const mr_plan P = make_plan(ctx, sh);
    if (workspace_bytes < P.total) return SLZ_E_INVALID_ARG;
    hipStream_t s = (hipStream_t)hip_stream;
    char *ws = (char *)workspace;
    uint64_t *rep = (uint64_t *)(ws + P.o_rep), *big = (uint64_t *)(ws + P.o_big), *res = (uint64_t *)(ws + P.o_res);
    uint64_t *packed = (uint64_t *)(ws + P.o_packed), *ys = (uint64_t *)(ws + P.o_ys), *sums = (uint64_t *)(ws + P.o_sums);
    uint64_t *tmp = (uint64_t *)(ws + P.o_tmp);
    uint32_t *idx = (uint32_t *)(ws + P.o_idx);
    int32_t *wts = (int32_t *)(ws + P.o_wts);
    const uint32_t k = sh->k, a = sh->a, b = sh->b, c = sh->c, n1 = (uint32_t)P.n1;
    const size_t N = ctx->prm.N;

    // Step 1: X' = X mod m', W' = W mod m'
    hipLaunchKernelGGL(k_mr_replicate, ew_grid(P.n_in * n1), dim3(MR_THREADS), 0, s, x, w, rep, idx, k, (size_t)a * b, (size_t)b * c, n1);
    int rc = lookup(ctx, P, rep, luts, idx, k, bskp, ksk, big, res, P.n_in, hip_stream);
    if (rc != SLZ_OK) return rc;
    // Step 2: partial products on the packed value 16 x' + w'
    hipLaunchKernelGGL(k_mr_pack, ew_grid(P.n_prod * n1), dim3(MR_THREADS), 0, s, res, packed, idx, k, a, b, c, n1);
    rc = lookup(ctx, P, packed, luts + (size_t)k * N, idx, k, bskp, ksk, big, ys, P.n_prod, hip_stream);
    if (rc != SLZ_OK) return rc;
    // Step 3: sums of at most 15 products per block (one linear combination with block-indicator weights), then the
    // running sum Y <- (Y + Y') mod m', one lookup per block
    hipLaunchKernelGGL(k_mr_weights, dim3((b * (uint32_t)P.nblk + 255) / 256), dim3(256), 0, s, wts, b, (uint32_t)P.nblk);
    const size_t groups = P.n_out;
    for (size_t g0 = 0; g0 < groups; g0 += 65535) {          // the linear combination takes at most 65535 groups per call
        const uint32_t ng = (uint32_t)(groups - g0 < 65535 ? groups - g0 : 65535);
        rc = slz_lwe_lincomb_batch(ctx, ys + g0 * b * n1, wts, sums + g0 * P.nblk * n1, ng, b, (uint32_t)P.nblk, hip_stream);
        if (rc != SLZ_OK) return rc;
    }
    for (uint32_t t = 0; t < P.nblk; t++) {
        hipLaunchKernelGGL(k_mr_accumulate, ew_grid(P.n_out * n1), dim3(MR_THREADS), 0, s, y, sums, tmp, idx, P.n_out, a * c,
                           (uint32_t)P.nblk, t, n1);
        rc = lookup(ctx, P, tmp, luts + (size_t)2 * k * N, idx, k, bskp, ksk, big, y, P.n_out, hip_stream);
        if (rc != SLZ_OK) return rc;
    }
    SLZ_HIP(hipGetLastError());
    return SLZ_OK;
}

// ---- RNS-to-MRNS conversion and sign determination -----------------------------------------------------------------
#define RNS_OFFSET 16u      // moves a difference of two residues (each below 16) into [1, 31]

static uint32_t gcd_u32(uint32_t a, uint32_t b) { while (b) { uint32_t t = a % b; a = b; b = t; } return a; }

static bool rns_shape_ok(const slz_params *p, const slz_rns_shape *sh) {
    if (!p || !sh || sh->k < 2 || sh->k > SLZ_MATMUL_RNS_MAX_K || sh->count == 0 || p->msg_bits < 8) return false;
    for (uint32_t i = 0; i < sh->k; i++) {
        if (sh->m[i] < 2 || sh->m[i] > 16) return false;
        for (uint32_t j = 0; j < i; j++)
            if (gcd_u32(sh->m[i], sh->m[j]) != 1) return false;
    }
    return (uint64_t)sh->k * sh->count < (1ull << 31);
}

static uint32_t pair_index(uint32_t k, uint32_t i, uint32_t j) { return i * k - i * (i + 1) / 2 + (j - i - 1); }

static uint32_t inv_mod(uint32_t a, uint32_t q) {
    for (uint32_t t = 1; t < q; t++)
        if ((a * t) % q == 1 % q) return t;
    return 0;       // q == 1 cannot happen (moduli are at least 2)
}

extern "C" int slz_rns_luts(const slz_params *p, const slz_rns_shape *sh, int32_t neg, int32_t zero, int32_t pos, uint64_t *luts_out) {
    if (!luts_out || !rns_shape_ok(p, sh)) return SLZ_E_INVALID_ARG;
    if (neg < -128 || neg > 127 || zero < -128 || zero > 127 || pos < -128 || pos > 127) return SLZ_E_INVALID_ARG;
    const uint64_t t = 1ull << p->msg_bits;
    const uint32_t k = sh->k, n_conv = k * (k - 1) / 2;
    std::vector<uint64_t> tab((size_t)(n_conv + 2) * t);
    for (uint32_t i = 0; i + 1 < k; i++)
        for (uint32_t j = i + 1; j < k; j++) {
            const int64_t q = sh->m[j], inv = inv_mod(sh->m[i] % sh->m[j], sh->m[j]);
            uint64_t *row = tab.data() + (size_t)pair_index(k, i, j) * t;
            for (uint64_t v = 0; v < t; v++) {
                const int64_t d = ((int64_t)v - (int64_t)RNS_OFFSET) % q;
                row[v] = (uint64_t)((((d + q) % q) * inv) % q);
            }
        }
    uint64_t *top = tab.data() + (size_t)n_conv * t, *sel = top + t;
    const uint64_t top_m = sh->m[k - 1];
    for (uint64_t v = 0; v < t; v++) {
        top[v] = (v < top_m && v >= top_m / 2) ? 1 : 0;
        const int64_t r = v == 0 ? zero : (v < 128 ? pos : neg);
        sel[v] = (uint64_t)((r + (int64_t)t) % (int64_t)t);
    }
    return slz_lut_encode(p, tab.data(), n_conv + 2, luts_out);
}

struct rns_plan {
    size_t n1, N1, chunk, total_cts;
    size_t o_idx, o_big, o_tmp, o_y, o_neg, total;
};

static rns_plan make_rns_plan(const slz_ctx *ctx, const slz_rns_shape *sh) {
    rns_plan P;
    P.n1 = ctx->prm.n + 1;
    P.N1 = (size_t)ctx->prm.k * ctx->prm.N + 1;
    P.total_cts = (size_t)sh->k * sh->count;
    P.chunk = P.total_cts < ctx->max_batch ? P.total_cts : ctx->max_batch;
    size_t o = 0;
    P.o_idx = o; o += up256(P.total_cts * 4);
    P.o_big = o; o += up256(P.chunk * P.N1 * 8);
    P.o_tmp = o; o += up256(P.total_cts * P.n1 * 8);      // differences of one round / the packed sign input
    P.o_y = o;   o += up256(P.total_cts * P.n1 * 8);      // digits (the sign gadget's private copy)
    P.o_neg = o; o += up256((size_t)sh->count * P.n1 * 8);
    P.total = o;
    return P;
}

extern "C" int slz_rns_workspace(const slz_ctx *ctx, const slz_rns_shape *sh, size_t *bytes) {
    if (!ctx || !bytes || !rns_shape_ok(&ctx->prm, sh)) return SLZ_E_INVALID_ARG;
    *bytes = make_rns_plan(ctx, sh).total;
    return SLZ_OK;
}

// tmp[j - i][e][.] = y[j][e][.] - y[i-1][e][.] + 16 (on the body), j = i .. k-1;  idx = pair (i-1, j)
__global__ void __launch_bounds__(MR_THREADS)
k_rns_diff(const uint64_t *__restrict__ y, uint64_t *__restrict__ tmp, uint32_t *__restrict__ idx, uint32_t k, uint32_t i, size_t count,
           uint32_t n1, uint64_t offset_body, uint32_t pair0) {
    const size_t total = (size_t)(k - i) * count * n1;
    for (size_t gid = (size_t)blockIdx.x * MR_THREADS + threadIdx.x; gid < total; gid += (size_t)gridDim.x * MR_THREADS) {
        const uint32_t word = (uint32_t)(gid % n1);
        const size_t ct = gid / n1;
        const size_t e = ct % count;
        const uint32_t jj = (uint32_t)(ct / count);
        uint64_t v = y[((size_t)(i + jj) * count + e) * n1 + word] - y[((size_t)(i - 1) * count + e) * n1 + word];
        if (word == n1 - 1) v += offset_body;
        tmp[gid] = v;
        if (word == 0) idx[ct] = pair0 + jj;
    }
}

// tmp[e][.] = sum_i y[i][e][.] + 128 neg[e][.]
__global__ void __launch_bounds__(MR_THREADS)
k_rns_sign_pack(const uint64_t *__restrict__ y, const uint64_t *__restrict__ neg, uint64_t *__restrict__ tmp, uint32_t k, size_t count,
                uint32_t n1) {
    const size_t total = count * n1;
    for (size_t gid = (size_t)blockIdx.x * MR_THREADS + threadIdx.x; gid < total; gid += (size_t)gridDim.x * MR_THREADS) {
        uint64_t v = 128ull * neg[gid];
        for (uint32_t i = 0; i < k; i++) v += y[(size_t)i * total + gid];
        tmp[gid] = v;
    }
}

static int lookup_n(slz_ctx *ctx, size_t chunk, size_t n1, const uint64_t *in, const uint64_t *luts, const uint32_t *idx, uint32_t n_luts,
                    const void *bskp, const uint64_t *ksk, uint64_t *big, uint64_t *out, size_t count, void *stream) {
    for (size_t c0 = 0; c0 < count; c0 += chunk) {
        const uint32_t nb = (uint32_t)(count - c0 < chunk ? count - c0 : chunk);
        int rc = slz_pbs_batch(ctx, in + c0 * n1, luts, idx ? idx + c0 : nullptr, n_luts, bskp, big, nb, stream);
        if (rc != SLZ_OK) return rc;
        rc = slz_keyswitch_batch(ctx, big, ksk, out + c0 * n1, nb, stream);
        if (rc != SLZ_OK) return rc;
    }
    return SLZ_OK;
}

static int rns_args_ok(slz_ctx *ctx, const slz_rns_shape *sh, const void *x, const void *luts, const void *bskp, const void *ksk,
                       const void *out, const void *ws) {
    if (!ctx || !x || !luts || !bskp || !ksk || !out || !ws || !rns_shape_ok(&ctx->prm, sh)) return 0;
    return !(((uintptr_t)ws & 255u) || ((uintptr_t)x & 7u) || ((uintptr_t)out & 7u) || ((uintptr_t)luts & 15u));
}

// digits into y (which already holds the residues): k - 1 dependent rounds
static int rns2mrns_inplace(slz_ctx *ctx, const slz_rns_shape *sh, const rns_plan &P, uint64_t *y, const uint64_t *luts, const void *bskp,
                            const uint64_t *ksk, char *ws, void *hip_stream) {
    hipStream_t s = (hipStream_t)hip_stream;
    uint32_t *idx = (uint32_t *)(ws + P.o_idx);
    uint64_t *big = (uint64_t *)(ws + P.o_big), *tmp = (uint64_t *)(ws + P.o_tmp);
    const uint32_t k = sh->k, n1 = (uint32_t)P.n1, n_conv = k * (k - 1) / 2;
    const size_t count = sh->count;
    const uint64_t offset_body = (uint64_t)RNS_OFFSET << (63 - ctx->prm.msg_bits);
    for (uint32_t i = 1; i < k; i++) {
        const size_t cts = (size_t)(k - i) * count;
        hipLaunchKernelGGL(k_rns_diff, ew_grid(cts * n1), dim3(MR_THREADS), 0, s, y, tmp, idx, k, i, count, n1, offset_body,
                           pair_index(k, i - 1, i));
        int rc = lookup_n(ctx, P.chunk, P.n1, tmp, luts, idx, n_conv, bskp, ksk, big, y + (size_t)i * count * n1, cts, hip_stream);
        if (rc != SLZ_OK) return rc;
    }
    return SLZ_OK;
}

extern "C" int slz_rns2mrns(slz_ctx *ctx, const slz_rns_shape *sh, const uint64_t *x, const uint64_t *luts, const void *bskp,
                            const uint64_t *ksk, uint64_t *y, void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!rns_args_ok(ctx, sh, x, luts, bskp, ksk, y, workspace)) return SLZ_E_INVALID_ARG;
    const rns_plan P = make_rns_plan(ctx, sh);
    if (workspace_bytes < P.total) return SLZ_E_INVALID_ARG;
    SLZ_HIP(hipMemcpyAsync(y, x, P.total_cts * P.n1 * 8, hipMemcpyDeviceToDevice, (hipStream_t)hip_stream));
    int rc = rns2mrns_inplace(ctx, sh, P, y, luts, bskp, ksk, (char *)workspace, hip_stream);
    if (rc != SLZ_OK) return rc;
    SLZ_HIP(hipGetLastError());
    return SLZ_OK;
}

extern "C" int slz_sign_rns(slz_ctx *ctx, const slz_rns_shape *sh, const uint64_t *x, const uint64_t *luts, const void *bskp,
                            const uint64_t *ksk, uint64_t *out, void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!rns_args_ok(ctx, sh, x, luts, bskp, ksk, out, workspace)) return SLZ_E_INVALID_ARG;
    if (sh->m[sh->k - 1] % 2) return SLZ_E_INVALID_ARG;
    const rns_plan P = make_rns_plan(ctx, sh);
    if (workspace_bytes < P.total) return SLZ_E_INVALID_ARG;
    hipStream_t s = (hipStream_t)hip_stream;
    char *ws = (char *)workspace;
    uint64_t *y = (uint64_t *)(ws + P.o_y), *neg = (uint64_t *)(ws + P.o_neg), *tmp = (uint64_t *)(ws + P.o_tmp);
    uint64_t *big = (uint64_t *)(ws + P.o_big);
    const uint32_t k = sh->k, n1 = (uint32_t)P.n1, n_conv = k * (k - 1) / 2;
    const size_t count = sh->count, N = ctx->prm.N;
    SLZ_HIP(hipMemcpyAsync(y, x, P.total_cts * P.n1 * 8, hipMemcpyDeviceToDevice, s));
    int rc = rns2mrns_inplace(ctx, sh, P, y, luts, bskp, ksk, ws, hip_stream);
    if (rc != SLZ_OK) return rc;
    // negative iff the top digit is in the upper half of its radix
    rc = lookup_n(ctx, P.chunk, P.n1, y + (size_t)(k - 1) * count * n1, luts + (size_t)n_conv * N, nullptr, 1, bskp, ksk, big, neg, count,
                  hip_stream);
    if (rc != SLZ_OK) return rc;
    hipLaunchKernelGGL(k_rns_sign_pack, ew_grid(count * n1), dim3(MR_THREADS), 0, s, y, neg, tmp, k, count, n1);
    rc = lookup_n(ctx, P.chunk, P.n1, tmp, luts + (size_t)(n_conv + 1) * N, nullptr, 1, bskp, ksk, big, out, count, hip_stream);
    if (rc != SLZ_OK) return rc;
    SLZ_HIP(hipGetLastError());
    return SLZ_OK;
}
