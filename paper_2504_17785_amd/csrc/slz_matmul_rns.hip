// Matmul^RNS (the paper's Algorithm "Matmul^RNS") on LWE ciphertexts: three rounds of table lookups
// (slz_pbs_batch + slz_keyswitch_batch) joined by element-wise kernels on ciphertext vectors.
#include "slz_gadget_util.h"
#include "../../include/silenzio_gadgets.h"
#include <vector>

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
__global__ void k_mr_weights(int32_t *wts, uint32_t b, uint32_t nblk, uint32_t block) {
    const uint32_t gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (gid < b * nblk) wts[gid] = (gid / nblk) / block == gid % nblk ? 1 : 0;
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

static int lookup(slz_ctx *ctx, const mr_plan &P, const uint64_t *in, const uint64_t *luts, const uint32_t *idx, uint32_t n_luts,
                  const void *bskp, const uint64_t *ksk, uint64_t *big, uint64_t *out, size_t count, void *stream) {
    return lookup_n(ctx, P.chunk, P.n1, in, luts, idx, n_luts, bskp, ksk, big, out, count, stream);
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
    hipLaunchKernelGGL(k_mr_weights, dim3((b * (uint32_t)P.nblk + 255) / 256), dim3(256), 0, s, wts, b, (uint32_t)P.nblk,
                       (uint32_t)SLZ_MATMUL_RNS_BLOCK);
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

// ---- MatmulHighRes^RNS (the paper's Algorithm of that name): 5-bit moduli, every intermediate within 8 bits --------------------
static bool highres_shape_ok(const slz_params *p, const slz_matmul_rns_shape *sh) {
    if (!p || !sh || sh->k == 0 || sh->k > SLZ_MATMUL_RNS_MAX_K || sh->a == 0 || sh->b == 0 || sh->c == 0) return false;
    if (p->msg_bits < 8) return false;
    for (uint32_t i = 0; i < sh->k; i++)
        if (sh->m[i] < 2 || sh->m[i] > 32) return false;
    const uint64_t prods = (uint64_t)sh->k * sh->a * sh->b * sh->c;
    return prods < (1ull << 31) && (uint64_t)sh->k * ((uint64_t)sh->a * sh->b + (uint64_t)sh->b * sh->c) < (1ull << 31);
}

extern "C" int slz_matmul_highres_luts(const slz_params *p, const slz_matmul_rns_shape *sh, uint64_t *luts_out) {
    if (!luts_out || !highres_shape_ok(p, sh)) return SLZ_E_INVALID_ARG;
    const uint64_t t = 1ull << p->msg_bits;
    const uint32_t k = sh->k;
    std::vector<uint64_t> tab((size_t)(4 * k + 3) * t, 0);
    for (uint64_t v = 0; v < t; v++) {
        const int64_t sv = v < t / 2 ? (int64_t)v : (int64_t)v - (int64_t)t;
        const uint64_t prod = v < 256 ? (v >> 5) * (v & 31) : 0;
        for (uint32_t i = 0; i < k; i++) {
            const int64_t q = sh->m[i];
            tab[(size_t)i * t + v] = (uint64_t)(((sv % q) + q) % q);
            tab[(size_t)(k + i) * t + v] = prod % (uint64_t)q;
            tab[(size_t)(2 * k + i) * t + v] = (8 * v) % (uint64_t)q;
            tab[(size_t)(3 * k + i) * t + v] = v % (uint64_t)q;
        }
        tab[(size_t)(4 * k) * t + v] = (v >> 3) & 3;
        tab[(size_t)(4 * k + 1) * t + v] = v & 7;
        tab[(size_t)(4 * k + 2) * t + v] = prod;
    }
    return slz_lut_encode(p, tab.data(), 4 * k + 3, luts_out);
}

struct hr_plan {
    size_t n1, N1, n_in, n_x, n_prod, n_out, nblk, chunk;
    size_t o_rep, o_idx, o_big, o_res, o_x1, o_x2, o_pk, o_y1, o_y2, o_sums, o_wts, o_tmp, total;
};

static hr_plan make_hr_plan(const slz_ctx *ctx, const slz_matmul_rns_shape *sh) {
    hr_plan P;
    P.n1 = ctx->prm.n + 1;
    P.N1 = (size_t)ctx->prm.k * ctx->prm.N + 1;
    P.n_in = (size_t)sh->k * ((size_t)sh->a * sh->b + (size_t)sh->b * sh->c);
    P.n_x = (size_t)sh->k * sh->a * sh->b;
    P.n_prod = (size_t)sh->k * sh->a * sh->b * sh->c;
    P.n_out = (size_t)sh->k * sh->a * sh->c;
    P.nblk = (sh->b + SLZ_MATMUL_HIGHRES_BLOCK - 1) / SLZ_MATMUL_HIGHRES_BLOCK;
    const size_t biggest = P.n_in > P.n_prod ? P.n_in : P.n_prod;
    P.chunk = biggest < ctx->max_batch ? biggest : ctx->max_batch;
    size_t o = 0;
    P.o_rep = o;  o += up256(P.n_in * P.n1 * 8);              // step 1 inputs, one copy per modulus
    P.o_idx = o;  o += up256(biggest * 4);                    // table index per ciphertext of the current lookup
    P.o_big = o;  o += up256(P.chunk * P.N1 * 8);             // bootstrapping outputs of one chunk
    P.o_res = o;  o += up256(P.n_in * P.n1 * 8);              // X', W'
    P.o_x1 = o;   o += up256(P.n_x * P.n1 * 8);               // bits 0..2 of X'
    P.o_x2 = o;   o += up256(P.n_x * P.n1 * 8);               // bits 3..4 of X'
    P.o_pk = o;   o += up256(P.n_prod * P.n1 * 8);            // packed inputs of the product lookups, [k][a][c][b]
    P.o_y1 = o;   o += up256(P.n_prod * P.n1 * 8);            // Y1*, later Y*
    P.o_y2 = o;   o += up256(P.n_prod * P.n1 * 8);            // Y2*
    P.o_sums = o; o += up256(P.n_out * P.nblk * P.n1 * 8);
    P.o_wts = o;  o += up256((size_t)sh->b * P.nblk * 4);
    P.o_tmp = o;  o += up256(P.n_out * P.n1 * 8);
    P.total = o;
    return P;
}

extern "C" int slz_matmul_highres_workspace(const slz_ctx *ctx, const slz_matmul_rns_shape *sh, size_t *bytes) {
    if (!ctx || !bytes || !highres_shape_ok(&ctx->prm, sh)) return SLZ_E_INVALID_ARG;
    *bytes = make_hr_plan(ctx, sh).total;
    return SLZ_OK;
}

// packed[i][r][s][j][.] = 32 xs[i][r][j][.] + res[i][a b + j c + s][.];  idx[...] = idx_base + i.   xs = [k][a b][n1], res = [k][ab + bc][n1]
__global__ void __launch_bounds__(MR_THREADS)
k_hr_pack(const uint64_t *__restrict__ xs, const uint64_t *__restrict__ res, uint64_t *__restrict__ packed, uint32_t *__restrict__ idx,
          uint32_t idx_base, uint32_t k, uint32_t a, uint32_t b, uint32_t c, uint32_t n1) {
    const size_t per = (size_t)a * b + (size_t)b * c;
    const size_t total = (size_t)k * a * c * b * n1;
    for (size_t gid = (size_t)blockIdx.x * MR_THREADS + threadIdx.x; gid < total; gid += (size_t)gridDim.x * MR_THREADS) {
        const uint32_t word = (uint32_t)(gid % n1);
        size_t ct = gid / n1;
        const uint32_t j = (uint32_t)(ct % b);
        const uint32_t s = (uint32_t)((ct / b) % c);
        const uint32_t r = (uint32_t)((ct / ((size_t)b * c)) % a);
        const uint32_t i = (uint32_t)(ct / ((size_t)a * b * c));
        const uint64_t xv = xs[(((size_t)i * a + r) * b + j) * n1 + word];
        const uint64_t wv = res[((size_t)i * per + (size_t)a * b + (size_t)j * c + s) * n1 + word];
        packed[gid] = 32ull * xv + wv;
        if (word == 0) idx[ct] = idx_base + i;
    }
}

// out = x + y on `total` words;  idx[ct] = idx_base + ct / per_mod
__global__ void __launch_bounds__(MR_THREADS)
k_hr_add(const uint64_t *__restrict__ x, const uint64_t *__restrict__ y, uint64_t *__restrict__ out, uint32_t *__restrict__ idx,
         uint32_t idx_base, size_t per_mod, size_t cts, uint32_t n1) {
    const size_t total = cts * n1;
    for (size_t gid = (size_t)blockIdx.x * MR_THREADS + threadIdx.x; gid < total; gid += (size_t)gridDim.x * MR_THREADS) {
        out[gid] = x[gid] + y[gid];
        if (gid % n1 == 0) idx[gid / n1] = idx_base + (uint32_t)((gid / n1) / per_mod);
    }
}

extern "C" int slz_matmul_highres(slz_ctx *ctx, const slz_matmul_rns_shape *sh, const uint64_t *x, const uint64_t *w, const uint64_t *luts,
                                  const void *bskp, const uint64_t *ksk, uint64_t *y, void *workspace, size_t workspace_bytes,
                                  void *hip_stream) {
    if (!ctx || !x || !w || !luts || !bskp || !ksk || !y || !workspace || !highres_shape_ok(&ctx->prm, sh)) return SLZ_E_INVALID_ARG;
    if (((uintptr_t)workspace & 255u) || ((uintptr_t)x & 7u) || ((uintptr_t)w & 7u) || ((uintptr_t)y & 7u) || ((uintptr_t)luts & 15u))
        return SLZ_E_INVALID_ARG;
    const hr_plan P = make_hr_plan(ctx, sh);
    if (workspace_bytes < P.total) return SLZ_E_INVALID_ARG;
    hipStream_t s = (hipStream_t)hip_stream;
    char *ws = (char *)workspace;
    uint64_t *rep = (uint64_t *)(ws + P.o_rep), *big = (uint64_t *)(ws + P.o_big), *res = (uint64_t *)(ws + P.o_res);
    uint64_t *x1 = (uint64_t *)(ws + P.o_x1), *x2 = (uint64_t *)(ws + P.o_x2), *pk = (uint64_t *)(ws + P.o_pk);
    uint64_t *y1 = (uint64_t *)(ws + P.o_y1), *y2 = (uint64_t *)(ws + P.o_y2), *sums = (uint64_t *)(ws + P.o_sums);
    uint64_t *tmp = (uint64_t *)(ws + P.o_tmp);
    uint32_t *idx = (uint32_t *)(ws + P.o_idx);
    int32_t *wts = (int32_t *)(ws + P.o_wts);
    const uint32_t k = sh->k, a = sh->a, b = sh->b, c = sh->c, n1 = (uint32_t)P.n1, n_tabs = 4 * k + 3;
    const size_t N = ctx->prm.N, ab = (size_t)a * b, per = ab + (size_t)b * c;
    auto look = [&](const uint64_t *in, const uint32_t *ix, uint64_t *out, size_t count) {
        return lookup_n(ctx, P.chunk, P.n1, in, luts, ix, n_tabs, bskp, ksk, big, out, count, hip_stream);
    };
    auto look1 = [&](const uint64_t *in, uint32_t table, uint64_t *out, size_t count) {
        return lookup_n(ctx, P.chunk, P.n1, in, luts + (size_t)table * N, nullptr, 1, bskp, ksk, big, out, count, hip_stream);
    };
    // Step 1: X' = X mod m', W' = W mod m'
    hipLaunchKernelGGL(k_mr_replicate, ew_grid(P.n_in * n1), dim3(MR_THREADS), 0, s, x, w, rep, idx, k, ab, (size_t)b * c, n1);
    int rc = look(rep, idx, res, P.n_in);
    if (rc != SLZ_OK) return rc;
    // Step 2: the bit chunks of X' (the X' of modulus i are the first a b ciphertexts of its slice of res)
    for (uint32_t i = 0; i < k; i++) {
        rc = look1(res + (size_t)i * per * n1, 4 * k, x2 + (size_t)i * ab * n1, ab);
        if (rc != SLZ_OK) return rc;
        rc = look1(res + (size_t)i * per * n1, 4 * k + 1, x1 + (size_t)i * ab * n1, ab);
        if (rc != SLZ_OK) return rc;
    }
    // Step 3: Y1* = X1' W' mod m'' on 32 x1 + w;  Y2* = X2' W' on 32 x2 + w, then v -> 8 v mod m''
    hipLaunchKernelGGL(k_hr_pack, ew_grid(P.n_prod * n1), dim3(MR_THREADS), 0, s, x1, res, pk, idx, k, k, a, b, c, n1);
    rc = look(pk, idx, y1, P.n_prod);
    if (rc != SLZ_OK) return rc;
    hipLaunchKernelGGL(k_hr_pack, ew_grid(P.n_prod * n1), dim3(MR_THREADS), 0, s, x2, res, pk, idx, 2 * k, k, a, b, c, n1);
    rc = look1(pk, 4 * k + 2, y2, P.n_prod);
    if (rc != SLZ_OK) return rc;
    rc = look(y2, idx, y2, P.n_prod);          // in place: each chunk is read before it is written
    if (rc != SLZ_OK) return rc;
    // Step 4: Y* = (Y1* + Y2*) mod m''
    hipLaunchKernelGGL(k_hr_add, ew_grid(P.n_prod * n1), dim3(MR_THREADS), 0, s, y1, y2, pk, idx, 3 * k, (size_t)a * b * c, P.n_prod, n1);
    rc = look(pk, idx, y1, P.n_prod);
    if (rc != SLZ_OK) return rc;
    // Step 5: sums of at most 7 entries per block, the running sum reduced by one lookup per block
    hipLaunchKernelGGL(k_mr_weights, dim3((b * (uint32_t)P.nblk + 255) / 256), dim3(256), 0, s, wts, b, (uint32_t)P.nblk,
                       (uint32_t)SLZ_MATMUL_HIGHRES_BLOCK);
    for (size_t g0 = 0; g0 < P.n_out; g0 += 65535) {
        const uint32_t ng = (uint32_t)(P.n_out - g0 < 65535 ? P.n_out - g0 : 65535);
        rc = slz_lwe_lincomb_batch(ctx, y1 + g0 * b * n1, wts, sums + g0 * P.nblk * n1, ng, b, (uint32_t)P.nblk, hip_stream);
        if (rc != SLZ_OK) return rc;
    }
    for (uint32_t t = 0; t < P.nblk; t++) {
        hipLaunchKernelGGL(k_mr_accumulate, ew_grid(P.n_out * n1), dim3(MR_THREADS), 0, s, y, sums, tmp, idx, P.n_out, a * c,
                           (uint32_t)P.nblk, t, n1);
        rc = lookup_n(ctx, P.chunk, P.n1, tmp, luts + (size_t)3 * k * N, idx, k, bskp, ksk, big, y, P.n_out, hip_stream);
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

// conversion tables and the two sign tables, appended to tab
static void rns_tables(const slz_params *p, const slz_rns_shape *sh, int32_t neg, int32_t zero, int32_t pos, std::vector<uint64_t> &out) {
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
    out.insert(out.end(), tab.begin(), tab.end());
}

extern "C" int slz_rns_luts(const slz_params *p, const slz_rns_shape *sh, int32_t neg, int32_t zero, int32_t pos, uint64_t *luts_out) {
    if (!luts_out || !rns_shape_ok(p, sh)) return SLZ_E_INVALID_ARG;
    if (neg < -128 || neg > 127 || zero < -128 || zero > 127 || pos < -128 || pos > 127) return SLZ_E_INVALID_ARG;
    std::vector<uint64_t> tab;
    rns_tables(p, sh, neg, zero, pos, tab);
    return slz_lut_encode(p, tab.data(), sh->k * (sh->k - 1) / 2 + 2, luts_out);
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

// sign of count numbers: residues x -> out; uses the plan's y, neg, tmp, big, idx buffers
static int sign_rns_run(slz_ctx *ctx, const slz_rns_shape *sh, const rns_plan &P, const uint64_t *x, const uint64_t *luts, const void *bskp,
                        const uint64_t *ksk, uint64_t *out, char *ws, void *hip_stream) {
    hipStream_t s = (hipStream_t)hip_stream;
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
    return lookup_n(ctx, P.chunk, P.n1, tmp, luts + (size_t)(n_conv + 1) * N, nullptr, 1, bskp, ksk, big, out, count, hip_stream);
}

extern "C" int slz_sign_rns(slz_ctx *ctx, const slz_rns_shape *sh, const uint64_t *x, const uint64_t *luts, const void *bskp,
                            const uint64_t *ksk, uint64_t *out, void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!rns_args_ok(ctx, sh, x, luts, bskp, ksk, out, workspace)) return SLZ_E_INVALID_ARG;
    if (sh->m[sh->k - 1] % 2) return SLZ_E_INVALID_ARG;
    const rns_plan P = make_rns_plan(ctx, sh);
    if (workspace_bytes < P.total) return SLZ_E_INVALID_ARG;
    int rc = sign_rns_run(ctx, sh, P, x, luts, bskp, ksk, out, (char *)workspace, hip_stream);
    if (rc != SLZ_OK) return rc;
    SLZ_HIP(hipGetLastError());
    return SLZ_OK;
}

// ---- Shift2MSBs^+ and Shift2MSBs^+- ----------------------------------------------------------------------------------
#define MAX_OFFSET 32u      // moves a difference of two bit positions (each at most 24) into the non-negative range

static bool shift_shape_ok(const slz_params *p, const slz_shift_shape *sh, slz_rns_shape *rs) {
    if (!p || !sh) return false;
    rs->k = sh->k; rs->count = sh->count;
    for (int i = 0; i < SLZ_MATMUL_RNS_MAX_K; i++) rs->m[i] = sh->m[i];
    if (!rns_shape_ok(p, rs)) return false;
    if (sh->w != 4 || sh->gamma < 1 || sh->gamma > 7 || sh->k > 6) return false;      // 4-bit digits; outputs and positions fit the tables
    return true;
}

static uint32_t bit_position(uint64_t x) { uint32_t b = 0; while (x) { b++; x >>= 1; } return b; }

static uint64_t shift_code(uint64_t max_bit, uint32_t i, uint32_t w, uint32_t gamma) {
    const int64_t any_shift = max_bit > w ? 1 : 0;
    const int64_t digit_shift = ((int64_t)gamma - ((int64_t)max_bit - (int64_t)(w * i))) * any_shift;
    if (digit_shift >= 0) return (uint64_t)(digit_shift < (int64_t)gamma - 1 ? digit_shift : (int64_t)gamma - 1);
    const int64_t r = -digit_shift;
    return 8 + (uint64_t)(r < (int64_t)w ? r : (int64_t)w);
}

// table counts: conversion + sign (k (k-1) / 2 + 2), shift (2k + 2), signed variant (k + 1)
static uint32_t shift_n_luts(uint32_t k) { return k * (k - 1) / 2 + 2 + 2 * k + 2 + k + 1; }

extern "C" int slz_shift2msbs_luts(const slz_params *p, const slz_shift_shape *sh, uint64_t *luts_out) {
    slz_rns_shape rs;
    if (!luts_out || !shift_shape_ok(p, sh, &rs)) return SLZ_E_INVALID_ARG;
    const uint64_t t = 1ull << p->msg_bits;
    const uint32_t k = sh->k, w = sh->w, gamma = sh->gamma;
    std::vector<uint64_t> tab;
    rns_tables(p, &rs, 1, 0, 0, tab);                          // the sign as the flag [x < 0]
    std::vector<uint64_t> row(t);
    for (uint32_t i = 0; i < k; i++) {                          // digit -> 1-indexed position of its highest set bit (+ i w), 0 for 0
        for (uint64_t v = 0; v < t; v++) row[v] = (v > 0 && v < 16) ? bit_position(v) + i * w : 0;
        tab.insert(tab.end(), row.begin(), row.end());
    }
    for (uint64_t v = 0; v < t; v++) row[v] = (v < 2 * MAX_OFFSET && v > MAX_OFFSET) ? v - MAX_OFFSET : 0;     // a - b + 32 -> ReLU(a - b)
    tab.insert(tab.end(), row.begin(), row.end());
    for (uint32_t i = 0; i < k; i++) {                          // maxBit -> shift code of digit i
        for (uint64_t v = 0; v < t; v++) row[v] = v <= (uint64_t)k * w ? shift_code(v, i, w, gamma) : 0;
        tab.insert(tab.end(), row.begin(), row.end());
    }
    for (uint64_t v = 0; v < t; v++) {                          // 16 code + digit -> shifted digit
        uint64_t r = 0;
        if (v < 256) {
            const uint64_t code = v >> 4, x = v & 15;
            r = code < 8 ? x << (code < 7 ? code : 7) : x >> (code - 8);
        }
        row[v] = r % t;
    }
    tab.insert(tab.end(), row.begin(), row.end());
    for (uint32_t i = 0; i < k; i++) {                          // 16 flag + residue -> |x| mod m_i
        const uint64_t q = sh->m[i];
        for (uint64_t v = 0; v < t; v++) row[v] = v < 16 ? v % q : (v < 32 ? (q - (v - 16) % q) % q : 0);
        tab.insert(tab.end(), row.begin(), row.end());
    }
    for (uint64_t v = 0; v < t; v++) row[v] = v < 128 ? v : (t - (v - 128)) % t;      // 128 flag + y -> s y, signed in Z_t
    tab.insert(tab.end(), row.begin(), row.end());
    return slz_lut_encode(p, tab.data(), shift_n_luts(k), luts_out);
}

struct shift_plan {
    rns_plan R;             // buffers of the conversion and the sign
    size_t o_u, o_u2, o_maxbit, o_codes, o_ys, o_xp, o_yp, o_flag, total;
};

static shift_plan make_shift_plan(const slz_ctx *ctx, const slz_rns_shape *rs) {
    shift_plan S;
    S.R = make_rns_plan(ctx, rs);
    const size_t n1 = S.R.n1, all = S.R.total_cts;
    size_t o = S.R.total;
    S.o_u = o;      o += up256(all * n1 * 8);                   // bit positions; levels of the maximum tree alternate u / u2
    S.o_u2 = o;     o += up256(all * n1 * 8);
    S.o_maxbit = o; o += up256(n1 * 8);
    S.o_codes = o;  o += up256((size_t)rs->k * n1 * 8);
    S.o_ys = o;     o += up256(all * n1 * 8);                   // shifted digits
    S.o_xp = o;     o += up256(all * n1 * 8);                   // |x| in RNS (signed variant)
    S.o_yp = o;     o += up256((size_t)rs->count * n1 * 8);     // Y^+ (signed variant)
    S.o_flag = o;   o += up256((size_t)rs->count * n1 * 8);     // [x < 0] (signed variant)
    S.total = o;
    return S;
}

extern "C" int slz_shift2msbs_workspace(const slz_ctx *ctx, const slz_shift_shape *sh, size_t *bytes) {
    slz_rns_shape rs;
    if (!ctx || !bytes || !shift_shape_ok(&ctx->prm, sh, &rs)) return SLZ_E_INVALID_ARG;
    *bytes = make_shift_plan(ctx, &rs).total;
    return SLZ_OK;
}

// idx[i * count + e] = i
__global__ void k_sh_row_index(uint32_t *idx, uint32_t k, size_t count) {
    const size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid < (size_t)k * count) idx[gid] = (uint32_t)(gid / count);
}

// tmp[j][.] = cur[2j][.] - cur[2j+1][.] + 32 (on the body), j < h
__global__ void __launch_bounds__(MR_THREADS)
k_sh_pair_diff(const uint64_t *__restrict__ cur, uint64_t *__restrict__ tmp, size_t h, uint32_t n1, uint64_t offset_body) {
    const size_t total = h * n1;
    for (size_t gid = (size_t)blockIdx.x * MR_THREADS + threadIdx.x; gid < total; gid += (size_t)gridDim.x * MR_THREADS) {
        const uint32_t word = (uint32_t)(gid % n1);
        const size_t j = gid / n1;
        uint64_t v = cur[(2 * j) * n1 + word] - cur[(2 * j + 1) * n1 + word];
        if (word == n1 - 1) v += offset_body;
        tmp[gid] = v;
    }
}

// nxt[j] = cur[2j+1] + d[j] for j < h; an odd last element of cur passes through as nxt[h]
__global__ void __launch_bounds__(MR_THREADS)
k_sh_pair_max(const uint64_t *__restrict__ cur, const uint64_t *__restrict__ d, uint64_t *__restrict__ nxt, size_t h, size_t n_cur, uint32_t n1) {
    const size_t n_next = h + (n_cur & 1);
    const size_t total = n_next * n1;
    for (size_t gid = (size_t)blockIdx.x * MR_THREADS + threadIdx.x; gid < total; gid += (size_t)gridDim.x * MR_THREADS) {
        const uint32_t word = (uint32_t)(gid % n1);
        const size_t j = gid / n1;
        nxt[gid] = j < h ? cur[(2 * j + 1) * n1 + word] + d[gid] : cur[(n_cur - 1) * n1 + word];
    }
}

// tmp[i][.] = src[.] for i < k;  idx[i] = i
__global__ void k_sh_broadcast(const uint64_t *__restrict__ src, uint64_t *__restrict__ tmp, uint32_t *__restrict__ idx, uint32_t k, uint32_t n1) {
    const uint32_t gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (gid < k * n1) tmp[gid] = src[gid % n1];
    if (gid < k) idx[gid] = gid;
}

// tmp[i][e][.] = mul * a[i or 0][.] (a per row when a_per_row, else per element e) + b[i][e][.]
// mode 0: a = codes[i] (one ciphertext per row);  mode 1: a = flag[e] (one per element)
__global__ void __launch_bounds__(MR_THREADS)
k_sh_pack(const uint64_t *__restrict__ a, const uint64_t *__restrict__ b, uint64_t *__restrict__ tmp, uint32_t k, size_t count, uint32_t n1,
          uint64_t mul, int mode) {
    const size_t total = (size_t)k * count * n1;
    for (size_t gid = (size_t)blockIdx.x * MR_THREADS + threadIdx.x; gid < total; gid += (size_t)gridDim.x * MR_THREADS) {
        const uint32_t word = (uint32_t)(gid % n1);
        const size_t ct = gid / n1;
        const size_t e = ct % count, i = ct / count;
        const uint64_t av = mode == 0 ? a[i * n1 + word] : a[e * n1 + word];
        tmp[gid] = mul * av + b[gid];
    }
}

// Y[e][.] = sum_i ys[i][e][.];  shift[.] = maxbit[.] - gamma (on the body)
__global__ void __launch_bounds__(MR_THREADS)
k_sh_sum(const uint64_t *__restrict__ ys, const uint64_t *__restrict__ maxbit, uint64_t *__restrict__ Y, uint64_t *__restrict__ shift, uint32_t k,
         size_t count, uint32_t n1, uint64_t gamma_body) {
    const size_t total = count * n1;
    for (size_t gid = (size_t)blockIdx.x * MR_THREADS + threadIdx.x; gid < total; gid += (size_t)gridDim.x * MR_THREADS) {
        uint64_t v = 0;
        for (uint32_t i = 0; i < k; i++) v += ys[(size_t)i * total + gid];
        Y[gid] = v;
        if (gid < n1) shift[gid] = maxbit[gid] - (gid == n1 - 1 ? gamma_body : 0);
    }
}

// Shift2MSBs^+ of the residues in x (device, k x count) -> Y, shift
static int shift_plus_run(slz_ctx *ctx, const slz_shift_shape *sh, const slz_rns_shape *rs, const shift_plan &S, const uint64_t *x,
                          const uint64_t *luts, const void *bskp, const uint64_t *ksk, uint64_t *Y, uint64_t *shift, char *ws, void *hip_stream) {
    hipStream_t s = (hipStream_t)hip_stream;
    const rns_plan &P = S.R;
    const uint32_t k = rs->k, n1 = (uint32_t)P.n1, n_conv = k * (k - 1) / 2;
    const size_t count = rs->count, all = P.total_cts, N = ctx->prm.N;
    uint32_t *idx = (uint32_t *)(ws + P.o_idx);
    uint64_t *big = (uint64_t *)(ws + P.o_big), *tmp = (uint64_t *)(ws + P.o_tmp), *y = (uint64_t *)(ws + P.o_y);
    uint64_t *u = (uint64_t *)(ws + S.o_u), *u2 = (uint64_t *)(ws + S.o_u2), *maxbit = (uint64_t *)(ws + S.o_maxbit);
    uint64_t *codes = (uint64_t *)(ws + S.o_codes), *ys = (uint64_t *)(ws + S.o_ys);
    const uint64_t *t_pos = luts + (size_t)(n_conv + 2) * N, *t_relu = t_pos + (size_t)k * N, *t_code = t_relu + N, *t_apply = t_code + (size_t)k * N;
    const uint32_t delta_shift = 63 - ctx->prm.msg_bits;
    // Step 1: digits
    SLZ_HIP(hipMemcpyAsync(y, x, all * n1 * 8, hipMemcpyDeviceToDevice, s));
    int rc = rns2mrns_inplace(ctx, rs, P, y, luts, bskp, ksk, ws, hip_stream);
    if (rc != SLZ_OK) return rc;
    // Step 2: position of the highest set bit of every digit, then the maximum over everything
    hipLaunchKernelGGL(k_sh_row_index, dim3((unsigned)((all + 255) / 256)), dim3(256), 0, s, idx, k, count);
    rc = lookup_n(ctx, P.chunk, P.n1, y, t_pos, idx, k, bskp, ksk, big, u, all, hip_stream);
    if (rc != SLZ_OK) return rc;
    uint64_t *cur = u, *nxt = u2;
    for (size_t n_cur = all; n_cur > 1;) {
        const size_t h = n_cur / 2;
        hipLaunchKernelGGL(k_sh_pair_diff, ew_grid(h * n1), dim3(MR_THREADS), 0, s, cur, tmp, h, n1, (uint64_t)MAX_OFFSET << delta_shift);
        rc = lookup_n(ctx, P.chunk, P.n1, tmp, t_relu, nullptr, 1, bskp, ksk, big, ys, h, hip_stream);      // ys is free until step 4
        if (rc != SLZ_OK) return rc;
        hipLaunchKernelGGL(k_sh_pair_max, ew_grid((h + 1) * n1), dim3(MR_THREADS), 0, s, cur, ys, nxt, h, n_cur, n1);
        uint64_t *sw = cur; cur = nxt; nxt = sw;
        n_cur = h + (n_cur & 1);
    }
    SLZ_HIP(hipMemcpyAsync(maxbit, cur, (size_t)n1 * 8, hipMemcpyDeviceToDevice, s));
    // Step 3: shift code per digit position
    hipLaunchKernelGGL(k_sh_broadcast, dim3((k * n1 + 255) / 256), dim3(256), 0, s, maxbit, tmp, idx, k, n1);
    rc = lookup_n(ctx, P.chunk, P.n1, tmp, t_code, idx, k, bskp, ksk, big, codes, k, hip_stream);
    if (rc != SLZ_OK) return rc;
    // Step 4: apply the shifts
    hipLaunchKernelGGL(k_sh_pack, ew_grid(all * n1), dim3(MR_THREADS), 0, s, codes, y, tmp, k, count, n1, (uint64_t)16, 0);
    rc = lookup_n(ctx, P.chunk, P.n1, tmp, t_apply, nullptr, 1, bskp, ksk, big, ys, all, hip_stream);
    if (rc != SLZ_OK) return rc;
    // Step 5: sum over the digits, Step 6: shift = maxBit - gamma
    hipLaunchKernelGGL(k_sh_sum, ew_grid(count * n1 > n1 ? count * n1 : n1), dim3(MR_THREADS), 0, s, ys, maxbit, Y, shift, k, count, n1,
                       (uint64_t)sh->gamma << delta_shift);
    return SLZ_OK;
}

static int shift_args_ok(slz_ctx *ctx, const slz_shift_shape *sh, slz_rns_shape *rs, const void *x, const void *luts, const void *bskp,
                         const void *ksk, const void *y, const void *shift, const void *ws) {
    if (!ctx || !x || !luts || !bskp || !ksk || !y || !shift || !ws || !shift_shape_ok(&ctx->prm, sh, rs)) return 0;
    return !(((uintptr_t)ws & 255u) || ((uintptr_t)x & 7u) || ((uintptr_t)y & 7u) || ((uintptr_t)shift & 7u) || ((uintptr_t)luts & 15u));
}

extern "C" int slz_shift2msbs_plus(slz_ctx *ctx, const slz_shift_shape *sh, const uint64_t *x, const uint64_t *luts, const void *bskp,
                                   const uint64_t *ksk, uint64_t *y, uint64_t *shift, void *workspace, size_t workspace_bytes, void *hip_stream) {
    slz_rns_shape rs;
    if (!shift_args_ok(ctx, sh, &rs, x, luts, bskp, ksk, y, shift, workspace)) return SLZ_E_INVALID_ARG;
    const shift_plan S = make_shift_plan(ctx, &rs);
    if (workspace_bytes < S.total) return SLZ_E_INVALID_ARG;
    int rc = shift_plus_run(ctx, sh, &rs, S, x, luts, bskp, ksk, y, shift, (char *)workspace, hip_stream);
    if (rc != SLZ_OK) return rc;
    SLZ_HIP(hipGetLastError());
    return SLZ_OK;
}

extern "C" int slz_shift2msbs_pm(slz_ctx *ctx, const slz_shift_shape *sh, const uint64_t *x, const uint64_t *luts, const void *bskp,
                                 const uint64_t *ksk, uint64_t *y, uint64_t *shift, void *workspace, size_t workspace_bytes, void *hip_stream) {
    slz_rns_shape rs;
    if (!shift_args_ok(ctx, sh, &rs, x, luts, bskp, ksk, y, shift, workspace)) return SLZ_E_INVALID_ARG;
    if (rs.m[rs.k - 1] % 2) return SLZ_E_INVALID_ARG;
    const shift_plan S = make_shift_plan(ctx, &rs);
    if (workspace_bytes < S.total) return SLZ_E_INVALID_ARG;
    hipStream_t s = (hipStream_t)hip_stream;
    char *ws = (char *)workspace;
    const rns_plan &P = S.R;
    const uint32_t k = rs.k, n1 = (uint32_t)P.n1, n_conv = k * (k - 1) / 2;
    const size_t count = rs.count, all = P.total_cts, N = ctx->prm.N;
    uint32_t *idx = (uint32_t *)(ws + P.o_idx);
    uint64_t *big = (uint64_t *)(ws + P.o_big), *tmp = (uint64_t *)(ws + P.o_tmp);
    uint64_t *xp = (uint64_t *)(ws + S.o_xp), *yp = (uint64_t *)(ws + S.o_yp), *flag = (uint64_t *)(ws + S.o_flag);
    const uint64_t *t_abs = luts + (size_t)(n_conv + 2 + 2 * k + 2) * N, *t_sign = t_abs + (size_t)k * N;
    // s = [x < 0] through the sign gadget
    int rc = sign_rns_run(ctx, &rs, P, x, luts, bskp, ksk, flag, ws, hip_stream);
    if (rc != SLZ_OK) return rc;
    // X^+ = s X mod m: a two-input lookup on 16 flag + residue
    hipLaunchKernelGGL(k_sh_pack, ew_grid(all * n1), dim3(MR_THREADS), 0, s, flag, x, tmp, k, count, n1, (uint64_t)16, 1);
    hipLaunchKernelGGL(k_sh_row_index, dim3((unsigned)((all + 255) / 256)), dim3(256), 0, s, idx, k, count);
    rc = lookup_n(ctx, P.chunk, P.n1, tmp, t_abs, idx, k, bskp, ksk, big, xp, all, hip_stream);
    if (rc != SLZ_OK) return rc;
    rc = shift_plus_run(ctx, sh, &rs, S, xp, luts, bskp, ksk, yp, shift, ws, hip_stream);
    if (rc != SLZ_OK) return rc;
    // Y = s Y^+: a two-input lookup on 128 flag + Y^+
    hipLaunchKernelGGL(k_sh_pack, ew_grid(count * n1), dim3(MR_THREADS), 0, s, flag, yp, tmp, 1u, count, n1, (uint64_t)128, 1);
    rc = lookup_n(ctx, P.chunk, P.n1, tmp, t_sign, nullptr, 1, bskp, ksk, big, y, count, hip_stream);
    if (rc != SLZ_OK) return rc;
    SLZ_HIP(hipGetLastError());
    return SLZ_OK;
}
