// Generic multi-kernel path: every step of the blind rotation as its own kernel over buffers in HBM.
// It works for every supported parameter set (any k, l, N up to 2^17) and is the path for shapes that
// have no fused kernel; it also prepares the bootstrapping key.  One CMux is
//   decompose (rotate, subtract, signed digits) -> forward transforms (2 primes) -> pointwise
//   multiply-accumulate with the prepared key -> inverse transforms -> CRT lift + accumulate.
#include "slz_internal.h"
#include "slz_modarith.h"

#define GEN_CH 2048u          // coefficients a workgroup transforms inside LDS
#define GEN_THREADS 256

// ---- accumulator initialisation, decomposition, extraction ---------------------------------

__global__ void __launch_bounds__(GEN_THREADS)
k_acc_init(const uint64_t *__restrict__ lwe_in, const uint64_t *__restrict__ luts, const uint32_t *__restrict__ lut_idx,
           uint64_t *__restrict__ acc, uint32_t n, uint32_t k, uint32_t N, uint32_t logN, uint32_t batch) {
    size_t gid = (size_t)blockIdx.x * GEN_THREADS + threadIdx.x;
    size_t total = (size_t)batch * (k + 1) * N;
    if (gid >= total) return;
    uint32_t x = (uint32_t)(gid % N);
    uint32_t c = (uint32_t)((gid / N) % (k + 1));
    uint32_t b = (uint32_t)(gid / ((size_t)N * (k + 1)));
    uint64_t v = 0;
    if (c == k) {
        uint32_t bt = slz_modswitch(lwe_in[(size_t)b * (n + 1) + n], logN + 1);
        uint32_t r = (2 * N - bt) & (2 * N - 1);
        const uint64_t *lut = luts + (size_t)(lut_idx ? lut_idx[b] : 0) * N;
        v = slz_rot_coeff([&](uint32_t j) { return lut[j]; }, x, r, N);
    }
    acc[gid] = v;
}

// dig[b][c*l + (j-1)][x] = d_j( (X^{a~} ACC_c - ACC_c)[x] ),  a~ = modswitch(lwe_in[b][step])
__global__ void __launch_bounds__(GEN_THREADS)
k_decompose(const uint64_t *__restrict__ acc, const uint64_t *__restrict__ lwe_in, uint32_t step, double *__restrict__ dig,
            uint32_t n, uint32_t k, uint32_t N, uint32_t logN, uint32_t beta, uint32_t l, uint32_t batch) {
    size_t gid = (size_t)blockIdx.x * GEN_THREADS + threadIdx.x;
    size_t total = (size_t)batch * (k + 1) * N;
    if (gid >= total) return;
    uint32_t x = (uint32_t)(gid % N);
    uint32_t c = (uint32_t)((gid / N) % (k + 1));
    uint32_t b = (uint32_t)(gid / ((size_t)N * (k + 1)));
    uint32_t at = slz_modswitch(lwe_in[(size_t)b * (n + 1) + step], logN + 1);
    const uint64_t *poly = acc + ((size_t)b * (k + 1) + c) * N;
    uint64_t lam = slz_rot_coeff([&](uint32_t j) { return poly[j]; }, x, at, N) - poly[x];
    uint64_t v = slz_round_top_bits(lam, beta * l);
    double *out = dig + ((size_t)b * (k + 1) + c) * l * N + x;
    for (int j = (int)l - 1; j >= 0; j--) out[(size_t)j * N] = (double)slz_next_digit(v, beta);
}

__global__ void __launch_bounds__(GEN_THREADS)
k_sample_extract(const uint64_t *__restrict__ acc, uint64_t *__restrict__ lwe_out, uint32_t k, uint32_t N, uint32_t batch) {
    size_t gid = (size_t)blockIdx.x * GEN_THREADS + threadIdx.x;
    size_t width = (size_t)k * N + 1;
    if (gid >= (size_t)batch * width) return;
    uint32_t b = (uint32_t)(gid / width);
    uint32_t x = (uint32_t)(gid % width);
    const uint64_t *a = acc + (size_t)b * (k + 1) * N;
    uint64_t v;
    if (x == k * N) v = a[(size_t)k * N];
    else {
        uint32_t r = x / N, j = x % N;
        v = (j == 0) ? a[(size_t)r * N] : (uint64_t)0 - a[(size_t)r * N + N - j];
    }
    lwe_out[gid] = v;
}

// ---- transforms --------------------------------------------------------------------------------
// Polynomials are addressed by a flat index Q; the prime of polynomial Q is (Q / group) & 1.
// src_div: the source polynomial of Q is src + (Q / src_div_a * src_div_b + Q % src_div_b) ... kept simple:
// when `bcast` != 0 the source has no prime axis: source index = (Q / (2*group)) * group + Q % group.

__device__ __forceinline__ size_t src_index(size_t Q, uint32_t group, int bcast) {
    return bcast ? (Q / (2 * (size_t)group)) * group + Q % group : Q;
}

// forward stages s in [s_begin, logN) inside LDS; requires 2*(N >> (s_begin+1)) <= chunk
__global__ void __launch_bounds__(GEN_THREADS)
k_fwd_lds(const double *src, double *dst, slz_tables t0, slz_tables t1, slz_mod m0, slz_mod m1,
          uint32_t N, uint32_t logN, uint32_t s_begin, uint32_t chunk, uint32_t group, int bcast, uint32_t reduce_mask) {
    __shared__ double sh[GEN_CH];
    uint32_t chunks = N / chunk;
    size_t Q = blockIdx.x / chunks;
    uint32_t cb = (blockIdx.x % chunks) * chunk;
    int prime = (int)((Q / group) & 1);
    const slz_mod m = prime ? m1 : m0;
    const double *tw = prime ? t1.fwd : t0.fwd;
    const double *s = src + src_index(Q, group, bcast) * N + cb;
    for (uint32_t x = threadIdx.x; x < chunk; x += GEN_THREADS) sh[x] = s[x];
    __syncthreads();
    for (uint32_t st = s_begin; st < logN; st++) {
        uint32_t t = N >> (st + 1), mblk = 1u << st;
        bool red = (reduce_mask >> st) & 1u;
        for (uint32_t bf = threadIdx.x; bf < chunk / 2; bf += GEN_THREADS) {
            uint32_t il = bf / t, j = bf % t;
            uint32_t i0 = 2 * il * t + j;
            double w = tw[mblk + cb / (2 * t) + il];
            double u = sh[i0], v = sh[i0 + t];
            if (red) { u = slz_reduce(u, m); v = slz_reduce(v, m); }
            v = slz_mulmod(v, w, m);
            sh[i0] = u + v;
            sh[i0 + t] = u - v;
        }
        __syncthreads();
    }
    double *d = dst + Q * N + cb;
    for (uint32_t x = threadIdx.x; x < chunk; x += GEN_THREADS) d[x] = sh[x];
}

// one forward stage in HBM (for strides that do not fit a chunk)
__global__ void __launch_bounds__(GEN_THREADS)
k_fwd_global(const double *src, double *dst, slz_tables t0, slz_tables t1, slz_mod m0, slz_mod m1,
             uint32_t N, uint32_t st, uint32_t group, int bcast, uint32_t reduce_mask, size_t n_polys) {
    size_t gid = (size_t)blockIdx.x * GEN_THREADS + threadIdx.x;
    if (gid >= n_polys * (N / 2)) return;
    size_t Q = gid / (N / 2);
    uint32_t bf = (uint32_t)(gid % (N / 2));
    int prime = (int)((Q / group) & 1);
    const slz_mod m = prime ? m1 : m0;
    const double *tw = prime ? t1.fwd : t0.fwd;
    uint32_t t = N >> (st + 1);
    uint32_t i = bf / t, j = bf % t, i0 = 2 * i * t + j;
    const double *s = src + src_index(Q, group, bcast) * N;
    double u = s[i0], v = s[i0 + t];
    if ((reduce_mask >> st) & 1u) { u = slz_reduce(u, m); v = slz_reduce(v, m); }
    v = slz_mulmod(v, tw[(1u << st) + i], m);
    dst[Q * N + i0] = u + v;
    dst[Q * N + i0 + t] = u - v;
}

// inverse (cyclic, bit-reversed input -> natural output) stages with half-size t = 1 .. chunk/2 inside LDS;
// when `last` the post-multiplication by psi^-j / N is applied as well.
__global__ void __launch_bounds__(GEN_THREADS)
k_inv_lds(double *__restrict__ data, slz_tables t0, slz_tables t1, slz_mod m0, slz_mod m1, uint32_t N, uint32_t chunk,
          uint32_t group, uint32_t reduce_mask, int last) {
    __shared__ double sh[GEN_CH];
    uint32_t chunks = N / chunk;
    size_t Q = blockIdx.x / chunks;
    uint32_t cb = (blockIdx.x % chunks) * chunk;
    int prime = (int)((Q / group) & 1);
    const slz_mod m = prime ? m1 : m0;
    const double *tw = prime ? t1.inv : t0.inv;
    const double *post = prime ? t1.post : t0.post;
    double *d = data + Q * N + cb;
    for (uint32_t x = threadIdx.x; x < chunk; x += GEN_THREADS) sh[x] = d[x];
    __syncthreads();
    uint32_t st = 0;
    for (uint32_t t = 1; t < chunk; t <<= 1, st++) {
        bool red = (reduce_mask >> st) & 1u;
        for (uint32_t bf = threadIdx.x; bf < chunk / 2; bf += GEN_THREADS) {
            uint32_t blk = bf / t, j = bf % t, i0 = 2 * blk * t + j;
            double u = sh[i0], v = sh[i0 + t];
            if (red) { u = slz_reduce(u, m); v = slz_reduce(v, m); }
            v = slz_mulmod(v, tw[t + j], m);
            sh[i0] = u + v;
            sh[i0 + t] = u - v;
        }
        __syncthreads();
    }
    for (uint32_t x = threadIdx.x; x < chunk; x += GEN_THREADS) {
        double v = sh[x];
        if (last) v = slz_mulmod(v, post[cb + x], m);
        d[x] = v;
    }
}

__global__ void __launch_bounds__(GEN_THREADS)
k_inv_global(double *__restrict__ data, slz_tables t0, slz_tables t1, slz_mod m0, slz_mod m1, uint32_t N, uint32_t t,
             uint32_t st, uint32_t group, uint32_t reduce_mask, int last, size_t n_polys) {
    size_t gid = (size_t)blockIdx.x * GEN_THREADS + threadIdx.x;
    if (gid >= n_polys * (N / 2)) return;
    size_t Q = gid / (N / 2);
    uint32_t bf = (uint32_t)(gid % (N / 2));
    int prime = (int)((Q / group) & 1);
    const slz_mod m = prime ? m1 : m0;
    const double *tw = prime ? t1.inv : t0.inv;
    const double *post = prime ? t1.post : t0.post;
    uint32_t blk = bf / t, j = bf % t, i0 = 2 * blk * t + j;
    double *d = data + Q * N;
    double u = d[i0], v = d[i0 + t];
    if ((reduce_mask >> st) & 1u) { u = slz_reduce(u, m); v = slz_reduce(v, m); }
    v = slz_mulmod(v, tw[t + j], m);
    double a = u + v, b = u - v;
    if (last) { a = slz_mulmod(a, post[i0], m); b = slz_mulmod(b, post[i0 + t], m); }
    d[i0] = a;
    d[i0 + t] = b;
}

// ---- pointwise multiply-accumulate with the prepared key, CRT lift -----------------------------

// outhat[b][q][c][x] = sum_r xhat[b][q][r][x] * bskp_i[q][r][c][pos(x)]   (reduced)
__global__ void __launch_bounds__(GEN_THREADS)
k_pointwise(const double *__restrict__ xhat, const double *__restrict__ bskp_i, double *__restrict__ outhat, slz_mod m0,
            slz_mod m1, uint32_t N, uint32_t R, uint32_t C, uint32_t batch) {
    size_t gid = (size_t)blockIdx.x * GEN_THREADS + threadIdx.x;
    if (gid >= (size_t)batch * 2 * C * N) return;
    uint32_t x = (uint32_t)(gid % N);
    uint32_t c = (uint32_t)((gid / N) % C);
    uint32_t q = (uint32_t)((gid / ((size_t)N * C)) & 1);
    size_t b = gid / ((size_t)N * C * 2);
    const slz_mod m = q ? m1 : m0;
    uint32_t pos = slz_prep_pos(x, N);
    double s = 0.0;
    for (uint32_t r = 0; r < R; r++) {
        double xv = slz_reduce(xhat[((b * 2 + q) * R + r) * N + x], m);     // forward outputs are lazy (up to ~7p)
        double kv = bskp_i[(((size_t)q * R + r) * C + c) * N + pos];
        s += slz_mulmod(xv, kv, m);                                         // each term <= 0.6 p
        if ((r & 7u) == 7u) s = slz_reduce(s, m);
    }
    outhat[gid] = slz_reduce(s, m);
}

// acc[b][c][x] += CRT(outhat[b][0][c][x], outhat[b][1][c][x]) mod 2^64
__global__ void __launch_bounds__(GEN_THREADS)
k_crt_acc(const double *__restrict__ outhat, uint64_t *__restrict__ acc, slz_mod m1, double p1inv, uint32_t N, uint32_t C,
          uint32_t batch) {
    size_t gid = (size_t)blockIdx.x * GEN_THREADS + threadIdx.x;
    if (gid >= (size_t)batch * C * N) return;
    size_t b = gid / ((size_t)C * N);
    size_t rem = gid % ((size_t)C * N);
    double r1 = outhat[(b * 2 + 0) * C * N + rem];
    double r2 = outhat[(b * 2 + 1) * C * N + rem];
    acc[gid] += slz_crt64(r1, r2, m1, p1inv);
}

// ---- key preparation ---------------------------------------------------------------------------

// tmp[q][poly][x] = centred residue of the signed key word bsk[poly][x] mod p_q
__global__ void __launch_bounds__(GEN_THREADS)
k_key_to_res(const uint64_t *__restrict__ bsk_i, double *__restrict__ tmp, slz_mod m0, slz_mod m1, double t0, double t1,
             size_t count) {
    size_t gid = (size_t)blockIdx.x * GEN_THREADS + threadIdx.x;
    if (gid >= 2 * count) return;
    int q = gid >= count;
    uint64_t w = bsk_i[gid - (q ? count : 0)];
    tmp[gid] = slz_i64_to_res(w, q ? m1 : m0, q ? t1 : t0);
}

// dst[q][poly][pos(x)] = reduce(tmp[q][poly][x])
__global__ void __launch_bounds__(GEN_THREADS)
k_store_prepared(const double *__restrict__ tmp, double *__restrict__ dst, slz_mod m0, slz_mod m1, uint32_t N, size_t polys) {
    size_t gid = (size_t)blockIdx.x * GEN_THREADS + threadIdx.x;
    if (gid >= 2 * polys * N) return;
    uint32_t x = (uint32_t)(gid % N);
    size_t Q = gid / N;
    int q = Q >= polys;
    dst[Q * N + slz_prep_pos(x, N)] = slz_reduce(tmp[gid], q ? m1 : m0);
}

// ---- host drivers ------------------------------------------------------------------------------

static inline unsigned blocks_for(size_t items) { return (unsigned)((items + GEN_THREADS - 1) / GEN_THREADS); }

// forward transform of n_polys polynomials, dst[Q] <- NTT(src[src_index(Q)])
static int fwd_all(slz_ctx *ctx, const double *src, double *dst, size_t n_polys, uint32_t group, int bcast, hipStream_t s) {
    const uint32_t N = ctx->prm.N, logN = ctx->logN;
    const uint32_t chunk = N < GEN_CH ? N : GEN_CH;
    uint32_t st = 0;
    const double *cur = src;
    int cur_bcast = bcast;
    while ((N >> st) > chunk) {      // stage st has stride N >> (st+1); it fits a chunk once 2*stride <= chunk
        hipLaunchKernelGGL(k_fwd_global, dim3(blocks_for(n_polys * (N / 2))), dim3(GEN_THREADS), 0, s, cur, dst, ctx->tab[0],
                           ctx->tab[1], ctx->mod[0], ctx->mod[1], N, st, group, cur_bcast, ctx->fwd_reduce_mask, n_polys);
        cur = dst; cur_bcast = 0; st++;
    }
    hipLaunchKernelGGL(k_fwd_lds, dim3((unsigned)(n_polys * (N / chunk))), dim3(GEN_THREADS), 0, s, cur, dst, ctx->tab[0],
                       ctx->tab[1], ctx->mod[0], ctx->mod[1], N, logN, st, chunk, group, cur_bcast, ctx->fwd_reduce_mask);
    SLZ_HIP(hipGetLastError());
    return SLZ_OK;
}

static int inv_all(slz_ctx *ctx, double *data, size_t n_polys, uint32_t group, hipStream_t s) {
    const uint32_t N = ctx->prm.N;
    const uint32_t chunk = N < GEN_CH ? N : GEN_CH;
    hipLaunchKernelGGL(k_inv_lds, dim3((unsigned)(n_polys * (N / chunk))), dim3(GEN_THREADS), 0, s, data, ctx->tab[0], ctx->tab[1],
                       ctx->mod[0], ctx->mod[1], N, chunk, group, ctx->inv_reduce_mask, chunk == N ? 1 : 0);
    uint32_t st = 0;
    for (uint32_t t = 1; t < chunk; t <<= 1) st++;
    for (uint32_t t = chunk; t < N; t <<= 1, st++)
        hipLaunchKernelGGL(k_inv_global, dim3(blocks_for(n_polys * (N / 2))), dim3(GEN_THREADS), 0, s, data, ctx->tab[0],
                           ctx->tab[1], ctx->mod[0], ctx->mod[1], N, t, st, group, ctx->inv_reduce_mask, (t * 2 == N) ? 1 : 0,
                           n_polys);
    SLZ_HIP(hipGetLastError());
    return SLZ_OK;
}

int slz_generic_bsk_prepare(slz_ctx *ctx, const uint64_t *bsk, double *dst, hipStream_t s) {
    const slz_params &p = ctx->prm;
    const uint32_t R = (p.k + 1) * p.pbs_level, C = p.k + 1;
    const size_t polys = (size_t)R * C;                 // polynomials of one GGSW
    const size_t count = polys * p.N;
    double *tmp = nullptr;
    SLZ_HIP(hipMalloc((void **)&tmp, 2 * count * sizeof(double)));
    int rc = SLZ_OK;
    for (uint32_t i = 0; i < p.n && rc == SLZ_OK; i++) {
        hipLaunchKernelGGL(k_key_to_res, dim3(blocks_for(2 * count)), dim3(GEN_THREADS), 0, s, bsk + (size_t)i * count, tmp,
                           ctx->mod[0], ctx->mod[1], ctx->two32[0], ctx->two32[1], count);
        rc = fwd_all(ctx, tmp, tmp, 2 * polys, (uint32_t)polys, 0, s);
        hipLaunchKernelGGL(k_store_prepared, dim3(blocks_for(2 * count)), dim3(GEN_THREADS), 0, s, tmp, dst + (size_t)i * 2 * count,
                           ctx->mod[0], ctx->mod[1], p.N, polys);
    }
    hipError_t e = hipStreamSynchronize(s);
    (void)hipFree(tmp);
    if (rc != SLZ_OK) return rc;
    return e == hipSuccess ? SLZ_OK : SLZ_E_HIP;
}

int slz_generic_blind_rotate(slz_ctx *ctx, const uint64_t *lwe_in, const uint64_t *luts, const uint32_t *lut_idx,
                             const double *bskp, uint32_t n_steps, uint64_t *acc_out, uint64_t *lwe_out, uint32_t batch,
                             hipStream_t s) {
    const slz_params &p = ctx->prm;
    const uint32_t R = (p.k + 1) * p.pbs_level, C = p.k + 1, N = p.N;
    uint64_t *acc = acc_out ? acc_out : ctx->acc;
    const size_t glwe = (size_t)batch * C * N;
    hipLaunchKernelGGL(k_acc_init, dim3(blocks_for(glwe)), dim3(GEN_THREADS), 0, s, lwe_in, luts, lut_idx, acc, p.n, p.k, N,
                       ctx->logN, batch);
    const size_t ggsw = (size_t)2 * R * C * N;
    if (ctx->has_bign && !ctx->force_generic) {
        int rc = slz_bign_cmux_steps(ctx, lwe_in, bskp, n_steps, acc, batch, s);
        if (rc != SLZ_OK) return rc;
        n_steps = 0;                                   // the per-step kernels below are skipped
    }
    for (uint32_t i = 0; i < n_steps; i++) {
        hipLaunchKernelGGL(k_decompose, dim3(blocks_for(glwe)), dim3(GEN_THREADS), 0, s, acc, lwe_in, i, ctx->dig, p.n, p.k, N,
                           ctx->logN, p.pbs_base_log, p.pbs_level, batch);
        int rc = fwd_all(ctx, ctx->dig, ctx->xhat, (size_t)batch * 2 * R, R, 1, s);
        if (rc != SLZ_OK) return rc;
        hipLaunchKernelGGL(k_pointwise, dim3(blocks_for((size_t)batch * 2 * C * N)), dim3(GEN_THREADS), 0, s, ctx->xhat,
                           bskp + (size_t)i * ggsw, ctx->outhat, ctx->mod[0], ctx->mod[1], N, R, C, batch);
        rc = inv_all(ctx, ctx->outhat, (size_t)batch * 2 * C, C, s);
        if (rc != SLZ_OK) return rc;
        hipLaunchKernelGGL(k_crt_acc, dim3(blocks_for(glwe)), dim3(GEN_THREADS), 0, s, ctx->outhat, acc, ctx->mod[1],
                           ctx->p1inv_mod_p2, N, C, batch);
    }
    if (lwe_out)
        hipLaunchKernelGGL(k_sample_extract, dim3(blocks_for((size_t)batch * (p.k * N + 1))), dim3(GEN_THREADS), 0, s, acc, lwe_out,
                           p.k, N, batch);
    SLZ_HIP(hipGetLastError());
    return SLZ_OK;
}
