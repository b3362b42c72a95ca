// Blind rotation for large polynomials, N = BS * G with block size BS = 1024 or 2048 and G in {2,4,8,16,32}, k = 1 (the
// 8-bit-precision-shaped parameter sets: N = 32768).  The accumulator (512 KiB per ciphertext at N = 32768) cannot stay
// on chip, so a CMux step is three passes over a per-ciphertext workspace that stays in L2 / Infinity Cache when
// ciphertexts are processed in chunks:
//   P1 "columns, forward":  per accumulator column c (coefficients BS i + c, i < G): rotate, subtract, decompose,
//                           then the first log2(G) transform stages (they pair coefficients BS rows apart, so a
//                           lane holding one column does them in registers), for every level and both primes.
//   P2 "rows":              per prime and block: the remaining forward stages with a wave-level transform (32 or 16
//                           coefficients per lane, block-specific twiddles), multiply-accumulate with the prepared
//                           key over all GGSW rows, the same number of inverse stages.
//   P3 "columns, inverse":  the last log2(G) inverse stages per column, the psi^-j / N twist, CRT lift, accumulate.
#include "slz_internal.h"
#include "slz_modarith.h"
#include "slz_wave_ntt.h"
#include <vector>

#define BIG_MAX_L 4

struct bign_tabs {                 // per prime
    const double *fwd;             // natural forward table of the full transform (fwd[m + blk])
    const double *rowA;            // [G][64]      block-specific twiddles of stages with 1..32 sub-blocks (uniform per wave)
    const double *rowB;            // [G][31][64]  block-specific per-lane twiddles of the last five forward stages
    const double *inv;             // natural inverse table
    const double *post;            // natural twist table
};

struct bign_args {
    const uint64_t *lwe_in;
    uint64_t *acc;                 // [batch][2][N]
    double *X;                     // [batch][2 primes][R][N]
    double *Y;                     // [batch][2 primes][2][N]
    const double *bskp_step;       // prepared GGSW of this step: [2][R][2][N]
    uint32_t n, step, N, logG, beta, l, batch;
    bign_tabs tab[2];
    slz_mod mod[2];
    double p1inv_mod_p2;
};

// ---- P1 ------------------------------------------------------------------------------------------
// BS: block size of the row pass (2048 or 1024); G = N / BS rows of BS columns
// SPLIT: one thread per (column, component, level, prime) instead of one per (column, component): four times (l = 2) as
// many threads, each repeating the cheap rotate / subtract / round and doing one column transform.  For a handful of
// ciphertexts, where the pass is one thread's latency.
template <int G, int BS, bool SPLIT>
__global__ void __launch_bounds__(256)
k_big_cols_fwd(bign_args A) {
    const uint32_t c = blockIdx.x * 256 + threadIdx.x;          // column, < BS
    const uint32_t b = blockIdx.z;
    const uint32_t comp = SPLIT ? blockIdx.y / (2 * A.l) : blockIdx.y;
    const int only_lev = SPLIT ? (int)((blockIdx.y >> 1) % A.l) : -1, only_q = SPLIT ? (int)(blockIdx.y & 1u) : -1;
    const uint32_t N = A.N, R = 2 * A.l;
    uint32_t logN2 = 1;                                          // log2(2N)
    for (uint32_t g = N; g > 1; g >>= 1) logN2++;
    const uint32_t at = slz_modswitch(A.lwe_in[(size_t)b * (A.n + 1) + A.step], logN2);
    const uint64_t *poly = A.acc + ((size_t)b * 2 + comp) * N;
    uint64_t lam[G];
#pragma unroll
    for (int i = 0; i < G; i++) {
        const uint32_t idx = (uint32_t)BS * i + c;
        lam[i] = slz_rot_coeff([&](uint32_t j) { return poly[j]; }, idx, at, N) - poly[idx];
        lam[i] = slz_round_top_bits(lam[i], A.beta * A.l);
    }
    for (int lev = (int)A.l - 1; lev >= 0; lev--) {              // least significant level first (carries go up)
        double d[G];
#pragma unroll
        for (int i = 0; i < G; i++) d[i] = (double)slz_next_digit(lam[i], A.beta);
        if (SPLIT && lev != only_lev) continue;                  // lower levels are only peeled for their carries
        for (int q = 0; q < 2; q++) {
            if (SPLIT && q != only_q) continue;
            const slz_mod m = A.mod[q];
            const double *tw = A.tab[q].fwd;
            double y[G];
#pragma unroll
            for (int i = 0; i < G; i++) y[i] = d[i];
            // stages with strides N/2 .. BS: pairs of rows, twiddle by block of rows (uniform)
#pragma unroll
            for (int half = G / 2, blocks = 1; half >= 1; half >>= 1, blocks <<= 1) {
#pragma unroll
                for (int blk = 0; blk < blocks; blk++) {
                    const double w = tw[blocks + blk];
#pragma unroll
                    for (int j = 0; j < half; j++) bfly(y[blk * 2 * half + j], y[blk * 2 * half + j + half], w, m);
                }
            }
            double *dst = A.X + (((size_t)b * 2 + q) * R + (comp * A.l + lev)) * N + c;
#pragma unroll
            for (int i = 0; i < G; i++) dst[(uint32_t)BS * i] = slz_reduce(y[i], m);
        }
        if (SPLIT) break;
    }
}

// ---- P2 ------------------------------------------------------------------------------------------
// one wave per (ciphertext, prime, 2048-block); four independent waves per workgroup
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
k_big_rows(bign_args A, uint32_t G, uint32_t n_tasks, int xcd_aware) {
    extern __shared__ double lds[];
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // Workgroups are dealt round-robin to the 8 XCDs, each with its own 4 MiB L2, and one step's key is as large as
    // one L2.  With xcd_aware the 2G (prime, block) combinations are split between the XCDs, so that an XCD only
    // touches its 1/8 of the key and re-reads it from its L2 for every ciphertext of the chunk.
    uint32_t task = blockIdx.x * 4 + wv;
    if (xcd_aware) {
        const uint32_t cpx = 2 * G / 8;                          // combinations per XCD
        const uint32_t xcd = blockIdx.x & 7u, v = (blockIdx.x >> 3) * 4 + wv;
        task = (v / cpx) * 2 * G + xcd * cpx + v % cpx;
    }
    if (task >= n_tasks) return;                                 // whole wave leaves; no workgroup barriers below
    double *T = lds + wv * TBUF;
    const uint32_t row = task % G, q = (task / G) & 1u, b = task / (2 * G);
    const uint32_t N = A.N, R = 2 * A.l, hh = lane >> 5;
    const slz_mod m = A.mod[q];
    const bign_tabs tb = A.tab[q];
    const double *twA = tb.rowA + (size_t)row * 64, *fwd6 = twA + 32, *fwdB = tb.rowB + (size_t)row * 31 * 64;
    double o0[32], o1[32];
    for (uint32_t r = 0; r < R; r++) {
        int z;
        asm volatile("s_mov_b32 %0, 0" : "=s"(z));              // tables are reloaded per GGSW row (they would spill if hoisted)
        double tw6[16];
#pragma unroll
        for (int mm = 0; mm < 16; mm++) tw6[mm] = ldl(fwd6 + 2 * mm + z, hh * 8u);
        const double *src = A.X + (((size_t)b * 2 + q) * R + r) * N + 2048u * row + z;
        double x[32];
#pragma unroll
        for (int e = 0; e < 32; e++) x[e] = ldl(src + 64 * e, lane * 8u);
        fused_fwd(x, T, tw6, twA, fwdB, m, lane, z);
        // multiply-accumulate with the key polynomials of GGSW row r (both components); spectrum index of x[i] is
        // 2048 row + 32 lane + i, stored at position i * (N/32) + 64 row + lane of the prepared polynomial
        const double *k0 = A.bskp_step + (((size_t)q * R + r) * 2 + 0) * N + 64u * row + z;
        const double *k1 = k0 + N;
        const uint32_t stride = N / 32;
#pragma unroll
        for (int g = 0; g < 8; g++) {
            double kk0[4], kk1[4], r0[4], r1[4];
#pragma unroll
            for (int u = 0; u < 4; u++) { kk0[u] = ldl(k0 + (size_t)(4 * g + u) * stride, lane * 8u); kk1[u] = ldl(k1 + (size_t)(4 * g + u) * stride, lane * 8u); }
            const double x4[4] = {x[4 * g], x[4 * g + 1], x[4 * g + 2], x[4 * g + 3]};
            mulmod_k<4>(r0, x4, kk0, m);
            mulmod_k<4>(r1, x4, kk1, m);
#pragma unroll
            for (int u = 0; u < 4; u++) {
                o0[4 * g + u] = (r == 0) ? r0[u] : o0[4 * g + u] + r0[u];
                o1[4 * g + u] = (r == 0) ? r1[u] : o1[4 * g + u] + r1[u];
            }
        }
        if ((r & 3u) == 3u && r + 1 < R) {                       // more than four rows: keep the running sums below 8 p
#pragma unroll
            for (int g = 0; g < 8; g++) {
                double a4[4], b4[4];
                const double xa[4] = {o0[4 * g], o0[4 * g + 1], o0[4 * g + 2], o0[4 * g + 3]};
                const double xb[4] = {o1[4 * g], o1[4 * g + 1], o1[4 * g + 2], o1[4 * g + 3]};
                reduce_k<4>(a4, xa, m);
                reduce_k<4>(b4, xb, m);
#pragma unroll
                for (int u = 0; u < 4; u++) { o0[4 * g + u] = a4[u]; o1[4 * g + u] = b4[u]; }
            }
        }
        wave_sync();
    }
    // inverse: first 11 stages inside the block, reduce, hand the block to the column pass
    for (int comp = 0; comp < 2; comp++) {
        int z;
        asm volatile("s_mov_b32 %0, 0" : "=s"(z));
        double x[32];
#pragma unroll
        for (int g = 0; g < 4; g++) {
            double r8[8], x8[8];
#pragma unroll
            for (int u = 0; u < 8; u++) x8[u] = comp ? o1[8 * g + u] : o0[8 * g + u];
            reduce_k<8>(r8, x8, m);
#pragma unroll
            for (int u = 0; u < 8; u++) x[8 * g + u] = r8[u];
        }
        fused_inv<false>(x, T, tb.inv, tb.inv, tb.post, m, lane, z);
        double *dst = A.Y + (((size_t)b * 2 + q) * 2 + comp) * N + 2048u * row;
#pragma unroll
        for (int g = 0; g < 4; g++) {
            double r8[8], x8[8];
#pragma unroll
            for (int u = 0; u < 8; u++) x8[u] = x[8 * g + u];
            reduce_k<8>(r8, x8, m);
#pragma unroll
            for (int u = 0; u < 8; u++) dst[64 * (8 * g + u) + lane] = r8[u];
        }
        wave_sync();
    }
}

// ---- P2 with 1024-blocks -------------------------------------------------------------------------
// One wave per (ciphertext, prime, 1024-block), 16 coefficients per lane: the accumulators of both components, the block
// and the tables fit 256 registers, so two waves share a SIMD and cover each other's memory latency (the 2048-block
// kernel above needs more than 256 and runs one wave per SIMD, 43 % of it waiting for memory).
// BOTH = false: one task per output component as well (twice the tasks, each with all R forward transforms but the products
// and the inverse transform of one component only): for a few ciphertexts, where a pass lasts as long as its longest task.
template <bool BOTH>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
k_big_rows16(bign_args A, uint32_t G, uint32_t n_tasks, int xcd_aware) {
    extern __shared__ double lds[];
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint32_t task = blockIdx.x * 4 + wv;
    if (xcd_aware) {                                             // as above: an XCD keeps to its 1/8 of the (prime, block) pairs
        const uint32_t cpx = 2 * G / 8;
        const uint32_t xcd = blockIdx.x & 7u, v = (blockIdx.x >> 3) * 4 + wv;
        task = (v / cpx) * 2 * G + xcd * cpx + v % cpx;
    }
    if (task >= n_tasks) return;                                 // whole wave leaves; no workgroup barriers below
    const uint32_t only = BOTH ? 0u : task & 1u;                 // the component of a one-component task
    if (!BOTH) task >>= 1;
    double *T = lds + wv * (TBUF16 + 1024u);
    double *twA = T + TBUF16, *twB = twA + 64;                  // this block's forward tables, staged in LDS
    const uint32_t row = task % G, q = (task / G) & 1u, b = task / (2 * G);
    const uint32_t N = A.N, R = 2 * A.l;
    const slz_mod m = A.mod[q];
    const bign_tabs tb = A.tab[q];
    {
        const double *gA = tb.rowA + (size_t)row * 64, *gB = tb.rowB + (size_t)row * 15 * 64;
        twA[lane] = gA[lane];
#pragma unroll
        for (int k = 0; k < 15; k++) twB[64 * k + lane] = gB[64 * k + lane];
        wave_sync();
    }
    // spectrum index of x[i] is 1024 row + 16 lane + i, stored at position (idx % 32) (N/32) + idx / 32 of the prepared
    // polynomial: register i of lane l sits at i (N/32) + [16 (l & 1) (N/32) + 32 row + l / 2]
    const uint32_t stride = N / 32;
    const uint32_t key_lane_off = (16u * (lane & 1u) * stride + (lane >> 1)) * 8u;
    double o0[16], o1[16];
    double xn[16];                                               // the next GGSW row's block, requested one row ahead
    {
        const double *src = A.X + (((size_t)b * 2 + q) * R + 0) * N + 1024u * row;
#pragma unroll
        for (int e = 0; e < 16; e++) xn[e] = ldl(src + 64 * e, lane * 8u);
    }
    for (uint32_t r = 0; r < R; r++) {
        int z;
        asm volatile("s_mov_b32 %0, 0" : "=s"(z));              // tables are reloaded per GGSW row (they would spill if hoisted)
        double x[16];
#pragma unroll
        for (int e = 0; e < 16; e++) x[e] = xn[e];
        // the key words of this row and then the next row's block are requested here (vector memory completes in issue
        // order) and arrive while the transform runs
        const double *k0 = A.bskp_step + (((size_t)q * R + r) * 2 + only) * N + 32u * row + z;
        const double *k1 = k0 + N;
        double kk0[16], kk1[16];
#pragma unroll
        for (int i = 0; i < 16; i++) {
            kk0[i] = ldl(k0 + (size_t)i * stride, key_lane_off);
            if (BOTH) kk1[i] = ldl(k1 + (size_t)i * stride, key_lane_off);
        }
        {
            const double *nxt = A.X + (((size_t)b * 2 + q) * R + (r + 1 < R ? r + 1 : r)) * N + 1024u * row + z;
#pragma unroll
            for (int e = 0; e < 16; e++) xn[e] = ldl(nxt + 64 * e, lane * 8u);
        }
        SCHED_FENCE();
        fwd16(x, T, twA, twB, m, lane, z);
        SCHED_FENCE();
#pragma unroll
        for (int g = 0; g < 4; g++) {
            double r0[4], r1[4];
            const double x4[4] = {x[4 * g], x[4 * g + 1], x[4 * g + 2], x[4 * g + 3]};
            const double ka[4] = {kk0[4 * g], kk0[4 * g + 1], kk0[4 * g + 2], kk0[4 * g + 3]};
            mulmod_k<4>(r0, x4, ka, m);
            if (BOTH) {
                const double kb[4] = {kk1[4 * g], kk1[4 * g + 1], kk1[4 * g + 2], kk1[4 * g + 3]};
                mulmod_k<4>(r1, x4, kb, m);
            }
#pragma unroll
            for (int u = 0; u < 4; u++) {
                o0[4 * g + u] = (r == 0) ? r0[u] : o0[4 * g + u] + r0[u];
                if (BOTH) o1[4 * g + u] = (r == 0) ? r1[u] : o1[4 * g + u] + r1[u];
            }
        }
        if ((r & 3u) == 3u && r + 1 < R) {                       // more than four rows: keep the running sums below 8 p
#pragma unroll
            for (int g = 0; g < 4; g++) {
                double a4[4], b4[4];
                const double xa[4] = {o0[4 * g], o0[4 * g + 1], o0[4 * g + 2], o0[4 * g + 3]};
                reduce_k<4>(a4, xa, m);
                if (BOTH) {
                    const double xb[4] = {o1[4 * g], o1[4 * g + 1], o1[4 * g + 2], o1[4 * g + 3]};
                    reduce_k<4>(b4, xb, m);
                }
#pragma unroll
                for (int u = 0; u < 4; u++) { o0[4 * g + u] = a4[u]; if (BOTH) o1[4 * g + u] = b4[u]; }
            }
        }
        wave_sync();
    }
    // inverse: first 10 stages inside the block, reduce, hand the block to the column pass
    for (int cc = 0; cc < (BOTH ? 2 : 1); cc++) {
        const uint32_t comp = BOTH ? (uint32_t)cc : only;
        int z;
        asm volatile("s_mov_b32 %0, 0" : "=s"(z));
        double x[16];
#pragma unroll
        for (int g = 0; g < 2; g++) {
            double r8[8], x8[8];
#pragma unroll
            for (int u = 0; u < 8; u++) x8[u] = (BOTH && cc) ? o1[8 * g + u] : o0[8 * g + u];
            reduce_k<8>(r8, x8, m);
#pragma unroll
            for (int u = 0; u < 8; u++) x[8 * g + u] = r8[u];
        }
        inv16(x, T, tb.inv, tb.inv, m, lane, z);
        double *dst = A.Y + (((size_t)b * 2 + q) * 2 + comp) * N + 1024u * row;
#pragma unroll
        for (int g = 0; g < 2; g++) {
            double r8[8], x8[8];
#pragma unroll
            for (int u = 0; u < 8; u++) x8[u] = x[8 * g + u];
            reduce_k<8>(r8, x8, m);
#pragma unroll
            for (int u = 0; u < 8; u++) dst[64 * (8 * g + u) + lane] = r8[u];
        }
        wave_sync();
    }
}

// ---- P3 ------------------------------------------------------------------------------------------
template <int G, int BS>
__global__ void __launch_bounds__(256)
k_big_cols_inv(bign_args A) {
    const uint32_t c = blockIdx.x * 256 + threadIdx.x;
    const uint32_t comp = blockIdx.y, b = blockIdx.z;
    const uint32_t N = A.N;
    double res[2][G];
    for (int q = 0; q < 2; q++) {
        const slz_mod m = A.mod[q];
        const double *src = A.Y + (((size_t)b * 2 + q) * 2 + comp) * N + c;
        const double *tw = A.tab[q].inv, *post = A.tab[q].post;
        double y[G];
#pragma unroll
        for (int i = 0; i < G; i++) y[i] = src[(uint32_t)BS * i];
        // stages with half-size t = BS * half: pairs of rows i, i + half; twiddle inv[t + BS (i mod half) + c]
#pragma unroll
        for (int half = 1; half < G; half <<= 1) {
#pragma unroll
            for (int j = 0; j < half; j++) {
                const double w = tw[(uint32_t)BS * half + (uint32_t)BS * j + c];
#pragma unroll
                for (int blk = 0; blk < G / (2 * half); blk++) bfly(y[blk * 2 * half + j], y[blk * 2 * half + j + half], w, m);
            }
        }
#pragma unroll
        for (int i = 0; i < G; i++) res[q][i] = slz_mulmod(y[i], post[(uint32_t)BS * i + c], m);
    }
    uint64_t *poly = A.acc + ((size_t)b * 2 + comp) * N + c;
#pragma unroll
    for (int i = 0; i < G; i++) poly[(uint32_t)BS * i] += slz_crt64(res[0][i], res[1][i], A.mod[1], A.p1inv_mod_p2);
}

// ---- a handful of ciphertexts: the same step cut into more, shorter pieces --------------------------------------------
// With few ciphertexts the chip is mostly empty and a step costs the latency of its longest thread: one row task runs R
// forward transforms, the products and two inverse transforms one after the other.  Here a row task is one GGSW row
// (k_big_rows16_lat_a: forward transform, products with both key columns, written to P) or one output component
// (k_big_rows16_lat_b: sum of the R partial products, inverse transform), and the inverse column pass runs the two primes
// of a column on two neighbouring lanes.  More launches and more traffic per step, several times the parallelism.
// P: [batch][2 primes][R][2 components][N], a row-block stored as [16 registers][64 lanes].
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
k_big_rows16_lat_a(bign_args A, double *__restrict__ P, uint32_t G, uint32_t n_tasks) {
    extern __shared__ double lds[];
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t task = blockIdx.x * 4 + wv;
    if (task >= n_tasks) return;                                 // whole wave leaves; no workgroup barriers below
    double *T = lds + wv * (TBUF16 + 1024u);
    double *twA = T + TBUF16, *twB = twA + 64;
    const uint32_t N = A.N, R = 2 * A.l;
    const uint32_t r = task % R, row = (task / R) % G, q = (task / (R * G)) & 1u, b = task / (2 * R * G);
    const slz_mod m = A.mod[q];
    const bign_tabs tb = A.tab[q];
    const uint32_t stride = N / 32;
    const uint32_t key_lane_off = (16u * (lane & 1u) * stride + (lane >> 1)) * 8u;
    int z;
    asm volatile("s_mov_b32 %0, 0" : "=s"(z));
    double x[16], kk0[16], kk1[16];
    {
        const double *src = A.X + (((size_t)b * 2 + q) * R + r) * N + 1024u * row;
#pragma unroll
        for (int e = 0; e < 16; e++) x[e] = ldl(src + 64 * e, lane * 8u);
        const double *gA = tb.rowA + (size_t)row * 64, *gB = tb.rowB + (size_t)row * 15 * 64;
        twA[lane] = gA[lane];
#pragma unroll
        for (int k = 0; k < 15; k++) twB[64 * k + lane] = gB[64 * k + lane];
        const double *k0 = A.bskp_step + (((size_t)q * R + r) * 2 + 0) * N + 32u * row;
        const double *k1 = k0 + N;
#pragma unroll
        for (int i = 0; i < 16; i++) { kk0[i] = ldl(k0 + (size_t)i * stride, key_lane_off); kk1[i] = ldl(k1 + (size_t)i * stride, key_lane_off); }
        wave_sync();
    }
    SCHED_FENCE();
    fwd16(x, T, twA, twB, m, lane, z);
    double *dst = P + ((((size_t)b * 2 + q) * R + r) * 2) * N + 1024u * row + lane;
#pragma unroll
    for (int g = 0; g < 4; g++) {
        double r0[4], r1[4];
        const double x4[4] = {x[4 * g], x[4 * g + 1], x[4 * g + 2], x[4 * g + 3]};
        const double ka[4] = {kk0[4 * g], kk0[4 * g + 1], kk0[4 * g + 2], kk0[4 * g + 3]};
        const double kb[4] = {kk1[4 * g], kk1[4 * g + 1], kk1[4 * g + 2], kk1[4 * g + 3]};
        mulmod_k<4>(r0, x4, ka, m);
        mulmod_k<4>(r1, x4, kb, m);
#pragma unroll
        for (int u = 0; u < 4; u++) {
            dst[64 * (4 * g + u)] = r0[u];
            dst[(size_t)N + 64 * (4 * g + u)] = r1[u];
        }
    }
}

__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
k_big_rows16_lat_b(bign_args A, const double *__restrict__ P, uint32_t G, uint32_t n_tasks) {
    extern __shared__ double lds[];
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t task = blockIdx.x * 4 + wv;
    if (task >= n_tasks) return;
    double *T = lds + wv * TBUF16;
    const uint32_t N = A.N, R = 2 * A.l;
    const uint32_t comp = task & 1u, row = (task >> 1) % G, q = (task / (2 * G)) & 1u, b = task / (4 * G);
    const slz_mod m = A.mod[q];
    const bign_tabs tb = A.tab[q];
    int z;
    asm volatile("s_mov_b32 %0, 0" : "=s"(z));
    double x[16];
    {
        const double *src = P + ((((size_t)b * 2 + q) * R) * 2 + comp) * N + 1024u * row + lane;
#pragma unroll
        for (int i = 0; i < 16; i++) x[i] = src[64 * i];
        for (uint32_t r = 1; r < R; r++) {
            const double *sr = src + (size_t)r * 2 * N;
#pragma unroll
            for (int i = 0; i < 16; i++) x[i] += sr[64 * i];
            if ((r & 3u) == 3u && r + 1 < R) {                   // as in the throughput kernel: at most four products per reduction
#pragma unroll
                for (int i = 0; i < 16; i++) x[i] = slz_reduce(x[i], m);
            }
        }
    }
#pragma unroll
    for (int g = 0; g < 2; g++) {
        double r8[8], x8[8];
#pragma unroll
        for (int u = 0; u < 8; u++) x8[u] = x[8 * g + u];
        reduce_k<8>(r8, x8, m);
#pragma unroll
        for (int u = 0; u < 8; u++) x[8 * g + u] = r8[u];
    }
    inv16(x, T, tb.inv, tb.inv, m, lane, z);
    double *dst = A.Y + (((size_t)b * 2 + q) * 2 + comp) * N + 1024u * row;
#pragma unroll
    for (int g = 0; g < 2; g++) {
        double r8[8], x8[8];
#pragma unroll
        for (int u = 0; u < 8; u++) x8[u] = x[8 * g + u];
        reduce_k<8>(r8, x8, m);
#pragma unroll
        for (int u = 0; u < 8; u++) dst[64 * (8 * g + u) + lane] = r8[u];
    }
}

// P3 with the two primes of a column on lanes 2j and 2j + 1: each lane runs its prime's column stages and twist, the
// lanes swap the halves they do not lift (rows below G/2 are lifted by the lane of prime 0, the others by prime 1's).
template <int G, int BS>
__global__ void __launch_bounds__(256)
k_big_cols_inv_lat(bign_args A) {
    const uint32_t c = blockIdx.x * 128 + (threadIdx.x >> 1);
    const uint32_t q = threadIdx.x & 1u;
    const uint32_t comp = blockIdx.y, b = blockIdx.z;
    const uint32_t N = A.N;
    const slz_mod m = A.mod[q];
    const double *src = A.Y + (((size_t)b * 2 + q) * 2 + comp) * N + c;
    const double *tw = A.tab[q].inv, *post = A.tab[q].post;
    double y[G];
#pragma unroll
    for (int i = 0; i < G; i++) y[i] = src[(uint32_t)BS * i];
#pragma unroll
    for (int half = 1; half < G; half <<= 1) {
#pragma unroll
        for (int j = 0; j < half; j++) {
            const double w = tw[(uint32_t)BS * half + (uint32_t)BS * j + c];
#pragma unroll
            for (int blk = 0; blk < G / (2 * half); blk++) bfly(y[blk * 2 * half + j], y[blk * 2 * half + j + half], w, m);
        }
    }
#pragma unroll
    for (int i = 0; i < G; i++) y[i] = slz_mulmod(y[i], post[(uint32_t)BS * i + c], m);
    uint64_t *poly = A.acc + ((size_t)b * 2 + comp) * N + c;
#pragma unroll
    for (int j = 0; j < G / 2; j++) {
        const double send = q ? y[j] : y[G / 2 + j];             // the half the partner lifts
        const double got = __shfl_xor(send, 1);
        const int i = q ? G / 2 + j : j;
        const double r1 = q ? got : y[j], r2 = q ? y[G / 2 + j] : got;
        poly[(uint32_t)BS * i] += slz_crt64(r1, r2, A.mod[1], A.p1inv_mod_p2);
    }
}

// ---- host ------------------------------------------------------------------------------------------

int slz_bign_supported(const slz_params *p) {
    if (p->k != 1 || p->pbs_level > BIG_MAX_L) return 0;
    for (uint32_t G = 2; G <= 32; G <<= 1)
        if (p->N == 2048u * G || p->N == 1024u * G) return 1;
    return 0;
}

static bool block_fits(uint32_t N, uint32_t BS) {
    const uint32_t G = N / BS;
    return N % BS == 0 && G >= 2 && G <= 32 && (G & (G - 1)) == 0;
}

// block-specific forward tables for blocks of BS = 64 * E coefficients (E = 32 or 16 per lane)
int slz_build_block_tables(slz_ctx *ctx, uint32_t BS, double **dA, double **dB) {
    const uint32_t N = ctx->prm.N, G = N / BS, E = BS / 64;
    int late = 0;                                   // stages done after the transposition: log2 E
    for (uint32_t e = E; e > 1; e >>= 1) late++;
    const uint32_t nB = E - 1;                      // per-lane twiddles of those stages
    std::vector<double> nat(N), rowA((size_t)2 * G * 64), rowB((size_t)2 * G * nB * 64);
    for (int q = 0; q < 2; q++) {
        SLZ_HIP(hipMemcpy(nat.data(), ctx->tab[q].fwd, (size_t)N * sizeof(double), hipMemcpyDeviceToHost));
        for (uint32_t row = 0; row < G; row++) {
            // block `row` continues the transform with sub-block counts m' = 1, 2, ..., BS / 2; its sub-block blk at that
            // stage is block (G + row) m' + blk of the whole transform: table entry fwd[(G + row) m' + blk]
            double *ra = &rowA[((size_t)q * G + row) * 64];
            ra[0] = 1.0;
            for (uint32_t x = 1; x < 64; x++) {
                uint32_t mp = 1;
                while (mp * 2 <= x) mp *= 2;
                ra[x] = nat[(size_t)(G + row) * mp + (x - mp)];
            }
            int kk = 0;
            for (int s = 0; s < late; s++) {
                const uint32_t t = (E / 2) >> s, mp = BS / (2 * t);
                for (uint32_t blk = 0; blk < (1u << s); blk++, kk++)
                    for (uint32_t l = 0; l < 64; l++)
                        rowB[(((size_t)q * G + row) * nB + kk) * 64 + l] = nat[(size_t)(G + row) * mp + (E * l) / (2 * t) + blk];
            }
        }
    }
    SLZ_HIP(hipMalloc((void **)dA, rowA.size() * sizeof(double)));
    SLZ_HIP(hipMalloc((void **)dB, rowB.size() * sizeof(double)));
    SLZ_HIP(hipMemcpy(*dA, rowA.data(), rowA.size() * sizeof(double), hipMemcpyHostToDevice));
    SLZ_HIP(hipMemcpy(*dB, rowB.data(), rowB.size() * sizeof(double), hipMemcpyHostToDevice));
    return SLZ_OK;
}

// worst-case bounds (units of p) of one block size: column stages start from digits, rows from reduced values
static bool bounds_ok(uint32_t N, uint32_t BS) {
    const uint32_t G = N / BS;
    double a = 1e-6;
    for (uint32_t g = G; g > 1; g >>= 1) a += slz_mulmod_bound(a);
    if (a > 7.5) return false;
    a = 0.5 + 1e-9;
    for (int s = 0; s < 6; s++) a += slz_mulmod_bound(a);        // block stages 1..6, then the reduction inside the wave transform
    if (a > 7.5) return false;
    a = 0.5 + 1e-9;
    for (int s = 0; s < (BS == 2048 ? 5 : 4); s++) a += slz_mulmod_bound(a);
    // sums over the GGSW rows are reduced after every fourth row
    if (0.5 + 4.0 * slz_mulmod_bound(a) > 7.5) return false;
    a = 0.5 + 1e-9;
    for (uint32_t g = G; g > 1; g >>= 1) a += slz_mulmod_bound(a);
    return slz_mulmod_bound(a) <= 1.95;
}

int slz_bign_init(slz_ctx *ctx) {
    const uint32_t N = ctx->prm.N;
    ctx->has_bign16 = 0;
    ctx->bign_block = 0;
    ctx->bign_lanes = 2;
    ctx->bign_latency = 1;
    bool any = false;
    if (block_fits(N, 2048) && bounds_ok(N, 2048)) {
        int rc = slz_build_block_tables(ctx, 2048, &ctx->bign_rowA, &ctx->bign_rowB);
        if (rc != SLZ_OK) return rc;
        SLZ_HIP(hipFuncSetAttribute((const void *)k_big_rows, hipFuncAttributeMaxDynamicSharedMemorySize, 4 * TBUF * sizeof(double)));
        ctx->bign_block = 2048;
        any = true;
    }
    if (block_fits(N, 1024) && bounds_ok(N, 1024)) {
        int rc = slz_build_block_tables(ctx, 1024, &ctx->bign16_rowA, &ctx->bign16_rowB);
        if (rc != SLZ_OK) return rc;
        SLZ_HIP(hipFuncSetAttribute((const void *)k_big_rows16<true>, hipFuncAttributeMaxDynamicSharedMemorySize, 4 * (TBUF16 + 1024) * sizeof(double)));
        SLZ_HIP(hipFuncSetAttribute((const void *)k_big_rows16<false>, hipFuncAttributeMaxDynamicSharedMemorySize, 4 * (TBUF16 + 1024) * sizeof(double)));
        SLZ_HIP(hipFuncSetAttribute((const void *)k_big_rows16_lat_a, hipFuncAttributeMaxDynamicSharedMemorySize, 4 * (TBUF16 + 1024) * sizeof(double)));
        SLZ_HIP(hipFuncSetAttribute((const void *)k_big_rows16_lat_b, hipFuncAttributeMaxDynamicSharedMemorySize, 4 * TBUF16 * sizeof(double)));
        ctx->has_bign16 = 1;
        ctx->bign_block = 1024;                                  // preferred: two waves per SIMD in the row pass
        any = true;
    }
    return any ? SLZ_OK : SLZ_E_UNSUPPORTED;
}

void slz_bign_destroy(slz_ctx *ctx) {
    if (ctx->bign_rowA) (void)hipFree(ctx->bign_rowA);
    if (ctx->bign_rowB) (void)hipFree(ctx->bign_rowB);
    if (ctx->bign16_rowA) (void)hipFree(ctx->bign16_rowA);
    if (ctx->bign16_rowB) (void)hipFree(ctx->bign16_rowB);
    if (ctx->bign_partial) (void)hipFree(ctx->bign_partial);
    ctx->bign_rowA = ctx->bign_rowB = ctx->bign16_rowA = ctx->bign16_rowB = ctx->bign_partial = nullptr;
    for (int j = 0; j < 2; j++) {
        if (ctx->bign_lane_stream[j]) (void)hipStreamDestroy((hipStream_t)ctx->bign_lane_stream[j]);
        if (ctx->bign_lane_done[j]) (void)hipEventDestroy((hipEvent_t)ctx->bign_lane_done[j]);
        ctx->bign_lane_stream[j] = ctx->bign_lane_done[j] = nullptr;
    }
    if (ctx->bign_fork) (void)hipEventDestroy((hipEvent_t)ctx->bign_fork);
    ctx->bign_fork = nullptr;
}

// mode 0: the throughput kernels; mode 1: the latency-oriented ones (forward pass split over levels and primes, inverse
// pass with the two primes of a column on neighbouring lanes)
template <int G, int BS>
static void launch_cols(bool fwd, int mode, const bign_args &A, uint32_t batch, hipStream_t s) {
    if (mode == 0) {
        dim3 grid(BS / 256, 2, batch);
        if (fwd) hipLaunchKernelGGL((k_big_cols_fwd<G, BS, false>), grid, dim3(256), 0, s, A);
        else hipLaunchKernelGGL((k_big_cols_inv<G, BS>), grid, dim3(256), 0, s, A);
    } else {
        if (fwd) hipLaunchKernelGGL((k_big_cols_fwd<G, BS, true>), dim3(BS / 256, 2 * A.l * 2, batch), dim3(256), 0, s, A);
        else hipLaunchKernelGGL((k_big_cols_inv_lat<G, BS>), dim3(BS / 128, 2, batch), dim3(256), 0, s, A);
    }
}

static void launch_cols_any(bool fwd, int mode, uint32_t G, uint32_t BS, const bign_args &A, uint32_t batch, hipStream_t s) {
    if (BS == 2048) {
        switch (G) {
            case 2: launch_cols<2, 2048>(fwd, mode, A, batch, s); break;
            case 4: launch_cols<4, 2048>(fwd, mode, A, batch, s); break;
            case 8: launch_cols<8, 2048>(fwd, mode, A, batch, s); break;
            case 16: launch_cols<16, 2048>(fwd, mode, A, batch, s); break;
            default: launch_cols<32, 2048>(fwd, mode, A, batch, s); break;
        }
    } else {
        switch (G) {
            case 2: launch_cols<2, 1024>(fwd, mode, A, batch, s); break;
            case 4: launch_cols<4, 1024>(fwd, mode, A, batch, s); break;
            case 8: launch_cols<8, 1024>(fwd, mode, A, batch, s); break;
            case 16: launch_cols<16, 1024>(fwd, mode, A, batch, s); break;
            default: launch_cols<32, 1024>(fwd, mode, A, batch, s); break;
        }
    }
}

// Streams and events of the concurrent lanes (created at the first use, default priority).
static int ensure_lanes(slz_ctx *ctx) {
    if (ctx->bign_lane_stream[0]) return SLZ_OK;
    for (int j = 0; j < 2; j++) {
        hipStream_t st;
        hipEvent_t ev;
        if (hipStreamCreateWithFlags(&st, hipStreamNonBlocking) != hipSuccess) return SLZ_E_HIP;
        ctx->bign_lane_stream[j] = st;
        if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) return SLZ_E_HIP;
        ctx->bign_lane_done[j] = ev;
    }
    hipEvent_t ev;
    if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) return SLZ_E_HIP;
    ctx->bign_fork = ev;
    return SLZ_OK;
}

// Ciphertexts the latency-oriented kernels are used for: while their row tasks (2 G per ciphertext) fill at most half of
// the 2048 resident-wave slots of the row pass.  Measured at N = 32768, us per CMux step against the throughput kernels:
// 34 / 47 at one ciphertext, 40 / 52 at 4, 41 / 57 at 8, 50 / 58 at 12, 53 / 61 at 16; from 20 on they are equal.
static uint32_t latency_max_batch(uint32_t G) { return 1024u / (2 * G) ? 1024u / (2 * G) : 1u; }
// Up to this many ciphertexts the row pass is cut into per-GGSW-row and per-component launches, above it into one launch
// of one-component tasks.
static uint32_t latency_split_rows_max(uint32_t G) { return 256u / (2 * G) ? 256u / (2 * G) : 1u; }

// Runs steps [0, n_steps) on accumulators that the caller has initialised in `acc` ([batch][2][N]).
int slz_bign_cmux_steps(slz_ctx *ctx, const uint64_t *lwe_in, const double *bskp, uint32_t n_steps, uint64_t *acc,
                        uint32_t batch, hipStream_t s) {
    const slz_params &p = ctx->prm;
    const uint32_t N = p.N, BS = (uint32_t)ctx->bign_block, G = N / BS, R = 2 * p.pbs_level;
    uint32_t logG = 0;
    while ((1u << logG) < G) logG++;
    // A handful of ciphertexts: every step in four shorter launches (1024-blocks only)
    const bool lat = ctx->bign_latency && BS == 1024 && batch <= latency_max_batch(G);
    if (lat && !ctx->bign_partial) {
        const size_t cts = ctx->max_batch < latency_max_batch(G) ? ctx->max_batch : latency_max_batch(G);
        void *buf = nullptr;
        if (slz_scratch_alloc(&buf, cts * 2 * R * 2 * N * sizeof(double)) != SLZ_OK) return SLZ_E_NOMEM;
        ctx->bign_partial = (double *)buf;
    }
    // Ciphertexts go through all steps in chunks whose workspace (X, Y, accumulators: (2R + 4 + 2) N doubles each) stays
    // in the 256 MB Infinity Cache; the key (read once per chunk and step) streams from HBM.
    const size_t per_ct = (size_t)(2 * R + 4 + 2) * N * 8;
    uint32_t chunk = (uint32_t)((size_t)224 * 1024 * 1024 / per_ct);
    const uint32_t slots = BS == 2048 ? 1024u : 2048u;              // resident row-pass waves: one or two per SIMD
    const uint32_t fill = slots / (2 * G) ? slots / (2 * G) : 1;     // ciphertexts whose row tasks fill the chip once
    chunk = chunk / fill * fill;
    if (chunk < fill) chunk = fill;
    // Two lanes: the chunk is cut in two halves that run on two streams, so that the row pass of one half (bound by
    // arithmetic) overlaps the column passes of the other (bound by memory).  Measured at N = 32768: 5 % faster than one
    // lane; three or four lanes of the same size overflow the Infinity Cache and are slower.
    uint32_t lanes = lat ? 1u : (uint32_t)ctx->bign_lanes;
    if (lanes >= 2) {
        uint32_t half = chunk / 2 / fill * fill;
        if (half < fill) half = fill;
        if (batch > half) chunk = half; else lanes = 1;
    }
    if (chunk > batch) chunk = batch;
    if (lanes >= 2) {
        int rc = ensure_lanes(ctx);
        if (rc != SLZ_OK) return rc;
        SLZ_HIP(hipEventRecord((hipEvent_t)ctx->bign_fork, s));
        for (uint32_t j = 0; j < lanes; j++) SLZ_HIP(hipStreamWaitEvent((hipStream_t)ctx->bign_lane_stream[j], (hipEvent_t)ctx->bign_fork, 0));
    }
    for (uint32_t g0 = 0; g0 < batch; g0 += lanes * chunk) {
        bign_args A[2];
        hipStream_t st[2];
        uint32_t n_tasks[2], nbs[2], used = 0;
        for (uint32_t j = 0; j < lanes; j++) {
            const uint32_t c0 = g0 + j * chunk;
            if (c0 >= batch) break;
            const uint32_t nb = (batch - c0 < chunk) ? batch - c0 : chunk;
            bign_args &a = A[j];
            a.lwe_in = lwe_in + (size_t)c0 * (p.n + 1);
            a.acc = acc + (size_t)c0 * 2 * N;
            a.X = ctx->xhat + (size_t)j * chunk * 2 * R * N;
            a.Y = ctx->outhat + (size_t)j * chunk * 2 * 2 * N;
            a.n = p.n; a.N = N; a.logG = logG; a.beta = p.pbs_base_log; a.l = p.pbs_level; a.batch = nb;
            for (int q = 0; q < 2; q++) {
                a.tab[q].fwd = ctx->tab[q].fwd;
                a.tab[q].rowA = (BS == 2048 ? ctx->bign_rowA : ctx->bign16_rowA) + (size_t)q * G * 64;
                a.tab[q].rowB = BS == 2048 ? ctx->bign_rowB + (size_t)q * G * 31 * 64 : ctx->bign16_rowB + (size_t)q * G * 15 * 64;
                a.tab[q].inv = ctx->tab[q].inv;
                a.tab[q].post = ctx->tab[q].post;
                a.mod[q] = ctx->mod[q];
            }
            a.p1inv_mod_p2 = ctx->p1inv_mod_p2;
            n_tasks[j] = nb * 2 * G;
            nbs[j] = nb;
            st[j] = lanes >= 2 ? (hipStream_t)ctx->bign_lane_stream[j] : s;
            used = j + 1;
        }
        for (uint32_t step = 0; step < n_steps; step++) {
            for (uint32_t j = 0; j < used; j++) {
                bign_args &a = A[j];
                a.step = step;
                a.bskp_step = bskp + (size_t)step * 2 * R * 2 * N;
                launch_cols_any(true, lat ? 1 : 0, G, BS, a, nbs[j], st[j]);
                if (lat && nbs[j] > latency_split_rows_max(G)) {
                    // upper part of the range: one launch of one-component row tasks
                    const uint32_t tc = n_tasks[j] * 2;
                    hipLaunchKernelGGL(k_big_rows16<false>, dim3((tc + 3) / 4), dim3(256), 4 * (TBUF16 + 1024) * sizeof(double), st[j], a, G,
                                       tc, 0);
                    launch_cols_any(false, 1, G, BS, a, nbs[j], st[j]);
                    continue;
                }
                if (lat) {
                    const uint32_t ta = n_tasks[j] * R, tb = n_tasks[j] * 2;
                    hipLaunchKernelGGL(k_big_rows16_lat_a, dim3((ta + 3) / 4), dim3(256), 4 * (TBUF16 + 1024) * sizeof(double), st[j], a,
                                       ctx->bign_partial, G, ta);
                    hipLaunchKernelGGL(k_big_rows16_lat_b, dim3((tb + 3) / 4), dim3(256), 4 * TBUF16 * sizeof(double), st[j], a,
                                       ctx->bign_partial, G, tb);
                    launch_cols_any(false, 1, G, BS, a, nbs[j], st[j]);
                    continue;
                }
                // the XCD-aware order needs the task count to split evenly over 8 XCDs x 4 waves x (2G/8) combinations
                const int xcd_aware = (2 * G) % 8 == 0 && n_tasks[j] % 32 == 0 && (n_tasks[j] / 8) % (2 * G / 8) == 0;
                if (BS == 2048)
                    hipLaunchKernelGGL(k_big_rows, dim3((n_tasks[j] + 3) / 4), dim3(256), 4 * TBUF * sizeof(double), st[j], a, G,
                                       n_tasks[j], xcd_aware);
                else
                    hipLaunchKernelGGL(k_big_rows16<true>, dim3((n_tasks[j] + 3) / 4), dim3(256), 4 * (TBUF16 + 1024) * sizeof(double), st[j], a,
                                       G, n_tasks[j], xcd_aware);
                launch_cols_any(false, 0, G, BS, a, nbs[j], st[j]);
            }
        }
    }
    if (lanes >= 2) {
        for (uint32_t j = 0; j < lanes; j++) {
            SLZ_HIP(hipEventRecord((hipEvent_t)ctx->bign_lane_done[j], (hipStream_t)ctx->bign_lane_stream[j]));
            SLZ_HIP(hipStreamWaitEvent(s, (hipEvent_t)ctx->bign_lane_done[j], 0));
        }
    }
    SLZ_HIP(hipGetLastError());
    return SLZ_OK;
}
