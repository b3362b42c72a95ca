// Fused blind rotation for N = 512, any base: l = 1 with k = 1 or 3 (k = 3 is the shape of 2-bit parameter sets), and
// k = 1 with l = 2 (second kernel, further down).
//
// One wavefront transforms two 512-point polynomials at once (the 1024-point wave transform without the stage that would
// pair them): in the coefficient domain registers 0..7 hold the first and 8..15 the second polynomial (coefficient
// 64 e + lane), in the transform domain lanes 0..31 hold the first and 32..63 the second (position 16 lane' + i).
// One workgroup of k + 1 wavefronts owns one ciphertext for the whole blind rotation.  Wave (q, hp): q = transform prime,
// hp = pair of GGSW rows / accumulator components (2 hp, 2 hp + 1).  It keeps 512 accumulator words in registers: for each
// of its two components the coefficients 64 (4 q + f) + lane, f < 4.  Per CMux step every wave
//   1. stages its accumulator words in LDS, reads the words it owns rotated by a~, subtracts, rounds, takes the signed
//      digit and hands the digits to the other prime's wave
//   2. forward transform of the two digit polynomials mod p_q
//   3. multiplies each by the k + 1 prepared key polynomials of its row; the two rows' products for a pair of columns are
//      added across the half-waves with one v_permlane32_swap (lanes 0..31 end up with the first column's sum, lanes
//      32..63 with the second's); the sums for the other wave's pair of columns go to it through LDS
//   4. inverse transform of its two columns and the psi^-j / N twist
//   5. exchanges half of the residues with the wave of the other prime, CRT-lifts its words and accumulates.
#include "slz_internal.h"
#include "slz_modarith.h"
#include "slz_fused_common.h"
#include <vector>

#include "slz_wave_ntt.h"

#define PN 512u
#define PLOGN 9u
#define P_STAGE_OFF 576u       // second half of a wave buffer: staging of 512 accumulator words
#define P_LDS_DOUBLES(P) (2u * (P) * TBUF16 + 2u * 1024u)

struct fused512_args : slz_fused_io {
    const double *rowA[2];    // [64]      forward twiddles of the stages before the transposition, both halves
    const double *rowB[2];    // [15][64]  per-lane forward twiddles of the last four stages
    double tw_inv[2][16];     // inv[t + j], t + j < 16
};

template <int K>
__global__ void __launch_bounds__(64 * (K + 1)) __attribute__((amdgpu_waves_per_eu(2, 2)))
k_fused_blind_rotate_n512(fused512_args A) {
    constexpr uint32_t C = K + 1, P = C / 2;          // components, pairs of components = waves per prime
    const uint32_t beta = A.beta;
    extern __shared__ double lds[];
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t q = w / P, hp = w % P;
    double *T = lds + w * TBUF16;                     // this wave's buffer
    double *Toth = lds + ((1u - q) * P + hp) * TBUF16;   // other prime, same pair
    const double *Tsib = lds + (q * P + (1u - hp)) * TBUF16;   // same prime, other pair (k = 3 only)
    double *twA = lds + 2u * P * TBUF16 + q * 1024u, *twB = twA + 64;
    if (hp == 0) {
        twA[lane] = A.rowA[q][lane];
#pragma unroll
        for (int k = 0; k < 15; k++) twB[64 * k + lane] = A.rowB[q][64 * k + lane];
    }
    __syncthreads();
    uint64_t *Smine = reinterpret_cast<uint64_t *>(T + P_STAGE_OFF);
    const slz_mod m = A.mod[q];
    const double *invt = A.inv[q], *post = A.post[q];
    const double *twS = A.tw_inv[q];
    const uint32_t hv = lane >> 5;                    // transform domain: which of my two polynomials this lane holds
    // transform-domain register i of lane l holds position idx = 16 (l & 31) + i of row 2 hp + hv; a prepared polynomial
    // keeps it at (idx % 32) 16 + idx / 32; the rows of a prime lie C N doubles apart
    const uint32_t key_lane_off = (hv * C * PN + 16u * (lane & 1u) * 16u + ((lane & 31u) >> 1)) * 8u;

    for (uint32_t c = blockIdx.x; c < A.batch; c += gridDim.x) {
        const uint64_t *lwe = A.lwe_in + (size_t)c * (A.n + 1);
        // ---- accumulator words: acc[4 t + f] = coefficient 64 (4 q + f) + lane of component 2 hp + t ----
        uint64_t acc[8];
#pragma unroll
        for (int u = 0; u < 8; u++) acc[u] = 0;
        if (hp == K / 2) {                            // the body component K is the second of the last pair
            const uint32_t bt = slz_modswitch(lwe[A.n], PLOGN + 1);
            const uint32_t r = (2 * PN - bt) & (2 * PN - 1);
            const uint64_t *lut = A.luts + (size_t)(A.lut_idx ? A.lut_idx[c] : 0) * PN;
#pragma unroll
            for (int f = 0; f < 4; f++)
                acc[4 + f] = slz_rot_coeff([&](uint32_t j) { return lut[j]; }, 64u * (4u * q + f) + lane, r, PN);
        }

        for (uint32_t step = 0; step < A.n_steps; step++) {
            // an opaque zero added to every table index keeps the per-lane table loads inside the step loop
            int z;
            asm volatile("s_mov_b32 %0, 0" : "=s"(z));
            const uint32_t at = slz_modswitch(lwe[step], PLOGN + 1);
            // [n][prime][row][comp][N]: row 2 hp of this prime; the lane offset moves the upper half-wave to row 2 hp + 1
            const double *krow = A.bskp + (((size_t)step * 2 + q) * C + 2u * hp) * C * PN + z;
            // 1. stage my words: slot u of the buffer of wave (q, hp)
#pragma unroll
            for (int u = 0; u < 8; u++) Smine[64 * u + lane] = acc[u];
            __syncthreads();
            int32_t dg[8];
            {
                uint32_t r = at, neg0 = 0;
                if (r >= PN) { r -= PN; neg0 = 1; }
                int32_t *pd = reinterpret_cast<int32_t *>(Toth);
#pragma unroll
                for (int u = 0; u < 8; u++) {
                    const uint32_t t = u >> 2, f = u & 3u;
                    const uint32_t idx = 64u * (4u * q + f) + lane;
                    const uint32_t j = (idx - r) & (PN - 1);
                    const uint32_t neg = neg0 ^ (idx < r ? 1u : 0u);
                    // word j of component 2 hp + t: wave (j >> 8, hp), slot 4 t + ((j >> 6) & 3), lane j & 63
                    const uint64_t *src = reinterpret_cast<const uint64_t *>(lds + ((j >> 8) * P + hp) * TBUF16 + P_STAGE_OFF);
                    const uint64_t a = src[64u * (4u * t + ((j >> 6) & 3u)) + (j & 63u)];
                    const uint64_t lam = (neg ? (uint64_t)0 - a : a) - acc[u];
                    uint64_t v = slz_round_top_bits(lam, beta);
                    dg[u] = slz_next_digit(v, beta);
                    pd[64 * u + lane] = dg[u];
                }
            }
            __syncthreads();                          // every wave has read the staged accumulator and sent its digits
            double x[16];
            {
                const int32_t *md = reinterpret_cast<const int32_t *>(T);
#pragma unroll
                for (int u = 0; u < 8; u++) {
                    const int t = u >> 2, f = u & 3;
                    if (q == 0) { x[8 * t + f] = (double)dg[u]; x[8 * t + 4 + f] = (double)md[64 * u + lane]; }
                    else { x[8 * t + 4 + f] = (double)dg[u]; x[8 * t + f] = (double)md[64 * u + lane]; }
                }
            }
            // 2. forward transform of both polynomials
            fwd16<true>(x, T, twA, twB, m, lane, z);
            // 3. products with the key polynomials of my rows, four positions at a time; sums of the two rows per column
            double xo[16];
            wave_sync();
#pragma unroll
            for (int g = 0; g < 4; g++) {
                double kk[C][4];
#pragma unroll
                for (int cc = 0; cc < (int)C; cc++)
#pragma unroll
                    for (int u = 0; u < 4; u++) kk[cc][u] = ldl(krow + (size_t)cc * PN + 16 * (4 * g + u), key_lane_off);
                const double x4[4] = {x[4 * g], x[4 * g + 1], x[4 * g + 2], x[4 * g + 3]};
#pragma unroll
                for (int pp = 0; pp < (int)P; pp++) {
                    double ra[4], rb[4];
                    mulmod_k<4>(ra, x4, kk[2 * pp], m);
                    mulmod_k<4>(rb, x4, kk[2 * pp + 1], m);
#pragma unroll
                    for (int u = 0; u < 4; u++) {
                        swap32(ra[u], rb[u]);         // ra: my first row's two products, rb: my second row's
                        const double sum = ra[u] + rb[u];
                        if (pp == (int)hp) xo[4 * g + u] = sum;
                        else T[64 * (4 * g + u) + lane] = sum;
                    }
                }
            }
            if (P == 2) {
                __syncthreads();
#pragma unroll
                for (int i = 0; i < 16; i++) xo[i] += Tsib[64 * i + lane];
            }
#pragma unroll
            for (int g = 0; g < 2; g++) {
                double r8[8], x8[8];
#pragma unroll
                for (int u = 0; u < 8; u++) x8[u] = xo[8 * g + u];
                reduce_k<8>(r8, x8, m);
#pragma unroll
                for (int u = 0; u < 8; u++) x[8 * g + u] = r8[u];
            }
            if (P == 2) __syncthreads();              // the other pair's wave has read my buffer before I reuse it
            // 4. inverse transform of my two columns, then the twist: register e holds coefficient 64 (e & 7) + lane
            double pw[8];
#pragma unroll
            for (int e = 0; e < 8; e++) pw[e] = ldl(post + 64 * e + z, lane * 8u);
            SCHED_FENCE();
            inv16<true>(x, T, twS, invt, m, lane, z);
#pragma unroll
            for (int g = 0; g < 4; g++) {
                double r4[4];
                const double x4[4] = {x[4 * g], x[4 * g + 1], x[4 * g + 2], x[4 * g + 3]};
                const double w4[4] = {pw[(4 * g) & 7], pw[(4 * g + 1) & 7], pw[(4 * g + 2) & 7], pw[(4 * g + 3) & 7]};
                mulmod_k<4>(r4, x4, w4, m);
#pragma unroll
                for (int u = 0; u < 4; u++) x[4 * g + u] = r4[u];
            }
            // 5. exchange the half I do not lift with the other prime's wave, CRT, accumulate
            wave_sync();
#pragma unroll
            for (int u = 0; u < 8; u++) {
                const int t = u >> 2, f = u & 3;
                T[64 * u + lane] = q == 0 ? x[8 * t + 4 + f] : x[8 * t + f];
            }
            __syncthreads();
#pragma unroll
            for (int u = 0; u < 8; u++) {
                const int t = u >> 2, f = u & 3;
                const double other = Toth[64 * u + lane];
                acc[u] += q == 0 ? slz_crt64(x[8 * t + f], other, A.mod[1], A.p1inv_mod_p2)
                                 : slz_crt64(other, x[8 * t + 4 + f], A.mod[1], A.p1inv_mod_p2);
            }
        }

        // ---- output: accumulator, or the extracted LWE ciphertext ----
#pragma unroll
        for (int u = 0; u < 8; u++) {
            const uint32_t comp = 2u * hp + (u >> 2), idx = 64u * (4u * q + (u & 3u)) + lane;
            if (A.acc_out) A.acc_out[((size_t)c * C + comp) * PN + idx] = acc[u];
            if (A.lwe_out) {
                uint64_t *dst = A.lwe_out + (size_t)c * (K * PN + 1);
                if (comp < (uint32_t)K) {             // mask component: a'[comp N] = ACC[0], a'[comp N + N - j] = -ACC[j]
                    if (idx == 0) dst[comp * PN] = acc[u];
                    else dst[comp * PN + PN - idx] = (uint64_t)0 - acc[u];
                } else if (idx == 0) {
                    dst[K * PN] = acc[u];
                }
            }
        }
        __syncthreads();                              // the next ciphertext reuses the LDS buffers
    }
}

// ---- k = 1, l = 2 (the shape of the smallest configuration) ------------------------------------------------------------
// Four waves (q, h): the two polynomials of a wave are the two decomposition levels of component h (GGSW rows (h, 0) and
// (h, 1)).  Each wave keeps 256 accumulator words (coefficients 64 (4 q + f) + lane of component h).  The products of both
// levels with the two key columns are added across the half-waves as above; the waves of component 1 hand their sums to
// the waves of component 0, which run the one inverse transform per prime (both columns at once) and leave the residues
// in LDS for the CRT lift of all four waves.
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
k_fused_blind_rotate_n512_l2(fused512_args A) {
    const uint32_t beta = A.beta;
    extern __shared__ double lds[];
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t q = w >> 1, h = w & 1u;
    double *T = lds + w * TBUF16;
    double *Toth = lds + (w ^ 2u) * TBUF16;           // other prime, same component
    const double *Tsib = lds + (w ^ 1u) * TBUF16;     // same prime, other component
    const double *Tres0 = lds, *Tres1 = lds + 2u * TBUF16;   // residues of prime 0 / prime 1: buffers of waves (0,0) and (1,0)
    double *twA = lds + 4u * TBUF16 + q * 1024u, *twB = twA + 64;
    if (h == 0) {
        twA[lane] = A.rowA[q][lane];
#pragma unroll
        for (int k = 0; k < 15; k++) twB[64 * k + lane] = A.rowB[q][64 * k + lane];
    }
    __syncthreads();
    uint64_t *Smine = reinterpret_cast<uint64_t *>(T + P_STAGE_OFF);
    const slz_mod m = A.mod[q];
    const double *invt = A.inv[q], *post = A.post[q];
    const double *twS = A.tw_inv[q];
    const uint32_t hv = lane >> 5;                    // transform domain: decomposition level held by this lane
    const uint32_t key_lane_off = (hv * 2u * PN + 16u * (lane & 1u) * 16u + ((lane & 31u) >> 1)) * 8u;

    for (uint32_t c = blockIdx.x; c < A.batch; c += gridDim.x) {
        const uint64_t *lwe = A.lwe_in + (size_t)c * (A.n + 1);
        uint64_t acc[4];
        if (h == 1) {
            const uint32_t bt = slz_modswitch(lwe[A.n], PLOGN + 1);
            const uint32_t r = (2 * PN - bt) & (2 * PN - 1);
            const uint64_t *lut = A.luts + (size_t)(A.lut_idx ? A.lut_idx[c] : 0) * PN;
#pragma unroll
            for (int f = 0; f < 4; f++)
                acc[f] = slz_rot_coeff([&](uint32_t j) { return lut[j]; }, 64u * (4u * q + f) + lane, r, PN);
        } else {
#pragma unroll
            for (int f = 0; f < 4; f++) acc[f] = 0;
        }

        for (uint32_t step = 0; step < A.n_steps; step++) {
            int z;
            asm volatile("s_mov_b32 %0, 0" : "=s"(z));
            const uint32_t at = slz_modswitch(lwe[step], PLOGN + 1);
            // [n][prime][row = 2 comp + level][comp][N]: row (h, 0); the lane offset moves the upper half-wave to row (h, 1)
            const double *krow = A.bskp + (((size_t)step * 2 + q) * 4 + 2u * h) * 2 * PN + z;
#pragma unroll
            for (int f = 0; f < 4; f++) Smine[64 * f + lane] = acc[f];
            __syncthreads();
            int32_t dg[8];                            // dg[4 level + f]
            {
                uint32_t r = at, neg0 = 0;
                if (r >= PN) { r -= PN; neg0 = 1; }
                int32_t *pd = reinterpret_cast<int32_t *>(Toth);
#pragma unroll
                for (int f = 0; f < 4; f++) {
                    const uint32_t idx = 64u * (4u * q + f) + lane;
                    const uint32_t j = (idx - r) & (PN - 1);
                    const uint32_t neg = neg0 ^ (idx < r ? 1u : 0u);
                    const uint64_t *src = reinterpret_cast<const uint64_t *>(lds + ((j >> 8) * 2u + h) * TBUF16 + P_STAGE_OFF);
                    const uint64_t a = src[64u * ((j >> 6) & 3u) + (j & 63u)];
                    const uint64_t lam = (neg ? (uint64_t)0 - a : a) - acc[f];
                    uint64_t v = slz_round_top_bits(lam, 2 * beta);
                    dg[4 + f] = slz_next_digit(v, beta);         // least significant level first: the carry goes up
                    dg[f] = slz_next_digit(v, beta);
                    pd[64 * f + lane] = dg[f];
                    pd[64 * (4 + f) + lane] = dg[4 + f];
                }
            }
            __syncthreads();
            double x[16];
            {
                const int32_t *md = reinterpret_cast<const int32_t *>(T);
#pragma unroll
                for (int u = 0; u < 8; u++) {
                    const int lev = u >> 2, f = u & 3;
                    if (q == 0) { x[8 * lev + f] = (double)dg[u]; x[8 * lev + 4 + f] = (double)md[64 * u + lane]; }
                    else { x[8 * lev + 4 + f] = (double)dg[u]; x[8 * lev + f] = (double)md[64 * u + lane]; }
                }
            }
            fwd16<true>(x, T, twA, twB, m, lane, z);
            wave_sync();
#pragma unroll
            for (int g = 0; g < 4; g++) {
                double k0[4], k1[4], ra[4], rb[4];
#pragma unroll
                for (int u = 0; u < 4; u++) {
                    k0[u] = ldl(krow + 16 * (4 * g + u), key_lane_off);
                    k1[u] = ldl(krow + PN + 16 * (4 * g + u), key_lane_off);
                }
                const double x4[4] = {x[4 * g], x[4 * g + 1], x[4 * g + 2], x[4 * g + 3]};
                mulmod_k<4>(ra, x4, k0, m);
                mulmod_k<4>(rb, x4, k1, m);
#pragma unroll
                for (int u = 0; u < 4; u++) {
                    swap32(ra[u], rb[u]);
                    x[4 * g + u] = ra[u] + rb[u];     // lanes 0..31: column 0 summed over the levels, lanes 32..63: column 1
                    if (h == 1) T[64 * (4 * g + u) + lane] = x[4 * g + u];
                }
            }
            __syncthreads();
            if (h == 0) {
#pragma unroll
                for (int g = 0; g < 2; g++) {
                    double r8[8], x8[8];
#pragma unroll
                    for (int u = 0; u < 8; u++) x8[u] = x[8 * g + u] + Tsib[64 * (8 * g + u) + lane];
                    reduce_k<8>(r8, x8, m);
#pragma unroll
                    for (int u = 0; u < 8; u++) x[8 * g + u] = r8[u];
                }
                double pw[8];
#pragma unroll
                for (int e = 0; e < 8; e++) pw[e] = ldl(post + 64 * e + z, lane * 8u);
                SCHED_FENCE();
                inv16<true>(x, T, twS, invt, m, lane, z);
                wave_sync();
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    double r4[4];
                    const double x4[4] = {x[4 * g], x[4 * g + 1], x[4 * g + 2], x[4 * g + 3]};
                    const double w4[4] = {pw[(4 * g) & 7], pw[(4 * g + 1) & 7], pw[(4 * g + 2) & 7], pw[(4 * g + 3) & 7]};
                    mulmod_k<4>(r4, x4, w4, m);
#pragma unroll
                    for (int u = 0; u < 4; u++) T[64 * (4 * g + u) + lane] = r4[u];   // register 8 comp + e: coefficient 64 e + lane
                }
            }
            __syncthreads();
#pragma unroll
            for (int f = 0; f < 4; f++) {
                const uint32_t slot = 64u * (8u * h + 4u * q + f) + lane;
                acc[f] += slz_crt64(Tres0[slot], Tres1[slot], A.mod[1], A.p1inv_mod_p2);
            }
            __syncthreads();                          // residues are read before the next step stages into the same buffers
        }

#pragma unroll
        for (int f = 0; f < 4; f++) {
            const uint32_t idx = 64u * (4u * q + f) + lane;
            if (A.acc_out) A.acc_out[((size_t)c * 2 + h) * PN + idx] = acc[f];
            if (A.lwe_out) {
                uint64_t *dst = A.lwe_out + (size_t)c * (PN + 1);
                if (h == 0) {
                    if (idx == 0) dst[0] = acc[f];
                    else dst[PN - idx] = (uint64_t)0 - acc[f];
                } else if (idx == 0) {
                    dst[PN] = acc[f];
                }
            }
        }
        __syncthreads();
    }
}

// ---- host side -----------------------------------------------------------------------------------

int slz_fused512_supported(const slz_params *p) {
    if (p->N != PN || p->pbs_base_log > 30) return 0;
    return ((p->k == 1 || p->k == 3) && p->pbs_level == 1) || (p->k == 1 && p->pbs_level == 2);
}

// Forward tables of the paired transform: the stage of the 1024-point schedule that works on m' sub-blocks of the whole
// array works on m' / 2 sub-blocks of each 512-point polynomial, and both halves take the same twiddles.
static int build_pair_tables(slz_ctx *ctx, double **dA, double **dB) {
    std::vector<double> nat(PN), rowA((size_t)2 * 64), rowB((size_t)2 * 15 * 64);
    for (int q = 0; q < 2; q++) {
        SLZ_HIP(hipMemcpy(nat.data(), ctx->tab[q].fwd, PN * sizeof(double), hipMemcpyDeviceToHost));
        double *ra = &rowA[(size_t)q * 64];
        ra[0] = ra[1] = 1.0;                           // index 1 would be the left-out pairing stage
        for (uint32_t x = 2; x < 64; x++) {
            uint32_t mp = 1;
            while (mp * 2 <= x) mp *= 2;
            const uint32_t mh = mp / 2;
            ra[x] = nat[mh + (x - mp) % mh];
        }
        int kk = 0;
        for (int s = 0; s < 4; s++) {
            const uint32_t t = 8u >> s, mp = 1024u / (2 * t), mh = mp / 2;
            for (uint32_t blk = 0; blk < (1u << s); blk++, kk++)
                for (uint32_t l = 0; l < 64; l++)
                    rowB[((size_t)q * 15 + kk) * 64 + l] = nat[mh + ((16 * l) / (2 * t) + blk) % mh];
        }
    }
    SLZ_HIP(hipMalloc((void **)dA, rowA.size() * sizeof(double)));
    SLZ_HIP(hipMalloc((void **)dB, rowB.size() * sizeof(double)));
    SLZ_HIP(hipMemcpy(*dA, rowA.data(), rowA.size() * sizeof(double), hipMemcpyHostToDevice));
    SLZ_HIP(hipMemcpy(*dB, rowB.data(), rowB.size() * sizeof(double), hipMemcpyHostToDevice));
    return SLZ_OK;
}

int slz_fused512_init(slz_ctx *ctx) {
    // five forward stages on the digits, reduction, four more; four products summed (k = 3); inverse 2 + 2 stages,
    // reduction, five stages, twist
    if (!slz_fused_schedule_ok(0, 5, 4, 4, 2, 5, false, 1)) return SLZ_E_UNSUPPORTED;
    int rc = build_pair_tables(ctx, &ctx->fused512_rowA, &ctx->fused512_rowB);
    if (rc != SLZ_OK) return rc;
    rc = slz_fused_load_inv_scalars(ctx);
    if (rc != SLZ_OK) return rc;
    SLZ_HIP(hipFuncSetAttribute((const void *)k_fused_blind_rotate_n512<1>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                P_LDS_DOUBLES(1) * sizeof(double)));
    SLZ_HIP(hipFuncSetAttribute((const void *)k_fused_blind_rotate_n512<3>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                P_LDS_DOUBLES(2) * sizeof(double)));
    SLZ_HIP(hipFuncSetAttribute((const void *)k_fused_blind_rotate_n512_l2, hipFuncAttributeMaxDynamicSharedMemorySize,
                                P_LDS_DOUBLES(2) * sizeof(double)));
    return SLZ_OK;
}

void slz_fused512_destroy(slz_ctx *ctx) {
    if (ctx->fused512_rowA) (void)hipFree(ctx->fused512_rowA);
    if (ctx->fused512_rowB) (void)hipFree(ctx->fused512_rowB);
    ctx->fused512_rowA = ctx->fused512_rowB = nullptr;
}

int slz_fused512_blind_rotate(slz_ctx *ctx, const uint64_t *lwe_in, const uint64_t *luts, const uint32_t *lut_idx,
                              const double *bskp, uint32_t n_steps, uint64_t *acc_out, uint64_t *lwe_out, uint32_t batch,
                              hipStream_t s) {
    fused512_args A;
    slz_fused_fill_io(A, ctx, lwe_in, luts, lut_idx, bskp, n_steps, acc_out, lwe_out, batch);
    for (int q = 0; q < 2; q++) {
        A.rowA[q] = ctx->fused512_rowA + (size_t)q * 64;
        A.rowB[q] = ctx->fused512_rowB + (size_t)q * 15 * 64;
        for (int x = 0; x < 16; x++) A.tw_inv[q][x] = ctx->fused_scalars[q][1][x];
    }
    if (ctx->prm.pbs_level == 2) {
        const uint32_t grid = slz_fused_grid(batch, 2);
        hipLaunchKernelGGL(k_fused_blind_rotate_n512_l2, dim3(grid), dim3(256), P_LDS_DOUBLES(2) * sizeof(double), s, A);
    } else if (ctx->prm.k == 3) {
        const uint32_t grid = slz_fused_grid(batch, 2);    // four waves per workgroup, two waves per SIMD
        hipLaunchKernelGGL(k_fused_blind_rotate_n512<3>, dim3(grid), dim3(256), P_LDS_DOUBLES(2) * sizeof(double), s, A);
    } else {
        const uint32_t grid = slz_fused_grid(batch, 4);    // two waves per workgroup
        hipLaunchKernelGGL(k_fused_blind_rotate_n512<1>, dim3(grid), dim3(128), P_LDS_DOUBLES(1) * sizeof(double), s, A);
    }
    SLZ_HIP(hipGetLastError());
    return SLZ_OK;
}
