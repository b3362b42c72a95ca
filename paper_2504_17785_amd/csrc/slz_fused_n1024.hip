// Fused blind rotation for N = 1024, l = 1, k = 1 or 2, any base: the N = 2048 kernel's design on the 16-coefficient-per-lane
// wave transform.
//
// One workgroup of 2 (k + 1) wavefronts owns one ciphertext for the whole blind rotation; the accumulator never leaves the
// chip.  Wave (q, h): q = transform prime, h = GGSW row = accumulator component; each wave keeps 512 accumulator words
// (8 per lane) in registers.  Per CMux step every wave
//   1. stages its accumulator words in LDS, reads its half of component h rotated by a~, subtracts, rounds, takes the
//      signed digit and hands the digits to the other prime's wave
//   2. forward transform of the digit polynomial mod p_q (fwd16: one wave = one polynomial)
//   3. multiplies by the k + 1 prepared key polynomials of row h, keeps the product for component h and hands the others
//      to the sibling waves through LDS (k = 2: one sibling at a time); sums and reduces
//   4. inverse transform (inv16) and the psi^-j / N twist
//   5. exchanges half of the residues with the wave of the other prime, CRT-lifts its half of component h and adds it
//      to its accumulator words.
// The forward twiddle tables of both primes (2 x 1024 doubles) are staged in LDS once per workgroup.
#include "slz_internal.h"
#include "slz_modarith.h"
#include "slz_fused_common.h"
#include <vector>

#include "slz_wave_ntt.h"

#define GN 1024u
#define GLOGN 10u
#define G_THREADS 256
#ifndef G_WAVES
#define G_WAVES 3           // waves per SIMD = workgroups per compute unit (3 x 52 KiB of LDS fit the 160 KiB); measured 5-10 % faster than 2
#endif
#define G_STAGE_OFF 576u       // second half of a wave buffer: staging of 512 accumulator words
#define G_LDS_DOUBLES(C) (2u * (C) * TBUF16 + 2u * 1024u)

struct fused1024_args : slz_fused_io {
    const double *rowA[2];    // [64]      lane-uniform and half-wave / row twiddles of the first six forward stages
    const double *rowB[2];    // [15][64]  per-lane twiddles of the last four forward stages
    double tw_inv[2][16];     // inv[t + j], t + j < 16: lane-uniform inverse twiddles (scalar loads)
};

template <int BETA, int K>
__global__ void __launch_bounds__(128 * (K + 1)) __attribute__((amdgpu_waves_per_eu(G_WAVES, G_WAVES)))
k_fused_blind_rotate_n1024(fused1024_args A) {
    constexpr uint32_t C = K + 1;                    // accumulator components = GGSW rows
    const uint32_t beta = BETA > 0 ? (uint32_t)BETA : A.beta;
    extern __shared__ double lds[];
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t q = w / C, h = w % C;
    double *T = lds + w * TBUF16;                    // this wave's buffer
    double *Toth = lds + ((1u - q) * C + h) * TBUF16;   // other prime, same row
    double *twA = lds + 2u * C * TBUF16 + q * 1024u, *twB = twA + 64;
    if (h == 0) {
        twA[lane] = A.rowA[q][lane];
#pragma unroll
        for (int k = 0; k < 15; k++) twB[64 * k + lane] = A.rowB[q][64 * k + lane];
    }
    __syncthreads();
    // staged ACC_h: words 0..511 in the buffer of wave (0,h), words 512..1023 in the buffer of wave (1,h)
    const uint64_t *Sh = reinterpret_cast<const uint64_t *>(lds + h * TBUF16 + G_STAGE_OFF);
    const double *Tsib = lds + (q * C + (h + C - 1u) % C) * TBUF16;    // same prime, the row before mine: it keeps my column first
    uint64_t *Smine = reinterpret_cast<uint64_t *>(T + G_STAGE_OFF);
    const slz_mod m = A.mod[q];
    const double *invt = A.inv[q], *post = A.post[q];
    const double *twS = A.tw_inv[q];
    // register i of lane l holds spectrum index 16 l + i, stored at position (idx % 32) 32 + idx / 32 of a prepared polynomial
    const uint32_t key_lane_off = (16u * (lane & 1u) * 32u + (lane >> 1)) * 8u;

    for (uint32_t c = blockIdx.x; c < A.batch; c += gridDim.x) {
        const uint64_t *lwe = A.lwe_in + (size_t)c * (A.n + 1);
        // ---- accumulator words: coefficients 64 (8 q + e) + lane of component h ----
        uint64_t acc[8];
        if (h == K) {
            const uint32_t bt = slz_modswitch(lwe[A.n], GLOGN + 1);
            const uint32_t r = (2 * GN - bt) & (2 * GN - 1);
            const uint64_t *lut = A.luts + (size_t)(A.lut_idx ? A.lut_idx[c] : 0) * GN;
#pragma unroll
            for (int e = 0; e < 8; e++)
                acc[e] = slz_rot_coeff([&](uint32_t j) { return lut[j]; }, 64u * (8u * q + e) + lane, r, GN);
        } else {
#pragma unroll
            for (int e = 0; e < 8; e++) acc[e] = 0;
        }

        for (uint32_t step = 0; step < A.n_steps; step++) {
            // an opaque zero added to every table index keeps the per-lane table loads inside the step loop
            int z;
            asm volatile("s_mov_b32 %0, 0" : "=s"(z));
            const uint32_t at = slz_modswitch(lwe[step], GLOGN + 1);
            const double *krow = A.bskp + (((size_t)step * 2 + q) * C + h) * C * GN + z;   // [n][prime][row][comp][N]
            const double *kown = krow + (size_t)h * GN, *ksib = krow + (size_t)((h + 1u) % C) * GN;
            // 1. stage my words, then read my half of component h rotated and unrotated
#pragma unroll
            for (int e = 0; e < 8; e++) Smine[64 * e + lane] = acc[e];
            __syncthreads();
            int32_t dg[8];
            {
                uint32_t r = at, neg0 = 0;
                if (r >= GN) { r -= GN; neg0 = 1; }
                int32_t *pd = reinterpret_cast<int32_t *>(Toth);
#pragma unroll
                for (int e = 0; e < 8; e++) {
                    const uint32_t idx = 512u * q + 64u * e + lane;
                    const uint32_t j = (idx - r) & (GN - 1);
                    const uint32_t neg = neg0 ^ (idx < r ? 1u : 0u);
                    const uint64_t a = Sh[(j >> 9) * (C * TBUF16) + (j & 511u)];
                    const uint64_t lam = (neg ? (uint64_t)0 - a : a) - acc[e];
                    uint64_t v = slz_round_top_bits(lam, beta);
                    dg[e] = slz_next_digit(v, beta);
                    pd[64 * e + lane] = dg[e];
                }
            }
            __syncthreads();                          // every wave has read the staged accumulator and sent its digits
            double x[16];
            {
                const int32_t *md = reinterpret_cast<const int32_t *>(T);
                if (q == 0) {
#pragma unroll
                    for (int e = 0; e < 8; e++) { x[e] = (double)dg[e]; x[8 + e] = (double)md[64 * e + lane]; }
                } else {
#pragma unroll
                    for (int e = 0; e < 8; e++) { x[8 + e] = (double)dg[e]; x[e] = (double)md[64 * e + lane]; }
                }
            }
            // the first half of this step's key words is requested here and arrives while the transform runs; the second
            // half is requested after the transform and arrives during the products of the first
            double ks[2][8], ko[2][8];
#pragma unroll
            for (int i = 0; i < 8; i++) { ks[0][i] = ldl(ksib + 32 * i, key_lane_off); ko[0][i] = ldl(kown + 32 * i, key_lane_off); }
            SCHED_FENCE();
            // 2. forward transform
            fwd16(x, T, twA, twB, m, lane, z);
            SCHED_FENCE();
#pragma unroll
            for (int i = 0; i < 8; i++) { ks[1][i] = ldl(ksib + 32 * (8 + i), key_lane_off); ko[1][i] = ldl(kown + 32 * (8 + i), key_lane_off); }
            SCHED_FENCE();
            // 3. row h of the GGSW times the digits: component h stays, component h + 1 goes to the sibling after mine
            //    (k = 2: the spectrum is kept for the second sibling's exchange)
            double xs[K == 2 ? 16 : 1];
            if (K == 2) {
#pragma unroll
                for (int i = 0; i < 16; i++) xs[i] = x[i];
            }
            wave_sync();
#pragma unroll
            for (int ch = 0; ch < 2; ch++) {
#pragma unroll
                for (int i = 0; i < 8; i += 2) {
                    double r4[4];
                    const double x4[4] = {x[8 * ch + i], x[8 * ch + i], x[8 * ch + i + 1], x[8 * ch + i + 1]};
                    const double w4[4] = {ks[ch][i], ko[ch][i], ks[ch][i + 1], ko[ch][i + 1]};
                    mulmod_k<4>(r4, x4, w4, m);
                    T[64 * (8 * ch + i) + lane] = r4[0];
                    x[8 * ch + i] = r4[1];
                    T[64 * (8 * ch + i + 1) + lane] = r4[2];
                    x[8 * ch + i + 1] = r4[3];
                }
                SCHED_FENCE();
            }
            __syncthreads();
#pragma unroll
            for (int g = 0; g < 2; g++) {
                double r8[8], x8[8];
#pragma unroll
                for (int u = 0; u < 8; u++) x8[u] = x[8 * g + u] + Tsib[64 * (8 * g + u) + lane];
                reduce_k<8>(r8, x8, m);
#pragma unroll
                for (int u = 0; u < 8; u++) x[8 * g + u] = r8[u];
            }
            __syncthreads();                          // sibling has read my buffer before I reuse it
            if (K == 2) {
                // second exchange: the product for component h + 2 through the same buffer; mine comes from the row after mine
                const double *k2 = krow + (size_t)((h + 2u) % C) * GN;
                const double *Tsib2 = lds + (q * C + (h + 1u) % C) * TBUF16;
                double kt[16];
#pragma unroll
                for (int i = 0; i < 16; i++) kt[i] = ldl(k2 + 32 * i, key_lane_off);
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    double r4[4];
                    const double x4[4] = {xs[4 * g], xs[4 * g + 1], xs[4 * g + 2], xs[4 * g + 3]};
                    const double w4[4] = {kt[4 * g], kt[4 * g + 1], kt[4 * g + 2], kt[4 * g + 3]};
                    mulmod_k<4>(r4, x4, w4, m);
#pragma unroll
                    for (int u = 0; u < 4; u++) T[64 * (4 * g + u) + lane] = r4[u];
                }
                __syncthreads();
#pragma unroll
                for (int g = 0; g < 2; g++) {
                    double r8[8], x8[8];
#pragma unroll
                    for (int u = 0; u < 8; u++) x8[u] = x[8 * g + u] + Tsib2[64 * (8 * g + u) + lane];
                    reduce_k<8>(r8, x8, m);
#pragma unroll
                    for (int u = 0; u < 8; u++) x[8 * g + u] = r8[u];
                }
                __syncthreads();
            }
            // 4. inverse transform, then the twist: coefficient 64 e + lane times psi^-(64 e + lane) / N
            double pw[16];
#pragma unroll
            for (int e = 0; e < 16; e++) pw[e] = ldl(post + 64 * e + z, lane * 8u);
            SCHED_FENCE();
            inv16(x, T, twS, invt, m, lane, z);
#pragma unroll
            for (int g = 0; g < 4; g++) {
                double r4[4];
                const double x4[4] = {x[4 * g], x[4 * g + 1], x[4 * g + 2], x[4 * g + 3]};
                const double w4[4] = {pw[4 * g], pw[4 * g + 1], pw[4 * g + 2], pw[4 * g + 3]};
                mulmod_k<4>(r4, x4, w4, m);
#pragma unroll
                for (int u = 0; u < 4; u++) x[4 * g + u] = r4[u];
            }
            // 5. exchange the half I do not lift with the other prime's wave, CRT, accumulate
            wave_sync();
            if (q == 0) {
#pragma unroll
                for (int e = 0; e < 8; e++) T[64 * e + lane] = x[8 + e];
            } else {
#pragma unroll
                for (int e = 0; e < 8; e++) T[64 * e + lane] = x[e];
            }
            __syncthreads();
            if (q == 0) {
#pragma unroll
                for (int e = 0; e < 8; e++) acc[e] += slz_crt64(x[e], Toth[64 * e + lane], A.mod[1], A.p1inv_mod_p2);
            } else {
#pragma unroll
                for (int e = 0; e < 8; e++) acc[e] += slz_crt64(Toth[64 * e + lane], x[8 + e], A.mod[1], A.p1inv_mod_p2);
            }
        }

        // ---- output: accumulator, or the extracted LWE ciphertext ----
        if (A.acc_out) {
            uint64_t *dst = A.acc_out + ((size_t)c * C + h) * GN;
#pragma unroll
            for (int e = 0; e < 8; e++) dst[64u * (8u * q + e) + lane] = acc[e];
        }
        if (A.lwe_out) {
            uint64_t *dst = A.lwe_out + (size_t)c * (K * GN + 1);
            if (h < K) {                              // mask component h: a'[h N] = ACC_h[0], a'[h N + N - j] = -ACC_h[j]
#pragma unroll
                for (int e = 0; e < 8; e++) {
                    const uint32_t idx = 64u * (8u * q + e) + lane;
                    if (idx == 0) dst[h * GN] = acc[e];
                    else dst[h * GN + GN - idx] = (uint64_t)0 - acc[e];
                }
            } else if (q == 0 && lane == 0) {
                dst[K * GN] = acc[0];
            }
        }
        __syncthreads();                              // the next ciphertext reuses the LDS buffers
    }
}

// ---- host side -----------------------------------------------------------------------------------

int slz_fused1024_supported(const slz_params *p) {
    return p->N == GN && (p->k == 1 || p->k == 2) && p->pbs_level == 1 && p->pbs_base_log <= 30;
}

int slz_fused1024_init(slz_ctx *ctx) {
    // six forward stages on the digits, reduction, four more; two products summed; inverse 2 + 2 stages, reduction, six
    // stages, twist
    if (!slz_fused_schedule_ok(0, 6, 4, 2, 2, 6, false, 1)) return SLZ_E_UNSUPPORTED;
    int rc = slz_build_block_tables(ctx, GN, &ctx->fused1024_rowA, &ctx->fused1024_rowB);
    if (rc != SLZ_OK) return rc;
    rc = slz_fused_load_inv_scalars(ctx);
    if (rc != SLZ_OK) return rc;
    SLZ_HIP(hipFuncSetAttribute((const void *)k_fused_blind_rotate_n1024<23, 1>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                G_LDS_DOUBLES(2) * sizeof(double)));
    SLZ_HIP(hipFuncSetAttribute((const void *)k_fused_blind_rotate_n1024<0, 1>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                G_LDS_DOUBLES(2) * sizeof(double)));
    SLZ_HIP(hipFuncSetAttribute((const void *)k_fused_blind_rotate_n1024<0, 2>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                G_LDS_DOUBLES(3) * sizeof(double)));
    return SLZ_OK;
}

void slz_fused1024_destroy(slz_ctx *ctx) {
    if (ctx->fused1024_rowA) (void)hipFree(ctx->fused1024_rowA);
    if (ctx->fused1024_rowB) (void)hipFree(ctx->fused1024_rowB);
    ctx->fused1024_rowA = ctx->fused1024_rowB = nullptr;
}

int slz_fused1024_blind_rotate(slz_ctx *ctx, const uint64_t *lwe_in, const uint64_t *luts, const uint32_t *lut_idx,
                               const double *bskp, uint32_t n_steps, uint64_t *acc_out, uint64_t *lwe_out, uint32_t batch,
                               hipStream_t s) {
    fused1024_args A;
    slz_fused_fill_io(A, ctx, lwe_in, luts, lut_idx, bskp, n_steps, acc_out, lwe_out, batch);
    for (int q = 0; q < 2; q++) {
        A.rowA[q] = ctx->fused1024_rowA + (size_t)q * 64;
        A.rowB[q] = ctx->fused1024_rowB + (size_t)q * 15 * 64;
        for (int x = 0; x < 16; x++) A.tw_inv[q][x] = ctx->fused_scalars[q][1][x];
    }
    if (ctx->prm.k == 2) {
        const uint32_t grid = slz_fused_grid(batch, 2);    // six waves and 70 KiB of LDS per workgroup: two per compute unit
        hipLaunchKernelGGL((k_fused_blind_rotate_n1024<0, 2>), dim3(grid), dim3(384), G_LDS_DOUBLES(3) * sizeof(double), s, A);
    } else {
        const uint32_t grid = slz_fused_grid(batch, G_WAVES);
        if (A.beta == 23)
            hipLaunchKernelGGL((k_fused_blind_rotate_n1024<23, 1>), dim3(grid), dim3(G_THREADS), G_LDS_DOUBLES(2) * sizeof(double), s, A);
        else
            hipLaunchKernelGGL((k_fused_blind_rotate_n1024<0, 1>), dim3(grid), dim3(G_THREADS), G_LDS_DOUBLES(2) * sizeof(double), s, A);
    }
    SLZ_HIP(hipGetLastError());
    return SLZ_OK;
}
