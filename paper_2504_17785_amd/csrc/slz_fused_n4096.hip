// Fused blind rotation for N = 4096, k = 1, l = 1, any base: one workgroup of eight wavefronts owns one ciphertext for the
// whole blind rotation; the accumulator (64 KiB) never leaves the chip.
//
// Wave (b, q, h): b = 2048-block of the transform, q = transform prime, h = GGSW row = accumulator component.  Each wave
// keeps 1024 accumulator words (16 per lane) in registers: coefficients 2048 b + 1024 q + 64 e + lane of component h.
// Per CMux step every wave
//   1. stages its accumulator words in LDS, reads the words it owns rotated by a~, subtracts, rounds, takes the signed
//      digit and leaves the digits in LDS for the four waves (both primes, both blocks) that transform row h
//   2. first forward stage across the two blocks (coefficient c with c + 2048), then the 2048-point wave transform of its
//      block with the block's twiddle tables
//   3. multiplies by the two prepared key polynomials of row h (its block of the spectrum), keeps the product for
//      component h and hands the other one to its sibling wave through LDS; sums and reduces
//   4. inverse wave transform of its block, last inverse stage across the two blocks (exchange through LDS), twist
//   5. exchanges half of the residues with the wave of the other prime, CRT-lifts its 1024 coefficients and adds them to
//      its accumulator words.
#include "slz_internal.h"
#include "slz_modarith.h"
#include "slz_fused_common.h"
#include <vector>

#include "slz_wave_ntt.h"

#define HN 4096u
#define HLOGN 12u
#define H_THREADS 512
#define H_STAGE_OFF 1088u      // second half of a wave buffer: staging of 1024 accumulator words

struct fused4096_args : slz_fused_io {
    const double *rowA[2];    // [2 blocks][64]      block twiddles of the stages with 1..32 sub-blocks
    const double *rowB[2];    // [2 blocks][31][64]  block twiddles of the last five forward stages, entry (k, lane)
    double tw_fwd[2][2][32];  // [prime][block]: rowA entries below 32 (lane-uniform, read with scalar loads)
    double tw_inv[2][32];     // inv[t + j], t + j < 32
    double w_first[2];        // fwd[1]: the twiddle of the stage across the two blocks
};

template <int BETA>
__global__ void __launch_bounds__(H_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2)))
k_fused_blind_rotate_n4096(fused4096_args A) {
    const uint32_t beta = BETA > 0 ? (uint32_t)BETA : A.beta;
    extern __shared__ double lds[];
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t b = w >> 2, q = (w >> 1) & 1u, h = w & 1u;
    double *T = lds + w * TBUF;                      // this wave's buffer
    const double *Tsib = lds + (w ^ 1u) * TBUF;      // same block and prime, other row
    const double *Toth = lds + (w ^ 2u) * TBUF;      // same block and row, other prime
    const double *Tblk = lds + (w ^ 4u) * TBUF;      // same prime and row, other block
    uint64_t *Smine = reinterpret_cast<uint64_t *>(T + H_STAGE_OFF);
    const slz_mod m = A.mod[q];
    const double *fwd6 = A.rowA[q] + b * 64u + 32u, *fwdB = A.rowB[q] + (size_t)b * 31u * 64u;
    const double *invt = A.inv[q], *post = A.post[q];
    const double *twA = A.tw_fwd[q][b], *twS = A.tw_inv[q];
    const double w1 = A.w_first[q];
    const uint32_t hh = lane >> 5;

    for (uint32_t c = blockIdx.x; c < A.batch; c += gridDim.x) {
        const uint64_t *lwe = A.lwe_in + (size_t)c * (A.n + 1);
        const uint32_t own0 = 2048u * b + 1024u * q;            // first coefficient of my accumulator words
        uint64_t acc[16];
        if (h == 1) {
            const uint32_t bt = slz_modswitch(lwe[A.n], HLOGN + 1);
            const uint32_t r = (2 * HN - bt) & (2 * HN - 1);
            const uint64_t *lut = A.luts + (size_t)(A.lut_idx ? A.lut_idx[c] : 0) * HN;
#pragma unroll
            for (int e = 0; e < 16; e++)
                acc[e] = slz_rot_coeff([&](uint32_t j) { return lut[j]; }, own0 + 64u * e + lane, r, HN);
        } else {
#pragma unroll
            for (int e = 0; e < 16; e++) acc[e] = 0;
        }

        for (uint32_t step = 0; step < A.n_steps; step++) {
            // an opaque zero added to every table index keeps the per-lane table loads inside the step loop
            int z;
            asm volatile("s_mov_b32 %0, 0" : "=s"(z));
            const uint32_t at = slz_modswitch(lwe[step], HLOGN + 1);
            const double *krow = A.bskp + ((size_t)step * 4 + q * 2 + h) * 2 * HN + 64u * b + z;   // [n][prime][row][comp][N]
            const double *kown = krow + (size_t)h * HN, *ksib = krow + (size_t)(1u - h) * HN;
            // 1. stage my words; word j of component h then sits in the buffer of wave (j >> 11, (j >> 10) & 1, h)
#pragma unroll
            for (int e = 0; e < 16; e++) Smine[64 * e + lane] = acc[e];
            __syncthreads();
            {
                uint32_t r = at, neg0 = 0;
                if (r >= HN) { r -= HN; neg0 = 1; }
                int32_t *pd = reinterpret_cast<int32_t *>(T);
#pragma unroll
                for (int e = 0; e < 16; e++) {
                    const uint32_t idx = own0 + 64u * e + lane;
                    const uint32_t j = (idx - r) & (HN - 1);
                    const uint32_t neg = neg0 ^ (idx < r ? 1u : 0u);
                    const uint32_t wj = ((j >> 11) << 2) | (((j >> 10) & 1u) << 1) | h;
                    const uint64_t a = reinterpret_cast<const uint64_t *>(lds + wj * TBUF + H_STAGE_OFF)[j & 1023u];
                    const uint64_t lam = (neg ? (uint64_t)0 - a : a) - acc[e];
                    uint64_t v = slz_round_top_bits(lam, beta);
                    pd[64 * e + lane] = slz_next_digit(v, beta);
                }
            }
            __syncthreads();                          // staged words are read, digits are in place
            // 2. digits of row h: coefficient 64 e + lane (block 0 half) and 2048 + 64 e + lane; first stage across the blocks
            double x[32];
#pragma unroll
            for (int g = 0; g < 8; g++) {
                double lo[4], hi[4], v4[4];
#pragma unroll
                for (int u = 0; u < 4; u++) {
                    const int e = 4 * g + u;
                    const uint32_t wp = (uint32_t)(e >> 4) << 1 | h;                     // producer (0, e >> 4, h)
                    const int32_t *p0 = reinterpret_cast<const int32_t *>(lds + wp * TBUF);
                    const int32_t *p1 = reinterpret_cast<const int32_t *>(lds + (wp | 4u) * TBUF);
                    lo[u] = (double)p0[64 * (e & 15) + lane];
                    hi[u] = (double)p1[64 * (e & 15) + lane];
                }
                const double w4[4] = {w1, w1, w1, w1};
                mulmod_k<4>(v4, hi, w4, m);
#pragma unroll
                for (int u = 0; u < 4; u++) x[4 * g + u] = b ? lo[u] - v4[u] : lo[u] + v4[u];
            }
            __syncthreads();                          // every wave has its digits: the buffers may be reused
            double tw6[16];
#pragma unroll
            for (int mm = 0; mm < 16; mm++) tw6[mm] = ldl(fwd6 + 2 * mm + z, hh * 8u);
            SCHED_FENCE();
            fused_fwd(x, T, tw6, twA, fwdB, m, lane, z);
            // 3. row h of the GGSW times the digits (spectrum index 2048 b + 32 lane + i sits at i N/32 + 64 b + lane):
            //    component h stays, component 1-h goes to the sibling.  Key words are fetched eight positions ahead.
            {
                double ks[2][8], ko[2][8];
#pragma unroll
                for (int i = 0; i < 8; i++) { ks[0][i] = ldl(ksib + 128 * i, lane * 8u); ko[0][i] = ldl(kown + 128 * i, lane * 8u); }
                wave_sync();
#pragma unroll
                for (int ch = 0; ch < 4; ch++) {
                    SCHED_FENCE();
                    if (ch < 3) {
#pragma unroll
                        for (int i = 0; i < 8; i++) {
                            ks[(ch + 1) & 1][i] = ldl(ksib + 128 * (8 * (ch + 1) + i), lane * 8u);
                            ko[(ch + 1) & 1][i] = ldl(kown + 128 * (8 * (ch + 1) + i), lane * 8u);
                        }
                    }
                    SCHED_FENCE();
#pragma unroll
                    for (int i = 0; i < 8; i += 2) {
                        double r4[4];
                        const double x4[4] = {x[8 * ch + i], x[8 * ch + i], x[8 * ch + i + 1], x[8 * ch + i + 1]};
                        const double w4[4] = {ks[ch & 1][i], ko[ch & 1][i], ks[ch & 1][i + 1], ko[ch & 1][i + 1]};
                        mulmod_k<4>(r4, x4, w4, m);
                        T[64 * (8 * ch + i) + lane] = r4[0];
                        x[8 * ch + i] = r4[1];
                        T[64 * (8 * ch + i + 1) + lane] = r4[2];
                        x[8 * ch + i + 1] = r4[3];
                    }
                }
            }
            __syncthreads();
#pragma unroll
            for (int g = 0; g < 4; g++) {
                double r8[8], x8[8];
#pragma unroll
                for (int u = 0; u < 8; u++) x8[u] = x[8 * g + u] + Tsib[64 * (8 * g + u) + lane];
                reduce_k<8>(r8, x8, m);
#pragma unroll
                for (int u = 0; u < 8; u++) x[8 * g + u] = r8[u];
            }
            __syncthreads();                          // sibling has read my buffer before I reuse it
            // 4. inverse transform inside the block, then the stage across the two blocks and the twist
            fused_inv<false>(x, T, twS, invt, post, m, lane, z);
            // twiddles of the stage across the blocks (inv[2048 + c]) and the twist (post[2048 b + c]), c = 64 e + lane: requested
            // one group of four coefficients ahead of their use, the first group before the exchange
            double wv[2][4], pw[2][4];
#pragma unroll
            for (int u = 0; u < 4; u++) {
                wv[0][u] = ldl(invt + 2048 + 64 * u + z, lane * 8u);
                pw[0][u] = ldl(post + 2048 * b + 64 * u + z, lane * 8u);
            }
            SCHED_FENCE();
            wave_sync();
#pragma unroll
            for (int g = 0; g < 4; g++) {
                double r8[8], x8[8];
#pragma unroll
                for (int u = 0; u < 8; u++) x8[u] = x[8 * g + u];
                reduce_k<8>(r8, x8, m);
#pragma unroll
                for (int u = 0; u < 8; u++) { x[8 * g + u] = r8[u]; T[64 * (8 * g + u) + lane] = r8[u]; }
            }
            __syncthreads();
#pragma unroll
            for (int g = 0; g < 8; g++) {
                SCHED_FENCE();
                if (g < 7) {
#pragma unroll
                    for (int u = 0; u < 4; u++) {
                        wv[(g + 1) & 1][u] = ldl(invt + 2048 + 64 * (4 * (g + 1) + u) + z, lane * 8u);
                        pw[(g + 1) & 1][u] = ldl(post + 2048 * b + 64 * (4 * (g + 1) + u) + z, lane * 8u);
                    }
                }
                SCHED_FENCE();
                double y1[4], v4[4], r4[4], s4[4];
#pragma unroll
                for (int u = 0; u < 4; u++) {
                    const double other = Tblk[64 * (4 * g + u) + lane];
                    y1[u] = b ? x[4 * g + u] : other;                                    // the value of block 1
                    if (b) x[4 * g + u] = other;                                         // x now holds the value of block 0
                }
                const double wg[4] = {wv[g & 1][0], wv[g & 1][1], wv[g & 1][2], wv[g & 1][3]};
                const double pg[4] = {pw[g & 1][0], pw[g & 1][1], pw[g & 1][2], pw[g & 1][3]};
                mulmod_k<4>(v4, y1, wg, m);
#pragma unroll
                for (int u = 0; u < 4; u++) s4[u] = b ? x[4 * g + u] - v4[u] : x[4 * g + u] + v4[u];
                mulmod_k<4>(r4, s4, pg, m);
#pragma unroll
                for (int u = 0; u < 4; u++) x[4 * g + u] = r4[u];
            }
            __syncthreads();                          // the other block's wave has read my buffer
            // 5. exchange the half I do not lift with the other prime's wave, CRT, accumulate
            if (q == 0) {
#pragma unroll
                for (int e = 0; e < 16; e++) T[64 * e + lane] = x[16 + e];
            } else {
#pragma unroll
                for (int e = 0; e < 16; e++) T[64 * e + lane] = x[e];
            }
            __syncthreads();
            if (q == 0) {
#pragma unroll
                for (int e = 0; e < 16; e++) acc[e] += slz_crt64(x[e], Toth[64 * e + lane], A.mod[1], A.p1inv_mod_p2);
            } else {
#pragma unroll
                for (int e = 0; e < 16; e++) acc[e] += slz_crt64(Toth[64 * e + lane], x[16 + e], A.mod[1], A.p1inv_mod_p2);
            }
        }

        // ---- output: accumulator, or the extracted LWE ciphertext ----
        if (A.acc_out) {
            uint64_t *dst = A.acc_out + ((size_t)c * 2 + h) * HN;
#pragma unroll
            for (int e = 0; e < 16; e++) dst[own0 + 64u * e + lane] = acc[e];
        }
        if (A.lwe_out) {
            uint64_t *dst = A.lwe_out + (size_t)c * (HN + 1);
            if (h == 0) {
#pragma unroll
                for (int e = 0; e < 16; e++) {
                    const uint32_t idx = own0 + 64u * e + lane;
                    if (idx == 0) dst[0] = acc[e];
                    else dst[HN - idx] = (uint64_t)0 - acc[e];
                }
            } else if (b == 0 && q == 0 && lane == 0) {
                dst[HN] = acc[0];
            }
        }
        __syncthreads();                              // the next ciphertext reuses the LDS buffers
    }
}

// ---- host side -----------------------------------------------------------------------------------

int slz_fused4096_supported(const slz_params *p) {
    return p->N == HN && p->k == 1 && p->pbs_level == 1 && p->pbs_base_log <= 30;
}

int slz_fused4096_init(slz_ctx *ctx) {
    // the stage across the blocks and six more on the digits, reduction, five more; two products summed; inverse 2 + 3
    // stages, reduction, six stages, reduction, the stage across the blocks, twist
    if (!slz_fused_schedule_ok(1, 6, 5, 2, 3, 6, true, 2)) return SLZ_E_UNSUPPORTED;
    int rc = slz_build_block_tables(ctx, 2048, &ctx->fused4096_rowA, &ctx->fused4096_rowB);
    if (rc != SLZ_OK) return rc;
    for (int q = 0; q < 2; q++) {
        SLZ_HIP(hipMemcpy(ctx->fused4096_scalars[q], ctx->fused4096_rowA + (size_t)q * 2 * 64, 2 * 64 * sizeof(double), hipMemcpyDeviceToHost));
        SLZ_HIP(hipMemcpy(ctx->fused_scalars[q][1], ctx->tab[q].inv, 32 * sizeof(double), hipMemcpyDeviceToHost));
        SLZ_HIP(hipMemcpy(&ctx->fused4096_w1[q], ctx->tab[q].fwd + 1, sizeof(double), hipMemcpyDeviceToHost));
    }
    SLZ_HIP(hipFuncSetAttribute((const void *)k_fused_blind_rotate_n4096<22>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                8 * TBUF * sizeof(double)));
    SLZ_HIP(hipFuncSetAttribute((const void *)k_fused_blind_rotate_n4096<0>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                8 * TBUF * sizeof(double)));
    return SLZ_OK;
}

void slz_fused4096_destroy(slz_ctx *ctx) {
    if (ctx->fused4096_rowA) (void)hipFree(ctx->fused4096_rowA);
    if (ctx->fused4096_rowB) (void)hipFree(ctx->fused4096_rowB);
    ctx->fused4096_rowA = ctx->fused4096_rowB = nullptr;
}

int slz_fused4096_blind_rotate(slz_ctx *ctx, const uint64_t *lwe_in, const uint64_t *luts, const uint32_t *lut_idx,
                               const double *bskp, uint32_t n_steps, uint64_t *acc_out, uint64_t *lwe_out, uint32_t batch,
                               hipStream_t s) {
    fused4096_args A;
    slz_fused_fill_io(A, ctx, lwe_in, luts, lut_idx, bskp, n_steps, acc_out, lwe_out, batch);
    for (int q = 0; q < 2; q++) {
        A.rowA[q] = ctx->fused4096_rowA + (size_t)q * 2 * 64;
        A.rowB[q] = ctx->fused4096_rowB + (size_t)q * 2 * 31 * 64;
        for (int blk = 0; blk < 2; blk++)
            for (int x = 0; x < 32; x++) A.tw_fwd[q][blk][x] = ctx->fused4096_scalars[q][blk * 64 + x];
        for (int x = 0; x < 32; x++) A.tw_inv[q][x] = ctx->fused_scalars[q][1][x];
        A.w_first[q] = ctx->fused4096_w1[q];
    }
    const uint32_t grid = slz_fused_grid(batch, 1);    // one workgroup (136 KiB of LDS, eight waves) per compute unit
    if (A.beta == 22)
        hipLaunchKernelGGL(k_fused_blind_rotate_n4096<22>, dim3(grid), dim3(H_THREADS), 8 * TBUF * sizeof(double), s, A);
    else
        hipLaunchKernelGGL(k_fused_blind_rotate_n4096<0>, dim3(grid), dim3(H_THREADS), 8 * TBUF * sizeof(double), s, A);
    SLZ_HIP(hipGetLastError());
    return SLZ_OK;
}
