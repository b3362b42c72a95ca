// Fused blind rotation for N = 2048, k = 1, l = 1, any base (the 128-bit-shaped low-precision parameter sets).
//
// One workgroup of four wavefronts owns one ciphertext for the whole blind rotation; the accumulator
// never leaves the chip.  Wave (q, h): q = transform prime, h = GGSW row = accumulator component.
// Per CMux step every wave
//   1. stages its quarter of the accumulator in LDS, reads component h rotated by a~ and unrotated,
//      subtracts, rounds and extracts the signed digit                      (rows are decomposed once per prime)
//   2. forward negacyclic transform of the digit polynomial mod p_q         (one wave = one polynomial,
//      32 coefficients per lane: 5 radix-2 stages in registers, one stage across the two half-waves with
//      v_permlane32_swap, one LDS transposition, 5 more stages in registers)
//   3. multiplies by the two prepared key polynomials of row h, keeps the product for component h and hands
//      the other one to its sibling wave through LDS; sums and reduces
//   4. inverse transform (cyclic decimation-in-time on the bit-reversed spectrum, then the psi^-j / N twist)
//   5. exchanges half of the residues with the wave of the other prime, CRT-lifts its half of component h
//      to an integer mod 2^64 and adds it to its quarter of the accumulator (kept in registers).
// Key rows are read straight from L2 (every workgroup on the chip reads the same 128 KiB per step).
#include "slz_internal.h"
#include "slz_modarith.h"
#include "slz_fused_common.h"
#include <vector>

#define STAGE_OFF 1088u       // second half of a wave buffer: staging of 1024 accumulator words
#define FUSED_THREADS 256

struct fused_args : slz_fused_io {
    // per-lane twiddle tables in HBM/L2, one per prime
    const double *fwd6[2];    // [32]      fwd[32 + x]: stage with stride 32 (one value per half-wave and register pair)
    const double *fwdB[2];    // [31][64]  last five forward stages, entry (k, lane)
    // lane-uniform twiddles travel in the kernel argument segment and are read with scalar loads
    double tw_fwd[2][32];     // fwd[m + blk], m + blk < 32: first five forward stages
    double tw_inv[2][32];     // inv[t + j], t + j < 32: first five inverse stages
    uint32_t *sync;           // [rounds] arrival counters of the pacing between ciphertexts (zeroed before the launch), or null
    uint32_t patience;        // 0: a pacing wait gives up at once (tests); otherwise it lasts up to the waiter's own round time
};

#define FUSED_SYNC_SLOTS 4096u        // rounds (ciphertexts per workgroup) one launch can pace

// sync[0 .. rounds) arrival counters, sync[FUSED_SYNC_SLOTS] the "a wait has timed out" flag
__global__ void k_fused_zero_sync(uint32_t *sync, uint32_t count) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) sync[i] = 0;
    if (i == 0) sync[FUSED_SYNC_SLOTS] = 0;
}

#include "slz_wave_ntt.h"

// BETA > 0: gadget base 2^BETA fixed at compile time (constant shifts in the decomposition are worth about 1 % of the
// kernel); BETA = 0: base taken from the arguments.
template <int BETA>
__global__ void __launch_bounds__(FUSED_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2)))
k_fused_blind_rotate_n2048(fused_args A) {
    const uint32_t beta = BETA > 0 ? (uint32_t)BETA : A.beta;
    extern __shared__ double lds[];
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t q = w >> 1, h = w & 1u;
    double *T = lds + w * TBUF;                      // this wave's buffer
    double *Tsib = lds + (w ^ 1u) * TBUF;            // same prime, other row
    double *Toth = lds + (w ^ 2u) * TBUF;            // other prime, same row
    // staged ACC_h: words 0..1023 in the buffer of wave (0,h), words 1024..2047 in the buffer of wave (1,h)
    const uint64_t *Sh = reinterpret_cast<const uint64_t *>(lds + h * TBUF + STAGE_OFF);
    uint64_t *Smine = reinterpret_cast<uint64_t *>(T + STAGE_OFF);
    const slz_mod m = A.mod[q];
    const double *fwd6 = A.fwd6[q], *fwdB = A.fwdB[q], *invt = A.inv[q], *post = A.post[q];
    const double *twA = A.tw_fwd[q], *twS = A.tw_inv[q];
    const uint32_t hh = lane >> 5;

    for (uint32_t c = blockIdx.x; c < A.batch; c += gridDim.x) {
        const long long t_round = A.sync ? wall_clock64() : 0;   // for the pacing at the end of the round
        const uint64_t *lwe = A.lwe_in + (size_t)c * (A.n + 1);
        // ---- accumulator quarter: coefficients 64*(16q + e) + lane of component h ----
        uint64_t acc[16];
        if (h == 1) {
            const uint32_t bt = slz_modswitch(lwe[A.n], FLOGN + 1);
            const uint32_t r = (2 * FN - bt) & (2 * FN - 1);
            const uint64_t *lut = A.luts + (size_t)(A.lut_idx ? A.lut_idx[c] : 0) * FN;
#pragma unroll
            for (int e = 0; e < 16; e++)
                acc[e] = slz_rot_coeff([&](uint32_t j) { return lut[j]; }, 64u * (16u * q + e) + lane, r, FN);
        } else {
#pragma unroll
            for (int e = 0; e < 16; e++) acc[e] = 0;
        }

        for (uint32_t step = 0; step < A.n_steps; step++) {
            // The tables do not change between steps, so the compiler would hoist their ~170 per-lane loads out of
            // this loop and spill them.  An opaque zero added to every table index makes each step issue them again.
            int z;
            asm volatile("s_mov_b32 %0, 0" : "=s"(z));
            const uint32_t at = slz_modswitch(lwe[step], FLOGN + 1);
            const double *krow = A.bskp + ((size_t)step * 4 + q * 2 + h) * 2 * FN + z;   // [n][prime][row][comp][N]
            const double *kown = krow + (size_t)h * FN, *ksib = krow + (size_t)(1u - h) * FN;
            double tw6[16];
#pragma unroll
            for (int mm = 0; mm < 16; mm++) tw6[mm] = ldl(fwd6 + 2 * mm + z, hh * 8u);
            SCHED_FENCE();
            // 1. stage my quarter, then read component h rotated and unrotated
#pragma unroll
            for (int e = 0; e < 16; e++) Smine[64 * e + lane] = acc[e];
            __syncthreads();
            // Each row is needed by both primes' waves: wave (q,h) decomposes the half of component h whose
            // unrotated words are its own accumulator quarter (registers) and passes the digits to wave (1-q,h)
            // through that wave's buffer, which nobody else touches between the two barriers.
            int32_t dg[16];
            {
                uint32_t r = at, neg0 = 0;
                if (r >= FN) { r -= FN; neg0 = 1; }
                int32_t *pd = reinterpret_cast<int32_t *>(Toth);
#pragma unroll
                for (int e = 0; e < 16; e++) {
                    const uint32_t idx = 1024u * q + 64u * e + lane;
                    const uint32_t j = (idx - r) & (FN - 1);
                    const uint32_t neg = neg0 ^ (idx < r ? 1u : 0u);
                    const uint64_t a = Sh[(j >> 10) * (2u * TBUF) + (j & 1023u)];
                    const uint64_t lam = (neg ? (uint64_t)0 - a : a) - acc[e];
                    uint64_t v = slz_round_top_bits(lam, beta);
                    dg[e] = slz_next_digit(v, beta);
                    pd[64 * e + lane] = dg[e];
                }
            }
            __syncthreads();                          // every wave has read the staged accumulator and sent its digits
            double x[32];
            {
                const int32_t *md = reinterpret_cast<const int32_t *>(T);
                if (q == 0) {
#pragma unroll
                    for (int e = 0; e < 16; e++) { x[e] = (double)dg[e]; x[16 + e] = (double)md[64 * e + lane]; }
                } else {
#pragma unroll
                    for (int e = 0; e < 16; e++) { x[16 + e] = (double)dg[e]; x[e] = (double)md[64 * e + lane]; }
                }
            }
            // 2. forward transform
            // 3. row h of the GGSW times the digits: component h stays, component 1-h goes to the sibling.
            //    Key words are fetched eight positions (two chunks of 2 x 8 doubles in flight) ahead, the first chunk from
            //    inside the forward transform (before its last three stages).
            double ks[2][8], ko[2][8];
            fused_fwd(x, T, tw6, twA, fwdB, m, lane, z, [&]() {
#pragma unroll
                for (int i = 0; i < 8; i++) { ks[0][i] = ldl(ksib + 64 * i, lane * 8u); ko[0][i] = ldl(kown + 64 * i, lane * 8u); }
            });
            {
                wave_sync();
#pragma unroll
                for (int ch = 0; ch < 4; ch++) {
                    SCHED_FENCE();
                    if (ch < 3) {
#pragma unroll
                        for (int i = 0; i < 8; i++) {
                            ks[(ch + 1) & 1][i] = ldl(ksib + 64 * (8 * (ch + 1) + i), lane * 8u);
                            ko[(ch + 1) & 1][i] = ldl(kown + 64 * (8 * (ch + 1) + i), lane * 8u);
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
            // 4. inverse transform
            fused_inv<true>(x, T, twS, invt, post, m, lane, z);
            // 5. exchange the half I do not lift with the other prime's wave, CRT, accumulate
            wave_sync();
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
            uint64_t *dst = A.acc_out + ((size_t)c * 2 + h) * FN;
#pragma unroll
            for (int e = 0; e < 16; e++) dst[64u * (16u * q + e) + lane] = acc[e];
        }
        if (A.lwe_out) {
            uint64_t *dst = A.lwe_out + (size_t)c * (FN + 1);
            if (h == 0) {
#pragma unroll
                for (int e = 0; e < 16; e++) {
                    const uint32_t idx = 64u * (16u * q + e) + lane;
                    if (idx == 0) dst[0] = acc[e];
                    else dst[FN - idx] = (uint64_t)0 - acc[e];
                }
            } else if (q == 0 && lane == 0) {
                dst[FN] = acc[0];
            }
        }
        __syncthreads();                              // the next ciphertext reuses the LDS buffers
        // Pacing: the workgroups of a launch read the same key rows, and an L2 (4 MiB per XCD) holds the rows of ten to thirty
        // steps.  Left alone the workgroups drift apart by more than that within a few ciphertexts and most key rows then
        // come from beyond the L2 (measured at 16 384 ciphertexts: 300 times the key's size per launch; paced: 20 times,
        // which is the eight L2s filling once per round, twice over).  So a workgroup that has another ciphertext to do
        // waits here until the others have finished this round as well.  A hint, not a dependency: the first wait that
        // lasts as long as the waiting workgroup's own round did (the two workgroups of a compute unit do not get equal
        // shares of it, so one may finish well before the other; longer than that means a workgroup that is not resident,
        // say beside another kernel) switches the pacing off for the rest of the launch.  Run time is the same either way:
        // beyond the L2 the key sits in the memory-side cache and the loads are issued far enough ahead.
        // A.patience == 0 (tests of the give-up path): the first wait that is not satisfied at once gives up.
        if (A.sync) {
            const bool more = c + gridDim.x < A.batch;
            if (threadIdx.x == 0) {
                const uint32_t round = c / gridDim.x;
                const uint32_t here = min(gridDim.x, A.batch - round * gridDim.x);       // workgroups with a ciphertext in this round
                __hip_atomic_fetch_add(&A.sync[round], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (more && !__hip_atomic_load(&A.sync[FUSED_SYNC_SLOTS], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
                    const long long t0 = wall_clock64(), limit = A.patience ? t0 - t_round : 0;
                    while (__hip_atomic_load(&A.sync[round], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < here) {
                        if (wall_clock64() - t0 >= limit) {
                            __hip_atomic_store(&A.sync[FUSED_SYNC_SLOTS], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            break;
                        }
                        __builtin_amdgcn_s_sleep(32);
                    }
                }
            }
            if (more) __syncthreads();
        }
    }
}

// ---- host side -----------------------------------------------------------------------------------

int slz_fused_supported(const slz_params *p) {
    return p->N == FN && p->k == 1 && p->pbs_level == 1 && p->pbs_base_log <= 30;
}

int slz_fused_init(slz_ctx *ctx) {
    // per-lane twiddles of the last five forward stages: stage with half-size t = 16 >> s, block `blk` of lane l
    // is block (N/(2t) index) (32 l)/(2t) + blk of the whole transform
    std::vector<double> host((size_t)2 * 31 * 64), nat(FN);
    for (int q = 0; q < 2; q++) {
        SLZ_HIP(hipMemcpy(nat.data(), ctx->tab[q].fwd, FN * sizeof(double), hipMemcpyDeviceToHost));
        int kk = 0;
        for (int s = 0; s < 5; s++) {
            const uint32_t t = 16u >> s, mblk = FN / (2 * t);
            for (uint32_t blk = 0; blk < (1u << s); blk++, kk++)
                for (uint32_t l = 0; l < 64; l++) host[((size_t)q * 31 + kk) * 64 + l] = nat[mblk + (32 * l) / (2 * t) + blk];
        }
    }
    for (int q = 0; q < 2; q++) {
        SLZ_HIP(hipMemcpy(ctx->fused_scalars[q][0], ctx->tab[q].fwd, 32 * sizeof(double), hipMemcpyDeviceToHost));
        SLZ_HIP(hipMemcpy(ctx->fused_scalars[q][1], ctx->tab[q].inv, 32 * sizeof(double), hipMemcpyDeviceToHost));
    }
    SLZ_HIP(hipMalloc((void **)&ctx->fused_tab, host.size() * sizeof(double)));
    SLZ_HIP(hipMalloc((void **)&ctx->fused_sync, (FUSED_SYNC_SLOTS + 1) * sizeof(uint32_t)));
    SLZ_HIP(hipMemcpy(ctx->fused_tab, host.data(), host.size() * sizeof(double), hipMemcpyHostToDevice));
    // six forward stages, reduction, five more; two products summed; inverse 2 + 3 stages, reduction, six stages, twist
    if (!slz_fused_schedule_ok(0, 6, 5, 2, 3, 6, false, 1)) return SLZ_E_UNSUPPORTED;
    SLZ_HIP(hipFuncSetAttribute((const void *)k_fused_blind_rotate_n2048<23>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                4 * TBUF * sizeof(double)));
    SLZ_HIP(hipFuncSetAttribute((const void *)k_fused_blind_rotate_n2048<0>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                4 * TBUF * sizeof(double)));
    return SLZ_OK;
}

void slz_fused_destroy(slz_ctx *ctx) {
    if (ctx->fused_tab) (void)hipFree(ctx->fused_tab);
    if (ctx->fused_sync) (void)hipFree(ctx->fused_sync);
    ctx->fused_tab = nullptr;
    ctx->fused_sync = nullptr;
}

int slz_fused_blind_rotate(slz_ctx *ctx, const uint64_t *lwe_in, const uint64_t *luts, const uint32_t *lut_idx,
                           const double *bskp, uint32_t n_steps, uint64_t *acc_out, uint64_t *lwe_out, uint32_t batch,
                           hipStream_t s) {
    fused_args A;
    slz_fused_fill_io(A, ctx, lwe_in, luts, lut_idx, bskp, n_steps, acc_out, lwe_out, batch);
    for (int q = 0; q < 2; q++) {
        A.fwd6[q] = ctx->tab[q].fwd + 32;
        A.fwdB[q] = ctx->fused_tab + (size_t)q * 31 * 64;
        for (int x = 0; x < 32; x++) { A.tw_fwd[q][x] = ctx->fused_scalars[q][0][x]; A.tw_inv[q][x] = ctx->fused_scalars[q][1][x]; }
    }
    const uint32_t grid = slz_fused_grid(batch, 2);    // two workgroups (68 KiB of LDS each) per compute unit
    const uint32_t rounds = (batch + grid - 1) / grid;
    A.sync = nullptr;
    A.patience = ctx->fused_pacing == 2 ? 0u : 1u;
    if (rounds > 2 && rounds <= FUSED_SYNC_SLOTS && ctx->fused_pacing) {   // counters cleared by a kernel (safe under graph capture)
        hipLaunchKernelGGL(k_fused_zero_sync, dim3((rounds + 255) / 256), dim3(256), 0, s, ctx->fused_sync, rounds);
        A.sync = ctx->fused_sync;
    }
    if (A.beta == 23)       // the base of the N = 2048 parameter sets
        hipLaunchKernelGGL(k_fused_blind_rotate_n2048<23>, dim3(grid), dim3(FUSED_THREADS), 4 * TBUF * sizeof(double), s, A);
    else
        hipLaunchKernelGGL(k_fused_blind_rotate_n2048<0>, dim3(grid), dim3(FUSED_THREADS), 4 * TBUF * sizeof(double), s, A);
    SLZ_HIP(hipGetLastError());
    return SLZ_OK;
}
