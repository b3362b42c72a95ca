// Fused blind rotation for N = 2048, k = 1, l = 1 (the 128-bit-shaped low-precision parameter sets).
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
#include <vector>
#include <cstdio>

#define FN 2048u
#define FLOGN 11u
#define TBUF 2176u            // doubles per wave buffer: 2048 + 2 pad doubles per 32 (bank-conflict-free transposition)
#define STAGE_OFF 1088u       // second half of a wave buffer: staging of 1024 accumulator words
#define FUSED_THREADS 256

struct fused_args {
    const uint64_t *lwe_in;
    const uint64_t *luts;
    const uint32_t *lut_idx;
    const double *bskp;
    uint64_t *acc_out;
    uint64_t *lwe_out;
    uint32_t n, n_steps, batch;
    // per-lane twiddle tables in HBM/L2, one per prime
    const double *fwd6[2];    // [32]      fwd[32 + x]: stage with stride 32 (one value per half-wave and register pair)
    const double *fwdB[2];    // [31][64]  last five forward stages, entry (k, lane)
    const double *inv[2];     // [N]       inv[t + j]: cyclic inverse twiddles (t >= 32 are per lane)
    const double *post[2];    // [N]       psi^-j / N
    // lane-uniform twiddles travel in the kernel argument segment and are read with scalar loads
    double tw_fwd[2][32];     // fwd[m + blk], m + blk < 32: first five forward stages
    double tw_inv[2][32];     // inv[t + j], t + j < 32: first five inverse stages
    slz_mod mod[2];
    double p1inv_mod_p2;
#ifdef SLZ_PHASE_TIMING
    unsigned long long *dbg;  // [4 waves][16 marks]: cycles spent before each mark, summed over the steps of block 0
#endif
};

#ifdef SLZ_PHASE_TIMING
#define MARK(k) do { if (blockIdx.x == 0) { unsigned long long t_ = __builtin_amdgcn_s_memtime(); \
                     if (lane == 0) A.dbg[w * 16 + (k)] += t_ - tprev; tprev = t_; } } while (0)
#else
#define MARK(k) do { } while (0)
#endif

// keeps the instruction scheduler from moving anything across this point: table and key loads are issued by hand
// one phase ahead of their use (software prefetch); letting the scheduler hoist them all spills, letting it sink
// them to their first use exposes the full L2 latency at two waves per SIMD
#define SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

// Per-lane table load as "uniform base (SGPR pair) + 32-bit lane offset": keeps one address register for all
// tables instead of a 64-bit address pair per load group (those pairs spill, and a spill reload drains the
// whole queue of prefetches in flight).
__device__ __forceinline__ double ldl(const double *uniform_base, uint32_t lane_byte_off) {
    return *reinterpret_cast<const double *>(reinterpret_cast<const char *>(uniform_base) + lane_byte_off);
}

__device__ __forceinline__ void wave_sync() {
    // orders this wave's LDS writes before its later LDS reads of other lanes' data
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// a <- (a.low half-wave, b.low half-wave), b <- (a.high half-wave, b.high half-wave)
__device__ __forceinline__ void swap32(double &a, double &b) {
    uint32_t alo = (uint32_t)__double2loint(a), ahi = (uint32_t)__double2hiint(a);
    uint32_t blo = (uint32_t)__double2loint(b), bhi = (uint32_t)__double2hiint(b);
    auto lo = __builtin_amdgcn_permlane32_swap(alo, blo, false, false);
    auto hi = __builtin_amdgcn_permlane32_swap(ahi, bhi, false, false);
    a = __hiloint2double((int)hi[0], (int)lo[0]);
    b = __hiloint2double((int)hi[1], (int)lo[1]);
}

__device__ __forceinline__ void bfly(double &a, double &b, double w, slz_mod m) {
    double v = slz_mulmod(b, w, m);
    b = a - v;
    a = a + v;
}
// K independent butterflies with their instructions interleaved step by step.  A dependent FP64 instruction can
// issue only every other slot (measured: 9 cycles per instruction in a dependent chain against 4.8 with four
// independent chains), so a wave that runs its butterflies one after the other uses half of its SIMD.
template <int K>
__device__ __forceinline__ void bfly_k(double *(&a)[K], double *(&b)[K], const double (&w)[K], slz_mod m) {
    double h[K], l[K], q[K];
#pragma unroll
    for (int i = 0; i < K; i++) h[i] = *b[i] * w[i];
#pragma unroll
    for (int i = 0; i < K; i++) q[i] = h[i] * m.pinv;
#pragma unroll
    for (int i = 0; i < K; i++) l[i] = __builtin_fma(*b[i], w[i], -h[i]);
#pragma unroll
    for (int i = 0; i < K; i++) q[i] = __builtin_rint(q[i]);
#pragma unroll
    for (int i = 0; i < K; i++) h[i] = __builtin_fma(-q[i], m.p, h[i]);
#pragma unroll
    for (int i = 0; i < K; i++) h[i] = h[i] + l[i];
#pragma unroll
    for (int i = 0; i < K; i++) *b[i] = *a[i] - h[i];
#pragma unroll
    for (int i = 0; i < K; i++) *a[i] = *a[i] + h[i];
}

// K independent modular multiplications / reductions, interleaved the same way
template <int K>
__device__ __forceinline__ void mulmod_k(double (&r)[K], const double (&xv)[K], const double (&w)[K], slz_mod m) {
    double h[K], l[K], q[K];
#pragma unroll
    for (int i = 0; i < K; i++) h[i] = xv[i] * w[i];
#pragma unroll
    for (int i = 0; i < K; i++) q[i] = h[i] * m.pinv;
#pragma unroll
    for (int i = 0; i < K; i++) l[i] = __builtin_fma(xv[i], w[i], -h[i]);
#pragma unroll
    for (int i = 0; i < K; i++) q[i] = __builtin_rint(q[i]);
#pragma unroll
    for (int i = 0; i < K; i++) h[i] = __builtin_fma(-q[i], m.p, h[i]);
#pragma unroll
    for (int i = 0; i < K; i++) r[i] = h[i] + l[i];
}
template <int K>
__device__ __forceinline__ void reduce_k(double (&r)[K], const double (&xv)[K], slz_mod m) {
    double q[K];
#pragma unroll
    for (int i = 0; i < K; i++) q[i] = xv[i] * m.pinv;
#pragma unroll
    for (int i = 0; i < K; i++) q[i] = __builtin_rint(q[i]);
#pragma unroll
    for (int i = 0; i < K; i++) r[i] = __builtin_fma(-q[i], m.p, xv[i]);
}

// all butterflies (x[ia], x[ib]) of a stage given by index lists, four at a time
#define BF4(i0, j0, w0, i1, j1, w1, i2, j2, w2, i3, j3, w3) do { \
    double *pa_[4] = {&x[i0], &x[i1], &x[i2], &x[i3]}; double *pb_[4] = {&x[j0], &x[j1], &x[j2], &x[j3]}; \
    const double pw_[4] = {w0, w1, w2, w3}; bfly_k<4>(pa_, pb_, pw_, m); } while (0)

__device__ __forceinline__ void bfly_nomul(double &a, double &b) {
    double v = b;
    b = a - v;
    a = a + v;
}

// Forward transform.  In: x[e] = coefficient 64e + lane (|x| tiny).  Out: x[i] = spectrum position 32*lane + i,
// |x| <= 4.9 p.  Worst-case growth per stage: a -> a + 1/2 + 0.1875 a (slz_mulmod_bound); six stages take the
// digits to 4.81 p, one full reduction brings them back to p/2, five more stages end at 4.81 p.
// tw6 (stage with stride 32) is loaded by the caller; twA = lane-uniform twiddles; the per-lane twiddles of the last
// five stages are fetched here before the first stage starts.  z is an opaque zero (see the kernel).
__device__ __forceinline__ void fused_fwd(double (&x)[32], double *T, const double (&tw6)[16], const double *twA,
                                          const double *fwdB, slz_mod m, uint32_t lane, int z) {
    const uint32_t hh = lane >> 5, l5 = lane & 31u;
    double twB[31];
#pragma unroll
    for (int k = 0; k < 15; k++) twB[k] = ldl(fwdB + k * 64 + z, lane * 8u);
    SCHED_FENCE();
#pragma unroll
    for (int s = 0; s < 5; s++) {
        const int half = 16 >> s;
#pragma unroll
        for (int g = 0; g < 4; g++) {                            // 16 butterflies per stage, four at a time
            // butterfly number b in [0,16): block b / half, position b % half; uniform twiddle per block
#define FA_I(b) (((b) / half) * 2 * half + (b) % half)
#define FA_W(b) twA[(1 << s) + (b) / half + z]
            BF4(FA_I(4 * g), FA_I(4 * g) + half, FA_W(4 * g), FA_I(4 * g + 1), FA_I(4 * g + 1) + half, FA_W(4 * g + 1),
                FA_I(4 * g + 2), FA_I(4 * g + 2) + half, FA_W(4 * g + 2), FA_I(4 * g + 3), FA_I(4 * g + 3) + half, FA_W(4 * g + 3));
        }
    }
    double *wb = T + 68u * hh + l5;
#pragma unroll
    for (int g = 0; g < 4; g++) {
#pragma unroll
        for (int mm = 4 * g; mm < 4 * g + 4; mm++) swap32(x[2 * mm], x[2 * mm + 1]);   // stride 32: partner sits 32 lanes away
        BF4(8 * g, 8 * g + 1, tw6[4 * g], 8 * g + 2, 8 * g + 3, tw6[4 * g + 1], 8 * g + 4, 8 * g + 5, tw6[4 * g + 2],
            8 * g + 6, 8 * g + 7, tw6[4 * g + 3]);
        {
            double r8[8];
            const double x8[8] = {x[8 * g], x[8 * g + 1], x[8 * g + 2], x[8 * g + 3], x[8 * g + 4], x[8 * g + 5], x[8 * g + 6], x[8 * g + 7]};
            reduce_k<8>(r8, x8, m);
#pragma unroll
            for (int u = 0; u < 4; u++) {
                wb[136 * (4 * g + u)] = r8[2 * u];
                wb[136 * (4 * g + u) + 34] = r8[2 * u + 1];
            }
        }
    }
    SCHED_FENCE();
#pragma unroll
    for (int k = 15; k < 31; k++) twB[k] = ldl(fwdB + k * 64 + z, lane * 8u);
    SCHED_FENCE();
    wave_sync();
    const double *rb = T + 34u * lane;
#pragma unroll
    for (int i = 0; i < 32; i += 2) {
        const double2 v = *reinterpret_cast<const double2 *>(rb + i);
        x[i] = v.x;
        x[i + 1] = v.y;
    }
#pragma unroll
    for (int s = 0; s < 5; s++) {
        const int t = 16 >> s;
#pragma unroll
        for (int g = 0; g < 4; g++) {
#define FB_I(b) (((b) / t) * 2 * t + (b) % t)
#define FB_W(b) twB[(1 << s) - 1 + (b) / t]
            BF4(FB_I(4 * g), FB_I(4 * g) + t, FB_W(4 * g), FB_I(4 * g + 1), FB_I(4 * g + 1) + t, FB_W(4 * g + 1),
                FB_I(4 * g + 2), FB_I(4 * g + 2) + t, FB_W(4 * g + 2), FB_I(4 * g + 3), FB_I(4 * g + 3) + t, FB_W(4 * g + 3));
        }
    }
}

// Inverse transform.  In: x[i] = spectrum position 32*lane + i, |x| <= 0.51 p.  Out: x[e] = coefficient 64e + lane
// of the product polynomial mod p, |x| <= 1.7 p.  Bounds: stages 1,2 have unit twiddles (no multiply): 0.5 -> 1 -> 2;
// stages 3..5 -> 2.88, 3.91, 5.15; reduce to 0.5; stages 6..11 -> 6.2; the final twist multiply gives 0.5 + 0.1875*6.2.
__device__ __forceinline__ void fused_inv(double (&x)[32], double *T, const double *twS, const double *inv,
                                          const double *post, slz_mod m, uint32_t lane, int z) {
    const uint32_t hh = lane >> 5, l5 = lane & 31u;
    // per-lane twiddles of the stages with half-size 32 .. 1024, fetched before the first stage
    double twL[31];
    const double w32 = ldl(inv + 32 + z, l5 * 8u);
    {
        int kk = 0;
#pragma unroll
        for (int s = 0; s < 4; s++)
#pragma unroll
            for (int j = 0; j < (1 << s); j++) twL[kk++] = ldl(inv + 64 * (1 << s) + 64 * j + z, lane * 8u);
    }
    SCHED_FENCE();
#pragma unroll
    for (int i = 0; i < 32; i += 2) bfly_nomul(x[i], x[i + 1]);                       // t = 1
    {
        const double w = twS[3 + z];
#pragma unroll
        for (int blk = 0; blk < 8; blk++) bfly_nomul(x[4 * blk], x[4 * blk + 2]);      // t = 2, unit twiddle
#pragma unroll
        for (int g = 0; g < 2; g++)                                                     // t = 2, twiddle inv[3]
            BF4(16 * g + 1, 16 * g + 3, w, 16 * g + 5, 16 * g + 7, w, 16 * g + 9, 16 * g + 11, w, 16 * g + 13, 16 * g + 15, w);
    }
#pragma unroll
    for (int s = 2; s < 5; s++) {                                                       // t = 4, 8, 16
        const int t = 1 << s;
#pragma unroll
        for (int g = 0; g < 4; g++) {
            // butterfly b in [0,16): position j = b % t in block b / t; the twiddle depends on j only (uniform)
#define IB_I(b) (((b) / t) * 2 * t + (b) % t)
#define IB_W(b) twS[t + (b) % t + z]
            BF4(IB_I(4 * g), IB_I(4 * g) + t, IB_W(4 * g), IB_I(4 * g + 1), IB_I(4 * g + 1) + t, IB_W(4 * g + 1),
                IB_I(4 * g + 2), IB_I(4 * g + 2) + t, IB_W(4 * g + 2), IB_I(4 * g + 3), IB_I(4 * g + 3) + t, IB_W(4 * g + 3));
        }
    }
    wave_sync();                                                                        // earlier reads of T are done
    double *wb = T + 34u * lane;
#pragma unroll
    for (int g = 0; g < 4; g++) {
        double r8[8];
        const double x8[8] = {x[8 * g], x[8 * g + 1], x[8 * g + 2], x[8 * g + 3], x[8 * g + 4], x[8 * g + 5], x[8 * g + 6], x[8 * g + 7]};
        reduce_k<8>(r8, x8, m);
#pragma unroll
        for (int u = 0; u < 4; u++) {
            double2 v;
            v.x = r8[2 * u];
            v.y = r8[2 * u + 1];
            *reinterpret_cast<double2 *>(wb + 8 * g + 2 * u) = v;
        }
    }
    wave_sync();
    const double *rb = T + 68u * hh + l5;
#pragma unroll
    for (int mm = 0; mm < 16; mm++) {
        x[2 * mm] = rb[136 * mm];
        x[2 * mm + 1] = rb[136 * mm + 34];
    }
#pragma unroll
    for (int g = 0; g < 4; g++) {                                                       // t = 32
        BF4(8 * g, 8 * g + 1, w32, 8 * g + 2, 8 * g + 3, w32, 8 * g + 4, 8 * g + 5, w32, 8 * g + 6, 8 * g + 7, w32);
#pragma unroll
        for (int mm = 4 * g; mm < 4 * g + 4; mm++) swap32(x[2 * mm], x[2 * mm + 1]);
    }
    SCHED_FENCE();
#pragma unroll
    for (int j = 0; j < 16; j++) twL[15 + j] = ldl(inv + 64 * 16 + 64 * j + z, lane * 8u);
    SCHED_FENCE();
    double pw[32];
#pragma unroll
    for (int s = 0; s < 5; s++) {                                                       // t = 64 .. 1024
        const int half = 1 << s;
        if (s == 3) {
            SCHED_FENCE();
#pragma unroll
            for (int e = 0; e < 16; e++) pw[e] = ldl(post + 64 * e + z, lane * 8u);
            SCHED_FENCE();
        }
        if (s == 4) {
            SCHED_FENCE();
#pragma unroll
            for (int e = 16; e < 32; e++) pw[e] = ldl(post + 64 * e + z, lane * 8u);
            SCHED_FENCE();
        }
#pragma unroll
        for (int g = 0; g < 4; g++) {
            // butterfly b in [0,16): position j = b % half in block b / half; per-lane twiddle twL[half - 1 + j]
#define IA_I(b) (((b) / half) * 2 * half + (b) % half)
#define IA_W(b) twL[half - 1 + (b) % half]
            BF4(IA_I(4 * g), IA_I(4 * g) + half, IA_W(4 * g), IA_I(4 * g + 1), IA_I(4 * g + 1) + half, IA_W(4 * g + 1),
                IA_I(4 * g + 2), IA_I(4 * g + 2) + half, IA_W(4 * g + 2), IA_I(4 * g + 3), IA_I(4 * g + 3) + half, IA_W(4 * g + 3));
        }
    }
#pragma unroll
    for (int g = 0; g < 8; g++) {
        double r4[4];
        const double x4[4] = {x[4 * g], x[4 * g + 1], x[4 * g + 2], x[4 * g + 3]};
        const double w4[4] = {pw[4 * g], pw[4 * g + 1], pw[4 * g + 2], pw[4 * g + 3]};
        mulmod_k<4>(r4, x4, w4, m);
#pragma unroll
        for (int u = 0; u < 4; u++) x[4 * g + u] = r4[u];
    }
}

__global__ void __launch_bounds__(FUSED_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2)))
k_fused_blind_rotate_n2048(fused_args A) {
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
#ifdef SLZ_PHASE_TIMING
            unsigned long long tprev = __builtin_amdgcn_s_memtime();
#endif
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
            MARK(0);
            __syncthreads();
            MARK(1);
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
                    uint64_t v = slz_round_top_bits(lam, 23);
                    dg[e] = slz_next_digit(v, 23);
                    pd[64 * e + lane] = dg[e];
                }
            }
            MARK(2);
            __syncthreads();                          // every wave has read the staged accumulator and sent its digits
            MARK(3);
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
            fused_fwd(x, T, tw6, twA, fwdB, m, lane, z);
            MARK(4);
            // 3. row h of the GGSW times the digits: component h stays, component 1-h goes to the sibling.
            //    Key words are fetched eight positions (two chunks of 2 x 8 doubles in flight) ahead.
            {
                double ks[2][8], ko[2][8];
#pragma unroll
                for (int i = 0; i < 8; i++) { ks[0][i] = ldl(ksib + 64 * i, lane * 8u); ko[0][i] = ldl(kown + 64 * i, lane * 8u); }
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
            MARK(5);
            __syncthreads();
            MARK(6);
#pragma unroll
            for (int g = 0; g < 4; g++) {
                double r8[8], x8[8];
#pragma unroll
                for (int u = 0; u < 8; u++) x8[u] = x[8 * g + u] + Tsib[64 * (8 * g + u) + lane];
                reduce_k<8>(r8, x8, m);
#pragma unroll
                for (int u = 0; u < 8; u++) x[8 * g + u] = r8[u];
            }
            MARK(7);
            __syncthreads();                          // sibling has read my buffer before I reuse it
            MARK(8);
            // 4. inverse transform
            fused_inv(x, T, twS, invt, post, m, lane, z);
            MARK(9);
            // 5. exchange the half I do not lift with the other prime's wave, CRT, accumulate
            wave_sync();
            if (q == 0) {
#pragma unroll
                for (int e = 0; e < 16; e++) T[64 * e + lane] = x[16 + e];
            } else {
#pragma unroll
                for (int e = 0; e < 16; e++) T[64 * e + lane] = x[e];
            }
            MARK(10);
            __syncthreads();
            MARK(11);
            if (q == 0) {
#pragma unroll
                for (int e = 0; e < 16; e++) acc[e] += slz_crt64(x[e], Toth[64 * e + lane], A.mod[1], A.p1inv_mod_p2);
            } else {
#pragma unroll
                for (int e = 0; e < 16; e++) acc[e] += slz_crt64(Toth[64 * e + lane], x[16 + e], A.mod[1], A.p1inv_mod_p2);
            }
            MARK(12);
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
    }
}

// ---- host side -----------------------------------------------------------------------------------

int slz_fused_supported(const slz_params *p) {
    return p->N == FN && p->k == 1 && p->pbs_level == 1 && p->pbs_base_log == 23;
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
    SLZ_HIP(hipMemcpy(ctx->fused_tab, host.data(), host.size() * sizeof(double), hipMemcpyHostToDevice));
    // worst-case bounds of the fixed reduction schedule (units of p); everything must stay below 2^53 = 8 p
    double a = 1e-6;
    for (int s = 0; s < 6; s++) a += slz_mulmod_bound(a);
    if (a > 7.5) return SLZ_E_UNSUPPORTED;
    a = 0.5 + 1e-9;
    for (int s = 0; s < 5; s++) a += slz_mulmod_bound(a);
    const double fwd_out = a;
    if (fwd_out > 7.5 || 2 * slz_mulmod_bound(fwd_out) > 7.5) return SLZ_E_UNSUPPORTED;
    a = 2.0 * (0.5 + 1e-9) * 2.0;                      // two multiply-free stages double the bound
    for (int s = 2; s < 5; s++) a += slz_mulmod_bound(a);
    if (a > 7.5) return SLZ_E_UNSUPPORTED;
    a = 0.5 + 1e-9;
    for (int s = 5; s < 11; s++) a += slz_mulmod_bound(a);
    if (a > 7.5 || slz_mulmod_bound(a) > 1.95) return SLZ_E_UNSUPPORTED;   // slz_d2i needs |r| < 2 p
    SLZ_HIP(hipFuncSetAttribute((const void *)k_fused_blind_rotate_n2048, hipFuncAttributeMaxDynamicSharedMemorySize,
                                4 * TBUF * sizeof(double)));
    return SLZ_OK;
}

void slz_fused_destroy(slz_ctx *ctx) {
    if (ctx->fused_tab) (void)hipFree(ctx->fused_tab);
    ctx->fused_tab = nullptr;
}

int slz_fused_blind_rotate(slz_ctx *ctx, const uint64_t *lwe_in, const uint64_t *luts, const uint32_t *lut_idx,
                           const double *bskp, uint32_t n_steps, uint64_t *acc_out, uint64_t *lwe_out, uint32_t batch,
                           hipStream_t s) {
    fused_args A;
    A.lwe_in = lwe_in; A.luts = luts; A.lut_idx = lut_idx; A.bskp = bskp; A.acc_out = acc_out; A.lwe_out = lwe_out;
    A.n = ctx->prm.n; A.n_steps = n_steps; A.batch = batch;
    for (int q = 0; q < 2; q++) {
        A.fwd6[q] = ctx->tab[q].fwd + 32;
        A.fwdB[q] = ctx->fused_tab + (size_t)q * 31 * 64;
        A.inv[q] = ctx->tab[q].inv;
        A.post[q] = ctx->tab[q].post;
        A.mod[q] = ctx->mod[q];
        for (int x = 0; x < 32; x++) { A.tw_fwd[q][x] = ctx->fused_scalars[q][0][x]; A.tw_inv[q][x] = ctx->fused_scalars[q][1][x]; }
    }
    A.p1inv_mod_p2 = ctx->p1inv_mod_p2;
#ifdef SLZ_PHASE_TIMING
    static unsigned long long *dbg = nullptr;
    if (!dbg) { SLZ_HIP(hipMalloc((void **)&dbg, 64 * 8)); }
    SLZ_HIP(hipMemsetAsync(dbg, 0, 64 * 8, s));
    A.dbg = dbg;
#endif
    const uint32_t resident = 2u * 256u;               // two workgroups (68 KiB of LDS each) per compute unit
    const uint32_t grid = batch < resident ? batch : resident;
    hipLaunchKernelGGL(k_fused_blind_rotate_n2048, dim3(grid), dim3(FUSED_THREADS), 4 * TBUF * sizeof(double), s, A);
    SLZ_HIP(hipGetLastError());
#ifdef SLZ_PHASE_TIMING
    {
        unsigned long long h[64];
        SLZ_HIP(hipMemcpy(h, dbg, sizeof(h), hipMemcpyDeviceToHost));
        static const char *names[13] = {"stage-write", "B1", "decompose", "B2", "fwd", "pointwise", "B3", "sum", "B4", "inverse",
                                        "xchg-write", "B5", "crt"};
        const double steps = (double)n_steps * ((batch + grid - 1) / grid);
        for (int w = 0; w < 4; w++) {
            fprintf(stderr, "wave %d cycles/step:", w);
            for (int k = 0; k < 13; k++) fprintf(stderr, " %s=%.0f", names[k], (double)h[w * 16 + k] / steps);
            fprintf(stderr, "\n");
        }
    }
#endif
    return SLZ_OK;
}
