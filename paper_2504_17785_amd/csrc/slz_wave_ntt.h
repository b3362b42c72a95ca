// Wave-level negacyclic transforms on doubles: 2048 points (one wavefront = one polynomial or one 2048-block of a larger
// one, 32 coefficients per lane), shared by the fused N = 2048 kernel and the large-N path, and 1024 points (16
// coefficients per lane, at the end of the file) for the large-N path.
#pragma once
#include "slz_internal.h"
#include "slz_modarith.h"

#define FN 2048u
#define FLOGN 11u
#define TBUF 2176u            // doubles per wave buffer: 2048 + 2 pad doubles per 32 (bank-conflict-free transposition)

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
struct fwd_no_hook { __device__ __forceinline__ void operator()() const {} };
// `hook` runs after the second of the last five stages: a place for the caller to request what it needs right after the
// transform (three stages of arithmetic then cover the loads' latency).
template <class Hook = fwd_no_hook>
__device__ __forceinline__ void fused_fwd(double (&x)[32], double *T, const double (&tw6)[16], const double *twA,
                                          const double *fwdB, slz_mod m, uint32_t lane, int z, Hook hook = Hook()) {
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
        if (s == 2) { SCHED_FENCE(); hook(); SCHED_FENCE(); }
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
// POST = false stops before the twist (the large-N path continues with stages across 2048-blocks first).
template <bool POST>
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
        if (POST && s == 3) {
            SCHED_FENCE();
#pragma unroll
            for (int e = 0; e < 16; e++) pw[e] = ldl(post + 64 * e + z, lane * 8u);
            SCHED_FENCE();
        }
        if (POST && s == 4) {
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
    if (!POST) return;
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


// ---- 1024-point wave transforms: 16 coefficients per lane ---------------------------------------------------------------
// Half the registers of the 2048-point version, so that a kernel holding accumulators besides the transform fits two
// waves per SIMD.  Ten stages: four over the register index, one across the two half-waves (v_permlane32_swap), one
// across the 16-lane rows (v_permlane16_swap), one LDS transposition, four more over the register index.
//   layout A: x[e] = coefficient 64 e + lane;                          layout B: x[i] = position 16 lane + i.
//   lane = 32 hh + 16 v + j.  After the two swap stages a lane's register 2 mm + u holds 64 (2 mm + hh) + 32 v + 16 u + j.
#define TBUF16 1152u          // doubles per wave buffer: 1024 + 2 pad doubles per 16 (16-byte reads at a 144-byte lane stride)

// a <- rows (a0, b0, a2, b2), b <- rows (a1, b1, a3, b3) of the four 16-lane rows of a and b
__device__ __forceinline__ void swap16(double &a, double &b) {
    uint32_t alo = (uint32_t)__double2loint(a), ahi = (uint32_t)__double2hiint(a);
    uint32_t blo = (uint32_t)__double2loint(b), bhi = (uint32_t)__double2hiint(b);
    auto lo = __builtin_amdgcn_permlane16_swap(alo, blo, false, false);
    auto hi = __builtin_amdgcn_permlane16_swap(ahi, bhi, false, false);
    a = __hiloint2double((int)hi[0], (int)lo[0]);
    b = __hiloint2double((int)hi[1], (int)lo[1]);
}

// Forward.  In: layout A, |x| tiny (digits after the column stages, reduced).  Out: layout B, |x| <= 3.7 p.
// twA: lane-uniform twiddles of this block, entry (sub-blocks m') + blk for m' = 1 .. 32 (64 doubles);
// twB_tab: [15][64] per-lane twiddles of the last four stages.  Bounds: six stages 0.5 -> 4.81 p, reduction, four more -> 3.63 p.
// PAIR: the 16 x 64 values are two independent 512-point polynomials (registers 0..7 and 8..15 on the way in, lanes
// 0..31 and 32..63 on the way out): the stage that would pair them is left out and the tables carry each half's twiddles.
template <bool PAIR = false>
__device__ __forceinline__ void fwd16(double (&x)[16], double *T, const double *twA, const double *twB_tab, slz_mod m, uint32_t lane,
                                      int z) {
    const uint32_t hh = lane >> 5, v = (lane >> 4) & 1u, j = lane & 15u;
    // twA and twB_tab are expected in LDS (the kernel stages its block's tables there once): their reads do not queue
    // behind the kernel's global loads and need no registers until the stage that uses them
#pragma unroll
    for (int s = PAIR ? 1 : 0; s < 4; s++) {
        const int half = 8 >> s;
#pragma unroll
        for (int g = 0; g < 2; g++) {
#define FA16_I(b) (((b) / half) * 2 * half + (b) % half)
#define FA16_W(b) twA[(1 << s) + (b) / half + z]
            BF4(FA16_I(4 * g), FA16_I(4 * g) + half, FA16_W(4 * g), FA16_I(4 * g + 1), FA16_I(4 * g + 1) + half, FA16_W(4 * g + 1),
                FA16_I(4 * g + 2), FA16_I(4 * g + 2) + half, FA16_W(4 * g + 2), FA16_I(4 * g + 3), FA16_I(4 * g + 3) + half, FA16_W(4 * g + 3));
        }
    }
#pragma unroll
    for (int g = 0; g < 2; g++) {                                           // stride 32: partner 32 lanes away
#pragma unroll
        for (int mm = 4 * g; mm < 4 * g + 4; mm++) swap32(x[2 * mm], x[2 * mm + 1]);
#define TW5(mm) ldl(twA + 16 + 2 * (mm) + z, hh * 8u)                       /* stride 32: block 2 mm + hh of 16 */
        BF4(8 * g, 8 * g + 1, TW5(4 * g), 8 * g + 2, 8 * g + 3, TW5(4 * g + 1), 8 * g + 4, 8 * g + 5, TW5(4 * g + 2), 8 * g + 6, 8 * g + 7,
            TW5(4 * g + 3));
    }
    double *wb = T + 72u * hh + 36u * v + j;
#pragma unroll
    for (int g = 0; g < 2; g++) {                                           // stride 16: partner 16 lanes away
#pragma unroll
        for (int mm = 4 * g; mm < 4 * g + 4; mm++) swap16(x[2 * mm], x[2 * mm + 1]);
#define TW6(mm) ldl(twA + 32 + 4 * (mm) + z, (lane >> 4) * 8u)              /* stride 16: block 4 mm + 2 hh + v of 32 */
        BF4(8 * g, 8 * g + 1, TW6(4 * g), 8 * g + 2, 8 * g + 3, TW6(4 * g + 1), 8 * g + 4, 8 * g + 5, TW6(4 * g + 2), 8 * g + 6, 8 * g + 7,
            TW6(4 * g + 3));
        double r8[8];
        const double x8[8] = {x[8 * g], x[8 * g + 1], x[8 * g + 2], x[8 * g + 3], x[8 * g + 4], x[8 * g + 5], x[8 * g + 6], x[8 * g + 7]};
        reduce_k<8>(r8, x8, m);
#pragma unroll
        for (int u = 0; u < 4; u++) {                                       // registers 2 mm, 2 mm + 1 with mm = 4 g + u
            wb[144 * (4 * g + u)] = r8[2 * u];
            wb[144 * (4 * g + u) + 18] = r8[2 * u + 1];
        }
    }
    wave_sync();
    const double *rb = T + 18u * lane;
#pragma unroll
    for (int i = 0; i < 16; i += 2) {
        const double2 t2 = *reinterpret_cast<const double2 *>(rb + i);
        x[i] = t2.x;
        x[i + 1] = t2.y;
    }
#pragma unroll
    for (int s = 0; s < 4; s++) {
        const int t = 8 >> s;
#pragma unroll
        for (int g = 0; g < 2; g++) {
#define FB16_I(b) (((b) / t) * 2 * t + (b) % t)
#define FB16_W(b) ldl(twB_tab + 64 * ((1 << s) - 1 + (b) / t) + z, lane * 8u)
            BF4(FB16_I(4 * g), FB16_I(4 * g) + t, FB16_W(4 * g), FB16_I(4 * g + 1), FB16_I(4 * g + 1) + t, FB16_W(4 * g + 1),
                FB16_I(4 * g + 2), FB16_I(4 * g + 2) + t, FB16_W(4 * g + 2), FB16_I(4 * g + 3), FB16_I(4 * g + 3) + t, FB16_W(4 * g + 3));
        }
    }
}

// Inverse (cyclic decimation-in-time on the bit-reversed spectrum; stops before the stages across 1024-blocks and the
// twist).  In: layout B, |x| <= 0.51 p.  Out: layout A, |x| <= 6.2 p.  twS: lane-uniform entries inv[t + j], t <= 8;
// inv: the same natural inverse table for the per-lane entries.  Bounds: 0.5 -> 1 -> 2 (unit twiddles) -> 2.88 -> 3.91,
// reduction, six more stages -> 6.2.
// PAIR: two independent 512-point polynomials (lanes 0..31 and 32..63 on the way in, registers 0..7 and 8..15 on the way
// out): the last stage, which would pair them, is left out (and its twiddles, which lie past a 512-entry table, are not read).
template <bool PAIR = false>
__device__ __forceinline__ void inv16(double (&x)[16], double *T, const double *twS, const double *inv, slz_mod m, uint32_t lane, int z) {
    const uint32_t hh = lane >> 5, v = (lane >> 4) & 1u, j = lane & 15u, l5 = lane & 31u;
    double twL[15];
    const double w16 = ldl(inv + 16 + z, j * 8u);
    const double w32 = ldl(inv + 32 + z, l5 * 8u);
    {
        int kk = 0;
#pragma unroll
        for (int s = 0; s < (PAIR ? 3 : 4); s++)
#pragma unroll
            for (int jj = 0; jj < (1 << s); jj++) twL[kk++] = ldl(inv + 64 * (1 << s) + 64 * jj + z, lane * 8u);
    }
    SCHED_FENCE();
#pragma unroll
    for (int i = 0; i < 16; i += 2) bfly_nomul(x[i], x[i + 1]);                        // t = 1
    {
        const double w = twS[3 + z];
#pragma unroll
        for (int blk = 0; blk < 4; blk++) bfly_nomul(x[4 * blk], x[4 * blk + 2]);       // t = 2, unit twiddle
        BF4(1, 3, w, 5, 7, w, 9, 11, w, 13, 15, w);                                     // t = 2, twiddle inv[3]
    }
#pragma unroll
    for (int s = 2; s < 4; s++) {                                                       // t = 4, 8
        const int t = 1 << s;
#pragma unroll
        for (int g = 0; g < 2; g++) {
#define IB16_I(b) (((b) / t) * 2 * t + (b) % t)
#define IB16_W(b) twS[t + (b) % t + z]
            BF4(IB16_I(4 * g), IB16_I(4 * g) + t, IB16_W(4 * g), IB16_I(4 * g + 1), IB16_I(4 * g + 1) + t, IB16_W(4 * g + 1),
                IB16_I(4 * g + 2), IB16_I(4 * g + 2) + t, IB16_W(4 * g + 2), IB16_I(4 * g + 3), IB16_I(4 * g + 3) + t, IB16_W(4 * g + 3));
        }
    }
    wave_sync();                                                                        // earlier reads of T are done
    double *wb = T + 18u * lane;
#pragma unroll
    for (int g = 0; g < 2; g++) {
        double r8[8];
        const double x8[8] = {x[8 * g], x[8 * g + 1], x[8 * g + 2], x[8 * g + 3], x[8 * g + 4], x[8 * g + 5], x[8 * g + 6], x[8 * g + 7]};
        reduce_k<8>(r8, x8, m);
#pragma unroll
        for (int u = 0; u < 4; u++) {
            double2 t2;
            t2.x = r8[2 * u];
            t2.y = r8[2 * u + 1];
            *reinterpret_cast<double2 *>(wb + 8 * g + 2 * u) = t2;
        }
    }
    wave_sync();
    const double *rb = T + 72u * hh + 36u * v + j;
#pragma unroll
    for (int mm = 0; mm < 8; mm++) {
        x[2 * mm] = rb[144 * mm];
        x[2 * mm + 1] = rb[144 * mm + 18];
    }
#pragma unroll
    for (int g = 0; g < 2; g++) {                                                       // t = 16
        BF4(8 * g, 8 * g + 1, w16, 8 * g + 2, 8 * g + 3, w16, 8 * g + 4, 8 * g + 5, w16, 8 * g + 6, 8 * g + 7, w16);
#pragma unroll
        for (int mm = 4 * g; mm < 4 * g + 4; mm++) swap16(x[2 * mm], x[2 * mm + 1]);
    }
#pragma unroll
    for (int g = 0; g < 2; g++) {                                                       // t = 32
        BF4(8 * g, 8 * g + 1, w32, 8 * g + 2, 8 * g + 3, w32, 8 * g + 4, 8 * g + 5, w32, 8 * g + 6, 8 * g + 7, w32);
#pragma unroll
        for (int mm = 4 * g; mm < 4 * g + 4; mm++) swap32(x[2 * mm], x[2 * mm + 1]);
    }
#pragma unroll
    for (int s = 0; s < (PAIR ? 3 : 4); s++) {                                          // t = 64 .. 512
        const int half = 1 << s;
#pragma unroll
        for (int g = 0; g < 2; g++) {
#define IA16_I(b) (((b) / half) * 2 * half + (b) % half)
#define IA16_W(b) twL[half - 1 + (b) % half]
            BF4(IA16_I(4 * g), IA16_I(4 * g) + half, IA16_W(4 * g), IA16_I(4 * g + 1), IA16_I(4 * g + 1) + half, IA16_W(4 * g + 1),
                IA16_I(4 * g + 2), IA16_I(4 * g + 2) + half, IA16_W(4 * g + 2), IA16_I(4 * g + 3), IA16_I(4 * g + 3) + half, IA16_W(4 * g + 3));
        }
    }
}
