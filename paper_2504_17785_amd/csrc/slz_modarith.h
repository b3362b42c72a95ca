// Device arithmetic modulo a prime p < 2^50 on doubles holding exact integers.
//
// Values are kept in a lazy, signed range |x| <= A*p with A a few units; every operation below is
// exact as long as all intermediate integers stay below 2^53 in magnitude, which the callers guarantee
// through the bound bookkeeping (slz_mulmod_bound on the host, the static bounds in the fused kernel).
#pragma once
#include "slz_internal.h"

// x*w mod p for |w| <= p/2.  h + l is the exact 100-bit product (l from the FMA), q the nearest integer to
// x*w/p up to a relative error 3*2^-53, so |result| <= p*(1/2 + 1.5*|x|*2^-53) (see slz_mulmod_bound).
__device__ __forceinline__ double slz_mulmod(double x, double w, slz_mod m) {
    double h = x * w;
    double l = __builtin_fma(x, w, -h);
    double q = __builtin_rint(h * m.pinv);
    return __builtin_fma(-q, m.p, h) + l;
}

// x mod p into |result| <= p/2 (+ a rounding sliver) for |x| < 2^53.
__device__ __forceinline__ double slz_reduce(double x, slz_mod m) {
    return __builtin_fma(-__builtin_rint(x * m.pinv), m.p, x);
}

// exact double (|x| < 2^51, integer valued) -> two's complement 64-bit integer
__device__ __forceinline__ int64_t slz_d2i(double x) {
    const double magic = 6755399441055744.0;   // 1.5 * 2^52
    return (int64_t)__double_as_longlong(x + magic) - (int64_t)__double_as_longlong(magic);
}

// a signed 64-bit integer (a key word) -> centred residue mod p, via its 32-bit halves
__device__ __forceinline__ double slz_i64_to_res(uint64_t w, slz_mod m, double two32) {
    double hi = (double)(int32_t)(w >> 32);
    double lo = (double)(uint32_t)w;
    double r = slz_mulmod(hi, two32, m) + lo;       // |r| < p + 2^32
    return slz_reduce(r, m);
}

// CRT lift of residues (r1 mod p1, r2 mod p2), |r1|,|r2| <= ~1.5 p, to the centred integer mod p1*p2,
// reduced mod 2^64.  t = (r2 - r1) / p1 mod p2 is made nearly canonical (|t| <= 0.6 p2), so the lift equals
// the true integer whenever that integer is below p1*p2/4 in magnitude.
__device__ __forceinline__ uint64_t slz_crt64(double r1, double r2, slz_mod m2, double p1inv_mod_p2) {
    double d = slz_reduce(r2 - r1, m2);
    double t = slz_mulmod(d, p1inv_mod_p2, m2);
    return (uint64_t)slz_d2i(r1) + (uint64_t)SLZ_P1_U64 * (uint64_t)slz_d2i(t);
}

// Signed gadget digit extraction.  v = the value already rounded to its top beta*l bits and shifted down
// (a beta*l-bit integer).  Peels level `l` first; digits in [-B/2, B/2), carry into the next level.
// Returns digit of the current lowest level and updates v.
__device__ __forceinline__ int32_t slz_next_digit(uint64_t &v, uint32_t beta) {
    uint64_t B = 1ull << beta;
    uint64_t d = v & (B - 1);
    v >>= beta;
    int64_t sd = (int64_t)d;
    if (d >= (B >> 1)) { sd -= (int64_t)B; v += 1; }
    return (int32_t)sd;
}

__device__ __forceinline__ uint64_t slz_round_top_bits(uint64_t x, uint32_t bits) {
    return bits >= 64 ? x : ((x + (1ull << (63 - bits))) >> (64 - bits));
}

__device__ __forceinline__ uint32_t slz_modswitch(uint64_t x, uint32_t log2N2) {
    uint32_t w = 64 - log2N2;
    return (uint32_t)((x + (1ull << (w - 1))) >> w) & ((1u << log2N2) - 1);
}

// coefficient j of X^r * P for r in [0, 2N), P given by a load functor
template <class Load>
__device__ __forceinline__ uint64_t slz_rot_coeff(Load ld, uint32_t j, uint32_t r, uint32_t N) {
    uint32_t neg = 0;
    if (r >= N) { r -= N; neg = 1; }
    uint64_t v;
    if (j >= r) v = ld(j - r);
    else { v = ld(j - r + N); neg ^= 1; }
    return neg ? (uint64_t)0 - v : v;
}
