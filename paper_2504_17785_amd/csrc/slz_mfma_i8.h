// Pieces shared by the int8 matrix-core contractions (keyswitch, clear-weight linear combination).
#pragma once
#include <stdint.h>

typedef int v16i __attribute__((ext_vector_type(16)));
typedef int v4i __attribute__((ext_vector_type(4)));

// A 64-bit word w as eight signed bytes s_p in [-128, 128) with w = sum_p s_p 2^(8p) (mod 2^64): byte p of the result,
// read as int8, is s_p.
__device__ __forceinline__ uint64_t slz_signed_bytes(uint64_t w) {
    return (w + 0x8080808080808080ull) ^ 0x8080808080808080ull;
}

// 4x4 byte transpose of four dwords: o[p] = byte p of a0, a1, a2, a3 (a0 in the low byte)
__device__ __forceinline__ void slz_tr4_bytes(uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3, uint32_t o[4]) {
    uint32_t t01l = __builtin_amdgcn_perm(a1, a0, 0x05010400u);   // a0.b0 a1.b0 a0.b1 a1.b1
    uint32_t t01h = __builtin_amdgcn_perm(a1, a0, 0x07030602u);   // a0.b2 a1.b2 a0.b3 a1.b3
    uint32_t t23l = __builtin_amdgcn_perm(a3, a2, 0x05010400u);
    uint32_t t23h = __builtin_amdgcn_perm(a3, a2, 0x07030602u);
    o[0] = __builtin_amdgcn_perm(t23l, t01l, 0x05040100u);
    o[1] = __builtin_amdgcn_perm(t23l, t01l, 0x07060302u);
    o[2] = __builtin_amdgcn_perm(t23h, t01h, 0x05040100u);
    o[3] = __builtin_amdgcn_perm(t23h, t01h, 0x07060302u);
}

// Eight words (rows 0..7 of one output column) to their eight byte-plane operands: plane[p] holds byte p of rows 0..7,
// row 0 in the lowest byte.
__device__ __forceinline__ void slz_byte_planes(const uint64_t (&w)[8], uint64_t (&plane)[8]) {
    uint32_t lo[8], hi[8];
#pragma unroll
    for (int t = 0; t < 8; t++) { lo[t] = (uint32_t)w[t]; hi[t] = (uint32_t)(w[t] >> 32); }
    uint32_t pl0[4], pl1[4], ph0[4], ph1[4];
    slz_tr4_bytes(lo[0], lo[1], lo[2], lo[3], pl0);               // planes 0..3, rows 0..3
    slz_tr4_bytes(lo[4], lo[5], lo[6], lo[7], pl1);               // planes 0..3, rows 4..7
    slz_tr4_bytes(hi[0], hi[1], hi[2], hi[3], ph0);               // planes 4..7, rows 0..3
    slz_tr4_bytes(hi[4], hi[5], hi[6], hi[7], ph1);
#pragma unroll
    for (int p = 0; p < 4; p++) {
        plane[p] = (uint64_t)pl0[p] | ((uint64_t)pl1[p] << 32);
        plane[p + 4] = (uint64_t)ph0[p] | ((uint64_t)ph1[p] << 32);
    }
}
