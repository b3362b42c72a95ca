// Internal declarations shared by the translation units of libsilenzio_pbs (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/silenzio_pbs.h"

// ---- exact transform arithmetic -------------------------------------------------------------
// Negacyclic products mod 2^64 are computed exactly through two number-theoretic transforms over
// primes just below 2^50 (both = 1 mod 2^18, so N up to 2^17 has a primitive 2N-th root) and a CRT
// lift.  Residues are held in doubles: on gfx950 an FP64 FMA issues at the full VALU rate and carries
// a 53-bit product, which makes a 50-bit modular multiply 6 instructions (see slz_modarith.h).
#define SLZ_P1 1125899902124033.0   /* 0x3ffffffb80001 */
#define SLZ_P2 1125899886395393.0   /* 0x3fffffec80001 */
#define SLZ_P1_U64 1125899902124033ull
#define SLZ_P2_U64 1125899886395393ull
#define SLZ_MAX_LOGN 17

struct slz_mod {          // one transform prime, passed to kernels by value
    double p;             // the prime
    double pinv;          // nearest double to 1/p
};

// Position of transform-domain coefficient `idx` (index in the bit-reversed output order of the
// forward transform) inside a prepared polynomial.  The fused kernels hold 32 consecutive outputs per
// lane, so the prepared key is stored register-major / lane-minor to make their loads coalesced.
__host__ __device__ static inline uint32_t slz_prep_pos(uint32_t idx, uint32_t N) {
    uint32_t E = N < 32 ? N : 32;
    return (idx % E) * (N / E) + idx / E;
}

struct slz_tables {       // device tables of one prime (all doubles, centred residues)
    double *fwd;          // [N]  fwd[m+i] = psi^bitrev(m+i): merged negacyclic forward twiddles
    double *inv;          // [N]  inv[t+j] = psi^(-(N/t) j), j < t: cyclic inverse twiddles of half-size t
    double *post;         // [N]  post[j] = psi^(-j) / N
};

struct slz_ctx {
    slz_params prm;
    uint32_t max_batch;
    int device;
    int force_generic;
    int has_fused;
    int has_fused4096;        // the N = 4096 fused kernel is available
    double *fused4096_rowA, *fused4096_rowB;   // its block tables: [2][2][64] and [2][2][31][64]
    double fused4096_scalars[2][128];          // host copy of fused4096_rowA (lane-uniform entries go into the kernel arguments)
    double fused4096_w1[2];                    // fwd[1] per prime: the twiddle of the stage across the two blocks
    int has_fused512;         // the N = 512 fused kernel is available
    double *fused512_rowA, *fused512_rowB;     // its forward tables: [2][64] and [2][15][64]
    int has_fused1024;        // the N = 1024 fused kernel is available
    double *fused1024_rowA, *fused1024_rowB;   // its forward tables: [2][64] and [2][15][64]
    uint32_t logN;
    slz_mod mod[2];
    double two32[2];          // 2^32 mod p_i (centred)
    double p1inv_mod_p2;      // p1^{-1} mod p2 (centred)
    slz_tables tab[2];
    double *fused_tab;        // tables re-laid-out for the fused kernel (or null)
    uint32_t *fused_sync;     // arrival counters of the fused kernel's pacing between ciphertexts
    int fused_pacing;         // 1: workgroups of the N = 2048 fused kernel wait for each other between ciphertexts
    double fused_scalars[2][2][32];   // [prime][forward, inverse]: the lane-uniform twiddles of the fused kernel
    int has_bign;             // large-N three-pass path available (N = 2048 G, k = 1)
    double *bign_rowA;        // [2][G][64] block-specific lane-uniform forward twiddles
    double *bign_rowB;        // [2][G][31][64] block-specific per-lane forward twiddles
    int has_bign16;           // large-N path with 1024-blocks available (N = 1024 G', G' = 2..32, k = 1)
    int bign_lanes;           // 1: one chunk at a time on the caller's stream; 2: two half chunks on two internal streams
    void *bign_lane_stream[2], *bign_lane_done[2], *bign_fork;   // hipStream_t / hipEvent_t of the lanes, created at first use
    int bign_block;           // block size the large-N path uses: 1024 or 2048
    int bign_latency;         // 1: a handful of ciphertexts take the latency-oriented kernels (four shorter launches per step)
    double *bign_partial;     // their partial products [few ciphertexts][2][R][2][N], allocated at first use
    double *bign16_rowA;      // [2][G'][64] as bign_rowA for 1024-blocks
    double *bign16_rowB;      // [2][G'][15][64] per-lane twiddles of the last four forward stages of a 1024-block
    // scratch for the generic path, sized for max_batch
    uint64_t *acc;            // [max_batch][k+1][N]
    double *dig;              // [max_batch][(k+1)l][N]
    double *xhat;             // [max_batch][2][(k+1)l][N]
    double *outhat;           // [max_batch][2][k+1][N]
    uint64_t *ks_first_small;   // slz_ks_pbs_batch: keyswitch outputs [max_batch][n+1], allocated on first use
    void *ks_dig;             // digit bytes of the matrix-core keyswitch (allocated at its first call)
    void *lc_dig;             // weight digit planes of the matrix-core linear combination (grown on demand)
    size_t lc_dig_bytes;
    uint32_t fwd_reduce_mask; // bit s: fully reduce all values before forward stage s (0-based)
    uint32_t inv_reduce_mask; // same for the inverse stages
    double fwd_out_bound;     // bound (in units of p) of forward outputs
};

#define SLZ_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) return SLZ_E_HIP; } while (0)

// scratch allocation of the entry points (slz_api.hip): SLZ_OK or SLZ_E_NOMEM, *out null on failure
int slz_scratch_alloc(void **out, size_t bytes);

// host side (slz_tables.cpp)
int slz_build_tables(slz_ctx *ctx);
void slz_free_tables(slz_ctx *ctx);
// bound bookkeeping shared by host checks
double slz_mulmod_bound(double in_bound);

// generic path (slz_generic.hip)
int slz_generic_bsk_prepare(slz_ctx *ctx, const uint64_t *bsk, double *dst, hipStream_t s);
int slz_generic_blind_rotate(slz_ctx *ctx, const uint64_t *lwe_in, const uint64_t *luts, const uint32_t *lut_idx,
                             const double *bskp, uint32_t n_steps, uint64_t *acc_out, uint64_t *lwe_out,
                             uint32_t batch, hipStream_t s);
// fused path for N = 4096 (slz_fused_n4096.hip)
int slz_fused4096_supported(const slz_params *p);
int slz_fused4096_init(slz_ctx *ctx);
void slz_fused4096_destroy(slz_ctx *ctx);
int slz_fused4096_blind_rotate(slz_ctx *ctx, const uint64_t *lwe_in, const uint64_t *luts, const uint32_t *lut_idx,
                               const double *bskp, uint32_t n_steps, uint64_t *acc_out, uint64_t *lwe_out, uint32_t batch,
                               hipStream_t s);
// fused path for N = 512 (slz_fused_n512.hip)
int slz_fused512_supported(const slz_params *p);
int slz_fused512_init(slz_ctx *ctx);
void slz_fused512_destroy(slz_ctx *ctx);
int slz_fused512_blind_rotate(slz_ctx *ctx, const uint64_t *lwe_in, const uint64_t *luts, const uint32_t *lut_idx,
                              const double *bskp, uint32_t n_steps, uint64_t *acc_out, uint64_t *lwe_out, uint32_t batch,
                              hipStream_t s);
// fused path for N = 1024 (slz_fused_n1024.hip)
int slz_fused1024_supported(const slz_params *p);
int slz_fused1024_init(slz_ctx *ctx);
void slz_fused1024_destroy(slz_ctx *ctx);
int slz_fused1024_blind_rotate(slz_ctx *ctx, const uint64_t *lwe_in, const uint64_t *luts, const uint32_t *lut_idx,
                               const double *bskp, uint32_t n_steps, uint64_t *acc_out, uint64_t *lwe_out, uint32_t batch,
                               hipStream_t s);
// forward twiddle tables of the blocks of size BS of the wave-level transforms (slz_bign.hip): *dA [2][N/BS][64],
// *dB [2][N/BS][BS/64 - 1][64], device memory owned by the caller
int slz_build_block_tables(slz_ctx *ctx, uint32_t BS, double **dA, double **dB);

// fused path (slz_fused.hip)
int slz_fused_supported(const slz_params *p);
int slz_fused_init(slz_ctx *ctx);
void slz_fused_destroy(slz_ctx *ctx);
int slz_fused_blind_rotate(slz_ctx *ctx, const uint64_t *lwe_in, const uint64_t *luts, const uint32_t *lut_idx,
                           const double *bskp, uint32_t n_steps, uint64_t *acc_out, uint64_t *lwe_out,
                           uint32_t batch, hipStream_t s);
// large-N path (slz_bign.hip)
int slz_bign_supported(const slz_params *p);
int slz_bign_init(slz_ctx *ctx);
void slz_bign_destroy(slz_ctx *ctx);
int slz_bign_cmux_steps(slz_ctx *ctx, const uint64_t *lwe_in, const double *bskp, uint32_t n_steps, uint64_t *acc,
                        uint32_t batch, hipStream_t s);
// keyswitch / lincomb (slz_keyswitch.hip)
int slz_keyswitch_launch(slz_ctx *ctx, const uint64_t *lwe_in, const uint64_t *ksk, uint64_t *lwe_out,
                         uint32_t batch, hipStream_t s);
// out = (0, .., 0, b') for every ciphertext: the start value of both keyswitch kernels
void slz_ks_init_launch(const uint64_t *lwe_in, uint64_t *lwe_out, uint32_t kN, uint32_t n, uint32_t batch, hipStream_t s);
// matrix-core keyswitch (slz_keyswitch_mfma.hip); lwe_out must already hold (0, .., 0, b')
int slz_ksm_supported(const slz_params *p);
void slz_ksm_destroy(slz_ctx *ctx);
int slz_ksm_launch(slz_ctx *ctx, const uint64_t *lwe_in, const uint64_t *ksk, const void *kskp, uint64_t *lwe_out, uint32_t batch,
                   hipStream_t s);
size_t slz_ksm_prepared_bytes(const slz_params *p);
int slz_ksm_prepare(slz_ctx *ctx, const uint64_t *ksk, void *dst, hipStream_t s);
// matrix-core linear combination (slz_lincomb_mfma.hip)
void slz_lcm_destroy(slz_ctx *ctx);
int slz_lcm_launch(slz_ctx *ctx, const uint64_t *cts, const int32_t *w, uint64_t *out, uint32_t G, uint32_t J, uint32_t O,
                   hipStream_t s);
int slz_lincomb_launch(slz_ctx *ctx, const uint64_t *cts, const int32_t *w, uint64_t *out, uint32_t G, uint32_t J,
                       uint32_t O, hipStream_t s);
