/*
 * silenzio_pbs.h -- C ABI of the MI355X (gfx950) library for batched TFHE programmable
 * bootstrapping (PBS) and LWE key switching, the operation behind every lookup-table step
 * ("lookupComp", mod, ReLU, max, shifts) of the Silenzio training scheme (paper Sec.
 * "TFHE & Concrete" and Sec. "Training Scheme"; the paper uses the PBS of TFHE/CGGI as a
 * black box, so the conventions below are the contract).
 *
 * Arithmetic: the discretised torus Z_q with q = 2^64 (uint64_t, wrapping).  Polynomials live
 * in Z_q[X]/(X^N+1).  Every result is exact: output ciphertexts are a deterministic function
 * of the input bytes (no floating-point error reaches them).
 *
 * Conventions
 *   - Return value: 0 (SLZ_OK) on success, a negative SLZ_E_* code otherwise.  No exceptions,
 *     no aborts, nothing printed.  slz_strerror() names a code.
 *   - "dev" pointers are device (HBM) addresses valid on the current HIP device; "host"
 *     pointers are ordinary host memory.  The caller owns every buffer it passes; the library
 *     never frees or retains caller memory (a context keeps its own scratch).
 *   - All device work is enqueued on the hipStream_t passed as `hip_stream` (a void*; NULL is
 *     the default stream) and is asynchronous: outputs are valid once the stream has been
 *     synchronised by the caller.  Inputs must stay alive and unmodified until then.
 *   - Input and output buffers must not overlap.  Keys, tables and prepared keys must be 16-byte aligned;
 *     ciphertext arrays 8-byte aligned (their rows have an odd number of words, so any sub-batch of a
 *     ciphertext array is a valid argument).
 *   - A context is bound to the device current at creation and is not thread-safe; separate
 *     contexts are independent.
 *
 * Layouts (row-major u64)
 *   LWE ciphertext of dimension d : d mask words, then the body.
 *   Accumulator / GLWE            : k mask polynomials, then the body polynomial.
 *   BSK (standard domain)         : [n][k+1 rows r][l levels j, most significant first][k+1 components][N]
 *                                   GGSW of LWE key bit i; row (r,j) = GLWE(0) with s_i * 2^(64 - j*beta)
 *                                   added to the constant coefficient of component r.
 *   KSK                           : [kN][l_ks levels j, most significant first][n+1],
 *                                   KSK[i][j] = LWE_s(s'_i * 2^(64 - j*beta_ks)).
 *   LUT polynomials               : [n_luts][N], the body of a trivial accumulator.
 */
#ifndef SILENZIO_PBS_H
#define SILENZIO_PBS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SLZ_OK             0
#define SLZ_E_INVALID_ARG (-1)   /* null pointer, zero size, N not a power of two, base*level > 64, ... */
#define SLZ_E_UNSUPPORTED (-2)   /* valid parameters for which this build has no exact kernel           */
#define SLZ_E_HIP         (-3)   /* a HIP runtime call failed                                            */
#define SLZ_E_NOMEM       (-4)   /* scratch allocation failed                                            */
#define SLZ_E_TOO_LARGE   (-5)   /* batch exceeds the context's max_batch (or the fixed scratch of a _static call) */

/* A TFHE parameter set.  Plain data, copied by the callee.  One padding bit is implied:
 * messages live in Z_t, t = 2^msg_bits, encoded at Delta = 2^(63 - msg_bits). */
typedef struct {
    uint32_t n;             /* small LWE dimension                       */
    uint32_t k;             /* GLWE dimension                            */
    uint32_t N;             /* polynomial size, a power of two >= 2      */
    uint32_t pbs_base_log;  /* beta: gadget base 2^beta of the PBS       */
    uint32_t pbs_level;     /* l: gadget levels of the PBS               */
    uint32_t ks_base_log;   /* beta_ks                                   */
    uint32_t ks_level;      /* l_ks                                      */
    uint32_t msg_bits;      /* p                                         */
} slz_params;

typedef struct slz_ctx slz_ctx;   /* opaque: parameter copy, twiddle tables, scratch for max_batch */

/* Context options for slz_ctx_set_option. */
#define SLZ_OPT_FORCE_GENERIC 1   /* value != 0: always use the multi-kernel global-memory blind rotation and the
                                     scalar-ALU keyswitch (the kernels every shape has; for cross-checks) */

#define SLZ_OPT_LARGE_N_BLOCK 2   /* value 1024 or 2048: block size of the row pass of the large-N path (default: 1024
                                     when N = 1024 G', G' <= 32, else 2048); SLZ_E_INVALID_ARG if this N cannot use it */

#define SLZ_OPT_LARGE_N_LANES 3   /* value 1 or 2: the large-N path runs one chunk of ciphertexts at a time on the caller's stream
                                     (1), or two half chunks at once on two internal streams that fork from and join
                                     the caller's stream (2, the default: the arithmetic-bound row pass of one half
                                     overlaps the memory-bound column passes of the other; results are identical);
                                     SLZ_E_INVALID_ARG when the context has no large-N path */

#define SLZ_OPT_LARGE_N_LATENCY 5 /* value 1 (default) or 0: on the large-N path with 1024-blocks, calls with so few ciphertexts that
                                     the chip stays mostly empty (at most 1024 / (2 N / 1024): 16 at N = 32768) run every CMux step
                                     as four shorter launches with four times the threads (lower latency, identical results; their
                                     scratch of 2 (k+1) l (k+1) N doubles per such ciphertext is allocated by the first such call);
                                     0 keeps the throughput kernels at every batch size; SLZ_E_INVALID_ARG without a large-N path */

#define SLZ_OPT_FUSED_PACING 6    /* value 1 (default) or 0: the N = 2048 fused kernel's workgroups wait for each other between
                                     ciphertexts (launches of more than 1024 ciphertexts) so that they keep reading the same key
                                     rows from the L2; a wait as long as the waiting workgroup's own ciphertext took ends the
                                     pacing for that launch; 0 lets them run free.  Value 2 (for tests of that give-up path):
                                     paced, but a wait that is not satisfied at once gives up.  Results are identical in
                                     every mode.  SLZ_E_INVALID_ARG on other paths */

#define SLZ_OPT_FAIL_ALLOC_AFTER 4 /* for tests of the out-of-memory handling: value v >= 0 makes the (v+1)-th scratch allocation
                                     from now (of any context of the process) return SLZ_E_NOMEM without touching the device,
                                     once; v < 0 disarms */

/* Allocation and graph capture: slz_pbs_batch, slz_blind_rotate_batch, slz_keyswitch_batch and slz_ks_pbs_batch allocate
 * their scratch (and the large-N path its two internal streams) in the first call on a context; later calls with a batch
 * no larger than max_batch record only kernels and event edges on the given stream and may be captured into a HIP graph
 * (warm up once outside the capture). */

/* Creates a context on the current device.  Allocates transform tables and scratch sized for
 * `max_batch` ciphertexts.  Fails with SLZ_E_UNSUPPORTED when the exactness bound
 * 4 * (k+1) * l * N * 2^(beta-1) * 2^63 <= p1 * p2 (the two ~2^50 transform primes) does not hold. */
int slz_ctx_create(const slz_params *params, uint32_t max_batch, slz_ctx **out);
int slz_ctx_destroy(slz_ctx *ctx);
int slz_ctx_set_option(slz_ctx *ctx, int option, int value);

/* LUT encoding (host, pure function): table f on Z_t -> accumulator body polynomial.
 * table: host u64 [n_tables][t], entries in [0, t).  lut_out: host u64 [n_tables][N].
 * With box = N/t and h = box/2: V[j] = Delta*f((j+h) div box) if (j+h) div box < t, else -Delta*f(0),
 * i.e. boxes of width N/t rotated down by half a box.  Requires N >= 2t.  The output message keeps
 * the input encoding (Delta_out = Delta_in). */
int slz_lut_encode(const slz_params *params, const uint64_t *table_host, uint32_t n_tables,
                   uint64_t *lut_out_host);

/* One-off key preparation: standard-domain BSK (device) -> library-private transform-domain form in
 * caller-provided device memory.  Call with dst_dev == NULL to obtain the required size in *dst_bytes;
 * otherwise *dst_bytes must be at least that size. */
int slz_bsk_prepare(slz_ctx *ctx, const uint64_t *bsk_dev, void *dst_dev, size_t *dst_bytes,
                    void *hip_stream);

/* Programmable bootstrapping of `batch` LWE ciphertexts (1 <= batch <= max_batch):
 *   modulus switch to 2N (add-half-then-shift), ACC = (0,..,0, X^{-b~} * LUT[lut_idx[c]]),
 *   for i = 0..n-1 in order: ACC <- ACC + BSK_i [.] (X^{a~_i} ACC - ACC)   (external product with the
 *   signed gadget decomposition, digits in [-B/2, B/2), rounding by add-half-then-shift),
 *   then sample extraction of the constant coefficient.
 * lwe_in_dev  [batch][n+1];  luts_dev [n_luts][N];  lut_idx_dev [batch] (values < n_luts, not checked
 * on device) or NULL (all ciphertexts use LUT 0);  bsk_prepared_dev from slz_bsk_prepare;
 * lwe_out_dev [batch][kN+1] under the flattened GLWE key. */
int slz_pbs_batch(slz_ctx *ctx, const uint64_t *lwe_in_dev, const uint64_t *luts_dev,
                  const uint32_t *lut_idx_dev, uint32_t n_luts, const void *bsk_prepared_dev,
                  uint64_t *lwe_out_dev, uint32_t batch, void *hip_stream);

/* The same pipeline stopped after `n_steps` CMux steps (0 <= n_steps <= n), returning the
 * accumulators instead of extracting: acc_out_dev [batch][k+1][N].  n_steps = 0 gives the
 * initial accumulators.  Used to check intermediate states of the blind rotation. */
int slz_blind_rotate_batch(slz_ctx *ctx, const uint64_t *lwe_in_dev, const uint64_t *luts_dev,
                           const uint32_t *lut_idx_dev, uint32_t n_luts, const void *bsk_prepared_dev,
                           uint32_t n_steps, uint64_t *acc_out_dev, uint32_t batch, void *hip_stream);

/* LWE key switching from dimension kN to n:
 *   out = (0,..,0, b') - sum_{i<kN} sum_{j=1..l_ks} d_j(a'_i) * KSK[i][j]   (vectors of n+1 words).
 * lwe_in_dev [batch][kN+1];  ksk_dev [kN][l_ks][n+1];  lwe_out_dev [batch][n+1].
 * With a keyswitch base of at most 2^8 and kN a multiple of 32 the contraction runs on the int8 matrix cores; its
 * digit scratch (32 * ceil(max_batch / 32) * kN * l_ks bytes) is allocated by the first such call (SLZ_E_NOMEM if
 * that fails) and larger batches are taken in chunks of max_batch. */
int slz_keyswitch_batch(slz_ctx *ctx, const uint64_t *lwe_in_dev, const uint64_t *ksk_dev,
                        uint64_t *lwe_out_dev, uint32_t batch, void *hip_stream);

/* The keyswitching key in the form the matrix-core contraction consumes (one-off, untimed, like slz_bsk_prepare): every
 * 64-bit key word as eight signed bytes b_p with word = sum_p b_p 2^(8p) (mod 2^64), laid out as the contraction's operands.
 * ksk_dev as for slz_keyswitch_batch; dst_dev: caller-provided device memory, 16-byte aligned; with dst_dev == NULL only
 * *dst_bytes is set (about 32 ceil((n+1)/32) kN l_ks bytes: the size of the key rounded up to 32 output words).
 * SLZ_E_UNSUPPORTED when the parameter set does not use the matrix cores (keyswitch base above 2^8, or kN not a multiple
 * of 32); SLZ_E_INVALID_ARG when *dst_bytes is too small. */
int slz_ksk_prepare(slz_ctx *ctx, const uint64_t *ksk_dev, void *dst_dev, size_t *dst_bytes, void *hip_stream);

/* slz_keyswitch_batch with the key from slz_ksk_prepare: same ciphertext layouts, same result bit for bit, without the
 * recoding of the key inside the contraction.  Scratch and chunking as for slz_keyswitch_batch. */
int slz_keyswitch_batch_prepared(slz_ctx *ctx, const uint64_t *lwe_in_dev, const void *ksk_prepared_dev,
                                 uint64_t *lwe_out_dev, uint32_t batch, void *hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): slz_keyswitch_batch on the int8 matrix cores with its digit scratch in a fixed device array of
 * SLZ_KS_STATIC_SCRATCH_BYTES inside the library instead of a buffer of the context.  The call itself allocates and
 * frees nothing, on the device or through any library.  Same arguments, layouts and result (bit for bit) as
 * slz_keyswitch_batch.  Limits: keyswitch base at most 2^8 and kN a multiple of 32 (SLZ_E_UNSUPPORTED otherwise);
 * 1024 * ceil(batch / 32) * (kN * l_ks / 32) bytes must fit the array (SLZ_E_TOO_LARGE otherwise: 1632 ciphertexts at
 * kN = 2048, l_ks = 5; 96 at kN = 32768, l_ks = 5); the context's device must be current (SLZ_E_INVALID_ARG otherwise).
 * All calls on one device share the one array, whatever their context or stream: calls that overlap on a device race,
 * so order them on one stream or with events.  The array keeps the last call's digits; every slot a call reads it has
 * written first. */
#define SLZ_KS_STATIC_SCRATCH_BYTES (16u << 20)
int slz_keyswitch_batch_static(slz_ctx *ctx, const uint64_t *lwe_in_dev, const uint64_t *ksk_dev,
                               uint64_t *lwe_out_dev, uint32_t batch, void *hip_stream);

/* Keyswitch-first order (the order in which a compiler for the scheme usually chains the two): ciphertexts stay under the
 * big key between lookups, and one lookup is   lwe_out = PBS(keyswitch(lwe_in)).
 * lwe_in_dev, lwe_out_dev [batch][kN+1] (they may be the same buffer); the other arguments as for slz_keyswitch_batch and
 * slz_pbs_batch; 1 <= batch <= max_batch (SLZ_E_TOO_LARGE above).  The n+1-word ciphertexts between the two steps live in
 * a scratch buffer of the context (max_batch rows, allocated by the first call; SLZ_E_NOMEM if that fails), so calls on one
 * context must not overlap.  The result is bit-identical to calling the two entry points one after the other. */
int slz_ks_pbs_batch(slz_ctx *ctx, const uint64_t *lwe_in_dev, const uint64_t *ksk_dev, const uint64_t *luts_dev,
                     const uint32_t *lut_idx_dev, uint32_t n_luts, const void *bsk_prepared_dev,
                     uint64_t *lwe_out_dev, uint32_t batch, void *hip_stream);

/* Integer linear combination of LWE ciphertexts with clear weights (the leveled sums of step 3 of
 * the paper's Matmul^RNS algorithm):  out[g][o] = sum_{j<J} w[j][o] * ct[g][j]  as vectors of n+1 words.
 * cts_dev [G][J][n+1];  w_dev int32 [J][O];  out_dev [G][O][n+1]. */
int slz_lwe_lincomb_batch(slz_ctx *ctx, const uint64_t *cts_dev, const int32_t *w_dev,
                          uint64_t *out_dev, uint32_t G, uint32_t J, uint32_t O, void *hip_stream);

/* Name of the kernel path slz_pbs_batch will use for this context ("fused_n512", "fused_n1024", "fused_n2048",
 * "fused_n4096", "three_pass_large_n", "generic"). */
const char *slz_pbs_path(const slz_ctx *ctx);

const char *slz_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* SILENZIO_PBS_H */
