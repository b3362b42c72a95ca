/* Gadgets built on the lookup primitive of silenzio_pbs.h (one lookup = slz_pbs_batch + slz_keyswitch_batch).
 *
 * Matmul^RNS (the paper's Algorithm "Matmul^RNS", Sec. "Low-bitwidth Matrix Multiplication"): the product of an
 * encrypted a x b matrix X and an encrypted b x c matrix W of signed 8-bit integers, returned as encrypted residues
 * modulo each modulus of an RNS base of 4-bit moduli.  The three steps run as the paper orders them:
 *   1. X' = X mod m', W' = W mod m'           one lookup per entry and modulus (table v -> signed(v) mod m_i)
 *   2. Y* = X' W' mod m (all a b c products)  one lookup per product on the packed value 16 x' + w'
 *   3. sums of at most 15 products, each running sum reduced modulo m_i by one lookup.
 * Every ciphertext lives in the context's message space, which must have msg_bits >= 8 (packed values and block sums
 * reach 255); signed inputs are encoded with negative values in the upper half of Z_{2^msg_bits}.
 *
 * Same conventions as silenzio_pbs.h: C ABI, plain pointers, caller owns every buffer, work is enqueued on the given
 * HIP stream, return codes are the SLZ_* codes.
 */
#ifndef SILENZIO_GADGETS_H
#define SILENZIO_GADGETS_H
#include "silenzio_pbs.h"

#ifdef __cplusplus
extern "C" {
#endif

#define SLZ_MATMUL_RNS_MAX_K 8
#define SLZ_MATMUL_RNS_BLOCK 15     /* summands per sub-sum in step 3 */

typedef struct {
    uint32_t k;                          /* number of moduli, 1..SLZ_MATMUL_RNS_MAX_K */
    uint32_t m[SLZ_MATMUL_RNS_MAX_K];    /* the RNS base; every modulus in [2, 16] */
    uint32_t a, b, c;                    /* X is a x b, W is b x c */
} slz_matmul_rns_shape;

/* Host, pure: the 3k lookup tables as accumulator polynomials (slz_lut_encode of each), luts_out [3k][N] host words:
 *   [0, k)    v -> signed(v) mod m_i   (step 1; signed(v) = v below 2^(msg_bits-1), v - 2^msg_bits above)
 *   [k, 2k)   u -> (u >> 4)(u & 15) mod m_i for u < 256, 0 above   (step 2)
 *   [2k, 3k)  v -> v mod m_i           (step 3)
 * SLZ_E_INVALID_ARG for a bad shape or msg_bits < 8. */
int slz_matmul_rns_luts(const slz_params *params, const slz_matmul_rns_shape *shape, uint64_t *luts_out);

/* Bytes of device workspace slz_matmul_rns needs for this shape on this context. */
int slz_matmul_rns_workspace(const slz_ctx *ctx, const slz_matmul_rns_shape *shape, size_t *bytes);

/* x_dev [a][b][n+1], w_dev [b][c][n+1]: LWE encryptions under the small key; luts_dev [3k][N]: the polynomials of
 * slz_matmul_rns_luts copied to the device; bsk_prepared_dev / ksk_dev as for slz_pbs_batch / slz_keyswitch_batch;
 * y_dev [k][a][c][n+1]: encrypted residues of X W; workspace_dev: at least slz_matmul_rns_workspace bytes, 256-byte
 * aligned, contents undefined before and after.  Lookups larger than the context's max_batch are taken in chunks.
 * Buffers must not overlap.  SLZ_E_INVALID_ARG for null or misaligned pointers, a bad shape, msg_bits < 8 or a
 * workspace that is too small. */
int slz_matmul_rns(slz_ctx *ctx, const slz_matmul_rns_shape *shape, const uint64_t *x_dev, const uint64_t *w_dev,
                   const uint64_t *luts_dev, const void *bsk_prepared_dev, const uint64_t *ksk_dev, uint64_t *y_dev,
                   void *workspace_dev, size_t workspace_bytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SILENZIO_GADGETS_H */
