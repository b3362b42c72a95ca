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

/* ---- MatmulHighRes^RNS (the paper's Algorithm of that name, appendix "Low-bitwidth high-resolution MatMul") -------------------
 * The same product modulo a base of 5-bit moduli (every modulus in [2, 32]) with every intermediate still within 8 bits:
 *   1. X' = X mod m', W' = W mod m'                         one lookup per entry and modulus
 *   2. X2' = bits 3..4 of X', X1' = bits 0..2 of X'          one lookup each
 *   3. Y1* = X1' W' mod m (two-input lookup on 32 x1 + w);  Y2* = X2' W' (two-input lookup on 32 x2 + w, the plain product),
 *      then the lookup v -> 8 v mod m
 *   4. Y* = (Y1* + Y2*) mod m                                one lookup per product
 *   5. sums of at most 7 entries, each running sum reduced modulo m_i by one lookup.
 * The shape struct is the one of slz_matmul_rns; conventions are the same. */
#define SLZ_MATMUL_HIGHRES_BLOCK 7     /* summands per sub-sum in step 5 */

/* Host, pure.  luts_out [4k + 3][N]: k tables v -> signed(v) mod m_i, k tables u -> (u >> 5)(u & 31) mod m_i (u < 256),
 * k tables v -> 8 v mod m_i, k tables v -> v mod m_i, then v -> (v >> 3) & 3, v -> v & 7 and u -> (u >> 5)(u & 31). */
int slz_matmul_highres_luts(const slz_params *params, const slz_matmul_rns_shape *shape, uint64_t *luts_out);
int slz_matmul_highres_workspace(const slz_ctx *ctx, const slz_matmul_rns_shape *shape, size_t *bytes);
/* Arguments as for slz_matmul_rns, with luts_dev the polynomials of slz_matmul_highres_luts. */
int slz_matmul_highres(slz_ctx *ctx, const slz_matmul_rns_shape *shape, const uint64_t *x_dev, const uint64_t *w_dev,
                       const uint64_t *luts_dev, const void *bsk_prepared_dev, const uint64_t *ksk_dev, uint64_t *y_dev,
                       void *workspace_dev, size_t workspace_bytes, void *hip_stream);

/* ---- RNS-to-MRNS conversion (the paper's Algorithm "RNS2MRNS") and sign determination (Sec. "Sign Determination in
 * RNS") on encrypted residues ---------------------------------------------------------------------------------------
 * A number x of Z_M, M = m_1 .. m_k, is given as k ciphertexts of its residues x_i = x mod m_i (all in the context's
 * message space, msg_bits >= 8).  The conversion returns the digits y_i of the associated mixed-radix system
 * (x = y_1 + y_2 m_1 + y_3 m_1 m_2 + ..): for i = 2..k, every later digit j >= i is replaced by
 * (y_j - y_{i-1}) (m_{i-1}^-1 mod m_j) mod m_j, one lookup per (i, j) on the difference moved up by the constant 16;
 * k - 1 dependent rounds, k (k - 1) / 2 lookups per number.
 * Sign_(n,z,p): n for negative x (upper half of Z_M; the top modulus must be even), z for zero, p for positive x.  After
 * the conversion: one lookup on the top digit (y_k >= m_k / 2), then one on (sum of the digits) + 128 [negative]. */
typedef struct {
    uint32_t k;                          /* number of moduli, 2..SLZ_MATMUL_RNS_MAX_K */
    uint32_t m[SLZ_MATMUL_RNS_MAX_K];    /* pairwise coprime moduli in [2, 16] */
    uint32_t count;                      /* numbers converted per call */
} slz_rns_shape;

/* Host, pure.  luts_out [k (k-1) / 2 + 2][N] host words: the conversion tables in the order (1,2), (1,3), .., (2,3), ..
 * (table v -> (v - 16) (m_i^-1 mod m_j) mod m_j), then the top-digit table and the final table of the sign gadget for
 * the results neg, zero, pos (each in [-128, 127], encoded with negatives in the upper half of the message space).
 * SLZ_E_INVALID_ARG for a bad shape (moduli not coprime included) or msg_bits < 8. */
int slz_rns_luts(const slz_params *params, const slz_rns_shape *shape, int32_t neg, int32_t zero, int32_t pos,
                 uint64_t *luts_out);

/* Bytes of device workspace slz_rns2mrns / slz_sign_rns need for this shape on this context. */
int slz_rns_workspace(const slz_ctx *ctx, const slz_rns_shape *shape, size_t *bytes);

/* x_dev [k][count][n+1] residues -> y_dev [k][count][n+1] mixed-radix digits.  luts_dev: the polynomials of slz_rns_luts
 * on the device.  Workspace and error conventions as for slz_matmul_rns. */
int slz_rns2mrns(slz_ctx *ctx, const slz_rns_shape *shape, const uint64_t *x_dev, const uint64_t *luts_dev,
                 const void *bsk_prepared_dev, const uint64_t *ksk_dev, uint64_t *y_dev, void *workspace_dev,
                 size_t workspace_bytes, void *hip_stream);

/* x_dev [k][count][n+1] residues -> s_dev [count][n+1] encryptions of neg / zero / pos (the values given to slz_rns_luts).
 * SLZ_E_INVALID_ARG also when the top modulus is odd. */
int slz_sign_rns(slz_ctx *ctx, const slz_rns_shape *shape, const uint64_t *x_dev, const uint64_t *luts_dev,
                 const void *bsk_prepared_dev, const uint64_t *ksk_dev, uint64_t *s_dev, void *workspace_dev,
                 size_t workspace_bytes, void *hip_stream);

/* ---- Shift2MSBs^+ and Shift2MSBs^+- (the paper's Algorithms of those names): approximate block scaling ---------------
 * The whole tensor (count numbers given as encrypted residues) is scaled down so that its largest element keeps its
 * gamma most significant bits, viewing the mixed-radix digits as w-bit chunks of a binary number:
 *   1. RNS-to-MRNS conversion;  2. per digit a lookup of the 1-indexed position of its highest set bit (0 for a zero
 *   digit) + i w, then the maximum over all digits of all numbers (binary tree of max(a, b) = b + ReLU(a - b), one lookup
 *   per pair and level);  3. per digit position a lookup maxBit -> shift code;  4. per digit a two-input lookup on
 *   16 code + digit applying the left or right shift;  5. the sum of the shifted digits;  6. shift = maxBit - gamma.
 * Shift2MSBs^+- handles signed numbers (negatives in the upper half of Z_M; even top modulus): flag [x < 0] by the sign
 * gadget, |x| per residue by a two-input lookup on 16 flag + residue, Shift2MSBs^+ with gamma, and the sign put back by
 * a lookup on 128 flag + Y^+.  Outputs: y_dev [count][n+1] (for +-: signed, negatives in the upper half of the message
 * space) and shift_dev [n+1], one ciphertext of maxBit - gamma (signed the same way). */
typedef struct {
    uint32_t k;                          /* number of moduli, 2..6 */
    uint32_t m[SLZ_MATMUL_RNS_MAX_K];    /* pairwise coprime moduli in [2, 16] */
    uint32_t count;                      /* numbers in the tensor */
    uint32_t w;                          /* digit bitwidth; must be 4 */
    uint32_t gamma;                      /* unsigned output bitwidth, 1..7 (for the signed variant: Gamma - 1) */
} slz_shift_shape;

/* Host, pure.  luts_out [k (k-1) / 2 + 3k + 5][N]: the tables of slz_rns_luts for (neg, zero, pos) = (1, 0, 0), then k bit-position
 * tables, the ReLU table of the maximum, k shift-code tables, the shift-application table, k absolute-value tables and
 * the sign-reapplication table. */
int slz_shift2msbs_luts(const slz_params *params, const slz_shift_shape *shape, uint64_t *luts_out);
int slz_shift2msbs_workspace(const slz_ctx *ctx, const slz_shift_shape *shape, size_t *bytes);
/* x_dev [k][count][n+1] residues of non-negative numbers.  Conventions as for slz_matmul_rns. */
int slz_shift2msbs_plus(slz_ctx *ctx, const slz_shift_shape *shape, const uint64_t *x_dev, const uint64_t *luts_dev,
                        const void *bsk_prepared_dev, const uint64_t *ksk_dev, uint64_t *y_dev, uint64_t *shift_dev,
                        void *workspace_dev, size_t workspace_bytes, void *hip_stream);
/* x_dev [k][count][n+1] residues of signed numbers.  SLZ_E_INVALID_ARG also when the top modulus is odd. */
int slz_shift2msbs_pm(slz_ctx *ctx, const slz_shift_shape *shape, const uint64_t *x_dev, const uint64_t *luts_dev,
                      const void *bsk_prepared_dev, const uint64_t *ksk_dev, uint64_t *y_dev, uint64_t *shift_dev,
                      void *workspace_dev, size_t workspace_bytes, void *hip_stream);

/* ---- Lookup with two encrypted inputs, IntCELossDeriv and the clipped weight update ------------------------------------
 * Two-input lookup (the paper's multivariate lookup; it gives no packing): x in [0, 2^x_bits) and y in [0, 2^y_bits) with
 * x_bits + y_bits <= msg_bits are packed as 2^y_bits x + y by a linear combination of the two ciphertexts, then one lookup;
 * the table is indexed by the packed value.
 * IntCELossDeriv (the paper's Algorithm of that name, Sec. "Integer Cross-Entropy Loss Derivative"), a rows of b classes:
 *   1. E = ReLU(logit)                       one lookup (logits signed, big_gamma bits, negatives in the upper half of Z_t)
 *   2. E = round(2^kappa e^(E - (2^(big_gamma-1) - 1)))      one lookup, ties to even
 *   3. S = sum of E over the row
 *   4. E = round((E 2^kappa + 1) / (S + 1))  two-input lookup on 2^sb E + S, ties to even
 *   5. E = E - label * (sum of E over the row)   the product by a two-input lookup on 2^sb label + sum
 *   6. sign(E)                               one lookup on E + t / 2, results -1 / 0 / 1 (negatives in the upper half)
 * with eb = kappa + 1 bits for an exponential and sb = bits of b 2^kappa for a row sum; eb + sb <= msg_bits is required.
 * Clipped weight update (last step of the paper's Algorithm "End-to-End Training"): clip(W - G) to the signed alpha-bit range
 * by one two-input lookup on 4 (W + 2^(alpha-1)) + code, W signed with negatives in the upper half of Z_t, code = G + 1 in
 * {0, 1, 2} (the sign gadget asked for the results 0 / 1 / 2); alpha + 2 <= msg_bits is required. */
typedef struct {
    uint32_t a, b;                       /* rows (samples) and classes, b <= 16 */
    uint32_t big_gamma;                  /* signed bitwidth of the logits, 2..msg_bits */
    uint32_t kappa;                      /* approximation level of the exponential, >= 1 */
} slz_loss_shape;

/* Bytes of device workspace slz_bivariate_lookup / slz_weight_update need for count ciphertext pairs. */
int slz_bivariate_workspace(const slz_ctx *ctx, uint32_t count, size_t *bytes);
/* x_dev, y_dev, out_dev [count][n+1] under the small key; luts_dev [n_luts][N] accumulator polynomials of tables indexed by
 * 2^y_bits x + y; lut_index_dev [count] device words, or null to use table 0 for every pair.  out_dev may be x_dev or y_dev.
 * SLZ_E_INVALID_ARG for null or misaligned pointers, count == 0, y_bits >= msg_bits or a workspace that is too small. */
int slz_bivariate_lookup(slz_ctx *ctx, const uint64_t *x_dev, const uint64_t *y_dev, uint32_t y_bits, const uint64_t *luts_dev,
                         const uint32_t *lut_index_dev, uint32_t n_luts, const void *bsk_prepared_dev, const uint64_t *ksk_dev,
                         uint64_t *out_dev, uint32_t count, void *workspace_dev, size_t workspace_bytes, void *hip_stream);

/* Host, pure.  luts_out [5][N]: the tables of steps 1, 2, 4, 5 and 6 above.  SLZ_E_INVALID_ARG for a shape that does not fit
 * the message space. */
int slz_loss_luts(const slz_params *params, const slz_loss_shape *shape, uint64_t *luts_out);
int slz_loss_workspace(const slz_ctx *ctx, const slz_loss_shape *shape, size_t *bytes);
/* logits_dev, labels_dev (one-hot, 0 / 1) and e_dev: [a][b][n+1] under the small key; e_dev receives the sign of the error.
 * Conventions as for slz_matmul_rns. */
int slz_int_ce_loss_deriv(slz_ctx *ctx, const slz_loss_shape *shape, const uint64_t *logits_dev, const uint64_t *labels_dev,
                          const uint64_t *luts_dev, const void *bsk_prepared_dev, const uint64_t *ksk_dev, uint64_t *e_dev,
                          void *workspace_dev, size_t workspace_bytes, void *hip_stream);

/* Host, pure.  luts_out [1][N]: the table 4 (w + 2^(alpha-1)) + code -> clip(w - (code - 1)), signed result encoded in Z_t (code 3
 * is read as 2).  SLZ_E_INVALID_ARG unless 2 <= alpha and alpha + 2 <= msg_bits. */
int slz_weight_update_luts(const slz_params *params, uint32_t alpha, uint64_t *luts_out);
/* w_dev, gcode_dev, w_out_dev [count][n+1]; workspace of slz_bivariate_workspace(count) bytes.  w_out_dev may be w_dev. */
int slz_weight_update(slz_ctx *ctx, uint32_t alpha, const uint64_t *w_dev, const uint64_t *gcode_dev, const uint64_t *luts_dev,
                      const void *bsk_prepared_dev, const uint64_t *ksk_dev, uint64_t *w_out_dev, uint32_t count,
                      void *workspace_dev, size_t workspace_bytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SILENZIO_GADGETS_H */
