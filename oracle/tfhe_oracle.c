/*
 * CPU oracle for batched TFHE programmable bootstrapping and LWE key switching.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the GPU
 * library is checked against.  It shares no code with the GPU path, is never
 * linked into it, and must not be called from product code.
 *
 * Everything is exact wrapping arithmetic on the discretised torus Z_q, q = 2^64
 * (uint64_t).  Polynomial products are schoolbook products in Z_q[X]/(X^N + 1).
 * The paper (Silenzio, Sec. "TFHE & Concrete" and Sec. "Training Scheme") uses the
 * programmable bootstrapping of TFHE/CGGI as a black box; the steps below are the
 * textbook CGGI definitions with the free conventions fixed as documented at each
 * function.  The only parallelism is an OpenMP loop over independent ciphertexts.
 *
 * Layouts (all row-major, u64):
 *   LWE ciphertext of dimension d : d mask words, then the body.
 *   GLWE ciphertext               : k mask polynomials, then the body polynomial.
 *   BSK  [n][k+1 (row r)][l (level j, most significant first)][k+1 (component)][N]
 *   KSK  [kN][l_ks (level j, most significant first)][n+1]
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    uint32_t n, k, N;
    uint32_t pbs_base_log, pbs_level;
    uint32_t ks_base_log, ks_level;
    uint32_t msg_bits;
} oracle_params;

/* ---- ring R_q = Z_q[X]/(X^N+1) ------------------------------------------------------------- */

/* Schoolbook negacyclic product: out[c] = sum_{a+b=c} P[a]Q[b] - sum_{a+b=c+N} P[a]Q[b]  (mod 2^64). */
void orc_negacyclic_mul(const uint64_t *P, const uint64_t *Q, uint32_t N, uint64_t *out)
{
    for (uint32_t c = 0; c < N; c++) out[c] = 0;
    for (uint32_t a = 0; a < N; a++) {
        uint64_t pa = P[a];
        if (pa == 0) continue;
        for (uint32_t b = 0; b < N; b++) {
            uint64_t term = pa * Q[b];
            uint32_t c = a + b;
            if (c < N) out[c] += term;
            else       out[c - N] -= term;
        }
    }
}

/* out = X^r * P for r in [0, 2N):  for r < N, out[j] = P[j-r] (j >= r) or -P[j-r+N] (j < r);
 * for r >= N negate and use r - N (because X^N = -1). */
void orc_monomial_mul(const uint64_t *P, uint32_t N, uint32_t r, uint64_t *out)
{
    int negate = 0;
    if (r >= N) { r -= N; negate = 1; }
    for (uint32_t j = 0; j < N; j++) {
        uint64_t v = (j >= r) ? P[j - r] : (uint64_t)0 - P[j - r + N];
        out[j] = negate ? (uint64_t)0 - v : v;
    }
}

/* ---- scalar steps ---------------------------------------------------------------------------- */

/* Signed gadget decomposition of x for base 2^beta and l levels (beta*l <= 64).
 * First round x to its top beta*l bits (add half, shift; ties up), then peel digits from the least
 * significant level upwards, moving every digit >= B/2 to digit - B with a carry into the next level.
 * The carry out of the most significant level is dropped (it is a multiple of 2^64).
 * digits[j-1] holds d_j, j = 1 (weight 2^(64-beta)) .. l (weight 2^(64-beta*l)); d_j in [-B/2, B/2). */
void orc_decompose(uint64_t x, uint32_t beta, uint32_t l, int64_t *digits)
{
    uint32_t bits = beta * l;
    uint64_t v;
    if (bits >= 64) v = x;
    else            v = (x + ((uint64_t)1 << (63 - bits))) >> (64 - bits);
    uint64_t B = (uint64_t)1 << beta;
    for (int j = (int)l; j >= 1; j--) {
        uint64_t d = v & (B - 1);
        v >>= beta;
        int64_t sd = (int64_t)d;
        if (d >= (B >> 1)) { sd -= (int64_t)B; v += 1; }
        digits[j - 1] = sd;
    }
}

/* Modulus switch from 2^64 to 2N: round(x * 2N / 2^64) mod 2N, by add-half-then-shift (ties up). */
uint32_t orc_modswitch(uint64_t x, uint32_t N)
{
    uint32_t log2N2 = 0;
    while (((uint32_t)1 << log2N2) < 2 * N) log2N2++;
    uint32_t w = 64 - log2N2;
    uint64_t y = (x + ((uint64_t)1 << (w - 1))) >> w;   /* wrapping add: words near 2^64 map to 0 */
    return (uint32_t)(y & (2 * N - 1));
}

/* Lookup table f: Z_t -> Z_t (t = 2^msg_bits) to an accumulator body polynomial.
 * Each table entry fills a box of N/t coefficients scaled by Delta = 2^(63-msg_bits); the whole
 * polynomial is then rotated down by half a box so that the rounding of the modulus switch lands in
 * the middle of a box: V[j] = Delta*f((j+h) div box) when (j+h) div box < t, else -Delta*f(0). */
int orc_lut_encode(const oracle_params *p, const uint64_t *table, uint32_t n_tables, uint64_t *out)
{
    uint32_t t = (uint32_t)1 << p->msg_bits;
    if (p->N < 2 * t) return -1;
    uint32_t box = p->N / t, h = box / 2;
    uint64_t delta = (uint64_t)1 << (63 - p->msg_bits);
    for (uint32_t q = 0; q < n_tables; q++)
        for (uint32_t j = 0; j < p->N; j++) {
            uint32_t idx = (j + h) / box;
            uint64_t v = (idx < t) ? delta * table[(size_t)q * t + idx]
                                   : (uint64_t)0 - delta * table[(size_t)q * t];
            out[(size_t)q * p->N + j] = v;
        }
    return 0;
}

/* ---- encryption, decryption, key generation (inputs: key bits, mask words, noise integers) ---- */

/* LWE: b = sum a_i s_i + pt + e. `mask` has dim words, ct has dim+1. */
void orc_lwe_encrypt(const uint64_t *sk, uint32_t dim, const uint64_t *mask, int64_t noise,
                     uint64_t pt, uint64_t *ct)
{
    uint64_t b = pt + (uint64_t)noise;
    for (uint32_t i = 0; i < dim; i++) { ct[i] = mask[i]; b += mask[i] * sk[i]; }
    ct[dim] = b;
}

/* phase = b - sum a_i s_i */
uint64_t orc_lwe_phase(const uint64_t *sk, uint32_t dim, const uint64_t *ct)
{
    uint64_t ph = ct[dim];
    for (uint32_t i = 0; i < dim; i++) ph -= ct[i] * sk[i];
    return ph;
}

/* GLWE: B = sum_r A_r (*) S_r + M + E.  sk [k][N], mask [k][N], noise [N], M [N] -> ct [k+1][N]. */
void orc_glwe_encrypt(const uint64_t *sk, uint32_t k, uint32_t N, const uint64_t *mask,
                      const int64_t *noise, const uint64_t *M, uint64_t *ct)
{
    uint64_t *tmp = (uint64_t *)malloc((size_t)N * 8);
    uint64_t *B = ct + (size_t)k * N;
    for (uint32_t j = 0; j < N; j++) B[j] = M[j] + (uint64_t)noise[j];
    for (uint32_t r = 0; r < k; r++) {
        memcpy(ct + (size_t)r * N, mask + (size_t)r * N, (size_t)N * 8);
        orc_negacyclic_mul(mask + (size_t)r * N, sk + (size_t)r * N, N, tmp);
        for (uint32_t j = 0; j < N; j++) B[j] += tmp[j];
    }
    free(tmp);
}

/* GLWE phase polynomial: B - sum_r A_r (*) S_r */
void orc_glwe_phase(const uint64_t *sk, uint32_t k, uint32_t N, const uint64_t *ct, uint64_t *phase)
{
    uint64_t *tmp = (uint64_t *)malloc((size_t)N * 8);
    memcpy(phase, ct + (size_t)k * N, (size_t)N * 8);
    for (uint32_t r = 0; r < k; r++) {
        orc_negacyclic_mul(ct + (size_t)r * N, sk + (size_t)r * N, N, tmp);
        for (uint32_t j = 0; j < N; j++) phase[j] -= tmp[j];
    }
    free(tmp);
}

/* Bootstrapping key: for every LWE key bit s_i a GGSW ciphertext.  Row (r, j) is a GLWE encryption of
 * zero with s_i * 2^(64 - j*beta) added to the constant coefficient of component r (components
 * 0..k-1 are the mask polynomials, component k is the body).
 * mask [n][k+1][l][k][N], noise [n][k+1][l][N] -> bsk [n][k+1][l][k+1][N]. */
void orc_bsk_gen(const oracle_params *p, const uint64_t *lwe_sk, const uint64_t *glwe_sk,
                 const uint64_t *mask, const int64_t *noise, uint64_t *bsk)
{
    uint32_t k = p->k, N = p->N, l = p->pbs_level;
    long rows = (long)p->n * (k + 1) * l;
#pragma omp parallel for schedule(dynamic, 4)
    for (long row = 0; row < rows; row++) {
        uint32_t i = (uint32_t)(row / ((k + 1) * l));
        uint32_t r = (uint32_t)((row / l) % (k + 1));
        uint32_t j = (uint32_t)(row % l) + 1;
        uint64_t *zero = (uint64_t *)calloc(N, 8);
        uint64_t *ct = bsk + (size_t)row * (k + 1) * N;
        orc_glwe_encrypt(glwe_sk, k, N, mask + (size_t)row * k * N, noise + (size_t)row * N, zero, ct);
        ct[(size_t)r * N] += lwe_sk[i] << (64 - j * p->pbs_base_log);
        free(zero);
    }
}

/* Key-switching key from the extracted key s' (kN bits) to the small key s:
 * KSK[i][j] = LWE_s( s'_i * 2^(64 - j*beta_ks) ).  mask [kN][l_ks][n], noise [kN][l_ks]. */
void orc_ksk_gen(const oracle_params *p, const uint64_t *big_sk, const uint64_t *lwe_sk,
                 const uint64_t *mask, const int64_t *noise, uint64_t *ksk)
{
    uint32_t kN = p->k * p->N, l = p->ks_level, n = p->n;
    for (uint32_t i = 0; i < kN; i++)
        for (uint32_t j = 1; j <= l; j++) {
            size_t row = (size_t)i * l + (j - 1);
            uint64_t pt = big_sk[i] << (64 - j * p->ks_base_log);
            orc_lwe_encrypt(lwe_sk, n, mask + row * n, noise[row], pt, ksk + row * (n + 1));
        }
}

/* ---- bootstrapping --------------------------------------------------------------------------- */

/* One CMux of the blind rotation:  ACC <- ACC + BSK_i [.] (X^a * ACC - ACC), where [.] is the external
 * product: every component of the difference is gadget-decomposed coefficient by coefficient and each
 * digit polynomial (signed integers, two's complement in u64) multiplies the matching GGSW row. */
void orc_cmux(const oracle_params *p, uint64_t *acc, const uint64_t *bsk_i, uint32_t a_tilde)
{
    uint32_t k = p->k, N = p->N, l = p->pbs_level;
    size_t glwe = (size_t)(k + 1) * N;
    uint64_t *lam = (uint64_t *)malloc(glwe * 8);
    uint64_t *dig = (uint64_t *)malloc((size_t)l * N * 8);
    uint64_t *prod = (uint64_t *)malloc((size_t)N * 8);
    int64_t d[64];
    for (uint32_t r = 0; r <= k; r++) {
        orc_monomial_mul(acc + (size_t)r * N, N, a_tilde, lam + (size_t)r * N);
        for (uint32_t c = 0; c < N; c++) lam[(size_t)r * N + c] -= acc[(size_t)r * N + c];
    }
    for (uint32_t r = 0; r <= k; r++) {
        for (uint32_t c = 0; c < N; c++) {
            orc_decompose(lam[(size_t)r * N + c], p->pbs_base_log, l, d);
            for (uint32_t j = 0; j < l; j++) dig[(size_t)j * N + c] = (uint64_t)d[j];
        }
        for (uint32_t j = 0; j < l; j++) {
            const uint64_t *row = bsk_i + ((size_t)r * l + j) * glwe;
            for (uint32_t comp = 0; comp <= k; comp++) {
                orc_negacyclic_mul(dig + (size_t)j * N, row + (size_t)comp * N, N, prod);
                for (uint32_t c = 0; c < N; c++) acc[(size_t)comp * N + c] += prod[c];
            }
        }
    }
    free(lam); free(dig); free(prod);
}

/* Modulus switch + accumulator initialisation + the first n_steps CMuxes (n_steps = n is the full
 * blind rotation).  acc [k+1][N]:  ACC = (0,...,0, X^{-b~} V), then for i = 0,1,... in this order
 * ACC <- CMux(BSK_i, a~_i). */
void orc_blind_rotate(const oracle_params *p, const uint64_t *lwe_in, const uint64_t *lut,
                      const uint64_t *bsk, uint32_t n_steps, uint64_t *acc)
{
    uint32_t k = p->k, N = p->N;
    size_t glwe = (size_t)(k + 1) * N;
    memset(acc, 0, glwe * 8);
    uint32_t bt = orc_modswitch(lwe_in[p->n], N);
    orc_monomial_mul(lut, N, (2 * N - bt) % (2 * N), acc + (size_t)k * N);
    size_t ggsw = (size_t)(k + 1) * p->pbs_level * glwe;
    for (uint32_t i = 0; i < n_steps && i < p->n; i++)
        orc_cmux(p, acc, bsk + (size_t)i * ggsw, orc_modswitch(lwe_in[i], N));
}

/* Sample extraction of the constant coefficient: an LWE ciphertext of dimension kN under the
 * flattened GLWE key.  a'_{rN} = A_r[0], a'_{rN+j} = -A_r[N-j] (j >= 1), b' = B[0]. */
void orc_sample_extract(const oracle_params *p, const uint64_t *acc, uint64_t *lwe_out)
{
    uint32_t k = p->k, N = p->N;
    for (uint32_t r = 0; r < k; r++) {
        lwe_out[(size_t)r * N] = acc[(size_t)r * N];
        for (uint32_t j = 1; j < N; j++) lwe_out[(size_t)r * N + j] = (uint64_t)0 - acc[(size_t)r * N + N - j];
    }
    lwe_out[(size_t)k * N] = acc[(size_t)k * N];
}

/* Programmable bootstrapping of a batch.  lwe_in [batch][n+1]; luts [n_luts][N]; lut_idx [batch] or
 * NULL (all use LUT 0); lwe_out [batch][kN+1]. */
void orc_pbs_batch(const oracle_params *p, const uint64_t *lwe_in, const uint64_t *luts,
                   const uint32_t *lut_idx, const uint64_t *bsk, uint64_t *lwe_out, uint32_t batch)
{
    size_t glwe = (size_t)(p->k + 1) * p->N;
#pragma omp parallel for schedule(dynamic, 1)
    for (long c = 0; c < (long)batch; c++) {
        uint64_t *acc = (uint64_t *)malloc(glwe * 8);
        uint32_t li = lut_idx ? lut_idx[c] : 0;
        orc_blind_rotate(p, lwe_in + (size_t)c * (p->n + 1), luts + (size_t)li * p->N, bsk, p->n, acc);
        orc_sample_extract(p, acc, lwe_out + (size_t)c * (p->k * p->N + 1));
        free(acc);
    }
}

/* Same as orc_pbs_batch but stops after n_steps CMuxes and returns the accumulators [batch][k+1][N]. */
void orc_blind_rotate_batch(const oracle_params *p, const uint64_t *lwe_in, const uint64_t *luts,
                            const uint32_t *lut_idx, const uint64_t *bsk, uint32_t n_steps,
                            uint64_t *acc_out, uint32_t batch)
{
    size_t glwe = (size_t)(p->k + 1) * p->N;
#pragma omp parallel for schedule(dynamic, 1)
    for (long c = 0; c < (long)batch; c++) {
        uint32_t li = lut_idx ? lut_idx[c] : 0;
        orc_blind_rotate(p, lwe_in + (size_t)c * (p->n + 1), luts + (size_t)li * p->N, bsk, n_steps,
                         acc_out + (size_t)c * glwe);
    }
}

/* LWE key switching from dimension kN to n:
 * out = (0,...,0, b') - sum_i sum_j d_j(a'_i) * KSK[i][j], digits from orc_decompose(beta_ks, l_ks). */
void orc_keyswitch_batch(const oracle_params *p, const uint64_t *lwe_in, const uint64_t *ksk,
                         uint64_t *lwe_out, uint32_t batch)
{
    uint32_t kN = p->k * p->N, n = p->n, l = p->ks_level;
#pragma omp parallel for schedule(dynamic, 1)
    for (long c = 0; c < (long)batch; c++) {
        const uint64_t *in = lwe_in + (size_t)c * (kN + 1);
        uint64_t *out = lwe_out + (size_t)c * (n + 1);
        int64_t d[64];
        for (uint32_t x = 0; x < n; x++) out[x] = 0;
        out[n] = in[kN];
        for (uint32_t i = 0; i < kN; i++) {
            orc_decompose(in[i], p->ks_base_log, l, d);
            for (uint32_t j = 0; j < l; j++) {
                const uint64_t *row = ksk + ((size_t)i * l + j) * (n + 1);
                uint64_t dj = (uint64_t)d[j];
                for (uint32_t x = 0; x <= n; x++) out[x] -= dj * row[x];
            }
        }
    }
}

/* Integer linear combination of LWE ciphertexts with clear weights (the leveled sums in step 3 of the
 * paper's Matmul^RNS algorithm): out[g][o] = sum_j w[j][o] * ct[g][j], as vectors of `width` = n+1 words.
 * cts [G][J][width], w [J][O] (int32), out [G][O][width]. */
void orc_lwe_lincomb_batch(const uint64_t *cts, const int32_t *w, uint64_t *out, uint32_t G, uint32_t J,
                           uint32_t O, uint32_t width)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (long go = 0; go < (long)G * O; go++) {
        uint32_t g = (uint32_t)(go / O), o = (uint32_t)(go % O);
        uint64_t *dst = out + (size_t)go * width;
        for (uint32_t x = 0; x < width; x++) dst[x] = 0;
        for (uint32_t j = 0; j < J; j++) {
            uint64_t wj = (uint64_t)(int64_t)w[(size_t)j * O + o];
            const uint64_t *src = cts + ((size_t)g * J + j) * width;
            for (uint32_t x = 0; x < width; x++) dst[x] += wj * src[x];
        }
    }
}

/* Threads the OpenMP loops above will use (for reporting). */
#ifdef _OPENMP
#include <omp.h>
int orc_num_threads(void) { return omp_get_max_threads(); }
#else
int orc_num_threads(void) { return 1; }
#endif
