// LWE key switching as an int8 matrix-core contraction (gfx950 v_mfma_i32_32x32x32_i8).
//
// out[c][x] -= sum_rho d_rho(c) * KSK_rho[x] (mod 2^64) is a dense product of the digit matrix (ciphertexts x key rows,
// digits in [-B/2, B/2), one byte each when B <= 2^8) with the key matrix (key rows x output words).  A 64-bit key word w
// is recoded into eight signed bytes s_p in [-128, 128) with w = sum_p s_p 2^(8p) (mod 2^64): s_p is byte p of
// (w + 0x80..80) with its top bit flipped.  Each byte plane is one int8 x int8 -> int32 contraction; the eight plane sums
// are recombined with shifts at the end.  Products are at most 2^14 in magnitude, so an int32 accumulator is exact for
// fewer than 2^17 key rows; the host keeps every segment of the row index below that.
//
// Row order inside the contraction is level-major, rho = j * kN + i, so that 16 consecutive rows are 16 consecutive mask
// words at one level (kN must be a multiple of 32).
#include "slz_internal.h"
#include "slz_modarith.h"
#include "slz_mfma_i8.h"

#define KM_WAVES 8                      // waves per workgroup = 32-ciphertext tiles per workgroup
#define KM_THREADS (64 * KM_WAVES)
#define KM_IT_KB (KM_WAVES / 2)         // 32-row blocks per iteration: each thread brings in 8 rows of one output word
#define KM_TARGET_WGS 768               // workgroups aimed for when the row index is cut into segments (three per CU)
#define KM_BUF_V4 (KM_IT_KB * 2 * 8 * 32)   // 16-byte slots per LDS buffer: [block][half][plane][x]

// ---- digits --------------------------------------------------------------------------------------------------------
// dig[tile][kb][lane] (16 bytes): the A operand of lane `lane` for 32-row block kb of 32-ciphertext tile `tile`:
// ciphertext 32 tile + lane % 32, rows 32 kb + 16 (lane / 32) + t for byte t.  Ciphertexts past the batch get zero digits.
// Signed digits without a carry chain: with H = sum_j (B/2) B^(l-j), digit j of v is ((v + H) >> beta (l-j)) mod B - B/2.
// A workgroup takes 32 ciphertexts x 128 mask words: every wave reads whole 512-byte runs of a ciphertext, the digit bytes
// are turned through LDS (rows of 128 + 16 bytes: the 16-byte reads of 8 neighbouring lanes then cover all banks), and
// every store instruction writes one 1 KiB operand block.
#define KD_WORDS 128
#define KD_PITCH (KD_WORDS + 16)
#define KD_LEVELS 8                     // levels turned through LDS at a time
__global__ void __launch_bounds__(256)
k_ksm_digits(const uint64_t *__restrict__ lwe_in, v4i *__restrict__ dig, uint32_t kN, uint32_t beta, uint32_t l, uint32_t batch,
             uint32_t n_kb) {
    __shared__ __attribute__((aligned(16))) unsigned char L[KD_LEVELS * 32 * KD_PITCH];
    const uint32_t lane = threadIdx.x % 64, wave = threadIdx.x / 64;
    const uint32_t w0 = blockIdx.x * KD_WORDS, tile = blockIdx.y;
    const uint32_t n_blk = min((kN - w0) / 32u, (uint32_t)KD_WORDS / 32u);    // 32-word blocks of this workgroup (kN % 32 == 0)
    const uint32_t bits = beta * l;
    const uint32_t half_b = 1u << (beta - 1);
    uint64_t H = 0;
    for (uint32_t j = 0; j < l; j++) H |= (uint64_t)half_b << (beta * j);
    // wave `wave` reads ciphertexts 8 wave .. 8 wave + 7 of the tile, lane words w0 + lane and w0 + 64 + lane
    uint64_t v[8][2];
#pragma unroll
    for (int q = 0; q < 8; q++) {
        const uint32_t c = tile * 32 + 8 * wave + q;
#pragma unroll
        for (int h = 0; h < 2; h++) {
            const uint32_t w = w0 + 64 * h + lane;
            const uint64_t a = (c < batch && w < kN) ? lwe_in[(size_t)c * (kN + 1) + w] : 0ull;
            v[q][h] = slz_round_top_bits(a, bits) + H;
        }
    }
    for (uint32_t j0 = 0; j0 < l; j0 += KD_LEVELS) {
        const uint32_t nj = min(l - j0, (uint32_t)KD_LEVELS);
        if (j0) __syncthreads();                                    // the previous group has been read
        for (uint32_t jj = 0; jj < nj; jj++) {                     // level j0 + jj + 1, most significant first
            const uint32_t sh = beta * (l - 1 - (j0 + jj));
#pragma unroll
            for (int q = 0; q < 8; q++)
#pragma unroll
                for (int h = 0; h < 2; h++) {
                    const uint32_t u = (uint32_t)(v[q][h] >> sh) & (2 * half_b - 1);
                    L[(jj * 32 + 8 * wave + q) * KD_PITCH + 64 * h + lane] = (unsigned char)(u - half_b);
                }
        }
        __syncthreads();
        // operand blocks (level, 32-word block) of this group, dealt to the waves; lane = ciphertext + 32 half
        for (uint32_t ob = wave; ob < nj * n_blk; ob += 4) {
            const uint32_t jj = ob / n_blk, kbl = ob % n_blk;
            const v4i o = *reinterpret_cast<const v4i *>(&L[(jj * 32 + lane % 32) * KD_PITCH + 32 * kbl + 16 * (lane / 32)]);
            const uint32_t kb = ((j0 + jj) * kN + w0) / 32 + kbl;
            dig[((size_t)tile * n_kb + kb) * 64 + lane] = o;
        }
    }
}

// ---- key in operand form ----------------------------------------------------------------------------------------------
// The contraction's B operands, ready to be copied into LDS: P[x tile][block kb][half][plane p][x in tile] (16 bytes):
// byte t = signed byte p of the key word of row 32 kb + 16 half + t, output word 32 (x tile) + x.  Words past n and
// blocks past the last row (the block count is padded to a multiple of 2 KM_IT_KB) are zero.  One iteration of a
// workgroup (KM_IT_KB blocks of one x tile) is KM_BUF_V4 consecutive entries, in the order of its LDS buffer.
#define KM_KB_PAD (2 * KM_IT_KB)
__host__ __device__ static inline uint32_t ksm_padded_blocks(uint32_t n_kb) { return (n_kb + KM_KB_PAD - 1) / KM_KB_PAD * KM_KB_PAD; }

__global__ void __launch_bounds__(256)
k_ksk_prepare(const uint64_t *__restrict__ ksk, v4i *__restrict__ out, uint32_t kN, uint32_t n, uint32_t l, uint32_t n_kb,
              uint32_t n_kb_pad, uint32_t x_tiles) {
    const uint32_t xl = threadIdx.x % 32, half = (threadIdx.x / 32) % 2;
    const uint32_t kb = blockIdx.x * 4 + threadIdx.x / 64, xt = blockIdx.y;
    if (kb >= n_kb_pad) return;
    const uint32_t x = xt * 32 + xl, width = n + 1;
    uint64_t w[16];
#pragma unroll
    for (int t = 0; t < 16; t++) {
        const uint32_t rho = 32 * kb + 16 * half + t;             // level-major row: rho = j kN + i
        const uint32_t j = rho / kN, i = rho % kN;
        w[t] = (kb < n_kb && x < width) ? slz_signed_bytes(ksk[((size_t)i * l + j) * width + x]) : 0ull;
    }
    uint64_t lo[8], hi[8], pl[8], ph[8];
#pragma unroll
    for (int t = 0; t < 8; t++) { lo[t] = w[t]; hi[t] = w[8 + t]; }
    slz_byte_planes(lo, pl);
    slz_byte_planes(hi, ph);
    v4i *dst = out + (((size_t)xt * n_kb_pad + kb) * 2 + half) * 8 * 32 + xl;
#pragma unroll
    for (int p = 0; p < 8; p++) {
        v4i o = {(int)(uint32_t)pl[p], (int)(uint32_t)(pl[p] >> 32), (int)(uint32_t)ph[p], (int)(uint32_t)(ph[p] >> 32)};
        dst[p * 32] = o;
    }
}

// ---- contraction ---------------------------------------------------------------------------------------------------
struct ksm_args {
    const uint64_t *ksk;
    const v4i *kskp;        // prepared key (k_ksk_prepare) or null
    const v4i *dig;
    const uint64_t *lwe_in; // this chunk's input ciphertexts (for the bodies when direct)
    uint64_t *out;
    uint32_t direct;        // one segment: a workgroup owns its output words and stores (0, b') - sum itself; otherwise
                            // `out` already holds (0, b') and the segments are combined with atomics
    uint32_t kN, n, l, batch;
    uint32_t n_tiles;       // 32-ciphertext tiles in dig
    uint32_t n_kb;          // 32-row blocks in total (l kN / 32)
    uint32_t kb_per_seg;    // multiple of 2 KM_IT_KB
    uint32_t x_tiles, ct_groups, total;   // work items: (segment, x tile, ciphertext group), group fastest
    uint32_t per_xcd;
};

// PREP: the key comes in operand form (A.kskp) and goes from global memory to LDS as it is; otherwise every thread recodes
// eight words of the standard key per iteration.
template <bool PREP>
__global__ void __launch_bounds__(KM_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2)))
k_ksm_main(ksm_args A) {
    __shared__ v4i lds[2 * KM_BUF_V4];                              // 64 KiB
    // work items are dealt so that one XCD (workgroups b, b+8, ...) walks a contiguous range: the workgroups resident on
    // it share a segment of the key and neighbouring output words, which its L2 then serves
    const uint32_t item = (blockIdx.x % 8) * A.per_xcd + blockIdx.x / 8;
    if (blockIdx.x / 8 >= A.per_xcd || item >= A.total) return;
    // inside a segment the order is (block of 8 ciphertext groups, x tile, group in the block): the 64 workgroups resident on
    // an XCD are then about 8 groups x 8 x tiles, and its L2 sees each of their digit and key streams once instead of the
    // digits of 64 groups against one x tile (the digit operands are the larger stream)
    const uint32_t per_seg = A.ct_groups * A.x_tiles;
    const uint32_t seg = item / per_seg, r = item % per_seg;
    const uint32_t n_full = A.ct_groups / 8, blk = 8 * A.x_tiles;
    uint32_t cg, xt;
    if (r < n_full * blk) {
        cg = (r / blk) * 8 + r % 8;
        xt = (r % blk) / 8;
    } else {                                                        // the last, narrower block
        const uint32_t rr = r - n_full * blk, w = A.ct_groups - n_full * 8;
        cg = n_full * 8 + rr % w;
        xt = rr / w;
    }
    const uint32_t lane = threadIdx.x % 64;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
    const uint32_t tile = cg * KM_WAVES + wave;
    const bool tile_ok = tile < A.n_tiles;
    const uint32_t kb_begin = seg * A.kb_per_seg;
    const uint32_t kb_end = min(A.n_kb, kb_begin + A.kb_per_seg);
    const uint32_t width = A.n + 1;

    // key-loading role: output word x, rows 8 oct .. 8 oct + 7 of the iteration's 32 KM_IT_KB rows
    const uint32_t xl = lane % 32;
    const uint32_t x = xt * 32 + xl;
    const uint32_t oct = 2 * wave + lane / 32;
    const bool x_ok = x < width;
    const size_t row_stride = (size_t)A.l * width;                  // words between consecutive mask indices at one level
    // level j and mask index i of this thread's first row; both advance by 32 KM_IT_KB rows per iteration
    uint32_t rho = kb_begin * 32 + 8 * oct;
    uint32_t j = rho / A.kN, i = rho % A.kN;
    const uint32_t lds_w = ((((oct / 4) * 2 + (oct / 2) % 2) * 8) * 32 + xl) * 2 + (oct & 1);   // in 8-byte units, plane 0

    // Two register stages of key words and digit operands: what iteration t consumes was requested during iteration t-2,
    // so a load has two iterations of MFMAs to arrive.  Loads are unconditional (rows or words out of range read a valid
    // address and are replaced by zero when consumed), which keeps the wait counts static.
    uint64_t kw0[8], kw1[8];
    bool ok0, ok1;
    v4i an0[KM_IT_KB], an1[KM_IT_KB];
    // operand form: the iteration's KM_BUF_V4 entries are consecutive; a thread moves entries tid + KM_THREADS u (the same
    // eight registers hold them as four 16-byte values)
    const uint32_t kb_pad = ksm_padded_blocks(A.n_kb);
    const v4i *pkey = PREP ? A.kskp + (size_t)xt * kb_pad * (2 * 8 * 32) + threadIdx.x : nullptr;
    auto load_key = [&](uint64_t (&kw)[8], bool &ok, uint32_t it) {
        if (PREP) {
            // blocks up to the padded count exist (zero past the last row); past that the read is clamped and unused
            const uint32_t itc = min(it, kb_pad - KM_IT_KB);
            const v4i *src = pkey + (size_t)itc * (2 * 8 * 32);
#pragma unroll
            for (int u = 0; u < 4; u++) {
                const v4i v = src[u * KM_THREADS];
                kw[2 * u] = (uint64_t)(uint32_t)v[0] | ((uint64_t)(uint32_t)v[1] << 32);
                kw[2 * u + 1] = (uint64_t)(uint32_t)v[2] | ((uint64_t)(uint32_t)v[3] << 32);
            }
            ok = true;
            return;
        }
        ok = x_ok && (it + oct / 4 < kb_end);
        const uint64_t *src = A.ksk + (ok ? ((size_t)i * A.l + j) * width + x : (size_t)0);
#pragma unroll
        for (int t = 0; t < 8; t++) kw[t] = src[(size_t)t * row_stride];
        i += 32 * KM_IT_KB;
        while (i >= A.kN) { i -= A.kN; j++; }
    };
    const size_t dig_base = (size_t)(tile_ok ? tile : 0) * A.n_kb;
    auto load_dig = [&](v4i (&an)[KM_IT_KB], uint32_t it) {
        // blocks past the end of the segment meet zero key bytes, so their digits need no masking
#pragma unroll
        for (int q = 0; q < KM_IT_KB; q++) an[q] = A.dig[(dig_base + min(it + q, A.n_kb - 1)) * 64 + lane];
    };

    v16i acc[8];
#pragma unroll
    for (int p = 0; p < 8; p++)
#pragma unroll
        for (int r = 0; r < 16; r++) acc[p][r] = 0;

    uint32_t buf = 0;
    auto body = [&](uint64_t (&kw)[8], bool &ok, v4i (&an)[KM_IT_KB], uint32_t it) {
        // recode to signed bytes, transpose 8 rows x 8 planes, park the plane operands in LDS
        if (PREP) {
            uint64_t *dst = reinterpret_cast<uint64_t *>(lds + buf * KM_BUF_V4 + threadIdx.x);
#pragma unroll
            for (int u = 0; u < 4; u++) {
                dst[u * KM_THREADS * 2] = kw[2 * u];
                dst[u * KM_THREADS * 2 + 1] = kw[2 * u + 1];
            }
        } else {
            uint64_t w[8], plane[8];
#pragma unroll
            for (int t = 0; t < 8; t++) w[t] = ok ? slz_signed_bytes(kw[t]) : 0ull;
            slz_byte_planes(w, plane);
            uint64_t *dst = reinterpret_cast<uint64_t *>(lds + buf * KM_BUF_V4) + lds_w;
#pragma unroll
            for (int p = 0; p < 8; p++) dst[(size_t)p * 64] = plane[p];
        }
        load_key(kw, ok, it + 2 * KM_IT_KB);
        __syncthreads();
        // one barrier per iteration is enough with two buffers: a wave reaches the barrier of iteration t only after it
        // has read everything of iteration t-1, and buffer (t+1)%2 is not written before that barrier
        if (tile_ok) {
            // the plane operands of the next half block are read from LDS while four MFMAs run
            const v4i *src = lds + buf * KM_BUF_V4 + (lane / 32) * (8 * 32) + xl;
            v4i bb[2][4];
#pragma unroll
            for (int p = 0; p < 4; p++) bb[0][p] = src[p * 32];
#pragma unroll
            for (int g = 0; g < 2 * KM_IT_KB; g++) {               // half block g: block g/2, planes 4 (g%2) .. +3
                if (g + 1 < 2 * KM_IT_KB) {
#pragma unroll
                    for (int p = 0; p < 4; p++) bb[(g + 1) & 1][p] = src[(((g + 1) / 2) * 2 * 8 + 4 * ((g + 1) % 2) + p) * 32];
                }
                __builtin_amdgcn_sched_barrier(0);      // keep the reads above the MFMAs they overlap with
#pragma unroll
                for (int p = 0; p < 4; p++)
                    acc[4 * (g % 2) + p] = __builtin_amdgcn_mfma_i32_32x32x32_i8(an[g / 2], bb[g & 1][p], acc[4 * (g % 2) + p], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        load_dig(an, it + 2 * KM_IT_KB);
        buf ^= 1;
    };
    load_key(kw0, ok0, kb_begin);
    load_dig(an0, kb_begin);
    load_key(kw1, ok1, kb_begin + KM_IT_KB);
    load_dig(an1, kb_begin + KM_IT_KB);
    for (uint32_t it = kb_begin; it < kb_end; it += 2 * KM_IT_KB) {  // kb_per_seg is a multiple of 2 KM_IT_KB
        body(kw0, ok0, an0, it);
        body(kw1, ok1, an1, it + KM_IT_KB);
    }
    if (!tile_ok || !x_ok) return;
    // accumulator register r of a lane is ciphertext 8 (r / 4) + 4 (lane / 32) + r % 4 of the tile, output word x
#pragma unroll
    for (int r = 0; r < 16; r++) {
        const uint32_t c = tile * 32 + 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
        if (c < A.batch) {
            uint64_t val = 0;
#pragma unroll
            for (int p = 0; p < 8; p++) val += (uint64_t)(int64_t)acc[p][r] << (8 * p);
            if (A.direct) {
                const uint64_t base = x == A.n ? A.lwe_in[(size_t)c * (A.kN + 1) + A.kN] : 0ull;
                A.out[(size_t)c * width + x] = base - val;
            } else {
                atomicAdd((unsigned long long *)&A.out[(size_t)c * width + x], (unsigned long long)(0 - val));
            }
        }
    }
}

int slz_ksm_supported(const slz_params *p) {
    return p->ks_base_log <= 8 && ((uint64_t)p->k * p->N) % 32 == 0;
}

void slz_ksm_destroy(slz_ctx *ctx) {
    if (ctx->ks_dig) (void)hipFree(ctx->ks_dig);
    ctx->ks_dig = nullptr;
}

// The launches of one keyswitch given its digit scratch (`dig`: room for max_tiles 32-ciphertext tiles).
static int ksm_run(const slz_params &p, void *dig, uint32_t max_tiles, const uint64_t *lwe_in, const uint64_t *ksk, const void *kskp,
                   uint64_t *lwe_out, uint32_t batch, hipStream_t s) {
    const uint32_t kN = p.k * p.N;
    const uint32_t n_kb = (uint32_t)((uint64_t)p.ks_level * kN / 32);
    ksm_args A;
    A.ksk = ksk;
    A.kskp = (const v4i *)kskp;
    A.dig = (const v4i *)dig;
    A.kN = kN; A.n = p.n; A.l = p.ks_level;
    A.n_kb = n_kb;
    A.x_tiles = (p.n + 1 + 31) / 32;
    // int32 accumulators: 32 kb_per_seg rows of |digit * byte| <= 2^(beta-1) * 2^7 must stay strictly below 2^31
    const uint32_t kb_cap = (1u << (20 - p.ks_base_log)) - 2 * KM_IT_KB;
    for (uint32_t c0 = 0; c0 < batch; c0 += max_tiles * 32) {
        const uint32_t nb = min(batch - c0, max_tiles * 32);
        A.batch = nb;
        A.n_tiles = (nb + 31) / 32;
        A.ct_groups = (A.n_tiles + KM_WAVES - 1) / KM_WAVES;
        A.out = lwe_out + (size_t)c0 * (p.n + 1);
        // segments of the row index: enough workgroups for three rounds over the 256 CUs (a workgroup spends about half
        // its time outside the MFMA loop at cfg2's ten iterations, so fewer, longer segments with idle CUs measured no better)
        uint32_t segs = (KM_TARGET_WGS + A.x_tiles * A.ct_groups - 1) / (A.x_tiles * A.ct_groups);
        segs = max(1u, min(segs, (n_kb + 7) / 8));
        uint32_t kbs = ((n_kb + segs - 1) / segs + 2 * KM_IT_KB - 1) / (2 * KM_IT_KB) * (2 * KM_IT_KB);
        kbs = min(kbs, kb_cap);
        segs = (n_kb + kbs - 1) / kbs;
        A.kb_per_seg = kbs;
        const uint64_t total = (uint64_t)segs * A.x_tiles * A.ct_groups;
        if (total > (1u << 30)) return SLZ_E_UNSUPPORTED;
        A.total = (uint32_t)total;
        A.per_xcd = (A.total + 7) / 8;
        A.lwe_in = lwe_in + (size_t)c0 * (kN + 1);
        A.direct = segs == 1;
        if (!A.direct) slz_ks_init_launch(A.lwe_in, A.out, kN, p.n, nb, s);
        hipLaunchKernelGGL(k_ksm_digits, dim3((kN + KD_WORDS - 1) / KD_WORDS, A.n_tiles), dim3(256), 0, s,
                           lwe_in + (size_t)c0 * (kN + 1), (v4i *)dig, kN, p.ks_base_log, p.ks_level, nb, n_kb);
        if (kskp) hipLaunchKernelGGL(k_ksm_main<true>, dim3(A.per_xcd * 8), dim3(KM_THREADS), 0, s, A);
        else hipLaunchKernelGGL(k_ksm_main<false>, dim3(A.per_xcd * 8), dim3(KM_THREADS), 0, s, A);
    }
    SLZ_HIP(hipGetLastError());
    return SLZ_OK;
}

// Size of the key in operand form, 0 when the parameter set does not use the matrix cores.
size_t slz_ksm_prepared_bytes(const slz_params *p) {
    if (!slz_ksm_supported(p)) return 0;
    const uint64_t n_kb64 = (uint64_t)p->ks_level * p->k * p->N / 32;
    if (n_kb64 > (1u << 26)) return 0;
    const size_t x_tiles = (p->n + 1 + 31) / 32;
    return x_tiles * ksm_padded_blocks((uint32_t)n_kb64) * (2 * 8 * 32) * sizeof(v4i);
}

int slz_ksm_prepare(slz_ctx *ctx, const uint64_t *ksk, void *dst, hipStream_t s) {
    const slz_params &p = ctx->prm;
    const uint32_t kN = p.k * p.N, n_kb = (uint32_t)((uint64_t)p.ks_level * kN / 32), n_kb_pad = ksm_padded_blocks(n_kb);
    const uint32_t x_tiles = (p.n + 1 + 31) / 32;
    hipLaunchKernelGGL(k_ksk_prepare, dim3((n_kb_pad + 3) / 4, x_tiles), dim3(256), 0, s, ksk, (v4i *)dst, kN, p.n, p.ks_level, n_kb,
                       n_kb_pad, x_tiles);
    SLZ_HIP(hipGetLastError());
    return SLZ_OK;
}

// Exactly one of ksk (standard form) and kskp (operand form) is given.  Writes every word of lwe_out.
int slz_ksm_launch(slz_ctx *ctx, const uint64_t *lwe_in, const uint64_t *ksk, const void *kskp, uint64_t *lwe_out, uint32_t batch,
                   hipStream_t s) {
    const slz_params &p = ctx->prm;
    const uint64_t n_kb64 = (uint64_t)p.ks_level * p.k * p.N / 32;
    if (n_kb64 > (1u << 26)) return SLZ_E_UNSUPPORTED;
    const uint32_t max_tiles = min((ctx->max_batch + 31) / 32, 32768u);
    if (!ctx->ks_dig) {     // digit scratch, sized for max_batch (larger batches go through in chunks)
        if (slz_scratch_alloc(&ctx->ks_dig, (size_t)max_tiles * n_kb64 * 1024) != SLZ_OK) return SLZ_E_NOMEM;
    }
    return ksm_run(p, ctx->ks_dig, max_tiles, lwe_in, ksk, kskp, lwe_out, batch, s);
}

// ---- the variant that allocates nothing ------------------------------------------------------------------------------
// Digit scratch for callers that cannot allocate: a file-scope device array (every device the library runs on holds its
// own copy until the process ends).  Host code never passes the array's name to a kernel: the device address is looked
// up once per device and kept in scratch_ptr.
#define SLZ_KS_STATIC_MAX_DEVICES 64
static __device__ __align__(256) unsigned char scratch[SLZ_KS_STATIC_SCRATCH_BYTES];
static void *scratch_ptr[SLZ_KS_STATIC_MAX_DEVICES];

extern "C" int slz_keyswitch_batch_static(slz_ctx *ctx, const uint64_t *lwe_in_dev, const uint64_t *ksk_dev, uint64_t *lwe_out_dev,
                                          uint32_t batch, void *hip_stream) {
    if (!ctx || !lwe_in_dev || !ksk_dev || !lwe_out_dev || batch == 0) return SLZ_E_INVALID_ARG;
    if (((uintptr_t)lwe_in_dev & 7u) || ((uintptr_t)ksk_dev & 15u) || ((uintptr_t)lwe_out_dev & 7u)) return SLZ_E_INVALID_ARG;
    const slz_params &p = ctx->prm;
    if (!slz_ksm_supported(&p)) return SLZ_E_UNSUPPORTED;
    const uint64_t n_kb64 = (uint64_t)p.ks_level * p.k * p.N / 32;
    if (n_kb64 > (1u << 26)) return SLZ_E_UNSUPPORTED;
    const uint64_t tiles = ((uint64_t)batch + 31) / 32;
    if (tiles * n_kb64 * 1024 > (uint64_t)SLZ_KS_STATIC_SCRATCH_BYTES) return SLZ_E_TOO_LARGE;
    int dev = -1;
    SLZ_HIP(hipGetDevice(&dev));
    if (dev != ctx->device || dev < 0 || dev >= SLZ_KS_STATIC_MAX_DEVICES) return SLZ_E_INVALID_ARG;
    if (!scratch_ptr[dev]) {
        void *ptr = nullptr;
        SLZ_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return SLZ_E_HIP;
        scratch_ptr[dev] = ptr;
    }
    hipStream_t s = (hipStream_t)hip_stream;
    // every digit slot of the tiles in use is rewritten by k_ksm_digits (ciphertexts past the batch get zeros), so the
    // contents the previous call left behind are never read
    return ksm_run(p, scratch_ptr[dev], (uint32_t)tiles, lwe_in_dev, ksk_dev, nullptr, lwe_out_dev, batch, s);
}
