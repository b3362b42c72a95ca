// LWE key switching and the clear-weight linear combination of LWE ciphertexts.
// Both are wrapping u64 integer contractions streamed from HBM; the order of summation is free.
#include "slz_internal.h"
#include "slz_modarith.h"

#define KS_THREADS 128
#define KS_TB 8            // ciphertexts per workgroup (each key word is reused KS_TB times from a register)
#define KS_IC 16           // mask words decomposed per LDS refill
#define KS_MAX_L 16
#define KS_MFMA_MIN_BATCH 16

__global__ void __launch_bounds__(KS_THREADS)
k_ks_init(const uint64_t *__restrict__ lwe_in, uint64_t *__restrict__ out, uint32_t kN, uint32_t n, uint32_t batch) {
    size_t gid = (size_t)blockIdx.x * KS_THREADS + threadIdx.x;
    if (gid >= (size_t)batch * (n + 1)) return;
    uint32_t x = (uint32_t)(gid % (n + 1));
    size_t c = gid / (n + 1);
    out[gid] = (x == n) ? lwe_in[c * (kN + 1) + kN] : 0ull;
}

// out[c][x] -= sum_{i in segment} sum_j d_j(a'_{c,i}) * KSK[i][j][x]
// grid: (x tiles, ciphertext tiles, segments of the mask index).
// The signed digit d in [-B/2, B/2) is held as u = d + B/2 >= 0, so that a product with a 64-bit key word is two
// 32x32+64 multiply-adds (low and high half of the word, separate 64-bit accumulators):
//   sum d w = sum u w - (B/2) sum w,   sum u w = accL + 2^32 accH  (mod 2^64).
__global__ void __launch_bounds__(KS_THREADS)
k_keyswitch(const uint64_t *__restrict__ lwe_in, const uint64_t *__restrict__ ksk, uint64_t *__restrict__ out, uint32_t kN,
            uint32_t n, uint32_t beta, uint32_t l, uint32_t batch, uint32_t seg_len) {
    __shared__ __attribute__((aligned(16))) uint32_t dig[KS_IC * KS_MAX_L * KS_TB];      // [ii][j][c]
    const uint32_t x = blockIdx.x * KS_THREADS + threadIdx.x;
    const uint32_t c0 = blockIdx.y * KS_TB;
    const uint32_t i_begin = blockIdx.z * seg_len;
    const uint32_t i_end = min(kN, i_begin + seg_len);
    const bool active = x <= n;
    const uint32_t half_b = 1u << (beta - 1);
    uint64_t accL[KS_TB], accH[KS_TB], sumw = 0;
#pragma unroll
    for (int c = 0; c < KS_TB; c++) { accL[c] = 0; accH[c] = 0; }
    for (uint32_t ib = i_begin; ib < i_end; ib += KS_IC) {
        __syncthreads();
        {   // decompose KS_TB x KS_IC mask words, one per thread; words past the end give u = B/2 (digit 0)
            uint32_t c = threadIdx.x / KS_IC, ii = threadIdx.x % KS_IC;
            uint32_t i = ib + ii;
            uint64_t v = 0;
            if (c0 + c < batch && i < i_end) v = slz_round_top_bits(lwe_in[(size_t)(c0 + c) * (kN + 1) + i], beta * l);
            for (int j = (int)l - 1; j >= 0; j--) dig[(ii * l + j) * KS_TB + c] = (uint32_t)(slz_next_digit(v, beta) + (int32_t)half_b);
        }
        __syncthreads();
        if (active) {
            const uint32_t cnt = min((uint32_t)KS_IC, i_end - ib) * l;
            const uint64_t *row = ksk + ((size_t)ib * l) * (n + 1) + x;
            // key words are requested four rows ahead of the multiply-adds that use them
            uint64_t wq[4];
#pragma unroll
            for (int u = 0; u < 4; u++) wq[u] = (uint32_t)u < cnt ? row[(size_t)u * (n + 1)] : 0ull;
            for (uint32_t r0 = 0; r0 < cnt; r0 += 4) {
                uint64_t wc[4];
#pragma unroll
                for (int u = 0; u < 4; u++) wc[u] = wq[u];
#pragma unroll
                for (int u = 0; u < 4; u++) wq[u] = (r0 + 4 + u < cnt) ? row[(size_t)(r0 + 4 + u) * (n + 1)] : 0ull;
#pragma unroll
                for (int u = 0; u < 4; u++) {
                    const uint32_t r = r0 + u;
                    if (r < cnt) {
                        const uint64_t w = wc[u];
                        const uint32_t wl = (uint32_t)w, wh = (uint32_t)(w >> 32);
                        const uint4 d0 = *reinterpret_cast<const uint4 *>(&dig[r * KS_TB]);
                        const uint4 d1 = *reinterpret_cast<const uint4 *>(&dig[r * KS_TB + 4]);
                        const uint32_t u8[KS_TB] = {d0.x, d0.y, d0.z, d0.w, d1.x, d1.y, d1.z, d1.w};
                        sumw += w;
#pragma unroll
                        for (int c = 0; c < KS_TB; c++) {
                            accL[c] += (uint64_t)u8[c] * wl;
                            accH[c] += (uint64_t)u8[c] * wh;
                        }
                    }
                }
            }
        }
    }
    if (active) {
        const uint64_t corr = sumw * (uint64_t)half_b;
#pragma unroll
        for (int c = 0; c < KS_TB; c++)
            if (c0 + c < batch) {
                const uint64_t delta = corr - (accL[c] + (accH[c] << 32));
                atomicAdd((unsigned long long *)&out[(size_t)(c0 + c) * (n + 1) + x], (unsigned long long)delta);
            }
    }
}

void slz_ks_init_launch(const uint64_t *lwe_in, uint64_t *lwe_out, uint32_t kN, uint32_t n, uint32_t batch, hipStream_t s) {
    const size_t total = (size_t)batch * (n + 1);
    hipLaunchKernelGGL(k_ks_init, dim3((unsigned)((total + KS_THREADS - 1) / KS_THREADS)), dim3(KS_THREADS), 0, s, lwe_in, lwe_out,
                       kN, n, batch);
}

int slz_keyswitch_launch(slz_ctx *ctx, const uint64_t *lwe_in, const uint64_t *ksk, uint64_t *lwe_out, uint32_t batch,
                         hipStream_t s) {
    const slz_params &p = ctx->prm;
    const uint32_t kN = p.k * p.N, n = p.n;
    if (p.ks_level > KS_MAX_L || p.ks_base_log > 31) return SLZ_E_UNSUPPORTED;
    static_assert(KS_THREADS == KS_TB * KS_IC, "one mask word per thread in the decomposition step");
    // digits of at most a byte: int8 MFMA contraction.  Measured faster than the scalar kernel below at every batch size,
    // one ciphertext included, except for a handful of ciphertexts against a key of HBM-streaming size (1.3 GB at
    // n = 1024, N = 32768: 0.33 ms against 0.27 ms), where the scalar kernel's plain row streaming wins.
    const size_t key_bytes = (size_t)kN * p.ks_level * (n + 1) * 8;
    if (!ctx->force_generic && (batch >= KS_MFMA_MIN_BATCH || key_bytes < ((size_t)512 << 20)) && slz_ksm_supported(&p)) {
        int rc = slz_ksm_launch(ctx, lwe_in, ksk, nullptr, lwe_out, batch, s);
        if (rc != SLZ_E_UNSUPPORTED) return rc;
    }
    slz_ks_init_launch(lwe_in, lwe_out, kN, n, batch, s);
    uint32_t xt = (n + 1 + KS_THREADS - 1) / KS_THREADS, ct = (batch + KS_TB - 1) / KS_TB;
    // enough segments of the mask index to give the 256 CUs several workgroups each
    uint32_t segs = 1;
    while ((size_t)xt * ct * segs < 4096 && segs < kN / (4 * KS_IC)) segs *= 2;
    uint32_t seg_len = ((kN + segs - 1) / segs + KS_IC - 1) / KS_IC * KS_IC;
    segs = (kN + seg_len - 1) / seg_len;
    if (ct > 65535 || segs > 65535) return SLZ_E_UNSUPPORTED;
    hipLaunchKernelGGL(k_keyswitch, dim3(xt, ct, segs), dim3(KS_THREADS), 0, s, lwe_in, ksk, lwe_out, kN, n, p.ks_base_log,
                       p.ks_level, batch, seg_len);
    SLZ_HIP(hipGetLastError());
    return SLZ_OK;
}

// ---- out[g][o][x] = sum_j w[j][o] * ct[g][j][x] ----------------------------------------------
#define LC_OT 16
__global__ void __launch_bounds__(KS_THREADS)
k_lincomb(const uint64_t *__restrict__ cts, const int32_t *__restrict__ w, uint64_t *__restrict__ out, uint32_t J, uint32_t O,
          uint32_t width) {
    const uint32_t x = blockIdx.x * KS_THREADS + threadIdx.x;
    const uint32_t o0 = blockIdx.y * LC_OT;
    const uint32_t g = blockIdx.z;
    if (x >= width) return;
    uint64_t acc[LC_OT];
#pragma unroll
    for (int o = 0; o < LC_OT; o++) acc[o] = 0;
    const uint64_t *src = cts + (size_t)g * J * width + x;
    for (uint32_t j = 0; j < J; j++) {
        uint64_t c = src[(size_t)j * width];
        const int32_t *wr = w + (size_t)j * O + o0;
#pragma unroll
        for (int o = 0; o < LC_OT; o++)
            if (o0 + o < O) acc[o] += (uint64_t)(int64_t)wr[o] * c;
    }
#pragma unroll
    for (int o = 0; o < LC_OT; o++)
        if (o0 + o < O) out[((size_t)g * O + o0 + o) * width + x] = acc[o];
}

int slz_lincomb_launch(slz_ctx *ctx, const uint64_t *cts, const int32_t *w, uint64_t *out, uint32_t G, uint32_t J, uint32_t O,
                       hipStream_t s) {
    const uint32_t width = ctx->prm.n + 1;
    if (!ctx->force_generic) {      // int8 MFMA contraction; shapes it does not take fall through to the scalar kernel
        int rc = slz_lcm_launch(ctx, cts, w, out, G, J, O, s);
        if (rc != SLZ_E_UNSUPPORTED) return rc;
    }
    hipLaunchKernelGGL(k_lincomb, dim3((width + KS_THREADS - 1) / KS_THREADS, (O + LC_OT - 1) / LC_OT, G), dim3(KS_THREADS), 0, s,
                       cts, w, out, J, O, width);
    SLZ_HIP(hipGetLastError());
    return SLZ_OK;
}
