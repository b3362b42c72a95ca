// Clear-weight linear combination of LWE ciphertexts (the leveled sums of Matmul^RNS, Algorithm 2 step 3) as an int8
// matrix-core contraction:  out[g][o][x] = sum_j w[j][o] * ct[g][j][x]  (mod 2^64).
//
// Per group g this is the product of the weight matrix (outputs x inputs) with the ciphertext matrix (inputs x words).
// A ciphertext word is recoded into eight signed bytes (byte planes, recombined with shifts at the end), exactly as the
// keyswitch does with its key.  An int32 weight W is recoded into five signed bytes, W = sum_b s_b 2^(8b) with
// s_b = byte b of (W + 0x80808080) - 128 for b < 4 and s_4 = (W + 0x80808080) >> 32; digit plane b multiplies the
// ciphertext word shifted left by 8 b bits, so every digit plane is just more rows of the same contraction.  A first
// kernel writes the digit planes in operand layout and records how many are non-zero anywhere (one, when every weight
// fits a signed byte); the contraction reads that count from device memory, so no host synchronisation is needed.
#include "slz_internal.h"
#include "slz_mfma_i8.h"

#define LM_MAX_PLANES 5

// ---- weights -------------------------------------------------------------------------------------------------------
// dig[otile][b][kb][lane] (16 bytes): A operand of lane `lane` for digit plane b, 32-row block kb of 32-output tile otile:
// output 32 otile + lane % 32, inputs j = 32 kb + 16 (lane / 32) + t for byte t; zero past J or O.
__global__ void k_lcm_clear(uint32_t *planes) { *planes = 1; }

__global__ void __launch_bounds__(64)
k_lcm_weights(const int32_t *__restrict__ w, v4i *__restrict__ dig, uint32_t *__restrict__ planes, uint32_t J, uint32_t O,
              uint32_t n_kb) {
    const uint32_t lane = threadIdx.x, kb = blockIdx.x, otile = blockIdx.y;
    const uint32_t o = otile * 32 + lane % 32;
    const uint32_t j0 = 32 * kb + 16 * (lane / 32);
    uint32_t wd[LM_MAX_PLANES][4];
#pragma unroll
    for (int b = 0; b < LM_MAX_PLANES; b++)
#pragma unroll
        for (int q = 0; q < 4; q++) wd[b][q] = 0;
    uint32_t used = 1;
#pragma unroll
    for (int t = 0; t < 16; t++) {
        const uint32_t j = j0 + t;
        const int64_t W = (o < O && j < J) ? (int64_t)w[(size_t)j * O + o] : 0;
        const int64_t T = W + 0x80808080ll;
#pragma unroll
        for (int b = 0; b < 4; b++) {
            const uint32_t s = (((uint32_t)(T >> (8 * b)) & 0xffu) - 128u) & 0xffu;
            wd[b][t / 4] |= s << (8 * (t % 4));
            if (s) used = max(used, (uint32_t)b + 1);
        }
        const uint32_t s4 = (uint32_t)(T >> 32) & 0xffu;
        wd[4][t / 4] |= s4 << (8 * (t % 4));
        if (s4) used = 5;
    }
#pragma unroll
    for (int b = 0; b < LM_MAX_PLANES; b++) {
        v4i v = {(int)wd[b][0], (int)wd[b][1], (int)wd[b][2], (int)wd[b][3]};
        dig[(((size_t)otile * LM_MAX_PLANES + b) * n_kb + kb) * 64 + lane] = v;
    }
    if (used > 1) atomicMax(planes, used);
}

// ---- contraction ---------------------------------------------------------------------------------------------------
struct lcm_args {
    const uint64_t *cts;    // [G][J][width]
    const v4i *dig;
    const uint32_t *planes;
    uint64_t *out;          // [G][O][width]
    uint32_t J, O, width;
    uint32_t n_kb;          // 32-row blocks per digit plane (ceil(J / 32))
    uint32_t n_otiles, o_groups, x_tiles, total, per_xcd;   // work items: (group g, x tile, output group), output group fastest
};

// W waves per workgroup: wave w owns output tile og W + w; every thread brings in 8 rows of one ciphertext word per
// iteration, so an iteration covers 16 W rows (W / 2 blocks of 32).
template <int W>
__global__ void __launch_bounds__(64 * W) __attribute__((amdgpu_waves_per_eu(2, 2)))
k_lcm_main(lcm_args A) {
    constexpr int IT_KB = W / 2;
    constexpr int BUF_V4 = IT_KB * 2 * 8 * 32;                      // 16-byte slots per LDS buffer: [block][half][plane][x]
    __shared__ v4i lds[2 * BUF_V4];
    // one XCD (workgroups b, b+8, ...) walks a contiguous range of work items: neighbouring word tiles of one group share
    // cache lines (rows are not line-aligned), which that XCD's L2 then serves
    const uint32_t item = (blockIdx.x % 8) * A.per_xcd + blockIdx.x / 8;
    if (blockIdx.x / 8 >= A.per_xcd || item >= A.total) return;
    const uint32_t og = item % A.o_groups;
    const uint32_t xt = (item / A.o_groups) % A.x_tiles;
    const uint32_t g = item / (A.o_groups * A.x_tiles);
    const uint32_t lane = threadIdx.x % 64;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
    const uint32_t otile = og * W + wave;
    const bool tile_ok = otile < A.n_otiles;
    const uint32_t planes = min(*A.planes, (uint32_t)LM_MAX_PLANES);
    const uint32_t kb_end = planes * A.n_kb;
    const uint32_t width = A.width;

    const uint32_t xl = lane % 32;
    const uint32_t x = xt * 32 + xl;
    const uint32_t oct = 2 * wave + lane / 32;
    const bool x_ok = x < width;
    const uint64_t *src = A.cts + (size_t)g * A.J * width + min(x, width - 1);
    // digit plane b and input index j of this thread's first row; they advance by 32 IT_KB rows per iteration
    const uint32_t plane_rows = 32 * A.n_kb;
    uint32_t b = (8 * oct) / plane_rows, j = (8 * oct) % plane_rows;
    const uint32_t lds_w = ((((oct / 4) * 2 + (oct / 2) % 2) * 8) * 32 + xl) * 2 + (oct & 1);   // in 8-byte units, plane 0

    // two register stages, as in the keyswitch: loads are unconditional, rows out of range are clamped and zeroed when used
    uint64_t kw0[8], kw1[8];
    uint32_t sh0, sh1, nv0, nv1;        // shift of the stage's digit plane; rows of the stage that exist
    v4i an0[IT_KB], an1[IT_KB];
    auto load_rows = [&](uint64_t (&kw)[8], uint32_t &sh, uint32_t &nv, uint32_t it) {
        const bool ok = x_ok && (it + oct / 4 < kb_end);
        nv = ok ? (j < A.J ? min(A.J - j, 8u) : 0u) : 0u;
        sh = 8 * b;
#pragma unroll
        for (int t = 0; t < 8; t++) kw[t] = src[(size_t)min(j + t, A.J - 1) * width];
        j += 32 * IT_KB;
        while (j >= plane_rows) { j -= plane_rows; b++; }
    };
    const size_t dig_base = (size_t)(tile_ok ? otile : 0) * LM_MAX_PLANES * A.n_kb;
    const uint32_t dig_last = LM_MAX_PLANES * A.n_kb - 1;
    auto load_dig = [&](v4i (&an)[IT_KB], uint32_t it) {
#pragma unroll
        for (int q = 0; q < IT_KB; q++) an[q] = A.dig[(dig_base + min(it + q, dig_last)) * 64 + lane];
    };

    v16i acc[8];
#pragma unroll
    for (int p = 0; p < 8; p++)
#pragma unroll
        for (int r = 0; r < 16; r++) acc[p][r] = 0;

    uint32_t buf = 0;
    auto body = [&](uint64_t (&kw)[8], uint32_t &sh, uint32_t &nv, v4i (&an)[IT_KB], uint32_t it) {
        {
            uint64_t w[8], plane[8];
#pragma unroll
            for (int t = 0; t < 8; t++) w[t] = (uint32_t)t < nv ? slz_signed_bytes(kw[t] << sh) : 0ull;
            slz_byte_planes(w, plane);
            uint64_t *dst = reinterpret_cast<uint64_t *>(lds + buf * BUF_V4) + lds_w;
#pragma unroll
            for (int p = 0; p < 8; p++) dst[(size_t)p * 64] = plane[p];
        }
        load_rows(kw, sh, nv, it + 2 * IT_KB);
        __syncthreads();    // one barrier per iteration suffices with two buffers (see the keyswitch kernel)
        if (tile_ok) {
            const v4i *bsrc = lds + buf * BUF_V4 + (lane / 32) * (8 * 32) + xl;
            v4i bb[2][4];
#pragma unroll
            for (int p = 0; p < 4; p++) bb[0][p] = bsrc[p * 32];
#pragma unroll
            for (int h = 0; h < 2 * IT_KB; h++) {                   // half block h: block h/2, planes 4 (h%2) .. +3
                if (h + 1 < 2 * IT_KB) {
#pragma unroll
                    for (int p = 0; p < 4; p++) bb[(h + 1) & 1][p] = bsrc[(((h + 1) / 2) * 2 * 8 + 4 * ((h + 1) % 2) + p) * 32];
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int p = 0; p < 4; p++)
                    acc[4 * (h % 2) + p] = __builtin_amdgcn_mfma_i32_32x32x32_i8(an[h / 2], bb[h & 1][p], acc[4 * (h % 2) + p], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        load_dig(an, it + 2 * IT_KB);
        buf ^= 1;
    };
    load_rows(kw0, sh0, nv0, 0);
    load_dig(an0, 0);
    load_rows(kw1, sh1, nv1, IT_KB);
    load_dig(an1, IT_KB);
    for (uint32_t it = 0; it < kb_end; it += 2 * IT_KB) {
        body(kw0, sh0, nv0, an0, it);
        body(kw1, sh1, nv1, an1, it + IT_KB);
    }
    if (!tile_ok || !x_ok) return;
    // accumulator register r of a lane is output 8 (r / 4) + 4 (lane / 32) + r % 4 of the tile, word x
#pragma unroll
    for (int r = 0; r < 16; r++) {
        const uint32_t o = otile * 32 + 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
        if (o < A.O) {
            uint64_t val = 0;
#pragma unroll
            for (int p = 0; p < 8; p++) val += (uint64_t)(int64_t)acc[p][r] << (8 * p);
            A.out[((size_t)g * A.O + o) * width + x] = val;
        }
    }
}

void slz_lcm_destroy(slz_ctx *ctx) {
    if (ctx->lc_dig) (void)hipFree(ctx->lc_dig);
    ctx->lc_dig = nullptr;
    ctx->lc_dig_bytes = 0;
}

int slz_lcm_launch(slz_ctx *ctx, const uint64_t *cts, const int32_t *w, uint64_t *out, uint32_t G, uint32_t J, uint32_t O,
                   hipStream_t s) {
    const uint32_t width = ctx->prm.n + 1;
    const uint32_t n_kb = (J + 31) / 32;
    // int32 accumulators: at most 5 planes x 32 n_kb rows of |digit * byte| <= 2^14
    if ((uint64_t)LM_MAX_PLANES * 32 * n_kb >= (1u << 17)) return SLZ_E_UNSUPPORTED;
    const uint32_t n_otiles = (O + 31) / 32;
    const size_t need = ((size_t)n_otiles * LM_MAX_PLANES * n_kb * 64 + 16) * 16;      // operands + the plane count
    if (ctx->lc_dig_bytes < need) {
        // the previous buffer may still be read by work queued on another stream: wait before letting it go
        if (ctx->lc_dig) { SLZ_HIP(hipDeviceSynchronize()); (void)hipFree(ctx->lc_dig); ctx->lc_dig = nullptr; ctx->lc_dig_bytes = 0; }
        if (slz_scratch_alloc(&ctx->lc_dig, need) != SLZ_OK) return SLZ_E_NOMEM;
        ctx->lc_dig_bytes = need;
    }
    v4i *dig = (v4i *)ctx->lc_dig;
    uint32_t *planes = (uint32_t *)(dig + (size_t)n_otiles * LM_MAX_PLANES * n_kb * 64);
    if (n_otiles > 65535) return SLZ_E_UNSUPPORTED;
    hipLaunchKernelGGL(k_lcm_clear, dim3(1), dim3(1), 0, s, planes);
    hipLaunchKernelGGL(k_lcm_weights, dim3(n_kb, n_otiles), dim3(64), 0, s, w, dig, planes, J, O, n_kb);
    lcm_args A;
    A.cts = cts; A.dig = dig; A.planes = planes; A.out = out;
    A.J = J; A.O = O; A.width = width; A.n_kb = n_kb; A.n_otiles = n_otiles;
    A.x_tiles = (width + 31) / 32;
    const int W = n_otiles <= 2 ? 2 : (n_otiles <= 4 ? 4 : 8);
    A.o_groups = (n_otiles + W - 1) / W;
    const uint64_t total = (uint64_t)G * A.x_tiles * A.o_groups;
    if (total > (1u << 30)) return SLZ_E_UNSUPPORTED;
    A.total = (uint32_t)total;
    A.per_xcd = (A.total + 7) / 8;
    const dim3 grid(A.per_xcd * 8);
    if (W == 2) hipLaunchKernelGGL(k_lcm_main<2>, grid, dim3(128), 0, s, A);
    else if (W == 4) hipLaunchKernelGGL(k_lcm_main<4>, grid, dim3(256), 0, s, A);
    else hipLaunchKernelGGL(k_lcm_main<8>, grid, dim3(512), 0, s, A);
    SLZ_HIP(hipGetLastError());
    return SLZ_OK;
}
