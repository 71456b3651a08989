// Block-wise absmax quantisation (Eq. "quan"), its inverse (Eq. "dequan") and the mixed-precision linear layer on
// the stored form, optionally with the cache fill fused into its epilogue (declared in include/pac_quant.h).
#include "../../include/pac_quant.h"
#include "pac_gemm.h"
#include "pac_internal.h"

namespace pac {

static inline bool q_aligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// ---------------------------------------------------------------------------
// quantise, any block size: one wavefront per block; lanes take pairs of neighbouring values (one byte of 4-bit codes)
// ---------------------------------------------------------------------------
template <int BITS>
__global__ __launch_bounds__(256) void k_quant(const float *__restrict__ x, int64_t n, int block, int64_t nblocks,
                                               int8_t *__restrict__ codes, float *__restrict__ consts)
{
    constexpr float qmax = BITS == 8 ? 127.f : 7.f;
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6), nwaves = (int64_t)gridDim.x * 4;
    for (int64_t b = wave; b < nblocks; b += nwaves) {
        const int64_t b0 = b * block;
        const int len = (int)(n - b0 < block ? n - b0 : block);
        float amax = 0.f;
        for (int e = lane; e < len; e += 64) amax = fmaxf(amax, fabsf(x[b0 + e]));
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o, 64));
        const float c = amax == 0.f ? 1.f : qmax / amax; // correctly rounded 32-bit division
        if (lane == 0) consts[b] = c;
        for (int e = 2 * lane; e < len; e += 128) {
            // 32-bit products, rounded on their own (no contraction with anything), then to the nearest integer, ties to even
            const int q0 = (int)rintf(__fmul_rn(c, x[b0 + e]));
            const int q1 = e + 1 < len ? (int)rintf(__fmul_rn(c, x[b0 + e + 1])) : 0;
            if (BITS == 8) {
                codes[b0 + e] = (int8_t)q0;
                if (e + 1 < len) codes[b0 + e + 1] = (int8_t)q1;
            } else {
                // block is even, so b0 + e is even: this pair is one byte, the even index in the low nibble
                reinterpret_cast<uint8_t *>(codes)[(b0 + e) >> 1] = (uint8_t)((q0 & 0xf) | ((q1 & 0xf) << 4));
            }
        }
    }
}

// The same for blocks of 4 .. 256 values that tile the tensor exactly (block = 4 x a power of two, n a multiple of
// block, 16-byte aligned input): a lane takes four neighbouring values with one 16-byte load, the block's lanes find
// the absmax with lane exchanges, and the four codes leave as one 4-byte (2-byte) store.  One group of four per
// thread, no strided walk.  Same arithmetic, same bits.
template <int BITS>
__global__ __launch_bounds__(256) void k_quant4(const f32x4 *__restrict__ x, int64_t ngroups, int lanes_per_block,
                                                int8_t *__restrict__ codes, float *__restrict__ consts)
{
    constexpr float qmax = BITS == 8 ? 127.f : 7.f;
    const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const bool live = q < ngroups; // (whole blocks never straddle the end: ngroups is a multiple of lanes_per_block)
    const f32x4 v = x[live ? q : ngroups - 1];
    float amax = fmaxf(fmaxf(fabsf(v[0]), fabsf(v[1])), fmaxf(fabsf(v[2]), fabsf(v[3])));
    for (int o = 1; o < lanes_per_block; o <<= 1) amax = fmaxf(amax, __shfl_xor(amax, o, 64));
    const float c = amax == 0.f ? 1.f : qmax / amax; // correctly rounded 32-bit division
    if (!live) return;
    if ((q & (lanes_per_block - 1)) == 0) consts[q / lanes_per_block] = c;
    int qv[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) qv[e] = (int)rintf(__fmul_rn(c, v[e]));
    if (BITS == 8)
        reinterpret_cast<uint32_t *>(codes)[q] = (uint32_t)(qv[0] & 0xff) | ((uint32_t)(qv[1] & 0xff) << 8) |
                                                 ((uint32_t)(qv[2] & 0xff) << 16) | ((uint32_t)(qv[3] & 0xff) << 24);
    else
        reinterpret_cast<uint16_t *>(codes)[q] = (uint16_t)((qv[0] & 0xf) | ((qv[1] & 0xf) << 4) | ((qv[2] & 0xf) << 8) |
                                                            ((qv[3] & 0xf) << 12));
}

__device__ __forceinline__ int nibble_value(uint32_t byte, int hi)
{
    const int nib = hi ? (int)(byte >> 4) & 0xf : (int)byte & 0xf;
    return nib >= 8 ? nib - 16 : nib;
}

template <int BITS>
__global__ __launch_bounds__(256) void k_dequant(const int8_t *__restrict__ codes, const float *__restrict__ consts,
                                                 int64_t n, int block, float *__restrict__ out)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
        const int q = BITS == 8 ? (int)codes[i] : nibble_value(reinterpret_cast<const uint8_t *>(codes)[i >> 1], (int)(i & 1));
        out[i] = __fdiv_rn((float)q, consts[i / block]);
    }
}

// ---------------------------------------------------------------------------
// linear layer on the stored form.  128 x 128 output tile per workgroup, four wavefronts of 2 x 2 accumulators of
// 32 x 32 each; K in steps of 32 staged through two LDS buffers (x as it is, the codes converted to bf16, which holds
// every code exactly).  A quantisation block's partial sum is kept apart (its first matrix instruction starts from
// zero) and enters the total multiplied by 1 / c of that block and column: in the 32 x 32 accumulator layout all 16
// values of a lane belong to one output column.
// ---------------------------------------------------------------------------
constexpr int kDqPitch = 32 * 2 + 16; // bytes per LDS row of a K step
constexpr int kDqTile = 128;

struct DqArgs {
    const bf16_t *x;
    int M, K, N, block;
    const int8_t *codes;
    const float *consts;
    float *y;          // dense output, or null
    // fused cache fill (y == null): row m of x is token m % n_max of sample m / n_max
    void *cache;
    int cache_f32, n_max, layer;
    BatchMeta meta;
};

__device__ __forceinline__ uint16_t dq_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7f800000u) == 0x7f800000u && (u & 0x007fffffu) != 0u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <int BITS> __global__ __launch_bounds__(256) void k_dq_linear(DqArgs a)
{
    __shared__ __attribute__((aligned(16))) char As[2][kDqTile * kDqPitch];
    __shared__ __attribute__((aligned(16))) char Bs[2][kDqTile * kDqPitch];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int i = lane & 31, g = lane >> 5;
    const int m0 = blockIdx.y * kDqTile, n0 = blockIdx.x * kDqTile;
    const int K = a.K, nsteps = K / 32, bpr = K / a.block, steps_per_block = a.block / 32;
    // this thread's share of a K step: 16 bytes of two x rows, 8 codes of two W rows (rows lrow and lrow + 64)
    const int lrow = t >> 2, lch = t & 3;
    const bf16_t *xp[2];
    const int8_t *wp[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int xm = min(m0 + lrow + 64 * h, a.M - 1), wr = min(n0 + lrow + 64 * h, a.N - 1);
        xp[h] = a.x + (int64_t)xm * K + lch * 8;
        wp[h] = a.codes + (BITS == 8 ? (int64_t)wr * K + lch * 8 : ((int64_t)wr * K + lch * 8) / 2);
    }
    auto load = [&](int s, u32x4 (&av)[2], uint64_t (&bv)[2]) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            av[h] = *reinterpret_cast<const u32x4 *>(xp[h] + s * 32);
            if (BITS == 8) bv[h] = *reinterpret_cast<const uint64_t *>(wp[h] + s * 32);
            else bv[h] = *reinterpret_cast<const uint32_t *>(wp[h] + s * 16);
        }
    };
    auto store = [&](int buf, const u32x4 (&av)[2], const uint64_t (&bv)[2]) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            *reinterpret_cast<u32x4 *>(As[buf] + (lrow + 64 * h) * kDqPitch + lch * 16) = av[h];
            // a code is an integer of at most 8 bits: its fp32 image has zero low mantissa bits, so the upper half of
            // that image IS its bf16 value (no rounding happens); two codes per 32-bit word
            u32x4 w;
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) {
                int q0, q1;
                if (BITS == 8) {
                    const uint32_t word = (uint32_t)(bv[h] >> (32 * (e2 >> 1)));
                    q0 = (int)(word << (24 - 16 * (e2 & 1))) >> 24;
                    q1 = (int)(word << (16 - 16 * (e2 & 1))) >> 24;
                } else {
                    const uint32_t word = (uint32_t)bv[h];
                    q0 = (int)(word << (28 - 8 * e2)) >> 28;
                    q1 = (int)(word << (24 - 8 * e2)) >> 28;
                }
                w[e2] = (__float_as_uint((float)q0) >> 16) | (__float_as_uint((float)q1) & 0xffff0000u);
            }
            *reinterpret_cast<u32x4 *>(Bs[buf] + (lrow + 64 * h) * kDqPitch + lch * 16) = w;
        }
    };
    f32x16 tot[2][2], part[2][2];
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y)
#pragma unroll
            for (int v = 0; v < 16; ++v) tot[x][y][v] = part[x][y][v] = 0.f;
    const float *crow[2];
#pragma unroll
    for (int y = 0; y < 2; ++y) crow[y] = a.consts + (int64_t)min(n0 + wn * 64 + y * 32 + i, a.N - 1) * bpr;
    auto compute = [&](int buf, bool first) {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            bf16x8 fa[2], fb[2];
#pragma unroll
            for (int x = 0; x < 2; ++x)
                fa[x] = *reinterpret_cast<const bf16x8 *>(As[buf] + (wm * 64 + x * 32 + i) * kDqPitch + ks * 32 + g * 16);
#pragma unroll
            for (int y = 0; y < 2; ++y)
                fb[y] = *reinterpret_cast<const bf16x8 *>(Bs[buf] + (wn * 64 + y * 32 + i) * kDqPitch + ks * 32 + g * 16);
#pragma unroll
            for (int x = 0; x < 2; ++x)
#pragma unroll
                for (int y = 0; y < 2; ++y) {
                    f32x16 c0 = part[x][y];
                    if (ks == 0 && first) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) c0[v] = 0.f; // a new block's partial sum starts from zero
                    }
                    part[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[x], fb[y], c0, 0, 0, 0);
                }
        }
    };
    u32x4 av[2];
    uint64_t bv[2];
    load(0, av, bv);
    store(0, av, bv);
    __syncthreads();
    int in_block = 0;
    for (int s = 0; s < nsteps; ++s) {
        const int buf = s & 1;
        if (s + 1 < nsteps) load(s + 1, av, bv);
        if (in_block == 0) compute(buf, true);
        else compute(buf, false);
        if (++in_block == steps_per_block) {
            in_block = 0;
            const int blk = s / steps_per_block;
#pragma unroll
            for (int y = 0; y < 2; ++y) {
                const float inv = __fdiv_rn(1.f, crow[y][blk]);
#pragma unroll
                for (int x = 0; x < 2; ++x)
#pragma unroll
                    for (int v = 0; v < 16; ++v) tot[x][y][v] += part[x][y][v] * inv;
            }
        }
        if (s + 1 < nsteps) store(buf ^ 1, av, bv);
        __syncthreads();
    }
#pragma unroll
    for (int y = 0; y < 2; ++y) {
        const int n = n0 + wn * 64 + y * 32 + i;
        if (n >= a.N) continue;
#pragma unroll
        for (int x = 0; x < 2; ++x)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm * 64 + x * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
                if (m >= a.M) continue;
                if (a.y) {
                    a.y[(int64_t)m * a.N + n] = tot[x][y][v];
                } else {
                    const int smp = m / a.n_max, tok = m - smp * a.n_max;
                    const int len = a.meta.len[smp];
                    if (tok >= len) continue;
                    const int64_t o = a.meta.off[smp] + ((int64_t)a.layer * len + tok) * a.N + n;
                    if (a.cache_f32) reinterpret_cast<float *>(a.cache)[o] = tot[x][y][v];
                    else reinterpret_cast<uint16_t *>(a.cache)[o] = dq_bf16_rne(tot[x][y][v]);
                }
            }
    }
}

static pac_status check_quant_args(const void *a, const void *b, const void *c, int64_t n, int32_t block, int32_t bits)
{
    if (!a || !b || !c) return PAC_ERR_NULL;
    if (bits != 8 && bits != 4) return PAC_ERR_SHAPE;
    if (n < 0 || block < 1 || (bits == 4 && (block & 1))) return PAC_ERR_RANGE;
    return PAC_OK;
}

hipError_t launch_dq_linear(const void *x, int M, int K, const int8_t *codes, const float *consts, int N, int block,
                            int bits, float *y, void *cache, int cache_f32, int n_max, int layer, const BatchMeta *meta,
                            hipStream_t st)
{
    DqArgs a{};
    a.x = static_cast<const bf16_t *>(x); a.M = M; a.K = K; a.N = N; a.block = block; a.codes = codes; a.consts = consts;
    a.y = y; a.cache = cache; a.cache_f32 = cache_f32; a.n_max = n_max; a.layer = layer;
    if (meta) a.meta = *meta;
    const dim3 grid((unsigned)((N + kDqTile - 1) / kDqTile), (unsigned)((M + kDqTile - 1) / kDqTile));
    if (bits == 8) hipLaunchKernelGGL(k_dq_linear<8>, grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL(k_dq_linear<4>, grid, dim3(256), 0, st, a);
    return hipGetLastError();
}

int check_dq_linear_args(const void *x, int32_t M, int32_t K, const int8_t *codes, const float *consts, int32_t N,
                                int32_t block, int32_t bits)
{
    if (!x || !codes || !consts) return PAC_ERR_NULL;
    if (bits != 8 && bits != 4) return PAC_ERR_SHAPE;
    if (M < 1 || N < 1 || K < 32 || K % 32) return PAC_ERR_SHAPE;
    if (block < 32 || block % 32 || K % block) return PAC_ERR_RANGE;
    if (!q_aligned(x, 16) || !q_aligned(codes, 8) || !q_aligned(consts, 4)) return PAC_ERR_ALIGN;
    return PAC_OK;
}

} // namespace pac

using namespace pac;

extern "C" {

pac_status pac_quant_blockwise(const float *x, int64_t n, int32_t block, int32_t bits, int8_t *codes, float *consts,
                               void *hip_stream)
{
    pac_status s = check_quant_args(x, codes, consts, n, block, bits);
    if (s != PAC_OK) return s;
    if (!q_aligned(x, 4) || !q_aligned(consts, 4)) return PAC_ERR_ALIGN;
    if (n == 0) return PAC_OK;
    (void)hipGetLastError();
    const int64_t nblocks = (n + block - 1) / block;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int lpb = block / 4;
    if (block % 4 == 0 && lpb <= 64 && (lpb & (lpb - 1)) == 0 && n % block == 0 && q_aligned(x, 16) &&
        q_aligned(codes, bits == 8 ? 4 : 2) && n / 4 <= ((int64_t)1 << 30) * 256) {
        const int64_t ngroups = n / 4;
        const unsigned g4 = (unsigned)((ngroups + 255) / 256);
        if (bits == 8)
            hipLaunchKernelGGL(k_quant4<8>, dim3(g4), dim3(256), 0, st, reinterpret_cast<const f32x4 *>(x), ngroups, lpb, codes, consts);
        else
            hipLaunchKernelGGL(k_quant4<4>, dim3(g4), dim3(256), 0, st, reinterpret_cast<const f32x4 *>(x), ngroups, lpb, codes, consts);
        return hipGetLastError() == hipSuccess ? PAC_OK : PAC_ERR_DEVICE;
    }
    int64_t grid = (nblocks + 3) / 4;
    if (grid > 256 * 16) grid = 256 * 16;
    if (bits == 8) hipLaunchKernelGGL(k_quant<8>, dim3((unsigned)grid), dim3(256), 0, st, x, n, block, nblocks, codes, consts);
    else hipLaunchKernelGGL(k_quant<4>, dim3((unsigned)grid), dim3(256), 0, st, x, n, block, nblocks, codes, consts);
    return hipGetLastError() == hipSuccess ? PAC_OK : PAC_ERR_DEVICE;
}

pac_status pac_dequant_blockwise(const int8_t *codes, const float *consts, int64_t n, int32_t block, int32_t bits,
                                 float *out, void *hip_stream)
{
    pac_status s = check_quant_args(codes, consts, out, n, block, bits);
    if (s != PAC_OK) return s;
    if (!q_aligned(out, 4) || !q_aligned(consts, 4)) return PAC_ERR_ALIGN;
    if (n == 0) return PAC_OK;
    (void)hipGetLastError();
    int64_t grid = (n + 255) / 256;
    if (grid > 256 * 32) grid = 256 * 32;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (bits == 8) hipLaunchKernelGGL(k_dequant<8>, dim3((unsigned)grid), dim3(256), 0, st, codes, consts, n, block, out);
    else hipLaunchKernelGGL(k_dequant<4>, dim3((unsigned)grid), dim3(256), 0, st, codes, consts, n, block, out);
    return hipGetLastError() == hipSuccess ? PAC_OK : PAC_ERR_DEVICE;
}

pac_status pac_dequant_linear(const void *x, int32_t M, int32_t K, const int8_t *codes, const float *consts, int32_t N,
                              int32_t block, int32_t bits, float *y, void *hip_stream)
{
    pac_status s = (pac_status)check_dq_linear_args(x, M, K, codes, consts, N, block, bits);
    if (s != PAC_OK) return s;
    if (!y) return PAC_ERR_NULL;
    if (!q_aligned(y, 4)) return PAC_ERR_ALIGN;
    (void)hipGetLastError();
    return launch_dq_linear(x, M, K, codes, consts, N, block, bits, y, nullptr, 0, 0, 0, nullptr,
                            static_cast<hipStream_t>(hip_stream)) == hipSuccess ? PAC_OK : PAC_ERR_DEVICE;
}

} // extern "C"
