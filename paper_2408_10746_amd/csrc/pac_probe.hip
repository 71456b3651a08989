// Measurement aids: what this chip sustains on a plain read of a device buffer and on a register-only loop of
// bf16 matrix instructions.  The step's kernels are set against these next to the published peaks.
#include "../../include/pac.h"
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kReadThreads = 256;
constexpr int kReadUnroll = 8; // 16-byte loads in flight per lane

// Each workgroup walks its own contiguous share of the buffer (a streaming kernel's access pattern): per round
// a lane issues kReadUnroll independent 16-byte loads, 1 KB apart per wavefront, then folds them.
__global__ __launch_bounds__(kReadThreads) void k_probe_read(const u32x4 *__restrict__ buf, int64_t nchunks, float *sink)
{
    const int64_t per_block = (nchunks + gridDim.x - 1) / gridDim.x;
    const int64_t begin = per_block * blockIdx.x;
    const int64_t end = begin + per_block < nchunks ? begin + per_block : nchunks;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (int64_t c = begin + threadIdx.x; c < end; c += (int64_t)kReadThreads * kReadUnroll) {
        u32x4 v[kReadUnroll];
#pragma unroll
        for (int u = 0; u < kReadUnroll; ++u) {
            const int64_t cc = c + (int64_t)u * kReadThreads;
            v[u] = buf[cc < end ? cc : end - 1];
        }
#pragma unroll
        for (int u = 0; u < kReadUnroll; ++u) acc ^= v[u];
    }
    // data-dependent, practically never true: keeps the loads alive without a store per lane
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u) sink[threadIdx.x] = 1.f;
}

constexpr int kMfmaPerRound = 4;
__global__ __launch_bounds__(256) void k_probe_mfma(int64_t iters, float *sink)
{
    bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = static_cast<__bf16>(1.f / (float)(1 + ((threadIdx.x + e) & 7)));
        b[e] = static_cast<__bf16>((float)((threadIdx.x * 3 + e) & 3) * 0.25f);
    }
    f32x16 acc[kMfmaPerRound];
#pragma unroll
    for (int q = 0; q < kMfmaPerRound; ++q)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[q][v] = 0.f;
    for (int64_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int q = 0; q < kMfmaPerRound; ++q) acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[q], 0, 0, 0);
    }
    float tot = 0.f;
#pragma unroll
    for (int q = 0; q < kMfmaPerRound; ++q)
#pragma unroll
        for (int v = 0; v < 16; ++v) tot += acc[q][v];
    if (tot == -1.f) sink[threadIdx.x] = tot; // never true (all terms are non-negative): keeps the loop alive
}

constexpr int kMfmaBlocks = 256 * 4; // four workgroups of four wavefronts per compute unit

typedef float f32x4 __attribute__((ext_vector_type(4)));
// the optimizer update's access mix: four 16-byte loads and three 16-byte stores per lane and round
__global__ __launch_bounds__(256) void k_probe_update(f32x4 *__restrict__ p, f32x4 *__restrict__ m, f32x4 *__restrict__ v,
                                                      const f32x4 *__restrict__ g, int64_t ngroups)
{
    for (int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x; q < ngroups; q += (int64_t)gridDim.x * 256) {
        const f32x4 gv = g[q];
        const f32x4 pv = p[q], mv = m[q], vv = v[q];
        p[q] = pv + 1e-9f * gv;
        m[q] = mv * 0.9f + gv;
        v[q] = vv * 0.999f + gv;
    }
}

} // namespace

extern "C" {

pac_status pac_probe_hbm_read(const void *buf, int64_t bytes, float *sink, void *hip_stream)
{
    if (!buf || !sink) return PAC_ERR_NULL;
    if (bytes <= 0 || bytes % 16) return PAC_ERR_RANGE;
    if (reinterpret_cast<uintptr_t>(buf) & 15) return PAC_ERR_ALIGN;
    (void)hipGetLastError();
    const int64_t nchunks = bytes / 16;
    int64_t blocks = (nchunks + (int64_t)kReadThreads * kReadUnroll - 1) / ((int64_t)kReadThreads * kReadUnroll);
    if (blocks > 256 * 8) blocks = 256 * 8; // eight workgroups per compute unit, each with a contiguous share
    hipLaunchKernelGGL(k_probe_read, dim3((unsigned)blocks), dim3(kReadThreads), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const u32x4 *>(buf), nchunks, sink);
    return hipGetLastError() == hipSuccess ? PAC_OK : PAC_ERR_DEVICE;
}

pac_status pac_probe_mfma_bf16(int64_t iters, float *sink, void *hip_stream)
{
    if (!sink) return PAC_ERR_NULL;
    if (iters <= 0) return PAC_ERR_RANGE;
    (void)hipGetLastError();
    hipLaunchKernelGGL(k_probe_mfma, dim3(kMfmaBlocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream), iters, sink);
    return hipGetLastError() == hipSuccess ? PAC_OK : PAC_ERR_DEVICE;
}

pac_status pac_probe_hbm_update(float *p, float *m, float *v, const float *g, int64_t n, void *hip_stream)
{
    if (!p || !m || !v || !g) return PAC_ERR_NULL;
    if (n <= 0 || n % 4) return PAC_ERR_RANGE;
    if ((reinterpret_cast<uintptr_t>(p) | reinterpret_cast<uintptr_t>(m) | reinterpret_cast<uintptr_t>(v) |
         reinterpret_cast<uintptr_t>(g)) & 15)
        return PAC_ERR_ALIGN;
    (void)hipGetLastError();
    const int64_t ngroups = n / 4;
    int64_t blocks = (ngroups + 255) / 256; // one group per thread, as the optimizer launch
    if (blocks > (int64_t)1 << 22) blocks = (int64_t)1 << 22;
    hipLaunchKernelGGL(k_probe_update, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       reinterpret_cast<f32x4 *>(p), reinterpret_cast<f32x4 *>(m), reinterpret_cast<f32x4 *>(v),
                       reinterpret_cast<const f32x4 *>(g), ngroups);
    return hipGetLastError() == hipSuccess ? PAC_OK : PAC_ERR_DEVICE;
}

double pac_probe_mfma_flops(int64_t iters)
{
    // per wavefront and round: kMfmaPerRound instructions of 32 x 32 x 16 multiply-adds
    return (double)iters * kMfmaPerRound * 2.0 * 32 * 32 * 16 * 4 /*wavefronts*/ * kMfmaBlocks;
}

} // extern "C"
