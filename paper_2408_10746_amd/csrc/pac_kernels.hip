// HIP kernels (gfx950) and their launchers for the cached Parallel-Adapter step.
//
// Per-layer formulation: the side state s_l and its gradient ds_l live in the
// workspace as fp32 [tokens][d]; each layer runs
//   forward : down-projection (gate + GEMM + bias + GELU), up-projection (GEMM + residual)
//   backward: dpre = (ds W_up^T) * GELU'(pre); token reductions for dW_up, dc_up,
//             dW_down, dc_down (split over tokens, partials summed in a fixed order);
//             dx = dpre W_down^T with dlambda and ds_{l-1} = ds_l + (1-lambda) dx fused.
// All contractions go through the MFMA core in pac_gemm.h.  Reductions are
// ordered (no floating-point atomics), so a step is bit-reproducible.
#include "pac_gemm.h"
#include "pac_internal.h"

namespace pac {

using T64 = Tile<2, 2, 1, 1, 1>;  // 64 x 64 workgroup tile, 64 bytes of K per step
template <int KU> using T64U = Tile<2, 2, 1, 1, KU>; // same tile, KU * 64 bytes of K per step
using T64K = Tile<2, 2, 1, 1, 4>; // same tile, 256 bytes of K per step (token reductions)

// launch, optionally bracketed by timing events of its kernel class
#define PAC_LAUNCH(prof, st, cls, ...)                         \
    do {                                                       \
        if (prof) (void)(prof)->mark((st), (cls), true);           \
        hipLaunchKernelGGL(__VA_ARGS__);                       \
        if (prof) (void)(prof)->mark((st), (cls), false);           \
    } while (0)

#define PAC_HIP_TRY(expr)                          \
    do {                                           \
        hipError_t e_ = (expr);                    \
        if (e_ != hipSuccess) return e_;           \
    } while (0)

static inline int64_t align256(int64_t x) { return (x + 255) & ~int64_t(255); }
static inline int cdiv(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

static int choose_splits(const Dims &D)
{
    // tiles of both weight-gradient contractions of one layer
    int64_t tiles = 2 * (int64_t)cdiv(D.r, 64) * cdiv(D.d, 64);
    int s = (int)((1024 + tiles - 1) / tiles);
    int max_by_rows = (int)((D.Mmax + 255) / 256); // at least 256 token rows per split
    if (s > max_by_rows) s = max_by_rows;
    if (s > 32) s = 32;
    if (s < 1) s = 1;
    return s;
}

void plan_workspace(const Dims &D, WsLayout &W)
{
    const int64_t tc = D.cache_dtype == 0 ? 2 : 4;
    int64_t o = 0;
    auto take = [&](int64_t bytes) { int64_t at = o; o = align256(o + bytes); return at; };
    W.rowoff = take(D.Mmax * 8);
    W.rowstride = take(D.Mmax * 4);
    W.rowsamp = take(D.Mmax * 4);
    W.samp_start = take((kMaxBatch + 1) * 4);
    W.samp_len = take(kMaxBatch * 4);
    const int64_t wbytes = (int64_t)D.L * D.d * D.r * tc;
    // The Gram-matrix formulation keeps no d-wide per-token state and needs two of the four projection copies:
    // the per-layer regions it never touches (gigabytes at the wide shapes) are not reserved for it.
    const bool gram = gram_path_kind(D) != 0;
    W.Wd = gram ? 0 : take(wbytes);
    W.WdT = take(wbytes);
    W.Wu = take(wbytes);
    W.WuT = gram ? 0 : take(wbytes);
    W.s_all = gram ? 0 : take((int64_t)D.L * D.Mmax * D.d * 4);
    W.pre_all = take((int64_t)D.L * D.Mmax * D.r * 4);
    W.h_all = take((int64_t)D.L * D.Mmax * D.r * tc);
    W.ds = gram ? 0 : take(D.Mmax * D.d * 4);
    W.dpre = gram ? 0 : take(D.Mmax * D.r * tc);
    W.pooled = take((int64_t)D.B_max * D.d * 4);
    W.logits = take((int64_t)D.B_max * D.C * 4);
    W.dz = take((int64_t)D.B_max * D.C * 4);
    W.splits = choose_splits(D);
    W.part = gram ? 0 : take((int64_t)W.splits * D.PL * 4);
    W.dlam_slots = cdiv(D.Mmax, 64) * cdiv(D.d, 64);
    if (W.dlam_slots < D.B_max * D.r) W.dlam_slots = D.B_max * D.r; // also holds the top layer's dh [B][r]
    W.dlam_part = gram ? 0 : take((int64_t)W.dlam_slots * 4);
    W.grads = take(D.P * 4);
    W.use_gram = 0;
    if (gram) plan_gram_workspace(D, W, o);
    W.total = o;
}

// ---------------------------------------------------------------------------
// cache fill: fp32/bf16 activations -> packed [sample][layer][token][d] blocks
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7f800000u) == 0x7f800000u && (u & 0x007fffffu) != 0u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// SRC/DST in {float, uint16_t (bf16 bits)}
template <typename SRC, typename DST>
__global__ __launch_bounds__(256) void k_cache_fill(DST *__restrict__ cache, const SRC *__restrict__ acts,
                                                    BatchMeta meta, int L, int n_max, int d)
{
    const int i = blockIdx.y;
    const int len = meta.len[i];
    const int64_t per_layer = (int64_t)len * d;
    const int64_t total = per_layer * L;
    const int64_t e0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;
    if (e0 >= total) return;
    const int l = (int)(e0 / per_layer);
    const int64_t rem = e0 - (int64_t)l * per_layer;
    const int t = (int)(rem / d);
    const int j = (int)(rem - (int64_t)t * d);
    const SRC *src = acts + (((int64_t)i * L + l) * n_max + t) * d + j;
    DST *dst = cache + meta.off[i] + e0;
    alignas(16) SRC in[8];
    alignas(16) DST out[8];
    if (sizeof(SRC) == 4) {
        *reinterpret_cast<uint4 *>(&in[0]) = *reinterpret_cast<const uint4 *>(src);
        *reinterpret_cast<uint4 *>(&in[4]) = *reinterpret_cast<const uint4 *>(src + 4);
    } else {
        *reinterpret_cast<uint4 *>(&in[0]) = *reinterpret_cast<const uint4 *>(src);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        if (sizeof(SRC) == 4 && sizeof(DST) == 2) {
            float f;
            __builtin_memcpy(&f, &in[e], 4);
            uint16_t h = f32_to_bf16_rne(f);
            __builtin_memcpy(&out[e], &h, 2);
        } else if (sizeof(SRC) == 2 && sizeof(DST) == 4) {
            uint16_t h;
            __builtin_memcpy(&h, &in[e], 2);
            float f = __uint_as_float((uint32_t)h << 16);
            __builtin_memcpy(&out[e], &f, 4);
        } else {
            __builtin_memcpy(&out[e], &in[e], sizeof(DST));
        }
    }
    if (sizeof(DST) == 4) {
        *reinterpret_cast<uint4 *>(dst) = *reinterpret_cast<uint4 *>(&out[0]);
        *reinterpret_cast<uint4 *>(dst + 4) = *reinterpret_cast<uint4 *>(&out[4]);
    } else {
        *reinterpret_cast<uint4 *>(dst) = *reinterpret_cast<uint4 *>(&out[0]);
    }
}

hipError_t launch_cache_fill(const Dims &D, void *cache, const void *acts, int acts_dtype,
                             const BatchMeta &meta, hipStream_t st, Profiler *prof)
{
    if (meta.B <= 0) return hipSuccess;
    int maxlen = 0;
    for (int i = 0; i < meta.B; ++i) maxlen = meta.len[i] > maxlen ? meta.len[i] : maxlen;
    const int64_t chunks = (int64_t)D.L * maxlen * D.d / 8;
    dim3 grid((unsigned)cdiv(chunks, 256), (unsigned)meta.B);
    const bool src_bf16 = acts_dtype == 0, dst_bf16 = D.cache_dtype == 0;
    if (!src_bf16 && dst_bf16)
        PAC_LAUNCH(prof, st, KC_CACHE_FILL, (k_cache_fill<float, uint16_t>), grid, dim3(256), 0, st, (uint16_t *)cache,
                           (const float *)acts, meta, D.L, D.n_max, D.d);
    else if (src_bf16 && dst_bf16)
        PAC_LAUNCH(prof, st, KC_CACHE_FILL, (k_cache_fill<uint16_t, uint16_t>), grid, dim3(256), 0, st, (uint16_t *)cache,
                           (const uint16_t *)acts, meta, D.L, D.n_max, D.d);
    else if (!src_bf16 && !dst_bf16)
        PAC_LAUNCH(prof, st, KC_CACHE_FILL, (k_cache_fill<float, float>), grid, dim3(256), 0, st, (float *)cache,
                           (const float *)acts, meta, D.L, D.n_max, D.d);
    else
        PAC_LAUNCH(prof, st, KC_CACHE_FILL, (k_cache_fill<uint16_t, float>), grid, dim3(256), 0, st, (float *)cache,
                           (const uint16_t *)acts, meta, D.L, D.n_max, D.d);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// batch gather: sample ids -> per-token-row cache addresses
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_setup(BatchMeta meta, int d, int64_t *rowoff, int32_t *rowstride,
                                               int32_t *rowsamp, int32_t *samp_start, int32_t *samp_len)
{
    const int m = blockIdx.x * 256 + threadIdx.x;
    if (blockIdx.x == 0 && threadIdx.x <= meta.B) {
        samp_start[threadIdx.x] = meta.tok_start[threadIdx.x];
        if ((int)threadIdx.x < meta.B) samp_len[threadIdx.x] = meta.len[threadIdx.x];
    }
    if (m >= meta.M) return;
    int s = 0;
    while (s + 1 < meta.B && meta.tok_start[s + 1] <= m) ++s;
    const int t = m - meta.tok_start[s];
    rowoff[m] = meta.off[s] + (int64_t)t * d;
    rowstride[m] = meta.len[s] * d;
    rowsamp[m] = s;
}

// ---------------------------------------------------------------------------
// compute-dtype copies of the projection matrices, in both orientations
// z = 0: W_down [d][r] -> Wd [d][r], WdT [r][d];  z = 1: W_up [r][d] -> Wu [r][d], WuT [d][r]
// ---------------------------------------------------------------------------
template <typename TC>
__global__ __launch_bounds__(256) void k_shadows(const float *__restrict__ params, int64_t PL, int d, int r,
                                                 TC *__restrict__ Wd, TC *__restrict__ WdT,
                                                 TC *__restrict__ Wu, TC *__restrict__ WuT)
{
    __shared__ float tile[32][33];
    const int layer = blockIdx.y, which = blockIdx.z;
    const int rows = which == 0 ? d : r, cols = which == 0 ? r : d;
    const int tiles_c = cols / 32;
    const int tr = blockIdx.x / tiles_c, tcx = blockIdx.x % tiles_c;
    if (tr >= rows / 32) return;
    const float *src = params + (int64_t)layer * PL + (which == 0 ? 0 : (int64_t)d * r + r);
    TC *same = (which == 0 ? Wd : Wu) + (int64_t)layer * d * r;
    TC *tran = (which == 0 ? WdT : WuT) + (int64_t)layer * d * r;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int y = ty; y < 32; y += 8) {
        float f = src[(int64_t)(tr * 32 + y) * cols + tcx * 32 + tx];
        tile[y][tx] = f;
        same[(int64_t)(tr * 32 + y) * cols + tcx * 32 + tx] = to_tc(f, TC());
    }
    __syncthreads();
    for (int y = ty; y < 32; y += 8)
        tran[(int64_t)(tcx * 32 + y) * rows + tr * 32 + tx] = to_tc(tile[tx][y], TC());
}

// ---------------------------------------------------------------------------
// GELU (erf form) and its derivative
// ---------------------------------------------------------------------------
__device__ __forceinline__ float gelu_f(float u) { return 0.5f * u * (1.f + erff(u * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_grad_f(float u)
{
    const float Phi = 0.5f * (1.f + erff(u * 0.70710678118654752f));
    const float phi = 0.3989422804014327f * expf(-0.5f * u * u);
    return Phi + u * phi;
}

// ---------------------------------------------------------------------------
// forward, layer l
// ---------------------------------------------------------------------------
template <typename TC> struct FwdDownArgs {
    const TC *cache;
    RowMap map;
    int layer, d, r;
    const float *s_prev; // [M][d] or null (layer 0)
    const TC *WdT;       // [r][d]
    const float *c_down; // [r]
    const float *lam;    // 1
    float *pre;          // [M][r]
    TC *h;               // [M][r]
};

template <typename TC> struct EpiFwdDown {
    static constexpr bool kBatched = true;
    const float *c_down;
    float *pre;
    TC *h;
    int r;
    __device__ void batch(int row_base, int col, const f32x16 &acc, int nrows, int ncols) const
    {
        const float cd = c_down[min(col, ncols - 1)];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = epi_row(row_base, v);
            if (row < nrows && col < ncols) {
                const float u = acc[v] + cd;
                pre[(int64_t)row * r + col] = u;
                h[(int64_t)row * r + col] = to_tc(gelu_f(u), TC());
            }
        }
    }
};

template <typename TC, bool MIX, int KU> __device__ __forceinline__ void fwd_down_tile(const FwdDownArgs<TC> &a, char *smem)
{
    LoadRowsX<TC, 64, KU, MIX> al;
    al.cache = a.cache; al.map = a.map; al.layer = a.layer; al.s_prev = a.s_prev; al.ld_s = a.d; al.lam = *a.lam;
    LoadRowsTC<TC, 64, KU> bl;
    bl.src = a.WdT; bl.ld = a.d; bl.nrows = a.r;
    EpiFwdDown<TC> epi{a.c_down, a.pre, a.h, a.r};
    gemm_tile<TC, T64U<KU>>(smem, al, bl, epi, 0, a.d, blockIdx.x * 64, blockIdx.y * 64, a.map.M, a.r);
}

// KU = 4 needs the contraction length to be a multiple of 4 * 64 bytes of K; else KU = 1
template <typename TC, int KU> __global__ __launch_bounds__(256) void k_fwd_down(FwdDownArgs<TC> a)
{
    __shared__ __attribute__((aligned(16))) char smem[tile_lds_bytes<TC, T64U<KU>>()];
    if (a.s_prev) fwd_down_tile<TC, true, KU>(a, smem);
    else fwd_down_tile<TC, false, KU>(a, smem);
}

template <typename TC> struct FwdUpArgs {
    const TC *h;    // [M][r]
    const TC *WuT;  // [d][r]
    const float *c_up;
    const float *s_prev; // or null
    float *s_out;        // [M][d]
    int M, d, r;
};

struct EpiFwdUp {
    static constexpr bool kBatched = true;
    const float *c_up;
    const float *s_prev;
    float *s_out;
    int d;
    __device__ void batch(int row_base, int col, const f32x16 &acc, int nrows, int ncols) const
    {
        const int cc = min(col, ncols - 1);
        const float cu = c_up[cc];
        float sp[16];
#pragma unroll
        for (int v = 0; v < 16; ++v)
            sp[v] = s_prev ? s_prev[(int64_t)min(epi_row(row_base, v), nrows - 1) * d + cc] : 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = epi_row(row_base, v);
            if (row < nrows && col < ncols) s_out[(int64_t)row * d + col] = sp[v] + acc[v] + cu;
        }
    }
};

template <typename TC, int KU> __global__ __launch_bounds__(256) void k_fwd_up(FwdUpArgs<TC> a)
{
    __shared__ __attribute__((aligned(16))) char smem[tile_lds_bytes<TC, T64U<KU>>()];
    LoadRowsTC<TC, 64, KU> al;
    al.src = a.h; al.ld = a.r; al.nrows = a.M;
    LoadRowsTC<TC, 64, KU> bl;
    bl.src = a.WuT; bl.ld = a.r; bl.nrows = a.d;
    EpiFwdUp epi{a.c_up, a.s_prev, a.s_out, a.d};
    gemm_tile<TC, T64U<KU>>(smem, al, bl, epi, 0, a.r, blockIdx.x * 64, blockIdx.y * 64, a.M, a.d);
}

// pooled[s][j] = mean_t ( b_L[t][j] + s_L[t][j] )
template <typename TC>
__global__ __launch_bounds__(256) void k_pool(const TC *__restrict__ cache, RowMap map, int last_layer, int d,
                                              const float *__restrict__ s_last, const int32_t *samp_start,
                                              const int32_t *samp_len, float *__restrict__ pooled)
{
    const int s = blockIdx.x, j = blockIdx.y * 256 + threadIdx.x;
    if (j >= d) return;
    const int m0 = samp_start[s], len = samp_len[s];
    float acc = 0.f;
    for (int t = 0; t < len; ++t) {
        const int m = m0 + t;
        const TC *b = cache + map.rowoff[m] + (int64_t)last_layer * map.rowstride[m];
        acc += to_f32(b[j]) + s_last[(int64_t)m * d + j];
    }
    pooled[(int64_t)s * d + j] = acc / (float)len;
}

// logits, loss, dz = (softmax - onehot)/B.  One workgroup.
__global__ __launch_bounds__(256) void k_head(const float *__restrict__ pooled, const float *__restrict__ Wcls,
                                              const float *__restrict__ ccls, const int32_t *__restrict__ labels,
                                              int B, int d, int C, float *__restrict__ logits_ws,
                                              float *__restrict__ logits_out, float *__restrict__ dz,
                                              float *__restrict__ loss_out)
{
    __shared__ float z[kMaxBatch * kMaxClasses];
    __shared__ float red[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int pair = wave; pair < B * C; pair += 4) {
        const int s = pair / C, c = pair % C;
        float acc = 0.f;
        for (int j = lane; j < d; j += 64) acc += pooled[(int64_t)s * d + j] * Wcls[(int64_t)j * C + c];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) acc += __shfl_down(acc, o, 64);
        if (lane == 0) z[pair] = acc + ccls[c];
    }
    __syncthreads();
    float my = 0.f;
    if ((int)threadIdx.x < B) {
        const int s = threadIdx.x;
        float zmax = -INFINITY;
        for (int c = 0; c < C; ++c) zmax = fmaxf(zmax, z[s * C + c]);
        float se = 0.f;
        for (int c = 0; c < C; ++c) se += expf(z[s * C + c] - zmax);
        const float lse = zmax + logf(se);
        const int y = labels[s];
        my = (y >= 0 && y < C) ? lse - z[s * C + y] : NAN;
        for (int c = 0; c < C; ++c) {
            const float zz = z[s * C + c];
            logits_ws[s * C + c] = zz;
            if (logits_out) logits_out[s * C + c] = zz;
            dz[s * C + c] = (expf(zz - lse) - (c == y ? 1.f : 0.f)) / (float)B;
        }
    }
    const float tot = block_sum(my, red);
    if (threadIdx.x == 0) *loss_out = tot / (float)B;
}

// dW_cls, dc_cls, and ds_L[m][j] = (dz_s W_cls^T)[j] / len_s for every token row
__global__ __launch_bounds__(256) void k_head_bwd(const float *__restrict__ pooled, const float *__restrict__ Wcls,
                                                  const float *__restrict__ dz, int B, int M, int d, int C,
                                                  const int32_t *__restrict__ rowsamp,
                                                  const int32_t *__restrict__ samp_len, float *__restrict__ gWcls,
                                                  float *__restrict__ gccls, float *__restrict__ ds,
                                                  int rows_per_block)
{
    __shared__ float sdz[kMaxBatch * kMaxClasses];
    for (int i = threadIdx.x; i < B * C; i += 256) sdz[i] = dz[i];
    __syncthreads();
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (blockIdx.x == 0 && blockIdx.y == 0 && (int)threadIdx.x < C) {
        float acc = 0.f;
        for (int s = 0; s < B; ++s) acc += sdz[s * C + threadIdx.x];
        gccls[threadIdx.x] = acc;
    }
    if (j >= d) return;
    float w[kMaxClasses];
    for (int c = 0; c < C; ++c) w[c] = Wcls[(int64_t)j * C + c];
    if (blockIdx.y == 0) {
        for (int c = 0; c < C; ++c) {
            float acc = 0.f;
            for (int s = 0; s < B; ++s) acc += pooled[(int64_t)s * d + j] * sdz[s * C + c];
            gWcls[(int64_t)j * C + c] = acc;
        }
    }
    const int m0 = blockIdx.y * rows_per_block;
    const int m1 = min(M, m0 + rows_per_block);
    int cur = -1;
    float val = 0.f;
    for (int m = m0; m < m1; ++m) {
        const int s = rowsamp[m];
        if (s != cur) {
            cur = s;
            float dp = 0.f;
            for (int c = 0; c < C; ++c) dp += sdz[s * C + c] * w[c];
            val = dp / (float)samp_len[s];
        }
        ds[(int64_t)m * d + j] = val;
    }
}

// ---------------------------------------------------------------------------
// backward, layer l
// ---------------------------------------------------------------------------
template <typename TC> struct BwdDpreArgs {
    const float *ds; // [M][d]
    const TC *Wu;    // [r][d]
    const float *pre;
    TC *dpre; // [M][r]
    int M, d, r;
};

template <typename TC> struct EpiDpre {
    static constexpr bool kBatched = true;
    const float *pre;
    TC *dpre;
    int r;
    __device__ void batch(int row_base, int col, const f32x16 &acc, int nrows, int ncols) const
    {
        const int cc = min(col, ncols - 1);
        float pv[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) pv[v] = pre[(int64_t)min(epi_row(row_base, v), nrows - 1) * r + cc];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = epi_row(row_base, v);
            if (row < nrows && col < ncols) dpre[(int64_t)row * r + col] = to_tc(acc[v] * gelu_grad_f(pv[v]), TC());
        }
    }
};

template <typename TC, int KU> __global__ __launch_bounds__(256) void k_bwd_dpre(BwdDpreArgs<TC> a)
{
    __shared__ __attribute__((aligned(16))) char smem[tile_lds_bytes<TC, T64U<KU>>()];
    LoadRowsF32<TC, 64, KU> al;
    al.src = a.ds; al.ld = a.d; al.nrows = a.M;
    LoadRowsTC<TC, 64, KU> bl;
    bl.src = a.Wu; bl.ld = a.d; bl.nrows = a.r;
    EpiDpre<TC> epi{a.pre, a.dpre, a.r};
    gemm_tile<TC, T64U<KU>>(smem, al, bl, epi, 0, a.d, blockIdx.x * 64, blockIdx.y * 64, a.M, a.r);
}

// Top layer: ds_L is the same vector for every token of a sample (dp_s / len_s), so
// dh_L = ds_L W_up^{LT} is computed once per sample in fp32 instead of through the matrix cores
// (rounding that vector to bf16 would put the same error on every token of the sample).
__global__ __launch_bounds__(256) void k_dh_top(const float *__restrict__ dz, const float *__restrict__ Wcls,
                                                const float *__restrict__ Wu /* [r][d] fp32 */,
                                                const int32_t *__restrict__ samp_len, int B, int d, int r, int C,
                                                float *__restrict__ dh /* [B][r] */)
{
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (row >= B * r) return;
    const int s = row / r, k = row % r;
    float acc = 0.f;
    for (int j = lane; j < d; j += 64) {
        float dp = 0.f;
        for (int c = 0; c < C; ++c) dp += dz[s * C + c] * Wcls[(int64_t)j * C + c];
        acc += dp * Wu[(int64_t)k * d + j];
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_down(acc, o, 64);
    if (lane == 0) dh[row] = acc / (float)samp_len[s];
}

template <typename TC>
__global__ __launch_bounds__(256) void k_dpre_top(const float *__restrict__ dh, const float *__restrict__ pre,
                                                  const int32_t *__restrict__ rowsamp, int M, int r,
                                                  TC *__restrict__ dpre)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)M * r) return;
    const int m = (int)(idx / r), k = (int)(idx % r);
    dpre[idx] = to_tc(dh[rowsamp[m] * r + k] * gelu_grad_f(pre[idx]), TC());
}

// Token reductions.  blockIdx.z = 0: dW_up[r][d] = h^T ds, dc_up = colsum(ds);
//                    blockIdx.z = 1: dW_down[d][r] = x^T dpre, dc_down = colsum(dpre).
// blockIdx.y = split over token rows; results go to part[split] in the layer-block layout.
template <typename TC> struct BwdWgradArgs {
    const TC *cache;
    RowMap map;
    int layer, d, r;
    const float *s_prev;
    const float *lam;
    const TC *h;     // [M][r]
    const float *ds; // [M][d]
    const TC *dpre;  // [M][r]
    float *part;     // [splits][PL]
    int64_t PL;
    int rows_per_split; // multiple of the K step
};

struct EpiStore {
    float *out;
    int ld;
    __device__ void operator()(int row, int col, float v) const { out[(int64_t)row * ld + col] = v; }
};

template <typename TC, class BL>
__device__ __forceinline__ void write_colsums(BL &bl, float *red /* 256 * CE floats of LDS */, float *dst,
                                              int ncols, int j0)
{
    // every thread owns the CE columns of i-block (t % IB); sum over the threads that share them
    using G = ColsGeom<TC, 64, 4>;
    __syncthreads();
    for (int e = 0; e < G::CE; ++e) red[threadIdx.x * G::CE + e] = bl.sums[e];
    __syncthreads();
    if ((int)threadIdx.x < 64) {
        const int col = threadIdx.x; // column within the tile
        const int blk = col / G::CE, e = col % G::CE;
        float acc = 0.f;
        for (int t = blk; t < kThreads; t += G::IB) acc += red[t * G::CE + e];
        if (j0 + col < ncols) dst[j0 + col] = acc;
    }
}

template <typename TC> __global__ __launch_bounds__(256) void k_bwd_wgrad(BwdWgradArgs<TC> a)
{
    __shared__ __attribute__((aligned(16))) char smem[tile_lds_bytes<TC, T64K>()];
    static_assert(tile_lds_bytes<TC, T64K>() >= 256 * 8 * 4, "column-sum scratch must fit");
    const int M = a.map.M;
    const int kbegin = blockIdx.y * a.rows_per_split;
    const int kend = min(M, kbegin + a.rows_per_split);
    float *part = a.part + (int64_t)blockIdx.y * a.PL;
    const int64_t dr = (int64_t)a.d * a.r;
    if (blockIdx.z == 0) {
        const int tj = a.d / 64 + (a.d % 64 ? 1 : 0);
        const int ti = blockIdx.x / tj, tjx = blockIdx.x % tj;
        LoadCols<TC, 64, 4, TC, false> al;
        al.src = a.h; al.ld = a.r; al.ncols = a.r; al.kend = kend;
        LoadCols<TC, 64, 4, float, true> bl;
        bl.src = a.ds; bl.ld = a.d; bl.ncols = a.d; bl.kend = kend;
        EpiStore epi{part + dr + a.r, a.d};
        gemm_tile<TC, T64K>(smem, al, bl, epi, kbegin, kend, ti * 64, tjx * 64, a.r, a.d);
        if (ti == 0) write_colsums<TC>(bl, reinterpret_cast<float *>(smem), part + 2 * dr + a.r, a.d, tjx * 64);
    } else {
        const int tj = a.r / 64 + (a.r % 64 ? 1 : 0);
        const int ti = blockIdx.x / tj, tjx = blockIdx.x % tj;
        LoadCols<TC, 64, 4, TC, true> bl;
        bl.src = a.dpre; bl.ld = a.r; bl.ncols = a.r; bl.kend = kend;
        EpiStore epi{part, a.r};
        if (a.s_prev) {
            LoadColsX<TC, 64, 4, true> al;
            al.cache = a.cache; al.map = a.map; al.layer = a.layer; al.s_prev = a.s_prev; al.ld_s = a.d;
            al.lam = *a.lam; al.ncols = a.d; al.kend = kend;
            gemm_tile<TC, T64K>(smem, al, bl, epi, kbegin, kend, ti * 64, tjx * 64, a.d, a.r);
        } else {
            LoadColsX<TC, 64, 4, false> al;
            al.cache = a.cache; al.map = a.map; al.layer = a.layer; al.s_prev = nullptr; al.ld_s = a.d;
            al.lam = *a.lam; al.ncols = a.d; al.kend = kend;
            gemm_tile<TC, T64K>(smem, al, bl, epi, kbegin, kend, ti * 64, tjx * 64, a.d, a.r);
        }
        if (ti == 0) write_colsums<TC>(bl, reinterpret_cast<float *>(smem), part + dr, a.r, tjx * 64);
    }
}

// dx = dpre W_down^T ; dlambda partial ; ds <- ds + (1 - lambda) dx   (in place)
template <typename TC> struct BwdDxArgs {
    const TC *dpre; // [M][r]
    const TC *Wd;   // [d][r]
    const TC *cache;
    RowMap map;
    int layer, d, r;
    const float *s_prev; // or null
    const float *lam;
    float *ds;        // [M][d] in/out
    float *dlam_part; // one per workgroup
};

template <typename TC> struct EpiDx {
    static constexpr bool kBatched = true;
    const TC *cache;
    RowMap map;
    int layer, d;
    const float *s_prev;
    float lam;
    float *ds;
    float dlam;
    __device__ void batch(int row_base, int col, const f32x16 &acc, int nrows, int ncols)
    {
        const int cc = min(col, ncols - 1);
        int64_t ro[16];
        int rs[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int rr = min(epi_row(row_base, v), nrows - 1);
            ro[v] = map.rowoff[rr];
            rs[v] = map.rowstride[rr];
        }
        float b[16], s[16], dsv[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int rr = min(epi_row(row_base, v), nrows - 1);
            const int64_t o = (int64_t)rr * d + cc;
            b[v] = to_f32(cache[ro[v] + (int64_t)layer * rs[v] + cc]);
            s[v] = s_prev ? s_prev[o] : 0.f;
            dsv[v] = ds[o];
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = epi_row(row_base, v);
            if (row < nrows && col < ncols) {
                dlam += (b[v] - s[v]) * acc[v];
                ds[(int64_t)row * d + col] = dsv[v] + (1.f - lam) * acc[v];
            }
        }
    }
};

template <typename TC, int KU> __global__ __launch_bounds__(256) void k_bwd_dx(BwdDxArgs<TC> a)
{
    __shared__ __attribute__((aligned(16))) char smem[tile_lds_bytes<TC, T64U<KU>>()];
    __shared__ float red[4];
    LoadRowsTC<TC, 64, KU> al;
    al.src = a.dpre; al.ld = a.r; al.nrows = a.map.M;
    LoadRowsTC<TC, 64, KU> bl;
    bl.src = a.Wd; bl.ld = a.r; bl.nrows = a.d;
    EpiDx<TC> epi{a.cache, a.map, a.layer, a.d, a.s_prev, *a.lam, a.ds, 0.f};
    gemm_tile<TC, T64U<KU>>(smem, al, bl, epi, 0, a.r, blockIdx.x * 64, blockIdx.y * 64, a.map.M, a.d);
    const float tot = block_sum(epi.dlam, red);
    if (threadIdx.x == 0) a.dlam_part[blockIdx.y * gridDim.x + blockIdx.x] = tot;
}

// grads of one layer = ordered sum of the split partials; dlambda = ordered sum of the dx partials
__global__ __launch_bounds__(256) void k_reduce_layer(const float *__restrict__ part, int splits, int64_t PL,
                                                      const float *__restrict__ dlam_part, int nslots,
                                                      float *__restrict__ g_layer)
{
    __shared__ float red[256];
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < PL - 1) {
        float acc = 0.f;
        for (int s = 0; s < splits; ++s) acc += part[(int64_t)s * PL + i];
        g_layer[i] = acc;
    }
    if ((int64_t)blockIdx.x == (PL - 1) / 256) {
        // the gate: the workgroup that owns it sums the dx partials, each thread a strided share in
        // slot order, the 256 shares combined in a fixed tree
        float acc = 0.f;
        for (int s0 = threadIdx.x; s0 < nslots; s0 += 256 * 8) {
            float p[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) p[u] = dlam_part[min(s0 + 256 * u, nslots - 1)];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (s0 + 256 * u < nslots) acc += p[u];
        }
        red[threadIdx.x] = acc;
        __syncthreads();
        for (int w = 128; w > 0; w >>= 1) {
            if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
            __syncthreads();
        }
        if (threadIdx.x == 0) g_layer[PL - 1] = red[0];
    }
}

// ---------------------------------------------------------------------------
// AdamW over the flat parameter vector
// ---------------------------------------------------------------------------
// One element of the update: element o of layer `layer`'s block (layer < L), or element o of the head
// (layer == L).  When the loss / gate-gradient sums were left to this launch (fin.used), the thread that
// owns a gate first sums that layer's partials in slot order.
// The kernel is a plain stream of 28 bytes per parameter, so the arithmetic has to stay well below the time the
// bytes take: the bias corrections arrive as reciprocals and the root and the quotient use the hardware's
// single-instruction forms (1 ulp each; the update they scale is lr-sized, so the parameter moves by less than
// 1e-9 of its own size against the correctly rounded forms).
__device__ __forceinline__ void adamw_elem(int layer, int64_t o, int L, float &pi, float &mi, float &vi, float &gi,
                                           int64_t PL, int64_t dr, int r, int64_t dC, const AdamArgs &a,
                                           const Deferred &fin)
{
    bool decayed;
    if (layer < L) {
        decayed = (o < dr) || (o >= dr + r && o < 2 * dr + r);
        if (fin.used && o == PL - 1) {
            const float *part = fin.dlam_part + (int64_t)layer * fin.slots;
            float acc = 0.f;
            for (int s = 0; s < fin.slots; ++s) acc += part[s];
            gi = acc;
        }
    } else {
        decayed = o < dC;
    }
    mi = a.beta1 * mi + (1.f - a.beta1) * gi;
    vi = a.beta2 * vi + (1.f - a.beta2) * gi * gi;
    if (decayed) pi -= a.lr * a.wd * pi;
    pi -= a.lr * (mi * a.inv_bc1) * __frcp_rn(__fsqrt_rn(vi * a.inv_bc2) + a.eps);
}

// VEC = 4: 16-byte accesses (all four arrays 16-byte aligned), the tail element by element.
// The position of a group's first element inside its layer block comes from a reciprocal multiplication with
// a correction step (exact for parameter counts below 2^31; one 64-bit division otherwise).
template <int VEC>
__global__ __launch_bounds__(256) void k_adamw(float *__restrict__ p, float *__restrict__ m, float *__restrict__ v,
                                               float *__restrict__ g, int64_t P, int64_t PL, int L, int d,
                                               int r, int C, AdamArgs a, Deferred fin)
{
    const int64_t dr = (int64_t)d * r;
    const int64_t head = (int64_t)L * PL, dC = (int64_t)d * C;
    if (fin.used && blockIdx.x == 0 && threadIdx.x == 0) {
        float tot = 0.f;
        for (int s = 0; s < fin.B; ++s) tot += fin.loss_part[s];
        *fin.loss_out = tot / (float)fin.B;
    }
    const bool small = P < (int64_t(1) << 31);
    const float inv_PL = 1.f / (float)PL;
    const int64_t ngroups = (P + VEC - 1) / VEC;
    for (int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x; q < ngroups; q += (int64_t)gridDim.x * 256) {
        const int64_t i0 = q * VEC;
        int layer;
        int64_t o;
        if (i0 >= head) {
            layer = L;
            o = i0 - head;
        } else if (small) {
            // the estimate is off by at most one: |error of (float)i0| <= 128 < PL (a layer block holds at least
            // 2 * 32 * 32 elements); the difference is formed modulo 2^32 and is small
            layer = (int)((float)i0 * inv_PL);
            int oo = (int)((uint32_t)i0 - (uint32_t)layer * (uint32_t)PL);
            if (oo < 0) { oo += (int)PL; --layer; }
            if (oo >= (int)PL) { oo -= (int)PL; ++layer; }
            o = oo;
        } else {
            layer = (int)(i0 / PL);
            o = i0 - (int64_t)layer * PL;
        }
        auto step = [&]() { // to the next element
            ++o;
            if (layer < L && o == PL) {
                o = 0;
                ++layer;
            }
        };
        if (VEC == 4 && i0 + 3 < P) {
            f32x4 pv = *reinterpret_cast<const f32x4 *>(p + i0), mv = *reinterpret_cast<const f32x4 *>(m + i0);
            f32x4 vv = *reinterpret_cast<const f32x4 *>(v + i0), gv = *reinterpret_cast<const f32x4 *>(g + i0);
            const f32x4 g_in = gv;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float pi = pv[e], mi = mv[e], vi = vv[e], gi = gv[e];
                adamw_elem(layer, o, L, pi, mi, vi, gi, PL, dr, r, dC, a, fin);
                pv[e] = pi; mv[e] = mi; vv[e] = vi; gv[e] = gi;
                step();
            }
            *reinterpret_cast<f32x4 *>(p + i0) = pv;
            *reinterpret_cast<f32x4 *>(m + i0) = mv;
            *reinterpret_cast<f32x4 *>(v + i0) = vv;
            if (fin.used && (gv[0] != g_in[0] || gv[1] != g_in[1] || gv[2] != g_in[2] || gv[3] != g_in[3]))
                *reinterpret_cast<f32x4 *>(g + i0) = gv; // a gate gradient was summed here: keep it
        } else {
            for (int64_t i = i0; i < P && i < i0 + VEC; ++i) {
                float pi = p[i], mi = m[i], vi = v[i], gi = g[i];
                const float g_in = gi;
                adamw_elem(layer, o, L, pi, mi, vi, gi, PL, dr, r, dC, a, fin);
                p[i] = pi; m[i] = mi; v[i] = vi;
                if (gi != g_in) g[i] = gi;
                step();
            }
        }
    }
}

hipError_t launch_adamw(const Dims &D, float *p, float *m, float *v, float *g, const AdamArgs &a, hipStream_t st,
                        Profiler *prof, const Deferred *fin)
{
    const Deferred f = fin ? *fin : Deferred();
    const bool vec = ((reinterpret_cast<uintptr_t>(p) | reinterpret_cast<uintptr_t>(m) | reinterpret_cast<uintptr_t>(v) |
                       reinterpret_cast<uintptr_t>(g)) & 15) == 0;
    // one 16-byte group per thread and as many workgroups as that takes: measured on the four-reads-three-writes
    // mix of this kernel, 4096 workgroups walking the vector in strides sustain 4.55 TB/s, one group per thread
    // 5.3 TB/s (the loop is kept for vectors beyond the grid limit)
    int64_t nb = (((D.P + (vec ? 3 : 0)) / (vec ? 4 : 1)) + 255) / 256;
    if (nb > (int64_t)1 << 22) nb = (int64_t)1 << 22;
    const int blocks = (int)nb;
    if (vec)
        PAC_LAUNCH(prof, st, KC_ADAMW, k_adamw<4>, dim3(blocks), dim3(256), 0, st, p, m, v, g, D.P, D.PL, D.L, D.d, D.r, D.C, a, f);
    else
        PAC_LAUNCH(prof, st, KC_ADAMW, k_adamw<1>, dim3(blocks), dim3(256), 0, st, p, m, v, g, D.P, D.PL, D.L, D.d, D.r, D.C, a, f);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// one batch: forward, loss, (optionally) backward
// ---------------------------------------------------------------------------
template <typename TC>
static hipError_t run_loss_grad(const Dims &D, const WsLayout &W, const BatchMeta &meta, const StepIO &io)
{
    hipStream_t st = io.stream;
    Profiler *prof = io.prof;
    char *ws = io.ws;
    const int M = meta.M, d = D.d, r = D.r, L = D.L;
    int64_t *rowoff = (int64_t *)(ws + W.rowoff);
    int32_t *rowstride = (int32_t *)(ws + W.rowstride);
    int32_t *rowsamp = (int32_t *)(ws + W.rowsamp);
    int32_t *samp_start = (int32_t *)(ws + W.samp_start);
    int32_t *samp_len = (int32_t *)(ws + W.samp_len);
    TC *Wd = (TC *)(ws + W.Wd), *WdT = (TC *)(ws + W.WdT), *Wu = (TC *)(ws + W.Wu), *WuT = (TC *)(ws + W.WuT);
    float *s_all = (float *)(ws + W.s_all);
    float *pre_all = (float *)(ws + W.pre_all);
    TC *h_all = (TC *)(ws + W.h_all);
    float *ds = (float *)(ws + W.ds);
    TC *dpre = (TC *)(ws + W.dpre);
    float *pooled = (float *)(ws + W.pooled);
    float *logits = (float *)(ws + W.logits);
    float *dz = (float *)(ws + W.dz);
    float *part = (float *)(ws + W.part);
    float *dlam_part = (float *)(ws + W.dlam_part);
    const TC *cache = (const TC *)io.cache;
    const float *params = io.params;
    const int64_t PL = D.PL, dr = (int64_t)d * r;
    const RowMap map{rowoff, rowstride, M};
    const int64_t Md = (int64_t)M * d, Mr = (int64_t)M * r;

    PAC_LAUNCH(prof, st, KC_SETUP, k_setup, dim3(cdiv(M, 256)), dim3(256), 0, st, meta, d, rowoff, rowstride, rowsamp,
                       samp_start, samp_len);
    PAC_LAUNCH(prof, st, KC_SHADOWS, (k_shadows<TC>), dim3((d / 32) * (r / 32), L, 2), dim3(256), 0, st, params, PL, d, r, Wd,
                       WdT, Wu, WuT);

    const dim3 g_rows_r(cdiv(M, 64), cdiv(r, 64)), g_rows_d(cdiv(M, 64), cdiv(d, 64));
    // long K steps where the contraction length allows them
    const bool wide_d = d % Stage<TC, 4>::BK == 0, wide_r = r % Stage<TC, 4>::BK == 0;
    for (int l = 0; l < L; ++l) {
        const float *pl = params + (int64_t)l * PL;
        const float *s_prev = l == 0 ? nullptr : s_all + (int64_t)(l - 1) * Md;
        FwdDownArgs<TC> fa{cache, map, l, d, r, s_prev, WdT + (int64_t)l * dr, pl + dr, pl + PL - 1,
                           pre_all + (int64_t)l * Mr, h_all + (int64_t)l * Mr};
        if (wide_d) PAC_LAUNCH(prof, st, KC_FWD_DOWN, (k_fwd_down<TC, 4>), g_rows_r, dim3(256), 0, st, fa);
        else PAC_LAUNCH(prof, st, KC_FWD_DOWN, (k_fwd_down<TC, 1>), g_rows_r, dim3(256), 0, st, fa);
        FwdUpArgs<TC> fu{h_all + (int64_t)l * Mr, WuT + (int64_t)l * dr, pl + 2 * dr + r, s_prev,
                         s_all + (int64_t)l * Md, M, d, r};
        if (wide_r) PAC_LAUNCH(prof, st, KC_FWD_UP, (k_fwd_up<TC, 4>), g_rows_d, dim3(256), 0, st, fu);
        else PAC_LAUNCH(prof, st, KC_FWD_UP, (k_fwd_up<TC, 1>), g_rows_d, dim3(256), 0, st, fu);
    }
    PAC_LAUNCH(prof, st, KC_POOL, (k_pool<TC>), dim3(meta.B, cdiv(d, 256)), dim3(256), 0, st, cache, map, L - 1, d,
                       s_all + (int64_t)(L - 1) * Md, samp_start, samp_len, pooled);
    const float *Wcls = params + (int64_t)L * PL;
    const float *ccls = Wcls + (int64_t)d * D.C;
    PAC_LAUNCH(prof, st, KC_HEAD, k_head, dim3(1), dim3(256), 0, st, pooled, Wcls, ccls, io.labels, meta.B, d, D.C, logits,
                       io.logits_out, dz, io.loss_out);
    PAC_HIP_TRY(hipGetLastError());
    if (!io.grads) return hipSuccess;

    float *grads = io.grads;
    const int rows_per_block = 64;
    PAC_LAUNCH(prof, st, KC_HEAD_BWD, k_head_bwd, dim3(cdiv(d, 256), cdiv(M, rows_per_block)), dim3(256), 0, st, pooled, Wcls, dz,
                       meta.B, M, d, D.C, rowsamp, samp_len, grads + (int64_t)L * PL,
                       grads + (int64_t)L * PL + (int64_t)d * D.C, ds, rows_per_block);

    const int kstep = Stage<TC, 4>::BK;
    int splits = W.splits;
    int rows_per_split = cdiv(cdiv(M, splits), kstep) * kstep;
    splits = cdiv(M, rows_per_split);
    const int wg_tiles = cdiv(r, 64) * cdiv(d, 64);
    for (int l = L - 1; l >= 0; --l) {
        const float *pl = params + (int64_t)l * PL;
        const float *s_prev = l == 0 ? nullptr : s_all + (int64_t)(l - 1) * Md;
        if (l == L - 1) {
            float *dh_top = dlam_part; // B*r floats; the dx kernel overwrites it afterwards
            PAC_LAUNCH(prof, st, KC_BWD_DPRE, k_dh_top, dim3(cdiv((int64_t)meta.B * r, 4)), dim3(256), 0, st, dz, Wcls,
                       pl + dr + r, samp_len, meta.B, d, r, D.C, dh_top);
            PAC_LAUNCH(prof, st, KC_BWD_DPRE, (k_dpre_top<TC>), dim3(cdiv(Mr, 256)), dim3(256), 0, st, dh_top,
                       pre_all + (int64_t)l * Mr, rowsamp, M, r, dpre);
        } else {
            BwdDpreArgs<TC> ba{ds, Wu + (int64_t)l * dr, pre_all + (int64_t)l * Mr, dpre, M, d, r};
            if (wide_d) PAC_LAUNCH(prof, st, KC_BWD_DPRE, (k_bwd_dpre<TC, 4>), g_rows_r, dim3(256), 0, st, ba);
            else PAC_LAUNCH(prof, st, KC_BWD_DPRE, (k_bwd_dpre<TC, 1>), g_rows_r, dim3(256), 0, st, ba);
        }
        BwdWgradArgs<TC> wa{cache, map, l, d, r, s_prev, pl + PL - 1, h_all + (int64_t)l * Mr, ds, dpre, part, PL,
                            rows_per_split};
        PAC_LAUNCH(prof, st, KC_BWD_WGRAD, (k_bwd_wgrad<TC>), dim3(wg_tiles, splits, 2), dim3(256), 0, st, wa);
        BwdDxArgs<TC> xa{dpre, Wd + (int64_t)l * dr, cache, map, l, d, r, s_prev, pl + PL - 1, ds, dlam_part};
        if (wide_r) PAC_LAUNCH(prof, st, KC_BWD_DX, (k_bwd_dx<TC, 4>), g_rows_d, dim3(256), 0, st, xa);
        else PAC_LAUNCH(prof, st, KC_BWD_DX, (k_bwd_dx<TC, 1>), g_rows_d, dim3(256), 0, st, xa);
        PAC_LAUNCH(prof, st, KC_REDUCE, k_reduce_layer, dim3(cdiv(PL, 256)), dim3(256), 0, st, part, splits, PL, dlam_part,
                           (int)(g_rows_d.x * g_rows_d.y), grads + (int64_t)l * PL);
    }
    return hipGetLastError();
}

hipError_t launch_loss_grad(const Dims &D, const WsLayout &W, const BatchMeta &meta, const StepIO &io)
{
    if (W.use_gram) return launch_gram_loss_grad(D, W, meta, io);
    if (D.cache_dtype == 0) return run_loss_grad<bf16_t>(D, W, meta, io);
    return run_loss_grad<float>(D, W, meta, io);
}

} // namespace pac
