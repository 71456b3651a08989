// The paper's default Parallel-Adapter architecture trained from the activation cache (Sec. 4.1 and
// Fig. "pa-detail", Sec. 6.1; cached phase Sec. 4.2 / 5.2): the w-wide ladder whose adapter is a reduced
// transformer layer.  C ABI in include/pac_ladder.h.
//
//   u_l = b_l W_down^l + c_down^l            (one batched launch streams the cache once: u does not depend on the ladder)
//   x_l = lambda_l u_l + (1 - lambda_l) a_{l-1}
//   a_l = Block_l(x_l): xn = LN1(x); q,k,v = xn W_qkv + b_qkv; o = softmax(q k^T / sqrt(dh)) v per sample and head;
//                       t = x + o W_o + b_o; tn = LN2(t); a = t + GELU(tn W_1 + b_1) W_2 + b_2
//   y = b_L + a_L W_up + c_up;  mean over the valid tokens;  classifier;  mean cross-entropy
//
// Launch plan of a gradient call (fp32 arithmetic throughout, fp32 matrix instructions through pac_gemm.h):
//   set-up -> down-projection of every layer (first pass over the cache slice)
//   per layer, forward : gate + LN1, qkv, attention, output projection (+x), LN2, FFN in (+GELU), FFN out (+t)
//   head               : token means, logits, loss, dz, the head's gradients, da_L
//   per layer, backward: FFN out^T (x GELU'), FFN in^T, LN2^T (+da), output projection^T, attention^T, qkv^T,
//                        LN1^T + gate^T (+dt, gate gradient partials, da_{l-1})
//   all token contractions of all layers in ONE launch (second pass over the cache slice for dW_down; the bias
//   gradients are the column sums its right-hand loaders keep), then one ordered reduction into the gradient.
// Every intermediate the reverse pass needs is kept in the workspace; every reduction runs in a fixed order.
#include "../../include/pac_ladder.h"
#include "pac_mma.h"
#include "pac_internal.h"

#include <cmath>
#include <mutex>

namespace pac {
namespace {

#define LAD_LAUNCH(prof, st, cls, ...)                   \
    do {                                                 \
        if (prof) (void)(prof)->mark((st), (cls), true);  \
        hipLaunchKernelGGL(__VA_ARGS__);                 \
        if (prof) (void)(prof)->mark((st), (cls), false); \
    } while (0)

#define LAD_TRY(expr)                    \
    do {                                 \
        hipError_t e_ = (expr);          \
        if (e_ != hipSuccess) return e_; \
    } while (0)

inline int64_t al256(int64_t x) { return (x + 255) & ~int64_t(255); }
inline int cdivi(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

using TL = Tile<2, 2, 1, 1, 4, 2>; // 64 x 64 workgroup tile, 64 fp32 values of K per step, two steps in flight
constexpr int kTileLds = tile_lds_bytes<float, TL>();
constexpr int kLnRows = 16;    // token rows per workgroup of the LayerNorm reverse kernels (four per wavefront)
constexpr int kFields = 15;    // tensors of one layer block

// Shapes, parameter offsets (elements) and workspace offsets (bytes).
struct Lad {
    int L, d, w, f, nh, dh, C, Bmax, cache_f32;
    int64_t Mmax;
    int64_t fo[kFields + 1]; // start of each field inside a layer block; fo[kFields] = block length
    int64_t PLb, oWup, ocup, oWcls, occls, P;
    // workspace
    int64_t rowoff, rowstride, rowsamp, samp_start, samp_len;
    int64_t U, X, XN, QKV, LSE, O, T, TN, F1, G, A, st1, st2;  // [L][Mmax][...]
    int64_t DA, DF1, DT, DQKV, DX;                             // [L][Mmax][...]
    int64_t DTN, DO_, DXN;                                     // [Mmax][w]
    int64_t WT;                                                // [L][2 w f + 4 w w]: W_2^T, W_1^T, W_o^T, W_qkv^T
    int64_t Wsp;                                               // [L][3][w][d] bf16: W_down^T as three bf16 terms, or -1
    int64_t ln1p, ln2p, dlamp;                                 // [L][nblk][2][w] x2, [L][nblk]
    int64_t bmean, abar, pooled, logits, dz, dp, daL, lossp;
    int64_t part;                                              // [splits][L * PLb]
    int64_t grads;
    int64_t total;
    int nblk, splits, rows_per_split;
    int items_per_layer, tiles[5][2], item0[6];
};
enum Field { F_WD = 0, F_CD, F_G1, F_H1, F_WQKV, F_BQKV, F_WO, F_BO, F_G2, F_H2, F_W1, F_B1, F_W2, F_B2, F_LAM };

// the parameter vector (does not depend on the head count)
bool lad_shapes(const Dims &D, Lad &a)
{
    a.L = D.L; a.d = D.d; a.w = D.r; a.f = 4 * D.r; a.C = D.C; a.Bmax = D.B_max; a.Mmax = D.Mmax;
    a.cache_f32 = D.cache_dtype != 0;
    if (a.w % 32 || a.w > 256) return false;
    const int64_t w = a.w, d = a.d, f = a.f;
    const int64_t n[kFields] = {d * w, w, w, w, w * 3 * w, 3 * w, w * w, w, w, w, w * f, f, f * w, w, 4};
    a.fo[0] = 0;
    for (int i = 0; i < kFields; ++i) a.fo[i + 1] = a.fo[i] + n[i];
    a.PLb = a.fo[kFields];
    a.oWup = (int64_t)a.L * a.PLb;
    a.ocup = a.oWup + w * d;
    a.oWcls = a.ocup + d;
    a.occls = a.oWcls + d * a.C;
    a.P = a.occls + a.C;
    return true;
}

bool lad_plan(const Dims &D, int heads, Lad &a)
{
    if (!lad_shapes(D, a)) return false;
    a.nh = heads;
    if (heads < 1 || a.w % heads) return false;
    a.dh = a.w / heads;
    if (a.dh != 4 && a.dh != 8 && a.dh != 16 && a.dh != 32 && a.dh != 64) return false;
    if ((int64_t)D.n_max * a.dh > 8192) return false;
    const int64_t w = a.w, d = a.d, f = a.f;
    int64_t o = 0;
    auto take = [&](int64_t bytes) { int64_t at = o; o = al256(o + bytes); return at; };
    const int64_t M = a.Mmax, LM = (int64_t)a.L * M;
    a.rowoff = take(M * 8); a.rowstride = take(M * 4); a.rowsamp = take(M * 4);
    a.samp_start = take((kMaxBatch + 1) * 4); a.samp_len = take(kMaxBatch * 4);
    a.U = take(LM * w * 4); a.X = take(LM * w * 4); a.XN = take(LM * w * 4); a.QKV = take(LM * 3 * w * 4);
    a.LSE = take(LM * a.nh * 4); a.O = take(LM * w * 4); a.T = take(LM * w * 4); a.TN = take(LM * w * 4);
    a.F1 = take(LM * f * 4); a.G = take(LM * f * 4); a.A = take(LM * w * 4);
    a.st1 = take(LM * 2 * 4); a.st2 = take(LM * 2 * 4);
    a.DA = take(LM * w * 4); a.DF1 = take(LM * f * 4); a.DT = take(LM * w * 4); a.DQKV = take(LM * 3 * w * 4);
    a.DX = take(LM * w * 4);
    a.DTN = take(M * w * 4); a.DO_ = take(M * w * 4); a.DXN = take(M * w * 4);
    a.WT = take((int64_t)a.L * (2 * w * f + 4 * w * w) * 4); // transposed copies for the fused reverse kernels
    a.Wsp = (!a.cache_f32 && w <= 128 && d % 32 == 0) ? take((int64_t)a.L * 3 * w * d * 2) : -1; // see k_ldown3
    a.nblk = cdivi(M, kLnRows);
    a.ln1p = take((int64_t)a.L * a.nblk * 2 * w * 4); a.ln2p = take((int64_t)a.L * a.nblk * 2 * w * 4);
    a.dlamp = take((int64_t)a.L * a.nblk * 4);
    a.bmean = take((int64_t)a.Bmax * d * 4); a.abar = take((int64_t)a.Bmax * w * 4);
    a.pooled = take((int64_t)a.Bmax * d * 4); a.logits = take((int64_t)a.Bmax * a.C * 4);
    a.dz = take((int64_t)a.Bmax * a.C * 4); a.dp = take((int64_t)a.Bmax * d * 4);
    a.daL = take((int64_t)a.Bmax * w * 4); a.lossp = take((int64_t)a.Bmax * 4);
    // tiles of the five token contractions of one layer: W_down [d][w], W_qkv [w][3w], W_o [w][w], W_1 [w][f], W_2 [f][w]
    const int rows[5] = {a.d, a.w, a.w, a.w, a.f}, cols[5] = {a.w, 3 * a.w, a.w, a.f, a.w};
    a.item0[0] = 0;
    for (int t = 0; t < 5; ++t) {
        a.tiles[t][0] = cdivi(rows[t], 64);
        a.tiles[t][1] = cdivi(cols[t], 64);
        a.item0[t + 1] = a.item0[t] + a.tiles[t][0] * a.tiles[t][1];
    }
    a.items_per_layer = a.item0[5];
    int s = cdivi(1024, (int64_t)a.items_per_layer * a.L);
    const int by_rows = cdivi(M, 256);
    if (s > by_rows) s = by_rows;
    if (s > 16) s = 16;
    if (s < 1) s = 1;
    a.rows_per_split = cdivi(cdivi(M, s), 64) * 64;
    a.splits = cdivi(M, a.rows_per_split);
    a.part = take((int64_t)a.splits * a.L * a.PLb * 4);
    a.grads = take(a.P * 4);
    a.total = o;
    return true;
}

// ---------------------------------------------------------------------------
// set-up: sample ids -> per-token-row cache addresses
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_lsetup(BatchMeta meta, int d, int64_t *rowoff, int32_t *rowstride,
                                                int32_t *rowsamp, int32_t *samp_start, int32_t *samp_len)
{
    const int m = blockIdx.x * 256 + threadIdx.x;
    if (blockIdx.x == 0 && (int)threadIdx.x <= meta.B) {
        samp_start[threadIdx.x] = meta.tok_start[threadIdx.x];
        if ((int)threadIdx.x < meta.B) samp_len[threadIdx.x] = meta.len[threadIdx.x];
    }
    if (m >= meta.M) return;
    int s = 0;
    while (s + 1 < meta.B && meta.tok_start[s + 1] <= m) ++s;
    rowoff[m] = meta.off[s] + (int64_t)(m - meta.tok_start[s]) * d;
    rowstride[m] = meta.len[s] * d;
    rowsamp[m] = s;
}

// ---------------------------------------------------------------------------
// Cache operands of the fp32 tiles: four consecutive elements of the cache dtype, widened exactly.
// ---------------------------------------------------------------------------
template <typename SRC> struct Raw4;
template <> struct Raw4<float> {
    typedef u32x4 type;
    static __device__ __forceinline__ void widen(const type &r, float (&f)[4])
    {
#pragma unroll
        for (int e = 0; e < 4; ++e) f[e] = __uint_as_float(r[e]);
    }
};
template <> struct Raw4<bf16_t> {
    typedef uint2 type;
    static __device__ __forceinline__ void widen(const type &r, float (&f)[4])
    {
        f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xffff0000u);
        f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xffff0000u);
    }
};

// operand[row][k] = b_layer[row][k]   (token rows of the batch, K = hidden index)
template <typename SRC, int ROWS, int KU> struct LoadRowsCache {
    static constexpr bool kSwizzled = false;
    using S = Stage<float, KU>;
    using G = RowsGeom<float, ROWS, KU>;
    using R = typename Raw4<SRC>::type;
    const SRC *cache;
    RowMap map;
    int layer, klim;
    const SRC *bp[G::NCH];
    bool ok[G::NCH];
    int kpos[2];
    R reg[2][G::NCH];
    __device__ void init(int row0)
    {
        const int t = threadIdx.x;
#pragma unroll
        for (int u = 0; u < G::NCH; ++u) {
            const int c = t + kThreads * u;
            const int row = row0 + c / S::CPK;
            ok[u] = c < G::TOTAL && row < map.M;
            const int rowc = ok[u] ? row : 0;
            bp[u] = cache + map.rowoff[rowc] + (int64_t)layer * map.rowstride[rowc] + (c % S::CPK) * 4;
        }
    }
    template <int SLOT> __device__ void fetch(int k0)
    {
        kpos[SLOT] = k0;
        const int t = threadIdx.x;
#pragma unroll
        for (int u = 0; u < G::NCH; ++u) {
            const int kc = ((t + kThreads * u) % S::CPK) * 4;
            // chunks past the end of the row re-read its start (and are stored as zeros)
            reg[SLOT][u] = *reinterpret_cast<const R *>(bp[u] + (k0 + kc < klim ? k0 : -kc));
        }
    }
    template <int SLOT> __device__ void store(float *lds, bool)
    {
        const int t = threadIdx.x;
#pragma unroll
        for (int u = 0; u < G::NCH; ++u) {
            const int c = t + kThreads * u;
            const bool keep = ok[u] && kpos[SLOT] + (c % S::CPK) * 4 < klim;
            float f[4];
            Raw4<SRC>::widen(reg[SLOT][u], f);
            const f32x4 v = {keep ? f[0] : 0.f, keep ? f[1] : 0.f, keep ? f[2] : 0.f, keep ? f[3] : 0.f};
            if (c < G::TOTAL) *reinterpret_cast<f32x4 *>(lds + (c / S::CPK) * S::LDP + (c % S::CPK) * 4) = v;
        }
    }
};

// operand[i][k] = b_layer[k][i]   (K = token row: the contraction over the tokens)
template <typename SRC, int ROWS, int KU> struct LoadColsCache {
    static constexpr bool kSwizzled = ColsSwizzle<float, KU>::value;
    using S = Stage<float, KU>;
    using G = ColsGeom<float, ROWS, KU>;
    using R = typename Raw4<SRC>::type;
    const SRC *cache;
    RowMap map;
    int layer, ncols, kend, i0;
    int kpos[2];
    R reg[2][G::NCH][4];
    __device__ void init(int i0_) { i0 = i0_; }
    template <int SLOT> __device__ void fetch(int k0)
    {
        kpos[SLOT] = k0;
        const int t = threadIdx.x;
#pragma unroll
        for (int u = 0; u < G::NCH; ++u) {
            const int c = (t + kThreads * u) % G::TOTAL;
            const int i = min(i0 + (c % G::IB) * 4, ncols - 4);
            const int kb = k0 + (c / G::IB) * 4;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const int k = min(kb + kk, kend - 1);
                reg[SLOT][u][kk] = *reinterpret_cast<const R *>(cache + map.rowoff[k] + (int64_t)layer * map.rowstride[k] + i);
            }
        }
    }
    template <int SLOT> __device__ void store(float *lds, bool)
    {
        const int t = threadIdx.x;
#pragma unroll
        for (int u = 0; u < G::NCH; ++u) {
            const int c = t + kThreads * u;
            const bool icol = i0 + (c % G::IB) * 4 < ncols;
            const int kb = kpos[SLOT] + (c / G::IB) * 4;
            Chunk<float> blk[4];
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const bool keep = icol && kb + kk < kend && c < G::TOTAL;
                float f[4];
                Raw4<SRC>::widen(reg[SLOT][u][kk], f);
#pragma unroll
                for (int e = 0; e < 4; ++e) blk[kk].e[e] = keep ? f[e] : 0.f;
            }
            if (c < G::TOTAL) cols_store_block<float, ROWS, KU>(lds, c, blk);
        }
    }
};

__device__ __forceinline__ float lgelu(float u) { return 0.5f * u * (1.f + erff(u * 0.70710678118654752f)); }
__device__ __forceinline__ float lgelu_grad(float u)
{
    const float Phi = 0.5f * (1.f + erff(u * 0.70710678118654752f));
    return Phi + u * 0.3989422804014327f * expf(-0.5f * u * u);
}

// ---------------------------------------------------------------------------
// u_l = b_l W_down^l + c_down^l for every layer (grid.z = layer)
// ---------------------------------------------------------------------------
struct DownArgs {
    const void *cache;
    RowMap map;
    const float *params;
    int64_t PLb, oWd, ocd;
    int d, w;
    float *U; // [L][Mmax][w]
    int64_t Mmax;
};
struct EpiBias {
    const float *bias;
    float *out;
    int ld;
    static constexpr bool kBatched = true; // the bias is read once, before the stores
    __device__ void batch(int row_base, int col, const f32x16 &acc, int nrows, int ncols) const
    {
        const float b = bias[min(col, ncols - 1)];
        if (col >= ncols) return;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = epi_row(row_base, v);
            if (row < nrows) out[(int64_t)row * ld + col] = acc[v] + b;
        }
    }
};
// The same on the bf16 matrix units, for a bf16 cache: W_down^l as three bf16 terms, transposed ([3][w][d], k_lsplit,
// once per step), one workgroup per 128 token rows and layer (gemm_nt_fold3).  The cache values are exactly bf16, so
// every product is exact in fp32 and only the order of the additions differs from the fp32 contraction.
__global__ __launch_bounds__(256) void k_lsplit(const float *params, int64_t PLb, int64_t oWd, int d, int w, bf16_t *Wsp)
{
    __shared__ float tile[64][33]; // 64 rows x 32 columns of W_down^l ([d][w])
    const int l = blockIdx.y, c0 = blockIdx.x * 64, n0 = blockIdx.z * 32;
    const float *W = params + (int64_t)l * PLb + oWd;
    float v[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const int e = threadIdx.x + 256 * q, c = e >> 5, n = e & 31;
        v[q] = c0 + c < d ? W[(int64_t)(c0 + c) * w + n0 + n] : 0.f;
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const int e = threadIdx.x + 256 * q;
        tile[e >> 5][e & 31] = v[q];
    }
    __syncthreads();
    bf16_t *out = Wsp + (int64_t)l * 3 * w * d;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const int e = threadIdx.x + 256 * q, n = e >> 6, c = e & 63;
        if (c0 + c >= d) continue;
        const float x = tile[c][n];
        const bf16_t hi = static_cast<bf16_t>(x);
        const float r1 = x - to_f32(hi);       // exact
        const bf16_t mid = static_cast<bf16_t>(r1);
        const float r2 = r1 - to_f32(mid);     // exact
        const bf16_t lo = static_cast<bf16_t>(r2);
        out[((int64_t)0 * w + n0 + n) * d + c0 + c] = hi;
        out[((int64_t)1 * w + n0 + n) * d + c0 + c] = mid;
        out[((int64_t)2 * w + n0 + n) * d + c0 + c] = lo;
    }
}
// K steps of 32 in a two-stage ring: 53 KB of LDS at w = 96, every tile of the launch resident at once (measured:
// K steps of 64, one workgroup per compute unit, 57 us; these 43 us; a third stage 45 us)
template <int WB> struct Down3Shapes { using TL = NtTile<4, 1, 1, 3 * WB, 32, 2>; };
template <int WB> __global__ __launch_bounds__(256) void k_ldown3(DownArgs a, const bf16_t *Wsp)
{
    using TL = typename Down3Shapes<WB>::TL;
    extern __shared__ __attribute__((aligned(1024))) char dsm[];
    const int l = blockIdx.y;
    const float *pl = a.params + (int64_t)l * a.PLb;
    const bf16_t *cache = static_cast<const bf16_t *>(a.cache);
    const RowMap map = a.map;
    const bf16_t *Wl = Wsp + (int64_t)l * 3 * a.w * a.d;
    const int d = a.d;
    auto arow = [&](int m) { return cache + map.rowoff[m] + (int64_t)l * map.rowstride[m]; };
    auto brow = [&](int c) { return Wl + (int64_t)c * d; };
    EpiBias epi{pl + a.ocd, a.U + (int64_t)l * a.Mmax * a.w, a.w};
    gemm_nt_fold3<TL>(dsm, arow, brow, epi, 0, a.d, blockIdx.x * TL::BM, a.map.M, a.w);
}

template <typename SRC> __global__ __launch_bounds__(256) void k_ldown(DownArgs a)
{
    __shared__ __attribute__((aligned(16))) char smem[kTileLds];
    const int l = blockIdx.z;
    const float *pl = a.params + (int64_t)l * a.PLb;
    LoadRowsCache<SRC, 64, 4> al;
    al.cache = static_cast<const SRC *>(a.cache); al.map = a.map; al.layer = l; al.klim = a.d;
    LoadCols<float, 64, 4, float, false> bl;
    bl.src = pl + a.oWd; bl.ld = a.w; bl.ncols = a.w; bl.kend = a.d;
    EpiBias epi{pl + a.ocd, a.U + (int64_t)l * a.Mmax * a.w, a.w};
    gemm_tile<float, TL>(smem, al, bl, epi, 0, a.d, blockIdx.x * 64, blockIdx.y * 64, a.map.M, a.w);
}

// ---------------------------------------------------------------------------
// out = A B (+ ...) for the w-wide activations.  BT false: B is [K][N] (a weight used forward);
// BT true: B is [N][K] (the same weight used in the reverse pass).
//   EPI 0: out = acc + bias            1: out = acc + bias + res
//       2: out = acc + bias, out2 = GELU(out)      3: out = acc * GELU'(aux)      4: out = acc
// ---------------------------------------------------------------------------
struct LinArgs {
    const float *A; int lda;
    const float *B; int ldb;
    int M, N, K;
    const float *bias, *res, *aux;
    float *out, *out2;
};
template <int EPI> struct EpiLin {
    // every value the epilogue reads is requested (from clamped indices) before the first store: element by element
    // each load would have to wait behind the store before it, which may alias it as far as the compiler knows
    static constexpr bool kBatched = true;
    LinArgs a;
    __device__ void batch(int row_base, int col, const f32x16 &acc, int nrows, int ncols) const
    {
        const int cc = min(col, ncols - 1);
        const float bias = (EPI <= 2) ? a.bias[cc] : 0.f;
        float x[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int64_t o = (int64_t)min(epi_row(row_base, v), nrows - 1) * a.N + cc;
            x[v] = EPI == 1 ? a.res[o] : EPI == 3 ? a.aux[o] : 0.f;
        }
        if (col >= ncols) return;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = epi_row(row_base, v);
            if (row < nrows) {
                const int64_t o = (int64_t)row * a.N + col;
                if (EPI == 0) a.out[o] = acc[v] + bias;
                if (EPI == 1) a.out[o] = acc[v] + bias + x[v];
                if (EPI == 2) { const float u = acc[v] + bias; a.out[o] = u; a.out2[o] = lgelu(u); }
                if (EPI == 3) a.out[o] = acc[v] * lgelu_grad(x[v]);
                if (EPI == 4) a.out[o] = acc[v];
            }
        }
    }
    // the same for a 16 x 16 block: rows row_base .. row_base + 3 of column col
    __device__ void batch4(int row_base, int col, const f32x4 &acc, int nrows, int ncols) const
    {
        const int cc = min(col, ncols - 1);
        const float bias = (EPI <= 2) ? a.bias[cc] : 0.f;
        float x[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int64_t o = (int64_t)min(row_base + v, nrows - 1) * a.N + cc;
            x[v] = EPI == 1 ? a.res[o] : EPI == 3 ? a.aux[o] : 0.f;
        }
        if (col >= ncols) return;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = row_base + v;
            if (row < nrows) {
                const int64_t o = (int64_t)row * a.N + col;
                if (EPI == 0) a.out[o] = acc[v] + bias;
                if (EPI == 1) a.out[o] = acc[v] + bias + x[v];
                if (EPI == 2) { const float u = acc[v] + bias; a.out[o] = u; a.out2[o] = lgelu(u); }
                if (EPI == 3) a.out[o] = acc[v] * lgelu_grad(x[v]);
                if (EPI == 4) a.out[o] = acc[v];
            }
        }
    }
};

// The same contraction on a 32 x 32 workgroup tile of 2 x 2 blocks of 16 x 16, one per wavefront (16x16x4 fp32 matrix
// instructions): four times as many blocks as the 32 x 32 form.  For outputs as narrow as the ladder (N = w): there the
// 32 x 32 blocks number a third of the SIMDs and a launch with K = 4 w spends 12 k cycles in one block's instructions.
// A lane reads four consecutive K values of its row and feeds one to each of four instructions (both operands use the
// same assignment, so the order of K inside a step does not matter).
constexpr int kTile16Lds = 64 * Stage<float, 4>::LDP * 4;
template <class ALoad, class BLoad, class Epi>
__device__ __forceinline__ void gemm_tile16(void *lds, ALoad &al, BLoad &bl, Epi &epi, int kbegin, int kend, int row0,
                                            int col0, int nrows, int ncols)
{
    using S = Stage<float, 4>;
    float *As = reinterpret_cast<float *>(lds);
    float *Bs = As + 32 * S::LDP;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1, i = lane & 15, g4 = lane >> 4;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    al.init(row0);
    bl.init(col0);
    const int nsteps = (kend - kbegin + S::BK - 1) / S::BK;
    auto mma = [&]() {
        const float *ap = As + (wm * 16 + i) * S::LDP + 4 * g4;
        const float *bp = Bs + (wn * 16 + i) * S::LDP + 4 * g4;
#pragma unroll
        for (int kk = 0; kk < S::BK / 16; ++kk) {
            const f32x4 a4 = *reinterpret_cast<const f32x4 *>(ap + 16 * kk);
            const f32x4 b4 = *reinterpret_cast<const f32x4 *>(bp + 16 * kk);
#pragma unroll
            for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[j], b4[j], acc, 0, 0, 0);
        }
    };
    if (nsteps > 0) { // two K steps in flight, as in gemm_tile
        const int klast = kbegin + (nsteps - 1) * S::BK;
        al.template fetch<0>(kbegin);
        bl.template fetch<0>(kbegin);
        al.template fetch<1>(min(kbegin + S::BK, klast));
        bl.template fetch<1>(min(kbegin + S::BK, klast));
        for (int st = 0; st < nsteps; st += 2) {
            const int k0 = kbegin + st * S::BK;
            al.template store<0>(As, true);
            bl.template store<0>(Bs, true);
            __syncthreads();
            al.template fetch<0>(min(k0 + 2 * S::BK, klast));
            bl.template fetch<0>(min(k0 + 2 * S::BK, klast));
            mma();
            __syncthreads();
            const bool live = st + 1 < nsteps;
            al.template store<1>(As, live);
            bl.template store<1>(Bs, live);
            __syncthreads();
            al.template fetch<1>(min(k0 + 3 * S::BK, klast));
            bl.template fetch<1>(min(k0 + 3 * S::BK, klast));
            if (live) mma();
            __syncthreads();
        }
    }
    epi.batch4(row0 + wm * 16 + 4 * g4, col0 + wn * 16 + i, acc, nrows, ncols);
}
template <bool BT, int EPI> __global__ __launch_bounds__(256) void k_llin16(LinArgs a)
{
    __shared__ __attribute__((aligned(16))) char smem[kTile16Lds];
    LoadRowsTC<float, 32, 4> al;
    al.src = a.A; al.ld = a.lda; al.nrows = a.M; al.klim = a.K;
    EpiLin<EPI> epi{a};
    if (BT) {
        LoadRowsTC<float, 32, 4> bl;
        bl.src = a.B; bl.ld = a.ldb; bl.nrows = a.N; bl.klim = a.K;
        gemm_tile16(smem, al, bl, epi, 0, a.K, blockIdx.x * 32, blockIdx.y * 32, a.M, a.N);
    } else {
        LoadCols<float, 32, 4, float, false> bl;
        bl.src = a.B; bl.ld = a.ldb; bl.ncols = a.N; bl.kend = a.K;
        gemm_tile16(smem, al, bl, epi, 0, a.K, blockIdx.x * 32, blockIdx.y * 32, a.M, a.N);
    }
}
template <bool BT, int EPI> __global__ __launch_bounds__(256) void k_llin(LinArgs a)
{
    __shared__ __attribute__((aligned(16))) char smem[kTileLds];
    LoadRowsTC<float, 64, 4> al;
    al.src = a.A; al.ld = a.lda; al.nrows = a.M; al.klim = a.K;
    EpiLin<EPI> epi{a};
    if (BT) {
        LoadRowsTC<float, 64, 4> bl;
        bl.src = a.B; bl.ld = a.ldb; bl.nrows = a.N; bl.klim = a.K;
        gemm_tile<float, TL>(smem, al, bl, epi, 0, a.K, blockIdx.x * 64, blockIdx.y * 64, a.M, a.N);
    } else {
        LoadCols<float, 64, 4, float, false> bl;
        bl.src = a.B; bl.ld = a.ldb; bl.ncols = a.N; bl.kend = a.K;
        gemm_tile<float, TL>(smem, al, bl, epi, 0, a.K, blockIdx.x * 64, blockIdx.y * 64, a.M, a.N);
    }
}

// ---------------------------------------------------------------------------
// The forward tail of a ladder layer in one launch (w <= 128): output projection + x, LayerNorm 2, FFN in + GELU,
// FFN out + t, for 16 token rows per workgroup.  Everything a later kernel reads is written exactly as the separate
// launches write it (T, TN, the LayerNorm statistics, F1, G, A); between the four steps the tile stays in LDS.
// Matrix instructions: 16x16x4 fp32, A operand = the tile's activations (lane (i, g4): token row i), B operand = the
// weight as stored ([K][N], N contiguous), read straight from global memory (L2): a lane takes two neighbouring
// columns 32 p + 2 i, + 1 per load, one for each of two accumulators, so that loads and stores are 8 bytes wide and
// rows of 128 bytes; K is walked in blocks of 8 (lane g4 takes k = 2 g4 + s of a block for its s-th instruction, the
// same assignment on both operands).  The two contractions with a narrow output (N = w) split K over the four
// wavefronts and meet in LDS; FFN in splits its 4 w columns over them.
// ---------------------------------------------------------------------------
typedef float f32x2 __attribute__((ext_vector_type(2)));
struct MlpArgs {
    const float *O, *X; // [M][w]: attention output, the layer's input (residual)
    const float *Wo, *bo, *g2, *h2, *W1, *b1, *W2, *b2;
    float *T, *TN, *st2, *F1, *G, *A;
    int M;
};
// A chunk of WB blocks of 8 K values of a weight, in registers: rows kbeg + 8 (c WB + b) + 2 g4 + s, columns
// n0 + 32 p + 2 i, + 1.  Weights depend on nothing computed here, so a chunk is requested well before it is used
// (the first chunks of the next contraction while the tile is still in the previous step's epilogue); the scheduling
// barriers keep the compiler from moving the requests down to their uses.
template <int WB> struct WChunk {
    f32x2 r[WB][2][WB];
    __device__ __forceinline__ void load(const float *W, int ldw, int kbeg, int n0, int c, int i, int g4)
    {
#pragma unroll
        for (int b = 0; b < WB; ++b)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                for (int pq = 0; pq < WB; ++pq)
                    r[b][s2][pq] = *reinterpret_cast<const f32x2 *>(W + (int64_t)(kbeg + 8 * (c * WB + b) + 2 * g4 + s2) * ldw + n0 + 32 * pq + 2 * i);
        __builtin_amdgcn_sched_barrier(0);
    }
    // acc += Alds[16][the chunk's K values] (chunk)
    __device__ __forceinline__ void mul(const float *Alds, int pitch, int kbeg, int c, f32x4 (&acc)[2 * WB], int i, int g4) const
    {
#pragma unroll
        for (int b = 0; b < WB; ++b) {
            const f32x2 av = *reinterpret_cast<const f32x2 *>(Alds + i * pitch + kbeg + 8 * (c * WB + b) + 2 * g4);
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                for (int pq = 0; pq < WB; ++pq) {
                    acc[2 * pq] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[s2], r[b][s2][pq][0], acc[2 * pq], 0, 0, 0);
                    acc[2 * pq + 1] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[s2], r[b][s2][pq][1], acc[2 * pq + 1], 0, 0, 0);
                }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
};
template <int WB> constexpr int mlp_lds_bytes() { return (96 * (32 * WB + 4) + 16 * (128 * WB + 4)) * 4; }

template <int WB> __global__ __launch_bounds__(256) void k_lmlp_fwd(MlpArgs a)
{
    constexpr int w = 32 * WB, f = 4 * w, NB = 2 * WB, PW = w + 4, PF = f + 4, T = 16;
    extern __shared__ __attribute__((aligned(16))) float msm[];
    float *bufA = msm, *bufT = bufA + T * PW, *bufG = bufT + T * PW, *part = bufG + T * PF; // part [4][T][PW]
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, i = lane & 15, g4 = lane >> 4;
    const int m0 = blockIdx.x * T, M = a.M;
    WChunk<WB> c0, c1;
    c0.load(a.Wo, w, wave * (w / 4), 0, 0, i, g4);
    for (int idx = t; idx < T * (w / 4); idx += 256) {
        const int row = idx / (w / 4), c4 = idx % (w / 4), m = min(m0 + row, M - 1);
        *reinterpret_cast<f32x4 *>(bufA + row * PW + 4 * c4) = *reinterpret_cast<const f32x4 *>(a.O + (int64_t)m * w + 4 * c4);
    }
    __syncthreads();
    f32x4 acc[NB];
    auto zero = [&]() {
#pragma unroll
        for (int q = 0; q < NB; ++q) acc[q] = f32x4{0.f, 0.f, 0.f, 0.f};
    };
    auto to_part = [&]() { // this wavefront's share of K: rows 4 g4 + v, columns 32 p + 2 i, + 1
        float *pp = part + (size_t)wave * T * PW;
#pragma unroll
        for (int pq = 0; pq < WB; ++pq)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                *reinterpret_cast<f32x2 *>(pp + (4 * g4 + v) * PW + 32 * pq + 2 * i) = f32x2{acc[2 * pq][v], acc[2 * pq + 1][v]};
    };
    // ---- t = o W_o + b_o + x ----
    zero();
    c0.mul(bufA, PW, wave * (w / 4), 0, acc, i, g4);
    c0.load(a.W1, f, 0, wave * w, 0, i, g4); // the first half of W_1's share, used after the LayerNorm
    c1.load(a.W1, f, 0, wave * w, 1, i, g4);
    to_part();
    __syncthreads();
    for (int idx = t; idx < T * (w / 2); idx += 256) {
        const int row = idx / (w / 2), col = 2 * (idx % (w / 2)), m = m0 + row, mc = min(m, M - 1);
        const f32x2 xr = *reinterpret_cast<const f32x2 *>(a.X + (int64_t)mc * w + col);
        f32x2 v = {a.bo[col] + xr[0], a.bo[col + 1] + xr[1]};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f32x2 pv = *reinterpret_cast<const f32x2 *>(part + ((size_t)q * T + row) * PW + col);
            v[0] += pv[0];
            v[1] += pv[1];
        }
        *reinterpret_cast<f32x2 *>(bufT + row * PW + col) = v;
        if (m < M) *reinterpret_cast<f32x2 *>(a.T + (int64_t)m * w + col) = v;
    }
    __syncthreads();
    // ---- LayerNorm 2: sixteen threads per row ----
    {
        const int row = t >> 4, sub = t & 15, m = m0 + row;
        float x[NB], sum = 0.f;
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            x[q] = bufT[row * PW + sub + 16 * q];
            sum += x[q];
        }
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) sum += __shfl_xor(sum, o, 64);
        const float mu = sum / (float)w;
        float ss = 0.f;
#pragma unroll
        for (int q = 0; q < NB; ++q) ss += (x[q] - mu) * (x[q] - mu);
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) ss += __shfl_xor(ss, o, 64);
        const float rstd = 1.f / sqrtf(ss / (float)w + 1e-5f);
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            const int c = sub + 16 * q;
            const float y = (x[q] - mu) * rstd * a.g2[c] + a.h2[c];
            bufA[row * PW + c] = y;
            if (m < M) a.TN[(int64_t)m * w + c] = y;
        }
        if (sub == 0 && m < M) {
            a.st2[2 * (int64_t)m] = mu;
            a.st2[2 * (int64_t)m + 1] = rstd;
        }
    }
    __syncthreads();
    // ---- f1 = tn W_1 + b_1, g = GELU(f1): this wavefront's w columns ----
    zero();
    c0.mul(bufA, PW, 0, 0, acc, i, g4);
    c0.load(a.W1, f, 0, wave * w, 2, i, g4);
    c1.mul(bufA, PW, 0, 1, acc, i, g4);
    c1.load(a.W1, f, 0, wave * w, 3, i, g4);
    c0.mul(bufA, PW, 0, 2, acc, i, g4);
    c0.load(a.W2, w, wave * w, 0, 0, i, g4); // W_2's first half, used after the GELU
    c1.mul(bufA, PW, 0, 3, acc, i, g4);
    c1.load(a.W2, w, wave * w, 0, 1, i, g4);
#pragma unroll
    for (int pq = 0; pq < WB; ++pq) {
        const int col = wave * w + 32 * pq + 2 * i;
        const f32x2 bb = *reinterpret_cast<const f32x2 *>(a.b1 + col);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = 4 * g4 + v, m = m0 + row;
            const f32x2 u = {acc[2 * pq][v] + bb[0], acc[2 * pq + 1][v] + bb[1]};
            const f32x2 gl = {lgelu(u[0]), lgelu(u[1])};
            *reinterpret_cast<f32x2 *>(bufG + row * PF + col) = gl;
            if (m < M) {
                *reinterpret_cast<f32x2 *>(a.F1 + (int64_t)m * f + col) = u;
                *reinterpret_cast<f32x2 *>(a.G + (int64_t)m * f + col) = gl;
            }
        }
    }
    __syncthreads();
    // ---- a = g W_2 + b_2 + t ----
    zero();
    c0.mul(bufG, PF, wave * w, 0, acc, i, g4);
    c0.load(a.W2, w, wave * w, 0, 2, i, g4);
    c1.mul(bufG, PF, wave * w, 1, acc, i, g4);
    c1.load(a.W2, w, wave * w, 0, 3, i, g4);
    c0.mul(bufG, PF, wave * w, 2, acc, i, g4);
    c1.mul(bufG, PF, wave * w, 3, acc, i, g4);
    to_part();
    __syncthreads();
    for (int idx = t; idx < T * (w / 2); idx += 256) {
        const int row = idx / (w / 2), col = 2 * (idx % (w / 2)), m = m0 + row;
        const f32x2 tr = *reinterpret_cast<const f32x2 *>(bufT + row * PW + col);
        f32x2 v = {a.b2[col] + tr[0], a.b2[col + 1] + tr[1]};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f32x2 pv = *reinterpret_cast<const f32x2 *>(part + ((size_t)q * T + row) * PW + col);
            v[0] += pv[0];
            v[1] += pv[1];
        }
        if (m < M) *reinterpret_cast<f32x2 *>(a.A + (int64_t)m * w + col) = v;
    }
}

// The reverse of that tail in one launch: dg = da W_2^T, df1 = dg GELU'(f1), dtn = df1 W_1^T, the reverse of
// LayerNorm 2 (dt, with its partial sums for the gain and offset gradients of this 16-row block), do = dt W_o^T.
// The three weights are read from transposed copies made once per step (k_ltrans): contracted along their contiguous
// index straight from the parameter vector, a load instruction touched sixteen rows of 32 bytes and the launch took
// as long as the four it replaces.
// WT[l] = [W_2^T (w x 4w) | W_1^T (4w x w) | W_o^T (w x w) | W_qkv^T (3w x w)] of every layer
__global__ __launch_bounds__(256) void k_ltrans(const float *params, int64_t PLb, int64_t oW2, int64_t oW1, int64_t oWo,
                                               int64_t oWqkv, int w, float *WT)
{
    const int f = 4 * w, per = 2 * w * f + 4 * w * w, l = blockIdx.y;
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= per) return;
    const float *pl = params + (int64_t)l * PLb;
    float v;
    if (e < w * f) v = pl[oW2 + (int64_t)(e % f) * w + e / f];                                 // W_2 [4w][w]
    else if (e < 2 * w * f) v = pl[oW1 + (int64_t)((e - w * f) % w) * f + (e - w * f) / w];    // W_1 [w][4w]
    else if (e < 2 * w * f + w * w) v = pl[oWo + (int64_t)((e - 2 * w * f) % w) * w + (e - 2 * w * f) / w]; // W_o [w][w]
    else v = pl[oWqkv + (int64_t)((e - 2 * w * f - w * w) % w) * 3 * w + (e - 2 * w * f - w * w) / w];        // W_qkv [w][3w]
    WT[(int64_t)l * per + e] = v;
}
struct MlpBwdArgs {
    const float *DA;                 // [M][w]: gradient of the layer's output (also the residual path of LayerNorm 2)
    const float *F1, *T, *st2;       // saved by the forward tail
    const float *W2T, *W1T, *WoT, *g2; // [w][4w], [4w][w], [w][w]
    float *DF1, *DT, *DO;            // [M][4w], [M][w], [M][w]
    float *ln2p;                     // this layer's [blocks][2][w] partial sums
    int M;
};
template <int WB> constexpr int mlp_bwd_lds_bytes() { return (112 * (32 * WB + 4) + 16 * (128 * WB + 4)) * 4; }

template <int WB> __global__ __launch_bounds__(256) void k_lmlp_bwd(MlpBwdArgs a)
{
    constexpr int w = 32 * WB, f = 4 * w, NB = 2 * WB, PW = w + 4, PF = f + 4, T = 16;
    extern __shared__ __attribute__((aligned(16))) float msm[];
    float *bufD = msm, *bufA = bufD + T * PW, *bufT = bufA + T * PW, *bufG = bufT + T * PW, *part = bufG + T * PF; // part [4][T][PW]
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, i = lane & 15, g4 = lane >> 4;
    const int m0 = blockIdx.x * T, M = a.M;
    WChunk<WB> c0, c1;
    // dg: this wavefront's w columns of 4 w, K = w = four chunks
    c0.load(a.W2T, f, 0, wave * w, 0, i, g4);
    c1.load(a.W2T, f, 0, wave * w, 1, i, g4);
    for (int idx = t; idx < T * (w / 4); idx += 256) {
        const int row = idx / (w / 4), c4 = idx % (w / 4), m = min(m0 + row, M - 1);
        *reinterpret_cast<f32x4 *>(bufD + row * PW + 4 * c4) = *reinterpret_cast<const f32x4 *>(a.DA + (int64_t)m * w + 4 * c4);
    }
    // f1 of this lane's outputs: rows 4 g4 + v, columns wave w + 32 p + 2 i, + 1
    f32x2 f1v[WB][4];
#pragma unroll
    for (int pq = 0; pq < WB; ++pq)
#pragma unroll
        for (int v = 0; v < 4; ++v)
            f1v[pq][v] = *reinterpret_cast<const f32x2 *>(a.F1 + (int64_t)min(m0 + 4 * g4 + v, M - 1) * f + wave * w + 32 * pq + 2 * i);
    __syncthreads();
    f32x4 acc[NB];
    auto zero = [&]() {
#pragma unroll
        for (int q = 0; q < NB; ++q) acc[q] = f32x4{0.f, 0.f, 0.f, 0.f};
    };
    auto to_part = [&]() {
        float *pp = part + (size_t)wave * T * PW;
#pragma unroll
        for (int pq = 0; pq < WB; ++pq)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                *reinterpret_cast<f32x2 *>(pp + (4 * g4 + v) * PW + 32 * pq + 2 * i) = f32x2{acc[2 * pq][v], acc[2 * pq + 1][v]};
    };
    zero();
    c0.mul(bufD, PW, 0, 0, acc, i, g4);
    c0.load(a.W2T, f, 0, wave * w, 2, i, g4);
    c1.mul(bufD, PW, 0, 1, acc, i, g4);
    c1.load(a.W2T, f, 0, wave * w, 3, i, g4);
    c0.mul(bufD, PW, 0, 2, acc, i, g4);
    c0.load(a.W1T, w, wave * w, 0, 0, i, g4); // dtn: K = 4 w split over the wavefronts
    c1.mul(bufD, PW, 0, 3, acc, i, g4);
    c1.load(a.W1T, w, wave * w, 0, 1, i, g4);
#pragma unroll
    for (int pq = 0; pq < WB; ++pq)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = 4 * g4 + v, m = m0 + row, col = wave * w + 32 * pq + 2 * i;
            const f32x2 d = {acc[2 * pq][v] * lgelu_grad(f1v[pq][v][0]), acc[2 * pq + 1][v] * lgelu_grad(f1v[pq][v][1])};
            *reinterpret_cast<f32x2 *>(bufG + row * PF + col) = d;
            if (m < M) *reinterpret_cast<f32x2 *>(a.DF1 + (int64_t)m * f + col) = d;
        }
    __syncthreads();
    zero();
    c0.mul(bufG, PF, wave * w, 0, acc, i, g4);
    c0.load(a.W1T, w, wave * w, 0, 2, i, g4);
    c1.mul(bufG, PF, wave * w, 1, acc, i, g4);
    c1.load(a.W1T, w, wave * w, 0, 3, i, g4);
    c0.mul(bufG, PF, wave * w, 2, acc, i, g4);
    c0.load(a.WoT, w, wave * (w / 4), 0, 0, i, g4); // do: K = w split over the wavefronts
    c1.mul(bufG, PF, wave * w, 3, acc, i, g4);
    to_part();
    __syncthreads();
    for (int idx = t; idx < T * w; idx += 256) {
        const int row = idx / w, col = idx % w;
        bufA[row * PW + col] = ((part[((size_t)0 * T + row) * PW + col] + part[((size_t)1 * T + row) * PW + col]) +
                                part[((size_t)2 * T + row) * PW + col]) + part[((size_t)3 * T + row) * PW + col];
    }
    __syncthreads();
    // ---- reverse of LayerNorm 2: sixteen threads per row; dy xh and dy of every row go to `part` for the block sums ----
    {
        const int row = t >> 4, sub = t & 15, m = m0 + row, mc = min(m, M - 1);
        const bool rowok = m < M;
        const float mu = a.st2[2 * (int64_t)mc], rstd = a.st2[2 * (int64_t)mc + 1];
        float xh[NB], dxh[NB], s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            const int c = sub + 16 * q;
            const float dy = rowok ? bufA[row * PW + c] : 0.f;
            xh[q] = rowok ? (a.T[(int64_t)mc * w + c] - mu) * rstd : 0.f;
            dxh[q] = dy * a.g2[c];
            part[(size_t)row * PW + c] = dy * xh[q];
            part[((size_t)T + row) * PW + c] = dy;
            s1 += dxh[q];
            s2 += dxh[q] * xh[q];
        }
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) {
            s1 += __shfl_xor(s1, o, 64);
            s2 += __shfl_xor(s2, o, 64);
        }
        const float m1 = s1 / (float)w, m2 = s2 / (float)w;
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            const int c = sub + 16 * q;
            const float dx = bufD[row * PW + c] + rstd * (dxh[q] - m1 - xh[q] * m2);
            bufT[row * PW + c] = dx;
            if (rowok) a.DT[(int64_t)m * w + c] = dx;
        }
    }
    __syncthreads();
    for (int c = t; c < 2 * w; c += 256) {
        const int which = c / w, col = c % w;
        float sum = 0.f;
#pragma unroll
        for (int row = 0; row < T; ++row) sum += part[((size_t)which * T + row) * PW + col];
        a.ln2p[(int64_t)blockIdx.x * 2 * w + c] = sum;
    }
    __syncthreads();
    // ---- do = dt W_o^T ----
    zero();
    c0.mul(bufT, PW, wave * (w / 4), 0, acc, i, g4);
    to_part();
    __syncthreads();
    for (int idx = t; idx < T * w; idx += 256) {
        const int row = idx / w, col = idx % w, m = m0 + row;
        if (m < M)
            a.DO[(int64_t)m * w + col] = ((part[((size_t)0 * T + row) * PW + col] + part[((size_t)1 * T + row) * PW + col]) +
                                          part[((size_t)2 * T + row) * PW + col]) + part[((size_t)3 * T + row) * PW + col];
    }
}

// The head of a ladder layer in one launch (w <= 128): gate mix x = lambda u + (1 - lambda) a_prev, LayerNorm 1 and the
// fused q, k, v projection for 16 token rows; three wavefronts take w of the 3 w output columns each.
struct QkvArgs {
    const float *U, *Aprev, *lam; // Aprev null in the first layer
    const float *g1, *h1, *Wqkv, *bqkv;
    float *X, *XN, *st1, *QKV;
    int M;
};
template <int WB> __global__ __launch_bounds__(256) void k_lqkv_fwd(QkvArgs a)
{
    constexpr int w = 32 * WB, NB = 2 * WB, PW = w + 4, T = 16;
    __shared__ __attribute__((aligned(16))) float bufA[T * PW];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, i = lane & 15, g4 = lane >> 4;
    const int m0 = blockIdx.x * T, M = a.M;
    WChunk<WB> c0, c1;
    if (wave < 3) {
        c0.load(a.Wqkv, 3 * w, 0, wave * w, 0, i, g4);
        c1.load(a.Wqkv, 3 * w, 0, wave * w, 1, i, g4);
    }
    {
        const int row = t >> 4, sub = t & 15, m = m0 + row, mc = min(m, M - 1);
        const float lam = *a.lam;
        float x[NB], sum = 0.f;
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            const int64_t o = (int64_t)mc * w + sub + 16 * q;
            x[q] = lam * a.U[o] + (1.f - lam) * (a.Aprev ? a.Aprev[o] : 0.f);
            if (m < M) a.X[o] = x[q];
            sum += x[q];
        }
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) sum += __shfl_xor(sum, o, 64);
        const float mu = sum / (float)w;
        float ss = 0.f;
#pragma unroll
        for (int q = 0; q < NB; ++q) ss += (x[q] - mu) * (x[q] - mu);
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) ss += __shfl_xor(ss, o, 64);
        const float rstd = 1.f / sqrtf(ss / (float)w + 1e-5f);
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            const int c = sub + 16 * q;
            const float y = (x[q] - mu) * rstd * a.g1[c] + a.h1[c];
            bufA[row * PW + c] = y;
            if (m < M) a.XN[(int64_t)m * w + c] = y;
        }
        if (sub == 0 && m < M) {
            a.st1[2 * (int64_t)m] = mu;
            a.st1[2 * (int64_t)m + 1] = rstd;
        }
    }
    __syncthreads();
    if (wave >= 3) return;
    f32x4 acc[NB];
#pragma unroll
    for (int q = 0; q < NB; ++q) acc[q] = f32x4{0.f, 0.f, 0.f, 0.f};
    c0.mul(bufA, PW, 0, 0, acc, i, g4);
    c0.load(a.Wqkv, 3 * w, 0, wave * w, 2, i, g4);
    c1.mul(bufA, PW, 0, 1, acc, i, g4);
    c1.load(a.Wqkv, 3 * w, 0, wave * w, 3, i, g4);
    c0.mul(bufA, PW, 0, 2, acc, i, g4);
    c1.mul(bufA, PW, 0, 3, acc, i, g4);
#pragma unroll
    for (int pq = 0; pq < WB; ++pq) {
        const int col = wave * w + 32 * pq + 2 * i;
        const f32x2 bb = *reinterpret_cast<const f32x2 *>(a.bqkv + col);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int m = m0 + 4 * g4 + v;
            if (m < M) *reinterpret_cast<f32x2 *>(a.QKV + (int64_t)m * 3 * w + col) = f32x2{acc[2 * pq][v] + bb[0], acc[2 * pq + 1][v] + bb[1]};
        }
    }
}

// Its reverse: dxn = dqkv W_qkv^T (K = 3 w split over the four wavefronts, transposed copy of the weight), the reverse
// of LayerNorm 1 with the residual path dt, and the reverse of the gate (its partial sum for this block, da_prev).
struct QkvBwdArgs {
    const float *DQKV, *WqkvT; // [M][3w], [3w][w]
    const float *X, *st1, *g1, *DT, *U, *Aprev, *lam;
    float *DX, *DAprev; // DAprev null in the first layer
    float *ln1p, *dlamp; // this layer's [blocks][2][w] and [blocks]
    int M;
};
template <int WB> constexpr int qkv_bwd_lds_bytes() { return (16 * (96 * WB + 4) + 80 * (32 * WB + 4) + 4) * 4; }
template <int WB> __global__ __launch_bounds__(256) void k_lqkv_bwd(QkvBwdArgs a)
{
    constexpr int w = 32 * WB, NB = 2 * WB, PW = w + 4, P3 = 3 * w + 4, T = 16;
    extern __shared__ __attribute__((aligned(16))) float msm[];
    float *bufQ = msm, *bufA = bufQ + T * P3, *part = bufA + T * PW, *redl = part + 4 * T * PW; // part [4][T][PW], redl [4]
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, i = lane & 15, g4 = lane >> 4;
    const int m0 = blockIdx.x * T, M = a.M;
    const int kb = wave * (3 * w / 4); // this wavefront's share of K: three chunks
    WChunk<WB> c0, c1;
    c0.load(a.WqkvT, w, kb, 0, 0, i, g4);
    c1.load(a.WqkvT, w, kb, 0, 1, i, g4);
    for (int idx = t; idx < T * (3 * w / 4); idx += 256) {
        const int row = idx / (3 * w / 4), c4 = idx % (3 * w / 4), m = min(m0 + row, M - 1);
        *reinterpret_cast<f32x4 *>(bufQ + row * P3 + 4 * c4) = *reinterpret_cast<const f32x4 *>(a.DQKV + (int64_t)m * 3 * w + 4 * c4);
    }
    __syncthreads();
    f32x4 acc[NB];
#pragma unroll
    for (int q = 0; q < NB; ++q) acc[q] = f32x4{0.f, 0.f, 0.f, 0.f};
    c0.mul(bufQ, P3, kb, 0, acc, i, g4);
    c0.load(a.WqkvT, w, kb, 0, 2, i, g4);
    c1.mul(bufQ, P3, kb, 1, acc, i, g4);
    c0.mul(bufQ, P3, kb, 2, acc, i, g4);
    {
        float *pp = part + (size_t)wave * T * PW;
#pragma unroll
        for (int pq = 0; pq < WB; ++pq)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                *reinterpret_cast<f32x2 *>(pp + (4 * g4 + v) * PW + 32 * pq + 2 * i) = f32x2{acc[2 * pq][v], acc[2 * pq + 1][v]};
    }
    __syncthreads();
    for (int idx = t; idx < T * w; idx += 256) {
        const int row = idx / w, col = idx % w;
        bufA[row * PW + col] = ((part[((size_t)0 * T + row) * PW + col] + part[((size_t)1 * T + row) * PW + col]) +
                                part[((size_t)2 * T + row) * PW + col]) + part[((size_t)3 * T + row) * PW + col];
    }
    __syncthreads();
    {
        const int row = t >> 4, sub = t & 15, m = m0 + row, mc = min(m, M - 1);
        const bool rowok = m < M;
        const float lam = *a.lam;
        const float mu = a.st1[2 * (int64_t)mc], rstd = a.st1[2 * (int64_t)mc + 1];
        float xh[NB], dxh[NB], s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            const int c = sub + 16 * q;
            const float dy = rowok ? bufA[row * PW + c] : 0.f;
            xh[q] = rowok ? (a.X[(int64_t)mc * w + c] - mu) * rstd : 0.f;
            dxh[q] = dy * a.g1[c];
            part[(size_t)row * PW + c] = dy * xh[q];
            part[((size_t)T + row) * PW + c] = dy;
            s1 += dxh[q];
            s2 += dxh[q] * xh[q];
        }
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) {
            s1 += __shfl_xor(s1, o, 64);
            s2 += __shfl_xor(s2, o, 64);
        }
        const float m1 = s1 / (float)w, m2 = s2 / (float)w;
        float dlam = 0.f;
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            const int64_t o = (int64_t)mc * w + sub + 16 * q;
            const float dx = a.DT[o] + rstd * (dxh[q] - m1 - xh[q] * m2);
            if (rowok) {
                a.DX[o] = dx;
                dlam += dx * (a.U[o] - (a.Aprev ? a.Aprev[o] : 0.f));
                if (a.DAprev) a.DAprev[o] = (1.f - lam) * dx;
            }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) dlam += __shfl_xor(dlam, o, 64);
        if (lane == 0) redl[wave] = dlam;
    }
    __syncthreads();
    for (int c = t; c < 2 * w; c += 256) {
        const int which = c / w, col = c % w;
        float sum = 0.f;
#pragma unroll
        for (int row = 0; row < T; ++row) sum += part[((size_t)which * T + row) * PW + col];
        a.ln1p[(int64_t)blockIdx.x * 2 * w + c] = sum;
    }
    if (t == 0) a.dlamp[blockIdx.x] = ((redl[0] + redl[1]) + redl[2]) + redl[3];
}

// ---------------------------------------------------------------------------
// Row kernels (one wavefront per token row, lane owns columns lane, lane + 64, ...; w <= 256)
// ---------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// x = lam u + (1 - lam) a_prev (MIX) or x = in (plain); xn = LayerNorm(x; g, h); stats = (mean, 1/sqrt(var + eps))
struct LnFwdArgs {
    const float *in, *a_prev, *lam; // a_prev may be null (first layer)
    const float *g, *h;
    float *x, *xn, *stats;
    int M, w;
};
template <bool MIX> __global__ __launch_bounds__(256) void k_lln_fwd(LnFwdArgs a)
{
    const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= a.M) return;
    const float lam = MIX ? *a.lam : 1.f;
    float x[4], s = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int c = lane + 64 * q;
        x[q] = 0.f;
        if (c < a.w) {
            const int64_t o = (int64_t)row * a.w + c;
            float v = a.in[o];
            if (MIX) {
                v = lam * v + (1.f - lam) * (a.a_prev ? a.a_prev[o] : 0.f);
                a.x[o] = v;
            }
            x[q] = v;
            s += v;
        }
    }
    const float mu = wave_sum(s) / (float)a.w;
    float ss = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q)
        if (lane + 64 * q < a.w) ss += (x[q] - mu) * (x[q] - mu);
    const float rstd = 1.f / sqrtf(wave_sum(ss) / (float)a.w + 1e-5f);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int c = lane + 64 * q;
        if (c < a.w) a.xn[(int64_t)row * a.w + c] = (x[q] - mu) * rstd * a.g[c] + a.h[c];
    }
    if (lane == 0) { a.stats[2 * row] = mu; a.stats[2 * row + 1] = rstd; }
}

// Reverse of LayerNorm with the residual path: dx = resid + (1/sigma)(dxh - mean(dxh) - xh mean(dxh xh)),
// dxh = dy g, xh = (x - mean) / sigma; per-workgroup partial sums of dg = sum dy xh and dh = sum dy.
// MIX: also the gate's reverse: dlam partial = sum dx (u - a_prev), da_prev = (1 - lam) dx.
struct LnBwdArgs {
    const float *dy, *x, *stats, *g, *resid;
    float *dx;
    float *part; // [nblk][2][w]
    const float *u, *a_prev, *lam;
    float *da_prev;  // null for the first layer
    float *dlam_part; // [nblk]
    int M, w;
};
template <int N> __device__ __forceinline__ void wave_sum_n(float (&v)[N])
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
#pragma unroll
        for (int k = 0; k < N; ++k) v[k] += __shfl_xor(v[k], o, 64);
}

template <bool MIX> __global__ __launch_bounds__(256) void k_lln_bwd(LnBwdArgs a)
{
    __shared__ float red[4][2][256];
    __shared__ float redl[4];
    constexpr int RB = 4; // rows a wavefront works on at once (independent loads and exchanges in flight)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float lam = MIX ? *a.lam : 0.f;
    float dg[4] = {0.f, 0.f, 0.f, 0.f}, dh[4] = {0.f, 0.f, 0.f, 0.f}, dlam = 0.f;
    float g[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) g[q] = lane + 64 * q < a.w ? a.g[lane + 64 * q] : 0.f;
    for (int rr = 0; rr < kLnRows / 4; rr += RB) {
        const int row0 = blockIdx.x * kLnRows + wave * (kLnRows / 4) + rr;
        if (row0 >= a.M) break;
        float xh[RB][4], dxh[RB][4], rs[RB][4], dyv[RB][4], sums[2 * RB];
        float mu[RB], rstd[RB];
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            const int row = min(row0 + r, a.M - 1);
            mu[r] = a.stats[2 * row];
            rstd[r] = a.stats[2 * row + 1];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int c = lane + 64 * q;
                const int64_t o = (int64_t)row * a.w + min(c, a.w - 1);
                dyv[r][q] = a.dy[o];
                xh[r][q] = a.x[o];
                rs[r][q] = a.resid[o];
            }
        }
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            const bool rowok = row0 + r < a.M;
            float s1 = 0.f, s2 = 0.f;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const bool ok = rowok && lane + 64 * q < a.w;
                const float dy = ok ? dyv[r][q] : 0.f;
                xh[r][q] = ok ? (xh[r][q] - mu[r]) * rstd[r] : 0.f;
                dxh[r][q] = dy * g[q];
                dg[q] += dy * xh[r][q];
                dh[q] += dy;
                s1 += dxh[r][q];
                s2 += dxh[r][q] * xh[r][q];
            }
            sums[2 * r] = s1;
            sums[2 * r + 1] = s2;
        }
        wave_sum_n(sums);
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            const int row = row0 + r;
            const float m1 = sums[2 * r] / (float)a.w, m2 = sums[2 * r + 1] / (float)a.w;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int c = lane + 64 * q;
                if (row < a.M && c < a.w) {
                    const int64_t o = (int64_t)row * a.w + c;
                    const float dx = rs[r][q] + rstd[r] * (dxh[r][q] - m1 - xh[r][q] * m2);
                    a.dx[o] = dx;
                    if (MIX) {
                        dlam += dx * (a.u[o] - (a.a_prev ? a.a_prev[o] : 0.f));
                        if (a.da_prev) a.da_prev[o] = (1.f - lam) * dx;
                    }
                }
            }
        }
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) { red[wave][0][lane + 64 * q] = dg[q]; red[wave][1][lane + 64 * q] = dh[q]; }
    if (MIX) {
        const float t = wave_sum(dlam);
        if (lane == 0) redl[wave] = t;
    }
    __syncthreads();
    for (int c = threadIdx.x; c < a.w; c += 256) {
        float *p = a.part + (int64_t)blockIdx.x * 2 * a.w;
        p[c] = ((red[0][0][c] + red[1][0][c]) + red[2][0][c]) + red[3][0][c];
        p[a.w + c] = ((red[0][1][c] + red[1][1][c]) + red[2][1][c]) + red[3][1][c];
    }
    if (MIX && threadIdx.x == 0) a.dlam_part[blockIdx.x] = ((redl[0] + redl[1]) + redl[2]) + redl[3];
}

// ---------------------------------------------------------------------------
// Attention of one sample and head per workgroup; a thread owns a query row (forward, reverse phase 1)
// or a key row (reverse phase 2).  K and V (and Q, dO in the reverse pass) of the head sit in LDS.
// ---------------------------------------------------------------------------
struct AttnArgs {
    const float *QKV; // [M][3w]
    const int32_t *samp_start, *samp_len;
    float *O;   // [M][w]
    float *LSE; // [M][nh]
    const float *dO; // reverse: [M][w]
    float *dQKV;     // reverse: [M][3w]
    int w, nh, n_max;
    float scale;
    int tpr;    // lanes per row: a power of two, 1 .. 8
    int nchunk; // workgroups per sample and head (blockIdx.y): each takes a contiguous share of the rows
};
// Probabilities are formed as 2^(score - max) with the scores scaled by log2(e) beforehand (folded into the query's
// scale): the hardware's exponential is base 2, so a natural exponential costs a multiply and range fix-ups per call,
// and these kernels are bound by their vector arithmetic.  Results below the normal range flush to zero.
constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;
__device__ __forceinline__ float lexp2(float x) { return __builtin_amdgcn_exp2f(x); }
// A row is shared by `tpr` neighbouring lanes (a power of two, chosen so that the sample's rows fill the
// workgroup); each takes every tpr-th key (query) and the partial results are combined with lane exchanges.
__device__ __forceinline__ float grp_sum(float v, int tpr)
{
    for (int o = 1; o < tpr; o <<= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float grp_max(float v, int tpr)
{
    for (int o = 1; o < tpr; o <<= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

template <int DH> __global__ __launch_bounds__(256) void k_lattn_fwd(AttnArgs a)
{
    extern __shared__ __attribute__((aligned(16))) float lsm[];
    const int s = blockIdx.x / a.nh, h = blockIdx.x % a.nh;
    const int m0 = a.samp_start[s], n = a.samp_len[s];
    const int w3 = 3 * a.w;
    float *ks = lsm, *vs = lsm + (int64_t)a.n_max * DH;
    for (int idx = threadIdx.x; idx < n * DH; idx += 256) {
        const int j = idx / DH, c = idx % DH;
        const float *row = a.QKV + (int64_t)(m0 + j) * w3 + h * DH + c;
        ks[idx] = row[a.w];
        vs[idx] = row[2 * a.w];
    }
    __syncthreads();
    const int tpr = a.tpr, part = threadIdx.x % tpr, rpp = 256 / tpr;
    const int rpc = (n + a.nchunk - 1) / a.nchunk, r_lo = blockIdx.y * rpc, r_hi = min(n, r_lo + rpc);
    // (every lane of a group runs the same number of rounds: the exchanges below need all of them)
    for (int i0 = r_lo; i0 < r_hi; i0 += rpp) {
        const int i = i0 + (int)threadIdx.x / tpr;
        const bool live = i < r_hi;
        const int ic = live ? i : n - 1;
        float q[DH];
        const float *qp = a.QKV + (int64_t)(m0 + ic) * w3 + h * DH;
#pragma unroll
        for (int c = 0; c < DH; ++c) q[c] = qp[c] * (a.scale * kLog2e); // scores in units of ln 2: one exp2 instruction each
        // running maximum, sum and weighted values over this lane's keys
        float mx = -INFINITY, l = 0.f, acc[DH];
#pragma unroll
        for (int c = 0; c < DH; ++c) acc[c] = 0.f;
        // four keys per round: one rescaling of the running sums per round instead of one per key
        for (int j0 = part; j0 < n; j0 += 4 * tpr) {
            float sc[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int j = j0 + u * tpr;
                const float *kr = ks + min(j, n - 1) * DH;
                float t = 0.f;
#pragma unroll
                for (int c = 0; c < DH; ++c) t += q[c] * kr[c];
                sc[u] = j < n ? t : -INFINITY;
            }
            const float mn = fmaxf(fmaxf(mx, fmaxf(sc[0], sc[1])), fmaxf(sc[2], sc[3])); // sc[0] is always a key: finite
            const float corr = lexp2(mx - mn);
            l *= corr;
#pragma unroll
            for (int c = 0; c < DH; ++c) acc[c] *= corr;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float p = lexp2(sc[u] - mn); // 0 for the slots past the last key
                const float *vr = vs + min(j0 + u * tpr, n - 1) * DH;
                l += p;
#pragma unroll
                for (int c = 0; c < DH; ++c) acc[c] += p * vr[c];
            }
            mx = mn;
        }
        const float mall = grp_max(mx, tpr);
        const float corr = mx == -INFINITY ? 0.f : lexp2(mx - mall);
        l = grp_sum(l * corr, tpr);
        const float inv = 1.f / l;
        float *op = a.O + (int64_t)(m0 + ic) * a.w + h * DH;
#pragma unroll
        for (int c = 0; c < DH; ++c) {
            const float v = grp_sum(acc[c] * corr, tpr) * inv;
            if (live && part == 0) op[c] = v;
        }
        if (live && part == 0) a.LSE[(int64_t)(m0 + i) * a.nh + h] = mall * kLn2 + logf(l); // natural logarithm
    }
}

template <int DH> __global__ __launch_bounds__(256) void k_lattn_bwd(AttnArgs a)
{
    extern __shared__ __attribute__((aligned(16))) float lsm[];
    const int s = blockIdx.x / a.nh, h = blockIdx.x % a.nh;
    const int m0 = a.samp_start[s], n = a.samp_len[s];
    const int w3 = 3 * a.w;
    const int64_t nd = (int64_t)a.n_max * DH;
    float *qs = lsm, *ks = lsm + nd, *vs = lsm + 2 * nd, *dos = lsm + 3 * nd, *lse = lsm + 4 * nd, *Dr = lse + a.n_max;
    for (int idx = threadIdx.x; idx < n * DH; idx += 256) {
        const int j = idx / DH, c = idx % DH;
        const float *row = a.QKV + (int64_t)(m0 + j) * w3 + h * DH + c;
        qs[idx] = row[0];
        ks[idx] = row[a.w];
        vs[idx] = row[2 * a.w];
        dos[idx] = a.dO[(int64_t)(m0 + j) * a.w + h * DH + c];
    }
    for (int i = threadIdx.x; i < n; i += 256) {
        lse[i] = a.LSE[(int64_t)(m0 + i) * a.nh + h] * kLog2e;
        const float *op = a.O + (int64_t)(m0 + i) * a.w + h * DH;
        const float *dp = a.dO + (int64_t)(m0 + i) * a.w + h * DH;
        float D = 0.f;
#pragma unroll
        for (int c = 0; c < DH; ++c) D += op[c] * dp[c];
        Dr[i] = D;
    }
    __syncthreads();
    const int tpr = a.tpr, part = threadIdx.x % tpr, rpp = 256 / tpr;
    const int rpc = (n + a.nchunk - 1) / a.nchunk, r_lo = blockIdx.y * rpc, r_hi = min(n, r_lo + rpc);
    // phase 1, query row i: dq_i = scale * sum_j P_ij (dO_i . v_j - D_i) k_j
    for (int i0 = r_lo; i0 < r_hi; i0 += rpp) {
        const int i = i0 + (int)threadIdx.x / tpr;
        const bool live = i < r_hi;
        const int ic = live ? i : n - 1;
        float q[DH], go[DH], dq[DH];
#pragma unroll
        for (int c = 0; c < DH; ++c) { q[c] = qs[ic * DH + c] * (a.scale * kLog2e); go[c] = dos[ic * DH + c]; dq[c] = 0.f; }
        const float li = lse[ic], Di = Dr[ic];
        for (int j = part; j < n; j += tpr) {
            float sc = 0.f, dpv = 0.f;
#pragma unroll
            for (int c = 0; c < DH; ++c) { sc += q[c] * ks[j * DH + c]; dpv += go[c] * vs[j * DH + c]; }
            const float ds = lexp2(sc - li) * (dpv - Di);
#pragma unroll
            for (int c = 0; c < DH; ++c) dq[c] += ds * ks[j * DH + c];
        }
        float *out = a.dQKV + (int64_t)(m0 + ic) * w3 + h * DH;
#pragma unroll
        for (int c = 0; c < DH; ++c) {
            const float v = grp_sum(dq[c], tpr) * a.scale;
            if (live && part == 0) out[c] = v;
        }
    }
    // phase 2, key row j: dv_j = sum_i P_ij dO_i ; dk_j = scale * sum_i P_ij (dO_i . v_j - D_i) q_i
    for (int j0 = r_lo; j0 < r_hi; j0 += rpp) {
        const int j = j0 + (int)threadIdx.x / tpr;
        const bool live = j < r_hi;
        const int jc = live ? j : n - 1;
        float k[DH], v[DH], dk[DH], dv[DH];
#pragma unroll
        for (int c = 0; c < DH; ++c) { k[c] = ks[jc * DH + c] * (a.scale * kLog2e); v[c] = vs[jc * DH + c]; dk[c] = 0.f; dv[c] = 0.f; }
        for (int i = part; i < n; i += tpr) {
            float sc = 0.f, dpv = 0.f;
#pragma unroll
            for (int c = 0; c < DH; ++c) { sc += qs[i * DH + c] * k[c]; dpv += dos[i * DH + c] * v[c]; }
            const float p = lexp2(sc - lse[i]);
            const float ds = p * (dpv - Dr[i]);
#pragma unroll
            for (int c = 0; c < DH; ++c) { dv[c] += p * dos[i * DH + c]; dk[c] += ds * qs[i * DH + c]; }
        }
        float *out = a.dQKV + (int64_t)(m0 + jc) * w3 + h * DH;
#pragma unroll
        for (int c = 0; c < DH; ++c) {
            const float gk = grp_sum(dk[c], tpr) * a.scale, gv = grp_sum(dv[c], tpr);
            if (live && part == 0) { out[a.w + c] = gk; out[2 * a.w + c] = gv; }
        }
    }
}

// ---------------------------------------------------------------------------
// Head: y = b_L + a_L W_up + c_up; its token mean; classifier; cross-entropy; the head's gradients; da_L.
// ---------------------------------------------------------------------------
struct HeadArgs {
    const void *cache;
    RowMap map;
    const int32_t *samp_start, *samp_len, *labels;
    const float *params;
    int64_t oWup, ocup, oWcls, occls;
    const float *A_last; // [M][w]
    float *bmean, *abar, *pooled, *logits, *dz, *dp, *daL, *lossp;
    float *DA_last; // [M][w]
    float *loss_out, *logits_out, *grads; // logits_out, grads may be null
    int B, d, w, C, last_layer;
};

// token means of b_L (blockIdx.y < column blocks of d) and of a_L (the last blockIdx.y): a lane owns four columns,
// the four wavefronts take every fourth token and their sums are combined in wavefront order
template <typename SRC> __global__ __launch_bounds__(256) void k_lpool(HeadArgs a)
{
    __shared__ float red[4][256];
    const int s = blockIdx.x, m0 = a.samp_start[s], len = a.samp_len[s];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nbd = (a.d + 255) / 256;
    const bool from_cache = (int)blockIdx.y < nbd;
    const int ncols = from_cache ? a.d : a.w;
    const int c0 = (from_cache ? blockIdx.y * 256 : 0) + lane * 4;
    const bool live = c0 < ncols; // (d and w are multiples of 4)
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    if (live) {
        if (from_cache) {
            // the tokens of a sample are consecutive rows of one cache block: one table look-up gives them all;
            // eight rows are requested per round
            const SRC *base = static_cast<const SRC *>(a.cache) + a.map.rowoff[m0] + (int64_t)a.last_layer * a.map.rowstride[m0] + c0;
            for (int t0 = wave; t0 < len; t0 += 32) {
                typename Raw4<SRC>::type raw[8];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    raw[u] = *reinterpret_cast<const typename Raw4<SRC>::type *>(base + (int64_t)min(t0 + 4 * u, len - 1) * a.d);
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (t0 + 4 * u < len) {
                        float f[4];
                        Raw4<SRC>::widen(raw[u], f);
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc[e] += f[e];
                    }
            }
        } else {
            for (int t0 = wave; t0 < len; t0 += 32) {
                f32x4 v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    v[u] = *reinterpret_cast<const f32x4 *>(a.A_last + (int64_t)(m0 + min(t0 + 4 * u, len - 1)) * a.w + c0);
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (t0 + 4 * u < len) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc[e] += v[u][e];
                    }
            }
        }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) red[wave][lane * 4 + e] = acc[e];
    __syncthreads();
    const int c = (from_cache ? blockIdx.y * 256 : 0) + threadIdx.x;
    if (c < ncols) {
        const float tot = ((red[0][threadIdx.x] + red[1][threadIdx.x]) + red[2][threadIdx.x]) + red[3][threadIdx.x];
        (from_cache ? a.bmean + (int64_t)s * a.d : a.abar + (int64_t)s * a.w)[c] = tot / (float)len;
    }
}

// pooled[s][j] = mean_t b_L[t][j] + c_up[j] + sum_c mean_t a_L[t][c] W_up[c][j]   (grid: sample x column block)
__global__ __launch_bounds__(256) void k_lpooled(HeadArgs a)
{
    __shared__ float ab[256];
    const int s = blockIdx.x, j = blockIdx.y * 256 + threadIdx.x;
    if ((int)threadIdx.x < a.w) ab[threadIdx.x] = a.abar[(int64_t)s * a.w + threadIdx.x];
    __syncthreads();
    if (j >= a.d) return;
    const float *Wup = a.params + a.oWup + j;
    float p = a.bmean[(int64_t)s * a.d + j] + a.params[a.ocup + j];
    for (int c0 = 0; c0 < a.w; c0 += 8) { // (w is a multiple of 32)
        float wv[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) wv[k] = Wup[(int64_t)(c0 + k) * a.d];
#pragma unroll
        for (int k = 0; k < 8; ++k) p += ab[c0 + k] * wv[k];
    }
    a.pooled[(int64_t)s * a.d + j] = p;
}

// one workgroup per sample: logits, loss term, dz
__global__ __launch_bounds__(256) void k_lhead_a(HeadArgs a)
{
    __shared__ float zpart[256][kMaxClasses];
    __shared__ float z[kMaxClasses];
    const int s = blockIdx.x, t = threadIdx.x;
    const float *Wcls = a.params + a.oWcls, *ccls = a.params + a.occls;
    float zc[kMaxClasses];
#pragma unroll
    for (int c = 0; c < kMaxClasses; ++c) zc[c] = 0.f;
    for (int j = t; j < a.d; j += 256) {
        const float p = a.pooled[(int64_t)s * a.d + j];
#pragma unroll
        for (int c = 0; c < kMaxClasses; ++c)
            if (c < a.C) zc[c] += p * Wcls[(int64_t)j * a.C + c];
    }
#pragma unroll
    for (int c = 0; c < kMaxClasses; ++c) zpart[t][c] = zc[c];
    __syncthreads();
    if (t < a.C) {
        float acc = 0.f;
        for (int k = 0; k < 256; ++k) acc += zpart[k][t];
        z[t] = acc + ccls[t];
    }
    __syncthreads();
    if (t == 0) {
        float mx = z[0];
        for (int c = 1; c < a.C; ++c) mx = fmaxf(mx, z[c]);
        float sum = 0.f;
        for (int c = 0; c < a.C; ++c) sum += expf(z[c] - mx);
        const float lse = mx + logf(sum);
        const int y = a.labels[s];
        a.lossp[s] = lse - z[y];
        for (int c = 0; c < a.C; ++c) {
            a.logits[s * a.C + c] = z[c];
            if (a.logits_out) a.logits_out[s * a.C + c] = z[c];
            a.dz[s * a.C + c] = (expf(z[c] - lse) - (c == y ? 1.f : 0.f)) / (float)a.B;
        }
    }
}

// thread per hidden column j (blockIdx.x) and a chunk of kUpChunk rows of W_up (blockIdx.y): dW_up[c][j] for the
// chunk; the first chunk's blocks also write dp[s][j], dc_up[j], dW_cls[j][.]; block (0, 0) the loss and dc_cls
constexpr int kUpChunk = 8;
__global__ __launch_bounds__(256) void k_lhead_b(HeadArgs a)
{
    __shared__ float dzs[kMaxBatch * kMaxClasses];
    __shared__ float ab[kMaxBatch * kUpChunk];
    const bool first = blockIdx.y == 0;
    const int cbase = blockIdx.y * kUpChunk;
    for (int q = threadIdx.x; q < a.B * a.C; q += 256) dzs[q] = a.dz[q];
    for (int q = threadIdx.x; q < a.B * kUpChunk; q += 256) {
        const int sidx = q / kUpChunk, c = cbase + q % kUpChunk;
        ab[q] = c < a.w ? a.abar[(int64_t)sidx * a.w + c] : 0.f;
    }
    __syncthreads();
    if (first && blockIdx.x == 0 && threadIdx.x == 0) {
        float tot = 0.f;
        for (int s = 0; s < a.B; ++s) tot += a.lossp[s];
        *a.loss_out = tot / (float)a.B;
    }
    if (!a.grads) return;
    if (first && blockIdx.x == 0 && (int)threadIdx.x < a.C) {
        float acc = 0.f;
        for (int s = 0; s < a.B; ++s) acc += dzs[s * a.C + threadIdx.x];
        a.grads[a.occls + threadIdx.x] = acc;
    }
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= a.d) return;
    const float *Wcls = a.params + a.oWcls + (int64_t)j * a.C;
    float wc[kMaxClasses], dwc[kMaxClasses];
#pragma unroll
    for (int c = 0; c < kMaxClasses; ++c) { wc[c] = c < a.C ? Wcls[c] : 0.f; dwc[c] = 0.f; }
    float dcup = 0.f, up[kUpChunk];
#pragma unroll
    for (int c = 0; c < kUpChunk; ++c) up[c] = 0.f;
#pragma unroll 4
    for (int s = 0; s < a.B; ++s) {
        float dp = 0.f;
#pragma unroll
        for (int c = 0; c < kMaxClasses; ++c)
            if (c < a.C) dp += dzs[s * a.C + c] * wc[c];
#pragma unroll
        for (int c = 0; c < kUpChunk; ++c) up[c] += ab[s * kUpChunk + c] * dp;
        if (first) {
            const float pl = a.pooled[(int64_t)s * a.d + j];
#pragma unroll
            for (int c = 0; c < kMaxClasses; ++c)
                if (c < a.C) dwc[c] += pl * dzs[s * a.C + c];
            a.dp[(int64_t)s * a.d + j] = dp;
            dcup += dp;
        }
    }
#pragma unroll
    for (int c = 0; c < kUpChunk; ++c)
        if (cbase + c < a.w) a.grads[a.oWup + (int64_t)(cbase + c) * a.d + j] = up[c];
    if (first) {
        a.grads[a.ocup + j] = dcup;
#pragma unroll
        for (int c = 0; c < kMaxClasses; ++c)
            if (c < a.C) a.grads[a.oWcls + (int64_t)j * a.C + c] = dwc[c];
    }
}

// da_L[s][c] = (dp_s . W_up[c][:]) / len_s for 16 columns c (grid: sample x column chunk), written to every token
// row of the sample
__global__ __launch_bounds__(256) void k_lhead_c(HeadArgs a)
{
    __shared__ float da[16];
    const int s = blockIdx.x, cb = blockIdx.y * 16, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m0 = a.samp_start[s], len = a.samp_len[s];
    const float *Wup = a.params + a.oWup;
    const float *dp = a.dp + (int64_t)s * a.d;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int j = lane; j < a.d; j += 64) {
        const float g = dp[j];
#pragma unroll
        for (int k = 0; k < 4; ++k) acc[k] += g * Wup[(int64_t)min(cb + wave * 4 + k, a.w - 1) * a.d + j];
    }
    wave_sum_n(acc);
    if (lane < 4) da[wave * 4 + lane] = (lane == 0 ? acc[0] : lane == 1 ? acc[1] : lane == 2 ? acc[2] : acc[3]) / (float)len;
    __syncthreads();
    for (int idx = threadIdx.x; idx < len * 16; idx += 256) {
        const int c = cb + (idx & 15);
        if (c < a.w) a.DA_last[(int64_t)(m0 + (idx >> 4)) * a.w + c] = da[idx & 15];
    }
}

// ---------------------------------------------------------------------------
// All contractions over the tokens, one launch: work item = (split, layer, tensor, tile).
//   W_down: b_l^T dx_l    W_qkv: xn_l^T dqkv_l    W_o: o_l^T dt_l    W_1: tn_l^T df1_l    W_2: g_l^T da_l
// The right-hand loader of the first row of tiles keeps the column sums: the bias gradients.
// Results go to part[split] at the tensors' offsets in the parameter vector.
// ---------------------------------------------------------------------------
struct WgArgs {
    const void *cache;
    RowMap map;
    const float *XN, *DQKV, *O, *DT, *TN, *DF1, *G, *DA, *DX;
    float *part;
    int64_t Mmax, PLb, LP; // LP = L * PLb
    int64_t fo[kFields + 1];
    int L, d, w, f, rows_per_split, items_per_layer;
    int tiles_j[5], item0[6];
};
struct EpiSt {
    float *out;
    int ld;
    __device__ void operator()(int row, int col, float v) const { out[(int64_t)row * ld + col] = v; }
};
template <class BL> __device__ __forceinline__ void lad_colsums(BL &bl, float *red, float *dst, int ncols, int j0)
{
    using G = ColsGeom<float, 64, 4>;
    __syncthreads();
    for (int e = 0; e < G::CE; ++e) red[threadIdx.x * G::CE + e] = bl.sums[e];
    __syncthreads();
    if ((int)threadIdx.x < 64) {
        const int col = threadIdx.x, blk = col / G::CE, e = col % G::CE;
        float acc = 0.f;
        for (int t = blk; t < kThreads; t += G::IB) acc += red[t * G::CE + e];
        if (j0 + col < ncols) dst[j0 + col] = acc;
    }
}
template <typename SRC> __global__ __launch_bounds__(256) void k_lwgrad(WgArgs a)
{
    __shared__ __attribute__((aligned(16))) char smem[kTileLds];
    static_assert(kTileLds >= 256 * 4 * 4, "column-sum scratch must fit");
    int b = blockIdx.x;
    const int per_split = a.items_per_layer * a.L;
    const int split = b / per_split;
    b -= split * per_split;
    const int l = b / a.items_per_layer, it = b % a.items_per_layer;
    int t = 0;
    while (t < 4 && it >= a.item0[t + 1]) ++t;
    const int ti = (it - a.item0[t]) / a.tiles_j[t], tj = (it - a.item0[t]) % a.tiles_j[t];
    const int M = a.map.M;
    const int kbegin = split * a.rows_per_split, kend = min(M, kbegin + a.rows_per_split);
    float *part = a.part + (int64_t)split * a.LP + (int64_t)l * a.PLb;
    const int64_t lm = (int64_t)l * a.Mmax;
    const int w = a.w, f = a.f;
    // right-hand operand, output field, bias field, shapes
    const float *Bsrc; int ncolsB; int fieldW, fieldB; const float *Asrc = nullptr; int nrowsA;
    switch (t) {
    case 0: Bsrc = a.DX + lm * w; ncolsB = w; fieldW = F_WD; fieldB = F_CD; nrowsA = a.d; break;
    case 1: Bsrc = a.DQKV + lm * 3 * w; ncolsB = 3 * w; fieldW = F_WQKV; fieldB = F_BQKV; Asrc = a.XN + lm * w; nrowsA = w; break;
    case 2: Bsrc = a.DT + lm * w; ncolsB = w; fieldW = F_WO; fieldB = F_BO; Asrc = a.O + lm * w; nrowsA = w; break;
    case 3: Bsrc = a.DF1 + lm * f; ncolsB = f; fieldW = F_W1; fieldB = F_B1; Asrc = a.TN + lm * w; nrowsA = w; break;
    default: Bsrc = a.DA + lm * w; ncolsB = w; fieldW = F_W2; fieldB = F_B2; Asrc = a.G + lm * f; nrowsA = f; break;
    }
    LoadCols<float, 64, 4, float, true> bl;
    bl.src = Bsrc; bl.ld = ncolsB; bl.ncols = ncolsB; bl.kend = kend;
    EpiSt epi{part + a.fo[fieldW], ncolsB};
    if (kbegin >= kend) return; // (no such item: splits are planned from the batch's own row count)
    if (t == 0) {
        LoadColsCache<SRC, 64, 4> al;
        al.cache = static_cast<const SRC *>(a.cache); al.map = a.map; al.layer = l; al.ncols = a.d; al.kend = kend;
        gemm_tile<float, TL>(smem, al, bl, epi, kbegin, kend, ti * 64, tj * 64, nrowsA, ncolsB);
    } else {
        LoadCols<float, 64, 4, float, false> al;
        al.src = Asrc; al.ld = nrowsA; al.ncols = nrowsA; al.kend = kend;
        gemm_tile<float, TL>(smem, al, bl, epi, kbegin, kend, ti * 64, tj * 64, nrowsA, ncolsB);
    }
    if (ti == 0) lad_colsums(bl, reinterpret_cast<float *>(smem), part + a.fo[fieldB], ncolsB, tj * 64);
}

// ordered sums into the gradient vector: thread per element of the layer blocks
struct RedArgs {
    const float *part, *ln1p, *ln2p, *dlamp, *params;
    float *grads;
    int64_t PLb, LP;
    int64_t fo[kFields + 1];
    int L, w, splits, nblk;
};
__global__ __launch_bounds__(256) void k_lreduce(RedArgs a)
{
    const int eblocks = (int)((a.LP + 255) / 256);
    if ((int)blockIdx.x >= eblocks) {
        // norm gains / offsets and the gate: one wavefront per element sums the row-block partials (lanes take
        // every 64th block, then a fixed exchange pattern: the same order on every run)
        const int lane = threadIdx.x & 63;
        const int task = ((int)blockIdx.x - eblocks) * 4 + (threadIdx.x >> 6);
        const int per_layer = 4 * a.w + 1;
        if (task >= a.L * per_layer) return;
        const int l = task / per_layer, e = task % per_layer;
        float acc = 0.f;
        int64_t dst;
        if (e == 4 * a.w) {
            for (int k = lane; k < a.nblk; k += 64) acc += a.dlamp[(int64_t)l * a.nblk + k];
            dst = a.fo[F_LAM];
        } else {
            const int which = e / a.w, c = e % a.w; // 0: ln1 gain, 1: ln1 offset, 2: ln2 gain, 3: ln2 offset
            const float *p = (which < 2 ? a.ln1p : a.ln2p) + (int64_t)l * a.nblk * 2 * a.w + (which & 1) * a.w + c;
            for (int k = lane; k < a.nblk; k += 64) acc += p[(int64_t)k * 2 * a.w];
            dst = a.fo[which == 0 ? F_G1 : which == 1 ? F_H1 : which == 2 ? F_G2 : F_H2] + c;
        }
        acc = wave_sum(acc);
        if (lane == 0) a.grads[(int64_t)l * a.PLb + dst] = acc;
        return;
    }
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= a.LP) return;
    const int l = (int)(i / a.PLb);
    const int64_t o = i - (int64_t)l * a.PLb;
    int fld = 0;
    while (fld < kFields - 1 && o >= a.fo[fld + 1]) ++fld;
    if (fld == F_G1 || fld == F_H1 || fld == F_G2 || fld == F_H2) return;
    float acc = 0.f;
    if (fld == F_LAM) {
        if (o == a.fo[F_LAM]) return;
    } else {
        for (int s = 0; s < a.splits; ++s) acc += a.part[(int64_t)s * a.LP + i];
        if (fld == F_WD || fld == F_CD) acc *= a.params[(int64_t)l * a.PLb + a.fo[F_LAM]]; // du = lambda dx
    }
    a.grads[i] = acc;
}

// AdamW over the ladder's parameter vector: decoupled decay on the matrices only
struct LAdamArgs {
    float *p, *m, *v;
    const float *g;
    int64_t P, PLb, LP, oWup, ocup, oWcls, occls;
    int64_t fo[kFields + 1];
    AdamArgs h;
};
__global__ __launch_bounds__(256) void k_ladamw(LAdamArgs a)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < a.P; i += (int64_t)gridDim.x * 256) {
        bool dec;
        if (i < a.LP) {
            const int64_t o = i % a.PLb;
            int fld = 0;
            while (fld < kFields - 1 && o >= a.fo[fld + 1]) ++fld;
            dec = fld == F_WD || fld == F_WQKV || fld == F_WO || fld == F_W1 || fld == F_W2;
        } else {
            dec = i < a.ocup || (i >= a.oWcls && i < a.occls);
        }
        const float g = a.g[i];
        float p = a.p[i];
        const float m = a.h.beta1 * a.m[i] + (1.f - a.h.beta1) * g;
        const float v = a.h.beta2 * a.v[i] + (1.f - a.h.beta2) * g * g;
        if (dec) p -= a.h.lr * a.h.wd * p;
        p -= a.h.lr * (m / a.h.bc1) / (sqrtf(v / a.h.bc2) + a.h.eps);
        a.p[i] = p; a.m[i] = m; a.v[i] = v;
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
template <auto Kern> hipError_t lds_once(int bytes)
{
    static std::once_flag once;
    static hipError_t result = hipSuccess;
    std::call_once(once, [&] {
        result = hipFuncSetAttribute(reinterpret_cast<const void *>(Kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     160 * 1024);
    });
    (void)bytes;
    return result;
}

template <int DH> hipError_t launch_attn(bool bwd, const AttnArgs &a, int B, hipStream_t st, Profiler *prof)
{
    if (!bwd) {
        const int lds = 2 * a.n_max * DH * 4;
        LAD_TRY((lds_once<&k_lattn_fwd<DH>>(lds)));
        LAD_LAUNCH(prof, st, KC_L_ATTN, (k_lattn_fwd<DH>), dim3(B * a.nh, a.nchunk), dim3(256), lds, st, a);
    } else {
        const int lds = (4 * a.n_max * DH + 2 * a.n_max) * 4;
        LAD_TRY((lds_once<&k_lattn_bwd<DH>>(lds)));
        LAD_LAUNCH(prof, st, KC_L_ATTN, (k_lattn_bwd<DH>), dim3(B * a.nh, a.nchunk), dim3(256), lds, st, a);
    }
    return hipSuccess;
}

hipError_t attn(int dh, bool bwd, const AttnArgs &a, int B, hipStream_t st, Profiler *prof)
{
    switch (dh) {
    case 4: return launch_attn<4>(bwd, a, B, st, prof);
    case 8: return launch_attn<8>(bwd, a, B, st, prof);
    case 16: return launch_attn<16>(bwd, a, B, st, prof);
    case 32: return launch_attn<32>(bwd, a, B, st, prof);
    case 64: return launch_attn<64>(bwd, a, B, st, prof);
    }
    return hipErrorInvalidValue;
}

template <bool BT, int EPI>
void lin(Profiler *prof, hipStream_t st, int cls, const float *A, int lda, const float *B, int ldb, int M, int N, int K,
         const float *bias, const float *res, const float *aux, float *out, float *out2)
{
    LinArgs a{A, lda, B, ldb, M, N, K, bias, res, aux, out, out2};
    if (N <= 128 && K > 128) { // narrow output, long contraction: 16 x 16 blocks
        LAD_LAUNCH(prof, st, cls, (k_llin16<BT, EPI>), dim3(cdivi(M, 32), cdivi(N, 32)), dim3(256), 0, st, a);
        return;
    }
    LAD_LAUNCH(prof, st, cls, (k_llin<BT, EPI>), dim3(cdivi(M, 64), cdivi(N, 64)), dim3(256), 0, st, a);
}

template <typename SRC>
hipError_t run_ladder(const Lad &a, const BatchMeta &meta, const void *cache, const int32_t *labels, const float *params,
                      char *ws, float *loss_out, float *logits_out, float *grads, hipStream_t st, Profiler *prof)
{
    const int M = meta.M, B = meta.B, L = a.L, w = a.w, f = a.f, d = a.d;
    auto F = [&](int64_t off) { return reinterpret_cast<float *>(ws + off); };
    int64_t *rowoff = reinterpret_cast<int64_t *>(ws + a.rowoff);
    int32_t *rowstride = reinterpret_cast<int32_t *>(ws + a.rowstride), *rowsamp = reinterpret_cast<int32_t *>(ws + a.rowsamp);
    int32_t *samp_start = reinterpret_cast<int32_t *>(ws + a.samp_start), *samp_len = reinterpret_cast<int32_t *>(ws + a.samp_len);
    const RowMap map{rowoff, rowstride, M};
    const int64_t Mm = a.Mmax;
    const int nblk = cdivi(M, kLnRows); // workgroups of the LayerNorm reverse kernels: stride of their partial sums
    auto lay = [&](int64_t off, int l, int width) { return F(off) + (int64_t)l * Mm * width; };

    LAD_LAUNCH(prof, st, KC_SETUP, k_lsetup, dim3(cdivi(M, 256)), dim3(256), 0, st, meta, d, rowoff, rowstride, rowsamp,
               samp_start, samp_len);
    {
        DownArgs da{cache, map, params, a.PLb, a.fo[F_WD], a.fo[F_CD], d, w, F(a.U), Mm};
        if (std::is_same<SRC, bf16_t>::value && a.Wsp >= 0) {
            bf16_t *Wsp = reinterpret_cast<bf16_t *>(ws + a.Wsp);
            LAD_LAUNCH(prof, st, KC_L_DOWN, k_lsplit, dim3(cdivi(d, 64), L, w / 32), dim3(256), 0, st, params, a.PLb, a.fo[F_WD], d, w, Wsp);
            const dim3 grid(cdivi(M, 128), L);
            switch (w / 32) {
            case 1: LAD_TRY((lds_once<&k_ldown3<1>>(0))); LAD_LAUNCH(prof, st, KC_L_DOWN, (k_ldown3<1>), grid, dim3(256), Down3Shapes<1>::TL::LDS_BYTES, st, da, Wsp); break;
            case 2: LAD_TRY((lds_once<&k_ldown3<2>>(0))); LAD_LAUNCH(prof, st, KC_L_DOWN, (k_ldown3<2>), grid, dim3(256), Down3Shapes<2>::TL::LDS_BYTES, st, da, Wsp); break;
            case 3: LAD_TRY((lds_once<&k_ldown3<3>>(0))); LAD_LAUNCH(prof, st, KC_L_DOWN, (k_ldown3<3>), grid, dim3(256), Down3Shapes<3>::TL::LDS_BYTES, st, da, Wsp); break;
            default: LAD_TRY((lds_once<&k_ldown3<4>>(0))); LAD_LAUNCH(prof, st, KC_L_DOWN, (k_ldown3<4>), grid, dim3(256), Down3Shapes<4>::TL::LDS_BYTES, st, da, Wsp); break;
            }
        } else {
            LAD_LAUNCH(prof, st, KC_L_DOWN, (k_ldown<SRC>), dim3(cdivi(M, 64), cdivi(w, 64), L), dim3(256), 0, st, da);
        }
    }
    const float scale = 1.f / sqrtf((float)a.dh);
    int nlong = 1; // longest sample of the batch: lanes per attention row so that its rows fill a workgroup
    for (int i = 0; i < B; ++i) nlong = meta.len[i] > nlong ? meta.len[i] : nlong;
    // several workgroups per sample and head (about 64 rows each: measured against 32 and 128 at 128-token samples),
    // the rows of one shared by up to 8 lanes
    int nchunk = nlong / 64;
    nchunk = nchunk < 1 ? 1 : (nchunk > 8 ? 8 : nchunk);
    const int rows_per_wg = (nlong + nchunk - 1) / nchunk;
    int tpr = 1;
    while (tpr < 8 && 2 * tpr * rows_per_wg <= 256) tpr *= 2;
    for (int l = 0; l < L; ++l) {
        const float *pl = params + (int64_t)l * a.PLb;
        if (w <= 128) { // gate, LayerNorm 1 and the q, k, v projection in one launch
            QkvArgs qa{lay(a.U, l, w), l ? lay(a.A, l - 1, w) : nullptr, pl + a.fo[F_LAM], pl + a.fo[F_G1], pl + a.fo[F_H1],
                       pl + a.fo[F_WQKV], pl + a.fo[F_BQKV], lay(a.X, l, w), lay(a.XN, l, w), lay(a.st1, l, 2),
                       lay(a.QKV, l, 3 * w), M};
            const dim3 grid(cdivi(M, 16));
            switch (w / 32) {
            case 1: LAD_LAUNCH(prof, st, KC_L_LIN, (k_lqkv_fwd<1>), grid, dim3(256), 0, st, qa); break;
            case 2: LAD_LAUNCH(prof, st, KC_L_LIN, (k_lqkv_fwd<2>), grid, dim3(256), 0, st, qa); break;
            case 3: LAD_LAUNCH(prof, st, KC_L_LIN, (k_lqkv_fwd<3>), grid, dim3(256), 0, st, qa); break;
            default: LAD_LAUNCH(prof, st, KC_L_LIN, (k_lqkv_fwd<4>), grid, dim3(256), 0, st, qa); break;
            }
        } else {
        LnFwdArgs n1{lay(a.U, l, w), l ? lay(a.A, l - 1, w) : nullptr, pl + a.fo[F_LAM], pl + a.fo[F_G1], pl + a.fo[F_H1],
                     lay(a.X, l, w), lay(a.XN, l, w), lay(a.st1, l, 2), M, w};
        LAD_LAUNCH(prof, st, KC_L_ROW, (k_lln_fwd<true>), dim3(cdivi(M, 4)), dim3(256), 0, st, n1);
        lin<false, 0>(prof, st, KC_L_LIN, lay(a.XN, l, w), w, pl + a.fo[F_WQKV], 3 * w, M, 3 * w, w, pl + a.fo[F_BQKV],
                      nullptr, nullptr, lay(a.QKV, l, 3 * w), nullptr);
        }
        AttnArgs at{lay(a.QKV, l, 3 * w), samp_start, samp_len, lay(a.O, l, w), lay(a.LSE, l, a.nh), nullptr, nullptr, w,
                    a.nh, (int)(Mm / a.Bmax), scale, tpr, nchunk};
        LAD_TRY(attn(a.dh, false, at, B, st, prof));
        if (w <= 128) { // the rest of the layer in one launch
            MlpArgs ma{lay(a.O, l, w), lay(a.X, l, w), pl + a.fo[F_WO], pl + a.fo[F_BO], pl + a.fo[F_G2], pl + a.fo[F_H2],
                       pl + a.fo[F_W1], pl + a.fo[F_B1], pl + a.fo[F_W2], pl + a.fo[F_B2], lay(a.T, l, w), lay(a.TN, l, w),
                       lay(a.st2, l, 2), lay(a.F1, l, f), lay(a.G, l, f), lay(a.A, l, w), M};
            const dim3 grid(cdivi(M, 16));
            switch (w / 32) {
            case 1: LAD_LAUNCH(prof, st, KC_L_LIN, (k_lmlp_fwd<1>), grid, dim3(256), mlp_lds_bytes<1>(), st, ma); break;
            case 2: LAD_LAUNCH(prof, st, KC_L_LIN, (k_lmlp_fwd<2>), grid, dim3(256), mlp_lds_bytes<2>(), st, ma); break;
            case 3: LAD_TRY((lds_once<&k_lmlp_fwd<3>>(mlp_lds_bytes<3>())));
                    LAD_LAUNCH(prof, st, KC_L_LIN, (k_lmlp_fwd<3>), grid, dim3(256), mlp_lds_bytes<3>(), st, ma); break;
            default: LAD_TRY((lds_once<&k_lmlp_fwd<4>>(mlp_lds_bytes<4>())));
                    LAD_LAUNCH(prof, st, KC_L_LIN, (k_lmlp_fwd<4>), grid, dim3(256), mlp_lds_bytes<4>(), st, ma); break;
            }
            continue;
        }
        lin<false, 1>(prof, st, KC_L_LIN, lay(a.O, l, w), w, pl + a.fo[F_WO], w, M, w, w, pl + a.fo[F_BO], lay(a.X, l, w),
                      nullptr, lay(a.T, l, w), nullptr);
        LnFwdArgs n2{lay(a.T, l, w), nullptr, nullptr, pl + a.fo[F_G2], pl + a.fo[F_H2], nullptr, lay(a.TN, l, w),
                     lay(a.st2, l, 2), M, w};
        LAD_LAUNCH(prof, st, KC_L_ROW, (k_lln_fwd<false>), dim3(cdivi(M, 4)), dim3(256), 0, st, n2);
        lin<false, 2>(prof, st, KC_L_LIN, lay(a.TN, l, w), w, pl + a.fo[F_W1], f, M, f, w, pl + a.fo[F_B1], nullptr, nullptr,
                      lay(a.F1, l, f), lay(a.G, l, f));
        lin<false, 1>(prof, st, KC_L_LIN, lay(a.G, l, f), f, pl + a.fo[F_W2], w, M, w, f, pl + a.fo[F_B2], lay(a.T, l, w),
                      nullptr, lay(a.A, l, w), nullptr);
    }
    HeadArgs h{cache, map, samp_start, samp_len, labels, params, a.oWup, a.ocup, a.oWcls, a.occls, lay(a.A, L - 1, w),
               F(a.bmean), F(a.abar), F(a.pooled), F(a.logits), F(a.dz), F(a.dp), F(a.daL), F(a.lossp),
               lay(a.DA, L - 1, w), loss_out, logits_out, grads, B, d, w, a.C, L - 1};
    LAD_LAUNCH(prof, st, KC_L_HEAD, (k_lpool<SRC>), dim3(B, cdivi(d, 256) + 1), dim3(256), 0, st, h);
    LAD_LAUNCH(prof, st, KC_L_HEAD, k_lpooled, dim3(B, cdivi(d, 256)), dim3(256), 0, st, h);
    LAD_LAUNCH(prof, st, KC_L_HEAD, k_lhead_a, dim3(B), dim3(256), 0, st, h);
    LAD_LAUNCH(prof, st, KC_L_HEAD, k_lhead_b, dim3(cdivi(d, 256), grads ? cdivi(w, kUpChunk) : 1), dim3(256), 0, st, h);
    if (!grads) return hipGetLastError();
    LAD_LAUNCH(prof, st, KC_L_HEAD, k_lhead_c, dim3(B, cdivi(w, 16)), dim3(256), 0, st, h);

    if (w <= 128)
        LAD_LAUNCH(prof, st, KC_SETUP, k_ltrans, dim3(cdivi(2 * w * f + 4 * w * w, 256), L), dim3(256), 0, st, params, a.PLb,
                   a.fo[F_W2], a.fo[F_W1], a.fo[F_WO], a.fo[F_WQKV], w, F(a.WT));
    for (int l = L - 1; l >= 0; --l) {
        const float *pl = params + (int64_t)l * a.PLb;
        float *DA = lay(a.DA, l, w), *DF1 = lay(a.DF1, l, f), *DT = lay(a.DT, l, w), *DQKV = lay(a.DQKV, l, 3 * w);
        float *DX = lay(a.DX, l, w);
        if (w <= 128) { // the reverse of the layer's tail in one launch
            const float *wt = F(a.WT) + (int64_t)l * (2 * w * f + 4 * w * w);
            MlpBwdArgs mb{DA, lay(a.F1, l, f), lay(a.T, l, w), lay(a.st2, l, 2), wt, wt + (int64_t)w * f, wt + (int64_t)2 * w * f,
                          pl + a.fo[F_G2], DF1, DT, F(a.DO_), F(a.ln2p) + (int64_t)l * nblk * 2 * w, M};
            const dim3 grid(cdivi(M, 16));
            switch (w / 32) {
            case 1: LAD_LAUNCH(prof, st, KC_L_LIN, (k_lmlp_bwd<1>), grid, dim3(256), mlp_bwd_lds_bytes<1>(), st, mb); break;
            case 2: LAD_LAUNCH(prof, st, KC_L_LIN, (k_lmlp_bwd<2>), grid, dim3(256), mlp_bwd_lds_bytes<2>(), st, mb); break;
            case 3: LAD_TRY((lds_once<&k_lmlp_bwd<3>>(mlp_bwd_lds_bytes<3>())));
                    LAD_LAUNCH(prof, st, KC_L_LIN, (k_lmlp_bwd<3>), grid, dim3(256), mlp_bwd_lds_bytes<3>(), st, mb); break;
            default: LAD_TRY((lds_once<&k_lmlp_bwd<4>>(mlp_bwd_lds_bytes<4>())));
                    LAD_LAUNCH(prof, st, KC_L_LIN, (k_lmlp_bwd<4>), grid, dim3(256), mlp_bwd_lds_bytes<4>(), st, mb); break;
            }
        } else {
        // dg = da W_2^T, df1 = dg * GELU'(f1)
        lin<true, 3>(prof, st, KC_L_LIN, DA, w, pl + a.fo[F_W2], w, M, f, w, nullptr, nullptr, lay(a.F1, l, f), DF1, nullptr);
        // dtn = df1 W_1^T
        lin<true, 4>(prof, st, KC_L_LIN, DF1, f, pl + a.fo[F_W1], f, M, w, f, nullptr, nullptr, nullptr, F(a.DTN), nullptr);
        LnBwdArgs b2{F(a.DTN), lay(a.T, l, w), lay(a.st2, l, 2), pl + a.fo[F_G2], DA, DT,
                     F(a.ln2p) + (int64_t)l * nblk * 2 * w, nullptr, nullptr, nullptr, nullptr, nullptr, M, w};
        LAD_LAUNCH(prof, st, KC_L_ROW, (k_lln_bwd<false>), dim3(cdivi(M, kLnRows)), dim3(256), 0, st, b2);
        // do = dt W_o^T
        lin<true, 4>(prof, st, KC_L_LIN, DT, w, pl + a.fo[F_WO], w, M, w, w, nullptr, nullptr, nullptr, F(a.DO_), nullptr);
        }
        AttnArgs at{lay(a.QKV, l, 3 * w), samp_start, samp_len, lay(a.O, l, w), lay(a.LSE, l, a.nh), F(a.DO_), DQKV, w,
                    a.nh, (int)(Mm / a.Bmax), scale, tpr, nchunk};
        LAD_TRY(attn(a.dh, true, at, B, st, prof));
        if (w <= 128) { // dxn, the reverse of LayerNorm 1 and of the gate in one launch
            const float *wt = F(a.WT) + (int64_t)l * (2 * w * f + 4 * w * w) + (int64_t)2 * w * f + (int64_t)w * w;
            QkvBwdArgs qb{DQKV, wt, lay(a.X, l, w), lay(a.st1, l, 2), pl + a.fo[F_G1], DT, lay(a.U, l, w),
                          l ? lay(a.A, l - 1, w) : nullptr, pl + a.fo[F_LAM], DX, l ? lay(a.DA, l - 1, w) : nullptr,
                          F(a.ln1p) + (int64_t)l * nblk * 2 * w, F(a.dlamp) + (int64_t)l * nblk, M};
            const dim3 grid(cdivi(M, 16));
            switch (w / 32) {
            case 1: LAD_LAUNCH(prof, st, KC_L_LIN, (k_lqkv_bwd<1>), grid, dim3(256), qkv_bwd_lds_bytes<1>(), st, qb); break;
            case 2: LAD_LAUNCH(prof, st, KC_L_LIN, (k_lqkv_bwd<2>), grid, dim3(256), qkv_bwd_lds_bytes<2>(), st, qb); break;
            case 3: LAD_LAUNCH(prof, st, KC_L_LIN, (k_lqkv_bwd<3>), grid, dim3(256), qkv_bwd_lds_bytes<3>(), st, qb); break;
            default: LAD_TRY((lds_once<&k_lqkv_bwd<4>>(qkv_bwd_lds_bytes<4>())));
                    LAD_LAUNCH(prof, st, KC_L_LIN, (k_lqkv_bwd<4>), grid, dim3(256), qkv_bwd_lds_bytes<4>(), st, qb); break;
            }
            continue;
        }
        // dxn = dqkv W_qkv^T
        lin<true, 4>(prof, st, KC_L_LIN, DQKV, 3 * w, pl + a.fo[F_WQKV], 3 * w, M, w, 3 * w, nullptr, nullptr, nullptr,
                     F(a.DXN), nullptr);
        LnBwdArgs b1{F(a.DXN), lay(a.X, l, w), lay(a.st1, l, 2), pl + a.fo[F_G1], DT, DX,
                     F(a.ln1p) + (int64_t)l * nblk * 2 * w, lay(a.U, l, w), l ? lay(a.A, l - 1, w) : nullptr,
                     pl + a.fo[F_LAM], l ? lay(a.DA, l - 1, w) : nullptr, F(a.dlamp) + (int64_t)l * nblk, M, w};
        LAD_LAUNCH(prof, st, KC_L_ROW, (k_lln_bwd<true>), dim3(cdivi(M, kLnRows)), dim3(256), 0, st, b1);
    }
    // token contractions: splits planned for the largest batch, the rows of this batch dealt over them
    const int rps = cdivi(cdivi(M, a.splits), 64) * 64;
    const int splits = cdivi(M, rps);
    WgArgs wg;
    wg.cache = cache; wg.map = map;
    wg.XN = F(a.XN); wg.DQKV = F(a.DQKV); wg.O = F(a.O); wg.DT = F(a.DT); wg.TN = F(a.TN); wg.DF1 = F(a.DF1);
    wg.G = F(a.G); wg.DA = F(a.DA); wg.DX = F(a.DX);
    wg.part = F(a.part); wg.Mmax = Mm; wg.PLb = a.PLb; wg.LP = (int64_t)L * a.PLb;
    for (int i = 0; i <= kFields; ++i) wg.fo[i] = a.fo[i];
    wg.L = L; wg.d = d; wg.w = w; wg.f = f; wg.rows_per_split = rps; wg.items_per_layer = a.items_per_layer;
    for (int t = 0; t < 5; ++t) wg.tiles_j[t] = a.tiles[t][1];
    for (int t = 0; t < 6; ++t) wg.item0[t] = a.item0[t];
    LAD_LAUNCH(prof, st, KC_L_WGRAD, (k_lwgrad<SRC>), dim3(splits * L * a.items_per_layer), dim3(256), 0, st, wg);
    RedArgs rd;
    rd.part = F(a.part); rd.ln1p = F(a.ln1p); rd.ln2p = F(a.ln2p); rd.dlamp = F(a.dlamp); rd.params = params;
    rd.grads = grads; rd.PLb = a.PLb; rd.LP = (int64_t)L * a.PLb;
    for (int i = 0; i <= kFields; ++i) rd.fo[i] = a.fo[i];
    rd.L = L; rd.w = w; rd.splits = splits; rd.nblk = nblk;
    LAD_LAUNCH(prof, st, KC_L_REDUCE, k_lreduce, dim3(cdivi(rd.LP, 256) + cdivi((int64_t)L * (4 * w + 1), 4)), dim3(256), 0, st, rd);
    return hipGetLastError();
}

pac_status ladder_common(pac_ctx *ctx, const void *cache, const int64_t *sample_ids, int32_t B, const int32_t *labels,
                         int32_t heads, const float *params, void *workspace, int64_t workspace_bytes, float *loss_out,
                         float *logits_out, float *grads, void *hip_stream, Lad &a)
{
    if (!ctx || !cache || !sample_ids || !labels || !params || !workspace || !loss_out) return PAC_ERR_NULL;
    auto al = [](const void *p, uintptr_t n) { return (reinterpret_cast<uintptr_t>(p) & (n - 1)) == 0; };
    if (!al(cache, 256) || !al(workspace, 256) || !al(params, 16) || !al(labels, 4) || !al(loss_out, 4) ||
        (logits_out && !al(logits_out, 4)) || (grads && !al(grads, 16)))
        return PAC_ERR_ALIGN;
    if (!lad_plan(ctx->D, heads, a)) return PAC_ERR_UNSUPPORTED;
    if (workspace_bytes < a.total) return PAC_ERR_WORKSPACE;
    BatchMeta meta;
    pac_status s = (pac_status)pac_ctx_build_meta(ctx, sample_ids, B, meta);
    if (s != PAC_OK) return s;
    (void)hipGetLastError();
    Profiler *prof = ctx->prof.on ? &ctx->prof : nullptr;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    char *ws = static_cast<char *>(workspace);
    hipError_t e = a.cache_f32 ? run_ladder<float>(a, meta, cache, labels, params, ws, loss_out, logits_out, grads, st, prof)
                               : run_ladder<bf16_t>(a, meta, cache, labels, params, ws, loss_out, logits_out, grads, st, prof);
    return e == hipSuccess ? PAC_OK : PAC_ERR_DEVICE;
}

} // namespace
} // namespace pac

using namespace pac;

extern "C" {

int64_t pac_ladder_param_count(const pac_ctx *ctx)
{
    if (!ctx) return -1;
    Lad a;
    return lad_shapes(ctx->D, a) ? a.P : -1;
}

int64_t pac_ladder_workspace_bytes(const pac_ctx *ctx, int32_t heads)
{
    if (!ctx) return -1;
    Lad a;
    return lad_plan(ctx->D, heads, a) ? a.total : -1;
}

pac_status pac_ladder_loss_grad(pac_ctx *ctx, const void *cache, const int64_t *sample_ids, int32_t B,
                                const int32_t *labels, int32_t heads, const float *params, void *workspace,
                                int64_t workspace_bytes, float *loss_out, float *logits_out, float *grads_out,
                                void *hip_stream)
{
    Lad a;
    return ladder_common(ctx, cache, sample_ids, B, labels, heads, params, workspace, workspace_bytes, loss_out, logits_out,
                         grads_out, hip_stream, a);
}

pac_status pac_ladder_step(pac_ctx *ctx, const void *cache, const int64_t *sample_ids, int32_t B, const int32_t *labels,
                           int32_t heads, float *params, float *m, float *v, int64_t *step, const pac_adamw *hp,
                           void *workspace, int64_t workspace_bytes, float *loss_out, float *grads_out, void *hip_stream)
{
    if (!m || !v || !step || !hp) return PAC_ERR_NULL;
    if (*step < 0) return PAC_ERR_RANGE;
    if (!(hp->beta1 >= 0.f && hp->beta1 < 1.f) || !(hp->beta2 >= 0.f && hp->beta2 < 1.f) || !(hp->eps >= 0.f) ||
        !(hp->lr >= 0.f) || !(hp->weight_decay >= 0.f))
        return PAC_ERR_RANGE;
    Lad a;
    if (!ctx) return PAC_ERR_NULL;
    if (!lad_plan(ctx->D, heads, a)) return PAC_ERR_UNSUPPORTED;
    float *grads = grads_out ? grads_out : (workspace ? reinterpret_cast<float *>(static_cast<char *>(workspace) + a.grads) : nullptr);
    pac_status s = ladder_common(ctx, cache, sample_ids, B, labels, heads, params, workspace, workspace_bytes, loss_out,
                                 nullptr, grads, hip_stream, a);
    if (s != PAC_OK) return s;
    const int64_t t = *step + 1;
    LAdamArgs aa;
    aa.p = params; aa.m = m; aa.v = v; aa.g = grads;
    aa.P = a.P; aa.PLb = a.PLb; aa.LP = (int64_t)a.L * a.PLb; aa.oWup = a.oWup; aa.ocup = a.ocup; aa.oWcls = a.oWcls;
    aa.occls = a.occls;
    for (int i = 0; i <= kFields; ++i) aa.fo[i] = a.fo[i];
    aa.h.lr = hp->lr; aa.h.beta1 = hp->beta1; aa.h.beta2 = hp->beta2; aa.h.eps = hp->eps; aa.h.wd = hp->weight_decay;
    aa.h.bc1 = (float)(1.0 - pow((double)hp->beta1, (double)t));
    aa.h.bc2 = (float)(1.0 - pow((double)hp->beta2, (double)t));
    aa.h.inv_bc1 = (float)(1.0 / (1.0 - pow((double)hp->beta1, (double)t)));
    aa.h.inv_bc2 = (float)(1.0 / (1.0 - pow((double)hp->beta2, (double)t)));
    int64_t nb = (a.P + 255) / 256; // one element per thread
    if (nb > (int64_t)1 << 22) nb = (int64_t)1 << 22;
    const int blocks = (int)nb;
    Profiler *prof = ctx->prof.on ? &ctx->prof : nullptr;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    LAD_LAUNCH(prof, st, KC_ADAMW, k_ladamw, dim3(blocks), dim3(256), 0, st, aa);
    if (hipGetLastError() != hipSuccess) return PAC_ERR_DEVICE;
    *step = t;
    return PAC_OK;
}

} // extern "C"
