// LDS-tiled MFMA contraction core for gfx950, shared by the per-layer kernels.
//
// One workgroup = 256 threads = 4 wavefronts (64 lanes each) arranged 2 x 2;
// every wavefront owns WTM x WTN accumulator tiles of 32 x 32, so the
// workgroup tile is (64*WTM) x (64*WTN).  Operands are staged through LDS in a
// K-contiguous layout for both sides ("A[i][k]" and "B[j][k]"), 64 bytes of K
// per row per step plus 16 bytes of padding, which is what the 32x32 MFMA
// wants: lane (i = lane%32, g = lane/32) supplies KV consecutive K values of
// row i (8 bf16, or 1 fp32), and the instruction contracts 2*KV of K.
// Because both operands use the same (g, element) -> K assignment, the result
// does not depend on how the hardware labels K inside an instruction.
//
// Accumulator layout of the 32x32 MFMA (public CDNA ISA): register v of lane l
// holds C[8*(v/4) + 4*(l/32) + v%4][l%32].
//
// The loaders decide what an operand *is*: a plain row-major matrix, an fp32
// matrix converted on the fly, a transposed view (for reductions over tokens),
// or the gated adapter input x = lambda*b + (1-lambda)*s built from the cache.
// The next K step is fetched into registers while the current one is in the
// matrix cores.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pac {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kRowBytes = 64;   // bytes of K staged per row per step
constexpr int kPitchBytes = 80; // LDS row pitch (64 + 16 padding)

template <typename TC> struct Traits;
template <> struct Traits<bf16_t> {
    static constexpr int CE = 8;   // elements per 16-byte chunk
    static constexpr int KV = 8;   // K values a lane feeds to one MFMA
    static constexpr int BK = 32;  // K elements per step
    static constexpr int LDP = 40; // LDS pitch in elements
};
template <> struct Traits<float> {
    static constexpr int CE = 4;
    static constexpr int KV = 1;
    static constexpr int BK = 16;
    static constexpr int LDP = 20;
};

// 16 bytes of compute-type elements
template <typename TC> struct alignas(16) Chunk { TC e[Traits<TC>::CE]; };

__device__ __forceinline__ bf16_t to_tc(float f, bf16_t) { return static_cast<bf16_t>(f); }
__device__ __forceinline__ float to_tc(float f, float) { return f; }
__device__ __forceinline__ float to_f32(bf16_t h) { return static_cast<float>(h); }
__device__ __forceinline__ float to_f32(float f) { return f; }

// ---------------------------------------------------------------------------
// Row-major loaders: operand[row][k] = src[row][k] (K contiguous in memory).
// Thread t handles rows t/4 + 64u (u < WT) and the 16-byte K chunk t%4.
// ---------------------------------------------------------------------------
template <typename TC, int WT> struct LoadRowsTC {
    using T = Traits<TC>;
    const TC *src;
    int64_t ld;
    int nrows;
    const TC *rp[WT];
    uint4 reg[WT];
    __device__ void init(int row0)
    {
        const int t = threadIdx.x;
        for (int u = 0; u < WT; ++u) {
            int row = row0 + (t >> 2) + 64 * u;
            rp[u] = row < nrows ? src + (int64_t)row * ld + (t & 3) * T::CE : nullptr;
        }
    }
    __device__ void fetch(int k0)
    {
        for (int u = 0; u < WT; ++u)
            reg[u] = rp[u] ? *reinterpret_cast<const uint4 *>(rp[u] + k0) : make_uint4(0, 0, 0, 0);
    }
    __device__ void store(TC *lds)
    {
        const int t = threadIdx.x;
        for (int u = 0; u < WT; ++u)
            *reinterpret_cast<uint4 *>(lds + ((t >> 2) + 64 * u) * T::LDP + (t & 3) * T::CE) = reg[u];
    }
};

template <typename TC, int WT> struct LoadRowsF32 {
    using T = Traits<TC>;
    const float *src;
    int64_t ld;
    int nrows;
    const float *rp[WT];
    Chunk<TC> reg[WT];
    __device__ void init(int row0)
    {
        const int t = threadIdx.x;
        for (int u = 0; u < WT; ++u) {
            int row = row0 + (t >> 2) + 64 * u;
            rp[u] = row < nrows ? src + (int64_t)row * ld + (t & 3) * T::CE : nullptr;
        }
    }
    __device__ void fetch(int k0)
    {
        for (int u = 0; u < WT; ++u) {
            if (rp[u]) {
                for (int q = 0; q < T::CE / 4; ++q) {
                    float4 f = *reinterpret_cast<const float4 *>(rp[u] + k0 + 4 * q);
                    reg[u].e[4 * q + 0] = to_tc(f.x, TC());
                    reg[u].e[4 * q + 1] = to_tc(f.y, TC());
                    reg[u].e[4 * q + 2] = to_tc(f.z, TC());
                    reg[u].e[4 * q + 3] = to_tc(f.w, TC());
                }
            } else {
                for (int e = 0; e < T::CE; ++e) reg[u].e[e] = to_tc(0.f, TC());
            }
        }
    }
    __device__ void store(TC *lds)
    {
        const int t = threadIdx.x;
        for (int u = 0; u < WT; ++u)
            *reinterpret_cast<Chunk<TC> *>(lds + ((t >> 2) + 64 * u) * T::LDP + (t & 3) * T::CE) = reg[u];
    }
};

// Where the rows of a batch live in the cache: token row m of layer l starts at
// cache + rowoff[m] + l * rowstride[m]   (elements).
struct RowMap {
    const int64_t *rowoff;
    const int32_t *rowstride;
    int M;
};

// x[m][k] = lam * b_l[m][k] + (1 - lam) * s_prev[m][k]   (s_prev == nullptr: s = 0)
template <typename TC, int WT> struct LoadRowsX {
    using T = Traits<TC>;
    const TC *cache;
    RowMap map;
    int layer;
    const float *s_prev;
    int64_t ld_s;
    float lam;
    const TC *bp[WT];
    const float *sp[WT];
    Chunk<TC> reg[WT];
    __device__ void init(int row0)
    {
        const int t = threadIdx.x;
        for (int u = 0; u < WT; ++u) {
            int row = row0 + (t >> 2) + 64 * u;
            if (row < map.M) {
                bp[u] = cache + map.rowoff[row] + (int64_t)layer * map.rowstride[row] + (t & 3) * T::CE;
                sp[u] = s_prev ? s_prev + (int64_t)row * ld_s + (t & 3) * T::CE : nullptr;
            } else {
                bp[u] = nullptr;
                sp[u] = nullptr;
            }
        }
    }
    __device__ void fetch(int k0)
    {
        for (int u = 0; u < WT; ++u) {
            if (bp[u]) {
                Chunk<TC> b = *reinterpret_cast<const Chunk<TC> *>(bp[u] + k0);
                if (sp[u]) {
                    for (int q = 0; q < T::CE / 4; ++q) {
                        float4 s = *reinterpret_cast<const float4 *>(sp[u] + k0 + 4 * q);
                        reg[u].e[4 * q + 0] = to_tc(lam * to_f32(b.e[4 * q + 0]) + (1.f - lam) * s.x, TC());
                        reg[u].e[4 * q + 1] = to_tc(lam * to_f32(b.e[4 * q + 1]) + (1.f - lam) * s.y, TC());
                        reg[u].e[4 * q + 2] = to_tc(lam * to_f32(b.e[4 * q + 2]) + (1.f - lam) * s.z, TC());
                        reg[u].e[4 * q + 3] = to_tc(lam * to_f32(b.e[4 * q + 3]) + (1.f - lam) * s.w, TC());
                    }
                } else {
                    for (int e = 0; e < T::CE; ++e) reg[u].e[e] = to_tc(lam * to_f32(b.e[e]), TC());
                }
            } else {
                for (int e = 0; e < T::CE; ++e) reg[u].e[e] = to_tc(0.f, TC());
            }
        }
    }
    __device__ void store(TC *lds)
    {
        const int t = threadIdx.x;
        for (int u = 0; u < WT; ++u)
            *reinterpret_cast<Chunk<TC> *>(lds + ((t >> 2) + 64 * u) * T::LDP + (t & 3) * T::CE) = reg[u];
    }
};

// ---------------------------------------------------------------------------
// Transposed loaders for contractions over the token index:
// operand[i][k] = src[k][i]  (i contiguous in memory, k = token row).
// A step stages BK token rows.  Chunk c = t + 256u covers token row
// c / CPR and the 16-byte i-chunk c % CPR, CPR = 64*WT / CE; the chunk is
// scattered into the K-contiguous LDS layout element by element.
// Rows k >= kend are zero.  Optionally keeps per-thread column sums.
// ---------------------------------------------------------------------------
template <typename TC, int WT> struct ColsGeom {
    using T = Traits<TC>;
    static constexpr int CPR = 64 * WT / T::CE;      // chunks per token row
    static constexpr int NCH = T::BK * CPR / kThreads; // chunks per thread
    static_assert(T::BK * CPR % kThreads == 0, "tile/threads mismatch");
    static_assert(kThreads % CPR == 0 || CPR % kThreads == 0, "column ownership must be fixed");
};

template <typename TC, int WT, typename SRC, bool SUMS> struct LoadCols {
    using T = Traits<TC>;
    using G = ColsGeom<TC, WT>;
    const SRC *src; // [k][ld]
    int64_t ld;
    int ncols; // valid i
    int kend;
    int i0;
    Chunk<TC> reg[G::NCH];
    float sums[SUMS ? G::NCH : 1][T::CE];
    __device__ void init(int i0_)
    {
        i0 = i0_;
        if (SUMS)
            for (int u = 0; u < G::NCH; ++u)
                for (int e = 0; e < T::CE; ++e) sums[u][e] = 0.f;
    }
    __device__ void fetch(int k0)
    {
        const int t = threadIdx.x;
        for (int u = 0; u < G::NCH; ++u) {
            int c = t + kThreads * u;
            int k = k0 + c / G::CPR;
            int i = i0 + (c % G::CPR) * T::CE;
            if (k < kend && i < ncols) {
                const SRC *p = src + (int64_t)k * ld + i;
                for (int e = 0; e < T::CE; ++e) {
                    float f = to_f32(p[e]);
                    if (SUMS) sums[u][e] += f;
                    reg[u].e[e] = to_tc(f, TC());
                }
            } else {
                for (int e = 0; e < T::CE; ++e) reg[u].e[e] = to_tc(0.f, TC());
            }
        }
    }
    __device__ void store(TC *lds)
    {
        const int t = threadIdx.x;
        for (int u = 0; u < G::NCH; ++u) {
            int c = t + kThreads * u;
            int kk = c / G::CPR;
            int ii = (c % G::CPR) * T::CE;
            for (int e = 0; e < T::CE; ++e) lds[(ii + e) * T::LDP + kk] = reg[u].e[e];
        }
    }
};

// operand[i][k] = x[k][i] = lam * b_l[k][i] + (1 - lam) * s_prev[k][i]
template <typename TC, int WT> struct LoadColsX {
    using T = Traits<TC>;
    using G = ColsGeom<TC, WT>;
    const TC *cache;
    RowMap map;
    int layer;
    const float *s_prev;
    int64_t ld_s;
    float lam;
    int ncols;
    int kend;
    int i0;
    Chunk<TC> reg[G::NCH];
    __device__ void init(int i0_) { i0 = i0_; }
    __device__ void fetch(int k0)
    {
        const int t = threadIdx.x;
        for (int u = 0; u < G::NCH; ++u) {
            int c = t + kThreads * u;
            int k = k0 + c / G::CPR;
            int i = i0 + (c % G::CPR) * T::CE;
            if (k < kend && i < ncols) {
                const TC *bp = cache + map.rowoff[k] + (int64_t)layer * map.rowstride[k] + i;
                Chunk<TC> b = *reinterpret_cast<const Chunk<TC> *>(bp);
                if (s_prev) {
                    const float *sp = s_prev + (int64_t)k * ld_s + i;
                    for (int e = 0; e < T::CE; ++e)
                        reg[u].e[e] = to_tc(lam * to_f32(b.e[e]) + (1.f - lam) * sp[e], TC());
                } else {
                    for (int e = 0; e < T::CE; ++e) reg[u].e[e] = to_tc(lam * to_f32(b.e[e]), TC());
                }
            } else {
                for (int e = 0; e < T::CE; ++e) reg[u].e[e] = to_tc(0.f, TC());
            }
        }
    }
    __device__ void store(TC *lds)
    {
        const int t = threadIdx.x;
        for (int u = 0; u < G::NCH; ++u) {
            int c = t + kThreads * u;
            int kk = c / G::CPR;
            int ii = (c % G::CPR) * T::CE;
            for (int e = 0; e < T::CE; ++e) lds[(ii + e) * T::LDP + kk] = reg[u].e[e];
        }
    }
};

// ---------------------------------------------------------------------------
// MFMA step on one staged K tile
// ---------------------------------------------------------------------------
template <int WTM, int WTN>
__device__ __forceinline__ void mma_tile(const bf16_t *As, const bf16_t *Bs, f32x16 (&acc)[WTM][WTN],
                                         int wm, int wn, int lane)
{
    using T = Traits<bf16_t>;
    const int i = lane & 31, g = lane >> 5;
#pragma unroll
    for (int q = 0; q < T::BK / (2 * T::KV); ++q) {
        bf16x8 a[WTM], b[WTN];
#pragma unroll
        for (int x = 0; x < WTM; ++x)
            a[x] = *reinterpret_cast<const bf16x8 *>(As + ((wm * WTM + x) * 32 + i) * T::LDP + q * 16 + g * 8);
#pragma unroll
        for (int y = 0; y < WTN; ++y)
            b[y] = *reinterpret_cast<const bf16x8 *>(Bs + ((wn * WTN + y) * 32 + i) * T::LDP + q * 16 + g * 8);
#pragma unroll
        for (int x = 0; x < WTM; ++x)
#pragma unroll
            for (int y = 0; y < WTN; ++y)
                acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[x], b[y], acc[x][y], 0, 0, 0);
    }
}

template <int WTM, int WTN>
__device__ __forceinline__ void mma_tile(const float *As, const float *Bs, f32x16 (&acc)[WTM][WTN],
                                         int wm, int wn, int lane)
{
    using T = Traits<float>;
    const int i = lane & 31, g = lane >> 5;
#pragma unroll
    for (int q = 0; q < T::BK / 2; ++q) {
        float a[WTM], b[WTN];
#pragma unroll
        for (int x = 0; x < WTM; ++x) a[x] = As[((wm * WTM + x) * 32 + i) * T::LDP + q * 2 + g];
#pragma unroll
        for (int y = 0; y < WTN; ++y) b[y] = Bs[((wn * WTN + y) * 32 + i) * T::LDP + q * 2 + g];
#pragma unroll
        for (int x = 0; x < WTM; ++x)
#pragma unroll
            for (int y = 0; y < WTN; ++y)
                acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[x], b[y], acc[x][y], 0, 0, 0);
    }
}

// C[row0.., col0..] = sum_{k in [kbegin, kend)} A[row][k] * B[col][k]; the
// epilogue functor receives (row, col, value) for every element inside
// (nrows, ncols).  kbegin must be a multiple of the K step.
template <typename TC, int WTM, int WTN, class ALoad, class BLoad, class Epi>
__device__ __forceinline__ void gemm_tile(ALoad &al, BLoad &bl, Epi &epi, int kbegin, int kend,
                                          int row0, int col0, int nrows, int ncols)
{
    using T = Traits<TC>;
    constexpr int BM = 64 * WTM, BN = 64 * WTN;
    __shared__ __attribute__((aligned(16))) TC As[BM * T::LDP];
    __shared__ __attribute__((aligned(16))) TC Bs[BN * T::LDP];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    f32x16 acc[WTM][WTN];
#pragma unroll
    for (int x = 0; x < WTM; ++x)
#pragma unroll
        for (int y = 0; y < WTN; ++y)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[x][y][v] = 0.f;

    al.init(row0);
    bl.init(col0);
    if (kbegin < kend) {
        al.fetch(kbegin);
        bl.fetch(kbegin);
    }
    for (int k0 = kbegin; k0 < kend; k0 += T::BK) {
        al.store(As);
        bl.store(Bs);
        __syncthreads();
        if (k0 + T::BK < kend) {
            al.fetch(k0 + T::BK);
            bl.fetch(k0 + T::BK);
        }
        mma_tile<WTM, WTN>(As, Bs, acc, wm, wn, lane);
        __syncthreads();
    }
    const int i = lane & 31, g = lane >> 5;
#pragma unroll
    for (int x = 0; x < WTM; ++x)
#pragma unroll
        for (int y = 0; y < WTN; ++y) {
            const int col = col0 + (wn * WTN + y) * 32 + i;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + (wm * WTM + x) * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
                if (row < nrows && col < ncols) epi(row, col, acc[x][y][v]);
            }
        }
}

// Sum of one float per thread over the workgroup; result valid in thread 0.
__device__ __forceinline__ float block_sum(float v, float *scratch /* >= 4 floats of LDS */)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = 0.f;
    if (threadIdx.x == 0)
        for (int w = 0; w < (int)(blockDim.x >> 6); ++w) r += scratch[w];
    return r;
}

} // namespace pac
