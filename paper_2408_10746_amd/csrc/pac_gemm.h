// LDS-tiled MFMA contraction core for gfx950, shared by all contraction kernels.
//
// One workgroup = 256 threads = 4 wavefronts (64 lanes each) arranged WM x WN;
// every wavefront owns WTM x WTN accumulator tiles of 32 x 32, so the
// workgroup tile is (32*WM*WTM) x (32*WN*WTN).  Operands are staged through
// LDS in a K-contiguous layout for both sides ("A[i][k]" and "B[j][k]"),
// KU*64 bytes of K per row per step plus 16 bytes of padding, which is what
// the 32x32 MFMA wants: lane (i = lane%32, g = lane/32) supplies KV
// consecutive K values of row i (8 bf16, or 1 fp32), and the instruction
// contracts 2*KV of K.  Because both operands use the same (g, element) -> K
// assignment, the result does not depend on how the hardware labels K inside
// an instruction.
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
#include <type_traits>

namespace pac {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4))); // 16 raw bytes held in registers

constexpr int kThreads = 256;

template <typename TC> struct Traits;
template <> struct Traits<bf16_t> {
    static constexpr int CE = 8;  // elements per 16-byte chunk
    static constexpr int KV = 8;  // K values a lane feeds to one MFMA
};
template <> struct Traits<float> {
    static constexpr int CE = 4;
    static constexpr int KV = 1;
};

// Geometry of one staged K step: KU * 64 bytes of K per row.
template <typename TC, int KU> struct Stage {
    static constexpr int CE = Traits<TC>::CE;
    static constexpr int BK = KU * 64 / (int)sizeof(TC);       // K elements per step
    static constexpr int LDP = (KU * 64 + 16) / (int)sizeof(TC); // LDS pitch in elements
    static constexpr int CPK = 4 * KU;                          // 16-byte chunks along K per row
};

// 16 bytes of compute-type elements
template <typename TC> struct alignas(16) Chunk { TC e[Traits<TC>::CE]; };

__device__ __forceinline__ bf16_t to_tc(float f, bf16_t) { return static_cast<bf16_t>(f); }
__device__ __forceinline__ float to_tc(float f, float) { return f; }
__device__ __forceinline__ float to_f32(bf16_t h) { return static_cast<float>(h); }
__device__ __forceinline__ float to_f32(float f) { return f; }

// ---------------------------------------------------------------------------
// Loaders.  Every loader keeps two register slots so that two K steps can be in flight.
// fetch<SLOT>(k0) issues its loads unconditionally, from addresses clamped into valid memory,
// and store<SLOT>() applies the validity masks when it writes the LDS image: with no branch
// around a load the compiler can count the loads in flight and wait only for the older slot.
// ---------------------------------------------------------------------------

// Row-major loaders: operand[row][k] = src[row][k] (K contiguous in memory).
// Chunk c = t + 256u covers row c / CPK and the 16-byte K chunk c % CPK.
template <typename TC, int ROWS, int KU> struct RowsGeom {
    using S = Stage<TC, KU>;
    static constexpr int TOTAL = ROWS * S::CPK;
    static constexpr int NCH = (TOTAL + kThreads - 1) / kThreads;
};

template <typename TC, int ROWS, int KU> struct LoadRowsTC {
    static constexpr bool kSwizzled = false;
    using S = Stage<TC, KU>;
    using G = RowsGeom<TC, ROWS, KU>;
    const TC *src;
    int64_t ld;
    int nrows;
    int kmin = 0, klim = 0x7fffffff; // K outside [kmin, klim) reads as zero (whole 16-byte chunks)
    const TC *rp[G::NCH];
    bool ok[G::NCH];
    int kpos[2];
    u32x4 reg[2][G::NCH];
    __device__ void init(int row0)
    {
        const int t = threadIdx.x;
#pragma unroll
        for (int u = 0; u < G::NCH; ++u) {
            const int c = t + kThreads * u;
            const int row = row0 + c / S::CPK;
            ok[u] = c < G::TOTAL && row < nrows;
            rp[u] = src + (ok[u] ? (int64_t)row * ld : 0) + (c % S::CPK) * S::CE;
        }
    }
    template <int SLOT> __device__ void fetch(int k0)
    {
        kpos[SLOT] = k0;
        const int t = threadIdx.x;
#pragma unroll
        for (int u = 0; u < G::NCH; ++u) {
            const int kc = ((t + kThreads * u) % S::CPK) * S::CE;
            const int k = k0 + kc;
            // masked chunks re-read the start of their row
            reg[SLOT][u] = *reinterpret_cast<const u32x4 *>(rp[u] + ((k >= kmin && k < klim) ? k0 : -kc));
        }
    }
    template <int SLOT> __device__ void store(TC *lds, bool live)
    {
        const int t = threadIdx.x;
#pragma unroll
        for (int u = 0; u < G::NCH; ++u) {
            const int c = t + kThreads * u;
            const int k = kpos[SLOT] + (c % S::CPK) * S::CE;
            const bool keep = ok[u] && k >= kmin && k < klim;
            if (c < G::TOTAL)
                *reinterpret_cast<u32x4 *>(lds + (c / S::CPK) * S::LDP + (c % S::CPK) * S::CE) =
                    keep ? reg[SLOT][u] : u32x4{0, 0, 0, 0};
        }
    }
};

template <typename TC, int ROWS, int KU> struct LoadRowsF32 {
    static constexpr bool kSwizzled = false;
    using S = Stage<TC, KU>;
    using G = RowsGeom<TC, ROWS, KU>;
    const float *src;
    int64_t ld;
    int nrows;
    const float *rp[G::NCH];
    bool ok[G::NCH];
    f32x4 reg[2][G::NCH][S::CE / 4];
    __device__ void init(int row0)
    {
        const int t = threadIdx.x;
#pragma unroll
        for (int u = 0; u < G::NCH; ++u) {
            const int c = t + kThreads * u;
            const int row = row0 + c / S::CPK;
            ok[u] = c < G::TOTAL && row < nrows;
            rp[u] = src + (ok[u] ? (int64_t)row * ld : 0) + (c % S::CPK) * S::CE;
        }
    }
    template <int SLOT> __device__ void fetch(int k0)
    {
#pragma unroll
        for (int u = 0; u < G::NCH; ++u)
#pragma unroll
            for (int q = 0; q < S::CE / 4; ++q) reg[SLOT][u][q] = *reinterpret_cast<const f32x4 *>(rp[u] + k0 + 4 * q);
    }
    template <int SLOT> __device__ void store(TC *lds, bool live)
    {
        const int t = threadIdx.x;
#pragma unroll
        for (int u = 0; u < G::NCH; ++u) {
            const int c = t + kThreads * u;
            Chunk<TC> v;
#pragma unroll
            for (int q = 0; q < S::CE / 4; ++q) {
                const f32x4 f = reg[SLOT][u][q];
                v.e[4 * q + 0] = to_tc(ok[u] ? f.x : 0.f, TC());
                v.e[4 * q + 1] = to_tc(ok[u] ? f.y : 0.f, TC());
                v.e[4 * q + 2] = to_tc(ok[u] ? f.z : 0.f, TC());
                v.e[4 * q + 3] = to_tc(ok[u] ? f.w : 0.f, TC());
            }
            if (c < G::TOTAL)
                *reinterpret_cast<Chunk<TC> *>(lds + (c / S::CPK) * S::LDP + (c % S::CPK) * S::CE) = v;
        }
    }
};

// Where the rows of a batch live in the cache: token row m of layer l starts at
// cache + rowoff[m] + l * rowstride[m]   (elements).
struct RowMap {
    const int64_t *rowoff;
    const int32_t *rowstride;
    int M;
};

// x[m][k] = lam * b_l[m][k] + (1 - lam) * s_prev[m][k]   (MIX == false: x = lam * b, s_prev unused)
// Whether the previous side state takes part is a compile-time choice: a run-time branch around
// some of the loads would bring back the conservative waits.
template <typename TC, int ROWS, int KU, bool MIX> struct LoadRowsX {
    static constexpr bool kSwizzled = false;
    using S = Stage<TC, KU>;
    using G = RowsGeom<TC, ROWS, KU>;
    const TC *cache;
    RowMap map;
    int layer;
    const float *s_prev;
    int64_t ld_s;
    float lam;
    const TC *bp[G::NCH];
    const float *sp[MIX ? G::NCH : 1];
    bool ok[G::NCH];
    u32x4 regb[2][G::NCH];
    f32x4 regs[2][MIX ? G::NCH : 1][S::CE / 4];
    __device__ void init(int row0)
    {
        const int t = threadIdx.x;
#pragma unroll
        for (int u = 0; u < G::NCH; ++u) {
            const int c = t + kThreads * u;
            const int row = row0 + c / S::CPK;
            ok[u] = c < G::TOTAL && row < map.M;
            const int rowc = ok[u] ? row : 0;
            bp[u] = cache + map.rowoff[rowc] + (int64_t)layer * map.rowstride[rowc] + (c % S::CPK) * S::CE;
            if (MIX) sp[u] = s_prev + (int64_t)rowc * ld_s + (c % S::CPK) * S::CE;
        }
    }
    template <int SLOT> __device__ void fetch(int k0)
    {
#pragma unroll
        for (int u = 0; u < G::NCH; ++u) {
            regb[SLOT][u] = *reinterpret_cast<const u32x4 *>(bp[u] + k0);
            if (MIX) {
#pragma unroll
                for (int q = 0; q < S::CE / 4; ++q)
                    regs[SLOT][u][q] = *reinterpret_cast<const f32x4 *>(sp[u] + k0 + 4 * q);
            }
        }
    }
    template <int SLOT> __device__ void store(TC *lds, bool live)
    {
        const int t = threadIdx.x;
#pragma unroll
        for (int u = 0; u < G::NCH; ++u) {
            const int c = t + kThreads * u;
            u32x4 out = regb[SLOT][u];
            if (MIX || lam != 1.f) {
                Chunk<TC> b, v;
                __builtin_memcpy(&b, &out, 16);
#pragma unroll
                for (int q = 0; q < S::CE / 4; ++q) {
                    f32x4 s = {0.f, 0.f, 0.f, 0.f};
                    if (MIX) s = regs[SLOT][u][q];
                    v.e[4 * q + 0] = to_tc(lam * to_f32(b.e[4 * q + 0]) + (1.f - lam) * s[0], TC());
                    v.e[4 * q + 1] = to_tc(lam * to_f32(b.e[4 * q + 1]) + (1.f - lam) * s[1], TC());
                    v.e[4 * q + 2] = to_tc(lam * to_f32(b.e[4 * q + 2]) + (1.f - lam) * s[2], TC());
                    v.e[4 * q + 3] = to_tc(lam * to_f32(b.e[4 * q + 3]) + (1.f - lam) * s[3], TC());
                }
                __builtin_memcpy(&out, &v, 16);
            }
            if (!ok[u]) out = u32x4{0, 0, 0, 0};
            if (c < G::TOTAL) *reinterpret_cast<u32x4 *>(lds + (c / S::CPK) * S::LDP + (c % S::CPK) * S::CE) = out;
        }
    }
};

// ---------------------------------------------------------------------------
// Transposed loaders for contractions over the token index:
// operand[i][k] = src[k][i]  (i contiguous in memory, k = token row).
// A thread owns CE x CE blocks (CE token rows x CE consecutive i): it loads CE
// 16-byte chunks, transposes them in registers and writes CE 16-byte chunks
// into the K-contiguous LDS layout.  Block c = t + 256u covers i-block c % IB
// and token block c / IB.  Token rows >= kend and columns >= ncols are zero.
// Optionally keeps per-thread column sums (fp32, before rounding).
// ---------------------------------------------------------------------------
template <typename TC, int ROWS, int KU> struct ColsGeom {
    using S = Stage<TC, KU>;
    static constexpr int CE = S::CE;
    static constexpr int IB = ROWS / CE;      // i-blocks per tile
    static constexpr int KB = S::BK / CE;     // token blocks per step
    static constexpr int TOTAL = IB * KB;
    static constexpr int NCH = (TOTAL + kThreads - 1) / kThreads; // blocks per thread
    static_assert(ROWS % CE == 0, "tile rows must be whole chunks");
};

__device__ __forceinline__ void transpose_block(const Chunk<bf16_t> (&in)[8], Chunk<bf16_t> (&out)[8])
{
    uint32_t a[8][4], o[8][4];
#pragma unroll
    for (int k = 0; k < 8; ++k) __builtin_memcpy(a[k], &in[k], 16);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int w = i >> 1;
#pragma unroll
        for (int wp = 0; wp < 4; ++wp) {
            const uint32_t x = a[2 * wp][w], y = a[2 * wp + 1][w]; // token rows 2wp, 2wp+1
            o[i][wp] = (i & 1) ? ((x >> 16) | (y & 0xffff0000u)) : ((x & 0xffffu) | (y << 16));
        }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) __builtin_memcpy(&out[i], o[i], 16);
}

__device__ __forceinline__ void transpose_block(const Chunk<float> (&in)[4], Chunk<float> (&out)[4])
{
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int k = 0; k < 4; ++k) out[i].e[k] = in[k].e[i];
}

// With 256-byte K rows of bf16 the transposed stores of one instruction hit rows 8 apart, i.e.
// the same LDS banks; the 16-byte chunk index of row i is therefore XOR-ed with (i / 16) % 8
// ("swizzle"), which spreads those stores over all banks.  The MFMA fragment reads apply the same XOR.
template <typename TC, int KU> struct ColsSwizzle {
    static constexpr bool value = sizeof(TC) == 2 && KU == 4;
};
__device__ __forceinline__ int swizzle_of_row(int row) { return (row >> 4) & 7; }

// Writes one thread's transposed blocks; `blk` holds the (already masked) CE x CE block of slot u.
template <typename TC, int ROWS, int KU>
__device__ __forceinline__ void cols_store_block(TC *lds, int c, const Chunk<TC> (&blk)[Traits<TC>::CE])
{
    using S = Stage<TC, KU>;
    using G = ColsGeom<TC, ROWS, KU>;
    const int ib = c % G::IB, kb = c / G::IB;
    Chunk<TC> tr[G::CE];
    transpose_block(blk, tr);
#pragma unroll
    for (int e = 0; e < G::CE; ++e) {
        const int row = ib * G::CE + e;
        const int chunk = ColsSwizzle<TC, KU>::value ? (kb ^ swizzle_of_row(row)) : kb;
        *reinterpret_cast<Chunk<TC> *>(lds + row * S::LDP + chunk * G::CE) = tr[e];
    }
}

template <typename SRC, int CE> struct alignas(16) SrcChunk { SRC e[CE]; };

template <typename TC, int ROWS, int KU, typename SRC, bool SUMS> struct LoadCols {
    static constexpr bool kSwizzled = ColsSwizzle<TC, KU>::value;
    using S = Stage<TC, KU>;
    using G = ColsGeom<TC, ROWS, KU>;
    static constexpr int NV = G::CE * (int)sizeof(SRC) / 16; // 16-byte registers per source chunk
    static_assert(!SUMS || kThreads % G::IB == 0, "column sums need a fixed column block per thread");
    const SRC *src; // [k][ld]
    int64_t ld;
    int ncols; // valid i
    int kend;
    int i0;
    int kpos[2];
    u32x4 reg[2][G::NCH][G::CE][NV];
    float sums[SUMS ? G::CE : 1];
    __device__ void init(int i0_)
    {
        i0 = i0_;
        if (SUMS)
            for (int e = 0; e < G::CE; ++e) sums[e] = 0.f;
    }
    template <int SLOT> __device__ void fetch(int k0)
    {
        kpos[SLOT] = k0;
        const int t = threadIdx.x;
#pragma unroll
        for (int u = 0; u < G::NCH; ++u) {
            const int c = (t + kThreads * u) % G::TOTAL; // out-of-range blocks re-read a valid one
            const int i = min(i0 + (c % G::IB) * G::CE, ncols - G::CE);
            const int kb = k0 + (c / G::IB) * G::CE;
#pragma unroll
            for (int kk = 0; kk < G::CE; ++kk) {
                const int k = min(kb + kk, kend - 1);
                const u32x4 *p = reinterpret_cast<const u32x4 *>(src + (int64_t)k * ld + i);
#pragma unroll
                for (int q = 0; q < NV; ++q) reg[SLOT][u][kk][q] = p[q];
            }
        }
    }
    template <int SLOT> __device__ void store(TC *lds, bool live)
    {
        const int t = threadIdx.x;
#pragma unroll
        for (int u = 0; u < G::NCH; ++u) {
            const int c = t + kThreads * u;
            const bool icol = i0 + (c % G::IB) * G::CE < ncols;
            const int kb = kpos[SLOT] + (c / G::IB) * G::CE;
            Chunk<TC> blk[G::CE];
#pragma unroll
            for (int kk = 0; kk < G::CE; ++kk) {
                const bool keep = icol && kb + kk < kend && c < G::TOTAL;
                SrcChunk<SRC, G::CE> in;
                __builtin_memcpy(&in, &reg[SLOT][u][kk][0], sizeof(in));
#pragma unroll
                for (int e = 0; e < G::CE; ++e) {
                    const float f = keep ? to_f32(in.e[e]) : 0.f;
                    if (SUMS) sums[e] += live ? f : 0.f;
                    blk[kk].e[e] = to_tc(f, TC());
                }
            }
            if (c < G::TOTAL) cols_store_block<TC, ROWS, KU>(lds, c, blk);
        }
    }
};

// operand[i][k] = x[k][i] = lam * b_l[k][i] + (1 - lam) * s_prev[k][i]   (MIX == false: lam * b)
template <typename TC, int ROWS, int KU, bool MIX> struct LoadColsX {
    static constexpr bool kSwizzled = ColsSwizzle<TC, KU>::value;
    using S = Stage<TC, KU>;
    using G = ColsGeom<TC, ROWS, KU>;
    static constexpr int NV = G::CE * 4 / 16;
    const TC *cache;
    RowMap map;
    int layer;
    const float *s_prev;
    int64_t ld_s;
    float lam;
    int ncols;
    int kend;
    int i0;
    int kpos[2];
    u32x4 regb[2][G::NCH][G::CE];
    u32x4 regs[2][MIX ? G::NCH : 1][G::CE][NV];
    __device__ void init(int i0_) { i0 = i0_; }
    template <int SLOT> __device__ void fetch(int k0)
    {
        kpos[SLOT] = k0;
        const int t = threadIdx.x;
#pragma unroll
        for (int u = 0; u < G::NCH; ++u) {
            const int c = (t + kThreads * u) % G::TOTAL;
            const int i = min(i0 + (c % G::IB) * G::CE, ncols - G::CE);
            const int kb = k0 + (c / G::IB) * G::CE;
#pragma unroll
            for (int kk = 0; kk < G::CE; ++kk) {
                const int k = min(kb + kk, kend - 1);
                regb[SLOT][u][kk] = *reinterpret_cast<const u32x4 *>(cache + map.rowoff[k] +
                                                                     (int64_t)layer * map.rowstride[k] + i);
                if (MIX) {
                    const u32x4 *p = reinterpret_cast<const u32x4 *>(s_prev + (int64_t)k * ld_s + i);
#pragma unroll
                    for (int q = 0; q < NV; ++q) regs[SLOT][u][kk][q] = p[q];
                }
            }
        }
    }
    template <int SLOT> __device__ void store(TC *lds, bool live)
    {
        const int t = threadIdx.x;
#pragma unroll
        for (int u = 0; u < G::NCH; ++u) {
            const int c = t + kThreads * u;
            const bool icol = i0 + (c % G::IB) * G::CE < ncols;
            const int kb = kpos[SLOT] + (c / G::IB) * G::CE;
            Chunk<TC> blk[G::CE];
#pragma unroll
            for (int kk = 0; kk < G::CE; ++kk) {
                const bool keep = icol && kb + kk < kend && c < G::TOTAL;
                Chunk<TC> b;
                __builtin_memcpy(&b, &regb[SLOT][u][kk], 16);
                SrcChunk<float, G::CE> sv;
                if (MIX) __builtin_memcpy(&sv, &regs[SLOT][u][kk][0], sizeof(sv));
#pragma unroll
                for (int e = 0; e < G::CE; ++e) {
                    float f = lam * to_f32(b.e[e]);
                    if (MIX) f += (1.f - lam) * sv.e[e];
                    blk[kk].e[e] = to_tc(keep ? f : 0.f, TC());
                }
            }
            if (c < G::TOTAL) cols_store_block<TC, ROWS, KU>(lds, c, blk);
        }
    }
};

// ---------------------------------------------------------------------------
// MFMA step on one staged K tile
// ---------------------------------------------------------------------------
template <int KU, int WTM, int WTN, bool SWA, bool SWB>
__device__ __forceinline__ void mma_tile(const bf16_t *As, const bf16_t *Bs, f32x16 (&acc)[WTM][WTN],
                                         int arow0, int brow0, int lane)
{
    using S = Stage<bf16_t, KU>;
    const int i = lane & 31, g = lane >> 5;
#pragma unroll
    for (int q = 0; q < S::BK / 16; ++q) {
        bf16x8 a[WTM], b[WTN];
#pragma unroll
        for (int x = 0; x < WTM; ++x) {
            const int row = arow0 + x * 32 + i;
            const int chunk = SWA ? ((2 * q + g) ^ swizzle_of_row(row)) : 2 * q + g;
            a[x] = *reinterpret_cast<const bf16x8 *>(As + row * S::LDP + chunk * 8);
        }
#pragma unroll
        for (int y = 0; y < WTN; ++y) {
            const int row = brow0 + y * 32 + i;
            const int chunk = SWB ? ((2 * q + g) ^ swizzle_of_row(row)) : 2 * q + g;
            b[y] = *reinterpret_cast<const bf16x8 *>(Bs + row * S::LDP + chunk * 8);
        }
#pragma unroll
        for (int x = 0; x < WTM; ++x)
#pragma unroll
            for (int y = 0; y < WTN; ++y)
                acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[x], b[y], acc[x][y], 0, 0, 0);
    }
}

template <int KU, int WTM, int WTN, bool SWA, bool SWB>
__device__ __forceinline__ void mma_tile(const float *As, const float *Bs, f32x16 (&acc)[WTM][WTN],
                                         int arow0, int brow0, int lane)
{
    using S = Stage<float, KU>;
    const int i = lane & 31, g = lane >> 5;
#pragma unroll
    for (int q = 0; q < S::BK / 2; ++q) {
        float a[WTM], b[WTN];
#pragma unroll
        for (int x = 0; x < WTM; ++x) a[x] = As[(arow0 + x * 32 + i) * S::LDP + q * 2 + g];
#pragma unroll
        for (int y = 0; y < WTN; ++y) b[y] = Bs[(brow0 + y * 32 + i) * S::LDP + q * 2 + g];
#pragma unroll
        for (int x = 0; x < WTM; ++x)
#pragma unroll
            for (int y = 0; y < WTN; ++y)
                acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[x], b[y], acc[x][y], 0, 0, 0);
    }
}

// Shape of a workgroup tile; PF = K steps kept in flight in registers (1 or 2).
template <int WM_, int WN_, int WTM_, int WTN_, int KU_, int PF_ = 1> struct Tile {
    static constexpr int WM = WM_, WN = WN_, WTM = WTM_, WTN = WTN_, KU = KU_, PF = PF_;
    static_assert(PF == 1 || PF == 2, "one or two K steps in flight");
    static constexpr int BM = 32 * WM * WTM, BN = 32 * WN * WTN;
    static_assert(WM * WN * 64 == kThreads, "four wavefronts per workgroup");
};

// Hands the accumulators to the epilogue functor.  A lane holds column col and the 16 rows
// row_base + 8 (v / 4) + v % 4 of each 32 x 32 block.  Plain functors get (row, col, value) for every
// element inside (nrows, ncols).  A functor that reads global memory should instead declare
// `static constexpr bool kBatched = true` and provide batch(row_base, col, values, nrows, ncols):
// it can then issue all its loads (from clamped indices) before the first use, where the
// element-wise form would wait for memory once per element.
template <class E, class = void> struct epi_is_batched : std::false_type {};
template <class E> struct epi_is_batched<E, std::void_t<decltype(E::kBatched)>> : std::true_type {};
__device__ __forceinline__ int epi_row(int row_base, int v) { return row_base + 8 * (v >> 2) + (v & 3); }

template <class TL, class Epi>
__device__ __forceinline__ void tile_epilogue(f32x16 (&acc)[TL::WTM][TL::WTN], Epi &epi, int wm, int wn, int lane,
                                              int row0, int col0, int nrows, int ncols)
{
    const int i = lane & 31, g = lane >> 5;
#pragma unroll
    for (int x = 0; x < TL::WTM; ++x)
#pragma unroll
        for (int y = 0; y < TL::WTN; ++y) {
            const int col = col0 + (wn * TL::WTN + y) * 32 + i;
            const int row_base = row0 + (wm * TL::WTM + x) * 32 + 4 * g;
            if constexpr (epi_is_batched<Epi>::value) {
                epi.batch(row_base, col, acc[x][y], nrows, ncols);
            } else {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = epi_row(row_base, v);
                    if (row < nrows && col < ncols) epi(row, col, acc[x][y][v]);
                }
            }
        }
}

// C[row0.., col0..] = sum_{k in [kbegin, kend)} A[row][k] * B[col][k]; the
// epilogue functor receives (row, col, value) for every element inside
// (nrows, ncols).  kbegin must be a multiple of the K step.
// LDS bytes one workgroup tile needs (both operands of one K step).
template <typename TC, class TL> constexpr int tile_lds_bytes()
{
    return (TL::BM + TL::BN) * Stage<TC, TL::KU>::LDP * (int)sizeof(TC);
}

template <typename TC, class TL, class ALoad, class BLoad, class Epi>
__device__ __forceinline__ void gemm_tile(void *lds /* tile_lds_bytes<TC, TL>(), 16-byte aligned */, ALoad &al,
                                          BLoad &bl, Epi &epi, int kbegin, int kend, int row0, int col0,
                                          int nrows, int ncols)
{
    using S = Stage<TC, TL::KU>;
    TC *As = reinterpret_cast<TC *>(lds);
    TC *Bs = As + TL::BM * S::LDP;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / TL::WN, wn = wave % TL::WN;
    f32x16 acc[TL::WTM][TL::WTN];
#pragma unroll
    for (int x = 0; x < TL::WTM; ++x)
#pragma unroll
        for (int y = 0; y < TL::WTN; ++y)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[x][y][v] = 0.f;

    al.init(row0);
    bl.init(col0);
    // One or two K steps are in flight.  Every path issues the same loads (steps past the end re-read
    // the last one and are never used), so the waits before the LDS stores cover only the older step.
    const int nsteps = (kend - kbegin + S::BK - 1) / S::BK;
    auto mma = [&]() {
        mma_tile<TL::KU, TL::WTM, TL::WTN, ALoad::kSwizzled, BLoad::kSwizzled>(As, Bs, acc, wm * TL::WTM * 32,
                                                                              wn * TL::WTN * 32, lane);
    };
    if (nsteps > 0 && TL::PF == 1) {
        const int klast = kbegin + (nsteps - 1) * S::BK;
        al.template fetch<0>(kbegin);
        bl.template fetch<0>(kbegin);
        for (int st = 0; st < nsteps; ++st) {
            al.template store<0>(As, true);
            bl.template store<0>(Bs, true);
            __syncthreads();
            al.template fetch<0>(min(kbegin + (st + 1) * S::BK, klast));
            bl.template fetch<0>(min(kbegin + (st + 1) * S::BK, klast));
            mma();
            __syncthreads();
        }
    }
    if (nsteps > 0 && TL::PF == 2) {
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
            const bool live = st + 1 < nsteps; // otherwise a repeat of the last step, staged but not used
            al.template store<1>(As, live);
            bl.template store<1>(Bs, live);
            __syncthreads();
            al.template fetch<1>(min(k0 + 3 * S::BK, klast));
            bl.template fetch<1>(min(k0 + 3 * S::BK, klast));
            if (live) mma();
            __syncthreads();
        }
    }
    tile_epilogue<TL>(acc, epi, wm, wn, lane, row0, col0, nrows, ncols);
}

// Sum of one float per thread over the workgroup; result valid in thread 0.
__device__ __forceinline__ float block_sum(float v, float *scratch /* >= 16 floats of LDS */)
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
