// Workgroup-tile contractions whose operands stream from global memory straight into LDS.
//
// The tile code in pac_gemm.h stages every K step through registers: the loads of a step are
// issued, the wavefront computes on the previous step, then waits for the loads and copies them to
// LDS.  That keeps few bytes in flight per compute unit.  Here each wavefront issues 16-byte
// global -> LDS transfers (no registers involved) for several K steps ahead into a ring of LDS
// stages, and a counted wait on its own transfers plus one barrier per K step hands a stage to the
// matrix instructions.
//
// LDS layout of a stage: "panels" of 128-byte rows (64 bf16).  A transfer instruction writes
// 64 lanes x 16 bytes = 1 KB contiguously, so padding rows is not possible; bank conflicts are
// avoided by an XOR swizzle of the 16-byte chunk index within a row, applied by choosing which
// global chunk each lane fetches.
//
//   gemm_nt: both operands have K contiguous in memory (rows of A, rows of B^T); fragments are read
//            with 16-byte LDS loads.
//   gemm_tn: the contraction runs over the token index, both operands are [token][column] in
//            memory; a stage holds token rows, and fragments are read with the transposing LDS load
//            (ds_read_b64_tr_b16).
#pragma once
#include "pac_gemm.h"

namespace pac {

// wait until at most N of this wavefront's vector-memory operations are outstanding
template <int N> __device__ __forceinline__ void wait_vm()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// 16 bytes per lane from global memory into LDS: lane i's chunk lands at lds_wave_base + 16 i.
// lds_wave_base must be the same for all lanes.  Written as assembly so that the compiler does not
// track these transfers itself: it would wait for all of them before every LDS read, which defeats
// transfers that run several stages ahead.  The code below counts them (wait_vm) instead; transfers
// the compiler does not know of can only make its own waits stricter, never looser, because the
// counter retires in issue order.
__device__ __forceinline__ void dma16(const void *g, void *lds_wave_base)
{
    const uint32_t l = __builtin_amdgcn_readfirstlane(
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)lds_wave_base);
    // one wait state between the write of M0 and the transfer that reads it
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(l), "v"(g) : "memory", "m0");
}

// ---------------------------------------------------------------------------
// K-contiguous operands
// ---------------------------------------------------------------------------
template <int WM_, int WN_, int WTM_, int WTN_, int BK_, int STAGES_> struct NtTile {
    static constexpr int WM = WM_, WN = WN_, WTM = WTM_, WTN = WTN_, BK = BK_, STAGES = STAGES_;
    static constexpr int BM = 32 * WM * WTM, BN = 32 * WN * WTN, ROWS = BM + BN;
    static constexpr int CPR = BK / 8;            // 16-byte chunks per row
    static constexpr int RPI = 64 / CPR;          // rows one transfer instruction covers
    static constexpr int TOTAL_I = ROWS / RPI;    // transfer instructions per stage
    static constexpr int NW = WM * WN;            // wavefronts per workgroup
    static constexpr int NI = (TOTAL_I + NW - 1) / NW; // per wavefront (the last ones may repeat a row group)
    static constexpr int STAGE_BYTES = ROWS * BK * 2;
    static constexpr int LDS_BYTES = STAGES * STAGE_BYTES;
    static_assert(BK == 32 || BK == 64, "K step of 32 or 64");
    static_assert(ROWS % RPI == 0, "whole transfer instructions");
    static_assert(STAGES >= 2 && NI * (STAGES - 1) < 64, "transfers in flight must fit the counter");
};

// Chunk swizzle of an LDS row.  The LDS has 64 banks of 4 bytes, and a 16-byte-per-lane read is served 16 lanes
// at a time: the 16 consecutive rows those lanes read must land on 16 different 16-byte positions of the
// 256-byte bank line.  Two 128-byte rows (four 64-byte rows) share a bank line, so the swizzle must differ
// between rows 2 (4) apart, for 8 (4) such rows.  (With row & 7 rows 8 apart collided: the counters showed
// every second cycle of the fragment reads as a bank conflict.)
template <int BK> __device__ __forceinline__ int nt_swz(int lds_row) { return BK == 64 ? ((lds_row >> 1) & 7) : ((lds_row >> 2) & 3); }

// C[row0.., col0..] = sum_{k in [kbegin, kend)} A[row][k] * B[col][k]; (kend - kbegin) % BK == 0.
// arow(row) / brow(col) return the address of element k = 0 of that row; rows >= nrows and
// columns >= ncols are read from the last valid one and their results are not passed on.
// The epilogue functor receives (row, col, value) for every element inside (nrows, ncols).
// PIPE: the K step is walked in its 16-deep sub-steps, each issuing its share of the next stage's transfers and
// the fragment reads of the following sub-step before its own matrix instructions, so that a wavefront's
// transfer issue, LDS reads and matrix instructions overlap (worth 10-25 % on long contractions with three
// stages; with two stages the later transfer issue costs more than it gains).
template <class TL, bool PIPE = false, class ARow, class BRow, class Epi>
__device__ __forceinline__ void gemm_nt(char *lds /* TL::LDS_BYTES, 1 KB aligned */, const ARow &arow, const BRow &brow,
                                        Epi &epi, int kbegin, int kend, int row0, int col0, int nrows, int ncols)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / TL::WN, wn = wave % TL::WN;
    f32x16 acc[TL::WTM][TL::WTN];
#pragma unroll
    for (int x = 0; x < TL::WTM; ++x)
#pragma unroll
        for (int y = 0; y < TL::WTN; ++y)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[x][y][v] = 0.f;

    const int nsteps = (kend - kbegin) / TL::BK;
    if (nsteps > 0) {
        // this lane's share of the transfers of a stage
        const bf16_t *gp[TL::NI];
        int ldso[TL::NI];
#pragma unroll
        for (int q = 0; q < TL::NI; ++q) {
            const int ii = min(wave + TL::NW * q, TL::TOTAL_I - 1);
            const int lr = ii * TL::RPI + lane / TL::CPR;
            const int lc = (lane % TL::CPR) ^ nt_swz<TL::BK>(lr);
            gp[q] = (lr < TL::BM ? arow(min(row0 + lr, nrows - 1)) : brow(min(col0 + lr - TL::BM, ncols - 1))) + lc * 8;
            ldso[q] = ii * 1024;
        }
        auto issue = [&](int slot, int step) {
            const int k0 = kbegin + min(step, nsteps - 1) * TL::BK; // past the end: repeat the last step, never used
#pragma unroll
            for (int q = 0; q < TL::NI; ++q) dma16(gp[q] + k0, lds + slot * TL::STAGE_BYTES + ldso[q]);
        };
#pragma unroll
        for (int s = 0; s < TL::STAGES - 1; ++s) issue(s, s);
        // fragment addresses within a stage
        const int i = lane & 31, g = lane >> 5;
        int arow_b[TL::WTM], brow_b[TL::WTN], asw[TL::WTM], bsw[TL::WTN];
#pragma unroll
        for (int x = 0; x < TL::WTM; ++x) {
            const int lr = (wm * TL::WTM + x) * 32 + i;
            arow_b[x] = lr * TL::BK * 2;
            asw[x] = nt_swz<TL::BK>(lr);
        }
#pragma unroll
        for (int y = 0; y < TL::WTN; ++y) {
            const int lr = TL::BM + (wn * TL::WTN + y) * 32 + i;
            brow_b[y] = lr * TL::BK * 2;
            bsw[y] = nt_swz<TL::BK>(lr);
        }
        int slot = 0;
        for (int st = 0; st < nsteps; ++st) {
            wait_vm<TL::NI * (TL::STAGES - 2)>(); // this wavefront's share of stage st has landed
            __syncthreads();                       // ... and everybody else's; stage st-1 is free
            const char *sb = lds + slot * TL::STAGE_BYTES;
            if constexpr (PIPE) {
                const int nslot = slot == 0 ? TL::STAGES - 1 : slot - 1;
                const int k0n = kbegin + min(st + TL::STAGES - 1, nsteps - 1) * TL::BK;
                constexpr int KS = TL::BK / 16;
                bf16x8 a[2][TL::WTM], b[2][TL::WTN];
                auto rd = [&](int ks) {
#pragma unroll
                    for (int x = 0; x < TL::WTM; ++x)
                        a[ks & 1][x] = *reinterpret_cast<const bf16x8 *>(sb + arow_b[x] + (((2 * ks + g) ^ asw[x]) << 4));
#pragma unroll
                    for (int y = 0; y < TL::WTN; ++y)
                        b[ks & 1][y] = *reinterpret_cast<const bf16x8 *>(sb + brow_b[y] + (((2 * ks + g) ^ bsw[y]) << 4));
                };
                rd(0);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    if (ks + 1 < KS) rd(ks + 1);
                    __builtin_amdgcn_sched_barrier(0); // the next sub-step's reads stay ahead of this one's matrix instructions
#pragma unroll
                    for (int q = ks * TL::NI / KS; q < (ks + 1) * TL::NI / KS; ++q)
                        dma16(gp[q] + k0n, lds + nslot * TL::STAGE_BYTES + ldso[q]);
#pragma unroll
                    for (int x = 0; x < TL::WTM; ++x)
#pragma unroll
                        for (int y = 0; y < TL::WTN; ++y)
                            acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks & 1][x], b[ks & 1][y], acc[x][y], 0, 0, 0);
                }
            } else {
            issue(slot == 0 ? TL::STAGES - 1 : slot - 1, st + TL::STAGES - 1);
            // all fragments of the stage are read before the first matrix instruction: with one or two
            // wavefronts per SIMD a read-wait-multiply sequence per K step would expose the LDS latency
            // BK / 16 times per stage
            bf16x8 a[TL::BK / 16][TL::WTM], b[TL::BK / 16][TL::WTN];
#pragma unroll
            for (int ks = 0; ks < TL::BK / 16; ++ks) {
#pragma unroll
                for (int x = 0; x < TL::WTM; ++x)
                    a[ks][x] = *reinterpret_cast<const bf16x8 *>(sb + arow_b[x] + (((2 * ks + g) ^ asw[x]) << 4));
#pragma unroll
                for (int y = 0; y < TL::WTN; ++y)
                    b[ks][y] = *reinterpret_cast<const bf16x8 *>(sb + brow_b[y] + (((2 * ks + g) ^ bsw[y]) << 4));
            }
            __builtin_amdgcn_sched_barrier(0); // keep the scheduler from sinking the reads to their uses
#pragma unroll
            for (int ks = 0; ks < TL::BK / 16; ++ks)
#pragma unroll
                for (int x = 0; x < TL::WTM; ++x)
#pragma unroll
                    for (int y = 0; y < TL::WTN; ++y)
                        acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks][x], b[ks][y], acc[x][y], 0, 0, 0);
            }
            slot = slot + 1 == TL::STAGES ? 0 : slot + 1;
        }
        wait_vm<0>(); // the repeated transfers of the last steps must not outlive this use of the LDS
        __syncthreads();
    }
    tile_epilogue<TL>(acc, epi, wm, wn, lane, row0, col0, nrows, ncols);
}

// gemm_nt whose B operand holds THREE row groups that all contribute to the same output columns:
//   C[row][col] = sum_k A[row][k] * (B[col][k] + B[ncols + col][k] + B[2 ncols + col][k]).
// It serves a product with an fp32 matrix written as three bf16 terms (value = hi + mid + lo, exact to 2^-24 of the
// value): with A exactly bf16 every product is exact in fp32 and the result differs from an fp32 contraction by the
// order of the additions only, at the bf16 matrix rate.  TL::BN is the stage's B row count (3 x the output tile's
// columns); brow(i) returns row i of the [3 ncols][K] operand; ncols = TL::BN / 3 must be the whole output width or the
// caller passes col0 = 0 only (one column tile).
template <class TL, class ARow, class BRow, class Epi>
__device__ __forceinline__ void gemm_nt_fold3(char *lds /* TL::LDS_BYTES, 1 KB aligned */, const ARow &arow, const BRow &brow,
                                              Epi &epi, int kbegin, int kend, int row0, int nrows, int ncols)
{
    static_assert(TL::WN == 1 && TL::WTN % 3 == 0, "three row groups of B per wavefront");
    constexpr int WTO = TL::WTN / 3; // output blocks per wavefront
    using TO = NtTile<TL::WM, 1, TL::WTM, WTO, TL::BK, TL::STAGES>;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave;
    f32x16 acc[TL::WTM][WTO];
#pragma unroll
    for (int x = 0; x < TL::WTM; ++x)
#pragma unroll
        for (int y = 0; y < WTO; ++y)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[x][y][v] = 0.f;
    const int nsteps = (kend - kbegin) / TL::BK;
    if (nsteps > 0) {
        const bf16_t *gp[TL::NI];
        int ldso[TL::NI];
#pragma unroll
        for (int q = 0; q < TL::NI; ++q) {
            const int ii = min(wave + TL::NW * q, TL::TOTAL_I - 1);
            const int lr = ii * TL::RPI + lane / TL::CPR;
            const int lc = (lane % TL::CPR) ^ nt_swz<TL::BK>(lr);
            // B row of the stage: group t = (lr - BM) / (BN / 3), column n inside it; columns past ncols repeat the last one
            const int br = lr - TL::BM, t = br / (TL::BN / 3), n = br - t * (TL::BN / 3);
            gp[q] = (lr < TL::BM ? arow(min(row0 + lr, nrows - 1)) : brow(t * ncols + min(n, ncols - 1))) + lc * 8;
            ldso[q] = ii * 1024;
        }
        auto issue = [&](int slot, int step) {
            const int k0 = kbegin + min(step, nsteps - 1) * TL::BK; // past the end: repeat the last step, never used
#pragma unroll
            for (int q = 0; q < TL::NI; ++q) dma16(gp[q] + k0, lds + slot * TL::STAGE_BYTES + ldso[q]);
        };
#pragma unroll
        for (int s = 0; s < TL::STAGES - 1; ++s) issue(s, s);
        const int i = lane & 31, g = lane >> 5;
        int arow_b[TL::WTM], brow_b[TL::WTN], asw[TL::WTM], bsw[TL::WTN];
#pragma unroll
        for (int x = 0; x < TL::WTM; ++x) {
            const int lr = (wm * TL::WTM + x) * 32 + i;
            arow_b[x] = lr * TL::BK * 2;
            asw[x] = nt_swz<TL::BK>(lr);
        }
#pragma unroll
        for (int y = 0; y < TL::WTN; ++y) {
            const int lr = TL::BM + y * 32 + i;
            brow_b[y] = lr * TL::BK * 2;
            bsw[y] = nt_swz<TL::BK>(lr);
        }
        int slot = 0;
        for (int st = 0; st < nsteps; ++st) {
            wait_vm<TL::NI * (TL::STAGES - 2)>();
            __syncthreads();
            const char *sb = lds + slot * TL::STAGE_BYTES;
            issue(slot == 0 ? TL::STAGES - 1 : slot - 1, st + TL::STAGES - 1);
#pragma unroll
            for (int ks = 0; ks < TL::BK / 16; ++ks) {
                bf16x8 a[TL::WTM], b[TL::WTN];
#pragma unroll
                for (int x = 0; x < TL::WTM; ++x)
                    a[x] = *reinterpret_cast<const bf16x8 *>(sb + arow_b[x] + (((2 * ks + g) ^ asw[x]) << 4));
#pragma unroll
                for (int y = 0; y < TL::WTN; ++y)
                    b[y] = *reinterpret_cast<const bf16x8 *>(sb + brow_b[y] + (((2 * ks + g) ^ bsw[y]) << 4));
#pragma unroll
                for (int x = 0; x < TL::WTM; ++x)
#pragma unroll
                    for (int y = 0; y < TL::WTN; ++y)
                        acc[x][y % WTO] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[x], b[y], acc[x][y % WTO], 0, 0, 0);
            }
            slot = slot + 1 == TL::STAGES ? 0 : slot + 1;
        }
        wait_vm<0>();
        __syncthreads();
    }
    tile_epilogue<TO>(acc, epi, wm, 0, lane, row0, 0, nrows, ncols);
}

// gemm_nt with rings of different depth for the two operands: SA stages for A (rows streamed from HBM once: the
// deeper ring keeps two stages of them in flight), SB = SA - 1 for B (rows shared by many tiles and found in L2).
// Per step the transfers of B for step st + SB - 1 are issued before those of A for step st + SA - 1, so that at the
// top of a step everything but the newest A stage has to have landed: one counted wait, as in gemm_nt.
template <class TL, int SA, class ARow, class BRow, class Epi>
__device__ __forceinline__ void gemm_nt_deepA(char *lds /* nt_deepA_lds<TL, SA>() bytes, 1 KB aligned */, const ARow &arow,
                                              const BRow &brow, Epi &epi, int kbegin, int kend, int row0, int col0,
                                              int nrows, int ncols)
{
    constexpr int SB = SA - 1;
    constexpr int A_I = TL::BM / TL::RPI, B_I = TL::BN / TL::RPI; // transfer instructions per stage
    static_assert(SB >= 2, "at least two stages of B");
    constexpr int NA = (A_I + TL::NW - 1) / TL::NW, NB = (B_I + TL::NW - 1) / TL::NW; // (the last ones may repeat a row group)
    constexpr int A_STAGE = TL::BM * TL::BK * 2, B_STAGE = TL::BN * TL::BK * 2;
    static_assert((NA + NB) * SB + NA < 64, "transfers in flight must fit the counter");
    char *ldsA = lds, *ldsB = lds + SA * A_STAGE;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / TL::WN, wn = wave % TL::WN;
    f32x16 acc[TL::WTM][TL::WTN];
#pragma unroll
    for (int x = 0; x < TL::WTM; ++x)
#pragma unroll
        for (int y = 0; y < TL::WTN; ++y)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[x][y][v] = 0.f;

    const int nsteps = (kend - kbegin) / TL::BK;
    if (nsteps > 0) {
        const bf16_t *gpa[NA], *gpb[NB];
        int offa[NA], offb[NB];
#pragma unroll
        for (int q = 0; q < NA; ++q) {
            const int ii = min(wave + TL::NW * q, A_I - 1);
            const int lr = ii * TL::RPI + lane / TL::CPR;
            gpa[q] = arow(min(row0 + lr, nrows - 1)) + ((lane % TL::CPR) ^ nt_swz<TL::BK>(lr)) * 8;
            offa[q] = ii * 1024;
        }
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            const int ii = min(wave + TL::NW * q, B_I - 1);
            const int lr = ii * TL::RPI + lane / TL::CPR;
            gpb[q] = brow(min(col0 + lr, ncols - 1)) + ((lane % TL::CPR) ^ nt_swz<TL::BK>(lr)) * 8;
            offb[q] = ii * 1024;
        }
        auto issueA = [&](int step) {
            const int k0 = kbegin + min(step, nsteps - 1) * TL::BK; // past the end: repeat the last step, never used
            char *dst = ldsA + (step % SA) * A_STAGE;
#pragma unroll
            for (int q = 0; q < NA; ++q) dma16(gpa[q] + k0, dst + offa[q]);
        };
        auto issueB = [&](int step) {
            const int k0 = kbegin + min(step, nsteps - 1) * TL::BK;
            char *dst = ldsB + (step % SB) * B_STAGE;
#pragma unroll
            for (int q = 0; q < NB; ++q) dma16(gpb[q] + k0, dst + offb[q]);
        };
#pragma unroll
        for (int s = 0; s < SB - 1; ++s) { issueA(s); issueB(s); }
        issueA(SB - 1);
        const int i = lane & 31, g = lane >> 5;
        int arow_b[TL::WTM], brow_b[TL::WTN], asw[TL::WTM], bsw[TL::WTN];
#pragma unroll
        for (int x = 0; x < TL::WTM; ++x) {
            const int lr = (wm * TL::WTM + x) * 32 + i;
            arow_b[x] = lr * TL::BK * 2;
            asw[x] = nt_swz<TL::BK>(lr);
        }
#pragma unroll
        for (int y = 0; y < TL::WTN; ++y) {
            const int lr = (wn * TL::WTN + y) * 32 + i;
            brow_b[y] = lr * TL::BK * 2;
            bsw[y] = nt_swz<TL::BK>(lr);
        }
        for (int st = 0; st < nsteps; ++st) {
            wait_vm<NA>();   // all but the newest A stage have landed (this wavefront's share)
            __syncthreads(); // ... and everybody else's; the stages of step st - 1 are free
            issueB(st + SB - 1);
            issueA(st + SA - 1);
            const char *sa = ldsA + (st % SA) * A_STAGE, *sb = ldsB + (st % SB) * B_STAGE;
            bf16x8 a[TL::BK / 16][TL::WTM], b[TL::BK / 16][TL::WTN];
#pragma unroll
            for (int ks = 0; ks < TL::BK / 16; ++ks) {
#pragma unroll
                for (int x = 0; x < TL::WTM; ++x)
                    a[ks][x] = *reinterpret_cast<const bf16x8 *>(sa + arow_b[x] + (((2 * ks + g) ^ asw[x]) << 4));
#pragma unroll
                for (int y = 0; y < TL::WTN; ++y)
                    b[ks][y] = *reinterpret_cast<const bf16x8 *>(sb + brow_b[y] + (((2 * ks + g) ^ bsw[y]) << 4));
            }
            __builtin_amdgcn_sched_barrier(0); // keep the scheduler from sinking the reads to their uses
#pragma unroll
            for (int ks = 0; ks < TL::BK / 16; ++ks)
#pragma unroll
                for (int x = 0; x < TL::WTM; ++x)
#pragma unroll
                    for (int y = 0; y < TL::WTN; ++y)
                        acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks][x], b[ks][y], acc[x][y], 0, 0, 0);
        }
        wait_vm<0>(); // the repeated transfers of the last steps must not outlive this use of the LDS
        __syncthreads();
    }
    tile_epilogue<TL>(acc, epi, wm, wn, lane, row0, col0, nrows, ncols);
}
template <class TL, int SA> constexpr int nt_deepA_lds() { return SA * TL::BM * TL::BK * 2 + (SA - 1) * TL::BN * TL::BK * 2; }

// ---------------------------------------------------------------------------
// Contractions over the token index: C[i][n] = sum_t A[t][i] * B[t][n], both operands row-major
// over tokens.  A stage holds KT token rows of BM columns of A and BN columns of B as 64-column
// panels ([token][64] bf16, 128 bytes per row).  The transposing LDS load hands a lane 4 values
// from 4 different token rows of one column, which is what the matrix instruction wants of both
// operands; the chunk index of token row t is XOR-ed with 2 * (t % 4), which makes the 16 lanes of
// one such load (4 token rows x 32 bytes) hit all banks once.
//
// The token rows of a stage come in groups of 8 (one transfer instruction each).  atok / btok are
// functors (step, group, row in group) -> address of column 0 of that token's row, or nullptr for
// an empty slot (past the end of the tokens, padding of a short tile), which is filled from `zeros`
// (at least 16 readable zero bytes).  They are called one step before the transfers that use them.
// ---------------------------------------------------------------------------
template <int WM_, int WN_, int WTM_, int WTN_, int KT_, int STAGES_> struct TnTile {
    static constexpr int WM = WM_, WN = WN_, WTM = WTM_, WTN = WTN_, KT = KT_, STAGES = STAGES_;
    static constexpr int BM = 32 * WM * WTM, BN = 32 * WN * WTN;
    static constexpr int NW = WM * WN;
    static constexpr int PA = BM / 64, PB = BN / 64, PANELS = PA + PB;
    static constexpr int GROUPS = KT / 8;                // 8-row groups per panel
    static constexpr int PANEL_BYTES = KT * 128;
    static constexpr int TOTAL_I = PANELS * GROUPS;      // transfer instructions per stage
    static constexpr int NI = (TOTAL_I + NW - 1) / NW;
    static constexpr int STAGE_BYTES = PANELS * PANEL_BYTES;
    static constexpr int LDS_BYTES = STAGES * STAGE_BYTES;
    static_assert(BM % 64 == 0 && BN % 64 == 0, "whole 64-column panels");
    static_assert(KT % 16 == 0, "whole 16-token matrix instruction steps");
    static_assert(STAGES >= 2 && NI * (STAGES - 1) < 64, "transfers in flight must fit the counter");
};

__device__ __forceinline__ bf16x8 tr_read2(const char *p0, const char *p1)
{
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(p0));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(p1));
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

// PIPE: as in gemm_nt, the 16-token sub-steps of a stage interleave transfer issue, fragment reads and matrix instructions
template <class TL, bool PIPE = false, class ATok, class BTok, class Epi>
__device__ __forceinline__ void gemm_tn(char *lds /* TL::LDS_BYTES, 1 KB aligned */, const ATok &atok, const BTok &btok,
                                        const void *zeros, Epi &epi, int nsteps, int row0, int col0, int a_ncols,
                                        int b_ncols, int nrows, int ncols)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / TL::WN, wn = wave % TL::WN;
    f32x16 acc[TL::WTM][TL::WTN];
#pragma unroll
    for (int x = 0; x < TL::WTM; ++x)
#pragma unroll
        for (int y = 0; y < TL::WTN; ++y)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[x][y][v] = 0.f;

    if (nsteps > 0) {
        // this lane's share of the transfers of a stage: instruction ii = panel * GROUPS + group
        int pan[TL::NI], grp[TL::NI], colo[TL::NI];
        const int r8 = lane >> 3;
#pragma unroll
        for (int q = 0; q < TL::NI; ++q) {
            const int ii = min(wave + TL::NW * q, TL::TOTAL_I - 1);
            pan[q] = ii / TL::GROUPS;
            grp[q] = ii % TL::GROUPS;
            const int t = grp[q] * 8 + r8;
            const int lc = (lane & 7) ^ (2 * (t & 3));
            // column of this lane's chunk, kept inside the operand (results of such columns are dropped)
            colo[q] = pan[q] < TL::PA ? min(row0 + 64 * pan[q] + lc * 8, a_ncols - 8)
                                      : min(col0 + 64 * (pan[q] - TL::PA) + lc * 8, b_ncols - 8);
        }
        auto source = [&](int q, int step) -> const bf16_t * {
            const int s2 = min(step, nsteps - 1); // past the end: repeat the last step, never used
            const bf16_t *p = pan[q] < TL::PA ? atok(s2, grp[q], r8) : btok(s2, grp[q], r8);
            return p ? p + colo[q] : reinterpret_cast<const bf16_t *>(zeros);
        };
        const bf16_t *nxt[TL::NI];
        auto issue = [&](int slot) {
#pragma unroll
            for (int q = 0; q < TL::NI; ++q)
                dma16(nxt[q], lds + slot * TL::STAGE_BYTES + pan[q] * TL::PANEL_BYTES + grp[q] * 1024);
        };
#pragma unroll
        for (int s = 0; s < TL::STAGES - 1; ++s) {
#pragma unroll
            for (int q = 0; q < TL::NI; ++q) nxt[q] = source(q, s);
            issue(s);
        }
#pragma unroll
        for (int q = 0; q < TL::NI; ++q) nxt[q] = source(q, TL::STAGES - 1);
        // fragment addresses: lane (G = lane / 16, j = lane % 16) points at token row 8 (G/2) + j/4 (+4 for the
        // second load), columns 16 (G%2) + 4 (j%4) .. +3 of its 32-column block
        const int G = lane >> 4, j = lane & 15;
        const int v4 = j >> 2, w4 = j & 3;
        const int trow = 8 * (G >> 1) + v4;           // + 16 ks + 4 rd
        int aoff[TL::WTM], boff[TL::WTN];
#pragma unroll
        for (int x = 0; x < TL::WTM; ++x) {
            const int c = (wm * TL::WTM + x) * 32 + 16 * (G & 1) + 4 * w4; // column inside the A tile
            aoff[x] = (c >> 6) * TL::PANEL_BYTES + trow * 128 + ((((c & 63) >> 3) ^ (2 * v4)) << 4) + ((c & 4) << 1);
        }
#pragma unroll
        for (int y = 0; y < TL::WTN; ++y) {
            const int c = (wn * TL::WTN + y) * 32 + 16 * (G & 1) + 4 * w4;
            boff[y] = (TL::PA + (c >> 6)) * TL::PANEL_BYTES + trow * 128 + ((((c & 63) >> 3) ^ (2 * v4)) << 4) + ((c & 4) << 1);
        }
        int slot = 0;
        for (int st = 0; st < nsteps; ++st) {
            wait_vm<TL::NI * (TL::STAGES - 2)>(); // this wavefront's share of stage st has landed
            __syncthreads();                       // ... and everybody else's; stage st-1 is free
            if constexpr (PIPE) {
                const int nslot = slot == 0 ? TL::STAGES - 1 : slot - 1;
                const char *sb = lds + slot * TL::STAGE_BYTES;
                constexpr int KS = TL::KT / 16;
                bf16x8 a[2][TL::WTM], b[2][TL::WTN];
                auto rd = [&](int ks) {
#pragma unroll
                    for (int x = 0; x < TL::WTM; ++x)
                        a[ks & 1][x] = tr_read2(sb + aoff[x] + ks * 2048, sb + aoff[x] + ks * 2048 + 512);
#pragma unroll
                    for (int y = 0; y < TL::WTN; ++y)
                        b[ks & 1][y] = tr_read2(sb + boff[y] + ks * 2048, sb + boff[y] + ks * 2048 + 512);
                };
                rd(0);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    if (ks + 1 < KS) rd(ks + 1);
#pragma unroll
                    for (int q = ks * TL::NI / KS; q < (ks + 1) * TL::NI / KS; ++q)
                        dma16(nxt[q], lds + nslot * TL::STAGE_BYTES + pan[q] * TL::PANEL_BYTES + grp[q] * 1024);
#pragma unroll
                    for (int x = 0; x < TL::WTM; ++x)
#pragma unroll
                        for (int y = 0; y < TL::WTN; ++y)
                            acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks & 1][x], b[ks & 1][y], acc[x][y], 0, 0, 0);
                }
#pragma unroll
                for (int q = 0; q < TL::NI; ++q) nxt[q] = source(q, st + TL::STAGES);
            } else {
            issue(slot == 0 ? TL::STAGES - 1 : slot - 1);
#pragma unroll
            for (int q = 0; q < TL::NI; ++q) nxt[q] = source(q, st + TL::STAGES);
            const char *sb = lds + slot * TL::STAGE_BYTES;
            // (all fragments of the stage first, as in gemm_nt)
            bf16x8 a[TL::KT / 16][TL::WTM], b[TL::KT / 16][TL::WTN];
#pragma unroll
            for (int ks = 0; ks < TL::KT / 16; ++ks) {
#pragma unroll
                for (int x = 0; x < TL::WTM; ++x)
                    a[ks][x] = tr_read2(sb + aoff[x] + ks * 2048, sb + aoff[x] + ks * 2048 + 512);
#pragma unroll
                for (int y = 0; y < TL::WTN; ++y)
                    b[ks][y] = tr_read2(sb + boff[y] + ks * 2048, sb + boff[y] + ks * 2048 + 512);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ks = 0; ks < TL::KT / 16; ++ks)
#pragma unroll
                for (int x = 0; x < TL::WTM; ++x)
#pragma unroll
                    for (int y = 0; y < TL::WTN; ++y)
                        acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks][x], b[ks][y], acc[x][y], 0, 0, 0);
            }
            slot = slot + 1 == TL::STAGES ? 0 : slot + 1;
        }
        wait_vm<0>(); // the repeated transfers of the last steps must not outlive this use of the LDS
        __syncthreads();
    }
    tile_epilogue<TL>(acc, epi, wm, wn, lane, row0, col0, nrows, ncols);
}

} // namespace pac
