// Gram-matrix formulation of the cached Parallel-Adapter step (bf16 cache, adapter width <= 512: up to 128
// with the chains over the layers as one launch per direction, above that launched layer by layer; widths
// above 256 in multiples of 64 and with at most 32 layers).
//
// The side state is a sum of rank-r terms, s_{l-1} = sum_{k<l} (h_k W_up^k + c_up^k), and so is its
// gradient, ds_l = ds_L + sum_{k>l} (1-lambda_k) dpre_k W_down^{kT}.  Substituting both into the
// step removes every per-token d-wide intermediate except the cache itself:
//
//   forward   U_l   = b_l W_down^l                                  (streams the cache once, all layers at once)
//             pre_l = lambda_l U_l + (1-lambda_l)(sum_{k<l} h_k Q_{kl} + chat_l) + c_down^l
//                     Q_{kl} = W_up^k W_down^l (r x r), chat_l = (sum_{k<l} c_up^k) W_down^l
//   head      logits from mean(b_L), per-sample sums of h_k and V = W_up^k W_cls
//   backward  dh_l  = (dz V_l^T)/len + sum_{k>l} (1-lambda_k) dpre_k Q_{lk}^T ,  dpre_l = dh_l * GELU'(pre_l)
//   tokens    E_l = b_l^T dpre_l (streams the cache a second time), G_{kl} = h_k^T dpre_l (k < l)
//   grads     dW_down^l = lambda_l E_l + (1-lambda_l) F_l,  F_l = sum_{k<l} W_up^{kT} G_{kl} + cusum_l^T colsum(dpre_l)
//             dW_up^l   = Z_l W_cls^T + sum_{k>l} (1-lambda_k) G_{lk} W_down^{kT},  Z_l = (sum_t h_l / len)^T dz
//             dlambda_l = <E_l - F_l, W_down^l>, dc_down^l = colsum(dpre_l),
//             dc_up^l   = (sum_s dz_s) W_cls^T + sum_{k>l} (1-lambda_k) W_down^k colsum(dpre_k)
//
// This is the same function as the per-layer kernels compute (the layer-by-layer definition is the
// oracle's); only the order of the floating-point operations differs.  Every reduction is ordered.
#include "pac_mma.h"
#include "pac_internal.h"
#include <mutex>
#include <type_traits>

namespace pac {

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

constexpr int kChainRows = 16;   // token rows per chain workgroup
constexpr int kChainPad = 8;     // bf16 elements of padding per LDS row
constexpr int kMaxD = 4096;
constexpr int kETileCols = 128; // columns of d one workgroup of the E contraction covers
constexpr int kMaxSplitTiles = 512; // 16-token tiles one workgroup of the E contraction walks over at most
constexpr int kMaxTiles = 8192;     // 16-token tiles of a batch (LDS table of the column-sum reduction)
constexpr int kSeqTile = 128;       // side of the workgroup tile of a per-layer chain contraction

// Slots of the chain kernels' LDS ring of per-token inputs.  Two suffice: the helper wavefront keeps the
// tiles of the next two steps in registers and writes the tile of step s+1 while the contracting
// wavefronts read that of step s; a barrier separates that from the write of step s+2 into the same slot.
constexpr int kRing = 2;

// LDS of the chain kernels (T = kChainRows):
//   Hs   [L][T][r+pad] bf16   h (forward) or dpre (backward) of every layer: the contraction operand
//   ring [kRing][T][r]        per-token inputs of the coming layers: U (fp32, forward) or GELU' (bf16, backward)
//   Gst  [2][T][r] bf16       forward only: GELU' of the layer just finished, on its way to global memory
//   vecS [L][r] fp32          per-layer vector: (1-lambda) chat + c_down (forward), ghat of the sample (backward)
//   Cs   [L][r] fp32 column sums, lamS [L] fp32, zs / dzs [kMaxClasses] fp32 each
static size_t chain_lds(int L, int r, bool fwd)
{
    const size_t hs = (size_t)L * kChainRows * (r + kChainPad) * 2;
    const size_t ring = (size_t)kRing * kChainRows * r * (fwd ? 4 : 2);
    const size_t gstage = fwd ? (size_t)2 * kChainRows * r * 2 : 0;
    return hs + ring + gstage + (size_t)L * r * 4 * 2 + (size_t)((L + 3) / 4 * 4) * 4 + 2 * kMaxClasses * 4;
}

// Side of the square workgroup tiles of the contractions outside the chains: 64 up to r = 128, 128 above
static int big_shapes(int r) { return r > 128; }

int gram_path_kind(const Dims &D)
{
    if (D.cache_dtype != 0 || (D.flags & 1)) return 0; // PAC_FLAG_PER_LAYER
    if (D.r > 512 || D.d > kMaxD || D.L > 128) return 0;
    // above 256: the vector part of the gradient launch deals eight threads over an r-wide row (16-byte pieces)
    // and 32 such rows over the layers
    if (D.r > 256 && (D.r % 64 != 0 || D.L > 32)) return 0;
    if ((int64_t)D.B_max * cdiv(D.n_max, kChainRows) > kMaxTiles) return 0;
    const bool lds_chain = D.r <= 128 && chain_lds(D.L, D.r, true) <= 160 * 1024;
    if (lds_chain && !(D.flags & 4)) return 1; // PAC_FLAG_LAYER_CHAIN
    // one chain launch per layer; the vector part of the gradient launch deals 64 threads over the layers
    return D.L <= (big_shapes(D.r) ? 64 : 128) ? 2 : 0;
}

void plan_gram_workspace(const Dims &D, WsLayout &W, int64_t &o)
{
    auto take = [&](int64_t bytes) { int64_t at = o; o = align256(o + bytes); return at; };
    const int64_t Lr = (int64_t)D.L * D.r;
    W.use_gram = gram_path_kind(D);
    W.max_tiles = D.B_max * cdiv(D.n_max, kChainRows);
    W.pairs = D.L * (D.L - 1) / 2;
    const int e_tiles = D.L * cdiv(D.d, kETileCols) * cdiv(D.r, 128);
    // Token splits of E (measured): with few tiles (T5-Base-shaped: 72) E's workgroups and the Gram tiles that
    // run beside them should all be resident at once, two per compute unit; with more tiles than that anyway
    // (Large-shaped: 192) two splits measured best (113 us for the launch against 117 with three, 152 with one).
    int se = cdiv(e_tiles >= 128 ? 384 : 288, e_tiles);
    const int max_by_rows = (int)((D.Mmax + 127) / 128);
    if (se > max_by_rows) se = max_by_rows;
    W.se = se < 1 ? 1 : (se > 16 ? 16 : se);
    if (cdiv(W.max_tiles, W.se) > kMaxSplitTiles) W.se = cdiv(W.max_tiles, kMaxSplitTiles); // LDS tile table of k_gtokred
    const int tg = cdiv(Lr, 128);
    // Token splits of the Gram matrix: about 128 of its workgroups (they run beside E's; at the T5-Base shape four
    // splits of 45 tiles measured 2 us faster in this launch than eight, and the ordered sum afterwards reads half the
    // partials).
    int sg = cdiv(128, (int64_t)tg * (tg + 1) / 2);
    // A power of two: the Gram tiles are numbered with the split fastest and dealt round-robin over the eight
    // dies, so a die then only ever reads the token rows of its own split(s) of H and DP (with six splits
    // every die fetched most of both matrices: 63 MB over the fabric for 19 MB of operands).
    for (int p2 = 1; p2 <= 16; p2 *= 2)
        if (sg <= p2) { sg = p2; break; }
    if (sg > max_by_rows) sg = max_by_rows;
    W.sg = sg < 1 ? 1 : (sg > 16 ? 16 : sg);
    W.g_zero = take(256);
    W.g_tile_row0 = take(W.max_tiles * 4);
    W.g_tile_rows = take(W.max_tiles * 4);
    W.g_tile_samp = take(W.max_tiles * 4);
    W.g_WuTs = take((int64_t)D.d * Lr * 2);
    W.g_Wds = take((int64_t)D.d * Lr * 2);
    W.g_cusum = take((int64_t)(D.L + 1) * D.d * 4);
    W.g_chat = take(Lr * 4);
    W.g_V = take(Lr * D.C * 4);
    const int64_t q_bytes = W.use_gram == 2 ? Lr * Lr * 2 : (int64_t)(W.pairs + 1) * D.r * D.r * 2;
    W.g_QpN = take(q_bytes);
    W.g_QpT = take(q_bytes);
    W.chain_group = 1;
    W.g_P = W.g_ghat = W.g_QgN = W.g_QgT = 0;
    if (W.use_gram == 2) {
        // layers per group of the layer-by-layer chains: about 1024 columns per wide contraction
        const int g = 1024 / D.r;
        W.chain_group = g < 1 ? 1 : (g > 8 ? 8 : g);
        W.g_P = take(D.Mmax * (int64_t)W.chain_group * D.r * 4);
        W.g_ghat = take((int64_t)D.B_max * Lr * 4);
        const int64_t in_group = (int64_t)cdiv(D.L, W.chain_group) * (W.chain_group * (W.chain_group - 1) / 2);
        W.g_QgN = take((in_group + 1) * D.r * D.r * 2);
        W.g_QgT = take((in_group + 1) * D.r * D.r * 2);
    }
    W.g_DP = take(D.Mmax * Lr * 2);
    W.g_Gp = take(D.Mmax * Lr * 2);
    W.g_HSpart = take((int64_t)W.max_tiles * Lr * 4);
    W.g_cspart = take((int64_t)W.max_tiles * Lr * 4);
    W.g_zpart = take((int64_t)W.max_tiles * D.C * 4);
    W.g_zpb = take((int64_t)D.B_max * cdiv(D.d, 256) * D.C * 4);
    W.g_Z = take(Lr * D.C * 4);
    W.g_dzsum = take(kMaxClasses * 4);
    W.g_cs = take(Lr * 4);
    W.g_Epart = take((int64_t)W.se * D.L * D.d * D.r * 4);
    W.g_GGpart = take((int64_t)W.sg * Lr * Lr * 4);
    W.g_E = take((int64_t)D.L * D.d * D.r * 4);
    W.g_GGT = take(Lr * Lr * 2);
    W.g_GGsc = take(Lr * Lr * 2);
    W.g_dlam_slots = cdiv(D.d, 64) * cdiv(D.r, 64);
    W.g_dlam_part = take((int64_t)D.L * W.g_dlam_slots * 4);
    W.g_samp_tile0 = take((kMaxBatch + 1) * 4);
    W.g_loss_part = take(kMaxBatch * 4);
}

// Copies n floats (n % 4 == 0, both sides 16-byte aligned) from global memory to LDS with all of a
// round's loads issued before its first store: a plain copy loop waits for memory once per iteration.
template <int NTHREADS> __device__ __forceinline__ void stage_to_lds(float *dst, const float *src, int n)
{
    const int nch = n >> 2;
    for (int base = 0; base < nch; base += NTHREADS * 8) {
        f32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            v[u] = *reinterpret_cast<const f32x4 *>(src + 4 * min(base + u * NTHREADS + (int)threadIdx.x, nch - 1));
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int c = base + u * NTHREADS + (int)threadIdx.x;
            if (c < nch) *reinterpret_cast<f32x4 *>(dst + 4 * c) = v[u];
        }
    }
}

__device__ __forceinline__ float gelu_f(float u) { return 0.5f * u * (1.f + erff(u * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_grad_f(float u)
{
    const float Phi = 0.5f * (1.f + erff(u * 0.70710678118654752f));
    const float phi = 0.3989422804014327f * expf(-0.5f * u * u);
    return Phi + u * phi;
}
__device__ __forceinline__ int pair_index(int k, int l) { return l * (l - 1) / 2 + k; } // k < l

// Workgroups are handed to the eight accelerator dies (each with its own L2) round-robin by block
// index.  Given a part's block number u in [0, n) (any numbering that differs from the hardware block
// index by a constant, or runs against it), this returns a tile number such that each die works
// through one contiguous range of tile numbers in order: tiles that share an operand and are numbered
// next to each other then meet in the same L2 instead of each die fetching the operand for itself.
__device__ __forceinline__ int die_chunk_order(int u, int n)
{
    const int q = n >> 3, rem = n & 7, x = u & 7, s = u >> 3;
    return x * q + min(x, rem) + s;
}
// The same in windows of 8 * gs blocks: within a window each die gets gs consecutive tile numbers, and
// the windows keep the launch's overall order (for parts whose tiles differ in cost and are numbered
// with that in mind).  The blocks past the last whole window keep their numbers.
__device__ __forceinline__ int die_group_order(int u, int n, int gs)
{
    const int w = 8 * gs;
    if (u >= (n / w) * w) return u;
    const int in = u % w;
    return u - in + (in & 7) * gs + (in >> 3);
}

// ---------------------------------------------------------------------------
// launch 1: batch gather, token tiles, projection copies, cusum/chat, V
// ---------------------------------------------------------------------------
constexpr int kPrepTiles = 4; // 32 x 32 tiles of the projection matrices one workgroup of the set-up launch copies

struct PrepArgs {
    int blk_off; // first block of this launch (parts may be launched separately for timing)
    BatchMeta meta;
    const float *params;
    int64_t PL;
    int L, d, r, C;
    int nb_setup, nb_shadow, nb_chat;
    int tile64; // the copy part works on 64 x 64 tiles (d, r multiples of 64; TPB = 4): every store a full 128-byte line
    int64_t *rowoff;
    int32_t *rowstride, *rowsamp, *samp_start, *samp_len;
    int32_t *tile_row0, *tile_rows, *tile_samp, *samp_tile0;
    bf16_t *WdT, *Wu, *WuTs, *Wds;
    float *cusum, *V;
    float *zero; // 64 floats kept at zero for the contractions' empty token slots
};

// TPB weight tiles per workgroup of the copy part, RPW rows of V per wavefront: 1, 1 for small shapes
template <int TPB, int RPW> __global__ __launch_bounds__(256) void k_gprep(PrepArgs a)
{
    __shared__ float sh[TPB * 32 * 33];
    const int b = blockIdx.x + a.blk_off, t = threadIdx.x;
    const int L = a.L, d = a.d, r = a.r, C = a.C;
    const int64_t Lr = (int64_t)L * r;
    if (b < a.nb_setup) {
        const BatchMeta &meta = a.meta;
        if (b == 0) {
            if (t <= meta.B) {
                a.samp_start[t] = meta.tok_start[t];
                if (t < meta.B) a.samp_len[t] = meta.len[t];
            }
            if (t < 64) a.zero[t] = 0.f;
            if (t < meta.B) {
                // tiles of sample t start after the tiles of the samples before it
                int nt = 0;
                for (int q = 0; q < t; ++q) nt += (meta.len[q] + kChainRows - 1) / kChainRows;
                a.samp_tile0[t] = nt;
                for (int t0 = 0; t0 < meta.len[t]; t0 += kChainRows) {
                    a.tile_row0[nt] = meta.tok_start[t] + t0;
                    a.tile_rows[nt] = min(kChainRows, meta.len[t] - t0);
                    a.tile_samp[nt] = t;
                    ++nt;
                }
                if (t == meta.B - 1) a.samp_tile0[meta.B] = nt;
            }
        }
        const int m = b * 256 + t;
        if (m >= meta.M) return;
        int lo = 0, hi = meta.B - 1; // last sample whose first row is <= m
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (meta.tok_start[mid] <= m) lo = mid; else hi = mid - 1;
        }
        const int s = lo;
        a.rowoff[m] = meta.off[s] + (int64_t)(m - meta.tok_start[s]) * d;
        a.rowstride[m] = meta.len[s] * d;
        a.rowsamp[m] = s;
        return;
    }
    if (TPB == 4 && a.tile64 && b < a.nb_setup + a.nb_shadow) {
        // One 64 x 64 tile of W_down^k (which = 0, [d][r]) or W_up^k (which = 1, [r][d]).  A wavefront stores 64
        // neighbouring bf16 values at a time, a whole 128-byte line, in the straight copy and in the transposed one:
        // with 32 x 32 tiles every store was half a line whose other half came from another workgroup much later, and
        // the launch fetched 1.75 x the parameter bytes.
        const int per_mat = (d / 64) * (r / 64);
        int idx = b - a.nb_setup;
        const int which = idx / (per_mat * L);
        idx -= which * per_mat * L;
        const int kk = idx / per_mat;
        idx -= kk * per_mat;
        const int cols = which == 0 ? r : d, tiles_c = cols / 64;
        const int r0 = (idx / tiles_c) * 64, c0 = (idx % tiles_c) * 64;
        const int tx = t & 63, ty = t >> 6;
        const float *src = a.params + (int64_t)kk * a.PL + (which == 0 ? 0 : (int64_t)d * r + r);
        float v[16];
#pragma unroll
        for (int yi = 0; yi < 16; ++yi) v[yi] = src[(int64_t)(r0 + ty + 4 * yi) * cols + c0 + tx];
        float(*tile)[65] = reinterpret_cast<float(*)[65]>(sh); // 64 x 65 floats = TPB * 32 * 33 * 4 bytes or less
        static_assert(TPB != 4 || 64 * 65 <= TPB * 32 * 33, "LDS of the 64 x 64 tile");
#pragma unroll
        for (int yi = 0; yi < 16; ++yi) {
            const int y = ty + 4 * yi, row = r0 + y, col = c0 + tx;
            tile[y][tx] = v[yi];
            if (which == 0) a.Wds[(int64_t)row * Lr + (int64_t)kk * r + col] = static_cast<bf16_t>(v[yi]);
            else a.Wu[((int64_t)kk * r + row) * d + col] = static_cast<bf16_t>(v[yi]);
        }
        __syncthreads();
#pragma unroll
        for (int yi = 0; yi < 16; ++yi) {
            // element (row = r0 + tx, col = c0 + y) written at the transposed position
            const int y = ty + 4 * yi, row = r0 + tx, col = c0 + y;
            const bf16_t w = static_cast<bf16_t>(tile[tx][y]);
            if (which == 0) a.WdT[((int64_t)kk * r + col) * d + row] = w;
            else a.WuTs[(int64_t)col * Lr + (int64_t)kk * r + row] = w;
        }
        return;
    }
    if (b < a.nb_setup + a.nb_shadow) {
        // TPB 32 x 32 tiles of W_down^k (which = 0, [d][r]) or W_up^k (which = 1, [r][d]); all loads first
        const int per_mat = (d / 32) * (r / 32);
        const int total = 2 * L * per_mat;
        const int t0 = (b - a.nb_setup) * TPB;
        const int tx = t & 31, ty = t >> 5;
        float v[TPB][4];
        int which[TPB], kk[TPB], trr[TPB], tcc[TPB];
#pragma unroll
        for (int q = 0; q < TPB; ++q) {
            int idx = min(t0 + q, total - 1);
            which[q] = idx / (per_mat * L);
            idx -= which[q] * per_mat * L;
            kk[q] = idx / per_mat;
            idx -= kk[q] * per_mat;
            const int cols = which[q] == 0 ? r : d;
            const int tiles_c = cols / 32;
            trr[q] = idx / tiles_c;
            tcc[q] = idx % tiles_c;
            const float *src = a.params + (int64_t)kk[q] * a.PL + (which[q] == 0 ? 0 : (int64_t)d * r + r);
#pragma unroll
            for (int yi = 0; yi < 4; ++yi)
                v[q][yi] = src[(int64_t)(trr[q] * 32 + ty + 8 * yi) * cols + tcc[q] * 32 + tx];
        }
        float(*tile)[32][33] = reinterpret_cast<float(*)[32][33]>(sh);
#pragma unroll
        for (int q = 0; q < TPB; ++q) {
            if (t0 + q >= total) continue;
#pragma unroll
            for (int yi = 0; yi < 4; ++yi) {
                const int y = ty + 8 * yi, row = trr[q] * 32 + y, col = tcc[q] * 32 + tx;
                tile[q][y][tx] = v[q][yi];
                if (which[q] == 0) a.Wds[(int64_t)row * Lr + (int64_t)kk[q] * r + col] = static_cast<bf16_t>(v[q][yi]);
                else a.Wu[((int64_t)kk[q] * r + row) * d + col] = static_cast<bf16_t>(v[q][yi]);
            }
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < TPB; ++q) {
            if (t0 + q >= total) continue;
#pragma unroll
            for (int yi = 0; yi < 4; ++yi) {
                // element (row = tr*32 + tx, col = tc*32 + y) written at the transposed position
                const int y = ty + 8 * yi, row = trr[q] * 32 + tx, col = tcc[q] * 32 + y;
                const bf16_t w = static_cast<bf16_t>(tile[q][tx][y]);
                if (which[q] == 0) a.WdT[((int64_t)kk[q] * r + col) * d + row] = w;
                else a.WuTs[(int64_t)col * Lr + (int64_t)kk[q] * r + row] = w;
            }
        }
        return;
    }
    if (b < a.nb_setup + a.nb_shadow + a.nb_chat) {
        // cusum_l = sum_{k<l} c_up^k for l = 0..L (fp32 master values)
        const int j = (b - a.nb_setup - a.nb_shadow) * 256 + t;
        if (j >= d) return;
        float acc = 0.f;
        a.cusum[j] = 0.f;
        for (int l0 = 0; l0 < L; l0 += 8) { // eight layers' loads issued together
            float cu[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                cu[u] = a.params[(int64_t)min(l0 + u, L - 1) * a.PL + 2 * (int64_t)d * r + r + j];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (l0 + u < L) {
                    acc += cu[u];
                    a.cusum[(int64_t)(l0 + u + 1) * d + j] = acc;
                }
        }
        return;
    }
    {
        // V[(k,a)][c] = sum_j W_up^k[a][j] W_cls[j][c]; a wavefront takes RPW consecutive rows and
        // reads each piece of W_cls once for all of them
        constexpr int kRpw = RPW;
        const int row0 = ((b - a.nb_setup - a.nb_shadow - a.nb_chat) * 4 + (t >> 6)) * kRpw;
        if (row0 >= Lr) return;
        const int lane = t & 63;
        const float *Wc = a.params + (int64_t)L * a.PL;
        const float *wu[kRpw];
        float acc[kRpw][kMaxClasses];
#pragma unroll
        for (int q = 0; q < kRpw; ++q) {
            const int row = min(row0 + q, (int)Lr - 1);
            wu[q] = a.params + (int64_t)(row / r) * a.PL + (int64_t)d * r + r + (int64_t)(row % r) * d;
#pragma unroll
            for (int c = 0; c < kMaxClasses; ++c) acc[q][c] = 0.f;
        }
        // eight columns per lane and round, their loads issued together (d is a multiple of 32)
        for (int j0 = 0; j0 < d; j0 += 64 * 8) {
            float w[kRpw][8];
#pragma unroll
            for (int q = 0; q < kRpw; ++q)
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int j = j0 + 64 * u + lane;
                    w[q][u] = j < d ? wu[q][j] : 0.f;
                }
#pragma unroll
            for (int c = 0; c < kMaxClasses; ++c) { // (unrolled: the accumulators stay in registers)
                if (c >= C) continue;
                float wc[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) wc[u] = Wc[(int64_t)min(j0 + 64 * u + lane, d - 1) * C + c];
#pragma unroll
                for (int q = 0; q < kRpw; ++q)
#pragma unroll
                    for (int u = 0; u < 8; ++u) acc[q][c] += w[q][u] * wc[u];
            }
        }
#pragma unroll
        for (int q = 0; q < kRpw; ++q) {
            if (row0 + q >= Lr) continue;
#pragma unroll
            for (int c = 0; c < kMaxClasses; ++c) {
                if (c >= C) continue;
                float v = acc[q][c];
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
                if (lane == 0) a.V[(int64_t)(row0 + q) * C + c] = v;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// launch 2: U_l = b_l W_down^l for every layer, Q_{kl} = W_up^k W_down^l, mean(b_L)
// ---------------------------------------------------------------------------
struct ProjArgs {
    int blk_off; // first block of this launch (parts may be launched separately for timing)
    const bf16_t *cache;
    RowMap map;
    int L, d, r, B;
    int nb_U, nb_Q, nb_C, row_tiles;
    const bf16_t *WdT, *Wu;
    const float *cusum; // [L+1][d]
    float *chat;        // [L][r]
    const float *params;
    int64_t PL;
    float *U;          // [L][M][r]
    bf16_t *QpN, *QpT; // [pairs][r][r] in fragment-major order (EpiQ), or (q_full) [L*r][L*r] each (EpiQFull)
    bf16_t *QgN, *QgT; // q_full: the pairs inside a group of chain_group layers once more, fragment-major
    int chain_group;
    const int32_t *samp_start, *samp_len;
    float *pb; // [B][d]
    int C;
    float *zpbp; // [B][ceil(d/256)][C]: ((mean b_L + sum of all c_up) W_cls) summed over this block's 256 columns
};

struct EpiStoreF32 {
    float *out;
    int64_t ld;
    __device__ void operator()(int row, int col, float v) const { out[(int64_t)row * ld + col] = v; }
};

// The Gram matrix straight from the token contraction where the tokens are not split: the two bf16 copies the
// gradient launch contracts (GG transposed; GG with column layer l scaled by 1 - lambda_l), for the 32 x 32 blocks
// with a row layer below a column layer, exactly what the ordered sum of the partials writes otherwise.
struct EpiGramDirect {
    static constexpr bool kBatched = true;
    bf16_t *ggt, *ggsc;
    int64_t Lr;
    int r;
    const float *params;
    int64_t PL;
    __device__ void batch(int row_base, int col, const f32x16 &acc, int nrows, int ncols) const
    {
        // (every condition below is the same for the two lanes lane and lane ^ 32, which hold the same column and the
        // two interleaved halves of the block's 32 rows: the exchange further down needs both)
        if (col >= ncols || (row_base & ~31) >= nrows) return; // nrows is a multiple of 32
        if ((row_base & ~31) / r >= ((col & ~31) + 31) / r) return;
        const float oml = 1.f - params[(int64_t)(col / r) * PL + PL - 1]; // read before the first store
        uint32_t t[4][2]; // this lane's rows 8 vg + 4 g .. + 3 of the block as bf16 pairs
#pragma unroll
        for (int vg = 0; vg < 4; ++vg) {
            const int row = row_base + 8 * vg;
            bf16_t t4[4];
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                ggsc[(int64_t)(row + w) * Lr + col] = static_cast<bf16_t>(oml * acc[4 * vg + w]);
                t4[w] = static_cast<bf16_t>(acc[4 * vg + w]);
            }
            __builtin_memcpy(t[vg], t4, 8);
        }
        // Transposed copy: a column's 32 rows are 64 contiguous bytes, of which this lane holds every other 8.  The
        // lane pair swaps two of its four pieces so that each lane stores two 16-byte pieces instead of four of 8.
        const int g = (threadIdx.x >> 5) & 1;
        uint32_t recv[2][2];
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int h = 0; h < 2; ++h) recv[u][h] = __shfl_xor(g ? t[2 * u][h] : t[2 * u + 1][h], 32, 64);
        bf16_t *dst = ggt + (int64_t)col * Lr + (row_base & ~31);
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            // g = 0: rows 16 u .. 16 u + 7 = own piece 2 u, then the partner's; g = 1: rows 16 u + 8 .. + 15 = the
            // partner's piece 2 u + 1, then own
            u32x4 v;
            if (g == 0) { v[0] = t[2 * u][0]; v[1] = t[2 * u][1]; v[2] = recv[u][0]; v[3] = recv[u][1]; }
            else { v[0] = recv[u][0]; v[1] = recv[u][1]; v[2] = t[2 * u + 1][0]; v[3] = t[2 * u + 1][1]; }
            *reinterpret_cast<u32x4 *>(dst + 16 * u + 8 * g) = v;
        }
    }
};

// Q is stored twice, each time in the order the chain kernels' matrix instructions consume it
// ("fragment-major"): for the contraction sum_kk A[.][kk] B[n][kk] in 16-column x 32-deep operand
// fragments, element B[n][kk] sits at
//   ((n/16 * r/32 + kk/32) * 64 + (n%16) + 16*((kk%32)/8)) * 8 + kk%8,
// so that one wavefront load of a fragment reads 1 KB contiguously.
__device__ __forceinline__ int64_t frag_index(int n, int kk, int r)
{
    return ((int64_t)((n >> 4) * (r >> 5) + (kk >> 5)) * 64 + (n & 15) + 16 * ((kk & 31) >> 3)) * 8 + (kk & 7);
}

struct EpiQ {
    bf16_t *qn, *qt;
    int r;
    float one_minus_lam; // of the later layer of the pair: the backward chain uses (1-lambda_l) Q_{kl}
    __device__ void operator()(int row, int col, float v) const
    {
        qn[frag_index(row, col, r)] = static_cast<bf16_t>(one_minus_lam * v); // backward: B[n=row][kk=col]
        qt[frag_index(col, row, r)] = static_cast<bf16_t>(v);                 // forward:  B[n=col][kk=row]
    }
};

// All products Q_{kl} of the single-launch chains from ONE contraction over the stacked projections: row (k, j) of the
// stacked up-projections against column (l, n) of the stacked down-projections; only k < l is kept.
struct EpiQStacked {
    static constexpr bool kBatched = true;
    static constexpr int kLayers = 6; // column layers one 128-column tile can touch (r >= 32)
    bf16_t *qn, *qt; // [pair][r x r], fragment-major (frag_index)
    int r, l0;       // first column layer of the tile
    float one_minus_lam[kLayers]; // of layers l0 .., read before the first store (a load behind a store waits for it)
    // r is a multiple of 32, so a 32 x 32 block of the stacked product lies inside one pair (k, l)
    __device__ void batch(int row_base, int col, const f32x16 &acc, int nrows, int ncols) const
    {
        if (col >= ncols || row_base >= nrows) return;
        const int k = row_base / r, l = col / r;
        if (k >= l) return;
        const int jb = row_base - k * r, n = col - l * r;
        float oml = one_minus_lam[0];
#pragma unroll
        for (int i = 1; i < kLayers; ++i) oml = l - l0 == i ? one_minus_lam[i] : oml;
        bf16_t *pn = qn + (int64_t)pair_index(k, l) * r * r, *pt = qt + (int64_t)pair_index(k, l) * r * r;
#pragma unroll
        for (int vg = 0; vg < 4; ++vg) {
            const int j = jb + 8 * vg; // four consecutive rows j .. j+3, j a multiple of 4
            bf16_t t4[4];
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                pn[frag_index(j + w, n, r)] = static_cast<bf16_t>(oml * acc[4 * vg + w]); // backward: B[n=row][kk=col]
                t4[w] = static_cast<bf16_t>(acc[4 * vg + w]);
            }
            __builtin_memcpy(pt + frag_index(n, j, r), t4, 8); // forward: B[n=col][kk=row], kk = j .. j+3 adjacent
        }
    }
};

// The layer-by-layer chains read Q from two [L*r][L*r] matrices whose row (layer, n) holds, K-contiguous
// over (layer', j), the second operand of their contractions:
//   qt[(l, col)][(k, row)] = Q_{kl}[row][col]  and  qn[(k, row)][(l, col)] = (1-lambda_l) Q_{kl}[row][col].
struct EpiQFull {
    static constexpr bool kBatched = true;
    bf16_t *qn, *qt;
    int r;
    float one_minus_lam;
    int k, l;
    int64_t Lr;
    bf16_t *gn, *gt; // this pair's fragment-major blocks when both layers are in one group, else null
    __device__ void batch(int row_base, int col, const f32x16 &acc, int nrows, int ncols) const
    {
        if (col >= ncols) return;
        if (gt) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = epi_row(row_base, v);
                if (row < nrows) {
                    gn[frag_index(row, col, r)] = static_cast<bf16_t>(one_minus_lam * acc[v]); // backward: B[n=row][kk=col]
                    gt[frag_index(col, row, r)] = static_cast<bf16_t>(acc[v]);                 // forward:  B[n=col][kk=row]
                }
            }
        }
        bf16_t *qt_row = qt + ((int64_t)l * r + col) * Lr + (int64_t)k * r;
        bf16_t *qn_col = qn + (int64_t)k * r * Lr + (int64_t)l * r + col;
#pragma unroll
        for (int vg = 0; vg < 4; ++vg) {
            const int row = row_base + 8 * vg; // four consecutive rows; nrows is a multiple of 4
            if (row < nrows) {
                bf16x4 pk;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    pk[e] = static_cast<bf16_t>(acc[4 * vg + e]);
                    qn_col[(int64_t)(row + e) * Lr] = static_cast<bf16_t>(one_minus_lam * acc[4 * vg + e]);
                }
                *reinterpret_cast<bf16x4 *>(qt_row + row) = pk;
            }
        }
    }
};

struct EpiChat {
    float *chat_l;
    __device__ void operator()(int row, int col, float v) const
    {
        if (row == 0) chat_l[col] = v;
    }
};

using T64 = Tile<2, 2, 1, 1, 1>;
using T64K = Tile<2, 2, 1, 1, 4>; // 128-token K step for the token contractions

// Stage counts are kept small on purpose: more workgroups per compute unit hide the memory latency
// better than deeper rings in fewer workgroups (measured both ways).
template <int NT, int BK, bool QFULL = false> struct ProjShapes {
    static constexpr bool BIG = NT > 4;
    static constexpr bool QSTACK = !BIG && !QFULL; // Q as one contraction over the stacked projections
    // r > 128: 128 x 256 tiles (all of r), eight wavefronts, three stages, interleaved sub-steps; one workgroup per CU
    using TBig = NtTile<2, 4, 2, 2, BK, 3>;
    using TU = typename std::conditional<BIG, TBig, NtTile<4, 1, 1, (BIG ? 1 : NT), BK, 2>>::type; // 128 token rows x r
    using TQ = typename std::conditional<BIG, TBig, typename std::conditional<QSTACK, NtTile<2, 2, 2, 2, BK, 2>, NtTile<2, 2, 1, 1, BK, 3>>::type>::type; // 128 x 128 of the stacked product, 64 x 64 of a pair, or 128 x 256
    static constexpr int kThreadsPerBlock = BIG ? 512 : 256;
    using TC = Tile<2, 2, 1, 1, BK / 32>;   // the one-row chat contraction (staged through registers)
    static constexpr int kUStages = 3; // the small shapes' U tile: three stages of cache rows, two of the projection
    static constexpr int kULds = BIG ? TU::LDS_BYTES : nt_deepA_lds<TU, kUStages>();
    static constexpr int kA = kULds > TQ::LDS_BYTES ? kULds : TQ::LDS_BYTES;
    static constexpr int kB = tile_lds_bytes<bf16_t, TC>() > 8 * 256 * 4 ? tile_lds_bytes<bf16_t, TC>() : 8 * 256 * 4;
    static constexpr int kLds = kA > kB ? kA : kB;
};

template <int NT, int BK, bool QFULL> __global__ __launch_bounds__(NT > 4 ? 512 : 256) void k_gproj(ProjArgs a)
{
    using SH = ProjShapes<NT, BK, QFULL>;
    using TU = typename SH::TU;
    using TQ = typename SH::TQ;
    constexpr int KU = BK / 32;
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    // Workgroups are numbered with the big streaming part first.  Where Q is one stacked contraction (few tiles) they
    // are dispatched in that order: every U tile starts at once, the few Q tiles take the slots left over, and Q is
    // the last thing written before the chain that reads it (time stamps: with Q as four 64 x 64 tiles per pair,
    // dispatched first, the median U tile waited 7 us for a slot).  The wide shapes dispatch in reverse: their small
    // latency-bound parts start at once and run alongside the stream.
    const int b = (SH::QSTACK ? (int)blockIdx.x : (int)(gridDim.x - 1 - blockIdx.x)) + a.blk_off;
    if (b < a.nb_U) {
        // (layer, row tile, column tile), the column tiles of a row tile next to each other
        // Wide shapes: the tiles of a layer go to one die, which then fetches that layer's projection once (numbered
        // round-robin every die fetched every layer's: half as many bytes again as the cache itself).
        const int uct = (a.r + TU::BN - 1) / TU::BN;
        const int v = SH::BIG ? die_group_order(b, a.nb_U, uct * a.row_tiles) : b;
        const int ct = v % uct, mt = (v / uct) % a.row_tiles, l = v / (uct * a.row_tiles);
        const bf16_t *cache = a.cache;
        const RowMap map = a.map;
        const bf16_t *W = a.WdT + (int64_t)l * a.r * a.d;
        const int d = a.d;
        auto arow = [&](int m) { return cache + map.rowoff[m] + (int64_t)l * map.rowstride[m]; };
        auto brow = [&](int c) { return W + (int64_t)c * d; };
        EpiStoreF32 epi{a.U + (int64_t)l * a.map.M * a.r, a.r};
        if constexpr (SH::BIG) gemm_nt<TU, true>(smem, arow, brow, epi, 0, a.d, mt * TU::BM, ct * TU::BN, a.map.M, a.r);
        else gemm_nt_deepA<TU, SH::kUStages>(smem, arow, brow, epi, 0, a.d, mt * TU::BM, ct * TU::BN, a.map.M, a.r);
        return;
    }
    const int tqm = (a.r + TQ::BM - 1) / TQ::BM, tqn = (a.r + TQ::BN - 1) / TQ::BN, tq2 = tqm * tqn, tc64 = (a.r + 63) / 64;
    if (b < a.nb_U + a.nb_Q) {
        if constexpr (SH::QSTACK) {
            // tile (ti, tj) of [L r] x [L r]; needed where some row layer is below some column layer
            const int Lr = a.L * a.r, tq = (Lr + TQ::BN - 1) / TQ::BN;
            const int idx = b - a.nb_U, ti = idx / tq, tj = idx % tq;
            if ((ti * TQ::BM) / a.r >= min(Lr - 1, tj * TQ::BN + TQ::BN - 1) / a.r) return;
            const bf16_t *Wu = a.Wu, *Wd = a.WdT;
            const int d = a.d;
            auto arow = [&](int row) { return Wu + (int64_t)row * d; };
            auto brow = [&](int c) { return Wd + (int64_t)c * d; };
            EpiQStacked epi;
            epi.qn = a.QpN; epi.qt = a.QpT; epi.r = a.r; epi.l0 = (tj * TQ::BN) / a.r;
#pragma unroll
            for (int i = 0; i < EpiQStacked::kLayers; ++i)
                epi.one_minus_lam[i] = 1.f - a.params[(int64_t)min(epi.l0 + i, a.L - 1) * a.PL + a.PL - 1];
            gemm_nt<TQ>(smem, arow, brow, epi, 0, a.d, ti * TQ::BM, tj * TQ::BN, Lr, Lr);
            return;
        }
        int idx, k, l, p;
        if constexpr (SH::BIG) {
            // Blocks of 4 x 4 layer pairs (k in 4 kb.., l in 4 lb.., kb <= lb), one block per die at a time: its tiles
            // read 4 + 4 projection matrices between them instead of two each (numbered pair by pair and round-robin,
            // the 134 MB of projections crossed the fabric ten times).  Slots with k >= l or past L are empty.
            const int per_block = 16 * tq2;
            int v = die_group_order(b - a.nb_U, a.nb_Q, per_block);
            const int blk = v / per_block;
            v -= blk * per_block;
            int lb = 0;
            while ((lb + 1) * (lb + 2) / 2 <= blk) ++lb;
            const int kb = blk - lb * (lb + 1) / 2;
            const int pr = v / tq2;
            idx = v - pr * tq2;
            k = 4 * kb + (pr & 3);
            l = 4 * lb + (pr >> 2);
            if (k >= l || l >= a.L) return;
            p = pair_index(k, l);
        } else {
            idx = b - a.nb_U;
            p = idx / tq2;
            idx -= p * tq2;
            // pair p = (k, l), k < l
            l = 1;
            while ((l + 1) * l / 2 <= p) ++l;
            k = p - l * (l - 1) / 2;
        }
        const bf16_t *Wu = a.Wu + (int64_t)k * a.r * a.d, *Wd = a.WdT + (int64_t)l * a.r * a.d;
        const int d = a.d;
        auto arow = [&](int row) { return Wu + (int64_t)row * d; };
        auto brow = [&](int c) { return Wd + (int64_t)c * d; };
        const float oml = 1.f - a.params[(int64_t)l * a.PL + a.PL - 1];
        if constexpr (QFULL) {
            // slot of an in-group pair: the forward chain reaches it at step (l - l0, k - l0) of its group, the
            // backward chain at step (l1 - 1 - k, l1 - 1 - l); slot of step (q, j) = q (q - 1) / 2 + j
            const int g = a.chain_group, gi = l / g;
            bf16_t *gn = nullptr, *gt = nullptr;
            if (k / g == gi) {
                const int l0 = gi * g, l1 = min(l0 + g, a.L), pg = g * (g - 1) / 2;
                const int qf = l - l0, jf = k - l0, qb = l1 - 1 - k, jb = l1 - 1 - l;
                gt = a.QgT + ((int64_t)gi * pg + qf * (qf - 1) / 2 + jf) * a.r * a.r;
                gn = a.QgN + ((int64_t)gi * pg + qb * (qb - 1) / 2 + jb) * a.r * a.r;
            }
            EpiQFull epi{a.QpN, a.QpT, a.r, oml, k, l, (int64_t)a.L * a.r, gn, gt};
            gemm_nt<TQ, true>(smem, arow, brow, epi, 0, a.d, (idx / tqn) * TQ::BM, (idx % tqn) * TQ::BN, a.r, a.r);
        } else {
            EpiQ epi{a.QpN + (int64_t)p * a.r * a.r, a.QpT + (int64_t)p * a.r * a.r, a.r, oml};
            gemm_nt<TQ, true>(smem, arow, brow, epi, 0, a.d, (idx / tqn) * TQ::BM, (idx % tqn) * TQ::BN, a.r, a.r);
        }
        return;
    }
    if (b < a.nb_U + a.nb_Q + a.nb_C) {
        // chat_l = cusum_l W_down^l: a one-row contraction on the same tile code (four wavefronts)
        if (SH::BIG && threadIdx.x >= 256) return;
        const int idx = b - a.nb_U - a.nb_Q;
        const int l = idx / tc64, nt = idx % tc64;
        LoadRowsF32<bf16_t, 64, KU> al;
        al.src = a.cusum + (int64_t)l * a.d; al.ld = a.d; al.nrows = 1;
        LoadRowsTC<bf16_t, 64, KU> bl;
        bl.src = a.WdT + (int64_t)l * a.r * a.d; bl.ld = a.d; bl.nrows = a.r;
        EpiChat epi{a.chat + (int64_t)l * a.r};
        gemm_tile<bf16_t, typename SH::TC>(smem, al, bl, epi, 0, a.d, 0, nt * 64, 1, a.r);
        return;
    }
    {
        // mean over the valid tokens of the last cached layer: 8 token groups x 32 column chunks.
        // The tokens of a sample are consecutive rows of one block, so one table lookup gives them all;
        // eight rows are requested per round.
        if (SH::BIG && threadIdx.x >= 256) return;
        int idx = b - a.nb_U - a.nb_Q - a.nb_C;
        const int jt = (a.d + 255) / 256;
        const int s = idx / jt, j0 = (idx % jt) * 256;
        const int t = threadIdx.x, tg = t >> 5, j = j0 + (t & 31) * 8;
        const int m0 = a.samp_start[s], len = a.samp_len[s];
        float acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0.f;
        if (j < a.d) {
            const bf16_t *base = a.cache + a.map.rowoff[m0] + (int64_t)(a.L - 1) * a.map.rowstride[m0] + j;
            for (int t0 = tg; t0 < len; t0 += 8 * 8) {
                u32x4 c[8];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    c[u] = *reinterpret_cast<const u32x4 *>(base + (int64_t)min(t0 + 8 * u, len - 1) * a.d);
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (t0 + 8 * u < len) {
                        Chunk<bf16_t> ch;
                        __builtin_memcpy(&ch, &c[u], 16);
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc[e] += to_f32(ch.e[e]);
                    }
            }
        }
        float *red = reinterpret_cast<float *>(smem); // [8][256]
#pragma unroll
        for (int e = 0; e < 8; ++e) red[tg * 256 + (t & 31) * 8 + e] = acc[e];
        __syncthreads();
        float pv = 0.f; // mean b_L + sum of all c_up, this thread's column
        const bool act = j0 + t < a.d;
        if (act) {
            float tot = 0.f;
#pragma unroll
            for (int q = 0; q < 8; ++q) tot += red[q * 256 + t];
            tot /= (float)len;
            a.pb[(int64_t)s * a.d + j0 + t] = tot;
            pv = tot + a.cusum[(int64_t)a.L * a.d + j0 + t];
        }
        // this block's share of the sample's logits: wavefront sums, then the four wavefronts in order
        const float *Wc = a.params + (int64_t)a.L * a.PL;
        __syncthreads(); // red is reused
        for (int c = 0; c < a.C; ++c) {
            float v = act ? pv * Wc[(int64_t)(j0 + t) * a.C + c] : 0.f;
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
            if ((t & 63) == 0) red[(t >> 6) * kMaxClasses + c] = v;
        }
        __syncthreads();
        if (t < a.C)
            a.zpbp[((int64_t)s * jt + (idx % jt)) * a.C + t] =
                (red[t] + red[kMaxClasses + t]) + (red[2 * kMaxClasses + t] + red[3 * kMaxClasses + t]);
    }
}

// ---------------------------------------------------------------------------
// launches 3 and 4: the r-wide chains over the layers, one 16-token tile per workgroup.
// Wavefront w owns columns [16w, 16w+16) of the r-wide state; earlier layers' tiles stay in LDS.
// ---------------------------------------------------------------------------
struct ChainArgs {
    int L, r, M;
    const int32_t *tile_row0, *tile_rows, *tile_samp;
    const float *params;
    int64_t PL;
    int d;
    const float *U;      // forward: [L][M][r] fp32
    bf16_t *Gp;          // GELU'(pre) as bf16 [L][M][r]: written by the forward chain, read by the backward chain
    const float *chat;   // [L][r]
    const bf16_t *Q;     // forward: QpT ; backward: QpN scaled by (1 - lambda) of the later layer
    bf16_t *Hg;          // forward: H [M][L*r] ; backward: DP [M][L*r]
    float *part;         // forward: HSpart ; backward: cspart   [tiles][L][r]
    // classifier head: the forward chain leaves each tile's share of the logits, the backward chain
    // (or k_glogits when no gradients are wanted) turns them into the loss and dz
    int B, C;
    const float *V;      // [L*r][C]
    float *zpart;        // [tiles][C]  sum_kk (column sums of h over the tile)[kk] V[kk][c]
    const float *zpbp;   // [B][nzb][C] shares of (mean b_L + sum of all c_up) W_cls, from the projection launch
    int nzb;
    const int32_t *samp_tile0, *samp_len, *labels;
    float *logits_ws, *logits_out, *dz, *loss_part;
};

// Logits, loss term and dz of sample s, by a whole workgroup (at least C threads).
// zs, dzs: C floats of LDS each; dzs holds dz of the sample on return.
__device__ __forceinline__ void sample_head(const ChainArgs &a, int s, bool write, float *zs, float *dzs)
{
    const int t = threadIdx.x, C = a.C;
    if (t < C) {
        const int tl0 = a.samp_tile0[s], tl1 = a.samp_tile0[s + 1];
        float z = 0.f;
#pragma unroll 8
        for (int k = tl0; k < tl1; ++k) z += a.zpart[(int64_t)k * C + t];
        const float *c_cls = a.params + (int64_t)a.L * a.PL + (int64_t)a.d * C;
        float zb = 0.f;
        for (int q = 0; q < a.nzb; ++q) zb += a.zpbp[((int64_t)s * a.nzb + q) * C + t];
        zs[t] = z / (float)a.samp_len[s] + zb + c_cls[t];
    }
    __syncthreads();
    if (t == 0) {
        float zmax = -INFINITY;
        for (int c = 0; c < C; ++c) zmax = fmaxf(zmax, zs[c]);
        float se = 0.f;
        for (int c = 0; c < C; ++c) se += expf(zs[c] - zmax);
        const float lse = zmax + logf(se);
        const int y = a.labels[s];
        float lossv = NAN;
        for (int c = 0; c < C; ++c) {
            const float gz = (expf(zs[c] - lse) - (c == y ? 1.f : 0.f)) / (float)a.B;
            dzs[c] = gz;
            if (c == y) lossv = lse - zs[c];
            if (write) {
                a.logits_ws[s * C + c] = zs[c];
                if (a.logits_out) a.logits_out[s * C + c] = zs[c];
                a.dz[s * C + c] = gz;
            }
        }
        if (write) a.loss_part[s] = lossv; // summed in sample order by k_gfinish
    }
    __syncthreads();
}

// forward-only calls: the head without a backward chain, one workgroup per sample
__global__ __launch_bounds__(64) void k_glogits(ChainArgs a)
{
    __shared__ float zs[kMaxClasses], dzs[kMaxClasses];
    sample_head(a, blockIdx.x, true, zs, dzs);
}

// Wavefronts 0..r/16-1 contract and apply the nonlinearity; one more wavefront only moves the
// per-token inputs of later layers from global memory into the ring, so that no contracting
// wavefront ever waits on those loads.

// GELU(u) and GELU'(u) from one exponential: erf by the five-term rational approximation of
// Abramowitz & Stegun 7.1.26 (absolute error below 1.5e-7), whose exp(-x^2) with x = |u|/sqrt(2)
// is the exp(-u^2/2) of the normal density.
__device__ __forceinline__ void gelu_pair(float u, float &h, float &gp)
{
    const float x = fabsf(u) * 0.70710678118654752f;
    const float t = __builtin_amdgcn_rcpf(1.f + 0.3275911f * x);
    const float ex = __expf(-0.5f * u * u);
    const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
    const float erf_abs = 1.f - poly * ex;
    const float Phi = 0.5f * (1.f + copysignf(erf_abs, u));
    h = u * Phi;
    gp = Phi + u * 0.3989422804014327f * ex;
}

// The chain runs in L steps; step s produces layer s (forward) or L-1-s (backward) and contracts the
// tiles of steps 0..s-1, oldest first, so that the tile finished last is also needed last.
// CMAX: classes the helper wavefront keeps accumulators and prefetched rows of V for (a.C <= CMAX); 4 where that
// holds, because with 16 the widest forward instantiation no longer fitted its registers (194 spilled)
template <bool FWD, int NT, int CMAX = kMaxClasses> __global__ __launch_bounds__(64 * (2 * NT + 1)) void k_gchain(ChainArgs a)
{
    extern __shared__ __attribute__((aligned(16))) char dyn_smem[];
    constexpr int r = 32 * NT, RP = r + kChainPad, KS = NT, NW = 2 * NT, T = kChainRows;
    using RingT = typename std::conditional<FWD, float, bf16_t>::type;
    constexpr int kTileBytes = T * r * (int)sizeof(RingT);
    constexpr int kChunksPerLane = kTileBytes / 16 / 64; // 16-byte chunks each helper lane moves per layer
    constexpr int kGChunks = (T * r * 2 / 16 + 63) / 64; // same for a GELU' tile (bf16), rounded up
    static_assert(kTileBytes % (16 * 64) == 0, "ring tile must split evenly over the helper wavefront");
    const int L = a.L;
    bf16_t *Hs = reinterpret_cast<bf16_t *>(dyn_smem);                              // [L][T][RP]
    RingT *ring = reinterpret_cast<RingT *>(Hs + (size_t)L * T * RP);               // [kRing][T][r]
    bf16_t *Gst = reinterpret_cast<bf16_t *>(ring + (size_t)kRing * T * r);         // [2][T][r] (forward)
    float *vecS = reinterpret_cast<float *>(Gst + (FWD ? (size_t)2 * T * r : 0));   // [L][r]
    float *Cs = vecS + (size_t)L * r;                                               // [L][r]
    float *lamS = Cs + (size_t)L * r;                                               // [L]
    float *zs = lamS + (L + 3) / 4 * 4, *dzs = zs + kMaxClasses;                    // [kMaxClasses] each
    const int tile = blockIdx.x;
    const int m0 = a.tile_row0[tile], nrows = a.tile_rows[tile], samp = a.tile_samp[tile];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t Lr = (int64_t)L * r;
    constexpr int64_t rr = (int64_t)r * r;
    constexpr int nthreads = 64 * (NW + 1);
    auto layer_at = [&](int step) { return FWD ? step : L - 1 - step; };

    // Requests that depend on nothing computed here go out first and are in flight while the
    // per-layer vectors are set up: the helper wavefront's tiles of the first three steps, and the
    // contracting wavefronts' operands of the first pairs.
    const RingT *src = FWD ? reinterpret_cast<const RingT *>(a.U) : reinterpret_cast<const RingT *>(a.Gp);
    constexpr int EPC = 16 / (int)sizeof(RingT); // elements per chunk
    auto fetch = [&](int step, u32x4(&reg)[kChunksPerLane]) {
        if (step >= L) return;
        const RingT *base = src + ((int64_t)layer_at(step) * a.M + m0) * r;
#pragma unroll
        for (int q = 0; q < kChunksPerLane; ++q) {
            // rows past the end of a short tile re-read the tile's last chunk (never used: the
            // contracting wavefronts mask those rows); no branch, no register is zeroed
            const int e = min((lane + 64 * q) * EPC, nrows * r - EPC);
            reg[q] = *reinterpret_cast<const u32x4 *>(base + e);
        }
    };
    auto put = [&](int step, const u32x4(&reg)[kChunksPerLane]) {
        if (step >= L) return;
        RingT *dst = ring + (size_t)(step % kRing) * T * r;
#pragma unroll
        for (int q = 0; q < kChunksPerLane; ++q) *reinterpret_cast<u32x4 *>(dst + (lane + 64 * q) * EPC) = reg[q];
    };
    // Tiles of a finished step, LDS -> global.  Backward: the dpre tile (the helper has nothing else to do there;
    // forward, where it also prepares vectors and logits, the same made its step longer than the contracting
    // wavefronts' and the h tiles go out together at the end instead).  Forward: the GELU' tile.
    auto drain = [&](int step) {
        if (step < 0 || step >= L) return;
        if (!FWD) {
            const int l = layer_at(step);
            constexpr int cpr = r / 8, nch = T * cpr; // 16-byte chunks per row, per tile
#pragma unroll
            for (int q = 0; q < (nch + 63) / 64; ++q) {
                const int c = lane + 64 * q, row = c / cpr, cc = c % cpr;
                if (c < nch && row < nrows)
                    *reinterpret_cast<u32x4 *>(a.Hg + (int64_t)(m0 + row) * Lr + (int64_t)l * r + cc * 8) =
                        *reinterpret_cast<const u32x4 *>(Hs + ((int64_t)l * T + row) * RP + cc * 8);
            }
        }
        if (!FWD) return;
        const bf16_t *st = Gst + (size_t)(step & 1) * T * r;
        bf16_t *dst = a.Gp + ((int64_t)layer_at(step) * a.M + m0) * r;
#pragma unroll
        for (int q = 0; q < kGChunks; ++q) {
            const int e = (lane + 64 * q) * 8;
            if (e < nrows * r) *reinterpret_cast<u32x4 *>(dst + e) = *reinterpret_cast<const u32x4 *>(st + e);
        }
    };
    constexpr int kDepth = NT == 1 ? 16 : NT == 2 ? 12 : NT == 3 ? 10 : 6; // bounded by the register file
    const int i = lane & 15, g = lane >> 4;
    const int n = 16 * wave + i;
    const int total_pairs = L * (L - 1) / 2;
    // next pair to request.  A request is issued for every FIFO slot on every path (once the
    // sequence is exhausted the last pair is requested again and never used): the compiler can
    // then count the loads in flight and wait only for the oldest ones.
    int is = 1, ij = 0;
    auto issue = [&](bf16x8(&bq)[KS]) {
        const int s = is < L ? is : L - 1;
        const int j = is < L ? ij : L - 2;
        const int ls = layer_at(s), lj = layer_at(j);
        const int pi = FWD ? pair_index(lj, ls) : pair_index(ls, lj);
        const bf16_t *Qp = a.Q + pi * rr + (int64_t)wave * KS * 512;
#pragma unroll
        for (int q = 0; q < KS; ++q) bq[q] = *reinterpret_cast<const bf16x8 *>(Qp + (q * 64 + lane) * 8);
        if (is < L && ++ij >= is) {
            ++is;
            ij = 0;
        }
    };
    // per-layer vectors.  Forward: the first step's here, the later ones by the helper wavefront, one
    // step ahead.  Backward: all of them here (leaving them to the helper was measured slower).
    // Called by both kinds of wavefront from inside their own branch, after their first requests have gone out:
    // written once before the branch, the helper's tile registers and the contracting wavefronts' operand FIFO
    // were both live across it, and the widest forward instantiation spilled 194 registers.
    auto per_layer_vectors = [&]() {
        if (!FWD) sample_head(a, samp, tile == a.samp_tile0[samp], zs, dzs);
        const float inv_len = 1.f / (float)a.samp_len[samp];
        for (int l = threadIdx.x; l < L; l += nthreads) lamS[l] = a.params[(int64_t)l * a.PL + a.PL - 1];
        if (FWD) {
            for (int nn = threadIdx.x; nn < r; nn += nthreads) {
                const float *pl = a.params;
                vecS[nn] = (1.f - pl[a.PL - 1]) * a.chat[nn] + pl[(int64_t)a.d * r + nn];
            }
        } else {
            for (int c = threadIdx.x; c < L * r; c += nthreads) {
                // ghat = dz V^T / len: what the head hands to every token of the sample
                float v = 0.f;
                for (int q = 0; q < a.C; ++q) v += dzs[q] * a.V[(int64_t)c * a.C + q];
                vecS[c] = v * inv_len;
            }
        }
    };

    if (wave == NW) {
        // The helper's few requests per step share the compute unit's memory pipeline with the contracting
        // wavefronts' operand stream; at equal priority it got one issue slot in nine and its tiles arrived late.
        __builtin_amdgcn_s_setprio(3);
        // Two tiles in registers (even steps in ra, odd in rb): the tile of step s+3 is requested into the registers
        // the tile of step s+1 has just left, and is needed one whole step later.  (A third set of registers bought
        // no more time than that and made the widest forward instantiation spill a tile in every step: the spill's
        // store waited for the request it had just issued, 4.8 us per step of the Large-shaped chain.)
        u32x4 ra[kChunksPerLane], rb[kChunksPerLane];
        fetch(0, ra);
        fetch(1, rb);
        per_layer_vectors();
        // ---- helper wavefront: all global traffic of the per-token tiles.  It requests the input tiles
        // three layers ahead and (forward) writes out the GELU' tile of the layer just finished,
        // so the contracting wavefronts issue no global store and wait on no per-token load.
        // Forward, the helper also prepares, one step ahead, what does not depend on the chain: the next
        // step's per-layer vector (vecS), and it folds the finished layers' column sums into this tile's
        // share of the logits.  Every value it uses was requested one step earlier, before that step's
        // tile request, so waiting for it never waits for a tile.
        constexpr int NP = (r + 63) / 64; // passes of the 64 lanes over the r columns
        float vpre[NP][CMAX];      // V rows of the layer finished last
        float cpre[NP][2];                // chat and c_down of the next step's layer
        float zacc[CMAX];
#pragma unroll
        for (int c = 0; c < CMAX; ++c) zacc[c] = 0.f;
        const int C = a.C;
        auto side_load = [&](int s) { // requests for what side_use(s + 1) needs
            if (!FWD) return;
            const int lv = min(max(s, 0), L - 1); // V rows of the layer of step s
            const int lc = min(s + 2, L - 1);     // chat, c_down of the layer of step s+2
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                const int nn = min(lane + 64 * p, r - 1);
#pragma unroll
                for (int c = 0; c < CMAX; ++c)
                    if (c < C) vpre[p][c] = a.V[((int64_t)lv * r + nn) * C + c];
                cpre[p][0] = a.chat[lc * r + nn];
                cpre[p][1] = a.params[(int64_t)lc * a.PL + (int64_t)a.d * r + nn];
            }
        };
        auto side_use = [&](int s) { // during step s
            if (!FWD) return;
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                const int nn = lane + 64 * p;
                if (nn >= r) continue;
                if (s + 1 < L) vecS[(s + 1) * r + nn] = (1.f - lamS[s + 1]) * cpre[p][0] + cpre[p][1];
                if (s >= 1) { // layer s-1 is finished: its column sums are final
                    const float hs = Cs[(s - 1) * r + nn];
#pragma unroll
                    for (int c = 0; c < CMAX; ++c)
                        if (c < C) zacc[c] += hs * vpre[p][c];
                }
            }
        };
        side_load(-1);
        put(0, ra);
        fetch(2, ra);
        __syncthreads();
        // before the barrier that ends step s the tile of step s+1 must be in the ring
        for (int s = 0; s < L; s += 2) {
            // the tile consumed here was requested a step ago; the new request goes out last, so that waiting
            // for anything older never means waiting for it
            put(s + 1, rb);
            side_use(s);
            drain(s - 1);
            side_load(s);
            fetch(s + 3, rb);
            __syncthreads();
            if (s + 1 < L) {
                put(s + 2, ra);
                side_use(s + 1);
                drain(s);
                side_load(s + 1);
                fetch(s + 4, ra);
                __syncthreads();
            }
        }
        drain(L - 1);
        if (FWD) {
            side_use(L); // the last layer's column sums
#pragma unroll
            for (int c = 0; c < CMAX; ++c)
                if (c < C) {
                    float v = zacc[c];
#pragma unroll
                    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
                    if (lane == 0) a.zpart[(int64_t)tile * C + c] = v;
                }
        }
    } else {
        // ---- contracting wavefronts ----
        bf16x8 fifo[kDepth][KS];
        if (total_pairs > 0) {
#pragma unroll
            for (int slot = 0; slot < kDepth; ++slot) issue(fifo[slot]);
        }
        per_layer_vectors();
        // two accumulators so that consecutive matrix instructions do not depend on each other
        f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
        auto contract = [&](const bf16x8(&bq)[KS], int j) {
            const bf16_t *Hk = Hs + ((int64_t)layer_at(j) * T + i) * RP;
            bf16x8 av[KS];
#pragma unroll
            for (int q = 0; q < KS; ++q) av[q] = *reinterpret_cast<const bf16x8 *>(Hk + 32 * q + 8 * g);
#pragma unroll
            for (int q = 0; q < KS; ++q) {
                if (q & 1) acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[q], bq[q], acc1, 0, 0, 0);
                else acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[q], bq[q], acc0, 0, 0, 0);
            }
        };
        auto finish_layer = [&](int step) { // nonlinearity, tiles to LDS, barrier
            const int l = layer_at(step);
            const float lam = lamS[l];
            const float cvec = vecS[l * r + n];
            const RingT *rt = ring + (size_t)(step % kRing) * T * r;
            bf16_t *gst = Gst + (size_t)(step & 1) * T * r;
            float colsum = 0.f;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = 4 * g + v;
                const bool valid = row < nrows;
                const float uin = to_f32(rt[row * r + n]);
                const float accv = acc0[v] + acc1[v];
                float out = 0.f;
                if (FWD) {
                    const float pre = lam * uin + (1.f - lam) * accv + cvec;
                    float h, gp;
                    gelu_pair(pre, h, gp);
                    if (valid) out = h;
                    gst[row * r + n] = static_cast<bf16_t>(gp);
                } else {
                    if (valid) out = (cvec + accv) * uin;
                }
                Hs[((int64_t)l * T + row) * RP + n] = static_cast<bf16_t>(out);
                colsum += out;
                acc0[v] = 0.f;
                acc1[v] = 0.f;
            }
            colsum += __shfl_xor(colsum, 16, 64);
            colsum += __shfl_xor(colsum, 32, 64);
            if (g == 0) Cs[l * r + n] = colsum;
            __syncthreads();
        };
        __syncthreads();
        finish_layer(0); // the first step has nothing to contract
        int cs = 1, cj = 0; // pair being contracted
        for (int p0 = 0; p0 < total_pairs; p0 += kDepth) {
#pragma unroll
            for (int slot = 0; slot < kDepth; ++slot) {
                if (p0 + slot < total_pairs) {
                    contract(fifo[slot], cj);
                    if (++cj >= cs) {
                        finish_layer(cs++);
                        cj = 0;
                    }
                }
                issue(fifo[slot]);
            }
        }
    }
    __syncthreads(); // every layer's tile and column sums are in LDS
    if (FWD) {
        // flush: 16-byte chunks of the valid rows (backward the tiles went out layer by layer)
        constexpr int chunks_per_row = r / 8;
        for (int c = threadIdx.x; c < L * T * chunks_per_row; c += nthreads) {
            const int l = c / (T * chunks_per_row);
            const int rem = c - l * T * chunks_per_row;
            const int row = rem / chunks_per_row, cc = rem % chunks_per_row;
            if (row < nrows)
                *reinterpret_cast<u32x4 *>(a.Hg + (int64_t)(m0 + row) * Lr + (int64_t)l * r + cc * 8) =
                    *reinterpret_cast<const u32x4 *>(Hs + ((int64_t)l * T + row) * RP + cc * 8);
        }
    }
    for (int c = threadIdx.x; c < L * r; c += nthreads) a.part[(int64_t)tile * Lr + c] = Cs[c];
}

// ---------------------------------------------------------------------------
// The chains as contractions launched layer by layer (adapter widths whose 16-token history of all
// layers does not fit the LDS).  Layer l of the forward chain needs sum_{k<l} h_k Q_{kl}: with H [M][L*r]
// and the matrix QT [(l,n)][(k,j)] = Q_{kl}[j][n] that is the product of the first l*r columns of H with
// rows (l, .) of QT, both K-contiguous; the backward chain takes columns (l+1)*r.. of DP and rows (l, .)
// of QN [(l,n)][(k,j)] = (1-lambda_k) Q_{lk}[n][j].
//
// The layers are taken in groups of g.  What the layers before a group contribute to all g layers of
// the group is one wide contraction (K = all earlier layers, N = g*r: enough 128 x 128 tiles to fill
// the chip without splitting K).  Inside the group each layer contracts over the group's earlier layers
// and then adds the wide contraction's result and applies the nonlinearity, so that no partial sums
// travel through memory more than once: up to r = 256 one launch walks all layers of the group per
// 16-token tile (k_gseq_group), above that each layer is a short tiled contraction of its own
// (k_gseq_layer).  The per-tile column sums the later launches need are taken from the finished bf16
// arrays in one pass per direction.
// ---------------------------------------------------------------------------
struct SeqBigArgs {
    const bf16_t *A;  // H or DP [M][L*r]
    const bf16_t *Bq; // QT or QN [L*r][L*r]
    float *P;         // [M][ldp]
    int L, r, M, ldp;
    int brow0, ncols;  // rows (group's first layer) * r .. + ncols of Bq
    int kbegin, kend;  // columns of A contracted
    int ctiles;
};

template <int BK> struct SeqShapes {
    using TB = NtTile<2, 2, 2, 2, BK, 3>; // kSeqTile x kSeqTile, three stages, interleaved sub-steps: there is one such workgroup per compute unit
    using TS = NtTile<2, 2, 1, 1, BK, 3>; // 64 x 64 for the short contractions inside a group
    static_assert(TB::BM == kSeqTile && TB::BN == kSeqTile, "tile side of the wide chain contraction");
};

template <int BK> __global__ __launch_bounds__(256) void k_gseq_big(SeqBigArgs a)
{
    using TL = typename SeqShapes<BK>::TB;
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    // a die's range of tiles: whole rows of column tiles, so that a row tile of A is fetched by one die only
    const int v = die_chunk_order(blockIdx.x, gridDim.x);
    const int ct = v % a.ctiles, rt = v / a.ctiles;
    const int64_t Lr = (int64_t)a.L * a.r;
    const bf16_t *A = a.A, *Bq = a.Bq + (int64_t)a.brow0 * Lr;
    auto arow = [&](int m) { return A + (int64_t)m * Lr; };
    auto brow = [&](int n) { return Bq + (int64_t)n * Lr; };
    EpiStoreF32 epi{a.P, a.ldp};
    gemm_nt<TL, true>(smem, arow, brow, epi, a.kbegin, a.kend, rt * kSeqTile, ct * kSeqTile, a.M, a.ncols);
}

struct SeqLayerArgs {
    const bf16_t *A;  // H or DP [M][L*r]
    const bf16_t *Bq; // QT or QN [L*r][L*r]
    const float *P;   // [M][ldp]: the wide contraction's result for this group, or null
    int ldp, pcol0;
    int l, L, r, M, d;
    int kbegin, kend; // columns of A contracted (inside the group)
    int ctiles;
    const float *U;     // forward: [L][M][r]
    bf16_t *Gp;         // [L][M][r]: written forward, read backward
    const float *chat;  // [L][r]
    const float *params;
    int64_t PL;
    bf16_t *Hg;         // forward: H, backward: DP   [M][L*r]
    const float *ghat;  // backward: [B][L*r]
    const int32_t *rowsamp;
};

// epilogue of a layer's contraction: the rest of the layer
template <bool FWD> struct EpiSeqLayer {
    static constexpr bool kBatched = true;
    const float *P;
    int ldp, pcol0;
    const float *U_l;
    bf16_t *Gp_l;
    bf16_t *Hg_l; // column l*r of row 0
    int64_t Lr;
    int r;
    float lam;
    const float *chat_l, *cd_l; // forward
    const float *ghat_l;        // backward: column l*r of sample 0
    const int32_t *rowsamp;
    __device__ void batch(int row_base, int col, const f32x16 &acc, int nrows, int ncols) const
    {
        const int cc = min(col, ncols - 1);
        float x[16], pb[16], gh[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int m = min(epi_row(row_base, v), nrows - 1);
            x[v] = FWD ? U_l[(int64_t)m * r + cc] : to_f32(Gp_l[(int64_t)m * r + cc]);
            pb[v] = P ? P[(int64_t)m * ldp + pcol0 + cc] : 0.f;
            gh[v] = FWD ? 0.f : ghat_l[(int64_t)rowsamp[m] * Lr + cc];
        }
        const float cvec = FWD ? (1.f - lam) * chat_l[cc] + cd_l[cc] : 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int m = epi_row(row_base, v);
            if (m < nrows && col < ncols) {
                float out;
                if (FWD) {
                    const float pre = lam * x[v] + (1.f - lam) * (acc[v] + pb[v]) + cvec;
                    float h, gp;
                    gelu_pair(pre, h, gp);
                    out = h;
                    Gp_l[(int64_t)m * r + col] = static_cast<bf16_t>(gp);
                } else {
                    out = (gh[v] + acc[v] + pb[v]) * x[v];
                }
                Hg_l[(int64_t)m * Lr + col] = static_cast<bf16_t>(out);
            }
        }
    }
};

template <bool FWD, int BK> __global__ __launch_bounds__(256) void k_gseq_layer(SeqLayerArgs a)
{
    using TL = typename SeqShapes<BK>::TS;
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int ct = blockIdx.x % a.ctiles, rt = blockIdx.x / a.ctiles;
    const int l = a.l, r = a.r;
    const int64_t Lr = (int64_t)a.L * r, Mr = (int64_t)a.M * r;
    const bf16_t *A = a.A, *Bq = a.Bq + (int64_t)l * r * Lr;
    auto arow = [&](int m) { return A + (int64_t)m * Lr; };
    auto brow = [&](int n) { return Bq + (int64_t)n * Lr; };
    const float *pl = a.params + (int64_t)l * a.PL;
    EpiSeqLayer<FWD> epi{a.P, a.ldp, a.pcol0, FWD ? a.U + (int64_t)l * Mr : nullptr, a.Gp + (int64_t)l * Mr,
                         a.Hg + (int64_t)l * r, Lr, r, pl[a.PL - 1], a.chat + (int64_t)l * r, pl + (int64_t)a.d * r,
                         FWD ? nullptr : a.ghat + (int64_t)l * r, a.rowsamp};
    gemm_nt<TL>(smem, arow, brow, epi, a.kbegin, a.kend, rt * TL::BM, ct * TL::BN, a.M, r);
}

// All layers of a group in one launch.  The chain is a recurrence per token, so a workgroup that owns 16 token rows
// can walk the group's layers by itself: h (or dpre) of the group's finished layers stays in LDS as the operand of
// the later ones, and the r x r operands stream from fragment-major copies of the group's pairs through a register
// FIFO that runs ahead across layer boundaries (they depend on nothing computed here).
//
// Contracting wavefronts (one per 32 columns of r) issue nothing but those operand requests: on this target loads
// and stores complete in order per wavefront, so a per-token load or a store between two operand requests would
// make every later operand wait for it.  Four helper wavefronts (four token rows each) do all per-token global
// traffic instead: they request the next layer's inputs one step ahead, fold them into the one tile the epilogue
// needs (forward t = lambda U + (1-lambda)(P + chat) + c_down; backward t = ghat + P and GELU'), put that into an
// LDS ring, and write the finished layer's tiles out while the next layer is contracted.
//
// The matrix instructions take the r x r fragment as their first operand and the token fragment as the second:
// lane (i, g4) then holds columns n0 + 16 cb + 4 g4 .. + 3 of token row i, four consecutive values per access.
struct SeqGroupArgs {
    SeqLayerArgs la;  // l, Bq, kbegin, kend, ctiles, pcol0 unused
    int l0, l1;       // the group's layers
    const bf16_t *Qg; // the group's pairs, fragment-major: block q (q - 1) / 2 + j for step q's operand of step j
};
constexpr int kGroupHelpers = 4;
constexpr int kGroupDepth = 8;   // K blocks of operands requested ahead per contracting wavefront
constexpr int kGroupMaxR = 256;  // eight contracting wavefronts
// LDS of the group kernel (T = kChainRows):
//   Hs   [layers][T][r + 8] bf16   h or dpre of the group's layers
//   ring [2][T][r + 4] fp32        the epilogue's per-token input t
//   xst  [2][T][r + 8] bf16        GELU': the backward chain's input, the forward chain's output on its way out
//   vecS [layers][r] fp32, lamS [layers] fp32
static size_t group_lds(int layers, int r)
{
    return (size_t)layers * kChainRows * (r + kChainPad) * 2 + (size_t)2 * kChainRows * (r + 4) * 4 +
           (size_t)2 * kChainRows * (r + kChainPad) * 2 + (size_t)layers * r * 4 + (size_t)((layers + 3) / 4 * 4) * 4;
}

template <bool FWD> __global__ __launch_bounds__(64 * (kGroupMaxR / 32 + kGroupHelpers)) void k_gseq_group(SeqGroupArgs ga)
{
    extern __shared__ __attribute__((aligned(16))) char dyn_smem[];
    const SeqLayerArgs &a = ga.la;
    constexpr int T = kChainRows, D = kGroupDepth;
    const int r = a.r, RP = r + kChainPad, RF = r + 4, KB = r >> 5, NWV = r >> 5, M = a.M;
    const int gl = ga.l1 - ga.l0;
    bf16_t *Hs = reinterpret_cast<bf16_t *>(dyn_smem);
    float *ring = reinterpret_cast<float *>(Hs + (size_t)gl * T * RP);
    bf16_t *xst = reinterpret_cast<bf16_t *>(ring + (size_t)2 * T * RF);
    float *vecS = reinterpret_cast<float *>(xst + (size_t)2 * T * RP);
    float *lamS = vecS + (size_t)gl * r;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m0 = blockIdx.x * T;
    const int64_t Lr = (int64_t)a.L * r, Mr = (int64_t)M * r;
    const int nthreads = 64 * (NWV + kGroupHelpers);
    auto layer_at = [&](int q) { return FWD ? ga.l0 + q : ga.l1 - 1 - q; };
    auto per_layer_vectors = [&]() {
        for (int c = threadIdx.x; c < gl * r; c += nthreads) {
            const int q = c / r, n = c - q * r, l = layer_at(q);
            const float *pl = a.params + (int64_t)l * a.PL;
            vecS[c] = FWD ? (1.f - pl[a.PL - 1]) * a.chat[(int64_t)l * r + n] + pl[(int64_t)a.d * r + n] : 0.f;
            if (n == 0) lamS[q] = pl[a.PL - 1];
        }
    };

    if (wave >= NWV) {
        // ---- helper wavefronts: rows 4 h .. 4 h + 3 of the tile ----
        __builtin_amdgcn_s_setprio(3);
        const int h = wave - NWV;
        const int cpr = r >> 2, nc = 4 * cpr; // 4-column chunks per row, chunks of this wavefront's four rows (<= 256)
        // element offsets of this lane's chunks in a layer of U / Gp, in P, in ghat (all below 2^31: at most 65536 token
        // rows of at most 1024 columns), and their row and column in the tile.  Chunks past the end repeat the last one.
        int off_u[4], off_p[4], off_g[4], trow[4], tcol[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = min(lane + 64 * u, nc - 1);
            const int row = 4 * h + c / cpr, col = 4 * (c % cpr);
            const int m = min(m0 + row, M - 1);
            off_u[u] = m * r + col;
            off_p[u] = m * a.ldp + col;
            off_g[u] = FWD ? 0 : a.rowsamp[m] * (int)Lr + col;
            trow[u] = row;
            tcol[u] = col;
        }
        // two tiles in registers (even steps in set 0, odd steps in set 1), each requested two steps before it is needed
        struct Regs {
            f32x4 ru[4], rp[4];
            bf16x4 rx[4];
        };
        Regs ra, rb;
        auto fetch = [&](int s, Regs &g) {
            if (s >= gl) return;
            const int l = layer_at(s);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (FWD) {
                    g.ru[u] = *reinterpret_cast<const f32x4 *>(a.U + (int64_t)l * Mr + off_u[u]);
                } else {
                    g.ru[u] = *reinterpret_cast<const f32x4 *>(a.ghat + (int64_t)l * r + off_g[u]);
                    g.rx[u] = *reinterpret_cast<const bf16x4 *>(a.Gp + (int64_t)l * Mr + off_u[u]);
                }
                g.rp[u] = a.P ? *reinterpret_cast<const f32x4 *>(a.P + (int64_t)(l - ga.l0) * r + off_p[u])
                              : f32x4{0.f, 0.f, 0.f, 0.f};
            }
        };
        auto put = [&](int s, const Regs &g) {
            if (s >= gl) return;
            float *rt = ring + (size_t)(s & 1) * T * RF;
            bf16_t *xt = xst + (size_t)(s & 1) * T * RP;
            const float lam = lamS[s];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                f32x4 t;
                if (FWD) {
                    const f32x4 cv = *reinterpret_cast<const f32x4 *>(vecS + s * r + tcol[u]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) t[e] = lam * g.ru[u][e] + (1.f - lam) * g.rp[u][e] + cv[e];
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) t[e] = g.ru[u][e] + g.rp[u][e];
                    *reinterpret_cast<bf16x4 *>(xt + trow[u] * RP + tcol[u]) = g.rx[u];
                }
                *reinterpret_cast<f32x4 *>(rt + trow[u] * RF + tcol[u]) = t;
            }
        };
        // tiles of a finished step, LDS -> global: h or dpre, and (forward) GELU'
        auto drain = [&](int s) {
            if (s < 0 || s >= gl) return;
            const int l = layer_at(s);
            const int cp8 = r >> 3; // 16-byte chunks per row
            const bf16_t *hq = Hs + (size_t)s * T * RP, *xq = xst + (size_t)(s & 1) * T * RP;
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int c = lane + 64 * u;
                const int row = 4 * h + c / cp8, cc = c % cp8, m = m0 + row;
                if (c < 4 * cp8 && m < M) {
                    *reinterpret_cast<u32x4 *>(a.Hg + (int64_t)m * Lr + (int64_t)l * r + cc * 8) =
                        *reinterpret_cast<const u32x4 *>(hq + row * RP + cc * 8);
                    if (FWD)
                        *reinterpret_cast<u32x4 *>(a.Gp + (int64_t)l * Mr + (int64_t)m * r + cc * 8) =
                            *reinterpret_cast<const u32x4 *>(xq + row * RP + cc * 8);
                }
            }
        };
        fetch(0, ra);
        fetch(1, rb);
        per_layer_vectors();
        __syncthreads(); // vectors
        put(0, ra);
        fetch(2, ra);
        __syncthreads(); // the first step's tile is in the ring
        for (int s = 0; s < gl; s += 2) {
            // during step s: the tile of step s+1 (requested two steps ago) goes into the ring slot step s-1 has left,
            // the tiles step s-1 produced go out, and the inputs of step s+3 are requested into the registers just freed
            put(s + 1, rb);
            drain(s - 1);
            fetch(s + 3, rb);
            __syncthreads();
            if (s + 1 < gl) {
                put(s + 2, ra);
                drain(s);
                fetch(s + 4, ra);
                __syncthreads();
            }
        }
        drain(gl - 1);
        return;
    }

    // ---- contracting wavefronts ----
    const int i = lane & 15, g4 = lane >> 4;
    const int n0 = 32 * wave;
    const int64_t rr = (int64_t)r * r;
    const bf16_t *Bl = ga.Qg + ((int64_t)2 * wave * KB * 64 + lane) * 8; // this lane's 16 bytes of a fragment
    const int total = gl * (gl - 1) / 2 * KB;
    // next request: (layer step, earlier step, K block).  Every FIFO slot is requested on every path; past the end
    // the last block is requested again and never used.
    int iq = 1, ik = 0, ib = 0;
    auto issue = [&](bf16x8(&bq)[2]) {
        const bool live = iq < gl;
        const int q = live ? iq : gl - 1, k = live ? ik : gl - 2, b = live ? ib : KB - 1;
        const bf16_t *p = Bl + (q * (q - 1) / 2 + k) * rr + b * 512;
        bq[0] = *reinterpret_cast<const bf16x8 *>(p);
        bq[1] = *reinterpret_cast<const bf16x8 *>(p + KB * 512);
        if (live && ++ib >= KB) {
            ib = 0;
            if (++ik >= iq) {
                ik = 0;
                ++iq;
            }
        }
    };
    bf16x8 fifo[D][2];
    if (total > 0) {
#pragma unroll
        for (int slot = 0; slot < D; ++slot) issue(fifo[slot]);
    }
    per_layer_vectors();
    const bool live_row = m0 + i < M;
    f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
    auto contract = [&](const bf16x8(&bq)[2], int k, int b) {
        const bf16x8 av = *reinterpret_cast<const bf16x8 *>(Hs + ((size_t)k * T + i) * RP + 32 * b + 8 * g4);
        acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bq[0], av, acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bq[1], av, acc[1], 0, 0, 0);
    };
    auto finish_layer = [&](int q) { // the rest of the layer, its tiles to LDS, barrier
        const float lam = lamS[q];
        const float *rt = ring + ((size_t)(q & 1) * T + i) * RF;
        bf16_t *xt = xst + ((size_t)(q & 1) * T + i) * RP;
        bf16_t *Hq = Hs + ((size_t)q * T + i) * RP;
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            const int col = n0 + 16 * cb + 4 * g4;
            const f32x4 t = *reinterpret_cast<const f32x4 *>(rt + col);
            bf16x4 o, gq;
            if (!FWD) gq = *reinterpret_cast<const bf16x4 *>(xt + col);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float out;
                if (FWD) {
                    float gp;
                    gelu_pair(t[v] + (1.f - lam) * acc[cb][v], out, gp);
                    gq[v] = static_cast<bf16_t>(gp);
                } else {
                    out = (t[v] + acc[cb][v]) * to_f32(gq[v]);
                }
                o[v] = static_cast<bf16_t>(live_row ? out : 0.f);
                acc[cb][v] = 0.f;
            }
            *reinterpret_cast<bf16x4 *>(Hq + col) = o;
            if (FWD) *reinterpret_cast<bf16x4 *>(xt + col) = gq;
        }
        __syncthreads();
    };
    __syncthreads(); // vectors
    __syncthreads(); // the first step's tile is in the ring
    finish_layer(0); // the group's first layer has nothing to contract inside the group
    int cq = 1, ck = 0, cb_ = 0; // block being contracted
    for (int p0 = 0; p0 < total; p0 += D) {
#pragma unroll
        for (int slot = 0; slot < D; ++slot) {
            if (p0 + slot < total) {
                contract(fifo[slot], ck, cb_);
                if (++cb_ >= KB) {
                    cb_ = 0;
                    if (++ck >= cq) {
                        finish_layer(cq++);
                        ck = 0;
                    }
                }
            }
            issue(fifo[slot]);
        }
    }
}

// part[tile][kk] = sum over the tile's valid rows of X[row][kk]   (X = H or DP, bf16 [M][L*r])
__global__ __launch_bounds__(256) void k_gseq_colsum(const bf16_t *X, int Lr, const int32_t *tile_row0,
                                                     const int32_t *tile_rows, float *part)
{
    const int tile = blockIdx.x, kk = blockIdx.y * 256 + threadIdx.x;
    if (kk >= Lr) return;
    const int m0 = tile_row0[tile], nrows = tile_rows[tile];
    float x[kChainRows];
#pragma unroll
    for (int row = 0; row < kChainRows; ++row) x[row] = to_f32(X[(int64_t)(m0 + min(row, nrows - 1)) * Lr + kk]);
    float acc = 0.f;
#pragma unroll
    for (int row = 0; row < kChainRows; ++row)
        if (row < nrows) acc += x[row];
    part[(int64_t)tile * Lr + kk] = acc;
}

// ghat[s][kk] = (dz_s V[kk]^T) / len_s: what the head hands to every token of sample s
__global__ __launch_bounds__(256) void k_gseq_ghat(const float *dz, const float *V, const int32_t *samp_len, int Lr, int C,
                                                   float *ghat)
{
    const int s = blockIdx.y, kk = blockIdx.x * 256 + threadIdx.x;
    if (kk >= Lr) return;
    float v = 0.f;
    for (int c = 0; c < C; ++c) v += dz[s * C + c] * V[(int64_t)kk * C + c];
    ghat[(int64_t)s * Lr + kk] = v / (float)samp_len[s];
}

// zpart[tile][c] = sum_kk (column sums of h over the tile)[kk] V[kk][c]
__global__ __launch_bounds__(256) void k_gseq_zpart(const float *HSpart, const float *V, int Lr, int C, float *zpart)
{
    __shared__ float red[16];
    const int tile = blockIdx.x, t = threadIdx.x;
    float acc[kMaxClasses];
#pragma unroll
    for (int c = 0; c < kMaxClasses; ++c) acc[c] = 0.f;
    for (int kk = t; kk < Lr; kk += 256) {
        const float hs = HSpart[(int64_t)tile * Lr + kk];
#pragma unroll
        for (int c = 0; c < kMaxClasses; ++c)
            if (c < C) acc[c] += hs * V[(int64_t)kk * C + c];
    }
    for (int c = 0; c < C; ++c) {
        const float tot = block_sum(acc[c], red);
        if (t == 0) zpart[(int64_t)tile * C + c] = tot;
    }
}

// ---------------------------------------------------------------------------
// launch 5: contractions over the tokens.  E_l = b_l^T dpre_l ; GG = H^T DP (all layer pairs at
// once, kept only as the two bf16 copies the last launch contracts) ; ordered sums of the tiles'
// column sums
// ---------------------------------------------------------------------------
struct TokRedArgs {
    int blk_off; // first block of this launch (parts may be launched separately for timing)
    const bf16_t *cache;
    RowMap map;
    int L, d, r;
    int nb_E, nb_G, e_tiles, se, sg, tiles_per_se, rows_per_sg, tg, tgn, reverse; // tg x tgn tiles of the Gram matrix
    const int32_t *tile_row0, *tile_rows;
    const void *zeros; // at least 16 zero bytes
    const bf16_t *H, *DP; // [M][L*r]
    float *Epart;         // [se][L][d][r]
    const float *params;
    int64_t PL;
    float *GGpart;        // [sg][L*r][L*r]
    bf16_t *GGT, *GGsc;   // written directly where sg == 1 (gg_direct)
    int gg_direct;
    int ntiles, B, C;
    const float *cspart, *HSpart, *dz;
    const int32_t *tile_samp, *samp_len;
    float *cs, *Z, *dzsum;
};

constexpr int kTokStages = 3;
constexpr int kTokKT = 32;    // tokens per stage of the token contractions (a multiple of 16)
template <int NT> struct TokRedShapes {
    static constexpr bool BIG = NT > 4;
    // r > 128: 128 x 256 tiles, eight wavefronts, three stages (E then covers all of r: the cache is read once)
    // r = 96: 64 tokens per stage in a two-stage ring (same LDS; half the barriers: 37.5 -> 36.9 us on the T5-Base-shaped
    // step; at r = 128, L = 24 the same measured 2 us slower and is not used)
    static constexpr int KT = NT == 3 ? 64 : kTokKT, ST = NT == 3 ? 2 : kTokStages;
    using TBig = TnTile<2, 4, 2, 2, kTokKT, 3>;
    // r = 96, 128: the same 128 x 128 tile as 4 x 2 wavefronts of 32 x 64 (eight wavefronts issue the transfers of a
    // stage in half the time each; measured 42 -> 39 us on the T5-Base-shaped step)
    static constexpr bool W8 = NT == 3 || NT == 4;
    using TE = typename std::conditional<BIG, TBig, typename std::conditional<W8, TnTile<4, 2, 1, 2, KT, ST>, TnTile<2, 2, kETileCols / 64, (NT > 2 ? 2 : 1), kTokKT, kTokStages>>::type>::type;
    using TG = typename std::conditional<BIG, TBig, typename std::conditional<W8, TnTile<4, 2, 1, 2, KT, ST>, TnTile<2, 2, 2, 2, kTokKT, kTokStages>>::type>::type; // tile of the Gram matrix
    static constexpr int kThreadsPerBlock = (BIG || W8) ? 512 : 256;
    static constexpr int kVecLds = 256 * (1 + kMaxClasses) * 4 + kMaxTiles * 4 + kMaxBatch * kMaxClasses * 4; // + tile and sample tables
    static constexpr int kTileLds = TE::LDS_BYTES > TG::LDS_BYTES ? TE::LDS_BYTES : TG::LDS_BYTES;
    static constexpr int kLds = kTileLds > kVecLds ? kTileLds : kVecLds;
};

template <int NT> __global__ __launch_bounds__(TokRedShapes<NT>::kThreadsPerBlock) void k_gtokred(TokRedArgs a)
{
    using TE = typename TokRedShapes<NT>::TE;
    using TG = typename TokRedShapes<NT>::TG;
    constexpr int KT = TokRedShapes<NT>::KT;
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    __shared__ int64_t t_aoff[kMaxSplitTiles]; // cache offset of the tile's first row in this layer
    __shared__ int32_t t_m0[kMaxSplitTiles], t_rows[kMaxSplitTiles];
    // dispatch order (measured): E first where its workgroups and the Gram tiles all fit the chip at once
    // (T5-Base-shaped), the Gram tiles and the column sums first where they do not (Large-shaped)
    const int b = (a.reverse ? (int)(gridDim.x - 1 - blockIdx.x) : (int)blockIdx.x) + a.blk_off, t = threadIdx.x;
    const int M = a.map.M;
    const int Lr = a.L * a.r;
    if (b < a.nb_E) {
        // E_l[d-tile] over the 16-token tiles [tl0, tl1) of this split
        const int ect = (a.r + TE::BN - 1) / TE::BN; // column tiles of r (one up to r = 128)
        // All tiles that contract the same token rows of dpre_l (one layer, one token split: e_tiles x ect tiles)
        // go to one die, so that those rows cross the fabric once and are then found in that die's L2; numbered
        // round-robin, every die fetched every layer's dpre for itself (as many bytes again as the cache pass).
        const int per_group = a.e_tiles * ect;
        const int v = die_group_order(b, a.nb_E, per_group);
        const int ct = v % ect;
        const int it = (v / ect) % a.e_tiles;
        const int split = (v / per_group) % a.se;
        const int l = v / (per_group * a.se);
        const int tl0 = split * a.tiles_per_se;
        const int ntl = min(a.ntiles, tl0 + a.tiles_per_se) - tl0;
        for (int q = t; q < ntl; q += (int)blockDim.x) {
            const int m0 = a.tile_row0[tl0 + q];
            t_m0[q] = m0;
            t_rows[q] = a.tile_rows[tl0 + q];
            t_aoff[q] = a.map.rowoff[m0] + (int64_t)l * a.map.rowstride[m0];
        }
        __syncthreads();
        const bf16_t *cache = a.cache;
        const bf16_t *dp = a.DP + (int64_t)l * a.r;
        const int d = a.d;
        auto atok = [&](int step, int grp, int r8) -> const bf16_t * {
            const int tl = step * (KT / 16) + (grp >> 1), row = (grp & 1) * 8 + r8;
            if (tl >= ntl || row >= t_rows[tl]) return nullptr;
            return cache + t_aoff[tl] + (int64_t)row * d;
        };
        auto btok = [&](int step, int grp, int r8) -> const bf16_t * {
            const int tl = step * (KT / 16) + (grp >> 1), row = (grp & 1) * 8 + r8;
            if (tl >= ntl || row >= t_rows[tl]) return nullptr;
            return dp + (int64_t)(t_m0[tl] + row) * Lr;
        };
        EpiStoreF32 epi{a.Epart + ((int64_t)split * a.L + l) * a.d * a.r, a.r};
        gemm_tn<TE, true>(smem, atok, btok, a.zeros, epi, (ntl * 16 + KT - 1) / KT, it * TE::BM, ct * TE::BN, a.d, a.r, a.d, a.r);
        return;
    }
    if (b < a.nb_E + a.nb_G) {
        int idx = b - a.nb_E;
        // (numbered row-major, a die sees every eighth column panel of DP only: already local to its L2)
        const int split = idx % a.sg;
        idx /= a.sg;
        const int ti = idx / a.tgn, tj = idx % a.tgn;
        // needed only where some row layer is below some column layer
        const int kmin = (ti * TG::BM) / a.r;
        const int lmax = min(Lr - 1, tj * TG::BN + TG::BN - 1) / a.r;
        if (kmin >= lmax) return;
        const int kbegin = split * a.rows_per_sg;
        const int kend = min(M, kbegin + a.rows_per_sg);
        const bf16_t *H = a.H, *DP = a.DP;
        auto atok = [&](int step, int grp, int r8) -> const bf16_t * {
            const int k = kbegin + step * KT + grp * 8 + r8;
            return k < kend ? H + (int64_t)k * Lr : nullptr;
        };
        auto btok = [&](int step, int grp, int r8) -> const bf16_t * {
            const int k = kbegin + step * KT + grp * 8 + r8;
            return k < kend ? DP + (int64_t)k * Lr : nullptr;
        };
        if (a.gg_direct) {
            EpiGramDirect epi{a.GGT, a.GGsc, Lr, a.r, a.params, a.PL};
            gemm_tn<TG, true>(smem, atok, btok, a.zeros, epi, (kend - kbegin + KT - 1) / KT, ti * TG::BM, tj * TG::BN, Lr, Lr, Lr, Lr);
        } else {
            EpiStoreF32 epi{a.GGpart + (int64_t)split * Lr * Lr, Lr};
            gemm_tn<TG, true>(smem, atok, btok, a.zeros, epi, (kend - kbegin + KT - 1) / KT, ti * TG::BM, tj * TG::BN, Lr, Lr, Lr, Lr);
        }
        return;
    }
    // cs[kk] = sum over the tiles of their column sums of dpre ;
    // Z[kk][c] = sum_s mean_t(h)[s][kk] dz[s][c], from the tiles' column sums of h.
    // 16 indices per block, the tiles dealt over 16 thread groups whose sums are combined in group order.
    if (t >= 256) return; // this part is written for four wavefronts
    const int C = a.C;
    float *red = reinterpret_cast<float *>(smem); // [16 groups][16 indices][1 + kMaxClasses]
    const int vb = b - a.nb_E - a.nb_G;
    const int ii = t & 15, grp = t >> 4;
    const int idx = vb * 16 + ii;
    float acc = 0.f;
    float zc[kMaxClasses];
#pragma unroll
    for (int c = 0; c < kMaxClasses; ++c) zc[c] = 0.f;
    // per-sample weights dz / len and the tiles' sample numbers, staged so that the sums below
    // read global memory only for the column sums themselves
    int32_t *tsamp = reinterpret_cast<int32_t *>(smem + 256 * (1 + kMaxClasses) * 4); // [ntiles]
    float *swt = reinterpret_cast<float *>(tsamp + a.ntiles);                          // [B][C]
    for (int k = t; k < a.ntiles; k += 256) tsamp[k] = a.tile_samp[k];
    for (int q = t; q < a.B * C; q += 256) swt[q] = a.dz[q] / (float)a.samp_len[q / C];
    __syncthreads();
    if (idx < Lr) {
        for (int k0 = grp; k0 < a.ntiles; k0 += 16 * 4) {
            float cp[4], hp[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int k = min(k0 + 16 * u, a.ntiles - 1);
                cp[u] = a.cspart[(int64_t)k * Lr + idx];
                hp[u] = a.HSpart[(int64_t)k * Lr + idx];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int k = k0 + 16 * u;
                if (k < a.ntiles) {
                    acc += cp[u];
                    const float *w = swt + tsamp[k] * C;
#pragma unroll
                    for (int c = 0; c < kMaxClasses; ++c)
                        if (c < C) zc[c] += hp[u] * w[c];
                }
            }
        }
    }
    __syncthreads();
    red[(grp * 16 + ii) * (1 + kMaxClasses)] = acc;
#pragma unroll
    for (int c = 0; c < kMaxClasses; ++c)
        if (c < C) red[(grp * 16 + ii) * (1 + kMaxClasses) + 1 + c] = zc[c];
    __syncthreads();
    // thread (index ii, value q): q = 0 is cs, q = 1 + c is Z[.][c]
    for (int q = grp; q < 1 + C; q += 16) {
        float tot = 0.f;
        for (int g2 = 0; g2 < 16; ++g2) tot += red[(g2 * 16 + ii) * (1 + kMaxClasses) + q];
        if (idx < Lr) {
            if (q == 0) a.cs[idx] = tot;
            else a.Z[(int64_t)idx * C + q - 1] = tot;
        }
    }
    if (vb == 0 && t < C) {
        float sum = 0.f;
        for (int s = 0; s < a.B; ++s) sum += a.dz[s * C + t];
        a.dzsum[t] = sum;
    }
}

// ---------------------------------------------------------------------------
// launch 6: ordered sums of the token-split partials: E, and the Gram matrix, kept as the two bf16
// copies the last launch contracts: GG transposed, and GG with column layer l scaled by (1 - lambda_l)
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_ggsum(int L, int r, int sg, const float *GGpart, const float *params,
                                               int64_t PL, bf16_t *GGT, bf16_t *GGsc, int nb_GG, int se,
                                               int64_t e_elems, const float *Epart, float *E)
{
    __shared__ float tile[32][33];
    const int Lr = L * r;
    const int b = blockIdx.x, t = threadIdx.x;
    if (b >= nb_GG) {
        // E = ordered sum of its token-split partials, four elements per thread
        const int64_t o = ((int64_t)(b - nb_GG) * 256 + t) * 4;
        if (o < e_elems) { // e_elems is a multiple of 4
            f32x4 p[16]; // se <= 16; all partials requested before the first add
#pragma unroll
            for (int s2 = 0; s2 < 16; ++s2)
                if (s2 < se) p[s2] = *reinterpret_cast<const f32x4 *>(Epart + (int64_t)s2 * e_elems + o);
            f32x4 acc = p[0];
#pragma unroll
            for (int s2 = 1; s2 < 16; ++s2)
                if (s2 < se) acc += p[s2];
            *reinterpret_cast<f32x4 *>(E + o) = acc;
        }
        return;
    }
    const int tg = Lr / 32;
    const int tr = b / tg, tcx = b % tg;
    // rows of layer k, columns of layer l: used only for k < l
    if ((tr * 32) / r >= (tcx * 32 + 31) / r) return;
    const int tx = t & 31, ty = t >> 5;
    const int col = tcx * 32 + tx;
    const float lam = params[(int64_t)(col / r) * PL + PL - 1];
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < sg; ++s) { // four independent loads per split
        float p[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) p[q] = GGpart[((int64_t)s * Lr + tr * 32 + ty + 8 * q) * Lr + col];
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[q] += p[q];
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int y = ty + 8 * q, row = tr * 32 + y;
        tile[y][tx] = acc[q];
        GGsc[(int64_t)row * Lr + col] = static_cast<bf16_t>((1.f - lam) * acc[q]);
    }
    __syncthreads();
#pragma unroll
    for (int y = ty; y < 32; y += 8)
        GGT[(int64_t)(tcx * 32 + y) * Lr + tr * 32 + tx] = static_cast<bf16_t>(tile[tx][y]);
}

// ---------------------------------------------------------------------------
// launch 7: the gradients
// ---------------------------------------------------------------------------
struct PostArgs {
    int blk_off; // first block of this launch (parts may be launched separately for timing)
    int L, d, r, C, B, se;
    int nb_F, nb_W, nb_vec;
    const float *params;
    int64_t PL;
    const bf16_t *WuTs, *Wds, *GGT, *GGsc;
    const float *Epart, *cusum, *cs, *Z, *dzsum, *dz, *pb;
    float *grads;
    float *dlam_part;
    int slots;
};

struct EpiF {
    static constexpr bool kBatched = true;
    const float *Epart;
    int se;
    int64_t split_stride;
    const float *cusum_l, *cs_l, *Wd_l;
    float *gWd;
    int r;
    float lam;
    float dlam;
    __device__ void batch(int row_base, int col, const f32x16 &acc, int nrows, int ncols)
    {
        const int cc = min(col, ncols - 1);
        const float csv = cs_l[cc];
        float E[16], W[16], cu[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int rr = min(epi_row(row_base, v), nrows - 1);
            const int64_t o = (int64_t)rr * r + cc;
            E[v] = Epart[o];
            W[v] = Wd_l[o];
            cu[v] = cusum_l[rr];
        }
        for (int s = 1; s < se; ++s) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int rr = min(epi_row(row_base, v), nrows - 1);
                E[v] += Epart[(int64_t)s * split_stride + (int64_t)rr * r + cc];
            }
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = epi_row(row_base, v);
            if (row < nrows && col < ncols) {
                const float F = acc[v] + cu[v] * csv;
                gWd[(int64_t)row * r + col] = lam * E[v] + (1.f - lam) * F;
                dlam += (E[v] - F) * W[v];
            }
        }
    }
};

struct EpiW {
    static constexpr bool kBatched = true;
    const float *Z_l, *Wc;
    float *gWu;
    int d, C;
    __device__ void batch(int row_base, int col, const f32x16 &acc, int nrows, int ncols) const
    {
        const int cc = min(col, ncols - 1);
        float out[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) out[v] = acc[v];
        for (int c = 0; c < C; ++c) {
            const float w = Wc[(int64_t)cc * C + c];
            float z[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) z[v] = Z_l[(int64_t)min(epi_row(row_base, v), nrows - 1) * C + c];
#pragma unroll
            for (int v = 0; v < 16; ++v) out[v] += z[v] * w;
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = epi_row(row_base, v);
            if (row < nrows && col < ncols) gWu[(int64_t)row * d + col] = out[v];
        }
    }
};

// wz[c] += sum_e u[e] Z[e][c] over 8 rows of CC classes each (Z 16-byte aligned)
template <int CC> __device__ __forceinline__ void zrows(const float *Z, const Chunk<bf16_t> &u8, float (&wz)[kMaxClasses])
{
    f32x4 z[2 * CC];
#pragma unroll
    for (int v = 0; v < 2 * CC; ++v) z[v] = *reinterpret_cast<const f32x4 *>(Z + 4 * v);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float u = to_f32(u8.e[e]);
#pragma unroll
        for (int c = 0; c < CC; ++c) wz[c] += u * z[(CC * e + c) >> 2][(CC * e + c) & 3];
    }
}

template <int BK, bool BIG, bool XW = false> struct PostShapes {
    // 64 x 64 with 64 KB of stages; or (r > 128) eight wavefronts, three stages, interleaved sub-steps:
    // 128 rows of d x 256 columns of r for F, 256 rows of r x 128 columns of d for W
    using TSmall = NtTile<2, 2, 1, 1, BK, BK == 64 ? 4 : 8>;
    using TFF = typename std::conditional<BIG, NtTile<2, 4, 2, 2, BK, 3>, TSmall>::type;
    using TFW = typename std::conditional<BIG, NtTile<4, 2, 2, 2, BK, 3>, TSmall>::type;
    static constexpr int NH = XW ? 8 : BIG ? 4 : 2; // threads sharing one r-wide row in the vector part (XW: r > 256)
    static constexpr int kThreadsPerBlock = BIG ? 512 : 256;
    static constexpr int kVecLds = 128 * 4 + 128 * kMaxClasses * 4 + kMaxBatch * kMaxClasses * 4;
    static constexpr int kLds = TFF::LDS_BYTES > TFW::LDS_BYTES ? TFF::LDS_BYTES : TFW::LDS_BYTES;
    static_assert(kLds >= kVecLds, "LDS budget of the gradient kernel");
};

// BK = 64 when r is a multiple of 64, else 32: every K range below is a multiple of r
template <int BK, bool BIG, bool XW> __global__ __launch_bounds__(BIG ? 512 : 256) void k_gpost(PostArgs a)
{
    using TFF = typename PostShapes<BK, BIG, XW>::TFF;
    using TFW = typename PostShapes<BK, BIG, XW>::TFW;
    constexpr int kVecLds = PostShapes<BK, BIG, XW>::kVecLds;
    constexpr int kLds = PostShapes<BK, BIG, XW>::kLds;
    constexpr int NH = PostShapes<BK, BIG, XW>::NH;
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    __shared__ float red[16];
    const int L = a.L, d = a.d, r = a.r, C = a.C;
    const int Lr = L * r;
    const int64_t dr = (int64_t)d * r;
    const int b = (int)(gridDim.x - 1 - blockIdx.x) + a.blk_off, t = threadIdx.x; // reverse dispatch, as in k_gproj
    if (b < a.nb_F) {
        const int ti_d = (d + TFF::BM - 1) / TFF::BM, ti_r = (r + TFF::BN - 1) / TFF::BN;
        // F_l = sum_{k<l} W_up^{kT} G_{kl}   ([d] x [l*r] times [l*r] x [r])
        int l, slot, it, nt;
        if (BIG && ti_d % 8 == 0) {
            // A die takes ti_d / 8 tiles along d for every layer: the rows of the stacked W_up copy those tiles read are
            // shared by all layers (each layer contracts a prefix of them), so they cross the fabric once per die
            // instead of once per layer.  Within a die the layers run from the last (longest contraction) down.
            const int per_die = ti_d / 8 * ti_r * L;
            const int v = die_chunk_order(b, a.nb_F);
            const int die = v / per_die, w = v % per_die;
            l = w / (ti_d / 8 * ti_r);
            const int q = w % (ti_d / 8 * ti_r);
            it = die * (ti_d / 8) + q / ti_r;
            nt = q % ti_r;
            slot = it * ti_r + nt;
        } else {
            const int v = BIG ? die_group_order(b, a.nb_F, 8) : b;
            l = v / (ti_d * ti_r);
            slot = v % (ti_d * ti_r);
            it = slot / ti_r;
            nt = slot % ti_r;
        }
        const float *pl = a.params + (int64_t)l * a.PL;
        const bf16_t *A = a.WuTs, *B = a.GGT + (int64_t)l * r * Lr;
        auto arow = [&](int row) { return A + (int64_t)row * Lr; };
        auto brow = [&](int c) { return B + (int64_t)c * Lr; };
        EpiF epi{a.Epart + (int64_t)l * dr, a.se, (int64_t)L * dr, a.cusum + (int64_t)l * d, a.cs + (int64_t)l * r,
                 pl, a.grads + (int64_t)l * a.PL, r, pl[a.PL - 1], 0.f};
        gemm_nt<TFF, true>(smem, arow, brow, epi, 0, l * r, it * TFF::BM, nt * TFF::BN, d, r);
        const float tot = block_sum(epi.dlam, red);
        if (t == 0) a.dlam_part[(int64_t)l * a.slots + slot] = tot; // summed in slot order by k_gfinish
        return;
    }
    if (b < a.nb_F + a.nb_W) {
        // dW_up^l = Z_l W_cls^T + sum_{k>l} (1-lambda_k) G_{lk} W_down^{kT}
        const int ti_r = (r + TFW::BM - 1) / TFW::BM, ti_d = (d + TFW::BN - 1) / TFW::BN;
        int l, at, jt;
        if (BIG && ti_d % 8 == 0) {
            // as for F: a die takes ti_d / 8 tiles along d (rows of the stacked W_down copy) for every layer
            const int per_die = ti_d / 8 * ti_r * L;
            const int v = die_chunk_order(b - a.nb_F, a.nb_W);
            const int die = v / per_die, w = v % per_die;
            l = L - 1 - w / (ti_d / 8 * ti_r); // the first layers have the longest contractions here
            const int q = w % (ti_d / 8 * ti_r);
            jt = die * (ti_d / 8) + q / ti_r;
            at = q % ti_r;
        } else {
            int idx = BIG ? die_group_order(b - a.nb_F, a.nb_W, 8) : b - a.nb_F;
            l = idx / (ti_d * ti_r);
            idx %= ti_d * ti_r;
            // (wide shapes: the row tiles of a column tile next to each other)
            at = BIG ? idx % ti_r : idx / ti_d;
            jt = BIG ? idx / ti_r : idx % ti_d;
        }
        const bf16_t *A = a.GGsc + (int64_t)l * r * Lr, *B = a.Wds;
        auto arow = [&](int row) { return A + (int64_t)row * Lr; };
        auto brow = [&](int c) { return B + (int64_t)c * Lr; };
        EpiW epi{a.Z + (int64_t)l * r * C, a.params + (int64_t)L * a.PL,
                 a.grads + (int64_t)l * a.PL + dr + r, d, C};
        gemm_nt<TFW, true>(smem, arow, brow, epi, (l + 1) * r, Lr, at * TFW::BM, jt * TFW::BN, r, d);
        return;
    }
    if (BIG && t >= 256) return; // the remaining parts are written for four wavefronts
    const int vb = b - a.nb_F - a.nb_W;
    if (vb < a.nb_vec - 1) {
        // thread (jj, k, hf): hidden index j = vb * jpb + jj, layer k, part hf (of NH) of the r-wide rows
        float *tsh = reinterpret_cast<float *>(smem);          // [jpb][L]      (1-lambda_k) W_down^k[j] . cs_k
        float *wsh = tsh + 128;                                // [jpb][L][C]   W_up^k[.][j] . Z_k + pooled part
        float *sdz = wsh + 128 * kMaxClasses;                  // [B][C]
        float *stage = sdz + kMaxBatch * kMaxClasses;          // cs [Lr], Z [Lr][C] when they fit
        const int jpb = (256 / NH) / L;
        const int hf = t % NH, jk = t / NH;
        const int jj = jk / L, k = jk % L;
        const int j = vb * jpb + jj;
        const bool act = jj < jpb && j < d;
        const int rh = r / NH; // a multiple of 8
        const float *Wc = a.params + (int64_t)L * a.PL;
        // this thread's two row segments, requested before anything else is waited for
        constexpr int kMaxChunks = 8; // r / NH <= 64
        u32x4 wv[kMaxChunks], uv[kMaxChunks];
        {
            const int64_t row = act ? (int64_t)j * Lr + (int64_t)k * r + hf * rh : 0;
#pragma unroll
            for (int q = 0; q < kMaxChunks; ++q) {
                const int qq = q * 8 < rh ? q * 8 : 0;
                wv[q] = *reinterpret_cast<const u32x4 *>(a.Wds + row + qq);
                uv[q] = *reinterpret_cast<const u32x4 *>(a.WuTs + row + qq);
            }
        }
        const bool staged = (int64_t)Lr * (1 + C) * 4 + kVecLds <= kLds;
        for (int q = t; q < a.B * C; q += 256) sdz[q] = a.dz[q];
        if (staged) {
            stage_to_lds<256>(stage, a.cs, Lr);
            stage_to_lds<256>(stage + Lr, a.Z, Lr * C);
        }
        float base = 0.f; // (sum_s dz_s) W_cls^T [j]
        {
            float dzs_r[kMaxClasses], wc_r[kMaxClasses];
#pragma unroll
            for (int c = 0; c < kMaxClasses; ++c)
                if (c < C) {
                    dzs_r[c] = a.dzsum[c];
                    wc_r[c] = Wc[(int64_t)(act ? j : 0) * C + c];
                }
#pragma unroll
            for (int c = 0; c < kMaxClasses; ++c)
                if (c < C) base += dzs_r[c] * wc_r[c];
        }
        float pbv[2]; // pooled last-layer means of the samples s = k + (NH q + hf) L this thread covers first
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int s2 = k + (NH * q + hf) * L;
            pbv[q] = (act && s2 < a.B) ? a.pb[(int64_t)s2 * d + j] : 0.f;
        }
        const float cl = act ? a.cusum[(int64_t)L * d + j] : 0.f;
        const float lamk = a.params[(int64_t)k * a.PL + a.PL - 1];
        __syncthreads();
        {
            const float *csk = (staged ? stage : a.cs) + (int64_t)k * r + hf * rh;
            const float *Zk = (staged ? stage + Lr : a.Z) + ((int64_t)k * r + hf * rh) * C;
            float acc = 0.f;
            float wz[kMaxClasses];
#pragma unroll
            for (int c = 0; c < kMaxClasses; ++c) wz[c] = 0.f;
            if (act) {
#pragma unroll
                for (int q = 0; q < kMaxChunks; ++q)
                    if (q * 8 < rh) {
                        Chunk<bf16_t> w8, u8;
                        __builtin_memcpy(&w8, &wv[q], 16);
                        __builtin_memcpy(&u8, &uv[q], 16);
                        // 16-byte reads of the column sums (both sides are 16-byte aligned: rh % 8 == 0)
                        const f32x4 c0 = *reinterpret_cast<const f32x4 *>(csk + q * 8);
                        const f32x4 c1 = *reinterpret_cast<const f32x4 *>(csk + q * 8 + 4);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            acc += c0[e] * to_f32(w8.e[e]);
                            acc += c1[e] * to_f32(w8.e[4 + e]);
                        }
                        // Z of these 8 rows: 8 C consecutive floats, read as 2 C 16-byte pieces
                        if (C == 3) zrows<3>(Zk + (int64_t)q * 8 * 3, u8, wz);
                        else if (C == 4) zrows<4>(Zk + (int64_t)q * 8 * 4, u8, wz);
                        else if (C == 2) zrows<2>(Zk + (int64_t)q * 8 * 2, u8, wz);
                        else {
#pragma unroll
                            for (int e = 0; e < 8; ++e) {
                                const float u = to_f32(u8.e[e]);
#pragma unroll
                                for (int c = 0; c < kMaxClasses; ++c)
                                    if (c < C) wz[c] += u * Zk[(int64_t)(q * 8 + e) * C + c];
                            }
                        }
                    }
                // pooled part of dW_cls, the samples dealt over (k, hf)
                for (int s2 = k + hf * L, q = 0; s2 < a.B; s2 += NH * L, ++q) {
                    const float pv = (q < 2 ? pbv[q] : a.pb[(int64_t)s2 * d + j]) + cl;
#pragma unroll
                    for (int c = 0; c < kMaxClasses; ++c)
                        if (c < C) wz[c] += pv * sdz[s2 * C + c];
                }
            }
            // the parts sit in neighbouring lanes
#pragma unroll
            for (int o = 1; o < NH; o <<= 1) {
                acc += __shfl_xor(acc, o, 64);
#pragma unroll
                for (int c = 0; c < kMaxClasses; ++c)
                    if (c < C) wz[c] += __shfl_xor(wz[c], o, 64);
            }
            if (act && hf == 0) {
                tsh[jj * L + k] = (1.f - lamk) * acc;
#pragma unroll
                for (int c = 0; c < kMaxClasses; ++c)
                    if (c < C) wsh[(jj * L + k) * C + c] = wz[c];
            }
        }
        __syncthreads();
        if (!act) return;
        if (hf == 0) {
            // dc_up^k[j] = (sum_s dz_s) W_cls^T [j] + sum_{k'>k} t[j][k']
            for (int k2 = k + 1; k2 < L; ++k2) base += tsh[jj * L + k2];
            a.grads[(int64_t)k * a.PL + 2 * dr + r + j] = base;
        }
        // dW_cls[j][c] = sum_s (pb[s][j] + cusum_L[j]) dz[s][c] + sum_k W_up^k[.][j] . Z_k[.][c]
        for (int c = NH * k + hf; c < C; c += NH * L) {
            float acc = 0.f;
            for (int k2 = 0; k2 < L; ++k2) acc += wsh[(jj * L + k2) * C + c];
            a.grads[(int64_t)L * a.PL + (int64_t)j * C + c] = acc;
        }
        return;
    }
    // dc_down^l = colsum(dpre_l) ; dc_cls = sum_s dz_s
    for (int idx = t; idx < Lr; idx += 256) {
        const int l = idx / r, nn = idx % r;
        a.grads[(int64_t)l * a.PL + dr + nn] = a.cs[idx];
    }
    if (t < C) a.grads[(int64_t)L * a.PL + (int64_t)d * C + t] = a.dzsum[t];
}

// last launch: the two scalar reductions whose inputs come from many workgroups, in a fixed order
__global__ __launch_bounds__(64) void k_gfinish(const float *loss_part, int B, float *loss_out,
                                                const float *dlam_part, int slots, int L, int64_t PL, float *grads)
{
    const int t = threadIdx.x;
    if (t == 0 && loss_out) {
        float tot = 0.f;
        for (int s = 0; s < B; ++s) tot += loss_part[s];
        *loss_out = tot / (float)B;
    }
    if (grads)
        for (int l = t; l < L; l += 64) {
            float acc = 0.f;
            for (int s = 0; s < slots; ++s) acc += dlam_part[(int64_t)l * slots + s];
            grads[(int64_t)l * PL + PL - 1] = acc;
        }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
// Launch a kernel whose block index selects one of several parts: in one go, or (for per-part
// timing) one launch per part with its own profile class.
template <class Args, class Kern>
static void launch_parts(Profiler *prof, hipStream_t st, bool split, Kern kern, Args a, int nparts, const int *counts,
                         const int *classes, int whole_class, unsigned threads, size_t lds = 0)
{
    int total = 0;
    for (int i = 0; i < nparts; ++i) total += counts[i];
    if (!split) {
        a.blk_off = 0;
        if (total > 0) PAC_LAUNCH(prof, st, whole_class, kern, dim3(total), dim3(threads), lds, st, a);
        return;
    }
    int off = 0;
    for (int i = 0; i < nparts; ++i) {
        a.blk_off = off;
        if (counts[i] > 0) PAC_LAUNCH(prof, st, classes[i], kern, dim3(counts[i]), dim3(threads), lds, st, a);
        off += counts[i];
    }
}

// Raises a kernel's dynamic LDS limit before its first launch: once per process and kernel, whichever host
// thread comes first (contexts may be stepped from several threads; the others wait for the call to finish
// and all see its result).
template <auto Kern> static hipError_t allow_lds_once(int lds)
{
    static std::once_flag once;
    static hipError_t result = hipSuccess;
    std::call_once(once, [&] {
        result = hipFuncSetAttribute(reinterpret_cast<const void *>(Kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    });
    return result;
}

template <int NT> static hipError_t run_gram(const Dims &D, const WsLayout &W, const BatchMeta &meta, const StepIO &io)
{
    hipStream_t st = io.stream;
    Profiler *prof = io.prof;
    char *ws = io.ws;
    const int L = D.L, d = D.d, r = D.r, C = D.C, M = meta.M, B = meta.B;
    const int Lr = L * r;
    const bool split = (D.flags & 2) != 0;
    int ntiles = 0;
    for (int s = 0; s < B; ++s) ntiles += cdiv(meta.len[s], kChainRows);

    int64_t *rowoff = (int64_t *)(ws + W.rowoff);
    int32_t *rowstride = (int32_t *)(ws + W.rowstride);
    int32_t *rowsamp = (int32_t *)(ws + W.rowsamp);
    int32_t *samp_start = (int32_t *)(ws + W.samp_start);
    int32_t *samp_len = (int32_t *)(ws + W.samp_len);
    int32_t *tile_row0 = (int32_t *)(ws + W.g_tile_row0);
    int32_t *tile_rows = (int32_t *)(ws + W.g_tile_rows);
    int32_t *tile_samp = (int32_t *)(ws + W.g_tile_samp);
    int32_t *samp_tile0 = (int32_t *)(ws + W.g_samp_tile0);
    float *loss_part = (float *)(ws + W.g_loss_part);
    bf16_t *WdT = (bf16_t *)(ws + W.WdT), *Wu = (bf16_t *)(ws + W.Wu);
    bf16_t *WuTs = (bf16_t *)(ws + W.g_WuTs), *Wds = (bf16_t *)(ws + W.g_Wds);
    float *cusum = (float *)(ws + W.g_cusum), *chat = (float *)(ws + W.g_chat), *V = (float *)(ws + W.g_V);
    bf16_t *QpN = (bf16_t *)(ws + W.g_QpN), *QpT = (bf16_t *)(ws + W.g_QpT);
    float *pre = (float *)(ws + W.pre_all);
    bf16_t *H = (bf16_t *)(ws + W.h_all), *DP = (bf16_t *)(ws + W.g_DP);
    float *pb = (float *)(ws + W.pooled);
    float *HSpart = (float *)(ws + W.g_HSpart), *cspart = (float *)(ws + W.g_cspart);
    float *logits = (float *)(ws + W.logits), *dz = (float *)(ws + W.dz);
    float *zpart = (float *)(ws + W.g_zpart), *zpb = (float *)(ws + W.g_zpb);
    float *Z = (float *)(ws + W.g_Z), *dzsum = (float *)(ws + W.g_dzsum);
    float *cs = (float *)(ws + W.g_cs);
    float *Epart = (float *)(ws + W.g_Epart), *GGpart = (float *)(ws + W.g_GGpart);
    bf16_t *GGT = (bf16_t *)(ws + W.g_GGT), *GGsc = (bf16_t *)(ws + W.g_GGsc);
    float *dlam_part = (float *)(ws + W.g_dlam_part);
    const RowMap map{rowoff, rowstride, M};
    const bf16_t *cache = (const bf16_t *)io.cache;

    {
        PrepArgs a;
        a.meta = meta; a.params = io.params; a.PL = D.PL; a.L = L; a.d = d; a.r = r; a.C = C;
        a.nb_setup = cdiv(M, 256); // several weight tiles per workgroup only where that still leaves thousands of workgroups
        const int tpb = (int64_t)(d / 32) * (r / 32) * L * 2 >= 8192 * kPrepTiles ? kPrepTiles : 1;
        a.nb_shadow = cdiv((int64_t)(d / 32) * (r / 32) * L * 2, tpb); a.nb_chat = cdiv(d, 256);
        a.tile64 = tpb == kPrepTiles && d % 64 == 0 && r % 64 == 0;
        if (a.tile64) a.nb_shadow = (d / 64) * (r / 64) * L * 2;
        a.rowoff = rowoff; a.rowstride = rowstride; a.rowsamp = rowsamp; a.samp_start = samp_start;
        a.samp_len = samp_len; a.tile_row0 = tile_row0; a.tile_rows = tile_rows; a.tile_samp = tile_samp; a.samp_tile0 = samp_tile0;
        a.WdT = WdT; a.Wu = Wu; a.WuTs = WuTs; a.Wds = Wds; a.cusum = cusum; a.V = V;
        a.zero = (float *)(ws + W.g_zero);
        const int v_rpw = tpb == 1 ? 1 : 4;
        const int counts[4] = {a.nb_setup, a.nb_shadow, a.nb_chat, cdiv(Lr, 4 * v_rpw)};
        const int classes[4] = {KC_G_PREP_SETUP, KC_G_PREP_COPY, KC_G_PREP_CHAT, KC_G_PREP_V};
        if (tpb == 1) launch_parts(prof, st, split, k_gprep<1, 1>, a, 4, counts, classes, KC_G_PREP, 256);
        else launch_parts(prof, st, split, k_gprep<kPrepTiles, 4>, a, 4, counts, classes, KC_G_PREP, 256);
    }
    // a launch that was refused leaves the tables the later kernels index with unwritten: stop here
    PAC_HIP_TRY(hipGetLastError());
    {
        ProjArgs a;
        a.cache = cache; a.map = map; a.L = L; a.d = d; a.r = r; a.B = B;
        constexpr int kQRows = NT > 4 ? 128 : 64, kQCols = NT > 4 ? 256 : 64; // ProjShapes<NT, .>::TQ
        constexpr int kProjThreads = NT > 4 ? 512 : 256;
        a.row_tiles = cdiv(M, 128); a.nb_U = a.row_tiles * L * (NT > 4 ? cdiv(r, 256) : 1);
        a.nb_Q = W.pairs * cdiv(r, kQRows) * cdiv(r, kQCols);
        if (NT <= 4 && W.use_gram != 2) a.nb_Q = L > 1 ? cdiv(Lr, 128) * cdiv(Lr, 128) : 0; // ProjShapes::QSTACK
        if (NT > 4) { // blocks of 4 x 4 layer pairs, see k_gproj
            const int nlb = cdiv(L, 4);
            a.nb_Q = L > 1 ? nlb * (nlb + 1) / 2 * 16 * cdiv(r, kQRows) * cdiv(r, kQCols) : 0;
        }
        a.nb_C = L * cdiv(r, 64);
        a.cusum = cusum; a.chat = chat; a.params = io.params; a.PL = D.PL;
        a.WdT = WdT; a.Wu = Wu; a.U = pre; a.QpN = QpN; a.QpT = QpT;
        a.QgN = (bf16_t *)(ws + W.g_QgN); a.QgT = (bf16_t *)(ws + W.g_QgT); a.chain_group = W.chain_group;
        a.samp_start = samp_start; a.samp_len = samp_len; a.pb = pb; a.C = C; a.zpbp = zpb;
        const int counts[4] = {a.nb_U, a.nb_Q, a.nb_C, B * cdiv(d, 256)};
        const int classes[4] = {KC_G_PROJ_U, KC_G_PROJ_Q, KC_G_PROJ_Q, KC_G_PROJ_PB};
        auto launch_proj = [&](auto kern, int lds) {
            launch_parts(prof, st, split, kern, a, 4, counts, classes, KC_G_PROJ, kProjThreads, lds);
        };
        const bool q_full = W.use_gram == 2;
        if (d % 64 == 0) {
            constexpr int lds = ProjShapes<NT, 64, true>::kLds > ProjShapes<NT, 64, false>::kLds ? ProjShapes<NT, 64, true>::kLds : ProjShapes<NT, 64, false>::kLds;
            if (q_full) { PAC_HIP_TRY((allow_lds_once<&k_gproj<NT, 64, true>>(lds))); launch_proj(&k_gproj<NT, 64, true>, lds); }
            else { PAC_HIP_TRY((allow_lds_once<&k_gproj<NT, 64, false>>(lds))); launch_proj(&k_gproj<NT, 64, false>, lds); }
        } else {
            constexpr int lds = ProjShapes<NT, 32, true>::kLds > ProjShapes<NT, 32, false>::kLds ? ProjShapes<NT, 32, true>::kLds : ProjShapes<NT, 32, false>::kLds;
            if (q_full) { PAC_HIP_TRY((allow_lds_once<&k_gproj<NT, 32, true>>(lds))); launch_proj(&k_gproj<NT, 32, true>, lds); }
            else { PAC_HIP_TRY((allow_lds_once<&k_gproj<NT, 32, false>>(lds))); launch_proj(&k_gproj<NT, 32, false>, lds); }
        }
    }
    PAC_HIP_TRY(hipGetLastError());
    PAC_HIP_TRY((allow_lds_once<&k_gtokred<NT>>(TokRedShapes<NT>::kLds)));
    ChainArgs ca;
    ca.L = L; ca.r = r; ca.M = M; ca.tile_row0 = tile_row0; ca.tile_rows = tile_rows; ca.tile_samp = tile_samp;
    ca.params = io.params; ca.PL = D.PL; ca.d = d; ca.U = pre; ca.Gp = (bf16_t *)(ws + W.g_Gp); ca.chat = chat;
    ca.B = B; ca.C = C; ca.V = V; ca.zpart = zpart; ca.zpbp = zpb; ca.nzb = cdiv(d, 256);
    ca.samp_tile0 = samp_tile0; ca.samp_len = samp_len; ca.labels = io.labels;
    ca.logits_ws = logits; ca.logits_out = io.logits_out; ca.dz = dz; ca.loss_part = loss_part;
    if (W.use_gram == 1) {
        if constexpr (NT <= 4) {
            const size_t lds_fwd = chain_lds(L, r, true), lds_bwd = chain_lds(L, r, false);
            PAC_HIP_TRY((allow_lds_once<&k_gchain<true, NT>>(160 * 1024)));
            PAC_HIP_TRY((allow_lds_once<&k_gchain<true, NT, 4>>(160 * 1024)));
            PAC_HIP_TRY((allow_lds_once<&k_gchain<false, NT>>(160 * 1024)));
            {
                ChainArgs a = ca;
                a.Q = QpT; a.Hg = H; a.part = HSpart;
                if (C <= 4) PAC_LAUNCH(prof, st, KC_G_CHAIN_FWD, (k_gchain<true, NT, 4>), dim3(ntiles), dim3(64 * (2 * NT + 1)), lds_fwd, st, a);
                else PAC_LAUNCH(prof, st, KC_G_CHAIN_FWD, (k_gchain<true, NT>), dim3(ntiles), dim3(64 * (2 * NT + 1)), lds_fwd, st, a);
            }
            if (!io.grads) {
                PAC_LAUNCH(prof, st, KC_G_HEAD, k_glogits, dim3(B), dim3(64), 0, st, ca);
                PAC_LAUNCH(prof, st, KC_G_FINISH, k_gfinish, dim3(1), dim3(64), 0, st, loss_part, B, io.loss_out, nullptr, 0, L,
                           D.PL, nullptr);
                return hipGetLastError();
            }
            {
                ChainArgs a = ca;
                a.Q = QpN; a.Hg = DP; a.part = cspart;
                PAC_LAUNCH(prof, st, KC_G_CHAIN_BWD, (k_gchain<false, NT>), dim3(ntiles), dim3(64 * (2 * NT + 1)), lds_bwd, st, a);
            }
        } else {
            return hipErrorInvalidValue;
        }
    } else {
        // groups of W.chain_group layers: one wide contraction per group, then the group's own layers
        const bool k64 = r % 64 == 0;
        const int big_lds = k64 ? SeqShapes<64>::TB::LDS_BYTES : SeqShapes<32>::TB::LDS_BYTES;
        const int small_lds = k64 ? SeqShapes<64>::TS::LDS_BYTES : SeqShapes<32>::TS::LDS_BYTES;
        PAC_HIP_TRY((allow_lds_once<&k_gseq_big<64>>(SeqShapes<64>::TB::LDS_BYTES)));
        PAC_HIP_TRY((allow_lds_once<&k_gseq_big<32>>(SeqShapes<32>::TB::LDS_BYTES)));
        PAC_HIP_TRY((allow_lds_once<&k_gseq_group<true>>(160 * 1024)));
        PAC_HIP_TRY((allow_lds_once<&k_gseq_group<false>>(160 * 1024)));
        float *P = (float *)(ws + W.g_P), *ghat = (float *)(ws + W.g_ghat);
        const int g = W.chain_group, ldp = g * r;
        const int rt128 = cdiv(M, kSeqTile), rt64 = cdiv(M, 64), ct64 = cdiv(r, 64);
        auto chain_group = [&](bool fwd, int l0) {
            const int l1 = l0 + g < L ? l0 + g : L;
            const int cls = fwd ? KC_G_CHAIN_FWD : KC_G_CHAIN_BWD;
            SeqBigArgs ba;
            ba.A = fwd ? H : DP; ba.Bq = fwd ? QpT : QpN; ba.P = P; ba.L = L; ba.r = r; ba.M = M; ba.ldp = ldp;
            ba.brow0 = l0 * r; ba.ncols = (l1 - l0) * r;
            ba.kbegin = fwd ? 0 : l1 * r; ba.kend = fwd ? l0 * r : Lr;
            ba.ctiles = cdiv(ba.ncols, kSeqTile);
            const bool have_big = ba.kend > ba.kbegin;
            if (have_big) {
                if (k64) PAC_LAUNCH(prof, st, cls, k_gseq_big<64>, dim3(rt128 * ba.ctiles), dim3(256), big_lds, st, ba);
                else PAC_LAUNCH(prof, st, cls, k_gseq_big<32>, dim3(rt128 * ba.ctiles), dim3(256), big_lds, st, ba);
            }
            if (r <= kGroupMaxR) {
                // one launch for the group's layers (wider adapters: one launch per layer, below)
                SeqGroupArgs ga;
                SeqLayerArgs &la = ga.la;
                la.A = ba.A; la.Bq = ba.Bq; la.P = have_big ? P : nullptr; la.ldp = ldp; la.pcol0 = 0;
                la.l = l0; la.L = L; la.r = r; la.M = M; la.d = d;
                la.kbegin = 0; la.kend = 0; la.ctiles = 0;
                la.U = pre; la.Gp = ca.Gp; la.chat = chat; la.params = io.params; la.PL = D.PL;
                la.Hg = fwd ? H : DP; la.ghat = ghat; la.rowsamp = rowsamp;
                ga.l0 = l0; ga.l1 = l1;
                ga.Qg = (const bf16_t *)(ws + (fwd ? W.g_QgT : W.g_QgN)) + (int64_t)(l0 / g) * (g * (g - 1) / 2) * r * r;
                const int lds = (int)group_lds(l1 - l0, r);
                const dim3 grid(cdiv(M, kChainRows)), block(64 * (r / 32 + kGroupHelpers));
                if (fwd) PAC_LAUNCH(prof, st, cls, (k_gseq_group<true>), grid, block, lds, st, ga);
                else PAC_LAUNCH(prof, st, cls, (k_gseq_group<false>), grid, block, lds, st, ga);
                return;
            }
            for (int q = 0; q < l1 - l0; ++q) {
                const int l = fwd ? l0 + q : l1 - 1 - q;
                SeqLayerArgs la;
                la.A = ba.A; la.Bq = ba.Bq; la.P = have_big ? P : nullptr; la.ldp = ldp; la.pcol0 = (l - l0) * r;
                la.l = l; la.L = L; la.r = r; la.M = M; la.d = d;
                la.kbegin = fwd ? l0 * r : (l + 1) * r; la.kend = fwd ? l * r : l1 * r; la.ctiles = ct64;
                la.U = pre; la.Gp = ca.Gp; la.chat = chat; la.params = io.params; la.PL = D.PL;
                la.Hg = fwd ? H : DP; la.ghat = ghat; la.rowsamp = rowsamp;
                const dim3 grid(rt64 * ct64);
                if (fwd) {
                    if (k64) PAC_LAUNCH(prof, st, cls, (k_gseq_layer<true, 64>), grid, dim3(256), small_lds, st, la);
                    else PAC_LAUNCH(prof, st, cls, (k_gseq_layer<true, 32>), grid, dim3(256), small_lds, st, la);
                } else {
                    if (k64) PAC_LAUNCH(prof, st, cls, (k_gseq_layer<false, 64>), grid, dim3(256), small_lds, st, la);
                    else PAC_LAUNCH(prof, st, cls, (k_gseq_layer<false, 32>), grid, dim3(256), small_lds, st, la);
                }
            }
        };
        const int ngroups = cdiv(L, g);
        for (int q = 0; q < ngroups; ++q) chain_group(true, q * g);
        PAC_LAUNCH(prof, st, KC_G_CHAIN_FWD, k_gseq_colsum, dim3(ntiles, cdiv(Lr, 256)), dim3(256), 0, st, H, Lr, tile_row0,
                   tile_rows, HSpart);
        PAC_LAUNCH(prof, st, KC_G_HEAD, k_gseq_zpart, dim3(ntiles), dim3(256), 0, st, HSpart, V, Lr, C, zpart);
        PAC_LAUNCH(prof, st, KC_G_HEAD, k_glogits, dim3(B), dim3(64), 0, st, ca);
        if (!io.grads) {
            PAC_LAUNCH(prof, st, KC_G_FINISH, k_gfinish, dim3(1), dim3(64), 0, st, loss_part, B, io.loss_out, nullptr, 0, L,
                       D.PL, nullptr);
            return hipGetLastError();
        }
        PAC_LAUNCH(prof, st, KC_G_CHAIN_BWD, k_gseq_ghat, dim3(cdiv(Lr, 256), B), dim3(256), 0, st, dz, V, samp_len, Lr, C, ghat);
        for (int q = ngroups - 1; q >= 0; --q) chain_group(false, q * g);
        PAC_LAUNCH(prof, st, KC_G_CHAIN_BWD, k_gseq_colsum, dim3(ntiles, cdiv(Lr, 256)), dim3(256), 0, st, DP, Lr, tile_row0,
                   tile_rows, cspart);
    }
    {
        TokRedArgs a;
        a.cache = cache; a.map = map; a.L = L; a.d = d; a.r = r;
        a.e_tiles = cdiv(d, kETileCols);
        {
            // W.se is fixed by the configuration (the partial buffers are sized for it)
            if (cdiv(ntiles, W.se) > kMaxSplitTiles) return hipErrorInvalidValue;
            a.tiles_per_se = cdiv(cdiv(ntiles, W.se), TokRedShapes<NT>::KT / 16) * (TokRedShapes<NT>::KT / 16);
            a.se = cdiv(ntiles, a.tiles_per_se);
        }
        a.tile_row0 = tile_row0; a.tile_rows = tile_rows; a.zeros = ws + W.g_zero;
        a.rows_per_sg = cdiv(cdiv(M, W.sg), 128) * 128;
        a.sg = cdiv(M, a.rows_per_sg);
        a.tg = cdiv(Lr, 128);
        a.tgn = cdiv(Lr, NT > 4 ? 256 : 128);
        a.nb_E = L * a.e_tiles * cdiv(r, NT > 4 ? 256 : 128) * a.se;
        a.reverse = NT <= 4 && L * a.e_tiles >= 128;
        a.nb_G = L > 1 ? a.tg * a.tgn * a.sg : 0;
        a.H = H; a.DP = DP; a.Epart = Epart; a.GGpart = GGpart;
        // tokens not split: the Gram tiles write the two bf16 copies themselves, and E needs no sum either
        a.gg_direct = a.sg == 1; a.GGT = GGT; a.GGsc = GGsc; a.params = io.params; a.PL = D.PL;
        a.ntiles = ntiles; a.B = B; a.C = C; a.cspart = cspart; a.HSpart = HSpart; a.dz = dz;
        a.tile_samp = tile_samp; a.samp_len = samp_len; a.cs = cs; a.Z = Z; a.dzsum = dzsum;
        {
            const int counts[3] = {a.nb_E, a.nb_G, cdiv(Lr, 16)};
            const int classes[3] = {KC_G_TOKRED_E, KC_G_TOKRED_G, KC_G_TOKRED_VEC};
            launch_parts(prof, st, split, k_gtokred<NT>, a, 3, counts, classes, KC_G_TOKRED, TokRedShapes<NT>::kThreadsPerBlock, TokRedShapes<NT>::kLds);
        }
        {
            const int nb_GG = L > 1 && !a.gg_direct ? (Lr / 32) * (Lr / 32) : 0;
            const int64_t e_elems = a.se > 1 ? (int64_t)L * d * r : 0;
            float *E = (float *)(ws + W.g_E);
            if (nb_GG + e_elems > 0)
                PAC_LAUNCH(prof, st, KC_G_GGSUM, k_ggsum, dim3(nb_GG + cdiv(e_elems / 4, 256)), dim3(256), 0, st, L, r, a.sg,
                           GGpart, io.params, D.PL, GGT, GGsc, nb_GG, a.se, e_elems, Epart, E);
        }
        const float *Esum = a.se > 1 ? (const float *)(ws + W.g_E) : Epart;
        PostArgs pa;
        pa.L = L; pa.d = d; pa.r = r; pa.C = C; pa.B = B; pa.se = 1;
        constexpr bool BIG = NT > 4, XW = NT > 8;
        constexpr int NH = PostShapes<64, BIG, XW>::NH;
        constexpr int kFRows = BIG ? 128 : 64, kFCols = BIG ? 256 : 64, kWRows = BIG ? 256 : 64, kWCols = BIG ? 128 : 64;
        constexpr int kPostThreads = BIG ? 512 : 256;
        pa.nb_F = L * cdiv(d, kFRows) * cdiv(r, kFCols); pa.nb_W = L * cdiv(r, kWRows) * cdiv(d, kWCols);
        pa.nb_vec = cdiv(d, (256 / NH) / L) + 1;
        pa.params = io.params; pa.PL = D.PL; pa.WuTs = WuTs; pa.Wds = Wds; pa.GGT = GGT; pa.GGsc = GGsc;
        pa.Epart = Esum; pa.cusum = cusum; pa.cs = cs; pa.Z = Z; pa.dzsum = dzsum; pa.dz = dz; pa.pb = pb;
        pa.grads = io.grads; pa.dlam_part = dlam_part;
        pa.slots = cdiv(d, kFRows) * cdiv(r, kFCols);
        {
            const int counts[3] = {pa.nb_F, pa.nb_W, pa.nb_vec};
            const int classes[3] = {KC_G_POST_F, KC_G_POST_W, KC_G_POST_VEC};
            PAC_HIP_TRY((allow_lds_once<&k_gpost<64, BIG, XW>>(PostShapes<64, BIG, XW>::kLds)));
            PAC_HIP_TRY((allow_lds_once<&k_gpost<32, BIG, XW>>(PostShapes<32, BIG, XW>::kLds)));
            if (r % 64 == 0)
                launch_parts(prof, st, split, k_gpost<64, BIG, XW>, pa, 3, counts, classes, KC_G_POST, kPostThreads, PostShapes<64, BIG, XW>::kLds);
            else
                launch_parts(prof, st, split, k_gpost<32, BIG, XW>, pa, 3, counts, classes, KC_G_POST, kPostThreads, PostShapes<32, BIG, XW>::kLds);
        }
        if (io.defer) { // the optimizer launch that follows does the last two sums
            io.defer->used = true;
            io.defer->loss_part = loss_part; io.defer->B = B; io.defer->loss_out = io.loss_out;
            io.defer->dlam_part = dlam_part; io.defer->slots = pa.slots; io.defer->grads = io.grads;
        } else {
            PAC_LAUNCH(prof, st, KC_G_FINISH, k_gfinish, dim3(1), dim3(64), 0, st, loss_part, B, io.loss_out, dlam_part,
                       pa.slots, L, D.PL, io.grads);
        }
    }
    return hipGetLastError();
}

hipError_t launch_gram_loss_grad(const Dims &D, const WsLayout &W, const BatchMeta &meta, const StepIO &io)
{
    switch (D.r / 32) {
    case 1: return run_gram<1>(D, W, meta, io);
    case 2: return run_gram<2>(D, W, meta, io);
    case 3: return run_gram<3>(D, W, meta, io);
    case 4: return run_gram<4>(D, W, meta, io);
    // above 128 the kernels take r as an argument: one instantiation up to 256, one above (gradient vector part)
    case 5: case 6: case 7: case 8: return run_gram<8>(D, W, meta, io);
    case 10: case 12: case 14: case 16: return run_gram<16>(D, W, meta, io);
    }
    return hipErrorInvalidValue;
}

} // namespace pac
