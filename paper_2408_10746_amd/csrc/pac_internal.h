// Host-side plan shared by the C ABI (pac_api.hip) and the kernel launchers
// (pac_kernels.hip).  Nothing here is visible outside the library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <vector>

namespace pac {

constexpr int kMaxBatch = 64;
constexpr int kMaxClasses = 16;

// Passed by value to the set-up kernel: where each batch sample's block lives.
struct BatchMeta {
    int32_t B;
    int32_t M;                       // total valid tokens of the batch
    int32_t tok_start[kMaxBatch + 1]; // first token row of each sample
    int32_t len[kMaxBatch];
    int64_t off[kMaxBatch];          // element offset of the sample's cache block
};

// Byte offsets of every workspace region (all 256-byte aligned).
struct WsLayout {
    int64_t rowoff, rowstride, rowsamp, samp_start, samp_len;
    int64_t Wd, WdT, Wu, WuT; // compute-dtype shadows, [L][d*r] each
    int64_t s_all, pre_all, h_all;
    int64_t ds, dpre;
    int64_t pooled, logits, dz;
    int64_t part, dlam_part;
    int64_t grads;
    int64_t total;
    int32_t splits;     // split count of the token reductions
    int32_t dlam_slots; // workgroups of the dx kernel at the largest batch

    // ---- regions of the Gram-matrix path (bf16, small adapter widths) ----
    int32_t use_gram;   // 0: per-layer kernels; 1: Gram-matrix path, chains in LDS; 2: Gram-matrix path, one chain launch per layer
    int32_t max_tiles;  // 32-row token tiles at the largest batch
    int32_t pairs;      // L (L - 1) / 2 layer pairs k < l
    int32_t se, sg;     // token splits of the E and Gram contractions
    int32_t chain_group; // layers per group of the layer-by-layer chains
    int64_t g_P;        // f32 [Mmax][chain_group * r]: what the layers outside a group contribute to the group's layers
    int64_t g_ghat;     // f32 [B_max][L*r]
    int64_t g_tile_row0, g_tile_rows, g_tile_samp;
    int64_t g_WuTs, g_Wds;          // bf16 [d][L*r] stacked projection copies
    int64_t g_cusum, g_chat, g_V;   // f32 [L+1][d], [L][r], [L*r][C]
    int64_t g_QpN, g_QpT;           // bf16 [pairs][r][r], both orientations (use_gram 2: [L*r][L*r] each)
    int64_t g_QgN, g_QgT;           // use_gram 2: bf16 [groups][g (g - 1) / 2][r][r], the pairs inside a group, fragment-major
    int64_t g_DP;                   // bf16 [Mmax][L*r]
    int64_t g_HSpart, g_cspart;     // f32 [max_tiles][L][r]
    int64_t g_zpart, g_zpb;         // f32 [max_tiles][C], [B_max][C]: shares of the logits
    int64_t g_Z, g_dzsum, g_cs;
    int64_t g_Epart, g_GGpart;      // f32 [se][L][d*r], [sg][L*r][L*r]
    int64_t g_GGT, g_GGsc;          // bf16 [L*r][L*r]
    int64_t g_dlam_part;            // f32 [L][slots]
    int64_t g_samp_tile0, g_loss_part, g_Gp, g_E, g_zero;
    int32_t g_dlam_slots;
};

struct Dims {
    int32_t L, d, n_max, r, C, B_max;
    int64_t N;
    int32_t cache_dtype; // 0 bf16, 1 f32
    int32_t flags;       // PAC_FLAG_* of the configuration
    int64_t PL;          // per-layer parameter block
    int64_t P;
    int64_t Mmax;
};

// Kernel classes for per-kernel timing.
enum KClass {
    KC_CACHE_FILL = 0, KC_SETUP, KC_SHADOWS, KC_FWD_DOWN, KC_FWD_UP, KC_POOL, KC_HEAD, KC_HEAD_BWD,
    KC_BWD_DPRE, KC_BWD_WGRAD, KC_BWD_DX, KC_REDUCE, KC_ADAMW,
    KC_G_PREP, KC_G_PROJ, KC_G_CHAIN_FWD, KC_G_HEAD, KC_G_CHAIN_BWD, KC_G_TOKRED, KC_G_GGSUM, KC_G_POST, KC_G_FINISH,
    // parts of the fused launches, seen only with PAC_FLAG_SPLIT_LAUNCH
    KC_G_PREP_SETUP, KC_G_PREP_COPY, KC_G_PREP_CHAT, KC_G_PREP_V, KC_G_PROJ_U, KC_G_PROJ_Q, KC_G_PROJ_PB,
    KC_G_TOKRED_E, KC_G_TOKRED_G, KC_G_TOKRED_VEC, KC_G_POST_F, KC_G_POST_W, KC_G_POST_VEC,
    // the ladder architecture (pac_ladder.hip)
    KC_L_DOWN, KC_L_ROW, KC_L_LIN, KC_L_ATTN, KC_L_HEAD, KC_L_WGRAD, KC_L_REDUCE,
    KC_COUNT
};

// Optional recorder: a pair of events around each launch.
struct Profiler {
    bool on = false;
    std::vector<hipEvent_t> ev; // begin/end pairs
    std::vector<int> cls;
    hipError_t mark(hipStream_t st, int c, bool begin)
    {
        if (!on) return hipSuccess;
        hipEvent_t e;
        hipError_t r = hipEventCreate(&e);
        if (r != hipSuccess) return r;
        ev.push_back(e);
        if (begin) cls.push_back(c);
        return hipEventRecord(e, st);
    }
};

struct StepIO {
    const void *cache;
    const int32_t *labels;
    const float *params;
    char *ws;
    float *loss_out;
    float *logits_out; // may be null
    float *grads;      // null: forward only
    hipStream_t stream;
    Profiler *prof; // may be null
    // A training step can leave the last two ordered sums (the loss over the samples, the gate
    // gradients over the workgroups' partials) to the optimizer launch.  When `defer` is set and the
    // path that ran supports it, it fills *defer and skips its own last launch.
    struct Deferred *defer = nullptr;
};

struct Deferred {
    bool used = false;
    const float *loss_part = nullptr; // [B]
    int B = 0;
    float *loss_out = nullptr;
    const float *dlam_part = nullptr; // [L][slots]
    int slots = 0;
    float *grads = nullptr; // where the gate gradients go as well
};

struct AdamArgs {
    float lr, beta1, beta2, eps, wd;
    float bc1, bc2;         // 1 - beta^t for the step being applied
    float inv_bc1, inv_bc2; // and their reciprocals
};

void plan_workspace(const Dims &D, WsLayout &W);

// Each returns the first HIP error met (hipSuccess otherwise).
hipError_t launch_cache_fill(const Dims &D, void *cache, const void *acts, int acts_dtype,
                             const BatchMeta &meta, hipStream_t st, Profiler *prof);
hipError_t launch_loss_grad(const Dims &D, const WsLayout &W, const BatchMeta &meta, const StepIO &io);
int gram_path_kind(const Dims &D); // a value of WsLayout::use_gram
void plan_gram_workspace(const Dims &D, WsLayout &W, int64_t &offset);
hipError_t launch_gram_loss_grad(const Dims &D, const WsLayout &W, const BatchMeta &meta, const StepIO &io);
// mixed-precision linear layer on block-wise quantised weights (pac_quant.hip)
// (returns a pac_status value)
int check_dq_linear_args(const void *x, int32_t M, int32_t K, const int8_t *codes, const float *consts, int32_t N,
                            int32_t block, int32_t bits);
hipError_t launch_dq_linear(const void *x, int M, int K, const int8_t *codes, const float *consts, int N, int block,
                            int bits, float *y, void *cache, int cache_f32, int n_max, int layer, const BatchMeta *meta,
                            hipStream_t st);
hipError_t launch_adamw(const Dims &D, float *p, float *m, float *v, float *g,
                        const AdamArgs &a, hipStream_t st, Profiler *prof, const Deferred *fin = nullptr);

} // namespace pac

// The host context behind the opaque pac_ctx of the C ABI.
struct pac_ctx {
    pac::Dims D;
    pac::WsLayout W;
    std::vector<int64_t> off; // element offset of each sample's block, -1 = never filled
    std::vector<int32_t> len;
    int64_t next_free; // elements
    pac::Profiler prof;
};

// Batch description of `B` filled samples (returns a pac_status value; validates ids and state).
int pac_ctx_build_meta(const pac_ctx *ctx, const int64_t *sample_ids, int32_t B, pac::BatchMeta &meta);
