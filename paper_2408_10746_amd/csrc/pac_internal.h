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
};

struct Dims {
    int32_t L, d, n_max, r, C, B_max;
    int64_t N;
    int32_t cache_dtype; // 0 bf16, 1 f32
    int64_t PL;          // per-layer parameter block
    int64_t P;
    int64_t Mmax;
};

// Kernel classes for per-kernel timing.
enum KClass {
    KC_CACHE_FILL = 0, KC_SETUP, KC_SHADOWS, KC_FWD_DOWN, KC_FWD_UP, KC_POOL, KC_HEAD, KC_HEAD_BWD,
    KC_BWD_DPRE, KC_BWD_WGRAD, KC_BWD_DX, KC_REDUCE, KC_ADAMW, KC_COUNT
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
};

struct AdamArgs {
    float lr, beta1, beta2, eps, wd;
    float bc1, bc2; // 1 - beta^t for the step being applied
};

void plan_workspace(const Dims &D, WsLayout &W);

// Each returns the first HIP error met (hipSuccess otherwise).
hipError_t launch_cache_fill(const Dims &D, void *cache, const void *acts, int acts_dtype,
                             const BatchMeta &meta, hipStream_t st, Profiler *prof);
hipError_t launch_loss_grad(const Dims &D, const WsLayout &W, const BatchMeta &meta, const StepIO &io);
hipError_t launch_adamw(const Dims &D, float *p, float *m, float *v, const float *g,
                        const AdamArgs &a, hipStream_t st, Profiler *prof);

} // namespace pac
