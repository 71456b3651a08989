// C ABI of libpac (declared in include/pac.h): host context, argument
// validation, and the hand-off to the kernel launchers.  All checks run on the
// host before anything is enqueued.
#include "../../include/pac.h"
#include "../../include/pac_quant.h"
#include "../../include/pac_tier.h"
#include "pac_internal.h"

#include <cmath>
#include <mutex>
#include <new>
#include <vector>
#include <algorithm>

using namespace pac;


static const char *const kClassNames[KC_COUNT] = {
    "cache_fill", "setup", "shadows", "fwd_down", "fwd_up", "pool", "head", "head_bwd",
    "bwd_dpre", "bwd_wgrad", "bwd_dx", "reduce", "adamw",
    "g_prep", "g_proj", "g_chain_fwd", "g_head", "g_chain_bwd", "g_tokred", "g_ggsum", "g_post", "g_finish",
    "g_prep.setup", "g_prep.copy", "g_prep.chat", "g_prep.V", "g_proj.U", "g_proj.Q", "g_proj.pb",
    "g_tokred.E", "g_tokred.G", "g_tokred.vec", "g_post.F", "g_post.W", "g_post.vec",
    "l_down", "l_row", "l_lin", "l_attn", "l_head", "l_wgrad", "l_reduce"};

static void drop_events(Profiler &p)
{
    for (hipEvent_t e : p.ev) (void)hipEventDestroy(e);
    p.ev.clear();
    p.cls.clear();
}

// Workspace of pac_adapter_step_static: device memory that belongs to the library's code object, so that no
// call of that entry point allocates.  In host code `scratch` is only a handle for the symbol; the address of
// each GPU's own copy comes from hipGetSymbolAddress, once per device, and only that address is ever handed to a
// kernel.  Nothing in it needs to start at zero: the step's first launch writes every table, counter and zero
// block the later launches read.
static __device__ __align__(256) unsigned char scratch[PAC_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[kMaxDevices]; // per device, null until asked for

static hipError_t static_scratch_address(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

static inline bool aligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
static inline int64_t elem_bytes(int32_t dt) { return dt == PAC_BF16 ? 2 : 4; }

extern "C" {

const char *pac_status_str(pac_status s)
{
    switch (s) {
    case PAC_OK: return "ok";
    case PAC_ERR_NULL: return "null pointer";
    case PAC_ERR_SHAPE: return "bad shape";
    case PAC_ERR_RANGE: return "value out of range";
    case PAC_ERR_ALIGN: return "misaligned pointer";
    case PAC_ERR_UNSUPPORTED: return "unsupported configuration";
    case PAC_ERR_WORKSPACE: return "buffer too small";
    case PAC_ERR_DEVICE: return "HIP runtime error";
    case PAC_ERR_STATE: return "sample not filled or length changed";
    }
    return "unknown status";
}

pac_status pac_create(const pac_config *cfg, pac_ctx **out)
{
    if (!cfg || !out) return PAC_ERR_NULL;
    if (cfg->L < 1 || cfg->d < 1 || cfg->n_max < 1 || cfg->r < 1 || cfg->C < 1 || cfg->B_max < 1 || cfg->N < 1)
        return PAC_ERR_SHAPE;
    if (cfg->cache_dtype != PAC_BF16 && cfg->cache_dtype != PAC_F32) return PAC_ERR_SHAPE;
    if (cfg->flags & ~(PAC_FLAG_PER_LAYER | PAC_FLAG_SPLIT_LAUNCH | PAC_FLAG_LAYER_CHAIN)) return PAC_ERR_SHAPE;
    if (cfg->d % 32 || cfg->r % 32) return PAC_ERR_UNSUPPORTED;
    if (cfg->C > kMaxClasses || cfg->B_max > kMaxBatch) return PAC_ERR_UNSUPPORTED;
    if ((int64_t)cfg->B_max * cfg->n_max > (int64_t)1 << 24) return PAC_ERR_UNSUPPORTED;
    if ((int64_t)cfg->n_max * cfg->d > (int64_t)1 << 30) return PAC_ERR_UNSUPPORTED;
    if (cfg->N > (int64_t)1 << 31) return PAC_ERR_UNSUPPORTED;
    pac_ctx *c = new (std::nothrow) pac_ctx;
    if (!c) return PAC_ERR_WORKSPACE;
    Dims &D = c->D;
    D.L = cfg->L; D.d = cfg->d; D.n_max = cfg->n_max; D.r = cfg->r; D.C = cfg->C; D.B_max = cfg->B_max;
    D.N = cfg->N; D.cache_dtype = cfg->cache_dtype; D.flags = cfg->flags;
    D.PL = 2 * (int64_t)D.d * D.r + D.r + D.d + 1;
    D.P = (int64_t)D.L * D.PL + (int64_t)D.d * D.C + D.C;
    D.Mmax = (int64_t)D.B_max * D.n_max;
    plan_workspace(D, c->W);
    try {
        c->off.assign((size_t)D.N, -1);
        c->len.assign((size_t)D.N, 0);
    } catch (...) {
        delete c;
        return PAC_ERR_WORKSPACE;
    }
    c->next_free = 0;
    *out = c;
    return PAC_OK;
}

void pac_destroy(pac_ctx *ctx)
{
    if (!ctx) return;
    drop_events(ctx->prof);
    delete ctx;
}

const char *pac_profile_class_name(int32_t cls) { return (cls >= 0 && cls < KC_COUNT) ? kClassNames[cls] : nullptr; }

pac_status pac_profile_begin(pac_ctx *ctx)
{
    if (!ctx) return PAC_ERR_NULL;
    drop_events(ctx->prof);
    ctx->prof.on = true;
    return PAC_OK;
}

pac_status pac_profile_end(pac_ctx *ctx, int32_t max_classes, float *ms, int32_t *launches, int32_t *n_classes)
{
    if (!ctx || !ms || !launches || !n_classes) return PAC_ERR_NULL;
    if (!ctx->prof.on) return PAC_ERR_STATE;
    if (max_classes < KC_COUNT) return PAC_ERR_WORKSPACE;
    Profiler &p = ctx->prof;
    p.on = false;
    for (int i = 0; i < KC_COUNT; ++i) { ms[i] = 0.f; launches[i] = 0; }
    pac_status st = PAC_OK;
    for (size_t k = 0; k + 1 < p.ev.size() && k / 2 < p.cls.size(); k += 2) {
        if (hipEventSynchronize(p.ev[k + 1]) != hipSuccess) { st = PAC_ERR_DEVICE; break; }
        float t = 0.f;
        if (hipEventElapsedTime(&t, p.ev[k], p.ev[k + 1]) != hipSuccess) { st = PAC_ERR_DEVICE; break; }
        ms[p.cls[k / 2]] += t;
        launches[p.cls[k / 2]] += 1;
    }
    drop_events(p);
    *n_classes = KC_COUNT;
    return st;
}

int64_t pac_param_count(const pac_ctx *ctx) { return ctx ? ctx->D.P : -1; }

pac_status pac_param_offsets(const pac_ctx *ctx, int32_t layer, int64_t out[5])
{
    if (!ctx || !out) return PAC_ERR_NULL;
    const Dims &D = ctx->D;
    const int64_t dr = (int64_t)D.d * D.r;
    if (layer == -1) {
        out[0] = (int64_t)D.L * D.PL;
        out[1] = out[0] + (int64_t)D.d * D.C;
        out[2] = out[3] = out[4] = -1;
        return PAC_OK;
    }
    if (layer < 0 || layer >= D.L) return PAC_ERR_RANGE;
    const int64_t o = (int64_t)layer * D.PL;
    out[0] = o;
    out[1] = o + dr;
    out[2] = o + dr + D.r;
    out[3] = o + 2 * dr + D.r;
    out[4] = o + 2 * dr + D.r + D.d;
    return PAC_OK;
}

int64_t pac_cache_bytes(const pac_ctx *ctx, const int32_t *lens, int64_t count)
{
    if (!ctx || count < 0) return -1;
    const Dims &D = ctx->D;
    int64_t tokens = 0;
    if (!lens) {
        tokens = count * D.n_max;
    } else {
        for (int64_t i = 0; i < count; ++i) {
            if (lens[i] < 1 || lens[i] > D.n_max) return -1;
            tokens += lens[i];
        }
    }
    return tokens * D.d * D.L * elem_bytes(D.cache_dtype);
}

int64_t pac_workspace_bytes(const pac_ctx *ctx) { return ctx ? ctx->W.total : -1; }

int32_t pac_step_path(const pac_ctx *ctx) { return ctx ? ctx->W.use_gram : -1; }

pac_status pac_cache_lookup(const pac_ctx *ctx, int64_t sample_id, int64_t *offset_elems, int32_t *len)
{
    if (!ctx || !offset_elems || !len) return PAC_ERR_NULL;
    if (sample_id < 0 || sample_id >= ctx->D.N) return PAC_ERR_RANGE;
    if (ctx->off[(size_t)sample_id] < 0) return PAC_ERR_STATE;
    *offset_elems = ctx->off[(size_t)sample_id];
    *len = ctx->len[(size_t)sample_id];
    return PAC_OK;
}

} // extern "C"

// Where the blocks of `count` samples go: a known sample keeps its block (and must keep its length), a new one is
// appended after the blocks placed so far.  Validates everything and touches nothing; commit_samples records the result.
static pac_status place_samples(const pac_ctx *ctx, int64_t cache_bytes, const int64_t *sample_ids, int32_t count,
                                const int32_t *lens, std::vector<int64_t> &new_off, int64_t &next_out)
{
    const Dims &D = ctx->D;
    const int64_t eb = elem_bytes(D.cache_dtype);
    new_off.assign((size_t)count, 0);
    std::vector<int64_t> sorted(sample_ids, sample_ids + count);
    std::sort(sorted.begin(), sorted.end());
    for (int32_t i = 0; i + 1 < count; ++i)
        if (sorted[(size_t)i] == sorted[(size_t)i + 1]) return PAC_ERR_RANGE;
    int64_t next = ctx->next_free;
    for (int32_t i = 0; i < count; ++i) {
        const int64_t id = sample_ids[i];
        if (id < 0 || id >= D.N) return PAC_ERR_RANGE;
        const int32_t ln = lens ? lens[i] : D.n_max;
        if (ln < 1 || ln > D.n_max) return PAC_ERR_RANGE;
        if (ctx->off[(size_t)id] >= 0) {
            if (ctx->len[(size_t)id] != ln) return PAC_ERR_STATE;
            new_off[(size_t)i] = ctx->off[(size_t)id];
        } else {
            new_off[(size_t)i] = next;
            next += (int64_t)D.L * ln * D.d;
        }
    }
    if (next * eb > cache_bytes) return PAC_ERR_WORKSPACE;
    next_out = next;
    return PAC_OK;
}

static void commit_samples(pac_ctx *ctx, const int64_t *sample_ids, int32_t count, const int32_t *lens,
                           const std::vector<int64_t> &new_off, int64_t next)
{
    for (int32_t i = 0; i < count; ++i) {
        ctx->off[(size_t)sample_ids[i]] = new_off[(size_t)i];
        ctx->len[(size_t)sample_ids[i]] = lens ? lens[i] : ctx->D.n_max;
    }
    ctx->next_free = next;
}

extern "C" {

pac_status pac_dequant_linear_to_cache(pac_ctx *ctx, void *cache, int64_t cache_bytes, const int64_t *sample_ids,
                                       int32_t count, const int32_t *lens, int32_t layer, const void *x, int32_t K,
                                       const int8_t *codes, const float *consts, int32_t block, int32_t bits,
                                       void *hip_stream)
{
    if (!ctx || !cache || !sample_ids) return PAC_ERR_NULL;
    if (count < 0) return PAC_ERR_RANGE;
    const Dims &D = ctx->D;
    if (layer < 0 || layer >= D.L) return PAC_ERR_RANGE;
    if (!aligned(cache, 256)) return PAC_ERR_ALIGN;
    if (count == 0) return PAC_OK;
    if ((int64_t)count * D.n_max > (int64_t)1 << 30) return PAC_ERR_RANGE;
    pac_status s = (pac_status)check_dq_linear_args(x, count * D.n_max, K, codes, consts, D.d, block, bits);
    if (s != PAC_OK) return s;
    std::vector<int64_t> new_off;
    int64_t next = 0;
    s = place_samples(ctx, cache_bytes, sample_ids, count, lens, new_off, next);
    if (s != PAC_OK) return s;
    (void)hipGetLastError();
    const int64_t per_sample_in = (int64_t)D.n_max * K * 2;
    for (int32_t base = 0; base < count; base += kMaxBatch) {
        BatchMeta meta{};
        meta.B = std::min<int32_t>(kMaxBatch, count - base);
        meta.M = 0;
        for (int32_t i = 0; i < meta.B; ++i) {
            meta.len[i] = lens ? lens[base + i] : D.n_max;
            meta.off[i] = new_off[(size_t)(base + i)];
            meta.tok_start[i] = meta.M;
            meta.M += meta.len[i];
        }
        meta.tok_start[meta.B] = meta.M;
        if (launch_dq_linear(static_cast<const char *>(x) + (int64_t)base * per_sample_in, meta.B * D.n_max, K, codes, consts,
                             D.d, block, bits, nullptr, cache, D.cache_dtype == PAC_F32, D.n_max, layer, &meta,
                             static_cast<hipStream_t>(hip_stream)) != hipSuccess)
            return PAC_ERR_DEVICE;
    }
    commit_samples(ctx, sample_ids, count, lens, new_off, next);
    return PAC_OK;
}

pac_status pac_cache_fill(pac_ctx *ctx, void *cache, int64_t cache_bytes, const int64_t *sample_ids, int32_t count,
                          const void *acts, int32_t acts_dtype, const int32_t *lens, void *hip_stream)
{
    if (!ctx || !cache || !sample_ids || !acts) return PAC_ERR_NULL;
    if (count < 0) return PAC_ERR_RANGE;
    if (acts_dtype != PAC_BF16 && acts_dtype != PAC_F32) return PAC_ERR_SHAPE;
    if (!aligned(cache, 256) || !aligned(acts, 16)) return PAC_ERR_ALIGN;
    if (count == 0) return PAC_OK;
    // The launches below are checked with hipGetLastError, which also reports an error left behind
    // by an earlier, unrelated HIP call of this thread (another library's probe of a host pointer,
    // say): drop such a leftover first.
    (void)hipGetLastError();
    const Dims &D = ctx->D;
    const int64_t eb = elem_bytes(D.cache_dtype);
    std::vector<int64_t> new_off;
    int64_t next = 0;
    pac_status ps = place_samples(ctx, cache_bytes, sample_ids, count, lens, new_off, next);
    if (ps != PAC_OK) return ps;
    // enqueue in groups the kernel argument block can describe
    const int64_t per_sample_in = (int64_t)D.L * D.n_max * D.d * elem_bytes(acts_dtype);
    for (int32_t base = 0; base < count; base += kMaxBatch) {
        BatchMeta meta{};
        meta.B = std::min<int32_t>(kMaxBatch, count - base);
        meta.M = 0;
        for (int32_t i = 0; i < meta.B; ++i) {
            meta.len[i] = lens ? lens[base + i] : D.n_max;
            meta.off[i] = new_off[(size_t)(base + i)];
            meta.tok_start[i] = meta.M;
            meta.M += meta.len[i];
        }
        meta.tok_start[meta.B] = meta.M;
        hipError_t e = launch_cache_fill(D, cache, static_cast<const char *>(acts) + (int64_t)base * per_sample_in,
                                         acts_dtype, meta, static_cast<hipStream_t>(hip_stream),
                                         ctx->prof.on ? &ctx->prof : nullptr);
        if (e != hipSuccess) return PAC_ERR_DEVICE;
    }
    commit_samples(ctx, sample_ids, count, lens, new_off, next);
    return PAC_OK;
}

// packed: the blocks sit back to back in batch order (a staged window) instead of at their recorded offsets
static pac_status build_meta(const pac_ctx *ctx, const int64_t *sample_ids, int32_t B, BatchMeta &meta, bool packed = false)
{
    const Dims &D = ctx->D;
    if (B < 1 || B > D.B_max) return PAC_ERR_RANGE;
    meta.B = B;
    meta.M = 0;
    for (int32_t i = 0; i < B; ++i) {
        const int64_t id = sample_ids[i];
        if (id < 0 || id >= D.N) return PAC_ERR_RANGE;
        if (ctx->off[(size_t)id] < 0) return PAC_ERR_STATE;
        meta.off[i] = packed ? (int64_t)D.L * meta.M * D.d : ctx->off[(size_t)id];
        meta.len[i] = ctx->len[(size_t)id];
        meta.tok_start[i] = meta.M;
        meta.M += meta.len[i];
    }
    meta.tok_start[B] = meta.M;
    for (int32_t i = B; i < kMaxBatch; ++i) {
        meta.off[i] = 0;
        meta.len[i] = 0;
        meta.tok_start[i + 1] = meta.M;
    }
    return PAC_OK;
}

static pac_status check_common(const pac_ctx *ctx, const void *cache, const int64_t *sample_ids,
                               const int32_t *labels, const float *params, const void *workspace,
                               int64_t workspace_bytes, const float *loss_out)
{
    if (!ctx || !cache || !sample_ids || !labels || !params || !workspace || !loss_out) return PAC_ERR_NULL;
    if (!aligned(cache, 256) || !aligned(workspace, 256) || !aligned(params, 4) || !aligned(labels, 4) ||
        !aligned(loss_out, 4))
        return PAC_ERR_ALIGN;
    if (workspace_bytes < ctx->W.total) return PAC_ERR_WORKSPACE;
    return PAC_OK;
}

static pac_status loss_grad_impl(pac_ctx *ctx, const void *cache, const int64_t *sample_ids, int32_t B,
                                 const int32_t *labels, const float *params, void *workspace,
                                 int64_t workspace_bytes, float *loss_out, float *logits_out, float *grads_out,
                                 void *hip_stream, bool packed)
{
    pac_status s = check_common(ctx, cache, sample_ids, labels, params, workspace, workspace_bytes, loss_out);
    if (s != PAC_OK) return s;
    if ((logits_out && !aligned(logits_out, 4)) || (grads_out && !aligned(grads_out, 4))) return PAC_ERR_ALIGN;
    BatchMeta meta;
    s = build_meta(ctx, sample_ids, B, meta, packed);
    if (s != PAC_OK) return s;
    StepIO io{cache, labels, params, static_cast<char *>(workspace), loss_out, logits_out, grads_out,
              static_cast<hipStream_t>(hip_stream), ctx->prof.on ? &ctx->prof : nullptr};
    (void)hipGetLastError(); // drop an error left behind by an unrelated earlier call (see pac_cache_fill)
    return launch_loss_grad(ctx->D, ctx->W, meta, io) == hipSuccess ? PAC_OK : PAC_ERR_DEVICE;
}

pac_status pac_adapter_loss_grad(pac_ctx *ctx, const void *cache, const int64_t *sample_ids, int32_t B,
                                 const int32_t *labels, const float *params, void *workspace,
                                 int64_t workspace_bytes, float *loss_out, float *logits_out, float *grads_out,
                                 void *hip_stream)
{
    return loss_grad_impl(ctx, cache, sample_ids, B, labels, params, workspace, workspace_bytes, loss_out, logits_out,
                          grads_out, hip_stream, false);
}

pac_status pac_adapter_loss_grad_staged(pac_ctx *ctx, const void *window, const int64_t *sample_ids, int32_t B,
                                        const int32_t *labels, const float *params, void *workspace,
                                        int64_t workspace_bytes, float *loss_out, float *logits_out, float *grads_out,
                                        void *hip_stream)
{
    return loss_grad_impl(ctx, window, sample_ids, B, labels, params, workspace, workspace_bytes, loss_out, logits_out,
                          grads_out, hip_stream, true);
}

// The step behind pac_adapter_step and pac_adapter_step_static: forward, loss, backward, AdamW on `workspace`.
static pac_status step_on_workspace(pac_ctx *ctx, const void *cache, const int64_t *sample_ids, int32_t B,
                                    const int32_t *labels, float *params, float *m, float *v, int64_t *step,
                                    const pac_adamw *hp, void *workspace, int64_t workspace_bytes, float *loss_out,
                                    float *grads_out, void *hip_stream, bool may_profile, bool packed = false)
{
    pac_status s = check_common(ctx, cache, sample_ids, labels, params, workspace, workspace_bytes, loss_out);
    if (s != PAC_OK) return s;
    if (!m || !v || !step || !hp) return PAC_ERR_NULL;
    if (!aligned(m, 4) || !aligned(v, 4) || (grads_out && !aligned(grads_out, 4))) return PAC_ERR_ALIGN;
    if (*step < 0) return PAC_ERR_RANGE;
    if (!(hp->beta1 >= 0.f && hp->beta1 < 1.f) || !(hp->beta2 >= 0.f && hp->beta2 < 1.f) || !(hp->eps >= 0.f) ||
        !(hp->lr >= 0.f) || !(hp->weight_decay >= 0.f))
        return PAC_ERR_RANGE;
    BatchMeta meta;
    s = build_meta(ctx, sample_ids, B, meta, packed);
    if (s != PAC_OK) return s;
    char *ws = static_cast<char *>(workspace);
    float *grads = grads_out ? grads_out : reinterpret_cast<float *>(ws + ctx->W.grads);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    Profiler *prof = (may_profile && ctx->prof.on) ? &ctx->prof : nullptr;
    StepIO io{cache, labels, params, ws, loss_out, nullptr, grads, st, prof};
    Deferred fin;
    io.defer = &fin;
    (void)hipGetLastError(); // drop an error left behind by an unrelated earlier call (see pac_cache_fill)
    if (launch_loss_grad(ctx->D, ctx->W, meta, io) != hipSuccess) return PAC_ERR_DEVICE;
    const int64_t t = *step + 1;
    AdamArgs a;
    a.lr = hp->lr; a.beta1 = hp->beta1; a.beta2 = hp->beta2; a.eps = hp->eps; a.wd = hp->weight_decay;
    a.bc1 = (float)(1.0 - pow((double)hp->beta1, (double)t));
    a.bc2 = (float)(1.0 - pow((double)hp->beta2, (double)t));
    a.inv_bc1 = (float)(1.0 / (1.0 - pow((double)hp->beta1, (double)t)));
    a.inv_bc2 = (float)(1.0 / (1.0 - pow((double)hp->beta2, (double)t)));
    if (launch_adamw(ctx->D, params, m, v, grads, a, st, prof, &fin) != hipSuccess) return PAC_ERR_DEVICE;
    *step = t;
    return PAC_OK;
}

pac_status pac_adapter_step(pac_ctx *ctx, const void *cache, const int64_t *sample_ids, int32_t B,
                            const int32_t *labels, float *params, float *m, float *v, int64_t *step,
                            const pac_adamw *hp, void *workspace, int64_t workspace_bytes, float *loss_out,
                            float *grads_out, void *hip_stream)
{
    return step_on_workspace(ctx, cache, sample_ids, B, labels, params, m, v, step, hp, workspace, workspace_bytes,
                             loss_out, grads_out, hip_stream, true);
}

pac_status pac_adapter_step_staged(pac_ctx *ctx, const void *window, const int64_t *sample_ids, int32_t B,
                                   const int32_t *labels, float *params, float *m, float *v, int64_t *step,
                                   const pac_adamw *hp, void *workspace, int64_t workspace_bytes, float *loss_out,
                                   float *grads_out, void *hip_stream)
{
    return step_on_workspace(ctx, window, sample_ids, B, labels, params, m, v, step, hp, workspace, workspace_bytes,
                             loss_out, grads_out, hip_stream, true, true);
}

int64_t pac_tier_window_bytes(const pac_ctx *ctx)
{
    if (!ctx) return -1;
    const Dims &D = ctx->D;
    return (int64_t)D.L * D.Mmax * D.d * elem_bytes(D.cache_dtype);
}

pac_status pac_tier_stage(const pac_ctx *ctx, const void *host_cache, const int64_t *sample_ids, int32_t B, void *window,
                          int64_t window_bytes, void *copy_stream)
{
    if (!ctx || !host_cache || !sample_ids || !window) return PAC_ERR_NULL;
    if (!aligned(host_cache, 256) || !aligned(window, 256)) return PAC_ERR_ALIGN;
    BatchMeta meta;
    pac_status s = build_meta(ctx, sample_ids, B, meta, true);
    if (s != PAC_OK) return s;
    const Dims &D = ctx->D;
    const int64_t eb = elem_bytes(D.cache_dtype);
    if ((int64_t)D.L * meta.M * D.d * eb > window_bytes) return PAC_ERR_WORKSPACE;
    (void)hipGetLastError();
    for (int32_t i = 0; i < B; ++i) {
        const int64_t bytes = (int64_t)D.L * meta.len[i] * D.d * eb;
        if (hipMemcpyAsync(static_cast<char *>(window) + meta.off[i] * eb,
                           static_cast<const char *>(host_cache) + ctx->off[(size_t)sample_ids[i]] * eb, (size_t)bytes,
                           hipMemcpyHostToDevice, static_cast<hipStream_t>(copy_stream)) != hipSuccess)
            return PAC_ERR_DEVICE;
    }
    return PAC_OK;
}

pac_status pac_tier_fill(pac_ctx *ctx, void *host_cache, int64_t host_bytes, const int64_t *sample_ids, int32_t count,
                         const void *acts, int32_t acts_dtype, const int32_t *lens, void *window, int64_t window_bytes,
                         void *hip_stream)
{
    if (!ctx || !host_cache || !sample_ids || !acts || !window) return PAC_ERR_NULL;
    if (count < 0 || count > ctx->D.B_max) return PAC_ERR_RANGE;
    if (acts_dtype != PAC_BF16 && acts_dtype != PAC_F32) return PAC_ERR_SHAPE;
    if (!aligned(host_cache, 256) || !aligned(window, 256) || !aligned(acts, 16)) return PAC_ERR_ALIGN;
    if (count == 0) return PAC_OK;
    const Dims &D = ctx->D;
    const int64_t eb = elem_bytes(D.cache_dtype);
    std::vector<int64_t> new_off;
    int64_t next = 0;
    pac_status s = place_samples(ctx, host_bytes, sample_ids, count, lens, new_off, next);
    if (s != PAC_OK) return s;
    BatchMeta meta{};
    meta.B = count;
    meta.M = 0;
    for (int32_t i = 0; i < count; ++i) {
        meta.len[i] = lens ? lens[i] : D.n_max;
        meta.off[i] = (int64_t)D.L * meta.M * D.d; // packed in the window
        meta.tok_start[i] = meta.M;
        meta.M += meta.len[i];
    }
    meta.tok_start[count] = meta.M;
    if ((int64_t)D.L * meta.M * D.d * eb > window_bytes) return PAC_ERR_WORKSPACE;
    (void)hipGetLastError();
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (launch_cache_fill(D, window, acts, acts_dtype, meta, st, nullptr) != hipSuccess) return PAC_ERR_DEVICE;
    for (int32_t i = 0; i < count; ++i) {
        const int64_t bytes = (int64_t)D.L * meta.len[i] * D.d * eb;
        if (hipMemcpyAsync(static_cast<char *>(host_cache) + new_off[(size_t)i] * eb,
                           static_cast<const char *>(window) + meta.off[i] * eb, (size_t)bytes, hipMemcpyDeviceToHost,
                           st) != hipSuccess)
            return PAC_ERR_DEVICE;
    }
    commit_samples(ctx, sample_ids, count, lens, new_off, next);
    return PAC_OK;
}

pac_status pac_adapter_step_static(pac_ctx *ctx, const void *cache, const int64_t *sample_ids, int32_t B,
                                   const int32_t *labels, float *params, float *m, float *v, int64_t *step,
                                   const pac_adamw *hp, float *loss_out, float *grads_out, void *hip_stream)
{
    if (!ctx) return PAC_ERR_NULL;
    if (ctx->W.total > PAC_STATIC_WORKSPACE_BYTES) return PAC_ERR_WORKSPACE;
    void *ws = nullptr;
    if (static_scratch_address(&ws) != hipSuccess || !ws) return PAC_ERR_DEVICE;
    return step_on_workspace(ctx, cache, sample_ids, B, labels, params, m, v, step, hp, ws, PAC_STATIC_WORKSPACE_BYTES,
                             loss_out, grads_out, hip_stream, false);
}

} // extern "C"

int pac_ctx_build_meta(const pac_ctx *ctx, const int64_t *sample_ids, int32_t B, pac::BatchMeta &meta)
{
    return (int)build_meta(ctx, sample_ids, B, meta, false);
}
