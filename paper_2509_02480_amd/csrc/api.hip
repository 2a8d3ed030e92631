// C ABI of libmlpo: errors, per-kernel timing, argument checking, per-step scalars and the entry points
// of the resident path.  The tiered pipeline is in pipeline.hip.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stddef.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "mlpo_internal.h"

namespace mlpo {

// ---- errors -----------------------------------------------------------------
static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

// ---- device ------------------------------------------------------------
int num_cus() {
    static std::mutex mu;
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return -1;
    std::lock_guard<std::mutex> lk(mu);
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return -1;
        cached[dev] = n;
    }
    return cached[dev];
}

// ---- per-kernel timing ---------------------------------------------------------------
namespace {
struct TimedLaunch {
    hipEvent_t start, stop;
};
struct TimingState {
    std::mutex mu;
    bool enabled = false;
    std::vector<TimedLaunch> rec[kTimedKinds];
    std::vector<TimedLaunch> pool;
};
TimingState& timing() {
    static TimingState t;
    return t;
}
constexpr size_t kMaxTimed = 16384;
}  // namespace

bool timing_enabled() { return timing().enabled; }

// Takes an event pair from the pool (or creates one); the caller holds the lock.
static bool timing_take_locked(TimingState& t, TimedLaunch* e) {
    if (!t.pool.empty()) {
        *e = t.pool.back();
        t.pool.pop_back();
        return true;
    }
    if (hipEventCreate(&e->start) != hipSuccess) return false;
    if (hipEventCreate(&e->stop) != hipSuccess) {
        (void)hipEventDestroy(e->start);
        return false;
    }
    return true;
}

bool timing_acquire(int which, hipEvent_t* start, hipEvent_t* stop) {
    TimingState& t = timing();
    std::lock_guard<std::mutex> lk(t.mu);
    if (!t.enabled || which < 0 || which >= kTimedKinds || t.rec[which].size() >= kMaxTimed) return false;
    TimedLaunch e;
    if (!timing_take_locked(t, &e)) return false;
    t.rec[which].push_back(e);
    *start = e.start;
    *stop = e.stop;
    return true;
}

// Both pairs or neither: a pair that is listed but never recorded would make mlpo_kernel_times wait for nothing.
bool timing_acquire_two(int which_a, hipEvent_t* a0, hipEvent_t* a1, int which_b, hipEvent_t* b0, hipEvent_t* b1) {
    TimingState& t = timing();
    std::lock_guard<std::mutex> lk(t.mu);
    if (!t.enabled || which_a < 0 || which_a >= kTimedKinds || which_b < 0 || which_b >= kTimedKinds ||
        which_a == which_b || t.rec[which_a].size() >= kMaxTimed || t.rec[which_b].size() >= kMaxTimed)
        return false;
    TimedLaunch ea, eb;
    if (!timing_take_locked(t, &ea)) return false;
    if (!timing_take_locked(t, &eb)) {
        t.pool.push_back(ea);
        return false;
    }
    t.rec[which_a].push_back(ea);
    t.rec[which_b].push_back(eb);
    *a0 = ea.start;
    *a1 = ea.stop;
    *b0 = eb.start;
    *b1 = eb.stop;
    return true;
}

static void timing_set(bool on) {
    TimingState& t = timing();
    std::lock_guard<std::mutex> lk(t.mu);
    for (auto& r : t.rec) {
        for (auto& e : r) t.pool.push_back(e);
        r.clear();
    }
    t.enabled = on;
}

// ---- hyper-parameters -------------------------------------------------------------
int validate_hparams(const mlpo_adamw_hparams* hp, int64_t step) {
    if (hp == nullptr) return fail(MLPO_EINVAL, "hparams is NULL");
    if (step < 1) return fail(MLPO_EINVAL, "step must be >= 1 (got %lld)", (long long)step);
    if (!(isfinite(hp->lr) && hp->lr >= 0.0f)) return fail(MLPO_EINVAL, "lr must be finite and >= 0");
    if (!(hp->beta1 >= 0.0f && hp->beta1 < 1.0f)) return fail(MLPO_EINVAL, "beta1 must be in [0, 1)");
    if (!(hp->beta2 >= 0.0f && hp->beta2 < 1.0f)) return fail(MLPO_EINVAL, "beta2 must be in [0, 1)");
    if (!(isfinite(hp->eps) && hp->eps >= 0.0f)) return fail(MLPO_EINVAL, "eps must be finite and >= 0");
    if (!(isfinite(hp->weight_decay) && hp->weight_decay >= 0.0f))
        return fail(MLPO_EINVAL, "weight_decay must be finite and >= 0");
    if (hp->l2_mode != 0 && hp->l2_mode != 1) return fail(MLPO_EINVAL, "l2_mode must be 0 or 1 (got %d)", hp->l2_mode);
    return MLPO_OK;
}

// The scalars of one step: exact expressions evaluated in double, then one rounding to fp32 each.
AdamwConsts make_consts(const mlpo_adamw_hparams& hp, int64_t step, int32_t half) {
    const double beta1 = hp.beta1, beta2 = hp.beta2;
    double corr1 = 1.0, corr2 = 1.0;
    if (hp.bias_correction != 0) {
        corr1 -= pow(beta1, (double)step);
        corr2 -= pow(beta2, (double)step);
    }
    AdamwConsts c;
    c.beta1 = hp.beta1;
    c.beta2 = hp.beta2;
    c.omb1 = (float)(1.0 - beta1);
    c.omb2 = (float)(1.0 - beta2);
    c.eps = hp.eps;
    c.step_size = (float)((double)hp.lr / corr1);
    c.sqbc2 = (float)sqrt(corr2);
    c.decay = (float)(1.0 - (double)hp.lr * (double)hp.weight_decay);
    c.l2 = 0.0f;
    c.l2_mode = hp.l2_mode;
    if (hp.l2_mode != 0) {  // the decay acts through the gradient only
        c.decay = 1.0f;
        c.l2 = hp.weight_decay;
    }
    c.half = half;
    return c;
}

// ---- subgroup checks ----------------------------------------------------------------
bool misaligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

uint64_t round_up(uint64_t x, uint64_t to) { return (x + to - 1) / to * to; }

int32_t table_half_format(const mlpo_subgroup* sg, int32_t n_sg) {
    return n_sg > 0 ? sg[0].half_format : MLPO_HALF_BF16;
}

int validate_subgroups(const mlpo_subgroup* sg, int32_t n_sg, bool grads_only, int allow_host) {
    if (n_sg < 0) return fail(MLPO_EINVAL, "n_sg is negative");
    if (n_sg > 0 && sg == nullptr) return fail(MLPO_EINVAL, "subgroup array is NULL");
    for (int32_t i = 0; i < n_sg; ++i) {
        const mlpo_subgroup& s = sg[i];
        if (s.half_format != MLPO_HALF_BF16 && s.half_format != MLPO_HALF_FP16)
            return fail(MLPO_EINVAL, "subgroup %d: unknown half format %d", i, s.half_format);
        if (s.half_format != sg[0].half_format)
            return fail(MLPO_EINVAL, "subgroup %d: all subgroups of a call must share one half format", i);
        if (s.lead < 0 || s.lead >= 1024 || s.lead % 4 != 0)
            return fail(MLPO_EINVAL, "subgroup %d: lead must be a multiple of 4 in 0..1020 (got %d)", i, s.lead);
        if (s.n > ((uint64_t)1 << 48)) return fail(MLPO_EINVAL, "subgroup %d: n is implausibly large", i);
        if (s.n != 0 && s.g == nullptr) return fail(MLPO_EINVAL, "subgroup %d: g is NULL", i);
        if (misaligned(s.g, 2)) return fail(MLPO_EINVAL, "subgroup %d: g is not 2-byte aligned", i);
        if (grads_only) continue;
        if (s.tier != MLPO_TIER_HBM && !host_tier(s.tier) && s.tier != MLPO_TIER_FILE)
            return fail(MLPO_EINVAL, "subgroup %d: unknown tier %d", i, s.tier);
        if (s.lead != 0 && (s.tier != MLPO_TIER_HBM || s.tile_elems <= 0))
            return fail(MLPO_EINVAL, "subgroup %d: lead is for HBM-tier subgroups in the tiled layout", i);
        if (host_tier(s.tier) && allow_host < 1)
            return fail(MLPO_EINVAL, "subgroup %d is host-tier: use mlpo_stream_update", i);
        if (s.tier == MLPO_TIER_FILE) {
            if (allow_host < 2) return fail(MLPO_EINVAL, "subgroup %d is file-tier: use mlpo_stream_update", i);
            if (s.p != nullptr || s.m != nullptr || s.v != nullptr)
                return fail(MLPO_EINVAL, "subgroup %d: a file-tier subgroup has no p/m/v pointers", i);
            if (s.tile_elems <= 0 || s.tile_elems % 1024 != 0)
                return fail(MLPO_EINVAL, "subgroup %d: a file-tier subgroup needs the tiled layout", i);
            if (s.n != 0 && s.p16 == nullptr) return fail(MLPO_EINVAL, "subgroup %d: p16 is NULL", i);
            if (misaligned(s.g, 8) || misaligned(s.p16, 8))
                return fail(MLPO_EINVAL, "subgroup %d: tiled state needs 8-byte aligned g and p16", i);
            continue;
        }
        if (s.n != 0 && (s.p == nullptr || s.m == nullptr || s.v == nullptr || s.p16 == nullptr))
            return fail(MLPO_EINVAL, "subgroup %d: NULL state pointer", i);
        if (misaligned(s.p, 4) || misaligned(s.m, 4) || misaligned(s.v, 4))
            return fail(MLPO_EINVAL, "subgroup %d: p/m/v not 4-byte aligned", i);
        if (misaligned(s.p16, 2)) return fail(MLPO_EINVAL, "subgroup %d: p16 is not 2-byte aligned", i);
        if (s.tile_elems < 0 || s.tile_elems % 1024 != 0)
            return fail(MLPO_EINVAL, "subgroup %d: tile_elems must be 0 or a positive multiple of 1024", i);
        if (s.tile_elems > 0 && s.n != 0) {
            if (misaligned(s.p, 256)) return fail(MLPO_EINVAL, "subgroup %d: tiled state must be 256-byte aligned", i);
            if (s.m != s.p + s.tile_elems || s.v != s.p + 2 * (ptrdiff_t)s.tile_elems)
                return fail(MLPO_EINVAL, "subgroup %d: tiled state needs m == p + T and v == p + 2T", i);
            if (misaligned(s.g, 8) || misaligned(s.p16, 8))
                return fail(MLPO_EINVAL, "subgroup %d: tiled state needs 8-byte aligned g and p16", i);
        }
    }
    return MLPO_OK;
}

static int check_accumulate(uint16_t* acc, const uint16_t* g, uint64_t n, int32_t blocks, int32_t half) {
    if (half != MLPO_HALF_BF16 && half != MLPO_HALF_FP16) return fail(MLPO_EINVAL, "unknown half format %d", half);
    if (acc == nullptr || g == nullptr) return fail(MLPO_EINVAL, "acc or g is NULL");
    if (misaligned(acc, 2) || misaligned(g, 2)) return fail(MLPO_EINVAL, "acc or g not 2-byte aligned");
    if (n > (1ull << 41)) return fail(MLPO_EINVAL, "n too large (at most 2^41 elements per call)");
    if (blocks < 0 || blocks > 4096) return fail(MLPO_EINVAL, "blocks must be 0..4096 (got %d)", blocks);
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(acc), g0 = reinterpret_cast<uintptr_t>(g);
    if (a0 < g0 + 2 * n && g0 < a0 + 2 * n) return fail(MLPO_EINVAL, "acc and g overlap");
    return MLPO_OK;
}

static int check_norm_workspace(void* workspace, size_t workspace_bytes) {
    if (workspace == nullptr || misaligned(workspace, 256))
        return fail(MLPO_EINVAL, "workspace is NULL or not 256-byte aligned");
    if (workspace_bytes < grad_norm_workspace_bytes())
        return fail(MLPO_ENOMEM, "workspace has %zu bytes, %zu needed", workspace_bytes, grad_norm_workspace_bytes());
    return MLPO_OK;
}

}  // namespace mlpo

using namespace mlpo;

extern "C" {

const char* mlpo_last_error(void) { return g_err; }

int32_t mlpo_version(void) { return 100; }

size_t mlpo_norm_workspace_bytes(void) { return grad_norm_workspace_bytes(); }

int mlpo_kernel_timing(int32_t on) {
    timing_set(on != 0);
    return MLPO_OK;
}

int mlpo_kernel_times(int32_t which, float* ms, int32_t cap, int32_t* count) {
    if (which < 0 || which >= kTimedKinds) return fail(MLPO_EINVAL, "which must be 0..%d", kTimedKinds - 1);
    if (count == nullptr || cap < 0 || (cap > 0 && ms == nullptr)) return fail(MLPO_EINVAL, "bad output arguments");
    TimingState& t = timing();
    std::lock_guard<std::mutex> lk(t.mu);
    int32_t n = 0;
    for (auto& e : t.rec[which]) {
        if (n < cap) {
            MLPO_HIP(hipEventSynchronize(e.stop));
            MLPO_HIP(hipEventElapsedTime(&ms[n], e.start, e.stop));
            ++n;
        }
        t.pool.push_back(e);
    }
    t.rec[which].clear();
    *count = n;
    return MLPO_OK;
}

int mlpo_grad_unscale_norm(const mlpo_subgroup* sg, int32_t n_sg, float inv_scale, float max_norm, void* workspace,
                           size_t workspace_bytes, mlpo_step_scalars* out, void* stream) {
    int rc = validate_subgroups(sg, n_sg, /*grads_only=*/true, 1);
    if (rc != MLPO_OK) return rc;
    if (!(isfinite(inv_scale) && inv_scale > 0.0f)) return fail(MLPO_EINVAL, "inv_scale must be finite and > 0");
    if (isnan(max_norm)) return fail(MLPO_EINVAL, "max_norm is NaN");
    rc = check_norm_workspace(workspace, workspace_bytes);
    if (rc != MLPO_OK) return rc;
    if (out == nullptr || misaligned(out, 16)) return fail(MLPO_EINVAL, "out is NULL or not 16-byte aligned");
    return launch_grad_norm(sg, n_sg, inv_scale, max_norm, workspace, out, static_cast<hipStream_t>(stream));
}

int mlpo_grad_unscale_norm_keep(const mlpo_subgroup* sg, int32_t n_sg, uint16_t* const* keep, float inv_scale,
                                float max_norm, void* workspace, size_t workspace_bytes, mlpo_step_scalars* out,
                                void* stream) {
    int rc = validate_subgroups(sg, n_sg, /*grads_only=*/true, 1);
    if (rc != MLPO_OK) return rc;
    if (n_sg > 0 && keep == nullptr) return fail(MLPO_EINVAL, "keep is NULL");
    for (int32_t i = 0; i < n_sg; ++i) {
        if (keep[i] == nullptr || sg[i].n == 0) continue;
        const uintptr_t a = reinterpret_cast<uintptr_t>(keep[i]), g = reinterpret_cast<uintptr_t>(sg[i].g);
        if (((a ^ g) & 15u) != 0)
            return fail(MLPO_EINVAL, "subgroup %d: the copy and the gradients must agree modulo 16 bytes", i);
        if (a < g + 2 * sg[i].n && g < a + 2 * sg[i].n)
            return fail(MLPO_EINVAL, "subgroup %d: the copy overlaps the gradients", i);
    }
    if (!(isfinite(inv_scale) && inv_scale > 0.0f)) return fail(MLPO_EINVAL, "inv_scale must be finite and > 0");
    if (isnan(max_norm)) return fail(MLPO_EINVAL, "max_norm is NaN");
    rc = check_norm_workspace(workspace, workspace_bytes);
    if (rc != MLPO_OK) return rc;
    if (out == nullptr || misaligned(out, 16)) return fail(MLPO_EINVAL, "out is NULL or not 16-byte aligned");
    return launch_grad_norm(sg, n_sg, inv_scale, max_norm, workspace, out, static_cast<hipStream_t>(stream), true, keep);
}

int mlpo_grad_unscale_norm_static(const mlpo_subgroup* sg, int32_t n_sg, float inv_scale, float max_norm,
                                  mlpo_step_scalars* out, void* stream) {
    if (n_sg > MLPO_STATIC_MAX_SUBGROUPS)
        return fail(MLPO_EINVAL, "%d subgroups: the call without a workspace takes at most %d", n_sg,
                    MLPO_STATIC_MAX_SUBGROUPS);
    int rc = validate_subgroups(sg, n_sg, /*grads_only=*/true, 1);
    if (rc != MLPO_OK) return rc;
    uint64_t total = 0;
    for (int32_t i = 0; i < n_sg; ++i) total += sg[i].n;  // each n is at most 2^48 (checked), so no overflow
    if (total > MLPO_STATIC_MAX_ELEMENTS)
        return fail(MLPO_EINVAL, "%llu gradients: the call without a workspace takes at most %llu",
                    (unsigned long long)total, (unsigned long long)MLPO_STATIC_MAX_ELEMENTS);
    if (!(isfinite(inv_scale) && inv_scale > 0.0f)) return fail(MLPO_EINVAL, "inv_scale must be finite and > 0");
    if (isnan(max_norm)) return fail(MLPO_EINVAL, "max_norm is NaN");
    if (out == nullptr || misaligned(out, 16)) return fail(MLPO_EINVAL, "out is NULL or not 16-byte aligned");
    void* ws = nullptr;
    rc = static_norm_workspace(&ws);
    if (rc != MLPO_OK) return rc;
    return launch_grad_norm(sg, n_sg, inv_scale, max_norm, ws, out, static_cast<hipStream_t>(stream),
                            /*may_time=*/false);
}

int mlpo_grad_accumulate(uint16_t* acc, const uint16_t* g, uint64_t n, int32_t first, int32_t blocks,
                         int32_t half_format, void* stream) {
    if (n == 0) return MLPO_OK;
    const int rc = check_accumulate(acc, g, n, blocks, half_format);
    if (rc != MLPO_OK) return rc;
    return launch_grad_accumulate(acc, g, n, first != 0, blocks, half_format, static_cast<hipStream_t>(stream));
}

int mlpo_grad_accumulate_norm(uint16_t* acc, const uint16_t* g, uint64_t n, int32_t first, int32_t blocks,
                              int32_t half_format, float inv_scale, void* workspace, size_t workspace_bytes,
                              int32_t begin, void* stream) {
    int rc = check_norm_workspace(workspace, workspace_bytes);
    if (rc != MLPO_OK) return rc;
    if (!(isfinite(inv_scale) && inv_scale > 0.0f)) return fail(MLPO_EINVAL, "inv_scale must be finite and > 0");
    if (n != 0) {
        rc = check_accumulate(acc, g, n, blocks, half_format);
        if (rc != MLPO_OK) return rc;
    }
    NormWorkspace* ws = static_cast<NormWorkspace*>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    int n_partials = 0;
    if (n != 0) {
        rc = launch_grad_accumulate(acc, g, n, first != 0, blocks, half_format, st, ws, inv_scale, &n_partials);
        if (rc != MLPO_OK) return rc;
    }
    if (n_partials == 0 && begin == 0) return MLPO_OK;
    return launch_norm_fold(ws, n_partials, begin != 0, false, inv_scale, 0.0f, nullptr, st);
}

int mlpo_grad_norm_finish(void* workspace, size_t workspace_bytes, float inv_scale, float max_norm,
                          mlpo_step_scalars* out, void* stream) {
    const int rc = check_norm_workspace(workspace, workspace_bytes);
    if (rc != MLPO_OK) return rc;
    if (!(isfinite(inv_scale) && inv_scale > 0.0f)) return fail(MLPO_EINVAL, "inv_scale must be finite and > 0");
    if (isnan(max_norm)) return fail(MLPO_EINVAL, "max_norm is NaN");
    if (out == nullptr || misaligned(out, 16)) return fail(MLPO_EINVAL, "out is NULL or not 16-byte aligned");
    return launch_norm_fold(static_cast<NormWorkspace*>(workspace), 0, false, true, inv_scale, max_norm, out,
                            static_cast<hipStream_t>(stream));
}

int mlpo_adamw_step(const mlpo_subgroup* sg, int32_t n_sg, const mlpo_adamw_hparams* hp, int64_t step,
                    const mlpo_step_scalars* scalars, void* stream) {
    int rc = validate_subgroups(sg, n_sg, false, /*allow_host=*/0);
    if (rc != MLPO_OK) return rc;
    rc = validate_hparams(hp, step);
    if (rc != MLPO_OK) return rc;
    if (scalars != nullptr && misaligned(scalars, 16)) return fail(MLPO_EINVAL, "scalars not 16-byte aligned");
    if (n_sg == 0) return MLPO_OK;
    const AdamwConsts c = make_consts(*hp, step, table_half_format(sg, n_sg));
    std::vector<SgView> views((size_t)n_sg);
    for (int32_t i = 0; i < n_sg; ++i) views[i] = view_of(sg[i]);
    return launch_adamw(views.data(), n_sg, c, scalars, static_cast<hipStream_t>(stream));
}

int32_t mlpo_line_lead(const void* p16) {
    return (int32_t)((reinterpret_cast<uintptr_t>(p16) / 2u) % 64u);
}

uint64_t mlpo_state_floats(uint64_t n, int32_t tile_elems) {
    if (tile_elems <= 0) return 3u * n;
    return round_up(n, (uint64_t)tile_elems) * 3u;
}

}  // extern "C"
