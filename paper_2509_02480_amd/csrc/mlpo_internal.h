// Internal declarations shared by the translation units of libmlpo (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "mlpo.h"

namespace mlpo {

// ---- error reporting -------------------------------------------------------
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
#define MLPO_HIP(call)                                                                   \
    do {                                                                                 \
        hipError_t e_ = (call);                                                          \
        if (e_ != hipSuccess) return ::mlpo::fail(MLPO_EHIP, "%s: %s", #call, hipGetErrorString(e_)); \
    } while (0)

int num_cus();  // compute units of the current device (cached); <= 0 on failure

// ---- optional per-kernel timing (the dispatch's own start / stop timestamps) ------------------
// When enabled, launch sites ask for an event pair and launch through hipExtLaunchKernelGGL, which stamps the events
// with the kernel's begin and end on the device rather than with the time markers reach the queue.
constexpr int kTimedUpdate = 0;  // the fused AdamW kernel (128-bit variant)
constexpr int kTimedGradPass = 1;  // pass 1 of the gradient pass
constexpr int kTimedFetch = 2;     // staged mode: one host-to-device transfer (markers on the copy stream)
constexpr int kTimedFlush = 3;     // staged mode: one device-to-host transfer
constexpr int kTimedAccumulate = 4;  // the gradient accumulation kernel (128-bit variant)
constexpr int kTimedKinds = 5;
bool timing_enabled();
bool timing_acquire(int which, hipEvent_t* start, hipEvent_t* stop);  // false: not enabled or table full
// The same for two kinds at once: both pairs or neither.
bool timing_acquire_two(int which_a, hipEvent_t* a0, hipEvent_t* a1, int which_b, hipEvent_t* b0, hipEvent_t* b1);

// ---- per-step scalars of the update, derived on the host ---------------------
struct AdamwConsts {
    float beta1, beta2, omb1, omb2, eps, step_size, sqbc2, decay;
    float l2;         // l2_mode: weight decay added to the gradient (decay is then 1)
    int32_t l2_mode;  // 0: AdamW, 1: Adam with the decay term in the gradient
    int32_t half;     // format of g and p16: MLPO_HALF_BF16 or MLPO_HALF_FP16
};
int validate_hparams(const mlpo_adamw_hparams* hp, int64_t step);
// Pointer / size / tier checks shared by the entry points; grads_only checks g and n alone.  allow_host: 0 = only
// HBM-tier subgroups, 1 = host tiers too, 2 = file tier too.
int validate_subgroups(const mlpo_subgroup* sg, int32_t n_sg, bool grads_only, int allow_host);
bool misaligned(const void* p, uintptr_t a);
uint64_t round_up(uint64_t x, uint64_t to);
AdamwConsts make_consts(const mlpo_adamw_hparams& hp, int64_t step, int32_t half);
// The half-precision format all subgroups of a table share (checked by validate_subgroups); bf16 for an empty table.
int32_t table_half_format(const mlpo_subgroup* sg, int32_t n_sg);

// ---- kernel-side view of a subgroup -------------------------------------------
struct SgView {
    float* p;
    float* m;
    float* v;
    const uint16_t* g;
    uint16_t* p16;
    uint64_t n;
    int32_t tile_elems;  // 0 = planar p/m/v; T > 0 = tiled state (m == p + T, v == p + 2T, layout tiles 3T apart)
    // Out-of-place update (tiled views only): the new p, m, v are stored out_delta floats behind where the old ones
    // were read, i.e. into another buffer of the same layout; 0 = in place.  A multiple of 4.
    int64_t out_delta = 0;
    // Exchange (with out_delta != 0 only): what the destination held before is stored evict_delta floats behind the
    // destination - the previous occupant of a staging slot leaves for its home while the new one arrives.  0 = the
    // destination's content is simply overwritten.  A multiple of 4.
    int64_t evict_delta = 0;
    // Padding in front (tiled views only): the view's first `lead` elements are no elements of the subgroup, nothing
    // is read or written for them (g and p16 point `lead` elements before the subgroup's first value, n counts the
    // padding).  A multiple of 4, smaller than a kernel tile.  It lets the caller shift a subgroup inside its state
    // buffer until the 128-byte lines of g and p16 and those of p, m, v begin at the same elements.
    uint32_t lead = 0;
};

// The view of a whole subgroup as the caller describes it (mlpo_subgroup::lead applied).
inline SgView view_of(const mlpo_subgroup& s) {
    SgView v{s.p, s.m, s.v, s.g, s.p16, s.n, s.tile_elems};
    if (s.lead > 0) {
        v.g -= s.lead;
        v.p16 -= s.lead;
        v.n += (uint64_t)s.lead;
        v.lead = (uint32_t)s.lead;
    }
    return v;
}

// Enqueues the fused update over `n` views (memory the device can address) on `stream`.  Views are split between
// the 128-bit kernel and the element-wise kernel by alignment; any number of views is accepted (several launches if
// needed).  persist_blocks > 0 runs the 128-bit kernel as that many persistent blocks (used when the state sits in
// pinned host memory and the number of workgroups on the link is to be bounded); 0 lets the launcher choose.
int launch_adamw(const SgView* views, int n, const AdamwConsts& c, const mlpo_step_scalars* scalars,
                 hipStream_t stream, int persist_blocks = 0);

// Enqueues the gradient pass (see mlpo_grad_unscale_norm).
// may_time = false: never stamps the launch with timing events (creating an event allocates).  keep (host array of
// n_sg device pointers, entries may be NULL; or NULL): where to leave a copy of each subgroup's gradients.
int launch_grad_norm(const mlpo_subgroup* sg, int n_sg, float inv_scale, float max_norm, void* workspace,
                     mlpo_step_scalars* out, hipStream_t stream, bool may_time = true,
                     uint16_t* const* keep = nullptr);
// The address, on the current device, of the library's own statically allocated gradient-pass workspace.
constexpr int kMaxDevices = 64;
int static_norm_workspace(void** out);
size_t grad_norm_workspace_bytes();

// Device workspace of the gradient statistics: per-workgroup partial sums of squares (fp64) and non-finite flags,
// and the running totals that a one-block kernel folds them into in index order.
constexpr int kNormMaxPartials = 16384;
struct NormWorkspace {
    double running_sum;
    uint32_t running_flag;
    uint32_t pad[61];
    double partial[kNormMaxPartials];
    uint32_t flag[kNormMaxPartials];
};
static_assert(offsetof(NormWorkspace, partial) == 256, "layout");
// Folds partial[0..n_partials) into the running totals (first: the totals start at zero); last: derives norm, clip
// coefficient, gradient multiplier and flag from the totals and writes them to out (out may be NULL otherwise).
int launch_norm_fold(NormWorkspace* ws, int n_partials, bool first, bool last, float inv_scale, float max_norm,
                     mlpo_step_scalars* out, hipStream_t st);

// Enqueues acc = first ? g : bf16(acc + g) over n elements; blocks > 0 bounds the persistent grid.  With stats the
// kernels also leave the statistics of the new acc values (unscaled by inv_scale) as partials in stats and
// *n_partials says how many; the grid is then always persistent.
int launch_grad_accumulate(uint16_t* acc, const uint16_t* g, uint64_t n, bool first, int blocks, int32_t half,
                           hipStream_t st, NormWorkspace* stats = nullptr, float inv_scale = 1.0f,
                           int* n_partials = nullptr);

inline bool host_tier(int32_t tier) { return tier == MLPO_TIER_HOST || tier == MLPO_TIER_HOST_GRADS; }

}  // namespace mlpo
