// The tiered pipeline (Algorithm 1 on the HBM / pinned-host pair): staged mode with staging slots and three streams,
// its slot cache, direct mode, and direct mode's scheduler for pieces that pass through bounce buffers (state in a
// file) or end up somewhere else than they came from (flush targets).  Host code only; the update itself is
// launch_adamw.
#include <stddef.h>
#include <string.h>

#include <mutex>
#include <string>
#include <vector>

#include "filetier.h"
#include "mlpo_internal.h"

namespace mlpo {

// ---- pipeline events --------------------------------------------------------------------
struct SlotEvents {
    hipEvent_t h2d_done, upd_done, d2h_done;
};
struct EventCache {
    std::mutex mu;
    int device = -1;
    std::vector<SlotEvents> slots;
    hipEvent_t fence = nullptr;   // orders streams at the start and end of a call
    hipEvent_t fence2 = nullptr;
    hipStream_t copy_in = nullptr;   // the library's own copy streams, used when the caller passes none
    hipStream_t copy_out = nullptr;
    std::vector<hipEvent_t> file_done;  // one per bounce buffer: the end of the kernel that updated it
    hipEvent_t pace[2] = {nullptr, nullptr};  // bound the launches queued on the link stream (file path)
};
static EventCache& events() {
    static EventCache c;
    return c;
}

static int release_events_locked(EventCache& c) {
    for (auto& s : c.slots) {
        (void)hipEventDestroy(s.h2d_done);
        (void)hipEventDestroy(s.upd_done);
        (void)hipEventDestroy(s.d2h_done);
    }
    c.slots.clear();
    if (c.fence) (void)hipEventDestroy(c.fence);
    if (c.fence2) (void)hipEventDestroy(c.fence2);
    c.fence = c.fence2 = nullptr;
    if (c.copy_in) (void)hipStreamDestroy(c.copy_in);
    if (c.copy_out) (void)hipStreamDestroy(c.copy_out);
    c.copy_in = c.copy_out = nullptr;
    for (hipEvent_t e : c.file_done) (void)hipEventDestroy(e);
    c.file_done.clear();
    for (hipEvent_t& e : c.pace) {
        if (e) (void)hipEventDestroy(e);
        e = nullptr;
    }
    c.device = -1;
    return MLPO_OK;
}

static int ensure_events_locked(EventCache& c, int n_slots) {
    int dev = 0;
    MLPO_HIP(hipGetDevice(&dev));
    if (c.device != dev) release_events_locked(c);
    c.device = dev;
    if (c.fence == nullptr) MLPO_HIP(hipEventCreateWithFlags(&c.fence, hipEventDisableTiming));
    if (c.fence2 == nullptr) MLPO_HIP(hipEventCreateWithFlags(&c.fence2, hipEventDisableTiming));
    if (c.copy_in == nullptr) MLPO_HIP(hipStreamCreateWithFlags(&c.copy_in, hipStreamNonBlocking));
    if (c.copy_out == nullptr) MLPO_HIP(hipStreamCreateWithFlags(&c.copy_out, hipStreamNonBlocking));
    while ((int)c.slots.size() < n_slots) {
        SlotEvents s;
        MLPO_HIP(hipEventCreateWithFlags(&s.h2d_done, hipEventDisableTiming));
        MLPO_HIP(hipEventCreateWithFlags(&s.upd_done, hipEventDisableTiming));
        MLPO_HIP(hipEventCreateWithFlags(&s.d2h_done, hipEventDisableTiming));
        c.slots.push_back(s);
    }
    return MLPO_OK;
}


static int ensure_file_events_locked(EventCache& c, int file_slots) {
    while ((int)c.file_done.size() < file_slots) {
        hipEvent_t e;  // writer threads sleep on these instead of spinning while the kernel runs
        MLPO_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming | hipEventBlockingSync));
        c.file_done.push_back(e);
    }
    for (hipEvent_t& e : c.pace)
        if (e == nullptr) MLPO_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
    return MLPO_OK;
}

// Floats the fp32 state of a piece of len elements takes in a staging slot: three arrays, each rounded so that the
// arrays of a slot keep their alignment (planar) or to whole layout tiles (tiled).
static uint64_t state_floats_of(const mlpo_subgroup& s, uint64_t len) {
    return 3u * round_up(len, s.tile_elems > 0 ? (uint64_t)s.tile_elems : 64u);
}

// Elements per transfer of a subgroup under the configuration's chunk_elems.  0 leaves the choice to the library:
// a subgroup of more than 2^25 elements moves in pieces of 2^24 elements (rounded down to whole layout tiles), which
// shortens the pipeline's fill and drain from a subgroup to a piece; smaller ones move whole.
constexpr uint64_t kAutoChunk = (uint64_t)1 << 24;
static uint64_t piece_elems(const mlpo_subgroup& s, uint64_t chunk_elems) {
    if (chunk_elems == MLPO_CHUNK_WHOLE) return s.n;
    if (chunk_elems == 0) {
        if (s.n <= 2 * kAutoChunk) return s.n;
        const uint64_t unit = s.tile_elems > 0 ? (uint64_t)s.tile_elems : 64u;
        return unit >= kAutoChunk ? unit : kAutoChunk / unit * unit;
    }
    return chunk_elems < s.n ? chunk_elems : s.n;
}

// Floats one host-tier subgroup needs in a staging slot when moved in pieces under chunk_elems: the state, and
// behind it the piece's bf16 gradients when those live on the host too.
static uint64_t slot_floats_of(const mlpo_subgroup& s, uint64_t chunk_elems) {
    const uint64_t len = piece_elems(s, chunk_elems);
    uint64_t f = state_floats_of(s, len);
    if (s.tier == MLPO_TIER_HOST_GRADS) f += round_up(len, 128) / 2u;
    return f;
}

static uint64_t slot_floats_for(const mlpo_subgroup* sg, int32_t n_sg, uint64_t chunk_elems) {
    uint64_t mx = 0;
    for (int32_t i = 0; i < n_sg; ++i)
        if (host_tier(sg[i].tier)) {
            const uint64_t f = slot_floats_of(sg[i], chunk_elems);
            if (f > mx) mx = f;
        }
    return mx;
}


// Bytes of one bounce buffer: the largest piece of any subgroup that comes from a file or goes to one (whole
// layout tiles).
static uint64_t bounce_slot_bytes(const mlpo_subgroup* sg, int32_t n_sg, uint64_t chunk_elems,
                                  const mlpo_flush_target* flush_to) {
    uint64_t mx = 0;
    for (int32_t i = 0; i < n_sg; ++i)
        if ((sg[i].tier == MLPO_TIER_FILE || (flush_to != nullptr && flush_to[i].tier == MLPO_TIER_FILE)) &&
            sg[i].tile_elems > 0) {
            const uint64_t b = state_floats_of(sg[i], piece_elems(sg[i], chunk_elems)) * sizeof(float);
            if (b > mx) mx = b;
        }
    return round_up(mx, 4096);
}

// One piece (a whole subgroup or a chunk of one) of a host-tier subgroup and where it lives on the device.
struct Piece {
    const mlpo_subgroup* s;
    uint64_t off, len;  // elements [off, off + len) of the subgroup
    float* state;       // tiled: the piece's layout tiles start here; planar: p starts here, m and v follow `arr` apart
    uint64_t arr;       // planar: floats from one array to the next on the device
    uint16_t* grads;    // where the piece's gradients live on the device when they come from the host with it
};

// A piece that has a staging slot to itself: state at the start of the slot, gradients behind it.
static Piece piece_in_own_slot(const mlpo_subgroup& s, uint64_t off, uint64_t len, float* slot) {
    return Piece{&s, off, len, slot, round_up(len, 64), reinterpret_cast<uint16_t*>(slot + state_floats_of(s, len))};
}

// A piece of a subgroup that occupies a slot as a whole (slot cache): every element has its fixed place in the slot,
// the gradients of the whole subgroup sit behind the whole state.  A planar subgroup is one piece (off = 0).
static Piece piece_of_resident(const mlpo_subgroup& s, uint64_t off, uint64_t len, float* slot) {
    uint16_t* grads = reinterpret_cast<uint16_t*>(slot + state_floats_of(s, s.n)) + off;
    if (s.tile_elems > 0) {
        const uint64_t T = (uint64_t)s.tile_elems;
        return Piece{&s, off, len, slot + (off / T) * 3u * T, 0, grads};
    }
    return Piece{&s, off, len, slot, round_up(s.n, 64), grads};
}

// Where the update reads the piece's gradients: in the slot when they come from the host with the state, else at
// their device home.
static const uint16_t* piece_grads(const Piece& pc) {
    const mlpo_subgroup& s = *pc.s;
    return s.tier == MLPO_TIER_HOST_GRADS ? pc.grads : s.g + pc.off;
}

// Host-to-device transfer of the piece's gradients into its slot (subgroups whose gradients live on the host).
static int fetch_grads(const Piece& pc, hipStream_t st) {
    const mlpo_subgroup& s = *pc.s;
    if (s.tier != MLPO_TIER_HOST_GRADS) return MLPO_OK;
    MLPO_HIP(hipMemcpyAsync(pc.grads, s.g + pc.off, (size_t)pc.len * sizeof(uint16_t), hipMemcpyHostToDevice, st));
    return MLPO_OK;
}

// The kernel's view of a piece on the device.
static SgView slot_view(const Piece& pc) {
    const mlpo_subgroup& s = *pc.s;
    if (s.tile_elems > 0) {
        const uint64_t T = (uint64_t)s.tile_elems;
        return SgView{pc.state, pc.state + T, pc.state + 2 * T, piece_grads(pc), s.p16 + pc.off, pc.len, s.tile_elems};
    }
    return SgView{pc.state, pc.state + pc.arr, pc.state + 2 * pc.arr, piece_grads(pc), s.p16 + pc.off, pc.len, 0};
}

// Host-to-device transfer of a piece to its place on the device; returns the kernel's view of it.
static int fetch_piece(const Piece& pc, hipStream_t st, SgView* view) {
    const mlpo_subgroup& s = *pc.s;
    const int rc = fetch_grads(pc, st);
    if (rc != MLPO_OK) return rc;
    if (s.tile_elems > 0) {
        // whole layout tiles travel as one contiguous block: p, m, v of the same elements stay together
        const uint64_t T = (uint64_t)s.tile_elems;
        const size_t bytes = (size_t)(round_up(pc.len, T) * 3u) * sizeof(float);
        const float* src = s.p + (pc.off / T) * 3u * T;
        MLPO_HIP(hipMemcpyAsync(pc.state, src, bytes, hipMemcpyHostToDevice, st));
    } else {
        const size_t bytes = (size_t)pc.len * sizeof(float);
        MLPO_HIP(hipMemcpyAsync(pc.state, s.p + pc.off, bytes, hipMemcpyHostToDevice, st));
        MLPO_HIP(hipMemcpyAsync(pc.state + pc.arr, s.m + pc.off, bytes, hipMemcpyHostToDevice, st));
        MLPO_HIP(hipMemcpyAsync(pc.state + 2 * pc.arr, s.v + pc.off, bytes, hipMemcpyHostToDevice, st));
    }
    *view = slot_view(pc);
    return MLPO_OK;
}

// Device-to-host transfer of a piece from the device back to the host tier.
static int flush_piece(const Piece& pc, hipStream_t st) {
    const mlpo_subgroup& s = *pc.s;
    if (s.tile_elems > 0) {
        const uint64_t T = (uint64_t)s.tile_elems;
        const size_t bytes = (size_t)(round_up(pc.len, T) * 3u) * sizeof(float);
        float* dst = s.p + (pc.off / T) * 3u * T;
        MLPO_HIP(hipMemcpyAsync(dst, pc.state, bytes, hipMemcpyDeviceToHost, st));
        return MLPO_OK;
    }
    const size_t bytes = (size_t)pc.len * sizeof(float);
    MLPO_HIP(hipMemcpyAsync(s.p + pc.off, pc.state, bytes, hipMemcpyDeviceToHost, st));
    MLPO_HIP(hipMemcpyAsync(s.m + pc.off, pc.state + pc.arr, bytes, hipMemcpyDeviceToHost, st));
    MLPO_HIP(hipMemcpyAsync(s.v + pc.off, pc.state + 2 * pc.arr, bytes, hipMemcpyDeviceToHost, st));
    return MLPO_OK;
}

constexpr uint32_t kCacheMagic = 0x4D4C5043u;  // "MLPC"

static void cache_reset(mlpo_slot_cache* c, int32_t n_slots) {
    memset(c, 0, sizeof *c);
    c->magic = kCacheMagic;
    c->n_slots = n_slots;
    for (int k = 0; k < MLPO_MAX_SLOTS; ++k) c->owner[k] = -1;
}

// Checks that a cache left by earlier calls still describes this subgroup table and this configuration.
static int cache_check(mlpo_slot_cache* c, const mlpo_subgroup* sg, int32_t n_sg, int32_t n_slots) {
    if (c->magic == 0) {
        cache_reset(c, n_slots);
        return MLPO_OK;
    }
    if (c->magic != kCacheMagic) return fail(MLPO_EINVAL, "slot cache is neither zero-initialised nor ours");
    if (c->n_slots != n_slots) return fail(MLPO_EINVAL, "slot cache was built for %d slots, not %d", c->n_slots, n_slots);
    for (int k = 0; k < n_slots; ++k) {
        const int32_t o = c->owner[k];
        if (o < 0) continue;
        if (o >= n_sg || sg[o].p != c->owner_p[k] || !host_tier(sg[o].tier))
            return fail(MLPO_EINVAL, "slot %d holds subgroup %d of a different subgroup table", k, o);
    }
    return MLPO_OK;
}


// What one call has to do, in processing order.
struct Plan {
    std::vector<SgView> resident;    // HBM-tier subgroups
    std::vector<SgView> host_views;  // host-tier subgroups as the device sees them in place (direct mode)
    std::vector<int32_t> host_ids;   // their indices in the caller's table
    std::vector<int32_t> file_ids;   // file-tier subgroups
    std::vector<int32_t> offloaded_ids;  // host-tier and file-tier subgroups together, in processing order
};

struct Streams {
    hipStream_t h2d, cmp, d2h;
};

static std::vector<uint64_t> file_paths_of(const mlpo_subgroup* sg, const std::vector<int32_t>& ids,
                                           const mlpo_stream_cfg* cfg);

static int check_stream_args(const mlpo_subgroup* sg, int32_t n_sg, const int32_t* order,
                             const mlpo_adamw_hparams* hp, int64_t step, const mlpo_step_scalars* scalars,
                             const mlpo_stream_cfg* cfg, uint64_t* slot_floats_out) {
    int rc = validate_subgroups(sg, n_sg, false, /*allow_host=*/2);
    if (rc != MLPO_OK) return rc;
    rc = validate_hparams(hp, step);
    if (rc != MLPO_OK) return rc;
    if (scalars != nullptr && misaligned(scalars, 16)) return fail(MLPO_EINVAL, "scalars not 16-byte aligned");
    if (cfg == nullptr) return fail(MLPO_EINVAL, "cfg is NULL");
    if (cfg->reserved != 0 || cfg->reserved2 != 0) return fail(MLPO_EINVAL, "cfg reserved field is not 0");
    if (cfg->mode != MLPO_STREAM_STAGED && cfg->mode != MLPO_STREAM_DIRECT)
        return fail(MLPO_EINVAL, "unknown mode %d", cfg->mode);
    const bool direct = cfg->mode == MLPO_STREAM_DIRECT;
    if (cfg->direct_blocks < 0 || cfg->direct_blocks > 4096)
        return fail(MLPO_EINVAL, "direct_blocks must be 0..4096 (got %d)", cfg->direct_blocks);
    if (!direct && (cfg->n_slots < 1 || cfg->n_slots > MLPO_MAX_SLOTS))
        return fail(MLPO_EINVAL, "n_slots must be 1..%d (got %d)", MLPO_MAX_SLOTS, cfg->n_slots);
    const bool explicit_chunk = cfg->chunk_elems != 0 && cfg->chunk_elems != MLPO_CHUNK_WHOLE;
    if (explicit_chunk && cfg->chunk_elems % 4 != 0) return fail(MLPO_EINVAL, "chunk_elems must be a multiple of 4");
    if (order != nullptr) {
        std::vector<char> seen((size_t)n_sg, 0);
        for (int32_t i = 0; i < n_sg; ++i) {
            if (order[i] < 0 || order[i] >= n_sg || seen[(size_t)order[i]])
                return fail(MLPO_EINVAL, "order is not a permutation of 0..n_sg-1");
            seen[(size_t)order[i]] = 1;
        }
    }
    bool any_file = false;       // does any subgroup's state live in a file?
    bool any_bounce = false;     // ... or go to one: both need the bounce buffers
    for (int32_t i = 0; i < n_sg; ++i) {
        const bool offloaded = host_tier(sg[i].tier) || sg[i].tier == MLPO_TIER_FILE ||
                               (cfg->flush_to != nullptr && cfg->flush_to[i].tier != MLPO_FLUSH_IN_PLACE);
        if (explicit_chunk && offloaded && sg[i].tile_elems > 0 && cfg->chunk_elems % (uint64_t)sg[i].tile_elems != 0)
            return fail(MLPO_EINVAL, "chunk_elems must be a multiple of subgroup %d's tile_elems", i);
        any_file = any_file || sg[i].tier == MLPO_TIER_FILE;
    }
    any_bounce = any_file;
    if (cfg->flush_to != nullptr) {
        for (int32_t i = 0; i < n_sg; ++i) {
            const mlpo_flush_target& to = cfg->flush_to[i];
            if (to.reserved != 0) return fail(MLPO_EINVAL, "flush target %d: reserved field is not 0", i);
            if (to.tier == MLPO_FLUSH_IN_PLACE || sg[i].n == 0) continue;
            if (to.tier != MLPO_TIER_HBM && to.tier != MLPO_TIER_HOST && to.tier != MLPO_TIER_FILE)
                return fail(MLPO_EINVAL, "flush target %d: tier must be MLPO_TIER_HBM, MLPO_TIER_HOST or MLPO_TIER_FILE",
                            i);
            if (!direct) return fail(MLPO_EINVAL, "flush targets need direct mode");
            if (sg[i].tile_elems <= 0)
                return fail(MLPO_EINVAL, "flush target %d: only subgroups in the tiled layout can move", i);
            if (sg[i].lead != 0)
                return fail(MLPO_EINVAL, "flush target %d: a subgroup with lead cannot move", i);
            if (sg[i].tier == MLPO_TIER_HBM && to.tier == MLPO_TIER_HBM)
                return fail(MLPO_EINVAL, "flush target %d: an HBM-tier subgroup can move to pinned memory or a file", i);
            if (sg[i].tier == MLPO_TIER_HOST_GRADS && to.tier == MLPO_TIER_HBM)
                return fail(MLPO_EINVAL, "flush target %d: the gradients of an HBM-tier subgroup live on the device", i);
            const uint64_t floats = state_floats_of(sg[i], sg[i].n);
            if (to.tier != MLPO_TIER_FILE) {
                if (to.state == nullptr || misaligned(to.state, 256))
                    return fail(MLPO_EINVAL, "flush target %d: state is NULL or not 256-byte aligned", i);
                if (sg[i].tier != MLPO_TIER_FILE && to.state < sg[i].p + floats && sg[i].p < to.state + floats)
                    return fail(MLPO_EINVAL, "flush target %d overlaps the subgroup's current state", i);
            } else {
                any_bounce = true;
            }
        }
    }
    if (cfg->path_stats_cap < 0 || (cfg->path_stats_cap > 0 && cfg->path_stats == nullptr))
        return fail(MLPO_EINVAL, "path_stats_cap is negative, or positive with path_stats NULL");
    if (cfg->file_threads < 0 || cfg->file_threads > 16)
        return fail(MLPO_EINVAL, "file_threads must be 0..16 (got %d)", cfg->file_threads);
    if (any_bounce) {
        if (!direct) return fail(MLPO_EINVAL, "file-tier subgroups need direct mode");
        if (any_file && cfg->files == nullptr) return fail(MLPO_EINVAL, "file-tier subgroups but cfg->files is NULL");
        if (cfg->file_slots < 1 || cfg->file_slots > MLPO_MAX_SLOTS)
            return fail(MLPO_EINVAL, "file_slots must be 1..%d (got %d)", MLPO_MAX_SLOTS, cfg->file_slots);
        if (cfg->bounce == nullptr || misaligned(cfg->bounce, 4096))
            return fail(MLPO_EINVAL, "bounce is NULL or not 4096-byte aligned");
        {
            std::vector<int32_t> all((size_t)n_sg);
            for (int32_t i = 0; i < n_sg; ++i) all[(size_t)i] = i;
            const size_t n_paths = file_paths_of(sg, all, cfg).size();
            if ((size_t)cfg->file_slots < n_paths)
                return fail(MLPO_EINVAL, "file_slots is %d but the files lie on %zu different paths: every path needs "
                            "a bounce buffer of its own", cfg->file_slots, n_paths);
        }
        const uint64_t need_bounce =
            bounce_slot_bytes(sg, n_sg, cfg->chunk_elems, cfg->flush_to) * (uint64_t)cfg->file_slots;
        if (cfg->bounce_bytes < need_bounce)
            return fail(MLPO_ENOMEM, "bounce has %zu bytes, %llu needed", cfg->bounce_bytes,
                        (unsigned long long)need_bounce);
        for (int32_t i = 0; i < n_sg; ++i) {
            if (sg[i].n == 0) continue;
            const uint64_t state_bytes = state_floats_of(sg[i], sg[i].n) * sizeof(float);
            if (sg[i].tier == MLPO_TIER_FILE) {
                rc = check_file_extent(cfg->files[i], state_bytes, i);
                if (rc != MLPO_OK) return rc;
            }
            if (cfg->flush_to != nullptr && cfg->flush_to[i].tier == MLPO_TIER_FILE) {
                rc = check_file_extent(cfg->flush_to[i].file, state_bytes, i);
                if (rc != MLPO_OK) return rc;
            }
        }
    }
    // with a slot cache every slot holds a whole subgroup, whatever size its misses travel in
    const uint64_t slot_floats =
        direct ? 0 : slot_floats_for(sg, n_sg, cfg->cache != nullptr ? MLPO_CHUNK_WHOLE : cfg->chunk_elems);
    const uint64_t need = slot_floats * 4u * (uint64_t)(direct ? 0 : cfg->n_slots);
    if (need > 0) {
        if (cfg->staging == nullptr || misaligned(cfg->staging, 256))
            return fail(MLPO_EINVAL, "staging is NULL or not 256-byte aligned");
        if (cfg->staging_bytes < need)
            return fail(MLPO_ENOMEM, "staging has %zu bytes, %llu needed", cfg->staging_bytes,
                        (unsigned long long)need);
    }
    if (cfg->cache != nullptr) {
        if (direct) return fail(MLPO_EINVAL, "a slot cache needs staged mode");
        rc = cache_check(cfg->cache, sg, n_sg, cfg->n_slots);
        if (rc != MLPO_OK) return rc;
    }
    *slot_floats_out = slot_floats;
    return MLPO_OK;
}

// Direct mode: the host tier is updated in place by a bounded number of persistent workgroups.  That kernel is
// enqueued first so that its workgroups are resident before the HBM-tier kernel fills the rest of the chip.
static int run_direct(const Plan& plan, const AdamwConsts& c, const mlpo_step_scalars* scalars,
                      const mlpo_stream_cfg* cfg, const Streams& st, EventCache& ec) {
    int rc;
    if (!plan.host_views.empty()) {
        MLPO_HIP(hipEventRecord(ec.fence2, st.cmp));  // gradients and scalars come from the compute stream
        MLPO_HIP(hipStreamWaitEvent(st.h2d, ec.fence2, 0));
        const int blocks = cfg->direct_blocks > 0 ? cfg->direct_blocks : 64;
        rc = launch_adamw(plan.host_views.data(), (int)plan.host_views.size(), c, scalars, st.h2d, blocks);
        if (rc != MLPO_OK) return rc;
    }
    if (!plan.resident.empty()) {
        rc = launch_adamw(plan.resident.data(), (int)plan.resident.size(), c, scalars, st.cmp);
        if (rc != MLPO_OK) return rc;
    }
    if (!plan.host_views.empty()) {
        MLPO_HIP(hipEventRecord(ec.fence, st.h2d));
        MLPO_HIP(hipStreamWaitEvent(st.cmp, ec.fence, 0));
    }
    return MLPO_OK;
}

// Where subgroup i's state goes after the update: nullptr = back to where it came from.
static const mlpo_flush_target* flush_target(const mlpo_stream_cfg* cfg, int32_t i) {
    if (cfg->flush_to == nullptr || cfg->flush_to[i].tier == MLPO_FLUSH_IN_PLACE) return nullptr;
    return &cfg->flush_to[i];
}

// Everything the link stream has to run for the offloaded subgroups, in processing order: pieces of at most
// chunk_elems elements (0 = whole subgroups) that either touch pinned memory only (host_pieces) or pass through a
// bounce buffer because their state comes from a file, goes to a file, or both (jobs; job i uses bounce buffer
// i mod file_slots).  A subgroup that changes its path does so at no extra cost: pinned -> file has no read side
// (the kernel reads the pinned state and stores into the bounce buffer), file -> pinned has no write side (the
// kernel stores straight into the pinned destination).  HBM is a source or a destination like pinned memory: a
// subgroup that enters or leaves it crosses the link once instead of twice.
struct LinkWork {
    std::vector<SgView> host_pieces;
    std::vector<FileJob> jobs;
    std::vector<uint64_t> pool_path;  // per pool: the identity of its path (file_path_id)
    std::vector<int> pool_slots;      // per pool: its share of the bounce buffers
};

// The paths that the file sides of this call lead to, in processing order: one pool of workers and bounce buffers
// each.  A piece belongs to the path it is read from, or, if it only goes to a file, to the path it is written to.
static std::vector<uint64_t> file_paths_of(const mlpo_subgroup* sg, const std::vector<int32_t>& ids,
                                           const mlpo_stream_cfg* cfg) {
    std::vector<uint64_t> paths;
    for (int32_t i : ids) {
        if (sg[i].n == 0) continue;  // an empty subgroup moves nothing and its file entry need not name a file
        const mlpo_flush_target* to =
            (cfg->flush_to != nullptr && cfg->flush_to[i].tier != MLPO_FLUSH_IN_PLACE) ? &cfg->flush_to[i] : nullptr;
        const bool from_file = sg[i].tier == MLPO_TIER_FILE;
        const bool to_file = to != nullptr ? to->tier == MLPO_TIER_FILE : from_file;
        if (!from_file && !to_file) continue;
        const int fd = from_file ? cfg->files[i].fd : to->file.fd;
        const uint64_t id = file_path_id(fd);
        bool seen = false;
        for (uint64_t q : paths) seen = seen || q == id;
        if (!seen) paths.push_back(id);
    }
    return paths;
}

static LinkWork link_work(const mlpo_subgroup* sg, const Plan& plan, const mlpo_stream_cfg* cfg,
                          uint64_t buffer_bytes) {
    LinkWork w;
    w.pool_path = file_paths_of(sg, plan.offloaded_ids, cfg);
    const size_t n_pools = w.pool_path.size();
    // the bounce buffers are divided evenly among the paths (checked: at least one each)
    std::vector<size_t> pool_base(n_pools, 0), pool_count(n_pools, 0);
    for (size_t p = 0; p < n_pools; ++p) {
        const int share = cfg->file_slots / (int)n_pools + ((int)p < cfg->file_slots % (int)n_pools ? 1 : 0);
        w.pool_slots.push_back(share);
        pool_base[p] = p == 0 ? 0 : pool_base[p - 1] + (size_t)w.pool_slots[p - 1];
    }
    for (int32_t i : plan.offloaded_ids) {
        const mlpo_subgroup& s = sg[i];
        const mlpo_flush_target* to = flush_target(cfg, i);
        const bool from_file = s.tier == MLPO_TIER_FILE;
        const bool to_file = to != nullptr ? to->tier == MLPO_TIER_FILE : from_file;
        const uint64_t T = (uint64_t)s.tile_elems;  // 0 only for planar host-tier subgroups, which stay in place
        const uint64_t step_elems = piece_elems(s, cfg->chunk_elems);
        size_t pool = 0;
        if (from_file || to_file) {
            const uint64_t id = file_path_id(from_file ? cfg->files[i].fd : to->file.fd);
            while (pool + 1 < n_pools && w.pool_path[pool] != id) ++pool;
        }
        for (uint64_t off = 0; off < s.n; off += step_elems) {
            const uint64_t len = (s.n - off < step_elems) ? (s.n - off) : step_elems;
            // chunk is a multiple of the layout tile, so a piece starts at a layout tile boundary
            const uint64_t state_off = T > 0 ? (off / T) * 3u * T : off;  // floats from the start of the state
            if (!from_file && !to_file) {
                SgView v{s.p + state_off, s.m + state_off, s.v + state_off, s.g + off, s.p16 + off, len, s.tile_elems};
                if (to != nullptr) v.out_delta = (to->state + state_off) - v.p;
                w.host_pieces.push_back(v);
                continue;
            }
            FileJob j;
            j.pool = (int)pool;
            j.bytes = (size_t)(round_up(len, T) * 3u * sizeof(float));
            const size_t slot = pool_base[pool] + pool_count[pool]++ % (size_t)w.pool_slots[pool];
            char* buf = static_cast<char*>(cfg->bounce) + slot * buffer_bytes;
            float* f = reinterpret_cast<float*>(buf);
            j.buffer = buf;
            j.has_read = from_file;
            j.has_write = to_file;
            if (from_file) {
                j.rd_fd = cfg->files[i].fd;
                j.rd_off = cfg->files[i].offset + state_off * sizeof(float);
                j.rd_io = file_io_kind(j.rd_fd);
            }
            if (to_file) {
                const mlpo_file_extent& x = to != nullptr ? to->file : cfg->files[i];
                j.wr_fd = x.fd;
                j.wr_off = x.offset + state_off * sizeof(float);
                j.wr_io = file_io_kind(j.wr_fd);
            }
            // the kernel reads the bounce buffer (state from a file) or the pinned source, and stores into the bounce
            // buffer (state bound for a file) or the pinned destination
            float* src = from_file ? f : s.p + state_off;
            float* dst = to_file ? f : to->state + state_off;
            j.view = SgView{src, src + T, src + 2 * T, s.g + off, s.p16 + off, len, s.tile_elems};
            j.view.out_delta = dst - src;
            w.jobs.push_back(j);
        }
    }
    return w;
}

// Direct mode with file-tier subgroups or flush targets: several paths behind the offloaded tier (Section 3.2 "Unified
// Multi-level, Multi-path Asynchronous Offloading using Virtual Tiers").  All of them end on the link, so their
// kernels share one stream: pinned-only pieces, and pieces that pass through a bounce buffer, each launched as soon
// as its read has finished (or, without a read side, as soon as its buffer is free).  Every file path has its own
// workers, bounce buffers and place in the queue, so a piece from a fast path is never behind one from a slow path.
// At most two launches are queued at a time, so a piece that arrives from a file waits for one other piece at
// most, and the files keep working while the link is busy with the host tier.
static int run_direct_files(const mlpo_subgroup* sg, int32_t n_sg, const Plan& plan, const AdamwConsts& c,
                            const mlpo_step_scalars* scalars, const mlpo_stream_cfg* cfg, const Streams& st,
                            EventCache& ec) {
    int rc = ensure_file_events_locked(ec, cfg->file_slots);
    if (rc != MLPO_OK) return rc;
    int device = 0;
    MLPO_HIP(hipGetDevice(&device));
    const int blocks = cfg->direct_blocks > 0 ? cfg->direct_blocks : 64;
    const uint64_t buffer_bytes = bounce_slot_bytes(sg, n_sg, cfg->chunk_elems, cfg->flush_to);
    LinkWork work = link_work(sg, plan, cfg, buffer_bytes);
    const std::vector<SgView>& host_pieces = work.host_pieces;
    const std::vector<uint64_t> pool_path = work.pool_path;
    FilePath files(std::move(work.jobs), work.pool_slots, cfg->file_threads > 0 ? cfg->file_threads : 2, device);
    const int n_pools = files.n_pools();

    MLPO_HIP(hipEventRecord(ec.fence2, st.cmp));  // gradients and scalars come from the compute stream
    MLPO_HIP(hipStreamWaitEvent(st.h2d, ec.fence2, 0));
    if (!files.start()) {
        std::string why;
        files.join(nullptr, &why);
        return fail(MLPO_EIO, "%s", why.c_str());
    }
    // Everything between the start of the I/O threads and their join runs inside this function, so that a failure
    // on the way still ends with the link stream fenced into the compute stream and the threads joined: the caller
    // gets its error code only after nothing of this call can touch its buffers any more.
    auto launch_all = [&]() -> int {
        if (!plan.resident.empty()) {
            const int r = launch_adamw(plan.resident.data(), (int)plan.resident.size(), c, scalars, st.cmp);
            if (r != MLPO_OK) return r;
        }
        size_t next_host = 0, launched = 0;
        std::vector<size_t> next((size_t)n_pools, 0);  // per path: its next piece
        int turn = 0;                                  // the path asked first: they take turns
        for (;;) {
            if (files.failed()) break;
            std::vector<size_t> waiting;  // the next piece of every path that still has one
            for (int p = 0; p < n_pools; ++p)
                if (next[(size_t)p] < files.pool_size(p)) waiting.push_back(files.pool_job(p, next[(size_t)p]));
            if (waiting.empty() && next_host >= host_pieces.size()) break;
            int ready = -1;
            for (int k = 0; k < n_pools && ready < 0; ++k) {
                const int p = (turn + k) % n_pools;
                if (next[(size_t)p] < files.pool_size(p) && files.is_read(files.pool_job(p, next[(size_t)p]))) ready = p;
            }
            if (ready < 0 && next_host >= host_pieces.size()) {  // only files are left and nothing has arrived yet
                if (!files.wait_any_read(waiting)) break;
                continue;
            }
            if (launched >= 2) MLPO_HIP(hipEventSynchronize(ec.pace[launched % 2]));  // the launch before the last
            if (ready >= 0) {
                const size_t i = files.pool_job(ready, next[(size_t)ready]);
                const FileJob& j = files.job(i);
                const int r = launch_adamw(&j.view, 1, c, scalars, st.h2d, blocks);
                if (r != MLPO_OK) return r;
                // one event per bounce buffer: the buffer's previous piece has been written, so its event is free
                const size_t buffer = (size_t)((static_cast<const char*>(j.buffer) - static_cast<const char*>(cfg->bounce)) /
                                               (ptrdiff_t)buffer_bytes);
                hipEvent_t done = ec.file_done[buffer];
                MLPO_HIP(hipEventRecord(done, st.h2d));
                files.hand_to_writer(i, done);
                ++next[(size_t)ready];
                turn = (ready + 1) % n_pools;
            } else {
                const int r = launch_adamw(&host_pieces[next_host], 1, c, scalars, st.h2d, blocks);
                if (r != MLPO_OK) return r;
                ++next_host;
            }
            MLPO_HIP(hipEventRecord(ec.pace[launched % 2], st.h2d));
            ++launched;
        }
        return MLPO_OK;
    };
    rc = launch_all();
    if (rc != MLPO_OK) files.stop();  // the threads leave at their next wait; error text of rc is already set
    const hipError_t fence_rec = hipEventRecord(ec.fence, st.h2d);
    const hipError_t fence_wait = fence_rec == hipSuccess ? hipStreamWaitEvent(st.cmp, ec.fence, 0) : fence_rec;
    if (fence_wait != hipSuccess) (void)hipStreamSynchronize(st.h2d);  // no fence: wait here instead
    std::string err;
    std::vector<mlpo_file_stats> per_pool;
    const bool io_ok = files.join(cfg->file_stats, &err, &per_pool);
    for (int32_t k = 0; k < cfg->path_stats_cap; ++k) {  // what each path moved, in the order the paths came up
        mlpo_path_stats& out = cfg->path_stats[k];
        out = mlpo_path_stats{};
        if ((size_t)k < per_pool.size()) {
            out.path_id = pool_path[(size_t)k];
            out.used = 1;
            out.stats = per_pool[(size_t)k];
        }
    }
    if (rc != MLPO_OK) return rc;
    if (fence_wait != hipSuccess) return fail(MLPO_EHIP, "fencing the link stream: %s", hipGetErrorString(fence_wait));
    if (!io_ok) return fail(MLPO_EIO, "%s", err.c_str());
    return MLPO_OK;
}

// Staged mode with a slot cache: slots keep their subgroup from one step to the next (Section 3.2 "Cache-Friendly
// Ordering").  A subgroup found in a slot is updated there without any transfer, and a slot changes its occupant only
// when another subgroup needs it (or is copied back on mlpo_stream_flush).  With the order reversed from step to step
// the subgroups processed last are the ones processed first next time.
// A miss of a tiled subgroup into a slot that is empty, clean, or holds a subgroup with the same layout tile is served
// by kernels on the link stream: a bounded number of persistent workgroups read the newcomer's state in pinned memory,
// update it and store it into the slot, and - tile by tile, just before they overwrite it - send what the slot held
// to the old occupant's home in pinned memory.  Both directions of the link are busy from the first tile to the
// last, there is no pipeline to fill or drain and nothing depends on how the runtime schedules copies of different
// streams.  Subgroups of equal length (all but the last of a shard) are exchanged by ONE launch; where the lengths
// differ, the common whole layout tiles are exchanged, the rest of the longer one follows on the same stream.
// Other misses (planar subgroups, occupants with another layout tile) move by copies: the old occupant goes back to
// the host, the newcomer takes its place piece by piece and every piece is updated as soon as it has arrived.
static int run_cached(const mlpo_subgroup* sg, const Plan& plan, const AdamwConsts& c,
                      const mlpo_step_scalars* scalars, const mlpo_stream_cfg* cfg, uint64_t slot_floats,
                      const Streams& st, EventCache& ec) {
    mlpo_slot_cache* cache = cfg->cache;
    float* staging = static_cast<float*>(cfg->staging);
    int rc;
    // workgroups of a miss served by a kernel (13 x 100 M elements, 4 slots, ms per step: 32 workgroups 246.7, 48 225.8,
    // 64 221.7, 80 220.6, 96 223.2, 128 230.7)
    const int link_blocks = cfg->direct_blocks > 0 ? cfg->direct_blocks : 80;
    bool link_used = false;
    // pieces a subgroup moves in while it enters or leaves a slot: planar subgroups whole (their arrays are spread
    // over the slot), tiled ones under the configuration's chunk_elems
    const auto step_of = [cfg](const mlpo_subgroup& s) { return s.tile_elems > 0 ? piece_elems(s, cfg->chunk_elems) : s.n; };
    for (int32_t i : plan.host_ids) {
        const mlpo_subgroup& s = sg[i];
        int k = -1;
        for (int q = 0; q < cfg->n_slots; ++q)
            if (cache->owner[q] == i) k = q;
        const bool hit = k >= 0;
        if (!hit) {
            for (int q = 0; q < cfg->n_slots && k < 0; ++q)
                if (cache->owner[q] < 0) k = q;
            if (k < 0) {  // least recently updated slot
                k = 0;
                for (int q = 1; q < cfg->n_slots; ++q)
                    if (cache->stamp[q] < cache->stamp[k]) k = q;
            }
        }
        SlotEvents& ev = ec.slots[(size_t)k];
        float* slot = staging + (uint64_t)k * slot_floats;
        if (hit) {
            const Piece pc = piece_of_resident(s, 0, s.n, slot);
            // an explicit flush of this slot may still be reading it
            MLPO_HIP(hipStreamWaitEvent(st.cmp, ev.d2h_done, 0));
            if (s.tier == MLPO_TIER_HOST_GRADS) {
                // the state stayed, this step's gradients still have to come in (after the last update read the old)
                MLPO_HIP(hipStreamWaitEvent(st.h2d, ev.upd_done, 0));
                rc = fetch_grads(pc, st.h2d);
                if (rc != MLPO_OK) return rc;
                MLPO_HIP(hipEventRecord(ev.h2d_done, st.h2d));
                MLPO_HIP(hipStreamWaitEvent(st.cmp, ev.h2d_done, 0));
            }
            const SgView view = slot_view(pc);
            rc = launch_adamw(&view, 1, c, scalars, st.cmp);
            if (rc != MLPO_OK) return rc;
            ++cache->hits;
        } else {
            const mlpo_subgroup* old = (cache->owner[k] >= 0 && cache->dirty[k]) ? &sg[cache->owner[k]] : nullptr;
            cache->owner[k] = -1;  // until the new occupant is in place
            cache->dirty[k] = 0;
            // the slot's last update and any earlier copy out of it are behind both copy streams
            MLPO_HIP(hipStreamWaitEvent(st.d2h, ev.upd_done, 0));
            MLPO_HIP(hipStreamWaitEvent(st.h2d, ev.d2h_done, 0));
            MLPO_HIP(hipStreamWaitEvent(st.h2d, ev.upd_done, 0));
            if (s.tile_elems > 0 && (old == nullptr || old->tile_elems == s.tile_elems)) {
                // Kernels on the link stream: the newcomer comes in updated, the old occupant (if any) goes home.
                // What both have - all of it when they are equally long, else their common whole layout tiles -
                // is exchanged in one pass; what only the old occupant has is copied out behind that, and what
                // only the newcomer has is then brought in by the out-of-place update.
                const uint64_t T = (uint64_t)s.tile_elems;
                const uint64_t n_old = old != nullptr ? old->n : 0;
                uint64_t both = n_old < s.n ? n_old : s.n;
                if (n_old != s.n) both = both / T * T;
                // elements [off, off + len) of the newcomer as the kernel sees them: state and (for subgroups that
                // keep them there) gradients in pinned memory, new state into the slot
                const auto part = [&](uint64_t off, uint64_t len) {
                    const uint64_t state_off = (off / T) * 3u * T;
                    SgView v{s.p + state_off, s.m + state_off, s.v + state_off, s.g + off, s.p16 + off, len, s.tile_elems};
                    v.out_delta = slot - s.p;
                    return v;
                };
                if (both > 0) {
                    SgView view = part(0, both);
                    view.evict_delta = old->p - slot;
                    rc = launch_adamw(&view, 1, c, scalars, st.h2d, link_blocks);
                    if (rc != MLPO_OK) return rc;
                }
                if (n_old > both) {
                    rc = flush_piece(piece_of_resident(*old, both, n_old - both, slot), st.h2d);
                    if (rc != MLPO_OK) return rc;
                }
                if (s.n > both) {
                    const SgView view = part(both, s.n - both);
                    rc = launch_adamw(&view, 1, c, scalars, st.h2d, link_blocks);
                    if (rc != MLPO_OK) return rc;
                }
                if (old != nullptr) ++cache->flushes;
                ++cache->fetches;
                MLPO_HIP(hipEventRecord(ev.upd_done, st.h2d));
                link_used = true;
                cache->owner[k] = i;
                cache->owner_p[k] = s.p;
                cache->dirty[k] = 1;
                cache->stamp[k] = ++cache->clock;
                continue;
            }
            // Copies: a planar subgroup, or an occupant with another layout tile.  The old occupant leaves first, the
            // newcomer follows piece by piece and every piece is updated as soon as it has arrived.
            if (old != nullptr) {
                const uint64_t step_old = step_of(*old);
                for (uint64_t off = 0; off < old->n; off += step_old) {
                    const uint64_t len = old->n - off < step_old ? old->n - off : step_old;
                    rc = flush_piece(piece_of_resident(*old, off, len, slot), st.d2h);
                    if (rc != MLPO_OK) return rc;
                }
                MLPO_HIP(hipEventRecord(ev.d2h_done, st.d2h));
                MLPO_HIP(hipStreamWaitEvent(st.h2d, ev.d2h_done, 0));
                ++cache->flushes;
            }
            const uint64_t step_new = step_of(s);
            for (uint64_t off = 0; off < s.n; off += step_new) {
                const uint64_t len = s.n - off < step_new ? s.n - off : step_new;
                SgView view;
                rc = fetch_piece(piece_of_resident(s, off, len, slot), st.h2d, &view);
                if (rc != MLPO_OK) return rc;
                MLPO_HIP(hipEventRecord(ev.h2d_done, st.h2d));
                MLPO_HIP(hipStreamWaitEvent(st.cmp, ev.h2d_done, 0));
                rc = launch_adamw(&view, 1, c, scalars, st.cmp);
                if (rc != MLPO_OK) return rc;
            }
            ++cache->fetches;
        }
        MLPO_HIP(hipEventRecord(ev.upd_done, st.cmp));
        cache->owner[k] = i;
        cache->owner_p[k] = s.p;
        cache->dirty[k] = 1;
        cache->stamp[k] = ++cache->clock;
    }
    if (link_used) {  // the compute stream sees the end of the kernels on the link stream
        MLPO_HIP(hipEventRecord(ec.fence2, st.h2d));
        MLPO_HIP(hipStreamWaitEvent(st.cmp, ec.fence2, 0));
    }
    return MLPO_OK;
}

// Staged mode: fetch -> update -> flush for every subgroup or chunk, slots reused round-robin; a slot is refilled
// only after its previous occupant has been flushed, so at most n_slots transfers are in flight.
static int run_staged(const mlpo_subgroup* sg, const Plan& plan, const AdamwConsts& c,
                      const mlpo_step_scalars* scalars, const mlpo_stream_cfg* cfg, uint64_t slot_floats,
                      const Streams& st, EventCache& ec) {
    float* staging = static_cast<float*>(cfg->staging);
    uint64_t piece = 0;
    int rc;
    for (int32_t i : plan.host_ids) {
        const mlpo_subgroup& s = sg[i];
        const uint64_t step_elems = piece_elems(s, cfg->chunk_elems);
        for (uint64_t off = 0; off < s.n; off += step_elems, ++piece) {
            const uint64_t len = (s.n - off < step_elems) ? (s.n - off) : step_elems;
            const int k = (int)(piece % (uint64_t)cfg->n_slots);
            SlotEvents& ev = ec.slots[(size_t)k];
            const Piece pc = piece_in_own_slot(s, off, len, staging + (uint64_t)k * slot_floats);
            hipEvent_t tf0 = nullptr, tf1 = nullptr, tw0 = nullptr, tw1 = nullptr;
            const bool timed =
                timing_enabled() && timing_acquire_two(kTimedFetch, &tf0, &tf1, kTimedFlush, &tw0, &tw1);
            // fetch
            if (piece >= (uint64_t)cfg->n_slots) MLPO_HIP(hipStreamWaitEvent(st.h2d, ev.d2h_done, 0));
            if (timed) MLPO_HIP(hipEventRecord(tf0, st.h2d));
            SgView view;
            rc = fetch_piece(pc, st.h2d, &view);
            if (rc != MLPO_OK) return rc;
            if (timed) MLPO_HIP(hipEventRecord(tf1, st.h2d));
            MLPO_HIP(hipEventRecord(ev.h2d_done, st.h2d));
            // update in the slot; gradients and bf16 parameters stay at their device homes
            MLPO_HIP(hipStreamWaitEvent(st.cmp, ev.h2d_done, 0));
            rc = launch_adamw(&view, 1, c, scalars, st.cmp);
            if (rc != MLPO_OK) return rc;
            MLPO_HIP(hipEventRecord(ev.upd_done, st.cmp));
            // flush
            MLPO_HIP(hipStreamWaitEvent(st.d2h, ev.upd_done, 0));
            if (timed) MLPO_HIP(hipEventRecord(tw0, st.d2h));
            rc = flush_piece(pc, st.d2h);
            if (rc != MLPO_OK) return rc;
            if (timed) MLPO_HIP(hipEventRecord(tw1, st.d2h));
            MLPO_HIP(hipEventRecord(ev.d2h_done, st.d2h));
        }
    }
    return MLPO_OK;
}

}  // namespace mlpo

using namespace mlpo;

extern "C" {

size_t mlpo_stream_staging_bytes(const mlpo_subgroup* sg, int32_t n_sg, int32_t n_slots, uint64_t chunk_elems) {
    if (sg == nullptr || n_sg <= 0 || n_slots <= 0) return 0;
    return (size_t)(slot_floats_for(sg, n_sg, chunk_elems) * 4u * (uint64_t)n_slots);
}

size_t mlpo_stream_bounce_bytes(const mlpo_subgroup* sg, int32_t n_sg, int32_t file_slots, uint64_t chunk_elems,
                                const mlpo_flush_target* flush_to) {
    if (sg == nullptr || n_sg <= 0 || file_slots <= 0) return 0;
    return (size_t)(bounce_slot_bytes(sg, n_sg, chunk_elems, flush_to) * (uint64_t)file_slots);
}

int mlpo_stream_update(const mlpo_subgroup* sg, int32_t n_sg, const int32_t* order, const mlpo_adamw_hparams* hp,
                       int64_t step, const mlpo_step_scalars* scalars, const mlpo_stream_cfg* cfg, int32_t* applied) {
    uint64_t slot_floats = 0;
    int rc = check_stream_args(sg, n_sg, order, hp, step, scalars, cfg, &slot_floats);
    if (rc != MLPO_OK) return rc;
    if (applied != nullptr) *applied = 1;
    if (cfg->file_stats != nullptr) memset(cfg->file_stats, 0, sizeof *cfg->file_stats);  // nothing moved so far
    for (int32_t k = 0; k < cfg->path_stats_cap; ++k) cfg->path_stats[k] = mlpo_path_stats{};
    if (n_sg == 0) return MLPO_OK;

    Streams st{static_cast<hipStream_t>(cfg->h2d), static_cast<hipStream_t>(cfg->compute),
               static_cast<hipStream_t>(cfg->d2h)};

    // Where the host issues transfers, starts I/O threads or keeps books (staged mode, the slot cache, file-tier
    // subgroups, flush targets), and where the caller asks whether the step was applied, the skip decision has to be
    // known here.  Plain direct mode does not need it: both of its kernels read the flag on the device and leave at
    // once when it is set, so with applied == NULL that call waits for nothing (and can be captured in a HIP graph).
    bool host_decides = cfg->mode != MLPO_STREAM_DIRECT || applied != nullptr;
    for (int32_t i = 0; i < n_sg && !host_decides; ++i)
        host_decides = sg[i].n != 0 && (sg[i].tier == MLPO_TIER_FILE ||
                                        (cfg->flush_to != nullptr && cfg->flush_to[i].tier != MLPO_FLUSH_IN_PLACE));
    if (scalars != nullptr && host_decides) {
        mlpo_step_scalars h;
        MLPO_HIP(hipMemcpyAsync(&h, scalars, sizeof h, hipMemcpyDeviceToHost, st.cmp));
        MLPO_HIP(hipStreamSynchronize(st.cmp));
        if (h.found_inf != 0u) {
            if (applied != nullptr) *applied = 0;
            return MLPO_OK;
        }
    }

    const AdamwConsts c = make_consts(*hp, step, table_half_format(sg, n_sg));
    Plan plan;
    for (int32_t k = 0; k < n_sg; ++k) {
        const int32_t i = order ? order[k] : k;
        if (sg[i].n == 0) continue;
        const SgView v = view_of(sg[i]);  // lead is 0 for everything but HBM-tier subgroups (checked)
        if (sg[i].tier == MLPO_TIER_HBM && flush_target(cfg, i) == nullptr) {
            plan.resident.push_back(v);
        } else if (sg[i].tier == MLPO_TIER_HBM) {
            plan.offloaded_ids.push_back(i);  // leaves HBM: its stores go over the link, so it runs with the link's pieces
        } else if (sg[i].tier == MLPO_TIER_FILE) {
            plan.file_ids.push_back(i);
            plan.offloaded_ids.push_back(i);
        } else {
            plan.offloaded_ids.push_back(i);
            plan.host_ids.push_back(i);
            plan.host_views.push_back(v);
        }
    }

    EventCache& ec = events();
    std::lock_guard<std::mutex> lk(ec.mu);
    if (plan.offloaded_ids.empty()) {  // nothing offloaded and nothing on its way out of HBM: this is mlpo_adamw_step
        if (plan.resident.empty()) return MLPO_OK;
        return launch_adamw(plan.resident.data(), (int)plan.resident.size(), c, scalars, st.cmp);
    }
    const bool direct = cfg->mode == MLPO_STREAM_DIRECT;
    rc = ensure_events_locked(ec, direct ? 0 : cfg->n_slots);
    if (rc != MLPO_OK) return rc;
    if (cfg->h2d == nullptr && cfg->d2h == nullptr) {
        // no copy streams given: the library's own pair (created on first use, one pair per device)
        st.h2d = ec.copy_in;
        st.d2h = ec.copy_out;
    }
    bool moves = false;  // does any subgroup go to another place than it came from?
    for (int32_t i : plan.offloaded_ids) moves = moves || flush_target(cfg, i) != nullptr;
    if (direct && (!plan.file_ids.empty() || moves)) return run_direct_files(sg, n_sg, plan, c, scalars, cfg, st, ec);
    if (direct) return run_direct(plan, c, scalars, cfg, st, ec);

    // Work enqueued earlier on the flush and compute streams (a previous step's copy back, the gradient pass) must
    // be complete before this step's first fetch overwrites a staging slot or reads the host tier.
    MLPO_HIP(hipEventRecord(ec.fence, st.d2h));
    MLPO_HIP(hipStreamWaitEvent(st.h2d, ec.fence, 0));
    MLPO_HIP(hipEventRecord(ec.fence2, st.cmp));
    MLPO_HIP(hipStreamWaitEvent(st.h2d, ec.fence2, 0));
    // HBM-tier subgroups first: their kernel runs while the first fetches are in flight.
    if (!plan.resident.empty()) {
        rc = launch_adamw(plan.resident.data(), (int)plan.resident.size(), c, scalars, st.cmp);
        if (rc != MLPO_OK) return rc;
    }
    rc = cfg->cache != nullptr ? run_cached(sg, plan, c, scalars, cfg, slot_floats, st, ec)
                               : run_staged(sg, plan, c, scalars, cfg, slot_floats, st, ec);
    if (rc != MLPO_OK) return rc;
    // join: the compute stream sees the end of the last flush
    MLPO_HIP(hipEventRecord(ec.fence, st.d2h));
    MLPO_HIP(hipStreamWaitEvent(st.cmp, ec.fence, 0));
    return MLPO_OK;
}

int mlpo_stream_flush(const mlpo_subgroup* sg, int32_t n_sg, const mlpo_stream_cfg* cfg) {
    int rc = validate_subgroups(sg, n_sg, false, /*allow_host=*/1);
    if (rc != MLPO_OK) return rc;
    if (cfg == nullptr || cfg->cache == nullptr) return fail(MLPO_EINVAL, "cfg or its slot cache is NULL");
    if (cfg->mode != MLPO_STREAM_STAGED || cfg->n_slots < 1 || cfg->n_slots > MLPO_MAX_SLOTS)
        return fail(MLPO_EINVAL, "not a staged configuration");
    mlpo_slot_cache* cache = cfg->cache;
    if (cache->magic == 0) return MLPO_OK;  // never used: nothing is held
    rc = cache_check(cache, sg, n_sg, cfg->n_slots);
    if (rc != MLPO_OK) return rc;
    const uint64_t slot_floats = slot_floats_for(sg, n_sg, MLPO_CHUNK_WHOLE);
    if (cfg->staging == nullptr || cfg->staging_bytes < slot_floats * 4u * (uint64_t)cfg->n_slots)
        return fail(MLPO_ENOMEM, "staging does not match the configuration the cache was filled with");
    EventCache& ec = events();
    std::lock_guard<std::mutex> lk(ec.mu);
    rc = ensure_events_locked(ec, cfg->n_slots);
    if (rc != MLPO_OK) return rc;
    hipStream_t s_cmp = static_cast<hipStream_t>(cfg->compute);
    hipStream_t s_d2h = (cfg->h2d == nullptr && cfg->d2h == nullptr) ? ec.copy_out : static_cast<hipStream_t>(cfg->d2h);
    float* staging = static_cast<float*>(cfg->staging);
    bool any = false;
    for (int k = 0; k < cfg->n_slots; ++k) {
        if (cache->owner[k] < 0 || !cache->dirty[k]) continue;
        const mlpo_subgroup& s = sg[cache->owner[k]];
        SlotEvents& ev = ec.slots[(size_t)k];
        MLPO_HIP(hipStreamWaitEvent(s_d2h, ev.upd_done, 0));
        rc = flush_piece(piece_of_resident(s, 0, s.n, staging + (uint64_t)k * slot_floats), s_d2h);
        if (rc != MLPO_OK) return rc;
        MLPO_HIP(hipEventRecord(ev.d2h_done, s_d2h));
        cache->dirty[k] = 0;
        ++cache->flushes;
        any = true;
    }
    if (any) {
        MLPO_HIP(hipEventRecord(ec.fence, s_d2h));
        MLPO_HIP(hipStreamWaitEvent(s_cmp, ec.fence, 0));
    }
    return MLPO_OK;
}

int mlpo_shutdown(void) {
    EventCache& c = events();
    std::lock_guard<std::mutex> lk(c.mu);
    return release_events_locked(c);
}

}  // extern "C"
