/*
 * mlpo.h - C ABI of the MI355X (gfx950) update-phase library for MLP-Offload (arXiv 2509.02480).
 *
 * The library runs the per-subgroup body of the paper's update phase (Algorithm 1: wait for the subgroup, upcast its
 * half-precision gradients on the fly, update the fp32 master parameters / momentum / variance, push the
 * half-precision parameters, flush, prefetch the next) with the GPU as the place of the update, HBM as the fast tier
 * and pinned host memory as the slow tier - the generalisation to a GPU-CPU tier pair that Section 3.2 "Unified
 * Multi-level, Multi-path Asynchronous Offloading using Virtual Tiers" mentions - and, optionally, a file as a second
 * path behind the slow tier.
 *
 * Conventions
 *   - mlpo_grad_unscale_norm, mlpo_adamw_step and mlpo_grad_accumulate* only enqueue kernels on the given stream (no
 *     allocation, no memset, no host wait), so they can be recorded into a HIP graph by stream capture; the
 *     per-step constants of the update are kernel arguments, so a captured update repeats the step number it was
 *     captured with (exact for every step when bias_correction is 0).
 *   - Every call returns 0 (MLPO_OK) or a negative code; mlpo_last_error() gives the text for the calling thread.
 *   - The caller owns every buffer.  The library allocates no device or host memory for user data, keeps no pointer
 *     after the work it enqueued has completed, and never frees anything passed in.
 *   - Calls enqueue work on the given HIP streams (passed as void*, i.e. a hipStream_t; NULL is the default stream)
 *     and return without waiting, except where stated.
 *   - "device" pointers are HBM addresses valid on the current HIP device; "pinned host" pointers are page-locked
 *     host memory (hipHostMalloc) mapped into the device's address space; "host" pointers are ordinary host memory
 *     read only during the call.
 *   - fp32 arrays must be 4-byte aligned and bf16 arrays 2-byte aligned.  The fast kernels are used for a subgroup
 *     whose p, m, v are 16-byte aligned and whose g, p16 are 8-byte aligned; anything else takes a slower
 *     element-wise kernel with identical results.
 *   - Half-precision values (bf16: the upper half of the IEEE fp32 word; or IEEE binary16, see MLPO_HALF_*) are
 *     passed as raw uint16_t bit patterns.  Where a comment says bf16 below, read "the call's half format".
 */
#ifndef MLPO_H
#define MLPO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MLPO_OK 0
#define MLPO_EINVAL (-1) /* NULL / misaligned pointer, bad size, bad hyper-parameter, bad tier */
#define MLPO_EHIP (-2)   /* a HIP runtime call failed; mlpo_last_error() names it */
#define MLPO_ENOMEM (-3) /* a caller-provided workspace or staging buffer is too small */
#define MLPO_EIO (-4)    /* reading or writing a file-tier subgroup failed; mlpo_last_error() gives errno's text */

/* Hyper-parameters, fp32 as stored.  bias_correction != 0 applies the 1 - beta^t corrections.  l2_mode 0 is AdamW
 * (decoupled weight decay: p shrinks by the factor 1 - lr * weight_decay); l2_mode 1 is Adam with the decay term
 * weight_decay * p added to the gradient before the moments are updated (the paper names Adam without saying which
 * form, Section 3.2 "Cache-Friendly Ordering"; every workload here uses AdamW). */
typedef struct {
    float lr, beta1, beta2, eps, weight_decay;
    int32_t bias_correction;
    int32_t l2_mode;
} mlpo_adamw_hparams;

/* One subgroup (Section 2 "Sharded Model and Optimizer States Into Subgroups"): n elements of fp32 master parameters
 * p, momentum m, variance v, the bf16 gradients g that drive the update and the bf16 working copy p16 that receives
 * the downcast parameters.  g and p16 are plain arrays of n elements; p16 is always device memory, g normally too.
 * tier says where p, m, v live: MLPO_TIER_HBM (device), MLPO_TIER_HOST (pinned host), or MLPO_TIER_HOST_GRADS
 * (pinned host, and g is pinned host memory as well).  Pinned host memory here is memory from hipHostMalloc (or a
 * framework's pinned allocator on top of it), which the device can address: direct mode and the slot cache work on
 * it from kernels, not through copies.
 * Host-side gradients (the paper keeps the half-precision gradients in a host accumulation buffer and converts them
 * only when the update needs them, Section 3.2 "Delayed In-place Mixed-Precision Gradient Conversion"): with
 * MLPO_TIER_HOST_GRADS, mlpo_grad_unscale_norm reads g over the link (2 bytes per element); mlpo_stream_update in
 * staged mode brings each piece's gradients into the staging slot together with its state (14 bytes per element in,
 * 12 out) and in direct mode reads them in place; the upcast happens in registers as always.  A MLPO_TIER_HOST
 * subgroup whose g is pinned host memory is also accepted by mlpo_grad_unscale_norm and by direct mode.
 *
 * MLPO_TIER_FILE: the fp32 state lives in a file (the slower alternative path of the offloaded tier, Section 3.2
 * "Unified Multi-level, Multi-path Asynchronous Offloading using Virtual Tiers"); p, m, v must be NULL, the layout
 * must be tiled, and mlpo_stream_cfg.files says where the state is.  g and p16 are device memory.  Accepted by
 * mlpo_stream_update in direct mode only.
 *
 * Layout of the fp32 state, chosen by tile_elems:
 *   0      planar: p, m, v are three independent arrays of n floats.
 *   T > 0  tiled: the state of the subgroup is ONE buffer of mlpo_state_floats(n, T) floats that starts at p and
 *          holds, for every run of T consecutive elements, T floats of p, then T of m, then T of v:
 *          x[i] of array X in {p, m, v} lives at X + (i / T) * 3T + (i % T), with m == p + T and v == p + 2T
 *          (checked).  T must be a multiple of 1024, p 256-byte aligned, g and p16 8-byte aligned.  With T = 8192
 *          (MLPO_TILE_DEFAULT) the three values an element needs sit close together and the whole update sweeps
 *          one address stream instead of three: the layout the library is fastest on.  A host-tier tiled subgroup
 *          also moves as one transfer per direction instead of three. */
#define MLPO_TIER_HBM 0
#define MLPO_TIER_HOST 1
#define MLPO_TIER_HOST_GRADS 2
#define MLPO_TIER_FILE 3
#define MLPO_TILE_DEFAULT 8192
/* Format of g and p16 (the paper allows FP16 or BF16, Section 2 "Mixed Precision Training", and writes FP16 in
 * Algorithm 1): bf16, the upper half of the fp32 word, or IEEE binary16.  All subgroups of one call share it. */
#define MLPO_HALF_BF16 0
#define MLPO_HALF_FP16 1
typedef struct {
    float* p;
    float* m;
    float* v;
    const uint16_t* g;
    uint16_t* p16;
    uint64_t n;
    int32_t tier;
    int32_t tile_elems;
    int32_t half_format; /* MLPO_HALF_BF16 (0) or MLPO_HALF_FP16 */
    int32_t lead;        /* 0, or see below (HBM tier, tiled layout) */
} mlpo_subgroup;
/* lead: the subgroup's elements start `lead` slots into the tiled buffer instead of at its beginning: x[i] lives at
 * X + ((i + lead) / T) * 3T + ((i + lead) % T), the first `lead` slots of p, m and v are padding that is never read
 * or written, and the buffer holds mlpo_state_floats(n + lead, T) floats.  g and p16 still point at the subgroup's
 * first value.  A multiple of 4 below 1024.  Why: g and p16 are slices of the caller's flat arrays and start wherever
 * the subgroup boundaries fall, rarely on a 128-byte line, while the state buffer is aligned; every workgroup's piece
 * of g and p16 then straddles lines that it shares with its neighbours, which costs about 3 % of the update's
 * speed (2.4 % for p16, whose lines are then written in two halves, 0.3 % for g).  With
 * lead = (address of p16 / 2) mod 64 the lines of p16 (and of g, if it is cut the same way) begin at the same
 * elements as the lines of p, m, v.  Accepted for MLPO_TIER_HBM subgroups only - the offloaded tiers are
 * bound by the link - and such a subgroup cannot be given a flush target. */

/* The lead that lines a subgroup's state up with its p16 array: (address of p16 / 2) mod 64.  A multiple of 4 when
 * p16 is 8-byte aligned, as the tiled layout requires. */
int32_t mlpo_line_lead(const void* p16);

/* Floats in the state buffer of a tiled subgroup: ceil(n / tile_elems) * 3 * tile_elems (3 * n if tile_elems is 0). */
uint64_t mlpo_state_floats(uint64_t n, int32_t tile_elems);

/*
 * Conversion between the two layouts (for state that arrives planar, e.g. from a checkpoint, or has to leave that
 * way).  mlpo_state_pack writes the tiled buffer `state` (mlpo_state_floats(n + lead, tile_elems) floats; the padding
 * in front and the unused tail of the last tile are set to zero) from three arrays of n floats; mlpo_state_unpack
 * does the reverse.  lead as in mlpo_subgroup (0 for a subgroup without padding).  All pointers must be addressable
 * by the device (device memory or pinned host memory) and 4-byte aligned; source and destination must not overlap.
 * One kernel on `stream`.  Errors: MLPO_EINVAL, MLPO_EHIP.
 */
int mlpo_state_pack(const float* p, const float* m, const float* v, uint64_t n, int32_t tile_elems, int32_t lead,
                    float* state, void* stream);
int mlpo_state_unpack(const float* state, uint64_t n, int32_t tile_elems, int32_t lead, float* p, float* m, float* v,
                      void* stream);

/* The four scalars that link the gradient pass to the update, kept in device memory so that no host round trip is
 * needed between the two (16 bytes, 16-byte aligned). */
typedef struct {
    float norm;         /* L2 norm of the unscaled gradients of all subgroups */
    float clip_coef;    /* max_norm / (norm + 1e-6) if clipping is on and norm > max_norm, else 1 */
    float gmul;         /* inv_scale * clip_coef: the factor the update applies to every raw gradient */
    uint32_t found_inf; /* 1 if any gradient is +-inf or NaN, or if the norm does not fit fp32 (the whole step must
                           then be skipped), else 0 */
} mlpo_step_scalars;

/* Text of the last error on the calling thread ("" if none).  The pointer stays valid until the thread's next
 * failing call. */
const char* mlpo_last_error(void);

/* Library version, major * 10000 + minor * 100 + patch. */
int32_t mlpo_version(void);

/* Bytes of device workspace mlpo_grad_unscale_norm needs (a constant; 256-byte alignment required). */
size_t mlpo_norm_workspace_bytes(void);

/*
 * Gradient pass before the update (the usual mixed-precision convention; Section 2 "Mixed Precision Training" of the
 * paper only says that the half-precision gradients are widened to fp32 for the optimizer): over the gradients of ALL
 * n_sg subgroups
 *   norm      = sqrt( sum_i ((double)(f32(g_i) * inv_scale))^2 ), rounded to fp32,
 *   found_inf = any g_i with its exponent field all ones (8 bits in bf16, 5 in fp16), or norm not finite (finite
 *               gradients whose norm overflows fp32: the clip factor would be 0 or infinity would enter the moments),
 *   clip_coef, gmul as described at mlpo_step_scalars.
 * The sum is taken in fp64 in a fixed order: the result is deterministic for a given argument list.
 *
 *   sg, n_sg     host array of subgroups; only .g and .n are read (n may be 0).  n_sg >= 0.
 *   inv_scale    1 / loss scale, finite and > 0.
 *   max_norm     clipping bound; <= 0 turns clipping off.
 *   workspace    device, >= mlpo_norm_workspace_bytes(), 256-byte aligned; contents need not be preserved or cleared.
 *   out          device, 16-byte aligned; written by the last kernel enqueued.
 *   stream       hipStream_t.
 * Errors: MLPO_EINVAL (arguments), MLPO_ENOMEM (workspace_bytes too small), MLPO_EHIP.
 */
int mlpo_grad_unscale_norm(const mlpo_subgroup* sg, int32_t n_sg, float inv_scale, float max_norm, void* workspace,
                           size_t workspace_bytes, mlpo_step_scalars* out, void* stream);

/*
 * The same gradient pass, which also leaves a device copy of the gradients it reads: for subgroups whose
 * half-precision gradients live in pinned host memory (the paper's placement, Section 3.2 "Delayed In-place
 * Mixed-Precision Gradient Conversion").  The pass has to read them over the link anyway; with the copy in HBM
 * (2 bytes per element of spare device memory) the update that follows reads them there - describe the subgroup to
 * mlpo_stream_update as MLPO_TIER_HOST with g = the copy - and 14 instead of 16 bytes per element cross the link
 * inbound, whichever way the gradients were accumulated.
 *   keep   host array of n_sg device pointers; keep[i] receives the n elements of sg[i].g, NULL keeps no copy of that
 *          subgroup.  keep[i] and sg[i].g must agree modulo 16 bytes and must not overlap.
 * Everything else as for mlpo_grad_unscale_norm; the record is the same bit for bit.
 * Errors: MLPO_EINVAL, MLPO_ENOMEM, MLPO_EHIP.
 */
int mlpo_grad_unscale_norm_keep(const mlpo_subgroup* sg, int32_t n_sg, uint16_t* const* keep, float inv_scale,
                                float max_norm, void* workspace, size_t workspace_bytes, mlpo_step_scalars* out,
                                void* stream);

/*
 * The same gradient pass for callers that cannot allocate and have no workspace to pass: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The per-workgroup partial sums go to an array in
 * the library's own device image (196 864 bytes, one copy per GPU, held until the process ends) instead of a
 * caller's workspace; the call allocates nothing and calls no allocating routine (no timing events either: its
 * launches are never recorded for mlpo_kernel_times).  Same kernels, same order of summation, hence the same record
 * bit for bit as mlpo_grad_unscale_norm.  Arguments as there.  Limits: at most MLPO_STATIC_MAX_SUBGROUPS subgroups
 * and MLPO_STATIC_MAX_ELEMENTS gradients per call; more gives MLPO_EINVAL.
 * Nothing in the array has to start at zero (every partial a call reads was written by that call), so there is
 * nothing to clear.  All calls on one GPU share that GPU's array: calls that overlap on one GPU - two streams, two
 * threads - race and give wrong results; order them.
 * Errors: MLPO_EINVAL, MLPO_EHIP.
 */
#define MLPO_STATIC_MAX_SUBGROUPS 1024
#define MLPO_STATIC_MAX_ELEMENTS (1ull << 40)
int mlpo_grad_unscale_norm_static(const mlpo_subgroup* sg, int32_t n_sg, float inv_scale, float max_norm,
                                  mlpo_step_scalars* out, void* stream);

/*
 * Gradient accumulation over micro-batches into the half-precision accumulation buffer that the update later
 * upcasts on the fly (Section 3.2 "Delayed In-place Mixed-Precision Gradient Conversion"; Section 4.5 runs 1-16
 * backward passes per update).  For every i < n:
 *   first != 0:  acc[i] = g[i]                                  (first micro-batch of a step: no clearing pass needed)
 *   first == 0:  acc[i] = half_rne(f32(acc[i]) + f32(g[i]))     (one fp32 addition; a NaN sum is stored as the
 *                                                                format's quiet NaN, 0x7FC0 for bf16, 0x7E00 for fp16)
 * The sum of two half-precision values rounded this way is the correctly rounded exact sum in either format.
 *   acc     bf16 accumulation buffer, n elements: device memory, or pinned host memory (then the kernel reads and
 *           writes it over the link, 2 bytes per element each way).
 *   g       bf16 gradients of this micro-batch, n elements, device memory (pinned host memory also works).
 *           Must not overlap acc.  Both 2-byte aligned; the 128-bit path needs acc and g congruent modulo 16 bytes,
 *           otherwise every element is moved on its own (much slower).
 *   blocks  0: one workgroup per 2048 elements (device buffers).  > 0: that many persistent workgroups (<= 4096),
 *           which bounds the requests in flight on the link when acc is on the host; 64 is a good value there.
 *   half_format  MLPO_HALF_BF16 or MLPO_HALF_FP16: the format of acc and g.
 *   stream  hipStream_t.  Asynchronous.  n = 0 is a no-op; n is at most 2^41.
 * Errors: MLPO_EINVAL, MLPO_EHIP.
 */
int mlpo_grad_accumulate(uint16_t* acc, const uint16_t* g, uint64_t n, int32_t first, int32_t blocks,
                         int32_t half_format, void* stream);

/*
 * The same accumulation, which also gathers the gradient statistics of the finished buffer, for the LAST micro-batch
 * of a step: the values it stores are the step's gradients, so their sum of squares (unscaled by inv_scale) and
 * their non-finite flag are taken from registers and mlpo_grad_unscale_norm need not read the buffer again (2 bytes
 * per element saved: over the link when the buffer is in host memory).  Calls for the pieces of one step (one per
 * subgroup, say) add up in the workspace in call order; mlpo_grad_norm_finish then writes the same record as
 * mlpo_grad_unscale_norm would over all the pieces together.
 *   acc, g, n, first, blocks, half_format   as for mlpo_grad_accumulate (first != 0: a step with a single
 *                micro-batch).  The grid is always persistent here (blocks = 0: eight workgroups per compute unit).
 *   inv_scale    1 / loss scale; the same value in every call of the step and in mlpo_grad_norm_finish.
 *   workspace    device, as for mlpo_grad_unscale_norm (same size and alignment); holds the running totals between
 *                the calls, so nothing else may use it until mlpo_grad_norm_finish has run.
 *   begin        != 0 in the first call of a step: the running totals start from zero.
 * n = 0 with begin != 0 just resets the totals.  All calls of a step go to the same stream, or are ordered otherwise.
 * Errors: MLPO_EINVAL, MLPO_ENOMEM, MLPO_EHIP.
 */
int mlpo_grad_accumulate_norm(uint16_t* acc, const uint16_t* g, uint64_t n, int32_t first, int32_t blocks,
                              int32_t half_format, float inv_scale, void* workspace, size_t workspace_bytes,
                              int32_t begin, void* stream);

/* Derives norm, clip coefficient, gradient multiplier and flag (see mlpo_grad_unscale_norm) from the totals that the
 * mlpo_grad_accumulate_norm calls of this step left in workspace, and writes them to out (device, 16-byte aligned).
 * Errors: MLPO_EINVAL, MLPO_ENOMEM, MLPO_EHIP. */
int mlpo_grad_norm_finish(void* workspace, size_t workspace_bytes, float inv_scale, float max_norm,
                          mlpo_step_scalars* out, void* stream);

/*
 * AdamW on HBM-resident subgroups, in place, with the gradient upcast and the parameter downcast fused in
 * (Algorithm 1's convert / update / push steps; Section 3.2 "Delayed In-place Mixed-Precision Gradient Conversion").
 * With the per-step scalars (computed on the host in fp64 and rounded once to fp32)
 *   omb1 = 1 - beta1, omb2 = 1 - beta2, bc1 = 1 - beta1^step, bc2 = 1 - beta2^step (both 1 without bias correction),
 *   step_size = lr / bc1, sqbc2 = sqrt(bc2), decay = 1 - lr * weight_decay
 * every element does, each operation rounded to fp32 once and none fused:
 *   g  = f32(g_bf16) * gmul              (l2_mode: then g = g + weight_decay * p, and decay = 1)
 *   m' = beta1 * m + omb1 * g
 *   v' = beta2 * v + omb2 * (g * g)
 *   p' = p * decay - step_size * (m' / (sqrt(v') / sqbc2 + eps))
 *   p16 = half(p') rounded to nearest, ties to even (fp16: magnitudes from 65520 up become infinity, results below
 *         2^-14 are subnormal)
 *
 *   sg, n_sg     host array; every tier must be MLPO_TIER_HBM; all pointers device; n may be 0.
 *   hp           host pointer.  lr, eps, weight_decay finite and >= 0; 0 <= beta < 1.
 *   step         1-based count of applied steps including this one (>= 1).
 *   scalars      device pointer to the record written by mlpo_grad_unscale_norm, or NULL.  When given, the kernel
 *                reads gmul from it and does nothing at all if found_inf is set (no state, no p16 is written);
 *                when NULL, gmul = 1 and the step is always applied.
 *   stream       hipStream_t.
 * The caller advances its step count only for applied steps.
 * Errors: MLPO_EINVAL, MLPO_EHIP.
 */
int mlpo_adamw_step(const mlpo_subgroup* sg, int32_t n_sg, const mlpo_adamw_hparams* hp, int64_t step,
                    const mlpo_step_scalars* scalars, void* stream);

#define MLPO_MAX_SLOTS 64

/* Memory of which subgroup each staging slot holds, kept by the caller between steps (host memory; zero-initialise
 * once, then leave it to the library).  Passing it in mlpo_stream_cfg.cache turns on the cache-friendly processing of
 * Section 3.2 "Cache-Friendly Ordering": a host-tier subgroup that is still in a slot from the previous step is
 * updated there with no transfer at all, and a slot is copied back to the host only when another subgroup needs it
 * (lazy flush).  Reversing the processing order from one step to the next makes the subgroups processed last the
 * ones processed first next time, so each step moves n_host - n_slots subgroups per direction instead of n_host.
 * While a subgroup sits dirty in a slot its host copy is stale; mlpo_stream_flush brings the host tier up to date. */
typedef struct {
    uint32_t magic;   /* 0 = not yet used */
    int32_t n_slots;
    uint64_t clock;   /* logical time of the last update */
    int32_t owner[MLPO_MAX_SLOTS];       /* index of the subgroup in each slot, -1 = empty */
    uint8_t dirty[MLPO_MAX_SLOTS];       /* the slot is newer than the host copy */
    uint64_t stamp[MLPO_MAX_SLOTS];      /* logical time of the slot's last update */
    const void* owner_p[MLPO_MAX_SLOTS]; /* p of the owning subgroup, to notice a changed subgroup table */
    uint64_t fetches, flushes, hits;     /* transfers issued and transfers saved since the cache was first used */
} mlpo_slot_cache;

/* Where the fp32 state of a MLPO_TIER_FILE subgroup lives: mlpo_state_floats(n, tile_elems) floats in the tiled
 * layout, starting offset bytes into the open file fd (offset a multiple of 4096).  The library only calls pread and
 * pwrite on the descriptor and never closes it.  A descriptor opened with O_DIRECT is served through page-aligned
 * blocks of the library's own, because memory pinned by the HIP runtime cannot be the target of direct I/O; a file
 * in tmpfs without holes (pageable host memory with a name) is copied through a mapping, which lets all the threads
 * write at once; anything else is read and written with plain pread / pwrite. */
typedef struct {
    int32_t fd;
    int32_t reserved; /* must be 0 */
    uint64_t offset;
} mlpo_file_extent;

/* Where the fp32 state of a subgroup goes after the update when that is not where it was read from.
 * Algorithm 1 assigns the path anew every time a subgroup is flushed, so that a re-estimated Eq. 1 (Section 3.3)
 * takes effect; as the update reads the whole state and writes the whole state anyway, sending it somewhere else
 * costs nothing extra: pinned -> file has no read from the file, file -> pinned has no write to it, and a subgroup
 * that enters or leaves HBM crosses the link once instead of twice.  Direct mode, tiled layout only; entries of
 * planar subgroups must say MLPO_FLUSH_IN_PLACE.  Allowed: from pinned memory or a file to any of the three tiers,
 * from HBM to pinned memory or a file (a MLPO_TIER_HOST_GRADS subgroup cannot go to HBM: its gradients would have to
 * move as well).  After an applied step the caller describes the subgroup by its new home (what the old one holds
 * is then stale); a skipped step moves nothing and the state stays where it was.  The targets of different
 * subgroups must not overlap each other or any other subgroup's state: the library checks a target only against
 * its own subgroup's current state. */
#define MLPO_FLUSH_IN_PLACE (-1)
typedef struct {
    int32_t tier;          /* MLPO_FLUSH_IN_PLACE, MLPO_TIER_HBM, MLPO_TIER_HOST or MLPO_TIER_FILE */
    int32_t reserved;      /* must be 0 */
    float* state;          /* MLPO_TIER_HBM / MLPO_TIER_HOST: device / pinned host buffer of
                              mlpo_state_floats(n, tile_elems) floats, 256-byte aligned, not overlapping the
                              subgroup's current state; the new p, m, v are stored there in the tiled layout */
    mlpo_file_extent file; /* MLPO_TIER_FILE: where the state is written (may be the extent it came from) */
} mlpo_flush_target;

/* What the file path of one mlpo_stream_update call did: bytes read and written, the time its threads spent
 * inside pread / pwrite (summed over the threads of a direction) and the wall time from the first read to the end of
 * the last write.  Section 3.3: the observed bandwidth of a path, B_i = bytes / seconds, is what
 * mlpo_update_bandwidth takes; bytes_read / wall_seconds is the rate at which the path delivered subgroups. */
typedef struct {
    uint64_t bytes_read, bytes_written;
    double read_seconds, write_seconds;
    double wall_seconds;
} mlpo_file_stats;

/* The same per file path (paths are told apart by the file system their descriptors lie on; path_id is that file
 * system's device number as fstat reports it, so a caller can match the entries with its descriptors).  used = 0
 * marks entries beyond the number of paths of the call. */
typedef struct {
    uint64_t path_id;
    int32_t used;
    int32_t reserved;
    mlpo_file_stats stats;
} mlpo_path_stats;

/* Configuration of the tiered pipeline.
 * mode MLPO_STREAM_STAGED: host-tier subgroups are fetched into device staging slots by asynchronous copies, updated
 *   there and flushed back (three stages on three streams, at most n_slots subgroups or chunks in flight).
 * mode MLPO_STREAM_DIRECT: the update kernel reads and writes the pinned host state in place over the link; there is
 *   no staging and nothing to copy.  The bound on what is in flight is direct_blocks, the number of persistent
 *   workgroups working on the host tier at once; the rest of the GPU updates the HBM-tier subgroups meanwhile.  The
 *   host-tier kernel is enqueued on the h2d stream, the HBM-tier kernel on the compute stream. */
#define MLPO_STREAM_STAGED 0
#define MLPO_STREAM_DIRECT 1
#define MLPO_CHUNK_WHOLE UINT64_MAX
typedef struct {
    int32_t n_slots;       /* staged: staging slots = bound on subgroups (or chunks) in flight; 1..MLPO_MAX_SLOTS */
    int32_t mode;          /* MLPO_STREAM_STAGED or MLPO_STREAM_DIRECT */
    uint64_t chunk_elems;  /* elements per transfer of an offloaded subgroup (staged mode; direct mode when pieces pass
                              through bounce buffers or change their home; otherwise unused there).
                              0 = the library chooses: subgroups of more than 2^25 elements move in pieces of 2^24
                              elements (rounded down to whole layout tiles), which shortens the pipeline's fill and
                              drain from a subgroup to a piece; smaller ones move whole.  MLPO_CHUNK_WHOLE = a whole
                              subgroup per transfer.  Any other value: that many elements, a multiple of 4 and of
                              every tile_elems in use (staged mode: pieces below 2^23 - 2^24 elements, depending on
                              the HIP runtime in the process, have been measured at 0.4-0.8 of the rate of larger
                              ones: copies that wait on other streams' events piece after piece overlap poorly;
                              results never depend on the value) */
    void* staging;         /* staged: device, 256-byte aligned, caller-owned */
    size_t staging_bytes;  /* staged: >= mlpo_stream_staging_bytes(...) */
    void* h2d;             /* hipStream_t for host-to-device copies (direct: for the host-tier kernel) */
    void* compute;         /* hipStream_t for kernels */
    void* d2h;             /* hipStream_t for device-to-host copies.  If h2d and d2h are both NULL the library uses a
                              pair of copy streams of its own (created on first use, kept until mlpo_shutdown); this
                              is the recommended setting: streams handed out by a framework's pool can share a
                              hardware queue, and the two copy directions then take turns instead of overlapping */
    int32_t direct_blocks; /* persistent workgroups of a kernel that works over the link (direct mode: the update of the
                              host tier; slot cache: the kernel that exchanges a slot's occupants); 0 = default
                              (64 and 80: the counts that were fastest on the 13 x 100 M-element workload); at most
                              4096 */
    int32_t reserved;      /* must be 0 */
    mlpo_slot_cache* cache; /* staged: slots keep their subgroups between steps; NULL = off.  Every slot then holds a
                               whole subgroup (size the staging buffer with MLPO_CHUNK_WHOLE).  A miss of a tiled
                               subgroup into a slot that is empty, already written back, or holds a subgroup of the
                               same tile_elems is served by kernels on the h2d stream (direct_blocks workgroups):
                               one launch updates the newcomer on its way from pinned memory into the slot and sends
                               what the slot held to the old occupant's home, tile by tile (where the two differ in
                               length, the rest of the longer one follows on the same stream).  Any other miss moves
                               by copies, in pieces of chunk_elems (tiled layout; planar subgroups enter and leave
                               whole) */
    /* The file path (direct mode; all zero / NULL when no subgroup is MLPO_TIER_FILE): */
    const mlpo_file_extent* files; /* host array with one entry per subgroup of the table; only the entries of
                                      MLPO_TIER_FILE subgroups are read */
    void* bounce;          /* pinned host memory (hipHostMalloc), 4096-byte aligned, caller-owned: file_slots buffers
                              through which file-tier pieces pass (read from the file, updated in place by the
                              kernel over the link, written back) */
    size_t bounce_bytes;   /* >= mlpo_stream_bounce_bytes(...) */
    int32_t file_slots;    /* 1..MLPO_MAX_SLOTS: bounce buffers = bound on file-tier pieces in flight.  They are divided
                              evenly among the file paths in use (files on different file systems: each path has
                              its own buffers, so at least one per path; 3 per path let read, update and write
                              overlap) */
    int32_t file_threads;  /* threads per direction AND PATH that move the pieces between file and bounce buffers,
                              each an equal share of every piece; 0 = default (2); at most 16 */
    mlpo_file_stats* file_stats; /* host pointer or NULL: receives what the file path moved and how long it took
                                    (all zero after a skipped step or when nothing is file-tier) */
    const mlpo_flush_target* flush_to; /* direct mode: host array with one entry per subgroup of the table, or NULL
                                          (everything goes back to where it came from).  A target in a file needs
                                          the bounce buffers even if no subgroup is file-tier yet */
    mlpo_path_stats* path_stats;   /* host array of path_stats_cap entries or NULL: receives what each file path moved,
                                      in the order in which the paths first come up in the processing order: the
                                      observed bandwidths that Eq. 1's re-estimation takes, path by path */
    int32_t path_stats_cap;        /* entries in path_stats (0 with NULL) */
    int32_t reserved2;             /* must be 0 */
} mlpo_stream_cfg;

/* Staging bytes needed for these subgroups under this n_slots / chunk_elems (0 if no subgroup is host-tier).  With a
 * slot cache pass MLPO_CHUNK_WHOLE: its slots hold whole subgroups. */
size_t mlpo_stream_staging_bytes(const mlpo_subgroup* sg, int32_t n_sg, int32_t n_slots, uint64_t chunk_elems);

/* Bounce bytes needed for the subgroups that come from a file or (flush_to, may be NULL) go to one, under this
 * file_slots / chunk_elems (0 if there are none). */
size_t mlpo_stream_bounce_bytes(const mlpo_subgroup* sg, int32_t n_sg, int32_t file_slots, uint64_t chunk_elems,
                                const mlpo_flush_target* flush_to);

/*
 * One update phase over subgroups of all tiers (Algorithm 1, with the fetch / update / flush overlap of Section 3.4
 * and the bound on subgroups in flight that Section 3.2 "Optimized Virtual Tier Concurrency Control" motivates).
 * HBM-tier subgroups are updated in place as in mlpo_adamw_step.  In staged mode each host-tier subgroup (or chunk of
 * one) is copied host-to-device into a free staging slot on the h2d stream, updated there on the compute stream (g
 * and p16 are read/written at their device homes; the gradients of a MLPO_TIER_HOST_GRADS subgroup travel into the
 * slot with the state; with a slot cache a hit fetches the step's gradients into the slot and a miss served by the
 * exchanging kernel reads them where they are), and copied back on the d2h stream;
 * a slot is reused only after its copy back has completed, so at most n_slots transfers are in flight.  In direct
 * mode the kernel works on the host state in place.  Results are bit-identical to the resident path whatever mode,
 * n_slots, chunk_elems, direct_blocks and order are.
 *
 * File-tier subgroups (direct mode): reading threads bring pieces of chunk_elems elements (see there for 0) from
 * the file into free bounce buffers, the update kernel works on a bounce buffer in place over the
 * link with direct_blocks workgroups, and writing threads put the piece back into the file once its kernel has
 * finished; a bounce buffer is refilled only after its piece has been written, so at most file_slots pieces are in
 * flight (the three-stage overlap of Section 3.4 on this path).  Files on different file systems are different
 * paths: each has its own reading and writing threads, its own share of the bounce buffers and its own place in the
 * queue, so a slow disk never holds up a faster path (Section 3.2: every path of a virtual tier has workers of its
 * own).  Host-tier and file-tier work share the link, so their kernels go to one stream, in pieces of chunk_elems, a
 * file-tier piece as soon as it has been read (the paths take turns) and host-tier pieces in between: the files
 * work while the link is busy with the host tier (the multi-path overlap of Section 3.2).  With file-tier subgroups the call returns only when their state is back in the file; the rest is
 * enqueued as usual.
 *
 * Flush targets (cfg->flush_to, direct mode; see mlpo_flush_target): a subgroup with a target is cut into pieces of
 * chunk_elems like the others and runs on the link's stream; its kernel loads the old state from the old home and
 * stores the new state at the new one.  A piece whose state comes from a file or goes to one passes through a bounce
 * buffer and counts against file_slots; the call then returns when the file holds what goes there, while stores to
 * pinned memory or HBM are complete when the compute stream has caught up, as for any other subgroup.
 *
 *   order        host array, a permutation of 0..n_sg-1 giving the processing order, or NULL for ascending.
 *   scalars      device pointer or NULL, as for mlpo_adamw_step.  When given, the call first copies the record to the
 *                host (a 16-byte copy and a wait on the compute stream) because the transfers are issued from the
 *                host: a step with found_inf set moves no data at all.  Direct mode without file-tier subgroups and
 *                flush targets issues nothing from the host - its kernels read the flag on the device and leave at
 *                once when it is set - so there the copy and the wait are left out when applied is NULL: the call
 *                then only enqueues, and a caller may capture it in a HIP graph (with h2d and compute given).
 *   applied      host pointer or NULL; receives 1 if the step was enqueued, 0 if it was skipped (with the wait that
 *                knowing this takes).
 *   cfg          host pointer.  The three streams may be distinct (needed for overlap) or equal; see the note at
 *                mlpo_stream_cfg.d2h about leaving the two copy streams to the library.
 * On return everything is enqueued; the compute stream is made to wait for the last copy back, so synchronising
 * cfg->compute alone is enough to see the final state.  Calls sharing a staging buffer must not overlap.
 * Errors: MLPO_EINVAL, MLPO_ENOMEM (staging or bounce too small), MLPO_EHIP, MLPO_EIO (a read or write failed or
 * was short; the file-tier state is then undefined for the pieces in flight).
 */
int mlpo_stream_update(const mlpo_subgroup* sg, int32_t n_sg, const int32_t* order, const mlpo_adamw_hparams* hp,
                       int64_t step, const mlpo_step_scalars* scalars, const mlpo_stream_cfg* cfg, int32_t* applied);

/*
 * Copies every subgroup that a slot of cfg->cache holds in a newer version than the host back to the host tier
 * (needed before the host copy is read: a checkpoint, the end of training, a change of the subgroup table).  The
 * slots keep their subgroups.  sg, n_sg and cfg as passed to mlpo_stream_update.  Enqueues on the flush stream; the
 * compute stream waits for it.  Errors: MLPO_EINVAL, MLPO_ENOMEM, MLPO_EHIP.
 */
int mlpo_stream_flush(const mlpo_subgroup* sg, int32_t n_sg, const mlpo_stream_cfg* cfg);

/*
 * Allocation of subgroups to the paths of a virtual tier in proportion to their bandwidth (Eq. 1, Section 3.3):
 *   T_i = ceil(M * B_i / sum_j B_j), then corrected so that the T_i add up to M.
 * The paper does not say how to adjust; here the surplus is taken back one subgroup at a time from the tier that
 * would finish last (largest T_i / B_i), which keeps the finishing times of the paths as close as integers allow.
 *   n_subgroups  M >= 0.
 *   n_tiers      N, 1..64.
 *   bandwidth    host, N values B_i > 0, any common unit (subgroups or bytes per second).
 *   capacity     host, N values or NULL: the most subgroups tier i can hold, < 0 = unlimited.  A tier that cannot hold
 *                its share keeps what it can, and Eq. 1 is applied again to the rest (this is how a small fast tier
 *                such as HBM enters).
 *   count        host, N values out: T_i.
 *   tier_of_subgroup  host, M values out or NULL: the tier of each subgroup id; slower tiers get the lower ids (after
 *                an ascending pass the high ids are the ones still on the fast tiers, Section 3.2).
 * Errors: MLPO_EINVAL; MLPO_ENOMEM if the capacities cannot hold M subgroups.
 */
int mlpo_assign_tiers(int32_t n_subgroups, int32_t n_tiers, const double* bandwidth, const int32_t* capacity,
                      int32_t* count, int32_t* tier_of_subgroup);

/*
 * Online re-estimation of the bandwidths (Section 3.3): after an iteration B_i becomes the average bandwidth observed
 * on tier i, bytes_moved[i] / seconds[i]; a tier that moved nothing keeps its estimate.  All arrays host, N values.
 */
int mlpo_update_bandwidth(int32_t n_tiers, double* bandwidth, const double* bytes_moved, const double* seconds);

/*
 * Per-kernel timing, for measurement (Section 4.3 of the paper reports the effective I/O throughput
 * 2 * bytes / (read time + write time) per subgroup; the roofline figures need a kernel's own duration).  After
 * mlpo_kernel_timing(1) every launch of the fused update kernel (which = 0) and of the gradient pass's streaming
 * kernel (which = 1) is stamped with HIP events that carry the dispatch's own begin and end on the device, and every
 * staged-mode transfer is bracketed by event markers on its copy stream (which = 2: host-to-device fetches,
 * which = 3: device-to-host flushes, one entry per subgroup or chunk).  which = 4: the 128-bit kernel of
 * mlpo_grad_accumulate.  mlpo_kernel_timing(0) turns it off and forgets what was recorded.  Process-wide; results
 * are the same with and without it.
 * mlpo_kernel_times waits for the recorded items, writes their durations in milliseconds to ms[0..cap) in issue order
 * (host memory), stores the number written in *count and forgets them.  At most 16384 items per kind are kept
 * between calls.
 * Errors: MLPO_EINVAL, MLPO_EHIP.
 */
int mlpo_kernel_timing(int32_t on);
int mlpo_kernel_times(int32_t which, float* ms, int32_t cap, int32_t* count);

/* Releases the events and copy streams the pipeline caches (optional; safe to call when idle). */
int mlpo_shutdown(void);

#ifdef __cplusplus
}
#endif
#endif /* MLPO_H */
