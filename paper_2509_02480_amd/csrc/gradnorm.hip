// Gradient pass before the update: non-finite check, L2 norm of the unscaled gradients, clip factor (gfx950).
//
// Pass 1 streams the half-precision gradients of a table of subgroups once (2 bytes per element) with 128-bit
// non-temporal loads after peeling each subgroup's unaligned head.  Every workgroup owns one contiguous run of 16 KiB
// tiles of ONE subgroup - as many tiles as it takes to cover the table with the workgroups the workspace has partials
// for - so it looks its subgroup up once and then only advances a pointer, with the loads of its next tile issued
// before the current tile is summed.  There are more workgroups than the chip holds at a time (a bare read sweep of
// this size is fastest as many short workgroups: the hardware's dispatcher keeps the memory system fed and evens out
// the tail).  Every lane widens its gradients, multiplies by 1/loss-scale in fp32 and accumulates the squares in
// fp64 - four lane operations per element.  The non-finite test costs nothing per element: squares are never
// negative and the largest finite half-precision value squared, times any element count, is far below the fp64
// range, so a lane's sum is non-finite exactly when one of its unscaled gradients was.  Lanes are combined by
// wavefront shuffles, wavefronts through LDS, and each block writes one fp64 partial and one flag.  Pass 2 (one
// block) adds the partials in a fixed order and derives norm, clip coefficient and the gradient multiplier.  No
// atomics: the result depends only on the argument list, not on scheduling.
#include <hip/hip_ext.h>
#include <math.h>

#include <mutex>

#include "mlpo_internal.h"

#pragma clang fp contract(off)

namespace mlpo {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBlock = 256;
constexpr int kUnroll = 4;                // 128-bit loads a lane has in flight
constexpr bool kSweep = false;
constexpr uint32_t kPiece = kBlock * 8;   // body elements per 4 KiB piece: one 128-bit load per lane
constexpr int kMaxSg = 96;
constexpr int kMaxGrid = kNormMaxPartials;
constexpr uint64_t kTargetBlocks = kMaxGrid - kMaxSg;  // every subgroup may round its share up by one workgroup

struct NormBatch {
    const uint16_t* body[kMaxSg];  // start of the vector body, on a 128-byte line
    uint64_t n_body[kMaxSg];       // elements from body to the end of the subgroup
    uint32_t block_begin[kMaxSg + 1];  // prefix sums of workgroups per subgroup
    uint8_t head[kMaxSg];  // elements before body (0..63), handled by the subgroup's first workgroup
    int64_t keep[kMaxSg];  // KEEP kernels: elements from a gradient to its device copy (0 = this array keeps none)
    int32_t n_sg;
    int32_t half;  // MLPO_HALF_BF16 or MLPO_HALF_FP16
    uint32_t pieces_per_block;
};

using Workspace = NormWorkspace;

// Two gradients packed in a 32-bit word / one gradient: unscale in fp32, square and accumulate in fp64.
// HALF: 0 = bf16, 1 = IEEE binary16.
template <int HALF>
__device__ __forceinline__ void accum_word(uint32_t w, float inv_scale, double& a0, double& a1) {
    float u0, u1;
    if constexpr (HALF == 0) {
        u0 = __uint_as_float(w << 16) * inv_scale;
        u1 = __uint_as_float(w & 0xFFFF0000u) * inv_scale;
    } else {
        u0 = (float)__builtin_bit_cast(_Float16, (uint16_t)w) * inv_scale;
        u1 = (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16)) * inv_scale;
    }
    a0 = fma((double)u0, (double)u0, a0);
    a1 = fma((double)u1, (double)u1, a1);
}

template <int HALF>
__device__ __forceinline__ void accum_half(uint16_t h, float inv_scale, double& acc) {
    const float u = (HALF == 0 ? __uint_as_float((uint32_t)h << 16) : (float)__builtin_bit_cast(_Float16, h)) * inv_scale;
    acc = fma((double)u, (double)u, acc);
}

template <int HALF>
__device__ __forceinline__ void accum_vec(u32x4 w, float inv_scale, double& a0, double& a1) {
    accum_word<HALF>(w.x, inv_scale, a0, a1);
    accum_word<HALF>(w.y, inv_scale, a0, a1);
    accum_word<HALF>(w.z, inv_scale, a0, a1);
    accum_word<HALF>(w.w, inv_scale, a0, a1);
}

// This lane's 128-bit word of 4 KiB piece `piece` of a subgroup's body (zero where the lane has none: zero bits are
// the value 0 in both formats and add nothing); the ragged end of the last piece is added to acc on the spot.
// keep != 0: what is read is also stored keep elements further on (the device copy of gradients that live in host
// memory: the update then need not read them over the link a second time).
template <int HALF, bool KEEP>
__device__ __forceinline__ u32x4 fetch(const uint16_t* __restrict__ body, uint64_t n_body, uint64_t piece,
                                       int64_t keep, float inv_scale, double& acc) {
    const uint32_t tid = threadIdx.x;
    const uint64_t e0 = piece * kPiece;
    const u32x4* __restrict__ q = reinterpret_cast<const u32x4*>(body + e0) + tid;
    const uint64_t e = e0 + (uint64_t)tid * 8;
    if (e + 8 <= n_body) {
        const u32x4 w = __builtin_nontemporal_load(q);
        if (KEEP && keep != 0) *reinterpret_cast<u32x4*>(const_cast<uint16_t*>(body) + e + keep) = w;
        return w;
    }
    for (uint64_t j = e; j < n_body; ++j) {
        const uint16_t h = body[j];
        if (KEEP && keep != 0) const_cast<uint16_t*>(body)[(int64_t)j + keep] = h;
        accum_half<HALF>(h, inv_scale, acc);
    }
    const u32x4 zero = {0u, 0u, 0u, 0u};
    return zero;
}

// The streaming part of the kernel below for one format.
template <int HALF, bool KEEP>
__device__ __forceinline__ void stats_run(const NormBatch& b, const float inv_scale, double& a0, double& a1) {
    const uint32_t tid = threadIdx.x;
    const uint32_t blk = blockIdx.x;
    int lo = 0, hi = b.n_sg;  // the subgroup this workgroup belongs to
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (blk >= b.block_begin[mid]) lo = mid; else hi = mid;
    }
    const uint32_t b_in = blk - b.block_begin[lo];
    const uint32_t blocks_s = b.block_begin[lo + 1] - b.block_begin[lo];
    const uint16_t* __restrict__ body = b.body[lo];
    const uint64_t n_body = b.n_body[lo];
    const int64_t keep = KEEP ? b.keep[lo] : 0;
    if (b_in == 0 && tid < b.head[lo]) {
        const uint16_t h = *(body - 1 - tid);
        if (KEEP && keep != 0) const_cast<uint16_t*>(body)[-1 - (int64_t)tid + keep] = h;
        accum_half<HALF>(h, inv_scale, a0);
    }
    const uint64_t n_pieces = (n_body + kPiece - 1) / kPiece;
    const uint32_t per_block = b.pieces_per_block;  // a multiple of kUnroll
    const u32x4 zero = {0u, 0u, 0u, 0u};
    for (uint32_t k0 = 0; k0 < per_block; k0 += kUnroll) {
        u32x4 w[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint64_t k = k0 + u;
            const uint64_t piece = kSweep ? b_in + k * blocks_s : (uint64_t)b_in * per_block + k;
            w[u] = piece < n_pieces ? fetch<HALF, KEEP>(body, n_body, piece, keep, inv_scale, a0) : zero;
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) accum_vec<HALF>(w[u], inv_scale, a0, a1);
    }
}

// KEEP = true: the form that also leaves a device copy of the gradients it reads (see fetch).
template <bool KEEP>
__global__ void __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(8, 8)))
grad_stats_kernel(const NormBatch b, const float inv_scale, Workspace* __restrict__ ws) {
    const uint32_t tid = threadIdx.x;
    double a0 = 0.0, a1 = 0.0;
    if (b.half == 0)
        stats_run<0, KEEP>(b, inv_scale, a0, a1);
    else
        stats_run<1, KEEP>(b, inv_scale, a0, a1);
    double acc = a0 + a1;
    // a sum of squares is non-finite exactly when one of its terms is (see the note at the top)
    uint32_t bad = (uint32_t)!(fabs(acc) <= 1.7976931348623157e308);
    // lanes -> wavefront (shuffle), wavefronts -> block (LDS), fixed order throughout
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        acc += __shfl_down(acc, off, 64);
        bad |= (uint32_t)__shfl_down((int)bad, off, 64);
    }
    __shared__ double s_acc[kBlock / 64];
    __shared__ uint32_t s_bad[kBlock / 64];
    if ((tid & 63u) == 0) {
        s_acc[tid >> 6] = acc;
        s_bad[tid >> 6] = bad;
    }
    __syncthreads();
    if (tid == 0) {
        double t = s_acc[0];
        uint32_t f = s_bad[0];
#pragma unroll
        for (int w = 1; w < kBlock / 64; ++w) {
            t += s_acc[w];
            f |= s_bad[w];
        }
        ws->partial[blockIdx.x] = t;
        ws->flag[blockIdx.x] = f;
    }
}

// One block: folds n_partials partials into the running sum; on the last group derives the outputs.  The kernel is
// all latency (a handful of loads per lane, then a tree), so it uses a full-size block, issues every lane's loads
// before it adds the first, and keeps the tree out of LDS as far as it can: thread t adds partials t, t + 1024, ...
// in that order, every wavefront folds its 64 sums by shuffles, the first wavefront folds the 16 wavefront sums the
// same way - one barrier, a fixed order throughout.
constexpr int kFinishBlock = 1024;
constexpr int kFinishLoads = 16;  // loads a lane issues together (16 x 1024 covers every partial of one launch)
__global__ void __launch_bounds__(kFinishBlock) grad_finish_kernel(Workspace* __restrict__ ws, const int n_partials,
                                                                   const int first, const int last,
                                                                   const float inv_scale, const float max_norm,
                                                                   mlpo_step_scalars* __restrict__ out) {
    const int tid = (int)threadIdx.x;
    double acc = 0.0;
    uint32_t bad = 0;
    for (int i0 = tid; i0 < n_partials; i0 += kFinishBlock * kFinishLoads) {
        double x[kFinishLoads];
        uint32_t f[kFinishLoads];
#pragma unroll
        for (int k = 0; k < kFinishLoads; ++k) {
            const int i = i0 + k * kFinishBlock;
            x[k] = i < n_partials ? ws->partial[i] : 0.0;
            f[k] = i < n_partials ? ws->flag[i] : 0u;
        }
#pragma unroll
        for (int k = 0; k < kFinishLoads; ++k) {
            acc += x[k];
            bad |= f[k];
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        acc += __shfl_down(acc, off, 64);
        bad |= (uint32_t)__shfl_down((int)bad, off, 64);
    }
    __shared__ double s_acc[kFinishBlock / 64];
    __shared__ uint32_t s_bad[kFinishBlock / 64];
    if ((tid & 63) == 0) {
        s_acc[tid >> 6] = acc;
        s_bad[tid >> 6] = bad;
    }
    __syncthreads();
    if (tid < 64) {
        acc = tid < kFinishBlock / 64 ? s_acc[tid] : 0.0;
        bad = tid < kFinishBlock / 64 ? s_bad[tid] : 0u;
#pragma unroll
        for (int off = kFinishBlock / 128; off > 0; off >>= 1) {
            acc += __shfl_down(acc, off, 64);
            bad |= (uint32_t)__shfl_down((int)bad, off, 64);
        }
    }
    if (tid == 0) {
        double sum = acc;
        uint32_t f = bad;
        if (!first) {
            sum += ws->running_sum;
            f |= ws->running_flag;
        }
        if (last) {
            const float norm = (float)sqrt(sum);
            // a norm that does not fit fp32 (finite gradients can do that: two of the largest bf16 value suffice)
            // would make the clip factor 0 or feed infinity into the moments: such a step is skipped as well
            if (!(norm <= 3.402823466e38f)) f = 1u;
            float coef = 1.0f;
            if (max_norm > 0.0f && norm > max_norm) coef = max_norm / (norm + 1e-6f);
            out->norm = norm;
            out->clip_coef = coef;
            out->gmul = inv_scale * coef;
            out->found_inf = f ? 1u : 0u;
        } else {
            ws->running_sum = sum;
            ws->running_flag = f;
        }
    }
}

// Cuts the batch into workgroups and launches it, then the fold.  pieces[i] = 4 KiB pieces of entry i (at least one,
// so that an array that is all head still has a workgroup).
int flush(NormBatch& b, const uint64_t* pieces, bool first, bool last, float inv_scale, float max_norm, Workspace* ws,
          mlpo_step_scalars* out, hipStream_t st, bool may_time, bool keeps) {
    uint32_t grid = 0;
    if (b.n_sg > 0) {
        uint64_t total = 0;
        for (int i = 0; i < b.n_sg; ++i) total += pieces[i];
        uint64_t per_block = (total + kTargetBlocks - 1) / kTargetBlocks;  // >= 1, below 2^32 (n <= 2^48 each)
        per_block = (per_block + kUnroll - 1) / kUnroll * kUnroll;
        b.pieces_per_block = (uint32_t)per_block;
        b.block_begin[0] = 0;
        for (int i = 0; i < b.n_sg; ++i)
            b.block_begin[i + 1] = b.block_begin[i] + (uint32_t)((pieces[i] + per_block - 1) / per_block);
        grid = b.block_begin[b.n_sg];  // <= kTargetBlocks + n_sg <= kMaxGrid
        hipEvent_t t0, t1;
        const auto kernel = keeps ? grad_stats_kernel<true> : grad_stats_kernel<false>;
        if (may_time && timing_enabled() && timing_acquire(kTimedGradPass, &t0, &t1))
            hipExtLaunchKernelGGL(kernel, dim3(grid), dim3(kBlock), 0, st, t0, t1, 0, b, inv_scale, ws);
        else
            hipLaunchKernelGGL(kernel, dim3(grid), dim3(kBlock), 0, st, b, inv_scale, ws);
        MLPO_HIP(hipGetLastError());
    }
    return launch_norm_fold(ws, (int)grid, first, last, inv_scale, max_norm, out, st);
}

}  // namespace

int launch_norm_fold(NormWorkspace* ws, int n_partials, bool first, bool last, float inv_scale, float max_norm,
                     mlpo_step_scalars* out, hipStream_t st) {
    hipLaunchKernelGGL(grad_finish_kernel, dim3(1), dim3(kFinishBlock), 0, st, ws, n_partials, first ? 1 : 0, last ? 1 : 0,
                       inv_scale, max_norm, out);
    MLPO_HIP(hipGetLastError());
    return MLPO_OK;
}

size_t grad_norm_workspace_bytes() { return sizeof(Workspace); }

int launch_grad_norm(const mlpo_subgroup* sg, int n_sg, float inv_scale, float max_norm, void* workspace,
                     mlpo_step_scalars* out, hipStream_t stream, bool may_time, uint16_t* const* keep) {
    Workspace* ws = static_cast<Workspace*>(workspace);
    NormBatch b;
    uint64_t pieces[kMaxSg];
    b.n_sg = 0;
    b.half = table_half_format(sg, n_sg);
    bool first = true;
    int rc = MLPO_OK;
    const bool keeps = keep != nullptr;
    // Adds the array [g, g + n) to the batch as one entry; delta: elements from g to its device copy, 0 = none.
    const auto push = [&](const uint16_t* g, uint64_t n, int64_t delta) -> int {
        if (b.n_sg == kMaxSg) {  // more arrays than one argument block holds: the running totals carry over
            const int r = flush(b, pieces, first, false, inv_scale, max_norm, ws, out, stream, may_time, keeps);
            if (r != MLPO_OK) return r;
            first = false;
            b.n_sg = 0;
        }
        // the vector body starts on a 128-byte line: a wavefront's kilobyte then covers eight lines, not nine
        uint64_t head = ((128u - (reinterpret_cast<uintptr_t>(g) & 127u)) & 127u) / 2u;
        if (head > n) head = n;
        const uint64_t n_body = n - head;
        b.body[b.n_sg] = g + head;
        b.n_body[b.n_sg] = n_body;
        b.head[b.n_sg] = (uint8_t)head;
        b.keep[b.n_sg] = delta;
        pieces[b.n_sg] = n_body == 0 ? 1 : (n_body + kPiece - 1) / kPiece;
        ++b.n_sg;
        return MLPO_OK;
    };
    // Subgroups are usually consecutive slices of one flat gradient buffer (Section 2 "Sharded Model and Optimizer
    // States Into Subgroups" cuts a flat shard into equal parts): slices that follow one another in memory (and whose
    // copies, if any, do too) are summed as one array, which has one unaligned head instead of one per subgroup.
    const uint16_t* run = nullptr;
    uint64_t run_n = 0;
    int64_t run_delta = 0;
    for (int i = 0; i < n_sg; ++i) {
        if (sg[i].n == 0) continue;
        const int64_t delta = (keeps && keep[i] != nullptr) ? keep[i] - sg[i].g : 0;
        if (run != nullptr && sg[i].g == run + run_n && delta == run_delta && run_n + sg[i].n <= ((uint64_t)1 << 48)) {
            run_n += sg[i].n;
            continue;
        }
        if (run != nullptr && (rc = push(run, run_n, run_delta)) != MLPO_OK) return rc;
        run = sg[i].g;
        run_n = sg[i].n;
        run_delta = delta;
    }
    if (run != nullptr && (rc = push(run, run_n, run_delta)) != MLPO_OK) return rc;
    return flush(b, pieces, first, true, inv_scale, max_norm, ws, out, stream, may_time, keeps);
}

// ---- the entry point that allocates nothing ------------------------------------------------------------------
// Its workspace is this array in the library's own device image: every GPU the library runs on holds one copy for as
// long as the process lives, and every call on a GPU uses that GPU's copy.
static __device__ __align__(256) unsigned char scratch[sizeof(NormWorkspace)];

namespace {
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};  // the array's address on each device, asked for once per device
}  // namespace

int static_norm_workspace(void** out) {
    int dev = 0;
    MLPO_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(MLPO_EHIP, "device index %d out of range", dev);
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (g_scratch_ptr[dev] == nullptr) {
        void* ptr = nullptr;
        MLPO_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));  // the current device's copy
        if (ptr == nullptr) return fail(MLPO_EHIP, "the scratch array has no address on device %d", dev);
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return MLPO_OK;
}

}  // namespace mlpo
