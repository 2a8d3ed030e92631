// Gradient pass before the update: non-finite check, L2 norm of the unscaled gradients, clip factor (gfx950).
//
// Pass 1 streams the half-precision gradients of a table of subgroups once (2 bytes per element): 128-bit
// non-temporal loads after peeling each subgroup's unaligned head, a persistent grid of eight workgroups per compute
// unit that strides over 4 KiB tiles, several tiles per lane in flight and the loads of the next round issued before
// the current round is summed, so that the memory system always has requests queued.  Every lane widens its
// gradients, multiplies by 1/loss-scale in fp32 and accumulates the squares in fp64 - four lane operations per
// element.  The non-finite test costs nothing per element: squares are never negative and the largest finite
// half-precision value squared, times any element count, is far below the fp64 range, so a lane's sum is non-finite
// exactly when one of its unscaled gradients was.  Lanes are combined by wavefront shuffles, wavefronts through LDS,
// and each block writes one fp64 partial and one flag.  Pass 2 (one block) adds the partials in a fixed order and
// derives norm, clip coefficient and the gradient multiplier.  No atomics: the result depends only on the argument
// list, not on scheduling.
#include <hip/hip_ext.h>
#include <math.h>

#include "mlpo_internal.h"

#pragma clang fp contract(off)

namespace mlpo {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBlock = 256;
constexpr int kUnroll = 4;                // tiles a lane has in flight per round
constexpr uint32_t kTile = kBlock * 8;    // body elements per tile: one 128-bit load per lane
constexpr int kBlocksPerCu = 8;
constexpr int kMaxSg = 96;

struct NormBatch {
    const uint16_t* body[kMaxSg];  // start of the vector body, on a 128-byte line
    uint64_t n_body[kMaxSg];       // elements from body to the end of the subgroup
    uint32_t tile_begin[kMaxSg + 1];
    uint8_t head[kMaxSg];  // elements before body (0..63), handled by the first tile
    int32_t n_sg;
    int32_t half;  // MLPO_HALF_BF16 or MLPO_HALF_FP16
};

using Workspace = NormWorkspace;
constexpr int kMaxGrid = kNormMaxPartials;

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

// This lane's 128-bit word of tile `tile` (zero where the lane has none: zero bits are the value 0 in both formats
// and add nothing).  What does not fit the 128-bit pattern - the elements in front of a subgroup's body, the ragged
// end of its last tile - is added to acc on the spot.  s walks forward through the subgroup table.
template <int HALF>
__device__ __forceinline__ u32x4 fetch(const NormBatch& b, uint32_t tile, int& s, float inv_scale, double& acc) {
    const uint32_t tid = threadIdx.x;
    while (tile >= b.tile_begin[s + 1]) ++s;
    const uint32_t t_in = tile - b.tile_begin[s];
    const uint16_t* __restrict__ body = b.body[s];
    const uint64_t n_body = b.n_body[s];
    if (t_in == 0 && tid < b.head[s]) accum_half<HALF>(*(body - 1 - tid), inv_scale, acc);
    const uint64_t base = (uint64_t)t_in * kTile;
    const u32x4* __restrict__ q = reinterpret_cast<const u32x4*>(body + base) + tid;
    if (n_body >= base + kTile) return __builtin_nontemporal_load(q);
    const u32x4 zero = {0u, 0u, 0u, 0u};
    if (n_body <= base) return zero;  // a subgroup that is all head
    const uint64_t rem = n_body - base;  // < kTile
    const uint64_t e = (uint64_t)tid * 8;
    if (e + 8 <= rem) return __builtin_nontemporal_load(q);
    if (e < rem)
        for (uint64_t j = base + e; j < n_body; ++j) accum_half<HALF>(body[j], inv_scale, acc);
    return zero;
}

// The streaming part of the kernel below for one format.  Round r of a block covers the tiles
// blockIdx + (r * kUnroll + u) * gridDim, u < kUnroll: at any time the whole grid works on one window of the table.
template <int HALF>
__device__ __forceinline__ void stats_tiles(const NormBatch& b, const float inv_scale, double& a0, double& a1) {
    const uint64_t total = b.tile_begin[b.n_sg];
    const uint64_t stride = gridDim.x;
    const u32x4 zero = {0u, 0u, 0u, 0u};
    int s = 0;
    uint64_t tile = blockIdx.x;
    if (tile >= total) return;
    u32x4 cur[kUnroll], nxt[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const uint64_t t = tile + (uint64_t)u * stride;
        cur[u] = t < total ? fetch<HALF>(b, (uint32_t)t, s, inv_scale, a0) : zero;
    }
    for (;;) {
        const uint64_t next = tile + (uint64_t)kUnroll * stride;
        const bool more = next < total;
        if (more) {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const uint64_t t = next + (uint64_t)u * stride;
                nxt[u] = t < total ? fetch<HALF>(b, (uint32_t)t, s, inv_scale, a0) : zero;
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) accum_vec<HALF>(cur[u], inv_scale, a0, a1);
        if (!more) break;
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) cur[u] = nxt[u];
        tile = next;
    }
}

__global__ void __launch_bounds__(kBlock) grad_stats_kernel(const NormBatch b, const float inv_scale,
                                                            Workspace* __restrict__ ws) {
    const uint32_t tid = threadIdx.x;
    double a0 = 0.0, a1 = 0.0;
    if (b.half == 0)
        stats_tiles<0>(b, inv_scale, a0, a1);
    else
        stats_tiles<1>(b, inv_scale, a0, a1);
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

// One block: folds n_partials partials into the running sum; on the last group derives the outputs.
__global__ void __launch_bounds__(kBlock) grad_finish_kernel(Workspace* __restrict__ ws, const int n_partials,
                                                             const int first, const int last, const float inv_scale,
                                                             const float max_norm, mlpo_step_scalars* __restrict__ out) {
    const uint32_t tid = threadIdx.x;
    double acc = 0.0;
    uint32_t bad = 0;
    for (int i = tid; i < n_partials; i += kBlock) {
        acc += ws->partial[i];
        bad |= ws->flag[i];
    }
    __shared__ double s_acc[kBlock];
    __shared__ uint32_t s_bad[kBlock];
    s_acc[tid] = acc;
    s_bad[tid] = bad;
    __syncthreads();
    for (int w = kBlock / 2; w > 0; w >>= 1) {
        if ((int)tid < w) {
            s_acc[tid] += s_acc[tid + w];
            s_bad[tid] |= s_bad[tid + w];
        }
        __syncthreads();
    }
    if (tid == 0) {
        double sum = s_acc[0];
        uint32_t f = s_bad[0];
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

int flush(const NormBatch& b, bool first, bool last, float inv_scale, float max_norm, Workspace* ws,
          mlpo_step_scalars* out, hipStream_t st) {
    const uint32_t total = b.tile_begin[b.n_sg];
    uint32_t grid = 0;
    if (total > 0) {
        const int cus = num_cus();
        if (cus <= 0) return fail(MLPO_EHIP, "cannot query the device's compute units");
        uint64_t cap = (uint64_t)cus * (uint64_t)kBlocksPerCu;
        if (cap > (uint64_t)kMaxGrid) cap = kMaxGrid;
        grid = total < cap ? total : (uint32_t)cap;
        hipEvent_t t0, t1;
        if (timing_enabled() && timing_acquire(kTimedGradPass, &t0, &t1))
            hipExtLaunchKernelGGL(grad_stats_kernel, dim3(grid), dim3(kBlock), 0, st, t0, t1, 0, b, inv_scale, ws);
        else
            hipLaunchKernelGGL(grad_stats_kernel, dim3(grid), dim3(kBlock), 0, st, b, inv_scale, ws);
        MLPO_HIP(hipGetLastError());
    }
    return launch_norm_fold(ws, (int)grid, first, last, inv_scale, max_norm, out, st);
}

}  // namespace

int launch_norm_fold(NormWorkspace* ws, int n_partials, bool first, bool last, float inv_scale, float max_norm,
                     mlpo_step_scalars* out, hipStream_t st) {
    hipLaunchKernelGGL(grad_finish_kernel, dim3(1), dim3(kBlock), 0, st, ws, n_partials, first ? 1 : 0, last ? 1 : 0,
                       inv_scale, max_norm, out);
    MLPO_HIP(hipGetLastError());
    return MLPO_OK;
}

size_t grad_norm_workspace_bytes() { return sizeof(Workspace); }

int launch_grad_norm(const mlpo_subgroup* sg, int n_sg, float inv_scale, float max_norm, void* workspace,
                     mlpo_step_scalars* out, hipStream_t stream) {
    Workspace* ws = static_cast<Workspace*>(workspace);
    NormBatch b;
    b.n_sg = 0;
    b.tile_begin[0] = 0;
    b.half = table_half_format(sg, n_sg);
    bool first = true;
    for (int i = 0; i < n_sg; ++i) {
        const uint64_t n = sg[i].n;
        if (n == 0) continue;
        const uintptr_t addr = reinterpret_cast<uintptr_t>(sg[i].g);
        // the vector body starts on a 128-byte line: a wavefront's kilobyte then covers eight lines, not nine
        uint64_t head = ((128u - (addr & 127u)) & 127u) / 2u;
        if (head > n) head = n;
        const uint64_t n_body = n - head;
        uint64_t tiles = (n_body + kTile - 1) / kTile;
        if (tiles == 0) tiles = 1;  // a subgroup that is all head still needs its first tile
        if (tiles > 0x7FFFFFFFull) return fail(MLPO_EINVAL, "subgroup %d too large", i);
        if (b.n_sg == kMaxSg || (uint64_t)b.tile_begin[b.n_sg] + tiles > 0xFFFFFFFFull) {
            const int rc = flush(b, first, false, inv_scale, max_norm, ws, out, stream);
            if (rc != MLPO_OK) return rc;
            first = false;
            b.n_sg = 0;
        }
        b.body[b.n_sg] = sg[i].g + head;
        b.n_body[b.n_sg] = n_body;
        b.head[b.n_sg] = (uint8_t)head;
        b.tile_begin[b.n_sg + 1] = b.tile_begin[b.n_sg] + (uint32_t)tiles;
        ++b.n_sg;
    }
    return flush(b, first, true, inv_scale, max_norm, ws, out, stream);
}

}  // namespace mlpo
