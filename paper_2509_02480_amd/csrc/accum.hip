// Gradient accumulation over micro-batches into the half-precision accumulation buffer (Section 3.2 "Delayed
// In-place Mixed-Precision Gradient Conversion": the buffer holds bf16 gradients until the update upcasts them).
//
// acc[i] = bf16_rne(f32(acc[i]) + f32(g[i])), or acc[i] = g[i] for the first micro-batch of a step.  Pure streaming:
// 6 bytes per element (4 read, 2 written; 4 for the first micro-batch), so the kernel is shaped like the update:
// 128-bit non-temporal accesses, one 2048-element tile per workgroup, or a bounded number of persistent workgroups
// when the buffer sits in pinned host memory and the traffic crosses the link.
//
// The last micro-batch of a step can also produce the statistics of the finished buffer (sum of squares of the
// unscaled values, non-finite flag) from the values it has in registers, which saves the gradient pass its own read
// of the buffer - over the link when the buffer is on the host.
#include <hip/hip_ext.h>
#include <math.h>

#include "mlpo_internal.h"

#pragma clang fp contract(off)

namespace mlpo {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBlock = 256;
// 128-bit vectors per lane and tile.  One tile per workgroup is fastest with a single vector per lane (measured:
// 6.47 TB/s against 6.09 with four on 1.3 G elements); a persistent grid wants more loads in flight per iteration.
constexpr int kUnrollOneTile = 1;
constexpr int kUnrollPersistent = 4;

// One half-precision sum, operands and result in the low 16 bits: widen both (exact), one fp32 addition, round to
// nearest even; a NaN sum becomes the format's canonical quiet NaN.  HALF: 0 = bf16, 1 = IEEE binary16.
template <int HALF>
__device__ __forceinline__ uint32_t add_one(uint32_t a, uint32_t g) {
    if constexpr (HALF == 0) {
        const float s = __uint_as_float(a << 16) + __uint_as_float(g << 16);
        const uint32_t r = __float_as_uint(s);
        const uint32_t rounded = (r + 0x7FFFu + ((r >> 16) & 1u)) >> 16;
        return (s != s) ? 0x7FC0u : rounded;
    } else {
        const float s = (float)__builtin_bit_cast(_Float16, (uint16_t)a) + (float)__builtin_bit_cast(_Float16, (uint16_t)g);
        const uint32_t rounded = (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)s);
        return (s != s) ? 0x7E00u : rounded;
    }
}

// Two sums packed in a 32-bit word.
template <int HALF>
__device__ __forceinline__ uint32_t add_word(uint32_t a, uint32_t g) {
    return add_one<HALF>(a & 0xFFFFu, g & 0xFFFFu) | (add_one<HALF>(a >> 16, g >> 16) << 16);
}

template <int HALF>
__device__ __forceinline__ u32x4 add_vec(u32x4 a, u32x4 g) {
    u32x4 r;
    r.x = add_word<HALF>(a.x, g.x);
    r.y = add_word<HALF>(a.y, g.y);
    r.z = add_word<HALF>(a.z, g.z);
    r.w = add_word<HALF>(a.w, g.w);
    return r;
}

// Statistics of one stored word (two new bf16 values): squares of the unscaled values in fp64, non-finite test on
// the exponent field - the arithmetic of the gradient pass, applied to values that are in registers anyway.
template <int HALF>
__device__ __forceinline__ void stats_one(uint32_t h, float inv_scale, double& sum, uint32_t& bad) {
    constexpr uint32_t kExp = HALF == 0 ? 0x7F80u : 0x7C00u;
    bad |= (uint32_t)((h & kExp) == kExp);
    const float u =
        (HALF == 0 ? __uint_as_float(h << 16) : (float)__builtin_bit_cast(_Float16, (uint16_t)h)) * inv_scale;
    sum = fma((double)u, (double)u, sum);
}

template <int HALF>
__device__ __forceinline__ void stats_word(uint32_t w, float inv_scale, double& sum, uint32_t& bad) {
    stats_one<HALF>(w & 0xFFFFu, inv_scale, sum, bad);
    stats_one<HALF>(w >> 16, inv_scale, sum, bad);
}

template <int HALF>
__device__ __forceinline__ void stats_vec(u32x4 r, float inv_scale, double& sum, uint32_t& bad) {
    stats_word<HALF>(r.x, inv_scale, sum, bad);
    stats_word<HALF>(r.y, inv_scale, sum, bad);
    stats_word<HALF>(r.z, inv_scale, sum, bad);
    stats_word<HALF>(r.w, inv_scale, sum, bad);
}

// Lanes -> wavefront (shuffle), wavefronts -> workgroup (LDS), in a fixed order; one partial per workgroup.
__device__ __forceinline__ void block_partial(double sum, uint32_t bad, NormWorkspace* __restrict__ ws, uint32_t slot) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        sum += __shfl_down(sum, off, 64);
        bad |= (uint32_t)__shfl_down((int)bad, off, 64);
    }
    __shared__ double s_sum[kBlock / 64];
    __shared__ uint32_t s_bad[kBlock / 64];
    const uint32_t tid = threadIdx.x;
    if ((tid & 63u) == 0) {
        s_sum[tid >> 6] = sum;
        s_bad[tid >> 6] = bad;
    }
    __syncthreads();
    if (tid == 0) {
        double t = s_sum[0];
        uint32_t f = s_bad[0];
#pragma unroll
        for (int w = 1; w < kBlock / 64; ++w) {
            t += s_sum[w];
            f |= s_bad[w];
        }
        ws->partial[slot] = t;
        ws->flag[slot] = f;
    }
}

// acc and g point at the 16-byte aligned vector body; n8 = number of 8-element vectors in it.  With STATS every
// workgroup also leaves the statistics of the values it stored in ws->partial / ws->flag [slot0 + blockIdx.x].
template <bool FIRST, bool STATS, int kUnroll, int HALF>
__global__ void __launch_bounds__(kBlock) accumulate_v8_kernel(u32x4* __restrict__ acc, const u32x4* __restrict__ g,
                                                               const uint64_t n8, const float inv_scale,
                                                               NormWorkspace* __restrict__ ws, const uint32_t slot0) {
    const uint64_t per_tile = (uint64_t)kBlock * kUnroll;
    const uint64_t tiles = (n8 + per_tile - 1) / per_tile;
    double sum = 0.0;
    uint32_t bad = 0;
    for (uint64_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
        const uint64_t base = tile * per_tile + threadIdx.x;
        if ((tile + 1) * per_tile <= n8) {
            u32x4 a[kUnroll], b[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                b[u] = __builtin_nontemporal_load(g + base + (uint64_t)u * kBlock);
                if (!FIRST) a[u] = __builtin_nontemporal_load(acc + base + (uint64_t)u * kBlock);
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const u32x4 r = FIRST ? b[u] : add_vec<HALF>(a[u], b[u]);
                __builtin_nontemporal_store(r, acc + base + (uint64_t)u * kBlock);
                if (STATS) stats_vec<HALF>(r, inv_scale, sum, bad);
            }
        } else {
            for (int u = 0; u < kUnroll; ++u) {
                const uint64_t i = base + (uint64_t)u * kBlock;
                if (i < n8) {
                    u32x4 r = __builtin_nontemporal_load(g + i);
                    if (!FIRST) r = add_vec<HALF>(__builtin_nontemporal_load(acc + i), r);
                    __builtin_nontemporal_store(r, acc + i);
                    if (STATS) stats_vec<HALF>(r, inv_scale, sum, bad);
                }
            }
        }
    }
    if (STATS) block_partial(sum, bad, ws, slot0 + blockIdx.x);
}

// Element-wise form for heads, tails and buffers whose addresses differ modulo 16.
template <bool FIRST, bool STATS, int HALF>
__global__ void __launch_bounds__(kBlock) accumulate_v1_kernel(uint16_t* __restrict__ acc,
                                                               const uint16_t* __restrict__ g, const uint64_t n,
                                                               const float inv_scale, NormWorkspace* __restrict__ ws,
                                                               const uint32_t slot0) {
    const uint64_t stride = (uint64_t)gridDim.x * kBlock;
    double sum = 0.0;
    uint32_t bad = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride) {
        const uint32_t r = FIRST ? (uint32_t)g[i] : add_one<HALF>(acc[i], g[i]);
        acc[i] = (uint16_t)r;
        if (STATS) stats_one<HALF>(r, inv_scale, sum, bad);
    }
    if (STATS) block_partial(sum, bad, ws, slot0 + blockIdx.x);
}

template <bool FIRST, bool STATS, int HALF>
int launch(uint16_t* acc, const uint16_t* g, uint64_t n, int blocks, hipStream_t st, NormWorkspace* ws,
           float inv_scale, int* n_partials) {
    const int cus = num_cus();
    if (cus <= 0) return fail(MLPO_EHIP, "cannot query the device's compute units");
    // every workgroup of a statistics launch owns one partial, so those grids are persistent and leave room for
    // the two single-workgroup launches of head and tail
    uint32_t persistent = blocks > 0 ? (uint32_t)blocks : (uint32_t)cus * 8u;
    if (persistent > (uint32_t)kNormMaxPartials - 2u) persistent = (uint32_t)kNormMaxPartials - 2u;
    uint32_t slot = 0;
    const uintptr_t a_addr = reinterpret_cast<uintptr_t>(acc);
    const uintptr_t g_addr = reinterpret_cast<uintptr_t>(g);
    if (((a_addr ^ g_addr) & 15u) != 0) {
        // no common 16-byte phase: everything goes element by element
        const uint64_t want = (n + kBlock - 1) / kBlock;
        const uint32_t grid = (uint32_t)(want < persistent ? want : persistent);
        hipLaunchKernelGGL((accumulate_v1_kernel<FIRST, STATS, HALF>), dim3(grid), dim3(kBlock), 0, st, acc, g, n, inv_scale,
                           ws, slot);
        MLPO_HIP(hipGetLastError());
        if (STATS) *n_partials = (int)grid;
        return MLPO_OK;
    }
    // The vector body starts on a 128-byte line of acc, the array that is written: a workgroup's tile then owns whole
    // lines (a line written in two halves by two workgroups costs more than the bytes say).  g + head is 16-byte
    // aligned because the two addresses agree modulo 16.
    uint64_t head = ((128u - (a_addr & 127u)) & 127u) / 2u;
    if (head > n) head = n;
    const uint64_t n8 = (n - head) / 8u;
    const uint64_t tail = n - head - n8 * 8u;
    if (n8 > 0) {
        const bool persistent_grid = blocks > 0 || STATS;
        const uint64_t per_tile = (uint64_t)kBlock * (persistent_grid ? kUnrollPersistent : kUnrollOneTile);
        const uint64_t tiles = (n8 + per_tile - 1) / per_tile;
        if (!persistent_grid && tiles > 0x7FFFFFFFull) return fail(MLPO_EINVAL, "n too large for one launch");
        const uint32_t grid = (uint32_t)(persistent_grid && tiles > persistent ? persistent : tiles);
        u32x4* av = reinterpret_cast<u32x4*>(acc + head);
        const u32x4* gv = reinterpret_cast<const u32x4*>(g + head);
        auto kernel = persistent_grid ? accumulate_v8_kernel<FIRST, STATS, kUnrollPersistent, HALF>
                                      : accumulate_v8_kernel<FIRST, STATS, kUnrollOneTile, HALF>;
        hipEvent_t t0, t1;
        if (timing_enabled() && timing_acquire(kTimedAccumulate, &t0, &t1))
            hipExtLaunchKernelGGL(kernel, dim3(grid), dim3(kBlock), 0, st, t0, t1, 0, av, gv, n8, inv_scale, ws, slot);
        else
            hipLaunchKernelGGL(kernel, dim3(grid), dim3(kBlock), 0, st, av, gv, n8, inv_scale, ws, slot);
        MLPO_HIP(hipGetLastError());
        slot += grid;
    }
    if (head > 0) {
        hipLaunchKernelGGL((accumulate_v1_kernel<FIRST, STATS, HALF>), dim3(1), dim3(kBlock), 0, st, acc, g, head, inv_scale,
                           ws, slot);
        MLPO_HIP(hipGetLastError());
        slot += 1;
    }
    if (tail > 0) {
        const uint64_t off = head + n8 * 8u;
        hipLaunchKernelGGL((accumulate_v1_kernel<FIRST, STATS, HALF>), dim3(1), dim3(kBlock), 0, st, acc + off, g + off, tail,
                           inv_scale, ws, slot);
        MLPO_HIP(hipGetLastError());
        slot += 1;
    }
    if (STATS) *n_partials = (int)slot;
    return MLPO_OK;
}

}  // namespace

template <int HALF>
static int launch_format(uint16_t* acc, const uint16_t* g, uint64_t n, bool first, int blocks, hipStream_t st,
                         NormWorkspace* stats, float inv_scale, int* n_partials) {
    if (stats != nullptr)
        return first ? launch<true, true, HALF>(acc, g, n, blocks, st, stats, inv_scale, n_partials)
                     : launch<false, true, HALF>(acc, g, n, blocks, st, stats, inv_scale, n_partials);
    return first ? launch<true, false, HALF>(acc, g, n, blocks, st, nullptr, 1.0f, nullptr)
                 : launch<false, false, HALF>(acc, g, n, blocks, st, nullptr, 1.0f, nullptr);
}

int launch_grad_accumulate(uint16_t* acc, const uint16_t* g, uint64_t n, bool first, int blocks, int32_t half,
                           hipStream_t st, NormWorkspace* stats, float inv_scale, int* n_partials) {
    return half == MLPO_HALF_FP16 ? launch_format<1>(acc, g, n, first, blocks, st, stats, inv_scale, n_partials)
                                  : launch_format<0>(acc, g, n, first, blocks, st, stats, inv_scale, n_partials);
}

}  // namespace mlpo
