// Gradient accumulation over micro-batches into the half-precision accumulation buffer (Section 3.2 "Delayed
// In-place Mixed-Precision Gradient Conversion": the buffer holds bf16 gradients until the update upcasts them).
//
// acc[i] = bf16_rne(f32(acc[i]) + f32(g[i])), or acc[i] = g[i] for the first micro-batch of a step.  Pure streaming:
// 6 bytes per element (4 read, 2 written; 4 for the first micro-batch), so the kernel is shaped like the update:
// 128-bit non-temporal accesses, one 8192-element tile per workgroup, or a bounded number of persistent workgroups
// when the buffer sits in pinned host memory and the traffic crosses the link.
#include <hip/hip_ext.h>

#include "mlpo_internal.h"

#pragma clang fp contract(off)

namespace mlpo {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBlock = 256;
constexpr int kUnroll = 4;

// One bf16 sum, operands and result in the low 16 bits.
__device__ __forceinline__ uint32_t add_one(uint32_t a, uint32_t g) {
    const float s = __uint_as_float(a << 16) + __uint_as_float(g << 16);
    const uint32_t r = __float_as_uint(s);
    const uint32_t rounded = (r + 0x7FFFu + ((r >> 16) & 1u)) >> 16;
    return (s != s) ? 0x7FC0u : rounded;
}

// Two bf16 sums packed in a 32-bit word.
__device__ __forceinline__ uint32_t add_word(uint32_t a, uint32_t g) {
    return add_one(a & 0xFFFFu, g & 0xFFFFu) | (add_one(a >> 16, g >> 16) << 16);
}

__device__ __forceinline__ u32x4 add_vec(u32x4 a, u32x4 g) {
    u32x4 r;
    r.x = add_word(a.x, g.x);
    r.y = add_word(a.y, g.y);
    r.z = add_word(a.z, g.z);
    r.w = add_word(a.w, g.w);
    return r;
}

// acc and g point at the 16-byte aligned vector body; n8 = number of 8-element vectors in it.
template <bool FIRST>
__global__ void __launch_bounds__(kBlock) accumulate_v8_kernel(u32x4* __restrict__ acc, const u32x4* __restrict__ g,
                                                               const uint64_t n8) {
    const uint64_t per_tile = (uint64_t)kBlock * kUnroll;
    const uint64_t tiles = (n8 + per_tile - 1) / per_tile;
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
            for (int u = 0; u < kUnroll; ++u)
                __builtin_nontemporal_store(FIRST ? b[u] : add_vec(a[u], b[u]), acc + base + (uint64_t)u * kBlock);
        } else {
            for (int u = 0; u < kUnroll; ++u) {
                const uint64_t i = base + (uint64_t)u * kBlock;
                if (i < n8) {
                    const u32x4 b = __builtin_nontemporal_load(g + i);
                    if (FIRST) {
                        __builtin_nontemporal_store(b, acc + i);
                    } else {
                        const u32x4 a = __builtin_nontemporal_load(acc + i);
                        __builtin_nontemporal_store(add_vec(a, b), acc + i);
                    }
                }
            }
        }
    }
}

// Element-wise form for heads, tails and buffers whose addresses differ modulo 16.
template <bool FIRST>
__global__ void __launch_bounds__(kBlock) accumulate_v1_kernel(uint16_t* __restrict__ acc,
                                                               const uint16_t* __restrict__ g, const uint64_t n) {
    const uint64_t stride = (uint64_t)gridDim.x * kBlock;
    for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride)
        acc[i] = FIRST ? g[i] : (uint16_t)add_one(acc[i], g[i]);
}

template <bool FIRST>
int launch(uint16_t* acc, const uint16_t* g, uint64_t n, int blocks, hipStream_t st) {
    const int cus = num_cus();
    if (cus <= 0) return fail(MLPO_EHIP, "cannot query the device's compute units");
    const uint32_t scalar_cap = blocks > 0 ? (uint32_t)blocks : (uint32_t)cus * 8u;
    const uintptr_t a_addr = reinterpret_cast<uintptr_t>(acc);
    const uintptr_t g_addr = reinterpret_cast<uintptr_t>(g);
    if (((a_addr ^ g_addr) & 15u) != 0) {
        // no common 16-byte phase: everything goes element by element
        const uint64_t want = (n + kBlock - 1) / kBlock;
        const uint32_t grid = (uint32_t)(want < scalar_cap ? want : scalar_cap);
        hipLaunchKernelGGL(accumulate_v1_kernel<FIRST>, dim3(grid), dim3(kBlock), 0, st, acc, g, n);
        MLPO_HIP(hipGetLastError());
        return MLPO_OK;
    }
    uint64_t head = ((16u - (a_addr & 15u)) & 15u) / 2u;
    if (head > n) head = n;
    const uint64_t n8 = (n - head) / 8u;
    const uint64_t tail = n - head - n8 * 8u;
    if (n8 > 0) {
        const uint64_t per_tile = (uint64_t)kBlock * kUnroll;
        const uint64_t tiles = (n8 + per_tile - 1) / per_tile;
        const uint64_t cap = blocks > 0 ? (uint64_t)blocks : 0x7FFFFFFFull;
        const uint32_t grid = (uint32_t)(tiles < cap ? tiles : cap);
        u32x4* av = reinterpret_cast<u32x4*>(acc + head);
        const u32x4* gv = reinterpret_cast<const u32x4*>(g + head);
        hipEvent_t t0, t1;
        if (timing_enabled() && timing_acquire(kTimedAccumulate, &t0, &t1))
            hipExtLaunchKernelGGL(accumulate_v8_kernel<FIRST>, dim3(grid), dim3(kBlock), 0, st, t0, t1, 0, av, gv, n8);
        else
            hipLaunchKernelGGL(accumulate_v8_kernel<FIRST>, dim3(grid), dim3(kBlock), 0, st, av, gv, n8);
        MLPO_HIP(hipGetLastError());
    }
    if (head > 0) {
        hipLaunchKernelGGL(accumulate_v1_kernel<FIRST>, dim3(1), dim3(kBlock), 0, st, acc, g, head);
        MLPO_HIP(hipGetLastError());
    }
    if (tail > 0) {
        const uint64_t off = head + n8 * 8u;
        hipLaunchKernelGGL(accumulate_v1_kernel<FIRST>, dim3(1), dim3(kBlock), 0, st, acc + off, g + off, tail);
        MLPO_HIP(hipGetLastError());
    }
    return MLPO_OK;
}

}  // namespace

int launch_grad_accumulate(uint16_t* acc, const uint16_t* g, uint64_t n, bool first, int blocks, hipStream_t st) {
    return first ? launch<true>(acc, g, n, blocks, st) : launch<false>(acc, g, n, blocks, st);
}

}  // namespace mlpo
