// Fused mixed-precision AdamW over a table of subgroups (gfx950).
//
// One launch covers many subgroups: the subgroup table travels by value in the kernel arguments, the element range
// of every subgroup is cut into tiles, and a persistent grid walks the concatenated tile list with a grid stride.
// Each lane moves 128-bit words: per four elements three 16-byte loads (p, m, v), one 8-byte load (four bf16
// gradients), three 16-byte stores and one 8-byte store (four bf16 parameters) - 28 bytes per element, the whole
// traffic of the step.  The gradient is widened in registers and never stored (Section 3.2 "Delayed In-place
// Mixed-Precision Gradient Conversion"); the half-precision parameters are produced by the same lane that wrote the
// fp32 ones (Algorithm 1's downcast).  There is no reuse, so nothing is staged through LDS and the accesses carry
// the non-temporal hint.
//
// Arithmetic: every operation is an individually rounded fp32 operation (no contraction into fused multiply-add,
// IEEE division and square root, denormals kept) so that results can be compared bit for bit with a plain CPU
// evaluation of the same sequence.
#include <math.h>

#include "mlpo_internal.h"

#pragma clang fp contract(off)

namespace mlpo {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kBlock = 256;
constexpr int kMaxSg = 40;  // subgroups per launch; keeps the argument block well under the 4 KiB limit

struct Batch {
    SgView sg[kMaxSg];
    uint32_t tile_begin[kMaxSg + 1];  // prefix sums of tiles per subgroup
    int32_t n_sg;
};

template <bool NT, class T>
__device__ __forceinline__ T ld(const T* p) {
    if constexpr (NT)
        return __builtin_nontemporal_load(p);
    else
        return *p;
}
template <bool NT, class T>
__device__ __forceinline__ void st(T* p, T x) {
    if constexpr (NT)
        __builtin_nontemporal_store(x, p);
    else
        *p = x;
}

// fp32 -> bf16 bits, round to nearest even; NaN -> quiet NaN with the sign kept.
__device__ __forceinline__ uint32_t bf16_rne(float f) {
    const uint32_t w = __float_as_uint(f);
    uint32_t r = (w + 0x7FFFu + ((w >> 16) & 1u)) >> 16;
    if ((w & 0x7FFFFFFFu) > 0x7F800000u) r = ((w >> 16) & 0x8000u) | 0x7FC0u;
    return r;
}

// One element.  graw is the widened bf16 gradient, still scaled.
__device__ __forceinline__ uint32_t update_one(float& p, float& m, float& v, float graw, float gmul,
                                               const AdamwConsts& c) {
    const float g = graw * gmul;
    const float mn = (c.beta1 * m) + (c.omb1 * g);
    const float vn = (c.beta2 * v) + (c.omb2 * (g * g));
    const float d = (sqrtf(vn) / c.sqbc2) + c.eps;
    const float pn = (p * c.decay) - (c.step_size * (mn / d));
    p = pn;
    m = mn;
    v = vn;
    return bf16_rne(pn);
}

__device__ __forceinline__ u32x2 update_four(f32x4& p, f32x4& m, f32x4& v, u32x2 g, float gmul,
                                             const AdamwConsts& c) {
    const float graw[4] = {__uint_as_float(g.x << 16), __uint_as_float(g.x & 0xFFFF0000u),
                           __uint_as_float(g.y << 16), __uint_as_float(g.y & 0xFFFF0000u)};
    uint32_t h[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        float pk = p[k], mk = m[k], vk = v[k];
        h[k] = update_one(pk, mk, vk, graw[k], gmul, c);
        p[k] = pk;
        m[k] = mk;
        v[k] = vk;
    }
    u32x2 out;
    out.x = h[0] | (h[1] << 16);
    out.y = h[2] | (h[3] << 16);
    return out;
}

// 128-bit kernel: p, m, v 16-byte aligned, g, p16 8-byte aligned.
template <int UNROLL, bool NT>
__global__ void __launch_bounds__(kBlock) adamw_v4_kernel(const Batch b, const AdamwConsts c,
                                                          const mlpo_step_scalars* __restrict__ sc) {
    float gmul = 1.0f;
    if (sc != nullptr) {
        if (sc->found_inf != 0u) return;  // skipped step: nothing is read or written
        gmul = sc->gmul;
    }
    constexpr uint32_t kTile = kBlock * 4 * UNROLL;
    const uint32_t total = b.tile_begin[b.n_sg];
    const uint32_t tid = threadIdx.x;
    int s = 0;
    for (uint32_t tile = blockIdx.x; tile < total; tile += gridDim.x) {
        while (tile >= b.tile_begin[s + 1]) ++s;
        const SgView& d = b.sg[s];
        const uint64_t base = (uint64_t)(tile - b.tile_begin[s]) * kTile;
        const uint64_t n = d.n;
        f32x4* __restrict__ p4 = reinterpret_cast<f32x4*>(d.p + base);
        f32x4* __restrict__ m4 = reinterpret_cast<f32x4*>(d.m + base);
        f32x4* __restrict__ v4 = reinterpret_cast<f32x4*>(d.v + base);
        const u32x2* __restrict__ g2 = reinterpret_cast<const u32x2*>(d.g + base);
        u32x2* __restrict__ h2 = reinterpret_cast<u32x2*>(d.p16 + base);
        if (n - base >= kTile) {
            f32x4 P[UNROLL], M[UNROLL], V[UNROLL];
            u32x2 G[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t i = u * kBlock + tid;
                P[u] = ld<NT>(p4 + i);
                M[u] = ld<NT>(m4 + i);
                V[u] = ld<NT>(v4 + i);
                G[u] = ld<NT>(g2 + i);
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t i = u * kBlock + tid;
                const u32x2 H = update_four(P[u], M[u], V[u], G[u], gmul, c);
                st<NT>(p4 + i, P[u]);
                st<NT>(m4 + i, M[u]);
                st<NT>(v4 + i, V[u]);
                st<NT>(h2 + i, H);
            }
        } else {
            const uint64_t rem = n - base;  // < kTile
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t i = u * kBlock + tid;
                const uint64_t e = (uint64_t)i * 4;
                if (e + 4 <= rem) {
                    f32x4 P = ld<NT>(p4 + i), M = ld<NT>(m4 + i), V = ld<NT>(v4 + i);
                    const u32x2 H = update_four(P, M, V, ld<NT>(g2 + i), gmul, c);
                    st<NT>(p4 + i, P);
                    st<NT>(m4 + i, M);
                    st<NT>(v4 + i, V);
                    st<NT>(h2 + i, H);
                } else if (e < rem) {
                    for (uint64_t j = base + e; j < n; ++j) {
                        float pp = d.p[j], mm = d.m[j], vv = d.v[j];
                        const float graw = __uint_as_float((uint32_t)d.g[j] << 16);
                        d.p16[j] = (uint16_t)update_one(pp, mm, vv, graw, gmul, c);
                        d.p[j] = pp;
                        d.m[j] = mm;
                        d.v[j] = vv;
                    }
                }
            }
        }
    }
}

// Element-wise kernel for subgroups whose pointers do not meet the 128-bit kernel's alignment.
template <int UNROLL>
__global__ void __launch_bounds__(kBlock) adamw_v1_kernel(const Batch b, const AdamwConsts c,
                                                          const mlpo_step_scalars* __restrict__ sc) {
    float gmul = 1.0f;
    if (sc != nullptr) {
        if (sc->found_inf != 0u) return;
        gmul = sc->gmul;
    }
    constexpr uint32_t kTile = kBlock * UNROLL;
    const uint32_t total = b.tile_begin[b.n_sg];
    int s = 0;
    for (uint32_t tile = blockIdx.x; tile < total; tile += gridDim.x) {
        while (tile >= b.tile_begin[s + 1]) ++s;
        const SgView& d = b.sg[s];
        const uint64_t base = (uint64_t)(tile - b.tile_begin[s]) * kTile;
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const uint64_t j = base + (uint32_t)(u * kBlock) + threadIdx.x;
            if (j < d.n) {
                float pp = d.p[j], mm = d.m[j], vv = d.v[j];
                const float graw = __uint_as_float((uint32_t)d.g[j] << 16);
                d.p16[j] = (uint16_t)update_one(pp, mm, vv, graw, gmul, c);
                d.p[j] = pp;
                d.m[j] = mm;
                d.v[j] = vv;
            }
        }
    }
}

bool vec_aligned(const SgView& s) {
    auto a = [](const void* q) { return reinterpret_cast<uintptr_t>(q); };
    return ((a(s.p) | a(s.m) | a(s.v)) & 15u) == 0 && ((a(s.g) | a(s.p16)) & 7u) == 0;
}

struct Variant {
    int unroll;
    bool nt;
};
constexpr Variant kVariants[] = {{2, true}, {1, true}, {4, true}, {2, false}, {1, false}, {4, false}};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

template <int UNROLL, bool NT>
void launch_v4(const Batch& b, uint32_t grid, const AdamwConsts& c, const mlpo_step_scalars* sc, hipStream_t st) {
    hipLaunchKernelGGL((adamw_v4_kernel<UNROLL, NT>), dim3(grid), dim3(kBlock), 0, st, b, c, sc);
}

int launch_batch(const Batch& b, bool vec, const AdamwConsts& c, const mlpo_step_scalars* sc, hipStream_t st) {
    const uint32_t total = b.tile_begin[b.n_sg];
    if (total == 0) return MLPO_OK;
    const int cus = num_cus();
    if (cus <= 0) return fail(MLPO_EHIP, "cannot query the device's compute units");
    const int per_cu = tuning().adamw_grid_per_cu;
    uint32_t grid = total;
    if (per_cu > 0) {
        const uint64_t cap = (uint64_t)cus * (uint64_t)per_cu;
        if (cap < grid) grid = (uint32_t)cap;
    }
    if (!vec) {
        hipLaunchKernelGGL((adamw_v1_kernel<4>), dim3(grid), dim3(kBlock), 0, st, b, c, sc);
    } else {
        int vi = tuning().adamw_variant;
        if (vi < 0 || vi >= kNumVariants) vi = 0;
        switch (vi) {
            case 0: launch_v4<2, true>(b, grid, c, sc, st); break;
            case 1: launch_v4<1, true>(b, grid, c, sc, st); break;
            case 2: launch_v4<4, true>(b, grid, c, sc, st); break;
            case 3: launch_v4<2, false>(b, grid, c, sc, st); break;
            case 4: launch_v4<1, false>(b, grid, c, sc, st); break;
            default: launch_v4<4, false>(b, grid, c, sc, st); break;
        }
    }
    MLPO_HIP(hipGetLastError());
    return MLPO_OK;
}

uint32_t tile_elems(bool vec) {
    if (!vec) return kBlock * 4;
    int vi = tuning().adamw_variant;
    if (vi < 0 || vi >= kNumVariants) vi = 0;
    return (uint32_t)kBlock * 4u * (uint32_t)kVariants[vi].unroll;
}

}  // namespace

int launch_adamw(const SgView* views, int n, const AdamwConsts& c, const mlpo_step_scalars* scalars,
                 hipStream_t stream) {
    for (int pass = 0; pass < 2; ++pass) {
        const bool vec = (pass == 0);
        const uint32_t te = tile_elems(vec);
        Batch b;
        b.n_sg = 0;
        b.tile_begin[0] = 0;
        for (int i = 0; i < n; ++i) {
            const SgView& s = views[i];
            if (s.n == 0 || vec_aligned(s) != vec) continue;
            const uint64_t tiles = (s.n + te - 1) / te;
            if (tiles > 0x7FFFFFFFull) return fail(MLPO_EINVAL, "subgroup %d too large (%llu elements)", i,
                                                   (unsigned long long)s.n);
            if (b.n_sg == kMaxSg || (uint64_t)b.tile_begin[b.n_sg] + tiles > 0xFFFFFFFFull) {
                const int rc = launch_batch(b, vec, c, scalars, stream);
                if (rc != MLPO_OK) return rc;
                b.n_sg = 0;
            }
            b.sg[b.n_sg] = s;
            b.tile_begin[b.n_sg + 1] = b.tile_begin[b.n_sg] + (uint32_t)tiles;
            ++b.n_sg;
        }
        if (b.n_sg > 0) {
            const int rc = launch_batch(b, vec, c, scalars, stream);
            if (rc != MLPO_OK) return rc;
        }
    }
    return MLPO_OK;
}

}  // namespace mlpo
