// Fused mixed-precision AdamW over a table of subgroups (gfx950).
//
// One launch covers many subgroups: the subgroup table travels by value in the kernel arguments and the element range
// of every subgroup is cut into tiles.  Either every block takes one tile, or a persistent grid walks the tile list
// with a grid stride and issues the loads of its next tile before it computes and stores the current one (on this
// architecture one counter tracks loads and stores in order, so loads issued after stores would wait for them).
// Each lane moves 128-bit words: per four elements three 16-byte loads (p, m, v), one 8-byte load (four bf16
// gradients), three 16-byte stores and one 8-byte store (four bf16 parameters) - 28 bytes per element, the whole
// traffic of the step.  The gradient is widened in registers and never stored (Section 3.2 "Delayed In-place
// Mixed-Precision Gradient Conversion"); the half-precision parameters are produced by the same lane that wrote the
// fp32 ones (Algorithm 1's downcast).  There is no reuse, so nothing is staged through LDS and all accesses but the
// stores of the half-precision parameters carry the non-temporal hint.  The grid-stride kernels also exist in an out-of-place form that stores the new p, m, v a
// per-subgroup distance away from where it loaded the old ones: that is how a subgroup changes its home (another
// pinned buffer, a bounce buffer bound for a file, HBM) while it is updated.  The exchanging form goes one step further:
// before a lane stores its new p, m, v at the destination it takes what the destination held and stores that a second
// per-subgroup distance away - a staging slot in HBM changes its occupant in one pass, the old one leaving for its
// home in pinned memory while the new one arrives from its own and is updated on the way, so both directions of the
// link are busy from the first tile to the last.
//
// Arithmetic: every operation is an individually rounded fp32 operation (no contraction into fused multiply-add,
// IEEE division and square root, denormals kept) so that results can be compared bit for bit with a plain CPU
// evaluation of the same sequence.
#include <hip/hip_ext.h>
#include <math.h>

#include "mlpo_internal.h"

#pragma clang fp contract(off)

namespace mlpo {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kMaxSg = 28;  // subgroups per launch; keeps the argument block well under the 4 KiB limit

// A subgroup as the 128-bit kernel sees it: counts are in groups of four elements.  The first tile of a subgroup is
// a short "head" of head4 groups chosen on the host so that every later tile starts on an address boundary of p
// (whole cache lines per wavefront access, no line shared between two blocks).  For the tiled state layout (p, m, v
// interleaved in runs of T elements inside one buffer) a kernel tile never straddles a layout tile, so the block
// computes one offset for its whole tile.
struct VecView {
    f32x4* p;
    f32x4* m;
    f32x4* v;
    const u32x2* g;
    u32x2* h;
    uint64_t n4;
    uint32_t head4;
    uint32_t tiles_per_T;  // 0: planar.  Else kernel tiles per layout tile (tiled state, head4 == 0)
    uint32_t S4;           // tiled: distance between layout tiles of one array, in groups of four
    uint32_t lead4;        // tiled: groups of padding at the front of the first tile (nothing is read or written there)
};
struct VecBatch {
    VecView sg[kMaxSg];
    uint32_t tile_begin[kMaxSg + 1];  // prefix sums of tiles per subgroup
    int32_t n_sg;
};
// Extra argument of the out-of-place kernels: where each subgroup's new p, m, v go, in groups of four behind where
// the old ones were read (kMove), and for the exchanging kernels also where the previous content of that destination
// goes, in groups of four behind the destination (kSwap; 0 = this subgroup displaces nothing).  The in-place kernels
// take the empty form.
constexpr int kInPlace = 0, kMove = 1, kSwap = 2;
template <int MOVE>
struct StoreShift {};
template <>
struct StoreShift<kMove> {
    int64_t out4[kMaxSg];
};
template <>
struct StoreShift<kSwap> {
    int64_t out4[kMaxSg];
    int64_t evict4[kMaxSg];
};

// Element-wise view for whatever the 128-bit kernel cannot take (unaligned subgroups, tails of 1-3 elements).
constexpr int kBlock1 = 256;
constexpr int kUnroll1 = 4;
struct ScalarBatch {
    SgView sg[kMaxSg];
    uint32_t tile_begin[kMaxSg + 1];
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

// fp32 -> IEEE binary16 bits, round to nearest even (the conversion instruction under the default rounding mode;
// overflow to infinity and subnormal results included); NaN -> quiet NaN with the sign kept.
__device__ __forceinline__ uint32_t f16_rne(float f) {
    const _Float16 h = (_Float16)f;
    uint32_t r = (uint32_t)__builtin_bit_cast(uint16_t, h);
    const uint32_t w = __float_as_uint(f);
    if ((w & 0x7FFFFFFFu) > 0x7F800000u) r = ((w >> 16) & 0x8000u) | 0x7E00u;
    return r;
}

// Half-precision bits (in the low 16 bits of x) -> fp32, exact.  HALF: 0 = bf16, 1 = IEEE binary16.
template <int HALF>
__device__ __forceinline__ float widen_low(uint32_t x) {
    if constexpr (HALF == 0)
        return __uint_as_float(x << 16);
    else
        return (float)__builtin_bit_cast(_Float16, (uint16_t)x);
}
// The same for the value in the high 16 bits of x.
template <int HALF>
__device__ __forceinline__ float widen_high(uint32_t x) {
    if constexpr (HALF == 0)
        return __uint_as_float(x & 0xFFFF0000u);
    else
        return (float)__builtin_bit_cast(_Float16, (uint16_t)(x >> 16));
}

// One element.  graw is the widened half-precision gradient, still scaled.
template <int HALF>
__device__ __forceinline__ uint32_t update_one(float& p, float& m, float& v, float graw, float gmul,
                                               const AdamwConsts& c) {
    float g = graw * gmul;
    if (c.l2_mode != 0) g = g + (c.l2 * p);
    const float mn = (c.beta1 * m) + (c.omb1 * g);
    const float vn = (c.beta2 * v) + (c.omb2 * (g * g));
    const float d = (sqrtf(vn) / c.sqbc2) + c.eps;
    const float pn = (p * c.decay) - (c.step_size * (mn / d));
    p = pn;
    m = mn;
    v = vn;
    return HALF == 0 ? bf16_rne(pn) : f16_rne(pn);
}

template <int HALF>
__device__ __forceinline__ u32x2 update_four(f32x4& p, f32x4& m, f32x4& v, u32x2 g, float gmul,
                                             const AdamwConsts& c) {
    const float graw[4] = {widen_low<HALF>(g.x), widen_high<HALF>(g.x), widen_low<HALF>(g.y), widen_high<HALF>(g.y)};
    uint32_t h[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        float pk = p[k], mk = m[k], vk = v[k];
        h[k] = update_one<HALF>(pk, mk, vk, graw[k], gmul, c);
        p[k] = pk;
        m[k] = mk;
        v[k] = vk;
    }
    u32x2 out;
    out.x = h[0] | (h[1] << 16);
    out.y = h[2] | (h[3] << 16);
    return out;
}

struct Tile {
    f32x4* p;
    f32x4* m;
    f32x4* v;
    const u32x2* g;
    u32x2* h;
    int64_t out4;    // kMove, kSwap: store offset of p, m, v relative to their load addresses, in groups of four
    int64_t evict4;  // kSwap: where the destination's previous content goes, relative to the destination (0: nowhere)
    uint32_t cnt;  // groups of four in this tile: lanes work on groups lo <= i < cnt
    uint32_t lo;   // 0 except in the first tile of a subgroup with padding in front
    bool full;     // every lane of every pass has a group
};

template <int T4, int MOVE>
__device__ __forceinline__ Tile locate(const VecBatch& b, const StoreShift<MOVE>& shift, uint32_t tile, int& s) {
    while (tile >= b.tile_begin[s + 1]) ++s;
    const VecView& d = b.sg[s];
    const uint32_t t_in = tile - b.tile_begin[s];
    const uint32_t head4 = d.head4;
    uint64_t q0;
    uint64_t left;
    if (head4 != 0u && t_in == 0u) {
        q0 = 0;
        left = head4;
    } else {
        q0 = (uint64_t)(t_in - (head4 != 0u ? 1u : 0u)) * T4 + head4;
        left = d.n4 - q0;
    }
    uint64_t off = q0;  // where the state of group q0 lives, relative to each array's base
    if (d.tiles_per_T != 0u) {
        const uint32_t j = t_in / d.tiles_per_T;
        const uint32_t r = t_in - j * d.tiles_per_T;
        off = (uint64_t)j * d.S4 + (uint64_t)r * T4;
    }
    Tile t;
    t.p = d.p + off;
    t.m = d.m + off;
    t.v = d.v + off;
    t.g = d.g + q0;
    t.h = d.h + q0;
    t.out4 = 0;
    t.evict4 = 0;
    if constexpr (MOVE != kInPlace) t.out4 = shift.out4[s];
    if constexpr (MOVE == kSwap) t.evict4 = shift.evict4[s];
    t.cnt = left < (uint64_t)T4 ? (uint32_t)left : (uint32_t)T4;
    t.lo = t_in == 0u ? d.lead4 : 0u;
    t.full = t.cnt == (uint32_t)T4 && t.lo == 0u;
    return t;
}

// MOVE = kInPlace stores p, m, v where they were loaded from; kMove stores them Tile::out4 groups further on; kSwap
// does the same after it has taken what lay there and stored it Tile::evict4 groups beyond (the loads of the old
// content are issued with the tile's other loads, and its stores come first, so nothing is overwritten before it
// has been read).
// The 128-bit accesses to p, m, v and the loads of g carry the non-temporal hint; the 64-bit stores of the
// half-precision parameters do not: with the hint they cost 6 % of the kernel's speed (measured; the other three
// combinations of hints on g and p16 are slower as well), without it the lines are put together in the cache.
template <int UNROLL, int MOVE>
struct OldContent {};
template <int UNROLL>
struct OldContent<UNROLL, kSwap> {
    f32x4 P[UNROLL], M[UNROLL], V[UNROLL];
};

template <int BLOCK, int UNROLL, bool NT, int MOVE>
struct Regs {
    f32x4 P[UNROLL], M[UNROLL], V[UNROLL];
    u32x2 G[UNROLL];
    OldContent<UNROLL, MOVE> old;

    __device__ __forceinline__ void load_group(const Tile& t, int u, uint32_t i) {
        P[u] = ld<NT>(t.p + i);
        M[u] = ld<NT>(t.m + i);
        V[u] = ld<NT>(t.v + i);
        G[u] = ld<NT>(t.g + i);
        if constexpr (MOVE == kSwap) {
            if (t.evict4 != 0) {
                old.P[u] = ld<NT>(t.p + t.out4 + i);
                old.M[u] = ld<NT>(t.m + t.out4 + i);
                old.V[u] = ld<NT>(t.v + t.out4 + i);
            }
        }
    }

    __device__ __forceinline__ void load(const Tile& t, uint32_t tid) {
        if (t.full) {
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) load_group(t, u, u * BLOCK + tid);
        } else {
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t i = u * BLOCK + tid;
                if (i >= t.lo && i < t.cnt) load_group(t, u, i);
            }
        }
    }

    __device__ __forceinline__ void update_store(const Tile& t, uint32_t tid, float gmul, const AdamwConsts& c) {
        if (c.half == 0)
            update_store_as<0>(t, tid, gmul, c);
        else
            update_store_as<1>(t, tid, gmul, c);
    }

    template <int HALF>
    __device__ __forceinline__ void store_group(const Tile& t, int u, uint32_t i, float gmul, const AdamwConsts& c) {
        const auto out = [&t](f32x4* q) { return MOVE != kInPlace ? q + t.out4 : q; };
        if constexpr (MOVE == kSwap) {
            if (t.evict4 != 0) {
                st<NT>(out(t.p) + t.evict4 + i, old.P[u]);
                st<NT>(out(t.m) + t.evict4 + i, old.M[u]);
                st<NT>(out(t.v) + t.evict4 + i, old.V[u]);
            }
        }
        const u32x2 H = update_four<HALF>(P[u], M[u], V[u], G[u], gmul, c);
        st<NT>(out(t.p) + i, P[u]);
        st<NT>(out(t.m) + i, M[u]);
        st<NT>(out(t.v) + i, V[u]);
        t.h[i] = H;  // no hint: see the note at Regs
    }

    template <int HALF>
    __device__ __forceinline__ void update_store_as(const Tile& t, uint32_t tid, float gmul, const AdamwConsts& c) {
        if (t.full) {
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) store_group<HALF>(t, u, u * BLOCK + tid, gmul, c);
        } else {
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t i = u * BLOCK + tid;
                if (i >= t.lo && i < t.cnt) store_group<HALF>(t, u, i, gmul, c);
            }
        }
    }
};

// 128-bit kernel: p, m, v 16-byte aligned, g, p16 8-byte aligned, element counts multiples of four.
// PERSIST = false: one tile per block.  PERSIST = true: grid-stride over tiles, next tile's loads in flight while the
// current tile is computed and stored.
template <int BLOCK, int UNROLL, bool NT, bool PERSIST, int MOVE>
__global__ void __launch_bounds__(BLOCK) adamw_v4_kernel(const VecBatch b, const AdamwConsts c,
                                                         const mlpo_step_scalars* __restrict__ sc,
                                                         const StoreShift<MOVE> shift) {
    float gmul = 1.0f;
    if (sc != nullptr) {
        if (sc->found_inf != 0u) return;  // skipped step: nothing is read or written
        gmul = sc->gmul;
    }
    constexpr int T4 = BLOCK * UNROLL;
    const uint32_t total = b.tile_begin[b.n_sg];
    const uint32_t tid = threadIdx.x;
    uint32_t tile = blockIdx.x;
    if (tile >= total) return;
    // One tile per workgroup: the tiles are taken from the end.  The gradient pass that precedes the update has just
    // read the gradients front to back, so what the last-level caches still hold of them is their end (measured on
    // 125 M elements: 503.9 against 505.4 us per launch).
    if constexpr (!PERSIST) tile = total - 1u - tile;
    int s = 0;
    if constexpr (!PERSIST) {
        // blocks are far apart in the table: find the subgroup by bisection instead of walking
        int lo = 0, hi = b.n_sg;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (tile >= b.tile_begin[mid]) lo = mid; else hi = mid;
        }
        s = lo;
        const Tile t = locate<T4, MOVE>(b, shift, tile, s);
        Regs<BLOCK, UNROLL, NT, MOVE> r;
        r.load(t, tid);
        r.update_store(t, tid, gmul, c);
    } else {
        Tile cur = locate<T4, MOVE>(b, shift, tile, s);
        Regs<BLOCK, UNROLL, NT, MOVE> rc;
        rc.load(cur, tid);
        for (;;) {
            const uint32_t next = tile + gridDim.x;
            const bool more = next < total && next > tile;
            Tile nxt = cur;
            Regs<BLOCK, UNROLL, NT, MOVE> rn;
            if (more) {
                nxt = locate<T4, MOVE>(b, shift, next, s);
                rn.load(nxt, tid);
            }
            rc.update_store(cur, tid, gmul, c);
            if (!more) break;
            cur = nxt;
            rc = rn;
            tile = next;
        }
    }
}

// Element-wise kernel, one tile per block.
__global__ void __launch_bounds__(kBlock1) adamw_v1_kernel(const ScalarBatch b, const AdamwConsts c,
                                                           const mlpo_step_scalars* __restrict__ sc) {
    float gmul = 1.0f;
    if (sc != nullptr) {
        if (sc->found_inf != 0u) return;
        gmul = sc->gmul;
    }
    constexpr uint32_t kTile = kBlock1 * kUnroll1;
    const uint32_t tile = blockIdx.x;
    if (tile >= b.tile_begin[b.n_sg]) return;
    int s = 0;
    while (tile >= b.tile_begin[s + 1]) ++s;
    const SgView& d = b.sg[s];
    const uint64_t base = (uint64_t)(tile - b.tile_begin[s]) * kTile;
#pragma unroll
    for (int u = 0; u < kUnroll1; ++u) {
        const uint64_t j = base + (uint32_t)(u * kBlock1) + threadIdx.x;
        if (j >= d.lead && j < d.n) {
            float pp = d.p[j], mm = d.m[j], vv = d.v[j];
            if (d.evict_delta != 0) {  // the destination's previous content moves on first
                const int64_t from = (int64_t)j + d.out_delta, to = from + d.evict_delta;
                const float po = d.p[from], mo = d.m[from], vo = d.v[from];
                d.p[to] = po;
                d.m[to] = mo;
                d.v[to] = vo;
            }
            if (c.half == 0)
                d.p16[j] = (uint16_t)update_one<0>(pp, mm, vv, widen_low<0>(d.g[j]), gmul, c);
            else
                d.p16[j] = (uint16_t)update_one<1>(pp, mm, vv, widen_low<1>(d.g[j]), gmul, c);
            d.p[j + d.out_delta] = pp;
            d.m[j + d.out_delta] = mm;
            d.v[j + d.out_delta] = vv;
        }
    }
}

bool vec_aligned(const SgView& s) {
    auto a = [](const void* q) { return reinterpret_cast<uintptr_t>(q); };
    return ((a(s.p) | a(s.m) | a(s.v)) & 15u) == 0 && ((a(s.g) | a(s.p16)) & 7u) == 0 && s.out_delta % 4 == 0 &&
           s.evict_delta % 4 == 0 && s.lead % 4 == 0;
}

// Two forms of the 128-bit kernel are built, both with 256 lanes and one group of four elements per lane (a kernel
// tile of 1024 elements, which divides every layout tile): one tile per workgroup - the fastest form in both layouts
// when the state is in HBM (planar, 125 M elements: 562 us against 570-573 us for larger tiles) - and the grid-stride
// form with next-tile prefetch, for a bounded number of persistent workgroups (state in pinned host memory) and, in
// its out-of-place instantiation, for subgroups that change their home.
constexpr int kLanes = 256;
constexpr uint64_t kTile4 = kLanes;  // groups of four per kernel tile

template <bool PERSIST, int MOVE = kInPlace>
void launch_v4(const VecBatch& b, uint32_t grid, const AdamwConsts& c, const mlpo_step_scalars* sc, hipStream_t st,
               const StoreShift<MOVE>& shift = StoreShift<MOVE>{}) {
    hipEvent_t t0, t1;
    if (timing_enabled() && timing_acquire(kTimedUpdate, &t0, &t1))
        hipExtLaunchKernelGGL((adamw_v4_kernel<kLanes, 1, true, PERSIST, MOVE>), dim3(grid), dim3(kLanes), 0, st, t0, t1,
                              0, b, c, sc, shift);
    else
        hipLaunchKernelGGL((adamw_v4_kernel<kLanes, 1, true, PERSIST, MOVE>), dim3(grid), dim3(kLanes), 0, st, b, c, sc,
                           shift);
}

// persist_blocks = 0: one tile per workgroup.  > 0: that many persistent workgroups at most.  shift != nullptr: an
// out-of-place form (always grid-stride; persist_blocks = 0 then means eight workgroups per compute unit), the
// exchanging one if any subgroup of the batch displaces what its destination held.
int launch_vec_batch(const VecBatch& b, const AdamwConsts& c, const mlpo_step_scalars* sc, hipStream_t st,
                     int persist_blocks, const StoreShift<kSwap>* shift) {
    const uint32_t total = b.tile_begin[b.n_sg];
    if (total == 0) return MLPO_OK;
    uint32_t grid = total;
    if (persist_blocks > 0) {
        if ((uint32_t)persist_blocks < grid) grid = (uint32_t)persist_blocks;
    } else if (shift != nullptr) {
        const int cus = num_cus();
        if (cus <= 0) return fail(MLPO_EHIP, "cannot query the device's compute units");
        const uint64_t cap = (uint64_t)cus * 8u;
        if (cap < grid) grid = (uint32_t)cap;
    }
    bool swaps = false;
    if (shift != nullptr)
        for (int i = 0; i < b.n_sg; ++i) swaps = swaps || shift->evict4[i] != 0;
    if (swaps) {
        launch_v4<true, kSwap>(b, grid, c, sc, st, *shift);
    } else if (shift != nullptr) {
        StoreShift<kMove> mv;
        for (int i = 0; i < kMaxSg; ++i) mv.out4[i] = shift->out4[i];
        launch_v4<true, kMove>(b, grid, c, sc, st, mv);
    } else if (persist_blocks > 0) {
        launch_v4<true>(b, grid, c, sc, st);
    } else {
        launch_v4<false>(b, grid, c, sc, st);  // grid == total: every tile has its workgroup
    }
    MLPO_HIP(hipGetLastError());
    return MLPO_OK;
}

int launch_scalar_batch(const ScalarBatch& b, const AdamwConsts& c, const mlpo_step_scalars* sc, hipStream_t st) {
    const uint32_t total = b.tile_begin[b.n_sg];
    if (total == 0) return MLPO_OK;
    hipLaunchKernelGGL(adamw_v1_kernel, dim3(total), dim3(kBlock1), 0, st, b, c, sc);
    MLPO_HIP(hipGetLastError());
    return MLPO_OK;
}

constexpr uint64_t kMaxTiles = 0x7FFFFFFFull;  // grid.x limit

}  // namespace

int launch_adamw(const SgView* views, int n, const AdamwConsts& c, const mlpo_step_scalars* scalars,
                 hipStream_t stream, int persist_blocks) {
    bool moves = false;  // does any subgroup's new state go somewhere else than the old one came from?
    for (int i = 0; i < n; ++i) {
        moves = moves || views[i].out_delta != 0;
        if (views[i].evict_delta != 0 && views[i].out_delta == 0)
            return fail(MLPO_EINVAL, "view %d displaces its destination's content but is updated in place", i);
    }
    const uint64_t t4 = kTile4;
    // Planar subgroups get a head tile that ends on a 256-byte boundary of p: whole cache lines per wavefront access and
    // no line shared between two workgroups (a subgroup that starts mid-line runs 13 % slower without it).
    constexpr uint64_t align = 256;
    constexpr uint64_t kTile1 = (uint64_t)kBlock1 * kUnroll1;

    VecBatch vb;
    vb.n_sg = 0;
    vb.tile_begin[0] = 0;
    StoreShift<kSwap> shift{};
    const StoreShift<kSwap>* shift_arg = moves ? &shift : nullptr;
    ScalarBatch sb;
    sb.n_sg = 0;
    sb.tile_begin[0] = 0;

    auto push_scalar = [&](const SgView& s) -> int {
        const uint64_t tiles = (s.n + kTile1 - 1) / kTile1;
        if (tiles > kMaxTiles) return fail(MLPO_EINVAL, "subgroup too large (%llu elements)", (unsigned long long)s.n);
        if (sb.n_sg == kMaxSg || (uint64_t)sb.tile_begin[sb.n_sg] + tiles > kMaxTiles) {
            const int rc = launch_scalar_batch(sb, c, scalars, stream);
            if (rc != MLPO_OK) return rc;
            sb.n_sg = 0;
        }
        sb.sg[sb.n_sg] = s;
        sb.tile_begin[sb.n_sg + 1] = sb.tile_begin[sb.n_sg] + (uint32_t)tiles;
        ++sb.n_sg;
        return MLPO_OK;
    };

    for (int i = 0; i < n; ++i) {
        const SgView& s = views[i];
        if (s.n == 0) continue;
        if (!vec_aligned(s)) {
            const int rc = push_scalar(s);
            if (rc != MLPO_OK) return rc;
            continue;
        }
        const uint64_t n4 = s.n / 4;
        const uint64_t tail = s.n - n4 * 4;
        if (tail != 0) {  // the last 1-3 elements go to the element-wise kernel
            const uint64_t o = n4 * 4;
            uint64_t po = o;  // position of element o in the state arrays
            if (s.tile_elems != 0) po = (o / (uint64_t)s.tile_elems) * 3u * (uint64_t)s.tile_elems + o % (uint64_t)s.tile_elems;
            const int rc = push_scalar(SgView{s.p + po, s.m + po, s.v + po, s.g + o, s.p16 + o, tail, 0, s.out_delta,
                                              s.evict_delta});
            if (rc != MLPO_OK) return rc;
        }
        if (n4 == 0) continue;
        uint64_t head4 = ((align - (reinterpret_cast<uintptr_t>(s.p) & (align - 1))) & (align - 1)) / 16;
        if (head4 >= n4 || s.tile_elems != 0) head4 = 0;  // tiled buffers are 256-byte aligned by contract
        const uint64_t tiles = (head4 != 0 ? 1 : 0) + (n4 - head4 + t4 - 1) / t4;
        if (tiles > kMaxTiles) return fail(MLPO_EINVAL, "subgroup %d too large (%llu elements)", i,
                                           (unsigned long long)s.n);
        if (vb.n_sg == kMaxSg || (uint64_t)vb.tile_begin[vb.n_sg] + tiles > kMaxTiles) {
            const int rc = launch_vec_batch(vb, c, scalars, stream, persist_blocks, shift_arg);
            if (rc != MLPO_OK) return rc;
            vb.n_sg = 0;
        }
        VecView& d = vb.sg[vb.n_sg];
        d.p = reinterpret_cast<f32x4*>(s.p);
        d.m = reinterpret_cast<f32x4*>(s.m);
        d.v = reinterpret_cast<f32x4*>(s.v);
        d.g = reinterpret_cast<const u32x2*>(s.g);
        d.h = reinterpret_cast<u32x2*>(s.p16);
        d.n4 = n4;
        d.head4 = (uint32_t)head4;
        d.tiles_per_T = s.tile_elems != 0 ? (uint32_t)((uint64_t)s.tile_elems / 4 / t4) : 0u;
        d.S4 = s.tile_elems != 0 ? (uint32_t)(3u * (uint64_t)s.tile_elems / 4) : 0u;
        d.lead4 = s.lead / 4;
        shift.out4[vb.n_sg] = s.out_delta / 4;
        shift.evict4[vb.n_sg] = s.evict_delta / 4;
        vb.tile_begin[vb.n_sg + 1] = vb.tile_begin[vb.n_sg] + (uint32_t)tiles;
        ++vb.n_sg;
    }
    int rc = launch_vec_batch(vb, c, scalars, stream, persist_blocks, shift_arg);
    if (rc != MLPO_OK) return rc;
    return launch_scalar_batch(sb, c, scalars, stream);
}

}  // namespace mlpo
