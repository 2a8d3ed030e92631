// Conversion between the planar fp32 state (three arrays) and the tiled state buffer (gfx950).
// Pure data movement for state that arrives or leaves planar (a checkpoint, another runtime): each lane moves four
// consecutive elements of one array, one block covers 1024 elements; not on the step's hot path.
#include "mlpo_internal.h"

namespace mlpo {
namespace {

constexpr int kBlock = 256;

// PACK: planar -> tiled (the padding in front and the unused tail of the last layout tile are zero-filled).  !PACK: tiled -> planar.
// Work is indexed over the tiled buffer's element slots: slot q of array a in layout tile j.
template <bool PACK>
__global__ void __launch_bounds__(kBlock) repack_kernel(float* __restrict__ p, float* __restrict__ m,
                                                        float* __restrict__ v, float* __restrict__ state,
                                                        const uint64_t n, const uint32_t T, const uint32_t lead) {
    // one block handles 1024 consecutive slots of one array inside one layout tile (T is a multiple of 1024)
    const uint32_t per_tile = T / 1024u;                 // blocks per array per layout tile
    const uint64_t b = blockIdx.x;
    const uint64_t j = b / (3u * per_tile);              // layout tile
    const uint32_t r = (uint32_t)(b - j * 3u * per_tile);
    const uint32_t a = r / per_tile;                     // 0 = p, 1 = m, 2 = v
    const uint32_t c = r - a * per_tile;                 // 1024-element chunk within the tile
    float* __restrict__ arr = a == 0 ? p : (a == 1 ? m : v);
    // position in the subgroup's element order; element e of the arrays sits at position e + lead
    const uint64_t q0 = j * T + (uint64_t)c * 1024u + (uint64_t)threadIdx.x * 4u;
    float* __restrict__ sp = state + j * 3u * (uint64_t)T + (uint64_t)a * T + (uint64_t)c * 1024u +
                             (uint64_t)threadIdx.x * 4u;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint64_t q = q0 + (uint64_t)k;
        const bool real = q >= lead && q - lead < n;
        if (PACK)
            sp[k] = real ? arr[q - lead] : 0.0f;
        else if (real)
            arr[q - lead] = sp[k];
    }
}

int launch(bool pack, float* p, float* m, float* v, float* state, uint64_t n, int32_t tile_elems, int32_t lead,
           hipStream_t st) {
    if (n == 0) return MLPO_OK;
    const uint64_t T = (uint64_t)tile_elems;
    const uint64_t tiles = (n + (uint64_t)lead + T - 1) / T;
    const uint64_t blocks = tiles * 3u * (T / 1024u);
    if (blocks > 0x7FFFFFFFull) return fail(MLPO_EINVAL, "state too large for one call (%llu elements)", (unsigned long long)n);
    if (pack)
        hipLaunchKernelGGL(repack_kernel<true>, dim3((uint32_t)blocks), dim3(kBlock), 0, st, p, m, v, state, n, (uint32_t)T,
                           (uint32_t)lead);
    else
        hipLaunchKernelGGL(repack_kernel<false>, dim3((uint32_t)blocks), dim3(kBlock), 0, st, p, m, v, state, n, (uint32_t)T,
                           (uint32_t)lead);
    MLPO_HIP(hipGetLastError());
    return MLPO_OK;
}

int check(const void* p, const void* m, const void* v, const void* state, uint64_t n, int32_t tile_elems,
          int32_t lead) {
    if (tile_elems <= 0 || tile_elems % 1024 != 0) return fail(MLPO_EINVAL, "tile_elems must be a positive multiple of 1024");
    if (lead < 0 || lead >= 1024 || lead % 4 != 0) return fail(MLPO_EINVAL, "lead must be a multiple of 4 in 0..1020");
    if (n > ((uint64_t)1 << 48)) return fail(MLPO_EINVAL, "n is implausibly large");
    if (n != 0 && (p == nullptr || m == nullptr || v == nullptr || state == nullptr)) return fail(MLPO_EINVAL, "NULL pointer");
    auto mis = [](const void* q) { return (reinterpret_cast<uintptr_t>(q) & 3u) != 0; };
    if (mis(p) || mis(m) || mis(v) || mis(state)) return fail(MLPO_EINVAL, "pointers must be 4-byte aligned");
    return MLPO_OK;
}

}  // namespace
}  // namespace mlpo

using namespace mlpo;

extern "C" {

int mlpo_state_pack(const float* p, const float* m, const float* v, uint64_t n, int32_t tile_elems, int32_t lead,
                    float* state, void* stream) {
    const int rc = check(p, m, v, state, n, tile_elems, lead);
    if (rc != MLPO_OK) return rc;
    return launch(true, const_cast<float*>(p), const_cast<float*>(m), const_cast<float*>(v), state, n, tile_elems,
                  lead, static_cast<hipStream_t>(stream));
}

int mlpo_state_unpack(const float* state, uint64_t n, int32_t tile_elems, int32_t lead, float* p, float* m, float* v,
                      void* stream) {
    const int rc = check(p, m, v, state, n, tile_elems, lead);
    if (rc != MLPO_OK) return rc;
    return launch(false, p, m, v, const_cast<float*>(state), n, tile_elems, lead, static_cast<hipStream_t>(stream));
}

}  // extern "C"
