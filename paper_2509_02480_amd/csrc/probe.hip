// Yardstick kernels (gfx950): what the memory system delivers for the access pattern of the update kernel without its
// arithmetic and without its 2-byte arrays - 128-bit non-temporal accesses, 256 lanes, one 4 KiB piece per workgroup.
// For measurement only; the update path does not use them.
#include "mlpo_internal.h"

namespace mlpo {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int kBlock = 256;

__global__ void __launch_bounds__(kBlock) probe_read(const f32x4* __restrict__ p, uint64_t n4, float* sink) {
    const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < n4) {
        const f32x4 v = __builtin_nontemporal_load(p + i);
        if (v.x == 123.456f && v.y == -7.0f && v.z == 1e30f) *sink = v.w;  // keeps the load alive; practically never true
    }
}

__global__ void __launch_bounds__(kBlock) probe_write(f32x4* __restrict__ p, uint64_t n4) {
    const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < n4) {
        const float x = (float)(i & 1023u);
        const f32x4 v = {x, x + 0.25f, x + 0.5f, x + 0.75f};
        __builtin_nontemporal_store(v, p + i);
    }
}

__global__ void __launch_bounds__(kBlock) probe_rmw(f32x4* __restrict__ p, uint64_t n4) {
    const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < n4) {
        f32x4 v = __builtin_nontemporal_load(p + i);
        v = v * 0.5f;
        __builtin_nontemporal_store(v, p + i);
    }
}

}  // namespace
}  // namespace mlpo

using namespace mlpo;

extern "C" int mlpo_probe_bandwidth(int32_t kind, void* buffer, size_t bytes, void* stream) {
    if (kind < MLPO_PROBE_READ || kind > MLPO_PROBE_UPDATE_IN_PLACE) return fail(MLPO_EINVAL, "unknown probe kind %d", kind);
    if (buffer == nullptr || misaligned(buffer, 16)) return fail(MLPO_EINVAL, "buffer is NULL or not 16-byte aligned");
    if (bytes < 32 || bytes % 16 != 0) return fail(MLPO_EINVAL, "bytes must be a multiple of 16, at least 32");
    // the last 16 bytes are kept out of the sweep: the read probe's (never taken) store goes there
    const uint64_t n4 = bytes / 16 - 1;
    const uint64_t blocks = (n4 + kBlock - 1) / kBlock;
    if (blocks > 0x7FFFFFFFull) return fail(MLPO_EINVAL, "buffer too large for one launch");
    f32x4* p = static_cast<f32x4*>(buffer);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (kind == MLPO_PROBE_READ)
        hipLaunchKernelGGL(probe_read, dim3((uint32_t)blocks), dim3(kBlock), 0, st, p, n4, reinterpret_cast<float*>(p + n4));
    else if (kind == MLPO_PROBE_WRITE)
        hipLaunchKernelGGL(probe_write, dim3((uint32_t)blocks), dim3(kBlock), 0, st, p, n4);
    else
        hipLaunchKernelGGL(probe_rmw, dim3((uint32_t)blocks), dim3(kBlock), 0, st, p, n4);
    MLPO_HIP(hipGetLastError());
    return MLPO_OK;
}
