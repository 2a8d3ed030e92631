// Yardsticks for bench.py (gfx950): what the memory system and the host link deliver for the access patterns of the
// update path WITHOUT its arithmetic.  A measuring aid beside the benchmark, built into its own shared object
// (libbench_yardsticks.so); the update library neither contains nor uses any of it.
//
//   ys_sweep          one pass over a buffer with 128-bit non-temporal accesses, 256 lanes, one 4 KiB piece per
//                     workgroup: read only, write only, or read-modify-write in place
//   ys_update_pattern the address streams of the fused update and nothing else: per group of four elements three
//                     16-byte loads and stores (p, m, v, in place) plus one 8-byte load (g) and one 8-byte store
//                     (p16), planar (three arrays) or tiled (p, m, v interleaved in runs of T elements)
//   ys_link           pinned-memory copies over the host link: each direction alone and both at once
// Compiled with -DYS_LINK_MAIN the file is also a small program that runs ys_link on buffers of its own
// (bench_link_yardstick).
//
// Every function returns 0 or a negative number and leaves a text for ys_last_error().
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <chrono>

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
constexpr int kBlock = 256;

thread_local char g_err[256] = "";
int fail(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return -1;
}
#define YS_HIP(call)                                                          \
    do {                                                                      \
        hipError_t e_ = (call);                                               \
        if (e_ != hipSuccess) return fail("%s: %s", #call, hipGetErrorString(e_)); \
    } while (0)

__global__ void __launch_bounds__(kBlock) sweep_read(const f32x4* __restrict__ p, uint64_t n4, float* sink) {
    const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < n4) {
        const f32x4 v = __builtin_nontemporal_load(p + i);
        if (v.x == 123.456f && v.y == -7.0f && v.z == 1e30f) *sink = v.w;  // keeps the load alive; practically never true
    }
}

__global__ void __launch_bounds__(kBlock) sweep_write(f32x4* __restrict__ p, uint64_t n4) {
    const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < n4) {
        const float x = (float)(i & 1023u);
        const f32x4 v = {x, x + 0.25f, x + 0.5f, x + 0.75f};
        __builtin_nontemporal_store(v, p + i);
    }
}

__global__ void __launch_bounds__(kBlock) sweep_rmw(f32x4* __restrict__ p, uint64_t n4) {
    const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < n4) {
        f32x4 v = __builtin_nontemporal_load(p + i);
        v = v * 0.5f;
        __builtin_nontemporal_store(v, p + i);
    }
}

// One workgroup per 1024 elements, as in the update kernel.  tiles_per_T = 0: planar, the three arrays are indexed
// alike.  Else the state is tiled: kernel tile t lives at (t / tiles_per_T) * S4 + (t % tiles_per_T) * 256 groups of
// four from each array's base (m = p + T, v = p + 2T are passed in as such).
__global__ void __launch_bounds__(kBlock) update_pattern(f32x4* __restrict__ p, f32x4* __restrict__ m,
                                                         f32x4* __restrict__ v, const u32x2* __restrict__ g,
                                                         u32x2* __restrict__ h, uint64_t n4, uint32_t tiles_per_T,
                                                         uint32_t S4) {
    const uint32_t t = blockIdx.x;
    const uint64_t q = (uint64_t)t * kBlock + threadIdx.x;
    if (q >= n4) return;
    uint64_t off = q;
    if (tiles_per_T != 0u) {
        const uint32_t j = t / tiles_per_T;
        off = (uint64_t)j * S4 + (uint64_t)(t - j * tiles_per_T) * kBlock + threadIdx.x;
    }
    f32x4 a = __builtin_nontemporal_load(p + off);
    f32x4 b = __builtin_nontemporal_load(m + off);
    f32x4 c = __builtin_nontemporal_load(v + off);
    const u32x2 w = __builtin_nontemporal_load(g + q);
    a = a * 0.5f;
    b = b * 0.5f;
    c = c * 0.5f;
    __builtin_nontemporal_store(a, p + off);
    __builtin_nontemporal_store(b, m + off);
    __builtin_nontemporal_store(c, v + off);
    u32x2 o;
    o.x = w.x ^ 0x00010001u;
    o.y = w.y ^ 0x00010001u;
    h[q] = o;
}

double now_seconds() {
    using clock = std::chrono::steady_clock;
    return std::chrono::duration<double>(clock::now().time_since_epoch()).count();
}

}  // namespace

extern "C" {

const char* ys_last_error(void) { return g_err; }

// kind 0: read, 1: write (word i gets x, x + 1/4, x + 1/2, x + 3/4 with x = i mod 1024), 2: halve every float in
// place.  buffer: device memory, 16-byte aligned; bytes a multiple of 16, at least 32; the last 16 bytes are left
// alone (the read sweep's never-taken store points there).  Asynchronous on stream.
int ys_sweep(int32_t kind, void* buffer, size_t bytes, void* stream) {
    if (kind < 0 || kind > 2) return fail("unknown sweep kind %d", kind);
    if (buffer == nullptr || (reinterpret_cast<uintptr_t>(buffer) & 15u) != 0) return fail("buffer is NULL or not 16-byte aligned");
    if (bytes < 32 || bytes % 16 != 0) return fail("bytes must be a multiple of 16, at least 32");
    const uint64_t n4 = bytes / 16 - 1;
    const uint64_t blocks = (n4 + kBlock - 1) / kBlock;
    if (blocks > 0x7FFFFFFFull) return fail("buffer too large for one launch");
    f32x4* p = static_cast<f32x4*>(buffer);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (kind == 0)
        hipLaunchKernelGGL(sweep_read, dim3((uint32_t)blocks), dim3(kBlock), 0, st, p, n4, reinterpret_cast<float*>(p + n4));
    else if (kind == 1)
        hipLaunchKernelGGL(sweep_write, dim3((uint32_t)blocks), dim3(kBlock), 0, st, p, n4);
    else
        hipLaunchKernelGGL(sweep_rmw, dim3((uint32_t)blocks), dim3(kBlock), 0, st, p, n4);
    YS_HIP(hipGetLastError());
    return 0;
}

// One ys_sweep launch stamped with its own begin and end on the device (events attached to the dispatch), waited for;
// *ms receives the duration.  What a single short kernel takes from its first wavefront to its last, ramp and tail
// included - back-to-back launches overlap those and look faster than any one of them is.
int ys_sweep_timed(int32_t kind, void* buffer, size_t bytes, void* stream, float* ms) {
    if (ms == nullptr) return fail("ms is NULL");
    if (kind < 0 || kind > 2) return fail("unknown sweep kind %d", kind);
    if (buffer == nullptr || (reinterpret_cast<uintptr_t>(buffer) & 15u) != 0) return fail("buffer is NULL or not 16-byte aligned");
    if (bytes < 32 || bytes % 16 != 0) return fail("bytes must be a multiple of 16, at least 32");
    const uint64_t n4 = bytes / 16 - 1;
    const uint64_t blocks = (n4 + kBlock - 1) / kBlock;
    if (blocks > 0x7FFFFFFFull) return fail("buffer too large for one launch");
    f32x4* p = static_cast<f32x4*>(buffer);
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipEvent_t t0 = nullptr, t1 = nullptr;
    YS_HIP(hipEventCreate(&t0));
    if (hipEventCreate(&t1) != hipSuccess) {
        (void)hipEventDestroy(t0);
        return fail("cannot create an event");
    }
    if (kind == 0)
        hipExtLaunchKernelGGL(sweep_read, dim3((uint32_t)blocks), dim3(kBlock), 0, st, t0, t1, 0, p, n4,
                              reinterpret_cast<float*>(p + n4));
    else if (kind == 1)
        hipExtLaunchKernelGGL(sweep_write, dim3((uint32_t)blocks), dim3(kBlock), 0, st, t0, t1, 0, p, n4);
    else
        hipExtLaunchKernelGGL(sweep_rmw, dim3((uint32_t)blocks), dim3(kBlock), 0, st, t0, t1, 0, p, n4);
    int rc = 0;
    if (hipGetLastError() != hipSuccess || hipEventSynchronize(t1) != hipSuccess ||
        hipEventElapsedTime(ms, t0, t1) != hipSuccess)
        rc = fail("timed launch failed");
    (void)hipEventDestroy(t0);
    (void)hipEventDestroy(t1);
    return rc;
}

// The update's address streams over n elements (a multiple of 4).  tile_elems = 0: p, m, v are three device arrays of
// n floats.  tile_elems = T (a multiple of 1024): p is one tiled buffer of ceil(n / T) * 3T floats and m, v are
// ignored.  g and h: n 16-bit values each, 8-byte aligned.  Halves p, m, v in place, writes g with the lowest
// mantissa bit of every value flipped to h.  Asynchronous on stream.
int ys_update_pattern(float* p, float* m, float* v, const uint16_t* g, uint16_t* h, uint64_t n, int32_t tile_elems,
                      void* stream) {
    if (p == nullptr || g == nullptr || h == nullptr) return fail("NULL pointer");
    if (n == 0 || n % 4 != 0) return fail("n must be a positive multiple of 4");
    if (tile_elems < 0 || tile_elems % 1024 != 0) return fail("tile_elems must be 0 or a multiple of 1024");
    if (tile_elems > 0) {
        m = p + tile_elems;
        v = p + 2 * (size_t)tile_elems;
    } else if (m == nullptr || v == nullptr) {
        return fail("NULL pointer");
    }
    const uint64_t n4 = n / 4;
    const uint64_t blocks = (n4 + kBlock - 1) / kBlock;
    if (blocks > 0x7FFFFFFFull) return fail("too large for one launch");
    hipLaunchKernelGGL(update_pattern, dim3((uint32_t)blocks), dim3(kBlock), 0, static_cast<hipStream_t>(stream),
                       reinterpret_cast<f32x4*>(p), reinterpret_cast<f32x4*>(m), reinterpret_cast<f32x4*>(v),
                       reinterpret_cast<const u32x2*>(g), reinterpret_cast<u32x2*>(h), n4,
                       tile_elems > 0 ? (uint32_t)(tile_elems / 1024) : 0u, (uint32_t)(3 * (uint64_t)tile_elems / 4));
    YS_HIP(hipGetLastError());
    return 0;
}

// Pinned-memory copies of `bytes` bytes, `reps` times each after one untimed round: host_src -> dev_dst alone,
// dev_src -> host_dst alone, then both at the same time on two streams of their own.  seconds[0..2] receive the wall
// time per repetition of the three legs (host clock around stream synchronisation).  The four buffers must not
// overlap; host buffers are pinned (hipHostMalloc).  Synchronous.
int ys_link(const void* host_src, void* dev_dst, const void* dev_src, void* host_dst, size_t bytes, int32_t reps,
            double* seconds) {
    if (host_src == nullptr || dev_dst == nullptr || dev_src == nullptr || host_dst == nullptr || seconds == nullptr)
        return fail("NULL pointer");
    if (bytes == 0 || reps < 1) return fail("bytes and reps must be positive");
    hipStream_t in = nullptr, out = nullptr;
    YS_HIP(hipStreamCreateWithFlags(&in, hipStreamNonBlocking));
    if (hipStreamCreateWithFlags(&out, hipStreamNonBlocking) != hipSuccess) {
        (void)hipStreamDestroy(in);
        return fail("cannot create a stream");
    }
    int rc = 0;
    for (int leg = 0; leg < 3 && rc == 0; ++leg) {
        const bool up = leg != 1, down = leg != 0;
        for (int r = -1; r < reps && rc == 0; ++r) {  // r = -1: warm-up
            if (r == 0) {
                if (hipStreamSynchronize(in) != hipSuccess || hipStreamSynchronize(out) != hipSuccess) rc = fail("sync failed");
                seconds[leg] = now_seconds();
            }
            if (up && hipMemcpyAsync(dev_dst, host_src, bytes, hipMemcpyHostToDevice, in) != hipSuccess) rc = fail("h2d copy failed");
            if (down && hipMemcpyAsync(host_dst, dev_src, bytes, hipMemcpyDeviceToHost, out) != hipSuccess) rc = fail("d2h copy failed");
        }
        if (rc == 0 && (hipStreamSynchronize(in) != hipSuccess || hipStreamSynchronize(out) != hipSuccess)) rc = fail("sync failed");
        if (rc == 0) seconds[leg] = (now_seconds() - seconds[leg]) / reps;
    }
    (void)hipStreamDestroy(in);
    (void)hipStreamDestroy(out);
    return rc;
}

}  // extern "C"

#ifdef YS_LINK_MAIN
// The same three legs as ys_link in a process of its own (bench.py starts it before it touches the GPU itself): two
// streams in a fresh process with nothing else on the device.  Prints one JSON line.
int main(int argc, char** argv) {
    const size_t bytes = (argc > 1 ? (size_t)atoll(argv[1]) : 400) << 20;
    void *ha = nullptr, *hb = nullptr, *da = nullptr, *db = nullptr;
    if (hipHostMalloc(&ha, bytes, 0) != hipSuccess || hipHostMalloc(&hb, bytes, 0) != hipSuccess ||
        hipMalloc(&da, bytes) != hipSuccess || hipMalloc(&db, bytes) != hipSuccess) {
        printf("{\"error\": \"allocation failed\"}\n");
        return 1;
    }
    memset(ha, 1, bytes);
    memset(hb, 2, bytes);
    double sec[3] = {0, 0, 0};
    if (ys_link(ha, da, db, hb, bytes, 4, sec) != 0) {
        printf("{\"error\": \"%s\"}\n", ys_last_error());
        return 1;
    }
    printf("{\"bytes\": %zu, \"h2d_GBs\": %.2f, \"d2h_GBs\": %.2f, \"bidir_GBs_per_dir\": %.2f}\n", bytes,
           bytes / sec[0] / 1e9, bytes / sec[1] / 1e9, bytes / sec[2] / 1e9);
    (void)hipHostFree(ha);
    (void)hipHostFree(hb);
    (void)hipFree(da);
    (void)hipFree(db);
    return 0;
}
#endif
