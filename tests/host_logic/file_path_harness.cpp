// CPU harness for the threading of the file path (csrc/filetier.hip is host-only code): many pieces, few bounce
// buffers, several I/O threads per direction; the "kernel" is a loop on the launching thread and the event wait a
// stub.  Every byte of the file must come back incremented exactly once; a read-only descriptor must surface as a
// write error.  Built by tests/test_file_path_host.py, plain and under ThreadSanitizer.
#include <atomic>
#include <fcntl.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <unistd.h>
#include <vector>
#include "filetier.h"
namespace mlpo { int fail(int code, const char*, ...) { return code; } }
static std::atomic<int> g_syncs{0};
hipError_t hipEventSynchronize(hipEvent_t) { ++g_syncs; return hipSuccess; }
using namespace mlpo;
int run(int n_jobs, int n_slots, int n_threads, size_t bytes, bool fail_write) {
    char path[] = "/tmp/mlpo_tsan_XXXXXX";
    int fd = mkstemp(path);
    std::vector<char> init((size_t)n_jobs * bytes);
    for (size_t i = 0; i < init.size(); ++i) init[i] = (char)(i * 7 + 3);
    if (pwrite(fd, init.data(), init.size(), 0) != (ssize_t)init.size()) return 10;
    int io_fd = fd;
    if (fail_write) io_fd = open(path, O_RDONLY);
    std::vector<char> bounce((size_t)n_slots * bytes + 4096);
    char* base = (char*)(((uintptr_t)bounce.data() + 4095) & ~(uintptr_t)4095);
    std::vector<FileJob> jobs;
    for (int i = 0; i < n_jobs; ++i) {
        FileJob j{};
        j.rd_fd = j.wr_fd = io_fd; j.rd_off = j.wr_off = (uint64_t)i * bytes; j.bytes = bytes;
        j.buffer = base + (size_t)(i % n_slots) * bytes;
        jobs.push_back(j);
    }
    FilePath fp(std::move(jobs), n_slots, n_threads, 0);
    if (!fp.start()) return 11;
    int rc = 0;
    for (size_t i = 0; i < fp.size(); ++i) {
        if (fp.failed() || !fp.wait_read(i)) { rc = 1; break; }
        char* b = (char*)fp.job(i).buffer;
        for (size_t k = 0; k < bytes; ++k) b[k] = (char)(b[k] + 1);      // the "kernel"
        fp.hand_to_writer(i, nullptr);
    }
    mlpo_file_stats st; std::string err;
    bool ok = fp.join(&st, &err);
    if (fail_write) { close(io_fd); unlink(path); close(fd); return (!ok && err.find("writing") != std::string::npos) ? 0 : 12; }
    if (!ok || rc) { fprintf(stderr, "failed: %s\n", err.c_str()); return 13; }
    std::vector<char> back(init.size());
    if (pread(fd, back.data(), back.size(), 0) != (ssize_t)back.size()) return 14;
    for (size_t i = 0; i < back.size(); ++i) if (back[i] != (char)(init[i] + 1)) { fprintf(stderr, "mismatch at %zu\n", i); return 15; }
    if (st.bytes_read != init.size() || st.bytes_written != init.size()) return 16;
    close(fd); unlink(path);
    return 0;
}
int main() {
    int bad = 0;
    for (int slots = 1; slots <= 4; ++slots)
        for (int threads = 1; threads <= 6; threads += 2)
            for (int jobs : {1, 2, 7, 40}) {
                int rc = run(jobs, slots, threads, 8192 * 3, false);
                if (rc) { printf("slots %d threads %d jobs %d -> %d\n", slots, threads, jobs, rc); bad = 1; }
            }
    int rc = run(9, 2, 3, 8192 * 3, true);
    if (rc) { printf("write failure case -> %d\n", rc); bad = 1; }
    printf(bad ? "FAILED\n" : "all cases ok (%d event waits)\n", g_syncs.load());
    return bad;
}
