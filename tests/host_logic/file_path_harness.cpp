// CPU harness for the threading of the file paths (csrc/filetier.hip is host-only code): many pieces, few bounce
// buffers, several I/O threads per direction and path; the "kernel" is a loop on the launching thread and the event
// wait a stub.  Every byte of every file must come back incremented exactly once; a read-only descriptor must
// surface as a write error; with two paths of which one is slow (its pieces are ten times as large) the pieces of the
// fast path must all be served without waiting for the slow one.  Built by tests/test_file_path_host.py, plain and
// under ThreadSanitizer.
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

struct TestFile {
    char path[32];
    int fd = -1;
    std::vector<char> init;
    bool make(size_t bytes, int salt) {
        strcpy(path, "/tmp/mlpo_tsan_XXXXXX");
        fd = mkstemp(path);
        init.resize(bytes);
        for (size_t i = 0; i < bytes; ++i) init[i] = (char)(i * 7 + 3 + salt);
        return fd >= 0 && pwrite(fd, init.data(), bytes, 0) == (ssize_t)bytes;
    }
    bool incremented_once() {
        std::vector<char> back(init.size());
        if (pread(fd, back.data(), back.size(), 0) != (ssize_t)back.size()) return false;
        for (size_t i = 0; i < back.size(); ++i)
            if (back[i] != (char)(init[i] + 1)) { fprintf(stderr, "mismatch at %zu\n", i); return false; }
        return true;
    }
    void drop() { close(fd); unlink(path); }
};

// The owner's loop as the library runs it: per path a cursor, a piece of any path as soon as it has been read.
static int drive(FilePath& fp, std::vector<size_t>* order) {
    const int n_pools = fp.n_pools();
    std::vector<size_t> next((size_t)n_pools, 0);
    for (;;) {
        if (fp.failed()) return 1;
        std::vector<size_t> waiting;
        for (int p = 0; p < n_pools; ++p)
            if (next[(size_t)p] < fp.pool_size(p)) waiting.push_back(fp.pool_job(p, next[(size_t)p]));
        if (waiting.empty()) return 0;
        int ready = -1;
        for (int p = 0; p < n_pools && ready < 0; ++p)
            if (next[(size_t)p] < fp.pool_size(p) && fp.is_read(fp.pool_job(p, next[(size_t)p]))) ready = p;
        if (ready < 0) {
            if (!fp.wait_any_read(waiting)) return 1;
            continue;
        }
        const size_t i = fp.pool_job(ready, next[(size_t)ready]++);
        char* b = (char*)fp.job(i).buffer;
        for (size_t k = 0; k < fp.job(i).bytes; ++k) b[k] = (char)(b[k] + 1);  // the "kernel"
        fp.hand_to_writer(i, nullptr);
        if (order) order->push_back(i);
    }
}

int run(int n_jobs, int n_slots, int n_threads, size_t bytes, bool fail_write) {
    TestFile f;
    if (!f.make((size_t)n_jobs * bytes, 0)) return 10;
    int io_fd = f.fd;
    if (fail_write) io_fd = open(f.path, O_RDONLY);
    std::vector<char> bounce((size_t)n_slots * bytes + 4096);
    char* base = (char*)(((uintptr_t)bounce.data() + 4095) & ~(uintptr_t)4095);
    std::vector<FileJob> jobs;
    for (int i = 0; i < n_jobs; ++i) {
        FileJob j{};
        j.rd_fd = j.wr_fd = io_fd; j.rd_off = j.wr_off = (uint64_t)i * bytes; j.bytes = bytes;
        j.buffer = base + (size_t)(i % n_slots) * bytes;
        jobs.push_back(j);
    }
    FilePath fp(std::move(jobs), std::vector<int>{n_slots}, n_threads, 0);
    if (!fp.start()) return 11;
    const int rc = drive(fp, nullptr);
    mlpo_file_stats st; std::string err;
    bool ok = fp.join(&st, &err);
    if (fail_write) { close(io_fd); f.drop(); return (!ok && err.find("writing") != std::string::npos) ? 0 : 12; }
    if (!ok || rc) { fprintf(stderr, "failed: %s\n", err.c_str()); return 13; }
    if (!f.incremented_once()) return 15;
    if (st.bytes_read != f.init.size() || st.bytes_written != f.init.size()) return 16;
    f.drop();
    return 0;
}

// Two paths with pools of their own: the slow one's pieces are ten times as large and interleaved in the job list
// in front of the fast one's.  Every byte of both files must come back incremented once, the per-path statistics
// must add up, and all pieces of the fast path must have been served before the last piece of the slow one.
int run_two_paths(int n_fast, int n_slow, int slots_each, int n_threads) {
    const size_t small = 4096 * 2, big = small * 10;
    TestFile fast, slow;
    if (!fast.make((size_t)n_fast * small, 1) || !slow.make((size_t)n_slow * big, 2)) return 20;
    std::vector<char> bounce((size_t)slots_each * (small + big) + 4096);
    char* base = (char*)(((uintptr_t)bounce.data() + 4095) & ~(uintptr_t)4095);
    char* base_slow = base;                                   // pool 0: the slow path
    char* base_fast = base + (size_t)slots_each * big;        // pool 1: the fast path
    std::vector<FileJob> jobs;
    int qs = 0, qf = 0;
    while (qs < n_slow || qf < n_fast) {                      // slow, fast, slow, fast, ...
        if (qs < n_slow) {
            FileJob j{};
            j.pool = 0; j.rd_fd = j.wr_fd = slow.fd; j.rd_off = j.wr_off = (uint64_t)qs * big; j.bytes = big;
            j.buffer = base_slow + (size_t)(qs % slots_each) * big;
            jobs.push_back(j); ++qs;
        }
        if (qf < n_fast) {
            FileJob j{};
            j.pool = 1; j.rd_fd = j.wr_fd = fast.fd; j.rd_off = j.wr_off = (uint64_t)qf * small; j.bytes = small;
            j.buffer = base_fast + (size_t)(qf % slots_each) * small;
            jobs.push_back(j); ++qf;
        }
    }
    FilePath fp(std::move(jobs), std::vector<int>{slots_each, slots_each}, n_threads, 0);
    if (fp.n_pools() != 2 || fp.pool_size(0) != (size_t)n_slow || fp.pool_size(1) != (size_t)n_fast) return 21;
    if (!fp.start()) return 22;
    std::vector<size_t> order;
    const int rc = drive(fp, &order);
    mlpo_file_stats st; std::string err; std::vector<mlpo_file_stats> per;
    if (!fp.join(&st, &err, &per) || rc) { fprintf(stderr, "failed: %s\n", err.c_str()); return 23; }
    if (!fast.incremented_once() || !slow.incremented_once()) return 24;
    if (per.size() != 2 || per[0].bytes_read != slow.init.size() || per[1].bytes_written != fast.init.size() ||
        st.bytes_read != slow.init.size() + fast.init.size())
        return 25;
    if (order.size() != (size_t)(n_slow + n_fast)) return 26;
    fast.drop(); slow.drop();
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
    for (int slots = 1; slots <= 3; ++slots)
        for (int threads : {1, 3}) {
            rc = run_two_paths(30, 6, slots, threads);
            if (rc) { printf("two paths: slots %d threads %d -> %d\n", slots, threads, rc); bad = 1; }
        }
    rc = run_two_paths(0, 5, 2, 2);      // a path without pieces starts no threads
    if (rc) { printf("two paths, one empty -> %d\n", rc); bad = 1; }
    printf(bad ? "FAILED\n" : "all cases ok (%d event waits)\n", g_syncs.load());
    return bad;
}
