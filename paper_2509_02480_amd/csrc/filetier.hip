// The file path of the offloaded tier: subgroups whose fp32 state lives in a file pass through pinned bounce buffers
// (Section 3.2 "Unified Multi-level, Multi-path Asynchronous Offloading using Virtual Tiers": alternative storage
// behind one tier, each path with its own workers; Section 3.4: read, update and write of different subgroups
// overlap).  Host code only: reading threads, writing threads, and the bookkeeping that lets the thread that
// launches kernels know when a piece has arrived and the writers know when its kernel has been enqueued.
#include <errno.h>
#include <fcntl.h>
#include <stdlib.h>
#include <string.h>
#include <sys/mman.h>
#include <sys/stat.h>
#include <sys/vfs.h>
#include <unistd.h>

#include <chrono>
#include <exception>

#include "filetier.h"

namespace mlpo {

namespace {

double now_seconds() {
    using clock = std::chrono::steady_clock;
    return std::chrono::duration<double>(clock::now().time_since_epoch()).count();
}

// pread / pwrite until the whole range has moved; false with errno set (0 = unexpected end of file) otherwise.
bool read_fully(int fd, char* buf, size_t bytes, uint64_t off) {
    while (bytes > 0) {
        const ssize_t r = pread(fd, buf, bytes, (off_t)off);
        if (r < 0) {
            if (errno == EINTR) continue;
            return false;
        }
        if (r == 0) {
            errno = 0;
            return false;
        }
        buf += r;
        off += (uint64_t)r;
        bytes -= (size_t)r;
    }
    return true;
}

bool write_fully(int fd, const char* buf, size_t bytes, uint64_t off) {
    while (bytes > 0) {
        const ssize_t r = pwrite(fd, buf, bytes, (off_t)off);
        if (r < 0) {
            if (errno == EINTR) continue;
            return false;
        }
        if (r == 0) {
            errno = 0;
            return false;
        }
        buf += r;
        off += (uint64_t)r;
        bytes -= (size_t)r;
    }
    return true;
}

// Page-aligned scratch of one I/O thread.  Memory that the HIP runtime pins cannot be the target of direct I/O (the
// kernel refuses to take its pages: EFAULT), so for a descriptor opened with O_DIRECT the data goes through this
// buffer, block by block, and is copied between it and the bounce buffer.
constexpr size_t kDirectBlock = 4u << 20;
struct AlignedBlock {
    char* p = nullptr;
    ~AlignedBlock() { free(p); }
    bool ensure() {
        if (p == nullptr && posix_memalign(reinterpret_cast<void**>(&p), 4096, kDirectBlock) != 0) p = nullptr;
        return p != nullptr;
    }
};

// A fully allocated file in tmpfs is host memory with a name: its pages are copied through a mapping, which -
// unlike write() on one inode - any number of threads can do at once.  off and bytes are multiples of 4096 here.
bool copy_mapped(int fd, char* mem, size_t bytes, uint64_t off, bool to_file) {
    void* m = mmap(nullptr, bytes, to_file ? (PROT_READ | PROT_WRITE) : PROT_READ, MAP_SHARED, fd, (off_t)off);
    if (m == MAP_FAILED) return false;
    if (to_file)
        memcpy(m, mem, bytes);
    else
        memcpy(mem, m, bytes);
    munmap(m, bytes);
    return true;
}

bool read_range(const FileJob& j, size_t begin, size_t bytes, AlignedBlock& tmp) {
    const int fd = j.rd_fd;
    char* dst = static_cast<char*>(j.buffer) + begin;
    uint64_t off = j.rd_off + begin;
    if (j.rd_io == FileIo::kMapped) return copy_mapped(fd, dst, bytes, off, false);
    if (j.rd_io == FileIo::kBuffered) return read_fully(fd, dst, bytes, off);
    if (!tmp.ensure()) {
        errno = ENOMEM;
        return false;
    }
    while (bytes > 0) {
        const size_t len = bytes < kDirectBlock ? bytes : kDirectBlock;
        if (!read_fully(fd, tmp.p, len, off)) return false;
        memcpy(dst, tmp.p, len);
        dst += len;
        off += len;
        bytes -= len;
    }
    return true;
}

bool write_range(const FileJob& j, size_t begin, size_t bytes, AlignedBlock& tmp) {
    const int fd = j.wr_fd;
    char* src = static_cast<char*>(j.buffer) + begin;
    uint64_t off = j.wr_off + begin;
    if (j.wr_io == FileIo::kMapped) return copy_mapped(fd, src, bytes, off, true);
    if (j.wr_io == FileIo::kBuffered) return write_fully(fd, src, bytes, off);
    if (!tmp.ensure()) {
        errno = ENOMEM;
        return false;
    }
    while (bytes > 0) {
        const size_t len = bytes < kDirectBlock ? bytes : kDirectBlock;
        memcpy(tmp.p, src, len);
        if (!write_fully(fd, tmp.p, len, off)) return false;
        src += len;
        off += len;
        bytes -= len;
    }
    return true;
}

// The part of a piece of `bytes` bytes that thread `r` of `n` moves: equal shares, cut at multiples of 4096.
void share_of(size_t bytes, int r, int n, size_t* begin, size_t* len) {
    const size_t per = ((bytes + (size_t)n - 1) / (size_t)n + 4095) / 4096 * 4096;
    const size_t b = per * (size_t)r < bytes ? per * (size_t)r : bytes;
    const size_t e = b + per < bytes ? b + per : bytes;
    *begin = b;
    *len = e - b;
}

}  // namespace

FilePath::FilePath(std::vector<FileJob> jobs, std::vector<int> slots, int n_threads, int device)
    : jobs_(std::move(jobs)), pool_jobs_(slots.size()), slots_(std::move(slots)), n_threads_(n_threads),
      device_(device), read_(jobs_.size(), 0), launched_(jobs_.size(), 0), written_(jobs_.size(), 0),
      done_(jobs_.size(), nullptr), stats_(slots_.size()) {
    for (size_t i = 0; i < jobs_.size(); ++i) pool_jobs_[(size_t)jobs_[i].pool].push_back(i);
}

FilePath::~FilePath() {
    stop();  // threads still waiting (the caller gave up early) leave at their next wait
    join_threads();
}

void FilePath::join_threads() {
    for (std::thread& t : threads_)
        if (t.joinable()) t.join();
}

bool FilePath::start() {
    t_begin_ = now_seconds();
    try {
        for (int p = 0; p < n_pools(); ++p) {
            if (pool_jobs_[(size_t)p].empty()) continue;
            for (int r = 0; r < n_threads_; ++r) {
                threads_.emplace_back(&FilePath::read_loop, this, p, r);
                threads_.emplace_back(&FilePath::write_loop, this, p, r);
            }
        }
    } catch (const std::exception& e) {  // the system refused a thread: nothing may cross the C boundary
        fail_with(std::string("starting an I/O thread: ") + e.what());
        return false;
    }
    return true;
}

void FilePath::fail_with(const std::string& why) {
    std::lock_guard<std::mutex> lk(mu_);
    if (error_.empty()) error_ = why;
    stopped_ = true;
    cv_.notify_all();
}

// Every reading thread of a pool walks over the pool's jobs and moves its share of each; the last one to finish a job
// marks it read.
void FilePath::read_loop(int pool, int r) {
    AlignedBlock tmp;
    const std::vector<size_t>& mine = pool_jobs_[(size_t)pool];
    const size_t slots = (size_t)slots_[(size_t)pool];
    for (size_t q = 0; q < mine.size(); ++q) {
        const size_t i = mine[q];
        {
            std::unique_lock<std::mutex> lk(mu_);
            // the bounce buffer is free once the piece that used it before has been written back
            cv_.wait(lk, [&] { return stopped_ || q < slots || written_[mine[q - slots]] == n_threads_; });
            if (stopped_) return;
        }
        const FileJob& j = jobs_[i];
        size_t begin, len;
        share_of(j.bytes, r, n_threads_, &begin, &len);
        const double t0 = now_seconds();
        if (!j.has_read) len = 0;  // the kernel fills this buffer: only the wait for the buffer above applies
        const bool ok = len == 0 || read_range(j, begin, len, tmp);
        const double t1 = now_seconds();
        if (!ok) {
            const int e = errno;
            fail_with(std::string("reading a file-tier piece: ") + (e ? strerror(e) : "unexpected end of file"));
            return;
        }
        std::lock_guard<std::mutex> lk(mu_);
        stats_[(size_t)pool].read_seconds += t1 - t0;
        stats_[(size_t)pool].bytes_read += len;
        if (++read_[i] == n_threads_) cv_.notify_all();
    }
}

void FilePath::write_loop(int pool, int r) {
    if (hipSetDevice(device_) != hipSuccess) {
        fail_with("hipSetDevice failed in a writing thread");
        return;
    }
    AlignedBlock tmp;
    for (const size_t i : pool_jobs_[(size_t)pool]) {
        hipEvent_t done;
        {
            std::unique_lock<std::mutex> lk(mu_);
            cv_.wait(lk, [&] { return stopped_ || launched_[i]; });
            if (!launched_[i]) return;
            done = done_[i];
        }
        const hipError_t e = hipEventSynchronize(done);
        if (e != hipSuccess) {
            fail_with(std::string("waiting for a file-tier piece's kernel: ") + hipGetErrorString(e));
            return;
        }
        const FileJob& j = jobs_[i];
        size_t begin, len;
        share_of(j.bytes, r, n_threads_, &begin, &len);
        const double t0 = now_seconds();
        if (!j.has_write) len = 0;  // the kernel stored the result elsewhere: the buffer is free once it has finished
        const bool ok = len == 0 || write_range(j, begin, len, tmp);
        const double t1 = now_seconds();
        if (!ok) {
            const int en = errno;
            fail_with(std::string("writing a file-tier piece: ") + (en ? strerror(en) : "nothing written"));
            return;
        }
        std::lock_guard<std::mutex> lk(mu_);
        PoolStats& ps = stats_[(size_t)pool];
        ps.write_seconds += t1 - t0;
        ps.bytes_written += len;
        if (t1 > ps.t_end) ps.t_end = t1;
        if (++written_[i] == n_threads_) cv_.notify_all();
    }
}

bool FilePath::is_read(size_t i) {
    std::lock_guard<std::mutex> lk(mu_);
    return read_[i] == n_threads_;
}

bool FilePath::wait_read(size_t i) {
    std::unique_lock<std::mutex> lk(mu_);
    cv_.wait(lk, [&] { return stopped_ || read_[i] == n_threads_; });
    return read_[i] == n_threads_;
}

bool FilePath::wait_any_read(const std::vector<size_t>& jobs) {
    const auto any = [&] {
        for (const size_t i : jobs)
            if (read_[i] == n_threads_) return true;
        return false;
    };
    std::unique_lock<std::mutex> lk(mu_);
    cv_.wait(lk, [&] { return stopped_ || any(); });
    return any();
}

bool FilePath::failed() {
    std::lock_guard<std::mutex> lk(mu_);
    return !error_.empty();
}

void FilePath::stop() {
    std::lock_guard<std::mutex> lk(mu_);
    stopped_ = true;
    cv_.notify_all();
}

void FilePath::hand_to_writer(size_t i, hipEvent_t done) {
    std::lock_guard<std::mutex> lk(mu_);
    done_[i] = done;
    launched_[i] = 1;
    cv_.notify_all();
}

bool FilePath::join(mlpo_file_stats* stats, std::string* error, std::vector<mlpo_file_stats>* per_pool) {
    join_threads();
    std::lock_guard<std::mutex> lk(mu_);
    mlpo_file_stats all{};
    if (per_pool != nullptr) per_pool->assign(stats_.size(), mlpo_file_stats{});
    for (size_t p = 0; p < stats_.size(); ++p) {
        const PoolStats& ps = stats_[p];
        mlpo_file_stats one{};
        one.bytes_read = ps.bytes_read;
        one.bytes_written = ps.bytes_written;
        one.read_seconds = ps.read_seconds;
        one.write_seconds = ps.write_seconds;
        one.wall_seconds = ps.t_end > t_begin_ ? ps.t_end - t_begin_ : 0.0;
        if (per_pool != nullptr) (*per_pool)[p] = one;
        all.bytes_read += one.bytes_read;
        all.bytes_written += one.bytes_written;
        all.read_seconds += one.read_seconds;
        all.write_seconds += one.write_seconds;
        if (one.wall_seconds > all.wall_seconds) all.wall_seconds = one.wall_seconds;
    }
    if (stats != nullptr) *stats = all;
    if (!error_.empty()) {
        *error = error_;
        return false;
    }
    return true;
}

uint64_t file_path_id(int fd) {
    struct stat sb;
    if (fstat(fd, &sb) != 0) return 0;
    return (uint64_t)sb.st_dev;
}

FileIo file_io_kind(int fd) {
    const int fl = fcntl(fd, F_GETFL);
    if (fl >= 0 && (fl & O_DIRECT) != 0) return FileIo::kDirect;
    struct statfs fs;
    struct stat sb;
    constexpr long kTmpfsMagic = 0x01021994;
    if (fstatfs(fd, &fs) == 0 && (long)fs.f_type == kTmpfsMagic && fstat(fd, &sb) == 0 &&
        (uint64_t)sb.st_blocks * 512u >= (uint64_t)sb.st_size)  // no holes: touching a page cannot fail
        return FileIo::kMapped;
    return FileIo::kBuffered;
}

int check_file_extent(const mlpo_file_extent& x, uint64_t state_bytes, int index) {
    if (x.reserved != 0) return fail(MLPO_EINVAL, "subgroup %d: reserved field of its file extent is not 0", index);
    if (x.offset % 4096u != 0) return fail(MLPO_EINVAL, "subgroup %d: file offset is not a multiple of 4096", index);
    struct stat sb;
    if (fstat(x.fd, &sb) != 0) return fail(MLPO_EINVAL, "subgroup %d: fd %d: %s", index, x.fd, strerror(errno));
    if (!S_ISREG(sb.st_mode)) return fail(MLPO_EINVAL, "subgroup %d: fd %d is not a regular file", index, x.fd);
    if ((uint64_t)sb.st_size < x.offset + state_bytes)
        return fail(MLPO_EINVAL, "subgroup %d: the file has %lld bytes, the state ends at %llu", index,
                    (long long)sb.st_size, (unsigned long long)(x.offset + state_bytes));
    return MLPO_OK;
}

}  // namespace mlpo
