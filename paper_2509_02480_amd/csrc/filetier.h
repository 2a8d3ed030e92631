// The file path of the offloaded tier (internal to libmlpo; see filetier.hip).
#pragma once

#include <condition_variable>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

#include "mlpo_internal.h"

namespace mlpo {

// How a descriptor's data is moved: pread / pwrite straight into the bounce buffer, the same through page-aligned
// blocks (O_DIRECT), or copies through a mapping (fully allocated tmpfs files).
enum class FileIo { kBuffered, kDirect, kMapped };
FileIo file_io_kind(int fd);

// One piece that passes through a bounce buffer: read from a file into the buffer (unless the piece comes from pinned
// memory and the kernel itself fills the buffer), updated by the kernel, written from the buffer to a file (unless the
// kernel stored the result straight into pinned memory).  At least one of the two file sides is present.
struct FileJob {
    bool has_read = true, has_write = true;
    int rd_fd = -1, wr_fd = -1;
    uint64_t rd_off = 0, wr_off = 0;  // byte offsets of the piece in the two files
    FileIo rd_io = FileIo::kBuffered, wr_io = FileIo::kBuffered;
    size_t bytes = 0;
    void* buffer = nullptr;  // its bounce buffer (pinned host): the pool's buffer (position in the pool) % (pool's slots)
    int pool = 0;            // the path whose workers move it and whose bounce buffers it passes through
    SgView view{};           // what the kernel reads and where it stores
};

// The workers of the file paths (Section 3.2 "Unified Multi-level, Multi-path Asynchronous Offloading using Virtual
// Tiers": every path has workers of its own, so that a slow path does not hold up a fast one).  Each pool - one per
// path - reads ITS jobs in order into ITS bounce buffers and writes each back after its kernel has finished, with
// n_threads threads per direction that each move an equal share of every piece.  The job at position q of a pool may
// be read once the job at position q - slots[pool] has been written (the buffer is the same), so at most slots[pool]
// pieces of a path are in flight; the pools do not wait for one another.
// The owner launches the kernels: it learns from is_read / wait_any_read that a piece has arrived and reports the
// event that marks the end of the piece's kernel with hand_to_writer.
class FilePath {
  public:
    // jobs in processing order, each with its pool; slots[p] = bounce buffers of pool p (>= 1).
    FilePath(std::vector<FileJob> jobs, std::vector<int> slots, int n_threads, int device);
    ~FilePath();
    FilePath(const FilePath&) = delete;
    FilePath& operator=(const FilePath&) = delete;

    bool start();  // false: a thread could not be started (join reports why)
    size_t size() const { return jobs_.size(); }
    const FileJob& job(size_t i) const { return jobs_[i]; }
    int n_pools() const { return (int)pool_jobs_.size(); }
    size_t pool_size(int p) const { return pool_jobs_[(size_t)p].size(); }
    size_t pool_job(int p, size_t q) const { return pool_jobs_[(size_t)p][q]; }  // index of the pool's q-th job
    bool is_read(size_t i);                         // never blocks
    bool wait_read(size_t i);                       // false: the path has stopped and the piece will not arrive
    // Waits until one of the jobs listed has been read; false: the paths have stopped and none of them will arrive.
    bool wait_any_read(const std::vector<size_t>& jobs);
    bool failed();
    void stop();                                    // the owner gave up: waiting threads leave without an error text
    void hand_to_writer(size_t i, hipEvent_t done);  // done: recorded behind the piece's kernel
    // Waits for all threads.  false: something failed, *error says what.  stats: all pools together; per_pool (may be
    // NULL): what each pool moved.
    bool join(mlpo_file_stats* stats, std::string* error, std::vector<mlpo_file_stats>* per_pool = nullptr);

  private:
    struct PoolStats {
        uint64_t bytes_read = 0, bytes_written = 0;
        double read_seconds = 0.0, write_seconds = 0.0, t_end = 0.0;
    };
    void read_loop(int pool, int r);
    void write_loop(int pool, int r);
    void join_threads();
    void fail_with(const std::string& why);

    std::vector<FileJob> jobs_;
    std::vector<std::vector<size_t>> pool_jobs_;  // per pool: its jobs, in order
    std::vector<int> slots_;
    int n_threads_, device_;
    std::mutex mu_;
    std::condition_variable cv_;
    std::vector<int> read_, launched_, written_;  // read_ / written_: threads that have moved their share
    std::vector<hipEvent_t> done_;
    bool stopped_ = false;
    std::string error_;
    std::vector<std::thread> threads_;
    std::vector<PoolStats> stats_;
    double t_begin_ = 0.0;
};

// Argument check of one extent: alignment, a regular file, long enough for state_bytes behind offset.
int check_file_extent(const mlpo_file_extent& x, uint64_t state_bytes, int index);

// The identity of the path a descriptor leads to: the device of its file system (0 if it cannot be told).  Files on
// one file system share its workers and bounce buffers.
uint64_t file_path_id(int fd);

}  // namespace mlpo
