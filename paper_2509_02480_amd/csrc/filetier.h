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
    void* buffer = nullptr;  // its bounce buffer (pinned host); job i uses buffer i % n_slots
    SgView view{};           // what the kernel reads and where it stores
};

// Reads the jobs in order into their bounce buffers and writes each back after its kernel has finished, with
// n_threads threads per direction that each move an equal share of every piece.  Job i may be read once job
// i - n_slots has been written (the buffer is the same), so at most n_slots pieces are in flight.
// The owner launches the kernels: it learns from is_read / wait_read that a piece has arrived and reports the event
// that marks the end of the piece's kernel with hand_to_writer.
class FilePath {
  public:
    FilePath(std::vector<FileJob> jobs, int n_slots, int n_threads, int device);
    ~FilePath();
    FilePath(const FilePath&) = delete;
    FilePath& operator=(const FilePath&) = delete;

    bool start();  // false: a thread could not be started (join reports why)
    size_t size() const { return jobs_.size(); }
    const FileJob& job(size_t i) const { return jobs_[i]; }
    bool is_read(size_t i);                         // never blocks
    bool wait_read(size_t i);                       // false: the path has stopped and the piece will not arrive
    bool failed();
    void stop();                                    // the owner gave up: waiting threads leave without an error text
    void hand_to_writer(size_t i, hipEvent_t done);  // done: recorded behind the piece's kernel
    // Waits for both threads.  false: something failed, *error says what.
    bool join(mlpo_file_stats* stats, std::string* error);

  private:
    void read_loop(int r);
    void write_loop(int r);
    void join_threads();
    void fail_with(const std::string& why);

    std::vector<FileJob> jobs_;
    int n_slots_, n_threads_, device_;
    std::mutex mu_;
    std::condition_variable cv_;
    std::vector<int> read_, launched_, written_;  // read_ / written_: threads that have moved their share
    std::vector<hipEvent_t> done_;
    bool stopped_ = false;
    std::string error_;
    std::vector<std::thread> threads_;
    uint64_t bytes_read_ = 0, bytes_written_ = 0;
    double read_seconds_ = 0.0, write_seconds_ = 0.0, t_begin_ = 0.0, t_end_ = 0.0;
};

// Argument check of one extent: alignment, a regular file, long enough for state_bytes behind offset.
int check_file_extent(const mlpo_file_extent& x, uint64_t state_bytes, int index);

}  // namespace mlpo
