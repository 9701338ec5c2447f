// A small pool of CPU threads that moves pieces between ordinary host memory or files and the
// engine's pinned ring (memcpy, pread, pwrite).
#pragma once

#include <fcntl.h>
#include <unistd.h>

#include <atomic>
#include <cerrno>
#include <condition_variable>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <thread>
#include <vector>

namespace zi {
namespace host {

constexpr size_t kCopyPieceBytes = 4u << 20;

// A few threads that copy a list of (dst, src, bytes) pieces between ordinary host memory and the
// pinned ring.  run() blocks until the whole list is copied; the calling thread takes part.
class CopyPool {
public:
    // op 0: memcpy(mem <- other).  op 1: pread(fd, mem, bytes, file_off), at least `need` bytes must
    // arrive (a read rounded up for direct I/O may end at the end of the file).  op 2: pwrite.
    // `bounce`: the descriptor does direct I/O.  Memory from the HIP page-locked allocator cannot be
    // the target of direct I/O on this driver stack (the kernel refuses to pin it again: EFAULT), so
    // such a piece goes through a 4096-byte aligned per-thread buffer in ordinary memory.
    struct Piece {
        int op;
        char* mem;
        const char* other;
        int fd;
        int64_t file_off;
        size_t bytes;
        size_t need;
        bool bounce;
    };

    explicit CopyPool(int n_threads) : bounce_((size_t)(n_threads < 1 ? 1 : n_threads), nullptr)
    {
        for (int i = 1; i < n_threads; ++i) workers_.emplace_back([this, i] { loop(i); });
    }
    ~CopyPool()
    {
        {
            std::lock_guard<std::mutex> lk(mu_);
            stop_ = true;
        }
        cv_job_.notify_all();
        for (auto& w : workers_) w.join();
        for (char* b : bounce_) std::free(b);
    }
    CopyPool(const CopyPool&) = delete;
    CopyPool& operator=(const CopyPool&) = delete;
    // Returns 0, or the errno of the first failed piece (EIO for a short transfer).
    int run(const std::vector<Piece>& pieces)
    {
        {
            std::lock_guard<std::mutex> lk(mu_);
            pieces_ = &pieces;
            error_.store(0);
            next_.store(0);
            pending_ = (int)workers_.size();
            ++generation_;
        }
        cv_job_.notify_all();
        drain(0);
        std::unique_lock<std::mutex> lk(mu_);
        cv_done_.wait(lk, [this] { return pending_ == 0; });
        pieces_ = nullptr;
        return error_.load();
    }

private:
    // `who`: 0 = the thread that called run(), i = worker i; selects the direct-I/O buffer.
    void drain(int who)
    {
        const std::vector<Piece>& ps = *pieces_;
        for (size_t i = next_.fetch_add(1); i < ps.size(); i = next_.fetch_add(1)) {
            const Piece& p = ps[i];
            if (p.op == 0) {
                std::memcpy(p.mem, p.other, p.bytes);
                continue;
            }
            char* io = p.mem;
            if (p.bounce) {
                char*& buf = bounce_[(size_t)who];
                if (!buf && posix_memalign((void**)&buf, 4096, kCopyPieceBytes) != 0) {
                    buf = nullptr;
                    int expected = 0;
                    error_.compare_exchange_strong(expected, ENOMEM);
                    continue;
                }
                io = buf;
                if (p.op == 2) std::memcpy(io, p.mem, p.bytes);
            }
            size_t done = 0;
            while (done < p.bytes) {
                const ssize_t r = p.op == 1 ? pread(p.fd, io + done, p.bytes - done, p.file_off + (int64_t)done)
                                            : pwrite(p.fd, io + done, p.bytes - done, p.file_off + (int64_t)done);
                if (r < 0) {
                    if (errno == EINTR) continue;
                    int expected = 0;
                    error_.compare_exchange_strong(expected, errno);
                    break;
                }
                if (r == 0) break;      // end of file
                done += (size_t)r;
            }
            if (done < (p.op == 1 ? p.need : p.bytes)) {
                int expected = 0;
                error_.compare_exchange_strong(expected, EIO);
            } else if (p.bounce && p.op == 1) {
                std::memcpy(p.mem, io, done);
            }
        }
    }
    void loop(int who)
    {
        uint64_t seen = 0;
        for (;;) {
            {
                std::unique_lock<std::mutex> lk(mu_);
                cv_job_.wait(lk, [&] { return stop_ || generation_ != seen; });
                if (stop_) return;
                seen = generation_;
            }
            drain(who);
            {
                std::lock_guard<std::mutex> lk(mu_);
                --pending_;
            }
            cv_done_.notify_one();
        }
    }
    std::vector<std::thread> workers_;
    std::vector<char*> bounce_;         // per thread, allocated on first direct-I/O piece
    std::mutex mu_;
    std::condition_variable cv_job_, cv_done_;
    const std::vector<Piece>* pieces_ = nullptr;
    std::atomic<size_t> next_{0};
    std::atomic<int> error_{0};
    uint64_t generation_ = 0;
    int pending_ = 0;
    bool stop_ = false;
};

}  // namespace host
}  // namespace zi
