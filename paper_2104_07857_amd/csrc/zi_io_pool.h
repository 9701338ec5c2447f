// CPU-side helpers of the streaming engine: a small pool of parked threads that runs index-space
// jobs (copies between ordinary host memory or files and the pinned ring; blocks of the host step),
// and a single parked thread that runs one stage of a pipeline.  All threads are created with the
// object and parked on a condition variable between jobs, so the calls that use them start none.
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

// n_threads - 1 parked workers plus the calling thread.  run() hands out the indices 0..n-1 one at a
// time and blocks until all are done; it returns 0 or the first non-zero value a task returned.
class TaskPool {
public:
    // `who`: 0 = the thread that called run(), i = worker i (selects per-thread scratch).
    typedef int (*TaskFn)(void* ctx, size_t index, int who);

    explicit TaskPool(int n_threads) : bounce_((size_t)(n_threads < 1 ? 1 : n_threads), nullptr)
    {
        for (int i = 1; i < n_threads; ++i) workers_.emplace_back([this, i] { loop(i); });
    }
    ~TaskPool()
    {
        {
            std::lock_guard<std::mutex> lk(mu_);
            stop_ = true;
        }
        cv_job_.notify_all();
        for (auto& w : workers_) w.join();
        for (char* b : bounce_) std::free(b);
    }
    TaskPool(const TaskPool&) = delete;
    TaskPool& operator=(const TaskPool&) = delete;

    int threads() const { return (int)workers_.size() + 1; }

    int run(size_t n, TaskFn fn, void* ctx)
    {
        {
            std::lock_guard<std::mutex> lk(mu_);
            fn_ = fn;
            ctx_ = ctx;
            count_ = n;
            error_.store(0);
            next_.store(0);
            pending_ = (int)workers_.size();
            ++generation_;
        }
        cv_job_.notify_all();
        drain(0);
        std::unique_lock<std::mutex> lk(mu_);
        cv_done_.wait(lk, [this] { return pending_ == 0; });
        fn_ = nullptr;
        return error_.load();
    }

    // A 4096-byte aligned buffer of kCopyPieceBytes owned by thread `who` (allocated on first use;
    // null if memory is short).  Direct I/O goes through it.
    char* bounce(int who)
    {
        char*& buf = bounce_[(size_t)who];
        if (!buf && posix_memalign((void**)&buf, 4096, kCopyPieceBytes) != 0) buf = nullptr;
        return buf;
    }

private:
    void drain(int who)
    {
        for (size_t i = next_.fetch_add(1); i < count_; i = next_.fetch_add(1)) {
            const int err = fn_(ctx_, i, who);
            if (err) {
                int expected = 0;
                error_.compare_exchange_strong(expected, err);
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
    std::vector<char*> bounce_;
    std::mutex mu_;
    std::condition_variable cv_job_, cv_done_;
    TaskFn fn_ = nullptr;
    void* ctx_ = nullptr;
    size_t count_ = 0;
    std::atomic<size_t> next_{0};
    std::atomic<int> error_{0};
    uint64_t generation_ = 0;
    int pending_ = 0;
    bool stop_ = false;
};

// One transfer between the pinned ring and the caller's state.
// op 0: memcpy(mem <- other).  op 1: pread(fd, mem, bytes, file_off), at least `need` bytes must
// arrive (a read rounded up for direct I/O may end at the end of the file).  op 2: pwrite.
// `bounce`: the descriptor does direct I/O.  Memory from the HIP page-locked allocator cannot be
// the target of direct I/O on this driver stack (the kernel refuses to pin it again: EFAULT), so
// such a piece goes through the thread's aligned buffer in ordinary memory.
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

struct PieceJob {
    const Piece* pieces;
    TaskPool* pool;
};

// Returns 0, or the errno of the failure (EIO for a short transfer).
inline int run_one_piece(void* ctx, size_t index, int who)
{
    const PieceJob& job = *static_cast<const PieceJob*>(ctx);
    const Piece& p = job.pieces[index];
    if (p.op == 0) {
        std::memcpy(p.mem, p.other, p.bytes);
        return 0;
    }
    char* io = p.mem;
    if (p.bounce) {
        io = job.pool->bounce(who);
        if (!io) return ENOMEM;
        if (p.op == 2) std::memcpy(io, p.mem, p.bytes);
    }
    size_t done = 0;
    while (done < p.bytes) {
        const ssize_t r = p.op == 1 ? pread(p.fd, io + done, p.bytes - done, p.file_off + (int64_t)done)
                                    : pwrite(p.fd, io + done, p.bytes - done, p.file_off + (int64_t)done);
        if (r < 0) {
            if (errno == EINTR) continue;
            return errno ? errno : EIO;
        }
        if (r == 0) break;      // end of file
        done += (size_t)r;
    }
    if (done < (p.op == 1 ? p.need : p.bytes)) return EIO;
    if (p.bounce && p.op == 1) std::memcpy(p.mem, io, done);
    return 0;
}

// Moves a list of pieces with the pool's threads; blocks until all are done.
inline int run_pieces(TaskPool& pool, const std::vector<Piece>& pieces)
{
    PieceJob job{pieces.data(), &pool};
    return pool.run(pieces.size(), run_one_piece, &job);
}

// One parked thread that runs one function at a time: a stage of a pipeline whose other stages run
// on the caller's thread.  start() posts the job, wait() blocks until it has returned.
class StageThread {
public:
    StageThread() : th_([this] { loop(); }) {}
    ~StageThread()
    {
        {
            std::lock_guard<std::mutex> lk(mu_);
            stop_ = true;
        }
        cv_.notify_all();
        th_.join();
    }
    StageThread(const StageThread&) = delete;
    StageThread& operator=(const StageThread&) = delete;

    void start(void (*fn)(void*), void* ctx)
    {
        {
            std::lock_guard<std::mutex> lk(mu_);
            fn_ = fn;
            ctx_ = ctx;
            state_ = 1;
        }
        cv_.notify_all();
    }
    void wait()
    {
        std::unique_lock<std::mutex> lk(mu_);
        cv_.wait(lk, [this] { return state_ == 0; });
    }

private:
    void loop()
    {
        for (;;) {
            void (*fn)(void*);
            void* ctx;
            {
                std::unique_lock<std::mutex> lk(mu_);
                cv_.wait(lk, [this] { return stop_ || state_ == 1; });
                if (stop_) return;
                state_ = 2;
                fn = fn_;
                ctx = ctx_;
            }
            fn(ctx);
            {
                std::lock_guard<std::mutex> lk(mu_);
                state_ = 0;
            }
            cv_.notify_all();
        }
    }
    std::mutex mu_;
    std::condition_variable cv_;
    void (*fn_)(void*) = nullptr;
    void* ctx_ = nullptr;
    int state_ = 0;          // 0 idle, 1 job posted, 2 running
    bool stop_ = false;
    std::thread th_;         // last member: the thread starts after everything above exists
};

}  // namespace host
}  // namespace zi
