// Host-only file I/O of the third tier (no HIP in this header, so the thread choreography can be
// built and checked on a CPU, e.g. under ThreadSanitizer): a small thread pool, exact-length
// positional reads / writes, and the window chain -- batches of pages pass through the slots of a
// host-memory window: read from the files, processed in the window by the caller, written back,
// the last write of a slot starting the read of the batch that reuses it (Alg. 2's updating actor
// fetching the states and offloading them again, batch by batch).
#pragma once

#include <fcntl.h>
#include <unistd.h>

#include <cerrno>
#include <condition_variable>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <functional>
#include <mutex>
#include <thread>
#include <vector>

namespace apm {
namespace io {

constexpr size_t kIoPiece = (size_t)8 << 20;  // bytes per pread / pwrite task

class IoPool {
 public:
    explicit IoPool(int n) {
        try {
            for (int k = 0; k < n; ++k) thr_.emplace_back([this] { run(); });
        } catch (...) {  // a thread could not be started: end the ones that run, then report
            stop_and_join();
            throw;
        }
    }
    ~IoPool() { stop_and_join(); }
    IoPool(const IoPool&) = delete;
    IoPool& operator=(const IoPool&) = delete;
    void submit(std::function<void()> f) {
        {
            std::lock_guard<std::mutex> g(m_);
            q_.push_back(std::move(f));
        }
        cv_.notify_one();
    }

 private:
    void stop_and_join() {
        {
            std::lock_guard<std::mutex> g(m_);
            stop_ = true;
        }
        cv_.notify_all();
        for (auto& t : thr_) t.join();
        thr_.clear();
    }
    void run() {
        for (;;) {
            std::function<void()> f;
            {
                std::unique_lock<std::mutex> g(m_);
                cv_.wait(g, [this] { return stop_ || !q_.empty(); });
                if (q_.empty()) return;  // stop requested and nothing left
                f = std::move(q_.front());
                q_.pop_front();
            }
            f();
        }
    }
    std::vector<std::thread> thr_;
    std::deque<std::function<void()>> q_;
    std::mutex m_;
    std::condition_variable cv_;
    bool stop_ = false;
};

// Reads or writes exactly `len` bytes at `off`; 0 or an errno value.
inline int io_full(int fd, char* buf, size_t len, off_t off, bool write) {
    while (len > 0) {
        const ssize_t r = write ? pwrite(fd, buf, len, off) : pread(fd, buf, len, off);
        if (r < 0) {
            if (errno == EINTR) continue;
            return errno;
        }
        if (r == 0) return EIO;  // a short file: the pool's files are created at full size
        buf += r;
        off += r;
        len -= (size_t)r;
    }
    return 0;
}

// Unbuffered I/O cannot address GPU-pinned host memory directly (the kernel refuses to pin the
// driver's mapping: EFAULT), so with `direct` every piece passes through an ordinary page-aligned
// buffer of the calling thread.
inline int io_piece(int fd, char* buf, size_t len, off_t off, bool write, bool direct) {
    if (!direct) return io_full(fd, buf, len, off, write);
    struct Bounce {
        void* p = nullptr;
        ~Bounce() { free(p); }
    };
    static thread_local Bounce bounce;
    if (!bounce.p && posix_memalign(&bounce.p, 4096, kIoPiece) != 0) {
        bounce.p = nullptr;
        return ENOMEM;
    }
    char* b = static_cast<char*>(bounce.p);
    while (len > 0) {
        const size_t n = len < kIoPiece ? len : kIoPiece;
        if (write) std::memcpy(b, buf, n);
        const int err = io_full(fd, b, n, off, write);
        if (err) return err;
        if (!write) std::memcpy(buf, b, n);
        buf += n;
        off += (off_t)n;
        len -= n;
    }
    return 0;
}

// The window: n_slots slots of B pages for each of three classes (one file and one window region
// per class).  run() passes all pages [0, n_pages) through it once.
class WindowChain {
 public:
    // win[c]: host memory of n_slots * B * page_bytes bytes; fd[c]: the class's file.
    WindowChain(IoPool* pool, const int fd[3], char* const win[3], size_t page_bytes, int64_t B, int n_slots,
                bool direct)
        : pool_(pool), pb_(page_bytes), B_(B), n_slots_(n_slots), direct_(direct),
          loaded_((size_t)n_slots, -1), pending_((size_t)n_slots, 0) {
        for (int c = 0; c < 3; ++c) {
            fd_[c] = fd[c];
            win_[c] = win[c];
        }
    }

    // process(batch, slot, first_page, n_batch_pages) works on the slot's pages in the window and
    // returns true if they are to be written back.  After a failed read or write, or once process
    // has returned false, the remaining batches are neither processed nor written, but still pass
    // through the chain so that it drains.  Returns 0, an errno value of the first failed I/O, or
    // -1 if process returned false.  Everything queued has completed when this returns.
    int run(int64_t n_pages, const std::function<bool(int64_t, int, int64_t, int64_t)>& process) {
        return run_list(nullptr, n_pages, process);
    }

    // The same for the pages pages[0 .. n_pages) only (ascending page indices; nullptr = pages
    // [0, n_pages)): batch b holds list positions [b*B, b*B + nb), position b*B + j sitting in page
    // j of the slot; process gets the first list position of the batch.  Pages that are not listed
    // are neither read nor written.  `pages` must stay valid until the call returns.
    int run_list(const int64_t* pages, int64_t n_pages,
                 const std::function<bool(int64_t, int, int64_t, int64_t)>& process) {
        int64_t nbatches;
        {
            std::lock_guard<std::mutex> g(m_);
            list_ = pages;
            n_pages_ = n_pages;
            nbatches = n_batches_ = (n_pages + B_ - 1) / B_;
            batches_written_ = 0;
            io_errno_ = 0;
            for (auto& x : loaded_) x = -1;
            for (auto& x : pending_) x = 0;
        }
        for (int64_t b = 0; b < nbatches && b < n_slots_; ++b) queue(b, false);
        bool refused = false;
        for (int64_t b = 0; b < nbatches; ++b) {
            const int slot = (int)(b % n_slots_);
            bool failed;
            {
                std::unique_lock<std::mutex> g(m_);
                cv_.wait(g, [&] { return loaded_[(size_t)slot] == b; });
                failed = io_errno_ != 0;
            }
            const int64_t first = b * B_;
            const int64_t nb = n_pages - first < B_ ? n_pages - first : B_;
            if (!failed && !refused && !process(b, slot, first, nb)) refused = true;
            if (!failed && !refused) {
                queue(b, true);
            } else {
                // nothing valid to write: account for the batch and keep the chain going
                {
                    std::lock_guard<std::mutex> g(m_);
                    ++batches_written_;
                }
                if (b + n_slots_ < nbatches) queue(b + n_slots_, false);
            }
        }
        std::unique_lock<std::mutex> g(m_);
        cv_.wait(g, [&] { return batches_written_ == nbatches; });
        if (io_errno_) return io_errno_;
        return refused ? -1 : 0;
    }

    char* slot_base(int cls, int slot) const { return win_[cls] + (size_t)slot * (size_t)B_ * pb_; }

 private:
    // Queues the reads (write == false) or writes of batch b.  When the last piece of a write
    // completes, the reads of the batch that reuses the slot are queued.
    void queue(int64_t b, bool write) {
        const int slot = (int)(b % n_slots_);
        const int64_t first = b * B_;
        int64_t n_pages;
        const int64_t* list;
        {
            std::lock_guard<std::mutex> g(m_);
            n_pages = n_pages_;
            list = list_;
        }
        const int64_t nb = n_pages - first < B_ ? n_pages - first : B_;
        // pieces: runs of consecutive file pages, cut at kIoPiece bytes
        struct Piece { size_t win_off; off_t file_off; size_t len; };
        std::vector<Piece> pieces;
        for (int64_t j = 0; j < nb;) {
            const int64_t p0 = list ? list[first + j] : first + j;
            int64_t n = 1;
            while (j + n < nb && (list ? list[first + j + n] : first + j + n) == p0 + n) ++n;
            const size_t bytes = pb_ * (size_t)n;
            for (size_t o = 0; o < bytes; o += kIoPiece)
                pieces.push_back({(size_t)j * pb_ + o, (off_t)((size_t)p0 * pb_ + o), bytes - o < kIoPiece ? bytes - o : kIoPiece});
            j += n;
        }
        {
            std::lock_guard<std::mutex> g(m_);
            pending_[(size_t)slot] = 3 * (int)pieces.size();
            (write ? bytes_written_ : bytes_read_) += 3 * (int64_t)(pb_ * (size_t)nb);
        }
        for (int c = 0; c < 3; ++c) {
            for (const Piece& pc : pieces) {
                char* buf = slot_base(c, slot) + pc.win_off;
                const off_t off = pc.file_off;
                const size_t len = pc.len;
                const int fd = fd_[c];
                pool_->submit([this, b, slot, write, fd, buf, len, off] {
                    const int err = io_piece(fd, buf, len, off, write, direct_);
                    bool last = false, chain = false;
                    {
                        std::lock_guard<std::mutex> g(m_);
                        if (err && !io_errno_) io_errno_ = err;
                        last = --pending_[(size_t)slot] == 0;
                        chain = last && write && b + n_slots_ < n_batches_;
                    }
                    if (!last) return;
                    // The slot's next read is queued before the write is counted: run() must not
                    // see the last write as done while a thread is still inside this object.
                    if (chain) queue(b + n_slots_, false);
                    {
                        std::lock_guard<std::mutex> g(m_);
                        if (write) ++batches_written_;
                        else loaded_[(size_t)slot] = b;
                        cv_.notify_all();
                    }
                });
            }
        }
    }

 public:
    // Bytes queued for reading / writing since construction (all three classes).
    void io_bytes(int64_t* read, int64_t* written) {
        std::lock_guard<std::mutex> g(m_);
        if (read) *read = bytes_read_;
        if (written) *written = bytes_written_;
    }

 private:
    IoPool* pool_;
    int fd_[3];
    char* win_[3];
    const size_t pb_;
    const int64_t B_;
    const int n_slots_;
    const bool direct_;
    std::mutex m_;
    std::condition_variable cv_;
    std::vector<int64_t> loaded_;  // per slot: batch whose pages are in the window, -1 = none
    std::vector<int> pending_;     // per slot: outstanding pieces of the current read or write
    int64_t batches_written_ = 0;
    int io_errno_ = 0;
    int64_t n_batches_ = 0, n_pages_ = 0;
    const int64_t* list_ = nullptr;  // the listed pages of the running pass, nullptr = all
    int64_t bytes_read_ = 0, bytes_written_ = 0;
};

}  // namespace io
}  // namespace apm
