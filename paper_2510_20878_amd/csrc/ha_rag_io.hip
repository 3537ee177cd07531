// File transfers of the disk tier: whole-slot reads and writes for the offline calls, and the
// I/O threads that move pieces of chunks into bounce buffers for the online ones.
#include "ha_rag_internal.h"

#include <unistd.h>

#include <algorithm>
#include <cerrno>
#include <condition_variable>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <thread>

namespace ha_rag_host {

int io_error(ha_rag_ctx *c, const char *what)
{
    c->err = std::string(what) + ": " + std::strerror(errno);
    return HA_RAG_EIO;
}

int read_full(ha_rag_ctx *c, int fd, uint8_t *dst, size_t n, off_t off)
{
    while (n) {
        const ssize_t r = pread(fd, dst, n, off);
        if (r < 0) {
            if (errno == EINTR) continue;
            return io_error(c, "pread");
        }
        if (r == 0) {
            c->err = "pread: unexpected end of file";
            return HA_RAG_EIO;
        }
        dst += r;
        off += r;
        n -= (size_t)r;
    }
    return HA_RAG_OK;
}

int write_full(ha_rag_ctx *c, int fd, const uint8_t *src, size_t n, off_t off)
{
    while (n) {
        const ssize_t r = pwrite(fd, src, n, off);
        if (r < 0) {
            if (errno == EINTR) continue;
            return io_error(c, "pwrite");
        }
        src += r;
        off += r;
        n -= (size_t)r;
    }
    return HA_RAG_OK;
}

// ---- transfers into bounce buffers, in pieces, on the context's I/O threads ----------------
//
// A piece is up to kPiece bytes of one chunk: read from the file (through the thread's own
// page-aligned buffer if the file is open with O_DIRECT, which cannot target GPU-pinned memory)
// or copied from pageable memory into the bounce buffer, and from there into the host slot that
// Algorithm 2 placed a copy in, if any.  Pieces of one chunk and of different chunks, from one
// caller or several, run side by side: that is the queue depth the file sees.
namespace {
constexpr size_t kPiece = 4u << 20;

struct Piece {
    std::shared_ptr<Transfer> t;
    size_t lo = 0, n = 0;
};

int move_piece(Transfer &t, size_t lo, size_t n, uint8_t *dio, std::string *err)
{
    uint8_t *dst = t.dst + lo;
    if (t.fd < 0) {
        std::memcpy(dst, t.src + lo, n);
    } else {
        // direct reads are whole 4096-byte units (lo is a multiple of kPiece, which is one)
        const size_t want = t.direct ? (n + kDirectAlign - 1) / kDirectAlign * kDirectAlign : n;
        uint8_t *buf = t.direct ? dio : dst;
        size_t done = 0;
        while (done < want) {
            const ssize_t r = pread(t.fd, buf + done, want - done, t.off + (off_t)(lo + done));
            if (r < 0 && errno == EINTR) continue;
            if (r < 0) {
                *err = std::string("pread: ") + std::strerror(errno);
                return HA_RAG_EIO;
            }
            if (r == 0) {
                if (done >= n) break;  // the padding of the last unit lies past the end of the file
                *err = "pread: unexpected end of file";
                return HA_RAG_EIO;
            }
            done += (size_t)r;
        }
        if (t.direct) std::memcpy(dst, dio, n);
    }
    if (t.dst2) std::memcpy(t.dst2 + lo, dst, n);
    return HA_RAG_OK;
}
}  // namespace

int Transfer::wait()
{
    std::unique_lock<std::mutex> lk(mu);
    cv.wait(lk, [&] { return pieces_left == 0; });
    return rc;
}

class IoPool {
public:
    IoPool(uint32_t n, bool direct)
    {
        for (uint32_t i = 0; i < n; ++i) {
            uint8_t *buf = nullptr;
            if (direct) {
                void *p = nullptr;
                if (posix_memalign(&p, kDirectAlign, kPiece) == 0) buf = static_cast<uint8_t *>(p);
            }
            bufs_.push_back(buf);
        }
        for (uint32_t i = 0; i < n; ++i) threads_.emplace_back([this, i] { run(i); });
    }
    ~IoPool()
    {
        {
            std::lock_guard<std::mutex> g(mu_);
            stop_ = true;
        }
        cv_.notify_all();
        for (std::thread &t : threads_) t.join();
        for (uint8_t *b : bufs_) std::free(b);
    }
    void start(const std::shared_ptr<Transfer> &t)
    {
        const size_t n_pieces = t->bytes ? (t->bytes + kPiece - 1) / kPiece : 0;
        {
            std::lock_guard<std::mutex> g(t->mu);
            t->pieces_left = n_pieces;
        }
        if (n_pieces == 0) return;
        {
            std::lock_guard<std::mutex> g(mu_);
            for (size_t i = 0; i < n_pieces; ++i)
                q_.push_back(Piece{t, i * kPiece, std::min(kPiece, t->bytes - i * kPiece)});
        }
        cv_.notify_all();
    }

private:
    void run(uint32_t me)
    {
        for (;;) {
            Piece pc;
            {
                std::unique_lock<std::mutex> lk(mu_);
                cv_.wait(lk, [&] { return stop_ || !q_.empty(); });
                if (q_.empty()) return;  // stop_, and nothing left to move
                pc = q_.front();
                q_.pop_front();
            }
            std::string err;
            int rc = HA_RAG_OK;
            if (pc.t->direct && !bufs_[me]) {
                rc = HA_RAG_EIO;
                err = "no page-aligned buffer for direct I/O";
            } else {
                rc = move_piece(*pc.t, pc.lo, pc.n, bufs_[me], &err);
            }
            std::lock_guard<std::mutex> g(pc.t->mu);
            if (rc && !pc.t->rc) {
                pc.t->rc = rc;
                pc.t->err = err;
            }
            if (--pc.t->pieces_left == 0) pc.t->cv.notify_all();
        }
    }
    std::mutex mu_;
    std::condition_variable cv_;
    std::deque<Piece> q_;
    bool stop_ = false;
    std::vector<std::thread> threads_;
    std::vector<uint8_t *> bufs_;
};

IoPool *io_pool_create(uint32_t n_threads, bool direct) { return new IoPool(n_threads, direct); }
void io_pool_destroy(IoPool *p) { delete p; }
void io_pool_start(IoPool *p, const std::shared_ptr<Transfer> &t) { p->start(t); }

}  // namespace ha_rag_host
