// File transfers of the disk tier: plain and O_DIRECT reads and writes of whole slots.
#include "ha_rag_internal.h"

#include <unistd.h>

#include <cerrno>
#include <condition_variable>
#include <cstring>
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

// O_DIRECT read of `bytes` at `off` into `dst` (GPU-pinned memory, which direct I/O cannot
// target): a helper thread reads pieces into the two halves of the page-aligned buffer
// c->dio while this thread copies the previous piece to dst, so the file read and the
// host copy overlap.
int read_direct(ha_rag_ctx *c, int fd, uint8_t *dst, size_t bytes, off_t off)
{
    const size_t half = c->dio_bytes / 2 / kDirectAlign * kDirectAlign;
    const size_t total = c->io_bytes(bytes);
    if (half == 0 || total <= half) {  // small: one read, one copy
        int rc = read_full(c, fd, c->dio, total, off);
        if (rc) return rc;
        std::memcpy(dst, c->dio, bytes);
        return HA_RAG_OK;
    }
    const size_t piece = std::min<size_t>(half, 4u << 20);
    const size_t n_pieces = (total + piece - 1) / piece;
    std::mutex mu;
    std::condition_variable cv;
    size_t produced = 0, consumed = 0;  // pieces read / pieces copied out
    int rc_reader = HA_RAG_OK;
    std::string err_reader;
    std::thread reader([&] {
        for (size_t i = 0; i < n_pieces; ++i) {
            {
                std::unique_lock<std::mutex> lk(mu);
                cv.wait(lk, [&] { return i < consumed + 2; });  // a free half
            }
            const size_t n = std::min(piece, total - i * piece);
            uint8_t *buf = c->dio + (i & 1) * half;
            size_t done = 0;
            int rc = HA_RAG_OK;
            while (done < n) {
                const ssize_t r = pread(fd, buf + done, n - done, off + (off_t)(i * piece + done));
                if (r < 0 && errno == EINTR) continue;
                if (r <= 0) {
                    err_reader = r < 0 ? std::string("pread: ") + std::strerror(errno)
                                       : std::string("pread: unexpected end of file");
                    rc = HA_RAG_EIO;
                    break;
                }
                done += (size_t)r;
            }
            std::lock_guard<std::mutex> lk(mu);
            if (rc) rc_reader = rc;
            produced = i + 1;
            cv.notify_all();
            if (rc) return;
        }
    });
    int rc = HA_RAG_OK;
    for (size_t i = 0; i < n_pieces; ++i) {
        {
            std::unique_lock<std::mutex> lk(mu);
            cv.wait(lk, [&] { return produced > i || rc_reader; });
            if (rc_reader) {
                rc = rc_reader;
                break;
            }
        }
        const size_t lo = i * piece;
        if (lo < bytes) std::memcpy(dst + lo, c->dio + (i & 1) * half, std::min(piece, bytes - lo));
        std::lock_guard<std::mutex> lk(mu);
        consumed = i + 1;
        cv.notify_all();
    }
    {
        std::lock_guard<std::mutex> lk(mu);
        consumed = n_pieces + 2;  // lets a reader that is still waiting run to its end
        cv.notify_all();
    }
    reader.join();
    if (rc) c->err = err_reader;
    return rc;
}

}  // namespace ha_rag_host
