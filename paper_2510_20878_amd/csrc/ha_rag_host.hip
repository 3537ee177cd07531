// Host runtime behind include/ha_rag.h: pool slabs in four tiers (GPU memory, pinned
// host memory, pageable host memory, files), hotness counters and ranks (Algorithm 1
// steps 1-2), the tier lookup / placement / LRU of Algorithm 2, and the stream/event
// pipeline that overlaps file reads, host copies and host -> HBM copies with the
// dequantize kernel.
#include <hip/hip_runtime.h>

#include <fcntl.h>
#include <sys/stat.h>
#include <unistd.h>

#include <algorithm>
#include <cerrno>
#include <condition_variable>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <list>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <unordered_map>
#include <vector>

#include "../../include/ha_rag.h"
#include "ha_rag_kernels.h"

using namespace ha_rag;

namespace {

constexpr uint64_t kPPM = 1000000ull;
constexpr uint32_t kNoRank = UINT32_MAX;
constexpr uint32_t kTiers = 4;        // HBM, pinned, pageable, disk
constexpr uint32_t kCacheTiers = 3;   // tiers with a capacity and an LRU order
constexpr size_t kDirectAlign = 4096; // offset / size / buffer alignment of O_DIRECT I/O
thread_local std::string g_create_err;  // why the last ha_rag_create on this thread failed

bool valid_group(uint32_t g)
{
    return g == 32 || g == 64 || g == 128 || g == 256 || g == 512;
}

uint32_t bits_of(uint32_t prec)  // storage bits per element
{
    return prec == HA_RAG_PREC_16 ? 16u : prec == HA_RAG_PREC_INT4 ? 4u : 8u;
}

bool has_meta(uint32_t prec) { return prec == HA_RAG_PREC_INT8 || prec == HA_RAG_PREC_INT4; }

uint32_t log2u(uint32_t v)
{
    uint32_t s = 0;
    while ((1u << s) < v) ++s;
    return s;
}

int chunk_bytes_impl(uint32_t L, uint32_t H, uint32_t D, uint32_t prec, uint32_t group,
                     uint32_t T, size_t *payload, size_t *meta, size_t *total,
                     uint32_t part = kPartKV)
{
    if (prec >= HA_RAG_N_PREC || L == 0 || H == 0 || D == 0 || (D % 8u)) return HA_RAG_EFORMAT;
    if (has_meta(prec) && (!valid_group(group) || (D % group))) return HA_RAG_EFORMAT;
    const uint64_t n_e = (uint64_t)T * D;
    if (n_e > 0x7FFFFFFFull) return HA_RAG_EINVAL;
    const uint64_t nblk = (n_e + kBlockElems - 1) / kBlockElems;
    if (part > kPartV) return HA_RAG_EINVAL;
    const uint64_t tiles = (part == kPartKV ? 2ull : 1ull) * L * H;
    const uint64_t pay = tiles * nblk * 256ull * bits_of(prec);
    const uint64_t met = has_meta(prec)               ? tiles * nblk * (kBlockElems / group) * 4ull
                         : prec == HA_RAG_PREC_GSE8 ? (nblk ? tiles * 16ull : 0)
                                                    : 0;
    if (payload) *payload = (size_t)pay;
    if (meta) *meta = (size_t)met;
    if (total) *total = (size_t)(pay + met);
    return HA_RAG_OK;
}

struct Chunk {
    uint64_t id = 0;
    uint32_t prec = 0, n_tokens = 0;
    uint32_t part = kPartKV;  // keys and values, or one of the two
    uint64_t bytes = 0;
    int32_t slot[kTiers] = {-1, -1, -1, -1};
    uint64_t count = 0;
    uint32_t rank = kNoRank;
    uint64_t last_use[kCacheTiers] = {0, 0, 0};  // sequence number of the last access per tier
    uint64_t made_by[kCacheTiers] = {0, 0, 0};   // load call that created this tier's copy (0: none)
    std::list<uint32_t>::iterator lru_it[kCacheTiers];

    int fastest() const
    {
        for (uint32_t t = 0; t < kTiers; ++t)
            if (slot[t] >= 0) return (int)t;
        return -1;
    }
    bool has_slower_copy(uint32_t tier) const
    {
        for (uint32_t t = tier + 1; t < kTiers; ++t)
            if (slot[t] >= 0) return true;
        return false;
    }
};

// Who touched a slot last.  HBM slots: the streams that wrote / read it, so that a
// different stream can be made to wait.  Pinned slots: the stream that wrote it (a
// device -> host copy) and the events of host -> device copies that read it, which the
// host waits for before it overwrites the slot.
struct SlotUse {
    hipStream_t writer = nullptr;
    bool has_writer = false;
    std::vector<hipStream_t> readers;
    std::vector<hipEvent_t> read_events;
};

struct Slab {
    uint8_t *base = nullptr;  // memory tiers
    int fd = -1;              // disk tier
    size_t slot_bytes = 0;
    uint32_t n_slots = 0;
    bool reg = false;
    std::vector<uint32_t> free_slots;  // stack
    std::vector<SlotUse> use;
    std::list<uint32_t> lru;           // chunk indices resident here, least recent first
    bool registered() const { return reg; }
    uint8_t *ptr(int32_t s) const { return base + (size_t)s * slot_bytes; }
    off_t offset(int32_t s) const { return (off_t)((size_t)s * slot_bytes); }
};

struct StagingSlot {
    hipEvent_t filled = nullptr, consumed = nullptr;
    bool consumed_valid = false;
};

struct BounceSlot {
    hipEvent_t h2d_done = nullptr;
    bool busy = false;
};

}  // namespace

struct ha_rag_ctx {
    ha_rag_config cfg{};
    uint32_t n_tiles = 0;
    std::mutex mu;
    std::string err;  // last failing HIP or I/O call

    std::vector<Chunk> chunks;
    std::unordered_map<uint64_t, uint32_t> index;
    Slab slab[kTiers][HA_RAG_N_PREC];

    uint32_t bound[3] = {0, 0, 0};  // ranks below bound[t] belong to the list of tier <= t
    uint64_t n_loads = 0, use_seq = 0, call_seq = 0;

    uint8_t *staging = nullptr;
    size_t staging_slot_bytes = 0;
    std::vector<StagingSlot> stg;
    uint64_t stg_next = 0;

    uint8_t *bounce = nullptr;  // pinned buffers that pageable / disk chunks pass through
    size_t bounce_slot_bytes = 0;
    uint8_t *dio = nullptr;     // page-aligned ordinary memory for O_DIRECT transfers: the
                                // kernel cannot do direct I/O on GPU-pinned host memory
    size_t dio_bytes = 0;
    std::vector<BounceSlot> bnc;
    uint64_t bnc_next = 0;

    std::vector<hipStream_t> copy_streams;
    uint64_t copy_rr = 0;
    std::unordered_map<hipStream_t, hipEvent_t> stream_done;

    K1Launch launch{64, 1, 2, true, true};

    uint32_t group_of(uint32_t prec) const
    {
        return prec == HA_RAG_PREC_INT8 ? cfg.group_int8 : prec == HA_RAG_PREC_INT4 ? cfg.group_int4 : 0;
    }
    bool dry() const { return cfg.dry_run != 0; }
    bool direct() const { return cfg.disk_o_direct != 0; }
    size_t io_bytes(uint64_t bytes) const  // what a file transfer of `bytes` moves
    {
        return direct() ? (size_t)((bytes + kDirectAlign - 1) / kDirectAlign * kDirectAlign) : (size_t)bytes;
    }
    // Algorithm 2 step 1: which list a rank belongs to
    uint32_t list_of(uint32_t rank) const
    {
        return rank < bound[0] ? HA_RAG_TIER_HBM
               : rank < bound[1] ? HA_RAG_TIER_PINNED
               : rank < bound[2] ? HA_RAG_TIER_PAGEABLE
                                 : HA_RAG_TIER_DISK;
    }
};

namespace {

#define HIPCHK(ctx, call)                                                      \
    do {                                                                       \
        hipError_t e_ = (call);                                                \
        if (e_ != hipSuccess) {                                                \
            (ctx)->err = std::string(#call) + ": " + hipGetErrorString(e_);    \
            return HA_RAG_EHIP;                                                \
        }                                                                      \
    } while (0)

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

int stream_event(ha_rag_ctx *c, hipStream_t s, hipEvent_t *out)
{
    auto it = c->stream_done.find(s);
    if (it == c->stream_done.end()) {
        hipEvent_t ev;
        HIPCHK(c, hipEventCreateWithFlags(&ev, hipEventDisableTiming));
        it = c->stream_done.emplace(s, ev).first;
    }
    *out = it->second;
    return HA_RAG_OK;
}

// Marks the end of a call's work on stream s, for later cross-stream waits.
int mark_stream(ha_rag_ctx *c, hipStream_t s)
{
    if (c->dry()) return HA_RAG_OK;
    hipEvent_t ev;
    int rc = stream_event(c, s, &ev);
    if (rc) return rc;
    HIPCHK(c, hipEventRecord(ev, s));
    return HA_RAG_OK;
}

int wait_for(ha_rag_ctx *c, hipStream_t s, hipStream_t other)
{
    if (c->dry() || other == s) return HA_RAG_OK;
    auto it = c->stream_done.find(other);
    if (it == c->stream_done.end()) return HA_RAG_OK;  // nothing was ever enqueued there
    HIPCHK(c, hipStreamWaitEvent(s, it->second, 0));
    return HA_RAG_OK;
}

int before_read(ha_rag_ctx *c, SlotUse &u, hipStream_t s)
{
    if (u.has_writer) {
        int rc = wait_for(c, s, u.writer);
        if (rc) return rc;
    }
    if (std::find(u.readers.begin(), u.readers.end(), s) == u.readers.end()) u.readers.push_back(s);
    return HA_RAG_OK;
}

int before_write(ha_rag_ctx *c, SlotUse &u, hipStream_t s)
{
    if (u.has_writer) {
        int rc = wait_for(c, s, u.writer);
        if (rc) return rc;
    }
    for (hipStream_t r : u.readers) {
        int rc = wait_for(c, s, r);
        if (rc) return rc;
    }
    u.readers.clear();
    u.writer = s;
    u.has_writer = true;
    return HA_RAG_OK;
}

// The host is about to overwrite a host-memory slot: wait until every device copy that
// reads or writes it has finished.
int before_host_write(ha_rag_ctx *c, SlotUse &u)
{
    if (!c->dry()) {
        for (hipEvent_t ev : u.read_events) HIPCHK(c, hipEventSynchronize(ev));
        if (u.has_writer) {
            auto it = c->stream_done.find(u.writer);
            if (it != c->stream_done.end()) HIPCHK(c, hipEventSynchronize(it->second));
        }
        for (hipStream_t r : u.readers) {
            auto it = c->stream_done.find(r);
            if (it != c->stream_done.end()) HIPCHK(c, hipEventSynchronize(it->second));
        }
    }
    u.read_events.clear();
    u.readers.clear();
    u.has_writer = false;
    return HA_RAG_OK;
}

Chunk *find_chunk(ha_rag_ctx *c, uint64_t id, uint32_t *idx = nullptr)
{
    auto it = c->index.find(id);
    if (it == c->index.end()) return nullptr;
    if (idx) *idx = it->second;
    return &c->chunks[it->second];
}

void tier_touch(ha_rag_ctx *c, uint32_t tier, uint32_t ci)  // queueX.get(C_i)
{
    if (tier >= kCacheTiers) return;
    Chunk &ch = c->chunks[ci];
    Slab &sl = c->slab[tier][ch.prec];
    sl.lru.splice(sl.lru.end(), sl.lru, ch.lru_it[tier]);  // most recent at the back
    ch.last_use[tier] = ++c->use_seq;
}

void tier_attach(ha_rag_ctx *c, uint32_t tier, uint32_t ci, int32_t slot)
{
    Chunk &ch = c->chunks[ci];
    ch.slot[tier] = slot;
    if (tier >= kCacheTiers) return;
    Slab &sl = c->slab[tier][ch.prec];
    ch.lru_it[tier] = sl.lru.insert(sl.lru.end(), ci);
    ch.last_use[tier] = ++c->use_seq;
}

void tier_detach(ha_rag_ctx *c, uint32_t tier, uint32_t ci)
{
    Chunk &ch = c->chunks[ci];
    Slab &sl = c->slab[tier][ch.prec];
    if (tier < kCacheTiers) sl.lru.erase(ch.lru_it[tier]);
    sl.free_slots.push_back((uint32_t)ch.slot[tier]);
    ch.slot[tier] = -1;
}

// A free slot of the slab (tier, prec); if the slab is full the least recently used chunk
// that also lives in a slower tier is dropped ("put C_i in queueX with LRU").  Returns -1 if
// nothing can be freed.  *evicted receives the dropped id.  Copies created by load call
// `keep_call` (non-zero) are passed over: a copy that the running call has itself just
// created is not dropped again by the same call, because a later read of it may already
// be planned.
int32_t tier_acquire(ha_rag_ctx *c, uint32_t tier, uint32_t prec, uint64_t *evicted,
                     uint64_t keep_call = 0)
{
    Slab &sl = c->slab[tier][prec];
    *evicted = HA_RAG_NO_CHUNK;
    if (!sl.registered()) return -1;
    if (sl.free_slots.empty() && tier < kCacheTiers) {
        for (uint32_t ci : sl.lru) {
            if (keep_call && c->chunks[ci].made_by[tier] == keep_call) continue;
            if (c->chunks[ci].has_slower_copy(tier)) {
                *evicted = c->chunks[ci].id;
                tier_detach(c, tier, ci);
                break;
            }
        }
    }
    if (sl.free_slots.empty()) return -1;
    const int32_t s = (int32_t)sl.free_slots.back();
    sl.free_slots.pop_back();
    return s;
}

void rerank_locked(ha_rag_ctx *c)
{
    const size_t n = c->chunks.size();
    std::vector<uint32_t> order(n);
    for (size_t i = 0; i < n; ++i) order[i] = (uint32_t)i;
    std::sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) {
        const Chunk &x = c->chunks[a], &y = c->chunks[b];
        if (x.count != y.count) return x.count > y.count;
        return x.id < y.id;
    });
    for (size_t r = 0; r < n; ++r) c->chunks[order[r]].rank = (uint32_t)r;
    // idx_1 = tau_GPU * N, idx_2 = tau_PIN * N + idx_1, idx_3 = tau_PAGE * N + idx_2
    const uint32_t tau[3] = {c->cfg.tau_gpu_ppm, c->cfg.tau_pin_ppm, c->cfg.tau_page_ppm};
    uint64_t acc = 0;
    for (int t = 0; t < 3; ++t) {
        acc = std::min<uint64_t>(n, acc + ((uint64_t)tau[t] * n) / kPPM);
        c->bound[t] = (uint32_t)acc;
    }
}

// Token rows of the key plane and of the value plane of one request's cache, as its chunks
// fill them in list order.  A whole chunk needs both planes at the same length.
struct PlaneCursor {
    uint64_t off[2];
    explicit PlaneCursor(uint64_t base) : off{base, base} {}
    bool place(uint32_t part, uint64_t n_tokens, uint64_t *at)
    {
        if (part == kPartKV) {
            if (off[0] != off[1]) return false;
            *at = off[0];
            off[0] += n_tokens;
            off[1] += n_tokens;
        } else {
            *at = off[part - kPartK];
            off[part - kPartK] += n_tokens;
        }
        return true;
    }
    bool closed() const { return off[0] == off[1]; }
    uint64_t end() const { return std::max(off[0], off[1]); }
};

struct Request {
    uint32_t begin, end;
    uint8_t *out;
    uint64_t cap, base;
    const ha_rag_paged_cache *paged = nullptr;  // set: `out` is unused, cap = table entries * P
};

// Checks a paged-cache description and returns the token rows its table covers.
int check_paged(const ha_rag_ctx *c, const ha_rag_paged_cache *pg, uint64_t *cap_tokens)
{
    if (!pg || !pg->base || !pg->page_table || pg->page_tokens == 0 || pg->n_pages == 0) return HA_RAG_EINVAL;
    if (((uintptr_t)pg->base & 15u) || ((uintptr_t)pg->page_table & 3u) || ((uintptr_t)pg->bad_pages & 3u))
        return HA_RAG_EINVAL;
    if ((pg->page_stride & 15u) || (pg->tile_stride & 15u)) return HA_RAG_EINVAL;
    const uint64_t page_bytes = (uint64_t)pg->page_tokens * c->cfg.head_dim * 2ull;
    if (page_bytes < 1024u) return HA_RAG_EINVAL;  // a wave's KiB may cross one page boundary only
    if ((uint64_t)pg->n_table * page_bytes > 0xFFFFFFFFull) return HA_RAG_EINVAL;
    *cap_tokens = (uint64_t)pg->n_table * pg->page_tokens;
    return HA_RAG_OK;
}

// What pass A decided for one chunk of a load.
struct Action {
    uint32_t ci;
    uint32_t req;
    uint64_t tok_off;
    enum Kind { HOT_EARLY, HOT_LATE, COLD } kind;
    uint8_t src_tier;      // tier the bytes come from
    int32_t src_slot;      // slot in that tier, as of the moment the action was decided (a
                           // later chunk of the same call may evict this copy)
    uint8_t place_tier;    // tier a new copy is placed into, or HA_RAG_TIER_NONE
    int32_t place_slot;
};

K1Chunk make_desc(const ha_rag_ctx *c, const Chunk &ch, const uint8_t *src, const Request &rq,
                  uint64_t tok_off, bool src_in_host_memory = false)
{
    K1Chunk d;
    const uint64_t D = c->cfg.head_dim;
    d.src = src;
    if (rq.paged) {  // the row's byte offset in the request's virtual tile rides in the pointer
        d.out = reinterpret_cast<uint8_t *>((uintptr_t)(tok_off * D * 2ull));
        d.out_tile_stride = 0;
    } else {
        d.out = rq.out + tok_off * D * 2ull;
        d.out_tile_stride = rq.cap * D * 2ull;
    }
    d.n_tokens = ch.n_tokens;
    const uint32_t g = c->group_of(ch.prec);
    d.fmt = ch.prec | ((g ? log2u(g) : 0u) << 8) | (ch.part << 16);
    if (src_in_host_memory) d.fmt |= kWholeBlockItems;
    return d;
}

struct Batch {
    K1Params p;
};

int flush(ha_rag_ctx *c, Batch &b, hipStream_t s, uint32_t *launches)
{
    if (b.p.n_chunks == 0) return HA_RAG_OK;
    if (!c->dry()) HIPCHK(c, launch_k1(b.p, c->launch, s));
    if (launches) ++*launches;
    b.p.n_chunks = 0;
    return HA_RAG_OK;
}

int push(ha_rag_ctx *c, Batch &b, const K1Chunk &d, hipStream_t s, uint32_t *launches)
{
    b.p.c[b.p.n_chunks++] = d;
    if (b.p.n_chunks == kMaxLaunchChunks) return flush(c, b, s, launches);
    return HA_RAG_OK;
}

void init_batch(const ha_rag_ctx *c, Batch &b, const ha_rag_paged_cache *pg = nullptr)
{
    b.p.n_layers = c->cfg.n_layers;
    b.p.n_kv_heads = c->cfg.n_kv_heads;
    b.p.head_dim = c->cfg.head_dim;
    b.p.n_chunks = 0;
    b.p.total_items = 0;
    std::memset(&b.p.paged, 0, sizeof b.p.paged);
    if (pg) {
        K1Paged &k = b.p.paged;
        k.enabled = 1;
        k.base = static_cast<uint8_t *>(pg->base);
        k.page_table = pg->page_table;
        k.bad_pages = pg->bad_pages;
        k.page_stride = pg->page_stride;
        k.tile_stride = pg->tile_stride;
        k.page_bytes = pg->page_tokens * c->cfg.head_dim * 2u;
        k.n_table = pg->n_table;
        k.n_pages = pg->n_pages;
    }
}

// Next bounce buffer, once the host -> device copy that last read it has finished.
int acquire_bounce(ha_rag_ctx *c, size_t *idx)
{
    const size_t b = (size_t)(c->bnc_next++ % c->bnc.size());
    if (!c->dry() && c->bnc[b].busy) {
        HIPCHK(c, hipEventSynchronize(c->bnc[b].h2d_done));
        c->bnc[b].busy = false;
    }
    *idx = b;
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

// Packed bytes of a chunk from its pageable or disk copy into a bounce buffer (host work,
// synchronous).
int fill_bounce(ha_rag_ctx *c, const Chunk &ch, uint32_t tier, int32_t slot, uint8_t *dst)
{
    if (c->dry()) return HA_RAG_OK;
    const Slab &sl = c->slab[tier][ch.prec];
    if (tier == HA_RAG_TIER_PAGEABLE) {
        std::memcpy(dst, sl.ptr(slot), ch.bytes);
        return HA_RAG_OK;
    }
    if (!c->direct()) return read_full(c, sl.fd, dst, ch.bytes, sl.offset(slot));
    return read_direct(c, sl.fd, dst, ch.bytes, sl.offset(slot));
}

int load_impl(ha_rag_ctx *c, const uint64_t *ids, const uint8_t *tags, const Request *reqs,
              uint32_t n_req, uint32_t n, hipStream_t s, ha_rag_load_stats *stats,
              ha_rag_chunk_trace *trace)
{
    const uint64_t D = c->cfg.head_dim;
    // ---- checks: nothing changes before all of them pass --------------------
    std::vector<uint32_t> cis(n);
    for (uint32_t r = 0; r < n_req; ++r) {
        const Request &rq = reqs[r];
        if (rq.end < rq.begin || rq.end > n) return HA_RAG_EINVAL;
        if (rq.end > rq.begin && !rq.paged && (rq.out == nullptr || ((uintptr_t)rq.out & 15u)))
            return HA_RAG_EINVAL;
        PlaneCursor cur(0);
        for (uint32_t i = rq.begin; i < rq.end; ++i) {
            Chunk *ch = find_chunk(c, ids[i], &cis[i]);
            if (!ch) return HA_RAG_ENOENT;
            if (tags && tags[i] != ch->prec) return HA_RAG_EFORMAT;
            const int f = ch->fastest();
            if (f < 0) return HA_RAG_ENOENT;
            // staging is needed by every DMA route: always from pageable memory and files,
            // from pinned memory if pinned_dma is set or a promotion into HBM is possible
            const bool via_staging =
                f >= (int)HA_RAG_TIER_PAGEABLE ||
                (f == (int)HA_RAG_TIER_PINNED &&
                 (c->cfg.pinned_dma || c->slab[HA_RAG_TIER_HBM][ch->prec].registered()));
            if (via_staging && (c->stg.size() < 2 || ch->bytes > c->staging_slot_bytes))
                return HA_RAG_ENOSPC;
            if (f >= (int)HA_RAG_TIER_PAGEABLE &&
                (c->bnc.size() < 2 || c->io_bytes(ch->bytes) > c->bounce_slot_bytes))
                return HA_RAG_ENOSPC;
            uint64_t at;
            if (!cur.place(ch->part, ch->n_tokens, &at)) return HA_RAG_EINVAL;
        }
        if (!cur.closed()) return HA_RAG_EINVAL;  // keys without their values, or the reverse
        if (rq.base > rq.cap || cur.end() > rq.cap - rq.base) return HA_RAG_ENOSPC;
    }

    if (c->cfg.rerank_interval && c->n_loads && (c->n_loads % c->cfg.rerank_interval) == 0)
        rerank_locked(c);
    ++c->n_loads;

    ha_rag_load_stats st;
    std::memset(&st, 0, sizeof st);
    st.n_chunks = n;

    // ---- pass A: Algorithm 2 step 2, chunk by chunk, in request order ---------
    std::vector<Action> acts;
    acts.reserve(n);
    // copies created by this call carry its number: they are not evicted again by this call
    const uint64_t call = ++c->call_seq;
    for (uint32_t r = 0; r < n_req; ++r) {
        const Request &rq = reqs[r];
        PlaneCursor cur(rq.base);
        for (uint32_t i = rq.begin; i < rq.end; ++i) {
            const uint32_t ci = cis[i];
            Chunk &ch = c->chunks[ci];
            ch.count += 1;
            uint64_t off = 0;
            (void)cur.place(ch.part, ch.n_tokens, &off);  // checked above
            const uint32_t found = (uint32_t)ch.fastest();
            Action a{ci, r, off, Action::COLD, (uint8_t)found, ch.slot[found], HA_RAG_TIER_NONE, -1};
            ha_rag_chunk_trace tr;
            std::memset(&tr, 0, sizeof tr);
            tr.tok_off = off;
            tr.evicted_id = HA_RAG_NO_CHUNK;
            tr.found_tier = (uint8_t)found;
            tr.placed_tier = HA_RAG_TIER_NONE;
            tier_touch(c, found, ci);
            switch (found) {
            case HA_RAG_TIER_HBM:
                a.kind = ch.made_by[HA_RAG_TIER_HBM] == call ? Action::HOT_LATE : Action::HOT_EARLY;
                ++st.n_hbm_hits;
                break;
            case HA_RAG_TIER_PINNED: ++st.n_pinned_hits; break;
            case HA_RAG_TIER_PAGEABLE:
                ++st.n_pageable_hits;
                st.bytes_host_copied += ch.bytes;
                break;
            default:
                ++st.n_disk_hits;
                st.bytes_disk_read += ch.bytes;
                break;
            }
            if (found != HA_RAG_TIER_HBM) {
                st.bytes_h2d += ch.bytes;
                // the list the chunk's rank belongs to says where a copy should be kept;
                // only a tier faster than the one it was found in gets one
                const uint32_t want = ch.rank == kNoRank ? HA_RAG_TIER_DISK : c->list_of(ch.rank);
                if (want < found && c->slab[want][ch.prec].registered()) {
                    uint64_t ev;
                    const int32_t slot = tier_acquire(c, want, ch.prec, &ev, call);
                    if (slot >= 0) {
                        tier_attach(c, want, ci, slot);
                        ch.made_by[want] = call;
                        a.place_tier = (uint8_t)want;
                        a.place_slot = slot;
                        tr.placed_tier = (uint8_t)want;
                        tr.evicted_id = ev;
                        if (ev != HA_RAG_NO_CHUNK) ++st.n_evicted;
                        if (want == HA_RAG_TIER_HBM) {
                            tr.promoted = 1;
                            ++st.n_promoted;
                            st.bytes_d2d += ch.bytes;
                        } else {
                            ++st.n_placed_host;
                            st.bytes_host_copied += ch.bytes;
                        }
                    } else {
                        tr.promote_skipped = 1;
                        ++st.n_promote_skipped;
                    }
                }
            }
            // Pinned copy that stays where it is: unless pinned_dma is set the kernel reads it
            // over the link itself (no staging, no copy stream).  A pinned copy written by this very
            // call is read after the transfers, which is when its bytes are in place.
            if (found == HA_RAG_TIER_PINNED && !c->cfg.pinned_dma && a.place_tier == HA_RAG_TIER_NONE)
                a.kind = ch.made_by[HA_RAG_TIER_PINNED] == call ? Action::HOT_LATE : Action::HOT_EARLY;
            if (ch.part != kPartV) st.tokens += ch.n_tokens;  // rows of the key plane
            st.packed_bytes_read += ch.bytes;
            st.bf16_bytes_written +=
                (uint64_t)ch.n_tokens * (ch.part == kPartKV ? c->n_tiles : c->n_tiles / 2) * D * 2ull;
            acts.push_back(a);
            if (trace) trace[i] = tr;
        }
    }

    // ---- pass B: enqueue ---------------------------------------------------------
    // 1. one kernel over every chunk that is read where it lies: copies already resident in
    //    HBM, and pinned copies when the kernel reads pinned memory itself
    // 2. transfers of the first cold chunks (as many as there are staging slots)
    // 3. per cold chunk: wait for its transfer, kernel, copy into the HBM slab if it was
    //    placed there, release the staging slot, start the transfer that reuses it
    // 4. one kernel over chunks whose copy was written in step 2 or 3
    // A transfer is a host -> HBM copy from the pinned slot, or, for pageable and disk
    // chunks, a host copy / file read into a pinned bounce buffer (synchronous, on this
    // thread; also the moment a pinned / pageable copy is written) followed by that copy.
    std::vector<uint32_t> cold;
    for (uint32_t k = 0; k < acts.size(); ++k)
        if (acts[k].kind == Action::COLD) cold.push_back(k);
    const size_t n_stg = c->stg.size();
    std::vector<size_t> cold_slot(cold.size());

    // If a HIP or file call fails midway, copies that pass A booked but that were never
    // written must not stay in the books.
    struct Undo {
        ha_rag_ctx *c;
        std::vector<Action> &acts;
        std::vector<uint8_t> written;  // per action: its placed copy has been written / enqueued
        bool ok = false;
        ~Undo()
        {
            if (ok) return;
            for (size_t k = 0; k < acts.size(); ++k) {
                const Action &a = acts[k];
                if (a.place_tier == HA_RAG_TIER_NONE || written[k]) continue;
                if (c->chunks[a.ci].slot[a.place_tier] == a.place_slot) tier_detach(c, a.place_tier, a.ci);
            }
        }
    } undo{c, acts, std::vector<uint8_t>(acts.size(), 0)};

    auto start_transfer = [&](size_t k) -> int {
        const Action &a = acts[cold[k]];
        const Chunk &ch = c->chunks[a.ci];
        const size_t sidx = (size_t)(c->stg_next++ % n_stg);
        cold_slot[k] = sidx;
        const uint8_t *src = nullptr;
        size_t bidx = 0;
        if (a.src_tier == HA_RAG_TIER_PINNED) {
            src = c->slab[HA_RAG_TIER_PINNED][ch.prec].ptr(a.src_slot);
        } else {
            int rc = acquire_bounce(c, &bidx);
            if (rc) return rc;
            uint8_t *bp = c->bounce + bidx * c->bounce_slot_bytes;
            rc = fill_bounce(c, ch, a.src_tier, a.src_slot, bp);
            if (rc) return rc;
            if (a.place_tier == HA_RAG_TIER_PINNED || a.place_tier == HA_RAG_TIER_PAGEABLE) {
                Slab &ds = c->slab[a.place_tier][ch.prec];
                rc = before_host_write(c, ds.use[a.place_slot]);
                if (rc) return rc;
                if (!c->dry()) std::memcpy(ds.ptr(a.place_slot), bp, ch.bytes);
                undo.written[cold[k]] = 1;
            }
            src = bp;
        }
        if (c->dry()) return HA_RAG_OK;
        StagingSlot &ss = c->stg[sidx];
        hipStream_t cs = c->copy_streams[c->copy_rr++ % c->copy_streams.size()];
        if (ss.consumed_valid) HIPCHK(c, hipStreamWaitEvent(cs, ss.consumed, 0));
        if (a.src_tier == HA_RAG_TIER_PINNED) {
            SlotUse &u = c->slab[HA_RAG_TIER_PINNED][ch.prec].use[a.src_slot];
            if (u.has_writer) {  // a device -> host copy may still be filling the slot
                int rc = wait_for(c, cs, u.writer);
                if (rc) return rc;
            }
            if (std::find(u.read_events.begin(), u.read_events.end(), ss.filled) == u.read_events.end())
                u.read_events.push_back(ss.filled);  // at most one per staging slot
        }
        HIPCHK(c, hipMemcpyAsync(c->staging + sidx * c->staging_slot_bytes, src, ch.bytes,
                                 hipMemcpyHostToDevice, cs));
        HIPCHK(c, hipEventRecord(ss.filled, cs));
        if (a.src_tier != HA_RAG_TIER_PINNED) {
            HIPCHK(c, hipEventRecord(c->bnc[bidx].h2d_done, cs));
            c->bnc[bidx].busy = true;
        }
        return HA_RAG_OK;
    };

    // Chunks read where they lie (HBM copies, and pinned copies unless pinned_dma is set) go
    // first: their slots may be handed to other chunks by the transfers below.
    Batch batch;
    init_batch(c, batch, n_req == 1 ? reqs[0].paged : nullptr);
    bool reads_pinned = false;
    for (const Action &a : acts) {
        if (a.kind != Action::HOT_EARLY) continue;
        const Chunk &ch = c->chunks[a.ci];
        Slab &hs = c->slab[a.src_tier][ch.prec];
        int rc = before_read(c, hs.use[a.src_slot], s);
        if (rc) return rc;
        reads_pinned |= a.src_tier == HA_RAG_TIER_PINNED;
        rc = push(c, batch,
                  make_desc(c, ch, hs.ptr(a.src_slot), reqs[a.req], a.tok_off,
                            a.src_tier == HA_RAG_TIER_PINNED),
                  s, &st.n_kernel_launches);
        if (rc) return rc;
    }
    int rc = flush(c, batch, s, &st.n_kernel_launches);
    if (rc) return rc;
    if (reads_pinned) {  // a host write into one of those pinned slots waits for this point
        rc = mark_stream(c, s);
        if (rc) return rc;
    }

    size_t started = 0;
    for (; started < cold.size() && started < n_stg; ++started) {
        rc = start_transfer(started);
        if (rc) return rc;
    }

    for (size_t k = 0; k < cold.size(); ++k) {
        const Action &a = acts[cold[k]];
        const Chunk &ch = c->chunks[a.ci];
        const size_t sidx = cold_slot[k];
        uint8_t *sp = c->staging + sidx * c->staging_slot_bytes;
        if (!c->dry()) HIPCHK(c, hipStreamWaitEvent(s, c->stg[sidx].filled, 0));
        rc = push(c, batch, make_desc(c, ch, sp, reqs[a.req], a.tok_off), s, &st.n_kernel_launches);
        if (rc) return rc;
        rc = flush(c, batch, s, &st.n_kernel_launches);
        if (rc) return rc;
        if (a.place_tier == HA_RAG_TIER_HBM) {
            Slab &hs = c->slab[HA_RAG_TIER_HBM][ch.prec];
            rc = before_write(c, hs.use[a.place_slot], s);
            if (rc) return rc;
            if (!c->dry())
                HIPCHK(c, hipMemcpyAsync(hs.ptr(a.place_slot), sp, ch.bytes,
                                         hipMemcpyDeviceToDevice, s));
            undo.written[cold[k]] = 1;
        }
        if (!c->dry()) {
            HIPCHK(c, hipEventRecord(c->stg[sidx].consumed, s));
            c->stg[sidx].consumed_valid = true;
        }
        if (started < cold.size()) {
            rc = start_transfer(started++);
            if (rc) return rc;
        }
    }

    for (const Action &a : acts) {
        if (a.kind != Action::HOT_LATE) continue;
        const Chunk &ch = c->chunks[a.ci];
        // `made_by` in pass A guarantees the copy written by this call is still in its slot
        if (ch.slot[a.src_tier] != a.src_slot) return HA_RAG_EINVAL;
        Slab &hs = c->slab[a.src_tier][ch.prec];
        rc = before_read(c, hs.use[a.src_slot], s);
        if (rc) return rc;
        rc = push(c, batch,
                  make_desc(c, ch, hs.ptr(a.src_slot), reqs[a.req], a.tok_off,
                            a.src_tier == HA_RAG_TIER_PINNED),
                  s, &st.n_kernel_launches);
        if (rc) return rc;
    }
    rc = flush(c, batch, s, &st.n_kernel_launches);
    if (rc) return rc;
    rc = mark_stream(c, s);
    if (rc) return rc;
    undo.ok = true;
    if (stats) *stats = st;
    return HA_RAG_OK;
}

int register_slab_common(ha_rag_ctx *c, Slab &sl, uint32_t prec, size_t bytes, size_t align)
{
    size_t total;
    int rc = chunk_bytes_impl(c->cfg.n_layers, c->cfg.n_kv_heads, c->cfg.head_dim, prec,
                              c->group_of(prec), c->cfg.max_chunk_tokens, nullptr, nullptr, &total,
                              c->cfg.half_slots ? kPartK : kPartKV);
    if (rc) return rc;
    const size_t slot = (total + align - 1) / align * align;
    if (bytes < slot) return HA_RAG_EINVAL;
    const size_t n_slots = bytes / slot;
    if (n_slots > 0x7FFFFFFFu) return HA_RAG_EINVAL;
    sl.slot_bytes = slot;
    sl.n_slots = (uint32_t)n_slots;
    sl.use.assign(n_slots, SlotUse());
    sl.free_slots.resize(n_slots);
    for (size_t i = 0; i < n_slots; ++i) sl.free_slots[i] = (uint32_t)(n_slots - 1 - i);  // slot 0 first
    sl.reg = true;
    return HA_RAG_OK;
}

}  // namespace

// ===========================================================================
// C ABI
// ===========================================================================
extern "C" {

int ha_rag_chunk_bytes(uint32_t L, uint32_t H, uint32_t D, uint32_t prec, uint32_t group,
                       uint32_t T, size_t *payload, size_t *meta, size_t *total)
{
    return chunk_bytes_impl(L, H, D, prec, group, T, payload, meta, total);
}

int ha_rag_alg1_classes(const uint64_t *af, size_t n, const uint32_t *tau_ppm, uint32_t n_tau,
                        uint8_t *cls_out, uint32_t *rank_out)
{
    if ((n && (!af || !cls_out)) || (n_tau && !tau_ppm) || n_tau > 254) return HA_RAG_EINVAL;
    std::vector<size_t> order(n);
    for (size_t i = 0; i < n; ++i) order[i] = i;
    std::sort(order.begin(), order.end(), [&](size_t a, size_t b) {
        if (af[a] != af[b]) return af[a] > af[b];
        return a < b;
    });
    std::vector<uint64_t> idx(n_tau);
    uint64_t acc = 0;
    for (uint32_t k = 0; k < n_tau; ++k) {
        if (tau_ppm[k] > kPPM) return HA_RAG_EINVAL;
        acc = std::min<uint64_t>(n, acc + ((uint64_t)tau_ppm[k] * n) / kPPM);
        idx[k] = acc;
    }
    for (size_t r = 0; r < n; ++r) {
        uint8_t cls = 0;
        for (uint32_t k = 0; k < n_tau; ++k)
            if (r >= idx[k]) ++cls;
        cls_out[order[r]] = cls;
        if (rank_out) rank_out[order[r]] = (uint32_t)r;
    }
    return HA_RAG_OK;
}

const char *ha_rag_strerror(int code)
{
    switch (code) {
    case HA_RAG_OK: return "ok";
    case HA_RAG_EINVAL: return "invalid argument";
    case HA_RAG_ENOENT: return "unknown chunk id";
    case HA_RAG_ENOSPC: return "no space (pool slab, staging, bounce buffer or output cache)";
    case HA_RAG_EFORMAT: return "precision tag / group / shape mismatch";
    case HA_RAG_EHIP: return "HIP call failed";
    case HA_RAG_EIO: return "file I/O failed";
    default: return "unknown error code";
    }
}

const char *ha_rag_version(void) { return "ha_rag 0.2 (gfx950)"; }

int ha_rag_create(const ha_rag_config *cfg, ha_rag_ctx **out)
{
    if (!cfg || !out) return HA_RAG_EINVAL;
    *out = nullptr;
    if (cfg->n_layers == 0 || cfg->n_kv_heads == 0 || cfg->max_chunk_tokens == 0) return HA_RAG_EINVAL;
    if (cfg->head_dim == 0 || (cfg->head_dim % 8u)) return HA_RAG_EFORMAT;
    if (!valid_group(cfg->group_int8) || !valid_group(cfg->group_int4)) return HA_RAG_EFORMAT;
    if ((cfg->head_dim % cfg->group_int8) || (cfg->head_dim % cfg->group_int4)) return HA_RAG_EFORMAT;
    if (cfg->tau_gpu_ppm > kPPM || cfg->tau_pin_ppm > kPPM || cfg->tau_page_ppm > kPPM ||
        cfg->n_copy_streams > 8)
        return HA_RAG_EINVAL;
    if ((uint64_t)cfg->max_chunk_tokens * cfg->head_dim > 0x7FFFFFFFull) return HA_RAG_EINVAL;
    ha_rag_ctx *c = new (std::nothrow) ha_rag_ctx();
    if (!c) return HA_RAG_EINVAL;
    c->cfg = *cfg;
    c->n_tiles = 2u * cfg->n_layers * cfg->n_kv_heads;
    if (!c->dry()) {
        const uint32_t k = cfg->n_copy_streams ? cfg->n_copy_streams : 2u;
        for (uint32_t i = 0; i < k; ++i) {
            hipStream_t s;
            hipError_t e = hipStreamCreateWithFlags(&s, hipStreamNonBlocking);
            if (e != hipSuccess) {
                g_create_err = std::string("hipStreamCreateWithFlags: ") + hipGetErrorString(e);
                for (hipStream_t t : c->copy_streams) (void)hipStreamDestroy(t);
                delete c;
                return HA_RAG_EHIP;
            }
            c->copy_streams.push_back(s);
        }
    }
    *out = c;
    return HA_RAG_OK;
}

int ha_rag_destroy(ha_rag_ctx *c)
{
    if (!c) return HA_RAG_EINVAL;
    if (!c->dry()) {
        for (hipStream_t s : c->copy_streams) {
            (void)hipStreamSynchronize(s);
            (void)hipStreamDestroy(s);
        }
        for (auto &kv : c->stream_done) (void)hipEventDestroy(kv.second);
        for (StagingSlot &s : c->stg) {
            if (s.filled) (void)hipEventDestroy(s.filled);
            if (s.consumed) (void)hipEventDestroy(s.consumed);
        }
        for (BounceSlot &b : c->bnc)
            if (b.h2d_done) (void)hipEventDestroy(b.h2d_done);
    }
    for (uint32_t p = 0; p < HA_RAG_N_PREC; ++p)
        if (c->slab[HA_RAG_TIER_DISK][p].fd >= 0) (void)close(c->slab[HA_RAG_TIER_DISK][p].fd);
    std::free(c->dio);
    delete c;
    return HA_RAG_OK;
}

const char *ha_rag_last_hip_error(ha_rag_ctx *c)
{
    return c ? c->err.c_str() : g_create_err.c_str();
}

int ha_rag_set_launch_params(ha_rag_ctx *c, const ha_rag_launch_params *lp)
{
    if (!c || !lp) return HA_RAG_EINVAL;
    if (lp->threads < 64 || lp->threads > 1024 || (lp->threads & 63u)) return HA_RAG_EINVAL;
    if (lp->planes16 != 1 && lp->planes16 != 2 && lp->planes16 != 4) return HA_RAG_EINVAL;
    if (lp->planes8 != 2 && lp->planes8 != 4) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    c->launch = K1Launch{lp->threads, lp->planes16, lp->planes8, lp->nt_store != 0,
                         lp->nt_load != 0};
    return HA_RAG_OK;
}

static int quantize_impl(ha_rag_ctx *c, const void *src, uint32_t n_tokens, uint32_t prec,
                         uint32_t group, void *dst, uint32_t *saturated, void *stream, uint32_t part)
{
    if (!c || !src || !dst) return HA_RAG_EINVAL;
    if (((uintptr_t)src & 15u) || ((uintptr_t)dst & 15u) || ((uintptr_t)saturated & 3u)) return HA_RAG_EINVAL;
    size_t total;
    int rc = chunk_bytes_impl(c->cfg.n_layers, c->cfg.n_kv_heads, c->cfg.head_dim, prec, group,
                              n_tokens, nullptr, nullptr, &total, part);
    if (rc) return rc;
    if (c->dry()) return HA_RAG_OK;
    std::lock_guard<std::mutex> g(c->mu);
    HIPCHK(c, launch_k2(src, dst, part == kPartKV ? c->n_tiles : c->n_tiles / 2, c->cfg.head_dim,
                        n_tokens, prec, has_meta(prec) ? group : 32u, saturated,
                        (hipStream_t)stream));
    return HA_RAG_OK;
}

int ha_rag_quantize_chunk(ha_rag_ctx *c, const void *src, uint32_t n_tokens, uint32_t prec,
                          uint32_t group, void *dst, uint32_t *saturated, void *stream)
{
    return quantize_impl(c, src, n_tokens, prec, group, dst, saturated, stream, kPartKV);
}

int ha_rag_quantize_half(ha_rag_ctx *c, const void *src, uint32_t n_tokens, uint32_t prec,
                         uint32_t group, void *dst, uint32_t *saturated, void *stream)
{
    // the tile records of a half do not depend on which plane it is
    return quantize_impl(c, src, n_tokens, prec, group, dst, saturated, stream, kPartK);
}

int ha_rag_chunk_sq_error(ha_rag_ctx *c, const void *src, const void *packed, uint32_t n_tokens,
                          uint32_t prec, uint32_t group, uint32_t part, double *sum_sq, void *stream)
{
    if (!c || !src || !packed || !sum_sq) return HA_RAG_EINVAL;
    if (((uintptr_t)src & 15u) || ((uintptr_t)packed & 15u) || ((uintptr_t)sum_sq & 7u)) return HA_RAG_EINVAL;
    int rc = chunk_bytes_impl(c->cfg.n_layers, c->cfg.n_kv_heads, c->cfg.head_dim, prec, group,
                              n_tokens, nullptr, nullptr, nullptr, part);
    if (rc) return rc;
    if (c->dry()) return HA_RAG_OK;
    std::lock_guard<std::mutex> g(c->mu);
    HIPCHK(c, launch_k3(src, packed, part == kPartKV ? c->n_tiles : c->n_tiles / 2, c->cfg.head_dim,
                        n_tokens, prec, has_meta(prec) ? group : 32u, sum_sq, (hipStream_t)stream));
    return HA_RAG_OK;
}

static int load_packed_impl(ha_rag_ctx *c, const ha_rag_packed_chunk *chunks, uint32_t n, void *out,
                            uint64_t cap_tokens, uint64_t tok_base, void *stream,
                            const ha_rag_paged_cache *paged)
{
    if (!c || (n && !chunks) || n > HA_RAG_MAX_REQUEST_CHUNKS) return HA_RAG_EINVAL;
    if (paged) {
        int rc = check_paged(c, paged, &cap_tokens);
        if (rc) return rc;
    } else if ((n && !out) || ((uintptr_t)out & 15u)) {
        return HA_RAG_EINVAL;
    }
    const uint64_t D = c->cfg.head_dim;
    PlaneCursor chk(0);
    for (uint32_t i = 0; i < n; ++i) {
        const ha_rag_packed_chunk &pc = chunks[i];
        int rc = chunk_bytes_impl(c->cfg.n_layers, c->cfg.n_kv_heads, c->cfg.head_dim, pc.prec,
                                  pc.group, pc.n_tokens, nullptr, nullptr, nullptr, pc.part);
        if (rc) return rc;
        if (pc.n_tokens && (!pc.packed || ((uintptr_t)pc.packed & 15u))) return HA_RAG_EINVAL;
        uint64_t at;
        if (!chk.place(pc.part, pc.n_tokens, &at)) return HA_RAG_EINVAL;
    }
    if (!chk.closed()) return HA_RAG_EINVAL;
    if (tok_base > cap_tokens || chk.end() > cap_tokens - tok_base) return HA_RAG_ENOSPC;
    if (cap_tokens * D > 0x7FFFFFFFFFFFull) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    Batch batch;
    init_batch(c, batch, paged);
    PlaneCursor cur(tok_base);
    for (uint32_t i = 0; i < n; ++i) {
        const ha_rag_packed_chunk &pc = chunks[i];
        if (pc.n_tokens == 0) continue;
        uint64_t off = 0;
        (void)cur.place(pc.part, pc.n_tokens, &off);  // checked above
        K1Chunk d;
        d.src = static_cast<const uint8_t *>(pc.packed);
        if (paged) {
            d.out = reinterpret_cast<uint8_t *>((uintptr_t)(off * D * 2ull));
            d.out_tile_stride = 0;
        } else {
            d.out = static_cast<uint8_t *>(out) + off * D * 2ull;
            d.out_tile_stride = cap_tokens * D * 2ull;
        }
        d.n_tokens = pc.n_tokens;
        d.fmt = pc.prec | ((has_meta(pc.prec) ? log2u(pc.group) : 0u) << 8) | (pc.part << 16);
        int rc = push(c, batch, d, (hipStream_t)stream, nullptr);
        if (rc) return rc;
    }
    return flush(c, batch, (hipStream_t)stream, nullptr);
}

int ha_rag_load_packed(ha_rag_ctx *c, const ha_rag_packed_chunk *chunks, uint32_t n, void *out,
                       uint64_t cap_tokens, uint64_t tok_base, void *stream)
{
    return load_packed_impl(c, chunks, n, out, cap_tokens, tok_base, stream, nullptr);
}

int ha_rag_load_packed_paged(ha_rag_ctx *c, const ha_rag_packed_chunk *chunks, uint32_t n,
                             const ha_rag_paged_cache *cache, uint64_t tok_base, void *stream)
{
    if (!cache) return HA_RAG_EINVAL;
    return load_packed_impl(c, chunks, n, nullptr, 0, tok_base, stream, cache);
}

int ha_rag_register_slab(ha_rag_ctx *c, uint32_t tier, uint32_t prec, void *base, size_t bytes)
{
    if (!c || !base || tier > HA_RAG_TIER_PAGEABLE || prec >= HA_RAG_N_PREC) return HA_RAG_EINVAL;
    if ((uintptr_t)base & (tier == HA_RAG_TIER_PAGEABLE ? 15u : 255u)) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    Slab &sl = c->slab[tier][prec];
    if (sl.registered()) return HA_RAG_EINVAL;
    int rc = register_slab_common(c, sl, prec, bytes, 256);
    if (rc) return rc;
    sl.base = static_cast<uint8_t *>(base);
    return HA_RAG_OK;
}

int ha_rag_register_disk(ha_rag_ctx *c, uint32_t prec, const char *path, size_t bytes)
{
    if (!c || !path || prec >= HA_RAG_N_PREC) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    Slab &sl = c->slab[HA_RAG_TIER_DISK][prec];
    if (sl.registered()) return HA_RAG_EINVAL;
    int rc = register_slab_common(c, sl, prec, bytes, kDirectAlign);
    if (rc) return rc;
    if (!c->dry()) {
        int flags = O_RDWR | O_CREAT;
        if (c->direct()) flags |= O_DIRECT;
        sl.fd = open(path, flags, 0600);
        if (sl.fd < 0) {
            sl.reg = false;
            return io_error(c, "open");
        }
        struct stat stt;
        if (fstat(sl.fd, &stt) != 0 ||
            ((size_t)stt.st_size < (size_t)sl.n_slots * sl.slot_bytes &&
             ftruncate(sl.fd, (off_t)((size_t)sl.n_slots * sl.slot_bytes)) != 0)) {
            rc = io_error(c, "ftruncate");
            (void)close(sl.fd);
            sl.fd = -1;
            sl.reg = false;
            return rc;
        }
    }
    return HA_RAG_OK;
}

int ha_rag_register_staging(ha_rag_ctx *c, void *base, size_t bytes)
{
    if (!c || !base || ((uintptr_t)base & 255u)) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    if (c->staging) return HA_RAG_EINVAL;
    size_t slot = 0;
    for (uint32_t t = HA_RAG_TIER_PINNED; t < kTiers; ++t)
        for (uint32_t p = 0; p < HA_RAG_N_PREC; ++p) slot = std::max(slot, c->slab[t][p].slot_bytes);
    if (slot == 0) return HA_RAG_EINVAL;  // register the host-side slabs first
    const size_t n = bytes / slot;
    if (n < 2) return HA_RAG_ENOSPC;
    c->stg.resize(n);
    if (!c->dry()) {
        for (StagingSlot &s : c->stg) {
            HIPCHK(c, hipEventCreateWithFlags(&s.filled, hipEventDisableTiming));
            HIPCHK(c, hipEventCreateWithFlags(&s.consumed, hipEventDisableTiming));
        }
    }
    c->staging = static_cast<uint8_t *>(base);
    c->staging_slot_bytes = slot;
    return HA_RAG_OK;
}

int ha_rag_register_bounce(ha_rag_ctx *c, void *base, size_t bytes)
{
    if (!c || !base || ((uintptr_t)base & (kDirectAlign - 1))) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    if (c->bounce) return HA_RAG_EINVAL;
    size_t slot = 0;
    for (uint32_t t = HA_RAG_TIER_PAGEABLE; t < kTiers; ++t)
        for (uint32_t p = 0; p < HA_RAG_N_PREC; ++p) slot = std::max(slot, c->slab[t][p].slot_bytes);
    if (slot == 0) return HA_RAG_EINVAL;  // register the pageable / disk slabs first
    slot = (slot + kDirectAlign - 1) / kDirectAlign * kDirectAlign;
    const size_t n = bytes / slot;
    if (n < 2) return HA_RAG_ENOSPC;
    if (c->direct() && !c->dry()) {
        void *p = nullptr;
        if (posix_memalign(&p, kDirectAlign, slot) != 0) return HA_RAG_ENOSPC;
        c->dio = static_cast<uint8_t *>(p);
        c->dio_bytes = slot;
    }
    c->bnc.resize(n);
    if (!c->dry())
        for (BounceSlot &b : c->bnc) HIPCHK(c, hipEventCreateWithFlags(&b.h2d_done, hipEventDisableTiming));
    c->bounce = static_cast<uint8_t *>(base);
    c->bounce_slot_bytes = slot;
    return HA_RAG_OK;
}

static int insert_impl(ha_rag_ctx *c, uint64_t id, uint32_t part, uint32_t prec, uint32_t n_tokens,
                       const void *packed, int packed_is_device, uint32_t tier, void *stream)
{
    if (!c || tier >= kTiers || prec >= HA_RAG_N_PREC || id == HA_RAG_NO_CHUNK) return HA_RAG_EINVAL;
    if (part > kPartV) return HA_RAG_EINVAL;
    if (n_tokens == 0 || n_tokens > c->cfg.max_chunk_tokens) return HA_RAG_EINVAL;
    if (part == kPartKV && c->cfg.half_slots) return HA_RAG_EFORMAT;  // slots hold halves only
    hipStream_t s = (hipStream_t)stream;
    std::lock_guard<std::mutex> g(c->mu);
    Slab &sl = c->slab[tier][prec];
    if (!sl.registered()) return HA_RAG_ENOSPC;
    size_t total;
    int rc = chunk_bytes_impl(c->cfg.n_layers, c->cfg.n_kv_heads, c->cfg.head_dim, prec,
                              c->group_of(prec), n_tokens, nullptr, nullptr, &total, part);
    if (rc) return rc;
    uint32_t ci;
    Chunk *ch = find_chunk(c, id, &ci);
    if (ch) {
        if (ch->slot[tier] >= 0) return HA_RAG_EINVAL;
        if (ch->prec != prec || ch->n_tokens != n_tokens || ch->part != part) return HA_RAG_EFORMAT;
    }
    // pageable / disk targets fed from device memory or through O_DIRECT need a bounce buffer
    const bool via_bounce = packed && tier >= HA_RAG_TIER_PAGEABLE && packed_is_device;
    if (packed && tier == HA_RAG_TIER_DISK && c->direct() && !c->dry() && !c->dio) return HA_RAG_ENOSPC;
    if (via_bounce && (c->bnc.size() < 2 || c->io_bytes(total) > c->bounce_slot_bytes)) return HA_RAG_ENOSPC;
    uint64_t ev;
    const int32_t slot = tier_acquire(c, tier, prec, &ev);
    if (slot < 0) return HA_RAG_ENOSPC;
    if (!ch) {
        ci = (uint32_t)c->chunks.size();
        c->chunks.emplace_back();
        ch = &c->chunks.back();
        ch->id = id;
        ch->prec = prec;
        ch->n_tokens = n_tokens;
        ch->part = part;
        ch->bytes = total;
        c->index.emplace(id, ci);
    }
    tier_attach(c, tier, ci, slot);
    if (!packed || c->dry()) return HA_RAG_OK;
    if (tier == HA_RAG_TIER_HBM) {
        rc = before_write(c, sl.use[slot], s);
        if (rc) return rc;
        HIPCHK(c, hipMemcpyAsync(sl.ptr(slot), packed, total,
                                 packed_is_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, s));
        return mark_stream(c, s);
    }
    if (tier == HA_RAG_TIER_PINNED) {
        rc = before_host_write(c, sl.use[slot]);
        if (rc) return rc;
        if (packed_is_device) {
            HIPCHK(c, hipMemcpyAsync(sl.ptr(slot), packed, total, hipMemcpyDeviceToHost, s));
            sl.use[slot].writer = s;
            sl.use[slot].has_writer = true;
            return mark_stream(c, s);
        }
        std::memcpy(sl.ptr(slot), packed, total);
        return HA_RAG_OK;
    }
    // pageable or disk: the bytes have to be in host memory first
    const uint8_t *host = static_cast<const uint8_t *>(packed);
    if (via_bounce) {
        size_t bidx;
        rc = acquire_bounce(c, &bidx);
        if (rc) return rc;
        uint8_t *bp = c->bounce + bidx * c->bounce_slot_bytes;
        if (packed_is_device) {
            HIPCHK(c, hipMemcpyAsync(bp, packed, total, hipMemcpyDeviceToHost, s));
            HIPCHK(c, hipStreamSynchronize(s));
        } else {
            std::memcpy(bp, packed, total);
        }
        host = bp;
    }
    if (tier == HA_RAG_TIER_PAGEABLE) {
        std::memcpy(sl.ptr(slot), host, total);
        return HA_RAG_OK;
    }
    if (!c->direct()) return write_full(c, sl.fd, host, total, sl.offset(slot));
    std::memcpy(c->dio, host, total);
    std::memset(c->dio + total, 0, c->io_bytes(total) - total);
    return write_full(c, sl.fd, c->dio, c->io_bytes(total), sl.offset(slot));
}

int ha_rag_pool_insert(ha_rag_ctx *c, uint64_t id, uint32_t prec, uint32_t n_tokens,
                       const void *packed, int packed_is_device, uint32_t tier, void *stream)
{
    return insert_impl(c, id, kPartKV, prec, n_tokens, packed, packed_is_device, tier, stream);
}

int ha_rag_pool_insert_half(ha_rag_ctx *c, uint64_t id, uint32_t part, uint32_t prec,
                            uint32_t n_tokens, const void *packed, int packed_is_device,
                            uint32_t tier, void *stream)
{
    if (part != kPartK && part != kPartV) return HA_RAG_EINVAL;
    return insert_impl(c, id, part, prec, n_tokens, packed, packed_is_device, tier, stream);
}

int ha_rag_pool_slot(ha_rag_ctx *c, uint64_t id, uint32_t tier, void **ptr, size_t *bytes)
{
    if (!c || tier > HA_RAG_TIER_PAGEABLE) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    Chunk *ch = find_chunk(c, id);
    if (!ch || ch->slot[tier] < 0) return HA_RAG_ENOENT;
    if (ptr) *ptr = c->slab[tier][ch->prec].ptr(ch->slot[tier]);
    if (bytes) *bytes = (size_t)ch->bytes;
    return HA_RAG_OK;
}

int ha_rag_pool_promote(ha_rag_ctx *c, uint64_t id, void *stream)
{
    if (!c) return HA_RAG_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    std::lock_guard<std::mutex> g(c->mu);
    uint32_t ci;
    Chunk *ch = find_chunk(c, id, &ci);
    if (!ch) return HA_RAG_ENOENT;
    if (ch->slot[HA_RAG_TIER_HBM] >= 0) return HA_RAG_OK;
    if (ch->slot[HA_RAG_TIER_PINNED] < 0) return HA_RAG_ENOENT;
    uint64_t ev;
    const int32_t slot = tier_acquire(c, HA_RAG_TIER_HBM, ch->prec, &ev);
    if (slot < 0) return HA_RAG_ENOSPC;
    tier_attach(c, HA_RAG_TIER_HBM, ci, slot);
    if (!c->dry()) {
        Slab &hs = c->slab[HA_RAG_TIER_HBM][ch->prec];
        Slab &ps = c->slab[HA_RAG_TIER_PINNED][ch->prec];
        int rc = before_write(c, hs.use[slot], s);
        if (rc) return rc;
        SlotUse &pu = ps.use[ch->slot[HA_RAG_TIER_PINNED]];
        if (pu.has_writer) {
            rc = wait_for(c, s, pu.writer);
            if (rc) return rc;
        }
        if (std::find(pu.readers.begin(), pu.readers.end(), s) == pu.readers.end()) pu.readers.push_back(s);
        HIPCHK(c, hipMemcpyAsync(hs.ptr(slot), ps.ptr(ch->slot[HA_RAG_TIER_PINNED]), ch->bytes,
                                 hipMemcpyHostToDevice, s));
        rc = mark_stream(c, s);
        if (rc) return rc;
    }
    return HA_RAG_OK;
}

int ha_rag_pool_evict(ha_rag_ctx *c, uint64_t id, uint32_t tier)
{
    if (!c || tier >= kCacheTiers) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    uint32_t ci;
    Chunk *ch = find_chunk(c, id, &ci);
    if (!ch || ch->slot[tier] < 0) return HA_RAG_ENOENT;
    if (!ch->has_slower_copy(tier)) return HA_RAG_EINVAL;
    tier_detach(c, tier, ci);
    return HA_RAG_OK;
}

int ha_rag_pool_query(ha_rag_ctx *c, uint64_t id, ha_rag_chunk_info *info)
{
    if (!c || !info) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    Chunk *ch = find_chunk(c, id);
    if (!ch) return HA_RAG_ENOENT;
    std::memset(info, 0, sizeof *info);
    info->prec = ch->prec;
    info->group = c->group_of(ch->prec);
    info->n_tokens = ch->n_tokens;
    info->part = ch->part;
    info->disk_slot = ch->slot[HA_RAG_TIER_DISK] >= 0 ? (uint32_t)ch->slot[HA_RAG_TIER_DISK] : UINT32_MAX;
    info->in_hbm = ch->slot[HA_RAG_TIER_HBM] >= 0;
    info->in_pinned = ch->slot[HA_RAG_TIER_PINNED] >= 0;
    info->in_pageable = ch->slot[HA_RAG_TIER_PAGEABLE] >= 0;
    info->on_disk = ch->slot[HA_RAG_TIER_DISK] >= 0;
    info->rank = ch->rank;
    info->count = ch->count;
    info->bytes = ch->bytes;
    if (info->in_hbm) info->hbm_ptr = c->slab[HA_RAG_TIER_HBM][ch->prec].ptr(ch->slot[HA_RAG_TIER_HBM]);
    if (info->in_pinned)
        info->pinned_ptr = c->slab[HA_RAG_TIER_PINNED][ch->prec].ptr(ch->slot[HA_RAG_TIER_PINNED]);
    return HA_RAG_OK;
}

int ha_rag_pool_lru(ha_rag_ctx *c, uint32_t tier, uint64_t *ids, size_t cap, size_t *n)
{
    if (!c || !n || (cap && !ids) || tier >= kCacheTiers) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    std::vector<const Chunk *> v;
    for (const Chunk &ch : c->chunks)
        if (ch.slot[tier] >= 0) v.push_back(&ch);
    std::sort(v.begin(), v.end(),
              [tier](const Chunk *a, const Chunk *b) { return a->last_use[tier] < b->last_use[tier]; });
    *n = std::min(cap, v.size());
    for (size_t i = 0; i < *n; ++i) ids[i] = v[i]->id;
    return HA_RAG_OK;
}

int ha_rag_pool_hbm_lru(ha_rag_ctx *c, uint64_t *ids, size_t cap, size_t *n)
{
    return ha_rag_pool_lru(c, HA_RAG_TIER_HBM, ids, cap, n);
}

// ---- the knowledge base survives the process: index of the file tier ---------------
namespace {

struct IndexHeader {
    char magic[8];  // "HARAGIX1"
    uint32_t n_layers, n_kv_heads, head_dim, max_chunk_tokens, group_int8, group_int4, half_slots;
    uint32_t n_prec;
    uint64_t slot_bytes[HA_RAG_N_PREC];  // of the file slab per tag, 0 = none registered
    uint64_t n_entries;
};

struct IndexEntry {
    uint64_t id, count;
    uint32_t prec, part, n_tokens;
    int32_t slot;
};

const char kIndexMagic[8] = {'H', 'A', 'R', 'A', 'G', 'I', 'X', '1'};

}  // namespace

int ha_rag_pool_save_index(ha_rag_ctx *c, const char *path)
{
    if (!c || !path) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    IndexHeader h;
    std::memset(&h, 0, sizeof h);
    std::memcpy(h.magic, kIndexMagic, 8);
    h.n_layers = c->cfg.n_layers;
    h.n_kv_heads = c->cfg.n_kv_heads;
    h.head_dim = c->cfg.head_dim;
    h.max_chunk_tokens = c->cfg.max_chunk_tokens;
    h.group_int8 = c->cfg.group_int8;
    h.group_int4 = c->cfg.group_int4;
    h.half_slots = c->cfg.half_slots;
    h.n_prec = HA_RAG_N_PREC;
    for (uint32_t p = 0; p < HA_RAG_N_PREC; ++p)
        h.slot_bytes[p] = c->slab[HA_RAG_TIER_DISK][p].registered() ? c->slab[HA_RAG_TIER_DISK][p].slot_bytes : 0;
    std::vector<IndexEntry> entries;
    for (const Chunk &ch : c->chunks) {
        if (ch.slot[HA_RAG_TIER_DISK] < 0) continue;
        IndexEntry e;
        std::memset(&e, 0, sizeof e);
        e.id = ch.id;
        e.count = ch.count;
        e.prec = ch.prec;
        e.part = ch.part;
        e.n_tokens = ch.n_tokens;
        e.slot = ch.slot[HA_RAG_TIER_DISK];
        entries.push_back(e);
    }
    h.n_entries = entries.size();
    FILE *f = std::fopen(path, "wb");
    if (!f) return io_error(c, "fopen");
    bool ok = std::fwrite(&h, sizeof h, 1, f) == 1;
    if (ok && !entries.empty())
        ok = std::fwrite(entries.data(), sizeof(IndexEntry), entries.size(), f) == entries.size();
    if (std::fclose(f) != 0) ok = false;
    if (!ok) return io_error(c, "fwrite");
    return HA_RAG_OK;
}

int ha_rag_pool_load_index(ha_rag_ctx *c, const char *path, size_t *n_loaded)
{
    if (!c || !path) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    FILE *f = std::fopen(path, "rb");
    if (!f) return io_error(c, "fopen");
    IndexHeader h;
    std::vector<IndexEntry> entries;
    bool ok = std::fread(&h, sizeof h, 1, f) == 1;
    long file_bytes = -1;
    if (ok && std::fseek(f, 0, SEEK_END) == 0) file_bytes = std::ftell(f);
    ok = ok && file_bytes >= 0 && std::fseek(f, (long)sizeof h, SEEK_SET) == 0;
    // the entry count has to be the one the file's size implies before anything is allocated
    if (ok && std::memcmp(h.magic, kIndexMagic, 8) == 0 &&
        h.n_entries == ((uint64_t)file_bytes - sizeof h) / sizeof(IndexEntry) &&
        ((uint64_t)file_bytes - sizeof h) % sizeof(IndexEntry) == 0) {
        entries.resize((size_t)h.n_entries);
        if (!entries.empty())
            ok = std::fread(entries.data(), sizeof(IndexEntry), entries.size(), f) == entries.size();
    } else {
        ok = false;
    }
    std::fclose(f);
    if (!ok) {
        c->err = "index file: truncated or not an index";
        return HA_RAG_EIO;
    }
    // the files hold bytes of one shape and one slot grid: both must be the ones of this context
    if (h.n_layers != c->cfg.n_layers || h.n_kv_heads != c->cfg.n_kv_heads ||
        h.head_dim != c->cfg.head_dim || h.max_chunk_tokens != c->cfg.max_chunk_tokens ||
        h.group_int8 != c->cfg.group_int8 || h.group_int4 != c->cfg.group_int4 ||
        h.half_slots != c->cfg.half_slots || h.n_prec != HA_RAG_N_PREC)
        return HA_RAG_EFORMAT;
    // checks first: nothing changes unless every entry fits
    std::vector<std::vector<uint8_t>> taken(HA_RAG_N_PREC);
    for (const IndexEntry &e : entries) {
        if (e.prec >= HA_RAG_N_PREC || e.part > kPartV || e.id == HA_RAG_NO_CHUNK) return HA_RAG_EFORMAT;
        const Slab &sl = c->slab[HA_RAG_TIER_DISK][e.prec];
        if (!sl.registered() || sl.slot_bytes != h.slot_bytes[e.prec]) return HA_RAG_EFORMAT;
        if (e.slot < 0 || (uint32_t)e.slot >= sl.n_slots) return HA_RAG_EFORMAT;
        if (e.n_tokens == 0 || e.n_tokens > c->cfg.max_chunk_tokens) return HA_RAG_EFORMAT;
        if (e.part == kPartKV && c->cfg.half_slots) return HA_RAG_EFORMAT;
        if (c->index.count(e.id)) return HA_RAG_EINVAL;
        if (taken[e.prec].empty()) {
            taken[e.prec].assign(sl.n_slots, 1);
            for (uint32_t fs : sl.free_slots) taken[e.prec][fs] = 0;
        }
        if (taken[e.prec][e.slot]) return HA_RAG_EINVAL;  // slot in use, or named twice
        taken[e.prec][e.slot] = 1;
    }
    {
        std::vector<uint64_t> ids(entries.size());
        for (size_t i = 0; i < entries.size(); ++i) ids[i] = entries[i].id;
        std::sort(ids.begin(), ids.end());
        if (std::adjacent_find(ids.begin(), ids.end()) != ids.end()) return HA_RAG_EINVAL;
    }
    for (const IndexEntry &e : entries) {
        size_t total = 0;
        (void)chunk_bytes_impl(c->cfg.n_layers, c->cfg.n_kv_heads, c->cfg.head_dim, e.prec,
                               c->group_of(e.prec), e.n_tokens, nullptr, nullptr, &total, e.part);
        const uint32_t ci = (uint32_t)c->chunks.size();
        c->chunks.emplace_back();
        Chunk &ch = c->chunks.back();
        ch.id = e.id;
        ch.prec = e.prec;
        ch.part = e.part;
        ch.n_tokens = e.n_tokens;
        ch.bytes = total;
        ch.count = e.count;
        ch.slot[HA_RAG_TIER_DISK] = e.slot;
        c->index.emplace(e.id, ci);
    }
    for (uint32_t p = 0; p < HA_RAG_N_PREC; ++p) {
        if (taken[p].empty()) continue;
        Slab &sl = c->slab[HA_RAG_TIER_DISK][p];
        sl.free_slots.clear();
        for (uint32_t i = sl.n_slots; i-- > 0;)
            if (!taken[p][i]) sl.free_slots.push_back(i);  // lowest slot on top of the stack
    }
    if (n_loaded) *n_loaded = entries.size();
    return HA_RAG_OK;
}

int ha_rag_touch(ha_rag_ctx *c, const uint64_t *ids, size_t n)
{
    if (!c || (n && !ids)) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    for (size_t i = 0; i < n; ++i)
        if (!find_chunk(c, ids[i])) return HA_RAG_ENOENT;
    for (size_t i = 0; i < n; ++i) find_chunk(c, ids[i])->count += 1;
    return HA_RAG_OK;
}

int ha_rag_set_counts(ha_rag_ctx *c, const uint64_t *ids, const uint64_t *counts, size_t n)
{
    if (!c || (n && (!ids || !counts))) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    for (size_t i = 0; i < n; ++i)
        if (!find_chunk(c, ids[i])) return HA_RAG_ENOENT;
    for (size_t i = 0; i < n; ++i) find_chunk(c, ids[i])->count = counts[i];
    return HA_RAG_OK;
}

int ha_rag_rerank(ha_rag_ctx *c)
{
    if (!c) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    rerank_locked(c);
    return HA_RAG_OK;
}

int ha_rag_get_rank(ha_rag_ctx *c, uint64_t id, uint32_t *rank)
{
    if (!c || !rank) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    Chunk *ch = find_chunk(c, id);
    if (!ch) return HA_RAG_ENOENT;
    *rank = ch->rank;
    return HA_RAG_OK;
}

int ha_rag_load_chunks(ha_rag_ctx *c, const uint64_t *ids, const uint8_t *tags, uint32_t n,
                       void *out, uint64_t cap_tokens, uint64_t tok_base, void *stream,
                       ha_rag_load_stats *stats, ha_rag_chunk_trace *trace)
{
    if (!c || (n && !ids) || n > HA_RAG_MAX_REQUEST_CHUNKS) return HA_RAG_EINVAL;
    if (cap_tokens * (uint64_t)c->cfg.head_dim > 0x7FFFFFFFFFFFull) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    Request rq{0, n, static_cast<uint8_t *>(out), cap_tokens, tok_base, nullptr};
    return load_impl(c, ids, tags, &rq, 1, n, (hipStream_t)stream, stats, trace);
}

int ha_rag_load_chunks_paged(ha_rag_ctx *c, const uint64_t *ids, const uint8_t *tags, uint32_t n,
                             const ha_rag_paged_cache *cache, uint64_t tok_base, void *stream,
                             ha_rag_load_stats *stats, ha_rag_chunk_trace *trace)
{
    if (!c || !cache || (n && !ids) || n > HA_RAG_MAX_REQUEST_CHUNKS) return HA_RAG_EINVAL;
    uint64_t cap = 0;
    int rc = check_paged(c, cache, &cap);
    if (rc) return rc;
    std::lock_guard<std::mutex> g(c->mu);
    Request rq{0, n, nullptr, cap, tok_base, cache};
    return load_impl(c, ids, tags, &rq, 1, n, (hipStream_t)stream, stats, trace);
}

int ha_rag_load_batch(ha_rag_ctx *c, const uint64_t *ids, const uint8_t *tags,
                      const uint32_t *request_starts, uint32_t n_requests, void *const *outs,
                      const uint64_t *cap_tokens, const uint64_t *tok_base, void *stream,
                      ha_rag_load_stats *stats, ha_rag_chunk_trace *trace)
{
    if (!c || !request_starts || (n_requests && (!outs || !cap_tokens))) return HA_RAG_EINVAL;
    const uint32_t n = request_starts[n_requests];
    if ((n && !ids) || n > HA_RAG_MAX_REQUEST_CHUNKS) return HA_RAG_EINVAL;
    std::vector<Request> reqs(n_requests);
    for (uint32_t r = 0; r < n_requests; ++r) {
        if (request_starts[r + 1] < request_starts[r]) return HA_RAG_EINVAL;
        if (cap_tokens[r] * (uint64_t)c->cfg.head_dim > 0x7FFFFFFFFFFFull) return HA_RAG_EINVAL;
        reqs[r] = Request{request_starts[r], request_starts[r + 1], static_cast<uint8_t *>(outs[r]),
                          cap_tokens[r], tok_base ? tok_base[r] : 0, nullptr};
    }
    std::lock_guard<std::mutex> g(c->mu);
    return load_impl(c, ids, tags, reqs.data(), n_requests, n, (hipStream_t)stream, stats, trace);
}

}  // extern "C"
