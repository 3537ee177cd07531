// Pools behind include/ha_rag.h: slabs in four tiers, slot bookkeeping, LRU lists, the
// stream / event rules that keep a slot from being overwritten while it is read, hotness
// counters and ranks (Algorithm 1 steps 1-2, Algorithm 2 step 1), and the index of the
// file tier.
#include "ha_rag_internal.h"

#include <fcntl.h>
#include <sys/stat.h>
#include <unistd.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>

namespace ha_rag_host {

int chunk_bytes_impl(uint32_t L, uint32_t H, uint32_t D, uint32_t prec, uint32_t group,
                     uint32_t T, size_t *payload, size_t *meta, size_t *total,
                     uint32_t part)
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

Chunk *find_chunk(ha_rag_ctx *c, uint64_t id, uint32_t *idx)
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
                     uint64_t keep_call)
{
    Slab &sl = c->slab[tier][prec];
    *evicted = HA_RAG_NO_CHUNK;
    if (!sl.registered()) return -1;
    if (sl.free_slots.empty() && tier < kCacheTiers) {
        for (uint32_t ci : sl.lru) {
            const Chunk &v = c->chunks[ci];
            if (keep_call && v.made_by[tier] == keep_call) continue;
            // a copy that a running call is still writing, or reading on the host, stays
            if (v.pending[tier] || sl.use[(size_t)v.slot[tier]].host_readers) continue;
            if (v.has_slower_copy(tier)) {
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

uint32_t new_chunk_entry(ha_rag_ctx *c)
{
    if (!c->dead.empty()) {
        const uint32_t ci = c->dead.back();
        c->dead.pop_back();
        c->chunks[ci] = Chunk();
        return ci;
    }
    c->chunks.emplace_back();
    return (uint32_t)(c->chunks.size() - 1);
}

void rerank_locked(ha_rag_ctx *c)
{
    // the sort keys next to each other (not reached through the chunk table by every comparison)
    struct Key {
        uint64_t count, id;
        uint32_t ci;
    };
    std::vector<Key> order;
    order.reserve(c->chunks.size());
    for (size_t i = 0; i < c->chunks.size(); ++i)
        if (c->chunks[i].id != HA_RAG_NO_CHUNK) order.push_back(Key{c->chunks[i].count, c->chunks[i].id, (uint32_t)i});
    const size_t n = order.size();  // N of Algorithm 2 step 1: the chunks that exist
    std::sort(order.begin(), order.end(), [](const Key &x, const Key &y) {
        if (x.count != y.count) return x.count > y.count;
        return x.id < y.id;
    });
    for (size_t r = 0; r < n; ++r) c->chunks[order[r].ci].rank = (uint32_t)r;
    // idx_1 = tau_GPU * N, idx_2 = tau_PIN * N + idx_1, idx_3 = tau_PAGE * N + idx_2
    const uint32_t tau[3] = {c->cfg.tau_gpu_ppm, c->cfg.tau_pin_ppm, c->cfg.tau_page_ppm};
    uint64_t acc = 0;
    for (int t = 0; t < 3; ++t) {
        acc = std::min<uint64_t>(n, acc + ((uint64_t)tau[t] * n) / kPPM);
        c->bound[t] = (uint32_t)acc;
    }
}

bool reserve_bounce(ha_rag_ctx *c, std::unique_lock<std::mutex> &lk, bool block, size_t *idx,
                    hipEvent_t *wait_ev)
{
    for (;;) {
        for (size_t k = 0; k < c->bnc.size(); ++k) {
            const size_t b = (size_t)(c->bnc_next++ % c->bnc.size());
            BounceSlot &bs = c->bnc[b];
            if (bs.reserved) continue;
            bs.reserved = true;
            *wait_ev = bs.busy ? bs.h2d_done : nullptr;
            bs.busy = false;
            *idx = b;
            return true;
        }
        if (!block) return false;
        c->cv.wait(lk);  // a running call hands one back when its copy is enqueued
    }
}

void release_bounce(ha_rag_ctx *c, size_t idx, bool copy_in_flight)
{
    c->bnc[idx].reserved = false;
    c->bnc[idx].busy = copy_in_flight;
    c->cv.notify_all();
}

void take_host_write_events(ha_rag_ctx *c, SlotUse &u, std::vector<hipEvent_t> *out)
{
    if (!c->dry()) {
        for (hipEvent_t ev : u.read_events) out->push_back(ev);
        if (u.has_writer) {
            auto it = c->stream_done.find(u.writer);
            if (it != c->stream_done.end()) out->push_back(it->second);
        }
        for (hipStream_t r : u.readers) {
            auto it = c->stream_done.find(r);
            if (it != c->stream_done.end()) out->push_back(it->second);
        }
    }
    u.read_events.clear();
    u.readers.clear();
    u.has_writer = false;
}

}  // namespace ha_rag_host

using namespace ha_rag_host;

namespace {

int register_slab_common(ha_rag_ctx *c, Slab &sl, uint32_t prec, size_t bytes, size_t align)
{
    size_t total;
    int rc = chunk_bytes_impl(c->cfg.n_layers, c->cfg.n_kv_heads, c->cfg.head_dim, prec,
                              c->group_of(prec), c->cfg.max_chunk_tokens, nullptr, nullptr, &total,
                              c->cfg.half_slots ? kPartK : kPartKV);
    if (rc) return rc;
    const size_t slot = (total + align - 1) / align * align;
    if (bytes < slot) return HA_RAG_EINVAL;
    if (bytes == SIZE_MAX) bytes = 0;  // a slab of caller-owned addresses: no slots yet
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

extern "C" {

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

int ha_rag_register_external(ha_rag_ctx *c, uint32_t prec)
{
    if (!c || prec >= HA_RAG_N_PREC) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    Slab &sl = c->slab[HA_RAG_TIER_PINNED][prec];
    if (sl.registered()) return HA_RAG_EINVAL;
    // a slab without memory of its own: slots are added as chunks are inserted
    int rc = register_slab_common(c, sl, prec, SIZE_MAX, 256);
    if (rc) return rc;
    sl.external = true;
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
    if (!c->no_io()) {
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
    if (c->direct() && !c->no_io()) {
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
    std::unique_lock<std::mutex> g(c->mu);
    Slab &sl = c->slab[tier][prec];
    if (!sl.registered()) return HA_RAG_ENOSPC;
    if (sl.external) return HA_RAG_EINVAL;  // its slots are the caller's memory: ha_rag_pool_insert_external
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
    // a direct write passes through the page-aligned buffer, which is as large as the largest
    // pageable / disk slot that was registered before the bounce buffers
    if (packed && tier == HA_RAG_TIER_DISK && c->direct() && !c->no_io() &&
        (!c->dio || c->io_bytes(total) > c->dio_bytes))
        return HA_RAG_ENOSPC;
    if (via_bounce && (c->bnc.size() < 2 || c->io_bytes(total) > c->bounce_slot_bytes)) return HA_RAG_ENOSPC;
    uint64_t ev;
    const int32_t slot = tier_acquire(c, tier, prec, &ev);
    if (slot < 0) return HA_RAG_ENOSPC;
    if (!ch) {
        ci = new_chunk_entry(c);
        ch = &c->chunks[ci];
        ch->id = id;
        ch->prec = prec;
        ch->n_tokens = n_tokens;
        ch->part = part;
        ch->bytes = total;
        c->index.emplace(id, ci);
    }
    tier_attach(c, tier, ci, slot);
    if (!packed || c->no_io()) return HA_RAG_OK;
    if (tier == HA_RAG_TIER_HBM) {
        if (c->dry()) return HA_RAG_OK;
        rc = before_write(c, sl.use[slot], s);
        if (rc) return rc;
        HIPCHK(c, hipMemcpyAsync(sl.ptr(slot), packed, total,
                                 packed_is_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, s));
        return mark_stream(c, s);
    }
    if (packed_is_device && c->dry()) return HA_RAG_OK;  // no device to copy from
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
    // This is the offline path (the knowledge base is built before it is served): the context
    // stays locked while the bytes are written.
    size_t bidx = 0;
    if (via_bounce) {
        hipEvent_t ev = nullptr;
        (void)reserve_bounce(c, g, true, &bidx, &ev);
        uint8_t *bp = c->bounce + bidx * c->bounce_slot_bytes;
        hipError_t e = ev ? hipEventSynchronize(ev) : hipSuccess;
        if (e == hipSuccess) e = hipMemcpyAsync(bp, packed, total, hipMemcpyDeviceToHost, s);
        if (e == hipSuccess) e = hipStreamSynchronize(s);
        if (e != hipSuccess) {
            release_bounce(c, bidx, false);
            c->err = std::string("device -> bounce buffer copy: ") + hipGetErrorString(e);
            return HA_RAG_EHIP;
        }
        host = bp;
    }
    if (tier == HA_RAG_TIER_PAGEABLE) {
        rc = before_host_write(c, sl.use[slot]);
        if (rc == HA_RAG_OK) std::memcpy(sl.ptr(slot), host, total);
    } else if (!c->direct()) {
        rc = write_full(c, sl.fd, host, total, sl.offset(slot));
    } else {
        std::memcpy(c->dio, host, total);
        std::memset(c->dio + total, 0, c->io_bytes(total) - total);
        rc = write_full(c, sl.fd, c->dio, c->io_bytes(total), sl.offset(slot));
    }
    if (via_bounce) release_bounce(c, bidx, false);
    return rc;
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

int ha_rag_pool_insert_external(ha_rag_ctx *c, uint64_t id, uint32_t part, uint32_t prec,
                                uint32_t n_tokens, const void *pinned)
{
    if (!c || prec >= HA_RAG_N_PREC || id == HA_RAG_NO_CHUNK || part > kPartV) return HA_RAG_EINVAL;
    if (!pinned || ((uintptr_t)pinned & 15u)) return HA_RAG_EINVAL;
    if (n_tokens == 0 || n_tokens > c->cfg.max_chunk_tokens) return HA_RAG_EINVAL;
    if (part == kPartKV && c->cfg.half_slots) return HA_RAG_EFORMAT;
    std::lock_guard<std::mutex> g(c->mu);
    size_t total;
    int rc = chunk_bytes_impl(c->cfg.n_layers, c->cfg.n_kv_heads, c->cfg.head_dim, prec,
                              c->group_of(prec), n_tokens, nullptr, nullptr, &total, part);
    if (rc) return rc;
    Slab &sl = c->slab[HA_RAG_TIER_PINNED][prec];
    if (!sl.registered()) return HA_RAG_ENOSPC;  // ha_rag_register_external first
    if (!sl.external) return HA_RAG_EINVAL;      // the library's own pinned slab holds this tag
    uint32_t ci;
    Chunk *ch = find_chunk(c, id, &ci);
    if (ch) {
        if (ch->slot[HA_RAG_TIER_PINNED] >= 0) return HA_RAG_EINVAL;
        if (ch->prec != prec || ch->n_tokens != n_tokens || ch->part != part) return HA_RAG_EFORMAT;
    }
    int32_t slot;
    if (!sl.free_slots.empty()) {
        slot = (int32_t)sl.free_slots.back();
        sl.free_slots.pop_back();
    } else {
        if (sl.n_slots == 0x7FFFFFFFu) return HA_RAG_ENOSPC;
        slot = (int32_t)sl.n_slots++;
        sl.use.emplace_back();
        sl.ext.push_back(nullptr);
    }
    sl.ext[(size_t)slot] = const_cast<uint8_t *>(static_cast<const uint8_t *>(pinned));
    if (!ch) {
        ci = new_chunk_entry(c);
        ch = &c->chunks[ci];
        ch->id = id;
        ch->prec = prec;
        ch->n_tokens = n_tokens;
        ch->part = part;
        ch->bytes = total;
        c->index.emplace(id, ci);
    }
    tier_attach(c, HA_RAG_TIER_PINNED, ci, slot);
    return HA_RAG_OK;
}

int ha_rag_pool_repoint_external(ha_rag_ctx *c, const uint64_t *ids, const void *const *pinned, size_t n)
{
    if (!c || (n && (!ids || !pinned))) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    for (size_t i = 0; i < n; ++i) {  // checks first: nothing changes unless every entry is good
        const Chunk *ch = find_chunk(c, ids[i]);
        if (!ch) return HA_RAG_ENOENT;
        if (ch->slot[HA_RAG_TIER_PINNED] < 0 || !c->slab[HA_RAG_TIER_PINNED][ch->prec].external)
            return HA_RAG_EINVAL;
        if (!pinned[i] || ((uintptr_t)pinned[i] & 15u)) return HA_RAG_EINVAL;
    }
    for (size_t i = 0; i < n; ++i) {
        const Chunk *ch = find_chunk(c, ids[i]);
        c->slab[HA_RAG_TIER_PINNED][ch->prec].ext[(size_t)ch->slot[HA_RAG_TIER_PINNED]] =
            const_cast<uint8_t *>(static_cast<const uint8_t *>(pinned[i]));
    }
    return HA_RAG_OK;
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
    std::unique_lock<std::mutex> g(c->mu);
    uint32_t ci;
    Chunk *ch = find_chunk(c, id, &ci);
    if (!ch || ch->slot[tier] < 0) return HA_RAG_ENOENT;
    // a running load may be writing this copy or reading it on the host: let it finish
    while (ch->pending[tier] || c->slab[tier][ch->prec].use[(size_t)ch->slot[tier]].host_readers) {
        c->cv.wait(g);
        ch = find_chunk(c, id, &ci);
        if (!ch || ch->slot[tier] < 0) return HA_RAG_ENOENT;
    }
    if (!ch->has_slower_copy(tier)) return HA_RAG_EINVAL;
    tier_detach(c, tier, ci);
    return HA_RAG_OK;
}

int ha_rag_pool_remove(ha_rag_ctx *c, uint64_t id)
{
    if (!c) return HA_RAG_EINVAL;
    std::unique_lock<std::mutex> g(c->mu);
    uint32_t ci;
    Chunk *ch = find_chunk(c, id, &ci);
    if (!ch) return HA_RAG_ENOENT;
    while (ch->in_calls) {  // a running load holds the entry: let it finish
        c->cv.wait(g);
        ch = find_chunk(c, id, &ci);
        if (!ch) return HA_RAG_ENOENT;
    }
    for (uint32_t t = 0; t < kTiers; ++t)
        if (ch->slot[t] >= 0) tier_detach(c, t, ci);
    c->index.erase(id);
    *ch = Chunk();
    ch->id = HA_RAG_NO_CHUNK;
    c->dead.push_back(ci);
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
        const uint32_t ci = new_chunk_entry(c);
        Chunk &ch = c->chunks[ci];
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

int ha_rag_forget_stream(ha_rag_ctx *c, void *stream)
{
    if (!c) return HA_RAG_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    std::unique_lock<std::mutex> g(c->mu);
    auto it = c->stream_done.find(s);
    if (it == c->stream_done.end()) return HA_RAG_OK;  // the library never enqueued anything there
    hipEvent_t ev = it->second;
    c->stream_done.erase(it);
    // Slots remember streams by handle, and a handle may come back for a new stream: take the
    // stream out of every slot's books.  What it enqueued is waited for here instead.
    for (uint32_t t = 0; t < kCacheTiers; ++t)
        for (uint32_t p = 0; p < HA_RAG_N_PREC; ++p)
            for (SlotUse &u : c->slab[t][p].use) {
                if (u.has_writer && u.writer == s) u.has_writer = false;
                u.readers.erase(std::remove(u.readers.begin(), u.readers.end(), s), u.readers.end());
            }
    g.unlock();
    if (!c->dry()) {
        hipError_t e = hipEventSynchronize(ev);
        (void)hipEventDestroy(ev);
        if (e != hipSuccess) {
            std::lock_guard<std::mutex> g2(c->mu);
            c->err = std::string("hipEventSynchronize: ") + hipGetErrorString(e);
            return HA_RAG_EHIP;
        }
    }
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

}  // extern "C"
