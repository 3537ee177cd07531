// The online load behind include/ha_rag.h (Algorithm 2 step 2 + decompression +
// concatenation): per-chunk lookup and placement, then the stream / event pipeline that
// overlaps file reads, host copies and host -> HBM copies with the dequantize kernel.
//
// Locking.  The context's mutex is held for bookkeeping and for enqueueing GPU work (both
// never block); it is released while the calling thread waits for an event or for its file /
// pageable bytes, which the context's I/O threads move in pieces.  So calls of several threads
// overlap their file reads with each other and with GPU work.  What a call has booked but not
// yet written is marked pending (other calls pass it over), what it reads on the host is
// counted in the slot (it is not evicted meanwhile), and chunk entries it holds by index are
// not removed meanwhile.
#include "ha_rag_internal.h"

#include <algorithm>
#include <cstring>
#include <memory>

using namespace ha_rag_host;

namespace {

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

// The host-side move of a chunk from its pageable or file copy into bounce buffer `bounce`,
// and on into the host slot a copy was placed in (dst2, nullable).  Called with the lock held:
// captures the addresses (the source slot's reader was counted when the action was decided).
std::shared_ptr<Transfer> make_transfer(ha_rag_ctx *c, const Chunk &ch, uint32_t tier, int32_t slot,
                                        uint8_t *bounce, uint8_t *dst2)
{
    auto t = std::make_shared<Transfer>();
    Slab &sl = c->slab[tier][ch.prec];
    if (tier == HA_RAG_TIER_PAGEABLE) {
        t->src = sl.ptr(slot);
    } else {
        t->fd = sl.fd;
        t->direct = c->direct();
        t->off = sl.offset(slot);
    }
    t->dst = bounce;
    t->dst2 = dst2;
    t->bytes = c->no_io() ? 0 : (size_t)ch.bytes;
    return t;
}

void done_reading(ha_rag_ctx *c, const Chunk &ch, uint32_t tier, int32_t slot)
{
    if (tier < kCacheTiers) --c->slab[tier][ch.prec].use[(size_t)slot].host_readers;
}

IoPool *io_pool(ha_rag_ctx *c)
{
    if (!c->io) c->io = io_pool_create(c->cfg.io_threads ? c->cfg.io_threads : 4u, c->direct());
    return c->io;
}

// Algorithm 2 step 2 for one chunk of a call: counts the access, touches the LRU order of the
// tier it is found in, and books a copy in the tier its rank's list names if that tier is
// faster than the one it was found in (floor_tier: no chunk is left in a tier slower than this;
// HA_RAG_TIER_DISK asks for nothing beyond the algorithm).  Fills the action, the trace entry and
// the statistics; moves no byte.
void alg2_step(ha_rag_ctx *c, uint32_t ci, uint32_t r, uint64_t off, uint64_t call, uint32_t floor_tier,
               Action &a, ha_rag_chunk_trace &tr, ha_rag_load_stats &st)
{
    const uint64_t D = c->cfg.head_dim;
    Chunk &ch = c->chunks[ci];
    ch.count += 1;
    const uint32_t found = (uint32_t)ch.fastest(call);
    a = Action{ci, r, off, Action::COLD, (uint8_t)found, ch.slot[found], HA_RAG_TIER_NONE, -1};
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
        uint32_t want = ch.rank == kNoRank ? HA_RAG_TIER_DISK : c->list_of(ch.rank);
        if (want > floor_tier) want = floor_tier;  // HA_RAG_TIER_DISK = no floor
        // a copy there that another running call is still writing: nothing to add
        if (want < found && c->slab[want][ch.prec].holds_copies() && ch.slot[want] < 0) {
            uint64_t ev;
            const int32_t slot = tier_acquire(c, want, ch.prec, &ev, call);
            if (slot >= 0) {
                tier_attach(c, want, ci, slot);
                ch.made_by[want] = call;
                ch.pending[want] = 1;  // until its bytes are in place (published by the call)
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
}

// What a call keeps about the chunks it works on, and how it lets go of them: entries it holds
// by index, host-side readers it counted, bounce buffers it reserved, copies it booked.  The
// destructor runs with the lock held; copies booked but never written leave the books again.
struct CallState {
    ha_rag_ctx *c;
    std::vector<Action> acts;
    std::vector<uint8_t> written;      // per action: its placed copy has been written / enqueued
    std::vector<uint8_t> reading;      // per action: counted as a host reader of its source slot
    std::vector<size_t> held_bounce;   // reserved by this call, not yet handed back
    std::vector<std::shared_ptr<Transfer>> moving;  // started on the I/O threads, not yet waited for
    explicit CallState(ha_rag_ctx *ctx) : c(ctx) {}
    void add(const Action &a)
    {
        acts.push_back(a);
        written.push_back(0);
        reading.push_back(0);
        Chunk &ch = c->chunks[a.ci];
        ++ch.in_calls;
        // A copy in pageable memory that the call will read on the host with the context
        // unlocked, and a copy that an earlier chunk of this call places and this one reads
        // afterwards: from now on nobody evicts them, neither another call nor a later chunk of
        // this one (which takes the next victim in LRU order instead).
        const bool host_read = a.kind == Action::COLD && a.src_tier == HA_RAG_TIER_PAGEABLE;
        if (host_read || a.kind == Action::HOT_LATE) {
            ++c->slab[a.src_tier][ch.prec].use[(size_t)a.src_slot].host_readers;
            reading.back() = 1;
        }
    }
    void publish(size_t k)  // the placed copy of action k holds its bytes (or its copy is enqueued)
    {
        const Action &a = acts[k];
        if (a.place_tier == HA_RAG_TIER_NONE || written[k]) return;
        written[k] = 1;
        Chunk &ch = c->chunks[a.ci];
        if (ch.slot[a.place_tier] == a.place_slot) ch.pending[a.place_tier] = 0;
    }
    void stop_reading(size_t k)
    {
        if (!reading[k]) return;
        reading[k] = 0;
        done_reading(c, c->chunks[acts[k].ci], acts[k].src_tier, acts[k].src_slot);
    }
    void drop_bounce(size_t b, bool copy_in_flight)
    {
        for (size_t i = 0; i < held_bounce.size(); ++i)
            if (held_bounce[i] == b) {
                held_bounce.erase(held_bounce.begin() + (long)i);
                break;
            }
        release_bounce(c, b, copy_in_flight);
    }
    ~CallState()
    {
        // a call that ends early: the I/O threads must be done with its buffers before they are
        // handed on (the transfers touch no context state, so waiting with the lock held is safe)
        for (const std::shared_ptr<Transfer> &t : moving) (void)t->wait();
        for (size_t k = 0; k < acts.size(); ++k) {
            const Action &a = acts[k];
            stop_reading(k);
            Chunk &ch = c->chunks[a.ci];
            if (a.place_tier != HA_RAG_TIER_NONE && !written[k] && ch.slot[a.place_tier] == a.place_slot) {
                ch.pending[a.place_tier] = 0;
                tier_detach(c, a.place_tier, a.ci);
            }
            --ch.in_calls;
        }
        for (size_t b : held_bounce) release_bounce(c, b, false);
        c->cv.notify_all();
    }
};

// A host move that must wait for its turn: it also fills a pinned / pageable slot (an earlier
// chunk of the call may still have to enqueue its read of the copy that slot held before: pass
// A has booked everything already), or it reads a copy that an earlier chunk of the call is
// still writing.
bool not_ahead(const ha_rag_ctx *c, const Action &a)
{
    if (a.place_tier == HA_RAG_TIER_PINNED || a.place_tier == HA_RAG_TIER_PAGEABLE) return true;
    return a.src_tier < kCacheTiers && c->chunks[a.ci].pending[a.src_tier] != 0;
}

// A chunk's bytes being moved into a bounce buffer by the I/O threads.
struct HostMove {
    size_t bounce = 0;
    std::shared_ptr<Transfer> t;
    bool started = false;
};

// Starts the host-side move of action k (source in pageable memory or a file).  Lock held on
// entry and on return; released while the calling thread waits for device work that still reads
// the buffers it is about to overwrite.  block: wait for a bounce buffer if other calls hold them
// all (otherwise *started stays false).
int start_host_move(ha_rag_ctx *c, std::unique_lock<std::mutex> &lk, CallState &cs, size_t k, bool block,
                    HostMove *hm)
{
    hipEvent_t bounce_ev = nullptr;
    if (!reserve_bounce(c, lk, block, &hm->bounce, &bounce_ev)) return HA_RAG_OK;
    cs.held_bounce.push_back(hm->bounce);
    const Action a = cs.acts[k];
    const Chunk &ch = c->chunks[a.ci];
    uint8_t *bp = c->bounce + hm->bounce * c->bounce_slot_bytes;
    uint8_t *dst2 = nullptr;
    std::vector<hipEvent_t> waits;
    if (bounce_ev) waits.push_back(bounce_ev);
    if (a.place_tier == HA_RAG_TIER_PINNED || a.place_tier == HA_RAG_TIER_PAGEABLE) {
        Slab &ds = c->slab[a.place_tier][ch.prec];
        take_host_write_events(c, ds.use[(size_t)a.place_slot], &waits);
        dst2 = ds.ptr(a.place_slot);
    }
    hm->t = make_transfer(c, ch, a.src_tier, a.src_slot, bp, dst2);
    IoPool *pool = io_pool(c);
    lk.unlock();
    hipError_t e = hipSuccess;
    if (!c->dry())
        for (hipEvent_t ev : waits)
            if (e == hipSuccess) e = hipEventSynchronize(ev);
    if (e == hipSuccess) io_pool_start(pool, hm->t);
    lk.lock();
    if (e != hipSuccess) {
        c->err = std::string("hipEventSynchronize: ") + hipGetErrorString(e);
        return HA_RAG_EHIP;
    }
    cs.moving.push_back(hm->t);
    hm->started = true;
    return HA_RAG_OK;
}

// Waits (lock released) until the bytes of action k are in its bounce buffer and in the host
// slot a copy was placed in; then that copy is published and the source slot let go of.
int finish_host_move(ha_rag_ctx *c, std::unique_lock<std::mutex> &lk, CallState &cs, size_t k, HostMove &hm)
{
    lk.unlock();
    const int rc = hm.t->wait();
    lk.lock();
    cs.moving.erase(std::find(cs.moving.begin(), cs.moving.end(), hm.t));
    cs.stop_reading(k);
    if (rc) {
        c->err = hm.t->err;
        return rc;
    }
    const Action &a = cs.acts[k];
    if (a.place_tier == HA_RAG_TIER_PINNED || a.place_tier == HA_RAG_TIER_PAGEABLE) cs.publish(k);
    return HA_RAG_OK;
}

int load_impl(ha_rag_ctx *c, std::unique_lock<std::mutex> &lk, const uint64_t *ids, const uint8_t *tags,
              const Request *reqs, uint32_t n_req, uint32_t n, hipStream_t s, ha_rag_load_stats *stats,
              ha_rag_chunk_trace *trace)
{
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
    CallState cs(c);
    cs.acts.reserve(n);
    // copies created by this call carry its number: they are not evicted again by this call
    const uint64_t call = ++c->call_seq;
    for (uint32_t r = 0; r < n_req; ++r) {
        const Request &rq = reqs[r];
        PlaneCursor cur(rq.base);
        for (uint32_t i = rq.begin; i < rq.end; ++i) {
            const uint32_t ci = cis[i];
            uint64_t off = 0;
            (void)cur.place(c->chunks[ci].part, c->chunks[ci].n_tokens, &off);  // checked above
            Action a;
            ha_rag_chunk_trace tr;
            alg2_step(c, ci, r, off, call, HA_RAG_TIER_DISK, a, tr, st);
            cs.add(a);
            if (trace) trace[i] = tr;
        }
    }
    const std::vector<Action> &acts = cs.acts;

    // ---- pass B: enqueue ---------------------------------------------------------
    // 1. one kernel over every chunk that is read where it lies: copies already resident in
    //    HBM, and pinned copies when the kernel reads pinned memory itself
    // 2. per cold chunk, in order: its bytes reach a staging slot (pinned source: one host ->
    //    HBM copy on a copy stream; pageable / file source: the I/O threads first move them
    //    into a bounce buffer, and into the pinned / pageable slot a copy was placed in, while
    //    this thread waits with the context unlocked), `stream` waits for that copy, kernel,
    //    copy into the HBM slab if the chunk was placed there, staging slot released.  The
    //    host moves of the next chunks are started ahead, as far as bounce buffers are free.
    // 3. one kernel over chunks whose copy was written in step 2
    std::vector<uint32_t> cold;
    for (uint32_t k = 0; k < acts.size(); ++k)
        if (acts[k].kind == Action::COLD) cold.push_back(k);
    const size_t n_stg = c->stg.size();

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

    std::vector<HostMove> moves(cold.size());
    size_t ahead = 0;  // cold chunks up to here have had their host move started (if they need one)
    auto needs_move = [&](size_t k) { return acts[cold[k]].src_tier >= HA_RAG_TIER_PAGEABLE; };

    for (size_t k = 0; k < cold.size(); ++k) {
        // host side: this chunk's move must run; later ones are started while buffers are free
        while (ahead < cold.size()) {
            if (!needs_move(ahead)) {
                ++ahead;
                continue;
            }
            const bool must = ahead <= k;
            if (!must && not_ahead(c, acts[cold[ahead]])) break;
            rc = start_host_move(c, lk, cs, cold[ahead], must, &moves[ahead]);
            if (rc) return rc;
            if (!moves[ahead].started) break;  // no free bounce buffer: later
            ++ahead;
        }
        if (needs_move(k)) {
            rc = finish_host_move(c, lk, cs, cold[k], moves[k]);
            if (rc) return rc;
        }
        // device side, enqueued in one go with the lock held
        const Action &a = acts[cold[k]];
        const Chunk &ch = c->chunks[a.ci];
        const size_t sidx = (size_t)(c->stg_next++ % n_stg);
        uint8_t *sp = c->staging + sidx * c->staging_slot_bytes;
        const uint8_t *src = needs_move(k) ? c->bounce + moves[k].bounce * c->bounce_slot_bytes
                                           : c->slab[HA_RAG_TIER_PINNED][ch.prec].ptr(a.src_slot);
        if (!c->dry()) {
            StagingSlot &ss = c->stg[sidx];
            hipStream_t cps = c->copy_streams[c->copy_rr++ % c->copy_streams.size()];
            if (ss.consumed_valid) HIPCHK(c, hipStreamWaitEvent(cps, ss.consumed, 0));
            if (a.src_tier == HA_RAG_TIER_PINNED) {
                SlotUse &u = c->slab[HA_RAG_TIER_PINNED][ch.prec].use[a.src_slot];
                if (u.has_writer) {  // a device -> host copy may still be filling the slot
                    rc = wait_for(c, cps, u.writer);
                    if (rc) return rc;
                }
                if (std::find(u.read_events.begin(), u.read_events.end(), ss.filled) == u.read_events.end())
                    u.read_events.push_back(ss.filled);  // at most one per staging slot
            }
            HIPCHK(c, hipMemcpyAsync(sp, src, ch.bytes, hipMemcpyHostToDevice, cps));
            HIPCHK(c, hipEventRecord(ss.filled, cps));
            if (needs_move(k)) HIPCHK(c, hipEventRecord(c->bnc[moves[k].bounce].h2d_done, cps));
            HIPCHK(c, hipStreamWaitEvent(s, ss.filled, 0));
        }
        if (needs_move(k)) cs.drop_bounce(moves[k].bounce, !c->dry());
        rc = push(c, batch, make_desc(c, ch, sp, reqs[a.req], a.tok_off), s, &st.n_kernel_launches);
        if (rc) return rc;
        rc = flush(c, batch, s, &st.n_kernel_launches);
        if (rc) return rc;
        if (a.place_tier == HA_RAG_TIER_HBM) {
            Slab &hs = c->slab[HA_RAG_TIER_HBM][ch.prec];
            rc = before_write(c, hs.use[a.place_slot], s);
            if (rc) return rc;
            if (!c->dry())
                HIPCHK(c, hipMemcpyAsync(hs.ptr(a.place_slot), sp, ch.bytes, hipMemcpyDeviceToDevice, s));
            // readers on other streams wait for this stream's event, which must cover the copy
            rc = mark_stream(c, s);
            if (rc) return rc;
            cs.publish(cold[k]);
        }
        if (!c->dry()) {
            HIPCHK(c, hipEventRecord(c->stg[sidx].consumed, s));
            c->stg[sidx].consumed_valid = true;
        }
    }

    for (size_t k = 0; k < acts.size(); ++k) {
        const Action &a = acts[k];
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
    if (stats) *stats = st;
    return HA_RAG_OK;
}


// Algorithm 2 step 2 without the decode: the same bookkeeping as a load, and the bytes of every
// copy it books are moved, but no cache is written.  A copy booked in HBM is filled by one
// host -> device copy straight into its slot (from the pinned copy, or from a bounce buffer that
// a pageable copy or a file was read into), so no staging slot is involved.
int place_impl(ha_rag_ctx *c, std::unique_lock<std::mutex> &lk, const uint64_t *ids, const uint8_t *tags,
               uint32_t n, uint32_t floor_tier, hipStream_t s, ha_rag_load_stats *stats,
               ha_rag_chunk_trace *trace)
{
    std::vector<uint32_t> cis(n);
    for (uint32_t i = 0; i < n; ++i) {
        Chunk *ch = find_chunk(c, ids[i], &cis[i]);
        if (!ch) return HA_RAG_ENOENT;
        if (tags && tags[i] != ch->prec) return HA_RAG_EFORMAT;
        const int f = ch->fastest();
        if (f < 0) return HA_RAG_ENOENT;
        if (f >= (int)HA_RAG_TIER_PAGEABLE &&
            (c->bnc.size() < 2 || c->io_bytes(ch->bytes) > c->bounce_slot_bytes))
            return HA_RAG_ENOSPC;
    }
    if (c->cfg.rerank_interval && c->n_loads && (c->n_loads % c->cfg.rerank_interval) == 0)
        rerank_locked(c);
    ++c->n_loads;

    ha_rag_load_stats st;
    std::memset(&st, 0, sizeof st);
    CallState cs(c);
    const uint64_t call = ++c->call_seq;
    for (uint32_t i = 0; i < n; ++i) {
        ha_rag_chunk_trace tr;
        Action a;
        alg2_step(c, cis[i], 0, 0, call, floor_tier, a, tr, st);
        cs.add(a);
        if (trace) trace[i] = tr;
    }
    const std::vector<Action> &acts = cs.acts;
    // the byte counters of a load do not apply: count what this call moves
    st.n_chunks = n;
    st.tokens = 0;
    st.bytes_h2d = st.bytes_d2d = st.packed_bytes_read = st.bf16_bytes_written = 0;
    st.bytes_disk_read = st.bytes_host_copied = 0;

    std::vector<uint32_t> todo;  // actions that place a copy
    for (uint32_t k = 0; k < n; ++k)
        if (acts[k].place_tier != HA_RAG_TIER_NONE) todo.push_back(k);
    std::vector<HostMove> moves(todo.size());
    size_t ahead = 0;
    auto needs_move = [&](size_t k) { return acts[todo[k]].src_tier >= HA_RAG_TIER_PAGEABLE; };

    for (size_t k = 0; k < todo.size(); ++k) {
        int rc;
        while (ahead < todo.size()) {
            if (!needs_move(ahead)) {
                ++ahead;
                continue;
            }
            const bool must = ahead <= k;
            if (!must && not_ahead(c, acts[todo[ahead]])) break;
            rc = start_host_move(c, lk, cs, todo[ahead], must, &moves[ahead]);
            if (rc) return rc;
            if (!moves[ahead].started) break;
            ++ahead;
        }
        const Action &a = acts[todo[k]];
        if (needs_move(k)) {
            rc = finish_host_move(c, lk, cs, todo[k], moves[k]);
            if (rc) return rc;
        }
        const Chunk &ch = c->chunks[a.ci];
        const uint8_t *src = nullptr;
        if (needs_move(k)) {
            if (a.src_tier == HA_RAG_TIER_PAGEABLE) st.bytes_host_copied += ch.bytes;
            else st.bytes_disk_read += ch.bytes;
            if (a.place_tier != HA_RAG_TIER_HBM) st.bytes_host_copied += ch.bytes;
            src = c->bounce + moves[k].bounce * c->bounce_slot_bytes;
        } else {
            src = c->slab[HA_RAG_TIER_PINNED][ch.prec].ptr(a.src_slot);
        }
        if (a.place_tier == HA_RAG_TIER_HBM) {
            Slab &hs = c->slab[HA_RAG_TIER_HBM][ch.prec];
            rc = before_write(c, hs.use[a.place_slot], s);
            if (rc) return rc;
            if (a.src_tier == HA_RAG_TIER_PINNED) {
                SlotUse &pu = c->slab[HA_RAG_TIER_PINNED][ch.prec].use[a.src_slot];
                if (pu.has_writer) {  // a device -> host copy may still be filling the slot
                    rc = wait_for(c, s, pu.writer);
                    if (rc) return rc;
                }
                if (std::find(pu.readers.begin(), pu.readers.end(), s) == pu.readers.end()) pu.readers.push_back(s);
            }
            if (!c->dry()) {
                HIPCHK(c, hipMemcpyAsync(hs.ptr(a.place_slot), src, ch.bytes, hipMemcpyHostToDevice, s));
                if (needs_move(k)) HIPCHK(c, hipEventRecord(c->bnc[moves[k].bounce].h2d_done, s));
            }
            // Readers of the new copy on other streams, and the host before it overwrites the
            // pinned source (a later chunk of this call may have been given that slot: pass A
            // has already booked everything), wait on the stream's event, which must therefore
            // be recorded after this copy, not at the end of the call.
            rc = mark_stream(c, s);
            if (rc) return rc;
            st.bytes_h2d += ch.bytes;
            cs.publish(todo[k]);
        }
        if (needs_move(k)) cs.drop_bounce(moves[k].bounce, a.place_tier == HA_RAG_TIER_HBM && !c->dry());
    }
    int rc = mark_stream(c, s);
    if (rc) return rc;
    if (stats) *stats = st;
    return HA_RAG_OK;
}

}  // namespace

extern "C" {

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

int ha_rag_load_chunks(ha_rag_ctx *c, const uint64_t *ids, const uint8_t *tags, uint32_t n,
                       void *out, uint64_t cap_tokens, uint64_t tok_base, void *stream,
                       ha_rag_load_stats *stats, ha_rag_chunk_trace *trace)
{
    if (!c || (n && !ids) || n > HA_RAG_MAX_REQUEST_CHUNKS) return HA_RAG_EINVAL;
    if (cap_tokens * (uint64_t)c->cfg.head_dim > 0x7FFFFFFFFFFFull) return HA_RAG_EINVAL;
    std::unique_lock<std::mutex> g(c->mu);
    Request rq{0, n, static_cast<uint8_t *>(out), cap_tokens, tok_base, nullptr};
    return load_impl(c, g, ids, tags, &rq, 1, n, (hipStream_t)stream, stats, trace);
}

int ha_rag_load_chunks_paged(ha_rag_ctx *c, const uint64_t *ids, const uint8_t *tags, uint32_t n,
                             const ha_rag_paged_cache *cache, uint64_t tok_base, void *stream,
                             ha_rag_load_stats *stats, ha_rag_chunk_trace *trace)
{
    if (!c || !cache || (n && !ids) || n > HA_RAG_MAX_REQUEST_CHUNKS) return HA_RAG_EINVAL;
    uint64_t cap = 0;
    int rc = check_paged(c, cache, &cap);
    if (rc) return rc;
    std::unique_lock<std::mutex> g(c->mu);
    Request rq{0, n, nullptr, cap, tok_base, cache};
    return load_impl(c, g, ids, tags, &rq, 1, n, (hipStream_t)stream, stats, trace);
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
    std::unique_lock<std::mutex> g(c->mu);
    return load_impl(c, g, ids, tags, reqs.data(), n_requests, n, (hipStream_t)stream, stats, trace);
}

int ha_rag_place_chunks(ha_rag_ctx *c, const uint64_t *ids, const uint8_t *tags, uint32_t n,
                        uint32_t flags, void *stream, ha_rag_load_stats *stats,
                        ha_rag_chunk_trace *trace)
{
    if (!c || (n && !ids) || n > HA_RAG_MAX_REQUEST_CHUNKS || (flags & ~(uint32_t)HA_RAG_PLACE_DEVICE_VISIBLE))
        return HA_RAG_EINVAL;
    std::unique_lock<std::mutex> g(c->mu);
    return place_impl(c, g, ids, tags, n,
                      (flags & HA_RAG_PLACE_DEVICE_VISIBLE) ? HA_RAG_TIER_PINNED : HA_RAG_TIER_DISK,
                      (hipStream_t)stream, stats, trace);
}

}  // extern "C"
