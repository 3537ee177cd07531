// Host runtime behind include/ha_rag.h: pool slabs, hotness counters and ranks
// (Algorithm 1 steps 1-2), the tier lookup / promotion / LRU of Algorithm 2 for
// the two fast tiers (GPU memory and pinned host memory), and the stream/event
// pipeline that overlaps pinned -> HBM copies with the dequantize kernel.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <list>
#include <mutex>
#include <new>
#include <string>
#include <unordered_map>
#include <vector>

#include "../../include/ha_rag.h"
#include "ha_rag_kernels.h"

using namespace ha_rag;

namespace {

constexpr uint64_t kPPM = 1000000ull;
thread_local std::string g_create_err;  // why the last ha_rag_create on this thread failed
constexpr uint32_t kNoRank = UINT32_MAX;

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
                     uint32_t T, size_t *payload, size_t *meta, size_t *total)
{
    if (prec >= HA_RAG_N_PREC || L == 0 || H == 0 || D == 0 || (D % 8u)) return HA_RAG_EFORMAT;
    if (has_meta(prec) && (!valid_group(group) || (D % group))) return HA_RAG_EFORMAT;
    const uint64_t n_e = (uint64_t)T * D;
    if (n_e > 0x7FFFFFFFull) return HA_RAG_EINVAL;
    const uint64_t nblk = (n_e + kBlockElems - 1) / kBlockElems;
    const uint64_t tiles = 2ull * L * H;
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
    uint64_t bytes = 0;
    int32_t slot[2] = {-1, -1};  // per tier
    uint64_t count = 0;
    uint32_t rank = kNoRank;
    uint64_t last_use = 0;       // global sequence number of the last HBM access
    std::list<uint32_t>::iterator lru_it;
};

// Which streams touched a slot last, so that a different stream can be made to
// wait before it overwrites (or first reads) the slot.
struct SlotUse {
    hipStream_t writer = nullptr;
    bool has_writer = false;
    std::vector<hipStream_t> readers;
};

struct Slab {
    uint8_t *base = nullptr;
    size_t slot_bytes = 0;
    uint32_t n_slots = 0;
    std::vector<uint32_t> free_slots;  // stack
    std::vector<SlotUse> use;
    std::list<uint32_t> lru;           // chunk indices resident here, least recent first
    bool registered() const { return base != nullptr; }
    uint8_t *ptr(int32_t s) const { return base + (size_t)s * slot_bytes; }
};

struct StagingSlot {
    hipEvent_t filled = nullptr, consumed = nullptr;
    bool consumed_valid = false;
};

}  // namespace

struct ha_rag_ctx {
    ha_rag_config cfg{};
    uint32_t n_tiles = 0;
    std::mutex mu;
    std::string hip_err;

    std::vector<Chunk> chunks;
    std::unordered_map<uint64_t, uint32_t> index;
    Slab slab[2][HA_RAG_N_PREC];

    uint32_t gpu_bound = 0;  // ranks below this are GPU_LIST
    uint64_t n_loads = 0, use_seq = 0;

    uint8_t *staging = nullptr;
    size_t staging_slot_bytes = 0;
    std::vector<StagingSlot> stg;
    uint64_t stg_next = 0;

    std::vector<hipStream_t> copy_streams;
    uint64_t copy_rr = 0;
    std::unordered_map<hipStream_t, hipEvent_t> stream_done;

    K1Launch launch{64, 1, 2, true, true};

    uint32_t group_of(uint32_t prec) const
    {
        return prec == HA_RAG_PREC_INT8 ? cfg.group_int8 : prec == HA_RAG_PREC_INT4 ? cfg.group_int4 : 0;
    }
    bool dry() const { return cfg.dry_run != 0; }
};

namespace {

#define HIPCHK(ctx, call)                                                              \
    do {                                                                               \
        hipError_t e_ = (call);                                                        \
        if (e_ != hipSuccess) {                                                        \
            (ctx)->hip_err = std::string(#call) + ": " + hipGetErrorString(e_);        \
            return HA_RAG_EHIP;                                                        \
        }                                                                              \
    } while (0)

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

Chunk *find_chunk(ha_rag_ctx *c, uint64_t id, uint32_t *idx = nullptr)
{
    auto it = c->index.find(id);
    if (it == c->index.end()) return nullptr;
    if (idx) *idx = it->second;
    return &c->chunks[it->second];
}

void hbm_touch(ha_rag_ctx *c, uint32_t ci)
{
    Chunk &ch = c->chunks[ci];
    Slab &sl = c->slab[HA_RAG_TIER_HBM][ch.prec];
    sl.lru.splice(sl.lru.end(), sl.lru, ch.lru_it);  // most recent at the back
    ch.last_use = ++c->use_seq;
}

void hbm_attach(ha_rag_ctx *c, uint32_t ci, int32_t slot)
{
    Chunk &ch = c->chunks[ci];
    Slab &sl = c->slab[HA_RAG_TIER_HBM][ch.prec];
    ch.slot[HA_RAG_TIER_HBM] = slot;
    ch.lru_it = sl.lru.insert(sl.lru.end(), ci);
    ch.last_use = ++c->use_seq;
}

void hbm_detach(ha_rag_ctx *c, uint32_t ci)
{
    Chunk &ch = c->chunks[ci];
    Slab &sl = c->slab[HA_RAG_TIER_HBM][ch.prec];
    sl.lru.erase(ch.lru_it);
    sl.free_slots.push_back((uint32_t)ch.slot[HA_RAG_TIER_HBM]);
    ch.slot[HA_RAG_TIER_HBM] = -1;
}

// A free HBM slot of the slab for `prec`, evicting the least recently used chunk
// that has a pinned master if the slab is full ("put C_i in queueGPU with LRU").
// Returns -1 if nothing can be freed.  *evicted receives the dropped id.  Chunks
// flagged in `keep` (indexed like ctx->chunks) are passed over: a copy that the
// running call has itself just created is not dropped again by the same call,
// because a later read of it may already be planned.
int32_t hbm_acquire(ha_rag_ctx *c, uint32_t prec, uint64_t *evicted,
                    const std::vector<uint8_t> *keep = nullptr)
{
    Slab &sl = c->slab[HA_RAG_TIER_HBM][prec];
    *evicted = HA_RAG_NO_CHUNK;
    if (!sl.registered()) return -1;
    if (sl.free_slots.empty()) {
        for (uint32_t ci : sl.lru) {
            if (keep && (*keep)[ci]) continue;
            if (c->chunks[ci].slot[HA_RAG_TIER_PINNED] >= 0) {
                *evicted = c->chunks[ci].id;
                hbm_detach(c, ci);
                break;
            }
        }
        if (sl.free_slots.empty()) return -1;
    }
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
    c->gpu_bound = (uint32_t)std::min<uint64_t>(n, ((uint64_t)c->cfg.tau_gpu_ppm * n) / kPPM);
}

struct Request {
    uint32_t begin, end;
    uint8_t *out;
    uint64_t cap, base;
};

// What pass A decided for one chunk of a load.
struct Action {
    uint32_t ci;
    uint32_t req;
    uint64_t tok_off;
    enum Kind { HOT_EARLY, HOT_LATE, COLD } kind;
    int32_t promote_slot;  // HBM slot to fill from staging, or -1
    int32_t hbm_slot;      // slot read by a HOT_* action, as of the moment it was decided
                           // (a later chunk of the same call may evict this one)
};

K1Chunk make_desc(const ha_rag_ctx *c, const Chunk &ch, const uint8_t *src, const Request &rq,
                  uint64_t tok_off)
{
    K1Chunk d;
    const uint64_t D = c->cfg.head_dim;
    d.src = src;
    d.out = rq.out + tok_off * D * 2ull;
    d.out_tile_stride = rq.cap * D * 2ull;
    d.n_tokens = ch.n_tokens;
    const uint32_t g = c->group_of(ch.prec);
    d.fmt = ch.prec | ((g ? log2u(g) : 0u) << 8);
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

void init_batch(const ha_rag_ctx *c, Batch &b)
{
    b.p.n_tiles = c->n_tiles;
    b.p.head_dim = c->cfg.head_dim;
    b.p.n_chunks = 0;
    b.p.total_items = 0;
}

int load_impl(ha_rag_ctx *c, const uint64_t *ids, const uint8_t *tags, const Request *reqs,
              uint32_t n_req, uint32_t n, hipStream_t s, ha_rag_load_stats *stats,
              ha_rag_chunk_trace *trace)
{
    const uint64_t D = c->cfg.head_dim;
    // ---- checks: nothing changes before all of them pass --------------------
    std::vector<uint32_t> cis(n);
    bool any_cold = false;
    for (uint32_t r = 0; r < n_req; ++r) {
        const Request &rq = reqs[r];
        if (rq.end < rq.begin || rq.end > n) return HA_RAG_EINVAL;
        if (rq.end > rq.begin && (rq.out == nullptr || ((uintptr_t)rq.out & 15u))) return HA_RAG_EINVAL;
        uint64_t tok = 0;
        for (uint32_t i = rq.begin; i < rq.end; ++i) {
            Chunk *ch = find_chunk(c, ids[i], &cis[i]);
            if (!ch) return HA_RAG_ENOENT;
            if (tags && tags[i] != ch->prec) return HA_RAG_EFORMAT;
            if (ch->slot[HA_RAG_TIER_HBM] < 0) {
                any_cold = true;
                if (c->stg.size() < 2 || ch->bytes > c->staging_slot_bytes) return HA_RAG_ENOSPC;
            }
            tok += ch->n_tokens;
        }
        if (rq.base > rq.cap || tok > rq.cap - rq.base) return HA_RAG_ENOSPC;
    }
    (void)any_cold;

    if (c->cfg.rerank_interval && c->n_loads && (c->n_loads % c->cfg.rerank_interval) == 0)
        rerank_locked(c);
    ++c->n_loads;

    ha_rag_load_stats st;
    std::memset(&st, 0, sizeof st);
    st.n_chunks = n;

    // ---- pass A: Algorithm 2 step 2, chunk by chunk, in request order ---------
    std::vector<Action> acts;
    acts.reserve(n);
    std::vector<uint8_t> written_now(c->chunks.size(), 0);  // HBM copy created by this call
    for (uint32_t r = 0; r < n_req; ++r) {
        const Request &rq = reqs[r];
        uint64_t off = rq.base;
        for (uint32_t i = rq.begin; i < rq.end; ++i) {
            const uint32_t ci = cis[i];
            Chunk &ch = c->chunks[ci];
            ch.count += 1;
            Action a{ci, r, off, Action::COLD, -1, -1};
            ha_rag_chunk_trace tr;
            std::memset(&tr, 0, sizeof tr);
            tr.tok_off = off;
            tr.evicted_id = HA_RAG_NO_CHUNK;
            if (ch.slot[HA_RAG_TIER_HBM] >= 0) {  // C_i in queueGPU
                hbm_touch(c, ci);
                a.kind = written_now[ci] ? Action::HOT_LATE : Action::HOT_EARLY;
                a.hbm_slot = ch.slot[HA_RAG_TIER_HBM];
                tr.found_tier = HA_RAG_TIER_HBM;
                ++st.n_hbm_hits;
            } else {                               // C_i in queuePIN
                tr.found_tier = HA_RAG_TIER_PINNED;
                ++st.n_pinned_hits;
                st.bytes_h2d += ch.bytes;
                if (ch.rank < c->gpu_bound && c->slab[HA_RAG_TIER_HBM][ch.prec].registered()) {
                    uint64_t ev;
                    const int32_t slot = hbm_acquire(c, ch.prec, &ev, &written_now);
                    if (slot >= 0) {
                        hbm_attach(c, ci, slot);
                        written_now[ci] = 1;
                        a.promote_slot = slot;
                        tr.promoted = 1;
                        tr.evicted_id = ev;
                        ++st.n_promoted;
                        st.bytes_d2d += ch.bytes;
                        if (ev != HA_RAG_NO_CHUNK) ++st.n_evicted;
                    } else {
                        tr.promote_skipped = 1;
                        ++st.n_promote_skipped;
                    }
                }
            }
            st.tokens += ch.n_tokens;
            st.packed_bytes_read += ch.bytes;
            st.bf16_bytes_written += (uint64_t)ch.n_tokens * c->n_tiles * D * 2ull;
            off += ch.n_tokens;
            acts.push_back(a);
            if (trace) trace[i] = tr;
        }
    }

    // ---- pass B: enqueue ---------------------------------------------------------
    // 1. copies of the first cold chunks (as many as there are staging slots)
    // 2. one kernel over every chunk that was already resident in HBM
    // 3. per cold chunk: wait for its copy, kernel, promotion copy, release the
    //    staging slot, start the copy of the cold chunk that reuses it
    // 4. one kernel over chunks whose HBM copy was written in step 3
    std::vector<uint32_t> cold;
    for (uint32_t k = 0; k < acts.size(); ++k)
        if (acts[k].kind == Action::COLD) cold.push_back(k);
    const size_t n_stg = c->stg.size();
    std::vector<size_t> cold_slot(cold.size());

    auto start_copy = [&](size_t k) -> int {
        const Action &a = acts[cold[k]];
        const Chunk &ch = c->chunks[a.ci];
        const size_t sidx = (size_t)(c->stg_next++ % n_stg);
        cold_slot[k] = sidx;
        if (c->dry()) return HA_RAG_OK;
        StagingSlot &ss = c->stg[sidx];
        hipStream_t cs = c->copy_streams[c->copy_rr++ % c->copy_streams.size()];
        if (ss.consumed_valid) HIPCHK(c, hipStreamWaitEvent(cs, ss.consumed, 0));
        const Slab &ps = c->slab[HA_RAG_TIER_PINNED][ch.prec];
        HIPCHK(c, hipMemcpyAsync(c->staging + sidx * c->staging_slot_bytes,
                                 ps.ptr(ch.slot[HA_RAG_TIER_PINNED]), ch.bytes,
                                 hipMemcpyHostToDevice, cs));
        HIPCHK(c, hipEventRecord(ss.filled, cs));
        return HA_RAG_OK;
    };

    size_t copies_started = 0;
    for (; copies_started < cold.size() && copies_started < n_stg; ++copies_started) {
        int rc = start_copy(copies_started);
        if (rc) return rc;
    }

    Batch batch;
    init_batch(c, batch);
    for (const Action &a : acts) {
        if (a.kind != Action::HOT_EARLY) continue;
        const Chunk &ch = c->chunks[a.ci];
        Slab &hs = c->slab[HA_RAG_TIER_HBM][ch.prec];
        int rc = before_read(c, hs.use[a.hbm_slot], s);
        if (rc) return rc;
        rc = push(c, batch, make_desc(c, ch, hs.ptr(a.hbm_slot), reqs[a.req], a.tok_off), s,
                  &st.n_kernel_launches);
        if (rc) return rc;
    }
    int rc = flush(c, batch, s, &st.n_kernel_launches);
    if (rc) return rc;

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
        if (a.promote_slot >= 0) {
            Slab &hs = c->slab[HA_RAG_TIER_HBM][ch.prec];
            rc = before_write(c, hs.use[a.promote_slot], s);
            if (rc) return rc;
            if (!c->dry())
                HIPCHK(c, hipMemcpyAsync(hs.ptr(a.promote_slot), sp, ch.bytes,
                                         hipMemcpyDeviceToDevice, s));
        }
        if (!c->dry()) {
            HIPCHK(c, hipEventRecord(c->stg[sidx].consumed, s));
            c->stg[sidx].consumed_valid = true;
        }
        if (copies_started < cold.size()) {
            rc = start_copy(copies_started++);
            if (rc) return rc;
        }
    }

    for (const Action &a : acts) {
        if (a.kind != Action::HOT_LATE) continue;
        const Chunk &ch = c->chunks[a.ci];
        // `keep` in pass A guarantees the copy written by this call is still in its slot
        if (ch.slot[HA_RAG_TIER_HBM] != a.hbm_slot) return HA_RAG_EINVAL;
        Slab &hs = c->slab[HA_RAG_TIER_HBM][ch.prec];
        rc = before_read(c, hs.use[a.hbm_slot], s);
        if (rc) return rc;
        rc = push(c, batch, make_desc(c, ch, hs.ptr(a.hbm_slot), reqs[a.req], a.tok_off), s,
                  &st.n_kernel_launches);
        if (rc) return rc;
    }
    rc = flush(c, batch, s, &st.n_kernel_launches);
    if (rc) return rc;
    rc = mark_stream(c, s);
    if (rc) return rc;
    if (stats) *stats = st;
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
    case HA_RAG_ENOSPC: return "no space (pool slab, staging or output cache)";
    case HA_RAG_EFORMAT: return "precision tag / group / shape mismatch";
    case HA_RAG_EHIP: return "HIP call failed";
    default: return "unknown error code";
    }
}

const char *ha_rag_version(void) { return "ha_rag 0.1 (gfx950)"; }

int ha_rag_create(const ha_rag_config *cfg, ha_rag_ctx **out)
{
    if (!cfg || !out) return HA_RAG_EINVAL;
    *out = nullptr;
    if (cfg->n_layers == 0 || cfg->n_kv_heads == 0 || cfg->max_chunk_tokens == 0) return HA_RAG_EINVAL;
    if (cfg->head_dim == 0 || (cfg->head_dim % 8u)) return HA_RAG_EFORMAT;
    if (!valid_group(cfg->group_int8) || !valid_group(cfg->group_int4)) return HA_RAG_EFORMAT;
    if ((cfg->head_dim % cfg->group_int8) || (cfg->head_dim % cfg->group_int4)) return HA_RAG_EFORMAT;
    if (cfg->tau_gpu_ppm > kPPM || cfg->n_copy_streams > 8) return HA_RAG_EINVAL;
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
    }
    delete c;
    return HA_RAG_OK;
}

const char *ha_rag_last_hip_error(ha_rag_ctx *c)
{
    return c ? c->hip_err.c_str() : g_create_err.c_str();
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

int ha_rag_quantize_chunk(ha_rag_ctx *c, const void *src, uint32_t n_tokens, uint32_t prec,
                          uint32_t group, void *dst, uint32_t *saturated, void *stream)
{
    if (!c || !src || !dst) return HA_RAG_EINVAL;
    if (((uintptr_t)src & 15u) || ((uintptr_t)dst & 15u) || ((uintptr_t)saturated & 3u)) return HA_RAG_EINVAL;
    size_t total;
    int rc = chunk_bytes_impl(c->cfg.n_layers, c->cfg.n_kv_heads, c->cfg.head_dim, prec, group,
                              n_tokens, nullptr, nullptr, &total);
    if (rc) return rc;
    if (c->dry()) return HA_RAG_OK;
    std::lock_guard<std::mutex> g(c->mu);
    HIPCHK(c, launch_k2(src, dst, c->n_tiles, c->cfg.head_dim, n_tokens, prec,
                        has_meta(prec) ? group : 32u, saturated, (hipStream_t)stream));
    return HA_RAG_OK;
}

int ha_rag_load_packed(ha_rag_ctx *c, const ha_rag_packed_chunk *chunks, uint32_t n, void *out,
                       uint64_t cap_tokens, uint64_t tok_base, void *stream)
{
    if (!c || (n && (!chunks || !out)) || n > HA_RAG_MAX_REQUEST_CHUNKS) return HA_RAG_EINVAL;
    if ((uintptr_t)out & 15u) return HA_RAG_EINVAL;
    const uint64_t D = c->cfg.head_dim;
    uint64_t tok = 0;
    for (uint32_t i = 0; i < n; ++i) {
        const ha_rag_packed_chunk &pc = chunks[i];
        int rc = chunk_bytes_impl(c->cfg.n_layers, c->cfg.n_kv_heads, c->cfg.head_dim, pc.prec,
                                  pc.group, pc.n_tokens, nullptr, nullptr, nullptr);
        if (rc) return rc;
        if (pc.n_tokens && (!pc.packed || ((uintptr_t)pc.packed & 15u))) return HA_RAG_EINVAL;
        tok += pc.n_tokens;
    }
    if (tok_base > cap_tokens || tok > cap_tokens - tok_base) return HA_RAG_ENOSPC;
    if (cap_tokens * D > 0x7FFFFFFFFFFFull) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    Batch batch;
    init_batch(c, batch);
    uint64_t off = tok_base;
    for (uint32_t i = 0; i < n; ++i) {
        const ha_rag_packed_chunk &pc = chunks[i];
        if (pc.n_tokens == 0) continue;
        K1Chunk d;
        d.src = static_cast<const uint8_t *>(pc.packed);
        d.out = static_cast<uint8_t *>(out) + off * D * 2ull;
        d.out_tile_stride = cap_tokens * D * 2ull;
        d.n_tokens = pc.n_tokens;
        d.fmt = pc.prec | ((has_meta(pc.prec) ? log2u(pc.group) : 0u) << 8);
        int rc = push(c, batch, d, (hipStream_t)stream, nullptr);
        if (rc) return rc;
        off += pc.n_tokens;
    }
    return flush(c, batch, (hipStream_t)stream, nullptr);
}

int ha_rag_register_slab(ha_rag_ctx *c, uint32_t tier, uint32_t prec, void *base, size_t bytes)
{
    if (!c || !base || tier > HA_RAG_TIER_PINNED || prec >= HA_RAG_N_PREC) return HA_RAG_EINVAL;
    if ((uintptr_t)base & 255u) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    Slab &sl = c->slab[tier][prec];
    if (sl.registered()) return HA_RAG_EINVAL;
    size_t total;
    int rc = chunk_bytes_impl(c->cfg.n_layers, c->cfg.n_kv_heads, c->cfg.head_dim, prec,
                              c->group_of(prec), c->cfg.max_chunk_tokens, nullptr, nullptr, &total);
    if (rc) return rc;
    const size_t slot = (total + 255u) & ~(size_t)255u;
    if (bytes < slot) return HA_RAG_EINVAL;
    const size_t n_slots = bytes / slot;
    if (n_slots > 0x7FFFFFFFu) return HA_RAG_EINVAL;
    sl.base = static_cast<uint8_t *>(base);
    sl.slot_bytes = slot;
    sl.n_slots = (uint32_t)n_slots;
    sl.use.assign(n_slots, SlotUse());
    sl.free_slots.resize(n_slots);
    for (size_t i = 0; i < n_slots; ++i) sl.free_slots[i] = (uint32_t)(n_slots - 1 - i);  // slot 0 first
    return HA_RAG_OK;
}

int ha_rag_register_staging(ha_rag_ctx *c, void *base, size_t bytes)
{
    if (!c || !base || ((uintptr_t)base & 255u)) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    if (c->staging) return HA_RAG_EINVAL;
    size_t slot = 0;
    for (uint32_t p = 0; p < HA_RAG_N_PREC; ++p)
        slot = std::max(slot, c->slab[HA_RAG_TIER_PINNED][p].slot_bytes);
    if (slot == 0) return HA_RAG_EINVAL;  // register the pinned slabs first
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

int ha_rag_pool_insert(ha_rag_ctx *c, uint64_t id, uint32_t prec, uint32_t n_tokens,
                       const void *packed, int packed_is_device, uint32_t tier, void *stream)
{
    if (!c || tier > HA_RAG_TIER_PINNED || prec >= HA_RAG_N_PREC || id == HA_RAG_NO_CHUNK) return HA_RAG_EINVAL;
    if (n_tokens == 0 || n_tokens > c->cfg.max_chunk_tokens) return HA_RAG_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    std::lock_guard<std::mutex> g(c->mu);
    Slab &sl = c->slab[tier][prec];
    if (!sl.registered()) return HA_RAG_ENOSPC;
    size_t total;
    int rc = chunk_bytes_impl(c->cfg.n_layers, c->cfg.n_kv_heads, c->cfg.head_dim, prec,
                              c->group_of(prec), n_tokens, nullptr, nullptr, &total);
    if (rc) return rc;
    uint32_t ci;
    Chunk *ch = find_chunk(c, id, &ci);
    if (ch) {
        if (ch->slot[tier] >= 0) return HA_RAG_EINVAL;
        if (ch->prec != prec || ch->n_tokens != n_tokens) return HA_RAG_EFORMAT;
    }
    int32_t slot;
    if (tier == HA_RAG_TIER_HBM) {
        uint64_t ev;
        slot = hbm_acquire(c, prec, &ev);
        if (slot < 0) return HA_RAG_ENOSPC;
    } else {
        if (sl.free_slots.empty()) return HA_RAG_ENOSPC;
        slot = (int32_t)sl.free_slots.back();
        sl.free_slots.pop_back();
    }
    if (!ch) {
        ci = (uint32_t)c->chunks.size();
        c->chunks.emplace_back();
        ch = &c->chunks.back();
        ch->id = id;
        ch->prec = prec;
        ch->n_tokens = n_tokens;
        ch->bytes = total;
        c->index.emplace(id, ci);
    }
    if (tier == HA_RAG_TIER_HBM) hbm_attach(c, ci, slot);
    else ch->slot[tier] = slot;
    if (packed && !c->dry()) {
        rc = before_write(c, sl.use[slot], s);
        if (rc) return rc;
        if (tier == HA_RAG_TIER_HBM) {
            HIPCHK(c, hipMemcpyAsync(sl.ptr(slot), packed, total,
                                     packed_is_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, s));
        } else if (packed_is_device) {
            HIPCHK(c, hipMemcpyAsync(sl.ptr(slot), packed, total, hipMemcpyDeviceToHost, s));
        } else {
            std::memcpy(sl.ptr(slot), packed, total);
        }
        rc = mark_stream(c, s);
        if (rc) return rc;
    }
    return HA_RAG_OK;
}

int ha_rag_pool_slot(ha_rag_ctx *c, uint64_t id, uint32_t tier, void **ptr, size_t *bytes)
{
    if (!c || tier > HA_RAG_TIER_PINNED) return HA_RAG_EINVAL;
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
    const int32_t slot = hbm_acquire(c, ch->prec, &ev);
    if (slot < 0) return HA_RAG_ENOSPC;
    hbm_attach(c, ci, slot);
    if (!c->dry()) {
        Slab &hs = c->slab[HA_RAG_TIER_HBM][ch->prec];
        int rc = before_write(c, hs.use[slot], s);
        if (rc) return rc;
        HIPCHK(c, hipMemcpyAsync(hs.ptr(slot),
                                 c->slab[HA_RAG_TIER_PINNED][ch->prec].ptr(ch->slot[HA_RAG_TIER_PINNED]),
                                 ch->bytes, hipMemcpyHostToDevice, s));
        rc = mark_stream(c, s);
        if (rc) return rc;
    }
    return HA_RAG_OK;
}

int ha_rag_pool_evict(ha_rag_ctx *c, uint64_t id)
{
    if (!c) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    uint32_t ci;
    Chunk *ch = find_chunk(c, id, &ci);
    if (!ch || ch->slot[HA_RAG_TIER_HBM] < 0) return HA_RAG_ENOENT;
    if (ch->slot[HA_RAG_TIER_PINNED] < 0) return HA_RAG_EINVAL;
    hbm_detach(c, ci);
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
    info->in_hbm = ch->slot[HA_RAG_TIER_HBM] >= 0;
    info->in_pinned = ch->slot[HA_RAG_TIER_PINNED] >= 0;
    info->rank = ch->rank;
    info->count = ch->count;
    info->bytes = ch->bytes;
    if (info->in_hbm) info->hbm_ptr = c->slab[HA_RAG_TIER_HBM][ch->prec].ptr(ch->slot[HA_RAG_TIER_HBM]);
    if (info->in_pinned)
        info->pinned_ptr = c->slab[HA_RAG_TIER_PINNED][ch->prec].ptr(ch->slot[HA_RAG_TIER_PINNED]);
    return HA_RAG_OK;
}

int ha_rag_pool_hbm_lru(ha_rag_ctx *c, uint64_t *ids, size_t cap, size_t *n)
{
    if (!c || !n || (cap && !ids)) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    std::vector<const Chunk *> v;
    for (const Chunk &ch : c->chunks)
        if (ch.slot[HA_RAG_TIER_HBM] >= 0) v.push_back(&ch);
    std::sort(v.begin(), v.end(), [](const Chunk *a, const Chunk *b) { return a->last_use < b->last_use; });
    *n = std::min(cap, v.size());
    for (size_t i = 0; i < *n; ++i) ids[i] = v[i]->id;
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
    Request rq{0, n, static_cast<uint8_t *>(out), cap_tokens, tok_base};
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
                          cap_tokens[r], tok_base ? tok_base[r] : 0};
    }
    std::lock_guard<std::mutex> g(c->mu);
    return load_impl(c, ids, tags, reqs.data(), n_requests, n, (hipStream_t)stream, stats, trace);
}

}  // extern "C"
