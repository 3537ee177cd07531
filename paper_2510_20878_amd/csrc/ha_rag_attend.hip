// Host side of attention over packed chunks: argument checks, the workspace layout, and the
// launches (one partial-attention launch per 416 documents, one merge launch per 64 requests).
#include "ha_rag_internal.h"

#include <cstdio>

using namespace ha_rag_host;

namespace {

// A list in storage its owner provides: the planning below fills such lists, so that one of
// its callers can keep them on the stack and allocate nothing.
template <class T>
struct Fixed {
    T *data = nullptr;
    uint32_t cap = 0, n = 0;
    Fixed() = default;
    Fixed(T *d, uint32_t c) : data(d), cap(c) {}
    explicit Fixed(std::vector<T> &v) : data(v.data()), cap((uint32_t)v.size()) {}
    bool push_back(const T &v)
    {
        if (n == cap) return false;
        data[n++] = v;
        return true;
    }
    T &operator[](size_t i) const { return data[i]; }
    uint32_t size() const { return n; }
    void clear() { n = 0; }
};

// One document of a request: keys and values, from one whole chunk or from a keys-only and a
// values-only chunk (paired in list order).
struct Doc {
    const uint8_t *k = nullptr, *v = nullptr;  // packed bytes holding the keys / the values
    uint64_t k_tile = 0, v_tile = 0;           // bytes of one tile record
    uint32_t k_first = 0, v_first = 0;         // tile record of (layer 0, head 0): 0, or H for the
                                               // values of a whole chunk; a layer is k_step records on
    uint32_t k_step = 0, v_step = 0;
    uint32_t n_tokens = 0, info = 0;
};

struct Plan {               // one request
    uint32_t first_doc = 0, n_docs = 0;  // its documents that hold tokens
    uint32_t n_mt = 1;
    uint32_t shared = 0;       // more than two query tiles: the kernel whose waves share each decoded block
    uint32_t run_blocks = 0;   // layout blocks per run (what one workgroup takes)
    uint64_t all_blocks = 0;   // layout blocks of all its documents
    uint32_t n_runs = 0;       // records per (KV head, tile)
    uint32_t final = 0;        // one run of the shared kernel is all there is: it writes the output itself
    uint64_t part_floats = 0;  // offset of its records in the workspace
};

// workgroups per (run, KV head) of a request
uint32_t tile_groups(const Plan &pl, uint32_t waves)
{
    return pl.shared ? (pl.n_mt + 2u * waves - 1u) / (2u * waves) : (pl.n_mt + 1u) / 2u;
}

// A run: the blocks one workgroup takes, a range of the request's blocks in list order.  For the
// shared kernel it may start and end inside a document and span several; for the kernel of at
// most two query tiles it is a piece of one document.
struct Run {
    uint32_t doc, first_block;  // first document (index into the request's documents) and block in it
    uint32_t n_docs, end_block; // documents touched; end of the range in the last of them
};
constexpr uint32_t kMaxRunDocs = 128;  // a run's documents are descriptors of one launch

// The run that starts at block `blk` of document `doc` of the request (both moved to the next
// run's start); false when the request has no block left.
bool next_run(const Plan &pl, const Doc *docs, uint32_t &doc, uint32_t &blk, Run *out)
{
    if (doc >= pl.n_docs) return false;
    out->doc = doc;
    out->first_block = blk;
    if (!pl.shared) {  // equal pieces of one document, none longer than run_blocks
        const uint32_t nb = (docs[doc].n_tokens + 15u) / 16u;
        const uint32_t n = (nb + pl.run_blocks - 1u) / pl.run_blocks, len = (nb + n - 1u) / n;
        out->n_docs = 1;
        out->end_block = nb - blk > len ? blk + len : nb;
        blk = out->end_block;
        if (blk == nb) {
            ++doc;
            blk = 0;
        }
        return true;
    }
    out->n_docs = 0;
    uint32_t left = pl.run_blocks;
    for (;;) {
        const uint32_t nb = (docs[doc].n_tokens + 15u) / 16u;
        ++out->n_docs;
        if (nb - blk > left) {  // the run ends inside this document
            blk += left;
            out->end_block = blk;
            return true;
        }
        left -= nb - blk;
        out->end_block = nb;
        ++doc;
        blk = 0;
        if (left == 0 || doc >= pl.n_docs || out->n_docs == kMaxRunDocs) return true;
    }
}

uint32_t count_runs(const Plan &pl, const Doc *docs)
{
    uint32_t doc = 0, blk = 0, n = 0;
    Run r;
    while (next_run(pl, docs, doc, blk, &r)) ++n;
    return n;
}

// Checks everything and lays the workspace out.  *floats = workspace size in binary32 words.
// plans: n_reqs entries; docs, open_k, open_v: filled here, ENOSPC if one of them is too small
// (never with lists as long as the call's chunk list).
int plan_attend(ha_rag_ctx *c, const ha_rag_packed_chunk *chunks, const ha_rag_attend_request *reqs,
                uint32_t n_reqs, uint32_t n_q_heads, Plan *plans, Fixed<Doc> *docs,
                Fixed<uint32_t> open_k, Fixed<uint32_t> open_v, uint64_t *floats,
                uint32_t *shared_waves, bool need_buffers)
{
    if (!c || !reqs || n_reqs == 0 || n_reqs > HA_RAG_MAX_ATTEND_REQUESTS) return HA_RAG_EINVAL;
    if (c->cfg.head_dim != kAttendHeadDim) return HA_RAG_EFORMAT;
    const uint32_t L = c->cfg.n_layers, H = c->cfg.n_kv_heads;
    if (n_q_heads == 0 || n_q_heads % H || n_q_heads / H > 64) return HA_RAG_EINVAL;
    const uint32_t G = n_q_heads / H;
    uint64_t total = 0, n_chunks = 0;
    docs->clear();
    // open_k / open_v: documents still waiting for their values / keys
    for (uint32_t r = 0; r < n_reqs; ++r) {
        const ha_rag_attend_request &rq = reqs[r];
        Plan &pl = plans[r];
        pl = Plan();
        if (rq.n_q == 0 || rq.n_q > HA_RAG_MAX_ATTEND_Q) return HA_RAG_EINVAL;
        if (need_buffers && (!rq.q || !rq.out || ((uintptr_t)rq.q & 15u) || ((uintptr_t)rq.out & 15u)))
            return HA_RAG_EINVAL;
        if (n_chunks + rq.n_chunks > HA_RAG_MAX_REQUEST_CHUNKS || (rq.n_chunks && !chunks))
            return HA_RAG_EINVAL;
        pl.first_doc = (uint32_t)docs->size();
        pl.n_mt = (rq.n_q * G + 15u) / 16u;
        pl.shared = pl.n_mt > 2u;
        open_k.clear();
        open_v.clear();
        size_t next_k = 0, next_v = 0;  // first entries of open_k / open_v not yet matched
        for (uint32_t i = 0; i < rq.n_chunks; ++i) {
            const ha_rag_packed_chunk &pc = chunks[n_chunks + i];
            size_t bytes = 0;
            int rc = chunk_bytes_impl(L, H, c->cfg.head_dim, pc.prec, pc.group, pc.n_tokens, nullptr,
                                      nullptr, &bytes, pc.part);
            if (rc) return rc;
            if (pc.n_tokens == 0) continue;  // holds nothing, pairs with nothing
            if (need_buffers && (!pc.packed || ((uintptr_t)pc.packed & 15u))) return HA_RAG_EINVAL;
            const uint8_t *ptr = static_cast<const uint8_t *>(pc.packed);
            const uint32_t fmt = pc.prec | ((has_meta(pc.prec) ? log2u(pc.group) : 0u) << 4);
            if (pc.part == HA_RAG_PART_KV) {
                Doc d;
                d.k = d.v = ptr;
                d.k_tile = d.v_tile = bytes / (2ull * L * H);
                d.k_first = 0;
                d.v_first = H;
                d.k_step = d.v_step = 2u * H;
                d.n_tokens = pc.n_tokens;
                d.info = fmt | (fmt << 8);
                if (!docs->push_back(d)) return HA_RAG_ENOSPC;
            } else {
                // the i-th keys-only chunk of the request and its i-th values-only chunk are one
                // document: they must hold the same tokens
                const bool is_k = pc.part == HA_RAG_PART_K;
                Fixed<uint32_t> &mine = is_k ? open_k : open_v, &other = is_k ? open_v : open_k;
                size_t &other_next = is_k ? next_v : next_k;
                uint32_t di;
                if (other_next < other.size()) {
                    di = other[other_next++];
                    if ((*docs)[di].n_tokens != pc.n_tokens) return HA_RAG_EINVAL;
                } else {
                    di = (uint32_t)docs->size();
                    if (!docs->push_back(Doc()) || !mine.push_back(di)) return HA_RAG_ENOSPC;
                    (*docs)[di].n_tokens = pc.n_tokens;
                }
                Doc &d = (*docs)[di];
                (is_k ? d.k : d.v) = ptr;
                (is_k ? d.k_tile : d.v_tile) = bytes / ((uint64_t)L * H);
                (is_k ? d.k_step : d.v_step) = H;
                d.info |= is_k ? fmt : fmt << 8;
            }
        }
        if (next_k != open_k.size() || next_v != open_v.size()) return HA_RAG_EINVAL;  // keys without values or the reverse
        pl.n_docs = (uint32_t)docs->size() - pl.first_doc;
        n_chunks += rq.n_chunks;
    }
    // The shared kernel runs with as many waves (two tiles each) as the call's largest request
    // has use for: 2, 4 or 8.
    uint32_t most_mt = 0;
    for (uint32_t r = 0; r < n_reqs; ++r)
        if (plans[r].shared && plans[r].n_mt > most_mt) most_mt = plans[r].n_mt;
    const uint32_t waves = most_mt > 8u ? 8u : most_mt > 4u ? 4u : 2u;
    *shared_waves = waves;
    // A workgroup takes a run of its request's blocks and writes one record per query tile for
    // it.  Requests of at most two query tiles: a run is a piece of one document, as long as
    // possible (every workgroup pays for fetching the queries and for writing a record), but
    // short enough that the launch fills the chip a few times over, since the hardware then
    // evens out what documents of different formats and lengths take.
    for (uint32_t r = 0; r < n_reqs; ++r) {
        Plan &pl = plans[r];
        pl.all_blocks = 0;
        for (uint32_t i = 0; i < pl.n_docs; ++i) pl.all_blocks += ((*docs)[pl.first_doc + i].n_tokens + 15u) / 16u;
    }
    auto groups_at = [&](uint32_t piece) {  // workgroups of the one/two-tile kernel with pieces this long
        uint64_t groups = 0;
        for (uint32_t r = 0; r < n_reqs; ++r) {
            const Plan &pl = plans[r];
            if (pl.shared) continue;
            uint64_t runs = 0;
            for (uint32_t i = 0; i < pl.n_docs; ++i)
                runs += (((*docs)[pl.first_doc + i].n_tokens + 15u) / 16u + piece - 1u) / piece;
            groups += runs * H * tile_groups(pl, waves);
        }
        return groups;
    };
    uint32_t piece = kAttendMaxRunBlocks;
    while (piece > kAttendMinRunBlocks && groups_at(piece) < kAttendTargetGroups) piece >>= 1;
    // A call of so few workgroups that even twice as many run side by side (four per CU) is
    // bound by how long one of them takes: halve once more (one request of 10 x 512 tokens:
    // 13.7 against 14.7 us; with two requests, 1,280 workgroups, it would cost 1.5 us).
    if (piece == kAttendMinRunBlocks && groups_at(piece / 2u) <= 4ull * kChipCUs) piece /= 2u;
    // The shared kernel: a run crosses document boundaries (records rival the packed bytes once
    // a request has hundreds of query rows; equal runs also finish together whatever the
    // documents' lengths).  Workgroups of one size finish in rounds of as many as the chip holds
    // side by side, so a launch takes rounds x blocks per run: the longest run with the least
    // of that is taken; a run is at least kAttendMinRunBlocks long.
    const uint64_t side_by_side = (uint64_t)kChipCUs * (8u / waves);  // two waves per SIMD: eight per CU
    uint64_t most_blocks = 0;
    for (uint32_t r = 0; r < n_reqs; ++r)
        if (plans[r].shared && plans[r].all_blocks > most_blocks) most_blocks = plans[r].all_blocks;
    uint64_t run_blocks = most_blocks, least = ~0ull;
    for (uint64_t n = 1; n <= most_blocks; ++n) {  // n runs for the largest request
        const uint64_t len = (most_blocks + n - 1u) / n;
        if (n > 1 && len < kAttendMinRunBlocks) break;
        uint64_t wgs = 0;
        for (uint32_t r = 0; r < n_reqs; ++r) {
            const Plan &pl = plans[r];
            if (pl.shared) wgs += (pl.all_blocks + len - 1u) / len * H * tile_groups(pl, waves);
        }
        const uint64_t cost = (wgs + side_by_side - 1u) / side_by_side * len;
        if (cost < least) {
            least = cost;
            run_blocks = len;
        }
        if (wgs >= 64u * side_by_side) break;  // finer than this gains nothing
    }
    for (uint32_t r = 0; r < n_reqs; ++r) {
        Plan &pl = plans[r];
        pl.run_blocks = !pl.shared ? piece : run_blocks > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)(run_blocks ? run_blocks : 1u);
        pl.n_runs = count_runs(pl, docs->data + pl.first_doc);
        pl.final = pl.shared && pl.n_runs == 1u;  // no record, no merge
        pl.part_floats = total;
        if (!pl.final) total += (uint64_t)pl.n_runs * H * pl.n_mt * kAttendRecFloats;
    }
    if (total * 4ull > (1ull << 40)) return HA_RAG_EINVAL;
    *floats = total;
    return HA_RAG_OK;
}


// Storage of one call's plan.  The ordinary entry points size it for the call on the heap; the
// entry point that allocates nothing keeps a small one on the stack.
struct PlanStore {
    Plan *plans;
    Fixed<Doc> docs;
    Fixed<uint32_t> open_k, open_v;
};

struct HeapPlanStore {
    std::vector<Plan> plans;
    std::vector<Doc> docs;
    std::vector<uint32_t> open_k, open_v;
    HeapPlanStore(const ha_rag_attend_request *reqs, uint32_t n_reqs)
    {
        uint64_t n = 0;
        if (reqs && n_reqs <= HA_RAG_MAX_ATTEND_REQUESTS)
            for (uint32_t r = 0; r < n_reqs; ++r) n += reqs[r].n_chunks;
        if (n > HA_RAG_MAX_REQUEST_CHUNKS) n = 0;  // the planning refuses the call anyway
        plans.resize(n_reqs <= HA_RAG_MAX_ATTEND_REQUESTS ? n_reqs : 0);
        docs.resize((size_t)n);
        open_k.resize((size_t)n);
        open_v.resize((size_t)n);
    }
    PlanStore store() { return PlanStore{plans.data(), Fixed<Doc>(docs), Fixed<uint32_t>(open_k), Fixed<uint32_t>(open_v)}; }
};

// checks, workspace layout and launches; the caller holds the context's lock.  *need (nullable)
// receives the workspace bytes the lists ask for, also when the call then fails with ENOSPC.
int attend_locked(ha_rag_ctx *c, PlanStore ps, const ha_rag_packed_chunk *chunks,
                  const ha_rag_attend_request *reqs, uint32_t n_reqs, uint32_t layer,
                  uint32_t n_q_heads, float sm_scale, void *workspace, size_t workspace_bytes,
                  void *stream, uint64_t *need = nullptr)
{
    uint64_t floats = 0;
    uint32_t waves = 2;
    int rc = plan_attend(c, chunks, reqs, n_reqs, n_q_heads, ps.plans, &ps.docs, ps.open_k, ps.open_v,
                         &floats, &waves, true);
    if (rc) return rc;
    const Plan *plans = ps.plans;
    const Fixed<Doc> &docs = ps.docs;
    if (need) *need = floats * 4ull;
    if (layer >= c->cfg.n_layers || !(sm_scale > 0.0f) || !(sm_scale < 1e30f)) return HA_RAG_EINVAL;
    if (floats && (!workspace || ((uintptr_t)workspace & 15u))) return HA_RAG_EINVAL;
    if (floats * 4ull > workspace_bytes) return HA_RAG_ENOSPC;
    // a context without a device fills and checks the launches' descriptors all the same
    const bool dry = c->dry();
    hipStream_t st = (hipStream_t)stream;
    const uint32_t H = c->cfg.n_kv_heads;
    float *ws = static_cast<float *>(workspace);

    // two launches in the making: requests of at most two query tiles, and the others
    K6Params kp{}, ks{};
    for (K6Params *q : {&kp, &ks}) {
        q->n_kv_heads = H;
        q->n_q_heads = n_q_heads;
        q->layer = layer;
        q->scale_log2 = sm_scale * 1.44269504088896341f;
    }
    auto doc_k = [&](const Doc &doc) { return doc.k + (uint64_t)(doc.k_first + layer * doc.k_step) * doc.k_tile; };
    auto doc_v = [&](const Doc &doc) { return doc.v + (uint64_t)(doc.v_first + layer * doc.v_step) * doc.v_tile; };
    // A launch lists its runs (one grid row each), then the runs' further documents run by run.
    // A run never straddles two launches: first count the runs that fit, then fill.
    struct RunPos {
        uint32_t r, doc, blk, run_no;  // request, start of the next run in it, number of that run
    };
    for (uint32_t sh = 0; sh < 2u; ++sh) {  // the kernel of at most two tiles, then the shared one
        K6Params &kq = sh ? ks : kp;
        auto settle = [&](RunPos &p) {  // moves p to the next run there is; false at the end
            while (p.r < n_reqs && (plans[p.r].shared != sh || p.doc >= plans[p.r].n_docs)) {
                ++p.r;
                p.doc = p.blk = p.run_no = 0;
            }
            return p.r < n_reqs;
        };
        auto take = [&](RunPos &p, Run *run) {  // the run at p; p moves behind it
            const Plan &pl = plans[p.r];
            next_run(pl, docs.data + pl.first_doc, p.doc, p.blk, run);
            ++p.run_no;
        };
        RunPos at = {0, 0, 0, 0};
        while (settle(at)) {
            uint32_t n_runs = 0, n_more = 0;
            for (RunPos p = at; settle(p);) {
                Run run;
                take(p, &run);
                if ((uint64_t)(K6Params::docs_behind(n_runs + 1u) + n_more + run.n_docs - 1u) > kAttendMaxDocs) break;
                ++n_runs;
                n_more += run.n_docs - 1u;
            }
            kq.n_runs = n_runs;
            kq.doc_first = K6Params::docs_behind(n_runs);
            uint32_t later = kq.doc_first;  // where the next run's further documents go
            for (uint32_t k = 0; k < n_runs; ++k) {
                settle(at);
                const Plan &pl = plans[at.r];
                const ha_rag_attend_request &rq = reqs[at.r];
                const uint32_t run_no = at.run_no;
                Run run;
                take(at, &run);
                const Doc &first = docs[pl.first_doc + run.doc];
                K6Run &d = kq.run[k];
                d.k = doc_k(first);
                d.v = doc_v(first);
                d.q = static_cast<const uint16_t *>(rq.q);
                d.part = pl.final ? rq.out : ws + pl.part_floats + (uint64_t)run_no * H * pl.n_mt * kAttendRecFloats;
                d.final = pl.final;
                d.lse = pl.final ? rq.lse : nullptr;
                d.n_tokens = first.n_tokens;
                d.info = first.info;
                d.n_q = rq.n_q;
                d.n_docs = run.n_docs;
                d.more = later;
                d.first_block = run.first_block;
                d.end_block = run.end_block;
                for (uint32_t i = 1; i < run.n_docs; ++i) {
                    const Doc &doc = docs[pl.first_doc + run.doc + i];
                    kq.doc[later++] = K6Doc{doc_k(doc), doc_v(doc), doc.n_tokens, doc.info};
                }
            }
            kq.doc_end = later;
            HIPCHK(c, sh ? launch_k6_shared(kq, waves, st, dry) : launch_k6(kq, st, dry));
        }
    }

    K7Params mp{};
    mp.n_kv_heads = H;
    mp.n_q_heads = n_q_heads;
    for (uint32_t r = 0; r < n_reqs; ++r) {
        if (plans[r].final) continue;  // written by the run's own workgroups
        K7Req &d = mp.r[mp.n_reqs++];
        d.part = ws + plans[r].part_floats;
        d.out = reqs[r].out;
        d.lse = reqs[r].lse;
        d.n_q = reqs[r].n_q;
        d.n_runs = plans[r].n_runs;
        d.pad[0] = d.pad[1] = 0;
        if (mp.n_reqs == kMaxMergeReqs) {
            HIPCHK(c, launch_k7(mp, st, dry));
            mp.n_reqs = 0;
        }
    }
    if (mp.n_reqs) HIPCHK(c, launch_k7(mp, st, dry));
    return HA_RAG_OK;
}

// ids -> descriptors of the copies the kernel can read in place (HBM, else pinned memory)
int resolve_ids(ha_rag_ctx *c, const uint64_t *ids, const ha_rag_attend_request *reqs,
                       uint32_t n_reqs, std::vector<ha_rag_packed_chunk> *out,
                       std::vector<uint32_t> *cis)
{
    if (!c || !reqs || n_reqs == 0 || n_reqs > HA_RAG_MAX_ATTEND_REQUESTS) return HA_RAG_EINVAL;
    uint64_t n = 0;
    for (uint32_t r = 0; r < n_reqs; ++r) n += reqs[r].n_chunks;
    if (n > HA_RAG_MAX_REQUEST_CHUNKS || (n && !ids)) return HA_RAG_EINVAL;
    out->resize((size_t)n);
    cis->resize((size_t)n);
    for (uint64_t i = 0; i < n; ++i) {
        uint32_t ci = 0;
        const Chunk *ch = find_chunk(c, ids[i], &ci);
        if (!ch) return HA_RAG_ENOENT;
        const int t = ch->fastest();
        if (t != (int)HA_RAG_TIER_HBM && t != (int)HA_RAG_TIER_PINNED) return HA_RAG_ENOENT;
        ha_rag_packed_chunk &pc = (*out)[(size_t)i];
        pc.packed = c->slab[t][ch->prec].ptr(ch->slot[t]);
        pc.n_tokens = ch->n_tokens;
        pc.prec = ch->prec;
        pc.group = c->group_of(ch->prec);
        pc.part = ch->part;
        (*cis)[(size_t)i] = ci;
    }
    return HA_RAG_OK;
}

// ---- scratch of ha_rag_attend_packed_static ------------------------------------------------
// The partial results of that entry point live in this array instead of a caller's workspace.
// Every GPU holds its own copy at its own address, from the moment the code object is loaded
// there until the process ends.  In host code the name is only a handle for
// hipGetSymbolAddress: what kernels and copies get is the address that call returned for the
// current device, kept in g_scratch_ptr.
constexpr size_t kStaticScratchBytes = (size_t)HA_RAG_ATTEND_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};

}  // namespace

namespace ha_rag_host {

// Address of the scratch array on the current device; looked up once per device.
int attend_static_scratch(void **ptr, std::string *err)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        if (err) *err = std::string("hipGetDevice: ") + (e != hipSuccess ? hipGetErrorString(e) : "device index out of range");
        return HA_RAG_EHIP;
    }
    std::lock_guard<std::mutex> g(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress((void **)&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            if (err) *err = std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e);
            return HA_RAG_EHIP;
        }
        g_scratch_ptr[dev] = p;
    }
    if (ptr) *ptr = g_scratch_ptr[dev];
    return HA_RAG_OK;
}

}  // namespace ha_rag_host

extern "C" {

int ha_rag_attend_workspace_bytes(ha_rag_ctx *c, const ha_rag_packed_chunk *chunks,
                                  const ha_rag_attend_request *reqs, uint32_t n_reqs,
                                  uint32_t n_q_heads, size_t *bytes)
{
    if (!bytes) return HA_RAG_EINVAL;
    HeapPlanStore hs(reqs, n_reqs);
    PlanStore ps = hs.store();
    uint64_t floats = 0;
    uint32_t waves = 0;
    int rc = plan_attend(c, chunks, reqs, n_reqs, n_q_heads, ps.plans, &ps.docs, ps.open_k, ps.open_v,
                         &floats, &waves, false);
    if (rc) return rc;
    *bytes = (size_t)(floats * 4ull);
    return HA_RAG_OK;
}

int ha_rag_attend_packed(ha_rag_ctx *c, const ha_rag_packed_chunk *chunks,
                         const ha_rag_attend_request *reqs, uint32_t n_reqs, uint32_t layer,
                         uint32_t n_q_heads, float sm_scale, void *workspace, size_t workspace_bytes,
                         void *stream)
{
    if (!c) return HA_RAG_EINVAL;
    HeapPlanStore hs(reqs, n_reqs);
    std::lock_guard<std::mutex> g(c->mu);
    return attend_locked(c, hs.store(), chunks, reqs, n_reqs, layer, n_q_heads, sm_scale, workspace,
                         workspace_bytes, stream);
}

int ha_rag_attend_packed_static(ha_rag_ctx *c, const ha_rag_packed_chunk *chunks,
                                const ha_rag_attend_request *reqs, uint32_t n_reqs, uint32_t layer,
                                uint32_t n_q_heads, float sm_scale, void *stream)
{
    if (!c || !reqs || n_reqs == 0) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    if (n_reqs > HA_RAG_ATTEND_STATIC_MAX_REQUESTS) {
        c->err = "ha_rag_attend_packed_static: more than " +
                 std::to_string(HA_RAG_ATTEND_STATIC_MAX_REQUESTS) + " requests in one call";
        return HA_RAG_ENOSPC;
    }
    // the plan of the call on the stack: no list here grows
    Plan plans[HA_RAG_ATTEND_STATIC_MAX_REQUESTS];
    Doc docs[HA_RAG_ATTEND_STATIC_MAX_DOCS];
    uint32_t open_k[HA_RAG_ATTEND_STATIC_MAX_DOCS], open_v[HA_RAG_ATTEND_STATIC_MAX_DOCS];
    PlanStore ps{plans, Fixed<Doc>(docs, HA_RAG_ATTEND_STATIC_MAX_DOCS),
                 Fixed<uint32_t>(open_k, HA_RAG_ATTEND_STATIC_MAX_DOCS),
                 Fixed<uint32_t>(open_v, HA_RAG_ATTEND_STATIC_MAX_DOCS)};
    void *ws = nullptr;
    if (!c->dry()) {
        int rc = attend_static_scratch(&ws, &c->err);
        if (rc) return rc;
    } else {
        ws = reinterpret_cast<void *>((uintptr_t)256);  // never dereferenced
    }
    uint64_t need = 0;
    int rc = attend_locked(c, ps, chunks, reqs, n_reqs, layer, n_q_heads, sm_scale, ws,
                           kStaticScratchBytes, stream, &need);
    if (rc == HA_RAG_ENOSPC) {
        char msg[192];
        if (need > kStaticScratchBytes)
            std::snprintf(msg, sizeof msg,
                          "ha_rag_attend_packed_static: the call needs %llu bytes of partial results, the scratch array holds %llu",
                          (unsigned long long)need, (unsigned long long)kStaticScratchBytes);
        else
            std::snprintf(msg, sizeof msg,
                          "ha_rag_attend_packed_static: more than %u documents in one call",
                          (unsigned)HA_RAG_ATTEND_STATIC_MAX_DOCS);
        c->err = msg;
    }
    return rc;
}

int ha_rag_attend_chunks_workspace_bytes(ha_rag_ctx *c, const uint64_t *ids,
                                         const ha_rag_attend_request *reqs, uint32_t n_reqs,
                                         uint32_t n_q_heads, size_t *bytes)
{
    if (!c || !bytes) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    std::vector<ha_rag_packed_chunk> chunks;
    std::vector<uint32_t> cis;
    int rc = resolve_ids(c, ids, reqs, n_reqs, &chunks, &cis);
    if (rc) return rc;
    HeapPlanStore hs(reqs, n_reqs);
    PlanStore ps = hs.store();
    uint64_t floats = 0;
    uint32_t waves = 0;
    rc = plan_attend(c, chunks.data(), reqs, n_reqs, n_q_heads, ps.plans, &ps.docs, ps.open_k, ps.open_v,
                     &floats, &waves, false);
    if (rc) return rc;
    *bytes = (size_t)(floats * 4ull);
    return HA_RAG_OK;
}

int ha_rag_attend_chunks(ha_rag_ctx *c, const uint64_t *ids, const ha_rag_attend_request *reqs,
                         uint32_t n_reqs, uint32_t layer, uint32_t n_q_heads, float sm_scale,
                         uint32_t flags, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!c || (flags & ~(uint32_t)HA_RAG_ATTEND_COUNT)) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    std::vector<ha_rag_packed_chunk> chunks;
    std::vector<uint32_t> cis;
    int rc = resolve_ids(c, ids, reqs, n_reqs, &chunks, &cis);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)stream;
    // the kernels read the slots where they lie: wait for whoever wrote them on another stream
    for (size_t i = 0; i < cis.size(); ++i) {
        const Chunk &ch = c->chunks[cis[i]];
        const int t = ch.fastest();
        rc = before_read(c, c->slab[t][ch.prec].use[ch.slot[t]], s);
        if (rc) return rc;
    }
    HeapPlanStore hs(reqs, n_reqs);
    rc = attend_locked(c, hs.store(), chunks.data(), reqs, n_reqs, layer, n_q_heads, sm_scale, workspace,
                       workspace_bytes, stream);
    if (rc) return rc;
    if (flags & HA_RAG_ATTEND_COUNT) {  // Algorithm 1's access counts and the LRU order of Algorithm 2
        if (c->cfg.rerank_interval && c->n_loads && (c->n_loads % c->cfg.rerank_interval) == 0)
            rerank_locked(c);
        ++c->n_loads;
        for (uint32_t ci : cis) {
            Chunk &ch = c->chunks[ci];
            ch.count += 1;
            tier_touch(c, (uint32_t)ch.fastest(), ci);
        }
    }
    return mark_stream(c, s);  // a later writer of one of these slots waits for this point
}

}  // extern "C"
