// Shared by the host sources behind include/ha_rag.h: the context, the pool bookkeeping
// structures and the helpers that more than one of those sources use.  Not installed, not
// part of the C ABI.
#pragma once
#include <hip/hip_runtime.h>

#include <condition_variable>
#include <cstdint>
#include <deque>
#include <list>
#include <memory>
#include <mutex>
#include <string>
#include <unordered_map>
#include <vector>

#include "../../include/ha_rag.h"
#include "ha_rag_kernels.h"

namespace ha_rag_host {

using namespace ha_rag;

constexpr uint64_t kPPM = 1000000ull;
constexpr uint32_t kNoRank = UINT32_MAX;
constexpr uint32_t kTiers = 4;        // HBM, pinned, pageable, disk
constexpr uint32_t kCacheTiers = 3;   // tiers with a capacity and an LRU order
constexpr size_t kDirectAlign = 4096; // offset / size / buffer alignment of O_DIRECT I/O

inline bool valid_group(uint32_t g)
{
    return g == 32 || g == 64 || g == 128 || g == 256 || g == 512;
}

inline uint32_t bits_of(uint32_t prec)  // storage bits per element
{
    return prec == HA_RAG_PREC_16 ? 16u : prec == HA_RAG_PREC_INT4 ? 4u : 8u;
}

inline bool has_meta(uint32_t prec) { return prec == HA_RAG_PREC_INT8 || prec == HA_RAG_PREC_INT4; }

inline uint32_t log2u(uint32_t v)
{
    uint32_t s = 0;
    while ((1u << s) < v) ++s;
    return s;
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
    // A copy that a running call has booked but whose bytes are not in place yet (the call moves
    // them with the context unlocked).  Other calls pass such a copy over: they read the chunk
    // from a slower tier, and neither evict the copy nor book a second one.
    uint8_t pending[kCacheTiers] = {0, 0, 0};
    uint32_t in_calls = 0;  // running calls that hold this entry by index: it is not removed meanwhile
    std::list<uint32_t>::iterator lru_it[kCacheTiers];

    bool readable(uint32_t t, uint64_t call) const
    {
        return slot[t] >= 0 && (t >= kCacheTiers || !pending[t] || (call && made_by[t] == call));
    }
    // fastest tier whose copy can be read; `call`: copies that this call itself booked count
    int fastest(uint64_t call = 0) const
    {
        for (uint32_t t = 0; t < kTiers; ++t)
            if (readable(t, call)) return (int)t;
        return -1;
    }
    bool has_slower_copy(uint32_t tier) const
    {
        for (uint32_t t = tier + 1; t < kTiers; ++t)
            if (readable(t, 0)) return true;
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
    uint32_t host_readers = 0;  // calls that are reading the slot on the host with the context unlocked
};

struct Slab {
    uint8_t *base = nullptr;  // memory tiers
    int fd = -1;              // disk tier
    size_t slot_bytes = 0;
    uint32_t n_slots = 0;
    bool reg = false;
    bool external = false;             // pinned tier only: every slot is a caller-owned address
    std::vector<uint8_t *> ext;        // ... kept here, one per slot; the slab grows on demand
    std::vector<uint32_t> free_slots;  // stack
    std::vector<SlotUse> use;
    std::list<uint32_t> lru;           // chunk indices resident here, least recent first
    bool registered() const { return reg; }
    bool holds_copies() const { return reg && !external; }  // Algorithm 2 may place copies here
    uint8_t *ptr(int32_t s) const { return external ? ext[(size_t)s] : base + (size_t)s * slot_bytes; }
    off_t offset(int32_t s) const { return (off_t)((size_t)s * slot_bytes); }
};

struct StagingSlot {
    hipEvent_t filled = nullptr, consumed = nullptr;
    bool consumed_valid = false;
};

struct BounceSlot {
    hipEvent_t h2d_done = nullptr;
    bool busy = false;      // a host -> device copy that reads it may be in flight (h2d_done tells)
    bool reserved = false;  // a running call owns it: being filled, or waiting for its copy to be enqueued
};

// One chunk's bytes on their way from a file or from pageable memory into a bounce buffer
// (and into the host slot Algorithm 2 placed a copy in), cut into pieces that the context's
// I/O threads move side by side.  Touches no context state.
struct Transfer {
    int fd = -1;                  // source: a file ...
    bool direct = false;
    off_t off = 0;
    const uint8_t *src = nullptr; // ... or host memory
    uint8_t *dst = nullptr;       // bounce buffer
    uint8_t *dst2 = nullptr;      // placed copy in pinned / pageable memory, or null
    size_t bytes = 0;
    std::mutex mu;
    std::condition_variable cv;
    size_t pieces_left = 0;
    int rc = 0;
    std::string err;
    int wait();  // blocks until every piece is done; returns the first error
};

class IoPool;

}  // namespace ha_rag_host

struct ha_rag_ctx {
    ha_rag_config cfg{};
    uint32_t n_tiles = 0;
    std::mutex mu;
    std::string err;  // last failing HIP or I/O call

    // entries of removed chunks keep id HA_RAG_NO_CHUNK.  A deque: entries stay where they are
    // when the table grows, so a call that releases the lock midway may keep references
    std::deque<ha_rag_host::Chunk> chunks;
    std::vector<uint32_t> dead;                // ... and wait here to be used again
    std::unordered_map<uint64_t, uint32_t> index;
    ha_rag_host::Slab slab[ha_rag_host::kTiers][HA_RAG_N_PREC];

    uint32_t bound[3] = {0, 0, 0};  // ranks below bound[t] belong to the list of tier <= t
    uint64_t n_loads = 0, use_seq = 0, call_seq = 0;

    uint8_t *staging = nullptr;
    size_t staging_slot_bytes = 0;
    std::vector<ha_rag_host::StagingSlot> stg;
    uint64_t stg_next = 0;

    uint8_t *bounce = nullptr;  // pinned buffers that pageable / disk chunks pass through
    size_t bounce_slot_bytes = 0;
    uint8_t *dio = nullptr;     // page-aligned ordinary memory for O_DIRECT writes: the
                                // kernel cannot do direct I/O on GPU-pinned host memory
    size_t dio_bytes = 0;
    std::condition_variable cv; // a bounce buffer was released, a pending copy published, ...
    ha_rag_host::IoPool *io = nullptr;  // threads that move file / pageable bytes (created on first use)
    std::vector<ha_rag_host::BounceSlot> bnc;
    uint64_t bnc_next = 0;

    std::vector<hipStream_t> copy_streams;
    uint64_t copy_rr = 0;
    std::unordered_map<hipStream_t, hipEvent_t> stream_done;

    ha_rag::K1Launch launch{64, 0, 0, true, true};  // 0: launch_k1 chooses

    uint32_t group_of(uint32_t prec) const
    {
        return prec == HA_RAG_PREC_INT8 ? cfg.group_int8 : prec == HA_RAG_PREC_INT4 ? cfg.group_int4 : 0;
    }
    bool dry() const { return cfg.dry_run != 0; }    // no HIP call is made
    bool no_io() const { return cfg.dry_run == 1; }  // nor is any byte moved on the host or to files
    bool direct() const { return cfg.disk_o_direct != 0; }
    size_t io_bytes(uint64_t bytes) const  // what a file transfer of `bytes` moves
    {
        return direct() ? (size_t)((bytes + ha_rag_host::kDirectAlign - 1) / ha_rag_host::kDirectAlign * ha_rag_host::kDirectAlign) : (size_t)bytes;
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

#define HIPCHK(ctx, call)                                                      \
    do {                                                                       \
        hipError_t e_ = (call);                                                \
        if (e_ != hipSuccess) {                                                \
            (ctx)->err = std::string(#call) + ": " + hipGetErrorString(e_);    \
            return HA_RAG_EHIP;                                                \
        }                                                                      \
    } while (0)

namespace ha_rag_host {

// why the last ha_rag_create on this thread failed
extern thread_local std::string g_create_err;

// ---- sizes (ha_rag_pool.hip) ----
int chunk_bytes_impl(uint32_t L, uint32_t H, uint32_t D, uint32_t prec, uint32_t group, uint32_t T,
                     size_t *payload, size_t *meta, size_t *total, uint32_t part = kPartKV);

// ---- files (ha_rag_io.hip) ----
int io_error(ha_rag_ctx *c, const char *what);
int read_full(ha_rag_ctx *c, int fd, uint8_t *dst, size_t n, off_t off);
int write_full(ha_rag_ctx *c, int fd, const uint8_t *src, size_t n, off_t off);
// The context's I/O threads (queue depth of the file tier).  start() cuts the transfer into
// pieces and returns at once; Transfer::wait() collects them.
IoPool *io_pool_create(uint32_t n_threads, bool direct);
void io_pool_destroy(IoPool *p);
void io_pool_start(IoPool *p, const std::shared_ptr<Transfer> &t);

// ---- streams, slots, tiers, ranks (ha_rag_pool.hip) ----
int stream_event(ha_rag_ctx *c, hipStream_t s, hipEvent_t *out);
int mark_stream(ha_rag_ctx *c, hipStream_t s);
int wait_for(ha_rag_ctx *c, hipStream_t s, hipStream_t other);
int before_read(ha_rag_ctx *c, SlotUse &u, hipStream_t s);
int before_write(ha_rag_ctx *c, SlotUse &u, hipStream_t s);
int before_host_write(ha_rag_ctx *c, SlotUse &u);
Chunk *find_chunk(ha_rag_ctx *c, uint64_t id, uint32_t *idx = nullptr);
void tier_touch(ha_rag_ctx *c, uint32_t tier, uint32_t ci);
void tier_attach(ha_rag_ctx *c, uint32_t tier, uint32_t ci, int32_t slot);
void tier_detach(ha_rag_ctx *c, uint32_t tier, uint32_t ci);
int32_t tier_acquire(ha_rag_ctx *c, uint32_t tier, uint32_t prec, uint64_t *evicted,
                     uint64_t keep_call = 0);
void rerank_locked(ha_rag_ctx *c);
uint32_t new_chunk_entry(ha_rag_ctx *c);  // index of a fresh entry of ctx->chunks
// A bounce buffer of this call's own: *wait_ev is the copy that may still read it (or null).  If
// all are taken by other calls: waits for one (block) or returns false.
bool reserve_bounce(ha_rag_ctx *c, std::unique_lock<std::mutex> &lk, bool block, size_t *idx,
                    hipEvent_t *wait_ev);
void release_bounce(ha_rag_ctx *c, size_t idx, bool copy_in_flight);
// Events of the device work that reads or writes a host slot, which the host has to wait for
// (outside the lock) before it overwrites the slot; the slot's lists are cleared.
void take_host_write_events(ha_rag_ctx *c, SlotUse &u, std::vector<hipEvent_t> *out);

// ---- attention (ha_rag_attend.hip) ----
// Address, on the current device, of the scratch array that ha_rag_attend_packed_static uses
// (looked up once per device; *ptr nullable).
int attend_static_scratch(void **ptr, std::string *err);

}  // namespace ha_rag_host
