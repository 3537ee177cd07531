// Several threads call into one context at once.  Meant to be built with -fsanitize=thread on
// the host side: the library promises that a context may be used from several threads, so the
// sanitizer must stay silent, and the pool must be consistent afterwards.
//   threads_host <ops>          dry_run = 1: host bookkeeping only, no HIP call, no byte moved
//   threads_host <ops> <dir>    dry_run = 2: no HIP call, but real bytes through pageable memory
//                               and real pool files in <dir> (also with O_DIRECT), moved by the
//                               context's I/O threads while the context is unlocked; every copy
//                               left in pinned or pageable memory must hold its chunk's bytes
#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <thread>
#include <vector>

#include "../../include/ha_rag.h"

#define REQUIRE(cond)                                                          \
    do {                                                                       \
        if (!(cond)) {                                                         \
            std::fprintf(stderr, "threads_host: %s failed at line %d\n", #cond, __LINE__); \
            std::exit(1);                                                      \
        }                                                                      \
    } while (0)

static uint64_t next(uint64_t &s)
{
    s ^= s << 13;
    s ^= s >> 7;
    s ^= s << 17;
    return s;
}

static std::vector<uint8_t> random_bytes(size_t n, uint64_t seed)
{
    std::vector<uint8_t> v(n);
    uint64_t s = seed * 0x9E3779B97F4A7C15ull + 1;
    for (size_t i = 0; i < n; ++i) v[i] = (uint8_t)next(s);
    return v;
}

static void *aligned(size_t bytes)
{
    void *p = nullptr;
    REQUIRE(posix_memalign(&p, 4096, bytes) == 0);
    std::memset(p, 0xEE, bytes);
    return p;
}

// Four threads load and place chunks whose masters are in a real file; Algorithm 2 copies them
// into small pinned and pageable slabs (ordinary memory here), evicting as it goes.
static void real_tiers(int ops, const std::string &dir, uint32_t direct)
{
    ha_rag_config cfg;
    std::memset(&cfg, 0, sizeof cfg);
    cfg.n_layers = 4;
    cfg.n_kv_heads = 4;
    cfg.head_dim = 128;
    cfg.max_chunk_tokens = 160;   // up to 5 MiB per 16-bit chunk: more than one piece
    cfg.group_int8 = 128;
    cfg.group_int4 = 128;
    cfg.tau_gpu_ppm = 0;
    cfg.tau_pin_ppm = 200000;
    cfg.tau_page_ppm = 300000;
    cfg.rerank_interval = 7;
    cfg.disk_o_direct = direct;
    cfg.io_threads = 3;
    cfg.dry_run = 2;
    ha_rag_ctx *ctx = nullptr;
    REQUIRE(ha_rag_create(&cfg, &ctx) == HA_RAG_OK);
    const uint32_t n_ids = 24;
    size_t total = 0;
    REQUIRE(ha_rag_chunk_bytes(4, 4, 128, HA_RAG_PREC_16, 0, cfg.max_chunk_tokens, nullptr, nullptr, &total) == HA_RAG_OK);
    const size_t slot = (total + 4095) & ~(size_t)4095;
    void *pin = aligned(slot * 3), *page = aligned(slot * 4), *bounce = aligned(slot * 3);
    REQUIRE(ha_rag_register_slab(ctx, HA_RAG_TIER_PINNED, HA_RAG_PREC_16, pin, slot * 3) == HA_RAG_OK);
    REQUIRE(ha_rag_register_slab(ctx, HA_RAG_TIER_PAGEABLE, HA_RAG_PREC_16, page, slot * 4) == HA_RAG_OK);
    const std::string path = dir + (direct ? "/threads_d.pool" : "/threads_b.pool");
    REQUIRE(ha_rag_register_disk(ctx, HA_RAG_PREC_16, path.c_str(), slot * n_ids) == HA_RAG_OK);
    REQUIRE(ha_rag_register_staging(ctx, (void *)0x300000000000ull, slot * 4) == HA_RAG_OK);
    REQUIRE(ha_rag_register_bounce(ctx, bounce, slot * 3) == HA_RAG_OK);
    std::vector<std::vector<uint8_t>> bytes(n_ids);
    std::vector<uint32_t> tokens(n_ids);
    for (uint32_t id = 0; id < n_ids; ++id) {
        tokens[id] = 20 + 6 * id;
        size_t nb = 0;
        REQUIRE(ha_rag_chunk_bytes(4, 4, 128, HA_RAG_PREC_16, 0, tokens[id], nullptr, nullptr, &nb) == HA_RAG_OK);
        bytes[id] = random_bytes(nb, id + 1);
        REQUIRE(ha_rag_pool_insert(ctx, id, HA_RAG_PREC_16, tokens[id], bytes[id].data(), 0, HA_RAG_TIER_DISK, nullptr) == HA_RAG_OK);
    }
    REQUIRE(ha_rag_rerank(ctx) == HA_RAG_OK);
    std::atomic<uint64_t> chunks{0}, disk_bytes{0};
    auto worker = [&](int t) {
        uint64_t s = 0xD1B54A32D192ED03ull * (uint64_t)(t + 1);
        for (int op = 0; op < ops; ++op) {
            uint64_t ids[4];
            const uint32_t n = 1 + (uint32_t)(next(s) % 4);
            // a skewed choice, so that some chunks are hot enough for the pinned and pageable lists
            for (uint32_t i = 0; i < n; ++i) ids[i] = (next(s) % 3 ? next(s) % 6 : next(s) % n_ids);
            ha_rag_load_stats st;
            const uint64_t what = next(s) % 10;
            if (what < 5) {
                REQUIRE(ha_rag_load_chunks(ctx, ids, nullptr, n, (void *)(0x500000000000ull + (uint64_t)t * 0x100000000ull),
                                           4 * 160, 0, nullptr, &st, nullptr) == HA_RAG_OK);
            } else if (what < 9) {
                REQUIRE(ha_rag_place_chunks(ctx, ids, nullptr, n, (uint32_t)(next(s) % 2), nullptr, &st, nullptr) == HA_RAG_OK);
            } else {
                int rc = ha_rag_pool_evict(ctx, next(s) % n_ids, 1 + (uint32_t)(next(s) % 2));
                REQUIRE(rc == HA_RAG_OK || rc == HA_RAG_ENOENT || rc == HA_RAG_EINVAL);
                continue;
            }
            REQUIRE(st.n_chunks == n);
            chunks.fetch_add(n);
            disk_bytes.fetch_add(st.bytes_disk_read);
        }
    };
    std::vector<std::thread> th;
    for (int t = 0; t < 4; ++t) th.emplace_back(worker, t);
    for (auto &x : th) x.join();
    uint64_t counted = 0, copies = 0;
    for (uint32_t id = 0; id < n_ids; ++id) {
        ha_rag_chunk_info info;
        REQUIRE(ha_rag_pool_query(ctx, id, &info) == HA_RAG_OK);
        counted += info.count;
        for (uint32_t tier : {(uint32_t)HA_RAG_TIER_PINNED, (uint32_t)HA_RAG_TIER_PAGEABLE}) {
            void *p = nullptr;
            size_t nb = 0;
            if (ha_rag_pool_slot(ctx, id, tier, &p, &nb) == HA_RAG_OK) {
                REQUIRE(nb == bytes[id].size() && std::memcmp(p, bytes[id].data(), nb) == 0);
                ++copies;
            }
        }
    }
    REQUIRE(counted == chunks.load());
    REQUIRE(copies > 0 && disk_bytes.load() > 0);
    REQUIRE(ha_rag_destroy(ctx) == HA_RAG_OK);
    std::free(pin);
    std::free(page);
    std::free(bounce);
    std::printf("threads_host real tiers (%s): %llu chunks, %llu bytes from the file, %llu copies checked\n",
                direct ? "O_DIRECT" : "buffered", (unsigned long long)chunks.load(),
                (unsigned long long)disk_bytes.load(), (unsigned long long)copies);
}

int main(int argc, char **argv)
{
    const int ops = argc > 1 ? std::atoi(argv[1]) : 3000;
    if (argc > 2) {
        real_tiers(ops, argv[2], 0);
        real_tiers(ops, argv[2], 1);
        std::printf("threads_host ok\n");
        return 0;
    }
    ha_rag_config cfg;
    std::memset(&cfg, 0, sizeof cfg);
    cfg.n_layers = 2;
    cfg.n_kv_heads = 2;
    cfg.head_dim = 128;
    cfg.max_chunk_tokens = 64;
    cfg.group_int8 = 64;
    cfg.group_int4 = 64;
    cfg.tau_gpu_ppm = 300000;
    cfg.tau_pin_ppm = 300000;
    cfg.rerank_interval = 5;
    cfg.dry_run = 1;
    ha_rag_ctx *ctx = nullptr;
    REQUIRE(ha_rag_create(&cfg, &ctx) == HA_RAG_OK);
    size_t total = 0;
    REQUIRE(ha_rag_chunk_bytes(2, 2, 128, HA_RAG_PREC_INT4, 64, 64, nullptr, nullptr, &total) == HA_RAG_OK);
    const size_t slot = (total + 4095) & ~(size_t)4095;   // file slots
    const size_t mslot = (total + 255) & ~(size_t)255;     // memory slots
    REQUIRE(ha_rag_register_slab(ctx, HA_RAG_TIER_HBM, HA_RAG_PREC_INT4, (void *)0x100000000000ull, mslot * 6) == HA_RAG_OK);
    REQUIRE(ha_rag_register_slab(ctx, HA_RAG_TIER_PINNED, HA_RAG_PREC_INT4, (void *)0x200000000000ull, mslot * 12) == HA_RAG_OK);
    REQUIRE(ha_rag_register_disk(ctx, HA_RAG_PREC_INT4, "/nonexistent/dry-run", slot * 256) == HA_RAG_OK);
    REQUIRE(ha_rag_register_staging(ctx, (void *)0x300000000000ull, slot * 4) == HA_RAG_OK);
    REQUIRE(ha_rag_register_bounce(ctx, (void *)0x400000000000ull, slot * 2) == HA_RAG_OK);
    for (uint64_t id = 0; id < 32; ++id)
        REQUIRE(ha_rag_pool_insert(ctx, id, HA_RAG_PREC_INT4, 48, nullptr, 0, HA_RAG_TIER_DISK, nullptr) == HA_RAG_OK);

    std::atomic<uint64_t> loads{0}, chunks{0};
    auto worker = [&](int t) {
        uint64_t s = 0x9E3779B97F4A7C15ull * (uint64_t)(t + 1);
        for (int op = 0; op < ops; ++op) {
            const uint64_t what = next(s) % 100;
            if (what < 12) {  // attention over pool chunks, counting accesses: only chunks with an
                              // HBM or pinned copy can be read in place
                uint64_t ids[4];
                const uint32_t n = 1 + (uint32_t)(next(s) % 4);
                for (uint32_t i = 0; i < n; ++i) ids[i] = next(s) % 32;
                ha_rag_attend_request rq;
                std::memset(&rq, 0, sizeof rq);
                rq.q = (const void *)0x600000000000ull;
                rq.out = (float *)(0x610000000000ull + (uint64_t)t * 0x10000000ull);
                rq.n_q = 1 + (uint32_t)(next(s) % 3);
                rq.n_chunks = n;
                size_t need = 0;
                int rc = ha_rag_attend_chunks_workspace_bytes(ctx, ids, &rq, 1, 4, &need);
                REQUIRE(rc == HA_RAG_OK || rc == HA_RAG_ENOENT);
                if (rc == HA_RAG_OK) {
                    // another thread may evict a copy between the two calls: ENOENT again, or a
                    // size that no longer fits is impossible (sizes depend on token counts only)
                    rc = ha_rag_attend_chunks(ctx, ids, &rq, 1, (uint32_t)(next(s) % 2), 4, 0.1f, HA_RAG_ATTEND_COUNT,
                                              (void *)(0x620000000000ull + (uint64_t)t * 0x10000000ull), need, nullptr);
                    REQUIRE(rc == HA_RAG_OK || rc == HA_RAG_ENOENT);
                    if (rc == HA_RAG_OK) chunks.fetch_add(n);
                }
            } else if (what < 22) {  // placement without a decode, every chunk ends up device-visible
                uint64_t ids[3];
                const uint32_t n = 1 + (uint32_t)(next(s) % 3);
                for (uint32_t i = 0; i < n; ++i) ids[i] = next(s) % 32;
                ha_rag_load_stats st;
                REQUIRE(ha_rag_place_chunks(ctx, ids, nullptr, n, (uint32_t)(next(s) % 2), nullptr, &st, nullptr) == HA_RAG_OK);
                REQUIRE(st.n_chunks == n);
                chunks.fetch_add(n);
            } else if (what < 60) {
                uint64_t ids[6];
                const uint32_t n = 1 + (uint32_t)(next(s) % 6);
                for (uint32_t i = 0; i < n; ++i) ids[i] = next(s) % 32;
                ha_rag_load_stats st;
                int rc = ha_rag_load_chunks(ctx, ids, nullptr, n, (void *)(0x500000000000ull + (uint64_t)t * 0x10000000ull),
                                            6 * 64, 0, nullptr, &st, nullptr);
                REQUIRE(rc == HA_RAG_OK);
                REQUIRE(st.n_chunks == n);
                loads.fetch_add(1);
                chunks.fetch_add(n);
            } else if (what < 70) {
                const uint64_t id = 100 + (uint64_t)t * 1000 + next(s) % 40;   // ids of this thread only
                int rc = ha_rag_pool_insert(ctx, id, HA_RAG_PREC_INT4, 1 + (uint32_t)(next(s) % 64), nullptr, 0,
                                            HA_RAG_TIER_DISK, nullptr);
                REQUIRE(rc == HA_RAG_OK || rc == HA_RAG_EINVAL || rc == HA_RAG_ENOSPC || rc == HA_RAG_EFORMAT);
            } else if (what < 78) {
                int rc = ha_rag_pool_evict(ctx, next(s) % 32, (uint32_t)(next(s) % 2));
                REQUIRE(rc == HA_RAG_OK || rc == HA_RAG_ENOENT || rc == HA_RAG_EINVAL);
            } else if (what < 84) {
                REQUIRE(ha_rag_rerank(ctx) == HA_RAG_OK);
            } else if (what < 92) {
                ha_rag_chunk_info info;
                REQUIRE(ha_rag_pool_query(ctx, next(s) % 32, &info) == HA_RAG_OK);
                REQUIRE(info.on_disk == 1);
            } else {
                uint64_t lru[64];
                size_t n = 0;
                REQUIRE(ha_rag_pool_lru(ctx, (uint32_t)(next(s) % 2), lru, 64, &n) == HA_RAG_OK);
                REQUIRE(n <= 12);
            }
        }
    };
    std::vector<std::thread> th;
    for (int t = 0; t < 4; ++t) th.emplace_back(worker, t);
    for (auto &x : th) x.join();

    // every access was counted exactly once
    uint64_t counted = 0;
    for (uint64_t id = 0; id < 32; ++id) {
        ha_rag_chunk_info info;
        REQUIRE(ha_rag_pool_query(ctx, id, &info) == HA_RAG_OK);
        counted += info.count;
    }
    REQUIRE(counted == chunks.load());
    REQUIRE(ha_rag_destroy(ctx) == HA_RAG_OK);
    std::printf("threads_host ok: %llu loads, %llu chunks\n", (unsigned long long)loads.load(),
                (unsigned long long)chunks.load());
    return 0;
}
