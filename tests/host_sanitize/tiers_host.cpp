// The pageable and file tiers with real bytes and real files, but no GPU: contexts with
// dry_run = 2 make no HIP call while host copies and file transfers happen, so slabs, bounce
// buffers and chunk sources are ordinary host memory here.  Meant to be built with
// -fsanitize=address,undefined on the host side; exits non-zero on the first violation.
//   argv[1] = directory for the pool files
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/ha_rag.h"

#define REQUIRE(cond)                                                          \
    do {                                                                       \
        if (!(cond)) {                                                         \
            std::fprintf(stderr, "tiers_host: %s failed at line %d\n", #cond, __LINE__); \
            std::exit(1);                                                      \
        }                                                                      \
    } while (0)

static uint64_t rng_state = 0x2545F4914F6CDD1Dull;
static uint64_t rnd()
{
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return rng_state;
}

static void *aligned(size_t bytes)
{
    void *p = nullptr;
    REQUIRE(posix_memalign(&p, 4096, bytes ? bytes : 4096) == 0);
    std::memset(p, 0xEE, bytes);
    return p;
}

static std::vector<uint8_t> random_bytes(size_t n)
{
    std::vector<uint8_t> v(n);
    for (size_t i = 0; i < n; ++i) v[i] = (uint8_t)rnd();
    return v;
}

static ha_rag_config base_config(uint32_t direct)
{
    ha_rag_config cfg;
    std::memset(&cfg, 0, sizeof cfg);
    cfg.n_layers = 2;
    cfg.n_kv_heads = 2;
    cfg.head_dim = 128;
    cfg.max_chunk_tokens = 48;
    cfg.group_int8 = 128;
    cfg.group_int4 = 128;
    cfg.tau_gpu_ppm = 0;
    cfg.tau_pin_ppm = 300000;
    cfg.tau_page_ppm = 300000;
    cfg.disk_o_direct = direct;
    cfg.dry_run = 2;
    return cfg;
}

static size_t chunk_bytes(const ha_rag_config &cfg, uint32_t prec, uint32_t tokens)
{
    size_t total = 0;
    REQUIRE(ha_rag_chunk_bytes(cfg.n_layers, cfg.n_kv_heads, cfg.head_dim, prec, 128, tokens, nullptr,
                               nullptr, &total) == HA_RAG_OK);
    return total;
}

// A file slab of a larger tag registered after the bounce buffers: the direct-I/O buffer was
// sized for the smaller one, and a host-source insert into the larger file must be refused, not
// written past that buffer.
static void direct_buffer_is_not_overrun(const std::string &dir)
{
    ha_rag_config cfg = base_config(1);
    ha_rag_ctx *ctx = nullptr;
    REQUIRE(ha_rag_create(&cfg, &ctx) == HA_RAG_OK);
    const size_t small = chunk_bytes(cfg, HA_RAG_PREC_INT4, cfg.max_chunk_tokens);
    const size_t large = chunk_bytes(cfg, HA_RAG_PREC_16, cfg.max_chunk_tokens);
    REQUIRE(large > small + 8192);
    REQUIRE(ha_rag_register_disk(ctx, HA_RAG_PREC_INT4, (dir + "/small.pool").c_str(), (small + 4096) * 4) == HA_RAG_OK);
    void *bounce = aligned((small + 4096) * 2);
    REQUIRE(ha_rag_register_bounce(ctx, bounce, (small + 4096) * 2) == HA_RAG_OK);
    REQUIRE(ha_rag_register_disk(ctx, HA_RAG_PREC_16, (dir + "/large.pool").c_str(), (large + 4096) * 4) == HA_RAG_OK);
    std::vector<uint8_t> a = random_bytes(small), b = random_bytes(large);
    REQUIRE(ha_rag_pool_insert(ctx, 1, HA_RAG_PREC_INT4, cfg.max_chunk_tokens, a.data(), 0, HA_RAG_TIER_DISK, nullptr) == HA_RAG_OK);
    REQUIRE(ha_rag_pool_insert(ctx, 2, HA_RAG_PREC_16, cfg.max_chunk_tokens, b.data(), 0, HA_RAG_TIER_DISK, nullptr) == HA_RAG_ENOSPC);
    ha_rag_chunk_info info;
    REQUIRE(ha_rag_pool_query(ctx, 2, &info) == HA_RAG_ENOENT);  // a refused insert leaves nothing behind
    REQUIRE(ha_rag_destroy(ctx) == HA_RAG_OK);
    std::free(bounce);
}

// Chunks inserted into files and pageable memory come back byte for byte in pinned memory
// through Algorithm 2's placement (file -> bounce buffer -> pinned slot), with and without
// direct I/O.
static void bytes_survive_the_tiers(const std::string &dir, uint32_t direct)
{
    ha_rag_config cfg = base_config(direct);
    ha_rag_ctx *ctx = nullptr;
    REQUIRE(ha_rag_create(&cfg, &ctx) == HA_RAG_OK);
    const uint32_t precs[3] = {HA_RAG_PREC_16, HA_RAG_PREC_INT8, HA_RAG_PREC_INT4};
    size_t slot[3], largest = 0;
    std::vector<void *> mem;
    const uint32_t n_pin = 3, n_page = 2, n_disk = 30;
    for (int k = 0; k < 3; ++k) {
        slot[k] = (chunk_bytes(cfg, precs[k], cfg.max_chunk_tokens) + 4095) & ~(size_t)4095;
        if (slot[k] > largest) largest = slot[k];
        void *pin = aligned(slot[k] * n_pin), *page = aligned(slot[k] * n_page);
        mem.push_back(pin);
        mem.push_back(page);
        REQUIRE(ha_rag_register_slab(ctx, HA_RAG_TIER_PINNED, precs[k], pin, slot[k] * n_pin) == HA_RAG_OK);
        REQUIRE(ha_rag_register_slab(ctx, HA_RAG_TIER_PAGEABLE, precs[k], page, slot[k] * n_page) == HA_RAG_OK);
        const std::string path = dir + "/tier" + std::to_string(k) + (direct ? "d" : "b") + ".pool";
        REQUIRE(ha_rag_register_disk(ctx, precs[k], path.c_str(), slot[k] * n_disk) == HA_RAG_OK);
    }
    void *bounce = aligned(largest * 3);
    mem.push_back(bounce);
    REQUIRE(ha_rag_register_bounce(ctx, bounce, largest * 3) == HA_RAG_OK);
    struct Doc {
        uint64_t id;
        uint32_t prec, tokens;
        std::vector<uint8_t> bytes;
    };
    std::vector<Doc> docs;
    for (uint64_t id = 0; id < 30; ++id) {
        Doc d;
        d.id = id;
        d.prec = precs[rnd() % 3];
        d.tokens = 1 + (uint32_t)(rnd() % cfg.max_chunk_tokens);
        d.bytes = random_bytes(chunk_bytes(cfg, d.prec, d.tokens));
        REQUIRE(ha_rag_pool_insert(ctx, id, d.prec, d.tokens, d.bytes.data(), 0, HA_RAG_TIER_DISK, nullptr) == HA_RAG_OK);
        docs.push_back(d);
    }
    std::vector<uint64_t> ids, counts;
    for (const Doc &d : docs) {
        ids.push_back(d.id);
        counts.push_back(1000 - d.id);
    }
    REQUIRE(ha_rag_set_counts(ctx, ids.data(), counts.data(), ids.size()) == HA_RAG_OK);
    REQUIRE(ha_rag_rerank(ctx) == HA_RAG_OK);
    for (int round = 0; round < 60; ++round) {
        uint64_t req[4];
        const uint32_t n = 1 + (uint32_t)(rnd() % 4);
        for (uint32_t i = 0; i < n; ++i) req[i] = rnd() % docs.size();
        ha_rag_load_stats st;
        ha_rag_chunk_trace tr[4];
        // odd rounds: every chunk ends up device-visible (a pinned copy); even rounds: plain
        // Algorithm 2 through a load whose kernels and device copies are skipped
        if (round & 1) {
            REQUIRE(ha_rag_place_chunks(ctx, req, nullptr, n, HA_RAG_PLACE_DEVICE_VISIBLE, nullptr, &st, tr) == HA_RAG_OK);
        } else {
            REQUIRE(ha_rag_place_chunks(ctx, req, nullptr, n, 0, nullptr, &st, tr) == HA_RAG_OK);
        }
        for (uint32_t i = 0; i < n; ++i) {
            const Doc &d = docs[req[i]];
            for (uint32_t tier : {(uint32_t)HA_RAG_TIER_PINNED, (uint32_t)HA_RAG_TIER_PAGEABLE}) {
                void *p = nullptr;
                size_t nb = 0;
                const int rc = ha_rag_pool_slot(ctx, d.id, tier, &p, &nb);
                REQUIRE(rc == HA_RAG_OK || rc == HA_RAG_ENOENT);
                if (rc == HA_RAG_OK) {
                    REQUIRE(nb == d.bytes.size());
                    REQUIRE(std::memcmp(p, d.bytes.data(), nb) == 0);
                }
            }
        }
    }
    // every resident copy, not only the ones just touched
    for (const Doc &d : docs) {
        for (uint32_t tier : {(uint32_t)HA_RAG_TIER_PINNED, (uint32_t)HA_RAG_TIER_PAGEABLE}) {
            void *p = nullptr;
            size_t nb = 0;
            if (ha_rag_pool_slot(ctx, d.id, tier, &p, &nb) == HA_RAG_OK)
                REQUIRE(nb == d.bytes.size() && std::memcmp(p, d.bytes.data(), nb) == 0);
        }
    }
    REQUIRE(ha_rag_destroy(ctx) == HA_RAG_OK);
    for (void *p : mem) std::free(p);
}

int main(int argc, char **argv)
{
    REQUIRE(argc > 1);
    const std::string dir = argv[1];
    direct_buffer_is_not_overrun(dir);
    bytes_survive_the_tiers(dir, 0);
    bytes_survive_the_tiers(dir, 1);
    std::printf("tiers_host ok\n");
    return 0;
}
