// Random sequences of pool / hotness / load calls on dry_run contexts (host
// bookkeeping only: no HIP call, no byte moved), meant to be built with
// -fsanitize=address,undefined on the host side.  Checks a few invariants after
// every call and exits non-zero on the first violation.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <set>
#include <vector>

#include "../../include/ha_rag.h"

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint64_t rnd()
{
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return rng_state;
}

#define REQUIRE(cond)                                                          \
    do {                                                                       \
        if (!(cond)) {                                                         \
            std::fprintf(stderr, "fuzz_host: %s failed at line %d\n", #cond, __LINE__); \
            std::exit(1);                                                      \
        }                                                                      \
    } while (0)

int main(int argc, char **argv)
{
    const int rounds = argc > 1 ? std::atoi(argv[1]) : 200;
    for (int round = 0; round < rounds; ++round) {
        ha_rag_config cfg;
        std::memset(&cfg, 0, sizeof cfg);
        cfg.n_layers = 1 + rnd() % 3;
        cfg.n_kv_heads = 1 + rnd() % 3;
        cfg.head_dim = 128;
        cfg.max_chunk_tokens = 16 + rnd() % 100;
        cfg.group_int8 = 128;
        cfg.group_int4 = 64;
        cfg.tau_gpu_ppm = (uint32_t)(rnd() % 1000001);
        cfg.rerank_interval = (uint32_t)(rnd() % 4);
        cfg.tau_pin_ppm = (uint32_t)(rnd() % 400001);
        cfg.tau_page_ppm = (uint32_t)(rnd() % 400001);
        cfg.disk_o_direct = (uint32_t)(rnd() % 2);
        cfg.half_slots = (uint32_t)(rnd() % 3 == 0);
        cfg.dry_run = 1;
        ha_rag_ctx *ctx = nullptr;
        REQUIRE(ha_rag_create(&cfg, &ctx) == HA_RAG_OK);
        const uint32_t hbm_slots = 1 + rnd() % 4, pin_slots = 4 + rnd() % 12;
        size_t slot[HA_RAG_N_PREC];
        for (uint32_t p = 0; p < HA_RAG_N_PREC; ++p) {
            size_t total;
            const uint32_t g = p == HA_RAG_PREC_INT8 ? 128 : 64;
            REQUIRE(ha_rag_chunk_bytes(cfg.n_layers, cfg.n_kv_heads, cfg.head_dim, p, g,
                                       cfg.max_chunk_tokens, nullptr, nullptr, &total) == HA_RAG_OK);
            if (cfg.half_slots) total /= 2;
            slot[p] = (total + 255) & ~(size_t)255;
            REQUIRE(ha_rag_register_slab(ctx, HA_RAG_TIER_HBM, p, (void *)(0x100000000000ull + p * 0x10000000000ull),
                                         slot[p] * hbm_slots) == HA_RAG_OK);
            REQUIRE(ha_rag_register_slab(ctx, HA_RAG_TIER_PINNED, p, (void *)(0x200000000000ull + p * 0x10000000000ull),
                                         slot[p] * pin_slots) == HA_RAG_OK);
            REQUIRE(ha_rag_register_slab(ctx, HA_RAG_TIER_PAGEABLE, p, (void *)(0x500000000000ull + p * 0x10000000000ull),
                                         slot[p] * (1 + rnd() % 4)) == HA_RAG_OK);
            REQUIRE(ha_rag_register_disk(ctx, p, "/nonexistent/dry-run", (slot[p] + 4096) * 24) == HA_RAG_OK);
        }
        REQUIRE(ha_rag_register_staging(ctx, (void *)0x300000000000ull, (slot[0] + 4096) * (2 + rnd() % 3)) == HA_RAG_OK);
        REQUIRE(ha_rag_register_bounce(ctx, (void *)0x600000000000ull, (slot[0] + 8192) * (2 + rnd() % 2)) == HA_RAG_OK);
        // Attention over well-formed lists of any shape: a context without a device still cuts the
        // requests' blocks into runs, fills every launch's descriptors and runs the launches' own
        // checks on them, so an inconsistent descriptor shows as a HIP error here.
        for (int k = 0; k < 3; ++k) {
            const uint32_t n_reqs = 1 + (uint32_t)(rnd() % 5);
            std::vector<ha_rag_attend_request> rq(n_reqs);
            std::vector<ha_rag_packed_chunk> ch;
            const uint32_t n_qh = cfg.n_kv_heads * (1 + (uint32_t)(rnd() % 8));
            for (uint32_t r = 0; r < n_reqs; ++r) {
                std::memset(&rq[r], 0, sizeof rq[r]);
                rq[r].q = (const void *)0x720000000000ull;
                rq[r].out = (float *)0x730000000000ull;
                rq[r].lse = rnd() % 2 ? nullptr : (float *)0x740000000000ull;
                const uint64_t kind = rnd() % 4;
                rq[r].n_q = kind == 0 ? 1 : kind == 1 ? 1 + (uint32_t)(rnd() % 8) : 1 + (uint32_t)(rnd() % 300);
                const uint64_t many = rnd() % 4;
                rq[r].n_chunks = many == 0 ? 100 + (uint32_t)(rnd() % 500) : (uint32_t)(rnd() % 12);
                for (uint32_t i = 0; i < rq[r].n_chunks; ++i) {
                    ha_rag_packed_chunk pc;
                    pc.packed = (const void *)(0x750000000000ull + 16 * (rnd() % 100000));
                    pc.n_tokens = many == 0 ? (uint32_t)(rnd() % 60) : (uint32_t)(rnd() % 4000);
                    pc.prec = (uint32_t)(rnd() % HA_RAG_N_PREC);
                    pc.group = pc.prec == HA_RAG_PREC_INT8 ? 128 : pc.prec == HA_RAG_PREC_INT4 ? 64 : 0;
                    pc.part = HA_RAG_PART_KV;
                    ch.push_back(pc);
                }
            }
            size_t need = 0;
            REQUIRE(ha_rag_attend_workspace_bytes(ctx, ch.data(), rq.data(), n_reqs, n_qh, &need) == HA_RAG_OK);
            const int rc = ha_rag_attend_packed(ctx, ch.data(), rq.data(), n_reqs, 0, n_qh, 0.1f,
                                                (void *)0x760000000000ull, need, nullptr);
            if (rc != HA_RAG_OK) std::fprintf(stderr, "fuzz_host: attend_packed %d: %s\n", rc, ha_rag_last_hip_error(ctx));
            REQUIRE(rc == HA_RAG_OK);
            const int rs = ha_rag_attend_packed_static(ctx, ch.data(), rq.data(), n_reqs, 0, n_qh, 0.1f, nullptr);
            REQUIRE(rs == HA_RAG_OK || rs == HA_RAG_ENOSPC);
        }
        std::vector<uint64_t> known;
        for (int op = 0; op < 400; ++op) {
            const uint64_t what = rnd() % 100;
            if (what < 25) {  // insert somewhere
                const uint64_t id = rnd() % 40;
                const uint32_t prec = rnd() % HA_RAG_N_PREC, tier = rnd() % 4;
                const uint32_t tok = 1 + rnd() % cfg.max_chunk_tokens;
                const uint32_t part = rnd() % 3;  // whole chunks, key units, value units
                int rc = part == HA_RAG_PART_KV
                             ? ha_rag_pool_insert(ctx, id, prec, tok, nullptr, 0, tier, nullptr)
                             : ha_rag_pool_insert_half(ctx, id, part, prec, tok, nullptr, 0, tier, nullptr);
                REQUIRE(rc == HA_RAG_OK || rc == HA_RAG_EINVAL || rc == HA_RAG_ENOSPC || rc == HA_RAG_EFORMAT);
                if (rc == HA_RAG_OK) known.push_back(id);
            } else if (what < 75 && !known.empty()) {  // a request (single or batch)
                const uint32_t n_req = 1 + rnd() % 3;
                std::vector<uint64_t> ids;
                std::vector<uint32_t> starts(1, 0);
                std::vector<void *> outs;
                std::vector<uint64_t> caps, bases;
                for (uint32_t r = 0; r < n_req; ++r) {
                    const uint32_t k = rnd() % 7;
                    for (uint32_t i = 0; i < k; ++i)
                        ids.push_back(rnd() % 50 == 0 ? 999 : known[rnd() % known.size()]);
                    starts.push_back((uint32_t)ids.size());
                    outs.push_back((void *)(0x400000000000ull + r * 0x1000000000ull));
                    caps.push_back(rnd() % 5 == 0 ? 10 : 7 * (uint64_t)cfg.max_chunk_tokens + 5);
                    bases.push_back(rnd() % 6);
                }
                std::vector<ha_rag_chunk_trace> tr(ids.size() + 1);
                ha_rag_load_stats st;
                int rc = ha_rag_load_batch(ctx, ids.data(), nullptr, starts.data(), n_req, outs.data(),
                                           caps.data(), bases.data(), nullptr, &st, tr.data());
                // EINVAL: key and value planes of a request that do not line up
                REQUIRE(rc == HA_RAG_OK || rc == HA_RAG_ENOENT || rc == HA_RAG_ENOSPC || rc == HA_RAG_EINVAL);
                if (rc == HA_RAG_OK) {
                    REQUIRE(st.n_chunks == ids.size());
                    REQUIRE(st.n_hbm_hits + st.n_pinned_hits + st.n_pageable_hits + st.n_disk_hits == st.n_chunks);
                    REQUIRE(st.n_evicted <= st.n_promoted + st.n_placed_host);
                }
            } else if (what < 79 && !known.empty()) {  // one request into a paged cache
                std::vector<uint64_t> ids;
                const uint32_t k = rnd() % 6;
                for (uint32_t i = 0; i < k; ++i) ids.push_back(known[rnd() % known.size()]);
                ha_rag_paged_cache pc;
                std::memset(&pc, 0, sizeof pc);
                pc.base = (void *)0x700000000000ull;
                pc.page_table = (const uint32_t *)0x710000000000ull;
                pc.page_tokens = 4u << (rnd() % 4);
                pc.n_table = (uint32_t)(rnd() % 64);
                pc.n_pages = 1 + (uint32_t)(rnd() % 100);
                pc.page_stride = 16 * (1 + rnd() % 1000);
                pc.tile_stride = 16 * (1 + rnd() % 1000);
                ha_rag_load_stats st;
                int rc = ha_rag_load_chunks_paged(ctx, ids.data(), nullptr, (uint32_t)ids.size(), &pc,
                                                  rnd() % 4, nullptr, &st, nullptr);
                REQUIRE(rc == HA_RAG_OK || rc == HA_RAG_ENOSPC || rc == HA_RAG_EINVAL || rc == HA_RAG_ENOENT);
            } else if (what < 80 && rnd() % 2) {  // attention over packed chunks: lists of random shape
                const uint32_t n_reqs = (uint32_t)(rnd() % 5);
                std::vector<ha_rag_attend_request> rq(n_reqs + 1);
                std::vector<ha_rag_packed_chunk> ch;
                for (uint32_t r = 0; r < n_reqs; ++r) {
                    std::memset(&rq[r], 0, sizeof rq[r]);
                    rq[r].q = (const void *)(0x720000000000ull + (rnd() % 8 == 0 ? 2 : 0));
                    rq[r].out = rnd() % 9 == 0 ? nullptr : (float *)0x730000000000ull;
                    rq[r].lse = rnd() % 2 ? nullptr : (float *)0x740000000000ull;
                    rq[r].n_q = (uint32_t)(rnd() % 10 == 0 ? 5000 : rnd() % 70);
                    rq[r].n_chunks = (uint32_t)(rnd() % 6);
                    for (uint32_t i = 0; i < rq[r].n_chunks; ++i) {
                        ha_rag_packed_chunk pc;
                        pc.packed = (const void *)(0x750000000000ull + 16 * (rnd() % 1000) + (rnd() % 16 == 0 ? 4 : 0));
                        pc.n_tokens = (uint32_t)(rnd() % 12 == 0 ? 0 : rnd() % 5000);
                        pc.prec = (uint32_t)(rnd() % (HA_RAG_N_PREC + 1));
                        pc.group = 32u << (rnd() % 4);
                        pc.part = (uint32_t)(rnd() % 8 == 0 ? rnd() % 4 : 0);
                        ch.push_back(pc);
                    }
                }
                const uint32_t n_qh = cfg.n_kv_heads * (uint32_t)(rnd() % 6) + (rnd() % 9 == 0 ? 1 : 0);
                size_t need = 0;
                int rc = ha_rag_attend_workspace_bytes(ctx, ch.data(), rq.data(), n_reqs, n_qh, &need);
                REQUIRE(rc == HA_RAG_OK || rc == HA_RAG_EINVAL || rc == HA_RAG_EFORMAT);
                const size_t have = rnd() % 4 == 0 ? need / 2 : need;
                int rc2 = ha_rag_attend_packed(ctx, ch.data(), rq.data(), n_reqs, (uint32_t)(rnd() % 4), n_qh,
                                               rnd() % 10 == 0 ? -1.0f : 0.1f, (void *)0x760000000000ull, have,
                                               nullptr);
                REQUIRE(rc2 == HA_RAG_OK || rc2 == HA_RAG_EINVAL || rc2 == HA_RAG_EFORMAT || rc2 == HA_RAG_ENOSPC);
                if (rc != HA_RAG_OK) REQUIRE(rc2 != HA_RAG_OK);
                if (rc2 == HA_RAG_ENOSPC) REQUIRE(have < need);
            } else if (what < 80) {  // save the index, damage a copy of it at random, load both
                const char *good = "/tmp/ha_rag_fuzz.idx", *bad = "/tmp/ha_rag_fuzz_bad.idx";
                REQUIRE(ha_rag_pool_save_index(ctx, good) == HA_RAG_OK);
                std::vector<unsigned char> bytes;
                if (FILE *f = std::fopen(good, "rb")) {
                    int ch;
                    while ((ch = std::fgetc(f)) != EOF) bytes.push_back((unsigned char)ch);
                    std::fclose(f);
                }
                REQUIRE(bytes.size() >= 64);
                const uint64_t how = rnd() % 3;
                if (how == 0) bytes.resize(rnd() % bytes.size());            // truncated
                else for (int k = 0; k < 4; ++k) bytes[rnd() % bytes.size()] ^= (unsigned char)(1u << (rnd() % 8));
                if (FILE *f = std::fopen(bad, "wb")) {
                    if (!bytes.empty()) std::fwrite(bytes.data(), 1, bytes.size(), f);
                    std::fclose(f);
                }
                ha_rag_ctx *other = nullptr;
                REQUIRE(ha_rag_create(&cfg, &other) == HA_RAG_OK);
                for (uint32_t p = 0; p < HA_RAG_N_PREC; ++p)
                    REQUIRE(ha_rag_register_disk(other, p, "/nonexistent/dry-run", (slot[p] + 4096) * 24) == HA_RAG_OK);
                size_t n_loaded = 0;
                int rc = ha_rag_pool_load_index(other, bad, &n_loaded);      // any verdict, no crash
                REQUIRE(rc == HA_RAG_OK || rc == HA_RAG_EIO || rc == HA_RAG_EFORMAT || rc == HA_RAG_EINVAL);
                if (rc != HA_RAG_OK) REQUIRE(ha_rag_pool_load_index(other, good, &n_loaded) == HA_RAG_OK);
                REQUIRE(ha_rag_destroy(other) == HA_RAG_OK);
            } else if (what < 81 && !known.empty()) {  // Algorithm 2 without the decode
                uint64_t ids3[5];
                const uint32_t k = (uint32_t)(rnd() % 6);
                for (uint32_t i = 0; i < k && i < 5; ++i) ids3[i] = rnd() % 30 == 0 ? 999 : known[rnd() % known.size()];
                ha_rag_load_stats st;
                ha_rag_chunk_trace tr[5];
                int rc = ha_rag_place_chunks(ctx, ids3, nullptr, k < 5 ? k : 5, (uint32_t)(rnd() % 2), nullptr, &st, tr);
                REQUIRE(rc == HA_RAG_OK || rc == HA_RAG_ENOENT || rc == HA_RAG_ENOSPC);
                if (rc == HA_RAG_OK) REQUIRE(st.n_kernel_launches == 0 && st.bf16_bytes_written == 0);
            } else if (what < 82 && !known.empty()) {
                int rc = ha_rag_pool_promote(ctx, known[rnd() % known.size()], nullptr);
                REQUIRE(rc == HA_RAG_OK || rc == HA_RAG_ENOSPC || rc == HA_RAG_ENOENT);
            } else if (what < 88 && !known.empty()) {
                int rc = ha_rag_pool_evict(ctx, known[rnd() % known.size()], (uint32_t)(rnd() % 3));
                REQUIRE(rc == HA_RAG_OK || rc == HA_RAG_EINVAL || rc == HA_RAG_ENOENT);
            } else if (what < 90 && !known.empty()) {
                int rc = ha_rag_pool_remove(ctx, known[rnd() % known.size()]);
                REQUIRE(rc == HA_RAG_OK || rc == HA_RAG_ENOENT);
            } else if (what < 94) {
                REQUIRE(ha_rag_rerank(ctx) == HA_RAG_OK);
            } else if (!known.empty()) {
                uint64_t ids2[3] = {known[rnd() % known.size()], known[rnd() % known.size()], rnd() % 60};
                int rc = ha_rag_touch(ctx, ids2, 3);
                REQUIRE(rc == HA_RAG_OK || rc == HA_RAG_ENOENT);
            }
            // invariants: residency lists are consistent with per-chunk queries
            uint64_t lru[256];
            size_t n_lru = 0;
            REQUIRE(ha_rag_pool_lru(ctx, HA_RAG_TIER_HBM, lru, 256, &n_lru) == HA_RAG_OK);
            REQUIRE(n_lru <= (size_t)hbm_slots * HA_RAG_N_PREC);
            std::set<uint64_t> seen;
            for (size_t i = 0; i < n_lru; ++i) {
                REQUIRE(seen.insert(lru[i]).second);
                ha_rag_chunk_info info;
                REQUIRE(ha_rag_pool_query(ctx, lru[i], &info) == HA_RAG_OK);
                REQUIRE(info.in_hbm == 1 && info.hbm_ptr != nullptr);
                void *p = nullptr;
                size_t nb = 0;
                REQUIRE(ha_rag_pool_slot(ctx, lru[i], HA_RAG_TIER_HBM, &p, &nb) == HA_RAG_OK);
                REQUIRE(p == info.hbm_ptr && nb == info.bytes && nb <= slot[info.prec]);
            }
        }
        REQUIRE(ha_rag_destroy(ctx) == HA_RAG_OK);
    }
    std::printf("fuzz_host ok: %d rounds\n", rounds);
    return 0;
}
