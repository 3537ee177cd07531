// Context life cycle, stateless helpers and the offline entry points of include/ha_rag.h
// (sizes, Algorithm 1's split, quantize-pack, the error metric of Eq. 1).
#include "ha_rag_internal.h"

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <new>

#include <unistd.h>

using namespace ha_rag_host;

namespace ha_rag_host {
thread_local std::string g_create_err;
}

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
    // group 0 = the context does not use that integer tag (a head_dim that no group size divides
    // can still hold 16-bit, FP8 and GSE-8 chunks)
    for (uint32_t grp : {cfg->group_int8, cfg->group_int4})
        if (grp != 0 && (!valid_group(grp) || (cfg->head_dim % grp))) return HA_RAG_EFORMAT;
    if (cfg->tau_gpu_ppm > kPPM || cfg->tau_pin_ppm > kPPM || cfg->tau_page_ppm > kPPM ||
        cfg->n_copy_streams > 8 || cfg->io_threads > 64)
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
        // the library's set-up on this device: where its static scratch array lives here, and
        // the LDS allowance of the eight-wave attention kernel
        hipError_t pe = hipSuccess;
        if (attend_static_scratch(nullptr, &g_create_err) != HA_RAG_OK ||
            (pe = ha_rag::prepare_k6_shared()) != hipSuccess) {
            if (pe != hipSuccess) g_create_err = std::string("hipFuncSetAttribute(k6_attend_shared): ") + hipGetErrorString(pe);
            for (hipStream_t t : c->copy_streams) (void)hipStreamDestroy(t);
            delete c;
            return HA_RAG_EHIP;
        }
    }
    *out = c;
    return HA_RAG_OK;
}

int ha_rag_destroy(ha_rag_ctx *c)
{
    if (!c) return HA_RAG_EINVAL;
    if (c->io) io_pool_destroy(c->io);  // joins the I/O threads; no call is running any more
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
    if (lp->planes16 != 0 && lp->planes16 != 1 && lp->planes16 != 2 && lp->planes16 != 4) return HA_RAG_EINVAL;
    if (lp->planes8 != 0 && lp->planes8 != 2 && lp->planes8 != 4) return HA_RAG_EINVAL;
    std::lock_guard<std::mutex> g(c->mu);
    c->launch = K1Launch{lp->threads, lp->planes16, lp->planes8, lp->nt_store != 0,
                         lp->nt_load != 0};
    return HA_RAG_OK;
}

// n chunks of one tag, one launch per kMaxK2Chunks of them
static int quantize_impl(ha_rag_ctx *c, const void *const *srcs, void *const *dsts, const uint32_t *n_tokens,
                         uint32_t n, uint32_t prec, uint32_t group, uint32_t *saturated, void *stream,
                         uint32_t part)
{
    if (!c || (n && (!srcs || !dsts || !n_tokens))) return HA_RAG_EINVAL;
    if ((uintptr_t)saturated & 3u) return HA_RAG_EINVAL;
    for (uint32_t i = 0; i < n; ++i) {
        if (!srcs[i] || !dsts[i] || ((uintptr_t)srcs[i] & 15u) || ((uintptr_t)dsts[i] & 15u)) return HA_RAG_EINVAL;
        int rc = chunk_bytes_impl(c->cfg.n_layers, c->cfg.n_kv_heads, c->cfg.head_dim, prec, group,
                                  n_tokens[i], nullptr, nullptr, nullptr, part);
        if (rc) return rc;
    }
    if (c->dry()) return HA_RAG_OK;
    std::lock_guard<std::mutex> g(c->mu);
    K2Params p{};
    p.n_tiles = part == kPartKV ? c->n_tiles : c->n_tiles / 2;
    p.head_dim = c->cfg.head_dim;
    p.saturated = saturated;
    for (uint32_t i = 0; i < n; ++i) {
        if (n_tokens[i] == 0) continue;  // holds nothing: nothing to write
        p.c[p.n_chunks++] = K2Chunk{static_cast<const uint8_t *>(srcs[i]), static_cast<uint8_t *>(dsts[i]),
                                    n_tokens[i], 0};
        if (p.n_chunks == kMaxK2Chunks) {
            HIPCHK(c, launch_k2(p, prec, has_meta(prec) ? group : 32u, (hipStream_t)stream));
            p.n_chunks = 0;
        }
    }
    if (p.n_chunks) HIPCHK(c, launch_k2(p, prec, has_meta(prec) ? group : 32u, (hipStream_t)stream));
    return HA_RAG_OK;
}

int ha_rag_quantize_chunk(ha_rag_ctx *c, const void *src, uint32_t n_tokens, uint32_t prec,
                          uint32_t group, void *dst, uint32_t *saturated, void *stream)
{
    return quantize_impl(c, &src, &dst, &n_tokens, 1, prec, group, saturated, stream, kPartKV);
}

int ha_rag_quantize_chunks(ha_rag_ctx *c, const void *const *srcs, void *const *dsts,
                           const uint32_t *n_tokens, uint32_t n, uint32_t prec, uint32_t group,
                           uint32_t *saturated, void *stream)
{
    return quantize_impl(c, srcs, dsts, n_tokens, n, prec, group, saturated, stream, kPartKV);
}

int ha_rag_quantize_half(ha_rag_ctx *c, const void *src, uint32_t n_tokens, uint32_t prec,
                         uint32_t group, void *dst, uint32_t *saturated, void *stream)
{
    // the tile records of a half do not depend on which plane it is
    return quantize_impl(c, &src, &dst, &n_tokens, 1, prec, group, saturated, stream, kPartK);
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
    HIPCHK(c, launch_k8(src, packed, part == kPartKV ? c->n_tiles : c->n_tiles / 2, c->cfg.head_dim,
                        n_tokens, prec, has_meta(prec) ? group : 32u, sum_sq, (hipStream_t)stream));
    return HA_RAG_OK;
}

}  // extern "C"
