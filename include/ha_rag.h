/*
 * ha_rag.h -- C ABI of the MI355X (gfx950) hotness-aware mixed-precision KV-chunk
 * load: the hot path of HA-RAG ("HA-RAG: Hotness-Aware RAG Acceleration via Mixed
 * Precision and Data Placement").
 *
 * A *chunk* is the precomputed K and V of one retrieved document (Sec. 1: the
 * KV of each document chunk is computed once, stored, and loaded on demand),
 * shape [L layers][2 = K,V][H kv heads][T tokens][D head_dim], BF16 at full
 * precision (Sec. 2.2.1).  Offline, each chunk is compressed to a precision
 * chosen from its access-frequency rank (Algorithm 1); online, the chunks a
 * request retrieved are looked up in a tiered pool (Algorithm 2: GPU memory, then
 * pinned host memory), moved to the GPU if needed, decompressed and laid one
 * after another along the token axis of one BF16 KV cache
 * out[L][2][H][cap_tokens][D] that prefill can consume (Sec. 2.1, Fig. 3).
 *
 * Conventions
 *  - Every function returns HA_RAG_OK (0) or a negative HA_RAG_E* code; nothing
 *    throws or aborts across this boundary.
 *  - "device pointer" = HBM address valid on the current HIP device; "host
 *    pointer" = ordinary host memory; "pinned pointer" = page-locked host memory
 *    (hipHostMalloc or equivalent).  The CALLER allocates and owns every device
 *    and pinned buffer; the library allocates host metadata, HIP events and its
 *    copy streams only, and never calls hipMalloc.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  GPU
 *    work is enqueued, not awaited: results are valid once the caller has
 *    synchronised `stream`.
 *  - Precision tags: HA_RAG_PREC_16 keeps the BF16 words verbatim; INT8 / INT4
 *    are unsigned codes with one fp16 scale and one fp16 zero per group of
 *    `group` consecutive head_dim elements (value = code * scale + zero).  The
 *    paper fixes only the code range of its integer scheme (Sec. 2.2.2); scale,
 *    zero, group and byte layout are this library's format.  FP8_E4M3 / FP8_E5M2
 *    store one 8-bit float per element (1-4-3, bias 7, no infinities, largest
 *    finite 448; 1-5-2, bias 15, largest finite 57344; Sec. 2.2.2, Fig. 6), encoded
 *    round-to-nearest-even and saturating at the largest finite value, decoded
 *    exactly; no scale/zero, payload laid out like the INT8 payload.  GSE8 stores
 *    sign, a 4-bit index k into the tile's shared exponents and a 3-bit field
 *    (Sec. 2.2.2, Fig. 7): value = +-field * 2^(G_k - 2), G_k = min(e_lo + 2 + 3k,
 *    e_hi), field = floor(|x| * 2^(2 - G_k)) for the smallest G_k >= exponent(x)
 *    (truncating, as the paper's shift does); e_lo / e_hi are the smallest /
 *    largest exponent of the tile's nonzero values (e_lo raised to e_hi - 47 if
 *    the tile spans more than 48 binades).  Payload like INT8, and each tile
 *    record ends with 16 bytes {int8 e_lo, int8 e_hi, 14 zero bytes}.
 *  - Packed byte layout of a chunk: tile records (l*2+kv)*H+h back to back; a tile
 *    is cut into blocks of 2048 elements (last one zero padded); payload blocks
 *    (256*bits bytes each) first, then meta blocks (2048/group entries of
 *    {u16 scale, u16 zero}).  Element r of a block: plane j=r/512, lane i=(r%512)/8,
 *    position p=r%8; the octet (j,i) starts at byte (j/P)*1024 + i*16 + (j%P)*bits
 *    of its payload block, P = 16/bits; group G=r/group is meta entry
 *    (G % (512/group))*4 + G/(512/group).
 *  - A context may be used from several threads.  Its bookkeeping is guarded by an internal
 *    mutex, which the online calls (ha_rag_load_chunks, ha_rag_load_batch, ha_rag_place_chunks)
 *    release while they wait for file reads, host copies or device events, so that requests of
 *    several threads overlap their I/O with each other and with GPU work (the disk tier is where
 *    Sec. 3.4 finds the time goes); a copy one call is still writing is passed over by the
 *    others, which read the chunk from a slower tier.  The offline calls (insert, quantize,
 *    index) keep it locked.  Work that overlaps on the GPU is ordered by the streams and events
 *    described at each function.
 */
#ifndef HA_RAG_H
#define HA_RAG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* the functions declared here are the only symbols the library exports */
#if defined(__GNUC__) || defined(__clang__)
#pragma GCC visibility push(default)
#endif

#define HA_RAG_OK 0
#define HA_RAG_EINVAL (-1)  /* null pointer, bad size, duplicate id, misaligned buffer  */
#define HA_RAG_ENOENT (-2)  /* unknown chunk id                                          */
#define HA_RAG_ENOSPC (-3)  /* pool slab full, output cache too small, staging too small */
#define HA_RAG_EFORMAT (-4) /* tag / group / shape mismatch                              */
#define HA_RAG_EHIP (-5)    /* a HIP call failed; see ha_rag_last_hip_error              */
#define HA_RAG_EIO (-6)     /* a file operation failed; see ha_rag_last_hip_error        */

#define HA_RAG_PREC_16 0
#define HA_RAG_PREC_INT8 1
#define HA_RAG_PREC_INT4 2
#define HA_RAG_PREC_FP8_E4M3 3 /* the paper's scheme S2 (Sec. 2.2.2, Sec. 3.2.1) */
#define HA_RAG_PREC_FP8_E5M2 4 /* the paper's scheme S3                           */
#define HA_RAG_PREC_GSE8 5     /* the paper's scheme S4, GSE-8 with the 1+4+3 split */
#define HA_RAG_N_PREC 6

#define HA_RAG_TIER_HBM 0      /* queueGPU of Algorithm 2                                  */
#define HA_RAG_TIER_PINNED 1   /* queuePIN: page-locked host memory, copied straight to HBM */
#define HA_RAG_TIER_PAGEABLE 2 /* queuePAGE: ordinary host memory; goes through a pinned
                                  bounce buffer on its way to HBM (Sec. 2.3, Fig. 8)       */
#define HA_RAG_TIER_DISK 3     /* a file; read into a pinned bounce buffer first           */
#define HA_RAG_TIER_NONE 255

/* What a chunk holds.  Algorithm 1 ranks the n key chunks and the n value chunks of a
 * knowledge base as 2n units, each with its own access frequency and precision; a
 * keys-only or values-only chunk is such a unit: shape [L][H][T][D], tile records
 * (l, h) back to back, exactly half the bytes of a whole chunk of the same length. */
#define HA_RAG_PART_KV 0 /* keys and values of a document under one id and one tag */
#define HA_RAG_PART_K 1
#define HA_RAG_PART_V 2

#define HA_RAG_NO_CHUNK UINT64_MAX
#define HA_RAG_MAX_REQUEST_CHUNKS 4096

typedef struct ha_rag_ctx ha_rag_ctx;

typedef struct ha_rag_config {
    uint32_t n_layers;         /* L                                                        */
    uint32_t n_kv_heads;       /* H                                                        */
    uint32_t head_dim;         /* D, multiple of 8                                         */
    uint32_t max_chunk_tokens; /* slot size of every slab is that of a chunk this long     */
    uint32_t group_int8;       /* group size of the INT8 tag: 32..512, power of 2, | D; 0 = the
                                  tag is not used by this context (EFORMAT wherever it is
                                  named), e.g. when no group size divides head_dim        */
    uint32_t group_int4;       /* the same for the INT4 tag                                */
    uint32_t tau_gpu_ppm;      /* Algorithm 2 step 1: GPU_LIST = ranks below
                                  idx1 = floor(tau_gpu_ppm * N / 1e6), N = chunks in the pool */
    uint32_t rerank_interval;  /* recompute ranks after this many load calls; 0 = only in
                                  ha_rag_rerank                                            */
    uint32_t n_copy_streams;   /* streams for pinned -> HBM copies (0 = 2, at most 8)      */
    uint32_t dry_run;          /* 1 = host bookkeeping only: no HIP call is ever made, no
                                  byte is moved (for host-logic tests without a GPU).
                                  2 = no HIP call either, but host copies and file transfers
                                  are real: slabs, bounce buffers and chunk sources are then
                                  ordinary host memory (for tests of the host and file tiers
                                  without a GPU)                                           */
    uint32_t tau_pin_ppm;      /* PIN_LIST = ranks [idx1, idx2), idx2 = idx1 +
                                  floor(tau_pin_ppm * N / 1e6)                             */
    uint32_t tau_page_ppm;     /* PAGE_LIST = ranks [idx2, idx3), idx3 = idx2 +
                                  floor(tau_page_ppm * N / 1e6); DISK_LIST = the rest      */
    uint32_t disk_o_direct;    /* 1 = open pool files with O_DIRECT (bypasses the OS page
                                  cache; transfers are rounded up to 4096 bytes and pass
                                  through one page-aligned host buffer that the library
                                  allocates in ha_rag_register_bounce, because direct I/O
                                  cannot target GPU-pinned memory)                         */
    uint32_t half_slots;       /* 1 = every slab slot is sized for a keys-only or values-only
                                  chunk of max_chunk_tokens (a pool that stores the 2n units
                                  of Algorithm 1); whole chunks are then refused (EFORMAT).
                                  0 = slots are sized for whole chunks; halves fit too     */
    uint32_t pinned_dma;       /* how a chunk served from pinned memory that gets no faster copy
                                  reaches the kernel.  0 = the dequantize kernel reads it
                                  straight over the link (pinned memory is device-visible):
                                  no staging slot, no copy stream, one launch per 64 chunks
                                  (measured faster, and insensitive to host load).  1 = it
                                  is copied to the staging area by DMA first, which keeps
                                  the compute units free while the link is busy.  Chunks
                                  that are promoted, or come from pageable memory or a
                                  file, always take the DMA route                         */
    uint32_t io_threads;       /* threads that move chunks from files and pageable memory into
                                  the bounce buffers, in pieces of 4 MiB: the queue depth the
                                  file tier sees from one call (0 = 4, at most 64; created at
                                  the first such transfer)                                 */
} ha_rag_config;

/* One packed chunk handed to ha_rag_load_packed (no pool involved). */
typedef struct ha_rag_packed_chunk {
    const void *packed; /* device pointer, 16-byte aligned, ha_rag_chunk_bytes() bytes */
    uint32_t n_tokens;
    uint32_t prec;      /* HA_RAG_PREC_*                                                */
    uint32_t group;     /* ignored for HA_RAG_PREC_16                                   */
    uint32_t part;      /* HA_RAG_PART_*; a half has half the bytes of a whole chunk    */
} ha_rag_packed_chunk;

typedef struct ha_rag_chunk_info {
    uint32_t prec, group, n_tokens;
    uint32_t in_hbm, in_pinned; /* 0 / 1                                      */
    uint32_t rank;              /* 0 = hottest, as of the last rerank         */
    uint32_t in_pageable, on_disk; /* 0 / 1                                   */
    uint32_t part;              /* HA_RAG_PART_*                              */
    uint32_t disk_slot;         /* slot index in the tag's pool file, or
                                   UINT32_MAX if the chunk has no file copy   */
    uint64_t count;             /* accesses so far (Algorithm 1's AF entry)   */
    uint64_t bytes;             /* packed size                                */
    const void *hbm_ptr;        /* slot address or NULL                       */
    const void *pinned_ptr;     /* slot address or NULL                       */
} ha_rag_chunk_info;

/* A paged KV cache as serving engines keep it: the request's token rows are cut into
 * pages of `page_tokens` rows, and row r lives in physical page page_table[r /
 * page_tokens] at row r % page_tokens.  The BF16 word of (layer l, K/V kv, head h, row r,
 * dim d) is at
 *   base + page * page_stride + ((l*2+kv)*H + h) * tile_stride
 *        + (r % page_tokens) * D * 2 + d * 2            (all strides in bytes).
 * Two common pools: every page one contiguous [L][2][H][page_tokens][D] block
 * (page_stride = 2*L*H*page_tokens*D*2, tile_stride = page_tokens*D*2), or the pool as
 * [L][2][H][n_pages][page_tokens][D] (tile_stride = n_pages*page_tokens*D*2,
 * page_stride = page_tokens*D*2).  The paper hands the loaded chunks to prefill as one
 * concatenated cache (Sec. 2.1); this is the same cache in the layout a paged attention
 * kernel reads. */
typedef struct ha_rag_paged_cache {
    void *base;                 /* device pointer, 16-byte aligned                           */
    const uint32_t *page_table; /* DEVICE pointer to n_table page ids, request order         */
    uint32_t *bad_pages;        /* nullable device pointer to a u32 the kernel adds to: the
                                   number of 16-byte stores it dropped because the table
                                   named a page >= n_pages                                   */
    uint64_t page_stride;       /* multiples of 16                                           */
    uint64_t tile_stride;
    uint32_t page_tokens;       /* page_tokens * D * 2 >= 1024 bytes                         */
    uint32_t n_table;           /* table entries: the request may hold n_table * page_tokens
                                   rows; n_table * page_tokens * D * 2 < 2^32                */
    uint32_t n_pages;           /* physical pages in the pool (page ids are checked against
                                   it on the device; the table itself is never read by the
                                   host)                                                     */
    uint32_t reserved;
} ha_rag_paged_cache;

/* What happened to one chunk of a load (Algorithm 2 step 2, per C_i). */
typedef struct ha_rag_chunk_trace {
    uint64_t tok_off;     /* first token row of this chunk in the cache (of its plane,
                             for a keys-only or values-only chunk)             */
    uint64_t evicted_id;  /* chunk dropped from HBM to make room, or NO_CHUNK  */
    uint8_t found_tier;   /* fastest tier that held the chunk (HA_RAG_TIER_*)   */
    uint8_t promoted;     /* 1 = copied into the HBM slab by this load         */
    uint8_t promote_skipped; /* 1 = its list asked for a faster copy but no slot could be freed */
    uint8_t placed_tier;  /* tier a new copy was placed into, or HA_RAG_TIER_NONE */
    uint8_t reserved[4];
} ha_rag_chunk_trace;

typedef struct ha_rag_load_stats {
    uint32_t n_chunks, n_hbm_hits, n_pinned_hits;
    uint32_t n_promoted;         /* copies placed into HBM                           */
    uint32_t n_evicted, n_promote_skipped, n_kernel_launches;
    uint32_t n_pageable_hits, n_disk_hits;
    uint32_t n_placed_host;      /* copies placed into pinned or pageable memory     */
    uint32_t reserved[2];
    uint64_t tokens;
    uint64_t bytes_h2d;          /* packed bytes that crossed the host link          */
    uint64_t bytes_d2d;          /* packed bytes copied staging -> HBM slab          */
    uint64_t packed_bytes_read;  /* payload + meta bytes the kernels read            */
    uint64_t bf16_bytes_written; /* bytes written to the cache                       */
    uint64_t bytes_disk_read;    /* packed bytes read from files                     */
    uint64_t bytes_host_copied;  /* packed bytes copied host -> host                 */
} ha_rag_load_stats;

/* ---- stateless helpers (no context, no GPU) ------------------------------- */

/* Packed size of a chunk in the layout described above.  `payload`, `meta`,
 * `total` may each be NULL.  EFORMAT if D % 8, group not in {32..512} power of two
 * or not dividing D (group is ignored for PREC_16), unknown prec. */
int ha_rag_chunk_bytes(uint32_t n_layers, uint32_t n_kv_heads, uint32_t head_dim,
                       uint32_t prec, uint32_t group, uint32_t n_tokens,
                       size_t *payload, size_t *meta, size_t *total);

/* Algorithm 1 steps 1-2: sort the n chunks by access frequency `af` (descending;
 * equal counts by ascending index), cut at idx_k = floor(tau_ppm[k] * n / 1e6) +
 * idx_{k-1}, and write the class (0 = hottest .. n_tau = coldest) of every chunk to
 * cls_out[n].  rank_out[n] (nullable) receives each chunk's position in the sort.
 * Host pointers. */
int ha_rag_alg1_classes(const uint64_t *af, size_t n, const uint32_t *tau_ppm, uint32_t n_tau,
                        uint8_t *cls_out, uint32_t *rank_out);

const char *ha_rag_strerror(int code);
const char *ha_rag_version(void);

/* ---- context --------------------------------------------------------------- */

/* Validates the configuration (EINVAL / EFORMAT) and creates a context with empty
 * pools.  Creates the copy streams unless dry_run. */
int ha_rag_create(const ha_rag_config *cfg, ha_rag_ctx **out);

/* Destroys events, copy streams and host metadata.  Synchronises the copy streams
 * first.  The caller's buffers are not touched. */
int ha_rag_destroy(ha_rag_ctx *ctx);

/* Name of the last failing HIP or file call and its error string, or the limit a call to
 * ha_rag_attend_packed_static exceeded ("" if none).
 * With ctx == NULL: the reason the calling thread's last ha_rag_create failed. */
const char *ha_rag_last_hip_error(ha_rag_ctx *ctx);

/* To be called before the caller destroys a stream it has passed to this context.  The
 * library orders work across streams (a slot is not overwritten while a load on another
 * stream may still read it: Algorithm 2's evictions under asynchronous execution) with one
 * event per stream it has seen, and slots remember their last reader and writer streams by
 * handle.  This call waits on the host for what the library enqueued on `stream` and drops the
 * stream from those books, so that a later stream that happens to get the same handle starts
 * clean and the table of events does not grow with every short-lived stream.  OK for a stream
 * the context has never seen. */
int ha_rag_forget_stream(ha_rag_ctx *ctx, void *stream);

/* Launch shape of the gather-dequantize-scatter kernel, for tuning sweeps; the
 * defaults (64 threads, 0, 0, 1, 1) are the measured best.  One wave handles one
 * *item*: some of the four 1024-byte output planes of one 2048-element block. */
typedef struct ha_rag_launch_params {
    uint32_t threads;   /* per workgroup: 64..1024, multiple of 64 (one item per wave)  */
    uint32_t planes16;  /* planes per item for 16-bit chunks: 1, 2 or 4; 0 = the library
                           chooses: 1 into a plain cache, 4 into a paged cache            */
    uint32_t planes8;   /* planes per item for the 8-bit tags (INT8, FP8, GSE8): 2 or 4;
                           0 = the library chooses: 2 into a plain cache, 4 into a paged
                           one.  INT4, GSE8, and any chunk read from host memory: always 4 */
    uint32_t nt_store;  /* 1 = nontemporal (streaming) stores to the cache              */
    uint32_t nt_load;   /* 1 = nontemporal loads of the packed payload                  */
} ha_rag_launch_params;
int ha_rag_set_launch_params(ha_rag_ctx *ctx, const ha_rag_launch_params *lp);

/* ---- offline: quantize + pack (Algorithm 1 step 3, Compression(S_i, chunk)) -- */

/* src  device pointer, BF16 [L][2][H][n_tokens][D] contiguous, 16-byte aligned,
 *      finite values.
 * dst  device pointer, 16-byte aligned, ha_rag_chunk_bytes() bytes; every byte is
 *      written (padding included).  May be a pool slot (ha_rag_pool_slot).
 * saturated  nullable device pointer to a u32 the kernel adds to: the number of
 *      groups whose zero or scale left the fp16 range (then stored as +-65504).
 * Per group: zero = min rounded toward -inf to fp16, scale = (max - zero)/(2^b-1)
 * in fp32 rounded toward +inf to fp16, code = clamp(rint((x - zero)/scale)) in fp32.
 * FP8 tags: each element rounded to the nearest FP8 value (ties to even),
 * saturating.  GSE8: per tile, exponent range then truncating encode.  For both
 * `group` is ignored and `saturated` is not touched.
 * EFORMAT on prec/group/shape; EINVAL on null or misaligned pointers. */
int ha_rag_quantize_chunk(ha_rag_ctx *ctx, const void *src, uint32_t n_tokens, uint32_t prec,
                          uint32_t group, void *dst, uint32_t *saturated, void *stream);

/* Algorithm 1 step 3 compresses a whole class at once, Compression(S_i, chunks_i): the same
 * as ha_rag_quantize_chunk for chunks i = 0..n-1 of one tag (srcs, dsts, n_tokens: host arrays;
 * every srcs[i] / dsts[i] as src / dst above, lengths may differ, a chunk of 0 tokens is
 * skipped), in one kernel launch per 128 chunks, so that short chunks do not each pay a
 * launch's ramp and tail.  The bytes written are those of n separate calls; `saturated`
 * receives the sum.  Nothing is enqueued unless every chunk passes the checks. */
int ha_rag_quantize_chunks(ha_rag_ctx *ctx, const void *const *srcs, void *const *dsts,
                           const uint32_t *n_tokens, uint32_t n, uint32_t prec, uint32_t group,
                           uint32_t *saturated, void *stream);

/* The same for a keys-only or values-only chunk: src is BF16 [L][H][n_tokens][D] (one
 * plane of a document's KV), dst takes half of ha_rag_chunk_bytes().  The bytes do not
 * depend on which of the two planes the chunk is. */
int ha_rag_quantize_half(ha_rag_ctx *ctx, const void *src, uint32_t n_tokens, uint32_t prec,
                         uint32_t group, void *dst, uint32_t *saturated, void *stream);

/* Squared error of a packed chunk against its source: adds to *sum_sq (device pointer to a
 * binary64, 8-byte aligned, which the caller has set, usually to 0) the sum over all elements
 * of (x - y)^2, x the source BF16 value and y the BF16 value a load would write for it.  The
 * paper's RMSE (Eq. 1; Sec. 3.2.1 orders the schemes S1..S4 by it) is sqrt(sum_sq / elements).
 * src as in ha_rag_quantize_chunk (part = HA_RAG_PART_KV) or ha_rag_quantize_half (PART_K or
 * PART_V); `packed` a device pointer to that chunk's packed bytes.  The sum is accumulated in
 * binary64 with one atomic add per workgroup, so its last bits depend on the order. */
int ha_rag_chunk_sq_error(ha_rag_ctx *ctx, const void *src, const void *packed, uint32_t n_tokens,
                          uint32_t prec, uint32_t group, uint32_t part, double *sum_sq, void *stream);

/* ---- online, no pool: gather-dequantize-scatter of caller-held packed chunks -- */

/* Chunk i of `chunks[n]` (host array, n <= HA_RAG_MAX_REQUEST_CHUNKS) is
 * dequantized as bf16_rne(fma(code, scale, zero)) (16-bit tag: copied) into token
 * rows [tok_base + sum_{j<i} n_tokens_j, ...) of every (layer, K/V, head) tile of
 * out[L][2][H][cap_tokens][D] (device, BF16, 16-byte aligned).  Rows outside those
 * ranges are not written.  ENOSPC if the chunks do not fit, before anything is
 * enqueued.  One kernel launch per 64 chunks.
 * Keys-only and values-only chunks (`part`) fill only their plane: the key plane and
 * the value plane each advance in list order by the chunks that hold them, so the keys
 * and the values of a document may sit anywhere in the list and differ in precision.
 * EINVAL, before anything is enqueued, if a whole chunk arrives while the two planes
 * differ in length, or if they differ at the end of the list.
 * The call makes no allocation, no copy and no synchronisation: it only launches kernels
 * on `stream`, so it may be recorded into a HIP graph (stream capture) and replayed; a
 * replay reads whatever the packed buffers hold at that time. */
int ha_rag_load_packed(ha_rag_ctx *ctx, const ha_rag_packed_chunk *chunks, uint32_t n,
                       void *out, uint64_t cap_tokens, uint64_t tok_base, void *stream);

/* The same into a paged cache.  Capacity is n_table * page_tokens rows; rows the chunks do
 * not cover, and pages the table does not name, are not written.  EINVAL for a cache
 * description that breaks the limits stated at ha_rag_paged_cache. */
int ha_rag_load_packed_paged(ha_rag_ctx *ctx, const ha_rag_packed_chunk *chunks, uint32_t n,
                             const ha_rag_paged_cache *cache, uint64_t tok_base, void *stream);

/* Algorithm 2 step 2 without the decode, for consumers that read the packed chunks themselves
 * (ha_rag_attend_chunks): for every listed chunk, in order, exactly the bookkeeping and the
 * copies of ha_rag_load_chunks (access count, LRU touch in the tier it is found in, a copy in
 * the tier its rank's list names if that is faster, evicting the least recently used chunk of
 * a full slab), but no cache is written and no staging slot is used: a copy booked in HBM is
 * filled by one host -> device copy on `stream`.  Pageable and file copies are read through a
 * bounce buffer (ENOSPC without one).
 * flags: HA_RAG_PLACE_DEVICE_VISIBLE = no chunk is left in pageable memory or a file only:
 * one that its rank's list would leave there also gets a copy in pinned memory (slot
 * permitting; see promote_skipped in the trace), so that the kernels can read every chunk of
 * the list in place afterwards.
 * stats: hit and placement counters as for a load; the byte counters hold what this call
 * moved (bytes_h2d: copies into HBM; bytes_disk_read, bytes_host_copied); tokens,
 * packed_bytes_read, bf16_bytes_written and bytes_d2d are 0. */
#define HA_RAG_PLACE_DEVICE_VISIBLE 1u
int ha_rag_place_chunks(ha_rag_ctx *ctx, const uint64_t *ids, const uint8_t *tags, uint32_t n,
                        uint32_t flags, void *stream, ha_rag_load_stats *stats,
                        ha_rag_chunk_trace *trace);

/* ---- online, no cache: attention straight over packed chunks ------------------ */

#define HA_RAG_MAX_ATTEND_REQUESTS 1024
#define HA_RAG_MAX_ATTEND_Q 4096

/* One request of ha_rag_attend_packed: the query vectors of its question tokens for one
 * layer, and where the result goes.  Its chunks are the next n_chunks entries of the call's
 * chunk list (requests take their chunks in order). */
typedef struct ha_rag_attend_request {
    const void *q;     /* device, BF16 [n_q][n_q_heads][D], 16-byte aligned                 */
    float *out;        /* device, binary32 [n_q][n_q_heads][D], 16-byte aligned             */
    float *lse;        /* device, binary32 [n_q][n_q_heads], or NULL                        */
    uint32_t n_q;      /* query tokens, 1..HA_RAG_MAX_ATTEND_Q                              */
    uint32_t n_chunks; /* chunks of this request                                            */
} ha_rag_attend_request;

/* The prefill of Sec. 2.1 attends from the question's tokens to the concatenated KV of the
 * retrieved chunks.  This call computes that attention for one layer without building the
 * BF16 cache: it reads the packed chunks (Sec. 2.2) and decodes them in registers to the
 * very values a load would write.  For every request r, query token i and query head hq
 * (which reads KV head hq / (n_q_heads / H)), over the tokens t of all chunks of r:
 *     s[t]   = sm_scale * sum_d q[i][hq][d] * K[t][d]
 *     out[i][hq][d] = sum_t softmax(s)[t] * V[t][d],   lse[i][hq] = log(sum_t exp(s[t]))
 * Every chunk token is visible to every query token (the question follows the chunks); out
 * and lse are what a caller needs to merge this with attention over other keys.  A request
 * whose chunks hold no token gets out = 0 and lse = -inf.
 * K and V values are exact; the softmax weights are rounded to BF16 before they multiply V
 * and sums are accumulated in binary32, so out differs from the exact result by about
 * 2^-8 * sum_t softmax(s)[t] * |V[t][d]| at most.
 * chunks[]: host array of chunks in device memory, any mix of tags.  A request may name
 * whole chunks and keys-only / values-only chunks: its i-th keys-only chunk and its i-th
 * values-only chunk form one document (their formats may differ) and must hold the same
 * number of tokens; EINVAL if they do not, or if keys are left without values or the reverse.
 * reqs[n_reqs]: host array, n_reqs <= HA_RAG_MAX_ATTEND_REQUESTS, all chunks together
 * <= HA_RAG_MAX_REQUEST_CHUNKS.  n_q_heads a multiple of H, at most 64 H.  sm_scale > 0.
 * workspace: device memory, 16-byte aligned, of at least the size
 * ha_rag_attend_workspace_bytes returns for the same lists (it holds partial results and
 * may be reused by the next call on the same stream; the size may be 0, and the pointer then
 * null, when no request needs a partial result); ENOSPC if smaller.
 * EFORMAT unless head_dim is 128.
 * Like ha_rag_load_packed the call only launches kernels on `stream`: one per 512 runs of
 * blocks (a workgroup's share of a request: a piece of a document, or for requests of many
 * query rows a range of blocks across documents) plus one per 64 requests. */
int ha_rag_attend_packed(ha_rag_ctx *ctx, const ha_rag_packed_chunk *chunks,
                         const ha_rag_attend_request *reqs, uint32_t n_reqs, uint32_t layer,
                         uint32_t n_q_heads, float sm_scale, void *workspace,
                         size_t workspace_bytes, void *stream);

/* ha_rag_attend_packed for callers that cannot allocate device memory or have none to hand
 * over as a workspace: code running under HIP graph capture, tight serving loops, harnesses
 * that forbid allocation.  The same computation, arguments, checks and kernels, but the partial
 * results go to an array of HA_RAG_ATTEND_STATIC_SCRATCH_BYTES bytes that is part of the
 * library's device code (each GPU the library runs on holds its own copy until the process
 * ends; its address on the current device is looked up once, in ha_rag_create or at the first
 * call on that device).  The call allocates nothing, neither on the device nor on the host: its
 * plan lives on the stack (about 120 KiB with the launch descriptors), which bounds what one
 * call may hold.
 * ENOSPC, before anything is enqueued, for more than HA_RAG_ATTEND_STATIC_MAX_REQUESTS requests,
 * more than HA_RAG_ATTEND_STATIC_MAX_DOCS documents (a whole chunk, or a keys-only chunk with its
 * values-only partner, that holds tokens), or lists whose partial results
 * (ha_rag_attend_workspace_bytes) exceed the array; ha_rag_last_hip_error then says which
 * limit and by how much.
 * All calls on one GPU share that GPU's array, which keeps the previous call's contents: every
 * record a call reads it has written first, so nothing needs clearing, but two calls whose
 * kernels overlap on one GPU (different streams, or different contexts) race on it -- order them
 * on one stream or by events. */
#define HA_RAG_ATTEND_STATIC_SCRATCH_BYTES (32u << 20)
#define HA_RAG_ATTEND_STATIC_MAX_REQUESTS 64
#define HA_RAG_ATTEND_STATIC_MAX_DOCS 416
int ha_rag_attend_packed_static(ha_rag_ctx *ctx, const ha_rag_packed_chunk *chunks,
                                const ha_rag_attend_request *reqs, uint32_t n_reqs, uint32_t layer,
                                uint32_t n_q_heads, float sm_scale, void *stream);

/* Workspace size for ha_rag_attend_packed: reads only n_tokens, prec, group, part of the chunks
 * and n_q, n_chunks of the requests. */
int ha_rag_attend_workspace_bytes(ha_rag_ctx *ctx, const ha_rag_packed_chunk *chunks,
                                  const ha_rag_attend_request *reqs, uint32_t n_reqs,
                                  uint32_t n_q_heads, size_t *bytes);

/* The same for chunks of the pool, named by id: ids[] holds the requests' chunk ids one
 * request after the other (reqs[r].n_chunks each).  Every chunk is read where its fastest
 * copy lies, which must be in HBM or in pinned memory (the kernel reads pinned memory over the
 * link); ENOENT for an unknown id and for a chunk whose only copies are in pageable memory or
 * a file (load or promote it first).  No copy is made and nothing is promoted or evicted:
 * placement is the business of ha_rag_load_chunks / ha_rag_pool_promote.
 * flags: HA_RAG_ATTEND_COUNT = count one access per listed chunk (Algorithm 1's AF) and move
 * it to the recent end of its tier's LRU order, as a load does; a caller that attends layer
 * after layer sets it for one layer of a step only.  Reads are ordered after writes to the
 * same slots on other streams like the loads' are. */
#define HA_RAG_ATTEND_COUNT 1u
int ha_rag_attend_chunks(ha_rag_ctx *ctx, const uint64_t *ids, const ha_rag_attend_request *reqs,
                         uint32_t n_reqs, uint32_t layer, uint32_t n_q_heads, float sm_scale,
                         uint32_t flags, void *workspace, size_t workspace_bytes, void *stream);

int ha_rag_attend_chunks_workspace_bytes(ha_rag_ctx *ctx, const uint64_t *ids,
                                         const ha_rag_attend_request *reqs, uint32_t n_reqs,
                                         uint32_t n_q_heads, size_t *bytes);

/* ---- pools (Algorithm 2's queueGPU / queuePIN / queuePAGE and the files) ------- */

/* Gives the context a slab for chunks of tag `prec` in a memory tier: `base` is a
 * device pointer (TIER_HBM) or a pinned pointer (TIER_PINNED), 256-byte aligned, or
 * a host pointer (TIER_PAGEABLE), 16-byte aligned.  It is cut into fixed slots of
 * ha_rag_chunk_bytes(prec, group_of(prec), max_chunk_tokens) rounded up to 256
 * bytes.  One slab per (tier, prec); EINVAL if registered twice or smaller than
 * one slot. */
int ha_rag_register_slab(ha_rag_ctx *ctx, uint32_t tier, uint32_t prec, void *base, size_t bytes);

/* Declares that the pinned-tier copies of chunks of tag `prec` are caller-owned: instead of a
 * slab that the library cuts into slots, every such chunk names the pinned address its packed
 * bytes lie at (ha_rag_pool_insert_external).  This is queuePIN of Algorithm 2 for a knowledge
 * base that the caller already keeps in page-locked memory (Sec. 2.3): the library reads those
 * bytes (the kernel over the link, or DMA) and never writes, moves or frees them; Algorithm 2
 * places no new copies in this tier for the tag (a chunk found in pageable memory or a file
 * keeps going through the bounce buffers), so nothing is ever evicted from it.  Takes the place
 * of ha_rag_register_slab(TIER_PINNED, prec): EINVAL if either was called before for the tag.
 * Register before ha_rag_register_staging, which sizes its slots by the tags declared so far. */
int ha_rag_register_external(ha_rag_ctx *ctx, uint32_t prec);

/* The disk tier for tag `prec`: the file `path` (created and grown if needed) cut
 * into slots rounded up to 4096 bytes.  It is kept open until ha_rag_destroy and
 * is not deleted.  EIO if it cannot be opened or grown. */
int ha_rag_register_disk(ha_rag_ctx *ctx, uint32_t prec, const char *path, size_t bytes);

/* Device staging area that chunks on the DMA route pass through on their way from
 * host memory to the kernel (256-byte aligned): chunks from pageable memory and
 * files, pinned chunks that are promoted to HBM, every pinned chunk under pinned_dma.
 * A pool whose pinned chunks are only ever read in place needs none.  It is cut into slots as large as the largest
 * host-side slot registered so far; at least 2 slots are required. */
int ha_rag_register_staging(ha_rag_ctx *ctx, void *base, size_t bytes);

/* Pinned bounce buffers that pageable and disk chunks are copied / read into before
 * they are copied to the device (4096-byte aligned pinned pointer).  Cut into slots
 * as large as the largest pageable / disk slot registered so far; at least 2. */
int ha_rag_register_bounce(ha_rag_ctx *ctx, void *base, size_t bytes);

/* Adds chunk `id` (tag `prec`, group = the context's group for that tag) to
 * `tier`.  If `packed` is non-NULL its ha_rag_chunk_bytes() bytes are copied into
 * the slot on `stream` (`packed_is_device` says where they are; host sources
 * should be pinned); if NULL the slot is only reserved and the caller fills it
 * (ha_rag_pool_slot + ha_rag_quantize_chunk).  Pageable and disk targets are written
 * by the calling thread before the call returns (device sources and O_DIRECT files
 * go through a bounce buffer and `stream` is synchronised).  Inserting an id that
 * exists in another tier adds a further copy (same tag and n_tokens required, else
 * EFORMAT).  The copy in the slowest tier is the master: a copy is evictable only
 * if a slower tier also holds the chunk.  EINVAL duplicate in that tier; ENOSPC
 * slab full of unevictable chunks (otherwise the least recently used evictable
 * chunk of that slab is dropped), file slab full, or bounce buffer missing. */
int ha_rag_pool_insert(ha_rag_ctx *ctx, uint64_t id, uint32_t prec, uint32_t n_tokens,
                       const void *packed, int packed_is_device, uint32_t tier, void *stream);

/* The same for a keys-only (HA_RAG_PART_K) or values-only (HA_RAG_PART_V) chunk: one of
 * the 2n units of Algorithm 1, with an id, an access count, a rank and a tag of its own.
 * `packed` holds half of ha_rag_chunk_bytes().  In a load (ha_rag_load_chunks,
 * ha_rag_load_batch) such chunks follow the rule given at ha_rag_load_packed, per
 * request.  EINVAL for any other `part`; EFORMAT if the id exists with another part. */
int ha_rag_pool_insert_half(ha_rag_ctx *ctx, uint64_t id, uint32_t part, uint32_t prec,
                            uint32_t n_tokens, const void *packed, int packed_is_device,
                            uint32_t tier, void *stream);

/* Adds chunk `id` (whole, or a keys-only / values-only unit: `part`) with its pinned-tier copy
 * at the caller's address `pinned` (page-locked, device-visible, 16-byte aligned,
 * ha_rag_chunk_bytes() bytes in the packed layout; halved for a unit), which must stay valid
 * and unchanged while the chunk is in the pool.  Several ids may name the same address.
 * ENOSPC unless ha_rag_register_external was called for the tag; otherwise like
 * ha_rag_pool_insert (EINVAL duplicate in the tier, EFORMAT if the id exists with another tag,
 * length or part).  The chunk can get an HBM copy through Algorithm 2 or ha_rag_pool_promote
 * like any other. */
int ha_rag_pool_insert_external(ha_rag_ctx *ctx, uint64_t id, uint32_t part, uint32_t prec,
                                uint32_t n_tokens, const void *pinned);

/* Moves the pinned-tier copies of ids[n] to the addresses pinned[n] (host arrays): later calls
 * read chunk ids[i] at pinned[i], work already enqueued keeps reading the old address, which the
 * caller therefore keeps intact until that work has finished.  For a knowledge base whose
 * pinned window moves over a larger store (Sec. 2.1: chunks are loaded on demand).  An HBM copy
 * made earlier keeps the bytes it was made from.  Nothing changes unless every entry is good:
 * ENOENT unknown id, EINVAL for a chunk without a caller-owned pinned copy or a bad address. */
int ha_rag_pool_repoint_external(ha_rag_ctx *ctx, const uint64_t *ids, const void *const *pinned,
                                 size_t n);

/* Address and size of the copy of chunk `id` in `tier` (HBM, pinned or pageable; ENOENT if
 * not there): where Algorithm 1 step 3's Compression writes a chunk whose slot was reserved with
 * ha_rag_pool_insert(packed = NULL), and where a consumer reads it in place. */
int ha_rag_pool_slot(ha_rag_ctx *ctx, uint64_t id, uint32_t tier, void **ptr, size_t *bytes);

/* Copies the pinned master of `id` into an HBM slot on `stream` regardless of its
 * rank (no-op if already there); LRU eviction as in insert.  ENOENT / ENOSPC. */
int ha_rag_pool_promote(ha_rag_ctx *ctx, uint64_t id, void *stream);

/* Drops the copy of `id` in `tier` (HBM, pinned or pageable; EINVAL if no slower
 * tier holds the chunk, ENOENT if it is not in that tier).  The slot is reused only
 * after the transfers and loads that read it have finished. */
int ha_rag_pool_evict(ha_rag_ctx *ctx, uint64_t id, uint32_t tier);

/* Takes chunk `id` out of the knowledge base: every copy is dropped, its slots (file slot
 * included; the file's bytes are left as they are) become free, its count is forgotten and
 * the id may be inserted again.  N of Algorithm 2 step 1 shrinks with the next rerank.
 * Slots are handed on under the same stream / event rules as after an eviction.  ENOENT
 * unknown id. */
int ha_rag_pool_remove(ha_rag_ctx *ctx, uint64_t id);

/* What the pool knows about chunk `id`: its tag (fixed offline, Algorithm 1 step 3), its access
 * count and rank (Algorithm 1 step 1, Algorithm 2 step 1) and which of Algorithm 2's queues hold
 * a copy.  ENOENT unknown id. */
int ha_rag_pool_query(ha_rag_ctx *ctx, uint64_t id, ha_rag_chunk_info *info);

/* The knowledge base is files (Sec. 2.1: the precomputed KV is stored and loaded on demand);
 * these two calls let it outlive the process.  save_index writes, for every chunk that
 * has a copy in the file tier, {id, access count, tag, part, n_tokens, file slot} plus the
 * shape, groups and slot sizes of the context to `path` (a small binary file, native byte
 * order).  load_index, on a fresh context with the same shape and groups and with the same
 * pool files registered again (ha_rag_register_disk keeps their contents), adds those
 * chunks back as file-tier masters with their counts; ranks follow the next ha_rag_rerank.
 * Faster tiers start empty and fill through Algorithm 2 as before.  Nothing changes unless
 * every entry fits.  EIO: file missing, truncated or not an index; EFORMAT: shape, group,
 * slot size or an entry does not match this context; EINVAL: an id already exists or a
 * slot is in use. */
int ha_rag_pool_save_index(ha_rag_ctx *ctx, const char *path);
int ha_rag_pool_load_index(ha_rag_ctx *ctx, const char *path, size_t *n_loaded);

/* The order Algorithm 2's "put C_i in queueX with LRU" evicts in: ids resident in `tier` (HBM,
 * pinned or pageable), least recently used first; returns how many were written (at most
 * `cap`) through *n. */
int ha_rag_pool_lru(ha_rag_ctx *ctx, uint32_t tier, uint64_t *ids, size_t cap, size_t *n);

/* ---- hotness (Algorithm 1 step 1, Algorithm 2 step 1) ------------------------ */

/* counts[id] += 1 for each listed id (ENOENT if one is unknown; none is counted
 * then).  ha_rag_load_chunks does this itself. */
int ha_rag_touch(ha_rag_ctx *ctx, const uint64_t *ids, size_t n);

/* Overwrites the access counts (an offline profile AF). */
int ha_rag_set_counts(ha_rag_ctx *ctx, const uint64_t *ids, const uint64_t *counts, size_t n);

/* Sorts all chunks by count (descending, ties by ascending id), assigns ranks and
 * recomputes the list boundaries idx1, idx2, idx3 of Algorithm 2 step 1. */
int ha_rag_rerank(ha_rag_ctx *ctx);

/* Position of `id` in the sort of Algorithm 1 step 1 as of the last rerank (0 = most frequent;
 * UINT32_MAX if the chunk was inserted since).  ENOENT unknown id. */
int ha_rag_get_rank(ha_rag_ctx *ctx, uint64_t id, uint32_t *rank);

/* ---- online: the load (Algorithm 2 step 2 + decompression + concatenation) --- */

/* For each id in request order: count the access; find the fastest tier that holds
 * the chunk and refresh its LRU position there; if that is HBM, read it in place,
 * and so for a pinned copy that gets no faster copy (the kernel reads pinned memory
 * over the link; see pinned_dma in ha_rag_config); else bring the packed bytes into
 * a staging slot (pinned: a host -> HBM copy on a copy stream; pageable / disk: the
 * calling thread first copies / reads them into a bounce buffer) and make `stream`
 * wait for that copy; dequantize-scatter the chunk to its token rows; and if the
 * list its rank belongs to (GPU_LIST, PIN_LIST,
 * PAGE_LIST) names a faster tier than the one it was found in, place a copy there
 * (HBM: copied from staging on `stream`; pinned / pageable: copied from the bounce
 * buffer by the calling thread), evicting the least recently used evictable chunk
 * of that slab if full (skipped, not an error, if nothing can be evicted).
 *   tags   nullable host array of HA_RAG_PREC_*; if given, tags[i] must equal the
 *          stored tag of ids[i] (EFORMAT otherwise)
 *   out    device BF16 [L][2][H][cap_tokens][D]; chunk i starts at token row
 *          tok_base + sum of the token counts before it
 *   stats, trace  nullable host outputs (trace has n entries)
 * All checks (ENOENT, EFORMAT, ENOSPC for the cache, staging or bounce buffers
 * missing for a chunk that needs them) happen before any state changes or work is
 * enqueued; EIO / EHIP can occur midway (a file read failed): chunks enqueued so
 * far are still loaded, access counts and evictions of the call stand, and copies
 * the call had booked but not yet written are taken out of the books again.  A slot
 * that another stream's load may still read is not overwritten before that load
 * has finished (the library records an event per stream after each load). */
int ha_rag_load_chunks(ha_rag_ctx *ctx, const uint64_t *ids, const uint8_t *tags, uint32_t n,
                       void *out, uint64_t cap_tokens, uint64_t tok_base, void *stream,
                       ha_rag_load_stats *stats, ha_rag_chunk_trace *trace);

/* A batch of requests in one call: request r owns ids[request_starts[r] ..
 * request_starts[r+1]) and is written to outs[r] (cap_tokens[r], tok_base[r]).
 * Hot chunks of all requests share kernel launches. */
int ha_rag_load_batch(ha_rag_ctx *ctx, const uint64_t *ids, const uint8_t *tags,
                      const uint32_t *request_starts, uint32_t n_requests, void *const *outs,
                      const uint64_t *cap_tokens, const uint64_t *tok_base, void *stream,
                      ha_rag_load_stats *stats, ha_rag_chunk_trace *trace);

/* ha_rag_load_chunks with a paged cache as the destination (one request per call).
 * Everything else -- lookup, placement, statistics, trace -- is the same. */
int ha_rag_load_chunks_paged(ha_rag_ctx *ctx, const uint64_t *ids, const uint8_t *tags, uint32_t n,
                             const ha_rag_paged_cache *cache, uint64_t tok_base, void *stream,
                             ha_rag_load_stats *stats, ha_rag_chunk_trace *trace);

#if defined(__GNUC__) || defined(__clang__)
#pragma GCC visibility pop
#endif

#ifdef __cplusplus
}
#endif
#endif /* HA_RAG_H */
