// Internal interface between the host runtime and the gfx950 kernels.
// Not part of the C ABI (that is include/ha_rag.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ha_rag {

constexpr uint32_t kBlockElems = 2048;   // elements per layout block

// storage formats (numbered like the HA_RAG_PREC_* tags of the C ABI)
enum Prec : uint32_t { kP16 = 0, kInt8 = 1, kInt4 = 2, kE4M3 = 3, kE5M2 = 4, kGSE8 = 5 };
constexpr uint32_t kMaxLaunchChunks = 64; // chunk descriptors per kernel launch

// One chunk of a gather-dequantize-scatter launch.  Travels in the kernel
// argument buffer, so no device-side descriptor table exists.
struct K1Chunk {
    const uint8_t *src;        // packed chunk (tile records back to back)
    uint8_t *out;              // cache address of tile 0, token row tok_off, dim 0; for a paged
                               // launch: byte offset of row tok_off in the request's virtual
                               // tile (tok_off * head_dim * 2), carried in the pointer
    uint64_t out_tile_stride;  // bytes between consecutive tiles of the cache (unused if paged)
    uint32_t n_tokens;
    uint32_t fmt;              // Prec | log2(group) << 8 | part << 16 | kWholeBlockItems
};

// fmt flag: 8-bit formats of this chunk are decoded a whole block (four planes) per item
// whatever K1Launch::planes8 says.  For sources in host memory, which no cache holds: a
// two-plane item re-reads the scale/zero words its sibling item already fetched.
constexpr uint32_t kWholeBlockItems = 1u << 18;

// what a chunk holds (numbered like HA_RAG_PART_* of the C ABI): keys and values of a
// document (tile records (l, kv, h)), or only its keys / only its values (records (l, h))
enum Part : uint32_t { kPartKV = 0, kPartK = 1, kPartV = 2 };

// The unit of work of one wave is an *item*: `planes` of the four 1024-byte output
// planes of one block (int4: always all four, fed by one 16-byte load per lane;
// int8 and FP8: two or four; 16-bit: one, two or four).
// A paged cache: token row r of the request lives in physical page page_table[r / P] at row
// r % P; byte address of (cache tile, row, dim 0) =
// base + page * page_stride + tile * tile_stride + (r % P) * head_dim * 2.
struct K1Paged {
    uint8_t *base;
    const uint32_t *page_table;  // device
    uint32_t *bad_pages;         // device counter of stores dropped for a page id >= n_pages, or null
    uint64_t page_stride, tile_stride;
    uint32_t page_bytes;         // P * head_dim * 2: one tile's rows of one page, >= 1024
    uint32_t n_table, n_pages;
    uint32_t enabled;
    uint32_t page_shift;         // log2(page_bytes) if that is a power of two, else 0 (set by launch_k1)
    uint32_t pad;
};

struct K1Params {
    uint32_t n_layers;     // the cache has n_layers * 2 * n_kv_heads tiles
    uint32_t n_kv_heads;
    uint32_t head_dim;
    uint32_t n_chunks;
    uint32_t total_items;        // n_layers * items_per_layer
    uint32_t items_per_layer;    // n_kv_heads * (items_per_tile[0] + items_per_tile[1])
    uint32_t items_per_tile[2];  // items of all chunks in one key tile / one value tile
    uint8_t planes16, planes8;
    uint8_t any_half;  // 1 = some chunk of the launch holds only keys or only values
    uint8_t pad;
    // per plane (keys, values): prefix sum over chunks of the items a chunk has in one
    // tile of that plane (none if the chunk does not hold that plane)
    uint32_t item_start[2][kMaxLaunchChunks + 1];
    K1Paged paged;
    K1Chunk c[kMaxLaunchChunks];
};

struct K1Launch {
    uint32_t threads;     // per workgroup, multiple of 64; one item per wave
    uint32_t planes16;    // 1, 2, 4
    uint32_t planes8;     // 2, 4
    bool nt_store, nt_load;
};

// Enqueues one launch covering p.n_chunks chunks (fills the item fields of p).
hipError_t launch_k1(K1Params &p, const K1Launch &cfg, hipStream_t stream);

// Quantize + pack the chunks of one launch (one tag, one group size; any lengths).  Chunk i:
// src BF16 [n_tiles][n_tokens][D], dst packed.  The descriptors travel in the kernel arguments
// (blockIdx.y = chunk), so that a whole class of Algorithm 1 is compressed by one launch and a
// short chunk does not pay for a launch's ramp and tail of its own.
struct K2Chunk {
    const uint8_t *src;
    uint8_t *dst;
    uint32_t n_tokens, pad;
};
constexpr uint32_t kMaxK2Chunks = 128;
struct K2Params {
    uint32_t n_chunks, n_tiles, head_dim, pad;
    uint32_t *saturated;   // device counter the integer tags add to, or null
    K2Chunk c[kMaxK2Chunks];
};
hipError_t launch_k2(const K2Params &p, uint32_t prec, uint32_t group, hipStream_t stream);

// Adds to *sum_sq (device, binary64) the squared error between src (BF16 [n_tiles][n_tokens][D])
// and what `packed` decodes to.
hipError_t launch_k8(const void *src, const void *packed, uint32_t n_tiles, uint32_t head_dim,
                     uint32_t n_tokens, uint32_t prec, uint32_t group, double *sum_sq,
                     hipStream_t stream);

// ---- attention over packed chunks (head_dim 128 only) ------------------------------------
// A partial result of one (chunk, KV head, token split, 16 query rows): unnormalised
// output [16][128] binary32, then the running maximum m[16] (base-2 exponent units) and the
// sum l[16] of 2^(score - m).
constexpr uint32_t kAttendHeadDim = 128;
constexpr uint32_t kAttendRecFloats = 16 * 128 + 32;
constexpr uint32_t kAttendMinRunBlocks = 8;    // a workgroup takes at least this many layout blocks (16 tokens each;
                                               // half as many in a call of very few workgroups),
constexpr uint32_t kAttendMaxRunBlocks = 128;  // and a piece of one document is at most this long (a power of two)
constexpr uint32_t kAttendTargetGroups = 2048; // pieces are halved while a launch has fewer workgroups
constexpr uint32_t kChipCUs = 256;            // compute units of the one GPU this library is built for
constexpr uint32_t kAttendWaves = 2;          // waves of a workgroup; they interleave its blocks
// Descriptors travel in the kernel argument buffer (36 KiB; launches with arguments of up to
// 62.5 KiB were checked to work on this runtime).  A workgroup fetches its run's descriptor in one go
// and one short descriptor per further document: the argument buffer may live in host memory,
// where every dependent read costs a trip over the link.
constexpr uint32_t kAttendArgBytes = 36864;

// One document: its keys and its values, which may come from one whole chunk or from a
// keys-only and a values-only chunk of different formats.
struct K6Doc {
    const uint8_t *k;     // tile record of (the launch's layer, KV head 0) of the keys; the
    const uint8_t *v;     // other heads' records follow.  The same for the values
    uint32_t n_tokens;
    uint32_t info;        // keys: Prec | log2(group) << 4; values: the same << 8
};

// A run: layout blocks first_block .. of its first document (described here), then n_docs - 2
// whole documents, then the blocks before end_block of its last one, all of one request.  One
// row of workgroups takes a run and writes one record per (KV head, query tile) for it.
struct K6Run {
    const uint8_t *k;
    const uint8_t *v;
    const uint16_t *q;    // BF16 [n_q][n_q_heads][128] of the request
    float *part;          // the run's records [n_kv_heads][n_mtiles]; or, if `final`, the request's
                          // output, binary32 [n_q][n_q_heads][128]
    uint32_t n_tokens;
    uint32_t info;
    uint32_t n_q;         // query tokens of the request
    uint32_t final;       // the run is all the request has (launch_k6_shared only): the workgroups
                          // normalise and write out and lse themselves, no record, no merge
    uint32_t n_docs;      // documents of the run (1 = this one only)
    uint32_t more;        // index in K6Params::doc of the run's second document; the third and
                          // later ones follow it
    uint32_t first_block;
    uint32_t end_block;   // of the run's last document; with n_docs == 1 that is this one
    float *lse;           // final runs: binary32 [n_q][n_q_heads] or null
};

constexpr uint32_t kAttendMaxRuns = kAttendArgBytes / sizeof(K6Run);
constexpr uint32_t kAttendMaxDocs = kAttendArgBytes / sizeof(K6Doc);

struct K6Params {
    uint32_t n_kv_heads, n_q_heads, layer;
    uint32_t n_runs;       // run[0 .. n_runs)
    uint32_t mtw;          // 16-row query tiles per workgroup: 1 or 2 (set by launch_k6)
    float scale_log2;      // sm_scale * log2(e)
    uint32_t doc_first;    // the runs' further documents: doc[doc_first .. doc_end), behind the runs
    uint32_t doc_end;
    union {                // two views of the same bytes
        K6Run run[kAttendMaxRuns];
        K6Doc doc[kAttendMaxDocs];
    };
    // index in doc of the first short descriptor behind n runs
    static constexpr uint32_t docs_behind(uint32_t n) { return (n * (uint32_t)sizeof(K6Run) + (uint32_t)sizeof(K6Doc) - 1u) / (uint32_t)sizeof(K6Doc); }
};

struct K7Req {
    const float *part;    // records [n_runs][n_kv_heads][n_mtiles]
    float *out;           // binary32 [n_q][n_q_heads][128]
    float *lse;           // binary32 [n_q][n_q_heads] or null
    uint32_t n_q, n_runs, pad[2];
};

constexpr uint32_t kMaxMergeReqs = 64;
struct K7Params {
    uint32_t n_kv_heads, n_q_heads, n_reqs, pad;
    K7Req r[kMaxMergeReqs];
};

// Partial attention of every run of the launch: run[0 .. n_runs), their further documents
// doc[doc_first .. doc_end) with doc_first = docs_behind(n_runs), each run's in a row (`more`).  The
// grid has one row of workgroups per run and none without work: rows of workgroups that exit
// at once, in a regular pattern, were measured to halve the workgroups a CU runs side by side.
// launch_k6 is for requests of at most two query tiles (sets mtw): a workgroup's two waves take
// the run's blocks in turn.  check_only (here and below): every check, no launch -- what a
// context without a device does with the descriptors it has filled.
hipError_t launch_k6(K6Params &p, hipStream_t stream, bool check_only = false);
// The same for requests with more than two query tiles: the `waves` (2, 4 or 8) waves of a
// workgroup share every decoded block, each wave with two tiles of its own.
hipError_t launch_k6_shared(K6Params &p, uint32_t waves, hipStream_t stream, bool check_only = false);
// What both check of their arguments (max_mt: most query tiles of a run's request; narrow: no 16-bit side).
hipError_t check_k6_args(const K6Params &p, uint32_t *max_mt, bool *narrow);
// Once per device, before the first launch of the eight-wave build (its LDS allowance).
hipError_t prepare_k6_shared();
// Merges the partial results of each request into out and lse.
hipError_t launch_k7(K7Params &p, hipStream_t stream, bool check_only = false);

}  // namespace ha_rag
