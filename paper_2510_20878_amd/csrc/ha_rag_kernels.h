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
constexpr uint32_t kAttendMinSplitBlocks = 8;   // a workgroup takes split_blocks layout blocks (16
constexpr uint32_t kAttendMaxSplitBlocks = 128; // tokens each) of one chunk: a power of two in this range
constexpr uint32_t kAttendTargetGroups = 2048;  // the host splits finer while a launch has fewer workgroups
constexpr uint32_t kChipCUs = 256;            // compute units of the one GPU this library is built for
constexpr uint32_t kAttendWaves = 2;          // waves of a workgroup; they interleave its blocks
// Descriptors travel in the kernel argument buffer (about 26 KiB when full; launches with
// arguments of 32 KiB were checked to work on this runtime).  A workgroup needs exactly one
// descriptor, which it fetches in one go: the argument buffer may live in host memory, where
// every dependent read costs a trip over the link.
constexpr uint32_t kAttendLaunchChunks = 416;  // chunk descriptors per launch

// One document of one request: its keys and its values, which may come from one whole chunk
// or from a keys-only and a values-only chunk of different formats.
struct K6Chunk {
    const uint8_t *k;     // tile record of (the launch's layer, KV head 0) of the keys; the
    const uint8_t *v;     // other heads' records follow.  The same for the values
    const uint16_t *q;    // BF16 [n_q][n_q_heads][128] of the chunk's request
    float *part;          // this document's records [n_kv_heads][n_split][n_mtiles]
    uint32_t n_tokens;
    uint32_t info;        // keys: Prec | log2(group) << 4; values: the same << 8
    uint32_t n_q;         // query tokens of the request
    uint32_t n_split;     // token splits of the request (the same for all its chunks)
    uint32_t run;         // launch_k6_shared: documents of the run this descriptor starts (1 = itself only)
    uint32_t more;        // launch_k6_shared: index of the descriptor of the run's second document;
                          // the third and later ones follow it
    uint32_t first_block; // launch_k6_shared: the run starts at this layout block of its first document
    uint32_t end_block;   // and ends before this one of its last document (all documents between whole)
};

struct K6Params {
    uint32_t n_kv_heads, n_q_heads, layer, n_chunks;
    uint32_t mtw;          // 16-row query tiles per workgroup: 1 or 2 (set by launch_k6)
    float scale_log2;      // sm_scale * log2(e)
    uint32_t split_blocks; // layout blocks per token split
    uint32_t pad;
    K6Chunk c[kAttendLaunchChunks];
};

struct K7Req {
    const float *part;    // records [n_chunks][n_kv_heads][n_split][n_mtiles]; n_chunks counts runs
    float *out;           // binary32 [n_q][n_q_heads][128]
    float *lse;           // binary32 [n_q][n_q_heads] or null
    uint32_t n_q, n_chunks, n_split, pad;
};

constexpr uint32_t kMaxMergeReqs = 64;
struct K7Params {
    uint32_t n_kv_heads, n_q_heads, n_reqs, pad;
    K7Req r[kMaxMergeReqs];
};

// Partial attention of every chunk of the launch (sets mtw).
hipError_t launch_k6(K6Params &p, hipStream_t stream);
// The same for requests with more than two query tiles: the `waves` (2, 4 or 8) waves of a
// workgroup share every decoded block, each wave with two tiles of its own.  A workgroup takes
// a run of blocks of one request, across its documents in list order (first_block, end_block;
// n_split must be 1): descriptors 0 .. n_runs - 1 are the runs' first documents
// (request, records in `part`, `run`, `more`), the runs' other documents come after them
// (k, v, n_tokens, info only).  The grid has no row without work: rows of workgroups that
// exit at once, in a regular pattern, were measured to halve the workgroups a CU runs side by side.
hipError_t launch_k6_shared(K6Params &p, uint32_t n_runs, uint32_t waves, hipStream_t stream);
// Once per device, before the first launch of the eight-wave build (its LDS allowance).
hipError_t prepare_k6_shared();
// Merges the partial results of each request into out and lse.
hipError_t launch_k7(K7Params &p, hipStream_t stream);

}  // namespace ha_rag
