// Internal interface between the host runtime and the gfx950 kernels.
// Not part of the C ABI (that is include/ha_rag.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ha_rag {

constexpr uint32_t kBlockElems = 2048;   // elements per layout block
constexpr uint32_t kMaxLaunchChunks = 64; // chunk descriptors per kernel launch

// One chunk of a gather-dequantize-scatter launch.  Travels in the kernel
// argument buffer, so no device-side descriptor table exists.
struct K1Chunk {
    const uint8_t *src;        // packed chunk (tile records back to back)
    uint8_t *out;              // cache address of tile 0, token row tok_off, dim 0
    uint64_t out_tile_stride;  // bytes between consecutive tiles of the cache
    uint32_t n_tokens;
    uint32_t fmt;              // bits (16, 8, 4) | log2(group) << 8
};

struct K1Params {
    uint32_t n_tiles;      // 2 * L * H
    uint32_t head_dim;
    uint32_t wg_per_tile;  // workgroups that share one tile (from the longest chunk)
    uint32_t n_chunks;
    K1Chunk c[kMaxLaunchChunks];
};

struct K1Launch {
    uint32_t threads;          // per workgroup, multiple of 64
    uint32_t blocks_per_wave;  // 1, 2, 4, 8
    bool nontemporal;
};

// Enqueues one launch covering p.n_chunks chunks.  max_tokens = longest chunk.
hipError_t launch_k1(const K1Params &p, uint32_t max_tokens, const K1Launch &cfg,
                     hipStream_t stream);

// Quantize + pack one chunk.  src BF16 [n_tiles][n_tokens][D]; dst packed.
hipError_t launch_k2(const void *src, void *dst, uint32_t n_tiles, uint32_t head_dim,
                     uint32_t n_tokens, uint32_t bits, uint32_t group, uint32_t *saturated,
                     hipStream_t stream);

}  // namespace ha_rag
