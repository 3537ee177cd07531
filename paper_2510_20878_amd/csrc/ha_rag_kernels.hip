// gfx950 kernels of the HA-RAG mixed-precision KV-chunk load.
//
//  k1_gather_dequant_scatter  online: packed chunks -> BF16 KV cache (the
//      "load + decompress + concatenate" stage of Sec. 2.1 / Fig. 3; the
//      decompression whose cost Table 2 compares)
//  k2_quantize_pack           offline: BF16 chunk -> packed chunk (Algorithm 1
//      step 3, Compression(S_i, chunk), for the per-group integer formats)
//
// Both kernels are HBM-bound streaming kernels: no matrix cores, no LDS.  The
// packed layout (see include/ha_rag.h) is built so that lane i of a 64-lane wave
// reads 16-byte word i of a 1024-byte run and writes 16-byte word i of four
// 1024-byte runs: every memory instruction of a wave covers one contiguous KiB.
#include <algorithm>

#include "ha_rag_kernels.h"
#include "ha_rag_decode.h"

namespace ha_rag {

// ---------------------------------------------------------------------------
// K1.  One item per wave (see K1Params); 1-D grid over all items of all chunks of
// the launch, so ragged chunks and mixed tags leave no empty workgroups.  Small
// items in many short-lived waves measured fastest on MI355X (one 16-byte load per
// lane feeding one or two 1 KiB stores per wave reaches the rate of a plain copy
// kernel; four loads then four stores per wave is ~10 % slower).  Items follow the
// workgroup index linearly: consecutive workgroups, which the hardware deals
// round robin to the 8 XCDs, touch consecutive KiB; handing each XCD its own
// contiguous range instead measured slower (nothing is reused, so there is no L2
// locality to gain, and the XCDs then drift apart).
// ---------------------------------------------------------------------------
template <bool NT>
__device__ __forceinline__ u32x4 ld16s(const uint8_t *p)
{
    if (NT) return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    return *reinterpret_cast<const u32x4 *>(p);
}

template <bool NT_ST, bool NT_LD, bool PAGED>
__global__ void __launch_bounds__(1024) k1_gather_dequant_scatter(const K1Params p)
{
    const uint32_t nwaves = blockDim.x >> 6;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t item = blockIdx.x * nwaves + wave;
    if (item >= p.total_items) return;

    // Items are ordered tile by tile of the cache ([layer][keys, values][head]), and inside a
    // tile chunk by chunk in request order: the launch then writes each tile front to back
    // as one sequential stream.  Key tiles and value tiles may hold different item counts
    // (a keys-only chunk has no items in a value tile).
    uint32_t layer, kv, head, rt, out_tile;
    if (!p.any_half) {
        // whole chunks only: every tile holds the same items, one division finds the tile
        out_tile = item / p.items_per_tile[0];
        rt = item - out_tile * p.items_per_tile[0];
        layer = head = kv = 0;  // not needed: tile records are numbered like cache tiles
    } else {
        layer = item / p.items_per_layer;
        uint32_t rl = item - layer * p.items_per_layer;
        const uint32_t k_items = p.n_kv_heads * p.items_per_tile[0];
        kv = rl >= k_items ? 1u : 0u;
        rl -= kv ? k_items : 0u;
        const uint32_t ipt = p.items_per_tile[kv];
        head = rl / ipt;
        rt = rl - head * ipt;
        out_tile = (layer * 2u + kv) * p.n_kv_heads + head;
    }
    const uint32_t *start = p.item_start[kv];
    uint32_t lo = 0, hi = p.n_chunks;  // start[lo] <= rt < start[hi]
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (rt >= start[mid]) lo = mid;
        else hi = mid;
    }
    const K1Chunk &c = p.c[lo];
    const uint32_t r = rt - start[lo];
    // tile record inside the chunk: (l, kv, h) for a whole chunk, (l, h) for a half
    const uint32_t tile = ((c.fmt >> 16) & 3u) ? layer * p.n_kv_heads + head : out_tile;
    const uint32_t n_e = c.n_tokens * p.head_dim;
    const uint32_t nblk = (n_e + kBlockElems - 1) / kBlockElems;
    const uint32_t prec = c.fmt & 0xFFu, gsh = (c.fmt >> 8) & 0xFFu;
    const uint32_t planes = prec == kInt4 ? 4u : prec == kP16 ? p.planes16
                            : (c.fmt & kWholeBlockItems) ? 4u : p.planes8;
    const uint32_t ipb_sh = planes == 4 ? 0u : planes == 2 ? 1u : 2u;  // log2(items per block)
    const uint32_t blk = r >> ipb_sh;
    const uint32_t j0 = (r - (blk << ipb_sh)) * planes;  // first plane of this item

    const uint32_t lane_b = lane * 16;
    const uint32_t e = blk * kBlockElems + lane * 8 + j0 * 512;  // element of plane j0
    // where plane k of this item goes: one contiguous KiB per wave in a plain cache
    uint8_t *o = nullptr;
    uint8_t *op[4] = {nullptr, nullptr, nullptr, nullptr};
    uint32_t dropped = 0;  // paged: stores of this lane that had no valid page
    if (!PAGED) {
        o = c.out + (uint64_t)out_tile * c.out_tile_stride + (uint64_t)blk * 4096u + j0 * 1024u +
            lane_b;
    }
    // Paged cache: called once per item after its payload loads have been issued, so that the
    // page-table reads overlap them.
    auto locate = [&]() {
        if (!PAGED) return;
        // In a paged cache the KiB of a wave may straddle one page boundary (page_bytes >= 1024).
        // The wave's first byte is located with one division; the next planes step by 1024.
        const K1Paged &pc = p.paged;
        const uint32_t vb = (uint32_t)(uintptr_t)c.out + blk * 4096u + j0 * 1024u;
        uint32_t pg = pc.page_shift ? vb >> pc.page_shift : vb / pc.page_bytes;
        uint32_t within = vb - pg * pc.page_bytes;
        uint8_t *tile_base = pc.base + (uint64_t)out_tile * pc.tile_stride;
        const uint32_t last = pc.n_table - 1u;
#pragma unroll
        for (uint32_t k = 0; k < 4; ++k) {
            if (k >= planes) break;
            const uint32_t w = within + lane_b;
            const bool live = e + k * 512u < n_e;  // rows past the chunk's end have no page
            // wave-uniform table reads and base addresses; most KiB lie inside one page
            const uint32_t id0 = pc.page_table[pg < last ? pg : last];
            uint8_t *b0 = tile_base + (uint64_t)id0 * pc.page_stride;
            if (within + 1024u <= pc.page_bytes) {
                if (live && pg <= last && id0 < pc.n_pages) op[k] = b0 + w;
                else if (live) ++dropped;
            } else {
                const uint32_t id1 = pc.page_table[pg + 1u < last ? pg + 1u : last];
                uint8_t *b1 = tile_base + (uint64_t)id1 * pc.page_stride - pc.page_bytes;
                const bool cross = w >= pc.page_bytes;
                const bool ok = pg + (cross ? 1u : 0u) <= last && (cross ? id1 : id0) < pc.n_pages;
                if (live && ok) op[k] = (cross ? b1 : b0) + w;
                else if (live) ++dropped;
            }
            within += 1024u;
            if (within >= pc.page_bytes) {
                within -= pc.page_bytes;
                ++pg;
            }
        }
    };
    auto put = [&](uint32_t k, u32x4 v) {
        if (PAGED) {
            if (op[k]) st16<NT_ST>(op[k], v);
        } else if (e + k * 512u < n_e) {
            st16<NT_ST>(o + k * 1024u, v);
        }
    };

    if (prec == kInt4) {
        const uint32_t meta_blk = 8192u >> gsh;
        const uint8_t *pay = c.src + (uint64_t)tile * ((uint64_t)nblk * (1024u + meta_blk));
        const uint8_t *meta = pay + (uint64_t)nblk * 1024u;
        const u32x4 w = ld16s<NT_LD>(pay + (uint64_t)blk * 1024u + lane_b);
        const u32x4 m = ld16(meta + (uint64_t)blk * meta_blk + ((lane * 8) >> gsh) * 16u);
        locate();
        put(0, dequant_octet4(w.x, m.x));
        put(1, dequant_octet4(w.y, m.y));
        put(2, dequant_octet4(w.z, m.z));
        put(3, dequant_octet4(w.w, m.w));
    } else if (prec == kInt8) {
        const uint32_t meta_blk = 8192u >> gsh;
        const uint8_t *pay = c.src + (uint64_t)tile * ((uint64_t)nblk * (2048u + meta_blk));
        const uint8_t *meta = pay + (uint64_t)nblk * 2048u;
        const uint8_t *b = pay + (uint64_t)blk * 2048u + lane_b;
        const uint8_t *mp = meta + (uint64_t)blk * meta_blk + ((lane * 8) >> gsh) * 16u;
        if (planes == 4) {
            const u32x4 w0 = ld16s<NT_LD>(b), w1 = ld16s<NT_LD>(b + 1024);
            const u32x4 m = ld16(mp);
            locate();
            put(0, dequant_octet8(w0.x, w0.y, m.x));
            put(1, dequant_octet8(w0.z, w0.w, m.y));
            put(2, dequant_octet8(w1.x, w1.y, m.z));
            put(3, dequant_octet8(w1.z, w1.w, m.w));
        } else {  // two planes: one 16-byte load, the two meta entries of those planes
            const u32x4 w = ld16s<NT_LD>(b + (j0 >> 1) * 1024u);
            const uint2 m = *reinterpret_cast<const uint2 *>(mp + j0 * 4u);
            locate();
            put(0, dequant_octet8(w.x, w.y, m.x));
            put(1, dequant_octet8(w.z, w.w, m.y));
        }
    } else if (prec == kE4M3 || prec == kE5M2) {
        const uint8_t *b = c.src + (uint64_t)tile * ((uint64_t)nblk * 2048u) +
                           (uint64_t)blk * 2048u + lane_b;
        const bool e5 = prec == kE5M2;
        if (planes == 4) {
            const u32x4 w0 = ld16s<NT_LD>(b), w1 = ld16s<NT_LD>(b + 1024);
            locate();
            put(0, e5 ? decode_octet_fp8<true>(w0.x, w0.y) : decode_octet_fp8<false>(w0.x, w0.y));
            put(1, e5 ? decode_octet_fp8<true>(w0.z, w0.w) : decode_octet_fp8<false>(w0.z, w0.w));
            put(2, e5 ? decode_octet_fp8<true>(w1.x, w1.y) : decode_octet_fp8<false>(w1.x, w1.y));
            put(3, e5 ? decode_octet_fp8<true>(w1.z, w1.w) : decode_octet_fp8<false>(w1.z, w1.w));
        } else {
            const u32x4 w = ld16s<NT_LD>(b + (j0 >> 1) * 1024u);
            locate();
            put(0, e5 ? decode_octet_fp8<true>(w.x, w.y) : decode_octet_fp8<false>(w.x, w.y));
            put(1, e5 ? decode_octet_fp8<true>(w.z, w.w) : decode_octet_fp8<false>(w.z, w.w));
        }
    } else if (prec == kGSE8) {
        const uint8_t *rec = c.src + (uint64_t)tile * ((uint64_t)nblk * 2048u + 16u);
        const uint8_t *b = rec + (uint64_t)blk * 2048u + lane_b;
        const uint32_t range = *reinterpret_cast<const uint32_t *>(rec + (uint64_t)nblk * 2048u);
        const int base = (int)(int8_t)(range & 0xFFu);              // e_lo + 2 - 2
        const int top = (int)(int8_t)((range >> 8) & 0xFFu) - 2;    // e_hi - 2
        if (planes == 4) {
            const u32x4 w0 = ld16s<NT_LD>(b), w1 = ld16s<NT_LD>(b + 1024);
            locate();
            put(0, decode_octet_gse8(w0.x, w0.y, base, top));
            put(1, decode_octet_gse8(w0.z, w0.w, base, top));
            put(2, decode_octet_gse8(w1.x, w1.y, base, top));
            put(3, decode_octet_gse8(w1.z, w1.w, base, top));
        } else {
            const u32x4 w = ld16s<NT_LD>(b + (j0 >> 1) * 1024u);
            locate();
            put(0, decode_octet_gse8(w.x, w.y, base, top));
            put(1, decode_octet_gse8(w.z, w.w, base, top));
        }
    } else {
        const uint8_t *b = c.src + (uint64_t)tile * ((uint64_t)nblk * 4096u) +
                           (uint64_t)blk * 4096u + j0 * 1024u + lane_b;
        if (planes == 1) {
            const u32x4 w0 = ld16s<NT_LD>(b);
            locate();
            put(0, w0);
        } else if (planes == 2) {
            const u32x4 w0 = ld16s<NT_LD>(b), w1 = ld16s<NT_LD>(b + 1024);
            locate();
            put(0, w0);
            put(1, w1);
        } else {
            u32x4 w[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) w[j] = ld16s<NT_LD>(b + j * 1024);
            locate();
#pragma unroll
            for (int j = 0; j < 4; ++j) put(j, w[j]);
        }
    }
    // reported last, so that no store precedes the page-table reads above (they can then be
    // scalar loads)
    if (PAGED && dropped && p.paged.bad_pages) atomicAdd(p.paged.bad_pages, dropped);
}

hipError_t launch_k1(K1Params &p, const K1Launch &given, hipStream_t stream)
{
    if (p.n_chunks == 0) return hipSuccess;
    // 0 planes = the measured best: one plane per item for 16-bit and two for the 8-bit tags
    // when the cache is plain; whole blocks when it is paged, where every item also pays for
    // its page-table reads and page addresses (+9 % at the 8B shape, +5 % at the 70B shape)
    K1Launch cfg = given;
    if (cfg.planes16 == 0) cfg.planes16 = p.paged.enabled ? 4u : 1u;
    if (cfg.planes8 == 0) cfg.planes8 = p.paged.enabled ? 4u : 2u;
    if (p.n_chunks > kMaxLaunchChunks || cfg.threads < 64 || cfg.threads > 1024 ||
        (cfg.threads & 63u))
        return hipErrorInvalidValue;
    if ((cfg.planes16 != 1 && cfg.planes16 != 2 && cfg.planes16 != 4) ||
        (cfg.planes8 != 2 && cfg.planes8 != 4))
        return hipErrorInvalidValue;
    if (p.paged.enabled) {
        const K1Paged &pc = p.paged;
        if (!pc.base || !pc.page_table || pc.n_table == 0 || pc.page_bytes < 1024u || (pc.page_bytes & 15u) ||
            ((uintptr_t)pc.base & 15u) || (pc.page_stride & 15u) || (pc.tile_stride & 15u) ||
            (uint64_t)pc.n_table * pc.page_bytes > 0xFFFFFFFFull)
            return hipErrorInvalidValue;
        p.paged.page_shift = 0;
        if ((pc.page_bytes & (pc.page_bytes - 1u)) == 0)
            while ((1u << p.paged.page_shift) < pc.page_bytes) ++p.paged.page_shift;
    }
    p.planes16 = (uint8_t)cfg.planes16;
    p.planes8 = (uint8_t)cfg.planes8;
    uint64_t per_tile[2] = {0, 0};
    p.any_half = 0;
    p.pad = 0;
    for (uint32_t i = 0; i < p.n_chunks; ++i) {
        // GSE-8 is decoded a whole block per item whatever planes8 says: its per-item set-up
        // (the tile's exponent range) and its long decode then serve four planes; measured
        // 6.1-6.2 TB/s against 5.5 with two-plane items (FP8 is the other way round, int8 indifferent)
        if ((p.c[i].fmt & 0xFFu) == kGSE8) p.c[i].fmt |= kWholeBlockItems;
        const uint64_t n_e = (uint64_t)p.c[i].n_tokens * p.head_dim;
        if (n_e > 0x7FFFFFFFull) return hipErrorInvalidValue;  // element indices are 32-bit
        const uint64_t nblk = (n_e + kBlockElems - 1) / kBlockElems;
        const uint32_t prec = p.c[i].fmt & 0xFFu, part = (p.c[i].fmt >> 16) & 3u;
        if (prec > kGSE8 || part > kPartV) return hipErrorInvalidValue;
        if (part != kPartKV) p.any_half = 1;
        const uint32_t planes = prec == kInt4 ? 4u : prec == kP16 ? cfg.planes16
                                : (p.c[i].fmt & kWholeBlockItems) ? 4u : cfg.planes8;
        for (uint32_t kv = 0; kv < 2; ++kv) {
            p.item_start[kv][i] = (uint32_t)per_tile[kv];
            if (part == kPartKV || part == kPartK + kv) per_tile[kv] += nblk * (4u / planes);
            if (per_tile[kv] > 0x7FFFFFFFull) return hipErrorInvalidValue;
        }
    }
    for (uint32_t kv = 0; kv < 2; ++kv) {
        p.item_start[kv][p.n_chunks] = (uint32_t)per_tile[kv];
        p.items_per_tile[kv] = (uint32_t)per_tile[kv];
    }
    const uint64_t per_layer = (per_tile[0] + per_tile[1]) * p.n_kv_heads;
    const uint64_t total = per_layer * p.n_layers;
    if (total > 0x7FFFFFFFull) return hipErrorInvalidValue;
    p.items_per_layer = (uint32_t)per_layer;
    p.total_items = (uint32_t)total;
    if (total == 0) return hipSuccess;
    const uint32_t nwaves = cfg.threads >> 6;
    const uint32_t wgs = (uint32_t)((total + nwaves - 1) / nwaves);
    dim3 grid(wgs), block(cfg.threads);
    const int variant = (cfg.nt_store ? 4 : 0) | (cfg.nt_load ? 2 : 0) | (p.paged.enabled ? 1 : 0);
    switch (variant) {
    case 0: hipLaunchKernelGGL((k1_gather_dequant_scatter<false, false, false>), grid, block, 0, stream, p); break;
    case 1: hipLaunchKernelGGL((k1_gather_dequant_scatter<false, false, true>), grid, block, 0, stream, p); break;
    case 2: hipLaunchKernelGGL((k1_gather_dequant_scatter<false, true, false>), grid, block, 0, stream, p); break;
    case 3: hipLaunchKernelGGL((k1_gather_dequant_scatter<false, true, true>), grid, block, 0, stream, p); break;
    case 4: hipLaunchKernelGGL((k1_gather_dequant_scatter<true, false, false>), grid, block, 0, stream, p); break;
    case 5: hipLaunchKernelGGL((k1_gather_dequant_scatter<true, false, true>), grid, block, 0, stream, p); break;
    case 6: hipLaunchKernelGGL((k1_gather_dequant_scatter<true, true, false>), grid, block, 0, stream, p); break;
    default: hipLaunchKernelGGL((k1_gather_dequant_scatter<true, true, true>), grid, block, 0, stream, p); break;
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// K2.  One wave per block of 2048 elements; a workgroup of 4 waves takes 4
// consecutive blocks of one tile.  Every element costs a correctly rounded division, so
// the kernel is kept short on vector instructions (about 14 per element): hardware directed
// rounding for scale and zero, one shared reciprocal per group, a hardware float -> byte
// conversion for the codes.
// ---------------------------------------------------------------------------

// fp32 -> fp16 with the rounding direction taken from the MODE register: bits [3:2] are the
// round mode of the half / double precision pipe, which v_cvt_f16_f32 obeys (1 = toward
// +inf, 2 = toward -inf; checked against a software reference on every finite fp32 value).
// The switch, the conversion and the switch back are one asm statement, so nothing can be
// scheduled in between; fp32 arithmetic is governed by bits [1:0] and is not affected.
__device__ __forceinline__ uint32_t cvt_f16_toward_neg_inf(float x)
{
    uint32_t h;
    asm volatile("s_setreg_imm32_b32 hwreg(HW_REG_MODE, 2, 2), 2\n\t"
                 "v_cvt_f16_f32 %0, %1\n\t"
                 "s_setreg_imm32_b32 hwreg(HW_REG_MODE, 2, 2), 0"
                 : "=v"(h)
                 : "v"(x));
    return h & 0xFFFFu;
}

__device__ __forceinline__ uint32_t cvt_f16_toward_pos_inf(float x)
{
    uint32_t h;
    asm volatile("s_setreg_imm32_b32 hwreg(HW_REG_MODE, 2, 2), 1\n\t"
                 "v_cvt_f16_f32 %0, %1\n\t"
                 "s_setreg_imm32_b32 hwreg(HW_REG_MODE, 2, 2), 0"
                 : "=v"(h)
                 : "v"(x));
    return h & 0xFFFFu;
}

// fp32 (finite) -> fp16 word, largest finite value <= x; sets sat if none exists
__device__ __forceinline__ uint32_t f16_round_down(float x, uint32_t &sat)
{
    uint32_t h = cvt_f16_toward_neg_inf(x);  // -inf below -65504; never +inf
    sat |= (h == 0xFC00u) ? 1u : 0u;
    h = (h == 0xFC00u) ? 0xFBFFu : h;
    return (h == 0x8000u) ? 0u : h;
}

// fp32 (finite) -> fp16 word, smallest finite value >= x; sets sat if none exists
__device__ __forceinline__ uint32_t f16_round_up(float x, uint32_t &sat)
{
    uint32_t h = cvt_f16_toward_pos_inf(x);  // +inf above 65504; never -inf
    sat |= (h == 0x7C00u) ? 1u : 0u;
    h = (h == 0x7C00u) ? 0x7BFFu : h;
    return (h == 0x8000u) ? 0u : h;
}

// value of another lane of the same 16-lane row, through the data-parallel-primitive path
template <int CTRL>
__device__ __forceinline__ float dpp(float v)
{
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

// min and max over the 2^(GSH-3) consecutive lanes that share a group; every lane gets both
template <int GSH>
__device__ __forceinline__ void group_minmax(float &mn, float &mx)
{
    constexpr int LPG = (1 << GSH) >> 3;
    if (LPG >= 2) {  // lane ^ 1: quad_perm [1,0,3,2]
        mn = fminf(mn, dpp<0xB1>(mn));
        mx = fmaxf(mx, dpp<0xB1>(mx));
    }
    if (LPG >= 4) {  // lane ^ 2: quad_perm [2,3,0,1]
        mn = fminf(mn, dpp<0x4E>(mn));
        mx = fmaxf(mx, dpp<0x4E>(mx));
    }
    if (LPG >= 8) {  // row_half_mirror: lane i <-> 7 - i inside each 8 lanes
        mn = fminf(mn, dpp<0x141>(mn));
        mx = fmaxf(mx, dpp<0x141>(mx));
    }
    if (LPG >= 16) {  // row_mirror: lane i <-> 15 - i inside each 16 lanes
        mn = fminf(mn, dpp<0x140>(mn));
        mx = fmaxf(mx, dpp<0x140>(mx));
    }
    if (LPG >= 32) {
        mn = fminf(mn, __shfl_xor(mn, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 16));
    }
    if (LPG >= 64) {
        mn = fminf(mn, __shfl_xor(mn, 32));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
    }
}

template <int BITS, int GSH>
__global__ void __launch_bounds__(256) k2_quantize_pack(const K2Params p)
{
    const K2Chunk c = p.c[blockIdx.y];
    const uint8_t *__restrict__ src = c.src;
    uint8_t *__restrict__ dst = c.dst;
    uint32_t *saturated = p.saturated;
    const uint32_t n_e = c.n_tokens * p.head_dim;
    const uint32_t nblk = (n_e + kBlockElems - 1) / kBlockElems;
    const uint32_t wg_per_tile = (nblk + 3u) / 4u;
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
    const uint32_t tile = blockIdx.x / wg_per_tile;
    const uint32_t blk = (blockIdx.x - tile * wg_per_tile) * 4 + wave;
    if (tile >= p.n_tiles || blk >= nblk) return;  // the grid is as wide as the longest chunk

    const uint8_t *in = src + (uint64_t)tile * n_e * 2u + (uint64_t)blk * 4096u + lane * 16u;
    const uint32_t e = blk * kBlockElems + lane * 8;
    u32x4 raw[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        raw[j] = u32x4{0, 0, 0, 0};
        if (e + j * 512 < n_e) raw[j] = ld16s<true>(in + j * 1024);
    }

    constexpr uint32_t meta_blk = 8192u >> GSH;
    constexpr uint32_t pay_blk = 256u * BITS;
    constexpr uint32_t lanes_per_group = (1u << GSH) >> 3;
    uint8_t *pay = dst + (uint64_t)tile * nblk * (pay_blk + meta_blk);
    uint8_t *meta = pay + (uint64_t)nblk * pay_blk;
    const float qmax = (float)((1 << BITS) - 1);

    u32x4 mrow;      // the four {scale, zero} entries of this lane's planes
    uint32_t code_lo[4], code_hi[4];  // int8: two dwords per plane; int4: code_lo only
    uint32_t n_sat = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float x[8];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            x[2 * k] = __builtin_bit_cast(float, raw[j][k] << 16);
            x[2 * k + 1] = __builtin_bit_cast(float, raw[j][k] & 0xFFFF0000u);
        }
        float mn = x[0], mx = x[0];
#pragma unroll
        for (int k = 1; k < 8; ++k) {
            mn = fminf(mn, x[k]);
            mx = fmaxf(mx, x[k]);
        }
        group_minmax<GSH>(mn, mx);
        uint32_t sat = 0;
        const uint32_t zh = f16_round_down(mn, sat);
        const float z = h2f(zh);
        const float range = mx - z;
        // range / qmax, correctly rounded, without the division sequence: with r the rounded
        // reciprocal of the constant, q0 = range * r is within an ulp and one exact residual
        // step lands on the IEEE quotient (checked on every non-negative finite fp32 value for
        // 15 and for 255).
        constexpr float rq = 1.0f / (float)((1 << BITS) - 1);
        const float sc0 = range * rq;
        const float sc = __builtin_fmaf(__builtin_fmaf(-qmax, sc0, range), rq, sc0);
        const uint32_t sh = f16_round_up(sc, sat);
        const float s = h2f(sh);
        n_sat += sat;
        mrow[j] = sh | (zh << 16);
        // A constant group has scale 0 and every x equal to zero: divide by 1 instead, the
        // quotient is 0.
        const float sd = (s != 0.0f) ? s : 1.0f;
        // d / sd eight times by the same divisor: the reciprocal is refined once (rcp, one
        // Newton step); each quotient is then a multiply plus one residual correction
        // (q1 = q0 + (d - sd*q0) * r1).  q1 can differ from the correctly rounded quotient
        // only when d/sd lies within ~2^-21 ulp of the midpoint of two floats, and the code
        // depends on the quotient only through its side of a half-integer k + 1/2.  Because
        // sd has at most 11 significant bits and k < 256, (k + 1/2) * sd is a float: an exact
        // tie (d equal to it) gives q1 = k + 1/2 exactly, and any other d puts the true
        // quotient more than 2^-13 ulp away from the float midpoints next to k + 1/2, so q1
        // falls on the same side as the correctly rounded quotient does.
        const float r0 = __builtin_amdgcn_rcpf(sd);
        const float r1 = __builtin_fmaf(__builtin_fmaf(-sd, r0, 1.0f), r0, r0);
        // v_cvt_pk_u8_f32 rounds to the nearest integer, ties to even, clamps to 0..255 and
        // drops the byte into a dword (checked on every finite fp32 value); clamping before
        // rounding equals rounding before clamping because the bounds are integers.
        uint32_t lo = 0, hi = 0;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const float d = x[k] - z;
            const float q0 = d * r1;
            float q1 = __builtin_fmaf(__builtin_fmaf(-sd, q0, d), r1, q0);
            if (BITS == 4) q1 = fminf(q1, qmax);
            if (k < 4) lo = __builtin_amdgcn_cvt_pk_u8_f32(q1, k, lo);
            else hi = __builtin_amdgcn_cvt_pk_u8_f32(q1, k - 4, hi);
        }
        if (BITS == 4) {
            // bytes 0 and 2 of x | x >> 4 hold two codes each; gather them from both dwords
            lo |= lo >> 4;
            hi |= hi >> 4;
            code_lo[j] = __builtin_amdgcn_perm(hi, lo, 0x06040200u);
        } else {
            code_lo[j] = lo;
            code_hi[j] = hi;
        }
    }
    if (BITS == 4) {
        st16<false>(pay + (uint64_t)blk * pay_blk + lane * 16u,
                    u32x4{code_lo[0], code_lo[1], code_lo[2], code_lo[3]});
    } else {
        uint8_t *o = pay + (uint64_t)blk * pay_blk + lane * 16u;
        st16<false>(o, u32x4{code_lo[0], code_hi[0], code_lo[1], code_hi[1]});
        st16<false>(o + 1024, u32x4{code_lo[2], code_hi[2], code_lo[3], code_hi[3]});
    }
    if ((lane & (lanes_per_group - 1)) == 0) {  // first lane of each group
        st16<false>(meta + (uint64_t)blk * meta_blk + ((lane * 8u) >> GSH) * 16u, mrow);
        if (saturated != nullptr && n_sat) atomicAdd(saturated, n_sat);
    }
}

// The 16-bit tag stores the BF16 words verbatim: one 1024-byte plane per wave (the shape
// that copies fastest), zero fill behind the last element of a tile.
__global__ void __launch_bounds__(64) k2_pack16(const K2Params p)
{
    const K2Chunk c = p.c[blockIdx.y];
    const uint8_t *__restrict__ src = c.src;
    uint8_t *__restrict__ dst = c.dst;
    const uint32_t n_e = c.n_tokens * p.head_dim;
    const uint32_t planes_per_tile = (n_e + kBlockElems - 1) / kBlockElems * 4u;
    const uint32_t tile = blockIdx.x / planes_per_tile;
    if (tile >= p.n_tiles) return;
    const uint32_t pl = blockIdx.x - tile * planes_per_tile;   // plane = 512 elements
    const uint32_t e = pl * 512u + threadIdx.x * 8u;
    u32x4 w = u32x4{0, 0, 0, 0};
    if (e < n_e) w = ld16s<true>(src + ((uint64_t)tile * n_e + e) * 2u);
    st16<false>(dst + ((uint64_t)tile * planes_per_tile * 512u + e) * 2u, w);
}

// FP8 tags: every element is rounded on its own (nearest, ties to even, by the hardware
// conversion) after clamping to the largest finite value; one wave per block.
template <bool E5M2>
__global__ void __launch_bounds__(256) k2_pack_fp8(const K2Params p)
{
    const K2Chunk c = p.c[blockIdx.y];
    const uint8_t *__restrict__ src = c.src;
    uint8_t *__restrict__ dst = c.dst;
    const uint32_t n_e = c.n_tokens * p.head_dim;
    const uint32_t nblk = (n_e + kBlockElems - 1) / kBlockElems;
    const uint32_t wg_per_tile = (nblk + 3u) / 4u;
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
    const uint32_t tile = blockIdx.x / wg_per_tile;
    const uint32_t blk = (blockIdx.x - tile * wg_per_tile) * 4 + wave;
    if (tile >= p.n_tiles || blk >= nblk) return;
    const uint8_t *in = src + (uint64_t)tile * n_e * 2u + (uint64_t)blk * 4096u + lane * 16u;
    const uint32_t e = blk * kBlockElems + lane * 8;
    const float vmax = E5M2 ? 57344.0f : 448.0f;
    uint32_t code[4][2];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        u32x4 raw = u32x4{0, 0, 0, 0};
        if (e + j * 512 < n_e) raw = ld16s<true>(in + j * 1024);
#pragma unroll
        for (int h = 0; h < 2; ++h) {  // four elements -> one dword of codes
            float x[4];
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                x[2 * k] = __builtin_bit_cast(float, raw[2 * h + k] << 16);
                x[2 * k + 1] = __builtin_bit_cast(float, raw[2 * h + k] & 0xFFFF0000u);
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) x[k] = __builtin_amdgcn_fmed3f(x[k], -vmax, vmax);
            int w = 0;
            if (E5M2) {
                w = __builtin_amdgcn_cvt_pk_bf8_f32(x[0], x[1], w, false);
                w = __builtin_amdgcn_cvt_pk_bf8_f32(x[2], x[3], w, true);
            } else {
                w = __builtin_amdgcn_cvt_pk_fp8_f32(x[0], x[1], w, false);
                w = __builtin_amdgcn_cvt_pk_fp8_f32(x[2], x[3], w, true);
            }
            code[j][h] = (uint32_t)w;
        }
    }
    uint8_t *o = dst + (uint64_t)tile * nblk * 2048u + (uint64_t)blk * 2048u + lane * 16u;
    st16<false>(o, u32x4{code[0][0], code[0][1], code[1][0], code[1][1]});
    st16<false>(o + 1024, u32x4{code[2][0], code[2][1], code[3][0], code[3][1]});
}

// GSE-8: one workgroup of up to 16 waves per tile (a tile is the unit that shares an exponent
// range, and 16 waves per tile keep a 512-tile chunk at full occupancy).  Pass 1 finds the
// smallest and largest exponent of the tile's nonzero values (BF16 subnormals count as
// exponent -126), pass 2 encodes.  Exponents are handled in biased form (field value, 1..254),
// and all arithmetic is 16-bit integer work on both BF16 words of a dword at once (packed
// 16-bit instructions): about half the instructions of an element-by-element version.
typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ u16x2 splat16(uint32_t v)
{
    return u16x2{(uint16_t)v, (uint16_t)v};
}

// the two codes of one dword of BF16 words, one per 16-bit half (code in the low byte).
// lo: biased e_lo; lo7: e_lo + 2 + 5 and hi5: e_hi + 5, the shared exponents with the shift's
// constant folded in
__device__ __forceinline__ uint32_t gse8_encode_pair(uint32_t r, u16x2 lo, u16x2 lo7, u16x2 hi5)
{
    const uint32_t magw = r & 0x7FFF7FFFu;
    const u16x2 mag = __builtin_bit_cast(u16x2, magw);
    const u16x2 eb = __builtin_elementwise_max(mag >> splat16(7), splat16(1));  // subnormal: 1
    const u16x2 rel = __builtin_elementwise_sub_sat(eb, lo);                    // exponent above e_lo
    const u16x2 k = (rel * splat16(171)) >> splat16(9);                         // rel / 3, rel < 254
    // G + 5, G the k-th shared exponent min(e_lo + 2 + 3k, e_hi)
    const u16x2 g5 = __builtin_elementwise_min(k * splat16(3) + lo7, hi5);
    // significand with its leading one (none for subnormals) as an 8-bit integer: |x| =
    // sig / 128 * 2^(eb - 127), so floor(|x| * 2^(2 - G)) = sig >> (G - eb + 5); G >= eb always.
    // min(mag, low seven bits | 0x80) is that integer: a normal value is at least 0x80
    const u16x2 sig = __builtin_elementwise_min(mag, __builtin_bit_cast(u16x2, (magw & 0x007F007Fu) | 0x00800080u));
    const u16x2 sh = __builtin_elementwise_min(g5 - eb, splat16(15));
    const u16x2 field = sig >> sh;                                               // 0..7
    // a zero field is stored with index 0
    // (0 - min(field, 1)) is all ones in a half with a nonzero field, else zero
    const uint32_t keep = __builtin_bit_cast(uint32_t, (u16x2)(splat16(0) - __builtin_elementwise_min(field, splat16(1))));
    const uint32_t k8 = __builtin_bit_cast(uint32_t, (u16x2)(k << splat16(3)));
    return ((k8 & keep) | __builtin_bit_cast(uint32_t, field)) | ((r >> 8) & 0x00800080u);
}

// HELD: blocks of the tile that every wave keeps in registers between the two passes (the
// tile is then read once); 0: the tile is longer than 16 waves can hold and pass 2 reads it
// again.
template <int HELD>
__global__ void __launch_bounds__(1024) k2_pack_gse8(const K2Params p)
{
    __shared__ uint32_t s_lo[16], s_hi[16];
    const K2Chunk c = p.c[blockIdx.y];
    const uint8_t *__restrict__ src = c.src;
    uint8_t *__restrict__ dst = c.dst;
    const uint32_t n_e = c.n_tokens * p.head_dim;
    const uint32_t nblk = (n_e + kBlockElems - 1) / kBlockElems;
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
    const uint32_t n_waves = blockDim.x >> 6;
    const uint32_t tile = blockIdx.x;
    const uint8_t *in = src + (uint64_t)tile * n_e * 2u;
    uint8_t *rec = dst + (uint64_t)tile * ((uint64_t)nblk * 2048u + 16u);
    constexpr int kHold = HELD > 0 ? HELD : 1;
    u32x4 held[kHold][4];

    // all four loads of a block are issued before the first use: a lane past the tile's end
    // re-reads the tile's first words, which changes neither extreme of the range
    auto load_block = [&](uint32_t blk, u32x4 *planes) {
        const uint32_t e = blk * kBlockElems + lane * 8;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t ej = e + j * 512;
            planes[j] = ld16(in + (uint64_t)(ej < n_e ? ej : 0u) * 2u);
        }
    };
    // The range follows from the largest magnitude and the smallest nonzero one (the exponent
    // is monotonic in the magnitude word).  mag - 1 wraps a zero to 0xFFFF, so zeros drop out of
    // the minimum; a tile without nonzero values ends with lo > hi.
    u16x2 lo2 = splat16(0xFFFFu), hi2 = splat16(0);
    auto range_block = [&](const u32x4 *planes) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const u32x4 raw = planes[j];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t r = raw[k];  // a copy: bit_cast of the vector element itself reads element 0
                const u16x2 mag = __builtin_bit_cast(u16x2, r & 0x7FFF7FFFu);
                lo2 = __builtin_elementwise_min(lo2, (u16x2)(mag - splat16(1)));
                hi2 = __builtin_elementwise_max(hi2, mag);
            }
        }
    };
    if (HELD > 0) {
#pragma unroll
        for (int i = 0; i < kHold; ++i)  // every wave's loads are all in flight together
            if (wave + i * n_waves < nblk) load_block(wave + i * n_waves, held[i]);
#pragma unroll
        for (int i = 0; i < kHold; ++i)
            if (wave + i * n_waves < nblk) range_block(held[i]);
    } else {
        for (uint32_t blk = wave; blk < nblk; blk += n_waves) {
            load_block(blk, held[0]);
            range_block(held[0]);
        }
    }
    // magnitudes -> biased exponents (a subnormal counts as 1; no nonzero value: 0xFFFF)
    const uint32_t lo_pair = __builtin_bit_cast(uint32_t, lo2), hi_pair = __builtin_bit_cast(uint32_t, hi2);
    const uint32_t min_m1 = (lo_pair & 0xFFFFu) < (lo_pair >> 16) ? (lo_pair & 0xFFFFu) : (lo_pair >> 16);
    const uint32_t max_m = (hi_pair & 0xFFFFu) > (hi_pair >> 16) ? (hi_pair & 0xFFFFu) : (hi_pair >> 16);
    uint32_t lo = min_m1 == 0xFFFFu ? 0xFFFFu : ((min_m1 + 1u) >> 7 ? (min_m1 + 1u) >> 7 : 1u);
    uint32_t hi = max_m >> 7 ? max_m >> 7 : 1u;
    for (int o = 32; o >= 1; o >>= 1) {
        const uint32_t l2 = (uint32_t)__shfl_xor((int)lo, o), h2 = (uint32_t)__shfl_xor((int)hi, o);
        lo = l2 < lo ? l2 : lo;
        hi = h2 > hi ? h2 : hi;
    }
    if (lane == 0) {
        s_lo[wave] = lo;
        s_hi[wave] = hi;
    }
    __syncthreads();
    lo = s_lo[0];
    hi = s_hi[0];
    for (uint32_t w = 1; w < n_waves; ++w) {
        lo = s_lo[w] < lo ? s_lo[w] : lo;
        hi = s_hi[w] > hi ? s_hi[w] : hi;
    }
    if (lo > hi) lo = hi = 127;          // all zero: range (e_lo, e_hi) = (0, 0)
    if (lo + 47 < hi) lo = hi - 47;      // 16 shared exponents, 3 apart, reach 48 binades

    const u16x2 vlo = splat16(lo), vlo2 = splat16(lo + 7u), vhi = splat16(hi + 5u);
    auto encode_block = [&](uint32_t blk, const u32x4 *planes) {
        const uint32_t e = blk * kBlockElems + lane * 8;
        uint32_t code[4][2];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const u32x4 raw = planes[j];
            const bool live = e + j * 512 < n_e;  // the padding behind the tile's end is zero bytes
#pragma unroll
            for (int d = 0; d < 2; ++d) {  // four elements -> one dword of codes
                const uint32_t c01 = gse8_encode_pair(raw[2 * d], vlo, vlo2, vhi);
                const uint32_t c23 = gse8_encode_pair(raw[2 * d + 1], vlo, vlo2, vhi);
                code[j][d] = live ? __builtin_amdgcn_perm(c23, c01, 0x06040200u) : 0u;  // low bytes of the halves
            }
        }
        uint8_t *o = rec + (uint64_t)blk * 2048u + lane * 16u;
        st16<false>(o, u32x4{code[0][0], code[0][1], code[1][0], code[1][1]});
        st16<false>(o + 1024, u32x4{code[2][0], code[2][1], code[3][0], code[3][1]});
    };
    if (HELD > 0) {
#pragma unroll
        for (int i = 0; i < kHold; ++i)
            if (wave + i * n_waves < nblk) encode_block(wave + i * n_waves, held[i]);
    } else {
        for (uint32_t blk = wave; blk < nblk; blk += n_waves) {
            load_block(blk, held[0]);
            encode_block(blk, held[0]);
        }
    }
    if (threadIdx.x == 0) {
        const uint32_t e_lo = (lo - 127u) & 0xFFu, e_hi = (hi - 127u) & 0xFFu;
        st16<false>(rec + (uint64_t)nblk * 2048u, u32x4{e_lo | (e_hi << 8), 0, 0, 0});
    }
}

template <int BITS>
static void launch_k2_g(uint32_t gsh, dim3 grid, hipStream_t stream, const K2Params &p)
{
    dim3 block(256);
    switch (gsh) {
    case 5: hipLaunchKernelGGL((k2_quantize_pack<BITS, 5>), grid, block, 0, stream, p); break;
    case 6: hipLaunchKernelGGL((k2_quantize_pack<BITS, 6>), grid, block, 0, stream, p); break;
    case 7: hipLaunchKernelGGL((k2_quantize_pack<BITS, 7>), grid, block, 0, stream, p); break;
    case 8: hipLaunchKernelGGL((k2_quantize_pack<BITS, 8>), grid, block, 0, stream, p); break;
    default: hipLaunchKernelGGL((k2_quantize_pack<BITS, 9>), grid, block, 0, stream, p); break;
    }
}

hipError_t launch_k2(const K2Params &p, uint32_t prec, uint32_t group, hipStream_t stream)
{
    const uint32_t bits = prec == kP16 ? 16u : prec == kInt4 ? 4u : 8u;
    if (p.n_chunks == 0 || p.n_tiles == 0) return hipSuccess;
    if (p.n_chunks > kMaxK2Chunks) return hipErrorInvalidValue;
    uint32_t max_blk = 0;  // blocks per tile of the longest chunk: the grid's width follows it
    for (uint32_t i = 0; i < p.n_chunks; ++i) {
        const K2Chunk &c = p.c[i];
        if (!c.src || !c.dst || c.n_tokens == 0) return hipErrorInvalidValue;
        const uint64_t n_e = (uint64_t)c.n_tokens * p.head_dim;
        if (n_e > 0x7FFFFFFFull) return hipErrorInvalidValue;
        max_blk = std::max(max_blk, (uint32_t)((n_e + kBlockElems - 1) / kBlockElems));
    }
    const uint64_t gx = (uint64_t)p.n_tiles * ((max_blk + 3) / 4);
    if (gx > 0x7FFFFFFFull) return hipErrorInvalidValue;
    uint32_t gsh = 0;
    while ((1u << gsh) < group) ++gsh;
    dim3 grid((uint32_t)gx, p.n_chunks);
    if (prec == kGSE8) {
        const uint32_t waves = max_blk < 16u ? max_blk : 16u;
        const dim3 g2(p.n_tiles, p.n_chunks), b2(waves * 64u);
        // up to four blocks per wave stay in registers between the passes (tiles of up to 1024
        // tokens x 128 dims); longer tiles are read twice
        if (max_blk <= 16u) hipLaunchKernelGGL(k2_pack_gse8<1>, g2, b2, 0, stream, p);
        else if (max_blk <= 32u) hipLaunchKernelGGL(k2_pack_gse8<2>, g2, b2, 0, stream, p);
        else if (max_blk <= 64u) hipLaunchKernelGGL(k2_pack_gse8<4>, g2, b2, 0, stream, p);
        else hipLaunchKernelGGL(k2_pack_gse8<0>, g2, b2, 0, stream, p);
    } else if (prec == kE4M3 || prec == kE5M2) {
        if (prec == kE5M2) hipLaunchKernelGGL(k2_pack_fp8<true>, grid, dim3(256), 0, stream, p);
        else hipLaunchKernelGGL(k2_pack_fp8<false>, grid, dim3(256), 0, stream, p);
    } else if (bits == 16) {
        const uint64_t planes = (uint64_t)p.n_tiles * max_blk * 4u;
        if (planes > 0x7FFFFFFFull) return hipErrorInvalidValue;
        hipLaunchKernelGGL(k2_pack16, dim3((uint32_t)planes, p.n_chunks), dim3(64), 0, stream, p);
    } else {
        if (gsh < 5 || gsh > 9 || (1u << gsh) != group) return hipErrorInvalidValue;
        if (prec == kInt8) launch_k2_g<8>(gsh, grid, stream, p);
        else if (prec == kInt4) launch_k2_g<4>(gsh, grid, stream, p);
        else return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// K8.  Squared error between a chunk's source words and what its packed form
// decodes to (Eq. 1 before the mean and the root; Sec. 3.2.1 orders the
// compression schemes by this figure).  One wave per block of 2048 elements:
// the block is decoded exactly as k1 decodes it, compared with the source
// plane by plane and summed in binary64; the grid strides over the blocks, and
// each workgroup adds its total to the caller's accumulator with one atomic.
// ---------------------------------------------------------------------------
__device__ __forceinline__ double sq_err8(u32x4 a, u32x4 b)
{
    double acc = 0.0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        // BF16 -> binary64 is exact, and so is the difference of two such values
        const double d0 = (double)__builtin_bit_cast(float, a[k] << 16) -
                          (double)__builtin_bit_cast(float, b[k] << 16);
        const double d1 = (double)__builtin_bit_cast(float, a[k] & 0xFFFF0000u) -
                          (double)__builtin_bit_cast(float, b[k] & 0xFFFF0000u);
        acc = __builtin_fma(d0, d0, acc);
        acc = __builtin_fma(d1, d1, acc);
    }
    return acc;
}

__global__ void __launch_bounds__(256) k8_sq_error(const uint8_t *__restrict__ src,
                                                   const uint8_t *__restrict__ packed,
                                                   uint32_t n_tokens, uint32_t head_dim,
                                                   uint32_t n_tiles, uint32_t prec, uint32_t gsh,
                                                   double *sum_sq)
{
    __shared__ double part[4];
    const uint32_t n_e = n_tokens * head_dim;
    const uint32_t nblk = (n_e + kBlockElems - 1) / kBlockElems;
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
    const uint32_t lane_b = lane * 16u;
    double acc = 0.0;
    // the grid strides over all (tile, block) pairs: few workgroups, one atomic each
    const uint64_t n_items = (uint64_t)n_tiles * nblk;
    for (uint64_t item = (uint64_t)blockIdx.x * 4u + wave; item < n_items;
         item += (uint64_t)gridDim.x * 4u) {
        const uint32_t tile = (uint32_t)(item / nblk);
        const uint32_t blk = (uint32_t)(item - (uint64_t)tile * nblk);
        const uint32_t e = blk * kBlockElems + lane * 8u;

        u32x4 dec[4];  // the four planes of this block as BF16 words, as k1 would store them
        if (prec == kInt4) {
            const uint32_t meta_blk = 8192u >> gsh;
            const uint8_t *pay = packed + (uint64_t)tile * ((uint64_t)nblk * (1024u + meta_blk));
            const uint8_t *meta = pay + (uint64_t)nblk * 1024u;
            const u32x4 w = ld16(pay + (uint64_t)blk * 1024u + lane_b);
            const u32x4 m = ld16(meta + (uint64_t)blk * meta_blk + ((lane * 8) >> gsh) * 16u);
#pragma unroll
            for (int j = 0; j < 4; ++j) dec[j] = dequant_octet4(w[j], m[j]);
        } else if (prec == kInt8) {
            const uint32_t meta_blk = 8192u >> gsh;
            const uint8_t *pay = packed + (uint64_t)tile * ((uint64_t)nblk * (2048u + meta_blk));
            const uint8_t *meta = pay + (uint64_t)nblk * 2048u;
            const uint8_t *b = pay + (uint64_t)blk * 2048u + lane_b;
            const u32x4 w0 = ld16(b), w1 = ld16(b + 1024);
            const u32x4 m = ld16(meta + (uint64_t)blk * meta_blk + ((lane * 8) >> gsh) * 16u);
            dec[0] = dequant_octet8(w0.x, w0.y, m.x);
            dec[1] = dequant_octet8(w0.z, w0.w, m.y);
            dec[2] = dequant_octet8(w1.x, w1.y, m.z);
            dec[3] = dequant_octet8(w1.z, w1.w, m.w);
        } else if (prec == kE4M3 || prec == kE5M2) {
            const uint8_t *b = packed + (uint64_t)tile * ((uint64_t)nblk * 2048u) + (uint64_t)blk * 2048u + lane_b;
            const u32x4 w0 = ld16(b), w1 = ld16(b + 1024);
            if (prec == kE5M2) {
                dec[0] = decode_octet_fp8<true>(w0.x, w0.y);
                dec[1] = decode_octet_fp8<true>(w0.z, w0.w);
                dec[2] = decode_octet_fp8<true>(w1.x, w1.y);
                dec[3] = decode_octet_fp8<true>(w1.z, w1.w);
            } else {
                dec[0] = decode_octet_fp8<false>(w0.x, w0.y);
                dec[1] = decode_octet_fp8<false>(w0.z, w0.w);
                dec[2] = decode_octet_fp8<false>(w1.x, w1.y);
                dec[3] = decode_octet_fp8<false>(w1.z, w1.w);
            }
        } else if (prec == kGSE8) {
            const uint8_t *rec = packed + (uint64_t)tile * ((uint64_t)nblk * 2048u + 16u);
            const uint8_t *b = rec + (uint64_t)blk * 2048u + lane_b;
            const uint32_t range = *reinterpret_cast<const uint32_t *>(rec + (uint64_t)nblk * 2048u);
            const int base = (int)(int8_t)(range & 0xFFu);
            const int top = (int)(int8_t)((range >> 8) & 0xFFu) - 2;
            const u32x4 w0 = ld16(b), w1 = ld16(b + 1024);
            dec[0] = decode_octet_gse8(w0.x, w0.y, base, top);
            dec[1] = decode_octet_gse8(w0.z, w0.w, base, top);
            dec[2] = decode_octet_gse8(w1.x, w1.y, base, top);
            dec[3] = decode_octet_gse8(w1.z, w1.w, base, top);
        } else {
            const uint8_t *b = packed + (uint64_t)tile * ((uint64_t)nblk * 4096u) + (uint64_t)blk * 4096u + lane_b;
#pragma unroll
            for (int j = 0; j < 4; ++j) dec[j] = ld16(b + j * 1024);
        }

        const uint8_t *in = src + (uint64_t)tile * n_e * 2u + (uint64_t)blk * 4096u + lane_b;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (e + j * 512 < n_e) acc += sq_err8(ld16(in + j * 1024), dec[j]);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
    if (lane == 0) part[wave] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        const double total = (part[0] + part[1]) + (part[2] + part[3]);
        if (total != 0.0) atomicAdd(sum_sq, total);
    }
}

hipError_t launch_k8(const void *src, const void *packed, uint32_t n_tiles, uint32_t head_dim,
                     uint32_t n_tokens, uint32_t prec, uint32_t group, double *sum_sq,
                     hipStream_t stream)
{
    if (n_tokens == 0 || n_tiles == 0) return hipSuccess;
    if (prec > kGSE8 || sum_sq == nullptr) return hipErrorInvalidValue;
    const uint64_t n_e = (uint64_t)n_tokens * head_dim;
    if (n_e > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const uint32_t nblk = (uint32_t)((n_e + kBlockElems - 1) / kBlockElems);
    const uint64_t wgs = ((uint64_t)n_tiles * nblk + 3) / 4;
    const uint32_t gx = (uint32_t)(wgs < 2048u ? wgs : 2048u);  // 8 workgroups per compute unit
    uint32_t gsh = 0;
    if (prec == kInt8 || prec == kInt4) {
        while ((1u << gsh) < group) ++gsh;
        if (gsh < 5 || gsh > 9 || (1u << gsh) != group) return hipErrorInvalidValue;
    }
    hipLaunchKernelGGL(k8_sq_error, dim3(gx), dim3(256), 0, stream,
                       static_cast<const uint8_t *>(src), static_cast<const uint8_t *>(packed),
                       n_tokens, head_dim, n_tiles, prec, gsh, sum_sq);
    return hipGetLastError();
}

}  // namespace ha_rag
