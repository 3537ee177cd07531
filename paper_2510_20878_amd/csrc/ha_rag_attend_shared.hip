// gfx950 kernel for attention over packed chunks when a request has more query rows than one
// wave can keep (more than two 16-row tiles: the question's prefill of Sec. 2.1, tens of query
// tokens times the query heads of a KV head).
//
//  k6_attend_shared<W>   one workgroup of W waves (2, 4 or 8) per (run of blocks across a request's
//      documents in list order, KV head, group of 2 W query tiles).  Every wave owns two query
//      tiles for the whole run: their queries, reference maxima, sums and output rows stay in its
//      registers.  The layout blocks are taken W at a time: half the waves decode the keys and
//      half the values of the round, two blocks each, to BF16 (the values a load would write)
//      and leave them in LDS in the form the MFMAs take their operands in; after one barrier
//      every wave scores all W blocks against its own tiles, two blocks (a pair) at a time.  A
//      block is therefore fetched and decoded once per 32 W query rows.  The rounds alternate
//      between two sets of LDS buffers, so one barrier per round is enough: a wave that writes
//      round r + 1 has passed barrier r, which every wave reaches only after it has read all of
//      round r - 1.
//
// Block geometry as for k6_attend_partial: lane (c = lane / 16, n = lane % 16) of the wave that
// reads a block holds, in plane j, token 4 j + c, dims 8 n .. 8 n + 7.
//   V: that is what the product P V takes from a lane, so the decoding wave stores its eight
//      operand words lane by lane, those of a pair's first and second block side by side (16
//      bytes per lane and operand), and every wave reads them back lane by lane: one 16x16x32
//      MFMA then contracts over the 32 tokens of the pair.
//   K: the score MFMA wants, per lane, 8 dims of the token of its column; the decoding wave
//      stores octet o of token t at 16-byte slot (o ^ t) of row t (256 bytes a row), which
//      both its own stores and the readers' loads reach without bank conflicts.
// A pair's buffer is 16 KiB: K of its first block, K of its second block, V of both.
#include "ha_rag_attend_dev.h"
#include <atomic>

namespace ha_rag {

namespace {

constexpr uint32_t kSharedBlockLds = 8192;  // LDS per block: K operands 4 KiB, V operands 4 KiB (laid out per pair)

struct SharedState {  // a wave's two query tiles
    bf16x8 qb[2][4];
    float m_run[2], l_run[2];
    f32x4 O[2][8];
};

struct SharedSide {  // the keys or the values of one document's (layer, head) tile (uniform values)
    gbytes tile, meta;
    uint32_t meta_blk, gsh;
    int base, top;
};

struct SharedLane {
    uint32_t lane, c_, n_;  // MFMA coordinates: lane group, lane column
    uint32_t k_rd;          // where the lane reads its K operand 0 inside a block's buffer; operand y: ^ 16 y
    uint32_t k_wr;          // where it writes the keys of its plane 0; plane j: (^ 64 j) + 1024 j
};

// a fresh copy of a lane constant: what is derived from it is computed where it is used and
// does not occupy registers across the whole loop
__device__ __forceinline__ uint32_t fresh(uint32_t v)
{
    asm volatile("" : "+v"(v));
    return v;
}

// Two blocks (a pair) against the wave's two tiles, in three steps: S^T = K Q^T of both blocks
// (shared_qk_pair), the running softmax (shared_softmax_pair), O += P V (shared_pv_pair).
//
// The product P V contracts over tokens, 16 per block; the 16x16x32 MFMA contracts over 32, so
// the two blocks of a pair share one: contraction index 8 c_ + i is token 4 i + c_ of the pair's
// first block for i < 4 and token 4 (i - 4) + c_ of its second block for i >= 4.  For the lane
// that is the weights of the first block next to those of the second (P8) and, per dim, the
// values of the first block next to those of the second, which is how the decoding waves lay
// the pair's V operands out (16 bytes per lane and operand: first block, second block).  Half
// the MFMAs of the 16x16x16 form, which is no faster per instruction.

// S[e][mt][jj] = q k (unscaled) of token 4 jj + c_ of block e of the pair and query row n_ of tile mt
__device__ __forceinline__ void shared_qk_pair(const uint8_t *pair, const SharedLane &ln, const SharedState &st,
                                               f32x4 (&S)[2][2])
{
    const uint32_t k_rd = fresh(ln.k_rd);
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        bf16x8 ka[4];
#pragma unroll
        for (uint32_t y = 0; y < 4; ++y)
            ka[y] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(pair + e * 4096u + (k_rd ^ (16u * y))));
        // both tiles side by side, so that their MFMA chains overlap
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) S[e][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int y = 0; y < 4; ++y)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
                S[e][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[y], st.qb[mt][y], S[e][mt], 0, 0, 0);
    }
}

// From the scores of the pair that starts at block b to the weights P8 (the A operands of P V).
// `end` = the first token that does not count: the document's end, or the end of the run's last
// block; only a pair that reaches beyond it is masked.  The caller sees to it that S is not read
// too early after its MFMAs (mfma_result_wait).
__device__ __forceinline__ void shared_softmax_pair(f32x4 (&S)[2][2], uint32_t b, uint32_t end, float scale_log2,
                                                    const SharedLane &ln, SharedState &st, bf16x8 (&P8)[2])
{
    const uint32_t c_ = ln.c_;
    if (b * 16u + 32u > end) {  // a ragged last block, or a last block without a partner
        const uint32_t tok = b * 16u + fresh(c_);  // computed only here
#pragma unroll
        for (int e = 0; e < 2; ++e)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
                    if (tok + 16u * e + 4u * jj >= end) S[e][mt][jj] = neg_inf();
    }
    float mx[2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        const float a = __builtin_fmaxf(__builtin_fmaxf(S[0][mt][0], S[0][mt][1]), __builtin_fmaxf(S[0][mt][2], S[0][mt][3]));
        const float bb = __builtin_fmaxf(__builtin_fmaxf(S[1][mt][0], S[1][mt][1]), __builtin_fmaxf(S[1][mt][2], S[1][mt][3]));
        mx[mt] = __builtin_fmaxf(a, bb) * scale_log2;
    }
    // The running maximum of a row is only a reference point for the exponentials, so it need
    // not be the true maximum: it is brought up to date (a reduction over the lane groups and a
    // rescaling of what is accumulated) only when some lane meets a score more than
    // kLazyMaxSlack above it, which bounds every weight by 2^kLazyMaxSlack.  After the first
    // blocks that almost never happens, and a pair costs one comparison instead of the reduction.
    if (__any(mx[0] > st.m_run[0] + kLazyMaxSlack || mx[1] > st.m_run[1] + kLazyMaxSlack)) {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            const float m_new = __builtin_fmaxf(st.m_run[mt], max_over_lane_groups(mx[mt]));
            const float alpha = __builtin_amdgcn_exp2f(st.m_run[mt] - m_new);  // 0 at the first block, 1 if nothing moved
            st.l_run[mt] *= alpha;
            st.m_run[mt] = m_new;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const float ar = __shfl(alpha, (int)(4u * c_ + jj));  // factor of output row 4 c_ + jj
#pragma unroll
                for (int pp = 0; pp < 8; ++pp) st.O[mt][pp][jj] *= ar;
            }
        }
    }
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        float pr[2][4];
#pragma unroll
        for (int e = 0; e < 2; ++e)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
                pr[e][jj] = __builtin_amdgcn_exp2f(__builtin_fmaf(S[e][mt][jj], scale_log2, -st.m_run[mt]));
        st.l_run[mt] += ((pr[0][0] + pr[0][1]) + (pr[0][2] + pr[0][3])) + ((pr[1][0] + pr[1][1]) + (pr[1][2] + pr[1][3]));
        const u32x4 pk = {pack_bf16(pr[0][0], pr[0][1]), pack_bf16(pr[0][2], pr[0][3]),
                          pack_bf16(pr[1][0], pr[1][1]), pack_bf16(pr[1][2], pr[1][3])};
        P8[mt] = __builtin_bit_cast(bf16x8, pk);
    }
}

// O += P V of a pair; `vsrc` = its V operands
__device__ __forceinline__ void shared_pv_pair(const uint8_t *vsrc, const SharedLane &ln, SharedState &st,
                                               const bf16x8 (&P8)[2])
{
    const uint32_t v_rd = fresh(ln.lane) * 16u;
    u32x4 vq[8];
#pragma unroll
    for (int pp = 0; pp < 8; ++pp) vq[pp] = *reinterpret_cast<const u32x4 *>(vsrc + pp * 1024u + v_rd);
#pragma unroll
    for (int pp = 0; pp < 8; ++pp) {
        const bf16x8 v = __builtin_bit_cast(bf16x8, vq[pp]);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
            st.O[mt][pp] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(P8[mt], v, st.O[mt][pp], 0, 0, 0);
    }
}

// The rounds of one document for a wave that decodes one side (IS_K: the keys) of format P:
// decoder number r of its side takes blocks 2 r and 2 r + 1 of every round of W blocks.
template <uint32_t P, bool IS_K, int W>
__device__ __forceinline__ void shared_rounds(const SharedSide &sd, uint32_t T, uint32_t b0, uint32_t b1,
                                              float scale_log2, uint32_t r, bool active, const SharedLane &ln,
                                              uint8_t (*lds)[W][kSharedBlockLds], uint32_t &set, SharedState &st)
{
    typedef Fmt<P> F;
    const uint32_t lane = ln.lane, c_ = ln.c_;
    u32x4 w[2][F::kWords], m[2];
    m[0] = m[1] = u32x4{0u, 0u, 0u, 0u};
    // the block is clamped to the range's last one instead of skipping the loads: no branch
    // around them, so nothing waits for them before they are needed
    auto fetch = [&](int e, uint32_t b) {
        b = b < b1 ? b : b1 - 1u;
#pragma unroll
        for (uint32_t a = 0; a < F::kWords; ++a)
            w[e][a] = ldg16(sd.tile + ((uint64_t)b * F::kPayload + a * 1024u + lane * 16u));
        if (F::kMeta) m[e] = ldg16(sd.meta + ((uint64_t)b * sd.meta_blk + ((lane * 8u) >> sd.gsh) * 16u));
    };
    fetch(0, b0 + 2u * r);
    fetch(1, b0 + 2u * r + 1u);
    for (uint32_t rb = b0; rb < b1; rb += W) {  // a round: blocks rb .. rb + W - 1
        // ---- this wave's two blocks of the round: decode into the round's buffers
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const uint32_t blk = rb + 2u * r + e;
            uint8_t *pair = lds[set][2u * r];  // this decoder's pair of the round: K 4 KiB + 4 KiB, then V 8 KiB
            if (blk >= b1) {
                // no such block.  If its partner exists, the pair's MFMAs still take this half of
                // the V operands, with weight zero: it must hold numbers (what the keys' half
                // holds does not matter, its scores are replaced)
                if (!IS_K && e == 1 && blk - 1u < b1) {
#pragma unroll
                    for (int pp = 0; pp < 8; ++pp)
                        *reinterpret_cast<u32x2 *>(pair + 8192u + pp * 1024u + fresh(lane) * 16u + 8u) = u32x2{0u, 0u};
                }
                continue;
            }
            uint8_t *dst = pair + e * 4096u;
            u32x4 o[4];  // o[j] = token 4 j + c_, dims 8 n_ .. 8 n_ + 7 as BF16
#pragma unroll
            for (int j = 0; j < 4; ++j) o[j] = decode_octet<P>(plane_raw<P>(w[e], j), m[e][j], sd.base, sd.top);
            if (IS_K) {
                // token t = 4 j + c_, octet n_: slot (n_ ^ t) of row t
                const uint32_t k_wr = fresh(ln.k_wr);
#pragma unroll
                for (uint32_t j = 0; j < 4; ++j)
                    *reinterpret_cast<u32x4 *>(dst + ((k_wr ^ (64u * j)) + 1024u * j)) = o[j];
            } else {
                if (blk * 16u + 16u > T) {  // rows past the document's end
#pragma unroll
                    for (uint32_t j = 0; j < 4; ++j)
                        if (blk * 16u + 4u * j + c_ >= T) o[j] = u32x4{0u, 0u, 0u, 0u};
                }
                // operand pp of P V: value pp of the octet of each of the lane's four tokens; the
                // pair's second block fills the second half of the lane's 16 bytes
                uint8_t *vdst = pair + 8192u + fresh(lane) * 16u + e * 8u;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    u32x2 lo, hi;
                    lo.x = __builtin_amdgcn_perm(o[1][q], o[0][q], 0x05040100u);
                    lo.y = __builtin_amdgcn_perm(o[3][q], o[2][q], 0x05040100u);
                    hi.x = __builtin_amdgcn_perm(o[1][q], o[0][q], 0x07060302u);
                    hi.y = __builtin_amdgcn_perm(o[3][q], o[2][q], 0x07060302u);
                    *reinterpret_cast<u32x2 *>(vdst + (2 * q) * 1024u) = lo;
                    *reinterpret_cast<u32x2 *>(vdst + (2 * q + 1) * 1024u) = hi;
                }
            }
        }
        __syncthreads();
        // the wave's blocks of the next round: in flight while this round is scored.  Issued
        // after the barrier, which waits for every memory access of the wave still under way
        fetch(0, rb + W + 2u * r);
        fetch(1, rb + W + 2u * r + 1u);

        // ---- every wave: its two tiles against the round's blocks, two blocks at a time.  The
        // loop over the pairs is kept a loop: unrolled, the pairs' operand loads and temporaries
        // overlap and the registers do not reach (the 16-bit instances then spill into the path
        // of the prefetch, whose wait a reload shares).
        if (active) {
            const uint32_t nb = b1 - rb < (uint32_t)W ? b1 - rb : (uint32_t)W;
            const uint32_t end = b1 * 16u < T ? b1 * 16u : T;  // the first token that does not count
            const uint8_t *base = lds[set][0];
#pragma unroll 1
            for (uint32_t pr = 0; 2u * pr < nb; ++pr) {
                {
                    const uint8_t *pair = base + pr * (2u * kSharedBlockLds);
                    f32x4 S[2][2];
                    bf16x8 P8[2];
                    shared_qk_pair(pair, ln, st, S);
                    mfma_result_wait();
                    shared_softmax_pair(S, rb + 2u * pr, end, scale_log2, ln, st, P8);
                    shared_pv_pair(pair + 8192u, ln, st, P8);
                }
            }
        }
        set ^= 1u;
    }
    // what follows the document's last P V MFMAs (moves of the output rows between registers, the
    // records) lies behind branches
    mfma_result_wait();
}

template <bool IS_K, int W>
__device__ __forceinline__ void shared_rounds_any(uint32_t prec, const SharedSide &sd, uint32_t T, uint32_t b0,
                                                  uint32_t b1, float scale_log2, uint32_t r, bool active,
                                                  const SharedLane &ln, uint8_t (*lds)[W][kSharedBlockLds],
                                                  uint32_t &set, SharedState &st)
{
    switch (prec) {
    case kP16: shared_rounds<kP16, IS_K, W>(sd, T, b0, b1, scale_log2, r, active, ln, lds, set, st); break;
    case kInt8: shared_rounds<kInt8, IS_K, W>(sd, T, b0, b1, scale_log2, r, active, ln, lds, set, st); break;
    case kInt4: shared_rounds<kInt4, IS_K, W>(sd, T, b0, b1, scale_log2, r, active, ln, lds, set, st); break;
    case kE4M3: shared_rounds<kE4M3, IS_K, W>(sd, T, b0, b1, scale_log2, r, active, ln, lds, set, st); break;
    case kE5M2: shared_rounds<kE5M2, IS_K, W>(sd, T, b0, b1, scale_log2, r, active, ln, lds, set, st); break;
    default: shared_rounds<kGSE8, IS_K, W>(sd, T, b0, b1, scale_log2, r, active, ln, lds, set, st); break;
    }
}

__device__ __forceinline__ SharedSide shared_side(const uint8_t *first, uint32_t prec, uint32_t gsh, uint32_t h,
                                                  uint32_t nblk, bool wanted)
{
    SharedSide sd;
    const bool has_meta = prec == kInt4 || prec == kInt8;
    const uint32_t pay = prec == kInt4 ? 1024u : prec == kP16 ? 4096u : 2048u;
    sd.gsh = gsh;
    sd.meta_blk = has_meta ? 8192u >> gsh : 0u;
    // `first` points at the layer's tile of head 0; the heads' tile records follow one another
    sd.tile = (gbytes)first + (uint64_t)h * ((uint64_t)nblk * (pay + sd.meta_blk) + (prec == kGSE8 ? 16u : 0u));
    sd.meta = sd.tile + (uint64_t)nblk * pay;
    sd.base = sd.top = 0;
    if (wanted && prec == kGSE8) {  // the tile's exponent range follows its payload
        const uint32_t rg = *(const uint32_t __attribute__((address_space(1))) *)(sd.tile + (uint64_t)nblk * 2048u);
        sd.base = (int)(int8_t)(rg & 0xFFu);
        sd.top = (int)(int8_t)((rg >> 8) & 0xFFu) - 2;
    }
    return sd;
}

}  // namespace

// W = 2, 4 or 8 waves, half of them decoding keys and half values; two waves per SIMD keep 256 registers
// each (two tiles of output, their queries, the raw words of two blocks).
template <int W>
__global__ void __launch_bounds__(64 * W, 2) k6_attend_shared(const K6Params p)
{
    // two sets of W block buffers; dynamic, because eight waves need 128 KiB (a workgroup may
    // declare 64 KiB at most statically)
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_bytes[];
    uint8_t (*lds)[W][kSharedBlockLds] = reinterpret_cast<uint8_t (*)[W][kSharedBlockLds]>(lds_bytes);
    K6Run c = p.run[blockIdx.y];
    AttendHdr hdr = {p.n_kv_heads, p.n_q_heads, p.layer, p.scale_log2};
    pin(c.k);
    pin(c.v);
    pin(c.q);
    pin(c.part);
    pin(c.n_tokens);
    pin(c.info);
    pin(c.n_q);
    pin(hdr.n_kv_heads);
    pin(hdr.n_q_heads);
    pin(hdr.scale_log2);
    uint32_t run = c.n_docs, more = c.more;  // the run's documents: this one, then descriptors more, more + 1, ..
    uint32_t first_block = c.first_block, end_block = c.end_block;  // where the run starts in its first and ends in its last
    pin(run);
    pin(more);
    pin(first_block);
    pin(end_block);
    const uint32_t H = hdr.n_kv_heads, G = hdr.n_q_heads / H, M = c.n_q * G;
    const uint32_t n_mt = (M + 15u) >> 4;
    const uint32_t n_mtg = (n_mt + 2u * W - 1u) / (2u * W);
    const uint32_t u = blockIdx.x;
    if (u >= H * n_mtg) return;  // the grid is as wide as the widest run
    const uint32_t mtg = u % n_mtg, h = u / n_mtg;

    SharedLane ln;
    ln.lane = threadIdx.x & 63u;
    ln.c_ = ln.lane >> 4;
    ln.n_ = ln.lane & 15u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t tile0 = (mtg * W + wave) * 2u;  // this wave's tiles: tile0, tile0 + 1
    const bool active = tile0 < n_mt;              // a wave without a tile still decodes
    const bool is_k = wave < (uint32_t)W / 2u;
    const uint32_t r = is_k ? wave : wave - (uint32_t)W / 2u;
    // where this lane reads its K operands: the token of MFMA row n_ is 4 (n_ % 4) + n_ / 4, so
    // that score register jj of lane group c_ belongs to token 4 jj + c_, the token whose values
    // the lane group's plane jj holds
    {
        const uint32_t tau = 4u * (ln.n_ & 3u) + (ln.n_ >> 2);
        ln.k_rd = tau * 256u + (((4u * ln.c_) ^ tau) & 15u) * 16u;  // octet 4 c_ + y of token tau: slot (4 c_ ^ tau) ^ y
        ln.k_wr = ln.c_ * 256u + ((ln.n_ ^ ln.c_) & 15u) * 16u;     // n_ ^ (4 j + c_) = (n_ ^ c_) ^ 4 j
    }

    // Q as the B operand of S^T = K Q^T: lane (c_, n_) holds, for MFMA y, dims
    // 32 c_ + 8 y .. + 7 of query row n_ of the tile (zero rows beyond M)
    SharedState st;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        const uint32_t row = (tile0 + mt) * 16u + ln.n_;
        u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int y = 0; y < 4; ++y) st.qb[mt][y] = __builtin_bit_cast(bf16x8, z);
        if (row < M) {
            const uint32_t qt = row / G, gq = row - qt * G;
            gbytes qp = (gbytes)c.q + ((uint64_t)(qt * hdr.n_q_heads + h * G + gq) * 128u + 32u * ln.c_) * 2u;
#pragma unroll
            for (int y = 0; y < 4; ++y) st.qb[mt][y] = __builtin_bit_cast(bf16x8, ldg16(qp + 16 * y));
        }
        st.m_run[mt] = neg_inf();
        st.l_run[mt] = 0.0f;
#pragma unroll
        for (int pp = 0; pp < 8; ++pp) st.O[mt][pp] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    uint32_t set = 0;
    for (uint32_t d = 0; d < run; ++d) {
        // ---- the document: descriptor d of the run (its first is already here)
        const uint8_t *dk = c.k, *dv = c.v;
        uint32_t T = c.n_tokens, dinfo = c.info;
        if (d) {
            const K6Doc &cd = p.doc[more + d - 1u];
            dk = cd.k;
            dv = cd.v;
            T = cd.n_tokens;
            dinfo = cd.info;
        }
        const uint32_t nblk = (T + 15u) >> 4;
        const uint32_t b0 = d ? 0u : first_block;
        const uint32_t b1 = d + 1u == run ? end_block : nblk;
        if (b0 >= b1) continue;  // cannot happen with a checked launch
        if (is_k) {
            const uint32_t prec = dinfo & 0xFu;
            const SharedSide sd = shared_side(dk, prec, (dinfo >> 4) & 0xFu, h, nblk, true);
            shared_rounds_any<true, W>(prec, sd, T, b0, b1, hdr.scale_log2, r, active, ln, lds, set, st);
        } else {
            const uint32_t prec = (dinfo >> 8) & 0xFu;
            const SharedSide sd = shared_side(dv, prec, (dinfo >> 12) & 0xFu, h, nblk, true);
            shared_rounds_any<false, W>(prec, sd, T, b0, b1, hdr.scale_log2, r, active, ln, lds, set, st);
        }
    }

    // ---- the wave's results, straight from its registers: lane (c_, n_) holds rows
    // 4 c_ + jj, dims 8 n_ + pp of each tile
    if (!active) return;
    uint32_t final = c.final;
    pin(final);
    const float *lse_ptr = c.lse;
    pin(lse_ptr);
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        const uint32_t tile = tile0 + mt;
        if (tile >= n_mt) continue;
        float l_tot = st.l_run[mt];
        l_tot += __shfl_xor(l_tot, 16);
        l_tot += __shfl_xor(l_tot, 32);
        if (final) {
            // The run is everything the request attends to: what the merge would do with its one
            // record is done here.  l_tot of row n_ is in every lane of column n_; the rows this
            // lane holds are 4 c_ + jj.
            gfloats out = (gfloats)c.part;
#pragma unroll
            for (uint32_t jj = 0; jj < 4; ++jj) {
                const uint32_t row = 4u * ln.c_ + jj, mrow = tile * 16u + row;
                const float l_row = __shfl(l_tot, (int)row);
                if (mrow >= M) continue;
                const uint32_t qt = mrow / G, gq = mrow - qt * G;
                f32x4 __attribute__((address_space(1))) *dst = (f32x4 __attribute__((address_space(1))) *)(
                    out + ((uint64_t)qt * hdr.n_q_heads + h * G + gq) * 128u + 8u * ln.n_);
                f32x4 w0, w1;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    w0[e] = l_row > 0.0f ? st.O[mt][e][jj] / l_row : 0.0f;
                    w1[e] = l_row > 0.0f ? st.O[mt][4 + e][jj] / l_row : 0.0f;
                }
                dst[0] = w0;
                dst[1] = w1;
            }
            const uint32_t mrow = tile * 16u + ln.n_;
            if (ln.c_ == 0 && lse_ptr && mrow < M) {
                const uint32_t qt = mrow / G, gq = mrow - qt * G;
                ((gfloats)lse_ptr)[(uint64_t)qt * hdr.n_q_heads + h * G + gq] =
                    l_tot > 0.0f ? (st.m_run[mt] + __builtin_log2f(l_tot)) * 0.69314718055994531f : neg_inf();
            }
            continue;
        }
        gfloats rec = (gfloats)c.part + ((uint64_t)h * n_mt + tile) * kAttendRecFloats;
#pragma unroll
        for (uint32_t jj = 0; jj < 4; ++jj) {
            const uint32_t row = 4u * ln.c_ + jj;
            if (tile * 16u + row >= M) continue;  // no query in this row: the merge never reads it
            f32x4 __attribute__((address_space(1))) *dst =
                (f32x4 __attribute__((address_space(1))) *)(rec + row * 128u + 8u * ln.n_);
            dst[0] = f32x4{st.O[mt][0][jj], st.O[mt][1][jj], st.O[mt][2][jj], st.O[mt][3][jj]};
            dst[1] = f32x4{st.O[mt][4][jj], st.O[mt][5][jj], st.O[mt][6][jj], st.O[mt][7][jj]};
        }
        if (ln.c_ == 0) {
            rec[2048 + ln.n_] = st.m_run[mt];
            rec[2048 + 16 + ln.n_] = l_tot;
        }
    }
}

// The eight-wave build takes 128 KiB of LDS per workgroup; more than 64 KiB has to be asked for
// once per device.  Called when a context is created on the device (not from inside a launch
// that a caller may be capturing into a graph) and, as a fallback, before the first such launch.
hipError_t prepare_k6_shared()
{
    static std::atomic<uint64_t> asked{0};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (asked.load(std::memory_order_acquire) >> dev & 1u) return hipSuccess;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(k6_attend_shared<8>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)(2u * 8u * kSharedBlockLds));
    if (e != hipSuccess) return e;
    asked.fetch_or(1ull << dev, std::memory_order_release);
    return hipSuccess;
}

hipError_t launch_k6_shared(K6Params &p, uint32_t waves, hipStream_t stream, bool check_only)
{
    if (p.n_runs == 0) return hipSuccess;
    if (waves != 2u && waves != 4u && waves != 8u) return hipErrorInvalidValue;
    uint32_t max_mt = 1;
    bool narrow = true;
    hipError_t e = check_k6_args(p, &max_mt, &narrow);
    if (e != hipSuccess) return e;
    const uint64_t width = (uint64_t)p.n_kv_heads * ((max_mt + 2u * waves - 1u) / (2u * waves));
    if (width > 0x7FFFFFFFull) return hipErrorInvalidValue;
    p.mtw = 2;
    if (check_only) return hipSuccess;
    dim3 grid((uint32_t)width, p.n_runs);
    const uint32_t lds_bytes = 2u * waves * kSharedBlockLds;
    if (waves == 2u) hipLaunchKernelGGL((k6_attend_shared<2>), grid, dim3(128), lds_bytes, stream, p);
    else if (waves == 4u) hipLaunchKernelGGL((k6_attend_shared<4>), grid, dim3(256), lds_bytes, stream, p);
    else {
        e = prepare_k6_shared();  // done at ha_rag_create; a no-op from then on
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((k6_attend_shared<8>), grid, dim3(512), lds_bytes, stream, p);
    }
    return hipGetLastError();
}

}  // namespace ha_rag
