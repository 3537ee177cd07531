// gfx950 kernels for attention of a request's query tokens over its packed chunks, without
// building the BF16 cache first (the prefill of Sec. 2.1 consumes the concatenated chunk KV;
// here the consumer reads the compressed chunks of Sec. 2.2 itself).
//
//  k6_attend_partial   one workgroup of kAttendWaves waves per (run of blocks of one document, KV
//      head, group of query rows); the waves take the layout blocks in turn: each decodes K and V blocks to
//      BF16 in registers (the values a load would write), scores them with MFMA and keeps a
//      running softmax; the waves' results are summed in LDS into one unnormalised partial result
//  k7_attend_merge     one workgroup per (query token, query head): merges the partial
//      results of the request's runs into out and the log-sum-exp
//
// head_dim 128 only: a layout block is then 16 tokens x 128 dims, and lane (a = lane/16,
// o = lane%16) of the wave that reads it holds, in plane j, token 4j + a, dims 8o .. 8o+7.
//
// V needs no rearrangement: for the product P V the 16x16x16 MFMA contracts 16 tokens, lane
// group a supplies 4 of them from its 4 planes, and lane column o supplies dim 8o + p, so
// MFMA number p (0..7) takes from each lane the p-th value of each of its 4 planes.
// K is contracted over dims, 8 per lane, with tokens across the 16 lane columns: the raw
// words go through LDS once (as codes, before decoding) and come back with token and dim
// roles of the lane index exchanged.  The score tile is computed transposed (tokens x query
// rows) so that its register layout is already the one P needs as an MFMA operand.
#include "ha_rag_attend_dev.h"

namespace ha_rag {


template <uint32_t KP, uint32_t VP>
struct BlockRegs {  // what a lane loads for one block
    u32x4 kw[Fmt<KP>::kWords], vw[Fmt<VP>::kWords];
    u32x4 vm;
    uint32_t km;
};

template <int MTW>
struct AttendLds {
    static constexpr uint32_t kExchange = kAttendWaves * 4096u;  // one 4 KiB region per wave
    static constexpr uint32_t kCombine = kAttendWaves * 16u * 128u * 4u;  // one output tile per wave, aliases it
    static constexpr uint32_t kBytes = kExchange > kCombine ? kExchange : kCombine;
};

// KP, VP: the formats of the chunk's keys and of its values (the same for a chunk stored whole).
// NARROW: the instance belongs to the kernel that runs three waves per SIMD (168 registers).
template <uint32_t KP, uint32_t VP, int MTW, bool NARROW>
__device__ __forceinline__ void attend_unit(const AttendHdr &p, const K6Run &c,
                                            uint32_t h, uint32_t mtg, uint8_t *lds_all,
                                            float (*sm)[MTW * 16], float (*sl)[MTW * 16])
{
    typedef Fmt<KP> FK;
    typedef Fmt<VP> FV;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t c_ = lane >> 4, n_ = lane & 15u;  // MFMA coordinates: lane group, lane column
    const uint32_t a_ = n_ >> 2, x_ = n_ & 3u;
    const uint32_t H = p.n_kv_heads, G = p.n_q_heads / H, M = c.n_q * G;
    const uint32_t n_mt = (M + 15u) >> 4;
    const uint32_t T = c.n_tokens, nblk = (T + 15u) >> 4;
    const uint32_t kgsh = (c.info >> 4) & 0xFu, vgsh = (c.info >> 12) & 0xFu;
    const uint32_t kmeta_blk = FK::kMeta ? 8192u >> kgsh : 0u, vmeta_blk = FV::kMeta ? 8192u >> vgsh : 0u;
    // c.k / c.v point at the layer's tile of head 0; the heads' tile records follow one another
    gbytes kt = (gbytes)c.k + (uint64_t)h * ((uint64_t)nblk * (FK::kPayload + kmeta_blk) + (KP == kGSE8 ? 16u : 0u));
    gbytes vt = (gbytes)c.v + (uint64_t)h * ((uint64_t)nblk * (FV::kPayload + vmeta_blk) + (VP == kGSE8 ? 16u : 0u));
    gbytes kmeta = kt + (uint64_t)nblk * FK::kPayload;
    gbytes vmeta = vt + (uint64_t)nblk * FV::kPayload;
    gfloats rec0 = (gfloats)c.part + (uint64_t)(h * n_mt) * kAttendRecFloats;

    const uint32_t b0 = c.first_block, b1 = c.end_block;  // the run: blocks of this one document

    int kbase = 0, ktop = 0, vbase = 0, vtop = 0;
    if (KP == kGSE8) {
        const uint32_t kr = *(const uint32_t __attribute__((address_space(1))) *)(kt + (uint64_t)nblk * 2048u);
        kbase = (int)(int8_t)(kr & 0xFFu);
        ktop = (int)(int8_t)((kr >> 8) & 0xFFu) - 2;
    }
    if (VP == kGSE8) {
        const uint32_t vr = *(const uint32_t __attribute__((address_space(1))) *)(vt + (uint64_t)nblk * 2048u);
        vbase = (int)(int8_t)(vr & 0xFFu);
        vtop = (int)(int8_t)((vr >> 8) & 0xFFu) - 2;
    }

    // Q as the B operand of S^T = K Q^T: lane (c_, n_) holds, for MFMA y, dims
    // 32 c_ + 8 y .. + 7 of query row n_ of the tile (zero rows beyond M)
    bf16x8 qb[MTW][4];
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt) {
        const uint32_t row = (mtg * MTW + mt) * 16u + n_;
        u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int y = 0; y < 4; ++y) qb[mt][y] = __builtin_bit_cast(bf16x8, z);
        if (row < M) {
            const uint32_t qt = row / G, gq = row - qt * G;
            gbytes qp = (gbytes)c.q +
                                ((uint64_t)(qt * p.n_q_heads + h * G + gq) * 128u + 32u * c_) * 2u;
#pragma unroll
            for (int y = 0; y < 4; ++y) qb[mt][y] = __builtin_bit_cast(bf16x8, ldg16(qp + 16 * y));
        }
    }

    float m_run[MTW], l_run[MTW];
    f32x4 O[MTW][8];
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt) {
        m_run[mt] = neg_inf();
        l_run[mt] = 0.0f;
#pragma unroll
        for (int pp = 0; pp < 8; ++pp) O[mt][pp] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // K after the exchange: this lane holds token tk = 4 x_ + a_ of the block and, for MFMA y,
    // the octet 4 c_ + y, which lane 16 a_ + 4 c_ + y loaded as its plane x_
    const uint32_t src_lane0 = 16u * a_ + 4u * c_;
    uint32_t k_entry = 0;  // scale/zero entry of (token tk, dims 32 c_ ..) in a meta block
    if (FK::kMeta) {
        const uint32_t grp = ((4u * x_ + a_) * 128u + 32u * c_) >> kgsh;
        k_entry = (grp & ((512u >> kgsh) - 1u)) * 4u + (grp >> (9u - kgsh));
    }
    uint8_t *lds = lds_all + wave * 4096u;
    u32x4 *lds_w = reinterpret_cast<u32x4 *>(lds);

    auto load_block = [&](uint32_t b, BlockRegs<KP, VP> &r) {
#pragma unroll
        for (uint32_t a = 0; a < FK::kWords; ++a)
            r.kw[a] = ldg16(kt + ((uint64_t)b * FK::kPayload + a * 1024u + lane * 16u));
#pragma unroll
        for (uint32_t a = 0; a < FV::kWords; ++a)
            r.vw[a] = ldg16(vt + ((uint64_t)b * FV::kPayload + a * 1024u + lane * 16u));
        r.km = 0;
        r.vm = u32x4{0u, 0u, 0u, 0u};
        if (FK::kMeta)
            r.km = *(const uint32_t __attribute__((address_space(1))) *)(kmeta + ((uint64_t)b * kmeta_blk + 4u * k_entry));
        if (FV::kMeta) r.vm = ldg16(vmeta + ((uint64_t)b * vmeta_blk + ((lane * 8u) >> vgsh) * 16u));
    };

    // the waves of the workgroup take the blocks of the run in turn; each wave fetches its
    // next block before it works on the current one
    auto process = [&](uint32_t b, const BlockRegs<KP, VP> &cur) {
        const bool ragged = b * 16u + 16u > T;  // only the chunk's last block can be

        // ---- K: exchange through LDS, decode, S^T = K Q^T
#pragma unroll
        for (uint32_t a = 0; a < FK::kWords; ++a) lds_w[a * 64u + lane] = cur.kw[a];
        wave_lds_sync();
        bf16x8 ka[4];
#pragma unroll
        for (int y = 0; y < 4; ++y) {
            const uint32_t i_src = src_lane0 + y;
            u32x4 raw = {0u, 0u, 0u, 0u};
            if (KP == kInt4) {
                raw.x = *reinterpret_cast<const uint32_t *>(lds + 16u * i_src + 4u * x_);
            } else if (KP == kP16) {
                raw = *reinterpret_cast<const u32x4 *>(lds + 1024u * x_ + 16u * i_src);
            } else {
                const u32x2 t = *reinterpret_cast<const u32x2 *>(lds + 1024u * (x_ >> 1) + 16u * i_src + 8u * (x_ & 1u));
                raw.x = t.x;
                raw.y = t.y;
            }
            ka[y] = __builtin_bit_cast(bf16x8, decode_octet<KP>(raw, cur.km, kbase, ktop));
        }
        wave_lds_sync();

        s16x4 pa[MTW];
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt) {
            f32x4 S = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int y = 0; y < 4; ++y)
                S = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[y], qb[mt][y], S, 0, 0, 0);
            mfma_result_wait();  // S is first read behind the branch below
            // S[jj] = q k (unscaled) of token 4 jj + c_ of the block and query row n_
            if (ragged) {
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
                    if (b * 16u + 4u * jj + c_ >= T) S[jj] = neg_inf();
            }
            const float mx = __builtin_fmaxf(__builtin_fmaxf(S[0], S[1]), __builtin_fmaxf(S[2], S[3])) * p.scale_log2;
            // The running maximum of a row is only a reference point for the exponentials: it
            // is brought up to date (a reduction over the lane groups and a rescaling of what is
            // accumulated) only when some lane meets a score more than kLazyMaxSlack above it,
            // which bounds every weight by 2^kLazyMaxSlack.  After the first blocks that almost
            // never happens, and a block costs one comparison instead of the reduction.
            if (__any(mx > m_run[mt] + kLazyMaxSlack)) {
                const float m_new = __builtin_fmaxf(m_run[mt], max_over_lane_groups(mx));
                const float alpha = __builtin_amdgcn_exp2f(m_run[mt] - m_new);  // 0 at the first block
                l_run[mt] *= alpha;
                m_run[mt] = m_new;
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const float ar = __shfl(alpha, (int)(4u * c_ + jj));  // factor of output row 4 c_ + jj
#pragma unroll
                    for (int pp = 0; pp < 8; ++pp) O[mt][pp][jj] *= ar;
                }
            }
            float pr[4];
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
                pr[jj] = __builtin_amdgcn_exp2f(__builtin_fmaf(S[jj], p.scale_log2, -m_run[mt]));
            l_run[mt] += (pr[0] + pr[1]) + (pr[2] + pr[3]);
            const u32x2 pk = {pack_bf16(pr[0], pr[1]), pack_bf16(pr[2], pr[3])};
            pa[mt] = __builtin_bit_cast(s16x4, pk);
        }

        // ---- V: decode the lane's four planes, regroup by position, O += P V
        u32x4 vr[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            vr[j] = decode_octet<VP>(plane_raw<VP>(cur.vw, j), cur.vm[j], vbase, vtop);
        if (ragged) {  // rows past the chunk's end
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (b * 16u + 4u * j + c_ >= T) vr[j] = u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int pp = 0; pp < 8; ++pp) {
            const uint32_t sel = (pp & 1) ? 0x07060302u : 0x05040100u;
            const u32x2 t = {__builtin_amdgcn_perm(vr[1][pp >> 1], vr[0][pp >> 1], sel),
                             __builtin_amdgcn_perm(vr[3][pp >> 1], vr[2][pp >> 1], sel)};
            const s16x4 vb = __builtin_bit_cast(s16x4, t);
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt)
                O[mt][pp] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pa[mt], vb, O[mt][pp], 0, 0, 0);
        }
    };
    // A ring of kStages register sets: while a block is worked on, the loads of the next
    // kStages - 1 blocks of this wave are in flight.  What is in flight per compute unit has
    // to cover the memory latency at full bandwidth, and a block of a 4-bit chunk is a quarter
    // of the bytes of a 16-bit one, so narrow formats get a deeper ring; the 16-bit pairs take
    // the registers that two waves per SIMD leave them (3 sets: 217 registers; 2 sets measured
    // 6 % slower on 16-bit chunks, 4 the same as 3).  The loop is unrolled over the ring so
    // that no block is copied from one set to another.
    constexpr uint32_t kWordsKV = FK::kWords + FV::kWords;
    constexpr int kStages = MTW > 1 ? 2  // registers are short
                            : NARROW ? (kWordsKV <= 2 ? 3 : 2)
                                     : (kWordsKV <= 2 ? 4 : 3);
    BlockRegs<KP, VP> ring[kStages];
    uint32_t b = b0 + wave;
    // Every load below is issued whether or not its block exists (a block past the run's end
    // is replaced by one this wave has already fetched, a hit in the cache): with a branch
    // around the loads the compiler has to wait as if they had not been issued, which then
    // waits for part of the block just requested - a full memory latency per block.
#pragma unroll
    for (int i = 0; i < kStages - 1; ++i) {
        const uint32_t first = b + i * kAttendWaves;
        load_block(first < b1 ? first : b1 - 1u, ring[i]);
    }
    if (b < b1) {
        for (;;) {
#pragma unroll
            for (int i = 0; i < kStages; ++i) {
                const uint32_t ahead = b + (kStages - 1) * kAttendWaves;
                load_block(ahead < b1 ? ahead : b, ring[(i + kStages - 1) % kStages]);
                process(b, ring[i]);
                b += kAttendWaves;
                if (b >= b1) goto blocks_done;
            }
        }
    }
blocks_done:

    // ---- the waves' results: each wave leaves its rows, maxima and sums in LDS; then all
    // threads bring them to one maximum per row, add them up and write the record
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt) {
        float l_tot = l_run[mt];
        l_tot += __shfl_xor(l_tot, 16);
        l_tot += __shfl_xor(l_tot, 32);
        if (c_ == 0) {
            sm[wave][mt * 16 + n_] = m_run[mt];
            sl[wave][mt * 16 + n_] = l_tot;
        }
    }
    float *acc = reinterpret_cast<float *>(lds_all);  // [wave][16 rows][128]
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt) {
        __syncthreads();  // the exchange areas (first tile) or the previous tile's sums are done with
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            f32x4 *dst = reinterpret_cast<f32x4 *>(acc + wave * 2048u + (4u * c_ + jj) * 128u + 8u * n_);
            dst[0] = f32x4{O[mt][0][jj], O[mt][1][jj], O[mt][2][jj], O[mt][3][jj]};
            dst[1] = f32x4{O[mt][4][jj], O[mt][5][jj], O[mt][6][jj], O[mt][7][jj]};
        }
        __syncthreads();
        const uint32_t mtile = mtg * MTW + mt;
        if (mtile >= n_mt) continue;
        gfloats rec = rec0 + (uint64_t)mtile * kAttendRecFloats;
#pragma unroll
        for (uint32_t k = 0; k < 512u / (64u * kAttendWaves); ++k) {  // 512 16-byte words of output per tile
            const uint32_t i = threadIdx.x + 64u * kAttendWaves * k, row = mt * 16u + (i >> 5);
            if (mtile * 16u + (i >> 5) >= M) continue;  // no query in this row: the merge never reads it
            float m_all = sm[0][row];
#pragma unroll
            for (uint32_t w = 1; w < kAttendWaves; ++w) m_all = __builtin_fmaxf(m_all, sm[w][row]);
            f32x4 sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (uint32_t w = 0; w < kAttendWaves; ++w) {
                // a wave that had no block has m = -inf and l = 0: nothing to add
                const float f = sl[w][row] > 0.0f ? __builtin_amdgcn_exp2f(sm[w][row] - m_all) : 0.0f;
                sum += reinterpret_cast<const f32x4 *>(acc + w * 2048u)[i] * f;
            }
            ((f32x4 __attribute__((address_space(1))) *)rec)[i] = sum;
        }
        if (threadIdx.x < 16u) {
            const uint32_t row = mt * 16u + threadIdx.x;
            float m_all = sm[0][row];
#pragma unroll
            for (uint32_t w = 1; w < kAttendWaves; ++w) m_all = __builtin_fmaxf(m_all, sm[w][row]);
            float l_all = 0.0f;
#pragma unroll
            for (uint32_t w = 0; w < kAttendWaves; ++w)
                if (sl[w][row] > 0.0f) l_all += sl[w][row] * __builtin_amdgcn_exp2f(sm[w][row] - m_all);
            rec[2048 + threadIdx.x] = m_all;
            rec[2048 + 16 + threadIdx.x] = l_all;
        }
    }
}

// One instance per pair of formats (whole chunks use the six on the diagonal).  The kernel for
// narrow formats leaves out every pair with a 16-bit side: those need more registers than three
// waves per SIMD leave.
template <uint32_t KP, uint32_t VP, int MTW, bool NARROW>
__device__ __forceinline__ void attend_pair(const AttendHdr &hdr, const K6Run &c, uint32_t h,
                                            uint32_t mtg, uint8_t *lds, float (*sm)[MTW * 16],
                                            float (*sl)[MTW * 16])
{
    if constexpr (!(NARROW && (KP == kP16 || VP == kP16)))
        attend_unit<KP, VP, MTW, NARROW>(hdr, c, h, mtg, lds, sm, sl);
}

template <uint32_t KP, int MTW, bool NARROW>
__device__ __forceinline__ void attend_values(const AttendHdr &hdr, const K6Run &c, uint32_t h,
                                              uint32_t mtg, uint8_t *lds, float (*sm)[MTW * 16],
                                              float (*sl)[MTW * 16])
{
    switch ((c.info >> 8) & 0xFu) {
    case kP16: attend_pair<KP, kP16, MTW, NARROW>(hdr, c, h, mtg, lds, sm, sl); break;
    case kInt8: attend_pair<KP, kInt8, MTW, NARROW>(hdr, c, h, mtg, lds, sm, sl); break;
    case kInt4: attend_pair<KP, kInt4, MTW, NARROW>(hdr, c, h, mtg, lds, sm, sl); break;
    case kE4M3: attend_pair<KP, kE4M3, MTW, NARROW>(hdr, c, h, mtg, lds, sm, sl); break;
    case kE5M2: attend_pair<KP, kE5M2, MTW, NARROW>(hdr, c, h, mtg, lds, sm, sl); break;
    default: attend_pair<KP, kGSE8, MTW, NARROW>(hdr, c, h, mtg, lds, sm, sl); break;
    }
}

// The second launch bound is waves per SIMD.  With two (256 registers) the accumulators stay in
// ordinary vector registers, with no copies to and from the accumulation registers around the
// rescale branch, and every pair of formats fits.  Without a 16-bit side one query tile fits
// in the 168 registers of three waves per SIMD, which measured 10 % faster (the kernel is bound
// by instruction issue); 16-bit pairs spill there and lose a quarter.
template <int MTW, bool NARROW>
__global__ void __launch_bounds__(64 * kAttendWaves, NARROW ? 3 : 2) k6_attend_partial(const K6Params p)
{
    __shared__ __attribute__((aligned(16))) uint8_t lds[AttendLds<MTW>::kBytes];
    __shared__ float sm[kAttendWaves][MTW * 16], sl[kAttendWaves][MTW * 16];
    // the whole descriptor and the header at once, before anything depends on a part of them
    K6Run c = p.run[blockIdx.y];
    AttendHdr hdr = {p.n_kv_heads, p.n_q_heads, p.layer, p.scale_log2};
    pin(c.k);
    pin(c.v);
    pin(c.q);
    pin(c.part);
    pin(c.n_tokens);
    pin(c.info);
    pin(c.n_q);
    pin(c.first_block);
    pin(c.end_block);
    pin(hdr.n_kv_heads);
    pin(hdr.n_q_heads);
    pin(hdr.layer);
    pin(hdr.scale_log2);
    const uint32_t G = hdr.n_q_heads / hdr.n_kv_heads;
    const uint32_t n_mt = (c.n_q * G + 15u) >> 4;
    const uint32_t n_mtg = (n_mt + MTW - 1u) / MTW;
    const uint32_t u = blockIdx.x;
    if (u >= hdr.n_kv_heads * n_mtg) return;  // the grid is as wide as the widest run
    const uint32_t mtg = u % n_mtg;
    const uint32_t h = u / n_mtg;
    switch (c.info & 0xFu) {
    case kP16: attend_values<kP16, MTW, NARROW>(hdr, c, h, mtg, lds, sm, sl); break;
    case kInt8: attend_values<kInt8, MTW, NARROW>(hdr, c, h, mtg, lds, sm, sl); break;
    case kInt4: attend_values<kInt4, MTW, NARROW>(hdr, c, h, mtg, lds, sm, sl); break;
    case kE4M3: attend_values<kE4M3, MTW, NARROW>(hdr, c, h, mtg, lds, sm, sl); break;
    case kE5M2: attend_values<kE5M2, MTW, NARROW>(hdr, c, h, mtg, lds, sm, sl); break;
    default: attend_values<kGSE8, MTW, NARROW>(hdr, c, h, mtg, lds, sm, sl); break;
    }
}

// Checks what both attention launches assume of their arguments: the runs, their further
// documents in rows behind them, every run's block range.  *max_mt receives the most query tiles
// of a run's request, *narrow whether no document has a 16-bit side.
hipError_t check_k6_args(const K6Params &p, uint32_t *max_mt, bool *narrow)
{
    if (p.n_runs == 0 || p.n_runs > kAttendMaxRuns || p.n_kv_heads == 0 || p.n_q_heads % p.n_kv_heads ||
        p.doc_first != K6Params::docs_behind(p.n_runs) || p.doc_end < p.doc_first || p.doc_end > kAttendMaxDocs)
        return hipErrorInvalidValue;
    const uint32_t G = p.n_q_heads / p.n_kv_heads;
    auto doc_ok = [&](const uint8_t *k, const uint8_t *v, uint32_t n_tokens, uint32_t info) {
        const uint32_t kprec = info & 0xFu, kgsh = (info >> 4) & 0xFu;
        const uint32_t vprec = (info >> 8) & 0xFu, vgsh = (info >> 12) & 0xFu;
        if (info >> 16 || kprec > kGSE8 || vprec > kGSE8 || !k || !v || ((uintptr_t)k & 15u) ||
            ((uintptr_t)v & 15u) || n_tokens == 0 || n_tokens > 0x7FFFFFFu)
            return false;
        if ((kprec == kInt4 || kprec == kInt8) && (kgsh < 5 || kgsh > 7)) return false;
        if ((vprec == kInt4 || vprec == kInt8) && (vgsh < 5 || vgsh > 7)) return false;
        if (kprec == kP16 || vprec == kP16) *narrow = false;
        return true;
    };
    *max_mt = 1;
    *narrow = true;
    for (uint32_t i = p.doc_first; i < p.doc_end; ++i)
        if (!doc_ok(p.doc[i].k, p.doc[i].v, p.doc[i].n_tokens, p.doc[i].info)) return hipErrorInvalidValue;
    uint32_t next = p.doc_first;  // the runs' further documents lie in the runs' order, without gaps
    for (uint32_t i = 0; i < p.n_runs; ++i) {
        const K6Run &c = p.run[i];
        if (!doc_ok(c.k, c.v, c.n_tokens, c.info) || c.n_docs == 0 || !c.q || !c.part || c.n_q == 0 ||
            ((uintptr_t)c.q & 15u) || ((uintptr_t)c.part & 15u) || (uint64_t)c.n_q * G > 0xFFFFFFull ||
            c.final > 1u || (!c.final && c.lse) || ((uintptr_t)c.lse & 3u))
            return hipErrorInvalidValue;
        if (c.n_docs > 1u && (c.more != next || c.n_docs - 1u > p.doc_end - next)) return hipErrorInvalidValue;
        next += c.n_docs - 1u;
        // the run's block range: starts inside its first document, ends inside its last, not empty
        const uint32_t nb_first = (c.n_tokens + 15u) >> 4;
        const uint32_t nb_last = c.n_docs > 1u ? (p.doc[next - 1u].n_tokens + 15u) >> 4 : nb_first;
        if (c.first_block >= nb_first || c.end_block > nb_last || c.end_block == 0 ||
            (c.n_docs == 1u && c.end_block <= c.first_block))
            return hipErrorInvalidValue;
        const uint32_t n_mt = (c.n_q * G + 15u) >> 4;
        if (n_mt > *max_mt) *max_mt = n_mt;
    }
    return next == p.doc_end ? hipSuccess : hipErrorInvalidValue;
}

hipError_t launch_k6(K6Params &p, hipStream_t stream, bool check_only)
{
    if (p.n_runs == 0) return hipSuccess;
    uint32_t max_mt = 1;
    bool narrow = true;  // no 16-bit side in this launch
    const hipError_t e = check_k6_args(p, &max_mt, &narrow);
    if (e != hipSuccess) return e;
    for (uint32_t i = 0; i < p.n_runs; ++i)
        if (p.run[i].n_docs != 1u || p.run[i].final) return hipErrorInvalidValue;  // this kernel's runs stay inside one document and always leave records
    // Two tiles (32 query rows) per workgroup is the most that still runs two waves per SIMD;
    // four tiles at one wave per SIMD measured 35 % slower than two passes of two.
    p.mtw = max_mt >= 2 ? 2u : 1u;
    const uint64_t width = (uint64_t)p.n_kv_heads * ((max_mt + p.mtw - 1u) / p.mtw);
    if (width > 0x7FFFFFFFull) return hipErrorInvalidValue;
    if (check_only) return hipSuccess;
    dim3 grid((uint32_t)width, p.n_runs), block(64 * kAttendWaves);
    if (p.mtw == 2) hipLaunchKernelGGL((k6_attend_partial<2, false>), grid, block, 0, stream, p);
    else if (narrow) hipLaunchKernelGGL((k6_attend_partial<1, true>), grid, block, 0, stream, p);
    else hipLaunchKernelGGL((k6_attend_partial<1, false>), grid, block, 0, stream, p);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// K7.  One workgroup per (query token, query head), made of groups of 32 threads (four dims
// each).  The groups share the row's records between them, so that a single request with many
// records (long chunks cut into many runs) is merged in one or two rounds of loads instead of record
// after record; then 128 threads, one per dim, merge the groups' results through LDS.
// ---------------------------------------------------------------------------
constexpr uint32_t kMergeGroups = 32;  // at most: 1024 threads

__global__ void __launch_bounds__(32 * kMergeGroups) k7_attend_merge(const K7Params p)
{
    __shared__ __attribute__((aligned(16))) float s_acc[kMergeGroups][128];
    __shared__ float s_m[kMergeGroups], s_l[kMergeGroups];
    // grid: x = row of the request (the grid is as wide as the largest), y = request; the
    // descriptor is fetched at once
    K7Req r = p.r[blockIdx.y];
    uint32_t n_kv_heads = p.n_kv_heads, n_q_heads = p.n_q_heads;
    pin(r.part);
    pin(r.out);
    pin(r.lse);
    pin(r.n_q);
    pin(r.n_runs);
    pin(n_kv_heads);
    pin(n_q_heads);
    const uint32_t rr = blockIdx.x;
    if (rr >= r.n_q * n_q_heads) return;  // the whole workgroup
    const uint32_t qt = rr / n_q_heads, hq = rr - qt * n_q_heads;
    const uint32_t G = n_q_heads / n_kv_heads;
    const uint32_t h = hq / G, gq = hq - h * G;
    const uint32_t mrow = qt * G + gq, mt = mrow >> 4, ri = mrow & 15u;
    const uint32_t n_mt = (r.n_q * G + 15u) >> 4;
    const uint32_t d4 = threadIdx.x & 31u, g = threadIdx.x >> 5, n_g = blockDim.x >> 5;  // n_g >= 4
    const uint64_t run_stride = (uint64_t)n_kv_heads * n_mt * kAttendRecFloats;  // records are [run][head][tile]
    const float *first = r.part + ((uint64_t)h * n_mt + mt) * kAttendRecFloats;

    // Group g takes records g, g + n_g, ..., four at a time: their maxima, sums and this
    // thread's four dims are fetched together (every thread of a group reads the same m and l:
    // broadcast loads), then folded into a running maximum like the blocks inside a record were.
    const uint32_t n_units = r.n_runs;
    float m_max = neg_inf(), l_sum = 0.0f;
    f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
    for (uint32_t u0 = g; u0 < n_units; u0 += 4u * n_g) {
        float m[4], l[4];
        f32x4 o[4];
#pragma unroll
        for (uint32_t k = 0; k < 4; ++k) {
            const bool have = u0 + k * n_g < n_units;
            const uint32_t u = have ? u0 + k * n_g : n_units - 1u;
            const float *rec = first + u * run_stride;
            m[k] = rec[2048 + ri];
            l[k] = have ? rec[2048 + 16 + ri] : 0.0f;
            o[k] = *reinterpret_cast<const f32x4 *>(rec + ri * 128u + 4u * d4);
        }
#pragma unroll
        for (uint32_t k = 0; k < 4; ++k) {
            if (l[k] > 0.0f) {  // the same for the whole group; an empty record holds no output rows
                const float m_new = __builtin_fmaxf(m_max, m[k]);
                const float fa = __builtin_amdgcn_exp2f(m_max - m_new);  // 0 at the first record
                const float fb = __builtin_amdgcn_exp2f(m[k] - m_new);
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[e] = __builtin_fmaf(o[k][e], fb, acc[e] * fa);
                l_sum = __builtin_fmaf(l[k], fb, l_sum * fa);
                m_max = m_new;
            }
        }
    }
    *reinterpret_cast<f32x4 *>(&s_acc[g][4u * d4]) = acc;
    if (d4 == 0) {
        s_m[g] = m_max;
        s_l[g] = l_sum;
    }
    __syncthreads();
    const uint32_t d = threadIdx.x;
    if (d >= 128u) return;
    // every group's maximum and sum at once (no branch between the LDS reads), then the weights
    float gm[kMergeGroups], gl[kMergeGroups];
#pragma unroll
    for (uint32_t i = 0; i < kMergeGroups; ++i) {
        gm[i] = s_m[i];
        gl[i] = i < n_g ? s_l[i] : 0.0f;  // what lies beyond the launch's groups was never written
    }
    m_max = neg_inf();
#pragma unroll
    for (uint32_t i = 0; i < kMergeGroups; ++i) m_max = gl[i] > 0.0f ? __builtin_fmaxf(m_max, gm[i]) : m_max;
    float out = 0.0f;
    l_sum = 0.0f;
#pragma unroll
    for (uint32_t i = 0; i < kMergeGroups; ++i) {
        const float a = s_acc[i][d];
        const float w = __builtin_amdgcn_exp2f(gm[i] - m_max);
        out = gl[i] > 0.0f ? __builtin_fmaf(a, w, out) : out;
        l_sum = gl[i] > 0.0f ? __builtin_fmaf(gl[i], w, l_sum) : l_sum;
    }
    const uint64_t o = (uint64_t)qt * n_q_heads + hq;
    r.out[o * 128u + d] = l_sum > 0.0f ? out / l_sum : 0.0f;
    if (d == 0 && r.lse)
        r.lse[o] = l_sum > 0.0f ? (m_max + __builtin_log2f(l_sum)) * 0.69314718055994531f : neg_inf();
}

// The merge for requests with many query rows: one workgroup per (request, KV head, 16-row
// query tile), 16 threads a row, 8 dims a thread.  A record is then read as the contiguous
// 8 KiB it is, by one workgroup, and a request of hundreds of rows needs hundreds of workgroups
// instead of one for each of its rows.
__global__ void __launch_bounds__(256) k7_attend_merge_tiles(const K7Params p)
{
    typedef const float __attribute__((address_space(1))) *gfloats;
    typedef const f32x4 __attribute__((address_space(1))) *gquads;
    K7Req r = p.r[blockIdx.y];
    uint32_t n_kv_heads = p.n_kv_heads, n_q_heads = p.n_q_heads;
    pin(r.part);
    pin(r.out);
    pin(r.lse);
    pin(r.n_q);
    pin(r.n_runs);
    pin(n_kv_heads);
    pin(n_q_heads);
    const uint32_t G = n_q_heads / n_kv_heads, M = r.n_q * G;
    const uint32_t n_mt = (M + 15u) >> 4;
    if (blockIdx.x >= n_kv_heads * n_mt) return;  // the grid is as wide as the largest request
    const uint32_t h = blockIdx.x / n_mt, mt = blockIdx.x - h * n_mt;
    const uint32_t ri = threadIdx.x >> 4, d8 = threadIdx.x & 15u;
    const uint32_t mrow = mt * 16u + ri;
    if (mrow >= M) return;  // rows without a query are not in the records either
    const uint64_t run_stride = (uint64_t)n_kv_heads * n_mt * kAttendRecFloats;  // records are [run][head][tile]
    gfloats first = (gfloats)r.part + ((uint64_t)h * n_mt + mt) * kAttendRecFloats;
    const uint32_t n_units = r.n_runs;
    float m_max = neg_inf(), l_sum = 0.0f;
    f32x4 acc[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
    for (uint32_t u0 = 0; u0 < n_units; u0 += 4u) {
        float m[4], l[4];
        f32x4 o[4][2];
#pragma unroll
        for (uint32_t k = 0; k < 4; ++k) {  // four records under way at a time
            const bool have = u0 + k < n_units;
            const uint32_t u = have ? u0 + k : n_units - 1u;
            gfloats rec = first + u * run_stride;
            m[k] = rec[2048 + ri];
            l[k] = have ? rec[2048 + 16 + ri] : 0.0f;
            o[k][0] = ((gquads)(rec + ri * 128u + 8u * d8))[0];
            o[k][1] = ((gquads)(rec + ri * 128u + 8u * d8))[1];
        }
#pragma unroll
        for (uint32_t k = 0; k < 4; ++k) {
            if (l[k] > 0.0f) {  // an empty record holds no output rows
                const float m_new = __builtin_fmaxf(m_max, m[k]);
                const float fa = __builtin_amdgcn_exp2f(m_max - m_new);  // 0 at the first record
                const float fb = __builtin_amdgcn_exp2f(m[k] - m_new);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    acc[0][e] = __builtin_fmaf(o[k][0][e], fb, acc[0][e] * fa);
                    acc[1][e] = __builtin_fmaf(o[k][1][e], fb, acc[1][e] * fa);
                }
                l_sum = __builtin_fmaf(l[k], fb, l_sum * fa);
                m_max = m_new;
            }
        }
    }
    const uint32_t qt = mrow / G, gq = mrow - qt * G;
    const uint64_t orow = (uint64_t)qt * n_q_heads + h * G + gq;
    f32x4 __attribute__((address_space(1))) *dst =
        (f32x4 __attribute__((address_space(1))) *)((float __attribute__((address_space(1))) *)r.out + orow * 128u + 8u * d8);
    f32x4 w0, w1;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        w0[e] = l_sum > 0.0f ? acc[0][e] / l_sum : 0.0f;
        w1[e] = l_sum > 0.0f ? acc[1][e] / l_sum : 0.0f;
    }
    dst[0] = w0;
    dst[1] = w1;
    if (d8 == 0 && r.lse)
        r.lse[orow] = l_sum > 0.0f ? (m_max + __builtin_log2f(l_sum)) * 0.69314718055994531f : neg_inf();
}

hipError_t launch_k7(K7Params &p, hipStream_t stream, bool check_only)
{
    if (p.n_reqs == 0) return hipSuccess;
    if (p.n_reqs > kMaxMergeReqs || p.n_kv_heads == 0 || p.n_q_heads % p.n_kv_heads)
        return hipErrorInvalidValue;
    uint64_t width = 0, max_units = 0, tile_width = 0;
    const uint32_t G = p.n_q_heads / p.n_kv_heads;
    uint32_t max_mt = 0;
    for (uint32_t i = 0; i < p.n_reqs; ++i) {
        const K7Req &r = p.r[i];
        // a request without a token to attend to (n_runs 0) gets zeros and lse = -inf
        if ((r.n_runs && !r.part) || !r.out || r.n_q == 0)
            return hipErrorInvalidValue;
        const uint64_t rows = (uint64_t)r.n_q * p.n_q_heads;
        if (rows > width) width = rows;
        const uint64_t n_mt = ((uint64_t)r.n_q * G + 15u) >> 4;
        if (n_mt > max_mt) max_mt = (uint32_t)(n_mt > 0xFFFFFFFFull ? 0xFFFFFFFFull : n_mt);
        if (n_mt * p.n_kv_heads > tile_width) tile_width = n_mt * p.n_kv_heads;
        if (r.n_runs > max_units) max_units = r.n_runs;
    }
    if (width > 0x7FFFFFFFull) return hipErrorInvalidValue;
    if (check_only) return hipSuccess;
    if (max_mt > 2u) {  // the requests of the shared kernel: merge tile by tile
        hipLaunchKernelGGL(k7_attend_merge_tiles, dim3((uint32_t)tile_width, p.n_reqs), dim3(256), 0, stream, p);
        return hipGetLastError();
    }
    // one group per two records of the longest row if that fits (a group fetches four at a
    // time), in whole waves, at least the 128 threads that write the row
    const uint64_t want = (max_units + 1u) / 2u;
    uint32_t groups = want < 4u ? 4u : want > kMergeGroups ? kMergeGroups : (uint32_t)want;
    groups = (groups + 1u) & ~1u;
    hipLaunchKernelGGL(k7_attend_merge, dim3((uint32_t)width, p.n_reqs), dim3(32 * groups), 0, stream, p);
    return hipGetLastError();
}

}  // namespace ha_rag
