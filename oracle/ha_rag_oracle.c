/*
 * CPU oracle for the hotness-aware mixed-precision KV-chunk load of HA-RAG
 * (Sec. 2.2.3 / Algorithm 1 step 3 "Compression(S_i, chunks_i)" and the online
 * "load + decompress" stage of Sec. 2.1, Fig. 3).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, single
 * threaded reference that only the tests, the smoke check and the CPU-baseline
 * leg of the benchmark may call.  It shares no source, header, table or helper
 * with the HIP library and includes nothing from it.
 *
 * What the paper fixes and what it leaves open.  The paper stores full
 * precision KV as BF16 (Sec. 2.2.1, Sec. 3.1 "Performance Baseline") and
 * compresses each chunk, as a whole, to a precision chosen from its access
 * frequency rank (Algorithm 1).  For its integer scheme it gives the code
 * range only (Sec. 2.2.2); it defines no scale, zero point, group or byte
 * layout.  The readings used here are this build's own and are stated where they
 * are applied below: unsigned codes, asymmetric, one fp16 scale and one fp16 zero
 * per group of g consecutive head_dim elements, directed rounding of scale and
 * zero, round-half-even codes, the block-permuted byte layout; for the paper's
 * FP8 and GSE-8 schemes see their sections.  Because the encoding is lossy, the
 * oracle is the algorithm taken step by step; every function is pinned by the tests in tests/test_oracle_*.py against
 * closed forms, invariants, exhaustive enumeration and library conversions.
 *
 * Arithmetic: the decision of a code is taken in IEEE binary32 (subtract,
 * divide, round-half-even), which is also what the GPU path uses, so that codes
 * can be compared bit for bit.  The dequantised value q*s+z is formed exactly
 * in binary64 (q has 8 bits, s and z are binary16, so the sum is exact), then
 * rounded once to binary32 and once more, half-to-even, to BF16.
 *
 * Build:  gcc -O2 -std=c99 -ffp-contract=off -fPIC -shared
 *             -o liboracle.so ha_rag_oracle.c -lm
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* number formats                                                      */
/* ------------------------------------------------------------------ */

/* BF16 word -> binary32 (exact: BF16 is the upper half of a binary32). */
float orc_bf16_to_f32(uint16_t w)
{
    uint32_t u = (uint32_t)w << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* binary32 -> BF16, round to nearest, ties to even (finite input). */
uint16_t orc_f32_to_bf16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t keep = u >> 16;       /* truncated result          */
    uint32_t rest = u & 0xFFFFu;   /* discarded 16 bits         */
    if (rest > 0x8000u) keep += 1; /* above the midpoint        */
    else if (rest == 0x8000u && (keep & 1u)) keep += 1; /* tie -> even */
    return (uint16_t)keep;
}

/* binary16 word -> binary64 (exact). */
double orc_fp16_to_f64(uint16_t h)
{
    int sign = h >> 15;
    int e = (h >> 10) & 31;
    int m = h & 1023;
    double v;
    if (e == 0) v = ldexp((double)m, -24);             /* subnormal or zero */
    else if (e == 31) v = m ? NAN : INFINITY;
    else v = ldexp((double)(1024 + m), e - 25);        /* 1.m * 2^(e-15)    */
    return sign ? -v : v;
}

/* A value that lies exactly on the finite binary16 grid -> its word.
 * Zero of either sign is encoded as +0. */
static uint16_t fp16_word_of_exact(double v)
{
    double a = fabs(v);
    if (a == 0.0) return 0;
    uint16_t sign = (v < 0.0) ? 0x8000u : 0;
    int ex;
    (void)frexp(a, &ex); /* a in [2^(ex-1), 2^ex) */
    int E = ex - 1;
    if (E < -14) {
        return (uint16_t)(sign | (uint16_t)ldexp(a, 24)); /* subnormal: a / 2^-24 */
    }
    int m = (int)ldexp(a, 10 - E); /* in [1024, 2048) */
    return (uint16_t)(sign | ((E + 15) << 10) | (m - 1024));
}

/* spacing of the binary16 grid around x (x finite, nonzero) */
static double fp16_quantum(double x)
{
    int ex;
    (void)frexp(fabs(x), &ex);
    int E = ex - 1;
    if (E < -14) E = -14;
    return ldexp(1.0, E - 10);
}

/* Largest finite binary16 value <= x.  If none exists (x < -65504) the result
 * is -65504 and *sat is set. */
uint16_t orc_fp16_round_down(float x, int *sat)
{
    double v;
    if (x == 0.0f) v = 0.0;
    else if (x >= 65504.0f) v = 65504.0;
    else if (x < -65504.0f) { v = -65504.0; if (sat) *sat = 1; }
    else {
        double q = fp16_quantum((double)x);
        v = floor((double)x / q) * q; /* exact: q is a power of two */
        if (v < -65504.0) { v = -65504.0; if (sat) *sat = 1; }
    }
    return fp16_word_of_exact(v);
}

/* Smallest finite binary16 value >= x.  If none exists (x > 65504 or x is not
 * finite) the result is 65504 and *sat is set. */
uint16_t orc_fp16_round_up(float x, int *sat)
{
    double v;
    if (x == 0.0f) v = 0.0;
    else if (!(x <= 65504.0f)) { v = 65504.0; if (sat) *sat = 1; }
    else if (x <= -65504.0f) v = -65504.0;
    else {
        double q = fp16_quantum((double)x);
        v = ceil((double)x / q) * q;
        if (v > 65504.0) { v = 65504.0; if (sat) *sat = 1; }
    }
    return fp16_word_of_exact(v);
}

/* ------------------------------------------------------------------ */
/* 8-bit floating point (the paper's schemes S2 = E4M3 and S3 = E5M2,    */
/* Sec. 2.2.2, Fig. 6, Sec. 3.2.1)                                       */
/* ------------------------------------------------------------------ */
/*
 * The paper names the two FP8 variants of its reference [FP8 formats for deep
 * learning] and quotes their ranges (about +-448 and +-57344); it does not say
 * how values are rounded or what happens beyond the range.  Readings:
 *   E4M3: 1 sign, 4 exponent (bias 7), 3 fraction bits, no infinities, the only
 *         NaN is S.1111.111, largest finite 448; subnormals m/8 * 2^-6.
 *   E5M2: 1 sign, 5 exponent (bias 15), 2 fraction bits, IEEE-like infinities
 *         and NaNs, largest finite 57344; subnormals m/4 * 2^-14.
 *   encode: round to nearest, ties to even, on the exact value; anything that
 *         would land beyond the largest finite value saturates to it; the sign
 *         of zero is kept.  Inputs are finite.
 *   decode: exact (every FP8 value is a BF16 value).
 * kind: 43 = E4M3, 52 = E5M2.
 */
static int fp8_params(int kind, int *ebits, int *mbits, int *bias, double *maxv)
{
    if (kind == 43) { *ebits = 4; *mbits = 3; *bias = 7; *maxv = 448.0; return 1; }
    if (kind == 52) { *ebits = 5; *mbits = 2; *bias = 15; *maxv = 57344.0; return 1; }
    return 0;
}

/* FP8 code -> value (NaN codes give NAN, E5M2 infinities give INFINITY). */
double orc_fp8_to_f64(uint8_t c, int kind)
{
    int eb, mb, bias;
    double maxv;
    if (!fp8_params(kind, &eb, &mb, &bias, &maxv)) return NAN;
    int sign = c >> 7;
    int e = (c >> mb) & ((1 << eb) - 1);
    int m = c & ((1 << mb) - 1);
    double v;
    if (kind == 43 && e == 15 && m == 7) v = NAN;
    else if (kind == 52 && e == 31) v = m ? NAN : INFINITY;
    else if (e == 0) v = ldexp((double)m, 1 - bias - mb);
    else v = ldexp((double)((1 << mb) + m), e - bias - mb);
    return sign ? -v : v;
}

/* finite value -> FP8 code: nearest, ties to even, saturating. */
uint8_t orc_f64_to_fp8(double x, int kind)
{
    int eb, mb, bias;
    double maxv;
    if (!fp8_params(kind, &eb, &mb, &bias, &maxv)) return 0;
    uint8_t sign = signbit(x) ? 0x80u : 0;
    double a = fabs(x);
    if (a == 0.0) return sign;
    int ex;
    (void)frexp(a, &ex);
    int E = ex - 1;                       /* a in [2^E, 2^(E+1)) */
    if (E < 1 - bias) E = 1 - bias;       /* subnormal spacing below the smallest normal */
    double q = ldexp(1.0, E - mb);        /* spacing of the FP8 grid around a */
    double n = nearbyint(a / q);          /* exact quotient; default mode = ties to even */
    double v = n * q;
    if (v > maxv) v = maxv;
    /* encode the grid value v */
    if (v == 0.0) return sign;
    (void)frexp(v, &ex);
    E = ex - 1;
    if (E < 1 - bias) return (uint8_t)(sign | (uint8_t)ldexp(v, bias - 1 + mb));
    int m = (int)ldexp(v, mb - E) - (1 << mb);
    return (uint8_t)(sign | ((E + bias) << mb) | m);
}

/* ------------------------------------------------------------------ */
/* GSE-8, the paper's scheme S4 (Sec. 2.2.2, Fig. 7; split 1+4+3 adopted */
/* in Sec. 3.2.1)                                                        */
/* ------------------------------------------------------------------ */
/*
 * One byte: sign, 4-bit index into an array of shared exponents, 3-bit fraction
 * field.  The paper's three conversion steps for a BF16 value x with exponent E:
 * pick the smallest shared exponent G >= E, let d = G - E, shift the fraction
 * right by d + 1 and set bit d + 1 (counted from the most significant end), i.e.
 * the field is the bit string 0^d 1 f1 f2 ... cut to 3 bits; the bits that fall
 * off are discarded (truncation).  Decoding finds the first 1, which gives d and
 * so E = G - d, and shifts the rest back.  Read as numbers, both directions are
 *     field = floor(|x| * 2^(2 - G)),     value = +-field * 2^(G - 2),
 * which is how they are written below.  A field of 0 is the value 0.
 *
 * Shared exponents (Sec. 2.2.2, last paragraph): the exponent range of the unit
 * is cut, from its lower end, into steps of 3 and the right end of every step is
 * a shared exponent, the last one clipped to the top of the range (the worked
 * example: range (-10, 10) gives -7, -4, -1, 2, 5, 8, 10).  Readings taken here:
 * the unit is one tile (one layer, K or V, one head of a chunk); the range is
 * (e_lo - 1, e_hi] with e_lo, e_hi the smallest and largest unbiased exponent of
 * the tile's nonzero values; 16 entries at step 3 reach 48 binades, so e_lo is
 * raised to e_hi - 47 if needed; a value more than 2 binades below the first
 * shared exponent shifts its leading one out of the field and becomes 0; the
 * index stored with a zero field is 0.  The array is not stored: the tile record ends with a
 * 16-byte block {int8 e_lo, int8 e_hi, 14 zero bytes} it is rebuilt from.
 */
#define ORC_GSE_STEP 3
#define ORC_GSE_ENTRIES 16

/* k-th shared exponent of the range (e_lo - 1, e_hi] */
int orc_gse_shared_exponent(int k, int e_lo, int e_hi)
{
    int g = e_lo - 1 + ORC_GSE_STEP * (k + 1);
    return g < e_hi ? g : e_hi;
}

/* unbiased exponent of a finite nonzero BF16 value (subnormals: -126) */
static int bf16_exponent(uint16_t w)
{
    int e = (w >> 7) & 0xFF;
    return e ? e - 127 : -126;
}

/* smallest / largest exponent over the nonzero values; returns 0 if all are zero.
 * e_lo is already raised to e_hi - 47. */
int orc_gse_range(const uint16_t *x, size_t n, int *e_lo, int *e_hi)
{
    int lo = 1000, hi = -1000;
    for (size_t i = 0; i < n; ++i) {
        if ((x[i] & 0x7FFF) == 0) continue;
        int e = bf16_exponent(x[i]);
        if (e < lo) lo = e;
        if (e > hi) hi = e;
    }
    if (hi == -1000) { *e_lo = 0; *e_hi = 0; return 0; }
    if (lo < hi - (ORC_GSE_STEP * ORC_GSE_ENTRIES - 1)) lo = hi - (ORC_GSE_STEP * ORC_GSE_ENTRIES - 1);
    *e_lo = lo;
    *e_hi = hi;
    return 1;
}

uint8_t orc_gse8_encode(uint16_t w, int e_lo, int e_hi)
{
    uint8_t sign = (uint8_t)((w >> 15) << 7);
    if ((w & 0x7FFF) == 0) return sign;
    int E = bf16_exponent(w);
    int k = 0;
    /* smallest shared exponent >= E; the index has 4 bits (Sec. 2.2.2), and a value whose
       exponent lies above e_hi is outside the contract (the range comes from the values
       themselves): it stops at the last index instead of searching for ever */
    while (k < 15 && orc_gse_shared_exponent(k, e_lo, e_hi) < E) ++k;
    int G = orc_gse_shared_exponent(k, e_lo, e_hi);
    double a = fabs((double)orc_bf16_to_f32(w));
    int field = (int)floor(ldexp(a, 2 - G));      /* at most 7 because E <= G */
    if (field == 0) return sign;                  /* E < G - 2: more than 2 places to shift, the
                                                     leading one falls off the field: value 0 */
    return (uint8_t)(sign | (k << 3) | field);
}

double orc_gse8_decode(uint8_t c, int e_lo, int e_hi)
{
    int field = c & 7, k = (c >> 3) & 15;
    double v = ldexp((double)field, orc_gse_shared_exponent(k, e_lo, e_hi) - 2);
    return (c & 0x80) ? -v : v;
}

/* ------------------------------------------------------------------ */
/* one group                                                           */
/* ------------------------------------------------------------------ */

/*
 * Asymmetric min/max quantisation of one group of g values to `bits` bits.
 *   zero  = min of the group, rounded toward -inf to binary16
 *   scale = (max - zero) / (2^bits - 1) in binary32, rounded toward +inf to binary16
 *   code  = clamp(round_half_even((x - zero) / scale), 0, 2^bits - 1), binary32
 * scale == 0 (a constant group whose value is on the binary16 grid): codes 0.
 * Returns 1 if scale or zero had to saturate (values outside the binary16
 * range), else 0.
 */
int orc_quantize_group(const float *x, int g, int bits,
                       uint16_t *scale_h, uint16_t *zero_h, uint8_t *codes)
{
    int sat = 0;
    float mn = x[0], mx = x[0];
    for (int i = 1; i < g; ++i) {
        if (x[i] < mn) mn = x[i];
        if (x[i] > mx) mx = x[i];
    }
    const float qmax = (float)((1 << bits) - 1);
    uint16_t zh = orc_fp16_round_down(mn, &sat);
    float z = (float)orc_fp16_to_f64(zh);
    float range = mx - z;
    float sc = range / qmax;
    uint16_t sh = orc_fp16_round_up(sc, &sat);
    float s = (float)orc_fp16_to_f64(sh);
    for (int i = 0; i < g; ++i) {
        float r = 0.0f;
        if (s != 0.0f) {
            float d = x[i] - z;
            float t = d / s;
            r = nearbyintf(t); /* default rounding mode: ties to even */
            if (r < 0.0f) r = 0.0f;
            if (r > qmax) r = qmax;
        }
        codes[i] = (uint8_t)r;
    }
    *scale_h = sh;
    *zero_h = zh;
    return sat;
}

/* Dequantised value before the BF16 rounding: the binary32 nearest to
 * code*scale + zero (one rounding; the sum is exact in binary64). */
float orc_dequant_f32(unsigned code, uint16_t scale_h, uint16_t zero_h)
{
    double exact = (double)code * orc_fp16_to_f64(scale_h) + orc_fp16_to_f64(zero_h);
    return (float)exact;
}

uint16_t orc_dequant_bf16(unsigned code, uint16_t scale_h, uint16_t zero_h)
{
    return orc_f32_to_bf16_rne(orc_dequant_f32(code, scale_h, zero_h));
}

/* ------------------------------------------------------------------ */
/* packed chunk layout                                                 */
/* ------------------------------------------------------------------ */
/*
 * A chunk holds K and V of one document: n_tiles = L*2*H tiles, tile index
 * (l*2 + kv)*H + h, each tile T*D elements in [token][head_dim] order
 * (element index e = t*D + d).  A tile is cut into blocks of 2048 elements;
 * the last block is padded with zero bytes.  Inside a block, element r is
 *   plane j = r / 512, lane i = (r % 512) / 8, position p = r % 8,
 * and the 8 elements sharing (j, i) form an octet of `bits` bytes.  With
 * P = 16/bits octets per 16-byte word, octet (j, i) starts at byte
 *   (j / P) * 1024 + i * 16 + (j % P) * bits
 * of the block's payload (256*bits bytes).  Inside the octet: 16-bit elements
 * are little-endian words in order; 8-bit codes one per byte; 4-bit codes two
 * per byte, even position in the low nibble.
 * The tile record is all payload blocks followed by all meta blocks.  A meta
 * block holds 2048/g entries of 4 bytes {u16 scale, u16 zero} (little endian);
 * the group with index G = r / g inside its block is entry
 *   (G % (512/g)) * 4 + G / (512/g).
 */
#define ORC_BLOCK 2048

/* `bits` names the storage format: 16 (BF16 verbatim), 8 / 4 (integer codes with
 * per-group scale and zero), 43 / 52 (FP8 E4M3 / E5M2, one byte per element, no
 * meta; the payload is laid out like the 8-bit integer payload). */
static int is_fp8(int bits) { return bits == 43 || bits == 52; }
static int is_gse(int bits) { return bits == 143; }  /* GSE-8 with the 1+4+3 split */
static int storage_bits(int bits) { return (is_fp8(bits) || is_gse(bits)) ? 8 : bits; }

static int valid_shape(int D, int bits, int g)
{
    if (bits != 16 && bits != 8 && bits != 4 && !is_fp8(bits) && !is_gse(bits)) return 0;
    if (D <= 0 || D % 8) return 0;
    if (bits == 16 || is_fp8(bits) || is_gse(bits)) return 1;
    if (g != 32 && g != 64 && g != 128 && g != 256 && g != 512) return 0;
    return D % g == 0;
}

size_t orc_tile_blocks(int T, int D)
{
    return ((size_t)T * D + ORC_BLOCK - 1) / ORC_BLOCK;
}

size_t orc_tile_payload_bytes(int T, int D, int bits)
{
    return orc_tile_blocks(T, D) * 256u * (size_t)storage_bits(bits);
}

size_t orc_tile_meta_bytes(int T, int D, int bits, int g)
{
    if (bits == 16 || is_fp8(bits)) return 0;
    if (is_gse(bits)) return T > 0 ? 16 : 0;
    return orc_tile_blocks(T, D) * (size_t)(ORC_BLOCK / g) * 4u;
}

size_t orc_chunk_bytes(int L, int H, int D, int T, int bits, int g)
{
    if (!valid_shape(D, bits, g) || T < 0) return 0;
    return (size_t)L * 2 * H *
           (orc_tile_payload_bytes(T, D, bits) + orc_tile_meta_bytes(T, D, bits, g));
}

/* byte offset, inside the tile's payload, of the octet holding element e */
static size_t octet_offset(size_t e, int bits)
{
    size_t k = e / ORC_BLOCK, r = e % ORC_BLOCK;
    size_t j = r / 512, i = (r % 512) / 8;
    size_t P = 16 / (size_t)bits;
    return k * 256u * (size_t)bits + (j / P) * 1024u + i * 16u + (j % P) * (size_t)bits;
}

/* byte offset, inside the tile's meta area, of the entry of element e's group */
static size_t meta_offset(size_t e, int g)
{
    size_t k = e / ORC_BLOCK, r = e % ORC_BLOCK;
    size_t G = r / (size_t)g;
    size_t per_plane = 512u / (size_t)g;
    size_t entry = (G % per_plane) * 4u + G / per_plane;
    return k * (size_t)(ORC_BLOCK / g) * 4u + entry * 4u;
}

/* exported for the layout pins */
size_t orc_octet_offset(size_t e, int bits) { return octet_offset(e, bits); }
size_t orc_meta_offset(size_t e, int g) { return meta_offset(e, g); }

static void put_code(uint8_t *payload, size_t e, int bits, unsigned q)
{
    uint8_t *o = payload + octet_offset(e, bits);
    unsigned p = (unsigned)(e % 8);
    if (bits == 8) o[p] = (uint8_t)q;
    else {
        uint8_t *b = o + p / 2;
        if (p & 1) *b = (uint8_t)((*b & 0x0Fu) | (q << 4));
        else *b = (uint8_t)((*b & 0xF0u) | (q & 0x0Fu));
    }
}

static unsigned get_code(const uint8_t *payload, size_t e, int bits)
{
    const uint8_t *o = payload + octet_offset(e, bits);
    unsigned p = (unsigned)(e % 8);
    if (bits == 8) return o[p];
    return (p & 1) ? (unsigned)(o[p / 2] >> 4) : (unsigned)(o[p / 2] & 0x0Fu);
}

/* n_tiles tiles of [T][D] BF16 words -> n_tiles tile records, back to back */
static long pack_tiles(const uint16_t *src, size_t n_tiles, int D, int T,
                       int bits, int g, uint8_t *dst)
{
    if (!valid_shape(D, bits, g) || T < 0) return -1;
    const size_t n_e = (size_t)T * D;
    const size_t pay = orc_tile_payload_bytes(T, D, bits);
    const size_t met = orc_tile_meta_bytes(T, D, bits, g);
    long saturated = 0;
    memset(dst, 0, n_tiles * (pay + met));
    for (size_t tile = 0; tile < n_tiles; ++tile) {
        const uint16_t *x = src + tile * n_e;
        uint8_t *payload = dst + tile * (pay + met);
        uint8_t *meta = payload + pay;
        if (bits == 16) {
            for (size_t e = 0; e < n_e; ++e) {
                uint8_t *o = payload + octet_offset(e, 16) + 2 * (e % 8);
                o[0] = (uint8_t)(x[e] & 0xFF);
                o[1] = (uint8_t)(x[e] >> 8);
            }
            continue;
        }
        if (is_fp8(bits)) {
            for (size_t e = 0; e < n_e; ++e)
                payload[octet_offset(e, 8) + e % 8] =
                    orc_f64_to_fp8((double)orc_bf16_to_f32(x[e]), bits);
            continue;
        }
        if (is_gse(bits)) {
            int e_lo, e_hi;
            (void)orc_gse_range(x, n_e, &e_lo, &e_hi);
            for (size_t e = 0; e < n_e; ++e)
                payload[octet_offset(e, 8) + e % 8] = orc_gse8_encode(x[e], e_lo, e_hi);
            meta[0] = (uint8_t)(int8_t)e_lo;
            meta[1] = (uint8_t)(int8_t)e_hi;
            continue;
        }
        float xs[512];
        uint8_t codes[512];
        for (size_t e0 = 0; e0 < n_e; e0 += (size_t)g) {
            uint16_t sh, zh;
            for (int i = 0; i < g; ++i) xs[i] = orc_bf16_to_f32(x[e0 + i]);
            saturated += orc_quantize_group(xs, g, bits, &sh, &zh, codes);
            for (int i = 0; i < g; ++i) put_code(payload, e0 + i, bits, codes[i]);
            uint8_t *m = meta + meta_offset(e0, g);
            m[0] = (uint8_t)(sh & 0xFF); m[1] = (uint8_t)(sh >> 8);
            m[2] = (uint8_t)(zh & 0xFF); m[3] = (uint8_t)(zh >> 8);
        }
    }
    return saturated;
}

/*
 * Quantise and pack one chunk (Algorithm 1 step 3 for one chunk).
 *   src   BF16 words, [L][2][H][T][D] contiguous
 *   dst   orc_chunk_bytes() bytes, fully written (padding included)
 * Returns <0 on a bad shape, else the number of groups that saturated.
 */
long orc_quantize_pack_chunk(const uint16_t *src, int L, int H, int D, int T,
                             int bits, int g, uint8_t *dst)
{
    return pack_tiles(src, (size_t)L * 2 * H, D, T, bits, g, dst);
}

/*
 * The same for a chunk that holds only the keys or only the values of a
 * document: Algorithm 1 takes the n key chunks and the n value chunks as 2n
 * units, each with its own access frequency and so its own precision.
 *   src   BF16 words, [L][H][T][D] contiguous (one half of the document's KV)
 *   dst   orc_half_bytes() bytes: the tile records (l, h) in that order
 */
long orc_quantize_pack_half(const uint16_t *src, int L, int H, int D, int T,
                            int bits, int g, uint8_t *dst)
{
    return pack_tiles(src, (size_t)L * H, D, T, bits, g, dst);
}

size_t orc_half_bytes(int L, int H, int D, int T, int bits, int g)
{
    if (!valid_shape(D, bits, g) || T < 0) return 0;
    return (size_t)L * H *
           (orc_tile_payload_bytes(T, D, bits) + orc_tile_meta_bytes(T, D, bits, g));
}

/*
 * Dequantise one packed chunk and scatter it into the request's KV cache
 * (the "load + decompress + concatenate" step of Sec. 2.1).
 *   out      BF16 words, [L][2][H][cap_tokens][D]
 *   tok_off  first token row this chunk occupies in every tile of `out`
 * Returns 0, or -1 on a bad shape / not enough room.
 */
/* kv < 0: the chunk holds keys and values; kv = 0 / 1: only the keys / only the values */
static int scatter_tiles(const uint8_t *packed, int L, int H, int D, int T,
                         int bits, int g, int kv,
                         uint16_t *out, size_t cap_tokens, size_t tok_off)
{
    if (!valid_shape(D, bits, g) || T < 0) return -1;
    if (tok_off + (size_t)T > cap_tokens) return -1;
    const size_t n_tiles = (size_t)L * (kv < 0 ? 2 : 1) * H;
    const size_t n_e = (size_t)T * D;
    const size_t pay = orc_tile_payload_bytes(T, D, bits);
    const size_t met = orc_tile_meta_bytes(T, D, bits, g);
    for (size_t tile = 0; tile < n_tiles; ++tile) {
        const uint8_t *payload = packed + tile * (pay + met);
        const uint8_t *meta = payload + pay;
        /* tile of the cache [L][2][H]: a half chunk's tile (l, h) lands in plane kv */
        const size_t out_tile = kv < 0 ? tile
            : ((tile / (size_t)H) * 2 + (size_t)kv) * (size_t)H + tile % (size_t)H;
        uint16_t *y = out + (out_tile * cap_tokens + tok_off) * (size_t)D;
        for (size_t e = 0; e < n_e; ++e) {
            if (bits == 16) {
                const uint8_t *o = payload + octet_offset(e, 16) + 2 * (e % 8);
                y[e] = (uint16_t)(o[0] | (o[1] << 8));
            } else if (is_fp8(bits)) {
                uint8_t c = payload[octet_offset(e, 8) + e % 8];
                y[e] = orc_f32_to_bf16_rne((float)orc_fp8_to_f64(c, bits)); /* exact */
            } else if (is_gse(bits)) {
                uint8_t c = payload[octet_offset(e, 8) + e % 8];
                double v = orc_gse8_decode(c, (int8_t)meta[0], (int8_t)meta[1]);
                y[e] = orc_f32_to_bf16_rne((float)v);                        /* exact */
            } else {
                const uint8_t *m = meta + meta_offset(e, g);
                uint16_t sh = (uint16_t)(m[0] | (m[1] << 8));
                uint16_t zh = (uint16_t)(m[2] | (m[3] << 8));
                y[e] = orc_dequant_bf16(get_code(payload, e, bits), sh, zh);
            }
        }
    }
    return 0;
}

int orc_dequant_scatter_chunk(const uint8_t *packed, int L, int H, int D, int T,
                              int bits, int g,
                              uint16_t *out, size_t cap_tokens, size_t tok_off)
{
    return scatter_tiles(packed, L, H, D, T, bits, g, -1, out, cap_tokens, tok_off);
}

/* A keys-only (kv = 0) or values-only (kv = 1) chunk into its plane of the cache. */
int orc_dequant_scatter_half(const uint8_t *packed, int L, int H, int D, int T,
                             int bits, int g, int kv,
                             uint16_t *out, size_t cap_tokens, size_t tok_off)
{
    if (kv != 0 && kv != 1) return -1;
    return scatter_tiles(packed, L, H, D, T, bits, g, kv, out, cap_tokens, tok_off);
}

/*
 * Unpack a chunk into canonical arrays (element order [tile][t][d]) without
 * any arithmetic: codes (or the 16-bit words, in codes16), scale and zero
 * words per group.  Used by the tests to compare packing field by field.
 */
int orc_unpack_chunk(const uint8_t *packed, int L, int H, int D, int T, int bits, int g,
                     uint8_t *codes, uint16_t *codes16, uint16_t *scale_h, uint16_t *zero_h)
{
    if (!valid_shape(D, bits, g) || T < 0) return -1;
    const size_t n_tiles = (size_t)L * 2 * H;
    const size_t n_e = (size_t)T * D;
    const size_t pay = orc_tile_payload_bytes(T, D, bits);
    const size_t met = orc_tile_meta_bytes(T, D, bits, g);
    for (size_t tile = 0; tile < n_tiles; ++tile) {
        const uint8_t *payload = packed + tile * (pay + met);
        const uint8_t *meta = payload + pay;
        for (size_t e = 0; e < n_e; ++e) {
            if (bits == 16) {
                const uint8_t *o = payload + octet_offset(e, 16) + 2 * (e % 8);
                codes16[tile * n_e + e] = (uint16_t)(o[0] | (o[1] << 8));
            } else if (is_fp8(bits) || is_gse(bits)) {
                codes[tile * n_e + e] = payload[octet_offset(e, 8) + e % 8];
            } else {
                codes[tile * n_e + e] = (uint8_t)get_code(payload, e, bits);
                if (e % (size_t)g == 0) {
                    const uint8_t *m = meta + meta_offset(e, g);
                    size_t G = (tile * n_e + e) / (size_t)g;
                    scale_h[G] = (uint16_t)(m[0] | (m[1] << 8));
                    zero_h[G] = (uint16_t)(m[2] | (m[3] << 8));
                }
            }
        }
    }
    return 0;
}

/* Root mean square error between two BF16 arrays (Eq. 1), in binary64. */
double orc_rmse_bf16(const uint16_t *a, const uint16_t *b, size_t n)
{
    double acc = 0.0;
    for (size_t i = 0; i < n; ++i) {
        double d = (double)orc_bf16_to_f32(a[i]) - (double)orc_bf16_to_f32(b[i]);
        acc += d * d;
    }
    return n ? sqrt(acc / (double)n) : 0.0;
}
