// Device-side decoders of the packed chunk formats: one octet (8 codes of one plane of a
// layout block) -> 8 BF16 values in one 16-byte word.  Shared by every kernel that reads
// packed chunks; the values are the ones a load writes into the cache:
// bf16_rne(fma(code, scale, zero)) for the integer formats, exact for FP8 and GSE-8.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ha_rag {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ u32x4 ld16(const uint8_t *p)
{
    return *reinterpret_cast<const u32x4 *>(p);
}

template <bool NT>
__device__ __forceinline__ void st16(uint8_t *p, u32x4 v)
{
    if (NT) __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(p));
    else *reinterpret_cast<u32x4 *>(p) = v;
}

__device__ __forceinline__ float h2f(uint32_t h16)
{
    return (float)__builtin_bit_cast(_Float16, (uint16_t)h16);
}

// two fp32 -> one dword of two BF16 (round to nearest even), a in the low half
__device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    f32x2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

__device__ __forceinline__ float byte_f(uint32_t w, int k)
{
    return (float)((w >> (8 * k)) & 0xFFu);  // one byte-to-float conversion each
}

// 8 int4 codes (one dword) of one plane -> 8 BF16 (16 bytes)
__device__ __forceinline__ u32x4 dequant_octet4(uint32_t c, uint32_t m)
{
    const float s = h2f(m & 0xFFFFu), z = h2f(m >> 16);
    const uint32_t ev = c & 0x0F0F0F0Fu;         // codes 0,2,4,6 one per byte
    const uint32_t od = (c >> 4) & 0x0F0F0F0Fu;  // codes 1,3,5,7
    u32x4 r;
    r.x = pack_bf16(__builtin_fmaf(byte_f(ev, 0), s, z), __builtin_fmaf(byte_f(od, 0), s, z));
    r.y = pack_bf16(__builtin_fmaf(byte_f(ev, 1), s, z), __builtin_fmaf(byte_f(od, 1), s, z));
    r.z = pack_bf16(__builtin_fmaf(byte_f(ev, 2), s, z), __builtin_fmaf(byte_f(od, 2), s, z));
    r.w = pack_bf16(__builtin_fmaf(byte_f(ev, 3), s, z), __builtin_fmaf(byte_f(od, 3), s, z));
    return r;
}

// 8 int8 codes (two dwords) of one plane -> 8 BF16
__device__ __forceinline__ u32x4 dequant_octet8(uint32_t c0, uint32_t c1, uint32_t m)
{
    const float s = h2f(m & 0xFFFFu), z = h2f(m >> 16);
    u32x4 r;
    r.x = pack_bf16(__builtin_fmaf(byte_f(c0, 0), s, z), __builtin_fmaf(byte_f(c0, 1), s, z));
    r.y = pack_bf16(__builtin_fmaf(byte_f(c0, 2), s, z), __builtin_fmaf(byte_f(c0, 3), s, z));
    r.z = pack_bf16(__builtin_fmaf(byte_f(c1, 0), s, z), __builtin_fmaf(byte_f(c1, 1), s, z));
    r.w = pack_bf16(__builtin_fmaf(byte_f(c1, 2), s, z), __builtin_fmaf(byte_f(c1, 3), s, z));
    return r;
}

// 8 FP8 codes (two dwords) of one plane -> 8 BF16.  The hardware conversion to fp32 is
// exact and every FP8 value is a BF16 value, so no rounding conversion is needed.
template <bool E5M2>
__device__ __forceinline__ u32x4 decode_octet_fp8(uint32_t c0, uint32_t c1)
{
    f32x2 a, b, c, d;
    if (E5M2) {
        a = __builtin_amdgcn_cvt_pk_f32_bf8(c0, false);
        b = __builtin_amdgcn_cvt_pk_f32_bf8(c0, true);
        c = __builtin_amdgcn_cvt_pk_f32_bf8(c1, false);
        d = __builtin_amdgcn_cvt_pk_f32_bf8(c1, true);
    } else {
        a = __builtin_amdgcn_cvt_pk_f32_fp8(c0, false);
        b = __builtin_amdgcn_cvt_pk_f32_fp8(c0, true);
        c = __builtin_amdgcn_cvt_pk_f32_fp8(c1, false);
        d = __builtin_amdgcn_cvt_pk_f32_fp8(c1, true);
    }
    // the upper halves of the binary32 results are the BF16 values: a byte permute per pair
    // (the elements are copied to scalars first: a bit cast of a vector element reads element 0)
    auto upper = [](f32x2 v) {
        const float lo = v.x, hi = v.y;
        return __builtin_amdgcn_perm(__builtin_bit_cast(uint32_t, hi), __builtin_bit_cast(uint32_t, lo), 0x07060302u);
    };
    u32x4 r;
    r.x = upper(a);
    r.y = upper(b);
    r.z = upper(c);
    r.w = upper(d);
    return r;
}

// 8 GSE-8 codes (two dwords) of one plane -> 8 BF16.  base = e_lo + 2 - 2 and top = e_hi - 2
// are the tile's exponent bounds already lowered by the 2 fraction places of the field:
// value = +-field * 2^min(base + 3k, top), exact in BF16.
__device__ __forceinline__ float decode_gse8(uint32_t w, uint32_t fields, int b, int base, int top)
{
    int n = (int)((w >> (8 * b + 3)) & 15u) * 3 + base;
    n = n < top ? n : top;
    return __builtin_ldexpf(byte_f(fields, b), n);
}

// two codes (bytes b, b+1 of w) -> one dword of two BF16; the sign bits are moved from bit 7
// of each code to bit 15 of each half by one byte permute
template <int B>
__device__ __forceinline__ uint32_t decode_pair_gse8(uint32_t w, uint32_t fields, int base, int top)
{
    // field * 2^n has three significant bits: the upper halves of the two binary32 results are
    // the BF16 values, no rounding conversion needed
    const uint32_t mag = __builtin_amdgcn_perm(__builtin_bit_cast(uint32_t, decode_gse8(w, fields, B + 1, base, top)),
                                               __builtin_bit_cast(uint32_t, decode_gse8(w, fields, B, base, top)),
                                               0x07060302u);
    constexpr uint32_t sel = 0x0Cu | (uint32_t(B) << 8) | (0x0Cu << 16) | (uint32_t(B + 1) << 24);
    return mag | (__builtin_amdgcn_perm(0u, w, sel) & 0x80008000u);
}

__device__ __forceinline__ u32x4 decode_octet_gse8(uint32_t c0, uint32_t c1, int base, int top)
{
    const uint32_t f0 = c0 & 0x07070707u, f1 = c1 & 0x07070707u;
    u32x4 r;
    r.x = decode_pair_gse8<0>(c0, f0, base, top);
    r.y = decode_pair_gse8<2>(c0, f0, base, top);
    r.z = decode_pair_gse8<0>(c1, f1, base, top);
    r.w = decode_pair_gse8<2>(c1, f1, base, top);
    return r;
}

}  // namespace ha_rag
