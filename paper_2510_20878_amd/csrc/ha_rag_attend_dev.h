// Device-side pieces shared by the attention kernels over packed chunks: the per-format block
// geometry, the decoders that give the BF16 values a load would write, and small helpers.
#pragma once
#include "ha_rag_kernels.h"
#include "ha_rag_decode.h"

namespace ha_rag {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <uint32_t PREC>
struct Fmt {
    static constexpr uint32_t kWords = PREC == kInt4 ? 1u : PREC == kP16 ? 4u : 2u;  // 16-byte words per lane and block
    static constexpr uint32_t kPayload = 1024u * kWords;
    static constexpr bool kMeta = PREC == kInt4 || PREC == kInt8;
};

// byte K of a dword -> float in one instruction.  Written as asm because the compiler
// otherwise folds the nibble mask into a bit-field extract per code and then converts byte 0
// (two instructions per code instead of one).
template <int K>
__device__ __forceinline__ float ubyte_f(uint32_t w)
{
    float r;
    if (K == 0) asm("v_cvt_f32_ubyte0 %0, %1" : "=v"(r) : "v"(w));
    else if (K == 1) asm("v_cvt_f32_ubyte1 %0, %1" : "=v"(r) : "v"(w));
    else if (K == 2) asm("v_cvt_f32_ubyte2 %0, %1" : "=v"(r) : "v"(w));
    else asm("v_cvt_f32_ubyte3 %0, %1" : "=v"(r) : "v"(w));
    return r;
}

// the same values as dequant_octet4 / dequant_octet8: bf16_rne(fma(code, scale, zero))
__device__ __forceinline__ u32x4 attend_octet4(uint32_t c, uint32_t m)
{
    const float s = h2f(m & 0xFFFFu), z = h2f(m >> 16);
    const uint32_t ev = c & 0x0F0F0F0Fu, od = (c >> 4) & 0x0F0F0F0Fu;
    u32x4 r;
    r.x = pack_bf16(__builtin_fmaf(ubyte_f<0>(ev), s, z), __builtin_fmaf(ubyte_f<0>(od), s, z));
    r.y = pack_bf16(__builtin_fmaf(ubyte_f<1>(ev), s, z), __builtin_fmaf(ubyte_f<1>(od), s, z));
    r.z = pack_bf16(__builtin_fmaf(ubyte_f<2>(ev), s, z), __builtin_fmaf(ubyte_f<2>(od), s, z));
    r.w = pack_bf16(__builtin_fmaf(ubyte_f<3>(ev), s, z), __builtin_fmaf(ubyte_f<3>(od), s, z));
    return r;
}

__device__ __forceinline__ u32x4 attend_octet8(uint32_t c0, uint32_t c1, uint32_t m)
{
    const float s = h2f(m & 0xFFFFu), z = h2f(m >> 16);
    u32x4 r;
    r.x = pack_bf16(__builtin_fmaf(ubyte_f<0>(c0), s, z), __builtin_fmaf(ubyte_f<1>(c0), s, z));
    r.y = pack_bf16(__builtin_fmaf(ubyte_f<2>(c0), s, z), __builtin_fmaf(ubyte_f<3>(c0), s, z));
    r.z = pack_bf16(__builtin_fmaf(ubyte_f<0>(c1), s, z), __builtin_fmaf(ubyte_f<1>(c1), s, z));
    r.w = pack_bf16(__builtin_fmaf(ubyte_f<2>(c1), s, z), __builtin_fmaf(ubyte_f<3>(c1), s, z));
    return r;
}

// the raw codes of one octet (x: int4; x, y: 8-bit formats; all four: 16-bit) -> 8 BF16
template <uint32_t PREC>
__device__ __forceinline__ u32x4 decode_octet(u32x4 raw, uint32_t meta, int base, int top)
{
    if (PREC == kInt4) return attend_octet4(raw.x, meta);
    if (PREC == kInt8) return attend_octet8(raw.x, raw.y, meta);
    if (PREC == kE4M3) return decode_octet_fp8<false>(raw.x, raw.y);
    if (PREC == kE5M2) return decode_octet_fp8<true>(raw.x, raw.y);
    if (PREC == kGSE8) return decode_octet_gse8(raw.x, raw.y, base, top);
    return raw;
}

// plane j of the words a lane loaded from a payload block
template <uint32_t PREC>
__device__ __forceinline__ u32x4 plane_raw(const u32x4 *w, int j)
{
    u32x4 r = {0u, 0u, 0u, 0u};
    if (PREC == kInt4) r.x = w[0][j];
    else if (PREC == kP16) r = w[j];
    else {
        r.x = w[j >> 1][(j & 1) * 2];
        r.y = w[j >> 1][(j & 1) * 2 + 1];
    }
    return r;
}

// The first instruction that reads an MFMA result has to come a fixed number of cycles after
// the MFMA (11 for the 8-pass 16x16x32).  The compiler inserts that wait where both are in one
// basic block; with a branch between them it was found to leave the wait out, and the reader
// then sees what the registers held before.  Called right after a chain whose result is first
// read behind a branch: nothing is scheduled across it, and it idles for 12 cycles.
__device__ __forceinline__ void mfma_result_wait()
{
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_nop 7\n\ts_nop 3");
    __builtin_amdgcn_sched_barrier(0);
}

// how far a score may exceed a row's running maximum before that maximum is brought up to
// date, in units of log2: weights stay below 2^8
constexpr float kLazyMaxSlack = 8.0f;

__device__ __forceinline__ float neg_inf() { return -__builtin_huge_valf(); }

// orders the LDS accesses of one wave: what its lanes wrote before is visible to all its
// lanes after.  The hardware executes the LDS instructions of a wave in issue order, so
// nothing has to be waited for; the fences keep the compiler from moving accesses across
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// the launch-wide scalars a workgroup needs, read from the argument buffer once
struct AttendHdr {
    uint32_t n_kv_heads, n_q_heads, layer;
    float scale_log2;
};

// keeps a value in a scalar register from here on: everything pinned at the top of the kernel
// is fetched from the argument buffer by loads issued together, not one by one where the
// values are first used
__device__ __forceinline__ void pin(uint32_t &v) { asm volatile("" : "+s"(v)); }
__device__ __forceinline__ void pin(float &v) { asm volatile("" : "+s"(v)); }
template <class T>
__device__ __forceinline__ void pin(T *&v)
{
    uint64_t a = reinterpret_cast<uint64_t>(v);
    asm volatile("" : "+s"(a));
    v = reinterpret_cast<T *>(a);
}

// Everything the attention kernels read or write outside LDS lies in global memory; saying so lets the
// loads run as global instructions (scalar base, 32-bit lane offset), which do not count
// against the LDS counter the way loads through generic pointers do.
typedef const uint8_t __attribute__((address_space(1))) *gbytes;
typedef float __attribute__((address_space(1))) *gfloats;

__device__ __forceinline__ u32x4 ldg16(gbytes p)
{
    return *(const u32x4 __attribute__((address_space(1))) *)p;
}

// max of a value over the four lanes l, l ^ 16, l ^ 32, l ^ 48 (one per lane group), in every
// lane.  The row swaps exchange registers between lane rows without a trip through LDS: after
// swapping the odd rows of one copy with the even rows of another, the two copies hold the
// value of rows r and r ^ 1 side by side; the same with halves of 32 lanes.
__device__ __forceinline__ float max_over_lane_groups(float x)
{
    typedef unsigned u2 __attribute__((ext_vector_type(2)));
    const unsigned xi = __builtin_bit_cast(unsigned, x);
    const u2 r = __builtin_amdgcn_permlane16_swap(xi, xi, false, false);
    const unsigned r0 = r.x, r1 = r.y;  // copied out first: a bit cast of a vector element reads element 0
    const float y = __builtin_fmaxf(__builtin_bit_cast(float, r0), __builtin_bit_cast(float, r1));
    const unsigned yi = __builtin_bit_cast(unsigned, y);
    const u2 t = __builtin_amdgcn_permlane32_swap(yi, yi, false, false);
    const unsigned t0 = t.x, t1 = t.y;
    return __builtin_fmaxf(__builtin_bit_cast(float, t0), __builtin_bit_cast(float, t1));
}

}  // namespace ha_rag
