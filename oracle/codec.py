"""ctypes view of the C oracle (ha_rag_oracle.c) plus thin numpy conveniences.

Every array is a numpy array on the host.  BF16 and binary16 values travel as
uint16 words.  Shapes follow the packed-chunk layout described at the top of
ha_rag_oracle.c.  Precision tags: bits 16 (BF16 words kept verbatim), 8, 4 (integer codes), 43 and 52
(FP8 E4M3 / E5M2), 143 (GSE-8 with the 1+4+3 split).
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None
_native = False


def select_library(native):
    """Which build of the oracle the calls below use: the -O2 one of the tests (default), or the
    -O3 -march=native one for the benchmark's timed CPU leg (compiled here, on the machine that
    times it).  The source is the same."""
    global _lib, _native
    if bool(native) != _native:
        _native = bool(native)
        _lib = None


def lib():
    global _lib
    if _lib is None:
        if _native:
            path = _build.build_native(force=False)
        else:
            path = _build.LIB
            if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
                _build.build()
        L = C.CDLL(path)
        u8p, u16p, f32p = C.POINTER(C.c_uint8), C.POINTER(C.c_uint16), C.POINTER(C.c_float)
        L.orc_bf16_to_f32.restype = C.c_float
        L.orc_bf16_to_f32.argtypes = [C.c_uint16]
        L.orc_f32_to_bf16_rne.restype = C.c_uint16
        L.orc_f32_to_bf16_rne.argtypes = [C.c_float]
        L.orc_fp16_to_f64.restype = C.c_double
        L.orc_fp16_to_f64.argtypes = [C.c_uint16]
        L.orc_fp16_round_down.restype = C.c_uint16
        L.orc_fp16_round_down.argtypes = [C.c_float, C.POINTER(C.c_int)]
        L.orc_fp16_round_up.restype = C.c_uint16
        L.orc_fp16_round_up.argtypes = [C.c_float, C.POINTER(C.c_int)]
        L.orc_fp8_to_f64.restype = C.c_double
        L.orc_fp8_to_f64.argtypes = [C.c_uint8, C.c_int]
        L.orc_f64_to_fp8.restype = C.c_uint8
        L.orc_f64_to_fp8.argtypes = [C.c_double, C.c_int]
        L.orc_gse_shared_exponent.restype = C.c_int
        L.orc_gse_shared_exponent.argtypes = [C.c_int, C.c_int, C.c_int]
        L.orc_gse_range.restype = C.c_int
        L.orc_gse_range.argtypes = [u16p, C.c_size_t, C.POINTER(C.c_int), C.POINTER(C.c_int)]
        L.orc_gse8_encode.restype = C.c_uint8
        L.orc_gse8_encode.argtypes = [C.c_uint16, C.c_int, C.c_int]
        L.orc_gse8_decode.restype = C.c_double
        L.orc_gse8_decode.argtypes = [C.c_uint8, C.c_int, C.c_int]
        L.orc_quantize_group.restype = C.c_int
        L.orc_quantize_group.argtypes = [f32p, C.c_int, C.c_int, u16p, u16p, u8p]
        L.orc_dequant_f32.restype = C.c_float
        L.orc_dequant_f32.argtypes = [C.c_uint, C.c_uint16, C.c_uint16]
        L.orc_dequant_bf16.restype = C.c_uint16
        L.orc_dequant_bf16.argtypes = [C.c_uint, C.c_uint16, C.c_uint16]
        for name in ("orc_tile_blocks",):
            getattr(L, name).restype = C.c_size_t
            getattr(L, name).argtypes = [C.c_int, C.c_int]
        L.orc_tile_payload_bytes.restype = C.c_size_t
        L.orc_tile_payload_bytes.argtypes = [C.c_int, C.c_int, C.c_int]
        L.orc_tile_meta_bytes.restype = C.c_size_t
        L.orc_tile_meta_bytes.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int]
        L.orc_chunk_bytes.restype = C.c_size_t
        L.orc_chunk_bytes.argtypes = [C.c_int] * 6
        L.orc_octet_offset.restype = C.c_size_t
        L.orc_octet_offset.argtypes = [C.c_size_t, C.c_int]
        L.orc_meta_offset.restype = C.c_size_t
        L.orc_meta_offset.argtypes = [C.c_size_t, C.c_int]
        L.orc_quantize_pack_chunk.restype = C.c_long
        L.orc_quantize_pack_chunk.argtypes = [u16p] + [C.c_int] * 6 + [u8p]
        L.orc_dequant_scatter_chunk.restype = C.c_int
        L.orc_dequant_scatter_chunk.argtypes = [u8p] + [C.c_int] * 6 + [u16p, C.c_size_t, C.c_size_t]
        L.orc_quantize_pack_half.restype = C.c_long
        L.orc_quantize_pack_half.argtypes = [u16p] + [C.c_int] * 6 + [u8p]
        L.orc_half_bytes.restype = C.c_size_t
        L.orc_half_bytes.argtypes = [C.c_int] * 6
        L.orc_dequant_scatter_half.restype = C.c_int
        L.orc_dequant_scatter_half.argtypes = [u8p] + [C.c_int] * 7 + [u16p, C.c_size_t, C.c_size_t]
        L.orc_unpack_chunk.restype = C.c_int
        L.orc_unpack_chunk.argtypes = [u8p] + [C.c_int] * 6 + [u8p, u16p, u16p, u16p]
        L.orc_rmse_bf16.restype = C.c_double
        L.orc_rmse_bf16.argtypes = [u16p, u16p, C.c_size_t]
        _lib = L
    return _lib


def _p(a, ctype):
    return a.ctypes.data_as(C.POINTER(ctype))


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


# ---- scalars ---------------------------------------------------------------
def bf16_to_f32(w):
    return lib().orc_bf16_to_f32(int(w))


def f32_to_bf16_rne(f):
    return lib().orc_f32_to_bf16_rne(float(np.float32(f)))


def fp16_to_f64(h):
    return lib().orc_fp16_to_f64(int(h))


def fp16_round_down(x):
    sat = C.c_int(0)
    return lib().orc_fp16_round_down(float(np.float32(x)), C.byref(sat)), bool(sat.value)


def fp16_round_up(x):
    sat = C.c_int(0)
    return lib().orc_fp16_round_up(float(np.float32(x)), C.byref(sat)), bool(sat.value)


def dequant_f32(code, scale_h, zero_h):
    return lib().orc_dequant_f32(int(code), int(scale_h), int(zero_h))


def dequant_bf16(code, scale_h, zero_h):
    return lib().orc_dequant_bf16(int(code), int(scale_h), int(zero_h))


def fp8_to_f64(code, kind):
    """kind: 43 = E4M3, 52 = E5M2."""
    return lib().orc_fp8_to_f64(int(code), kind)


def f64_to_fp8(x, kind):
    return lib().orc_f64_to_fp8(float(x), kind)


def gse_shared_exponents(e_lo, e_hi, n=16):
    """The shared-exponent array of the range (e_lo - 1, e_hi]."""
    return [lib().orc_gse_shared_exponent(k, e_lo, e_hi) for k in range(n)]


def gse_range(words):
    """(e_lo, e_hi, any_nonzero) of BF16 words."""
    w = _c(words, np.uint16).ravel()
    lo, hi = C.c_int(0), C.c_int(0)
    r = lib().orc_gse_range(_p(w, C.c_uint16), w.size, C.byref(lo), C.byref(hi))
    return lo.value, hi.value, bool(r)


def gse8_encode(word, e_lo, e_hi):
    return lib().orc_gse8_encode(int(word), e_lo, e_hi)


def gse8_decode(code, e_lo, e_hi):
    return lib().orc_gse8_decode(int(code), e_lo, e_hi)


# ---- one group ---------------------------------------------------------------
def quantize_group(x, bits):
    """x: float32 values of one group.  Returns (scale_h, zero_h, codes, saturated)."""
    x = _c(x, np.float32)
    codes = np.zeros(x.size, np.uint8)
    sh, zh = C.c_uint16(0), C.c_uint16(0)
    sat = lib().orc_quantize_group(_p(x, C.c_float), x.size, bits, C.byref(sh), C.byref(zh),
                                   _p(codes, C.c_uint8))
    return sh.value, zh.value, codes, bool(sat)


# ---- layout ----------------------------------------------------------------
def chunk_bytes(L, H, D, T, bits, g=128):
    return lib().orc_chunk_bytes(L, H, D, T, bits, g)


def half_bytes(L, H, D, T, bits, g=128):
    """Bytes of a keys-only or values-only chunk."""
    return lib().orc_half_bytes(L, H, D, T, bits, g)


def tile_payload_bytes(T, D, bits):
    return lib().orc_tile_payload_bytes(T, D, bits)


def tile_meta_bytes(T, D, bits, g):
    return lib().orc_tile_meta_bytes(T, D, bits, g)


def octet_offset(e, bits):
    return lib().orc_octet_offset(e, bits)


def meta_offset(e, g):
    return lib().orc_meta_offset(e, g)


# ---- chunks ------------------------------------------------------------------
def quantize_pack_chunk(src, bits, g=128):
    """src: uint16 BF16 words, shape [L][2][H][T][D].  Returns (packed uint8, n_saturated)."""
    src = _c(src, np.uint16)
    L, two, H, T, D = src.shape
    assert two == 2
    n = chunk_bytes(L, H, D, T, bits, g)
    if n == 0 and T > 0:
        raise ValueError("bad shape/bits/group")
    dst = np.zeros(n, np.uint8)
    r = lib().orc_quantize_pack_chunk(_p(src, C.c_uint16), L, H, D, T, bits, g, _p(dst, C.c_uint8))
    if r < 0:
        raise ValueError("bad shape/bits/group")
    return dst, int(r)


def quantize_pack_half(src, bits, g=128):
    """src: uint16 BF16 words of one half of a document's KV, shape [L][H][T][D]
    (Algorithm 1 treats key chunks and value chunks as separate units)."""
    src = _c(src, np.uint16)
    L, H, T, D = src.shape
    n = half_bytes(L, H, D, T, bits, g)
    if n == 0 and T > 0:
        raise ValueError("bad shape/bits/group")
    dst = np.zeros(n, np.uint8)
    r = lib().orc_quantize_pack_half(_p(src, C.c_uint16), L, H, D, T, bits, g, _p(dst, C.c_uint8))
    if r < 0:
        raise ValueError("bad shape/bits/group")
    return dst, int(r)


def dequant_scatter_half(packed, shape, T, bits, g, kv, out, tok_off):
    """A keys-only (kv=0) or values-only (kv=1) chunk into plane kv of out [L][2][H][cap][D]."""
    L, H, D = shape
    assert out.dtype == np.uint16 and out.flags.c_contiguous
    assert out.shape[0] == L and out.shape[1] == 2 and out.shape[2] == H and out.shape[4] == D
    packed = _c(packed, np.uint8)
    assert packed.size >= half_bytes(L, H, D, T, bits, g)
    r = lib().orc_dequant_scatter_half(_p(packed, C.c_uint8), L, H, D, T, bits, g, kv,
                                       _p(out, C.c_uint16), out.shape[3], tok_off)
    if r != 0:
        raise ValueError("bad shape, plane or not enough room in out")


def dequant_scatter_chunk(packed, shape, T, bits, g, out, tok_off):
    """out: uint16 [L][2][H][cap][D], written in place."""
    L, H, D = shape
    assert out.dtype == np.uint16 and out.flags.c_contiguous
    assert out.shape[0] == L and out.shape[1] == 2 and out.shape[2] == H and out.shape[4] == D
    packed = _c(packed, np.uint8)
    assert packed.size >= chunk_bytes(L, H, D, T, bits, g)
    r = lib().orc_dequant_scatter_chunk(_p(packed, C.c_uint8), L, H, D, T, bits, g,
                                        _p(out, C.c_uint16), out.shape[3], tok_off)
    if r != 0:
        raise ValueError("bad shape or not enough room in out")


def unpack_chunk(packed, shape, T, bits, g=128):
    """Returns (codes [L,2,H,T,D] uint8 or uint16, scale_h, zero_h [L,2,H,T,D//g])."""
    L, H, D = shape
    packed = _c(packed, np.uint8)
    n = L * 2 * H * T * D
    codes = np.zeros(n, np.uint8)
    codes16 = np.zeros(n if bits == 16 else 1, np.uint16)
    ng = n // g if bits in (8, 4) else 1
    sh = np.zeros(max(ng, 1), np.uint16)
    zh = np.zeros(max(ng, 1), np.uint16)
    r = lib().orc_unpack_chunk(_p(packed, C.c_uint8), L, H, D, T, bits, g, _p(codes, C.c_uint8),
                               _p(codes16, C.c_uint16), _p(sh, C.c_uint16), _p(zh, C.c_uint16))
    if r != 0:
        raise ValueError("bad shape")
    if bits == 16:
        return codes16.reshape(L, 2, H, T, D), None, None
    if bits in (43, 52, 143):
        return codes.reshape(L, 2, H, T, D), None, None
    return (codes.reshape(L, 2, H, T, D), sh.reshape(L, 2, H, T, D // g),
            zh.reshape(L, 2, H, T, D // g))


def load_chunks(packed_list, shape, tokens, bits_list, g_list, order, cap_tokens=None,
                tok_base=0, out=None, parts=None):
    """The whole request: chunks gathered in `order`, dequantised and laid one
    after another along the token axis of one BF16 cache [L][2][H][cap][D]
    (Sec. 2.1: load, decompress, concatenate).  Returns (out, tok_off list).

    parts[c] (optional) is 0 for a chunk holding keys and values, 1 keys only, 2 values
    only: the key plane and the value plane then fill independently, each in list order,
    and must end at the same length."""
    L, H, D = shape
    if parts is not None:
        return _load_parts(packed_list, shape, tokens, bits_list, g_list, order, cap_tokens,
                           tok_base, out, parts)
    total = sum(tokens[c] for c in order)
    if cap_tokens is None:
        cap_tokens = tok_base + total
    if tok_base + total > cap_tokens:
        raise ValueError("request does not fit in the cache")
    if out is None:
        out = np.zeros((L, 2, H, cap_tokens, D), np.uint16)
    offs = []
    off = tok_base
    for c in order:
        offs.append(off)
        dequant_scatter_chunk(packed_list[c], shape, tokens[c], bits_list[c], g_list[c], out, off)
        off += tokens[c]
    return out, offs


def _load_parts(packed_list, shape, tokens, bits_list, g_list, order, cap_tokens, tok_base,
                out, parts):
    L, H, D = shape
    need = [sum(tokens[c] for c in order if parts[c] in (0, 1 + kv)) for kv in (0, 1)]
    if need[0] != need[1]:
        raise ValueError("key plane and value plane end at different lengths")
    if cap_tokens is None:
        cap_tokens = tok_base + need[0]
    if tok_base + need[0] > cap_tokens:
        raise ValueError("request does not fit in the cache")
    if out is None:
        out = np.zeros((L, 2, H, cap_tokens, D), np.uint16)
    off = [tok_base, tok_base]
    offs = []
    for c in order:
        if parts[c] == 0:
            if off[0] != off[1]:
                raise ValueError("a whole chunk needs both planes at the same length")
            offs.append(off[0])
            dequant_scatter_chunk(packed_list[c], shape, tokens[c], bits_list[c], g_list[c], out, off[0])
            off[0] += tokens[c]
            off[1] += tokens[c]
        else:
            kv = parts[c] - 1
            offs.append(off[kv])
            dequant_scatter_half(packed_list[c], shape, tokens[c], bits_list[c], g_list[c], kv,
                                 out, off[kv])
            off[kv] += tokens[c]
    return out, offs


def rmse_bf16(a, b):
    a = _c(a, np.uint16).ravel()
    b = _c(b, np.uint16).ravel()
    assert a.size == b.size
    return lib().orc_rmse_bf16(_p(a, C.c_uint16), _p(b, C.c_uint16), a.size)


# ---- paged cache ---------------------------------------------------------------
def paged_view(pages, layout, L, H, P, D):
    """The physical page pool as an array indexed [page][l][kv][h][row in page][d].

    pages is a flat uint16 array holding n_pages pages of P token rows.  layout
    "page_major": each page is one contiguous [L][2][H][P][D] block; "tile_major": the pool
    is [L][2][H][n_pages][P][D] (every tile's pages side by side).  Returns a view (writes
    through)."""
    n_pages = pages.size // (L * 2 * H * P * D)
    if layout == "page_major":
        return pages.reshape(n_pages, L, 2, H, P, D)
    if layout == "tile_major":
        return pages.reshape(L, 2, H, n_pages, P, D).transpose(3, 0, 1, 2, 4, 5)
    raise ValueError(layout)


def load_chunks_paged(packed_list, shape, tokens, bits_list, g_list, order, pages, layout, P,
                      page_table, tok_base=0, parts=None):
    """The request of load_chunks, written into a paged cache: token row r of the request
    (r counted from 0, the chunks starting at tok_base) lives in physical page
    page_table[r // P] at row r % P.  Rows the request does not cover are left alone.
    Built from load_chunks itself: the contiguous cache is computed first and its rows are
    then copied to their pages one by one."""
    L, H, D = shape
    virt, offs = load_chunks(packed_list, shape, tokens, bits_list, g_list, order,
                             tok_base=tok_base, parts=parts)
    end = virt.shape[3]
    if end > len(page_table) * P:
        raise ValueError("request does not fit in the page table")
    view = paged_view(pages, layout, L, H, P, D)
    for r in range(tok_base, end):
        view[page_table[r // P], :, :, :, r % P, :] = virt[:, :, :, r, :]
    return offs
