"""Pins for the oracle's GSE-8 (1+4+3): the array the paper works out, the paper's
three conversion steps and its decoding rule restated on bit strings and run over
every BF16 value / every code, and invariants of a truncating encoder."""
import json
import os

import numpy as np
import pytest

from oracle import codec
from paper_2510_20878_amd import workloads as wl


def _gold(golden_dir):
    return json.load(open(os.path.join(golden_dir, "paper_values.json")))["gse8"]


def test_shared_exponent_array_of_the_papers_example(golden_dir):
    g = _gold(golden_dir)
    lo, hi = g["range"]                    # the open-closed exponent range (lo, hi]
    arr = codec.gse_shared_exponents(lo + 1, hi, 16)
    n = len(g["shared_exponents"])
    assert arr[:n] == g["shared_exponents"]
    assert all(a == hi for a in arr[n:])                       # clipped at the top
    assert all(b - a <= g["step"] for a, b in zip(arr[:-1], arr[1:]))
    assert g["split"] == [1, 4, 3]


# ---- the paper's procedure on bit strings ----------------------------------------
def _steps_encode(word, shared):
    """Sec. 2.2.2: (1) take the exponent E; (2) smallest shared exponent G >= E,
    d = G - E; (3) shift the fraction right by d + 1 and set bit d + 1 from the top.
    The field keeps the 3 leading bits of that string."""
    sign = word >> 15
    if word & 0x7FFF == 0:
        return sign << 7
    e_field, frac = (word >> 7) & 0xFF, word & 0x7F
    if e_field == 0:                                 # BF16 subnormal: 0.frac * 2^-126
        E, bits = -126, [0] + [(frac >> (6 - i)) & 1 for i in range(7)]
    else:
        E, bits = e_field - 127, [1] + [(frac >> (6 - i)) & 1 for i in range(7)]
    k = next(i for i, g in enumerate(shared) if g >= E)
    d = shared[k] - E
    string = [0] * d + bits                          # leading one now at position d + 1
    field = string[0] * 4 + string[1] * 2 + string[2]
    if field == 0:
        return sign << 7
    return (sign << 7) | (k << 3) | field


def _steps_decode(code, shared):
    """Sec. 2.2.2: index and position of the first 1 give the exponent; the bits after
    it, shifted back, are the fraction."""
    sign, k, field = code >> 7, (code >> 3) & 15, code & 7
    if field == 0:
        return -0.0 if sign else 0.0
    bits = [(field >> 2) & 1, (field >> 1) & 1, field & 1]
    d = bits.index(1)
    rest = bits[d + 1:]
    frac = sum(b / 2 ** (i + 1) for i, b in enumerate(rest))
    v = (1 + frac) * 2.0 ** (shared[k] - d)
    return -v if sign else v


@pytest.mark.parametrize("e_lo,e_hi", [(-9, 10), (-6, 3), (-20, 4), (0, 0), (-126, -100), (2, 40)])
def test_encode_equals_the_papers_three_steps_for_every_bf16_value(e_lo, e_hi):
    shared = codec.gse_shared_exponents(e_lo, e_hi)
    words = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    f = wl.bf16_words_to_f32(words)
    for w in words[np.isfinite(f)]:
        e = ((int(w) >> 7) & 0xFF)
        E = e - 127 if e else -126
        if E > e_hi and (w & 0x7FFF):
            continue                                  # cannot occur: e_hi is the tile maximum
        assert codec.gse8_encode(int(w), e_lo, e_hi) == _steps_encode(int(w), shared), hex(int(w))


@pytest.mark.parametrize("e_lo,e_hi", [(-9, 10), (-6, 3), (0, 0), (-47, 0)])
def test_decode_equals_the_papers_rule_for_every_code(e_lo, e_hi):
    shared = codec.gse_shared_exponents(e_lo, e_hi)
    for c in range(256):
        got, ref = codec.gse8_decode(c, e_lo, e_hi), _steps_decode(c, shared)
        assert got == ref and np.signbit(got) == np.signbit(ref), c
        # every decoded value is a BF16 value
        assert wl.bf16_words_to_f32(wl.f32_to_bf16_words(np.array([got], np.float32)))[0] == got


def test_truncation_invariants():
    rng = np.random.default_rng(3)
    x = (rng.standard_normal(20000) * np.exp(rng.normal(0, 2, 20000))).astype(np.float32)
    words = wl.f32_to_bf16_words(x)
    xb = wl.bf16_words_to_f32(words)
    e_lo, e_hi, nz = codec.gse_range(words)
    assert nz and e_hi - e_lo <= 47
    shared = codec.gse_shared_exponents(e_lo, e_hi)
    for w, v in zip(words[:5000], xb[:5000]):
        c = codec.gse8_encode(int(w), e_lo, e_hi)
        y = codec.gse8_decode(c, e_lo, e_hi)
        assert abs(y) <= abs(v) and (y == 0 or np.sign(y) == np.sign(v))     # never rounds up
        if v != 0 and np.floor(np.log2(abs(v))) >= e_lo:
            E = int(np.floor(np.log2(abs(v))))
            d = next(g for g in shared if g >= E) - E
            assert 0 <= d <= 2
            assert abs(v) - abs(y) < 2.0 ** (E - (2 - d))                    # 2 - d fraction bits kept
        # a decoded value is a fixed point of the encoder
        yw = int(wl.f32_to_bf16_words(np.array([y], np.float32))[0])
        assert codec.gse8_decode(codec.gse8_encode(yw, e_lo, e_hi), e_lo, e_hi) == y
    # powers of two inside the range are exact
    for E in range(e_lo, e_hi + 1):
        w = int(wl.f32_to_bf16_words(np.array([2.0 ** E], np.float32))[0])
        assert codec.gse8_decode(codec.gse8_encode(w, e_lo, e_hi), e_lo, e_hi) == 2.0 ** E


def test_range_rules():
    w = wl.f32_to_bf16_words(np.array([0.0, -0.0, 3.0, -0.02, 1e-30], np.float32))
    assert codec.gse_range(w[:2]) == (0, 0, False)                # nothing but zeros
    assert codec.gse_range(w[:4]) == (-6, 1, True)                # 0.02 = 1.28 * 2^-6, 3 = 1.5 * 2^1
    e_lo, e_hi, _ = codec.gse_range(w)
    assert (e_lo, e_hi) == (1 - 47, 1)                            # 48 binades at most
    assert codec.gse8_encode(int(w[4]), e_lo, e_hi) == 0          # 1e-30 is flushed
    assert codec.gse8_encode(int(w[1]), e_lo, e_hi) == 0x80       # the sign of zero is kept


def test_chunk_path_sizes_meta_and_decode(golden_dir):
    L, H, D, T = 2, 2, 64, 100
    src = wl.kv_chunk(L, H, D, T, 31, outlier_channels=1)
    packed, _ = codec.quantize_pack_chunk(src, 143)
    tile_bytes = 4 * 2048 + 16                                    # 4 blocks + the range block
    assert packed.size == codec.chunk_bytes(L, H, D, T, 143) == L * 2 * H * tile_bytes
    ratio = codec.chunk_bytes(32, 8, 128, 512, 16) / codec.chunk_bytes(32, 8, 128, 512, 143)
    assert abs(ratio - _gold(golden_dir)["compression_ratio"]) < 2e-4      # Table 2 prints 1.9996
    codes, _, _ = codec.unpack_chunk(packed, (L, H, D), T, 143)
    out = np.zeros((L, 2, H, T, D), np.uint16)
    codec.dequant_scatter_chunk(packed, (L, H, D), T, 143, 0, out, 0)
    y = wl.bf16_words_to_f32(out).reshape(L * 2 * H, T * D)
    x = wl.bf16_words_to_f32(src).reshape(L * 2 * H, T * D)
    flat = src.reshape(L * 2 * H, T * D)
    for tile in range(L * 2 * H):
        rec = packed[tile * tile_bytes:(tile + 1) * tile_bytes]
        e_lo, e_hi = int(rec[-16:].view(np.int8)[0]), int(rec[-16:].view(np.int8)[1])
        assert (e_lo, e_hi, True) == codec.gse_range(flat[tile])
        assert not rec[-14:].any()
        for e in range(0, T * D, 97):
            assert codes.reshape(L * 2 * H, T * D)[tile, e] == codec.gse8_encode(int(flat[tile, e]), e_lo, e_hi)
            assert y[tile, e] == codec.gse8_decode(int(codes.reshape(L * 2 * H, T * D)[tile, e]), e_lo, e_hi)
    assert np.all(np.abs(y) <= np.abs(x))


def test_rmse_order_of_the_four_schemes_matches_the_paper():
    """Fig. 9: INT8 < E4M3 < E5M2 < GSE-8."""
    src = wl.kv_chunk(2, 4, 128, 128, 5)
    r = {}
    for bits in (8, 43, 52, 143):
        packed, _ = codec.quantize_pack_chunk(src, bits, 128)
        out = np.zeros_like(src)
        codec.dequant_scatter_chunk(packed, (2, 4, 128), 128, bits, 128, out, 0)
        r[bits] = codec.rmse_bf16(out, src)
    assert r[8] < r[43] < r[52] < r[143]
