"""Pins for the oracle's quantise / dequantise arithmetic: error bound, exact
round trips, exhaustive code enumeration, closed-form RMSE, library reductions."""
import json
import os

import numpy as np
import pytest

from oracle import codec
from paper_2510_20878_amd import workloads as wl

F16 = lambda v: int(np.float16(v).view(np.uint16))


def _f64(h):
    return codec.fp16_to_f64(h)


# ---- P4: exhaustive codes ------------------------------------------------------
@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("z,s", [(-3.5, 0.25), (0.0, 1.0), (-128.0, 1.0), (12.0, 0.0625),
                                 (0.0, 2.0 ** -24), (-2.0 ** -14, 2.0 ** -20)])
def test_every_code_is_reached_and_dequantises_exactly(bits, z, s):
    qmax = (1 << bits) - 1
    x = (np.float64(z) + np.arange(qmax + 1) * np.float64(s)).astype(np.float32)
    assert np.all(x.astype(np.float64) == z + np.arange(qmax + 1) * s)   # inputs are exact
    sh, zh, codes, sat = codec.quantize_group(x, bits)
    assert not sat
    assert (sh, zh) == (F16(s), F16(z))
    assert np.array_equal(codes, np.arange(qmax + 1, dtype=np.uint8))
    for q in range(qmax + 1):
        assert codec.dequant_f32(q, sh, zh) == x[q]


@pytest.mark.parametrize("bits", [4, 8])
def test_every_code_through_the_chunk_path(bits):
    # integers 0..255 and -128..127 are exact in BF16; one group holds all codes
    qmax = (1 << bits) - 1
    g = 256 if bits == 8 else 32
    L, H, D, T = 1, 1, 256, 8
    rng = np.random.default_rng(3)
    vals = np.empty((L, 2, H, T, D), np.float32)
    for idx in np.ndindex(L, 2, H, T, D // g):
        grp = rng.integers(0, qmax + 1, g)
        grp[rng.permutation(g)[:qmax + 1]] = np.arange(qmax + 1)   # all codes present
        l, kv, h, t, gi = idx
        vals[l, kv, h, t, gi * g:(gi + 1) * g] = grp - (128 if kv else 0)
    src = wl.f32_to_bf16_words(vals)
    packed, sat = codec.quantize_pack_chunk(src, bits, g)
    assert sat == 0
    codes, sh, zh = codec.unpack_chunk(packed, (L, H, D), T, bits, g)
    expect = vals.copy()
    expect[:, 1] += 128
    assert np.array_equal(codes, expect.astype(np.uint8))
    assert np.all(sh == F16(1.0))
    assert np.all(zh[:, 0] == F16(0.0)) and np.all(zh[:, 1] == F16(-128.0))
    out = np.zeros((L, 2, H, T, D), np.uint16)
    codec.dequant_scatter_chunk(packed, (L, H, D), T, bits, g, out, 0)
    assert np.array_equal(out, src)           # exact round trip


def test_ties_round_to_even_code():
    x = np.array([0.0, 0.5, 1.5, 2.5, 3.5, 4.5, 15.0, 14.5], np.float32)
    sh, zh, codes, _ = codec.quantize_group(x, 4)
    assert (sh, zh) == (F16(1.0), F16(0.0))
    assert list(codes) == [0, 0, 2, 2, 4, 4, 15, 14]


# ---- P1: error bound, directed rounding -----------------------------------------
@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("g", [32, 64, 128, 512])
def test_error_bound_half_scale(bits, g):
    rng = np.random.default_rng(10 + bits + g)
    qmax = (1 << bits) - 1
    n_groups = 3000 if g < 512 else 1000
    scales = np.minimum(np.exp(rng.normal(0, 3, n_groups)), 500.0)
    offs = rng.normal(0, 5, n_groups) * scales
    for k in range(n_groups):
        x = (rng.standard_normal(g) * scales[k] + offs[k]).astype(np.float32)
        x = wl.bf16_words_to_f32(wl.f32_to_bf16_words(x))       # BF16-valued inputs
        sh, zh, codes, sat = codec.quantize_group(x, bits)
        assert not sat
        s, z = _f64(sh), _f64(zh)
        assert z <= float(x.min())                               # zero rounded down
        assert s >= (float(x.max()) - z) / qmax * (1 - 2 ** -23)  # scale rounded up
        assert codes.max() <= qmax
        rec = codes.astype(np.float64) * s + z
        err = np.abs(rec - x.astype(np.float64))
        assert np.all(err <= s / 2 * (1 + 2 ** -12)), (k, err.max(), s)
        # scale is the *smallest* fp16 >= the fp32 quotient, zero the largest <= min
        quo = np.float32(np.float32(x.max()) - np.float32(z)) / np.float32(qmax)
        if sh > 0:
            assert _f64(sh - 1) < float(quo) <= s
        zdn, _ = codec.fp16_round_down(x.min())
        assert zdn == zh


def test_bf16_output_adds_at_most_half_ulp():
    rng = np.random.default_rng(5)
    for _ in range(20000):
        q = int(rng.integers(0, 256))
        sh = int(rng.integers(0, 0x7C00))
        zh = int(rng.integers(0, 0x7C00)) | (int(rng.integers(0, 2)) << 15)
        exact = q * _f64(sh) + _f64(zh)
        f = codec.dequant_f32(q, sh, zh)
        assert f == np.float32(exact)                     # one rounding of the exact sum
        y = codec.bf16_to_f32(codec.dequant_bf16(q, sh, zh))
        if f != 0 and np.isfinite(y):
            ulp = 2.0 ** (np.floor(np.log2(abs(float(f)))) - 7)
            assert abs(y - float(f)) <= ulp / 2


# ---- P5: code stability ----------------------------------------------------------
@pytest.mark.parametrize("bits", [4, 8])
def test_requantising_dequantised_values_with_stored_meta_is_stable(bits):
    rng = np.random.default_rng(6)
    qmax = (1 << bits) - 1
    for _ in range(500):
        x = (rng.standard_normal(64) * np.exp(rng.normal(0, 2))).astype(np.float32)
        sh, zh, codes, _ = codec.quantize_group(x, bits)
        s, z = np.float32(_f64(sh)), np.float32(_f64(zh))
        rec = np.array([codec.dequant_f32(int(q), sh, zh) for q in codes], np.float32)
        again = np.clip(np.rint((rec - z) / s), 0, qmax).astype(np.uint8) if s else codes * 0
        assert np.array_equal(again, codes)


# ---- P6: reductions to library routines -------------------------------------------
@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("g", [64, 512])
def test_codes_equal_numpy_expression_given_stored_meta(bits, g):
    if g == 64:
        tiny = wl.tiny_config(0)
        L, H, D = tiny["shape"]
        src = tiny["chunks"][1]
    else:                                    # the widest group: one per row of a 512-wide head
        L, H, D = 1, 2, 512
        src = wl.kv_chunk(L, H, D, 128, 31)
    packed, _ = codec.quantize_pack_chunk(src, bits, g)
    codes, sh, zh = codec.unpack_chunk(packed, (L, H, D), 128, bits, g)
    x = wl.bf16_words_to_f32(src).reshape(L, 2, H, 128, D // g, g)
    s = sh.view(np.float16).astype(np.float32)[..., None]
    z = zh.view(np.float16).astype(np.float32)[..., None]
    q = np.clip(np.rint((x - z) / s), 0, (1 << bits) - 1).astype(np.uint8)
    assert np.array_equal(q.reshape(codes.shape), codes)
    # group min / max against numpy reductions
    assert np.all(z[..., 0] <= x.min(-1))
    nxt = np.nextafter(zh.view(np.float16), np.float16(np.inf)).astype(np.float32)
    assert np.all(nxt > x.min(-1))


def test_all_16bit_load_is_a_concatenate():
    tiny = wl.tiny_config(1)
    shape, order = tiny["shape"], tiny["order"]
    packed = [codec.quantize_pack_chunk(c, 16)[0] for c in tiny["chunks"]]
    out, offs = codec.load_chunks(packed, shape, tiny["tokens"], [16] * 4, [64] * 4, order)
    ref = np.concatenate([tiny["chunks"][c] for c in order], axis=3)
    assert np.array_equal(out, ref)
    assert offs == [0, 128, 256, 384]


def test_16bit_tag_round_trips_every_bf16_word():
    words = np.arange(65536, dtype=np.uint32).astype(np.uint16)    # NaN payloads too
    src = words.reshape(1, 2, 1, 256, 128)
    packed, _ = codec.quantize_pack_chunk(src, 16)
    out = np.zeros_like(src)
    codec.dequant_scatter_chunk(packed, (1, 1, 128), 256, 16, 128, out, 0)
    assert np.array_equal(out, src)


# ---- P7: order and offsets ---------------------------------------------------------
def test_gather_order_and_token_offsets():
    L, H, D = 2, 2, 64
    toks = [24, 40, 8, 64]
    chunks = [wl.patterned_chunk(L, H, D, t, i) for i, t in enumerate(toks)]
    bits = [16, 8, 4, 8]
    packed = [codec.quantize_pack_chunk(c, b, 64)[0] for c, b in zip(chunks, bits)]
    order = [3, 0, 2, 1, 0]                     # a repeated id is loaded twice
    out, offs = codec.load_chunks(packed, (L, H, D), toks, bits, [64] * 4, order,
                                  cap_tokens=200, tok_base=5)
    f = wl.bf16_words_to_f32(out)
    pos = 5
    for c in order:
        blk = f[:, :, :, pos:pos + toks[c], :]
        assert np.all(blk[..., 1:] == c)                 # chunk number in every other column
        assert np.all(blk[..., 0] == np.arange(toks[c])[None, None, None, :])  # token index
        pos += toks[c]
    assert np.all(out[:, :, :, :5] == 0) and np.all(out[:, :, :, pos:] == 0)  # untouched rows
    assert offs == [5, 69, 93, 101, 141]


def test_load_rejects_overflowing_request():
    tiny = wl.tiny_config(0)
    packed = [codec.quantize_pack_chunk(c, 16)[0] for c in tiny["chunks"]]
    with pytest.raises(ValueError):
        codec.load_chunks(packed, tiny["shape"], tiny["tokens"], [16] * 4, [64] * 4,
                          tiny["order"], cap_tokens=500)


# ---- P8: closed-form RMSE (Eq. 1) --------------------------------------------------
def test_rmse_matches_uniform_quantiser_closed_form():
    rng = np.random.default_rng(7)
    g, n_groups = 128, 2000
    res = {}
    for bits in (4, 8):
        qmax = (1 << bits) - 1
        sq, n = 0.0, 0
        for _ in range(n_groups):
            x = rng.uniform(0.0, 15.0, g).astype(np.float32)
            x[0], x[1] = 0.0, 15.0                      # pin min and max: s = 15/qmax
            sh, zh, codes, _ = codec.quantize_group(x, bits)
            s = _f64(sh)
            assert abs(s - 15.0 / qmax) <= 15.0 / qmax * 2 ** -10
            rec = codes.astype(np.float64) * s + _f64(zh)
            sq += float(np.sum((rec - x) ** 2))
            n += g
        res[bits] = np.sqrt(sq / n)
        assert abs(res[bits] / ((15.0 / qmax) / np.sqrt(12)) - 1) < 0.03
    assert abs(res[4] / res[8] - 17.0) < 0.8            # 255 / 15


def test_rmse_function_is_eq1():
    a = wl.f32_to_bf16_words(np.array([1.0, 2.0, 3.0, 4.0], np.float32))
    b = wl.f32_to_bf16_words(np.array([1.0, 0.0, 3.0, 8.0], np.float32))
    assert codec.rmse_bf16(a, b) == pytest.approx(np.sqrt((0 + 4 + 0 + 16) / 4))


# ---- P9 and the Tiny configuration ---------------------------------------------------
def test_tiny_outlier_groups_have_wider_scale_and_keep_the_bound():
    tiny = wl.tiny_config(0)
    L, H, D = tiny["shape"]
    src = tiny["chunks"][2]
    x = wl.bf16_words_to_f32(src)
    packed, sat = codec.quantize_pack_chunk(src, 4, 64)
    assert sat == 0
    codes, sh, zh = codec.unpack_chunk(packed, (L, H, D), 128, 4, 64)
    s = sh.view(np.float16).astype(np.float64)
    z = zh.view(np.float16).astype(np.float64)
    rec = codes.astype(np.float64) * s + z           # one group per row (D == g)
    assert np.all(np.abs(rec - x) <= s / 2 * (1 + 2 ** -12))
    plain, _ = codec.quantize_pack_chunk(wl.kv_chunk(L, H, D, 128, 2, key_spread=False), 4, 64)
    s_plain = codec.unpack_chunk(plain, (L, H, D), 128, 4, 64)[1].view(np.float16).astype(np.float64)
    assert 4.0 < np.median(s) / np.median(s_plain) < 15.0   # x15 channels widen the range


def test_value_ranges_of_synthetic_kv_match_the_paper(golden_dir):
    gold = json.load(open(os.path.join(golden_dir, "paper_values.json")))["value_ranges"]
    x = wl.bf16_words_to_f32(wl.kv_chunk(4, 8, 128, 256, 11))
    k, v = np.abs(x[:, 0]), np.abs(x[:, 1])
    assert np.quantile(k, 0.995) < gold["key_abs_max"]      # "primarily" inside the range
    assert v.max() < gold["value_abs_max"]
    assert k.std() > 1.5 * v.std()                     # Keys spread wider than Values


# ---- degenerate groups ------------------------------------------------------------------
def test_constant_group():
    for v in (0.0, 1.5, -7.0):
        sh, zh, codes, sat = codec.quantize_group(np.full(64, v, np.float32), 4)
        assert (sh, zh, sat) == (0, F16(v), False) and not codes.any()
        assert codec.dequant_f32(0, sh, zh) == np.float32(v)
    # a constant that fp16 cannot hold: zero rounds down, scale up, bound still holds
    x = np.full(32, wl.bf16_words_to_f32(wl.f32_to_bf16_words(np.array([3.3e-6], np.float32)))[0])
    sh, zh, codes, sat = codec.quantize_group(x, 8)
    s, z = _f64(sh), _f64(zh)
    assert not sat and z <= x[0]
    rec = codes.astype(np.float64) * s + z
    assert np.all(np.abs(rec - x) <= s / 2 * (1 + 2 ** -12))


def test_negative_zero_minimum_is_stored_as_plus_zero():
    x = np.array([-0.0, 0.0, 1.0, 2.0], np.float32)
    sh, zh, codes, _ = codec.quantize_group(x, 4)
    assert zh == 0


def test_saturation_is_reported():
    x = np.array([-1e5, 0.0, 1.0, 2.0], np.float32)
    assert codec.quantize_group(x, 8)[3]
    x = np.array([0.0, 3e7, 1.0, 2.0], np.float32)       # scale 3e7/15 > 65504
    sh, zh, codes, sat = codec.quantize_group(x, 4)
    assert sat and sh == 0x7BFF
    x = np.array([0.0, 6e4, 1.0, 2.0], np.float32)
    assert not codec.quantize_group(x, 4)[3]
