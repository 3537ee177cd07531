"""Pins for the oracle's FP8 (E4M3 / E5M2) encode and decode: the library's own
float8 conversions, exhaustive enumeration, and the ranges the paper prints."""
import json
import os

import numpy as np
import pytest
import torch

from oracle import codec
from paper_2510_20878_amd import workloads as wl

KINDS = {43: torch.float8_e4m3fn, 52: torch.float8_e5m2}


@pytest.mark.parametrize("kind", [43, 52])
def test_decode_all_256_codes_equals_torch(kind):
    ref = torch.arange(256, dtype=torch.uint8).view(KINDS[kind]).to(torch.float32).numpy()
    for c in range(256):
        got = codec.fp8_to_f64(c, kind)
        if np.isnan(ref[c]):
            assert np.isnan(got)
        else:
            assert got == ref[c], hex(c)


def test_ranges_and_field_widths_the_paper_prints(golden_dir):
    gold = json.load(open(os.path.join(golden_dir, "paper_values.json")))["fp8_formats"]
    for kind, key in ((43, "e4m3"), (52, "e5m2")):
        vals = np.array([codec.fp8_to_f64(c, kind) for c in range(256)])
        fin = vals[np.isfinite(vals)]
        assert fin.max() == gold[key]["max"] and fin.min() == -gold[key]["max"]
        # field widths: distinct finite magnitudes = 2^(e+m) minus the NaN/inf codes
        e, m = gold[key]["exponent"], gold[key]["fraction"]
        n_special = 1 if kind == 43 else 2 ** m          # E4M3: one NaN; E5M2: inf + NaNs
        assert np.unique(np.abs(fin)).size == 2 ** (e + m) - n_special
    assert abs(gold["e5m2"]["max_printed"] - gold["e5m2"]["max"]) == 10   # the printed typo


@pytest.mark.parametrize("kind", [43, 52])
def test_encode_every_finite_bf16_value(kind):
    """In range: equal to torch's round-to-nearest-even conversion.  Beyond the largest
    finite value (torch gives NaN / inf there): saturates, keeping the sign."""
    w = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    f = wl.bf16_words_to_f32(w)
    ref = torch.from_numpy(f.copy()).to(KINDS[kind]).view(torch.uint8).numpy()
    max_code = 0x7E if kind == 43 else 0x7B
    for i in np.flatnonzero(np.isfinite(f)):
        got = codec.f64_to_fp8(float(f[i]), kind)
        if np.isfinite(codec.fp8_to_f64(int(ref[i]), kind)):
            assert got == ref[i], (hex(int(w[i])), got, ref[i])
        else:
            assert got == (max_code | (0x80 if f[i] < 0 else 0))


@pytest.mark.parametrize("kind", [43, 52])
def test_round_trip_nearest_and_ties(kind):
    vals = sorted({codec.fp8_to_f64(c, kind) for c in range(256)
                   if np.isfinite(codec.fp8_to_f64(c, kind))})
    for c in range(256):                                   # every code is a fixed point
        v = codec.fp8_to_f64(c, kind)
        if np.isfinite(v):
            assert codec.f64_to_fp8(v, kind) == c
    # midpoints of neighbours go to the code with the even fraction; just off the
    # midpoint goes to the nearer neighbour (brute force over the whole grid)
    for lo, hi in zip(vals[:-1], vals[1:]):
        mid = (lo + hi) / 2
        got = codec.f64_to_fp8(mid, kind)
        assert codec.fp8_to_f64(got, kind) in (lo, hi) and got % 2 == 0     # -0.0 == 0.0
        assert codec.fp8_to_f64(codec.f64_to_fp8(np.nextafter(mid, hi), kind), kind) == hi
        assert codec.fp8_to_f64(codec.f64_to_fp8(np.nextafter(mid, lo), kind), kind) == lo
    assert codec.f64_to_fp8(-0.0, kind) == 0x80 and codec.f64_to_fp8(0.0, kind) == 0
    assert codec.f64_to_fp8(1e9, kind) == (0x7E if kind == 43 else 0x7B)
    assert codec.f64_to_fp8(-1e9, kind) == (0xFE if kind == 43 else 0xFB)


@pytest.mark.parametrize("kind", [43, 52])
def test_chunk_path_sizes_codes_and_exact_decode(kind):
    L, H, D, T = 2, 2, 64, 100                          # ragged: 3.125 blocks per tile
    src = wl.kv_chunk(L, H, D, T, 21, outlier_channels=1)
    packed, sat = codec.quantize_pack_chunk(src, kind)
    assert sat == 0
    assert packed.size == codec.chunk_bytes(L, H, D, T, kind) == L * 2 * H * 4 * 2048
    assert codec.chunk_bytes(32, 8, 128, 512, 16) / codec.chunk_bytes(32, 8, 128, 512, kind) == 2.0
    codes, _, _ = codec.unpack_chunk(packed, (L, H, D), T, kind)
    x = wl.bf16_words_to_f32(src)
    ref = torch.from_numpy(x.copy()).to(KINDS[kind]).view(torch.uint8).numpy()
    assert np.array_equal(codes, ref)                   # all values are in range here
    out = np.zeros((L, 2, H, T, D), np.uint16)
    codec.dequant_scatter_chunk(packed, (L, H, D), T, kind, 128, out, 0)
    dec = torch.from_numpy(ref.copy()).view(KINDS[kind]).to(torch.float32).numpy()
    assert np.array_equal(wl.bf16_words_to_f32(out), dec)    # decode is exact in BF16
    # relative error of a normal value is at most 2^-(fraction bits + 1)
    big = np.abs(x) > (2.0 ** -6 if kind == 43 else 2.0 ** -14)
    rel = np.abs(dec[big] - x[big]) / np.abs(x[big])
    assert rel.max() <= 2.0 ** -(4 if kind == 43 else 3)
    # payload layout is that of the 8-bit integer tag
    e = 3 * 2048 + 77
    assert packed[codec.octet_offset(e, 8) + e % 8] == codes.reshape(L * 2 * H, T * D)[0, e]


def test_error_order_matches_the_paper():
    """Sec. 3.2.1, Fig. 9: E5M2 loses more than E4M3 (fewer fraction bits); the 8-bit
    integer scheme loses least on KV-like data."""
    src = wl.kv_chunk(2, 4, 128, 128, 5)
    rmse = {}
    for bits in (8, 43, 52):
        packed, _ = codec.quantize_pack_chunk(src, bits, 128)
        out = np.zeros_like(src)
        codec.dequant_scatter_chunk(packed, (2, 4, 128), 128, bits, 128, out, 0)
        rmse[bits] = codec.rmse_bf16(out, src)
    assert rmse[8] < rmse[43] < rmse[52]
