"""Pins for the oracle's number-format helpers: every conversion is compared
with a library conversion (numpy float16, torch bfloat16) or enumerated."""
import numpy as np
import torch

from oracle import codec


def _finite_fp16_words():
    w = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    f = w.view(np.float16)
    return w[np.isfinite(f)]


def test_fp16_decode_matches_numpy_all_words():
    for h in range(65536):
        ref = float(np.uint16(h).view(np.float16))
        got = codec.fp16_to_f64(h)
        if np.isnan(ref):
            assert np.isnan(got)
        else:
            assert got == ref, hex(h)


def test_bf16_decode_matches_torch_all_words():
    w = torch.arange(65536, dtype=torch.int32).to(torch.int16)
    ref = w.view(torch.bfloat16).to(torch.float32).numpy()
    for h in range(0, 65536, 7):
        got = codec.bf16_to_f32(h)
        if np.isnan(ref[h]):
            assert np.isnan(got)
        else:
            assert got == ref[h]


def test_bf16_rne_matches_torch():
    rng = np.random.default_rng(1)
    hi = np.arange(65536, dtype=np.uint32)
    lows = [0, 1, 0x7FFF, 0x8000, 0x8001, 0xFFFF]
    words = np.concatenate([(hi << 16) | lo for lo in lows] +
                           [rng.integers(0, 2**32, 200000, dtype=np.uint64).astype(np.uint32)])
    f = words.view(np.float32)
    f = f[np.isfinite(f)]
    ref = torch.from_numpy(f.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    # subsample the enumerated part to keep the ctypes loop short, keep every tie case
    idx = np.arange(f.size)
    keep = idx[(idx % 5 == 0) | ((f.view(np.uint32) & 0xFFFF) == 0x8000)]
    for i in keep:
        assert codec.f32_to_bf16_rne(f[i]) == ref[i], hex(int(f.view(np.uint32)[i]))


def _canon(h):
    return 0 if h == 0x8000 else int(h)


def test_fp16_directed_rounding_on_grid_and_neighbours():
    words = _finite_fp16_words()
    f16 = words.view(np.float16)
    with np.errstate(over="ignore"):
        up16 = np.nextafter(f16, np.float16(np.inf))     # library successor on the fp16 grid
        dn16 = np.nextafter(f16, np.float16(-np.inf))
    x = f16.astype(np.float32)
    x_above = np.nextafter(x, np.float32(np.inf))     # just above the grid point, in fp32
    x_below = np.nextafter(x, np.float32(-np.inf))
    for k in range(0, words.size, 3):
        h = int(words[k])
        rd, s1 = codec.fp16_round_down(x[k])
        ru, s2 = codec.fp16_round_up(x[k])
        assert rd == _canon(h) and ru == _canon(h) and not s1 and not s2
        # just above: down -> h, up -> successor (or saturate at the top)
        rd, s1 = codec.fp16_round_down(x_above[k])
        ru, s2 = codec.fp16_round_up(x_above[k])
        assert rd == _canon(h) and not s1
        if np.isfinite(up16[k]):
            assert ru == _canon(int(up16[k].view(np.uint16))) and not s2
        else:
            assert ru == 0x7BFF and s2
        # just below: up -> h, down -> predecessor (or saturate at the bottom)
        ru, s2 = codec.fp16_round_up(x_below[k])
        rd, s1 = codec.fp16_round_down(x_below[k])
        assert ru == _canon(h) and not s2
        if np.isfinite(dn16[k]):
            assert rd == _canon(int(dn16[k].view(np.uint16))) and not s1
        else:
            assert rd == 0xFBFF and s1


def test_fp16_directed_rounding_brackets_random_fp32():
    rng = np.random.default_rng(2)
    x = np.concatenate([
        rng.standard_normal(20000).astype(np.float32) * np.float32(30.0),
        (rng.standard_normal(5000) * 1e-6).astype(np.float32),
        (rng.standard_normal(5000) * 2e4).astype(np.float32),
        np.array([1e-40, -1e-40, 6e-8, -6e-8, 65504.0, -65504.0, 65519.9, 0.0, -0.0], np.float32),
    ])
    with np.errstate(over="ignore"):
        rne = x.astype(np.float16)
    for k in range(x.size):
        xv = float(x[k])
        rd, s1 = codec.fp16_round_down(x[k])
        ru, s2 = codec.fp16_round_up(x[k])
        lo, hi = codec.fp16_to_f64(rd), codec.fp16_to_f64(ru)
        if abs(xv) <= 65504.0:
            assert not s1 and not s2
            assert lo <= xv <= hi
            if lo == hi:
                assert lo == xv
            else:  # adjacent grid points
                assert float(np.nextafter(np.float16(lo), np.float16(np.inf))) == hi
            if np.isfinite(rne[k]):
                assert float(rne[k]) in (lo, hi)     # nearest-even lands on one of the two


def test_fp16_saturation_flags():
    assert codec.fp16_round_down(-70000.0) == (0xFBFF, True)
    assert codec.fp16_round_down(70000.0) == (0x7BFF, False)
    assert codec.fp16_round_up(70000.0) == (0x7BFF, True)
    assert codec.fp16_round_up(-70000.0) == (0xFBFF, False)
    assert codec.fp16_round_up(float("inf")) == (0x7BFF, True)
    # smallest positive input rounds up to the smallest subnormal, down to +0
    assert codec.fp16_round_up(1e-30) == (0x0001, False)
    assert codec.fp16_round_down(1e-30) == (0x0000, False)
    assert codec.fp16_round_down(-1e-30) == (0x8001, False)
    assert codec.fp16_round_up(-1e-30) == (0x0000, False)      # -0 is stored as +0
    assert codec.fp16_round_down(-0.0) == (0x0000, False)
