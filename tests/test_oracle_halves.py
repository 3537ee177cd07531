"""Keys-only and values-only chunks in the oracle (Algorithm 1 counts the n key chunks and
the n value chunks as 2n units).  The pin: since every tile is encoded on its own, packing
the two halves of a document separately must give exactly the tile records that packing
the whole document gives, and loading the two halves must rebuild the same cache."""
import numpy as np
import pytest

from oracle import codec
from paper_2510_20878_amd import workloads as wl

FORMATS = [(16, 64), (8, 64), (4, 32), (43, 64), (52, 64), (143, 64)]


@pytest.mark.parametrize("bits,g", FORMATS)
def test_halves_are_the_tiles_of_the_whole(bits, g):
    L, H, D, T = 3, 2, 64, 37
    src = wl.kv_chunk(L, H, D, T, 5)
    whole, _ = codec.quantize_pack_chunk(src, bits, g)
    k, _ = codec.quantize_pack_half(src[:, 0], bits, g)
    v, _ = codec.quantize_pack_half(src[:, 1], bits, g)
    assert k.size == v.size == codec.half_bytes(L, H, D, T, bits, g)
    assert 2 * k.size == whole.size == codec.chunk_bytes(L, H, D, T, bits, g)
    rec = whole.size // (L * 2 * H)
    w = whole.reshape(L, 2, H, rec)
    assert np.array_equal(w[:, 0].ravel(), k)
    assert np.array_equal(w[:, 1].ravel(), v)


@pytest.mark.parametrize("bits,g", FORMATS)
def test_two_halves_load_like_the_whole(bits, g):
    L, H, D, T = 2, 3, 64, 21
    src = wl.kv_chunk(L, H, D, T, 9)
    whole, _ = codec.quantize_pack_chunk(src, bits, g)
    k, _ = codec.quantize_pack_half(src[:, 0], bits, g)
    v, _ = codec.quantize_pack_half(src[:, 1], bits, g)
    a = np.full((L, 2, H, T + 5, D), 0x7FC0, np.uint16)
    b = a.copy()
    codec.dequant_scatter_chunk(whole, (L, H, D), T, bits, g, a, 3)
    codec.dequant_scatter_half(k, (L, H, D), T, bits, g, 0, b, 3)
    assert np.array_equal(b[:, 1], np.full_like(b[:, 1], 0x7FC0))     # values untouched so far
    codec.dequant_scatter_half(v, (L, H, D), T, bits, g, 1, b, 3)
    assert np.array_equal(a, b)


def test_half_with_16_bits_is_a_copy_into_its_plane():
    L, H, D, T = 2, 2, 64, 16
    src = wl.kv_chunk(L, H, D, T, 1)
    v, _ = codec.quantize_pack_half(src[:, 1], 16, 64)
    out = np.zeros((L, 2, H, T, D), np.uint16)
    codec.dequant_scatter_half(v, (L, H, D), T, 16, 64, 1, out, 0)
    assert np.array_equal(out[:, 1], src[:, 1])
    assert not out[:, 0].any()


def test_request_with_keys_and_values_at_different_precision():
    """K at int8, V at int4 for every document, one whole 16-bit document in the middle:
    the result equals concatenating, per plane, what each unit decodes to alone."""
    L, H, D = 2, 2, 64
    Ts = [16, 24, 8]
    docs = [wl.kv_chunk(L, H, D, t, 20 + i) for i, t in enumerate(Ts)]
    packed, tokens, bits, parts = [], [], [], []
    for i, d in enumerate(docs):
        if i == 1:
            packed.append(codec.quantize_pack_chunk(d, 16, 64)[0]); tokens.append(Ts[i])
            bits.append(16); parts.append(0)
            continue
        packed.append(codec.quantize_pack_half(d[:, 0], 8, 64)[0]); tokens.append(Ts[i])
        bits.append(8); parts.append(1)
        packed.append(codec.quantize_pack_half(d[:, 1], 4, 64)[0]); tokens.append(Ts[i])
        bits.append(4); parts.append(2)
    order = [0, 1, 2, 3, 4]           # K0 V0 whole1 K2 V2
    out, offs = codec.load_chunks(packed, (L, H, D), tokens, bits, [64] * 5, order, parts=parts)
    assert offs == [0, 0, 16, 40, 40]
    assert out.shape[3] == sum(Ts)
    assert np.array_equal(out[:, :, :, 16:40], docs[1])
    for kv, b in ((0, 8), (1, 4)):
        alone = np.zeros((L, 2, H, 16, D), np.uint16)
        codec.dequant_scatter_chunk(codec.quantize_pack_chunk(docs[0], b, 64)[0], (L, H, D), 16, b, 64,
                                    alone, 0)
        assert np.array_equal(out[:, kv, :, 0:16], alone[:, kv])
    # the values of a document may come before its keys: planes fill independently
    out2, offs2 = codec.load_chunks(packed, (L, H, D), tokens, bits, [64] * 5, [1, 0, 2, 4, 3],
                                    parts=parts)
    assert offs2 == [0, 0, 16, 40, 40]
    assert np.array_equal(out, out2)


def test_request_errors_with_halves():
    L, H, D = 1, 1, 64
    d = wl.kv_chunk(L, H, D, 8, 3)
    k = codec.quantize_pack_half(d[:, 0], 8, 64)[0]
    w = codec.quantize_pack_chunk(d, 8, 64)[0]
    with pytest.raises(ValueError):        # keys without values
        codec.load_chunks([k], (L, H, D), [8], [8], [64], [0], parts=[1])
    with pytest.raises(ValueError):        # a whole chunk while the planes differ in length
        codec.load_chunks([k, w, k], (L, H, D), [8, 8, 8], [8, 8, 8], [64] * 3, [0, 1, 2], parts=[1, 0, 2])
    with pytest.raises(ValueError):
        out = np.zeros((L, 2, H, 8, D), np.uint16)
        codec.dequant_scatter_half(k, (L, H, D), 8, 8, 64, 2, out, 0)
