"""Pins for the packed-chunk layout of the oracle: closed-form sizes, the paper's
storage arithmetic, bijectivity, and the property the layout exists for -- a
64-lane wave that reads consecutive 16-byte words emits consecutive 16-byte
stores."""
import json
import os

import numpy as np
import pytest

from oracle import codec
from paper_2510_20878_amd import workloads as wl

MiB = 1 << 20


def test_paper_storage_example(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "paper_values.json")))["storage_example"]
    # the paper's chunk is K or V alone; a chunk here is K and V of one document
    ours = codec.chunk_bytes(g["layers"], g["heads"], g["head_dim"], g["tokens_per_chunk"], 16)
    assert ours == 2 * 128 * MiB
    assert ours // 2 * g["chunks"] == g["total_gib"] << 30


@pytest.mark.parametrize("shape,T,bits,grp,expect", [
    ((32, 8, 128), 512, 16, 128, 64 * MiB),
    ((32, 8, 128), 512, 8, 128, 33 * MiB),
    ((32, 8, 128), 512, 4, 128, 17 * MiB),
    ((32, 8, 128), 512, 4, 64, 18 * MiB),
    ((32, 8, 128), 1024, 4, 64, 36 * MiB),
    ((80, 8, 128), 1024, 8, 128, 165 * MiB),
    ((80, 8, 128), 1024, 4, 128, 85 * MiB),
    ((2, 2, 64), 128, 16, 64, 128 << 10),
    ((2, 2, 64), 128, 8, 64, 68 << 10),
    ((2, 2, 64), 128, 4, 64, 36 << 10),
])
def test_chunk_sizes_closed_form(shape, T, bits, grp, expect):
    L, H, D = shape
    assert codec.chunk_bytes(L, H, D, T, bits, grp) == expect
    E = L * 2 * H * T * D
    if bits != 16:
        assert expect == E * bits // 8 + 4 * (E // grp)       # payload + 4 bytes per group


def test_compression_ratios(golden_dir):
    gold = json.load(open(os.path.join(golden_dir, "paper_values.json")))["compression_ratio_8bit"]
    full = codec.chunk_bytes(32, 8, 128, 512, 16)
    r = {(b, g): full / codec.chunk_bytes(32, 8, 128, 512, b, g) for b in (8, 4) for g in (64, 128)}
    assert r[(8, 128)] == pytest.approx(2 / (1 + 4 / 128))      # 1.9394
    assert r[(4, 128)] == pytest.approx(2 / (0.5 + 4 / 128))    # 3.7647
    assert r[(8, 64)] == pytest.approx(1.8824, abs=1e-4)
    assert r[(4, 64)] == pytest.approx(3.5556, abs=1e-4)
    assert r[(8, 128)] < gold["upper_bound"]                   # any 8-bit format is below 2


def test_ragged_tile_is_padded_to_whole_blocks():
    # 100 tokens x 64 = 6400 elements = 3.125 blocks -> 4 blocks
    assert codec.tile_payload_bytes(100, 64, 4) == 4 * 1024
    assert codec.tile_meta_bytes(100, 64, 4, 64) == 4 * 32 * 4
    assert codec.chunk_bytes(2, 2, 64, 100, 4, 64) == 8 * (4096 + 512)
    assert codec.chunk_bytes(2, 2, 64, 0, 4, 64) == 0
    assert codec.chunk_bytes(2, 2, 60, 100, 4, 64) == 0        # head_dim not a multiple of 8
    assert codec.chunk_bytes(2, 2, 64, 100, 4, 128) == 0       # group does not divide head_dim
    src = wl.kv_chunk(2, 2, 64, 100, 3)
    packed, _ = codec.quantize_pack_chunk(src, 4, 64)
    tile = packed.reshape(8, 4096 + 512)
    used = 6400 - 3 * 2048                                     # elements in the last block: 256
    last = tile[:, 3 * 1024:4 * 1024].reshape(8, 64, 16)       # [lane][16 bytes = 4 planes x 4 B]
    # plane 0 holds elements 0..511 of the block: lanes 0..31 used, the rest and planes 1..3 zero
    assert used == 256
    assert not last[:, 32:, :].any() and not last[:, :, 4:].any()
    meta_last = tile[:, 4096 + 3 * 128:].reshape(8, 8, 4, 4)    # [rho][plane][4 bytes]
    assert not meta_last[:, :, 1:, :].any() and not meta_last[:, 4:, 0, :].any()
    out = np.zeros((2, 2, 2, 100, 64), np.uint16)
    codec.dequant_scatter_chunk(packed, (2, 2, 64), 100, 4, 64, out, 0)
    x, y = wl.bf16_words_to_f32(src), wl.bf16_words_to_f32(out)
    assert np.abs(x - y).max() < 8.0 and np.abs(x - y).mean() < 0.5


# an independent statement of the layout, straight from its definition ----------------
def _octet_offset(e, bits):
    k, r = divmod(e, 2048)
    j, i = r // 512, (r % 512) // 8
    P = 16 // bits
    return k * 256 * bits + (j // P) * 1024 + i * 16 + (j % P) * bits


@pytest.mark.parametrize("bits", [4, 8, 16])
def test_octets_tile_the_payload_exactly(bits):
    n_e = 3 * 2048
    seen = np.zeros(n_e * bits // 8, np.int32)
    for e in range(0, n_e, 8):
        o = codec.octet_offset(e, bits)
        assert o == _octet_offset(e, bits)
        assert all(codec.octet_offset(e + p, bits) == o for p in range(8))
        seen[o:o + bits] += 1
    assert np.all(seen == 1)


@pytest.mark.parametrize("g", [32, 64, 128, 256, 512])
def test_meta_entries_tile_the_meta_block_exactly(g):
    n_e = 2 * 2048
    per_block = 2048 // g
    seen = np.zeros(2 * per_block, np.int32)
    for e in range(0, n_e, g):
        o = codec.meta_offset(e, g)
        assert o % 4 == 0 and all(codec.meta_offset(e + p, g) == o for p in range(0, g, 8))
        seen[o // 4] += 1
    assert np.all(seen == 1)


def _coded_chunk(bits, g, T, D, rng):
    """BF16 source whose groups have zero 0 and scale 1, so code == value."""
    qmax = (1 << bits) - 1
    v = rng.integers(0, qmax + 1, (1, 2, 1, T, D)).astype(np.float32)
    v = v.reshape(1, 2, 1, T, D // g, g)
    v[..., 0], v[..., 1] = 0, qmax
    return v.reshape(1, 2, 1, T, D)


@pytest.mark.parametrize("bits,g,D", [(4, 64, 64), (4, 128, 128), (8, 64, 128), (8, 32, 64),
                                      (8, 256, 256), (4, 32, 96), (4, 256, 256), (8, 512, 512),
                                      (4, 512, 512)])
def test_wave_view_consecutive_words_give_consecutive_stores(bits, g, D):
    """Simulate what the layout is for.  Lane i of a 64-lane wave reads 16-byte
    word i of each 1024-byte slab of a block; octet number w of what the lane has
    read so far belongs to plane j = w, whose 16-byte store goes to byte
    j*1024 + i*16 of the block's 4096 output bytes.  The scale/zero the lane needs
    for plane j is entry j of the 16-byte meta word number (8*i) // g."""
    rng = np.random.default_rng(bits * 100 + g)
    T = 48 if D != 96 else 64
    vals = _coded_chunk(bits, g, T, D, rng)
    # give every group its own zero so that a wrong meta entry shows
    zero = rng.integers(-64, 1 if bits == 8 else 64, (1, 2, 1, T, D // g)).astype(np.float32)  # stays BF16-exact
    src = wl.f32_to_bf16_words((vals.reshape(1, 2, 1, T, D // g, g) + zero[..., None])
                               .reshape(1, 2, 1, T, D))
    packed, sat = codec.quantize_pack_chunk(src, bits, g)
    assert sat == 0
    n_e = T * D
    nblk = -(-n_e // 2048)
    pay, met = nblk * 256 * bits, nblk * (2048 // g) * 4
    P = 16 // bits
    for tile in range(2):
        rec = packed[tile * (pay + met):(tile + 1) * (pay + met)]
        out = np.zeros(nblk * 2048, np.float32)
        for k in range(nblk):
            blk = rec[k * 256 * bits:(k + 1) * 256 * bits]
            mblk = rec[pay + k * (2048 // g) * 4: pay + (k + 1) * (2048 // g) * 4]
            for i in range(64):
                mword = mblk[((8 * i) // g) * 16:((8 * i) // g) * 16 + 16] if g <= 512 else None
                for a in range(4 // P):                       # 16-byte loads of this lane
                    word = blk[a * 1024 + i * 16: a * 1024 + i * 16 + 16]
                    for w in range(P):
                        j = a * P + w
                        octet = word[w * bits:(w + 1) * bits]
                        if bits == 8:
                            q = octet.astype(np.float32)
                        else:
                            q = np.stack([octet & 15, octet >> 4], 1).reshape(8).astype(np.float32)
                        entry = mword[4 * j:4 * j + 4]
                        s = float(entry[:2].copy().view(np.float16)[0])
                        z = float(entry[2:].copy().view(np.float16)[0])
                        out[k * 2048 + j * 512 + i * 8: k * 2048 + j * 512 + i * 8 + 8] = q * s + z
        ref = wl.bf16_words_to_f32(src).reshape(2, n_e)[tile]
        assert np.array_equal(out[:n_e], ref)
        assert not out[n_e:].any()


def test_16bit_payload_is_the_source_bytes_in_order():
    src = wl.kv_chunk(1, 2, 64, 40, 9)                        # 2560 elements per tile
    packed, _ = codec.quantize_pack_chunk(src, 16)
    rec = packed.reshape(4, 2 * 4096)
    flat = src.reshape(4, 2560)
    assert np.array_equal(rec[:, :5120].copy().view(np.uint16), flat)
    assert not rec[:, 5120:].any()


def test_pack_unpack_every_byte_value_and_nibble_position():
    # int8: all 256 byte values; int4: each of the 32 nibble positions of a 16-byte word
    L, H, D, T = 1, 1, 256, 8
    v = np.tile(np.arange(256, dtype=np.float32), (1, 2, 1, T, 1))
    src = wl.f32_to_bf16_words(v)
    packed, _ = codec.quantize_pack_chunk(src, 8, 256)
    assert set(packed[:2048].tolist()) == set(range(256))
    codes, _, _ = codec.unpack_chunk(packed, (L, H, D), T, 8, 256)
    assert np.array_equal(codes, v.astype(np.uint8))
    for pos in range(32):
        v4 = np.zeros((1, 2, 1, 16, 128), np.float32)
        v4[..., 1] = 15                                        # every group: min 0, max 15
        # element whose code lands in nibble `pos` of lane 0's word: plane pos//8, position pos%8
        e = (pos // 8) * 512 + pos % 8
        t, d = divmod(e, 128)
        if d != 1:
            v4[0, 0, 0, t, d] = 9
        packed, _ = codec.quantize_pack_chunk(wl.f32_to_bf16_words(v4), 4, 128)
        word = packed[:16]
        nib = (word[pos // 2] >> (4 * (pos % 2))) & 15
        assert nib == (15 if d == 1 else 9), pos
