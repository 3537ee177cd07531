"""The oracle's paged-cache scatter.  Pins: with an identity page table the tile-major pool
IS the contiguous cache; a permuted table equals numpy's take along the page axis; both
layouts hold the same rows; rows outside the request keep their contents."""
import numpy as np
import pytest

from oracle import codec
from paper_2510_20878_amd import workloads as wl

L, H, D, G = 2, 2, 64, 64


def _request(seed=0):
    tokens = [37, 16, 50]
    bits = [8, 16, 4]
    packed = [codec.quantize_pack_chunk(wl.kv_chunk(L, H, D, t, seed + i), b, G)[0]
              for i, (t, b) in enumerate(zip(tokens, bits))]
    return packed, tokens, bits


@pytest.mark.parametrize("P", [8, 16, 64])
def test_identity_table_tile_major_is_the_contiguous_cache(P):
    packed, tokens, bits = _request()
    order = [2, 0, 1]
    total = sum(tokens)
    n_pages = -(-total // P)
    ref, _ = codec.load_chunks(packed, (L, H, D), tokens, bits, [G] * 3, order, cap_tokens=n_pages * P)
    pages = np.zeros(L * 2 * H * n_pages * P * D, np.uint16)
    codec.load_chunks_paged(packed, (L, H, D), tokens, bits, [G] * 3, order, pages, "tile_major", P,
                            list(range(n_pages)))
    assert np.array_equal(pages.reshape(L, 2, H, n_pages * P, D), ref)


@pytest.mark.parametrize("layout", ["tile_major", "page_major"])
def test_permuted_table_is_a_take_along_the_page_axis(layout):
    P = 16
    packed, tokens, bits = _request(3)
    order = [1, 2, 0]
    total = sum(tokens)
    need = -(-total // P)
    n_pages = need + 5
    rng = np.random.default_rng(1)
    table = rng.permutation(n_pages)[:need].tolist()
    ref, _ = codec.load_chunks(packed, (L, H, D), tokens, bits, [G] * 3, order, cap_tokens=need * P)
    canary = 0x7FC1
    pages = np.full(L * 2 * H * n_pages * P * D, canary, np.uint16)
    codec.load_chunks_paged(packed, (L, H, D), tokens, bits, [G] * 3, order, pages, layout, P, table)
    view = codec.paged_view(pages, layout, L, H, P, D)            # [page][l][kv][h][row][d]
    got = np.take(view, table, axis=0)                             # request order
    got = got.transpose(1, 2, 3, 0, 4, 5).reshape(L, 2, H, need * P, D)
    assert np.array_equal(got[:, :, :, :total], ref[:, :, :, :total])
    assert np.all(got[:, :, :, total:] == canary)                  # tail of the last page untouched
    unused = [p for p in range(n_pages) if p not in table]
    assert np.all(view[unused] == canary)


def test_both_layouts_hold_the_same_rows_and_tok_base_skips_rows():
    P = 8
    packed, tokens, bits = _request(5)
    order = [0, 1]
    base = 11
    total = base + tokens[0] + tokens[1]
    need = -(-total // P)
    table = list(range(need))[::-1]
    a = np.full(L * 2 * H * need * P * D, 0x7FC1, np.uint16)
    b = a.copy()
    offs = codec.load_chunks_paged(packed, (L, H, D), tokens, bits, [G] * 3, order, a, "tile_major", P,
                                   table, tok_base=base)
    codec.load_chunks_paged(packed, (L, H, D), tokens, bits, [G] * 3, order, b, "page_major", P, table,
                            tok_base=base)
    assert offs == [11, 48]
    va, vb = codec.paged_view(a, "tile_major", L, H, P, D), codec.paged_view(b, "page_major", L, H, P, D)
    assert np.array_equal(va, vb)
    # rows 0..10 of the request (page table[0], rows 0..7 and table[1], rows 0..2) were not written
    assert np.all(va[table[0]] == 0x7FC1) and np.all(va[table[1], :, :, :, :3] == 0x7FC1)
    assert not np.any(va[table[1], :, :, :, 3:] == 0x7FC1)
    with pytest.raises(ValueError):
        codec.load_chunks_paged(packed, (L, H, D), tokens, bits, [G] * 3, order, a, "tile_major", P,
                                table[:-1], tok_base=base)
