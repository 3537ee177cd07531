"""The load into a paged KV cache on the GPU against the oracle: every word of the page pool
identical (written rows and untouched rows alike)."""
import numpy as np
import pytest
import torch

from oracle import codec
from paper_2510_20878_amd import binding as B
from paper_2510_20878_amd import workloads as wl

pytestmark = pytest.mark.gpu

CANARY = 0x7FC1
ORC = {B.PREC_16: 16, B.PREC_INT8: 8, B.PREC_INT4: 4, B.PREC_FP8_E4M3: 43, B.PREC_FP8_E5M2: 52,
       B.PREC_GSE8: 143}


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the GPU"
    B.lib()
    yield
    torch.cuda.synchronize()


def dev_u8(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint8)).cuda()


def host_u16(t):
    return t.cpu().numpy().view(np.uint16)


def _case(shape, g, spec, order, P, layout, tok_base, seed, launch=None, extra_pages=3):
    """spec: (prec, n_tokens[, part]) per chunk.  Returns (got pool, ref pool, bad count)."""
    L, H, D = shape
    packed, parts = [], []
    for i, s_ in enumerate(spec):
        prec, t = s_[:2]
        part = s_[2] if len(s_) > 2 else B.PART_KV
        doc = wl.kv_chunk(L, H, D, t, seed * 31 + i)
        if part == B.PART_KV:
            packed.append(codec.quantize_pack_chunk(doc, ORC[prec], g)[0])
        else:
            packed.append(codec.quantize_pack_half(np.ascontiguousarray(doc[:, part - 1]), ORC[prec], g)[0])
        parts.append(part)
    tokens = [s_[1] for s_ in spec]
    total = tok_base + sum(tokens[c] for c in order if parts[c] != B.PART_V)
    need = -(-total // P)
    n_pages = need + extra_pages
    rng = np.random.default_rng(seed)
    table = rng.permutation(n_pages)[:need].astype(np.uint32)
    ref = np.full(L * 2 * H * n_pages * P * D, CANARY, np.uint16)
    codec.load_chunks_paged(packed, shape, tokens, [ORC[s_[0]] for s_ in spec], [g] * len(spec), order,
                            ref, layout, P, table.tolist(), tok_base=tok_base,
                            parts=parts if any(parts) else None)
    ctx = B.Context(L, H, D, max(tokens), group_int8=g, group_int4=g)
    if launch:
        ctx.set_launch_params(*launch)
    pool = torch.full((L * 2 * H * n_pages * P * D,), CANARY, dtype=torch.int16, device="cuda")
    tab = torch.from_numpy(table.view(np.int32)).cuda()
    bad = torch.zeros(1, dtype=torch.int32, device="cuda")
    cache = B.paged_cache(pool, tab, P, n_pages, layout, L, H, D, bad_pages=bad)
    dev = [dev_u8(p) for p in packed]
    ctx.load_packed_paged([(dev[c], tokens[c], spec[c][0], g, parts[c]) for c in order], cache, tok_base)
    torch.cuda.synchronize()
    ctx.destroy()
    return host_u16(pool), ref, int(bad.item())


ALL = [B.PREC_16, B.PREC_INT8, B.PREC_INT4, B.PREC_FP8_E4M3, B.PREC_FP8_E5M2, B.PREC_GSE8]


@pytest.mark.parametrize("layout", ["page_major", "tile_major"])
@pytest.mark.parametrize("P", [8, 16, 64])
def test_paged_load_all_tags_ragged_chunks(layout, P):
    spec = [(p, t) for p, t in zip(ALL, [37, 128, 5, 64, 99, 16])]
    got, ref, bad = _case((2, 2, 64), 64, spec, [5, 0, 3, 1, 4, 2], P, layout, tok_base=3, seed=P)
    assert bad == 0
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("launch", [(256, 2, 4, 0, 0), (1024, 4, 2, 1, 1), (64, 1, 4, 1, 0)])
def test_paged_load_launch_shapes_and_odd_head_dim(launch):
    # head_dim 96: a page of 8 rows is 1536 bytes, so runs of 1 KiB cross pages at every offset
    spec = [(B.PREC_INT4, 50), (B.PREC_16, 23), (B.PREC_INT8, 77), (B.PREC_GSE8, 31)]
    got, ref, bad = _case((1, 3, 96), 32, spec, [2, 0, 3, 1], 8, "page_major", tok_base=1, seed=2,
                          launch=launch)
    assert bad == 0
    assert np.array_equal(got, ref)


def test_paged_load_with_key_and_value_units():
    K, V = B.PART_K, B.PART_V
    spec = [(B.PREC_INT8, 40, K), (B.PREC_INT4, 40, V), (B.PREC_16, 9), (B.PREC_FP8_E4M3, 70, V),
            (B.PREC_INT8, 70, K)]
    got, ref, bad = _case((2, 2, 128), 128, spec, [0, 1, 2, 3, 4], 16, "tile_major", tok_base=0, seed=7)
    assert bad == 0
    assert np.array_equal(got, ref)


def test_page_ids_outside_the_pool_are_dropped_and_counted():
    L, H, D, g, P, T = 1, 2, 64, 64, 16, 64
    src = wl.kv_chunk(L, H, D, T, 3)
    packed = codec.quantize_pack_chunk(src, 8, g)[0]
    n_pages = 6
    table = np.array([4, 99, 1, 2], np.uint32)               # 99 is not a page of the pool
    ref = np.full(L * 2 * H * n_pages * P * D, CANARY, np.uint16)
    view = codec.paged_view(ref, "page_major", L, H, P, D)
    virt, _ = codec.load_chunks([packed], (L, H, D), [T], [8], [g], [0])
    for r in range(T):
        if table[r // P] < n_pages:
            view[table[r // P], :, :, :, r % P] = virt[:, :, :, r]
    ctx = B.Context(L, H, D, T, group_int8=g, group_int4=g)
    pool = torch.full((ref.size,), CANARY, dtype=torch.int16, device="cuda")
    bad = torch.zeros(1, dtype=torch.int32, device="cuda")
    tab = torch.from_numpy(table.view(np.int32)).cuda()      # must outlive the launch
    cache = B.paged_cache(pool, tab, P, n_pages, "page_major", L, H, D, bad_pages=bad)
    dev = dev_u8(packed)
    ctx.load_packed_paged([(dev, T, B.PREC_INT8, g)], cache)
    torch.cuda.synchronize()
    assert np.array_equal(host_u16(pool), ref)
    assert int(bad.item()) == L * 2 * H * P * D * 2 // 16   # one dropped 16-byte store per 8 words
    ctx.destroy()


@pytest.mark.parametrize("pinned_dma", [False, True])
def test_pool_load_into_a_paged_cache(pinned_dma):
    """ha_rag_load_chunks_paged: hot and cold chunks of three tags (pinned chunks read in place or
    through staging), promotion, then the same request again."""
    L, H, D, T, g, P = 2, 2, 64, 64, 64, 16
    n = 9
    precs_all = [B.PREC_INT4, B.PREC_INT8, B.PREC_FP8_E4M3]
    ctx = B.Context(L, H, D, T, group_int8=g, group_int4=g, tau_gpu_ppm=500_000, pinned_dma=pinned_dma)
    big = 0
    for p in precs_all:
        slot = (ctx.chunk_bytes(p, T) + 255) // 256 * 256
        big = max(big, slot)
        ctx.register_slab(B.TIER_HBM, p, torch.zeros(slot * 2, dtype=torch.uint8, device="cuda"))
        ctx.register_slab(B.TIER_PINNED, p, torch.zeros(slot * n, dtype=torch.uint8).pin_memory())
    ctx.register_staging(torch.zeros(big * 2, dtype=torch.uint8, device="cuda"))
    tokens = [T - 7 * (i % 3) for i in range(n)]
    precs = [precs_all[i % 3] for i in range(n)]
    packed = [codec.quantize_pack_chunk(wl.kv_chunk(L, H, D, tokens[i], 60 + i), ORC[precs[i]], g)[0]
              for i in range(n)]
    for i in range(n):
        ctx.pool_insert(i, precs[i], tokens[i], torch.from_numpy(packed[i]).pin_memory(), B.TIER_PINNED)
    ctx.set_counts(list(range(n)), [100 - i for i in range(n)])
    ctx.rerank()                                     # GPU_LIST = ids 0..3
    req = [5, 0, 2, 7, 1, 8]
    total = sum(tokens[c] for c in req)
    need = -(-total // P)
    n_pages = need + 2
    table = np.random.default_rng(0).permutation(n_pages)[:need].astype(np.uint32)
    ref = np.full(L * 2 * H * n_pages * P * D, CANARY, np.uint16)
    codec.load_chunks_paged(packed, (L, H, D), tokens, [ORC[p] for p in precs], [g] * n, req, ref,
                            "tile_major", P, table.tolist())
    tab = torch.from_numpy(table.view(np.int32)).cuda()
    for rnd in range(2):
        pool = torch.full((ref.size,), CANARY, dtype=torch.int16, device="cuda")
        cache = B.paged_cache(pool, tab, P, n_pages, "tile_major", L, H, D)
        st, tr = ctx.load_chunks_paged(req, cache, want_trace=True)
        torch.cuda.synchronize()
        assert np.array_equal(host_u16(pool), ref), rnd
        if rnd == 0:
            assert st["n_pinned_hits"] == 6 and [t.promoted for t in tr] == [0, 1, 1, 0, 1, 0]
        else:
            assert [t.found_tier for t in tr] == [B.TIER_PINNED, B.TIER_HBM, B.TIER_HBM, B.TIER_PINNED,
                                                  B.TIER_HBM, B.TIER_PINNED]
    ctx.destroy()


def test_llama3_8b_request_into_pages_sampled_rows_match_oracle():
    """The headline request (ten 512-token chunks, 2 x 16-bit + 3 x int8 + 5 x int4) into a
    page-major pool of 16-token pages; sampled (layer, head) tiles recomputed by the oracle
    and looked up through the page table."""
    L, H, D, T, g, P = 32, 8, 128, 512, 128, 16
    ctx = B.Context(L, H, D, T, group_int8=g, group_int4=g)
    precs = [B.PREC_16] * 2 + [B.PREC_INT8] * 3 + [B.PREC_INT4] * 5
    order = [4, 9, 0, 6, 2, 8, 1, 5, 3, 7]
    srcs, packs = [], []
    for i, p in enumerate(precs):
        s_ = wl.kv_chunk_device(L, H, D, T, 1500 + i)
        dst = torch.empty(ctx.chunk_bytes(p, T), dtype=torch.uint8, device="cuda")
        ctx.quantize_chunk(s_, T, p, g, dst)
        srcs.append(s_)
        packs.append(dst)
    need = 10 * T // P
    n_pages = need + 11
    rng = np.random.default_rng(4)
    table = rng.permutation(n_pages)[:need].astype(np.uint32)
    pool = torch.full((n_pages, L, 2, H, P, D), CANARY, dtype=torch.int16, device="cuda")
    bad = torch.zeros(1, dtype=torch.int32, device="cuda")
    tab = torch.from_numpy(table.view(np.int32)).cuda()
    cache = B.paged_cache(pool, tab, P, n_pages, "page_major", L, H, D, bad_pages=bad)
    ctx.load_packed_paged([(packs[c], T, precs[c], g) for c in order], cache)
    torch.cuda.synchronize()
    assert int(bad.item()) == 0
    unused = sorted(set(range(n_pages)) - set(table.tolist()))
    assert bool((pool[unused] == np.int16(np.uint16(CANARY).view(np.int16))).all())
    tab_l = torch.from_numpy(table.astype(np.int64)).cuda()
    for pos, c in enumerate(order):
        pages = tab_l[pos * T // P:(pos + 1) * T // P]
        for _ in range(2):
            l, h = int(rng.integers(L)), int(rng.integers(H))
            got = host_u16(pool[pages, l, :, h].permute(1, 0, 2, 3).reshape(2, T, D).contiguous())
            src_kv = host_u16(srcs[c][l, :, h].contiguous().view(torch.int16)).reshape(1, 2, 1, T, D)
            ref_pack, _ = codec.quantize_pack_chunk(src_kv, ORC[precs[c]], g)
            ref_out = np.zeros((1, 2, 1, T, D), np.uint16)
            codec.dequant_scatter_chunk(ref_pack, (1, 1, D), T, ORC[precs[c]], g, ref_out, 0)
            assert np.array_equal(got, ref_out[0, :, 0])
    ctx.destroy()
