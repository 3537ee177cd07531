"""Host logic of the library without a GPU (dry_run contexts: bookkeeping only,
no HIP call, no byte moved): sizes, Algorithm 1 split, Algorithm 2 lookup /
promotion / LRU against the oracle's plain-Python simulation, error codes."""
import numpy as np
import pytest

from oracle import codec, placement as pl
from paper_2510_20878_amd import binding as B
from paper_2510_20878_amd import workloads as wl

# the oracle's name for each storage format
ORC = {B.PREC_16: 16, B.PREC_INT8: 8, B.PREC_INT4: 4, B.PREC_FP8_E4M3: 43, B.PREC_FP8_E5M2: 52,
       B.PREC_GSE8: 143}
FAKE_HBM = 0x7F0000000000     # never dereferenced in dry_run
FAKE_PIN = 0x7E0000000000
FAKE_STG = 0x7D0000000000


@pytest.mark.parametrize("shape", [(32, 8, 128), (80, 8, 128), (2, 2, 64), (1, 1, 96)])
@pytest.mark.parametrize("T", [1, 7, 100, 128, 512, 1024])
def test_chunk_bytes_equals_oracle(shape, T):
    L, H, D = shape
    for prec, bits in ORC.items():
        for g in (32, 64, 128):
            if D % g:
                with pytest.raises(B.HaRagError) as e:
                    B.ha_rag_chunk_bytes(L, H, D, B.PREC_INT4, g, T)
                assert e.value.code == B.EFORMAT
                continue
            pay, meta, total = B.ha_rag_chunk_bytes(L, H, D, prec, g, T)
            assert total == codec.chunk_bytes(L, H, D, T, bits, g)
            assert pay == L * 2 * H * codec.tile_payload_bytes(T, D, bits)
            assert pay + meta == total
            assert (meta == 0) == (prec in (B.PREC_16, B.PREC_FP8_E4M3, B.PREC_FP8_E5M2))
            if prec == B.PREC_GSE8:
                assert meta == 16 * L * 2 * H


def test_chunk_bytes_rejects_bad_shapes():
    for args in [(2, 2, 60, B.PREC_INT4, 64, 8), (2, 2, 64, 7, 64, 8), (2, 2, 64, B.PREC_INT8, 48, 8),
                 (0, 2, 64, B.PREC_16, 0, 8)]:
        with pytest.raises(B.HaRagError) as e:
            B.ha_rag_chunk_bytes(*args)
        assert e.value.code == B.EFORMAT


def test_alg1_classes_equal_oracle():
    rng = np.random.default_rng(0)
    for n in (1, 2, 9, 10, 38, 257, 1000):
        af = rng.integers(0, 12, n).tolist()         # many ties
        for taus in ([100_000, 100_000, 100_000], [200_000, 300_000], [999_999], []):
            cls, ranks = B.ha_rag_alg1_classes(af, taus)
            assert cls == pl.classes_by_rank(af, taus)
            assert ranks == pl.ranks(af)


def _ctx(cap_hbm, n_pinned, tau_gpu_ppm, L=2, H=2, D=64, T=128, prec=B.PREC_INT4, staging=4,
         rerank_interval=0):
    ctx = B.Context(L, H, D, T, group_int8=64, group_int4=64, tau_gpu_ppm=tau_gpu_ppm,
                    rerank_interval=rerank_interval, dry_run=True)
    slot = (ctx.chunk_bytes(prec, T) + 255) // 256 * 256
    if cap_hbm:
        ctx.register_slab(B.TIER_HBM, prec, FAKE_HBM, slot * cap_hbm)
    ctx.register_slab(B.TIER_PINNED, prec, FAKE_PIN, slot * n_pinned)
    if staging:
        ctx.register_staging(FAKE_STG, slot * staging)
    return ctx


def test_alg2_two_tier_trace_equals_oracle():
    """Every chunk has a pinned master; GPU_LIST = hottest 10 %; HBM holds 3."""
    n, cap = 50, 3
    ctx = _ctx(cap, n, 100_000)
    for c in range(n):
        ctx.pool_insert(c, B.PREC_INT4, 128, None, B.TIER_PINNED)
    counts = [1000 - c for c in range(n)]            # rank == id
    ctx.set_counts(list(range(n)), counts)
    ctx.rerank()
    assert [ctx.get_rank(c) for c in (0, 7, 49)] == [0, 7, 49]
    sim = pl.TierSim(list(range(n)), [100_000, 900_000, 0], (cap, None, 0))
    sim.seed(sim.PIN, range(n))
    rng = np.random.default_rng(1)
    seq = [0, 1, 2, 3, 0, 7, 4, 1, 2, 2, 30, 0] + rng.integers(0, 8, 200).tolist()
    for c in seq:                                     # one chunk per load call
        st, tr = ctx.load_chunks([c], FAKE_HBM, 128, want_trace=True)
        tier, placed = sim.access(c)
        assert tr[0].found_tier == (B.TIER_HBM if tier == sim.GPU else B.TIER_PINNED)
        assert bool(tr[0].promoted) == bool(placed)
        exp_ev = placed[0][1] if placed and placed[0][1] is not None else B.NO_CHUNK
        assert tr[0].evicted_id == exp_ev
        assert ctx.pool_hbm_lru() == sim.resident(sim.GPU)
        assert st["n_hbm_hits"] + st["n_pinned_hits"] == 1
    # counters moved with every access; ranks did not (no rerank since)
    assert ctx.pool_query(0).count == counts[0] + seq.count(0)
    assert ctx.get_rank(7) == 7


def test_multi_chunk_request_bookkeeping_and_offsets():
    n = 20
    ctx = _ctx(8, n, 500_000)
    toks = [128 - 3 * c for c in range(n)]
    for c in range(n):
        ctx.pool_insert(c, B.PREC_INT4, toks[c], None, B.TIER_PINNED)
    ctx.set_counts(list(range(n)), [100 - c for c in range(n)])
    ctx.rerank()
    sim = pl.TierSim(list(range(n)), [500_000, 500_000, 0], (8, None, 0))
    sim.seed(sim.PIN, range(n))
    req = [3, 0, 15, 2, 1, 3, 12]
    st, tr = ctx.load_chunks(req, FAKE_HBM, 1000, tok_base=11, want_trace=True)
    off = 11
    for i, c in enumerate(req):
        tier, placed = sim.access(c)
        assert tr[i].tok_off == off
        assert tr[i].found_tier == (B.TIER_HBM if tier == sim.GPU else B.TIER_PINNED)
        assert bool(tr[i].promoted) == bool(placed)
        off += toks[c]
    assert st["tokens"] == sum(toks[c] for c in req)
    assert st["n_promoted"] == 4 and st["n_hbm_hits"] == 1 and st["n_pinned_hits"] == 6
    per_tok = 2 * 2 * 2 * 64 * 2
    assert st["bf16_bytes_written"] == st["tokens"] * per_tok
    assert st["packed_bytes_read"] == sum(ctx.chunk_bytes(B.PREC_INT4, toks[c]) for c in req)
    assert st["bytes_h2d"] == sum(ctx.chunk_bytes(B.PREC_INT4, toks[c]) for c in req) - \
        ctx.chunk_bytes(B.PREC_INT4, toks[3])
    assert ctx.pool_hbm_lru() == sim.resident(sim.GPU)
    # launches: one for the chunks read where they lie (15 and 12 stay in pinned memory), one per
    # promoted chunk (through staging), one for the repeat of 3
    assert st["n_kernel_launches"] == 1 + 4 + 1


def test_hbm_only_chunks_are_never_evicted_and_promotion_is_skipped():
    ctx = _ctx(2, 10, 1_000_000)
    ctx.pool_insert(100, B.PREC_INT4, 128, None, B.TIER_HBM)       # no pinned master
    ctx.pool_insert(101, B.PREC_INT4, 128, None, B.TIER_HBM)
    ctx.pool_insert(5, B.PREC_INT4, 128, None, B.TIER_PINNED)
    ctx.rerank()
    st, tr = ctx.load_chunks([5], FAKE_HBM, 128, want_trace=True)
    assert tr[0].promote_skipped == 1 and tr[0].promoted == 0 and st["n_promote_skipped"] == 1
    with pytest.raises(B.HaRagError) as e:
        ctx.pool_insert(102, B.PREC_INT4, 128, None, B.TIER_HBM)
    assert e.value.code == B.ENOSPC
    with pytest.raises(B.HaRagError) as e:
        ctx.pool_evict(100)
    assert e.value.code == B.EINVAL
    # once a master exists the copy becomes evictable
    ctx.pool_insert(100, B.PREC_INT4, 128, None, B.TIER_PINNED)
    st, tr = ctx.load_chunks([5], FAKE_HBM, 128, want_trace=True)
    assert tr[0].promoted == 1 and tr[0].evicted_id == 100


def test_rerank_interval_and_gpu_list_boundary():
    n = 10
    ctx = _ctx(4, n, 200_000, rerank_interval=3)          # GPU_LIST = 2 hottest
    for c in range(n):
        ctx.pool_insert(c, B.PREC_INT4, 128, None, B.TIER_PINNED)
    # no rank yet: nothing is promoted
    st, _ = ctx.load_chunks([9], FAKE_HBM, 128)
    assert st["n_promoted"] == 0
    ctx.load_chunks([9], FAKE_HBM, 128)
    ctx.load_chunks([8], FAKE_HBM, 128)
    # 4th call: automatic rerank first -> 9 (2 hits) rank 0, 8 rank 1
    st, tr = ctx.load_chunks([8], FAKE_HBM, 128, want_trace=True)
    assert ctx.get_rank(9) == 0 and ctx.get_rank(8) == 1 and ctx.get_rank(0) == 2
    assert tr[0].promoted == 1
    st, _ = ctx.load_chunks([0], FAKE_HBM, 128)
    assert st["n_promoted"] == 0                      # rank 2 is outside GPU_LIST


def test_error_paths_change_nothing():
    ctx = _ctx(2, 4, 1_000_000)
    for c in range(3):
        ctx.pool_insert(c, B.PREC_INT4, 128, None, B.TIER_PINNED)
    ctx.rerank()

    def code(fn, *a, **k):
        with pytest.raises(B.HaRagError) as e:
            fn(*a, **k)
        return e.value.code

    assert code(ctx.load_chunks, [0, 77], FAKE_HBM, 1000) == B.ENOENT
    assert code(ctx.load_chunks, [0, 1], FAKE_HBM, 255) == B.ENOSPC          # cache too small
    assert code(ctx.load_chunks, [0, 1], FAKE_HBM, 300, tok_base=50) == B.ENOSPC
    assert code(ctx.load_chunks, [0], FAKE_HBM, 128, tags=[B.PREC_INT8]) == B.EFORMAT
    assert code(ctx.load_chunks, [0], FAKE_HBM + 8, 128) == B.EINVAL         # misaligned cache
    assert code(ctx.pool_insert, 0, B.PREC_INT4, 128, None, B.TIER_PINNED) == B.EINVAL   # duplicate
    assert code(ctx.pool_insert, 0, B.PREC_INT4, 64, None, B.TIER_HBM) == B.EFORMAT     # other length
    assert code(ctx.pool_insert, 9, B.PREC_INT8, 128, None, B.TIER_PINNED) == B.ENOSPC  # no such slab
    assert code(ctx.pool_insert, 9, B.PREC_INT4, 129, None, B.TIER_PINNED) == B.EINVAL  # too long
    ctx.pool_insert(3, B.PREC_INT4, 128, None, B.TIER_PINNED)
    assert code(ctx.pool_insert, 4, B.PREC_INT4, 128, None, B.TIER_PINNED) == B.ENOSPC  # slab full
    assert code(ctx.pool_promote, 77) == B.ENOENT
    assert code(ctx.pool_slot, 0, B.TIER_HBM) == B.ENOENT
    assert code(ctx.touch, [0, 77]) == B.ENOENT
    for c in range(3):
        q = ctx.pool_query(c)
        assert q.count == 0 and q.in_hbm == 0         # failed calls counted nothing, moved nothing
    ptr, nbytes = ctx.pool_slot(1, B.TIER_PINNED)
    slot = (nbytes + 255) // 256 * 256
    assert nbytes == codec.chunk_bytes(2, 2, 64, 128, 4, 64) and (ptr - FAKE_PIN) % slot == 0
    # cold chunk without a staging area
    ctx2 = _ctx(2, 4, 0, staging=0)
    ctx2.pool_insert(0, B.PREC_INT4, 128, None, B.TIER_PINNED)
    assert code(ctx2.load_chunks, [0], FAKE_HBM, 128) == B.ENOSPC
    assert code(B.Context, 2, 2, 60, 128, dry_run=True) == B.EFORMAT
    assert code(B.Context, 2, 2, 64, 128, group_int4=128, dry_run=True) == B.EFORMAT


def test_batch_load_bookkeeping():
    n = 12
    ctx = _ctx(12, n, 1_000_000)
    for c in range(n):
        ctx.pool_insert(c, B.PREC_INT4, 128, None, B.TIER_PINNED)
    ctx.rerank()
    reqs = [[0, 1, 2], [3, 1], [], [4, 5, 6, 0]]
    st, tr = ctx.load_batch(reqs, [FAKE_HBM + 4096 * i for i in range(4)], [384, 256, 0, 600],
                            tok_base=[0, 0, 0, 88], want_trace=True)
    assert [t.tok_off for t in tr] == [0, 128, 256, 0, 128, 88, 216, 344, 472]
    assert [t.found_tier for t in tr] == [1, 1, 1, 1, 0, 1, 1, 1, 0]   # repeats hit HBM
    assert st["n_promoted"] == 7 and st["tokens"] == 9 * 128
    with pytest.raises(B.HaRagError) as e:
        ctx.load_batch([[0, 1, 2]], [FAKE_HBM], [383])
    assert e.value.code == B.ENOSPC


def test_zipf_workload_hit_rate_is_high_once_warm():
    """The placement the paper motivates: with ~1 % of ids drawing most accesses,
    an HBM tier holding the hottest few percent serves most chunk loads."""
    n = 2000
    ctx = _ctx(100, n, 50_000)                      # tau_GPU = 5 % (the paper's setting)
    for c in range(n):
        ctx.pool_insert(c, B.PREC_INT4, 128, None, B.TIER_PINNED)
    reqs = wl.zipf_requests(n, 600, 8, seed=3)
    for r in reqs[:300]:
        ctx.load_chunks(r.tolist(), FAKE_HBM, 8 * 128)
    ctx.rerank()
    hits = tot = 0
    for r in reqs[300:]:
        st, _ = ctx.load_chunks(r.tolist(), FAKE_HBM, 8 * 128)
        hits += st["n_hbm_hits"]
        tot += 8
    assert hits / tot > 0.6


def test_chunk_hit_early_in_a_call_may_be_evicted_later_in_the_same_call():
    """Algorithm 2 handles the chunks of a request one after another: a chunk served
    from HBM at the start of a request can be the LRU victim of a promotion further
    down the same request.  The early read keeps the slot it was decided for."""
    n = 6
    ctx = _ctx(2, n, 1_000_000)
    for c in range(n):
        ctx.pool_insert(c, B.PREC_INT4, 128, None, B.TIER_PINNED)
    ctx.rerank()
    ctx.load_chunks([0, 1], FAKE_HBM, 256)               # both promoted, slab full
    sim = pl.TierSim(list(range(n)), [1_000_000, 0, 0], (2, None, 0))
    sim.seed(sim.PIN, range(n))
    for c in (0, 1):
        sim.access(c)
    st, tr = ctx.load_chunks([0, 1, 2, 0], FAKE_HBM, 512, want_trace=True)
    exp = [sim.access(c) for c in (0, 1, 2, 0)]
    # 2 evicts 0 (least recent); the last 0 is cold again and evicts 1
    assert [t.found_tier for t in tr] == [0, 0, 1, 1]
    assert [t.evicted_id for t in tr] == [B.NO_CHUNK, B.NO_CHUNK, 0, 1]
    assert [e[0] for e in exp] == [sim.GPU, sim.GPU, sim.PIN, sim.PIN]
    assert ctx.pool_hbm_lru() == sim.resident(sim.GPU) == [2, 0]
    assert st["n_kernel_launches"] == 1 + 2              # one for the early hits, one per cold chunk


def test_copy_made_by_a_call_is_not_dropped_by_the_same_call():
    """Where this library departs from plain LRU: with fewer slots than a request
    promotes, the later promotions are skipped instead of evicting copies that the
    same call has just made (and may still be about to read)."""
    ctx = _ctx(2, 6, 1_000_000)
    for c in range(6):
        ctx.pool_insert(c, B.PREC_INT4, 128, None, B.TIER_PINNED)
    ctx.rerank()
    st, tr = ctx.load_chunks([0, 1, 2, 1, 3], FAKE_HBM, 5 * 128, want_trace=True)
    assert [t.promoted for t in tr] == [1, 1, 0, 0, 0]
    assert [t.promote_skipped for t in tr] == [0, 0, 1, 0, 1]
    assert tr[3].found_tier == B.TIER_HBM                # the repeat of 1 reads the new copy
    assert ctx.pool_hbm_lru() == [0, 1]


def test_limits_are_rejected_not_wrapped():
    # element indices inside a tile are 32-bit: tokens * head_dim must stay below 2^31
    with pytest.raises(B.HaRagError) as e:
        B.ha_rag_chunk_bytes(1, 1, 128, B.PREC_INT4, 128, 2**24)
    assert e.value.code == B.EINVAL
    with pytest.raises(B.HaRagError) as e:
        B.Context(1, 1, 128, 2**24, dry_run=True)
    assert e.value.code == B.EINVAL
    pay, meta, total = B.ha_rag_chunk_bytes(1, 1, 128, B.PREC_INT4, 128, 2**24 - 1)
    assert total == codec.chunk_bytes(1, 1, 128, 2**24 - 1, 4, 128)
    # a request may list at most 4096 chunks
    ctx = _ctx(2, 4, 0)
    ctx.pool_insert(0, B.PREC_INT4, 128, None, B.TIER_HBM)
    st, _ = ctx.load_chunks([0] * 4096, FAKE_HBM, 4096 * 128)
    assert st["tokens"] == 4096 * 128 and st["n_kernel_launches"] == 64
    with pytest.raises(B.HaRagError) as e:
        ctx.load_chunks([0] * 4097, FAKE_HBM, 4097 * 128)
    assert e.value.code == B.EINVAL
    st, _ = ctx.load_chunks([], FAKE_HBM, 0)              # an empty request is legal
    assert st["n_chunks"] == 0 and st["n_kernel_launches"] == 0


# ---- four tiers (Algorithm 2 in full) -------------------------------------------------
FAKE_PAGE = 0x7C0000000000
FAKE_BNC = 0x7B0000000000


def _ctx4(n, caps, taus, prec=B.PREC_INT4, T=128, rerank_interval=0):
    """Every chunk lives on disk; HBM / pinned / pageable hold caps[0..2] chunks."""
    ctx = B.Context(2, 2, 64, T, group_int8=64, group_int4=64, tau_gpu_ppm=taus[0],
                    tau_pin_ppm=taus[1], tau_page_ppm=taus[2], rerank_interval=rerank_interval,
                    dry_run=True)
    slot = (ctx.chunk_bytes(prec, T) + 255) // 256 * 256
    dslot = (ctx.chunk_bytes(prec, T) + 4095) // 4096 * 4096
    for tier, base, cap in ((B.TIER_HBM, FAKE_HBM, caps[0]), (B.TIER_PINNED, FAKE_PIN, caps[1]),
                            (B.TIER_PAGEABLE, FAKE_PAGE, caps[2])):
        if cap:
            ctx.register_slab(tier, prec, base, slot * cap)
    ctx.register_disk(prec, "/nonexistent/never-opened-in-dry-run", dslot * n)
    ctx.register_staging(FAKE_STG, dslot * 3)
    ctx.register_bounce(FAKE_BNC, dslot * 2)
    for c in range(n):
        ctx.pool_insert(c, prec, T, None, B.TIER_DISK)
    return ctx


def test_alg2_four_tier_trace_equals_oracle(golden_dir):
    import json
    import os
    gold = json.load(open(os.path.join(golden_dir, "paper_values.json")))["alg2_thresholds_percent"]
    taus = [gold["tau_gpu"] * 10_000, gold["tau_pin"] * 10_000, gold["tau_page"] * 10_000]
    n, caps = 100, (3, 4, 6)                    # lists of 5 / 5 / 10 chunks, smaller queues
    ctx = _ctx4(n, caps, taus)
    ctx.set_counts(list(range(n)), [1000 - c for c in range(n)])     # rank == id
    ctx.rerank()
    sim = pl.TierSim(list(range(n)), taus, caps)
    assert sim.bounds == (5, 10, 20)
    rng = np.random.default_rng(5)
    hot = rng.integers(0, 25, 600)
    cold = rng.integers(0, n, 600)
    seq = np.where(rng.random(600) < 0.8, hot, cold).tolist()
    tiers = (B.TIER_HBM, B.TIER_PINNED, B.TIER_PAGEABLE)
    seen = set()
    for c in seq:
        st, tr = ctx.load_chunks([c], FAKE_HBM, 128, want_trace=True)
        found, placed = sim.access(c)
        assert tr[0].found_tier == found, (c, tr[0].found_tier, found)
        if placed:
            assert tr[0].placed_tier == placed[0][0]
            assert tr[0].evicted_id == (placed[0][1] if placed[0][1] is not None else B.NO_CHUNK)
        else:
            assert tr[0].placed_tier == B.TIER_NONE and tr[0].evicted_id == B.NO_CHUNK
        for t in tiers:
            assert ctx.pool_lru(t) == sim.resident(t), (c, t)
        seen.add((found, placed[0][0] if placed else None))
        assert st["n_hbm_hits"] + st["n_pinned_hits"] + st["n_pageable_hits"] + st["n_disk_hits"] == 1
    # the sequence exercised every branch of the lookup cascade
    assert {(3, 0), (3, 1), (3, 2), (3, None), (0, None), (1, None), (2, None)} <= seen
    q = ctx.pool_query(0)
    assert q.on_disk == 1 and q.count == 1000 + seq.count(0)


def test_four_tier_multi_chunk_request_and_stats():
    n = 40
    ctx = _ctx4(n, (4, 4, 8), [100_000, 100_000, 200_000])    # lists: 4 / 4 / 8 chunks
    ctx.set_counts(list(range(n)), [1000 - c for c in range(n)])
    ctx.rerank()
    req = [0, 5, 9, 30, 1, 5, 0]
    st, tr = ctx.load_chunks(req, FAKE_HBM, 7 * 128, want_trace=True)
    assert [t.found_tier for t in tr] == [3, 3, 3, 3, 3, 1, 0]      # repeats find the new copies
    assert [t.placed_tier for t in tr] == [0, 1, 2, 255, 0, 255, 255]
    cb = ctx.chunk_bytes(B.PREC_INT4, 128)
    assert st["n_disk_hits"] == 5 and st["n_pinned_hits"] == 1 and st["n_hbm_hits"] == 1
    assert st["n_promoted"] == 2 and st["n_placed_host"] == 2
    assert st["bytes_disk_read"] == 5 * cb and st["bytes_h2d"] == 6 * cb
    assert st["bytes_host_copied"] == 2 * cb and st["bytes_d2d"] == 2 * cb
    # kernels: none for early hits, the five chunks from files one by one, one for the two
    # repeats (the pinned copy of 5 and the HBM copy of 0, both written by this call)
    assert st["n_kernel_launches"] == 6
    assert ctx.pool_lru(B.TIER_HBM) == [1, 0] and ctx.pool_lru(B.TIER_PINNED) == [5]
    assert ctx.pool_lru(B.TIER_PAGEABLE) == [9]
    # eviction by hand: only copies that have a slower copy can go
    ctx.pool_evict(5, B.TIER_PINNED)
    with pytest.raises(B.HaRagError) as e:
        ctx.pool_evict(5, B.TIER_PINNED)
    assert e.value.code == B.ENOENT
    assert ctx.pool_query(5).in_pinned == 0 and ctx.pool_query(5).on_disk == 1


def test_slow_tiers_need_bounce_buffers():
    ctx = B.Context(2, 2, 64, 128, group_int8=64, group_int4=64, dry_run=True)
    slot = (ctx.chunk_bytes(B.PREC_INT4, 128) + 4095) // 4096 * 4096
    ctx.register_slab(B.TIER_PAGEABLE, B.PREC_INT4, FAKE_PAGE, slot * 4)
    ctx.register_staging(FAKE_STG, slot * 2)
    ctx.pool_insert(1, B.PREC_INT4, 128, None, B.TIER_PAGEABLE)
    with pytest.raises(B.HaRagError) as e:
        ctx.load_chunks([1], FAKE_HBM, 128)
    assert e.value.code == B.ENOSPC                   # no bounce buffers registered
    with pytest.raises(B.HaRagError) as e:
        ctx.register_bounce(FAKE_BNC + 8, slot * 2)   # not 4096-byte aligned
    assert e.value.code == B.EINVAL
    ctx.register_bounce(FAKE_BNC, slot * 2)
    st, _ = ctx.load_chunks([1], FAKE_HBM, 128)
    assert st["n_pageable_hits"] == 1 and st["bytes_host_copied"] == ctx.chunk_bytes(B.PREC_INT4, 128)


# ---- keys-only / values-only chunks: Algorithm 1's 2n units --------------------------
def _half_ctx(half_slots, n_slots=16, T=128):
    ctx = B.Context(2, 2, 64, T, group_int8=64, group_int4=64, tau_gpu_ppm=500_000, dry_run=True,
                    half_slots=half_slots)
    for prec in (B.PREC_INT8, B.PREC_INT4):
        whole = (ctx.chunk_bytes(prec, T) + 255) // 256 * 256
        half = (ctx.chunk_bytes(prec, T, part=B.PART_K) + 255) // 256 * 256
        slot = half if half_slots else whole
        ctx.register_slab(B.TIER_HBM, prec, FAKE_HBM + prec * (1 << 32), slot * n_slots)
        ctx.register_slab(B.TIER_PINNED, prec, FAKE_PIN + prec * (1 << 32), slot * n_slots)
    ctx.register_staging(FAKE_STG, (ctx.chunk_bytes(B.PREC_INT8, T) + 255) // 256 * 256 * 4)
    return ctx


def test_half_chunk_sizes_are_half_the_oracle_whole():
    ctx = _half_ctx(False)
    for prec, bits in ((B.PREC_INT8, 8), (B.PREC_INT4, 4)):
        for T in (1, 37, 128):
            assert ctx.chunk_bytes(prec, T, part=B.PART_V) == codec.half_bytes(2, 2, 64, T, bits, 64)
    ctx.destroy()


def test_planes_fill_independently_and_must_close():
    ctx = _half_ctx(False)
    # documents 0..2: keys int8 under id 10+d, values int4 under id 20+d; document 3 whole (id 3)
    toks = [100, 128, 64]
    for d, t in enumerate(toks):
        ctx.pool_insert_half(10 + d, B.PART_K, B.PREC_INT8, t, None, B.TIER_PINNED)
        ctx.pool_insert_half(20 + d, B.PART_V, B.PREC_INT4, t, None, B.TIER_PINNED)
    ctx.pool_insert(3, B.PREC_INT4, 50, None, B.TIER_PINNED)
    info = ctx.pool_query(21)
    assert info.part == B.PART_V and info.bytes == codec.half_bytes(2, 2, 64, 128, 4, 64)
    assert ctx.pool_query(3).part == B.PART_KV

    req = [10, 11, 20, 21, 3, 22, 12]             # K0 K1 V0 V1 whole V2 K2
    st, tr = ctx.load_chunks(req, FAKE_HBM, 1000, tok_base=5, want_trace=True)
    assert [t.tok_off for t in tr] == [5, 105, 5, 105, 233, 283, 283]
    assert st["tokens"] == 100 + 128 + 50 + 64
    assert st["bf16_bytes_written"] == st["tokens"] * 2 * 2 * 2 * 64 * 2
    assert st["packed_bytes_read"] == sum(ctx.pool_query(c).bytes for c in req)
    # every unit has its own access count (the AF entries of Algorithm 1)
    assert ctx.pool_query(10).count == 1 and ctx.pool_query(20).count == 1

    def refused(req, code, cap=1000):
        before = [ctx.pool_query(c).count for c in (10, 20, 3)]
        with pytest.raises(B.HaRagError) as e:
            ctx.load_chunks(req, FAKE_HBM, cap)
        assert e.value.code == code
        assert [ctx.pool_query(c).count for c in (10, 20, 3)] == before   # nothing happened

    refused([10], B.EINVAL)                        # keys without values
    refused([10, 21], B.EINVAL)                    # planes end at different lengths (100 vs 128)
    refused([10, 3, 20], B.EINVAL)                 # a whole chunk while the planes differ
    refused([10, 20], B.ENOSPC, cap=99)
    ctx.load_chunks([20, 10], FAKE_HBM, 100)       # values first is fine
    # the same id cannot be a key chunk here and a value chunk there
    with pytest.raises(B.HaRagError) as e:
        ctx.pool_insert_half(10, B.PART_V, B.PREC_INT8, 100, None, B.TIER_HBM)
    assert e.value.code == B.EFORMAT
    for bad in (B.PART_KV, 3):
        with pytest.raises(B.HaRagError) as e:
            ctx.pool_insert_half(99, bad, B.PREC_INT8, 100, None, B.TIER_PINNED)
        assert e.value.code == B.EINVAL
    ctx.destroy()


def test_batch_of_requests_with_halves_checks_each_request():
    ctx = _half_ctx(False)
    for d in range(2):
        ctx.pool_insert_half(10 + d, B.PART_K, B.PREC_INT8, 64, None, B.TIER_PINNED)
        ctx.pool_insert_half(20 + d, B.PART_V, B.PREC_INT4, 64, None, B.TIER_PINNED)
    st, tr = ctx.load_batch([[10, 20], [21, 11, 10, 20]], [FAKE_HBM, FAKE_HBM + (1 << 30)], [64, 200],
                            tok_base=[0, 7], want_trace=True)
    assert [t.tok_off for t in tr] == [0, 0, 7, 7, 71, 71]
    with pytest.raises(B.HaRagError) as e:         # second request leaves the value plane short
        ctx.load_batch([[10, 20], [11, 10, 20]], [FAKE_HBM, FAKE_HBM + (1 << 30)], [64, 200])
    assert e.value.code == B.EINVAL
    ctx.destroy()


def test_half_slots_pool_refuses_whole_chunks_and_promotes_units_on_their_own():
    ctx = _half_ctx(True, n_slots=4)
    with pytest.raises(B.HaRagError) as e:
        ctx.pool_insert(1, B.PREC_INT4, 128, None, B.TIER_PINNED)
    assert e.value.code == B.EFORMAT
    # keys hot, values cold: only the key chunks are in GPU_LIST (top half of 4 units)
    for d in range(2):
        ctx.pool_insert_half(10 + d, B.PART_K, B.PREC_INT8, 128, None, B.TIER_PINNED)
        ctx.pool_insert_half(20 + d, B.PART_V, B.PREC_INT4, 128, None, B.TIER_PINNED)
    ctx.set_counts([10, 11, 20, 21], [50, 40, 3, 2])
    ctx.rerank()
    st, tr = ctx.load_chunks([10, 20, 11, 21], FAKE_HBM, 256, want_trace=True)
    assert [t.promoted for t in tr] == [1, 0, 1, 0]
    assert ctx.pool_query(10).in_hbm and not ctx.pool_query(20).in_hbm
    st, tr = ctx.load_chunks([10, 20], FAKE_HBM, 256, want_trace=True)
    assert [t.found_tier for t in tr] == [B.TIER_HBM, B.TIER_PINNED]
    ctx.destroy()


# ---- paged destination ------------------------------------------------------------------
def test_paged_cache_description_is_checked():
    ctx = _ctx(2, 8, 500_000)                     # L2 H2 D64, int4 chunks of up to 128 tokens
    for c in range(4):
        ctx.pool_insert(c, B.PREC_INT4, 100, None, B.TIER_PINNED)

    def cache(**kw):
        a = dict(base=FAKE_HBM, page_table=FAKE_HBM + (1 << 20), page_tokens=16, n_pages=64,
                 layout="page_major", n_layers=2, n_kv_heads=2, head_dim=64, n_table=16)
        a.update(kw)
        return B.paged_cache(**a)

    st, tr = ctx.load_chunks_paged([0, 1], cache(), tok_base=3, want_trace=True)
    assert [t.tok_off for t in tr] == [3, 103] and st["tokens"] == 200
    for bad, code in [(cache(n_table=12), B.ENOSPC),              # 192 rows < 3 + 200
                      (cache(page_tokens=4), B.EINVAL),            # 4 * 64 * 2 = 512 B < 1 KiB
                      (cache(base=FAKE_HBM + 8), B.EINVAL),
                      (cache(page_table=0), B.EINVAL),
                      (cache(n_pages=0), B.EINVAL),
                      (cache(page_tokens=1 << 16, n_table=1 << 10), B.EINVAL)]:   # virtual tile >= 4 GiB
        with pytest.raises(B.HaRagError) as e:
            ctx.load_chunks_paged([0, 1], bad, tok_base=3)
        assert e.value.code == code
    c2 = cache()
    c2.page_stride += 8
    with pytest.raises(B.HaRagError) as e:
        ctx.load_chunks_paged([0], c2)
    assert e.value.code == B.EINVAL
    assert ctx.pool_query(0).count == 1           # refused calls changed nothing
    ctx.destroy()


def test_hundred_thousand_ids_ranks_lists_and_trace_equal_oracle():
    """The id count of the Zipf configuration (100k logical ids): ranks after a rerank equal
    Algorithm 1's sort, list boundaries equal the floors, and 600 Zipf requests of 8 ids
    through four tiers leave the same trace as the plain simulation."""
    N = 100_000
    taus = [10_000, 40_000, 100_000]
    caps = (50, 300, 2000)
    ctx = B.Context(2, 2, 64, 128, group_int8=64, group_int4=64, tau_gpu_ppm=taus[0], tau_pin_ppm=taus[1],
                    tau_page_ppm=taus[2], dry_run=True)
    nb = ctx.chunk_bytes(B.PREC_INT4, 128)
    slot = (nb + 255) // 256 * 256
    ctx.register_slab(B.TIER_HBM, B.PREC_INT4, FAKE_HBM, slot * caps[0])
    ctx.register_slab(B.TIER_PINNED, B.PREC_INT4, FAKE_PIN, slot * caps[1])
    ctx.register_slab(B.TIER_PAGEABLE, B.PREC_INT4, 0x7A0000000000, slot * caps[2])
    ctx.register_disk(B.PREC_INT4, "/nonexistent/dry-run", (nb + 4095) // 4096 * 4096 * N)
    ctx.register_staging(FAKE_STG, slot * 4)
    ctx.register_bounce(0x790000000000, ((nb + 4095) // 4096 * 4096) * 2)
    for c in range(N):
        ctx.pool_insert(c, B.PREC_INT4, 128, None, B.TIER_DISK)
    rng = np.random.default_rng(7)
    counts = rng.multinomial(2_000_000, wl.zipf_pmf(N, 1.1))[rng.permutation(N)].tolist()   # many ties
    ctx.set_counts(list(range(N)), counts)
    ctx.rerank()
    ranks = pl.ranks(counts)
    probe = rng.integers(0, N, 500).tolist() + [0, N - 1]
    assert [ctx.get_rank(c) for c in probe] == [ranks[c] for c in probe]
    sim = pl.TierSim(ranks, taus, caps)
    order = pl.rank_order(counts)
    for req in wl.zipf_requests(N, 600, 8, 3):
        ids = [order[int(r)] for r in req]            # rank r -> the chunk id holding it
        st, tr = ctx.load_chunks(ids, FAKE_HBM, 8 * 128, want_trace=True)
        for c, t in zip(ids, tr):
            tier, placed = sim.access(c)
            assert t.found_tier == tier
            assert t.placed_tier == (placed[0][0] if placed else B.TIER_NONE)
            assert t.evicted_id == (placed[0][1] if placed and placed[0][1] is not None else B.NO_CHUNK)
    for tier in (B.TIER_HBM, B.TIER_PINNED, B.TIER_PAGEABLE):
        assert ctx.pool_lru(tier) == sim.resident(tier)
    ctx.destroy()


def test_caller_owned_pinned_masters_of_a_hundred_thousand_ids():
    """The Zipf configuration's pool as the benchmark builds it: 100k ids whose pinned copies
    are caller-owned addresses (a small ring of buffers that many ids share), an HBM slab that
    holds GPU_LIST, promotion by Algorithm 2.  The trace equals the plain simulation with an
    unbounded pinned queue that holds every chunk; addresses follow insert and repoint."""
    N = 100_000
    taus = [30_000, 970_000, 0]
    cap = 3000
    ctx = B.Context(2, 2, 64, 128, group_int8=64, group_int4=64, tau_gpu_ppm=taus[0], tau_pin_ppm=taus[1],
                    rerank_interval=0, dry_run=True)
    slot = (ctx.chunk_bytes(B.PREC_16, 128) + 255) // 256 * 256
    ring = [0x7B0000000000 + 4096 * k for k in range(64)]
    with pytest.raises(B.HaRagError) as e:
        ctx.pool_insert_external(0, B.PREC_16, 128, ring[0])
    assert e.value.code == B.ENOSPC                       # the tag was not declared
    ctx.register_external(B.PREC_16)
    with pytest.raises(B.HaRagError) as e:
        ctx.register_slab(B.TIER_PINNED, B.PREC_16, FAKE_PIN, slot * 4)
    assert e.value.code == B.EINVAL                       # one pinned tier per tag
    ctx.register_slab(B.TIER_HBM, B.PREC_16, FAKE_HBM, slot * cap)
    ctx.register_staging(FAKE_STG, slot * 4)
    for c in range(N):
        ctx.pool_insert_external(c, B.PREC_16, 128, ring[c % 64])
    with pytest.raises(B.HaRagError) as e:
        ctx.pool_insert_external(5, B.PREC_16, 128, ring[1])
    assert e.value.code == B.EINVAL                       # already there
    with pytest.raises(B.HaRagError) as e:
        ctx.pool_insert(N, B.PREC_16, 128, None, B.TIER_PINNED)
    assert e.value.code == B.EINVAL                       # that tier's slots are the caller's
    with pytest.raises(B.HaRagError) as e:
        ctx.pool_insert_external(N, B.PREC_16, 128, ring[1] + 4)
    assert e.value.code == B.EINVAL                       # misaligned
    info = ctx.pool_query(70)
    assert info.in_pinned and info.pinned_ptr == ring[70 % 64] and not info.in_hbm
    ctx.pool_repoint_external([70, 71], [ring[3], ring[4]])
    assert ctx.pool_query(70).pinned_ptr == ring[3] and ctx.pool_slot(71, B.TIER_PINNED)[0] == ring[4]
    with pytest.raises(B.HaRagError) as e:
        ctx.pool_repoint_external([70, N + 5], [ring[9], ring[9]])
    assert e.value.code == B.ENOENT and ctx.pool_query(70).pinned_ptr == ring[3]
    ctx.rerank()                                          # no counts yet: ranks follow the ids
    sim = pl.TierSim(list(range(N)), taus, (cap, None, 0))
    sim.seed(sim.PIN, range(N))
    hits = 0
    for k, req in enumerate(wl.zipf_requests(N, 1500, 8, 5)):
        ids = [int(r) for r in req]
        st, tr = ctx.load_chunks(ids, FAKE_HBM, 8 * 128, want_trace=True)
        hits += st["n_hbm_hits"]
        for c, t in zip(ids, tr):
            tier, placed = sim.access(c)
            assert t.found_tier == tier
            assert t.placed_tier == (placed[0][0] if placed else B.TIER_NONE)
            assert t.evicted_id == (placed[0][1] if placed and placed[0][1] is not None else B.NO_CHUNK)
    assert ctx.pool_lru(B.TIER_HBM) == sim.resident(sim.GPU)
    assert hits / (1500 * 8) > 0.6                        # the top 3 % of ranks draw most accesses
    # an evicted chunk falls back to the caller's address, and a removed one frees its entry
    victim = ctx.pool_lru(B.TIER_HBM)[0]
    ctx.pool_evict(victim, B.TIER_HBM)
    assert not ctx.pool_query(victim).in_hbm and ctx.pool_query(victim).in_pinned
    ctx.pool_remove(victim)
    ctx.pool_insert_external(victim, B.PREC_16, 100, ring[7])
    assert ctx.pool_query(victim).pinned_ptr == ring[7] and ctx.pool_query(victim).n_tokens == 100
    ctx.destroy()


def test_forget_stream_on_a_context_without_a_gpu():
    ctx = _ctx(2, 4, 500_000)
    ctx.forget_stream(None)
    ctx.forget_stream(0x1234)
    assert B.lib().ha_rag_forget_stream(None, None) == B.EINVAL
    ctx.destroy()


def test_pinned_only_pool_needs_no_staging_unless_dma_is_asked_for():
    for dma in (False, True):
        ctx = B.Context(2, 2, 64, 128, group_int8=64, group_int4=64, tau_gpu_ppm=500_000, dry_run=True,
                        pinned_dma=dma)
        slot = (ctx.chunk_bytes(B.PREC_INT4, 128) + 255) // 256 * 256
        ctx.register_slab(B.TIER_PINNED, B.PREC_INT4, FAKE_PIN, slot * 4)
        for c in range(4):
            ctx.pool_insert(c, B.PREC_INT4, 100, None, B.TIER_PINNED)
        if dma:
            with pytest.raises(B.HaRagError) as e:
                ctx.load_chunks([0, 1, 2], FAKE_HBM, 300)
            assert e.value.code == B.ENOSPC               # DMA needs the staging area
            ctx.register_staging(FAKE_STG, slot * 2)
            st, _ = ctx.load_chunks([0, 1, 2], FAKE_HBM, 300)
            assert st["n_kernel_launches"] == 3           # one per transferred chunk
        else:
            st, _ = ctx.load_chunks([0, 1, 2], FAKE_HBM, 300)
            assert st["n_kernel_launches"] == 1           # read in place, one launch
        assert st["n_pinned_hits"] == 3 and st["bytes_h2d"] == 3 * ctx.chunk_bytes(B.PREC_INT4, 100)
        # once an HBM slab exists a promotion may need the staging area
        ctx.register_slab(B.TIER_HBM, B.PREC_INT4, FAKE_HBM, slot * 2)
        if not dma:
            with pytest.raises(B.HaRagError) as e:
                ctx.load_chunks([3], FAKE_HBM, 300)
            assert e.value.code == B.ENOSPC
        ctx.destroy()


# ---- the file tier's index outlives the context -------------------------------------------
def _disk_ctx(n_slots, half_slots=False, T=128, group4=64):
    ctx = B.Context(2, 2, 64, T, group_int8=64, group_int4=group4, tau_gpu_ppm=200_000, dry_run=True,
                    half_slots=half_slots)
    for prec in (B.PREC_INT4, B.PREC_INT8):
        nb = ctx.chunk_bytes(prec, T, part=B.PART_K if half_slots else B.PART_KV)
        ctx.register_disk(prec, "/nonexistent/dry-run", (nb + 4095) // 4096 * 4096 * n_slots)
        ctx.register_slab(B.TIER_HBM, prec, FAKE_HBM + prec * (1 << 32), (nb + 255) // 256 * 256 * 2)
    big = (ctx.chunk_bytes(B.PREC_INT8, T) + 4095) // 4096 * 4096
    ctx.register_staging(FAKE_STG, big * 2)
    ctx.register_bounce(FAKE_BNC, big * 2)
    return ctx


def test_index_round_trip_restores_masters_counts_and_slots(tmp_path):
    path = str(tmp_path / "kb.idx")
    a = _disk_ctx(8)
    ids = [7, 3, 900, 12, 5]
    for k, cid in enumerate(ids):
        a.pool_insert(cid, B.PREC_INT4 if k % 2 else B.PREC_INT8, 100 + k, None, B.TIER_DISK)
    a.pool_insert(77, B.PREC_INT4, 50, None, B.TIER_HBM)          # no file copy: not in the index
    a.set_counts(ids, [10, 40, 30, 20, 50])
    a.rerank()
    a.load_chunks([3, 5], FAKE_HBM, 400)                          # counts move, 5 and 3 get HBM copies
    a.pool_save_index(path)
    before = {cid: a.pool_query(cid) for cid in ids}
    slots = {cid: before[cid].disk_slot for cid in ids}
    assert len({(before[c].prec, slots[c]) for c in ids}) == len(ids)
    a.destroy()

    b = _disk_ctx(8)
    assert b.pool_load_index(path) == len(ids)
    for cid in ids:
        q = b.pool_query(cid)
        assert (q.prec, q.n_tokens, q.part, q.count, q.bytes) == \
            (before[cid].prec, before[cid].n_tokens, before[cid].part, before[cid].count, before[cid].bytes)
        assert q.on_disk == 1 and q.in_hbm == 0                   # faster tiers start empty
        assert q.disk_slot == slots[cid]
    with pytest.raises(B.HaRagError) as e:
        b.pool_query(77)
    assert e.value.code == B.ENOENT
    b.rerank()
    assert sorted(ids, key=lambda c: b.get_rank(c)) == sorted(ids, key=lambda c: (-before[c].count, c))
    # restored slots are taken: new chunks get other slots, and a full file slab says so
    used = {slots[c] for c in ids if before[c].prec == B.PREC_INT4}
    b.pool_insert(1000, B.PREC_INT4, 10, None, B.TIER_DISK)
    assert b.pool_query(1000).disk_slot not in used
    st, tr = b.load_chunks([5, 3, 12], FAKE_HBM, 400, want_trace=True)
    assert [t.found_tier for t in tr] == [B.TIER_DISK] * 3
    with pytest.raises(B.HaRagError) as e:                        # the same index twice: ids exist
        b.pool_load_index(path)
    assert e.value.code == B.EINVAL
    b.destroy()


def test_index_is_refused_by_a_context_that_does_not_match(tmp_path):
    path = str(tmp_path / "kb.idx")
    a = _disk_ctx(4)
    a.pool_insert(1, B.PREC_INT4, 100, None, B.TIER_DISK)
    a.pool_save_index(path)
    a.destroy()
    for make, code in ((lambda: _disk_ctx(4, T=64), B.EFORMAT),          # other slot size / max tokens
                       (lambda: _disk_ctx(4, group4=32), B.EFORMAT),
                       (lambda: _disk_ctx(4, half_slots=True), B.EFORMAT)):
        c = make()
        with pytest.raises(B.HaRagError) as e:
            c.pool_load_index(path)
        assert e.value.code == code
        with pytest.raises(B.HaRagError):
            c.pool_query(1)                                               # nothing was added
        c.destroy()
    c = _disk_ctx(4)
    with pytest.raises(B.HaRagError) as e:
        c.pool_load_index(str(tmp_path / "missing.idx"))
    assert e.value.code == B.EIO
    bad = tmp_path / "bad.idx"
    bad.write_bytes(open(path, "rb").read()[:40])
    with pytest.raises(B.HaRagError) as e:
        c.pool_load_index(str(bad))
    assert e.value.code == B.EIO
    c.pool_insert(1, B.PREC_INT8, 10, None, B.TIER_DISK)                  # id 1 exists already
    with pytest.raises(B.HaRagError) as e:
        c.pool_load_index(path)
    assert e.value.code == B.EINVAL
    c.destroy()


def test_index_with_key_and_value_units(tmp_path):
    path = str(tmp_path / "kb.idx")
    a = _disk_ctx(6, half_slots=True)
    a.pool_insert_half(10, B.PART_K, B.PREC_INT8, 90, None, B.TIER_DISK)
    a.pool_insert_half(20, B.PART_V, B.PREC_INT4, 90, None, B.TIER_DISK)
    a.pool_save_index(path)
    a.destroy()
    b = _disk_ctx(6, half_slots=True)
    assert b.pool_load_index(path) == 2
    assert b.pool_query(10).part == B.PART_K and b.pool_query(20).part == B.PART_V
    st, tr = b.load_chunks([20, 10], FAKE_HBM, 90, want_trace=True)
    assert [t.tok_off for t in tr] == [0, 0]
    b.destroy()


def test_context_without_integer_tags_for_head_dims_no_group_divides():
    for D in (8, 24, 80):
        with pytest.raises(B.HaRagError) as e:
            B.Context(2, 2, D, 64, group_int8=32, group_int4=64, dry_run=True)
        assert e.value.code == B.EFORMAT
        ctx = B.Context(2, 2, D, 64, group_int8=0, group_int4=0, dry_run=True)
        for prec, bits in ((B.PREC_16, 16), (B.PREC_FP8_E5M2, 52), (B.PREC_GSE8, 143)):
            assert ctx.chunk_bytes(prec, 37) == codec.chunk_bytes(2, 2, D, 37, bits, 32)
            slot = (ctx.chunk_bytes(prec, 64) + 255) // 256 * 256
            ctx.register_slab(B.TIER_PINNED, prec, FAKE_PIN + prec * (1 << 32), slot * 2)
            ctx.pool_insert(prec, prec, 37, None, B.TIER_PINNED)
        for prec in (B.PREC_INT8, B.PREC_INT4):
            with pytest.raises(B.HaRagError) as e:
                ctx.register_slab(B.TIER_PINNED, prec, FAKE_PIN + prec * (1 << 32), 1 << 20)
            assert e.value.code == B.EFORMAT
        st, _ = ctx.load_chunks([B.PREC_16, B.PREC_GSE8], FAKE_HBM, 100)
        assert st["tokens"] == 74
        ctx.destroy()
    # one integer tag may be off while the other is on
    ctx = B.Context(2, 2, 96, 64, group_int8=32, group_int4=0, dry_run=True)
    assert ctx.chunk_bytes(B.PREC_INT8, 10) == codec.chunk_bytes(2, 2, 96, 10, 8, 32)
    with pytest.raises(B.HaRagError):
        ctx.chunk_bytes(B.PREC_INT4, 10)
    ctx.destroy()


def test_remove_takes_a_chunk_out_of_every_tier_and_frees_its_slots():
    n = 6
    ctx = _ctx4(n, (2, 2, 2), [340_000, 340_000, 0])        # lists of 2 / 2 chunks of 6
    ctx.set_counts(list(range(n)), [100 - c for c in range(n)])
    ctx.rerank()
    ctx.load_chunks([0, 1, 2, 3], FAKE_HBM, 4 * 128)         # 0, 1 -> HBM; 2, 3 -> pinned
    assert ctx.pool_hbm_lru() == [0, 1] and ctx.pool_lru(B.TIER_PINNED) == [2, 3]
    ctx.pool_remove(0)
    ctx.pool_remove(2)
    for cid in (0, 2):
        with pytest.raises(B.HaRagError) as e:
            ctx.pool_query(cid)
        assert e.value.code == B.ENOENT
        with pytest.raises(B.HaRagError) as e:
            ctx.load_chunks([cid], FAKE_HBM, 128)
        assert e.value.code == B.ENOENT
    with pytest.raises(B.HaRagError) as e:
        ctx.pool_remove(0)
    assert e.value.code == B.ENOENT
    assert ctx.pool_hbm_lru() == [1] and ctx.pool_lru(B.TIER_PINNED) == [3]
    # N is now 4: lists of floor(0.34 * 4) = 1 / 1 chunk; ranks close up
    ctx.rerank()
    assert [ctx.get_rank(c) for c in (1, 3, 4, 5)] == [0, 1, 2, 3]
    st, tr = ctx.load_chunks([4, 5], FAKE_HBM, 256, want_trace=True)
    assert [t.placed_tier for t in tr] == [B.TIER_NONE, B.TIER_NONE]       # ranks 2, 3: DISK_LIST
    # the file slab was full (6 slots, 6 chunks): the freed slots take new chunks, the old id may return
    used = {ctx.pool_query(c).disk_slot for c in (1, 3, 4, 5)}
    ctx.pool_insert(0, B.PREC_INT4, 77, None, B.TIER_DISK)
    ctx.pool_insert(99, B.PREC_INT4, 128, None, B.TIER_DISK)
    assert ctx.pool_query(0).n_tokens == 77 and ctx.pool_query(0).count == 0
    assert len(used | {ctx.pool_query(0).disk_slot, ctx.pool_query(99).disk_slot}) == 6
    with pytest.raises(B.HaRagError) as e:
        ctx.pool_insert(100, B.PREC_INT4, 128, None, B.TIER_DISK)
    assert e.value.code == B.ENOSPC
    ctx.destroy()


def _attend_ctx(D=128, L=4, H=2):
    return B.Context(L, H, D, 512, group_int8=min(D, 128), group_int4=min(D, 64), dry_run=True)


def test_attend_launch_descriptors_are_filled_and_checked_without_a_device():
    """A dry-run context cuts the requests' blocks into runs, fills every launch's descriptors and
    runs the launches' own argument checks (only the launch itself is left out), so lists of any
    shape must come back OK: more runs than one launch holds, runs that span more documents than
    a run may (128), requests for both kernels in one call, the workspace exactly as large as
    asked for."""
    ctx = _attend_ctx(H=8)
    P = 0x7F0000001000
    ch = lambda t, p=B.PREC_INT4, g=64: (P, t, p, g, B.PART_KV)
    req = lambda chunks, n_q: (chunks, P, P, P, n_q)
    precs = [(B.PREC_INT4, 64), (B.PREC_INT8, 128), (B.PREC_16, 0), (B.PREC_FP8_E4M3, 0), (B.PREC_GSE8, 0)]
    lists = [
        [req([ch(1, *precs[i % 5]) for i in range(600)], 40)],                        # one block per document
        [req([ch(3 + 7 * i % 50, *precs[i % 5]) for i in range(700)], 1)],             # 700 runs: two launches
        [req([ch(2000)] * 40, 1), req([ch(2000)] * 40, 64), req([ch(17)], 9), req([], 3)],
        [req([ch(16 * (1 + i % 9), *precs[(i + r) % 5]) for i in range(60)], 1 + 13 * r) for r in range(20)],
    ]
    for reqs in lists:
        n = ctx.attend_workspace_bytes(reqs, 32)
        ctx.attend_packed(reqs, 1, 32, 0.088, P, n)
        if n:
            with pytest.raises(B.HaRagError) as e:
                ctx.attend_packed(reqs, 1, 32, 0.088, P, n - 4)
            assert e.value.code == B.ENOSPC
    ctx.destroy()


def test_attend_workspace_size_and_argument_checks():
    ctx = _attend_ctx()
    P = 0x7F0000001000
    ch = lambda t, p=B.PREC_INT4, g=64, part=B.PART_KV: (P, t, p, g, part)
    req = lambda chunks, n_q: (chunks, P, P, None, n_q)
    REC = (16 * 128 + 32) * 4
    # records: runs x KV heads x 16-row query tiles.  With at most two query tiles a run is a
    # piece of one document: equal pieces, none longer than 2048 tokens; that bound is halved
    # (down to 128 tokens) while the call has fewer than 2048 workgroups (runs x KV heads x pairs
    # of query tiles), and once more (64 tokens) if the call then still has at most 1024
    assert ctx.attend_workspace_bytes([req([ch(512), ch(100)], 1)], 8) == (8 + 2) * 2 * 1 * REC
    assert ctx.attend_workspace_bytes([req([ch(512), ch(0)], 5)], 8) == 8 * 2 * 2 * REC
    c2 = B.Context(4, 2, 128, 2000, group_int8=128, group_int4=64, dry_run=True)
    # 1100 tokens = 69 blocks: 18 pieces of 4 blocks (the last one 1)
    assert c2.attend_workspace_bytes([req([ch(1100), ch(10)], 4), req([], 1), req([ch(16)], 9)], 4) == \
        ((18 + 1) * 2 * 1 + 0 + 1 * 2 * 2) * REC
    # 300 chunks x 2 heads x 4 pieces of at most 512 tokens make 2400 workgroups: no finer pieces
    big = [req([ch(2000)] * 100, 1) for _ in range(3)]
    assert c2.attend_workspace_bytes(big, 4) == 300 * 4 * 2 * 1 * REC
    c2.destroy()
    ok = [req([ch(512), ch(100, B.PREC_16, 0)], 3)]
    n = ctx.attend_workspace_bytes(ok, 8)
    ctx.attend_packed(ok, 3, 8, 0.1, P, n)

    def fails(code, reqs, layer=0, n_qh=8, scale=0.1, ws=P, ws_bytes=n):
        with pytest.raises(B.HaRagError) as e:
            ctx.attend_packed(reqs, layer, n_qh, scale, ws, ws_bytes)
        assert e.value.code == code, e.value.code

    fails(B.EINVAL, ok, layer=4)
    fails(B.EINVAL, ok, n_qh=7)
    fails(B.EINVAL, ok, n_qh=0)
    fails(B.EINVAL, ok, n_qh=2 * 65)
    fails(B.EINVAL, ok, scale=0.0)
    fails(B.EINVAL, ok, scale=float("nan"))
    fails(B.EINVAL, ok, ws=P + 4)
    fails(B.EINVAL, ok, ws=None)
    fails(B.ENOSPC, ok, ws_bytes=n - 1)
    fails(B.EINVAL, [])
    fails(B.EINVAL, [req([ch(16)], 0)])
    fails(B.EINVAL, [req([ch(16)], 4097)])
    fails(B.EINVAL, [(([ch(16)]), P + 2, P, None, 1)])              # q misaligned
    fails(B.EINVAL, [(([ch(16)]), P, None, None, 1)])               # no out
    fails(B.EINVAL, [req([(P + 8, 16, B.PREC_INT4, 64, B.PART_KV)], 1)])
    fails(B.EINVAL, [req([ch(16, part=B.PART_K)], 1)])                                   # keys without values
    fails(B.EINVAL, [req([ch(16, part=B.PART_V), ch(16)], 1)])
    fails(B.EINVAL, [req([ch(16, part=B.PART_K), ch(32, part=B.PART_V)], 1)])            # lengths differ
    fails(B.EINVAL, [req([ch(16, part=B.PART_K)], 1), req([ch(16, part=B.PART_V)], 1)])  # pairs do not cross requests
    # keys and values of two documents in any interleaving, formats of their own, next to a whole chunk
    pairs = [req([ch(64, part=B.PART_V), ch(64, B.PREC_16, 0, B.PART_K), ch(100), ch(40, B.PREC_INT8, 128, B.PART_K),
                  ch(40, part=B.PART_V)], 2)]
    assert ctx.attend_workspace_bytes(pairs, 8) == 4 * 2 * 1 * REC     # three documents, the one of 7 blocks in two pieces
    ctx.attend_packed(pairs, 0, 8, 0.1, P, 4 * 2 * REC)
    fails(B.EFORMAT, [req([ch(16, g=48)], 1)])
    fails(B.EFORMAT, [req([ch(16, p=9)], 1)])
    ctx.destroy()
    other = _attend_ctx(D=64)
    with pytest.raises(B.HaRagError) as e:
        other.attend_workspace_bytes([req([ch(16, g=64)], 1)], 2)
    assert e.value.code == B.EFORMAT
    other.destroy()


def test_attend_chunks_reads_hbm_or_pinned_copies_and_counts_on_request():
    n = 6
    ctx = B.Context(2, 2, 128, 128, group_int8=128, group_int4=64, dry_run=True,
                    tau_gpu_ppm=340_000, tau_pin_ppm=340_000, tau_page_ppm=0)
    for tier, base, slots in ((B.TIER_HBM, FAKE_HBM, 2), (B.TIER_PINNED, FAKE_PIN, 3),
                              (B.TIER_PAGEABLE, 0x500000000000, 2)):
        slot = (ctx.chunk_bytes(B.PREC_INT4, 128) + 255) // 256 * 256
        ctx.register_slab(tier, B.PREC_INT4, base, slot * slots)
    ctx.pool_insert(0, B.PREC_INT4, 128, None, B.TIER_HBM)
    ctx.pool_insert(1, B.PREC_INT4, 100, None, B.TIER_PINNED)
    ctx.pool_insert(2, B.PREC_INT4, 64, None, B.TIER_PINNED)
    ctx.pool_insert(3, B.PREC_INT4, 128, None, B.TIER_PAGEABLE)
    P = 0x7F0000001000
    reqs = [([1, 0], P, P, None, 1), ([2], P, P, P, 3)]
    nb = ctx.attend_chunks_workspace_bytes(reqs, 8)
    packed_view = [([(P, 100, B.PREC_INT4, 64), (P, 128, B.PREC_INT4, 64)], P, P, None, 1),
                   ([(P, 64, B.PREC_INT4, 64)], P, P, P, 3)]
    assert nb == ctx.attend_workspace_bytes(packed_view, 8) > 0
    ctx.attend_chunks(reqs, 1, 8, 0.1, P, nb)                          # no bookkeeping
    assert [ctx.pool_query(i).count for i in range(4)] == [0, 0, 0, 0]
    assert ctx.pool_lru(B.TIER_PINNED) == [1, 2]
    ctx.attend_chunks(reqs, 0, 8, 0.1, P, nb, count=True)
    assert [ctx.pool_query(i).count for i in range(4)] == [1, 1, 1, 0]
    ctx.attend_chunks([([1], P, P, None, 1)], 0, 8, 0.1, P, nb, count=True)
    assert ctx.pool_query(1).count == 2 and ctx.pool_lru(B.TIER_PINNED) == [2, 1]
    for bad, code in (([([3], P, P, None, 1)], B.ENOENT),             # only a pageable copy
                      ([([9], P, P, None, 1)], B.ENOENT),             # unknown id
                      ([([0], P, P, None, 0)], B.EINVAL)):
        with pytest.raises(B.HaRagError) as e:
            ctx.attend_chunks(bad, 0, 8, 0.1, P, nb)
        assert e.value.code == code
    with pytest.raises(B.HaRagError) as e:
        ctx.attend_chunks(reqs, 0, 8, 0.1, P, nb - 1)
    assert e.value.code == B.ENOSPC
    assert [ctx.pool_query(i).count for i in range(4)] == [1, 2, 1, 0]     # failed calls count nothing
    rc = B.lib().ha_rag_attend_chunks(ctx._h, None, None, 0, 0, 8, 0.1, 2, None, 0, None)
    assert rc == B.EINVAL                                              # unknown flag
    ctx.destroy()


def test_place_chunks_is_algorithm_2_without_the_decode():
    """The same sequence as the four-tier trace test, with placement-only calls and loads
    mixed, with and without the floor that keeps every chunk device-visible: lookups, placements,
    evictions and residency equal the oracle's after every call."""
    taus = [50_000, 50_000, 100_000]
    n, caps = 100, (3, 4, 6)
    ctx = _ctx4(n, caps, taus)
    ctx.set_counts(list(range(n)), [1000 - c for c in range(n)])
    ctx.rerank()
    sim = pl.TierSim(list(range(n)), taus, caps)
    rng = np.random.default_rng(11)
    hot = rng.integers(0, 25, 500)
    cold = rng.integers(0, n, 500)
    seq = np.where(rng.random(500) < 0.8, hot, cold).tolist()
    tiers = (B.TIER_HBM, B.TIER_PINNED, B.TIER_PAGEABLE)
    cb = ctx.chunk_bytes(B.PREC_INT4, 128)
    kinds = set()
    for k, c in enumerate(seq):
        mode = k % 3                                           # load, place, place with the floor
        if mode == 0:
            st, tr = ctx.load_chunks([c], FAKE_HBM, 128, want_trace=True)
            found, placed = sim.access(c)
        else:
            st, tr = ctx.place_chunks([c], device_visible=(mode == 2), want_trace=True)
            found, placed = sim.access(c, floor=pl.TierSim.PIN if mode == 2 else None)
            assert st["n_kernel_launches"] == 0 and st["bf16_bytes_written"] == 0 and st["bytes_d2d"] == 0
            to = placed[0][0] if placed else None
            assert st["bytes_h2d"] == (cb if to == 0 else 0)
            assert st["bytes_disk_read"] == (cb if placed and found == 3 else 0)
            assert st["bytes_host_copied"] == cb * ((1 if placed and found == 2 else 0) + (1 if to in (1, 2) else 0))
            if mode == 2:
                kinds.add((found, to))
        assert tr[0].found_tier == found, (k, c)
        if placed:
            assert tr[0].placed_tier == placed[0][0]
            assert tr[0].evicted_id == (placed[0][1] if placed[0][1] is not None else B.NO_CHUNK)
        else:
            assert tr[0].placed_tier == B.TIER_NONE
        for t in tiers:
            assert ctx.pool_lru(t) == sim.resident(t), (k, c, t)
    # with the floor, chunks of the PAGE and DISK lists found in a file or in pageable memory went to pinned memory
    assert (3, 1) in kinds and (2, 1) in kinds and (3, 0) in kinds
    assert sum(ctx.pool_query(c).count for c in range(n)) == sum(1000 - c for c in range(n)) + len(seq)
    # several chunks in one call, a repeat among them; afterwards every one of them can be attended in place
    st, tr = ctx.place_chunks([70, 71, 70, 2], device_visible=True, want_trace=True)
    assert all(ctx.pool_query(c).in_hbm or ctx.pool_query(c).in_pinned for c in (70, 71, 2))
    assert tr[2].found_tier == B.TIER_PINNED and tr[2].placed_tier == B.TIER_NONE
    with pytest.raises(B.HaRagError) as e:
        ctx.place_chunks([1, 1000])
    assert e.value.code == B.ENOENT
    rc = B.lib().ha_rag_place_chunks(ctx._h, None, None, 0, 4, None, None, None)
    assert rc == B.EINVAL
    ctx.destroy()
