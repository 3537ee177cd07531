"""Keys-only and values-only chunks (the 2n units of Algorithm 1) on the GPU against the
oracle: packed bytes bit-exact, cache words identical, plane offsets exact."""
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


def dev_u16(a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda()


def dev_u8(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint8)).cuda()


def host_u16(t):
    return t.cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("prec", sorted(ORC))
@pytest.mark.parametrize("shape", [(2, 2, 64, 128, 64), (3, 1, 128, 37, 32), (1, 3, 96, 100, 32)])
def test_quantize_half_bytes_equal_oracle(prec, shape):
    L, H, D, T, g = shape
    ctx = B.Context(L, H, D, T, group_int8=g, group_int4=g)
    src = wl.kv_chunk(L, H, D, T, 77)
    n = ctx.chunk_bytes(prec, T, part=B.PART_K)
    for kv in (0, 1):
        half = np.ascontiguousarray(src[:, kv])
        ref, ref_sat = codec.quantize_pack_half(half, ORC[prec], g)
        assert ref.size == n
        dst = torch.full((n + 64,), 0xAB, dtype=torch.uint8, device="cuda")
        sat = torch.zeros(1, dtype=torch.int32, device="cuda")
        ctx.quantize_half(dev_u16(half), T, prec, g, dst, saturated=sat)
        torch.cuda.synchronize()
        got = dst.cpu().numpy()
        assert np.all(got[n:] == 0xAB), "quantize wrote past the half chunk"
        assert np.array_equal(got[:n], ref)
        assert int(sat.item()) == ref_sat
    ctx.destroy()


def _units(L, H, D, g, spec, seed):
    """spec: list of (part, prec, n_tokens).  Returns packed oracle bytes per unit."""
    packed = []
    for i, (part, prec, t) in enumerate(spec):
        doc = wl.kv_chunk(L, H, D, t, seed * 50 + i)
        if part == B.PART_KV:
            packed.append(codec.quantize_pack_chunk(doc, ORC[prec], g)[0])
        else:
            packed.append(codec.quantize_pack_half(np.ascontiguousarray(doc[:, part - 1]), ORC[prec], g)[0])
    return packed


@pytest.mark.parametrize("launch", [None, (256, 2, 4, 0, 0), (1024, 4, 2, 1, 1)])
def test_load_packed_keys_and_values_at_different_precision(launch):
    """K at int8 and V at int4 (and other pairings), ragged lengths, a whole chunk in
    between, values of one document ahead of its keys."""
    L, H, D, g = 3, 2, 64, 32
    K, V, W = B.PART_K, B.PART_V, B.PART_KV
    spec = [(K, B.PREC_INT8, 100), (V, B.PREC_INT4, 100), (W, B.PREC_16, 17),
            (V, B.PREC_GSE8, 61), (V, B.PREC_FP8_E5M2, 40), (K, B.PREC_FP8_E4M3, 101),
            (W, B.PREC_INT4, 33), (K, B.PREC_16, 9), (V, B.PREC_INT8, 9)]
    packed = _units(L, H, D, g, spec, 3)
    n = len(spec)
    tokens = [s[2] for s in spec]
    base, extra = 3, 5
    cap = base + 100 + 17 + 101 + 33 + 9 + extra
    ref = np.full((L, 2, H, cap, D), CANARY, np.uint16)
    _, offs = codec.load_chunks(packed, (L, H, D), tokens, [ORC[s[1]] for s in spec], [g] * n,
                                list(range(n)), cap_tokens=cap, tok_base=base, out=ref,
                                parts=[s[0] for s in spec])
    assert offs == [3, 3, 103, 120, 181, 120, 221, 254, 254]
    ctx = B.Context(L, H, D, 128, group_int8=g, group_int4=g)
    if launch:
        ctx.set_launch_params(*launch)
    dev = [dev_u8(p) for p in packed]
    out = torch.full((L, 2, H, cap, D), CANARY, dtype=torch.int16, device="cuda")
    ctx.load_packed([(dev[i], tokens[i], spec[i][1], g, spec[i][0]) for i in range(n)], out, cap, base)
    torch.cuda.synchronize()
    got = host_u16(out)
    assert np.array_equal(got, ref)
    assert np.all(got[:, :, :, :base] == CANARY) and np.all(got[:, :, :, cap - extra:] == CANARY)
    ctx.destroy()


def test_load_packed_refuses_open_planes_and_writes_nothing():
    L, H, D, g = 1, 2, 64, 64
    spec = [(B.PART_K, B.PREC_INT8, 16), (B.PART_V, B.PREC_INT8, 24), (B.PART_KV, B.PREC_INT8, 8)]
    packed = [dev_u8(p) for p in _units(L, H, D, g, spec, 1)]
    ctx = B.Context(L, H, D, 32, group_int8=g, group_int4=g)
    out = torch.full((L, 2, H, 64, D), CANARY, dtype=torch.int16, device="cuda")
    for lst in ([0], [0, 1], [0, 2, 1]):
        with pytest.raises(B.HaRagError) as e:
            ctx.load_packed([(packed[i], spec[i][2], spec[i][1], g, spec[i][0]) for i in lst], out, 64)
        assert e.value.code == B.EINVAL
    with pytest.raises(B.HaRagError) as e:
        ctx.load_packed([(packed[0], 16, B.PREC_INT8, g, 3)], out, 64)
    assert e.value.code == B.EINVAL
    torch.cuda.synchronize()
    assert np.all(host_u16(out) == CANARY)
    ctx.destroy()


def test_more_units_than_one_launch_holds():
    L, H, D, g, T = 1, 2, 64, 64, 8
    n_docs = 70                                    # 140 units > 2 launches of 64
    spec = []
    for d in range(n_docs):
        spec += [(B.PART_K, B.PREC_INT8 if d % 2 else B.PREC_16, T), (B.PART_V, B.PREC_INT4, T)]
    packed = _units(L, H, D, g, spec, 9)
    n = len(spec)
    cap = n_docs * T
    ref, _ = codec.load_chunks(packed, (L, H, D), [T] * n, [ORC[s[1]] for s in spec], [g] * n,
                               list(range(n)), cap_tokens=cap, parts=[s[0] for s in spec])
    ctx = B.Context(L, H, D, T, group_int8=g, group_int4=g)
    out = torch.full((L, 2, H, cap, D), CANARY, dtype=torch.int16, device="cuda")
    dev = [dev_u8(p) for p in packed]
    ctx.load_packed([(dev[i], T, spec[i][1], g, spec[i][0]) for i in range(n)], out, cap)
    torch.cuda.synchronize()
    assert np.array_equal(host_u16(out), ref)
    ctx.destroy()


def test_pool_of_units_keys_hot_values_cold():
    """A pool whose slots hold halves: key chunks int8 and hot (promoted to HBM), value
    chunks int4 and cold (served through staging); then the same request from the tiers
    the first one left behind."""
    L, H, D, T, g = 2, 2, 64, 64, 64
    n_docs = 6
    ctx = B.Context(L, H, D, T, group_int8=g, group_int4=g, tau_gpu_ppm=500_000, half_slots=True)
    keep = []
    big = 0
    for prec in (B.PREC_INT8, B.PREC_INT4):
        slot = (ctx.chunk_bytes(prec, T, part=B.PART_K) + 255) // 256 * 256
        big = max(big, slot)
        hb = torch.zeros(slot * 4, dtype=torch.uint8, device="cuda")
        pn = torch.zeros(slot * n_docs, dtype=torch.uint8).pin_memory()
        ctx.register_slab(B.TIER_HBM, prec, hb)
        ctx.register_slab(B.TIER_PINNED, prec, pn)
    ctx.register_staging(torch.zeros(big * 3, dtype=torch.uint8, device="cuda"))
    spec, ids = [], []
    for d in range(n_docs):
        t = T - 3 * d
        spec += [(B.PART_K, B.PREC_INT8, t), (B.PART_V, B.PREC_INT4, t)]
        ids += [100 + d, 200 + d]
    packed = _units(L, H, D, g, spec, 4)
    for i, (part, prec, t) in enumerate(spec):
        ctx.pool_insert_half(ids[i], part, prec, t, torch.from_numpy(packed[i]).pin_memory(), B.TIER_PINNED)
    # keys were accessed often, values rarely: GPU_LIST (top half of 12 units) = the 6 key chunks
    ctx.set_counts(ids, [1000 - i if spec[i][0] == B.PART_K else 10 - i // 2 for i in range(len(ids))])
    ctx.rerank()
    docs = [4, 0, 2, 5]
    req = [x for d in docs for x in (2 * d, 2 * d + 1)]          # unit indices K_d, V_d
    tokens = [s[2] for s in spec]
    cap = sum(tokens[2 * d] for d in docs) + 2
    ref = np.full((L, 2, H, cap, D), CANARY, np.uint16)
    codec.load_chunks(packed, (L, H, D), tokens, [ORC[s[1]] for s in spec], [g] * len(spec), req,
                      cap_tokens=cap, out=ref, parts=[s[0] for s in spec])
    for rnd in range(2):
        out = torch.full((L, 2, H, cap, D), CANARY, dtype=torch.int16, device="cuda")
        st, tr = ctx.load_chunks([ids[u] for u in req], out, cap, want_trace=True)
        torch.cuda.synchronize()
        assert np.array_equal(host_u16(out), ref), rnd
        if rnd == 0:
            assert [t.promoted for t in tr] == [1, 0] * 4
            assert st["n_pinned_hits"] == 8
        else:
            assert [t.found_tier for t in tr] == [B.TIER_HBM, B.TIER_PINNED] * 4
            assert st["bytes_h2d"] == sum(len(packed[u]) for u in req if spec[u][0] == B.PART_V)
    ctx.destroy()


def test_llama3_8b_units_sampled_tiles_match_oracle():
    """The headline shape with every document split into a key chunk and a value chunk of
    different precision (keys int8, values int4, two documents kept at 16 bits), in the
    launch configuration the benchmark uses; sampled tiles recomputed by the oracle."""
    L, H, D, T, g = 32, 8, 128, 512, 128
    ctx = B.Context(L, H, D, T, group_int8=g, group_int4=g)
    n_docs = 10
    kprec = [B.PREC_16] * 2 + [B.PREC_INT8] * 8
    vprec = [B.PREC_16] * 2 + [B.PREC_INT4] * 8
    srcs, chunks, packs = [], [], []
    for d in range(n_docs):
        s_ = wl.kv_chunk_device(L, H, D, T, 900 + d)           # [L][2][H][T][D]
        srcs.append(s_)
        for kv, prec in ((0, kprec[d]), (1, vprec[d])):
            half = s_[:, kv].contiguous()
            dst = torch.empty(ctx.chunk_bytes(prec, T, part=B.PART_K), dtype=torch.uint8, device="cuda")
            ctx.quantize_half(half, T, prec, g, dst)
            packs.append(dst)
            chunks.append((dst, T, prec, g, B.PART_K + kv))
    order = [7, 2, 9, 0, 4, 1, 8, 3, 6, 5]
    cap = n_docs * T
    out = torch.empty((L, 2, H, cap, D), dtype=torch.int16, device="cuda")
    # all keys first, then all values: planes fill independently
    ctx.load_packed([chunks[2 * d] for d in order] + [chunks[2 * d + 1] for d in order], out, cap)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    for pos, d in enumerate(order):
        for kv, prec in ((0, kprec[d]), (1, vprec[d])):
            if prec == B.PREC_16:
                assert torch.equal(out[:, kv, :, pos * T:(pos + 1) * T], srcs[d][:, kv].view(torch.int16))
            for _ in range(2):
                l, h = int(rng.integers(L)), int(rng.integers(H))
                tile = host_u16(srcs[d][l, kv, h].contiguous().view(torch.int16)).reshape(1, 1, T, D)
                ref_pack, _ = codec.quantize_pack_half(tile, ORC[prec], g)
                rec = ref_pack.size
                got_pack = packs[2 * d + kv][(l * H + h) * rec:(l * H + h + 1) * rec].cpu().numpy()
                assert np.array_equal(got_pack, ref_pack)
                ref_out = np.zeros((1, 2, 1, T, D), np.uint16)
                codec.dequant_scatter_half(ref_pack, (1, 1, D), T, ORC[prec], g, kv, ref_out, 0)
                assert np.array_equal(host_u16(out[l, kv, h, pos * T:(pos + 1) * T]), ref_out[0, kv, 0])
    ctx.destroy()
