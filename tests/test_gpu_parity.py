"""Parity of the HIP path against the CPU oracle, through the C ABI, on a real
MI355X.  Bars: packed bytes (codes, scale, zero, padding) bit-exact; BF16 cache
within 1 ulp (0 expected); order, offsets and untouched rows exact."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import codec
from paper_2510_20878_amd import binding as B
from paper_2510_20878_amd import workloads as wl

pytestmark = pytest.mark.gpu

CANARY = 0x7FC1          # a BF16 NaN pattern no kernel output can contain
# the oracle's name for each storage format
ORC = {B.PREC_16: 16, B.PREC_INT8: 8, B.PREC_INT4: 4, B.PREC_FP8_E4M3: 43, B.PREC_FP8_E5M2: 52,
       B.PREC_GSE8: 143}


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the GPU"
    B.lib()              # raises if the HIP library was not built: no fallback
    yield
    torch.cuda.synchronize()


def dev_u16(a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda()


def dev_u8(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint8)).cuda()


def host_u16(t):
    return t.cpu().numpy().view(np.uint16)


def ulp_distance(a, b):
    """Distance between BF16 words on the sign-magnitude ordered number line."""
    def key(w):
        w = w.astype(np.int32)
        return np.where(w & 0x8000, -(w & 0x7FFF), w & 0x7FFF)
    return np.abs(key(a) - key(b))


def gpu_quantize(ctx, src_words, prec, group):
    L, _, H, T, D = src_words.shape
    n = B.ha_rag_chunk_bytes(L, H, D, prec, group, T)[2]
    src = dev_u16(src_words)
    dst = torch.full((n + 64,), 0xAB, dtype=torch.uint8, device="cuda")
    sat = torch.zeros(1, dtype=torch.int32, device="cuda")
    ctx.quantize_chunk(src, T, prec, group, dst, saturated=sat)
    torch.cuda.synchronize()
    out = dst.cpu().numpy()
    assert np.all(out[n:] == 0xAB), "quantize wrote past the chunk"
    return out[:n], int(sat.item())


def special_values_chunk(L, H, D, T, seed):
    """Gaussian data salted with the awkward cases: constant groups, exact ties,
    BF16 subnormals, negative zeros, tiny and huge ranges, a saturating group."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((L, 2, H, T, D)).astype(np.float32)
    rows = x.reshape(-1, D)
    n = rows.shape[0]
    rows[0 % n] = 1.5                                           # constant group
    rows[1 % n] = 0.0
    rows[2 % n] = np.where(np.arange(D) % 2, -0.0, 0.0)         # both zeros
    rows[3 % n] = (np.arange(D) % 16) * 0.5                     # exact ties at scale 1 (int4: 7.5/15)
    rows[4 % n] = np.arange(D) % 16                             # codes == values for int4
    rows[5 % n] = rng.standard_normal(D) * 1e-39                # BF16 subnormals
    rows[6 % n] = rng.standard_normal(D) * 1e-7                 # range below the smallest fp16 normal
    rows[7 % n] = rng.standard_normal(D) * 3e3                  # large range
    rows[8 % n] = 1e-30
    rows[9 % n] = np.where(np.arange(D) == 3, 7e4, 1.0)         # zero fits, scale fits
    rows[10 % n] = np.where(np.arange(D) == 5, -7e4, 1.0)       # minimum below -65504: saturates
    rows[11 % n] = np.where(np.arange(D) == 5, 3e7, -3e7)       # scale above 65504: saturates
    rows[12 % n] = -rng.random(D).astype(np.float32) * 1e-6
    rows[13 % n] = 65504.0 - (np.arange(D) % 4) * 32.0
    return wl.f32_to_bf16_words(x)


SHAPES = [  # (L, H, D, T, group)
    (2, 2, 64, 128, 64),     # the Tiny configuration: 4 blocks per tile
    (1, 2, 128, 100, 128),   # ragged: 6.25 blocks
    (1, 1, 128, 1, 128),     # a single token
    (2, 1, 96, 40, 32),      # head_dim that is not a power of two
    (1, 2, 128, 272, 64),    # 17 blocks: spans several workgroups
    (1, 1, 256, 24, 256),
    (1, 1, 64, 7, 32),       # less than one block
    (1, 2, 512, 21, 512),    # the widest group: one per row, one scale/zero entry per plane
    (1, 1, 512, 5, 256),
]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("prec", [B.PREC_16, B.PREC_INT8, B.PREC_INT4])
def test_quantize_pack_bytes_equal_oracle(shape, prec):
    L, H, D, T, g = shape
    ctx = B.Context(L, H, D, max(T, 1), group_int8=g, group_int4=g)
    for seed, maker in [(1, lambda: wl.kv_chunk(L, H, D, T, 1)),
                        (2, lambda: wl.kv_chunk(L, H, D, T, 2, key_spread=False, outlier_channels=2)),
                        (3, lambda: special_values_chunk(L, H, D, T, 3))]:
        src = maker()
        ref, ref_sat = codec.quantize_pack_chunk(src, B.BITS[prec], g)
        got, got_sat = gpu_quantize(ctx, src, prec, g)
        bad = np.flatnonzero(got != ref)
        assert bad.size == 0, f"seed {seed}: {bad.size} bytes differ, first at {bad[:5]}"
        assert got_sat == ref_sat
    ctx.destroy()


@pytest.mark.parametrize("prec,g", [(B.PREC_INT8, 128), (B.PREC_INT4, 64), (B.PREC_INT8, 32)])
def test_quantize_codes_bit_exact_on_tens_of_millions_of_elements(prec, g):
    """The kernel divides by a shared refined reciprocal; the oracle by IEEE division.
    Rows get widely different magnitudes and offsets so that scales, zeros and quotients
    cover many binades and many near-half-integer quotients occur."""
    L, H, D, T = 16, 8, 128, 1024                      # 33.5 M elements
    rng = np.random.Generator(np.random.PCG64(99 + prec + g))
    x = rng.standard_normal((L, 2, H, T, D), dtype=np.float32)
    x *= np.exp(rng.normal(0, 2.5, (L, 2, H, T, 1))).astype(np.float32)
    x += (rng.normal(0, 3, (L, 2, H, T, 1)) * np.exp(rng.normal(0, 2, (L, 2, H, T, 1)))).astype(np.float32)
    # a share of rows on a coarse grid: many exact ties
    x[:, :, :, ::7] = np.round(x[:, :, :, ::7] * 2) / 2
    src = wl.f32_to_bf16_words(x)
    ctx = B.Context(L, H, D, T, group_int8=g, group_int4=g)
    ref, ref_sat = codec.quantize_pack_chunk(src, B.BITS[prec], g)
    got, got_sat = gpu_quantize(ctx, src, prec, g)
    bad = np.flatnonzero(got != ref)
    assert bad.size == 0, f"{bad.size} bytes differ, first at {bad[:5]}"
    assert got_sat == ref_sat
    ctx.destroy()


@pytest.mark.parametrize("prec", sorted(ORC))
def test_a_class_of_chunks_in_one_launch_equals_chunk_by_chunk_oracle(prec):
    """ha_rag_quantize_chunks: ragged lengths in one launch, bytes equal to the oracle's for
    every chunk, nothing written past any chunk, the saturation count summed."""
    L, H, D, g = 2, 2, 128, 64
    tokens = [1, 40, 16, 77, 130, 5, 64]
    ctx = B.Context(L, H, D, max(tokens), group_int8=g, group_int4=g)
    srcs = [special_values_chunk(L, H, D, t, 50 + i) if i % 3 == 0 else wl.kv_chunk(L, H, D, t, 60 + i)
            for i, t in enumerate(tokens)]
    refs = [codec.quantize_pack_chunk(s_, ORC[prec], g) for s_ in srcs]
    dsrc = [dev_u16(s_) for s_ in srcs]
    ddst = [torch.full((len(r[0]) + 64,), 0xAB, dtype=torch.uint8, device="cuda") for r in refs]
    sat = torch.zeros(1, dtype=torch.int32, device="cuda")
    ctx.quantize_chunks(dsrc, tokens, prec, g, ddst, saturated=sat)
    torch.cuda.synchronize()
    for i, (ref, _) in enumerate(refs):
        got = ddst[i].cpu().numpy()
        assert np.array_equal(got[:len(ref)], ref), i
        assert np.all(got[len(ref):] == 0xAB), i
    if prec in (B.PREC_INT8, B.PREC_INT4):
        assert int(sat.item()) == sum(r[1] for r in refs)
    ctx.destroy()


def test_more_chunks_than_one_quantize_launch_holds():
    L, H, D, T, g = 1, 1, 64, 20, 64
    n = 150                                              # two launches of at most 128 descriptors
    ctx = B.Context(L, H, D, T, group_int8=g, group_int4=g)
    srcs = [wl.kv_chunk(L, H, D, T - i % 7, 900 + i) for i in range(n)]
    tokens = [T - i % 7 for i in range(n)]
    dsrc = [dev_u16(s_) for s_ in srcs]
    ddst = [torch.zeros(ctx.chunk_bytes(B.PREC_INT4, t), dtype=torch.uint8, device="cuda") for t in tokens]
    ctx.quantize_chunks(dsrc, tokens, B.PREC_INT4, g, ddst)
    torch.cuda.synchronize()
    for i in range(n):
        assert np.array_equal(ddst[i].cpu().numpy(), codec.quantize_pack_chunk(srcs[i], 4, g)[0]), i
    # a bad chunk anywhere in the list: nothing is enqueued
    with pytest.raises(B.HaRagError) as e:
        ctx.quantize_chunks(dsrc[:3], [T, T + 100000000, T], B.PREC_INT4, g, ddst[:3])
    assert e.value.code in (B.EINVAL, B.EFORMAT)
    ctx.destroy()


def _load_case(shape, tokens, precs, g, order, seed, cap_extra=0, tok_base=0, launch=None):
    L, H, D = shape
    ctx = B.Context(L, H, D, max(tokens), group_int8=g, group_int4=g)
    if launch:
        ctx.set_launch_params(*launch)
    srcs = [wl.kv_chunk(L, H, D, t, seed * 100 + i) if i % 2 else special_values_chunk(L, H, D, t, seed + i)
            for i, t in enumerate(tokens)]
    packed = [codec.quantize_pack_chunk(s, B.BITS[p], g)[0] for s, p in zip(srcs, precs)]
    total = sum(tokens[c] for c in order)
    cap = tok_base + total + cap_extra
    ref = np.full((L, 2, H, cap, D), CANARY, np.uint16)
    codec.load_chunks(packed, shape, tokens, [B.BITS[p] for p in precs], [g] * len(tokens), order,
                      cap_tokens=cap, tok_base=tok_base, out=ref)
    dev = [dev_u8(p) for p in packed]
    out = torch.full((L, 2, H, cap, D), CANARY, dtype=torch.int16, device="cuda")
    ctx.load_packed([(dev[c], tokens[c], precs[c], g) for c in order], out, cap, tok_base)
    torch.cuda.synchronize()
    got = host_u16(out)
    ctx.destroy()
    return got, ref


def test_tiny_configuration_gather_order_3_0_2_1():
    tiny = wl.tiny_config(0)
    L, H, D = tiny["shape"]
    ctx = B.Context(L, H, D, 128, group_int8=64, group_int4=64)
    precs = [B.PREC_OF_BITS[b] for b in tiny["bits"]]
    # GPU builds the knowledge base; bytes must equal the oracle's
    packed_ref = [codec.quantize_pack_chunk(c, b, 64)[0] for c, b in zip(tiny["chunks"], tiny["bits"])]
    packed_dev = []
    for c, p, ref in zip(tiny["chunks"], precs, packed_ref):
        got, _ = gpu_quantize(ctx, c, p, 64)
        assert np.array_equal(got, ref)
        packed_dev.append(dev_u8(got))
    ref, offs = codec.load_chunks(packed_ref, (L, H, D), tiny["tokens"], tiny["bits"], tiny["group"],
                                  tiny["order"])
    out = torch.zeros((L, 2, H, 512, D), dtype=torch.int16, device="cuda")
    ctx.load_packed([(packed_dev[c], 128, precs[c], 64) for c in tiny["order"]], out, 512)
    torch.cuda.synchronize()
    got = host_u16(out)
    assert ulp_distance(got, ref).max() <= 1
    assert np.array_equal(got, ref)                      # in fact identical
    # the 16-bit chunk (id 0) sits second and is the source, word for word
    assert np.array_equal(got[:, :, :, 128:256], tiny["chunks"][0])
    ctx.destroy()


@pytest.mark.parametrize("launch", [None, (64, 1, 2, 0, 1), (256, 2, 4, 1, 0), (512, 4, 2, 0, 0),
                                    (1024, 1, 4, 1, 1), (128, 2, 2, 1, 1), (64, 4, 4, 1, 0)])
def test_load_mixed_tags_ragged_tokens_all_launch_shapes(launch):
    tokens = [100, 1, 272, 7, 33, 64]
    precs = [B.PREC_INT4, B.PREC_16, B.PREC_INT8, B.PREC_INT4, B.PREC_INT8, B.PREC_16]
    order = [5, 2, 0, 3, 1, 4, 2]                        # a repeated chunk is loaded twice
    got, ref = _load_case((1, 2, 128), tokens, precs, 64, order, seed=5, cap_extra=9, tok_base=3,
                          launch=launch)
    finite = ref != CANARY
    assert np.array_equal(got == CANARY, ~finite)        # untouched rows keep the canary
    assert ulp_distance(got[finite], ref[finite]).max() <= 1
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("shape,g", [((2, 2, 64), 64), ((2, 1, 96), 32), ((1, 1, 256), 256),
                                     ((1, 2, 128), 128), ((1, 1, 128), 32), ((1, 2, 512), 512),
                                     ((1, 1, 512), 256)])
def test_load_shapes_and_groups(shape, g):
    tokens = [40, 128, 17]
    precs = [B.PREC_INT4, B.PREC_INT8, B.PREC_INT4]
    got, ref = _load_case(shape, tokens, precs, g, [2, 0, 1], seed=9, cap_extra=5)
    assert np.array_equal(got, ref)


def test_more_chunks_than_one_launch_holds():
    n = 150                                              # 3 launches of at most 64 descriptors
    tokens = [1 + (i * 7) % 13 for i in range(n)]
    precs = [(B.PREC_INT4, B.PREC_INT8, B.PREC_16)[i % 3] for i in range(n)]
    order = list(np.random.default_rng(0).permutation(n))
    got, ref = _load_case((1, 1, 64), tokens, precs, 64, order, seed=11)
    assert np.array_equal(got, ref)


def test_the_most_chunks_one_call_takes_and_one_more():
    """HA_RAG_MAX_REQUEST_CHUNKS = 4096 descriptors (64 launches), every tag, 1..3 tokens each,
    some of them empty; 4097 is refused before anything is enqueued."""
    L, H, D, g = 1, 1, 64, 32
    precs_all = sorted(ORC)
    n = 4096
    rng = np.random.default_rng(12)
    tokens = rng.integers(0, 4, n).tolist()
    precs = [precs_all[i % 6] for i in range(n)]
    base = {}
    for p in precs_all:                       # one source per (tag, length): contents repeat, slots do not
        for t in range(4):
            src = wl.kv_chunk(L, H, D, t, 300 + 7 * p + t) if t else np.zeros((L, 2, H, 0, D), np.uint16)
            base[(p, t)] = codec.quantize_pack_chunk(src, ORC[p], g)[0]
    packed = [base[(precs[i], tokens[i])] for i in range(n)]
    cap = sum(tokens) + 1
    ref = np.full((L, 2, H, cap, D), CANARY, np.uint16)
    codec.load_chunks(packed, (L, H, D), tokens, [ORC[p] for p in precs], [g] * n, list(range(n)),
                      cap_tokens=cap, out=ref)
    ctx = B.Context(L, H, D, 4, group_int8=g, group_int4=g)
    dev = {k: dev_u8(np.concatenate([v, np.zeros(16, np.uint8)])) for k, v in base.items()}
    chunks = [(dev[(precs[i], tokens[i])], tokens[i], precs[i], g) for i in range(n)]
    out = torch.full((L, 2, H, cap, D), CANARY, dtype=torch.int16, device="cuda")
    ctx.load_packed(chunks, out, cap)
    torch.cuda.synchronize()
    assert np.array_equal(host_u16(out), ref)
    out.fill_(CANARY)
    with pytest.raises(B.HaRagError) as e:
        ctx.load_packed(chunks + [chunks[0]], out, cap + 8)
    assert e.value.code == B.EINVAL
    torch.cuda.synchronize()
    assert bool((out == CANARY).all())
    ctx.destroy()


@pytest.mark.parametrize("prec", [B.PREC_INT4, B.PREC_16])
def test_one_very_long_chunk(prec):
    """100,003 tokens in one chunk: 3,126 blocks per tile and a ragged last block."""
    L, H, D, g, T = 1, 1, 64, 64, 100_003
    src = wl.kv_chunk(L, H, D, T, 77)
    ctx = B.Context(L, H, D, T, group_int8=g, group_int4=g)
    got_pack, _ = gpu_quantize(ctx, src, prec, g)
    ref_pack, _ = codec.quantize_pack_chunk(src, ORC[prec], g)
    assert np.array_equal(got_pack, ref_pack)
    ref = np.full((L, 2, H, T + 2, D), CANARY, np.uint16)
    codec.dequant_scatter_chunk(ref_pack, (L, H, D), T, ORC[prec], g, ref, 1)
    out = torch.full((L, 2, H, T + 2, D), CANARY, dtype=torch.int16, device="cuda")
    ctx.load_packed([(dev_u8(got_pack), T, prec, g)], out, T + 2, 1)
    torch.cuda.synchronize()
    assert np.array_equal(host_u16(out), ref)
    ctx.destroy()


def test_empty_and_error_calls_touch_nothing():
    ctx = B.Context(2, 2, 64, 128, group_int8=64, group_int4=64)
    out = torch.full((2, 2, 2, 64, 64), CANARY, dtype=torch.int16, device="cuda")
    ctx.load_packed([], out, 64)
    src = wl.kv_chunk(2, 2, 64, 48, 1)
    p = dev_u8(codec.quantize_pack_chunk(src, 4, 64)[0])
    with pytest.raises(B.HaRagError) as e:
        ctx.load_packed([(p, 48, B.PREC_INT4, 64), (p, 48, B.PREC_INT4, 64)], out, 64)   # 96 > 64
    assert e.value.code == B.ENOSPC
    with pytest.raises(B.HaRagError) as e:
        ctx.load_packed([(p, 48, B.PREC_INT4, 128)], out, 64)                            # 128 does not divide 64
    assert e.value.code == B.EFORMAT
    with pytest.raises(B.HaRagError) as e:
        ctx.load_packed([(p.data_ptr() + 4, 48, B.PREC_INT4, 64)], out, 64)              # misaligned
    assert e.value.code == B.EINVAL
    with pytest.raises(B.HaRagError) as e:
        ctx.quantize_chunk(p, 48, B.PREC_INT4, 48, p)
    assert e.value.code == B.EFORMAT
    torch.cuda.synchronize()
    assert np.all(host_u16(out) == CANARY)
    ctx.destroy()


# ---- FP8 tags (the paper's schemes S2 and S3) ------------------------------------------
@pytest.mark.parametrize("prec", [B.PREC_FP8_E4M3, B.PREC_FP8_E5M2])
def test_fp8_encode_every_finite_bf16_value(prec):
    words = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    f = wl.bf16_words_to_f32(words)
    words = np.where(np.isfinite(f), words, 0).astype(np.uint16)       # inputs are finite by contract
    src = words.reshape(1, 2, 1, 256, 128)
    ctx = B.Context(1, 1, 128, 256)
    ref, _ = codec.quantize_pack_chunk(src, ORC[prec])
    got, _ = gpu_quantize(ctx, src, prec, 0)
    bad = np.flatnonzero(got != ref)
    assert bad.size == 0, f"{bad.size} codes differ, first at {bad[:8]}"
    ctx.destroy()


@pytest.mark.parametrize("prec", [B.PREC_FP8_E4M3, B.PREC_FP8_E5M2])
def test_fp8_decode_every_code(prec):
    kind = ORC[prec]
    codes = np.arange(256, dtype=np.uint8)
    finite = np.array([np.isfinite(codec.fp8_to_f64(int(c), kind)) for c in codes])
    codes = np.where(finite, codes, 0).astype(np.uint8)                 # NaN / inf codes are never written
    L, H, D, T = 1, 1, 128, 32                                           # 2 blocks per tile
    per_tile = np.tile(codes, T * D // 256)
    # build the packed chunk through the oracle's layout: one byte per element
    packed = np.zeros(codec.chunk_bytes(L, H, D, T, kind), np.uint8)
    for tile in range(2):
        for e in range(T * D):
            packed[tile * 4096 + codec.octet_offset(e, 8) + e % 8] = per_tile[(e + 37 * tile) % per_tile.size]
    ref = np.zeros((L, 2, H, T, D), np.uint16)
    codec.dequant_scatter_chunk(packed, (L, H, D), T, kind, 128, ref, 0)
    ctx = B.Context(L, H, D, T)
    out = torch.zeros((L, 2, H, T, D), dtype=torch.int16, device="cuda")
    ctx.load_packed([(dev_u8(packed), T, prec, 0)], out, T)
    torch.cuda.synchronize()
    assert np.array_equal(host_u16(out), ref)
    ctx.destroy()


# ---- GSE-8 (the paper's scheme S4) -------------------------------------------------------
def _gse_roundtrip(src, T):
    L, _, H, _, D = src.shape
    ctx = B.Context(L, H, D, T, group_int8=32, group_int4=32)
    ref, _ = codec.quantize_pack_chunk(src, 143)
    got, _ = gpu_quantize(ctx, src, B.PREC_GSE8, 0)
    bad = np.flatnonzero(got != ref)
    assert bad.size == 0, f"{bad.size} bytes differ, first at {bad[:8]}"
    ref_out = np.full((L, 2, H, T + 2, D), CANARY, np.uint16)
    codec.dequant_scatter_chunk(ref, (L, H, D), T, 143, 0, ref_out, 1)
    out = torch.full((L, 2, H, T + 2, D), CANARY, dtype=torch.int16, device="cuda")
    ctx.load_packed([(dev_u8(got), T, B.PREC_GSE8, 0)], out, T + 2, 1)
    torch.cuda.synchronize()
    assert np.array_equal(host_u16(out), ref_out)
    ctx.destroy()


def test_gse8_every_finite_bf16_value_in_tiles_of_different_ranges():
    words = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    f = wl.bf16_words_to_f32(words)
    words = np.where(np.isfinite(f), words, 0).astype(np.uint16)
    tiles = []
    # tile 0: everything (range clipped to 48 binades below the top); the others: slices of
    # the exponent axis, among them BF16 subnormals only, and an all-zero tile
    for lo_e, hi_e in [(0, 255), (100, 140), (120, 128), (0, 1), (1, 30), (126, 127), (200, 254), (0, 0)]:
        e = (words >> 7) & 0xFF
        keep = (e >= lo_e) & (e <= hi_e) if hi_e else (words & 0x7FFF) == 0
        tiles.append(np.where(keep, words, 0).astype(np.uint16))
    src = np.stack(tiles).reshape(2, 2, 2, 512, 128)
    _gse_roundtrip(src, 512)


@pytest.mark.parametrize("shape", [(2, 2, 64, 128), (1, 2, 128, 100), (1, 1, 128, 1), (2, 1, 96, 40),
                                   (1, 2, 128, 272)])
def test_gse8_shapes(shape):
    L, H, D, T = shape
    _gse_roundtrip(wl.kv_chunk(L, H, D, T, 77, outlier_channels=1), T)
    _gse_roundtrip(special_values_chunk(L, H, D, T, 78), T)


def test_all_six_tags_in_one_request_through_the_pool():
    L, H, D, T, g = 2, 2, 128, 72, 64
    precs = [B.PREC_FP8_E5M2, B.PREC_INT4, B.PREC_16, B.PREC_FP8_E4M3, B.PREC_INT8, B.PREC_GSE8]
    tokens = [72, 40, 9, 72, 33, 1]
    ctx = _pool_ctx(L, H, D, T, g, hbm_slots=2, pin_slots=3, stg_slots=2, tau_gpu_ppm=400_000,
                    precs=sorted(set(precs)))
    srcs = [wl.kv_chunk(L, H, D, t, 900 + i, outlier_channels=1) for i, t in enumerate(tokens)]
    packed = []
    for i, (s_, p, t) in enumerate(zip(srcs, precs, tokens)):
        ref, _ = codec.quantize_pack_chunk(s_, ORC[p], g)
        got, _ = gpu_quantize(B.Context(L, H, D, t, group_int8=g, group_int4=g), s_, p, g)
        assert np.array_equal(got, ref), f"chunk {i}"
        packed.append(ref)
        ctx.pool_insert(i, p, t, dev_u8(got), B.TIER_PINNED, packed_is_device=True)
    torch.cuda.synchronize()
    ctx.set_counts(list(range(6)), [9, 8, 7, 6, 5, 4])
    ctx.rerank()                                             # GPU_LIST = ids 0, 1
    for order in ([5, 0, 3, 1, 4, 2], [0, 1, 2, 3, 4, 5, 0]):
        total = sum(tokens[c] for c in order)
        out = torch.full((L, 2, H, total + 3, D), CANARY, dtype=torch.int16, device="cuda")
        st, _ = ctx.load_chunks(order, out, total + 3, tok_base=1, tags=[precs[c] for c in order])
        torch.cuda.synchronize()
        ref = np.full((L, 2, H, total + 3, D), CANARY, np.uint16)
        codec.load_chunks(packed, (L, H, D), tokens, [ORC[p] for p in precs], [g] * 6, order,
                          cap_tokens=total + 3, tok_base=1, out=ref)
        assert np.array_equal(host_u16(out), ref), order
    assert st["n_hbm_hits"] == 3                             # ids 0, 1 promoted by the first request
    ctx.destroy()


# ---- pools, cold path, promotion -------------------------------------------------
def _pool_ctx(L, H, D, T, g, hbm_slots, pin_slots, stg_slots, tau_gpu_ppm, precs, pinned_dma=False):
    ctx = B.Context(L, H, D, T, group_int8=g, group_int4=g, tau_gpu_ppm=tau_gpu_ppm,
                    pinned_dma=pinned_dma)
    keep = []
    biggest = 0
    for p in precs:
        slot = (ctx.chunk_bytes(p, T) + 255) // 256 * 256
        biggest = max(biggest, slot)
        if hbm_slots:
            hb = torch.zeros(slot * hbm_slots, dtype=torch.uint8, device="cuda")
            ctx.register_slab(B.TIER_HBM, p, hb)
        pn = torch.zeros(slot * pin_slots, dtype=torch.uint8).pin_memory()
        ctx.register_slab(B.TIER_PINNED, p, pn)
    if stg_slots:
        ctx.register_staging(torch.zeros(biggest * stg_slots, dtype=torch.uint8, device="cuda"))
    return ctx


def test_pool_cold_path_promotion_and_hits_match_oracle():
    L, H, D, T, g = 2, 2, 64, 128, 64
    n = 12
    precs_all = [B.PREC_INT4, B.PREC_INT8, B.PREC_16]
    ctx = _pool_ctx(L, H, D, T, g, hbm_slots=2, pin_slots=n, stg_slots=3, tau_gpu_ppm=500_000,
                    precs=precs_all)
    tokens = [T - 5 * (i % 4) for i in range(n)]
    precs = [precs_all[i % 3] for i in range(n)]
    srcs = [wl.kv_chunk(L, H, D, tokens[i], 40 + i) for i in range(n)]
    packed = [codec.quantize_pack_chunk(s, B.BITS[p], g)[0] for s, p in zip(srcs, precs)]
    for i in range(n):
        ctx.pool_insert(i, precs[i], tokens[i], packed[i], B.TIER_PINNED)
    ctx.set_counts(list(range(n)), [100 - i for i in range(n)])
    ctx.rerank()                                         # GPU_LIST = ids 0..5

    def run(req, base=0):
        total = sum(tokens[c] for c in req)
        cap = base + total + 4
        out = torch.full((L, 2, H, cap, D), CANARY, dtype=torch.int16, device="cuda")
        st, tr = ctx.load_chunks(req, out, cap, tok_base=base, want_trace=True,
                                 tags=[precs[c] for c in req])
        torch.cuda.synchronize()
        ref = np.full((L, 2, H, cap, D), CANARY, np.uint16)
        codec.load_chunks(packed, (L, H, D), tokens, [B.BITS[p] for p in precs], [g] * n, req,
                          cap_tokens=cap, tok_base=base, out=ref)
        assert np.array_equal(host_u16(out), ref), req
        return st, tr

    # all cold; 7 cold chunks through 3 staging slots; ids 0..5 are promoted while slots last
    st, tr = run([7, 0, 3, 9, 1, 4, 11], base=2)
    assert st["n_pinned_hits"] == 7 and st["n_hbm_hits"] == 0
    assert [t.promoted for t in tr] == [0, 1, 1, 0, 1, 1, 0]
    assert st["bytes_h2d"] == sum(len(packed[c]) for c in [7, 0, 3, 9, 1, 4, 11])
    for c in (0, 3, 1, 4):
        info = ctx.pool_query(c)
        assert info.in_hbm and info.in_pinned
    # the promoted copies are now served from HBM (and must hold the master's bytes)
    st, tr = run([0, 3, 1, 4, 0])
    assert st["n_hbm_hits"] == 5 and st["n_pinned_hits"] == 0 and st["bytes_h2d"] == 0
    # a request mixing hits, cold chunks, a promotion that evicts, and a repeat of the promoted id
    st, tr = run([0, 6, 2, 3, 2, 10])
    assert [t.found_tier for t in tr] == [B.TIER_HBM, B.TIER_PINNED, B.TIER_PINNED, B.TIER_HBM,
                                          B.TIER_HBM, B.TIER_PINNED]
    assert [t.promoted for t in tr] == [0, 0, 1, 0, 0, 0]
    # fill the int4 slab's two slots with 0 and 3, then promote... 9 is outside GPU_LIST;
    # give it a rank inside and watch it evict the least recently used (0 was used last -> 3 goes)
    ctx.set_counts([9], [1000])
    ctx.rerank()
    st, tr = run([3, 0, 9])
    assert tr[2].promoted == 1 and tr[2].evicted_id == 3
    st, tr = run([9, 3])
    assert [t.found_tier for t in tr] == [B.TIER_HBM, B.TIER_PINNED]
    ctx.destroy()


def test_pinned_chunks_read_by_the_kernel_itself():
    """Chunks that stay in pinned memory are dequantized straight from it (one launch, no staging
    traffic) unless pinned_dma is set; chunks that are promoted pass through staging; the
    result is the same either way."""
    L, H, D, T, g = 2, 2, 64, 96, 32
    n = 10
    precs_all = [B.PREC_INT4, B.PREC_INT8, B.PREC_FP8_E5M2]
    tokens = [T - 11 * (i % 4) for i in range(n)]
    precs = [precs_all[i % 3] for i in range(n)]
    packed = [codec.quantize_pack_chunk(wl.kv_chunk(L, H, D, tokens[i], 700 + i), ORC[precs[i]], g)[0]
              for i in range(n)]
    req = [7, 0, 3, 9, 1, 4, 8, 0]
    cap = sum(tokens[c] for c in req) + 1
    ref = np.full((L, 2, H, cap, D), CANARY, np.uint16)
    codec.load_chunks(packed, (L, H, D), tokens, [ORC[p] for p in precs], [g] * n, req, cap_tokens=cap,
                      out=ref)
    for zero_copy in (True, False):
        ctx = B.Context(L, H, D, T, group_int8=g, group_int4=g, tau_gpu_ppm=300_000,
                        pinned_dma=not zero_copy)
        big = 0
        for p in precs_all:
            slot = (ctx.chunk_bytes(p, T) + 255) // 256 * 256
            big = max(big, slot)
            ctx.register_slab(B.TIER_HBM, p, torch.zeros(slot * 2, dtype=torch.uint8, device="cuda"))
            ctx.register_slab(B.TIER_PINNED, p, torch.zeros(slot * n, dtype=torch.uint8).pin_memory())
        ctx.register_staging(torch.zeros(big * 2, dtype=torch.uint8, device="cuda"))
        for i in range(n):
            ctx.pool_insert(i, precs[i], tokens[i], packed[i], B.TIER_PINNED)
        ctx.set_counts(list(range(n)), [100 - i for i in range(n)])
        ctx.rerank()                                   # GPU_LIST = ids 0, 1, 2
        out = torch.full((L, 2, H, cap, D), CANARY, dtype=torch.int16, device="cuda")
        st, tr = ctx.load_chunks(req, out, cap, want_trace=True)
        torch.cuda.synchronize()
        assert np.array_equal(host_u16(out), ref), zero_copy
        assert [t.promoted for t in tr] == [0, 1, 0, 0, 1, 0, 0, 0]
        # promoted chunks go through staging (one launch each); the others share one launch
        assert st["n_kernel_launches"] == (4 if zero_copy else 8)
        out.fill_(CANARY)
        st, tr = ctx.load_chunks(req, out, cap, want_trace=True)
        torch.cuda.synchronize()
        assert np.array_equal(host_u16(out), ref), zero_copy
        assert st["n_kernel_launches"] == (1 if zero_copy else 6)
        ctx.destroy()


def test_explicit_promote_evict_and_insert_from_device():
    L, H, D, T, g = 1, 2, 128, 64, 128
    ctx = _pool_ctx(L, H, D, T, g, hbm_slots=2, pin_slots=4, stg_slots=2, tau_gpu_ppm=0,
                    precs=[B.PREC_INT4])
    srcs = [wl.kv_chunk(L, H, D, T, 70 + i) for i in range(4)]
    packed = [codec.quantize_pack_chunk(s, 4, g)[0] for s in srcs]
    # chunk 0: quantized by the GPU straight into a reserved pinned... HBM slot
    ctx.pool_insert(0, B.PREC_INT4, T, None, B.TIER_HBM)
    ptr, nb = ctx.pool_slot(0, B.TIER_HBM)
    ctx.quantize_chunk(dev_u16(srcs[0]), T, B.PREC_INT4, g, ptr)
    # chunk 1: device bytes -> pinned master; chunk 2, 3: host bytes -> pinned
    ctx.pool_insert(1, B.PREC_INT4, T, dev_u8(packed[1]), B.TIER_PINNED, packed_is_device=True)
    ctx.pool_insert(2, B.PREC_INT4, T, packed[2], B.TIER_PINNED)
    ctx.pool_insert(3, B.PREC_INT4, T, packed[3], B.TIER_PINNED)
    torch.cuda.synchronize()
    ctx.pool_promote(1)
    assert ctx.pool_query(1).in_hbm == 1
    with pytest.raises(B.HaRagError) as e:                 # 0 has no master, 1 ... evictable
        ctx.pool_evict(0)
    assert e.value.code == B.EINVAL
    ctx.pool_promote(2)                                    # evicts 1 (LRU among evictable)
    assert ctx.pool_query(1).in_hbm == 0 and ctx.pool_query(2).in_hbm == 1
    order = [2, 0, 1, 3]
    out = torch.zeros((L, 2, H, 4 * T, D), dtype=torch.int16, device="cuda")
    st, _ = ctx.load_chunks(order, out, 4 * T)
    torch.cuda.synchronize()
    ref, _ = codec.load_chunks(packed, (L, H, D), [T] * 4, [4] * 4, [g] * 4, order)
    assert np.array_equal(host_u16(out), ref)
    assert st["n_hbm_hits"] == 2 and st["n_pinned_hits"] == 2 and st["n_promoted"] == 0
    ctx.destroy()


def test_concurrent_requests_on_separate_streams():
    """Four requests, each on its own stream, all chunks cold and distinct, sharing
    a staging ring smaller than one request."""
    L, H, D, T, g = 2, 2, 64, 128, 64
    n_req, per = 4, 6
    ctx = _pool_ctx(L, H, D, T, g, hbm_slots=0, pin_slots=n_req * per, stg_slots=4, tau_gpu_ppm=0,
                    precs=[B.PREC_INT4])
    srcs = [wl.kv_chunk(L, H, D, T, 200 + i) for i in range(n_req * per)]
    packed = [codec.quantize_pack_chunk(s, 4, g)[0] for s in srcs]
    for i, p in enumerate(packed):
        ctx.pool_insert(i, B.PREC_INT4, T, p, B.TIER_PINNED)
    streams = [torch.cuda.Stream() for _ in range(n_req)]
    outs = [torch.zeros((L, 2, H, per * T, D), dtype=torch.int16, device="cuda") for _ in range(n_req)]
    torch.cuda.synchronize()
    for rep in range(2):
        for r in range(n_req):
            ids = list(range(r * per, (r + 1) * per))
            ctx.load_chunks(ids, outs[r], per * T, stream=streams[r])
    torch.cuda.synchronize()
    for r in range(n_req):
        ids = list(range(r * per, (r + 1) * per))
        ref, _ = codec.load_chunks(packed, (L, H, D), [T] * len(packed), [4] * len(packed),
                                   [g] * len(packed), ids)
        assert np.array_equal(host_u16(outs[r]), ref)
    ctx.destroy()


def test_short_lived_streams_are_forgotten():
    """A caller that makes a stream per request and destroys it afterwards: ha_rag_forget_stream
    takes the stream out of the library's books before it goes, so that stream after stream
    (handles come back) promote, evict and load the same few slots correctly."""
    L, H, D, T, g = 2, 2, 64, 128, 64
    n = 8
    ctx = _pool_ctx(L, H, D, T, g, hbm_slots=2, pin_slots=n, stg_slots=2, tau_gpu_ppm=1_000_000,
                    precs=[B.PREC_INT4])
    packed = [codec.quantize_pack_chunk(wl.kv_chunk(L, H, D, T, 260 + i), 4, g)[0] for i in range(n)]
    for i, p in enumerate(packed):
        ctx.pool_insert(i, B.PREC_INT4, T, p, B.TIER_PINNED)
    ctx.rerank()                                   # every chunk belongs in HBM: two slots, constant eviction
    ctx.forget_stream(torch.cuda.Stream())         # a stream the context has never seen: nothing to do
    for rep in range(12):
        s_ = torch.cuda.Stream()
        ids = [(3 * rep + k) % n for k in range(3)]
        out = torch.zeros((L, 2, H, 3 * T, D), dtype=torch.int16, device="cuda")
        with torch.cuda.stream(s_):
            ctx.load_chunks(ids, out, 3 * T, stream=s_)
        ctx.forget_stream(s_)                      # waits for what the library enqueued there
        ref, _ = codec.load_chunks(packed, (L, H, D), [T] * n, [4] * n, [g] * n, ids)
        assert np.array_equal(host_u16(out), ref), rep
        del s_
    ctx.destroy()


def test_batch_of_requests_one_call():
    L, H, D, T, g = 1, 2, 128, 96, 128
    n = 10
    ctx = _pool_ctx(L, H, D, T, g, hbm_slots=n, pin_slots=n, stg_slots=2, tau_gpu_ppm=1_000_000,
                    precs=[B.PREC_INT8])
    srcs = [wl.kv_chunk(L, H, D, T, 300 + i) for i in range(n)]
    packed = [codec.quantize_pack_chunk(s, 8, g)[0] for s in srcs]
    for i, p in enumerate(packed):
        ctx.pool_insert(i, B.PREC_INT8, T, p, B.TIER_PINNED)
        if i < 5:
            ctx.pool_insert(i, B.PREC_INT8, T, p, B.TIER_HBM)
    ctx.rerank()
    reqs = [[0, 7, 3], [9, 9, 1, 2], [4]]
    outs = [torch.zeros((L, 2, H, len(r) * T, D), dtype=torch.int16, device="cuda") for r in reqs]
    st, _ = ctx.load_batch(reqs, outs, [len(r) * T for r in reqs])
    torch.cuda.synchronize()
    for r, o in zip(reqs, outs):
        ref, _ = codec.load_chunks(packed, (L, H, D), [T] * n, [8] * n, [g] * n, r)
        assert np.array_equal(host_u16(o), ref)
    assert st["n_hbm_hits"] == 6 and st["n_pinned_hits"] == 2 and st["n_promoted"] == 2
    ctx.destroy()


# ---- four tiers: HBM, pinned, pageable, files -----------------------------------------
@pytest.mark.parametrize("o_direct", [False, True])
def test_four_tier_placement_end_to_end(tmp_path, o_direct):
    """Every chunk starts in a file.  Requests pull chunks through bounce buffers and the
    staging ring; Algorithm 2 leaves copies in HBM / pinned / pageable memory according to
    rank; whatever tier serves a chunk, the cache must equal the oracle's."""
    L, H, D, T, g = 2, 2, 64, 128, 64
    n = 12
    precs_all = [B.PREC_INT4, B.PREC_FP8_E4M3]
    ctx = B.Context(L, H, D, T, group_int8=g, group_int4=g, tau_gpu_ppm=170_000,
                    tau_pin_ppm=170_000, tau_page_ppm=250_000, disk_o_direct=o_direct)
    biggest = 0
    for p in precs_all:
        slot = (ctx.chunk_bytes(p, T) + 4095) // 4096 * 4096
        biggest = max(biggest, slot)
        ctx.register_slab(B.TIER_HBM, p, torch.zeros(slot * 1, dtype=torch.uint8, device="cuda"))
        ctx.register_slab(B.TIER_PINNED, p, torch.zeros(slot * 1, dtype=torch.uint8).pin_memory())
        ctx.register_slab(B.TIER_PAGEABLE, p, torch.zeros(slot * 2, dtype=torch.uint8))
        try:
            ctx.register_disk(p, str(tmp_path / f"pool_{p}.bin"), slot * n)
        except B.HaRagError as e:
            if o_direct and e.code == B.EIO:
                pytest.skip("this filesystem refuses O_DIRECT")
            raise
    ctx.register_staging(torch.zeros(biggest * 2, dtype=torch.uint8, device="cuda"))
    ctx.register_bounce(torch.zeros(biggest * 2, dtype=torch.uint8).pin_memory())
    tokens = [T - 7 * (i % 3) for i in range(n)]
    precs = [precs_all[i % 2] for i in range(n)]
    srcs = [wl.kv_chunk(L, H, D, tokens[i], 1200 + i) for i in range(n)]
    packed = [codec.quantize_pack_chunk(s_, ORC[p], g)[0] for s_, p in zip(srcs, precs)]
    for i in range(n):
        if i % 3 == 0:      # device bytes -> file (through a bounce buffer)
            ctx.pool_insert(i, precs[i], tokens[i], dev_u8(packed[i]), B.TIER_DISK, packed_is_device=True)
        else:               # host bytes -> file
            ctx.pool_insert(i, precs[i], tokens[i], packed[i], B.TIER_DISK)
    ctx.set_counts(list(range(n)), [100 - i for i in range(n)])
    ctx.rerank()            # lists: GPU {0,1}, PIN {2,3}, PAGE {4,5,6}, DISK the rest

    def run(req):
        total = sum(tokens[c] for c in req)
        out = torch.full((L, 2, H, total + 2, D), CANARY, dtype=torch.int16, device="cuda")
        st, tr = ctx.load_chunks(req, out, total + 2, tok_base=1, want_trace=True)
        torch.cuda.synchronize()
        ref = np.full((L, 2, H, total + 2, D), CANARY, np.uint16)
        codec.load_chunks(packed, (L, H, D), tokens, [ORC[p] for p in precs], [g] * n, req,
                          cap_tokens=total + 2, tok_base=1, out=ref)
        assert np.array_equal(host_u16(out), ref), req
        return st, tr

    st, tr = run([0, 2, 4, 9, 1, 3, 5, 6])
    assert [t.found_tier for t in tr] == [3] * 8
    assert [t.placed_tier for t in tr] == [0, 1, 2, 255, 0, 1, 2, 2]
    assert st["bytes_disk_read"] == sum(len(packed[c]) for c in [0, 2, 4, 9, 1, 3, 5, 6])
    # now served from where Algorithm 2 left them (one slot per tag in HBM / pinned, two in pageable)
    st, tr = run([0, 1, 2, 3, 4, 5, 6, 9, 0])
    assert [t.found_tier for t in tr] == [0, 0, 1, 1, 2, 2, 2, 3, 0]
    assert st["n_disk_hits"] == 1 and st["n_pageable_hits"] == 3
    # 8 and 10 are int4, 7 is e4m3: give 10 a GPU rank -> it evicts 0 from HBM (same tag slab)
    ctx.set_counts([10], [1000])
    ctx.rerank()
    st, tr = run([10, 7, 0, 10])
    assert tr[0].found_tier == 3 and tr[0].placed_tier == 0 and tr[0].evicted_id == 0
    assert tr[2].found_tier == 3                              # 0 lost its only fast copy
    assert tr[3].found_tier == 0
    # pageable insert from the host and from the device, then load
    ctx.pool_evict(4, B.TIER_PAGEABLE)
    ctx.pool_insert(4, precs[4], tokens[4], packed[4], B.TIER_PAGEABLE)
    st, tr = run([4, 11, 8])
    assert tr[0].found_tier == 2
    ctx.destroy()


def test_file_read_failure_is_reported_and_rolled_back(tmp_path):
    L, H, D, T, g = 1, 2, 64, 64, 64
    ctx = B.Context(L, H, D, T, group_int8=g, group_int4=g, tau_gpu_ppm=1_000_000)
    p = B.PREC_INT8
    slot = (ctx.chunk_bytes(p, T) + 4095) // 4096 * 4096
    ctx.register_slab(B.TIER_HBM, p, torch.zeros(slot * 4, dtype=torch.uint8, device="cuda"))
    path = tmp_path / "pool.bin"
    ctx.register_disk(p, str(path), slot * 4)
    ctx.register_staging(torch.zeros(slot * 2, dtype=torch.uint8, device="cuda"))
    ctx.register_bounce(torch.zeros(slot * 2, dtype=torch.uint8).pin_memory())
    srcs = [wl.kv_chunk(L, H, D, T, 1300 + i) for i in range(3)]
    packed = [codec.quantize_pack_chunk(s_, 8, g)[0] for s_ in srcs]
    for i in range(3):
        ctx.pool_insert(i, p, T, packed[i], B.TIER_DISK)
    ctx.rerank()                                       # everything belongs to GPU_LIST
    out = torch.zeros((L, 2, H, 3 * T, D), dtype=torch.int16, device="cuda")
    st, _ = ctx.load_chunks([0], out, 3 * T)
    assert st["n_promoted"] == 1 and ctx.pool_query(0).in_hbm == 1
    with open(path, "r+b") as f:                       # the pool file loses chunks 1 and 2
        f.truncate(slot)
    with pytest.raises(B.HaRagError) as e:
        ctx.load_chunks([0, 1, 2], out, 3 * T)
    assert e.value.code == B.EIO and "pread" in str(e.value)
    torch.cuda.synchronize()
    assert ctx.pool_query(1).in_hbm == 0 and ctx.pool_query(2).in_hbm == 0   # booked copies undone
    assert ctx.pool_query(1).count == 1                # the access itself was counted
    # the context keeps working: chunk 0 is still served from HBM, correctly
    out.fill_(0)
    st, _ = ctx.load_chunks([0], out, 3 * T)
    torch.cuda.synchronize()
    ref, _ = codec.load_chunks(packed, (L, H, D), [T] * 3, [8] * 3, [g] * 3, [0], cap_tokens=3 * T)
    assert st["n_hbm_hits"] == 1 and np.array_equal(host_u16(out), ref)
    ctx.destroy()


# ---- the benchmark's own shapes and launch configuration ----------------------------
def _check_sampled_tiles(ctx, shape, T, g, precs, order, srcs, packs, out, n_samples, rng):
    """K/V tile pairs sampled across the chunks of a request are recomputed by the oracle from
    the same source words: packed tile records and cache rows must match."""
    L, H, D = shape
    pos_of = {}
    pos = 0
    for c in order:
        pos_of.setdefault(c, pos)
        pos += T
    for c in sorted(set(order)):
        bits = B.BITS[precs[c]]
        tile_bytes = codec.chunk_bytes(1, 1, D, T, bits, g) // 2
        for _ in range(n_samples):
            l, h = int(rng.integers(L)), int(rng.integers(H))
            src_kv = srcs[c][l, :, h].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
            ref_pack, _ = codec.quantize_pack_chunk(src_kv.reshape(1, 2, 1, T, D), bits, g)
            for kv in range(2):
                tile = (l * 2 + kv) * H + h
                got = packs[c][tile * tile_bytes:(tile + 1) * tile_bytes].cpu().numpy()
                assert np.array_equal(got, ref_pack[kv * tile_bytes:(kv + 1) * tile_bytes])
            ref_out = np.zeros((1, 2, 1, T, D), np.uint16)
            codec.dequant_scatter_chunk(ref_pack, (1, 1, D), T, bits, g, ref_out, 0)
            p0 = pos_of[c]
            got_out = host_u16(out[l, :, h, p0:p0 + T])
            assert ulp_distance(got_out, ref_out[0, :, 0]).max() <= 1
            assert np.array_equal(got_out, ref_out[0, :, 0])


def test_llama3_8b_request_sampled_tiles_match_oracle():
    """One request of the headline workload (32 layers, 8 KV heads, head_dim 128, ten
    512-token chunks: 2 x 16-bit, 3 x int8, 5 x int4, group 128) built and loaded by
    the GPU in the launch configuration the benchmark times."""
    L, H, D, T, g = 32, 8, 128, 512, 128
    ctx = B.Context(L, H, D, T, group_int8=g, group_int4=g)
    precs = [B.PREC_16] * 2 + [B.PREC_INT8] * 3 + [B.PREC_INT4] * 5
    order = [4, 9, 0, 6, 2, 8, 1, 5, 3, 7]
    srcs, packs = [], []
    for i, p in enumerate(precs):
        s_ = wl.kv_chunk_device(L, H, D, T, 500 + i)
        dst = torch.empty(ctx.chunk_bytes(p, T), dtype=torch.uint8, device="cuda")
        ctx.quantize_chunk(s_, T, p, g, dst)
        srcs.append(s_)
        packs.append(dst)
    cap = 10 * T
    out = torch.empty((L, 2, H, cap, D), dtype=torch.int16, device="cuda")
    ctx.load_packed([(packs[c], T, precs[c], g) for c in order], out, cap)
    torch.cuda.synchronize()
    _check_sampled_tiles(ctx, (L, H, D), T, g, precs, order, srcs, packs, out, 3,
                         np.random.default_rng(0))
    # a property that holds at any size: 16-bit chunks are copied word for word
    for pos, c in enumerate(order):
        if precs[c] == B.PREC_16:
            assert torch.equal(out[:, :, :, pos * T:(pos + 1) * T], srcs[c].view(torch.int16))
    ctx.destroy()


def test_llama3_70b_request_sampled_tiles_match_oracle():
    """80 layers, 8 KV heads, head_dim 128, sixteen 1024-token chunks, int8 and int4
    alternating (group 128): 5 GiB of cache written by one launch."""
    L, H, D, T, g = 80, 8, 128, 1024, 128
    ctx = B.Context(L, H, D, T, group_int8=g, group_int4=g)
    n_distinct = 4                                     # sources are reused: 16 x 320 MiB is a lot
    precs = [B.PREC_INT8, B.PREC_INT4] * (n_distinct // 2)
    srcs, packs = [], []
    for i, p in enumerate(precs):
        s_ = wl.kv_chunk_device(L, H, D, T, 600 + i)
        dst = torch.empty(ctx.chunk_bytes(p, T), dtype=torch.uint8, device="cuda")
        ctx.quantize_chunk(s_, T, p, g, dst)
        srcs.append(s_)
        packs.append(dst)
    order = [i % n_distinct for i in range(16)]
    cap = 16 * T
    out = torch.empty((L, 2, H, cap, D), dtype=torch.int16, device="cuda")
    ctx.load_packed([(packs[c], T, precs[c], g) for c in order], out, cap)
    torch.cuda.synchronize()
    _check_sampled_tiles(ctx, (L, H, D), T, g, precs, order[:n_distinct], srcs, packs, out, 2,
                         np.random.default_rng(1))
    # every repeat of a chunk must equal its first occurrence, over the whole 5 GiB
    for pos in range(n_distinct, 16):
        first = order[pos]
        assert torch.equal(out[:, :, :, pos * T:(pos + 1) * T], out[:, :, :, first * T:(first + 1) * T])
    ctx.destroy()


@pytest.mark.parametrize("pinned_dma", [False, True])
def test_cold_stress_shape_through_the_pool(pinned_dma):
    """The cold-path stress shape: 8B KV, 1024-token int4 chunks with group 64, every chunk in
    pinned memory, two requests on two streams; read by the kernel straight from pinned memory
    (the default) or copied through a 3-slot staging ring (pinned_dma)."""
    L, H, D, T, g = 32, 8, 128, 1024, 64
    n = 6
    ctx = _pool_ctx(L, H, D, T, g, hbm_slots=0, pin_slots=n, stg_slots=3, tau_gpu_ppm=0,
                    precs=[B.PREC_INT4], pinned_dma=pinned_dma)
    srcs, packs = [], []
    for i in range(n):
        s_ = wl.kv_chunk_device(L, H, D, T, 700 + i)
        dst = torch.empty(ctx.chunk_bytes(B.PREC_INT4, T), dtype=torch.uint8, device="cuda")
        ctx.quantize_chunk(s_, T, B.PREC_INT4, g, dst)
        ctx.pool_insert(i, B.PREC_INT4, T, dst, B.TIER_PINNED, packed_is_device=True)
        srcs.append(s_)
        packs.append(dst)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    orders = [[2, 0, 1], [5, 3, 4]]
    outs = [torch.empty((L, 2, H, 3 * T, D), dtype=torch.int16, device="cuda") for _ in range(2)]
    for r in range(2):
        st, _ = ctx.load_chunks(orders[r], outs[r], 3 * T, stream=streams[r])
        assert st["n_pinned_hits"] == 3 and st["bytes_h2d"] == 3 * ctx.chunk_bytes(B.PREC_INT4, T)
        assert st["n_kernel_launches"] == (3 if pinned_dma else 1)
    torch.cuda.synchronize()
    for r in range(2):
        _check_sampled_tiles(ctx, (L, H, D), T, g, [B.PREC_INT4] * n, orders[r], srcs, packs,
                             outs[r], 2, np.random.default_rng(2 + r))
    ctx.destroy()


@pytest.mark.parametrize("pinned_dma", [False, True])
def test_cold_stress_at_its_full_request_shape(pinned_dma):
    """The cold-path stress configuration as stated: 4 concurrent requests on 4 streams, each
    32 chunks x 1024 tokens, int4 with group 64, 8B KV shape, all 128 chunks distinct and in pinned
    host memory (4.5 GiB), 4 GiB of cache per request.  Three chunks of every request are
    rebuilt from their seed and tiles sampled from them recomputed by the oracle; the first and
    the last rows of every chunk of every request are compared with a second, single-stream
    load of the same chunk."""
    L, H, D, T, g = 32, 8, 128, 1024, 64
    n_req, per_req = 4, 32
    n = n_req * per_req
    ctx = _pool_ctx(L, H, D, T, g, hbm_slots=0, pin_slots=n, stg_slots=4, tau_gpu_ppm=0,
                    precs=[B.PREC_INT4], pinned_dma=pinned_dma)
    nbytes = ctx.chunk_bytes(B.PREC_INT4, T)
    dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    for i in range(n):
        ctx.quantize_chunk(wl.kv_chunk_device(L, H, D, T, 4000 + i), T, B.PREC_INT4, g, dst)
        ctx.pool_insert(i, B.PREC_INT4, T, dst, B.TIER_PINNED, packed_is_device=True)
        torch.cuda.synchronize()
    rng = np.random.default_rng(11)
    perm = rng.permutation(n)
    orders = [[int(c) for c in perm[r * per_req:(r + 1) * per_req]] for r in range(n_req)]
    streams = [torch.cuda.Stream() for _ in range(n_req)]
    outs = [torch.empty((L, 2, H, per_req * T, D), dtype=torch.int16, device="cuda") for _ in range(n_req)]
    print("four loads on four streams", flush=True)
    for r in range(n_req):
        st, _ = ctx.load_chunks(orders[r], outs[r], per_req * T, stream=streams[r])
        assert st["n_pinned_hits"] == per_req and st["bytes_h2d"] == per_req * nbytes
        assert st["tokens"] == per_req * T
    torch.cuda.synchronize()
    one = torch.empty((L, 2, H, T, D), dtype=torch.int16, device="cuda")
    for r in range(n_req):
        print("checking request", r, flush=True)
        for pos in sorted(rng.choice(per_req, 3, replace=False)):
            c = orders[r][pos]
            src = wl.kv_chunk_device(L, H, D, T, 4000 + c)
            ptr, nb = ctx.pool_slot(c, B.TIER_PINNED)
            pk = torch.empty(nb, dtype=torch.uint8, device="cuda")
            ctx.quantize_chunk(src, T, B.PREC_INT4, g, pk)      # the same bytes the pool holds
            torch.cuda.synchronize()
            held = np.frombuffer(ctypes.string_at(ptr, nb), np.uint8)
            assert np.array_equal(held, pk.cpu().numpy()), (r, pos, c)
            view = outs[r][:, :, :, pos * T:(pos + 1) * T]
            _check_sampled_tiles(ctx, (L, H, D), T, g, {c: B.PREC_INT4}, [c], {c: src}, {c: pk},
                                 view, 2, rng)
        # every chunk: its first and last token rows against a plain single-stream load
        for pos, c in enumerate(orders[r]):
            ctx.load_chunks([c], one, T)
            torch.cuda.synchronize()
            for row in (0, T - 1):
                assert torch.equal(outs[r][:, :, :, pos * T + row], one[:, :, :, row]), (r, pos, c)
    ctx.destroy()


@pytest.mark.parametrize("pinned_dma", [False, True])
def test_mixed_tier_batch_at_the_8b_shape_sampled_tiles_match_oracle(pinned_dma):
    """The Zipf batch workload in small: 4 requests x 8 chunks of the 8B shape in one
    ha_rag_load_batch call, chunks split between the HBM pool and pinned memory, tags by
    rank class, promotion on; tiles sampled from every request are recomputed by the oracle."""
    L, H, D, T, g = 32, 8, 128, 512, 128
    n = 16
    precs = [B.PREC_16] * 3 + [B.PREC_INT8] * 5 + [B.PREC_INT4] * 8
    ctx = B.Context(L, H, D, T, group_int8=g, group_int4=g, tau_gpu_ppm=500_000, pinned_dma=pinned_dma)
    keep = []
    for p in (B.PREC_16, B.PREC_INT8, B.PREC_INT4):
        slot = (ctx.chunk_bytes(p, T) + 255) // 256 * 256
        ctx.register_slab(B.TIER_HBM, p, torch.empty(slot * 4, dtype=torch.uint8, device="cuda"))
        ctx.register_slab(B.TIER_PINNED, p, torch.empty(slot * precs.count(p), dtype=torch.uint8,
                                                        pin_memory=True))
    ctx.register_staging(torch.empty(((ctx.chunk_bytes(B.PREC_16, T) + 255) // 256 * 256) * 3,
                                     dtype=torch.uint8, device="cuda"))
    srcs, packs = [], []
    for i, p in enumerate(precs):
        s_ = wl.kv_chunk_device(L, H, D, T, 800 + i)
        dst = torch.empty(ctx.chunk_bytes(p, T), dtype=torch.uint8, device="cuda")
        ctx.quantize_chunk(s_, T, p, g, dst)
        ctx.pool_insert(i, p, T, dst, B.TIER_PINNED, packed_is_device=True)
        if i % 4 == 0:
            ctx.pool_insert(i, p, T, dst, B.TIER_HBM, packed_is_device=True)
        srcs.append(s_)
        packs.append(dst)
    torch.cuda.synchronize()
    ctx.set_counts(list(range(n)), [100 - i for i in range(n)])
    ctx.rerank()
    rng = np.random.default_rng(7)
    reqs = [rng.permutation(n)[:8].tolist() for _ in range(4)]
    outs = [torch.empty((L, 2, H, 8 * T, D), dtype=torch.int16, device="cuda") for _ in reqs]
    st, tr = ctx.load_batch(reqs, outs, [8 * T] * 4, want_trace=True)
    torch.cuda.synchronize()
    assert st["n_chunks"] == 32 and st["n_hbm_hits"] + st["n_pinned_hits"] == 32
    assert st["n_promoted"] >= 1 and st["n_hbm_hits"] >= 4
    for r, o in zip(reqs, outs):
        _check_sampled_tiles(ctx, (L, H, D), T, g, precs, r, srcs, packs, o, 1, rng)
    ctx.destroy()


def test_load_packed_can_be_captured_in_a_hip_graph_and_replayed():
    """ha_rag_load_packed only launches kernels (descriptors travel in the kernel arguments),
    so a serving loop may capture it once per request shape.  Replays see the packed bytes
    that are in the buffers at replay time; eager work runs between the replays."""
    L, H, D, g = 2, 2, 64, 64
    tokens = [40, 128, 7]
    precs = [B.PREC_INT4, B.PREC_INT8, B.PREC_16]
    ctx = B.Context(L, H, D, 128, group_int8=g, group_int4=g)
    cap = sum(tokens) + 3
    bufs = [torch.zeros(ctx.chunk_bytes(p, t) + 16, dtype=torch.uint8, device="cuda")
            for p, t in zip(precs, tokens)]
    out = torch.full((L, 2, H, cap, D), CANARY, dtype=torch.int16, device="cuda")
    chunks = [(bufs[i], tokens[i], precs[i], g) for i in (2, 0, 1)]
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        ctx.load_packed(chunks, out, cap, 2, stream=side)          # warm-up outside the capture
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            ctx.load_packed(chunks, out, cap, 2, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    for rnd in range(3):
        packed = [codec.quantize_pack_chunk(wl.kv_chunk(L, H, D, t, 900 + 10 * rnd + i), B.BITS[p], g)[0]
                  for i, (p, t) in enumerate(zip(precs, tokens))]
        for b, pk in zip(bufs, packed):
            b[:pk.size].copy_(torch.from_numpy(pk))
        ref = np.full((L, 2, H, cap, D), CANARY, np.uint16)
        codec.load_chunks(packed, (L, H, D), tokens, [B.BITS[p] for p in precs], [g] * 3, [2, 0, 1],
                          cap_tokens=cap, tok_base=2, out=ref)
        out.fill_(CANARY)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(host_u16(out), ref), rnd
    ctx.destroy()


def test_knowledge_base_files_survive_the_context(tmp_path):
    """Pool files plus the saved index are the knowledge base: a second context that registers
    the same files and loads the index serves the same bytes (whole chunks and key / value
    units, buffered and O_DIRECT files)."""
    L, H, D, T, g = 2, 2, 64, 64, 32
    for o_direct in (False, True):
        def make():
            ctx = B.Context(L, H, D, T, group_int8=g, group_int4=g, tau_gpu_ppm=300_000,
                            disk_o_direct=o_direct)
            big = 0
            for p in (B.PREC_INT4, B.PREC_GSE8):
                slot = (ctx.chunk_bytes(p, T) + 4095) // 4096 * 4096
                big = max(big, slot)
                ctx.register_slab(B.TIER_HBM, p, torch.zeros(slot * 2, dtype=torch.uint8, device="cuda"))
                ctx.register_disk(p, str(tmp_path / f"kb_{int(o_direct)}_{p}.bin"), slot * 8)
            ctx.register_staging(torch.zeros(big * 2, dtype=torch.uint8, device="cuda"))
            ctx.register_bounce(torch.zeros(big * 2, dtype=torch.uint8).pin_memory())
            return ctx
        try:
            a = make()
        except B.HaRagError as e:
            if o_direct and e.code == B.EIO:
                pytest.skip("this filesystem refuses O_DIRECT")
            raise
        spec = [(B.PART_KV, B.PREC_INT4, 64), (B.PART_K, B.PREC_GSE8, 40), (B.PART_V, B.PREC_INT4, 40),
                (B.PART_KV, B.PREC_GSE8, 17), (B.PART_KV, B.PREC_INT4, 33)]
        packed = []
        for i, (part, prec, t) in enumerate(spec):
            doc = wl.kv_chunk(L, H, D, t, 2100 + i)
            if part == B.PART_KV:
                pk = codec.quantize_pack_chunk(doc, ORC[prec], g)[0]
                a.pool_insert(50 + i, prec, t, pk, B.TIER_DISK)
            else:
                pk = codec.quantize_pack_half(np.ascontiguousarray(doc[:, part - 1]), ORC[prec], g)[0]
                a.pool_insert_half(50 + i, part, prec, t, pk, B.TIER_DISK)
            packed.append(pk)
        a.set_counts([50, 51, 52, 53, 54], [5, 4, 3, 2, 1])
        idx = str(tmp_path / f"kb_{int(o_direct)}.idx")
        a.pool_save_index(idx)
        a.destroy()

        b = make()
        assert b.pool_load_index(idx) == 5
        b.rerank()
        req = [4, 1, 2, 0, 3]
        tokens = [s_[2] for s_ in spec]
        cap = 33 + 40 + 64 + 17
        ref = np.full((L, 2, H, cap, D), CANARY, np.uint16)
        codec.load_chunks(packed, (L, H, D), tokens, [ORC[s_[1]] for s_ in spec], [g] * 5, req,
                          cap_tokens=cap, out=ref, parts=[s_[0] for s_ in spec])
        for rnd in range(2):          # first from the files, then partly from the HBM copies made
            out = torch.full((L, 2, H, cap, D), CANARY, dtype=torch.int16, device="cuda")
            st, tr = b.load_chunks([50 + c for c in req], out, cap, want_trace=True)
            torch.cuda.synchronize()
            assert np.array_equal(host_u16(out), ref), (o_direct, rnd)
            if rnd == 0:
                assert st["n_disk_hits"] == 5
        b.destroy()


@pytest.mark.parametrize("D", [8, 24, 40])
def test_smallest_head_dims_without_groups(D):
    """head_dim only has to be a multiple of 8 for the tags that carry no per-group meta
    (16-bit, FP8, GSE-8); a context for such a shape names no integer group (0), and the
    integer tags are refused there."""
    L, H, g = 2, 3, 32
    tokens = [1, 300, 7]
    precs = [B.PREC_16, B.PREC_FP8_E4M3, B.PREC_GSE8]
    with pytest.raises(B.HaRagError) as e:
        B.Context(L, H, D, max(tokens), group_int8=32, group_int4=32)
    assert e.value.code == B.EFORMAT
    ctx = B.Context(L, H, D, max(tokens), group_int8=0, group_int4=0)
    with pytest.raises(B.HaRagError) as e:
        ctx.chunk_bytes(B.PREC_INT4, 7)
    assert e.value.code == B.EFORMAT
    srcs = [wl.kv_chunk(L, H, D, t, 3100 + i) for i, t in enumerate(tokens)]
    packed_ref = [codec.quantize_pack_chunk(s_, ORC[p], g)[0] for s_, p in zip(srcs, precs)]
    dev = []
    for s_, p, ref in zip(srcs, precs, packed_ref):
        got, _ = gpu_quantize(ctx, s_, p, g)
        assert np.array_equal(got, ref)
        dev.append(dev_u8(got))
    order = [1, 0, 2, 1]
    cap = sum(tokens[c] for c in order) + 2
    ref = np.full((L, 2, H, cap, D), CANARY, np.uint16)
    codec.load_chunks(packed_ref, (L, H, D), tokens, [ORC[p] for p in precs], [g] * 3, order,
                      cap_tokens=cap, tok_base=1, out=ref)
    out = torch.full((L, 2, H, cap, D), CANARY, dtype=torch.int16, device="cuda")
    ctx.load_packed([(dev[c], tokens[c], precs[c], g) for c in order], out, cap, 1)
    torch.cuda.synchronize()
    assert np.array_equal(host_u16(out), ref)
    ctx.destroy()


def test_a_removed_chunk_is_gone_and_its_id_and_slots_serve_new_content():
    L, H, D, T, g = 2, 2, 64, 128, 64
    n = 4
    ctx = _pool_ctx(L, H, D, T, g, hbm_slots=2, pin_slots=n, stg_slots=2, tau_gpu_ppm=500_000,
                    precs=[B.PREC_INT4])                 # GPU_LIST holds two of the four chunks
    tokens = [T, T - 3, T - 17, 40]
    srcs = [wl.kv_chunk(L, H, D, tokens[i], 900 + i) for i in range(n)]
    packed = [codec.quantize_pack_chunk(s, 4, g)[0] for s in srcs]
    for i in range(n):
        ctx.pool_insert(i, B.PREC_INT4, tokens[i], packed[i], B.TIER_PINNED)
    ctx.set_counts(list(range(n)), [10, 9, 8, 7])
    ctx.rerank()

    def run(req):
        cap = sum(tokens[c] for c in req) + 2
        out = torch.full((L, 2, H, cap, D), CANARY, dtype=torch.int16, device="cuda")
        st, tr = ctx.load_chunks(req, out, cap, want_trace=True)
        torch.cuda.synchronize()
        ref = np.full((L, 2, H, cap, D), CANARY, np.uint16)
        codec.load_chunks(packed, (L, H, D), tokens, [4] * n, [g] * n, req, cap_tokens=cap, out=ref)
        assert np.array_equal(host_u16(out), ref), req
        return st, tr

    st, tr = run([0, 1])                                  # both promoted: the HBM slab is full
    assert [t.promoted for t in tr] == [1, 1]
    ctx.pool_remove(0)
    with pytest.raises(B.HaRagError) as e:
        ctx.load_chunks([0], torch.zeros(1, device="cuda"), 1)
    assert e.value.code == B.ENOENT
    # the same id comes back with other content and length, into the freed pinned slot; the
    # freed HBM slot takes its promotion without evicting chunk 1
    tokens[0] = 77
    srcs[0] = wl.kv_chunk(L, H, D, 77, 990)
    packed[0] = codec.quantize_pack_chunk(srcs[0], 4, g)[0]
    ctx.pool_insert(0, B.PREC_INT4, 77, packed[0], B.TIER_PINNED)
    ctx.set_counts([0], [100])
    ctx.rerank()
    st, tr = run([1, 0, 2])
    assert [t.found_tier for t in tr] == [B.TIER_HBM, B.TIER_PINNED, B.TIER_PINNED]
    assert tr[1].promoted == 1 and tr[1].evicted_id == B.NO_CHUNK
    st, tr = run([0, 1])
    assert st["n_hbm_hits"] == 2
    ctx.destroy()
