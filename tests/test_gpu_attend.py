"""Attention straight over packed chunks (HIP, through the C ABI) against the CPU oracle:
binary64 softmax attention over the BF16 cache the load oracle builds from the same packed
bytes.

Tolerance (derived from the kernel's arithmetic; K and V values are exact on both sides):
  * the softmax weights are rounded to BF16 (8 significant bits: relative 2^-8 each at worst)
    before they multiply V while the normaliser keeps them in binary32: |out error| <=
    2^-8 * spread, spread = sum_t softmax(s)[t] |V[t][d]| (the oracle returns it);
  * scores are sums of 128 exact products accumulated in binary32: |s error| <= 2^-17 * sabs,
    sabs = sm_scale * sum_d |q[d] K[t][d]| (max over t); it shifts lse by as much and the
    weights by that relative amount.  The bar adds 2^-15 * (1 + sabs) (times spread for out),
    which also covers the hardware exp2 / log2 (about 1 ulp of binary32).
"""
import numpy as np
import pytest
import torch

from oracle import attend as A
from oracle import codec
from paper_2510_20878_amd import binding as B
from paper_2510_20878_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the GPU"
    B.lib()
    yield
    torch.cuda.synchronize()


def dev_u8(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint8)).cuda()


def q_words(n_q, n_qh, D, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    return wl.f32_to_bf16_words(rng.standard_normal((n_q, n_qh, D), dtype=np.float32))


def check(out, lse, ref_out, ref_lse, spread, sabs):
    """sabs: [n_q][n_qh] bound on sum |q k| * scale."""
    slack = 2.0 ** -15 * (1.0 + sabs)
    err = np.abs(out.astype(np.float64) - ref_out)
    bar = 2.0 ** -8 * spread + slack[..., None] * spread + 1e-30
    assert np.all(err <= bar), (float((err / bar).max()), float(err.max()))
    lerr = np.abs(lse.astype(np.float64) - ref_lse)
    assert np.all(lerr <= slack), (float((lerr / slack).max()), float(lerr.max()))
    return float((err / bar).max()), float((lerr / slack).max())


def score_bound(cache, layer, n_kv, qw, scale, H):
    q = np.abs(A.bf16_words_to_f64(qw))
    n_q, n_qh, D = q.shape
    G = n_qh // H
    out = np.zeros((n_q, n_qh))
    for hq in range(n_qh):
        K = np.abs(A.bf16_words_to_f64(cache[layer, 0, hq // G, :n_kv]))
        out[:, hq] = scale * (q[:, hq] @ K.T).max(axis=1)
    return out


def run_case(shape, reqs, layer, n_qh, scale, seed, g8=128, g4=128, max_tokens=None, want_lse=True):
    """reqs: list of (tokens list, precs list, n_q).  Chunk i of a request is drawn from seed.
    want_lse=False: the requests ask for no log-sum-exp (a null pointer); only out is checked."""
    L, H, D = shape
    T_max = max_tokens or max([t for r in reqs for t in r[0]] + [16])
    ctx = B.Context(L, H, D, T_max, group_int8=g8, group_int4=g4)
    grp = {B.PREC_INT8: g8, B.PREC_INT4: g4}
    ORC = {B.PREC_16: 16, B.PREC_INT8: 8, B.PREC_INT4: 4, B.PREC_FP8_E4M3: 43, B.PREC_FP8_E5M2: 52,
           B.PREC_GSE8: 143}
    keep, call, refs = [], [], []
    k = 0
    for ri, (tokens, precs, n_q) in enumerate(reqs):
        packs = []
        for t, p in zip(tokens, precs):
            src = wl.kv_chunk(L, H, D, t, seed + k) if t else np.zeros((L, 2, H, 0, D), np.uint16)
            k += 1
            packs.append(codec.quantize_pack_chunk(src, ORC[p], grp.get(p, 128))[0] if t
                         else np.zeros(0, np.uint8))
        qw = q_words(n_q, n_qh, D, seed + 1000 + ri)
        q_d = torch.from_numpy(qw.view(np.int16)).cuda()
        out_d = torch.full((n_q, n_qh, D), float("nan"), dtype=torch.float32, device="cuda")
        lse_d = torch.full((n_q, n_qh), float("nan"), dtype=torch.float32, device="cuda")
        packs_d = [dev_u8(p) if len(p) else None for p in packs]
        keep += [q_d, out_d, lse_d, packs_d]
        call.append(([(pd, t, p, grp.get(p, 0)) for pd, t, p in zip(packs_d, tokens, precs)],
                     q_d, out_d, lse_d if want_lse else None, n_q))
        refs.append((packs, tokens, precs, qw, out_d, lse_d))
    nbytes = ctx.attend_workspace_bytes(call, n_qh)
    ws = torch.full((max(nbytes, 16) // 4,), float("nan"), dtype=torch.float32, device="cuda")
    ctx.attend_packed(call, layer, n_qh, scale, ws, nbytes)
    torch.cuda.synchronize()
    worst = (0.0, 0.0)
    for packs, tokens, precs, qw, out_d, lse_d in refs:
        n_kv = sum(tokens)
        out, lse = out_d.cpu().numpy(), lse_d.cpu().numpy()
        if n_kv == 0:
            assert np.all(out == 0) and (np.all(np.isneginf(lse)) if want_lse else np.all(np.isnan(lse)))
            continue
        live = [i for i, t in enumerate(tokens) if t]
        cache, _ = codec.load_chunks(packs, shape, tokens, [ORC[p] for p in precs],
                                     [grp.get(p, 128) for p in precs], live)
        ref_out, ref_lse, spread = A.attend(cache, layer, n_kv, qw, scale)
        if not want_lse:
            assert np.all(np.isnan(lse))  # untouched
            lse = ref_lse
        w = check(out, lse, ref_out, ref_lse, spread, score_bound(cache, layer, n_kv, qw, scale, H))
        worst = (max(worst[0], w[0]), max(worst[1], w[1]))
    ctx.destroy()
    return worst


ALL = [B.PREC_16, B.PREC_INT8, B.PREC_INT4, B.PREC_FP8_E4M3, B.PREC_FP8_E5M2, B.PREC_GSE8]


def test_all_six_tags_ragged_chunks_one_request():
    tokens = [40, 16, 77, 1, 33, 128]
    print("worst error / bar:", run_case((2, 2, 128), [(tokens, ALL, 3)], 1, 8, 128 ** -0.5, 10))


@pytest.mark.parametrize("prec", ALL)
@pytest.mark.parametrize("n_q,n_qh", [(1, 2), (1, 8), (5, 8), (16, 8), (21, 8), (3, 32)])
def test_each_tag_and_query_tile_count(prec, n_q, n_qh):
    run_case((2, 2, 128), [([50, 96], [prec, prec], n_q)], 0, n_qh, 0.1, 20 + n_q)


@pytest.mark.parametrize("g", [32, 64])
def test_smaller_groups(g):
    run_case((1, 2, 128), [([70, 30], [B.PREC_INT4, B.PREC_INT8], 2)], 0, 4, 0.09, 30, g8=g, g4=g)


def test_a_chunk_cut_into_pieces_and_a_sharp_softmax():
    # few workgroups, so the shortest pieces: 1100 tokens = 69 blocks = 17 pieces of 4 blocks and one of 1,
    # 513 tokens = 33 blocks = 8 pieces of 4 and one of 1, a record each; a large scale makes few keys
    # dominate, so the running maximum keeps moving and accumulated sums are rescaled many times
    run_case((1, 1, 128), [([1100, 513], [B.PREC_INT4, B.PREC_INT8], 4)], 0, 4, 0.5, 40)


def test_many_long_chunks_take_long_pieces():
    # 120 chunks x 8 heads: pieces of at most 64 blocks (82 blocks in 2, 44 in 1) give 1440 workgroups,
    # of at most 32 blocks (3 of 28, 28, 26 and 2 of 22) 2400, which is enough: no shorter ones
    reqs = [([1300, 700], [B.PREC_INT4, B.PREC_INT8], 2) for _ in range(60)]
    run_case((1, 8, 128), reqs, 0, 16, 0.09, 45)


@pytest.mark.parametrize("n_docs", [1, 3, 8, 9, 63, 64, 65, 150, 300])
def test_merge_of_one_request_with_few_and_with_many_records(n_docs):
    """The merge kernel shares a row's records between groups of threads (launch_k7): one record,
    fewer than the smallest launch's groups, one or two per group, and more than the largest
    launch's groups fetch in one round (128), with a ragged last round."""
    tokens = [5 + (11 * i) % 28 for i in range(n_docs)]
    precs = [ALL[(i * 5 + 1) % 6] for i in range(n_docs)]
    run_case((1, 2, 128), [(tokens, precs, 3)], 0, 4, 0.11, 70 + n_docs)


def test_batch_of_requests_with_different_shapes_empty_chunks_and_an_empty_request():
    reqs = [([30, 0, 65], [B.PREC_INT4, B.PREC_16, B.PREC_INT8], 1),
            ([], [], 2),
            ([16], [B.PREC_GSE8], 17),
            ([0], [B.PREC_INT4], 1),
            ([600, 20, 48, 48], [B.PREC_FP8_E4M3, B.PREC_INT4, B.PREC_INT4, B.PREC_FP8_E5M2], 6)]
    run_case((2, 2, 128), reqs, 1, 4, 0.088, 50)


def test_more_chunks_and_requests_than_one_launch_holds():
    reqs = [([16 + (3 * i + j) % 20 for j in range(8)], [ALL[(i + j) % 6] for j in range(8)], 1 + i % 3)
            for i in range(140)]                     # 1120 chunks, 140 requests: three launches of runs, three of merges
    run_case((1, 1, 128), reqs, 0, 2, 0.1, 60)


def test_runs_of_documents_per_workgroup_across_launches_of_the_many_rows_kernel():
    """Requests with more than two query tiles go to the kernel whose waves share each decoded
    block.  A workgroup takes a run of the request's blocks in list order, across documents
    (here 2 x 270 short documents of 1 to 3 blocks x 8 heads x 2 tile groups: runs of several
    documents, cut where the blocks run out, not at document ends), and writes one record per
    run; 540 documents also need two launches, and no run straddles them.  Formats change inside
    a run and documents end ragged."""
    n_docs = 270
    reqs = [([3 + (7 * i + 5 * r) % 41 for i in range(n_docs)], [ALL[(i * 5 + r) % 6] for i in range(n_docs)],
             40 - 7 * r) for r in range(2)]
    run_case((1, 8, 128), reqs, 0, 32, 0.1, 90)


@pytest.mark.parametrize("n_q,n_qh,H", [(12, 4, 1), (40, 4, 1), (9, 32, 2)])
def test_many_rows_kernel_with_runs_inside_long_documents(n_q, n_qh, H):
    """Few, long documents and many query rows: the call has few workgroups, so the runs are
    the shortest there are (8 blocks = 128 tokens) and most of them start and end inside a
    document; every run writes its own record for the tile-wise merge; 3, 10 and 9 query tiles
    take workgroups of 2, 8 and 8 waves.  The second document's last block is ragged and the
    last run of each request short."""
    reqs = [([2500, 700], [B.PREC_INT4, B.PREC_INT8], n_q), ([1333], [B.PREC_16], n_q)]
    run_case((1, H, 128), reqs, 0, n_qh, 0.07, 110 + n_q)


@pytest.mark.parametrize("tokens", [[1], [16], [48], [33, 16, 1, 80], [15, 17, 31, 47, 49]])
def test_many_rows_kernel_with_blocks_that_have_no_partner(tokens):
    """The many-rows kernel scores two blocks per step.  Documents of one block, of an odd number
    of whole blocks, and ragged ones whose last block opens a pair: the missing half of a pair
    must not count (its keys are whatever the buffer held, its values are written as zeros), in
    the first round of a workgroup (nothing decoded yet) and in later ones."""
    precs = [ALL[(3 * i + len(tokens)) % 6] for i in range(len(tokens))]
    run_case((1, 2, 128), [(tokens, precs, 40), (tokens[::-1], precs[::-1], 9)], 0, 8, 0.1, 130 + len(tokens))


def test_requests_that_ask_for_no_log_sum_exp():
    """lse may be null: in the merge kernels (a decode request, a many-rows request of several
    runs) and in the many-rows workgroups that write their request's output themselves (one run),
    next to an empty request."""
    reqs = [([50, 33], [B.PREC_INT4, B.PREC_16], 1),
            ([700, 260], [B.PREC_INT8, B.PREC_GSE8], 24),
            ([40], [B.PREC_FP8_E4M3], 30),
            ([], [], 2)]
    run_case((1, 2, 128), reqs, 0, 4, 0.09, 140, want_lse=False)


def test_one_call_with_requests_for_both_attention_kernels():
    """One query token next to 24 and 70 of them: the first request takes the kernel of at most
    two query tiles, the others the many-rows kernel (3 and 9 tiles, so one workgroup of four
    waves has idle waves for the former); one merge launch serves all of them."""
    reqs = [([50, 33], [B.PREC_INT4, B.PREC_16], 1),
            ([70, 16, 129], [B.PREC_INT8, B.PREC_GSE8, B.PREC_INT4], 24),
            ([300, 45], [B.PREC_FP8_E4M3, B.PREC_16], 70),
            ([20], [B.PREC_FP8_E5M2], 2)]
    run_case((2, 2, 128), reqs, 1, 4, 0.09, 95)


def test_llama3_8b_request_sampled_heads_match_oracle():
    """One request of the headline workload (32 layers, 8 KV heads, head_dim 128, ten
    512-token chunks: 2 x 16-bit, 3 x int8, 5 x int4, group 128; 32 query heads, one and
    sixteen query tokens) in the launch configuration the benchmark times; (layer, KV head)
    pairs are sampled and recomputed by the oracle from the same source words."""
    L, H, D, T, g, n_qh = 32, 8, 128, 512, 128, 32
    G = n_qh // H
    ctx = B.Context(L, H, D, T, group_int8=g, group_int4=g)
    precs = [B.PREC_16] * 2 + [B.PREC_INT8] * 3 + [B.PREC_INT4] * 5
    order = [4, 9, 0, 6, 2, 8, 1, 5, 3, 7]
    srcs, packs = [], []
    for i, p in enumerate(precs):
        s_ = wl.kv_chunk_device(L, H, D, T, 700 + i)
        dst = torch.empty(ctx.chunk_bytes(p, T), dtype=torch.uint8, device="cuda")
        ctx.quantize_chunk(s_, T, p, g, dst)
        srcs.append(s_)
        packs.append(dst)
    rng = np.random.default_rng(1)
    scale = D ** -0.5
    for n_q in (1, 16):
        qw = q_words(n_q, n_qh, D, 800 + n_q)
        q_d = torch.from_numpy(qw.view(np.int16)).cuda()
        out_d = torch.full((n_q, n_qh, D), float("nan"), dtype=torch.float32, device="cuda")
        lse_d = torch.full((n_q, n_qh), float("nan"), dtype=torch.float32, device="cuda")
        call = [([(packs[c], T, precs[c], g) for c in order], q_d, out_d, lse_d, n_q)]
        nbytes = ctx.attend_workspace_bytes(call, n_qh)
        ws = torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device="cuda")
        for layer, h in [(0, 0), (31, 7)] + [(int(rng.integers(L)), int(rng.integers(H))) for _ in range(2)]:
            ctx.attend_packed(call, layer, n_qh, scale, ws, nbytes)
            torch.cuda.synchronize()
            cache = np.zeros((1, 2, 1, len(order) * T, D), np.uint16)
            for pos, c in enumerate(order):
                bits = B.BITS[precs[c]]
                src_kv = srcs[c][layer, :, h].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
                ref_pack, _ = codec.quantize_pack_chunk(src_kv.reshape(1, 2, 1, T, D), bits, g)
                codec.dequant_scatter_chunk(ref_pack, (1, 1, D), T, bits, g, cache, pos * T)
            qh = np.ascontiguousarray(qw[:, h * G:(h + 1) * G])
            ref_out, ref_lse, spread = A.attend(cache, 0, len(order) * T, qh, scale)
            check(out_d[:, h * G:(h + 1) * G].cpu().numpy(), lse_d[:, h * G:(h + 1) * G].cpu().numpy(),
                  ref_out, ref_lse, spread, score_bound(cache, 0, len(order) * T, qh, scale, 1))
    ctx.destroy()


def _pool_case():
    """Six chunks in a pool: ids 0..2 have an HBM copy, 3..5 only a pinned one."""
    L, H, D, T, g = 2, 2, 128, 96, 64
    ORC = {B.PREC_16: 16, B.PREC_INT8: 8, B.PREC_INT4: 4, B.PREC_GSE8: 143}
    ctx = B.Context(L, H, D, T, group_int8=g, group_int4=g)
    precs = [B.PREC_INT4, B.PREC_INT8, B.PREC_16, B.PREC_INT4, B.PREC_GSE8, B.PREC_INT8]
    tokens = [96, 50, 33, 80, 96, 17]
    keep = []
    for p in sorted(set(precs)):
        slot = (ctx.chunk_bytes(p, T) + 255) // 256 * 256
        hb = torch.zeros(slot * 3, dtype=torch.uint8, device="cuda")
        pn = torch.zeros(slot * 3, dtype=torch.uint8).pin_memory()
        ctx.register_slab(B.TIER_HBM, p, hb)
        ctx.register_slab(B.TIER_PINNED, p, pn)
        keep += [hb, pn]
    packs = []
    for i, (p, t) in enumerate(zip(precs, tokens)):
        pk = codec.quantize_pack_chunk(wl.kv_chunk(L, H, D, t, 300 + i), ORC[p], g)[0]
        packs.append(pk)
        ctx.pool_insert(i, p, t, pk, B.TIER_HBM if i < 3 else B.TIER_PINNED)
    return ctx, (L, H, D), g, precs, tokens, packs, ORC, keep


def test_attend_over_pool_chunks_in_hbm_and_in_pinned_memory():
    ctx, shape, g, precs, tokens, packs, ORC, keep = _pool_case()
    L, H, D = shape
    n_qh, scale, layer = 8, 0.09, 1
    lists = [[4, 0, 3], [2, 5, 1, 0]]
    call, refs = [], []
    for r, ids in enumerate(lists):
        n_q = 1 + 2 * r
        qw = q_words(n_q, n_qh, D, 400 + r)
        q_d = torch.from_numpy(qw.view(np.int16)).cuda()
        out_d = torch.full((n_q, n_qh, D), float("nan"), dtype=torch.float32, device="cuda")
        lse_d = torch.full((n_q, n_qh), float("nan"), dtype=torch.float32, device="cuda")
        call.append((ids, q_d, out_d, lse_d, n_q))
        refs.append((ids, qw, out_d, lse_d))
    nb = ctx.attend_chunks_workspace_bytes(call, n_qh)
    ws = torch.full((nb // 4,), float("nan"), dtype=torch.float32, device="cuda")
    ctx.attend_chunks(call, layer, n_qh, scale, ws, nb, count=True)
    torch.cuda.synchronize()
    for ids, qw, out_d, lse_d in refs:
        cache, _ = codec.load_chunks(packs, shape, tokens, [ORC[p] for p in precs], [g] * len(precs), ids)
        n_kv = sum(tokens[i] for i in ids)
        ref_out, ref_lse, spread = A.attend(cache, layer, n_kv, qw, scale)
        check(out_d.cpu().numpy(), lse_d.cpu().numpy(), ref_out, ref_lse, spread,
              score_bound(cache, layer, n_kv, qw, scale, H))
    assert [ctx.pool_query(i).count for i in range(6)] == [2, 1, 1, 1, 1, 1]
    assert all(not ctx.pool_query(i).in_hbm for i in (3, 4, 5))       # nothing was promoted
    ctx.destroy()


@pytest.mark.parametrize("n_q", [2, 40])
def test_attend_can_be_captured_in_a_hip_graph_and_replayed(n_q):
    """The call only launches kernels, so a per-layer loop can be recorded once and replayed;
    every replay is checked against the eager result, with eager work in between.  2 query
    tokens take the kernel of at most two query tiles, 40 the many-rows kernel with eight
    waves (whose LDS allowance was set when the context was created, not inside the capture)."""
    ctx, shape, g, precs, tokens, packs, ORC, keep = _pool_case()
    L, H, D = shape
    n_qh, scale = 8, 0.09
    devs = [dev_u8(p) for p in packs]
    qw = q_words(n_q, n_qh, D, 500)
    q_d = torch.from_numpy(qw.view(np.int16)).cuda()
    outs = [torch.zeros((n_q, n_qh, D), dtype=torch.float32, device="cuda") for _ in range(L)]
    lses = [torch.zeros((n_q, n_qh), dtype=torch.float32, device="cuda") for _ in range(L)]
    per_layer = [[([(devs[i], tokens[i], precs[i], g) for i in (1, 3, 0, 4)], q_d, outs[l], lses[l], n_q)]
                 for l in range(L)]
    nb = ctx.attend_workspace_bytes(per_layer[0], n_qh)
    ws = torch.zeros(nb // 4, dtype=torch.float32, device="cuda")
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for l in range(L):
            ctx.attend_packed(per_layer[l], l, n_qh, scale, ws, nb, stream=stream)
    torch.cuda.synchronize()
    eager = [(o.clone(), s.clone()) for o, s in zip(outs, lses)]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        for l in range(L):
            ctx.attend_packed(per_layer[l], l, n_qh, scale, ws, nb, stream=torch.cuda.current_stream())
    for rep in range(3):
        for o, s in zip(outs, lses):
            o.fill_(float("nan"))
            s.fill_(float("nan"))
        ws.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for l in range(L):
            assert torch.equal(outs[l], eager[l][0]) and torch.equal(lses[l], eager[l][1]), (rep, l)
    ctx.destroy()


def test_llama3_8b_batch_of_32_requests_sampled_heads_match_oracle():
    """The batch the benchmark times: 32 requests x 10 chunks x 512 tokens of the 8B shape in
    one call (one partial-attention launch over 320 chunks), one query token each, then 64 each.  Sampled
    (request, layer, KV head) triples are recomputed by the oracle from the source words."""
    L, H, D, T, g, n_qh, R = 32, 8, 128, 512, 128, 32, 32
    G = n_qh // H
    ctx = B.Context(L, H, D, T, group_int8=g, group_int4=g)
    mix = [B.PREC_16] * 2 + [B.PREC_INT8] * 3 + [B.PREC_INT4] * 5
    rng = np.random.default_rng(3)
    srcs, packs, precs = [], [], []
    for r in range(R):
        order = rng.permutation(10)
        for k in range(10):
            p = mix[order[k]]
            s_ = wl.kv_chunk_device(L, H, D, T, 9000 + 10 * r + k)
            dst = torch.empty(ctx.chunk_bytes(p, T), dtype=torch.uint8, device="cuda")
            ctx.quantize_chunk(s_, T, p, g, dst)
            srcs.append(s_)
            packs.append(dst)
            precs.append(p)
    qw = q_words(R, n_qh, D, 901)                                   # one query token per request
    q_d = torch.from_numpy(qw.view(np.int16)).cuda()
    out_d = torch.full((R, n_qh, D), float("nan"), dtype=torch.float32, device="cuda")
    lse_d = torch.full((R, n_qh), float("nan"), dtype=torch.float32, device="cuda")
    call = [([(packs[10 * r + k], T, precs[10 * r + k], g) for k in range(10)],
             q_d[r:r + 1], out_d[r:r + 1], lse_d[r:r + 1], 1) for r in range(R)]
    lists = ctx.attend_lists(call)
    nbytes = ctx.attend_workspace_bytes(lists, n_qh)
    ws = torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device="cuda")
    scale = D ** -0.5
    for layer in (0, 17, 31):
        ctx.attend_packed(lists, layer, n_qh, scale, ws, nbytes)
        torch.cuda.synchronize()
        assert not torch.isnan(out_d).any() and not torch.isnan(lse_d).any()
        for r, h in [(0, 0), (R - 1, H - 1), (int(rng.integers(R)), int(rng.integers(H)))]:
            cache = np.zeros((1, 2, 1, 10 * T, D), np.uint16)
            for k in range(10):
                bits = B.BITS[precs[10 * r + k]]
                src_kv = srcs[10 * r + k][layer, :, h].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
                ref_pack, _ = codec.quantize_pack_chunk(src_kv.reshape(1, 2, 1, T, D), bits, g)
                codec.dequant_scatter_chunk(ref_pack, (1, 1, D), T, bits, g, cache, k * T)
            qh = np.ascontiguousarray(qw[r:r + 1, h * G:(h + 1) * G])
            ref_out, ref_lse, spread = A.attend(cache, 0, 10 * T, qh, scale)
            check(out_d[r:r + 1, h * G:(h + 1) * G].cpu().numpy(), lse_d[r:r + 1, h * G:(h + 1) * G].cpu().numpy(),
                  ref_out, ref_lse, spread, score_bound(cache, 0, 10 * T, qh, scale, 1))
    # the same batch with the 64 query tokens of a question per request (the benchmark's other
    # attention leg): 256 query rows per KV head, eight-wave workgroups, one run per request and head
    n_q = 64
    qw = q_words(R * n_q, n_qh, D, 902).reshape(R, n_q, n_qh, D)
    q_d = torch.from_numpy(qw.view(np.int16)).cuda()
    out_d = torch.full((R, n_q, n_qh, D), float("nan"), dtype=torch.float32, device="cuda")
    lse_d = torch.full((R, n_q, n_qh), float("nan"), dtype=torch.float32, device="cuda")
    call = [([(packs[10 * r + k], T, precs[10 * r + k], g) for k in range(10)], q_d[r], out_d[r], lse_d[r], n_q)
            for r in range(R)]
    lists = ctx.attend_lists(call)
    nbytes = ctx.attend_workspace_bytes(lists, n_qh)
    ws = torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device="cuda")
    layer = 23
    ctx.attend_packed(lists, layer, n_qh, scale, ws, nbytes)
    torch.cuda.synchronize()
    assert not torch.isnan(out_d).any() and not torch.isnan(lse_d).any()
    for r, h in [(0, H - 1), (int(rng.integers(R)), int(rng.integers(H)))]:
        cache = np.zeros((1, 2, 1, 10 * T, D), np.uint16)
        for k in range(10):
            bits = B.BITS[precs[10 * r + k]]
            src_kv = srcs[10 * r + k][layer, :, h].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
            ref_pack, _ = codec.quantize_pack_chunk(src_kv.reshape(1, 2, 1, T, D), bits, g)
            codec.dequant_scatter_chunk(ref_pack, (1, 1, D), T, bits, g, cache, k * T)
        qh = np.ascontiguousarray(qw[r, :, h * G:(h + 1) * G])
        ref_out, ref_lse, spread = A.attend(cache, 0, 10 * T, qh, scale)
        check(out_d[r, :, h * G:(h + 1) * G].cpu().numpy(), lse_d[r, :, h * G:(h + 1) * G].cpu().numpy(),
              ref_out, ref_lse, spread, score_bound(cache, 0, 10 * T, qh, scale, 1))
    ctx.destroy()


def test_documents_stored_as_key_and_value_units_with_their_own_formats():
    """The paper's 2n units (Alg. 1 counts key chunks and value chunks separately): the i-th
    keys-only and the i-th values-only chunk of a request are one document; formats differ."""
    L, H, D, g, n_qh, scale, layer = 2, 2, 128, 64, 8, 0.09, 1
    ORC = {B.PREC_16: 16, B.PREC_INT8: 8, B.PREC_INT4: 4, B.PREC_FP8_E4M3: 43, B.PREC_FP8_E5M2: 52,
           B.PREC_GSE8: 143}
    ctx = B.Context(L, H, D, 128, group_int8=g, group_int4=g)
    docs = {"A": (70, B.PREC_16, B.PREC_INT4), "C": (128, B.PREC_INT8, B.PREC_GSE8),
            "D": (17, B.PREC_FP8_E4M3, B.PREC_FP8_E5M2), "E": (96, B.PREC_INT4, B.PREC_16)}
    src = {k: wl.kv_chunk(L, H, D, t, 600 + i) for i, (k, (t, _, _)) in enumerate(docs.items())}
    src["B"] = wl.kv_chunk(L, H, D, 33, 650)
    # the request's list: (name, part); keys and values interleaved, a whole chunk between them
    order = [("A", 1), ("C", 1), ("A", 2), ("C", 2), ("B", 0), ("D", 2), ("D", 1), ("E", 1), ("E", 2)]
    packed, tokens, bits, parts, call_chunks = [], [], [], [], []
    for name, part in order:
        if part == 0:
            pk = codec.quantize_pack_chunk(src[name], 8, g)[0]
            t, prec = 33, B.PREC_INT8
        else:
            t, kp, vp = docs[name]
            prec = kp if part == 1 else vp
            pk = codec.quantize_pack_half(np.ascontiguousarray(src[name][:, part - 1]), ORC[prec], g)[0]
        packed.append(pk)
        tokens.append(t)
        bits.append(ORC[prec])
        parts.append(part)
        call_chunks.append((dev_u8(pk), t, prec, g if prec in (B.PREC_INT8, B.PREC_INT4) else 0, part))
    n_kv = 70 + 128 + 33 + 17 + 96
    for n_q in (1, 7, 20):                                    # 20: the many-rows kernel
        qw = q_words(n_q, n_qh, D, 660 + n_q)
        q_d = torch.from_numpy(qw.view(np.int16)).cuda()
        out_d = torch.full((n_q, n_qh, D), float("nan"), dtype=torch.float32, device="cuda")
        lse_d = torch.full((n_q, n_qh), float("nan"), dtype=torch.float32, device="cuda")
        call = [(call_chunks, q_d, out_d, lse_d, n_q)]
        nb = ctx.attend_workspace_bytes(call, n_qh)
        ws = torch.full((nb // 4,), float("nan"), dtype=torch.float32, device="cuda")
        ctx.attend_packed(call, layer, n_qh, scale, ws, nb)
        torch.cuda.synchronize()
        cache, _ = codec.load_chunks(packed, (L, H, D), tokens, bits, [g] * len(order), list(range(len(order))),
                                     parts=parts)
        ref_out, ref_lse, spread = A.attend(cache, layer, n_kv, qw, scale)
        check(out_d.cpu().numpy(), lse_d.cpu().numpy(), ref_out, ref_lse, spread,
              score_bound(cache, layer, n_kv, qw, scale, H))
    ctx.destroy()


@pytest.mark.parametrize("kp,vp", [(a, b) for a in range(6) for b in range(6) if a != b])
def test_every_pair_of_key_and_value_formats(kp, vp):
    L, H, D, g, T = 1, 1, 128, 128, 40
    ORC = [16, 8, 4, 43, 52, 143]
    ctx = B.Context(L, H, D, T, group_int8=g, group_int4=g)
    src = wl.kv_chunk(L, H, D, T, 700 + 6 * kp + vp)
    pk = codec.quantize_pack_half(np.ascontiguousarray(src[:, 0]), ORC[kp], g)[0]
    pv = codec.quantize_pack_half(np.ascontiguousarray(src[:, 1]), ORC[vp], g)[0]
    n_q = 2 if (kp + vp) % 2 else 40                            # 40 query tokens: the many-rows kernel
    qw = q_words(n_q, 2, D, 770)
    q_d = torch.from_numpy(qw.view(np.int16)).cuda()
    out_d = torch.full((n_q, 2, D), float("nan"), dtype=torch.float32, device="cuda")
    lse_d = torch.full((n_q, 2), float("nan"), dtype=torch.float32, device="cuda")
    grp = lambda p: g if p in (B.PREC_INT8, B.PREC_INT4) else 0
    call = [([(dev_u8(pk), T, kp, grp(kp), B.PART_K), (dev_u8(pv), T, vp, grp(vp), B.PART_V)], q_d, out_d, lse_d, n_q)]
    nb = ctx.attend_workspace_bytes(call, 2)
    ws = torch.full((nb // 4,), float("nan"), dtype=torch.float32, device="cuda")
    ctx.attend_packed(call, 0, 2, 0.1, ws, nb)
    torch.cuda.synchronize()
    cache, _ = codec.load_chunks([pk, pv], (L, H, D), [T, T], [ORC[kp], ORC[vp]], [g, g], [0, 1], parts=[1, 2])
    ref_out, ref_lse, spread = A.attend(cache, 0, T, qw, 0.1)
    check(out_d.cpu().numpy(), lse_d.cpu().numpy(), ref_out, ref_lse, spread, score_bound(cache, 0, T, qw, 0.1, H))
    ctx.destroy()


@pytest.mark.parametrize("with_16_bit", [True, False])
def test_every_pair_of_formats_as_documents_of_one_request(with_16_bit):
    """One launch holds every pair: with 16-bit units among them the launch takes the kernel
    that fits all pairs, without them the one for narrow formats (launch_k6)."""
    L, H, D, g, n_qh = 1, 2, 128, 64, 4
    ORC = [16, 8, 4, 43, 52, 143]
    precs = range(6) if with_16_bit else range(1, 6)
    ctx = B.Context(L, H, D, 64, group_int8=g, group_int4=g)
    grp = lambda p: g if p in (B.PREC_INT8, B.PREC_INT4) else 0
    packed, tokens, bits, parts, units = [], [], [], [], []
    for i, (kp, vp) in enumerate((a, b) for a in precs for b in precs):
        T = 9 + (7 * i) % 40                                     # ragged, one to three blocks
        src = wl.kv_chunk(L, H, D, T, 900 + i)
        for part, prec in ((B.PART_K, kp), (B.PART_V, vp)):
            pk = codec.quantize_pack_half(np.ascontiguousarray(src[:, part - 1]), ORC[prec], g)[0]
            packed.append(pk)
            tokens.append(T)
            bits.append(ORC[prec])
            parts.append(part)
            units.append((dev_u8(pk), T, prec, grp(prec), part))
    n_kv = sum(tokens) // 2
    for n_q in (1, 5):                                           # 4 and 20 rows: one tile, two tiles
        qw = q_words(n_q, n_qh, D, 990 + n_q)
        q_d = torch.from_numpy(qw.view(np.int16)).cuda()
        out_d = torch.full((n_q, n_qh, D), float("nan"), dtype=torch.float32, device="cuda")
        lse_d = torch.full((n_q, n_qh), float("nan"), dtype=torch.float32, device="cuda")
        call = [(units, q_d, out_d, lse_d, n_q)]
        nb = ctx.attend_workspace_bytes(call, n_qh)
        ws = torch.full((nb // 4,), float("nan"), dtype=torch.float32, device="cuda")
        ctx.attend_packed(call, 0, n_qh, 0.1, ws, nb)
        torch.cuda.synchronize()
        cache, _ = codec.load_chunks(packed, (L, H, D), tokens, bits, [g] * len(units), list(range(len(units))),
                                     parts=parts)
        ref_out, ref_lse, spread = A.attend(cache, 0, n_kv, qw, 0.1)
        check(out_d.cpu().numpy(), lse_d.cpu().numpy(), ref_out, ref_lse, spread,
              score_bound(cache, 0, n_kv, qw, 0.1, H))
    ctx.destroy()


def test_the_most_query_tokens_and_the_widest_head_group_one_call_takes():
    # 4096 query tokens of one head group member (4096 query rows = 256 tiles over one chunk)
    run_case((1, 1, 128), [([48], [B.PREC_INT4], 4096)], 0, 1, 0.1, 810)
    # 64 query heads per KV head, one token
    run_case((1, 2, 128), [([20, 16], [B.PREC_INT8, B.PREC_16], 1)], 0, 128, 0.1, 811)


def test_the_most_requests_one_call_takes_and_one_more():
    reqs = [([16 + i % 5], [ALL[i % 6]], 1) for i in range(1024)]
    run_case((1, 1, 128), reqs, 0, 1, 0.1, 820)
    ctx = B.Context(1, 1, 128, 16, dry_run=True)
    P = 0x7F0000001000
    too_many = [([(P, 16, B.PREC_16, 0)], P, P, None, 1)] * 1025
    with pytest.raises(B.HaRagError) as e:
        ctx.attend_workspace_bytes(too_many, 1)
    assert e.value.code == B.EINVAL
    ctx.destroy()


@pytest.mark.parametrize("o_direct", [False, True])
def test_place_then_attend_with_every_chunk_starting_in_a_file(tmp_path, o_direct):
    """Algorithm 2 without the decode, then attention over the chunks where it left them: HBM
    copies filled straight from bounce buffers or pinned copies, pinned copies read over the
    link.  Afterwards a load of the same chunks must still equal the oracle's cache (the copies
    hold the right bytes)."""
    L, H, D, T, g = 2, 2, 128, 96, 64
    ORC = {B.PREC_INT4: 4, B.PREC_FP8_E4M3: 43}
    n = 10
    precs_all = [B.PREC_INT4, B.PREC_FP8_E4M3]
    ctx = B.Context(L, H, D, T, group_int8=g, group_int4=g, tau_gpu_ppm=200_000,
                    tau_pin_ppm=200_000, tau_page_ppm=200_000, disk_o_direct=o_direct)
    biggest, keep = 0, []
    for p in precs_all:
        slot = (ctx.chunk_bytes(p, T) + 4095) // 4096 * 4096
        biggest = max(biggest, slot)
        bufs = [torch.zeros(slot * 1, dtype=torch.uint8, device="cuda"), torch.zeros(slot * 4, dtype=torch.uint8).pin_memory(),
                torch.zeros(slot * 1, dtype=torch.uint8)]
        keep += bufs
        ctx.register_slab(B.TIER_HBM, p, bufs[0])
        ctx.register_slab(B.TIER_PINNED, p, bufs[1])
        ctx.register_slab(B.TIER_PAGEABLE, p, bufs[2])
        try:
            ctx.register_disk(p, str(tmp_path / f"pool_{p}.bin"), slot * n)
        except B.HaRagError as e:
            if o_direct and e.code == B.EIO:
                pytest.skip("this filesystem refuses O_DIRECT")
            raise
    ctx.register_staging(torch.zeros(biggest * 2, dtype=torch.uint8, device="cuda"))
    ctx.register_bounce(torch.zeros(biggest * 2, dtype=torch.uint8).pin_memory())
    tokens = [T - 5 * (i % 4) for i in range(n)]
    precs = [precs_all[i % 2] for i in range(n)]
    packed = [codec.quantize_pack_chunk(wl.kv_chunk(L, H, D, tokens[i], 1300 + i), ORC[p], g)[0]
              for i, p in enumerate(precs)]
    for i in range(n):
        ctx.pool_insert(i, precs[i], tokens[i], packed[i], B.TIER_DISK)
    ctx.set_counts(list(range(n)), [100 - i for i in range(n)])
    ctx.rerank()            # lists: GPU {0,1}, PIN {2,3}, PAGE {4,5}, DISK the rest

    ids = [0, 2, 4, 7, 1, 3, 8]
    # without the floor the chunks of the PAGE and DISK lists stay out of the kernels' reach
    st, tr = ctx.place_chunks(ids, want_trace=True)
    assert [t.found_tier for t in tr] == [3] * 7
    assert [t.placed_tier for t in tr] == [0, 1, 2, 255, 0, 1, 255]
    n_qh, scale, layer = 8, 0.09, 1
    qw = q_words(3, n_qh, D, 1400)
    q_d = torch.from_numpy(qw.view(np.int16)).cuda()
    out_d = torch.full((3, n_qh, D), float("nan"), dtype=torch.float32, device="cuda")
    lse_d = torch.full((3, n_qh), float("nan"), dtype=torch.float32, device="cuda")
    call = [(ids, q_d, out_d, lse_d, 3)]
    with pytest.raises(B.HaRagError) as e:
        ctx.attend_chunks_workspace_bytes(call, n_qh)
    assert e.value.code == B.ENOENT
    st, tr = ctx.place_chunks(ids, device_visible=True, want_trace=True)
    assert [t.found_tier for t in tr] == [0, 1, 2, 3, 0, 1, 3]
    assert [t.placed_tier for t in tr] == [255, 255, 1, 1, 255, 255, 1]
    nb = ctx.attend_chunks_workspace_bytes(call, n_qh)
    ws = torch.full((nb // 4,), float("nan"), dtype=torch.float32, device="cuda")
    ctx.attend_chunks(call, layer, n_qh, scale, ws, nb)
    torch.cuda.synchronize()
    cache, _ = codec.load_chunks(packed, (L, H, D), tokens, [ORC[p] for p in precs], [g] * n, ids)
    n_kv = sum(tokens[i] for i in ids)
    ref_out, ref_lse, spread = A.attend(cache, layer, n_kv, qw, scale)
    check(out_d.cpu().numpy(), lse_d.cpu().numpy(), ref_out, ref_lse, spread,
          score_bound(cache, layer, n_kv, qw, scale, H))
    # the copies hold the chunks' bytes: a load served from them equals the oracle's cache
    out = torch.zeros((L, 2, H, n_kv, D), dtype=torch.int16, device="cuda")
    st, tr = ctx.load_chunks(ids, out, n_kv, want_trace=True)
    torch.cuda.synchronize()
    assert all(t.found_tier in (0, 1) for t in tr)
    assert np.array_equal(out.cpu().numpy().view(np.uint16), cache)
    ctx.destroy()


def test_place_more_chunks_than_the_pinned_slab_holds_in_one_call(tmp_path):
    """One ha_rag_place_chunks call whose later chunks are given the pinned slots that its earlier
    chunks are still being copied out of: chunks 0 and 1 sit in the two pinned slots and belong
    in HBM (host -> device copies, queued behind other work on the stream); chunks 2 and 3 come
    from a file and belong in pinned memory, so they take over those very slots.  The host write
    into a slot has to wait for the copy that reads it: the HBM copies must hold the bytes the
    oracle packs for chunks 0 and 1, the pinned slots those of 2 and 3."""
    L, H, D, T = 8, 8, 128, 1024                              # 32 MiB per 16-bit chunk
    n = 4
    ctx = B.Context(L, H, D, T, tau_gpu_ppm=500_000, tau_pin_ppm=500_000)
    slot = (ctx.chunk_bytes(B.PREC_16, T) + 4095) // 4096 * 4096
    hbm = torch.zeros(slot * n, dtype=torch.uint8, device="cuda")
    pin = torch.zeros(slot * 2, dtype=torch.uint8).pin_memory()
    ctx.register_slab(B.TIER_HBM, B.PREC_16, hbm)
    ctx.register_slab(B.TIER_PINNED, B.PREC_16, pin)
    ctx.register_disk(B.PREC_16, str(tmp_path / "pool16.bin"), slot * n)
    ctx.register_bounce(torch.zeros(slot * 2, dtype=torch.uint8).pin_memory())
    packed = [codec.quantize_pack_chunk(wl.kv_chunk(L, H, D, T, 1500 + i), 16)[0] for i in range(n)]
    for i in range(n):
        ctx.pool_insert(i, B.PREC_16, T, packed[i], B.TIER_DISK)
    for i in range(2):
        ctx.pool_insert(i, B.PREC_16, T, packed[i], B.TIER_PINNED)
    ctx.set_counts(list(range(n)), [100 - i for i in range(n)])
    ctx.rerank()                                              # GPU list {0, 1}, PIN list {2, 3}
    stream = torch.cuda.Stream()
    a = torch.randn((8192, 8192), device="cuda")
    with torch.cuda.stream(stream):                           # work that the copies queue behind
        for _ in range(12):
            a = (a @ a) * 1e-4
    st, tr = ctx.place_chunks([0, 1, 2, 3], stream=stream, want_trace=True)
    assert [t.found_tier for t in tr] == [1, 1, 3, 3]
    assert [t.placed_tier for t in tr] == [0, 0, 1, 1]
    assert sorted(t.evicted_id for t in tr[2:]) == [0, 1]
    torch.cuda.synchronize()
    for i in range(n):
        tier = B.TIER_HBM if i < 2 else B.TIER_PINNED
        ptr, nbytes = ctx.pool_slot(i, tier)
        buf = hbm if i < 2 else pin
        off = ptr - buf.data_ptr()
        got = buf[off:off + nbytes].cpu().numpy()
        assert nbytes == len(packed[i]) and np.array_equal(got, packed[i]), i
    ctx.destroy()


def test_extreme_scores_and_values():
    """Query rows that are zero, tiny and huge; keys that tie, one that dominates, a masked tail;
    values of both signs up to 1e30: the running maximum, its rescaling and the normaliser must
    hold up (16-bit chunks, so that the awkward values survive storage unchanged)."""
    L, H, D, n_qh, T = 1, 1, 128, 4, 70                      # 70 tokens: a ragged fifth block
    rng = np.random.default_rng(77)
    x = rng.standard_normal((L, 2, H, T, D)).astype(np.float32)
    x[0, 0, 0, 10] = x[0, 0, 0, 11]                          # two identical keys
    x[0, 0, 0, 40] *= 30.0                                   # a key far out
    x[0, 0, 0, 69] *= 50.0                                   # the last valid token dominates some rows
    x[0, 1, 0, 5] = 1e30
    x[0, 1, 0, 6] = -1e30
    x[0, 1, 0, 20, :64] = 0.0
    src = wl.f32_to_bf16_words(x)
    q = rng.standard_normal((4, n_qh, D)).astype(np.float32)
    q[0, 0] = 0.0
    q[1, 1] *= 1e-20
    q[2, 2] *= 40.0
    q[3, 3] = x[0, 0, 0, 69] / 50.0                          # aligned with the far key
    qw = wl.f32_to_bf16_words(q)
    pk = codec.quantize_pack_chunk(src, 16)[0]
    ctx = B.Context(L, H, D, T)
    q_d = torch.from_numpy(qw.view(np.int16)).cuda()
    out_d = torch.full((4, n_qh, D), float("nan"), dtype=torch.float32, device="cuda")
    lse_d = torch.full((4, n_qh), float("nan"), dtype=torch.float32, device="cuda")
    call = [([(dev_u8(pk), T, B.PREC_16, 0)], q_d, out_d, lse_d, 4)]
    nb = ctx.attend_workspace_bytes(call, n_qh)
    ws = torch.full((nb // 4,), float("nan"), dtype=torch.float32, device="cuda")
    for scale in (0.088, 3.0):
        ctx.attend_packed(call, 0, n_qh, scale, ws, nb)
        torch.cuda.synchronize()
        cache, _ = codec.load_chunks([pk], (L, H, D), [T], [16], [128], [0])
        ref_out, ref_lse, spread = A.attend(cache, 0, T, qw, scale)
        out, lse = out_d.cpu().numpy(), lse_d.cpu().numpy()
        assert np.all(np.isfinite(out)) and np.all(np.isfinite(lse))
        check(out, lse, ref_out, ref_lse, spread, score_bound(cache, 0, T, qw, scale, H))
        assert abs(lse[0, 0] - np.log(T)) < 1e-5              # a zero query: uniform weights
    ctx.destroy()
