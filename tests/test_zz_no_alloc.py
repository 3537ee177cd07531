"""ha_rag_attend_packed_static (the entry point that allocates nothing: its partial results live
in a static device array of the library) against ha_rag_attend_packed (caller's workspace) and
against the CPU oracle, through the C ABI, on two calls in a row on the same GPU, the second with
a smaller input: the array still holds the first call's records then.

Both entry points run the same kernels over the same plan, so their results are compared bit for
bit; the oracle comparison uses the tolerance derived in test_gpu_attend.py."""
import numpy as np
import pytest
import torch

from oracle import attend as A
from oracle import codec
from paper_2510_20878_amd import binding as B
from paper_2510_20878_amd import workloads as wl

pytestmark = pytest.mark.gpu

ORC = {B.PREC_16: 16, B.PREC_INT8: 8, B.PREC_INT4: 4, B.PREC_FP8_E4M3: 43, B.PREC_FP8_E5M2: 52,
       B.PREC_GSE8: 143}


def _one_call(ctx, shape, reqs, layer, n_qh, scale, seed, g=128):
    """reqs: list of (tokens, precs, n_q).  Runs both entry points and checks them."""
    L, H, D = shape
    keep, call_ws, call_st, refs = [], [], [], []
    k = 0
    for ri, (tokens, precs, n_q) in enumerate(reqs):
        packs = []
        for t, p in zip(tokens, precs):
            packs.append(codec.quantize_pack_chunk(wl.kv_chunk(L, H, D, t, seed + k), ORC[p], g)[0])
            k += 1
        rng = np.random.Generator(np.random.PCG64(seed + 1000 + ri))
        qw = wl.f32_to_bf16_words(rng.standard_normal((n_q, n_qh, D), dtype=np.float32))
        q_d = torch.from_numpy(qw.view(np.int16)).cuda()
        packs_d = [torch.from_numpy(p).cuda() for p in packs]
        chunks = [(pd, t, p, g if p in (B.PREC_INT8, B.PREC_INT4) else 0)
                  for pd, t, p in zip(packs_d, tokens, precs)]
        outs = []
        for _ in range(2):
            outs.append((torch.full((n_q, n_qh, D), float("nan"), dtype=torch.float32, device="cuda"),
                         torch.full((n_q, n_qh), float("nan"), dtype=torch.float32, device="cuda")))
        call_ws.append((chunks, q_d, outs[0][0], outs[0][1], n_q))
        call_st.append((chunks, q_d, outs[1][0], outs[1][1], n_q))
        keep += [q_d, packs_d, outs]
        refs.append((packs, tokens, precs, qw, outs))
    nbytes = ctx.attend_workspace_bytes(call_ws, n_qh)
    assert 0 < nbytes <= B.ATTEND_STATIC_SCRATCH_BYTES
    ws = torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device="cuda")
    print(f"attend_packed: {len(reqs)} requests, workspace {nbytes} bytes", flush=True)
    ctx.attend_packed(call_ws, layer, n_qh, scale, ws, nbytes)
    print("attend_packed_static", flush=True)
    ctx.attend_packed_static(call_st, layer, n_qh, scale)
    torch.cuda.synchronize()
    for packs, tokens, precs, qw, outs in refs:
        out_ws, lse_ws = outs[0][0].cpu().numpy(), outs[0][1].cpu().numpy()
        out_st, lse_st = outs[1][0].cpu().numpy(), outs[1][1].cpu().numpy()
        assert np.array_equal(out_st, out_ws) and np.array_equal(lse_st, lse_ws)
        n_kv = sum(tokens)
        cache, _ = codec.load_chunks(packs, shape, tokens, [ORC[p] for p in precs], [g] * len(precs),
                                     list(range(len(tokens))))
        ref_out, ref_lse, spread = A.attend(cache, layer, n_kv, qw, scale)
        qa = np.abs(A.bf16_words_to_f64(qw))
        G = n_qh // H
        sabs = np.stack([scale * (qa[:, hq] @ np.abs(A.bf16_words_to_f64(cache[layer, 0, hq // G, :n_kv])).T).max(axis=1)
                         for hq in range(n_qh)], axis=1)
        slack = 2.0 ** -15 * (1.0 + sabs)
        err = np.abs(out_st.astype(np.float64) - ref_out)
        assert np.all(err <= 2.0 ** -8 * spread + slack[..., None] * spread + 1e-30)
        assert np.all(np.abs(lse_st.astype(np.float64) - ref_lse) <= slack)
    return nbytes


def test_static_scratch_entry_equals_the_workspace_entry_on_two_calls_in_a_row():
    assert torch.cuda.is_available(), "this test needs the GPU"
    shape = (2, 2, 128)
    ctx = B.Context(*shape, 1300)
    first = [([1100, 513], [B.PREC_INT4, B.PREC_INT8], 4),
             ([40, 16, 77, 1, 33, 128], [B.PREC_16, B.PREC_INT8, B.PREC_INT4, B.PREC_FP8_E4M3,
                                         B.PREC_FP8_E5M2, B.PREC_GSE8], 3),
             ([300], [B.PREC_GSE8], 21)]
    n1 = _one_call(ctx, shape, first, 1, 8, 0.12, 700)
    # smaller: fewer records, other shapes of them; the array still holds the first call's
    second = [([50, 96], [B.PREC_INT4, B.PREC_16], 1)]
    n2 = _one_call(ctx, shape, second, 0, 8, 0.1, 800)
    assert n2 < n1
    ctx.destroy()


def test_static_scratch_entry_refuses_what_exceeds_its_limits():
    assert torch.cuda.is_available(), "this test needs the GPU"
    shape = (1, 1, 128)
    ctx = B.Context(*shape, 4096)
    pk = torch.zeros(ctx.chunk_bytes(B.PREC_INT4, 4096), dtype=torch.uint8, device="cuda")
    # 2,048 query tiles in 128 groups of eight-wave workgroups: two runs of the document's 256 blocks
    # fill the chip's 256 places, and two records per tile are 34 MB (one run would need no record at all)
    n_q, n_qh = 1024, 32
    q = torch.zeros((n_q, n_qh, 128), dtype=torch.int16, device="cuda")
    out = torch.zeros((n_q, n_qh, 128), dtype=torch.float32, device="cuda")
    big = [([(pk, 4096, B.PREC_INT4, 128)], q, out, None, n_q)]
    assert ctx.attend_workspace_bytes(big, n_qh) > B.ATTEND_STATIC_SCRATCH_BYTES
    with pytest.raises(B.HaRagError) as e:
        ctx.attend_packed_static(big, 0, n_qh, 0.1)
    assert e.value.code == B.ENOSPC and "scratch array holds" in str(e.value)
    small = [([(pk, 16, B.PREC_INT4, 128)], q, out, None, 1)]
    with pytest.raises(B.HaRagError) as e:
        ctx.attend_packed_static(small * (B.ATTEND_STATIC_MAX_REQUESTS + 1), 0, n_qh, 0.1)
    assert e.value.code == B.ENOSPC and "requests" in str(e.value)
    with pytest.raises(B.HaRagError) as e:
        ctx.attend_packed_static([([(pk, 16, B.PREC_INT4, 128)] * (B.ATTEND_STATIC_MAX_DOCS + 1),
                                   q, out, None, 1)], 0, n_qh, 0.1)
    assert e.value.code == B.ENOSPC and "documents" in str(e.value)
    torch.cuda.synchronize()
    ctx.destroy()
