"""Pins of the attention oracle (CPU): a library routine, closed forms, invariances and brute
force, each of which a plausible slip (head mapping, missing scale, K/V planes swapped, wrong
normaliser, wrong layer) breaks."""
import math

import numpy as np
import torch

from oracle import attend as A
from oracle import codec


def _words(x):
    """float array -> BF16 words (library conversion)."""
    return torch.from_numpy(np.ascontiguousarray(x, np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def _case(L=2, H=2, D=16, n=37, n_q=3, G=2, seed=0, cap_extra=5):
    rng = np.random.default_rng(seed)
    cache = _words(rng.standard_normal((L, 2, H, n + cap_extra, D)))
    q = _words(rng.standard_normal((n_q, H * G, D)))
    return cache, q


def test_equals_torch_sdpa_with_grouped_heads():
    L, H, D, n, n_q, G = 3, 2, 32, 150, 5, 4
    cache, q = _case(L, H, D, n, n_q, G, seed=1)
    scale = 0.3
    for layer in range(L):
        out, lse, _ = A.attend(cache, layer, n, q, scale)
        c = torch.from_numpy(cache.view(np.int16)).view(torch.bfloat16).double()
        K = c[layer, 0, :, :n]                                     # [H][n][D]
        V = c[layer, 1, :, :n]
        Q = torch.from_numpy(q.view(np.int16)).view(torch.bfloat16).double().permute(1, 0, 2)   # [Hq][n_q][D]
        ref = torch.nn.functional.scaled_dot_product_attention(
            Q[None], K[None], V[None], scale=scale, enable_gqa=True)[0].permute(1, 0, 2).numpy()
        assert np.allclose(out, ref, rtol=0, atol=1e-12)
        s = scale * torch.einsum("hqd,hnd->hqn", Q, K.repeat_interleave(G, dim=0))
        assert np.allclose(lse, torch.logsumexp(s, -1).T.numpy(), rtol=0, atol=1e-12)


def test_brute_force_loops_on_a_tiny_case():
    L, H, D, n, n_q, G = 1, 2, 4, 3, 2, 2
    cache, q = _case(L, H, D, n, n_q, G, seed=2, cap_extra=2)
    f = lambda w: float(A.bf16_words_to_f64(np.array([w], np.uint16))[0])
    out, lse, spread = A.attend(cache, 0, n, q, 0.5)
    for i in range(n_q):
        for hq in range(H * G):
            h = hq // G
            s = [0.5 * sum(f(q[i, hq, d]) * f(cache[0, 0, h, t, d]) for d in range(D)) for t in range(n)]
            z = sum(math.exp(x) for x in s)
            assert abs(lse[i, hq] - math.log(z)) < 1e-12
            for d in range(D):
                o = sum(math.exp(s[t]) * f(cache[0, 1, h, t, d]) for t in range(n)) / z
                a = sum(math.exp(s[t]) * abs(f(cache[0, 1, h, t, d])) for t in range(n)) / z
                assert abs(out[i, hq, d] - o) < 1e-12 and abs(spread[i, hq, d] - a) < 1e-12


def test_zero_keys_give_the_mean_of_the_values_and_log_n():
    cache, q = _case(n=64, seed=3)
    cache[:, 0] = 0
    out, lse, _ = A.attend(cache, 1, 64, q, 1.0)
    V = A.bf16_words_to_f64(cache[1, 1, :, :64])                   # [H][n][D]
    assert np.allclose(out[:, 0::2], V.mean(1)[None], atol=1e-12) and np.allclose(out[:, 1::2], V.mean(1)[None], atol=1e-12)
    assert np.allclose(lse, math.log(64), atol=1e-12)


def test_one_dominant_key_selects_its_value_row():
    L, H, D, n = 1, 1, 8, 20
    cache, q = _case(L, H, D, n, n_q=1, G=1, seed=4)
    cache[0, 0, 0, :n] = 0
    qv = np.zeros(D, np.float32); qv[2] = 4.0
    q[0, 0] = _words(qv)
    kv = np.zeros(D, np.float32); kv[2] = 64.0                     # score 256 * scale against 0 elsewhere
    cache[0, 0, 0, 7] = _words(kv)
    out, lse, _ = A.attend(cache, 0, n, q, 1.0)
    assert np.allclose(out[0, 0], A.bf16_words_to_f64(cache[0, 1, 0, 7]), atol=1e-100)
    assert abs(lse[0, 0] - 256.0) < 1e-12


def test_rows_beyond_n_kv_and_other_layers_do_not_matter():
    cache, q = _case(L=2, n=30, cap_extra=9, seed=5)
    a = A.attend(cache, 0, 30, q, 0.7)
    cache2 = cache.copy()
    cache2[:, :, :, 30:] = _words(np.full(cache[:, :, :, 30:].shape, 99.0))
    cache2[1] = 0
    b = A.attend(cache2, 0, 30, q, 0.7)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))


def test_adding_one_vector_to_every_key_shifts_lse_only():
    cache, q = _case(H=1, G=2, D=8, n=40, seed=6)
    u = np.array([0.5, -1, 0, 2, 0, 0, 0.25, 0], np.float64)
    K = A.bf16_words_to_f64(cache[0, 0, 0])
    cache2 = cache.copy()
    K2 = np.round(K * 4) / 4                                       # quarters: the sums stay BF16 values
    cache[0, 0, 0] = _words(K2)
    cache2[0, 0, 0] = _words(K2 + u)
    assert np.array_equal(A.bf16_words_to_f64(cache2[0, 0, 0]), A.bf16_words_to_f64(cache[0, 0, 0]) + u)
    o1, l1, _ = A.attend(cache, 0, 40, q, 0.2)
    o2, l2, _ = A.attend(cache2, 0, 40, q, 0.2)
    assert np.allclose(o1, o2, atol=1e-12)
    assert np.allclose(l2 - l1, 0.2 * (A.bf16_words_to_f64(q)[:, :, :] @ u), atol=1e-12)


def test_merging_two_halves_equals_the_whole():
    cache, q = _case(n=50, seed=7)
    whole = A.attend(cache, 1, 50, q, 0.4)
    first = A.attend(cache, 1, 20, q, 0.4)
    rest = cache.copy()
    rest[:, :, :, :30] = cache[:, :, :, 20:50]
    second = A.attend(rest, 1, 30, q, 0.4)
    out, lse = A.merge(first[0], first[1], second[0], second[1])
    assert np.allclose(out, whole[0], atol=1e-12) and np.allclose(lse, whole[1], atol=1e-12)


def test_over_loaded_chunks_the_full_precision_tag_is_attention_over_the_sources():
    """With every chunk at 16 bits the cache is the concatenation of the sources, so the
    result is attention over the concatenated source rows."""
    L, H, D = 2, 2, 64
    rng = np.random.default_rng(8)
    tokens = [20, 7, 33]
    srcs = [_words(rng.standard_normal((L, 2, H, t, D))) for t in tokens]
    packed = [codec.quantize_pack_chunk(s, 16)[0] for s in srcs]
    order = [2, 0, 1]
    cache, _ = codec.load_chunks(packed, (L, H, D), tokens, [16] * 3, [64] * 3, order)
    q = _words(rng.standard_normal((2, 4, D)))
    cat = np.concatenate([srcs[c] for c in order], axis=3)
    a = A.attend(cache, 1, sum(tokens), q, 0.125)
    b = A.attend(cat, 1, sum(tokens), q, 0.125)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
