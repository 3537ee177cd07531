"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws random numbers and lays them out; it contains none of
the method's arithmetic (no quantisation, packing or dequantisation) and is the
one module that both the tests' CPU oracle and the HIP path are fed from.

The paper measures on KV chunks computed by LLaMA-2-7B from MS MARCO passages
(Sec. 3.1); neither is available here, so Gaussian tensors stand in for them.
Sec. 2.2.1 reports Keys within about (-25, 25) and Values within (-10, 10): Keys
get a per-channel log-normal spread, Values stay unit Gaussian.  Sec. 1 reports
that about 1 % of the documents draw most retrievals: chunk ids are drawn from a
Zipf law.
"""
import numpy as np
import torch


def f32_to_bf16_words(x: np.ndarray) -> np.ndarray:
    """float32 array -> uint16 array of BF16 words (library conversion, nearest-even)."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bf16_words_to_f32(w: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(w, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def kv_chunk(L, H, D, T, seed, key_spread=True, outlier_channels=0, outlier_gain=15.0):
    """One document's KV as BF16 words, shape [L][2][H][T][D].

    key_spread        K (index 0 of axis 1) is multiplied per (l, h, d) channel by
                      a lognormal(0, 1) factor; V stays N(0, 1).
    outlier_channels  that many head_dim channels per (l, kv, h), picked by the
                      same generator, are multiplied by outlier_gain on all tokens.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.standard_normal((L, 2, H, T, D), dtype=np.float32)
    if key_spread:
        c = rng.lognormal(0.0, 1.0, size=(L, 1, H, 1, D)).astype(np.float32)
        x[:, 0:1] *= c
    if outlier_channels:
        for l in range(L):
            for kv in range(2):
                for h in range(H):
                    ch = rng.choice(D, size=outlier_channels, replace=False)
                    x[l, kv, h, :, ch] *= np.float32(outlier_gain)
    return f32_to_bf16_words(x)


def tiny_config(seed=0):
    """The small parity case: 2 layers, 2 KV heads, head_dim 64, 4 chunks x 128
    tokens, tags [16, 8, 4, 4] bits, group 64, N(0,1) with 2 outlier channels per
    head scaled x15, gathered in the order [3, 0, 2, 1]."""
    L, H, D, T = 2, 2, 64, 128
    chunks = [kv_chunk(L, H, D, T, seed * 1000 + i, key_spread=False, outlier_channels=2)
              for i in range(4)]
    return dict(shape=(L, H, D), tokens=[T] * 4, bits=[16, 8, 4, 4], group=[64] * 4,
                order=[3, 0, 2, 1], chunks=chunks)


def patterned_chunk(L, H, D, T, chunk_no):
    """Every element encodes (chunk, token) in a value BF16 holds exactly
    (integers below 256), to check gather order and token offsets by eye."""
    x = np.zeros((L, 2, H, T, D), np.float32)
    x[...] = float(chunk_no % 128)
    x[..., 0] = (np.arange(T, dtype=np.float32) % 256)[None, None, None, :]
    return f32_to_bf16_words(x)


def zipf_pmf(n, s=1.1):
    w = 1.0 / np.power(np.arange(1, n + 1, dtype=np.float64), s)
    return w / w.sum()


def zipf_requests(n_ids, n_requests, per_request, seed, s=1.1):
    """Ranks (0 = hottest) drawn from Zipf(s); ids inside one request are distinct
    (a repeated draw is drawn again).  Returns int64 [n_requests][per_request]."""
    rng = np.random.Generator(np.random.PCG64(seed))
    cdf = np.cumsum(zipf_pmf(n_ids, s))
    out = np.empty((n_requests, per_request), np.int64)
    for r in range(n_requests):
        seen = []
        while len(seen) < per_request:
            c = int(np.searchsorted(cdf, rng.random(), side="right"))
            c = min(c, n_ids - 1)
            if c not in seen:
                seen.append(c)
        out[r] = seen
    return out


def tags_by_rank_fraction(n, fractions=(0.2, 0.3), bits=(16, 8, 4)):
    """Bits per rank position: the first fractions[0] of the ranks get bits[0], ..."""
    out = np.full(n, bits[-1], np.int32)
    lo = 0
    for f, b in zip(fractions, bits):
        hi = lo + int(f * n)
        out[lo:hi] = b
        lo = hi
    return out


def kv_chunk_device(L, H, D, T, seed, device="cuda", key_spread=True):
    """Same distribution as kv_chunk, drawn on the device by torch's generator
    (for pools too large to draw on the host).  Returns a bf16 tensor."""
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    x = torch.randn((L, 2, H, T, D), generator=g, device=device, dtype=torch.float32)
    if key_spread:
        c = torch.exp(torch.randn((L, 1, H, 1, D), generator=g, device=device))
        x[:, 0:1] *= c
    return x.to(torch.bfloat16)
