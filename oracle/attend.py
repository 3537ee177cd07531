"""Oracle for attention of a request's query tokens over its loaded chunks.

Test infrastructure only: the product never imports this file.

The paper's workflow (Sec. 2.1) hands the concatenated KV of the retrieved chunks to the
prefill of the question; what prefill computes with them is the textbook scaled dot-product
attention of the question's query vectors over those keys and values, which the paper does
not restate.  This file writes that definition out in binary64 on the BF16 cache the load
oracle produces:

    s[t]   = sm_scale * sum_d q[d] * K[t][d]
    out[d] = sum_t softmax(s)[t] * V[t][d],      lse = log(sum_t exp(s[t]))

for every query token and query head; query head hq reads KV head hq // (n_q_heads // H)
(grouped-query attention as LLaMA lays its heads out), every chunk token is visible to
every query token (the question follows the chunks), and (out, lse) is the pair a caller
merges with attention over other keys.
"""
import numpy as np


def bf16_words_to_f64(w):
    """BF16 words (uint16) to binary64, exactly."""
    return (np.asarray(w, np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def attend(cache_words, layer, n_kv, q_words, sm_scale):
    """cache_words: uint16 [L][2][H][cap][D] as the load oracle writes it, rows [0, n_kv) used.
    q_words: uint16 [n_q][n_q_heads][D].  Returns (out [n_q][n_q_heads][D], lse [n_q][n_q_heads],
    spread [n_q][n_q_heads][D]) in binary64; spread = sum_t softmax(s)[t] * |V[t][d]|, the
    quantity rounding errors of the weights scale with."""
    cache_words = np.asarray(cache_words)
    H, D = cache_words.shape[2], cache_words.shape[4]
    q = bf16_words_to_f64(q_words)
    n_q, n_qh, Dq = q.shape
    assert Dq == D and n_qh % H == 0 and 0 < n_kv <= cache_words.shape[3]
    G = n_qh // H
    out = np.zeros((n_q, n_qh, D))
    spread = np.zeros((n_q, n_qh, D))
    lse = np.zeros((n_q, n_qh))
    for hq in range(n_qh):
        K = bf16_words_to_f64(cache_words[layer, 0, hq // G, :n_kv])      # [n_kv][D]
        V = bf16_words_to_f64(cache_words[layer, 1, hq // G, :n_kv])
        for i in range(n_q):
            s = sm_scale * (K @ q[i, hq])
            m = s.max()
            p = np.exp(s - m)
            z = p.sum()
            out[i, hq] = (p @ V) / z
            spread[i, hq] = (p @ np.abs(V)) / z
            lse[i, hq] = m + np.log(z)
    return out, lse, spread


def merge(out_a, lse_a, out_b, lse_b):
    """Attention over the union of two disjoint key sets from the two partial results."""
    m = np.maximum(lse_a, lse_b)
    wa, wb = np.exp(lse_a - m), np.exp(lse_b - m)
    out = (out_a * wa[..., None] + out_b * wb[..., None]) / (wa + wb)[..., None]
    return out, m + np.log(wa + wb)
