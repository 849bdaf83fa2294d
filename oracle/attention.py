"""CPU oracle, attention-side operators: rotary embedding with the QKV layout transformation
(section 3.6 of the paper) and the two matrix products of attention with the KV cache in the
role of weights (section 3.8).

TEST INFRASTRUCTURE ONLY (same rule as the package).  Plain numpy in fp64, one function per
operator, nothing blocked or reordered.  It imports nothing from the GPU package.

The paper gives the layouts - queries as (B * h_kv, S * h_q / h_kv, d_h), the K cache as
(cache_size, d_h) per KV head (K^T of the product Q K^T), the V cache as (d_h, cache_size) - and
no formulas; rotary embedding and scaled-dot-product attention are taken in their standard form
(rotation of the pairs (i, i + d_h / 2) by pos * base^(-2 i / d_h); softmax(Q K^T / sqrt(d_h)) V
with a causal mask).
"""
from __future__ import annotations

import numpy as np


def rope(x, pos, base: float) -> np.ndarray:
    """Rotary embedding of vectors x [..., d] at integer positions pos (broadcast over the leading
    axes): (x[i], x[i + d/2]) is rotated by the angle pos * base^(-2 i / d).  fp64."""
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    half = d // 2
    i = np.arange(half, dtype=np.float64)
    ang = np.asarray(pos, dtype=np.float64)[..., None] * base ** (-2.0 * i / d)
    c, s = np.cos(ang), np.sin(ang)
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def rope_qkv_layout_exact(qkv, pos0: int, h_q: int, h_kv: int, d: int, base: float):
    """The same transformation on real (fp64) projection outputs [B, S, (h_q + 2 h_kv) d], nothing
    rounded: what the merged operator (QKV layer + rotary embedding + layout transformation,
    section 3.6) computes before its single rounding to binary16.  Returns q [B * h_kv, S * g, d],
    k [B * h_kv, S, d], v [B * h_kv, S, d] in fp64."""
    x = np.asarray(qkv, dtype=np.float64)
    B, S, W = x.shape
    g = h_q // h_kv
    assert W == (h_q + 2 * h_kv) * d and h_q == g * h_kv
    pos = pos0 + np.arange(S)
    q = x[:, :, : h_q * d].reshape(B, S, h_kv, g, d)
    k = x[:, :, h_q * d: (h_q + h_kv) * d].reshape(B, S, h_kv, d)
    v = x[:, :, (h_q + h_kv) * d:].reshape(B, S, h_kv, d)
    q = rope(q, pos[None, :, None, None], base)
    k = rope(k, pos[None, :, None], base)
    q = q.transpose(0, 2, 1, 3, 4).reshape(B * h_kv, S * g, d)
    k = k.transpose(0, 2, 1, 3).reshape(B * h_kv, S, d)
    v = v.transpose(0, 2, 1, 3).reshape(B * h_kv, S, d)
    return q, k, v


def rope_qkv_layout(qkv_f16, pos0: int, h_q: int, h_kv: int, d: int, base: float):
    """From the QKV projection's output [B, S, (h_q + 2 h_kv) d] (query heads, then key heads, then
    value heads) to the attention layouts, all rounded once to binary16:
      q  [B * h_kv, S * g, d], g = h_q / h_kv, row s * g + j = query head kv * g + j at token s, rotated
      k  [B * h_kv, S, d]      rotated: the rows appended to the K cache at positions pos0 + s
      v  [B * h_kv, S, d]      as is: appended to the V cache as columns pos0 + s
    """
    x = np.asarray(qkv_f16, dtype=np.float16).astype(np.float64)
    q, k, v = rope_qkv_layout_exact(x, pos0, h_q, h_kv, d, base)
    return q.astype(np.float16), k.astype(np.float16), v.astype(np.float16)


def attention(q_f16, kcache_f16, vcache_f16, n_ctx: int, S: int) -> np.ndarray:
    """out[G, S * g, d] = softmax(q K^T / sqrt(d)) V per group G = (batch, KV head), fp64.

    q [G, S * g, d]; kcache [G, C, d] (rows = positions); vcache [G, d, C] (columns = positions);
    the first n_ctx positions are valid and the S query tokens are the last S of them: the rows of
    token s see positions 0 .. n_ctx - S + s.
    """
    q = np.asarray(q_f16, dtype=np.float16).astype(np.float64)
    K = np.asarray(kcache_f16, dtype=np.float16).astype(np.float64)
    V = np.asarray(vcache_f16, dtype=np.float16).astype(np.float64)
    G, M, d = q.shape
    g = M // S
    out = np.empty((G, M, d), dtype=np.float64)
    for gi in range(G):
        for m in range(M):
            lim = n_ctx - S + m // g + 1
            sc = K[gi, :lim] @ q[gi, m] / np.sqrt(d)
            p = np.exp(sc - sc.max())
            p /= p.sum()
            out[gi, m] = V[gi, :, :lim] @ p
    return out
