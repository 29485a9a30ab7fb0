"""Plain fp64 numpy oracle of ONE transformer layer around the block-diagonal encode attention.

TEST INFRASTRUCTURE ONLY (imported by tests and by bench.py's optional layer check; never by the
product path).  The paper (arXiv 2502.05431) measures end-to-end prefill of Llama-3-8B
(Section 5.4); it prints no layer equations, so the layer is the published Llama architecture:

    h  = RMSNorm(x; w_attn_norm)                         x: [M, hidden], the packed contexts
    q, k, v = h Wq^T, h Wk^T, h Wv^T                     rows reshaped [heads, d]
    q, k <- rotary embedding, token j of every context at position prefix_len + j
            (positions re-used across contexts, Section 1)
    a  = block-diagonal causal attention of Section 2.2 / 4.1 (prefix KV + own context)
    x1 = x + a Wo^T
    y  = x1 + (SiLU(g) * u) Wd^T,  [g, u] = RMSNorm(x1; w_mlp_norm) [Wg; Wu]^T

RMSNorm(x; w) = x / sqrt(mean(x^2) + eps) * w;  SiLU(t) = t / (1 + exp(-t)).
Weights are [out_features, in_features] row-major.  The attention step calls the C oracle
(``ape_oracle.encode``), which reads float32: q, k, v are rounded to float32 on the way in
(relative 6e-8, far below every tolerance used with this oracle); everything else is float64.
"""
from __future__ import annotations

import numpy as np

from . import ape_oracle


def rmsnorm(x, w, eps):
    x = np.asarray(x, dtype=np.float64)
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * np.asarray(w, dtype=np.float64)


def rope_f64(x, chunk_lens, position_offset, base):
    """Rotary embedding, half-split pairing, positions restarting in every segment; x [M, H, d] float64."""
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    half = d // 2
    pos = np.concatenate([position_offset + np.arange(l, dtype=np.float64) for l in chunk_lens]) if len(chunk_lens) else np.zeros(0)
    inv = np.power(float(base), -2.0 * np.arange(half, dtype=np.float64) / d)
    ang = pos[:, None] * inv[None, :]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(t):
    return t / (1.0 + np.exp(-t))


def layer_encode(x, w, chunk_lens, k_prefix, v_prefix, n_q_heads, n_kv_heads, head_dim, rope_base, eps, rows=None):
    """One layer over the packed contexts ``x`` [M, hidden].

    ``w``: dict with attn_norm [hidden], wq [Hq d, hidden], wk, wv [Hkv d, hidden], wo [hidden, Hq d],
    mlp_norm [hidden], wg, wu [I, hidden], wd [hidden, I].  ``k_prefix``/``v_prefix``: this layer's
    cached prefix KV [l_P, Hkv, d] (already rotated).  ``rows``: packed row indices to return (default all).
    Returns dict(y [n, hidden], k [M, Hkv, d] rotated, v [M, Hkv, d], q [M, Hq, d] rotated, x1 [n, hidden]).
    """
    f = lambda a: np.asarray(a, dtype=np.float64)
    x = f(x)
    m = x.shape[0]
    lp = 0 if k_prefix is None else k_prefix.shape[0]
    h = rmsnorm(x, w["attn_norm"], eps)
    q = (h @ f(w["wq"]).T).reshape(m, n_q_heads, head_dim)
    k = (h @ f(w["wk"]).T).reshape(m, n_kv_heads, head_dim)
    v = (h @ f(w["wv"]).T).reshape(m, n_kv_heads, head_dim)
    q = rope_f64(q, chunk_lens, lp, rope_base)
    k = rope_f64(k, chunk_lens, lp, rope_base)
    sel = np.arange(m) if rows is None else np.asarray(rows)
    pairs = [(int(r), hh) for r in sel for hh in range(n_q_heads)]
    a, _ = ape_oracle.encode(q.astype(np.float32), k_prefix, v_prefix, k.astype(np.float32), v.astype(np.float32),
                             list(chunk_lens), pairs=pairs)
    a = a.reshape(len(sel), n_q_heads * head_dim)
    x1 = x[sel] + a @ f(w["wo"]).T
    h2 = rmsnorm(x1, w["mlp_norm"], eps)
    g, u = h2 @ f(w["wg"]).T, h2 @ f(w["wu"]).T
    y = x1 + (silu(g) * u) @ f(w["wd"]).T
    return {"y": y, "k": k, "v": v, "q": q, "x1": x1}
