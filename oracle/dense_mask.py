"""Dense-mask brute force of the whole APE attention pattern (numpy, fp64).

TEST INFRASTRUCTURE ONLY, for tiny inputs: it materialises the full score
matrix of the sequence ``[prefix ; C_1 ; ... ; C_N ; query]`` and applies the
paper's equations with raw ``exp`` and ``**`` -- no max-subtraction, no
LogSumExp, no blocks -- so that it shares no trick with ``ape_oracle.c`` and
none with the GPU kernels.

Rows and what they see (arXiv 2502.05431, Sections 2.2, 4.1, 4.4):
  prefix row r        : prefix tokens 0..r                      (plain causal)
  row r of context i  : all prefix tokens + tokens 0..r of C_i  (plain causal)
  query row r         : all prefix, ALL context tokens, query tokens 0..r,
                        with the refined equation of Section 4.4 ("Eq.5"):
                        context scores divided by T, the context partition sum
                        raised to the power S.
"""
from __future__ import annotations

import numpy as np


def ape_dense(q_all, k_all, v_all, prefix_len, chunk_lens, T, S):
    """All arrays are [L, heads, d] over the concatenated sequence
    L = prefix_len + sum(chunk_lens) + l_query (q_all: Hq heads; k/v: Hkv heads).

    Returns (out [L, Hq, d], weights [Hq, L, L]) in float64.
    """
    q_all = np.asarray(q_all, dtype=np.float64)
    k_all = np.asarray(k_all, dtype=np.float64)
    v_all = np.asarray(v_all, dtype=np.float64)
    L, hq, d = q_all.shape
    hkv = k_all.shape[1]
    g = hq // hkv
    m = int(sum(chunk_lens))
    q0 = prefix_len + m                       # first query row
    # token kinds: -1 prefix, i >= 0 context i, -2 query
    kind = np.full(L, -2, dtype=np.int64)
    kind[:prefix_len] = -1
    t = prefix_len
    for i, li in enumerate(chunk_lens):
        kind[t:t + li] = i
        t += li
    idx = np.arange(L)
    causal = idx[None, :] <= idx[:, None]
    same = kind[None, :] == kind[:, None]
    is_prefix_col = (kind == -1)[None, :]
    is_ctx_col = (kind >= 0)[None, :]
    is_query_row = (kind == -2)[:, None]
    # visibility mask [row, col]
    mask = (is_prefix_col & causal) | (same & causal) | (is_query_row & is_ctx_col)

    out = np.zeros((L, hq, d))
    weights = np.zeros((hq, L, L))
    for h in range(hq):
        hk = h // g
        s = q_all[:, h, :] @ k_all[:, hk, :].T / np.sqrt(d)          # [L, L]
        # query rows x context columns carry the temperature
        s_eff = np.where(is_query_row & is_ctx_col, s / T, s)
        a = np.where(mask, np.exp(s_eff), 0.0)
        ctx_part = is_query_row & is_ctx_col & mask
        z_ctx = np.where(ctx_part, a, 0.0).sum(axis=1, keepdims=True)          # sum of a'
        z_other = np.where(~ctx_part, a, 0.0).sum(axis=1, keepdims=True)       # prefix + own
        has_ctx = z_ctx > 0
        z_ctx_safe = np.where(has_ctx, z_ctx, 1.0)
        denom = z_other + np.where(has_ctx, z_ctx_safe ** S, 0.0)
        numer = np.where(ctx_part, a * z_ctx_safe ** (S - 1.0), a)
        w = numer / denom
        weights[h] = w
        out[:, h, :] = w @ v_all[:, hk, :]
    return out, weights
