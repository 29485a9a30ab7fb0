"""Pins of the fp64 layer oracle (the published Llama layer around the block-diagonal encode
attention of arXiv 2502.05431, Sections 2.2 / 4.1) against torch's own operators."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import ape_oracle, layer_oracle


def _weights(rng, hidden, hq, hkv, d, inter, scale=1.0):
    g = lambda *s: rng.standard_normal(s) * scale
    return {"attn_norm": 1.0 + 0.1 * g(hidden), "wq": g(hq * d, hidden) / np.sqrt(hidden), "wk": g(hkv * d, hidden) / np.sqrt(hidden),
            "wv": g(hkv * d, hidden) / np.sqrt(hidden), "wo": g(hidden, hq * d) / np.sqrt(hq * d), "mlp_norm": 1.0 + 0.1 * g(hidden),
            "wg": g(inter, hidden) / np.sqrt(hidden), "wu": g(inter, hidden) / np.sqrt(hidden), "wd": g(hidden, inter) / np.sqrt(inter)}


def _torch_layer(x, w, hq, hkv, d, base, eps):
    """One causal sequence, no prefix: the layer composed from torch operators in fp64."""
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    x = t(x)
    m, hidden = x.shape
    h = F.rms_norm(x, (hidden,), t(w["attn_norm"]), eps)
    q = F.linear(h, t(w["wq"])).view(m, hq, d)
    k = F.linear(h, t(w["wk"])).view(m, hkv, d)
    v = F.linear(h, t(w["wv"])).view(m, hkv, d)
    half = d // 2
    inv = base ** (-torch.arange(half, dtype=torch.float64) * 2.0 / d)
    ang = torch.arange(m, dtype=torch.float64)[:, None] * inv[None, :]
    cos, sin = ang.cos()[:, None, :], ang.sin()[:, None, :]
    rot = lambda z: torch.cat([z[..., :half] * cos - z[..., half:] * sin, z[..., half:] * cos + z[..., :half] * sin], dim=-1)
    q, k = rot(q), rot(k)
    rep = hq // hkv
    a = F.scaled_dot_product_attention(q.permute(1, 0, 2)[None], k.permute(1, 0, 2).repeat_interleave(rep, 0)[None],
                                       v.permute(1, 0, 2).repeat_interleave(rep, 0)[None], is_causal=True)[0]
    a = a.permute(1, 0, 2).reshape(m, hq * d)
    x1 = x + F.linear(a, t(w["wo"]))
    h2 = F.rms_norm(x1, (hidden,), t(w["mlp_norm"]), eps)
    y = x1 + F.linear(F.silu(F.linear(h2, t(w["wg"]))) * F.linear(h2, t(w["wu"])), t(w["wd"]))
    return y.numpy()


def test_single_context_layer_equals_torch_composition():
    rng = np.random.default_rng(0)
    hidden, hq, hkv, d, inter, m = 48, 4, 2, 16, 80, 21
    w = _weights(rng, hidden, hq, hkv, d, inter)
    x = rng.standard_normal((m, hidden))
    got = layer_oracle.layer_encode(x, w, [m], None, None, hq, hkv, d, 10000.0, 1e-5)
    ref = _torch_layer(x, w, hq, hkv, d, 10000.0, 1e-5)
    np.testing.assert_allclose(got["y"], ref, atol=2e-6)       # q, k, v pass through float32 on the way to the attention oracle


def test_contexts_are_independent_and_share_positions():
    """Two contexts in one call = each context alone (block-diagonal attention, positions restart)."""
    rng = np.random.default_rng(1)
    hidden, hq, hkv, d, inter = 32, 2, 1, 16, 40
    w = _weights(rng, hidden, hq, hkv, d, inter)
    x = rng.standard_normal((19, hidden))
    both = layer_oracle.layer_encode(x, w, [12, 7], None, None, hq, hkv, d, 10000.0, 1e-5)["y"]
    a = layer_oracle.layer_encode(x[:12], w, [12], None, None, hq, hkv, d, 10000.0, 1e-5)["y"]
    b = layer_oracle.layer_encode(x[12:], w, [7], None, None, hq, hkv, d, 10000.0, 1e-5)["y"]
    np.testing.assert_allclose(both, np.concatenate([a, b]), atol=1e-12)
    b_torch = _torch_layer(x[12:], w, hq, hkv, d, 10000.0, 1e-5)
    np.testing.assert_allclose(both[12:], b_torch, atol=2e-6)


def test_prefix_shifts_positions_and_is_attended():
    """With a cached prefix of l_P tokens the contexts start at position l_P: the layer over
    [prefix ; context] as one sequence gives the same context rows."""
    rng = np.random.default_rng(2)
    hidden, hq, hkv, d, inter, lp, m = 32, 2, 2, 16, 40, 5, 9
    w = _weights(rng, hidden, hq, hkv, d, inter)
    xp, xc = rng.standard_normal((lp, hidden)), rng.standard_normal((m, hidden))
    pre = layer_oracle.layer_encode(xp, w, [lp], None, None, hq, hkv, d, 10000.0, 1e-5)
    got = layer_oracle.layer_encode(xc, w, [m], pre["k"].astype(np.float32), pre["v"].astype(np.float32), hq, hkv, d, 10000.0, 1e-5)["y"]
    ref = _torch_layer(np.concatenate([xp, xc]), w, hq, hkv, d, 10000.0, 1e-5)[lp:]
    np.testing.assert_allclose(got, ref, atol=5e-6)


def test_pieces():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((4, 24))
    wn = rng.standard_normal(24)
    ref = F.rms_norm(torch.from_numpy(x), (24,), torch.from_numpy(wn), 1e-6).numpy()
    np.testing.assert_allclose(layer_oracle.rmsnorm(x, wn, 1e-6), ref, atol=1e-14)
    t = rng.standard_normal(100) * 4
    np.testing.assert_allclose(layer_oracle.silu(t), F.silu(torch.from_numpy(t)).numpy(), atol=1e-14)
    z = rng.standard_normal((11, 3, 32)).astype(np.float32)
    np.testing.assert_allclose(layer_oracle.rope_f64(z, [4, 7], 3, 500000.0), ape_oracle.rope(z, [4, 7], 3, 500000.0), atol=1e-13)
    # zero output projections: the layer is the identity
    w = _weights(rng, 24, 2, 1, 8, 16)
    w["wo"] = np.zeros_like(w["wo"]); w["wd"] = np.zeros_like(w["wd"])
    np.testing.assert_array_equal(layer_oracle.layer_encode(x, w, [4], None, None, 2, 1, 8, 1e4, 1e-5)["y"], x)


def test_row_selection():
    rng = np.random.default_rng(4)
    w = _weights(rng, 32, 2, 1, 16, 40)
    x = rng.standard_normal((15, 32))
    full = layer_oracle.layer_encode(x, w, [8, 7], None, None, 2, 1, 16, 1e4, 1e-5)["y"]
    some = layer_oracle.layer_encode(x, w, [8, 7], None, None, 2, 1, 16, 1e4, 1e-5, rows=[0, 7, 8, 14])["y"]
    np.testing.assert_allclose(some, full[[0, 7, 8, 14]], atol=1e-13)
