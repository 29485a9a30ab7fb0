"""GPU parity of the layer library (ape_layer_encode: one transformer layer around the
block-diagonal encode attention; ape_layers_encode: a stack of them) against the fp64 layer oracle,
through the C ABI.  The attention inside the layer is also checked on its own inputs, at the
tolerance stated for the attention entry points."""
import numpy as np
import pytest
import torch

from oracle import layer_oracle
from paper_2502_05431_amd import binding as B
from paper_2502_05431_amd import workloads as W

import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _close(got, ref, name, what, layers=1):
    """The bf16 bounds of the attention outputs (rel-L2 5e-3, max-abs 2e-2) are stated for values
    of magnitude <= 1; the residual stream of a layer is larger (|y| up to ~5, bf16 spacing 2^-6
    there), so the absolute bound scales with the largest reference value.  After a stack of L
    layers, each of which rounds its hidden states to bf16 independently of the others, the bounds
    grow by sqrt(L) (independent rounding errors add in quadrature).  fp32: see the tests."""
    if name == "f32":
        return H.check_close(got, ref, name, what)
    grow = float(layers) ** 0.5
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape and np.isfinite(got).all(), what
    rel = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300)
    err = np.abs(got - ref).max()
    assert rel <= H.BF16_REL_L2 * grow, "%s: rel-L2 %.3e" % (what, rel)
    assert err <= H.BF16_MAX_ABS * grow * max(1.0, np.abs(ref).max()), "%s: max-abs %.3e (largest value %.2f)" % (what, err, np.abs(ref).max())


def _make(hidden, inter, hq, hkv, d, dtype, seed):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    rn = lambda *s, scale=1.0: (torch.randn(s, generator=g, device=DEV, dtype=torch.float32) * scale).to(dtype).contiguous()
    qkvd = (hq + 2 * hkv) * d
    w = {"attn_norm": (1.0 + 0.1 * torch.randn(hidden, generator=g, device=DEV)).to(dtype),
         "w_qkv": rn(qkvd, hidden, scale=hidden ** -0.5), "w_o": rn(hidden, hq * d, scale=(hq * d) ** -0.5),
         "mlp_norm": (1.0 + 0.1 * torch.randn(hidden, generator=g, device=DEV)).to(dtype),
         "w_gate_up": rn(2 * inter, hidden, scale=hidden ** -0.5), "w_down": rn(hidden, inter, scale=inter ** -0.5)}
    return w, rn


def _oracle_weights(w, hq, hkv, d, inter):
    n = W.to_numpy_f32
    qkv, gu = n(w["w_qkv"]), n(w["w_gate_up"])
    return {"attn_norm": n(w["attn_norm"]), "wq": qkv[:hq * d], "wk": qkv[hq * d:(hq + hkv) * d], "wv": qkv[(hq + hkv) * d:],
            "wo": n(w["w_o"]), "mlp_norm": n(w["mlp_norm"]), "wg": gu[:inter], "wu": gu[inter:], "wd": n(w["w_down"])}


def _run_layer(shape, lw, x, kp, vp, lens, hkv, d, hidden, inter, taps=None):
    m = sum(lens)
    cu = [0]
    for l in lens:
        cu.append(cu[-1] + l)
    cu_dev = torch.tensor(cu, dtype=torch.int32, device=DEV)
    kc = torch.full((m, hkv, d), float("nan"), dtype=x.dtype, device=DEV)
    vc = torch.full_like(kc, float("nan"))
    y = torch.full_like(x, float("nan"))
    ws = H.poisoned_workspace(B.layer_workspace_bytes(shape, hidden, inter, m), DEV)
    B.layer_encode(shape, lw, x, kp, vp, cu, cu_dev, kc, vc, y, ws,
                   q_rot_tap=None if taps is None else taps[0], attn_tap=None if taps is None else taps[1])
    torch.cuda.synchronize()
    return y, kc, vc


def _layer_case(hidden, inter, hq, hkv, d, dtype, lp, lens, seed, sample_rows=None, tol=None):
    name = "f32" if dtype == torch.float32 else "bf16"
    w, rn = _make(hidden, inter, hq, hkv, d, dtype, seed)
    shape = B.make_shape(hq, hkv, d, dtype)
    lw = B.layer_weights(hidden, inter, 1e-5, 500000.0, w["attn_norm"], w["w_qkv"], w["w_o"], w["mlp_norm"], w["w_gate_up"], w["w_down"])
    ow = _oracle_weights(w, hq, hkv, d, inter)
    xp, xc = rn(lp, hidden) if lp else None, rn(sum(lens), hidden)
    n = W.to_numpy_f32
    kp = vp = None
    okp = ovp = None
    if lp:
        # the prefix is one more sequence at positions 0..: its layer pass yields this layer's prefix KV
        yp, kp, vp = _run_layer(shape, lw, xp, None, None, [lp], hkv, d, hidden, inter)
        op = layer_oracle.layer_encode(n(xp), ow, [lp], None, None, hq, hkv, d, 500000.0, 1e-5)
        _close(H.f64(yp), op["y"], name, "prefix rows y") if tol is None else None
        okp, ovp = op["k"].astype(np.float32), op["v"].astype(np.float32)
    m = sum(lens)
    taps = (torch.full((m, hq, d), float("nan"), dtype=dtype, device=DEV), torch.full((m, hq, d), float("nan"), dtype=dtype, device=DEV))
    y, kc, vc = _run_layer(shape, lw, xc, kp, vp, lens, hkv, d, hidden, inter, taps=taps)
    # The attention inside the layer, on the inputs the layer itself handed it (its rotated queries,
    # the keys and values it cached, its prefix KV), against the attention oracle at the tolerance of
    # the attention entry points: fp32 max-abs 1e-5; bf16 rel-L2 5e-3 and max-abs 2e-2.
    from oracle import ape_oracle
    rows = list(range(m)) if sample_rows is None else list(sample_rows)
    pairs = [(r, hh) for r in rows for hh in range(hq)]
    a_ref, _ = ape_oracle.encode(n(taps[0]), None if kp is None else n(kp), None if vp is None else n(vp), n(kc), n(vc), list(lens), pairs=pairs)
    a_got = H.f64(taps[1])[np.asarray(rows)].reshape(-1, d)
    H.check_close(a_got, a_ref, name, "attention inside the layer")
    ref = layer_oracle.layer_encode(n(xc), ow, lens, okp, ovp, hq, hkv, d, 500000.0, 1e-5, rows=sample_rows)
    got = H.f64(y) if sample_rows is None else H.f64(y)[np.asarray(sample_rows)]
    if tol is None:
        _close(got, ref["y"], name, "layer y")
    else:
        err = np.abs(got - ref["y"]).max()
        assert err <= tol, "layer y: max-abs %.3e > %.1e" % (err, tol)
    if tol is None:
        _close(H.f64(kc).reshape(-1, d), ref["k"].reshape(-1, d), name, "cached k")
        _close(H.f64(vc).reshape(-1, d), ref["v"].reshape(-1, d), name, "cached v")
    else:
        assert np.abs(H.f64(kc) - ref["k"]).max() <= tol and np.abs(H.f64(vc) - ref["v"]).max() <= tol
    assert torch.isfinite(y.float()).all()
    return np.abs(got - ref["y"]).max()


# fp32: the path is a chain of six fp32 stages (two norms, four GEMMs with up to 512-term dot
# products, attention), each within a few 1e-6 of the fp64 result on O(1) values: 4e-5 on y.
def test_layer_fp32_small_generic_attention():
    _layer_case(64, 96, 4, 2, 64, torch.float32, 8, [32, 17, 40, 5], 1, tol=4e-5)
    _layer_case(64, 96, 4, 2, 64, torch.float32, 0, [33, 0, 1, 64], 2, tol=4e-5)


def test_layer_bf16_matrix_core_attention():
    _layer_case(256, 512, 4, 2, 128, torch.bfloat16, 7, [100, 1, 65, 300, 31], 3)
    _layer_case(256, 512, 8, 8, 128, torch.bfloat16, 0, [257, 255], 4)


def test_layer_llama_shape_sampled_rows():
    """Llama-3-8B layer shape (hidden 4096, MLP 14336, 32 q / 8 kv heads): sampled rows of two contexts."""
    lens = [300, 257]
    rows = [0, 1, 31, 32, 150, 299, 300, 301, 400, 556]
    _layer_case(4096, 14336, 32, 8, 128, torch.bfloat16, 32, lens, 5, sample_rows=rows)


def test_layer_more_rows_than_one_mlp_slab():
    """17 000 rows: the MLP runs in two slabs of rows; cheap widths so that the oracle stays quick."""
    lens = [9000, 8000]
    rows = [0, 8999, 9000, 16383, 16384, 16385, 16999]
    _layer_case(64, 64, 2, 1, 128, torch.bfloat16, 0, lens, 6, sample_rows=rows)


def _stack_case(n_layers, hidden, inter, hq, hkv, d, dtype, lp, lens, seed):
    """ape_layers_encode against the layer oracle applied n_layers times (each layer with its own
    weights, prefix KV and cache)."""
    name = "f32" if dtype == torch.float32 else "bf16"
    n = W.to_numpy_f32
    shape = B.make_shape(hq, hkv, d, dtype)
    ws_all, lws, ows = [], [], []
    rn = None
    for l in range(n_layers):
        w, rn = _make(hidden, inter, hq, hkv, d, dtype, seed + 10 * l)
        ws_all.append(w)
        lws.append(B.layer_weights(hidden, inter, 1e-5, 500000.0, w["attn_norm"], w["w_qkv"], w["w_o"], w["mlp_norm"], w["w_gate_up"], w["w_down"]))
        ows.append(_oracle_weights(w, hq, hkv, d, inter))
    m = sum(lens)
    xp, xc = (rn(lp, hidden) if lp else None), rn(m, hidden)
    cu = [0]
    for l in lens:
        cu.append(cu[-1] + l)
    cu_dev = torch.tensor(cu, dtype=torch.int32, device=DEV)
    new_cache = lambda rows: [torch.full((rows, hkv, d), float("nan"), dtype=dtype, device=DEV) for _ in range(n_layers)]
    kps = vps = None
    if lp:
        # the prefix goes through the same stack first: that yields every layer's prefix KV
        kps, vps = new_cache(lp), new_cache(lp)
        yp = torch.full_like(xp, float("nan"))
        wsb = H.poisoned_workspace(B.layer_workspace_bytes(shape, hidden, inter, lp, n_layers=n_layers), DEV)
        B.layers_encode(shape, lws, xp, None, None, [0, lp], torch.tensor([0, lp], dtype=torch.int32, device=DEV), kps, vps, yp, wsb)
    kcs, vcs = new_cache(m), new_cache(m)
    y = torch.full_like(xc, float("nan"))
    wsb = H.poisoned_workspace(B.layer_workspace_bytes(shape, hidden, inter, m, n_layers=n_layers), DEV)
    B.layers_encode(shape, lws, xc, kps, vps, cu, cu_dev, kcs, vcs, y, wsb)
    torch.cuda.synchronize()
    # oracle: the same stack in fp64, prefix first
    hp, hc = (None if not lp else n(xp).astype(np.float64)), n(xc).astype(np.float64)
    for l in range(n_layers):
        okp = ovp = None
        if lp:
            op = layer_oracle.layer_encode(hp, ows[l], [lp], None, None, hq, hkv, d, 500000.0, 1e-5)
            okp, ovp, hp = op["k"].astype(np.float32), op["v"].astype(np.float32), op["y"]
        oc = layer_oracle.layer_encode(hc, ows[l], lens, okp, ovp, hq, hkv, d, 500000.0, 1e-5)
        hc = oc["y"]
        # every layer's cache, not only the last hidden states
        if name == "bf16":
            _close(H.f64(kcs[l]).reshape(-1, d), oc["k"].reshape(-1, d), name, "layer %d cached k" % l, layers=l + 1)
            _close(H.f64(vcs[l]).reshape(-1, d), oc["v"].reshape(-1, d), name, "layer %d cached v" % l, layers=l + 1)
        else:
            assert np.abs(H.f64(kcs[l]) - oc["k"]).max() <= 4e-5 * (l + 1) and np.abs(H.f64(vcs[l]) - oc["v"]).max() <= 4e-5 * (l + 1)
    if name == "bf16":
        _close(H.f64(y), hc, name, "stack of %d layers y" % n_layers, layers=n_layers)
    else:
        assert np.abs(H.f64(y) - hc).max() <= 4e-5 * n_layers
    assert torch.isfinite(y.float()).all()


def test_stack_of_layers_fp32_and_bf16():
    """Three layers (odd: the hidden states end in y after passing through the spare buffer twice) and
    two (even), fp32 on the portable attention and bf16 on the matrix-core attention."""
    _stack_case(3, 64, 96, 4, 2, 64, torch.float32, 8, [32, 17, 40, 5], 11)
    _stack_case(2, 64, 96, 4, 2, 64, torch.float32, 0, [33, 1, 64], 12)
    _stack_case(3, 256, 512, 4, 2, 128, torch.bfloat16, 7, [100, 1, 65, 300, 31], 13)
    _stack_case(2, 256, 512, 8, 8, 128, torch.bfloat16, 0, [257, 255], 14)
