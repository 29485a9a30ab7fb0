"""GPU parity of ape_layer_encode (one transformer layer around the block-diagonal encode
attention) against the fp64 layer oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import layer_oracle
from paper_2502_05431_amd import binding as B
from paper_2502_05431_amd import workloads as W

import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _close(got, ref, name, what):
    """The bf16 bounds of the attention outputs (rel-L2 5e-3, max-abs 2e-2) are stated for values
    of magnitude <= 1; the residual stream of a layer is larger (|y| up to ~5, bf16 spacing 2^-6
    there), so the absolute bound scales with the largest reference value.  fp32: see the test."""
    if name == "f32":
        return H.check_close(got, ref, name, what)
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape and np.isfinite(got).all(), what
    rel = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300)
    err = np.abs(got - ref).max()
    assert rel <= H.BF16_REL_L2, "%s: rel-L2 %.3e" % (what, rel)
    assert err <= H.BF16_MAX_ABS * max(1.0, np.abs(ref).max()), "%s: max-abs %.3e (largest value %.2f)" % (what, err, np.abs(ref).max())


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


def _run_layer(shape, lw, x, kp, vp, lens, hkv, d, hidden, inter):
    m = sum(lens)
    cu = [0]
    for l in lens:
        cu.append(cu[-1] + l)
    cu_dev = torch.tensor(cu, dtype=torch.int32, device=DEV)
    kc = torch.full((m, hkv, d), float("nan"), dtype=x.dtype, device=DEV)
    vc = torch.full_like(kc, float("nan"))
    y = torch.full_like(x, float("nan"))
    ws = H.poisoned_workspace(B.layer_workspace_bytes(shape, hidden, inter, m), DEV)
    B.layer_encode(shape, lw, x, kp, vp, cu, cu_dev, kc, vc, y, ws)
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
    y, kc, vc = _run_layer(shape, lw, xc, kp, vp, lens, hkv, d, hidden, inter)
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
