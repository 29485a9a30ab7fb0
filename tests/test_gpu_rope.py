"""GPU parity of the rotary embedding + KV-cache write (positions re-used across contexts,
Section 1) against the fp64 oracle, through the C ABI; and the whole chain raw -> rotate ->
encode -> query attention in fp32 against the oracle's chain."""
import numpy as np
import pytest
import torch

from oracle import ape_oracle
from paper_2502_05431_amd import binding as B
from paper_2502_05431_amd import workloads as W

import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _raw(n, heads, d, dtype, seed, scale=1.0):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    return (torch.randn((n, heads, d), generator=g, device=DEV, dtype=torch.float32) * scale).to(dtype).contiguous()


def _run(hq, hkv, d, dtype, lens, offset, base, packed_cache=True, in_place=False, with_q=True, with_v=True, seed=0):
    m = sum(lens)
    shape = B.make_shape(hq, hkv, d, dtype)
    q, k, v = _raw(m, hq, d, dtype, seed + 1), _raw(m, hkv, d, dtype, seed + 2), _raw(m, hkv, d, dtype, seed + 3)
    cu = [0]
    for l in lens:
        cu.append(cu[-1] + l)
    cu_dev = torch.tensor(cu, dtype=torch.int32, device=DEV)
    if packed_cache:
        kbuf = torch.full_like(k, float("nan")); vbuf = torch.full_like(v, float("nan"))
        kc = [kbuf[cu[i]:cu[i + 1]] for i in range(len(lens))]
        vc = [vbuf[cu[i]:cu[i + 1]] for i in range(len(lens))]
    else:
        kc = [torch.full((max(l, 1), hkv, d), float("nan"), dtype=dtype, device=DEV) for l in lens]
        vc = [torch.full((max(l, 1), hkv, d), float("nan"), dtype=dtype, device=DEV) for l in lens]
    kt = torch.tensor([t.data_ptr() for t in kc], dtype=torch.int64, device=DEV)
    vt = torch.tensor([t.data_ptr() for t in vc], dtype=torch.int64, device=DEV)
    q_in = q.clone()
    q_out = q_in if in_place else torch.full_like(q, float("nan"))
    B.rope_write_cache(shape, q_in if with_q else None, k, v if with_v else None, cu, cu_dev, offset, base,
                       q_out if with_q else None, kt, vt if with_v else None)
    torch.cuda.synchronize()
    k_got = torch.cat([kc[i][:lens[i]] for i in range(len(lens))]) if m else k
    v_got = torch.cat([vc[i][:lens[i]] for i in range(len(lens))]) if m else v
    return q, k, v, q_out, k_got, v_got


def _check(hq, hkv, d, dtype, lens, offset, base, **kw):
    q, k, v, q_got, k_got, v_got = _run(hq, hkv, d, dtype, lens, offset, base, **kw)
    name = "f32" if dtype == torch.float32 else "bf16"
    if kw.get("with_q", True):
        ref = ape_oracle.rope(W.to_numpy_f32(q), lens, offset, base)
        H.check_close(H.f64(q_got).reshape(-1, d), ref.reshape(-1, d), name, "rotated q %s" % (lens,))
    ref = ape_oracle.rope(W.to_numpy_f32(k), lens, offset, base)
    H.check_close(H.f64(k_got).reshape(-1, d), ref.reshape(-1, d), name, "rotated k %s" % (lens,))
    if kw.get("with_v", True):
        assert torch.equal(v_got, v)                      # a copy: bit exact


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_rope_small_shapes(dtype):
    _check(4, 2, 64, dtype, [32, 32, 32, 32], 8, 500000.0)
    _check(4, 2, 64, dtype, [33, 0, 1, 64, 7], 0, 10000.0, packed_cache=False)
    _check(32, 8, 128, dtype, [100, 1, 65, 300, 31], 32, 500000.0, in_place=True)
    _check(8, 8, 256, dtype, [17, 40], 5, 500000.0, with_v=False)
    _check(6, 2, 40, dtype, [9, 3], 2, 10000.0)           # head_dim/2 not a multiple of the vector width (bf16)
    _check(2, 1, 8, dtype, [5], 1, 100.0, with_q=False)


def test_rope_far_positions_keep_fp32_accuracy():
    """At position 100 000 an fp32 angle would be off by 1e-2 rad; the kernel reduces in fp64."""
    _check(4, 2, 64, torch.float32, [40, 40], 100000, 500000.0)
    _check(4, 2, 64, torch.float32, [3], 2000000, 10000.0)


def test_rope_llama_shape_2048_token_contexts():
    _check(32, 8, 128, torch.bfloat16, [2048, 2048, 1000], 32, 500000.0)


def test_chain_rotate_encode_attend_fp32():
    """raw Q/K/V -> rotate with re-used positions + cache write -> encode -> query prefill, against
    the oracle's chain (its fp64 rotation, rounded to fp32, feeding its attention routines)."""
    spec = W.CONFIGS[1]
    hq, hkv, d, lp = spec.n_q_heads, spec.n_kv_heads, spec.head_dim, spec.prefix_len
    lens = [32, 17, 40, 5]
    base, T, S = 500000.0, 0.8, 0.9
    shape = B.make_shape(hq, hkv, d, torch.float32)
    m, lq = sum(lens), spec.q_len
    raw = {n: _raw(rows, heads, d, torch.float32, 100 + i) for i, (n, rows, heads) in enumerate(
        [("qp", lp, hq), ("kp", lp, hkv), ("vp", lp, hkv), ("qc", m, hq), ("kc", m, hkv), ("vc", m, hkv),
         ("qs", lq, hq), ("ks", lq, hkv), ("vs", lq, hkv)])}

    def rotate(q, k, v, seg_lens, offset):
        cu = [0]
        for l in seg_lens:
            cu.append(cu[-1] + l)
        cu_dev = torch.tensor(cu, dtype=torch.int32, device=DEV)
        kb, vb, qo = torch.empty_like(k), torch.empty_like(v), torch.empty_like(q)
        kt = torch.tensor([kb[cu[i]:].data_ptr() for i in range(len(seg_lens))], dtype=torch.int64, device=DEV)
        vt = torch.tensor([vb[cu[i]:].data_ptr() for i in range(len(seg_lens))], dtype=torch.int64, device=DEV)
        B.rope_write_cache(shape, q, k, v, cu, cu_dev, offset, base, qo, kt, vt)
        return qo, kb, vb, cu, cu_dev
    qp, kp, vp, _, _ = rotate(raw["qp"], raw["kp"], raw["vp"], [lp], 0)
    qc, kc, vc, cu, cu_dev = rotate(raw["qc"], raw["kc"], raw["vc"], lens, lp)
    qs, ks, vs, _, _ = rotate(raw["qs"], raw["ks"], raw["vs"], [lq], lp + max(lens))

    o_ctx = torch.empty_like(qc)
    B.encode_chunks(shape, None, kp, vp, qc, kc, vc, cu, cu_dev, None, o_ctx)
    req = B.Request(kp, vp, [kc[cu[i]:cu[i + 1]] for i in range(len(lens))], [vc[cu[i]:cu[i + 1]] for i in range(len(lens))],
                    ks, vs, lq, T, S)
    out = torch.empty_like(qs)
    ws = H.poisoned_workspace(B.workspace_bytes(B.APE_OP_PREFILL, shape, 1, lq), DEV)
    B.attention_prefill(shape, req, qs, out, None, ws)
    torch.cuda.synchronize()

    n = W.to_numpy_f32
    f32 = lambda a: a.astype(np.float32)
    o_qp = f32(ape_oracle.rope(n(raw["qp"]), [lp], 0, base)); o_kp = f32(ape_oracle.rope(n(raw["kp"]), [lp], 0, base))
    o_qc = f32(ape_oracle.rope(n(raw["qc"]), lens, lp, base)); o_kc = f32(ape_oracle.rope(n(raw["kc"]), lens, lp, base))
    o_qs = f32(ape_oracle.rope(n(raw["qs"]), [lq], lp + max(lens), base)); o_ks = f32(ape_oracle.rope(n(raw["ks"]), [lq], lp + max(lens), base))
    ref_enc, _ = ape_oracle.encode(o_qc, o_kp, n(raw["vp"]), o_kc, n(raw["vc"]), lens)
    ref_out, _, _ = ape_oracle.attention(o_qs, o_kp, n(raw["vp"]), o_kc, n(raw["vc"]), lens, o_ks, n(raw["vs"]), T, S)
    H.check_close(H.f64(o_ctx).reshape(-1, d), ref_enc, "f32", "chain encode")
    H.check_close(H.f64(out).reshape(-1, d), ref_out, "f32", "chain prefill")
    assert o_qp.shape == tuple(qp.shape)
