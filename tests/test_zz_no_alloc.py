"""GPU test of ``ape_attention_decode_static`` (the decode entry point that allocates nothing:
its partial results live in a fixed buffer inside the library): through the C ABI, against
``ape_attention_decode`` on the same inputs, on two calls in a row -- the second with a smaller
input, so that it runs over what the first call left in the shared buffer -- and against the
fp64 oracle."""
import numpy as np
import pytest
import torch

from paper_2502_05431_amd import binding as B
from paper_2502_05431_amd import workloads as W

import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _decode_both(spec, rs, self_lens):
    """One decode step through both entry points; returns (static out, static lse, plain out, plain lse)."""
    shape = B.make_shape(spec.n_q_heads, spec.n_kv_heads, spec.head_dim, spec.torch_dtype)
    reqs = [H.make_binding_request(r, sl) for r, sl in zip(rs, self_lens)]
    q = torch.stack([r.q_self[sl - 1] for r, sl in zip(rs, self_lens)]).contiguous()
    out_s = torch.full_like(q, float("nan"))
    lse_s = torch.full((len(rs), spec.n_q_heads), float("nan"), dtype=torch.float32, device=DEV)
    B.attention_decode_static(shape, reqs, q, out_s, lse_s, self_lens=list(self_lens))
    torch.cuda.synchronize()
    out_p, lse_p = H.run_decode(spec, rs, self_lens, reqs=reqs)
    return out_s, lse_s, out_p, lse_p


def _check(spec, rs, self_lens, what):
    out_s, lse_s, out_p, lse_p = _decode_both(spec, rs, self_lens)
    # same kernels, same split plan, same order of operations: the two entry points agree bit for bit
    assert torch.equal(out_s, out_p), what + ": static and workspace entry points differ"
    assert torch.equal(lse_s, lse_p), what + ": LogSumExp differs"
    for i, (r, sl) in enumerate(zip(rs, self_lens)):
        h = H.HostArrays(r)
        ref, ref_lse, _ = H.oracle_prefill(h, 1, sl, r.temperature, r.scale)
        H.check_close(H.f64(out_s[i]).reshape(-1, spec.head_dim), ref, spec.dtype, "%s request %d" % (what, i))
        assert np.abs(H.f64(lse_s[i]).reshape(-1) - ref_lse).max() <= H.lse_tol(spec.dtype), what + " lse"


def test_two_calls_in_a_row_second_smaller():
    # first call: 6 requests over 9 ragged contexts each (several splits per request); second call:
    # 2 requests over short contexts (fewer splits, fewer units) -- it must not pick up anything
    # the first call left in the shared buffer
    big = W.CONFIGS[5].replace(chunk_lens=(1024, 700, 1024, 333, 1024, 1024, 64, 1024, 900), decode_steps=3)
    rs = [W.make_request(big, DEV, request=i) for i in range(6)]
    _check(big, rs, [1, 2, 3, 1, 2, 3], "first call")
    small = W.CONFIGS[5].replace(chunk_lens=(300, 40), decode_steps=2)
    rs2 = [W.make_request(small, DEV, request=i) for i in range(2)]
    _check(small, rs2, [2, 1], "second, smaller call")
    # and the portable kernels (fp32, other head_dim) share the same buffer
    tiny = W.CONFIGS[1]
    r1 = W.make_request(tiny, DEV)
    _check(tiny, [r1], [tiny.q_len + 1], "fp32 call")


def test_too_large_for_the_static_buffer_is_refused():
    # 512 requests of the Llama shape need 512 * 32 * (splits + 1) * 516 B > 8 MiB: refused on the
    # host, nothing launched, outputs untouched
    spec = W.CONFIGS[5].replace(chunk_lens=(64,), decode_steps=1)
    r = W.make_request(spec, DEV)
    n = 512
    shape = B.make_shape(spec.n_q_heads, spec.n_kv_heads, spec.head_dim, spec.torch_dtype)
    reqs = [H.make_binding_request(r, 1)] * n
    q = r.q_self[:1].expand(n, -1, -1).contiguous()
    out = torch.full_like(q, 7.0)
    with pytest.raises(B.ApeError) as e:
        B.attention_decode_static(shape, reqs, q, out, None, self_lens=[1] * n)
    assert e.value.status == B.APE_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
