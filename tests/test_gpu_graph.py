"""The entry points allocate nothing, copy nothing and never synchronise, so a launch-bound loop
of them can be recorded into a HIP graph.  A decode loop (and a prefill) is captured, replayed
several times with other work and synchronisations in between, and every replay is compared with
the eager result and with the oracle."""
import numpy as np
import pytest
import torch

from paper_2502_05431_amd import binding as B
from paper_2502_05431_amd import workloads as W

import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_decode_steps_and_prefill_in_a_graph():
    spec = W.CONFIGS[2].replace(chunk_lens=(512,) * 6, q_len=32, decode_steps=6)
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    shape = B.make_shape(spec.n_q_heads, spec.n_kv_heads, spec.head_dim, spec.torch_dtype)
    req = H.make_binding_request(r, spec.q_len)
    q = r.q_self[:spec.q_len].contiguous()
    out_p = torch.zeros_like(q)
    steps = spec.decode_steps
    qd = [r.q_self[spec.q_len + i:spec.q_len + i + 1].contiguous() for i in range(steps)]
    outd = [torch.zeros_like(qd[0]) for _ in range(steps)]
    ws = torch.empty(max(B.workspace_bytes(B.APE_OP_PREFILL, shape, 1, spec.q_len),
                         B.workspace_bytes(B.APE_OP_DECODE, shape, 1, 1)) // 4, dtype=torch.float32, device=DEV)

    def work():
        B.attention_prefill(shape, req, q, out_p, None, ws, self_len=spec.q_len)
        for i in range(steps):
            B.attention_decode(shape, [req], qd[i], outd[i], None, ws, self_lens=[spec.q_len + i + 1])

    work()                                               # eager, also warms up every kernel
    torch.cuda.synchronize()
    eager_p = out_p.clone()
    eager_d = [o.clone() for o in outd]

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            work()
    torch.cuda.synchronize()

    scratch = torch.empty(1 << 20, device=DEV)
    for replay in range(4):
        out_p.fill_(float("nan"))
        for o in outd:
            o.fill_(float("nan"))
        ws.fill_(float("nan"))                           # partial results of the last replay must not be needed
        scratch.normal_()                                # the program's own eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_p, eager_p), "prefill differs on replay %d" % replay
        for i in range(steps):
            assert torch.equal(outd[i], eager_d[i]), "decode step %d differs on replay %d" % (i, replay)

    ref, _, _ = H.oracle_prefill(h, spec.q_len, spec.q_len, r.temperature, r.scale)
    H.check_close(H.f64(out_p).reshape(-1, spec.head_dim), ref, "bf16", "graph prefill")
    refd, _, _ = H.oracle_prefill(h, 1, spec.q_len + steps, r.temperature, r.scale)
    H.check_close(H.f64(outd[-1]).reshape(-1, spec.head_dim), refd, "bf16", "graph decode")
