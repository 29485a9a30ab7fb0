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


def test_calls_on_two_streams_with_their_own_workspaces_do_not_disturb_each_other():
    """The library keeps no state between calls: two requests served at the same time on two streams
    (default priority), each with its own workspace and outputs, give bit for bit what they give one
    after the other."""
    specs = [W.CONFIGS[2].replace(chunk_lens=(2048,) * 12, q_len=64, decode_steps=8),
             W.CONFIGS[2].replace(chunk_lens=(300, 4000, 77, 1024), q_len=40, decode_steps=8, prefix_len=9)]
    jobs = []
    for i, spec in enumerate(specs):
        r = W.make_request(spec, DEV, request=i)
        shape = B.make_shape(spec.n_q_heads, spec.n_kv_heads, spec.head_dim, spec.torch_dtype)
        req = H.make_binding_request(r, spec.q_len)
        q = r.q_self[:spec.q_len].contiguous()
        qd = [r.q_self[spec.q_len + s:spec.q_len + s + 1].contiguous() for s in range(spec.decode_steps)]
        ws = torch.empty(max(B.workspace_bytes(B.APE_OP_PREFILL, shape, 1, spec.q_len),
                             B.workspace_bytes(B.APE_OP_DECODE, shape, 1, 1)) // 4, dtype=torch.float32, device=DEV)
        jobs.append(dict(spec=spec, r=r, shape=shape, req=req, q=q, qd=qd, ws=ws,
                         out=torch.zeros_like(q), outd=[torch.zeros_like(qd[0]) for _ in qd]))

    def run(job):
        sp = job["spec"]
        B.attention_prefill(job["shape"], job["req"], job["q"], job["out"], None, job["ws"], self_len=sp.q_len)
        for s in range(sp.decode_steps):
            B.attention_decode(job["shape"], [job["req"]], job["qd"][s], job["outd"][s], None, job["ws"], self_lens=[sp.q_len + s + 1])

    for job in jobs:                                     # one after the other, on the current stream
        run(job)
    torch.cuda.synchronize()
    serial = [(job["out"].clone(), [o.clone() for o in job["outd"]]) for job in jobs]
    h0 = H.HostArrays(jobs[0]["r"])
    ref, _, _ = H.oracle_prefill(h0, specs[0].q_len, specs[0].q_len, jobs[0]["r"].temperature, jobs[0]["r"].scale)
    H.check_close(H.f64(serial[0][0]).reshape(-1, specs[0].head_dim), ref, "bf16", "serial prefill")

    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for rounds in range(3):
        for job in jobs:
            job["out"].fill_(float("nan"))
            job["ws"].fill_(float("nan"))
            for o in job["outd"]:
                o.fill_(float("nan"))
        torch.cuda.synchronize()
        for job, st in zip(jobs, streams):               # both queues filled before either is waited for
            with torch.cuda.stream(st):
                run(job)
        torch.cuda.synchronize()
        for job, (sp_out, sp_outd) in zip(jobs, serial):
            assert torch.equal(job["out"], sp_out), "prefill differs when run next to another call"
            for got, want in zip(job["outd"], sp_outd):
                assert torch.equal(got, want), "decode differs when run next to another call"
