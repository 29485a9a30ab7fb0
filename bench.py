"""Benchmark of the APE attention hot path on one MI355X.

A "step" is one pass of the whole path over the 128K-context workload (benchmark config 3,
the configuration the headline metric is quoted on): ``ape_encode_chunks`` over 64 chunks x 2048
tokens with the shared 32-token prefix, ``ape_attention_prefill`` of a 256-token query over the
131K cached KV, then ``--decode-steps`` single-token ``ape_attention_decode`` steps over the same
cache.  All inputs are synthetic, seeded and resident in HBM before the timed region.

Printed: ONE JSON line.  ``value`` = algorithmic FLOPs of the whole step / step time.  Per-phase
figures (prefill TFLOP/s = the headline, decode GB/s, and the batched-decode workload of config
5 timed in a region of its own) are in ``phases``.  ``roofline`` describes the kernel that
dominates the step's time; ``cpu_baseline`` is the fp64 oracle timed on the host cores on a
bounded sample of the same workload.

FLOP convention: 4*head_dim per unmasked (query, key) pair per query head.  Byte convention for
decode: every cached K and V element once + Q and O.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0          # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0              # MI355X HBM3E

# HBM traffic per launch.  Hardware counters cannot be read from inside this process: the figures
# come from two rocprofv3 --pmc runs of THIS script (FETCH_SIZE, then WRITE_SIZE, KiB per dispatch),
# each scaled by the same counter's reading for the 1 GiB device copy of --calibrate-copy in the same
# run (FETCH_SIZE x 2.0, WRITE_SIZE x 1.0).  TRAFFIC_SOURCE names the summary that holds the commands
# and the raw readings; the line printed below carries it next to the number.
MEASURED_TRAFFIC_BYTES = {"flash_encode_kernel": (786711 * 2 + 1048580) * 1024,     # 2.685 GB
                          "flash_prefill_kernel": (272240 * 2 + 45082) * 1024,     # 0.604 GB
                          "flash_prefill_kernel (decode)": (262914 * 2 + 536) * 1024}    # 0.539 GB
TRAFFIC_SOURCE = "profiles/bench_cfg3_hbm_traffic_pmc.md"
WARM_MS = 150.0                    # GPU time of untimed load in front of every timed region


def pair_counts(spec):
    """Unmasked (query, key) pairs per query head for the phases of one step."""
    lp, m, lq = spec.prefix_len, spec.total_ctx_len, spec.q_len
    enc = sum(li * (li + 1) // 2 + li * lp for li in spec.chunk_lens)
    pre = lq * (lp + m) + lq * (lq + 1) // 2
    return enc, pre


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=25,
                    help="untimed steps.  The chip raises its clocks over the first ~100 ms of load (a 10-step run of "
                         "the prefill measures 0.67 ms per call, a 1000-step run 0.55 ms), so whatever this says the "
                         "untimed steps go on until 150 ms of GPU time have passed (the count used is printed as warm_steps)")
    ap.add_argument("--decode-steps", type=int, default=8, help="decode steps per step over the 128K cache")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-cfg5", action="store_true", help="skip the batched-decode (config 5) region")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target wall time of the oracle sample")
    ap.add_argument("--sequential-comparator", action="store_true",
                    help="also time the causal attention that the parallel encoding replaces: the same 131K context "
                         "tokens encoded as ONE chunk (Eq.2), for an attention-only prefill ratio on this GPU")
    ap.add_argument("--tree-variants", action="store_true",
                    help="also time the query prefill and one decode step of the same 128K cache through the tree "
                         "entry point: one pooled node, a scaling factor per context, and a two-level tree")
    ap.add_argument("--all-configs", action="store_true", help="(default now; kept so that old command lines still parse)")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip encode, query prefill and one decode step of the other bf16 configurations "
                         "(2: RAG-shaped 20 x 512; 4: many-shot 512 x 256), each call looped on its own")
    ap.add_argument("--layers", type=int, default=0,
                    help="also time a stack of this many Llama-3-8B-shaped layers (ape_layers_encode) over the same contexts")
    ap.add_argument("--layer", action="store_true",
                    help="also time one whole Llama-3-8B-shaped layer (hidden 4096, MLP 14336, random weights) of the "
                         "context pre-caching pass over the same 64 x 2048 contexts")
    ap.add_argument("--prefill-batch", type=int, default=0,
                    help="also time the batched query prefill: this many requests, each over its own 128K cache")
    ap.add_argument("--rope-write", action="store_true",
                    help="also time the rotary embedding + KV-cache write in front of the encode (raw Q/K/V of the "
                         "same 64 x 2048 contexts), a bandwidth-bound kernel")
    ap.add_argument("--gemm-reference", action="store_true",
                    help="also time torch's bf16 GEMM (the vendor library) on zero and on random operands: context "
                         "for the MFMA roofline, which on this chip depends on the operand data (power limit)")
    ap.add_argument("--sdpa-reference", action="store_true",
                    help="also time torch's scaled_dot_product_attention (the vendor's fused attention) on the two "
                         "contractions of config 3: causal attention over 64 sequences of 2048 tokens (the encode without "
                         "its shared prefix) and 256 query rows over 131K keys (the context group of the prefill)")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the probes of the box's own ceilings (MFMA rate on zero and on random operands, the same "
                         "with a softmax's vector work beside it, a read-only HBM stream)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one device-to-device copy of 1 GiB (a kernel of known HBM traffic, to scale "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE readings in a --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (no collectives, no sharding "
              "in this path)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2502_05431_amd import binding as B
    from paper_2502_05431_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    B.load()

    def timed(fn, iters, warm_ms=WARM_MS):
        """Average ms per call of fn over `iters` calls, after calling it untimed for at least warm_ms of
        GPU time (the chip raises its clocks over the first ~100 ms of load; a region that follows host-side
        set-up starts from low clocks again)."""
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn()
        torch.cuda.synchronize()
        spent = 0.0
        while spent < warm_ms:
            e0.record()
            for _ in range(4):
                fn()
            e1.record()
            torch.cuda.synchronize()
            spent += e0.elapsed_time(e1)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    spec = W.CONFIGS[3].replace(decode_steps=args.decode_steps)
    r = W.make_request(spec, dev)
    hq, hkv, d = spec.n_q_heads, spec.n_kv_heads, spec.head_dim
    shape = B.make_shape(hq, hkv, d, spec.torch_dtype)
    cu = [0]
    for li in r.chunk_lens:
        cu.append(cu[-1] + li)
    cu_dev = torch.tensor(cu, dtype=torch.int32, device=dev)
    ks, vs = r.chunk_views()
    req = B.Request(r.k_prefix, r.v_prefix, ks, vs, r.k_self, r.v_self, spec.q_len, r.temperature, r.scale)
    o_ctx = torch.empty_like(r.q_ctx)
    q = r.q_self[:spec.q_len].contiguous()
    out = torch.empty_like(q)
    ws = torch.empty(max(B.workspace_bytes(B.APE_OP_PREFILL, shape, 1, spec.q_len, spec.total_ctx_len),
                         B.workspace_bytes(B.APE_OP_DECODE, shape, 1, 1, spec.total_ctx_len)) // 4, dtype=torch.float32, device=dev)
    qd = [r.q_self[spec.q_len + i:spec.q_len + i + 1].contiguous() for i in range(args.decode_steps)]
    outd = torch.empty_like(qd[0]) if qd else None
    # decode calls marshalled once (argument marshalling only; the request's self_len grows by one per token)
    dec_calls = []
    for i in range(args.decode_steps):
        fn, arr = B.decode_call(shape, [req], qd[i], outd, None, ws)
        arr[0].self_len = spec.q_len + i + 1
        dec_calls.append((fn, arr))

    def step(ev=None):
        if ev: ev[0].record()
        B.encode_chunks(shape, None, r.k_prefix, r.v_prefix, r.q_ctx, r.k_ctx, r.v_ctx, cu, cu_dev, None, o_ctx)
        if ev: ev[1].record()
        B.attention_prefill(shape, req, q, out, None, ws)
        if ev: ev[2].record()
        for fn, _ in dec_calls:
            fn()
        if ev: ev[3].record()

    # untimed steps: the requested count, then on until WARM_MS of GPU time have been spent under load
    warm_ev = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
    warm_steps, warm_spent = 0, 0.0
    while warm_steps < args.warmup or warm_spent < WARM_MS:
        warm_ev[0].record()
        step()
        warm_ev[1].record()
        torch.cuda.synchronize()
        warm_spent += warm_ev[0].elapsed_time(warm_ev[1])
        warm_steps += 1
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(events[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_step = (t1 - t0) * 1e3 / args.steps
    ph = np.array([[e[i].elapsed_time(e[i + 1]) for i in range(3)] for e in events])      # ms
    ms_enc, ms_pre, ms_dec = ph.mean(axis=0)

    enc_pairs, pre_pairs = pair_counts(spec)
    fl_enc, fl_pre = 4.0 * d * hq * enc_pairs, 4.0 * d * hq * pre_pairs
    kv_row_bytes = 2 * hkv * d * 2
    dec_tokens = [spec.prefix_len + spec.total_ctx_len + spec.q_len + i + 1 for i in range(args.decode_steps)]
    fl_dec = sum(4.0 * d * hq * t for t in dec_tokens)
    by_dec = sum(kv_row_bytes * t + 2 * hq * d * 2 for t in dec_tokens)
    value = (fl_enc + fl_pre + fl_dec) / (ms_step * 1e-3) / 1e12

    ms_med, ms_min = np.median(ph, axis=0), ph.min(axis=0)
    phases = {
        "encode": {"ms": float(ms_enc), "tflops": fl_enc / (ms_enc * 1e-3) / 1e12, "frac_mfma_peak": fl_enc / (ms_enc * 1e-3) / 1e12 / PEAK_BF16_TFLOPS},
        "prefill": {"ms": float(ms_pre), "tflops": fl_pre / (ms_pre * 1e-3) / 1e12, "frac_mfma_peak": fl_pre / (ms_pre * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                    "note": "flash kernel + merge kernel"},
    }
    for i, name in enumerate(("encode", "prefill")):
        phases[name]["ms_median"], phases[name]["ms_min"] = float(ms_med[i]), float(ms_min[i])
    # the same prefill call looped on its own (inside the step it follows the encode, under which the
    # chip runs at lower clocks)
    ms_pre_alone = timed(lambda: B.attention_prefill(shape, req, q, out, None, ws), 100)
    phases["prefill_looped_alone"] = {"ms": ms_pre_alone, "tflops": fl_pre / (ms_pre_alone * 1e-3) / 1e12,
                                      "frac_mfma_peak": fl_pre / (ms_pre_alone * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                                      "note": "the prefill call of the step, 100 calls back to back"}
    if args.decode_steps:
        phases["decode_128k_batch1"] = {"ms_per_token": float(ms_dec) / args.decode_steps,
                                        "gbs": by_dec / (ms_dec * 1e-3) / 1e9, "frac_hbm_peak": by_dec / (ms_dec * 1e-3) / 1e9 / PEAK_HBM_GBS,
                                        "ms_per_token_median": float(ms_med[2]) / args.decode_steps,
                                        "ms_per_token_min": float(ms_min[2]) / args.decode_steps,
                                        "note": "538 MB of KV per token, batch 1"}

    # the kernel that dominates the step
    if ms_enc >= ms_pre and ms_enc >= ms_dec:
        roof = {"kernel": "flash_encode_kernel", "bound": "mfma", "achieved": fl_enc / (ms_enc * 1e-3) / 1e12,
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s"}
    elif ms_pre >= ms_dec:
        roof = {"kernel": "flash_prefill_kernel", "bound": "mfma", "achieved": fl_pre / (ms_pre * 1e-3) / 1e12,
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s"}
    else:
        roof = {"kernel": "flash_prefill_kernel (decode)", "bound": "hbm", "achieved": by_dec / (ms_dec * 1e-3) / 1e9,
                "peak": PEAK_HBM_GBS, "unit": "GB/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = MEASURED_TRAFFIC_BYTES.get(roof["kernel"])
    roof["traffic_source"] = TRAFFIC_SOURCE
    roof["launch_ms"] = float({"flash_encode_kernel": ms_enc, "flash_prefill_kernel": ms_pre, "flash_prefill_kernel (decode)": ms_dec / max(1, args.decode_steps)}[roof["kernel"]])

    seq_cmp = None
    if args.sequential_comparator:
        m_tok = spec.total_ctx_len
        cu1 = [0, m_tok]
        cu1_dev = torch.tensor(cu1, dtype=torch.int32, device=dev)

        def seq_encode():
            B.encode_chunks(shape, None, r.k_prefix, r.v_prefix, r.q_ctx, r.k_ctx, r.v_ctx, cu1, cu1_dev, None, o_ctx)
        ms_seq = timed(seq_encode, 3, warm_ms=100.0)
        fl_seq = 4.0 * d * hq * (m_tok * (m_tok + 1) // 2 + m_tok * spec.prefix_len)
        seq_cmp = {"ms": ms_seq, "tflops": fl_seq / (ms_seq * 1e-3) / 1e12,
                   "attention_time_ratio_vs_parallel_encode": ms_seq / ms_enc,
                   "note": "one causal chunk of %d tokens vs %d chunks of %d encoded in parallel" % (m_tok, len(r.chunk_lens), r.chunk_lens[0])}

    tree_var = None
    if args.tree_variants:
        n_ch = len(r.chunk_lens)
        ws_t = torch.empty(max(B.tree_workspace_bytes(shape, spec.total_ctx_len, n_ch + 1, spec.q_len),
                               B.tree_workspace_bytes(shape, spec.total_ctx_len, n_ch + 1, 1)) // 4, dtype=torch.float32, device=dev)
        qd1 = r.q_self[spec.q_len - 1:spec.q_len].contiguous()
        od1 = torch.empty_like(qd1)
        tree_var = {}
        for name, nodes in (("pooled_one_node", W.tree_pooled(n_ch, r.scale)),
                            ("scaling_factor_per_context", W.tree_per_context(n_ch, r.scale)),
                            ("two_levels_groups_of_8", W.tree_grouped(n_ch, 8, 0.9, r.scale))):
            tree = B.make_tree(nodes, dev)
            res = {"nodes": len(nodes)}
            for kind, fn in (("prefill_ms", lambda: B.attention_tree(shape, req, tree, q, out, None, ws_t)),
                             ("decode_ms_per_token", lambda: B.attention_tree(shape, req, tree, qd1, od1, None, ws_t))):
                res[kind] = timed(fn, 50)
            res["prefill_tflops"] = fl_pre / (res["prefill_ms"] * 1e-3) / 1e12
            res["decode_gbs"] = (kv_row_bytes * (spec.prefix_len + spec.total_ctx_len + spec.q_len)) / (res["decode_ms_per_token"] * 1e-3) / 1e9
            tree_var[name] = res
        tree_var["note"] = ("same cache and query as the prefill phase (flat entry point: %.3f ms); the contexts of every "
                            "node are attended in splits of their own and the tree merge replaces the two-group merge" % ms_pre)
        del ws_t

    cfg_res = None
    if not args.no_other_configs:
        cfg_res = {}
        for cfg in (2, 4):
            sp = W.CONFIGS[cfg]
            rr = W.make_request(sp, dev)
            cu_c = [0]
            for li in rr.chunk_lens:
                cu_c.append(cu_c[-1] + li)
            cu_c_dev = torch.tensor(cu_c, dtype=torch.int32, device=dev)
            kc_, vc_ = rr.chunk_views()
            rq = B.Request(rr.k_prefix, rr.v_prefix, kc_, vc_, rr.k_self, rr.v_self, sp.q_len, rr.temperature, rr.scale)
            oc = torch.empty_like(rr.q_ctx)
            qq = rr.q_self[:sp.q_len].contiguous()
            oo = torch.empty_like(qq)
            q1 = rr.q_self[sp.q_len:sp.q_len + 1].contiguous()
            o1 = torch.empty_like(q1)
            wsc = torch.empty(max(B.workspace_bytes(B.APE_OP_PREFILL, shape, 1, sp.q_len, sp.total_ctx_len),
                                  B.workspace_bytes(B.APE_OP_DECODE, shape, 1, 1, sp.total_ctx_len)) // 4, dtype=torch.float32, device=dev)
            fn_dec, arr_dec = B.decode_call(shape, [rq], q1, o1, None, wsc)
            arr_dec[0].self_len = sp.q_len + 1
            ms_e = timed(lambda: B.encode_chunks(shape, None, rr.k_prefix, rr.v_prefix, rr.q_ctx, rr.k_ctx, rr.v_ctx, cu_c, cu_c_dev, None, oc), 50)
            ms_p = timed(lambda: B.attention_prefill(shape, rq, qq, oo, None, wsc), 100)
            ms_d = timed(fn_dec, 200)
            e_pairs, p_pairs = pair_counts(sp)
            kv_tok = sp.prefix_len + sp.total_ctx_len + sp.q_len + 1
            enc_bytes = 2.0 * (2 * rr.q_ctx.numel() + rr.k_ctx.numel() + rr.v_ctx.numel())       # Q read, O written, K and V read
            cfg_res[sp.name] = {
                "encode_ms": ms_e, "encode_tflops": 4.0 * d * hq * e_pairs / (ms_e * 1e-3) / 1e12,
                "encode_frac_mfma_peak": 4.0 * d * hq * e_pairs / (ms_e * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                "encode_hbm_gbs": enc_bytes / (ms_e * 1e-3) / 1e9, "encode_frac_hbm_peak": enc_bytes / (ms_e * 1e-3) / 1e9 / PEAK_HBM_GBS,
                "prefill_ms": ms_p, "prefill_tflops": 4.0 * d * hq * p_pairs / (ms_p * 1e-3) / 1e12,
                "prefill_frac_mfma_peak": 4.0 * d * hq * p_pairs / (ms_p * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                "decode_ms_per_token": ms_d, "decode_gbs": (kv_row_bytes * kv_tok) / (ms_d * 1e-3) / 1e9,
                "decode_frac_hbm_peak": (kv_row_bytes * kv_tok) / (ms_d * 1e-3) / 1e9 / PEAK_HBM_GBS,
                "shape": "%d chunks x %d, prefix %d, %d query rows" % (len(sp.chunk_lens), sp.chunk_lens[0], sp.prefix_len, sp.q_len)}
            if kv_row_bytes * kv_tok < 128e6:
                # a cache this small stays in the last-level cache when one call is looped: rotate over
                # copies of the request that together exceed it (16 x 42 MB against 256 MB), so that
                # every call reads its KV from HBM
                n_rot = 16
                rot = []
                for i in range(n_rot):
                    ri = W.make_request(sp, dev, run_index=i + 1)
                    ki, vi = ri.chunk_views()
                    rqi = B.Request(ri.k_prefix, ri.v_prefix, ki, vi, ri.k_self, ri.v_self, sp.q_len, ri.temperature, ri.scale)
                    fi, ai = B.decode_call(shape, [rqi], q1, o1, None, wsc)
                    ai[0].self_len = sp.q_len + 1
                    rot.append((fi, ai, ri, rqi))

                def rotated():
                    for fi, _, _, _ in rot:
                        fi()
                ms_rot = timed(rotated, 20) / n_rot
                cfg_res[sp.name]["decode_note"] = "one call looped: its %.0f MB of KV stay in the last-level cache" % (kv_row_bytes * kv_tok / 1e6)
                cfg_res[sp.name]["decode_rotated_ms_per_token"] = ms_rot
                cfg_res[sp.name]["decode_rotated_gbs"] = (kv_row_bytes * kv_tok) / (ms_rot * 1e-3) / 1e9
                cfg_res[sp.name]["decode_rotated_frac_hbm_peak"] = (kv_row_bytes * kv_tok) / (ms_rot * 1e-3) / 1e9 / PEAK_HBM_GBS
                cfg_res[sp.name]["decode_rotated_note"] = "%d copies of the request in turn (%.0f MB): every call reads from HBM" % (n_rot, n_rot * kv_row_bytes * kv_tok / 1e6)
                del rot
            del rr, rq, oc, wsc

    layer_res = None
    if args.layer:
        hidden, inter = 4096, 14336
        gw = torch.Generator(device=dev)
        gw.manual_seed(r.seed + 7)
        rn = lambda *sh, scale=1.0: (torch.randn(sh, generator=gw, device=dev, dtype=torch.float32) * scale).to(torch.bfloat16)
        wts = dict(attn_norm=torch.ones(hidden, dtype=torch.bfloat16, device=dev), w_qkv=rn((hq + 2 * hkv) * d, hidden, scale=hidden ** -0.5),
                   w_o=rn(hidden, hq * d, scale=(hq * d) ** -0.5), mlp_norm=torch.ones(hidden, dtype=torch.bfloat16, device=dev),
                   w_gate_up=rn(2 * inter, hidden, scale=hidden ** -0.5), w_down=rn(hidden, inter, scale=inter ** -0.5))
        lw = B.layer_weights(hidden, inter, 1e-5, 500000.0, **wts)
        m_tok = spec.total_ctx_len
        xl = rn(m_tok, hidden)
        yl = torch.empty_like(xl)
        kcl, vcl = torch.empty_like(r.k_ctx), torch.empty_like(r.v_ctx)
        ws_l = torch.empty(B.layer_workspace_bytes(shape, hidden, inter, m_tok) // 4, dtype=torch.float32, device=dev)

        def layer_call():
            B.layer_encode(shape, lw, xl, r.k_prefix, r.v_prefix, cu, cu_dev, kcl, vcl, yl, ws_l)
        ms_l = timed(layer_call, 5)
        fl_gemm = 2.0 * m_tok * hidden * ((hq + 2 * hkv) * d + hq * d + 3 * inter)
        layer_res = {"ms": ms_l, "tflops": (fl_gemm + fl_enc) / (ms_l * 1e-3) / 1e12, "gemm_flop": fl_gemm, "attention_flop": fl_enc,
                     "attention_share_of_time": float(ms_enc) / ms_l,
                     "projected_32_layer_prefill_s": 32 * ms_l * 1e-3,
                     "note": "hidden 4096, MLP 14336, 32 q / 8 kv heads, bf16; 131072 context tokens as 64 x 2048; the four "
                             "projections are rocBLAS GEMMs"}
        del xl, yl, kcl, vcl, ws_l, wts

    layers_res = None
    if args.layers > 0:
        hidden, inter, nl = 4096, 14336, args.layers
        gw = torch.Generator(device=dev)
        gw.manual_seed(r.seed + 9)
        rn = lambda *sh, scale=1.0: (torch.randn(sh, generator=gw, device=dev, dtype=torch.float32) * scale).to(torch.bfloat16)
        keep, lws = [], []
        for _ in range(nl):
            wts = dict(attn_norm=torch.ones(hidden, dtype=torch.bfloat16, device=dev), w_qkv=rn((hq + 2 * hkv) * d, hidden, scale=hidden ** -0.5),
                       w_o=rn(hidden, hq * d, scale=(hq * d) ** -0.5), mlp_norm=torch.ones(hidden, dtype=torch.bfloat16, device=dev),
                       w_gate_up=rn(2 * inter, hidden, scale=hidden ** -0.5), w_down=rn(hidden, inter, scale=inter ** -0.5))
            keep.append(wts)
            lws.append(B.layer_weights(hidden, inter, 1e-5, 500000.0, **wts))
        m_tok = spec.total_ctx_len
        xl = rn(m_tok, hidden)
        yl = torch.empty_like(xl)
        kcs = [torch.empty_like(r.k_ctx) for _ in range(nl)]
        vcs = [torch.empty_like(r.v_ctx) for _ in range(nl)]
        kps, vps = [r.k_prefix] * nl, [r.v_prefix] * nl
        ws_l = torch.empty(B.layer_workspace_bytes(shape, hidden, inter, m_tok, n_layers=nl) // 4, dtype=torch.float32, device=dev)
        ms_ls = timed(lambda: B.layers_encode(shape, lws, xl, kps, vps, cu, cu_dev, kcs, vcs, yl, ws_l), 2)
        layers_res = {"layers": nl, "ms": ms_ls, "ms_per_layer": ms_ls / nl,
                      "note": "ape_layers_encode: %d Llama-3-8B-shaped layers (random weights), 131072 context tokens as 64 x 2048, "
                              "every layer writing its own KV cache" % nl}
        del xl, yl, kcs, vcs, ws_l, keep

    batch_res = None
    if args.prefill_batch > 0:
        nb = args.prefill_batch
        rb = [r] + [W.make_request(spec, dev, request=b) for b in range(1, nb)]
        reqs_b = [req]
        for rr in rb[1:]:
            kb_, vb_ = rr.chunk_views()
            reqs_b.append(B.Request(rr.k_prefix, rr.v_prefix, kb_, vb_, rr.k_self, rr.v_self, spec.q_len, rr.temperature, rr.scale))
        qb = torch.stack([rr.q_self[:spec.q_len] for rr in rb]).contiguous()
        ob = torch.empty_like(qb)
        ws_b = torch.empty(B.workspace_bytes(B.APE_OP_PREFILL, shape, nb, spec.q_len, spec.total_ctx_len) // 4, dtype=torch.float32, device=dev)

        def batch_call():
            B.attention_prefill_batch(shape, reqs_b, qb, ob, None, ws_b)
        ms_b = timed(batch_call, 20)
        batch_res = {"batch": nb, "ms": ms_b, "tflops": nb * fl_pre / (ms_b * 1e-3) / 1e12,
                     "frac_mfma_peak": nb * fl_pre / (ms_b * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                     "note": "%d requests x 256 query rows, each over its own 128K cache (T, S per request)" % nb}
        del rb, reqs_b, qb, ob, ws_b

    rope_res = None
    if args.rope_write:
        q_raw = torch.empty_like(r.q_ctx).normal_()
        k_raw = torch.empty_like(r.k_ctx).normal_()
        v_raw = torch.empty_like(r.v_ctx).normal_()
        q_rot, k_c, v_c = torch.empty_like(q_raw), torch.empty_like(k_raw), torch.empty_like(v_raw)
        kt = torch.tensor([k_c[cu[i]:].data_ptr() for i in range(len(r.chunk_lens))], dtype=torch.int64, device=dev)
        vt = torch.tensor([v_c[cu[i]:].data_ptr() for i in range(len(r.chunk_lens))], dtype=torch.int64, device=dev)

        def rope_call():
            B.rope_write_cache(shape, q_raw, k_raw, v_raw, cu, cu_dev, spec.prefix_len, 500000.0, q_rot, kt, vt)
        ms_rope = timed(rope_call, 30)
        by_rope = 2.0 * (q_raw.numel() + k_raw.numel() + v_raw.numel()) * 2          # every element read once, written once
        rope_res = {"ms": ms_rope, "gbs": by_rope / (ms_rope * 1e-3) / 1e9, "frac_hbm_peak": by_rope / (ms_rope * 1e-3) / 1e9 / PEAK_HBM_GBS,
                    "bytes": by_rope, "note": "131072 tokens x (32 q + 8 k + 8 v heads) x 128, bf16, read once and written once"}
        del q_raw, k_raw, v_raw, q_rot, k_c, v_c

    gemm_ref = None
    if args.gemm_reference:
        n = 8192
        gemm_ref = {}
        for name in ("zeros", "random"):
            a_ = torch.zeros(n, n, dtype=torch.bfloat16, device=dev)
            b_ = torch.zeros(n, n, dtype=torch.bfloat16, device=dev)
            if name == "random":
                a_.normal_(); b_.normal_()
            ms_g = timed(lambda: torch.matmul(a_, b_), 20)
            gemm_ref["torch_bf16_gemm_8192_tflops_" + name] = 2.0 * n ** 3 / (ms_g * 1e-3) / 1e12
            del a_, b_

    sdpa_ref = None
    if args.sdpa_reference:
        import torch.nn.functional as F
        from torch.nn.attention import SDPBackend, sdpa_kernel
        sdpa_ref = {}
        n_ch, l_ch = len(spec.chunk_lens), spec.chunk_lens[0]
        g = hq // hkv
        # K and V heads repeated for the query heads (torch's fused kernels take equal head counts)
        qe = r.q_ctx.view(n_ch, l_ch, hq, d).transpose(1, 2).contiguous()
        ke = r.k_ctx.view(n_ch, l_ch, hkv, d).transpose(1, 2).repeat_interleave(g, dim=1).contiguous()
        ve = r.v_ctx.view(n_ch, l_ch, hkv, d).transpose(1, 2).repeat_interleave(g, dim=1).contiguous()
        qp = q.view(1, spec.q_len, hq, d).transpose(1, 2).contiguous()
        kp, vp = ke.transpose(0, 1).reshape(1, hq, n_ch * l_ch, d), ve.transpose(0, 1).reshape(1, hq, n_ch * l_ch, d)
        cases = (("encode_like_causal_%dx%d" % (n_ch, l_ch), lambda: F.scaled_dot_product_attention(qe, ke, ve, is_causal=True),
                  4.0 * d * hq * n_ch * l_ch * (l_ch + 1) / 2),
                 ("prefill_like_%d_rows_over_%d_keys" % (spec.q_len, n_ch * l_ch), lambda: F.scaled_dot_product_attention(qp, kp, vp),
                  4.0 * d * hq * spec.q_len * n_ch * l_ch))
        for name, fn, flops in cases:
            try:
                with sdpa_kernel([SDPBackend.FLASH_ATTENTION, SDPBackend.EFFICIENT_ATTENTION]):
                    ms_s = timed(fn, 20)
                sdpa_ref[name] = {"ms": ms_s, "tflops": flops / (ms_s * 1e-3) / 1e12}
            except Exception as exc:                      # no fused kernel for this shape on this build of torch
                sdpa_ref[name] = {"error": str(exc)[:200]}
        sdpa_ref["note"] = ("torch.nn.functional.scaled_dot_product_attention, fused backends only, K/V heads repeated to 32; "
                            "same flop convention (unmasked pairs only)")
        del qe, ke, ve, qp, kp, vp

    # ---- what this machine can do at all: the published peaks assume clocks the chip does not hold under
    # a full matrix-core load on random data (it is power-limited), so the measured ceilings are
    # reported next to them.  Context for the roofline fractions, which stay against the published peaks.
    ceilings = None
    if not args.no_ceilings:
        sink = torch.zeros(4, dtype=torch.float32, device=dev)
        ops_zero = torch.zeros(65536 // 2, dtype=torch.bfloat16, device=dev)
        gp = torch.Generator(device=dev)
        gp.manual_seed(r.seed + 31)
        ops_rand = torch.randn(65536 // 2, generator=gp, device=dev, dtype=torch.float32).to(torch.bfloat16)
        big = torch.empty(1 << 29, dtype=torch.float32, device=dev).normal_()      # 2 GiB, beyond the last-level cache
        ceilings = {
            "mfma_bf16_zero_operands_tflops": B.probe_mfma(ops_zero, 0, sink),
            "mfma_bf16_random_operands_tflops": B.probe_mfma(ops_rand, 0, sink),
            "mfma_bf16_random_operands_with_softmax_valu_tflops": B.probe_mfma(ops_rand, 1, sink),
            "mfma_bf16_random_operands_softmax_lds_fragments_tflops": B.probe_mfma(ops_rand, 2, sink),
            "mfma_bf16_random_operands_block_loop_skeleton_tflops": B.probe_mfma(ops_rand, 3, sink),
            "mfma_bf16_random_operands_block_loop_skeleton_narrow_tile_tflops": B.probe_mfma(ops_rand, 4, sink),
            "hbm_read_only_gbs": B.probe_hbm_read(big, sink),
            "softmax_valu_ns_per_instruction_per_simd": {str(w): B.probe_valu_issue(w, sink) for w in (1, 2, 4)},
            "note": "libape_probe.so: MFMA 32x32x16 bf16 back to back, one wavefront per SIMD on every CU (no LDS, no loads); "
                    "the third figure adds the vector work of a flash-attention softmax (per pair of scores 2 FMA, 2 exp, 2 add, "
                    "1 packed conversion) in the MFMAs' shadows; the fourth also fetches the A operands from LDS as a flash body "
                    "fetches its K and V^T fragments; the fifth also loads a 16 KB block per 32 MFMAs straight into an LDS ring (out of "
                    "the cache), waits and passes a workgroup barrier: a flash block loop without bookkeeping, masks and HBM traffic "
                    "(the sixth: the same for the narrow tile, 32 rows per wavefront, two workgroups per CU); "
                    "read-only stream over 2 GiB; the softmax's vector instructions alone with 1, 2 and 4 wavefronts per SIMD",
        }
        for key in ("mfma_bf16_zero_operands_tflops", "mfma_bf16_random_operands_tflops", "mfma_bf16_random_operands_with_softmax_valu_tflops",
                    "mfma_bf16_random_operands_softmax_lds_fragments_tflops", "mfma_bf16_random_operands_block_loop_skeleton_tflops",
                    "mfma_bf16_random_operands_block_loop_skeleton_narrow_tile_tflops"):
            ceilings[key.replace("_tflops", "_frac_of_published_peak")] = ceilings[key] / PEAK_BF16_TFLOPS
        ceilings["hbm_read_only_frac_of_published_peak"] = ceilings["hbm_read_only_gbs"] / PEAK_HBM_GBS
        del big, ops_zero, ops_rand

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                                                  # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    # ---- batched decode (config 5): the clean HBM measurement, timed in its own region
    if not args.no_cfg5:
        spec5 = W.CONFIGS[5]
        rs = [W.make_request(spec5, dev, request=b) for b in range(spec5.batch)]
        reqs = []
        for rr in rs:
            k5, v5 = rr.chunk_views()
            reqs.append(B.Request(rr.k_prefix, rr.v_prefix, k5, v5, rr.k_self, rr.v_self, 1, rr.temperature, rr.scale))
        q5 = torch.stack([rr.q_self for rr in rs], dim=1).contiguous()          # [steps, batch, Hq, d]
        o5 = torch.empty_like(q5[0])
        ws5 = torch.empty(B.workspace_bytes(B.APE_OP_DECODE, shape, spec5.batch, 1, spec5.total_ctx_len) // 4, dtype=torch.float32, device=dev)

        calls5 = []
        for s in range(spec5.decode_steps):
            fn, arr = B.decode_call(shape, reqs, q5[s], o5, None, ws5)
            for b in range(spec5.batch):
                arr[b].self_len = s + 1
            calls5.append((fn, arr))

        def decode_pass():
            for fn, _ in calls5:
                fn()
        ms5 = timed(decode_pass, 5)
        tok5 = [spec5.batch * (spec5.prefix_len + spec5.total_ctx_len + s + 1) for s in range(spec5.decode_steps)]
        by5 = sum(kv_row_bytes * t + spec5.batch * 2 * hq * d * 2 for t in tok5)
        phases["decode_cfg5_batch32"] = {"ms_per_step": ms5 / spec5.decode_steps, "gbs": by5 / (ms5 * 1e-3) / 1e9,
                                         "frac_hbm_peak": by5 / (ms5 * 1e-3) / 1e9 / PEAK_HBM_GBS,
                                         "note": "32 requests x 16.4K KV tokens, 128 steps, 2.15 GB per step"}
        del calls5, rs, reqs, q5, o5, ws5

    # ---- the oracle beside it, on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import ape_oracle
        n = W.to_numpy_f32
        kc, vc, kp, vp = n(r.k_ctx), n(r.v_ctx), n(r.k_prefix), n(r.v_prefix)
        ksf, vsf, qs = n(r.k_self[:spec.q_len]), n(r.v_self[:spec.q_len]), n(q)
        rng = np.random.default_rng(0)

        def sample(n_pairs):
            pairs = [(int(rng.integers(spec.q_len)), int(rng.integers(hq))) for _ in range(n_pairs)]
            t = time.perf_counter()
            ape_oracle.attention(qs, kp, vp, kc, vc, r.chunk_lens, ksf, vsf, r.temperature, r.scale, pairs=pairs)
            dt = time.perf_counter() - t
            fl = sum(4.0 * d * (spec.prefix_len + spec.total_ctx_len + row + 1) for row, _ in pairs)
            return dt, fl
        threads = ape_oracle.num_threads()
        dt, fl = sample(2 * threads)                                    # calibration
        n_pairs = int(max(2 * threads, min(8192, args.cpu_seconds / max(dt, 1e-3) * 2 * threads)))
        dt, fl = sample(n_pairs)
        cpu = {"value": fl / dt / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
               "sample": "%d random (row, head) pairs of the config-3 query prefill, each over its full 131K KV, fp64, %.1f s" % (n_pairs, dt)}

    line = {
        "metric": "APE attn TFLOP/s (query prefill over 128K cached KV) + decode HBM GB/s",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "warm_steps": warm_steps, "warm_ms": warm_spent,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "config 3: 128K context (64 chunks x 2048 + prefix 32), Llama-3-8B heads (32q/8kv, d=128), "
                               "encode + 256-row query prefill + %d decode steps, T=0.8 S=0.85, batch 1" % args.decode_steps,
                   "seed": r.seed, "generator": r.generator},
        "headline_prefill_tflops": phases["prefill"]["tflops"],
        "headline_decode_gbs": phases.get("decode_cfg5_batch32", {}).get("gbs"),
        "phases": phases, "roofline": roof, "cpu_baseline": cpu,
    }
    if ceilings is not None:
        line["measured_ceilings"] = ceilings
    if gemm_ref is not None:
        line["gemm_reference"] = gemm_ref
    if sdpa_ref is not None:
        line["sdpa_reference"] = sdpa_ref
    if seq_cmp is not None:
        line["sequential_comparator"] = seq_cmp
    if tree_var is not None:
        line["tree_variants"] = tree_var
    if rope_res is not None:
        line["rope_write_cache"] = rope_res
    if batch_res is not None:
        line["prefill_batch"] = batch_res
    if layer_res is not None:
        line["layer_encode"] = layer_res
    if layers_res is not None:
        line["layers_encode"] = layers_res
    if cfg_res is not None:
        line["other_configs"] = cfg_res
    print(json.dumps(line))


if __name__ == "__main__":
    main()
