"""GPU parity at the full benchmark sizes (configs 3, 4, 5), in the launch configuration bench.py
times.  The oracle computes outputs one by one -- each (row, head) pair exactly, over its full KV:
every output of the query prefills (8192 at config 3, 4096 at config 4) and of the batched decode;
4096 distinct sampled rows of each encode (drawn without replacement) -- always including
first/last rows and heads and rows at tile and chunk boundaries; size-independent properties cover
the rest."""
import numpy as np
import pytest
import torch

from paper_2502_05431_amd import binding as B
from paper_2502_05431_amd import workloads as W

import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _pairs(rng, n_rows, n_heads, n, must_rows=()):
    """n DISTINCT (row, head) pairs (all of them when there are no more than n): the required rows
    with the first and last head, the rest drawn without replacement."""
    total = n_rows * n_heads
    if n >= total:
        return [(r, h) for r in range(n_rows) for h in range(n_heads)]
    rows = {0, n_rows - 1, *[r for r in must_rows if 0 <= r < n_rows]}
    pairs = [(r, h) for r in sorted(rows) for h in sorted({0, n_heads - 1})]
    seen = set(pairs)
    for idx in rng.permutation(total):
        if len(pairs) >= n:
            break
        pr = (int(idx) // n_heads, int(idx) % n_heads)
        if pr not in seen:
            seen.add(pr)
            pairs.append(pr)
    assert len(set(pairs)) == len(pairs) == n
    return pairs


def _gather(t: torch.Tensor, pairs, head_major=False):
    a = t.detach().float().cpu().numpy().astype(np.float64)      # one copy, then host indexing
    rows = np.array([r for r, _ in pairs]); heads = np.array([h for _, h in pairs])
    return a[heads, rows] if head_major else a[rows, heads]      # head_major: [Hq, rows]


def test_cfg3_128k_encode_and_prefill_sampled():
    spec = W.CONFIGS[3]
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    rng = np.random.default_rng(3)

    # query prefill: 256 rows over the 131K cached KV -- every one of the 8192 (row, head) outputs
    out, lse = H.run_prefill(spec, r, spec.q_len, spec.q_len)
    pairs = _pairs(rng, spec.q_len, spec.n_q_heads, spec.q_len * spec.n_q_heads)
    assert len(pairs) == 8192
    ref, ref_lse, _ = H.oracle_prefill(h, spec.q_len, spec.q_len, r.temperature, r.scale, pairs=pairs)
    H.check_close(_gather(out, pairs), ref, "bf16", "cfg3 prefill")
    assert np.abs(_gather(lse, pairs, head_major=True) - ref_lse).max() <= H.lse_tol("bf16")
    assert torch.isfinite(out.float()).all()

    # encode: 64 chunks x 2048 rows; sample rows at chunk starts/ends and tile edges
    o_ctx, lse_ctx, o_p, _ = H.run_encode(spec, r)
    m = spec.total_ctx_len
    must = [0, 1, 63, 64, 2047, 2048, 2049, 4095, 4096, m - 2048, m - 2047, m - 1, 2048 * 17 + 1023, 2048 * 40 + 64]
    pairs = _pairs(rng, m, spec.n_q_heads, 4096, must_rows=must)
    ref, ref_lse = H.oracle_encode(h, pairs=pairs)
    H.check_close(_gather(o_ctx, pairs), ref, "bf16", "cfg3 encode")
    assert np.abs(_gather(lse_ctx, pairs, head_major=True) - ref_lse).max() <= H.lse_tol("bf16")
    assert torch.isfinite(o_ctx.float()).all()
    refp, _ = H.oracle_encode_prefix(h)
    H.check_close(H.f64(o_p).reshape(-1, spec.head_dim), refp, "bf16", "cfg3 prefix rows")


def test_cfg3_rows_sum_to_one_at_full_size():
    spec = W.CONFIGS[3]
    r = W.make_request(spec, DEV)
    for name in ("v_prefix", "v_ctx", "v_self"):
        getattr(r, name).fill_(1.0)
    out, _ = H.run_prefill(spec, r, spec.q_len, spec.q_len)
    assert (out.float() - 1.0).abs().max().item() <= 2 ** -8
    o_ctx, _, _, _ = H.run_encode(spec, r, with_prefix_rows=False, want_lse=False)
    assert (o_ctx.float() - 1.0).abs().max().item() <= 2 ** -8


def test_cfg4_manyshot_prefill_and_decode_sampled():
    spec = W.CONFIGS[4]
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    rng = np.random.default_rng(4)
    out, lse = H.run_prefill(spec, r, spec.q_len, spec.q_len)
    pairs = [(row, head) for row in range(spec.q_len) for head in range(spec.n_q_heads)]      # every output: 4096
    ref, ref_lse, _ = H.oracle_prefill(h, spec.q_len, spec.q_len, r.temperature, r.scale, pairs=pairs)
    H.check_close(_gather(out, pairs), ref, "bf16", "cfg4 prefill")
    assert np.abs(_gather(lse, pairs, head_major=True) - ref_lse).max() <= H.lse_tol("bf16")
    for step in sorted({*range(0, 64, 4), 63}):           # 16 of the 64 decode steps spread over the run, and the last
        sl = spec.q_len + step + 1
        outd, lsed = H.run_decode(spec, [r], [sl])
        refd, refd_lse, _ = H.oracle_prefill(h, 1, sl, r.temperature, r.scale)
        H.check_close(H.f64(outd).reshape(-1, spec.head_dim), refd, "bf16", "cfg4 decode step %d" % step)
        assert np.abs(H.f64(lsed).reshape(-1) - refd_lse).max() <= H.lse_tol("bf16")
    # encode of 512 short chunks
    o_ctx, _, _, _ = H.run_encode(spec, r, with_prefix_rows=False, want_lse=False)
    m = spec.total_ctx_len
    pairs = _pairs(rng, m, spec.n_q_heads, 4096, must_rows=(255, 256, 257, m - 256, 256 * 300 + 63, 256 * 300 + 64))
    ref, _ = H.oracle_encode(h, pairs=pairs)
    H.check_close(_gather(o_ctx, pairs), ref, "bf16", "cfg4 encode")


def test_cfg5_batched_decode_all_outputs():
    """32 requests x 16.4K KV tokens, per-request T and S: every (request, head) output at the
    first, a middle and the last decode step."""
    spec = W.CONFIGS[5]
    rs = [W.make_request(spec, DEV, request=b) for b in range(spec.batch)]
    assert len({round(r.temperature, 4) for r in rs}) > 8 and len({round(r.scale, 4) for r in rs}) > 8
    for step in (0, 64, 127):
        sl = step + 1
        out, lse = H.run_decode(spec, rs, [sl] * spec.batch)
        for b in (range(spec.batch) if step == 127 else (0, 13, 31)):
            h = H.HostArrays(rs[b])
            ref, ref_lse, _ = H.oracle_prefill(h, 1, sl, rs[b].temperature, rs[b].scale)
            H.check_close(H.f64(out[b]), ref, "bf16", "cfg5 request %d step %d" % (b, step))
            assert np.abs(H.f64(lse[b]) - ref_lse).max() <= H.lse_tol("bf16")


def test_long_chunks_take_the_wide_tile_encode_sampled():
    """Chunks beyond 4096 tokens (the shape of the sequential-encoding comparator: few, long causal
    chunks) run on the wide query tile with long fast stretches; sampled rows at chunk starts and
    ends, tile edges and deep inside."""
    spec = W.CONFIGS[3].replace(chunk_lens=(6000, 4500, 33), q_len=8, decode_steps=0)
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    rng = np.random.default_rng(7)
    o_ctx, lse_ctx, _, _ = H.run_encode(spec, r, with_prefix_rows=False)
    m = spec.total_ctx_len
    must = [0, 1, 63, 64, 65, 4095, 4096, 5999, 6000, 6001, 6063, 6064, 10499, 10500, 10501, m - 1, 3000, 8200]
    pairs = _pairs(rng, m, spec.n_q_heads, 320, must_rows=must)
    ref, ref_lse = H.oracle_encode(h, pairs=pairs)
    H.check_close(_gather(o_ctx, pairs), ref, "bf16", "long chunks encode")
    assert np.abs(_gather(lse_ctx, pairs, head_major=True) - ref_lse).max() <= H.lse_tol("bf16")
    assert torch.isfinite(o_ctx.float()).all()


def test_outlier_keys_move_the_softmax_reference_on_the_wide_tile():
    """The lazily updated softmax reference on the WIDE tile, whose long stretches of full blocks run in
    groups of bodies with the softmax dealt over the MFMA slots: keys planted deep inside long contexts
    (prefill over 50K tokens) and deep inside a long chunk (encode), each aligned with one query row so
    that its score towers over everything before it, force the rare path in the middle of such a stretch."""
    spec = W.CONFIGS[3].replace(chunk_lens=(30000, 20000), q_len=64, prefix_len=32, decode_steps=0)
    r = W.make_request(spec, DEV)
    g = spec.n_q_heads // spec.n_kv_heads
    rows = []
    for hk in range(spec.n_kv_heads):
        r.k_ctx[15000 + 40 * hk, hk] = 6.0 * r.q_self[5 + hk, hk * g]             # chunk 0, deep inside a split
        r.k_ctx[30000 + 17000, hk] = 6.0 * r.q_self[40, hk * g + g - 1]           # chunk 1
        r.k_ctx[9000, hk] = 5.0 * r.q_ctx[20000, hk * g + 1]                      # encode: row 20000 of chunk 0 sees token 9000
        r.k_ctx[30000 + 5000, hk] = 5.0 * r.q_ctx[30000 + 19999, hk * g + 2]      # ... chunk 1: its last row, token 5000
        rows.append(5 + hk)
    h = H.HostArrays(r)
    rng = np.random.default_rng(23)
    out, lse = H.run_prefill(spec, r, spec.q_len, spec.q_len)
    pairs = _pairs(rng, spec.q_len, spec.n_q_heads, 160, must_rows=rows + [40])
    pairs += [pr for pr in ([(5 + hk, hk * g) for hk in range(spec.n_kv_heads)] + [(40, hk * g + g - 1) for hk in range(spec.n_kv_heads)]) if pr not in pairs]
    ref, ref_lse, _ = H.oracle_prefill(h, spec.q_len, spec.q_len, r.temperature, r.scale, pairs=pairs)
    H.check_close(_gather(out, pairs), ref, "bf16", "wide prefill with outliers")
    assert np.abs(_gather(lse, pairs, head_major=True) - ref_lse).max() <= H.lse_tol("bf16")
    o_ctx, lse_ctx, _, _ = H.run_encode(spec, r, with_prefix_rows=False)
    m = spec.total_ctx_len
    pairs = _pairs(rng, m, spec.n_q_heads, 96, must_rows=[20000, 49999, 9000, 35000])
    pairs += [pr for pr in ([(20000, hk * g + 1) for hk in range(spec.n_kv_heads)] + [(49999, hk * g + 2) for hk in range(spec.n_kv_heads)]) if pr not in pairs]
    ref, ref_lse = H.oracle_encode(h, pairs=pairs)
    H.check_close(_gather(o_ctx, pairs), ref, "bf16", "wide encode with outliers")
    assert np.abs(_gather(lse_ctx, pairs, head_major=True) - ref_lse).max() <= H.lse_tol("bf16")
    assert torch.isfinite(out.float()).all() and torch.isfinite(o_ctx.float()).all()
    # the planted keys really are beyond the lazy threshold (2^40 ~ 27.7 in natural-log units)
    qk = (r.q_self[5].float()[0] * r.k_ctx[15000, 0].float()).sum().item() / spec.head_dim ** 0.5 / r.temperature
    assert qk > 40.0


@pytest.mark.parametrize("chunk_lens, q_len, self_extra", [
    ((20000, 1, 13000, 333, 9000, 64, 31), 50, 0),        # just above the switch; 200 ragged rows on one wide tile
    ((12000, 0, 12000, 12000, 6999, 3), 130, 70),         # three wide tiles, the last ragged; long own span
    ((9000, 9000, 2000), 8, 0),                           # few rows, 20K context: twice the workgroups per row tile
    ((30000, 10959), 32, 3),                              # 128 rows per KV head just below the switch: the most splits of any plan
    ((40960,), 50, 0),                                    # the last context length on the narrow tile
    ((40961,), 50, 0),                                    # the first one on the wide tile
    ((20000, 480), 1024, 0),                              # 4096 rows per KV head: the last context length on the narrow tile
    ((20000, 481), 1024, 0),                              # ... and the first on the wide one
    ((6145,), 2048, 0),                                   # 8192 rows per KV head: the wide tile from 6145 context tokens
])
def test_prefill_tile_switch_by_context_length_sampled(chunk_lens, q_len, self_extra):
    """The query prefill takes the narrow query tile up to 40960 context tokens (20480 with 4096 or more
    query rows per KV head, 6144 with 8192 or more) and the wide one beyond (when a KV head has more than
    128 query rows): ragged contexts on both sides of the switch, sampled rows at tile edges."""
    spec = W.CONFIGS[3].replace(chunk_lens=chunk_lens, q_len=q_len, prefix_len=7, decode_steps=self_extra, k_scale=1.0)
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    rng = np.random.default_rng(11)
    self_len = q_len + self_extra
    out, lse = H.run_prefill(spec, r, q_len, self_len)
    pairs = _pairs(rng, q_len, spec.n_q_heads, 192, must_rows=(31, 32, 33, 63, 64, 65, 127, 128))
    ref, ref_lse, _ = H.oracle_prefill(h, q_len, self_len, r.temperature, r.scale, pairs=pairs)
    H.check_close(_gather(out, pairs), ref, "bf16", "prefill %s" % (chunk_lens,))
    assert np.abs(_gather(lse, pairs, head_major=True) - ref_lse).max() <= H.lse_tol("bf16")
    assert torch.isfinite(out.float()).all()


@pytest.mark.parametrize("hq, hkv", [(8, 8), (16, 8), (16, 2)])
def test_wide_tile_with_other_head_ratios_sampled(hq, hkv):
    """The wide query tile (prefill beyond 40960 context tokens, encode of chunks beyond 4096 tokens)
    for 1, 2 and 8 query heads per KV head; ragged rows and contexts, sampled outputs."""
    g = hq // hkv
    q_len = 300 // g + 3                                  # more than one wide tile of (token, head) rows, the last ragged
    spec = W.CONFIGS[3].replace(n_q_heads=hq, n_kv_heads=hkv, chunk_lens=(30000, 5000, 1, 6037), q_len=q_len,
                                prefix_len=19, decode_steps=5, k_scale=1.0)
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    rng = np.random.default_rng(100 + g)
    self_len = q_len + 5
    out, lse = H.run_prefill(spec, r, q_len, self_len)
    pairs = _pairs(rng, q_len, hq, 160, must_rows=(256 // g - 1, 256 // g, 128 // g, 64 // g))
    ref, ref_lse, _ = H.oracle_prefill(h, q_len, self_len, r.temperature, r.scale, pairs=pairs)
    H.check_close(_gather(out, pairs), ref, "bf16", "wide prefill G=%d" % g)
    assert np.abs(_gather(lse, pairs, head_major=True) - ref_lse).max() <= H.lse_tol("bf16")
    o_ctx, lse_ctx, _, _ = H.run_encode(spec, r, with_prefix_rows=False)
    m = spec.total_ctx_len
    pairs = _pairs(rng, m, hq, 200, must_rows=(0, 63, 64, 4095, 4096, 29999, 30000, 30001, 34999, 35000, 35001, m - 1))
    ref, ref_lse = H.oracle_encode(h, pairs=pairs)
    H.check_close(_gather(o_ctx, pairs), ref, "bf16", "wide encode G=%d" % g)
    assert np.abs(_gather(lse_ctx, pairs, head_major=True) - ref_lse).max() <= H.lse_tol("bf16")
    assert torch.isfinite(out.float()).all() and torch.isfinite(o_ctx.float()).all()


def test_batched_prefill_on_the_wide_tile_sampled():
    """Three requests in one batched prefill whose longest context (45 000 tokens) puts the call on the
    wide query tile: the short and the empty context leave most of their splits untouched."""
    base = W.CONFIGS[3].replace(temperature=None, scale=None, decode_steps=30, k_scale=1.0)
    q_len = 48                                            # 192 (token, head) rows per KV head: one ragged wide tile
    specs = [base.replace(chunk_lens=(20000, 25000), q_len=q_len), base.replace(chunk_lens=(300,), q_len=q_len, prefix_len=7),
             base.replace(chunk_lens=(), q_len=q_len)]
    self_lens = [48, 61, 78]
    rs = [W.make_request(sp, DEV, request=b) for b, sp in enumerate(specs)]
    shape = B.make_shape(base.n_q_heads, base.n_kv_heads, base.head_dim, base.torch_dtype)
    reqs = [H.make_binding_request(r, sl) for r, sl in zip(rs, self_lens)]
    q = torch.stack([r.q_self[sl - q_len:sl] for r, sl in zip(rs, self_lens)]).contiguous()
    out = torch.full_like(q, float("nan"))
    lse = torch.full((len(rs), base.n_q_heads, q_len), float("nan"), dtype=torch.float32, device=DEV)
    ws = H.poisoned_workspace(B.workspace_bytes(B.APE_OP_PREFILL, shape, len(rs), q_len), DEV)
    B.attention_prefill_batch(shape, reqs, q, out, lse, ws, self_lens=self_lens)
    torch.cuda.synchronize()
    rng = np.random.default_rng(21)
    for b, (r, sl) in enumerate(zip(rs, self_lens)):
        h = H.HostArrays(r)
        pairs = _pairs(rng, q_len, base.n_q_heads, 128, must_rows=(31, 32, 33))
        ref, ref_lse, _ = H.oracle_prefill(h, q_len, sl, r.temperature, r.scale, pairs=pairs)
        H.check_close(_gather(out[b], pairs), ref, "bf16", "request %d" % b)
        assert np.abs(_gather(lse[b], pairs, head_major=True) - ref_lse).max() <= H.lse_tol("bf16")
    assert torch.isfinite(out.float()).all()
