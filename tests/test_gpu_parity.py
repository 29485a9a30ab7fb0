"""GPU parity: the HIP library (through its C ABI) against the fp64 CPU oracle, element by
element, on the same seeded inputs.  Sizes here are the ones the oracle finishes in seconds;
full-size sampled parity lives in test_gpu_fullsize.py."""
import numpy as np
import pytest
import torch

from paper_2502_05431_amd import binding as B
from paper_2502_05431_amd import workloads as W

import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _check_query(spec, r, h, q_len, self_len, generic=False, req=None, what=""):
    out, lse = H.run_prefill(spec, r, q_len, self_len, generic=generic, req=req)
    ref, ref_lse, _ = H.oracle_prefill(h, q_len, self_len, r.temperature, r.scale)
    H.check_close(H.f64(out).reshape(-1, spec.head_dim), ref, spec.dtype, what + " prefill out")
    got_lse = H.f64(lse).T.reshape(-1)                  # [Hq, q_len] -> (row, head) order
    assert np.abs(got_lse - ref_lse).max() <= H.lse_tol(spec.dtype), what + " prefill lse"


def _check_decode(spec, r, h, self_len, generic=False, what=""):
    out, lse = H.run_decode(spec, [r], [self_len], generic=generic)
    ref, ref_lse, _ = H.oracle_prefill(h, 1, self_len, r.temperature, r.scale)
    H.check_close(H.f64(out).reshape(-1, spec.head_dim), ref, spec.dtype, what + " decode out")
    assert np.abs(H.f64(lse).reshape(-1) - ref_lse).max() <= H.lse_tol(spec.dtype), what + " decode lse"


def _check_encode(spec, r, h, generic=False, what=""):
    o_ctx, lse_ctx, o_p, lse_p = H.run_encode(spec, r, generic=generic)
    ref, ref_lse = H.oracle_encode(h)
    H.check_close(H.f64(o_ctx).reshape(-1, spec.head_dim), ref, spec.dtype, what + " encode out")
    assert np.abs(H.f64(lse_ctx).T.reshape(-1) - ref_lse).max() <= H.lse_tol(spec.dtype), what + " encode lse"
    if o_p is not None:
        refp, refp_lse = H.oracle_encode_prefix(h)
        H.check_close(H.f64(o_p).reshape(-1, spec.head_dim), refp, spec.dtype, what + " encode prefix rows")
        assert np.abs(H.f64(lse_p).T.reshape(-1) - refp_lse).max() <= H.lse_tol(spec.dtype)


# ------------------------------------------------------------------ workload 1 (fp32)
@pytest.mark.parametrize("T,S", [(1.0, 1.0), (0.8, 1.0), (1.0, 0.9), (0.8, 0.9)])
def test_cfg1_fp32_all_rows(T, S):
    spec = W.CONFIGS[1].replace(temperature=T, scale=S)
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    _check_encode(spec, r, h, what="cfg1")
    _check_query(spec, r, h, spec.q_len, spec.q_len, what="cfg1")
    for step in range(spec.decode_steps):
        _check_decode(spec, r, h, spec.q_len + step + 1, what="cfg1 step %d" % step)


def test_cfg1_fp32_matches_pooled_not_per_context_scale():
    """The library implements the pooled scaling factor of the main-text equation; the
    per-context reading of Appendix C.2 differs by far more than the fp32 tolerance."""
    spec = W.CONFIGS[1]
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    out, _ = H.run_prefill(spec, r, spec.q_len, spec.q_len)
    pooled, _, _ = H.oracle_prefill(h, spec.q_len, spec.q_len, r.temperature, r.scale, form="hier")
    per_ctx, _, _ = H.oracle_prefill(h, spec.q_len, spec.q_len, r.temperature, r.scale, form="hier_per_context")
    got = H.f64(out).reshape(-1, spec.head_dim)
    assert np.abs(got - pooled).max() <= H.F32_MAX_ABS
    assert np.abs(got - per_ctx).max() > 100 * H.F32_MAX_ABS


def test_fp32_ragged_and_degenerate():
    base = W.CONFIGS[1]
    for kw in (dict(chunk_lens=(1, 70, 3, 64, 129)), dict(chunk_lens=()), dict(prefix_len=0),
               dict(prefix_len=0, chunk_lens=()), dict(chunk_lens=(5,), q_len=1, decode_steps=2),
               dict(head_dim=40, n_q_heads=6, n_kv_heads=2), dict(head_dim=256, n_q_heads=2, n_kv_heads=2, chunk_lens=(9, 9))):
        spec = base.replace(**kw)
        r = W.make_request(spec, DEV)
        h = H.HostArrays(r)
        what = "fp32 %s" % (kw,)
        if spec.chunk_lens:
            _check_encode(spec, r, h, what=what)
        _check_query(spec, r, h, spec.q_len, spec.q_len, what=what)
        _check_decode(spec, r, h, spec.self_len_max, what=what)


def test_decode_of_a_long_context_at_batch_one_merges_many_splits():
    """One request, one query row and thousands of context tokens: the planner cuts the context into
    32 or more splits for a handful of (row, head) units, and the merge then runs its many-wavefront
    variant (fp32 and bf16, ragged contexts so that the last split is short)."""
    for cfg, generic in ((1, False), (2, True)):
        spec = W.CONFIGS[cfg].replace(chunk_lens=(3000, 1, 2500, 2700, 37), q_len=1, decode_steps=3)
        r = W.make_request(spec, DEV)
        h = H.HostArrays(r)
        for sl in (1, 4):
            _check_decode(spec, r, h, sl, generic=generic, what="cfg%d many splits self_len %d" % (cfg, sl))


# ------------------------------------------------------------------ bf16, generic kernels
def test_bf16_generic_small():
    spec = W.CONFIGS[1].replace(dtype="bf16", chunk_lens=(33, 64, 7), q_len=20)
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    _check_encode(spec, r, h, what="bf16 d64")
    _check_query(spec, r, h, spec.q_len, spec.q_len, what="bf16 d64")
    _check_decode(spec, r, h, spec.self_len_max, what="bf16 d64")


# ------------------------------------------------------------------ bf16, matrix-core kernels
SMALL_MFMA = [
    dict(chunk_lens=(64, 64), q_len=64, prefix_len=32),                       # exact tiles
    dict(chunk_lens=(100, 1, 65, 300, 31), q_len=50, prefix_len=7, k_scale=1.0),   # ragged everything, peaky scores
    dict(chunk_lens=(130,), q_len=1, prefix_len=0, decode_steps=3),           # no prefix, single row
    dict(chunk_lens=(), q_len=70, prefix_len=40),                             # no context
    dict(chunk_lens=(257, 255), q_len=96, prefix_len=32, n_q_heads=8, n_kv_heads=8),    # G = 1
    dict(chunk_lens=(257, 255), q_len=33, prefix_len=32, n_q_heads=16, n_kv_heads=8),   # G = 2
    dict(chunk_lens=(200, 90), q_len=40, prefix_len=5, n_q_heads=16, n_kv_heads=2),     # G = 8
    dict(chunk_lens=(512,) * 3, q_len=130, prefix_len=32, decode_steps=70, k_scale=1.0),   # several q tiles, long self
]


@pytest.mark.parametrize("kw", SMALL_MFMA, ids=[str(i) for i in range(len(SMALL_MFMA))])
def test_bf16_mfma_small_shapes(kw):
    kw = dict(kw)
    spec = W.CONFIGS[2].replace(decode_steps=kw.pop("decode_steps", 5), **kw)
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    what = "mfma %s" % (kw,)
    if spec.chunk_lens:
        _check_encode(spec, r, h, what=what)
    _check_query(spec, r, h, spec.q_len, spec.q_len, what=what)
    # query rows in the middle of a longer self KV (chunked prefill of the query)
    if spec.q_len > 8:
        _check_query(spec, r, h, spec.q_len - 7, spec.q_len, what=what + " offset")
    for sl in {spec.q_len + 1, spec.self_len_max}:
        _check_decode(spec, r, h, sl, what=what)


def test_cfg2_rag_bf16_all_rows():
    spec = W.CONFIGS[2]
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    _check_encode(spec, r, h, what="cfg2")
    _check_query(spec, r, h, spec.q_len, spec.q_len, what="cfg2")
    for step in sorted({*range(0, 256, 15), 1, 255}):      # 19 of the 256 decode steps, spread over the run
        _check_decode(spec, r, h, spec.q_len + step + 1, what="cfg2 step %d" % step)


@pytest.mark.parametrize("n_chunks, chunk_len, hq, hkv", [(300, 100, 16, 2), (700, 33, 32, 8), (129, 1024, 8, 8)])
def test_many_short_chunks_of_one_length_all_rows(n_chunks, chunk_len, hq, hkv):
    """Many short chunks of one length: the encode then runs resident workgroups that each walk
    several tiles in a fixed deal (rounds that do not fill up, teams that pad the grid, 1, 4 and 8
    heads per KV head): every row against the oracle."""
    spec = W.CONFIGS[2].replace(chunk_lens=(chunk_len,) * n_chunks, n_q_heads=hq, n_kv_heads=hkv, q_len=8, decode_steps=0,
                                prefix_len=19, k_scale=1.0)
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    _check_encode(spec, r, h, what="%d x %d" % (n_chunks, chunk_len))


def test_cfg2_generic_path_agrees():
    """The portable kernels on the same bf16 workload (cross-check of the two GPU paths through
    the oracle, each to the bf16 tolerance)."""
    spec = W.CONFIGS[2].replace(chunk_lens=(512,) * 4, q_len=32)
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    _check_encode(spec, r, h, generic=True, what="cfg2 generic")
    _check_query(spec, r, h, spec.q_len, spec.q_len, generic=True, what="cfg2 generic")
    _check_decode(spec, r, h, spec.q_len + 3, generic=True, what="cfg2 generic")


def test_values_all_ones_rows_sum_to_one():
    """Rows of Eq.5 sum to 1: with all-ones values the output is all-ones (holds at any size)."""
    spec = W.CONFIGS[2].replace(chunk_lens=(512,) * 8, q_len=64)
    r = W.make_request(spec, DEV)
    for name in ("v_prefix", "v_ctx", "v_self"):
        getattr(r, name).fill_(1.0)
    out, _ = H.run_prefill(spec, r, spec.q_len, spec.q_len)
    assert (H.f64(out) - 1.0).__abs__().max() <= 2 ** -8          # one bf16 ulp at 1.0
    out, _ = H.run_decode(spec, [r], [spec.q_len + 1])
    assert (H.f64(out) - 1.0).__abs__().max() <= 2 ** -8
    o_ctx, _, o_p, _ = H.run_encode(spec, r)
    assert (H.f64(o_ctx) - 1.0).__abs__().max() <= 2 ** -8
    assert (H.f64(o_p) - 1.0).__abs__().max() <= 2 ** -8


def test_late_outlier_keys_move_the_softmax_reference():
    """The flash kernels keep a lazily updated softmax reference and take a rare path when a score
    exceeds it by more than 2^40.  Keys planted deep inside long segments, aligned with one query
    each so that their scores tower over everything before them, force that path in the middle
    of a stretch of full blocks (context chunk, own chunk of the encode, self segment)."""
    spec = W.CONFIGS[2].replace(chunk_lens=(1024, 700), q_len=64, prefix_len=32, decode_steps=5)
    r = W.make_request(spec, DEV)
    g = spec.n_q_heads // spec.n_kv_heads
    for hk in range(spec.n_kv_heads):
        r.k_ctx[600 + hk, hk] = 6.0 * r.q_self[5 + hk, hk * g]            # prefill row 5+hk, chunk 0, block 18
        r.k_ctx[1024 + 650, hk] = 6.0 * r.q_self[40, hk * g + g - 1]      # chunk 1
        r.k_ctx[900, hk] = 5.0 * r.q_ctx[950, hk * g + 1]                 # encode: row 950 of chunk 0 sees token 900 (diagonal tile)
        r.k_ctx[500, hk] = 5.0 * r.q_ctx[1000, hk * g + 2]                # ... and row 1000 token 500 (deep inside the stretch)
        r.k_self[33, hk] = 6.0 * r.q_self[60, hk * g]                     # self segment, second block
    h = H.HostArrays(r)
    _check_encode(spec, r, h, what="outliers")
    _check_query(spec, r, h, spec.q_len, spec.q_len, what="outliers")
    _check_decode(spec, r, h, spec.q_len + 1, what="outliers")
    # the planted keys really are beyond the lazy threshold (2^40 ~ 27.7 in natural-log units)
    qk = (r.q_self[5].float()[0] * r.k_ctx[600, 0].float()).sum().item() / spec.head_dim ** 0.5 / r.temperature
    assert qk > 40.0


def test_chunk_table_order_and_separate_buffers():
    """Contexts live in separately allocated buffers reached through the table; permuting the
    table leaves the result unchanged within tolerance (Eq.5 is a sum over contexts)."""
    spec = W.CONFIGS[2].replace(chunk_lens=(300, 512, 64, 700, 129), q_len=48)
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    ref, _, _ = H.oracle_prefill(h, spec.q_len, spec.q_len, r.temperature, r.scale)
    for order in (None, [3, 0, 4, 2, 1]):
        req = H.make_binding_request(r, spec.q_len, separate_buffers=True, order=order)
        out, _ = H.run_prefill(spec, r, spec.q_len, spec.q_len, req=req)
        H.check_close(H.f64(out).reshape(-1, spec.head_dim), ref, "bf16", "order %s" % (order,))
        reqd = H.make_binding_request(r, spec.q_len + 2, separate_buffers=True, order=order)
        outd, _ = H.run_decode(spec, [r], [spec.q_len + 2], reqs=[reqd])
        refd, _, _ = H.oracle_prefill(h, 1, spec.q_len + 2, r.temperature, r.scale)
        H.check_close(H.f64(outd).reshape(-1, spec.head_dim), refd, "bf16", "decode order %s" % (order,))


@pytest.mark.parametrize("batch", [35, 16, 2])
def test_batched_decode_mixed_requests(batch):
    """Requests of different context sizes, T and S in one decode call: more than one launch's
    worth of descriptors (35), and batches whose split plan differs (the number of context splits
    depends on the batch; the shorter requests leave some of them empty)."""
    base = W.CONFIGS[5].replace(batch=batch, decode_steps=9)
    rs, hs, lens = [], [], []
    for b in range(base.batch):
        n_chunks = 1 + b % 4
        spec = base.replace(chunk_lens=tuple(64 + 37 * ((b + i) % 5) for i in range(n_chunks)), prefix_len=(b % 3) * 16)
        r = W.make_request(spec, DEV, request=b)
        rs.append(r); hs.append(H.HostArrays(r)); lens.append(1 + b % 9)
    out, lse = H.run_decode(base, rs, lens)
    for b, (r, h) in enumerate(zip(rs, hs)):
        ref, ref_lse, _ = H.oracle_prefill(h, 1, lens[b], r.temperature, r.scale)
        H.check_close(H.f64(out[b]), ref, "bf16", "request %d" % b)
        assert np.abs(H.f64(lse[b]) - ref_lse).max() <= H.lse_tol("bf16")


def test_errors_leave_outputs_untouched():
    spec = W.CONFIGS[2].replace(chunk_lens=(64,), q_len=8)
    r = W.make_request(spec, DEV)
    shape = B.make_shape(spec.n_q_heads, spec.n_kv_heads, spec.head_dim, spec.torch_dtype)
    req = H.make_binding_request(r, spec.q_len)
    q = r.q_self[:spec.q_len].contiguous()
    out = torch.full_like(q, 7.0)
    small = torch.zeros(64, dtype=torch.float32, device=DEV)
    with pytest.raises(B.ApeError) as e:
        B.attention_prefill(shape, req, q, out, None, small)
    assert e.value.status == B.APE_ERR_WORKSPACE
    req.temperature = 0.0
    ws = H.poisoned_workspace(B.workspace_bytes(B.APE_OP_PREFILL, shape, 1, spec.q_len), DEV)
    with pytest.raises(B.ApeError) as e:
        B.attention_prefill(shape, req, q, out, None, ws)
    assert e.value.status == B.APE_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert (out == 7.0).all()


# ------------------------------------------------------------------ batched query prefill
def _check_prefill_batch(specs, q_len, self_lens, generic=False, what=""):
    rs = [W.make_request(sp, DEV, request=b) for b, sp in enumerate(specs)]
    sp0 = specs[0]
    shape = B.make_shape(sp0.n_q_heads, sp0.n_kv_heads, sp0.head_dim, sp0.torch_dtype, generic=generic)
    reqs = [H.make_binding_request(r, sl) for r, sl in zip(rs, self_lens)]
    q = torch.stack([r.q_self[sl - q_len:sl] for r, sl in zip(rs, self_lens)]).contiguous()
    out = torch.full_like(q, float("nan"))
    lse = torch.full((len(rs), sp0.n_q_heads, q_len), float("nan"), dtype=torch.float32, device=DEV)
    ws = H.poisoned_workspace(B.workspace_bytes(B.APE_OP_PREFILL, shape, len(rs), q_len), DEV)
    B.attention_prefill_batch(shape, reqs, q, out, lse, ws, self_lens=list(self_lens))
    torch.cuda.synchronize()
    for b, (r, sl) in enumerate(zip(rs, self_lens)):
        h = H.HostArrays(r)
        ref, ref_lse, _ = H.oracle_prefill(h, q_len, sl, r.temperature, r.scale)
        H.check_close(H.f64(out[b]).reshape(-1, sp0.head_dim), ref, sp0.dtype, "%s request %d" % (what, b))
        assert np.abs(H.f64(lse[b]).T.reshape(-1) - ref_lse).max() <= H.lse_tol(sp0.dtype), "%s request %d lse" % (what, b)


def test_batched_prefill_mixed_requests_bf16():
    """Four requests in one call: different numbers and lengths of contexts (one without any),
    prefix lengths, self lengths, T and S; the shorter contexts leave trailing splits unwritten."""
    base = W.CONFIGS[2].replace(temperature=None, scale=None, decode_steps=40)
    specs = [base.replace(chunk_lens=(512,) * 6, q_len=48),
             base.replace(chunk_lens=(100, 1, 65, 300, 31), q_len=48, prefix_len=7),
             base.replace(chunk_lens=(), q_len=48),
             base.replace(chunk_lens=(2000,), q_len=48, prefix_len=0)]
    _check_prefill_batch(specs, 48, [48, 60, 48, 88], what="bf16 batch")
    _check_prefill_batch(specs[:2], 33, [33, 70], what="bf16 batch of 2")
    _check_prefill_batch(specs, 48, [48, 60, 48, 88], generic=True, what="bf16 generic batch")


def test_batched_prefill_fp32_and_more_than_one_launch():
    base = W.CONFIGS[1].replace(temperature=None, scale=None)
    specs = [base.replace(chunk_lens=tuple(5 + (3 * b + i) % 29 for i in range(1 + b % 4))) for b in range(35)]   # > 32 requests
    _check_prefill_batch(specs, 6, [6 + b % 5 for b in range(35)], what="fp32 batch of 35")


# ------------------------------------------------------------------ paged caches
def test_paged_cache_is_a_chunk_table_of_pages():
    """A paged KV cache needs no entry point of its own: under the pooled scaling factor the
    chunk table may just as well list PAGES (here 64-token pages scattered over separate
    buffers, the last page of a context partly filled), and under the tree entry point a node per
    context lists that context's pages, which merge exactly.  Both must match the oracle run on
    the unpaged contexts."""
    spec = W.CONFIGS[2].replace(chunk_lens=(300, 64, 513, 100), q_len=40, decode_steps=6)
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    page = 64
    ks, vs = r.chunk_views()
    k_pages, v_pages, pages_of = [], [], []
    for k, v in zip(ks, vs):
        first = len(k_pages)
        for p0 in range(0, k.shape[0], page):
            k_pages.append(k[p0:p0 + page].clone())
            v_pages.append(v[p0:p0 + page].clone())
        pages_of.append((first, len(k_pages) - first))
    order = list(range(len(k_pages)))[::-1]                # the table need not follow allocation order ...
    req = B.Request(r.k_prefix, r.v_prefix, [k_pages[i] for i in order], [v_pages[i] for i in order],
                    r.k_self, r.v_self, spec.q_len, r.temperature, r.scale)
    _check_query(spec, r, h, spec.q_len, spec.q_len, req=req, what="pages, pooled")
    # ... but a tree node owns a run of consecutive table entries: table in context order here
    req = B.Request(r.k_prefix, r.v_prefix, k_pages, v_pages, r.k_self, r.v_self, spec.q_len, r.temperature, r.scale)
    nodes = [(1.0, 1, len(pages_of), False)] + [(0.85, first, n, True) for first, n in pages_of]
    shape = B.make_shape(spec.n_q_heads, spec.n_kv_heads, spec.head_dim, spec.torch_dtype)
    tree = B.make_tree(nodes, DEV)
    for q_len, sl in ((spec.q_len, spec.q_len), (1, spec.self_len_max)):
        q = r.q_self[sl - q_len:sl].contiguous()
        out = torch.full_like(q, float("nan"))
        ws = H.poisoned_workspace(B.tree_workspace_bytes(shape, spec.total_ctx_len, len(nodes), q_len), DEV)
        B.attention_tree(shape, req, tree, q, out, None, ws, self_len=sl)
        torch.cuda.synchronize()
        ref, _ = H.oracle_tree(h, q_len, sl, r.temperature, W.tree_per_context(4, 0.85))
        H.check_close(H.f64(out).reshape(-1, spec.head_dim), ref, "bf16", "pages under one node per context, q_len %d" % q_len)


# ------------------------------------------------------------------ the ends of the paper's hyper-parameter grid
@pytest.mark.parametrize("T,S", [(0.1, 0.1), (0.1, 1.0), (1.0, 0.1), (0.5, 0.5)])
def test_hyperparameter_grid_corners(T, S):
    """The paper searches T and S over [0.1, 1.0] (end of Section 4.4).  T = 0.1 multiplies the
    context scores by ten (standard deviation ~10 here: probabilities spanning e^60 within a row),
    S = 0.1 all but removes the context mass.  Prefill, decode and the tree entry point, bf16
    matrix-core path and fp32 path."""
    spec = W.CONFIGS[2].replace(chunk_lens=(512, 300, 1, 700), q_len=40, decode_steps=4, k_scale=1.0, temperature=T, scale=S)
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    _check_query(spec, r, h, spec.q_len, spec.q_len, what="bf16 T=%g S=%g" % (T, S))
    _check_decode(spec, r, h, spec.self_len_max, what="bf16 T=%g S=%g" % (T, S))
    out, _ = H.run_tree(spec, r, W.tree_per_context(4, S), spec.q_len, spec.q_len)
    ref, _ = H.oracle_tree(h, spec.q_len, spec.q_len, T, W.tree_per_context(4, S))
    H.check_close(H.f64(out).reshape(-1, spec.head_dim), ref, "bf16", "tree T=%g S=%g" % (T, S))
    # fp32: a score of magnitude |s| carries an absolute rounding error of a few |s| * 6e-8, which is the
    # relative error of its probability; N(0,1) inputs at T = 0.1 give |s| up to ~40, still inside 1e-5
    spec1 = W.CONFIGS[1].replace(temperature=T, scale=S, rope_base=None)
    r1 = W.make_request(spec1, DEV)
    h1 = H.HostArrays(r1)
    _check_query(spec1, r1, h1, spec1.q_len, spec1.q_len, what="fp32 T=%g S=%g" % (T, S))
    _check_decode(spec1, r1, h1, spec1.self_len_max, what="fp32 T=%g S=%g" % (T, S))


# ------------------------------------------------------------------ short chunks
@pytest.mark.parametrize("kw", [
    dict(chunk_lens=(256,) * 5, prefix_len=32),                                   # the many-shot shape
    dict(chunk_lens=(256, 1, 33, 64, 255, 129, 200, 97), prefix_len=7),           # ragged, partial last blocks
    dict(chunk_lens=(288, 40, 65), prefix_len=0),                                 # no prefix: nine chunk blocks
    dict(chunk_lens=(224, 100), prefix_len=64),                                   # two prefix blocks
    dict(chunk_lens=(250, 130), prefix_len=32, n_q_heads=8, n_kv_heads=8),        # G = 1
    dict(chunk_lens=(250, 130), prefix_len=32, n_q_heads=16, n_kv_heads=8),       # G = 2
    dict(chunk_lens=(250, 60), prefix_len=5, n_q_heads=16, n_kv_heads=2),         # G = 8
], ids=lambda kw: "x".join(str(v) for v in kw["chunk_lens"][:3]) + "_p%d" % kw["prefix_len"])
def test_bf16_encode_short_chunks(kw):
    """Many-shot shapes: streams of two to ten blocks per query tile, where every body is a generic
    one (block tails, the causal diagonal) and the ring never wraps."""
    spec = W.CONFIGS[2].replace(q_len=8, decode_steps=0, **kw)
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    _check_encode(spec, r, h, what="short chunks %s" % (kw,))
