"""GPU parity of the tree entry point (a scaling factor per node of a tree of contexts:
Appendix C.2 applied per node, Appendix C.5) against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2502_05431_amd import binding as B
from paper_2502_05431_amd import workloads as W

import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _check_tree(spec, r, h, nodes, q_len, self_len, generic=False, what=""):
    out, lse = H.run_tree(spec, r, nodes, q_len, self_len, generic=generic)
    ref, ref_lse = H.oracle_tree(h, q_len, self_len, r.temperature, nodes)
    H.check_close(H.f64(out).reshape(-1, spec.head_dim), ref, spec.dtype, what + " tree out")
    got_lse = H.f64(lse).T.reshape(-1)
    assert np.abs(got_lse - ref_lse).max() <= H.lse_tol(spec.dtype), what + " tree lse"
    return out, lse


def _trees(n_chunks, S):
    yield "pooled", W.tree_pooled(n_chunks, S)
    yield "per-context", W.tree_per_context(n_chunks, S)
    if n_chunks >= 3:
        yield "grouped", W.tree_grouped(n_chunks, 2, 0.95, S)
    for seed in (11, 12):
        yield "random%d" % seed, W.tree_random(n_chunks, seed)


# ------------------------------------------------------------------ fp32, portable kernels
def test_cfg1_fp32_trees_all_rows():
    spec = W.CONFIGS[1]
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    for name, nodes in _trees(len(spec.chunk_lens), 0.9):
        _check_tree(spec, r, h, nodes, spec.q_len, spec.q_len, what="cfg1 " + name)
        _check_tree(spec, r, h, nodes, 1, spec.self_len_max, what="cfg1 decode " + name)


def test_fp32_pooled_tree_equals_the_flat_entry_point_and_per_context_does_not():
    spec = W.CONFIGS[1]
    r = W.make_request(spec, DEV)
    flat, flat_lse = H.run_prefill(spec, r, spec.q_len, spec.q_len)
    pooled, pooled_lse = H.run_tree(spec, r, W.tree_pooled(4, r.scale), spec.q_len, spec.q_len)
    per_ctx, _ = H.run_tree(spec, r, W.tree_per_context(4, r.scale), spec.q_len, spec.q_len)
    assert (flat - pooled).abs().max().item() <= 2e-6
    assert (flat_lse - pooled_lse).abs().max().item() <= 2e-5
    assert (flat - per_ctx).abs().max().item() > 1e-3


def test_fp32_ragged_contexts_empty_context_and_deep_tree():
    spec = W.CONFIGS[1].replace(chunk_lens=(33, 0, 1, 64, 7, 100, 2), q_len=9, prefix_len=0)
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    for name, nodes in _trees(7, 0.8):
        _check_tree(spec, r, h, nodes, spec.q_len, spec.q_len, what="ragged " + name)
    # a chain of single-child nodes above one node that holds everything (16 levels)
    chain = [(0.97, i + 1, 1, False) for i in range(B.APE_TREE_MAX_DEPTH - 1)] + [(0.9, 0, 7, True)]
    _check_tree(spec, r, h, chain, spec.q_len, spec.q_len, what="chain")
    # the subtrees in another order than the chunk table
    swapped = [(0.9, 1, 3, False), (0.8, 5, 2, True), (0.7, 0, 2, True), (0.85, 2, 3, True)]
    _check_tree(spec, r, h, swapped, spec.q_len, spec.q_len, what="groups out of table order")


def test_fp32_wide_levels():
    """More than 64 nodes on a level (one thread per node) next to narrow levels (one wavefront per node)."""
    n = 150
    spec = W.CONFIGS[1].replace(chunk_lens=tuple(1 + (7 * i) % 5 for i in range(n)), q_len=3)
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    _check_tree(spec, r, h, W.tree_per_context(n, 0.85), spec.q_len, spec.q_len, what="150 one-context nodes")
    _check_tree(spec, r, h, W.tree_grouped(n, 2, 0.9, 0.8), spec.q_len, spec.q_len, what="75 pairs")
    _check_tree(spec, r, h, W.tree_pooled(n, 0.85), 1, spec.self_len_max, what="one node, 150 children")
    _check_tree(spec, r, h, W.tree_random(n, 5, max_children=9), spec.q_len, spec.q_len, what="random wide")


# ------------------------------------------------------------------ bf16, matrix-core kernels
SMALL = [
    dict(chunk_lens=(64, 64), q_len=64, prefix_len=32),
    dict(chunk_lens=(100, 1, 65, 300, 31, 0, 32), q_len=50, prefix_len=7, k_scale=1.0),
    dict(chunk_lens=(130,), q_len=1, prefix_len=0),
    dict(chunk_lens=(257, 255, 3), q_len=96, prefix_len=32, n_q_heads=8, n_kv_heads=8),
    dict(chunk_lens=(200, 90, 64), q_len=40, prefix_len=5, n_q_heads=16, n_kv_heads=2),
    dict(chunk_lens=(3000, 2500), q_len=130, prefix_len=32, k_scale=1.0),      # few long contexts: several splits each
    dict(chunk_lens=(700, 5, 1200, 64, 900, 33, 2048, 1), q_len=17, prefix_len=32),   # very unequal groups
]


@pytest.mark.parametrize("kw", SMALL, ids=[str(i) for i in range(len(SMALL))])
def test_bf16_mfma_trees_small_shapes(kw):
    spec = W.CONFIGS[2].replace(decode_steps=5, **kw)
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    for name, nodes in _trees(len(spec.chunk_lens), 0.85):
        what = "mfma %s %s" % (kw, name)
        _check_tree(spec, r, h, nodes, spec.q_len, spec.q_len, what=what)
        _check_tree(spec, r, h, nodes, 1, spec.self_len_max, what=what + " decode")


def test_bf16_generic_path_trees():
    spec = W.CONFIGS[2].replace(chunk_lens=(100, 1, 65, 300), q_len=20, decode_steps=3)
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    for name, nodes in _trees(4, 0.85):
        _check_tree(spec, r, h, nodes, spec.q_len, spec.q_len, generic=True, what="generic " + name)


def test_bf16_pooled_tree_agrees_with_the_flat_entry_point():
    spec = W.CONFIGS[2]
    r = W.make_request(spec, DEV)
    flat, flat_lse = H.run_prefill(spec, r, spec.q_len, spec.q_len)
    pooled, pooled_lse = H.run_tree(spec, r, W.tree_pooled(len(spec.chunk_lens), r.scale), spec.q_len, spec.q_len)
    # same arithmetic per block, different cuts of the contexts: equal to bf16 output rounding
    assert (flat.float() - pooled.float()).abs().max().item() <= 2 ** -7
    assert (flat_lse - pooled_lse).abs().max().item() <= 1e-4


# ------------------------------------------------------------------ full benchmark sizes, sampled
def _pairs(rng, n_rows, n_heads, n, must_rows=()):
    rows = {0, n_rows - 1, *[x for x in must_rows if 0 <= x < n_rows]}
    pairs = [(x, hd) for x in sorted(rows) for hd in (0, n_heads - 1)]
    while len(pairs) < n:
        pairs.append((int(rng.integers(n_rows)), int(rng.integers(n_heads))))
    return pairs


def _check_sampled(spec, r, h, nodes, q_len, self_len, pairs, what):
    out, lse = H.run_tree(spec, r, nodes, q_len, self_len)
    ref, ref_lse = H.oracle_tree(h, q_len, self_len, r.temperature, nodes, pairs=pairs)
    got = np.stack([out[x, hd].float().cpu().numpy().astype(np.float64) for x, hd in pairs])
    H.check_close(got, ref, "bf16", what)
    got_lse = np.array([float(lse[hd, x]) for x, hd in pairs])
    assert np.abs(got_lse - ref_lse).max() <= H.lse_tol("bf16"), what + " lse"
    assert torch.isfinite(out.float()).all()


def test_cfg3_128k_scaling_factor_per_context_sampled():
    spec = W.CONFIGS[3]
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    rng = np.random.default_rng(33)
    pairs = _pairs(rng, spec.q_len, spec.n_q_heads, 256, must_rows=(63, 64, 127, 128))
    _check_sampled(spec, r, h, W.tree_per_context(64, r.scale), spec.q_len, spec.q_len, pairs, "cfg3 per-context S")


def test_cfg4_manyshot_two_level_tree_sampled():
    spec = W.CONFIGS[4]
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    rng = np.random.default_rng(44)
    nodes = W.tree_grouped(512, 8, 0.9, r.scale)           # 64 groups of 8 demonstrations
    pairs = _pairs(rng, spec.q_len, spec.n_q_heads, 128, must_rows=(31, 32))
    _check_sampled(spec, r, h, nodes, spec.q_len, spec.q_len, pairs, "cfg4 grouped prefill")
    sl = spec.q_len + 7
    pairs = [(0, hd) for hd in range(spec.n_q_heads)]
    _check_sampled(spec, r, h, nodes, 1, sl, pairs, "cfg4 grouped decode")
    _check_sampled(spec, r, h, W.tree_per_context(512, r.scale), 1, sl, pairs, "cfg4 per-context decode")


def test_contexts_that_are_all_empty():
    """A chunk table whose contexts hold no token at all: plain causal attention over prefix + self,
    through the flat and the tree entry points (a tree whose every node is empty has weight zero)."""
    for dtype, cfg in (("bf16", 2), ("f32", 1)):
        spec = W.CONFIGS[cfg].replace(chunk_lens=(0, 0, 0), q_len=12, decode_steps=2)
        r = W.make_request(spec, DEV)
        h = H.HostArrays(r)
        ref, _, _ = H.oracle_prefill(h, spec.q_len, spec.q_len, r.temperature, r.scale)
        dummy = torch.zeros((1, spec.n_kv_heads, spec.head_dim), dtype=spec.torch_dtype, device=DEV)
        req = B.Request(r.k_prefix, r.v_prefix, [dummy[:0]] * 3, [dummy[:0]] * 3, r.k_self, r.v_self, spec.q_len,
                        r.temperature, r.scale)
        out, _ = H.run_prefill(spec, r, spec.q_len, spec.q_len, req=req)
        H.check_close(H.f64(out).reshape(-1, spec.head_dim), ref, dtype, "flat, empty contexts")
        for nodes in (W.tree_pooled(3, 0.9), W.tree_per_context(3, 0.9)):
            out, _ = H.run_tree(spec, r, nodes, spec.q_len, spec.q_len, req=req)
            H.check_close(H.f64(out).reshape(-1, spec.head_dim), ref, dtype, "tree, empty contexts")
            out, _ = H.run_tree(spec, r, nodes, 1, spec.q_len + 1, req=req)
            refd, _, _ = H.oracle_prefill(h, 1, spec.q_len + 1, r.temperature, r.scale)
            H.check_close(H.f64(out).reshape(-1, spec.head_dim), refd, dtype, "tree decode, empty contexts")


def test_tree_at_its_size_limits():
    """The largest tree the entry point takes: 2048 nodes (a root over 2047 one-context nodes), and a
    chain of the maximum depth above a node with 300 contexts."""
    n = B.APE_TREE_MAX_NODES - 1
    spec = W.CONFIGS[1].replace(chunk_lens=tuple(1 + i % 3 for i in range(n)), q_len=2, decode_steps=1)
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    nodes = W.tree_per_context(n, 0.9)
    assert len(nodes) == B.APE_TREE_MAX_NODES
    _check_tree(spec, r, h, nodes, spec.q_len, spec.q_len, what="2048 nodes, fp32")
    spec = W.CONFIGS[2].replace(chunk_lens=tuple(1 + i % 3 for i in range(n)), q_len=1, decode_steps=1, k_scale=1.0)
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    _check_tree(spec, r, h, nodes, 1, 2, what="2048 nodes, bf16 decode")
    _check_tree(spec, r, h, nodes, 1, 1, what="2048 nodes, bf16 one row")
    spec = W.CONFIGS[2].replace(chunk_lens=(40,) * 300, q_len=33, decode_steps=0)
    r = W.make_request(spec, DEV)
    h = H.HostArrays(r)
    chain = [(0.97, i + 1, 1, False) for i in range(B.APE_TREE_MAX_DEPTH - 1)] + [(0.9, 0, 300, True)]
    _check_tree(spec, r, h, chain, spec.q_len, spec.q_len, what="depth 16 over 300 contexts")
