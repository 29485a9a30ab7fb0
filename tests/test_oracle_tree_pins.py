"""Pins of the tree-merge oracle (Appendix C.2 applied per node, Appendix C.5 of arXiv 2502.05431).

Each test checks the recursive oracle against something that is not that recursion: the weights
form of the main-text equation, a library softmax, products of raw partition sums written out by
hand for a fixed tree, or an invariant of the definition.
"""
import numpy as np
import pytest
import scipy.special

from oracle import ape_oracle
from paper_2502_05431_amd import workloads as W


def tiny(chunk_lens=(32,) * 4, **kw):
    spec = W.CONFIGS[1].replace(chunk_lens=tuple(chunk_lens), **kw)
    r = W.make_request(spec, "cpu")
    a = {k: W.to_numpy_f32(getattr(r, k)) for k in ("k_prefix", "v_prefix", "k_ctx", "v_ctx", "q_self", "k_self", "v_self")}
    return spec, a


def tree_attention(a, lens, q_len, self_len, T, nodes, pairs=None, v_ctx=None):
    return ape_oracle.attention_tree(a["q_self"][self_len - q_len:self_len], a["k_prefix"], a["v_prefix"],
                                     a["k_ctx"], a["v_ctx"] if v_ctx is None else v_ctx, lens,
                                     a["k_self"][:self_len], a["v_self"][:self_len], T, nodes, pairs=pairs)


def flat_attention(a, lens, q_len, self_len, T, S, form):
    return ape_oracle.attention(a["q_self"][self_len - q_len:self_len], a["k_prefix"], a["v_prefix"],
                                a["k_ctx"], a["v_ctx"], lens, a["k_self"][:self_len], a["v_self"][:self_len],
                                T, S, form=form)


# ---------------------------------------------------------------- T1
def test_single_node_tree_is_the_main_text_equation():
    """A root with scale S over all contexts pools them before S is applied: Section 4.4."""
    spec, a = tiny()
    lens = list(spec.chunk_lens)
    o, l = tree_attention(a, lens, spec.q_len, spec.q_len, 0.8, W.tree_pooled(len(lens), 0.9))
    ow, lw, _ = flat_attention(a, lens, spec.q_len, spec.q_len, 0.8, 0.9, "weights")
    np.testing.assert_allclose(o, ow, atol=1e-12)
    np.testing.assert_allclose(l, lw, atol=1e-12)


# ---------------------------------------------------------------- T2
def test_one_node_per_context_is_appendix_c2():
    spec, a = tiny((32, 17, 40, 5))
    lens = list(spec.chunk_lens)
    o, l = tree_attention(a, lens, spec.q_len, spec.q_len, 0.8, W.tree_per_context(len(lens), 0.9))
    oc, lc, _ = flat_attention(a, lens, spec.q_len, spec.q_len, 0.8, 0.9, "hier_per_context")
    np.testing.assert_allclose(o, oc, atol=1e-12)
    np.testing.assert_allclose(l, lc, atol=1e-12)


# ---------------------------------------------------------------- T3
@pytest.mark.parametrize("seed", [1, 2, 3])
def test_all_scales_one_is_one_softmax_whatever_the_tree(seed):
    """With S_n = 1 everywhere every merge is exact (Appendix C.1): the result is a single softmax
    over prefix, contexts (scores over T) and self, for any tree shape."""
    spec, a = tiny((8, 3, 21, 16, 9, 1, 30))
    lens = list(spec.chunk_lens)
    nodes = [(1.0, f, c, leaf) for (_, f, c, leaf) in W.tree_random(len(lens), seed)]
    T, q_len, d = 0.7, spec.q_len, spec.head_dim
    o, l = tree_attention(a, lens, q_len, q_len, T, nodes)
    g = spec.n_q_heads // spec.n_kv_heads
    for r in range(q_len):
        for h in range(spec.n_q_heads):
            hk = h // g
            q = a["q_self"][r, h].astype(np.float64)
            sp = a["k_prefix"][:, hk].astype(np.float64) @ q / np.sqrt(d)
            sc = a["k_ctx"][:, hk].astype(np.float64) @ q / np.sqrt(d) / T
            ss = a["k_self"][:r + 1, hk].astype(np.float64) @ q / np.sqrt(d)
            w = scipy.special.softmax(np.concatenate([sp, sc, ss]))
            v = np.concatenate([a["v_prefix"][:, hk], a["v_ctx"][:, hk], a["v_self"][:r + 1, hk]]).astype(np.float64)
            np.testing.assert_allclose(o[r * spec.n_q_heads + h], w @ v, atol=1e-12)
            np.testing.assert_allclose(l[r * spec.n_q_heads + h], scipy.special.logsumexp(np.concatenate([sp, sc, ss])), atol=1e-12)


# ---------------------------------------------------------------- T4
def test_three_level_tree_against_products_of_raw_partition_sums():
    """A fixed tree, every weight written out by hand with raw exp and ** (no LogSumExp, no
    recursion):   root(S0) -> A(S1: ctx 0,1), B(S2: ctx 2), C(S3) -> D(S4: ctx 3), E(S5: ctx 4,5)."""
    S0, S1, S2, S3, S4, S5 = 0.9, 0.8, 0.7, 0.85, 0.6, 0.95
    lens = [12, 7, 20, 9, 4, 15]
    spec, a = tiny(lens, k_scale=0.5)
    nodes = [(S0, 1, 3, False), (S1, 0, 2, True), (S2, 2, 1, True), (S3, 4, 2, False),
             (S4, 3, 1, True), (S5, 4, 2, True)]
    T, q_len, d = 0.8, spec.q_len, spec.head_dim
    o, l = tree_attention(a, lens, q_len, q_len, T, nodes)
    cu = np.concatenate([[0], np.cumsum(lens)])
    g = spec.n_q_heads // spec.n_kv_heads
    for r in (0, 5, q_len - 1):
        for h in range(spec.n_q_heads):
            hk = h // g
            q = a["q_self"][r, h].astype(np.float64)
            ac = np.exp(a["k_ctx"][:, hk].astype(np.float64) @ q / (T * np.sqrt(d)))
            ao = np.exp(np.concatenate([a["k_prefix"][:, hk], a["k_self"][:r + 1, hk]]).astype(np.float64) @ q / np.sqrt(d))
            Z = [ac[cu[i]:cu[i + 1]].sum() for i in range(6)]
            ZA, ZB = (Z[0] + Z[1]) ** S1, Z[2] ** S2
            ZD, ZE = Z[3] ** S4, (Z[4] + Z[5]) ** S5
            ZC = (ZD + ZE) ** S3
            ZR = (ZA + ZB + ZC) ** S0
            D = ZR + ao.sum()
            node_w = {0: ZA / (ZA + ZB + ZC) / (Z[0] + Z[1]), 1: ZA / (ZA + ZB + ZC) / (Z[0] + Z[1]),
                      2: ZB / (ZA + ZB + ZC) / Z[2],
                      3: ZC / (ZA + ZB + ZC) * ZD / (ZD + ZE) / Z[3],
                      4: ZC / (ZA + ZB + ZC) * ZE / (ZD + ZE) / (Z[4] + Z[5]),
                      5: ZC / (ZA + ZB + ZC) * ZE / (ZD + ZE) / (Z[4] + Z[5])}
            wc = np.concatenate([ac[cu[i]:cu[i + 1]] * node_w[i] * ZR / D for i in range(6)])
            wo = ao / D
            assert abs(wc.sum() + wo.sum() - 1.0) < 1e-12
            vo = np.concatenate([a["v_prefix"][:, hk], a["v_self"][:r + 1, hk]]).astype(np.float64)
            ref = wc @ a["v_ctx"][:, hk].astype(np.float64) + wo @ vo
            np.testing.assert_allclose(o[r * spec.n_q_heads + h], ref, atol=1e-12)
            np.testing.assert_allclose(l[r * spec.n_q_heads + h], np.log(D), atol=1e-12)


# ---------------------------------------------------------------- T5
def test_scale_one_wrappers_and_sibling_order_change_nothing():
    lens = [12, 7, 20, 9]
    spec, a = tiny(lens)
    base = [(0.9, 1, 2, False), (0.8, 0, 2, True), (0.7, 2, 2, True)]
    o, l = tree_attention(a, lens, spec.q_len, spec.q_len, 0.8, base)
    # a scale-1 node between the root and each child
    wrapped = [(0.9, 1, 2, False), (1.0, 3, 1, False), (1.0, 4, 1, False), (0.8, 0, 2, True), (0.7, 2, 2, True)]
    o2, l2 = tree_attention(a, lens, spec.q_len, spec.q_len, 0.8, wrapped)
    np.testing.assert_allclose(o2, o, atol=1e-12)
    np.testing.assert_allclose(l2, l, atol=1e-12)
    # the two subtrees swapped, the chunk table left alone
    swapped = [(0.9, 1, 2, False), (0.7, 2, 2, True), (0.8, 0, 2, True)]
    o3, l3 = tree_attention(a, lens, spec.q_len, spec.q_len, 0.8, swapped)
    np.testing.assert_allclose(o3, o, atol=1e-12)
    np.testing.assert_allclose(l3, l, atol=1e-12)


# ---------------------------------------------------------------- T6
def test_one_hot_values_expose_each_context_share():
    """With value = indicator of the owning context the output lists the mass of each context;
    under a shared parent two contexts split that parent's mass in the ratio of their Z."""
    lens = [10, 10, 10]
    spec, a = tiny(lens, head_dim=64)
    v = np.zeros_like(a["v_ctx"])
    for i in range(3):
        v[10 * i:10 * (i + 1), :, i] = 1.0
    nodes = [(0.9, 1, 2, False), (0.5, 0, 2, True), (0.5, 2, 1, True)]
    T = 0.8
    a = dict(a, v_prefix=np.zeros_like(a["v_prefix"]), v_self=np.zeros_like(a["v_self"]))
    o, _ = tree_attention(a, lens, 1, 1, T, nodes, v_ctx=v)
    g = spec.n_q_heads // spec.n_kv_heads
    for h in range(spec.n_q_heads):
        q = a["q_self"][0, h].astype(np.float64)
        z = [np.exp(a["k_ctx"][10 * i:10 * (i + 1), h // g].astype(np.float64) @ q / (T * 8.0)).sum() for i in range(3)]
        np.testing.assert_allclose(o[h, 0] / o[h, 1], z[0] / z[1], rtol=1e-10)
        # node masses: (Z0+Z1)^0.5 against Z2^0.5
        np.testing.assert_allclose((o[h, 0] + o[h, 1]) / o[h, 2], ((z[0] + z[1]) / z[2]) ** 0.5, rtol=1e-10)


# ---------------------------------------------------------------- T7
def test_empty_context_and_bad_trees():
    lens = [12, 0, 20]
    spec, a = tiny(lens)
    o, l = tree_attention(a, lens, 2, 2, 0.8, W.tree_per_context(3, 0.9))
    o2, l2 = ape_oracle.attention_tree(a["q_self"][:2], a["k_prefix"], a["v_prefix"], a["k_ctx"], a["v_ctx"], [12, 20],
                                       a["k_self"][:2], a["v_self"][:2], 0.8, W.tree_per_context(2, 0.9))
    assert np.isfinite(o).all()
    np.testing.assert_allclose(o, o2, atol=1e-13)
    np.testing.assert_allclose(l, l2, atol=1e-13)
    for bad in ([(0.9, 0, 1, False)],                       # a node as its own child
                [(0.9, 1, 1, False), (0.9, 0, 0, True)],    # no children
                [(0.0, 0, 3, True)],                        # scale must be > 0
                [(0.9, 0, 4, True)]):                       # context index out of range
        with pytest.raises(ValueError):
            tree_attention(a, lens, 2, 2, 0.8, bad)


# ---------------------------------------------------------------- T8
@pytest.mark.parametrize("seed", range(6))
def test_random_tree_builder_is_breadth_first_and_covers_every_context(seed):
    n = 5 + 7 * seed
    nodes = W.tree_random(n, seed)
    nxt, seen = 1, []
    for i, (s, first, count, leaf) in enumerate(nodes):
        assert s > 0 and count >= 1
        if leaf:
            seen.extend(range(first, first + count))
        else:
            assert first == nxt and first > i
            nxt += count
    assert nxt == len(nodes) and sorted(seen) == list(range(n))
