"""Randomised checks of the host-side logic of the C-ABI library (no GPU): the tree validator
against an independent Python statement of the numbering rules, and the workspace sizes against
what the calls themselves demand."""
import ctypes
import random

import pytest

from paper_2502_05431_amd import binding as B
from paper_2502_05431_amd import workloads as W

FAKE = 0x1000


def _valid_tree(nodes, n_chunks):
    """The numbering rules of ape_tree_node, restated: breadth-first child ranges, every context
    owned exactly once, at most APE_TREE_MAX_DEPTH levels."""
    if not nodes or len(nodes) > B.APE_TREE_MAX_NODES or not 1 <= n_chunks <= B.APE_TREE_MAX_CONTEXTS:
        return False
    owned, nxt = [0] * n_chunks, 1
    for s, first, count, leaf in nodes:
        if not (s > 0 and s != float("inf")) or count < 1:
            return False
        if leaf:
            if first < 0 or first + count > n_chunks:
                return False
            for c in range(first, first + count):
                owned[c] += 1
        else:
            if first != nxt:
                return False
            nxt += count
            if nxt > len(nodes):
                return False
    if nxt != len(nodes) or any(o != 1 for o in owned):
        return False
    level, depth = [0], 1
    while True:
        kids = [c for n in level if not nodes[n][3] for c in range(nodes[n][1], nodes[n][1] + nodes[n][2])]
        if not kids:
            return depth <= B.APE_TREE_MAX_DEPTH
        level, depth = kids, depth + 1


def _call_tree(nodes, n_chunks, total_ctx=4096, q_len=4):
    sh = B.make_shape(32, 8, 128, B.APE_BF16)
    arr = (B.ApeTreeNode * max(len(nodes), 1))(*[B.ApeTreeNode(float(s), f, c, 1 if leaf else 0) for s, f, c, leaf in nodes])
    r = B.ApeRequest()
    r.k_prefix = FAKE; r.v_prefix = FAKE; r.prefix_len = 4; r.n_chunks = n_chunks
    r.k_chunks = FAKE; r.v_chunks = FAKE; r.cu_chunk_lens = FAKE; r.total_ctx_len = total_ctx
    r.self_len = q_len; r.k_self = FAKE; r.v_self = FAKE; r.temperature = 0.9; r.scale = 0.9
    # no workspace: a valid tree gets as far as the workspace check and nothing is ever launched
    return B.load().ape_attention_tree(ctypes.byref(sh), ctypes.byref(r), ctypes.cast(arr, ctypes.c_void_p), FAKE, len(nodes),
                                       FAKE, q_len, FAKE, None, None, 0, None)


@pytest.mark.parametrize("seed", range(40))
def test_tree_validator_agrees_with_the_rules(seed):
    rng = random.Random(seed)
    n_chunks = rng.randint(1, 40)
    nodes = W.tree_random(n_chunks, seed, max_children=rng.randint(2, 6))
    assert _valid_tree(nodes, n_chunks)
    assert _call_tree(nodes, n_chunks) == B.APE_ERR_WORKSPACE
    # one random mutation: still judged the same way by both
    for _ in range(12):
        m = [list(n) for n in nodes]
        i = rng.randrange(len(m))
        field = rng.choice(["scale", "first", "count", "leaf", "drop", "dup"])
        if field == "scale":
            m[i][0] = rng.choice([0.0, -1.0, 0.5, float("inf")])
        elif field == "first":
            m[i][1] += rng.choice([-1, 1, 2])
        elif field == "count":
            m[i][2] += rng.choice([-1, 1])
        elif field == "leaf":
            m[i][3] = not m[i][3]
        elif field == "drop" and len(m) > 1:
            del m[i]
        else:
            m.append(list(m[i]))
        mt = [tuple(n) for n in m]
        expect_ok = _valid_tree(mt, n_chunks)
        rc = _call_tree(mt, n_chunks)
        assert (rc == B.APE_ERR_WORKSPACE) == expect_ok, (mt, rc)
        assert rc in (B.APE_ERR_WORKSPACE, B.APE_ERR_INVALID_ARG, B.APE_ERR_UNSUPPORTED)


@pytest.mark.parametrize("seed", range(10))
def test_workspace_sizes_are_what_the_calls_demand(seed):
    """A call with one byte less than ape_*_workspace_bytes reports is refused for the workspace;
    sizes grow with the tree and the batch."""
    rng = random.Random(100 + seed)
    sh = B.make_shape(32, 8, 128, B.APE_BF16)
    n_chunks = rng.randint(1, 64)
    total = rng.randint(n_chunks, 200000)
    q_len = rng.choice([1, 7, 64, 256])
    nodes = W.tree_random(n_chunks, seed)
    need = B.tree_workspace_bytes(sh, total, len(nodes), q_len)
    assert need > 0 and need % 256 == 0
    assert B.tree_workspace_bytes(sh, total, len(nodes) + 5, q_len) > need
    arr = (B.ApeTreeNode * len(nodes))(*[B.ApeTreeNode(float(s), f, c, 1 if leaf else 0) for s, f, c, leaf in nodes])
    r = B.ApeRequest()
    r.k_prefix = FAKE; r.v_prefix = FAKE; r.prefix_len = 4; r.n_chunks = n_chunks
    r.k_chunks = FAKE; r.v_chunks = FAKE; r.cu_chunk_lens = FAKE; r.total_ctx_len = total
    r.self_len = q_len; r.k_self = FAKE; r.v_self = FAKE; r.temperature = 0.9; r.scale = 0.9
    rc = B.load().ape_attention_tree(ctypes.byref(sh), ctypes.byref(r), ctypes.cast(arr, ctypes.c_void_p), FAKE, len(nodes),
                                     FAKE, q_len, FAKE, None, FAKE * 256, need - 1, None)
    assert rc == B.APE_ERR_WORKSPACE
    # flat entry points: at least the context group and the prefix+self group per (request, head); the
    # bound need not grow with the batch (the number of splits per request depends on it), it does
    # grow with the context length at a fixed batch
    batch = rng.randint(1, 40)
    d1 = B.workspace_bytes(B.APE_OP_DECODE, sh, batch, 1)
    assert d1 >= batch * 32 * 2 * 516
    lens = sorted(rng.randint(1, 200000) for _ in range(6))
    sizes = [B.workspace_bytes(B.APE_OP_DECODE, sh, batch, 1, n) for n in lens]
    assert sizes == sorted(sizes) and sizes[-1] <= d1
    assert B.workspace_bytes(B.APE_OP_PREFILL, sh, 1, q_len) > 0           # (not monotone in q_len: more row tiles, fewer splits)
    rq = B.ApeRequest()
    for k in ("k_prefix", "v_prefix", "k_chunks", "v_chunks", "cu_chunk_lens", "k_self", "v_self"):
        setattr(rq, k, FAKE)
    rq.prefix_len = 4; rq.n_chunks = n_chunks; rq.total_ctx_len = total; rq.self_len = q_len; rq.temperature = 0.9; rq.scale = 0.9
    rc = B.load().ape_attention_prefill(ctypes.byref(sh), ctypes.byref(rq), FAKE, q_len, FAKE, None, FAKE * 256, 1, None)
    assert rc == B.APE_ERR_WORKSPACE


def _needed(call):
    """Workspace a call demands, read from the message of its refusal (the call gets 1 byte and launches nothing)."""
    assert call() == B.APE_ERR_WORKSPACE
    msg = B.load().ape_last_error().decode()
    return int(msg.split(" bytes given, ")[1].split(" needed")[0])


@pytest.mark.parametrize("seed", range(8))
def test_workspace_bound_covers_every_context_length(seed):
    """ape_workspace_bytes knows batch and rows only; whatever the context length makes of the split
    plan (the workgroup target changes at 12 288 context tokens, the query tile at 40 960, 20 480 or
    6144 depending on the number of query rows), the demand stays within it."""
    rng = random.Random(500 + seed)
    lib = B.load()
    sh = B.make_shape(32, 8, 128, B.APE_BF16) if seed % 2 == 0 else B.make_shape(rng.choice([8, 16, 64]), 8, 128, B.APE_BF16)
    edges = [0, 1, 63, 64, 65, 255, 256, 257, 4096, 6143, 6144, 6145, 12287, 12288, 12289, 16384, 20479, 20480, 20481, 40959, 40960, 40961, 65536,
             131072, 1 << 20, (1 << 31) - 1]
    for _ in range(60):
        batch = rng.choice([1, 1, 2, 4, 7, 32, 33])
        q_len = rng.choice([1, 2, 31, 32, 33, 64, 100, 128, 256, 1000, 1024, 2048])
        ctx = rng.choice(edges + [rng.randint(1, 300000)])
        arr = (B.ApeRequest * batch)()
        for b in range(batch):
            r = arr[b]
            for k in ("k_prefix", "v_prefix", "k_chunks", "v_chunks", "cu_chunk_lens", "k_self", "v_self"):
                setattr(r, k, FAKE)
            r.prefix_len = 4; r.n_chunks = 3 if ctx else 0
            r.total_ctx_len = ctx if b == 0 else rng.randint(0, ctx) if ctx else 0      # request 0 holds the longest context
            if r.total_ctx_len == 0:
                r.n_chunks = 0
            r.self_len = q_len; r.temperature = 0.9; r.scale = 0.9
        bound_p = B.workspace_bytes(B.APE_OP_PREFILL, sh, batch, q_len)
        need_p = _needed(lambda: lib.ape_attention_prefill_batch(ctypes.byref(sh), arr, batch, FAKE, q_len, FAKE, None, FAKE * 256, 1, None))
        assert need_p <= bound_p, (batch, q_len, ctx, need_p, bound_p)
        # the bound for a stated longest context covers this call whenever its contexts are no longer
        for cap in (ctx, ctx + rng.randint(0, 5000), 2 * ctx + 1):
            capped = B.workspace_bytes(B.APE_OP_PREFILL, sh, batch, q_len, cap)
            assert need_p <= capped <= bound_p, (batch, q_len, ctx, cap, need_p, capped, bound_p)
        for b in range(batch):
            arr[b].self_len = max(1, arr[b].self_len)
        bound_d = B.workspace_bytes(B.APE_OP_DECODE, sh, batch, 1)
        need_d = _needed(lambda: lib.ape_attention_decode(ctypes.byref(sh), arr, batch, FAKE, FAKE, None, FAKE * 256, 1, None))
        assert need_d <= bound_d, (batch, ctx, need_d, bound_d)
        for cap in (ctx, ctx + rng.randint(0, 5000), 2 * ctx + 1):
            capped = B.workspace_bytes(B.APE_OP_DECODE, sh, batch, 1, cap)
            assert need_d <= capped <= bound_d, (batch, ctx, cap, need_d, capped, bound_d)


@pytest.mark.parametrize("hq, q_len, batch", [(32, 1, 1), (32, 32, 1), (32, 33, 1), (32, 256, 1), (8, 100, 3), (64, 5, 2)])
def test_prefill_workspace_bound_over_a_sweep_of_context_lengths(hq, q_len, batch):
    """Every context length in a fine sweep up to 70 000 tokens (both changes of the plan lie inside),
    then coarser up to 3 M: the demand never passes ape_workspace_bytes."""
    lib = B.load()
    sh = B.make_shape(hq, 8, 128, B.APE_BF16)
    bound = B.workspace_bytes(B.APE_OP_PREFILL, sh, batch, q_len)
    arr = (B.ApeRequest * batch)()
    for b in range(batch):
        for k in ("k_prefix", "v_prefix", "k_chunks", "v_chunks", "cu_chunk_lens", "k_self", "v_self"):
            setattr(arr[b], k, FAKE)
        arr[b].prefix_len = 4; arr[b].n_chunks = 2; arr[b].self_len = q_len; arr[b].temperature = 0.9; arr[b].scale = 0.9
    worst = 0
    for ctx in list(range(1, 70000, 5)) + list(range(70000, 3000000, 9973)):
        for b in range(batch):
            arr[b].total_ctx_len = ctx
        need = _needed(lambda: lib.ape_attention_prefill_batch(ctypes.byref(sh), arr, batch, FAKE, q_len, FAKE, None, FAKE * 256, 1, None))
        assert need <= bound, (ctx, need, bound)
        if ctx % 7 == 0:                                   # ... nor the bound stated for a cap at or above this length
            for cap in (ctx, ctx + 4097):
                capped = B.workspace_bytes(B.APE_OP_PREFILL, sh, batch, q_len, cap)
                assert need <= capped <= bound, (ctx, cap, need, capped, bound)
        worst = max(worst, need)
    assert worst > bound // 2                              # and the bound is not idle: some length comes within a factor of two


def _decode_splits(sh, batch, ctx):
    """Context splits per request that a decode step over contexts of `ctx` tokens uses, read off the
    workspace it asks for (partial results of (splits + 1) groups per (request, head))."""
    units = batch * sh.n_q_heads
    for n in range(1, 66):
        need = -(-units * (n + 1) * sh.head_dim * 4 // 256) * 256 + -(-units * (n + 1) * 4 // 256) * 256
        if need == B.workspace_bytes(B.APE_OP_DECODE, sh, batch, 1, ctx):
            return n
    raise AssertionError("no split count explains the workspace size")


@pytest.mark.parametrize("batch,ctx,splits", [
    (32, 16384, 1),      # 32 x 8 KV heads = 256 long workgroups: one per CU
    (16, 16384, 2), (8, 131072, 4), (1, 131072, 32), (2, 131072, 16), (64, 8192, 1), (24, 16384, 4), (48, 16384, 2),
    (128, 4096, 1),      # 1024 = 4 x 256
    (1, 2048, 8),        # a short context: never splits below 256 tokens
    (17, 16384, 16),     # 136 x n is a multiple of 256 only at n = 32 (4352 workgroups: too many) -> many workgroups
])
def test_decode_split_plan_fills_the_cus_evenly(batch, ctx, splits):
    """The decode plan takes the smallest number of context splits that makes requests x KV heads x
    splits a multiple of 256 (the CUs), as long as the splits keep 256 tokens and the count 2048."""
    sh = B.make_shape(32, 8, 128, B.APE_BF16)
    n = _decode_splits(sh, batch, ctx)
    assert n == splits, (batch, ctx, n)
    if batch * 8 * n <= 2048 and ctx >= 256 * n and (batch * 8 * n) % 256 == 0:
        assert all((batch * 8 * m) % 256 != 0 for m in range(1, n))
