"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
public header declares, sizes workspaces, and rejects bad arguments before launching anything."""
import ctypes

import numpy as np
import os
import re

import pytest

from paper_2502_05431_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions(header="ape.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ape_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.load()
    names = header_functions()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None
    assert re.match(rb"\d+\.\d+\.\d+", lib.ape_version())


def test_layer_library_exports_every_declared_symbol_and_the_attention_library_needs_no_gemm_library():
    lib = B.load_layer()
    names = header_functions("ape_layer.h")
    assert set(names) == set(B.LAYER_EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None
    # the attention library depends on the HIP runtime alone; rocBLAS comes in with the layer library only
    import subprocess
    needed = lambda path: subprocess.run(["readelf", "-d", path], capture_output=True, text=True).stdout
    assert "rocblas" not in needed(B.LIB_PATH)
    assert "rocblas" in needed(B.LAYER_LIB_PATH) and "libape_hip.so" in needed(B.LAYER_LIB_PATH)
    sh = B.make_shape(32, 8, 128, B.APE_BF16)
    one = B.layer_workspace_bytes(sh, 4096, 14336, 1000)
    assert one > 0 and one % 256 == 0
    assert B.layer_workspace_bytes(sh, 4096, 14336, 1000, n_layers=4) == one + (1000 * 4096 * 2 + 255) // 256 * 256
    assert B.layer_workspace_bytes(sh, 4095, 14336, 1000) == 0


def test_probe_library_exports_every_declared_symbol():
    lib = B.load_probe()
    names = header_functions("ape_probe.h")
    assert set(names) == set(B.PROBE_EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None
    out = ctypes.c_double(0.0)
    assert lib.ape_probe_mfma(None, 0, None, 0.0, None, ctypes.byref(out)) != 0      # refused on the host, nothing launched
    assert lib.ape_probe_hbm_read(None, 0, None, 0.0, None, ctypes.byref(out)) != 0
    # a level or a wavefront count the probes do not have: refused before anything touches the GPU
    fake = ctypes.c_void_p(0x1000)
    assert lib.ape_probe_mfma(fake, 5, fake, 0.0, None, ctypes.byref(out)) != 0
    assert lib.ape_probe_mfma(fake, -1, fake, 0.0, None, ctypes.byref(out)) != 0
    assert lib.ape_probe_valu_issue(3, fake, 0.0, None, ctypes.byref(out)) != 0
    assert lib.ape_probe_valu_issue(1, None, 0.0, None, ctypes.byref(out)) != 0


def test_status_strings():
    lib = B.load()
    for code in (0, -1, -2, -3, -4):
        assert lib.ape_status_string(code)
    assert lib.ape_status_string(-99) == b"unknown status"


def test_workspace_bytes():
    sh = B.make_shape(32, 8, 128, B.APE_BF16)
    assert B.workspace_bytes(B.APE_OP_ENCODE, sh, 1, 1) == 0
    d = B.workspace_bytes(B.APE_OP_DECODE, sh, 32, 1)
    p = B.workspace_bytes(B.APE_OP_PREFILL, sh, 1, 256)
    assert d > 0 and p > d
    assert d % 256 == 0 and p % 256 == 0
    # decode ignores q_len; a batched prefill needs room for every request
    assert B.workspace_bytes(B.APE_OP_DECODE, sh, 32, 77) == d
    p4 = B.workspace_bytes(B.APE_OP_PREFILL, sh, 4, 256)
    assert p < p4 <= 4 * p                                 # more requests, fewer context splits each
    bad = B.make_shape(32, 7, 128, B.APE_BF16)
    assert B.workspace_bytes(B.APE_OP_DECODE, bad, 1, 1) == 0
    assert B.workspace_bytes(99, sh, 1, 1) == 0
    # with the longest context stated, the bound is what calls up to that length need and no more:
    # never above the any-length bound, growing with the length, one split (prefix + self) for none
    unit = 516                                             # (head_dim + 1) fp32 per (row, head) and split
    assert B.workspace_bytes(B.APE_OP_DECODE, sh, 1, 1, 0) < 2 * 32 * unit + 512
    d128k = B.workspace_bytes(B.APE_OP_DECODE, sh, 1, 1, 131072)
    d16k = B.workspace_bytes(B.APE_OP_DECODE, sh, 1, 1, 16384)
    assert 0 < B.workspace_bytes(B.APE_OP_DECODE, sh, 1, 1, 1024) < d16k <= d128k <= B.workspace_bytes(B.APE_OP_DECODE, sh, 1, 1, -1)
    p128k = B.workspace_bytes(B.APE_OP_PREFILL, sh, 1, 256, 131072)
    assert 0 < p128k <= p and B.workspace_bytes(B.APE_OP_PREFILL, sh, 1, 256, 1 << 40) == p
    assert p128k < 12 * 8192 * unit                        # config 3: 8 context splits + 1, not the 65-split worst case


FAKE = 0x1000  # never dereferenced: every call below fails validation before any launch


def _req(**kw):
    r = B.ApeRequest()
    r.k_prefix = FAKE; r.v_prefix = FAKE; r.prefix_len = 4; r.n_chunks = 2
    r.k_chunks = FAKE; r.v_chunks = FAKE; r.cu_chunk_lens = FAKE; r.total_ctx_len = 64
    r.self_len = 8; r.k_self = FAKE; r.v_self = FAKE; r.temperature = 0.9; r.scale = 0.9
    for k, v in kw.items():
        setattr(r, k, v)
    return r


def _prefill(shape, req, q_len=8, q=FAKE, out=FAKE, ws=None, ws_bytes=0):
    return B.load().ape_attention_prefill(ctypes.byref(shape), ctypes.byref(req), q, q_len, out, None, ws, ws_bytes, None)


@pytest.mark.parametrize("kw,code", [
    (dict(temperature=0.0), B.APE_ERR_INVALID_ARG),
    (dict(temperature=float("nan")), B.APE_ERR_INVALID_ARG),
    (dict(temperature=float("inf")), B.APE_ERR_INVALID_ARG),
    (dict(scale=-0.5), B.APE_ERR_INVALID_ARG),
    (dict(scale=float("nan")), B.APE_ERR_INVALID_ARG),
    (dict(self_len=7), B.APE_ERR_INVALID_ARG),            # fewer self tokens than query rows
    (dict(prefix_len=-1), B.APE_ERR_INVALID_ARG),
    (dict(k_prefix=None), B.APE_ERR_INVALID_ARG),
    (dict(k_chunks=None), B.APE_ERR_INVALID_ARG),
    (dict(cu_chunk_lens=None), B.APE_ERR_INVALID_ARG),
    (dict(n_chunks=0), B.APE_ERR_INVALID_ARG),            # context length without chunks
    (dict(k_self=None), B.APE_ERR_INVALID_ARG),
    (dict(), B.APE_ERR_WORKSPACE),                        # valid request, no workspace
])
def test_prefill_argument_errors(kw, code):
    sh = B.make_shape(32, 8, 128, B.APE_BF16)
    assert _prefill(sh, _req(**kw)) == code
    assert B.load().ape_last_error()


def test_misaligned_data_pointers_are_refused():
    """The kernels use 16-byte accesses; pointers the host can see are checked before any launch."""
    lib = B.load()
    sh = B.make_shape(32, 8, 128, B.APE_BF16)
    for kw in (dict(k_self=FAKE + 2), dict(v_prefix=FAKE + 8), dict(k_chunks=FAKE + 4), dict(cu_chunk_lens=FAKE + 2)):
        assert _prefill(sh, _req(**kw)) == B.APE_ERR_INVALID_ARG, kw
        assert b"aligned" in lib.ape_last_error()
    assert _prefill(sh, _req(), q=FAKE + 8) == B.APE_ERR_INVALID_ARG
    assert _prefill(sh, _req(), out=FAKE + 4) == B.APE_ERR_INVALID_ARG
    assert _prefill(sh, _req(k_chunks=FAKE + 8)) == B.APE_ERR_WORKSPACE          # a table may start at any of its elements
    cu = (ctypes.c_int32 * 2)(0, 64)
    rc = lib.ape_encode_chunks(ctypes.byref(sh), None, FAKE, FAKE, 4, FAKE + 6, FAKE, FAKE, ctypes.cast(cu, ctypes.c_void_p), FAKE, 1,
                               None, FAKE, None, None, None, 0, None)
    assert rc == B.APE_ERR_INVALID_ARG and b"aligned" in lib.ape_last_error()


def test_shape_errors():
    r = _req()
    assert _prefill(B.make_shape(32, 7, 128, B.APE_BF16), r) == B.APE_ERR_INVALID_ARG
    assert _prefill(B.make_shape(0, 8, 128, B.APE_BF16), r) == B.APE_ERR_INVALID_ARG
    assert _prefill(B.make_shape(32, 8, 100, B.APE_BF16), r) == B.APE_ERR_UNSUPPORTED
    assert _prefill(B.make_shape(32, 8, 512, B.APE_BF16), r) == B.APE_ERR_UNSUPPORTED
    assert _prefill(B.make_shape(32, 8, 128, 7), r) == B.APE_ERR_UNSUPPORTED
    sh = B.make_shape(32, 8, 128, B.APE_BF16)
    assert _prefill(sh, r, q_len=0) == B.APE_ERR_INVALID_ARG
    assert _prefill(sh, r, q=None) == B.APE_ERR_INVALID_ARG
    assert _prefill(sh, r, ws=FAKE + 4, ws_bytes=1 << 40) == B.APE_ERR_WORKSPACE     # misaligned
    assert B.load().ape_attention_prefill(None, ctypes.byref(r), FAKE, 8, FAKE, None, None, 0, None) == B.APE_ERR_INVALID_ARG


def test_decode_and_encode_argument_errors():
    lib = B.load()
    sh = B.make_shape(32, 8, 128, B.APE_BF16)
    arr = (B.ApeRequest * 2)(_req(self_len=1), _req(self_len=0))
    assert lib.ape_attention_decode(ctypes.byref(sh), arr, 2, FAKE, FAKE, None, None, 0, None) == B.APE_ERR_INVALID_ARG
    assert b"request 1" in lib.ape_last_error()
    assert lib.ape_attention_decode(ctypes.byref(sh), arr, 0, FAKE, FAKE, None, None, 0, None) == B.APE_ERR_INVALID_ARG
    cu = (ctypes.c_int32 * 3)(0, 5, 3)
    enc = lambda cu_host, cu_dev, **kw: lib.ape_encode_chunks(
        ctypes.byref(sh), kw.get("q_prefix"), FAKE, FAKE, kw.get("prefix_len", 4), FAKE, FAKE, FAKE,
        cu_host, cu_dev, 2, kw.get("o_prefix"), FAKE, None, None, None, 0, None)
    assert enc(ctypes.cast(cu, ctypes.c_void_p), FAKE) == B.APE_ERR_INVALID_ARG        # not non-decreasing
    assert enc(None, FAKE) == B.APE_ERR_INVALID_ARG
    cu2 = (ctypes.c_int32 * 3)(0, 5, 9)
    assert enc(ctypes.cast(cu2, ctypes.c_void_p), None) == B.APE_ERR_INVALID_ARG       # no device copy
    assert enc(ctypes.cast(cu2, ctypes.c_void_p), FAKE, q_prefix=FAKE) == B.APE_ERR_INVALID_ARG   # q_prefix without o_prefix
    assert enc(ctypes.cast(cu2, ctypes.c_void_p), FAKE, prefix_len=-2) == B.APE_ERR_INVALID_ARG


def test_size_limits_are_refused_before_any_launch():
    """Calls whose grids would pass 2^32 work items, or whose counts would not fit the kernels' 32-bit
    indices, return APE_ERR_UNSUPPORTED with a message that names the limit."""
    lib = B.load()
    sh = B.make_shape(32, 8, 128, B.APE_BF16)
    # query prefill: fewer than 2^24 (row, head) outputs pass the check (and stop at the missing workspace);
    # exactly 2^24 would be 2^32 work items in the merge launch and is refused
    rows_ok = (1 << 24) // 32 - 1
    assert _prefill(sh, _req(self_len=rows_ok), q_len=rows_ok) == B.APE_ERR_WORKSPACE
    assert _prefill(sh, _req(self_len=rows_ok + 1), q_len=rows_ok + 1) == B.APE_ERR_UNSUPPORTED
    assert b"outputs in one call" in lib.ape_last_error()
    assert B.workspace_bytes(B.APE_OP_PREFILL, sh, 1, rows_ok) > 0 and B.workspace_bytes(B.APE_OP_PREFILL, sh, 1, rows_ok + 1) == 0
    assert _tree([(0.9, 0, 4, 1)], req=_req(n_chunks=4, total_ctx_len=200, self_len=rows_ok + 1), q_len=rows_ok + 1) == B.APE_ERR_UNSUPPORTED
    # a tree call sizes its attention grid from the bound on the splits: many nodes x many query rows
    # pass 2^24 workgroups and are refused on the host (not by the launch)
    n_ctx = 2000
    big_tree = [(1.0, 1, n_ctx, 0)] + [(0.9, i, 1, 1) for i in range(n_ctx)]
    assert _tree(big_tree, req=_req(n_chunks=n_ctx, total_ctx_len=n_ctx * 64, self_len=131072), q_len=131072) == B.APE_ERR_UNSUPPORTED
    assert b"workgroups" in lib.ape_last_error()
    # encode on the matrix-core path: contexts x KV heads x query tiles of the longest context
    n = 4096
    lens = [1 << 17] + [1] * (n - 1)                      # one long context makes every context's share of the grid long
    cu = (ctypes.c_int32 * (n + 1))(*np.concatenate([[0], np.cumsum(lens)]).tolist())
    enc = lambda shape: lib.ape_encode_chunks(ctypes.byref(shape), None, FAKE, FAKE, 4, FAKE, FAKE, FAKE,
                                              ctypes.cast(cu, ctypes.c_void_p), FAKE, n, None, FAKE, None, None, None, 0, None)
    assert enc(sh) == B.APE_ERR_UNSUPPORTED
    assert b"workgroups" in lib.ape_last_error()
    # the generic path counts (row, head) outputs instead
    cu2 = (ctypes.c_int32 * 2)(0, 1 << 22)
    enc1 = lambda shape: lib.ape_encode_chunks(ctypes.byref(shape), None, FAKE, FAKE, 4, FAKE, FAKE, FAKE,
                                               ctypes.cast(cu2, ctypes.c_void_p), FAKE, 1, None, FAKE, None, None, None, 0, None)
    assert enc1(B.make_shape(32, 8, 128, B.APE_F32)) == B.APE_ERR_UNSUPPORTED
    assert b"generic path" in lib.ape_last_error()


def _tree(nodes, req=None, nodes_dev=FAKE, n_nodes=None, ws=None, ws_bytes=0, q_len=8):
    sh = B.make_shape(32, 8, 128, B.APE_BF16)
    arr = (B.ApeTreeNode * max(len(nodes), 1))(*[B.ApeTreeNode(*n) for n in nodes])
    r = req or _req(n_chunks=4, total_ctx_len=200)
    return B.load().ape_attention_tree(ctypes.byref(sh), ctypes.byref(r), ctypes.cast(arr, ctypes.c_void_p), nodes_dev,
                                       len(nodes) if n_nodes is None else n_nodes, FAKE, q_len, FAKE, None,
                                       ws, ws_bytes, None)


@pytest.mark.parametrize("nodes,code,text", [
    ([(0.9, 0, 4, 1)], B.APE_ERR_WORKSPACE, b"workspace"),                              # a valid tree: fails only on the workspace
    ([(1.0, 1, 2, 0), (0.9, 0, 2, 1), (0.8, 2, 2, 1)], B.APE_ERR_WORKSPACE, b"workspace"),
    ([(1.0, 1, 2, 0), (0.9, 0, 1, 1), (0.8, 3, 1, 0), (0.7, 1, 3, 1)], B.APE_ERR_WORKSPACE, b"workspace"),   # mixed depths
    ([(0.0, 0, 4, 1)], B.APE_ERR_INVALID_ARG, b"scale"),
    ([(float("nan"), 0, 4, 1)], B.APE_ERR_INVALID_ARG, b"scale"),
    ([(0.9, 0, 0, 1)], B.APE_ERR_INVALID_ARG, b"count"),
    ([(0.9, 0, 5, 1)], B.APE_ERR_INVALID_ARG, b"outside the chunk table"),
    ([(0.9, -1, 2, 1)], B.APE_ERR_INVALID_ARG, b"outside the chunk table"),
    ([(0.9, 0, 3, 1)], B.APE_ERR_INVALID_ARG, b"belongs to no tree node"),
    ([(1.0, 1, 2, 0), (0.9, 0, 3, 1), (0.8, 2, 2, 1)], B.APE_ERR_INVALID_ARG, b"already belongs"),
    ([(1.0, 0, 1, 0)], B.APE_ERR_INVALID_ARG, b"must start at 1"),                       # a node as its own child
    ([(1.0, 2, 1, 0), (0.9, 0, 4, 1), (0.9, 0, 4, 1)], B.APE_ERR_INVALID_ARG, b"must start at 1"),
    ([(1.0, 1, 3, 0), (0.9, 0, 4, 1)], B.APE_ERR_INVALID_ARG, b"run past"),
    ([(0.9, 0, 2, 1), (0.9, 2, 2, 1)], B.APE_ERR_INVALID_ARG, b"reachable"),             # an orphan node
    ([], B.APE_ERR_INVALID_ARG, b"at least one node"),
])
def test_tree_validation(nodes, code, text):
    assert _tree(nodes) == code
    assert text in B.load().ape_last_error()


def test_tree_limits_and_workspace_size():
    lib = B.load()
    assert _tree([(0.9, 0, 4, 1)], nodes_dev=None, ws=FAKE * 256, ws_bytes=1 << 40) == B.APE_ERR_INVALID_ARG
    assert _tree([(0.9, 0, 4, 1)], req=_req(n_chunks=0, total_ctx_len=0)) == B.APE_ERR_INVALID_ARG       # a tree needs contexts
    assert _tree([(0.9, 0, 4, 1)], req=_req(n_chunks=4, total_ctx_len=200, self_len=3)) == B.APE_ERR_INVALID_ARG
    # a chain deeper than the supported number of levels
    depth = B.APE_TREE_MAX_DEPTH + 1
    chain = [(1.0, i + 1, 1, 0) for i in range(depth - 1)] + [(0.9, 0, 4, 1)]
    assert _tree(chain) == B.APE_ERR_UNSUPPORTED and b"deeper" in lib.ape_last_error()
    assert _tree(chain[1:-1] + [(0.9, 0, 4, 1)]) == B.APE_ERR_INVALID_ARG              # numbering now off by one
    ok_chain = [(1.0, i + 1, 1, 0) for i in range(B.APE_TREE_MAX_DEPTH - 1)] + [(0.9, 0, 4, 1)]
    assert _tree(ok_chain) == B.APE_ERR_WORKSPACE
    too_many = [(1.0, 1, B.APE_TREE_MAX_NODES, 0)] + [(0.9, 0, 1, 1)] * B.APE_TREE_MAX_NODES
    assert _tree(too_many) == B.APE_ERR_UNSUPPORTED
    sh = B.make_shape(32, 8, 128, B.APE_BF16)
    w1 = B.tree_workspace_bytes(sh, 131072, 65, 256)
    assert w1 > 0 and w1 % 256 == 0
    # one split per context node at least, plus the prefix+self block: 65 partial results of 256*32 units
    assert w1 >= 65 * 256 * 32 * (128 + 1) * 4
    assert B.tree_workspace_bytes(sh, 131072, 0, 256) == 0
    assert B.tree_workspace_bytes(sh, 131072, B.APE_TREE_MAX_NODES + 1, 1) == 0
    assert B.tree_workspace_bytes(sh, -1, 4, 1) == 0
    # a one-node tree needs what the flat entry point needs plus one spare split and the plan
    flat = B.workspace_bytes(B.APE_OP_PREFILL, sh, 1, 256)
    assert flat <= B.tree_workspace_bytes(sh, 131072, 1, 256) <= flat * 10 // 9 + 65536
    assert B.tree_workspace_bytes(sh, 200, 1, 8) < (1 << 22)
    assert _tree([(0.9, 0, 4, 1)], ws=FAKE * 256, ws_bytes=B.tree_workspace_bytes(sh, 200, 1, 8) - 1) == B.APE_ERR_WORKSPACE


def test_batched_prefill_argument_errors():
    lib = B.load()
    sh = B.make_shape(32, 8, 128, B.APE_BF16)
    arr = (B.ApeRequest * 2)(_req(), _req(self_len=3))
    call = lambda n, q_len=8, q=FAKE: lib.ape_attention_prefill_batch(ctypes.byref(sh), arr, n, q, q_len, FAKE, None, None, 0, None)
    assert call(2) == B.APE_ERR_INVALID_ARG and b"request 1" in lib.ape_last_error()     # self_len 3 < q_len 8
    assert call(0) == B.APE_ERR_INVALID_ARG
    assert call(1, q_len=0) == B.APE_ERR_INVALID_ARG
    assert call(1, q=None) == B.APE_ERR_INVALID_ARG
    assert call(1) == B.APE_ERR_WORKSPACE


def test_layer_argument_errors():
    lib = B.load_layer()
    sh = B.make_shape(32, 8, 128, B.APE_BF16)
    cu = (ctypes.c_int32 * 3)(0, 5, 9)
    cuh = ctypes.cast(cu, ctypes.c_void_p)

    def weights(**kw):
        w = B.ApeLayerWeights(4096, 14336, 1e-5, 500000.0, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE)
        for k, v in kw.items():
            setattr(w, k, v)
        return w

    def layer(w=None, x=FAKE, kp=FAKE, vp=FAKE, lp=4, cu_host=cuh, cu_dev=FAKE, n=2, kc=FAKE, vc=FAKE, y=FAKE + 256, ws=None, wsb=0):
        w = w or weights()
        return lib.ape_layer_encode(ctypes.byref(sh), ctypes.byref(w), x, kp, vp, lp, cu_host, cu_dev, n, kc, vc, y, None, ws, wsb, None)
    assert layer(w=weights(hidden=4095)) == B.APE_ERR_UNSUPPORTED
    assert layer(w=weights(intermediate=0)) == B.APE_ERR_UNSUPPORTED
    assert layer(w=weights(rms_eps=-1.0)) == B.APE_ERR_INVALID_ARG
    assert layer(w=weights(rope_base=0.0)) == B.APE_ERR_INVALID_ARG
    assert layer(w=weights(w_o=None)) == B.APE_ERR_INVALID_ARG
    assert layer(kp=None) == B.APE_ERR_INVALID_ARG
    assert layer(lp=-1) == B.APE_ERR_INVALID_ARG
    assert layer(cu_host=None) == B.APE_ERR_INVALID_ARG
    assert layer(x=None) == B.APE_ERR_INVALID_ARG
    assert layer(kc=None) == B.APE_ERR_INVALID_ARG
    assert layer() == B.APE_ERR_WORKSPACE
    assert layer(ws=FAKE + 8, wsb=1 << 40) == B.APE_ERR_WORKSPACE
    assert layer(n=0) == B.APE_OK                                  # nothing to do
    assert layer(y=FAKE, x=FAKE + 0) == B.APE_ERR_INVALID_ARG      # y aliases x
    assert b"alias" in B.load().ape_last_error()                   # (one error text for both libraries)

    # a stack of layers: per-layer tables on the host
    def stack(n_layers=2, ws=None, wsb=0, widths=(4096, 4096), kc_null=False, lp=4):
        warr = (B.ApeLayerWeights * n_layers)(*[weights(hidden=widths[i % len(widths)]) for i in range(n_layers)])
        tab = (ctypes.c_void_p * max(n_layers, 1))(*[FAKE] * n_layers)
        kc = (ctypes.c_void_p * max(n_layers, 1))(*([FAKE] * (n_layers - 1) + [None if kc_null else FAKE])[:n_layers])
        return lib.ape_layers_encode(ctypes.byref(sh), warr, n_layers, FAKE, tab, tab, lp, cuh, FAKE, 2, kc, tab, FAKE + 256, ws, wsb, None)
    assert stack(n_layers=0) == B.APE_ERR_INVALID_ARG
    assert stack(widths=(4096, 2048)) == B.APE_ERR_INVALID_ARG     # layers of different widths
    assert stack(kc_null=True) == B.APE_ERR_INVALID_ARG
    assert stack() == B.APE_ERR_WORKSPACE
    assert stack(ws=FAKE * 256, wsb=B.layer_workspace_bytes(sh, 4096, 14336, 9, n_layers=2) - 1) == B.APE_ERR_WORKSPACE
    need = B.layer_workspace_bytes(sh, 4096, 14336, 131072)
    assert need % 256 == 0 and 4 * 2 ** 30 < need < 8 * 2 ** 30    # the MLP runs in slabs: a few GiB, not 16
    assert B.layer_workspace_bytes(sh, 4095, 14336, 10) == 0


def test_rope_argument_errors():
    lib = B.load()
    sh = B.make_shape(32, 8, 128, B.APE_BF16)
    cu = (ctypes.c_int32 * 3)(0, 5, 9)
    cuh = ctypes.cast(cu, ctypes.c_void_p)

    def rope(cu_host=cuh, cu_dev=FAKE, n=2, off=32, base=500000.0, q=FAKE, k=FAKE, v=FAKE, qo=FAKE, kc=FAKE, vc=FAKE, shape=sh):
        return lib.ape_rope_write_cache(ctypes.byref(shape), q, k, v, cu_host, cu_dev, n, off, base, qo, kc, vc, None)
    assert rope(off=-1) == B.APE_ERR_INVALID_ARG
    assert rope(base=0.0) == B.APE_ERR_INVALID_ARG
    assert rope(base=float("inf")) == B.APE_ERR_INVALID_ARG
    assert rope(qo=None) == B.APE_ERR_INVALID_ARG            # q_raw without q_rot
    assert rope(k=None) == B.APE_ERR_INVALID_ARG             # k_cache without k_raw
    assert rope(vc=None) == B.APE_ERR_INVALID_ARG
    assert rope(cu_host=None) == B.APE_ERR_INVALID_ARG
    assert rope(cu_dev=None) == B.APE_ERR_INVALID_ARG
    assert rope(n=-1) == B.APE_ERR_INVALID_ARG
    bad = (ctypes.c_int32 * 3)(0, 5, 3)
    assert rope(cu_host=ctypes.cast(bad, ctypes.c_void_p)) == B.APE_ERR_INVALID_ARG
    assert rope(shape=B.make_shape(32, 8, 100, B.APE_BF16)) == B.APE_ERR_UNSUPPORTED
    assert rope(n=0, cu_host=None, cu_dev=None) == B.APE_OK    # nothing to do, nothing launched
    empty = (ctypes.c_int32 * 3)(0, 0, 0)
    assert rope(cu_host=ctypes.cast(empty, ctypes.c_void_p)) == B.APE_OK


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="missing"):
        B.load()


def test_binding_structs_have_the_layout_of_the_header(tmp_path):
    """The ctypes mirrors of the C structs against the compiler's view of include/ape.h: size and the
    offset of every field (a drifted binding would hand the library shifted arguments)."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("needs gcc")
    structs = {"ape_shape": B.ApeShape, "ape_request": B.ApeRequest, "ape_tree_node": B.ApeTreeNode,
               "ape_layer_weights": B.ApeLayerWeights, "ape_layer_taps": B.ApeLayerTaps}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "ape.h"', '#include "ape_layer.h"', 'int main(void) {']
    for cname, cls in structs.items():
        lines.append('printf("%s size %%zu\\n", sizeof(%s));' % (cname, cname))
        for fname, _ in cls._fields_:
            lines.append('printf("%s %s %%zu\\n", offsetof(%s, %s));' % (cname, fname, cname, fname))
    lines += ['return 0; }']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = str(tmp_path / "layout")
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    subprocess.check_call(["gcc", "-std=c11", "-Wall", "-I", inc, "-o", exe, str(src)])
    out = subprocess.run([exe], capture_output=True, text=True, check=True).stdout.split("\n")
    seen = 0
    for line in filter(None, out):
        cname, fname, value = line.split()
        cls = structs[cname]
        if fname == "size":
            assert ctypes.sizeof(cls) == int(value), line
        else:
            assert getattr(cls, fname).offset == int(value), line
        seen += 1
    assert seen == sum(len(c._fields_) + 1 for c in structs.values())


def test_a_plain_c_program_links_and_calls_the_library(tmp_path):
    """The boundary is a C ABI: a C11 program that includes ape.h links against the library and calls
    the entry points that need no GPU (sizes, status strings, an argument error)."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("needs gcc")
    B.load()                                              # fails loudly if the library has not been built
    src = tmp_path / "consumer.c"
    src.write_text(r'''
#include <stdio.h>
#include <string.h>
#include "ape.h"
int main(void) {
    ape_shape sh = {32, 8, 128, APE_BF16};
    size_t ws = ape_workspace_bytes(APE_OP_DECODE, &sh, 32, 1, 16384);
    if (ws == 0 || ws % 256) return 1;
    if (ape_workspace_bytes(APE_OP_ENCODE, &sh, 1, 1, -1) != 0) return 2;
    if (strlen(ape_status_string(APE_ERR_WORKSPACE)) == 0) return 3;
    ape_request r;
    memset(&r, 0, sizeof r);
    r.temperature = 0.f;                                  /* invalid: refused on the host, nothing is launched */
    int rc = ape_attention_prefill(&sh, &r, (const void*)256, 1, (void*)256, NULL, NULL, 0, NULL);
    if (rc != APE_ERR_INVALID_ARG || strlen(ape_last_error()) == 0) return 4;
    printf("%s %zu\n", ape_version(), ws);
    return 0;
}
''')
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    lib_dir = os.path.dirname(B.LIB_PATH)
    exe = str(tmp_path / "consumer")
    subprocess.check_call(["gcc", "-std=c11", "-Wall", "-Werror", "-I", os.path.join(root, "include"), "-o", exe, str(src),
                           "-L", lib_dir, "-lape_hip", "-Wl,-rpath," + lib_dir, "-Wl,-rpath-link,/opt/rocm/lib"])
    env = dict(os.environ)
    env["LD_LIBRARY_PATH"] = lib_dir + os.pathsep + "/opt/rocm/lib" + os.pathsep + env.get("LD_LIBRARY_PATH", "")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, (run.returncode, run.stdout, run.stderr)
    assert run.stdout.split()[1].isdigit()
