"""ctypes front end of the plain fp64 CPU oracle (``ape_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the tests, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of ``bench.py``.  The product path never
touches it.  It holds no arithmetic of its own: argument marshalling only.

All array arguments are numpy ``float32`` (they carry fp32 or bf16-rounded
inputs exactly), row-major ``[tokens, heads, head_dim]``; results are
``float64``.  See the C file for what each routine computes and which passage
of the paper (arXiv 2502.05431) it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ape_oracle.c")
_LIB = os.path.join(_HERE, "libape_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP over independent rows only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
                               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        fp, ip, dp = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
        i, d, l = ctypes.c_int, ctypes.c_double, ctypes.c_long
        lib.ape_oracle_attention.argtypes = [i, i, i, fp, fp, i, fp, fp, ip, i, fp, fp, i, fp, i, d, d,
                                             ip, ip, l, dp, dp, dp]
        lib.ape_oracle_attention.restype = i
        lib.ape_oracle_attention_hier.argtypes = [i, i, i, fp, fp, i, fp, fp, ip, i, fp, fp, i, fp, i, d, d, i,
                                                  ip, ip, l, dp, dp]
        lib.ape_oracle_attention_hier.restype = i
        lib.ape_oracle_attention_tree.argtypes = [i, i, i, fp, fp, i, fp, fp, ip, i, fp, fp, i, fp, i, d,
                                                  dp, ip, ip, ip, i, ip, ip, l, dp, dp]
        lib.ape_oracle_attention_tree.restype = i
        lib.ape_oracle_encode.argtypes = [i, i, i, fp, fp, i, fp, fp, fp, ip, i, ip, ip, l, dp, dp]
        lib.ape_oracle_encode.restype = i
        lib.ape_oracle_num_threads.restype = i
        lib.ape_oracle_rope.argtypes = [fp, i, i, ip, i, l, d, dp]
        lib.ape_oracle_rope.restype = i
        _lib = lib
    return _lib


def num_threads() -> int:
    """Threads the oracle's OpenMP loops use."""
    return int(_load().ape_oracle_num_threads())


def _f32(a, shape_tail: Tuple[int, int]) -> np.ndarray:
    if a is None:
        return np.zeros((0,) + shape_tail, dtype=np.float32)
    a = np.ascontiguousarray(a, dtype=np.float32)
    assert a.ndim == 3 and a.shape[1:] == shape_tail, (a.shape, shape_tail)
    return a


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _pairs(pairs, n_rows: int, n_heads: int):
    if pairs is None:
        return None, None, n_rows * n_heads
    pr = np.ascontiguousarray([p[0] for p in pairs], dtype=np.int32)
    ph = np.ascontiguousarray([p[1] for p in pairs], dtype=np.int32)
    return pr, ph, len(pr)


def _cu(chunk_lens: Sequence[int]) -> np.ndarray:
    cu = np.zeros(len(chunk_lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(np.asarray(chunk_lens, dtype=np.int64))
    return cu


def attention(q, k_prefix, v_prefix, k_ctx, v_ctx, chunk_lens, k_self, v_self, T: float, S: float,
              pairs=None, form: str = "weights"):
    """APE attention of ``q`` [q_len, Hq, d] (Section 4.4 / Appendix C).

    ``k_ctx``/``v_ctx`` are the packed contexts [sum(chunk_lens), Hkv, d].
    ``form``: "weights" (Eq.5), "hier" (Appendix C, contexts pooled) or
    "hier_per_context" (Appendix C.2 literal: S per context).
    ``pairs``: optional list of (row, head); default every pair, row-major.
    Returns (out [n, d] float64, lse [n] float64, ctx_mass [n] float64 or None).
    """
    lib = _load()
    q = np.ascontiguousarray(q, dtype=np.float32)
    q_len, hq, d = q.shape
    k_self = np.ascontiguousarray(k_self, dtype=np.float32)
    hkv = k_self.shape[1]
    tail = (hkv, d)
    k_self, v_self = _f32(k_self, tail), _f32(v_self, tail)
    k_prefix, v_prefix = _f32(k_prefix, tail), _f32(v_prefix, tail)
    k_ctx, v_ctx = _f32(k_ctx, tail), _f32(v_ctx, tail)
    cu = _cu(chunk_lens)
    assert cu[-1] == k_ctx.shape[0] == v_ctx.shape[0]
    pr, ph, n = _pairs(pairs, q_len, hq)
    out = np.empty((n, d), dtype=np.float64)
    lse = np.empty(n, dtype=np.float64)
    if form == "weights":
        mass = np.empty(n, dtype=np.float64)
        rc = lib.ape_oracle_attention(hq, hkv, d, _ptr(k_prefix), _ptr(v_prefix), k_prefix.shape[0],
                                      _ptr(k_ctx), _ptr(v_ctx), _ptr(cu), len(chunk_lens),
                                      _ptr(k_self), _ptr(v_self), k_self.shape[0], _ptr(q), q_len,
                                      float(T), float(S), _ptr(pr), _ptr(ph), n,
                                      _ptr(out), _ptr(lse), _ptr(mass))
    elif form in ("hier", "hier_per_context"):
        mass = None
        rc = lib.ape_oracle_attention_hier(hq, hkv, d, _ptr(k_prefix), _ptr(v_prefix), k_prefix.shape[0],
                                           _ptr(k_ctx), _ptr(v_ctx), _ptr(cu), len(chunk_lens),
                                           _ptr(k_self), _ptr(v_self), k_self.shape[0], _ptr(q), q_len,
                                           float(T), float(S), int(form == "hier_per_context"),
                                           _ptr(pr), _ptr(ph), n, _ptr(out), _ptr(lse))
    else:
        raise ValueError(form)
    if rc != 0:
        raise ValueError("ape_oracle: bad arguments")
    return out, lse, mass


def attention_tree(q, k_prefix, v_prefix, k_ctx, v_ctx, chunk_lens, k_self, v_self, T: float, nodes,
                   pairs=None):
    """APE attention over a tree of contexts (Appendix C.2 applied per node, Appendix C.5).

    ``nodes``: list of (scale, first, count, leaf_children); node 0 is the root.  The children
    of node n are contexts first .. first+count-1 when ``leaf_children`` is true, else nodes
    first .. first+count-1 (indices above n).  Returns (out [n, d], lse [n]).
    """
    lib = _load()
    q = np.ascontiguousarray(q, dtype=np.float32)
    q_len, hq, d = q.shape
    k_self = np.ascontiguousarray(k_self, dtype=np.float32)
    hkv = k_self.shape[1]
    tail = (hkv, d)
    k_self, v_self = _f32(k_self, tail), _f32(v_self, tail)
    k_prefix, v_prefix = _f32(k_prefix, tail), _f32(v_prefix, tail)
    k_ctx, v_ctx = _f32(k_ctx, tail), _f32(v_ctx, tail)
    cu = _cu(chunk_lens)
    assert cu[-1] == k_ctx.shape[0] == v_ctx.shape[0]
    scale = np.ascontiguousarray([n[0] for n in nodes], dtype=np.float64)
    first = np.ascontiguousarray([n[1] for n in nodes], dtype=np.int32)
    count = np.ascontiguousarray([n[2] for n in nodes], dtype=np.int32)
    leaf = np.ascontiguousarray([1 if n[3] else 0 for n in nodes], dtype=np.int32)
    pr, ph, n = _pairs(pairs, q_len, hq)
    out = np.empty((n, d), dtype=np.float64)
    lse = np.empty(n, dtype=np.float64)
    rc = lib.ape_oracle_attention_tree(hq, hkv, d, _ptr(k_prefix), _ptr(v_prefix), k_prefix.shape[0],
                                       _ptr(k_ctx), _ptr(v_ctx), _ptr(cu), len(chunk_lens),
                                       _ptr(k_self), _ptr(v_self), k_self.shape[0], _ptr(q), q_len,
                                       float(T), _ptr(scale), _ptr(first), _ptr(count), _ptr(leaf), len(nodes),
                                       _ptr(pr), _ptr(ph), n, _ptr(out), _ptr(lse))
    if rc != 0:
        raise ValueError("ape_oracle: bad arguments")
    return out, lse


def encode(q_ctx, k_prefix, v_prefix, k_ctx, v_ctx, chunk_lens, pairs=None):
    """Block-diagonal causal encoding of the packed contexts (Sections 2.2, 4.1).

    Row r of context i attends to the whole prefix and to rows 0..r of context
    i.  Returns (out [n, d], lse [n]) for the selected (packed row, head) pairs.
    """
    lib = _load()
    q_ctx = np.ascontiguousarray(q_ctx, dtype=np.float32)
    m, hq, d = q_ctx.shape
    k_ctx = np.ascontiguousarray(k_ctx, dtype=np.float32)
    hkv = k_ctx.shape[1]
    tail = (hkv, d)
    k_ctx, v_ctx = _f32(k_ctx, tail), _f32(v_ctx, tail)
    k_prefix, v_prefix = _f32(k_prefix, tail), _f32(v_prefix, tail)
    cu = _cu(chunk_lens)
    assert cu[-1] == m == k_ctx.shape[0] == v_ctx.shape[0]
    pr, ph, n = _pairs(pairs, m, hq)
    out = np.empty((n, d), dtype=np.float64)
    lse = np.empty(n, dtype=np.float64)
    rc = lib.ape_oracle_encode(hq, hkv, d, _ptr(k_prefix), _ptr(v_prefix), k_prefix.shape[0],
                               _ptr(q_ctx), _ptr(k_ctx), _ptr(v_ctx), _ptr(cu), len(chunk_lens),
                               _ptr(pr), _ptr(ph), n, _ptr(out), _ptr(lse))
    if rc != 0:
        raise ValueError("ape_oracle: bad arguments")
    return out, lse


def rope(x, chunk_lens, position_offset: int, base: float):
    """Rotary position embedding of packed segments ``x`` [sum(chunk_lens), heads, d]: token j of
    every segment sits at position ``position_offset + j`` (positions re-used across contexts,
    Section 1).  Half-split pairing.  Returns float64 [M, heads, d]."""
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float32)
    assert x.ndim == 3
    cu = _cu(chunk_lens)
    assert cu[-1] == x.shape[0]
    y = np.empty(x.shape, dtype=np.float64)
    rc = lib.ape_oracle_rope(_ptr(x), x.shape[1], x.shape[2], _ptr(cu), len(chunk_lens),
                             int(position_offset), float(base), _ptr(y))
    if rc != 0:
        raise ValueError("ape_oracle: bad arguments")
    return y
