"""Thin ctypes binding of ``libape_hip.so`` (the C ABI in ``include/ape.h``).

Argument marshalling only: every step of the attention path runs in the HIP
kernels.  torch is used for device memory and streams.  The library must have
been built (``python -m paper_2502_05431_amd.build``); loading fails loudly if it
is missing -- there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libape_hip.so")
LAYER_LIB_PATH = os.path.join(_PKG, "libape_layer.so")
PROBE_LIB_PATH = os.path.join(_PKG, "libape_probe.so")

APE_OK = 0
APE_ERR_INVALID_ARG, APE_ERR_UNSUPPORTED, APE_ERR_WORKSPACE, APE_ERR_DEVICE = -1, -2, -3, -4
APE_F32, APE_BF16 = 0, 1
APE_DTYPE_FLAG_GENERIC = 0x100
APE_OP_ENCODE, APE_OP_PREFILL, APE_OP_DECODE = 0, 1, 2

EXPORTS = ("ape_workspace_bytes", "ape_encode_chunks", "ape_attention_prefill", "ape_attention_decode",
           "ape_attention_prefill_batch", "ape_attention_decode_static",
           "ape_tree_workspace_bytes", "ape_attention_tree", "ape_rope_write_cache",
           "ape_status_string", "ape_last_error", "ape_version")
PROBE_EXPORTS = ("ape_probe_mfma", "ape_probe_hbm_read", "ape_probe_valu_issue")
LAYER_EXPORTS = ("ape_layer_workspace_bytes", "ape_layers_workspace_bytes", "ape_layer_encode", "ape_layers_encode")
APE_TREE_MAX_NODES, APE_TREE_MAX_CONTEXTS, APE_TREE_MAX_DEPTH = 2048, 4096, 16
APE_STATIC_SCRATCH_BYTES = 8 << 20


class ApeShape(ctypes.Structure):
    _fields_ = [("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32)]


class ApeRequest(ctypes.Structure):
    _fields_ = [("k_prefix", ctypes.c_void_p), ("v_prefix", ctypes.c_void_p),
                ("prefix_len", ctypes.c_int32), ("n_chunks", ctypes.c_int32),
                ("k_chunks", ctypes.c_void_p), ("v_chunks", ctypes.c_void_p),
                ("cu_chunk_lens", ctypes.c_void_p),
                ("total_ctx_len", ctypes.c_int32), ("self_len", ctypes.c_int32),
                ("k_self", ctypes.c_void_p), ("v_self", ctypes.c_void_p),
                ("temperature", ctypes.c_float), ("scale", ctypes.c_float)]


class ApeTreeNode(ctypes.Structure):
    _fields_ = [("scale", ctypes.c_float), ("first", ctypes.c_int32), ("count", ctypes.c_int32),
                ("leaf_children", ctypes.c_int32)]


class ApeLayerWeights(ctypes.Structure):
    _fields_ = [("hidden", ctypes.c_int32), ("intermediate", ctypes.c_int32), ("rms_eps", ctypes.c_float),
                ("rope_base", ctypes.c_float), ("attn_norm", ctypes.c_void_p), ("w_qkv", ctypes.c_void_p),
                ("w_o", ctypes.c_void_p), ("mlp_norm", ctypes.c_void_p), ("w_gate_up", ctypes.c_void_p),
                ("w_down", ctypes.c_void_p)]


class ApeLayerTaps(ctypes.Structure):
    _fields_ = [("q_rot", ctypes.c_void_p), ("attn", ctypes.c_void_p)]


class ApeError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("ape status %d: %s" % (status, message))
        self.status = status


_lib = None


def load() -> ctypes.CDLL:
    """Load the HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("%s is missing: build it with `python -m paper_2502_05431_amd.build` "
                               "(there is no fallback path)" % LIB_PATH)
        lib = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        lib.ape_workspace_bytes.argtypes = [ctypes.c_int, ctypes.POINTER(ApeShape), i32, i32, ctypes.c_int64]
        lib.ape_workspace_bytes.restype = sz
        lib.ape_encode_chunks.argtypes = [ctypes.POINTER(ApeShape), vp, vp, vp, i32, vp, vp, vp, vp, vp, i32,
                                          vp, vp, vp, vp, vp, sz, vp]
        lib.ape_encode_chunks.restype = ctypes.c_int
        lib.ape_attention_prefill.argtypes = [ctypes.POINTER(ApeShape), ctypes.POINTER(ApeRequest), vp, i32, vp, vp,
                                              vp, sz, vp]
        lib.ape_attention_prefill.restype = ctypes.c_int
        lib.ape_attention_prefill_batch.argtypes = [ctypes.POINTER(ApeShape), ctypes.POINTER(ApeRequest), i32, vp, i32, vp, vp,
                                                    vp, sz, vp]
        lib.ape_attention_prefill_batch.restype = ctypes.c_int
        lib.ape_attention_decode.argtypes = [ctypes.POINTER(ApeShape), ctypes.POINTER(ApeRequest), i32, vp, vp, vp,
                                             vp, sz, vp]
        lib.ape_attention_decode.restype = ctypes.c_int
        lib.ape_attention_decode_static.argtypes = [ctypes.POINTER(ApeShape), ctypes.POINTER(ApeRequest), i32, vp, vp, vp, vp]
        lib.ape_attention_decode_static.restype = ctypes.c_int
        lib.ape_tree_workspace_bytes.argtypes = [ctypes.POINTER(ApeShape), i32, i32, i32]
        lib.ape_tree_workspace_bytes.restype = sz
        lib.ape_attention_tree.argtypes = [ctypes.POINTER(ApeShape), ctypes.POINTER(ApeRequest), vp, vp, i32,
                                           vp, i32, vp, vp, vp, sz, vp]
        lib.ape_attention_tree.restype = ctypes.c_int
        lib.ape_rope_write_cache.argtypes = [ctypes.POINTER(ApeShape), vp, vp, vp, vp, vp, i32, i32, ctypes.c_float,
                                             vp, vp, vp, vp]
        lib.ape_rope_write_cache.restype = ctypes.c_int
        lib.ape_status_string.argtypes = [ctypes.c_int]
        lib.ape_status_string.restype = ctypes.c_char_p
        lib.ape_last_error.restype = ctypes.c_char_p
        lib.ape_version.restype = ctypes.c_char_p
        _lib = lib
    return _lib


_layer_lib = None


def load_layer() -> ctypes.CDLL:
    """Load the layer library (rocBLAS-backed layers around the attention); raises if it has not been built."""
    global _layer_lib
    if _layer_lib is None:
        load()                                         # the attention library first: the layer library links against it
        if not os.path.exists(LAYER_LIB_PATH):
            raise RuntimeError("%s is missing: build it with `python -m paper_2502_05431_amd.build`" % LAYER_LIB_PATH)
        lib = ctypes.CDLL(LAYER_LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        lib.ape_layer_workspace_bytes.argtypes = [ctypes.POINTER(ApeShape), i32, i32, i32]
        lib.ape_layer_workspace_bytes.restype = sz
        lib.ape_layers_workspace_bytes.argtypes = [ctypes.POINTER(ApeShape), i32, i32, i32, i32]
        lib.ape_layers_workspace_bytes.restype = sz
        lib.ape_layer_encode.argtypes = [ctypes.POINTER(ApeShape), ctypes.POINTER(ApeLayerWeights), vp, vp, vp, i32,
                                         vp, vp, i32, vp, vp, vp, ctypes.POINTER(ApeLayerTaps), vp, sz, vp]
        lib.ape_layer_encode.restype = ctypes.c_int
        lib.ape_layers_encode.argtypes = [ctypes.POINTER(ApeShape), ctypes.POINTER(ApeLayerWeights), i32, vp, vp, vp, i32,
                                          vp, vp, i32, vp, vp, vp, vp, sz, vp]
        lib.ape_layers_encode.restype = ctypes.c_int
        _layer_lib = lib
    return _layer_lib


_probe_lib = None


def load_probe() -> ctypes.CDLL:
    """Load the probe library (microbenchmarks of the box's ceilings, used by bench.py)."""
    global _probe_lib
    if _probe_lib is None:
        if not os.path.exists(PROBE_LIB_PATH):
            raise RuntimeError("%s is missing: build it with `python -m paper_2502_05431_amd.build`" % PROBE_LIB_PATH)
        lib = ctypes.CDLL(PROBE_LIB_PATH)
        vp = ctypes.c_void_p
        lib.ape_probe_mfma.argtypes = [vp, ctypes.c_int, vp, ctypes.c_float, vp, ctypes.POINTER(ctypes.c_double)]
        lib.ape_probe_mfma.restype = ctypes.c_int
        lib.ape_probe_hbm_read.argtypes = [vp, ctypes.c_size_t, vp, ctypes.c_float, vp, ctypes.POINTER(ctypes.c_double)]
        lib.ape_probe_hbm_read.restype = ctypes.c_int
        lib.ape_probe_valu_issue.argtypes = [ctypes.c_int, vp, ctypes.c_float, vp, ctypes.POINTER(ctypes.c_double)]
        lib.ape_probe_valu_issue.restype = ctypes.c_int
        _probe_lib = lib
    return _probe_lib


def probe_mfma(operands: torch.Tensor, level, sink: torch.Tensor, warm_ms: float = 150.0, stream=None) -> float:
    """``ape_probe_mfma``: TFLOP/s of back-to-back bf16 MFMAs on the given 64 KiB of operand data; level 0..4
    adds the softmax's vector work, LDS operand reads, a block loop's loads and barrier; 4 is the narrow tile's loop."""
    assert operands.is_cuda and operands.numel() * operands.element_size() >= 65536
    out = ctypes.c_double(0.0)
    if load_probe().ape_probe_mfma(_ptr(operands), int(level), _ptr(sink), warm_ms, _stream(stream), ctypes.byref(out)):
        raise RuntimeError("ape_probe_mfma failed")
    return out.value


def probe_valu_issue(waves_per_simd: int, sink: torch.Tensor, warm_ms: float = 50.0, stream=None) -> float:
    """``ape_probe_valu_issue``: ns per softmax vector instruction per SIMD with 1, 2 or 4 wavefronts per SIMD."""
    out = ctypes.c_double(0.0)
    if load_probe().ape_probe_valu_issue(int(waves_per_simd), _ptr(sink), warm_ms, _stream(stream), ctypes.byref(out)):
        raise RuntimeError("ape_probe_valu_issue failed")
    return out.value


def probe_hbm_read(buf: torch.Tensor, sink: torch.Tensor, warm_ms: float = 150.0, stream=None) -> float:
    """``ape_probe_hbm_read``: GB/s of a read-only kernel over ``buf``."""
    out = ctypes.c_double(0.0)
    if load_probe().ape_probe_hbm_read(_ptr(buf), buf.numel() * buf.element_size(), _ptr(sink), warm_ms, _stream(stream), ctypes.byref(out)):
        raise RuntimeError("ape_probe_hbm_read failed")
    return out.value


def _check(rc: int):
    if rc != APE_OK:
        lib = load()
        raise ApeError(rc, "%s: %s" % (lib.ape_status_string(rc).decode(), lib.ape_last_error().decode()))


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_contiguous(), "tensors handed to the library must be contiguous"
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def make_shape(n_q_heads: int, n_kv_heads: int, head_dim: int, dtype, generic: bool = False) -> ApeShape:
    code = {torch.float32: APE_F32, torch.bfloat16: APE_BF16}.get(dtype, dtype)
    if not isinstance(code, int):
        raise ValueError("dtype must be torch.float32 or torch.bfloat16")
    return ApeShape(n_q_heads, n_kv_heads, head_dim, code | (APE_DTYPE_FLAG_GENERIC if generic else 0))


def workspace_bytes(op: int, shape: ApeShape, batch: int = 1, q_len: int = 1, max_total_kv: int = -1) -> int:
    """``ape_workspace_bytes``; ``max_total_kv`` = longest context the workspace will serve (-1: any)."""
    return int(load().ape_workspace_bytes(op, ctypes.byref(shape), batch, q_len, max_total_kv))


@dataclass
class Request:
    """One request's KV for ``attention_prefill`` / ``attention_decode``: holds the device
    tensors (keeping them alive) and the device-resident chunk table."""
    k_prefix: Optional[torch.Tensor]
    v_prefix: Optional[torch.Tensor]
    k_chunks: Sequence[torch.Tensor]
    v_chunks: Sequence[torch.Tensor]
    k_self: torch.Tensor
    v_self: torch.Tensor
    self_len: int
    temperature: float
    scale: float
    _k_table: Optional[torch.Tensor] = field(default=None, repr=False)
    _v_table: Optional[torch.Tensor] = field(default=None, repr=False)
    _cu: Optional[torch.Tensor] = field(default=None, repr=False)
    total_ctx_len: int = 0

    def __post_init__(self):
        dev = self.k_self.device
        n = len(self.k_chunks)
        assert n == len(self.v_chunks)
        if n:
            for t in list(self.k_chunks) + list(self.v_chunks):
                assert t.is_contiguous()
            self._k_table = torch.tensor([t.data_ptr() for t in self.k_chunks], dtype=torch.int64, device=dev)
            self._v_table = torch.tensor([t.data_ptr() for t in self.v_chunks], dtype=torch.int64, device=dev)
            cu = [0]
            for t in self.k_chunks:
                cu.append(cu[-1] + t.shape[0])
            self.total_ctx_len = cu[-1]
            self._cu = torch.tensor(cu, dtype=torch.int32, device=dev)

    def as_struct(self, self_len: Optional[int] = None) -> ApeRequest:
        r = ApeRequest()
        lp = 0 if self.k_prefix is None else self.k_prefix.shape[0]
        r.k_prefix = self.k_prefix.data_ptr() if lp else None
        r.v_prefix = self.v_prefix.data_ptr() if lp else None
        r.prefix_len = lp
        r.n_chunks = len(self.k_chunks)
        r.k_chunks = self._k_table.data_ptr() if self._k_table is not None else None
        r.v_chunks = self._v_table.data_ptr() if self._v_table is not None else None
        r.cu_chunk_lens = self._cu.data_ptr() if self._cu is not None else None
        r.total_ctx_len = self.total_ctx_len
        r.self_len = self.self_len if self_len is None else self_len
        r.k_self = self.k_self.data_ptr()
        r.v_self = self.v_self.data_ptr()
        r.temperature = self.temperature
        r.scale = self.scale
        return r


def encode_chunks(shape: ApeShape, q_prefix, k_prefix, v_prefix, q_chunks, k_chunks, v_chunks,
                  cu_chunk_lens: Sequence[int], cu_chunk_lens_dev: Optional[torch.Tensor],
                  o_prefix, o_chunks, lse_prefix=None, lse_chunks=None, workspace=None, stream=None):
    """``ape_encode_chunks``: packed contexts [M, H, d]; ``cu_chunk_lens`` is the host prefix-sum list,
    ``cu_chunk_lens_dev`` its int32 device copy."""
    n_chunks = len(cu_chunk_lens) - 1 if cu_chunk_lens is not None and len(cu_chunk_lens) else 0
    cu_host = (ctypes.c_int32 * (n_chunks + 1))(*cu_chunk_lens) if n_chunks else None
    prefix_len = 0 if k_prefix is None else k_prefix.shape[0]
    rc = load().ape_encode_chunks(ctypes.byref(shape), _ptr(q_prefix), _ptr(k_prefix), _ptr(v_prefix), prefix_len,
                                  _ptr(q_chunks), _ptr(k_chunks), _ptr(v_chunks),
                                  ctypes.cast(cu_host, ctypes.c_void_p) if cu_host is not None else None,
                                  _ptr(cu_chunk_lens_dev), n_chunks,
                                  _ptr(o_prefix), _ptr(o_chunks), _ptr(lse_prefix), _ptr(lse_chunks),
                                  _ptr(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(),
                                  _stream(stream))
    _check(rc)


def attention_prefill(shape: ApeShape, req: Request, q: torch.Tensor, out: torch.Tensor,
                      lse_out: Optional[torch.Tensor], workspace: torch.Tensor, stream=None, self_len=None):
    """``ape_attention_prefill``: q/out [q_len, Hq, d]; lse_out fp32 [Hq, q_len] or None."""
    r = req.as_struct(self_len)
    rc = load().ape_attention_prefill(ctypes.byref(shape), ctypes.byref(r), _ptr(q), q.shape[0], _ptr(out), _ptr(lse_out),
                                      _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc)


def attention_prefill_batch(shape: ApeShape, reqs: Sequence[Request], q: torch.Tensor, out: torch.Tensor,
                            lse_out: Optional[torch.Tensor], workspace: torch.Tensor, stream=None,
                            self_lens: Optional[Sequence[int]] = None):
    """``ape_attention_prefill_batch``: q/out [batch, q_len, Hq, d]; lse_out fp32 [batch, Hq, q_len] or None."""
    n = len(reqs)
    arr = (ApeRequest * n)(*[r.as_struct(None if self_lens is None else self_lens[i]) for i, r in enumerate(reqs)])
    rc = load().ape_attention_prefill_batch(ctypes.byref(shape), arr, n, _ptr(q), q.shape[1], _ptr(out), _ptr(lse_out),
                                            _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc)


def attention_decode(shape: ApeShape, reqs: Sequence[Request], q: torch.Tensor, out: torch.Tensor,
                     lse_out: Optional[torch.Tensor], workspace: torch.Tensor, stream=None,
                     self_lens: Optional[Sequence[int]] = None):
    """``ape_attention_decode``: q/out [batch, Hq, d]; lse_out fp32 [batch, Hq] or None."""
    n = len(reqs)
    arr = (ApeRequest * n)(*[r.as_struct(None if self_lens is None else self_lens[i]) for i, r in enumerate(reqs)])
    rc = load().ape_attention_decode(ctypes.byref(shape), arr, n, _ptr(q), _ptr(out), _ptr(lse_out),
                                     _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc)


def attention_decode_static(shape: ApeShape, reqs: Sequence[Request], q: torch.Tensor, out: torch.Tensor,
                            lse_out: Optional[torch.Tensor], stream=None, self_lens: Optional[Sequence[int]] = None):
    """``ape_attention_decode_static``: the decode step with the library's own fixed buffer for the
    partial results (no workspace argument, no allocation)."""
    n = len(reqs)
    arr = (ApeRequest * n)(*[r.as_struct(None if self_lens is None else self_lens[i]) for i, r in enumerate(reqs)])
    rc = load().ape_attention_decode_static(ctypes.byref(shape), arr, n, _ptr(q), _ptr(out), _ptr(lse_out), _stream(stream))
    _check(rc)


@dataclass
class Tree:
    """A context tree for ``attention_tree``: the host array of ``ape_tree_node`` and its device copy."""
    host: ctypes.Array
    dev: torch.Tensor
    n_nodes: int


def make_tree(nodes: Sequence, device) -> Tree:
    """``nodes``: sequence of (scale, first, count, leaf_children), node 0 the root."""
    n = len(nodes)
    host = (ApeTreeNode * max(n, 1))(*[ApeTreeNode(float(s), int(f), int(c), 1 if leaf else 0) for s, f, c, leaf in nodes])
    raw = torch.frombuffer(bytearray(bytes(host)), dtype=torch.int32).clone()      # bit copy, 4 words per node
    return Tree(host=host, dev=raw.to(device), n_nodes=n)


def tree_workspace_bytes(shape: ApeShape, total_ctx_len: int, n_nodes: int, q_len: int) -> int:
    return int(load().ape_tree_workspace_bytes(ctypes.byref(shape), total_ctx_len, n_nodes, q_len))


def attention_tree(shape: ApeShape, req: Request, tree: Tree, q: torch.Tensor, out: torch.Tensor,
                   lse_out: Optional[torch.Tensor], workspace: torch.Tensor, stream=None, self_len=None):
    """``ape_attention_tree``: q/out [q_len, Hq, d]; lse_out fp32 [Hq, q_len] or None."""
    r = req.as_struct(self_len)
    rc = load().ape_attention_tree(ctypes.byref(shape), ctypes.byref(r), ctypes.cast(tree.host, ctypes.c_void_p),
                                   _ptr(tree.dev), tree.n_nodes, _ptr(q), q.shape[0], _ptr(out),
                                   _ptr(lse_out), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                   _stream(stream))
    _check(rc)


def rope_write_cache(shape: ApeShape, q_raw, k_raw, v_raw, cu_chunk_lens: Sequence[int], cu_chunk_lens_dev,
                     position_offset: int, rope_base: float, q_rot, k_cache_table, v_cache_table, stream=None):
    """``ape_rope_write_cache``: packed raw rows [M, H, d]; ``k_cache_table`` / ``v_cache_table`` are int64
    device tensors holding one device pointer per segment (or None)."""
    n_chunks = len(cu_chunk_lens) - 1 if cu_chunk_lens is not None and len(cu_chunk_lens) else 0
    cu_host = (ctypes.c_int32 * (n_chunks + 1))(*cu_chunk_lens) if n_chunks else None
    rc = load().ape_rope_write_cache(ctypes.byref(shape), _ptr(q_raw), _ptr(k_raw), _ptr(v_raw),
                                     ctypes.cast(cu_host, ctypes.c_void_p) if cu_host is not None else None,
                                     _ptr(cu_chunk_lens_dev), n_chunks, position_offset, rope_base,
                                     _ptr(q_rot), _ptr(k_cache_table), _ptr(v_cache_table), _stream(stream))
    _check(rc)


def layer_weights(hidden: int, intermediate: int, rms_eps: float, rope_base: float, attn_norm, w_qkv, w_o, mlp_norm,
                  w_gate_up, w_down) -> ApeLayerWeights:
    """``ape_layer_weights`` over device tensors (the caller keeps them alive)."""
    for t in (attn_norm, w_qkv, w_o, mlp_norm, w_gate_up, w_down):
        assert t.is_contiguous()
    return ApeLayerWeights(hidden, intermediate, rms_eps, rope_base, attn_norm.data_ptr(), w_qkv.data_ptr(), w_o.data_ptr(),
                           mlp_norm.data_ptr(), w_gate_up.data_ptr(), w_down.data_ptr())


def layer_workspace_bytes(shape: ApeShape, hidden: int, intermediate: int, total_rows: int, n_layers: int = 1) -> int:
    if n_layers == 1:
        return int(load_layer().ape_layer_workspace_bytes(ctypes.byref(shape), hidden, intermediate, total_rows))
    return int(load_layer().ape_layers_workspace_bytes(ctypes.byref(shape), hidden, intermediate, total_rows, n_layers))


def _cu_host(cu_chunk_lens):
    n_chunks = len(cu_chunk_lens) - 1 if cu_chunk_lens is not None and len(cu_chunk_lens) else 0
    cu_host = (ctypes.c_int32 * (n_chunks + 1))(*cu_chunk_lens) if n_chunks else None
    return n_chunks, cu_host, (ctypes.cast(cu_host, ctypes.c_void_p) if cu_host is not None else None)


def layer_encode(shape: ApeShape, weights: ApeLayerWeights, x, k_prefix, v_prefix, cu_chunk_lens: Sequence[int],
                 cu_chunk_lens_dev, k_cache, v_cache, y, workspace, stream=None, q_rot_tap=None, attn_tap=None):
    """``ape_layer_encode``: x/y [M, hidden]; k_cache/v_cache packed [M, Hkv, d]; the taps, if given,
    receive the rotated queries and the attention output [M, Hq, d]."""
    n_chunks, _keep, cu_ptr = _cu_host(cu_chunk_lens)
    prefix_len = 0 if k_prefix is None else k_prefix.shape[0]
    taps = None
    if q_rot_tap is not None or attn_tap is not None:
        taps = ApeLayerTaps(None if q_rot_tap is None else q_rot_tap.data_ptr(), None if attn_tap is None else attn_tap.data_ptr())
    rc = load_layer().ape_layer_encode(ctypes.byref(shape), ctypes.byref(weights), _ptr(x), _ptr(k_prefix), _ptr(v_prefix), prefix_len,
                                       cu_ptr, _ptr(cu_chunk_lens_dev), n_chunks, _ptr(k_cache), _ptr(v_cache), _ptr(y),
                                       ctypes.byref(taps) if taps is not None else None,
                                       _ptr(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(),
                                       _stream(stream))
    _check(rc)


def layers_encode(shape: ApeShape, weights: Sequence[ApeLayerWeights], x, k_prefix: Optional[Sequence], v_prefix: Optional[Sequence],
                  cu_chunk_lens: Sequence[int], cu_chunk_lens_dev, k_cache: Sequence, v_cache: Sequence, y, workspace, stream=None):
    """``ape_layers_encode``: a stack of layers; per-layer lists of prefix KV (or None) and cache tensors."""
    n_layers = len(weights)
    n_chunks, _keep, cu_ptr = _cu_host(cu_chunk_lens)
    warr = (ApeLayerWeights * n_layers)(*weights)
    table = lambda ts: (ctypes.c_void_p * n_layers)(*[t.data_ptr() for t in ts])
    prefix_len = 0 if not k_prefix else k_prefix[0].shape[0]
    kp = table(k_prefix) if prefix_len else None
    vp = table(v_prefix) if prefix_len else None
    kc, vc = table(k_cache), table(v_cache)
    rc = load_layer().ape_layers_encode(ctypes.byref(shape), warr, n_layers, _ptr(x), kp, vp, prefix_len,
                                        cu_ptr, _ptr(cu_chunk_lens_dev), n_chunks, kc, vc, _ptr(y),
                                        _ptr(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(),
                                        _stream(stream))
    _check(rc)


def decode_call(shape: ApeShape, reqs: Sequence[Request], q, out, lse_out, workspace, stream=None):
    """Pre-marshalled decode call for tight loops: returns ``(fn, structs)`` where ``structs`` is
    the ctypes array of ape_request whose ``self_len`` fields the caller bumps between steps."""
    lib = load()
    n = len(reqs)
    arr = (ApeRequest * n)(*[r.as_struct() for r in reqs])
    sh = ctypes.byref(shape)
    args = (_ptr(q), _ptr(out), _ptr(lse_out), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))

    def fn():
        rc = lib.ape_attention_decode(sh, arr, n, *args)
        if rc != APE_OK:
            _check(rc)
    return fn, arr
