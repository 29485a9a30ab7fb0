"""Seeded synthetic inputs for the APE attention path.

This module serves both the HIP library's tests/bench and the CPU oracle, and
therefore holds NONE of the method's arithmetic (no attention, no softmax, no
temperature, no scaling factor): it only draws Q/K/V arrays with the shapes and
value structure of the five benchmark workloads and lays them out as
``[tokens, heads, head_dim]``.

The workloads stand in for the settings the paper (arXiv 2502.05431) evaluates
-- retrieval-augmented generation with tens of chunks, many-shot in-context
learning with hundreds, the 128K-context efficiency study (Section 5.4) and
batched serving -- whose datasets and model weights are not available; only
shapes (Llama-3-8B attention heads) and coarse value structure (key outlier
channels, per-chunk key offsets) are taken.

Position convention (Section 1 / 2.2: every context reuses the same position
range): prefix at 0..l_P-1, every chunk at l_P..l_P+l_i-1, the query starts at
l_P + max_i l_i, generated tokens follow.  Positions matter only to the RoPE
pre-rotation of workload 1; the kernels and the oracle read rotated arrays.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import torch

BASE_SEED = 20250205


@dataclass(frozen=True)
class WorkloadSpec:
    name: str
    cfg: int                       # 1..5: which of the five benchmark configurations
    dtype: str                     # "f32" | "bf16"
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    prefix_len: int
    chunk_lens: Tuple[int, ...]
    q_len: int                     # query-prefill rows (0: decode only)
    decode_steps: int
    batch: int = 1
    temperature: Optional[float] = None      # None: per request ~ U[t_range]
    scale: Optional[float] = None            # None: per request ~ U[s_range]
    t_range: Tuple[float, float] = (0.6, 1.0)
    s_range: Tuple[float, float] = (0.7, 1.0)
    k_scale: float = 1.0                     # multiplies every key
    rope_base: Optional[float] = None        # pre-rotate Q and K (half-split pairing)
    outlier_channels: int = 0                # per KV head, channels of K multiplied by outlier_gain
    outlier_gain: float = 1.0
    chunk_key_mean_std: float = 0.0          # per (chunk, KV head) key offset ~ N(0, std^2)

    @property
    def total_ctx_len(self) -> int:
        return int(sum(self.chunk_lens))

    @property
    def self_len_max(self) -> int:
        return self.q_len + self.decode_steps

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    def replace(self, **kw) -> "WorkloadSpec":
        return dataclasses.replace(self, **kw)


def _llama(name, cfg, **kw) -> WorkloadSpec:
    return WorkloadSpec(name=name, cfg=cfg, dtype="bf16", n_q_heads=32, n_kv_heads=8, head_dim=128, **kw)


CONFIGS = {
    1: WorkloadSpec(name="tiny_fp32", cfg=1, dtype="f32", n_q_heads=4, n_kv_heads=2, head_dim=64,
                    prefix_len=8, chunk_lens=(32,) * 4, q_len=16, decode_steps=4,
                    temperature=0.8, scale=0.9, rope_base=500000.0),
    2: _llama("rag_10k", 2, prefix_len=32, chunk_lens=(512,) * 20, q_len=64, decode_steps=256,
              temperature=0.9, scale=0.9, k_scale=128 ** -0.5),
    3: _llama("ctx_128k", 3, prefix_len=32, chunk_lens=(2048,) * 64, q_len=256, decode_steps=0,
              temperature=0.8, scale=0.85, outlier_channels=4, outlier_gain=8.0),
    4: _llama("manyshot_128k", 4, prefix_len=32, chunk_lens=(256,) * 512, q_len=128, decode_steps=64,
              temperature=0.7, scale=0.8, chunk_key_mean_std=0.5),
    5: _llama("batched_decode", 5, prefix_len=32, chunk_lens=(1024,) * 16, q_len=0, decode_steps=128,
              batch=32),
}


@dataclass
class RequestData:
    """One request's tensors, all ``[tokens, heads, head_dim]`` on one device."""
    q_prefix: torch.Tensor
    k_prefix: torch.Tensor
    v_prefix: torch.Tensor
    q_ctx: torch.Tensor            # packed chunks [M, Hq, d]
    k_ctx: torch.Tensor            # packed chunks [M, Hkv, d]
    v_ctx: torch.Tensor
    chunk_lens: List[int]
    q_self: torch.Tensor           # [q_len + decode_steps, Hq, d]
    k_self: torch.Tensor           # [q_len + decode_steps, Hkv, d]
    v_self: torch.Tensor
    temperature: float
    scale: float
    seed: int = 0
    generator: str = ""

    def chunk_views(self):
        """Per-chunk (k, v) views into the packed arrays."""
        ks, vs, t = [], [], 0
        for li in self.chunk_lens:
            ks.append(self.k_ctx[t:t + li])
            vs.append(self.v_ctx[t:t + li])
            t += li
        return ks, vs


def rope_rotate(x: torch.Tensor, positions: torch.Tensor, base: float) -> torch.Tensor:
    """Rotary position embedding, half-split pairing (x_c, x_{c+d/2}),
    theta_c = base^(-2c/d).  x: [tokens, heads, d] fp32; positions: [tokens]."""
    d = x.shape[-1]
    half = d // 2
    inv = base ** (-torch.arange(half, dtype=torch.float64, device=x.device) * 2.0 / d)
    ang = positions.to(torch.float64)[:, None] * inv[None, :]
    cos, sin = ang.cos()[:, None, :].to(x.dtype), ang.sin()[:, None, :].to(x.dtype)
    x1, x2 = x[..., :half], x[..., half:]
    return torch.cat([x1 * cos - x2 * sin, x2 * cos + x1 * sin], dim=-1)


def request_seed(spec: WorkloadSpec, run_index: int = 0, request: int = 0) -> int:
    return BASE_SEED + 1000 * spec.cfg + run_index + 100003 * request


def make_request(spec: WorkloadSpec, device="cpu", run_index: int = 0, request: int = 0) -> RequestData:
    """Draw one request of ``spec`` (request index matters only for batch > 1)."""
    device = torch.device(device)
    seed = request_seed(spec, run_index, request)
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    hq, hkv, d = spec.n_q_heads, spec.n_kv_heads, spec.head_dim
    lp, m, ls = spec.prefix_len, spec.total_ctx_len, spec.self_len_max

    def normal(n, h):
        return torch.randn((n, h, d), generator=gen, device=device, dtype=torch.float32)

    def uniform(lo, hi):
        return float(lo + (hi - lo) * torch.rand((), generator=gen, device=device, dtype=torch.float32).item())

    t_val = spec.temperature if spec.temperature is not None else uniform(*spec.t_range)
    s_val = spec.scale if spec.scale is not None else uniform(*spec.s_range)

    q_prefix, k_prefix, v_prefix = normal(lp, hq), normal(lp, hkv), normal(lp, hkv)
    q_ctx, k_ctx, v_ctx = normal(m, hq), normal(m, hkv), normal(m, hkv)
    q_self, k_self, v_self = normal(ls, hq), normal(ls, hkv), normal(ls, hkv)

    if spec.chunk_key_mean_std > 0.0:
        # one key offset per (chunk, KV head): varies the attention mass across chunks
        mu = normal(len(spec.chunk_lens), hkv) * spec.chunk_key_mean_std
        reps = torch.tensor(spec.chunk_lens, device=device)
        k_ctx = k_ctx + torch.repeat_interleave(mu, reps, dim=0)

    if spec.outlier_channels > 0:
        # per KV head, a few channels of every key (prefix, chunks, self) are amplified
        gain = torch.ones((hkv, d), device=device, dtype=torch.float32)
        for h in range(hkv):
            ch = torch.randperm(d, generator=gen, device=device)[:spec.outlier_channels]
            gain[h, ch] = spec.outlier_gain
        k_prefix, k_ctx, k_self = k_prefix * gain, k_ctx * gain, k_self * gain

    if spec.k_scale != 1.0:
        k_prefix, k_ctx, k_self = k_prefix * spec.k_scale, k_ctx * spec.k_scale, k_self * spec.k_scale

    if spec.rope_base is not None:
        pos_p = torch.arange(lp, device=device)
        pos_c = torch.cat([lp + torch.arange(li, device=device) for li in spec.chunk_lens]) if m else \
            torch.zeros(0, dtype=torch.long, device=device)
        pos_s = lp + (max(spec.chunk_lens) if spec.chunk_lens else 0) + torch.arange(ls, device=device)
        q_prefix, k_prefix = rope_rotate(q_prefix, pos_p, spec.rope_base), rope_rotate(k_prefix, pos_p, spec.rope_base)
        q_ctx, k_ctx = rope_rotate(q_ctx, pos_c, spec.rope_base), rope_rotate(k_ctx, pos_c, spec.rope_base)
        q_self, k_self = rope_rotate(q_self, pos_s, spec.rope_base), rope_rotate(k_self, pos_s, spec.rope_base)

    dt = spec.torch_dtype
    c = lambda x: x.to(dt).contiguous()
    return RequestData(q_prefix=c(q_prefix), k_prefix=c(k_prefix), v_prefix=c(v_prefix),
                       q_ctx=c(q_ctx), k_ctx=c(k_ctx), v_ctx=c(v_ctx), chunk_lens=list(spec.chunk_lens),
                       q_self=c(q_self), k_self=c(k_self), v_self=c(v_self),
                       temperature=t_val, scale=s_val, seed=seed,
                       generator="torch.Generator(%s).manual_seed" % device.type)


def to_numpy_f32(x: torch.Tensor):
    """Exact fp32 copy of an fp32/bf16 tensor on the host (what the oracle reads)."""
    return x.detach().to(torch.float32).cpu().numpy()


# ---- context trees (Appendix C.5): structure only, (scale, first, count, leaf_children) per node.
# Node 0 is the root; the children of a node are either contexts first..first+count-1 of the
# chunk table or nodes first..first+count-1, and node children are numbered in the order of
# their parents (breadth-first), so every child index is above its parent's.

def tree_pooled(n_chunks: int, scale: float):
    """One node over all contexts: the pooled scaling factor of the main-text equation."""
    return [(float(scale), 0, n_chunks, True)]


def tree_per_context(n_chunks: int, scale: float):
    """Root of scale 1 over one node per context, each with the scaling factor (Appendix C.2)."""
    return [(1.0, 1, n_chunks, False)] + [(float(scale), i, 1, True) for i in range(n_chunks)]


def tree_grouped(n_chunks: int, group: int, root_scale: float, group_scale: float):
    """Two levels: consecutive runs of `group` contexts under one node each."""
    n_groups = (n_chunks + group - 1) // group
    nodes = [(float(root_scale), 1, n_groups, False)]
    for g in range(n_groups):
        first = g * group
        nodes.append((float(group_scale), first, min(group, n_chunks - first), True))
    return nodes


def tree_random(n_chunks: int, seed: int, max_children: int = 4, s_range=(0.6, 1.0)):
    """A random tree of mixed depth over the contexts in table order.  Built top-down: a node
    that owns a run of contexts either takes them as leaf children or deals them out to child
    nodes; breadth-first numbering falls out of the work queue."""
    import random
    rng = random.Random(seed)
    nodes, queue = [], [(0, n_chunks)]
    while queue:
        lo, hi = queue.pop(0)
        scale = rng.uniform(*s_range)
        n = hi - lo
        if n <= 2 or rng.random() < 0.3:
            nodes.append((scale, lo, n, True))
            continue
        k = rng.randint(2, min(max_children, n))
        cuts = sorted(rng.sample(range(lo + 1, hi), k - 1))
        bounds = [lo] + cuts + [hi]
        first_child = len(nodes) + 1 + len(queue)
        nodes.append((scale, first_child, k, False))
        queue.extend((bounds[i], bounds[i + 1]) for i in range(k))
    return nodes
