"""Seeded synthetic workloads shaped like the paper's attention benchmarks.

This module only draws random tensors; it holds none of the method's arithmetic
(no means, scores, quantisation or softmax) so that both the CPU oracle's tests
and the HIP path can be fed exactly the same bits.

Shapes follow the paper's kernel benchmark (batch 1, 32 heads, head_dim 128,
context up to 131072; Fig. 4 caption and App. B "Context, and decoding") and a
Qwen3-8B layer (32 query heads sharing 8 KV heads).  The value structure is
planted to mimic what Sec. 3.1 attributes to real attention: a few key blocks
with much larger scores than the rest, attention sinks at the first positions,
and a handful of outlier channels.

Every tensor is generated on the CPU with a per-head ``torch.Generator`` seeded
``seed * 1000003 + stream * 4099 + head`` and cast once to fp16 / bf16.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional, Sequence, Tuple

import torch


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    B: int
    Hq: int
    Hkv: int
    N: int
    D: int
    dtype: str  # "f16" | "bf16"
    Bq: int
    Bk: int
    causal: bool
    budgets: Tuple[float, ...]
    seed: int = 0
    outlier_channels: int = 4
    outlier_scale: float = 8.0
    planted_blocks: int = 0
    planted_gain: float = 24.0
    sink_tokens: int = 0
    sink_gain: float = 6.0
    query_mean_gain: float = 2.0
    heavy_tail_nu: float = 0.0  # 0 -> Gaussian keys; >0 -> Student-t keys
    # decode only
    decode: bool = False
    split_blocks: int = 256

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float16 if self.dtype == "f16" else torch.bfloat16

    @property
    def group(self) -> int:
        return self.Hq // self.Hkv


# The five configurations the benchmark description names, in its order.
TINY = Workload("tiny_causal_prefill", 1, 1, 1, 2048, 128, "f16", 64, 64, True, (0.05,),
                seed=0, planted_blocks=2)
QWEN3_32K = Workload("qwen3_8b_prefill_32k", 1, 32, 8, 32768, 128, "bf16", 128, 64, True, (0.05,),
                     seed=0, sink_tokens=4)
QWEN3_131K = Workload("qwen3_8b_prefill_131k", 1, 32, 8, 131072, 128, "bf16", 128, 64, True,
                      (0.05, 0.10, 0.25), seed=0, sink_tokens=4)
DECODE_131K = Workload("qwen3_8b_decode_131k", 16, 32, 8, 131072, 128, "f16", 1, 64, False, (0.05,),
                       seed=0, sink_tokens=4, decode=True, split_blocks=256)
SKEWED_64K = Workload("skewed_prefill_64k", 1, 64, 8, 65536, 128, "bf16", 128, 64, True,
                      (0.0, 0.01, 0.02, 0.05, 0.10, 0.25, 1.0), seed=0, outlier_channels=8,
                      outlier_scale=12.0, planted_blocks=16, heavy_tail_nu=3.0)

CONFIGS: Dict[str, Workload] = {w.name: w for w in (TINY, QWEN3_32K, QWEN3_131K, DECODE_131K, SKEWED_64K)}


def scaled(w: Workload, **kw) -> Workload:
    """Copy of a workload with some fields replaced (smaller N, fewer heads...)."""
    return dataclasses.replace(w, **kw)


def _gen(seed: int, stream: int, head: int, device="cpu") -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed * 1000003 + stream * 4099 + head)
    return g


def _unit(g: torch.Generator, D: int) -> torch.Tensor:
    u = torch.randn(D, generator=g, dtype=torch.float32)
    return u / u.norm()


def _randn(n, d, g: torch.Generator) -> torch.Tensor:
    return torch.randn(n, d, generator=g, dtype=torch.float32, device=g.device)


def group_direction(w: Workload, b: int, kvh: int) -> torch.Tensor:
    """Unit vector shared by the query heads of one KV group (fp32, [D])."""
    return _unit(_gen(w.seed, 7, b * w.Hkv + kvh), w.D)


def planted_block_ids(w: Workload, b: int, kvh: int) -> List[int]:
    """Key-block ids that receive the planted bias (none in block 0 or the last block)."""
    if w.planted_blocks <= 0:
        return []
    Tk = w.N // w.Bk
    g = _gen(w.seed, 11, b * w.Hkv + kvh)
    perm = torch.randperm(max(Tk - 2, 1), generator=g) + 1
    return sorted(int(x) for x in perm[: min(w.planted_blocks, Tk - 2)])


def _outlier_idx(w: Workload, stream: int, b: int, head: int) -> torch.Tensor:
    g = _gen(w.seed, stream, b * 4096 + head)
    return torch.randperm(w.D, generator=g)[: w.outlier_channels]


def make_q_head(w: Workload, b: int, h: int, n_rows: Optional[int] = None, device="cpu") -> torch.Tensor:
    """Queries of one head: [N, D] (or [n_rows, D]) in the workload's dtype.

    ``device``: where the normal draws are made.  The CPU and the GPU generators give different
    (equally distributed) bits, so parity checks draw on the CPU and copy; the throughput runs may
    draw on the GPU.  The planted structure (directions, channels, block ids) is always drawn on the CPU.
    """
    n = w.N if n_rows is None else n_rows
    g = _gen(w.seed, 1, b * w.Hq + h, device)
    q = _randn(n, w.D, g)
    q += w.query_mean_gain * group_direction(w, b, h // w.group).to(q.device)
    if w.outlier_channels:
        q[:, _outlier_idx(w, 3, b, h).to(q.device)] *= w.outlier_scale
    return q.to(w.torch_dtype)


def make_kv_head(w: Workload, b: int, kvh: int, device="cpu") -> Tuple[torch.Tensor, torch.Tensor]:
    """Keys and values of one KV head: two [N, D] tensors in the workload's dtype."""
    g = _gen(w.seed, 2, b * w.Hkv + kvh, device)
    if w.heavy_tail_nu > 0:
        nu = int(w.heavy_tail_nu)
        z = _randn(w.N, w.D, g)
        chi = torch.zeros_like(z)
        for _ in range(nu):
            chi += _randn(w.N, w.D, g) ** 2
        k = z / torch.sqrt(chi / nu) / math.sqrt(nu / (nu - 2.0))
    else:
        k = _randn(w.N, w.D, g)
    v = _randn(w.N, w.D, g)
    if w.outlier_channels:
        k[:, _outlier_idx(w, 5, b, kvh).to(k.device)] *= w.outlier_scale
    u = group_direction(w, b, kvh).to(k.device)
    for blk in planted_block_ids(w, b, kvh):
        k[blk * w.Bk:(blk + 1) * w.Bk] += w.planted_gain * u
    if w.sink_tokens:
        k[: w.sink_tokens] = w.sink_gain * math.sqrt(w.D) * u
    return k.to(w.torch_dtype), v.to(w.torch_dtype)


def make_prefill(w: Workload, q_heads: Optional[Sequence[int]] = None, device="cpu"):
    """Full prefill tensors: q [B,Hq',N,D], k,v [B,Hkv',N,D] on the CPU.

    ``q_heads`` restricts generation to some query heads (and the KV heads they
    use, re-indexed densely) so that large shapes can be checked on a subset.
    Returns (q, k, v, q_head_ids, kv_head_ids).
    """
    assert not w.decode
    qh = list(range(w.Hq)) if q_heads is None else list(q_heads)
    kvh = sorted({h // w.group for h in qh})
    if q_heads is not None:
        # a subset must keep whole groups so that the GQA mapping h -> h // group survives
        assert all(sorted(h for h in qh if h // w.group == g) == list(range(g * w.group, (g + 1) * w.group)) for g in kvh)
    q = torch.empty(w.B, len(qh), w.N, w.D, dtype=w.torch_dtype, device=device)
    k = torch.empty(w.B, len(kvh), w.N, w.D, dtype=w.torch_dtype, device=device)
    v = torch.empty_like(k)
    for b in range(w.B):
        for i, h in enumerate(qh):
            q[b, i] = make_q_head(w, b, h, device=device)
        for i, g in enumerate(kvh):
            k[b, i], v[b, i] = make_kv_head(w, b, g, device=device)
    return q, k, v, qh, kvh


def make_decode(w: Workload, batch: Optional[int] = None, device="cpu"):
    """Decode tensors: q [B,Hq,D] (the query at the last position) and the
    high-precision cache k,v [B,Hkv,N,D]; quantised copies and block means are
    produced by the library under test (or by the oracle), not here."""
    assert w.decode
    B = w.B if batch is None else batch
    q = torch.empty(B, w.Hq, w.D, dtype=w.torch_dtype, device=device)
    k = torch.empty(B, w.Hkv, w.N, w.D, dtype=w.torch_dtype, device=device)
    v = torch.empty_like(k)
    for b in range(B):
        for h in range(w.Hq):
            q[b, h] = make_q_head(w, b, h, n_rows=1, device=device)[0]
        for g in range(w.Hkv):
            k[b, g], v[b, g] = make_kv_head(w, b, g, device=device)
    return q, k, v
