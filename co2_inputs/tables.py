"""Segment tables and workload configurations (no arithmetic of the method).

A segment table is a list of S+1 non-decreasing int64 offsets into the flat
parameter vector, one segment per parameter tensor.  The shapes below are
synthetic stand-ins for the GPT-2-style and 7B-class models the CO2 paper trains
(its Table 5): tensor sizes only, no weights or data.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional


def _offsets(sizes: List[int]) -> List[int]:
    off = [0]
    for s in sizes:
        off.append(off[-1] + int(s))
    return off


def equal_table(n: int, S: int) -> List[int]:
    """S equal segments (the last absorbs any remainder)."""
    base = n // S
    sizes = [base] * S
    sizes[-1] += n - base * S
    return _offsets(sizes)


def gpt_table(layers: int, d: int, ffn: int, vocab: int, ctx: int) -> List[int]:
    """GPT-2-style decoder with learned positions and biases:
    tok-emb, pos-emb, per layer {ln1 w,b; qkv W,b; proj W,b; ln2 w,b; fc W,b;
    fc-proj W,b}, final ln w,b."""
    sizes = [vocab * d, ctx * d]
    for _ in range(layers):
        sizes += [d, d, d * 3 * d, 3 * d, d * d, d, d, d, d * ffn, ffn, ffn * d, d]
    sizes += [d, d]
    return _offsets(sizes)


def llama_table(layers: int, d: int, ffn: int, vocab: int) -> List[int]:
    """Bias-free gated-MLP decoder: emb, per layer {norm, q, k, v, o, norm, gate,
    up, down}, final norm, untied head."""
    sizes = [vocab * d]
    for _ in range(layers):
        sizes += [d, d * d, d * d, d * d, d * d, d, d * ffn, d * ffn, ffn * d]
    sizes += [d, vocab * d]
    return _offsets(sizes)


def shard_of_table(table: List[int], rank: int, world: int) -> List[int]:
    """Segment table of one contiguous 1/world slice of a flat vector (a
    ZeRO-style shard): boundaries of the full table that fall strictly inside
    the slice, re-based to the slice's start.  First and last segment may be
    partial tensors."""
    n = table[-1]
    assert n % world == 0
    lo, hi = rank * (n // world), (rank + 1) * (n // world)
    inner = [o - lo for o in table if lo < o < hi]
    return [0] + inner + [hi - lo]


@dataclass
class WorkloadConfig:
    name: str
    K: int
    beta: float
    phi: float
    c: float
    alpha: float = 1.0
    tau: int = 4
    steps: int = 1
    drift: str = "normal"        # "normal" | "student_t"
    drift_scale: float = 1e-3
    drift_nu: int = 3
    param_std: float = 0.02
    momentum_std: float = 0.02
    seed: int = 0
    table_args: dict = field(default_factory=dict)
    # AdamW leg (overlapped-round workload only)
    adamw: Optional[dict] = None


CONFIGS = {
    # n = 2^20 in 8 equal segments, K = 4.
    "tiny": WorkloadConfig(name="tiny", K=4, beta=0.9, phi=1.0, c=0.5, steps=1,
                           momentum_std=0.02,
                           table_args=dict(kind="equal", n=1 << 20, S=8)),
    # GPT-2-small-shaped, 124 439 808 params in 148 ragged segments, K = 8.
    "gpt2s": WorkloadConfig(name="gpt2s", K=8, beta=0.9, phi=1.0, c=0.5, steps=10,
                            momentum_std=1e-4,
                            table_args=dict(kind="gpt", layers=12, d=768, ffn=3072,
                                            vocab=50257, ctx=1024)),
    # 1.3B-shaped, 1 343 868 928 params in 292 segments, K = 8, heavy-tailed drift.
    "1p3b": WorkloadConfig(name="1p3b", K=8, beta=0.95, phi=0.5, c=1.0, steps=20,
                           drift="student_t", drift_scale=1e-3, drift_nu=3,
                           momentum_std=1e-4,
                           table_args=dict(kind="gpt", layers=24, d=2048, ffn=8192,
                                           vocab=64000, ctx=2048)),
    # One 1/16 slice of a 7B-shaped model (6 738 415 616 / 16 = 421 150 976).
    "7b_shard": WorkloadConfig(name="7b_shard", K=8, beta=0.9, phi=1.0, c=1.0, steps=20,
                               drift_scale=5e-4, momentum_std=1e-4,
                               table_args=dict(kind="llama_shard", layers=32, d=4096,
                                               ffn=11008, vocab=32000, rank=1, world=16)),
    # 350M-shaped model for the overlapped round (tau AdamW steps + outer step).
    "350m_overlap": WorkloadConfig(name="350m_overlap", K=8, beta=0.9, phi=1.0, c=1.0,
                                   steps=50, tau=4, momentum_std=1e-4,
                                   table_args=dict(kind="gpt", layers=24, d=1024, ffn=4096,
                                                   vocab=50257, ctx=1024),
                                   adamw=dict(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8,
                                              weight_decay=0.1, grad_std=1e-3)),
}


def config_table(cfg: WorkloadConfig, rank: Optional[int] = None) -> List[int]:
    a = dict(cfg.table_args)
    kind = a.pop("kind")
    if kind == "equal":
        return equal_table(a["n"], a["S"])
    if kind == "gpt":
        return gpt_table(**a)
    if kind == "llama_shard":
        r = a.pop("rank")
        world = a.pop("world")
        if rank is not None:
            r = rank
        return shard_of_table(llama_table(**a), r, world)
    raise ValueError(kind)
