"""Seeded synthetic MoE routing workloads (inputs only).

This module produces the *inputs* of the dispatch/combine path -- token
activations, top-k expert ids and gate weights -- for the five workload shapes
this build is measured on.  It contains none of the method's arithmetic (no
counting, no slot assignment, no row movement, no reduction); both the CPU
oracle's tests and the HIP path's tests feed on the arrays it returns, so the
two sides always see identical bytes.

Shapes follow the paper's evaluation: the low-latency benchmark uses 256
experts, hidden 7168, 128 tokens per rank, top-8, bf16 (Sec. VII-A), and the
high-throughput regime is "4096+ tokens" per rank (Sec. I, Table III).  The
paper's routing traces and model weights are not available; gate logits drawn
from N(0,1) (optionally with a Zipf or hot-rank prior) stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Optional

import numpy as np

EP_LAYOUT_CONCAT = 0  # 2-D [rows, H] output with per-expert counts (HT mode)
EP_LAYOUT_PADDED = 1  # 3-D [E, C, H] expert-major output (LL mode)


@dataclass(frozen=True)
class WorkloadSpec:
    name: str
    config_id: int
    R: int  # simulated ranks
    T: int  # tokens on this rank
    H: int  # hidden size (bf16 elements per row)
    E: int  # experts in total (E % R == 0)
    K: int  # top-k
    prior: str = "uniform"  # "uniform" | "zipf" | "zipf_identity" | "hot_ranks"
    zipf_s: float = 1.2
    hot_ranks: int = 8
    hot_mass: float = 0.5
    expert_scale: bool = True  # stand-in expert: y = x * (1 + e/256); False = identity
    my_rank: int = 0

    @property
    def L(self) -> int:
        return self.E // self.R

    @property
    def row_bytes(self) -> int:
        return 2 * self.H


SPECS: Dict[str, WorkloadSpec] = {
    "tiny": WorkloadSpec("tiny", 1, R=2, T=64, H=256, E=8, K=2, expert_scale=False),
    "ll_decode": WorkloadSpec("ll_decode", 2, R=32, T=128, H=7168, E=256, K=8),
    "ht_prefill": WorkloadSpec("ht_prefill", 3, R=32, T=4096, H=7168, E=256, K=8),
    "skew": WorkloadSpec("skew", 4, R=16, T=4096, H=4096, E=128, K=8, prior="zipf"),
    "skew_rank0": WorkloadSpec("skew_rank0", 4, R=16, T=4096, H=4096, E=128, K=8,
                               prior="zipf_identity"),
    "stress": WorkloadSpec("stress", 5, R=64, T=8192, H=7168, E=256, K=8),
    "stress_hot": WorkloadSpec("stress_hot", 5, R=64, T=8192, H=7168, E=256, K=8,
                               prior="hot_ranks"),
}


@dataclass
class Workload:
    spec: WorkloadSpec
    x_bits: np.ndarray  # uint16 [T, H]   bf16 bit patterns of the token activations
    topk_idx: np.ndarray  # int32 [T, K]  expert ids, descending gate probability
    topk_w: np.ndarray  # float32 [T, K]  gate weights renormalised over the top-k
    log_prior: Optional[np.ndarray] = field(default=None)  # float32 [E] or None


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 bit patterns (round-to-nearest-even, NaN kept quiet)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    nan = np.isnan(a)
    if nan.any():
        r = np.where(nan, (u >> np.uint32(16)) | np.uint32(0x40), r)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _log_prior(spec: WorkloadSpec, seed: int) -> Optional[np.ndarray]:
    E = spec.E
    if spec.prior == "uniform":
        return None
    if spec.prior in ("zipf", "zipf_identity"):
        if spec.prior == "zipf":
            perm = np.random.default_rng(seed).permutation(E)
        else:
            perm = np.arange(E)
        prior = (perm.astype(np.float64) + 1.0) ** (-spec.zipf_s)
        prior /= prior.sum()
        return np.log(prior).astype(np.float32)
    if spec.prior == "hot_ranks":
        hot = np.sort(np.random.default_rng(seed).permutation(spec.R)[: spec.hot_ranks])
        is_hot = np.isin(np.arange(E) // spec.L, hot)
        n_hot = int(is_hot.sum())
        prior = np.where(is_hot, spec.hot_mass / n_hot, (1.0 - spec.hot_mass) / (E - n_hot))
        return np.log(prior).astype(np.float32)
    raise ValueError(f"unknown prior {spec.prior!r}")


def make_routing(spec: WorkloadSpec, T: Optional[int] = None, seed_offset: int = 0):
    """Top-k expert ids and renormalised gate weights from seeded gate logits.

    logits ~ N(0,1) (+ log prior); p = softmax(logits); the K largest p are
    taken in descending order, ties going to the lower expert id; weights are
    p_topk / sum(p_topk) in float32.
    """
    T = spec.T if T is None else T
    seed = 2000 + spec.config_id + spec.my_rank + seed_offset
    rng = np.random.default_rng(seed)
    logits = rng.standard_normal((T, spec.E), dtype=np.float32)
    lp = _log_prior(spec, 3000 + spec.config_id)
    if lp is not None:
        logits = logits + lp[None, :]
    m = logits.max(axis=1, keepdims=True) if T else logits
    p = np.exp(logits - m, dtype=np.float32)
    p = p / p.sum(axis=1, keepdims=True, dtype=np.float32)
    order = np.argsort(-p, axis=1, kind="stable")[:, : spec.K]
    topk_idx = order.astype(np.int32)
    pk = np.take_along_axis(p, order, axis=1).astype(np.float32)
    topk_w = (pk / pk.sum(axis=1, keepdims=True, dtype=np.float32)).astype(np.float32)
    return np.ascontiguousarray(topk_idx), np.ascontiguousarray(topk_w), lp


def make_tokens(spec: WorkloadSpec, T: Optional[int] = None, seed_offset: int = 0) -> np.ndarray:
    """bf16 bit patterns of x[T, H] ~ N(0,1), seed 1000 + config id."""
    T = spec.T if T is None else T
    rng = np.random.default_rng(1000 + spec.config_id + seed_offset)
    out = np.empty((T, spec.H), dtype=np.uint16)
    step = max(1, (1 << 24) // max(spec.H, 1))
    for t0 in range(0, T, step):
        t1 = min(T, t0 + step)
        out[t0:t1] = f32_to_bf16_bits(rng.standard_normal((t1 - t0, spec.H), dtype=np.float32))
    return out


def make_workload(name_or_spec, T: Optional[int] = None, seed_offset: int = 0, **overrides) -> Workload:
    spec = SPECS[name_or_spec] if isinstance(name_or_spec, str) else name_or_spec
    if overrides:
        spec = replace(spec, **overrides)
    if T is not None:
        spec = replace(spec, T=T)
    topk_idx, topk_w, lp = make_routing(spec, seed_offset=seed_offset)
    x_bits = make_tokens(spec, seed_offset=seed_offset)
    return Workload(spec=spec, x_bits=x_bits, topk_idx=topk_idx, topk_w=topk_w, log_prior=lp)


def expert_scale_table(spec: WorkloadSpec) -> np.ndarray:
    """Per-expert multiplier of the stand-in expert network: 1 + e/256 (1 for identity)."""
    if not spec.expert_scale:
        return np.ones(spec.E, dtype=np.float32)
    return (np.float32(1.0) + np.arange(spec.E, dtype=np.float32) / np.float32(256.0)).astype(np.float32)


def algorithmic_bytes(spec: WorkloadSpec, rows: Optional[int] = None) -> Dict[str, int]:
    """Bytes the method itself must move per call (inputs read once, outputs written once).

    dispatch: T rows read, M rows written, 8 bytes of map/weight per routed entry.
    combine : M rows read, T rows written, 8 bytes of map/weight per routed entry.
    layout  : 4 bytes per entry in, about 16 per entry plus 4 per expert out.
    """
    M = spec.T * spec.K if rows is None else rows
    row = spec.row_bytes
    return {
        "layout": 4 * spec.T * spec.K + 16 * spec.T * spec.K + 4 * spec.E,
        "dispatch": spec.T * row + M * row + 8 * M,
        "combine": M * row + spec.T * row + 8 * M,
    }
