"""Several simulated source ranks sending into ONE receiver-shaped tensor (test glue).

What a receiver holds after every source has dispatched is fixed by the ordering rule alone:
within an expert's region the rows come in (source rank, token index) order (k order for a
token that names the expert twice).  `expected_receiver` writes that down directly -- a stable
sort of all entries of all sources by (expert, source rank, token, k) -- without calling the
oracle; the tests compare it with the composition of per-source oracle calls (CPU) and the
composition of per-source HIP dispatches (GPU).

Two receiver layouts (Sec. III-E): padded [E, R*C, H], where source r owns columns
[r*C, (r+1)*C) of every expert (Sec. IV-B sub-regions, no exchange needed), and concatenated
[rows, H], where source r's rows of expert e start at the expert's first row plus the rows of
the lower-ranked sources (what the handle-time metadata exchange of Sec. III-C delivers, here
computed from the sources' routings and handed to the layout as expert_base)."""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np

from paper_2603_13606_amd import workloads as wl


@dataclass
class Source:
    rank: int
    topk: np.ndarray    # int32 [T, K], -1 = not routed
    w: np.ndarray       # float32 [T, K]
    x_bits: np.ndarray  # uint16 [T, H]


def make_sources(spec: wl.WorkloadSpec, n_src: int, tokens: List[int], masked: float = 0.02) -> List[Source]:
    """n_src seeded sources with their own routing, tokens and (ragged) token counts."""
    out = []
    for r in range(n_src):
        T = tokens[r % len(tokens)]
        topk, w, _ = wl.make_routing(spec, T=T, seed_offset=1000 + 17 * r)
        rng = np.random.default_rng(500 + r)
        topk = topk.copy()
        topk[rng.random(topk.shape) < masked] = -1
        out.append(Source(r, topk, w, wl.make_tokens(spec, T=T, seed_offset=1000 + 17 * r)))
    return out


def expert_bases(sources: List[Source], E: int) -> np.ndarray:
    """int32 [n_src, E]: first row of source r's rows of expert e in the concatenated receiver."""
    counts = np.array([np.bincount(s.topk[(s.topk >= 0) & (s.topk < E)], minlength=E) for s in sources])
    start = np.concatenate([[0], np.cumsum(counts.sum(0))])[:-1]
    lower = np.cumsum(counts, axis=0) - counts  # rows of lower-ranked sources per expert
    return (start[None, :] + lower).astype(np.int32)


def expected_receiver(sources: List[Source], E: int, H: int, padded: bool, C: int, fill: int):
    """(rows, recv_src, recv_w, recv_rank) of the receiver by a stable sort of all entries by
    (expert, source rank, token, k).  rows: uint16 [E*R*C, H] (padded) or [total, H]."""
    ent = []
    for s in sources:
        T, K = s.topk.shape
        for t in range(T):
            for k in range(K):
                e = int(s.topk[t, k])
                if 0 <= e < E:
                    ent.append((e, s.rank, t, k))
    ent.sort()  # tuples sort lexicographically; all keys distinct
    n_src = len(sources)
    nrows = E * n_src * C if padded else len(ent)
    rows = np.full((nrows, H), fill, np.uint16)
    src = np.full(nrows, -9, np.int32)
    wgt = np.full(nrows, np.float32(-3.5), np.float32)
    rank = np.full(nrows, -1, np.int32)
    seen = {}
    for pos, (e, r, t, k) in enumerate(ent):
        if padded:
            slot = seen.get((e, r), 0)
            seen[(e, r)] = slot + 1
            if slot >= C:
                continue
            row = (e * n_src + r) * C + slot
        else:
            row = pos
        rows[row] = sources[r].x_bits[t]
        src[row] = t
        wgt[row] = sources[r].w[t, k]
        rank[row] = r
    return rows, src, wgt, rank
