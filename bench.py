#!/usr/bin/env python3
"""Benchmark of the dispatch/combine hot path on one MI355X.

One step = layout + dispatch + combine (+ handle destroy) over one batch of synthetic
routing.  Inputs (tokens, top-k ids, gate weights, expert outputs) are resident in HBM
before the timed region.  Prints ONE JSON line.

Headline: the high-throughput prefill shape.  By default the group is configured with
EP_ORDER_DESTINATION and the layout call is ep_layout_prefetch (the tokens are announced
to it); --dispatch-order 0 times the token-ordered dispatch with plain ep_layout.  The
same line carries every other workload shape (`all_configs`), the once-per-rank dispatch
and the CPU oracle's rate on the host cores.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload ht_prefill]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
ORDER_NAMES = ["EP_ORDER_TOKEN", "EP_ORDER_DESTINATION + ep_layout_prefetch", "EP_ORDER_DESTINATION_RESIDENT"]


def _profiled(workload: str, kernel: str):
    """What the committed rocprofv3 summaries say about one kernel of one workload: HBM bytes per
    launch (FETCH_SIZE + WRITE_SIZE scaled by the calibration copy) and its average duration,
    with the commit and date of the profiled run.  None when there is no such line."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    meta, found = {}, None
    try:
        with open(path) as f:
            for line in f:
                parts = line.split()
                if line.startswith("#") and len(parts) >= 3 and parts[1] in ("commit", "date", "command"):
                    meta[parts[1]] = " ".join(parts[2:])
                elif len(parts) >= 3 and parts[0] == workload and parts[1] == kernel:
                    found = {"traffic": int(parts[2]), "kernel_us": float(parts[3]) if len(parts) > 3 else None}
    except (OSError, ValueError):
        return None
    if found:
        found.update(meta)
    return found


def cpu_baseline(w, steps_budget_s: float = 12.0):
    """The oracle, as it stands, on this host: same three calls, single thread."""
    import numpy as np

    import oracle
    from paper_2603_13606_amd import workloads as wl

    spec = w.spec
    oracle.build()
    lay = oracle.layout(w.topk_idx, E=spec.E, R=spec.R, C_rank=spec.T)
    rows = int(lay.expert_offset[-1])
    recv = np.zeros((rows, spec.H), np.uint16)
    t_total, reps = 0.0, 0
    while t_total < steps_budget_s and reps < 40:
        t0 = time.perf_counter()
        lay = oracle.layout(w.topk_idx, E=spec.E, R=spec.R, C_rank=spec.T)
        oracle.dispatch(w.x_bits, w.topk_w, lay, recv)
        oracle.combine(recv, w.topk_w, lay, spec.H, acc="f64")
        t_total += time.perf_counter() - t0
        reps += 1
    ab = wl.algorithmic_bytes(spec, rows)
    nbytes = ab["layout"] + ab["dispatch"] + ab["combine"]
    return {
        "value": round(nbytes * reps / t_total / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": f"{reps} full steps (layout+dispatch+combine, T={spec.T}) of the same workload, "
                  f"{t_total / reps * 1e3:.0f} ms each, host has {os.cpu_count()} logical cores",
        "ms_per_step": round(t_total / reps * 1e3, 2),
    }


def cpu_baseline_all_cores(w, threads: int, budget_s: float = 4.0):
    """The same oracle calls with the tokens cut into `threads` contiguous ranges, one Python thread
    per range (the C loops release the interpreter lock): dispatch and combine of different tokens
    touch different rows, the layout stays sequential.  Nothing in the oracle is changed for this."""
    import dataclasses
    from concurrent.futures import ThreadPoolExecutor

    import numpy as np

    import oracle
    from paper_2603_13606_amd import workloads as wl

    spec = w.spec
    T, H = spec.T, spec.H
    oracle.build()
    lay = oracle.layout(w.topk_idx, E=spec.E, R=spec.R, C_rank=T)
    rows = int(lay.expert_offset[-1])
    recv = np.zeros((rows, H), np.uint16)
    out = np.zeros((T, H), np.uint16)
    cuts = [T * i // threads for i in range(threads + 1)]
    parts = [(a, b) for a, b in zip(cuts[:-1], cuts[1:]) if b > a]

    def part(ab, lay):
        a, b = ab
        sub = dataclasses.replace(lay, T=b - a, dst_row=lay.dst_row[a:b])
        oracle.dispatch(w.x_bits[a:b], w.topk_w[a:b], sub, recv)

    def part2(ab, lay):
        a, b = ab
        sub = dataclasses.replace(lay, T=b - a, dst_row=lay.dst_row[a:b])
        out[a:b] = oracle.combine(recv, w.topk_w[a:b], sub, H, acc="f64")

    t_total, reps = 0.0, 0
    with ThreadPoolExecutor(max_workers=threads) as pool:
        while t_total < budget_s and reps < 40:
            t0 = time.perf_counter()
            lay = oracle.layout(w.topk_idx, E=spec.E, R=spec.R, C_rank=T)
            list(pool.map(lambda ab: part(ab, lay), parts))
            list(pool.map(lambda ab: part2(ab, lay), parts))
            t_total += time.perf_counter() - t0
            reps += 1
    # the threaded result must be the sequential one
    ref = oracle.combine(recv, w.topk_w, lay, H, acc="f64")
    assert np.array_equal(out, ref)
    ab = wl.algorithmic_bytes(spec, rows)
    nbytes = ab["layout"] + ab["dispatch"] + ab["combine"]
    return {"value": round(nbytes * reps / t_total / 1e9, 4), "unit": "GB/s", "cores": len(parts), "kind": "oracle",
            "sample": f"{reps} full steps, dispatch and combine cut into {len(parts)} token ranges run by as many "
                      f"threads, layout sequential; {t_total / reps * 1e3:.0f} ms each",
            "ms_per_step": round(t_total / reps * 1e3, 2)}


class StepBench:
    """One workload prepared for timing: `nsets` rotated input/window sets resident in HBM, the
    expert outputs that combine reads computed once, the call descriptors built once.  A step is
    then three or four foreign-function calls:
        inputs of at most 1024 routed entries:  ep_layout_dispatch, ep_combine, ep_handle_destroy
        larger ones:  ep_layout[_prefetch], ep_dispatch, ep_combine, ep_handle_destroy"""

    def __init__(self, ep, hx, wl, torch, np, workload: str, mode: str = "ht", slots: int = 0, order: int = 1,
                 nsets: int = 3):
        self.ep, self.torch, self.np, self.wl = ep, torch, np, wl
        self.w = wl.make_workload(workload)
        spec = self.spec = self.w.spec
        T, K, H, E = spec.T, spec.K, spec.H, spec.E
        self.ll = mode == "ll"
        self.C = (slots or max(1, 2 * T * K // E)) if self.ll else 0
        self.order = order
        self.nsets = nsets
        self.fused = T * K <= 1024
        cfg = ep.make_config(spec.R, E, H, K, T, mode=ep.EP_MODE_LL if self.ll else ep.EP_MODE_HT,
                             slots_per_subregion=self.C, max_handles=nsets + 2,  # no allocation later
                             dispatch_order=order)
        self.cfg = cfg
        self.group = ep.ep_group_create(cfg)
        self.sets = []
        scale = wl.expert_scale_table(spec)
        for s in range(nsets):
            ws = self.w if s == 0 else wl.make_workload(workload, seed_offset=10 * s)
            x = hx.bits_to_dev(ws.x_bits)
            topk = torch.from_numpy(ws.topk_idx).to(hx.DEV)
            gate = torch.from_numpy(ws.topk_w).to(hx.DEV)
            recv = torch.zeros((E, self.C, H) if self.ll else (T * K, H), dtype=torch.bfloat16, device=hx.DEV)
            out = torch.zeros((T, H), dtype=torch.bfloat16, device=hx.DEV)
            # expert outputs for combine: stand-in experts applied once to the dispatched rows
            h = ep.ep_layout(self.group, topk)
            ep.ep_dispatch(h, x, recv)
            info = ep.ep_handle_query(h)
            counts = ep.read_device_i32(info.expert_count, E).numpy()
            row_e = torch.from_numpy(np.repeat(np.arange(E), self.C if self.ll else counts)).to(hx.DEV)
            y = torch.empty_like(recv)
            flat_in, flat_out = recv.view(-1, H), y.view(-1, H)
            for r0 in range(0, flat_in.shape[0], 8192):
                flat_out[r0:r0 + 8192] = hx.expert_standin(flat_in[r0:r0 + 8192], row_e[r0:r0 + 8192], scale)
            if s == 0:
                self.rows, self.dropped = int(info.rows_kept), int(info.rows_dropped)
            ep.ep_handle_destroy(h)
            self.sets.append((x, topk, gate, recv, y, out))
        torch.cuda.synchronize()
        self.stream_ptr = torch.cuda.current_stream().cuda_stream
        self._destroy = ep.load().ep_handle_destroy
        self.prefetch = order == 1 and not self.fused
        if self.fused:
            self.prepared = [(ep.PreparedLayoutDispatch(self.group, topk, x, recv, topk_weights=gate), None,
                              ep.prepare_combine(y, out, topk_weights=gate)) for (x, topk, gate, recv, y, out) in self.sets]
        else:
            self.prepared = [(ep.PreparedLayout(self.group, topk, tokens=x if self.prefetch else None),
                              ep.prepare_dispatch(x, recv, topk_weights=gate), ep.prepare_combine(y, out, topk_weights=gate))
                             for (x, topk, gate, recv, y, out) in self.sets]
        ab = wl.algorithmic_bytes(spec, self.rows)
        self.bytes = ab
        self.step_bytes = ab["layout"] + ab["dispatch"] + ab["combine"]
        self.calls = ("ep_layout_dispatch (layout and dispatch in one launch) + ep_combine" if self.fused else
                      ("ep_layout_prefetch" if self.prefetch else "ep_layout") + " + ep_dispatch + ep_combine")

    def step(self, i: int, ev=None) -> None:
        a, b, c = self.prepared[i % self.nsets]
        sp = self.stream_ptr
        if ev:
            ev[0].record()
        h = a(sp)
        if ev:
            ev[1].record()
        if b is not None:
            b(h, sp)
        if ev:
            ev[2].record()
        c(h, sp)
        if ev:
            ev[3].record()
        self._destroy(h)

    def timed(self, steps: int, first: int = 0) -> float:
        """Seconds for exactly `steps` steps, bracketed by synchronisation on both sides."""
        torch = self.torch
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            self.step(first + i)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    def per_op(self, steps: int):
        """Microseconds per call from HIP events around every call of `steps` steps (they include
        the gap between two dependent launches, and recording them slows the step itself, so
        this is a pass of its own): arrays layout, dispatch, combine.  In the one-launch case
        `layout` is the layout+dispatch call and `dispatch` is empty."""
        torch, np = self.torch, self.np
        events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
        for i in range(steps):
            self.step(i, events[i])
        torch.cuda.synchronize()
        f = lambda a, b: np.array([e[a].elapsed_time(e[b]) for e in events]) * 1e3
        return f(0, 1), f(1, 2), f(2, 3)

    def summary(self, steps: int, warmup: int, repeats: int = 10) -> dict:
        """Median / min / max over `repeats` timed regions of `steps` steps, per-op medians, rates."""
        np = self.np
        for i in range(warmup):
            self.step(i)
        per_step = np.array([self.timed(steps, first=r * steps) / steps * 1e6 for r in range(repeats)])
        lay, dis, com = self.per_op(max(12, min(steps, 40)))
        spec = self.spec
        med = float(np.median(per_step))
        res = {"workload": f"{spec.name}: R={spec.R} T={spec.T} H={spec.H} E={spec.E} K={spec.K} bf16, "
                           f"{'padded layout [E, C=%d, H]' % self.C if self.ll else 'concatenated layout'}"
                           f"{', ' + ORDER_NAMES[self.order] if not self.fused else ''}",
               "calls": self.calls, "rows": self.rows, "rows_dropped": self.dropped,
               "step_us": round(med, 2), "step_us_min": round(float(per_step.min()), 2),
               "step_us_max": round(float(per_step.max()), 2), "repeats": repeats, "steps_per_repeat": steps,
               "gbps": round(self.step_bytes / (med * 1e-6) / 1e9, 1),
               "pct_of_hbm_peak": round(100.0 * self.step_bytes / (med * 1e-6) / 1e9 / HBM_PEAK_GBS, 2),
               "algorithmic_bytes": self.bytes}
        if self.fused:
            res["layout_dispatch_us"] = round(float(np.median(lay)), 2)
        else:
            res["layout_us"] = round(float(np.median(lay)), 2)
            res["dispatch_us"] = round(float(np.median(dis)), 2)
            res["layout_plus_dispatch_us"] = round(float(np.median(lay + dis)), 2)
        res["combine_us"] = round(float(np.median(com)), 2)
        return res

    def close(self) -> None:
        self.ep.ep_group_destroy(self.group)
        self.sets, self.prepared = [], []
        self.torch.cuda.empty_cache()


def _timed_us(torch, np, fn, iters: int = 20) -> float:
    for _ in range(3):
        fn()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]
    for i in range(iters):
        ev[i].record()
        fn()
    ev[iters].record()
    torch.cuda.synchronize()
    return float(np.mean([ev[i].elapsed_time(ev[i + 1]) for i in range(iters)])) * 1e3


def once_per_rank(ep, torch, np, spec, sets, rows, stream_ptr):
    """The dispatch variant that sends a token once per destination rank and fans out on arrival
    (send + receiver ranking + fan-out), timed over the rotated input sets; HIP events."""
    T, K, H, E = spec.T, spec.K, spec.H, spec.E
    cfg = ep.make_config(spec.R, E, H, K, T, mode=ep.EP_MODE_HT, dispatch_path=ep.EP_PATH_RANK_DEDUP,
                         max_handles=len(sets))
    g2 = ep.ep_group_create(cfg)
    hs = [ep.ep_layout(g2, s[1]) for s in sets]
    calls = [ep.prepare_dispatch(s[0], s[3], topk_weights=s[2], topk_idx=s[1]) for s in sets]
    info = ep.ep_handle_query(hs[0])
    ginfo = ep.ep_group_query(g2)
    it = [0]

    def one():
        i = it[0] % len(sets)
        it[0] += 1
        calls[i](hs[i], stream_ptr)

    us = _timed_us(torch, np, one, iters=21)
    msgs, P = int(info.rank_messages), int(ginfo.msg_bytes)
    nbytes = T * 2 * H + msgs * P + msgs * P + rows * 2 * H + 8 * rows
    res = {"dispatch_us": round(us, 2), "messages": msgs, "algorithmic_bytes": nbytes,
           "gbps": round(nbytes / (us * 1e-6) / 1e9, 1),
           "pct_of_hbm_peak": round(100.0 * nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 2),
           "staging_bytes": int(ginfo.staging_slots) * int(ginfo.msg_stride),
           "what": "ep_dispatch of a group with EP_PATH_RANK_DEDUP: token read + one message per destination "
                   "rank written, then messages read + expert rows written (about 2.6 times the bytes of the "
                   "direct path on one GPU; what it buys is staging footprint)"}
    for h in hs:
        ep.ep_handle_destroy(h)
    ep.ep_group_destroy(g2)
    return res


def hbm_copy_reference(ep, hx, torch):
    """Plain streaming kernels over 512 MiB: a copy (the reference point for mixed traffic, and the
    kernel of known size that scales the rocprofv3 byte counters), a fill and a read (what the memory
    sustains in one direction: dispatch mostly writes, combine mostly reads)."""
    cal_src = torch.empty(512 << 20, dtype=torch.uint8, device=hx.DEV).fill_(1)
    cal_dst = torch.empty_like(cal_src)
    sink = torch.zeros(4, dtype=torch.int32, device=hx.DEV)

    def best_us(fn):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(7)]
        fn()
        for j in range(6):
            ev[j].record()
            fn()
        ev[6].record()
        torch.cuda.synchronize()
        return min(ev[j].elapsed_time(ev[j + 1]) for j in range(6)) * 1e3

    n = cal_src.numel()
    cal_us = best_us(lambda: ep.ep_calibration_copy(cal_dst, cal_src))
    fill_us = best_us(lambda: ep.ep_calibration_fill(cal_dst))
    read_us = best_us(lambda: ep.ep_calibration_read(cal_src, sink))
    return {"gbps": round(2 * n / (cal_us * 1e-6) / 1e9, 1),
            "write_only_gbps": round(n / (fill_us * 1e-6) / 1e9, 1),
            "read_only_gbps": round(n / (read_us * 1e-6) / 1e9, 1),
            "what": "plain 16-byte-per-lane kernels over 512 MiB, best of 6 launches each: copy (read + write "
                    "bytes), fill (bytes written), read (bytes read)"}


def extras(ep, hx, wl, torch, np, group, spec, first_set, rows, stream_ptr, iters: int = 20):
    """Timings of the dispatch variants outside the headline step (HIP events, mean of iters)."""
    x, topk, gate, recv, y, out = first_set
    T, K, H, E = spec.T, spec.K, spec.H, spec.E
    res = {}
    timed = lambda fn: _timed_us(torch, np, fn, iters)

    if H % 128 == 0:
        q = torch.empty((T * K, H), dtype=torch.uint8, device=hx.DEV).view(torch.float8_e4m3fn)
        sc = torch.empty((T * K, H // 128), dtype=torch.float32, device=hx.DEV)
        nbytes = T * 2 * H + rows * (H + 4 * (H // 128)) + 8 * rows
        for order, key in ((ep.EP_ORDER_TOKEN, "fp8_dispatch"),):
            g5 = ep.ep_group_create(ep.make_config(spec.R, E, H, K, T, mode=ep.EP_MODE_HT, dispatch_order=order))
            h = ep.ep_layout(g5, topk)
            call = ep.prepare_dispatch(x, q, topk_weights=gate, recv_scales=sc)
            us = timed(lambda: call(h, stream_ptr))
            res[key] = {"us": round(us, 2), "algorithmic_bytes": nbytes, "gbps": round(nbytes / (us * 1e-6) / 1e9, 1)}
            ep.ep_handle_destroy(h)
            ep.ep_group_destroy(g5)
        # the same with the quantisation moved into the layout launch (group option quantize_ahead): layout and
        # dispatch are rated together, once for the token walk (plain layout + quantising dispatch) and once for
        # the staged rows copied in destination order
        pair = {}
        for key, order, ahead in (("token_walk", ep.EP_ORDER_TOKEN, 0), ("quantize_ahead", ep.EP_ORDER_DESTINATION, 1)):
            g6 = ep.ep_group_create(ep.make_config(spec.R, E, H, K, T, mode=ep.EP_MODE_HT, dispatch_order=order,
                                                   quantize_ahead=ahead))
            lay6 = ep.PreparedLayout(g6, topk, tokens=x if ahead else None)
            call = ep.prepare_dispatch(x, q, topk_weights=gate, recv_scales=sc)

            def both():
                h6 = lay6(stream_ptr)
                call(h6, stream_ptr)
                ep.ep_handle_destroy(h6)

            def lay_only():
                ep.ep_handle_destroy(lay6(stream_ptr))

            us, us_l = timed(both), timed(lay_only)
            pair[key] = {"layout_plus_dispatch_us": round(us, 2), "layout_us": round(us_l, 2),
                         "gbps": round((nbytes + 4 * T * K) / (us * 1e-6) / 1e9, 1)}
            ep.ep_group_destroy(g6)
        res["fp8_layout_plus_dispatch"] = pair
        del q, sc
    # destination-ordered dispatch: with its read pass, and without it for cache-resident tokens
    for order, key in ((ep.EP_ORDER_DESTINATION, "dispatch_destination_order"),
                       (ep.EP_ORDER_DESTINATION_RESIDENT, "dispatch_destination_order_resident")):
        cfg = ep.make_config(spec.R, E, H, K, T, mode=ep.EP_MODE_HT, dispatch_order=order)
        g4 = ep.ep_group_create(cfg)
        h4 = ep.ep_layout(g4, topk)
        call = ep.prepare_dispatch(x, recv, topk_weights=gate)
        us = timed(lambda: call(h4, stream_ptr))
        nbytes = T * 2 * H + rows * 2 * H + 8 * rows
        res[key] = {"us": round(us, 2), "algorithmic_bytes": nbytes, "gbps": round(nbytes / (us * 1e-6) / 1e9, 1),
                    "note": "same tokens and same window every iteration: the tokens are resident in the memory-side "
                            "cache, and part of the 470 MB of writes may be absorbed by it too"}
        ep.ep_handle_destroy(h4)
        ep.ep_group_destroy(g4)

    # training step: forward (layout, dispatch, combine) and backward with the handle of the forward pass
    # (combine backward = output gradient scaled into the rows + gate-weight gradients from the rows;
    # dispatch backward = unweighted combine of the row gradients)
    g_out = torch.randn((T, H), device=hx.DEV).bfloat16()
    grad_y = torch.empty_like(recv)
    grad_w = torch.empty((T, K), dtype=torch.float32, device=hx.DEV)
    grad_x = torch.empty((T, H), dtype=torch.bfloat16, device=hx.DEV)
    lay_call = ep.PreparedLayout(group, topk, tokens=x)
    fwd_d = ep.prepare_dispatch(x, recv, topk_weights=gate)
    fwd_c = ep.prepare_combine(y, out, topk_weights=gate)
    bwd_c = ep.prepare_combine_backward(g_out, grad_y, topk_weights=gate, y=y, grad_w=grad_w)
    bwd_d = ep.prepare_combine(grad_y, grad_x)

    def train_step():
        h = lay_call(stream_ptr)
        fwd_d(h, stream_ptr)
        fwd_c(h, stream_ptr)
        bwd_c(h, stream_ptr)
        bwd_d(h, stream_ptr)
        ep.ep_handle_destroy(h)

    def backward_only(h):
        bwd_c(h, stream_ptr)
        bwd_d(h, stream_ptr)

    hb = lay_call(stream_ptr)
    us_b = timed(lambda: backward_only(hb))
    us_cb = timed(lambda: bwd_c(hb, stream_ptr))
    ep.ep_handle_destroy(hb)
    us_t = timed(train_step)
    b_cb = T * 2 * H + 2 * rows * 2 * H + 8 * rows + 4 * T * K
    b_db = rows * 2 * H + T * 2 * H + 4 * rows
    b_fwd = (T * 2 * H + rows * 2 * H) * 2 + 20 * rows
    res["training_step"] = {
        "forward_plus_backward_us": round(us_t, 2), "backward_us": round(us_b, 2),
        "combine_backward_us": round(us_cb, 2),
        "combine_backward_gbps": round(b_cb / (us_cb * 1e-6) / 1e9, 1),
        "algorithmic_bytes": {"forward": b_fwd, "combine_backward": b_cb, "dispatch_backward": b_db},
        "gbps": round((b_fwd + b_cb + b_db) / (us_t * 1e-6) / 1e9, 1),
        "what": "layout + dispatch + combine, then ep_combine_backward (gradient rows and gate-weight gradients) "
                "and the unweighted combine of the gradient rows, all on one handle"}
    del grad_y, grad_w, grad_x, g_out

    # staged execution (send phase + ep_complete) and the two-level combine order
    cfg = ep.make_config(spec.R, E, H, K, T, mode=ep.EP_MODE_HT, staged_buffers=2, ranks_per_node=8)
    g3 = ep.ep_group_create(cfg)
    h3 = ep.ep_layout(g3, topk)
    dis = ep.PreparedCall("ep_dispatch", [(x, ep.EP_TAG_TOKENS), (gate, ep.EP_TAG_TOPK_WEIGHTS)],
                          [(recv, ep.EP_TAG_TOKENS)], send_only=1)
    complete = ep.load().ep_complete

    def staged_dispatch():
        dis(h3, stream_ptr)
        complete(h3, None, stream_ptr)

    res["staged_dispatch_plus_complete"] = {"us": round(timed(staged_dispatch), 2)}
    com = ep.PreparedCall("ep_combine", [(y, ep.EP_TAG_TOKENS), (gate, ep.EP_TAG_TOPK_WEIGHTS)], [(out, ep.EP_TAG_TOKENS)], send_only=1)

    def staged_combine():
        com(h3, stream_ptr)
        complete(h3, None, stream_ptr)

    us = timed(staged_combine)
    nbytes = 2 * rows * 2 * H + rows * 2 * H + T * 2 * H + 16 * rows
    res["staged_combine_plus_complete"] = {"us": round(us, 2), "algorithmic_bytes": nbytes,
                                           "gbps": round(nbytes / (us * 1e-6) / 1e9, 1)}
    hier = ep.prepare_combine(y, out, topk_weights=gate)
    us = timed(lambda: hier(h3, stream_ptr))
    nbytes = rows * 2 * H + T * 2 * H + 12 * rows
    res["two_level_combine"] = {"us": round(us, 2), "ranks_per_node": 8, "algorithmic_bytes": nbytes,
                                "gbps": round(nbytes / (us * 1e-6) / 1e9, 1)}
    ep.ep_handle_destroy(h3)
    ep.ep_group_destroy(g3)
    return res


# every other shape of the workload list, in the configuration the headline uses
ALL_CONFIGS = [
    ("tiny", "tiny", "ht", 0),
    ("ll_decode", "ll_decode", "ll", 128),
    ("skew", "skew", "ht", 0),
    ("skew_padded_C512", "skew", "ll", 512),
    ("skew_rank0", "skew_rank0", "ht", 0),
    ("stress", "stress", "ht", 0),
    ("stress_hot", "stress_hot", "ht", 0),
]


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="ht_prefill")
    ap.add_argument("--sets", type=int, default=3, help="input/window sets rotated between steps")
    ap.add_argument("--dispatch-order", type=int, default=1, choices=(0, 1, 2),
                    help="EP_ORDER_TOKEN (0); EP_ORDER_DESTINATION with the tokens announced to the layout "
                         "call, ep_layout_prefetch (1, default); EP_ORDER_DESTINATION_RESIDENT (2)")
    ap.add_argument("--mode", choices=("ht", "ll"), default="ht",
                    help="window layout: ht = concatenated [rows, H] (default), ll = padded [E, C, H]")
    ap.add_argument("--slots", type=int, default=0,
                    help="C of the padded layout (default: twice the mean rows per expert, 2*T*K/E)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--step-only", action="store_true",
                    help="leave out the add-on measurements (all_configs, once_per_rank, per-op events, CPU "
                         "baselines): only the kernels of the step run, which is what the rocprofv3 summaries are "
                         "taken with")
    ap.add_argument("--calibrate", action="store_true",
                    help="with --step-only: also run the 512 MiB calibration copy (the kernel of known size the "
                         "rocprofv3 byte counters are scaled by)")
    ap.add_argument("--headline-only", action="store_true",
                    help="the headline step with its per-op times and roofline, without all_configs, once_per_rank "
                         "and the CPU baselines")
    ap.add_argument("--repeats", type=int, default=10,
                    help="timed regions of --steps steps per workload; medians over them are reported next to "
                         "the one region the headline value is taken from")
    ap.add_argument("--graph", action="store_true",
                    help="also replay the step from captured HIP graphs (reported in a 'graph' object)")
    ap.add_argument("--extras", action="store_true",
                    help="also time the FP8 quantising dispatch, the staged calls and the two-level combine "
                         "(reported in an 'extras' object; the headline numbers are unaffected)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one rank's share on ONE GPU; this build has no multi-GPU path "
              "(run with --gpus 1).", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import ep_harness as hx
    from paper_2603_13606_amd import binding as ep
    from paper_2603_13606_amd import workloads as wl

    hx.ensure_built()  # rebuilds a library that does not match the sources; there is no fallback path
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    nsets = max(1, args.sets)
    sb = StepBench(ep, hx, wl, torch, np, args.workload, args.mode, args.slots, args.dispatch_order, nsets)
    spec, ab, rows = sb.spec, sb.bytes, sb.rows
    T, K, H, E = spec.T, spec.K, spec.H, spec.E

    # the plain copy / fill / read reference first: it is reported next to the result, and the card has
    # left its idle state by the time the warm-up steps start
    copy_reference = hbm_copy_reference(ep, hx, torch) if (not args.step_only or args.calibrate) else None
    for i in range(args.warmup):
        sb.step(i)
    # THE timed region: exactly --steps steps between two synchronisations
    elapsed = sb.timed(args.steps, first=args.warmup)
    value = sb.step_bytes * args.steps / elapsed / 1e9

    line = {
        "metric": "dispatch+combine µs and effective HBM GB/s (% of peak), 1 MI355X",
        "value_is": "effective HBM GB/s of one step = layout + dispatch + combine algorithmic bytes / wall time; "
                    "the µs per op are in 'us', the % of the 8 TB/s peak in 'pct_of_hbm_peak'",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(elapsed / args.steps * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{spec.name}: R={spec.R} T={T} H={H} E={E} K={K} bf16, "
                               f"{'padded layout [E, C=%d, H]' % sb.C if sb.ll else 'concatenated layout'}, "
                               f"direct dispatch {ORDER_NAMES[args.dispatch_order]}, "
                               f"gate logits N(0,1) prior={spec.prior}",
                   "rows": rows, "input_sets_rotated": nsets, "calls": sb.calls},
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "algorithmic_bytes": ab,
        "build_id": ep.ep_build_id(),
    }
    if not args.step_only:
        # more regions of the same length: how much one region moves
        per_step = np.array([sb.timed(args.steps, first=r * args.steps) / args.steps * 1e6 for r in range(args.repeats)])
        line["step_us_over_repeats"] = {"median": round(float(np.median(per_step)), 2), "min": round(float(per_step.min()), 2),
                                        "max": round(float(per_step.max()), 2), "regions": args.repeats}
        # per call, from HIP events around every call (a pass of its own: recording slows the step)
        lay_us, dis_us, com_us = sb.per_op(max(30, min(args.steps, 100)))

        def stats(a):
            return {"mean": round(float(a.mean()), 2), "p10": round(float(np.percentile(a, 10)), 2),
                    "p50": round(float(np.percentile(a, 50)), 2), "p90": round(float(np.percentile(a, 90)), 2)}

        lpd = lay_us + dis_us
        if sb.fused:  # one launch lays out and dispatches: there is no dispatch call of its own
            lpd = lay_us
            line["us"] = {"layout_plus_dispatch": stats(lay_us), "combine": stats(com_us),
                          "samples": int(lay_us.size)}
            dis_us = lay_us
        else:
            line["us"] = {"layout": stats(lay_us), "dispatch": stats(dis_us), "combine": stats(com_us),
                          "layout_plus_dispatch": stats(lpd),
                          "dispatch_plus_combine_mean": round(float(dis_us.mean() + com_us.mean()), 2),
                          "samples": int(lay_us.size)}
        line["us"].update({
                      "note": "HIP events on the launch stream around each call; they include the gap between two "
                              "dependent launches, so they read a few us above the kernel durations of rocprofv3"})
        row = spec.row_bytes
        gb = lambda nbytes, us: round(nbytes / (us * 1e-6) / 1e9, 1)
        line["gbps"] = {"layout_plus_dispatch": gb(ab["layout"] + ab["dispatch"], lpd.mean()),
                        "combine": gb(ab["combine"], com_us.mean()),
                        "step": round(value, 1)}
        if sb.prefetch:
            line["gbps"]["note"] = ("the tokens are read in the layout launch (ep_layout_prefetch) and found in the "
                                    "memory-side cache by the dispatch: the dispatch call alone is not credited with "
                                    "that read, layout + dispatch are rated together")
            dispatch_bytes = ab["dispatch"] - T * row  # what the copy launch itself moves through HBM
        else:
            line["gbps"]["dispatch"] = gb(ab["dispatch"], dis_us.mean())
            dispatch_bytes = ab["dispatch"]
        # roofline of the dominant kernel (the longer of the two row kernels)
        dom = "dispatch" if dis_us.mean() >= com_us.mean() else "combine"
        dom_us = dis_us.mean() if dom == "dispatch" else com_us.mean()
        dom_bytes = dispatch_bytes if dom == "dispatch" else ab["combine"]
        run_order = args.dispatch_order != 0 and T * K >= 8192
        kernel_name = {"dispatch": "layout_dispatch_kernel" if sb.fused else
                                   "dispatch_runs_kernel" if run_order else "dispatch_direct_kernel",
                       "combine": "combine_kernel"}[dom]
        traffic_key = spec.name + ("_padded" if sb.ll else "") + ["_token_order", "", "_destination_order_resident"][args.dispatch_order]
        if dom == "combine":
            # rows of 14 336 bytes in whole rounds of resident wavefronts take the library's whole-row combine kernel
            cus = torch.cuda.get_device_properties(0).multi_processor_count
            if ep.ep_combine_plan(sb.cfg, T, cus).whole_row:
                kernel_name = "combine_row_kernel"
        prof = _profiled(traffic_key, kernel_name) or {}
        achieved = dom_bytes / (dom_us * 1e-6) / 1e9
        line["roofline"] = {"bound": "hbm", "kernel": kernel_name, "achieved": round(achieved, 1),
                            "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                            "traffic": prof.get("traffic"),
                            "algorithmic_bytes_per_launch": int(dom_bytes),
                            "kernel_us_events": round(float(dom_us), 2),
                            "kernel_us_profiled": prof.get("kernel_us"),
                            "profile": {k: prof.get(k) for k in ("commit", "date", "command")} if prof else None,
                            "timing": f"HIP events on the launch stream around the kernel, mean of {int(lay_us.size)} "
                                      "consecutive steps (launch gap included); traffic and kernel_us_profiled are "
                                      "rocprofv3 figures of the committed run named in 'profile'"}
    if copy_reference is not None:
        line["hbm_copy_reference"] = copy_reference
        if "roofline" in line and rows > 0:
            # the same kernel against what THIS card sustains in each direction (the plain read and fill kernels
            # of this process): time the kernel's reads would take alone plus time its writes would take alone
            rd, wr = (T * row, rows * row) if dom == "dispatch" else (rows * row, T * row)
            if dom == "dispatch" and sb.prefetch:
                rd = 0  # the tokens come from the memory-side cache (read there by the layout launch)
            floor_us = (rd / copy_reference["read_only_gbps"] + wr / copy_reference["write_only_gbps"]) * 1e-3
            line["roofline"]["against_measured_rates"] = {
                "floor_us": round(floor_us, 2), "frac": round(floor_us / float(dom_us), 4),
                "what": "bytes read / read-only rate + bytes written / write-only rate of hbm_copy_reference, over "
                        "kernel_us_events: how close the kernel is to what plain kernels reach on this card, as "
                        "opposed to the published peak"}
    if args.graph:
        # one graph per input set: layout + dispatch + combine captured on a side stream
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        sp = side.cuda_stream
        destroy = ep.load().ep_handle_destroy
        graphs, live = [], []
        for a, b, c in sb.prepared:
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr, stream=side):
                hh = a(sp)
                if b is not None:
                    b(hh, sp)
                c(hh, sp)
            graphs.append(gr)
            live.append(hh)
        for i in range(args.warmup):
            graphs[i % nsets].replay()
        torch.cuda.synchronize()
        tg = time.perf_counter()
        for i in range(args.steps):
            graphs[i % nsets].replay()
        torch.cuda.synchronize()
        el = time.perf_counter() - tg
        line["graph"] = {"ms_per_step": round(el / args.steps * 1e3, 4),
                         "value": round(sb.step_bytes * args.steps / el / 1e9, 2), "unit": "GB/s",
                         "what": "the same step replayed from a captured HIP graph (one graph per input set)"}
        del graphs
        for hh in live:
            destroy(hh)
    addons = not args.step_only and not args.headline_only
    if T * K >= 1024 and not sb.ll and addons:
        line["once_per_rank"] = once_per_rank(ep, torch, np, spec, sb.sets, rows, sb.stream_ptr)
    if args.extras and not sb.ll:
        line["extras"] = extras(ep, hx, wl, torch, np, sb.group, spec, sb.sets[0], rows, sb.stream_ptr)
    w = sb.w
    sb.close()
    if spec.name == "ht_prefill" and addons:
        # the other workload shapes, each in the configuration of the headline (their own groups and inputs)
        allc = {}
        for key, name, mode, slots in ALL_CONFIGS:
            b2 = StepBench(ep, hx, wl, torch, np, name, mode, slots, args.dispatch_order, nsets)
            allc[key] = b2.summary(args.steps, args.warmup, args.repeats)
            b2.close()
            del b2
        line["all_configs"] = allc
        line["decode_shape"] = allc["ll_decode"]
    if not args.no_cpu_baseline and addons:
        line["cpu_baseline"] = cpu_baseline(w)
        # box share of one GPU: 16 cores, whatever os.cpu_count() shows
        line["cpu_baseline_all_cores"] = cpu_baseline_all_cores(w, threads=min(16, os.cpu_count() or 1))
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
