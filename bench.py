#!/usr/bin/env python3
"""Benchmark of the dispatch/combine hot path on one MI355X.

One step = ep_layout + ep_dispatch + ep_combine (+ handle destroy) over one batch
of synthetic routing.  Inputs (tokens, top-k ids, gate weights, expert outputs)
are resident in HBM before the timed region.  Prints ONE JSON line.

By default the group is configured with EP_ORDER_DESTINATION and the layout call is
ep_layout_prefetch (the tokens are announced to it); --dispatch-order 0 times the
token-ordered dispatch with plain ep_layout.

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


def _traffic(workload: str, kernel: str):
    """HBM bytes per launch measured with rocprofv3 counters (FETCH_SIZE + WRITE_SIZE scaled
    by the calibration copy), read from the committed summary; None if there is none."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    try:
        with open(path) as f:
            for line in f:
                parts = line.split()
                if len(parts) == 3 and parts[0] == workload and parts[1] == kernel:
                    return int(parts[2])
    except (OSError, ValueError):
        pass
    return None


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


def once_per_rank(ep, torch, np, spec, sets, stream_ptr):
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
    rows = sets[0][6]
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


def decode_shape(ep, hx, wl, torch, np, stream_ptr, steps: int = 200):
    """The low-latency decode shape (R=32, T=128, H=7168, E=256, K=8) in the padded [E, C, H] window
    layout: microseconds per call (HIP events on every 4th step) and per whole step (wall clock)."""
    w = wl.make_workload("ll_decode")
    spec = w.spec
    T, K, H, E = spec.T, spec.K, spec.H, spec.E
    C = T
    g = ep.ep_group_create(ep.make_config(spec.R, E, H, K, T, mode=ep.EP_MODE_LL, slots_per_subregion=C, max_handles=4))
    x = hx.bits_to_dev(w.x_bits)
    topk = torch.from_numpy(w.topk_idx).to(hx.DEV)
    gate = torch.from_numpy(w.topk_w).to(hx.DEV)
    recv = torch.zeros((E, C, H), dtype=torch.bfloat16, device=hx.DEV)
    out = torch.zeros((T, H), dtype=torch.bfloat16, device=hx.DEV)
    lay, dis, com = ep.PreparedLayout(g, topk), ep.prepare_dispatch(x, recv, topk_weights=gate), \
        ep.prepare_combine(recv, out, topk_weights=gate)
    destroy = ep.load().ep_handle_destroy

    def step(ev=None):
        if ev:
            ev[0].record()
        h = lay(stream_ptr)
        if ev:
            ev[1].record()
        dis(h, stream_ptr)
        if ev:
            ev[2].record()
        com(h, stream_ptr)
        if ev:
            ev[3].record()
        destroy(h)

    for _ in range(20):
        step()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps // 4)]
    t0 = time.perf_counter()
    for i in range(steps):
        step(events[i // 4] if i % 4 == 0 else None)
    torch.cuda.synchronize()
    el = time.perf_counter() - t0
    us = lambda a, b: round(float(np.mean([e[a].elapsed_time(e[b]) for e in events])) * 1e3, 2)
    ab = wl.algorithmic_bytes(spec, T * K)
    res = {"workload": f"ll_decode: R={spec.R} T={T} H={H} E={E} K={K} bf16, padded layout [E, C={C}, H], token order",
           "step_us": round(el / steps * 1e6, 2), "layout_us": us(0, 1), "dispatch_us": us(1, 2), "combine_us": us(2, 3),
           "algorithmic_bytes": ab, "note": "launch and latency bound: 16.5 MB per call is 2 us at the HBM peak"}
    ep.ep_group_destroy(g)
    return res


def extras(ep, hx, wl, torch, np, group, spec, first_set, stream_ptr, iters: int = 20):
    """Timings of the dispatch variants outside the headline step (HIP events, mean of iters)."""
    x, topk, gate, recv, y, out, rows = first_set
    T, K, H, E = spec.T, spec.K, spec.H, spec.E
    res = {}

    def timed(fn):
        for _ in range(3):
            fn()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]
        for i in range(iters):
            ev[i].record()
            fn()
        ev[iters].record()
        torch.cuda.synchronize()
        return float(np.mean([ev[i].elapsed_time(ev[i + 1]) for i in range(iters)])) * 1e3

    h = ep.ep_layout(group, topk)
    if H % 128 == 0:
        q = torch.empty((T * K, H), dtype=torch.uint8, device=hx.DEV).view(torch.float8_e4m3fn)
        sc = torch.empty((T * K, H // 128), dtype=torch.float32, device=hx.DEV)
        call = ep.prepare_dispatch(x, q, topk_weights=gate, recv_scales=sc)
        us = timed(lambda: call(h, stream_ptr))
        nbytes = T * 2 * H + rows * (H + 4 * (H // 128)) + 8 * rows
        res["fp8_dispatch"] = {"us": round(us, 2), "algorithmic_bytes": nbytes,
                               "gbps": round(nbytes / (us * 1e-6) / 1e9, 1)}
        del q, sc
    ep.ep_handle_destroy(h)
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
                    help="leave out the add-on measurements (decode_shape, once_per_rank, CPU baselines): only the "
                         "kernels of the headline step run, which is what the rocprofv3 summaries are taken with")
    ap.add_argument("--event-every", type=int, default=4,
                    help="record the per-op HIP events on every n-th timed step only (four event "
                         "records cost about 12 us of a step, so they are sampled)")
    ap.add_argument("--graph", action="store_true",
                    help="also replay the step from captured HIP graphs (reported in a 'graph' object)")
    ap.add_argument("--extras", action="store_true",
                    help="also time the FP8 quantising dispatch and the once-per-rank dispatch (reported "
                         "in an 'extras' object; the headline numbers are unaffected)")
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

    hx.ensure_built()  # builds only if no library is in the tree; there is no fallback path
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    w = wl.make_workload(args.workload)
    spec = w.spec
    T, K, H, E = spec.T, spec.K, spec.H, spec.E
    nsets = max(1, args.sets)
    ll = args.mode == "ll"
    C = (args.slots or max(1, 2 * T * K // E)) if ll else 0
    cfg = ep.make_config(spec.R, E, H, K, T, mode=ep.EP_MODE_LL if ll else ep.EP_MODE_HT, slots_per_subregion=C,
                         max_handles=nsets + 2,  # no allocation later
                         dispatch_order=args.dispatch_order)
    group = ep.ep_group_create(cfg)

    nsets = max(1, args.sets)
    sets = []
    scale = wl.expert_scale_table(spec)
    for s in range(nsets):
        ws = w if s == 0 else wl.make_workload(args.workload, seed_offset=10 * s)
        x = hx.bits_to_dev(ws.x_bits)
        topk = torch.from_numpy(ws.topk_idx).to(hx.DEV)
        gate = torch.from_numpy(ws.topk_w).to(hx.DEV)
        recv = torch.zeros((E, C, H) if ll else (T * K, H), dtype=torch.bfloat16, device=hx.DEV)
        out = torch.zeros((T, H), dtype=torch.bfloat16, device=hx.DEV)
        # expert outputs for combine: stand-in experts applied once to the dispatched rows
        h = ep.ep_layout(group, topk)
        ep.ep_dispatch(h, x, recv)
        info = ep.ep_handle_query(h)
        counts = ep.read_device_i32(info.expert_count, E).numpy()
        row_e = torch.from_numpy(np.repeat(np.arange(E), C if ll else counts)).to(hx.DEV)
        y = torch.empty_like(recv)
        flat_in, flat_out = recv.view(-1, H), y.view(-1, H)
        step_rows = 8192
        for r0 in range(0, flat_in.shape[0], step_rows):
            flat_out[r0:r0 + step_rows] = hx.expert_standin(flat_in[r0:r0 + step_rows], row_e[r0:r0 + step_rows], scale)
        rows = int(info.rows_kept)
        ep.ep_handle_destroy(h)
        sets.append((x, topk, gate, recv, y, out, rows))
    torch.cuda.synchronize()

    # descriptors are built once per input set; a step is then four foreign-function calls
    stream_ptr = torch.cuda.current_stream().cuda_stream
    destroy = ep.load().ep_handle_destroy
    prepared = [(ep.PreparedLayout(group, topk, tokens=x if args.dispatch_order == 1 else None), ep.prepare_dispatch(x, recv, topk_weights=gate),
                 ep.prepare_combine(y, out, topk_weights=gate)) for (x, topk, gate, recv, y, out, _) in sets]

    def step(i, ev=None):
        lay, dis, com = prepared[i % nsets]
        if ev:
            ev[0].record()
        h = lay(stream_ptr)
        if ev:
            ev[1].record()
        dis(h, stream_ptr)
        if ev:
            ev[2].record()
        com(h, stream_ptr)
        if ev:
            ev[3].record()
        destroy(h)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # reference point: what a plain streaming copy of 512 MiB reaches on this GPU
    cal_src = torch.empty(512 << 20, dtype=torch.uint8, device=hx.DEV).fill_(1)
    cal_dst = torch.empty_like(cal_src)
    cal_ev = [torch.cuda.Event(enable_timing=True) for _ in range(7)]
    ep.ep_calibration_copy(cal_dst, cal_src)
    for j in range(6):
        cal_ev[j].record()
        ep.ep_calibration_copy(cal_dst, cal_src)
    cal_ev[6].record()
    torch.cuda.synchronize()
    cal_us = min(cal_ev[j].elapsed_time(cal_ev[j + 1]) for j in range(6)) * 1e3
    copy_gbps = 2 * cal_src.numel() / (cal_us * 1e-6) / 1e9
    del cal_src, cal_dst
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, events[i] if i % args.event_every == 0 else None)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    events = [e for i, e in enumerate(events) if i % args.event_every == 0]

    lay_us = np.array([e[0].elapsed_time(e[1]) for e in events]) * 1e3
    dis_us = np.array([e[1].elapsed_time(e[2]) for e in events]) * 1e3
    com_us = np.array([e[2].elapsed_time(e[3]) for e in events]) * 1e3
    rows = sets[0][6]
    ab = wl.algorithmic_bytes(spec, rows)
    step_bytes = ab["layout"] + ab["dispatch"] + ab["combine"]
    value = step_bytes * args.steps / elapsed / 1e9
    dom = "dispatch" if dis_us.mean() >= com_us.mean() else "combine"
    dom_us = dis_us.mean() if dom == "dispatch" else com_us.mean()
    kernel_name = {"dispatch": "dispatch_runs_kernel" if args.dispatch_order else "dispatch_direct_kernel",
                   "combine": "combine_kernel"}[dom]
    traffic_key = spec.name + ["_token_order", "", "_destination_order_resident"][args.dispatch_order]
    achieved = ab[dom] / (dom_us * 1e-6) / 1e9

    def stats(a):
        return {"mean": round(float(a.mean()), 2), "p10": round(float(np.percentile(a, 10)), 2),
                "p50": round(float(np.percentile(a, 50)), 2), "p90": round(float(np.percentile(a, 90)), 2)}

    line = {
        "metric": "dispatch+combine µs and effective HBM GB/s (% of peak), 1 MI355X",
        "value_is": "effective HBM GB/s of one step = layout + dispatch + combine algorithmic bytes / wall time; "
                    "the µs per op are in 'us', the % of the 8 TB/s peak in 'pct_of_hbm_peak'",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(elapsed / args.steps * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{spec.name}: R={spec.R} T={T} H={H} E={E} K={K} bf16, "
                               f"{'padded layout [E, C=%d, H]' % C if ll else 'concatenated layout'}, "
                               f"direct dispatch {['EP_ORDER_TOKEN', 'EP_ORDER_DESTINATION + ep_layout_prefetch', 'EP_ORDER_DESTINATION_RESIDENT'][args.dispatch_order]}, "
                               f"gate logits N(0,1) prior={spec.prior}",
                   "rows": rows, "input_sets_rotated": nsets},
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "us": {"layout": stats(lay_us), "dispatch": stats(dis_us), "combine": stats(com_us),
               "dispatch_plus_combine_mean": round(float(dis_us.mean() + com_us.mean()), 2)},
        "gbps": {"dispatch": round(ab["dispatch"] / (dis_us.mean() * 1e-6) / 1e9, 1),
                 "combine": round(ab["combine"] / (com_us.mean() * 1e-6) / 1e9, 1),
                 "dispatch_plus_combine": round((ab["dispatch"] + ab["combine"]) /
                                                ((dis_us.mean() + com_us.mean()) * 1e-6) / 1e9, 1)},
        "algorithmic_bytes": ab,
        "hbm_copy_reference": {"gbps": round(copy_gbps, 1), "what": "plain 16-byte-per-lane copy of 512 MiB "
                               "(read + write bytes / best of 6 launches)"},
        "roofline": {"bound": "hbm", "kernel": kernel_name, "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": _traffic(traffic_key, kernel_name),
                     "timing": f"HIP events on the launch stream around the kernel, mean over every "
                               f"{args.event_every}-th step of the timed region ({len(events)} samples)"},
    }
    if args.graph:
        # one graph per input set: layout + dispatch + combine captured on a side stream
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        sp = side.cuda_stream
        graphs, live = [], []
        for lay, dis, com in prepared:
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr, stream=side):
                hh = lay(sp)
                dis(hh, sp)
                com(hh, sp)
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
                         "value": round(step_bytes * args.steps / el / 1e9, 2), "unit": "GB/s",
                         "what": "the same step replayed from a captured HIP graph (one graph per input set)"}
        del graphs
        for hh in live:
            destroy(hh)
    if spec.name == "ht_prefill" and not args.step_only:
        line["decode_shape"] = decode_shape(ep, hx, wl, torch, np, stream_ptr)
    if spec.T * spec.K >= 1024 and not ll and not args.step_only:
        line["once_per_rank"] = once_per_rank(ep, torch, np, spec, sets, stream_ptr)
    if args.extras and not ll:
        line["extras"] = extras(ep, hx, wl, torch, np, group, spec, sets[0], stream_ptr)
    ep.ep_group_destroy(group)
    if not args.no_cpu_baseline and not args.step_only:
        line["cpu_baseline"] = cpu_baseline(w)
        # box share of one GPU: 16 cores, whatever os.cpu_count() shows
        line["cpu_baseline_all_cores"] = cpu_baseline_all_cores(w, threads=min(16, os.cpu_count() or 1))
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
