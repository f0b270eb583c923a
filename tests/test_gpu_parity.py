"""Parity of the HIP path (through the C ABI) with the CPU oracle on identical
seeded inputs: bit-exact for the layout, slot maps and dispatched rows; combine
within 1e-2 absolute or 4e-3 relative of (in fact bit-exact with) the oracle's
float32 k-ascending accumulation, and within one bf16 ulp of its float64 sum."""
import ctypes
import sys

import numpy as np
import pytest
import torch

from paper_2603_13606_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ep():
    from paper_2603_13606_amd import binding
    import ep_harness
    ep_harness.ensure_built()
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return binding


@pytest.fixture(scope="module")
def hx():
    import ep_harness
    return ep_harness


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _group(ep, spec, T_max, mode, C=0, **kw):
    cfg = ep.make_config(spec.R, spec.E, spec.H, spec.K, max(T_max, 1), mode=mode,
                         slots_per_subregion=C, **kw)
    return ep.ep_group_create(cfg)


def _mess_up(topk, E, seed, frac_masked=0.02, n_invalid=0):
    rng = np.random.default_rng(seed)
    topk = topk.copy()
    topk[rng.random(topk.shape) < frac_masked] = -1
    for _ in range(n_invalid):
        t, k = rng.integers(topk.shape[0]), rng.integers(topk.shape[1])
        topk[t, k] = E + int(rng.integers(0, 5))
    return topk


# ------------------------------------------------------------------------------ layout

LAYOUT_CASES = [
    # name, T override, mode, C, masked fraction
    ("tiny", None, "ht", 0, 0.0),
    ("tiny", None, "ll", 6, 0.0),
    ("tiny", 1, "ht", 0, 0.0),
    ("tiny", 33, "ll", 0, 0.1),
    ("ll_decode", None, "ll", 0, 0.0),
    ("ll_decode", None, "ht", 0, 0.02),
    ("ll_decode", 127, "ll", 16, 0.02),
    ("ll_decode", 512, "ht", 0, 0.0),      # 4096 entries: largest one-launch case
    ("ll_decode", 513, "ht", 0, 0.0),      # first three-launch case, ragged
    ("ht_prefill", None, "ht", 0, 0.0),
    ("ht_prefill", 4095, "ht", 0, 0.05),
    ("skew", None, "ll", 512, 0.0),        # hot experts overflow C
    ("skew", None, "ht", 0, 0.0),
    ("skew_rank0", 3001, "ll", 512, 0.01),
    ("stress", None, "ht", 0, 0.0),
    ("stress_hot", None, "ht", 0, 0.0),
    ("stress_hot", 8191, "ll", 300, 0.03),
    ("ht_prefill", 20000, "ht", 0, 0.01),  # 160000 entries: several load groups per wave
    ("stress", 33333, "ll", 700, 0.0),     # 266664 entries
]


@pytest.mark.parametrize("name,T,mode,C,masked", LAYOUT_CASES)
def test_layout_parity(ep, hx, oracle_mod, name, T, mode, C, masked):
    spec = wl.SPECS[name]
    topk, _, _ = wl.make_routing(spec, T=T)
    T = topk.shape[0]
    if masked:
        topk = _mess_up(topk, spec.E, seed=T, frac_masked=masked)
    _say(f"layout case {name} T={T} mode={mode} C={C}")
    ll = mode == "ll"
    g = _group(ep, spec, T, ep.EP_MODE_LL if ll else ep.EP_MODE_HT, C=C)
    try:
        d_topk = torch.from_numpy(topk).to(hx.DEV)
        h = ep.ep_layout(g, d_topk)
        got = hx.fetch_layout(h, T, spec.K, spec.E, spec.R)
        Cc = C if C else T
        want = oracle_mod.layout(topk, E=spec.E, R=spec.R,
                                 layout=oracle_mod.LAYOUT_PADDED if ll else oracle_mod.LAYOUT_CONCAT,
                                 C=Cc if ll else 0, C_rank=T)
        hx.assert_layout_equal(got, want)
        routed = (topk >= 0) & (topk < spec.E)
        assert np.array_equal(got.arrays["entry_rank"], np.where(routed, topk // spec.L, -1))
        assert ep.ep_handle_get_num_recv_tokens(h) == want.kept
        assert bool(got.info.status & ep.STATUS_CAPACITY_DROP) == (want.dropped > 0)
        ep.ep_handle_destroy(h)
    finally:
        ep.ep_group_destroy(g)


@pytest.mark.parametrize("E,R,K,T", [(1, 1, 1, 70), (24, 4, 3, 500), (6, 6, 6, 129), (1024, 64, 16, 2048),
                                     (1000, 8, 5, 3000), (64, 1, 8, 1025)])
def test_layout_odd_shapes(ep, hx, oracle_mod, E, R, K, T):
    """Non-power-of-two experts per rank, K not dividing 64, the limits of E."""
    spec = wl.WorkloadSpec("odd", 9, R=R, T=T, H=64, E=E, K=K)
    topk, _, _ = wl.make_routing(spec)
    topk = _mess_up(topk, E, seed=E + K, frac_masked=0.05)
    _say(f"layout odd E={E} R={R} K={K} T={T}")
    for mode, ll in ((ep.EP_MODE_HT, False), (ep.EP_MODE_LL, True)):
        C = max(1, (2 * T * K) // (3 * E))
        g = _group(ep, spec, T, mode, C=C)
        try:
            h = ep.ep_layout(g, torch.from_numpy(topk).to(hx.DEV))
            got = hx.fetch_layout(h, T, K, E, R)
            want = oracle_mod.layout(topk, E=E, R=R, layout=int(ll), C=C if ll else 0, C_rank=T)
            hx.assert_layout_equal(got, want)
            ep.ep_handle_destroy(h)
        finally:
            ep.ep_group_destroy(g)


def test_layout_duplicate_experts_and_strided_topk(ep, hx, oracle_mod):
    spec = wl.SPECS["tiny"]
    rng = np.random.default_rng(8)
    T, K = 200, 4
    topk = rng.integers(0, 3, (T, K)).astype(np.int32)  # many duplicates within a token
    spec = wl.WorkloadSpec("dup", 9, R=2, T=T, H=64, E=4, K=K)
    g = _group(ep, spec, T, ep.EP_MODE_HT)
    try:
        wide = torch.full((T, K + 3), 77, dtype=torch.int32, device=hx.DEV)
        wide[:, :K] = torch.from_numpy(topk).to(hx.DEV)
        h = ep.ep_layout(g, wide[:, :K])  # row stride K + 3
        got = hx.fetch_layout(h, T, K, 4, 2)
        hx.assert_layout_equal(got, oracle_mod.layout(topk, E=4, R=2, C_rank=T))
        ep.ep_handle_destroy(h)
    finally:
        ep.ep_group_destroy(g)


def test_layout_empty_batch(ep, hx, oracle_mod):
    spec = wl.SPECS["ll_decode"]
    g = _group(ep, spec, 16, ep.EP_MODE_HT)
    try:
        h = ep.ep_layout(g, torch.zeros((0, spec.K), dtype=torch.int32, device=hx.DEV))
        got = hx.fetch_layout(h, 0, spec.K, spec.E, spec.R)
        want = oracle_mod.layout(np.zeros((0, spec.K), np.int32), E=spec.E, R=spec.R, C_rank=1)
        hx.assert_layout_equal(got, want)
        x = torch.zeros((0, spec.H), dtype=torch.bfloat16, device=hx.DEV)
        recv = hx.poison_bf16((4, spec.H))
        out = torch.zeros((0, spec.H), dtype=torch.bfloat16, device=hx.DEV)
        ep.ep_dispatch(h, x, recv)
        ep.ep_combine(h, recv, out)
        torch.cuda.synchronize()
        assert np.all(hx.dev_to_bits(recv) == hx.POISON)
        ep.ep_handle_destroy(h)
    finally:
        ep.ep_group_destroy(g)


@pytest.mark.parametrize("mode,kw", [
    ("ht", {}), ("ll", {}), ("ht", dict(dispatch_order=1)), ("ll", dict(dispatch_order=2)),
    ("ht", dict(dispatch_order=1, quantize_ahead=1)), ("ht", dict(dispatch_path=1)), ("ll", dict(dispatch_path=1)),
    ("ht", dict(staged_buffers=2)), ("ht", dict(ranks_per_node=8))])
def test_empty_batch_through_every_call(ep, hx, oracle_mod, mode, kw):
    """No tokens: every call succeeds, writes no row, reports zero counts, and leaves the output
    tensors as they were (the per-expert counter, which it sets to zero, aside)."""
    _say(f"empty batch mode={mode} {kw}")
    spec = wl.SPECS["ll_decode"]   # H = 7168: a multiple of 128, so the FP8 calls are allowed
    ll = mode == "ll"
    kw = dict(kw)
    if "dispatch_path" in kw:
        kw["dispatch_path"] = ep.EP_PATH_RANK_DEDUP
    g = _group(ep, spec, 64, ep.EP_MODE_LL if ll else ep.EP_MODE_HT, C=4 if ll else 0, **kw)
    try:
        topk = torch.zeros((0, spec.K), dtype=torch.int32, device=hx.DEV)
        x = torch.zeros((0, spec.H), dtype=torch.bfloat16, device=hx.DEV)
        gate = torch.zeros((0, spec.K), dtype=torch.float32, device=hx.DEV)
        rows = spec.E * 4 if ll else 8
        store = hx.poison_bf16((rows, spec.H))
        recv = store.view(spec.E, 4, spec.H) if ll else store
        r_w = torch.full((rows,), -3.5, dtype=torch.float32, device=hx.DEV)
        r_src = torch.full((rows,), -9, dtype=torch.int32, device=hx.DEV)
        cnt = torch.full((spec.E,), -1, dtype=torch.int32, device=hx.DEV)
        out = torch.zeros((0, spec.H), dtype=torch.bfloat16, device=hx.DEV)
        want = oracle_mod.layout(np.zeros((0, spec.K), np.int32), E=spec.E, R=spec.R, layout=int(ll), C=4 if ll else 0, C_rank=64)
        direct = "dispatch_path" not in kw
        for call in ("layout", "prefetch", "one call"):
            if call == "one call":
                if not direct:
                    continue
                h = ep.ep_layout_dispatch(g, topk, x, recv, topk_weights=gate, recv_w=r_w, recv_src=r_src, recv_count=cnt)
            else:
                h = ep.ep_layout(g, topk) if call == "layout" else ep.ep_layout_prefetch(g, topk, x)
                ep.ep_dispatch(h, x, recv, topk_weights=gate, recv_w=r_w, recv_src=r_src, recv_count=cnt,
                               topk_idx=None if direct else topk)  # the once-per-rank headers carry the routing vector
            hx.assert_layout_equal(hx.fetch_layout(h, 0, spec.K, spec.E, spec.R), want)
            assert ep.ep_handle_get_num_recv_tokens(h) == 0
            ep.ep_combine(h, recv, out, topk_weights=gate)
            ep.ep_combine(h, recv, out)
            if direct and not kw.get("ranks_per_node"):
                gy = hx.poison_bf16((rows, spec.H))
                gw = torch.zeros((0, spec.K), dtype=torch.float32, device=hx.DEV)
                gyv = gy.view(spec.E, 4, spec.H) if ll else gy
                ep.ep_combine_backward(h, out, gyv, topk_weights=gate, y=recv, grad_w=gw)
                ep.ep_combine_backward(h, out, gyv, topk_weights=gate)
                if spec.H % 128 == 0:
                    q = torch.full((rows, spec.H), 0x55, dtype=torch.uint8, device=hx.DEV).view(torch.float8_e4m3fn)
                    sc = torch.full((rows, spec.H // 128), -2.0, dtype=torch.float32, device=hx.DEV)
                    ep.ep_dispatch(h, x, q.view(spec.E, 4, spec.H) if ll else q, recv_scales=sc)
                    torch.cuda.synchronize()
                    assert bool((q.view(torch.uint8) == 0x55).all()) and bool((sc == -2.0).all())
                    assert np.all(hx.dev_to_bits(gy) == hx.POISON)
            if kw.get("staged_buffers"):
                ep.ep_dispatch(h, x, recv, send_only=1)
                ep.ep_complete(h)
                ep.ep_combine(h, recv, out, send_only=1)
                ep.ep_complete(h)
            torch.cuda.synchronize()
            assert np.all(hx.dev_to_bits(store) == hx.POISON)
            assert bool((r_w == -3.5).all()) and bool((r_src == -9).all())
            assert np.all(cnt.cpu().numpy() == 0)
            cnt.fill_(-1)
            ep.ep_handle_destroy(h)
    finally:
        ep.ep_group_destroy(g)


def test_layout_invalid_ids_are_flagged_and_skipped(ep, hx, oracle_mod):
    spec = wl.SPECS["ll_decode"]
    topk, _, _ = wl.make_routing(spec)
    topk = _mess_up(topk, spec.E, seed=1, frac_masked=0.01, n_invalid=7)
    topk[5, 1] = -2
    g = _group(ep, spec, spec.T, ep.EP_MODE_HT)
    try:
        h = ep.ep_layout(g, torch.from_numpy(topk).to(hx.DEV))
        got = hx.fetch_layout(h, spec.T, spec.K, spec.E, spec.R, ok=(ep.EP_ERR_INVALID_ROUTING,))
        assert got.info.last_code == ep.EP_ERR_INVALID_ROUTING
        assert got.info.status & ep.STATUS_INVALID_IDS
        want = oracle_mod.layout(topk, E=spec.E, R=spec.R, C_rank=spec.T)
        assert want.invalid >= 1
        hx.assert_layout_equal(got, want)
        ep.ep_handle_destroy(h)
    finally:
        ep.ep_group_destroy(g)


def test_layout_expert_base(ep, hx, oracle_mod):
    """Rows of this source start where lower-ranked sources end: base offsets built
    from seeded routings of the other ranks (stand-in for the metadata exchange)."""
    spec = wl.SPECS["ll_decode"]
    my_rank = 3
    counts = []
    for r in range(spec.R):
        tk, _, _ = wl.make_routing(wl.SPECS["ll_decode"], seed_offset=100 + r)
        counts.append(np.bincount(tk.reshape(-1), minlength=spec.E))
    counts = np.array(counts)
    expert_start = np.concatenate([[0], np.cumsum(counts.sum(0))])[:-1]
    base = (expert_start + counts[:my_rank].sum(0)).astype(np.int32)
    topk, _, _ = wl.make_routing(spec, seed_offset=100 + my_rank)
    g = _group(ep, spec, spec.T, ep.EP_MODE_HT, my_rank=my_rank)
    try:
        h = ep.ep_layout(g, torch.from_numpy(topk).to(hx.DEV), expert_base=torch.from_numpy(base).to(hx.DEV))
        got = hx.fetch_layout(h, spec.T, spec.K, spec.E, spec.R)
        want = oracle_mod.layout(topk, E=spec.E, R=spec.R, expert_base=base, C_rank=spec.T)
        hx.assert_layout_equal(got, want)
        ep.ep_handle_destroy(h)
    finally:
        ep.ep_group_destroy(g)


@pytest.mark.parametrize("n_src,padded,order", [(4, True, 0), (8, True, 0), (4, False, 0), (8, False, 1), (5, False, 2)])
def test_several_sources_into_one_receiver_tensor(ep, hx, oracle_mod, n_src, padded, order):
    """What one GPU can show of (source rank, token index) order: n_src simulated source ranks, each
    with its own routing and group (my_rank = r), dispatch one after another into ONE receiver-shaped
    tensor -- padded [E, R*C, H] through each source's strided view, concatenated [rows, H] through
    expert_base -- and the whole tensor, the side arrays and every count equal the stable sort of
    all entries by (expert, source rank, token, k).  Each source then combines from the shared
    tensor, and its output equals the oracle's for that source."""
    import multi_source as ms
    big = order != 0
    spec = wl.WorkloadSpec("ms", 78, R=n_src, T=2100 if big else 300, H=512 if big else 1000, E=n_src * 4, K=5)
    E, H, K = spec.E, spec.H, spec.K
    tokens = [spec.T, spec.T - 123, 1700 if big else 1, spec.T - 7]
    sources = ms.make_sources(spec, n_src, tokens)
    C = 41
    fill = hx.POISON
    _say(f"several sources: n_src={n_src} padded={padded} order={order}")
    want_rows, want_src, want_w, want_rank = ms.expected_receiver(sources, E, H, padded, C, fill)
    nrows = want_rows.shape[0]
    store = hx.poison_bf16((nrows + 1, H))
    scale = wl.expert_scale_table(spec)
    bases = None if padded else ms.expert_bases(sources, E)
    r_w = torch.full((nrows + 1,), -3.5, dtype=torch.float32, device=hx.DEV)
    r_src = torch.full((nrows + 1,), -9, dtype=torch.int32, device=hx.DEV)
    groups, handles = [], []
    try:
        for s in sources:
            T = s.topk.shape[0]
            cfg = ep.make_config(n_src, E, H, K, spec.T, mode=ep.EP_MODE_LL if padded else ep.EP_MODE_HT,
                                 my_rank=s.rank, slots_per_subregion=C if padded else 0, dispatch_order=order)
            g = ep.ep_group_create(cfg)
            groups.append(g)
            topk = torch.from_numpy(s.topk).to(hx.DEV)
            x = hx.bits_to_dev(s.x_bits)
            gate = torch.from_numpy(s.w).to(hx.DEV)
            cnt = torch.full((E,), -1, dtype=torch.int32, device=hx.DEV)
            if padded:
                recv = store[:nrows].view(E, n_src * C, H)[:, s.rank * C:(s.rank + 1) * C, :]
                lay = oracle_mod.layout(s.topk, E=E, R=n_src, layout=oracle_mod.LAYOUT_PADDED, C=C, C_rank=spec.T)
                side_w = torch.full((E * C,), -3.5, dtype=torch.float32, device=hx.DEV)
                side_src = torch.full((E * C,), -9, dtype=torch.int32, device=hx.DEV)
                h = ep.ep_layout(g, topk)
                ep.ep_dispatch(h, x, recv, topk_weights=gate, recv_w=side_w, recv_src=side_src, recv_count=cnt)
                torch.cuda.synchronize()
                assert np.array_equal(side_src.cpu().numpy(), want_src.reshape(E, n_src, C)[:, s.rank, :].reshape(-1))
                assert np.array_equal(side_w.cpu().numpy(), want_w.reshape(E, n_src, C)[:, s.rank, :].reshape(-1))
            else:
                base = torch.from_numpy(bases[s.rank]).to(hx.DEV)
                lay = oracle_mod.layout(s.topk, E=E, R=n_src, expert_base=bases[s.rank], C_rank=spec.T)
                h = ep.ep_layout_prefetch(g, topk, x, expert_base=base) if order == 1 else ep.ep_layout(g, topk, expert_base=base)
                ep.ep_dispatch(h, x, store[:nrows], topk_weights=gate, recv_w=r_w[:nrows], recv_src=r_src[:nrows], recv_count=cnt)
            hx.assert_layout_equal(hx.fetch_layout(h, T, K, E, n_src), lay)
            assert np.array_equal(cnt.cpu().numpy(), lay.expert_kept)
            handles.append((h, lay, s, gate, base if not padded else None))
        torch.cuda.synchronize()
        got = hx.dev_to_bits(store)
        assert np.array_equal(got[:nrows], want_rows), "receiver tensor differs from the global ordering"
        assert np.all(got[nrows:] == fill)
        if not padded:
            assert np.array_equal(r_src.cpu().numpy()[:nrows], want_src) and np.array_equal(r_w.cpu().numpy()[:nrows], want_w)
        # experts run on the shared tensor; every source combines its own tokens back
        if padded:
            row_e = np.repeat(np.arange(E), n_src * C)
        else:
            row_e = np.repeat(np.arange(E), np.diff(np.concatenate([bases[0], [nrows]])))
        o_y = hx.expert_standin_np(want_rows, row_e, scale)
        d_y = hx.expert_standin(store[:nrows], torch.from_numpy(row_e).to(hx.DEV), scale)
        assert np.array_equal(hx.dev_to_bits(d_y), o_y)
        for h, lay, s, gate, base in handles:
            T = s.topk.shape[0]
            out = hx.poison_bf16((T, H))
            if padded:
                y_view = d_y.view(E, n_src * C, H)[:, s.rank * C:(s.rank + 1) * C, :]
                ep.ep_combine(h, y_view, out, topk_weights=gate)
                o_view = o_y.reshape(E, n_src * C, H)[:, s.rank * C:(s.rank + 1) * C, :]
                ref = oracle_mod.combine(o_view, s.w, lay, H, acc="f32", stride0=n_src * C * H, stride1=H)
            else:
                ep.ep_combine(h, d_y, out, topk_weights=gate)
                ref = oracle_mod.combine(o_y, s.w, lay, H, acc="f32")
            torch.cuda.synchronize()
            assert np.array_equal(hx.dev_to_bits(out), ref), f"combine of source {s.rank} differs"
    finally:
        for h, *_ in handles:
            ep.ep_handle_destroy(h)
        for g in groups:
            ep.ep_group_destroy(g)


def test_layout_many_launches_on_one_slab(ep, hx, oracle_mod):
    """The workgroups of a layout launch tell each other's published counts from stale ones by a
    tag that counts the launches on the handle's slab and starts over after 255 of them (the
    published words are cleared at that point): more than two such cycles on one slab, every
    result equal to the oracle's."""
    spec = wl.SPECS["skew"]
    T = 1200  # 9600 entries: several workgroups
    g = _group(ep, spec, T, ep.EP_MODE_HT, max_handles=1)
    try:
        want = {}
        tops = []
        for v in range(3):
            topk, _, _ = wl.make_routing(spec, T=T, seed_offset=v)
            tops.append((torch.from_numpy(topk).to(hx.DEV), oracle_mod.layout(topk, E=spec.E, R=spec.R, C_rank=T)))
        n = T * spec.K
        for it in range(600):
            d_topk, lay = tops[it % 3]
            h = ep.ep_layout(g, d_topk)
            info = ep.ep_handle_query(h)
            got = ep.read_device_i32(info.dst_row, n).numpy().reshape(T, spec.K)
            assert np.array_equal(got, lay.dst_row), f"launch {it}"
            assert int(info.status) == 0 and int(info.rows_kept) == lay.kept
            if it % 85 == 0 or it in (254, 255, 256, 509, 510, 511):
                hx.assert_layout_equal(hx.fetch_layout(h, T, spec.K, spec.E, spec.R), lay)
            ep.ep_handle_destroy(h)
    finally:
        ep.ep_group_destroy(g)


def test_layout_is_deterministic(ep, hx):
    spec = wl.SPECS["stress_hot"]
    topk, _, _ = wl.make_routing(spec)
    g = _group(ep, spec, spec.T, ep.EP_MODE_HT, max_handles=3)
    try:
        d = torch.from_numpy(topk).to(hx.DEV)
        first = None
        for i in range(10):
            h = ep.ep_layout(g, d)
            got = hx.fetch_layout(h, spec.T, spec.K, spec.E, spec.R)
            blob = np.concatenate([v.reshape(-1) for v in got.arrays.values()])
            if first is None:
                first = blob
            assert np.array_equal(first, blob), f"run {i} differs"
            ep.ep_handle_destroy(h)
    finally:
        ep.ep_group_destroy(g)


# ------------------------------------------------------------------------------ dispatch + combine

PATH_CASES = [
    # name, T override, H override, mode, C
    ("tiny", None, None, "ht", 0),
    ("tiny", None, None, "ll", 6),
    ("ll_decode", None, None, "ll", 0),
    ("ll_decode", 77, None, "ht", 0),
    ("ll_decode", 50, 1000, "ht", 0),      # row of 2000 bytes: ragged last 1 KiB segment
    ("ll_decode", 50, 8, "ll", 9),         # smallest row: one 16-byte unit
    ("skew", 1111, None, "ll", 139),
    ("skew", 1111, None, "ht", 0),
    ("ht_prefill", None, None, "ht", 0),   # full benchmark shape
    ("skew", None, None, "ll", 512),       # full skewed shape, hot experts overflow C = 2*T*K/E
    ("stress_hot", None, None, "ht", 0),   # full stress shape, 8 of 64 ranks take half the traffic
    ("stress", None, None, "ht", 0),       # full stress shape, uniform routing
    # more entries per token than the 8 a combine wave gathers at a time, up to the limit of 64
    (("skew", dict(K=17)), 300, 520, "ht", 0),
    (("skew", dict(K=33)), 300, 520, "ll", 90),
    (("skew", dict(K=64)), 130, 1000, "ht", 0),
    (("skew", dict(K=64)), 130, 256, "ll", 70),
    # long enough for combine's two 1 KiB segments per wavefront, rows that end inside the second one
    ("skew", 1100, 8136, "ht", 0),         # 1017 units: the last segment holds 57
    ("skew", 1100, 7688, "ll", 139),       # 961 units: the last segment holds one; entries without rows
    # 14 336-byte rows in whole rounds of resident wavefronts (2048 tokens on 256 compute units): combine gives
    # a whole row to one wavefront; fewer and more than its eight straight-line entries, entries without rows,
    # a last workgroup with a token missing
    (("ht_prefill", dict(K=5)), 2048, None, "ht", 0),
    (("ht_prefill", dict(K=17)), 2048, None, "ht", 0),
    ("ht_prefill", 2048, None, "ll", 40),
    ("ht_prefill", 3899, None, "ht", 0),
]


def _run_path(ep, hx, oracle_mod, name, T, H, mode, C, masked=0.01, weights=True, order=0, prefetch=False, fused=False,
              reroute=None):
    over = {}
    if isinstance(name, tuple):  # (workload name, overrides of its shape)
        name, over = name[0], dict(name[1])
    w = wl.make_workload(name, T=T, **({"H": H} if H else {}), **over)
    spec = w.spec
    T = spec.T
    topk = _mess_up(w.topk_idx, spec.E, seed=T + spec.H, frac_masked=masked)
    if reroute is not None:  # a degenerate routing in place of the seeded one
        topk = np.ascontiguousarray(reroute(topk, spec).astype(np.int32))
    ll = mode == "ll"
    Cc = (C if C else T) if ll else 0
    lay = oracle_mod.layout(topk, E=spec.E, R=spec.R, layout=int(ll), C=Cc, C_rank=T)
    rows = spec.E * Cc if ll else int(lay.expert_offset[-1])
    guard = 2
    # ---- oracle side
    o_recv = np.full((rows + guard, spec.H), hx.POISON, np.uint16)
    o_w = np.full(rows + guard, np.float32(-3.5), np.float32)
    o_src = np.full(rows + guard, -9, np.int32)
    oracle_mod.dispatch(w.x_bits, w.topk_w if weights else None, lay, o_recv, o_w, o_src)
    # ---- HIP side
    g = _group(ep, spec, T, ep.EP_MODE_LL if ll else ep.EP_MODE_HT, C=C, dispatch_order=order)
    try:
        x = hx.bits_to_dev(w.x_bits)
        d_w = torch.from_numpy(w.topk_w).to(hx.DEV)
        store = hx.poison_bf16((rows + guard, spec.H))
        recv = store[:rows].view(spec.E, Cc, spec.H) if ll else store[:rows]
        r_w = torch.full((rows + guard,), -3.5, dtype=torch.float32, device=hx.DEV)
        r_src = torch.full((rows + guard,), -9, dtype=torch.int32, device=hx.DEV)
        r_cnt = torch.full((spec.E,), -1, dtype=torch.int32, device=hx.DEV)
        outs = dict(topk_weights=d_w if weights else None, recv_w=r_w[:rows] if rows else r_w[:0],
                    recv_src=r_src[:rows], recv_count=r_cnt)
        if fused:  # layout and dispatch in one call (one launch for small inputs)
            h = ep.ep_layout_dispatch(g, torch.from_numpy(topk).to(hx.DEV), x, recv, **outs)
            hx.assert_layout_equal(hx.fetch_layout(h, T, spec.K, spec.E, spec.R, ok=(ep.EP_SUCCESS, ep.EP_ERR_INVALID_ROUTING)), lay)
        else:
            if prefetch:
                h = ep.ep_layout_prefetch(g, torch.from_numpy(topk).to(hx.DEV), x)
                hx.assert_layout_equal(hx.fetch_layout(h, T, spec.K, spec.E, spec.R, ok=(ep.EP_SUCCESS, ep.EP_ERR_INVALID_ROUTING)), lay)
            else:
                h = ep.ep_layout(g, torch.from_numpy(topk).to(hx.DEV))
            ep.ep_dispatch(h, x, recv, **outs)
        torch.cuda.synchronize()
        got = hx.dev_to_bits(store)
        assert np.array_equal(got, o_recv), "dispatched rows differ"
        assert np.array_equal(r_w.cpu().numpy(), o_w)  # without gate weights: 1.0 at every placed row
        assert np.array_equal(r_src.cpu().numpy(), o_src)
        assert np.array_equal(r_cnt.cpu().numpy(), lay.expert_kept)
        # ---- experts (harness), then combine
        scale = wl.expert_scale_table(spec)
        if ll:
            row_e = np.repeat(np.arange(spec.E), Cc)
        else:
            row_e = np.repeat(np.arange(spec.E), lay.expert_count)
        o_y = hx.expert_standin_np(o_recv[:rows], row_e, scale)
        d_y_store = hx.poison_bf16((rows + guard, spec.H))
        d_y_store[:rows] = hx.expert_standin(store[:rows], torch.from_numpy(row_e).to(hx.DEV), scale)
        assert np.array_equal(hx.dev_to_bits(d_y_store[:rows]), o_y), "stand-in experts differ (harness)"
        d_y = d_y_store[:rows].view(spec.E, Cc, spec.H) if ll else d_y_store[:rows]
        for use_w in ((True, False) if weights else (False,)):
            out_store = hx.poison_bf16((T + guard, spec.H))
            ep.ep_combine(h, d_y, out_store[:T], topk_weights=d_w if use_w else None)
            torch.cuda.synchronize()
            got_out = hx.dev_to_bits(out_store)
            assert np.all(got_out[T:] == hx.POISON), "combine wrote past its output"
            wts = w.topk_w if use_w else None
            # the accumulation the path is specified with: float32, k ascending
            ref32 = oracle_mod.combine(o_y, wts, lay, spec.H, acc="f32")
            ok, worst = hx.combine_tolerance_ok(got_out[:T], ref32)
            assert ok, f"combine outside tolerance, worst abs diff {worst}"
            assert np.array_equal(got_out[:T], ref32), "combine differs from ordered float32 accumulation"
            # against the float64 definition the float32 sum may land on the other side of a
            # bf16 rounding boundary: equal or adjacent bf16 values, and only rarely adjacent
            ref64 = oracle_mod.combine(o_y, wts, lay, spec.H, acc="f64")
            dist = hx.bf16_ulp_distance(got_out[:T], ref64)
            assert dist.max(initial=0) <= 1, "combine more than one bf16 ulp from the float64 oracle"
            assert (dist != 0).mean() < 2e-3 if dist.size else True
        ep.ep_handle_destroy(h)
    finally:
        ep.ep_group_destroy(g)


def _all_masked(topk, spec):
    return np.full_like(topk, -1)


def _one_expert(topk, spec):          # every token has one entry, all for the same expert
    out = np.full_like(topk, -1)
    out[:, 0] = 5
    return out


def _same_experts(topk, spec):        # every token names experts 0 .. K-1: K bins hold everything
    return np.broadcast_to(np.arange(spec.K, dtype=np.int32), topk.shape).copy()


def _k_times_one_expert(topk, spec):  # all K entries of a token name one expert: K rows of it, one message to its rank
    return np.repeat((np.arange(topk.shape[0], dtype=np.int32) * 7 % spec.E)[:, None], spec.K, axis=1)


def _last_expert_only(topk, spec):    # the highest expert id takes everything but a few masked entries
    out = np.full_like(topk, spec.E - 1)
    out[::13, 1] = -1
    return out


@pytest.mark.parametrize("order", [0, 1])
@pytest.mark.parametrize("mode,C", [("ht", 0), ("ll", 139)])
@pytest.mark.parametrize("reroute", [_all_masked, _one_expert, _same_experts, _k_times_one_expert, _last_expert_only])
def test_degenerate_routings(ep, hx, oracle_mod, reroute, mode, C, order):
    """Routings at the edges of what the layout can be given: nothing routed, one expert or K experts
    taking everything (one long run of rows; in padded windows nearly everything cut), K rows of one
    token in one expert; in both walks of the dispatch (8800 entries: the destination order applies)."""
    _say(f"degenerate routing {reroute.__name__} mode={mode} C={C} order={order}")
    _run_path(ep, hx, oracle_mod, "skew", 1100, 1024, mode, C, masked=0.0, order=order, reroute=reroute)


@pytest.mark.parametrize("T,H", [(64, 520), (1100, 8192), (2048, 7168)])  # one segment, two segments, whole rows per wavefront
def test_combine_strided_windows_and_output(ep, hx, oracle_mod, T, H):
    """Expert outputs and the combined tokens as column slices of wider tensors (row pitch larger than H):
    the rows are found through the strides, and nothing is written between the rows of the output."""
    _say(f"combine strided T={T} H={H}")
    spec = wl.WorkloadSpec("strided", 32, R=8, T=T, H=H, E=64, K=8)
    topk, gate, _ = wl.make_routing(spec)
    topk = _mess_up(topk, spec.E, seed=T + 1, frac_masked=0.02)
    lay = oracle_mod.layout(topk, E=spec.E, R=spec.R, C_rank=T)
    rows = int(lay.expert_offset[-1])
    rng = np.random.default_rng(H - T)
    y_bits = wl.f32_to_bf16_bits(rng.standard_normal((rows, H)).astype(np.float32))
    g = _group(ep, spec, T, ep.EP_MODE_HT)
    try:
        h = ep.ep_layout(g, torch.from_numpy(topk).to(hx.DEV))
        y_wide = hx.poison_bf16((rows, H + 64))
        y_wide[:, :H] = hx.bits_to_dev(y_bits)
        out_wide = hx.poison_bf16((T, H + 40))
        ep.ep_combine(h, y_wide[:, :H], out_wide[:, :H], topk_weights=torch.from_numpy(gate).to(hx.DEV))
        torch.cuda.synchronize()
        got = hx.dev_to_bits(out_wide)
        assert np.array_equal(got[:, :H], oracle_mod.combine(y_bits, gate, lay, H, acc="f32"))
        assert np.all(got[:, H:] == hx.POISON), "combine wrote between the rows of its output"
        ep.ep_handle_destroy(h)
    finally:
        ep.ep_group_destroy(g)


@pytest.mark.parametrize("T,H", [(64, 520), (1100, 8192), (2048, 7168)])  # one segment, two segments, whole rows per wavefront
def test_combine_special_values(ep, hx, oracle_mod, T, H):
    """Expert outputs and gate weights full of the values arithmetic treats specially -- NaNs of either
    sign, infinities, signed zeros, bf16 and float32 subnormals, the largest finite values, weights of
    0, -0, infinity and NaN -- combine bit for bit like the oracle's ordered float32 sum: products that
    overflow, inf - inf, 0 * inf, subnormal products (no flush to zero), every NaN leaving as 0x7FC0."""
    _say(f"combine special values T={T} H={H}")
    spec = wl.WorkloadSpec("special", 31, R=8, T=T, H=H, E=64, K=8)
    topk, gate, _ = wl.make_routing(spec)
    topk = _mess_up(topk, spec.E, seed=T, frac_masked=0.02)
    lay = oracle_mod.layout(topk, E=spec.E, R=spec.R, C_rank=T)
    rows = int(lay.expert_offset[-1])
    rng = np.random.default_rng(H + T)
    y_bits = wl.f32_to_bf16_bits(rng.standard_normal((rows, H)).astype(np.float32))
    pool = np.array([0x7FC0, 0xFFC0, 0x7FA1, 0x7F80, 0xFF80, 0x0000, 0x8000, 0x0001, 0x8001, 0x007F, 0x0080,
                     0x7F7F, 0xFF7F, 0x7F00, 0x0C00, 0x8C00], np.uint16)
    pick = rng.random((rows, H)) < 0.02
    y_bits[pick] = pool[rng.integers(0, pool.size, int(pick.sum()))]
    wpool = np.array([0.0, -0.0, 1.0, -1.0, np.inf, -np.inf, np.nan, 3.0e38, -3.0e38, 1.0e-38, 1.0e-45, 2.0 ** -100],
                     np.float32)
    wts = gate.copy()
    wpick = rng.random(wts.shape) < 0.05
    wts[wpick] = wpool[rng.integers(0, wpool.size, int(wpick.sum()))]
    g = _group(ep, spec, T, ep.EP_MODE_HT)
    try:
        h = ep.ep_layout(g, torch.from_numpy(topk).to(hx.DEV))
        d_y = hx.bits_to_dev(y_bits)
        d_w = torch.from_numpy(wts).to(hx.DEV)
        for use_w in (True, False):
            out = hx.poison_bf16((T, H))
            ep.ep_combine(h, d_y, out, topk_weights=d_w if use_w else None)
            torch.cuda.synchronize()
            got = hx.dev_to_bits(out)
            want = oracle_mod.combine(y_bits, wts if use_w else None, lay, H, acc="f32")
            nan = (want & 0x7FFF) > 0x7F80
            assert nan.any() and ((want & 0x7FFF) == 0x7F80).any()  # the inputs do produce NaNs and infinities
            assert np.all(want[nan] == 0x7FC0)
            assert np.array_equal(got, want), f"{int((got != want).sum())} of {got.size} outputs differ"
        ep.ep_handle_destroy(h)
    finally:
        ep.ep_group_destroy(g)


@pytest.mark.parametrize("name,T,H,mode,C", PATH_CASES)
def test_dispatch_combine_parity(ep, hx, oracle_mod, name, T, H, mode, C):
    _say(f"path case {name} T={T} H={H} mode={mode} C={C}")
    _run_path(ep, hx, oracle_mod, name, T, H, mode, C)


FUSED_CASES = [
    # inputs of at most 1024 routed entries: ep_layout_dispatch lays out and dispatches in one launch
    ("ll_decode", None, None, "ll", 0, 0),     # the decode shape, padded windows
    ("ll_decode", None, None, "ht", 0, 0),     # concatenated windows
    ("ll_decode", 127, None, "ll", 16, 0),     # capacity drops, ragged last wave
    ("ll_decode", 50, 1000, "ht", 0, 1),       # ragged last 1 KiB segment; group set to the destination order
    ("ll_decode", 50, 8, "ll", 9, 0),          # smallest row: one 16-byte unit
    ("tiny", None, None, "ht", 0, 0),
    ("tiny", None, None, "ll", 6, 0),
    ("tiny", 1, None, "ht", 0, 0),             # one token
    ("skew", 100, None, "ll", 7, 0),           # 800 entries on 128 experts, most of them dropped
    ("skew", 128, 4096, "ht", 0, 0),           # exactly 1024 entries
    ("ll_decode", 129, 512, "ht", 0, 0),       # 1032 entries: falls back to two launches
    ("ht_prefill", 1500, 256, "ht", 0, 1),     # large input: two launches, destination order with read-ahead
]


@pytest.mark.parametrize("weights", [True, False])
@pytest.mark.parametrize("name,T,H,mode,C,order", FUSED_CASES)
def test_layout_dispatch_one_call_parity(ep, hx, oracle_mod, name, T, H, mode, C, order, weights):
    """ep_layout_dispatch = ep_layout + ep_dispatch: every array of the layout, the dispatched rows,
    side arrays and counts equal the oracle's, untouched rows stay untouched, and combine on the
    handle it returns is unchanged."""
    _say(f"one-call case {name} T={T} H={H} mode={mode} C={C} order={order} weights={weights}")
    _run_path(ep, hx, oracle_mod, name, T, H, mode, C, order=order, weights=weights, fused=True)


def test_layout_dispatch_one_call_random_shapes(ep, hx, oracle_mod):
    """Thirty seeded random small configurations (odd expert counts per rank, K up to 64, strided
    top-k rows, invalid and masked ids, expert_base) through ep_layout_dispatch."""
    rng = np.random.default_rng(31337)
    for case in range(30):
        R = int(rng.choice([1, 2, 3, 4, 8, 16, 32]))
        L = int(rng.choice([1, 2, 3, 4, 8, 13]))
        E = R * L
        K = int(rng.choice([1, 2, 3, 5, 8, 17, 33, 64]))
        K = min(K, E)
        T = int(rng.integers(1, 1024 // K + 1))
        H = int(rng.choice([8, 64, 200, 512, 520, 1024, 7168]))
        ll = bool(rng.integers(0, 2))
        C = int(rng.integers(1, max(2, (3 * T * K) // (2 * E) + 2))) if ll else 0
        use_base = (not ll) and bool(rng.integers(0, 2))
        spec = wl.WorkloadSpec(f"randsmall{case}", 240 + case, R=R, T=T, H=H, E=E, K=K)
        w = wl.make_workload(spec)
        topk = _mess_up(w.topk_idx, E, seed=case, frac_masked=float(rng.choice([0.0, 0.05, 0.5])),
                        n_invalid=int(rng.integers(0, 3)))
        base = None
        if use_base:  # rows of lower-ranked sources precede this source's rows in every expert region
            cnt = np.bincount(topk[(topk >= 0) & (topk < E)], minlength=E)
            other = rng.integers(0, 5, size=E)
            base = (np.concatenate([[0], np.cumsum(cnt + other)[:-1]]) + other // 2).astype(np.int32)
        _say(f"one-call random case {case}: E={E} R={R} K={K} T={T} H={H} ll={ll} C={C} base={use_base}")
        lay = oracle_mod.layout(topk, E=E, R=R, layout=int(ll), C=C if ll else 0, C_rank=T, expert_base=base)
        rows = E * C if ll else int(lay.expert_offset[-1])
        o_recv = np.full((rows + 1, H), hx.POISON, np.uint16)
        o_w = np.full(rows + 1, np.float32(-3.5), np.float32)
        o_src = np.full(rows + 1, -9, np.int32)
        oracle_mod.dispatch(w.x_bits, w.topk_w, lay, o_recv, o_w, o_src)
        g = _group(ep, spec, T, ep.EP_MODE_LL if ll else ep.EP_MODE_HT, C=C)
        try:
            wide = torch.full((T, K + 3), -1, dtype=torch.int32, device=hx.DEV)  # strided top-k rows
            wide[:, :K] = torch.from_numpy(topk).to(hx.DEV)
            store = hx.poison_bf16((rows + 1, H))
            recv = store[:rows].view(E, C, H) if ll else store[:rows]
            r_w = torch.full((rows + 1,), -3.5, dtype=torch.float32, device=hx.DEV)
            r_src = torch.full((rows + 1,), -9, dtype=torch.int32, device=hx.DEV)
            r_cnt = torch.full((E,), -1, dtype=torch.int32, device=hx.DEV)
            gate = torch.from_numpy(w.topk_w).to(hx.DEV)
            h = ep.ep_layout_dispatch(g, wide[:, :K], hx.bits_to_dev(w.x_bits), recv, topk_weights=gate,
                                      recv_w=r_w[:rows], recv_src=r_src[:rows], recv_count=r_cnt,
                                      expert_base=torch.from_numpy(base).to(hx.DEV) if use_base else None)
            got = hx.fetch_layout(h, T, K, E, R, ok=(ep.EP_SUCCESS, ep.EP_ERR_INVALID_ROUTING))
            hx.assert_layout_equal(got, lay)
            out = hx.poison_bf16((T, H))
            ep.ep_combine(h, recv, out, topk_weights=gate)
            torch.cuda.synchronize()
            assert np.array_equal(hx.dev_to_bits(store), o_recv), f"case {case}: rows differ"
            assert np.array_equal(r_w.cpu().numpy(), o_w) and np.array_equal(r_src.cpu().numpy(), o_src)
            assert np.array_equal(r_cnt.cpu().numpy(), lay.expert_kept)
            ref = oracle_mod.combine(o_recv[:rows], w.topk_w, lay, H, acc="f32")
            assert np.array_equal(hx.dev_to_bits(out), ref), f"case {case}: combine differs"
            ep.ep_handle_destroy(h)
        finally:
            ep.ep_group_destroy(g)


def test_layout_dispatch_one_call_errors_and_overflow(ep, hx, oracle_mod):
    """A bad dispatch argument returns no handle and leaves none alive; an output with too few
    rows is flagged (status bit 2) and not overrun, in the one-launch path as in ep_dispatch."""
    w = wl.make_workload("ll_decode", T=100, H=256)
    spec = w.spec
    g = _group(ep, spec, 100, ep.EP_MODE_HT)
    try:
        topk = torch.from_numpy(w.topk_idx).to(hx.DEV)
        x = hx.bits_to_dev(w.x_bits)
        lay = oracle_mod.layout(w.topk_idx, E=spec.E, R=spec.R, C_rank=100)
        rows = lay.kept
        with pytest.raises(ep.EpError) as e:
            ep.ep_layout_dispatch(g, topk, x[:50], hx.poison_bf16((rows, spec.H)))  # tokens of the wrong length
        assert e.value.code == ep.EP_ERR_INVALID_ARG
        assert ep.ep_group_query(g).live_handles == 0
        short = rows - 37
        store = hx.poison_bf16((rows, spec.H))
        h = ep.ep_layout_dispatch(g, topk, x, store[:short])
        info = ep.ep_handle_query(h, ok=(ep.EP_ERR_OVERFLOW,))
        assert info.status & ep.STATUS_OUTPUT_OVERFLOW
        torch.cuda.synchronize()
        o_recv = np.full((rows, spec.H), hx.POISON, np.uint16)
        oracle_mod.dispatch(w.x_bits, None, lay, o_recv)
        o_recv[short:] = hx.POISON
        assert np.array_equal(hx.dev_to_bits(store), o_recv)
        ep.ep_handle_destroy(h)
    finally:
        ep.ep_group_destroy(g)


ORDER_CASES = [
    # inputs of at least 8192 routed entries take the destination-ordered kernel
    ("ht_prefill", None, None, "ht", 0),
    ("skew", None, None, "ll", 512),        # padded windows, capacity drops, 8 KiB rows
    ("skew", 1111, None, "ht", 0),          # 8888 entries: just above the switch, ragged last chunk
    ("ll_decode", 1100, 1000, "ht", 0),     # 125 units per row: uneven slices, the last one short
    ("ll_decode", 1030, 64, "ll", 40),      # one unit per slice, heavy drops
    ("stress_hot", None, None, "ht", 0),    # 117 MB of tokens: two read passes
    ("ll_decode", 200, None, "ht", 0),      # below the switch: token order whatever the setting
    (("skew", dict(K=33)), 300, 520, "ht", 0),   # 9900 entries of 33 per token
    (("skew", dict(K=64)), 200, 1024, "ll", 150),
]


@pytest.mark.parametrize("order", [1, 2, "1 with ep_layout_prefetch", "0 with ep_layout_prefetch"])
@pytest.mark.parametrize("name,T,H,mode,C", ORDER_CASES)
def test_dispatch_destination_order_parity(ep, hx, oracle_mod, name, T, H, mode, C, order):
    """The destination-ordered dispatch (with and without its read pass) writes exactly the
    bytes of the oracle's dispatch, side arrays and counts included, and leaves the rest of the
    windows untouched; combine on top of it is unchanged."""
    _say(f"order case {name} T={T} H={H} mode={mode} C={C} order={order}")
    prefetch = isinstance(order, str)  # the layout launch also reads the tokens (a hint: same results)
    _run_path(ep, hx, oracle_mod, name, T, H, mode, C, order=int(str(order)[0]), prefetch=prefetch)


def test_layout_dispatch_one_call_quantises_ahead(ep, hx, oracle_mod):
    """ep_layout_dispatch on a large input with FP8 outputs in a group that quantises ahead: the
    layout part quantises the tokens it is given, the dispatch part copies the staged rows; codes,
    scales and the layout equal the oracle's.  The same call on a group without the option
    quantises in the dispatch."""
    w = wl.make_workload("skew", T=1200, H=1024)
    spec = w.spec
    T, G = spec.T, spec.H // 128
    topk = _mess_up(w.topk_idx, spec.E, seed=11, frac_masked=0.01)
    lay = oracle_mod.layout(topk, E=spec.E, R=spec.R, C_rank=T)
    rows = int(lay.expert_offset[-1])
    o_q = np.full((rows + 1, spec.H), 0xAB, np.uint8)
    o_s = np.full((rows + 1, G), np.float32(-2.0), np.float32)
    oracle_mod.dispatch_fp8(w.x_bits, lay, o_q, o_s)
    for ahead in (1, 0):
        _say(f"one call, fp8, quantize_ahead={ahead}")
        g = _group(ep, spec, T, ep.EP_MODE_HT, dispatch_order=1, quantize_ahead=ahead)
        try:
            store = torch.full((rows + 1, spec.H), 0xAB, dtype=torch.uint8, device=hx.DEV)
            scales = torch.full((rows + 1, G), -2.0, dtype=torch.float32, device=hx.DEV)
            h = ep.ep_layout_dispatch(g, torch.from_numpy(topk).to(hx.DEV), hx.bits_to_dev(w.x_bits),
                                      store[:rows].view(torch.float8_e4m3fn), recv_scales=scales[:rows])
            torch.cuda.synchronize()
            hx.assert_layout_equal(hx.fetch_layout(h, T, spec.K, spec.E, spec.R), lay)
            assert np.array_equal(store.cpu().numpy(), o_q) and np.array_equal(scales.cpu().numpy(), o_s)
            ep.ep_handle_destroy(h)
        finally:
            ep.ep_group_destroy(g)
    # the option needs the destination order, the direct path and whole 128-channel groups
    for bad in (dict(dispatch_order=0), dict(dispatch_order=2), dict(dispatch_path=ep.EP_PATH_RANK_DEDUP, dispatch_order=1)):
        with pytest.raises(ep.EpError) as e:
            _group(ep, spec, T, ep.EP_MODE_HT, quantize_ahead=1, **bad)
        assert e.value.code == ep.EP_ERR_INVALID_ARG
    with pytest.raises(ep.EpError):
        ep.ep_group_create(ep.make_config(spec.R, spec.E, 1000, spec.K, T, dispatch_order=1, quantize_ahead=1))


def test_padded_destination_order_follows_the_drop_hint(ep, hx, oracle_mod):
    """Padded windows in a destination-ordered group: the layout leaves the kept / dropped row
    counts where the host can see them, and a later dispatch walks the tokens when the capacity
    cut most entries.  The hint is what the oracle counts; every dispatch -- before the hint is
    there (run order), with a hint that says "mostly dropped" (token walk), and after routing
    without drops has turned it back -- writes the oracle's bytes."""
    w = wl.make_workload("skew", T=1100, H=512)          # 8800 entries: above the run-order switch
    spec = w.spec
    T, C = spec.T, 80   # the skewed routing loses 6324 of 8800 entries to it, the even one 20
    rng = np.random.default_rng(5)
    flat = np.stack([rng.permutation(spec.E)[: spec.K] for _ in range(T)]).astype(np.int32)  # even routing
    g = _group(ep, spec, T, ep.EP_MODE_LL, C=C, dispatch_order=ep.EP_ORDER_DESTINATION)
    try:
        x = hx.bits_to_dev(w.x_bits)
        d_w = torch.from_numpy(w.topk_w).to(hx.DEV)
        rows = spec.E * C
        assert (ep.ep_group_query(g).hint_rows_kept, ep.ep_group_query(g).hint_rows_dropped) == (0, 0)
        seen = []
        for step, topk in enumerate([w.topk_idx, w.topk_idx, flat, flat, w.topk_idx]):
            _say(f"drop hint step {step}")
            lay = oracle_mod.layout(topk, E=spec.E, R=spec.R, layout=1, C=C, C_rank=T)
            o_recv = np.full((rows, spec.H), hx.POISON, np.uint16)
            o_w = np.full(rows, np.float32(-3.5), np.float32)
            o_src = np.full(rows, -9, np.int32)
            oracle_mod.dispatch(w.x_bits, w.topk_w, lay, o_recv, o_w, o_src)
            store = hx.poison_bf16((rows, spec.H))
            r_w = torch.full((rows,), -3.5, dtype=torch.float32, device=hx.DEV)
            r_src = torch.full((rows,), -9, dtype=torch.int32, device=hx.DEV)
            h = ep.ep_layout_prefetch(g, torch.from_numpy(topk).to(hx.DEV), x)
            ep.ep_dispatch(h, x, store.view(spec.E, C, spec.H), topk_weights=d_w, recv_w=r_w, recv_src=r_src)
            torch.cuda.synchronize()
            assert np.array_equal(hx.dev_to_bits(store), o_recv)
            assert np.array_equal(r_w.cpu().numpy(), o_w) and np.array_equal(r_src.cpu().numpy(), o_src)
            info = ep.ep_group_query(g)
            assert (info.hint_rows_kept, info.hint_rows_dropped) == (int(lay.kept), int(lay.dropped))
            seen.append(2 * int(lay.dropped) > int(lay.kept))
            ep.ep_handle_destroy(h)
        assert seen == [True, True, False, False, True], "the two routings should sit on either side of the switch"
    finally:
        ep.ep_group_destroy(g)
    # a group that walks the tokens anyway keeps no hint
    g0 = _group(ep, spec, T, ep.EP_MODE_LL, C=C, dispatch_order=ep.EP_ORDER_TOKEN)
    h = ep.ep_layout(g0, torch.from_numpy(w.topk_idx).to(hx.DEV))
    torch.cuda.synchronize()
    assert ep.ep_group_query(g0).hint_rows_dropped == 0
    ep.ep_handle_destroy(h)
    ep.ep_group_destroy(g0)


def test_destination_order_output_too_small_is_flagged_not_overrun(ep, hx, oracle_mod):
    w = wl.make_workload("ll_decode", T=1100, H=256)
    spec = w.spec
    lay = oracle_mod.layout(w.topk_idx, E=spec.E, R=spec.R, C_rank=spec.T)
    cap = 5000
    g = _group(ep, spec, spec.T, ep.EP_MODE_HT, dispatch_order=ep.EP_ORDER_DESTINATION)
    try:
        h = ep.ep_layout(g, torch.from_numpy(w.topk_idx).to(hx.DEV))
        store = hx.poison_bf16((spec.T * spec.K, spec.H))
        ep.ep_dispatch(h, hx.bits_to_dev(w.x_bits), store[:cap])
        info = ep.ep_handle_query(h, ok=(ep.EP_ERR_OVERFLOW,))
        assert info.last_code == ep.EP_ERR_OVERFLOW and info.status & ep.STATUS_OUTPUT_OVERFLOW
        got = hx.dev_to_bits(store)
        assert np.all(got[cap:] == hx.POISON)
        o = np.full((spec.T * spec.K, spec.H), hx.POISON, np.uint16)
        oracle_mod.dispatch(w.x_bits, None, lay, o)
        assert np.array_equal(got[:cap], o[:cap])
        ep.ep_handle_destroy(h)
    finally:
        ep.ep_group_destroy(g)


def test_layout_prefetch_rejects_a_wrong_tokens_tensor(ep, hx):
    w = wl.make_workload("ll_decode", T=1100, H=256)
    spec = w.spec
    g = _group(ep, spec, spec.T, ep.EP_MODE_HT, dispatch_order=ep.EP_ORDER_DESTINATION)
    try:
        topk = torch.from_numpy(w.topk_idx).to(hx.DEV)
        x = hx.bits_to_dev(w.x_bits)
        for bad in (x[:-1], x[:, :128], x.float()):
            with pytest.raises(ep.EpError) as ei:
                ep.ep_layout_prefetch(g, topk, bad)
            assert ei.value.code == ep.EP_ERR_INVALID_ARG
        assert ep.ep_group_query(g).live_handles == 0
        h = ep.ep_layout_prefetch(g, topk, x)
        ep.ep_handle_destroy(h)
    finally:
        ep.ep_group_destroy(g)


def test_round_trip_identity_experts(ep, hx):
    """combine(dispatch(x)) with identity experts and renormalised weights returns x
    to within one bf16 ulp; unweighted it returns exactly K * x."""
    w = wl.make_workload("tiny")
    spec = w.spec
    g = _group(ep, spec, spec.T, ep.EP_MODE_HT)
    try:
        x = hx.bits_to_dev(w.x_bits)
        h = ep.ep_layout(g, torch.from_numpy(w.topk_idx).to(hx.DEV))
        recv = torch.zeros((spec.T * spec.K, spec.H), dtype=torch.bfloat16, device=hx.DEV)
        out = torch.zeros((spec.T, spec.H), dtype=torch.bfloat16, device=hx.DEV)
        ep.ep_dispatch(h, x, recv)
        ep.ep_combine(h, recv, out, topk_weights=torch.from_numpy(w.topk_w).to(hx.DEV))
        torch.cuda.synchronize()
        xf = x.float().cpu().numpy()
        of = out.float().cpu().numpy()
        assert np.all(np.abs(of - xf) <= np.abs(xf) * 2.0 ** -7)
        ep.ep_combine(h, recv, out)
        torch.cuda.synchronize()
        assert np.array_equal(out.float().cpu().numpy(), xf * spec.K)
        ep.ep_handle_destroy(h)
    finally:
        ep.ep_group_destroy(g)


def test_ll_windows_as_strided_view_of_receiver_tensor(ep, hx, oracle_mod):
    """LL output [E, C, H] given as this source's sub-regions inside a receiver-shaped
    tensor [E, R*C, H]; nothing outside them may change.  x is a strided view too."""
    w = wl.make_workload("tiny")
    spec = w.spec
    C, my_rank = 6, 1
    lay = oracle_mod.layout(w.topk_idx, E=spec.E, R=spec.R, layout=oracle_mod.LAYOUT_PADDED, C=C, C_rank=spec.T)
    o_full = np.full((spec.E, spec.R * C, spec.H), hx.POISON, np.uint16)
    oracle_mod.dispatch(w.x_bits, None, lay, o_full[:, my_rank * C:(my_rank + 1) * C, :],
                        stride0=spec.R * C * spec.H, stride1=spec.H)
    g = _group(ep, spec, spec.T, ep.EP_MODE_LL, C=C, my_rank=my_rank)
    try:
        xw = hx.poison_bf16((spec.T, spec.H + 24))
        xw[:, 8:8 + spec.H] = hx.bits_to_dev(w.x_bits)
        full = hx.poison_bf16((spec.E, spec.R * C, spec.H))
        h = ep.ep_layout(g, torch.from_numpy(w.topk_idx).to(hx.DEV))
        ep.ep_dispatch(h, xw[:, 8:8 + spec.H], full[:, my_rank * C:(my_rank + 1) * C, :])
        torch.cuda.synchronize()
        assert np.array_equal(hx.dev_to_bits(full), o_full)
        out = hx.poison_bf16((spec.T, spec.H + 8))
        ep.ep_combine(h, full[:, my_rank * C:(my_rank + 1) * C, :], out[:, :spec.H],
                      topk_weights=torch.from_numpy(w.topk_w).to(hx.DEV))
        torch.cuda.synchronize()
        ref = oracle_mod.combine(o_full[:, my_rank * C:(my_rank + 1) * C, :].copy(), w.topk_w, lay, spec.H, acc="f32")
        got = hx.dev_to_bits(out)
        assert np.array_equal(got[:, :spec.H], ref) and np.all(got[:, spec.H:] == hx.POISON)
        ep.ep_handle_destroy(h)
    finally:
        ep.ep_group_destroy(g)


@pytest.mark.parametrize("variant", ["order 1 + read-ahead", "order 1", "order 2", "fp8", "fp8 ahead", "once per rank"])
@pytest.mark.parametrize("mode", ["ht", "ll"])
def test_large_inputs_through_strided_tensors(ep, hx, oracle_mod, mode, variant):
    """The kernels of large inputs (8800 entries: destination-ordered copy, token read-ahead, quantising
    walks, once-per-rank send and fan-out) with every tensor a slice of a wider one: tokens with a row
    pitch larger than H, concatenated windows likewise, padded windows as this source's sub-regions of
    a receiver-shaped [E, R*C, H] tensor.  Everything outside the slices keeps its fill."""
    _say(f"strided large input mode={mode} variant={variant}")
    w = wl.make_workload("skew", T=1100, H=1024)
    spec = w.spec
    T, H, E, R = spec.T, spec.H, spec.E, spec.R
    ll = mode == "ll"
    C, my_rank = 139, 2
    topk = _mess_up(w.topk_idx, E, seed=5, frac_masked=0.01)
    lay = oracle_mod.layout(topk, E=E, R=R, layout=int(ll), C=C if ll else 0, C_rank=T)
    fp8 = variant.startswith("fp8")
    kw = {"order 1 + read-ahead": dict(dispatch_order=1), "order 1": dict(dispatch_order=1), "order 2": dict(dispatch_order=2),
          "fp8": {}, "fp8 ahead": dict(dispatch_order=1, quantize_ahead=1),
          "once per rank": dict(dispatch_path=ep.EP_PATH_RANK_DEDUP)}[variant]
    announce = variant in ("order 1 + read-ahead", "fp8 ahead")
    g = _group(ep, spec, T, ep.EP_MODE_LL if ll else ep.EP_MODE_HT, C=C if ll else 0, my_rank=my_rank, **kw)
    try:
        xw = hx.poison_bf16((T, H + 24))
        xw[:, 8:8 + H] = hx.bits_to_dev(w.x_bits)
        x = xw[:, 8:8 + H]
        d_topk = torch.from_numpy(topk).to(hx.DEV)
        gate = torch.from_numpy(w.topk_w).to(hx.DEV)
        h = ep.ep_layout_prefetch(g, d_topk, x) if announce else ep.ep_layout(g, d_topk)
        elem = torch.uint8 if fp8 else torch.int16
        fill = 0xAB if fp8 else int(np.array(hx.POISON, np.uint16).view(np.int16))
        if ll:  # this source's columns [my_rank*C, (my_rank+1)*C) of every expert of the receiver's tensor
            full = torch.full((E, R * C, H), fill, dtype=elem, device=hx.DEV)
            recv = full[:, my_rank * C:(my_rank + 1) * C, :]
            rows = E * C
        else:
            rows = int(lay.expert_offset[-1])
            full = torch.full((rows + 3, H + 48), fill, dtype=elem, device=hx.DEV)
            recv = full[:rows, :H]
        recv_t = recv.view(torch.float8_e4m3fn) if fp8 else recv.view(torch.bfloat16)
        if fp8:
            G = H // 128
            scales = torch.full((rows, G), -2.0, dtype=torch.float32, device=hx.DEV)
            ep.ep_dispatch(h, x, recv_t, topk_weights=gate, recv_scales=scales)
        else:
            ep.ep_dispatch(h, x, recv_t, topk_weights=gate, topk_idx=d_topk if variant == "once per rank" else None)
        torch.cuda.synchronize()
        got = full.cpu().numpy()
        if fp8:
            o_q = np.full((rows, H), 0xAB, np.uint8)
            o_s = np.full((rows, G), np.float32(-2.0), np.float32)
            oracle_mod.dispatch_fp8(w.x_bits, lay, o_q, o_s)
            assert np.array_equal(scales.cpu().numpy().view(np.uint32), o_s.view(np.uint32))
            want_rows = o_q
        else:
            want_rows = np.full((rows, H), hx.POISON, np.uint16)
            oracle_mod.dispatch(w.x_bits, None, lay, want_rows)
        if ll:
            want = np.full((E, R * C, H), fill, got.dtype)
            want[:, my_rank * C:(my_rank + 1) * C, :] = want_rows.reshape(E, C, H).view(got.dtype)
        else:
            want = np.full((rows + 3, H + 48), fill, got.dtype)
            want[:rows, :H] = want_rows.view(got.dtype)
        assert np.array_equal(got, want), "rows differ, or something outside the windows was written"
        assert np.all(hx.dev_to_bits(xw.view(torch.bfloat16))[:, :8] == hx.POISON)  # the tokens' surroundings are only read
        ep.ep_handle_destroy(h)
    finally:
        ep.ep_group_destroy(g)


def test_handle_reuse_forward_and_backward(ep, hx, oracle_mod):
    """One handle serves several dispatch/combine pairs (Sec. III-C: shared between the
    forward and backward passes)."""
    w = wl.make_workload("ll_decode", T=64, H=512)
    spec = w.spec
    lay = oracle_mod.layout(w.topk_idx, E=spec.E, R=spec.R, C_rank=spec.T)
    g = _group(ep, spec, spec.T, ep.EP_MODE_HT)
    try:
        h = ep.ep_layout(g, torch.from_numpy(w.topk_idx).to(hx.DEV))
        d_w = torch.from_numpy(w.topk_w).to(hx.DEV)
        for it in range(3):
            xb = wl.make_tokens(spec, seed_offset=it)
            recv = torch.zeros((spec.T * spec.K, spec.H), dtype=torch.bfloat16, device=hx.DEV)
            out = torch.zeros((spec.T, spec.H), dtype=torch.bfloat16, device=hx.DEV)
            ep.ep_dispatch(h, hx.bits_to_dev(xb), recv)
            ep.ep_combine(h, recv, out, topk_weights=d_w)
            torch.cuda.synchronize()
            o_recv = np.zeros((spec.T * spec.K, spec.H), np.uint16)
            oracle_mod.dispatch(xb, None, lay, o_recv)
            assert np.array_equal(hx.dev_to_bits(recv), o_recv)
            assert np.array_equal(hx.dev_to_bits(out), oracle_mod.combine(o_recv, w.topk_w, lay, spec.H, acc="f32"))
        ep.ep_handle_destroy(h)
    finally:
        ep.ep_group_destroy(g)


def test_output_too_small_is_flagged_not_overrun(ep, hx, oracle_mod):
    w = wl.make_workload("ll_decode", T=32, H=256)
    spec = w.spec
    lay = oracle_mod.layout(w.topk_idx, E=spec.E, R=spec.R, C_rank=spec.T)
    cap = 100
    g = _group(ep, spec, spec.T, ep.EP_MODE_HT)
    try:
        h = ep.ep_layout(g, torch.from_numpy(w.topk_idx).to(hx.DEV))
        store = hx.poison_bf16((spec.T * spec.K, spec.H))
        ep.ep_dispatch(h, hx.bits_to_dev(w.x_bits), store[:cap])
        info = ep.ep_handle_query(h, ok=(ep.EP_ERR_OVERFLOW,))
        assert info.last_code == ep.EP_ERR_OVERFLOW and info.status & ep.STATUS_OUTPUT_OVERFLOW
        got = hx.dev_to_bits(store)
        assert np.all(got[cap:] == hx.POISON)
        o = np.full((spec.T * spec.K, spec.H), hx.POISON, np.uint16)
        oracle_mod.dispatch(w.x_bits, None, lay, o)
        assert np.array_equal(got[:cap], o[:cap])
        ep.ep_handle_destroy(h)
    finally:
        ep.ep_group_destroy(g)


def test_slab_reuse_on_another_stream_waits_for_the_previous_handle(ep, hx, oracle_mod):
    """A handle is destroyed while its dispatches and combines are still queued on stream A; the
    next layout, on stream B, takes the same slab (the group has one) with another routing.  It
    must not overwrite the arrays the queued work reads: every result of stream A is the oracle's."""
    w = wl.make_workload("ht_prefill", T=2048, H=2048)
    spec = w.spec
    T = spec.T
    lay = oracle_mod.layout(w.topk_idx, E=spec.E, R=spec.R, C_rank=T)
    rows = int(lay.expert_offset[-1])
    o_recv = np.zeros((rows, spec.H), np.uint16)
    oracle_mod.dispatch(w.x_bits, None, lay, o_recv)
    ref = oracle_mod.combine(o_recv, w.topk_w, lay, spec.H, acc="f32")
    topk2, _, _ = wl.make_routing(spec, T=T, seed_offset=99)
    lay2 = oracle_mod.layout(topk2, E=spec.E, R=spec.R, C_rank=T)
    g = _group(ep, spec, T, ep.EP_MODE_HT, max_handles=1)
    try:
        x = hx.bits_to_dev(w.x_bits)
        gate = torch.from_numpy(w.topk_w).to(hx.DEV)
        d_topk = torch.from_numpy(w.topk_idx).to(hx.DEV)
        d_topk2 = torch.from_numpy(topk2).to(hx.DEV)
        sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        for rep in range(3):
            recv = hx.poison_bf16((rows, spec.H))
            outs = [hx.poison_bf16((T, spec.H)) for _ in range(12)]
            torch.cuda.synchronize()
            h = ep.ep_layout(g, d_topk, stream=sa)
            for o in outs:  # a queue of work that reads the handle's arrays
                ep.ep_dispatch(h, x, recv, stream=sa)
                ep.ep_combine(h, recv, o, topk_weights=gate, stream=sa)
            ep.ep_handle_destroy(h)
            h2 = ep.ep_layout(g, d_topk2, stream=sb)  # same slab, other stream, other routing
            got2 = hx.fetch_layout(h2, T, spec.K, spec.E, spec.R)
            hx.assert_layout_equal(got2, lay2)
            torch.cuda.synchronize()
            assert np.array_equal(hx.dev_to_bits(recv), o_recv), f"round {rep}: rows differ"
            for i, o in enumerate(outs):
                assert np.array_equal(hx.dev_to_bits(o), ref), f"round {rep}: combine {i} differs"
            ep.ep_handle_destroy(h2)
    finally:
        ep.ep_group_destroy(g)


def test_overflow_status_stays_set_for_the_handle(ep, hx, oracle_mod):
    """Status bit 2 (rows beyond the output) is sticky: once a dispatch has raised it, queries of
    that handle keep reporting it, also after a dispatch into a tensor that is large enough; a new
    handle starts clean."""
    w = wl.make_workload("ll_decode", T=90, H=256)
    spec = w.spec
    g = _group(ep, spec, 90, ep.EP_MODE_HT)
    try:
        topk = torch.from_numpy(w.topk_idx).to(hx.DEV)
        x = hx.bits_to_dev(w.x_bits)
        rows = 90 * spec.K
        h = ep.ep_layout(g, topk)
        ep.ep_dispatch(h, x, hx.poison_bf16((rows - 10, spec.H)))
        assert ep.ep_handle_query(h, ok=(ep.EP_ERR_OVERFLOW,)).status & ep.STATUS_OUTPUT_OVERFLOW
        ep.ep_dispatch(h, x, hx.poison_bf16((rows, spec.H)))
        assert ep.ep_handle_query(h, ok=(ep.EP_ERR_OVERFLOW,)).status & ep.STATUS_OUTPUT_OVERFLOW
        ep.ep_handle_destroy(h)
        h = ep.ep_layout(g, topk)
        ep.ep_dispatch(h, x, hx.poison_bf16((rows, spec.H)))
        assert ep.ep_handle_query(h).status == 0
        ep.ep_handle_destroy(h)
    finally:
        ep.ep_group_destroy(g)


def test_allocator_callbacks_and_lifecycle(ep, hx):
    spec = wl.SPECS["tiny"]
    held = {}

    def alloc(pp, nbytes):
        t = torch.empty(int(nbytes), dtype=torch.uint8, device=hx.DEV)
        held[t.data_ptr()] = t
        pp[0] = t.data_ptr()
        return 0

    def free(p):
        return 0 if held.pop(p, None) is not None else 1

    a, f = ep.ALLOC_FN(alloc), ep.FREE_FN(free)
    cfg = ep.make_config(spec.R, spec.E, spec.H, spec.K, spec.T, max_handles=1)
    g = ep.ep_group_create(cfg, alloc_fn=a, free_fn=f)
    assert len(held) == 1
    topk = torch.from_numpy(wl.make_routing(spec)[0]).to(hx.DEV)
    h1 = ep.ep_layout(g, topk)
    h2 = ep.ep_layout(g, topk)  # pool exhausted: one more slab through the callback
    assert len(held) == 2 and ep.ep_group_query(g).live_handles == 2
    with pytest.raises(ep.EpError) as e:
        ep.ep_group_destroy(g)
    assert e.value.code == ep.EP_ERR_BUSY
    a1 = hx.fetch_layout(h1, spec.T, spec.K, spec.E, spec.R).arrays
    a2 = hx.fetch_layout(h2, spec.T, spec.K, spec.E, spec.R).arrays
    assert all(np.array_equal(a1[k], a2[k]) for k in a1)
    ep.ep_handle_destroy(h1)
    ep.ep_handle_destroy(h2)
    ep.ep_group_destroy(g)
    assert not held


@pytest.mark.parametrize("nbytes", [16, 4096 + 16, (3 << 20) + 48, 17 * 4096 * 16 + 16 * 1023])
def test_measurement_kernels(ep, hx, nbytes):
    """The copy, fill and read kernels the bandwidth figures are measured against: the copy moves
    exactly the bytes given, the fill writes bf16 1.0 to exactly those bytes, the read leaves its
    source alone; ragged sizes span whole trips and a tail."""
    _say(f"measurement kernels nbytes={nbytes}")
    g = torch.Generator().manual_seed(nbytes)
    host = torch.randint(0, 256, (nbytes + 64,), dtype=torch.uint8, generator=g)
    src = host.to(hx.DEV)
    dst = torch.full((nbytes + 64,), 7, dtype=torch.uint8, device=hx.DEV)
    ep.ep_calibration_copy(dst[:nbytes], src[:nbytes])
    torch.cuda.synchronize()
    got = dst.cpu()
    assert torch.equal(got[:nbytes], host[:nbytes]) and bool((got[nbytes:] == 7).all())
    ep.ep_calibration_fill(dst[:nbytes])
    torch.cuda.synchronize()
    got = dst.cpu()
    assert bool((got[:nbytes].view(torch.int16) == 0x3F80).all()) and bool((got[nbytes:] == 7).all())
    sink = torch.zeros(1, dtype=torch.int32, device=hx.DEV)
    ep.ep_calibration_read(src[:nbytes], sink)
    torch.cuda.synchronize()
    assert torch.equal(src.cpu(), host)
    for bad in (8, 24):
        with pytest.raises(ep.EpError):
            ep.ep_calibration_fill(dst[:bad])
        with pytest.raises(ep.EpError):
            ep.ep_calibration_read(src[:bad], sink)


def test_argument_errors_on_device(ep, hx):
    spec = wl.SPECS["tiny"]
    g = _group(ep, spec, spec.T, ep.EP_MODE_HT)
    try:
        topk = torch.from_numpy(wl.make_routing(spec)[0]).to(hx.DEV)
        for bad in (topk[:, :1], torch.zeros((spec.T + 1, spec.K), dtype=torch.int32, device=hx.DEV),
                    topk.float()):
            with pytest.raises((ep.EpError, KeyError)) as e:
                ep.ep_layout(g, bad)
        h = ep.ep_layout(g, topk)
        x = torch.zeros((spec.T, spec.H), dtype=torch.bfloat16, device=hx.DEV)
        recv = torch.zeros((spec.T * spec.K, spec.H), dtype=torch.bfloat16, device=hx.DEV)
        for args in ((x[:-1], recv), (x, recv[:, :-8]), (x.float(), recv), (x, recv.view(-1)[1:-(spec.H - 1)].view(-1, spec.H))):
            with pytest.raises(ep.EpError) as e:
                ep.ep_dispatch(h, *args)
            assert e.value.code == ep.EP_ERR_INVALID_ARG
        with pytest.raises(ep.EpError) as e:
            ep.ep_dispatch(h, x, recv, send_only=1)
        assert e.value.code == ep.EP_ERR_UNSUPPORTED
        with pytest.raises(ep.EpError) as e:
            ep.ep_combine(h, recv, x[:, :-8])
        assert e.value.code == ep.EP_ERR_INVALID_ARG
        ep.ep_handle_destroy(h)
    finally:
        ep.ep_group_destroy(g)


# ------------------------------------------------------------------------------ once per destination rank

DEDUP_CASES = [
    # name, T, H, mode, C, weights
    ("tiny", None, None, "ht", 0, True),
    ("tiny", None, None, "ll", 6, True),
    ("ll_decode", None, 512, "ll", 0, True),
    ("ll_decode", 100, None, "ll", 5, False),
    ("skew", 700, 1000, "ht", 0, True),
    ("skew_rank0", 900, 256, "ll", 60, True),
    ("stress_hot", 600, 128, "ht", 0, True),
    ("ht_prefill", None, None, "ht", 0, True),   # full benchmark shape
    ("stress_hot", None, 256, "ht", 0, True),    # 8192 tokens: hot ranks' windows take several passes per wave
    (("ll_decode", dict(R=1, E=64, K=4)), 300, 128, "ht", 0, True),   # one window, 64 local experts
    (("ll_decode", dict(R=4, E=24, K=3)), 333, 64, "ll", 50, True),   # K and L not powers of two, drops
    (("ll_decode", dict(R=8, E=1024, K=16)), 200, 64, "ht", 0, False),  # 128 local experts, 16 ids per header
    (("tiny", dict(dup=True)), 64, None, "ht", 0, True),              # a token naming one expert twice
    (("skew", dict(K=17)), 300, 520, "ht", 0, True),                   # headers of 17, 33 and 64 ids (up to 528 bytes)
    (("skew", dict(K=33)), 200, 256, "ll", 80, True),
    (("skew", dict(K=64)), 130, 1000, "ht", 0, False),
    # degenerate routings: nothing routed; one window takes every message; K rows of one message in one expert
    (("skew", dict(reroute="all_masked")), 300, 256, "ht", 0, True),
    (("skew", dict(reroute="one_expert")), 600, 256, "ht", 0, True),
    (("skew", dict(reroute="same_experts")), 600, 256, "ll", 100, True),
    (("skew", dict(reroute="k_times_one_expert")), 600, 256, "ht", 0, True),
    (("skew", dict(reroute="last_expert_only")), 600, 256, "ll", 700, False),
]


@pytest.mark.parametrize("name,T,H,mode,C,weights", DEDUP_CASES)
def test_once_per_rank_dispatch_parity(ep, hx, oracle_mod, name, T, H, mode, C, weights):
    """Staging windows byte-for-byte equal to the oracle's messages; final windows equal to
    the oracle's direct dispatch (and to its own fan-out)."""
    over = {}
    if isinstance(name, tuple):
        name, over = name[0], dict(name[1])
    dup = over.pop("dup", False)
    reroute = over.pop("reroute", None)
    w = wl.make_workload(name, T=T, **({"H": H} if H else {}), **over)
    spec = w.spec
    T = spec.T
    _say(f"once-per-rank case {name} {over} {reroute} T={T} H={spec.H} mode={mode} C={C}")
    topk = _mess_up(w.topk_idx, spec.E, seed=T, frac_masked=0.02)
    if reroute:
        topk = np.ascontiguousarray(globals()["_" + reroute](topk, spec).astype(np.int32))
    if dup:
        topk[::3, 1] = topk[::3, 0]  # duplicates: each occurrence gets its own row
    ll = mode == "ll"
    Cc = (C if C else T) if ll else 0
    lay = oracle_mod.layout(topk, E=spec.E, R=spec.R, layout=int(ll), C=Cc, C_rank=T)
    rows = spec.E * Cc if ll else int(lay.expert_offset[-1])
    n_slots = spec.R * T if ll else T * min(spec.R, spec.K)
    wts = w.topk_w if weights else None
    o_win = oracle_mod.dedup_send(w.x_bits, topk, wts, lay, n_slots)
    o_recv = np.full((rows + 1, spec.H), hx.POISON, np.uint16)
    o_w = np.full(rows + 1, np.float32(-3.5), np.float32)
    o_src = np.full(rows + 1, -9, np.int32)
    oracle_mod.dispatch(w.x_bits, wts, lay, o_recv, o_w, o_src)
    if not weights:
        o_w[:rows][o_src[:rows] >= 0] = 1.0  # the header carries 1.0 when no weights are given
    v_recv = np.full((rows + 1, spec.H), hx.POISON, np.uint16)
    v_w = np.full(rows + 1, np.float32(-3.5), np.float32)
    v_src = np.full(rows + 1, -9, np.int32)
    o_cnt, o_drop = oracle_mod.dedup_recv(o_win, lay, spec.H, v_recv, v_w, v_src)
    assert np.array_equal(v_recv, o_recv) and np.array_equal(v_src, o_src) and np.array_equal(v_w, o_w)

    held = {}

    def alloc(pp, nbytes):
        t = torch.full((int(nbytes),), 0xA5, dtype=torch.uint8, device=hx.DEV)
        held[t.data_ptr()] = t
        pp[0] = t.data_ptr()
        return 0

    def free(p):
        return 0 if held.pop(p, None) is not None else 1

    a_fn, f_fn = ep.ALLOC_FN(alloc), ep.FREE_FN(free)
    cfg = ep.make_config(spec.R, spec.E, spec.H, spec.K, T, mode=ep.EP_MODE_LL if ll else ep.EP_MODE_HT,
                         slots_per_subregion=C, dispatch_path=ep.EP_PATH_RANK_DEDUP)
    g = ep.ep_group_create(cfg, alloc_fn=a_fn, free_fn=f_fn)
    try:
        ginfo = ep.ep_group_query(g)
        assert ginfo.staging_slots == n_slots and ginfo.msg_bytes == o_win.shape[1]
        assert ginfo.msg_header_bytes == oracle_mod.msg_header_bytes(spec.K)
        staging = held[ginfo.staging]
        d_topk = torch.from_numpy(topk).to(hx.DEV)
        h = ep.ep_layout(g, d_topk)
        store = hx.poison_bf16((rows + 1, spec.H))
        recv = store[:rows].view(spec.E, Cc, spec.H) if ll else store[:rows]
        r_w = torch.full((rows + 1,), -3.5, dtype=torch.float32, device=hx.DEV)
        r_src = torch.full((rows + 1,), -9, dtype=torch.int32, device=hx.DEV)
        r_cnt = torch.full((spec.E,), -1, dtype=torch.int32, device=hx.DEV)
        ep.ep_dispatch(h, hx.bits_to_dev(w.x_bits), recv, topk_weights=torch.from_numpy(w.topk_w).to(hx.DEV) if weights else None,
                       recv_w=r_w[:rows], recv_src=r_src[:rows], recv_count=r_cnt, topk_idx=d_topk)
        torch.cuda.synchronize()
        stride, lead = int(ginfo.msg_stride), int(ginfo.msg_lead)
        assert stride % 256 == 0 and (lead + ginfo.msg_header_bytes) % 256 == 0 and lead + ginfo.msg_bytes <= stride
        slots = staging[: n_slots * stride].cpu().numpy().reshape(n_slots, stride)
        assert np.array_equal(slots[:, lead:lead + ginfo.msg_bytes], o_win), "staging windows differ from the oracle's messages"
        assert np.all(slots[:, :lead] == 0xA5) and np.all(slots[:, lead + ginfo.msg_bytes:] == 0xA5), "slot padding was written"
        assert np.array_equal(hx.dev_to_bits(store), o_recv), "fanned-out rows differ"
        assert np.array_equal(r_src.cpu().numpy(), o_src)
        assert np.array_equal(r_w.cpu().numpy(), o_w)
        assert np.array_equal(r_cnt.cpu().numpy(), lay.expert_kept) and np.array_equal(o_cnt, lay.expert_kept)
        info = ep.ep_handle_query(h)
        assert int(info.rank_messages) == lay.n_msgs
        # the direct-path dispatch of another group must give the same windows
        ep.ep_handle_destroy(h)
        with pytest.raises(ep.EpError):
            h2 = ep.ep_layout(g, d_topk)
            try:
                ep.ep_dispatch(h2, hx.bits_to_dev(w.x_bits), recv)  # TOPK_IDX is required on this path
            finally:
                ep.ep_handle_destroy(h2)
    finally:
        ep.ep_group_destroy(g)
    assert not held


# ------------------------------------------------------------------------------ quantising dispatch (FP8 + scales)

FP8_CASES = [
    # name, T, H, mode, C, wide dynamic range, dispatch order of the group
    ("tiny", None, None, "ht", 0, False, 0),
    ("tiny", None, 384, "ll", 6, True, 0),
    ("ll_decode", None, None, "ll", 0, False, 0),
    ("ll_decode", 90, 1152, "ht", 0, True, 0),     # ragged last 1024-channel segment
    ("skew", 500, None, "ht", 0, True, 0),
    ("ht_prefill", None, None, "ht", 0, False, 0),  # full benchmark shape
    # groups set to the order of the destination rows (the quantising dispatch walks the tokens all the same)
    ("ht_prefill", 4095, None, "ht", 0, True, 2),   # ragged, wide range and special values
    ("skew", None, None, "ht", 0, True, 1),         # hot experts
    ("ll_decode", 1100, 1024, "ht", 0, True, 2),
    ("skew", None, None, "ll", 512, True, 1),       # padded windows, capacity drops
    # groups that quantise ahead: the layout call quantises the announced tokens into a staging copy
    # and the dispatch copies staged rows in destination order
    ("ht_prefill", None, None, "ht", 0, True, "ahead"),    # full benchmark shape
    ("ht_prefill", 4095, None, "ht", 0, True, "ahead"),    # ragged
    ("skew", None, None, "ll", 512, True, "ahead"),        # padded windows, capacity drops
    ("ll_decode", 1100, 1152, "ht", 0, True, "ahead"),     # 36 bytes of scales per row: a part-filled last unit
    ("ll_decode", 1100, 128, "ll", 60, True, "ahead"),     # one group per row
    ("ll_decode", 90, 1152, "ht", 0, True, "ahead"),       # too small for the destination order: token walk
    ("stress_hot", None, None, "ht", 0, False, "ahead"),   # 117 MB of tokens, more than one read-ahead covers
    (("skew", dict(K=33)), 300, 512, "ht", 0, True, "ahead"),
]


@pytest.mark.parametrize("name,T,H,mode,C,wide,order", FP8_CASES)
def test_fp8_dispatch_parity(ep, hx, oracle_mod, name, T, H, mode, C, wide, order):
    """E4M3 codes and float scales bit-exact with the oracle (special values included: NaN, infinities,
    subnormal groups whose 448 / amax overflows); untouched rows keep their fill."""
    over = {}
    if isinstance(name, tuple):
        name, over = name[0], dict(name[1])
    w = wl.make_workload(name, T=T, **({"H": H} if H else {}), **over)
    spec = w.spec
    T = spec.T
    _say(f"fp8 case {name} T={T} H={spec.H} mode={mode} C={C} wide={wide} order={order}")
    ahead = order == "ahead"
    x_bits = w.x_bits.copy()
    if wide:  # spread magnitudes over 2^-24 .. 2^12, plus zero groups, signed zeros and special values
        rng = np.random.default_rng(T)
        xf = wl.bf16_bits_to_f32(x_bits) * np.exp2(rng.integers(-24, 13, x_bits.shape)).astype(np.float32)
        x_bits = wl.f32_to_bf16_bits(xf)
        x_bits[0, :128] = 0
        x_bits[1 % T, 128:256] = 0x8000
        x_bits[2 % T, 5] = 0x7F7F  # largest finite bf16
        if T > 8 and spec.H >= 384:
            x_bits[3, 130] = 0x7FC0       # NaN in a group of ordinary values
            x_bits[4, 131] = 0xFFC1       # a negative NaN
            x_bits[5, 7] = 0x7F80         # +infinity: the scale is infinite, every other code of the group 0
            x_bits[6, 300] = 0xFF80       # -infinity
            x_bits[7, 256:384] = rng.integers(0, 4, 128).astype(np.uint16) | (rng.integers(0, 2, 128).astype(np.uint16) << 15)
            x_bits[7, 257] = 0x0003       # a group of bf16 subnormals: 448 / amax overflows
    topk = _mess_up(w.topk_idx, spec.E, seed=T + 3, frac_masked=0.01)
    ll = mode == "ll"
    Cc = (C if C else T) if ll else 0
    lay = oracle_mod.layout(topk, E=spec.E, R=spec.R, layout=int(ll), C=Cc, C_rank=T)
    rows = spec.E * Cc if ll else int(lay.expert_offset[-1])
    G = spec.H // 128
    o_q = np.full((rows + 1, spec.H), 0xAB, np.uint8)
    o_s = np.full((rows + 1, G), np.float32(-2.0), np.float32)
    oracle_mod.dispatch_fp8(x_bits, lay, o_q, o_s)
    g = _group(ep, spec, T, ep.EP_MODE_LL if ll else ep.EP_MODE_HT, C=C, dispatch_order=1 if ahead else order,
               quantize_ahead=int(ahead))
    try:
        d_x = hx.bits_to_dev(x_bits)
        d_topk = torch.from_numpy(topk).to(hx.DEV)
        h = ep.ep_layout_prefetch(g, d_topk, d_x) if ahead else ep.ep_layout(g, d_topk)
        store = torch.full((rows + 1, spec.H), 0xAB, dtype=torch.uint8, device=hx.DEV)
        recv = store[:rows].view(torch.float8_e4m3fn)
        recv = recv.view(spec.E, Cc, spec.H) if ll else recv
        scales = torch.full((rows + 1, G), -2.0, dtype=torch.float32, device=hx.DEV)
        r_src = torch.full((rows + 1,), -9, dtype=torch.int32, device=hx.DEV)
        r_cnt = torch.full((spec.E,), -1, dtype=torch.int32, device=hx.DEV)
        r_w = torch.full((rows + 1,), -3.5, dtype=torch.float32, device=hx.DEV)
        d_w = torch.from_numpy(w.topk_w).to(hx.DEV)
        # twice on the same handle: a staging copy made by the layout call serves the first dispatch only
        for again in range(2 if ahead else 1):
            if again:
                store.fill_(0xAB); scales.fill_(-2.0); r_src.fill_(-9); r_cnt.fill_(-1); r_w.fill_(-3.5)
            ep.ep_dispatch(h, d_x, recv, topk_weights=d_w, recv_w=r_w[:rows], recv_scales=scales[:rows],
                           recv_src=r_src[:rows], recv_count=r_cnt)
            torch.cuda.synchronize()
            got_q = store.cpu().numpy()
            got_s = scales.cpu().numpy()
            assert np.array_equal(got_s.view(np.uint32), o_s.view(np.uint32)), "scales differ"
            assert np.array_equal(got_q, o_q), "E4M3 codes differ"
            assert np.array_equal(r_cnt.cpu().numpy(), lay.expert_kept)
            valid = lay.dst_row >= 0
            want_w = np.full(rows + 1, np.float32(-3.5), np.float32)
            want_w[lay.dst_row[valid]] = w.topk_w[valid]
            want_src = np.full(rows + 1, -9, np.int32)
            want_src[lay.dst_row[valid]] = np.nonzero(valid)[0]
            assert np.array_equal(r_w.cpu().numpy(), want_w) and np.array_equal(r_src.cpu().numpy(), want_src)
        src = r_src.cpu().numpy()
        for t in range(0, T, max(1, T // 16)):
            for k in range(spec.K):
                if lay.dst_row[t, k] >= 0:
                    assert src[lay.dst_row[t, k]] == t
        # FP8 output without scales (or the reverse) is refused
        with pytest.raises(ep.EpError) as e:
            ep.ep_dispatch(h, d_x, recv)
        assert e.value.code == ep.EP_ERR_INVALID_ARG
        ep.ep_handle_destroy(h)
    finally:
        ep.ep_group_destroy(g)


# ------------------------------------------------------------------------------ HIP graph capture


@pytest.mark.parametrize("T,order", [(96, 0), (1100, 1), (96, "one call")])
def test_graph_capture_and_replay(ep, hx, oracle_mod, T, order):
    """layout + dispatch + combine captured once into a HIP graph and replayed with new
    token data each time; every replay must equal the eager result and the oracle.  The
    library records no memset nodes (it never calls one) and allocates nothing while a
    slab is free in the group's pool, so the three calls are capturable as they are.  The
    second case captures the read-ahead layout call and the destination-ordered dispatch, the
    third the one-launch layout + dispatch of a small input."""
    fused = order == "one call"
    order = 0 if fused else order
    w = wl.make_workload("ll_decode", T=T, H=1024)
    spec = w.spec
    lay = oracle_mod.layout(w.topk_idx, E=spec.E, R=spec.R, C_rank=spec.T)
    rows = int(lay.expert_offset[-1])
    g = _group(ep, spec, spec.T, ep.EP_MODE_HT, max_handles=2, dispatch_order=order)
    try:
        topk = torch.from_numpy(w.topk_idx).to(hx.DEV)
        gate = torch.from_numpy(w.topk_w).to(hx.DEV)
        x = hx.bits_to_dev(w.x_bits)
        recv = torch.zeros((rows, spec.H), dtype=torch.bfloat16, device=hx.DEV)
        out = torch.zeros((spec.T, spec.H), dtype=torch.bfloat16, device=hx.DEV)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):  # warm-up outside capture
            h0 = ep.ep_layout(g, topk)
            ep.ep_dispatch(h0, x, recv, topk_weights=gate)
            ep.ep_combine(h0, recv, out, topk_weights=gate)
        side.synchronize()
        ep.ep_handle_destroy(h0)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            if fused:
                h = ep.ep_layout_dispatch(g, topk, x, recv, topk_weights=gate)
            else:
                h = ep.ep_layout_prefetch(g, topk, x) if order else ep.ep_layout(g, topk)
                ep.ep_dispatch(h, x, recv, topk_weights=gate)
            ep.ep_combine(h, recv, out, topk_weights=gate)
        for it in range(4):
            xb = wl.make_tokens(spec, seed_offset=50 + it)
            x.copy_(hx.bits_to_dev(xb))          # eager work between the replays
            recv.zero_()
            out.zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            o_recv = np.zeros((rows, spec.H), np.uint16)
            oracle_mod.dispatch(xb, None, lay, o_recv)
            assert np.array_equal(hx.dev_to_bits(recv), o_recv), f"replay {it}: dispatched rows differ"
            ref = oracle_mod.combine(o_recv, w.topk_w, lay, spec.H, acc="f32")
            assert np.array_equal(hx.dev_to_bits(out), ref), f"replay {it}: combine differs"
            # the same step run eagerly gives the same bits
            out2 = torch.zeros_like(out)
            recv2 = torch.zeros_like(recv)
            h2 = ep.ep_layout(g, topk)
            ep.ep_dispatch(h2, x, recv2, topk_weights=gate)
            ep.ep_combine(h2, recv2, out2, topk_weights=gate)
            torch.cuda.synchronize()
            ep.ep_handle_destroy(h2)
            assert torch.equal(out2.view(torch.int16), out.view(torch.int16))
        del graph
        ep.ep_handle_destroy(h)
    finally:
        ep.ep_group_destroy(g)


# ------------------------------------------------------------------------------ two-level combine order


@pytest.mark.parametrize("name,T,H,rpn,mode", [("ll_decode", None, 512, 8, "ht"), ("ll_decode", 77, 1000, 4, "ll"),
                                               ("stress_hot", 300, 256, 8, "ht"), ("skew", 200, 512, 2, "ht"),
                                               ("ht_prefill", None, None, 8, "ht"),
                                               # 16 and 6 nodes, 17 to 64 entries per token
                                               (("skew", dict(K=17)), 300, 520, 1, "ht"),
                                               (("skew", dict(K=33)), 200, 256, 3, "ll"),
                                               (("skew", dict(K=64)), 130, 1000, 1, "ht")])
def test_combine_two_level_order(ep, hx, oracle_mod, name, T, H, rpn, mode):
    """Sum per node of rpn ranks first, then across nodes: bit-exact with the oracle's
    two-level float32 order, within one bf16 ulp of the flat order and of the float64 sum."""
    over = {}
    if isinstance(name, tuple):
        name, over = name[0], dict(name[1])
    w = wl.make_workload(name, T=T, **({"H": H} if H else {}), **over)
    spec = w.spec
    T = spec.T
    _say(f"two-level combine {name} T={T} H={spec.H} ranks_per_node={rpn} mode={mode}")
    topk = _mess_up(w.topk_idx, spec.E, seed=T, frac_masked=0.02)
    ll = mode == "ll"
    Cc = T if ll else 0
    lay = oracle_mod.layout(topk, E=spec.E, R=spec.R, layout=int(ll), C=Cc, C_rank=T)
    rows = spec.E * Cc if ll else int(lay.expert_offset[-1])
    y_bits = wl.f32_to_bf16_bits(np.random.default_rng(T).standard_normal((rows, spec.H)).astype(np.float32) * 2)
    ref = oracle_mod.combine_hier(y_bits, w.topk_w, lay, topk, spec.H, ranks_per_node=rpn)
    cfg = ep.make_config(spec.R, spec.E, spec.H, spec.K, T, mode=ep.EP_MODE_LL if ll else ep.EP_MODE_HT,
                         ranks_per_node=rpn, staged_buffers=1 if T <= 300 else 0)
    g = ep.ep_group_create(cfg)
    try:
        h = ep.ep_layout(g, torch.from_numpy(topk).to(hx.DEV))
        y = hx.bits_to_dev(y_bits)
        y = y.view(spec.E, Cc, spec.H) if ll else y
        gate = torch.from_numpy(w.topk_w).to(hx.DEV)
        out = hx.poison_bf16((T, spec.H))
        ep.ep_combine(h, y, out, topk_weights=gate)
        torch.cuda.synchronize()
        got = hx.dev_to_bits(out)
        assert np.array_equal(got, ref), "differs from the two-level float32 order"
        if T <= 300:
            # another association of the same float32 sum: equal or adjacent bf16 values, except
            # where the terms cancel -- there the difference is bounded by the float32 rounding
            # of the terms, (K + 1) * 2^-24 * sum_k |w_k y_k|
            yf = wl.bf16_bits_to_f32(y_bits)
            rows_k = np.clip(lay.dst_row, 0, None)
            terms = np.abs(w.topk_w)[:, :, None] * np.abs(yf[rows_k]) * (lay.dst_row >= 0)[:, :, None]
            bound = terms.sum(1) * (spec.K + 1) * 2.0 ** -24
            for other in (oracle_mod.combine(y_bits, w.topk_w, lay, spec.H, acc="f32"),
                          oracle_mod.combine(y_bits, w.topk_w, lay, spec.H, acc="f64")):
                near = hx.bf16_ulp_distance(got, other) <= 1
                diff = np.abs(wl.bf16_bits_to_f32(got).astype(np.float64) - wl.bf16_bits_to_f32(other))
                assert np.all(near | (diff <= 2 * bound + 1e-30))
            out2 = hx.poison_bf16((T, spec.H))   # the staged combine uses the same order
            ep.ep_combine(h, y, out2, topk_weights=gate, send_only=1)
            ep.ep_complete(h)
            torch.cuda.synchronize()
            assert np.array_equal(hx.dev_to_bits(out2), ref)
            ep.ep_combine(h, y, out2)            # unweighted
            torch.cuda.synchronize()
            assert np.array_equal(hx.dev_to_bits(out2), oracle_mod.combine_hier(y_bits, None, lay, topk, spec.H, rpn))
        ep.ep_handle_destroy(h)
    finally:
        ep.ep_group_destroy(g)


# ------------------------------------------------------------------------------ randomised shapes


def test_random_shapes_end_to_end(ep, hx, oracle_mod):
    """Forty seeded random configurations (E, R, K, T, H, mode, capacity, masked fraction):
    layout, dispatch and combine against the oracle in each."""
    rng = np.random.default_rng(2024)
    for case in range(40):
        R = int(rng.choice([1, 2, 3, 4, 8, 16, 32, 64]))
        L = int(rng.choice([1, 2, 3, 4, 8, 13]))
        E = R * L
        if E > 1024:
            continue
        K = int(rng.integers(1, min(E, 12) + 1))
        T = int(rng.choice([1, 2, 7, 63, 64, 65, 127, 129, 500, 513, 1000, 2049]))
        H = int(rng.choice([8, 64, 200, 512, 520, 1024, 1536]))
        ll = bool(rng.integers(0, 2))
        C = int(rng.integers(1, max(2, (3 * T * K) // (2 * E) + 2))) if ll else 0
        spec = wl.WorkloadSpec(f"rand{case}", 40 + case, R=R, T=T, H=H, E=E, K=K)
        w = wl.make_workload(spec)
        topk = _mess_up(w.topk_idx, E, seed=case, frac_masked=float(rng.choice([0.0, 0.05, 0.5])),
                        n_invalid=int(rng.integers(0, 3)))
        _say(f"random case {case}: E={E} R={R} K={K} T={T} H={H} ll={ll} C={C}")
        lay = oracle_mod.layout(topk, E=E, R=R, layout=int(ll), C=C if ll else 0, C_rank=T)
        rows = E * C if ll else int(lay.expert_offset[-1])
        o_recv = np.full((rows + 1, H), hx.POISON, np.uint16)
        oracle_mod.dispatch(w.x_bits, None, lay, o_recv)
        g = _group(ep, spec, T, ep.EP_MODE_LL if ll else ep.EP_MODE_HT, C=C)
        try:
            h = ep.ep_layout(g, torch.from_numpy(topk).to(hx.DEV))
            ok_codes = (ep.EP_SUCCESS, ep.EP_ERR_INVALID_ROUTING)
            got = hx.fetch_layout(h, T, K, E, R, ok=ok_codes)
            hx.assert_layout_equal(got, lay)
            store = hx.poison_bf16((rows + 1, H))
            recv = store[:rows].view(E, C, H) if ll else store[:rows]
            ep.ep_dispatch(h, hx.bits_to_dev(w.x_bits), recv)
            out = hx.poison_bf16((T, H))
            gate = torch.from_numpy(w.topk_w).to(hx.DEV)
            ep.ep_combine(h, recv, out, topk_weights=gate)
            torch.cuda.synchronize()
            assert np.array_equal(hx.dev_to_bits(store), o_recv), f"case {case}: rows differ"
            ref = oracle_mod.combine(o_recv[:rows], w.topk_w, lay, H, acc="f32")
            assert np.array_equal(hx.dev_to_bits(out), ref), f"case {case}: combine differs"
            ep.ep_handle_destroy(h)
        finally:
            ep.ep_group_destroy(g)


def test_random_large_shapes_destination_order(ep, hx, oracle_mod):
    """Twenty-four seeded random configurations of at least 8192 routed entries (so that the
    destination-ordered kernel runs), odd row sizes, expert counts and top-k included; every other
    case announces its tokens to the layout call.  Layout and dispatched rows, side arrays and
    counts against the oracle."""
    rng = np.random.default_rng(777)
    done = 0
    case = 0
    while done < 24:
        case += 1
        R = int(rng.choice([1, 2, 4, 8, 16, 32, 64]))
        L = int(rng.choice([1, 2, 3, 4, 8]))
        E = R * L
        K = int(rng.integers(1, min(E, 9) + 1))
        T = int(rng.choice([8192 // K + 1, 9001 // K + 3, 20000 // K, 3000, 4099]))
        if T * K < 8192 or T * K > 70000:
            continue
        H = int(rng.choice([64, 72, 200, 512, 1000, 1536, 2048]))
        ll = bool(rng.integers(0, 2))
        C = int(rng.integers(max(1, (T * K) // (2 * E)), (3 * T * K) // (2 * E) + 2)) if ll else 0
        order = int(rng.choice([1, 2]))
        spec = wl.WorkloadSpec(f"randbig{case}", 140 + case, R=R, T=T, H=H, E=E, K=K,
                               prior=str(rng.choice(["uniform", "zipf"])))
        w = wl.make_workload(spec)
        topk = _mess_up(w.topk_idx, E, seed=case, frac_masked=float(rng.choice([0.0, 0.03])),
                        n_invalid=int(rng.integers(0, 2)))
        _say(f"random large case {case}: E={E} R={R} K={K} T={T} H={H} ll={ll} C={C} order={order}")
        lay = oracle_mod.layout(topk, E=E, R=R, layout=int(ll), C=C if ll else 0, C_rank=T)
        rows = E * C if ll else int(lay.expert_offset[-1])
        o_recv = np.full((rows + 1, H), hx.POISON, np.uint16)
        o_w = np.full(rows + 1, np.float32(-3.5), np.float32)
        o_src = np.full(rows + 1, -9, np.int32)
        oracle_mod.dispatch(w.x_bits, w.topk_w, lay, o_recv, o_w, o_src)
        g = _group(ep, spec, T, ep.EP_MODE_LL if ll else ep.EP_MODE_HT, C=C, dispatch_order=order)
        try:
            x = hx.bits_to_dev(w.x_bits)
            d_topk = torch.from_numpy(topk).to(hx.DEV)
            h = ep.ep_layout_prefetch(g, d_topk, x) if case % 2 else ep.ep_layout(g, d_topk)
            got = hx.fetch_layout(h, T, K, E, R, ok=(ep.EP_SUCCESS, ep.EP_ERR_INVALID_ROUTING))
            hx.assert_layout_equal(got, lay)
            store = hx.poison_bf16((rows + 1, H))
            recv = store[:rows].view(E, C, H) if ll else store[:rows]
            r_w = torch.full((rows + 1,), -3.5, dtype=torch.float32, device=hx.DEV)
            r_src = torch.full((rows + 1,), -9, dtype=torch.int32, device=hx.DEV)
            r_cnt = torch.full((E,), -1, dtype=torch.int32, device=hx.DEV)
            ep.ep_dispatch(h, x, recv, topk_weights=torch.from_numpy(w.topk_w).to(hx.DEV), recv_w=r_w[:rows],
                           recv_src=r_src[:rows], recv_count=r_cnt)
            torch.cuda.synchronize()
            assert np.array_equal(hx.dev_to_bits(store), o_recv), f"case {case}: rows differ"
            assert np.array_equal(r_w.cpu().numpy(), o_w) and np.array_equal(r_src.cpu().numpy(), o_src)
            assert np.array_equal(r_cnt.cpu().numpy(), lay.expert_kept)
            ep.ep_handle_destroy(h)
        finally:
            ep.ep_group_destroy(g)
        done += 1


def test_random_large_shapes_quantise_ahead(ep, hx, oracle_mod):
    """Sixteen seeded random configurations of at least 8192 routed entries in groups that quantise
    ahead: FP8 codes, scales, side arrays and counts of the staged, destination-ordered dispatch
    against the oracle (row sizes from one 128-channel group up, scale rows that end inside a
    16-byte unit, padded windows with and without drops); the handle's second quantising dispatch
    (token walk) must give the same."""
    rng = np.random.default_rng(4242)
    done = 0
    case = 0
    while done < 16:
        case += 1
        R = int(rng.choice([1, 2, 4, 8, 16, 32]))
        L = int(rng.choice([1, 2, 3, 4, 8]))
        E = R * L
        K = int(rng.integers(1, min(E, 9) + 1))
        T = int(rng.choice([8192 // K + 1, 9001 // K + 3, 16000 // K, 3000, 4099]))
        if T * K < 8192 or T * K > 40000:
            continue
        H = int(rng.choice([128, 256, 384, 640, 1024, 1152, 2048]))
        ll = bool(rng.integers(0, 2))
        C = int(rng.integers(max(1, (T * K) // (2 * E)), (3 * T * K) // (2 * E) + 2)) if ll else 0
        spec = wl.WorkloadSpec(f"randq{case}", 340 + case, R=R, T=T, H=H, E=E, K=K,
                               prior=str(rng.choice(["uniform", "zipf"])))
        w = wl.make_workload(spec)
        topk = _mess_up(w.topk_idx, E, seed=case, frac_masked=float(rng.choice([0.0, 0.03])))
        _say(f"random quantise-ahead case {case}: E={E} R={R} K={K} T={T} H={H} ll={ll} C={C}")
        lay = oracle_mod.layout(topk, E=E, R=R, layout=int(ll), C=C if ll else 0, C_rank=T)
        rows = E * C if ll else int(lay.expert_offset[-1])
        G = H // 128
        o_q = np.full((rows + 1, H), 0xAB, np.uint8)
        o_s = np.full((rows + 1, G), np.float32(-2.0), np.float32)
        oracle_mod.dispatch_fp8(w.x_bits, lay, o_q, o_s)
        valid = lay.dst_row >= 0
        want_src = np.full(rows + 1, -9, np.int32)
        want_src[lay.dst_row[valid]] = np.nonzero(valid)[0]
        g = _group(ep, spec, T, ep.EP_MODE_LL if ll else ep.EP_MODE_HT, C=C, dispatch_order=1, quantize_ahead=1)
        try:
            x = hx.bits_to_dev(w.x_bits)
            h = ep.ep_layout_prefetch(g, torch.from_numpy(topk).to(hx.DEV), x)
            store = torch.full((rows + 1, H), 0xAB, dtype=torch.uint8, device=hx.DEV)
            recv = store[:rows].view(torch.float8_e4m3fn)
            recv = recv.view(E, C, H) if ll else recv
            scales = torch.full((rows + 1, G), -2.0, dtype=torch.float32, device=hx.DEV)
            r_src = torch.full((rows + 1,), -9, dtype=torch.int32, device=hx.DEV)
            r_cnt = torch.full((E,), -1, dtype=torch.int32, device=hx.DEV)
            for again in range(2):
                if again:
                    store.fill_(0xAB); scales.fill_(-2.0); r_src.fill_(-9); r_cnt.fill_(-1)
                ep.ep_dispatch(h, x, recv, recv_scales=scales[:rows], recv_src=r_src[:rows], recv_count=r_cnt)
                torch.cuda.synchronize()
                assert np.array_equal(store.cpu().numpy(), o_q), f"case {case}: codes differ (dispatch {again})"
                assert np.array_equal(scales.cpu().numpy().view(np.uint32), o_s.view(np.uint32)), f"case {case}: scales differ"
                assert np.array_equal(r_src.cpu().numpy(), want_src)
                assert np.array_equal(r_cnt.cpu().numpy(), lay.expert_kept)
            ep.ep_handle_destroy(h)
        finally:
            ep.ep_group_destroy(g)
        done += 1
