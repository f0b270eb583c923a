"""ep_layout_static -- the layout entry point that allocates nothing -- against ep_layout
on the same inputs, array for array and bit for bit, on two calls in a row, the second with
a smaller input (the scratch array inside the library keeps the first call's contents)."""
import sys

import numpy as np
import pytest
import torch

from paper_2603_13606_amd import workloads as wl

pytestmark = pytest.mark.gpu

FILL = -77  # what the output arrays hold before a call


@pytest.fixture(scope="module")
def ep():
    from paper_2603_13606_amd import binding
    import ep_harness
    ep_harness.ensure_built()
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return binding


def _static_layout(ep, hx, cfg, topk, E, R, K, B):
    """One ep_layout_static call into freshly filled arrays sized for the group's maximum."""
    n_max = B * K
    sizes = dict(totals=16, expert_count=E, expert_kept=E, expert_offset=E + 1, rank_pair_count=R,
                 rank_token_count=R, rank_offset=R + 1, dst_row=n_max, slot=n_max, rank_row=n_max,
                 entry_rank=n_max, sorted_token=n_max, sorted_k=n_max, sorted_row=n_max)
    arrays = {k: torch.full((v,), FILL, dtype=torch.int32, device=hx.DEV) for k, v in sizes.items()}
    ep.ep_layout_static(cfg, topk, arrays)
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in arrays.items()}


@pytest.mark.parametrize("name,mode,C,T1,T2", [
    ("ht_prefill", "ht", 0, 4096, 1000),   # 32768 entries (32 chunk histograms in the scratch), then 8000
    ("skew", "ll", 512, 4096, 128),        # padded windows with capacity drops, then one workgroup's worth
    ("ll_decode", "ll", 0, 128, 31),       # at most 1024 entries: the one-workgroup kernel, then a ragged one
    ("stress", "ht", 0, 8192, 0),          # 65536 entries, then an empty batch
])
def test_layout_static_matches_ep_layout_twice(ep, name, mode, C, T1, T2):
    import ep_harness as hx
    spec = wl.SPECS[name]
    E, R, K, B = spec.E, spec.R, spec.K, T1
    ll = mode == "ll"
    cfg = ep.make_config(R, E, spec.H, K, B, mode=ep.EP_MODE_LL if ll else ep.EP_MODE_HT, slots_per_subregion=C)
    g = ep.ep_group_create(cfg)
    try:
        for T in (T1, T2):
            print(f"static layout case {name} mode={mode} C={C} T={T}", flush=True)
            sys.stdout.flush()
            topk_np, _, _ = wl.make_routing(spec, T=T, seed_offset=T)
            if T:
                topk_np[np.random.default_rng(T).random(topk_np.shape) < 0.02] = -1
            topk = torch.from_numpy(topk_np).to(hx.DEV) if T else torch.zeros((0, K), dtype=torch.int32, device=hx.DEV)
            got = _static_layout(ep, hx, cfg, topk, E, R, K, B)
            h = ep.ep_layout(g, topk)
            want = hx.fetch_layout(h, T, K, E, R)
            n, ns = T * K, int(want.info.entries_sorted)
            for key in ("expert_count", "expert_kept", "expert_offset", "rank_pair_count", "rank_token_count",
                        "rank_offset"):
                assert np.array_equal(got[key], want.arrays[key]), key
            for key in ("dst_row", "slot", "rank_row", "entry_rank"):
                assert np.array_equal(got[key][:n], want.arrays[key].reshape(-1)), key
                assert np.all(got[key][n:] == FILL), f"{key} written beyond T*K"
            for key in ("sorted_token", "sorted_k", "sorted_row"):
                assert np.array_equal(got[key][:ns], want.arrays[key]), key
                assert np.all(got[key][ns:] == FILL), f"{key} written beyond the sorted entries"
            i = want.info
            assert list(got["totals"][:8]) == [int(i.rows_kept), int(i.rows_dropped), int(i.entries_masked),
                                               int(i.entries_invalid), int(i.entries_sorted), int(i.rank_messages),
                                               int(i.status), int(i.rows_end)]
            ep.ep_handle_destroy(h)
    finally:
        ep.ep_group_destroy(g)


def test_layout_static_optional_arrays_and_errors(ep):
    import ep_harness as hx
    spec = wl.SPECS["ll_decode"]
    E, R, K, T = spec.E, spec.R, spec.K, 700
    cfg = ep.make_config(R, E, spec.H, K, T, mode=ep.EP_MODE_HT)
    topk_np, _, _ = wl.make_routing(spec, T=T)
    topk = torch.from_numpy(topk_np).to(hx.DEV)
    need = dict(totals=16, expert_count=E, expert_kept=E, expert_offset=E + 1, rank_pair_count=R,
                rank_token_count=R, rank_offset=R + 1, dst_row=T * K)
    arrays = {k: torch.full((v,), FILL, dtype=torch.int32, device=hx.DEV) for k, v in need.items()}
    ep.ep_layout_static(cfg, topk, arrays)  # only the required arrays
    g = ep.ep_group_create(cfg)
    h = ep.ep_layout(g, topk)
    want = hx.fetch_layout(h, T, K, E, R)
    torch.cuda.synchronize()
    assert np.array_equal(arrays["dst_row"].cpu().numpy(), want.arrays["dst_row"].reshape(-1))
    assert np.array_equal(arrays["expert_offset"].cpu().numpy(), want.arrays["expert_offset"])
    ep.ep_handle_destroy(h)
    ep.ep_group_destroy(g)
    # a missing required array, two of the three sorted arrays, a batch beyond the configured maximum,
    # a configuration beyond the limits the scratch array is sized for
    for bad in (dict(drop="dst_row"), dict(add=("sorted_token", "sorted_k")), dict(T=T + 1), dict(E=2048)):
        a = dict(arrays)
        c, tk = cfg, topk
        if "drop" in bad:
            del a[bad["drop"]]
        if "add" in bad:
            for k in bad["add"]:
                a[k] = torch.empty(T * K, dtype=torch.int32, device=hx.DEV)
        if "T" in bad:
            tk = torch.zeros((bad["T"], K), dtype=torch.int32, device=hx.DEV)
        if "E" in bad:
            c = ep.make_config(R, bad["E"], spec.H, K, T)
        with pytest.raises(ep.EpError) as e:
            ep.ep_layout_static(c, tk, a)
        assert e.value.code == ep.EP_ERR_INVALID_ARG, bad
