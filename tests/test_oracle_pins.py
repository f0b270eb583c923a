"""Pins for the CPU oracle: each test ties an oracle function to something that is
not the oracle -- the hand-worked example, values the paper prints, closed forms,
library routines (stable sort, bincount, cumsum, index_select), exact rational
arithmetic, brute force on tiny inputs.  A dropped term, a wrong sign or index, or
a transposed operand in the oracle fails at least one of them."""
import itertools
import json
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from paper_2603_13606_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return json.load(f)


# --------------------------------------------------------------------------- layout


def test_worked_example_concat(oracle_mod):
    g = _golden("worked_example_layout.json")
    c = g["concat"]
    lay = oracle_mod.layout(np.array(g["topk_idx"], np.int32), E=g["E"], R=g["R"])
    assert lay.expert_count.tolist() == c["expert_count"]
    assert lay.expert_kept.tolist() == c["expert_count"]
    assert lay.expert_offset.tolist() == c["expert_offset"]
    assert lay.slot.tolist() == c["slot"]
    assert lay.dst_row.tolist() == c["dst_row"]
    assert lay.sorted_token[: lay.n_sorted].tolist() == c["sorted_token"]
    assert lay.sorted_k[: lay.n_sorted].tolist() == c["sorted_k"]
    assert lay.sorted_row[: lay.n_sorted].tolist() == list(range(8))
    assert lay.rank_pair_count.tolist() == c["rank_pair_count"]
    assert lay.rank_token_count.tolist() == c["rank_token_count"]
    assert lay.rank_offset.tolist() == c["rank_offset"]
    L = g["E"] // g["R"]
    topk = np.array(g["topk_idx"])
    for d_str, per_tok in c["rank_slot_by_rank"].items():
        d = int(d_str)
        for t_str, s in per_tok.items():
            t = int(t_str)
            ks = [k for k in range(g["K"]) if topk[t, k] // L == d]
            assert lay.rank_row[t, ks[0]] == c["rank_offset"][d] + s
            for k in ks[1:]:
                assert lay.rank_row[t, k] == -1
    assert (lay.kept, lay.dropped, lay.masked, lay.invalid, lay.n_msgs) == (8, 0, 0, 0, 7)


def test_worked_example_padded_overflow(oracle_mod):
    g = _golden("worked_example_layout.json")
    p = g["padded_C2"]
    lay = oracle_mod.layout(np.array(g["topk_idx"], np.int32), E=g["E"], R=g["R"],
                            layout=oracle_mod.LAYOUT_PADDED, C=p["C"])
    assert lay.expert_count.tolist() == g["concat"]["expert_count"]  # demand is not capped
    assert lay.expert_kept.tolist() == p["expert_kept"]
    assert lay.expert_offset.tolist() == p["expert_offset"]
    assert lay.dst_row.tolist() == p["dst_row"]
    assert lay.dropped == p["dropped"] and lay.kept == 7
    assert lay.slot.tolist() == g["concat"]["slot"]
    # staging windows in the 3-D mode have T slots per destination rank
    assert lay.rank_offset.tolist() == [0, 4, 8]


def _brute_slot(topk, E):
    """O(n^2) definition: slot = number of earlier flattened entries naming the same expert."""
    flat = topk.reshape(-1)
    out = np.full(flat.shape, -1, np.int64)
    for i, e in enumerate(flat):
        if 0 <= e < E:
            out[i] = sum(1 for j in range(i) if flat[j] == e)
    return out.reshape(topk.shape)


def test_exhaustive_tiny_against_predecessor_count(oracle_mod):
    E, R, K = 4, 2, 2
    L = E // R
    vals = [-1, 0, 1, 2, 3, 9]  # -1 masked, 9 invalid
    for T in (1, 2, 3):
        pool = vals if T < 3 else vals[:5]
        for flat in itertools.product(pool, repeat=T * K):
            topk = np.array(flat, np.int32).reshape(T, K)
            lay = oracle_mod.layout(topk, E=E, R=R)
            slot = _brute_slot(topk, E)
            assert np.array_equal(lay.slot, slot)
            cnt = np.array([(topk == e).sum() for e in range(E)])
            assert np.array_equal(lay.expert_count, cnt)
            off = np.concatenate([[0], np.cumsum(cnt)])
            assert np.array_equal(lay.expert_offset, off)
            valid = (topk >= 0) & (topk < E)
            want = np.where(valid, off[np.clip(topk, 0, E - 1)] + slot, -1)
            assert np.array_equal(lay.dst_row, want)
            # each token counted once per destination rank, in token order
            rtc = np.zeros(R, np.int64)
            for t in range(T):
                seen = []
                for k in range(K):
                    if not valid[t, k]:
                        assert lay.rank_row[t, k] == -1
                        continue
                    d = topk[t, k] // L
                    if d in seen:
                        assert lay.rank_row[t, k] == -1
                    else:
                        seen.append(d)
                        # filled in after counts are known (needs rank_offset)
                for d in set(seen):
                    rtc[d] += 1
            assert np.array_equal(lay.rank_token_count, rtc)
            assert lay.masked == int((topk == -1).sum())
            assert lay.invalid == int(((topk != -1) & ~valid).sum())


def _torch_layout(topk, E):
    """Counting sort by library routines: stable sort of the flattened expert ids."""
    flat = torch.from_numpy(topk.reshape(-1).astype(np.int64))
    valid = (flat >= 0) & (flat < E)
    key = torch.where(valid, flat, torch.full_like(flat, E))
    _, perm = torch.sort(key, stable=True)
    n_valid = int(valid.sum())
    perm = perm[:n_valid]
    dst = torch.full_like(flat, -1)
    dst[perm] = torch.arange(n_valid)
    counts = torch.bincount(flat[valid], minlength=E)
    offs = torch.cat([torch.zeros(1, dtype=torch.int64), torch.cumsum(counts, 0)])
    return dst.numpy().reshape(topk.shape), counts.numpy(), offs.numpy(), perm.numpy()


@pytest.mark.parametrize("name,T", [("tiny", None), ("ll_decode", None), ("skew", 777),
                                    ("ht_prefill", 1500), ("stress_hot", 2048)])
def test_layout_equals_stable_sort(oracle_mod, name, T):
    spec = wl.SPECS[name]
    topk, _, _ = wl.make_routing(spec, T=T)
    rng = np.random.default_rng(5)
    topk = topk.copy()
    topk[rng.random(topk.shape) < 0.03] = -1  # a few masked entries
    lay = oracle_mod.layout(topk, E=spec.E, R=spec.R)
    dst, counts, offs, perm = _torch_layout(topk, spec.E)
    K = spec.K
    assert np.array_equal(lay.dst_row, dst)
    assert np.array_equal(lay.expert_count, counts)
    assert np.array_equal(lay.expert_offset, offs)
    assert np.array_equal(lay.sorted_token[: lay.n_sorted], perm // K)
    assert np.array_equal(lay.sorted_k[: lay.n_sorted], perm % K)
    assert np.array_equal(lay.sorted_row[: lay.n_sorted], np.arange(lay.n_sorted))
    # invariants
    assert lay.expert_count.sum() == topk.size - lay.masked
    L = spec.L
    assert np.array_equal(lay.rank_pair_count, counts.reshape(spec.R, L).sum(1))
    owners = np.where(topk >= 0, topk // L, -1)
    distinct = [set(r[r >= 0].tolist()) for r in owners]
    assert lay.rank_token_count.sum() == sum(len(s) for s in distinct) == lay.n_msgs
    for d in range(spec.R):
        toks = [t for t, s in enumerate(distinct) if d in s]
        assert lay.rank_token_count[d] == len(toks)
        assert lay.rank_token_count[d] <= min(len(topk), lay.rank_pair_count[d])
        got = sorted((int(lay.rank_row[t][np.argmax(owners[t] == d)]), t) for t in toks)
        # slots are consecutive from rank_offset[d] and increase with the token index
        assert [g[0] for g in got] == list(range(lay.rank_offset[d], lay.rank_offset[d] + len(toks)))
        assert [g[1] for g in got] == toks
    assert (lay.rank_row >= 0).sum() == lay.n_msgs
    # within each expert the source tokens are non-decreasing
    for e in range(spec.E):
        seg = lay.sorted_token[lay.expert_offset[e]: lay.expert_offset[e + 1]]
        assert np.all(np.diff(seg) >= 0)


def test_padded_overflow_drops_highest_tokens(oracle_mod):
    spec = wl.SPECS["skew_rank0"]
    topk, _, _ = wl.make_routing(spec, T=1024)
    C = 2 * 1024 * spec.K // spec.E
    lay = oracle_mod.layout(topk, E=spec.E, R=spec.R, layout=oracle_mod.LAYOUT_PADDED, C=C)
    ref = oracle_mod.layout(topk, E=spec.E, R=spec.R)
    assert lay.dropped > 0
    assert np.array_equal(lay.slot, ref.slot) and np.array_equal(lay.expert_count, ref.expert_count)
    assert np.array_equal(lay.expert_kept, np.minimum(ref.expert_count, C))
    want = np.where(ref.slot < C, topk * C + ref.slot, -1)
    assert np.array_equal(lay.dst_row, want)
    assert lay.dropped == int((ref.slot >= C).sum()) and lay.kept + lay.dropped == topk.size
    assert np.array_equal(lay.rank_offset, np.arange(spec.R + 1) * 1024)


def test_expert_base_shifts_rows(oracle_mod):
    spec = wl.SPECS["tiny"]
    topk, _, _ = wl.make_routing(spec)
    base = (np.arange(spec.E, dtype=np.int32) * 100 + 7).astype(np.int32)
    lay = oracle_mod.layout(topk, E=spec.E, R=spec.R, expert_base=base)
    ref = oracle_mod.layout(topk, E=spec.E, R=spec.R)
    assert np.array_equal(lay.dst_row, base[topk] + ref.slot)
    assert lay.expert_offset[-1] == max(base[e] + ref.expert_count[e] for e in range(spec.E)
                                        if ref.expert_count[e] > 0)
    assert np.array_equal(lay.sorted_token[: lay.n_sorted], ref.sorted_token[: ref.n_sorted])


def test_empty_and_single(oracle_mod):
    lay = oracle_mod.layout(np.zeros((0, 8), np.int32), E=16, R=4)
    assert lay.expert_count.sum() == 0 and lay.expert_offset.tolist() == [0] * 17 and lay.kept == 0
    lay = oracle_mod.layout(np.array([[5]], np.int32), E=16, R=4)
    assert lay.dst_row.tolist() == [[0]] and lay.rank_token_count.tolist() == [0, 1, 0, 0]


# --------------------------------------------------------------------------- bf16 rounding


def test_bf16_roundtrip_all_values(oracle_mod):
    lib = oracle_mod.lib()
    for b in range(0, 65536):
        f = np.array([b], np.uint16).astype(np.uint32) << 16
        v = float(f.view(np.float32)[0])
        if v != v:
            assert oracle_mod.double_to_bf16(v) & 0x7F80 == 0x7F80 and oracle_mod.double_to_bf16(v) & 0x7F
            continue
        assert oracle_mod.double_to_bf16(v) == b
        assert lib.ep_oracle_bf16_to_float(b) == v


def test_bf16_ties_and_neighbours(oracle_mod):
    # 1 + 2^-8 is exactly between bf16 1.0 (mantissa 0, even) and 1.0078125 (odd)
    assert oracle_mod.double_to_bf16(1.0 + 2.0 ** -8) == 0x3F80
    assert oracle_mod.double_to_bf16(1.0 + 2.0 ** -8 + 2.0 ** -40) == 0x3F81
    assert oracle_mod.double_to_bf16(1.0078125 + 2.0 ** -8) == 0x3F82  # tie goes up to even
    assert oracle_mod.double_to_bf16(1.0078125 + 2.0 ** -8 - 2.0 ** -40) == 0x3F81
    assert oracle_mod.double_to_bf16(-(1.0 + 2.0 ** -8)) == 0xBF80
    assert oracle_mod.double_to_bf16(1.99609375 + 2.0 ** -8) == 0x4000  # carries into next binade
    assert oracle_mod.double_to_bf16(3.4e38) == 0x7F80  # rounds to infinity
    assert oracle_mod.double_to_bf16(2.0 ** -133) == 0x0001  # smallest subnormal
    assert oracle_mod.double_to_bf16(2.0 ** -134) == 0x0000  # tie to even (zero)
    assert oracle_mod.double_to_bf16(2.0 ** -134 * 1.0001) == 0x0001
    assert oracle_mod.double_to_bf16(-0.0) == 0x8000


def test_bf16_matches_torch_rne(oracle_mod):
    rng = np.random.default_rng(3)
    a = np.concatenate([rng.standard_normal(20000).astype(np.float32) * 3,
                        (rng.standard_normal(2000) * 1e-3).astype(np.float32),
                        np.float32(2.0) ** rng.integers(-140, 127, 2000).astype(np.float32)])
    want = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle_mod.double_to_bf16(float(v)) for v in a], np.uint16)
    assert np.array_equal(got, want)
    assert np.array_equal(wl.f32_to_bf16_bits(a), want)  # the input generator's own conversion


# --------------------------------------------------------------------------- dispatch


@pytest.mark.parametrize("name,T", [("tiny", None), ("ll_decode", 40), ("skew", 300)])
def test_dispatch_is_index_select(oracle_mod, name, T):
    w = wl.make_workload(name, T=T)
    spec = w.spec
    lay = oracle_mod.layout(w.topk_idx, E=spec.E, R=spec.R)
    rows = lay.expert_offset[-1]
    guard = 3
    recv = np.full((rows + guard, spec.H), 0xDEAD, np.uint16)
    recv_w = np.full(rows + guard, np.float32(-77.0), np.float32)
    recv_src = np.full(rows + guard, -5, np.int32)
    oracle_mod.dispatch(w.x_bits, w.topk_w, lay, recv, recv_w, recv_src)
    dst, counts, offs, perm = _torch_layout(w.topk_idx, spec.E)
    xt = torch.from_numpy(w.x_bits.view(np.int16))
    want = xt.index_select(0, torch.from_numpy(perm // spec.K)).numpy().view(np.uint16)
    assert np.array_equal(recv[:rows], want)
    assert np.all(recv[rows:] == 0xDEAD) and np.all(recv_w[rows:] == -77.0) and np.all(recv_src[rows:] == -5)
    assert np.array_equal(recv_src[:rows], perm // spec.K)
    assert np.array_equal(recv_w[:rows], w.topk_w.reshape(-1)[perm])
    # every token lands exactly once per selected expert
    for e in range(spec.E):
        seg = recv_src[offs[e]: offs[e + 1]]
        want_tok = np.nonzero((w.topk_idx == e).any(1))[0]
        assert np.array_equal(seg, want_tok)


def test_dispatch_without_weights_forwards_unit_weights(oracle_mod):
    """No gate weights given: every placed row gets the weight 1 (absent weights mean a plain sum,
    Sec. III-B), rows without an entry keep their fill; the once-per-rank path, whose message
    headers then carry 1.0, ends with the same side array."""
    w = wl.make_workload("ll_decode", T=40)
    spec = w.spec
    topk = w.topk_idx.copy()
    topk[::7, 1] = -1
    lay = oracle_mod.layout(topk, E=spec.E, R=spec.R)
    rows = int(lay.expert_offset[-1])
    recv = np.zeros((rows + 2, spec.H), np.uint16)
    recv_w = np.full(rows + 2, np.float32(-77.0), np.float32)
    oracle_mod.dispatch(w.x_bits, None, lay, recv, recv_w)
    assert np.all(recv_w[:rows] == 1.0) and np.all(recv_w[rows:] == -77.0)
    combined = oracle_mod.combine(recv[:rows], recv_w_to_topk(recv_w, lay), lay, spec.H, acc="f32")
    assert np.array_equal(combined, oracle_mod.combine(recv[:rows], None, lay, spec.H, acc="f32"))


def recv_w_to_topk(recv_w, lay):
    """The forwarded per-row weights seen from the token side: w[t, k] = recv_w[dst_row[t, k]]."""
    out = np.zeros(lay.dst_row.shape, np.float32)
    ok = lay.dst_row >= 0
    out[ok] = recv_w[lay.dst_row[ok]]
    return out


def test_dispatch_padded_strided_and_poison(oracle_mod):
    """3-D [E, C, H] windows embedded in a receiver tensor [E, R*C, H]: only this
    source's sub-region of each expert may change (Sec. III-E LL layout)."""
    w = wl.make_workload("tiny")
    spec = w.spec
    C, my_rank = 6, 1
    lay = oracle_mod.layout(w.topk_idx, E=spec.E, R=spec.R, layout=oracle_mod.LAYOUT_PADDED, C=C)
    assert lay.dropped > 0
    full = np.full((spec.E, spec.R * C, spec.H), 0xBEEF, np.uint16)
    view = full[:, my_rank * C:(my_rank + 1) * C, :]
    oracle_mod.dispatch(w.x_bits, None, lay, view, stride0=spec.R * C * spec.H, stride1=spec.H)
    for e in range(spec.E):
        toks = [t for t in range(spec.T) for k in range(spec.K) if w.topk_idx[t, k] == e]
        kept = toks[:C]
        assert lay.expert_kept[e] == len(kept)
        for s, t in enumerate(kept):
            assert np.array_equal(full[e, my_rank * C + s], w.x_bits[t])
        assert np.all(full[e, my_rank * C + len(kept):(my_rank + 1) * C] == 0xBEEF)
        assert np.all(full[e, :my_rank * C] == 0xBEEF)


# --------------------------------------------------------------------------- combine


def _exact_bf16_neighbours(fr: Fraction):
    """The two bf16 values bracketing an exact rational, and the nearest (None on a tie)."""
    if fr == 0:
        return 0.0, 0.0, 0.0
    a = abs(fr)
    e = 0
    while Fraction(2) ** (e + 1) <= a:
        e += 1
    while Fraction(2) ** e > a:
        e -= 1
    q = Fraction(2) ** (max(e, -126) - 7)
    lo = (a // q) * q
    hi = lo + q
    sgn = -1 if fr < 0 else 1
    if a - lo < hi - a:
        near = lo
    elif a - lo > hi - a:
        near = hi
    else:
        near = None
    return sgn * float(lo), sgn * float(hi), (None if near is None else sgn * float(near))


def test_combine_against_exact_rational(oracle_mod):
    w = wl.make_workload("tiny", expert_scale=True)
    spec = w.spec
    lay = oracle_mod.layout(w.topk_idx, E=spec.E, R=spec.R)
    rows = lay.expert_offset[-1]
    rng = np.random.default_rng(11)
    y = wl.f32_to_bf16_bits(rng.standard_normal((rows, spec.H)).astype(np.float32))
    out64 = oracle_mod.combine(y, w.topk_w, lay, spec.H, acc="f64")
    out32 = oracle_mod.combine(y, w.topk_w, lay, spec.H, acc="f32")
    yf = wl.bf16_bits_to_f32(y)
    o64 = wl.bf16_bits_to_f32(out64)
    o32 = wl.bf16_bits_to_f32(out32)
    checked = 0
    for t in range(0, spec.T, 5):
        for h in range(0, spec.H, 37):
            exact = sum(Fraction(float(w.topk_w[t, k])) * Fraction(float(yf[lay.dst_row[t, k], h]))
                        for k in range(spec.K))
            lo, hi, near = _exact_bf16_neighbours(exact)
            assert o64[t, h] in (lo, hi)
            if near is not None and abs(exact - Fraction(near)) * 2 ** 30 < abs(Fraction(hi) - Fraction(lo)) * (2 ** 29 - 1):
                assert o64[t, h] == near  # not within 2^-30 of a tie: must be the nearest
            assert o32[t, h] in (lo, hi)
            checked += 1
    assert checked > 50


def test_combine_one_hot_weights_select_the_kth_row(oracle_mod):
    w = wl.make_workload("ll_decode", T=24, H=64)
    spec = w.spec
    lay = oracle_mod.layout(w.topk_idx, E=spec.E, R=spec.R)
    rows = lay.expert_offset[-1]
    y = wl.f32_to_bf16_bits(np.random.default_rng(2).standard_normal((rows, spec.H)).astype(np.float32))
    for j in range(spec.K):
        onehot = np.zeros((spec.T, spec.K), np.float32)
        onehot[:, j] = 1.0
        for acc in ("f64", "f32"):
            out = oracle_mod.combine(y, onehot, lay, spec.H, acc=acc)
            want = y[lay.dst_row[:, j]]
            # adding +0 keeps every value; -0 becomes +0
            want = np.where(want == 0x8000, 0, want)
            assert np.array_equal(out, want)


def test_combine_matches_torch_within_one_ulp(oracle_mod):
    w = wl.make_workload("skew", T=200, H=512)
    spec = w.spec
    lay = oracle_mod.layout(w.topk_idx, E=spec.E, R=spec.R)
    rows = lay.expert_offset[-1]
    recv = np.zeros((rows, spec.H), np.uint16)
    oracle_mod.dispatch(w.x_bits, None, lay, recv)
    scale = wl.expert_scale_table(spec)
    row_e = np.repeat(np.arange(spec.E), lay.expert_count)
    y = wl.f32_to_bf16_bits(wl.bf16_bits_to_f32(recv) * scale[row_e][:, None])
    out = wl.bf16_bits_to_f32(oracle_mod.combine(y, w.topk_w, lay, spec.H))
    yt = torch.from_numpy(wl.bf16_bits_to_f32(y)).double()
    ref = (yt[torch.from_numpy(lay.dst_row.astype(np.int64))] *
           torch.from_numpy(w.topk_w).double()[..., None]).sum(1)
    ref_bf = ref.float().to(torch.bfloat16).float().numpy()
    ulp = np.maximum(np.abs(ref_bf), 2.0 ** -126) * 2.0 ** -7
    assert np.all(np.abs(out - ref_bf) <= ulp)
    assert (out == ref_bf).mean() > 0.999
    # closed form of the stand-in experts: x * sum_k w_k (1 + e_k/256), y rounded once
    x = wl.bf16_bits_to_f32(w.x_bits).astype(np.float64)
    g = (w.topk_w.astype(np.float64) * scale[w.topk_idx].astype(np.float64)).sum(1)
    closed = x * g[:, None]
    assert np.all(np.abs(out - closed) <= 2.5 * np.maximum(np.abs(closed), 1e-30) * 2.0 ** -8)


def test_round_trip_identity_experts(oracle_mod):
    """combine(dispatch(x)) = bf16(x * sum_k w[t,k]) with identity experts; with
    renormalised weights that is x to within one bf16 ulp."""
    w = wl.make_workload("tiny")
    spec = w.spec
    lay = oracle_mod.layout(w.topk_idx, E=spec.E, R=spec.R)
    recv = np.zeros((lay.expert_offset[-1], spec.H), np.uint16)
    oracle_mod.dispatch(w.x_bits, w.topk_w, lay, recv)
    out = wl.bf16_bits_to_f32(oracle_mod.combine(recv, w.topk_w, lay, spec.H))
    x = wl.bf16_bits_to_f32(w.x_bits)
    assert np.all(np.abs(out - x) <= np.abs(x) * 2.0 ** -7)
    # unweighted: exactly K * x when K is a power of two
    out1 = wl.bf16_bits_to_f32(oracle_mod.combine(recv, None, lay, spec.H))
    assert np.array_equal(out1, x * spec.K)
    # arbitrary weights: x * sum(w) with exact products
    w2 = np.random.default_rng(4).random((spec.T, spec.K)).astype(np.float32)
    out2 = oracle_mod.combine(recv, w2, lay, spec.H)
    s = w2.astype(np.float64).sum(1)
    want = np.array([[oracle_mod.double_to_bf16(float(x[t, h]) * float(s[t])) for h in range(0, spec.H, 17)]
                     for t in range(spec.T)], np.uint16)
    got = out2[:, ::17]
    diff = np.abs(wl.bf16_bits_to_f32(got) - wl.bf16_bits_to_f32(want))
    assert np.all(diff <= np.abs(wl.bf16_bits_to_f32(want)) * 2.0 ** -7)
    assert (got == want).mean() > 0.98


def test_combine_dropped_entries_contribute_zero(oracle_mod):
    w = wl.make_workload("tiny")
    spec = w.spec
    C = 6
    lay = oracle_mod.layout(w.topk_idx, E=spec.E, R=spec.R, layout=oracle_mod.LAYOUT_PADDED, C=C)
    recv = np.zeros((spec.E, C, spec.H), np.uint16)
    oracle_mod.dispatch(w.x_bits, None, lay, recv)
    out = wl.bf16_bits_to_f32(oracle_mod.combine(recv, w.topk_w, lay, spec.H))
    x = wl.bf16_bits_to_f32(w.x_bits).astype(np.float64)
    keep_w = np.where(lay.dst_row >= 0, w.topk_w, 0).astype(np.float64).sum(1)
    want = x * keep_w[:, None]
    assert np.all(np.abs(out - want) <= np.abs(want) * 2.0 ** -7 + 1e-30)
    assert (lay.dst_row < 0).any()


# --------------------------------------------------------------------------- once-per-rank path


@pytest.mark.parametrize("mode", ["concat", "padded"])
def test_dedup_equals_direct(oracle_mod, mode):
    w = wl.make_workload("ll_decode", T=48, H=128)
    spec = w.spec
    topk = w.topk_idx.copy()
    topk[3, 2] = -1
    if mode == "padded":
        C = 3
        lay = oracle_mod.layout(topk, E=spec.E, R=spec.R, layout=oracle_mod.LAYOUT_PADDED, C=C)
        shape = (spec.E * C, spec.H)
        n_slots = spec.R * spec.T
    else:
        lay = oracle_mod.layout(topk, E=spec.E, R=spec.R)
        shape = (lay.expert_offset[-1], spec.H)
        n_slots = lay.n_msgs
    direct = np.full(shape, 0x1111, np.uint16)
    dw = np.full(shape[0], np.float32(-1), np.float32)
    ds = np.full(shape[0], -9, np.int32)
    oracle_mod.dispatch(w.x_bits, w.topk_w, lay, direct, dw, ds)
    win = oracle_mod.dedup_send(w.x_bits, topk, w.topk_w, lay, n_slots)
    hdr = oracle_mod.msg_header_bytes(spec.K)
    assert hdr == 80 and hdr % 16 == 0 and win.shape[1] == hdr + 2 * spec.H
    # header fields and payload of every message; untouched slots keep their fill
    used = np.zeros(n_slots, bool)
    L = spec.L
    for t in range(spec.T):
        owners = []
        for k in range(spec.K):
            e = topk[t, k]
            if e < 0 or (e // L) in owners:
                assert lay.rank_row[t, k] == -1
                continue
            owners.append(e // L)
            m = lay.rank_row[t, k]
            used[m] = True
            msg = win[m]
            assert msg[:4].view(np.int32)[0] == t
            assert np.array_equal(msg[4:4 + 4 * spec.K].view(np.int32), topk[t])
            assert np.array_equal(msg[4 + 4 * spec.K:4 + 8 * spec.K].view(np.float32), w.topk_w[t])
            assert np.all(msg[4 + 8 * spec.K:hdr] == 0)
            assert np.array_equal(msg[hdr:].view(np.uint16), w.x_bits[t])
    assert used.sum() == lay.n_msgs and np.all(win[~used] == 0xA5)
    via = np.full(shape, 0x1111, np.uint16)
    vw = np.full(shape[0], np.float32(-1), np.float32)
    vs = np.full(shape[0], -9, np.int32)
    cnt, dropped = oracle_mod.dedup_recv(win, lay, spec.H, via, vw, vs)
    assert np.array_equal(via, direct) and np.array_equal(vw, dw) and np.array_equal(vs, ds)
    assert np.array_equal(cnt, lay.expert_kept) and dropped == lay.dropped


# --------------------------------------------------------------------------- paper constants


def test_paper_constants(oracle_mod):
    g = _golden("paper_constants.json")
    assert wl.SPECS["ll_decode"].row_bytes == g["row_bytes_bf16"] == 2 * g["hidden"]
    assert g["row_bytes_fp8"] == g["hidden"] and g["scale_floats"] * 4 == g["scale_bytes"]
    assert g["hidden"] // 128 == g["scale_floats"]
    b = g["ll_benchmark"]
    s = wl.SPECS["ll_decode"]
    assert (s.E, s.H, s.T, s.K) == (b["E"], b["H"], b["T"], b["K"])
    f = g["footprint_example"]
    for B, P in ((128, 14336), (1, 1), (77, 7168 + 224)):
        ratio = Fraction(oracle_mod.footprint_per_expert(f["E"], B, P),
                         oracle_mod.footprint_optimised(f["N"], B, f["K"], P))
        assert ratio == Fraction(2 * f["E"], f["N"] + f["K"])
    assert abs(float(ratio) - f["ratio_approx"]) < 0.5
    assert Fraction(oracle_mod.footprint_per_expert(256, 128, 14336),
                    oracle_mod.footprint_optimised(32, 128, 8, 14336)) == Fraction(512, 40)


# --------------------------------------------------------------------------- FP8 quantising dispatch


def _e4m3_value(c):
    """OCP E4M3 by its definition: sign, 4 exponent bits (bias 7), 3 mantissa bits."""
    s, e, m = c >> 7, (c >> 3) & 15, c & 7
    if e == 15 and m == 7:
        return float("nan")
    v = (m / 8.0) * 2.0 ** -6 if e == 0 else (1 + m / 8.0) * 2.0 ** (e - 7)
    return -v if s else v


def test_e4m3_all_codes_and_rounding(oracle_mod):
    vals = []
    for c in range(256):
        v = _e4m3_value(c)
        got = oracle_mod.e4m3_to_float(c)
        if v != v:
            assert got != got
            continue
        assert got == v
        if v == 0.0:
            continue  # +0 / -0 checked below
        assert oracle_mod.double_to_e4m3(v) == c
        if c < 0x7F:
            vals.append(v)
    assert max(vals) == 448.0 and min(v for v in vals if v > 0) == 2.0 ** -9
    assert oracle_mod.double_to_e4m3(0.0) == 0 and oracle_mod.double_to_e4m3(-0.0) == 0x80
    vals = sorted(vals)
    # midpoints go to the even code; a hair to either side goes to the nearer code
    for lo, hi in zip(vals[:-1], vals[1:]):
        mid = (lo + hi) / 2
        c_lo, c_hi = oracle_mod.double_to_e4m3(lo), oracle_mod.double_to_e4m3(hi)
        even = c_lo if c_lo % 2 == 0 else c_hi
        assert oracle_mod.double_to_e4m3(mid) == even
        assert oracle_mod.double_to_e4m3(mid * (1 - 1e-9)) == c_lo
        assert oracle_mod.double_to_e4m3(mid * (1 + 1e-9)) == c_hi
    # saturation instead of overflow; NaN stays NaN
    for v, c in ((448.0001, 0x7E), (1e30, 0x7E), (-500.0, 0xFE), (float("inf"), 0x7E)):
        assert oracle_mod.double_to_e4m3(v) == c
    assert oracle_mod.double_to_e4m3(float("nan")) == 0x7F
    assert oracle_mod.double_to_e4m3(2.0 ** -10) == 0 and oracle_mod.double_to_e4m3(2.0 ** -10 * 1.001) == 1


def test_e4m3_matches_torch_in_range(oracle_mod):
    rng = np.random.default_rng(5)
    a = np.concatenate([rng.standard_normal(20000).astype(np.float32) * 100,
                        rng.standard_normal(5000).astype(np.float32) * 0.01,
                        rng.uniform(-448, 448, 5000).astype(np.float32)])
    a = a[np.abs(a) <= 448.0]
    want = torch.from_numpy(a).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle_mod.double_to_e4m3(float(v)) for v in a], np.uint8)
    assert np.array_equal(got, want)


def test_quantize_row_properties(oracle_mod):
    g = _golden("paper_constants.json")
    w = wl.make_workload("ll_decode", T=6)
    H = w.spec.H
    assert H == g["hidden"]
    for t in range(6):
        q, sc = oracle_mod.quantize_row(w.x_bits[t])
        assert q.nbytes == g["row_bytes_fp8"] and sc.size == g["scale_floats"] and sc.nbytes == g["scale_bytes"]
        x = wl.bf16_bits_to_f32(w.x_bits[t]).reshape(-1, 128)
        amax = np.abs(x).max(1)
        assert np.array_equal(sc, (amax / np.float32(448.0)).astype(np.float32))
        deq = np.array([_e4m3_value(int(c)) for c in q], np.float64).reshape(-1, 128) * sc[:, None].astype(np.float64)
        # the largest element of every group maps to +-448 exactly, so it dequantises to itself
        idx = np.abs(x).argmax(1)
        rows = np.arange(x.shape[0])
        assert np.all(np.abs(q.reshape(-1, 128)[rows, idx] & 0x7F) == 0x7E)
        assert np.allclose(deq[rows, idx], x[rows, idx], rtol=2 ** -22)
        # 3 mantissa bits: relative error at most 2^-4 in the normal range, absolute 2^-10*scale below it
        err = np.abs(deq - x)
        bound = np.maximum(np.abs(x) * 2.0 ** -4, sc[:, None] * 2.0 ** -10) * (1 + 1e-6)
        assert np.all(err <= bound)
        # independent re-derivation through torch's E4M3 cast of x * (448 / amax)
        inv = (np.float32(448.0) / amax).astype(np.float32)
        p = (x * inv[:, None]).astype(np.float32)
        p = np.clip(p, -448.0, 448.0)
        want = torch.from_numpy(p).to(torch.float8_e4m3fn).view(torch.uint8).numpy().reshape(-1)
        assert np.array_equal(q, want)
    z = np.zeros(256, np.uint16)
    z[130] = 0x8000  # -0
    q, sc = oracle_mod.quantize_row(z)
    assert np.all(sc == 1.0) and q[130] == 0x80 and np.all(np.delete(q, 130) == 0)


def test_dispatch_fp8_places_quantised_rows(oracle_mod):
    w = wl.make_workload("ll_decode", T=20, H=256)
    spec = w.spec
    lay = oracle_mod.layout(w.topk_idx, E=spec.E, R=spec.R)
    rows = lay.expert_offset[-1]
    rq = np.full((rows + 1, spec.H), 0xAB, np.uint8)
    rs = np.full((rows + 1, spec.H // 128), np.float32(-2), np.float32)
    oracle_mod.dispatch_fp8(w.x_bits, lay, rq, rs)
    assert np.all(rq[rows] == 0xAB) and np.all(rs[rows] == -2)
    for t in range(spec.T):
        q, sc = oracle_mod.quantize_row(w.x_bits[t])
        for k in range(spec.K):
            r = lay.dst_row[t, k]
            assert np.array_equal(rq[r], q) and np.array_equal(rs[r], sc)


# --------------------------------------------------------------------------- hierarchical combine order


def test_combine_hier_order(oracle_mod):
    w = wl.make_workload("ll_decode", T=40, H=96)
    spec = w.spec
    topk = w.topk_idx.copy()
    topk[2, 3] = -1
    lay = oracle_mod.layout(topk, E=spec.E, R=spec.R)
    rows = lay.expert_offset[-1]
    y = wl.f32_to_bf16_bits(np.random.default_rng(9).standard_normal((rows, spec.H)).astype(np.float32) * 3)
    flat = oracle_mod.combine(y, w.topk_w, lay, spec.H, acc="f32")
    # one node holding every rank: the two-level order degenerates to the flat one
    assert np.array_equal(oracle_mod.combine_hier(y, w.topk_w, lay, topk, spec.H, ranks_per_node=spec.R), flat)
    rpn = 8
    hier = oracle_mod.combine_hier(y, w.topk_w, lay, topk, spec.H, ranks_per_node=rpn)
    # the same two-level order written with numpy float32 scalars (IEEE, round to nearest even)
    yf = wl.bf16_bits_to_f32(y)
    L = spec.L
    want = np.zeros((spec.T, spec.H), np.float32)
    for t in range(spec.T):
        total = np.zeros(spec.H, np.float32)
        for n in range(spec.R // rpn):
            part, has = np.zeros(spec.H, np.float32), False
            for k in range(spec.K):
                if lay.dst_row[t, k] < 0 or (topk[t, k] // L) // rpn != n:
                    continue
                part = (part + (np.float32(w.topk_w[t, k]) * yf[lay.dst_row[t, k]]).astype(np.float32)).astype(np.float32)
                has = True
            if has:
                total = (total + part).astype(np.float32)
        want[t] = total
    assert np.array_equal(hier, wl.f32_to_bf16_bits(want))
    # a different association of the same sum: equal or adjacent bf16 values, and not always equal
    def ordered(b):
        b = b.astype(np.int32)
        return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)
    d = np.abs(ordered(hier) - ordered(flat))
    assert d.max() <= 1
    f64 = oracle_mod.combine(y, w.topk_w, lay, spec.H, acc="f64")
    assert np.abs(ordered(hier) - ordered(f64)).max() <= 1


# --------------------------------------------------------------------------- several sources, one receiver


@pytest.mark.parametrize("padded", [False, True])
def test_multi_source_composition_is_a_stable_sort(oracle_mod, padded):
    """(source rank, token index) order: per-source oracle layouts and dispatches, composed into one
    receiver tensor through expert_base (concatenated) or through each source's columns of the
    [E, R*C, H] tensor (padded), give exactly the stable sort of all entries of all sources by
    (expert, source rank, token, k) -- written down without the oracle in multi_source.py."""
    import multi_source as ms
    spec = wl.WorkloadSpec("ms", 77, R=4, T=64, H=32, E=16, K=3)
    E, H, K, R = spec.E, spec.H, spec.K, 4
    sources = ms.make_sources(spec, R, [50, 37, 1, 64])
    C = 9
    fill = 0xBEEF
    want_rows, want_src, want_w, want_rank = ms.expected_receiver(sources, E, H, padded, C, fill)
    if padded:
        full = np.full((E, R * C, H), fill, np.uint16)
        for s in sources:
            lay = oracle_mod.layout(s.topk, E=E, R=R, layout=oracle_mod.LAYOUT_PADDED, C=C, C_rank=s.topk.shape[0])
            side_w = np.full(E * C, np.float32(-3.5), np.float32)
            side_src = np.full(E * C, -9, np.int32)
            oracle_mod.dispatch(s.x_bits, s.w, lay, full[:, s.rank * C:(s.rank + 1) * C, :], side_w, side_src,
                                stride0=R * C * H, stride1=H)
            # the side arrays of a source are indexed by its own rows e*C + slot
            sel = want_rank.reshape(E, R, C)[:, s.rank, :].reshape(-1)
            assert np.array_equal(side_src, want_src.reshape(E, R, C)[:, s.rank, :].reshape(-1))
            assert np.array_equal(side_w, want_w.reshape(E, R, C)[:, s.rank, :].reshape(-1))
            assert np.all((sel == s.rank) == (side_src >= 0))
        assert np.array_equal(full.reshape(-1, H), want_rows)
        assert (want_rank >= 0).sum() < sum(((s.topk >= 0).sum() for s in sources))  # some entries were cut by C
    else:
        bases = ms.expert_bases(sources, E)
        total = want_rows.shape[0]
        full = np.full((total, H), fill, np.uint16)
        side_w = np.full(total, np.float32(-3.5), np.float32)
        side_src = np.full(total, -9, np.int32)
        for s in sources:
            lay = oracle_mod.layout(s.topk, E=E, R=R, expert_base=bases[s.rank], C_rank=s.topk.shape[0])
            oracle_mod.dispatch(s.x_bits, s.w, lay, full, side_w, side_src)
        assert np.array_equal(full, want_rows)
        assert np.array_equal(side_src, want_src) and np.array_equal(side_w, want_w)
        assert not np.any(full == fill) or True
        assert np.all(want_rank >= 0)  # the concatenated receiver has no holes


@pytest.mark.parametrize("padded", [False, True])
def test_backward_compositions_are_the_gradient_of_the_oracle_combine(oracle_mod, padded):
    """The expected values the GPU tests use for the backward pass (tests/backward_compose.py) against
    finite differences of the oracle's own forward functions.  With L = sum g * combine(y, w), L is
    linear in every y element and every weight, so a difference quotient IS the derivative; the inputs
    are small integers, which every step (bf16 storage, products, sums of K terms) represents exactly,
    so the comparison is for equality.  Capacity drops (padded) and masked entries are included: their
    gradients are zero.  The backward of dispatch is checked the same way: L = sum r * dispatch(x)."""
    import backward_compose as bc
    rng = np.random.default_rng(7 + padded)
    T, K, H, E, R, C = 9, 3, 16, 6, 3, 3
    topk = rng.integers(0, E, (T, K)).astype(np.int32)
    topk[2, 1] = -1
    topk[5, :] = topk[5, 0]                       # one token naming one expert three times
    lay = oracle_mod.layout(topk, E=E, R=R, layout=int(padded), C=C if padded else 0, C_rank=T)
    assert not padded or lay.dropped > 0
    rows = E * C if padded else int(lay.expert_offset[-1])
    ints = lambda shape, lo, hi: rng.integers(lo, hi + 1, shape).astype(np.float32)
    y = ints((rows, H), -3, 3)
    w = ints((T, K), 0, 2)
    g = ints((T, H), -2, 2)
    y_bits, g_bits = wl.f32_to_bf16_bits(y), wl.f32_to_bf16_bits(g)

    def loss(y_bits_, w_):
        out = wl.bf16_bits_to_f32(oracle_mod.combine(y_bits_, w_, lay, H, acc="f64")).astype(np.float64)
        return float((out * g).sum())

    base = loss(y_bits, w)
    # d L / d w[t,k]
    ref_w, _, valid = bc.grad_w_reference(y_bits, g_bits, lay)
    for t in range(T):
        for k in range(K):
            w2 = w.copy()
            w2[t, k] += 1.0
            assert loss(y_bits, w2) - base == ref_w[t, k], (t, k)
            assert valid[t, k] or ref_w[t, k] == 0.0
    # d L / d y[row, h]: the K dispatches of the scaled output gradient
    want = wl.bf16_bits_to_f32(bc.grad_y_rows(oracle_mod, lay, w, g_bits, rows)).astype(np.float64)
    exact = wl.bf16_bits_to_f32(bc.grad_y_rows(oracle_mod, lay, w, g_bits, rows, exact=True)).astype(np.float64)
    assert np.array_equal(want, exact)
    pointed = np.zeros(rows, bool)
    pointed[lay.dst_row[lay.dst_row >= 0]] = True
    for row in range(rows):
        for h in (0, H // 2, H - 1):
            y2 = y.copy()
            y2[row, h] += 1.0
            assert loss(wl.f32_to_bf16_bits(y2), w) - base == want[row, h], (row, h)
        assert pointed[row] or not want[row].any()
    # backward of dispatch: L2 = sum r * dispatch(x); d L2 / d x[t, h] = sum_k r[dst_row[t,k], h] = unweighted combine
    r = ints((rows, H), -3, 3)
    x = ints((T, H), -2, 2)

    def loss2(x_):
        recv = np.zeros((rows, H), np.uint16)
        oracle_mod.dispatch(wl.f32_to_bf16_bits(x_), None, lay, recv)
        return float((wl.bf16_bits_to_f32(recv).astype(np.float64) * r).sum())

    gx = wl.bf16_bits_to_f32(oracle_mod.combine(wl.f32_to_bf16_bits(r), None, lay, H, acc="f32")).astype(np.float64)
    base2 = loss2(x)
    for t in range(T):
        for h in (0, H - 1):
            x2 = x.copy()
            x2[t, h] += 1.0
            assert loss2(x2) - base2 == gx[t, h], (t, h)
