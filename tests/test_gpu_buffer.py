"""The framework-facing buffer (dispatch / combine / counters / autograd reuse of one
handle) against the oracle and a dense float64 reference."""
import numpy as np
import pytest
import torch

from paper_2603_13606_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hx():
    import ep_harness
    ep_harness.ensure_built()
    assert torch.cuda.is_available()
    return ep_harness


def test_buffer_forward_matches_oracle_and_counts(hx, oracle_mod):
    from paper_2603_13606_amd.buffer import EPBuffer
    w = wl.make_workload("ll_decode", T=100, H=512)
    spec = w.spec
    lay = oracle_mod.layout(w.topk_idx, E=spec.E, R=spec.R, C_rank=128)
    buf = EPBuffer(spec.R, spec.E, spec.H, spec.K, max_tokens_per_rank=128, mode="ht")
    try:
        x = hx.bits_to_dev(w.x_bits)
        topk = torch.from_numpy(w.topk_idx).to(hx.DEV)
        gate = torch.from_numpy(w.topk_w).to(hx.DEV)
        recv_x, recv_src, recv_w, h, ev = buf.dispatch(x, topk, gate, previous_event=buf.capture())
        assert buf.get_tokens_per_expert_list() == lay.expert_count.tolist()
        rows = buf.get_num_recv_tokens(h)
        assert rows == lay.kept
        o_recv = np.zeros((rows, spec.H), np.uint16)
        o_w = np.zeros(rows, np.float32)
        o_src = np.zeros(rows, np.int32)
        oracle_mod.dispatch(w.x_bits, w.topk_w, lay, o_recv, o_w, o_src)
        assert np.array_equal(hx.dev_to_bits(recv_x[:rows]), o_recv)
        assert np.array_equal(recv_src[:rows].cpu().numpy(), o_src)
        assert np.array_equal(recv_w[:rows].cpu().numpy(), o_w)
        assert np.array_equal(buf.routing_rows(h).cpu().numpy(), lay.dst_row)
        out, _ = buf.combine(recv_x, h, gate)
        torch.cuda.synchronize()
        assert np.array_equal(hx.dev_to_bits(out), oracle_mod.combine(o_recv, w.topk_w, lay, spec.H, acc="f32"))
        # cached dispatch with the same handle (backward pass), FP8 output
        (q, sc), _, _, h2, _ = buf.dispatch(x, handle=h, fp8=True)
        assert h2 is h
        o_q = np.zeros((rows, spec.H), np.uint8)
        o_s = np.zeros((rows, spec.H // 128), np.float32)
        oracle_mod.dispatch_fp8(w.x_bits, lay, o_q, o_s)
        torch.cuda.synchronize()
        assert np.array_equal(q[:rows].view(torch.uint8).cpu().numpy(), o_q)
        assert np.array_equal(sc[:rows].cpu().numpy(), o_s)
        buf.destroy_handle(h)
    finally:
        buf.close()


@pytest.mark.parametrize("name,T,H,mode,C,order", [
    ("tiny", None, None, "ht", 0, 0), ("tiny", None, None, "ll", 6, 0),
    ("ll_decode", 100, 1000, "ht", 0, 0), ("skew", 700, 512, "ll", 30, 0),
    ("ht_prefill", 1500, 7168, "ht", 0, 0),
    # groups in destination order, inputs of 8192 entries and more: the backward kernel walks the rows as they lie
    ("ht_prefill", 1500, 7168, "ht", 0, 1),
    ("skew", 1100, 520, "ll", 30, 1),          # padded windows, most entries cut by the capacity, 65 units per row
    ("skew", 1100, 512, "ll", 1100, 2),        # padded, nothing cut
    ("ll_decode", 1030, 64, "ht", 0, 1),       # rows of 8 units: one wave, most lanes idle
    ("ll_decode", 300, 256, "ht", 0, 1),       # too small for the row order: token walk
])
def test_backward_calls_match_the_oracle_composition(hx, oracle_mod, name, T, H, mode, C, order):
    """The backward pass with the handle of the forward pass, piece by piece against oracle calls:
    grad_x (backward of dispatch) = unweighted oracle.combine of the row gradients, bit-exact;
    grad_y (backward of combine) = oracle.dispatch, entry by entry, of the output gradient scaled by
    the entry's gate weight -- bit-exact with the float32 product, within one bf16 ulp of the
    float64 one; grad_w = row dot products, within the float32 summation bound of the float64 sums
    (far inside 1e-3 relative wherever the terms do not cancel)."""
    import backward_compose as bc
    from paper_2603_13606_amd.buffer import EPBuffer
    w = wl.make_workload(name, T=T, **({"H": H} if H else {}))
    spec = w.spec
    T, K, Hh = spec.T, spec.K, spec.H
    ll = mode == "ll"
    Cc = (C if C else T) if ll else 0
    topk = w.topk_idx.copy()
    topk[::11, 0] = -1
    lay = oracle_mod.layout(topk, E=spec.E, R=spec.R, layout=int(ll), C=Cc, C_rank=T)
    rows = spec.E * Cc if ll else T * K
    buf = EPBuffer(spec.R, spec.E, Hh, K, max_tokens_per_rank=T, mode=mode, slots_per_subregion=C, dispatch_order=order)
    try:
        rng = np.random.default_rng(T + Hh)
        d_topk = torch.from_numpy(topk).to(hx.DEV)
        gate = torch.from_numpy(w.topk_w).to(hx.DEV)
        x = hx.bits_to_dev(w.x_bits)
        _, _, _, h, _ = buf.dispatch(x, d_topk)
        # stand-in expert outputs and an output gradient, both arbitrary bf16 data
        y_bits = wl.f32_to_bf16_bits(rng.standard_normal((rows, Hh)).astype(np.float32))
        g_bits = wl.f32_to_bf16_bits(rng.standard_normal((T, Hh)).astype(np.float32))
        y = hx.bits_to_dev(y_bits)
        y = y.view(spec.E, Cc, Hh) if ll else y
        g = hx.bits_to_dev(g_bits)
        grad_y, grad_w, _ = buf.combine_backward(g, h, gate, y)
        torch.cuda.synchronize()
        want32 = bc.grad_y_rows(oracle_mod, lay, w.topk_w, g_bits, rows)
        want64 = bc.grad_y_rows(oracle_mod, lay, w.topk_w, g_bits, rows, exact=True)
        got_gy = hx.dev_to_bits(grad_y.reshape(rows, Hh))
        assert np.array_equal(got_gy, want32), "grad_y differs from the dispatched, scaled gradient"
        assert hx.bf16_ulp_distance(got_gy, want64).max() <= 1
        ref_w, mag, valid = bc.grad_w_reference(y_bits, g_bits, lay)
        bound = mag * 64 * 2.0 ** -24 + 1e-30
        got_w = grad_w.cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got_w - ref_w) <= np.where(valid, bound, 0.0)), "grad_w outside the float32 summation bound"
        big = valid & (np.abs(ref_w) > 0.05 * mag)
        assert np.all(np.abs(got_w - ref_w)[big] <= 1e-3 * np.abs(ref_w)[big])
        assert np.all(got_w[~valid] == 0.0)
        # backward of dispatch: the row gradients summed per token, no weights
        r_bits = wl.f32_to_bf16_bits(rng.standard_normal((rows, Hh)).astype(np.float32))
        gr = hx.bits_to_dev(r_bits)
        gx, _ = buf.combine(gr.view(spec.E, Cc, Hh) if ll else gr, h)
        torch.cuda.synchronize()
        assert np.array_equal(hx.dev_to_bits(gx), oracle_mod.combine(r_bits, None, lay, Hh, acc="f32"))
        # without the expert outputs only grad_y is produced; y without grad_w is refused
        gy2, gw2, _ = buf.combine_backward(g, h, gate)
        torch.cuda.synchronize()
        assert gw2 is None and np.array_equal(hx.dev_to_bits(gy2.reshape(rows, Hh)), want32)
        from paper_2603_13606_amd import binding as ep
        with pytest.raises(ep.EpError):
            ep.ep_combine_backward(h.raw, g, grad_y, topk_weights=gate, y=y)
        buf.destroy_handle(h)
    finally:
        buf.close()


@pytest.mark.parametrize("mode", ["ht", "ll"])
def test_buffer_autograd_reuses_handle(hx, oracle_mod, mode):
    """One handle through forward and backward of the autograd wrappers: the gradients that come
    out are the composition of the backward calls checked above with the stand-in experts'
    own backward (torch), compared bit for bit with that composition run by hand on the GPU
    tensors, and with a dense float64 reference at the precision bf16 intermediates allow."""
    from paper_2603_13606_amd.buffer import EPBuffer, EPCombineFn, EPDispatchFn
    w = wl.make_workload("tiny")
    spec = w.spec
    buf = EPBuffer(spec.R, spec.E, spec.H, spec.K, max_tokens_per_rank=spec.T, mode=mode)
    try:
        topk = torch.from_numpy(w.topk_idx).to(hx.DEV)
        x = hx.bits_to_dev(w.x_bits).requires_grad_(True)
        gate = torch.from_numpy(w.topk_w).to(hx.DEV).requires_grad_(True)
        scale = (1.0 + torch.arange(spec.E, device=hx.DEV, dtype=torch.float32) / 8.0)
        # forward: handle created by a first dispatch, then reused by the autograd functions
        _, _, _, h, _ = buf.dispatch(x.detach(), topk)
        recv = EPDispatchFn.apply(x, buf, h)
        if mode == "ll":
            row_scale = scale[:, None, None].expand(spec.E, spec.T, 1)
        else:
            counts = torch.bincount(topk.reshape(-1).long(), minlength=spec.E)
            row_scale = torch.repeat_interleave(scale, counts)[:, None]
        y = (recv.float() * row_scale).to(torch.bfloat16)   # stand-in experts
        y.retain_grad()
        out = EPCombineFn.apply(y, gate, buf, h)
        G = torch.randn(spec.T, spec.H, device=hx.DEV, generator=torch.Generator(hx.DEV).manual_seed(3)).bfloat16()
        (out.float() * G.float()).sum().backward()
        torch.cuda.synchronize()
        # the same backward by hand: combine_backward, the experts' backward, unweighted combine
        gy, gw, _ = buf.combine_backward(G, h, gate.detach(), y.detach())
        g_recv = (gy.float() * row_scale).to(torch.bfloat16)
        gx, _ = buf.combine(g_recv, h)
        torch.cuda.synchronize()
        assert torch.equal(y.grad, gy) and torch.equal(gate.grad, gw) and torch.equal(x.grad, gx)
        # dense float64 reference
        xd = x.detach().double()
        wd = gate.detach().double()
        s = scale.double()[topk.long()]                      # [T, K]
        coef = (wd * s).sum(1)                               # [T]
        out_ref = xd * coef[:, None]
        assert torch.allclose(out.detach().double(), out_ref, rtol=2 ** -6, atol=1e-6)
        gx_ref = G.double() * coef[:, None]
        gw_ref = s * (xd * G.double()).sum(1)[:, None]
        assert torch.allclose(x.grad.double(), gx_ref, rtol=2 ** -5, atol=2e-2)
        # y is x * s rounded to bf16 (relative error 2^-9 per element): the dot products inherit it
        mag = s * (xd.abs() * G.double().abs()).sum(1)[:, None]
        assert torch.all((gate.grad.double() - gw_ref).abs() <= 2 ** -8 * mag + 1e-6)
        buf.destroy_handle(h)
    finally:
        buf.close()


def test_buffer_destination_order_gives_the_same_tensors(hx):
    """A buffer configured for the destination order (its dispatch announces the tokens to the
    layout call) returns bit for bit what the default buffer returns."""
    from paper_2603_13606_amd import binding as ep
    from paper_2603_13606_amd.buffer import EPBuffer
    w = wl.make_workload("ll_decode", T=1100, H=512)
    spec = w.spec
    topk = torch.from_numpy(w.topk_idx).to(hx.DEV)
    x = hx.bits_to_dev(w.x_bits)
    gate = torch.from_numpy(w.topk_w).to(hx.DEV)
    got = []
    for order in (ep.EP_ORDER_TOKEN, ep.EP_ORDER_DESTINATION):
        buf = EPBuffer(spec.R, spec.E, spec.H, spec.K, max_tokens_per_rank=spec.T, mode="ht", dispatch_order=order)
        try:
            recv_x, recv_src, recv_w, h, _ = buf.dispatch(x, topk, gate)
            n = sum(buf.get_tokens_per_expert_list())
            out, _ = buf.combine(recv_x, h, gate)
            torch.cuda.synchronize()
            got.append((hx.dev_to_bits(recv_x[:n]), recv_src[:n].cpu().numpy(), recv_w[:n].cpu().numpy(),
                        hx.dev_to_bits(out), n))
            buf.destroy_handle(h)
        finally:
            buf.close()
    assert got[0][4] == got[1][4] == spec.T * spec.K
    for a, b in zip(got[0][:4], got[1][:4]):
        assert np.array_equal(a, b)
