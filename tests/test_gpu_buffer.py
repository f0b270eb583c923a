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


@pytest.mark.parametrize("mode", ["ht", "ll"])
def test_buffer_autograd_reuses_handle(hx, mode):
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
        dst_row = buf.routing_rows(h)
        recv = EPDispatchFn.apply(x, buf, h)
        if mode == "ll":
            row_scale = scale[:, None, None].expand(spec.E, spec.T, 1)
        else:
            counts = torch.bincount(topk.reshape(-1).long(), minlength=spec.E)
            row_scale = torch.repeat_interleave(scale, counts)[:, None]
        y = (recv.float() * row_scale).to(torch.bfloat16)   # stand-in experts
        out = EPCombineFn.apply(y, gate, buf, h, dst_row)
        G = torch.randn(spec.T, spec.H, device=hx.DEV, generator=torch.Generator(hx.DEV).manual_seed(3))
        (out.float() * G).sum().backward()
        torch.cuda.synchronize()
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
        assert torch.allclose(gate.grad.double(), gw_ref, rtol=2 ** -5, atol=0.5)
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
