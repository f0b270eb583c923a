"""Framework-facing buffer over the C ABI (Sec. VI-A "Common Backend Architecture",
Table V "Buffer operations"): `dispatch`, `combine`, `get_tokens_per_expert_list`,
`get_comm_stream`, `capture`, `destroy_handle`, `combine_backward`, plus autograd wrappers that reuse one
handle for the forward and the backward pass (Sec. III-F training pattern, Sec. VI-B).

What it adds to the binding is resource plumbing only, as the paper describes it:
  - the group's allocations go through torch's caching allocator (allocator
    callbacks, pointers kept in a map; Sec. VI-A "Memory and streams");
  - a dedicated communication stream; it waits for the compute stream before each
    call and the compute stream waits for the returned event (the paper's
    synchronous scheme);
  - per-expert counts land in pinned, device-mapped host memory, so reading them needs
    an event wait but no device-to-host copy (Sec. VI-A "Expert counts").
Every data-path step still runs in the library's kernels.
"""
from __future__ import annotations

import ctypes
from typing import List, Optional, Tuple

import torch

from . import binding as ep


class EPHandle:
    """One routing decision (Sec. III-C "MoE Handle"): the C handle plus what is needed to
    size outputs and to run the backward pass."""

    def __init__(self, raw, topk_idx: torch.Tensor, num_tokens: int):
        self.raw = raw
        self.topk_idx = topk_idx
        self.num_tokens = num_tokens
        self.alive = True


class EPBuffer:
    def __init__(self, num_ranks: int, num_experts: int, hidden: int, top_k: int,
                 max_tokens_per_rank: int, mode: str = "ht", my_rank: int = 0,
                 slots_per_subregion: int = 0, dispatch_path: str = "direct", max_handles: int = 4,
                 device: str = "cuda:0", dispatch_order: int = ep.EP_ORDER_TOKEN, quantize_ahead: bool = False):
        ep.load()
        self.device = torch.device(device)
        self.R, self.E, self.H, self.K, self.B = num_ranks, num_experts, hidden, top_k, max_tokens_per_rank
        self.ll = mode == "ll"
        self.C = (slots_per_subregion or max_tokens_per_rank) if self.ll else 0
        self._held = {}

        def _alloc(pp, nbytes):
            t = torch.empty(int(nbytes), dtype=torch.uint8, device=self.device)
            self._held[t.data_ptr()] = t
            pp[0] = t.data_ptr()
            return 0

        def _free(p):
            return 0 if self._held.pop(p, None) is not None else 1

        self._alloc_cb, self._free_cb = ep.ALLOC_FN(_alloc), ep.FREE_FN(_free)
        cfg = ep.make_config(num_ranks, num_experts, hidden, top_k, max_tokens_per_rank,
                             mode=ep.EP_MODE_LL if self.ll else ep.EP_MODE_HT, my_rank=my_rank,
                             slots_per_subregion=slots_per_subregion,
                             dispatch_path=ep.EP_PATH_RANK_DEDUP if dispatch_path == "once_per_rank" else ep.EP_PATH_DIRECT,
                             max_handles=max_handles, dispatch_order=dispatch_order, quantize_ahead=int(quantize_ahead))
        self._dedup = dispatch_path == "once_per_rank"
        with torch.cuda.device(self.device):
            self.group = ep.ep_group_create(cfg, alloc_fn=self._alloc_cb, free_fn=self._free_cb)
            self.comm_stream = torch.cuda.Stream()
        # pinned host memory, written by the dispatch kernel through its device mapping
        self.recv_expert_counter = torch.zeros(num_experts, dtype=torch.int32, pin_memory=True)
        self._counter_dev_ptr = _device_pointer_of_pinned(self.recv_expert_counter)
        self._last_event: Optional[torch.cuda.Event] = None

    # ------------------------------------------------------------------ streams and events
    def get_comm_stream(self) -> torch.cuda.Stream:
        return self.comm_stream

    def capture(self) -> torch.cuda.Event:
        """An event on the compute stream, as the callers pass between layers."""
        ev = torch.cuda.Event()
        ev.record(torch.cuda.current_stream())
        return ev

    def _enter(self, previous_event: Optional[torch.cuda.Event]):
        if previous_event is not None:
            self.comm_stream.wait_event(previous_event)
        else:
            self.comm_stream.wait_stream(torch.cuda.current_stream())

    def _leave(self) -> torch.cuda.Event:
        ev = torch.cuda.Event()
        ev.record(self.comm_stream)
        torch.cuda.current_stream().wait_event(ev)  # compute waits for communication
        self._last_event = ev
        return ev

    # ------------------------------------------------------------------ operations
    def dispatch(self, x: torch.Tensor, topk_idx: Optional[torch.Tensor] = None,
                 topk_weights: Optional[torch.Tensor] = None, handle: Optional[EPHandle] = None,
                 previous_event: Optional[torch.cuda.Event] = None, fp8: bool = False):
        """recv_x, recv_src, recv_w, handle, event = dispatch(x, topk_idx, topk_weights, handle).

        With `handle` given this is the cached dispatch of the backward pass: the routing of
        the forward pass is reused.  HT mode returns [T*K, H] storage (rows beyond the
        handle's count are unused); LL mode returns [E, C, H].  With fp8=True recv_x is a
        pair (codes float8_e4m3fn, scales float32 [rows, H/128])."""
        T = x.shape[0]
        self._enter(previous_event)
        sp = self.comm_stream.cuda_stream
        with torch.cuda.stream(self.comm_stream):
            if handle is None:
                assert topk_idx is not None
                # the tokens are about to be dispatched: let the layout launch read them ahead
                # (only a destination-ordered group makes use of the hint)
                raw = ep.ep_layout_prefetch(self.group, topk_idx, x, stream=sp)
                handle = EPHandle(raw, topk_idx, T)
            rows = self.E * self.C if self.ll else T * self.K
            dt = torch.float8_e4m3fn if fp8 else torch.bfloat16
            store = torch.empty((rows, self.H), dtype=dt, device=self.device)
            recv_x = store.view(self.E, self.C, self.H) if self.ll else store
            recv_w = torch.empty(rows, dtype=torch.float32, device=self.device) if topk_weights is not None else None
            recv_src = torch.empty(rows, dtype=torch.int32, device=self.device)
            scales = torch.empty((rows, self.H // 128), dtype=torch.float32, device=self.device) if fp8 else None
            counter = _as_tensor_desc_override(self.recv_expert_counter, self._counter_dev_ptr)
            _dispatch_with_counter(handle.raw, x, recv_x, topk_weights, recv_w, recv_src, counter, scales,
                                   handle.topk_idx if self._dedup else None, sp)
            for t in (x, recv_x, recv_src) + ((topk_weights, recv_w) if topk_weights is not None else ()):
                t.record_stream(self.comm_stream)
        ev = self._leave()
        return ((recv_x, scales) if fp8 else recv_x), recv_src, recv_w, handle, ev

    def combine(self, y: torch.Tensor, handle: EPHandle, topk_weights: Optional[torch.Tensor] = None,
                previous_event: Optional[torch.cuda.Event] = None):
        """out, event = combine(y, handle, topk_weights)."""
        self._enter(previous_event)
        sp = self.comm_stream.cuda_stream
        with torch.cuda.stream(self.comm_stream):
            out = torch.empty((handle.num_tokens, self.H), dtype=torch.bfloat16, device=self.device)
            ep.ep_combine(handle.raw, y, out, topk_weights=topk_weights, stream=sp)
            y.record_stream(self.comm_stream)
            out.record_stream(self.comm_stream)
        return out, self._leave()

    def combine_backward(self, grad_out: torch.Tensor, handle: EPHandle, topk_weights: Optional[torch.Tensor] = None,
                         y: Optional[torch.Tensor] = None, previous_event: Optional[torch.cuda.Event] = None):
        """grad_y, grad_w, event = combine_backward(grad_out, handle, topk_weights, y): the gradient of a
        weighted combine with respect to the expert outputs (windows like y, rows without an entry
        zero) and, when y is given, with respect to the gate weights [T, K]."""
        self._enter(previous_event)
        sp = self.comm_stream.cuda_stream
        with torch.cuda.stream(self.comm_stream):
            if y is not None:
                grad_y = torch.zeros(y.shape, dtype=torch.bfloat16, device=self.device)
            else:
                rows = self.E * self.C if self.ll else handle.num_tokens * self.K
                store = torch.zeros((rows, self.H), dtype=torch.bfloat16, device=self.device)
                grad_y = store.view(self.E, self.C, self.H) if self.ll else store
            grad_w = torch.empty((handle.num_tokens, self.K), dtype=torch.float32, device=self.device) if y is not None else None
            ep.ep_combine_backward(handle.raw, grad_out, grad_y, topk_weights=topk_weights, y=y, grad_w=grad_w, stream=sp)
            for t in (grad_out, grad_y) + ((y, grad_w) if y is not None else ()):
                t.record_stream(self.comm_stream)
        return grad_y, grad_w, self._leave()

    def get_tokens_per_expert_list(self) -> List[int]:
        """Rows placed per expert by the last dispatch, read from the pinned counter."""
        if self._last_event is not None:
            self._last_event.synchronize()
        return self.recv_expert_counter.tolist()

    def routing_rows(self, handle: EPHandle) -> torch.Tensor:
        """dst_row [T, K] of the handle as a device tensor (a copy; -1 = no row)."""
        info = ep.ep_handle_query(handle.raw, ok=(ep.EP_SUCCESS, ep.EP_ERR_INVALID_ROUTING, ep.EP_ERR_OVERFLOW))
        out = torch.empty((handle.num_tokens, self.K), dtype=torch.int32, device=self.device)
        if out.numel():
            hip = ep._hip_runtime()
            rc = hip.hipMemcpy(ctypes.c_void_p(out.data_ptr()), ctypes.c_void_p(info.dst_row),
                               ctypes.c_size_t(4 * out.numel()), ctypes.c_int(3))  # 3 = device to device
            if rc != 0:
                raise RuntimeError(f"hipMemcpy failed with {rc}")
        return out

    def get_num_recv_tokens(self, handle: EPHandle) -> int:
        return ep.ep_handle_get_num_recv_tokens(handle.raw)

    def destroy_handle(self, handle: EPHandle) -> None:
        """Deferred destruction (Sec. VI-B): wait for the last recorded event, then release."""
        if handle.alive:
            if self._last_event is not None:
                self._last_event.synchronize()
            ep.ep_handle_destroy(handle.raw)
            handle.alive = False

    def close(self) -> None:
        if self.group is not None:
            self.comm_stream.synchronize()
            ep.ep_group_destroy(self.group, stream=self.comm_stream.cuda_stream)
            self.group = None
            assert not self._held, "group did not return all its allocations"


def _device_pointer_of_pinned(t: torch.Tensor) -> int:
    """Device address of a pinned host tensor (hipHostGetDevicePointer)."""
    hip = ep._hip_runtime()
    dev = ctypes.c_void_p()
    hip.hipHostGetDevicePointer.restype = ctypes.c_int
    rc = hip.hipHostGetDevicePointer(ctypes.byref(dev), ctypes.c_void_p(t.data_ptr()), ctypes.c_uint(0))
    if rc != 0 or not dev.value:
        raise RuntimeError(f"hipHostGetDevicePointer failed with {rc}")
    return int(dev.value)


def _as_tensor_desc_override(t: torch.Tensor, ptr: int) -> ep.ep_tensor_t:
    d = ep.tensor_desc(t, ep.EP_TAG_RECV_EXPERT_COUNTER_HOST)
    d.data = ptr
    return d


def _dispatch_with_counter(raw, x, recv_x, w, recv_w, recv_src, counter_desc, scales, topk_idx, sp) -> None:
    ins = [ep.tensor_desc(x, ep.EP_TAG_TOKENS)]
    if w is not None:
        ins.append(ep.tensor_desc(w, ep.EP_TAG_TOPK_WEIGHTS))
    if topk_idx is not None:
        ins.append(ep.tensor_desc(topk_idx, ep.EP_TAG_TOPK_IDX))
    outs = [ep.tensor_desc(recv_x, ep.EP_TAG_TOKENS), ep.tensor_desc(recv_src, ep.EP_TAG_RECV_SRC_TOKEN), counter_desc]
    if recv_w is not None:
        outs.append(ep.tensor_desc(recv_w, ep.EP_TAG_TOPK_WEIGHTS))
    if scales is not None:
        outs.append(ep.tensor_desc(scales, ep.EP_TAG_SCALES))
    ia = (ep.ep_tensor_t * len(ins))(*ins)
    oa = (ep.ep_tensor_t * len(outs))(*outs)
    code = ep.load().ep_dispatch(raw, ia, len(ins), oa, len(outs), 0, sp)
    if code != ep.EP_SUCCESS:
        raise ep.EpError(code, "ep_dispatch")


# ---------------------------------------------------------------------- autograd wrappers


class EPDispatchFn(torch.autograd.Function):
    """Forward: dispatch x.  Backward: the gradient of a row copy is the sum of the row
    gradients, i.e. an unweighted combine with the same handle."""

    @staticmethod
    def forward(ctx, x, buf: EPBuffer, handle: EPHandle):
        recv_x, _, _, _, _ = buf.dispatch(x, handle=handle)
        ctx.buf, ctx.handle = buf, handle
        return recv_x

    @staticmethod
    def backward(ctx, grad_recv):
        gx, _ = ctx.buf.combine(grad_recv.contiguous(), ctx.handle)
        return gx, None, None


class EPCombineFn(torch.autograd.Function):
    """Forward: weighted combine.  Backward: one call with the same handle -- the output gradient
    dispatched to the rows of y, each copy scaled by its gate weight, and the weight gradient as
    the dot product of every expert output row with the gradient of its token."""

    @staticmethod
    def forward(ctx, y, topk_weights, buf: EPBuffer, handle: EPHandle):
        out, _ = buf.combine(y, handle, topk_weights)
        ctx.buf, ctx.handle = buf, handle
        ctx.save_for_backward(y, topk_weights)
        return out

    @staticmethod
    def backward(ctx, grad_out):
        y, w = ctx.saved_tensors
        grad_y, grad_w, _ = ctx.buf.combine_backward(grad_out.contiguous(), ctx.handle, w, y)
        return grad_y, grad_w, None, None
