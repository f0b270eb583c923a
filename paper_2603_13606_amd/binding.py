"""ctypes binding of libep_mi355x.so: same names as the C ABI, argument marshalling only.

Torch tensors are used as owners of device memory; each call turns them into
`ep_tensor_t` descriptors (pointer, shape, strides in elements, dtype, tag) and
passes the raw `hipStream_t` of the current torch stream.  No step of the data
path runs here, and there is no fallback: if the shared library is missing the
import of this module's functions raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch  # loaded first on purpose: the library must bind to the HIP runtime torch uses

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libep_mi355x.so")

EP_SUCCESS = 0
EP_ERR_INVALID_ARG = 1
EP_ERR_INVALID_ROUTING = 2
EP_ERR_OVERFLOW = 3
EP_ERR_UNSUPPORTED = 4
EP_ERR_BUSY = 5
EP_ERR_HIP = 6
EP_ERR_NOMEM = 7
EP_ERR_TIMEOUT = 8

EP_MODE_LL, EP_MODE_HT = 0, 1
EP_PATH_DIRECT, EP_PATH_RANK_DEDUP = 0, 1
EP_ORDER_TOKEN, EP_ORDER_DESTINATION, EP_ORDER_DESTINATION_RESIDENT = 0, 1, 2
EP_DTYPE_BF16, EP_DTYPE_F32, EP_DTYPE_I32, EP_DTYPE_U8, EP_DTYPE_FP8_E4M3 = 0, 1, 2, 3, 4

EP_TAG_NONE = 0
EP_TAG_TOKENS = 1
EP_TAG_TOPK_IDX = 2
EP_TAG_TOPK_WEIGHTS = 3
EP_TAG_SCALES = 4
EP_TAG_RECV_EXPERT_COUNTER_DEVICE = 5
EP_TAG_RECV_EXPERT_COUNTER_HOST = 6
EP_TAG_TOKENS_PER_EXPERTS = 7
EP_TAG_RECV_SRC_TOKEN = 8
EP_TAG_EXPERT_BASE = 9
EP_TAG_EXPERT_TOKENS = 10

STATUS_INVALID_IDS, STATUS_CAPACITY_DROP, STATUS_OUTPUT_OVERFLOW, STATUS_TIMEOUT = 1, 2, 4, 8

EXPORTS = [
    "ep_error_string", "ep_version", "ep_build_id", "ep_layout_plan", "ep_dispatch_plan", "ep_combine_plan", "ep_calibration_copy", "ep_calibration_fill", "ep_calibration_read", "ep_group_create", "ep_group_destroy", "ep_group_query",
    "ep_layout", "ep_layout_prefetch", "ep_layout_static", "ep_layout_dispatch", "ep_handle_query", "ep_handle_get_num_recv_tokens", "ep_handle_destroy",
    "ep_dispatch", "ep_combine", "ep_combine_backward", "ep_complete", "ep_group_reset_signals",
]


class ep_tensor_t(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("ndim", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("tag", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("shape", ctypes.c_int64 * 4), ("stride", ctypes.c_int64 * 4)]


class ep_group_config_t(ctypes.Structure):
    _fields_ = [("size", ctypes.c_uint32), ("num_ranks", ctypes.c_int32), ("my_rank", ctypes.c_int32),
                ("num_experts", ctypes.c_int32), ("hidden", ctypes.c_int32), ("top_k", ctypes.c_int32),
                ("max_tokens_per_rank", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("mode", ctypes.c_int32), ("slots_per_subregion", ctypes.c_int32),
                ("dispatch_path", ctypes.c_int32), ("max_handles", ctypes.c_int32),
                ("staged_buffers", ctypes.c_int32), ("ranks_per_node", ctypes.c_int32),
                ("dispatch_order", ctypes.c_int32), ("quantize_ahead", ctypes.c_int32)]


class ep_complete_config_t(ctypes.Structure):
    _fields_ = [("size", ctypes.c_uint32), ("spin_limit", ctypes.c_int32)]


class ep_group_info_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("num_ranks", "my_rank", "num_experts", "experts_per_rank", "hidden", "top_k",
                 "max_tokens_per_rank", "mode", "slots_per_subregion", "dispatch_path")] + [
        ("row_bytes", ctypes.c_int64), ("msg_header_bytes", ctypes.c_int64),
        ("msg_bytes", ctypes.c_int64), ("staging_slots", ctypes.c_int64),
        ("staging", ctypes.c_void_p), ("footprint_per_expert_bytes", ctypes.c_int64),
        ("footprint_optimised_bytes", ctypes.c_int64), ("live_handles", ctypes.c_int32),
        ("staged_buffers", ctypes.c_int32), ("staging_sets", ctypes.c_void_p * 2),
        ("signals", ctypes.c_void_p * 2), ("combine_staging", ctypes.c_void_p * 2),
        ("msg_stride", ctypes.c_int64), ("msg_lead", ctypes.c_int64),
        ("hint_rows_kept", ctypes.c_int32), ("hint_rows_dropped", ctypes.c_int32)]


_INFO_PTRS = ("expert_count", "expert_kept", "expert_offset", "rank_pair_count", "rank_token_count",
              "rank_offset", "slot", "dst_row", "rank_row", "sorted_token", "sorted_k", "sorted_row",
              "entry_rank")


class ep_dispatch_plan_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("run_order", "group", "blocks", "block_entries", "splits", "slice_units", "threads_per_piece",
                 "blocks_per_launch", "launches", "read_passes")]


class ep_combine_plan_t(ctypes.Structure):
    _fields_ = [("segments_per_wavefront", ctypes.c_int32), ("whole_row", ctypes.c_int32), ("workgroups", ctypes.c_int64)]


class ep_layout_info_t(ctypes.Structure):
    _fields_ = [("num_tokens", ctypes.c_int32), ("status", ctypes.c_int32)] + [
        (n, ctypes.c_int64) for n in ("rows_kept", "rows_dropped", "entries_masked", "entries_invalid",
                                      "entries_sorted", "rank_messages", "rows_end")] + [
        (n, ctypes.c_void_p) for n in _INFO_PTRS]


_ARRAY_PTRS = ("totals", "expert_count", "expert_kept", "expert_offset", "rank_pair_count", "rank_token_count",
               "rank_offset", "dst_row", "slot", "rank_row", "entry_rank", "sorted_token", "sorted_k", "sorted_row")


class ep_layout_arrays_t(ctypes.Structure):
    _fields_ = [("size", ctypes.c_uint32), ("reserved", ctypes.c_uint32)] + [(n, ctypes.c_void_p) for n in _ARRAY_PTRS]


ALLOC_FN = ctypes.CFUNCTYPE(ctypes.c_int, ctypes.POINTER(ctypes.c_void_p), ctypes.c_size_t)
FREE_FN = ctypes.CFUNCTYPE(ctypes.c_int, ctypes.c_void_p)

_lib: Optional[ctypes.CDLL] = None


class EpError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {error_string(code)} (code {code})")


def load() -> ctypes.CDLL:
    """Open the shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: run `python -m paper_2603_13606_amd.build` "
                "(or __graft_entry__.build()) first; there is no fallback path")
        lib = ctypes.CDLL(LIB_PATH)
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        lib.ep_error_string.restype = ctypes.c_char_p
        lib.ep_error_string.argtypes = [ctypes.c_int]
        lib.ep_version.restype = i32
        lib.ep_version.argtypes = []
        lib.ep_build_id.restype = ctypes.c_char_p
        lib.ep_build_id.argtypes = []
        lib.ep_group_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(ep_group_config_t), vp, vp, vp]
        lib.ep_group_destroy.argtypes = [vp, vp]
        lib.ep_group_query.argtypes = [vp, ctypes.POINTER(ep_group_info_t)]
        lib.ep_layout.argtypes = [ctypes.POINTER(vp), vp, ctypes.POINTER(ep_tensor_t),
                                  ctypes.POINTER(ep_tensor_t), vp]
        lib.ep_layout_prefetch.argtypes = [ctypes.POINTER(vp), vp, ctypes.POINTER(ep_tensor_t),
                                           ctypes.POINTER(ep_tensor_t), ctypes.POINTER(ep_tensor_t), vp]
        lib.ep_layout_static.argtypes = [ctypes.POINTER(ep_group_config_t), ctypes.POINTER(ep_tensor_t),
                                         ctypes.POINTER(ep_tensor_t), ctypes.POINTER(ep_layout_arrays_t), vp]
        lib.ep_layout_dispatch.argtypes = [ctypes.POINTER(vp), vp, ctypes.POINTER(ep_tensor_t), ctypes.POINTER(ep_tensor_t),
                                           ctypes.POINTER(ep_tensor_t), i32, ctypes.POINTER(ep_tensor_t), i32, vp]
        lib.ep_handle_query.argtypes = [vp, ctypes.POINTER(ep_layout_info_t)]
        lib.ep_handle_get_num_recv_tokens.argtypes = [vp, ctypes.POINTER(ctypes.c_int64)]
        lib.ep_handle_destroy.argtypes = [vp]
        for fn in (lib.ep_dispatch, lib.ep_combine):
            fn.argtypes = [vp, ctypes.POINTER(ep_tensor_t), i32, ctypes.POINTER(ep_tensor_t), i32, i32, vp]
        lib.ep_combine_backward.argtypes = [vp, ctypes.POINTER(ep_tensor_t), i32, ctypes.POINTER(ep_tensor_t), i32, vp]
        lib.ep_calibration_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
        lib.ep_calibration_fill.argtypes = [vp, ctypes.c_size_t, vp]
        lib.ep_calibration_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
        lib.ep_complete.argtypes = [vp, ctypes.POINTER(ep_complete_config_t), vp]
        lib.ep_group_reset_signals.argtypes = [vp, vp]
        lib.ep_layout_plan.argtypes = [ctypes.c_int64, ctypes.POINTER(i32), ctypes.POINTER(i32)]
        lib.ep_dispatch_plan.argtypes = [ctypes.POINTER(ep_group_config_t), ctypes.c_int64, ctypes.c_int64,
                                         ctypes.POINTER(ep_dispatch_plan_t)]
        lib.ep_combine_plan.argtypes = [ctypes.POINTER(ep_group_config_t), ctypes.c_int64, ctypes.c_int32,
                                        ctypes.POINTER(ep_combine_plan_t)]
        for name in EXPORTS[3:]:
            getattr(lib, name).restype = ctypes.c_int
        _lib = lib
    return _lib


def error_string(code: int) -> str:
    return load().ep_error_string(code).decode()


ep_error_string = error_string


def ep_version() -> int:
    return int(load().ep_version())


def ep_build_id() -> str:
    return load().ep_build_id().decode()


def ep_dispatch_plan(cfg: "ep_group_config_t", num_tokens: int, prefetched_rows: int = 0) -> ep_dispatch_plan_t:
    """How ep_dispatch of a group configured like cfg would walk num_tokens tokens (host arithmetic)."""
    plan = ep_dispatch_plan_t()
    _check(load().ep_dispatch_plan(ctypes.byref(cfg), num_tokens, prefetched_rows, ctypes.byref(plan)),
           "ep_dispatch_plan")
    return plan


def ep_layout_plan(num_entries: int):
    """(passes, wave_chunks) ep_layout would use for num_entries = T*K routing entries."""
    p, w = ctypes.c_int32(), ctypes.c_int32()
    _check(load().ep_layout_plan(num_entries, ctypes.byref(p), ctypes.byref(w)), "ep_layout_plan")
    return int(p.value), int(w.value)


def ep_combine_plan(cfg: "ep_group_config_t", num_tokens: int, compute_units: int) -> ep_combine_plan_t:
    """How ep_combine of a group configured like cfg would cut num_tokens tokens into wavefronts (host arithmetic)."""
    plan = ep_combine_plan_t()
    _check(load().ep_combine_plan(ctypes.byref(cfg), num_tokens, compute_units, ctypes.byref(plan)), "ep_combine_plan")
    return plan


def ep_calibration_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes and dst.is_contiguous() and src.is_contiguous()
    _check(load().ep_calibration_copy(dst.data_ptr(), src.data_ptr(), nbytes, _stream_ptr(stream)),
           "ep_calibration_copy")


def ep_calibration_fill(dst: torch.Tensor, stream=None) -> None:
    assert dst.is_contiguous()
    _check(load().ep_calibration_fill(dst.data_ptr(), dst.numel() * dst.element_size(), _stream_ptr(stream)),
           "ep_calibration_fill")


def ep_calibration_read(src: torch.Tensor, sink: torch.Tensor, stream=None) -> None:
    assert src.is_contiguous() and sink.numel() * sink.element_size() >= 4
    _check(load().ep_calibration_read(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(),
                                      _stream_ptr(stream)), "ep_calibration_read")


_DTYPES = {torch.bfloat16: EP_DTYPE_BF16, torch.float32: EP_DTYPE_F32, torch.int32: EP_DTYPE_I32,
           torch.uint8: EP_DTYPE_U8, torch.float8_e4m3fn: EP_DTYPE_FP8_E4M3}


def tensor_desc(t: torch.Tensor, tag: int) -> ep_tensor_t:
    """Describe a torch tensor (device memory owner) as an ep_tensor_t."""
    d = ep_tensor_t()
    d.data = t.data_ptr() if t.numel() > 0 or t.data_ptr() else None
    d.ndim = t.dim()
    d.dtype = _DTYPES[t.dtype]
    d.tag = tag
    for i in range(t.dim()):
        d.shape[i] = t.shape[i]
        d.stride[i] = t.stride(i)
    return d


def _stream_ptr(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream() if torch.cuda.is_available() else 0
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def _check(code: int, where: str, ok: Sequence[int] = (EP_SUCCESS,)) -> int:
    if code not in ok:
        raise EpError(code, where)
    return code


def make_config(num_ranks: int, num_experts: int, hidden: int, top_k: int, max_tokens_per_rank: int,
                mode: int = EP_MODE_HT, my_rank: int = 0, slots_per_subregion: int = 0,
                dispatch_path: int = EP_PATH_DIRECT, max_handles: int = 0,
                dtype: int = EP_DTYPE_BF16, staged_buffers: int = 0, ranks_per_node: int = 0,
                dispatch_order: int = 0, quantize_ahead: int = 0) -> ep_group_config_t:
    c = ep_group_config_t()
    c.size = ctypes.sizeof(ep_group_config_t)
    c.num_ranks, c.my_rank, c.num_experts, c.hidden, c.top_k = num_ranks, my_rank, num_experts, hidden, top_k
    c.max_tokens_per_rank, c.dtype, c.mode = max_tokens_per_rank, dtype, mode
    c.slots_per_subregion, c.dispatch_path, c.max_handles = slots_per_subregion, dispatch_path, max_handles
    c.staged_buffers = staged_buffers
    c.ranks_per_node = ranks_per_node
    c.dispatch_order = dispatch_order
    c.quantize_ahead = quantize_ahead
    return c


def ep_group_create(cfg: ep_group_config_t, stream=None, alloc_fn=None, free_fn=None) -> ctypes.c_void_p:
    g = ctypes.c_void_p()
    a = ctypes.cast(alloc_fn, ctypes.c_void_p) if alloc_fn is not None else None
    f = ctypes.cast(free_fn, ctypes.c_void_p) if free_fn is not None else None
    _check(load().ep_group_create(ctypes.byref(g), ctypes.byref(cfg), _stream_ptr(stream), a, f),
           "ep_group_create")
    return g


def ep_group_destroy(group, stream=None) -> None:
    _check(load().ep_group_destroy(group, _stream_ptr(stream)), "ep_group_destroy")


def ep_group_query(group) -> ep_group_info_t:
    info = ep_group_info_t()
    _check(load().ep_group_query(group, ctypes.byref(info)), "ep_group_query")
    return info


def ep_layout(group, topk_idx: torch.Tensor, expert_base: Optional[torch.Tensor] = None,
              stream=None) -> ctypes.c_void_p:
    h = ctypes.c_void_p()
    td = tensor_desc(topk_idx, EP_TAG_TOPK_IDX)
    bd = ctypes.byref(tensor_desc(expert_base, EP_TAG_EXPERT_BASE)) if expert_base is not None else None
    _check(load().ep_layout(ctypes.byref(h), group, ctypes.byref(td), bd, _stream_ptr(stream)), "ep_layout")
    return h


def ep_layout_prefetch(group, topk_idx: torch.Tensor, tokens: torch.Tensor,
                       expert_base: Optional[torch.Tensor] = None, stream=None) -> ctypes.c_void_p:
    h = ctypes.c_void_p()
    td = tensor_desc(topk_idx, EP_TAG_TOPK_IDX)
    bd = ctypes.byref(tensor_desc(expert_base, EP_TAG_EXPERT_BASE)) if expert_base is not None else None
    xd = tensor_desc(tokens, EP_TAG_TOKENS)
    _check(load().ep_layout_prefetch(ctypes.byref(h), group, ctypes.byref(td), bd, ctypes.byref(xd),
                                     _stream_ptr(stream)), "ep_layout_prefetch")
    return h


def ep_layout_static(cfg: ep_group_config_t, topk_idx: torch.Tensor, arrays: dict,
                     expert_base: Optional[torch.Tensor] = None, stream=None) -> None:
    """ep_layout into int32 tensors of the caller (`arrays`: field name of ep_layout_arrays_t -> tensor)."""
    out = ep_layout_arrays_t()
    out.size = ctypes.sizeof(ep_layout_arrays_t)
    for name, t in arrays.items():
        assert name in _ARRAY_PTRS and t.dtype == torch.int32 and t.is_contiguous()
        setattr(out, name, t.data_ptr())
    td = tensor_desc(topk_idx, EP_TAG_TOPK_IDX)
    bd = ctypes.byref(tensor_desc(expert_base, EP_TAG_EXPERT_BASE)) if expert_base is not None else None
    _check(load().ep_layout_static(ctypes.byref(cfg), ctypes.byref(td), bd, ctypes.byref(out), _stream_ptr(stream)),
           "ep_layout_static")


def ep_handle_query(handle, ok: Sequence[int] = (EP_SUCCESS,)) -> ep_layout_info_t:
    info = ep_layout_info_t()
    info.last_code = _check(load().ep_handle_query(handle, ctypes.byref(info)), "ep_handle_query", ok)
    return info


def ep_handle_get_num_recv_tokens(handle) -> int:
    n = ctypes.c_int64()
    _check(load().ep_handle_get_num_recv_tokens(handle, ctypes.byref(n)), "ep_handle_get_num_recv_tokens")
    return int(n.value)


def ep_handle_destroy(handle) -> None:
    _check(load().ep_handle_destroy(handle), "ep_handle_destroy")


def ep_complete(handle, spin_limit: int = 0, stream=None) -> None:
    cfg = ep_complete_config_t()
    cfg.size = ctypes.sizeof(ep_complete_config_t)
    cfg.spin_limit = spin_limit
    _check(load().ep_complete(handle, ctypes.byref(cfg), _stream_ptr(stream)), "ep_complete")


def ep_group_reset_signals(group, stream=None) -> None:
    _check(load().ep_group_reset_signals(group, _stream_ptr(stream)), "ep_group_reset_signals")


def _descs(pairs) -> "ctypes.Array":
    arr = (ep_tensor_t * max(len(pairs), 1))()
    for i, (t, tag) in enumerate(pairs):
        arr[i] = tensor_desc(t, tag)
    return arr


def _dispatch_tensors(x, recv_x, topk_weights=None, recv_w=None, recv_src=None, recv_count=None, topk_idx=None,
                      recv_scales=None):
    """(inputs, outputs) of a dispatch call as lists of (tensor, tag)."""
    ins = [(x, EP_TAG_TOKENS)]
    if topk_weights is not None:
        ins.append((topk_weights, EP_TAG_TOPK_WEIGHTS))
    if topk_idx is not None:
        ins.append((topk_idx, EP_TAG_TOPK_IDX))
    outs = [(recv_x, EP_TAG_TOKENS)]
    if recv_w is not None:
        outs.append((recv_w, EP_TAG_TOPK_WEIGHTS))
    if recv_src is not None:
        outs.append((recv_src, EP_TAG_RECV_SRC_TOKEN))
    if recv_count is not None:
        outs.append((recv_count, EP_TAG_RECV_EXPERT_COUNTER_DEVICE))
    if recv_scales is not None:
        outs.append((recv_scales, EP_TAG_SCALES))
    return ins, outs


def ep_layout_dispatch(group, topk_idx: torch.Tensor, x: torch.Tensor, recv_x: torch.Tensor,
                       topk_weights: Optional[torch.Tensor] = None, recv_w: Optional[torch.Tensor] = None,
                       recv_src: Optional[torch.Tensor] = None, recv_count: Optional[torch.Tensor] = None,
                       expert_base: Optional[torch.Tensor] = None, recv_scales: Optional[torch.Tensor] = None,
                       pass_topk_idx: bool = False, stream=None) -> ctypes.c_void_p:
    """ep_layout + ep_dispatch in one call; returns the handle."""
    h = ctypes.c_void_p()
    td = tensor_desc(topk_idx, EP_TAG_TOPK_IDX)
    bd = ctypes.byref(tensor_desc(expert_base, EP_TAG_EXPERT_BASE)) if expert_base is not None else None
    ins, outs = _dispatch_tensors(x, recv_x, topk_weights, recv_w, recv_src, recv_count,
                                  topk_idx if pass_topk_idx else None, recv_scales)
    _check(load().ep_layout_dispatch(ctypes.byref(h), group, ctypes.byref(td), bd, _descs(ins), len(ins), _descs(outs),
                                     len(outs), _stream_ptr(stream)), "ep_layout_dispatch")
    return h


def ep_dispatch(handle, x: torch.Tensor, recv_x: torch.Tensor, topk_weights: Optional[torch.Tensor] = None,
                recv_w: Optional[torch.Tensor] = None, recv_src: Optional[torch.Tensor] = None,
                recv_count: Optional[torch.Tensor] = None, send_only: int = 0, stream=None,
                topk_idx: Optional[torch.Tensor] = None, recv_scales: Optional[torch.Tensor] = None) -> None:
    ins, outs = _dispatch_tensors(x, recv_x, topk_weights, recv_w, recv_src, recv_count, topk_idx, recv_scales)
    _check(load().ep_dispatch(handle, _descs(ins), len(ins), _descs(outs), len(outs), send_only,
                              _stream_ptr(stream)), "ep_dispatch")


def ep_combine(handle, y: torch.Tensor, out: torch.Tensor, topk_weights: Optional[torch.Tensor] = None,
               send_only: int = 0, stream=None) -> None:
    ins = [(y, EP_TAG_TOKENS)]
    if topk_weights is not None:
        ins.append((topk_weights, EP_TAG_TOPK_WEIGHTS))
    outs = [(out, EP_TAG_TOKENS)]
    _check(load().ep_combine(handle, _descs(ins), len(ins), _descs(outs), len(outs), send_only,
                             _stream_ptr(stream)), "ep_combine")


def ep_combine_backward(handle, grad_out: torch.Tensor, grad_y: torch.Tensor, topk_weights: Optional[torch.Tensor] = None,
                        y: Optional[torch.Tensor] = None, grad_w: Optional[torch.Tensor] = None, stream=None) -> None:
    """Backward of the weighted combine: grad_y (windows) and, when y is given, grad_w [T, K]."""
    ins = [(grad_out, EP_TAG_TOKENS)]
    if topk_weights is not None:
        ins.append((topk_weights, EP_TAG_TOPK_WEIGHTS))
    if y is not None:
        ins.append((y, EP_TAG_EXPERT_TOKENS))
    outs = [(grad_y, EP_TAG_TOKENS)]
    if grad_w is not None:
        outs.append((grad_w, EP_TAG_TOPK_WEIGHTS))
    _check(load().ep_combine_backward(handle, _descs(ins), len(ins), _descs(outs), len(outs), _stream_ptr(stream)),
           "ep_combine_backward")


class PreparedCall:
    """Descriptors of one ep_dispatch / ep_combine call built once and reused: the
    per-call cost drops to a single foreign-function call.  The tensors must stay
    alive and keep their shapes; only the handle and the stream change per call."""

    def __init__(self, fn_name: str, ins, outs, send_only: int = 0):
        self._fn = getattr(load(), fn_name)
        self._name = fn_name
        self._keep = [t for t, _ in ins] + [t for t, _ in outs]
        self._ins, self._n_in = _descs(ins), len(ins)
        self._outs, self._n_out = _descs(outs), len(outs)
        self._send_only = send_only

    def __call__(self, handle, stream_ptr: int = 0) -> None:
        if self._name == "ep_combine_backward":  # the one call of this shape without a send_only argument
            code = self._fn(handle, self._ins, self._n_in, self._outs, self._n_out, stream_ptr)
        else:
            code = self._fn(handle, self._ins, self._n_in, self._outs, self._n_out, self._send_only, stream_ptr)
        if code != EP_SUCCESS:
            raise EpError(code, self._name)


def prepare_dispatch(x, recv_x, topk_weights=None, recv_w=None, recv_src=None, recv_count=None,
                     topk_idx=None, recv_scales=None) -> PreparedCall:
    ins, outs = _dispatch_tensors(x, recv_x, topk_weights, recv_w, recv_src, recv_count, topk_idx, recv_scales)
    return PreparedCall("ep_dispatch", ins, outs)


class PreparedLayoutDispatch:
    """ep_layout_dispatch with its descriptors built once; calling it returns the handle."""

    def __init__(self, group, topk_idx, x, recv_x, topk_weights=None, recv_w=None, recv_src=None, recv_count=None,
                 expert_base=None):
        self._fn = load().ep_layout_dispatch
        self._group = group
        ins, outs = _dispatch_tensors(x, recv_x, topk_weights, recv_w, recv_src, recv_count)
        self._keep = [topk_idx, expert_base] + [t for t, _ in ins] + [t for t, _ in outs]
        self._td = tensor_desc(topk_idx, EP_TAG_TOPK_IDX)
        self._bd = tensor_desc(expert_base, EP_TAG_EXPERT_BASE) if expert_base is not None else None
        self._ins, self._n_in = _descs(ins), len(ins)
        self._outs, self._n_out = _descs(outs), len(outs)

    def __call__(self, stream_ptr: int = 0) -> ctypes.c_void_p:
        h = ctypes.c_void_p()
        code = self._fn(ctypes.byref(h), self._group, ctypes.byref(self._td),
                        ctypes.byref(self._bd) if self._bd is not None else None, self._ins, self._n_in,
                        self._outs, self._n_out, stream_ptr)
        if code != EP_SUCCESS:
            raise EpError(code, "ep_layout_dispatch")
        return h


def prepare_combine(y, out, topk_weights=None) -> PreparedCall:
    ins = [(y, EP_TAG_TOKENS)]
    if topk_weights is not None:
        ins.append((topk_weights, EP_TAG_TOPK_WEIGHTS))
    return PreparedCall("ep_combine", ins, [(out, EP_TAG_TOKENS)])


def prepare_combine_backward(grad_out, grad_y, topk_weights=None, y=None, grad_w=None) -> PreparedCall:
    ins = [(grad_out, EP_TAG_TOKENS)]
    if topk_weights is not None:
        ins.append((topk_weights, EP_TAG_TOPK_WEIGHTS))
    if y is not None:
        ins.append((y, EP_TAG_EXPERT_TOKENS))
    outs = [(grad_y, EP_TAG_TOKENS)]
    if grad_w is not None:
        outs.append((grad_w, EP_TAG_TOPK_WEIGHTS))
    return PreparedCall("ep_combine_backward", ins, outs)


class PreparedLayout:
    """ep_layout (ep_layout_prefetch when tokens are given) with its descriptors built once."""

    def __init__(self, group, topk_idx, expert_base=None, tokens=None):
        self._fn = load().ep_layout_prefetch
        self._group = group
        self._keep = (topk_idx, expert_base, tokens)
        self._td = tensor_desc(topk_idx, EP_TAG_TOPK_IDX)
        self._bd = tensor_desc(expert_base, EP_TAG_EXPERT_BASE) if expert_base is not None else None
        self._xd = tensor_desc(tokens, EP_TAG_TOKENS) if tokens is not None else None

    def __call__(self, stream_ptr: int = 0) -> ctypes.c_void_p:
        h = ctypes.c_void_p()
        code = self._fn(ctypes.byref(h), self._group, ctypes.byref(self._td),
                        ctypes.byref(self._bd) if self._bd is not None else None,
                        ctypes.byref(self._xd) if self._xd is not None else None, stream_ptr)
        if code != EP_SUCCESS:
            raise EpError(code, "ep_layout")
        return h


def read_device_i32(ptr: int, n: int) -> torch.Tensor:
    """Copy n int32 from a borrowed device pointer (as returned by ep_handle_query) to the host."""
    out = torch.empty(max(n, 0), dtype=torch.int32)
    if n > 0:
        hip = _hip_runtime()
        rc = hip.hipMemcpy(ctypes.c_void_p(out.data_ptr()), ctypes.c_void_p(ptr),
                           ctypes.c_size_t(4 * n), ctypes.c_int(2))  # 2 = device to host
        if rc != 0:
            raise RuntimeError(f"hipMemcpy failed with {rc}")
    return out


_hip = None


def _hip_runtime():
    global _hip
    if _hip is None:
        tl = os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")
        _hip = ctypes.CDLL(tl if os.path.exists(tl) else "libamdhip64.so")
        _hip.hipMemcpy.restype = ctypes.c_int
    return _hip
