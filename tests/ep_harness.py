"""Glue shared by the GPU parity tests, the smoke check and the benchmark: moves
seeded inputs to the device, calls the HIP path through the C-ABI binding and
brings results back as numpy arrays.  Holds no arithmetic of the method; the
only computation here is the stand-in expert network (y = x * scale[e], rounded
to bf16), which is harness, not library."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np
import torch

from paper_2603_13606_amd import binding as ep
from paper_2603_13606_amd import workloads as wl

def ensure_built() -> None:
    """Build the HIP library unless the one in the tree was built from the sources in the
    tree (harness convenience; the binding itself never builds and never falls back).  Must
    run before the library is first loaded: a loaded library cannot be replaced."""
    from paper_2603_13606_amd import build
    if not build.is_current():
        build.build()
    ep.load()
    assert ep.ep_build_id() == build.source_id(), "the loaded library does not match the sources"


DEV = "cuda:0"
POISON = 0x4B4B  # a finite bf16 bit pattern (about 1.3e7) no seeded input contains


def bits_to_dev(bits: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bit patterns -> bf16 tensor on the GPU (bit-preserving)."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(DEV).view(torch.bfloat16)


def dev_to_bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def poison_bf16(shape, value: int = POISON) -> torch.Tensor:
    """A bf16 tensor filled with a recognisable bit pattern."""
    t = torch.empty(shape, dtype=torch.int16, device=DEV)
    t.fill_(np.array(value, np.uint16).view(np.int16).item())
    return t.view(torch.bfloat16)


@dataclass
class GpuLayout:
    info: object
    arrays: Dict[str, np.ndarray]


def fetch_layout(handle, T: int, K: int, E: int, R: int, ok=(ep.EP_SUCCESS,)) -> GpuLayout:
    info = ep.ep_handle_query(handle, ok=ok)
    n = T * K
    sizes = dict(expert_count=E, expert_kept=E, expert_offset=E + 1, rank_pair_count=R,
                 rank_token_count=R, rank_offset=R + 1, slot=n, dst_row=n, rank_row=n, entry_rank=n,
                 sorted_token=int(info.entries_sorted), sorted_k=int(info.entries_sorted),
                 sorted_row=int(info.entries_sorted))
    arrays = {k: ep.read_device_i32(getattr(info, k), v).numpy() for k, v in sizes.items()}
    for k in ("slot", "dst_row", "rank_row", "entry_rank"):
        arrays[k] = arrays[k].reshape(T, K)
    return GpuLayout(info=info, arrays=arrays)


def assert_layout_equal(g: GpuLayout, o) -> None:
    """Bit-exact comparison of every array of the layout with the oracle's."""
    a = g.arrays
    for name in ("expert_count", "expert_kept", "expert_offset", "rank_pair_count", "rank_token_count",
                 "rank_offset", "slot", "dst_row", "rank_row"):
        want = getattr(o, name)
        assert np.array_equal(a[name], want), f"{name} differs"
    ns = o.n_sorted
    assert int(g.info.entries_sorted) == ns
    for name in ("sorted_token", "sorted_k", "sorted_row"):
        assert np.array_equal(a[name], getattr(o, name)[:ns]), f"{name} differs"
    i = g.info
    assert (int(i.rows_kept), int(i.rows_dropped), int(i.entries_masked), int(i.entries_invalid),
            int(i.rank_messages), int(i.rows_end)) == (o.kept, o.dropped, o.masked, o.invalid, o.n_msgs,
                                                       int(o.expert_offset[-1]))


def expert_standin(recv_x: torch.Tensor, row_expert: torch.Tensor, scale: np.ndarray) -> torch.Tensor:
    """Stand-in expert network on the GPU: y[row] = bf16(f32(x[row]) * scale[expert of row])."""
    s = torch.from_numpy(scale).to(recv_x.device)[row_expert.long()]
    return (recv_x.float() * s[:, None]).to(torch.bfloat16)


def expert_standin_np(recv_bits: np.ndarray, row_expert: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """Same stand-in on the host for the oracle side."""
    out = np.empty_like(recv_bits)
    step = 4096
    for r0 in range(0, recv_bits.shape[0], step):
        r1 = min(recv_bits.shape[0], r0 + step)
        f = wl.bf16_bits_to_f32(recv_bits[r0:r1]) * scale[row_expert[r0:r1]][:, None]
        out[r0:r1] = wl.f32_to_bf16_bits(f.astype(np.float32))
    return out


def bf16_ulp_distance(a_bits: np.ndarray, b_bits: np.ndarray) -> np.ndarray:
    """Distance in representable bf16 values between two arrays of bit patterns."""
    def ordered(b):
        b = b.astype(np.int32)
        return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)
    return np.abs(ordered(a_bits) - ordered(b_bits))


def combine_tolerance_ok(got_bits: np.ndarray, ref_bits: np.ndarray):
    """The acceptance rule for combine: every element within 1e-2 absolute or 4e-3
    relative of the oracle that accumulates as the target statement prescribes
    (float32, k ascending)."""
    got = wl.bf16_bits_to_f32(got_bits).astype(np.float64)
    ref = wl.bf16_bits_to_f32(ref_bits).astype(np.float64)
    both_nan = np.isnan(got) & np.isnan(ref)
    diff = np.abs(got - ref)
    ok = both_nan | (diff <= 1e-2) | (diff <= 4e-3 * np.abs(ref)) | ((got == ref))
    return bool(ok.all()), float(np.nanmax(np.where(both_nan, 0, diff))) if diff.size else 0.0
