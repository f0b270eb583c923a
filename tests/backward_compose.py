"""Expected values of the backward pass as compositions of oracle calls (test glue).

The backward pass has no oracle function of its own.  With L = sum_{t,h} g[t,h] * out[t,h] and
out = combine(y, w) (Sec. III-B: out[t] = sum_k w[t,k] * y[dst_row[t,k]]) its gradients are

    grad_y[dst_row[t,k], :] = w[t,k] * g[t, :]          rows no entry points at: untouched
    grad_w[t,k]             = sum_h y[dst_row[t,k], h] * g[t,h]     (0 for an entry without a row)
    grad_x[t, :]            = sum_k grad_rows[dst_row[t,k], :]      (dispatch copies, so its backward adds)

`grad_y_rows` writes the first line as K oracle dispatches (one per entry column, of the output
gradient scaled by that column's weights), `grad_w_reference` the second as float64 row dot
products, and the third is oracle.combine without weights.  tests/test_oracle_pins.py checks these
compositions against finite differences of oracle.combine on inputs every step represents exactly
(the loss is linear in y and in w, so the differences are the gradient); the GPU tests compare the
HIP backward kernels with the same functions."""
from __future__ import annotations

import dataclasses

import numpy as np

from paper_2603_13606_amd import workloads as wl


def f64_to_bf16_bits(v: np.ndarray) -> np.ndarray:
    """Round float64 values of normal bf16 magnitude to bf16 in ONE rounding (nearest even)."""
    m, e = np.frexp(v)
    r = np.ldexp(np.rint(m * 256.0), e - 8).astype(np.float32)   # exact: 8 significant bits
    return (r.view(np.uint32) >> 16).astype(np.uint16)


def grad_y_rows(oracle_mod, lay, w: np.ndarray, g_bits: np.ndarray, rows: int, fill: int = 0, exact: bool = False):
    """[rows, H] bf16 bits: row dst_row[t,k] = bf16(w[t,k] * g[t]) -- the float32 product rounded once
    (what the kernel computes), or with exact=True the float64 product rounded once."""
    gf = wl.bf16_bits_to_f32(g_bits)
    want = np.full((rows, g_bits.shape[1]), fill, np.uint16)
    for k in range(lay.dst_row.shape[1]):  # one oracle dispatch per entry column
        col = dataclasses.replace(lay, K=1, dst_row=np.ascontiguousarray(lay.dst_row[:, k:k + 1]))
        if exact:
            scaled = f64_to_bf16_bits(w[:, k:k + 1].astype(np.float64) * gf.astype(np.float64))
        else:
            scaled = wl.f32_to_bf16_bits(w[:, k:k + 1] * gf)
        oracle_mod.dispatch(scaled, None, col, want)
    return want


def grad_w_reference(y_bits: np.ndarray, g_bits: np.ndarray, lay):
    """float64 [T, K] row dot products, the terms' absolute sums (for error bounds), and which entries have rows."""
    yf = wl.bf16_bits_to_f32(y_bits).astype(np.float64)
    gf = wl.bf16_bits_to_f32(g_bits).astype(np.float64)
    valid = lay.dst_row >= 0
    terms = yf[np.clip(lay.dst_row, 0, None)] * gf[:, None, :]          # [T, K, H]
    return np.where(valid, terms.sum(-1), 0.0), np.abs(terms).sum(-1), valid
