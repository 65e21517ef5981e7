"""Helpers shared by the GPU parity tests (not a test module)."""
from __future__ import annotations

from typing import Optional

import numpy as np

import workloads as W
from oracle import lora_oracle as O

REL_FRO = 5e-3     # relative Frobenius error bound of the delta (bf16 in, fp32 accumulate)
MAX_ABS = 2e-2     # absolute bound on any element of the delta


def oracle_projection(b: W.Batch, ws: W.WeightSource, layer: int, j: int,
                      rows: Optional[np.ndarray] = None, use_y: bool = True):
    """fp64 oracle of projection j over all rows or a sample of them."""
    w = b.workload
    p = w.projs[j]
    x = b.inputs[p.input]
    aid = b.adapter_id
    eid = b.expert_id
    src = None if p.input == "mid" else b.token_of_pair
    y = b.y_in[p.name] if use_y else None
    if rows is not None:
        aid = aid[rows]
        eid = None if eid is None else eid[rows]
        src = rows.astype(np.int32) if src is None else src[rows]
        y = None if y is None else np.ascontiguousarray(y[rows])
    n_units = w.n_adapters * w.n_experts
    A_units = [None] * n_units
    B_units = [None] * n_units
    e_arr = eid if eid is not None else np.zeros_like(aid)
    for a, e in set(zip(aid[aid >= 0].tolist(), e_arr[aid >= 0].tolist())):
        if 0 <= a < w.n_adapters and 0 <= e < w.n_experts:
            A, B = ws.unit_arrays(a, layer, e, j)
            A_units[a * w.n_experts + e] = np.ascontiguousarray(A)
            B_units[a * w.n_experts + e] = np.ascontiguousarray(B)
    if all(u is None for u in A_units):   # no active row: any unit defines the shapes
        A, B = ws.unit_arrays(0, layer, 0, j)
        A_units[0], B_units[0] = np.ascontiguousarray(A), np.ascontiguousarray(B)
    return O.delta(x, aid, A_units, B_units, b.scale, n_adapters=w.n_adapters,
                   n_experts=w.n_experts, expert_id=eid, src_row=src, y_in=y)


def bf16_order(bits: np.ndarray) -> np.ndarray:
    """Map bf16 bit patterns to integers whose difference counts representable steps."""
    b = bits.astype(np.int64)
    mag = b & 0x7FFF
    return np.where(b & 0x8000, -mag, mag)


# What the checks below measured in this process: (kind, what) -> dict.  tests/conftest.py
# writes it out at the end of a GPU session so that the worst cases behind the tolerances are
# on file.
MEASURED = {}


def check_delta(got_f64: np.ndarray, want_delta: np.ndarray, what: str = ""):
    """The tolerance of the floating-point path: relative Frobenius <= 5e-3, max abs <= 2e-2."""
    diff = got_f64 - want_delta
    den = np.linalg.norm(want_delta)
    rel = np.linalg.norm(diff) / den if den > 0 else np.linalg.norm(diff)
    mx = float(np.max(np.abs(diff))) if diff.size else 0.0
    MEASURED[("delta", what)] = dict(rel_fro=float(rel), max_abs=mx, elements=int(diff.size))
    assert rel <= REL_FRO, f"{what}: rel Frobenius {rel:.3e} > {REL_FRO}"
    assert mx <= MAX_ABS, f"{what}: max abs {mx:.3e} > {MAX_ABS}"
    return rel, mx


ACC_REL = 3e-5     # fp32 accumulation error of a delta element, relative to its row's scale


def bf16_ulp(v: np.ndarray) -> np.ndarray:
    """Spacing of bf16 values at |v| (8 significant bits; subnormal floor 2^-133)."""
    a = np.maximum(np.abs(v), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(a)) - 7)


def check_accumulate(got_bits: np.ndarray, res, what: str = ""):
    """Accumulate mode, y = bf16_rne(fp32(y_in) + delta).

    Element bound: one bf16 step at the exact sum (half a step from the final rounding, the
    rest for the tie that an fp32 sum can fall on the other side of) plus the error of the
    delta itself before the addition, ACC_REL times the largest delta of the row (fp32
    accumulation over K; it is what remains visible when y_in and delta cancel).  Where the
    sum does not cancel this is the same as "within one bf16 step of the oracle's
    once-rounded sum", which is also counted.  Whole output: the Frobenius bound.
    """
    got = W.bf16_bits_to_f32(got_bits).astype(np.float64)
    err = np.abs(got - res.y_out)
    row_scale = np.max(np.abs(res.delta), axis=1, keepdims=True) if res.delta.size else 0.0
    bound = bf16_ulp(res.y_out) + ACC_REL * row_scale
    bad = err > bound
    if err.size:
        # the ACC_REL this output would have needed, and how many elements sit more than one
        # bf16 step from the oracle's once-rounded sum
        excess = (err - bf16_ulp(res.y_out)) / np.maximum(row_scale, 1e-300)
        steps_ = np.abs(bf16_order(got_bits) - bf16_order(res.y_bf16))
        MEASURED[("accumulate", what)] = dict(
            acc_rel_needed=float(max(0.0, excess.max())), worst_ratio=float((err / bound).max()),
            frac_more_than_one_step=float((steps_ > 1).mean()), max_steps=int(steps_.max()),
            elements=int(err.size))
    assert not bad.any(), (f"{what}: {int(bad.sum())} elements beyond one bf16 step + accumulation "
                           f"tolerance; worst ratio {float((err / bound).max()):.2f}")
    steps = np.abs(bf16_order(got_bits) - bf16_order(res.y_bf16))
    frac_off = float((steps > 1).mean()) if steps.size else 0.0
    assert frac_off <= 1e-3, f"{what}: {frac_off:.2e} of the elements more than one step off"
    den = np.linalg.norm(res.y_out)
    rel = np.linalg.norm(got - res.y_out) / den if den > 0 else 0.0
    assert rel <= REL_FRO, f"{what}: rel Frobenius of y {rel:.3e}"
    return int(steps.max(initial=0)), rel
