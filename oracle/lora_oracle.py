"""ctypes front end of the C oracle (oracle/lora_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the benchmark's
cpu_baseline leg, never by the product path.  Marshals numpy arrays into the C calls;
all arithmetic lives in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "lora_oracle.c")
_LIB = os.path.join(_DIR, "liblora_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _declare(lib):
    """Argument and result types of the oracle's C functions on a loaded library."""
    if True:
        lib.lora_oracle_delta.restype = C.c_int
        lib.lora_oracle_delta.argtypes = [
            C.c_int, C.c_int, C.c_int, C.c_int,
            C.c_void_p, C.c_int64, C.c_void_p,
            C.c_void_p, C.c_void_p, C.c_int, C.c_int,
            C.c_void_p, C.c_void_p, C.c_void_p,
            C.c_void_p, C.c_int64,
            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.lora_oracle_combine.restype = None
        lib.lora_oracle_combine.argtypes = [C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        lib.lora_oracle_segments.restype = C.c_int
        lib.lora_oracle_segments.argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_int,
                                             C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.lora_oracle_adapter_bytes.restype = C.c_int64
        lib.lora_oracle_adapter_bytes.argtypes = [C.c_int, C.c_int, C.c_int, C.c_void_p,
                                                  C.c_void_p, C.c_int]
        lib.lora_oracle_bf16_rne.restype = C.c_uint16
        lib.lora_oracle_bf16_rne.argtypes = [C.c_double]
        lib.lora_oracle_bf16_to_f64.restype = C.c_double
        lib.lora_oracle_bf16_to_f64.argtypes = [C.c_uint16]
    return lib


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = _declare(C.CDLL(_LIB))
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def n_threads() -> int:
    """Threads the OpenMP loop will use (OMP_NUM_THREADS or the visible cores)."""
    v = os.environ.get("OMP_NUM_THREADS")
    if v:
        try:
            return max(1, int(v.split(",")[0]))
        except ValueError:
            pass
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


class DeltaResult:
    __slots__ = ("v", "delta", "y_out", "y_bf16", "status")


def delta(x: np.ndarray, adapter_id: np.ndarray, A_units: Sequence[Optional[np.ndarray]],
          B_units: Sequence[Optional[np.ndarray]], scale: np.ndarray, *, n_adapters: int,
          n_experts: int = 1, expert_id: Optional[np.ndarray] = None,
          src_row: Optional[np.ndarray] = None, y_in: Optional[np.ndarray] = None,
          want_v: bool = True) -> DeltaResult:
    """One projection of one layer.

    x: uint16 (bf16 bits) [rows][h_in]; A_units/B_units: n_adapters*n_experts entries indexed
    adapter*n_experts+expert, each a C-contiguous uint16 array A[h_in][r] / B[r][h_out] (None
    allowed for units no row selects).  Returns v, delta, y_out (float64) and y_bf16 (uint16).
    """
    lib = _load()
    assert x.dtype == np.uint16 and x.ndim == 2 and x.strides[1] == 2
    adapter_id = np.ascontiguousarray(adapter_id, dtype=np.int32)
    P = adapter_id.shape[0]
    if expert_id is not None:
        expert_id = np.ascontiguousarray(expert_id, dtype=np.int32)
    if src_row is not None:
        src_row = np.ascontiguousarray(src_row, dtype=np.int32)
    n_units = n_adapters * n_experts
    assert len(A_units) == n_units and len(B_units) == n_units
    h_in = r = h_out = None
    Ap = np.zeros(n_units, dtype=np.uint64)
    Bp = np.zeros(n_units, dtype=np.uint64)
    keep = []
    for u in range(n_units):
        A, B = A_units[u], B_units[u]
        if A is None:
            continue
        assert A.dtype == np.uint16 and B.dtype == np.uint16
        assert A.flags.c_contiguous and B.flags.c_contiguous
        if h_in is None:
            h_in, r = A.shape
            h_out = B.shape[1]
        assert A.shape == (h_in, r) and B.shape == (r, h_out)
        Ap[u] = A.ctypes.data
        Bp[u] = B.ctypes.data
        keep.append((A, B))
    assert h_in is not None, "no unit given"
    assert x.shape[1] == h_in
    ldx = x.strides[0] // 2
    scale = np.ascontiguousarray(scale, dtype=np.float32)
    assert scale.shape[0] == n_adapters
    ldy = 0
    if y_in is not None:
        assert y_in.dtype == np.uint16 and y_in.shape == (P, h_out) and y_in.strides[1] == 2
        ldy = y_in.strides[0] // 2
    res = DeltaResult()
    res.v = np.empty((P, r), dtype=np.float64) if want_v else None
    res.delta = np.empty((P, h_out), dtype=np.float64)
    res.y_out = np.empty((P, h_out), dtype=np.float64)
    res.y_bf16 = np.empty((P, h_out), dtype=np.uint16)
    res.status = lib.lora_oracle_delta(
        P, h_in, h_out, r, _ptr(x), ldx, _ptr(src_row), _ptr(adapter_id), _ptr(expert_id),
        n_adapters, n_experts, _ptr(Ap), _ptr(Bp), _ptr(scale), _ptr(y_in), ldy,
        _ptr(res.v), _ptr(res.delta), _ptr(res.y_out), _ptr(res.y_bf16))
    del keep
    return res


class CombineResult:
    __slots__ = ("y_out", "y_bf16", "combined")


def combine(delta: np.ndarray, adapter_id: np.ndarray, route_w: np.ndarray, top_k: int,
            y_in: Optional[np.ndarray] = None) -> CombineResult:
    """Token rows after the routing-weighted combine of the per-pair updates `delta`
    ([T*k][h_out] float64, as delta() returns them).  adapter_id: per pair, -1 = no adapter
    (out-of-range ids must already have been mapped to -1).  y_in: bf16 bits [T][h_out]."""
    lib = _load()
    delta = np.ascontiguousarray(delta, dtype=np.float64)
    P, h_out = delta.shape
    assert P % top_k == 0
    T = P // top_k
    adapter_id = np.ascontiguousarray(adapter_id, dtype=np.int32)
    route_w = np.ascontiguousarray(route_w, dtype=np.float32)
    assert adapter_id.shape == (P,) and route_w.shape == (P,)
    ldy = 0
    if y_in is not None:
        assert y_in.dtype == np.uint16 and y_in.shape == (T, h_out) and y_in.strides[1] == 2
        ldy = y_in.strides[0] // 2
    res = CombineResult()
    res.y_out = np.empty((T, h_out), dtype=np.float64)
    res.y_bf16 = np.empty((T, h_out), dtype=np.uint16)
    lib.lora_oracle_combine(T, top_k, h_out, _ptr(delta), _ptr(adapter_id), _ptr(route_w),
                            _ptr(y_in), ldy, _ptr(res.y_out), _ptr(res.y_bf16))
    base = 0.0 if y_in is None else (y_in.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    res.combined = res.y_out - base
    return res


class Segments:
    __slots__ = ("perm", "seg_start", "seg_key", "S", "P_act", "n_bad")


def segments(adapter_id: np.ndarray, expert_id: Optional[np.ndarray], n_adapters: int,
             n_experts: int = 1) -> Segments:
    lib = _load()
    adapter_id = np.ascontiguousarray(adapter_id, dtype=np.int32)
    P = adapter_id.shape[0]
    if expert_id is not None:
        expert_id = np.ascontiguousarray(expert_id, dtype=np.int32)
    perm = np.full(max(P, 1), -1, dtype=np.int32)
    seg_start = np.full(P + 1, -1, dtype=np.int32)
    seg_key = np.full(max(P, 1), -1, dtype=np.int32)
    counts = np.zeros(2, dtype=np.int32)
    s = Segments()
    s.n_bad = lib.lora_oracle_segments(P, _ptr(adapter_id), _ptr(expert_id), n_adapters,
                                       n_experts, _ptr(perm), _ptr(seg_start), _ptr(seg_key),
                                       _ptr(counts))
    s.S, s.P_act = int(counts[0]), int(counts[1])
    s.perm = perm[:s.P_act].copy()
    s.seg_start = seg_start[:s.S + 1].copy()
    s.seg_key = seg_key[:s.S].copy()
    return s


def adapter_bytes(n_layers: int, n_experts: int, projs: Sequence[tuple], rank: int) -> int:
    lib = _load()
    hi = np.array([p[0] for p in projs], dtype=np.int32)
    ho = np.array([p[1] for p in projs], dtype=np.int32)
    return int(lib.lora_oracle_adapter_bytes(n_layers, n_experts, len(projs), _ptr(hi), _ptr(ho),
                                             rank))


def bf16_rne(v: float) -> int:
    return int(_load().lora_oracle_bf16_rne(float(v)))


def bf16_to_f64(bits: int) -> float:
    return float(_load().lora_oracle_bf16_to_f64(int(bits)))
