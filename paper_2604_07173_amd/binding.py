"""ctypes binding of liblora.so: same names as include/lora.h, argument marshalling only.

Device buffers are passed as torch CUDA tensors (or raw integer addresses); torch is used
for device memory and streams, nothing else.  Every step of the path runs in the library's
kernels; if the library is missing the import of a symbol raises LoraError.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

LORA_DTYPE_BF16, LORA_DTYPE_F32 = 0, 1
LORA_MOE_UPGATE, LORA_MOE_DOWN = 0, 1
LORA_ACT_AUTO, LORA_ACT_RESIDENT, LORA_ACT_STREAMING = 0, 1, 2
LORA_MAX_PROJ = 8
LORA_MAX_ROWS = 1 << 14
LORA_MAX_ROWS_LONG = 1 << 20
LORA_STATIC_WS_BYTES = 16 << 20

EXPORTED_SYMBOLS = [
    "lora_strerror", "lora_last_hip_error", "lora_pool_bytes", "lora_register_pool",
    "lora_pool_load_unit", "lora_pool_load_adapter_layer", "lora_pool_adapter_layer_bytes",
    "lora_pool_load_adapter_async", "lora_pool_set_adapter", "lora_pool_set_activation_policy", "lora_pool_activation_policy", "lora_pool_wait_layer", "lora_pool_layer_ready", "lora_pool_read_unit",
    "lora_pool_unit_layout", "lora_pool_device_table", "lora_pool_destroy",
    "lora_segments_ws_bytes", "lora_segments_launches", "lora_build_segments", "lora_v_bytes", "lora_shrink",
    "lora_provision_iar", "lora_provision_min_cache", "lora_provision_memory_bytes",
    "lora_expand", "lora_apply", "lora_group_ws_bytes", "lora_group_launches", "lora_apply_group", "lora_build_apply_group", "lora_build_apply_launches", "lora_moe_ws_bytes", "lora_moe_apply", "lora_moe_build_apply", "lora_moe_apply_static", "lora_moe_combine_ws_bytes", "lora_moe_down_combine", "lora_moe_shrink", "lora_moe_expand",
]


class LoraError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str = ""):
        self.status = status
        msg = f"{where}: {lora_strerror(status)} ({status})"
        if detail:
            msg += f": {detail}"
        super().__init__(msg)


class _ProjDesc(C.Structure):
    _fields_ = [("h_in", C.c_int32), ("h_out", C.c_int32)]


class _PoolDesc(C.Structure):
    _fields_ = [("n_adapters", C.c_int32), ("n_layers", C.c_int32), ("n_experts", C.c_int32),
                ("n_proj", C.c_int32), ("rank", C.c_int32), ("dtype", C.c_int32),
                ("proj", _ProjDesc * LORA_MAX_PROJ),
                ("scale", C.POINTER(C.c_float)), ("adapter_rank", C.POINTER(C.c_int32))]


class _Segments(C.Structure):
    _fields_ = [("P", C.c_int32), ("tile_rows", C.c_int32), ("n_keys", C.c_int32),
                ("reserved", C.c_int32), ("perm", C.c_void_p),
                ("seg_start", C.c_void_p), ("seg_key", C.c_void_p), ("tiles", C.c_void_p),
                ("counts", C.c_void_p), ("status", C.c_void_p)]


_lib = None


def lib_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "liblora.so")


def load_library():
    """Load liblora.so (built in-tree by paper_2604_07173_amd/build.py). No fallback."""
    global _lib
    if _lib is not None:
        return _lib
    # torch ships its own HIP runtime; import it first so that liblora binds to the same one
    # that owns the tensors' memory and streams (two runtimes in one process do not mix)
    import torch  # noqa: F401
    path = lib_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is not built; run `python -m paper_2604_07173_amd.build` "
                           "(there is no CPU fallback)")
    lib = C.CDLL(path)
    vp, i32, i64, sz = C.c_void_p, C.c_int, C.c_int64, C.c_size_t
    lib.lora_strerror.restype = C.c_char_p
    lib.lora_strerror.argtypes = [i32]
    lib.lora_last_hip_error.restype = C.c_char_p
    lib.lora_last_hip_error.argtypes = []
    lib.lora_pool_bytes.restype = sz
    lib.lora_pool_bytes.argtypes = [C.POINTER(_PoolDesc)]
    lib.lora_register_pool.restype = i32
    lib.lora_register_pool.argtypes = [C.POINTER(_PoolDesc), vp, sz, vp, vp, vp, C.POINTER(vp)]
    lib.lora_pool_load_unit.restype = i32
    lib.lora_pool_load_unit.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp]
    lib.lora_pool_load_adapter_layer.restype = i32
    lib.lora_pool_load_adapter_layer.argtypes = [vp, i32, i32, vp, vp]
    lib.lora_pool_adapter_layer_bytes.restype = C.c_size_t
    lib.lora_pool_adapter_layer_bytes.argtypes = [vp, i32]
    lib.lora_pool_load_adapter_async.restype = i32
    lib.lora_pool_load_adapter_async.argtypes = [vp, i32, vp, vp, C.c_size_t, vp]
    lib.lora_pool_set_adapter.restype = i32
    lib.lora_pool_set_adapter.argtypes = [vp, i32, i32, C.c_float, vp]
    lib.lora_pool_set_activation_policy.restype = i32
    lib.lora_pool_set_activation_policy.argtypes = [vp, i32]
    lib.lora_pool_activation_policy.restype = i32
    lib.lora_pool_activation_policy.argtypes = [vp]
    lib.lora_pool_wait_layer.restype = i32
    lib.lora_pool_wait_layer.argtypes = [vp, i32, i32, vp]
    lib.lora_pool_layer_ready.restype = i32
    lib.lora_pool_layer_ready.argtypes = [vp, i32, i32]
    lib.lora_pool_read_unit.restype = i32
    lib.lora_pool_read_unit.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp]
    lib.lora_pool_unit_layout.restype = i32
    lib.lora_pool_unit_layout.argtypes = [vp, i32, i32, i32, i32, C.POINTER(sz), C.POINTER(sz),
                                          C.POINTER(sz), C.POINTER(sz), C.POINTER(C.c_int32),
                                          C.POINTER(C.c_float)]
    lib.lora_pool_device_table.restype = vp
    lib.lora_pool_device_table.argtypes = [vp]
    lib.lora_pool_destroy.restype = i32
    lib.lora_pool_destroy.argtypes = [vp]
    lib.lora_segments_ws_bytes.restype = sz
    lib.lora_segments_ws_bytes.argtypes = [i32]
    lib.lora_segments_launches.restype = i32
    lib.lora_segments_launches.argtypes = [vp, i32]
    lib.lora_build_segments.restype = i32
    lib.lora_build_segments.argtypes = [vp, vp, vp, i32, C.POINTER(_Segments), vp, sz, vp]
    lib.lora_v_bytes.restype = sz
    lib.lora_v_bytes.argtypes = [vp, i32, i32]
    lib.lora_shrink.restype = i32
    lib.lora_shrink.argtypes = [vp, i32, i32, vp, i64, vp, C.POINTER(_Segments), vp, vp]
    lib.lora_expand.restype = i32
    lib.lora_expand.argtypes = [vp, i32, i32, vp, C.POINTER(_Segments), vp, i64, i32, vp]
    lib.lora_apply.restype = i32
    lib.lora_apply.argtypes = [vp, i32, i32, vp, i64, vp, C.POINTER(_Segments), vp, i64, i32, vp, vp]
    lib.lora_group_ws_bytes.restype = sz
    lib.lora_group_ws_bytes.argtypes = [vp, i32, i32, i32]
    lib.lora_group_launches.restype = i32
    lib.lora_group_launches.argtypes = [vp, i32, i32, i32, C.POINTER(_Segments)]
    lib.lora_apply_group.restype = i32
    lib.lora_apply_group.argtypes = [vp, i32, i32, i32, vp, i64, vp, C.POINTER(_Segments),
                                     C.POINTER(vp), C.POINTER(i64), i32, vp, sz, vp]
    lib.lora_build_apply_group.restype = i32
    lib.lora_build_apply_group.argtypes = [vp, i32, i32, i32, vp, i64, vp, vp, vp, i32, C.POINTER(_Segments),
                                           vp, sz, C.POINTER(vp), C.POINTER(i64), i32, vp, sz, vp]
    lib.lora_build_apply_launches.restype = i32
    lib.lora_build_apply_launches.argtypes = [vp, i32, i32, i32, i32]
    lib.lora_moe_build_apply.restype = i32
    lib.lora_moe_build_apply.argtypes = [vp, i32, i32, vp, i64, vp, vp, vp, i32, C.POINTER(_Segments), vp, sz,
                                         vp, vp, i64, vp, sz, vp]
    lib.lora_moe_ws_bytes.restype = sz
    lib.lora_moe_ws_bytes.argtypes = [vp, i32]
    lib.lora_moe_apply.restype = i32
    lib.lora_moe_apply.argtypes = [vp, i32, i32, vp, i64, vp, C.POINTER(_Segments), vp, vp, i64,
                                   vp, sz, vp]
    lib.lora_moe_apply_static.restype = i32
    lib.lora_moe_apply_static.argtypes = [vp, i32, i32, vp, i64, vp, C.POINTER(_Segments), vp, vp, i64, vp]
    lib.lora_moe_shrink.restype = i32
    lib.lora_moe_shrink.argtypes = [vp, i32, i32, vp, i64, vp, C.POINTER(_Segments), vp, sz, vp]
    lib.lora_moe_expand.restype = i32
    lib.lora_moe_expand.argtypes = [vp, i32, i32, C.POINTER(_Segments), vp, vp, i64, vp, sz, vp]
    lib.lora_moe_combine_ws_bytes.restype = sz
    lib.lora_moe_combine_ws_bytes.argtypes = [vp, i32]
    lib.lora_moe_down_combine.restype = i32
    lib.lora_moe_down_combine.argtypes = [vp, i32, vp, i64, vp, vp, C.POINTER(_Segments), vp, i32, vp, i64,
                                          vp, sz, vp]
    dp = C.POINTER(C.c_double)
    lib.lora_provision_iar.restype = i32
    lib.lora_provision_iar.argtypes = [dp, i32, C.c_double, i32, dp, dp, dp]
    lib.lora_provision_min_cache.restype = i32
    lib.lora_provision_min_cache.argtypes = [dp, i32, C.c_double, C.c_double, C.POINTER(C.c_int), dp]
    lib.lora_provision_memory_bytes.restype = C.c_int64
    lib.lora_provision_memory_bytes.argtypes = [i32, C.c_int64]
    _lib = lib
    return lib


def lora_strerror(status: int) -> str:
    try:
        return load_library().lora_strerror(int(status)).decode()
    except RuntimeError:
        return "liblora not built"


def _check(status: int, where: str):
    if status != 0:
        detail = load_library().lora_last_hip_error().decode() if status == -6 else ""
        raise LoraError(status, where, detail)


def _addr(t) -> Optional[int]:
    """torch tensor / int / None -> device address."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return int(t.data_ptr())


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream) or None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


class PoolDesc:
    """Host description of a pool (mirrors lora_pool_desc)."""

    def __init__(self, n_adapters: int, n_layers: int, n_experts: int,
                 projs: Sequence[Sequence[int]], rank: int, scale=None, adapter_rank=None,
                 dtype: int = LORA_DTYPE_BF16):
        self.n_adapters, self.n_layers, self.n_experts = n_adapters, n_layers, n_experts
        self.projs = [(int(a), int(b)) for a, b in projs]
        self.rank, self.dtype = rank, dtype
        self.scale = None if scale is None else [float(s) for s in scale]
        self.adapter_rank = None if adapter_rank is None else [int(r) for r in adapter_rank]

    def to_c(self) -> _PoolDesc:
        d = _PoolDesc()
        d.n_adapters, d.n_layers, d.n_experts = self.n_adapters, self.n_layers, self.n_experts
        d.n_proj = len(self.projs)
        d.rank, d.dtype = self.rank, self.dtype
        for i, (a, b) in enumerate(self.projs[:LORA_MAX_PROJ]):
            d.proj[i].h_in, d.proj[i].h_out = a, b
        self._keep = []
        if self.scale is not None:
            arr = (C.c_float * len(self.scale))(*self.scale)
            self._keep.append(arr)
            d.scale = C.cast(arr, C.POINTER(C.c_float))
        if self.adapter_rank is not None:
            arr = (C.c_int32 * len(self.adapter_rank))(*self.adapter_rank)
            self._keep.append(arr)
            d.adapter_rank = C.cast(arr, C.POINTER(C.c_int32))
        return d


class Pool:
    """Owner of a lora_pool handle and of the slab tensor it lives in."""

    def __init__(self, handle: int, desc: PoolDesc, slab):
        self.handle, self.desc, self.slab = handle, desc, slab

    def __del__(self):
        try:
            if self.handle:
                lora_pool_destroy(self)
        except Exception:
            pass


def _h(pool) -> Optional[int]:
    return pool.handle if isinstance(pool, Pool) else pool


def lora_pool_bytes(desc: PoolDesc) -> int:
    d = desc.to_c()
    return int(load_library().lora_pool_bytes(C.byref(d)))


def lora_register_pool(desc: PoolDesc, slab, slab_bytes: Optional[int] = None,
                       A_src: Optional[Sequence] = None, B_src: Optional[Sequence] = None,
                       stream=None) -> Pool:
    """slab: torch uint8 CUDA tensor (or address + slab_bytes). A_src/B_src: sequences of
    device tensors/addresses in [adapter][layer][expert][proj] order, or None."""
    lib = load_library()
    d = desc.to_c()
    if slab_bytes is None:
        slab_bytes = slab.numel() * slab.element_size()
    a_arr = b_arr = None
    if A_src is not None:
        a_arr = (C.c_void_p * len(A_src))(*[_addr(t) for t in A_src])
    if B_src is not None:
        b_arr = (C.c_void_p * len(B_src))(*[_addr(t) for t in B_src])
    out = C.c_void_p()
    st = lib.lora_register_pool(C.byref(d), _addr(slab), slab_bytes,
                                C.cast(a_arr, C.c_void_p) if a_arr is not None else None,
                                C.cast(b_arr, C.c_void_p) if b_arr is not None else None,
                                _stream(stream), C.byref(out))
    _check(st, "lora_register_pool")
    return Pool(out.value, desc, slab)


def lora_pool_load_unit(pool, adapter, layer, expert, proj, A, B, stream=None):
    _check(load_library().lora_pool_load_unit(_h(pool), adapter, layer, expert, proj, _addr(A),
                                              _addr(B), _stream(stream)), "lora_pool_load_unit")


def lora_pool_load_adapter_layer(pool, adapter, layer, src, stream=None):
    _check(load_library().lora_pool_load_adapter_layer(_h(pool), adapter, layer, _addr(src),
                                                       _stream(stream)),
           "lora_pool_load_adapter_layer")


def lora_pool_adapter_layer_bytes(pool, adapter) -> int:
    return int(load_library().lora_pool_adapter_layer_bytes(_h(pool), adapter))


def lora_pool_load_adapter_async(pool, adapter, host_src, staging, load_stream=None):
    """host_src: pinned host tensor (all layers back to back); staging: device tensor."""
    _check(load_library().lora_pool_load_adapter_async(
        _h(pool), adapter, _addr(host_src), _addr(staging),
        staging.numel() * staging.element_size(), _stream(load_stream)),
        "lora_pool_load_adapter_async")


def lora_pool_set_activation_policy(pool, policy):
    _check(load_library().lora_pool_set_activation_policy(_h(pool), int(policy)),
           "lora_pool_set_activation_policy")


def lora_pool_activation_policy(pool) -> int:
    rc = load_library().lora_pool_activation_policy(_h(pool))
    _check(min(rc, 0), "lora_pool_activation_policy")
    return rc


def lora_pool_set_adapter(pool, adapter, rank, scale, stream=None):
    _check(load_library().lora_pool_set_adapter(_h(pool), adapter, rank, float(scale), _stream(stream)),
           "lora_pool_set_adapter")


def lora_pool_wait_layer(pool, adapter, layer, stream=None):
    _check(load_library().lora_pool_wait_layer(_h(pool), adapter, layer, _stream(stream)),
           "lora_pool_wait_layer")


def lora_pool_layer_ready(pool, adapter, layer) -> bool:
    rc = load_library().lora_pool_layer_ready(_h(pool), adapter, layer)
    if rc < 0:
        _check(rc, "lora_pool_layer_ready")
    return rc == 1


def lora_pool_read_unit(pool, adapter, layer, expert, proj, A_out, B_out, stream=None):
    _check(load_library().lora_pool_read_unit(_h(pool), adapter, layer, expert, proj,
                                              _addr(A_out), _addr(B_out), _stream(stream)),
           "lora_pool_read_unit")


def lora_pool_unit_layout(pool, adapter, layer, expert, proj) -> dict:
    ao, ab, bo, bb = C.c_size_t(), C.c_size_t(), C.c_size_t(), C.c_size_t()
    rk, sc = C.c_int32(), C.c_float()
    _check(load_library().lora_pool_unit_layout(_h(pool), adapter, layer, expert, proj,
                                                C.byref(ao), C.byref(ab), C.byref(bo),
                                                C.byref(bb), C.byref(rk), C.byref(sc)),
           "lora_pool_unit_layout")
    return dict(A_offset=ao.value, A_bytes=ab.value, B_offset=bo.value, B_bytes=bb.value,
                rank=rk.value, scale=sc.value)


def lora_pool_destroy(pool):
    h = _h(pool)
    st = load_library().lora_pool_destroy(h)
    if isinstance(pool, Pool):
        pool.handle = None
    _check(st, "lora_pool_destroy")


def lora_segments_ws_bytes(P: int) -> int:
    return int(load_library().lora_segments_ws_bytes(P))


def lora_segments_launches(pool, P: int) -> int:
    return int(load_library().lora_segments_launches(_h(pool), P))


class Segments:
    """Device buffers of a lora_segments plus the C struct that points at them."""

    def __init__(self, P_max: int, device="cuda"):
        import torch
        n = max(P_max, 1)
        self.perm = torch.empty(n, dtype=torch.int32, device=device)
        self.seg_start = torch.empty(n + 1, dtype=torch.int32, device=device)
        self.seg_key = torch.empty(n, dtype=torch.int32, device=device)
        self.tiles = torch.empty((n, 4), dtype=torch.int32, device=device)
        self.counts = torch.zeros(4, dtype=torch.int32, device=device)
        self.status = torch.zeros(1, dtype=torch.int32, device=device)
        self.ws = torch.empty(max(lora_segments_ws_bytes(P_max), 256), dtype=torch.uint8,
                              device=device)
        self.c = _Segments()
        self.c.P, self.c.tile_rows = 0, 0
        self.c.perm, self.c.seg_start = self.perm.data_ptr(), self.seg_start.data_ptr()
        self.c.seg_key, self.c.tiles = self.seg_key.data_ptr(), self.tiles.data_ptr()
        self.c.counts, self.c.status = self.counts.data_ptr(), self.status.data_ptr()
        self.P_max = P_max


def lora_build_segments(pool, adapter_id, expert_id, P: int, seg: Segments, stream=None):
    _check(load_library().lora_build_segments(_h(pool), _addr(adapter_id), _addr(expert_id), P,
                                              C.byref(seg.c), _addr(seg.ws),
                                              seg.ws.numel(), _stream(stream)),
           "lora_build_segments")


def lora_v_bytes(pool, proj: int, P: int) -> int:
    return int(load_library().lora_v_bytes(_h(pool), proj, P))


def lora_shrink(pool, layer, proj, x, ldx, src_row, seg: Segments, v, stream=None):
    _check(load_library().lora_shrink(_h(pool), layer, proj, _addr(x), ldx, _addr(src_row),
                                      C.byref(seg.c), _addr(v), _stream(stream)), "lora_shrink")


def lora_expand(pool, layer, proj, v, seg: Segments, y, ldy, out_dtype=LORA_DTYPE_BF16,
                stream=None):
    _check(load_library().lora_expand(_h(pool), layer, proj, _addr(v), C.byref(seg.c), _addr(y),
                                      ldy, out_dtype, _stream(stream)), "lora_expand")


def lora_apply(pool, layer, proj, x, ldx, src_row, seg: Segments, y, ldy, v,
               out_dtype=LORA_DTYPE_BF16, stream=None):
    _check(load_library().lora_apply(_h(pool), layer, proj, _addr(x), ldx, _addr(src_row),
                                     C.byref(seg.c), _addr(y), ldy, out_dtype, _addr(v),
                                     _stream(stream)), "lora_apply")


def lora_group_ws_bytes(pool, proj0: int, n_proj: int, P: int) -> int:
    return int(load_library().lora_group_ws_bytes(_h(pool), proj0, n_proj, P))


def lora_group_launches(pool, proj0: int, n_proj: int, P: int, seg: Segments,
                        out_dtype=LORA_DTYPE_BF16) -> int:
    """Kernel launches lora_apply_group would enqueue for this group and these (built) segments."""
    rc = load_library().lora_group_launches(_h(pool), proj0, n_proj, out_dtype, C.byref(seg.c))
    if rc < 0:
        _check(rc, "lora_group_launches")
    return rc


def lora_apply_group(pool, layer, proj0, x, ldx, src_row, seg: Segments, ys, ldys, ws,
                     out_dtype=LORA_DTYPE_BF16, stream=None):
    """ys / ldys: one output tensor and row stride per projection of the group."""
    n = len(ys)
    y_arr = (C.c_void_p * n)(*[_addr(y) for y in ys])
    ld_arr = (C.c_int64 * n)(*[int(v) for v in ldys])
    _check(load_library().lora_apply_group(_h(pool), layer, proj0, n, _addr(x), ldx, _addr(src_row),
                                           C.byref(seg.c), y_arr, ld_arr, out_dtype, _addr(ws),
                                           ws.numel() * ws.element_size(), _stream(stream)),
           "lora_apply_group")


def lora_build_apply_group(pool, layer, proj0, x, ldx, src_row, adapter_id, expert_id, P: int,
                           seg: Segments, ys, ldys, ws, out_dtype=LORA_DTYPE_BF16, stream=None):
    """lora_build_segments + lora_apply_group in one call (the first group of a layer call)."""
    n = len(ys)
    y_arr = (C.c_void_p * n)(*[_addr(y) for y in ys])
    ld_arr = (C.c_int64 * n)(*[int(v) for v in ldys])
    _check(load_library().lora_build_apply_group(
        _h(pool), layer, proj0, n, _addr(x), ldx, _addr(src_row), _addr(adapter_id), _addr(expert_id), P,
        C.byref(seg.c), _addr(seg.ws), seg.ws.numel(), y_arr, ld_arr, out_dtype, _addr(ws),
        ws.numel() * ws.element_size(), _stream(stream)), "lora_build_apply_group")


def lora_build_apply_launches(pool, proj0: int, n_proj: int, P: int, out_dtype=LORA_DTYPE_BF16) -> int:
    rc = load_library().lora_build_apply_launches(_h(pool), proj0, n_proj, out_dtype, P)
    if rc < 0:
        _check(rc, "lora_build_apply_launches")
    return int(rc)


def lora_moe_ws_bytes(pool, P: int) -> int:
    return int(load_library().lora_moe_ws_bytes(_h(pool), P))


def lora_moe_build_apply(pool, layer, which, inp, ld_in, token_of_pair, adapter_id, expert_id, P: int,
                         seg: Segments, y0, y1, ldy, ws, ws_bytes=None, stream=None):
    """lora_build_segments + lora_moe_apply in one call."""
    if ws_bytes is None:
        ws_bytes = ws.numel() * ws.element_size()
    _check(load_library().lora_moe_build_apply(
        _h(pool), layer, which, _addr(inp), ld_in, _addr(token_of_pair), _addr(adapter_id),
        _addr(expert_id), P, C.byref(seg.c), _addr(seg.ws), seg.ws.numel(), _addr(y0), _addr(y1), ldy,
        _addr(ws), ws_bytes, _stream(stream)), "lora_moe_build_apply")


def lora_moe_apply(pool, layer, which, inp, ld_in, token_of_pair, seg: Segments, y0, y1, ldy,
                   ws, ws_bytes=None, stream=None):
    if ws_bytes is None:
        ws_bytes = ws.numel() * ws.element_size()
    _check(load_library().lora_moe_apply(_h(pool), layer, which, _addr(inp), ld_in,
                                         _addr(token_of_pair), C.byref(seg.c), _addr(y0),
                                         _addr(y1), ldy, _addr(ws), ws_bytes, _stream(stream)),
           "lora_moe_apply")


def lora_moe_apply_static(pool, layer, which, inp, ld_in, token_of_pair, seg: Segments, y0, y1, ldy,
                          stream=None):
    _check(load_library().lora_moe_apply_static(_h(pool), layer, which, _addr(inp), ld_in,
                                                _addr(token_of_pair), C.byref(seg.c), _addr(y0),
                                                _addr(y1), ldy, _stream(stream)),
           "lora_moe_apply_static")


def lora_moe_shrink(pool, layer, which, inp, ld_in, token_of_pair, seg: Segments, ws,
                    ws_bytes=None, stream=None):
    if ws_bytes is None:
        ws_bytes = ws.numel() * ws.element_size()
    _check(load_library().lora_moe_shrink(_h(pool), layer, which, _addr(inp), ld_in,
                                          _addr(token_of_pair), C.byref(seg.c), _addr(ws),
                                          ws_bytes, _stream(stream)), "lora_moe_shrink")


def lora_moe_expand(pool, layer, which, seg: Segments, y0, y1, ldy, ws, ws_bytes=None,
                    stream=None):
    if ws_bytes is None:
        ws_bytes = ws.numel() * ws.element_size()
    _check(load_library().lora_moe_expand(_h(pool), layer, which, C.byref(seg.c), _addr(y0),
                                          _addr(y1), ldy, _addr(ws), ws_bytes, _stream(stream)),
           "lora_moe_expand")


def lora_moe_combine_ws_bytes(pool, P: int) -> int:
    return int(load_library().lora_moe_combine_ws_bytes(_h(pool), P))


def lora_moe_down_combine(pool, layer, hmid, ld_in, adapter_id, expert_id, seg: Segments, route_w,
                          top_k, y_tok, ldy, ws, ws_bytes=None, stream=None):
    if ws_bytes is None:
        ws_bytes = ws.numel() * ws.element_size()
    _check(load_library().lora_moe_down_combine(_h(pool), layer, _addr(hmid), ld_in, _addr(adapter_id),
                                                _addr(expert_id), C.byref(seg.c), _addr(route_w),
                                                int(top_k), _addr(y_tok), ldy, _addr(ws), ws_bytes,
                                                _stream(stream)), "lora_moe_down_combine")


# ---- cache provisioning (include/lora_provision.h): host arrays in, numbers out ----------------


class ProvisionError(ValueError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status}")


def _doubles(values):
    arr = (C.c_double * len(values))(*[float(v) for v in values])
    return arr


def lora_provision_iar(p, LB: float, M: int):
    """IAR(M), tau* and the residency probabilities q_i (a list) for invocation probabilities p."""
    n = len(p)
    arr, q = _doubles(p), (C.c_double * n)()
    iar, tau = C.c_double(), C.c_double()
    st = load_library().lora_provision_iar(arr, n, float(LB), int(M), C.byref(iar), C.byref(tau), q)
    if st != 0:
        raise ProvisionError(st, "lora_provision_iar")
    return iar.value, tau.value, list(q)


def lora_provision_min_cache(p, LB: float, alpha: float):
    """(M*, IAR(M*)): the smallest cache capacity whose IAR reaches alpha."""
    arr = _doubles(p)
    m, iar = C.c_int(), C.c_double()
    st = load_library().lora_provision_min_cache(arr, len(p), float(LB), float(alpha), C.byref(m),
                                                 C.byref(iar))
    if st != 0:
        raise ProvisionError(st, "lora_provision_min_cache")
    return m.value, iar.value


def lora_provision_memory_bytes(M: int, adapter_bytes: int) -> int:
    return int(load_library().lora_provision_memory_bytes(int(M), int(adapter_bytes)))
