"""CPU-only checks of the C-ABI library: it loads, exports what include/lora.h declares, and
rejects host-detectable mistakes before touching the device."""
import ctypes as C
import os
import re

import pytest

import paper_2604_07173_amd as L
from paper_2604_07173_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(L.lib_path()):
        from paper_2604_07173_amd import build
        build.build()
    return L.load_library()


def declared_functions():
    names = set()
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if fn.endswith(".h"):
            text = open(os.path.join(inc, fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names.update(re.findall(r"\b(lora_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert len(names) >= 15
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/lora.h but not exported"
    assert sorted(L.EXPORTED_SYMBOLS) == names


def test_activation_policy_calls_reject_a_missing_pool(lib):
    assert lib.lora_pool_set_activation_policy(None, L.LORA_ACT_STREAMING) == -5
    assert lib.lora_pool_activation_policy(None) == -5
    assert (L.LORA_ACT_AUTO, L.LORA_ACT_RESIDENT, L.LORA_ACT_STREAMING) == (0, 1, 2)


def test_strerror(lib):
    assert L.lora_strerror(0) == "ok"
    assert "rank" in L.lora_strerror(-3)
    assert L.lora_strerror(-99) == "unknown status"


def test_pool_bytes_and_desc_validation(lib):
    good = L.PoolDesc(4, 1, 1, [(1024, 1024)], 8)
    n = L.lora_pool_bytes(good)
    assert n >= 4 * (1024 * 8 * 2) * 2 and n % 256 == 0
    # Sec. 2.3: one Mixtral-8x7B rank-64 adapter is 1.69 GB; the slab adds only the table
    mix = L.PoolDesc(1, 32, 8, [(4096, 14336), (4096, 14336), (14336, 4096)], 64)
    assert L.lora_pool_bytes(mix) == 1811939328 + 32 * 8 * 3 * 32
    assert L.lora_pool_bytes(L.PoolDesc(4, 1, 1, [(1024, 1024)], 12)) == 0     # rank
    assert L.lora_pool_bytes(L.PoolDesc(4, 1, 1, [(1020, 1024)], 8)) == 0      # width % 8
    assert L.lora_pool_bytes(L.PoolDesc(0, 1, 1, [(1024, 1024)], 8)) == 0
    assert L.lora_pool_bytes(L.PoolDesc(4, 1, 1, [], 8)) == 0


def _register(lib, desc, slab, nbytes):
    d = desc.to_c()
    out = C.c_void_p()
    return lib.lora_register_pool(C.byref(d), slab, nbytes, None, None, None, C.byref(out)), out


def test_register_pool_rejects_bad_arguments_without_a_gpu(lib):
    desc = L.PoolDesc(4, 1, 1, [(1024, 1024)], 8)
    need = L.lora_pool_bytes(desc)
    assert _register(lib, desc, None, need)[0] == -1                       # NULL slab
    assert _register(lib, desc, 0x1000 + 8, need)[0] == -7                 # misaligned
    assert _register(lib, desc, 0x1000, need - 1)[0] == -4                 # too small
    assert _register(lib, L.PoolDesc(4, 1, 1, [(1024, 1024)], 48), 0x1000, 1 << 30)[0] == -3
    assert _register(lib, L.PoolDesc(4, 1, 1, [(1024, 1028)], 8), 0x1000, 1 << 30)[0] == -2
    assert _register(lib, L.PoolDesc(4, 1, 1, [(1024, 1024)], 8, adapter_rank=[8, 8, 9, 8]),
                     0x1000, 1 << 30)[0] == -3
    d = desc.to_c()
    assert lib.lora_register_pool(C.byref(d), 0x1000, need, None, None, None, None) == -1


def test_calls_on_missing_pool_or_segments(lib):
    seg = B._Segments()
    assert lib.lora_build_segments(None, None, None, 4, C.byref(seg), None, 0, None) == -5
    assert lib.lora_shrink(None, 0, 0, None, 0, None, C.byref(seg), None, None) == -5
    assert lib.lora_expand(None, 0, 0, None, C.byref(seg), None, 0, 0, None) == -5
    assert lib.lora_moe_apply(None, 0, 0, None, 0, None, C.byref(seg), None, None, 0, None, 0, None) == -5
    assert lib.lora_apply(None, 0, 0, None, 0, None, C.byref(seg), None, 0, 0, None, None) == -5
    assert lib.lora_apply_group(None, 0, 0, 2, None, 0, None, C.byref(seg), None, None, 0, None, 0,
                                None) == -5
    assert lib.lora_group_ws_bytes(None, 0, 2, 16) == 0
    assert lib.lora_pool_destroy(None) == -5
    assert lib.lora_v_bytes(None, 0, 16) == 0
    assert lib.lora_moe_ws_bytes(None, 16) == 0
    assert lib.lora_segments_ws_bytes(-1) == 0
    assert lib.lora_segments_ws_bytes(1024) > 0
