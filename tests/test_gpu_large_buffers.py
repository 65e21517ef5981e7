"""Buffers of more than 4 GiB: the largest batch the library takes (2^20 rows) with row strides
that put the last rows of x and y beyond byte offset 2^32, in both kernel families.  Sampled rows
(the last ones, those on either side of the 4 GiB crossing, random ones) against the fp64 oracle;
the padding between the rows stays untouched."""
import numpy as np
import pytest
import torch

import paper_2604_07173_amd as L
import workloads as W
from gpu_common import check_delta, oracle_projection
from harness import DevicePool, to_dev

pytestmark = pytest.mark.gpu

H_IN, H_OUT, LDX, LDY = 40, 72, 2304, 2176


@pytest.mark.parametrize("family,n_adapters,rank", [("long", 24, 16), ("decode", 65536, 8)])
def test_strided_rows_beyond_4_gib(family, n_adapters, rank):
    P = L.LORA_MAX_ROWS_LONG
    assert P * LDX * 2 > 1 << 32 and P * LDY * 2 > 1 << 32
    w = W.Workload("t", "dense", n_adapters, 1, 1, rank, (W.Proj("p", H_IN, H_OUT, "x"),), P, "uniform", 0.0)
    print(f"[large buffers/{family}] P={P} adapters={n_adapters} batch...", flush=True)
    b = W.make_batch(w, 3, y_mode="zero", no_adapter_frac=0.01)
    ws = W.make_weights(w, 3, bank_elems=1 << 20)
    dp = DevicePool(ws, b.scale)
    x = torch.zeros((P, LDX), dtype=torch.int16, device="cuda")
    x[:, :H_IN] = to_dev(b.inputs["x"])
    y = torch.zeros((P, LDY), dtype=torch.int16, device="cuda")
    seg = L.Segments(P)
    v = torch.empty(max(L.lora_group_ws_bytes(dp.pool, 0, 1, P), 256) // 4, dtype=torch.float32, device="cuda")
    print(f"[large buffers/{family}] build + apply...", flush=True)
    L.lora_build_segments(dp.pool, to_dev(b.adapter_id), None, P, seg)
    L.lora_apply_group(dp.pool, 0, 0, x, LDX, None, seg, [y], [LDY], v, L.LORA_DTYPE_BF16)
    torch.cuda.synchronize()
    assert seg.c.tile_rows == (32 if family == "long" else 16)
    assert not bool((y[:, H_OUT:] != 0).any())
    rng = np.random.default_rng(3)
    cross_x, cross_y = (1 << 32) // (2 * LDX), (1 << 32) // (2 * LDY)
    rows = np.unique(np.concatenate([rng.choice(P, size=384, replace=False), np.arange(P - 64, P),
                                     np.arange(cross_x - 16, cross_x + 16),
                                     np.arange(cross_y - 16, cross_y + 16), np.arange(0, 8)]))
    res = oracle_projection(b, ws, 0, 0, rows=rows)
    got = y[torch.from_numpy(rows).cuda(), :H_OUT].cpu().numpy().view(np.uint16)
    check_delta(W.bf16_bits_to_f32(got).astype(np.float64), res.delta, f"rows beyond 4 GiB/{family}")
    none = b.adapter_id[rows] < 0
    assert none.any() and not got[none].any()
    del x, y, dp
    torch.cuda.empty_cache()
