"""Adapter pool and pointer table: repacking is a bit-exact permutation, the device table
points where the host layout says, both loading routes fill the slab identically."""
import numpy as np
import pytest
import torch

import paper_2604_07173_amd as L
import workloads as W
from harness import DevicePool, bits_from_dev, to_dev

pytestmark = pytest.mark.gpu


def small_workload(rank, E=2, n=3, h_in=72, h_out=200):
    projs = (W.Proj("gate", h_in, h_out, "x"), W.Proj("up", h_in, h_out, "x"),
             W.Proj("down", h_out, h_in, "mid"))
    return W.Workload("t", "moe", n, E, 2, rank, projs, 16, "uniform")


@pytest.mark.parametrize("rank", [8, 16, 32, 64])
def test_pack_unpack_roundtrip_is_bit_exact(rank):
    w = small_workload(rank)
    ws = W.make_weights(w, 5, n_layers=2, bank_elems=1 << 18)
    dp = DevicePool(ws, np.ones(w.n_adapters, np.float32))
    for a in range(w.n_adapters):
        for layer in range(2):
            for e in range(w.n_experts):
                for j, p in enumerate(w.projs):
                    A_out = torch.full((p.h_in, rank), -1, dtype=torch.int16, device="cuda")
                    B_out = torch.full((rank, p.h_out), -1, dtype=torch.int16, device="cuda")
                    L.lora_pool_read_unit(dp.pool, a, layer, e, j, A_out, B_out)
                    torch.cuda.synchronize()
                    A, B = ws.unit_arrays(a, layer, e, j)
                    assert np.array_equal(bits_from_dev(A_out), A)
                    assert np.array_equal(bits_from_dev(B_out), B)


def test_device_table_matches_host_layout():
    w = small_workload(16)
    ws = W.make_weights(w, 6, n_layers=2, bank_elems=1 << 18)
    scale = np.array([0.5, 1.0, 1.5], np.float32)
    dp = DevicePool(ws, scale)
    n_entries = 2 * w.n_adapters * w.n_experts * 3
    raw = dp.slab[:n_entries * 32].cpu().numpy()
    ent = raw.view(np.dtype([("A", "<u8"), ("B", "<u8"), ("scale", "<f4"), ("rank", "<i4"),
                             ("pad", "<i4", 2)]))
    base = dp.slab.data_ptr()
    seen = set()
    i = 0
    for layer in range(2):
        for a in range(w.n_adapters):
            for e in range(w.n_experts):
                for j in range(3):
                    lay = L.lora_pool_unit_layout(dp.pool, a, layer, e, j)
                    assert ent["A"][i] == base + lay["A_offset"]
                    assert ent["B"][i] == base + lay["B_offset"]
                    assert ent["scale"][i] == scale[a] and ent["rank"][i] == 16
                    assert lay["A_offset"] % 256 == 0 and lay["B_offset"] % 256 == 0
                    assert lay["A_offset"] + lay["A_bytes"] <= dp.nbytes
                    assert lay["B_offset"] + lay["B_bytes"] <= dp.nbytes
                    for lo, n in ((lay["A_offset"], lay["A_bytes"]), (lay["B_offset"], lay["B_bytes"])):
                        assert not any(lo < hi2 and lo2 < lo + n for lo2, hi2 in seen)
                        seen.add((lo, lo + n))
                    i += 1


def test_register_with_pointer_arrays_equals_layerwise_loading():
    w = small_workload(8, E=2, n=2)
    ws = W.make_weights(w, 7, n_layers=1, bank_elems=1 << 18)
    dp = DevicePool(ws, np.ones(2, np.float32))
    desc = L.PoolDesc(2, 1, 2, [(p.h_in, p.h_out) for p in w.projs], 8, scale=[1.0, 1.0])
    slab = torch.zeros(L.lora_pool_bytes(desc), dtype=torch.uint8, device="cuda")
    keep, A_src, B_src = [], [], []
    for a in range(2):
        for e in range(2):
            for j in range(3):
                A, B = ws.unit_arrays(a, 0, e, j)
                tA, tB = to_dev(np.ascontiguousarray(A)), to_dev(np.ascontiguousarray(B))
                keep += [tA, tB]
                A_src.append(tA)
                B_src.append(tB)
    pool = L.lora_register_pool(desc, slab, A_src=A_src, B_src=B_src)
    torch.cuda.synchronize()
    n_table = 2 * 2 * 3 * 32
    # tables differ only in the absolute addresses; packed data must be identical
    assert torch.equal(slab[256 * ((n_table + 255) // 256):], dp.slab[256 * ((n_table + 255) // 256):])
    del pool


def test_lower_adapter_rank_is_zero_padded():
    w = small_workload(16, E=1, n=2)
    w4 = W.scaled(w, rank=8)           # source matrices of rank 8 inside a rank-16 pool
    ws = W.make_weights(w4, 8, n_layers=1, bank_elems=1 << 18)
    desc = L.PoolDesc(2, 1, 1, [(p.h_in, p.h_out) for p in w.projs], 16, adapter_rank=[8, 8])
    slab = torch.empty(L.lora_pool_bytes(desc), dtype=torch.uint8, device="cuda")
    pool = L.lora_register_pool(desc, slab)
    bank = to_dev(ws.bank)
    for a in range(2):
        L.lora_pool_load_adapter_layer(pool, a, 0, bank.data_ptr() + 2 * int(ws.window[a, 0]))
    p = w.projs[0]
    A_out = torch.full((p.h_in, 16), -1, dtype=torch.int16, device="cuda")
    B_out = torch.full((16, p.h_out), -1, dtype=torch.int16, device="cuda")
    L.lora_pool_read_unit(pool, 1, 0, 0, 0, A_out, B_out)
    torch.cuda.synchronize()
    A, B = ws.unit_arrays(1, 0, 0, 0)
    assert np.array_equal(bits_from_dev(A_out)[:, :8], A) and not bits_from_dev(A_out)[:, 8:].any()
    assert np.array_equal(bits_from_dev(B_out)[:8], B) and not bits_from_dev(B_out)[8:].any()
    assert L.lora_pool_unit_layout(pool, 1, 0, 0, 0)["rank"] == 8


def test_layerwise_loading_on_a_second_stream_overlaps_with_compute():
    """Sec. 5.3: an adapter is loaded layer by layer while earlier layers already compute.
    Host-pinned windows are copied and repacked on a loading stream, one event per layer; the
    compute stream waits for a layer's event, then runs that layer.  Every layer's output
    must match the oracle."""
    from gpu_common import check_accumulate, oracle_projection
    from harness import DeviceBatch, LayerRunner

    n_layers = 4
    w = W.Workload("t", "dense", 6, 1, 1, 16, (W.Proj("p", 264, 392, "x"),), 80, "uniform", 0.0)
    b = W.make_batch(w, 71, y_mode="normal", hetero_scale=True)
    ws = W.make_weights(w, 71, n_layers=n_layers, bank_elems=1 << 20)
    desc = L.PoolDesc(w.n_adapters, n_layers, 1, [(264, 392)], 16, scale=[float(s) for s in b.scale])
    slab = torch.zeros(L.lora_pool_bytes(desc), dtype=torch.uint8, device="cuda")
    pool = L.lora_register_pool(desc, slab)
    torch.cuda.synchronize()

    win = (264 + 392) * 16                                  # elements of one (adapter, layer) window
    host = [[torch.from_numpy(ws.bank[int(ws.window[a, l]):int(ws.window[a, l]) + win].view(np.int16).copy())
             .pin_memory() for a in range(w.n_adapters)] for l in range(n_layers)]
    staging = [[torch.empty(win, dtype=torch.int16, device="cuda") for _ in range(w.n_adapters)]
               for _ in range(n_layers)]
    load_stream, compute_stream = torch.cuda.Stream(), torch.cuda.Stream()
    ready = [torch.cuda.Event() for _ in range(n_layers)]

    db = DeviceBatch(b)
    holder = type("P", (), {})()                            # what LayerRunner needs of a DevicePool
    holder.workload, holder.pool, holder.device = w, pool, "cuda"
    run = LayerRunner(holder, db)
    ys = []
    with torch.cuda.stream(load_stream):
        for l in range(n_layers):
            for a in range(w.n_adapters):
                staging[l][a].copy_(host[l][a], non_blocking=True)
                L.lora_pool_load_adapter_layer(pool, a, l, staging[l][a], stream=load_stream)
            ready[l].record(load_stream)
    with torch.cuda.stream(compute_stream):
        run.build_segments(stream=compute_stream)
        for l in range(n_layers):
            compute_stream.wait_event(ready[l])
            y = to_dev(b.y_in["p"])
            x = db.inputs["x"]
            L.lora_apply(pool, l, 0, x, x.shape[1], None, db.seg, y, y.shape[1], run.v,
                         stream=compute_stream)
            ys.append(y)
    torch.cuda.synchronize()
    for l in range(n_layers):
        check_accumulate(bits_from_dev(ys[l]), oracle_projection(b, ws, l, 0), f"layer {l}")


def _async_case(n_layers=5, n_experts=3, seed=83):
    w = W.Workload("t", "moe", 4, n_experts, 2, 16,
                   (W.Proj("up", 136, 264, "x"), W.Proj("down", 264, 136, "h")), 48, "uniform", 0.0)
    b = W.make_batch(w, seed, y_mode="normal", hetero_scale=True)
    ws = W.make_weights(w, seed, n_layers=n_layers, bank_elems=1 << 21)
    desc = L.PoolDesc(w.n_adapters, n_layers, n_experts, [(136, 264), (264, 136)], 16,
                      scale=[float(s) for s in b.scale])
    slab = torch.zeros(L.lora_pool_bytes(desc), dtype=torch.uint8, device="cuda")
    pool = L.lora_register_pool(desc, slab)
    torch.cuda.synchronize()
    return w, b, ws, pool, slab


def test_async_adapter_load_layer_by_layer_matches_oracle():
    """Sec. 5.3 through the library's own calls: every adapter is loaded from pinned host
    memory on a loading stream, layer after layer; the compute stream waits for a layer of
    all adapters, then runs that layer.  Every layer's output must match the oracle."""
    from gpu_common import check_accumulate, oracle_projection
    from harness import DeviceBatch

    n_layers = 5
    w, b, ws, pool, slab = _async_case(n_layers)
    window = L.lora_pool_adapter_layer_bytes(pool, 0)
    assert window == w.n_experts * sum((p.h_in + p.h_out) * 16 for p in w.projs) * 2
    win = window // 2
    host = []
    for a in range(w.n_adapters):
        rows = [ws.bank[int(ws.window[a, l]):int(ws.window[a, l]) + win].view(np.int16) for l in range(n_layers)]
        host.append(torch.from_numpy(np.concatenate(rows)).pin_memory())
    staging = [torch.empty(win, dtype=torch.int16, device="cuda") for _ in range(w.n_adapters)]
    load_stream, compute_stream = torch.cuda.Stream(), torch.cuda.Stream()

    db = DeviceBatch(b)
    v = torch.empty(max(L.lora_v_bytes(pool, 0, db.P), 256) // 4, dtype=torch.float32, device="cuda")
    assert L.lora_pool_layer_ready(pool, 0, 0)              # nothing enqueued yet
    for a in range(w.n_adapters):
        L.lora_pool_load_adapter_async(pool, a, host[a], staging[a], load_stream=load_stream)
    ys = []
    with torch.cuda.stream(compute_stream):
        L.lora_build_segments(pool, db.adapter_id, db.expert_id, db.P, db.seg, stream=compute_stream)
        for l in range(n_layers):
            for a in range(w.n_adapters):
                L.lora_pool_wait_layer(pool, a, l, stream=compute_stream)
            y = to_dev(b.y_in["up"])
            x = db.inputs["x"]
            L.lora_apply(pool, l, 0, x, x.shape[1], db.token_of_pair, db.seg, y, y.shape[1], v,
                         stream=compute_stream)
            ys.append(y)
    torch.cuda.synchronize()
    assert all(L.lora_pool_layer_ready(pool, a, l) for a in range(w.n_adapters) for l in range(n_layers))
    for l in range(n_layers):
        check_accumulate(bits_from_dev(ys[l]), oracle_projection(b, ws, l, 0), f"layer {l}")
    # the repacked units read back bit-exact
    p0 = w.projs[0]
    A_out = torch.empty((p0.h_in, 16), dtype=torch.int16, device="cuda")
    B_out = torch.empty((16, p0.h_out), dtype=torch.int16, device="cuda")
    L.lora_pool_read_unit(pool, 2, n_layers - 1, 1, 0, A_out, B_out)
    torch.cuda.synchronize()
    A, B = ws.unit_arrays(2, n_layers - 1, 1, 0)
    assert np.array_equal(bits_from_dev(A_out), A) and np.array_equal(bits_from_dev(B_out), B)


def test_async_load_replaces_an_adapter_in_its_slot():
    """A second load into the same slot (eviction) ordered behind the work that used the
    first: results switch from the first adapter's weights to the second's."""
    from gpu_common import check_accumulate, oracle_projection
    from harness import DeviceBatch

    n_layers = 2
    w, b, ws, pool, slab = _async_case(n_layers, seed=85)
    ws2 = W.make_weights(w, 86, n_layers=n_layers, bank_elems=1 << 21)
    win = L.lora_pool_adapter_layer_bytes(pool, 0) // 2

    def pinned(src, a):
        rows = [src.bank[int(src.window[a, l]):int(src.window[a, l]) + win].view(np.int16) for l in range(n_layers)]
        return torch.from_numpy(np.concatenate(rows)).pin_memory()

    staging = torch.empty(win, dtype=torch.int16, device="cuda")
    stream = torch.cuda.Stream()
    db = DeviceBatch(b)
    v = torch.empty(max(L.lora_v_bytes(pool, 0, db.P), 256) // 4, dtype=torch.float32, device="cuda")
    keep = []
    for src in (ws, ws2):
        hosts = [pinned(src, a) for a in range(w.n_adapters)]
        keep.append(hosts)
        with torch.cuda.stream(stream):
            for a in range(w.n_adapters):           # one staging window, one stream: loads are ordered
                L.lora_pool_load_adapter_async(pool, a, hosts[a], staging, load_stream=stream)
            L.lora_build_segments(pool, db.adapter_id, db.expert_id, db.P, db.seg, stream=stream)
            y = to_dev(b.y_in["up"])
            x = db.inputs["x"]
            L.lora_apply(pool, 1, 0, x, x.shape[1], db.token_of_pair, db.seg, y, y.shape[1], v, stream=stream)
        torch.cuda.synchronize()
        check_accumulate(bits_from_dev(y), oracle_projection(b, src, 1, 0), "slot contents")


def test_slot_replacement_with_another_rank_and_scale():
    """Sec. 4.2: the resident set changes over time.  A slot that held a rank-16 adapter takes a
    rank-8 adapter with another scale: lora_pool_set_adapter rewrites the slot's table entries
    and the source stride of later loads, the load zero-pads the lower rank.  Rows of the
    replaced slot must follow the new adapter and scale, all other rows stay as they were."""
    from gpu_common import check_accumulate, check_delta, oracle_projection
    from harness import DeviceBatch

    n_layers, slot, new_scale = 2, 1, 0.75
    w, b, ws, pool, slab = _async_case(n_layers, seed=87)
    w8 = W.scaled(w, rank=8)
    ws8 = W.make_weights(w8, 88, n_layers=n_layers, bank_elems=1 << 21)
    win = L.lora_pool_adapter_layer_bytes(pool, 0) // 2

    def pinned(src, a, n):
        rows = [src.bank[int(src.window[a, l]):int(src.window[a, l]) + n].view(np.int16) for l in range(n_layers)]
        return torch.from_numpy(np.concatenate(rows)).pin_memory()

    staging = torch.empty(win, dtype=torch.int16, device="cuda")
    stream = torch.cuda.Stream()
    b0 = W.make_batch(w, 87, y_mode="zero", hetero_scale=True)
    assert (b0.adapter_id == slot).any() and (b0.adapter_id != slot).any()
    db = DeviceBatch(b0)
    v = torch.empty(max(L.lora_v_bytes(pool, 0, db.P), 256) // 4, dtype=torch.float32, device="cuda")
    hosts = [pinned(ws, a, win) for a in range(w.n_adapters)]
    with torch.cuda.stream(stream):
        for a in range(w.n_adapters):
            L.lora_pool_load_adapter_async(pool, a, hosts[a], staging, load_stream=stream)
        # the replacement: table first, then the load that reads its source at the new rank
        L.lora_pool_set_adapter(pool, slot, 8, new_scale, stream=stream)
        win8 = L.lora_pool_adapter_layer_bytes(pool, slot) // 2
        assert win8 * 2 == win
        host8 = pinned(ws8, slot, win8)
        L.lora_pool_load_adapter_async(pool, slot, host8, staging, load_stream=stream)
        L.lora_build_segments(pool, db.adapter_id, db.expert_id, db.P, db.seg, stream=stream)
        y = to_dev(b0.y_in["up"])
        x = db.inputs["x"]
        L.lora_apply(pool, 1, 0, x, x.shape[1], db.token_of_pair, db.seg, y, y.shape[1], v, stream=stream)
    torch.cuda.synchronize()
    lay = L.lora_pool_unit_layout(pool, slot, 1, 2, 0)
    assert lay["rank"] == 8 and lay["scale"] == new_scale
    assert L.lora_pool_unit_layout(pool, 0, 1, 2, 0)["rank"] == 16
    got = W.bf16_bits_to_f32(bits_from_dev(y)).astype(np.float64)
    mine = np.flatnonzero(b0.adapter_id == slot)
    rest = np.flatnonzero(b0.adapter_id != slot)
    b_new = W.Batch(w, b0.adapter_id, b0.expert_id, b0.token_of_pair, b0.inputs, b0.y_in, b0.scale.copy())
    b_new.scale[slot] = new_scale
    check_delta(got[mine], oracle_projection(b_new, ws8, 1, 0, rows=mine).delta, "replaced slot")
    check_delta(got[rest], oracle_projection(b0, ws, 1, 0, rows=rest).delta, "other slots")
    # the padding rank entries of the slot read back as zeros
    p0 = w.projs[0]
    A_out = torch.full((p0.h_in, 16), -1, dtype=torch.int16, device="cuda")
    B_out = torch.full((16, p0.h_out), -1, dtype=torch.int16, device="cuda")
    L.lora_pool_read_unit(pool, slot, 1, 2, 0, A_out, B_out)
    torch.cuda.synchronize()
    A, B = ws8.unit_arrays(slot, 1, 2, 0)
    assert np.array_equal(bits_from_dev(A_out)[:, :8], A) and not bits_from_dev(A_out)[:, 8:].any()
    assert np.array_equal(bits_from_dev(B_out)[:8], B) and not bits_from_dev(B_out)[8:].any()
    for args, status in [((slot, 0, 1.0), -3), ((slot, 17, 1.0), -3), ((99, 8, 1.0), -2),
                         ((slot, 8, float("nan")), -1)]:
        with pytest.raises(L.LoraError) as e:
            L.lora_pool_set_adapter(pool, *args)
        assert e.value.status == status, args


def test_async_load_argument_errors():
    w, b, ws, pool, slab = _async_case(2)
    win = L.lora_pool_adapter_layer_bytes(pool, 0) // 2
    host = torch.zeros(2 * win, dtype=torch.int16).pin_memory()
    small = torch.empty(win - 8, dtype=torch.int16, device="cuda")
    ok = torch.empty(win, dtype=torch.int16, device="cuda")
    with pytest.raises(L.LoraError):
        L.lora_pool_load_adapter_async(pool, 0, host, small)
    with pytest.raises(L.LoraError):
        L.lora_pool_load_adapter_async(pool, 99, host, ok)
    with pytest.raises(L.LoraError):
        L.lora_pool_wait_layer(pool, 0, 7)
    with pytest.raises(L.LoraError):
        L.lora_pool_layer_ready(pool, -1, 0)
    assert L.lora_pool_adapter_layer_bytes(pool, 99) == 0
    torch.cuda.synchronize()
