"""lora_moe_apply_static (the workspace is a device array inside the library, the call allocates
nothing) against lora_moe_apply with a caller-provided workspace: same kernels, so the outputs
must agree bit for bit, on two calls in a row of which the second is smaller, and both must
meet the delta tolerance against the oracle."""
import numpy as np
import pytest
import torch

import paper_2604_07173_amd as L
import workloads as W
from gpu_common import check_delta, oracle_projection
from harness import DeviceBatch, DevicePool, bits_from_dev, to_dev

pytestmark = pytest.mark.gpu


def moe_layer(dp, db, layer, static, ws=None):
    """Segments, up/gate and down of one batch through one of the two entry points; returns
    fresh output tensors."""
    b = db.batch
    L.lora_build_segments(dp.pool, db.adapter_id, db.expert_id, db.P, db.seg)
    y = {k: to_dev(v) for k, v in b.y_in.items()}
    x, mid = db.inputs["x"], db.inputs["mid"]
    ldy_u, ldy_d = y["gate"].shape[1], y["down"].shape[1]
    if static:
        L.lora_moe_apply_static(dp.pool, layer, L.LORA_MOE_UPGATE, x, x.shape[1], db.token_of_pair,
                                db.seg, y["gate"], y["up"], ldy_u)
        L.lora_moe_apply_static(dp.pool, layer, L.LORA_MOE_DOWN, mid, mid.shape[1], None, db.seg,
                                y["down"], None, ldy_d)
    else:
        L.lora_moe_apply(dp.pool, layer, L.LORA_MOE_UPGATE, x, x.shape[1], db.token_of_pair, db.seg,
                         y["gate"], y["up"], ldy_u, ws)
        L.lora_moe_apply(dp.pool, layer, L.LORA_MOE_DOWN, mid, mid.shape[1], None, db.seg,
                         y["down"], None, ldy_d, ws)
    torch.cuda.synchronize()
    return y


def test_static_workspace_entry_point_matches_the_workspace_one():
    projs = (W.Proj("gate", 520, 1160, "x"), W.Proj("up", 520, 1160, "x"), W.Proj("down", 1160, 520, "mid"))
    big = W.Workload("t", "moe", 12, 4, 2, 16, projs, 300, "zipf", 1.0)
    small = W.scaled(big, tokens=37)
    ws_src = W.make_weights(big, 91, n_layers=2, bank_elems=1 << 22)
    batches = [W.make_batch(big, 91, y_mode="zero", no_adapter_frac=0.05, hetero_scale=True),
               W.make_batch(small, 92, y_mode="zero", no_adapter_frac=0.05, hetero_scale=True)]
    dp = DevicePool(ws_src, batches[0].scale)
    dbs = [DeviceBatch(b) for b in batches]
    # reference results first, each with a workspace of its own
    want = []
    for db in dbs:
        ws = torch.empty(L.lora_moe_ws_bytes(dp.pool, db.P), dtype=torch.uint8, device="cuda")
        want.append(moe_layer(dp, db, 1, static=False, ws=ws))
    # the two static calls in a row: the larger batch, then the smaller one (the array still
    # holds the larger one's intermediates)
    print("static call 1: P =", dbs[0].P, flush=True)
    got0 = moe_layer(dp, dbs[0], 1, static=True)
    print("static call 2: P =", dbs[1].P, flush=True)
    got1 = moe_layer(dp, dbs[1], 1, static=True)
    for got, ref, b, tag in ((got0, want[0], batches[0], "first"), (got1, want[1], batches[1], "second")):
        for j, p in enumerate(big.projs):
            assert torch.equal(got[p.name], ref[p.name]), f"{tag} call, {p.name}"
            res = oracle_projection(b, ws_src, 1, j)
            check_delta(W.bf16_bits_to_f32(bits_from_dev(got[p.name])).astype(np.float64), res.delta,
                        f"static {tag}/{p.name}")
            none = b.adapter_id < 0
            assert not bits_from_dev(got[p.name])[none].any()


def test_static_workspace_entry_point_rejects_what_does_not_fit():
    """A batch whose intermediates exceed the array is refused on the host, before any device
    work; argument mistakes give the same codes as lora_moe_apply."""
    projs = (W.Proj("gate", 64, 64, "x"), W.Proj("up", 64, 64, "x"), W.Proj("down", 64, 64, "mid"))
    w = W.Workload("t", "moe", 8, 2, 1, 64, projs, 16, "uniform")
    b = W.make_batch(w, 93, y_mode="zero")
    dp = DevicePool(W.make_weights(w, 93, bank_elems=1 << 18), b.scale)
    P = L.LORA_MAX_ROWS                                  # long segments: parts and operand images
    assert L.lora_moe_ws_bytes(dp.pool, P) > L.LORA_STATIC_WS_BYTES
    rng = np.random.default_rng(93)
    aid = to_dev(rng.integers(0, 8, size=P).astype(np.int32))
    eid = to_dev(rng.integers(0, 2, size=P).astype(np.int32))
    seg = L.Segments(P)
    L.lora_build_segments(dp.pool, aid, eid, P, seg)
    x = torch.zeros((P, 64), dtype=torch.int16, device="cuda")
    y0, y1 = torch.zeros_like(x), torch.zeros_like(x)
    tok = to_dev(np.arange(P, dtype=np.int32))
    with pytest.raises(L.LoraError) as e:
        L.lora_moe_apply_static(dp.pool, 0, L.LORA_MOE_UPGATE, x, 64, tok, seg, y0, y1, 64)
    assert e.value.status == -8
    torch.cuda.synchronize()
    assert not y0.any() and not y1.any()
    small = DeviceBatch(b)
    L.lora_build_segments(dp.pool, small.adapter_id, small.expert_id, small.P, small.seg)
    with pytest.raises(L.LoraError) as e:               # bad projection selector
        L.lora_moe_apply_static(dp.pool, 0, 5, small.inputs["x"], 64, small.token_of_pair, small.seg,
                                small.y["gate"], small.y["up"], 64)
    assert e.value.status == -1
    with pytest.raises(L.LoraError) as e:               # layer out of range
        L.lora_moe_apply_static(dp.pool, 3, L.LORA_MOE_DOWN, small.inputs["mid"], 64, None, small.seg,
                                small.y["down"], None, 64)
    assert e.value.status == -2
