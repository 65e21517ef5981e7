"""Shrink and expand as one launch (small decode batches with short inputs and narrow outputs)
against the oracle and against the two-launch path, on both sides of every limit that decides
which of the two runs."""
import numpy as np
import pytest
import torch

import paper_2604_07173_amd as L
import workloads as W
from gpu_common import bf16_ulp, check_accumulate, check_delta, oracle_projection
from harness import DeviceBatch, DevicePool, LayerRunner, bits_from_dev, to_dev

pytestmark = pytest.mark.gpu


def two_launch_reference(dp, db, run, j, c, layer=0):
    """The same group through lora_shrink + lora_expand per projection (always two launches)."""
    w = dp.workload
    outs = {}
    for q in range(j, j + c):
        p = w.projs[q]
        x = db.inputs[p.input]
        y = to_dev(db.batch.y_in[p.name])
        v = torch.empty(max(L.lora_v_bytes(dp.pool, q, db.P), 256) // 4, dtype=torch.float32, device="cuda")
        src = db.token_of_pair if w.kind == "moe" and p.input != "mid" else None
        L.lora_shrink(dp.pool, layer, q, x, x.shape[1], src, db.seg, v)
        L.lora_expand(dp.pool, layer, q, v, db.seg, y, y.shape[1])
        outs[p.name] = y
    torch.cuda.synchronize()
    return outs


def close_to(a_bits, b_bits):
    a = W.bf16_bits_to_f32(a_bits).astype(np.float64)
    b = W.bf16_bits_to_f32(b_bits).astype(np.float64)
    # the same sums in another fp32 order: one bf16 step where the value is of normal size; where
    # terms cancel, what remains is the fp32 rounding of the row's largest values
    row = np.maximum(np.abs(a).max(axis=1, keepdims=True), np.abs(b).max(axis=1, keepdims=True))
    bound = bf16_ulp(np.maximum(np.abs(a), np.abs(b))) + 3e-5 * row
    assert (np.abs(a - b) <= bound).all() and (a_bits != b_bits).mean() < 0.02


CASES = [
    # rank, h_in, widths of the group, adapters, tokens, one launch expected
    (8, 200, (328,), 5, 70, True),
    (16, 1032, (392, 136, 136), 7, 90, True),           # q/k/v-like group, ragged K
    (32, 264, (520, 136), 6, 40, True),
    (64, 4096, (1032,), 3, 33, True),                   # the longest input still taken
    (16, 4104, (392,), 4, 40, False),                   # input too long
    (16, 264, (8200,), 4, 40, False),                   # output too wide (65 chunks)
    (16, 264, (392,), 60, 200, False),                  # too many tiles (bound 60 + 12)
    (16, 264, (392,), 40, 300, True),                   # bound 40 + 18 = 58 tiles, several per segment
]


@pytest.mark.parametrize("y_mode", ["zero", "normal"])
@pytest.mark.parametrize("rank,h_in,widths,n,tokens,one", CASES)
def test_group_in_one_launch_matches_oracle_and_two_launches(rank, h_in, widths, n, tokens, one, y_mode):
    projs = tuple(W.Proj(f"p{i}", h_in, h, "x") for i, h in enumerate(widths))
    w = W.Workload("t", "dense", n, 1, 1, rank, projs, tokens, "zipf", 0.8)
    b = W.make_batch(w, 7, y_mode=y_mode, no_adapter_frac=0.1, hetero_scale=True)
    ws = W.make_weights(w, 7, n_layers=2, bank_elems=1 << 22)
    dp, db = DevicePool(ws, b.scale), DeviceBatch(b)
    run = LayerRunner(dp, db)
    run.build_segments()
    assert run.groups == [(0, len(widths))]
    assert (L.lora_group_launches(dp.pool, 0, len(widths), tokens, db.seg) == 1) == one
    run.v.fill_(float("nan"))                           # one launch must not depend on the workspace
    run.apply(1)
    torch.cuda.synchronize()
    ref = two_launch_reference(dp, db, run, 0, len(widths), layer=1)
    none = b.adapter_id < 0
    for j, p in enumerate(projs):
        got = bits_from_dev(db.y[p.name])
        res = oracle_projection(b, ws, 1, j)
        if y_mode == "zero":
            check_delta(W.bf16_bits_to_f32(got).astype(np.float64), res.delta, f"one launch r{rank} {p.name}")
        else:
            check_accumulate(got, res, f"one launch r{rank} {p.name}")
        assert np.array_equal(got[none], b.y_in[p.name][none])
        if one:
            close_to(got, bits_from_dev(ref[p.name]))
        else:
            assert np.array_equal(got, bits_from_dev(ref[p.name]))


def test_moe_application_in_one_launch():
    """lora_moe_apply on a small MoE batch: up/gate (two projections sharing the gathered token
    rows) and down each run as one launch."""
    projs = (W.Proj("gate", 520, 1160, "x"), W.Proj("up", 520, 1160, "x"), W.Proj("down", 1160, 520, "mid"))
    w = W.Workload("t", "moe", 6, 4, 2, 16, projs, 24, "zipf", 1.0)
    for y_mode in ("zero", "normal"):
        b = W.make_batch(w, 11, y_mode=y_mode, no_adapter_frac=0.1, hetero_scale=True)
        ws = W.make_weights(w, 11, bank_elems=1 << 22)
        dp, db = DevicePool(ws, b.scale), DeviceBatch(b)
        run = LayerRunner(dp, db)
        run.build_segments()
        assert L.lora_group_launches(dp.pool, 0, 2, db.P, db.seg) == 1
        assert L.lora_group_launches(dp.pool, 2, 1, db.P, db.seg) == 1
        run.apply(0)
        torch.cuda.synchronize()
        for j, p in enumerate(projs):
            got = bits_from_dev(db.y[p.name])
            res = oracle_projection(b, ws, 0, j)
            if y_mode == "zero":
                check_delta(W.bf16_bits_to_f32(got).astype(np.float64), res.delta, f"one launch moe {p.name}")
            else:
                check_accumulate(got, res, f"one launch moe {p.name}")


def test_one_launch_is_bit_identical_run_to_run_and_in_a_graph():
    w = W.Workload("t", "dense", 9, 1, 1, 16, (W.Proj("p", 1032, 392, "x"),), 100, "zipf", 1.0)
    b = W.make_batch(w, 13, y_mode="normal", no_adapter_frac=0.05)
    ws = W.make_weights(w, 13, bank_elems=1 << 21)
    dp, db = DevicePool(ws, b.scale), DeviceBatch(b)
    run = LayerRunner(dp, db)
    run.step(0)
    torch.cuda.synchronize()
    assert L.lora_group_launches(dp.pool, 0, 1, db.P, db.seg) == 1
    want = db.y["p"].clone()
    for _ in range(2):
        db.reset_y()
        run.step(0)
        torch.cuda.synchronize()
        assert torch.equal(db.y["p"], want)
    db.reset_y()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run.step(0)
    torch.cuda.synchronize()
    for replay in range(3):
        db.reset_y()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(db.y["p"], want), replay
    check_accumulate(bits_from_dev(db.y["p"]), oracle_projection(b, ws, 0, 0), "one launch in a graph")


def test_f32_output_and_long_segments_take_two_or_more_launches(monkeypatch):
    w = W.Workload("t", "dense", 2, 1, 1, 16, (W.Proj("p", 264, 392, "x"),), 40, "uniform", 0.0)
    b = W.make_batch(w, 17)
    dp, db = DevicePool(W.make_weights(w, 17, bank_elems=1 << 20), b.scale), DeviceBatch(b)
    LayerRunner(dp, db).build_segments()
    assert L.lora_group_launches(dp.pool, 0, 1, db.P, db.seg) == 1
    assert L.lora_group_launches(dp.pool, 0, 1, db.P, db.seg, L.LORA_DTYPE_F32) == 2
    monkeypatch.setenv("LORA_TILE_ROWS", "32")        # the long-segment kernels, forced for so few rows
    w2 = W.scaled(w, tokens=400)
    b2 = W.make_batch(w2, 17)
    db2 = DeviceBatch(b2)
    LayerRunner(dp, db2).build_segments()
    assert db2.seg.c.tile_rows == 32
    assert L.lora_group_launches(dp.pool, 0, 1, db2.P, db2.seg) == 3
    with pytest.raises(L.LoraError):
        L.lora_group_launches(dp.pool, 0, 2, db.P, db.seg)
