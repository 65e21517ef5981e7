"""lora_pool_set_activation_policy: the cache hints on the activation streams change where rows
are kept, never what is computed.  Every policy gives bit-identical outputs; the streaming forms
of the kernels are also compared with the fp64 oracle."""
import numpy as np
import pytest
import torch

import paper_2604_07173_amd as L
import workloads as W
from gpu_common import check_accumulate, check_delta, oracle_projection
from harness import DeviceBatch, DevicePool, LayerRunner, bits_from_dev, to_dev

pytestmark = pytest.mark.gpu

POLICIES = (L.LORA_ACT_AUTO, L.LORA_ACT_RESIDENT, L.LORA_ACT_STREAMING)


def test_policy_is_kept_and_checked():
    w = W.Workload("t", "dense", 3, 1, 1, 8, (W.Proj("p", 40, 24, "x"),), 16, "uniform", 0.0)
    b = W.make_batch(w, 1)
    dp = DevicePool(W.make_weights(w, 1, bank_elems=1 << 16), b.scale)
    assert L.lora_pool_activation_policy(dp.pool) == L.LORA_ACT_AUTO
    for p in POLICIES:
        L.lora_pool_set_activation_policy(dp.pool, p)
        assert L.lora_pool_activation_policy(dp.pool) == p
    with pytest.raises(L.LoraError) as e:
        L.lora_pool_set_activation_policy(dp.pool, 3)
    assert e.value.status == -1
    assert L.lora_pool_activation_policy(dp.pool) == L.LORA_ACT_STREAMING


@pytest.mark.parametrize("rank", [8, 16, 64])
@pytest.mark.parametrize("y_mode", ["zero", "normal"])
def test_moe_layer_is_bit_identical_under_every_policy(rank, y_mode):
    """Both MoE applications of a layer (264 -> 520 -> 264, 6 adapters x 4 experts, 640 tokens x
    top-2: too many tiles for the one-launch kernel, which has no streaming form) under the three
    policies: the streaming one against the oracle, the others bit for bit against it."""
    projs = (W.Proj("gate", 264, 520, "x"), W.Proj("up", 264, 520, "x"), W.Proj("down", 520, 264, "mid"))
    w = W.Workload("t", "moe", 6, 4, 2, rank, projs, 640, "zipf", 1.0)
    b = W.make_batch(w, 11, y_mode=y_mode, no_adapter_frac=0.05, hetero_scale=True)
    ws = W.make_weights(w, 11, bank_elems=1 << 20)
    dp, db = DevicePool(ws, b.scale), DeviceBatch(b)
    run = LayerRunner(dp, db)
    out = {}
    for policy in POLICIES:
        L.lora_pool_set_activation_policy(dp.pool, policy)
        db.reset_y()
        run.step(0)
        assert L.lora_group_launches(dp.pool, 0, 2, db.P, db.seg) == 2
        assert L.lora_group_launches(dp.pool, 2, 1, db.P, db.seg) == 2
        torch.cuda.synchronize()
        out[policy] = {p.name: bits_from_dev(db.y[p.name]).copy() for p in w.projs}
    for j, p in enumerate(w.projs):
        res = oracle_projection(b, ws, 0, j)
        got = out[L.LORA_ACT_STREAMING][p.name]
        if y_mode == "zero":
            check_delta(W.bf16_bits_to_f32(got).astype(np.float64), res.delta, f"streaming policy r{rank}/{p.name}")
        else:
            check_accumulate(got, res, f"streaming policy r{rank}/{p.name}")
        for policy in POLICIES:
            assert np.array_equal(out[policy][p.name], got), (policy, p.name)


def test_fp32_output_and_two_call_path_under_the_streaming_policy():
    """lora_shrink + lora_expand with fp32 output rows, streaming policy against resident."""
    w = W.Workload("t", "dense", 5, 1, 1, 32, (W.Proj("p", 200, 328, "x"),), 70, "uniform", 0.0)
    b = W.make_batch(w, 5, y_mode="normal", hetero_scale=True)
    ws = W.make_weights(w, 5, bank_elems=1 << 20)
    dp, db = DevicePool(ws, b.scale), DeviceBatch(b)
    run = LayerRunner(dp, db)
    run.build_segments()
    x = db.inputs["x"]
    got = {}
    for policy in (L.LORA_ACT_RESIDENT, L.LORA_ACT_STREAMING):
        L.lora_pool_set_activation_policy(dp.pool, policy)
        y = torch.from_numpy(W.bf16_bits_to_f32(b.y_in["p"])).cuda()
        L.lora_shrink(dp.pool, 0, 0, x, x.shape[1], None, db.seg, run.v)
        L.lora_expand(dp.pool, 0, 0, run.v, db.seg, y, y.shape[1], L.LORA_DTYPE_F32)
        torch.cuda.synchronize()
        got[policy] = y.cpu().numpy()
    assert np.array_equal(got[L.LORA_ACT_RESIDENT], got[L.LORA_ACT_STREAMING])
    res = oracle_projection(b, ws, 0, 0)
    assert np.abs(got[L.LORA_ACT_STREAMING] - res.y_out).max() <= 2e-2


def test_routing_weighted_combine_under_the_streaming_policy():
    """lora_moe_down_combine (its expand writes the pair rows instead of updating them)."""
    from test_gpu_combine import moe_workload, routing_weights
    w = moe_workload(16, 136, 264, 6, 4, 2, 64)
    b = W.make_batch(w, 3, y_mode="zero", no_adapter_frac=0.1, hetero_scale=True)
    dp = DevicePool(W.make_weights(w, 3, bank_elems=1 << 20), b.scale)
    db = DeviceBatch(b)
    L.lora_build_segments(dp.pool, db.adapter_id, db.expert_id, db.P, db.seg)
    ws = torch.empty(L.lora_moe_combine_ws_bytes(dp.pool, db.P), dtype=torch.uint8, device="cuda")
    route_w = to_dev(routing_weights(w, 3))
    mid = db.inputs["mid"]
    got = {}
    for policy in (L.LORA_ACT_RESIDENT, L.LORA_ACT_STREAMING):
        L.lora_pool_set_activation_policy(dp.pool, policy)
        ws.fill_(0xFF)
        y = torch.zeros((w.tokens, 136), dtype=torch.int16, device="cuda")
        L.lora_moe_down_combine(dp.pool, 0, mid, mid.shape[1], db.adapter_id, db.expert_id, db.seg,
                                route_w, w.top_k, y, 136, ws)
        torch.cuda.synchronize()
        got[policy] = bits_from_dev(y).copy()
    assert got[L.LORA_ACT_RESIDENT].any()
    assert np.array_equal(got[L.LORA_ACT_RESIDENT], got[L.LORA_ACT_STREAMING])


def test_rows_beyond_the_thresholds_are_streamed_by_default():
    """4096 rows of 8192 inputs (64 MiB, read once) and 32768 outputs (256 MiB) over 256 adapters at
    rank 16: the default policy streams both; bit-identical to the resident policy, sampled rows
    against the oracle."""
    w = W.Workload("t", "dense", 256, 1, 1, 16, (W.Proj("p", 8192, 32768, "x"),), 4096, "zipf", 0.8)
    assert w.pairs * 8192 * 2 >= 64 << 20 and w.pairs * 32768 * 2 >= 256 << 20
    print("[cache policy] 4096 x 8192 -> 32768 batch...", flush=True)
    b = W.make_batch(w, 9, y_mode="zero")
    ws = W.make_weights(w, 9, bank_elems=1 << 22)
    dp, db = DevicePool(ws, b.scale), DeviceBatch(b)
    run = LayerRunner(dp, db)
    out = {}
    for policy in (L.LORA_ACT_AUTO, L.LORA_ACT_RESIDENT):
        print(f"[cache policy] policy {policy}...", flush=True)
        L.lora_pool_set_activation_policy(dp.pool, policy)
        db.y["p"].zero_()
        run.step(0, one_call=False)
        torch.cuda.synchronize()
        assert db.seg.c.tile_rows == 16
        out[policy] = db.y["p"].clone()
    assert torch.equal(out[L.LORA_ACT_AUTO], out[L.LORA_ACT_RESIDENT])
    rows = np.sort(np.random.default_rng(9).choice(w.pairs, size=48, replace=False))
    res = oracle_projection(b, ws, 0, 0, rows=rows)
    got = bits_from_dev(out[L.LORA_ACT_AUTO][torch.from_numpy(rows).cuda()])
    check_delta(W.bf16_bits_to_f32(got).astype(np.float64), res.delta, "streamed by default")
    del dp, db, out
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name", ["dense_small", "llama8b_decode", "mixtral_moe_decode", "finegrained_moe_decode"])
def test_full_size_workloads_are_bit_identical_under_the_streaming_policy(name):
    """The decode workloads at their full sizes, as the benchmark's cold-activation measurement
    runs them: LORA_ACT_STREAMING against the default policy, every output row bit for bit (the
    default policy's outputs are compared with the oracle in test_gpu_configs.py)."""
    w = W.WORKLOADS[name]
    b = W.make_batch(w, 1234, y_mode="normal")
    ws = W.make_weights(w, 1234, n_layers=1)
    dp, db = DevicePool(ws, b.scale), DeviceBatch(b)
    run = LayerRunner(dp, db)
    out = {}
    for policy in (L.LORA_ACT_AUTO, L.LORA_ACT_STREAMING):
        L.lora_pool_set_activation_policy(dp.pool, policy)
        db.reset_y()
        run.step(0)
        torch.cuda.synchronize()
        out[policy] = {p.name: db.y[p.name].clone() for p in w.projs}
    for p in w.projs:
        assert torch.equal(out[L.LORA_ACT_AUTO][p.name], out[L.LORA_ACT_STREAMING][p.name]), p.name
        assert not torch.equal(out[L.LORA_ACT_AUTO][p.name], to_dev(b.y_in[p.name])), p.name
    del dp, db, out
    torch.cuda.empty_cache()


@pytest.mark.parametrize("rank,n_proj", [(8, 1), (16, 2), (16, 3), (32, 1)])
def test_streamed_inputs_at_a_ragged_width(rank, n_proj):
    """2100 rows of 16392 inputs (65.7 MiB, read once: streamed, at ranks 8 and 16 as whole cache
    lines through LDS) over 150 adapters, groups of one to three projections of 136 to 264 outputs;
    the width is not a whole number of 128-value steps and the tiles are ragged.  Every row against
    the oracle, and bit-identical to the resident policy (plain loads in operand layout)."""
    projs = tuple(W.Proj(f"p{j}", 16392, 136 + 64 * j, "x") for j in range(n_proj))
    w = W.Workload("t", "dense", 150, 1, 1, rank, projs, 2100, "zipf", 0.7)
    assert w.pairs * 16392 * 2 >= 64 << 20
    b = W.make_batch(w, 21, y_mode="zero", no_adapter_frac=0.03, hetero_scale=True)
    ws = W.make_weights(w, 21, bank_elems=1 << 22)
    dp, db = DevicePool(ws, b.scale), DeviceBatch(b)
    run = LayerRunner(dp, db)
    out = {}
    for policy in (L.LORA_ACT_AUTO, L.LORA_ACT_RESIDENT):
        L.lora_pool_set_activation_policy(dp.pool, policy)
        db.reset_y()
        run.step(0, one_call=False)
        torch.cuda.synchronize()
        assert db.seg.c.tile_rows == 16
        out[policy] = {p.name: bits_from_dev(db.y[p.name]).copy() for p in projs}
    for j, p in enumerate(projs):
        assert np.array_equal(out[L.LORA_ACT_AUTO][p.name], out[L.LORA_ACT_RESIDENT][p.name]), p.name
        res = oracle_projection(b, ws, 0, j)
        check_delta(W.bf16_bits_to_f32(out[L.LORA_ACT_AUTO][p.name]).astype(np.float64), res.delta,
                    f"streamed ragged inputs r{rank}/{p.name}")
    del dp, db
    torch.cuda.empty_cache()
