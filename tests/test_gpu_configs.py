"""The five workloads at their full sizes, in the launch configuration the benchmark times,
against the fp64 oracle (all rows where that takes seconds, a seeded sample of rows for the
prefill workload)."""
import numpy as np
import pytest
import torch

import paper_2604_07173_amd as L
import workloads as W
from gpu_common import check_accumulate, check_delta, oracle_projection
from oracle import lora_oracle as O
from harness import DeviceBatch, DevicePool, LayerRunner, bits_from_dev

pytestmark = pytest.mark.gpu


def run_config(name, seed, y_mode, sample=None, n_layers=1, layer=0, w=None):
    w = w or W.WORKLOADS[name]
    b = W.make_batch(w, seed, y_mode=y_mode)
    ws = W.make_weights(w, seed, n_layers=n_layers)
    print(f"[{name}] seed={seed} y={y_mode} P={w.pairs} pool...", flush=True)
    dp = DevicePool(ws, b.scale)
    db = DeviceBatch(b)
    LayerRunner(dp, db).step(layer)
    torch.cuda.synchronize()
    # segments of the full batch, bit-exact
    o = O.segments(b.adapter_id, b.expert_id, w.n_adapters, w.n_experts)
    counts = db.seg.counts.cpu().numpy()
    assert counts[0] == o.S and counts[1] == o.P_act
    assert np.array_equal(db.seg.perm.cpu().numpy()[:o.P_act], o.perm)
    rows = None
    if sample is not None:
        rows = np.sort(np.random.default_rng(seed).choice(w.pairs, size=sample, replace=False))
    worst = 0.0
    for j, p in enumerate(w.projs):
        res = oracle_projection(b, ws, layer, j, rows=rows)
        got = bits_from_dev(db.y[p.name])
        if rows is not None:
            got = np.ascontiguousarray(got[rows])
        if y_mode == "zero":
            rel, _ = check_delta(W.bf16_bits_to_f32(got).astype(np.float64), res.delta, f"{name}/{p.name}")
        else:
            _, rel = check_accumulate(got, res, f"{name}/{p.name}")
        worst = max(worst, rel)
    print(f"[{name}] worst rel Frobenius {worst:.2e}", flush=True)
    del dp, db
    torch.cuda.empty_cache()


@pytest.mark.parametrize("y_mode", ["zero", "normal"])
def test_dense_small(y_mode):
    run_config("dense_small", 1234, y_mode)


@pytest.mark.parametrize("y_mode", ["zero", "normal"])
def test_llama8b_decode(y_mode):
    run_config("llama8b_decode", 1234, y_mode)


@pytest.mark.parametrize("y_mode", ["zero", "normal"])
def test_mixtral_moe_decode(y_mode):
    run_config("mixtral_moe_decode", 1234, y_mode, n_layers=2, layer=1)


@pytest.mark.parametrize("y_mode", ["zero", "normal"])
def test_finegrained_moe_decode(y_mode):
    run_config("finegrained_moe_decode", 1234, y_mode)


def test_finegrained_moe_batch_beyond_one_workgroup_of_the_segment_builder():
    """The fine-grained MoE shapes with 2304 tokens x top-8 = 18432 rows over 32768 (adapter,
    expert) keys: more rows than one workgroup of the segment builder sorts and more keys than one
    8-bit pass covers; segments bit-exact, sampled rows of every projection against the oracle."""
    w = W.scaled(W.WORKLOADS["finegrained_moe_decode"], tokens=2304)
    assert w.pairs > L.LORA_MAX_ROWS
    run_config("finegrained_moe_18432_rows", 7, "zero", sample=512, w=w)


def test_prefill_sampled_rows():
    run_config("prefill", 1234, "normal", sample=384)
    run_config("prefill", 1, "zero", sample=128)


@pytest.mark.parametrize("y_mode", ["zero", "normal"])
def test_prefill_one_whole_request(y_mode):
    """Every row of one 2048-row request of the full prefill batch (64 consecutive 32-row
    tiles, sixteen four-tile groups of the shrink, all column chunks of both projections),
    next to the sampled rows of the test above."""
    name, seed, request = "prefill", 2, 3
    w = W.WORKLOADS[name]
    b = W.make_batch(w, seed, y_mode=y_mode)
    ws = W.make_weights(w, seed)
    dp, db = DevicePool(ws, b.scale), DeviceBatch(b)
    LayerRunner(dp, db).step(0)
    torch.cuda.synchronize()
    assert db.seg.c.tile_rows == 32
    per = w.tokens // w.n_requests
    rows = np.arange(request * per, (request + 1) * per)
    assert (b.adapter_id[rows] == request).all() and (b.adapter_id == request).sum() == per
    for j, p in enumerate(w.projs):
        res = oracle_projection(b, ws, 0, j, rows=rows)
        got = np.ascontiguousarray(bits_from_dev(db.y[p.name])[rows])
        if y_mode == "zero":
            check_delta(W.bf16_bits_to_f32(got).astype(np.float64), res.delta, f"prefill request/{p.name}")
        else:
            check_accumulate(got, res, f"prefill request/{p.name}")
    del dp, db
    torch.cuda.empty_cache()


@pytest.mark.parametrize("y_mode", ["zero", "normal"])
@pytest.mark.parametrize("rank", [32, 64])
def test_mixtral_widths_at_rank_32_and_64(rank, y_mode):
    """The decode kernels (16-row tiles) at the ranks of the paper's evaluation (Table 3) and
    the full Mixtral widths 4096 -> 14336 and 14336 -> 4096: the kernel-microbenchmark shape of
    App. A.2.2 with the adapter count and the batch cut so that the pool and the oracle stay
    small (16 adapters x 8 experts, 256 tokens x top-2, Zipf 1.2)."""
    w = W.scaled(W.WORKLOADS["mixtral_r64_microbench"], n_adapters=16, tokens=256, rank=rank)
    b = W.make_batch(w, 7, y_mode=y_mode, no_adapter_frac=0.03)
    ws = W.make_weights(w, 7)
    dp, db = DevicePool(ws, b.scale), DeviceBatch(b)
    LayerRunner(dp, db).step(0)
    torch.cuda.synchronize()
    assert db.seg.c.tile_rows == 16
    counts = db.seg.counts.cpu().numpy()
    assert counts[2] > counts[0] > 60          # several segments span more than one tile
    for j, p in enumerate(w.projs):
        res = oracle_projection(b, ws, 0, j)
        got = bits_from_dev(db.y[p.name])
        if y_mode == "zero":
            check_delta(W.bf16_bits_to_f32(got).astype(np.float64), res.delta, f"mixtral r{rank}/{p.name}")
        else:
            check_accumulate(got, res, f"mixtral r{rank}/{p.name}")
        none = b.adapter_id < 0
        assert np.array_equal(got[none], b.y_in[p.name][none])
    del dp, db
    torch.cuda.empty_cache()


def test_batch_longer_than_one_workgroup_sorts():
    """24 requests x 1024 tokens = 24576 rows (more than the 16384 a single workgroup of the
    segment builder holds), 6 adapters, rank 16, 1032 -> 776: segments by the multi-workgroup
    builder, long-segment kernels; sampled rows and one whole request against the oracle."""
    w = W.Workload("t", "dense", 6, 1, 1, 16, (W.Proj("p", 1032, 776, "x"),), 24 * 1024, "contiguous",
                   n_requests=24)
    b = W.make_batch(w, 5, y_mode="zero")
    ws = W.make_weights(w, 5, bank_elems=1 << 21)
    dp, db = DevicePool(ws, b.scale), DeviceBatch(b)
    LayerRunner(dp, db).step(0)
    torch.cuda.synchronize()
    assert db.P > L.LORA_MAX_ROWS and db.seg.c.tile_rows == 32
    o = O.segments(b.adapter_id, None, w.n_adapters, 1)
    counts = db.seg.counts.cpu().numpy()
    assert counts[0] == o.S == 6 and counts[1] == o.P_act == db.P
    assert np.array_equal(db.seg.perm.cpu().numpy(), o.perm)
    rows = np.sort(np.concatenate([np.random.default_rng(5).choice(db.P, size=256, replace=False),
                                   np.arange(17 * 1024, 18 * 1024)]))
    rows = np.unique(rows)
    res = oracle_projection(b, ws, 0, 0, rows=rows)
    got = np.ascontiguousarray(bits_from_dev(db.y["p"])[rows])
    check_delta(W.bf16_bits_to_f32(got).astype(np.float64), res.delta, "24576-row batch")
