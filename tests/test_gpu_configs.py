"""The five workloads at their full sizes, in the launch configuration the benchmark times,
against the fp64 oracle (all rows where that takes seconds, a seeded sample of rows for the
prefill workload)."""
import numpy as np
import pytest
import torch

import workloads as W
from gpu_common import check_accumulate, check_delta, oracle_projection
from oracle import lora_oracle as O
from paper_2604_07173_amd.harness import DeviceBatch, DevicePool, LayerRunner, bits_from_dev

pytestmark = pytest.mark.gpu


def run_config(name, seed, y_mode, sample=None, n_layers=1, layer=0):
    w = W.WORKLOADS[name]
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


def test_finegrained_moe_decode():
    run_config("finegrained_moe_decode", 1234, "normal")


def test_prefill_sampled_rows():
    run_config("prefill", 1234, "normal", sample=384)
    run_config("prefill", 1, "zero", sample=128)
