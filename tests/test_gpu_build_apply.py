"""lora_moe_build_apply / lora_build_apply_group: the segment build and the first application of a
layer call in one entry point.  Small decode batches are sorted inside the first shrink kernel;
the segments must equal the oracle's bit for bit, the outputs those of lora_build_segments followed
by the application bit for bit, on both sides of every limit that decides which way it runs."""
import numpy as np
import pytest
import torch

import paper_2604_07173_amd as L
import workloads as W
from gpu_common import check_delta, oracle_projection
from harness import DeviceBatch, DevicePool, LayerRunner, bits_from_dev
from test_gpu_segments import compare

pytestmark = pytest.mark.gpu


def poison_segments(seg):
    for t in (seg.perm, seg.seg_start, seg.seg_key, seg.tiles, seg.counts):
        t.fill_(-7)
    seg.status.fill_(5)


def run_both(w, seed, no_adapter_frac=0.1, bad_ids=False):
    """The layer call through the one-call entry points, then through lora_build_segments and the
    applications one by one on fresh outputs; returns (batch, weights, outputs, reference outputs,
    segments of the one-call path)."""
    b = W.make_batch(w, seed, y_mode="normal", no_adapter_frac=no_adapter_frac, hetero_scale=True)
    if bad_ids:
        b.adapter_id[::37] = w.n_adapters + 2
        if b.expert_id is not None:
            b.expert_id[5::41] = w.n_experts
    ws = W.make_weights(w, seed, n_layers=2, bank_elems=1 << 22)
    dp, db = DevicePool(ws, b.scale), DeviceBatch(b)
    run = LayerRunner(dp, db)
    poison_segments(db.seg)
    run.step(1, one_call=True)
    torch.cuda.synchronize()
    got = {k: bits_from_dev(v) for k, v in db.y.items()}
    seg_one = db.seg
    db.seg = L.Segments(db.P)
    poison_segments(db.seg)
    db.reset_y()
    run.step(1, one_call=False)
    torch.cuda.synchronize()
    ref = {k: bits_from_dev(v) for k, v in db.y.items()}
    for name in ("perm", "seg_start", "seg_key", "tiles", "counts", "status"):
        a, c = getattr(seg_one, name), getattr(db.seg, name)
        n = {"perm": int(db.seg.counts[1]), "seg_start": int(db.seg.counts[0]) + 1,
             "seg_key": int(db.seg.counts[0]), "tiles": int(db.seg.counts[2])}.get(name, a.shape[0])
        assert torch.equal(a[:n], c[:n]), name
    return b, ws, dp, got, ref, seg_one


MOE_CASES = [
    # rank, h, f, adapters, experts, top_k, tokens, sorted inside the shrink
    (16, 264, 392, 4, 2, 2, 1, True),
    (16, 520, 1160, 32, 8, 2, 100, True),              # 256 keys
    (8, 264, 392, 3, 5, 2, 517, True),                 # ragged last group of 64 rows
    (32, 264, 520, 16, 16, 2, 1024, True),             # 2048 rows, the most taken
    (64, 136, 264, 2, 2, 2, 40, True),
    (16, 264, 392, 16, 16, 2, 1025, False),            # 2050 rows
    (16, 264, 392, 257, 1, 1, 300, False),             # 257 keys
]


@pytest.mark.parametrize("rank,h,f,n,E,k,tokens,inline", MOE_CASES)
def test_moe_layer_call_with_the_build_inside(rank, h, f, n, E, k, tokens, inline):
    projs = (W.Proj("gate", h, f, "x"), W.Proj("up", h, f, "x"), W.Proj("down", f, h, "mid"))
    w = W.Workload("t", "moe", n, E, k, rank, projs, tokens, "zipf", 1.0)
    b, ws, dp, got, ref, seg = run_both(w, 11)
    P = tokens * k
    launches = L.lora_build_apply_launches(dp.pool, 0, 2, P)
    fused = L.lora_group_launches(dp.pool, 0, 2, P, seg) == 1
    if fused:
        assert launches == (1 if inline else 2)         # build, shrink and expand in a single launch
    else:
        assert launches == (2 if inline else 3)
    compare(seg, b.adapter_id, b.expert_id, n, E)
    assert int(seg.status.cpu()[0]) == 0
    for name in ("gate", "up", "down"):
        assert np.array_equal(got[name], ref[name]), name
    res = oracle_projection(b, ws, 1, 0)
    delta = W.bf16_bits_to_f32(got["gate"]).astype(np.float64) - W.bf16_bits_to_f32(b.y_in["gate"]).astype(np.float64)
    act = b.adapter_id >= 0
    assert np.abs(delta[~act]).max(initial=0.0) == 0.0
    # the accumulated output carries the rounding of y; the update itself must be there
    assert np.linalg.norm(delta[act] - res.delta[act]) <= 0.25 * np.linalg.norm(res.delta[act]) + 1e-6


def test_dense_layer_call_with_the_build_inside():
    """q/k/v-like first group (three projections sharing x), then two more groups that use the
    segments the first shrink wrote out."""
    projs = (W.Proj("q", 1032, 520, "x"), W.Proj("k", 1032, 136, "x"), W.Proj("v", 1032, 136, "x"),
             W.Proj("o", 520, 1032, "a"), W.Proj("down", 2056, 1032, "m"))
    w = W.Workload("t", "dense", 100, 1, 1, 16, projs, 300, "zipf", 1.0)
    b, ws, dp, got, ref, seg = run_both(w, 12)
    assert L.lora_build_apply_launches(dp.pool, 0, 3, 300) == 2
    compare(seg, b.adapter_id, None, 100, 1)
    for p in projs:
        assert np.array_equal(got[p.name], ref[p.name]), p.name


def test_small_dense_call_is_a_single_launch():
    """A batch small enough for shrink and expand in one launch: with the build inside, the whole
    call (segments, shrink, expand) is one kernel."""
    projs = (W.Proj("p", 1032, 392, "x"),)
    w = W.Workload("t", "dense", 5, 1, 1, 8, projs, 70, "zipf", 0.8)
    b, ws, dp, got, ref, seg = run_both(w, 16)
    assert L.lora_build_apply_launches(dp.pool, 0, 1, 70) == 1
    compare(seg, b.adapter_id, None, 5, 1)
    # the same arithmetic as the call on segments built before: bit-identical
    assert np.array_equal(got["p"], ref["p"])
    res = oracle_projection(b, ws, 1, 0)
    delta = W.bf16_bits_to_f32(got["p"]).astype(np.float64) - W.bf16_bits_to_f32(b.y_in["p"]).astype(np.float64)
    act = b.adapter_id >= 0
    assert np.linalg.norm(delta[act] - res.delta[act]) <= 0.25 * np.linalg.norm(res.delta[act]) + 1e-6


def test_random_batches_through_the_one_call_entry_point():
    """Sixty random batches (1 to 2048 rows, 1 to 256 keys, uniform or skewed ids, rows without
    adapter) through lora_build_apply_group on a narrow projection: segments against the oracle,
    outputs bit-identical to lora_build_segments + lora_apply_group.  Small ones run as a single
    launch, the others build inside the shrink."""
    rng = np.random.default_rng(2025)
    single = inside = 0
    for case in range(60):
        n = int(rng.choice([1, 2, 5, 16, 64, 200, 256]))
        P = int(rng.choice([1, 3, 16, 17, 63, 64, 65, 255, 257, 700, 1024, 1500, 2047, 2048]))
        alpha = float(rng.choice([0.0, 0.7, 1.3]))
        ids = "uniform" if alpha == 0.0 else "zipf"
        w = W.Workload("t", "dense", n, 1, 1, 8, (W.Proj("p", 40, 24, "x"),), P, ids, alpha)
        b = W.make_batch(w, 1000 + case, y_mode="normal", no_adapter_frac=float(rng.choice([0.0, 0.1, 0.6])))
        ws = W.make_weights(w, 1000 + case, bank_elems=1 << 18)
        dp, db = DevicePool(ws, b.scale), DeviceBatch(b)
        run = LayerRunner(dp, db)
        launches = L.lora_build_apply_launches(dp.pool, 0, 1, P)
        assert launches in (1, 2)
        single += launches == 1
        inside += launches == 2
        poison_segments(db.seg)
        run.step(0, one_call=True)
        torch.cuda.synchronize()
        got = bits_from_dev(db.y["p"])
        compare(db.seg, b.adapter_id, None, n, 1)
        db.seg = L.Segments(db.P)
        db.reset_y()
        run.step(0, one_call=False)
        torch.cuda.synchronize()
        assert np.array_equal(got, bits_from_dev(db.y["p"])), (case, n, P)
    assert single >= 5 and inside >= 5


def test_ids_outside_the_pool_are_reported_and_dropped():
    projs = (W.Proj("gate", 264, 392, "x"), W.Proj("up", 264, 392, "x"), W.Proj("down", 392, 264, "mid"))
    w = W.Workload("t", "moe", 8, 4, 2, 16, projs, 200, "uniform")
    b, ws, dp, got, ref, seg = run_both(w, 13, bad_ids=True)
    assert int(seg.status.cpu()[0]) == 3
    compare(seg, b.adapter_id, b.expert_id, 8, 4)
    for name in ("gate", "up", "down"):
        assert np.array_equal(got[name], ref[name]), name


def test_batch_without_any_adapter_and_empty_batch():
    projs = (W.Proj("gate", 264, 392, "x"), W.Proj("up", 264, 392, "x"), W.Proj("down", 392, 264, "mid"))
    w = W.Workload("t", "moe", 8, 4, 2, 16, projs, 50, "uniform")
    b, ws, dp, got, ref, seg = run_both(w, 14, no_adapter_frac=1.0)
    assert seg.counts.cpu().tolist() == [0, 0, 0, 0]
    for name in ("gate", "up", "down"):
        assert np.array_equal(got[name], b.y_in[name])
    # P = 0: the call still writes the counts
    db = DeviceBatch(b)
    poison_segments(db.seg)
    wsb = torch.empty(256, dtype=torch.uint8, device="cuda")
    x = db.inputs["x"]
    L.lora_moe_build_apply(dp.pool, 0, L.LORA_MOE_UPGATE, x, x.shape[1], db.token_of_pair, db.adapter_id,
                           db.expert_id, 0, db.seg, db.y["gate"], db.y["up"], db.y["gate"].shape[1], wsb)
    torch.cuda.synchronize()
    assert db.seg.counts.cpu().tolist() == [0, 0, 0, 0]


def test_an_error_enqueues_nothing():
    projs = (W.Proj("gate", 264, 392, "x"), W.Proj("up", 264, 392, "x"), W.Proj("down", 392, 264, "mid"))
    w = W.Workload("t", "moe", 8, 4, 2, 16, projs, 50, "uniform")
    b = W.make_batch(w, 15, y_mode="normal")
    ws = W.make_weights(w, 15, bank_elems=1 << 20)
    dp, db = DevicePool(ws, b.scale), DeviceBatch(b)
    run = LayerRunner(dp, db)
    poison_segments(db.seg)
    x = db.inputs["x"]
    with pytest.raises(L.LoraError):                    # misaligned output
        L.lora_moe_build_apply(dp.pool, 0, L.LORA_MOE_UPGATE, x, x.shape[1], db.token_of_pair, db.adapter_id,
                               db.expert_id, db.P, db.seg, db.y["gate"].view(-1)[1:], db.y["up"],
                               db.y["gate"].shape[1], run.ws)
    torch.cuda.synchronize()
    assert db.seg.counts.cpu().tolist() == [-7, -7, -7, -7]
    for k, v in db.y.items():
        assert np.array_equal(bits_from_dev(v), b.y_in[k])


def test_mixtral_decode_sorts_inside_the_shrink():
    """The headline workload takes the path: four launches for the layer call."""
    w = W.WORKLOADS["mixtral_moe_decode"]
    b = W.make_batch(w, 1234, y_mode="zero")
    ws = W.make_weights(w, 1234)
    dp, db = DevicePool(ws, b.scale), DeviceBatch(b)
    assert L.lora_build_apply_launches(dp.pool, 0, 2, db.P) == 2
    LayerRunner(dp, db).step(0)
    torch.cuda.synchronize()
    compare(db.seg, b.adapter_id, b.expert_id, w.n_adapters, w.n_experts)
    for j, p in enumerate(w.projs):
        res = oracle_projection(b, ws, 0, j)
        check_delta(W.bf16_bits_to_f32(bits_from_dev(db.y[p.name])).astype(np.float64), res.delta,
                    f"build inside {p.name}")
