"""Shrink / expand / MoE application against the fp64 oracle, element by element, at sizes
that span several tiles, K parts and column chunks with ragged tails."""
import numpy as np
import pytest
import torch

import paper_2604_07173_amd as L
import workloads as W
from gpu_common import bf16_ulp, check_accumulate, check_delta, oracle_projection
from harness import DeviceBatch, DevicePool, LayerRunner, bits_from_dev, to_dev

pytestmark = pytest.mark.gpu


def dense_workload(rank, h_in, h_out, n=5, tokens=70, ids="uniform", alpha=0.0):
    return W.Workload("t", "dense", n, 1, 1, rank, (W.Proj("p", h_in, h_out, "x"),), tokens, ids,
                      alpha)


def moe_workload(rank, h, f, n=6, E=4, k=2, tokens=40, alpha=1.0):
    projs = (W.Proj("gate", h, f, "x"), W.Proj("up", h, f, "x"), W.Proj("down", f, h, "mid"))
    return W.Workload("t", "moe", n, E, k, rank, projs, tokens, "zipf", alpha)


def run_dense(w, seed, y_mode, out_f32=False, drop=0.0, hetero=True, n_layers=1, layer=0):
    b = W.make_batch(w, seed, y_mode=y_mode, no_adapter_frac=drop, hetero_scale=hetero)
    ws = W.make_weights(w, seed, n_layers=n_layers, bank_elems=1 << 20)
    dp = DevicePool(ws, b.scale)
    db = DeviceBatch(b)
    run = LayerRunner(dp, db)
    run.build_segments()
    p = w.projs[0]
    x = db.inputs["x"]
    L.lora_shrink(dp.pool, layer, 0, x, x.shape[1], None, db.seg, run.v)
    if out_f32:
        y = torch.from_numpy(W.bf16_bits_to_f32(b.y_in["p"])).cuda()
        L.lora_expand(dp.pool, layer, 0, run.v, db.seg, y, y.shape[1], L.LORA_DTYPE_F32)
        torch.cuda.synchronize()
        got = y.cpu().numpy().astype(np.float64)
    else:
        y = db.y["p"]
        L.lora_expand(dp.pool, layer, 0, run.v, db.seg, y, y.shape[1], L.LORA_DTYPE_BF16)
        torch.cuda.synchronize()
        got = bits_from_dev(y)
    return b, ws, got, (dp, db, run)


def assert_same_up_to_rounding(a_bits, b_bits):
    """Two bf16 results of the same sums formed in a different fp32 order: equal almost
    everywhere, never more than one bf16 step apart."""
    a = W.bf16_bits_to_f32(a_bits).astype(np.float64)
    b = W.bf16_bits_to_f32(b_bits).astype(np.float64)
    # the same sums in another fp32 order: one bf16 step where the value is of normal size; where
    # terms cancel, what remains is the fp32 rounding of the row's largest values
    row = np.maximum(np.abs(a).max(axis=1, keepdims=True), np.abs(b).max(axis=1, keepdims=True))
    bound = bf16_ulp(np.maximum(np.abs(a), np.abs(b))) + 3e-5 * row
    assert (np.abs(a - b) <= bound).all() and (a_bits != b_bits).mean() < 0.02


SHAPES = [(8, 200, 328), (16, 200, 328), (32, 72, 136), (64, 264, 520), (16, 1024, 1024),
          (8, 40, 8), (16, 8, 1032)]


@pytest.mark.parametrize("rank,h_in,h_out", SHAPES)
def test_delta_mode_bf16(rank, h_in, h_out):
    w = dense_workload(rank, h_in, h_out)
    b, ws, got, _ = run_dense(w, 11, "zero")
    res = oracle_projection(b, ws, 0, 0)
    check_delta(W.bf16_bits_to_f32(got).astype(np.float64), res.delta, f"r{rank} {h_in}x{h_out}")


@pytest.mark.parametrize("rank,h_in,h_out", SHAPES)
def test_delta_mode_f32_output(rank, h_in, h_out):
    w = dense_workload(rank, h_in, h_out)
    b, ws, got, _ = run_dense(w, 12, "zero", out_f32=True)
    res = oracle_projection(b, ws, 0, 0)
    rel, _ = check_delta(got, res.delta, f"r{rank} {h_in}x{h_out} f32")
    assert rel < 1e-4     # fp32 output: only the accumulation order and the hi/lo split remain


@pytest.mark.parametrize("rank,h_in,h_out", SHAPES)
def test_accumulate_mode_and_untouched_rows(rank, h_in, h_out):
    w = dense_workload(rank, h_in, h_out)
    b, ws, got, _ = run_dense(w, 13, "normal", drop=0.25)
    res = oracle_projection(b, ws, 0, 0)
    check_accumulate(got, res, f"r{rank} {h_in}x{h_out}")
    none = b.adapter_id < 0
    assert none.any()
    assert np.array_equal(got[none], b.y_in["p"][none])      # rows without adapter: bit-identical


def test_f32_accumulate_keeps_base():
    w = dense_workload(16, 136, 264)
    b, ws, got, _ = run_dense(w, 14, "normal", out_f32=True, drop=0.2)
    res = oracle_projection(b, ws, 0, 0)
    np.testing.assert_allclose(got, res.y_out, rtol=0, atol=2e-5 * max(1.0, np.abs(res.y_out).max()))
    none = b.adapter_id < 0
    assert np.array_equal(got[none], W.bf16_bits_to_f32(b.y_in["p"][none]).astype(np.float64))


@pytest.mark.parametrize("forced", ["", "32"], ids=["family by size", "32-row tiles"])
@pytest.mark.parametrize("tokens", [1, 15, 16, 17, 31, 32, 33, 64, 65, 130])
def test_segment_lengths_around_tile_boundaries(tokens, forced, monkeypatch):
    """One adapter only: the segment has exactly `tokens` rows (1 .. several 32-row tiles), with the
    kernels the library picks for so few rows and with the long-segment kernels forced."""
    if forced:
        monkeypatch.setenv("LORA_TILE_ROWS", forced)
    w = dense_workload(16, 264, 392, n=1, tokens=tokens)
    b, ws, got, _ = run_dense(w, 15, "normal")
    res = oracle_projection(b, ws, 0, 0)
    check_accumulate(got, res, f"{tokens} rows")


@pytest.mark.parametrize("out_f32", [False, True])
@pytest.mark.parametrize("rank,n,tokens", [(8, 3, 100), (16, 7, 300), (32, 5, 149), (64, 9, 500)])
def test_segments_of_several_16_row_tiles(rank, n, tokens, out_f32):
    """8 to 63 rows per adapter: still the 16-row-tile kernels, but most segments span two to
    four tiles (an odd number of tiles in all, ragged last tiles); the expand then hands
    neighbouring waves the same slice of neighbouring tiles."""
    w = dense_workload(rank, 264, 648, n=n, tokens=tokens, ids="zipf", alpha=0.8)
    assert 8 * n <= tokens < 64 * n
    b, ws, got, (dp, db, run) = run_dense(w, 16 + rank, "normal", out_f32=out_f32, drop=0.1)
    assert db.seg.c.tile_rows == 16
    counts = db.seg.counts.cpu().numpy()
    assert counts[2] > counts[0]                       # more tiles than segments
    res = oracle_projection(b, ws, 0, 0)
    if out_f32:
        np.testing.assert_allclose(got, res.y_out, rtol=0, atol=2e-5 * max(1.0, np.abs(res.y_out).max()))
    else:
        check_accumulate(got, res, f"r{rank} n{n} t{tokens}")


@pytest.mark.parametrize("y_mode", ["zero", "normal"])
@pytest.mark.parametrize("rank,h_in", [(8, 200), (8, 64), (16, 200), (32, 104), (64, 72)])
def test_thousands_of_small_tiles_one_wave_per_tile(rank, h_in, y_mode):
    """More than 4096 tiles over a short K range: the shrink runs one wave per tile with the
    K range not split (one K part)."""
    w = dense_workload(rank, h_in, 136, n=4400, tokens=4500)
    b, ws, got, (dp, db, run) = run_dense(w, 21, y_mode, drop=0.02)
    assert L.lora_v_bytes(dp.pool, 0, 4500) < 2 * 4500 * rank * 4      # a single K part
    assert int(db.seg.counts.cpu()[2]) > 2000
    res = oracle_projection(b, ws, 0, 0)
    if y_mode == "zero":
        check_delta(W.bf16_bits_to_f32(got).astype(np.float64), res.delta, f"wave per tile r{rank} k{h_in}")
    else:
        check_accumulate(got, res, f"wave per tile r{rank} k{h_in}")


@pytest.mark.parametrize("out_f32", [False, True])
@pytest.mark.parametrize("rank,h_in,h_out,n,tokens", [(8, 200, 328, 5, 70), (16, 2080, 392, 4, 72),
                                                      (64, 4104, 1160, 6, 40)])
def test_apply_is_bit_identical_to_shrink_then_expand(rank, h_in, h_out, n, tokens, out_f32):
    w = dense_workload(rank, h_in, h_out, n=n, tokens=tokens)
    b = W.make_batch(w, 31, y_mode="normal", no_adapter_frac=0.1, hetero_scale=True)
    ws = W.make_weights(w, 31, bank_elems=1 << 20)
    dp, db = DevicePool(ws, b.scale), DeviceBatch(b)
    run = LayerRunner(dp, db)
    run.build_segments()
    x = db.inputs["x"]
    dt = L.LORA_DTYPE_F32 if out_f32 else L.LORA_DTYPE_BF16

    def fresh_y():
        if out_f32:
            return torch.from_numpy(W.bf16_bits_to_f32(b.y_in["p"])).cuda()
        return to_dev(b.y_in["p"])

    y_ref, y = fresh_y(), fresh_y()
    L.lora_shrink(dp.pool, 0, 0, x, x.shape[1], None, db.seg, run.v)
    L.lora_expand(dp.pool, 0, 0, run.v, db.seg, y_ref, y_ref.shape[1], dt)
    run.v.fill_(float("nan"))
    L.lora_apply(dp.pool, 0, 0, x, x.shape[1], None, db.seg, y, y.shape[1], run.v, dt)
    torch.cuda.synchronize()
    bits = torch.int32 if out_f32 else torch.int16
    if L.lora_group_launches(dp.pool, 0, 1, tokens, db.seg, dt) == 2:
        assert torch.equal(y.view(bits), y_ref.view(bits))
    else:
        # one launch: the K range is split differently, so sums differ in fp32 rounding only
        assert_same_up_to_rounding(bits_from_dev(y), bits_from_dev(y_ref))
    if not out_f32:
        check_accumulate(bits_from_dev(y), oracle_projection(b, ws, 0, 0), "apply")


@pytest.mark.parametrize("rank", [8, 16, 32, 64])
@pytest.mark.parametrize("tokens,n", [(70, 5), (2100, 3)])      # decode tiles / long segments
def test_group_of_three_projections_matches_single_calls(rank, tokens, n, monkeypatch):
    """q/k/v-like group: same input, widths 392 / 136 / 136; bit-identical to per-projection
    lora_apply calls and within tolerance of the oracle.  The long batch runs on the long-segment
    kernels (forced: the library takes them from rows x rank = 2^17 on)."""
    if tokens == 2100:
        monkeypatch.setenv("LORA_TILE_ROWS", "32")
    projs = (W.Proj("q", 264, 392, "x"), W.Proj("k", 264, 136, "x"), W.Proj("v", 264, 136, "x"))
    w = W.Workload("t", "dense", n, 1, 1, rank, projs, tokens, "uniform", 0.0)
    b = W.make_batch(w, 41, y_mode="normal", no_adapter_frac=0.1, hetero_scale=True)
    ws = W.make_weights(w, 41, bank_elems=1 << 20)
    dp, db = DevicePool(ws, b.scale), DeviceBatch(b)
    run = LayerRunner(dp, db)
    run.build_segments()
    assert run.groups == [(0, 3)]
    x = db.inputs["x"]
    ref = {}
    for j, p in enumerate(projs):
        y = to_dev(b.y_in[p.name])
        L.lora_apply(dp.pool, 0, j, x, x.shape[1], None, db.seg, y, y.shape[1], run.v)
        ref[p.name] = y
    run.apply(0)
    torch.cuda.synchronize()
    one_launch = L.lora_group_launches(dp.pool, 0, 3, tokens, db.seg) == 1
    assert one_launch == (tokens == 70)            # the small batch runs as one launch
    for j, p in enumerate(projs):
        if one_launch:
            assert_same_up_to_rounding(bits_from_dev(db.y[p.name]), bits_from_dev(ref[p.name]))
        else:
            assert torch.equal(db.y[p.name], ref[p.name]), p.name
        check_accumulate(bits_from_dev(db.y[p.name]), oracle_projection(b, ws, 0, j), p.name)


@pytest.mark.parametrize("y_mode", ["zero", "normal"])
@pytest.mark.parametrize("rank", [16, 64])
def test_long_segment_kernels_with_many_short_segments(rank, y_mode, monkeypatch):
    """The 32-row-tile kernels (forced for this small batch) on a Zipf draw over 24 adapters that
    leaves many segments of a few rows next to long ones, so most four-tile groups of the
    shrink straddle a segment boundary and the expand reloads B inside its tile groups."""
    monkeypatch.setenv("LORA_TILE_ROWS", "32")
    w = W.Workload("t", "dense", 24, 1, 1, rank, (W.Proj("p", 328, 264, "x"),), 2048, "zipf", 1.3)
    b, ws, got, (dp, db, run) = run_dense(w, 51, y_mode, drop=0.05)
    assert db.seg.c.tile_rows == 32
    lens = np.bincount(b.adapter_id[b.adapter_id >= 0], minlength=24)
    assert lens.max() > 300 and (lens[lens > 0] < 32).sum() >= 4
    res = oracle_projection(b, ws, 0, 0)
    if y_mode == "zero":
        check_delta(W.bf16_bits_to_f32(got).astype(np.float64), res.delta, f"long kernels, short segments r{rank}")
    else:
        check_accumulate(got, res, f"long kernels, short segments r{rank}")


@pytest.mark.parametrize("y_mode", ["zero", "normal"])
@pytest.mark.parametrize("rank,h_in,h_out", [(16, 40, 8), (64, 72, 136), (32, 264, 520), (16, 136, 1032), (64, 2056, 72)])
def test_long_segment_kernels_at_ragged_widths(rank, h_in, h_out, y_mode, monkeypatch):
    """The 32-row-tile kernels (forced for this small batch) at widths that are not whole stages of
    128 K values nor whole chunks of 128 columns (the shrink fetches x a stage of whole lines at a
    time): 3 adapters, 400 rows, every row against the oracle."""
    monkeypatch.setenv("LORA_TILE_ROWS", "32")
    w = dense_workload(rank, h_in, h_out, n=3, tokens=400)
    b, ws, got, (dp, db, run) = run_dense(w, 53, y_mode, drop=0.03)
    assert db.seg.c.tile_rows == 32
    res = oracle_projection(b, ws, 0, 0)
    if y_mode == "zero":
        check_delta(W.bf16_bits_to_f32(got).astype(np.float64), res.delta, f"long ragged r{rank} {h_in}x{h_out}")
    else:
        check_accumulate(got, res, f"long ragged r{rank} {h_in}x{h_out}")
    none = b.adapter_id < 0
    assert np.array_equal(got[none], b.y_in["p"][none])


@pytest.mark.parametrize("rank,n,tokens,tile_rows", [(16, 200, 8191, 16), (16, 200, 8192, 32), (16, 200, 2048, 16),
                                                     (64, 8, 2047, 16), (64, 8, 2048, 32), (16, 64, 4096, 16),
                                                     (32, 300, 8192, 16)])
def test_kernel_family_switch_for_long_decode_batches(rank, n, tokens, tile_rows):
    """The 32-row-tile kernels are taken from rows x rank = 2^17 on (8192 rows at rank 16, 2048 at
    rank 64) if there are at least 32 rows per key: both sides of the limits, against the oracle
    (all rows)."""
    w = W.Workload("t", "dense", n, 1, 1, rank, (W.Proj("p", 264, 136, "x"),), tokens, "zipf", 0.6)
    b, ws, got, (dp, db, run) = run_dense(w, 52, "zero", drop=0.02)
    assert db.seg.c.tile_rows == tile_rows
    res = oracle_projection(b, ws, 0, 0)
    check_delta(W.bf16_bits_to_f32(got).astype(np.float64), res.delta, f"family switch r{rank} {n} keys {tokens}")


@pytest.mark.parametrize("tokens,forced", [(1, ""), (40, ""), (5000, ""), (5000, "32")])
def test_batch_without_any_adapter_leaves_everything_untouched(tokens, forced, monkeypatch):
    """Every row has id -1: no segment, no tile; y keeps its bits (both kernel families)."""
    if forced:
        monkeypatch.setenv("LORA_TILE_ROWS", forced)
    w = dense_workload(16, 200, 136, n=3, tokens=tokens)
    b = W.make_batch(w, 61, y_mode="normal")
    b.adapter_id[:] = -1
    ws = W.make_weights(w, 61, bank_elems=1 << 20)
    dp, db = DevicePool(ws, b.scale), DeviceBatch(b)
    run = LayerRunner(dp, db)
    run.build_segments()
    assert db.seg.counts.cpu().tolist()[:3] == [0, 0, 0]
    run.apply(0)
    torch.cuda.synchronize()
    assert np.array_equal(bits_from_dev(db.y["p"]), b.y_in["p"])


def test_single_row_batch():
    w = dense_workload(64, 264, 392, n=2, tokens=1)
    b, ws, got, _ = run_dense(w, 62, "normal")
    check_accumulate(got, oracle_projection(b, ws, 0, 0), "one row")


def test_shrink_output_matches_oracle_v_and_src_row():
    w = dense_workload(16, 2080, 136, n=4, tokens=72)
    b = W.make_batch(w, 16, hetero_scale=True)
    ws = W.make_weights(w, 16, bank_elems=1 << 20)
    dp, db = DevicePool(ws, b.scale), DeviceBatch(b)
    run = LayerRunner(dp, db)
    run.build_segments()
    rng = np.random.default_rng(16)
    src = rng.integers(0, 72, size=72).astype(np.int32)
    x = db.inputs["x"]
    L.lora_shrink(dp.pool, 0, 0, x, x.shape[1], to_dev(src), db.seg, run.v)
    torch.cuda.synchronize()
    P, r = 72, 16
    n_parts = L.lora_v_bytes(dp.pool, 0, P) // (P * r * 4)
    assert n_parts >= 2      # 2080 inputs: more than one K part
    v = run.v.cpu().numpy()[:n_parts * P * r].reshape(n_parts, P, r).astype(np.float64).sum(0)
    b.token_of_pair = src
    res = oracle_projection(b, ws, 0, 0)
    perm = db.seg.perm.cpu().numpy()[:int(db.seg.counts.cpu()[1])]
    np.testing.assert_allclose(v[:len(perm)], res.v[perm], rtol=1e-5, atol=1e-5)


def test_leading_dimensions_larger_than_widths():
    w = dense_workload(16, 200, 136, tokens=50)
    b = W.make_batch(w, 17, y_mode="normal")
    ws = W.make_weights(w, 17, bank_elems=1 << 20)
    dp, db = DevicePool(ws, b.scale), DeviceBatch(b)
    run = LayerRunner(dp, db)
    run.build_segments()
    xpad = torch.full((50, 216), 0x7FC0, dtype=torch.int16, device="cuda")   # NaN padding
    xpad[:, :200] = db.inputs["x"]
    ypad = torch.full((50, 160), 0x1234, dtype=torch.int16, device="cuda")
    ypad[:, :136] = db.y["p"]
    L.lora_shrink(dp.pool, 0, 0, xpad, 216, None, db.seg, run.v)
    L.lora_expand(dp.pool, 0, 0, run.v, db.seg, ypad, 160, L.LORA_DTYPE_BF16)
    torch.cuda.synchronize()
    got = bits_from_dev(ypad)
    assert (got[:, 136:] == 0x1234).all()
    check_accumulate(np.ascontiguousarray(got[:, :136]), oracle_projection(b, ws, 0, 0), "ld")


def test_tiny_integer_cases_are_bit_exact():
    """Small integer inputs: every product and sum is exact in fp32 and bf16, so the GPU
    output must equal the oracle bit for bit."""
    rng = np.random.default_rng(18)
    w = W.Workload("t", "moe", 2, 2, 1, 8, (W.Proj("gate", 8, 8, "x"), W.Proj("up", 8, 8, "x"),
                                            W.Proj("down", 8, 8, "mid")), 4, "uniform")
    for trial in range(4):
        b = W.make_batch(w, 100 + trial, y_mode="normal", no_adapter_frac=0.3)
        ints = lambda shape: W.f32_to_bf16_bits(rng.integers(-3, 4, size=shape).astype(np.float32))
        b.inputs = {"x": ints((4, 8)), "mid": ints((4, 8))}
        b.y_in = {k: ints((4, 8)) for k in ("gate", "up", "down")}
        b.scale = np.array([0.5, 2.0], np.float32)
        ws = W.make_weights(w, 100 + trial, bank_elems=1 << 16)
        ws.bank[:] = ints(ws.bank.shape)
        dp, db = DevicePool(ws, b.scale), DeviceBatch(b)
        LayerRunner(dp, db).step(0)
        torch.cuda.synchronize()
        for j, p in enumerate(w.projs):
            res = oracle_projection(b, ws, 0, j)
            assert np.array_equal(bits_from_dev(db.y[p.name]), res.y_bf16), (trial, p.name)


@pytest.mark.parametrize("rank,h,f,E,k,tokens", [(16, 264, 392, 4, 2, 40), (8, 136, 776, 8, 4, 33),
                                                 (64, 136, 264, 2, 2, 50), (32, 72, 136, 3, 1, 20)])
def test_moe_apply_matches_oracle(rank, h, f, E, k, tokens):
    w = moe_workload(rank, h, f, E=E, k=k, tokens=tokens)
    b = W.make_batch(w, 19, y_mode="normal", no_adapter_frac=0.1, hetero_scale=True)
    ws = W.make_weights(w, 19, n_layers=2, bank_elems=1 << 21)
    dp, db = DevicePool(ws, b.scale), DeviceBatch(b)
    run = LayerRunner(dp, db)
    run.step(1)                      # second layer of the pool
    torch.cuda.synchronize()
    for j, p in enumerate(w.projs):
        res = oracle_projection(b, ws, 1, j)
        got = bits_from_dev(db.y[p.name])
        check_accumulate(got, res, f"moe {p.name}")
        none = b.adapter_id < 0
        assert np.array_equal(got[none], b.y_in[p.name][none])
    # delta mode on the same batch
    b0 = W.make_batch(w, 19, y_mode="zero", no_adapter_frac=0.1, hetero_scale=True)
    db0 = DeviceBatch(b0)
    LayerRunner(dp, db0).step(1)
    torch.cuda.synchronize()
    for j, p in enumerate(w.projs):
        res = oracle_projection(b0, ws, 1, j)
        check_delta(W.bf16_bits_to_f32(bits_from_dev(db0.y[p.name])).astype(np.float64), res.delta,
                    f"moe delta {p.name}")


def test_two_layer_calls_in_flight_on_two_streams():
    """Two different batches on one pool, issued alternately on two streams without any
    synchronisation between them: a call's state is only its own segments and workspace, so
    both must come out exactly as when they run alone."""
    w = moe_workload(16, 520, 776, E=4, k=2, tokens=300)
    ws = W.make_weights(w, 23, n_layers=2, bank_elems=1 << 21)
    batches = [W.make_batch(w, 23 + i, y_mode="normal", no_adapter_frac=0.05) for i in range(2)]
    dp = DevicePool(ws, batches[0].scale)
    alone = []
    for b in batches:
        db = DeviceBatch(b)
        LayerRunner(dp, db).step(1)
        torch.cuda.synchronize()
        alone.append({k: v.clone() for k, v in db.y.items()})
    dbs = [DeviceBatch(b) for b in batches]
    runs = [LayerRunner(dp, db) for db in dbs]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for rep in range(5):                 # y accumulates, so each repetition first restores the
        for i in range(2):               # base output, on the call's own stream
            with torch.cuda.stream(streams[i]):
                for k, v in batches[i].y_in.items():
                    dbs[i].y[k].copy_(to_dev(v), non_blocking=True)
                runs[i].step(1, stream=streams[i])
    torch.cuda.synchronize()
    for i in range(2):
        for k in alone[i]:
            assert torch.equal(dbs[i].y[k], alone[i][k]), f"batch {i} {k}"
    res = oracle_projection(batches[1], ws, 1, 2)
    check_accumulate(bits_from_dev(dbs[1].y["down"]), res, "down of the second batch")


def test_results_are_bit_identical_run_to_run():
    w = moe_workload(16, 520, 264, E=4, k=2, tokens=200)
    b = W.make_batch(w, 20, y_mode="normal")
    ws = W.make_weights(w, 20, bank_elems=1 << 21)
    dp = DevicePool(ws, b.scale)
    outs = []
    for _ in range(3):
        db = DeviceBatch(b)
        LayerRunner(dp, db).step(0)
        torch.cuda.synchronize()
        outs.append({k: v.clone() for k, v in db.y.items()})
    for k in outs[0]:
        assert torch.equal(outs[0][k], outs[1][k]) and torch.equal(outs[0][k], outs[2][k])


def test_row_permutation_invariance_on_gpu():
    """Sec. 2.2: each row's update is independent of the batch it travels in."""
    w = dense_workload(16, 264, 136, n=4, tokens=90)
    b = W.make_batch(w, 21, y_mode="normal", no_adapter_frac=0.1)
    ws = W.make_weights(w, 21, bank_elems=1 << 20)
    dp = DevicePool(ws, b.scale)
    db = DeviceBatch(b)
    LayerRunner(dp, db).step(0)
    perm = np.random.default_rng(21).permutation(90)
    b2 = W.Batch(w, b.adapter_id[perm], None, b.token_of_pair.copy(),
                 {"x": np.ascontiguousarray(b.inputs["x"][perm])},
                 {"p": np.ascontiguousarray(b.y_in["p"][perm])}, b.scale)
    db2 = DeviceBatch(b2)
    LayerRunner(dp, db2).step(0)
    torch.cuda.synchronize()
    a, c = bits_from_dev(db.y["p"]), bits_from_dev(db2.y["p"])
    # rows of a segment are summed independently, so even the bits agree
    assert np.array_equal(a[perm], c)


def test_argument_errors_on_the_device_path():
    w = dense_workload(16, 200, 136, tokens=20)
    b = W.make_batch(w, 22)
    ws = W.make_weights(w, 22, bank_elems=1 << 20)
    dp, db = DevicePool(ws, b.scale), DeviceBatch(b)
    run = LayerRunner(dp, db)
    x = db.inputs["x"]
    with pytest.raises(L.LoraError) as e:      # segments not built yet
        L.lora_shrink(dp.pool, 0, 0, x, 200, None, db.seg, run.v)
    assert e.value.status == -5
    run.build_segments()
    for args, status in [((1, 0, x, 200), -2), ((0, 1, x, 200), -2), ((0, 0, x, 192), -2),
                         ((0, 0, x, 204), -2), ((0, 0, x.data_ptr() + 2, 200), -7),
                         ((0, 0, None, 200), -1)]:
        with pytest.raises(L.LoraError) as e:
            L.lora_shrink(dp.pool, args[0], args[1], args[2], args[3], None, db.seg, run.v)
        assert e.value.status == status, args
    with pytest.raises(L.LoraError) as e:
        L.lora_expand(dp.pool, 0, 0, run.v, db.seg, db.y["p"], 136, 7)
    assert e.value.status == -1
    with pytest.raises(L.LoraError) as e:
        L.lora_moe_apply(dp.pool, 0, 0, x, 200, None, db.seg, db.y["p"], db.y["p"], 136, run.v)
    assert e.value.status == -2            # not a three-projection pool
    y = db.y["p"]
    small = torch.empty(16, dtype=torch.float32, device="cuda")
    for n_proj, ws, status in [(2, run.v, -2), (4, run.v, -1), (0, run.v, -1), (1, small, -4)]:
        with pytest.raises(L.LoraError) as e:      # group beyond the pool / too many / none / small ws
            L.lora_apply_group(dp.pool, 0, 0, x, 200, None, db.seg, [y] * n_proj, [136] * n_proj, ws)
        assert e.value.status == status, n_proj
    with pytest.raises(L.LoraError) as e:
        L.lora_apply(dp.pool, 0, 0, x, 200, None, db.seg, y, 128, run.v)
    assert e.value.status == -2            # ldy smaller than the width
