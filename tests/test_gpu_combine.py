"""lora_moe_down_combine (down projection plus the routing-weighted combine of a token's top-k
pairs into its token row) against the fp64 oracle."""
import numpy as np
import pytest
import torch

import paper_2604_07173_amd as L
import workloads as W
from gpu_common import ACC_REL, MEASURED, bf16_order, bf16_ulp, check_delta, oracle_projection
from harness import DeviceBatch, DevicePool, bits_from_dev, to_dev
from oracle import lora_oracle as O

pytestmark = pytest.mark.gpu


def moe_workload(rank, h, f, n, E, k, tokens, alpha=1.0):
    projs = (W.Proj("gate", h, f, "x"), W.Proj("up", h, f, "x"), W.Proj("down", f, h, "mid"))
    return W.Workload("t", "moe", n, E, k, rank, projs, tokens, "zipf", alpha)


def routing_weights(w, seed):
    """Softmax over the k selected logits of every token (what a router hands out), fp32."""
    rng = np.random.default_rng(seed ^ 0xC0B1)
    logits = rng.standard_normal((w.tokens, w.top_k)).astype(np.float32)
    e = np.exp(logits - logits.max(axis=1, keepdims=True))
    return (e / e.sum(axis=1, keepdims=True)).astype(np.float32).reshape(-1)


def run_combine(w, seed, y_mode, drop=0.1, bad_token=None, n_layers=1, layer=0, dp=None):
    b = W.make_batch(w, seed, y_mode="zero", no_adapter_frac=drop, hetero_scale=True)
    if bad_token is not None:                      # an id outside the pool: dropped like -1
        b.adapter_id[bad_token * w.top_k:(bad_token + 1) * w.top_k] = w.n_adapters + 5
    ws_src = W.make_weights(w, seed, n_layers=n_layers, bank_elems=1 << 22)
    rng = np.random.default_rng(seed + 1)
    h_out = w.projs[2].h_out
    if y_mode == "zero":
        y_tok = np.zeros((w.tokens, h_out), np.uint16)
    else:
        y_tok = W.f32_to_bf16_bits(rng.standard_normal((w.tokens, h_out), dtype=np.float32))
    route_w = routing_weights(w, seed)
    dp = dp or DevicePool(ws_src, b.scale)
    db = DeviceBatch(b)
    L.lora_build_segments(dp.pool, db.adapter_id, db.expert_id, db.P, db.seg)
    ws = torch.empty(L.lora_moe_combine_ws_bytes(dp.pool, db.P), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)                                 # NaN patterns: nothing may be read unwritten
    y_dev = to_dev(y_tok)
    mid = db.inputs["mid"]
    L.lora_moe_down_combine(dp.pool, layer, mid, mid.shape[1], db.adapter_id, db.expert_id, db.seg,
                            to_dev(route_w), w.top_k, y_dev, h_out, ws)
    torch.cuda.synchronize()
    got = bits_from_dev(y_dev)
    # oracle: per-pair updates of the down projection, then the weighted sum per token
    aid = np.where((b.adapter_id >= 0) & (b.adapter_id < w.n_adapters), b.adapter_id, -1).astype(np.int32)
    b_valid = W.Batch(w, aid, b.expert_id, b.token_of_pair, b.inputs, b.y_in, b.scale)
    pair = oracle_projection(b_valid, ws_src, layer, 2, use_y=False)
    want = O.combine(pair.delta, aid, route_w, w.top_k, y_in=y_tok)
    spread = np.abs(route_w.astype(np.float64)[:, None] * pair.delta).reshape(w.tokens, w.top_k, -1).sum(1)
    return dict(b=b, aid=aid, got=got, want=want, y_tok=y_tok, spread=spread, dp=dp, db=db, ws=ws,
                route_w=route_w, pair=pair)


def check_combined(r, what, y_mode):
    got = W.bf16_bits_to_f32(r["got"]).astype(np.float64)
    want = r["want"]
    if y_mode == "zero":
        check_delta(got, want.combined, what)
        return
    # accumulate mode.  Per element: one bf16 step at the exact sum for the final rounding, plus
    # the rounding of every pair's update to bf16 before it is weighted (half a step each,
    # 2^-9 relative; 2^-8 leaves room for the hi/lo split and the fp32 sums), plus the fp32
    # accumulation error of the update itself.
    err = np.abs(got - want.y_out)
    row_scale = np.max(np.abs(want.combined), axis=1, keepdims=True)
    bound = bf16_ulp(want.y_out) + 2.0 ** -8 * r["spread"] + ACC_REL * row_scale
    assert not (err > bound).any(), f"{what}: worst ratio {float((err / bound).max()):.2f}"
    steps = np.abs(bf16_order(r["got"]) - bf16_order(want.y_bf16))
    MEASURED[("combine accumulate", what)] = dict(worst_ratio=float((err / bound).max()),
                                                  frac_more_than_one_step=float((steps > 1).mean()),
                                                  elements=int(err.size))
    den = np.linalg.norm(want.y_out)
    assert np.linalg.norm(got - want.y_out) / den <= 5e-3


CASES = [
    ("mixtral-like", dict(rank=16, h=520, f=776, n=12, E=4, k=2, tokens=150)),
    ("fine-grained-like", dict(rank=8, h=264, f=136, n=40, E=16, k=8, tokens=64)),
    ("rank 64", dict(rank=64, h=392, f=264, n=5, E=3, k=3, tokens=50)),
    ("long segments", dict(rank=16, h=264, f=200, n=2, E=2, k=2, tokens=300)),
]


@pytest.mark.parametrize("y_mode", ["zero", "normal"])
@pytest.mark.parametrize("name,shape", CASES, ids=[c[0] for c in CASES])
def test_down_combine_matches_oracle(name, shape, y_mode, monkeypatch):
    if name == "long segments":                    # the long-segment kernels, forced for so few rows
        monkeypatch.setenv("LORA_TILE_ROWS", "32")
    w = moe_workload(**shape)
    r = run_combine(w, 101, y_mode, bad_token=3)
    assert r["db"].seg.c.tile_rows == (32 if name == "long segments" else 16)
    assert int(r["db"].seg.status.cpu()[0]) & 1           # the id outside the pool was reported
    check_combined(r, f"combine {name}", y_mode)
    # token rows without any valid pair keep their bits
    untouched = (r["aid"].reshape(w.tokens, w.top_k) < 0).all(axis=1)
    assert untouched[3] and untouched.sum() >= 2
    assert np.array_equal(r["got"][untouched], r["y_tok"][untouched])


def test_down_combine_at_the_mixtral_shape():
    """Full widths (14336 -> 4096), 512 tokens x top-2, 32 adapters x 8 experts."""
    w = W.WORKLOADS["mixtral_moe_decode"]
    r = run_combine(w, 1234, "zero", drop=0.02)
    check_combined(r, "combine mixtral_moe_decode", "zero")
    r2 = run_combine(w, 1234, "normal", drop=0.02, dp=r["dp"])
    check_combined(r2, "combine mixtral_moe_decode", "normal")


def test_down_combine_is_bit_identical_run_to_run_and_partial_tokens_count():
    w = moe_workload(16, 264, 392, n=6, E=4, k=4, tokens=40)
    r = run_combine(w, 7, "normal", drop=0.0)
    b, db, dp = r["b"], r["db"], r["dp"]
    # a token with only some of its pairs active: make two pairs of token 5 adapter-less
    aid = b.adapter_id.copy()
    aid[5 * 4 + 1] = -1
    aid[5 * 4 + 3] = -1
    dev_aid = to_dev(aid)
    L.lora_build_segments(dp.pool, dev_aid, db.expert_id, db.P, db.seg)
    outs = []
    for _ in range(3):
        y = to_dev(r["y_tok"])
        mid = db.inputs["mid"]
        L.lora_moe_down_combine(dp.pool, 0, mid, mid.shape[1], dev_aid, db.expert_id, db.seg,
                                to_dev(r["route_w"]), 4, y, y.shape[1], r["ws"])
        torch.cuda.synchronize()
        outs.append(bits_from_dev(y))
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])
    want = O.combine(r["pair"].delta, aid, r["route_w"], 4, y_in=r["y_tok"])
    r.update(got=outs[0], want=want, aid=aid)
    act = (aid >= 0)[:, None]
    r["spread"] = (np.abs(r["route_w"].astype(np.float64)[:, None] * r["pair"].delta) * act).reshape(40, 4, -1).sum(1)
    check_combined(r, "combine partial token", "normal")
    assert not np.array_equal(want.y_out[5], O.combine(r["pair"].delta, b.adapter_id, r["route_w"], 4,
                                                       y_in=r["y_tok"]).y_out[5])


def test_down_combine_argument_errors():
    w = moe_workload(16, 136, 200, n=3, E=2, k=2, tokens=10)
    r = run_combine(w, 9, "zero", drop=0.0)
    dp, db, ws = r["dp"], r["db"], r["ws"]
    mid = db.inputs["mid"]
    y = to_dev(r["y_tok"])
    rw = to_dev(r["route_w"])

    def call(top_k=2, ws_=ws, ldy=136, layer=0, rw_=rw, aid=db.adapter_id):
        L.lora_moe_down_combine(dp.pool, layer, mid, mid.shape[1], aid, db.expert_id, db.seg, rw_,
                                top_k, y, ldy, ws_)

    for kwargs, status in [(dict(top_k=0), -1), (dict(top_k=17), -1), (dict(top_k=3), -2),
                           (dict(ws_=torch.empty(64, dtype=torch.uint8, device="cuda")), -4),
                           (dict(ldy=128), -2), (dict(layer=1), -2), (dict(rw_=None), -1),
                           (dict(aid=None), -1)]:
        with pytest.raises(L.LoraError) as e:
            call(**kwargs)
        assert e.value.status == status, kwargs
    torch.cuda.synchronize()
    assert np.array_equal(bits_from_dev(y), r["y_tok"])       # nothing was enqueued
