"""Pins for the fp64 CPU oracle (CPU only).

Each test fixes the oracle to something other than itself: values the paper prints, closed
forms, library routines on special cases, invariants, brute force with exact rational
arithmetic on tiny inputs.  Together they are meant to catch a dropped term, a wrong sign
or index, a transposed operand, a mis-selected unit, a wrong rounding rule.
"""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

import workloads as W
from oracle import lora_oracle as O


def bits(a):
    return W.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def f64(b):
    return W.bf16_bits_to_f32(b).astype(np.float64)


def rand_case(seed, P=9, h=40, r=4, d=24, n=3, E=1, std_w=0.5):
    rng = np.random.default_rng(seed)
    x = bits(rng.standard_normal((P, h)))
    A = [bits(rng.standard_normal((h, r)) * std_w) for _ in range(n * E)]
    B = [bits(rng.standard_normal((r, d)) * std_w) for _ in range(n * E)]
    aid = rng.integers(0, n, size=P).astype(np.int32)
    eid = rng.integers(0, E, size=P).astype(np.int32) if E > 1 else None
    scale = (0.5 + rng.random(n)).astype(np.float32)
    y = bits(rng.standard_normal((P, d)))
    return x, A, B, aid, eid, scale, y


# ------------------------------------------------------------------ paper-printed values


def _read_golden(path):
    out = {}
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, *v = line.split()
        out.setdefault(k, []).append([float(t) for t in v])
    return out


def test_adapter_footprint_matches_paper(golden_dir):
    """Sec. 2.3 prints 1.69 GB per Mixtral-8x7B rank-64 adapter (Table 3 shapes)."""
    g = _read_golden(os.path.join(golden_dir, "mixtral_r64_adapter_footprint.txt"))
    projs = [(int(a), int(b)) for a, b in g["proj"]]
    nbytes = O.adapter_bytes(int(g["layers"][0][0]), int(g["experts"][0][0]), projs,
                             int(g["rank"][0][0]))
    assert nbytes == 1811939328
    assert round(nbytes / 2 ** 30, 2) == g["paper_gb"][0][0]
    # the fused-upgate reading (one LoRA over a 2f-wide matrix) does not give the paper's figure
    fused = O.adapter_bytes(32, 8, [(4096, 2 * 14336), (14336, 4096)], 64)
    assert round(fused / 2 ** 30, 2) != g["paper_gb"][0][0]


def test_hand_example(golden_dir):
    g = _read_golden(os.path.join(golden_dir, "hand_example.txt"))
    h, r, d = int(g["h"][0][0]), int(g["r"][0][0]), int(g["d"][0][0])
    x = bits(np.array(g["x"][0]).reshape(1, h))
    A = bits(np.array(g["A"][0]).reshape(h, r))
    B = bits(np.array(g["B"][0]).reshape(r, d))
    y = bits(np.array(g["y_in"][0]).reshape(1, d))
    res = O.delta(x, np.array([0], np.int32), [A], [B], np.array(g["s"][0], np.float32),
                  n_adapters=1, y_in=y)
    assert res.status == 0
    assert res.v.tolist() == [g["v"][0]]
    assert res.delta.tolist() == [g["delta"][0]]
    assert res.y_out.tolist() == [g["y_out"][0]]
    assert f64(res.y_bf16).tolist() == [g["y_out"][0]]  # 28.5 and 31 are bf16 values


# ------------------------------------------------------------------ closed forms


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_merged_weight_form(seed):
    """delta = s * x (A B): form the merged update A B first (Sec. 2.2, W' = W + AB)."""
    x, A, B, aid, _, scale, y = rand_case(seed)
    res = O.delta(x, aid, A, B, scale, n_adapters=3, y_in=y)
    for p in range(x.shape[0]):
        a = aid[p]
        M = f64(A[a]) @ f64(B[a])               # h x d, non-square: a transposed operand fails
        want = float(scale[a]) * (f64(x[p]) @ M)
        np.testing.assert_allclose(res.delta[p], want, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(res.y_out[p], f64(y[p]) + want, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(res.v[p], f64(x[p]) @ f64(A[a]), rtol=1e-12, atol=1e-13)


def test_zero_B_gives_zero_delta_and_identical_output():
    x, A, B, aid, _, scale, y = rand_case(3)
    B = [np.zeros_like(b) for b in B]
    res = O.delta(x, aid, A, B, scale, n_adapters=3, y_in=y)
    assert np.all(res.delta == 0.0)
    assert np.array_equal(res.y_bf16, y)
    assert np.array_equal(res.y_out, f64(y))


def test_rank1_closed_form():
    rng = np.random.default_rng(4)
    P, h, d = 5, 33, 17
    x = bits(rng.standard_normal((P, h)))
    a = bits(rng.standard_normal((h, 1)))
    b = bits(rng.standard_normal((1, d)))
    s = np.array([1.5], np.float32)
    res = O.delta(x, np.zeros(P, np.int32), [a], [b], s, n_adapters=1)
    for p in range(P):
        dot = float(np.sum(f64(x[p]) * f64(a)[:, 0]))
        np.testing.assert_allclose(res.delta[p], 1.5 * dot * f64(b)[0], rtol=1e-12, atol=1e-14)


def test_single_adapter_is_a_plain_gemm():
    rng = np.random.default_rng(5)
    P, h, r, d = 12, 64, 8, 48
    x = bits(rng.standard_normal((P, h)))
    A = bits(rng.standard_normal((h, r)) * 0.1)
    B = bits(rng.standard_normal((r, d)) * 0.1)
    res = O.delta(x, np.zeros(P, np.int32), [A], [B], np.array([1.0], np.float32), n_adapters=1)
    want = np.matmul(np.matmul(f64(x), f64(A)), f64(B))
    np.testing.assert_allclose(res.delta, want, rtol=1e-12, atol=1e-14)


def test_linearity_in_scale_and_input():
    x, A, B, aid, _, scale, _ = rand_case(6)
    r1 = O.delta(x, aid, A, B, scale, n_adapters=3)
    r2 = O.delta(x, aid, A, B, (scale * np.float32(4.0)).astype(np.float32), n_adapters=3)
    assert np.array_equal(r2.delta, 4.0 * r1.delta)        # power-of-two factor: exact
    x2 = bits(W.bf16_bits_to_f32(x) * np.float32(2.0))     # exact in bf16
    r3 = O.delta(x2, aid, A, B, scale, n_adapters=3)
    assert np.array_equal(r3.delta, 2.0 * r1.delta)
    assert np.array_equal(r3.v, 2.0 * r1.v)


# ------------------------------------------------------------------ invariants


def test_row_permutation_permutes_outputs_exactly():
    """Sec. 2.2: each request computes its own update independently of the batch."""
    x, A, B, aid, eid, scale, y = rand_case(7, P=16, n=3, E=2)
    res = O.delta(x, aid, A, B, scale, n_adapters=3, n_experts=2, expert_id=eid, y_in=y)
    perm = np.random.default_rng(70).permutation(16)
    resp = O.delta(np.ascontiguousarray(x[perm]), aid[perm], A, B, scale, n_adapters=3,
                   n_experts=2, expert_id=eid[perm], y_in=np.ascontiguousarray(y[perm]))
    assert np.array_equal(resp.delta, res.delta[perm])
    assert np.array_equal(resp.y_bf16, res.y_bf16[perm])
    # a row computed alone equals the same row inside the batch
    one = O.delta(x[5:6], aid[5:6], A, B, scale, n_adapters=3, n_experts=2, expert_id=eid[5:6],
                  y_in=y[5:6])
    assert np.array_equal(one.delta[0], res.delta[5])


def test_rows_without_adapter_are_untouched():
    x, A, B, aid, _, scale, y = rand_case(8, P=10)
    aid = aid.copy()
    aid[[1, 4, 9]] = -1
    res = O.delta(x, aid, A, B, scale, n_adapters=3, y_in=y)
    assert res.status == 0
    for p in (1, 4, 9):
        assert np.array_equal(res.y_bf16[p], y[p])
        assert np.all(res.delta[p] == 0.0) and np.all(res.v[p] == 0.0)
    full = O.delta(x, np.where(aid < 0, 0, aid).astype(np.int32), A, B, scale, n_adapters=3, y_in=y)
    keep = aid >= 0
    assert np.array_equal(res.delta[keep], full.delta[keep])


def test_out_of_range_ids_are_reported():
    x, A, B, aid, _, scale, _ = rand_case(9)
    aid = aid.copy()
    aid[2] = 3
    assert O.delta(x, aid, A, B, scale, n_adapters=3).status == -1
    aid[2] = -2
    assert O.delta(x, aid, A, B, scale, n_adapters=3).status == -1


def test_unit_selection_by_adapter_and_expert():
    """Sec. 4.1: units form an n x l x e tensor; a row uses the unit of (its adapter, its
    expert).  Tag every unit so that the delta names the unit that was used."""
    n, E, h, d = 3, 4, 8, 8
    x = bits(np.ones((n * E, h)))
    A = [bits(np.ones((h, 1))) for _ in range(n * E)]
    B = [bits(np.full((1, d), float(u + 1))) for u in range(n * E)]
    aid = np.repeat(np.arange(n), E).astype(np.int32)
    eid = np.tile(np.arange(E), n).astype(np.int32)
    res = O.delta(x, aid, A, B, np.ones(n, np.float32), n_adapters=n, n_experts=E, expert_id=eid)
    for p in range(n * E):
        assert np.all(res.delta[p] == h * (aid[p] * E + eid[p] + 1))


def test_src_row_indirection():
    x, A, B, aid, _, scale, _ = rand_case(10, P=8)
    src = np.array([3, 3, 0, 7, 1, 1, 2, 6], np.int32)
    res = O.delta(x, aid, A, B, scale, n_adapters=3, src_row=src)
    ref = O.delta(np.ascontiguousarray(x[src]), aid, A, B, scale, n_adapters=3)
    assert np.array_equal(res.delta, ref.delta)


# ------------------------------------------------------------------ brute force, exact


def test_tiny_exhaustive_exact_rational():
    """All inputs small integers: every product and sum is exact, so the oracle must equal
    exact rational arithmetic written straight from y' = xW + s*xAB, for every assignment of
    two rows to {none, adapter 0, adapter 1} x {expert 0, expert 1}."""
    vals = [-2, -1, 0, 1, 3]
    rng = np.random.default_rng(11)
    h, r, d, n, E = 3, 2, 2, 2, 2
    for trial in range(6):
        xi = rng.choice(vals, size=(2, h))
        Ai = [rng.choice(vals, size=(h, r)) for _ in range(n * E)]
        Bi = [rng.choice(vals, size=(r, d)) for _ in range(n * E)]
        yi = rng.choice(vals, size=(2, d))
        sc = [Fraction(1, 2), Fraction(2)]
        for ids in itertools.product([(-1, 0), (0, 0), (0, 1), (1, 0), (1, 1)], repeat=2):
            aid = np.array([i[0] for i in ids], np.int32)
            eid = np.array([i[1] for i in ids], np.int32)
            res = O.delta(bits(xi), aid, [bits(a) for a in Ai], [bits(b) for b in Bi],
                          np.array([float(s) for s in sc], np.float32), n_adapters=n, n_experts=E,
                          expert_id=eid, y_in=bits(yi))
            for p in range(2):
                for dd in range(d):
                    want = Fraction(int(yi[p, dd]))
                    if aid[p] >= 0:
                        u = aid[p] * E + eid[p]
                        acc = Fraction(0)
                        for j in range(r):
                            vj = sum(Fraction(int(xi[p, c])) * int(Ai[u][c, j]) for c in range(h))
                            acc += vj * int(Bi[u][j, dd])
                        want += sc[aid[p]] * acc
                    assert Fraction(res.y_out[p, dd]) == want


# ------------------------------------------------------------------ rounding rule


def test_bf16_rounding_ties_to_even_and_matches_bit_trick():
    assert O.bf16_rne(1.0) == 0x3F80
    assert O.bf16_rne(1.0 + 2 ** -8) == 0x3F80            # tie -> even (down)
    assert O.bf16_rne(1.0 + 3 * 2 ** -8) == 0x3F82        # tie -> even (up)
    assert O.bf16_rne(1.0 + 2 ** -8 + 2 ** -30) == 0x3F81  # just above a tie
    assert O.bf16_rne(-2.5) == 0xC020
    assert O.bf16_rne(0.0) == 0 and O.bf16_rne(-0.0) == 0x8000
    assert O.bf16_rne(float("inf")) == 0x7F80
    assert O.bf16_rne(3.4e38) == 0x7F80                     # overflow rounds to inf
    assert O.bf16_rne(2.0 ** -133) == 0x0001                # smallest subnormal
    assert O.bf16_rne(2.0 ** -134) == 0x0000                # tie at half of it -> even (0)
    rng = np.random.default_rng(12)
    f = (rng.standard_normal(4000) * np.exp(rng.uniform(-30, 30, 4000))).astype(np.float32)
    trick = W.f32_to_bf16_bits(f)   # integer add-and-shift rule, an independent implementation
    got = np.array([O.bf16_rne(float(v)) for v in f], dtype=np.uint16)
    assert np.array_equal(got, trick)
    for b in (0x3F80, 0x0001, 0x7F7F, 0xC2F7):
        assert O.bf16_rne(O.bf16_to_f64(b)) == b


def test_y_bf16_is_single_rounding_of_the_exact_sum():
    x, A, B, aid, _, scale, y = rand_case(13)
    res = O.delta(x, aid, A, B, scale, n_adapters=3, y_in=y)
    got = res.y_bf16.ravel()
    want = np.array([O.bf16_rne(v) for v in res.y_out.ravel()], dtype=np.uint16)
    assert np.array_equal(got, want)
    err = np.abs(f64(res.y_bf16) - res.y_out)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(res.y_out), 1e-30))) - 7)
    assert np.all(err <= 0.5 * ulp + 1e-300)


# ------------------------------------------------------------------ segments


def brute_segments(aid, eid, n, E):
    e = eid if eid is not None else np.zeros_like(aid)
    ok = (aid >= 0) & (aid < n) & (e >= 0) & (e < E)
    rows = np.nonzero(ok)[0]
    keys = aid[rows].astype(np.int64) * E + e[rows]
    order = np.argsort(keys, kind="stable")      # library stable sort
    perm = rows[order]
    sk = keys[order]
    uniq, first = np.unique(sk, return_index=True)
    return perm.astype(np.int32), np.append(first, len(perm)).astype(np.int32), uniq.astype(np.int32)


@pytest.mark.parametrize("seed,P,n,E", [(0, 0, 3, 1), (1, 1, 1, 1), (2, 50, 4, 1), (3, 200, 7, 5),
                                         (4, 333, 64, 1), (5, 1000, 32, 8), (6, 64, 300, 3)])
def test_segments_against_library_stable_sort(seed, P, n, E):
    rng = np.random.default_rng(seed)
    aid = rng.integers(-1, n, size=P).astype(np.int32)
    eid = rng.integers(0, E, size=P).astype(np.int32) if E > 1 else None
    s = O.segments(aid, eid, n, E)
    perm, start, keys = brute_segments(aid, eid, n, E)
    assert s.n_bad == 0
    assert np.array_equal(s.perm, perm)
    assert np.array_equal(s.seg_start, start)
    assert np.array_equal(s.seg_key, keys)
    assert s.P_act == len(perm) and s.S == len(keys)
    # properties that hold at any size
    e = eid if eid is not None else np.zeros_like(aid)
    k = aid[s.perm].astype(np.int64) * E + e[s.perm]
    assert np.all(np.diff(k) >= 0)
    assert sorted(s.perm.tolist()) == np.nonzero(aid >= 0)[0].tolist()
    for i in range(s.S):
        seg = s.perm[s.seg_start[i]:s.seg_start[i + 1]]
        assert len(seg) > 0 and np.all(np.diff(seg) > 0)
        assert np.all(k[s.seg_start[i]:s.seg_start[i + 1]] == s.seg_key[i])
    hist = np.bincount(k, minlength=n * E) if len(k) else np.zeros(n * E, int)
    assert np.array_equal(np.diff(s.seg_start), hist[hist > 0])


def test_segments_invalid_ids_dropped_and_counted():
    aid = np.array([0, 5, -1, 2, -7, 1], np.int32)
    eid = np.array([0, 0, 0, 9, 0, 1], np.int32)
    s = O.segments(aid, eid, 3, 2)
    assert s.n_bad == 3                     # adapter 5, expert 9, adapter -7
    assert s.perm.tolist() == [0, 5] and s.seg_key.tolist() == [0, 3]
    assert s.seg_start.tolist() == [0, 1, 2]


def test_workload_structure_matches_paper_counts():
    """Sec. 4.1: a batch of b requests with top-k routing activates b*k units per layer;
    Zipf ids (Sec. 6.1) make distinct units grow sub-linearly with batch size (App. A.2.1)."""
    w = W.WORKLOADS["mixtral_moe_decode"]
    b = W.make_batch(W.scaled(w, projs=(W.Proj("gate", 64, 64, "x"),)), 1234)
    assert b.adapter_id.shape[0] == w.tokens * w.top_k
    s = O.segments(b.adapter_id, b.expert_id, w.n_adapters, w.n_experts)
    assert s.P_act == w.tokens * w.top_k
    small = W.scaled(w, tokens=128, projs=(W.Proj("gate", 64, 64, "x"),))
    bs = W.make_batch(small, 1234)
    ss = O.segments(bs.adapter_id, bs.expert_id, w.n_adapters, w.n_experts)
    assert ss.S < s.S < 4 * ss.S
    # every token's k experts are distinct
    assert all(len(set(r)) == w.top_k for r in b.expert_id.reshape(-1, w.top_k))


# ------------------------------------------------------------------ weighted top-k combine


def combine_case(seed, T=7, k=3, h=24, r=4, d=16, n=3, E=4, drop=0.2):
    """Per-pair updates of a small MoE down projection plus routing weights and token rows."""
    rng = np.random.default_rng(seed)
    P = T * k
    x = bits(rng.standard_normal((P, h)))
    A = [bits(rng.standard_normal((h, r)) * 0.5) for _ in range(n * E)]
    B = [bits(rng.standard_normal((r, d)) * 0.5) for _ in range(n * E)]
    tok_a = rng.integers(0, n, size=T).astype(np.int32)
    tok_a[rng.random(T) < drop] = -1
    aid = np.repeat(tok_a, k).astype(np.int32)
    eid = np.stack([rng.permutation(E)[:k] for _ in range(T)]).reshape(P).astype(np.int32)
    scale = (0.5 + rng.random(n)).astype(np.float32)
    w = rng.random(P).astype(np.float32)
    y = bits(rng.standard_normal((T, d)))
    res = O.delta(x, aid, A, B, scale, n_adapters=n, n_experts=E, expert_id=eid)
    return dict(x=x, A=A, B=B, aid=aid, eid=eid, scale=scale, w=w, y=y, delta=res.delta, T=T, k=k,
                n=n, E=E)


def test_combine_hand_example(golden_dir):
    g = _read_golden(os.path.join(golden_dir, "combine_hand_example.txt"))
    k, d = int(g["k"][0][0]), int(g["h_out"][0][0])
    delta = np.array(g["delta"][0]).reshape(-1, d)
    res = O.combine(delta, np.array(g["adapter"][0], np.int32), np.array(g["w"][0], np.float32), k,
                    y_in=bits(np.array(g["y_in"][0]).reshape(-1, d)))
    assert res.y_out.reshape(-1).tolist() == g["y_out"][0]
    assert f64(res.y_bf16).reshape(-1).tolist() == g["y_out"][0]      # all bf16 values


def test_combine_against_a_library_contraction():
    """sum_j w_j delta_j per token is an einsum over the pair axis."""
    for seed in range(4):
        c = combine_case(seed)
        res = O.combine(c["delta"], c["aid"], c["w"], c["k"], y_in=c["y"])
        d3 = c["delta"].reshape(c["T"], c["k"], -1)
        w2 = c["w"].astype(np.float64).reshape(c["T"], c["k"])
        want = f64(c["y"]) + np.einsum("tj,tjd->td", w2, d3)
        np.testing.assert_allclose(res.y_out, want, rtol=1e-13, atol=1e-13)
        np.testing.assert_allclose(res.combined, want - f64(c["y"]), rtol=0, atol=1e-12)


def test_combine_with_one_expert_and_unit_weight_is_the_plain_update():
    """k = 1 and w = 1: the token row receives exactly what the per-row update gives."""
    x, A, B, aid, eid, scale, y = rand_case(40, E=3)
    aid[2] = -1
    plain = O.delta(x, aid, A, B, scale, n_adapters=3, n_experts=3, expert_id=eid, y_in=y)
    res = O.combine(plain.delta, aid, np.ones(len(aid), np.float32), 1, y_in=y)
    assert np.array_equal(res.y_out, plain.y_out)
    assert np.array_equal(res.y_bf16, plain.y_bf16)


def test_combine_merged_weight_form():
    """sum_j w_j s x_j A_j B_j with the products A_j B_j formed first (fp64 re-association)."""
    c = combine_case(5, T=5, k=2)
    res = O.combine(c["delta"], c["aid"], c["w"], c["k"])
    for t in range(c["T"]):
        want = np.zeros(c["delta"].shape[1])
        for j in range(c["k"]):
            p = t * c["k"] + j
            if c["aid"][p] < 0:
                continue
            u = c["aid"][p] * c["E"] + c["eid"][p]
            W_merged = f64(c["A"][u]) @ f64(c["B"][u])
            want += float(c["w"][p]) * float(c["scale"][c["aid"][p]]) * (f64(c["x"][p]) @ W_merged)
        np.testing.assert_allclose(res.y_out[t], want, rtol=1e-12, atol=1e-12)


def test_combine_leaves_tokens_without_adapter_untouched_and_is_linear_in_w():
    c = combine_case(6, drop=0.4)
    res = O.combine(c["delta"], c["aid"], c["w"], c["k"], y_in=c["y"])
    tok_none = (c["aid"].reshape(c["T"], c["k"]) < 0).all(axis=1)
    assert tok_none.any() and not tok_none.all()
    assert np.array_equal(res.y_bf16[tok_none], c["y"][tok_none])
    assert np.array_equal(res.y_out[tok_none], f64(c["y"])[tok_none])
    # zero weights: nothing is added; doubling the weights doubles what is added
    zero = O.combine(c["delta"], c["aid"], np.zeros_like(c["w"]), c["k"], y_in=c["y"])
    assert np.array_equal(zero.y_bf16, c["y"])
    twice = O.combine(c["delta"], c["aid"], 2 * c["w"], c["k"], y_in=c["y"])
    np.testing.assert_allclose(twice.combined, 2 * res.combined, rtol=1e-14, atol=0)
    # a pair's garbage update is ignored when the pair has no adapter
    d2 = c["delta"].copy()
    d2[c["aid"] < 0] = 1e30
    assert np.array_equal(O.combine(d2, c["aid"], c["w"], c["k"], y_in=c["y"]).y_out, res.y_out)


def test_combine_is_invariant_under_reordering_a_tokens_experts():
    """The sum over a token's experts does not depend on their order beyond fp64 rounding."""
    c = combine_case(7, T=6, k=4, E=6)
    res = O.combine(c["delta"], c["aid"], c["w"], c["k"])
    rng = np.random.default_rng(7)
    order = np.concatenate([t * c["k"] + rng.permutation(c["k"]) for t in range(c["T"])])
    res2 = O.combine(c["delta"][order], c["aid"][order], c["w"][order], c["k"])
    np.testing.assert_allclose(res2.y_out, res.y_out, rtol=1e-13, atol=1e-13)
