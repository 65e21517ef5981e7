"""lora_build_segments against the oracle's canonical segments: bit-exact."""
import numpy as np
import pytest
import torch

import paper_2604_07173_amd as L
import workloads as W
from oracle import lora_oracle as O
from harness import to_dev

pytestmark = pytest.mark.gpu


def make_pool(n, E):
    desc = L.PoolDesc(n, 1, E, [(8, 8)], 8)
    slab = torch.empty(L.lora_pool_bytes(desc), dtype=torch.uint8, device="cuda")
    return L.lora_register_pool(desc, slab)


def run_segments(pool, aid, eid, P=None):
    P = len(aid) if P is None else P
    seg = L.Segments(max(P, 1))
    for t in (seg.perm, seg.seg_start, seg.seg_key, seg.tiles):
        t.fill_(-7)
    d_aid = to_dev(aid) if len(aid) else torch.empty(1, dtype=torch.int32, device="cuda")
    d_eid = None if eid is None else (to_dev(eid) if len(eid) else torch.empty(1, dtype=torch.int32, device="cuda"))
    L.lora_build_segments(pool, d_aid, d_eid, P, seg)
    torch.cuda.synchronize()
    return seg


def compare(seg, aid, eid, n, E):
    o = O.segments(aid, eid, n, E)
    counts = seg.counts.cpu().numpy()
    assert counts[0] == o.S and counts[1] == o.P_act and counts[3] == 0
    assert np.array_equal(seg.perm.cpu().numpy()[:o.P_act], o.perm)
    assert np.array_equal(seg.seg_start.cpu().numpy()[:o.S + 1], o.seg_start)
    assert np.array_equal(seg.seg_key.cpu().numpy()[:o.S], o.seg_key)
    # tiles: each segment cut in order into blocks of at most tile_rows rows
    tr = seg.c.tile_rows
    want = []
    for s in range(o.S):
        b, e = int(o.seg_start[s]), int(o.seg_start[s + 1])
        for r0 in range(b, e, tr):
            want.append((int(o.seg_key[s]), r0, min(tr, e - r0), s))
    assert counts[2] == len(want)
    got = seg.tiles.cpu().numpy()[:len(want)]
    assert np.array_equal(got, np.array(want, dtype=np.int32).reshape(-1, 4))
    return o


CASES = [
    # seed, P, n_adapters, n_experts, fraction of -1
    (0, 1, 1, 1, 0.0), (1, 64, 4, 1, 0.0), (2, 65, 4, 1, 0.3), (3, 256, 64, 1, 0.0),
    (4, 1000, 7, 5, 0.1), (5, 1024, 32, 8, 0.0), (6, 1025, 32, 8, 0.5), (7, 4097, 3, 2, 0.0),
    (8, 8192, 256, 128, 0.0), (9, 16384, 8, 1, 0.0), (10, 5000, 300, 300, 0.2),
    (11, 777, 1, 1, 1.0), (12, 16384, 1000, 64, 0.01),
    # long batches of few keys: several workgroups, two launches
    (13, 4096, 8, 1, 0.0), (14, 4097, 16, 16, 0.1), (15, 6143, 1, 1, 0.0), (16, 16385, 8, 1, 0.0),
    (17, 40000, 32, 8, 0.05), (18, 65536 + 37, 3, 5, 0.3), (19, 200000, 256, 1, 0.01),
    (20, 20480, 2, 1, 1.0),
    # beyond 16384 rows with more than 256 keys: several workgroups, one pass per 8 key bits, then
    # the segment boundaries from the sorted keys (two and three passes)
    (21, 16385, 257, 1, 0.0), (22, 32768, 256, 128, 0.0), (23, 40000, 300, 7, 0.1),
    (24, 100000, 70000, 1, 0.02), (25, 65536 + 2049, 3, 30000, 0.0), (26, 30000, 600, 500, 0.0),
    (27, 20000, 300, 300, 1.0), (28, 262144 + 5, 512, 128, 0.01),
    # the largest batch the library takes (LORA_MAX_ROWS_LONG rows): one pass, and three passes
    (29, 1 << 20, 16, 1, 0.0), (30, 1 << 20, 1000, 100, 0.01),
]
assert CASES[-1][1] == L.LORA_MAX_ROWS_LONG


@pytest.mark.parametrize("seed,P,n,E,drop", CASES)
def test_segments_match_oracle(seed, P, n, E, drop):
    rng = np.random.default_rng(seed)
    aid = rng.integers(0, n, size=P).astype(np.int32)
    aid[rng.random(P) < drop] = -1
    eid = rng.integers(0, E, size=P).astype(np.int32) if E > 1 else None
    pool = make_pool(n, E)
    seg = run_segments(pool, aid, eid)
    compare(seg, aid, eid, n, E)
    assert int(seg.status.cpu()[0]) == 0
    # bit-identical on a second run
    seg2 = run_segments(pool, aid, eid)
    P_act = int(seg.counts.cpu()[1])
    assert torch.equal(seg.perm[:P_act], seg2.perm[:P_act])


@pytest.mark.parametrize("P,n,E,hot", [(2000, 64, 1, 0.7), (8192, 128, 8, 0.2), (1024, 256, 1, 1.0),
                                       (300, 5, 1, 0.95)])
def test_one_hot_key_among_many(P, n, E, hot):
    """Many keys but one of them holds a large share of the rows (the counting path hands
    such a batch over to the radix path inside the kernel)."""
    rng = np.random.default_rng(P + n)
    aid = rng.integers(0, n, size=P).astype(np.int32)
    eid = rng.integers(0, E, size=P).astype(np.int32) if E > 1 else None
    mask = rng.random(P) < hot
    aid[mask] = n // 2
    if eid is not None:
        eid[mask] = E - 1
    pool = make_pool(n, E)
    seg = run_segments(pool, aid, eid)
    compare(seg, aid, eid, n, E)
    assert int(seg.status.cpu()[0]) == 0


@pytest.mark.parametrize("n,E", [(1, 2), (3, 1), (2, 3), (65536, 1), (257, 255), (1, 65535)])
def test_key_count_edges(n, E):
    """Odd and extreme numbers of keys, first and last key occupied."""
    P = 777
    rng = np.random.default_rng(n * 7 + E)
    aid = rng.integers(0, n, size=P).astype(np.int32)
    eid = rng.integers(0, E, size=P).astype(np.int32) if E > 1 else None
    aid[:3] = 0
    aid[3:6] = n - 1
    if eid is not None:
        eid[:3] = 0
        eid[3:6] = E - 1
    pool = make_pool(n, E)
    seg = run_segments(pool, aid, eid)
    compare(seg, aid, eid, n, E)


def test_random_shapes_and_skews():
    """Sixty random batches: sizes, key counts, share of rows without adapter and skew of
    the adapter popularity all drawn at random; every one bit-exact against the oracle."""
    rng = np.random.default_rng(20240607)
    for case in range(60):
        P = int(rng.choice([1, 2, 63, 64, 65, 127, 500, 1023, 1024, 2049, 4096, 7000, 16384]))
        n = int(rng.choice([1, 2, 5, 16, 64, 255, 256, 257, 1000, 4096]))
        E = int(rng.choice([1, 1, 2, 8, 16, 60, 128]))
        if n * E > 2 ** 24:
            E = 1
        power = float(rng.choice([1.0, 2.0, 4.0]))          # 1 = uniform, larger = more skew
        aid = np.minimum((n * rng.random(P) ** power).astype(np.int32), n - 1)
        aid[rng.random(P) < float(rng.choice([0.0, 0.05, 0.5]))] = -1
        eid = rng.integers(0, E, size=P).astype(np.int32) if E > 1 else None
        pool = make_pool(n, E)
        seg = run_segments(pool, aid, eid)
        try:
            compare(seg, aid, eid, n, E)
        except AssertionError as err:
            raise AssertionError(f"case {case}: P={P} n={n} E={E} power={power}") from err


def test_radix_path_forced_by_environment_gives_the_same_segments():
    """LORA_SEGMENT_PATH=radix is read once per process, so the forced run is a child process;
    it must print the digest this process computes on the default path."""
    import hashlib
    import os
    import subprocess
    import sys

    code = (
        "import numpy as np, torch, hashlib, sys\n"
        "sys.path.insert(0, 'tests')\n"
        "import test_gpu_segments as T\n"
        "print(T.digest_of_cases())\n")
    env = dict(os.environ, LORA_SEGMENT_PATH="radix")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    out = subprocess.run([sys.executable, "-c", code], cwd=root, env=env, capture_output=True, text=True,
                         timeout=300)
    assert out.returncode == 0, out.stderr[-2000:]
    assert out.stdout.strip().splitlines()[-1] == digest_of_cases()


def digest_of_cases():
    """Digest of the segment arrays of a few batches that take the counting path by default."""
    import hashlib
    h = hashlib.sha256()
    for seed, P, n, E, drop in [(5, 1024, 32, 8, 0.0), (8, 8192, 256, 128, 0.0), (2, 65, 4, 1, 0.3),
                                (10, 5000, 300, 100, 0.2)]:
        rng = np.random.default_rng(seed)
        aid = rng.integers(0, n, size=P).astype(np.int32)
        aid[rng.random(P) < drop] = -1
        eid = rng.integers(0, E, size=P).astype(np.int32) if E > 1 else None
        seg = run_segments(make_pool(n, E), aid, eid)
        o = compare(seg, aid, eid, n, E)
        c = seg.counts.cpu().numpy()
        for t, k in ((seg.perm, c[1]), (seg.seg_start, c[0] + 1), (seg.seg_key, c[0])):
            h.update(t.cpu().numpy()[:k].tobytes())
        h.update(seg.tiles.cpu().numpy()[:c[2]].tobytes())
    return h.hexdigest()


def test_empty_batch_writes_zero_counts():
    pool = make_pool(4, 1)
    seg = L.Segments(1)
    seg.counts.fill_(9)
    L.lora_build_segments(pool, None, None, 0, seg)
    torch.cuda.synchronize()
    assert seg.counts.cpu().tolist() == [0, 0, 0, 0]


def test_invalid_ids_raise_status_bits_and_are_dropped():
    aid = np.array([0, 5, -1, 2, -7, 1, 2], np.int32)
    eid = np.array([0, 0, 0, 9, 0, 1, -1], np.int32)
    pool = make_pool(3, 2)
    seg = run_segments(pool, aid, eid)
    o = compare(seg, aid, eid, 3, 2)
    assert o.n_bad == 4
    assert int(seg.status.cpu()[0]) == 3      # bad adapter | bad expert
    seg = run_segments(pool, np.array([0, 1], np.int32), np.array([0, 7], np.int32))
    assert int(seg.status.cpu()[0]) == 2
    seg = run_segments(pool, np.array([0, 1], np.int32), np.array([0, 1], np.int32))
    assert int(seg.status.cpu()[0]) == 0


def test_workload_id_structures():
    """The id structure of the five workloads: Zipf adapters, top-k experts, contiguous
    prefill requests and their shuffled variant."""
    for name in ("dense_small", "llama8b_decode", "mixtral_moe_decode", "finegrained_moe_decode",
                 "prefill"):
        w = W.WORKLOADS[name]
        tiny = W.scaled(w, projs=(W.Proj("p", 8, 8, "x"),) if w.kind == "dense" else
                        (W.Proj("gate", 8, 8, "x"), W.Proj("up", 8, 8, "x"), W.Proj("down", 8, 8, "mid")))
        for seed in (1234, 1):
            b = W.make_batch(tiny, seed)
            pool = make_pool(w.n_adapters, w.n_experts)
            seg = run_segments(pool, b.adapter_id, b.expert_id)
            compare(seg, b.adapter_id, b.expert_id, w.n_adapters, w.n_experts)
    w = W.WORKLOADS["prefill"]
    b = W.make_batch(W.scaled(w, projs=(W.Proj("p", 8, 8, "x"),)), 3)
    aid = np.random.default_rng(3).permutation(b.adapter_id)
    pool = make_pool(w.n_adapters, 1)
    compare(run_segments(pool, aid, None), aid, None, w.n_adapters, 1)


def test_too_many_rows_is_a_host_error():
    """Batches of up to LORA_MAX_ROWS_LONG rows are taken, whatever the pool; beyond that the call
    refuses before it looks at any buffer."""
    seg = L.Segments(8)
    for pool in (make_pool(2, 1), make_pool(257, 1)):
        with pytest.raises(L.LoraError) as e:
            L.lora_build_segments(pool, seg.perm, None, L.LORA_MAX_ROWS_LONG + 1, seg)
        assert e.value.status == -8
    # a workspace sized for fewer rows is refused too
    with pytest.raises(L.LoraError) as e:
        L.lora_build_segments(make_pool(257, 1), seg.perm, None, L.LORA_MAX_ROWS + 1, seg)
    assert e.value.status == -4
    assert L.lora_segments_ws_bytes(L.LORA_MAX_ROWS_LONG) >= 12 * L.LORA_MAX_ROWS_LONG
    assert L.lora_segments_ws_bytes(L.LORA_MAX_ROWS) < 64 * 1024


def test_launch_counts_of_the_segment_builder():
    assert L.lora_segments_launches(make_pool(32, 8), 1024) == 1
    assert L.lora_segments_launches(make_pool(32, 8), 16384) == 2
    assert L.lora_segments_launches(make_pool(256, 128), 8192) == 1
    assert L.lora_segments_launches(make_pool(256, 128), 16385) == 6      # 15 key bits: two passes
    assert L.lora_segments_launches(make_pool(70000, 1), 100000) == 8     # 17 key bits: three passes


def test_one_hot_key_among_thousands_in_a_long_batch():
    """Most of 60000 rows on one of 40000 keys: a segment that spans dozens of chunks of the sorted
    order, next to chunks with a thousand short segments."""
    P, n, E = 60000, 400, 100
    rng = np.random.default_rng(78)
    aid = rng.integers(0, n, size=P).astype(np.int32)
    eid = rng.integers(0, E, size=P).astype(np.int32)
    hot = rng.random(P) < 0.8
    aid[hot], eid[hot] = 311, 42
    aid[rng.random(P) < 0.02] = -1
    eid[::7000] = E                          # ids outside the pool: reported and dropped
    pool = make_pool(n, E)
    seg = run_segments(pool, aid, eid)
    compare(seg, aid, eid, n, E)
    assert int(seg.status.cpu()[0]) == 2


def test_one_hot_key_in_a_long_batch():
    """Almost all of 50000 rows on one of 200 keys, the rest spread: chunks whose waves see a
    single digit next to chunks that see many."""
    P, n = 50000, 200
    rng = np.random.default_rng(77)
    aid = rng.integers(0, n, size=P).astype(np.int32)
    aid[rng.random(P) < 0.9] = 137
    aid[rng.random(P) < 0.02] = -1
    aid[::5000] = n + 3                     # ids outside the pool: reported and dropped
    pool = make_pool(n, 1)
    seg = run_segments(pool, aid, None)
    compare(seg, aid, None, n, 1)
    assert int(seg.status.cpu()[0]) == 1
