#!/usr/bin/env python3
"""Benchmark of the batched heterogeneous-adapter LoRA delta on one MI355X.

A "step" is one layer call of the whole hot path over one synthetic batch: build segments,
then shrink and expand of every projection (for MoE workloads the up/gate and the down
application).  Weights, activations, ids and outputs are resident in HBM before the timed
region.  The layer index rotates over several layers' worth of pool so that adapter weights
come from HBM, not from the 256 MB last-level cache, as they do in layer-by-layer decoding.

Prints one JSON line (the README lists the fields).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth
COLD_SETS = 24          # copies of the activation buffers of the cold-activation measurement (2.5 GB for the Mixtral batch)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="mixtral_moe_decode")
    ap.add_argument("--layers", type=int, default=0, help="layers in the pool (0 = per-workload default)")
    ap.add_argument("--seed", type=int, default=1234)
    ap.add_argument("--hot", action="store_true", help="reuse one layer (weights warm in cache)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-two-calls", action="store_true",
                    help="skip the two-calls-in-flight measurement (kernel traces then hold one stream only)")
    ap.add_argument("--all", action="store_true",
                    help="also measure the other workloads and the layer-wise adapter load (extra field)")
    ap.add_argument("--down-combine", action="store_true",
                    help="MoE workloads: replace the down application (update added to every pair's "
                         "row) by lora_moe_down_combine (routing-weighted sum into token rows); "
                         "a variant for comparison, not the headline")
    ap.add_argument("--activation-sets", type=int, default=1,
                    help="rotate the steps over this many copies of the batch's device buffers (ids, "
                         "activations, base outputs): with enough copies no activation byte of a "
                         "step is still in a cache when the step comes round again")
    ap.add_argument("--activation-policy", choices=["auto", "resident", "streaming"], default="auto",
                    help="lora_pool_set_activation_policy for the pool of the run")
    ap.add_argument("--no-cold-activations", action="store_true",
                    help="skip the extra measurement over rotated copies of the activation buffers")
    ap.add_argument("--tokens", type=int, default=0,
                    help="run the workload's shapes with another number of tokens (0 = as defined)")
    ap.add_argument("--steps-only", action="store_true",
                    help="only the warm-up and the timed steps, launched on the stream, then a short "
                         "JSON line: what a kernel trace or a counter run should see")
    ap.add_argument("--launch", choices=["graph", "stream"], default="graph",
                    help="how the timed steps are launched: one HIP graph holding all K steps "
                         "(as a serving engine captures a decode iteration), or plain stream launches")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy a few times (reference for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


DEFAULT_LAYERS = {"dense_small": 8, "llama8b_decode": 8, "prefill": 4, "mixtral_moe_decode": 8,
                  "finegrained_moe_decode": 4, "mixtral_r64_microbench": 1}


class Phase:
    def __init__(self, name, fn, bytes_):
        self.name, self.fn, self.bytes = name, fn, bytes_


def make_phases(L, W, dp, db, run, acct, down_combine=False):
    """The launches of one step, each with the algorithmic bytes it must move."""
    w = dp.workload
    pool, seg = dp.pool, db.seg
    S, P_act, T_act, r = acct["S"], acct["P_act"], acct["T_act"], w.rank
    phases = [Phase("build_segments", lambda layer: run.build_segments(), 12 * db.P)]
    if w.kind == "moe":
        g, d = w.projs[0], w.projs[2]
        x, mid = db.inputs["x"], db.inputs["mid"]
        phases.append(Phase(
            "upgate_shrink",
            lambda layer: L.lora_moe_shrink(pool, layer, L.LORA_MOE_UPGATE, x, x.shape[1],
                                            db.token_of_pair, seg, run.ws),
            2 * S * r * g.h_in * 2 + T_act * g.h_in * 2))
        phases.append(Phase(
            "upgate_expand",
            lambda layer: L.lora_moe_expand(pool, layer, L.LORA_MOE_UPGATE, seg, db.y["gate"],
                                            db.y["up"], db.y["gate"].shape[1], run.ws),
            2 * (S * r * g.h_out * 2 + P_act * g.h_out * 4)))
        if down_combine:
            import numpy as np
            import torch
            from harness import to_dev
            k, T = w.top_k, w.tokens
            rng = np.random.default_rng(7)
            route_w = to_dev(rng.dirichlet(np.ones(k), size=T).astype(np.float32).reshape(-1))
            y_tok = to_dev(W.f32_to_bf16_bits(rng.standard_normal((T, d.h_out), dtype=np.float32)))
            cws = torch.empty(L.lora_moe_combine_ws_bytes(pool, db.P), dtype=torch.uint8, device="cuda")
            # shrink as before; every touched B once; the pair rows written and read once (bf16);
            # token rows read and written once
            phases.append(Phase(
                "down_combine",
                lambda layer: L.lora_moe_down_combine(pool, layer, mid, mid.shape[1], db.adapter_id,
                                                      db.expert_id, seg, route_w, k, y_tok, d.h_out, cws),
                S * r * d.h_in * 2 + P_act * d.h_in * 2 + S * r * d.h_out * 2 + P_act * d.h_out * 4
                + T_act * d.h_out * 4))
            return phases
        phases.append(Phase(
            "down_shrink",
            lambda layer: L.lora_moe_shrink(pool, layer, L.LORA_MOE_DOWN, mid, mid.shape[1], None,
                                            seg, run.ws),
            S * r * d.h_in * 2 + P_act * d.h_in * 2))
        phases.append(Phase(
            "down_expand",
            lambda layer: L.lora_moe_expand(pool, layer, L.LORA_MOE_DOWN, seg, db.y["down"], None,
                                            db.y["down"].shape[1], run.ws),
            S * r * d.h_out * 2 + P_act * d.h_out * 4))
    else:
        # one call per run of projections that share an input (q/k/v, gate/up): a shrink launch
        # and an expand launch for the whole group
        seen = set()
        for j, c in run.groups:
            projs = w.projs[j:j + c]
            xb = 0 if projs[0].input in seen else P_act * projs[0].h_in * 2
            seen.add(projs[0].input)
            nbytes = xb + sum(S * r * (p.h_in + p.h_out) * 2 + P_act * p.h_out * 4 for p in projs)
            phases.append(Phase("+".join(p.name for p in projs) + "_apply",
                                lambda layer, j=j, c=c: run.apply_group(layer, j, c), nbytes))
    return phases


def launches_per_step(w, dp, db, run, combine=False):
    """How many kernel launches one step takes: 1 or 2 for the segment build, then per group of
    projections 1 if the library runs shrink and expand as one launch, else 2 (3 for batches of
    long segments, whose expand has a launch of its own for the operand images).  With the
    routing-weighted combine the down call is shrink, expand into pair rows and the combine."""
    import paper_2604_07173_amd as L
    one = getattr(L, "lora_group_launches", None)
    if one is None:
        return None
    groups = [(0, 2), (2, 1)] if w.kind == "moe" else run.groups
    if combine:
        return (L.lora_segments_launches(dp.pool, db.P) + L.lora_group_launches(dp.pool, 0, 2, db.P, db.seg) + 3
                + (2 if db.seg.c.tile_rows > 16 else 0))
    j0, c0 = groups[0]       # the first application of the call builds the segments
    return L.lora_build_apply_launches(dp.pool, j0, c0, db.P) + sum(L.lora_group_launches(dp.pool, j, c, db.P, db.seg)
                                                                     for j, c in groups[1:])


def measure(name, args, steps, warmup, with_cpu_baseline):
    import numpy as np
    import torch

    import paper_2604_07173_amd as L
    import workloads as W
    from harness import DeviceBatch, DevicePool, LayerRunner

    w = W.WORKLOADS[name]
    if getattr(args, "tokens", 0):
        w = W.scaled(w, tokens=args.tokens)
    n_layers = 1 if args.hot else (args.layers or DEFAULT_LAYERS.get(name, 4))
    b = W.make_batch(w, args.seed, y_mode="normal")
    ws = W.make_weights(w, args.seed, n_layers=n_layers)
    dp = DevicePool(ws, b.scale)
    policies = {"auto": L.LORA_ACT_AUTO, "resident": L.LORA_ACT_RESIDENT, "streaming": L.LORA_ACT_STREAMING}
    policy = policies[getattr(args, "activation_policy", "auto")]
    L.lora_pool_set_activation_policy(dp.pool, policy)
    db = DeviceBatch(b)
    run = LayerRunner(dp, db)
    acct = W.algorithmic_bytes(w, b.adapter_id, b.expert_id)
    phases = make_phases(L, W, dp, db, run, acct, getattr(args, "down_combine", False) and w.kind == "moe")

    combine = getattr(args, "down_combine", False) and w.kind == "moe"

    n_sets = 1 if combine else max(1, getattr(args, "activation_sets", 1))
    runs = [run]
    for _ in range(n_sets - 1):
        runs.append(LayerRunner(dp, DeviceBatch(b)))

    def step(it):
        # the calls a server makes for one layer: lora_build_segments, then lora_moe_apply for
        # up/gate and for down (MoE) or lora_apply_group per run of projections that share an
        # input (dense).  The library decides by itself whether shrink and expand of a group run
        # as one launch or two; the phases below time the two halves on their own.
        layer = it % n_layers
        if combine:
            for ph in phases:
                ph.fn(layer)
        else:
            runs[it % n_sets].step(layer)

    # ---- whole-step throughput ----------------------------------------------------------
    for it in range(warmup):
        step(it)
    torch.cuda.synchronize()
    launches = launches_per_step(w, dp, db, run, combine)      # the segments are built by now
    t0 = time.perf_counter()
    for it in range(steps):
        step(warmup + it)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    stream_ms_per_step = (t1 - t0) * 1e3 / steps
    ms_per_step = stream_ms_per_step
    if getattr(args, "steps_only", False):
        return dict(workload=name, tokens=w.tokens, rows=int(db.P), ms_per_step=ms_per_step,
                    launches_per_step=launches, segments=acct["S"], active_rows=acct["P_act"],
                    algorithmic_bytes=int(acct["total"]),
                    phase_bytes={ph.name: int(ph.bytes) for ph in phases})
    replay_ms = []
    if args.launch == "graph":
        # the same K steps recorded once into a HIP graph and replayed: no allocation, no
        # synchronisation and no memset inside, so the library's launches capture as they are
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for it in range(steps):
                step(warmup + it)
        torch.cuda.synchronize()
        graph.replay()                      # untimed: first replay uploads the graph
        torch.cuda.synchronize()
        # the timed region: EXACTLY `steps` steps (one replay); further replays of the same
        # graph only tell how far single measurements scatter
        t0 = time.perf_counter()
        graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms_per_step = (t1 - t0) * 1e3 / steps
        for _ in range(9):
            t0 = time.perf_counter()
            graph.replay()
            torch.cuda.synchronize()
            replay_ms.append((time.perf_counter() - t0) * 1e3 / steps)
        replay_ms.append(ms_per_step)
        del graph

    # ---- the same steps without the segment build (App. A.2.2 times shrink and expand only) --
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for it in range(steps):
        for ph in phases[1:]:
            ph.fn((warmup + it) % n_layers)
    torch.cuda.synchronize()
    nobuild_ms_per_step = (time.perf_counter() - t0) * 1e3 / steps

    # ---- two independent layer calls in flight (a second batch of the same workload, its own
    # segments and workspace, on a second stream): what a server that takes the calls of two
    # LLM instances at once gets out of the same kernels; the dispatch gaps of one call are
    # filled by the other.  Not the headline: the paper's server runs calls one by one. --------
    two_ms_per_step, bytes2 = float("nan"), acct["total"]
    if not getattr(args, "no_two_calls", False):
        b2 = W.make_batch(w, args.seed + 1, y_mode="normal")
        db2 = DeviceBatch(b2)
        run2 = LayerRunner(dp, db2)
        lanes = [(run, torch.cuda.Stream()), (run2, torch.cuda.Stream())]

        def two_calls(n):
            for it in range(n):
                r, st = lanes[it & 1]
                with torch.cuda.stream(st):
                    r.step((warmup + it) % n_layers, stream=st)

        two_calls(2 * max(2, warmup // 2))
        torch.cuda.synchronize()
        n2 = steps + (steps & 1)
        t0 = time.perf_counter()
        two_calls(n2)
        torch.cuda.synchronize()
        two_ms_per_step = (time.perf_counter() - t0) * 1e3 / n2
        bytes2 = W.algorithmic_bytes(w, b2.adapter_id, b2.expert_id)["total"]
        del lanes, run2, db2

    # ---- the same steps over rotated copies of the batch's device buffers: the timed steps above
    # reuse one set of buffers, so their activations (not the weights, which rotate over layers)
    # are still in the 256 MiB memory-side cache when a step comes round again, as they are when
    # the kernel before the call has just written them.  With kColdSets copies they are not.
    # Measured under the run's policy and under LORA_ACT_STREAMING, the policy meant for that case.
    cold = None
    if n_sets == 1 and not combine and not getattr(args, "no_cold_activations", False) \
            and args.launch == "graph":
        cold_runs = [LayerRunner(dp, DeviceBatch(b)) for _ in range(COLD_SETS)]

        def cold_ms(pol):
            L.lora_pool_set_activation_policy(dp.pool, pol)
            for it in range(COLD_SETS):
                cold_runs[it].step(it % n_layers)
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                for it in range(steps):
                    cold_runs[it % COLD_SETS].step((warmup + it) % n_layers)
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            ms = []
            for _ in range(3):
                t0 = time.perf_counter()
                g.replay()
                torch.cuda.synchronize()
                ms.append((time.perf_counter() - t0) * 1e3 / steps)
            del g
            return sorted(ms)[1]

        cold = dict(sets=COLD_SETS, ms_per_step=cold_ms(policy),
                    ms_per_step_streaming_policy=cold_ms(L.LORA_ACT_STREAMING))
        L.lora_pool_set_activation_policy(dp.pool, policy)
        del cold_runs
        torch.cuda.empty_cache()

    # ---- spread over the steps: an event between consecutive steps (stream launches; the
    # event records add a little to every step, so the median sits above ms_per_step) -------
    n_ev = min(steps, 200)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(n_ev + 1)]
    torch.cuda.synchronize()
    evs[0].record()
    for it in range(n_ev):
        step(warmup + it)
        evs[it + 1].record()
    torch.cuda.synchronize()
    per_step_us = np.array([evs[i].elapsed_time(evs[i + 1]) * 1e3 for i in range(n_ev)])

    # ---- per-launch durations with events on the launch stream ---------------------------
    # Each launch of the step is repeated back to back between two events (layers rotating,
    # so weights stay cold), which is how a kernel trace sees it; recording an event after
    # every single launch would add the event's own cost to each of them.
    reps = max(8, min(steps, 40))
    per_phase = {}
    for k, ph in enumerate(phases):
        step(0)                                   # valid segments / intermediates for this phase
        ph.fn(0)                                  # the launch's first use in the process is not timed
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for r in range(reps):
            ph.fn(r % n_layers)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / reps
        per_phase[ph.name] = dict(us=float(us), bytes=int(ph.bytes),
                                  gbs=float(ph.bytes / (us * 1e-6) / 1e9))
    dom = max(phases[1:], key=lambda ph: per_phase[ph.name]["us"])
    d = per_phase[dom.name]
    traffic, traffic_note = read_traffic(name, dom.name)
    roofline = dict(bound="hbm", kernel=dom.name, achieved=round(d["gbs"], 1), peak=HBM_PEAK_GBS,
                    unit="GB/s", frac=round(d["gbs"] / HBM_PEAK_GBS, 4),
                    traffic=traffic, traffic_source=traffic_note, us_per_launch=round(d["us"], 2),
                    algorithmic_bytes=int(dom.bytes))

    total_bytes = acct["total"]
    res = dict(
        workload=name, ms_per_step=ms_per_step, stream_ms_per_step=stream_ms_per_step,
        replay_ms=sorted(replay_ms),
        nobuild_ms_per_step=nobuild_ms_per_step,
        step_us_p10=float(np.percentile(per_step_us, 10)), step_us_p50=float(np.percentile(per_step_us, 50)),
        step_us_p90=float(np.percentile(per_step_us, 90)),
        tokens_per_s=w.tokens / (ms_per_step * 1e-3),
        pairs_per_s=w.pairs / (ms_per_step * 1e-3),
        step_gbs=total_bytes / (ms_per_step * 1e-3) / 1e9,
        step_frac_of_peak=total_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        two_calls=dict(ms_per_step=two_ms_per_step, tokens_per_s=w.tokens / (two_ms_per_step * 1e-3),
                       hbm_frac_of_peak=(total_bytes + bytes2) / 2 / (two_ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS),
        algorithmic_bytes=int(total_bytes), segments=acct["S"], pairs=acct["P_act"],
        layers_in_pool=n_layers, pool_gib=dp.nbytes / 2 ** 30, phases=per_phase, roofline=roofline,
        launches_per_step=launches, cold_activations=cold)

    if with_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(w, b, ws)
    del dp, db, run, runs
    torch.cuda.empty_cache()
    return res


def copy_ceiling_gbs():
    """What a plain device-to-device copy of 1 GiB reaches on this machine (bytes read + written
    per second): the practical ceiling for traffic that is part read, part write."""
    import torch
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(10):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / 10
    del src, dst
    torch.cuda.empty_cache()
    return 2 * (1 << 30) / (ms * 1e-3) / 1e9


def kernel_sources_digest():
    """Digest of the kernel sources the library is built from (comments and white space left
    out): a counter summary under profiles/ names the digest it was taken with, so a summary of
    other kernels is recognised as stale."""
    import hashlib
    import re
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2604_07173_amd", "csrc")
    for fn in sorted(os.listdir(csrc)):
        if fn.endswith((".hip", ".h")):
            text = open(os.path.join(csrc, fn), "r", errors="replace").read()
            # the code only: comments and layout do not change what the kernels do
            text = re.sub(r"/\*.*?\*/", " ", text, flags=re.S)
            text = re.sub(r"//[^\n]*", " ", text)
            h.update(fn.encode())
            h.update(" ".join(text.split()).encode())
    return h.hexdigest()[:16]


def read_traffic(workload, kernel):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE) in separate
    runs of this program, taken from the summary on file under profiles/.  The counters cannot
    be read from inside a timed run, so the figure is a measurement of an earlier run of the
    same kernels: it is reported only if the summary names the digest of the present kernel
    sources; otherwise traffic is null and the note says why."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    if not os.path.exists(path):
        return None, "no counter summary on file for this workload"
    value, digest = None, None
    for line in open(path):
        parts = line.split()
        if len(parts) >= 2 and parts[0] == f"{kernel}_traffic_bytes_per_launch:":
            try:
                value = int(float(parts[1]))
            except ValueError:
                value = None
        if len(parts) >= 2 and parts[0] == "kernel_sources_digest:":
            digest = parts[1]
    rel = os.path.relpath(path, ROOT)
    if value is None:
        return None, f"{rel} has no figure for {kernel}"
    if digest != kernel_sources_digest():
        return None, f"{rel} was taken with other kernel sources (digest {digest}); not reported"
    return value, f"{rel} (rocprofv3 --pmc run of the same kernel sources, digest {digest})"


def cpu_baseline(w, b, ws):
    """The fp64 oracle, as it stands, on this machine's host cores: one full layer call."""
    import numpy as np

    from oracle import lora_oracle as O

    def layer_call():
        O.segments(b.adapter_id, b.expert_id, w.n_adapters, w.n_experts)
        e_arr = b.expert_id if b.expert_id is not None else np.zeros_like(b.adapter_id)
        act = b.adapter_id >= 0
        units = sorted(set(zip(b.adapter_id[act].tolist(), e_arr[act].tolist())))
        for j, p in enumerate(w.projs):
            A_units = [None] * w.n_keys
            B_units = [None] * w.n_keys
            for a, e in units:
                A, B = ws.unit_arrays(a, 0, e, j)
                A_units[a * w.n_experts + e] = A
                B_units[a * w.n_experts + e] = B
            O.delta(b.inputs[p.input], b.adapter_id, A_units, B_units, b.scale,
                    n_adapters=w.n_adapters, n_experts=w.n_experts, expert_id=b.expert_id,
                    src_row=None if p.input == "mid" else b.token_of_pair, y_in=b.y_in[p.name],
                    want_v=False)

    t0 = time.perf_counter()
    layer_call()                      # first call also builds/loads the oracle
    first = time.perf_counter() - t0
    times = [first] if first > 5.0 else []     # a call of many seconds (prefill) is timed once
    t_all = time.perf_counter()
    while not times or (first <= 5.0 and (len(times) < 3 or
                                          (time.perf_counter() - t_all < 10.0 and len(times) < 20))):
        t0 = time.perf_counter()
        layer_call()
        times.append(time.perf_counter() - t0)
    t = float(np.median(times))
    return dict(value=w.tokens / t, unit="tokens/s", cores=O.n_threads(), kind="oracle",
                sample=f"full layer call of {w.name} ({w.tokens} tokens, {w.pairs} rows, "
                       f"{len(w.projs)} projections), median of {len(times)} runs, {t:.3f} s each")


def measure_adapter_load(args):
    """Sec. 5.3, layer-wise loading: one Mixtral-shaped adapter (8 experts, gate/up/down,
    rank 16) goes from pinned host memory into its pool slot layer by layer on a loading
    stream, alone and while the decode layer call keeps running on the compute stream.
    The slot is re-loaded with the bytes it already holds, so the concurrent steps read
    the same values throughout."""
    import numpy as np
    import torch

    import paper_2604_07173_amd as L
    import workloads as W
    from harness import DeviceBatch, DevicePool, LayerRunner

    w = W.WORKLOADS["mixtral_moe_decode"]
    n_layers = args.layers or DEFAULT_LAYERS.get("mixtral_moe_decode", 8)
    b = W.make_batch(w, args.seed, y_mode="normal")
    ws = W.make_weights(w, args.seed, n_layers=n_layers)
    dp = DevicePool(ws, b.scale)
    db = DeviceBatch(b)
    run = LayerRunner(dp, db)
    slot = w.n_adapters - 1
    window = L.lora_pool_adapter_layer_bytes(dp.pool, slot)
    win = window // 2
    host = torch.from_numpy(np.concatenate(
        [ws.bank[int(ws.window[slot, l]):int(ws.window[slot, l]) + win].view(np.int16)
         for l in range(n_layers)])).pin_memory()
    staging = torch.empty(win, dtype=torch.int16, device="cuda")
    load_stream = torch.cuda.Stream()

    def load_and_poll():
        t0 = time.perf_counter()
        L.lora_pool_load_adapter_async(dp.pool, slot, host, staging, load_stream=load_stream)
        while not L.lora_pool_layer_ready(dp.pool, slot, 0):
            pass
        t_first = time.perf_counter()
        while not L.lora_pool_layer_ready(dp.pool, slot, n_layers - 1):
            pass
        return t_first - t0, time.perf_counter() - t0

    def steps(n):
        for it in range(n):
            run.step(it % n_layers)

    for _ in range(2):
        load_and_poll()
    torch.cuda.synchronize()
    alone = sorted(load_and_poll() for _ in range(7))[3]
    # compute alone, then compute with a load in flight
    n = 4 * max(1, int(alone[1] / 110e-6))
    steps(20)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    steps(n)
    e1.record()
    torch.cuda.synchronize()
    step_alone = e0.elapsed_time(e1) / n
    e0.record()
    steps(n)
    e1.record()
    under = load_and_poll()
    torch.cuda.synchronize()
    step_loading = e0.elapsed_time(e1) / n
    total = window * n_layers
    return {"adapter_bytes": total, "layers": n_layers, "layer_bytes": window,
            "first_layer_ready_ms": round(alone[0] * 1e3, 3), "all_layers_ready_ms": round(alone[1] * 1e3, 3),
            "h2d_gbs": round(total / alone[1] / 1e9, 1),
            "with_decode_running": {"first_layer_ready_ms": round(under[0] * 1e3, 3),
                                    "all_layers_ready_ms": round(under[1] * 1e3, 3),
                                    "h2d_gbs": round(total / under[1] / 1e9, 1),
                                    "decode_ms_per_step_alone": round(step_alone, 5),
                                    "decode_ms_per_step_while_loading": round(step_loading, 5),
                                    "steps_enqueued": n}}


def spread(ms):
    """[min, median, max] of the per-step times of the graph replays (None without a graph)."""
    if not ms:
        return None
    ms = sorted(ms)
    return [round(ms[0], 5), round(ms[len(ms) // 2], 5), round(ms[-1], 5)]


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU; this build has no multi-GPU path (--gpus must be 1)",
              file=sys.stderr)
        return 2
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 1
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()
    if args.steps_only:
        print(json.dumps(measure(args.workload, args, args.steps, args.warmup, False)))
        return 0
    ceiling = copy_ceiling_gbs()
    main_res = measure(args.workload, args, args.steps, args.warmup, not args.no_cpu_baseline)
    out = {
        "metric": "LoRA-delta tokens/s (MoE-LoRA decode layer call) on 1 MI355X",
        "value": round(main_res["tokens_per_s"], 1),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(main_res["ms_per_step"], 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "layers_in_pool": main_res["layers_in_pool"],
                   "weights": "hot (one layer)" if args.hot else "cold (layer rotation)",
                   "launch": "one HIP graph of all timed steps" if args.launch == "graph"
                   else "stream launches",
                   "seed": args.seed, "segments": main_res["segments"], "rows": main_res["pairs"],
                   "activation_policy": args.activation_policy,
                   **({"down": "lora_moe_down_combine (token rows)"} if args.down_combine else {})},
        "graph_replays_ms_per_step_min_median_max": spread(main_res["replay_ms"]),
        "stream_launch_ms_per_step": round(main_res["stream_ms_per_step"], 5),
        "ms_per_step_without_segment_build": round(main_res["nobuild_ms_per_step"], 5),
        "step_us_p10_p50_p90": [round(main_res["step_us_p10"], 2), round(main_res["step_us_p50"], 2),
                                round(main_res["step_us_p90"], 2)],
        "hbm_gbs": round(main_res["step_gbs"], 1),
        "hbm_frac_of_peak": round(main_res["step_frac_of_peak"], 4),
        "copy_ceiling_gbs": round(ceiling, 1),
        "hbm_frac_of_copy_ceiling": round(main_res["step_gbs"] / ceiling, 4),
        "algorithmic_bytes_per_step": main_res["algorithmic_bytes"],
        "launches_per_step": main_res["launches_per_step"],
        "pairs_per_s": round(main_res["pairs_per_s"], 1),
        "phases": {k: {"us": round(v["us"], 2), "GB/s": round(v["gbs"], 1)}
                   for k, v in main_res["phases"].items()},
        "roofline": main_res["roofline"],
    }
    if not args.no_two_calls:
        out["two_calls_in_flight"] = {
            "ms_per_step": round(main_res["two_calls"]["ms_per_step"], 5),
            "tokens_per_s": round(main_res["two_calls"]["tokens_per_s"], 1),
            "hbm_frac_of_peak": round(main_res["two_calls"]["hbm_frac_of_peak"], 4),
            "note": "two independent layer calls on two streams; not the headline"}
    if main_res.get("cold_activations"):
        c = main_res["cold_activations"]
        out["cold_activations"] = {
            "buffer_sets": c["sets"], "ms_per_step": round(c["ms_per_step"], 5),
            "ms_per_step_streaming_policy": round(c["ms_per_step_streaming_policy"], 5),
            "note": "steps rotate over copies of the activation buffers, so no activation is "
                    "cache-resident when its step starts; not the headline"}
    if "cpu_baseline" in main_res:
        out["cpu_baseline"] = main_res["cpu_baseline"]
    if args.all:
        extra = {}
        for name in ("dense_small", "llama8b_decode", "prefill", "finegrained_moe_decode"):
            if name == args.workload:
                continue
            r = measure(name, args, max(20, args.steps // 4), max(5, args.warmup // 2),
                        not args.no_cpu_baseline)
            extra[name] = {"ms_per_step": round(r["ms_per_step"], 5),
                           "tokens_per_s": round(r["tokens_per_s"], 1),
                           "hbm_gbs": round(r["step_gbs"], 1),
                           "hbm_frac_of_peak": round(r["step_frac_of_peak"], 4),
                           "algorithmic_bytes_per_step": r["algorithmic_bytes"],
                           "launches_per_step": r["launches_per_step"],
                           "graph_replays_ms_per_step_min_median_max": spread(r["replay_ms"]),
                           "two_calls_in_flight_ms_per_step":
                               None if args.no_two_calls else round(r["two_calls"]["ms_per_step"], 5),
                           "phases": {k: {"us": round(v["us"], 2), "GB/s": round(v["gbs"], 1)}
                                      for k, v in r["phases"].items()},
                           "roofline": r["roofline"]}
            if r.get("cold_activations"):
                c = r["cold_activations"]
                extra[name]["cold_activations_ms_per_step"] = round(c["ms_per_step"], 5)
                extra[name]["cold_activations_ms_per_step_streaming_policy"] = round(
                    c["ms_per_step_streaming_policy"], 5)
            if "cpu_baseline" in r:
                extra[name]["cpu_baseline"] = r["cpu_baseline"]
        extra["adapter_load_mixtral"] = measure_adapter_load(args)
        out["extra"] = extra
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
