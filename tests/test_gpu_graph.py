"""The library's launches inside a captured HIP graph: every replay must reproduce the eager
result bit for bit (no allocation, synchronisation or memset happens inside the calls)."""
import numpy as np
import pytest
import torch

import workloads as W
from harness import DeviceBatch, DevicePool, LayerRunner

pytestmark = pytest.mark.gpu


def test_graph_replays_match_eager():
    projs = (W.Proj("gate", 520, 1160, "x"), W.Proj("up", 520, 1160, "x"), W.Proj("down", 1160, 520, "mid"))
    w = W.Workload("t", "moe", 12, 4, 2, 16, projs, 150, "zipf", 1.0)
    b = W.make_batch(w, 31, y_mode="normal", no_adapter_frac=0.05)
    ws = W.make_weights(w, 31, n_layers=2, bank_elems=1 << 22)
    dp, db = DevicePool(ws, b.scale), DeviceBatch(b)
    run = LayerRunner(dp, db)
    # eager reference: two layers applied one after the other
    run.step(0)
    run.step(1)
    torch.cuda.synchronize()
    want = {k: v.clone() for k, v in db.y.items()}

    db.reset_y()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run.step(0)
        run.step(1)
    torch.cuda.synchronize()
    for replay in range(4):
        db.reset_y()                      # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in want:
            assert torch.equal(db.y[k], want[k]), (replay, k)
    # segments inside the graph are rebuilt from the ids at replay time
    db.adapter_id.copy_(torch.roll(db.adapter_id, 2))     # same tokens' pairs stay together
    db.reset_y()
    run.step(0)
    run.step(1)
    torch.cuda.synchronize()
    want2 = {k: v.clone() for k, v in db.y.items()}
    db.reset_y()
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    for k in want2:
        assert torch.equal(db.y[k], want2[k]), k
