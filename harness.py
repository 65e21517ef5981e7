"""Glue between the synthetic workloads and the library: builds a pool from a weight bank,
uploads a batch, and issues the calls of one layer.  Marshalling only — used by the GPU
tests, the smoke check and the benchmark.  Holds no arithmetic of the method.
"""
from __future__ import annotations

from typing import Dict, List, Optional

import numpy as np
import torch

import workloads as W

import paper_2604_07173_amd as L


def to_dev(a: np.ndarray, device="cuda") -> torch.Tensor:
    """numpy -> device tensor; uint16 (bf16 bits) travels as int16, uint32 as int32."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    elif a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).to(device)


def bits_from_dev(t: torch.Tensor) -> np.ndarray:
    """device int16 tensor of bf16 bits -> numpy uint16."""
    return t.detach().cpu().numpy().view(np.uint16)


class DevicePool:
    """A pool in HBM filled from a WeightSource (bank windows -> lora_pool_load_adapter_layer)."""

    def __init__(self, ws: W.WeightSource, scale: np.ndarray, device="cuda",
                 adapter_rank: Optional[List[int]] = None, stream=None):
        w = ws.workload
        self.workload, self.ws, self.device = w, ws, device
        self.desc = L.PoolDesc(w.n_adapters, ws.n_layers, w.n_experts,
                               [(p.h_in, p.h_out) for p in w.projs], w.rank,
                               scale=[float(s) for s in scale], adapter_rank=adapter_rank)
        nbytes = L.lora_pool_bytes(self.desc)
        if nbytes == 0:
            raise ValueError("invalid pool description")
        self.slab = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.bank = to_dev(ws.bank, device)
        self.pool = L.lora_register_pool(self.desc, self.slab, stream=stream)
        base = self.bank.data_ptr()
        for layer in range(ws.n_layers):
            for a in range(w.n_adapters):
                L.lora_pool_load_adapter_layer(self.pool, a, layer,
                                               base + 2 * int(ws.window[a, layer]), stream=stream)
        torch.cuda.synchronize()

    @property
    def nbytes(self) -> int:
        return self.slab.numel()


class DeviceBatch:
    """One batch's ids, activations and base outputs on the device."""

    def __init__(self, b: W.Batch, device="cuda"):
        self.batch = b
        w = b.workload
        self.P = b.adapter_id.shape[0]
        self.adapter_id = to_dev(b.adapter_id, device)
        self.expert_id = None if b.expert_id is None else to_dev(b.expert_id, device)
        self.token_of_pair = to_dev(b.token_of_pair, device)
        self.inputs: Dict[str, torch.Tensor] = {k: to_dev(v, device) for k, v in b.inputs.items()}
        self.y: Dict[str, torch.Tensor] = {k: to_dev(v, device) for k, v in b.y_in.items()}
        self.seg = L.Segments(self.P, device)

    def reset_y(self):
        for k, v in self.batch.y_in.items():
            self.y[k].copy_(to_dev(v, self.y[k].device))


def projection_groups(w: W.Workload):
    """Runs of consecutive projections that read the same input (q/k/v, gate/up): (first, count),
    at most three per group."""
    groups, j = [], 0
    while j < len(w.projs):
        n = 1
        while (j + n < len(w.projs) and n < 3 and w.projs[j + n].input == w.projs[j].input
               and w.projs[j + n].h_in == w.projs[j].h_in):
            n += 1
        groups.append((j, n))
        j += n
    return groups


class LayerRunner:
    """Issues the calls of one layer over a DeviceBatch: build segments, then per projection
    lora_apply_group per run of projections sharing an input (dense) or the two MoE applications."""

    def __init__(self, dp: DevicePool, db: DeviceBatch):
        self.dp, self.db = dp, db
        w = dp.workload
        P = db.P
        self.moe = w.kind == "moe"
        if self.moe:
            self.ws = torch.empty(max(L.lora_moe_ws_bytes(dp.pool, P), 256), dtype=torch.uint8,
                                  device=dp.device)
        else:
            self.groups = projection_groups(w)
            n = max(max(L.lora_group_ws_bytes(dp.pool, j, c, P) for j, c in self.groups),
                    max(L.lora_v_bytes(dp.pool, j, P) for j in range(len(w.projs))))
            self.v = torch.empty(max(n, 256) // 4, dtype=torch.float32, device=dp.device)

    def build_segments(self, stream=None):
        db = self.db
        L.lora_build_segments(self.dp.pool, db.adapter_id, db.expert_id, db.P, db.seg, stream=stream)

    def apply(self, layer: int, stream=None):
        dp, db = self.dp, self.db
        w = dp.workload
        if self.moe:
            x, mid = db.inputs["x"], db.inputs["mid"]
            L.lora_moe_apply(dp.pool, layer, L.LORA_MOE_UPGATE, x, x.shape[1], db.token_of_pair,
                             db.seg, db.y["gate"], db.y["up"], db.y["gate"].shape[1], self.ws,
                             stream=stream)
            L.lora_moe_apply(dp.pool, layer, L.LORA_MOE_DOWN, mid, mid.shape[1], None, db.seg,
                             db.y["down"], None, db.y["down"].shape[1], self.ws, stream=stream)
        else:
            for j, c in self.groups:
                self.apply_group(layer, j, c, stream)

    def apply_group(self, layer: int, j: int, c: int, stream=None):
        dp, db = self.dp, self.db
        projs = dp.workload.projs[j:j + c]
        x = db.inputs[projs[0].input]
        ys = [db.y[p.name] for p in projs]
        L.lora_apply_group(dp.pool, layer, j, x, x.shape[1], None, db.seg, ys,
                           [y.shape[1] for y in ys], self.v, L.LORA_DTYPE_BF16, stream=stream)

    def step(self, layer: int, stream=None, one_call: bool = True):
        """One layer call.  one_call: the segment build and the first application go through
        lora_moe_build_apply / lora_build_apply_group (the library decides whether the first shrink
        sorts the batch itself); otherwise lora_build_segments and the applications one by one."""
        if not one_call:
            self.build_segments(stream)
            self.apply(layer, stream)
            return
        dp, db = self.dp, self.db
        if self.moe:
            x, mid = db.inputs["x"], db.inputs["mid"]
            L.lora_moe_build_apply(dp.pool, layer, L.LORA_MOE_UPGATE, x, x.shape[1], db.token_of_pair,
                                   db.adapter_id, db.expert_id, db.P, db.seg, db.y["gate"], db.y["up"],
                                   db.y["gate"].shape[1], self.ws, stream=stream)
            L.lora_moe_apply(dp.pool, layer, L.LORA_MOE_DOWN, mid, mid.shape[1], None, db.seg,
                             db.y["down"], None, db.y["down"].shape[1], self.ws, stream=stream)
        else:
            for i, (j, c) in enumerate(self.groups):
                if i:
                    self.apply_group(layer, j, c, stream)
                    continue
                projs = dp.workload.projs[j:j + c]
                x = db.inputs[projs[0].input]
                ys = [db.y[p.name] for p in projs]
                L.lora_build_apply_group(dp.pool, layer, j, x, x.shape[1], None, db.adapter_id, db.expert_id,
                                         db.P, db.seg, ys, [y.shape[1] for y in ys], self.v,
                                         L.LORA_DTYPE_BF16, stream=stream)
