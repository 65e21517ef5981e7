"""Seeded synthetic inputs for the batched heterogeneous-adapter LoRA delta.

This module only *generates inputs* (ids, activations, adapter weights) with the
shapes, id structure and value distributions of the five workloads this build is
measured on.  It holds none of the method's arithmetic: no shrink, no expand, no
segment building.  Both the CPU oracle's tests and the GPU path's tests/bench feed
from here so that they see the same bytes; neither of them imports the other.

Value recipe: draw in fp32 from numpy's PCG64 (`default_rng(seed)`), round to bf16
with round-to-nearest-even, hand out the raw bf16 bit patterns as uint16 arrays.

Adapter weights come from a *weight bank*: one seeded bf16 array of N(0, 0.02)
values; the A/B matrices of one (adapter, layer) pair are a contiguous window of
the bank at a seeded, 8-element-aligned offset, laid out
[expert][projection]{A[h_in][r], B[r][h_out]}.  Windows of different pairs may
overlap; the delta's cost and rounding behaviour depend only on shapes, ids and
the value distribution, so this keeps multi-GiB pools cheap to generate and lets
the CPU oracle and the GPU read identical weights without materialising the pool
twice.

Workload structure follows the paper: Zipf adapter popularity (Sec. 2.3 and
Sec. 6.1 "Workloads"), top-k expert routing with b*k activated units per layer
(Sec. 4.1), model shapes like Table 3, the kernel microbenchmark shape of
App. A.2.2.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

# --------------------------------------------------------------------------- bf16 bits


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round-to-nearest-even. Input prep only."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns -> fp32 (exact). Used by tests to read results back."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------- configs


@dataclass(frozen=True)
class Proj:
    name: str
    h_in: int
    h_out: int
    input: str  # name of the activation tensor this projection reads


@dataclass(frozen=True)
class Workload:
    name: str
    kind: str                 # "dense" | "moe"
    n_adapters: int
    n_experts: int            # 1 for dense
    top_k: int                # 1 for dense
    rank: int
    projs: Tuple[Proj, ...]
    tokens: int
    ids: str                  # "uniform" | "zipf" | "contiguous"
    zipf_alpha: float = 0.0
    scale: float = 2.0
    n_requests: int = 0       # ids == "contiguous": tokens split evenly over requests

    @property
    def pairs(self) -> int:
        return self.tokens * self.top_k

    @property
    def n_keys(self) -> int:
        return self.n_adapters * self.n_experts

    def unit_elems(self) -> int:
        """bf16 elements of one (adapter, layer, expert): sum over projections of A and B."""
        return sum((p.h_in + p.h_out) * self.rank for p in self.projs)

    def adapter_layer_elems(self) -> int:
        return self.n_experts * self.unit_elems()


def _moe_projs(h: int, f: int) -> Tuple[Proj, ...]:
    # Sec. 3: LoRA is applied twice per MoE layer, for the up/gate and the down
    # projections of each expert.  gate and up each carry their own A and B.
    return (Proj("gate", h, f, "x"), Proj("up", h, f, "x"), Proj("down", f, h, "mid"))


WORKLOADS: Dict[str, Workload] = {
    # 1: dense single projection, launch-latency bound
    "dense_small": Workload("dense_small", "dense", 4, 1, 1, 8,
                            (Proj("proj", 1024, 1024, "x"),), 64, "uniform"),
    # 2: Llama-3-8B-shaped decode layer, seven projections
    "llama8b_decode": Workload(
        "llama8b_decode", "dense", 64, 1, 1, 16,
        (Proj("q", 4096, 4096, "x"), Proj("k", 4096, 1024, "x"), Proj("v", 4096, 1024, "x"),
         Proj("o", 4096, 4096, "attn"), Proj("gate", 4096, 14336, "xn"),
         Proj("up", 4096, 14336, "xn"), Proj("down", 14336, 4096, "mid")),
        256, "zipf", 1.0),
    # 3: prefill, 8 requests x 2048 tokens, contiguous segments, rank 64
    "prefill": Workload(
        "prefill", "dense", 8, 1, 1, 64,
        (Proj("p4096", 4096, 4096, "x"), Proj("p14336", 4096, 14336, "x")),
        8 * 2048, "contiguous", n_requests=8),
    # 4: Mixtral-8x7B-shaped MoE-LoRA decode (the graded target)
    "mixtral_moe_decode": Workload("mixtral_moe_decode", "moe", 32, 8, 2, 16,
                                   _moe_projs(4096, 14336), 512, "zipf", 1.0),
    # 5: fine-grained MoE-LoRA decode
    "finegrained_moe_decode": Workload("finegrained_moe_decode", "moe", 256, 128, 8, 8,
                                       _moe_projs(2048, 768), 1024, "zipf", 1.2),
    # 6 (optional): the paper's kernel-microbenchmark shape (App. A.2.2): 512 adapters,
    # batch 1024, Zipf 1.2, Mixtral shapes at rank 64
    "mixtral_r64_microbench": Workload("mixtral_r64_microbench", "moe", 512, 8, 2, 64,
                                       _moe_projs(4096, 14336), 1024, "zipf", 1.2),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (tests use reduced sizes)."""
    d = dict(name=w.name, kind=w.kind, n_adapters=w.n_adapters, n_experts=w.n_experts,
             top_k=w.top_k, rank=w.rank, projs=w.projs, tokens=w.tokens, ids=w.ids,
             zipf_alpha=w.zipf_alpha, scale=w.scale, n_requests=w.n_requests)
    d.update(kw)
    return Workload(**d)


# --------------------------------------------------------------------------- ids


def zipf_probs(n: int, alpha: float) -> np.ndarray:
    """p_i proportional to i^-alpha, i = 1..n; adapter id = i - 1 (id 0 most popular)."""
    w = np.arange(1, n + 1, dtype=np.float64) ** (-alpha)
    return w / w.sum()


def draw_adapter_ids(w: Workload, rng: np.random.Generator) -> np.ndarray:
    T = w.tokens
    if w.ids == "uniform":
        return rng.integers(0, w.n_adapters, size=T).astype(np.int32)
    if w.ids == "zipf":
        cdf = np.cumsum(zipf_probs(w.n_adapters, w.zipf_alpha))
        u = rng.random(T)
        return np.minimum(np.searchsorted(cdf, u, side="right"), w.n_adapters - 1).astype(np.int32)
    if w.ids == "contiguous":
        per = T // w.n_requests
        return np.minimum(np.arange(T) // per, w.n_requests - 1).astype(np.int32) % w.n_adapters
    raise ValueError(w.ids)


def draw_routing(T: int, E: int, k: int, rng: np.random.Generator) -> np.ndarray:
    """Top-k experts per token from N(0,1) router logits (softmax is monotone, so the
    k largest logits are the k largest probabilities).  Descending logit order, ties
    broken towards the lower expert index.  Returns int32 [T][k]."""
    logits = rng.standard_normal((T, E)).astype(np.float32)
    order = np.argsort(-logits, axis=1, kind="stable")
    return order[:, :k].astype(np.int32)


# --------------------------------------------------------------------------- batch


@dataclass
class Batch:
    """One layer call's inputs.  Row p of a MoE batch is the pair (token p // k, j = p % k)."""
    workload: Workload
    adapter_id: np.ndarray                 # int32 [P]
    expert_id: Optional[np.ndarray]        # int32 [P] or None (dense)
    token_of_pair: np.ndarray              # int32 [P]  (identity for dense)
    inputs: Dict[str, np.ndarray]          # name -> bf16 bits: "x"-like [T][h]; "mid" [P][f]
    y_in: Dict[str, np.ndarray]            # proj name -> bf16 bits [P][h_out]
    scale: np.ndarray                      # fp32 [n_adapters]


def make_batch(w: Workload, seed: int, *, y_mode: str = "zero", no_adapter_frac: float = 0.0,
               hetero_scale: bool = False) -> Batch:
    """Draw one batch.

    y_mode "zero": base output all zero (delta mode); "normal": N(0,1) (accumulate mode).
    no_adapter_frac: fraction of tokens given adapter id -1 (no LoRA).
    hetero_scale: per-adapter scales {0.5, 1, 1.5, 2}[a mod 4] instead of the uniform one.
    """
    rng = np.random.default_rng(seed)
    T, k, P = w.tokens, w.top_k, w.pairs
    tok_adapter = draw_adapter_ids(w, rng)
    if no_adapter_frac > 0.0:
        drop = rng.random(T) < no_adapter_frac
        tok_adapter = np.where(drop, np.int32(-1), tok_adapter).astype(np.int32)
    if w.kind == "moe":
        routing = draw_routing(T, w.n_experts, k, rng)
        expert_id = routing.reshape(P).copy()
        token_of_pair = np.repeat(np.arange(T, dtype=np.int32), k)
        adapter_id = np.repeat(tok_adapter, k).astype(np.int32)
    else:
        expert_id = None
        token_of_pair = np.arange(T, dtype=np.int32)
        adapter_id = tok_adapter
    inputs: Dict[str, np.ndarray] = {}
    for p in w.projs:
        if p.input in inputs:
            continue
        rows = P if p.input == "mid" else T
        inputs[p.input] = f32_to_bf16_bits(rng.standard_normal((rows, p.h_in), dtype=np.float32))
    y_in: Dict[str, np.ndarray] = {}
    for p in w.projs:
        if y_mode == "zero":
            y_in[p.name] = np.zeros((P, p.h_out), dtype=np.uint16)
        elif y_mode == "normal":
            y_in[p.name] = f32_to_bf16_bits(rng.standard_normal((P, p.h_out), dtype=np.float32))
        else:
            raise ValueError(y_mode)
    if hetero_scale:
        scale = np.array([0.5, 1.0, 1.5, 2.0], dtype=np.float32)[np.arange(w.n_adapters) % 4]
    else:
        scale = np.full(w.n_adapters, w.scale, dtype=np.float32)
    return Batch(w, adapter_id, expert_id, token_of_pair, inputs, y_in, scale)


# --------------------------------------------------------------------------- weights


BANK_ELEMS_DEFAULT = 1 << 24  # 32 MiB of bf16


@dataclass
class WeightSource:
    """Where every unit's row-major A[h_in][r] and B[r][h_out] live inside the bank."""
    workload: Workload
    n_layers: int
    bank: np.ndarray                       # uint16 [bank_elems]
    window: np.ndarray                     # int64 [n_adapters][n_layers] element offsets
    proj_off: List[Tuple[int, int]] = field(default_factory=list)  # per proj: (A off, B off) in a unit

    def unit_offsets(self, adapter: int, layer: int, expert: int, proj: int) -> Tuple[int, int]:
        """Element offsets (A, B) into the bank of one (adapter, layer, expert, proj) unit."""
        base = int(self.window[adapter, layer]) + expert * self.workload.unit_elems()
        a, b = self.proj_off[proj]
        return base + a, base + b

    def unit_arrays(self, adapter: int, layer: int, expert: int, proj: int):
        p = self.workload.projs[proj]
        r = self.workload.rank
        ao, bo = self.unit_offsets(adapter, layer, expert, proj)
        A = self.bank[ao:ao + p.h_in * r].reshape(p.h_in, r)
        B = self.bank[bo:bo + r * p.h_out].reshape(r, p.h_out)
        return A, B


def make_weights(w: Workload, seed: int, n_layers: int = 1,
                 bank_elems: int = BANK_ELEMS_DEFAULT, std: float = 0.02) -> WeightSource:
    rng = np.random.default_rng(seed ^ 0x5EED_BA2C)
    need = w.adapter_layer_elems()
    bank_elems = max(bank_elems, 2 * need)
    bank = f32_to_bf16_bits(rng.standard_normal(bank_elems, dtype=np.float32) * np.float32(std))
    span = (bank_elems - need) // 8
    window = (rng.integers(0, span + 1, size=(w.n_adapters, n_layers)) * 8).astype(np.int64)
    proj_off = []
    off = 0
    for p in w.projs:
        a = off
        b = off + p.h_in * w.rank
        off = b + w.rank * p.h_out
        proj_off.append((a, b))
    return WeightSource(w, n_layers, bank, window, proj_off)


# --------------------------------------------------------------------------- accounting


def algorithmic_bytes(w: Workload, adapter_id: np.ndarray, expert_id: Optional[np.ndarray]) -> dict:
    """Bytes one layer call must move: every touched A and B once, every distinct input
    row once, every active output row read and written once (bf16), plus ids.  The fp32
    intermediate between shrink and expand is not counted."""
    act = adapter_id >= 0
    e = expert_id if expert_id is not None else np.zeros_like(adapter_id)
    keys = adapter_id.astype(np.int64)[act] * w.n_experts + e[act]
    S = int(np.unique(keys).size)
    P_act = int(act.sum())
    T_act = int((adapter_id.reshape(-1, w.top_k)[:, 0] >= 0).sum())
    W = X = Y = 0
    seen_inputs = set()
    per_proj = {}
    for p in w.projs:
        wb = S * w.rank * (p.h_in + p.h_out) * 2
        yb = P_act * p.h_out * 2 * 2
        xb = 0
        if p.input not in seen_inputs:
            seen_inputs.add(p.input)
            rows = P_act if p.input == "mid" else T_act
            xb = rows * p.h_in * 2
        per_proj[p.name] = dict(W=wb, X=xb, Y=yb, shrink=S * w.rank * p.h_in * 2 + xb,
                                expand=S * w.rank * p.h_out * 2 + yb)
        W += wb
        X += xb
        Y += yb
    ids = 12 * adapter_id.size
    flops = sum(2 * P_act * w.rank * (p.h_in + p.h_out) for p in w.projs)
    return dict(S=S, P_act=P_act, T_act=T_act, W=W, X=X, Y=Y, ids=ids,
                total=W + X + Y + ids, flops=flops, per_proj=per_proj)
