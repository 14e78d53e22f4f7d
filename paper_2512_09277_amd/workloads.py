"""Seeded synthetic inputs for the METRO hot path (routing + decode expert FFN).

This module only *draws inputs*: expert popularity, a replica placement, top-k
traces, gating weights, activations and expert weights.  It contains none of
the method's arithmetic (no routing decision, no permutation, no FFN), so both
the CPU oracle's tests and the HIP path's tests may feed from it and see the
same byte buffers.

The paper measures on router traces of Qwen3-30B/235B and DeepSeek-V3 (Sec. 6.1,
"Workloads and traces").  Those traces are not available; Zipf-skewed synthetic
traces with the same shapes (experts, top-k, EP ranks, decode batch, replication
ratio 1.125x; Sec. 6.1 and Table 2) stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional, Tuple

import numpy as np

BASE_SEED = 0x9277


@dataclass(frozen=True)
class Workload:
    """One synthetic decode-layer shape.

    N experts, top-k, G logical EP ranks, spr replica slots per rank
    (S = G*spr slots, R = S - N redundant replicas), T tokens in the global
    decode batch, Zipf exponent s, FFN hidden H / inter I, element dtype of
    activations and weights ("bf16" or "f32"), number of independent layers.
    """

    name: str
    index: int
    N: int
    k: int
    G: int
    spr: int
    T: int
    s: float
    H: int = 0
    I: int = 0
    dtype: str = "bf16"
    layers: int = 1
    replication: str = "greedy"  # "greedy": popularity-greedy; "top": +1 to each of the R most popular

    @property
    def S(self) -> int:
        return self.G * self.spr

    @property
    def R(self) -> int:
        return self.S - self.N

    def seed(self, layer: int = 0, stream: int = 0) -> int:
        return BASE_SEED + 1000 * self.index + layer + 100003 * stream

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


TINY = Workload("tiny", 1, N=16, k=2, G=4, spr=5, T=32, s=1.0, H=256, I=128, dtype="f32", replication="top")
QWEN3_30B = Workload("qwen3_30b_a3b_decode", 2, N=128, k=8, G=8, spr=18, T=256, s=0.8, H=2048, I=768)
QWEN3_235B = Workload("qwen3_235b_a22b_decode", 3, N=128, k=8, G=8, spr=18, T=512, s=1.0, H=4096, I=1536)
DSV3 = Workload("deepseek_v3_decode", 4, N=256, k=8, G=8, spr=36, T=1024, s=1.0, H=7168, I=2048)
DSV3_SWEEP = Workload("deepseek_v3_routing_sweep", 5, N=256, k=8, G=16, spr=18, T=1024, s=1.0, layers=58)
SWEEP_T = (64, 256, 1024, 4096)
SWEEP_S = (0.6, 1.0, 1.4)

WORKLOADS = {w.name: w for w in (TINY, QWEN3_30B, QWEN3_235B, DSV3, DSV3_SWEEP)}


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(seed))


# --------------------------------------------------------------------------- bf16 bit helpers
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even), returned as uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns (uint16) to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------- routing inputs
def popularity(N: int, s: float, seed: int) -> np.ndarray:
    """Zipf popularity over a seeded permutation of expert ids: p_e ~ 1/(pi(e)+1)^s, float64, sums to 1."""
    pi = _rng(seed).permutation(N)
    p = 1.0 / np.power(pi.astype(np.float64) + 1.0, s)
    return p / p.sum()


def replica_counts(p: np.ndarray, G: int, R: int, mode: str = "greedy") -> np.ndarray:
    """Replica count per expert (>=1 each).  "greedy": R times, one more replica to
    argmax p_e/r_e among experts with r_e < G (ties -> lowest id).  "top": one
    extra replica for each of the R most popular experts."""
    N = p.shape[0]
    r = np.ones(N, dtype=np.int64)
    if mode == "top":
        order = np.lexsort((np.arange(N), -p))
        r[order[:R]] += 1
        return r
    for _ in range(R):
        score = np.where(r < G, p / r, -1.0)
        r[int(np.argmax(score))] += 1
    return r


def placement(p: np.ndarray, G: int, spr: int, mode: str = "greedy") -> np.ndarray:
    """slot_to_expert[S] (int32): slot s lives on rank s // spr.

    Stand-in for EPLB replication + placement (Sec. 2.3): replicas sorted by expected
    per-replica load p_e/r_e (desc, expert id asc), each placed on the rank with the
    least accumulated load among ranks that have a free slot and do not already host
    that expert (ties -> lowest rank); slot index on a rank = arrival order.
    """
    N = p.shape[0]
    S = G * spr
    R = S - N
    if R < 0:
        raise ValueError("fewer slots than experts")
    r = replica_counts(p, G, R, mode)
    reps = [(-(p[e] / r[e]), e) for e in range(N) for _ in range(int(r[e]))]
    reps.sort()
    load = np.zeros(G, dtype=np.float64)
    fill = np.zeros(G, dtype=np.int64)
    hosts = [set() for _ in range(G)]
    s2e = np.full(S, -1, dtype=np.int32)
    for negw, e in reps:
        best = -1
        for g in range(G):
            if fill[g] >= spr or e in hosts[g]:
                continue
            if best < 0 or load[g] < load[best]:
                best = g
        if best < 0:  # only a rank already hosting e has room: allowed as a last resort
            best = int(np.argmin(np.where(fill < spr, load, np.inf)))
        s2e[best * spr + fill[best]] = e
        fill[best] += 1
        load[best] += -negw
        hosts[best].add(e)
    return s2e


def topk_trace(p: np.ndarray, T: int, k: int, seed: int) -> np.ndarray:
    """ids[T,k] int32: each token draws k distinct experts sequentially without
    replacement, proportionally to p (renormalised after every draw), stored in draw
    order.  Drawn with the exponential-race form of that process: order experts by
    E_e/p_e with E_e ~ Exp(1) and keep the first k."""
    N = p.shape[0]
    e = _rng(seed).exponential(size=(T, N))
    key = e / p[None, :]
    part = np.argpartition(key, k - 1, axis=1)[:, :k]
    sub = np.take_along_axis(key, part, axis=1)
    order = np.argsort(sub, axis=1, kind="stable")
    return np.take_along_axis(part, order, axis=1).astype(np.int32)


def gating_weights(T: int, k: int, seed: int) -> np.ndarray:
    """topk_w[T,k] float32: softmax over k i.i.d. N(0,1) logits."""
    z = _rng(seed).standard_normal((T, k))
    z = np.exp(z - z.max(axis=1, keepdims=True))
    return (z / z.sum(axis=1, keepdims=True)).astype(np.float32)


def routing_inputs(w: Workload, layer: int = 0, T: Optional[int] = None, s: Optional[float] = None
                   ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """(p[N], slot_to_expert[S], ids[T,k]) of one layer of a workload."""
    T = w.T if T is None else T
    s = w.s if s is None else s
    p = popularity(w.N, s, w.seed(layer, 0))
    s2e = placement(p, w.G, w.spr, w.replication)
    ids = topk_trace(p, T, w.k, w.seed(layer, 1) + 7 * T)
    return p, s2e, ids


def routing_inputs_layers(w: Workload, T: Optional[int] = None, s: Optional[float] = None
                          ) -> Tuple[np.ndarray, np.ndarray]:
    """(slot_to_expert[L,S], ids[L,T,k]) stacked over the workload's layers."""
    s2e, ids = [], []
    for layer in range(w.layers):
        _, a, b = routing_inputs(w, layer, T, s)
        s2e.append(a)
        ids.append(b)
    return np.stack(s2e), np.stack(ids)


# --------------------------------------------------------------------------- FFN inputs (host, small shapes)
def activations(T: int, H: int, seed: int, dtype: str) -> np.ndarray:
    """x[T,H] ~ N(0,1); float32 for "f32", uint16 bfloat16 bit patterns for "bf16"."""
    x = _rng(seed).standard_normal((T, H)).astype(np.float32)
    return x if dtype == "f32" else f32_to_bf16_bits(x)


def expert_weights(N: int, H: int, I: int, seed: int, dtype: str) -> Tuple[np.ndarray, np.ndarray]:
    """Per *logical* expert: w13[N,2I,H] (rows 0..I-1 gate, I..2I-1 up) and w2[N,H,I],
    all ~ N(0,0.02), K-contiguous.  Replicas of an expert are copies of these."""
    g = _rng(seed)
    w13 = (0.02 * g.standard_normal((N, 2 * I, H))).astype(np.float32)
    w2 = (0.02 * g.standard_normal((N, H, I))).astype(np.float32)
    if dtype == "f32":
        return w13, w2
    return f32_to_bf16_bits(w13), f32_to_bf16_bits(w2)


def gate_weights(N: int, H: int, seed: int, dtype: str) -> np.ndarray:
    """Router weights w_gate[N,H] ~ N(0, 1/H), so that logits of N(0,1) activations are ~ N(0,1);
    float32 for "f32", uint16 bfloat16 bit patterns for "bf16"."""
    wg = (_rng(seed).standard_normal((N, H)) / np.sqrt(H)).astype(np.float32)
    return wg if dtype == "f32" else f32_to_bf16_bits(wg)


def rank_share(w: np.ndarray, slot_to_expert: np.ndarray, g: int, spr: int) -> np.ndarray:
    """Weights of the spr slots of rank g, [spr, ...]; an empty slot (-1) holds zeros."""
    ex = slot_to_expert[g * spr:(g + 1) * spr]
    out = w[np.maximum(ex, 0)].copy()
    out[ex < 0] = 0
    return out


# --------------------------------------------------------------------------- FFN inputs (device, full shapes)
def device_expert_weights(w: Workload, device, layer: int = 0):
    """Logical-expert weights drawn on the device (torch bf16/f32 tensors) for the
    full-size shapes, where a host draw would take minutes: w13[N,2I,H], w2[N,H,I]
    ~ N(0,0.02).  The oracle is fed host copies of the same bytes."""
    import torch

    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    gen = torch.Generator(device=device)
    gen.manual_seed(w.seed(layer, 2))
    w13 = torch.empty((w.N, 2 * w.I, w.H), dtype=dt, device=device)
    w2 = torch.empty((w.N, w.H, w.I), dtype=dt, device=device)
    for e in range(w.N):  # per expert, so that the fp32 staging buffer stays small
        w13[e] = (0.02 * torch.randn((2 * w.I, w.H), generator=gen, device=device)).to(dt)
        w2[e] = (0.02 * torch.randn((w.H, w.I), generator=gen, device=device)).to(dt)
    return w13, w2


def device_activations(w: Workload, device, layer: int = 0, T: Optional[int] = None):
    import torch

    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    gen = torch.Generator(device=device)
    gen.manual_seed(w.seed(layer, 3))
    return torch.randn((w.T if T is None else T, w.H), generator=gen, device=device).to(dt)


def padded_pitch(K: int, elt_bytes: int = 2) -> int:
    """Row pitch in elements for weight rows of K elements: rows whose byte length is a multiple of
    4096 get 128 more elements, so that the rows one load instruction touches spread over the HBM
    channels instead of piling onto a few of them."""
    return K + 128 if (K * elt_bytes) % 4096 == 0 else K


def device_rank_share(wt, slot_to_expert: np.ndarray, g: int, spr: int, pad: bool = False):
    """Device copy of rank g's slots, [spr, rows, K]; empty slots hold zeros.  pad=True returns a view
    of a buffer whose rows are padded_pitch(K) elements apart (same values, different layout)."""
    import torch

    ex = torch.as_tensor(slot_to_expert[g * spr:(g + 1) * spr].astype(np.int64), device=wt.device)
    K = wt.shape[2]
    ld = padded_pitch(K, wt.element_size()) if pad else K
    buf = torch.zeros((spr, wt.shape[1], ld), dtype=wt.dtype, device=wt.device)
    out = buf[:, :, :K]
    out.copy_(wt.index_select(0, ex.clamp(min=0)))
    out[ex < 0] = 0
    return out
