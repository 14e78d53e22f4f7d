#!/usr/bin/env python3
"""Benchmark of the METRO hot path on one MI355X.

A step is one pass of the whole path over one synthetic decode batch, inputs resident in HBM:
    metro_route -> moe_permute (slowest rank) -> moe_grouped_ffn (gate/up, down) -> moe_unpermute.
The workload is the DeepSeek-V3-shaped decode layer (E=256, top-8, G=8 logical ranks, 36 slots per
rank, T=1024, Zipf s=1.0, H=7168, I=2048, bf16) -- the shape the HBM-roofline target is stated on.
"Slowest rank" = the rank whose expert FFN takes longest when measured (all G shares resident).

Prints ONE JSON line: `value` = achieved algorithmic HBM GB/s of the slowest rank's expert FFN under
METRO routing; the route latency, FFN times under both routers, the roofline of the dominant kernel
(gate/up) and the CPU-oracle baseline ride along in the same object.

METRO and token-balanced routing are compared inside one timed loop that alternates a METRO step and a
token-balanced step (each on its own slowest rank), so that clock and power drift hit both sides alike; the
same comparison at the two Qwen3-shaped configs rides along in `per_config`.

Every timed loop runs W warm-up steps and then exactly K timed steps; before that come 0.3 s of untimed steps, and
no device memory is handed back to the driver until the timed work is done (see `settle` and
`release_device_memory` for what each of these keeps out of the timed region).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
METRIC = "METRO route µs/batch; slowest-rank expert-FFN µs & HBM GB/s (decode)"


def algorithmic_bytes(active: int, P: int, H: int, I: int, elt: int = 2):
    """Bytes the method itself must move for one rank: every activated slot's weights once, the
    gathered activations, the intermediate act (written by gate/up, read by down) and y_perm."""
    gate_up = active * 2 * I * H * elt + P * H * elt + P * I * elt + 4 * P
    down = active * H * I * elt + P * I * elt + P * H * elt
    return gate_up, down


class HotPath:
    """Device buffers and the step function for one (routing, rank) choice."""

    def __init__(self, api, torch, w, d_ids, d_s2e, x, tw, shares, routing: str):
        self.api, self.torch, self.w = api, torch, w
        self.d_ids, self.d_s2e, self.x, self.tw, self.shares = d_ids, d_s2e, x, tw, shares
        self.route_fn = api.metro_route if routing == "metro" else api.metro_route_token_balanced
        self.fused_fn = api.metro_route_permute if routing == "metro" else api.metro_route_token_balanced_permute
        dev = x.device
        self.rb = api.route_buffers(1, w.T, w.k, w.N, w.G, dev)
        self.pb = api.permute_buffers(w.T, w.k, w.spr, dev)
        self.y = torch.empty((w.T * w.k, w.H), dtype=x.dtype, device=dev)
        self.out = torch.empty((w.T, w.H), dtype=x.dtype, device=dev)
        self.ws = torch.empty((api.moe_grouped_ffn_workspace_bytes(w.T, w.k, w.spr, w.H, w.I, x.dtype),),
                              dtype=torch.uint8, device=dev)
        self.copies = {}      # rank -> distinct copies of its weights, rotated so that no step finds them cached
        self.calls = 0

    def weights(self, g: int):
        """The rank's weights; shares smaller than ~1.5 GB are rotated over several copies at distinct
        addresses so that the working set stays well above the 256 MB Infinity Cache."""
        if g not in self.copies:
            w13, w2 = self.shares[g]
            nbytes = w13.numel() * w13.element_size() + w2.numel() * w2.element_size()
            n = max(1, -(-1536 * 2**20 // nbytes))
            def same_layout(t):
                c = self.torch.empty_strided(t.size(), t.stride(), dtype=t.dtype, device=t.device)
                c.copy_(t)
                return c

            self.copies[g] = [(w13, w2)] + [(same_layout(w13), same_layout(w2)) for _ in range(n - 1)]
        c = self.copies[g]
        self.calls += 1
        return c[self.calls % len(c)]

    STAGES = ["route", "permute", "gate_up", "down", "unpermute"]

    def step(self, g: int, marks=None, separate: bool = False):
        """One pass of the path.  marks: 6 events (or None entries) recorded at the stage boundaries.  The routing
        solve and the rank's token lists come from one launch (metro_route_permute); separate=True runs them as the
        two calls, so that each can be bracketed by events."""
        api, w = self.api, self.w
        m = (lambda i: marks[i] is not None and marks[i].record()) if marks is not None else (lambda i: None)
        m(0)
        if separate:
            self.route_fn(self.d_ids, self.d_s2e, w.N, w.G, w.spr, out=self.rb)
            m(1)
            api.moe_permute(self.rb["pair_slot"][0], g, w.spr, out=self.pb)
        else:
            self.fused_fn(self.d_ids, self.d_s2e, w.N, w.G, w.spr, g, out=self.rb, lists=self.pb)
        w13, w2 = self.weights(g)
        api.moe_grouped_ffn_stages(self.x, self.pb["perm_pair"], self.pb["group_offsets"], w.k, w13, w2, self.y,
                                   self.ws, between=lambda i: m(2 + i))
        api.moe_unpermute(self.y, self.pb["pair_row"], self.tw, out=self.out)
        m(5)

    def graph_ms_per_step(self, g: int, replays: int = 10) -> float:
        """The same step replayed from a HIP graph: what a serving loop that captures the layer would see; no
        events inside.  At least eight steps are captured per graph (a multiple of the weight copies, so the
        rotation is kept): one graph launch costs tens of microseconds that back-to-back eager launches hide,
        and a graph holding a single 0.7 ms step would charge all of it to that step."""
        torch = self.torch
        n = len(self.copies[g])
        n = n * max(1, -(-8 // n))
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        self.step(g)
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for _ in range(n):
                    self.step(g)
        torch.cuda.synchronize()
        for _ in range(1 + 200 // n):                    # ~0.15 s untimed: capture kept the GPU idle (see settle)
            graph.replay()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(replays):
            graph.replay()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / (n * replays)

    def ffn_only_us(self, g: int, iters: int = 5) -> float:
        """Median gate/up + down time of `iters` steps queued back to back after ten untimed ones (the search for the
        slowest rank).  The first handful of launches that touch a rank's weights for the first time run ~10 % slower
        (745 us, then 662-667 us on the DeepSeek-V3-shaped METRO rank), hence the ten."""
        torch = self.torch
        evs = [[None, None] + [torch.cuda.Event(enable_timing=True) for _ in range(3)] + [None] for _ in range(iters)]
        for _ in range(10):
            self.step(g)
        for ev in evs:
            self.step(g, ev)
        torch.cuda.synchronize()
        return 1e3 * float(np.median([ev[2].elapsed_time(ev[4]) for ev in evs]))

    def stage_breakdown(self, g: int, n: int = 20):
        """Mean duration of every stage from a pass that brackets each stage with events (not part of the
        timed steps: an event costs a few microseconds of stream time, which matters next to the short stages)."""
        torch = self.torch
        for _ in range(150):                             # ~0.1 s of steps: the clocks are back up after the host-side pause
            self.step(g)
        full = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(n)]
        for e in full:
            self.step(g, e, separate=True)
        fused = [[torch.cuda.Event(enable_timing=True), None, torch.cuda.Event(enable_timing=True), None, None, None]
                 for _ in range(n)]
        for e in fused:
            self.step(g, e)
        torch.cuda.synchronize()
        out = {name: 1e3 * float(np.mean([e[i].elapsed_time(e[i + 1]) for e in full]))
               for i, name in enumerate(self.STAGES)}
        out["route_and_permute_one_launch"] = 1e3 * float(np.mean([e[0].elapsed_time(e[2]) for e in fused]))
        return out


def interleaved(torch, sides, steps: int, warmup: int):
    """W untimed + K timed iterations; an iteration runs one step of every side in turn (METRO step, then
    token-balanced step), so whatever drifts during the run drifts for both.  One event separates consecutive
    steps and three bracket the two FFN kernels of each step.  Returns per side: ms per step (device time between
    its boundary events), wall-clock ms of the whole loop, and the per-step FFN stage times in us."""
    ev = lambda: torch.cuda.Event(enable_timing=True)
    for _ in range(warmup):
        for hp, g in sides:
            hp.step(g)
    n = len(sides)
    bound = [ev() for _ in range(steps * n + 1)]
    inner = [[(ev(), ev(), ev()) for _ in range(steps)] for _ in sides]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    bound[0].record()
    for s in range(steps):
        for i, (hp, g) in enumerate(sides):
            a, b, c = inner[i][s]
            hp.step(g, [None, None, a, b, c, bound[s * n + i + 1]])
    torch.cuda.synchronize()
    wall_ms = 1e3 * (time.perf_counter() - t0)
    out = []
    for i in range(n):
        step_ms = np.array([bound[s * n + i].elapsed_time(bound[s * n + i + 1]) for s in range(steps)])
        gu = np.array([1e3 * a.elapsed_time(b) for a, b, _ in inner[i]])
        dn = np.array([1e3 * b.elapsed_time(c) for _, b, c in inner[i]])
        out.append(dict(ms_per_step=float(step_ms.mean()), gate_up_us=gu, down_us=dn))
    dev_ms = bound[0].elapsed_time(bound[-1])
    # the driver's clock sees the whole loop: never report a step shorter than its share of the wall clock
    scale = max(1.0, wall_ms / dev_ms)
    for o in out:
        o["ms_per_step"] *= scale
    return out, wall_ms


def settle(torch, sides, seconds: float = 0.3):
    """Untimed steps for `seconds` before a timed loop, on top of the W warm-up steps: the set-up before it (weight
    gathers, the per-rank search with a host sync per call) leaves the first ~0.1 s of back-to-back steps 1-2 % slower
    than the rest (gate/up 425 us, then 416 us for as long as the loop runs), and a short K would time only those."""
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(10):
            for hp, g in sides:
                hp.step(g)
        torch.cuda.synchronize()


def graph_replay_us(torch, launch, reps: int = 20, replays: int = 10) -> float:
    """Kernel-only latency of `launch()`: `reps` launches captured into one HIP graph (no memsets, no
    events inside), mean over `replays` replays."""
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    launch()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            for _ in range(reps):
                launch()
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(replays):
        graph.replay()
    b.record()
    torch.cuda.synchronize()
    return 1e3 * a.elapsed_time(b) / (reps * replays)


def routing_sweep(api, torch, W, quick: bool):
    """Routing-only latency and max activated experts per rank at the sweep shape (G=16, 58 layers,
    each with its own popularity permutation): T x Zipf s grid, METRO vs token-balanced.  Per cell:
    us per batch with all 58 layers in one launch, us of a single-layer launch (events around 50
    back-to-back launches), the same inside a HIP graph replay (kernel only), mean max-activated."""
    w = W.DSV3_SWEEP
    rows = []
    cells = [(1024, 1.0)] if quick else [(T, s) for T in W.SWEEP_T for s in W.SWEEP_S]
    for T, s in cells:
        s2e, ids = W.routing_inputs_layers(w, T=T, s=s)
        d_ids, d_s2e = torch.from_numpy(ids).cuda(), torch.from_numpy(s2e).cuda()
        ref = {}
        for name, fn in (("metro", api.metro_route), ("token_balanced", api.metro_route_token_balanced)):
            buf = api.route_buffers(w.layers, T, w.k, w.N, w.G, "cuda")
            one = api.route_buffers(1, T, w.k, w.N, w.G, "cuda")
            for _ in range(5):
                fn(d_ids, d_s2e, w.N, w.G, w.spr, out=buf)
                fn(d_ids[:1], d_s2e[:1], w.N, w.G, w.spr, out=one)
            a, b, c = (torch.cuda.Event(enable_timing=True) for _ in range(3))
            n = 50
            torch.cuda.synchronize()
            a.record()
            for _ in range(n):
                fn(d_ids, d_s2e, w.N, w.G, w.spr, out=buf)
            b.record()
            for _ in range(n):
                fn(d_ids[:1], d_s2e[:1], w.N, w.G, w.spr, out=one)
            c.record()
            torch.cuda.synchronize()
            assert int(buf["err_flag"].abs().sum().item()) == 0
            ref[name] = dict(us_per_batch_58_layers_per_launch=round(1e3 * a.elapsed_time(b) / n / w.layers, 3),
                             us_per_single_layer_launch=round(1e3 * b.elapsed_time(c) / n, 3),
                             us_single_layer_graph_replay=round(graph_replay_us(
                                 torch, lambda: fn(d_ids[:1], d_s2e[:1], w.N, w.G, w.spr, out=one)), 3),
                             max_activated_per_rank_mean=round(float(buf["rank_active"].max(dim=1).values.float().mean()), 3))
        rows.append(dict(T=T, s=s, **ref))
    return rows


def gate_topk_timing(api, torch, W, w, x):
    """Router gate + top-k at the workload's shape (the step before the path; not part of a step)."""
    wg = torch.from_numpy(W.gate_weights(w.N, w.H, w.seed(0, 5), "bf16")).view(torch.bfloat16).cuda()
    out = api.moe_gate_topk(x, wg, w.k)
    ws = torch.empty((api.load().moe_gate_topk_workspace_bytes(w.T, w.H, w.N, api.DTYPE_BF16),), dtype=torch.uint8,
                     device="cuda")
    run = lambda: api.moe_gate_topk(x, wg, w.k, out=out, ws=ws)
    for _ in range(5):
        run()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n = 50
    torch.cuda.synchronize()
    a.record()
    for _ in range(n):
        run()
    b.record()
    torch.cuda.synchronize()
    flop = 2.0 * w.T * w.H * w.N
    us = 1e3 * a.elapsed_time(b) / n
    return dict(us_per_call=round(us, 2), us_graph_replay=round(graph_replay_us(torch, run), 2),
                tflops=round(flop / us / 1e6, 1), operand_mb=round((w.T + w.N) * w.H * 2 / 1e6, 1))


def fp32_path_timing(api, torch, W):
    """The fp32 / odd-shape FFN path (LDS-tiled vector-ALU kernels, 1e-5 parity): expert FFN time of the busiest
    METRO rank at the Tiny config and at the Qwen3-30B-shaped layer stored in fp32."""
    out = {}
    for w in (W.TINY, W.QWEN3_30B.with_(dtype="f32")):
        _, s2e, ids = W.routing_inputs(w)
        rb = api.metro_route(torch.from_numpy(ids).cuda(), torch.from_numpy(s2e).cuda(), w.N, w.G, w.spr)
        ps = rb["pair_slot"][0]
        g = int(torch.bincount((ps[ps >= 0] // w.spr).reshape(-1), minlength=w.G).argmax().item())
        lw13, lw2 = W.device_expert_weights(w, "cuda")
        w13, w2 = W.device_rank_share(lw13, s2e, g, w.spr), W.device_rank_share(lw2, s2e, g, w.spr)
        del lw13, lw2
        x = W.device_activations(w, "cuda")
        pm = api.moe_permute(ps, g, w.spr)
        y = torch.empty((w.T * w.k, w.H), dtype=torch.float32, device="cuda")
        ws = torch.empty((api.moe_grouped_ffn_workspace_bytes(w.T, w.k, w.spr, w.H, w.I, torch.float32),), dtype=torch.uint8,
                         device="cuda")
        run = lambda: api.moe_grouped_ffn(x, pm["perm_pair"], pm["group_offsets"], w.k, w13, w2, y_perm=y, ws=ws)
        for _ in range(5):
            run()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        n = 30
        torch.cuda.synchronize()
        a.record()
        for _ in range(n):
            run()
        b.record()
        torch.cuda.synchronize()
        us = 1e3 * a.elapsed_time(b) / n
        sizes = torch.diff(pm["group_offsets"]).cpu().numpy()
        active, P = int((sizes > 0).sum()), int(sizes.sum())
        gu, dn = algorithmic_bytes(active, P, w.H, w.I, elt=4)
        out[w.name] = dict(dtype="f32", H=w.H, I=w.I, rank=g, activated=active, pairs=P, ffn_us=round(us, 1),
                           algorithmic_gbs=round((gu + dn) / us / 1e3, 1))
    return out


def routing_quality(oracle, W, sweep_rows):
    """Sec. 4.2's exact solver (binary search on lambda + bipartite matching, the oracle's CPU code) on the
    same sweep cells: mean optimal lambda next to the measured METRO / token-balanced means, METRO's gap,
    and the solver's CPU time per batch."""
    w = W.DSV3_SWEEP
    out = []
    for row in sweep_rows:
        s2e, ids = W.routing_inputs_layers(w, T=row["T"], s=row["s"])
        cnts = [oracle.count(ids[l], w.N) for l in range(w.layers)]
        t0 = time.perf_counter()
        opt = [oracle.matching_opt(cnts[l], s2e[l], w.N, w.G, w.spr) for l in range(w.layers)]
        us = 1e6 * (time.perf_counter() - t0) / w.layers
        lam_opt, lam_me = float(np.mean(opt)), row["metro"]["max_activated_per_rank_mean"]
        out.append(dict(T=row["T"], s=row["s"], lambda_opt_mean=round(lam_opt, 3), lambda_metro_mean=lam_me,
                        lambda_token_balanced_mean=row["token_balanced"]["max_activated_per_rank_mean"],
                        metro_gap_pct=round(100.0 * (lam_me / lam_opt - 1.0), 2),
                        exact_solver_us_per_batch_cpu=round(us, 1)))
    return out


def cpu_baseline(oracle, W, w, ids, s2e, host_x, host_w13, host_w2, perm, ffn_bytes, budget_s: float):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample."""
    t0 = time.perf_counter()
    n_route = 0
    while time.perf_counter() - t0 < 1.0:
        oracle.route_metro(ids, s2e, w.N, w.G, w.spr)
        n_route += 1
    route_us = 1e6 * (time.perf_counter() - t0) / n_route
    P = perm["n_pairs"]
    threads = oracle.num_threads()
    rng = np.random.default_rng(0)
    probe = np.sort(rng.choice(P, size=min(P, threads), replace=False))
    t0 = time.perf_counter()
    oracle.ffn(host_x, perm["perm_pair"], perm["group_offsets"], w.k, host_w13, host_w2, rows=probe)
    per_batch = time.perf_counter() - t0
    n = int(min(P, max(threads, threads * int(budget_s / max(per_batch, 1e-3)))))
    rows = np.sort(rng.choice(P, size=n, replace=False))
    t0 = time.perf_counter()
    oracle.ffn(host_x, perm["perm_pair"], perm["group_offsets"], w.k, host_w13, host_w2, rows=rows)
    dt = time.perf_counter() - t0
    full_s = dt * P / n
    return dict(value=round(ffn_bytes / full_s / 1e9, 4), unit="GB/s", cores=threads, kind="oracle",
                sample=f"{n} of the slowest rank's {P} rows (all columns) in {dt:.1f} s, scaled to {P} rows; "
                       f"routing oracle: 1 core, {n_route} batches",
                ffn_us_extrapolated=round(1e6 * full_s, 1), route_us_per_batch=round(route_us, 2))


def release_device_memory(torch):
    """Hands the allocator's cached blocks back to the driver, then waits until the driver is done with them.
    The driver clears released device memory in the background, and while it does the FFN kernels lose about
    5 % of their bandwidth (gate/up of the DeepSeek-V3-shaped METRO rank: 440 us during the 1.5 s after 45 GB
    were released, 416 us from then on; 0.6 s after 22 GB).  Timed regions therefore never follow a release
    directly: either nothing is released before them (the cache is kept), or this wait comes first."""
    before = torch.cuda.memory_reserved()
    torch.cuda.empty_cache()
    freed = before - torch.cuda.memory_reserved()
    torch.cuda.synchronize()
    if freed > 0:
        time.sleep(0.5 + freed / 15e9)


def quantiles(v):
    return [round(float(np.percentile(v, q)), 1) for q in (10, 50, 90)]


def compare_routings(api, torch, W, w, steps: int, warmup: int, routings=("metro", "token_balanced"), lw=None,
                     ranks=None, pad: bool = True, stages: bool = False, alone_first: bool = False):
    """One workload under the given routings: each side's slowest rank is found with all G shares resident, then
    the sides are timed in one interleaved loop.  alone_first: before that, the first side runs its own W + K
    steps back to back (the benchmark's timed region: K steps of the hot path and nothing else); its figures
    land under "alone" in that side's result.  Returns {routing: result dict} and the objects the caller may still
    need (inputs, the sides' HotPath objects)."""
    _, s2e, ids = W.routing_inputs(w)
    d_ids = torch.from_numpy(ids).cuda().unsqueeze(0)
    d_s2e = torch.from_numpy(s2e).cuda().unsqueeze(0)
    x = W.device_activations(w, "cuda")
    tw = torch.from_numpy(W.gating_weights(w.T, w.k, w.seed(0, 4))).cuda()
    lw13, lw2 = lw if lw is not None else W.device_expert_weights(w, "cuda")
    ranks = list(range(w.G)) if ranks is None else list(ranks)
    shares = {g: (W.device_rank_share(lw13, s2e, g, w.spr, pad=pad), W.device_rank_share(lw2, s2e, g, w.spr, pad=pad))
              for g in ranks}
    del lw13, lw2
    sides, per_rank = [], {}
    for routing in routings:
        hp = HotPath(api, torch, w, d_ids, d_s2e, x, tw, shares, routing)
        settle(torch, [(hp, ranks[0])])
        per_rank[routing] = {g: hp.ffn_only_us(g) for g in ranks}
        g = max(per_rank[routing], key=per_rank[routing].get)
        hp.copies = {g: hp.copies[g]}
        sides.append((hp, g))
    keep = {g for _, g in sides}
    for g in list(shares):
        if g not in keep:
            del shares[g]                                # back to the allocator's cache, not to the driver
    settle(torch, sides)
    alone = None
    if alone_first and len(sides) > 1:
        (alone,), _ = interleaved(torch, sides[:1], steps, warmup)
    timed, wall_ms = interleaved(torch, sides, steps, warmup)
    out = {}
    for routing, (hp, g), t in zip(routings, sides, timed):
        assert int(hp.rb["err_flag"].item()) == 0
        active = int(hp.rb["rank_active"][0, g].item())
        P = int(hp.pb["n_pairs"].item())
        gu_b, dn_b = algorithmic_bytes(active, P, w.H, w.I)
        ffn = t["gate_up_us"] + t["down_us"]
        out[routing] = dict(rank=g, ms_per_step=t["ms_per_step"], ffn_q=quantiles(ffn), ffn_us=float(ffn.mean()),
                            gate_up_us=float(t["gate_up_us"].mean()), down_us=float(t["down_us"].mean()),
                            active=active, pairs=P, bytes=(gu_b, dn_b), lam=int(hp.rb["rank_active"].max().item()),
                            per_rank_ffn_us={int(k): round(v, 1) for k, v in per_rank[routing].items()},
                            stage_us=({k: round(v, 2) for k, v in hp.stage_breakdown(g).items()} if stages else None))
    first = out[routings[0]]
    if alone is not None:
        ffn = alone["gate_up_us"] + alone["down_us"]
        first["alone"] = dict(ms_per_step=alone["ms_per_step"], ffn_q=quantiles(ffn), ffn_us=float(ffn.mean()),
                              gate_up_us=float(alone["gate_up_us"].mean()), down_us=float(alone["down_us"].mean()))
    else:                                               # a single side was timed alone anyway
        first["alone"] = {k: first[k] for k in ("ms_per_step", "ffn_q", "ffn_us", "gate_up_us", "down_us")}
    return out, dict(ids=ids, s2e=s2e, x=x, tw=tw, d_ids=d_ids, d_s2e=d_s2e, shares=shares, sides=dict(zip(routings, sides)),
                     wall_ms=wall_ms)


def ratio_of(res):
    """METRO over token-balanced FFN time (medians); worth stating only when the gap exceeds both sides' spread."""
    me, tb = res["metro"], res["token_balanced"]
    gap = abs(me["ffn_q"][1] - tb["ffn_q"][1])
    spread = max(me["ffn_q"][2] - me["ffn_q"][0], tb["ffn_q"][2] - tb["ffn_q"][0])
    return {"ffn_time_ratio": round(me["ffn_q"][1] / tb["ffn_q"][1], 3), "conclusive": bool(gap > spread),
            "measured": "interleaved steps in one loop"}


def config_summary(w, res):
    """The comparison at one workload, as it goes into the JSON line."""
    d = {"T": w.T, "H": w.H, "I": w.I, "slots_per_rank": w.spr, "metro_vs_token_balanced": ratio_of(res)}
    for routing, r in res.items():
        gu_b, dn_b = r["bytes"]
        d[routing] = {"rank": r["rank"], "activated": r["active"], "pairs": r["pairs"], "max_activated_per_rank": r["lam"],
                      "ffn_us_p10_p50_p90": r["ffn_q"], "ms_per_step": round(r["ms_per_step"], 4),
                      "gate_up": {"us": round(r["gate_up_us"], 1), "algorithmic_gbs": round(gu_b / r["gate_up_us"] / 1e3, 1),
                                  "frac_of_hbm_peak": round(gu_b / r["gate_up_us"] / 1e3 / HBM_PEAK_GBS, 4)},
                      "down": {"us": round(r["down_us"], 1), "algorithmic_gbs": round(dn_b / r["down_us"] / 1e3, 1),
                               "frac_of_hbm_peak": round(dn_b / r["down_us"] / 1e3 / HBM_PEAK_GBS, 4)},
                      "ffn_algorithmic_gbs": round((gu_b + dn_b) / r["ffn_us"] / 1e3, 1)}
    return d


def replication_sweep(api, torch, W, steps: int, warmup: int):
    """The paper's main axis (Sec. 6.2, Fig. 10): replication ratio 1.0x .. 1.5x at the three FFN
    shapes, at the config's batch and at the 32-tokens-per-rank decode batch.  Per cell and router:
    max activated experts per rank, pairs on the slowest rank, its FFN time (gate/up + down events)."""
    rows = []
    for base in (W.QWEN3_30B, W.QWEN3_235B, W.DSV3):
        lw = W.device_expert_weights(base, "cuda")
        for ratio in (1.0, 1.125, 1.25, 1.5):
            spr = int(round(base.N * ratio / base.G))
            for T in sorted({32 * base.G, base.T}):
                w = base.with_(spr=spr, T=T)
                res, keep = compare_routings(api, torch, W, w, steps, warmup, lw=lw)
                cell = dict(workload=base.name, replication=ratio, slots_per_rank=spr, T=T)
                for routing, r in res.items():
                    cell[routing] = dict(max_activated=r["lam"], slowest_rank=r["rank"], activated=r["active"],
                                         pairs=r["pairs"], ffn_us=round(r["ffn_us"], 1), ffn_us_p10_p50_p90=r["ffn_q"])
                cell["ffn_time_metro_over_token_balanced"] = ratio_of(res)["ffn_time_ratio"]
                rows.append(cell)
                print(json.dumps(cell), file=sys.stderr, flush=True)
                del keep, res
                release_device_memory(torch)
        del lw
        release_device_memory(torch)
    return rows


def optional(fn, *a, **kw):
    """Side measurements must not take the benchmark line down with them: an exception becomes a field."""
    try:
        return fn(*a, **kw)
    except Exception as e:  # noqa: BLE001 - reported, not hidden
        print(f"bench.py: {getattr(fn, '__name__', fn)} failed: {e!r}", file=sys.stderr)
        return {"error": repr(e)}


def ffn_source_sha16() -> str:
    """Identifies the FFN kernel build a byte-counter profile belongs to: a hash of the kernel sources (the GPU machine
    has no git history to ask)."""
    import hashlib

    h = hashlib.sha256()
    for name in ("ffn.hip", "device_utils.h", "host_utils.h"):
        with open(os.path.join(ROOT, "paper_2512_09277_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def recorded_traffic(workload: str, routing: str, rank: int):
    """HBM-side bytes per launch of the two FFN kernels from the committed rocprofv3 counter summary
    (profiles/ffn_traffic_<workload>.json, written by paper_2512_09277_amd/rocprof_summary.py), or None with the
    reason when that summary was taken on another rank, routing or kernel source than this run's."""
    path = os.path.join(ROOT, "profiles", f"ffn_traffic_{workload}.json")
    if not os.path.exists(path):
        return None, "no counter summary for this workload"
    rec = json.load(open(path))
    for key, have in (("routing", routing), ("rank", rank), ("ffn_source_sha16", ffn_source_sha16())):
        if rec.get(key) != have:
            return None, f"counter summary is for {key}={rec.get(key)!r}, this run has {have!r}"
    return rec, None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="deepseek_v3_decode")
    ap.add_argument("--rank", type=int, default=-1, help="pin the measured rank (skips the per-rank search)")
    ap.add_argument("--only-metro", action="store_true",
                    help="METRO routing only: no token-balanced comparison, no other configs, no sweep")
    ap.add_argument("--only-token-balanced", action="store_true",
                    help="run the path under token-balanced routing only and print a reduced line (for profiling "
                         "the baseline's rank with rocprofv3)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-budget", type=float, default=12.0, help="seconds of oracle FFN work")
    ap.add_argument("--dense-weights", action="store_true",
                    help="weight rows back to back (default: rows of a multiple of 4096 bytes are padded by 128 "
                         "elements, the layout the library recommends)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference reading for rocprofv3 byte counters)")
    ap.add_argument("--no-hip-graph", action="store_true", help="skip the HIP-graph replay of the step")
    ap.add_argument("--no-per-config", action="store_true", help="skip the two Qwen3-shaped configs")
    ap.add_argument("--replication-sweep", action="store_true",
                    help="instead of the benchmark line: METRO vs token-balanced over replication ratios "
                         "1.0x..1.5x at the three FFN shapes (one JSON line of its own)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the G expert-parallel ranks are logical); "
              "--gpus must be 1", file=sys.stderr)
        return 2

    import torch

    from paper_2512_09277_amd import api
    from paper_2512_09277_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    api.load()
    torch.cuda.set_device(0)
    if args.replication_sweep:
        print(json.dumps({"mode": "replication_sweep", "unit": "us (slowest-rank expert FFN)", "steps": args.steps,
                          "rows": replication_sweep(api, torch, W, args.steps, args.warmup)}))
        return 0
    w = W.WORKLOADS[args.workload]
    if w.H == 0:
        print("that workload has no FFN shape", file=sys.stderr)
        return 2

    if args.calibration_copy:
        src = torch.empty((1 << 30,), dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        src.fill_(1)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    routings = (("token_balanced",) if args.only_token_balanced else ("metro",) if args.only_metro
                else ("metro", "token_balanced"))
    ranks = None if args.rank < 0 else [args.rank]
    result, keep = compare_routings(api, torch, W, w, args.steps, args.warmup, routings=routings, ranks=ranks,
                                    pad=not args.dense_weights, stages=True, alone_first=True)
    d_ids, d_s2e, x = keep["d_ids"], keep["d_s2e"], keep["x"]
    for routing, (hp, g) in keep["sides"].items():
        r = result[routing]
        r["graph_ms"] = None if args.no_hip_graph else optional(hp.graph_ms_per_step, g)
        r["route_graph_us"] = None if args.no_hip_graph else optional(
            graph_replay_us, torch, lambda hp=hp: hp.route_fn(d_ids, d_s2e, w.N, w.G, w.spr, out=hp.rb))
        r["perm"] = {k: v.cpu().numpy() for k, v in hp.pb.items()}
    if args.only_token_balanced:
        tb = result["token_balanced"]
        print(json.dumps({"mode": "token_balanced_only", "workload": w.name, "steps": args.steps, "rank": tb["rank"],
                          "activated": tb["active"], "pairs": tb["pairs"], "stage_us": tb["stage_us"],
                          "ffn_source_sha16": ffn_source_sha16(),
                          "algorithmic_bytes_per_launch": {"gate_up": tb["bytes"][0], "down": tb["bytes"][1]}}))
        return 0
    me = result["metro"]
    solo = me["alone"]                  # the timed region of the contract: K METRO steps back to back
    gu_b, dn_b = me["bytes"]
    ffn_gbs = (gu_b + dn_b) / (solo["ffn_us"] * 1e-6) / 1e9
    gu_gbs = gu_b / (solo["gate_up_us"] * 1e-6) / 1e9
    dn_gbs = dn_b / (solo["down_us"] * 1e-6) / 1e9
    rec, why = recorded_traffic(w.name, "metro", me["rank"])
    shares = keep["shares"]
    num = lambda v: round(v, 4) if isinstance(v, float) else v

    line = {
        "metric": METRIC, "value": round(ffn_gbs, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(solo["ms_per_step"], 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "E": w.N, "top_k": w.k, "G_logical_ranks": w.G, "slots_per_rank": w.spr,
                   "T": w.T, "zipf_s": w.s, "H": w.H, "I": w.I, "measured_rank": me["rank"], "routing": "metro",
                   "weight_row_pitch": {"w13": shares[me["rank"]][0].stride(1), "w2": shares[me["rank"]][1].stride(1)},
                   "timed_loop": "value, ms_per_step, ffn_us.metro and roofline: W + K METRO steps back to back; "
                                 "metro_vs_token_balanced, ffn_us_p10_p50_p90 and per_config: a second loop of W + K "
                                 "iterations that alternates a METRO step and a token-balanced step"},
        "route_us_per_batch": me["stage_us"]["route"],
        "route_us_per_batch_graph_replay": {"metro": num(me["route_graph_us"])},
        "ffn_us": {"metro": round(solo["ffn_us"], 1)},
        "ffn_us_p10_p50_p90": {"metro": me["ffn_q"], "metro_steps_back_to_back": solo["ffn_q"]},
        "max_activated_per_rank": {"metro": me["lam"]},
        "slowest_rank": {"metro": {"rank": me["rank"], "activated": me["active"], "pairs": me["pairs"]}},
        "stage_us": me["stage_us"],
        "ms_per_step_hip_graph": {"metro": num(me["graph_ms"])},
        "per_rank_ffn_us": {"metro": me["per_rank_ffn_us"]},
        "roofline": {"kernel": "ffn_mfma_kernel<gate_up>", "bound": "hbm", "achieved": round(gu_gbs, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gu_gbs / HBM_PEAK_GBS, 4),
                     "traffic": (rec["gate_up"]["fetch_bytes"] + rec["gate_up"]["write_bytes"]) if rec else None,
                     "traffic_source": (f"profiles/ffn_traffic_{w.name}.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, "
                                        f"kernel source {rec['ffn_source_sha16']})") if rec else why,
                     "algorithmic_bytes_per_launch": gu_b, "launch_duration_us": round(solo["gate_up_us"], 1),
                     "in_the_alternating_loop": {"launch_duration_us": round(me["gate_up_us"], 1),
                                                 "frac": round(gu_b / me["gate_up_us"] / 1e3 / HBM_PEAK_GBS, 4)},
                     "down_kernel": {"achieved": round(dn_gbs, 1), "frac": round(dn_gbs / HBM_PEAK_GBS, 4),
                                     "launch_duration_us": round(solo["down_us"], 1),
                                     "algorithmic_bytes_per_launch": dn_b,
                                     "traffic": (rec["down"]["fetch_bytes"] + rec["down"]["write_bytes"]) if rec else None}},
    }
    if not args.only_metro:
        line["gate_topk"] = optional(gate_topk_timing, api, torch, W, w, x)
        line["fp32_general_path"] = optional(fp32_path_timing, api, torch, W)
    if "token_balanced" in result:
        tb = result["token_balanced"]
        line["ffn_us"]["token_balanced"] = round(tb["ffn_us"], 1)
        line["ffn_us"]["metro_in_the_alternating_loop"] = round(me["ffn_us"], 1)
        line["ffn_us_p10_p50_p90"]["token_balanced"] = tb["ffn_q"]
        tb_gu = tb["bytes"][0] / (tb["gate_up_us"] * 1e-6) / 1e9
        line["roofline"]["same_kernel_on_token_balanced_rank"] = {
            "achieved": round(tb_gu, 1), "frac": round(tb_gu / HBM_PEAK_GBS, 4),
            "algorithmic_bytes_per_launch": tb["bytes"][0], "pairs": tb["pairs"]}
        line["metro_vs_token_balanced"] = ratio_of(result)
        line["max_activated_per_rank"]["token_balanced"] = tb["lam"]
        line["slowest_rank"]["token_balanced"] = {"rank": tb["rank"], "activated": tb["active"], "pairs": tb["pairs"]}
        line["per_rank_ffn_us"]["token_balanced"] = tb["per_rank_ffn_us"]
        line["ms_per_step_token_balanced"] = round(tb["ms_per_step"], 4)
        line["ms_per_step_metro_in_the_alternating_loop"] = round(me["ms_per_step"], 4)
        line["stage_us_token_balanced"] = tb["stage_us"]
        line["route_us_per_batch_graph_replay"]["token_balanced"] = num(tb["route_graph_us"])
        line["ms_per_step_hip_graph"]["token_balanced"] = num(tb["graph_ms"])
    host = lambda t: t.contiguous().cpu().view(torch.int16).numpy().view(np.uint16)
    cpu_in = None
    if not args.no_cpu_baseline:
        g = me["rank"]
        perm = dict(me["perm"])
        perm["n_pairs"] = int(perm["n_pairs"][0])
        cpu_in = (keep["ids"], keep["s2e"], host(x), host(shares[g][0]), host(shares[g][1]), perm)
    del keep, shares, x, d_ids, d_s2e, result           # stays in the allocator's cache for the runs below
    if "token_balanced" in routings:
        if not args.no_per_config:
            per = {w.name: config_summary(w, {k: v for k, v in (("metro", me), ("token_balanced", tb))})}
            for other in (W.QWEN3_235B, W.QWEN3_30B):
                if other.name == w.name:
                    continue
                got = optional(lambda: config_summary(other, compare_routings(api, torch, W, other, args.steps,
                                                                                args.warmup)[0]))
                per[other.name] = got
            line["per_config"] = per
        line["routing_sweep"] = optional(routing_sweep, api, torch, W, quick=False)
    if cpu_in is not None:
        from oracle import metro_oracle as oracle

        oracle.build()
        ids, s2e, hx, h13, h2, perm = cpu_in
        line["cpu_baseline"] = cpu_baseline(oracle, W, w, ids, s2e, hx, h13, h2, perm, gu_b + dn_b, args.cpu_budget)
        cnt = oracle.count(ids, w.N)
        t0 = time.perf_counter()
        lam_opt = oracle.matching_opt(cnt, s2e, w.N, w.G, w.spr)
        line["cpu_baseline"]["exact_solver"] = dict(lambda_opt=int(lam_opt), lambda_metro=me["lam"],
                                                    us_per_batch_cpu=round(1e6 * (time.perf_counter() - t0), 1))
        if isinstance(line.get("routing_sweep"), list):
            line["cpu_baseline"]["routing_quality"] = routing_quality(oracle, W, line["routing_sweep"])
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
