"""Parity of the HIP path (through the C ABI) against the CPU oracle, on the same seeded inputs.

Integer outputs (routing, permutation) must match bit for bit.  FFN outputs are compared with
    err = max|gpu - ref| / max|ref|      over the output tensor,
within 2e-2 for bf16 storage (the kernel rounds silu(gate)*up and y to bf16; the oracle never
rounds) and 1e-5 for fp32.  That is the contract.  Every-row comparisons also hold the kernels to what
the arithmetic actually gives (see check_close): the tensor-wide error within half the contract, the same
measure taken row by row (a wrong row cannot hide behind a larger one), and the element-wise relative
error with the denominator floored at 1e-3 * max|ref| reported and bounded at its median.
"""
import numpy as np
import pytest

from paper_2512_09277_amd import workloads as W

pytestmark = pytest.mark.gpu

BF16_TOL = 2e-2
F32_TOL = 1e-5


@pytest.fixture(scope="module")
def api():
    import torch

    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2512_09277_amd import api as a

    a.load()
    return a


def dev_i32(a):
    import torch

    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def dev_fp(a):
    """float32 array, or uint16 bf16 bit patterns -> device tensor of that dtype."""
    import torch

    if a.dtype == np.uint16:
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def host_f64(t):
    import torch

    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def rel_err(got, ref):
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))


def error_metrics(got, ref):
    """tensor-wide max|d|/max|ref|; the same per row (rows of at most 1e-6 of the tensor's scale are measured
    against that scale); element-wise |d|/max(|ref|, 1e-3 max|ref|): its maximum and 99.9th percentile."""
    d = np.abs(got - ref)
    scale = max(float(np.abs(ref).max()), 1e-30)
    row_scale = np.maximum(np.abs(ref).reshape(ref.shape[0], -1).max(axis=1), 1e-6 * scale)
    elem = d / np.maximum(np.abs(ref), 1e-3 * scale)
    return dict(tensor=float(d.max() / scale), row=float((d.reshape(d.shape[0], -1).max(axis=1) / row_scale).max()),
                elem_max=float(elem.max()), elem_p999=float(np.quantile(elem, 0.999)), elem_median=float(np.median(elem)))


def check_close(got, ref, tol, what):
    """The contract (tensor-wide error <= tol) and the tighter bounds the arithmetic supports: two bf16
    roundings (relative 2^-9 each) on sums of hundreds to thousands of terms leave a tensor-wide error of a few
    1e-3, so half the contract must hold tensor-wide and the whole contract row by row.  The element-wise
    measure is reported (maximum, 99.9th percentile) and bounded at its median: every element carries about the
    same absolute error, so the few elements near the 1e-3 floor are off by a large fraction of themselves
    whatever the kernel does (at most tensor error / 1e-3), while the typical element must be good to half the
    contract."""
    if got.size == 0:
        return None
    m = error_metrics(got, ref)
    print(f"{what}: tensor {m['tensor']:.2e} per-row {m['row']:.2e} element-wise max {m['elem_max']:.2e} "
          f"p99.9 {m['elem_p999']:.2e} median {m['elem_median']:.2e} (contract {tol:.0e})", flush=True)
    assert m["tensor"] <= tol / 2, f"{what}: tensor-wide error {m['tensor']}"
    assert m["row"] <= tol, f"{what}: per-row error {m['row']}"
    assert m["elem_median"] <= tol / 2, f"{what}: element-wise median {m['elem_median']}"
    assert m["elem_max"] <= m["tensor"] / 1e-3 * (1 + 1e-9)
    return m


def check_routing(api, oracle, ids, s2e, N, G, spr):
    """ids [L,T,k], s2e [L,S]: both routers on the GPU vs the oracle, bit for bit."""
    L = ids.shape[0]
    d_ids, d_s2e = dev_i32(ids), dev_i32(s2e)
    me = api.metro_route(d_ids, d_s2e, N, G, spr)
    tb = api.metro_route_token_balanced(d_ids, d_s2e, N, G, spr)
    me = {k: v.cpu().numpy() for k, v in me.items()}
    tb = {k: v.cpu().numpy() for k, v in tb.items()}
    for l in range(L):
        rm = oracle.route_metro(ids[l], s2e[l], N, G, spr)
        rt = oracle.route_token_balanced(ids[l], s2e[l], N, G, spr)
        assert me["err_flag"][l] == 0 and tb["err_flag"][l] == 0
        assert np.array_equal(me["pair_slot"][l], rm["pair_slot"]), f"METRO pair_slot, layer {l}"
        assert np.array_equal(me["expert_slot"][l], rm["expert_slot"])
        assert np.array_equal(me["rank_active"][l], rm["rank_active"])
        assert np.array_equal(me["rank_bitmap"][l].view(np.uint64), rm["rank_bitmap"])
        assert np.array_equal(tb["pair_slot"][l], rt["pair_slot"]), f"token-balanced pair_slot, layer {l}"
        assert np.array_equal(tb["rank_active"][l], rt["rank_active"])
        assert np.array_equal(tb["rank_bitmap"][l].view(np.uint64), rt["rank_bitmap"])
    return me, tb


# ----------------------------------------------------------------------------- routing
@pytest.mark.parametrize("w", [W.TINY, W.QWEN3_30B, W.QWEN3_235B, W.DSV3], ids=lambda w: w.name)
def test_routing_configs(api, oracle, w):
    print(f"routing parity {w.name}", flush=True)
    s2e, ids = W.routing_inputs_layers(w.with_(layers=4))
    check_routing(api, oracle, ids, s2e, w.N, w.G, w.spr)


@pytest.mark.parametrize("T", W.SWEEP_T)
def test_routing_sweep_58_layers(api, oracle, T):
    """The routing-only sweep at its launch shape: 58 layers in one launch, G=16."""
    w = W.DSV3_SWEEP
    for s in W.SWEEP_S:
        print(f"routing sweep T={T} s={s}", flush=True)
        s2e, ids = W.routing_inputs_layers(w, T=T, s=s)
        check_routing(api, oracle, ids, s2e, w.N, w.G, w.spr)


@pytest.mark.parametrize("seed", range(12))
def test_routing_random_edge_cases(api, oracle, seed):
    """Ragged T*k (no 16-byte multiple), padded pairs, empty slots, duplicates on a rank,
    experts without tokens, N not a multiple of 64, up to the 512-expert / 64-rank limits."""
    rng = np.random.default_rng(4242 + seed)
    N = int(rng.choice([1, 3, 16, 63, 65, 130, 257, 512]))
    G = int(rng.choice([1, 2, 5, 16, 33, 64]))
    if -(-N // G) > 64:
        G = -(-N // 64)
    spr = int(min(64, -(-N // G) + rng.integers(0, 4)))
    assert G * spr >= N and G * spr <= 2048
    k = int(min(N, rng.choice([1, 2, 3, 8])))
    T = int(rng.choice([0, 1, 5, 64, 67, 333, 1500]))
    print(f"edge case seed={seed} N={N} G={G} spr={spr} k={k} T={T}", flush=True)
    S = G * spr
    L = 3
    s2e = np.full((L, S), -1, np.int32)
    ids = np.empty((L, T, k), np.int32)
    for l in range(L):
        order = rng.permutation(S)
        s2e[l, order[:N]] = rng.permutation(N)
        extra = order[N:]
        fill = rng.random(extra.size) < 0.6
        s2e[l, extra[fill]] = rng.integers(0, N, size=int(fill.sum()))      # may duplicate on a rank
        hot = rng.permutation(N)[: max(1, N // 2)]                           # half the experts get no token
        for t in range(T):
            ids[l, t] = rng.choice(hot, size=k, replace=hot.size < k)
        pad = rng.random((T, k)) < 0.05
        ids[l][pad] = -1
    check_routing(api, oracle, ids, s2e, N, G, spr)


def test_largest_batch_routing_and_token_lists(api, oracle):
    """T*k = 2^24 - 8, the largest batch the calls accept (the DeepSeek-V3 placement shape): both routers
    and the token lists of one rank, bit for bit; one more token is refused on the host."""
    import torch

    N, G, spr, k = 256, 8, 36, 8
    T = (1 << 21) - 1
    rng = np.random.default_rng(99)
    s2e = np.full(G * spr, -1, np.int32)
    order = rng.permutation(G * spr)
    s2e[order[:N]] = rng.permutation(N)
    s2e[order[N:]] = rng.choice(N, size=G * spr - N, replace=False)        # 32 second replicas
    # k distinct experts per token: an arithmetic progression with an odd step modulo N (a power of two)
    base, step = rng.integers(0, N, size=(T, 1)), 2 * rng.integers(0, N // 2, size=(T, 1)) + 1
    ids = ((base + step * np.arange(k)) % N).astype(np.int32)
    ids[rng.random((T, k)) < 0.01] = -1
    print(f"largest batch: T={T} k={k}", flush=True)
    me, tb = check_routing(api, oracle, ids[None], s2e[None], N, G, spr)
    for ps in (me["pair_slot"][0], tb["pair_slot"][0]):
        g = 3
        pm = api.moe_permute(dev_i32(ps), g, spr)
        ref = oracle.permute(ps, g, spr)
        n = ref["n_pairs"]
        assert int(pm["n_pairs"].item()) == n
        assert np.array_equal(pm["group_offsets"].cpu().numpy(), ref["group_offsets"])
        assert np.array_equal(pm["perm_pair"].cpu().numpy()[:n], ref["perm_pair"])
        assert np.array_equal(pm["pair_row"].cpu().numpy(), ref["pair_row"])
    with pytest.raises(api.MetroError):
        api.metro_route(torch.zeros((1, T + 1, k), dtype=torch.int32, device="cuda"), dev_i32(s2e[None]), N, G, spr)


def test_routing_is_deterministic(api):
    w = W.DSV3_SWEEP
    s2e, ids = W.routing_inputs_layers(w.with_(layers=8), T=1024)
    d_ids, d_s2e = dev_i32(ids), dev_i32(s2e)
    first = api.metro_route(d_ids, d_s2e, w.N, w.G, w.spr)["pair_slot"].clone()
    first_tb = api.metro_route_token_balanced(d_ids, d_s2e, w.N, w.G, w.spr)["pair_slot"].clone()
    import torch

    bad = torch.zeros((), dtype=torch.int64, device="cuda")
    for _ in range(1000):                                       # mismatches accumulate on the device: no sync per call
        bad += (api.metro_route(d_ids, d_s2e, w.N, w.G, w.spr)["pair_slot"] != first).sum()
        bad += (api.metro_route_token_balanced(d_ids, d_s2e, w.N, w.G, w.spr)["pair_slot"] != first_tb).sum()
    assert int(bad.item()) == 0


def test_routing_error_flags(api):
    s2e = dev_i32(np.array([[0, 1, 2, -1]]))
    out = api.metro_route(dev_i32(np.array([[[3]]])), s2e, 4, 2, 2)
    assert out["err_flag"].item() == api.FLAG_NO_REPLICA
    out = api.metro_route_token_balanced(dev_i32(np.array([[[3]]])), s2e, 4, 2, 2)
    assert out["err_flag"].item() == api.FLAG_NO_REPLICA and out["pair_slot"].item() == -1
    out = api.metro_route(dev_i32(np.array([[[7], [1]]])), s2e, 4, 2, 2)
    assert out["err_flag"].item() == api.FLAG_BAD_ID
    assert out["pair_slot"].cpu().numpy().reshape(-1).tolist() == [-1, 1]
    out = api.metro_route_token_balanced(dev_i32(np.array([[[-5], [1]]])), s2e, 4, 2, 2)
    assert out["err_flag"].item() == api.FLAG_BAD_ID
    bad = dev_i32(np.array([[0, 1, 9, -1]]))
    assert api.metro_route(dev_i32(np.array([[[1]]])), bad, 4, 2, 2)["err_flag"].item() == api.FLAG_BAD_PLACEMENT


# ----------------------------------------------------------------------------- permute
@pytest.mark.parametrize("w", [W.TINY, W.QWEN3_30B, W.DSV3], ids=lambda w: w.name)
def test_permute_all_ranks(api, oracle, w):
    _, s2e, ids = W.routing_inputs(w)
    for route in (oracle.route_metro, oracle.route_token_balanced):
        ps = route(ids, s2e, w.N, w.G, w.spr)["pair_slot"]
        d_ps = dev_i32(ps)
        for g in range(w.G):
            ref = oracle.permute(ps, g, w.spr)
            got = api.moe_permute(d_ps, g, w.spr)
            n = int(got["n_pairs"].item())
            assert n == ref["n_pairs"]
            assert np.array_equal(got["group_offsets"].cpu().numpy(), ref["group_offsets"])
            assert np.array_equal(got["perm_pair"].cpu().numpy()[:n], ref["perm_pair"])
            assert np.array_equal(got["pair_row"].cpu().numpy(), ref["pair_row"])


@pytest.mark.parametrize("w", [W.TINY, W.QWEN3_30B, W.QWEN3_235B, W.DSV3], ids=lambda w: w.name)
def test_route_and_token_lists_in_one_launch(api, oracle, w):
    """metro_route_permute / metro_route_token_balanced_permute: the routing outputs and one rank's token lists
    from a single launch equal the separate calls and the oracle, bit for bit, for every rank."""
    _, s2e, ids = W.routing_inputs(w)
    d_ids, d_s2e = dev_i32(ids), dev_i32(s2e)
    for fused, route_ref in ((api.metro_route_permute, oracle.route_metro),
                             (api.metro_route_token_balanced_permute, oracle.route_token_balanced)):
        ref = route_ref(ids, s2e, w.N, w.G, w.spr)
        for g in range(w.G):
            out, pm = fused(d_ids, d_s2e, w.N, w.G, w.spr, g)
            assert int(out["err_flag"].item()) == 0
            assert np.array_equal(out["pair_slot"][0].cpu().numpy(), ref["pair_slot"])
            assert np.array_equal(out["rank_active"][0].cpu().numpy(), ref["rank_active"])
            assert np.array_equal(out["rank_bitmap"][0].cpu().numpy().view(np.uint64), ref["rank_bitmap"])
            rp = oracle.permute(ref["pair_slot"], g, w.spr)
            n = rp["n_pairs"]
            assert int(pm["n_pairs"].item()) == n
            assert np.array_equal(pm["group_offsets"].cpu().numpy(), rp["group_offsets"])
            assert np.array_equal(pm["perm_pair"].cpu().numpy()[:n], rp["perm_pair"])
            assert np.array_equal(pm["pair_row"].cpu().numpy(), rp["pair_row"])
    # ragged pair count (no 16-byte multiple), padded pairs, an empty rank
    rng = np.random.default_rng(5)
    N, G, spr, k, T = 33, 5, 9, 3, 333
    s2e = np.full(G * spr, -1, np.int32)
    s2e[rng.permutation((G - 1) * spr)[:N]] = np.arange(N)       # the last rank hosts nothing
    ids = np.stack([rng.permutation(N)[:k] for _ in range(T)]).astype(np.int32)
    ids[rng.random(ids.shape) < 0.1] = -1
    for fused, route_ref in ((api.metro_route_permute, oracle.route_metro),
                             (api.metro_route_token_balanced_permute, oracle.route_token_balanced)):
        ref = route_ref(ids, s2e, N, G, spr)
        for g in (0, 2, G - 1):
            out, pm = fused(dev_i32(ids), dev_i32(s2e), N, G, spr, g)
            rp = oracle.permute(ref["pair_slot"], g, spr)
            assert np.array_equal(out["pair_slot"][0].cpu().numpy(), ref["pair_slot"])
            assert int(pm["n_pairs"].item()) == rp["n_pairs"]
            assert np.array_equal(pm["group_offsets"].cpu().numpy(), rp["group_offsets"])
            assert np.array_equal(pm["perm_pair"].cpu().numpy()[:rp["n_pairs"]], rp["perm_pair"])
            assert np.array_equal(pm["pair_row"].cpu().numpy(), rp["pair_row"])
    with pytest.raises(api.MetroError):
        api.metro_route_permute(dev_i32(ids), dev_i32(s2e), N, G, spr, G)          # rank out of range


def test_permute_edge_cases(api, oracle):
    rng = np.random.default_rng(9)
    for T, k, spr, G in [(1, 1, 1, 1), (67, 3, 64, 2), (4096, 8, 18, 16), (5, 2, 7, 3)]:
        ps = rng.integers(-1, G * spr, size=(T, k)).astype(np.int32)
        for g in {0, G - 1}:
            ref = oracle.permute(ps, g, spr)
            got = api.moe_permute(dev_i32(ps), g, spr)
            n = int(got["n_pairs"].item())
            assert n == ref["n_pairs"]
            assert np.array_equal(got["group_offsets"].cpu().numpy(), ref["group_offsets"])
            assert np.array_equal(got["perm_pair"].cpu().numpy()[:n], ref["perm_pair"])
            assert np.array_equal(got["pair_row"].cpu().numpy(), ref["pair_row"])
    none = np.full((8, 2), 5, np.int32)                                      # nothing on rank 0
    got = api.moe_permute(dev_i32(none), 0, 3)
    assert got["n_pairs"].item() == 0 and (got["pair_row"] == -1).all() and (got["group_offsets"] == 0).all()


# ----------------------------------------------------------------------------- FFN + combine
def ffn_call(api, x, perm_pair, group_offsets, k, w13, w2):
    """moe_grouped_ffn into an output and a workspace pre-filled with 0xFF bytes (NaN in bf16 and
    f32): a row the kernels skip cannot pass on values left behind by an earlier call."""
    import torch

    T, H = x.shape
    spr, I = w13.shape[0], w13.shape[1] // 2
    y = torch.full((T * k, H), float("nan"), dtype=x.dtype, device=x.device)
    ws = torch.full((api.moe_grouped_ffn_workspace_bytes(T, k, spr, H, I, x.dtype),), 0xFF, dtype=torch.uint8,
                    device=x.device)
    return api.moe_grouped_ffn(x, perm_pair, group_offsets, k, w13, w2, y_perm=y, ws=ws)


def run_rank(api, oracle, x, w13, w2, tw, ps, g, spr, k, tol, rows=None):
    """One rank end to end on the GPU (permute -> FFN -> unpermute) against the oracle."""
    d_ps = dev_i32(ps)
    pm = api.moe_permute(d_ps, g, spr)
    ref_pm = oracle.permute(ps, g, spr)
    n = ref_pm["n_pairs"]
    y = ffn_call(api, dev_fp(x), pm["perm_pair"], pm["group_offsets"], k, dev_fp(w13), dev_fp(w2))
    out = api.moe_unpermute(y, pm["pair_row"], dev_fp(tw))
    ref_y = oracle.ffn(x, ref_pm["perm_pair"], ref_pm["group_offsets"], k, w13, w2, rows=rows)
    got_y = host_f64(y)[:n] if rows is None else host_f64(y)[np.asarray(rows)]
    if n:
        check_close(got_y, ref_y, tol, f"y_perm rank {g}")
    if rows is None:
        ref_out = oracle.unpermute(ref_y, ref_pm["pair_row"], tw)
        got_out = host_f64(out)
        if n:
            check_close(got_out, ref_out, tol, f"out rank {g}")
        assert (got_out[(ref_pm["pair_row"] < 0).all(axis=1)] == 0).all()
        return got_out, ref_out
    return None, None


@pytest.mark.parametrize("dtype,tol", [("f32", F32_TOL), ("bf16", BF16_TOL)])
def test_tiny_layer_all_ranks(api, oracle, dtype, tol):
    """Tiny config, every rank, both routers; the summed partial outputs also equal each other
    (the layer output does not depend on the routing)."""
    w = W.TINY
    _, s2e, ids = W.routing_inputs(w)
    x = W.activations(w.T, w.H, w.seed(0, 3), dtype)
    w13, w2 = W.expert_weights(w.N, w.H, w.I, w.seed(0, 2), dtype)
    tw = W.gating_weights(w.T, w.k, w.seed(0, 4))
    d_ids, d_s2e = dev_i32(ids), dev_i32(s2e)
    totals = []
    for route in (api.metro_route, api.metro_route_token_balanced):
        ps = route(d_ids, d_s2e, w.N, w.G, w.spr)["pair_slot"][0].cpu().numpy()
        total, total_ref = 0, 0
        for g in range(w.G):
            print(f"tiny {dtype} {route.__name__} rank {g}", flush=True)
            got, ref = run_rank(api, oracle, x, W.rank_share(w13, s2e, g, w.spr), W.rank_share(w2, s2e, g, w.spr),
                                tw, ps, g, w.spr, w.k, tol)
            total, total_ref = total + got, total_ref + ref
        assert rel_err(total, total_ref) <= tol
        totals.append(total)
    assert rel_err(totals[0], totals[1]) <= 2 * tol


@pytest.mark.parametrize("dtype,H,I,tol", [("bf16", 512, 256, BF16_TOL), ("bf16", 384, 128, BF16_TOL),
                                           ("bf16", 2048, 1024, BF16_TOL),
                                           ("bf16", 200, 72, BF16_TOL), ("f32", 200, 72, F32_TOL)])
def test_ragged_groups_span_tiles(api, oracle, dtype, H, I, tol):
    """Groups of 0, 1, 15, 16, 17, 33, 64, 100, 129 and 300 rows: every sub-tile count, a ragged tail,
    a group longer than two work tiles, a one-tile group that the mid shape cuts in two, an empty slot.  The small shapes cut groups into 32-row
    tiles, (2048, 1024) into 128-row tiles on the streaming path, (200, 72) takes the general kernel."""
    sizes = [17, 0, 1, 300, 16, 33, 129, 15, 64, 100]
    spr, k = len(sizes), 4
    n = sum(sizes)
    T = 200
    rng = np.random.default_rng(77)
    pairs = rng.permutation(T * k)[:n]
    ps = np.full(T * k, -1, np.int32)
    at = 0
    for l, m in enumerate(sizes):
        ps[pairs[at:at + m]] = 2 * spr + l                                    # rank 2 of G=3
        at += m
    ps = ps.reshape(T, k)
    x = W.activations(T, H, 5, dtype)
    w13, w2 = W.expert_weights(spr, H, I, 6, dtype)
    tw = W.gating_weights(T, k, 7)
    print(f"ragged {dtype} H={H} I={I}", flush=True)
    run_rank(api, oracle, x, w13, w2, tw, ps, 2, spr, k, tol)


@pytest.mark.parametrize("dtype,H,I,tol", [("bf16", 512, 256, BF16_TOL), ("f32", 200, 72, F32_TOL)])
def test_padded_weight_rows(api, oracle, dtype, H, I, tol):
    """Weights stored with a row pitch larger than the row (the layout the benchmark uses): same result."""
    import torch

    sizes = [17, 0, 140, 5]
    spr, k, T = len(sizes), 2, 120
    rng = np.random.default_rng(3)
    pairs = rng.permutation(T * k)[:sum(sizes)]
    ps = np.full(T * k, -1, np.int32)
    at = 0
    for l, m in enumerate(sizes):
        ps[pairs[at:at + m]] = l
        at += m
    ps = ps.reshape(T, k)
    x = W.activations(T, H, 5, dtype)
    w13, w2 = W.expert_weights(spr, H, I, 6, dtype)

    def padded(a, extra):
        t = dev_fp(a)
        buf = torch.full((t.shape[0], t.shape[1], t.shape[2] + extra), 7.0, dtype=t.dtype, device="cuda")
        view = buf[:, :, :t.shape[2]]
        view.copy_(t)
        return view

    pm = api.moe_permute(dev_i32(ps), 0, spr)
    y = ffn_call(api, dev_fp(x), pm["perm_pair"], pm["group_offsets"], k, padded(w13, 128), padded(w2, 64))
    ref_pm = oracle.permute(ps, 0, spr)
    ref = oracle.ffn(x, ref_pm["perm_pair"], ref_pm["group_offsets"], k, w13, w2)
    assert rel_err(host_f64(y)[:ref_pm["n_pairs"]], ref) <= tol


def test_wide_and_stream_tiles_large_shape(api, oracle):
    """H*I large enough that groups above 32 rows leave the stream path: one-tile groups of every
    wide variant (33..64, 65..96 and 97..128 rows: 40, 33, 80, 96, 120, 128), groups of several tiles with
    remainders in each of those classes and a narrow one (300, 257, 208, 352, 248, 460, 600), narrow groups,
    an empty slot; every row is compared."""
    H, I, k, T = 4096, 2048, 4, 1024
    sizes = [300, 40, 0, 20, 128, 33, 1, 129 + 128, 32, 80, 96, 120, 128 + 80, 2 * 128 + 96, 128 + 120, 460, 600]
    spr = len(sizes)
    rng = np.random.default_rng(5)
    pairs = rng.permutation(T * k)[:sum(sizes)]
    ps = np.full(T * k, -1, np.int32)
    at = 0
    for l, m in enumerate(sizes):
        ps[pairs[at:at + m]] = l
        at += m
    ps = ps.reshape(T, k)
    x = W.activations(T, H, 15, "bf16")
    w13, w2 = W.expert_weights(spr, H, I, 16, "bf16")
    tw = W.gating_weights(T, k, 17)
    print("wide + stream tiles, H=4096 I=2048", flush=True)
    run_rank(api, oracle, x, w13, w2, tw, ps, 0, spr, k, BF16_TOL)


@pytest.mark.parametrize("dtype,H,I,k,T,sizes,tol", [
    ("bf16", 256, 128, 8, 4096, [20000, 3, 0, 4097, 1], BF16_TOL),          # 626 + 129 tiles of 32 rows
    ("f32", 256, 128, 8, 4096, [20000, 3, 0, 4097, 1], F32_TOL),            # general kernels, 1251 tiles of 16 rows
    ("bf16", 4096, 2048, 2, 2048, [3000, 500, 96, 17], BF16_TOL),           # 23 + 3 full wide tiles and remainders
], ids=["bf16-small-shape", "f32-small-shape", "bf16-large-shape"])
def test_many_row_tiles(api, oracle, dtype, H, I, k, T, sizes, tol):
    """A slot with far more rows than one tile holds (an expert that nearly every token of a large batch
    picked): hundreds of row tiles in one slot, work-item ids in the thousands; every row is compared."""
    spr = len(sizes)
    rng = np.random.default_rng(41)
    pairs = rng.permutation(T * k)[:sum(sizes)]
    ps = np.full(T * k, -1, np.int32)
    at = 0
    for l, m in enumerate(sizes):
        ps[pairs[at:at + m]] = l
        at += m
    ps = ps.reshape(T, k)
    x = W.activations(T, H, 42, dtype)
    w13, w2 = W.expert_weights(spr, H, I, 43, dtype)
    tw = W.gating_weights(T, k, 44)
    print(f"many row tiles {dtype} H={H} I={I} sizes={sizes}", flush=True)
    run_rank(api, oracle, x, w13, w2, tw, ps, 0, spr, k, tol)


def test_ffn_stage_calls_and_workspace_reuse(api, oracle):
    """The two stage calls (gate_up, down) equal the whole call, and a workspace can be used again
    without being cleared: the same rows come out on every pass."""
    import torch

    H, I, k, T = 512, 256, 4, 200
    sizes = [17, 0, 1, 300, 16, 33, 129, 15, 64]
    spr = len(sizes)
    rng = np.random.default_rng(78)
    pairs = rng.permutation(T * k)[:sum(sizes)]
    ps = np.full(T * k, -1, np.int32)
    at = 0
    for l, m in enumerate(sizes):
        ps[pairs[at:at + m]] = l
        at += m
    ps = ps.reshape(T, k)
    x = dev_fp(W.activations(T, H, 5, "bf16"))
    w13h, w2h = W.expert_weights(spr, H, I, 6, "bf16")
    w13, w2 = dev_fp(w13h), dev_fp(w2h)
    pm = api.moe_permute(dev_i32(ps), 0, spr)
    ref_pm = oracle.permute(ps, 0, spr)
    n = ref_pm["n_pairs"]
    ref = oracle.ffn(W.activations(T, H, 5, "bf16"), ref_pm["perm_pair"], ref_pm["group_offsets"], k, w13h, w2h)
    ws = torch.full((api.moe_grouped_ffn_workspace_bytes(T, k, spr, H, I, torch.bfloat16),), 0xFF, dtype=torch.uint8,
                    device="cuda")
    y = torch.empty((T * k, H), dtype=torch.bfloat16, device="cuda")
    lib, st = api.load(), api._stream()
    args = (T, k, spr, H, I, api.DTYPE_BF16)
    go, pp = pm["group_offsets"], pm["perm_pair"]
    for _ in range(3):                                   # stage calls, same workspace
        y.fill_(float("nan"))
        assert lib.moe_grouped_ffn_gate_up(x.data_ptr(), pp.data_ptr(), go.data_ptr(), *args, w13.data_ptr(), H,
                                           ws.data_ptr(), ws.numel(), st) == 0
        assert lib.moe_grouped_ffn_down(go.data_ptr(), *args, w2.data_ptr(), I, y.data_ptr(), ws.data_ptr(),
                                        ws.numel(), st) == 0
        torch.cuda.synchronize()
        assert rel_err(host_f64(y)[:n], ref) <= BF16_TOL
    for _ in range(2):                                   # whole call, same workspace
        y.fill_(float("nan"))
        api.moe_grouped_ffn(x, pp, go, k, w13, w2, y_perm=y, ws=ws)
        assert rel_err(host_f64(y)[:n], ref) <= BF16_TOL


def test_empty_rank_ffn(api):
    """No pair on the rank: nothing is written, nothing faults."""
    import torch

    T, k, spr, H, I = 16, 2, 4, 256, 128
    ps = dev_i32(np.full((T, k), -1))
    pm = api.moe_permute(ps, 0, spr)
    x = torch.zeros((T, H), dtype=torch.bfloat16, device="cuda")
    w13 = torch.zeros((spr, 2 * I, H), dtype=torch.bfloat16, device="cuda")
    w2 = torch.zeros((spr, H, I), dtype=torch.bfloat16, device="cuda")
    y = torch.full((T * k, H), 3.0, dtype=torch.bfloat16, device="cuda")
    api.moe_grouped_ffn(x, pm["perm_pair"], pm["group_offsets"], k, w13, w2, y_perm=y)
    out = api.moe_unpermute(y, pm["pair_row"], torch.ones((T, k), device="cuda"))
    torch.cuda.synchronize()
    assert (y == 3.0).all() and (out == 0).all()


@pytest.mark.parametrize("dtype,H,I", [("bf16", 256, 128), ("f32", 200, 72)])
def test_malformed_lists_stay_in_bounds(api, dtype, H, I):
    """group_offsets that are no partition of the rows and perm_pair entries that are no pair index are
    clamped by the kernels (every row index stays below T*k, every token below T, every slot below spr):
    the call must not touch memory past its buffers.  Checked with guard regions after y_perm and after
    the workspace; the results of such a call are unspecified."""
    import torch

    T, k, spr = 40, 4, 6
    cap = T * k
    x = dev_fp(W.activations(T, H, 71, dtype))
    w13, w2 = (dev_fp(a) for a in W.expert_weights(spr, H, I, 72, dtype))
    guard = 64
    y_buf = torch.full((cap + guard, H), 7.0, dtype=x.dtype, device="cuda")
    need = api.moe_grouped_ffn_workspace_bytes(T, k, spr, H, I, x.dtype)
    ws_buf = torch.full((need + 4096,), 0x5A, dtype=torch.uint8, device="cuda")
    rng = np.random.default_rng(73)
    for go in ([0, 50, 20, 10**9, -7, 90, cap + 1000], [cap] * (spr + 1), [-5] * (spr + 1),
               [0, cap, 0, cap, 0, cap, 0], rng.integers(-300, 600, size=spr + 1).tolist()):
        pp = rng.integers(-10**6, 10**6, size=cap)
        print(f"malformed offsets {go}", flush=True)
        api.moe_grouped_ffn(x, dev_i32(pp), dev_i32(go), k, w13, w2, y_perm=y_buf[:cap], ws=ws_buf[:need])
        torch.cuda.synchronize()
        assert (y_buf[cap:] == 7.0).all(), "wrote past y_perm"
        assert (ws_buf[need:] == 0x5A).all(), "wrote past the workspace"
    # the combine skips rows outside [0, T*k)
    out_buf = torch.full((T + 8, H), 7.0, dtype=x.dtype, device="cuda")
    pr = rng.integers(-10**6, 10**6, size=(T, k))
    pr[0] = [0, cap - 1, cap, -1]
    tw = torch.ones((T, k), dtype=torch.float32, device="cuda")
    y_buf[:cap] = 1.0
    api.moe_unpermute(y_buf[:cap], dev_i32(pr), tw, out=out_buf[:T])
    torch.cuda.synchronize()
    assert (out_buf[T:] == 7.0).all(), "wrote past out"
    valid = ((pr >= 0) & (pr < cap)).sum(axis=1)
    assert valid[0] == 2 and np.array_equal(host_f64(out_buf[:T])[:, 0], valid.astype(np.float64))


@pytest.mark.parametrize("w,routing", [(W.QWEN3_30B, "metro"), (W.QWEN3_30B, "token_balanced"),
                                       (W.QWEN3_235B, "metro"), (W.QWEN3_235B, "token_balanced"),
                                       (W.DSV3, "metro"), (W.DSV3, "token_balanced")],
                         ids=lambda v: getattr(v, "name", v))
def test_full_size_every_row(api, oracle, w, routing):
    """Full shapes in the launch configuration the benchmark times (padded weight rows, the busiest rank under
    the given routing, weights drawn on the device): EVERY row of y_perm and the whole combined output are
    compared with the oracle, which works from host copies of the same bytes."""
    import torch

    _, s2e, ids = W.routing_inputs(w)
    route, route_ref = ((api.metro_route, oracle.route_metro) if routing == "metro" else
                        (api.metro_route_token_balanced, oracle.route_token_balanced))
    out = route(dev_i32(ids), dev_i32(s2e), w.N, w.G, w.spr)
    ps = out["pair_slot"][0].cpu().numpy()
    ref = route_ref(ids, s2e, w.N, w.G, w.spr)
    assert np.array_equal(ps, ref["pair_slot"])
    g = int(np.argmax(np.bincount(ps.reshape(-1) // w.spr, minlength=w.G)))
    lw13, lw2 = W.device_expert_weights(w, "cuda")
    w13 = W.device_rank_share(lw13, s2e, g, w.spr, pad=True)       # the layout bench.py times
    w2 = W.device_rank_share(lw2, s2e, g, w.spr, pad=True)
    del lw13, lw2
    x = W.device_activations(w, "cuda")
    tw = W.gating_weights(w.T, w.k, w.seed(0, 4))
    pm = api.moe_permute(out["pair_slot"][0], g, w.spr)
    y = ffn_call(api, x, pm["perm_pair"], pm["group_offsets"], w.k, w13, w2)
    res = api.moe_unpermute(y, pm["pair_row"], dev_fp(tw))
    torch.cuda.synchronize()
    ref_pm = oracle.permute(ps, g, w.spr)
    go = ref_pm["group_offsets"]
    n = ref_pm["n_pairs"]
    print(f"full size {w.name} {routing}: rank {g}, {n} rows, groups {sorted(np.diff(go).tolist(), reverse=True)[:6]}",
          flush=True)
    assert np.array_equal(pm["group_offsets"].cpu().numpy(), go)
    assert np.array_equal(pm["pair_row"].cpu().numpy(), ref_pm["pair_row"])
    assert not torch.isnan(y[:n]).any(), "a row of the rank was not computed"
    host = lambda t: t.contiguous().cpu().view(torch.int16).numpy().view(np.uint16)
    ref_y = oracle.ffn(host(x), ref_pm["perm_pair"], go, w.k, host(w13), host(w2))
    check_close(host_f64(y[:n]), ref_y, BF16_TOL, f"{w.name} {routing} y_perm")
    ref_out = oracle.unpermute(ref_y, ref_pm["pair_row"], tw)
    got_out = host_f64(res)
    check_close(got_out, ref_out, BF16_TOL, f"{w.name} {routing} out")
    # rows of tokens with no pair on this rank are exactly zero
    assert (got_out[(ref_pm["pair_row"] < 0).all(axis=1)] == 0).all()


def test_nan_rows_stay_nan(api):
    """A NaN activation makes every output of its rows NaN -- never Inf or a finite number (rounding a NaN
    to bf16 by adding the rounding bias to its bits could carry it into the exponent) -- and leaves the other
    tokens' rows finite."""
    import torch

    T, k, spr, H, I = 64, 2, 4, 512, 256
    rng = np.random.default_rng(11)
    ps = rng.integers(0, spr, size=(T, k)).astype(np.int32)
    x = dev_fp(W.activations(T, H, 21, "bf16")).clone()
    xb = x.view(torch.int16)
    xb[5, 7] = 0x7F81                       # signalling NaN with only low mantissa bits set
    xb[9, :] = -1                           # 0xFFFF: every mantissa bit set, sign set
    w13, w2 = (dev_fp(a) for a in W.expert_weights(spr, H, I, 22, "bf16"))
    pm = api.moe_permute(dev_i32(ps), 0, spr)
    y = ffn_call(api, x, pm["perm_pair"], pm["group_offsets"], k, w13, w2)
    out = api.moe_unpermute(y, pm["pair_row"], torch.full((T, k), 0.5, device="cuda"))
    torch.cuda.synchronize()
    bad = torch.zeros(T, dtype=torch.bool, device="cuda")
    bad[5] = bad[9] = True
    assert torch.isnan(out[bad]).all()
    assert torch.isfinite(out[~bad]).all()
    rows = pm["pair_row"][bad].reshape(-1).long()
    assert torch.isnan(y[rows]).all()
