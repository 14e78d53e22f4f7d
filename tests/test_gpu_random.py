"""Randomised GPU parity: every call of the library on seeded random shapes and placements against the
CPU oracle (routing and token lists bit-exact; FFN, combine and gate within the stated tolerances).
Shapes are drawn so that every kernel variant appears: general and matrix-core FFN paths, 32-, 64- and
128-row tiles, the direct and the LDS-staged gate kernels, N up to 512, G up to 64, padded pairs."""
import numpy as np
import pytest

from paper_2512_09277_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    import torch

    from paper_2512_09277_amd import api as binding

    assert torch.cuda.is_available()
    binding.load()
    return binding


def dev_i(a):
    import torch

    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def dev_fp(a):
    import torch

    t = torch.from_numpy(np.ascontiguousarray(a))
    return (t.view(torch.bfloat16) if a.dtype == np.uint16 else t).cuda()


def random_placement(rng, N, G, spr):
    """Every expert once, extra replicas at random (never twice on a rank), some slots empty."""
    S = G * spr
    s2e = np.full(S, -1, np.int32)
    s2e[rng.permutation(S)[:N]] = np.arange(N)
    for s in np.flatnonzero(s2e < 0):
        if rng.random() < 0.6:
            here = set(s2e[(s // spr) * spr:(s // spr + 1) * spr].tolist())
            cand = [e for e in rng.integers(0, N, size=4).tolist() if e not in here]
            if cand:
                s2e[s] = cand[0]
    return s2e


@pytest.mark.parametrize("seed", [21, 22])
def test_random_routing_and_token_lists(api, oracle, seed):
    rng = np.random.default_rng(seed)
    for it in range(150):
        G = int(rng.choice([1, 2, 3, 8, 16, 33, 64]))
        spr = min(int(rng.integers(1, 65)), 2048 // G)
        S = G * spr
        N = int(rng.integers(1, min(S, 512) + 1))
        k = int(rng.integers(1, min(N, 12) + 1))
        T = int(rng.choice([1, 2, 7, 64, 300, 1031]))
        s2e = random_placement(rng, N, G, spr)
        ids = np.stack([rng.permutation(N)[:k] for _ in range(T)]).astype(np.int32)
        if rng.random() < 0.3:
            ids[rng.random(ids.shape) < 0.1] = -1
        what = f"seed {seed} case {it}: N={N} G={G} spr={spr} k={k} T={T}"
        for fn, ofn in ((api.metro_route, oracle.route_metro),
                        (api.metro_route_token_balanced, oracle.route_token_balanced)):
            out = fn(dev_i(ids).unsqueeze(0), dev_i(s2e).unsqueeze(0), N, G, spr)
            ref = ofn(ids, s2e, N, G, spr)
            assert int(out["err_flag"].item()) == 0, what
            assert np.array_equal(out["pair_slot"][0].cpu().numpy(), ref["pair_slot"]), what
            assert np.array_equal(out["rank_active"][0].cpu().numpy(), ref["rank_active"]), what
        g = int(rng.integers(0, G))
        pm = api.moe_permute(out["pair_slot"][0], g, spr)
        rp = oracle.permute(ref["pair_slot"], g, spr)
        n = rp["n_pairs"]
        assert int(pm["n_pairs"].item()) == n, what
        assert np.array_equal(pm["group_offsets"].cpu().numpy(), rp["group_offsets"]), what
        assert np.array_equal(pm["perm_pair"].cpu().numpy()[:n], rp["perm_pair"]), what
        assert np.array_equal(pm["pair_row"].cpu().numpy(), rp["pair_row"]), what


def test_random_ffn_and_combine(api, oracle):
    import torch

    rng = np.random.default_rng(23)
    for it in range(30):
        H = int(rng.choice([128, 256, 384, 200, 2048]))
        I = int(rng.choice([128, 256, 72, 1024 if H == 2048 else 128]))
        dtype = "bf16" if rng.random() < 0.8 else "f32"
        spr, k, T = int(rng.integers(1, 9)), int(rng.integers(1, 5)), int(rng.choice([1, 5, 64, 130]))
        ps = rng.integers(-1, spr, size=(T, k)).astype(np.int32)
        if rng.random() < 0.3:
            ps[:] = rng.integers(0, spr)                                  # one group holds every pair
        x = W.activations(T, H, 100 + it, dtype)
        w13, w2 = W.expert_weights(spr, H, I, 200 + it, dtype)
        tw = W.gating_weights(T, k, 300 + it)
        pm = api.moe_permute(dev_i(ps), 0, spr)
        rp = oracle.permute(ps, 0, spr)
        n = rp["n_pairs"]
        y = torch.full((T * k, H), float("nan"), dtype=dev_fp(x).dtype, device="cuda")
        api.moe_grouped_ffn(dev_fp(x), pm["perm_pair"], pm["group_offsets"], k, dev_fp(w13), dev_fp(w2), y_perm=y)
        out = api.moe_unpermute(y, pm["pair_row"], torch.from_numpy(tw).cuda())
        if n == 0:
            continue
        what = f"case {it}: H={H} I={I} {dtype} spr={spr} k={k} T={T}"
        tol = 2e-2 if dtype == "bf16" else 1e-5
        ref = oracle.ffn(x, rp["perm_pair"], rp["group_offsets"], k, w13, w2)
        got = y[:n].float().cpu().numpy().astype(np.float64)
        assert np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30) <= tol, what
        want = oracle.unpermute(ref, rp["pair_row"], tw)
        assert np.abs(out.float().cpu().numpy() - want).max() / max(np.abs(want).max(), 1e-30) <= tol, what


@pytest.mark.parametrize("seed", [31, 32, 33])
def test_random_ffn_large_shape(api, oracle, seed):
    """Random group sizes at a shape large enough (H*I >= 4096*2048) for every tile class of the bandwidth-bound
    regime: narrow, one-tile wide and several-tile groups, with one group that may hold most of the rows."""
    import torch

    rng = np.random.default_rng(seed)
    H, I = 4096, 2048
    spr, k, T = int(rng.integers(3, 7)), int(rng.integers(2, 5)), int(rng.choice([200, 450, 700]))
    probs = rng.dirichlet(np.full(spr, 0.4))
    ps = rng.choice(spr, size=(T, k), p=probs).astype(np.int32)
    ps[rng.random((T, k)) < 0.1] = -1
    x = W.activations(T, H, 600 + seed, "bf16")
    w13, w2 = W.expert_weights(spr, H, I, 700 + seed, "bf16")
    tw = W.gating_weights(T, k, 800 + seed)
    pm = api.moe_permute(dev_i(ps), 0, spr)
    rp = oracle.permute(ps, 0, spr)
    n = rp["n_pairs"]
    what = f"seed {seed}: spr={spr} k={k} T={T} groups {np.diff(rp['group_offsets']).tolist()}"
    print(what, flush=True)
    y = torch.full((T * k, H), float("nan"), dtype=torch.bfloat16, device="cuda")
    api.moe_grouped_ffn(dev_fp(x), pm["perm_pair"], pm["group_offsets"], k, dev_fp(w13), dev_fp(w2), y_perm=y)
    out = api.moe_unpermute(y, pm["pair_row"], torch.from_numpy(tw).cuda())
    ref = oracle.ffn(x, rp["perm_pair"], rp["group_offsets"], k, w13, w2)
    got = y[:n].float().cpu().numpy().astype(np.float64)
    row_err = np.abs(got - ref).max(axis=1) / np.abs(ref).max(axis=1)
    assert row_err.max() <= 2e-2, f"{what}: row {int(row_err.argmax())} off by {row_err.max()}"
    want = oracle.unpermute(ref, rp["pair_row"], tw)
    assert np.abs(out.float().cpu().numpy() - want).max() / np.abs(want).max() <= 1e-2, what


def test_random_gate_topk(api, oracle):
    rng = np.random.default_rng(24)
    for it in range(30):
        N = int(rng.choice([7, 16, 64, 128, 192, 256, 512]))
        H = int(rng.choice([32, 96, 200, 256, 1024]))
        T = int(rng.choice([1, 17, 64, 300, 1100]))
        k = int(rng.integers(1, min(N, 12) + 1))
        dtype = "bf16" if rng.random() < 0.8 else "f32"
        what = f"case {it}: N={N} H={H} T={T} k={k} {dtype}"
        x, wg = W.activations(T, H, 400 + it, dtype), W.gate_weights(N, H, 500 + it, dtype)
        ref = oracle.gate_topk(x, wg, k, want_logits=True)
        got = api.moe_gate_topk(dev_fp(x), dev_fp(wg), k)
        ids, L = got["topk_ids"].cpu().numpy(), ref["logits"]
        eps = 1e-3 if dtype == "bf16" else 1e-4                           # near-tie margin of the fp32 logits
        sel = np.take_along_axis(L, ids.astype(np.int64), axis=1)
        ref_sel = np.take_along_axis(L, ref["ids"].astype(np.int64), axis=1)
        assert (np.abs(sel - ref_sel)[ids != ref["ids"]] <= eps).all(), what
        assert np.array_equal(got["expert_count"].cpu().numpy(), np.bincount(ids.reshape(-1), minlength=N)), what
        z = np.exp(sel - sel.max(axis=1, keepdims=True))
        assert np.abs(got["topk_w"].cpu().numpy() - z / z.sum(axis=1, keepdims=True)).max() <= 2e-3, what
