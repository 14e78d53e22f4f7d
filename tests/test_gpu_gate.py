"""GPU parity of moe_gate_topk (router logits + top-k + gating weights) against the CPU oracle.

The ids are decided by floating-point logits: the kernel accumulates in fp32, the oracle in fp64, so
two experts whose logits are closer than the fp32 accumulation error may legitimately swap.  What is
unique is compared exactly (every position whose neighbours are further apart than EPS, the expert
counts against the kernel's own ids), the rest is checked for validity (a swapped-in expert's oracle
logit is within EPS of the one it replaced; nothing above the cut by more than EPS is missing)."""
import numpy as np
import pytest

from paper_2512_09277_amd import workloads as W

pytestmark = pytest.mark.gpu

EPS = {"bf16": 1e-3, "f32": 1e-4}        # H fp32 additions of O(1) partial sums: <= H * 2^-24 ~ 4e-4 at H = 7168
W_TOL = {"bf16": 2e-3, "f32": 1e-4}


@pytest.fixture(scope="module")
def api():
    import torch

    from paper_2512_09277_amd import api as binding

    assert torch.cuda.is_available()
    binding.load()
    return binding


def dev(a):
    import torch

    t = torch.from_numpy(np.ascontiguousarray(a))
    return (t.view(torch.bfloat16) if a.dtype == np.uint16 else t).cuda()


def check(got, ref, k, N, dtype):
    ids, w, cnt = got["topk_ids"].cpu().numpy(), got["topk_w"].cpu().numpy(), got["expert_count"].cpu().numpy()
    L, eps = ref["logits"], EPS[dtype]
    T = ids.shape[0]
    assert ids.min() >= 0 and ids.max() < N
    assert all(len(set(row)) == k for row in ids.tolist())
    assert np.array_equal(cnt, np.bincount(ids.reshape(-1), minlength=N))
    sel = np.take_along_axis(L, ids.astype(np.int64), axis=1)              # oracle logits of the kernel's picks
    ref_sel = np.take_along_axis(L, ref["ids"].astype(np.int64), axis=1)
    differs = ids != ref["ids"]
    assert (np.abs(sel - ref_sel)[differs] <= eps).all(), "a pick differs from the oracle's by more than a near-tie"
    assert (np.diff(sel, axis=1) <= eps).all()                              # descending up to near-ties
    kth = ref_sel[:, -1:]
    assert (sel >= kth - eps).all()
    above = L > kth + eps
    picked = np.zeros_like(above)
    np.put_along_axis(picked, ids.astype(np.int64), True, axis=1)
    assert not (above & ~picked).any(), "an expert clearly above the cut was not selected"
    z = np.exp(sel - sel.max(axis=1, keepdims=True))
    assert np.abs(w - z / z.sum(axis=1, keepdims=True)).max() <= W_TOL[dtype]
    return float(differs.mean()), T


CASES = [  # T, H, N, k, dtype, padded rows
    (32, 256, 16, 2, "f32", 0),          # Tiny config's shape (general kernel)
    (32, 256, 16, 2, "bf16", 0),         # general kernel, bf16 storage
    (5, 64, 64, 4, "bf16", 0),           # one block per wave, one token tile with a ragged tail
    (37, 2048, 128, 8, "bf16", 0),       # Qwen3-shaped router, ragged tail
    (256, 2048, 128, 8, "bf16", 0),
    (1024, 7168, 256, 8, "bf16", 0),     # DeepSeek-V3-shaped router at the benchmark's batch
    (1024, 7168, 256, 8, "bf16", 64),    # the same with padded weight rows
    (1100, 512, 128, 8, "bf16", 0),      # LDS-staged kernel (T >= 1024), ragged last token tile
    (1030, 128, 384, 5, "bf16", 64),     # LDS-staged kernel, one K chunk of two steps, three expert tiles, padded rows
    (19, 96, 512, 6, "bf16", 0),         # direct kernel, eight expert tiles
    (9, 200, 192, 3, "bf16", 0),         # H and N the matrix-core kernel does not take
    (3, 128, 64, 64, "bf16", 0),         # k = N = 64: everything selected
]


@pytest.mark.parametrize("T,H,N,k,dtype,pad", CASES)
def test_gate_topk_matches_oracle(api, oracle, T, H, N, k, dtype, pad):
    import torch

    print(f"gate T={T} H={H} N={N} k={k} {dtype} pad={pad}", flush=True)
    x, wg = W.activations(T, H, 51, dtype), W.gate_weights(N, H, 52, dtype)
    ref = oracle.gate_topk(x, wg, k, want_logits=True)
    d_wg = dev(wg)
    if pad:
        buf = torch.full((N, H + pad), 3.0, dtype=d_wg.dtype, device="cuda")
        buf[:, :H].copy_(d_wg)
        d_wg = buf[:, :H]
    got = api.moe_gate_topk(dev(x), d_wg, k)
    torch.cuda.synchronize()
    frac, _ = check(got, ref, k, N, dtype)
    assert frac <= 0.02, f"{frac:.3%} of the picks are near-tie swaps: more than rounding explains"
    again = api.moe_gate_topk(dev(x), d_wg, k)
    torch.cuda.synchronize()
    for key in ("topk_ids", "topk_w", "expert_count"):
        assert torch.equal(got[key], again[key]), "two runs differ"


def test_exact_ties_go_to_the_lower_id(api, oracle):
    """Duplicate router rows give bit-identical logits on both sides: the tie rule decides."""
    T, H, N, k = 20, 64, 64, 8
    x = W.activations(T, H, 61, "bf16")
    wg = W.gate_weights(N, H, 62, "bf16")
    wg[1::2] = wg[0::2]                                        # experts 2i and 2i+1 are identical
    ref = oracle.gate_topk(x, wg, k, want_logits=True)
    got = api.moe_gate_topk(dev(x), dev(wg), k)
    ids = got["topk_ids"].cpu().numpy()
    assert (ids[:, 0::2] % 2 == 0).all() and (ids[:, 1::2] == ids[:, 0::2] + 1).all()
    check(got, ref, k, N, "bf16")


def test_gate_feeds_the_routing_solve(api, oracle):
    """Gate -> metro_route on the device equals the oracle's routing of the same ids."""
    import torch

    w = W.QWEN3_30B
    _, s2e, _ = W.routing_inputs(w)
    x, wg = W.activations(w.T, w.H, 71, "bf16"), W.gate_weights(w.N, w.H, 72, "bf16")
    got = api.moe_gate_topk(dev(x), dev(wg), w.k)
    ids = got["topk_ids"]
    out = api.metro_route(ids.unsqueeze(0), torch.from_numpy(s2e).cuda().unsqueeze(0), w.N, w.G, w.spr)
    ref = oracle.route_metro(ids.cpu().numpy(), s2e, w.N, w.G, w.spr)
    assert np.array_equal(out["pair_slot"][0].cpu().numpy(), ref["pair_slot"])
    assert np.array_equal(got["expert_count"].cpu().numpy(), oracle.count(ids.cpu().numpy(), w.N))


def test_empty_batch_zeroes_the_counts(api):
    """T == 0: no id or weight is written, and expert_count -- which a caller reuses across batches -- is zero."""
    import torch

    H, N, k = 64, 64, 4
    out = dict(topk_ids=torch.empty((0, k), dtype=torch.int32, device="cuda"),
               topk_w=torch.empty((0, k), dtype=torch.float32, device="cuda"),
               expert_count=torch.full((N,), 7, dtype=torch.int32, device="cuda"))
    x = torch.empty((0, H), dtype=torch.bfloat16, device="cuda")
    api.moe_gate_topk(x, dev(W.gate_weights(N, H, 81, "bf16")), k, out=out)
    torch.cuda.synchronize()
    assert (out["expert_count"] == 0).all()


@pytest.mark.parametrize("T,n_real", [(256, 200), (1024, 1000), (64, 0), (32, 32), (16, 77)])
def test_padded_batch(api, oracle, T, n_real):
    """A batch padded to a fixed size (Sec. 5): tokens past *n_valid get ids -1 and weight 0 and count nothing;
    the real tokens are exactly what the unpadded call gives.  n_valid lives on the device and is clamped to T."""
    import torch

    H, N, k = 512, 128, 8
    x, wg = W.activations(T, H, 91, "bf16"), W.gate_weights(N, H, 92, "bf16")
    full = api.moe_gate_topk(dev(x), dev(wg), k)
    nv = torch.tensor([n_real], dtype=torch.int32, device="cuda")
    got = api.moe_gate_topk(dev(x), dev(wg), k, n_valid=nv)
    torch.cuda.synchronize()
    n = min(n_real, T)
    assert torch.equal(got["topk_ids"][:n], full["topk_ids"][:n]) and torch.equal(got["topk_w"][:n], full["topk_w"][:n])
    assert (got["topk_ids"][n:] == -1).all() and (got["topk_w"][n:] == 0).all()
    ids = got["topk_ids"][:n].cpu().numpy().reshape(-1)
    assert np.array_equal(got["expert_count"].cpu().numpy(), np.bincount(ids, minlength=N))
    ref = oracle.gate_topk(x[:n], wg, k, want_logits=True) if n else None
    if n:
        check(dict(topk_ids=got["topk_ids"][:n], topk_w=got["topk_w"][:n], expert_count=got["expert_count"]), ref, k, N,
              "bf16")
