"""moe_grouped_ffn_static_ws (the entry point for callers that cannot allocate) against moe_grouped_ffn:
same kernels on the library's built-in workspace, so the outputs must be bit-identical; two calls in a row,
the second on a smaller input (all calls on one GPU share the built-in array)."""
import numpy as np
import pytest

from paper_2512_09277_amd import workloads as W

pytestmark = pytest.mark.gpu


def _case(api, T, k, spr, H, I, seed, dtype="bf16"):
    import torch

    rng = np.random.default_rng(seed)
    ps = rng.integers(-1, spr, size=(T, k)).astype(np.int32)
    ps[: T // 3] = 0                                            # one group much larger than the others
    conv = (lambda a: torch.from_numpy(np.ascontiguousarray(a)).view(torch.bfloat16).cuda()) if dtype == "bf16" \
        else (lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda())
    x = conv(W.activations(T, H, seed + 1, dtype))
    w13, w2 = (conv(a) for a in W.expert_weights(spr, H, I, seed + 2, dtype))
    pm = api.moe_permute(torch.from_numpy(ps).cuda(), 0, spr)
    want = torch.full((T * k, H), float("nan"), dtype=x.dtype, device="cuda")
    api.moe_grouped_ffn(x, pm["perm_pair"], pm["group_offsets"], k, w13, w2, y_perm=want)
    got = torch.full((T * k, H), float("nan"), dtype=x.dtype, device="cuda")
    api.moe_grouped_ffn_static_ws(x, pm["perm_pair"], pm["group_offsets"], k, w13, w2, got)
    torch.cuda.synchronize()
    n = int(pm["n_pairs"].item())
    assert n > 0 and not torch.isnan(want[:n].float()).any()
    assert torch.equal(got[:n].view(torch.int16 if dtype == "bf16" else torch.int32),
                       want[:n].view(torch.int16 if dtype == "bf16" else torch.int32)), (T, k, spr, H, I, dtype)
    assert torch.isnan(got[n:].float()).all()                   # rows past n_pairs are never written


def test_static_workspace_matches_the_caller_workspace():
    import torch

    assert torch.cuda.is_available()
    from paper_2512_09277_amd import api

    api.load()
    print("static ws: large call", flush=True)
    _case(api, 700, 4, 6, 2048, 1024, 900)                      # 11 MB of intermediate activations, several tiles
    print("static ws: smaller call", flush=True)
    _case(api, 90, 2, 5, 512, 256, 910)                         # smaller, right after: stale contents must not matter
    print("static ws: fp32 general path", flush=True)
    _case(api, 33, 2, 3, 200, 72, 920, dtype="f32")
    # beyond the built-in buffer: refused on the host
    big = torch.empty((1025, 7168), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(api.MetroError) as e:
        api._check(api.load().moe_grouped_ffn_static_ws(big.data_ptr(), big.data_ptr(), big.data_ptr(), 1025, 8, 36,
                                                        7168, 2048, api.DTYPE_BF16, big.data_ptr(), 7168,
                                                        big.data_ptr(), 2048, big.data_ptr(), None))
    assert e.value.status == api.ERR_TOO_LARGE
