"""The whole layer -- gate + top-k, METRO routing, token lists, grouped FFN, combine -- captured in ONE HIP graph
for a batch padded to a power of two (Sec. 5: the routing kernel lives inside the captured decode graphs and
batches are padded to fixed sizes), replayed on different inputs and real-token counts, every replay compared
with the CPU oracle: routing and token lists bit for bit on the ids the gate produced, FFN and combined
output at the bf16 tolerance.  No memset node is captured: the library clears nothing with memsets, and the test
fills its inputs outside the graph."""
import numpy as np
import pytest

from paper_2512_09277_amd import workloads as W

pytestmark = pytest.mark.gpu

BF16_TOL = 2e-2


def dev(a):
    import torch

    t = torch.from_numpy(np.ascontiguousarray(a))
    return (t.view(torch.bfloat16) if a.dtype == np.uint16 else t).cuda()


def host_bits(t):
    import torch

    return t.contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


@pytest.mark.parametrize("routing", ["metro", "token_balanced"])
def test_captured_layer_replays_match_the_oracle(oracle, routing):
    import torch

    from paper_2512_09277_amd import api

    api.load()
    w = W.QWEN3_30B                                              # N=128, k=8, G=8, 18 slots per rank
    T, H, I, g = 256, 512, 256, 3                                # T: the padded batch, a power of two
    _, s2e, _ = W.routing_inputs(w)
    wg = W.gate_weights(w.N, H, 5, "bf16")
    w13, w2 = W.expert_weights(w.N, H, I, 6, "bf16")
    s13, s2 = W.rank_share(w13, s2e, g, w.spr), W.rank_share(w2, s2e, g, w.spr)
    d_s2e = torch.from_numpy(s2e).cuda().unsqueeze(0)
    d_wg, d_13, d_2 = dev(wg), dev(s13), dev(s2)
    route = api.metro_route if routing == "metro" else api.metro_route_token_balanced
    route_ref = oracle.route_metro if routing == "metro" else oracle.route_token_balanced

    # static buffers of the captured graph
    x = torch.zeros((T, H), dtype=torch.bfloat16, device="cuda")
    n_valid = torch.zeros((1,), dtype=torch.int32, device="cuda")
    gate_out = dict(topk_ids=torch.empty((T, w.k), dtype=torch.int32, device="cuda"),
                    topk_w=torch.empty((T, w.k), dtype=torch.float32, device="cuda"),
                    expert_count=torch.empty((w.N,), dtype=torch.int32, device="cuda"))
    gate_ws = torch.empty((api.load().moe_gate_topk_workspace_bytes(T, H, w.N, api.DTYPE_BF16),), dtype=torch.uint8,
                          device="cuda")
    rb = api.route_buffers(1, T, w.k, w.N, w.G, "cuda")
    pb = api.permute_buffers(T, w.k, w.spr, "cuda")
    y = torch.empty((T * w.k, H), dtype=torch.bfloat16, device="cuda")
    ffn_ws = torch.empty((api.moe_grouped_ffn_workspace_bytes(T, w.k, w.spr, H, I, torch.bfloat16),), dtype=torch.uint8,
                         device="cuda")
    out = torch.empty((T, H), dtype=torch.bfloat16, device="cuda")

    def layer():
        api.moe_gate_topk(x, d_wg, w.k, out=gate_out, ws=gate_ws, n_valid=n_valid)
        route(gate_out["topk_ids"].unsqueeze(0), d_s2e, w.N, w.G, w.spr, out=rb)
        api.moe_permute(rb["pair_slot"][0], g, w.spr, out=pb)
        api.moe_grouped_ffn(x, pb["perm_pair"], pb["group_offsets"], w.k, d_13, d_2, y_perm=y, ws=ffn_ws)
        api.moe_unpermute(y, pb["pair_row"], gate_out["topk_w"], out=out)

    x.copy_(dev(W.activations(T, H, 100, "bf16")))
    n_valid.fill_(T)
    layer()                                                      # eager once: loads the kernels before the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            layer()
    torch.cuda.synchronize()

    for replay, (seed, n_real) in enumerate([(101, 200), (102, 256), (103, 131), (101, 200)]):
        print(f"graph replay {replay}: {routing}, seed {seed}, {n_real} real tokens of {T}", flush=True)
        hx = W.activations(T, H, seed, "bf16")
        x.copy_(dev(hx))                                         # eager work between the replays
        n_valid.fill_(n_real)
        y.fill_(float("nan"))
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ids = gate_out["topk_ids"].cpu().numpy()
        tw = gate_out["topk_w"].cpu().numpy()
        # gate: padded rows, validity of the real rows (near-ties may swap, as in the gate's own tests)
        assert (ids[n_real:] == -1).all() and (tw[n_real:] == 0).all()
        ref_gate = oracle.gate_topk(hx[:n_real], wg, w.k, want_logits=True)
        L = ref_gate["logits"]
        sel = np.take_along_axis(L, ids[:n_real].astype(np.int64), axis=1)
        ref_sel = np.take_along_axis(L, ref_gate["ids"].astype(np.int64), axis=1)
        assert (np.abs(sel - ref_sel)[ids[:n_real] != ref_gate["ids"]] <= 1e-3).all()
        assert np.array_equal(gate_out["expert_count"].cpu().numpy(), oracle.count(ids, w.N))
        # routing and token lists: bit for bit on the ids the gate produced
        ref_route = route_ref(ids, s2e, w.N, w.G, w.spr)
        assert int(rb["err_flag"].item()) == 0
        assert np.array_equal(rb["pair_slot"][0].cpu().numpy(), ref_route["pair_slot"])
        assert np.array_equal(rb["rank_active"][0].cpu().numpy(), ref_route["rank_active"])
        ref_pm = oracle.permute(ref_route["pair_slot"], g, w.spr)
        n = ref_pm["n_pairs"]
        assert int(pb["n_pairs"].item()) == n and n > 0
        assert np.array_equal(pb["group_offsets"].cpu().numpy(), ref_pm["group_offsets"])
        assert np.array_equal(pb["perm_pair"].cpu().numpy()[:n], ref_pm["perm_pair"])
        assert np.array_equal(pb["pair_row"].cpu().numpy(), ref_pm["pair_row"])
        assert (ref_pm["pair_row"][n_real:] == -1).all()         # padded tokens reach no expert
        # FFN and combine
        ref_y = oracle.ffn(hx, ref_pm["perm_pair"], ref_pm["group_offsets"], w.k, s13, s2)
        got_y = y[:n].float().cpu().numpy().astype(np.float64)
        err = np.abs(got_y - ref_y).max() / np.abs(ref_y).max()
        assert err <= BF16_TOL, f"replay {replay}: y_perm off by {err}"
        ref_out = oracle.unpermute(ref_y, ref_pm["pair_row"], tw)
        got_out = out.float().cpu().numpy().astype(np.float64)
        err = np.abs(got_out - ref_out).max() / np.abs(ref_out).max()
        assert err <= BF16_TOL, f"replay {replay}: out off by {err}"
        assert (got_out[n_real:] == 0).all()                     # padded rows of the output are zero
        # the same inputs run eagerly give the same bits as the replay
        keep = {k: v.clone() for k, v in dict(out=out, y=y[:n], ps=rb["pair_slot"], ids=gate_out["topk_ids"]).items()}
        layer()
        torch.cuda.synchronize()
        assert torch.equal(keep["ids"], gate_out["topk_ids"]) and torch.equal(keep["ps"], rb["pair_slot"])
        assert torch.equal(keep["y"].view(torch.int16), y[:n].view(torch.int16))
        assert torch.equal(keep["out"].view(torch.int16), out.view(torch.int16))
