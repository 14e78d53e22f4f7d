"""Pins of the routing oracle against what the paper and the mathematics fix.

Nothing here compares the oracle with itself or with the HIP path: expected values are
the paper's statements (Sec. 3.2 toy, eqs. (1)-(4), Lemma 1, Sec. 4.2, Sec. 6.1), closed
forms, hand-worked executions of Alg. 1 (tests/golden) and exhaustive enumeration.
"""
import math
import os

import numpy as np
import pytest

from paper_2512_09277_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def popcount(v) -> int:
    return bin(int(v)).count("1")


def hosts(s2e, N, G, spr):
    """A[e] = set of ranks hosting e, straight from the placement."""
    A = [set() for _ in range(N)]
    for s, e in enumerate(s2e):
        if e >= 0:
            A[e].add(s // spr)
    return A


def check_feasible(ids, s2e, G, spr, out, one_replica_per_expert):
    """Eqs. (2)-(4) of Sec. 4.1: no pair dropped, every pair on a slot that holds its expert,
    a replica counts as activated iff it receives a pair; Lemma 1 for METRO."""
    ps = out["pair_slot"]
    assert ps.shape == ids.shape
    S = G * spr
    for p, e in enumerate(ids.reshape(-1)):
        s = ps.reshape(-1)[p]
        if e < 0:
            assert s == -1
            continue
        assert 0 <= s < S and s2e[s] == e
    used = {}
    for e, s in zip(ids.reshape(-1), ps.reshape(-1)):
        if e >= 0:
            used.setdefault(int(e), set()).add(int(s))
    if one_replica_per_expert:
        assert all(len(v) == 1 for v in used.values())
    all_slots = set().union(*used.values()) if used else set()
    for g in range(G):
        mine = {s - g * spr for s in all_slots if s // spr == g}
        assert out["rank_bitmap"][g] == sum(1 << l for l in mine)
        assert out["rank_active"][g] == len(mine) == popcount(out["rank_bitmap"][g])
    return used


def random_instance(rng, N, G, spr, T, k, p_empty=0.0):
    """Random placement where every expert has >= 1 replica and no rank hosts one twice."""
    S = G * spr
    assert S >= N
    while True:
        s2e = np.full(S, -1, np.int32)
        order = rng.permutation(S)
        s2e[order[:N]] = rng.permutation(N)
        for s in order[N:]:
            if rng.random() < p_empty:
                continue
            g = s // spr
            here = set(s2e[g * spr:(g + 1) * spr].tolist())
            cand = [e for e in range(N) if e not in here]
            if cand:
                s2e[s] = rng.choice(cand)
        break
    ids = np.stack([rng.permutation(N)[:k] for _ in range(T)]).astype(np.int32)
    return s2e, ids


# ----------------------------------------------------------------------------- P5: the paper's toy
def test_fig4_toy(oracle):
    kv = {}
    for line in open(os.path.join(GOLDEN, "fig4_toy.txt")):
        if line.strip() and not line.startswith("#"):
            a, b = line.split()
            kv[a] = int(b)
    G, N, k, spr = kv["G"], kv["N"], kv["k"], kv["spr"]
    s2e = np.full(G * spr, -1, np.int32)
    for j in range(N):
        s2e[j * spr + 0] = j                      # expert j on rank j ...
        s2e[((j + 1) % G) * spr + 1] = j          # ... and on rank j+1
    ids = np.repeat(np.arange(N, dtype=np.int32), 2).reshape(kv["tokens"], k)
    tb = oracle.route_token_balanced(ids, s2e, N, G, spr)
    me = oracle.route_metro(ids, s2e, N, G, spr)
    assert (tb["rank_active"] == kv["activated_per_rank_token_balanced"]).all()
    assert (me["rank_active"] == kv["activated_per_rank_ideal"]).all()
    for out in (tb, me):
        per_rank = np.bincount(out["pair_slot"].reshape(-1) // spr, minlength=G)
        assert (per_rank == kv["tokens_per_rank"]).all()
    cnt = oracle.count(ids, N)
    assert oracle.bruteforce_opt(cnt, s2e, N, G, spr) == kv["activated_per_rank_ideal"]
    assert oracle.matching_opt(cnt, s2e, N, G, spr) == kv["activated_per_rank_ideal"]


# ----------------------------------------------------------------------------- hand-worked Alg. 1
def _golden_cases():
    for line in open(os.path.join(GOLDEN, "alg1_hand_worked.txt")):
        if not line.strip() or line.startswith("#"):
            continue
        f = [x.split() for x in line.split("|")]
        yield (f[0][0], np.array(f[1], np.int32), [int(v) for v in f[2]], np.array(f[3], np.int32),
               np.array(f[4], np.int32), int(f[5][0]), int(f[6][0]))


@pytest.mark.parametrize("case", list(_golden_cases()), ids=lambda c: c[0])
def test_alg1_hand_worked(oracle, case):
    _, s2e, active, expert_slot, rank_active, lam, opt = case
    G, spr = 2, 3
    N = len(expert_slot)
    ids = np.array([[e] for e in active for _ in range(3)], np.int32)      # 3 tokens each, top-1
    out = oracle.route_metro(ids, s2e, N, G, spr)
    assert out["expert_slot"].tolist() == expert_slot.tolist()
    assert out["rank_active"].tolist() == rank_active.tolist()
    assert out["rank_active"].max() == lam
    cnt = oracle.count(ids, N)
    assert oracle.bruteforce_opt(cnt, s2e, N, G, spr) == opt
    assert oracle.matching_opt(cnt, s2e, N, G, spr) == opt
    # order of the pairs in the batch must not matter (only T[i] > 0 enters Alg. 1)
    out2 = oracle.route_metro(ids[::-1].copy(), s2e, N, G, spr)
    assert out2["expert_slot"].tolist() == expert_slot.tolist()


# ----------------------------------------------------------------------------- P1, P2, P3, P7, P9
@pytest.mark.parametrize("seed", range(40))
def test_micro_instances_against_enumeration(oracle, seed):
    rng = np.random.default_rng(1000 + seed)
    N = int(rng.integers(2, 9))
    G = int(rng.integers(1, 5))
    spr = int(rng.integers(math.ceil(N / G), math.ceil(N / G) + 3))
    k = int(rng.integers(1, min(N, 3) + 1))
    T = int(rng.integers(1, 9))
    s2e, ids = random_instance(rng, N, G, spr, T, k, p_empty=0.3)
    if seed % 5 == 0:
        ids[rng.integers(0, T), rng.integers(0, k)] = -1                  # a padded pair
    A = hosts(s2e, N, G, spr)
    cnt = oracle.count(ids, N)
    assert cnt.tolist() == [int((ids == e).sum()) for e in range(N)]
    me = oracle.route_metro(ids, s2e, N, G, spr)
    tb = oracle.route_token_balanced(ids, s2e, N, G, spr)
    check_feasible(ids, s2e, G, spr, me, True)
    used_tb = check_feasible(ids, s2e, G, spr, tb, False)
    active = [e for e in range(N) if cnt[e] > 0]
    assert me["rank_active"].sum() == len(active)
    assert [e for e in range(N) if me["expert_slot"][e] >= 0] == active
    assert me["inspected"] == sum(len(A[e]) for e in active)              # each entry of A once (Sec. 4.3)
    opt = oracle.bruteforce_opt(cnt, s2e, N, G, spr)
    assert opt == oracle.matching_opt(cnt, s2e, N, G, spr)                # Sec. 4.2 solver == enumeration
    assert math.ceil(len(active) / G) <= opt <= spr
    assert opt <= me["rank_active"].max()                                 # greedy never beats the optimum
    assert opt <= tb["rank_active"].max()                                 # Lemma 1
    for e in active:                                                      # even spread, replicas by slot id
        slots = sorted(s for s in range(G * spr) if s2e[s] == e)
        got = tb["pair_slot"][ids == e]
        assert got.tolist() == [slots[q % len(slots)] for q in range(cnt[e])]
        assert len(used_tb[e]) == min(cnt[e], len(slots))


def test_bruteforce_is_exhaustive_independent_check(oracle):
    """Enumerate with itertools here (no oracle code) on a few instances."""
    import itertools

    rng = np.random.default_rng(7)
    for _ in range(10):
        N, G, spr = 6, 3, 4
        s2e, ids = random_instance(rng, N, G, spr, 5, 2, p_empty=0.2)
        A = hosts(s2e, N, G, spr)
        cnt = [int((ids == e).sum()) for e in range(N)]
        active = [e for e in range(N) if cnt[e] > 0]
        best = min(max(np.bincount(choice, minlength=G)) for choice in
                   itertools.product(*[sorted(A[e]) for e in active]))
        assert oracle.bruteforce_opt(np.array(cnt), s2e, N, G, spr) == best


# ----------------------------------------------------------------------------- P4: closed forms
def test_no_replication_is_forced(oracle):
    """1.0x replication: no routing decision exists (Sec. 6.1), both routers are the forced map."""
    rng = np.random.default_rng(3)
    N, G, spr, T, k = 24, 4, 6, 50, 3
    s2e = rng.permutation(N).astype(np.int32)
    ids = np.stack([rng.permutation(N)[:k] for _ in range(T)]).astype(np.int32)
    where = np.empty(N, np.int32)
    where[s2e] = np.arange(N)
    me = oracle.route_metro(ids, s2e, N, G, spr)
    tb = oracle.route_token_balanced(ids, s2e, N, G, spr)
    assert (me["pair_slot"] == where[ids]).all() and (tb["pair_slot"] == where[ids]).all()
    assert (me["rank_active"] == tb["rank_active"]).all()


def test_full_replication_is_round_robin(oracle):
    """Every expert on every rank: greedy deals active experts round-robin, lambda = ceil(active/G)."""
    N, G = 7, 3
    spr = N
    s2e = np.tile(np.arange(N, dtype=np.int32), G)
    ids = np.array([[0, 2], [3, 5], [6, 2], [5, 0]], np.int32)          # active: 0 2 3 5 6
    me = oracle.route_metro(ids, s2e, N, G, spr)
    active = [0, 2, 3, 5, 6]
    for n, e in enumerate(active):
        assert me["expert_slot"][e] == (n % G) * spr + e
    assert me["rank_active"].tolist() == [2, 2, 1]
    assert me["rank_active"].max() == math.ceil(len(active) / G)
    assert oracle.bruteforce_opt(oracle.count(ids, N), s2e, N, G, spr) == 2


def test_duplicate_on_one_rank_collapses(oracle):
    """A is binary (Sec. 4.1): a second copy on the same rank is never a separate replica."""
    s2e = np.array([0, 0, 1, 1, 2, -1], np.int32)                       # G=2, spr=3
    ids = np.array([[0], [0], [0], [1], [1]], np.int32)
    me = oracle.route_metro(ids, s2e, 3, 2, 3)
    tb = oracle.route_token_balanced(ids, s2e, 3, 2, 3)
    assert me["expert_slot"].tolist() == [0, 3, -1]                      # e1: rank 0 has L=1 -> rank 1
    assert tb["pair_slot"].reshape(-1).tolist() == [0, 0, 0, 2, 3]


def test_error_codes(oracle):
    s2e = np.array([0, 1, 2, -1], np.int32)
    with pytest.raises(oracle.OracleError) as ei:
        oracle.route_metro(np.array([[3]], np.int32), s2e, 4, 2, 2)       # expert 3 has no replica
    assert ei.value.code == oracle.NO_REPLICA
    with pytest.raises(oracle.OracleError) as ei:
        oracle.route_token_balanced(np.array([[4]], np.int32), s2e, 4, 2, 2)
    assert ei.value.code == oracle.BAD_ID
    with pytest.raises(oracle.OracleError) as ei:
        oracle.route_metro(np.array([[-2]], np.int32), s2e, 4, 2, 2)
    assert ei.value.code == oracle.BAD_ID


# ----------------------------------------------------------------------------- the configs' shapes
@pytest.mark.parametrize("w", [W.TINY, W.QWEN3_30B, W.QWEN3_235B, W.DSV3, W.DSV3_SWEEP], ids=lambda w: w.name)
def test_config_shapes_invariants(oracle, w):
    for layer in range(min(w.layers, 3)):
        _, s2e, ids = W.routing_inputs(w, layer)
        assert s2e.shape == (w.S,) and ids.shape == (w.T, w.k)
        assert sorted(set(s2e.tolist())) == list(range(w.N))             # every expert placed, no empty slot
        for g in range(w.G):
            here = s2e[g * w.spr:(g + 1) * w.spr]
            assert len(set(here.tolist())) == w.spr                      # no rank hosts an expert twice
        assert all(len(set(row)) == w.k for row in ids.tolist())        # top-k without replacement
        cnt = oracle.count(ids, w.N)
        me = oracle.route_metro(ids, s2e, w.N, w.G, w.spr)
        tb = oracle.route_token_balanced(ids, s2e, w.N, w.G, w.spr)
        check_feasible(ids, s2e, w.G, w.spr, me, True)
        check_feasible(ids, s2e, w.G, w.spr, tb, False)
        opt = oracle.matching_opt(cnt, s2e, w.N, w.G, w.spr)
        n_active = int((cnt > 0).sum())
        assert math.ceil(n_active / w.G) <= opt <= w.spr
        assert opt <= me["rank_active"].max() <= w.spr
        assert opt <= tb["rank_active"].max() <= w.spr
        if w is W.TINY:                                                  # <= 2^4 assignments: enumerate
            assert oracle.bruteforce_opt(cnt, s2e, w.N, w.G, w.spr) == opt
            for T in range(1, 9):
                c8 = oracle.count(ids[:T], w.N)
                assert oracle.bruteforce_opt(c8, s2e, w.N, w.G, w.spr) == oracle.matching_opt(c8, s2e, w.N, w.G, w.spr)


def test_tiny_placement_matches_the_config_text():
    """Tiny: 16 experts, 20 slots, one extra replica for each of the 4 most popular experts."""
    p, s2e, _ = W.routing_inputs(W.TINY)
    rc = np.bincount(s2e, minlength=16)
    top4 = set(np.argsort(-p)[:4].tolist())
    assert set(np.nonzero(rc == 2)[0].tolist()) == top4 and rc.sum() == 20 and rc.min() == 1


# ----------------------------------------------------------------------------- permute
@pytest.mark.parametrize("seed", range(6))
def test_permute_is_a_stable_sort(oracle, seed):
    rng = np.random.default_rng(seed)
    T, k, G, spr = 37, 3, 3, 5
    pair_slot = rng.integers(-1, G * spr, size=(T, k)).astype(np.int32)
    for g in range(G):
        out = oracle.permute(pair_slot, g, spr)
        flat = pair_slot.reshape(-1)
        mine = np.nonzero((flat >= g * spr) & (flat < (g + 1) * spr))[0]
        order = mine[np.argsort(flat[mine], kind="stable")]               # library stable sort
        assert out["n_pairs"] == mine.size
        assert out["perm_pair"].tolist() == order.tolist()
        counts = np.bincount(flat[mine] - g * spr, minlength=spr)
        assert out["group_offsets"].tolist() == np.concatenate([[0], np.cumsum(counts)]).tolist()
        inv = np.full(T * k, -1)
        inv[order] = np.arange(order.size)
        assert out["pair_row"].reshape(-1).tolist() == inv.tolist()


def test_permute_empty_rank(oracle):
    out = oracle.permute(np.full((4, 2), 7, np.int32), 0, 3)
    assert out["n_pairs"] == 0 and out["group_offsets"].tolist() == [0, 0, 0, 0]
    assert (out["pair_row"] == -1).all()
