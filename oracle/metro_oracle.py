"""ctypes front end of the CPU oracle (metro_oracle.c) -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this.
It shares nothing with the HIP library: it neither imports the product package nor is
imported by it.  `build()` compiles the C file with gcc; the functions below marshal
numpy arrays and call it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "metro_oracle.c")
_LIB = os.path.join(_HERE, "libmetro_oracle.so")
_lib = None

OK, BAD_ID, NO_REPLICA, BAD_ARG, TOO_LARGE = 0, -1, -2, -3, -4


class OracleError(RuntimeError):
    def __init__(self, code: int):
        super().__init__(f"oracle status {code}")
        self.code = code


def build(force: bool = False) -> str:
    """Compile the oracle (gcc -O2 -fopenmp).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-std=c11", "-Wall", "-Wextra", "-shared", "-fPIC",
                               _SRC, "-o", _LIB, "-lm"])
        if force:   # the sanitizer driver is built and run by tests/test_oracle_sanitize.py; here only "does it compile"
            subprocess.check_call(["gcc", "-O1", "-std=gnu11", "-Wall", "-Wextra", "-c",
                                   os.path.join(_HERE, "sanitize_check.c"), "-o", os.path.join(_HERE, "sanitize_check.o")])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _check(rc: int) -> int:
    if rc < 0:
        raise OracleError(rc)
    return rc


def num_threads() -> int:
    """Threads the FFN oracle's row loop runs on (OpenMP)."""
    return int(_load().oracle_num_threads())


def count(ids: np.ndarray, N: int) -> np.ndarray:
    ids = _i32(ids).reshape(-1)
    cnt = np.empty(N, np.int32)
    _check(_load().oracle_count(_p(ids), ctypes.c_int64(ids.size), N, _p(cnt)))
    return cnt


def route_metro(ids: np.ndarray, slot_to_expert: np.ndarray, N: int, G: int, spr: int) -> dict:
    """ids[T,k] -> dict(pair_slot[T,k], expert_slot[N], rank_active[G], rank_bitmap[G], inspected)."""
    ids = _i32(ids)
    T, k = ids.shape
    s2e = _i32(slot_to_expert)
    assert s2e.size == G * spr
    pair_slot = np.empty((T, k), np.int32)
    expert_slot = np.empty(N, np.int32)
    rank_active = np.empty(G, np.int32)
    rank_bitmap = np.empty(G, np.uint64)
    inspected = ctypes.c_int64(0)
    _check(_load().oracle_route_metro(_p(ids), T, k, _p(s2e), N, G, spr, _p(pair_slot), _p(expert_slot),
                                      _p(rank_active), _p(rank_bitmap), ctypes.byref(inspected)))
    return dict(pair_slot=pair_slot, expert_slot=expert_slot, rank_active=rank_active,
                rank_bitmap=rank_bitmap, inspected=inspected.value)


def route_token_balanced(ids: np.ndarray, slot_to_expert: np.ndarray, N: int, G: int, spr: int) -> dict:
    ids = _i32(ids)
    T, k = ids.shape
    s2e = _i32(slot_to_expert)
    assert s2e.size == G * spr
    pair_slot = np.empty((T, k), np.int32)
    rank_active = np.empty(G, np.int32)
    rank_bitmap = np.empty(G, np.uint64)
    _check(_load().oracle_route_token_balanced(_p(ids), T, k, _p(s2e), N, G, spr, _p(pair_slot),
                                               _p(rank_active), _p(rank_bitmap)))
    return dict(pair_slot=pair_slot, rank_active=rank_active, rank_bitmap=rank_bitmap)


def bruteforce_opt(cnt: np.ndarray, slot_to_expert: np.ndarray, N: int, G: int, spr: int,
                   max_assignments: int = 1 << 22) -> int:
    cnt, s2e = _i32(cnt), _i32(slot_to_expert)
    return _check(_load().oracle_bruteforce_opt(_p(cnt), _p(s2e), N, G, spr, ctypes.c_int64(max_assignments)))


def matching_opt(cnt: np.ndarray, slot_to_expert: np.ndarray, N: int, G: int, spr: int) -> int:
    cnt, s2e = _i32(cnt), _i32(slot_to_expert)
    return _check(_load().oracle_matching_opt(_p(cnt), _p(s2e), N, G, spr))


def permute(pair_slot: np.ndarray, rank: int, spr: int) -> dict:
    """pair_slot[T,k] -> dict(group_offsets[spr+1], perm_pair[n], pair_row[T,k], n_pairs)."""
    ps = _i32(pair_slot)
    T, k = ps.shape
    group_offsets = np.empty(spr + 1, np.int32)
    perm_pair = np.full(T * k, -1, np.int32)
    pair_row = np.empty((T, k), np.int32)
    n = ctypes.c_int32(0)
    _check(_load().oracle_permute(_p(ps), T, k, rank, spr, _p(group_offsets), _p(perm_pair), _p(pair_row),
                                  ctypes.byref(n)))
    return dict(group_offsets=group_offsets, perm_pair=perm_pair[:n.value].copy(), pair_row=pair_row,
                n_pairs=n.value)


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.uint16:
        return 1
    raise TypeError("oracle FFN inputs are float32 or uint16 (bfloat16 bits)")


def ffn(x: np.ndarray, perm_pair: np.ndarray, group_offsets: np.ndarray, k: int, w13: np.ndarray,
        w2: np.ndarray, rows: Optional[Sequence[int]] = None, want_act: bool = False):
    """x[T,H], w13[spr,2I,H], w2[spr,H,I] (float32, or uint16 bfloat16 bits) -> y[n_rows,H] float64
    (and act[n_rows,I] when want_act).  rows=None: every row of the rank's lists."""
    x = np.ascontiguousarray(x)
    w13 = np.ascontiguousarray(w13)
    w2 = np.ascontiguousarray(w2)
    code = _dtype_code(x)
    assert _dtype_code(w13) == code and _dtype_code(w2) == code
    spr, two_i, H = w13.shape
    I = two_i // 2
    assert w2.shape == (spr, H, I) and x.shape[1] == H
    perm_pair, group_offsets = _i32(perm_pair), _i32(group_offsets)
    assert group_offsets.size == spr + 1
    if rows is None:
        rows_arr, n_rows = None, int(group_offsets[spr])
    else:
        rows_arr = _i32(rows)
        n_rows = rows_arr.size
    y = np.empty((n_rows, H), np.float64)
    act = np.empty((n_rows, I), np.float64) if want_act else None
    _check(_load().oracle_ffn(_p(x), code, _p(perm_pair), _p(group_offsets), k, spr, H, I, _p(w13), _p(w2),
                              _p(rows_arr), n_rows, _p(act), _p(y)))
    return (y, act) if want_act else y


def unpermute(y_perm: np.ndarray, pair_row: np.ndarray, topk_w: np.ndarray) -> np.ndarray:
    """y_perm[n,H] float64, pair_row[T,k], topk_w[T,k] float32 -> out[T,H] float64."""
    y = np.ascontiguousarray(y_perm, dtype=np.float64)
    pr = _i32(pair_row)
    w = np.ascontiguousarray(topk_w, dtype=np.float32)
    T, k = pr.shape
    H = y.shape[1]
    out = np.empty((T, H), np.float64)
    _check(_load().oracle_unpermute(_p(y), _p(pr), _p(w), T, k, H, _p(out)))
    return out


def gate_topk(x: np.ndarray, w_gate: np.ndarray, k: int, want_logits: bool = False) -> dict:
    """x[T,H], w_gate[N,H] (float32, or uint16 bfloat16 bits) -> ids[T,k] int32 (descending logit, ties
    to the lower id), w[T,k] float64 (softmax over the selected logits), cnt[N] int32 (pairs per expert);
    logits[T,N] float64 when want_logits."""
    x = np.ascontiguousarray(x)
    w_gate = np.ascontiguousarray(w_gate)
    code = _dtype_code(x)
    assert _dtype_code(w_gate) == code and x.shape[1] == w_gate.shape[1]
    T, H = x.shape
    N = w_gate.shape[0]
    ids = np.empty((T, k), np.int32)
    w = np.empty((T, k), np.float64)
    cnt = np.empty(N, np.int32)
    logits = np.empty((T, N), np.float64) if want_logits else None
    _check(_load().oracle_gate_topk(_p(x), _p(w_gate), code, T, H, N, k, _p(ids), _p(w), _p(logits), _p(cnt)))
    out = dict(ids=ids, w=w, cnt=cnt)
    if want_logits:
        out["logits"] = logits
    return out
