"""Thin Python binding of libmetro.so (see include/metro.h): argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI; torch supplies device
memory and the current stream.  There is no CPU fallback: if the library has not been
built, loading fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmetro.so")
_lib = None

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP, ERR_TOO_LARGE = 0, -1, -2, -3, -4, -5
FLAG_BAD_ID, FLAG_NO_REPLICA, FLAG_BAD_PLACEMENT = 1, 2, 4
DTYPE_F32, DTYPE_BF16 = 0, 1

EXPORTS = ("metro_status_string", "metro_route", "metro_route_token_balanced", "moe_permute",
           "moe_grouped_ffn_workspace_bytes", "moe_grouped_ffn", "moe_grouped_ffn_gate_up",
           "moe_grouped_ffn_down", "moe_unpermute", "moe_gate_topk_workspace_bytes", "moe_gate_topk",
           "moe_grouped_ffn_static_ws_bytes", "moe_grouped_ffn_static_ws", "metro_route_permute",
           "metro_route_token_balanced_permute")


class MetroError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"libmetro: {text} (status {status})")
        self.status = status


def load() -> ctypes.CDLL:
    """Load the in-tree library; raises if it was not built (python -m paper_2512_09277_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2512_09277_amd.build` "
                               "(there is no fallback path)")
        lib = ctypes.CDLL(LIB_PATH)
        vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        lib.metro_status_string.restype = ctypes.c_char_p
        lib.metro_status_string.argtypes = [ci]
        lib.metro_route.restype = ci
        lib.metro_route.argtypes = [vp, vp, ci, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp]
        lib.metro_route_token_balanced.restype = ci
        lib.metro_route_token_balanced.argtypes = [vp, vp, ci, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp]
        lib.metro_route_permute.restype = ci
        lib.metro_route_permute.argtypes = [vp, vp, ci, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        lib.metro_route_token_balanced_permute.restype = ci
        lib.metro_route_token_balanced_permute.argtypes = [vp, vp, ci, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        lib.moe_permute.restype = ci
        lib.moe_permute.argtypes = [vp, ci, ci, ci, ci, vp, vp, vp, vp, vp]
        lib.moe_grouped_ffn_workspace_bytes.restype = sz
        lib.moe_grouped_ffn_workspace_bytes.argtypes = [ci, ci, ci, ci, ci, ci]
        lib.moe_grouped_ffn.restype = ci
        lib.moe_grouped_ffn.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, ci, vp, ci, vp, ci, vp, vp, sz, vp]
        lib.moe_grouped_ffn_gate_up.restype = ci
        lib.moe_grouped_ffn_gate_up.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, ci, vp, ci, vp, sz, vp]
        lib.moe_grouped_ffn_down.restype = ci
        lib.moe_grouped_ffn_down.argtypes = [vp, ci, ci, ci, ci, ci, ci, vp, ci, vp, vp, sz, vp]
        lib.moe_grouped_ffn_static_ws_bytes.restype = sz
        lib.moe_grouped_ffn_static_ws_bytes.argtypes = []
        lib.moe_grouped_ffn_static_ws.restype = ci
        lib.moe_grouped_ffn_static_ws.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, ci, vp, ci, vp, ci, vp, vp]
        lib.moe_unpermute.restype = ci
        lib.moe_unpermute.argtypes = [vp, vp, vp, ci, ci, ci, ci, vp, vp]
        lib.moe_gate_topk_workspace_bytes.restype = sz
        lib.moe_gate_topk_workspace_bytes.argtypes = [ci, ci, ci, ci]
        lib.moe_gate_topk.restype = ci
        lib.moe_gate_topk.argtypes = [vp, vp, ci, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp, sz, vp]
        _lib = lib
    return _lib


def _check(status: int) -> None:
    if status != OK:
        raise MetroError(status, load().metro_status_string(status).decode())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, dtype: torch.dtype, name: str) -> int:
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name}: expected a contiguous {dtype} device tensor, got {t.dtype} on {t.device}")
    return t.data_ptr()


def _weights(t: torch.Tensor, dtype: torch.dtype, name: str):
    """Weights [slots, rows, K]: K contiguous, rows `ld` elements apart, slots rows*ld apart (a dense
    tensor, or a [:, :, :K] view of a buffer with padded rows).  Returns (pointer, ld)."""
    if not (t.is_cuda and t.dtype == dtype and t.dim() == 3):
        raise TypeError(f"{name}: expected a 3-d {dtype} device tensor")
    slots, rows, K = t.shape
    ld = t.stride(1) if rows > 1 else max(K, t.stride(1))
    if t.stride(2) != 1 or ld < K or (slots > 1 and t.stride(0) != rows * ld):
        raise TypeError(f"{name}: rows must be K-contiguous with a uniform pitch (strides {t.stride()})")
    return t.data_ptr(), ld


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return DTYPE_BF16
    if t.dtype == torch.float32:
        return DTYPE_F32
    raise TypeError("activations and weights are bfloat16 or float32")


def route_buffers(L: int, T: int, k: int, N: int, G: int, device) -> Dict[str, torch.Tensor]:
    """Output buffers of the routing calls (reusable across calls of the same shape)."""
    return dict(pair_slot=torch.empty((L, T, k), dtype=torch.int32, device=device),
                expert_slot=torch.empty((L, N), dtype=torch.int32, device=device),
                rank_active=torch.empty((L, G), dtype=torch.int32, device=device),
                rank_bitmap=torch.empty((L, G), dtype=torch.int64, device=device),
                err_flag=torch.empty((L,), dtype=torch.int32, device=device))


def _route(fn_name: str, topk_ids: torch.Tensor, slot_to_expert: torch.Tensor, N: int, G: int, spr: int,
           out: Optional[Dict[str, torch.Tensor]]) -> Dict[str, torch.Tensor]:
    if topk_ids.dim() == 2:
        topk_ids = topk_ids.unsqueeze(0)
    if slot_to_expert.dim() == 1:
        slot_to_expert = slot_to_expert.unsqueeze(0)
    L, T, k = topk_ids.shape
    if tuple(slot_to_expert.shape) != (L, G * spr):
        raise ValueError(f"slot_to_expert must be [L={L}, G*spr={G * spr}]")
    if out is None:
        out = route_buffers(L, T, k, N, G, topk_ids.device)
    lib = load()
    ids_p = _dev(topk_ids, torch.int32, "topk_ids")
    s2e_p = _dev(slot_to_expert, torch.int32, "slot_to_expert")
    ps = _dev(out["pair_slot"], torch.int32, "pair_slot")
    ra = _dev(out["rank_active"], torch.int32, "rank_active")
    rb = _dev(out["rank_bitmap"], torch.int64, "rank_bitmap")
    ef = _dev(out["err_flag"], torch.int32, "err_flag")
    if fn_name == "metro_route":
        es = _dev(out["expert_slot"], torch.int32, "expert_slot")
        _check(lib.metro_route(ids_p, s2e_p, L, T, k, N, G, spr, ps, es, ra, rb, ef, _stream()))
    else:
        _check(lib.metro_route_token_balanced(ids_p, s2e_p, L, T, k, N, G, spr, ps, ra, rb, ef, _stream()))
    return out


def metro_route(topk_ids, slot_to_expert, N: int, G: int, spr: int, out=None) -> Dict[str, torch.Tensor]:
    """topk_ids [L,T,k] (or [T,k]) int32, slot_to_expert [L,S] (or [S]) int32 -> dict of device tensors
    pair_slot [L,T,k], expert_slot [L,N], rank_active [L,G], rank_bitmap [L,G] (int64 bits), err_flag [L]."""
    return _route("metro_route", topk_ids, slot_to_expert, N, G, spr, out)


def metro_route_token_balanced(topk_ids, slot_to_expert, N: int, G: int, spr: int, out=None):
    """Same as metro_route for the token-balanced baseline; expert_slot is left untouched."""
    return _route("metro_route_token_balanced", topk_ids, slot_to_expert, N, G, spr, out)


def permute_buffers(T: int, k: int, spr: int, device) -> Dict[str, torch.Tensor]:
    return dict(group_offsets=torch.empty((spr + 1,), dtype=torch.int32, device=device),
                perm_pair=torch.empty((T * k,), dtype=torch.int32, device=device),
                pair_row=torch.empty((T, k), dtype=torch.int32, device=device),
                n_pairs=torch.empty((1,), dtype=torch.int32, device=device))


def moe_permute(pair_slot: torch.Tensor, rank: int, spr: int, out=None) -> Dict[str, torch.Tensor]:
    """pair_slot [T,k] int32 -> dict(group_offsets [spr+1], perm_pair [T*k], pair_row [T,k], n_pairs [1])."""
    T, k = pair_slot.shape
    if out is None:
        out = permute_buffers(T, k, spr, pair_slot.device)
    _check(load().moe_permute(_dev(pair_slot, torch.int32, "pair_slot"), T, k, rank, spr,
                              _dev(out["group_offsets"], torch.int32, "group_offsets"),
                              _dev(out["perm_pair"], torch.int32, "perm_pair"),
                              _dev(out["pair_row"], torch.int32, "pair_row"),
                              _dev(out["n_pairs"], torch.int32, "n_pairs"), _stream()))
    return out


def _route_permute(fn_name: str, topk_ids, slot_to_expert, N: int, G: int, spr: int, rank: int, out, lists):
    if topk_ids.dim() == 3:
        if topk_ids.shape[0] != 1:
            raise ValueError("the fused call takes one layer")
        topk_ids = topk_ids[0]
    if slot_to_expert.dim() == 2:
        slot_to_expert = slot_to_expert[0]
    T, k = topk_ids.shape
    if slot_to_expert.numel() != G * spr:
        raise ValueError(f"slot_to_expert must hold G*spr={G * spr} entries")
    if out is None:
        out = route_buffers(1, T, k, N, G, topk_ids.device)
    if lists is None:
        lists = permute_buffers(T, k, spr, topk_ids.device)
    lib = load()
    head = [_dev(topk_ids, torch.int32, "topk_ids"), _dev(slot_to_expert, torch.int32, "slot_to_expert"), T, k, N, G, spr,
            rank, _dev(out["pair_slot"], torch.int32, "pair_slot")]
    tail = [_dev(out["rank_active"], torch.int32, "rank_active"), _dev(out["rank_bitmap"], torch.int64, "rank_bitmap"),
            _dev(out["err_flag"], torch.int32, "err_flag"), _dev(lists["group_offsets"], torch.int32, "group_offsets"),
            _dev(lists["perm_pair"], torch.int32, "perm_pair"), _dev(lists["pair_row"], torch.int32, "pair_row"),
            _dev(lists["n_pairs"], torch.int32, "n_pairs"), _stream()]
    if fn_name == "metro_route_permute":
        _check(lib.metro_route_permute(*head, _dev(out["expert_slot"], torch.int32, "expert_slot"), *tail))
    else:
        _check(lib.metro_route_token_balanced_permute(*head, *tail))
    return out, lists


def metro_route_permute(topk_ids, slot_to_expert, N: int, G: int, spr: int, rank: int, out=None, lists=None):
    """metro_route (one layer) and moe_permute(rank) in one launch -> (routing dict, token-list dict)."""
    return _route_permute("metro_route_permute", topk_ids, slot_to_expert, N, G, spr, rank, out, lists)


def metro_route_token_balanced_permute(topk_ids, slot_to_expert, N: int, G: int, spr: int, rank: int, out=None,
                                       lists=None):
    """metro_route_token_balanced (one layer) and moe_permute(rank) in one launch."""
    return _route_permute("metro_route_token_balanced_permute", topk_ids, slot_to_expert, N, G, spr, rank, out, lists)


def moe_grouped_ffn_workspace_bytes(T: int, k: int, spr: int, H: int, I: int, dtype: torch.dtype) -> int:
    code = DTYPE_BF16 if dtype == torch.bfloat16 else DTYPE_F32
    return int(load().moe_grouped_ffn_workspace_bytes(T, k, spr, H, I, code))


def moe_grouped_ffn(x: torch.Tensor, perm_pair: torch.Tensor, group_offsets: torch.Tensor, k: int,
                    w13: torch.Tensor, w2: torch.Tensor, y_perm: Optional[torch.Tensor] = None,
                    ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """x [T,H], w13 [spr,2I,H], w2 [spr,H,I] (bf16 or f32) -> y_perm [T*k,H] (rows < n_pairs written)."""
    T, H = x.shape
    spr, two_i, _ = w13.shape
    I = two_i // 2
    if tuple(w13.shape) != (spr, 2 * I, H) or tuple(w2.shape) != (spr, H, I):
        raise ValueError("weight shapes must be w13 [spr,2I,H] and w2 [spr,H,I]")
    if perm_pair.numel() < T * k or group_offsets.numel() != spr + 1:
        raise ValueError("perm_pair must hold T*k entries and group_offsets spr+1")
    code = _dtype_code(x)
    if y_perm is None:
        y_perm = torch.empty((T * k, H), dtype=x.dtype, device=x.device)
    need = int(load().moe_grouped_ffn_workspace_bytes(T, k, spr, H, I, code))
    if ws is None:
        ws = torch.empty((need,), dtype=torch.uint8, device=x.device)
    p13, ld13 = _weights(w13, x.dtype, "w13")
    p2, ld2 = _weights(w2, x.dtype, "w2")
    _check(load().moe_grouped_ffn(_dev(x, x.dtype, "x"), _dev(perm_pair, torch.int32, "perm_pair"),
                                  _dev(group_offsets, torch.int32, "group_offsets"), T, k, spr, H, I, code,
                                  p13, ld13, p2, ld2, _dev(y_perm, x.dtype, "y_perm"),
                                  _dev(ws, torch.uint8, "ws"), ws.numel(), _stream()))
    return y_perm


def moe_grouped_ffn_static_ws(x: torch.Tensor, perm_pair: torch.Tensor, group_offsets: torch.Tensor, k: int,
                              w13: torch.Tensor, w2: torch.Tensor, y_perm: torch.Tensor) -> torch.Tensor:
    """moe_grouped_ffn on the library's built-in workspace: the caller passes inputs and the output only."""
    T, H = x.shape
    spr, two_i, _ = w13.shape
    I = two_i // 2
    if tuple(w13.shape) != (spr, 2 * I, H) or tuple(w2.shape) != (spr, H, I):
        raise ValueError("weight shapes must be w13 [spr,2I,H] and w2 [spr,H,I]")
    if perm_pair.numel() < T * k or group_offsets.numel() != spr + 1 or tuple(y_perm.shape) != (T * k, H):
        raise ValueError("perm_pair must hold T*k entries, group_offsets spr+1, y_perm [T*k,H]")
    p13, ld13 = _weights(w13, x.dtype, "w13")
    p2, ld2 = _weights(w2, x.dtype, "w2")
    _check(load().moe_grouped_ffn_static_ws(_dev(x, x.dtype, "x"), _dev(perm_pair, torch.int32, "perm_pair"),
                                            _dev(group_offsets, torch.int32, "group_offsets"), T, k, spr, H, I,
                                            _dtype_code(x), p13, ld13, p2, ld2, _dev(y_perm, x.dtype, "y_perm"),
                                            _stream()))
    return y_perm


def moe_grouped_ffn_stages(x, perm_pair, group_offsets, k: int, w13, w2, y_perm, ws, between=None):
    """moe_grouped_ffn as its two stage calls; `between(i)` (i = 0..2) is called before, between and
    after the stages, e.g. to record events on the current stream."""
    T, H = x.shape
    spr, two_i, _ = w13.shape
    I = two_i // 2
    code = _dtype_code(x)
    lib = load()
    go = _dev(group_offsets, torch.int32, "group_offsets")
    wsp, wsn = _dev(ws, torch.uint8, "ws"), ws.numel()
    mark = between if between is not None else (lambda i: None)
    p13, ld13 = _weights(w13, x.dtype, "w13")
    p2, ld2 = _weights(w2, x.dtype, "w2")
    mark(0)
    _check(lib.moe_grouped_ffn_gate_up(_dev(x, x.dtype, "x"), _dev(perm_pair, torch.int32, "perm_pair"), go, T, k,
                                       spr, H, I, code, p13, ld13, wsp, wsn, _stream()))
    mark(1)
    _check(lib.moe_grouped_ffn_down(go, T, k, spr, H, I, code, p2, ld2, _dev(y_perm, x.dtype, "y_perm"), wsp, wsn,
                                    _stream()))
    mark(2)
    return y_perm


def moe_unpermute(y_perm: torch.Tensor, pair_row: torch.Tensor, topk_w: torch.Tensor,
                  out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """y_perm [T*k,H], pair_row [T,k] int32, topk_w [T,k] float32 -> out [T,H]."""
    T, k = pair_row.shape
    H = y_perm.shape[1]
    code = _dtype_code(y_perm)
    if out is None:
        out = torch.empty((T, H), dtype=y_perm.dtype, device=y_perm.device)
    _check(load().moe_unpermute(_dev(y_perm, y_perm.dtype, "y_perm"), _dev(pair_row, torch.int32, "pair_row"),
                                _dev(topk_w, torch.float32, "topk_w"), T, k, H, code,
                                _dev(out, y_perm.dtype, "out"), _stream()))
    return out


def moe_gate_topk(x: torch.Tensor, w_gate: torch.Tensor, k: int, out: Optional[dict] = None,
                  ws: Optional[torch.Tensor] = None, n_valid: Optional[torch.Tensor] = None) -> dict:
    """x [T,H], w_gate [N,H] (bf16 or f32; rows may be strided) -> dict(topk_ids [T,k] int32,
    topk_w [T,k] float32, expert_count [N] int32).  n_valid: int32 device tensor of one element, the number of
    real tokens of a padded batch (tokens past it get ids -1 and weights 0)."""
    T, H = x.shape
    N = w_gate.shape[0]
    if w_gate.shape[1] != H or w_gate.stride(1) != 1:
        raise ValueError("w_gate must be [N,H] with contiguous rows")
    code = _dtype_code(x)
    if out is None:
        out = dict(topk_ids=torch.empty((T, k), dtype=torch.int32, device=x.device),
                   topk_w=torch.empty((T, k), dtype=torch.float32, device=x.device),
                   expert_count=torch.empty((N,), dtype=torch.int32, device=x.device))
    if ws is None:
        ws = torch.empty((int(load().moe_gate_topk_workspace_bytes(T, H, N, code)),), dtype=torch.uint8,
                         device=x.device)
    if not (w_gate.is_cuda and w_gate.dtype == x.dtype):
        raise TypeError(f"w_gate: expected a {x.dtype} device tensor")
    ldw = w_gate.stride(0) if N > 1 else H
    nv = None if n_valid is None else _dev(n_valid, torch.int32, "n_valid")
    _check(load().moe_gate_topk(_dev(x, x.dtype, "x"), w_gate.data_ptr(), ldw, T, H, N, k, code, nv,
                                _dev(out["topk_ids"], torch.int32, "topk_ids"),
                                _dev(out["topk_w"], torch.float32, "topk_w"),
                                _dev(out["expert_count"], torch.int32, "expert_count"),
                                _dev(ws, torch.uint8, "ws"), ws.numel(), _stream()))
    return out
