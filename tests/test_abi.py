"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every function the
header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "metro.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2512_09277_amd import api

    if not os.path.exists(api.LIB_PATH):
        from paper_2512_09277_amd import build

        build.build()
    return api.load()


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return re.findall(r"^\s*(?:const\s+char\s*\*|int|size_t)\s+(\w+)\s*\(", text, flags=re.M)


def test_header_declares_the_boundary():
    names = declared_functions()
    for want in ("metro_route", "metro_route_token_balanced", "moe_permute", "moe_grouped_ffn", "moe_unpermute"):
        assert want in names


def test_every_declared_symbol_is_exported(lib):
    from paper_2512_09277_amd import api

    names = declared_functions()
    assert sorted(names) == sorted(api.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_status_strings(lib):
    assert lib.metro_status_string(0) == b"ok"
    for code in (-1, -2, -3, -4, -5):
        assert lib.metro_status_string(code) not in (b"ok", b"unknown status")
    assert lib.metro_status_string(-99) == b"unknown status"


def test_host_side_argument_checks(lib):
    """Rejected before any launch: null pointers, bad sizes, sizes past the limits, small workspace."""
    one = ctypes.c_void_p(256)                       # never dereferenced: the checks fail first
    assert lib.metro_route(None, one, 1, 4, 2, 8, 2, 4, one, one, one, one, one, None) == -1
    assert lib.metro_route(one, None, 1, 0, 2, 8, 2, 4, one, one, one, one, one, None) == -1
    assert lib.metro_route(one, one, 1, 4, 9, 8, 2, 4, one, one, one, one, one, None) == -1     # k > N
    assert lib.metro_route(one, one, 0, 4, 2, 8, 2, 4, one, one, one, one, one, None) == -1     # L < 1
    assert lib.metro_route(one, one, 1, 4, 2, 513, 2, 4, one, one, one, one, one, None) == -2   # N > 512
    assert lib.metro_route(one, one, 1, 4, 2, 8, 65, 4, one, one, one, one, one, None) == -2    # G > 64
    assert lib.metro_route_token_balanced(one, one, 1, 4, 2, 8, 2, 65, one, one, one, one, None) == -2
    assert lib.moe_permute(one, 4, 2, 0, 65, one, one, one, one, None) == -2
    assert lib.moe_permute(one, 4, 0, 0, 4, one, one, one, one, None) == -1
    assert lib.moe_unpermute(one, one, one, 4, 2, 16, 7, one, None) == -2                       # dtype
    need = lib.moe_grouped_ffn_workspace_bytes(4, 2, 3, 256, 128, 1)
    assert need >= 4 * 2 * 128 * 2
    assert lib.moe_grouped_ffn(one, one, one, 4, 2, 3, 256, 128, 1, one, 256, one, 128, one, one, need - 1, None) == -3
    assert lib.moe_grouped_ffn(one, one, one, 4, 2, 3, 256, 128, 1, ctypes.c_void_p(8), 256, one, 128, one, one,
                               need, None) == -1                                               # misaligned w13
    assert lib.moe_grouped_ffn(one, one, one, 4, 2, 3, 256, 128, 1, one, 255, one, 128, one, one, need,
                               None) == -1                                                     # pitch < H
    assert lib.moe_grouped_ffn(one, one, one, 4, 2, 3, 256, 128, 5, one, 256, one, 128, one, one, need, None) == -2
    gate_ws = lib.moe_gate_topk_workspace_bytes(32, 256, 64, 1)
    assert gate_ws >= 32 * 64 * 4
    assert lib.moe_gate_topk(one, one, 256, 32, 256, 64, 65, 1, None, one, one, None, one, gate_ws, None) == -1    # k > N
    assert lib.moe_gate_topk(one, one, 255, 32, 256, 64, 8, 1, None, one, one, None, one, gate_ws, None) == -1     # pitch < H
    assert lib.moe_gate_topk(one, one, 256, 32, 256, 513, 8, 1, None, one, one, None, one, 1 << 20, None) == -2    # N > 512
    assert lib.moe_gate_topk(one, one, 256, 32, 256, 64, 8, 3, None, one, one, None, one, gate_ws, None) == -2     # dtype
    assert lib.moe_gate_topk(one, None, 256, 32, 256, 64, 8, 1, None, one, one, None, one, gate_ws, None) == -1    # null
    assert lib.moe_gate_topk(one, one, 256, 32, 256, 64, 8, 1, None, one, one, None, one, gate_ws - 1, None) == -3
    assert lib.moe_gate_topk(None, None, 256, 0, 256, 64, 8, 1, None, None, None, None, None, 0, None) == 0        # empty batch


def test_size_queries_take_every_batch_size(lib):
    """The workspace queries are plain host arithmetic: an empty batch and bad sizes must not trap."""
    assert lib.moe_gate_topk_workspace_bytes(0, 256, 64, 1) >= 0
    assert lib.moe_gate_topk_workspace_bytes(0, 7168, 256, 1) >= 0
    assert lib.moe_gate_topk_workspace_bytes(-1, 256, 64, 1) == 0
    assert lib.moe_grouped_ffn_workspace_bytes(0, 2, 3, 256, 128, 1) >= 0
    assert lib.moe_grouped_ffn_workspace_bytes(4, 0, 3, 256, 128, 1) == 0
    cap = lib.moe_grouped_ffn_static_ws_bytes()
    assert cap >= lib.moe_grouped_ffn_workspace_bytes(1024, 8, 36, 7168, 2048, 1)     # the headline shape fits
    one = ctypes.c_void_p(256)
    # one row more than fits: refused on the host, before anything touches the device
    assert lib.moe_grouped_ffn_workspace_bytes(1025, 8, 36, 7168, 2048, 1) > cap
    assert lib.moe_grouped_ffn_static_ws(one, one, one, 1025, 8, 36, 7168, 2048, 1, one, 7168, one, 2048, one,
                                         None) == -5
    assert lib.moe_grouped_ffn_static_ws(one, one, one, 4, 2, 65, 256, 128, 1, one, 256, one, 128, one, None) == -2


def test_binding_fails_loudly_without_the_library(monkeypatch):
    from paper_2512_09277_amd import api

    monkeypatch.setattr(api, "_lib", None)
    monkeypatch.setattr(api, "LIB_PATH", "/nonexistent/libmetro.so")
    with pytest.raises(RuntimeError):
        api.load()
