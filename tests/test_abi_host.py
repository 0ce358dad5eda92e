"""Host-only checks of the C ABI: the library loads, exports every symbol that
include/moe.h declares, and rejects bad arguments before touching a GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    import paper_2402_07033_amd as m
    if not os.path.exists(m.lib_path()):
        from paper_2402_07033_amd import build
        build.build()
    return m.lib()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "moe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported(L):
    names = _declared_functions()
    assert "moe_route" in names and "moe_expert_ffn" in names and len(names) >= 12
    for n in names:
        assert hasattr(L, n), f"{n} declared in include/moe.h but not exported"
    from paper_2402_07033_amd import binding
    assert sorted(binding.EXPORTS) == names


def test_status_strings(L):
    import paper_2402_07033_amd as m
    assert m.moe_status_string(0) == "ok"
    seen = {m.moe_status_string(s) for s in (-1, -2, -3, -4)}
    assert len(seen) == 4 and "unknown status" not in seen
    assert m.moe_status_string(-99) == "unknown status"


def test_argument_errors_return_before_any_launch(L):
    INVALID, WORKSPACE = -1, -3
    buf = (C.c_char * 4096)()
    p = C.c_void_p((C.addressof(buf) + 255) & ~255)          # aligned fake pointer
    mis = C.c_void_p(p.value + 4)                            # misaligned
    assert L.moe_route(None, 4, 8, 2, p, p, None) == INVALID           # null logits
    assert L.moe_route(p, -1, 8, 2, p, p, None) == INVALID             # T < 0
    assert L.moe_route(p, 4, 8, 9, p, p, None) == INVALID              # k > E
    assert L.moe_route(p, 4, 65, 2, p, p, None) == INVALID             # E > 64
    assert L.moe_route(p, 4, 16, 9, p, p, None) == INVALID             # k > 8
    assert L.moe_route(mis, 4, 8, 2, p, p, None) == INVALID            # misaligned
    assert L.moe_route(p, 0, 8, 2, p, p, None) == 0                    # T == 0 no-op
    assert L.moe_permute(p, 4, 8, 2, p, 100, 0, p, p, p, p, p, None) == INVALID   # d % 64
    assert L.moe_permute(p, 4, 8, 2, p, 128, 0, p, p, p, p, None, None) == INVALID  # x w/o xg
    assert L.moe_permute(p, 4, 8, 2, None, 0, 0, None, p, p, p, None, None) == INVALID
    assert L.moe_combine(p, p, p, 4, 2, 100, p, None) == INVALID
    assert L.moe_combine(p, p, p, 0, 2, 128, p, None) == 0
    h = C.c_void_p()
    assert L.moe_weights_pack(p, p, p, 8, 4096, 100, 1, C.byref(h), None) == INVALID
    assert L.moe_weights_pack(p, p, p, 8, 4096, 14336, 7, C.byref(h), None) == INVALID
    assert L.moe_weights_pack(p, p, None, 8, 4096, 14336, 1, C.byref(h), None) == INVALID
    assert h.value is None
    assert L.moe_expert_ffn(None, p, 0, p, 4, p, 1 << 20, p, None) == INVALID
    assert L.moe_weights_free(None) == 0
    assert L.moe_rmsnorm(p, 2, 100, C.c_float(1e-5), p, None) == INVALID
    assert L.moe_router_logits(p, p, 2, 128, 65, p, None) == INVALID
    assert L.moe_residual_add(None, p, 2, 128, None) == INVALID


def test_workspace_query(L):
    assert L.moe_expert_ffn_workspace(0, 8, 4096, 14336, 1) >= 256
    assert L.moe_expert_ffn_workspace(-1, 8, 4096, 14336, 1) == 0
    assert L.moe_expert_ffn_workspace(16, 8, 4096, 100, 1) == 0
    a = L.moe_expert_ffn_workspace(32, 8, 4096, 14336, 0)
    b = L.moe_expert_ffn_workspace(8192, 8, 4096, 14336, 1)
    assert 32 * 14336 * 4 <= a < b
    assert L.moe_weights_bytes(None) == 0


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2402_07033_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, fn)).read()
                assert "oracle" not in src.lower(), f"{fn} mentions the oracle"
