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


def _declared_functions(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported(L):
    from paper_2402_07033_amd import binding
    names = _declared_functions("moe.h")
    assert "moe_route" in names and "moe_expert_ffn" in names and len(names) >= 12
    probes = _declared_functions("moe_probe.h")
    assert "moe_hbm_read_probe" in probes
    for n in names + probes:
        assert hasattr(L, n), f"{n} declared under include/ but not exported"
    assert sorted(binding.EXPORTS) == names
    assert sorted(binding.PROBE_EXPORTS) == probes
    orch = _declared_functions("moe_orch.h")
    for n in orch:
        assert hasattr(L, n), f"{n} declared in include/moe_orch.h but not exported"
    assert sorted(binding.ORCH_EXPORTS) == orch
    # the measurement probes and the split-layer calls are not declared in the layer's header
    assert not set(names) & set(probes) and not set(names) & set(orch)


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
    # fused front ends: an output that overlaps an input every workgroup reads is refused
    big = (C.c_char * (1 << 16))()
    q = (C.addressof(big) + 255) & ~255
    x, h, xg, rest = (C.c_void_p(q + o) for o in (0, 4096, 8192, 32768))
    args = (2, 256, 8, 2, C.c_float(1e-5))   # T, d, E, k, eps: x is 2 KiB
    ok_tail = (rest,) * 7
    assert L.moe_norm_route_permute(x, rest, *args, x, *ok_tail, xg, None) == INVALID   # h == x
    assert L.moe_norm_route_permute(x, rest, *args, h, *ok_tail, x, None) == INVALID    # xg == x
    mis_gate = C.c_void_p(rest.value + 4)
    assert L.moe_norm_route_permute(x, mis_gate, *args, h, *ok_tail, xg, None) == INVALID
    assert L.moe_route_permute(rest, 2, 8, 2, x, 256, *(rest,) * 6, x, None) == INVALID   # xg == x
    # seam: x_out == x_in, h == x_in, n_parts < 1
    seam = lambda xin, xout, hh, parts: L.moe_combine_norm_route_permute(
        rest, parts, rest, rest, 2, xin, xout, rest, *args, hh, *ok_tail, xg, None)
    assert seam(x, x, h, 1) == INVALID and seam(x, h, x, 1) == INVALID
    assert seam(x, C.c_void_p(q + 16384), h, 0) == INVALID
    # combine over parts: y inside the slabs
    assert L.moe_combine_parts(x, 2, rest, rest, 2, 2, 256, x, 0, None, None) == INVALID
    assert L.moe_combine_parts(x, 0, rest, rest, 2, 2, 256, h, 0, None, None) == INVALID
    # decode layer: null handle, and the plan query validates without a device
    assert L.moe_decode_layer(None, x, rest, 1, 2, *(rest,) * 6, None, rest, 1 << 20, None, h,
                              None) == INVALID
    # block step and its gating sums: null handle / null pointers / unsupported sizes
    assert L.moe_decode_block(None, x, None, 0, C.c_float(1e-5), rest, 1, 2, *(rest,) * 6, rest,
                              1 << 20, h, None, None, None) == INVALID
    assert L.moe_gate_sums(None, rest, 1, 256, 8, rest, None) == INVALID
    assert L.moe_gate_sums(x, rest, 1, 256, 24, rest, None) == -2      # more than 16 experts
    assert L.moe_gate_sums_stride(1, 8) == 32 and L.moe_gate_sums_stride(0, 8) == 0
    assert L.moe_decode_block_supported(1, 8, 2, 4096, 14336, 1) == 1
    assert L.moe_decode_block_supported(1, 8, 2, 4096, 14336, 0) == 0  # fp32 weights
    assert L.moe_decode_block_supported(4, 8, 2, 4096, 14336, 1) == 0  # eight routed rows


def test_ffn_plan_query(L):
    import paper_2402_07033_amd as m
    pl = m.moe_expert_ffn_plan(32, 8, 4096, 14336)
    assert pl["path"] == m.MOE_FFN_STREAM and pl["n_parts"] == 4 and pl["up_tile_rows"] == 0
    # one token's rows: the second projection finishes its reduction in one kernel
    assert m.moe_expert_ffn_plan(2, 8, 4096, 14336)["n_parts"] == 1
    pl = m.moe_expert_ffn_plan(8192, 8, 4096, 14336)
    assert pl["path"] == m.MOE_FFN_GROUPED and pl["n_parts"] == 1
    assert pl["up_tile_rows"] == 256 and pl["down_tile_features"] == 256
    assert m.moe_expert_ffn_plan(512, 8, 4096, 14336, path=m.MOE_FFN_GROUPED)["up_tile_rows"] == 128
    assert m.moe_expert_ffn_plan(80, 8, 4096, 14336)["path"] == m.MOE_FFN_MID
    assert m.moe_expert_ffn_plan(32, 16, 4096, 6400)["n_parts"] == 4
    with pytest.raises(m.MoeError):
        m.moe_expert_ffn_plan(16, 8, 4096, 100)


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
