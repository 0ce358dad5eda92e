"""GPU parity: every entry point of the C ABI against the fp64 CPU oracle on
the same seeded inputs.  Integer outputs must match bit for bit; fp32 outputs
within the stated tolerances (1e-5 max-norm relative for the all-fp32 layer,
2e-2 for bf16-weight layers, 1e-6 absolute for gate weights)."""
import numpy as np
import pytest
import torch

import moe_inputs as mi
from gpu_util import max_rel, pack_layer, skewed_logits, to_dev, to_host
from oracle import moe_oracle as orc

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-5
TOL_BF16 = 2e-2
TOL_GATE = 1e-6


@pytest.fixture(scope="module")
def moe():
    assert torch.cuda.is_available(), "GPU tests need a device"
    import paper_2402_07033_amd as m
    m.lib()  # raises if the HIP library is missing: no fallback
    return m


# ------------------------------------------------------------------ route ----

@pytest.mark.parametrize("T,E,k", [(1, 8, 2), (16, 8, 2), (4096, 8, 2), (1000, 8, 2), (37, 1, 1),
                                   (129, 3, 2), (300, 5, 5), (257, 16, 4), (511, 64, 8),
                                   (65, 33, 1), (64, 8, 8)])
def test_route_bit_exact(moe, T, E, k):
    rng = np.random.default_rng(100 + T + E)
    lg = rng.standard_normal((T, E)).astype(np.float32)
    if T >= 16 and E > 1:  # plant exact ties, signed zeros and all-equal rows
        lg[3, :] = lg[3, 0]
        lg[5, : E // 2 + 1] = 0.0
        lg[5, 0] = -0.0
        lg[7, E - 1] = lg[7, 0] = lg[7].max() + 1.0
    ref_idx, ref_w = orc.route(lg, k)
    idx, w = moe.moe_route(to_dev(lg), k)
    assert (to_host(idx) == ref_idx).all()
    w = to_host(w).astype(np.float64)
    assert np.max(np.abs(w - ref_w)) <= TOL_GATE
    assert np.max(np.abs(w.sum(axis=1) - 1.0)) <= 3e-7


def test_route_zipf_workload_logits(moe):
    for name in ("beam_t16", "prefill_t4096"):
        cfg = mi.CONFIGS[name]
        _, lg, _ = mi.make_activations(cfg)
        ref_idx, ref_w = orc.route(lg, cfg.k)
        idx, w = moe.moe_route(to_dev(lg), cfg.k)
        assert (to_host(idx) == ref_idx).all()
        assert np.max(np.abs(to_host(w) - ref_w)) <= TOL_GATE


# ---------------------------------------------------------------- permute ----

@pytest.mark.parametrize("T,E,k,d,xdt", [(1, 8, 2, 4096, "f32"), (16, 8, 2, 4096, "f32"),
                                         (512, 8, 2, 256, "bf16"), (513, 8, 2, 128, "f32"),
                                         (4096, 8, 2, 4096, "bf16"), (3000, 64, 8, 64, "f32"),
                                         (700, 5, 1, 64, "bf16"), (1024, 16, 1, 64, "f32")])
def test_permute_bit_exact(moe, T, E, k, d, xdt):
    lg = skewed_logits(T, E, 200 + T, empty=(1,) if E > 2 else ())
    idx, _ = orc.route(lg, k)
    x32 = mi.normal_f32(300 + T, 0, (T, d))
    x = mi.f32_to_bf16_bits(x32) if xdt == "bf16" else x32
    rc, ro, rp, ri, rxg = orc.permute(idx, E, mi.to_f64(x))
    c, o, p, ip, xg = moe.moe_permute(to_dev(idx), E, to_dev(x))
    assert (to_host(c) == rc).all() and (to_host(o) == ro).all()
    assert (to_host(p) == rp).all() and (to_host(ip) == ri).all()
    assert (to_host(xg) == x[rp // k]).all()            # bit copy of the rows
    assert (mi.to_f64(to_host(xg)) == rxg).all()
    if E > 2:
        assert rc[1] == 0                                # an empty expert is present


def test_permute_index_only_and_T0_and_determinism(moe):
    lg = skewed_logits(2048, 8, 77)
    idx, _ = orc.route(lg, 2)
    rc, ro, rp, ri, _ = orc.permute(idx, 8, np.zeros((2048, 1)))
    didx = to_dev(idx)
    first = None
    for _ in range(20):
        c, o, p, ip, xg = moe.moe_permute(didx, 8, None)
        got = [to_host(t) for t in (c, o, p, ip)]
        assert xg is None
        if first is None:
            first = got
            assert (got[0] == rc).all() and (got[1] == ro).all()
            assert (got[2] == rp).all() and (got[3] == ri).all()
        else:
            assert all((a == b).all() for a, b in zip(first, got))
    c, o, p, ip, xg = moe.moe_permute(torch.empty((0, 2), dtype=torch.int32, device="cuda"), 8,
                                      torch.empty((0, 64), device="cuda"))
    assert to_host(c).tolist() == [0] * 8 and to_host(o).tolist() == [0] * 9


# ---------------------------------------------------------------- combine ----

@pytest.mark.parametrize("T,k,d", [(1, 2, 4096), (16, 2, 256), (777, 3, 128), (4096, 2, 512)])
def test_combine(moe, T, k, d):
    rng = np.random.default_rng(T)
    yg = rng.standard_normal((T * k, d)).astype(np.float32)
    inv = rng.permutation(T * k).astype(np.int32)
    w = rng.random((T, k)).astype(np.float32)
    ref = orc.combine(yg.astype(np.float64), inv, w.astype(np.float64))
    y = moe.moe_combine(to_dev(yg), to_dev(inv), to_dev(w))
    assert max_rel(to_host(y), ref) <= 1e-6


# ------------------------------------------------------- fp32 layer (tiny) ----

def _layer_parity(moe, cfg, li, tol, path=0, check_yg=True):
    x64 = mi.to_f64(li.x)
    ref = orc.layer(x64, li.logits, li.w1, li.w3, li.w2, cfg.k)
    W = pack_layer(li)
    out = moe.moe_layer(W, to_dev(li.x), to_dev(li.logits), cfg.k, path=path)
    torch.cuda.synchronize()
    for key in ("idx", "counts", "offsets", "perm", "inv_perm"):
        assert (to_host(out[key]) == ref[key]).all(), key
    assert np.max(np.abs(to_host(out["w"]) - ref["w"])) <= TOL_GATE
    e_yg = max_rel(to_host(out["yg"]), ref["yg"])
    e_y = max_rel(to_host(out["y"]), ref["y"])
    print(f"{cfg.name} path={path}: counts={ref['counts'].tolist()} err yg={e_yg:.3e} y={e_y:.3e}")
    if check_yg:
        assert e_yg <= tol
    assert e_y <= tol
    W.free()
    return e_y


def test_layer_tiny_fp32(moe):
    cfg = mi.CONFIGS["tiny_fp32"]
    _layer_parity(moe, cfg, mi.make_layer(cfg, threads=1), TOL_F32)


@pytest.mark.parametrize("T,d,f,E,k", [(5, 64, 64, 4, 2), (70, 128, 192, 3, 1), (33, 256, 512, 8, 2),
                                       (100, 64, 128, 16, 4)])
def test_layer_fp32_shapes(moe, T, d, f, E, k):
    cfg = mi.small_config("f32s", T, d, f, E, k, 400 + T, zipf_s=1.2)
    _layer_parity(moe, cfg, mi.make_layer(cfg, threads=1), TOL_F32)


# ------------------------------------------- bf16-weight layers, small shapes ----

@pytest.mark.parametrize("T,d,f,E,k,xdt", [
    (1, 256, 512, 8, 2, mi.F32), (16, 256, 512, 8, 2, mi.F32), (16, 512, 1024, 8, 2, mi.BF16),
    (7, 1024, 1792, 4, 2, mi.F32), (40, 256, 512, 8, 1, mi.F32), (3, 2048, 3584, 8, 2, mi.F32),
    (16, 128, 256, 3, 3, mi.F32),
    # reductions of 10 steps per wave (f / 32 = 20 and 50; d / 32 = 10 for the first projection)
    (5, 320, 640, 4, 2, mi.F32), (2, 256, 1600, 8, 2, mi.BF16)])
def test_layer_bf16_stream_path(moe, T, d, f, E, k, xdt):
    cfg = mi.small_config("st", T, d, f, E, k, 500 + T + d, w_dtype=mi.BF16, x_dtype=xdt,
                          zipf_s=1.2)
    e = _layer_parity(moe, cfg, mi.make_layer(cfg, threads=1), TOL_BF16, path=moe.MOE_FFN_STREAM)
    if xdt == mi.F32:
        assert e <= 1e-4  # hi/lo split keeps fp32 activations


@pytest.mark.parametrize("T,d,f,E,k,xdt", [
    (1, 256, 512, 8, 2, mi.F32), (100, 256, 512, 8, 2, mi.BF16), (600, 256, 384, 4, 2, mi.BF16),
    (300, 512, 1024, 8, 2, mi.F32), (1100, 256, 256, 3, 1, mi.BF16),
    # few rows per expert (tiles mostly padding); f = 2304 cuts left-over tiles along the
    # reduction
    (70, 256, 384, 8, 2, mi.F32), (150, 512, 2304, 8, 2, mi.BF16), (9, 256, 2048, 16, 2, mi.BF16),
    # 41..96 rows per expert: the 128-token x 512-feature tile (first projection needs
    # f % 256 == 0, second d % 512 == 0, else that projection keeps the default tile);
    # d = 2048 / f = 2304 also cut left-over tiles along the reduction
    (380, 1024, 2304, 8, 2, mi.BF16), (300, 256, 512, 8, 2, mi.F32), (330, 512, 384, 4, 1, mi.BF16),
    (370, 2048, 512, 8, 2, mi.BF16),
    # 97..256 rows per expert: the 192-token x 256-feature tile (hot experts span several
    # tiles, the last one ragged); f = 2304 / d = 2048 cut left-over tiles along the reduction
    (500, 512, 1024, 8, 2, mi.BF16), (900, 1024, 2304, 8, 2, mi.BF16), (1000, 256, 384, 8, 2, mi.F32),
    (460, 2048, 512, 4, 1, mi.BF16)])
def test_layer_bf16_grouped_path(moe, T, d, f, E, k, xdt):
    cfg = mi.small_config("gg", T, d, f, E, k, 600 + T + d, w_dtype=mi.BF16, x_dtype=xdt,
                          zipf_s=1.2)
    _layer_parity(moe, cfg, mi.make_layer(cfg, threads=1), TOL_BF16, path=moe.MOE_FFN_GROUPED)


@pytest.mark.parametrize("T,d,f,E,k,xdt", [
    (1, 256, 512, 8, 2, mi.F32), (16, 256, 512, 8, 2, mi.BF16), (100, 256, 512, 8, 2, mi.BF16),
    (300, 512, 1024, 8, 2, mi.F32), (700, 256, 384, 4, 2, mi.BF16), (260, 1024, 2048, 16, 2, mi.F32),
    (150, 512, 2304, 8, 2, mi.BF16), (500, 256, 4096, 2, 1, mi.BF16)])
def test_layer_bf16_mid_path(moe, T, d, f, E, k, xdt):
    """Weight-streaming grouped GEMM: experts of 0 to several hundred rows (several 192-row
    tiles), 4/8/12-block bodies, one and several reduction parts in the second projection."""
    cfg = mi.small_config("md", T, d, f, E, k, 700 + T + d, w_dtype=mi.BF16, x_dtype=xdt,
                          zipf_s=1.2)
    _layer_parity(moe, cfg, mi.make_layer(cfg, threads=1), TOL_BF16, path=moe.MOE_FFN_MID)


def test_mid_path_is_deterministic(moe):
    cfg = mi.small_config("mdd", 200, 256, 4096, 4, 2, 771, w_dtype=mi.BF16, x_dtype=mi.BF16,
                          zipf_s=1.2)
    li = mi.make_layer(cfg, threads=1)
    W = pack_layer(li)
    outs = [to_host(moe.moe_layer(W, to_dev(li.x), to_dev(li.logits), cfg.k,
                                  path=moe.MOE_FFN_MID)["yg"]) for _ in range(3)]
    assert (outs[0] == outs[1]).all() and (outs[0] == outs[2]).all()
    W.free()


@pytest.mark.parametrize("T,d,f,E,k,wdt,xdt,path_name", [
    (16, 256, 512, 8, 2, mi.F32, mi.F32, "fp32"), (70, 128, 192, 3, 1, mi.F32, mi.F32, "fp32"),
    (16, 512, 1024, 8, 2, mi.BF16, mi.F32, "stream"), (9, 256, 1600, 16, 2, mi.BF16, mi.BF16, "stream"),
    (60, 512, 1024, 16, 2, mi.BF16, mi.BF16, "mid"), (300, 512, 1024, 8, 2, mi.BF16, mi.F32, "grouped"),
    (1100, 256, 384, 4, 3, mi.BF16, mi.BF16, "grouped")])
def test_ffn_tokens_reads_rows_through_perm(moe, T, d, f, E, k, wdt, xdt, path_name):
    """moe_expert_ffn_tokens (rows read as x[perm[i] / k], no gathered copy) gives the bits of
    moe_expert_ffn on the gathered rows, in every kernel family, and matches the oracle."""
    cfg = mi.small_config("tok", T, d, f, E, k, 2300 + T + d, w_dtype=wdt, x_dtype=xdt, zipf_s=1.2)
    li = mi.make_layer(cfg, threads=1)
    W = pack_layer(li)
    want = {"fp32": moe.MOE_FFN_AUTO, "stream": moe.MOE_FFN_STREAM, "mid": moe.MOE_FFN_MID,
            "grouped": moe.MOE_FFN_GROUPED}[path_name]
    got = moe.moe_expert_ffn_plan(cfg.N, E, d, f, moe.MOE_F32 if wdt == mi.F32 else moe.MOE_BF16)
    assert got["path"] == want
    x = to_dev(li.x)
    idx, w = moe.moe_route(to_dev(li.logits), k)
    counts, offsets, perm, inv_perm, none = moe.moe_permute(idx, E, None)   # indices only
    assert none is None
    yg = torch.full((cfg.N, d), float("nan"), device="cuda")
    moe.moe_expert_ffn_tokens(W, x, k, perm, offsets, yg=yg)
    _, _, _, _, xg = moe.moe_permute(idx, E, x)
    ref_gpu = moe.moe_expert_ffn(W, xg, offsets)
    assert torch.equal(yg, ref_gpu)
    ref = orc.layer(mi.to_f64(li.x), li.logits, li.w1, li.w3, li.w2, k)
    assert max_rel(to_host(yg), ref["yg"]) <= (TOL_F32 if wdt == mi.F32 else TOL_BF16)
    y = moe.moe_combine(yg, inv_perm, w)
    assert max_rel(to_host(y), ref["y"]) <= (TOL_F32 if wdt == mi.F32 else TOL_BF16)
    W.free()


def test_ffn_rejects_short_workspace_and_bad_path(moe):
    cfg = mi.small_config("ws", 4, 256, 512, 8, 2, 9, w_dtype=mi.BF16)
    li = mi.make_layer(cfg, threads=1)
    W = pack_layer(li)
    xg = torch.zeros((8, 256), device="cuda")
    off = torch.tensor([0, 1, 2, 3, 4, 5, 6, 7, 8], dtype=torch.int32, device="cuda")
    with pytest.raises(moe.MoeError) as ei:
        moe.moe_expert_ffn(W, xg, off, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert ei.value.status == -3
    with pytest.raises(moe.MoeError) as ei:
        moe.moe_expert_ffn(W, xg, off, path=7)
    assert ei.value.status == -1
    W.free()


# ------------------------------------------------------------ edge cases ----

def test_empty_inputs_are_noops(moe):
    z = torch.empty((0, 8), device="cuda")
    idx, w = moe.moe_route(z, 2)
    assert tuple(idx.shape) == (0, 2) and tuple(w.shape) == (0, 2)
    cfg = mi.small_config("e", 4, 256, 512, 8, 2, 5, w_dtype=mi.BF16)
    li = mi.make_layer(cfg, threads=1)
    W = pack_layer(li)
    off = torch.zeros(9, dtype=torch.int32, device="cuda")
    yg = moe.moe_expert_ffn(W, torch.empty((0, 256), device="cuda"), off)
    assert tuple(yg.shape) == (0, 256)
    y = moe.moe_combine(yg, torch.empty(0, dtype=torch.int32, device="cuda"),
                        torch.empty((0, 2), device="cuda"))
    assert tuple(y.shape) == (0, 256)
    W.free()


@pytest.mark.parametrize("path_name,T,xdt", [("stream", 16, mi.F32), ("stream", 48, mi.F32),
                                             ("grouped", 16, mi.BF16), ("grouped", 700, mi.BF16)])
def test_all_tokens_to_one_expert_and_k_equals_E(moe, path_name, T, xdt):
    path = moe.MOE_FFN_STREAM if path_name == "stream" else moe.MOE_FFN_GROUPED
    # every token picks experts (5, 2) in that order: six experts stay empty
    cfg = mi.small_config("one", T, 256, 512, 8, 2, 900 + T, w_dtype=mi.BF16, x_dtype=xdt)
    li = mi.make_layer(cfg, threads=1)
    lg = np.full((T, 8), -4.0, np.float32)
    lg[:, 5] = 3.0
    lg[:, 2] = 1.0
    li.logits = lg
    _layer_parity(moe, cfg, li, TOL_BF16, path=path)
    # k == E: every expert used by every token (full softmax)
    cfg = mi.small_config("kE", T, 256, 512, 4, 4, 950 + T, w_dtype=mi.BF16, x_dtype=xdt,
                          zipf_s=1.2)
    _layer_parity(moe, cfg, mi.make_layer(cfg, threads=1), TOL_BF16, path=path)


def test_single_expert_layer_and_auto_threshold(moe):
    cfg = mi.small_config("E1", 9, 256, 512, 1, 1, 77, w_dtype=mi.BF16)
    _layer_parity(moe, cfg, mi.make_layer(cfg, threads=1), TOL_BF16)
    # AUTO on either side of its switches: decode kernels up to 72 routed rows, the
    # weight-streaming grouped GEMM up to 10 rows per expert (80 rows here), then the
    # LDS-tiled grouped GEMM (128 x 512 tile up to 96 rows per expert, 192 x 256 up to 256,
    # 256 x 256 above)
    for T in (36, 37, 40, 41, 384, 385, 1024, 1025):
        cfg = mi.small_config("thr", T, 256, 512, 8, 2, 80 + T, w_dtype=mi.BF16, zipf_s=1.2)
        _layer_parity(moe, cfg, mi.make_layer(cfg, threads=1), TOL_BF16)


def test_grouped_path_is_deterministic(moe):
    cfg = mi.small_config("det", 300, 256, 512, 8, 2, 31, w_dtype=mi.BF16, x_dtype=mi.BF16,
                          zipf_s=1.2)
    li = mi.make_layer(cfg, threads=1)
    W = pack_layer(li)
    x, lg = to_dev(li.x), to_dev(li.logits)
    first = moe.moe_layer(W, x, lg, 2, path=moe.MOE_FFN_GROUPED)["yg"].clone()
    for _ in range(5):
        again = moe.moe_layer(W, x, lg, 2, path=moe.MOE_FFN_GROUPED)["yg"]
        assert torch.equal(first, again)
    W.free()


def test_measurement_probes_run_and_validate(moe):
    """The two roofline probes: they launch, report what they did, and refuse bad arguments."""
    ops = torch.randn(32768, device="cuda").to(torch.bfloat16)
    out = torch.empty(512 * 256, dtype=torch.float32, device="cuda")
    flops = moe.moe_mfma_rate_probe(ops, 2, out)
    assert flops > 0
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    buf = torch.zeros(96 << 20, dtype=torch.uint8, device="cuda")
    read = moe.moe_hbm_read_probe(buf, sink)
    torch.cuda.synchronize()
    assert 0 < read <= buf.numel() and read % (16 * 1024) == 0
    assert int(sink[0]) == 0
    with pytest.raises(moe.MoeError):  # less than one ring of loads per wave
        moe.moe_hbm_read_probe(torch.zeros(1 << 20, dtype=torch.uint8, device="cuda"), sink)
