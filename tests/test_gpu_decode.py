"""GPU parity of the decode-sized paths: the weight-streaming kernels at shapes whose
per-wave reduction is 10 steps, the one-call decode step (moe_decode_layer), the combine
over unsummed reduction parts, and run-to-run determinism of all of them.

Everything is compared with the fp64 oracle on the same seeded inputs; the one-call step is
also compared with the four separate calls, which must give the same bits."""
import numpy as np
import pytest
import torch

import moe_inputs as mi
from gpu_util import max_rel, pack_layer, skewed_logits, to_dev, to_host
from oracle import moe_oracle as orc

pytestmark = pytest.mark.gpu
TOL_BF16 = 2e-2
TOL_GATE = 1e-6


@pytest.fixture(scope="module")
def moe():
    assert torch.cuda.is_available()
    import paper_2402_07033_amd as m
    m.lib()
    return m


def _check_indices(out, ref):
    for key in ("idx", "counts", "offsets", "perm", "inv_perm"):
        assert (to_host(out[key]) == ref[key]).all(), key
    assert np.max(np.abs(to_host(out["w"]) - ref["w"])) <= TOL_GATE


# d / 32 = 80 and 30 give 10 reduction steps per wave in the first projection (two matrices:
# 20 fragment loads per unit, kept in a ring of 10); f = 4096 with up to 32 routed rows gives
# every workgroup more than one unit, so the ring is carried across unit borders.
@pytest.mark.parametrize("d,f,T,xdt", [(2560, 4096, 16, mi.F32), (2560, 4096, 16, mi.BF16),
                                       (960, 4096, 16, mi.F32), (960, 4096, 9, mi.BF16),
                                       (1600, 2560, 16, mi.F32), (320, 4096, 16, mi.F32)])
def test_stream_path_ten_step_reductions(moe, d, f, T, xdt):
    cfg = mi.small_config("st10", T, d, f, 8, 2, 1500 + d + T, w_dtype=mi.BF16, x_dtype=xdt,
                          zipf_s=1.2)
    li = mi.make_layer(cfg, threads=8)
    ref = orc.layer(mi.to_f64(li.x), li.logits, li.w1, li.w3, li.w2, cfg.k)
    W = pack_layer(li)
    pl = moe.moe_expert_ffn_plan(cfg.N, cfg.E, d, f, path=moe.MOE_FFN_STREAM)
    assert pl["path"] == moe.MOE_FFN_STREAM
    out = moe.moe_layer(W, to_dev(li.x), to_dev(li.logits), cfg.k, path=moe.MOE_FFN_STREAM)
    torch.cuda.synchronize()
    _check_indices(out, ref)
    e_yg, e_y = max_rel(to_host(out["yg"]), ref["yg"]), max_rel(to_host(out["y"]), ref["y"])
    print(f"stream d={d} f={f} T={T} {xdt}: err yg={e_yg:.3e} y={e_y:.3e}")
    assert e_yg <= (1e-4 if xdt == mi.F32 else TOL_BF16) and e_y <= TOL_BF16
    W.free()


@pytest.mark.parametrize("T,d,f,E,k", [(1, 256, 512, 8, 2), (16, 256, 512, 8, 2), (7, 1024, 1792, 4, 2),
                                       (16, 512, 1024, 16, 4), (3, 2048, 3584, 8, 2), (5, 320, 640, 4, 2),
                                       (16, 128, 256, 3, 3), (9, 256, 1600, 16, 1), (8, 256, 512, 8, 8),
                                       (4, 256, 7168, 8, 2),
                                       # one to four routed rows: the second projection finishes its
                                       # reduction and the combine in one kernel; f = 1600 leaves
                                       # the waves of a row unequal shares of the reduction
                                       (1, 256, 1600, 8, 1), (1, 512, 1600, 8, 3), (1, 512, 1600, 8, 2), (2, 256, 512, 8, 2),
                                       (1, 1024, 7168, 8, 4), (2, 320, 640, 4, 1), (4, 256, 512, 4, 1),
                                       (1, 4096, 2048, 8, 2), (1, 128, 14336, 8, 2)])
def test_decode_layer_small_shapes(moe, T, d, f, E, k):
    """moe_decode_layer against the oracle and, bit for bit, against the four calls."""
    cfg = mi.small_config("dl", T, d, f, E, k, 1700 + T + d, w_dtype=mi.BF16, zipf_s=1.2)
    li = mi.make_layer(cfg, threads=1)
    ref = orc.layer(mi.to_f64(li.x), li.logits, li.w1, li.w3, li.w2, k)
    W = pack_layer(li)
    x, lg = to_dev(li.x), to_dev(li.logits)
    yg = torch.full((T * k, d), float("nan"), device="cuda")
    out = moe.moe_decode_layer(W, x, lg, k, yg=yg, want_xg=True)
    four = moe.moe_layer(W, x, lg, k, path=moe.MOE_FFN_STREAM)
    torch.cuda.synchronize()
    _check_indices(out, ref)
    assert (to_host(out["xg"]) == li.x[ref["perm"] // k]).all()
    assert not torch.isnan(out["yg"]).any() and not torch.isnan(out["y"]).any()
    e_yg, e_y = max_rel(to_host(out["yg"]), ref["yg"]), max_rel(to_host(out["y"]), ref["y"])
    print(f"decode_layer T={T} d={d} f={f} E={E} k={k}: counts={ref['counts'].tolist()} "
          f"err yg={e_yg:.3e} y={e_y:.3e}")
    assert e_yg <= 1e-4 and e_y <= 1e-4
    assert torch.equal(out["yg"], four["yg"]) and torch.equal(out["y"], four["y"])
    # without the optional outputs: same y
    out2 = moe.moe_decode_layer(W, x, lg, k)
    assert out2["xg"] is None and torch.equal(out2["y"], out["y"])
    W.free()


@pytest.mark.parametrize("T,E,k", [(16, 8, 2), (16, 16, 4), (8, 3, 3), (4, 5, 1), (2, 2, 2), (1, 8, 2)])
def test_decode_gating_with_ties(moe, T, E, k):
    """The gating inside the first-projection kernel (every wave routes for itself) on logits
    with exact ties, signed zeros and all-equal rows: the indices of the oracle (larger logit
    first, lower expert index among equals), bit for bit; the same through moe_decode_block."""
    d, f = 256, 512
    cfg = mi.small_config("tie", T, d, f, E, k, 2300 + T + E, w_dtype=mi.BF16)
    li = mi.make_layer(cfg, threads=1)
    rng = np.random.default_rng(23 * T + E)
    lg = rng.standard_normal((T, E)).astype(np.float32)
    lg[0, :] = lg[0, 0]                                # an all-equal row
    if T > 1:
        lg[1, : E // 2 + 1] = 0.0                      # zeros of both signs
        lg[1, 0] = -0.0
    if T > 2:
        lg[2, E - 1] = lg[2, 0] = lg[2].max() + 1.0    # the first and the last expert tie at the top
    ref_idx, ref_w = orc.route(lg, k)
    W = pack_layer(li)
    out = moe.moe_decode_layer(W, to_dev(li.x), to_dev(lg), k)
    assert (to_host(out["idx"]) == ref_idx).all()
    assert np.max(np.abs(to_host(out["w"]) - ref_w)) <= TOL_GATE
    ref = orc.layer(mi.to_f64(li.x), lg, li.w1, li.w3, li.w2, k)
    _check_indices(out, ref)
    assert max_rel(to_host(out["y"]), ref["y"]) <= 1e-4
    if moe.moe_decode_block_supported(T, E, k, d, f):
        blk = moe.moe_decode_block(W, to_dev(li.x), k, logits=to_dev(lg))
        assert (to_host(blk["idx"]) == ref_idx).all()
        assert torch.equal(blk["x_out"], to_dev(li.x) + out["y"])
    W.free()


def test_decode_layer_unsupported_and_errors(moe):
    cfg = mi.small_config("dle", 4, 256, 512, 8, 2, 99, w_dtype=mi.BF16)
    li = mi.make_layer(cfg, threads=1)
    W = pack_layer(li)
    x17 = torch.zeros((17, 256), device="cuda")
    with pytest.raises(moe.MoeError) as ei:       # T > 16
        moe.moe_decode_layer(W, x17, torch.zeros((17, 8), device="cuda"), 2)
    assert ei.value.status == -2
    x = to_dev(li.x)
    with pytest.raises(moe.MoeError) as ei:       # workspace too small
        moe.moe_decode_layer(W, x, to_dev(li.logits), 2,
                             workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert ei.value.status == -3
    with pytest.raises(moe.MoeError) as ei:       # y overlaps x
        moe.moe_decode_layer(W, x, to_dev(li.logits), 2, y=x)
    assert ei.value.status == -1
    W.free()
    cfg = mi.small_config("dlf", 4, 256, 512, 8, 2, 98)   # fp32 weights: no decode kernels
    Wf = pack_layer(mi.make_layer(cfg, threads=1))
    with pytest.raises(moe.MoeError) as ei:
        moe.moe_decode_layer(Wf, x, to_dev(li.logits), 2)
    assert ei.value.status == -2
    Wf.free()


def test_decode_paths_are_deterministic(moe):
    """20 runs of the four calls (decode kernels) and of the one-call step: identical bits.
    f = 7168 cuts the second projection's reduction into two parts."""
    cfg = mi.small_config("det", 16, 1024, 7168, 8, 2, 1801, w_dtype=mi.BF16, zipf_s=1.2)
    li = mi.make_layer(cfg, threads=8)
    W = pack_layer(li)
    assert moe.moe_expert_ffn_plan(cfg.N, cfg.E, cfg.d, cfg.f, path=moe.MOE_FFN_STREAM)["n_parts"] > 1
    x, lg = to_dev(li.x), to_dev(li.logits)
    first = moe.moe_layer(W, x, lg, cfg.k, path=moe.MOE_FFN_STREAM)
    yg0, y0 = first["yg"].clone(), first["y"].clone()
    for _ in range(20):
        again = moe.moe_layer(W, x, lg, cfg.k, path=moe.MOE_FFN_STREAM)
        assert torch.equal(again["yg"], yg0) and torch.equal(again["y"], y0)
        yg = torch.empty_like(yg0)
        one = moe.moe_decode_layer(W, x, lg, cfg.k, yg=yg)
        assert torch.equal(one["yg"], yg0) and torch.equal(one["y"], y0)
    W.free()


@pytest.mark.parametrize("T,k,d,P", [(1, 2, 4096, 4), (16, 2, 256, 1), (5, 3, 128, 7), (300, 2, 512, 2)])
def test_combine_parts(moe, T, k, d, P):
    rng = np.random.default_rng(10 * T + P)
    parts = rng.standard_normal((P, T * k, d)).astype(np.float32)
    inv = rng.permutation(T * k).astype(np.int32)
    w = rng.random((T, k)).astype(np.float32)
    yg_ref = parts.astype(np.float64).sum(axis=0)
    y_ref = orc.combine(yg_ref, inv, w.astype(np.float64))
    yg = torch.full((T * k, d), float("nan"), device="cuda")
    y = moe.moe_combine_parts(to_dev(parts), P, to_dev(inv), to_dev(w), yg=yg)
    assert max_rel(to_host(y), y_ref) <= 2e-6 and max_rel(to_host(yg), yg_ref) <= 1e-6
    # residual form: y0 + combine
    y0 = rng.standard_normal((T, d)).astype(np.float32)
    yr = to_dev(y0.copy())
    moe.moe_combine_parts(to_dev(parts), P, to_dev(inv), to_dev(w), y=yr, residual=True)
    assert max_rel(to_host(yr), y0.astype(np.float64) + y_ref) <= 2e-6
    # one part: the plain combine, bit for bit
    if P == 1:
        assert torch.equal(y, moe.moe_combine(to_dev(parts[0]), to_dev(inv), to_dev(w)))


def test_expert_ffn_parts_sum_to_yg(moe):
    """The unsummed parts of the decode kernels add up, in part order, to what moe_expert_ffn
    returns; other kernel families write one slab."""
    cfg = mi.small_config("pt", 12, 512, 7168, 8, 2, 1901, w_dtype=mi.BF16, zipf_s=1.2)
    li = mi.make_layer(cfg, threads=8)
    W = pack_layer(li)
    idx, _ = moe.moe_route(to_dev(li.logits), cfg.k)
    _, offsets, _, _, xg = moe.moe_permute(idx, cfg.E, to_dev(li.x))
    P = moe.moe_expert_ffn_plan(cfg.N, cfg.E, cfg.d, cfg.f)["n_parts"]
    assert P > 1
    parts = torch.full((P, cfg.N, cfg.d), float("nan"), device="cuda")
    assert moe.moe_expert_ffn_parts(W, xg, offsets, parts) == P
    yg = moe.moe_expert_ffn(W, xg, offsets)
    acc = parts[0].clone()
    for p in range(1, P):
        acc += parts[p]
    assert torch.equal(acc, yg)
    with pytest.raises(moe.MoeError):   # fewer slabs than the shape needs
        moe.moe_expert_ffn_parts(W, xg, offsets, parts[:1].contiguous())
    W.free()
    # a prefill-sized call: one slab, equal to moe_expert_ffn
    cfg = mi.small_config("pg", 300, 256, 512, 8, 2, 1902, w_dtype=mi.BF16, x_dtype=mi.BF16, zipf_s=1.2)
    li = mi.make_layer(cfg, threads=1)
    W = pack_layer(li)
    idx, _ = moe.moe_route(to_dev(li.logits), cfg.k)
    _, offsets, _, _, xg = moe.moe_permute(idx, cfg.E, to_dev(li.x))
    parts = torch.full((2, cfg.N, cfg.d), float("nan"), device="cuda")
    assert moe.moe_expert_ffn_parts(W, xg, offsets, parts) == 1
    assert torch.equal(parts[0], moe.moe_expert_ffn(W, xg, offsets))
    W.free()
    # one token: the second projection sums inside its workgroups and leaves one slab, even
    # where more rows of the same shape leave several
    cfg = mi.small_config("p1", 1, 512, 7168, 8, 2, 1903, w_dtype=mi.BF16)
    li = mi.make_layer(cfg, threads=8)
    W = pack_layer(li)
    assert moe.moe_expert_ffn_plan(64, cfg.E, cfg.d, cfg.f)["n_parts"] > 1
    assert moe.moe_expert_ffn_plan(cfg.N, cfg.E, cfg.d, cfg.f)["n_parts"] == 1
    idx, _ = moe.moe_route(to_dev(li.logits), cfg.k)
    _, offsets, _, _, xg = moe.moe_permute(idx, cfg.E, to_dev(li.x))
    parts = torch.full((1, cfg.N, cfg.d), float("nan"), device="cuda")
    assert moe.moe_expert_ffn_parts(W, xg, offsets, parts) == 1
    assert torch.equal(parts[0], moe.moe_expert_ffn(W, xg, offsets))
    ref = orc.layer(mi.to_f64(li.x), li.logits, li.w1, li.w3, li.w2, cfg.k)
    assert max_rel(to_host(parts[0]), ref["yg"]) <= 1e-4
    W.free()
