"""GPU parity at the full layer shapes bench.py times: Mixtral-8x7B (d=4096,
f=14336, E=8, top-2, bf16 weights) and the 16-expert shape (d=4096, f=6400,
E=16, top-2), in the launch configuration of the bench.

The oracle runs whole for the decode-sized workloads (1 and 16 tokens); for the
prefill-sized ones it runs on sampled rows: one row of every 16-row block of
every expert segment (so every workgroup tile, every piece of a tile whose
reduction was split, and every fix-up block is covered) plus the first and last
row of every segment -- the full fp64 layer at 4096 tokens is ~2.9 TFLOP of CPU
work.  Which kernel family and tile shape ran is asserted through
moe_expert_ffn_plan, so that a test cannot silently fall onto another kernel."""
import numpy as np
import pytest
import torch

import moe_inputs as mi
from gpu_util import max_rel, pack_layer, to_dev, to_host
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


def _weights(cfg_name):
    cfg = mi.CONFIGS[cfg_name]
    w1, w3, w2 = mi.make_weights(cfg, threads=16)
    W = pack_layer(mi.LayerInputs(cfg, None, None, w1, w3, w2))
    return dict(w1=w1, w3=w3, w2=w2, W=W)


@pytest.fixture(scope="module")
def mixtral(moe):
    """One set of Mixtral-shaped expert matrices (weight seed 1002), host + packed."""
    m = _weights("decode_t1")
    yield m
    m["W"].free()


@pytest.fixture(scope="module")
def e16(moe):
    """One set of 16-expert-shaped matrices (weight seed 1005), host + packed."""
    m = _weights("e16_decode_t1")
    yield m
    m["W"].free()


@pytest.fixture
def shape_weights(request):
    return request.getfixturevalue("e16" if request.param.startswith("e16") else "mixtral")


def _check_index_outputs(out, ref):
    for key in ("idx", "counts", "offsets", "perm", "inv_perm"):
        assert (to_host(out[key]) == ref[key]).all(), key
    assert np.max(np.abs(to_host(out["w"]) - ref["w"])) <= TOL_GATE


DECODE_SIZED = ["decode_t1", "beam_t16", "e16_decode_t1", "e16_beam_t16"]


@pytest.mark.parametrize("name,shape_weights", [(n, n) for n in DECODE_SIZED],
                         indirect=["shape_weights"])
def test_decode_sized_layer_full(moe, shape_weights, name):
    mixtral = shape_weights
    cfg = mi.CONFIGS[name]
    x, logits, _ = mi.make_activations(cfg)
    ref = orc.layer(mi.to_f64(x), logits, mixtral["w1"], mixtral["w3"], mixtral["w2"], cfg.k)
    out = moe.moe_layer(mixtral["W"], to_dev(x), to_dev(logits), cfg.k)
    torch.cuda.synchronize()
    _check_index_outputs(out, ref)
    e_yg, e_y = max_rel(to_host(out["yg"]), ref["yg"]), max_rel(to_host(out["y"]), ref["y"])
    print(f"{name}: counts={ref['counts'].tolist()} err yg={e_yg:.3e} y={e_y:.3e}")
    assert e_yg <= TOL_BF16 and e_y <= TOL_BF16
    # every row of yg must have been written by exactly the kernels of this call
    out2 = moe.moe_layer(mixtral["W"], to_dev(x), to_dev(logits), cfg.k)
    assert max_rel(to_host(out2["y"]), ref["y"]) <= TOL_BF16


def _layer_with_nan_canary(moe, W, x, logits, k, path=0):
    """The four calls with yg pre-filled with NaN: a row the kernels do not write stays NaN."""
    idx, w = moe.moe_route(logits, k)
    counts, offsets, perm, inv_perm, xg = moe.moe_permute(idx, W.E, x)
    yg = torch.full((x.shape[0] * k, W.d), float("nan"), device="cuda")
    moe.moe_expert_ffn(W, xg, offsets, yg=yg, path=path)
    y = moe.moe_combine(yg, inv_perm, w)
    torch.cuda.synchronize()
    return dict(idx=idx, w=w, counts=counts, offsets=offsets, perm=perm, inv_perm=inv_perm,
                xg=xg, yg=yg, y=y)


def _sample_rows(offsets, E, per_block=True):
    """One row of every 16-row block of every segment (its position inside the block varies
    with the block), plus each segment's first and last row."""
    rows = []
    for e in range(E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi <= lo:
            continue
        cand = {lo, hi - 1}
        if per_block:
            for b in range((hi - lo + 15) // 16):
                cand.add(min(hi - 1, lo + 16 * b + (5 * b + 3) % 16))
        rows += sorted(cand)
    return np.array(rows)


def _check_sampled(moe, wts, cfg, x, logits, out, rows):
    """yg rows `rows` against the oracle, the combine of all tokens on the GPU's own yg, the
    tokens whose k rows were all sampled end to end, and that every row of yg was written."""
    idx, w = orc.route(logits, cfg.k)
    counts, offsets, perm, inv_perm, _ = orc.permute(idx, cfg.E, np.zeros((cfg.T, 1)))
    _check_index_outputs(out, dict(idx=idx, w=w, counts=counts, offsets=offsets, perm=perm,
                                   inv_perm=inv_perm))
    x64 = mi.to_f64(x)
    xg_s = x64[perm[rows] // cfg.k]
    seg = np.searchsorted(offsets[1:], rows, side="right")
    s_off = np.concatenate([[0], np.cumsum(np.bincount(seg, minlength=cfg.E))]).astype(np.int32)
    yg_ref = orc.expert_ffn(xg_s, s_off, wts["w1"], wts["w3"], wts["w2"])
    yg = to_host(out["yg"])
    assert np.isfinite(yg).all(), "a row of yg was not written"
    scale = float(np.max(np.abs(yg_ref)))
    e_yg = float(np.max(np.abs(yg[rows] - yg_ref)) / scale)
    y_from_gpu_yg = orc.combine(yg.astype(np.float64), inv_perm, w)
    assert max_rel(to_host(out["y"]), y_from_gpu_yg) <= 1e-6
    inv_rows = {int(r): i for i, r in enumerate(rows)}
    toks = [t for t in range(cfg.T)
            if all(int(inv_perm[t * cfg.k + j]) in inv_rows for j in range(cfg.k))]
    y_gpu = to_host(out["y"])
    for t in toks:
        y_ref = sum(w[t, j] * yg_ref[inv_rows[int(inv_perm[t * cfg.k + j])]] for j in range(cfg.k))
        assert np.max(np.abs(y_gpu[t] - y_ref)) / scale <= TOL_BF16
    return e_yg, counts, len(toks)


@pytest.mark.parametrize("name,shape_weights",
                         [(n, n) for n in ["prefill_t4096", "e16_prefill_t4096"]],
                         indirect=["shape_weights"])
def test_prefill_layer_sampled_rows(moe, shape_weights, name):
    cfg = mi.CONFIGS[name]
    x, logits, _ = mi.make_activations(cfg)
    pl = moe.moe_expert_ffn_plan(cfg.N, cfg.E, cfg.d, cfg.f)
    assert pl["path"] == moe.MOE_FFN_GROUPED
    out = _layer_with_nan_canary(moe, shape_weights["W"], to_dev(x), to_dev(logits), cfg.k)
    rows = _sample_rows(to_host(out["offsets"]), cfg.E)
    e_yg, counts, n_tok = _check_sampled(moe, shape_weights, cfg, x, logits, out, rows)
    print(f"{name}: plan={pl} counts={counts.tolist()} sampled rows={len(rows)} "
          f"(tokens end to end: {n_tok}) err={e_yg:.3e}")
    assert e_yg <= TOL_BF16


def _balanced_config(T, seed):
    """Mixtral shape, bf16 activations, router logits without expert bias: every expert gets
    about T*k/E rows."""
    return mi.MoEConfig(f"bal_t{T}", T, 4096, 14336, 8, 2, mi.BF16, mi.BF16, seed, 0.0, 1002)


def _tiles_beyond_first(counts, tile_rows):
    tiles = sum((int(c) + tile_rows - 1) // tile_rows for c in counts)
    return tiles, tiles - sum(1 for c in counts if c > 0)


# The tile shapes that the 32-layer stack at 512 tokens and the sweeps between decode and
# prefill run, at the Mixtral shape, with balanced routing so that (nearly) every expert has a
# single token tile and the kernel streams the weights past L2 (its device-side rule: token
# tiles beyond an expert's first are at most 15 % of all token tiles).
@pytest.mark.parametrize("T,tile_rows,tile_features", [(512, 192, 256), (256, 128, 512),
                                                       (384, 128, 512)])
def test_grouped_small_tiles_full_size(moe, mixtral, T, tile_rows, tile_features):
    cfg = _balanced_config(T, 1100 + T)
    x, logits, _ = mi.make_activations(cfg)
    pl = moe.moe_expert_ffn_plan(cfg.N, cfg.E, cfg.d, cfg.f)
    assert pl["path"] == moe.MOE_FFN_GROUPED
    assert (pl["up_tile_rows"], pl["up_tile_features"]) == (tile_rows, tile_features)
    assert (pl["down_tile_rows"], pl["down_tile_features"]) == (tile_rows, tile_features)
    out = _layer_with_nan_canary(moe, mixtral["W"], to_dev(x), to_dev(logits), cfg.k)
    counts = to_host(out["counts"])
    tiles, beyond = _tiles_beyond_first(counts, tile_rows)
    assert beyond * 100 <= 15 * tiles, "routing does not select the streamed-weight body"
    rows = _sample_rows(to_host(out["offsets"]), cfg.E)
    e_yg, counts, n_tok = _check_sampled(moe, mixtral, cfg, x, logits, out, rows)
    print(f"balanced T={T}: plan={pl} counts={counts.tolist()} sampled rows={len(rows)} "
          f"(tokens end to end: {n_tok}) err={e_yg:.3e}")
    assert e_yg <= TOL_BF16


def test_grouped_small_tile_with_weights_through_l2_full_size(moe, mixtral):
    """Same 192 x 256 tile with skewed routing: hot experts span several token tiles, so the
    kernel's rule keeps the weights in L2 (the other copy of its loop)."""
    cfg = mi.MoEConfig("zipf_t512", 512, 4096, 14336, 8, 2, mi.BF16, mi.BF16, 1177, 1.2, 1002)
    x, logits, _ = mi.make_activations(cfg)
    pl = moe.moe_expert_ffn_plan(cfg.N, cfg.E, cfg.d, cfg.f)
    assert (pl["path"], pl["up_tile_rows"]) == (moe.MOE_FFN_GROUPED, 192)
    out = _layer_with_nan_canary(moe, mixtral["W"], to_dev(x), to_dev(logits), cfg.k)
    tiles, beyond = _tiles_beyond_first(to_host(out["counts"]), 192)
    assert beyond * 100 > 15 * tiles
    rows = _sample_rows(to_host(out["offsets"]), cfg.E)
    e_yg, counts, _ = _check_sampled(moe, mixtral, cfg, x, logits, out, rows)
    print(f"zipf T=512: counts={counts.tolist()} sampled rows={len(rows)} err={e_yg:.3e}")
    assert e_yg <= TOL_BF16


@pytest.mark.parametrize("T", [37, 40])
def test_mid_kernel_full_size(moe, mixtral, T):
    """73..80 routed rows at 8 experts: AUTO takes the weight-streaming grouped GEMM."""
    cfg = mi.MoEConfig(f"mid_t{T}", T, 4096, 14336, 8, 2, mi.BF16, mi.F32, 1200 + T, 1.2, 1002)
    x, logits, _ = mi.make_activations(cfg)
    assert moe.moe_expert_ffn_plan(cfg.N, cfg.E, cfg.d, cfg.f)["path"] == moe.MOE_FFN_MID
    out = _layer_with_nan_canary(moe, mixtral["W"], to_dev(x), to_dev(logits), cfg.k)
    rows = np.arange(cfg.N)  # every row
    e_yg, counts, n_tok = _check_sampled(moe, mixtral, cfg, x, logits, out, rows)
    print(f"mid T={T}: counts={counts.tolist()} err={e_yg:.3e}")
    assert n_tok == T and e_yg <= TOL_BF16


@pytest.mark.parametrize("name,shape_weights", [(n, n) for n in DECODE_SIZED],
                         indirect=["shape_weights"])
def test_decode_layer_full_size(moe, shape_weights, name):
    """The one-call decode step at the full shapes: oracle parity, and the same bits as the
    four calls."""
    cfg = mi.CONFIGS[name]
    x, logits, _ = mi.make_activations(cfg)
    ref = orc.layer(mi.to_f64(x), logits, shape_weights["w1"], shape_weights["w3"],
                    shape_weights["w2"], cfg.k)
    xd, lg = to_dev(x), to_dev(logits)
    yg = torch.full((cfg.N, cfg.d), float("nan"), device="cuda")
    out = moe.moe_decode_layer(shape_weights["W"], xd, lg, cfg.k, yg=yg)
    four = moe.moe_layer(shape_weights["W"], xd, lg, cfg.k)
    torch.cuda.synchronize()
    _check_index_outputs(out, ref)
    e_yg, e_y = max_rel(to_host(out["yg"]), ref["yg"]), max_rel(to_host(out["y"]), ref["y"])
    print(f"decode_layer {name}: err yg={e_yg:.3e} y={e_y:.3e}")
    assert e_yg <= TOL_BF16 and e_y <= TOL_BF16
    assert torch.equal(out["yg"], four["yg"]) and torch.equal(out["y"], four["y"])


@pytest.mark.parametrize("name,shape_weights", [("decode_t1", "decode_t1"), ("e16_decode_t1", "e16_decode_t1")],
                         indirect=["shape_weights"])
def test_decode_block_full_size(moe, shape_weights, name):
    """The two-launch block step at the full shapes (one token): the small-row second
    projection is the kernel that runs (one slab), RMSNorm scale and logits from the gating
    sums, layer output + residual and the next block's sums against fp64."""
    cfg = mi.CONFIGS[name]
    eps = 1e-5
    T, E, k, d = cfg.T, cfg.E, cfg.k, cfg.d
    assert moe.moe_decode_block_supported(T, E, k, d, cfg.f)
    assert moe.moe_expert_ffn_plan(cfg.N, E, d, cfg.f)["n_parts"] == 1
    x, _, _ = mi.make_activations(cfg)
    x_in = (x * np.float32(2.5)).astype(np.float32)
    wg = mi.normal_f32(cfg.seed, 7, (d, E), d ** -0.5) * np.float32(2.0)
    wg_next = mi.normal_f32(cfg.seed, 8, (d, E), d ** -0.5)
    xd = to_dev(x_in)
    s0 = moe.moe_gate_sums(xd, to_dev(wg))
    out = moe.moe_decode_block(shape_weights["W"], xd, k, gate_sums=s0, n_shares=1, eps=eps,
                               w_gate_next=to_dev(wg_next))
    torch.cuda.synchronize()
    x64 = x_in.astype(np.float64)
    scale = 1.0 / np.sqrt((x64 ** 2).mean(axis=1) + eps)
    lg_ref = (x64 @ wg.astype(np.float64)) * scale[:, None]
    lg_gpu = to_host(out["logits"])
    assert np.max(np.abs(lg_gpu - lg_ref)) <= 2e-5 * max(1.0, np.max(np.abs(lg_ref)))
    ref = orc.layer(x64 * scale[:, None], lg_gpu, shape_weights["w1"], shape_weights["w3"],
                    shape_weights["w2"], k)
    _check_index_outputs(out, ref)
    x_out = to_host(out["x_out"])
    e_x = max_rel(x_out, x64 + ref["y"])
    xo64 = x_out.astype(np.float64)
    Sn_ref = np.concatenate([xo64 @ wg_next.astype(np.float64), (xo64 ** 2).sum(axis=1, keepdims=True)], axis=1)
    Sn_gpu = to_host(out["gate_sums_next"]).astype(np.float64).sum(axis=0)[:T * (E + 1)].reshape(T, E + 1)
    e_s = np.max(np.abs(Sn_gpu - Sn_ref)) / np.max(np.abs(Sn_ref))
    print(f"decode_block {name}: err x={e_x:.3e} sums={e_s:.3e}")
    assert e_x <= TOL_BF16 and e_s <= 1e-5
