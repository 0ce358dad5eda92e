"""GPU parity at the full layer shapes bench.py times: Mixtral-8x7B (d=4096,
f=14336, E=8, top-2, bf16 weights) and the 16-expert shape (d=4096, f=6400,
E=16, top-2), in the launch configuration of the bench.

The oracle runs whole for the decode-sized workloads (1 and 16 tokens); for the
4096-token prefill it runs on sampled rows of every expert segment (first, last
and two inner rows), because the full fp64 layer is ~2.9 TFLOP of CPU work."""
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


@pytest.mark.parametrize("name,shape_weights",
                         [(n, n) for n in ["prefill_t4096", "e16_prefill_t4096"]],
                         indirect=["shape_weights"])
def test_prefill_layer_sampled_rows(moe, shape_weights, name):
    mixtral = shape_weights
    cfg = mi.CONFIGS[name]
    x, logits, _ = mi.make_activations(cfg)
    idx, w = orc.route(logits, cfg.k)
    counts, offsets, perm, inv_perm, _ = orc.permute(idx, cfg.E, np.zeros((cfg.T, 1)))
    out = moe.moe_layer(mixtral["W"], to_dev(x), to_dev(logits), cfg.k)
    torch.cuda.synchronize()
    ref = dict(idx=idx, w=w, counts=counts, offsets=offsets, perm=perm, inv_perm=inv_perm)
    _check_index_outputs(out, ref)
    print("prefill counts", counts.tolist())
    # sampled rows of yg: first, last, two inner rows of each expert segment, plus rows of
    # several 16-row blocks of its first and last tile
    rows = []
    for e in range(cfg.E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi > lo:
            cand = {lo, hi - 1, lo + (hi - lo) // 3, lo + (2 * (hi - lo)) // 3}
            # and rows in other 16-row blocks of the first and the last 256-row tile
            last_tile = lo + ((hi - lo - 1) // 256) * 256
            cand |= {base + 16 * b + 5 for base in (lo, last_tile) for b in (1, 6, 11, 15)}
            rows += sorted(r for r in cand if lo <= r < hi)
    rows = np.array(rows)
    x64 = mi.to_f64(x)
    xg_s = x64[perm[rows] // cfg.k]
    seg = np.searchsorted(offsets[1:], rows, side="right")
    s_off = np.concatenate([[0], np.cumsum(np.bincount(seg, minlength=cfg.E))]).astype(np.int32)
    yg_ref = orc.expert_ffn(xg_s, s_off, mixtral["w1"], mixtral["w3"], mixtral["w2"])
    yg = to_host(out["yg"])
    scale = float(np.max(np.abs(yg_ref)))
    e_yg = float(np.max(np.abs(yg[rows] - yg_ref)) / scale)
    print(f"prefill sampled yg rows={len(rows)} err={e_yg:.3e}")
    assert e_yg <= TOL_BF16
    # combine on the GPU's own yg must agree with the oracle's combine of it (all tokens)
    y_from_gpu_yg = orc.combine(yg.astype(np.float64), inv_perm, w)
    assert max_rel(to_host(out["y"]), y_from_gpu_yg) <= 1e-6
    # and tokens whose k rows were all sampled are checked end to end
    inv_rows = {int(r): i for i, r in enumerate(rows)}
    toks = [t for t in range(cfg.T)
            if all(int(inv_perm[t * cfg.k + j]) in inv_rows for j in range(cfg.k))]
    for t in toks:
        y_ref = sum(w[t, j] * yg_ref[inv_rows[int(inv_perm[t * cfg.k + j])]] for j in range(cfg.k))
        assert np.max(np.abs(to_host(out["y"][t]) - y_ref)) / scale <= TOL_BF16
    # no NaN/Inf anywhere and every row written (magnitudes match the sampled scale)
    assert np.isfinite(yg).all()
    assert np.all(np.max(np.abs(yg), axis=1) > 1e-3 * scale)
