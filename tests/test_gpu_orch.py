"""GPU parity of the split-layer execution (the paper's Algorithm 1 over the expert kernels):
whatever Algorithm 1 decides per expert -- resident on the device, device after a weight
transfer, or host -- the layer's output must match the fp64 oracle, and the decisions must be
those of the plain restatement in oracle/orch_oracle.py."""
import numpy as np
import pytest
import torch

import moe_inputs as mi
from gpu_util import max_rel, to_dev, to_host
from oracle import moe_oracle as orc
from oracle import orch_oracle as oo

pytestmark = pytest.mark.gpu
TOL_BF16 = 2e-2


@pytest.fixture(scope="module")
def moe():
    assert torch.cuda.is_available()
    import paper_2402_07033_amd as m
    m.lib()
    return m


# latency constants that force each branch of Algorithm 1 for the non-resident experts
ALWAYS_CPU = dict(gpu_lat_us=1e6, cpu_lat_us_per_row=1.0, transfer_lat_us=1e6)
ALWAYS_TRANSFER = dict(gpu_lat_us=0.0, cpu_lat_us_per_row=1.0, transfer_lat_us=0.0)
MIXED = dict(gpu_lat_us=10.0, cpu_lat_us_per_row=10.0, transfer_lat_us=30.0)   # host up to 4 rows


@pytest.mark.parametrize("T,d,f,E,k,at_gpu,lat", [
    (16, 256, 512, 8, 2, [1, 0, 1, 0, 0, 1, 0, 0], ALWAYS_CPU),
    (16, 256, 512, 8, 2, [1, 0, 1, 0, 0, 1, 0, 0], ALWAYS_TRANSFER),
    (24, 512, 1024, 8, 2, [0, 1, 0, 0, 1, 0, 0, 0], MIXED),
    (300, 256, 512, 4, 2, [0, 1, 0, 1], MIXED),        # prefill-sized segments on both sides
    (5, 256, 7168, 4, 1, [0, 0, 0, 0], MIXED),         # nothing resident
    (9, 256, 512, 4, 2, [1, 1, 1, 1], ALWAYS_CPU)])    # everything resident
def test_split_layer_matches_oracle(moe, T, d, f, E, k, at_gpu, lat):
    cfg = mi.small_config("orch", T, d, f, E, k, 3300 + T + d, w_dtype=mi.BF16, zipf_s=1.2)
    li = mi.make_layer(cfg, threads=4)
    ref = orc.layer(mi.to_f64(li.x), li.logits, li.w1, li.w3, li.w2, k)
    layer = moe.OrchLayer(li.w1, li.w3, li.w2, at_gpu, max_rows=cfg.N)
    idx, w = moe.moe_route(to_dev(li.logits), k)
    counts, offsets, perm, inv_perm, xg = moe.moe_permute(idx, E, to_dev(li.x))
    yg = torch.full((cfg.N, d), float("nan"), device="cuda")
    for rep in range(2):   # the second call reuses the staging slot and the pinned buffers
        _, dec = layer.expert_ffn(lat, xg, offsets, yg=yg)
        torch.cuda.synchronize()
        assert (dec == oo.decide(at_gpu, ref["counts"], lat)).all()
        e_yg = max_rel(to_host(yg), ref["yg"])
        assert e_yg <= TOL_BF16, (rep, e_yg)
        yg_h = to_host(yg)
        # rows that ran on the host are fp32 arithmetic on exact bf16 weights: tighter
        for j in range(E):
            if dec[j] == oo.CPU:
                lo, hi = ref["offsets"][j], ref["offsets"][j + 1]
                assert max_rel(yg_h[lo:hi], ref["yg"][lo:hi]) <= 1e-5
    y = moe.moe_combine(yg, inv_perm, w)
    assert max_rel(to_host(y), ref["y"]) <= TOL_BF16
    print(f"split layer T={T} at_gpu={at_gpu}: decisions={dec.tolist()} counts={ref['counts'].tolist()} "
          f"err={e_yg:.3e}")
    layer.free()


def test_calibration_and_errors(moe):
    cfg = mi.small_config("cal", 16, 1024, 2048, 4, 2, 3400, w_dtype=mi.BF16)
    li = mi.make_layer(cfg, threads=4)
    layer = moe.OrchLayer(li.w1, li.w3, li.w2, [1, 0, 1, 0], max_rows=32)
    lat = layer.calibrate()
    print("calibrated latency model:", lat)
    assert all(v > 0 and np.isfinite(v) for v in lat.values())
    # the calibrated model drives a call like any other
    idx, w = moe.moe_route(to_dev(li.logits), 2)
    counts, offsets, perm, inv_perm, xg = moe.moe_permute(idx, 4, to_dev(li.x))
    yg, dec = layer.expert_ffn(lat, xg, offsets)
    torch.cuda.synchronize()
    ref = orc.layer(mi.to_f64(li.x), li.logits, li.w1, li.w3, li.w2, 2)
    assert (dec == oo.decide([1, 0, 1, 0], ref["counts"], lat)).all()
    assert max_rel(to_host(yg), ref["yg"]) <= TOL_BF16
    # more rows than the handle was created for
    big = torch.zeros((64, 1024), device="cuda")
    off = torch.tensor([0, 64, 64, 64, 64], dtype=torch.int32, device="cuda")
    with pytest.raises(moe.MoeError):
        layer.expert_ffn(lat, big, off)
    layer.free()
    # a layer with nothing in host memory has nothing to calibrate against
    full = moe.OrchLayer(li.w1, li.w3, li.w2, [1, 1, 1, 1], max_rows=32)
    with pytest.raises(moe.MoeError) as ei:
        full.calibrate()
    assert ei.value.status == -2
    full.free()
