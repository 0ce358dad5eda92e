"""The decode paths under HIP graph capture: the library launches kernels only (no memset, no
allocation, no host synchronisation), so a captured decode stack replays bit for bit.

Every replay is checked against the eager result of the same input, with eager work and
synchronisations between the replays."""
import numpy as np
import pytest
import torch

import moe_inputs as mi
from gpu_util import pack_layer, to_dev, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def moe():
    assert torch.cuda.is_available()
    import paper_2402_07033_amd as m
    m.lib()
    return m


def _layers(T, d, f, E, k, L, seed):
    out = []
    for l in range(L):
        cfg = mi.small_config(f"g{l}", T, d, f, E, k, seed + l, w_dtype=mi.BF16)
        w1, w3, w2 = mi.make_weights(cfg, threads=8)
        w_gate = mi.normal_f32(cfg.seed, 1, (d, E), d ** -0.5)
        out.append((pack_layer(mi.LayerInputs(cfg, None, None, w1, w3, w2, w_gate)), to_dev(w_gate)))
    return out


@pytest.mark.parametrize("T,k", [(1, 2), (3, 2), (16, 2)])
def test_stack_forward_replays_from_a_graph(moe, T, k):
    """T = 1: two launches per block (moe_decode_block); T = 3: the seam kernel and the
    reduction parts; T = 16: the separate front-end kernels."""
    d, f, E, L = 512, 1024, 8, 4
    layers = _layers(T, d, f, E, k, L, 8100 + T)
    bufs = moe.StackBuffers(T, E, k, d, f)
    xs = [to_dev(mi.normal_f32(8200 + i, 0, (T, d))) for i in range(3)]
    # eager results (also the warm-up: one-time attribute and occupancy queries happen here)
    eager = []
    for x0 in xs:
        x = x0.clone()
        moe.moe_stack_forward(layers, x, k, bufs=bufs)
        torch.cuda.synchronize()
        eager.append(x.clone())
    x_static = xs[0].clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):       # capture on a stream of the default priority
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            moe.moe_stack_forward(layers, x_static, k, bufs=bufs)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for rep in range(2):
        for x0, ref in zip(xs, eager):
            x_static.copy_(x0)
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(x_static, ref), f"replay {rep} differs from the eager pass"
            # eager work between the replays
            y = x0.clone()
            moe.moe_stack_forward(layers, y, k, bufs=bufs)
            torch.cuda.synchronize()
            assert torch.equal(y, ref)
    del graph
    for W, _ in layers:
        W.free()


def test_decode_layer_replays_from_a_graph(moe):
    T, d, f, E, k = 4, 1024, 2048, 8, 2
    cfg = mi.small_config("gd", T, d, f, E, k, 8300, w_dtype=mi.BF16, zipf_s=1.2)
    li = mi.make_layer(cfg, threads=8)
    W = pack_layer(li)
    i32 = dict(dtype=torch.int32, device="cuda")
    N = T * k
    x, lg = to_dev(li.x), to_dev(li.logits)
    outs = (torch.empty(E, **i32), torch.empty(E + 1, **i32), torch.empty(N, **i32), torch.empty(N, **i32), None)
    idx, w = torch.empty((T, k), **i32), torch.empty((T, k), device="cuda")
    ws = torch.empty(moe.moe_expert_ffn_workspace(N, E, d, f, moe.MOE_F32), dtype=torch.uint8, device="cuda")
    y = torch.empty((T, d), device="cuda")
    ref = moe.moe_decode_layer(W, x, lg, k)["y"].clone()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            moe.moe_decode_layer(W, x, lg, k, idx=idx, weights=w, out=outs, workspace=ws, y=y)
    torch.cuda.current_stream().wait_stream(side)
    for _ in range(3):
        y.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, ref)
        assert torch.equal(moe.moe_decode_layer(W, x, lg, k)["y"], ref)
    del graph
    W.free()
