"""The entry point that allocates nothing (moe_expert_ffn_noalloc: scratch in a static
device array of the library) against moe_expert_ffn with a caller's workspace: same kernels,
so the same bits, on two calls in a row, the second with a smaller input (the array keeps
the first call's contents)."""
import numpy as np
import pytest
import torch

import moe_inputs as mi
from gpu_util import pack_layer, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def moe():
    assert torch.cuda.is_available()
    import paper_2402_07033_amd as m
    m.lib()
    return m


def _routed(moe, W, li, k, T):
    x, lg = to_dev(li.x[:T].copy()), to_dev(li.logits[:T].copy())
    idx, _ = moe.moe_route(lg, k)
    _, offsets, _, _, xg = moe.moe_permute(idx, W.E, x)
    return xg, offsets


@pytest.mark.parametrize("d,f,E,k,T1,T2,wdt", [(1024, 7168, 8, 2, 16, 5, mi.BF16),
                                              (4096, 14336, 8, 2, 16, 1, mi.BF16),
                                              (256, 512, 8, 2, 16, 3, mi.F32)])
def test_noalloc_matches_workspace_call_twice(moe, d, f, E, k, T1, T2, wdt):
    cfg = mi.small_config("na", T1, d, f, E, k, 2100 + d, w_dtype=wdt, zipf_s=1.2)
    li = mi.make_layer(cfg, threads=16)
    W = pack_layer(li)
    for T in (T1, T2):   # the second call is smaller and finds the first call's scratch
        xg, offsets = _routed(moe, W, li, k, T)
        ref = moe.moe_expert_ffn(W, xg, offsets)
        yg = torch.full((T * k, d), float("nan"), device="cuda")
        moe.moe_expert_ffn_noalloc(W, xg, offsets, yg)
        torch.cuda.synchronize()
        assert torch.isfinite(yg).all()
        assert torch.equal(yg, ref), f"T={T}"
    W.free()


def test_noalloc_rejects_what_does_not_fit(moe):
    assert moe.moe_expert_ffn_noalloc_max_bytes() == 32 << 20
    cfg = mi.small_config("nb", 4, 256, 512, 8, 2, 2200, w_dtype=mi.BF16)
    W = pack_layer(mi.make_layer(cfg, threads=1))
    N = 40000   # prefill-sized: the grouped kernels' scratch is far beyond 32 MiB
    xg = torch.zeros((N, 256), dtype=torch.bfloat16, device="cuda")
    off = torch.tensor([0] + [N] * 8, dtype=torch.int32, device="cuda")
    yg = torch.zeros((N, 256), device="cuda")
    with pytest.raises(moe.MoeError) as ei:
        moe.moe_expert_ffn_noalloc(W, xg, off, yg)
    assert ei.value.status == -3
    # an empty call is a no-op, as in moe_expert_ffn
    moe.moe_expert_ffn_noalloc(W, xg[:0], torch.zeros(9, dtype=torch.int32, device="cuda"), yg[:0])
    W.free()
