"""GPU parity of the layer-stack workload (RMSNorm -> router logits -> MoE layer
-> residual add, repeated) and of its support kernels.

Routing is compared bit for bit under teacher forcing: the oracle's stack routes
on the GPU's own fp32 router logits of every layer (its activations are fp64 and
drift from the GPU's within tolerance, so its own logits may differ in the last
bits and flip a near-tie).  The final activations must agree within 2e-2."""
import numpy as np
import pytest
import torch

import moe_inputs as mi
from gpu_util import max_rel, pack_layer, to_dev, to_host
from oracle import moe_oracle as orc

pytestmark = pytest.mark.gpu
TOL_BF16 = 2e-2


@pytest.fixture(scope="module")
def moe():
    assert torch.cuda.is_available()
    import paper_2402_07033_amd as m
    m.lib()
    return m


def test_support_kernels(moe):
    rng = np.random.default_rng(3)
    for T, d, E in [(1, 4096, 8), (16, 256, 8), (513, 1024, 16), (40, 64, 3)]:
        x = (rng.standard_normal((T, d)) * 3.0).astype(np.float32)
        wg = (rng.standard_normal((d, E)) / np.sqrt(d)).astype(np.float32)
        h_ref = orc.rmsnorm(x.astype(np.float64), 1e-5)
        h = moe.moe_rmsnorm(to_dev(x), 1e-5)
        assert max_rel(to_host(h), h_ref) <= 2e-6
        lg_ref = orc.router_logits(to_host(h).astype(np.float64), wg)
        lg = moe.moe_router_logits(h, to_dev(wg))
        assert np.max(np.abs(to_host(lg) - lg_ref)) <= 1e-5 * max(1.0, np.max(np.abs(lg_ref)))
        # both in one launch: same h, logits = (x . w_gate) / rms(x) against the fp64 oracle
        h2, lg2 = moe.moe_rmsnorm_router_logits(to_dev(x), to_dev(wg), 1e-5)
        assert max_rel(to_host(h2), h_ref) <= 2e-6
        lg_ref2 = orc.router_logits(h_ref, wg)
        assert np.max(np.abs(to_host(lg2) - lg_ref2)) <= 2e-5 * max(1.0, np.max(np.abs(lg_ref2)))
        y = rng.standard_normal((T, d)).astype(np.float32)
        xd = to_dev(x)
        moe.moe_residual_add(xd, to_dev(y))
        assert (to_host(xd) == x + y).all()
    # more than 16 experts: the separate kernels serve, the fused call says unsupported
    x = to_dev(rng.standard_normal((5, 256)).astype(np.float32))
    wg = to_dev((rng.standard_normal((256, 24)) / 16.0).astype(np.float32))
    lg = moe.moe_router_logits(moe.moe_rmsnorm(x, 1e-5), wg)
    assert lg.shape == (5, 24) and torch.isfinite(lg).all()
    with pytest.raises(moe.MoeError):
        moe.moe_rmsnorm_router_logits(x, wg, 1e-5)


def test_fused_front_ends_match_separate_calls(moe):
    rng = np.random.default_rng(11)
    d, E, k = 4096, 8, 2
    wg = to_dev((rng.standard_normal((d, E)) / np.sqrt(d)).astype(np.float32))
    i32 = dict(dtype=torch.int32, device="cuda")

    def outs(T, N):
        return (torch.zeros(E, **i32), torch.zeros(E + 1, **i32), torch.zeros(N, **i32),
                torch.zeros(N, **i32), torch.zeros((N, d), device="cuda"))

    for T in (1, 2, 4, 7, 16):
        N = T * k
        x = to_dev(rng.standard_normal((T, d)).astype(np.float32) * 2.0)
        # --- route + permute on given logits ---
        lg = to_dev(rng.standard_normal((T, E)).astype(np.float32))
        idx_s, w_s = moe.moe_route(lg, k)
        sep = moe.moe_permute(idx_s, E, x)
        idx_f = torch.zeros((T, k), **i32)
        w_f = torch.zeros((T, k), device="cuda")
        fo = outs(T, N)
        moe.moe_route_permute(lg, k, x, idx_f, w_f, fo)
        assert torch.equal(idx_f, idx_s) and torch.equal(w_f, w_s)
        for a, b in zip(fo, sep):
            assert torch.equal(a, b)
        # oracle: bit-exact routing on the same logits
        ref_idx, _ = orc.route(to_host(lg), k)
        assert (to_host(idx_f) == ref_idx).all()
        if T > 4:
            continue
        # --- rmsnorm + logits + route + permute ---
        h_s = moe.moe_rmsnorm(x, 1e-5)
        h_f = torch.zeros_like(x)
        lg_f = torch.zeros((T, E), device="cuda")
        fo = outs(T, N)
        moe.moe_norm_route_permute(x, wg, k, 1e-5, h_f, lg_f, idx_f, w_f, fo)
        assert max_rel(to_host(h_f), to_host(h_s)) <= 2e-6
        lg_ref = orc.router_logits(to_host(h_f).astype(np.float64), to_host(wg))
        assert np.max(np.abs(to_host(lg_f) - lg_ref)) <= 2e-5 * max(1.0, np.max(np.abs(lg_ref)))
        # routing is bit-exact on the logits the kernel itself reports
        ref_idx, ref_w = orc.route(to_host(lg_f), k)
        assert (to_host(idx_f) == ref_idx).all()
        assert np.max(np.abs(to_host(w_f) - ref_w)) <= 1e-6
        rc, ro, rp, ri, _ = orc.permute(ref_idx, E, np.zeros((T, 1)))
        assert (to_host(fo[0]) == rc).all() and (to_host(fo[1]) == ro).all()
        assert (to_host(fo[2]) == rp).all() and (to_host(fo[3]) == ri).all()
        assert torch.equal(fo[4], h_f[torch.from_numpy(rp // k).cuda().long()])
    # combine + residual == combine then add
    T = 5
    yg = to_dev(rng.standard_normal((T * k, d)).astype(np.float32))
    inv = to_dev(rng.permutation(T * k).astype(np.int32))
    w = to_dev(rng.random((T, k)).astype(np.float32))
    x0 = rng.standard_normal((T, d)).astype(np.float32)
    xa, xb = to_dev(x0.copy()), to_dev(x0.copy())
    moe.moe_combine_residual(yg, inv, w, xa)
    moe.moe_residual_add(xb, moe.moe_combine(yg, inv, w))
    assert torch.equal(xa, xb)


@pytest.mark.parametrize("T,E,k,k_prev,d", [(1, 8, 2, 2, 4096), (1, 16, 2, 2, 4096), (2, 8, 2, 3, 512),
                                            (4, 6, 3, 2, 256), (3, 16, 8, 8, 4096)])
def test_seam_call_matches_separate_calls(moe, T, E, k, k_prev, d):
    """moe_combine_norm_route_permute == moe_combine_residual followed by
    moe_norm_route_permute, bit for bit (same fp32 arithmetic)."""
    rng = np.random.default_rng(100 * T + E + k)
    i32 = dict(dtype=torch.int32, device="cuda")
    wg = to_dev((rng.standard_normal((d, E)) / np.sqrt(d)).astype(np.float32))
    Np, N = T * k_prev, T * k
    yg = to_dev(rng.standard_normal((Np + 3, d)).astype(np.float32))
    inv = to_dev(rng.permutation(Np + 3)[:Np].astype(np.int32))
    wp = to_dev(rng.random((T, k_prev)).astype(np.float32))
    x0 = (rng.standard_normal((T, d)) * 1.5).astype(np.float32)

    def outs():
        return (torch.zeros(E, **i32), torch.zeros(E + 1, **i32), torch.zeros(N, **i32),
                torch.zeros(N, **i32), torch.zeros((N, d), device="cuda"))

    def small():
        return (torch.zeros((T, d), device="cuda"), torch.zeros((T, E), device="cuda"),
                torch.zeros((T, k), **i32), torch.zeros((T, k), device="cuda"))

    # separate calls
    xa = to_dev(x0.copy())
    moe.moe_combine_residual(yg, inv, wp, xa)
    ha, la, ia, wa = small()
    oa = outs()
    moe.moe_norm_route_permute(xa, wg, k, 1e-5, ha, la, ia, wa, oa)
    # one launch
    xin, xout = to_dev(x0.copy()), torch.zeros((T, d), device="cuda")
    hb, lb, ib, wb = small()
    ob = outs()
    moe.moe_combine_norm_route_permute(yg, inv, wp, xin, xout, wg, k, 1e-5, hb, lb, ib, wb, ob)
    torch.cuda.synchronize()
    assert torch.equal(xin, to_dev(x0))  # the input stream is left alone
    assert torch.equal(xout, xa)
    assert torch.equal(hb, ha) and torch.equal(lb, la)
    assert torch.equal(ib, ia) and torch.equal(wb, wa)
    for a, b in zip(oa, ob):
        assert torch.equal(a, b)
    # aliasing the previous block's buffers is refused
    with pytest.raises(moe.MoeError):
        moe.moe_combine_norm_route_permute(yg, inv, wp, xin, xin, wg, k, 1e-5, hb, lb, ib, wb, ob)
    if k == k_prev:
        with pytest.raises(moe.MoeError):
            moe.moe_combine_norm_route_permute(yg, ob[3], wb, xin, xout, wg, k, 1e-5, hb, lb, ib,
                                               wb, ob)


@pytest.mark.parametrize("T", [3, 1])
def test_stack_seam_on_off(moe, T):
    """T = 3: the stack with the combine folded into the next front end gives the same bits
    as with the separate combine+residual launches.  T = 1 runs every block as the two
    launches of moe_decode_block, whose sums are ordered differently: same routing, final
    activations equal to rounding."""
    L, k = 5, 2
    cfgs = [mi.small_config(f"m{l}", T, 512, 1024, 8, k, 4100 + l, w_dtype=mi.BF16) for l in range(L)]
    layers = []
    for cfg in cfgs:
        w1, w3, w2 = mi.make_weights(cfg, threads=8)
        w_gate = mi.normal_f32(cfg.seed, 1, (cfg.d, cfg.E), cfg.d ** -0.5)
        layers.append((pack_layer(mi.LayerInputs(cfg, None, None, w1, w3, w2, w_gate)),
                       to_dev(w_gate)))
    assert moe.moe_decode_block_supported(T, 8, k, 512, 1024) == (T == 1)
    x0 = mi.normal_f32(4100, 0, (T, 512))
    res = []
    for seam in (True, False):
        xd = to_dev(x0.copy())
        idx = []
        moe.moe_stack_forward(layers, xd, k, idx_out=idx, seam=seam)
        torch.cuda.synchronize()
        res.append((to_host(xd), [to_host(i) for i in idx]))
    if T == 1:
        assert max_rel(res[0][0], res[1][0].astype(np.float64)) <= 1e-5
    else:
        assert (res[0][0] == res[1][0]).all()
    for a, b in zip(res[0][1], res[1][1]):
        assert (a == b).all()
    for W, _ in layers:
        W.free()


@pytest.mark.parametrize("T,k,E,d,f", [(1, 2, 8, 1024, 3584), (2, 2, 8, 512, 1024), (1, 4, 16, 2048, 1024),
                                       (4, 1, 4, 256, 512), (1, 2, 8, 256, 1600), (1, 1, 3, 4096, 512),
                                       (3, 1, 9, 320, 640), (2, 1, 15, 4096, 512)])
def test_decode_block(moe, T, k, E, d, f):
    """moe_decode_block against the fp64 oracle: RMSNorm scale and router logits derived from
    the gating sums, layer output + residual, the next block's sums; against moe_decode_layer
    (same bits on given logits); in place; and run to run."""
    eps = 1e-5
    cfg = mi.small_config("blk", T, d, f, E, k, 5200 + T + d + E, w_dtype=mi.BF16)
    li = mi.make_layer(cfg, threads=4)
    W = pack_layer(li)
    assert moe.moe_decode_block_supported(T, E, k, d, f)
    stride = moe.moe_gate_sums_stride(T, E)
    assert stride == 32 and T * (E + 1) <= stride
    x_in = (li.x * np.float32(1.7)).astype(np.float32)            # the residual stream
    wg = mi.normal_f32(cfg.seed, 4, (d, E), d ** -0.5) * np.float32(3.0)
    wg_next = mi.normal_f32(cfg.seed, 5, (d, E), d ** -0.5)
    xd = to_dev(x_in)
    # ---- the first block's sums: one share
    s0 = moe.moe_gate_sums(xd, to_dev(wg))
    x64 = x_in.astype(np.float64)
    S_ref = np.concatenate([x64 @ wg.astype(np.float64), (x64 ** 2).sum(axis=1, keepdims=True)], axis=1)
    S_gpu = to_host(s0)[:T * (E + 1)].reshape(T, E + 1)
    assert np.max(np.abs(S_gpu - S_ref)) <= 1e-5 * np.max(np.abs(S_ref))
    # ---- the block
    out = moe.moe_decode_block(W, xd, k, gate_sums=s0, n_shares=1, eps=eps, w_gate_next=to_dev(wg_next))
    torch.cuda.synchronize()
    scale_ref = 1.0 / np.sqrt(S_ref[:, E] / d + eps)
    lg_ref = S_ref[:, :E] * scale_ref[:, None]
    lg_gpu = to_host(out["logits"])
    e_l = np.max(np.abs(lg_gpu - lg_ref)) / max(1.0, np.max(np.abs(lg_ref)))
    # routing on the logits the kernel reports (a near-tie may fall either way in fp32)
    h64 = x64 * scale_ref[:, None]
    ref = orc.layer(h64, lg_gpu, li.w1, li.w3, li.w2, k)
    for key in ("idx", "counts", "offsets", "perm", "inv_perm"):
        assert (to_host(out[key]) == ref[key]).all(), key
    assert np.max(np.abs(to_host(out["w"]) - ref["w"])) <= 1e-6
    x_out = to_host(out["x_out"])
    assert not np.isnan(x_out).any()
    e_x = max_rel(x_out, x64 + ref["y"])
    # the next block's sums, in fp64 from the rows the kernel itself wrote, shares added up
    xo64 = x_out.astype(np.float64)
    Sn_ref = np.concatenate([xo64 @ wg_next.astype(np.float64), (xo64 ** 2).sum(axis=1, keepdims=True)], axis=1)
    shares = to_host(out["gate_sums_next"]).astype(np.float64)
    assert shares.shape == (d // 16, stride)
    Sn_gpu = shares.sum(axis=0)[:T * (E + 1)].reshape(T, E + 1)
    e_s = np.max(np.abs(Sn_gpu - Sn_ref)) / np.max(np.abs(Sn_ref))
    print(f"decode_block T={T} k={k} E={E} d={d} f={f}: err x={e_x:.3e} logits={e_l:.3e} sums={e_s:.3e}")
    assert e_x <= 1e-4 and e_l <= 2e-5 and e_s <= 1e-5
    # chained: the next call derives its logits from these shares
    nxt = moe.moe_decode_block(W, out["x_out"], k, gate_sums=out["gate_sums_next"], eps=eps)
    scale_n = 1.0 / np.sqrt(Sn_ref[:, E] / d + eps)
    lgn_ref = Sn_ref[:, :E] * scale_n[:, None]
    assert np.max(np.abs(to_host(nxt["logits"]) - lgn_ref)) <= 2e-5 * max(1.0, np.max(np.abs(lgn_ref)))
    assert nxt["gate_sums_next"] is None
    # given logits, no scale: the same bits as moe_decode_layer plus the residual add
    lg = to_dev(li.logits)
    dl = moe.moe_decode_layer(W, xd, lg, k)
    plain = moe.moe_decode_block(W, xd, k, logits=lg)
    assert torch.equal(plain["x_out"], xd + dl["y"]) and torch.equal(plain["idx"], dl["idx"])
    # in place; repeated: identical bits
    for _ in range(5):
        xi = to_dev(x_in.copy())
        again = moe.moe_decode_block(W, xi, k, gate_sums=s0, eps=eps, x_out=xi, w_gate_next=to_dev(wg_next))
        assert torch.equal(xi, out["x_out"]) and torch.equal(again["logits"], out["logits"])
        n = T * (E + 1)   # (the padding floats of a share are never written)
        assert torch.equal(again["gate_sums_next"][:, :n], out["gate_sums_next"][:, :n])
    W.free()


def test_decode_block_unsupported_and_errors(moe):
    cfg = mi.small_config("blke", 4, 256, 512, 8, 2, 97, w_dtype=mi.BF16)
    li = mi.make_layer(cfg, threads=1)
    W = pack_layer(li)
    x, lg = to_dev(li.x), to_dev(li.logits)
    assert not moe.moe_decode_block_supported(4, 8, 2, 256, 512)      # 8 routed rows
    assert not moe.moe_decode_block_supported(4, 16, 1, 256, 512)     # 4 * 17 sums
    with pytest.raises(moe.MoeError) as ei:
        moe.moe_decode_block(W, x, 2, logits=lg)
    assert ei.value.status == -2
    x1, lg1 = x[:1].contiguous(), lg[:1].contiguous()
    with pytest.raises(moe.MoeError) as ei:       # workspace too small
        moe.moe_decode_block(W, x1, 2, logits=lg1, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert ei.value.status == -3
    sums = torch.zeros((16, 32), device="cuda")
    with pytest.raises(moe.MoeError) as ei:       # the next sums over this call's sums
        moe.moe_decode_block(W, x1, 2, gate_sums=sums, n_shares=16,
                             w_gate_next=torch.zeros((256, 8), device="cuda"), gate_sums_next=sums)
    assert ei.value.status == -1
    with pytest.raises(moe.MoeError) as ei:       # more shares than a wave adds
        moe.moe_decode_block(W, x1, 2, gate_sums=torch.zeros((300, 32), device="cuda"), n_shares=300)
    assert ei.value.status == -1
    W.free()


def _run_stack(moe, cfgs, T, k, fused=True, free_running=True):
    """cfgs: one MoEConfig per layer.  Returns (gpu final x, oracle result, info)."""
    host_layers, dev_layers = [], []
    for cfg in cfgs:
        w1, w3, w2 = mi.make_weights(cfg, threads=16)
        w_gate = mi.normal_f32(cfg.seed, 1, (cfg.d, cfg.E), cfg.d ** -0.5)
        li = mi.LayerInputs(cfg, None, None, w1, w3, w2, w_gate)
        dev_layers.append((pack_layer(li), to_dev(w_gate)))
        host_layers.append((w_gate, w1, w3, w2))
    x0 = mi.normal_f32(cfgs[0].seed, 0, (T, cfgs[0].d))
    xd = to_dev(x0.copy())
    logits, idx = [], []
    moe.moe_stack_forward(dev_layers, xd, k, logits_out=logits, idx_out=idx, fused=fused)
    torch.cuda.synchronize()
    gpu_logits = [to_host(t) for t in logits]
    ref = orc.stack(x0.astype(np.float64), host_layers, k, forced_logits=gpu_logits)
    for l in range(len(cfgs)):
        assert (to_host(idx[l]) == ref["idx"][l]).all(), f"routing differs at layer {l}"
    info = {}
    if free_running:  # information only: the oracle routing on its own logits
        free = orc.stack(x0.astype(np.float64), host_layers, k)
        same = np.mean([np.mean(a == b) for a, b in zip(free["idx"], ref["idx"])])
        info = dict(same_routing_free_running=float(same), err_free=max_rel(to_host(xd), free["x"]))
    for W, _ in dev_layers:
        W.free()
    return to_host(xd), ref, info


@pytest.mark.parametrize("T,L,d,f,fused", [(1, 6, 256, 512, True), (1, 6, 256, 512, False),
                                           (3, 4, 256, 512, True), (24, 4, 256, 512, True),
                                           (300, 3, 256, 512, True), (7, 4, 512, 1024, False)])
def test_stack_small_shapes(moe, T, L, d, f, fused):
    cfgs = [mi.small_config(f"s{l}", T, d, f, 8, 2, 3000 + 10 * l + T, w_dtype=mi.BF16)
            for l in range(L)]
    x, ref, info = _run_stack(moe, cfgs, T, 2, fused=fused)
    err = max_rel(x, ref["x"])
    print(f"stack T={T} L={L} d={d}: err={err:.3e} {info}")
    assert err <= TOL_BF16


# The stack workload at the Mixtral shape (independent seeded weights per layer, 2.8 GB
# each): single-token decode through 8 layers (the one-launch seam between blocks, reduction
# parts added inside it), beam-sized and 512-token prefill through 2 layers (the whole fp64
# oracle: 2 x 1024 rows).
@pytest.mark.parametrize("T,L", [(1, 8), (16, 2), (512, 2)])
def test_stack_mixtral_shape(moe, T, L):
    cfgs = [mi.stack_layer_config(l, T) for l in range(L)]
    if T == 512:
        pl = moe.moe_expert_ffn_plan(T * 2, 8, 4096, 14336)
        assert (pl["path"], pl["up_tile_rows"]) == (moe.MOE_FFN_GROUPED, 192)
    x, ref, info = _run_stack(moe, cfgs, T, 2, free_running=(T != 512))
    err = max_rel(x, ref["x"])
    print(f"stack mixtral T={T} L={L}: err={err:.3e} {info}")
    assert err <= TOL_BF16


@pytest.mark.parametrize("T,E,k,k_prev,d,P", [(1, 8, 2, 2, 4096, 4), (4, 8, 2, 2, 512, 2),
                                              (2, 16, 3, 3, 256, 3)])
def test_seam_call_with_reduction_parts(moe, T, E, k, k_prev, d, P):
    """The seam call on P unsummed reduction parts == moe_combine_parts (residual form)
    followed by moe_norm_route_permute, bit for bit; more than 4 parts are refused."""
    rng = np.random.default_rng(7 * T + P)
    i32 = dict(dtype=torch.int32, device="cuda")
    wg = to_dev((rng.standard_normal((d, E)) / np.sqrt(d)).astype(np.float32))
    Np, N = T * k_prev, T * k
    parts = to_dev(rng.standard_normal((P, Np, d)).astype(np.float32))
    inv = to_dev(rng.permutation(Np).astype(np.int32))
    wp = to_dev(rng.random((T, k_prev)).astype(np.float32))
    x0 = (rng.standard_normal((T, d)) * 1.5).astype(np.float32)

    def outs():
        return (torch.zeros(E, **i32), torch.zeros(E + 1, **i32), torch.zeros(N, **i32),
                torch.zeros(N, **i32), torch.zeros((N, d), device="cuda"))

    def small():
        return (torch.zeros((T, d), device="cuda"), torch.zeros((T, E), device="cuda"),
                torch.zeros((T, k), **i32), torch.zeros((T, k), device="cuda"))

    xa = to_dev(x0.copy())
    moe.moe_combine_parts(parts, P, inv, wp, y=xa, residual=True)
    ha, la, ia, wa = small()
    oa = outs()
    moe.moe_norm_route_permute(xa, wg, k, 1e-5, ha, la, ia, wa, oa)
    xin, xout = to_dev(x0.copy()), torch.zeros((T, d), device="cuda")
    hb, lb, ib, wb = small()
    ob = outs()
    moe.moe_combine_norm_route_permute(parts, inv, wp, xin, xout, wg, k, 1e-5, hb, lb, ib, wb, ob,
                                       n_parts_prev=P)
    torch.cuda.synchronize()
    assert torch.equal(xout, xa)
    assert torch.equal(hb, ha) and torch.equal(lb, la)
    assert torch.equal(ib, ia) and torch.equal(wb, wa)
    for a, b in zip(oa, ob):
        assert torch.equal(a, b)
    # and against fp64: x_out = x + sum_j w_j * (sum of the parts)
    yg64 = to_host(parts).astype(np.float64).sum(axis=0)
    ref = x0.astype(np.float64) + orc.combine(yg64, to_host(inv), to_host(wp).astype(np.float64))
    assert max_rel(to_host(xout), ref) <= 2e-6
    five = torch.zeros((5, Np, d), device="cuda")
    with pytest.raises(moe.MoeError) as ei:
        moe.moe_combine_norm_route_permute(five, inv, wp, xin, xout, wg, k, 1e-5, hb, lb, ib, wb,
                                           ob, n_parts_prev=5)
    assert ei.value.status == -2
