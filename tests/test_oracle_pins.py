"""Pins of the CPU oracle (oracle/moe_oracle.c) to things other than itself:
closed forms, invariants, hand-worked index examples, numpy library routines
and a dense brute force written separately (oracle/brute_force.py).

The paper prints no worked numeric example of the MoE layer (its per-expert
latencies live only in figures), so nothing here is a paper-printed value
except the shapes in tests/golden/paper_shapes.txt.
"""
import numpy as np
import pytest
from scipy.special import softmax as sp_softmax

import moe_inputs as mi
from oracle import brute_force as bf
from oracle import moe_oracle as orc
from conftest import read_golden


def _rel(a, b):
    return np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300)


def _tiny(seed=7, T=5, d=8, f=12, E=4, k=2, w_dtype=mi.F32, zipf=None):
    cfg = mi.small_config("t", T, d, f, E, k, seed, w_dtype=w_dtype, zipf_s=zipf)
    return cfg, mi.make_layer(cfg, threads=1)


# ---------------------------------------------------------------- route ----

def test_route_all_equal_logits():
    for E, k in [(8, 2), (5, 3), (4, 4), (1, 1)]:
        idx, w = orc.route(np.full((3, E), 0.25, np.float32), k)
        assert (idx == np.arange(k)[None, :]).all()
        assert np.allclose(w, 1.0 / k, rtol=0, atol=1e-16)


def test_route_k_equals_E_is_full_softmax():
    rng = np.random.default_rng(1)
    lg = rng.standard_normal((6, 7)).astype(np.float32)
    idx, w = orc.route(lg, 7)
    ref = sp_softmax(lg.astype(np.float64), axis=1)
    for t in range(6):
        assert sorted(idx[t]) == list(range(7))
        assert np.allclose(w[t], ref[t, idx[t]], rtol=1e-14, atol=0)
        assert (np.diff(lg[t, idx[t]]) <= 0).all()  # descending logits


def test_route_k2_is_sigmoid():
    g = read_golden("closed_forms.txt")
    lg = np.array([[0.0, np.log(3.0), -5.0]], dtype=np.float32)
    idx, w = orc.route(lg, 2)
    assert idx.tolist() == [[1, 0]]
    diff = float(lg[0, 1]) - float(lg[0, 0])
    assert abs(w[0, 0] - 1.0 / (1.0 + np.exp(-diff))) < 1e-15
    assert abs(w[0, 0] - g["sigmoid_ln3"]) < 1e-7  # ln3 rounded to fp32
    rng = np.random.default_rng(2)
    lg = rng.standard_normal((50, 8)).astype(np.float32)
    idx, w = orc.route(lg, 2)
    l64 = lg.astype(np.float64)
    top = np.take_along_axis(l64, idx.astype(np.int64), axis=1)
    assert np.allclose(w[:, 0], 1.0 / (1.0 + np.exp(top[:, 1] - top[:, 0])), rtol=1e-14)


def test_route_k1_weight_is_one():
    rng = np.random.default_rng(3)
    lg = rng.standard_normal((9, 6)).astype(np.float32)
    idx, w = orc.route(lg, 1)
    assert (idx[:, 0] == lg.argmax(axis=1)).all()
    assert (w == 1.0).all()


def test_route_ties_go_to_lower_index():
    lg = np.array([
        [1.0, 3.0, 3.0, 3.0],      # three-way tie at the top
        [2.0, 2.0, 2.0, 5.0],      # tie for second place
        [-0.0, 0.0, -1.0, -1.0],   # -0.0 == +0.0
        [0.0, -0.0, -1.0, -1.0],
        [7.0, 1.0, 7.0, 1.0],
    ], dtype=np.float32)
    idx, w = orc.route(lg, 2)
    assert idx.tolist() == [[1, 2], [3, 0], [0, 1], [0, 1], [0, 2]]
    assert w[0, 0] == 0.5 and w[2, 0] == 0.5 and w[4, 1] == 0.5
    idx3, _ = orc.route(lg, 3)
    assert idx3.tolist() == [[1, 2, 3], [3, 0, 1], [0, 1, 2], [0, 1, 2], [0, 2, 1]]


def test_route_invariants_and_brute_force_gates():
    rng = np.random.default_rng(4)
    for E, k in [(8, 2), (16, 2), (64, 8), (3, 1), (8, 3)]:
        lg = rng.standard_normal((40, E)).astype(np.float32)
        lg[::5, : E // 2] = lg[::5, :1]  # plant exact ties
        idx, w = orc.route(lg, k)
        assert idx.min() >= 0 and idx.max() < E
        assert all(len(set(r)) == k for r in idx.tolist())
        assert np.allclose(w.sum(axis=1), 1.0, rtol=0, atol=2e-16 * k)
        assert (np.diff(w, axis=1) <= 0).all()
        dense = np.zeros((40, E))
        np.put_along_axis(dense, idx.astype(np.int64), w, axis=1)
        assert np.allclose(dense, bf.dense_gates(lg, k), rtol=1e-13, atol=1e-300)


def test_route_rejects_nonfinite_and_bad_k():
    lg = np.zeros((2, 4), np.float32)
    lg[1, 2] = np.nan
    with pytest.raises(ValueError):
        orc.route(lg, 2)
    lg[1, 2] = np.inf
    with pytest.raises(ValueError):
        orc.route(lg, 2)
    with pytest.raises(ValueError):
        orc.route(np.zeros((2, 4), np.float32), 5)


# -------------------------------------------------------------- permute ----

def test_permute_hand_example():
    # flat slots p=t*k+j: experts 2,0,0,1,2,1
    idx = np.array([[2, 0], [0, 1], [2, 1]], dtype=np.int32)
    x = np.arange(3 * 2, dtype=np.float64).reshape(3, 2) + 10.0
    counts, offsets, perm, inv, xg = orc.permute(idx, 3, x)
    assert counts.tolist() == [2, 2, 2]
    assert offsets.tolist() == [0, 2, 4, 6]
    assert perm.tolist() == [1, 2, 3, 5, 0, 4]
    assert inv.tolist() == [4, 0, 1, 2, 5, 3]
    assert (xg == x[[0, 1, 1, 2, 0, 2]]).all()


def test_permute_empty_experts_and_T0():
    idx = np.array([[3, 1]], dtype=np.int32)
    counts, offsets, perm, inv, xg = orc.permute(idx, 5, np.ones((1, 4)))
    assert counts.tolist() == [0, 1, 0, 1, 0]
    assert offsets.tolist() == [0, 0, 1, 1, 2, 2]
    assert perm.tolist() == [1, 0] and inv.tolist() == [1, 0]
    counts, offsets, perm, inv, xg = orc.permute(np.zeros((0, 2), np.int32), 4, np.zeros((0, 3)))
    assert counts.tolist() == [0, 0, 0, 0] and offsets.tolist() == [0] * 5 and perm.size == 0


def test_permute_invariants_random():
    rng = np.random.default_rng(5)
    for T, E, k in [(1, 8, 2), (16, 8, 2), (257, 8, 2), (100, 16, 4), (33, 3, 1)]:
        lg = rng.standard_normal((T, E)).astype(np.float32)
        idx, _ = orc.route(lg, k)
        x = rng.standard_normal((T, 6))
        counts, offsets, perm, inv, xg = orc.permute(idx, E, x)
        N = T * k
        assert counts.sum() == N and offsets[0] == 0 and offsets[E] == N
        assert (np.diff(offsets) == counts).all()
        assert (counts == np.bincount(idx.ravel(), minlength=E)).all()
        assert sorted(perm.tolist()) == list(range(N))            # bijection
        assert (inv[perm] == np.arange(N)).all() and (perm[inv] == np.arange(N)).all()
        flat = idx.ravel()
        assert (np.diff(flat[perm]) >= 0).all()                   # grouped by expert
        for e in range(E):
            seg = perm[offsets[e]:offsets[e + 1]]
            assert (flat[seg] == e).all() and (np.diff(seg) > 0).all()  # stable
        assert (perm == np.argsort(flat, kind="stable")).all()   # library stable sort
        assert (xg == x[perm // k]).all()


def test_permute_rejects_out_of_range_index():
    with pytest.raises(ValueError):
        orc.permute(np.array([[0, 4]], np.int32), 4, np.zeros((1, 2)))


# ----------------------------------------------------------- expert_ffn ----

def test_ffn_scalar_closed_form():
    g = read_golden("closed_forms.txt")
    one = np.ones((1, 1, 1), np.float32)
    yg = orc.expert_ffn(np.ones((1, 1)), np.array([0, 1], np.int32), one, one, one)
    assert abs(yg[0, 0] - g["scalar_silu_one"]) < 1e-15
    yg = orc.expert_ffn(-np.ones((1, 1)), np.array([0, 1], np.int32), one, -one, one)
    # a = -1, b = +1  ->  silu(-1) * 1
    assert abs(yg[0, 0] - g["silu_minus_one"]) < 1e-15


def test_ffn_matches_numpy_matmul_per_expert():
    rng = np.random.default_rng(6)
    E, d, f = 3, 10, 14  # d != f so a transposed operand cannot pass
    w1 = rng.standard_normal((E, d, f)).astype(np.float32)
    w3 = rng.standard_normal((E, d, f)).astype(np.float32)
    w2 = rng.standard_normal((E, f, d)).astype(np.float32)
    offsets = np.array([0, 4, 4, 9], np.int32)  # expert 1 empty
    xg = rng.standard_normal((9, d))
    yg = orc.expert_ffn(xg, offsets, w1, w3, w2)
    for e in range(E):
        s = slice(offsets[e], offsets[e + 1])
        ref = bf.dense_ffn(xg[s], w1[e].astype(np.float64), w3[e].astype(np.float64),
                           w2[e].astype(np.float64))
        assert ref.shape[0] == 0 or _rel(yg[s], ref) < 1e-13
    # w1 and w3 are not interchangeable: silu acts on the w1 branch only
    swapped = orc.expert_ffn(xg, offsets, w3, w1, w2)
    assert _rel(swapped, yg) > 1e-3


def test_ffn_bf16_weights_are_widened_exactly():
    rng = np.random.default_rng(7)
    E, d, f = 2, 8, 16
    w = [mi.f32_to_bf16_bits(rng.standard_normal(s).astype(np.float32))
         for s in [(E, d, f), (E, d, f), (E, f, d)]]
    xg = rng.standard_normal((5, d))
    offsets = np.array([0, 2, 5], np.int32)
    y_bits = orc.expert_ffn(xg, offsets, *w)
    y_f32 = orc.expert_ffn(xg, offsets, *[mi.bf16_bits_to_f32(a) for a in w])
    assert (y_bits == y_f32).all()


def test_ffn_zero_w1_gives_zero_and_w2_scaling_is_linear():
    rng = np.random.default_rng(8)
    E, d, f = 2, 6, 9
    w1 = rng.standard_normal((E, d, f)).astype(np.float32)
    w3 = rng.standard_normal((E, d, f)).astype(np.float32)
    w2 = rng.standard_normal((E, f, d)).astype(np.float32)
    xg = rng.standard_normal((4, d))
    offsets = np.array([0, 1, 4], np.int32)
    assert (orc.expert_ffn(xg, offsets, np.zeros_like(w1), w3, w2) == 0.0).all()
    y1 = orc.expert_ffn(xg, offsets, w1, w3, w2)
    y4 = orc.expert_ffn(xg, offsets, w1, w3, (w2 * np.float32(4.0)))
    assert np.allclose(y4, 4.0 * y1, rtol=1e-15, atol=0)


def test_ffn_skips_empty_experts_without_touching_output():
    one = np.ones((3, 2, 2), np.float32)
    yg = orc.expert_ffn(np.zeros((0, 2)), np.zeros(4, np.int32), one, one, one)
    assert yg.shape == (0, 2)


# -------------------------------------------------------------- combine ----

def test_combine_hand_example():
    yg = np.array([[1.0, 2.0], [10.0, 20.0], [100.0, 200.0], [1000.0, 2000.0]])
    inv = np.array([2, 0, 3, 1], np.int32)   # token0 -> rows 2,0 ; token1 -> rows 3,1
    w = np.array([[0.75, 0.25], [0.5, 0.5]])
    y = orc.combine(yg, inv, w)
    assert np.allclose(y, [[75.25, 150.5], [505.0, 1010.0]], rtol=1e-15)


# ---------------------------------------------------------------- layer ----

@pytest.mark.parametrize("shape", [(5, 8, 12, 4, 2), (7, 6, 10, 5, 3), (4, 8, 8, 3, 1),
                                   (6, 4, 6, 4, 4)])
def test_layer_matches_dense_brute_force(shape):
    T, d, f, E, k = shape
    cfg, li = _tiny(seed=11 + T, T=T, d=d, f=f, E=E, k=k)
    x = mi.to_f64(li.x)
    out = orc.layer(x, li.logits, li.w1, li.w3, li.w2, k)
    ref = bf.layer(x, li.logits, mi.to_f64(li.w1), mi.to_f64(li.w3), mi.to_f64(li.w2), k)
    assert _rel(out["y"], ref) < 1e-12


def test_layer_tiny_fp32_config_matches_brute_force_and_zipf_bf16():
    cfg = mi.CONFIGS["tiny_fp32"]
    li = mi.make_layer(cfg, threads=1)
    x = mi.to_f64(li.x)
    out = orc.layer(x, li.logits, li.w1, li.w3, li.w2, cfg.k)
    ref = bf.layer(x, li.logits, mi.to_f64(li.w1), mi.to_f64(li.w3), mi.to_f64(li.w2), cfg.k)
    assert _rel(out["y"], ref) < 1e-12
    cfg, li = _tiny(seed=21, T=16, d=16, f=24, E=8, k=2, w_dtype=mi.BF16, zipf=1.2)
    x = mi.to_f64(li.x)
    out = orc.layer(x, li.logits, li.w1, li.w3, li.w2, 2)
    ref = bf.layer(x, li.logits, mi.to_f64(li.w1), mi.to_f64(li.w3), mi.to_f64(li.w2), 2)
    assert _rel(out["y"], ref) < 1e-12


def test_identical_experts_reduce_to_one_dense_ffn():
    cfg, li = _tiny(seed=31, T=9, d=8, f=12, E=4, k=2)
    w1 = np.repeat(li.w1[:1], 4, axis=0)
    w3 = np.repeat(li.w3[:1], 4, axis=0)
    w2 = np.repeat(li.w2[:1], 4, axis=0)
    x = mi.to_f64(li.x)
    out = orc.layer(x, li.logits, w1, w3, w2, 2)
    ref = bf.dense_ffn(x, w1[0].astype(np.float64), w3[0].astype(np.float64),
                       w2[0].astype(np.float64))
    assert _rel(out["y"], ref) < 1e-13


def test_permuting_tokens_permutes_outputs():
    cfg, li = _tiny(seed=41, T=8, d=8, f=12, E=4, k=2)
    x = mi.to_f64(li.x)
    p = np.random.default_rng(0).permutation(8)
    y = orc.layer(x, li.logits, li.w1, li.w3, li.w2, 2)["y"]
    yp = orc.layer(x[p], li.logits[p], li.w1, li.w3, li.w2, 2)["y"]
    assert np.allclose(yp, y[p], rtol=1e-14, atol=1e-300)


# ------------------------------------------------- stack support steps ----

def test_rmsnorm_closed_form_and_router_logits():
    x = np.full((2, 16), 3.0)
    h = orc.rmsnorm(x, 1e-5)
    assert np.allclose(h, 3.0 / np.sqrt(9.0 + 1e-5), rtol=1e-15)
    rng = np.random.default_rng(9)
    x = rng.standard_normal((4, 32))
    h = orc.rmsnorm(x, 1e-5)
    assert np.allclose(h, x / np.sqrt((x * x).mean(axis=1, keepdims=True) + 1e-5), rtol=1e-14)
    wg = rng.standard_normal((32, 8)).astype(np.float32)
    lg = orc.router_logits(h, wg)
    assert lg.dtype == np.float32
    assert np.allclose(lg, (h @ wg.astype(np.float64)).astype(np.float32), rtol=1e-6)


# ------------------------------------------------ paper-stated shapes ----

def test_paper_shapes_and_sizes():
    g = read_golden("paper_shapes.txt")
    cfg = mi.CONFIGS["decode_t1"]
    assert (cfg.d, cfg.f, cfg.E) == (g["d_model"], g["d_ff"], g["experts_per_layer"])
    expert_bytes = g["matrices_per_expert"] * cfg.d * cfg.f * g["bytes_per_weight"]
    assert expert_bytes == 352321536 and expert_bytes > g["expert_bytes_lower_bound"]
    assert g["layers"] * g["experts_per_layer"] == g["experts_total"]
    assert expert_bytes * g["experts_total"] > g["model_bytes_lower_bound"]


# ------------------------------------------------------ input recipe ----

def test_bf16_rounding_is_nearest_even():
    f = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -9, -1.0 - 2 ** -8,
                  1.0 + 2 ** -8 + 2 ** -20], dtype=np.float32)
    b = mi.bf16_bits_to_f32(mi.f32_to_bf16_bits(f))
    # halfway cases go to the even mantissa; anything above halfway rounds up
    assert b.tolist() == [1.0, 1.0, 1.0 + 2 ** -6, 1.0, -1.0, 1.0 + 2 ** -7]


def test_zipf_pmf_and_seed_determinism():
    p = np.exp(mi.zipf_log_pmf(8, 1.2))
    assert abs(p.sum() - 1.0) < 1e-15 and (np.diff(p) < 0).all()
    assert np.allclose(p[:3], [0.4286, 0.1866, 0.1147], atol=5e-4)
    a = mi.make_layer(mi.CONFIGS["tiny_fp32"], threads=1)
    b = mi.make_layer(mi.CONFIGS["tiny_fp32"], threads=4)
    assert (a.w2 == b.w2).all() and (a.x == b.x).all() and (a.logits == b.logits).all()


def test_stack_is_norm_route_layer_residual():
    rng = np.random.default_rng(12)
    T, d, f, E, k = 5, 8, 12, 4, 2
    layers = []
    for l in range(3):
        cfg, li = _tiny(seed=50 + l, T=T, d=d, f=f, E=E, k=k)
        layers.append((li.w_gate, li.w1, li.w3, li.w2))
    x0 = rng.standard_normal((T, d))
    out = orc.stack(x0, layers, k)
    # written out by hand with numpy + the dense brute force
    x = x0.copy()
    for w_gate, w1, w3, w2 in layers:
        h = x / np.sqrt((x * x).mean(axis=1, keepdims=True) + 1e-5)
        lg = (h @ w_gate.astype(np.float64)).astype(np.float32)
        x = x + bf.layer(h, lg, mi.to_f64(w1), mi.to_f64(w3), mi.to_f64(w2), k)
    assert _rel(out["x"], x) < 1e-12
    # forcing the oracle's own logits changes nothing
    forced = orc.stack(x0, layers, k, forced_logits=out["logits"])
    assert (forced["x"] == out["x"]).all()


# ------------------------------------------------- sanitizer run of the oracle ----

def test_oracle_is_clean_under_address_and_undefined_sanitizers():
    """The oracle's C source, driven over small layers with the edge cases (an empty expert,
    k == E, no tokens, both weight dtypes), built with -fsanitize=address,undefined: the run
    must finish without a report and print what the plain build of the same program prints."""
    import subprocess
    from oracle import build
    san = subprocess.run([build.build_sanitize_check(True)], capture_output=True, text=True, timeout=120)
    plain = subprocess.run([build.build_sanitize_check(False)], capture_output=True, text=True, timeout=120)
    assert san.returncode == 0 and plain.returncode == 0, san.stderr[-2000:]
    assert "ERROR" not in san.stderr and "runtime error" not in san.stderr, san.stderr[-2000:]
    assert san.stdout == plain.stdout and san.stdout.count("rc=0") == 4
