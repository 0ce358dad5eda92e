"""Host-only tests of the paper's own method (placement by popularity, latency model,
Algorithm 1) and of the host-side expert kernel.

The plain restatement in oracle/orch_oracle.py is pinned first -- against the values the
paper prints (tests/golden/placement_hit_rates.txt), closed forms and brute force over all
placements -- and then the library's moe_orch_* functions are compared with it.  The
host-side expert (case (c) of Sec. 3.2) is compared with the fp64 oracle."""
import itertools

import numpy as np
import pytest

import moe_inputs as mi
from oracle import moe_oracle as orc
from oracle import orch_oracle as oo


@pytest.fixture(scope="module")
def moe():
    import os
    import paper_2402_07033_amd as m
    if not os.path.exists(m.lib_path()):
        from paper_2402_07033_amd import build
        build.build()
    m.lib()
    return m


# ------------------------------------------------------------ pins of the oracle ----

def test_uniform_popularity_gives_the_papers_random_hit_rates(golden):
    g = golden("placement_hit_rates.txt")
    pop = np.ones((32, 8))
    for cap, key in ((56, "random_hit_rate_56_of_256"), (125, "random_hit_rate_125_of_256")):
        at = oo.place(pop, cap)
        assert at.sum() == cap
        assert abs(oo.hit_rate(pop, at) - cap / 256) < 1e-15
        assert abs(oo.hit_rate(pop, at) - g[key]) <= 5e-4       # the paper rounds to 0.1 %
        # equal popularity: the lower flat indices are taken
        assert at.reshape(-1)[:cap].all() and not at.reshape(-1)[cap:].any()


def test_placement_maximises_hit_rate_brute_force():
    rng = np.random.default_rng(5)
    for trial in range(6):
        L, E, cap = 2, 4, int(rng.integers(1, 7))
        pop = rng.integers(0, 6, size=(L, E)).astype(np.float64)   # ties on purpose
        at = oo.place(pop, cap)
        assert at.sum() == cap
        best = worst = None
        for sub in itertools.combinations(range(L * E), cap):
            m = np.zeros(L * E, np.uint8)
            m[list(sub)] = 1
            h = oo.hit_rate(pop, m.reshape(L, E))
            best = h if best is None else max(best, h)
            worst = h if worst is None else min(worst, h)
        got = oo.hit_rate(pop, at)
        assert abs(got - best) < 1e-15 and got >= worst
        # best >= random (= capacity / all) whenever the profile is not all zero
        if pop.sum() > 0:
            assert got >= cap / (L * E) - 1e-15
    assert oo.hit_rate(np.zeros((2, 2)), np.ones((2, 2))) == 0.0
    assert oo.place(np.array([[3.0, 1.0]]), 5).tolist() == [[1, 1]]       # capacity beyond all


def test_algorithm1_hand_cases():
    lat = dict(gpu_lat_us=100.0, cpu_lat_us_per_row=50.0, transfer_lat_us=900.0)
    # cpu_lat(s) = 50 s; gpu_lat + trans_lat = 1000: the host wins up to s = 20 (50*20 = 1000
    # is not greater), the device after a transfer from s = 21
    at = np.array([1, 0, 0, 0, 1, 0], np.uint8)
    size = np.array([7, 0, 20, 21, 0, 1], np.int32)
    assert oo.decide(at, size, lat).tolist() == [oo.GPU_RESIDENT, oo.SKIP, oo.CPU, oo.GPU_TRANSFER,
                                                 oo.SKIP, oo.CPU]
    # the decision for a non-resident expert switches exactly once as the input grows
    d = [int(oo.decide([0], [s], lat)[0]) for s in range(1, 60)]
    assert d == [oo.CPU] * 20 + [oo.GPU_TRANSFER] * 39
    # a free transfer and a free device: everything non-resident goes to the device
    free = dict(gpu_lat_us=0.0, cpu_lat_us_per_row=1.0, transfer_lat_us=0.0)
    assert oo.decide([0, 0], [1, 9], free).tolist() == [oo.GPU_TRANSFER] * 2
    # a resident expert never leaves the device, whatever the constants
    slow = dict(gpu_lat_us=1e9, cpu_lat_us_per_row=1e-9, transfer_lat_us=1e9)
    assert oo.decide([1], [1000], slow).tolist() == [oo.GPU_RESIDENT]


# ----------------------------------------------------- the library vs the oracle ----

def test_library_policy_matches_the_oracle(moe):
    rng = np.random.default_rng(17)
    for trial in range(20):
        L, E = int(rng.integers(1, 6)), int(rng.integers(1, 9))
        pop = rng.integers(0, 5, size=(L, E)).astype(np.float64)
        cap = int(rng.integers(0, L * E + 3))
        at = moe.moe_orch_place(pop, cap)
        assert (at == oo.place(pop, cap)).all()
        assert abs(moe.moe_orch_hit_rate(pop, at) - oo.hit_rate(pop, at)) < 1e-15
        lat = dict(gpu_lat_us=float(rng.random() * 300), cpu_lat_us_per_row=float(rng.random() * 90),
                   transfer_lat_us=float(rng.random() * 5000))
        size = rng.integers(0, 70, size=E).astype(np.int32)
        size[rng.random(E) < 0.3] = 0
        assert (moe.moe_orch_decide(at[0], size, lat) == oo.decide(at[0], size, lat)).all()
    pop = np.ones((32, 8))
    assert abs(moe.moe_orch_hit_rate(pop, moe.moe_orch_place(pop, 56)) - 56 / 256) < 1e-15
    with pytest.raises(moe.MoeError):
        moe.moe_orch_place(np.array([[1.0, -2.0]]), 1)            # negative popularity
    with pytest.raises(moe.MoeError):
        moe.moe_orch_place(np.array([[1.0, np.nan]]), 1)


@pytest.mark.parametrize("s,d,f", [(1, 64, 128), (5, 256, 512), (3, 128, 448), (17, 64, 64)])
def test_host_side_expert_matches_the_oracle(moe, s, d, f):
    cfg = mi.small_config("cpu", s, d, f, 1, 1, 3100 + s + d, w_dtype=mi.BF16)
    li = mi.make_layer(cfg, threads=1)
    y = moe.moe_orch_cpu_expert_ffn(li.x, li.w1[0], li.w3[0], li.w2[0])
    ref = orc.expert_ffn(li.x.astype(np.float64), np.array([0, s], np.int32), li.w1, li.w3, li.w2)
    err = np.max(np.abs(y - ref)) / np.max(np.abs(ref))
    assert err <= 1e-5, err
    assert moe.moe_orch_cpu_expert_ffn(li.x[:0], li.w1[0], li.w3[0], li.w2[0]).shape == (0, d)
