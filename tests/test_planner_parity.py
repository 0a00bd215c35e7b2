"""The library's planner (C ABI of include/asteroid_planner.h, host code) against the planner
oracle on the same seeded profiler tables: allocations, step times, latencies, dominant steps
and whole plans, exactly (the tables hold whole numbers, so no sum depends on its order)."""
import itertools
import math

import numpy as np
import pytest

from asteroid_workloads.planner_gen import planner_problem
from oracle import planner as O

KINDS = ["linear", "affine", "stair"]
MEMS = ["loose", "tight"]


@pytest.fixture(scope="module")
def PL():
    from paper_2408_08015_amd import planner
    planner._lib()
    return planner


def both(PL, seed, L, N, B, M, **kw):
    d = planner_problem(seed, L, N, B, M, **kw)
    o = O.Problem(d["tf"].tolist(), d["tb"].tolist(), d["a"].tolist(), d["act"].tolist(), d["w"].tolist(),
                  d["u"].tolist(), d["bw"].tolist(), B, M, block=d["block"])
    h = PL.Problem(d["tf"], d["tb"], d["a"], d["act"], d["w"], d["u"], d["bw"], B, M, block=d["block"])
    return o, h


@pytest.mark.parametrize("seed", range(4))
def test_stage_memory(PL, seed):
    o, h = both(PL, seed, 9, 3, 16, 4)
    for lo, hi in [(0, 9), (2, 5), (8, 9)]:
        for K in (1, 3, 5):
            for beta in (0, 1, 7, 16):
                assert PL.stage_memory(h, lo, hi, K, beta) == O.stage_memory(o, lo, hi, K, beta)


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("memory", MEMS)
@pytest.mark.parametrize("seed", range(8))
def test_allocate(PL, seed, kind, memory):
    L, N, B = 12, 6, 32
    o, h = both(PL, 40 + seed, L, N, B, 8, kind=kind, memory=memory, block=1 + seed % 4)
    rng = np.random.default_rng(seed)
    for _ in range(40):
        lo = int(rng.integers(0, L))
        hi = int(rng.integers(lo + 1, L + 1))
        g = int(rng.integers(1, N + 1))
        G = [int(x) for x in rng.permutation(N)[:g]]
        K = int(rng.choice([1, 3, 5, 11]))
        want = O.allocate(o, lo, hi, G, K)
        got = PL.allocate(h, lo, hi, G, K)
        if want is None:
            assert got is None
            continue
        y, Ef, Eb = got
        assert y == want
        assert (Ef, Eb) == O.step_times(o, lo, hi, G, want)


@pytest.mark.parametrize("seed", range(30))
def test_round_latency(PL, seed):
    rng = np.random.default_rng(seed)
    S = int(rng.choice([1, 3, 5, 7, 9, 11]))
    M = int(rng.choice([1, 4, 16, 64]))
    Ef = rng.integers(1, 1000, size=S).astype(np.float64)
    Eb = rng.integers(1, 2000, size=S).astype(np.float64)
    Ta = np.where(np.arange(S) % 2 == 0, rng.integers(0, 5000, size=S), 0).astype(np.float64)
    assert PL.round_latency(Ef, Eb, Ta, M) == O.round_latency(Ef.tolist(), Eb.tolist(), Ta.tolist(), M)


CASES = [(s, k, m) for s, (k, m) in enumerate(itertools.product(KINDS, MEMS))]
CASES += [(10 + s, "affine", "tight") for s in range(4)] + [(20 + s, "stair", "loose") for s in range(3)]


@pytest.mark.parametrize("seed,kind,memory", CASES)
def test_plan_hpp(PL, seed, kind, memory):
    shapes = [(6, 3, 6, 4), (7, 4, 8, 8), (9, 3, 5, 6), (5, 5, 4, 4)]
    L, N, B, M = shapes[seed % len(shapes)]
    o, h = both(PL, 300 + seed, L, N, B, M, kind=kind, memory=memory, block=1 + seed % 2)
    lat_o, stages_o, ys_o = O.plan_hpp(o)
    lat_h, stages_h, y_h = PL.plan_hpp(h)
    if stages_o is None:
        assert stages_h is None and math.isinf(lat_h)
        return
    assert lat_h == lat_o
    assert stages_h == stages_o
    merged = {}
    for y in ys_o:
        merged.update(y)
    assert y_h == merged


@pytest.mark.parametrize("L,N,B,M", [(1, 1, 1, 1), (1, 4, 8, 2), (6, 1, 4, 4), (3, 3, 1, 8), (2, 5, 3, 1), (8, 2, 16, 64)])
def test_plan_hpp_degenerate_sizes(PL, L, N, B, M):
    """One layer, one device, one sample, one micro-batch, more devices than layers or samples."""
    for seed, memory in ((0, "loose"), (1, "tight")):
        o, h = both(PL, 700 + seed, L, N, B, M, kind="stair", memory=memory)
        lat_o, stages_o, ys_o = O.plan_hpp(o)
        lat_h, stages_h, y_h = PL.plan_hpp(h)
        if stages_o is None:
            assert stages_h is None and math.isinf(lat_h)
            continue
        assert (lat_h, stages_h) == (lat_o, stages_o)
        assert len(stages_h) <= min(L, N) and sum(y_h.values()) == B * len(stages_h)
        for G in ([0], list(range(N))):
            want = O.allocate(o, 0, L, G, 1)
            got = PL.allocate(h, 0, L, G, 1)
            assert (got is None) == (want is None)
            if want is not None:
                assert got[0] == want


def test_plan_hpp_real_valued_tables_agree_to_rounding(PL):
    """Measured tables are not whole numbers: sums taken in a different order then differ in
    the last bits, so the latency agrees to rounding (and the plan unless two candidates tie)."""
    for seed in range(4):
        d = planner_problem(500 + seed, 7, 3, 6, 8, kind="affine")
        rng = np.random.default_rng(seed)
        d["tf"] = d["tf"] * rng.uniform(0.9, 1.1, size=d["tf"].shape)
        d["tb"] = d["tb"] * rng.uniform(0.9, 1.1, size=d["tb"].shape)
        o = O.Problem(d["tf"].tolist(), d["tb"].tolist(), d["a"].tolist(), d["act"].tolist(), d["w"].tolist(),
                      d["u"].tolist(), d["bw"].tolist(), 6, 8)
        h = PL.Problem(d["tf"], d["tb"], d["a"], d["act"], d["w"], d["u"], d["bw"], 6, 8)
        lat_o, stages_o, _ = O.plan_hpp(o)
        lat_h, stages_h, _ = PL.plan_hpp(h)
        assert abs(lat_h - lat_o) <= 1e-12 * lat_o
        assert stages_h == stages_o


def test_bad_arguments_are_reported(PL):
    from paper_2408_08015_amd import AsteroidError
    _, h = both(PL, 1, 4, 2, 4, 4)
    with pytest.raises(AsteroidError):
        PL.stage_memory(h, 2, 2, 1, 1)
    with pytest.raises(AsteroidError):
        PL.stage_memory(h, 0, 4, 0, 1)
    with pytest.raises(AsteroidError):
        PL.allocate(h, 0, 4, [0, 0], 1)
    with pytest.raises(AsteroidError):
        PL.allocate(h, 0, 5, [0], 1)
    with pytest.raises(AsteroidError):
        PL.round_latency([1.0, 2.0], [1.0, 2.0], [0.0, 0.0], 4)


def test_planning_time_at_the_papers_problem_size(PL):
    """Table 7's setting: six devices, a model of some 150 layers, micro-batches up to 32: the
    whole dynamic programme takes seconds, not minutes."""
    import time
    d = planner_problem(77, 150, 6, 32, 16, kind="affine", memory="tight", block=4)
    h = PL.Problem(d["tf"], d["tb"], d["a"], d["act"], d["w"], d["u"], d["bw"], 32, 16, block=4)
    t0 = time.time()
    lat, stages, y = PL.plan_hpp(h)
    dt = time.time() - t0
    assert stages is not None and sum(y.values()) == 32 * len(stages)
    assert dt < 60.0


def test_fixed_bytes_per_layer_enter_the_memory_check(PL):
    """The optional fixed term (workspace, derived weight copies: outside Eq. (3)) adds its layer sum to the
    stage footprint, NULL leaves the paper's formula, and Alg. 1 sees it: a micro-batch that fits without it
    is cut down, and refused when the fixed bytes alone exceed the budget."""
    L, N, B = 3, 1, 8
    t = np.zeros((N, L, B + 1))
    t[:, :, 1:] = np.arange(1, B + 1)[None, None, :]
    act, w = [10.0, 20.0, 30.0], [100.0, 200.0, 400.0]
    plain = PL.Problem(t, t, [1.0] * L, act, w, [3000.0], [[1.0]], B, 4)
    fixed = PL.Problem(t, t, [1.0] * L, act, w, [3000.0], [[1.0]], B, 4, fixed=[5.0, 50.0, 500.0])
    assert PL.stage_memory(plain, 1, 3, 3, 4) == 1200 + 600 + 3 * 200
    assert PL.stage_memory(fixed, 1, 3, 3, 4) == 1200 + 600 + 3 * 200 + 550
    assert PL.stage_memory(fixed, 0, 1, 1, 0) == 300 + 5
    # whole model on the one device, K = 1: 2100 + 60 beta (+ 555) <= 3000
    assert PL.allocate(plain, 0, 3, [0], 1)[0] == {0: 8}
    tight = PL.Problem(t, t, [1.0] * L, act, w, [2100.0 + 60 * 8 + 100], [[1.0]], B, 4, fixed=[5.0, 50.0, 500.0])
    assert PL.allocate(tight, 0, 3, [0], 1) is None                    # 2655 + 60 beta > 2680 for beta = 8: cannot hold B
    none = PL.Problem(t, t, [1.0] * L, act, w, [2500.0], [[1.0]], B, 4, fixed=[5.0, 50.0, 500.0])
    assert PL.allocate(none, 0, 3, [0], 1) is None                     # 2655 > 2500 even for an empty micro-batch
    with pytest.raises(ValueError):
        PL.Problem(t, t, [1.0] * L, act, w, [1.0], [[1.0]], B, 4, fixed=[1.0])
