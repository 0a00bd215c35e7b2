"""CPU-only checks: the C-ABI library loads and exports every declared symbol, host-side
planning (shape inference, Eq. (3) byte counts, argument errors), the warm-up depth
formula, and the seeded generators."""
import ctypes
import os
import re

import numpy as np
import pytest

from asteroid_workloads import configs as C
from asteroid_workloads import gen, get_config

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def A():
    import paper_2408_08015_amd as A
    A.load_library()
    return A


def test_library_exports_every_declared_symbol(A):
    import glob
    hdr = "".join(open(h).read() for h in sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))))
    names = sorted(set(re.findall(r"\b(asteroid_[a-z_0-9]+)\s*\(", hdr)))
    assert "asteroid_stage_create" in names and "asteroid_stage_step" in names and len(names) >= 19
    assert "asteroid_plan_hpp" in names and "asteroid_plan_allocate" in names
    lib = ctypes.CDLL(A.lib_path())
    for n in names:
        assert hasattr(lib, n), n


def test_kp_matches_the_papers_example(A):
    # Sec. 3.2: K_p = 2(P - p) - 1; the paper's 3-stage pipeline has K_0 = 5, K_1 = 3, K_2 = 1
    assert [A.kp(3, p) for p in range(3)] == [5, 3, 1]
    assert A.kp(1, 0) == 1
    assert A.kp(3, 3) == -1 and A.kp(0, 0) == -1 and A.kp(2, -1) == -1


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
def test_plan_memory_follows_eq3(A, name):
    """Eq. (3): Mem = MOD + OPT + K * ACT.  MOD = fp32 params + fp32 accumulated gradients
    (+ derived weight copies), OPT = fp32 velocity, ACT independent of K and M."""
    cfg = get_config(name)
    n = gen.num_params(cfg.layers)
    args = (cfg.layers, cfg.B, cfg.M)
    m1 = A.plan_memory(*args, 1, cfg.in_shape, cfg.dtype, cfg.layout, cfg.needs_input_grad)
    m3 = A.plan_memory(*args, cfg.M, cfg.in_shape, cfg.dtype, cfg.layout, cfg.needs_input_grad)
    assert m1 == m3                               # per-micro-batch stash does not depend on K
    mod, opt, act, ws = m1
    assert opt == 4 * n
    if cfg.dtype == "f32":
        # two packed layouts of each pointwise-conv matrix, padded to 32 x 8 tiles
        assert 8 * n <= mod <= 8 * n + 2 * 4 * 2 * n + 65536
    else:
        assert mod > 8 * n and mod <= 8 * n + 2 * 2 * n + 64   # two bf16 layouts of each matrix
    # the stash holds at least the stage input and every conv / linear input
    x_bytes = int(np.prod(cfg.in_shape)) * cfg.B * (2 if cfg.dtype == "bf16" else 4)
    assert act >= x_bytes
    # a bigger micro-batch needs a proportionally bigger stash (activations dominate)
    big = A.plan_memory(cfg.layers, 2 * cfg.B, cfg.M, 1, cfg.in_shape, cfg.dtype, cfg.layout, cfg.needs_input_grad)
    assert 1.8 * act < big[2] < 2.2 * act


def test_plan_errors(A):
    ok = C.cfg1()
    with pytest.raises(A.AsteroidError) as e:
        A.plan_memory(ok.layers, 4, 2, 3, ok.in_shape)           # K > M
    assert e.value.status == -1
    with pytest.raises(A.AsteroidError) as e:
        A.plan_memory(ok.layers, 4, 2, 1, (16, 8, 8))            # channel mismatch
    assert e.value.status == -1
    with pytest.raises(A.AsteroidError) as e:
        A.plan_memory([dict(kind="res_add")], 4, 2, 1, (16, 8, 8))
    assert e.value.status == -1
    with pytest.raises(A.AsteroidError) as e:
        A.plan_memory([dict(kind="res_begin"), dict(kind="relu")], 4, 2, 1, (16, 8, 8))
    assert e.value.status == -1
    with pytest.raises(A.AsteroidError) as e:                     # loss tail must be last
        A.plan_memory([dict(kind="global_avgpool"), dict(kind="softmax_ce"), dict(kind="relu")], 4, 2, 1, (16, 8, 8))
    assert e.value.status == -1
    with pytest.raises(A.AsteroidError) as e:                     # fp32 stages are NCHW
        A.plan_memory(ok.layers, 4, 2, 1, ok.in_shape, "f32", "nhwc")
    assert e.value.status == -5
    with pytest.raises(A.AsteroidError) as e:                     # bf16 BatchNorm is not covered
        A.plan_memory(ok.layers, 4, 2, 1, ok.in_shape, "bf16", "nhwc")
    assert e.value.status == -5
    with pytest.raises(A.AsteroidError) as e:                     # 32-bit pixel indices: B*H*W < 2^31
        A.plan_memory([dict(kind="conv2d", cin=8, cout=8, k=1, stride=1, pad=0, groups=1, bias=False)], 32, 1, 1, (8, 8192, 8192))
    assert e.value.status == -5 and "2^31" in str(e.value)
    with pytest.raises(A.AsteroidError):
        A.plan_memory(ok.layers, 0, 2, 1, ok.in_shape)


def test_generators_are_seeded_and_ordered():
    cfg = C.cfg1()
    a, b = gen.make_inputs(cfg), gen.make_inputs(cfg)
    for k in a:
        assert np.array_equal(a[k], b[k])
    rng = np.random.Generator(np.random.PCG64(cfg.seed))
    x = rng.standard_normal((8, 32, 16, 16)).astype(np.float32)
    assert np.array_equal(a["x"], x)                       # x is drawn first
    lab = rng.integers(0, 10, size=8).astype(np.int32)
    assert np.array_equal(a["labels"], lab)                # then the labels
    assert a["params"].size == 30026
    assert [gen.num_params(get_config(n).layers) for n in ("cfg2", "cfg3", "cfg4", "cfg5")] == \
        [39696, 3504872, 1475328, 18914304]


def test_bf16_rounding_helper():
    v = np.array([1.0, 1.00390625, 1.01171875, -3.14159, 65504.0, 1e-40], np.float32)
    r = gen.round_to_bf16(v)
    assert np.all((r.view(np.uint32) & 0xFFFF) == 0)
    assert r[0] == 1.0
    assert r[1] == 1.0            # 1 + 2^-8 is a tie: rounds to even (1.0)
    assert r[2] == np.float32(1.015625)   # 1 + 3*2^-8 ties to the even neighbour 1 + 2^-6
    assert abs(r[3] + 3.140625) < 1e-6
    c4 = get_config("cfg4", B=1, M=1, hw=4, cin=8, c=8)
    inp = gen.make_inputs(c4)
    assert np.array_equal(gen.round_to_bf16(inp["x"]), inp["x"]) and inp["x"].shape == (1, 4, 4, 8)


def test_profiler_units_cut_only_where_a_stage_may_end():
    """Sec. 3.3: the model is a layer sequence split between layers; the profiler's units are
    the shortest runs a stage can consist of (never inside a residual block, a BatchNorm or
    activation stays with its convolution, the loss with the classifier)."""
    from paper_2408_08015_amd.profiler import split_units
    L = C.mobilenetv2_layers(10)
    units = split_units(L)
    assert units[0] == (0, 3) and units[-1] == (len(L) - 3, len(L))
    assert [u[0] for u in units[1:]] == [u[1] for u in units[:-1]]
    for lo, hi in units:
        kinds = [l["kind"] for l in L[lo:hi]]
        assert kinds.count("res_begin") == kinds.count("res_add")
        assert kinds[0] in ("conv2d", "res_begin", "global_avgpool")
    enc = C.encoder_layer(64, 2, 128) * 2
    assert split_units(enc) == [(0, 4), (4, 10), (10, 14), (14, 20)]
    assert split_units(C.vgg_layers(8, 16)) == [(0, 2), (2, 4), (4, 7)]
    mb = C.mbconv(24, 40, 5, 2, 6)       # expand, depthwise, squeeze-and-excitation, project
    assert split_units(mb) == [(0, 3), (3, 6), (6, 13), (13, 15)]
    assert len(split_units(C.mbconv(40, 40, 5, 1, 6))) == 1


def test_profiler_table_interpolation():
    from paper_2408_08015_amd.profiler import tables_for_planner
    units = [dict(tf={1: 10.0, 4: 16.0}, tb={1: 20.0, 4: 32.0}, a=8, act=24.0, w=100)]
    tf, tb, a, act, w, fixed = tables_for_planner(units, 6, n_devices=3)
    assert tf.shape == (3, 1, 7)
    assert list(tf[2, 0]) == [0.0, 10.0, 12.0, 14.0, 16.0, 18.0, 20.0]      # last slope continues
    assert list(tb[0, 0]) == [0.0, 20.0, 24.0, 28.0, 32.0, 36.0, 40.0]
    assert (a[0], act[0], w[0], fixed[0]) == (8.0, 24.0, 100.0, 0.0)


@pytest.mark.parametrize("name", ["cfg3", "cfg4", "cfg5"])
def test_profiler_memory_terms_cover_what_the_library_allocates(A, name):
    """Eq. (3) has no term for the workspace or the derived weight copies.  What the profiler hands the
    planner for a unit (w_l, act_l, fixed_l), put through the planner's memory check, must never fall below
    the bytes asteroid_stage_plan_memory reports for a stage made of that unit - for K = 1 and K = 3, at the
    power-of-two micro-batch sizes up to the profiled one - nor, summed over its units, for a stage of
    several units, which at the profiled size with K = 1 it over-states by less than 30 %."""
    from asteroid_workloads.gen import out_shape
    from paper_2408_08015_amd import planner as PL
    from paper_2408_08015_amd.profiler import split_units, unit_memory
    cfg = get_config(name)
    units = split_units(cfg.layers)[:6]
    shape, bmax = list(cfg.in_shape), cfg.B
    first_shape, rows = list(shape), []
    for lo, hi in units:
        sub = cfg.layers[lo:hi]
        out = list(out_shape(sub, shape))
        a_l = int(np.prod(out)) * (2 if cfg.dtype == "bf16" else 4)
        rows.append(unit_memory(sub, bmax, shape, cfg.dtype, cfg.layout, cfg.needs_input_grad or lo > 0, a_l))
        shape = out
    L = len(units)
    act, w, fixed = (np.array(c, dtype=np.float64) for c in zip(*rows))
    z = np.zeros((1, L, bmax + 1))
    pr = PL.Problem(z, z, [1.0] * L, act, w, [1e18], [[1.0]], bmax, 4, fixed=fixed)
    betas = sorted({bmax} | {b for b in (1, 2, 4, 8, 16) if b < bmax})
    shape = list(first_shape)
    for u, (lo, hi) in enumerate(units):
        sub = cfg.layers[lo:hi]
        for K in (1, 3):
            for beta in betas:
                mod, opt, a_, ws = A.plan_memory(sub, beta, max(K, 4), K, shape, cfg.dtype, cfg.layout,
                                                 cfg.needs_input_grad or lo > 0)
                model = PL.stage_memory(pr, u, u + 1, K, beta)
                assert mod + opt + K * a_ + ws <= model + 1e-6, (u, K, beta)
        shape = list(out_shape(sub, shape))
    sub = cfg.layers[units[0][0]:units[-1][1]]
    for K in (1, 3):
        mod, opt, a_, ws = A.plan_memory(sub, bmax, max(K, 4), K, first_shape, cfg.dtype, cfg.layout,
                                         cfg.needs_input_grad)
        model = PL.stage_memory(pr, 0, L, K, bmax)
        assert mod + opt + K * a_ + ws <= model + 1e-6, K
        if K == 1:
            assert model <= 1.3 * (mod + opt + a_ + ws), (model, mod + opt + a_ + ws)
