"""Forward passes on a second stream (asteroid_stage_set_forward_stream): with K >= 2 stashes the
forward of a later micro-batch runs beside the backward of an earlier one.  The arithmetic and its
order are those of the one-stream execution, so every result is compared bit for bit with it; the
one-stream execution is the one the other GPU tests score against the oracle."""
import numpy as np
import pytest

import harness
from asteroid_workloads import configs as C
from asteroid_workloads import gen

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def A():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2408_08015_amd as A
    return A


CASES = {
    "cfg1": lambda: C.cfg1(),
    "cfg2": lambda: C.cfg2(B=3, M=4, hw=18),
    "cfg3": lambda: C.cfg3(B=4, M=3, hw=64, num_classes=10),
    "cfg6": lambda: C.cfg6(B=2, M=3, hw=12),
    "cfg7": lambda: C.cfg7(B=2, M=3, hw=8),
    "cfg4": lambda: C.cfg4(B=2, M=4, hw=12, cin=64, c=64),
    "cfg5": lambda: C.cfg5(B=2, M=4, S=64, d=128, heads=2, ffn=256, nlayers=2),
}


@pytest.mark.parametrize("name", sorted(CASES))
@pytest.mark.parametrize("K", [2, 3])
def test_forward_stream_is_bit_identical(A, name, K):
    cfg = CASES[name]()
    K = min(K, cfg.M)
    inp = gen.make_inputs(cfg, randomize_affine=True)
    one, _, mem1 = harness.run_hip(cfg, inp, K=K, rounds=3)
    two, _, mem2 = harness.run_hip(cfg, inp, K=K, rounds=3, forward_stream=True)
    assert mem1 == mem2
    for r, (a, b) in enumerate(zip(one, two)):
        for k in ("y", "dx", "G", "W"):
            if a[k] is None:
                continue
            assert r > 0 or np.isfinite(a[k]).all(), (name, K, k)
            assert np.array_equal(a[k], b[k], equal_nan=True), (name, K, r, k)
        if cfg.loss_tail:
            assert a["loss"] == b["loss"], (name, K, r)


@pytest.mark.parametrize("name", ["cfg2", "cfg5"])
def test_forward_stream_with_the_allocation_free_backward(A, name):
    """asteroid_stage_backward_static beside forward passes on the second stream: the backward's workspace is
    the static array, the forward's scratch stays in the stage's own workspace."""
    cfg = CASES[name]()
    inp = gen.make_inputs(cfg, randomize_affine=True)
    one, _, _ = harness.run_hip(cfg, inp, K=2, rounds=2)
    two, _, _ = harness.run_hip(cfg, inp, K=2, rounds=2, forward_stream=True, static_backward=True)
    for r, (a, b) in enumerate(zip(one, two)):
        for k in ("y", "dx", "G", "W"):
            assert np.array_equal(a[k], b[k], equal_nan=True), (name, r, k)


@pytest.mark.parametrize("name", ["cfg2", "cfg3", "cfg4", "cfg5"])
def test_full_size_forward_stream_is_bit_identical(A, name):
    """bench.py's second timing configuration (K = 3 stashes, forward passes on a second stream) at the
    full size of the benchmark configurations: the same bits as the K = 1, one-stream round that the
    full-size tests score against the stored oracle values."""
    from asteroid_workloads import get_config
    cfg = get_config(name)
    inp = gen.make_inputs(cfg)
    v0 = harness.golden_velocity(cfg, inp["params"].size)
    one = harness.run_hip_one_round(cfg, inp, v0=v0, K=1)
    two = harness.run_hip_one_round(cfg, inp, v0=v0, K=3, forward_stream=True)
    for k in ("y", "dx", "G", "W", "V"):
        if one[k] is None:
            continue
        assert np.isfinite(one[k]).all(), (name, k)
        assert np.array_equal(one[k], two[k]), (name, k)
    assert one["loss"] == two["loss"]


def test_forward_stream_with_one_stash_and_switching_back(A):
    """K = 1 leaves nothing to overlap (every forward waits for the slot's backward) and must still be
    right; NULL returns to one stream; the call is refused inside a round."""
    import torch
    cfg = C.cfg2(B=2, M=3, hw=10)
    inp = gen.make_inputs(cfg, randomize_affine=True)
    one, _, _ = harness.run_hip(cfg, inp, K=1, rounds=2)
    two, _, _ = harness.run_hip(cfg, inp, K=1, rounds=2, forward_stream=True)
    for a, b in zip(one, two):
        for k in ("y", "dx", "G", "W"):
            assert np.array_equal(a[k], b[k]), k
    st = A.Stage(cfg.layers, cfg.B, cfg.M, 2, cfg.in_shape)
    fs = torch.cuda.Stream()
    st.set_forward_stream(fs.cuda_stream)
    st.set_forward_stream(None)
    st.set_forward_stream(fs.cuda_stream)
    x = torch.zeros((2, 24, 10, 10), device="cuda:0")
    y = torch.zeros((2, 32, 5, 5), device="cuda:0")
    torch.cuda.synchronize()
    st.forward(0, x, None, y)
    with pytest.raises(A.AsteroidError) as e:
        st.set_forward_stream(None)
    assert e.value.status == -2
    st.close()


@pytest.mark.parametrize("name,forward_stream", [("cfg2", False), ("cfg2", True), ("cfg5", False), ("cfg5", True)])
def test_round_captured_in_a_graph_replays_bit_identically(A, name, forward_stream):
    """A whole round (K forward passes, 1F1B, the update) is kernel launches and event waits on the
    stage's streams - no allocation, no memset, no host synchronisation - so a caller may capture it
    into a HIP graph.  Every replay is checked against the eager run of the same round, with eager
    work and synchronisations between the replays."""
    import torch
    cfg = CASES[name]()
    K = 2
    inp = gen.make_inputs(cfg, randomize_affine=True)
    eager, _, _ = harness.run_hip(cfg, inp, K=K, rounds=4, forward_stream=forward_stream)

    dev = torch.device("cuda:0")
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    cs = torch.cuda.Stream()
    B, M = cfg.B, cfg.M
    with torch.cuda.stream(cs):
        st = A.Stage(cfg.layers, B, M, K, cfg.in_shape, cfg.dtype, cfg.layout, cfg.needs_input_grad,
                     stream=cs.cuda_stream)
        st.set_params(inp["params"])
        fs = None
        if forward_stream:
            fs = torch.cuda.Stream()
            st.set_forward_stream(fs.cuda_stream)
        x = torch.from_numpy(inp["x"]).to(dev).to(tdt).contiguous()
        dy = torch.from_numpy(inp["dy"]).to(dev).to(tdt).contiguous()
        xs = [x[m * B:(m + 1) * B].clone() for m in range(M)]
        dys = [dy[m * B:(m + 1) * B].clone() for m in range(M)]
        ys = [torch.zeros_like(d) for d in dys]
        dxs = [torch.zeros_like(v) for v in xs]
        torch.cuda.synchronize()

        def one_round():
            for m in range(K):
                st.forward(m, xs[m], None, ys[m])
            for m in range(M):
                st.backward(m, dys[m], dxs[m])
                if m + K < M:
                    st.forward(m + K, xs[m + K], None, ys[m + K])
            st.step(cfg.lr, cfg.momentum)

        def state():
            torch.cuda.synchronize()
            return dict(y=torch.cat(ys).float().cpu().numpy(), dx=torch.cat(dxs).float().cpu().numpy(), W=st.get_params())

        one_round()                       # round 0 eagerly
        s0 = state()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=cs):
            one_round()                   # recorded, not run
        torch.cuda.synchronize()
        got = [s0]
        for r in range(1, 4):
            g.replay()
            got.append(state())           # synchronises, copies to the host: eager work between the replays
            junk = torch.randn(1 << 16, device=dev).sum().item()
            assert junk == junk
        st.close()
    for r in range(4):
        for k in ("y", "dx", "W"):
            assert np.array_equal(got[r][k], eager[r][k], equal_nan=True), (name, forward_stream, r, k)
