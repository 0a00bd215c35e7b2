"""GPU test of asteroid_stage_backward_static (the backward entry point that allocates nothing:
its workspace is a file-scope device array): results bit-identical to asteroid_stage_backward,
on two calls in a row, the second on a smaller stage (the array keeps the first call's
contents), and the size limit is refused with AST_EINVAL."""
import numpy as np
import pytest

import harness
from asteroid_workloads import configs as C
from asteroid_workloads import gen

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def A():
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    import paper_2408_08015_amd as A
    A.load_library()
    return A


def both(cfg, K):
    inp = gen.make_inputs(cfg, randomize_affine=True)
    ref, _, mem = harness.run_hip(cfg, inp, K=K, rounds=2)
    got, _, _ = harness.run_hip(cfg, inp, K=K, rounds=2, static_backward=True)
    assert mem[3] <= 32 << 20, "test stage must fit the static workspace"
    for r in range(2):
        for k in ("y", "dx", "G", "W"):
            if ref[r][k] is None:
                continue
            assert np.array_equal(ref[r][k], got[r][k]), (cfg.name, r, k)
        if ref[r]["loss"] is not None:
            assert ref[r]["loss"] == got[r]["loss"]


def test_backward_static_matches_backward(A):
    # first the larger stage, then smaller ones: leftovers of a call must not reach the next
    both(C.cfg2(B=4, M=2, hw=28), K=1)
    both(C.cfg1(B=4, M=2, hw=16), K=2)
    both(C.cfg1(B=2, M=2, hw=8), K=1)
    both(C.cfg5(B=2, M=2, S=32, d=128, heads=2, ffn=256, nlayers=1), K=1)
    both(C.cfg4(B=1, M=2, hw=8, cin=16, c=24), K=1)


def test_backward_static_refuses_a_large_stage(A):
    import torch
    cfg = C.cfg2(B=32, M=1, hw=56)   # workspace of a few hundred MB
    st = A.Stage(cfg.layers, cfg.B, cfg.M, 1, cfg.in_shape, cfg.dtype, cfg.layout, cfg.needs_input_grad,
                 stream=torch.cuda.current_stream().cuda_stream)
    assert st.memory()[3] > 32 << 20
    x = torch.zeros((cfg.B,) + tuple(cfg.in_shape), device="cuda")
    y = torch.zeros((cfg.B,) + tuple(gen.out_shape(cfg.layers, cfg.in_shape)), device="cuda")
    st.forward(0, x, None, y, None)
    with pytest.raises(A.AsteroidError) as e:
        st.backward_static(0, torch.zeros_like(y), torch.zeros_like(x))
    assert e.value.status == -1 and "AST_STATIC_SCRATCH_BYTES" in str(e.value)
    st.backward(0, torch.zeros_like(y), torch.zeros_like(x))   # the stage is still usable
    torch.cuda.synchronize()
    st.close()
