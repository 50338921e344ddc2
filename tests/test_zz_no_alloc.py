"""rglru_forward_static (the entry point that takes its scratch from a static device array)
against rglru_forward on the same inputs: two calls in a row through the C ABI, the second on a
smaller input, each bit for bit equal to the call with a caller-provided workspace; a shape
beyond the array's size is refused before anything is launched."""
import numpy as np
import pytest

import rglru_inputs as gen

pytestmark = pytest.mark.gpu


def run_both(B, T, D, nb, seed):
    import torch
    import paper_2402_19427_amd as R
    import paper_2402_19427_amd.runner as rn
    inp = gen.make_inputs(B, T, D, nb, act="bf16", seed=seed, h0=True, state=True, bias=True)
    dp = rn.DeviceProblem(inp, B, T, D, nb, "bf16")
    u = rn.to_device(inp["u"], "bf16")
    h0 = rn.to_device(inp["h0"], "f32")
    ring = rn.to_device(gen.ring_from_chrono(inp["state"], 5), "bf16")
    sh = dp.shape()
    assert 0 < R.rglru_workspace_bytes(sh, R.OP_FORWARD) <= R.STATIC_SCRATCH_BYTES
    y_ref, hT_ref, st_ref = dp.forward(u, h0=h0, state_in=ring, pos0=5)
    y, hT, st = dp.empty_act(B, T, D), dp.empty_f32(B, D), dp.empty_act(B, 3, D)
    y.fill_(float("nan")); hT.fill_(float("nan")); st.fill_(float("nan"))
    R.rglru_forward_static(sh, dp.params, u, h0, ring, 5, y, hT, st)
    torch.cuda.synchronize()
    for got, want in ((y, y_ref), (hT, hT_ref), (st, st_ref)):
        np.testing.assert_array_equal(rn.to_host(got), rn.to_host(want))
    return rn.to_host(y)


def test_static_scratch_forward_equals_the_workspace_call_twice_in_a_row():
    # sliced in time (64 units x 4 slices: the scratch carries records between workgroups) ...
    y1 = run_both(8, 600, 2048, 8, seed=21)
    # ... then a smaller input, one unit in 16 slices, on what the first call left in the array
    y2 = run_both(1, 300, 256, 1, seed=22)
    assert np.isfinite(y1).all() and np.isfinite(y2).all()


def test_static_scratch_forward_refuses_shapes_beyond_its_array():
    import paper_2402_19427_amd as R
    # 64 blocks of 256 channels in 4 time slices: 8 MiB of records + 8 MiB of weights + the status word
    sh = R.make_shape(1, 2048, 16384, 64, R.BF16)
    assert R.rglru_workspace_bytes(sh, R.OP_FORWARD) > R.STATIC_SCRATCH_BYTES
    par = R.make_params(0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000)
    with pytest.raises(R.RglruError) as e:
        R.rglru_forward_static(sh, par, 0x1000, None, None, 0, 0x1000, None, None)
    assert e.value.code == R.ERR_WORKSPACE and "static" in str(e.value)
