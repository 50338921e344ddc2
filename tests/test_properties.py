"""Property tests (hypothesis, derandomised): identities of the method that hold for any shape,
split point or mask - on the float64 oracle (CPU) and on the HIP library (GPU, through the C
ABI). Section 2.3 (Conv1D state), Section 2.4 eq. (4) (the recurrence is affine in h_{t-1}),
Section 5 / Appendix F (decode with carried states)."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import oracle
import rglru_inputs as gen

CFG = dict(max_examples=12, deadline=None, derandomize=True)


def f64(inp):
    return {k: (None if v is None else np.asarray(v, np.float64)) for k, v in inp.items()}


def params(q):
    return q["W_a"], q["W_x"], q["b_a"], q["b_x"], q["Lambda"], q["conv_w"]


# ------------------------------------------------------------------------- oracle (CPU)
@settings(**CFG)
@given(seed=st.integers(0, 10 ** 6), T=st.integers(1, 40), cuts=st.lists(st.integers(0, 40), max_size=4))
def test_oracle_any_split_in_time_equals_one_shot(seed, T, cuts):
    q = f64(gen.make_inputs(2, T, 8, 2, act="f32", seed=seed, h0=True, state=True, bias=True))
    y, hT, s_out = oracle.forward(q["u"], *params(q), conv_b=q["conv_b"], h0=q["h0"], state_in=q["state"])
    edges = sorted({0, T, *[c for c in cuts if c < T]})
    h, state, ys = q["h0"], q["state"], []
    for lo, hi in zip(edges, edges[1:]):
        yp, h, state = oracle.forward(q["u"][:, lo:hi], *params(q), conv_b=q["conv_b"], h0=h, state_in=state)
        ys.append(yp)
    np.testing.assert_allclose(np.concatenate(ys, axis=1), y, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(h, hT, rtol=1e-12, atol=1e-14)
    np.testing.assert_array_equal(state, s_out)


@settings(**CFG)
@given(seed=st.integers(0, 10 ** 6), T=st.integers(1, 30), alpha=st.floats(-2.0, 3.0))
def test_oracle_outputs_are_affine_in_the_initial_state(seed, T, alpha):
    q = f64(gen.make_inputs(2, T, 8, 2, act="f32", seed=seed, h0=True, bias=True))
    rng = np.random.default_rng(seed)
    h1, h2 = q["h0"], rng.normal(size=q["h0"].shape)
    run = lambda h: oracle.forward(q["u"], *params(q), conv_b=q["conv_b"], h0=h)[0]
    mix = run(alpha * h1 + (1 - alpha) * h2)
    np.testing.assert_allclose(mix, alpha * run(h1) + (1 - alpha) * run(h2), rtol=1e-10, atol=1e-12)


@settings(**CFG)
@given(seed=st.integers(0, 10 ** 6), T=st.integers(1, 30), data=st.data())
def test_oracle_packed_row_equals_its_documents_run_alone(seed, T, data):
    mask = np.array(data.draw(st.lists(st.booleans(), min_size=T, max_size=T)), np.uint8)[None, :]
    q = f64(gen.make_inputs(1, T, 8, 2, act="f32", seed=seed, h0=True, state=True, bias=True, dy=True))
    y, hT, _ = oracle.forward(q["u"], *params(q), conv_b=q["conv_b"], h0=q["h0"], state_in=q["state"], reset=mask)
    g = oracle.backward(q["u"], *params(q), q["dy"], conv_b=q["conv_b"], h0=q["h0"], state_in=q["state"],
                        dhT=q["dhT"], reset=mask)
    starts = [0] + [t for t in range(1, T) if mask[0, t]]
    dW = np.zeros_like(g["dW_a"])
    for lo, hi in zip(starts, starts[1:] + [T]):
        carried = lo == 0 and not mask[0, 0]
        kw = dict(conv_b=q["conv_b"], h0=q["h0"] if carried else None, state_in=q["state"] if carried else None)
        yd, hd, _ = oracle.forward(q["u"][:, lo:hi], *params(q), **kw)
        np.testing.assert_allclose(y[:, lo:hi], yd, rtol=1e-13, atol=1e-300)
        gd = oracle.backward(q["u"][:, lo:hi], *params(q), q["dy"][:, lo:hi], dhT=q["dhT"] if hi == T else None, **kw)
        np.testing.assert_allclose(g["du"][:, lo:hi], gd["du"], rtol=1e-11, atol=1e-300)
        dW += gd["dW_a"]
    np.testing.assert_allclose(hT, hd, rtol=1e-13)
    np.testing.assert_allclose(g["dW_a"], dW, rtol=1e-10, atol=1e-13)


# ------------------------------------------------------------------------- HIP library (GPU)
SHAPES_GPU = [(2, 96, 3, "f32"), (2, 512, 2, "bf16"), (1, 320, 2, "bf16"), (2, 1024, 2, "bf16")]
CLOSE = {"f32": 2e-6, "bf16": 1e-2}   # two results of the library against each other, each rounded to its storage type


def runner():
    import paper_2402_19427_amd.runner as rn
    return rn


@pytest.mark.gpu
@settings(**CFG)
@given(shape=st.sampled_from(SHAPES_GPU), seed=st.integers(0, 10 ** 6), T=st.integers(2, 200),
       cuts=st.lists(st.integers(1, 199), max_size=3))
def test_gpu_any_split_in_time_equals_one_shot(shape, seed, T, cuts):
    rn = runner()
    B, D, nb, act = shape
    inp = gen.make_inputs(B, T, D, nb, act=act, seed=seed, h0=True, bias=True)
    dp = rn.DeviceProblem(inp, B, T, D, nb, act)
    u = rn.to_device(inp["u"], act)
    y, hT, s_out = dp.forward(u, h0=rn.to_device(inp["h0"], "f32"))
    edges = sorted({0, T, *[c for c in cuts if c < T]})
    h, state, ys = rn.to_device(inp["h0"], "f32"), None, []
    for lo, hi in zip(edges, edges[1:]):
        yp, h, state = dp.forward(u[:, lo:hi].contiguous(), h0=h, state_in=state, pos0=lo)
        ys.append(rn.to_host(yp))
    assert gen.rel_err(np.concatenate(ys, axis=1), rn.to_host(y)) < CLOSE[act]
    assert gen.rel_err(rn.to_host(h), rn.to_host(hT)) < CLOSE[act]
    np.testing.assert_array_equal(gen.chrono_from_ring(rn.to_host(state), T), gen.chrono_from_ring(rn.to_host(s_out), T))


@pytest.mark.gpu
@settings(**CFG)
@given(shape=st.sampled_from(SHAPES_GPU), seed=st.integers(0, 10 ** 6), T=st.integers(1, 24))
def test_gpu_decode_steps_equal_the_forward_over_the_same_tokens(shape, seed, T):
    rn = runner()
    B, D, nb, act = shape
    inp = gen.make_inputs(B, T, D, nb, act=act, seed=seed, h0=True, state=True, bias=True)
    dp = rn.DeviceProblem(inp, B, T, D, nb, act)
    pos0 = seed % 7
    u = rn.to_device(inp["u"], act)
    ring0 = gen.ring_from_chrono(inp["state"], pos0)
    y, hT, s_out = dp.forward(u, h0=rn.to_device(inp["h0"], "f32"), state_in=rn.to_device(ring0, act), pos0=pos0)
    h, ring, ys = rn.to_device(inp["h0"], "f32"), rn.to_device(ring0, act), []
    for t in range(T):
        ys.append(rn.to_host(dp.decode_step(u[:, t].contiguous(), h, ring, pos0 + t)))
    assert gen.rel_err(np.stack(ys, axis=1), rn.to_host(y)) < CLOSE[act]
    assert gen.rel_err(rn.to_host(h), rn.to_host(hT)) < CLOSE[act]
    np.testing.assert_array_equal(rn.to_host(ring), rn.to_host(s_out))


@pytest.mark.gpu
@settings(**CFG)
@given(shape=st.sampled_from(SHAPES_GPU), seed=st.integers(0, 10 ** 6), T=st.integers(1, 150),
       alpha=st.floats(-1.0, 2.0))
def test_gpu_final_state_is_affine_in_the_initial_state(shape, seed, T, alpha):
    rn = runner()
    B, D, nb, act = shape
    inp = gen.make_inputs(B, T, D, nb, act=act, seed=seed, h0=True, bias=True)
    dp = rn.DeviceProblem(inp, B, T, D, nb, act)
    u = rn.to_device(inp["u"], act)
    h1 = inp["h0"]
    h2 = np.random.default_rng(seed).standard_normal(h1.shape).astype(np.float32)
    a = np.float32(alpha)
    run = lambda h: rn.to_host(dp.forward(u, h0=rn.to_device(h, "f32"))[1]).astype(np.float64)   # hT: fp32, unrounded
    mix, e1, e2 = run(a * h1 + (1 - a) * h2), run(h1), run(h2)
    assert gen.rel_err(mix, float(a) * e1 + (1 - float(a)) * e2) < 2e-5


@pytest.mark.gpu
@settings(**CFG)
@given(shape=st.sampled_from(SHAPES_GPU), seed=st.integers(0, 10 ** 6), T=st.integers(1, 150), data=st.data())
def test_gpu_packed_calls_match_the_oracle_for_any_mask(shape, seed, T, data):
    import torch
    rn = runner()
    B, D, nb, act = shape
    density = data.draw(st.sampled_from([0.02, 0.2, 0.7]))
    rng = np.random.default_rng(seed)
    reset = (rng.random((B, T)) < density).astype(np.uint8)
    inp = gen.make_inputs(B, T, D, nb, act=act, seed=seed, h0=True, state=True, bias=True, dy=True)
    dp = rn.DeviceProblem(inp, B, T, D, nb, act)
    pos0 = seed % 5
    u, h0 = rn.to_device(inp["u"], act), rn.to_device(inp["h0"], "f32")
    ring = rn.to_device(gen.ring_from_chrono(inp["state"], pos0), act)
    r_dev = torch.from_numpy(reset).cuda()
    y, hT, s_out = dp.forward_packed(u, r_dev, h0=h0, state_in=ring, pos0=pos0)
    q = f64(inp)
    kw = dict(conv_b=q["conv_b"], h0=q["h0"], state_in=q["state"], reset=reset)
    y_ref, hT_ref, st_ref = oracle.forward(q["u"], *params(q), **kw)
    tol = 1e-5 if act == "f32" else 2e-2
    assert gen.rel_err(rn.to_host(y), y_ref) < tol
    assert gen.rel_err(rn.to_host(hT), hT_ref) < tol
    np.testing.assert_array_equal(gen.chrono_from_ring(rn.to_host(s_out), pos0 + T), st_ref)
    g = dp.backward_packed(u, r_dev, y, rn.to_device(inp["dy"], act), h0=h0, state_in=ring, pos0=pos0,
                           dhT=rn.to_device(inp["dhT"], "f32"))
    ref = oracle.backward(q["u"], *params(q), q["dy"], dhT=q["dhT"], **kw)
    for k in ("du", "dh0", "dW_a", "dW_x", "db_a", "db_x", "dLambda", "dconv_w", "dconv_b"):
        assert gen.rel_err(rn.to_host(g[k]), ref[k]) < tol, k
