"""Pins for the float64 oracle: every part of it is checked against something other than
itself - a library routine on a special case, a closed form, an invariant stated by the
paper, a brute-force expansion, high-precision spot values, or finite differences.

Citations: Conv1D - Section 2.3 (recurrent block); gates, decay and recurrence - Section 2.4
eqs. (1)-(4); log-space form - Appendix A; alpha^2 + beta^2 = 1 - Appendix A "Gate behaviour";
state sizes - Appendix F "Cache sizes"; initialisation range - Section 2.4.
"""
import mpmath
import numpy as np
import pytest
import scipy.linalg
import scipy.signal

import oracle
import rglru_inputs as gen


def sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def small(seed=0, B=2, T=9, D=8, nb=2, **kw):
    inp = gen.make_inputs(B=B, T=T, D=D, nb=nb, act="f32", seed=seed, **kw)
    return {k: (None if v is None else v.astype(np.float64)) for k, v in inp.items()}


# ------------------------------------------------------------------ Conv1D
def test_conv_equals_numpy_convolve():
    p = small(seed=1, B=2, T=13, D=5, nb=1)
    x = oracle.conv1d(p["u"], p["conv_w"])
    for b in range(2):
        for d in range(5):
            want = np.convolve(p["u"][b, :, d], p["conv_w"][:, d])[:13]
            np.testing.assert_allclose(x[b, :, d], want, rtol=0, atol=1e-14)


def test_conv_delta_and_delay_taps():
    p = small(seed=2, T=10)
    w = np.zeros((4, 8)); w[0] = 1.0
    np.testing.assert_array_equal(oracle.conv1d(p["u"], w), p["u"])
    w = np.zeros((4, 8)); w[3] = 1.0
    x = oracle.conv1d(p["u"], w)
    np.testing.assert_array_equal(x[:, 3:], p["u"][:, :-3])
    np.testing.assert_array_equal(x[:, :3], 0.0)
    # a tap on lag 1 only sees the previous input: strictly causal
    w = np.zeros((4, 8)); w[1] = 2.0
    x = oracle.conv1d(p["u"], w)
    np.testing.assert_array_equal(x[:, 1:], 2.0 * p["u"][:, :-1])


def test_conv_bias_is_added_once():
    p = small(seed=3)
    bias = np.arange(8, dtype=np.float64)
    x0 = oracle.conv1d(p["u"], p["conv_w"])
    x1 = oracle.conv1d(p["u"], p["conv_w"], conv_b=bias)
    np.testing.assert_allclose(x1 - x0, np.broadcast_to(bias, x0.shape), atol=1e-14)


@pytest.mark.parametrize("T1", [0, 1, 2, 3, 5])
def test_conv_state_carry_equals_one_shot(T1):
    p = small(seed=4, T=11)
    full, st_full = oracle.conv1d(p["u"], p["conv_w"], want_state=True)
    xa, st = oracle.conv1d(p["u"][:, :T1], p["conv_w"], want_state=True)
    xb, st2 = oracle.conv1d(p["u"][:, T1:], p["conv_w"], state_in=st, want_state=True)
    np.testing.assert_allclose(np.concatenate([xa, xb], axis=1), full, atol=1e-14)
    np.testing.assert_array_equal(st2, st_full)
    np.testing.assert_array_equal(st_full, p["u"][:, -3:])


def test_conv_state_out_short_sequences():
    # fewer than 3 new tokens: the outgoing state keeps carried-in rows, oldest first
    p = small(seed=5, T=2, state=True)
    _, st = oracle.conv1d(p["u"], p["conv_w"], state_in=p["state"], want_state=True)
    np.testing.assert_array_equal(st[:, 0], p["state"][:, 2])
    np.testing.assert_array_equal(st[:, 1:], p["u"])
    _, st0 = oracle.conv1d(p["u"], p["conv_w"], want_state=True)  # no state = zero padding
    np.testing.assert_array_equal(st0[:, 0], 0.0)


def test_conv_state_is_the_three_previous_inputs():
    # Appendix F: the cache of a width-4 filter is 3 inputs. A state equal to the last three
    # inputs of a prefix must reproduce the continuation exactly.
    p = small(seed=6, T=12)
    full = oracle.conv1d(p["u"], p["conv_w"])
    tail = oracle.conv1d(p["u"][:, 7:], p["conv_w"], state_in=p["u"][:, 4:7])
    np.testing.assert_allclose(tail, full[:, 7:], atol=1e-14)


# ------------------------------------------------------- block-diagonal gates
def test_gates_equal_dense_block_diag_matmul():
    p = small(seed=7, B=2, T=6, D=12, nb=3, bias=True)
    x = p["u"]
    _, _, g = oracle.rglru(x, p["W_a"], p["W_x"], p["b_a"], p["b_x"], p["Lambda"],
                           want_gates=True)
    Wa = scipy.linalg.block_diag(*p["W_a"])
    Wx = scipy.linalg.block_diag(*p["W_x"])
    np.testing.assert_allclose(g["r"], sigmoid(x @ Wa.T + p["b_a"]), rtol=1e-13)
    np.testing.assert_allclose(g["i"], sigmoid(x @ Wx.T + p["b_x"]), rtol=1e-13)


def test_gates_single_block_is_dense_layer_and_full_split_is_per_channel_scale():
    p = small(seed=8, B=1, T=5, D=6, nb=1, bias=True)
    _, _, g = oracle.rglru(p["u"], p["W_a"], p["W_x"], p["b_a"], p["b_x"], p["Lambda"],
                           want_gates=True)
    np.testing.assert_allclose(g["r"], sigmoid(p["u"] @ p["W_a"][0].T + p["b_a"]), rtol=1e-13)
    p = small(seed=9, B=1, T=5, D=6, nb=6, bias=True)
    _, _, g = oracle.rglru(p["u"], p["W_a"], p["W_x"], p["b_a"], p["b_x"], p["Lambda"],
                           want_gates=True)
    np.testing.assert_allclose(g["i"], sigmoid(p["u"] * p["W_x"][:, 0, 0] + p["b_x"]), rtol=1e-13)


def test_gate_weight_orientation_is_out_by_in():
    # W[g][j][k] multiplies input k and lands on output j: a single nonzero entry shows it
    D = 4
    Wa = np.zeros((1, D, D)); Wa[0, 1, 3] = 2.0
    x = np.zeros((1, 1, D)); x[0, 0, 3] = 0.7
    z = np.zeros(D)
    _, _, g = oracle.rglru(x, Wa, np.zeros((1, D, D)), z, z, np.full(D, 5.0), want_gates=True)
    want = np.full(D, 0.5); want[1] = sigmoid(1.4)
    np.testing.assert_allclose(g["r"][0, 0], want, rtol=1e-14)


# ------------------------------------------------------------- decay a_t, m_t
def test_decay_power_form_equals_log_form_and_is_strictly_inside_unit_interval():
    p = small(seed=10, B=2, T=7, D=8, nb=2, bias=True)
    _, _, g = oracle.rglru(p["u"], p["W_a"], p["W_x"], p["b_a"], p["b_x"], p["Lambda"],
                           want_gates=True)
    power = sigmoid(p["Lambda"]) ** (8.0 * g["r"])          # eq. (3) as printed
    np.testing.assert_allclose(g["a"], power, rtol=1e-13)
    assert np.all(g["a"] > 0.0) and np.all(g["a"] < 1.0)


def test_decay_with_open_gate_lies_in_the_initialisation_range():
    # r = 1 (huge b_a) gives a_t = sigmoid(Lambda)^8, which the generator draws in [0.9, 0.999].
    # The sign printed in Appendix A (softplus(+Lambda)) would give ~1e-15 here.
    p = small(seed=11, B=1, T=3, D=16, nb=2)
    _, _, g = oracle.rglru(p["u"], p["W_a"], p["W_x"], np.full(16, 60.0), p["b_x"], p["Lambda"],
                           want_gates=True)
    assert np.all(g["a"] >= 0.9 - 1e-6) and np.all(g["a"] <= 0.999 + 1e-6)
    np.testing.assert_allclose(g["a"][0, 0], sigmoid(p["Lambda"]) ** 8, rtol=1e-12)


def test_decay_against_50_digit_arithmetic():
    mpmath.mp.dps = 50
    lam = np.array([-3.0, 0.0, 4.3, 9.0])
    bias = np.array([-2.0, 0.5, 0.0, 3.0])
    z = np.zeros((1, 4, 4))
    _, _, g = oracle.rglru(np.zeros((1, 1, 4)), z, z, bias, np.zeros(4), lam, want_gates=True)
    for d in range(4):
        r = 1 / (1 + mpmath.exp(-mpmath.mpf(bias[d])))
        a = (1 / (1 + mpmath.exp(-mpmath.mpf(lam[d])))) ** (8 * r)
        m = mpmath.sqrt(1 - a * a)
        assert abs(g["a"][0, 0, d] - float(a)) <= 4e-16 * float(a)
        assert abs(g["m"][0, 0, d] - float(m)) <= 1e-14 * float(m)


def test_alpha_squared_plus_beta_squared_is_one():
    p = small(seed=12, B=2, T=7, D=8, nb=2, bias=True)
    _, _, g = oracle.rglru(p["u"], p["W_a"], p["W_x"], p["b_a"], p["b_x"], p["Lambda"],
                           want_gates=True)
    np.testing.assert_allclose(g["a"] ** 2 + g["m"] ** 2, 1.0, atol=1e-15)


# ------------------------------------------------------------------ recurrence
def test_zero_input_is_pure_decay_closed_form():
    # u = 0 and zero biases: r = 1/2, so a_t = sigmoid(Lambda)^4 and h_t = h0 a^(t+1)
    p = small(seed=13, B=2, T=20, D=8, nb=2, h0=True)
    y, hT, _ = oracle.forward(np.zeros_like(p["u"]), p["W_a"], p["W_x"], p["b_a"], p["b_x"],
                              p["Lambda"], p["conv_w"], h0=p["h0"])
    t = np.arange(1, 21)[None, :, None]
    want = p["h0"][:, None, :] * sigmoid(p["Lambda"]) ** (4.0 * t)
    np.testing.assert_allclose(y, want, rtol=1e-12)
    np.testing.assert_allclose(hT, want[:, -1], rtol=1e-12)


def test_closed_input_gate_decays_by_the_product_of_a():
    # b_x = -1e4 closes the input gate exactly (i = 0) while a_t still varies with x
    p = small(seed=14, B=2, T=12, D=8, nb=2, h0=True)
    y, _, g = oracle.rglru(p["u"], p["W_a"], p["W_x"], p["b_a"], np.full(8, -1e4), p["Lambda"],
                           h0=p["h0"], want_gates=True)
    np.testing.assert_array_equal(g["i"], 0.0)
    np.testing.assert_allclose(y, p["h0"][:, None, :] * np.cumprod(g["a"], axis=1), rtol=1e-13)


def test_constant_input_geometric_series_and_fixed_point():
    D, T = 6, 4000
    rng = np.random.default_rng(15)
    lam = gen.make_lambda(rng, D).astype(np.float64)
    ba, bx = rng.normal(size=D), rng.normal(size=D)
    xc = rng.normal(size=D)
    h0 = rng.normal(size=(1, D))
    z = np.zeros((1, D, D))
    x = np.broadcast_to(xc, (1, T, D)).copy()
    y, hT = oracle.rglru(x, z, z, ba, bx, lam, h0=h0)
    a = sigmoid(lam) ** (8.0 * sigmoid(ba))
    b = np.sqrt(1 - a * a) * sigmoid(bx) * xc
    n = np.arange(1, T + 1)[:, None]
    want = a ** n * h0 + b * (1 - a ** n) / (1 - a)
    np.testing.assert_allclose(y[0], want, rtol=1e-11, atol=1e-13)
    # the same through a library IIR filter: h_t - a h_{t-1} = b
    for d in range(D):
        zi = np.array([a[d] * h0[0, d]])
        f, _ = scipy.signal.lfilter([b[d]], [1.0, -a[d]], np.ones(T), zi=zi)
        np.testing.assert_allclose(y[0, :, d], f, rtol=1e-10, atol=1e-13)
    # fixed point b/(1-a) = sqrt((1+a)/(1-a)) i x, reached where a^T is negligible
    fast = a ** T < 1e-14
    assert fast.any()
    fp = np.sqrt((1 + a) / (1 - a)) * sigmoid(bx) * xc
    np.testing.assert_allclose(hT[0][fast], fp[fast], rtol=1e-10)


@pytest.mark.parametrize("T", [1, 2, 5, 8])
def test_recurrence_equals_unrolled_sum(T):
    p = small(seed=16 + T, B=2, T=T, D=8, nb=2, h0=True, bias=True)
    y, hT, g = oracle.rglru(p["u"], p["W_a"], p["W_x"], p["b_a"], p["b_x"], p["Lambda"],
                            h0=p["h0"], want_gates=True)
    a = g["a"]
    b = g["m"] * g["i"] * p["u"]
    for t in range(T):
        acc = np.prod(a[:, : t + 1], axis=1) * p["h0"]
        for j in range(t + 1):
            acc = acc + np.prod(a[:, j + 1 : t + 1], axis=1) * b[:, j]
        np.testing.assert_allclose(y[:, t], acc, rtol=1e-13, atol=1e-15)
    np.testing.assert_array_equal(hT, y[:, -1])


def test_output_is_affine_in_h0_with_slope_prod_a():
    # the gates do not depend on the state (Section 2.4), so y(h0+d) - y(h0) = d * prod a
    p = small(seed=30, B=2, T=10, D=8, nb=2, h0=True)
    args = (p["u"], p["W_a"], p["W_x"], p["b_a"], p["b_x"], p["Lambda"])
    y0, _, g = oracle.rglru(*args, h0=p["h0"], want_gates=True)
    delta = np.random.default_rng(1).normal(size=p["h0"].shape)
    y1, _ = oracle.rglru(*args, h0=p["h0"] + delta)
    np.testing.assert_allclose(y1 - y0, delta[:, None] * np.cumprod(g["a"], axis=1),
                               rtol=1e-9, atol=1e-13)
    yz, _ = oracle.rglru(*args, h0=None)
    y00, _ = oracle.rglru(*args, h0=np.zeros_like(p["h0"]))
    np.testing.assert_array_equal(yz, y00)


def test_stationary_variance_is_one_for_open_input_gate():
    # i = 1, constant a, iid unit-variance x: Var(h) -> (1-a^2)/(1-a^2) = 1
    rng = np.random.default_rng(31)
    D, T = 4, 200000
    z = np.zeros((1, D, D))
    x = rng.normal(size=(1, T, D))
    lam = np.array([2.0, 3.0, 4.0, 5.0])
    y, _ = oracle.rglru(x, z, z, np.zeros(D), np.full(D, 60.0), lam)
    var = y[0, 2000:].var(axis=0)
    np.testing.assert_allclose(var, 1.0, atol=0.08)


def test_forward_is_conv_then_rglru_and_splits_in_time():
    p = small(seed=32, B=2, T=14, D=8, nb=2, h0=True, bias=True)
    params = (p["W_a"], p["W_x"], p["b_a"], p["b_x"], p["Lambda"], p["conv_w"])
    y, hT, st = oracle.forward(p["u"], *params, conv_b=p["conv_b"], h0=p["h0"])
    x = oracle.conv1d(p["u"], p["conv_w"], conv_b=p["conv_b"])
    y2, hT2 = oracle.rglru(x, *params[:5], h0=p["h0"])
    np.testing.assert_array_equal(y, y2)
    np.testing.assert_array_equal(hT, hT2)
    ya, ha, sa = oracle.forward(p["u"][:, :5], *params, conv_b=p["conv_b"], h0=p["h0"])
    yb, hb, sb = oracle.forward(p["u"][:, 5:], *params, conv_b=p["conv_b"], h0=ha, state_in=sa)
    np.testing.assert_allclose(np.concatenate([ya, yb], 1), y, rtol=1e-14, atol=1e-15)
    np.testing.assert_allclose(hb, hT, rtol=1e-14)
    np.testing.assert_array_equal(sb, st)


# ---------------------------------------------------------------------- decode
def test_decode_steps_equal_one_forward():
    p = small(seed=33, B=3, T=9, D=8, nb=2, h0=True, bias=True, state=True)
    params = (p["W_a"], p["W_x"], p["b_a"], p["b_x"], p["Lambda"], p["conv_w"])
    y, hT, st = oracle.forward(p["u"], *params, conv_b=p["conv_b"], h0=p["h0"],
                               state_in=p["state"])
    h = p["h0"].copy()
    state = p["state"].copy()
    for t in range(9):
        yt = oracle.decode_step(p["u"][:, t], *params, h, state, conv_b=p["conv_b"])
        np.testing.assert_allclose(yt, y[:, t], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(h, hT, rtol=1e-13)
    np.testing.assert_array_equal(state, st)


def test_ring_layout_round_trip_and_slot_rule():
    rng = np.random.default_rng(34)
    st = rng.normal(size=(2, 3, 5))
    for pos in range(0, 8):
        ring = gen.ring_from_chrono(st, pos)
        np.testing.assert_array_equal(gen.chrono_from_ring(ring, pos), st)
        # the newest token (absolute position pos-1) sits in slot (pos-1) mod 3
        np.testing.assert_array_equal(ring[:, (pos - 1) % 3], st[:, 2])


# -------------------------------------------------------------------- backward
def _loss(p, dy, dhT, **over):
    q = dict(p); q.update(over)
    y, hT, _ = oracle.forward(q["u"], q["W_a"], q["W_x"], q["b_a"], q["b_x"], q["Lambda"],
                              q["conv_w"], conv_b=q["conv_b"], h0=q["h0"], state_in=q["state"])
    return float(np.sum(dy * y) + np.sum(dhT * hT))


@pytest.mark.parametrize("T,with_state", [(5, False), (3, True), (1, True), (7, True)])
def test_backward_matches_central_finite_differences(T, with_state):
    p = small(seed=40 + T, B=2, T=T, D=8, nb=2, h0=True, bias=True, dy=True, state=with_state)
    dy, dhT = p["dy"], p["dhT"]
    g = oracle.backward(p["u"], p["W_a"], p["W_x"], p["b_a"], p["b_x"], p["Lambda"], p["conv_w"],
                        dy, conv_b=p["conv_b"], h0=p["h0"], state_in=p["state"], dhT=dhT)
    names = {"u": "du", "h0": "dh0", "W_a": "dW_a", "W_x": "dW_x", "b_a": "db_a", "b_x": "db_x",
             "Lambda": "dLambda", "conv_w": "dconv_w", "conv_b": "dconv_b"}
    eps = 1e-6
    for k, gk in names.items():
        base = p[k]
        fd = np.zeros_like(base)
        it = np.nditer(base, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            hi = base.copy(); hi[idx] += eps
            lo = base.copy(); lo[idx] -= eps
            fd[idx] = (_loss(p, dy, dhT, **{k: hi}) - _loss(p, dy, dhT, **{k: lo})) / (2 * eps)
        scale = np.abs(fd).max() + 1e-12
        err = np.abs(g[gk] - fd).max() / scale
        assert err < 2e-7, (k, err)


def test_backward_directional_derivative_larger_shape():
    p = small(seed=50, B=3, T=17, D=24, nb=3, h0=True, bias=True, dy=True, state=True)
    dy, dhT = p["dy"], p["dhT"]
    g = oracle.backward(p["u"], p["W_a"], p["W_x"], p["b_a"], p["b_x"], p["Lambda"], p["conv_w"],
                        dy, conv_b=p["conv_b"], h0=p["h0"], state_in=p["state"], dhT=dhT)
    names = {"u": "du", "h0": "dh0", "W_a": "dW_a", "W_x": "dW_x", "b_a": "db_a", "b_x": "db_x",
             "Lambda": "dLambda", "conv_w": "dconv_w", "conv_b": "dconv_b"}
    rng = np.random.default_rng(51)
    eps = 1e-6
    for k, gk in names.items():
        v = rng.normal(size=p[k].shape)
        fd = (_loss(p, dy, dhT, **{k: p[k] + eps * v}) -
              _loss(p, dy, dhT, **{k: p[k] - eps * v})) / (2 * eps)
        an = float(np.sum(g[gk] * v))
        assert abs(an - fd) <= 1e-6 * (abs(fd) + 1.0), (k, an, fd)


def test_backward_without_optional_arguments():
    p = small(seed=52, B=2, T=6, D=8, nb=2, dy=True)
    g = oracle.backward(p["u"], p["W_a"], p["W_x"], p["b_a"], p["b_x"], p["Lambda"], p["conv_w"],
                        p["dy"])
    g0 = oracle.backward(p["u"], p["W_a"], p["W_x"], p["b_a"], p["b_x"], p["Lambda"],
                         p["conv_w"], p["dy"], h0=np.zeros((2, 8)), dhT=np.zeros((2, 8)),
                         state_in=np.zeros((2, 3, 8)), conv_b=np.zeros(8))
    for k in g:
        np.testing.assert_allclose(g[k], g0[k], rtol=1e-14, atol=1e-300)


def test_dh0_closed_form_with_closed_input_gate():
    # i = 0: y_t = h0 prod_{s<=t} a_s, so dL/dh0 = sum_t dy_t prod_{s<=t} a_s
    p = small(seed=53, B=2, T=9, D=8, nb=2, h0=True, dy=True)
    bx = np.full(8, -1e4)
    w = np.zeros((4, 8)); w[0] = 1.0
    _, _, gts = oracle.rglru(p["u"], p["W_a"], p["W_x"], p["b_a"], bx, p["Lambda"], h0=p["h0"],
                             want_gates=True)
    g = oracle.backward(p["u"], p["W_a"], p["W_x"], p["b_a"], bx, p["Lambda"], w, p["dy"],
                        h0=p["h0"])
    want = np.sum(p["dy"] * np.cumprod(gts["a"], axis=1), axis=1)
    np.testing.assert_allclose(g["dh0"], want, rtol=1e-12)


# --------------------------------------------------------- generator and helpers
def test_generator_distributions_and_bf16_rounding():
    p = gen.make_inputs(B=2, T=64, D=512, nb=2, act="bf16", seed=1001)
    a8 = sigmoid(p["Lambda"].astype(np.float64)) ** 8
    assert a8.min() >= 0.9 - 1e-5 and a8.max() <= 0.999 + 1e-5
    assert abs(p["u"].std() - 1.0) < 0.02
    assert abs(p["W_a"].std() * 16.0 - 1.0) < 0.05          # N(0, 1/bs), bs = 256
    assert abs(p["conv_w"].std() * 2.0 - 1.0) < 0.1          # N(0, 1/4)
    # stored values are exactly representable in bf16
    np.testing.assert_array_equal(gen.round_to_act(p["u"], "bf16"), p["u"])
    # round-to-nearest-even on the 16 dropped bits
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20, 1.0 + 3 * 2 ** -8], np.float32)
    np.testing.assert_array_equal(gen.round_to_act(x, "bf16"),
                                  np.array([1.0, 1.0, 1.0 + 2 ** -7, 1.0 + 2 ** -6], np.float32))
    q = gen.make_inputs(B=2, T=64, D=512, nb=2, act="bf16", seed=1001)
    np.testing.assert_array_equal(p["u"], q["u"])


def test_oracle_threads_do_not_change_results():
    p = small(seed=60, B=3, T=12, D=16, nb=4, h0=True)
    args = (p["u"], p["W_a"], p["W_x"], p["b_a"], p["b_x"], p["Lambda"], p["conv_w"])
    y1, h1, _ = oracle.forward(*args, h0=p["h0"])
    oracle.set_threads(4)
    try:
        y4, h4, _ = oracle.forward(*args, h0=p["h0"])
    finally:
        oracle.set_threads(1)
    np.testing.assert_array_equal(y1, y4)
    np.testing.assert_array_equal(h1, h4)


# ------------------------------------------------------------------ eq. (4) as a linear scan
def _scan_inputs(B, T, D, seed):
    rng = np.random.default_rng(seed)
    a = rng.uniform(0.5, 0.999, size=(B, T, D))
    g = rng.standard_normal((B, T, D))
    h0 = rng.standard_normal((B, D))
    return a, g, h0


def test_scan_special_cases_are_cumsum_and_cumprod():
    a, g, h0 = _scan_inputs(2, 40, 5, 0)
    # a = 1 without the input scale: a running sum on top of h0 (library routine)
    h, hT = oracle.scan(np.ones_like(a), g, h0, normalize=False)
    np.testing.assert_allclose(h, h0[:, None, :] + np.cumsum(g, axis=1), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(hT, h[:, -1], rtol=0, atol=0)
    # zero input: pure decay by the running product of a_t
    h, _ = oracle.scan(a, np.zeros_like(g), h0)
    np.testing.assert_allclose(h, h0[:, None, :] * np.cumprod(a, axis=1), rtol=1e-12)
    # no h0 means a zero initial state
    h_a, _ = oracle.scan(a, g, None)
    h_b, _ = oracle.scan(a, g, np.zeros_like(h0))
    np.testing.assert_array_equal(h_a, h_b)


def test_scan_constant_inputs_closed_form():
    # h_t = alpha^(t+1) h0 + sqrt(1 - alpha^2) beta (1 - alpha^(t+1)) / (1 - alpha)
    alpha, beta, T = 0.9, 0.7, 60
    a = np.full((1, T, 3), alpha)
    g = np.full((1, T, 3), beta)
    h0 = np.array([[0.0, 1.5, -2.0]])
    h, hT = oracle.scan(a, g, h0)
    k = np.arange(1, T + 1)[None, :, None]
    want = alpha ** k * h0[:, None, :] + np.sqrt(1 - alpha ** 2) * beta * (1 - alpha ** k) / (1 - alpha)
    np.testing.assert_allclose(h, want, rtol=1e-12)
    # the same without the input scale
    h, _ = oracle.scan(a, g, h0, normalize=False)
    np.testing.assert_allclose(h, alpha ** k * h0[:, None, :] + beta * (1 - alpha ** k) / (1 - alpha), rtol=1e-12)


@pytest.mark.parametrize("normalize", [True, False])
def test_scan_equals_unrolled_sum(normalize):
    a, g, h0 = _scan_inputs(1, 7, 2, 3)
    h, _ = oracle.scan(a, g, h0, normalize=normalize)
    for t in range(7):
        for d in range(2):
            tot = h0[0, d] * np.prod(a[0, :t + 1, d])
            for s in range(t + 1):
                m = np.sqrt(1 - a[0, s, d] ** 2) if normalize else 1.0
                tot += np.prod(a[0, s + 1:t + 1, d]) * m * g[0, s, d]
            assert abs(h[0, t, d] - tot) < 1e-12


def test_scan_log_form_equals_direct_form_and_keeps_precision_near_one():
    a, g, h0 = _scan_inputs(2, 30, 4, 4)
    h_dir, _ = oracle.scan(a, g, h0)
    h_log, _ = oracle.scan(np.log(a), g, h0, a_is_log=True)
    np.testing.assert_allclose(h_log, h_dir, rtol=1e-12, atol=1e-13)
    # log a = -eps: sqrt(1 - a^2) = sqrt(2 eps) (1 - eps/2 + O(eps^2)), which 1 - a*a cannot resolve
    eps = 1e-13
    h, _ = oracle.scan(np.full((1, 1, 1), -eps), np.ones((1, 1, 1)), None, a_is_log=True)
    assert abs(h[0, 0, 0] / (np.sqrt(2 * eps) * (1 - eps / 2)) - 1) < 1e-12


def test_scan_on_the_layer_s_own_gates_reproduces_the_layer():
    inp = gen.make_inputs(2, 25, 32, 4, act="f32", seed=5, h0=True)
    q = {k: (None if v is None else np.asarray(v, np.float64)) for k, v in inp.items()}
    x = oracle.conv1d(q["u"], q["conv_w"])
    y, hT, gates = oracle.rglru(x, q["W_a"], q["W_x"], q["b_a"], q["b_x"], q["Lambda"], h0=q["h0"],
                                want_gates=True)
    h, hT2 = oracle.scan(gates["a"], gates["i"] * x, q["h0"])
    np.testing.assert_allclose(h, y, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(hT2, hT, rtol=1e-11, atol=1e-13)
    # and the scale it applies is the layer's sqrt(1 - a^2)
    h3, _ = oracle.scan(gates["a"], gates["m"] * gates["i"] * x, q["h0"], normalize=False)
    np.testing.assert_allclose(h3, y, rtol=1e-11, atol=1e-13)


# ------------------------------------------------------------------ the block's merge (Section 2.3)
def test_gelu_is_z_times_the_normal_cdf():
    from scipy.stats import norm
    z = np.linspace(-8, 8, 801)
    np.testing.assert_allclose(oracle.gelu(z), z * norm.cdf(z), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(oracle.gelu_grad(z), norm.cdf(z) + z * norm.pdf(z), rtol=1e-13, atol=1e-15)
    # table values of Phi: Phi(1) = 0.841344746..., Phi(2) = 0.977249868..., Phi(0.5) = 0.691462461...
    np.testing.assert_allclose(oracle.gelu(np.array([0.0, 1.0, -1.0, 2.0, 0.5])),
                               [0.0, 0.8413447460685429, -0.15865525393145707, 1.9544997361036416,
                                0.34573123063700656], rtol=1e-14, atol=0)
    assert oracle.gelu_grad(np.array([0.0]))[0] == 0.5
    for approx in (False, True):      # z Phi(z) - (-z) Phi(-z) = z for either form
        np.testing.assert_allclose(oracle.gelu(z, approx) - oracle.gelu(-z, approx), z, rtol=0, atol=1e-14)


def test_gelu_tanh_form_stays_within_its_known_distance_of_the_exact_form():
    z = np.linspace(-8, 8, 3201)
    dev = np.abs(oracle.gelu(z, True) - oracle.gelu(z)).max()
    assert 4.6e-4 < dev < 4.8e-4            # 4.73e-4 near |z| = 2.7; a wrong constant leaves this band
    for approx in (False, True):
        e = 1e-6
        fd = (oracle.gelu(z + e, approx) - oracle.gelu(z - e, approx)) / (2 * e)
        np.testing.assert_allclose(oracle.gelu_grad(z, approx), fd, rtol=0, atol=2e-9)


@pytest.mark.parametrize("approx", [False, True])
def test_merge_and_its_adjoint(approx):
    rng = np.random.default_rng(11)
    y, br, dout = (rng.standard_normal((2, 9, 6)) for _ in range(3))
    out = oracle.merge(y, br, approx)
    np.testing.assert_allclose(out, y * oracle.gelu(br, approx), rtol=0, atol=0)
    dy, dbr = oracle.merge_backward(y, br, dout, approx)
    e = 1e-6
    for idx in [(0, 0, 0), (1, 8, 5), (0, 4, 3)]:
        for which, got in (("y", dy), ("br", dbr)):
            yp, ym, bp, bm = y.copy(), y.copy(), br.copy(), br.copy()
            if which == "y":
                yp[idx] += e
                ym[idx] -= e
            else:
                bp[idx] += e
                bm[idx] -= e
            fd = (np.sum(dout * oracle.merge(yp, bp, approx)) - np.sum(dout * oracle.merge(ym, bm, approx))) / (2 * e)
            assert abs(got[idx] - fd) < 1e-8


def test_backward_merge_matches_finite_differences_through_the_whole_path():
    inp = gen.make_inputs(2, 11, 16, 2, act="f32", seed=21, h0=True)
    q = {k: (None if v is None else np.asarray(v, np.float64)) for k, v in inp.items()}
    rng = np.random.default_rng(22)
    br = rng.standard_normal(q["u"].shape)
    dout = rng.standard_normal(q["u"].shape)
    args = (q["W_a"], q["W_x"], q["b_a"], q["b_x"], q["Lambda"], q["conv_w"])

    def loss(u, b):
        return np.sum(dout * oracle.forward_merge(u, b, *args, h0=q["h0"])[0])

    g = oracle.backward_merge(q["u"], br, *args, dout, h0=q["h0"])
    e = 1e-6
    for idx in [(0, 0, 0), (1, 10, 15), (0, 5, 7)]:
        up, um = q["u"].copy(), q["u"].copy()
        up[idx] += e
        um[idx] -= e
        assert abs(g["du"][idx] - (loss(up, br) - loss(um, br)) / (2 * e)) < 1e-7
        bp, bm = br.copy(), br.copy()
        bp[idx] += e
        bm[idx] -= e
        assert abs(g["dbranch"][idx] - (loss(q["u"], bp) - loss(q["u"], bm)) / (2 * e)) < 1e-7
    # a branch of large positive values is the identity: GeLU(z) -> z, so out = y * z
    big = np.full_like(br, 40.0)
    out, y, _, _ = oracle.forward_merge(q["u"], big, *args, h0=q["h0"])
    np.testing.assert_allclose(out, 40.0 * y, rtol=1e-14)


# ------------------------------------------------------------------ adjoint of the scan
def test_scan_adjoint_is_the_transpose_of_the_scan():
    # <dy, scan(b)> + <dhT, h_{T-1}> == <delta, b> + <dh0, h0> for the linear map (b, h0) -> h
    a, b, h0 = _scan_inputs(2, 23, 4, 8)
    rng = np.random.default_rng(9)
    dy = rng.standard_normal(a.shape)
    dhT = rng.standard_normal(h0.shape)
    h, hT = oracle.scan(a, b, h0, normalize=False)
    delta, dh0 = oracle.scan_adjoint(a, dy, dhT)
    lhs = np.sum(dy * h) + np.sum(dhT * hT)
    rhs = np.sum(delta * b) + np.sum(dh0 * h0)
    assert abs(lhs - rhs) < 1e-10 * max(1.0, abs(lhs))
    # the same recurrence run on flipped arrays: delta = flip(scan(flip(shifted a), flip(dy), dhT))
    a_next = np.concatenate([a[:, 1:], np.ones_like(a[:, :1])], axis=1)
    d2, _ = oracle.scan(a_next[:, ::-1].copy(), dy[:, ::-1].copy(), dhT, normalize=False)
    np.testing.assert_allclose(delta, d2[:, ::-1], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(dh0, a[:, 0] * delta[:, 0], rtol=1e-13)
    # log form, and no dhT
    d3, dh3 = oracle.scan_adjoint(np.log(a), dy, dhT, a_is_log=True)
    np.testing.assert_allclose(d3, delta, rtol=1e-12, atol=1e-13)
    d4, _ = oracle.scan_adjoint(a, dy, None)
    d5, _ = oracle.scan_adjoint(a, dy, np.zeros_like(dhT))
    np.testing.assert_array_equal(d4, d5)


def test_scan_adjoint_gives_the_gradient_of_the_decays_by_finite_differences():
    a, b, h0 = _scan_inputs(1, 9, 3, 10)
    rng = np.random.default_rng(11)
    dy = rng.standard_normal(a.shape)
    h, _ = oracle.scan(a, b, h0, normalize=False)
    delta, _ = oracle.scan_adjoint(a, dy)
    h_prev = np.concatenate([h0[:, None, :], h[:, :-1]], axis=1)
    da = delta * h_prev                       # dL/da_t = delta_t h_{t-1}
    e = 1e-6
    for idx in [(0, 0, 0), (0, 4, 1), (0, 8, 2)]:
        ap, am = a.copy(), a.copy()
        ap[idx] += e
        am[idx] -= e
        fd = (np.sum(dy * oracle.scan(ap, b, h0, normalize=False)[0])
              - np.sum(dy * oracle.scan(am, b, h0, normalize=False)[0])) / (2 * e)
        assert abs(da[idx] - fd) < 1e-7


# --------------------------------------------- document boundaries in packed sequences
# A row of the batch may hold several documents back to back; reset[b, t] != 0 marks the first
# step of a document. Nothing crosses such a step (no recurrent state, no Conv1D history), so a
# packed row must give exactly what its documents give when each is run alone as its own
# sequence - by the calls without a mask, which the pins above cover.
def _documents(reset_row, T):
    starts = [0] + [t for t in range(1, T) if reset_row[t]]
    return list(zip(starts, starts[1:] + [T]))


def _packed_case(seed, T=17):
    p = small(seed=seed, B=2, T=T, D=8, nb=2, h0=True, bias=True, dy=True, state=True)
    reset = np.zeros((2, T), np.uint8)
    reset[0, [4, 5, 11]] = 1            # a one-step document (4), no boundary at step 0
    reset[1, [0, 9, T - 2]] = 1         # boundary at step 0; the last document has 2 steps
    return p, reset


def test_reset_forward_equals_each_document_run_alone():
    p, reset = _packed_case(60)
    T = reset.shape[1]
    params = (p["W_a"], p["W_x"], p["b_a"], p["b_x"], p["Lambda"], p["conv_w"])
    y, hT, st = oracle.forward(p["u"], *params, conv_b=p["conv_b"], h0=p["h0"],
                               state_in=p["state"], reset=reset)
    for b in range(2):
        for lo, hi in _documents(reset[b], T):
            carried = lo == 0 and not reset[b, 0]
            yd, hd, sd = oracle.forward(p["u"][b:b + 1, lo:hi], *params, conv_b=p["conv_b"],
                                        h0=p["h0"][b:b + 1] if carried else None,
                                        state_in=p["state"][b:b + 1] if carried else None)
            np.testing.assert_allclose(y[b, lo:hi], yd[0], rtol=1e-14, atol=1e-300)
        np.testing.assert_allclose(hT[b], hd[0], rtol=1e-14)
        np.testing.assert_array_equal(st[b], sd[0])
    # row 1's last document has two steps: the oldest state row is the zero in front of it
    np.testing.assert_array_equal(st[1, 0], np.zeros(8))
    np.testing.assert_array_equal(st[1, 1:], p["u"][1, T - 2:])


def test_reset_special_cases():
    p = small(seed=61, B=2, T=11, D=8, nb=2, h0=True, bias=True, state=True)
    params = (p["W_a"], p["W_x"], p["b_a"], p["b_x"], p["Lambda"], p["conv_w"])
    kw = dict(conv_b=p["conv_b"], h0=p["h0"], state_in=p["state"])
    plain = oracle.forward(p["u"], *params, **kw)
    none = oracle.forward(p["u"], *params, reset=np.zeros((2, 11), np.uint8), **kw)
    for a, b in zip(plain, none):
        np.testing.assert_array_equal(a, b)
    # a boundary at step 0 alone = a fresh sequence: the states handed in are not used
    first = np.zeros((2, 11), np.uint8); first[:, 0] = 1
    fresh = oracle.forward(p["u"], *params, conv_b=p["conv_b"])
    at0 = oracle.forward(p["u"], *params, reset=first, **kw)
    for a, b in zip(fresh, at0):
        np.testing.assert_array_equal(a, b)
    # a boundary at every step: each output is the one-step layer on u_t alone,
    # y_t = sqrt(1 - a_t^2) i_t (w_0 u_t + b) with gates taken from that same x_t
    every = np.ones((2, 11), np.uint8)
    y, hT, st = oracle.forward(p["u"], *params, reset=every, **kw)
    x = p["conv_w"][0] * p["u"] + p["conv_b"]
    _, _, g = oracle.rglru(x, *params[:5], want_gates=True)
    np.testing.assert_allclose(y, np.sqrt(1 - g["a"] ** 2) * g["i"] * x, rtol=1e-11, atol=1e-300)
    np.testing.assert_array_equal(hT, y[:, -1])
    np.testing.assert_array_equal(st[:, :2], np.zeros((2, 2, 8)))
    np.testing.assert_array_equal(st[:, 2], p["u"][:, -1])


def test_reset_conv_and_recurrence_are_masked_separately_and_consistently():
    p, reset = _packed_case(62)
    params = (p["W_a"], p["W_x"], p["b_a"], p["b_x"], p["Lambda"], p["conv_w"])
    y, hT, st = oracle.forward(p["u"], *params, conv_b=p["conv_b"], h0=p["h0"],
                               state_in=p["state"], reset=reset)
    x, st2 = oracle.conv1d(p["u"], p["conv_w"], conv_b=p["conv_b"], state_in=p["state"],
                           want_state=True, reset=reset)
    y2, hT2 = oracle.rglru(x, *params[:5], h0=p["h0"], reset=reset)
    np.testing.assert_array_equal(y, y2)
    np.testing.assert_array_equal(hT, hT2)
    np.testing.assert_array_equal(st, st2)
    # the masked Conv1D by hand: lags that reach behind the document's first step drop out
    T = reset.shape[1]
    for b in range(2):
        for lo, hi in _documents(reset[b], T):
            for t in range(lo, hi):
                want = p["conv_b"].copy()
                for k in range(4):
                    s = t - k
                    if s >= lo:
                        want += p["conv_w"][k] * p["u"][b, s]
                    elif lo == 0 and not reset[b, 0]:
                        want += p["conv_w"][k] * p["state"][b, 3 + s]
                np.testing.assert_allclose(x[b, t], want, rtol=1e-14, atol=1e-15)


def test_reset_backward_equals_the_sum_over_documents_run_alone():
    p, reset = _packed_case(63)
    T = reset.shape[1]
    params = (p["W_a"], p["W_x"], p["b_a"], p["b_x"], p["Lambda"], p["conv_w"])
    g = oracle.backward(p["u"], *params, p["dy"], conv_b=p["conv_b"], h0=p["h0"],
                        state_in=p["state"], dhT=p["dhT"], reset=reset)
    total = {k: np.zeros_like(v) for k, v in g.items() if k not in ("du", "dh0")}
    for b in range(2):
        docs = _documents(reset[b], T)
        for lo, hi in docs:
            carried = lo == 0 and not reset[b, 0]
            gd = oracle.backward(p["u"][b:b + 1, lo:hi], *params, p["dy"][b:b + 1, lo:hi],
                                 conv_b=p["conv_b"],
                                 h0=p["h0"][b:b + 1] if carried else None,
                                 state_in=p["state"][b:b + 1] if carried else None,
                                 dhT=p["dhT"][b:b + 1] if hi == T else None)
            np.testing.assert_allclose(g["du"][b, lo:hi], gd["du"][0], rtol=1e-12, atol=1e-300)
            if lo == 0:
                want = gd["dh0"][0] if carried else np.zeros(8)
                np.testing.assert_allclose(g["dh0"][b], want, rtol=1e-12, atol=0)
            for k in total:
                total[k] += gd[k]
    for k in total:
        np.testing.assert_allclose(g[k], total[k], rtol=1e-11, atol=1e-14, err_msg=k)


def test_reset_backward_matches_central_finite_differences():
    p = small(seed=64, B=2, T=7, D=8, nb=2, h0=True, bias=True, dy=True, state=True)
    reset = np.zeros((2, 7), np.uint8)
    reset[0, [2, 3]] = 1
    reset[1, [0, 5]] = 1
    dy, dhT = p["dy"], p["dhT"]

    def loss(**over):
        q = dict(p); q.update(over)
        y, hT, _ = oracle.forward(q["u"], q["W_a"], q["W_x"], q["b_a"], q["b_x"], q["Lambda"],
                                  q["conv_w"], conv_b=q["conv_b"], h0=q["h0"],
                                  state_in=q["state"], reset=reset)
        return float(np.sum(dy * y) + np.sum(dhT * hT))

    g = oracle.backward(p["u"], p["W_a"], p["W_x"], p["b_a"], p["b_x"], p["Lambda"], p["conv_w"],
                        dy, conv_b=p["conv_b"], h0=p["h0"], state_in=p["state"], dhT=dhT,
                        reset=reset)
    names = {"u": "du", "h0": "dh0", "W_a": "dW_a", "W_x": "dW_x", "b_a": "db_a", "b_x": "db_x",
             "Lambda": "dLambda", "conv_w": "dconv_w", "conv_b": "dconv_b"}
    eps = 1e-6
    for k, gk in names.items():
        base = p[k]
        fd = np.zeros_like(base)
        it = np.nditer(base, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            hi = base.copy(); hi[idx] += eps
            lo = base.copy(); lo[idx] -= eps
            fd[idx] = (loss(**{k: hi}) - loss(**{k: lo})) / (2 * eps)
        scale = np.abs(fd).max() + 1e-12
        err = np.abs(g[gk] - fd).max() / scale
        assert err < 2e-7, (k, err)
    np.testing.assert_array_equal(g["dh0"][1], np.zeros(8))
