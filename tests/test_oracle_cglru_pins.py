"""Pins for the complex-gated LRU oracle (Appendix B): each checks it against something other
than itself - the real layer's pinned oracle on the special case theta = 0, the recurrence
written out in real 2x2 rotation arithmetic, brute-force unrolled sums, closed forms,
invariants the appendix states (half as many gate / state dimensions, |a~_t| < 1,
|a~_t|^2 + (1 - |a~_t|^2) = 1), and central finite differences for the adjoint."""
import cmath
import math

import numpy as np
import pytest

import oracle
import rglru_inputs as gen


def small(seed=0, B=2, T=9, D=16, nb=2, **kw):
    inp = gen.make_cg_inputs(B=B, T=T, D=D, nb=nb, act="f32", seed=seed, **kw)
    return {k: (None if v is None else v.astype(np.float64)) for k, v in inp.items()}


def params(p):
    return p["W_a"], p["W_x"], p["b_a"], p["b_x"], p["Lambda"], p["theta"]


def test_shapes_gate_and_state_dimensions_are_half_the_input_s():
    p = small(seed=1, h0=True, bias=True)
    y, hT, g = oracle.cg_lru(p["u"], *params(p), h0=p["h0"], want_gates=True)
    assert y.shape == (2, 9, 16) and hT.shape == (2, 16)
    for k in ("r", "i", "a", "m"):
        assert g[k].shape == (2, 9, 8)
    assert np.iscomplexobj(g["a"]) and not np.iscomplexobj(g["r"])
    np.testing.assert_array_equal(hT, y[:, -1])


def test_decay_modulus_and_phase():
    p = small(seed=2, bias=True)
    g = oracle.cg_gates(p["u"], *params(p))
    mod = np.abs(g["a"])
    sig = 1.0 / (1.0 + np.exp(-p["Lambda"]))
    np.testing.assert_allclose(mod, sig ** (8.0 * g["r"]), rtol=1e-13)
    assert np.all(mod < 1.0) and np.all(mod > 0.0)
    # phase c r theta, here inside (-pi, pi) so the principal angle is the phase itself
    assert np.all(8.0 * g["r"] * p["theta"] < np.pi)
    np.testing.assert_allclose(np.angle(g["a"]), 8.0 * g["r"] * p["theta"], rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(mod ** 2 + g["m"] ** 2, 1.0, rtol=1e-14)
    # against 40-digit arithmetic on a few entries: a~^(c r) with a~ = sigmoid(Lambda) e^{i theta}
    import mpmath
    mpmath.mp.dps = 40
    for (b, t, h) in [(0, 0, 0), (1, 4, 5), (1, 8, 7)]:
        base = mpmath.mpf(1) / (1 + mpmath.exp(-mpmath.mpf(float(p["Lambda"][h])))) * mpmath.exp(1j * mpmath.mpf(float(p["theta"][h])))
        want = complex(base ** (8 * mpmath.mpf(float(g["r"][b, t, h]))))
        assert abs(g["a"][b, t, h] - want) < 1e-14


def test_gate_blocks_see_real_and_imaginary_parts_of_their_own_channels():
    p = small(seed=3, B=1, T=4, D=16, nb=2, bias=True)   # H = 8, hs = 4
    g = oracle.cg_gates(p["u"], *params(p))
    x, H, hs = p["u"], 8, 4
    for blk in range(2):
        for j in range(hs):
            for t in range(4):
                acc = p["b_a"][blk * hs + j]
                for k in range(hs):
                    acc += p["W_a"][blk, j, k] * x[0, t, blk * hs + k]
                    acc += p["W_a"][blk, j, hs + k] * x[0, t, H + blk * hs + k]
                assert abs(g["r"][0, t, blk * hs + j] - 1 / (1 + math.exp(-acc))) < 1e-14
    # one block = the appendix's dense H x D matrix with columns in the order of x_t
    q = small(seed=4, B=1, T=3, D=12, nb=1, bias=True)
    g1 = oracle.cg_gates(q["u"], *params(q))
    dense = q["W_x"][0]                       # [6][12]
    want = 1 / (1 + np.exp(-(q["u"] @ dense.T + q["b_x"])))
    np.testing.assert_allclose(g1["i"], want, rtol=1e-13)


def test_theta_zero_reduces_to_the_real_layer():
    """theta = 0 and gate weights that ignore the imaginary half: the real part is the RG-LRU
    on the first half of the channels; the imaginary part is the same linear recurrence (same
    gates) fed with the second half."""
    p = small(seed=5, B=2, T=11, D=16, nb=2, h0=True, bias=True)
    H, hs = 8, 4
    W_a, W_x = p["W_a"].copy(), p["W_x"].copy()
    W_a[:, :, hs:] = 0.0
    W_x[:, :, hs:] = 0.0
    theta = np.zeros(H)
    y, hT = oracle.cg_lru(p["u"], W_a, W_x, p["b_a"], p["b_x"], p["Lambda"], theta, h0=p["h0"])
    y_re, hT_re, gts = oracle.rglru(p["u"][..., :H], W_a[:, :, :hs], W_x[:, :, :hs], p["b_a"], p["b_x"],
                                    p["Lambda"], h0=p["h0"][:, :H], want_gates=True)
    np.testing.assert_allclose(y[..., :H], y_re, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(hT[:, :H], hT_re, rtol=1e-12)
    y_im, _ = oracle.scan(gts["a"], gts["i"] * p["u"][..., H:], h0=p["h0"][:, H:])
    np.testing.assert_allclose(y[..., H:], y_im, rtol=1e-12, atol=1e-15)


def test_recurrence_in_real_rotation_arithmetic():
    """The complex product written out on (real, imaginary) pairs: multiplying by a~_t scales by
    |a~_t| and rotates by its phase."""
    p = small(seed=6, B=2, T=7, D=12, nb=3, h0=True, bias=True)
    H = 6
    y, _, g = oracle.cg_lru(p["u"], *params(p), h0=p["h0"], want_gates=True)
    for b in range(2):
        for h in range(H):
            re, im = p["h0"][b, h], p["h0"][b, H + h]
            for t in range(7):
                rho = math.exp(g["log_mod"][b, t, h])
                co, si = math.cos(g["phase"][b, t, h]), math.sin(g["phase"][b, t, h])
                gain = math.sqrt(1 - rho * rho) * g["i"][b, t, h]
                re, im = (rho * (co * re - si * im) + gain * p["u"][b, t, h],
                          rho * (si * re + co * im) + gain * p["u"][b, t, H + h])
                assert abs(y[b, t, h] - re) < 1e-13 and abs(y[b, t, H + h] - im) < 1e-13


@pytest.mark.parametrize("T", [1, 6])
def test_recurrence_equals_unrolled_sum(T):
    p = small(seed=7, B=1, T=T, D=8, nb=1, h0=True, bias=True)
    H = 4
    y, _, g = oracle.cg_lru(p["u"], *params(p), h0=p["h0"], want_gates=True)
    for h in range(H):
        for t in range(T):
            tot = complex(p["h0"][0, h], p["h0"][0, H + h])
            for k in range(t + 1):
                tot *= complex(g["a"][0, k, h])
            for s in range(t + 1):
                term = g["m"][0, s, h] * g["i"][0, s, h] * complex(p["u"][0, s, h], p["u"][0, s, H + h])
                for k in range(s + 1, t + 1):
                    term *= complex(g["a"][0, k, h])
                tot += term
            assert abs(complex(y[0, t, h], y[0, t, H + h]) - tot) < 1e-13


def test_constant_gates_closed_form_geometric_series():
    # W = 0: gates are constants r = sigmoid(b_a), i = sigmoid(b_x); constant input x~:
    # h~_t = a~^(t+1) h~_0 + m i x~ (1 - a~^(t+1)) / (1 - a~)
    p = small(seed=8, B=1, T=12, D=8, nb=2, h0=True, bias=True)
    H = 4
    W0 = np.zeros_like(p["W_a"])
    x = np.broadcast_to(p["u"][:, :1], p["u"].shape).copy()
    y, _ = oracle.cg_lru(x, W0, W0, p["b_a"], p["b_x"], p["Lambda"], p["theta"], h0=p["h0"])
    for h in range(H):
        r = 1 / (1 + math.exp(-p["b_a"][h])); i = 1 / (1 + math.exp(-p["b_x"][h]))
        base = 1 / (1 + math.exp(-p["Lambda"][h])) * cmath.exp(1j * p["theta"][h])
        a = cmath.exp(8 * r * cmath.log(base))
        m = math.sqrt(1 - abs(a) ** 2)
        xt = complex(x[0, 0, h], x[0, 0, H + h]); h0 = complex(p["h0"][0, h], p["h0"][0, H + h])
        for t in range(12):
            want = a ** (t + 1) * h0 + m * i * xt * (1 - a ** (t + 1)) / (1 - a)
            assert abs(complex(y[0, t, h], y[0, t, H + h]) - want) < 1e-12


def test_closed_input_gate_is_a_decaying_rotation_of_the_initial_state():
    p = small(seed=9, B=2, T=9, D=8, nb=1, h0=True, bias=True)
    H = 4
    bx = np.full(H, -1e4)
    y, _, g = oracle.cg_lru(p["u"], p["W_a"], p["W_x"], p["b_a"], bx, p["Lambda"], p["theta"], h0=p["h0"],
                            want_gates=True)
    hc = y[..., :H] + 1j * y[..., H:]
    h0 = p["h0"][:, :H] + 1j * p["h0"][:, H:]
    np.testing.assert_allclose(np.abs(hc), np.abs(h0)[:, None] * np.exp(np.cumsum(g["log_mod"], axis=1)), rtol=1e-12)
    turned = np.angle(hc * np.conj(h0)[:, None])
    want = np.cumsum(g["phase"], axis=1)
    np.testing.assert_allclose(np.exp(1j * turned), np.exp(1j * want), rtol=0, atol=1e-12)


def test_forward_is_conv_then_layer_splits_in_time_and_decodes_step_by_step():
    p = small(seed=10, B=2, T=13, D=8, nb=2, h0=True, bias=True, state=True)
    kw = dict(conv_w=p["conv_w"], conv_b=p["conv_b"])
    y, hT, st = oracle.cg_forward(p["u"], *params(p), h0=p["h0"], state_in=p["state"], **kw)
    # the Conv1D in front is Section 2.3's: the real layer's pinned routine gives the same x
    x, st_ref = oracle.conv1d(p["u"], p["conv_w"], conv_b=p["conv_b"], state_in=p["state"], want_state=True)
    y2, hT2 = oracle.cg_lru(x, *params(p), h0=p["h0"])
    np.testing.assert_allclose(y, y2, rtol=1e-13, atol=1e-15)
    np.testing.assert_array_equal(st, st_ref)
    ya, ha, sa = oracle.cg_forward(p["u"][:, :2], *params(p), h0=p["h0"], state_in=p["state"], **kw)
    yb, hb, sb = oracle.cg_forward(p["u"][:, 2:], *params(p), h0=ha, state_in=sa, **kw)
    np.testing.assert_allclose(np.concatenate([ya, yb], 1), y, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(hb, hT, rtol=1e-13)
    np.testing.assert_array_equal(sb, st)
    h, state = p["h0"].copy(), p["state"].copy()
    for t in range(13):
        yt = oracle.cg_decode_step(p["u"][:, t], *params(p), h, state, **kw)
        np.testing.assert_allclose(yt, y[:, t], rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(h, hT, rtol=1e-12)
    np.testing.assert_array_equal(state, st)
    # without the Conv1D the input is x_t itself
    y3, hT3, st3 = oracle.cg_forward(x, *params(p), h0=p["h0"])
    np.testing.assert_array_equal(y3, y2)
    assert st3 is None


def _loss(p, dy, dhT, conv, **over):
    q = dict(p); q.update(over)
    y, hT, _ = oracle.cg_forward(q["u"], q["W_a"], q["W_x"], q["b_a"], q["b_x"], q["Lambda"], q["theta"],
                                 conv_w=q["conv_w"] if conv else None, conv_b=q["conv_b"] if conv else None,
                                 h0=q["h0"], state_in=q["state"] if conv else None)
    return float(np.sum(dy * y) + np.sum(dhT * hT))


@pytest.mark.parametrize("T,conv", [(5, True), (1, True), (4, False)])
def test_backward_matches_central_finite_differences(T, conv):
    p = small(seed=20 + T, B=2, T=T, D=8, nb=2, h0=True, bias=True, dy=True, state=True)
    dy, dhT = p["dy"], p["dhT"]
    g = oracle.cg_backward(p["u"], *params(p), dy, conv_w=p["conv_w"] if conv else None,
                           conv_b=p["conv_b"] if conv else None, h0=p["h0"],
                           state_in=p["state"] if conv else None, dhT=dhT)
    names = {"u": "du", "h0": "dh0", "W_a": "dW_a", "W_x": "dW_x", "b_a": "db_a", "b_x": "db_x",
             "Lambda": "dLambda", "theta": "dtheta"}
    if conv:
        names.update({"conv_w": "dconv_w", "conv_b": "dconv_b"})
    else:
        assert "dconv_w" not in g
    eps = 1e-6
    for k, gk in names.items():
        base = p[k]
        fd = np.zeros_like(base)
        it = np.nditer(base, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            hi = base.copy(); hi[idx] += eps
            lo = base.copy(); lo[idx] -= eps
            fd[idx] = (_loss(p, dy, dhT, conv, **{k: hi}) - _loss(p, dy, dhT, conv, **{k: lo})) / (2 * eps)
        scale = np.abs(fd).max() + 1e-12
        err = np.abs(g[gk] - fd).max() / scale
        assert err < 2e-7, (k, err)


def test_backward_directional_derivative_larger_shape():
    p = small(seed=30, B=3, T=17, D=24, nb=3, h0=True, bias=True, dy=True, state=True)
    dy, dhT = p["dy"], p["dhT"]
    g = oracle.cg_backward(p["u"], *params(p), dy, conv_w=p["conv_w"], conv_b=p["conv_b"], h0=p["h0"],
                           state_in=p["state"], dhT=dhT)
    names = {"u": "du", "h0": "dh0", "W_a": "dW_a", "W_x": "dW_x", "b_a": "db_a", "b_x": "db_x",
             "Lambda": "dLambda", "theta": "dtheta", "conv_w": "dconv_w", "conv_b": "dconv_b"}
    rng = np.random.default_rng(31)
    eps = 1e-6
    for k, gk in names.items():
        v = rng.normal(size=p[k].shape)
        fd = (_loss(p, dy, dhT, True, **{k: p[k] + eps * v}) - _loss(p, dy, dhT, True, **{k: p[k] - eps * v})) / (2 * eps)
        an = float(np.sum(g[gk] * v))
        assert abs(an - fd) <= 1e-6 * (abs(fd) + 1.0), (k, an, fd)


def test_backward_with_theta_zero_reduces_to_the_real_layer_s_adjoint():
    p = small(seed=32, B=2, T=10, D=16, nb=2, h0=True, bias=True, dy=True)
    H, hs = 8, 4
    W_a, W_x = p["W_a"].copy(), p["W_x"].copy()
    W_a[:, :, hs:] = 0.0
    W_x[:, :, hs:] = 0.0
    dy = p["dy"].copy(); dy[..., H:] = 0.0          # loss on the real part only
    dhT = p["dhT"].copy(); dhT[:, H:] = 0.0
    h0 = p["h0"].copy(); h0[:, H:] = 0.0
    u = p["u"].copy(); u[..., H:] = 0.0            # imaginary part identically zero
    g = oracle.cg_backward(u, W_a, W_x, p["b_a"], p["b_x"], p["Lambda"], np.zeros(H), dy, h0=h0, dhT=dhT)
    w = np.zeros((4, H)); w[0] = 1.0
    ref = oracle.backward(u[..., :H], W_a[:, :, :hs], W_x[:, :, :hs], p["b_a"], p["b_x"], p["Lambda"], w,
                          dy[..., :H], h0=h0[:, :H], dhT=dhT[:, :H])
    np.testing.assert_allclose(g["du"][..., :H], ref["du"], rtol=1e-11, atol=1e-15)
    np.testing.assert_allclose(g["dW_a"][:, :, :hs], ref["dW_a"], rtol=1e-11, atol=1e-15)
    np.testing.assert_allclose(g["dW_x"][:, :, :hs], ref["dW_x"], rtol=1e-11, atol=1e-15)
    for k in ("db_a", "db_x", "dLambda"):
        np.testing.assert_allclose(g[k], ref[k], rtol=1e-11, atol=1e-15)
    np.testing.assert_allclose(g["dh0"][:, :H], ref["dh0"], rtol=1e-11)
