"""GPU parity of the complex-gated LRU (Appendix B) against its complex128 oracle, through the
C ABI, on the same seeded inputs. Tolerances as for the real layer: 1e-5 in fp32 storage, 2e-2
in bf16 storage (relative error with an rms floor)."""
import numpy as np
import pytest

import oracle
import rglru_inputs as gen

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}

SHAPES = [
    # B, T, D, nb, act
    (2, 37, 96, 3, "f32"),       # hs = 16, ragged T
    (3, 5, 40, 5, "f32"),        # hs = 4, fewer steps than a tile
    (1, 1, 16, 1, "f32"),        # one step, one dense block
    (2, 130, 512, 2, "bf16"),    # hs = 128
    (2, 100, 640, 2, "bf16"),    # hs = 160: ten column blocks of the matrix-core passes
    (3, 70, 192, 2, "bf16"),     # hs = 48: a partial column block
    (2, 70, 384, 2, "bf16"),     # hs = 96: the fused forward with one of its four waves idle
    (1, 200, 256, 2, "bf16"),    # hs = 64: ... with two
    (40, 45, 512, 4, "bf16"),    # 160 (gate block, sequence) pairs: the backward recomputes with the fused kernel
    (1, 300, 1024, 1, "bf16"),   # hs = 512: more outputs than threads
    (4, 20, 24, 12, "bf16"),     # hs = 1: per-channel gates
]


def runner():
    import paper_2402_19427_amd.runner as rn
    return rn


def f64(inp):
    return {k: (None if v is None else np.asarray(v, np.float64)) for k, v in inp.items()}


def params(q):
    return q["W_a"], q["W_x"], q["b_a"], q["b_x"], q["Lambda"], q["theta"]


@pytest.mark.parametrize("B,T,D,nb,act", SHAPES)
@pytest.mark.parametrize("conv", [True, False])
def test_cg_forward_and_backward_match_oracle(B, T, D, nb, act, conv):
    rn = runner()
    inp = gen.make_cg_inputs(B, T, D, nb, act=act, seed=B * 10 + T + D, h0=True, state=True, bias=True, dy=True)
    pos0 = 7
    dp = rn.CgDeviceProblem(inp, B, T, D, nb, act, conv=conv)
    u, h0 = rn.to_device(inp["u"], act), rn.to_device(inp["h0"], "f32")
    ring = rn.to_device(gen.ring_from_chrono(inp["state"], pos0), act) if conv else None
    y, hT, st = dp.forward(u, h0=h0, state_in=ring, pos0=pos0)
    # the same call without the optional scratch (one pass instead of two)
    y1, hT1, _ = dp.forward(u, h0=h0, state_in=ring, pos0=pos0, scratch=False)
    assert gen.rel_err(rn.to_host(y1), rn.to_host(y)) < (2e-6 if act == "f32" else 1e-2)
    # (bf16 storage: the two-pass form takes x_t in half precision into its gate products)
    assert gen.rel_err(rn.to_host(hT1), rn.to_host(hT)) < (2e-6 if act == "f32" else 1e-2)
    q = f64(inp)
    kw = dict(conv_w=q["conv_w"], conv_b=q["conv_b"], state_in=q["state"]) if conv else {}
    y_ref, hT_ref, st_ref = oracle.cg_forward(q["u"], *params(q), h0=q["h0"], **kw)
    assert gen.rel_err(rn.to_host(y), y_ref) < TOL[act]
    assert gen.rel_err(rn.to_host(hT), hT_ref) < TOL[act]
    if conv:
        np.testing.assert_array_equal(gen.chrono_from_ring(rn.to_host(st), pos0 + T), st_ref)
    g = dp.backward(u, rn.to_device(inp["dy"], act), h0=h0, state_in=ring, pos0=pos0,
                    dhT=rn.to_device(inp["dhT"], "f32"))
    ref = oracle.cg_backward(q["u"], *params(q), q["dy"], h0=q["h0"], dhT=q["dhT"], **kw)
    assert set(g) == set(ref)
    errs = {k: gen.rel_err(rn.to_host(g[k]), ref[k]) for k in ref}
    print("errors:", {k: float("%.3g" % v) for k, v in errs.items()})
    for k in ref:
        assert errs[k] < TOL[act], (k, errs)


@pytest.mark.parametrize("B,D,nb,act", [(5, 64, 2, "f32"), (19, 512, 2, "bf16"), (3, 1024, 1, "bf16")])
@pytest.mark.parametrize("conv", [True, False])
def test_cg_decode_steps_match_oracle_and_forward(B, D, nb, act, conv):
    rn = runner()
    nsteps = 7
    inp = gen.make_cg_inputs(B, 1, D, nb, act=act, seed=B + D, h0=True, state=True, decode_tokens=nsteps, bias=True)
    dp = rn.CgDeviceProblem(inp, B, 1, D, nb, act, conv=conv)
    pos = 11
    h = rn.to_device(inp["h0"], "f32")
    ring = rn.to_device(gen.ring_from_chrono(inp["state"], pos), act) if conv else None
    q = f64(inp)
    h_ref, st_ref = q["h0"].copy(), q["state"].copy()
    kw = dict(conv_w=q["conv_w"], conv_b=q["conv_b"]) if conv else {}
    for s in range(nsteps):
        y = dp.decode_step(rn.to_device(inp["u_dec"][s], act), h, ring, pos + s)
        y_ref = oracle.cg_decode_step(q["u_dec"][s], *params(q), h_ref, st_ref, **kw)
        assert gen.rel_err(rn.to_host(y), y_ref) < TOL[act], s
        assert gen.rel_err(rn.to_host(h), h_ref) < TOL[act], s
        if conv:
            np.testing.assert_array_equal(gen.chrono_from_ring(rn.to_host(ring), pos + s + 1), st_ref)


def test_cg_forward_in_pieces_equals_one_shot():
    rn = runner()
    B, T, D, nb, act = 2, 45, 128, 2, "bf16"
    inp = gen.make_cg_inputs(B, T, D, nb, act=act, seed=3, h0=True, bias=True)
    dp = rn.CgDeviceProblem(inp, B, T, D, nb, act)
    u = rn.to_device(inp["u"], act)
    y_all, hT_all, st_all = dp.forward(u, h0=rn.to_device(inp["h0"], "f32"))
    h, state, pos, ys = rn.to_device(inp["h0"], "f32"), None, 0, []
    for T1 in (1, 2, 13, 29):
        y, h, state = dp.forward(u[:, pos:pos + T1].contiguous(), h0=h, state_in=state, pos0=pos)
        ys.append(rn.to_host(y))
        pos += T1
    # (short pieces run in one pass with fp32 gate products, long ones on the matrix cores with
    # x_t in half precision: equal up to that rounding, a bf16 step of y here and there)
    assert gen.rel_err(np.concatenate(ys, axis=1), rn.to_host(y_all)) < 1e-2
    assert gen.rel_err(rn.to_host(h), rn.to_host(hT_all)) < 1e-2
    np.testing.assert_array_equal(rn.to_host(state), rn.to_host(st_all))


def test_cg_at_the_paper_s_block_shape_full_width():
    """The complex-gated layer at width 2560 in 10 blocks (hs = 128, the [128][256] gate matrices the
    matrix-core passes are built for), 2048 steps: forward and every gradient against the oracle."""
    rn = runner()
    B, T, D, nb, act = 2, 2048, 2560, 10, "bf16"
    inp = gen.make_cg_inputs(B, T, D, nb, act=act, seed=11, h0=True, bias=True, dy=True)
    dp = rn.CgDeviceProblem(inp, B, T, D, nb, act)
    u, h0 = rn.to_device(inp["u"], act), rn.to_device(inp["h0"], "f32")
    y, hT, _ = dp.forward(u, h0=h0)
    g = dp.backward(u, rn.to_device(inp["dy"], act), h0=h0, dhT=rn.to_device(inp["dhT"], "f32"))
    q = f64(inp)
    kw = dict(conv_w=q["conv_w"], conv_b=q["conv_b"])
    y_ref, hT_ref, _ = oracle.cg_forward(q["u"], *params(q), h0=q["h0"], **kw)
    assert gen.rel_err(rn.to_host(y), y_ref) < TOL[act]
    assert gen.rel_err(rn.to_host(hT), hT_ref) < TOL[act]
    ref = oracle.cg_backward(q["u"], *params(q), q["dy"], h0=q["h0"], dhT=q["dhT"], **kw)
    errs = {k: gen.rel_err(rn.to_host(g[k]), ref[k]) for k in ref}
    print("errors:", {k: float("%.3g" % v) for k, v in errs.items()})
    for k in ref:
        assert errs[k] < TOL[act], (k, errs)
