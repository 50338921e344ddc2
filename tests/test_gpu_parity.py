"""GPU parity: the HIP library, called through its C ABI, against the float64 oracle on the
same seeded inputs, element by element.

Tolerances (relative error with an rms floor, rglru_inputs.rel_err):
  fp32 storage  : 1e-5
  bf16 storage  : 2e-2   (bf16 in / fp32 state and accumulation)
Bit-exact where the work is a copy (conv ring state).
"""
import numpy as np
import pytest

import oracle
import rglru_inputs as gen

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}
# parameter gradients are long sums of rounded products (compensated in the fp32 kernels); the
# same bars apply to each tensor
GRAD_TOL = {"f32": 1e-5, "bf16": 2e-2}


def runner():
    import paper_2402_19427_amd.runner as rn
    return rn


def f64(inp):
    return {k: (None if v is None else np.asarray(v, np.float64)) for k, v in inp.items()}


def oracle_forward(inp, h0=None, state=None):
    q = f64(inp)
    oracle.set_threads(8 if q["u"].size > (1 << 20) else 1)   # same results for any thread count
    return oracle.forward(q["u"], q["W_a"], q["W_x"], q["b_a"], q["b_x"], q["Lambda"],
                          q["conv_w"], conv_b=q.get("conv_b"), h0=h0, state_in=state)


SHAPES = [
    # B, T, D, nb, act            what it exercises
    (1, 256, 256, 4, "f32"),     # workload C0
    (2, 37, 96, 3, "f32"),       # ragged T, bs = 32
    (3, 5, 40, 5, "f32"),        # bs = 8, fewer steps than one tile
    (1, 1, 16, 1, "f32"),        # single step, single dense block
    (2, 130, 512, 2, "bf16"),    # bs = 256: the tuned block size, ragged T
    (2, 70, 320, 2, "bf16"),     # bs = 160: the paper's 16 blocks at width 2560 (MFMA path, padded tile)
    (3, 300, 2560, 16, "bf16"),  # the same at full width: 48 units x 5 slices, ragged T
    (1, 1100, 384, 2, "bf16"),   # bs = 192, 16 slices
    (40, 40, 288, 2, "bf16"),    # bs = 144 (a multiple of 16 only), one workgroup per unit
    (2, 100, 2816, 8, "bf16"),   # bs = 352 (16 blocks at width 5632): separate passes, 2 K chunks
    (1, 700, 1024, 2, "bf16"),   # bs = 512 (16 blocks at width 8192), scan in time slices
    (3, 70, 256, 4, "bf16"),     # bs = 64: separate passes, one partial K chunk
    (1, 130, 1536, 2, "bf16"),   # bs = 768: three K chunks
    (2, 37, 96, 2, "bf16"),      # bs = 48, width not a multiple of 256: generic kernels
    (4, 1, 1024, 2, "bf16"),     # bs = 512, a single step: four rows in all
    (1, 3, 512, 8, "bf16"),      # bs = 64, fewer rows than a tile
    (1, 9, 24, 24, "bf16"),      # nb = D: per-channel gates
    (2, 300, 600, 2, "bf16"),    # bs = 300 > workgroup size
    (1, 1, 256, 1, "bf16"),      # MFMA path, one step
    (1, 1500, 256, 1, "bf16"),   # MFMA path, one unit in 16 time slices
    (33, 70, 1024, 4, "bf16"),   # MFMA path, 132 units: one workgroup per unit, no slicing
    (8, 600, 2048, 8, "bf16"),   # MFMA path, 64 units x 4 slices, record ring wraps (19 tiles > 16)
    (1, 12400, 512, 2, "bf16"),  # MFMA path, few units and a long sequence: contiguous windows in two passes, ragged end
    (2, 12320, 320, 2, "bf16"),  # the same with narrower blocks in the padded tile, two sequences
]


@pytest.mark.parametrize("B,T,D,nb,act", SHAPES)
@pytest.mark.parametrize("full", [False, True])
def test_forward_matches_oracle(B, T, D, nb, act, full):
    rn = runner()
    inp = gen.make_inputs(B, T, D, nb, act=act, seed=B * 1000 + T + D, h0=full, state=full,
                          bias=full)
    pos0 = 5 if full else 0
    dp = rn.DeviceProblem(inp, B, T, D, nb, act)
    u = rn.to_device(inp["u"], act)
    h0 = rn.to_device(inp["h0"], "f32")
    ring = None
    if full:
        ring = rn.to_device(gen.ring_from_chrono(inp["state"], pos0), act)
    y, hT, st = dp.forward(u, h0=h0, state_in=ring, pos0=pos0)
    y_ref, hT_ref, st_ref = oracle_forward(inp, h0=inp["h0"], state=inp["state"])
    assert gen.rel_err(rn.to_host(y), y_ref) < TOL[act]
    assert gen.rel_err(rn.to_host(hT), hT_ref) < TOL[act]
    np.testing.assert_array_equal(gen.chrono_from_ring(rn.to_host(st), pos0 + T), st_ref)


@pytest.mark.parametrize("act,D,nb", [("f32", 64, 2), ("bf16", 64, 2),
                                      ("bf16", 512, 2),    # fused kernel
                                      ("bf16", 320, 2),    # fused kernel, narrower blocks in the padded tile
                                      ("bf16", 256, 4)])   # separate passes (blocks of 64 channels)
def test_forward_in_pieces_equals_one_shot_and_states_may_alias(act, D, nb):
    rn = runner()
    B, T = 2, 45
    inp = gen.make_inputs(B, T, D, nb, act=act, seed=77, h0=True)
    dp = rn.DeviceProblem(inp, B, T, D, nb, act)
    u = rn.to_device(inp["u"], act)
    y_ref, hT_ref, st_ref = oracle_forward(inp, h0=inp["h0"])
    h = rn.to_device(inp["h0"], "f32")
    state = None
    import paper_2402_19427_amd as R
    ys = []
    pos = 0
    for T1 in (1, 2, 13, 29):   # pieces shorter than the filter, then longer ones
        piece = u[:, pos:pos + T1].contiguous()
        sh = dp.shape(T=T1)
        ws, n = dp.workspace(sh, R.OP_FORWARD)
        y = dp.empty_act(B, T1, D)
        st_out = state if state is not None else dp.empty_act(B, 3, D)
        R.rglru_forward(sh, dp.params, piece, h, state, pos, y, h, st_out, ws, n)  # in place
        state = st_out
        ys.append(rn.to_host(y))
        pos += T1
    assert pos == T
    assert gen.rel_err(np.concatenate(ys, axis=1), y_ref) < TOL[act]
    assert gen.rel_err(rn.to_host(h), hT_ref) < TOL[act]
    np.testing.assert_array_equal(gen.chrono_from_ring(rn.to_host(state), T), st_ref)


def test_a_long_prompt_in_windows_equals_the_capped_call_and_carries_states_in_place():
    """A single long sequence runs as contiguous windows in two passes. The same call with the
    time slices capped at one (a single workgroup per unit walks the sequence) must agree to
    rounding; the call continues from a carried state and Conv1D ring, which may be given in place."""
    import paper_2402_19427_amd as R
    rn = runner()
    B, T, D, nb, act = 1, 12700, 512, 2, "bf16"
    inp = gen.make_inputs(B, T, D, nb, act=act, seed=31, h0=True, state=True, bias=True)
    dp = rn.DeviceProblem(inp, B, T, D, nb, act)
    u = rn.to_device(inp["u"], act)
    pos0 = 4
    ring = rn.to_device(gen.ring_from_chrono(inp["state"], pos0), act)
    h0 = rn.to_device(inp["h0"], "f32")
    y, hT, st = dp.forward(u, h0=h0, state_in=ring, pos0=pos0)
    R.rglru_set_max_time_slices(1)
    try:
        y1, hT1, st1 = dp.forward(u, h0=h0, state_in=ring, pos0=pos0)
    finally:
        R.rglru_set_max_time_slices(0)
    assert gen.rel_err(rn.to_host(y), rn.to_host(y1)) < 1e-2      # (bf16 steps of y here and there)
    assert gen.rel_err(rn.to_host(hT), rn.to_host(hT1)) < 1e-5
    assert torch_equal(st, st1)
    # states in place
    sh = dp.shape()
    ws, n = dp.workspace(sh, R.OP_FORWARD)
    h_io, ring_io, y2 = h0.clone(), ring.clone(), dp.empty_act(B, T, D)
    R.rglru_forward(sh, dp.params, u, h_io, ring_io, pos0, y2, h_io, ring_io, ws, n)
    assert torch_equal(h_io, hT) and torch_equal(ring_io, st) and torch_equal(y2, y)
    y_ref, hT_ref, st_ref = oracle_forward(inp, h0=inp["h0"], state=inp["state"])
    assert gen.rel_err(rn.to_host(y), y_ref) < TOL[act]
    assert gen.rel_err(rn.to_host(hT), hT_ref) < TOL[act]


def torch_equal(a, b):
    import torch
    return bool(torch.equal(a, b))


def test_forward_zero_length_passes_states_through():
    rn = runner()
    B, D, nb = 2, 32, 2
    inp = gen.make_inputs(B, 4, D, nb, act="bf16", seed=5, h0=True, state=True)
    dp = rn.DeviceProblem(inp, B, 0, D, nb, "bf16")
    u = dp.empty_act(B, 0, D)
    ring = rn.to_device(gen.ring_from_chrono(inp["state"], 7), "bf16")
    y, hT, st = dp.forward(u, h0=rn.to_device(inp["h0"], "f32"), state_in=ring, pos0=7)
    np.testing.assert_array_equal(rn.to_host(hT), inp["h0"])
    np.testing.assert_array_equal(rn.to_host(st), rn.to_host(ring))


@pytest.mark.parametrize("B,T,D,act", [(2, 50, 96, "f32"), (3, 2, 40, "bf16"), (1, 700, 512, "bf16")])
@pytest.mark.parametrize("full", [False, True])
def test_conv1d_matches_oracle(B, T, D, act, full):
    rn = runner()
    inp = gen.make_inputs(B, T, D, 1, act=act, seed=T + D, state=full, bias=full)
    pos0 = 4 if full else 0
    dp = rn.DeviceProblem(inp, B, T, D, 1, act)
    ring = rn.to_device(gen.ring_from_chrono(inp["state"], pos0), act) if full else None
    x, st = dp.conv1d(rn.to_device(inp["u"], act), state_in=ring, pos0=pos0)
    q = f64(inp)
    x_ref, st_ref = oracle.conv1d(q["u"], q["conv_w"], conv_b=q.get("conv_b"),
                                  state_in=q["state"], want_state=True)
    assert gen.rel_err(rn.to_host(x), x_ref) < (1e-6 if act == "f32" else 5e-3)
    np.testing.assert_array_equal(gen.chrono_from_ring(rn.to_host(st), pos0 + T), st_ref)


@pytest.mark.parametrize("B,D,nb,act", [(5, 64, 2, "f32"), (19, 512, 2, "bf16"), (3, 320, 2, "bf16"),
                                        (64, 1024, 4, "bf16"), (33, 256, 1, "bf16"),
                                        (37, 1024, 2, "bf16"),    # bs = 512: two chunks of input channels
                                        (5, 704, 2, "bf16"),      # bs = 352: a partial second chunk
                                        (70, 1536, 2, "bf16"),    # bs = 768: three chunks
                                        (3, 256, 4, "bf16")])     # bs = 64: one partial chunk
def test_decode_steps_match_oracle_and_wrap_the_ring(B, D, nb, act):
    rn = runner()
    nsteps = 7
    inp = gen.make_inputs(B, 1, D, nb, act=act, seed=B + D, h0=True, state=True,
                          decode_tokens=nsteps, bias=True)
    dp = rn.DeviceProblem(inp, B, 1, D, nb, act)
    pos = 11
    h = rn.to_device(inp["h0"], "f32")
    ring = rn.to_device(gen.ring_from_chrono(inp["state"], pos), act)
    q = f64(inp)
    h_ref, st_ref = q["h0"].copy(), q["state"].copy()
    for s in range(nsteps):
        y = dp.decode_step(rn.to_device(inp["u_dec"][s], act), h, ring, pos + s)
        y_ref = oracle.decode_step(q["u_dec"][s], q["W_a"], q["W_x"], q["b_a"], q["b_x"],
                                   q["Lambda"], q["conv_w"], h_ref, st_ref, conv_b=q["conv_b"])
        assert gen.rel_err(rn.to_host(y), y_ref) < TOL[act], s
        assert gen.rel_err(rn.to_host(h), h_ref) < TOL[act], s
        np.testing.assert_array_equal(gen.chrono_from_ring(rn.to_host(ring), pos + s + 1), st_ref)


@pytest.mark.parametrize("B,D,nb,act", [(5, 64, 2, "f32"), (19, 512, 2, "bf16"), (3, 320, 2, "bf16"),
                                        (37, 1024, 2, "bf16"), (5, 704, 2, "bf16"), (40, 600, 2, "bf16")])
def test_decode_steps_with_a_position_per_sequence(B, D, nb, act):
    """Sequences of one batch at different lengths: every row's ring follows its own position,
    the arithmetic is that of the ordinary step (tuned, chunked and generic kernels)."""
    import torch
    rn = runner()
    nsteps = 5
    inp = gen.make_inputs(B, 1, D, nb, act=act, seed=B + D + 2, h0=True, state=True,
                          decode_tokens=nsteps, bias=True)
    dp = rn.DeviceProblem(inp, B, 1, D, nb, act)
    pos = np.array([3 + (5 * b) % 11 + 1000003 * (b % 3) for b in range(B)], dtype=np.int64)
    h = rn.to_device(inp["h0"], "f32")
    ring_host = np.stack([gen.ring_from_chrono(inp["state"][b:b + 1], int(pos[b]))[0] for b in range(B)])
    ring = rn.to_device(ring_host, act)
    q = f64(inp)
    h_ref, st_ref = q["h0"].copy(), q["state"].copy()
    for s in range(nsteps):
        pos_dev = torch.from_numpy(pos + s).cuda()
        y = dp.decode_step_at(rn.to_device(inp["u_dec"][s], act), h, ring, pos_dev)
        y_ref = oracle.decode_step(q["u_dec"][s], q["W_a"], q["W_x"], q["b_a"], q["b_x"],
                                   q["Lambda"], q["conv_w"], h_ref, st_ref, conv_b=q["conv_b"])
        assert gen.rel_err(rn.to_host(y), y_ref) < TOL[act], s
        assert gen.rel_err(rn.to_host(h), h_ref) < TOL[act], s
        got = rn.to_host(ring)
        for b in range(B):
            np.testing.assert_array_equal(gen.chrono_from_ring(got[b:b + 1], int(pos[b]) + s + 1)[0], st_ref[b])


def test_decode_with_equal_positions_is_the_ordinary_step():
    import torch
    rn = runner()
    B, D, nb, act = 33, 2560, 10, "bf16"
    inp = gen.make_inputs(B, 1, D, nb, act=act, seed=77, h0=True, state=True, decode_tokens=1)
    dp = rn.DeviceProblem(inp, B, 1, D, nb, act)
    u = rn.to_device(inp["u_dec"][0], act)
    res = []
    for per_seq in (False, True):
        h = rn.to_device(inp["h0"], "f32")
        ring = rn.to_device(gen.ring_from_chrono(inp["state"], 10), act)
        y = (dp.decode_step_at(u, h, ring, torch.full((B,), 10, dtype=torch.int64, device="cuda"))
             if per_seq else dp.decode_step(u, h, ring, 10))
        res.append([rn.to_host(t) for t in (y, h, ring)])
    for a, b in zip(*res):
        np.testing.assert_array_equal(a, b)


def test_decode_continues_a_forward_call():
    rn = runner()
    B, T, D, nb, act = 4, 21, 512, 2, "bf16"
    inp = gen.make_inputs(B, T + 1, D, nb, act=act, seed=9)
    dp = rn.DeviceProblem(inp, B, T, D, nb, act)
    u = rn.to_device(inp["u"], act)
    _, hT, st = dp.forward(u[:, :T].contiguous())
    y_last = dp.decode_step(u[:, T].contiguous(), hT, st, T)
    y_ref, hT_ref, _ = oracle_forward(inp)
    assert gen.rel_err(rn.to_host(y_last), y_ref[:, T]) < TOL[act]
    assert gen.rel_err(rn.to_host(hT), hT_ref) < TOL[act]


BWD_SHAPES = [
    (2, 19, 64, 2, "f32"),
    (1, 256, 256, 4, "f32"),
    (3, 3, 40, 5, "f32"),
    (2, 1, 16, 1, "f32"),
    (2, 75, 512, 2, "bf16"),
    (2, 33, 320, 2, "bf16"),      # bs = 160: the problem is widened to 256-channel blocks
    (3, 300, 2560, 16, "bf16"),   # the same at the paper's width, 16 blocks
    (1, 1100, 384, 2, "bf16"),    # bs = 192, long sequence in time slices
    (2, 100, 2816, 8, "bf16"),    # bs = 352: pointwise part in passes, contractions on the generic kernels
    (1, 700, 1024, 2, "bf16"),    # bs = 512, adjoint scan in time slices
    (3, 70, 256, 4, "bf16"),      # bs = 64
    (4, 1, 1024, 2, "bf16"),      # bs = 512, a single step
    (1, 24, 512, 8, "bf16"),      # bs = 64, B T a multiple of 8 but smaller than a tile
    (1, 270, 600, 2, "bf16"),
    (1, 1, 256, 1, "bf16"),       # MFMA path, single step
    (2, 31, 256, 1, "bf16"),      # MFMA path, one partial tile
    (1, 700, 256, 1, "bf16"),     # MFMA path, one unit in 16 time slices
    (1, 13000, 256, 1, "bf16"),   # ... over a long sequence: 26 rounds of the slices, the record rings wrap (forward: windows)
    (33, 70, 1024, 4, "bf16"),    # MFMA path, 132 units, no slicing
    (8, 300, 2048, 8, "bf16"),    # MFMA path, 64 units x 4 slices
]


@pytest.mark.parametrize("B,T,D,nb,act", BWD_SHAPES)
@pytest.mark.parametrize("full", [False, True])
def test_backward_matches_oracle(B, T, D, nb, act, full):
    rn = runner()
    inp = gen.make_inputs(B, T, D, nb, act=act, seed=31 * B + T + D, h0=full, state=full,
                          bias=full, dy=True)
    pos0 = 2 if full else 0
    dp = rn.DeviceProblem(inp, B, T, D, nb, act)
    u = rn.to_device(inp["u"], act)
    h0 = rn.to_device(inp["h0"], "f32")
    ring = rn.to_device(gen.ring_from_chrono(inp["state"], pos0), act) if full else None
    dhT = rn.to_device(inp["dhT"], "f32") if full else None
    y, _, _ = dp.forward(u, h0=h0, state_in=ring, pos0=pos0, want_state=False)
    out = dp.backward(u, y, rn.to_device(inp["dy"], act), h0=h0, state_in=ring, pos0=pos0,
                      dhT=dhT)
    q = f64(inp)
    oracle.set_threads(8 if q["u"].size > (1 << 20) else 1)
    ref = oracle.backward(q["u"], q["W_a"], q["W_x"], q["b_a"], q["b_x"], q["Lambda"],
                          q["conv_w"], q["dy"], conv_b=q.get("conv_b"), h0=q["h0"],
                          state_in=q["state"], dhT=q["dhT"] if full else None)
    for k in ("du", "dh0", "dW_a", "dW_x", "db_a", "db_x", "dLambda", "dconv_w", "dconv_b"):
        err = gen.rel_err(rn.to_host(out[k]), ref[k])
        assert err < GRAD_TOL[act], (k, err)


def test_backward_optional_outputs_can_be_skipped():
    rn = runner()
    import paper_2402_19427_amd as R
    B, T, D, nb, act = 2, 12, 32, 2, "f32"
    inp = gen.make_inputs(B, T, D, nb, act=act, seed=3, dy=True)
    dp = rn.DeviceProblem(inp, B, T, D, nb, act)
    u = rn.to_device(inp["u"], act)
    y, _, _ = dp.forward(u, want_state=False)
    full = dp.backward(u, y, rn.to_device(inp["dy"], act))
    g = dp.alloc_grads()
    pg = R.make_param_grads(g["dW_a"], g["dW_x"], g["db_a"], g["db_x"], g["dLambda"],
                            g["dconv_w"], None)
    sh = dp.shape()
    ws, n = dp.workspace(sh, R.OP_BACKWARD)
    du = dp.empty_act(B, T, D)
    R.rglru_backward(sh, dp.params, u, None, None, 0, y, rn.to_device(inp["dy"], act), None, du,
                     None, pg, ws, n)
    np.testing.assert_array_equal(rn.to_host(du), rn.to_host(full["du"]))
    np.testing.assert_array_equal(rn.to_host(g["dW_a"]), rn.to_host(full["dW_a"]))


@pytest.mark.parametrize("B,T,D,nb", [(2, 200, 512, 2),       # fused kernels
                                      (2, 200, 2560, 16),     # narrower blocks: padded tile, widened copy
                                      (2, 200, 1024, 2),      # 512-channel blocks: passes
                                      (10, 300, 2048, 8)])    # fused kernels with time slices
def test_results_are_deterministic_run_to_run(B, T, D, nb):
    rn = runner()
    act = "bf16"
    inp = gen.make_inputs(B, T, D, nb, act=act, seed=8, h0=True, dy=True)
    dp = rn.DeviceProblem(inp, B, T, D, nb, act)
    u = rn.to_device(inp["u"], act)
    h0 = rn.to_device(inp["h0"], "f32")
    outs = []
    for _ in range(3):
        y, hT, _ = dp.forward(u, h0=h0)
        g = dp.backward(u, y, rn.to_device(inp["dy"], act), h0=h0)
        outs.append((rn.to_host(y), rn.to_host(hT), rn.to_host(g["du"]), rn.to_host(g["dW_a"]),
                     rn.to_host(g["dW_x"]), rn.to_host(g["dLambda"]), rn.to_host(g["dconv_w"])))
    for o in outs[1:]:
        for a, b in zip(outs[0], o):
            np.testing.assert_array_equal(a, b)


def test_whole_step_replays_as_a_hip_graph():
    """forward + decode step + backward captured into one HIP graph (the library launches fill
    kernels, never memsets, and allocates nothing): every replay, with eager work and
    synchronisations in between, gives the bits of the eager run."""
    import torch
    import paper_2402_19427_amd as R
    rn = runner()
    B, T, D, nb, act = 8, 300, 2048, 8, "bf16"   # 64 units x 4 time slices: records cross workgroups
    inp = gen.make_inputs(B, T + 1, D, nb, act=act, seed=21, dy=True)
    dp = rn.DeviceProblem(inp, B, T, D, nb, act)
    u_all = rn.to_device(inp["u"], act)
    u, u_next = u_all[:, :T].contiguous(), u_all[:, T].contiguous()
    dy = rn.to_device(inp["dy"][:, :T], act)
    sh, sh1 = dp.shape(), dp.shape(T=1)
    ws_f, n_f = dp.workspace(sh, R.OP_FORWARD)
    ws_b, n_b = dp.workspace(sh, R.OP_BACKWARD)
    y, hT, st = dp.empty_act(B, T, D), dp.empty_f32(B, D), dp.empty_act(B, 3, D)
    y1, du, dh0 = dp.empty_act(B, D), dp.empty_act(B, T, D), dp.empty_f32(B, D)
    g = dp.alloc_grads()
    pg = R.make_param_grads(g["dW_a"], g["dW_x"], g["db_a"], g["db_x"], g["dLambda"],
                            g["dconv_w"], g["dconv_b"])
    outs = dict(y=y, hT=hT, st=st, y1=y1, du=du, dh0=dh0, **g)

    def step(stream):
        R.rglru_forward(sh, dp.params, u, None, None, 0, y, hT, st, ws_f, n_f, stream)
        R.rglru_backward(sh, dp.params, u, None, None, 0, y, dy, None, du, dh0, pg, ws_b, n_b, stream)
        R.rglru_decode_step(sh1, dp.params, u_next, hT, st, T, y1, stream)   # updates hT, st in place

    step(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    eager = {k: v.clone() for k, v in outs.items()}
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(torch.cuda.current_stream().cuda_stream)   # the capturing stream
    for rep in range(3):
        for v in outs.values():
            v.fill_(7.0)                                 # eager work between the replays
        ws_f.fill_(rep + 1)                              # stale records must not matter
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k, v in outs.items():
            assert torch.equal(v, eager[k]), (rep, k)


def test_long_prompt_forward_replays_as_a_hip_graph():
    """The windows of a single long prompt (ring pass, aggregate pass, chain, forward proper) captured
    into a HIP graph: every replay gives the bits of the eager run, whatever the workspace held."""
    import torch
    import paper_2402_19427_amd as R
    rn = runner()
    B, T, D, nb, act = 1, 12500, 256, 1, "bf16"
    inp = gen.make_inputs(B, T, D, nb, act=act, seed=23, h0=True)
    dp = rn.DeviceProblem(inp, B, T, D, nb, act)
    u, h0 = rn.to_device(inp["u"], act), rn.to_device(inp["h0"], "f32")
    sh = dp.shape()
    ws, n = dp.workspace(sh, R.OP_FORWARD)
    y, hT, st = dp.empty_act(B, T, D), dp.empty_f32(B, D), dp.empty_act(B, 3, D)
    outs = dict(y=y, hT=hT, st=st)

    def step(stream):
        R.rglru_forward(sh, dp.params, u, h0, None, 0, y, hT, st, ws, n, stream)

    step(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    eager = {k: v.clone() for k, v in outs.items()}
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(torch.cuda.current_stream().cuda_stream)
    for rep in range(3):
        for v in outs.values():
            v.fill_(7.0)
        ws.fill_(rep + 1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k, v in outs.items():
            assert torch.equal(v, eager[k]), (rep, k)


@pytest.mark.parametrize("D,nb", [(2560, 16),     # 160-channel blocks: padded tile, backward on the widened copy
                                  (1024, 2)])      # 512-channel blocks: forward and decode as separate kernels
def test_merge_step_replays_as_a_hip_graph(D, nb):
    """forward + merge, backward + merge and a decode step + merge captured into one HIP graph on
    the paths of the other block sizes: every replay gives the bits of the eager run."""
    import torch
    import paper_2402_19427_amd as R
    rn = runner()
    B, T, act = 3, 200, "bf16"
    inp = gen.make_inputs(B, T + 1, D, nb, act=act, seed=22, dy=True)
    dp = rn.DeviceProblem(inp, B, T, D, nb, act)
    u_all = rn.to_device(inp["u"], act)
    u, u_next = u_all[:, :T].contiguous(), u_all[:, T].contiguous()
    br_all = rn.to_device(gen.make_branch(B, T + 1, D, act=act, seed=23), act)
    br, br_next = br_all[:, :T].contiguous(), br_all[:, T].contiguous()
    dout = rn.to_device(inp["dy"][:, :T], act)
    sh, sh1 = dp.shape(), dp.shape(T=1)
    ws_f, n_f = dp.workspace(sh, R.OP_FORWARD_MERGE)
    ws_b, n_b = dp.workspace(sh, R.OP_BACKWARD_MERGE)
    out, y, hT, st = dp.empty_act(B, T, D), dp.empty_act(B, T, D), dp.empty_f32(B, D), dp.empty_act(B, 3, D)
    o1, du, dbr, dh0 = dp.empty_act(B, D), dp.empty_act(B, T, D), dp.empty_act(B, T, D), dp.empty_f32(B, D)
    g = dp.alloc_grads()
    pg = R.make_param_grads(g["dW_a"], g["dW_x"], g["db_a"], g["db_x"], g["dLambda"],
                            g["dconv_w"], g["dconv_b"])
    outs = dict(out=out, y=y, hT=hT, st=st, o1=o1, du=du, dbr=dbr, dh0=dh0, **g)

    def step(stream):
        R.rglru_forward_merge(sh, dp.params, u, br, None, None, 0, 0, out, y, hT, st, ws_f, n_f, stream)
        R.rglru_backward_merge(sh, dp.params, u, br, None, None, 0, 0, y, dout, None, du, dbr, dh0, pg,
                               ws_b, n_b, stream)
        R.rglru_decode_step_merge(sh1, dp.params, u_next, br_next, hT, st, T, 0, o1, stream)

    step(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    eager = {k: v.clone() for k, v in outs.items()}
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(torch.cuda.current_stream().cuda_stream)
    for rep in range(3):
        for v in outs.values():
            v.fill_(7.0)
        ws_f.fill_(rep + 1)
        ws_b.fill_(rep + 1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k, v in outs.items():
            assert torch.equal(v, eager[k]), (rep, k)


SCAN_SHAPES = [
    # B, T, D, act
    (2, 37, 96, "f32"),          # generic kernel, ragged everything
    (1, 1, 8, "f32"),
    (3, 50, 40, "bf16"),         # generic kernel: width not a multiple of 256
    (2, 100, 256, "bf16"),       # tiled kernel, ragged last tile
    (1, 1, 256, "bf16"),
    (1, 3000, 256, "bf16"),      # one unit in 16 time slices
    (8, 1024, 1024, "bf16"),     # the shape the paper times (Appendix A.3), shortest length
    (40, 70, 2048, "bf16"),      # 320 units: no time slices
]


@pytest.mark.parametrize("B,T,D,act", SCAN_SHAPES)
@pytest.mark.parametrize("log_a,scale", [(False, True), (True, True), (False, False)])
def test_scan_matches_oracle(B, T, D, act, log_a, scale):
    import paper_2402_19427_amd as R
    rn = runner()
    inp = gen.make_scan_inputs(B, T, D, act=act, seed=B + T + D, log_a=log_a)
    flags = (R.SCAN_LOG_A if log_a else 0) | (0 if scale else R.SCAN_NO_INPUT_SCALE)
    h, hT = rn.scan(rn.to_device(inp["a"], act), rn.to_device(inp["g"], act),
                    rn.to_device(inp["h0"], "f32"), flags=flags, act=act)
    oracle.set_threads(1)
    h_ref, hT_ref = oracle.scan(inp["a"], inp["g"], inp["h0"], a_is_log=log_a, normalize=scale)
    assert gen.rel_err(rn.to_host(h), h_ref) < TOL[act]
    assert gen.rel_err(rn.to_host(hT), hT_ref) < (1e-5 if act == "f32" else 1e-4)   # hT is fp32


@pytest.mark.parametrize("B,T,D,act", SCAN_SHAPES)
@pytest.mark.parametrize("log_a", [False, True])
def test_scan_adjoint_matches_oracle(B, T, D, act, log_a):
    import paper_2402_19427_amd as R
    rn = runner()
    inp = gen.make_scan_inputs(B, T, D, act=act, seed=2 * B + T + D, log_a=log_a)
    flags = R.SCAN_ADJOINT | R.SCAN_NO_INPUT_SCALE | (R.SCAN_LOG_A if log_a else 0)
    delta, dh0 = rn.scan(rn.to_device(inp["a"], act), rn.to_device(inp["g"], act),
                         rn.to_device(inp["h0"], "f32"), flags=flags, act=act)
    oracle.set_threads(1)
    d_ref, dh0_ref = oracle.scan_adjoint(inp["a"], inp["g"], inp["h0"], a_is_log=log_a)
    assert gen.rel_err(rn.to_host(delta), d_ref) < TOL[act]
    assert gen.rel_err(rn.to_host(dh0), dh0_ref) < TOL[act]


def test_scan_without_h0_and_without_hT_and_empty():
    import torch
    import paper_2402_19427_amd as R
    rn = runner()
    inp = gen.make_scan_inputs(2, 45, 512, act="bf16", seed=3, h0=False)
    a, g = rn.to_device(inp["a"], "bf16"), rn.to_device(inp["g"], "bf16")
    h, hT = rn.scan(a, g, None)
    h_ref, hT_ref = oracle.scan(inp["a"], inp["g"], None)
    assert gen.rel_err(rn.to_host(h), h_ref) < TOL["bf16"]
    sh = R.make_shape(2, 45, 512, 1, R.BF16)
    n = R.rglru_workspace_bytes(sh, R.OP_SCAN)
    ws = torch.empty(max(n, 256), dtype=torch.uint8, device="cuda:0")
    h2 = torch.empty_like(a)
    R.rglru_scan(sh, a, g, None, 0, h2, None, ws, n)        # no hT asked for
    assert torch.equal(h2, h)
    # T == 0: the state passes through
    h0 = torch.randn(2, 512, device="cuda:0")
    hT0 = torch.empty_like(h0)
    R.rglru_scan(R.make_shape(2, 0, 512, 1, R.BF16), None, None, h0, 0, None, hT0, None, 0)
    assert torch.equal(hT0, h0)


def test_workspace_status_reports_an_expired_wait():
    """After sliced calls the health check is clean; a flag planted from the host (no kernel
    misbehaves for this) is reported as a timeout."""
    import torch
    import paper_2402_19427_amd as R
    rn = runner()
    B, T, D, nb = 1, 700, 256, 1          # one unit in 16 time slices: records cross workgroups
    inp = gen.make_inputs(B, T, D, nb, act="bf16", seed=4, dy=True)
    dp = rn.DeviceProblem(inp, B, T, D, nb, "bf16")
    u, dy = rn.to_device(inp["u"], "bf16"), rn.to_device(inp["dy"], "bf16")
    y, _, _ = dp.forward(u)
    dp.backward(u, y, dy)
    sh = dp.shape()
    for op in (R.OP_FORWARD, R.OP_BACKWARD):
        ws, n = dp.workspace(sh, op)
        assert n > 0
        R.rglru_workspace_status(sh, op, ws)          # raises on a timeout
    # scan
    si = gen.make_scan_inputs(1, 3000, 256, act="bf16", seed=1)
    a, g = rn.to_device(si["a"], "bf16"), rn.to_device(si["g"], "bf16")
    ssh = R.make_shape(1, 3000, 256, 1, R.BF16)
    n = R.rglru_workspace_bytes(ssh, R.OP_SCAN)
    ws = torch.empty(n, dtype=torch.uint8, device="cuda:0")
    h = torch.empty_like(a)
    R.rglru_scan(ssh, a, g, None, 0, h, None, ws, n)
    R.rglru_workspace_status(ssh, R.OP_SCAN, ws)
    ws[:4] = torch.tensor([1, 0, 0, 0], dtype=torch.uint8, device="cuda:0")   # plant the flag
    with pytest.raises(R.RglruError) as e:
        R.rglru_workspace_status(ssh, R.OP_SCAN, ws)
    assert e.value.code == R.ERR_TIMEOUT
    # shapes that need no workspace have nothing to report
    R.rglru_workspace_status(R.make_shape(40, 70, 2048, 8, R.F32), R.OP_FORWARD, None)


# ------------------------------------------------------------------ the block's merge as epilogue
MERGE_SHAPES = [
    (2, 37, 96, 3, "f32"),       # generic kernels, ragged T
    (1, 9, 24, 24, "bf16"),      # generic kernels, element count not a multiple of 8... (216)
    (3, 5, 40, 5, "f32"),
    (2, 130, 512, 2, "bf16"),    # MFMA path, ragged T
    (33, 70, 1024, 4, "bf16"),   # MFMA path, one workgroup per unit
    (8, 600, 2048, 8, "bf16"),   # MFMA path, time slices
    (1, 1500, 256, 1, "bf16"),   # MFMA path, 16 time slices: the merge runs as a kernel of its own
    (1, 12500, 256, 1, "bf16"),  # MFMA path, contiguous windows in two passes, merge as epilogue of the second
    (3, 300, 2560, 16, "bf16"),  # bs = 160 in the padded tile, merge as epilogue
    (2, 100, 2816, 8, "bf16"),   # bs = 352: separate passes, then the merge kernel
]


@pytest.mark.parametrize("B,T,D,nb,act", MERGE_SHAPES)
@pytest.mark.parametrize("tanh_form", [False, True])
@pytest.mark.parametrize("keep_y", [False, True])
def test_forward_merge_matches_oracle(B, T, D, nb, act, tanh_form, keep_y):
    import paper_2402_19427_amd as R
    rn = runner()
    inp = gen.make_inputs(B, T, D, nb, act=act, seed=3 * B + T + D, h0=True, bias=True)
    br = gen.make_branch(B, T, D, act=act, seed=T)
    dp = rn.DeviceProblem(inp, B, T, D, nb, act)
    out, y, hT, st = dp.forward_merge(rn.to_device(inp["u"], act), rn.to_device(br, act),
                                      h0=rn.to_device(inp["h0"], "f32"),
                                      flags=R.MERGE_GELU_TANH if tanh_form else 0, keep_y=keep_y)
    q = f64(inp)
    out_ref, y_ref, hT_ref, st_ref = oracle.forward_merge(
        q["u"], br, q["W_a"], q["W_x"], q["b_a"], q["b_x"], q["Lambda"], q["conv_w"],
        conv_b=q.get("conv_b"), h0=q["h0"], approx=tanh_form)
    assert gen.rel_err(rn.to_host(out), out_ref) < TOL[act]
    assert gen.rel_err(rn.to_host(hT), hT_ref) < TOL[act]
    if keep_y:
        assert gen.rel_err(rn.to_host(y), y_ref) < TOL[act]
    np.testing.assert_array_equal(gen.chrono_from_ring(rn.to_host(st), T), st_ref)


@pytest.mark.parametrize("B,T,D,nb,act", [(2, 37, 96, 3, "f32"), (1, 9, 24, 24, "bf16"),
                                          (2, 130, 512, 2, "bf16"), (8, 600, 2048, 8, "bf16"),
                                          (3, 300, 2560, 16, "bf16"),   # widened copy behind the merge adjoint
                                          (2, 100, 2816, 8, "bf16")])   # backward in passes behind it
@pytest.mark.parametrize("tanh_form", [False, True])
def test_backward_merge_matches_oracle(B, T, D, nb, act, tanh_form):
    import paper_2402_19427_amd as R
    rn = runner()
    inp = gen.make_inputs(B, T, D, nb, act=act, seed=5 * B + T + D, h0=True, dy=True, bias=True)
    br = gen.make_branch(B, T, D, act=act, seed=T + 1)
    dp = rn.DeviceProblem(inp, B, T, D, nb, act)
    flags = R.MERGE_GELU_TANH if tanh_form else 0
    u, brd, h0 = rn.to_device(inp["u"], act), rn.to_device(br, act), rn.to_device(inp["h0"], "f32")
    out, y, hT, st = dp.forward_merge(u, brd, h0=h0, flags=flags)
    dhT = rn.to_device(inp["dhT"], "f32")
    g = dp.backward_merge(u, brd, y, rn.to_device(inp["dy"], act), h0=h0, dhT=dhT, flags=flags)
    q = f64(inp)
    # against the float64 adjoint of the whole composition, nothing rounded in between
    ref = oracle.backward_merge(q["u"], br, q["W_a"], q["W_x"], q["b_a"], q["b_x"], q["Lambda"], q["conv_w"],
                                q["dy"], conv_b=q.get("conv_b"), h0=q["h0"], dhT=q["dhT"], approx=tanh_form)
    for k in ("du", "dbranch", "dh0"):
        assert gen.rel_err(rn.to_host(g[k]), ref[k]) < TOL[act], k
    for k in ("dW_a", "dW_x", "db_a", "db_x", "dLambda", "dconv_w", "dconv_b"):
        assert gen.rel_err(rn.to_host(g[k]), ref[k]) < GRAD_TOL[act], k
    sh = dp.shape()
    ws, _ = dp.workspace(sh, R.OP_BACKWARD_MERGE)
    R.rglru_workspace_status(sh, R.OP_BACKWARD_MERGE, ws)


def test_forward_merge_zero_length_passes_states_through():
    import paper_2402_19427_amd as R
    rn = runner()
    B, D, nb = 2, 512, 2
    inp = gen.make_inputs(B, 4, D, nb, act="bf16", seed=5, h0=True, state=True)
    dp = rn.DeviceProblem(inp, B, 0, D, nb, "bf16")
    ring = rn.to_device(gen.ring_from_chrono(inp["state"], 7), "bf16")
    out, y, hT, st = dp.forward_merge(dp.empty_act(B, 0, D), dp.empty_act(B, 0, D),
                                      h0=rn.to_device(inp["h0"], "f32"), state_in=ring, pos0=7)
    np.testing.assert_array_equal(rn.to_host(hT), inp["h0"])
    np.testing.assert_array_equal(rn.to_host(st), rn.to_host(ring))
    assert out.numel() == 0


def test_merge_calls_reject_bad_arguments():
    import paper_2402_19427_amd as R
    rn = runner()
    B, T, D, nb = 1, 4, 32, 2
    inp = gen.make_inputs(B, T, D, nb, act="bf16", seed=1)
    dp = rn.DeviceProblem(inp, B, T, D, nb, "bf16")
    u = rn.to_device(inp["u"], "bf16")
    sh = dp.shape()
    ws, n = dp.workspace(sh, R.OP_FORWARD_MERGE)
    out = dp.empty_act(B, T, D)
    with pytest.raises(R.RglruError):       # out aliases branch
        R.rglru_forward_merge(sh, dp.params, u, out, None, None, 0, 0, out, None, None, None, ws, n)
    with pytest.raises(R.RglruError):       # unknown flag
        R.rglru_forward_merge(sh, dp.params, u, u, None, None, 0, 8, out, None, None, None, ws, n)
    with pytest.raises(R.RglruError):       # branch missing
        R.rglru_forward_merge(sh, dp.params, u, None, None, None, 0, 0, out, None, None, None, ws, n)


@pytest.mark.parametrize("B,D,nb,act", [(5, 64, 2, "f32"), (3, 320, 2, "bf16"), (64, 1024, 4, "bf16"),
                                        (33, 256, 1, "bf16"), (37, 1024, 2, "bf16"), (5, 704, 2, "bf16"),
                                        (1, 512, 2, "bf16")])
@pytest.mark.parametrize("tanh_form", [False, True])
def test_decode_steps_with_merge_match_oracle(B, D, nb, act, tanh_form):
    import paper_2402_19427_amd as R
    rn = runner()
    nsteps = 4
    inp = gen.make_inputs(B, 1, D, nb, act=act, seed=B + D + 1, h0=True, state=True,
                          decode_tokens=nsteps, bias=True)
    br = gen.make_branch(nsteps, B, D, act=act, seed=B)
    dp = rn.DeviceProblem(inp, B, 1, D, nb, act)
    pos = 8
    h = rn.to_device(inp["h0"], "f32")
    ring = rn.to_device(gen.ring_from_chrono(inp["state"], pos), act)
    q = f64(inp)
    h_ref, st_ref = q["h0"].copy(), q["state"].copy()
    for s in range(nsteps):
        out = dp.decode_step_merge(rn.to_device(inp["u_dec"][s], act), rn.to_device(br[s], act), h, ring,
                                   pos + s, flags=R.MERGE_GELU_TANH if tanh_form else 0)
        y_ref = oracle.decode_step(q["u_dec"][s], q["W_a"], q["W_x"], q["b_a"], q["b_x"],
                                   q["Lambda"], q["conv_w"], h_ref, st_ref, conv_b=q["conv_b"])
        out_ref = oracle.merge(y_ref, br[s], approx=tanh_form)
        assert gen.rel_err(rn.to_host(out), out_ref) < TOL[act], s
        assert gen.rel_err(rn.to_host(h), h_ref) < TOL[act], s
        np.testing.assert_array_equal(gen.chrono_from_ring(rn.to_host(ring), pos + s + 1), st_ref)


# ------------------------------------------------------------------ the layer without its Conv1D
@pytest.mark.parametrize("B,T,D,nb,act", [(2, 37, 96, 3, "f32"),      # generic kernels
                                          (2, 130, 512, 2, "bf16"),   # fused kernels
                                          (1, 1100, 256, 1, "bf16"),  # fused, 16 time slices
                                          (1, 12300, 256, 1, "bf16"), # fused, contiguous windows in two passes
                                          (2, 70, 320, 2, "bf16"),    # padded tile
                                          (1, 75, 1024, 2, "bf16")])  # passes of the wide blocks
def test_conv_width_zero_is_the_rglru_layer_alone(B, T, D, nb, act):
    """conv_width = 0: the input is already x_t (eqs. 1-4 of Section 2.4 without the Conv1D of
    Section 2.3). Forward, one decode step and the backward against the oracle's RG-LRU layer;
    conv parameters and states are not passed at all."""
    import paper_2402_19427_amd as R
    rn = runner()
    inp = gen.make_inputs(B, T + 1, D, nb, act=act, seed=3 * B + T + D, h0=True, dy=True, bias=True)
    dp = rn.DeviceProblem(inp, B, T, D, nb, act)
    q = f64(inp)
    x_all, x = q["u"], q["u"][:, :T]
    par = R.make_params(dp.W_a, dp.W_x, dp.b_a, dp.b_x, dp.Lambda, None, None)
    dt = R.BF16 if act == "bf16" else R.F32
    sh = R.make_shape(B, T, D, nb, dt, conv_width=0)
    u_dev = rn.to_device(inp["u"][:, :T], act)
    h0 = rn.to_device(inp["h0"], "f32")
    ws, n = dp.workspace(sh, R.OP_FORWARD)
    y, hT = dp.empty_act(B, T, D), dp.empty_f32(B, D)
    R.rglru_forward(sh, par, u_dev, h0, None, 0, y, hT, None, ws, n)
    y_ref, hT_ref = oracle.rglru(x_all, q["W_a"], q["W_x"], q["b_a"], q["b_x"], q["Lambda"], h0=q["h0"])
    assert gen.rel_err(rn.to_host(y), y_ref[:, :T]) < TOL[act]
    hT_mid, _ = oracle.rglru(x, q["W_a"], q["W_x"], q["b_a"], q["b_x"], q["Lambda"], h0=q["h0"])[1], None
    assert gen.rel_err(rn.to_host(hT), hT_mid) < TOL[act]
    # backward: the oracle's backward with the identity filter (1, 0, 0, 0) is the layer's own adjoint
    dy = rn.to_device(inp["dy"][:, :T], act)
    dhT = rn.to_device(inp["dhT"], "f32")
    wsb, nb_ = dp.workspace(sh, R.OP_BACKWARD)
    g = dp.alloc_grads()
    pg = R.make_param_grads(g["dW_a"], g["dW_x"], g["db_a"], g["db_x"], g["dLambda"], None, None)
    du, dh0 = dp.empty_act(B, T, D), dp.empty_f32(B, D)
    R.rglru_backward(sh, par, u_dev, h0, None, 0, y, dy, dhT, du, dh0, pg, wsb, nb_)
    ident = np.zeros((4, D)); ident[0] = 1.0
    ref = oracle.backward(x, q["W_a"], q["W_x"], q["b_a"], q["b_x"], q["Lambda"], ident, q["dy"][:, :T],
                          h0=q["h0"], dhT=q["dhT"])
    for k, got in (("du", du), ("dh0", dh0)):
        assert gen.rel_err(rn.to_host(got), ref[k]) < TOL[act], k
    for k in ("dW_a", "dW_x", "db_a", "db_x", "dLambda"):
        assert gen.rel_err(rn.to_host(g[k]), ref[k]) < GRAD_TOL[act], k
    R.rglru_workspace_status(sh, R.OP_BACKWARD, wsb)
    # one decode step continuing the sequences: no ring at all
    sh1 = R.make_shape(B, 1, D, nb, dt, conv_width=0)
    y1 = dp.empty_act(B, D)
    R.rglru_decode_step(sh1, par, rn.to_device(inp["u"][:, T], act), hT, None, T, y1)
    assert gen.rel_err(rn.to_host(y1), y_ref[:, T]) < TOL[act]
    assert gen.rel_err(rn.to_host(hT), hT_ref) < TOL[act]


def test_an_expired_wait_poisons_later_calls_until_it_is_reported():
    """The mark an expired wait leaves in a workspace (planted here from the host: no kernel
    misbehaves) makes the next calls on that workspace return NaN instead of plausible numbers;
    rglru_workspace_status reports it once and clears it; with the time slices capped at one
    nothing waits and the same results come out."""
    import struct
    import torch
    import paper_2402_19427_amd as R
    rn = runner()
    B, T, D, nb = 1, 700, 256, 1          # one unit in 16 time slices
    inp = gen.make_inputs(B, T, D, nb, act="bf16", seed=9, dy=True)
    dp = rn.DeviceProblem(inp, B, T, D, nb, "bf16")
    u, dy = rn.to_device(inp["u"], "bf16"), rn.to_device(inp["dy"], "bf16")
    sh = dp.shape()
    y_ok, hT_ok, _ = dp.forward(u)
    g_ok = dp.backward(u, y_ok, dy)
    torch.cuda.synchronize()
    mark = torch.tensor(list(struct.pack("<4I", 0x4c474c52, 0x58452d55, 0x45524950, 0xb3d3b3ad)),
                        dtype=torch.uint8, device="cuda:0")
    # forward
    ws, n = dp.workspace(sh, R.OP_FORWARD)
    ws[:16] = mark
    y_bad, hT_bad, _ = dp.forward(u)
    assert torch.isnan(y_bad.float()).all() and torch.isnan(hT_bad).all()
    with pytest.raises(R.RglruError) as e:
        R.rglru_workspace_status(sh, R.OP_FORWARD, ws)
    assert e.value.code == R.ERR_TIMEOUT
    R.rglru_workspace_status(sh, R.OP_FORWARD, ws)          # reported once, then clean
    y_again, _, _ = dp.forward(u)
    assert torch.equal(y_again, y_ok)
    # backward: the word sits in front of its record rings, inside the workspace
    wsb, nb_ = dp.workspace(sh, R.OP_BACKWARD)
    R.rglru_workspace_status(sh, R.OP_BACKWARD, wsb)
    # uninitialised scratch that merely looks non-zero is not the mark: results stay valid
    wsb.fill_(0x5a)
    g_fill = dp.backward(u, y_ok, dy)
    assert torch.equal(g_fill["du"], g_ok["du"])
    R.rglru_workspace_status(sh, R.OP_BACKWARD, wsb)
    # the retry that cannot time out: one workgroup per (sequence, block)
    R.rglru_set_max_time_slices(1)
    try:
        y_one, hT_one, _ = dp.forward(u)
        q = f64(inp)
        y_ref, _, _ = oracle.forward(q["u"], q["W_a"], q["W_x"], q["b_a"], q["b_x"], q["Lambda"], q["conv_w"])
        assert gen.rel_err(rn.to_host(y_one), y_ref) < TOL["bf16"]
        g_one = dp.backward(u, y_one, dy)
        assert gen.rel_err(rn.to_host(g_one["du"]), rn.to_host(g_ok["du"])) < 1e-2
    finally:
        R.rglru_set_max_time_slices(0)


# ------------------------------------------------- packed sequences (document boundaries)
PACKED = [
    # B, T, D, nb, act, mean document length
    (2, 37, 96, 3, "f32", 6),
    (3, 5, 40, 5, "f32", 2),
    (3, 300, 512, 2, "bf16", 40),
    (2, 130, 320, 2, "bf16", 16),
    (1, 700, 1024, 2, "bf16", 100),
    (4, 2, 64, 2, "bf16", 1),      # fewer steps than the filter is wide, a boundary at most steps
    (8, 600, 2048, 8, "bf16", 50),  # fused forward: 64 units x 4 time slices
    (1, 1500, 256, 1, "bf16", 200), # fused forward: 16 time slices, most tiles without a boundary
    (3, 300, 2560, 16, "bf16", 7),  # fused forward, blocks of 160 channels, a boundary in most tiles
    (33, 70, 1024, 4, "bf16", 30),  # fused forward, one workgroup per unit
    (2, 130, 512, 2, "bf16", 3),    # a boundary every few steps, ragged last tile
    (5, 70, 256, 1, "bf16", 8),     # tiles of the flattened rows straddle sequences (weight gradients)
    (16, 4096, 256, 1, "bf16", 300),  # long rows: 16 workgroups x 16 time slices
]


@pytest.mark.parametrize("B,T,D,nb,act,mean_len", PACKED)
def test_packed_forward_and_backward_match_oracle(B, T, D, nb, act, mean_len):
    import torch
    rn = runner()
    inp = gen.make_inputs(B, T, D, nb, act=act, seed=B * 100 + T + D + 1, h0=True, state=True,
                          bias=True, dy=True)
    reset = gen.make_resets(B, T, seed=T + D, mean_len=mean_len)
    pos0 = 4
    dp = rn.DeviceProblem(inp, B, T, D, nb, act)
    u, h0 = rn.to_device(inp["u"], act), rn.to_device(inp["h0"], "f32")
    ring = rn.to_device(gen.ring_from_chrono(inp["state"], pos0), act)
    rdev = torch.from_numpy(reset).cuda()
    y, hT, st = dp.forward_packed(u, rdev, h0=h0, state_in=ring, pos0=pos0)
    q = f64(inp)
    args = (q["u"], q["W_a"], q["W_x"], q["b_a"], q["b_x"], q["Lambda"], q["conv_w"])
    y_ref, hT_ref, st_ref = oracle.forward(*args, conv_b=q["conv_b"], h0=q["h0"],
                                           state_in=q["state"], reset=reset)
    assert gen.rel_err(rn.to_host(y), y_ref) < TOL[act]
    assert gen.rel_err(rn.to_host(hT), hT_ref) < TOL[act]
    np.testing.assert_array_equal(gen.chrono_from_ring(rn.to_host(st), pos0 + T), st_ref)
    g = dp.backward_packed(u, rdev, y, rn.to_device(inp["dy"], act), h0=h0, state_in=ring,
                           pos0=pos0, dhT=rn.to_device(inp["dhT"], "f32"))
    ref = oracle.backward(*args, q["dy"], conv_b=q["conv_b"], h0=q["h0"], state_in=q["state"],
                          dhT=q["dhT"], reset=reset)
    for k in ("du", "dh0"):
        assert gen.rel_err(rn.to_host(g[k]), ref[k]) < TOL[act], k
    for k in ("dW_a", "dW_x", "db_a", "db_x", "dLambda", "dconv_w", "dconv_b"):
        assert gen.rel_err(rn.to_host(g[k]), ref[k]) < GRAD_TOL[act], k
    # rows that start a document at step 0 take nothing from, and send nothing to, the states
    for b in range(B):
        if reset[b, 0]:
            np.testing.assert_array_equal(rn.to_host(g["dh0"])[b], np.zeros(D, np.float32))


def test_packed_calls_without_a_mask_are_the_plain_calls():
    rn = runner()
    B, T, D, nb, act = 2, 50, 96, 3, "f32"
    inp = gen.make_inputs(B, T, D, nb, act=act, seed=9, h0=True, dy=True)
    dp = rn.DeviceProblem(inp, B, T, D, nb, act)
    u, h0 = rn.to_device(inp["u"], act), rn.to_device(inp["h0"], "f32")
    y, hT, st = dp.forward(u, h0=h0)
    y2, hT2, st2 = dp.forward_packed(u, None, h0=h0)
    np.testing.assert_array_equal(rn.to_host(y), rn.to_host(y2))
    np.testing.assert_array_equal(rn.to_host(hT), rn.to_host(hT2))
    np.testing.assert_array_equal(rn.to_host(st), rn.to_host(st2))
    dy = rn.to_device(inp["dy"], act)
    g, g2 = dp.backward(u, y, dy, h0=h0), dp.backward_packed(u, None, y, dy, h0=h0)
    for k in g:
        np.testing.assert_array_equal(rn.to_host(g[k]), rn.to_host(g2[k]))


@pytest.mark.parametrize("B,T,D,nb,act", [(2, 37, 96, 3, "f32"), (3, 300, 512, 2, "bf16"), (8, 200, 2048, 8, "bf16")])
def test_packed_calls_without_the_conv1d(B, T, D, nb, act):
    """conv_width = 0 together with document boundaries: only the recurrence restarts (general
    kernels, fused kernels with and without time slices)."""
    import torch
    import paper_2402_19427_amd as R
    rn = runner()
    inp = gen.make_inputs(B, T, D, nb, act=act, seed=B + T + D + 7, h0=True, dy=True, bias=True)
    reset = gen.make_resets(B, T, seed=D, mean_len=20)
    dp = rn.DeviceProblem(inp, B, T, D, nb, act)
    par = R.make_params(dp.W_a, dp.W_x, dp.b_a, dp.b_x, dp.Lambda, None, None)
    sh = R.make_shape(B, T, D, nb, R.BF16 if act == "bf16" else R.F32, conv_width=0)
    u, h0, r_dev = rn.to_device(inp["u"], act), rn.to_device(inp["h0"], "f32"), torch.from_numpy(reset).cuda()
    ws, n = dp.workspace(sh, R.OP_FORWARD_PACKED)
    y, hT = dp.empty_act(B, T, D), dp.empty_f32(B, D)
    R.rglru_forward_packed(sh, par, u, r_dev, h0, None, 0, y, hT, None, ws, n)
    q = f64(inp)
    y_ref, hT_ref = oracle.rglru(q["u"], q["W_a"], q["W_x"], q["b_a"], q["b_x"], q["Lambda"], h0=q["h0"], reset=reset)
    assert gen.rel_err(rn.to_host(y), y_ref) < TOL[act]
    assert gen.rel_err(rn.to_host(hT), hT_ref) < TOL[act]
    wsb, nbytes = dp.workspace(sh, R.OP_BACKWARD_PACKED)
    g = dp.alloc_grads()
    pg = R.make_param_grads(g["dW_a"], g["dW_x"], g["db_a"], g["db_x"], g["dLambda"], None, None)
    du, dh0 = dp.empty_act(B, T, D), dp.empty_f32(B, D)
    R.rglru_backward_packed(sh, par, u, r_dev, h0, None, 0, y, rn.to_device(inp["dy"], act),
                            rn.to_device(inp["dhT"], "f32"), du, dh0, pg, wsb, nbytes)
    ident = np.zeros((4, D)); ident[0] = 1.0
    ref = oracle.backward(q["u"], q["W_a"], q["W_x"], q["b_a"], q["b_x"], q["Lambda"], ident, q["dy"],
                          h0=q["h0"], dhT=q["dhT"], reset=reset)
    for k, got in (("du", du), ("dh0", dh0)):
        assert gen.rel_err(rn.to_host(got), ref[k]) < TOL[act], k
    for k in ("dW_a", "dW_x", "db_a", "db_x", "dLambda"):
        assert gen.rel_err(rn.to_host(g[k]), ref[k]) < GRAD_TOL[act], k
