"""Parity at the full sizes of the five workloads, in the launch configuration bench.py times.

The oracle cannot run a whole workload in seconds, so outputs are checked on sampled
(sequence, gate block) pairs: the path is independent across sequences and across gate blocks
(depthwise Conv1D, block-diagonal gates, diagonal recurrence), so the oracle evaluates one pair
as a problem of its own (B = 1, nb = 1, D = bs) from the same inputs. Parameter gradients sum
over sequences, so for a sampled block every sequence is run through the oracle.
"""
import numpy as np
import pytest

import oracle
import rglru_inputs as gen

pytestmark = pytest.mark.gpu
TOL = 2e-2   # bf16 storage, fp32 state and accumulation


def block_params(inp, g, bs):
    sl = slice(g * bs, (g + 1) * bs)
    f = lambda a: np.asarray(a, np.float64)
    return sl, (f(inp["W_a"][g:g + 1]), f(inp["W_x"][g:g + 1]), f(inp["b_a"][sl]), f(inp["b_x"][sl]),
                f(inp["Lambda"][sl]), f(inp["conv_w"][:, sl]))


def run_forward_full(name, pairs):
    import paper_2402_19427_amd.runner as rn
    w = gen.CONFIGS[name]
    inp = gen.make_workload(name, dy=False)
    dp = rn.DeviceProblem(inp, w.B, w.T, w.D, w.nb, w.act)
    u = rn.to_device(inp["u"], w.act)
    h0 = rn.to_device(inp["h0"], "f32")
    y, hT, st = dp.forward(u, h0=h0)
    y_h, hT_h, st_h = rn.to_host(y), rn.to_host(hT), rn.to_host(st)
    del y, u
    oracle.set_threads(1)
    for b, g in pairs:
        sl, par = block_params(inp, g, w.bs)
        h0_u = None if inp["h0"] is None else np.asarray(inp["h0"][b:b + 1, sl], np.float64)
        y_ref, hT_ref, st_ref = oracle.forward(np.asarray(inp["u"][b:b + 1, :, sl], np.float64), *par,
                                               h0=h0_u)
        assert gen.rel_err(y_h[b:b + 1, :, sl], y_ref) < TOL, (name, b, g)
        assert gen.rel_err(hT_h[b:b + 1, sl], hT_ref) < TOL, (name, b, g)
        np.testing.assert_array_equal(gen.chrono_from_ring(st_h[b:b + 1, :, sl], w.T), st_ref)
    # a property that holds for every element: the outputs are finite
    assert np.isfinite(y_h).all() and np.isfinite(hT_h).all()


def test_c1_training_shaped_forward_full_size():
    run_forward_full("C1", [(0, 0), (3, 7), (7, 9)])


def test_c2_long_sequence_forward_full_size():
    # one sequence of 32768 steps with a random initial state: every tile boundary and every
    # time slice of the carry exchange lies on the path to the last outputs
    run_forward_full("C2", [(0, 0), (0, 9)])


def test_long_prompt_with_sixteen_blocks_forward_in_interleaved_slices():
    """One sequence of 16384 steps at width 4096 with 16 gate blocks: more units than the windows of
    a single prompt take, so all 256 compute units run it as 16 interleaved time slices per unit,
    32 rounds of them. Two of the blocks against the oracle, every output finite."""
    import paper_2402_19427_amd.runner as rn
    B, T, D, nb, act = 1, 16384, 4096, 16, "bf16"
    inp = gen.make_inputs(B, T, D, nb, act=act, seed=41, h0=True)
    dp = rn.DeviceProblem(inp, B, T, D, nb, act)
    y, hT, st = dp.forward(rn.to_device(inp["u"], act), h0=rn.to_device(inp["h0"], "f32"))
    y_h, hT_h = rn.to_host(y), rn.to_host(hT)
    oracle.set_threads(1)
    for g in (0, 11):
        sl, par = block_params(inp, g, D // nb)
        y_ref, hT_ref, _ = oracle.forward(np.asarray(inp["u"][:, :, sl], np.float64), *par,
                                          h0=np.asarray(inp["h0"][:, sl], np.float64))
        assert gen.rel_err(y_h[:, :, sl], y_ref) < TOL, g
        assert gen.rel_err(hT_h[:, sl], hT_ref) < TOL, g
    assert np.isfinite(y_h).all() and np.isfinite(hT_h).all()


def run_train_full(name, g, y_rows, decode=False):
    """forward (+ one decode step continuing it) + backward at the workload's full size; every
    sequence of gate block g goes through the oracle (parameter gradients sum over the batch)."""
    import paper_2402_19427_amd.runner as rn
    w = gen.CONFIGS[name]
    inp = gen.make_inputs(w.B, w.T + 1, w.D, w.nb, act=w.act, seed=w.seed, dy=True)
    T = w.T
    dp = rn.DeviceProblem(inp, w.B, T, w.D, w.nb, w.act)
    u_all = rn.to_device(inp["u"], w.act)
    u = u_all[:, :T].contiguous()
    dy = rn.to_device(inp["dy"][:, :T], w.act)
    y, hT, st = dp.forward(u)
    y1_h = hT1_h = None
    if decode:
        hT1 = hT.clone()
        y1_h = rn.to_host(dp.decode_step(u_all[:, T].contiguous(), hT1, st, T))
        hT1_h = rn.to_host(hT1)
    out = dp.backward(u, y, dy)
    y_h, du_h, dh0_h = rn.to_host(y), rn.to_host(out["du"]), rn.to_host(out["dh0"])
    small = {k: rn.to_host(out[k]) for k in ("dW_a", "dW_x", "db_a", "db_x", "dLambda", "dconv_w",
                                             "dconv_b")}
    del y, u, dy, out, u_all
    sl, par = block_params(inp, g, w.bs)
    acc = None
    oracle.set_threads(1)
    for b in range(w.B):
        ub = np.asarray(inp["u"][b:b + 1, :T, sl], np.float64)
        dyb = np.asarray(inp["dy"][b:b + 1, :T, sl], np.float64)
        ref = oracle.backward(ub, *par, dyb)
        if b in y_rows:
            y_ref, hT_ref, st_ref = oracle.forward(ub, *par)
            assert gen.rel_err(y_h[b:b + 1, :, sl], y_ref) < TOL, b
            if decode:
                y1_ref = oracle.decode_step(np.asarray(inp["u"][b:b + 1, T, sl], np.float64), *par,
                                            hT_ref, st_ref)
                assert gen.rel_err(y1_h[b:b + 1, sl], y1_ref) < TOL, b
                assert gen.rel_err(hT1_h[b:b + 1, sl], hT_ref) < TOL, b   # updated in place
        assert gen.rel_err(du_h[b:b + 1, :, sl], ref["du"]) < TOL, b
        assert gen.rel_err(dh0_h[b:b + 1, sl], ref["dh0"]) < TOL, b
        if acc is None:
            acc = {k: ref[k].copy() for k in small}
        else:
            for k in small:
                acc[k] += ref[k]
    assert gen.rel_err(small["dW_a"][g], acc["dW_a"][0]) < TOL
    assert gen.rel_err(small["dW_x"][g], acc["dW_x"][0]) < TOL
    for k in ("db_a", "db_x", "dLambda", "dconv_b"):
        assert gen.rel_err(small[k][sl], acc[k]) < TOL, k
    assert gen.rel_err(small["dconv_w"][:, sl], acc["dconv_w"]) < TOL
    assert np.isfinite(du_h).all() and all(np.isfinite(v).all() for v in small.values())


def test_c4_forward_and_backward_full_size():
    run_train_full("C4", 5, (0, 9))


def test_c1_whole_step_as_benchmarked():
    # the step bench.py times: forward, one decode step continuing it, backward (3 time slices
    # per (sequence, block) at this size)
    run_train_full("C1", 3, (0, 6), decode=True)


def test_c3_batched_decode_full_size():
    import paper_2402_19427_amd.runner as rn
    w = gen.CONFIGS["C3"]
    inp = gen.make_workload("C3")
    dp = rn.DeviceProblem(inp, w.B, 1, w.D, w.nb, w.act)
    pos0 = 4096
    h = rn.to_device(inp["h0"], "f32")
    ring = rn.to_device(gen.ring_from_chrono(inp["state"], pos0), w.act)
    toks = [rn.to_device(inp["u_dec"][i], w.act) for i in range(8)]
    blocks = (0, 11)
    refs = {}
    for g in blocks:
        sl, par = block_params(inp, g, w.bs)
        refs[g] = (sl, par, np.asarray(inp["h0"][:, sl], np.float64).copy(),
                   np.asarray(inp["state"][:, :, sl], np.float64).copy())
    for s in range(64):
        y = dp.decode_step(toks[s % 8], h, ring, pos0 + s)
        check = s < 4 or s == 63
        if check:
            y_h, h_h, ring_h = rn.to_host(y), rn.to_host(h), rn.to_host(ring)
        for g in blocks:
            sl, par, h_ref, st_ref = refs[g]
            y_ref = oracle.decode_step(np.asarray(inp["u_dec"][s % 8][:, sl], np.float64), *par,
                                       h_ref, st_ref)
            if check:
                assert gen.rel_err(y_h[:, sl], y_ref) < TOL, (s, g)
                assert gen.rel_err(h_h[:, sl], h_ref) < TOL, (s, g)
                np.testing.assert_array_equal(
                    gen.chrono_from_ring(ring_h[:, :, sl], pos0 + s + 1), st_ref)


def test_c0_tiny_fp32_full_size():
    import paper_2402_19427_amd.runner as rn
    w = gen.CONFIGS["C0"]
    inp = gen.make_workload("C0")
    dp = rn.DeviceProblem(inp, w.B, w.T, w.D, w.nb, w.act)
    y, hT, _ = dp.forward(rn.to_device(inp["u"], w.act))
    q = {k: (None if v is None else np.asarray(v, np.float64)) for k, v in inp.items()}
    y_ref, hT_ref, _ = oracle.forward(q["u"], q["W_a"], q["W_x"], q["b_a"], q["b_x"], q["Lambda"],
                                      q["conv_w"])
    assert gen.rel_err(rn.to_host(y), y_ref) < 1e-5
    assert gen.rel_err(rn.to_host(hT), hT_ref) < 1e-5


def test_scan_at_the_paper_s_measurement_shape_full_size():
    """rglru_scan at batch 8, width 1024, 65536 steps (the longest length of the timing sweep):
    channels are independent, so the oracle runs on a sample of them."""
    import torch
    import paper_2402_19427_amd as R
    import paper_2402_19427_amd.runner as rn
    B, T, D = 8, 65536, 1024
    rng = np.random.Generator(np.random.PCG64(77))
    base = rng.uniform(0.9, 0.999, size=D) ** 0.125
    la = (8.0 * rng.uniform(0.0, 1.0, size=(B, T, D)).astype(np.float32) * np.log(base).astype(np.float32))
    la = gen.round_to_act(la, "bf16")                       # log a_t as stored
    g = gen.round_to_act(rng.standard_normal((B, T, D), dtype=np.float32), "bf16")
    h0 = rng.standard_normal((B, D), dtype=np.float32)
    h, hT = rn.scan(rn.to_device(la, "bf16"), rn.to_device(g, "bf16"), rn.to_device(h0, "f32"),
                    flags=R.SCAN_LOG_A)
    h_h, hT_h = rn.to_host(h), rn.to_host(hT)
    del h
    torch.cuda.empty_cache()
    ch = np.arange(5, D, 37)                                 # 28 channels across all four groups
    h_ref, hT_ref = oracle.scan(la[:, :, ch], g[:, :, ch], h0[:, ch], a_is_log=True)
    assert gen.rel_err(h_h[:, :, ch], h_ref) < TOL
    assert gen.rel_err(hT_h[:, ch], hT_ref) < 1e-4
    assert np.isfinite(h_h).all()


@pytest.mark.parametrize("name,pairs", [("C1", [(0, 0), (5, 4)]), ("C2", [(0, 3)])])
def test_forward_with_the_block_s_merge_full_size(name, pairs):
    # C1: merge as the recurrence kernel's epilogue; C2: 16 time slices, where the library runs it
    # as a kernel of its own
    import paper_2402_19427_amd.runner as rn
    w = gen.CONFIGS[name]
    inp = gen.make_workload(name, dy=False)
    br = gen.make_branch(w.B, w.T, w.D, act=w.act, seed=w.seed)
    dp = rn.DeviceProblem(inp, w.B, w.T, w.D, w.nb, w.act)
    out, y, hT, st = dp.forward_merge(rn.to_device(inp["u"], w.act), rn.to_device(br, w.act),
                                      h0=rn.to_device(inp["h0"], "f32"), keep_y=False)
    out_h, hT_h = rn.to_host(out), rn.to_host(hT)
    del out
    oracle.set_threads(1)
    for b, g in pairs:
        sl, par = block_params(inp, g, w.bs)
        h0_u = None if inp["h0"] is None else np.asarray(inp["h0"][b:b + 1, sl], np.float64)
        out_ref, _, hT_ref, _ = oracle.forward_merge(np.asarray(inp["u"][b:b + 1, :, sl], np.float64),
                                                     br[b:b + 1, :, sl], *par, h0=h0_u)
        assert gen.rel_err(out_h[b:b + 1, :, sl], out_ref) < TOL, (name, b, g)
        assert gen.rel_err(hT_h[b:b + 1, sl], hT_ref) < TOL, (name, b, g)
    assert np.isfinite(out_h).all()


def test_the_paper_s_sixteen_blocks_at_width_2560_full_size():
    # Section 4.1's 16 gate blocks at width 2560 (160 channels each) at C1's size: forward in the
    # padded tile, backward on the widened copy; one sampled (sequence, block) pair for the
    # activations, every sequence for the block's parameter gradients
    import dataclasses
    import paper_2402_19427_amd.runner as rn
    w = dataclasses.replace(gen.CONFIGS["C1"], nb=16)
    inp = gen.make_inputs(w.B, w.T, w.D, w.nb, act=w.act, seed=w.seed, dy=True)
    dp = rn.DeviceProblem(inp, w.B, w.T, w.D, w.nb, w.act)
    u = rn.to_device(inp["u"], w.act)
    y, hT, st = dp.forward(u)
    grads = dp.backward(u, y, rn.to_device(inp["dy"], w.act))
    y_h, du_h = rn.to_host(y), rn.to_host(grads["du"])
    dW_h, dL_h = rn.to_host(grads["dW_a"]), rn.to_host(grads["dLambda"])
    oracle.set_threads(8)
    g = 11
    sl, par = block_params(inp, g, w.bs)
    dW = np.zeros((w.bs, w.bs))
    dL = np.zeros(w.bs)
    for b in range(w.B):
        ub = np.asarray(inp["u"][b:b + 1, :, sl], np.float64)
        dyb = np.asarray(inp["dy"][b:b + 1, :, sl], np.float64)
        ref = oracle.backward(ub, *par, dyb)
        dW += ref["dW_a"][0]
        dL += ref["dLambda"]
        if b == 5:
            y_ref, _, _ = oracle.forward(ub, *par)
            assert gen.rel_err(y_h[b:b + 1, :, sl], y_ref) < TOL
            assert gen.rel_err(du_h[b:b + 1, :, sl], ref["du"]) < TOL
    assert gen.rel_err(dW_h[g], dW) < TOL
    assert gen.rel_err(dL_h[sl], dL) < TOL
    assert np.isfinite(y_h).all() and np.isfinite(du_h).all() and np.isfinite(dW_h).all()


@pytest.mark.parametrize("D", [5632, 8192])
def test_sixteen_blocks_at_the_larger_widths_forward_full_size(D):
    # 16 gate blocks at widths 5632 and 8192 (352 and 512 channels per block): the forward as
    # separate passes on the matrix cores, C1's batch and length, two sampled (sequence, block) pairs
    import dataclasses
    import paper_2402_19427_amd as R
    import paper_2402_19427_amd.runner as rn
    w = dataclasses.replace(gen.CONFIGS["C1"], D=D, nb=16)
    inp = gen.make_inputs(w.B, w.T, w.D, w.nb, act=w.act, seed=w.seed + D, h0=True)
    dp = rn.DeviceProblem(inp, w.B, w.T, w.D, w.nb, w.act)
    y, hT, st = dp.forward(rn.to_device(inp["u"], w.act), h0=rn.to_device(inp["h0"], "f32"))
    sh = dp.shape()
    ws, _ = dp.workspace(sh, R.OP_FORWARD)
    R.rglru_workspace_status(sh, R.OP_FORWARD, ws)
    y_h, hT_h = rn.to_host(y), rn.to_host(hT)
    del y
    oracle.set_threads(8)
    for b, g in [(0, 0), (6, 15)]:
        sl, par = block_params(inp, g, w.bs)
        y_ref, hT_ref, _ = oracle.forward(np.asarray(inp["u"][b:b + 1, :, sl], np.float64), *par,
                                          h0=np.asarray(inp["h0"][b:b + 1, sl], np.float64))
        assert gen.rel_err(y_h[b:b + 1, :, sl], y_ref) < TOL, (D, b, g)
        assert gen.rel_err(hT_h[b:b + 1, sl], hT_ref) < TOL, (D, b, g)
    assert np.isfinite(y_h).all()


def test_sixteen_blocks_at_width_5632_backward_full_size():
    # 352 channels per block: the backward as passes on the matrix cores at C1's batch and length;
    # one sampled block, every sequence through the oracle for its parameter gradients
    import dataclasses
    import paper_2402_19427_amd as R
    import paper_2402_19427_amd.runner as rn
    w = dataclasses.replace(gen.CONFIGS["C1"], D=5632, nb=16)
    inp = gen.make_inputs(w.B, w.T, w.D, w.nb, act=w.act, seed=w.seed + 7, dy=True)
    dp = rn.DeviceProblem(inp, w.B, w.T, w.D, w.nb, w.act)
    u = rn.to_device(inp["u"], w.act)
    y, hT, st = dp.forward(u)
    grads = dp.backward(u, y, rn.to_device(inp["dy"], w.act))
    sh = dp.shape()
    ws, _ = dp.workspace(sh, R.OP_BACKWARD)
    R.rglru_workspace_status(sh, R.OP_BACKWARD, ws)
    du_h = rn.to_host(grads["du"])
    dWa_h, dWx_h, dL_h = rn.to_host(grads["dW_a"]), rn.to_host(grads["dW_x"]), rn.to_host(grads["dLambda"])
    dcw_h = rn.to_host(grads["dconv_w"])
    oracle.set_threads(8)
    g = 9
    sl, par = block_params(inp, g, w.bs)
    acc = dict(dW_a=np.zeros((w.bs, w.bs)), dW_x=np.zeros((w.bs, w.bs)), dLambda=np.zeros(w.bs),
               dconv_w=np.zeros((4, w.bs)))
    for b in range(w.B):
        ref = oracle.backward(np.asarray(inp["u"][b:b + 1, :, sl], np.float64), *par,
                              np.asarray(inp["dy"][b:b + 1, :, sl], np.float64))
        acc["dW_a"] += ref["dW_a"][0]
        acc["dW_x"] += ref["dW_x"][0]
        acc["dLambda"] += ref["dLambda"]
        acc["dconv_w"] += ref["dconv_w"]
        if b == 2:
            assert gen.rel_err(du_h[b:b + 1, :, sl], ref["du"]) < TOL
    assert gen.rel_err(dWa_h[g], acc["dW_a"]) < TOL
    assert gen.rel_err(dWx_h[g], acc["dW_x"]) < TOL
    assert gen.rel_err(dL_h[sl], acc["dLambda"]) < TOL
    assert gen.rel_err(dcw_h[:, sl], acc["dconv_w"]) < TOL
    assert np.isfinite(du_h).all() and np.isfinite(dWa_h).all() and np.isfinite(dWx_h).all()


@pytest.mark.parametrize("name,backward,packed", [("C4", True, False), ("C1", True, False), ("C2", False, False),
                                                  ("C4", True, True), ("C1", True, True), ("C2", False, True)])
def test_every_unit_gives_the_same_result_on_replicated_inputs_full_size(name, backward, packed):
    """Sampling (sequence, gate block) pairs would miss a mis-indexed block or a bad block-id
    remapping on a pair that is not sampled. Here every pair gets the SAME data (inputs, weights,
    states, upstream gradient replicated over sequences and blocks): all units then have to agree
    bit for bit with unit (0, 0) - the arithmetic of a unit does not depend on where it sits - and
    unit (0, 0) is checked against the oracle. Gradients that sum over the batch are B times one
    sequence's contribution in every block alike."""
    import torch
    import paper_2402_19427_amd.runner as rn
    w = gen.CONFIGS[name]
    B, T, D, nb, bs = w.B, w.T, w.D, w.nb, w.bs
    one = gen.make_inputs(1, T, bs, 1, act=w.act, seed=w.seed + 50, h0=True, dy=True, bias=True)
    tile_c = lambda a: np.tile(a, (1,) * (a.ndim - 1) + (nb,))         # replicate along the channel axis
    inp = dict(one)
    inp["W_a"], inp["W_x"] = np.repeat(one["W_a"], nb, axis=0), np.repeat(one["W_x"], nb, axis=0)
    for k in ("b_a", "b_x", "Lambda", "conv_w", "conv_b"):
        inp[k] = tile_c(one[k])
    dp = rn.DeviceProblem(inp, B, T, D, nb, w.act)
    rep = lambda a, act: rn.to_device(a, act)[:, :, None, :].expand(B, T, nb, bs).reshape(B, T, D).contiguous()
    u = rep(one["u"], w.act)
    h0 = rn.to_device(one["h0"], "f32")[:, None, :].expand(B, nb, bs).reshape(B, D).contiguous()
    reset = gen.make_resets(1, T, seed=w.seed, mean_len=300) if packed else None   # the same documents in every row
    r_dev = torch.from_numpy(np.repeat(reset, B, axis=0)).cuda() if packed else None
    y, hT, st = dp.forward_packed(u, r_dev, h0=h0) if packed else dp.forward(u, h0=h0)
    units = lambda t: t.reshape(B, -1, nb, bs)
    assert bool((units(y) == units(y)[:1, :, :1]).all()), "y differs between units"
    assert bool((units(hT) == units(hT)[:1, :, :1]).all()) and bool((units(st) == units(st)[:1, :, :1]).all())
    q = {k: (None if v is None else np.asarray(v, np.float64)) for k, v in one.items()}
    par = (q["W_a"], q["W_x"], q["b_a"], q["b_x"], q["Lambda"], q["conv_w"])
    oracle.set_threads(1)
    y_ref, hT_ref, _ = oracle.forward(q["u"], *par, conv_b=q["conv_b"], h0=q["h0"], reset=reset)
    assert gen.rel_err(rn.to_host(y[:1, :, :bs]), y_ref) < TOL
    assert gen.rel_err(rn.to_host(hT[:1, :bs]), hT_ref) < TOL
    if not backward:
        return
    dy = rep(one["dy"], w.act)
    dhT = rn.to_device(one["dhT"], "f32")[:, None, :].expand(B, nb, bs).reshape(B, D).contiguous()
    g = dp.backward_packed(u, r_dev, y, dy, h0=h0, dhT=dhT) if packed else dp.backward(u, y, dy, h0=h0, dhT=dhT)
    for k in ("du", "dh0"):
        assert bool((units(g[k]) == units(g[k])[:1, :, :1]).all()), k
    for k in ("dW_a", "dW_x"):
        assert bool((g[k] == g[k][:1]).all()), k
    for k in ("db_a", "db_x", "dLambda", "dconv_b"):
        v = g[k].reshape(nb, bs)
        assert bool((v == v[:1]).all()), k
    v = g["dconv_w"].reshape(4, nb, bs)
    assert bool((v == v[:, :1]).all())
    ref = oracle.backward(q["u"], *par, q["dy"], conv_b=q["conv_b"], h0=q["h0"], dhT=q["dhT"], reset=reset)
    assert gen.rel_err(rn.to_host(g["du"][:1, :, :bs]), ref["du"]) < TOL
    assert gen.rel_err(rn.to_host(g["dh0"][:1, :bs]), ref["dh0"]) < TOL
    assert gen.rel_err(rn.to_host(g["dW_a"][0]), B * ref["dW_a"][0]) < TOL
    assert gen.rel_err(rn.to_host(g["dW_x"][0]), B * ref["dW_x"][0]) < TOL
    for k in ("db_a", "db_x", "dLambda", "dconv_b"):
        assert gen.rel_err(rn.to_host(g[k][:bs]), B * ref[k]) < TOL, k
    assert gen.rel_err(rn.to_host(g["dconv_w"][:, :bs]), B * ref["dconv_w"]) < TOL
