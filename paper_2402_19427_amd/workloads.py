"""Per-workload timing report of the Conv1D -> RG-LRU path on one MI355X.

    python -m paper_2402_19427_amd.workloads [--configs C0,C1,C2,C3,C4,SCAN,MERGE,NB16,CG] [--json]

For each of the five synthetic workloads it times the calls that workload is about (forward;
forward and backward for the training shape; the single-token decode step for the decode shape,
launch by launch and as one HIP graph of 1000 steps) with HIP events on the stream the library
launches on, and prints median / minimum time, tokens/s, the algorithmic bytes of the call
divided by the time (GB/s and fraction of the 8 TB/s HBM peak) and the gate-product FLOP rate
against the dense bf16 MFMA peak. Small workloads rotate several buffer sets so that the
footprint of consecutive iterations exceeds the 256 MB last-level cache ("cold"); the decode
step is also timed on one buffer set ("hot"). SCAN is the scan-only entry point (eq. 4 over
given decays and gated inputs) at the shape the paper times it: batch 8, width 1024, a sweep of
sequence lengths. MERGE times the calls that take the recurrent block's merge with its GeLU
branch along (as the kernels' epilogue, and as a kernel of its own for comparison) on the
workloads C1-C4. NB16 repeats C1 (forward, backward) and a decode step at width 2560 with the
paper's 16 gate blocks of 160 channels (Section 4.1) instead of 10 blocks of 256. Inputs are
seeded and synthetic.
"""
import argparse
import dataclasses
import json
import sys

import numpy as np
import torch

import rglru_inputs as gen
from . import binding as R
from . import runner as rn

HBM_PEAK = 8.0e12
MFMA_PEAK = 2.5e15
LLC_BYTES = 256 << 20


def alg_bytes(kind, B, T, D, nb, act_b):
    """Bytes the method itself must move per call: inputs read once, outputs written once."""
    bs = D // nb
    N = B * T * D
    w = 2 * nb * bs * bs * (2 if act_b == 2 else 4)
    vec = 8 * D * 4
    if kind == "forward":      # u in, y out, weights, h_T and conv state out
        return 2 * act_b * N + w + vec + (4 + 3 * act_b) * B * D
    if kind == "backward":     # u, y, dy in; du out; dW out (fp32)
        return 4 * act_b * N + w + vec + 2 * nb * bs * bs * 4
    if kind == "decode":       # u_t, 3 ring slots in + 1 out, h in + out, y_t, weights
        return (act_b + 3 * act_b + act_b + 8 + act_b) * B * D + w + vec
    if kind == "forward_merge":        # u, branch in; out out
        return alg_bytes("forward", B, T, D, nb, act_b) + act_b * N
    if kind == "forward_merge_keep":   # ... and y kept for the backward
        return alg_bytes("forward", B, T, D, nb, act_b) + 2 * act_b * N
    if kind == "backward_merge":       # u, y, branch, dout in; du, dbranch out
        return alg_bytes("backward", B, T, D, nb, act_b) + 2 * act_b * N
    if kind == "decode_merge":
        return alg_bytes("decode", B, T, D, nb, act_b) + act_b * B * D
    raise ValueError(kind)


def gate_flops(kind, B, T, D, nb):
    bs = D // nb
    N = B * T * D
    return {"forward": 4, "decode": 4, "backward": 12}[kind.split("_")[0]] * bs * N


def time_calls(fn, nsets, iters, warmup):
    """Times fn(set_index) per call with events on the current stream; returns ms per call."""
    for i in range(warmup):
        fn(i % nsets)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(iters)]
    for i in range(iters):
        ev[i][0].record()
        fn(i % nsets)
        ev[i][1].record()
    torch.cuda.synchronize()
    return np.array([a.elapsed_time(b) for a, b in ev])


def row(name, phase, note, ms, tokens, nbytes, flops):
    med, mn = float(np.median(ms)), float(ms.min())
    return {"workload": name, "call": phase, "note": note, "ms_median": med, "ms_min": mn,
            "tokens_per_s": tokens / (med * 1e-3), "alg_bytes": nbytes,
            "alg_GBs": nbytes / (med * 1e-3) / 1e9, "hbm_frac": nbytes / (med * 1e-3) / HBM_PEAK,
            "mfma_frac": flops / (med * 1e-3) / MFMA_PEAK}


def run_sequence_workload(w, dev, out, label="forward"):
    B, T, D, nb = w.B, w.T, w.D, w.nb
    act_b = 2 if w.act == "bf16" else 4
    inp = gen.make_inputs(1, 8, D, nb, act=w.act, seed=w.seed)       # parameters only
    dp = rn.DeviceProblem(inp, B, T, D, nb, w.act, device=dev)
    sh = dp.shape()
    per_set = 2 * act_b * B * T * D
    nsets = int(min(8, max(1, -(-LLC_BYTES * 5 // 4 // per_set))))
    iters = 100 if B * T * D < (1 << 27) else 30
    draws = rn.SeededDraws(w.seed + 200, dev)
    us = [draws.normal(B, T, D, act=w.act) for _ in range(nsets)]
    h0 = draws.normal(B, D) if w.h0 else None
    ys = [dp.empty_act(B, T, D) for _ in range(nsets)]
    hT = dp.empty_f32(B, D)
    st = dp.empty_act(B, 3, D)
    ws_f, n_f = dp.workspace(sh, R.OP_FORWARD)
    sp = torch.cuda.current_stream().cuda_stream

    def fwd(i):
        R.rglru_forward(sh, dp.params, us[i], h0, None, 0, ys[i], hT, st, ws_f, n_f, sp)

    note = "%d buffer set%s" % (nsets, "s" if nsets > 1 else "")
    ms = time_calls(fwd, nsets, iters, 10)
    out.append(row(w.name, label, note, ms, B * T, alg_bytes("forward", B, T, D, nb, act_b),
                   gate_flops("forward", B, T, D, nb)))
    if w.kind != "train" and w.name != "C1":
        return
    for i in range(nsets):
        fwd(i)
    dys = [draws.normal(B, T, D, act=w.act) for _ in range(nsets)]
    du = dp.empty_act(B, T, D)
    dh0 = dp.empty_f32(B, D)
    g = dp.alloc_grads()
    pg = R.make_param_grads(g["dW_a"], g["dW_x"], g["db_a"], g["db_x"], g["dLambda"],
                            g["dconv_w"], g["dconv_b"])
    ws_b, n_b = dp.workspace(sh, R.OP_BACKWARD)

    def bwd(i):
        R.rglru_backward(sh, dp.params, us[i], h0, None, 0, ys[i], dys[i], None, du, dh0, pg,
                         ws_b, n_b, sp)

    ms = time_calls(bwd, nsets, iters, 5)
    out.append(row(w.name, label.replace("forward", "backward"), note, ms, B * T,
                   alg_bytes("backward", B, T, D, nb, act_b),
                   gate_flops("backward", B, T, D, nb)))


def run_decode_workload(w, dev, out, steps=1000, graph_only=False, label="decode,"):
    B, D, nb = w.B, w.D, w.nb
    act_b = 2 if w.act == "bf16" else 4
    inp = gen.make_inputs(1, 8, D, nb, act=w.act, seed=w.seed)
    dp = rn.DeviceProblem(inp, B, 1, D, nb, w.act, device=dev)
    sh = dp.shape(T=1)
    nbytes = alg_bytes("decode", B, 1, D, nb, act_b)
    flops = gate_flops("decode", B, 1, D, nb)
    per_set = (6 * act_b + 8) * B * D
    ncold = int(-(-LLC_BYTES * 5 // 4 // per_set))
    draws = rn.SeededDraws(w.seed + 200, dev)

    def make_set():
        return dict(u=draws.normal(B, D, act=w.act),
                    h=draws.normal(B, D),
                    st=draws.normal(B, 3, D, act=w.act),
                    y=dp.empty_act(B, D))

    sets = [make_set() for _ in range(ncold)]
    sp = torch.cuda.current_stream().cuda_stream
    pos = [3]

    def step(i):
        s = sets[i]
        R.rglru_decode_step(sh, dp.params, s["u"], s["h"], s["st"], pos[0], s["y"], sp)
        pos[0] += 1

    label_head = label
    for nsets, label in ((1, "hot: 1 buffer set"), (ncold, "cold: %d buffer sets" % ncold)):
        ms = time_calls(step, nsets, 20 if graph_only else steps, 20)
        if not graph_only:
            out.append(row(w.name, "decode, per launch", label, ms, B, nbytes, flops))
            # the same 1000 steps back to back: launch overhead overlaps with execution
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(steps):
                step(i % nsets)
            e1.record()
            torch.cuda.synchronize()
            ms = np.array([e0.elapsed_time(e1) / steps])
            out.append(row(w.name, "decode, %d launches back to back" % steps, label, ms, B, nbytes, flops))
        # ... and replayed as one HIP graph (the position is baked in at capture: timing only)
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph):
            spg = torch.cuda.current_stream().cuda_stream    # the capturing stream
            for i in range(steps):
                s = sets[i % nsets]
                R.rglru_decode_step(sh, dp.params, s["u"], s["h"], s["st"], 3 + i, s["y"], spg)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        reps = []
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            graph.replay()
            e1.record()
            torch.cuda.synchronize()
            reps.append(e0.elapsed_time(e1) / steps)
        out.append(row(w.name, "%s one graph of %d steps" % (label_head, steps), label, np.array(reps), B,
                       nbytes, flops))
        del graph


def run_scan_workload(dev, out, lengths=(1024, 4096, 16384, 65536)):
    """rglru_scan at batch 8, width 1024 (Appendix A.3), bf16 storage: a_t and g_t read, h_t
    written, 6 bytes per element; the state lives on chip."""
    B, D = 8, 1024
    for T in lengths:
        per_set = 3 * 2 * B * T * D
        nsets = int(min(8, max(1, -(-LLC_BYTES * 5 // 4 // per_set))))
        sh = R.make_shape(B, T, D, 1, R.BF16)
        n = R.rglru_workspace_bytes(sh, R.OP_SCAN)
        ws = torch.empty(max(n, 256), dtype=torch.uint8, device=dev)
        sets = []
        for i in range(nsets):
            # decays distributed like the layer's (the seeded generator of the parity tests):
            # base^8 ~ U[0.9, 0.999], power 8 r with r ~ U(0, 1); a_t and log a_t of different draws
            si = gen.make_scan_inputs(B, T, D, act="bf16", seed=7000 + 2 * i, h0=(i == 0))
            sl = gen.make_scan_inputs(B, T, D, act="bf16", seed=7001 + 2 * i, log_a=True, h0=False)
            if i == 0:
                h0 = rn.to_device(si["h0"], "f32", dev)
            sets.append(dict(a=rn.to_device(si["a"], "bf16", dev), la=rn.to_device(sl["a"], "bf16", dev),
                             g=rn.to_device(si["g"], "bf16", dev),
                             h=torch.empty(B, T, D, dtype=torch.bfloat16, device=dev)))
            del si, sl
        hT = torch.empty(B, D, device=dev)
        sp = torch.cuda.current_stream().cuda_stream
        nbytes = per_set + 8 * B * D
        note = "%d buffer set%s" % (nsets, "s" if nsets > 1 else "")
        iters = 100 if T <= 16384 else 30
        for key, flags, label in (("a", 0, "scan T=%d" % T), ("la", R.SCAN_LOG_A, "scan T=%d, log a_t" % T),
                                  ("a", R.SCAN_ADJOINT | R.SCAN_NO_INPUT_SCALE, "scan adjoint T=%d" % T)):
            def call(i):
                st = sets[i]
                R.rglru_scan(sh, st[key], st["g"], h0, flags, st["h"], hT, ws, n, sp)
            ms = time_calls(call, nsets, iters, 10)
            out.append(row("SCAN", label, note, ms, B * T, nbytes, 0))
        del sets
        torch.cuda.empty_cache()


def run_merge_workload(dev, out, names=("C1", "C2", "C3", "C4"), steps=1000):
    """The calls with the block's merge (Section 2.3) on the sequence workloads and the decode
    workload: out = y * GeLU(branch) as the kernels' epilogue, against the same merge run as a
    streaming kernel of its own after the plain forward."""
    sp = torch.cuda.current_stream().cuda_stream
    for name in names:
        w = gen.CONFIGS[name]
        B, T, D, nb = w.B, w.T, w.D, w.nb
        act_b = 2
        inp = gen.make_inputs(1, 8, D, nb, act=w.act, seed=w.seed)
        draws = rn.SeededDraws(w.seed + 201, dev)
        if w.kind == "decode":
            dp = rn.DeviceProblem(inp, B, 1, D, nb, w.act, device=dev)
            sh = dp.shape(T=1)
            u, br = (draws.normal(B, D, act=w.act) for _ in range(2))
            h = draws.normal(B, D)
            st = draws.normal(B, 3, D, act=w.act)
            o = dp.empty_act(B, D)
            for label, call in (
                    ("decode", lambda i, q: R.rglru_decode_step(sh, dp.params, u, h, st, 3 + i, o, q)),
                    ("decode + merge", lambda i, q: R.rglru_decode_step_merge(sh, dp.params, u, br, h, st,
                                                                              3 + i, 0, o, q))):
                kind = "decode_merge" if "merge" in label else "decode"
                graph = torch.cuda.CUDAGraph()
                torch.cuda.synchronize()
                with torch.cuda.graph(graph):
                    spg = torch.cuda.current_stream().cuda_stream
                    for i in range(steps):
                        call(i, spg)
                torch.cuda.synchronize()
                graph.replay()
                reps = []
                for _ in range(3):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    graph.replay()
                    e1.record()
                    torch.cuda.synchronize()
                    reps.append(e0.elapsed_time(e1) / steps)
                out.append(row("MERGE", "%s %s, one graph of %d steps" % (name, label, steps),
                               "hot: 1 buffer set", np.array(reps), B, alg_bytes(kind, B, 1, D, nb, act_b),
                               gate_flops("decode", B, 1, D, nb)))
                del graph
            continue
        dp = rn.DeviceProblem(inp, B, T, D, nb, w.act, device=dev)
        sh = dp.shape()
        per_set = 3 * act_b * B * T * D
        nsets = int(min(8, max(1, -(-LLC_BYTES * 5 // 4 // per_set))))
        iters = 100 if B * T * D < (1 << 27) else 30
        us = [draws.normal(B, T, D, act=w.act) for _ in range(nsets)]
        brs = [draws.normal(B, T, D, act=w.act) for _ in range(nsets)]
        outs = [dp.empty_act(B, T, D) for _ in range(nsets)]
        ys = [dp.empty_act(B, T, D) for _ in range(nsets)]
        h0 = draws.normal(B, D) if w.h0 else None
        hT, st = dp.empty_f32(B, D), dp.empty_act(B, 3, D)
        ws_f, n_f = dp.workspace(sh, R.OP_FORWARD_MERGE)
        note = "%d buffer set%s" % (nsets, "s" if nsets > 1 else "")

        def fwd(flags, keep):
            def call(i):
                R.rglru_forward_merge(sh, dp.params, us[i], brs[i], h0, None, 0, flags, outs[i],
                                      ys[i] if keep else None, hT, st, ws_f, n_f, sp)
            return call

        for label, flags, keep in (("forward, merge as a kernel of its own", R.MERGE_SEPARATE, False),
                                   ("forward + merge", 0, False),
                                   ("forward + merge, tanh form", R.MERGE_GELU_TANH, False),
                                   ("forward + merge, y kept", 0, True)):
            ms = time_calls(fwd(flags, keep), nsets, iters, 10)
            kind = "forward_merge_keep" if keep else "forward_merge"
            out.append(row("MERGE", "%s %s" % (name, label), note, ms, B * T,
                           alg_bytes(kind, B, T, D, nb, act_b), gate_flops("forward", B, T, D, nb)))
        if w.kind != "train" and name != "C1":
            del us, brs, outs, ys
            torch.cuda.empty_cache()
            continue
        douts = [draws.normal(B, T, D, act=w.act) for _ in range(nsets)]
        du, dbr, dh0 = dp.empty_act(B, T, D), dp.empty_act(B, T, D), dp.empty_f32(B, D)
        g = dp.alloc_grads()
        pg = R.make_param_grads(g["dW_a"], g["dW_x"], g["db_a"], g["db_x"], g["dLambda"],
                                g["dconv_w"], g["dconv_b"])
        ws_b, n_b = dp.workspace(sh, R.OP_BACKWARD_MERGE)

        def bwd(i):
            R.rglru_backward_merge(sh, dp.params, us[i], brs[i], h0, None, 0, 0, ys[i], douts[i], None,
                                   du, dbr, dh0, pg, ws_b, n_b, sp)

        ms = time_calls(bwd, nsets, iters, 5)
        out.append(row("MERGE", "%s backward + merge" % name, note, ms, B * T,
                       alg_bytes("backward_merge", B, T, D, nb, act_b), gate_flops("backward", B, T, D, nb)))
        del us, brs, outs, ys, douts
        torch.cuda.empty_cache()


def run_cg_workload(dev, out, sizes=((8, 2048, 2560, 10), (16, 4096, 4096, 16)), steps=200):
    """The complex-gated variant (Appendix B), bf16 storage: forward (with its optional scratch) and
    backward at C1's and C4's sizes, a decode step at batch 256. Algorithmic bytes: u in, y out
    (backward: u, dy in, du out - this backward takes no y), the [hs][2 hs] gate matrices; gate FLOPs
    2 (D / nb) per element forward, three times that backward."""
    sp = torch.cuda.current_stream().cuda_stream
    for (B, T, D, nb) in sizes:
        inp = gen.make_cg_inputs(1, 8, D, nb, act="bf16", seed=3)       # parameters only
        cg = rn.CgDeviceProblem(inp, B, T, D, nb, "bf16", device=dev)
        sh = cg.shape()
        H, hs = D // 2, D // 2 // nb
        draws = rn.SeededDraws(300 + D, dev)
        u, dy = draws.normal(B, T, D, act="bf16"), draws.normal(B, T, D, act="bf16")
        y = torch.empty_like(u)
        hT = torch.empty(B, D, dtype=torch.float32, device=dev)
        st = torch.empty(B, 3, D, dtype=torch.bfloat16, device=dev)
        n_f = R.rglru_workspace_bytes(sh, R.OP_CG_FORWARD)
        ws_f = torch.empty(max(n_f, 256), dtype=torch.uint8, device=dev)
        n_b = R.rglru_workspace_bytes(sh, R.OP_CG_BACKWARD)
        ws_b = torch.empty(max(n_b, 256), dtype=torch.uint8, device=dev)
        f32 = lambda *shape: torch.empty(*shape, dtype=torch.float32, device=dev)
        g = [f32(nb, hs, 2 * hs), f32(nb, hs, 2 * hs), f32(H), f32(H), f32(H), f32(H), f32(4, D), f32(D)]
        pg = R.make_cg_param_grads(*g)
        du, dh0 = torch.empty_like(u), f32(B, D)
        size = "B%d T%d D%d nb%d" % (B, T, D, nb)
        N, wcg, vec = B * T * D, 2 * nb * hs * 2 * hs * 2, 9 * H * 4 + 5 * D * 4
        fwd_bytes = 4 * N + wcg + vec + 10 * B * D
        bwd_bytes = 6 * N + wcg + vec + 2 * nb * hs * 2 * hs * 4
        fwd_flops = 2 * (D // nb) * N

        def fwd(i):
            R.rglru_cg_forward(sh, cg.params, u, None, None, 0, y, hT, st, ws_f, n_f, sp)

        def bwd(i):
            R.rglru_cg_backward(sh, cg.params, u, None, None, 0, dy, None, du, dh0, pg, ws_b, n_b, sp)

        iters = 30 if B * T * D < (1 << 27) else 10
        ms = time_calls(fwd, 1, iters, 3)
        out.append(row("CG", "forward, " + size, "1 buffer set", ms, B * T, fwd_bytes, fwd_flops))
        ms = time_calls(bwd, 1, iters, 2)
        out.append(row("CG", "backward, " + size, "1 buffer set", ms, B * T, bwd_bytes, 3 * fwd_flops))
        del ws_f, ws_b, u, dy, y, du
        torch.cuda.empty_cache()
    B, D, nb = 256, 2560, 10
    inp = gen.make_cg_inputs(1, 8, D, nb, act="bf16", seed=3)
    cg = rn.CgDeviceProblem(inp, B, 1, D, nb, "bf16", device=dev)
    draws = rn.SeededDraws(77, dev)
    u_t, h = draws.normal(B, D, act="bf16"), draws.normal(B, D)
    ring = draws.normal(B, 3, D, act="bf16")
    y_t = torch.empty_like(u_t)
    sh = cg.shape(T=1, B=B)
    pos = [3]

    def step(i):
        R.rglru_cg_decode_step(sh, cg.params, u_t, h, ring, pos[0], y_t, sp)
        pos[0] += 1

    ms = time_calls(step, 1, steps, 10)
    out.append(row("CG", "decode step, B%d D%d nb%d, per launch" % (B, D, nb), "hot: 1 buffer set", ms, B,
                   alg_bytes("decode", B, 1, D, nb, 2) - 2 * nb * (D // nb) * (D // nb), 2 * (D // nb) * B * D))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--configs", default="C0,C1,C2,C3,C4,SCAN,MERGE,NB16,CG")
    ap.add_argument("--scan-lengths", default="1024,4096,16384,65536")
    ap.add_argument("--json", action="store_true", help="print one JSON object per row instead of the table")
    args = ap.parse_args()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    out = []
    for name in args.configs.split(","):
        n0 = len(out)
        w = gen.CONFIGS.get(name)
        if name == "SCAN":
            run_scan_workload(dev, out, tuple(int(x) for x in args.scan_lengths.split(",")))
        elif name == "MERGE":
            run_merge_workload(dev, out)
        elif name == "CG":
            run_cg_workload(dev, out)
        elif name == "NB16":
            c1 = gen.CONFIGS["C1"]
            run_sequence_workload(dataclasses.replace(c1, name="NB16", nb=16, kind="train"), dev, out)
            run_decode_workload(dataclasses.replace(gen.CONFIGS["C3"], name="NB16", D=2560), dev, out,
                                graph_only=True)
            # the larger widths of the model family, 352 and 512 channels per block: forward only
            # (separate passes on the matrix cores)
            for D in (5632, 8192):
                run_sequence_workload(dataclasses.replace(c1, name="NB16", D=D, nb=16, kind="train"),
                                      dev, out, label="forward, width %d" % D)
                run_decode_workload(dataclasses.replace(gen.CONFIGS["C3"], name="NB16", D=D), dev, out,
                                    graph_only=True, label="decode, width %d," % D)
        elif w.kind == "decode":
            run_decode_workload(w, dev, out)
        else:
            run_sequence_workload(w, dev, out)
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        for r in out[n0:]:
            if args.json:
                print(json.dumps(r), flush=True)
            else:
                print("%-5s %-46s %-22s median %9.2f us  min %9.2f us  %8.2f M tok/s  %7.1f GB/s "
                      "= %5.1f%% of HBM peak  %5.1f%% of MFMA peak"
                      % (r["workload"], r["call"], r["note"], r["ms_median"] * 1e3, r["ms_min"] * 1e3,
                         r["tokens_per_s"] / 1e6, r["alg_GBs"], 100 * r["hbm_frac"],
                         100 * r["mfma_frac"]), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
