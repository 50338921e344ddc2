#!/usr/bin/env python3
"""Benchmark of the Conv1D -> RG-LRU hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic input, inputs already
resident in HBM: rglru_forward over [B,T,D], one rglru_decode_step continuing the B sequences
by one token from the states the forward call produced, and rglru_backward over the same
batch. Prints ONE JSON line (see the keys below). Everything is seeded and synthetic.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C1]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA, published


def algorithmic_costs(B, T, D, nb):
    """Bytes each entry point must move (every input read once, every output written once,
    intermediates never touching HBM) and the gate-contraction FLOPs it must execute."""
    bs = D // nb
    N = B * T * D
    w_bytes = 2 * nb * bs * bs * 2                     # both gate matrices, bf16
    vec = 8 * D * 4                                     # b_a, b_x, Lambda, conv_w, conv_b-sized slack
    fwd = dict(bytes=4 * N + w_bytes + vec + 4 * B * D + 6 * B * D,   # u in, y out, hT, conv state
               flops=4 * bs * N)                        # two [T x bs] x [bs x bs] products
    dec = dict(bytes=(2 + 6 + 2 + 4 + 4 + 2) * B * D + w_bytes + vec, flops=4 * bs * B * D)
    bwd = dict(bytes=8 * N + w_bytes + vec + 2 * nb * bs * bs * 4 + 8 * B * D,  # u,y,dy in; du out; dW
               flops=12 * bs * N)                       # gate recompute + dgrad + wgrad
    return fwd, dec, bwd


def cpu_baseline(w, seconds_hint=20.0):
    """The float64 oracle as it stands, one thread, on a bounded sample of the same workload:
    B_s sequences at the full width and length, forward + one decode step + backward."""
    import numpy as np
    import oracle
    import rglru_inputs as gen
    B_s, T_s = 2, min(w.T, 2048)
    inp = gen.make_inputs(B_s, T_s + 1, w.D, w.nb, act=w.act, seed=w.seed, dy=True)
    q = {k: (None if v is None else np.asarray(v, np.float64)) for k, v in inp.items()}
    par = (q["W_a"], q["W_x"], q["b_a"], q["b_x"], q["Lambda"], q["conv_w"])
    oracle.set_threads(1)
    t0 = time.perf_counter()
    y, hT, st = oracle.forward(q["u"][:, :T_s], *par)
    oracle.decode_step(q["u"][:, T_s], *par, hT, st)
    oracle.backward(q["u"][:, :T_s], *par, q["dy"][:, :T_s])
    dt = time.perf_counter() - t0
    return {"value": B_s * (T_s + 1) / dt, "unit": "tokens/s", "cores": 1, "kind": "oracle",
            "sample": "%d sequences x %d steps x D=%d (nb=%d) of the workload: forward + 1 decode "
                      "step + backward in %.1f s" % (B_s, T_s, w.D, w.nb, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C1")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; --gpus %d is not supported "
                 "(no collectives or sharding are part of it)" % args.gpus)

    import numpy as np
    import torch
    import rglru_inputs as gen
    import paper_2402_19427_amd as R
    import paper_2402_19427_amd.runner as rn

    w = gen.CONFIGS[args.workload]
    B, T, D, nb = w.B, w.T, w.D, w.nb
    dev = "cuda:0"
    torch.cuda.set_device(0)
    inp = gen.make_inputs(B, T + 1, D, nb, act=w.act, seed=w.seed, h0=w.h0, dy=True)
    dp = rn.DeviceProblem(inp, B, T, D, nb, w.act, device=dev)
    u_all = rn.to_device(inp["u"], w.act, dev)
    u = u_all[:, :T].contiguous()
    u_next = u_all[:, T].contiguous()
    dy = rn.to_device(inp["dy"][:, :T], w.act, dev)
    h0 = rn.to_device(inp["h0"], "f32", dev)
    del u_all, inp

    sh = dp.shape()
    sh1 = dp.shape(T=1)
    ws_f, n_f = dp.workspace(sh, R.OP_FORWARD)
    ws_b, n_b = dp.workspace(sh, R.OP_BACKWARD)
    y = dp.empty_act(B, T, D)
    hT = dp.empty_f32(B, D)
    st = dp.empty_act(B, 3, D)
    y1 = dp.empty_act(B, D)
    du = dp.empty_act(B, T, D)
    dh0 = dp.empty_f32(B, D)
    g = dp.alloc_grads()
    pg = R.make_param_grads(g["dW_a"], g["dW_x"], g["db_a"], g["db_x"], g["dLambda"],
                            g["dconv_w"], g["dconv_b"])
    stream = torch.cuda.current_stream()
    sh_ptr = stream.cuda_stream

    def step(ev=None):
        if ev:
            ev[0].record(stream)
        R.rglru_forward(sh, dp.params, u, h0, None, 0, y, hT, st, ws_f, n_f, sh_ptr)
        if ev:
            ev[1].record(stream)
        R.rglru_decode_step(sh1, dp.params, u_next, hT, st, T, y1, sh_ptr)
        if ev:
            ev[2].record(stream)
        R.rglru_backward(sh, dp.params, u, h0, None, 0, y, dy, None, du, dh0, pg, ws_b, n_b, sh_ptr)
        if ev:
            ev[3].record(stream)

    for _ in range(args.warmup):
        step()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(events[k])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    ms = [[e[i].elapsed_time(e[i + 1]) for i in range(3)] for e in events]
    avg = [float(np.mean([m[i] for m in ms])) for i in range(3)]   # fwd, decode, bwd (ms)
    tokens = B * T + B
    ms_per_step = 1e3 * elapsed / args.steps
    fwd_c, dec_c, bwd_c = algorithmic_costs(B, T, D, nb)

    def roof(name, cost, t_ms):
        t_hbm = cost["bytes"] / (HBM_PEAK_GBS * 1e9)
        t_mfma = cost["flops"] / (MFMA_BF16_PEAK_TFLOPS * 1e12)
        if t_hbm >= t_mfma:
            ach = cost["bytes"] / (t_ms * 1e-3) / 1e9
            return {"kernel": name, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": ach / HBM_PEAK_GBS, "traffic": None,
                    "algorithmic_bytes": cost["bytes"], "avg_ms": t_ms}
        ach = cost["flops"] / (t_ms * 1e-3) / 1e12
        return {"kernel": name, "bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": ach / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                "algorithmic_flops": cost["flops"], "avg_ms": t_ms}

    roofs = [roof("rglru_forward", fwd_c, avg[0]), roof("rglru_decode_step", dec_c, avg[1]),
             roof("rglru_backward", bwd_c, avg[2])]
    dominant = max(range(3), key=lambda i: avg[i])

    out = {
        "metric": "RG-LRU block tokens/sec and achieved HBM GB/s (% of MI355X peak)",
        "value": tokens / (elapsed / args.steps),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.act == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": "%s: B=%d T=%d D=%d nb=%d %s, forward + 1 decode step + backward"
                               % (w.name, B, T, D, nb, w.act),
                   "global_batch": B, "seq_len": T},
        "roofline": roofs[dominant],
        "entry_points": roofs,
        "hbm_gbs_step": (fwd_c["bytes"] + dec_c["bytes"] + bwd_c["bytes"]) / (elapsed / args.steps) / 1e9,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
