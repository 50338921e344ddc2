#!/usr/bin/env python3
"""Benchmark of the Conv1D -> RG-LRU hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic input, inputs already
resident in HBM. The default workload is the largest single-GPU one, C4 (B=16 T=4096 D=4096,
16 gate blocks of 256, bf16): rglru_forward over [B,T,D], rglru_backward over the same batch, and
one rglru_decode_step for a batch of 256 sequences at the same width (the decode workload C3).
Other workloads (--workload): C1 = forward + backward + a decode step continuing its B
sequences, C2 = the long forward alone, C3 = the decode step alone. Prints ONE JSON line.
Everything is seeded and synthetic (numpy PCG64, see rglru_inputs.py).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C4]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA, published
LLC_BYTES = 256 << 20           # last-level cache behind the L2s
DECODE_BATCH = 256              # batch of the decode workload (C3)


def algorithmic_costs(B, T, D, nb, B_dec):
    """Per kernel: the bytes of the METHOD's own inputs and outputs that the kernel touches
    (each read or written once; tensors that exist only because the backward is split into
    three kernels are not algorithmic traffic) and the gate-contraction FLOPs it executes."""
    bs = D // nb
    N = B * T * D
    w_bytes = 2 * nb * bs * bs * 2                      # both gate matrices, bf16
    vec = 8 * D * 4                                      # b_a, b_x, Lambda, conv_w, conv_b
    gemm = 4 * bs * N                                    # two [rows x bs] x [bs x bs] products
    return {
        # u in, y out, weights, hT and conv state out
        "fwd_mfma_kernel": dict(bytes=4 * N + w_bytes + vec + 10 * B * D, flops=gemm),
        # the aggregate pass of a single long prompt's forward (contiguous windows in two passes;
        # the forward proper then is a launch of fwd_mfma_kernel): u in, weights
        "fwd_agg_mfma_kernel": dict(bytes=2 * N + w_bytes + vec, flops=gemm),
        # u_t, 3 ring slots read + 1 written, h read + written, y_t, weights
        "decode_mfma_kernel": dict(bytes=(2 + 6 + 2 + 4 + 4 + 2) * B_dec * D + w_bytes + vec,
                                   flops=4 * bs * B_dec * D),
        # u, y, dy in (gate recompute + reverse scan + pointwise adjoints)
        "bwd_gates_kernel": dict(bytes=6 * N + w_bytes + vec + 8 * B * D, flops=gemm),
        # u in (for dconv_w), du out
        "bwd_dgrad_kernel": dict(bytes=4 * N + w_bytes + vec, flops=gemm),
        # dW_a, dW_x out (fp32)
        "bwd_wgrad_kernel": dict(bytes=2 * nb * bs * bs * 4, flops=gemm),
    }


def read_traffic(workload):
    """HBM-side bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE): taken
    from the committed summary profiles/hbm_traffic_<workload>.txt (lines `traffic_bytes kernel
    bytes`), NOT measured in this run; None for a kernel or workload without a summary."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_%s.txt" % workload)
    out = {}
    if os.path.exists(path):
        for line in open(path):
            if line.startswith("traffic_bytes "):
                _, name, val = line.split()
                out[name] = float(val)
    return out, (os.path.relpath(path, ROOT) if out else None)


def cpu_baseline(w, legs):
    """The float64 oracle as it stands on a bounded sample of the same workload: one full-length
    sequence at the full width (all gate blocks), the same calls as the GPU step. Timed twice:
    on one thread and on all host cores (OpenMP over the independent (sequence, gate block)
    pairs; identical results)."""
    import numpy as np
    import oracle
    import rglru_inputs as gen
    B_s = 1
    T_s = w.T if w.kind != "decode" else 1
    B_run = B_s if w.kind != "decode" else 16
    inp = gen.make_inputs(B_run, T_s + 1, w.D, w.nb, act=w.act, seed=w.seed, dy=True, state=True)
    q = {k: (None if v is None else np.asarray(v, np.float64)) for k, v in inp.items()}
    par = (q["W_a"], q["W_x"], q["b_a"], q["b_x"], q["Lambda"], q["conv_w"])
    h0 = np.zeros((B_run, w.D))

    def run():
        toks = 0
        if "forward" in legs:
            y, hT, st = oracle.forward(q["u"][:, :T_s], *par)
            toks += B_run * T_s
        if "backward" in legs:
            oracle.backward(q["u"][:, :T_s], *par, q["dy"][:, :T_s])
        if "decode" in legs:
            oracle.decode_step(q["u"][:, T_s], *par, h0, q["state"])
            toks += B_run
        return toks

    nproc = os.cpu_count() or 1
    try:
        nproc = len(os.sched_getaffinity(0))
    except (AttributeError, OSError):
        pass
    res = {}
    for label, nt in (("one_core", 1), ("all_cores", nproc)):
        oracle.set_threads(nt)
        t0 = time.perf_counter()
        toks = run()
        dt = time.perf_counter() - t0
        res[label] = {"value": toks / dt, "cores": nt, "seconds": dt}
    oracle.set_threads(1)
    return {"value": res["all_cores"]["value"], "unit": "tokens/s", "cores": res["all_cores"]["cores"],
            "kind": "oracle", "nproc": nproc,
            "one_core": {"value": res["one_core"]["value"], "cores": 1,
                         "seconds": res["one_core"]["seconds"]},
            "all_cores_seconds": res["all_cores"]["seconds"],
            "sample": "%d sequence(s) x %d steps x D=%d (nb=%d) of the workload, legs %s"
                      % (B_run, T_s, w.D, w.nb, "+".join(legs))}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C4", choices=["C1", "C2", "C3", "C4"],
                    help="default C4: the largest single-GPU workload (forward + backward at "
                         "B16 T4096 D4096 plus a decode step at batch 256). Per-call timings of all "
                         "five workloads: python -m paper_2402_19427_amd.workloads")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 256 MiB device copy, the reference that scales the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run")
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
    legs = {"C1": ("forward", "backward", "decode"), "C2": ("forward",),
            "C3": ("decode",), "C4": ("forward", "backward", "decode")}[w.name]
    seq = "forward" in legs
    B_dec = {"C1": B, "C3": B, "C4": DECODE_BATCH}.get(w.name, 0)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    act_b = 2

    # parameters (seeded); the big activation tensors are drawn set by set below
    par_inp = gen.make_inputs(1, 8, D, nb, act=w.act, seed=w.seed)
    dp = rn.DeviceProblem(par_inp, B, T, D, nb, w.act, device=dev)
    sp = torch.cuda.current_stream().cuda_stream

    # buffer sets: enough of them that consecutive steps do not find their inputs in the
    # last-level cache (one set when a step's own footprint already exceeds it twice over)
    per_set = (4 if "backward" in legs else 2) * act_b * B * T * D if seq else 20 * B_dec * D
    nsets = int(min(16, max(1, -(-2 * LLC_BYTES // per_set))))
    rng = np.random.Generator(np.random.PCG64(w.seed + 100))

    def draw(*shape):   # seeded N(0,1), stored as the activation type
        return rn.to_device(gen.round_to_act(rng.standard_normal(shape, dtype=np.float32), w.act),
                            w.act, dev)

    sets = []
    for i in range(nsets):
        s = {}
        if seq:
            s["u"] = draw(B, T, D)
            s["y"] = dp.empty_act(B, T, D)
            s["hT"] = dp.empty_f32(B, D)
            s["st"] = dp.empty_act(B, 3, D)
            if "backward" in legs:
                s["dy"] = draw(B, T, D)
                s["du"] = dp.empty_act(B, T, D)
        if "decode" in legs:
            s["u_t"] = draw(B_dec, D)
            s["y_t"] = dp.empty_act(B_dec, D)
            if w.name != "C1":   # own states (C1 continues the sequences of its forward call)
                s["h"] = rn.to_device(rng.standard_normal((B_dec, D), dtype=np.float32), "f32", dev)
                s["ring"] = draw(B_dec, 3, D)
        sets.append(s)
    h0 = rn.to_device(rng.standard_normal((B, D), dtype=np.float32), "f32", dev) if (seq and w.h0) else None

    sh = dp.shape()
    sh_dec = dp.shape(T=1, B=B_dec) if B_dec else None
    ws_f, n_f = dp.workspace(sh, R.OP_FORWARD) if seq else (None, 0)
    ws_b, n_b = dp.workspace(sh, R.OP_BACKWARD) if "backward" in legs else (None, 0)
    dh0 = dp.empty_f32(B, D)
    g = dp.alloc_grads()
    pg = R.make_param_grads(g["dW_a"], g["dW_x"], g["db_a"], g["db_x"], g["dLambda"],
                            g["dconv_w"], g["dconv_b"])
    pos_dec = [T if w.name == "C1" else 3]

    def step(k):
        s = sets[k % nsets]
        if seq:
            R.rglru_forward(sh, dp.params, s["u"], h0, None, 0, s["y"], s["hT"], s["st"], ws_f, n_f, sp)
        if "decode" in legs:
            if w.name == "C1":
                R.rglru_decode_step(sh_dec, dp.params, s["u_t"], s["hT"], s["st"], T, s["y_t"], sp)
            else:
                R.rglru_decode_step(sh_dec, dp.params, s["u_t"], s["h"], s["ring"], pos_dec[0], s["y_t"], sp)
                pos_dec[0] += 1
        if "backward" in legs:
            R.rglru_backward(sh, dp.params, s["u"], h0, None, 0, s["y"], s["dy"], None, s["du"], dh0,
                             pg, ws_b, n_b, sp)

    if args.calibration_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)   # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst
    for k in range(args.warmup):
        step(k)
    torch.cuda.synchronize()

    def timed_kernels():
        per = {}
        for i in range(R.rglru_timing_count()):
            name, ms = R.rglru_timing_get(i)
            tot, cnt = per.get(name, (0.0, 0))
            per[name] = (tot + ms, cnt + 1)
        return per

    # Untimed profile pass: every kernel launch bracketed by HIP events on its own stream. It
    # gives the per-kernel table and names the dominant kernel; two event records per launch
    # cost several percent of a step, so this pass does not count towards `value`.
    prof_steps = max(2, min(5, args.steps))
    R.rglru_timing_select(None)
    R.rglru_timing_enable(True)
    for k in range(prof_steps):
        step(k)
    torch.cuda.synchronize()
    R.rglru_timing_enable(False)
    per_kernel = timed_kernels()
    costs = algorithmic_costs(B, T, D, nb, B_dec)
    dominant = max((n for n in per_kernel if n in costs), key=lambda n: per_kernel[n][0])

    # Timed region: exactly `steps` steps; only the dominant kernel is bracketed by events.
    R.rglru_timing_select(dominant)
    R.rglru_timing_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(k)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    R.rglru_timing_enable(False)
    R.rglru_timing_select(None)
    dom_tot, dom_cnt = timed_kernels()[dominant]
    # no bounded wait between workgroups expired during the run (raises otherwise)
    if seq:
        R.rglru_workspace_status(sh, R.OP_FORWARD, ws_f)
    if "backward" in legs:
        R.rglru_workspace_status(sh, R.OP_BACKWARD, ws_b)
    dominant_ms = dom_tot / dom_cnt

    tokens = (B * T if seq else 0) + B_dec
    step_s = elapsed / args.steps
    traffic, traffic_src = read_traffic(w.name)

    def roof(name, t_ms):
        cost = costs[name]
        t_hbm = cost["bytes"] / (HBM_PEAK_GBS * 1e9)
        t_mfma = cost["flops"] / (MFMA_BF16_PEAK_TFLOPS * 1e12)
        r = {"kernel": name, "traffic": traffic.get(name), "traffic_source": traffic_src,
             "algorithmic_bytes": cost["bytes"], "algorithmic_flops": cost["flops"], "avg_ms": t_ms,
             "frac_hbm": t_hbm / (t_ms * 1e-3), "frac_mfma": t_mfma / (t_ms * 1e-3)}
        if t_hbm >= t_mfma:
            ach = cost["bytes"] / (t_ms * 1e-3) / 1e9
            r.update({"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                      "frac": ach / HBM_PEAK_GBS})
        else:
            ach = cost["flops"] / (t_ms * 1e-3) / 1e12
            r.update({"bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS,
                      "unit": "TFLOP/s", "frac": ach / MFMA_BF16_PEAK_TFLOPS})
        return r

    kernels = {n: {"avg_ms": tot / cnt, "launches_per_step": cnt / prof_steps,
                   "ms_per_step": tot / prof_steps} for n, (tot, cnt) in per_kernel.items()}
    roofs = [roof(n, kernels[n]["avg_ms"]) for n in costs if n in kernels]
    # method-level roofs of the whole step: forward 4 B/element, backward 8 B/element, the
    # decode step's own bytes; gate products 4*bs FLOP/element forward, 12*bs backward
    N = B * T * D if seq else 0
    bs = D // nb
    step_bytes = (4 * N if "forward" in legs else 0) + (8 * N if "backward" in legs else 0) + \
                 (costs["decode_mfma_kernel"]["bytes"] if "decode" in legs else 0)
    step_flops = (4 * bs * N if "forward" in legs else 0) + (12 * bs * N if "backward" in legs else 0) + \
                 (4 * bs * B_dec * D if "decode" in legs else 0)
    t_hbm = step_bytes / (HBM_PEAK_GBS * 1e9)
    t_mfma = step_flops / (MFMA_BF16_PEAK_TFLOPS * 1e12)

    out = {
        "metric": "RG-LRU block tokens/sec and achieved HBM GB/s (% of MI355X peak)",
        "value": tokens / step_s,
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * step_s,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.act == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": "%s: B=%d T=%d D=%d nb=%d %s, %s%s"
                               % (w.name, B, T, D, nb, w.act, " + ".join(legs),
                                  (" (decode step at batch %d)" % B_dec) if "decode" in legs and seq else ""),
                   "global_batch": B, "seq_len": T, "buffer_sets": nsets},
        "roofline": roof(dominant, dominant_ms),
        "kernel_rooflines": roofs,
        "kernels": kernels,
        "step_roofs": {"algorithmic_bytes": step_bytes, "algorithmic_flops": step_flops,
                       "hbm_GBs": step_bytes / step_s / 1e9,
                       "frac_hbm_roof": t_hbm / step_s,
                       "frac_mfma_roof": t_mfma / step_s,
                       "frac_of_binding_roof": max(t_hbm, t_mfma) / step_s,
                       "binding_roof": "hbm" if t_hbm >= t_mfma else "mfma"},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, legs)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
