"""Host-side checks of the measurement code: the algorithmic byte and FLOP counts that the
benchmark and the workload report divide by are fixed by the method (every input read once,
every output written once, weights once), so they are pinned here to hand-computed figures."""
import importlib
import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import rglru_inputs as gen


def test_workload_report_algorithmic_bytes():
    wl = importlib.import_module("paper_2402_19427_amd.workloads")
    c1, c2, c3, c4 = (gen.CONFIGS[k] for k in ("C1", "C2", "C3", "C4"))
    # forward: u in + y out (2 B each) + both gate matrices (bf16) + vectors + h_T + conv state
    n1 = c1.B * c1.T * c1.D
    assert n1 == 41_943_040
    fwd1 = wl.alg_bytes("forward", c1.B, c1.T, c1.D, c1.nb, 2)
    assert fwd1 == 4 * n1 + 2 * 10 * 256 * 256 * 2 + 8 * 2560 * 4 + (4 + 6) * 8 * 2560
    assert abs(fwd1 / 1e6 - 170.7) < 0.5
    fwd2 = wl.alg_bytes("forward", c2.B, c2.T, c2.D, c2.nb, 2)
    assert abs(fwd2 / 1e6 - 338.2) < 0.5
    # decode: u_t 2 + three ring slots read 6 + one written 2 + h read and written 8 + y_t 2
    dec = wl.alg_bytes("decode", c3.B, 1, c3.D, c3.nb, 2)
    assert dec == 20 * 256 * 4096 + 2 * 16 * 256 * 256 * 2 + 8 * 4096 * 4
    assert abs(dec / 1e6 - 25.3) < 0.1
    # backward: u, y, dy in and du out (2 B each) + dW_a, dW_x out in fp32 + weights in
    n4 = c4.B * c4.T * c4.D
    bwd4 = wl.alg_bytes("backward", c4.B, c4.T, c4.D, c4.nb, 2)
    assert abs(bwd4 / 1e9 - (8 * n4 + 8.4e6 + 4.2e6) / 1e9) < 0.001
    # gate products: two [rows x bs] x [bs x bs] products forward, three times that backward
    assert wl.gate_flops("forward", c1.B, c1.T, c1.D, c1.nb) == 1024 * n1
    assert wl.gate_flops("backward", c4.B, c4.T, c4.D, c4.nb) == 3072 * n4
    assert wl.gate_flops("decode", c3.B, 1, c3.D, c3.nb) == 1024 * 256 * 4096
    # with the block's merge: the other branch in (forward), y kept on top of out (training),
    # the branch in and its gradient out (backward); one more [B][D] row per decode step
    assert wl.alg_bytes("forward_merge", c1.B, c1.T, c1.D, c1.nb, 2) == fwd1 + 2 * n1
    assert wl.alg_bytes("forward_merge_keep", c1.B, c1.T, c1.D, c1.nb, 2) == fwd1 + 4 * n1
    assert wl.alg_bytes("backward_merge", c4.B, c4.T, c4.D, c4.nb, 2) == bwd4 + 4 * n4
    assert wl.alg_bytes("decode_merge", c3.B, 1, c3.D, c3.nb, 2) == dec + 2 * 256 * 4096
    assert wl.gate_flops("forward_merge", c1.B, c1.T, c1.D, c1.nb) == 1024 * n1


def test_bench_costs_and_single_gpu_contract():
    bench = importlib.import_module("bench")
    c1 = gen.CONFIGS["C1"]
    n = c1.B * c1.T * c1.D
    costs = bench.algorithmic_costs(c1.B, c1.T, c1.D, c1.nb, c1.B)
    assert costs["fwd_mfma_kernel"]["flops"] == 1024 * n
    assert abs(costs["fwd_mfma_kernel"]["bytes"] / 1e6 - 170.7) < 0.5
    assert costs["bwd_gates_kernel"]["bytes"] >= 6 * n          # u, y, dy
    assert costs["bwd_dgrad_kernel"]["bytes"] >= 4 * n          # u in, du out
    assert costs["bwd_wgrad_kernel"]["bytes"] == 2 * 10 * 256 * 256 * 4
    # the default workload is the largest one, with the decode leg at the decode workload's batch
    c4, c3 = gen.CONFIGS["C4"], gen.CONFIGS["C3"]
    assert bench.DECODE_BATCH == c3.B
    big = bench.algorithmic_costs(c4.B, c4.T, c4.D, c4.nb, c3.B)
    assert abs(big["decode_mfma_kernel"]["bytes"] / 1e6 - 25.3) < 0.1
    assert big["bwd_gates_kernel"]["flops"] == 1024 * c4.B * c4.T * c4.D
    # more than one GPU is refused with a message
    argv = sys.argv
    sys.argv = ["bench.py", "--gpus", "2"]
    try:
        with pytest.raises(SystemExit) as e:
            bench.main()
        assert "ONE GPU" in str(e.value)
    finally:
        sys.argv = argv
