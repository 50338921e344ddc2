"""Seeded synthetic inputs for the Conv1D -> RG-LRU path.

This module serves both the HIP library's tests/benchmark and the CPU oracle and
therefore holds NONE of the method's arithmetic: only random draws, the paper's
initialisation recipe (Section 2.4: LeCun-normal gate weights, Lambda such that
sigmoid(Lambda)^8 is uniform in [0.9, 0.999]), bf16 storage conversion and the
error metric used by the parity tests.

The tensors take the shapes of the paper's own workloads (RNN widths 2560 and
4096 from the model-scale table of Appendix C, training length 2048, longest
evaluation length 32768) and stand in for activations of a trained model, which
are not available.

Draw order for a workload (numpy PCG64, seed = 1000 + config index):
u, W_a, W_x, conv_w, Lambda-uniforms, h0, dy, conv state, decode tokens.
"""
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    index: int
    B: int
    T: int
    D: int
    nb: int
    act: str          # "f32" or "bf16": dtype of u / y / dy / du / conv state / W
    h0: bool          # random nonzero initial state
    kind: str         # "forward", "decode", "train"

    @property
    def bs(self):
        return self.D // self.nb

    @property
    def seed(self):
        return 1000 + self.index


# The five workloads named by the build's baseline description.
CONFIGS = {
    "C0": Workload("C0", 0, B=1, T=256, D=256, nb=4, act="f32", h0=False, kind="forward"),
    "C1": Workload("C1", 1, B=8, T=2048, D=2560, nb=10, act="bf16", h0=False, kind="forward"),
    "C2": Workload("C2", 2, B=1, T=32768, D=2560, nb=10, act="bf16", h0=True, kind="forward"),
    "C3": Workload("C3", 3, B=256, T=1, D=4096, nb=16, act="bf16", h0=True, kind="decode"),
    "C4": Workload("C4", 4, B=16, T=4096, D=4096, nb=16, act="bf16", h0=False, kind="train"),
}

CONV_WIDTH = 4
C_CONST = 8.0


# ---------------------------------------------------------------- bf16 storage
def f32_to_bf16_bits(a):
    """Round float32 to bfloat16 (round-to-nearest-even); returns uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32)
    rounded = bits + (np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1)))
    out = (rounded >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(a)
    if nan.any():
        out[nan] = np.uint16(0x7FC0)
    return out


def bf16_bits_to_f32(b):
    """Exact widening of bfloat16 bit patterns (uint16) to float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_act(a, act):
    """The float32 values a tensor holds once stored in dtype `act`."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return bf16_bits_to_f32(f32_to_bf16_bits(a)) if act == "bf16" else a


# -------------------------------------------------------------------- generator
def make_lambda(rng, D):
    """Lambda with sigmoid(Lambda)^8 ~ U[0.9, 0.999] (Section 2.4 initialisation)."""
    v = rng.uniform(0.9, 0.999, size=D)
    return (-np.log(v ** (-1.0 / C_CONST) - 1.0)).astype(np.float32)


def make_inputs(B, T, D, nb, act="bf16", seed=0, h0=False, dy=False, state=False,
                decode_tokens=0, bias=False):
    """Seeded tensors for one workload. All values are float32 arrays that are exactly
    representable in their storage dtype (bf16-rounded when act == "bf16").

    Returns a dict: u [B,T,D], W_a/W_x [nb,bs,bs], b_a/b_x/Lambda [D], conv_w [4,D],
    h0 [B,D] or None, dy [B,T,D] or None, dhT [B,D] or None,
    state [B,3,D] chronological or None, u_dec [decode_tokens,B,D] or None.
    Biases are zero unless bias=True (then small normal draws, made after everything else).
    """
    assert D % nb == 0
    bs = D // nb
    rng = np.random.Generator(np.random.PCG64(seed))
    nrm = lambda *shape: rng.standard_normal(shape, dtype=np.float32)
    out = {}
    out["u"] = round_to_act(nrm(B, T, D), act)
    scale = np.float32(1.0 / np.sqrt(bs))
    out["W_a"] = round_to_act(nrm(nb, bs, bs) * scale, act)
    out["W_x"] = round_to_act(nrm(nb, bs, bs) * scale, act)
    out["conv_w"] = nrm(CONV_WIDTH, D) * np.float32(0.5)
    out["Lambda"] = make_lambda(rng, D)
    out["h0"] = nrm(B, D) if h0 else None
    out["dy"] = round_to_act(nrm(B, T, D), act) if dy else None
    out["dhT"] = nrm(B, D) if dy else None
    out["state"] = round_to_act(nrm(B, CONV_WIDTH - 1, D), act) if state else None
    out["u_dec"] = round_to_act(nrm(decode_tokens, B, D), act) if decode_tokens else None
    if bias:
        out["b_a"] = nrm(D) * np.float32(0.5)
        out["b_x"] = nrm(D) * np.float32(0.5)
        out["conv_b"] = nrm(D) * np.float32(0.1)
    else:
        out["b_a"] = np.zeros(D, np.float32)
        out["b_x"] = np.zeros(D, np.float32)
        out["conv_b"] = None
    return out


def make_cg_inputs(B, T, D, nb, act="bf16", seed=0, h0=False, dy=False, state=False,
                   decode_tokens=0, bias=False):
    """Seeded tensors for the complex-gated variant (Appendix B): D real channels, H = D/2
    complex ones, gate weights [nb, hs, 2 hs] with hs = H / nb (LeCun normal over the 2 hs
    inputs of a block), b_a / b_x / Lambda / theta [H]. Lambda as for the real layer. The
    appendix gives no initialisation for theta: it is drawn uniform in [0, pi/10] (small
    phases, the choice of the LRU paper the appendix builds on). Everything else as make_inputs."""
    assert D % 2 == 0 and (D // 2) % nb == 0
    H = D // 2
    hs = H // nb
    rng = np.random.Generator(np.random.PCG64(seed))
    nrm = lambda *shape: rng.standard_normal(shape, dtype=np.float32)
    out = {}
    out["u"] = round_to_act(nrm(B, T, D), act)
    scale = np.float32(1.0 / np.sqrt(2 * hs))
    out["W_a"] = round_to_act(nrm(nb, hs, 2 * hs) * scale, act)
    out["W_x"] = round_to_act(nrm(nb, hs, 2 * hs) * scale, act)
    out["conv_w"] = nrm(CONV_WIDTH, D) * np.float32(0.5)
    out["Lambda"] = make_lambda(rng, H)
    out["theta"] = rng.uniform(0.0, np.pi / 10, size=H).astype(np.float32)
    out["h0"] = nrm(B, D) if h0 else None
    out["dy"] = round_to_act(nrm(B, T, D), act) if dy else None
    out["dhT"] = nrm(B, D) if dy else None
    out["state"] = round_to_act(nrm(B, CONV_WIDTH - 1, D), act) if state else None
    out["u_dec"] = round_to_act(nrm(decode_tokens, B, D), act) if decode_tokens else None
    if bias:
        out["b_a"] = nrm(H) * np.float32(0.5)
        out["b_x"] = nrm(H) * np.float32(0.5)
        out["conv_b"] = nrm(D) * np.float32(0.1)
    else:
        out["b_a"] = np.zeros(H, np.float32)
        out["b_x"] = np.zeros(H, np.float32)
        out["conv_b"] = None
    return out


def make_scan_inputs(B, T, D, act="bf16", seed=0, log_a=False, h0=True):
    """Seeded inputs of the scan-only entry point: decays distributed like the layer's own
    (a base decay per channel with base^8 ~ U[0.9, 0.999], raised to a per-element power in
    (0, 8)), stored as a_t or as log a_t; gated inputs ~ N(0, 1); h0 ~ N(0, 1).
    Returns a dict of float32 arrays, a / g exactly representable in dtype `act`."""
    rng = np.random.Generator(np.random.PCG64(seed))
    base = rng.uniform(0.9, 0.999, size=D) ** (1.0 / C_CONST)
    power = C_CONST * rng.uniform(0.0, 1.0, size=(B, T, D))
    log_decay = power * np.log(base)
    a = log_decay if log_a else np.exp(log_decay)
    out = {"a": round_to_act(a.astype(np.float32), act),
           "g": round_to_act(rng.standard_normal((B, T, D), dtype=np.float32), act),
           "h0": rng.standard_normal((B, D), dtype=np.float32) if h0 else None}
    return out


def make_branch(B, T, D, act="bf16", seed=0):
    """Seeded stand-in for the recurrent block's second branch before its GeLU (the output of a
    linear layer on a normalised input): N(0, 1) values, exactly representable in `act`.
    Returns float32 [B,T,D]."""
    rng = np.random.Generator(np.random.PCG64(seed + 7919))
    return round_to_act(rng.standard_normal((B, T, D), dtype=np.float32), act)


def make_resets(B, T, seed=0, mean_len=64):
    """Document-boundary mask [B,T] uint8 for packed sequences: non-zero where a document
    starts. Document lengths are geometric with mean `mean_len` (at least one step), the length
    mix of short and long documents packed into fixed-length training rows; row b starts a
    document at step 0 when b is odd (even rows continue a document carried in through h0 and
    the conv state). Row 0 additionally gets a one-step document and a boundary at the very
    last step where they fit."""
    rng = np.random.Generator(np.random.PCG64(5000 + seed))
    m = np.zeros((B, T), np.uint8)
    for b in range(B):
        t = 0 if b % 2 == 1 else int(rng.geometric(1.0 / mean_len))
        while t < T:
            m[b, t] = 1
            t += int(rng.geometric(1.0 / mean_len))
    if T >= 8:
        m[0, 4] = m[0, 5] = 1
        m[0, T - 1] = 1
    return m


def make_workload(name, **override):
    """Inputs of one of the named workloads C0..C4 (sizes may be overridden for sampling)."""
    w = CONFIGS[name]
    kw = dict(B=w.B, T=w.T, D=w.D, nb=w.nb, act=w.act, seed=w.seed, h0=w.h0,
              dy=(w.kind == "train"), state=(w.kind == "decode"),
              decode_tokens=(8 if w.kind == "decode" else 0))
    kw.update(override)
    return make_inputs(**kw)


# ------------------------------------------------------------------ state layout
def ring_from_chrono(state, pos):
    """[B,3,D] chronological rows (oldest first = tokens pos-3, pos-2, pos-1) -> ring layout
    where the token at absolute position n sits in slot n mod 3."""
    S = state.shape[1]
    ring = np.empty_like(state)
    for r in range(S):
        n = pos - S + r
        ring[:, n % S, :] = state[:, r, :]
    return ring


def chrono_from_ring(ring, pos):
    """Inverse of ring_from_chrono for a stream that has consumed `pos` tokens."""
    S = ring.shape[1]
    st = np.empty_like(ring)
    for r in range(S):
        n = pos - S + r
        st[:, r, :] = ring[:, n % S, :]
    return st


# -------------------------------------------------------------------- error metric
def rel_err(got, want):
    """max_i |got_i - want_i| / (|want_i| + rms(want)): relative error with a scale floor,
    so that elements near zero do not dominate."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    if want.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(want * want)))
    if rms == 0.0:
        rms = 1.0
    return float(np.max(np.abs(got - want) / (np.abs(want) + rms)))
