"""Convenience layer for tests, smoke and the benchmark: moves numpy inputs into device
memory with torch (used for allocation and streams only) and calls the C ABI through the
ctypes binding. It performs no arithmetic of the method.
"""
import numpy as np
import torch

import rglru_inputs as gen

from . import binding as R


def _bits_to_bf16_tensor(a_f32, device):
    """float32 numpy values that are exactly representable in bf16 -> torch.bfloat16 tensor."""
    bits = (np.ascontiguousarray(a_f32, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)
    return torch.from_numpy(bits.view(np.int16)).to(device).view(torch.bfloat16)


def to_device(a, act, device="cuda:0"):
    """numpy float32 -> device tensor stored as `act` ("f32" | "bf16"); None passes through."""
    if a is None:
        return None
    if act == "bf16":
        return _bits_to_bf16_tensor(a, device)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)


def to_host(t):
    return None if t is None else t.detach().float().cpu().numpy()


class SeededDraws:
    """Seeded synthetic tensors on the device: numpy PCG64 draws on the host (the generator of
    rglru_inputs), rounded to the storage type and uploaded."""

    def __init__(self, seed, device="cuda:0"):
        self.rng = np.random.Generator(np.random.PCG64(seed))
        self.device = device

    def normal(self, *shape, act="f32"):
        a = self.rng.standard_normal(shape, dtype=np.float32)
        return to_device(gen.round_to_act(a, act) if act != "f32" else a, act, self.device)

    def uniform(self, *shape):
        return to_device(self.rng.random(shape, dtype=np.float32), "f32", self.device)


class DeviceProblem:
    """Device copies of one workload's parameters plus the shape/params structs."""

    def __init__(self, inp, B, T, D, nb, act, device="cuda:0", c=8.0):
        self.B, self.T, self.D, self.nb, self.act, self.device = B, T, D, nb, act, device
        self.dt = R.BF16 if act == "bf16" else R.F32
        self.tdtype = torch.bfloat16 if act == "bf16" else torch.float32
        self.c = c
        self.W_a = to_device(inp["W_a"], act, device)
        self.W_x = to_device(inp["W_x"], act, device)
        self.b_a = to_device(inp["b_a"], "f32", device)
        self.b_x = to_device(inp["b_x"], "f32", device)
        self.Lambda = to_device(inp["Lambda"], "f32", device)
        self.conv_w = to_device(inp["conv_w"], "f32", device)
        self.conv_b = to_device(inp.get("conv_b"), "f32", device)
        self.params = R.make_params(self.W_a, self.W_x, self.b_a, self.b_x, self.Lambda,
                                    self.conv_w, self.conv_b)
        self._ws = {}

    def shape(self, T=None, B=None):
        return R.make_shape(self.B if B is None else B, self.T if T is None else T, self.D,
                            self.nb, self.dt, c=self.c)

    def workspace(self, shape, op):
        n = R.rglru_workspace_bytes(shape, op)
        key = (op, n)
        if key not in self._ws:
            self._ws[key] = torch.empty(max(n, 256), dtype=torch.uint8, device=self.device)
        return self._ws[key], n

    def empty_act(self, *shape):
        return torch.empty(*shape, dtype=self.tdtype, device=self.device)

    def empty_f32(self, *shape):
        return torch.empty(*shape, dtype=torch.float32, device=self.device)

    # ---- one-call helpers (allocate outputs, call the library, leave results on device)
    def conv1d(self, u, state_in=None, pos0=0, want_state=True):
        B, T, D = u.shape
        sh = self.shape(T=T, B=B)
        x = self.empty_act(B, T, D)
        st = self.empty_act(B, 3, D) if want_state else None
        R.rglru_conv1d(sh, u, self.conv_w, self.conv_b, state_in, pos0, x, st)
        return x, st

    def forward(self, u, h0=None, state_in=None, pos0=0, want_state=True, stream=None):
        B, T, D = u.shape
        sh = self.shape(T=T, B=B)
        ws, n = self.workspace(sh, R.OP_FORWARD)
        y = self.empty_act(B, T, D)
        hT = self.empty_f32(B, D)
        st = self.empty_act(B, 3, D) if want_state else None
        R.rglru_forward(sh, self.params, u, h0, state_in, pos0, y, hT, st, ws, n, stream)
        return y, hT, st

    def forward_packed(self, u, reset, h0=None, state_in=None, pos0=0, stream=None):
        """reset: uint8 device tensor [B,T], non-zero where a document starts."""
        B, T, D = u.shape
        sh = self.shape(T=T, B=B)
        y = self.empty_act(B, T, D)
        hT = self.empty_f32(B, D)
        st = self.empty_act(B, 3, D)
        ws, n = self.workspace(sh, R.OP_FORWARD_PACKED)
        R.rglru_forward_packed(sh, self.params, u, reset, h0, state_in, pos0, y, hT, st, ws, n, stream)
        return y, hT, st

    def backward_packed(self, u, reset, y, dy, h0=None, state_in=None, pos0=0, dhT=None,
                        stream=None):
        B, T, D = u.shape
        sh = self.shape(T=T, B=B)
        ws, n = self.workspace(sh, R.OP_BACKWARD_PACKED)
        du = self.empty_act(B, T, D)
        dh0 = self.empty_f32(B, D)
        g = self.alloc_grads()
        pg = R.make_param_grads(g["dW_a"], g["dW_x"], g["db_a"], g["db_x"], g["dLambda"],
                                g["dconv_w"], g["dconv_b"])
        R.rglru_backward_packed(sh, self.params, u, reset, h0, state_in, pos0, y, dy, dhT, du,
                                dh0, pg, ws, n, stream)
        out = dict(g)
        out["du"], out["dh0"] = du, dh0
        return out

    def forward_merge(self, u, branch, h0=None, state_in=None, pos0=0, flags=0, keep_y=True,
                      stream=None):
        B, T, D = u.shape
        sh = self.shape(T=T, B=B)
        ws, n = self.workspace(sh, R.OP_FORWARD_MERGE)
        out = self.empty_act(B, T, D)
        y = self.empty_act(B, T, D) if keep_y else None
        hT = self.empty_f32(B, D)
        st = self.empty_act(B, 3, D)
        R.rglru_forward_merge(sh, self.params, u, branch, h0, state_in, pos0, flags, out, y, hT, st,
                              ws, n, stream)
        return out, y, hT, st

    def decode_step(self, u_t, h, conv_state, pos, stream=None):
        B, D = u_t.shape
        sh = self.shape(T=1, B=B)
        y = self.empty_act(B, D)
        R.rglru_decode_step(sh, self.params, u_t, h, conv_state, pos, y, stream)
        return y

    def decode_step_at(self, u_t, h, conv_state, pos, stream=None):
        """pos: int64 device tensor [B], a position per sequence."""
        B, D = u_t.shape
        sh = self.shape(T=1, B=B)
        y = self.empty_act(B, D)
        R.rglru_decode_step_at(sh, self.params, u_t, h, conv_state, pos, y, stream)
        return y

    def decode_step_merge(self, u_t, branch_t, h, conv_state, pos, flags=0, stream=None):
        B, D = u_t.shape
        sh = self.shape(T=1, B=B)
        out = self.empty_act(B, D)
        R.rglru_decode_step_merge(sh, self.params, u_t, branch_t, h, conv_state, pos, flags, out,
                                  stream)
        return out

    def alloc_grads(self):
        bs = self.D // self.nb
        g = dict(dW_a=self.empty_f32(self.nb, bs, bs), dW_x=self.empty_f32(self.nb, bs, bs),
                 db_a=self.empty_f32(self.D), db_x=self.empty_f32(self.D),
                 dLambda=self.empty_f32(self.D), dconv_w=self.empty_f32(4, self.D),
                 dconv_b=self.empty_f32(self.D))
        return g

    def backward(self, u, y, dy, h0=None, state_in=None, pos0=0, dhT=None, grads=None,
                 stream=None):
        B, T, D = u.shape
        sh = self.shape(T=T, B=B)
        ws, n = self.workspace(sh, R.OP_BACKWARD)
        du = self.empty_act(B, T, D)
        dh0 = self.empty_f32(B, D)
        g = grads if grads is not None else self.alloc_grads()
        pg = R.make_param_grads(g["dW_a"], g["dW_x"], g["db_a"], g["db_x"], g["dLambda"],
                                g["dconv_w"], g["dconv_b"])
        R.rglru_backward(sh, self.params, u, h0, state_in, pos0, y, dy, dhT, du, dh0, pg, ws, n,
                         stream)
        out = dict(g)
        out["du"], out["dh0"] = du, dh0
        return out


    def backward_merge(self, u, branch, y, dout, h0=None, state_in=None, pos0=0, dhT=None, flags=0,
                       grads=None, stream=None):
        B, T, D = u.shape
        sh = self.shape(T=T, B=B)
        ws, n = self.workspace(sh, R.OP_BACKWARD_MERGE)
        du = self.empty_act(B, T, D)
        dbranch = self.empty_act(B, T, D)
        dh0 = self.empty_f32(B, D)
        g = grads if grads is not None else self.alloc_grads()
        pg = R.make_param_grads(g["dW_a"], g["dW_x"], g["db_a"], g["db_x"], g["dLambda"],
                                g["dconv_w"], g["dconv_b"])
        R.rglru_backward_merge(sh, self.params, u, branch, h0, state_in, pos0, flags, y, dout, dhT,
                               du, dbranch, dh0, pg, ws, n, stream)
        out = dict(g)
        out["du"], out["dbranch"], out["dh0"] = du, dbranch, dh0
        return out


class CgDeviceProblem:
    """Device copies of a complex-gated layer's parameters (Appendix B) and one-call helpers."""

    def __init__(self, inp, B, T, D, nb, act, device="cuda:0", c=8.0, conv=True):
        self.B, self.T, self.D, self.nb, self.act, self.device, self.c = B, T, D, nb, act, device, c
        self.dt = R.BF16 if act == "bf16" else R.F32
        self.tdtype = torch.bfloat16 if act == "bf16" else torch.float32
        self.conv = conv
        self.t = {k: to_device(inp[k], act if k in ("W_a", "W_x") else "f32", device)
                  for k in ("W_a", "W_x", "b_a", "b_x", "Lambda", "theta", "conv_w", "conv_b")
                  if inp.get(k) is not None}
        self.params = R.make_cg_params(self.t["W_a"], self.t["W_x"], self.t["b_a"], self.t["b_x"],
                                       self.t["Lambda"], self.t["theta"],
                                       self.t["conv_w"] if conv else None,
                                       self.t.get("conv_b") if conv else None)

    def shape(self, T=None, B=None):
        return R.make_shape(self.B if B is None else B, self.T if T is None else T, self.D, self.nb,
                            self.dt, c=self.c, conv_width=4 if self.conv else 0)

    def forward(self, u, h0=None, state_in=None, pos0=0, stream=None, scratch=True):
        """scratch: bring the optional workspace (two passes parallel over time) or not (one pass)."""
        B, T, D = u.shape
        y = torch.empty(B, T, D, dtype=self.tdtype, device=self.device)
        hT = torch.empty(B, D, dtype=torch.float32, device=self.device)
        st = torch.empty(B, 3, D, dtype=self.tdtype, device=self.device) if self.conv else None
        sh = self.shape(T=T, B=B)
        n = R.rglru_workspace_bytes(sh, R.OP_CG_FORWARD) if scratch else 0
        ws = torch.empty(n, dtype=torch.uint8, device=self.device) if n else None
        R.rglru_cg_forward(sh, self.params, u, h0, state_in, pos0, y, hT, st, ws, n, stream)
        return y, hT, st

    def decode_step(self, u_t, h, conv_state, pos, stream=None):
        B, D = u_t.shape
        y = torch.empty(B, D, dtype=self.tdtype, device=self.device)
        R.rglru_cg_decode_step(self.shape(T=1, B=B), self.params, u_t, h, conv_state, pos, y, stream)
        return y

    def backward(self, u, dy, h0=None, state_in=None, pos0=0, dhT=None, stream=None):
        B, T, D = u.shape
        H, hs = D // 2, D // 2 // self.nb
        f32 = lambda *s: torch.empty(*s, dtype=torch.float32, device=self.device)
        g = dict(dW_a=f32(self.nb, hs, 2 * hs), dW_x=f32(self.nb, hs, 2 * hs), db_a=f32(H), db_x=f32(H),
                 dLambda=f32(H), dtheta=f32(H))
        if self.conv:
            g["dconv_w"], g["dconv_b"] = f32(4, D), f32(D)
        pg = R.make_cg_param_grads(g["dW_a"], g["dW_x"], g["db_a"], g["db_x"], g["dLambda"], g["dtheta"],
                                   g.get("dconv_w"), g.get("dconv_b"))
        sh = self.shape(T=T, B=B)
        n = R.rglru_workspace_bytes(sh, R.OP_CG_BACKWARD)
        ws = torch.empty(max(n, 256), dtype=torch.uint8, device=self.device)
        du = torch.empty(B, T, D, dtype=self.tdtype, device=self.device)
        dh0 = f32(B, D)
        R.rglru_cg_backward(sh, self.params, u, h0, state_in, pos0, dy, dhT, du, dh0, pg, ws, n, stream)
        g["du"], g["dh0"] = du, dh0
        return g


def scan(a, g, h0=None, flags=0, act="bf16", device="cuda:0", stream=None):
    """rglru_scan on device tensors a, g [B,T,D] (dtype of `act`); returns h, hT."""
    B, T, D = a.shape
    dt = R.BF16 if act == "bf16" else R.F32
    sh = R.make_shape(B, T, D, 1, dt)
    n = R.rglru_workspace_bytes(sh, R.OP_SCAN)
    ws = torch.empty(max(n, 256), dtype=torch.uint8, device=device)
    h = torch.empty_like(a)
    hT = torch.empty(B, D, dtype=torch.float32, device=device)
    R.rglru_scan(sh, a, g, h0, flags, h, hT, ws, n, stream)
    return h, hT
