"""Float64 CPU oracle for the Conv1D -> RG-LRU path (test infrastructure).

This package wraps ``rglru_oracle.c`` (plain sequential double-precision loops
written from Sections 2.3-2.4 and Appendix A of the Griffin/Hawk paper) with
numpy marshalling.  It shares no code with the HIP library and imports nothing
from it.  Only the test suite, the smoke check and the benchmark's
``cpu_baseline`` leg may import it; the product path never does.

Every function takes and returns float64 numpy arrays in the layouts given at
the top of ``rglru_oracle.c``.  The complex-gated variant of Appendix B lives in
``cglru.py`` (plain numpy, complex128) and is re-exported here.
"""
import ctypes
import os
import subprocess

import numpy as np

from .cglru import cg_backward, cg_decode_step, cg_forward, cg_gates, cg_lru  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rglru_oracle.c")
_LIB = os.path.join(_HERE, "librglru_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with gcc (-O2, no fast-math, OpenMP for the timing leg)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    tmp = _LIB + ".tmp%d" % os.getpid()
    subprocess.check_call(
        ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-o", tmp, _SRC, "-lm"])
    os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_max_threads.restype = ctypes.c_int
        _lib.oracle_set_threads(1)  # canonical parity order: one thread
    return _lib


def _p(a):
    """double* for a C-contiguous float64 array, or NULL for None."""
    if a is None:
        return ctypes.c_void_p(0)
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.c_void_p)


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def _mask(reset, B, T):
    """unsigned char* for a document-boundary mask [B,T] (non-zero: a new document starts at
    that step), or NULL for None. Returns (keep-alive array, pointer)."""
    if reset is None:
        return None, ctypes.c_void_p(0)
    m = np.ascontiguousarray(np.asarray(reset) != 0, dtype=np.uint8)
    assert m.shape == (B, T)
    return m, m.ctypes.data_as(ctypes.c_void_p)


def set_threads(n):
    """Threads for the (batch, gate-block) loop; 1 is the canonical order."""
    _load().oracle_set_threads(int(n))


def max_threads():
    return int(_load().oracle_max_threads())


def conv1d(u, conv_w, conv_b=None, state_in=None, want_state=False, reset=None):
    """Causal separable Conv1D (Section 2.3). u [B,T,D], conv_w [K,D] lag-indexed.

    state_in / returned state: [B,K-1,D] chronological (row 0 oldest).
    """
    u, conv_w, conv_b, state_in = _f64(u), _f64(conv_w), _f64(conv_b), _f64(state_in)
    B, T, D = u.shape
    K = conv_w.shape[0]
    assert conv_w.shape == (K, D)
    x = np.empty((B, T, D))
    st = np.empty((B, K - 1, D)) if want_state else None
    keep, mp = _mask(reset, B, T)
    _load().oracle_conv1d(B, T, D, K, _p(u), _p(conv_w), _p(conv_b), _p(state_in), _p(x), _p(st), mp)
    return (x, st) if want_state else x


def rglru(x, W_a, W_x, b_a, b_x, Lambda, h0=None, c=8.0, want_gates=False, reset=None):
    """RG-LRU eqs. (1)-(4) on convolved input x [B,T,D]; W [nb,bs,bs]. Returns y, hT[, gates]."""
    x, W_a, W_x, b_a, b_x, Lambda, h0 = map(_f64, (x, W_a, W_x, b_a, b_x, Lambda, h0))
    B, T, D = x.shape
    nb, bs, _ = W_a.shape
    assert nb * bs == D and W_a.shape == W_x.shape == (nb, bs, bs)
    y = np.empty((B, T, D))
    hT = np.empty((B, D))
    g = [np.empty((B, T, D)) for _ in range(4)] if want_gates else [None] * 4
    _load().oracle_rglru(B, T, D, nb, ctypes.c_double(c), _p(x), _p(W_a), _p(W_x), _p(b_a),
                         _p(b_x), _p(Lambda), _p(h0), _p(y), _p(hT), *map(_p, g),
                         (_keep := _mask(reset, B, T))[1])
    if T == 0:
        hT[...] = 0.0 if h0 is None else h0
    if want_gates:
        return y, hT, dict(r=g[0], i=g[1], a=g[2], m=g[3])
    return y, hT


def scan(a, g, h0=None, a_is_log=False, normalize=True):
    """Eq. (4) alone as a linear scan (Section 4.2): h_t = a_t h_{t-1} + m_t g_t with
    m_t = sqrt(1 - a_t^2) (normalize) or 1. ``a`` holds a_t, or log a_t when a_is_log.
    a, g [B,T,D]; h0 [B,D] or None. Returns h [B,T,D], hT [B,D]."""
    a, g, h0 = map(_f64, (a, g, h0))
    B, T, D = a.shape
    assert g.shape == (B, T, D) and (h0 is None or h0.shape == (B, D))
    h = np.empty((B, T, D))
    hT = np.empty((B, D))
    _load().oracle_scan(B, T, D, int(bool(a_is_log)), int(bool(normalize)), _p(a), _p(g), _p(h0),
                        _p(h), _p(hT))
    return h, hT


def scan_adjoint(a, dy, dhT=None, a_is_log=False):
    """Adjoint of the unscaled scan h_t = a_t h_{t-1} + b_t: delta_t = dy_t + a_{t+1} delta_{t+1}
    (delta_{T-1} = dy_{T-1} + dhT). Returns delta [B,T,D] (= dL/db) and dh0 = a_0 delta_0 [B,D]."""
    a, dy, dhT = map(_f64, (a, dy, dhT))
    B, T, D = a.shape
    assert dy.shape == (B, T, D) and (dhT is None or dhT.shape == (B, D))
    delta = np.empty((B, T, D))
    dh0 = np.empty((B, D))
    _load().oracle_scan_adjoint(B, T, D, int(bool(a_is_log)), _p(a), _p(dy), _p(dhT), _p(delta), _p(dh0))
    if T == 0:
        dh0[...] = 0.0 if dhT is None else dhT
    return delta, dh0


def gelu(z, approx=False):
    """GeLU(z) = z Phi(z) (Section 2.3's non-linearity); approx selects the tanh form."""
    lib = _load()
    lib.oracle_gelu.restype = ctypes.c_double
    z = np.asarray(z, dtype=np.float64)
    return np.array([lib.oracle_gelu(ctypes.c_double(v), int(bool(approx))) for v in z.ravel()]
                    ).reshape(z.shape)


def gelu_grad(z, approx=False):
    lib = _load()
    lib.oracle_gelu_grad.restype = ctypes.c_double
    z = np.asarray(z, dtype=np.float64)
    return np.array([lib.oracle_gelu_grad(ctypes.c_double(v), int(bool(approx)))
                     for v in z.ravel()]).reshape(z.shape)


def merge(y, branch, approx=False):
    """The recurrent block's merge (Section 2.3): out = y * GeLU(branch), element by element."""
    y, branch = _f64(y), _f64(branch)
    assert y.shape == branch.shape
    out = np.empty(y.shape)
    _load().oracle_merge(ctypes.c_size_t(y.size), int(bool(approx)), _p(y), _p(branch), _p(out))
    return out


def merge_backward(y, branch, dout, approx=False):
    """Adjoint of ``merge``: returns dy, dbranch."""
    y, branch, dout = _f64(y), _f64(branch), _f64(dout)
    assert y.shape == branch.shape == dout.shape
    dy, dbranch = np.empty(y.shape), np.empty(y.shape)
    _load().oracle_merge_backward(ctypes.c_size_t(y.size), int(bool(approx)), _p(y), _p(branch),
                                  _p(dout), _p(dy), _p(dbranch))
    return dy, dbranch


def forward_merge(u, branch, W_a, W_x, b_a, b_x, Lambda, conv_w, conv_b=None, h0=None,
                  state_in=None, c=8.0, approx=False):
    """Conv1D -> RG-LRU -> merge with the other branch. Returns out, y, hT, state_out."""
    y, hT, st = forward(u, W_a, W_x, b_a, b_x, Lambda, conv_w, conv_b, h0, state_in, c)
    return merge(y, branch, approx), y, hT, st


def backward_merge(u, branch, W_a, W_x, b_a, b_x, Lambda, conv_w, dout, conv_b=None, h0=None,
                   state_in=None, dhT=None, c=8.0, approx=False):
    """Adjoint of ``forward_merge`` for L = sum(dout*out) + sum(dhT*hT): the dict of
    ``backward`` plus ``dbranch``."""
    y, _, _ = forward(u, W_a, W_x, b_a, b_x, Lambda, conv_w, conv_b, h0, state_in, c)
    dy, dbranch = merge_backward(y, branch, dout, approx)
    out = backward(u, W_a, W_x, b_a, b_x, Lambda, conv_w, dy, conv_b, h0, state_in, dhT, c)
    out["dbranch"] = dbranch
    return out


def forward(u, W_a, W_x, b_a, b_x, Lambda, conv_w, conv_b=None, h0=None, state_in=None, c=8.0,
            reset=None):
    """Conv1D then RG-LRU. Returns y [B,T,D], hT [B,D], state_out [B,K-1,D] (chronological)."""
    u, W_a, W_x, b_a, b_x, Lambda, conv_w, conv_b, h0, state_in = map(
        _f64, (u, W_a, W_x, b_a, b_x, Lambda, conv_w, conv_b, h0, state_in))
    B, T, D = u.shape
    nb, bs, _ = W_a.shape
    K = conv_w.shape[0]
    assert nb * bs == D
    y = np.empty((B, T, D))
    hT = np.empty((B, D))
    st = np.empty((B, K - 1, D))
    _load().oracle_forward(B, T, D, nb, K, ctypes.c_double(c), _p(u), _p(W_a), _p(W_x), _p(b_a),
                           _p(b_x), _p(Lambda), _p(conv_w), _p(conv_b), _p(h0), _p(state_in),
                           _p(y), _p(hT), _p(st), (_keep := _mask(reset, B, T))[1])
    if T == 0:
        hT[...] = 0.0 if h0 is None else h0
    return y, hT, st


def decode_step(u_t, W_a, W_x, b_a, b_x, Lambda, conv_w, h, state, conv_b=None, c=8.0):
    """One token per sequence. u_t [B,D]; h [B,D] and state [B,K-1,D] (chronological) are
    float64 arrays UPDATED IN PLACE. Returns y_t [B,D]."""
    u_t, W_a, W_x, b_a, b_x, Lambda, conv_w, conv_b = map(
        _f64, (u_t, W_a, W_x, b_a, b_x, Lambda, conv_w, conv_b))
    assert h.dtype == np.float64 and state.dtype == np.float64
    B, D = u_t.shape
    nb, bs, _ = W_a.shape
    K = conv_w.shape[0]
    assert state.shape == (B, K - 1, D) and h.shape == (B, D)
    y = np.empty((B, D))
    _load().oracle_decode_step(B, D, nb, K, ctypes.c_double(c), _p(u_t), _p(W_a), _p(W_x),
                               _p(b_a), _p(b_x), _p(Lambda), _p(conv_w), _p(conv_b), _p(h),
                               _p(state), _p(y))
    return y


def backward(u, W_a, W_x, b_a, b_x, Lambda, conv_w, dy, conv_b=None, h0=None, state_in=None,
             dhT=None, c=8.0, reset=None):
    """Adjoint of ``forward`` for L = sum(dy*y) + sum(dhT*hT). Returns a dict of float64 grads:
    du, dh0, dW_a, dW_x, db_a, db_x, dLambda, dconv_w, dconv_b."""
    u, W_a, W_x, b_a, b_x, Lambda, conv_w, conv_b, h0, state_in, dy, dhT = map(
        _f64, (u, W_a, W_x, b_a, b_x, Lambda, conv_w, conv_b, h0, state_in, dy, dhT))
    B, T, D = u.shape
    nb, bs, _ = W_a.shape
    K = conv_w.shape[0]
    out = dict(du=np.empty((B, T, D)), dh0=np.empty((B, D)), dW_a=np.empty((nb, bs, bs)),
               dW_x=np.empty((nb, bs, bs)), db_a=np.empty(D), db_x=np.empty(D),
               dLambda=np.empty(D), dconv_w=np.empty((K, D)), dconv_b=np.empty(D))
    _load().oracle_backward(B, T, D, nb, K, ctypes.c_double(c), _p(u), _p(W_a), _p(W_x), _p(b_a),
                            _p(b_x), _p(Lambda), _p(conv_w), _p(conv_b), _p(h0), _p(state_in),
                            _p(dy), _p(dhT), _p(out["du"]), _p(out["dh0"]), _p(out["dW_a"]),
                            _p(out["dW_x"]), _p(out["db_a"]), _p(out["db_x"]),
                            _p(out["dLambda"]), _p(out["dconv_w"]), _p(out["dconv_b"]),
                            (_keep := _mask(reset, B, T))[1])
    return out
