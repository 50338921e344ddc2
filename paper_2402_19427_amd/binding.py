"""ctypes binding of librglru: argument marshalling only.

Functions mirror the C ABI of include/rglru.h one to one and take raw device addresses
(ints) or torch CUDA tensors; every step of the path runs inside the library's HIP kernels.
There is no CPU fallback: if the shared library is missing, importing this module raises.
"""
import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("RGLRU_LIB", os.path.join(_PKG, "librglru.so"))

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP, ERR_TIMEOUT = 0, -1, -2, -3, -4, -5
F32, BF16 = 0, 1
OP_CONV1D, OP_FORWARD, OP_DECODE, OP_BACKWARD, OP_SCAN = 0, 1, 2, 3, 4
OP_FORWARD_MERGE, OP_BACKWARD_MERGE = 5, 6
OP_FORWARD_PACKED, OP_BACKWARD_PACKED = 7, 8
OP_CG_BACKWARD, OP_CG_FORWARD = 9, 10
MERGE_GELU_TANH, MERGE_SEPARATE = 1, 2
SCAN_LOG_A, SCAN_NO_INPUT_SCALE, SCAN_ADJOINT = 1, 2, 4
STATIC_SCRATCH_BYTES = 16 << 20


class Shape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("T", ctypes.c_int32), ("D", ctypes.c_int32),
                ("num_blocks", ctypes.c_int32), ("conv_width", ctypes.c_int32),
                ("c", ctypes.c_float), ("act_dtype", ctypes.c_int32), ("w_dtype", ctypes.c_int32)]


class Params(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("W_a", "W_x", "b_a", "b_x", "Lambda", "conv_w", "conv_b")]


class ParamGrads(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("dW_a", "dW_x", "db_a", "db_x", "dLambda", "dconv_w", "dconv_b")]


class CgParams(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("W_a", "W_x", "b_a", "b_x", "Lambda", "theta", "conv_w", "conv_b")]


class CgParamGrads(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("dW_a", "dW_x", "db_a", "db_x", "dLambda", "dtheta", "dconv_w", "dconv_b")]


class RglruError(RuntimeError):
    def __init__(self, code, message):
        super().__init__("librglru error %d: %s" % (code, message))
        self.code = code


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "%s is missing: build it with `python -m paper_2402_19427_amd.build` "
            "(there is no fallback implementation)" % LIB_PATH)
    # torch ships its own HIP runtime; it has to be in the process before librglru is
    # loaded so that the library binds to that same runtime (one runtime, one set of devices
    # and streams) instead of pulling in a second copy from /opt/rocm.
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t
    sp, pp, gp = ctypes.POINTER(Shape), ctypes.POINTER(Params), ctypes.POINTER(ParamGrads)
    lib.rglru_conv1d.argtypes = [sp, vp, vp, vp, vp, i64, vp, vp, vp]
    lib.rglru_forward.argtypes = [sp, pp, vp, vp, vp, i64, vp, vp, vp, vp, sz, vp]
    lib.rglru_forward_static.argtypes = [sp, pp, vp, vp, vp, i64, vp, vp, vp, vp]
    lib.rglru_forward_static.restype = ctypes.c_int
    lib.rglru_decode_step.argtypes = [sp, pp, vp, vp, vp, i64, vp, vp]
    lib.rglru_decode_step_at.argtypes = [sp, pp, vp, vp, vp, vp, vp, vp]
    lib.rglru_backward.argtypes = [sp, pp, vp, vp, vp, i64, vp, vp, vp, vp, vp, gp, vp, sz, vp]
    lib.rglru_forward_packed.argtypes = [sp, pp, vp, vp, vp, vp, i64, vp, vp, vp, vp, sz, vp]
    lib.rglru_forward_packed.restype = ctypes.c_int
    lib.rglru_backward_packed.argtypes = [sp, pp, vp, vp, vp, vp, i64, vp, vp, vp, vp, vp, gp, vp, sz, vp]
    lib.rglru_backward_packed.restype = ctypes.c_int
    cp, cgp = ctypes.POINTER(CgParams), ctypes.POINTER(CgParamGrads)
    lib.rglru_cg_forward.argtypes = [sp, cp, vp, vp, vp, i64, vp, vp, vp, vp, sz, vp]
    lib.rglru_cg_decode_step.argtypes = [sp, cp, vp, vp, vp, i64, vp, vp]
    lib.rglru_cg_backward.argtypes = [sp, cp, vp, vp, vp, i64, vp, vp, vp, vp, cgp, vp, sz, vp]
    for f in (lib.rglru_cg_forward, lib.rglru_cg_decode_step, lib.rglru_cg_backward):
        f.restype = ctypes.c_int
    lib.rglru_forward_merge.argtypes = [sp, pp, vp, vp, vp, vp, i64, ctypes.c_uint, vp, vp, vp, vp, vp, sz, vp]
    lib.rglru_backward_merge.argtypes = [sp, pp, vp, vp, vp, vp, i64, ctypes.c_uint, vp, vp, vp, vp, vp, vp,
                                         gp, vp, sz, vp]
    lib.rglru_decode_step_merge.argtypes = [sp, pp, vp, vp, vp, vp, i64, ctypes.c_uint, vp, vp]
    lib.rglru_scan.argtypes = [sp, vp, vp, vp, ctypes.c_uint, vp, vp, vp, sz, vp]
    lib.rglru_set_max_time_slices.argtypes = [ctypes.c_int]
    lib.rglru_set_max_time_slices.restype = ctypes.c_int
    lib.rglru_workspace_status.argtypes = [sp, ctypes.c_int, vp, vp]
    lib.rglru_workspace_status.restype = ctypes.c_int
    lib.rglru_workspace_bytes.argtypes = [sp, ctypes.c_int]
    lib.rglru_workspace_bytes.restype = sz
    lib.rglru_last_error.restype = ctypes.c_char_p
    lib.rglru_version.restype = ctypes.c_int
    lib.rglru_timing_enable.argtypes = [ctypes.c_int]
    lib.rglru_timing_select.argtypes = [ctypes.c_char_p]
    lib.rglru_timing_get.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_char_p),
                                     ctypes.POINTER(ctypes.c_float)]
    for f in (lib.rglru_conv1d, lib.rglru_forward, lib.rglru_decode_step, lib.rglru_backward,
              lib.rglru_scan):
        f.restype = ctypes.c_int
    return lib


_lib = _load()


def _addr(t):
    """Device address of a torch tensor, an int address, or NULL for None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("tensors handed to librglru must be contiguous")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        return None
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream  # torch.cuda.Stream


def _ref(struct):
    """Pointer to a ctypes struct, or NULL for None."""
    return None if struct is None else ctypes.byref(struct)


def _check(rc):
    if rc != OK:
        raise RglruError(rc, _lib.rglru_last_error().decode())


def make_shape(B, T, D, num_blocks, act_dtype, w_dtype=None, conv_width=4, c=8.0):
    return Shape(B, T, D, num_blocks, conv_width, c, act_dtype,
                 act_dtype if w_dtype is None else w_dtype)


def make_params(W_a, W_x, b_a, b_x, Lambda, conv_w, conv_b=None):
    return Params(*[_addr(t) for t in (W_a, W_x, b_a, b_x, Lambda, conv_w, conv_b)])


def make_param_grads(dW_a, dW_x, db_a, db_x, dLambda, dconv_w, dconv_b=None):
    return ParamGrads(*[_addr(t) for t in (dW_a, dW_x, db_a, db_x, dLambda, dconv_w, dconv_b)])


def make_cg_params(W_a, W_x, b_a, b_x, Lambda, theta, conv_w=None, conv_b=None):
    return CgParams(*[_addr(t) for t in (W_a, W_x, b_a, b_x, Lambda, theta, conv_w, conv_b)])


def make_cg_param_grads(dW_a, dW_x, db_a, db_x, dLambda, dtheta, dconv_w=None, dconv_b=None):
    return CgParamGrads(*[_addr(t) for t in (dW_a, dW_x, db_a, db_x, dLambda, dtheta, dconv_w, dconv_b)])


def rglru_version():
    return _lib.rglru_version()


def rglru_last_error():
    return _lib.rglru_last_error().decode()


def rglru_timing_enable(enable):
    _check(_lib.rglru_timing_enable(1 if enable else 0))


def rglru_timing_select(kernel_name):
    """Time only the kernels of this name (None: all kernels)."""
    _check(_lib.rglru_timing_select(kernel_name.encode() if kernel_name else None))


def rglru_timing_count():
    return int(_lib.rglru_timing_count())


def rglru_timing_get(index):
    """(kernel name, milliseconds) of timing record `index`; synchronise the stream first."""
    name, ms = ctypes.c_char_p(), ctypes.c_float()
    _check(_lib.rglru_timing_get(index, ctypes.byref(name), ctypes.byref(ms)))
    return name.value.decode(), float(ms.value)


def rglru_workspace_bytes(shape, op):
    return int(_lib.rglru_workspace_bytes(_ref(shape), op))


def rglru_conv1d(shape, u, conv_w, conv_b, conv_state_in, pos0, x_out, conv_state_out,
                 stream=None):
    _check(_lib.rglru_conv1d(_ref(shape), _addr(u), _addr(conv_w), _addr(conv_b),
                             _addr(conv_state_in), pos0, _addr(x_out), _addr(conv_state_out),
                             _stream(stream)))


def rglru_forward(shape, params, u, h0, conv_state_in, pos0, y, hT, conv_state_out, workspace,
                  workspace_bytes, stream=None):
    _check(_lib.rglru_forward(_ref(shape), _ref(params), _addr(u), _addr(h0),
                              _addr(conv_state_in), pos0, _addr(y), _addr(hT),
                              _addr(conv_state_out), _addr(workspace), workspace_bytes,
                              _stream(stream)))


def rglru_forward_static(shape, params, u, h0, conv_state_in, pos0, y, hT, conv_state_out, stream=None):
    _check(_lib.rglru_forward_static(_ref(shape), _ref(params), _addr(u), _addr(h0),
                                     _addr(conv_state_in), pos0, _addr(y), _addr(hT),
                                     _addr(conv_state_out), _stream(stream)))


def rglru_decode_step(shape, params, u_t, h, conv_state, pos, y_t, stream=None):
    _check(_lib.rglru_decode_step(_ref(shape), _ref(params), _addr(u_t), _addr(h),
                                  _addr(conv_state), pos, _addr(y_t), _stream(stream)))


def rglru_decode_step_at(shape, params, u_t, h, conv_state, pos, y_t, stream=None):
    _check(_lib.rglru_decode_step_at(_ref(shape), _ref(params), _addr(u_t), _addr(h),
                                     _addr(conv_state), _addr(pos), _addr(y_t), _stream(stream)))


def rglru_backward(shape, params, u, h0, conv_state_in, pos0, y, dy, dhT, du, dh0, grads,
                   workspace, workspace_bytes, stream=None):
    _check(_lib.rglru_backward(_ref(shape), _ref(params), _addr(u), _addr(h0),
                               _addr(conv_state_in), pos0, _addr(y), _addr(dy), _addr(dhT),
                               _addr(du), _addr(dh0), _ref(grads), _addr(workspace),
                               workspace_bytes, _stream(stream)))


def rglru_forward_packed(shape, params, u, reset, h0, conv_state_in, pos0, y, hT, conv_state_out,
                         workspace, workspace_bytes, stream=None):
    _check(_lib.rglru_forward_packed(_ref(shape), _ref(params), _addr(u), _addr(reset), _addr(h0),
                                     _addr(conv_state_in), pos0, _addr(y), _addr(hT),
                                     _addr(conv_state_out), _addr(workspace), workspace_bytes,
                                     _stream(stream)))


def rglru_backward_packed(shape, params, u, reset, h0, conv_state_in, pos0, y, dy, dhT, du, dh0,
                          grads, workspace, workspace_bytes, stream=None):
    _check(_lib.rglru_backward_packed(_ref(shape), _ref(params), _addr(u), _addr(reset), _addr(h0),
                                      _addr(conv_state_in), pos0, _addr(y), _addr(dy), _addr(dhT),
                                      _addr(du), _addr(dh0), _ref(grads), _addr(workspace),
                                      workspace_bytes, _stream(stream)))


def rglru_cg_forward(shape, params, u, h0, conv_state_in, pos0, y, hT, conv_state_out, workspace=None,
                     workspace_bytes=0, stream=None):
    _check(_lib.rglru_cg_forward(_ref(shape), _ref(params), _addr(u), _addr(h0), _addr(conv_state_in),
                                 pos0, _addr(y), _addr(hT), _addr(conv_state_out), _addr(workspace),
                                 workspace_bytes, _stream(stream)))


def rglru_cg_decode_step(shape, params, u_t, h, conv_state, pos, y_t, stream=None):
    _check(_lib.rglru_cg_decode_step(_ref(shape), _ref(params), _addr(u_t), _addr(h),
                                     _addr(conv_state), pos, _addr(y_t), _stream(stream)))


def rglru_cg_backward(shape, params, u, h0, conv_state_in, pos0, dy, dhT, du, dh0, grads,
                      workspace, workspace_bytes, stream=None):
    _check(_lib.rglru_cg_backward(_ref(shape), _ref(params), _addr(u), _addr(h0),
                                  _addr(conv_state_in), pos0, _addr(dy), _addr(dhT),
                                  _addr(du), _addr(dh0), _ref(grads), _addr(workspace),
                                  workspace_bytes, _stream(stream)))


def rglru_forward_merge(shape, params, u, branch, h0, conv_state_in, pos0, flags, out, y, hT,
                        conv_state_out, workspace, workspace_bytes, stream=None):
    _check(_lib.rglru_forward_merge(_ref(shape), _ref(params), _addr(u), _addr(branch), _addr(h0),
                                    _addr(conv_state_in), pos0, flags, _addr(out), _addr(y),
                                    _addr(hT), _addr(conv_state_out), _addr(workspace),
                                    workspace_bytes, _stream(stream)))


def rglru_decode_step_merge(shape, params, u_t, branch_t, h, conv_state, pos, flags, out_t,
                            stream=None):
    _check(_lib.rglru_decode_step_merge(_ref(shape), _ref(params), _addr(u_t), _addr(branch_t),
                                        _addr(h), _addr(conv_state), pos, flags, _addr(out_t),
                                        _stream(stream)))


def rglru_backward_merge(shape, params, u, branch, h0, conv_state_in, pos0, flags, y, dout, dhT, du,
                         dbranch, dh0, grads, workspace, workspace_bytes, stream=None):
    _check(_lib.rglru_backward_merge(_ref(shape), _ref(params), _addr(u), _addr(branch), _addr(h0),
                                     _addr(conv_state_in), pos0, flags, _addr(y), _addr(dout),
                                     _addr(dhT), _addr(du), _addr(dbranch), _addr(dh0),
                                     _ref(grads), _addr(workspace), workspace_bytes,
                                     _stream(stream)))


def rglru_scan(shape, a, g, h0, flags, h, hT, workspace, workspace_bytes, stream=None):
    _check(_lib.rglru_scan(_ref(shape), _addr(a), _addr(g), _addr(h0), flags, _addr(h), _addr(hT),
                           _addr(workspace), workspace_bytes, _stream(stream)))


def rglru_set_max_time_slices(max_slices):
    _check(_lib.rglru_set_max_time_slices(int(max_slices)))


def rglru_workspace_status(shape, op, workspace, stream=None):
    """Waits for the stream and raises RglruError(ERR_TIMEOUT) if a bounded wait expired."""
    _check(_lib.rglru_workspace_status(_ref(shape), op, _addr(workspace), _stream(stream)))
