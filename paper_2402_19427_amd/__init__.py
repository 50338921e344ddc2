"""MI355X-native Conv1D -> RG-LRU path of the Griffin/Hawk recurrent block.

The work happens in librglru.so (hand-written HIP for gfx950, C ABI in include/rglru.h);
`paper_2402_19427_amd.binding` is the thin ctypes layer with the same names, re-exported
here. The binding is loaded on first use so that `python -m paper_2402_19427_amd.build` can
run before the library exists; using any entry point without the built library raises
ImportError (there is no fallback implementation).
"""
import importlib

_EXPORTS = (
    "BF16", "F32", "OK", "ERR_HIP", "ERR_TIMEOUT", "rglru_workspace_status", "rglru_set_max_time_slices", "ERR_INVALID_ARG", "ERR_UNSUPPORTED", "ERR_WORKSPACE",
    "OP_CG_BACKWARD", "OP_CG_FORWARD", "CgParams", "CgParamGrads", "make_cg_params", "make_cg_param_grads",
    "rglru_cg_forward", "rglru_cg_decode_step", "rglru_cg_backward",
    "OP_FORWARD_PACKED", "OP_BACKWARD_PACKED", "rglru_forward_packed", "rglru_backward_packed",
    "OP_BACKWARD", "OP_BACKWARD_MERGE", "OP_FORWARD_MERGE", "MERGE_GELU_TANH", "MERGE_SEPARATE", "rglru_forward_merge", "rglru_decode_step_merge",
    "rglru_backward_merge", "OP_CONV1D", "OP_DECODE", "OP_FORWARD", "OP_SCAN", "SCAN_LOG_A", "SCAN_ADJOINT",
    "SCAN_NO_INPUT_SCALE", "rglru_scan", "LIB_PATH", "ParamGrads", "Params",
    "RglruError", "Shape", "make_param_grads", "make_params", "make_shape", "rglru_backward",
    "rglru_conv1d", "rglru_forward_static", "STATIC_SCRATCH_BYTES", "rglru_decode_step", "rglru_decode_step_at", "rglru_forward", "rglru_last_error", "rglru_version",
    "rglru_workspace_bytes", "rglru_timing_enable", "rglru_timing_select", "rglru_timing_count", "rglru_timing_get",
)
__all__ = list(_EXPORTS)


def __getattr__(name):
    if name in _EXPORTS:
        return getattr(importlib.import_module(".binding", __name__), name)
    raise AttributeError(name)
