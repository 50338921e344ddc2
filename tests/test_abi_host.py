"""Host-side checks that need no GPU: the shared library loads, exports every function the
public header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

import paper_2402_19427_amd as R  # noqa: E402

FAKE = 0x1000  # a non-NULL, 256-byte aligned address that is never dereferenced on error paths


def declared_functions():
    text = open(os.path.join(ROOT, "include", "rglru.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rglru_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"rglru_conv1d", "rglru_forward", "rglru_decode_step", "rglru_backward",
            "rglru_workspace_bytes", "rglru_last_error", "rglru_version"} <= set(names)
    lib = ctypes.CDLL(R.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert R.rglru_version() >= 100


def test_binding_exposes_the_same_names():
    for n in declared_functions():
        assert callable(getattr(R, n)), n


def params():
    return R.make_params(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE)


def fwd(shape, p=None, u=FAKE, y=FAKE, ws=None, ws_bytes=0, pos0=0, h0=None):
    R.rglru_forward(shape, p or params(), u, h0, None, pos0, y, None, None, ws, ws_bytes)


@pytest.mark.parametrize("kw,code", [
    (dict(B=0), R.ERR_INVALID_ARG),
    (dict(D=0), R.ERR_INVALID_ARG),
    (dict(T=-1), R.ERR_INVALID_ARG),
    (dict(num_blocks=0), R.ERR_INVALID_ARG),
    (dict(num_blocks=3), R.ERR_INVALID_ARG),            # 16 % 3 != 0
    (dict(c=0.0), R.ERR_INVALID_ARG),
    (dict(act_dtype=7), R.ERR_INVALID_ARG),
    (dict(conv_width=3), R.ERR_UNSUPPORTED),
    (dict(conv_width=5), R.ERR_UNSUPPORTED),
    (dict(act_dtype=R.BF16, w_dtype=R.F32), R.ERR_UNSUPPORTED),
    (dict(D=4096 * 4, num_blocks=1), R.ERR_UNSUPPORTED),  # block larger than the LDS tile
    (dict(B=70000), R.ERR_UNSUPPORTED),
])
def test_forward_rejects_bad_shapes(kw, code):
    base = dict(B=2, T=8, D=16, num_blocks=2, act_dtype=R.F32)
    base.update(kw)
    with pytest.raises(R.RglruError) as e:
        fwd(R.make_shape(**base))
    assert e.value.code == code
    assert R.rglru_last_error() != ""


def test_conv_width_zero_needs_no_conv_arguments_and_conv1d_needs_the_filter():
    # no Conv1D: the filter taps may be NULL (everything else is validated as usual) ...
    s0 = R.make_shape(2, 8, 16, 2, R.F32, conv_width=0)
    no_taps = R.make_params(FAKE, FAKE, FAKE, FAKE, FAKE, None)
    with pytest.raises(R.RglruError) as e:
        R.rglru_forward(s0, no_taps, None, None, None, 0, FAKE, None, None, None, 0)
    assert e.value.code == R.ERR_INVALID_ARG and "u is NULL" in str(e.value)
    # ... with the filter they are required
    with pytest.raises(R.RglruError) as e:
        fwd(R.make_shape(2, 8, 16, 2, R.F32), p=no_taps)
    assert e.value.code == R.ERR_INVALID_ARG and "conv_w" in str(e.value)
    # the Conv1D alone has no width 0
    with pytest.raises(R.RglruError) as e:
        R.rglru_conv1d(s0, FAKE, FAKE, None, None, 0, FAKE, None)
    assert e.value.code == R.ERR_UNSUPPORTED


def test_null_and_misaligned_pointers():
    s = R.make_shape(2, 8, 16, 2, R.F32)
    with pytest.raises(R.RglruError) as e:
        fwd(s, u=None)
    assert e.value.code == R.ERR_INVALID_ARG and "u is NULL" in str(e.value)
    with pytest.raises(R.RglruError) as e:
        fwd(s, y=None)
    assert e.value.code == R.ERR_INVALID_ARG
    with pytest.raises(R.RglruError) as e:
        fwd(s, u=FAKE + 2)
    assert e.value.code == R.ERR_INVALID_ARG and "aligned" in str(e.value)
    with pytest.raises(R.RglruError) as e:
        fwd(s, p=R.make_params(None, FAKE, FAKE, FAKE, FAKE, FAKE))
    assert e.value.code == R.ERR_INVALID_ARG and "W_a" in str(e.value)
    with pytest.raises(R.RglruError) as e:
        fwd(s, pos0=-1)
    assert e.value.code == R.ERR_INVALID_ARG
    with pytest.raises(R.RglruError) as e:
        R.rglru_forward(s, None, FAKE, None, None, 0, FAKE, None, None, None, 0)
    assert e.value.code == R.ERR_INVALID_ARG


def test_decode_and_conv_validation():
    s = R.make_shape(2, 1, 16, 2, R.BF16)
    with pytest.raises(R.RglruError) as e:
        R.rglru_decode_step(s, params(), FAKE, None, FAKE, 0, FAKE)
    assert e.value.code == R.ERR_INVALID_ARG and "h is NULL" in str(e.value)
    with pytest.raises(R.RglruError) as e:
        R.rglru_decode_step(s, params(), FAKE, FAKE, FAKE, -5, FAKE)
    assert e.value.code == R.ERR_INVALID_ARG
    with pytest.raises(R.RglruError) as e:
        R.rglru_conv1d(s, FAKE, None, None, None, 0, FAKE, None)
    assert e.value.code == R.ERR_INVALID_ARG and "conv_w" in str(e.value)
    # conv1d ignores num_blocks
    s2 = R.make_shape(2, 4, 16, 5, R.BF16)
    with pytest.raises(R.RglruError) as e:
        R.rglru_conv1d(s2, None, FAKE, None, None, 0, FAKE, None)
    assert "u is NULL" in str(e.value)


def test_backward_validation_and_workspace():
    s = R.make_shape(2, 8, 16, 2, R.F32)
    need = R.rglru_workspace_bytes(s, R.OP_BACKWARD)
    assert need > 0 and need % 256 == 0
    g = R.make_param_grads(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE)
    args = (s, params(), FAKE, None, None, 0, FAKE, FAKE, None, FAKE, None, g)
    with pytest.raises(R.RglruError) as e:
        R.rglru_backward(*args, None, 0)
    assert e.value.code == R.ERR_WORKSPACE
    with pytest.raises(R.RglruError) as e:
        R.rglru_backward(*args, FAKE, need - 1)
    assert e.value.code == R.ERR_WORKSPACE
    with pytest.raises(R.RglruError) as e:
        R.rglru_backward(*args, FAKE + 64, need)
    assert e.value.code == R.ERR_INVALID_ARG
    g2 = R.make_param_grads(FAKE, FAKE, None, FAKE, FAKE, FAKE)
    with pytest.raises(R.RglruError) as e:
        R.rglru_backward(s, params(), FAKE, None, None, 0, FAKE, FAKE, None, FAKE, None, g2,
                         FAKE, need)
    assert e.value.code == R.ERR_INVALID_ARG and "db_a" in str(e.value)
    s0 = R.make_shape(2, 0, 16, 2, R.F32)
    with pytest.raises(R.RglruError) as e:
        R.rglru_backward(s0, params(), FAKE, None, None, 0, FAKE, FAKE, None, FAKE, None, g,
                         FAKE, 1 << 20)
    assert e.value.code == R.ERR_INVALID_ARG


def test_packed_calls_validation_and_workspace():
    s = R.make_shape(2, 8, 512, 2, R.BF16)
    fneed = R.rglru_workspace_bytes(s, R.OP_FORWARD_PACKED)
    assert fneed >= R.rglru_workspace_bytes(s, R.OP_FORWARD) + 2 * 16 and fneed % 256 == 0
    # the general kernels: scratch for their two-pass forward (optional: without it they run one pass)
    gneed = R.rglru_workspace_bytes(R.make_shape(2, 8, 96, 3, R.F32), R.OP_FORWARD_PACKED)
    assert gneed == R.rglru_workspace_bytes(R.make_shape(2, 8, 96, 3, R.F32), R.OP_FORWARD) and 0 < gneed < (1 << 20)
    need = R.rglru_workspace_bytes(s, R.OP_BACKWARD_PACKED)
    assert need >= 4 * 2 * 8 * 512 * 4 and need % 256 == 0
    with pytest.raises(R.RglruError) as e:
        R.rglru_forward_packed(s, params(), None, FAKE, None, None, 0, FAKE, None, None, FAKE, fneed)
    assert e.value.code == R.ERR_INVALID_ARG and "u" in str(e.value)
    with pytest.raises(R.RglruError) as e:
        R.rglru_forward_packed(s, params(), FAKE, FAKE, None, None, -1, FAKE, None, None, FAKE, fneed)
    assert e.value.code == R.ERR_INVALID_ARG
    with pytest.raises(R.RglruError) as e:
        R.rglru_forward_packed(s, params(), FAKE, FAKE, None, None, 0, FAKE, None, None, FAKE, fneed - 1)
    assert e.value.code == R.ERR_WORKSPACE
    g = R.make_param_grads(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE)
    args = (s, params(), FAKE, FAKE + 1, None, None, 0, FAKE, FAKE, None, FAKE, None, g)   # the mask is bytes: any address
    with pytest.raises(R.RglruError) as e:
        R.rglru_backward_packed(*args, FAKE, need - 1)
    assert e.value.code == R.ERR_WORKSPACE
    with pytest.raises(R.RglruError) as e:
        R.rglru_backward_packed(*args, None, 0)
    assert e.value.code == R.ERR_WORKSPACE
    with pytest.raises(R.RglruError) as e:
        R.rglru_workspace_status(s, R.OP_CG_BACKWARD, None)
    assert e.value.code == R.ERR_INVALID_ARG


def test_cg_calls_validation_and_workspace():
    cg = R.make_cg_params(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE)
    s = R.make_shape(2, 8, 64, 2, R.F32)
    need = R.rglru_workspace_bytes(s, R.OP_CG_BACKWARD)
    assert need >= 6 * 2 * 8 * 64 * 4 and need % 256 == 0
    for bad, what in ((R.make_shape(2, 8, 63, 1, R.F32), "even"), (R.make_shape(2, 8, 64, 3, R.F32), "multiple"),
                      (R.make_shape(2, 8, 8192, 1, R.BF16), "exceeds")):
        with pytest.raises(R.RglruError) as e:
            R.rglru_cg_forward(bad, cg, FAKE, None, None, 0, FAKE, None, None, None, 0)
        assert what in str(e.value)
        assert R.rglru_workspace_bytes(bad, R.OP_CG_BACKWARD) == 0
    no_theta = R.make_cg_params(FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE)
    with pytest.raises(R.RglruError) as e:
        R.rglru_cg_forward(s, no_theta, FAKE, None, None, 0, FAKE, None, None, None, 0)
    assert e.value.code == R.ERR_INVALID_ARG and "theta" in str(e.value)
    with pytest.raises(R.RglruError) as e:
        R.rglru_cg_decode_step(s, cg, FAKE, None, FAKE, 0, FAKE)
    assert e.value.code == R.ERR_INVALID_ARG and "h" in str(e.value)
    g = R.make_cg_param_grads(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE)
    with pytest.raises(R.RglruError) as e:
        R.rglru_cg_backward(s, cg, FAKE, None, None, 0, FAKE, None, FAKE, None, g, FAKE, need - 1)
    assert e.value.code == R.ERR_WORKSPACE
    g2 = R.make_cg_param_grads(FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE)
    with pytest.raises(R.RglruError) as e:
        R.rglru_cg_backward(s, cg, FAKE, None, None, 0, FAKE, None, FAKE, None, g2, FAKE, need)
    assert e.value.code == R.ERR_INVALID_ARG and "dtheta" in str(e.value)


def test_workspace_query_is_zero_for_invalid_shapes_and_keeps_error_string():
    bad = R.make_shape(2, 8, 16, 3, R.F32)
    with pytest.raises(R.RglruError):
        fwd(bad)
    msg = R.rglru_last_error()
    assert R.rglru_workspace_bytes(bad, R.OP_FORWARD) == 0
    assert R.rglru_workspace_bytes(bad, 99) == 0
    assert R.rglru_last_error() == msg


def test_scan_validation():
    s = R.make_shape(2, 8, 16, 5, R.BF16)     # num_blocks is not used by the scan
    with pytest.raises(R.RglruError) as e:
        R.rglru_scan(s, None, FAKE, None, 0, FAKE, None, None, 0)
    assert e.value.code == R.ERR_INVALID_ARG and "a is NULL" in str(e.value)
    with pytest.raises(R.RglruError) as e:
        R.rglru_scan(s, FAKE, FAKE, None, 0, None, None, None, 0)
    assert e.value.code == R.ERR_INVALID_ARG and "h is NULL" in str(e.value)
    with pytest.raises(R.RglruError) as e:
        R.rglru_scan(s, FAKE, FAKE, None, 8, FAKE, None, None, 0)
    assert e.value.code == R.ERR_INVALID_ARG and "flags" in str(e.value)
    with pytest.raises(R.RglruError) as e:      # the adjoint exists for the unscaled recurrence only
        R.rglru_scan(s, FAKE, FAKE, None, R.SCAN_ADJOINT, FAKE, None, None, 0)
    assert e.value.code == R.ERR_INVALID_ARG and "ADJOINT" in str(e.value)
    with pytest.raises(R.RglruError) as e:
        R.rglru_scan(s, FAKE + 1, FAKE, None, 0, FAKE, None, None, 0)
    assert e.value.code == R.ERR_INVALID_ARG and "aligned" in str(e.value)
    # the tiled kernel needs a workspace when sequences are cut into time slices
    big = R.make_shape(8, 4096, 1024, 1, R.BF16)
    need = R.rglru_workspace_bytes(big, R.OP_SCAN)
    assert need % 256 == 0
    if need:
        with pytest.raises(R.RglruError) as e:
            R.rglru_scan(big, FAKE, FAKE, None, 0, FAKE, None, None, 0)
        assert e.value.code == R.ERR_WORKSPACE
    assert R.rglru_workspace_bytes(R.make_shape(8, 4096, 1000, 1, R.F32), R.OP_SCAN) == 0


def test_workspace_status_validation():
    s = R.make_shape(2, 8, 16, 2, R.F32)
    with pytest.raises(R.RglruError) as e:
        R.rglru_workspace_status(s, R.OP_DECODE, FAKE)
    assert e.value.code == R.ERR_INVALID_ARG
    with pytest.raises(R.RglruError) as e:
        R.rglru_workspace_status(None, R.OP_FORWARD, FAKE)
    assert e.value.code == R.ERR_INVALID_ARG


def test_merge_calls_validation_and_workspace():
    s = R.make_shape(2, 8, 16, 2, R.BF16)
    OUT, Y = FAKE + 4096, FAKE + 8192
    with pytest.raises(R.RglruError) as e:
        R.rglru_forward_merge(s, params(), FAKE, None, None, None, 0, 0, OUT, None, None, None, None, 0)
    assert e.value.code == R.ERR_INVALID_ARG and "branch is NULL" in str(e.value)
    with pytest.raises(R.RglruError) as e:
        R.rglru_forward_merge(s, params(), FAKE, FAKE, None, None, 0, 4, OUT, None, None, None, None, 0)
    assert e.value.code == R.ERR_INVALID_ARG and "flags" in str(e.value)
    with pytest.raises(R.RglruError) as e:
        R.rglru_forward_merge(s, params(), FAKE, Y, None, None, 0, 0, Y, None, None, None, None, 0)
    assert e.value.code == R.ERR_INVALID_ARG and "alias" in str(e.value)
    # the backward needs room for dy on top of the plain backward's workspace: in bf16 storage as
    # two bf16 tensors (dy as stored and what its rounding took away), so that it reaches the
    # backward with 16 significant bits
    plain = R.rglru_workspace_bytes(s, R.OP_BACKWARD)
    need = R.rglru_workspace_bytes(s, R.OP_BACKWARD_MERGE)
    assert need == plain + 2 * (2 * 8 * 16 * 2) and need % 256 == 0
    s32 = R.make_shape(2, 8, 16, 2, R.F32)
    assert (R.rglru_workspace_bytes(s32, R.OP_BACKWARD_MERGE)
            == R.rglru_workspace_bytes(s32, R.OP_BACKWARD) + 2 * 8 * 16 * 4)
    assert R.rglru_workspace_bytes(s, R.OP_FORWARD_MERGE) == R.rglru_workspace_bytes(s, R.OP_FORWARD)
    g = R.make_param_grads(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE)
    args = (s, params(), FAKE, FAKE, None, None, 0, 0, Y, FAKE, None, OUT, FAKE + 12288, None, g)
    with pytest.raises(R.RglruError) as e:
        R.rglru_backward_merge(*args, FAKE, need - 1)
    assert e.value.code == R.ERR_WORKSPACE
    with pytest.raises(R.RglruError) as e:
        R.rglru_backward_merge(s, params(), FAKE, FAKE, None, None, 0, 0, Y, FAKE, None, OUT, None, None, g,
                               FAKE, need)
    assert e.value.code == R.ERR_INVALID_ARG and "dbranch is NULL" in str(e.value)
    g2 = R.make_param_grads(FAKE, FAKE, None, FAKE, FAKE, FAKE)
    with pytest.raises(R.RglruError) as e:   # found by the plain backward's checks, before any launch
        R.rglru_backward_merge(s, params(), FAKE, FAKE, None, None, 0, 0, Y, FAKE, None, OUT, FAKE + 12288,
                               None, g2, FAKE, need)
    assert e.value.code == R.ERR_INVALID_ARG and "db_a" in str(e.value)


def test_decode_step_at_validation():
    s = R.make_shape(2, 1, 16, 2, R.BF16)
    with pytest.raises(R.RglruError, match="pos") as e:
        R.rglru_decode_step_at(s, params(), FAKE, FAKE, FAKE, None, FAKE)
    assert e.value.code == R.ERR_INVALID_ARG
    with pytest.raises(R.RglruError, match="pos"):
        R.rglru_decode_step_at(s, params(), FAKE, FAKE, FAKE, FAKE + 4, FAKE)


def test_decode_step_merge_validation():
    s = R.make_shape(2, 1, 16, 2, R.BF16)
    OUT = FAKE + 4096
    with pytest.raises(R.RglruError) as e:
        R.rglru_decode_step_merge(s, params(), FAKE, None, FAKE, FAKE, 0, 0, OUT)
    assert e.value.code == R.ERR_INVALID_ARG and "branch_t is NULL" in str(e.value)
    with pytest.raises(R.RglruError) as e:
        R.rglru_decode_step_merge(s, params(), FAKE, FAKE, FAKE, FAKE, 0, R.MERGE_SEPARATE, OUT)
    assert e.value.code == R.ERR_INVALID_ARG and "flags" in str(e.value)
    with pytest.raises(R.RglruError) as e:
        R.rglru_decode_step_merge(s, params(), FAKE, OUT, FAKE, FAKE, 0, 0, OUT)
    assert e.value.code == R.ERR_INVALID_ARG and "alias" in str(e.value)
    with pytest.raises(R.RglruError) as e:
        R.rglru_decode_step_merge(s, params(), FAKE, FAKE, FAKE, FAKE, -1, 0, OUT)
    assert e.value.code == R.ERR_INVALID_ARG and "pos" in str(e.value)


def test_workspace_sizes_for_narrower_gate_blocks():
    # 16 blocks of 160 channels (bf16): forward in the padded tile needs the record rings of the
    # tuned kernel and, like it, W_x once more in half precision; the backward a widened copy
    # (four activation tensors of nb*256 channels) plus the tuned backward's workspace at that width
    narrow = R.make_shape(8, 2048, 2560, 16, R.BF16)
    wide = R.make_shape(8, 2048, 4096, 16, R.BF16)
    assert (R.rglru_workspace_bytes(narrow, R.OP_FORWARD) - 16 * 160 * 160 * 2
            == R.rglru_workspace_bytes(wide, R.OP_FORWARD) - 16 * 256 * 256 * 2 > 0)
    # one workgroup per (sequence, block), no records: the status word and the weight copy
    assert R.rglru_workspace_bytes(R.make_shape(16, 4096, 4096, 16, R.BF16), R.OP_FORWARD) == 256 + 16 * 256 * 256 * 2
    need = R.rglru_workspace_bytes(narrow, R.OP_BACKWARD)
    inner = R.rglru_workspace_bytes(wide, R.OP_BACKWARD)
    assert need > inner + 4 * 8 * 2048 * 4096 * 2 and need % 256 == 0
    # other multiples of 16 (bf16) run as separate passes: four activation-sized buffers (x twice,
    # log a_t, b_t), the gate weights in half precision, and the scan's records
    n = 8 * 2048 * 2560 * 2
    for nb in (8, 32):      # bs = 320, 80
        w = R.rglru_workspace_bytes(R.make_shape(8, 2048, 2560, nb, R.BF16), R.OP_FORWARD)
        bs = 2560 // nb
        wf = 2 * nb * bs * bs * 2          # both gates' weights once more, in half precision
        assert w - 4 * n - wf == R.rglru_workspace_bytes(R.make_shape(8, 2048, 2560, 1, R.BF16), R.OP_SCAN)
    # fp32 storage and block sizes that are no multiple of 16 stay on the generic kernels
    # fp32 storage and the block sizes no matrix-core kernel takes: the general kernels' two-pass
    # scratch, capped (a chunk of the time axis at a time), and optional
    for sh in (R.make_shape(8, 2048, 2560, 16, R.F32), R.make_shape(8, 2048, 2560, 64, R.BF16)):   # (bs 40)
        n = R.rglru_workspace_bytes(sh, R.OP_FORWARD)
        assert 0 < n <= 256 + 8 * 2560 * 4 + 2 * (64 << 20) + 1024 and n % 256 == 0
