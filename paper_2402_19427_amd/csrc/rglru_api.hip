// C ABI of librglru: argument validation on the host, choice of kernel family, launches.
// Nothing here touches the GPU before validation has passed, so every error path can be
// exercised on a machine without one.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>

#include "rglru_internal.h"
#include "rglru_mfma.h"

using namespace rglru;

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

}  // namespace

void rglru::set_last_error(const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

namespace {

bool aligned(const void *p, size_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

size_t act_size(const rglru_shape *s) { return s->act_dtype == RGLRU_BF16 ? 2 : 4; }

constexpr int MAX_BLOCK = 2048;  // largest gate block the generic kernels stage in LDS

// Checks everything about `s` that does not involve pointers. need_blocks: the op uses the
// gate matrices. Returns RGLRU_OK or an error code with the message set.
int check_shape(const rglru_shape *s, bool need_blocks, bool need_T, int min_T, bool conv_optional = true) {
  if (!s) return fail(RGLRU_ERR_INVALID_ARG, "shape is NULL");
  if (s->B < 1) return fail(RGLRU_ERR_INVALID_ARG, "B must be >= 1 (got %d)", s->B);
  if (s->D < 1) return fail(RGLRU_ERR_INVALID_ARG, "D must be >= 1 (got %d)", s->D);
  if (need_T && s->T < min_T)
    return fail(RGLRU_ERR_INVALID_ARG, "T must be >= %d (got %d)", min_T, s->T);
  if (!(s->c > 0.f) || !std::isfinite(s->c))
    return fail(RGLRU_ERR_INVALID_ARG, "c must be finite and positive");
  if (s->act_dtype != RGLRU_F32 && s->act_dtype != RGLRU_BF16)
    return fail(RGLRU_ERR_INVALID_ARG, "unknown act_dtype %d", s->act_dtype);
  if (s->w_dtype != RGLRU_F32 && s->w_dtype != RGLRU_BF16)
    return fail(RGLRU_ERR_INVALID_ARG, "unknown w_dtype %d", s->w_dtype);
  if (need_blocks) {
    if (s->num_blocks < 1)
      return fail(RGLRU_ERR_INVALID_ARG, "num_blocks must be >= 1 (got %d)", s->num_blocks);
    if (s->D % s->num_blocks != 0)
      return fail(RGLRU_ERR_INVALID_ARG, "D (%d) is not a multiple of num_blocks (%d)", s->D,
                  s->num_blocks);
  }
  if (s->conv_width != 4 && !(s->conv_width == 0 && conv_optional))
    return fail(RGLRU_ERR_UNSUPPORTED, "conv_width %d is not supported (4%s)", s->conv_width,
                conv_optional ? ", or 0: the input is already x_t" : " only");
  if (s->act_dtype != s->w_dtype)
    return fail(RGLRU_ERR_UNSUPPORTED,
                "act_dtype %d with w_dtype %d is not supported (use f32/f32 or bf16/bf16)",
                s->act_dtype, s->w_dtype);
  if (need_blocks && s->D / s->num_blocks > MAX_BLOCK)
    return fail(RGLRU_ERR_UNSUPPORTED, "gate block size %d exceeds %d", s->D / s->num_blocks,
                MAX_BLOCK);
  if (s->B > 65535) return fail(RGLRU_ERR_UNSUPPORTED, "B %d exceeds 65535", s->B);
  return RGLRU_OK;
}

int check_ptr(const void *p, const char *name, size_t align, bool required) {
  if (!p) return required ? fail(RGLRU_ERR_INVALID_ARG, "%s is NULL", name) : RGLRU_OK;
  if (!aligned(p, align))
    return fail(RGLRU_ERR_INVALID_ARG, "%s is not %zu-byte aligned", name, align);
  return RGLRU_OK;
}

#define CHECK(expr)               \
  do {                            \
    int rc_ = (expr);             \
    if (rc_ != RGLRU_OK) return rc_; \
  } while (0)

int check_params(const rglru_shape *s, const rglru_params *p) {
  if (!p) return fail(RGLRU_ERR_INVALID_ARG, "params is NULL");
  const size_t ws = s->w_dtype == RGLRU_BF16 ? 2 : 4;
  CHECK(check_ptr(p->W_a, "params.W_a", ws, true));
  CHECK(check_ptr(p->W_x, "params.W_x", ws, true));
  CHECK(check_ptr(p->b_a, "params.b_a", 4, true));
  CHECK(check_ptr(p->b_x, "params.b_x", 4, true));
  CHECK(check_ptr(p->Lambda, "params.Lambda", 4, true));
  CHECK(check_ptr(p->conv_w, "params.conv_w", 4, s->conv_width != 0));   // (ignored without the Conv1D)
  CHECK(check_ptr(p->conv_b, "params.conv_b", 4, false));
  return RGLRU_OK;
}

int check_workspace(const void *ws, size_t have, size_t need) {
  if (need == 0) return RGLRU_OK;
  if (!ws) return fail(RGLRU_ERR_WORKSPACE, "workspace is NULL but %zu bytes are needed", need);
  if (have < need)
    return fail(RGLRU_ERR_WORKSPACE, "workspace has %zu bytes, %zu are needed", have, need);
  if (!aligned(ws, 256)) return fail(RGLRU_ERR_INVALID_ARG, "workspace is not 256-byte aligned");
  return RGLRU_OK;
}

// the forward on the general kernels can do without scratch (one pass, serial in time): a missing
// or short workspace is not an error there, a misaligned one is
bool forward_on_general_kernels(const rglru_shape *s);
int check_forward_workspace(const rglru_shape *s, const void *ws, size_t have, size_t need) {
  if (!forward_on_general_kernels(s)) return check_workspace(ws, have, need);
  if (ws && !aligned(ws, 256)) return fail(RGLRU_ERR_INVALID_ARG, "workspace is not 256-byte aligned");
  return RGLRU_OK;
}

int hip_fail(hipError_t e, const char *what) {
  return fail(RGLRU_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

void fill_params(Problem &q, const rglru_shape *s, const rglru_params *p) {
  q.B = s->B; q.T = s->T; q.D = s->D;
  q.nb = s->num_blocks; q.bs = s->D / s->num_blocks;
  q.c = s->c;
  q.W_a = p->W_a; q.W_x = p->W_x;
  q.b_a = p->b_a; q.b_x = p->b_x; q.Lambda = p->Lambda;
  q.conv_w = p->conv_w; q.conv_b = p->conv_b;
  if (s->conv_width == 0) q.conv_w = q.conv_b = nullptr;   // the kernels read a null tap array as x_t = u_t
}

// the complex-gated variant: D even, the D / 2 complex channels in num_blocks gate blocks
int check_cg_shape(const rglru_shape *s) {
  if (s->D % 2 != 0) return fail(RGLRU_ERR_INVALID_ARG, "D (%d) must be even: two real channels per complex one", s->D);
  if ((s->D / 2) % s->num_blocks != 0)
    return fail(RGLRU_ERR_INVALID_ARG, "D / 2 (%d) is not a multiple of num_blocks (%d)", s->D / 2, s->num_blocks);
  if (s->D / 2 / s->num_blocks > 1024)
    return fail(RGLRU_ERR_UNSUPPORTED, "%d complex channels per gate block exceed 1024", s->D / 2 / s->num_blocks);
  return RGLRU_OK;
}

int check_cg_params(const rglru_shape *s, const rglru_cg_params *p) {
  if (!p) return fail(RGLRU_ERR_INVALID_ARG, "params is NULL");
  const size_t ws = s->w_dtype == RGLRU_BF16 ? 2 : 4;
  CHECK(check_ptr(p->W_a, "params.W_a", ws, true));
  CHECK(check_ptr(p->W_x, "params.W_x", ws, true));
  CHECK(check_ptr(p->b_a, "params.b_a", 4, true));
  CHECK(check_ptr(p->b_x, "params.b_x", 4, true));
  CHECK(check_ptr(p->Lambda, "params.Lambda", 4, true));
  CHECK(check_ptr(p->theta, "params.theta", 4, true));
  CHECK(check_ptr(p->conv_w, "params.conv_w", 4, s->conv_width != 0));
  CHECK(check_ptr(p->conv_b, "params.conv_b", 4, false));
  return RGLRU_OK;
}

void fill_cg_params(Problem &q, const rglru_shape *s, const rglru_cg_params *p) {
  q.B = s->B; q.T = s->T; q.D = s->D;
  q.nb = s->num_blocks; q.bs = s->D / 2 / s->num_blocks;
  q.c = s->c;
  q.W_a = p->W_a; q.W_x = p->W_x;
  q.b_a = p->b_a; q.b_x = p->b_x; q.Lambda = p->Lambda; q.theta = p->theta;
  q.conv_w = p->conv_w; q.conv_b = p->conv_b;
  if (s->conv_width == 0) q.conv_w = q.conv_b = nullptr;
}

// dy between the merge adjoint and the backward: one fp32 tensor, or in bf16 storage two bf16
// tensors (dy as stored and what its rounding took away)
size_t merge_dy_part(const rglru_shape *s) {
  const size_t n = (size_t)s->B * s->T * s->D * (s->act_dtype == RGLRU_BF16 ? 2 : 4);
  return (n + 255) & ~(size_t)255;
}
size_t merge_dy_bytes(const rglru_shape *s) { return (s->act_dtype == RGLRU_BF16 ? 2 : 1) * merge_dy_part(s); }

// narrower gate blocks in bf16: the backward runs on a copy widened to 256-channel blocks
bool backward_via_padding(const rglru_shape *s) {
  return s->act_dtype == RGLRU_BF16 && backward_padded_block(s->D / s->num_blocks) && s->T >= 1 &&
         (size_t)s->T * s->num_blocks * 256 * 4 < ((size_t)1 << 32);
}

// the other multiples of 16 at widths that are multiples of 256: the backward's pointwise pass
// runs as passes on the tuned kernels (its workspace contains the generic kernels' own)
bool backward_in_passes(const rglru_shape *s) {
  return s->act_dtype == RGLRU_BF16 && forward_wide_block(s->D / s->num_blocks) && s->D % 256 == 0 &&
         s->T >= 1 && (size_t)s->B * s->T * s->D * 4 < ((size_t)1 << 31);
}

size_t workspace_need(const rglru_shape *s, int op);
size_t workspace_need(const rglru_shape *s, int op) {
  switch (op) {
    case RGLRU_OP_BACKWARD:
      if (s->act_dtype == RGLRU_BF16 && s->D / s->num_blocks == 256 &&
          (size_t)s->T * s->D * 4 < ((size_t)1 << 32))
        return backward_mfma_ws_bytes(s->B, s->T, s->D, s->num_blocks);
      if (backward_via_padding(s)) {
        // (the generic kernels remain the fallback for loosely aligned pointers)
        const size_t a = backward_padded_ws_bytes(s->B, s->T, s->D, s->num_blocks);
        const size_t b = backward_generic_ws_bytes(s->B, s->T, s->D, s->num_blocks);
        return a > b ? a : b;
      }
      if (backward_in_passes(s)) return backward_wide_ws_bytes(s->B, s->T, s->D, s->num_blocks);
      return backward_generic_ws_bytes(s->B, s->T, s->D, s->num_blocks);
    case RGLRU_OP_SCAN:
      if (s->act_dtype == RGLRU_BF16 && s->D % 256 == 0 && s->T >= 1)
        return scan_tiled_ws_bytes(s->B, s->T, s->D);
      return 0;
    case RGLRU_OP_FORWARD_PACKED:   // the fused kernel's own scratch, then the boundary masks
      if (s->act_dtype == RGLRU_BF16 && forward_mfma_block(s->D / s->num_blocks) && s->T >= 1)
        return forward_mfma_ws_bytes(s->B, s->T, s->D, s->num_blocks) + forward_mfma_mask_bytes(s->B, s->T);
      return forward_generic_ws_bytes(s->B, s->T, s->D);
    case RGLRU_OP_BACKWARD_PACKED: {   // fused kernels for blocks of 256 channels (the general kernels remain the
                                       // fallback for loosely aligned pointers), the general kernels otherwise
      const size_t gen = backward_generic_ws_bytes(s->B, s->T, s->D, s->num_blocks);
      if (s->act_dtype == RGLRU_BF16 && s->D / s->num_blocks == 256 && (size_t)s->T * s->D * 4 < ((size_t)1 << 32)) {
        const size_t fused = backward_mfma_packed_ws_bytes(s->B, s->T, s->D, s->num_blocks);
        return fused > gen ? fused : gen;
      }
      return gen;
    }
    case RGLRU_OP_CG_BACKWARD:
      return cg_backward_ws_bytes(s->B, s->T, s->D, s->num_blocks);
    case RGLRU_OP_CG_FORWARD:   // optional: the two-pass forward of the general kernels
      return forward_generic_ws_bytes(s->B, s->T, s->D);
    case RGLRU_OP_BACKWARD_MERGE:   // dy (+ dy_lo) between the merge adjoint and the backward, then the backward's own
      return merge_dy_bytes(s) + workspace_need(s, RGLRU_OP_BACKWARD);
    case RGLRU_OP_FORWARD_MERGE:
    case RGLRU_OP_FORWARD:
      if (s->act_dtype == RGLRU_BF16 && forward_mfma_block(s->D / s->num_blocks) && s->T >= 1)
        return forward_mfma_ws_bytes(s->B, s->T, s->D, s->num_blocks);
      if (s->act_dtype == RGLRU_BF16 && forward_wide_block(s->D / s->num_blocks) && s->T >= 1 &&
          s->D % 256 == 0 && (size_t)s->B * s->T * s->D * 2 < ((size_t)1 << 31))
        return forward_wide_ws_bytes(s->B, s->T, s->D, s->num_blocks);
      return forward_generic_ws_bytes(s->B, s->T, s->D);   // the general kernels, two passes
    default:
      return 0;
  }
}

bool forward_on_general_kernels(const rglru_shape *s) {
  const bool bf = s->act_dtype == RGLRU_BF16;
  if (bf && forward_mfma_block(s->D / s->num_blocks) && s->T >= 1) return false;
  if (bf && forward_wide_block(s->D / s->num_blocks) && s->T >= 1 && s->D % 256 == 0 &&
      (size_t)s->B * s->T * s->D * 2 < ((size_t)1 << 31))
    return false;
  return true;
}

}  // namespace

// ---- benchmark timing
namespace {
constexpr int MAX_TIMED = 8192;
struct TimedRecord {
  const char *name;
  hipEvent_t start, stop;
};
thread_local bool g_timing = false;
thread_local int g_ntimed = 0;
thread_local TimedRecord *g_timed = nullptr;   // events are created once and reused
thread_local int g_events_made = 0;
thread_local char g_only[64] = "";             // if not empty: the only kernel name that is timed
}  // namespace

rglru::KernelTimer::KernelTimer(const char *name, hipStream_t stream) : s(stream), slot(-1) {
  if (!g_timing || g_ntimed >= MAX_TIMED) return;
  if (g_only[0] && strcmp(g_only, name) != 0) return;
  if (!g_timed) g_timed = new TimedRecord[MAX_TIMED];
  if (g_ntimed >= g_events_made) {
    if (hipEventCreate(&g_timed[g_ntimed].start) != hipSuccess) return;
    if (hipEventCreate(&g_timed[g_ntimed].stop) != hipSuccess) return;
    g_events_made = g_ntimed + 1;
  }
  slot = g_ntimed++;
  g_timed[slot].name = name;
  (void)hipEventRecord(g_timed[slot].start, s);
}
rglru::KernelTimer::~KernelTimer() {
  if (slot >= 0) (void)hipEventRecord(g_timed[slot].stop, s);
}

namespace {
int backward_checks(const rglru_shape *shape, const rglru_params *params, const void *u,
                    const float *h0, const void *conv_state_in, int64_t pos0, const void *y,
                    const void *dy, const float *dhT, void *du, float *dh0,
                    const rglru_param_grads *grads, void *workspace, size_t workspace_bytes,
                    bool with_workspace = true) {
  CHECK(check_shape(shape, true, true, 1));
  CHECK(check_params(shape, params));
  const size_t as = act_size(shape);
  if (pos0 < 0) return fail(RGLRU_ERR_INVALID_ARG, "pos0 must be >= 0");
  CHECK(check_ptr(u, "u", as, true));
  CHECK(check_ptr(y, "y", as, true));
  CHECK(check_ptr(dy, "dy", as, true));
  CHECK(check_ptr(du, "du", as, true));
  CHECK(check_ptr(h0, "h0", 4, false));
  CHECK(check_ptr(dhT, "dhT", 4, false));
  CHECK(check_ptr(dh0, "dh0", 4, false));
  CHECK(check_ptr(conv_state_in, "conv_state_in", as, false));
  if (!grads) return fail(RGLRU_ERR_INVALID_ARG, "grads is NULL");
  CHECK(check_ptr(grads->dW_a, "grads.dW_a", 4, true));
  CHECK(check_ptr(grads->dW_x, "grads.dW_x", 4, true));
  CHECK(check_ptr(grads->db_a, "grads.db_a", 4, true));
  CHECK(check_ptr(grads->db_x, "grads.db_x", 4, true));
  CHECK(check_ptr(grads->dLambda, "grads.dLambda", 4, true));
  CHECK(check_ptr(grads->dconv_w, "grads.dconv_w", 4, shape->conv_width != 0));
  CHECK(check_ptr(grads->dconv_b, "grads.dconv_b", 4, false));
  if (with_workspace)
    CHECK(check_workspace(workspace, workspace_bytes, workspace_need(shape, RGLRU_OP_BACKWARD)));
  return RGLRU_OK;
}
}  // namespace

namespace {
// the forward over whole sequences on the fastest kernels that take the shape; y and the new
// ring state are written
int forward_dispatch(const Problem &q, bool bf, hipStream_t s) {
  hipError_t e;
  if (forward_mfma_supported(q, bf)) {
    e = launch_forward_mfma(q, s);  // writes the new ring state itself
  } else if (forward_wide_supported(q, bf) && q.ws &&
             q.ws_bytes >= forward_wide_ws_bytes(q.B, q.T, q.D, q.nb)) {
    e = launch_forward_wide(q, s);
  } else {
    e = launch_forward_generic(q, bf, s);
    if (e != hipSuccess) return hip_fail(e, "forward launch");
    // the generic kernels never wait on each other; where the shape would have taken kernels
    // that do (pointers too loosely aligned for them), their status word is cleared all the same
    if (q.ws && q.ws_bytes >= 256) {
      e = launch_clear(q.ws, 16, s);
      if (e != hipSuccess) return hip_fail(e, "forward launch");
    }
    // the new ring state is written after the last read of the incoming one (they may alias)
    e = launch_state_update(q, bf, s);
  }
  if (e != hipSuccess) return hip_fail(e, "forward launch");
  return RGLRU_OK;
}
}  // namespace

extern "C" {

int rglru_timing_enable(int enable) {
  g_timing = enable != 0;
  if (g_timing) g_ntimed = 0;
  return RGLRU_OK;
}

int rglru_timing_select(const char *kernel_name) {
  if (kernel_name && strlen(kernel_name) >= sizeof(g_only))
    return fail(RGLRU_ERR_INVALID_ARG, "kernel name longer than %zu characters", sizeof(g_only) - 1);
  snprintf(g_only, sizeof(g_only), "%s", kernel_name ? kernel_name : "");
  return RGLRU_OK;
}

int rglru_timing_count(void) { return g_ntimed; }

int rglru_timing_get(int index, const char **name, float *ms) {
  if (index < 0 || index >= g_ntimed || !name || !ms)
    return fail(RGLRU_ERR_INVALID_ARG, "timing record %d does not exist", index);
  *name = g_timed[index].name;
  hipError_t e = hipEventElapsedTime(ms, g_timed[index].start, g_timed[index].stop);
  if (e != hipSuccess) return hip_fail(e, "hipEventElapsedTime");
  return RGLRU_OK;
}

const char *rglru_last_error(void) { return g_err; }

int rglru_version(void) { return 320; }

int rglru_set_max_time_slices(int max_slices) {
  if (max_slices < 0) return fail(RGLRU_ERR_INVALID_ARG, "max_slices must be >= 0 (0 = automatic)");
  rglru::mfma::set_slice_cap(max_slices);
  return RGLRU_OK;
}

size_t rglru_workspace_bytes(const rglru_shape *shape, int op) {
  if (op < RGLRU_OP_CONV1D || op > RGLRU_OP_CG_FORWARD) return 0;
  char keep[sizeof(g_err)];
  memcpy(keep, g_err, sizeof(g_err));
  const bool blocks = op != RGLRU_OP_CONV1D && op != RGLRU_OP_SCAN;
  const bool bwd = op == RGLRU_OP_BACKWARD || op == RGLRU_OP_BACKWARD_MERGE || op == RGLRU_OP_BACKWARD_PACKED ||
                   op == RGLRU_OP_CG_BACKWARD;
  int rc = check_shape(shape, blocks, op != RGLRU_OP_DECODE, bwd ? 1 : 0);
  if (rc == RGLRU_OK && (op == RGLRU_OP_CG_BACKWARD || op == RGLRU_OP_CG_FORWARD)) rc = check_cg_shape(shape);
  memcpy(g_err, keep, sizeof(g_err));  // a size query does not disturb the error string
  if (rc != RGLRU_OK) return 0;
  return workspace_need(shape, op);
}

int rglru_workspace_status(const rglru_shape *shape, int op, const void *workspace, void *stream) {
  if (op != RGLRU_OP_FORWARD && op != RGLRU_OP_BACKWARD && op != RGLRU_OP_SCAN &&
      op != RGLRU_OP_FORWARD_MERGE && op != RGLRU_OP_BACKWARD_MERGE && op != RGLRU_OP_FORWARD_PACKED &&
      op != RGLRU_OP_BACKWARD_PACKED)
    return fail(RGLRU_ERR_INVALID_ARG, "op %d has no workspace status", op);
  const bool bwd = op == RGLRU_OP_BACKWARD || op == RGLRU_OP_BACKWARD_MERGE || op == RGLRU_OP_BACKWARD_PACKED;
  CHECK(check_shape(shape, op != RGLRU_OP_SCAN, true, bwd ? 1 : 0));
  const size_t need = workspace_need(shape, op);
  hipError_t e = hipStreamSynchronize((hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "hipStreamSynchronize");
  if (need == 0) return RGLRU_OK;   // no time slices, no waits
  if ((op == RGLRU_OP_FORWARD || op == RGLRU_OP_FORWARD_MERGE || op == RGLRU_OP_FORWARD_PACKED) &&
      forward_on_general_kernels(shape))
    return RGLRU_OK;                // the general kernels never wait on each other (their scratch is optional)
  if (!workspace) return fail(RGLRU_ERR_INVALID_ARG, "workspace is NULL");
  size_t off = 0;   // forward and scan keep the flag in the first word
  if ((op == RGLRU_OP_FORWARD || op == RGLRU_OP_FORWARD_MERGE) &&
      !forward_mfma_block(shape->D / shape->num_blocks)) {   // (packed: no workspace at these block sizes)
    // the passes of the other block sizes: only the scan waits, its workspace follows the
    // activation-sized buffers
    const size_t sw = scan_tiled_ws_bytes(shape->B, shape->T, shape->D);
    if (sw == 0) return RGLRU_OK;
    off = need - sw;
  }
  if (bwd) {
    if (shape->act_dtype == RGLRU_BF16 && shape->D / shape->num_blocks == 256 &&
        (size_t)shape->T * shape->D * 4 < ((size_t)1 << 32))
      off = backward_mfma_flag_offset(shape->B, shape->T, shape->D, shape->num_blocks);
    else if (op == RGLRU_OP_BACKWARD_PACKED)
      return RGLRU_OK;              // packed sequences at other block sizes: the general kernels
    else if (backward_via_padding(shape))
      off = backward_padded_flag_offset(shape->B, shape->T, shape->D, shape->num_blocks);
    else if (backward_in_passes(shape) &&
             (off = backward_wide_flag_offset(shape->B, shape->T, shape->D, shape->num_blocks)) != 0)
      ;                             // only the adjoint scan of that path waits
    else
      return RGLRU_OK;              // the generic kernels do not wait on each other
    if (op == RGLRU_OP_BACKWARD_MERGE) off += merge_dy_bytes(shape);
  }
  int flag = 0;
  e = hipMemcpy(&flag, (const char *)workspace + off, sizeof(flag), hipMemcpyDeviceToHost);
  if (e != hipSuccess) return hip_fail(e, "hipMemcpy");
  if (flag != 0) {
    // reported once: the word is cleared, so that the next call on this workspace starts afresh
    e = hipMemset((char *)const_cast<void *>(workspace) + off, 0, 16);
    if (e != hipSuccess) return hip_fail(e, "hipMemset");
    return fail(RGLRU_ERR_TIMEOUT, "a bounded wait between workgroups expired: the outputs of the calls on this "
                                   "workspace since then are invalid (filled with NaN)");
  }
  g_err[0] = 0;
  return RGLRU_OK;
}

int rglru_conv1d(const rglru_shape *shape, const void *u, const float *conv_w,
                 const float *conv_b, const void *conv_state_in, int64_t pos0, void *x_out,
                 void *conv_state_out, void *stream) {
  CHECK(check_shape(shape, false, true, 0, false));
  const size_t as = act_size(shape);
  if (pos0 < 0) return fail(RGLRU_ERR_INVALID_ARG, "pos0 must be >= 0");
  CHECK(check_ptr(u, "u", as, shape->T > 0));
  CHECK(check_ptr(x_out, "x_out", as, shape->T > 0));
  CHECK(check_ptr(conv_w, "conv_w", 4, true));
  CHECK(check_ptr(conv_b, "conv_b", 4, false));
  CHECK(check_ptr(conv_state_in, "conv_state_in", as, false));
  CHECK(check_ptr(conv_state_out, "conv_state_out", as, false));

  Problem q;
  memset(&q, 0, sizeof(q));
  q.B = shape->B; q.T = shape->T; q.D = shape->D; q.nb = 1; q.bs = shape->D;
  q.c = shape->c; q.pos0 = pos0;
  q.u = u; q.conv_w = conv_w; q.conv_b = conv_b;
  q.state_in = conv_state_in; q.state_out = conv_state_out;
  const bool bf = shape->act_dtype == RGLRU_BF16;
  hipStream_t s = (hipStream_t)stream;
  hipError_t e = launch_conv1d_generic(q, bf, x_out, s);
  if (e != hipSuccess) return hip_fail(e, "conv1d launch");
  e = launch_state_update(q, bf, s);
  if (e != hipSuccess) return hip_fail(e, "conv state launch");
  g_err[0] = 0;
  return RGLRU_OK;
}

int rglru_forward(const rglru_shape *shape, const rglru_params *params, const void *u,
                  const float *h0, const void *conv_state_in, int64_t pos0, void *y, float *hT,
                  void *conv_state_out, void *workspace, size_t workspace_bytes, void *stream) {
  CHECK(check_shape(shape, true, true, 0));
  CHECK(check_params(shape, params));
  const size_t as = act_size(shape);
  if (pos0 < 0) return fail(RGLRU_ERR_INVALID_ARG, "pos0 must be >= 0");
  CHECK(check_ptr(u, "u", as, shape->T > 0));
  CHECK(check_ptr(y, "y", as, shape->T > 0));
  CHECK(check_ptr(h0, "h0", 4, false));
  CHECK(check_ptr(hT, "hT", 4, false));
  CHECK(check_ptr(conv_state_in, "conv_state_in", as, false));
  CHECK(check_ptr(conv_state_out, "conv_state_out", as, false));
  CHECK(check_forward_workspace(shape, workspace, workspace_bytes, workspace_need(shape, RGLRU_OP_FORWARD)));

  Problem q;
  memset(&q, 0, sizeof(q));
  fill_params(q, shape, params);
  q.pos0 = pos0; q.u = u; q.h0 = h0; q.state_in = conv_state_in;
  q.y = y; q.hT = hT; q.state_out = conv_state_out;
  if (shape->conv_width == 0) q.state_in = q.state_out = nullptr;   // no Conv1D, no ring
  q.ws = workspace; q.ws_bytes = workspace_bytes;
  const bool bf = shape->act_dtype == RGLRU_BF16;
  hipStream_t s = (hipStream_t)stream;
  CHECK(forward_dispatch(q, bf, s));
  g_err[0] = 0;
  return RGLRU_OK;
}

int rglru_forward_packed(const rglru_shape *shape, const rglru_params *params, const void *u,
                         const uint8_t *reset, const float *h0, const void *conv_state_in, int64_t pos0,
                         void *y, float *hT, void *conv_state_out, void *workspace, size_t workspace_bytes,
                         void *stream) {
  CHECK(check_shape(shape, true, true, 0));
  CHECK(check_params(shape, params));
  const size_t as = act_size(shape);
  if (pos0 < 0) return fail(RGLRU_ERR_INVALID_ARG, "pos0 must be >= 0");
  CHECK(check_ptr(u, "u", as, shape->T > 0));
  CHECK(check_ptr(y, "y", as, shape->T > 0));
  CHECK(check_ptr(reset, "reset", 1, false));
  CHECK(check_ptr(h0, "h0", 4, false));
  CHECK(check_ptr(hT, "hT", 4, false));
  CHECK(check_ptr(conv_state_in, "conv_state_in", as, false));
  CHECK(check_ptr(conv_state_out, "conv_state_out", as, false));
  CHECK(check_forward_workspace(shape, workspace, workspace_bytes, workspace_need(shape, RGLRU_OP_FORWARD_PACKED)));

  Problem q;
  memset(&q, 0, sizeof(q));
  fill_params(q, shape, params);
  q.pos0 = pos0; q.u = u; q.h0 = h0; q.state_in = conv_state_in; q.reset = reset;
  q.y = y; q.hT = hT; q.state_out = conv_state_out;
  if (shape->conv_width == 0) q.state_in = q.state_out = nullptr;
  q.ws = workspace; q.ws_bytes = workspace_bytes;
  const bool bf = shape->act_dtype == RGLRU_BF16;
  hipStream_t s = (hipStream_t)stream;
  hipError_t e;
  if (forward_mfma_supported(q, bf)) {
    e = launch_forward_mfma(q, s);   // the fused kernel takes the boundaries as bit masks per tile
  } else {
    e = launch_forward_generic(q, bf, s);
    // where the shape would have taken the fused kernel (pointers too loosely aligned for it),
    // its status word is cleared all the same
    if (e == hipSuccess && q.ws && q.ws_bytes >= 256) e = launch_clear(q.ws, 16, s);
    // the new ring state is written after the last read of the incoming one (they may alias)
    if (e == hipSuccess) e = launch_state_update(q, bf, s);
  }
  if (e != hipSuccess) return hip_fail(e, "forward launch");
  g_err[0] = 0;
  return RGLRU_OK;
}

int rglru_scan(const rglru_shape *shape, const void *a, const void *g, const float *h0,
               unsigned flags, void *h, float *hT, void *workspace, size_t workspace_bytes,
               void *stream) {
  CHECK(check_shape(shape, false, true, 0));
  if (flags & ~(RGLRU_SCAN_LOG_A | RGLRU_SCAN_NO_INPUT_SCALE | RGLRU_SCAN_ADJOINT))
    return fail(RGLRU_ERR_INVALID_ARG, "unknown scan flags 0x%x", flags);
  if ((flags & RGLRU_SCAN_ADJOINT) && !(flags & RGLRU_SCAN_NO_INPUT_SCALE))
    return fail(RGLRU_ERR_INVALID_ARG, "scan flags: RGLRU_SCAN_ADJOINT needs RGLRU_SCAN_NO_INPUT_SCALE");
  const size_t as = act_size(shape);
  CHECK(check_ptr(a, "a", as, shape->T > 0));
  CHECK(check_ptr(g, "g", as, shape->T > 0));
  CHECK(check_ptr(h, "h", as, shape->T > 0));
  CHECK(check_ptr(h0, "h0", 4, false));
  CHECK(check_ptr(hT, "hT", 4, false));
  CHECK(check_workspace(workspace, workspace_bytes, workspace_need(shape, RGLRU_OP_SCAN)));

  ScanProblem q;
  memset(&q, 0, sizeof(q));
  q.B = shape->B; q.T = shape->T; q.D = shape->D; q.flags = flags;
  q.a = a; q.g = g; q.h0 = h0; q.h = h; q.hT = hT;
  q.ws = workspace; q.ws_bytes = workspace_bytes;
  const bool bf = shape->act_dtype == RGLRU_BF16;
  hipStream_t s = (hipStream_t)stream;
  hipError_t e;
  if (scan_tiled_supported(q, bf)) {
    e = launch_scan_tiled(q, s);
  } else {
    e = launch_scan_generic(q, bf, s);
    if (e == hipSuccess && workspace && workspace_bytes >= 256) e = launch_clear(workspace, 16, s);
  }
  if (e != hipSuccess) return hip_fail(e, "scan launch");
  g_err[0] = 0;
  return RGLRU_OK;
}

int rglru_decode_step(const rglru_shape *shape, const rglru_params *params, const void *u_t,
                      float *h, void *conv_state, int64_t pos, void *y_t, void *stream) {
  CHECK(check_shape(shape, true, false, 0));
  CHECK(check_params(shape, params));
  const size_t as = act_size(shape);
  if (pos < 0) return fail(RGLRU_ERR_INVALID_ARG, "pos must be >= 0");
  CHECK(check_ptr(u_t, "u_t", as, true));
  CHECK(check_ptr(h, "h", 4, true));
  CHECK(check_ptr(conv_state, "conv_state", as, shape->conv_width != 0));
  CHECK(check_ptr(y_t, "y_t", as, true));

  Problem q;
  memset(&q, 0, sizeof(q));
  fill_params(q, shape, params);
  q.T = 1; q.pos0 = pos; q.u = u_t; q.hT = h; q.state_in = conv_state;
  q.state_out = conv_state; q.y = y_t;
  if (shape->conv_width == 0) q.state_in = q.state_out = nullptr;
  const bool bf = shape->act_dtype == RGLRU_BF16;
  hipError_t e = decode_mfma_supported(q, bf)   ? launch_decode_mfma(q, (hipStream_t)stream)
                 : decode_wide_supported(q, bf) ? launch_decode_wide(q, (hipStream_t)stream)
                                                : launch_decode_generic(q, bf, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "decode launch");
  g_err[0] = 0;
  return RGLRU_OK;
}

int rglru_decode_step_at(const rglru_shape *shape, const rglru_params *params, const void *u_t,
                         float *h, void *conv_state, const int64_t *pos, void *y_t, void *stream) {
  CHECK(check_shape(shape, true, false, 0));
  CHECK(check_params(shape, params));
  const size_t as = act_size(shape);
  CHECK(check_ptr(u_t, "u_t", as, true));
  CHECK(check_ptr(h, "h", 4, true));
  CHECK(check_ptr(conv_state, "conv_state", as, shape->conv_width != 0));
  CHECK(check_ptr(pos, "pos", 8, true));
  CHECK(check_ptr(y_t, "y_t", as, true));

  Problem q;
  memset(&q, 0, sizeof(q));
  fill_params(q, shape, params);
  q.T = 1; q.pos_rows = (const long long *)pos; q.u = u_t; q.hT = h; q.state_in = conv_state;
  q.state_out = conv_state; q.y = y_t;
  if (shape->conv_width == 0) q.state_in = q.state_out = nullptr;
  const bool bf = shape->act_dtype == RGLRU_BF16;
  hipError_t e = decode_mfma_supported(q, bf)   ? launch_decode_mfma(q, (hipStream_t)stream)
                 : decode_wide_supported(q, bf) ? launch_decode_wide(q, (hipStream_t)stream)
                                                : launch_decode_generic(q, bf, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "decode launch");
  g_err[0] = 0;
  return RGLRU_OK;
}

}  // extern "C"

namespace {
// rglru_backward with the upstream gradient given as dy + dy_lo (dy_lo null: dy alone)
int backward_run(const rglru_shape *shape, const rglru_params *params, const void *u,
                 const float *h0, const void *conv_state_in, int64_t pos0, const void *y,
                 const void *dy, const void *dy_lo, const float *dhT, void *du, float *dh0,
                 const rglru_param_grads *grads, void *workspace, size_t workspace_bytes,
                 void *stream) {
  CHECK(backward_checks(shape, params, u, h0, conv_state_in, pos0, y, dy, dhT, du, dh0, grads, workspace,
                        workspace_bytes));
  Problem q;
  memset(&q, 0, sizeof(q));
  fill_params(q, shape, params);
  q.pos0 = pos0; q.u = u; q.h0 = h0; q.state_in = conv_state_in;
  q.y_in = y; q.dy = dy; q.dy_lo = dy_lo; q.dhT = dhT; q.du = du; q.dh0 = dh0; q.g = *grads;
  if (shape->conv_width == 0) {   // no Conv1D: no carried inputs, no tap gradients
    q.state_in = nullptr;
    q.g.dconv_w = q.g.dconv_b = nullptr;
  }
  q.ws = workspace; q.ws_bytes = workspace_bytes;
  const bool bf = shape->act_dtype == RGLRU_BF16;
  hipError_t e;
  if (backward_mfma_supported(q, bf)) {
    e = launch_backward_mfma(q, (hipStream_t)stream);
  } else if (backward_padded_supported(q, bf)) {
    e = launch_backward_padded(q, (hipStream_t)stream);
  } else if (backward_wide_supported(q, bf) &&
             workspace_bytes >= backward_wide_ws_bytes(shape->B, shape->T, shape->D, shape->num_blocks)) {
    e = launch_backward_wide(q, (hipStream_t)stream);
  } else {
    // pointers too loosely aligned for the MFMA kernels: the generic kernels need more scratch
    CHECK(check_workspace(workspace, workspace_bytes,
                          backward_generic_ws_bytes(shape->B, shape->T, shape->D, shape->num_blocks)));
    e = launch_backward_generic(q, bf, (hipStream_t)stream);
    // where the shape would have taken kernels that wait on each other, their timeout flag
    // lies inside the scratch the generic kernels have just used: leave it cleared
    if (e == hipSuccess && bf && shape->D / shape->num_blocks == 256 &&
        (size_t)shape->T * shape->D * 4 < ((size_t)1 << 32))
      e = launch_clear((char *)workspace + backward_mfma_flag_offset(shape->B, shape->T, shape->D, shape->num_blocks),
                       16, (hipStream_t)stream);
    else if (e == hipSuccess && backward_via_padding(shape))
      e = launch_clear((char *)workspace + backward_padded_flag_offset(shape->B, shape->T, shape->D, shape->num_blocks),
                       16, (hipStream_t)stream);
  }
  if (e != hipSuccess) return hip_fail(e, "backward launch");
  g_err[0] = 0;
  return RGLRU_OK;
}
}  // namespace

extern "C" {

int rglru_backward(const rglru_shape *shape, const rglru_params *params, const void *u,
                   const float *h0, const void *conv_state_in, int64_t pos0, const void *y,
                   const void *dy, const float *dhT, void *du, float *dh0,
                   const rglru_param_grads *grads, void *workspace, size_t workspace_bytes,
                   void *stream) {
  return backward_run(shape, params, u, h0, conv_state_in, pos0, y, dy, nullptr, dhT, du, dh0, grads, workspace,
                      workspace_bytes, stream);
}

int rglru_backward_packed(const rglru_shape *shape, const rglru_params *params, const void *u,
                          const uint8_t *reset, const float *h0, const void *conv_state_in, int64_t pos0,
                          const void *y, const void *dy, const float *dhT, void *du, float *dh0,
                          const rglru_param_grads *grads, void *workspace, size_t workspace_bytes,
                          void *stream) {
  CHECK(backward_checks(shape, params, u, h0, conv_state_in, pos0, y, dy, dhT, du, dh0, grads, nullptr, 0,
                        false));
  CHECK(check_ptr(reset, "reset", 1, false));
  CHECK(check_workspace(workspace, workspace_bytes, workspace_need(shape, RGLRU_OP_BACKWARD_PACKED)));
  Problem q;
  memset(&q, 0, sizeof(q));
  fill_params(q, shape, params);
  q.pos0 = pos0; q.u = u; q.h0 = h0; q.state_in = conv_state_in; q.reset = reset;
  q.y_in = y; q.dy = dy; q.dhT = dhT; q.du = du; q.dh0 = dh0; q.g = *grads;
  if (shape->conv_width == 0) {
    q.state_in = nullptr;
    q.g.dconv_w = q.g.dconv_b = nullptr;
  }
  q.ws = workspace; q.ws_bytes = workspace_bytes;
  const bool bf = shape->act_dtype == RGLRU_BF16;
  hipError_t e;
  if (reset && backward_mfma_supported(q, bf)) {
    e = launch_backward_mfma(q, (hipStream_t)stream);   // the fused kernels take the boundaries as bit masks
  } else {
    e = launch_backward_generic(q, bf, (hipStream_t)stream);
    // where the shape would have taken the fused kernels, their status word lies inside the
    // scratch the general kernels have just used: leave it cleared
    if (e == hipSuccess && bf && shape->D / shape->num_blocks == 256 &&
        (size_t)shape->T * shape->D * 4 < ((size_t)1 << 32))
      e = launch_clear((char *)workspace + backward_mfma_flag_offset(shape->B, shape->T, shape->D, shape->num_blocks),
                       16, (hipStream_t)stream);
  }
  if (e != hipSuccess) return hip_fail(e, "backward launch");
  g_err[0] = 0;
  return RGLRU_OK;
}

int rglru_forward_merge(const rglru_shape *shape, const rglru_params *params, const void *u,
                        const void *branch, const float *h0, const void *conv_state_in,
                        int64_t pos0, unsigned flags, void *out, void *y, float *hT,
                        void *conv_state_out, void *workspace, size_t workspace_bytes,
                        void *stream) {
  CHECK(check_shape(shape, true, true, 0));
  CHECK(check_params(shape, params));
  if (flags & ~(RGLRU_MERGE_GELU_TANH | RGLRU_MERGE_SEPARATE))
    return fail(RGLRU_ERR_INVALID_ARG, "unknown merge flags 0x%x", flags);
  const size_t as = act_size(shape);
  if (pos0 < 0) return fail(RGLRU_ERR_INVALID_ARG, "pos0 must be >= 0");
  CHECK(check_ptr(u, "u", as, shape->T > 0));
  CHECK(check_ptr(branch, "branch", as, shape->T > 0));
  CHECK(check_ptr(out, "out", as, shape->T > 0));
  CHECK(check_ptr(y, "y", as, false));
  CHECK(check_ptr(h0, "h0", 4, false));
  CHECK(check_ptr(hT, "hT", 4, false));
  CHECK(check_ptr(conv_state_in, "conv_state_in", as, false));
  CHECK(check_ptr(conv_state_out, "conv_state_out", as, false));
  CHECK(check_forward_workspace(shape, workspace, workspace_bytes, workspace_need(shape, RGLRU_OP_FORWARD_MERGE)));
  if (shape->T > 0 && (out == y || out == branch || out == u))
    return fail(RGLRU_ERR_INVALID_ARG, "out must not alias y, branch or u");

  Problem q;
  memset(&q, 0, sizeof(q));
  fill_params(q, shape, params);
  q.pos0 = pos0; q.u = u; q.h0 = h0; q.state_in = conv_state_in;
  q.hT = hT; q.state_out = conv_state_out;
  if (shape->conv_width == 0) q.state_in = q.state_out = nullptr;
  q.ws = workspace; q.ws_bytes = workspace_bytes;
  const bool bf = shape->act_dtype == RGLRU_BF16;
  const bool tanh_form = (flags & RGLRU_MERGE_GELU_TANH) != 0;
  hipStream_t s = (hipStream_t)stream;
  hipError_t e;
  q.merge = tanh_form ? 2 : 1; q.branch = branch; q.out = out; q.y = y;
  if (!(flags & RGLRU_MERGE_SEPARATE) && forward_mfma_supported(q, bf) && forward_mfma_merge_fused(q)) {
    e = launch_forward_mfma(q, s);
    if (e != hipSuccess) return hip_fail(e, "forward launch");
    g_err[0] = 0;
    return RGLRU_OK;
  }
  // without the fused epilogue: y goes to its own buffer, or through `out` when it is not kept
  q.merge = 0;
  q.y = y ? y : out;
  CHECK(forward_dispatch(q, bf, s));
  e = launch_merge_forward(q.y, branch, out, (size_t)shape->B * shape->T * shape->D, bf, tanh_form, s);
  if (e != hipSuccess) return hip_fail(e, "merge launch");
  g_err[0] = 0;
  return RGLRU_OK;
}

int rglru_decode_step_merge(const rglru_shape *shape, const rglru_params *params, const void *u_t,
                            const void *branch_t, float *h, void *conv_state, int64_t pos,
                            unsigned flags, void *out_t, void *stream) {
  CHECK(check_shape(shape, true, false, 0));
  CHECK(check_params(shape, params));
  if (flags & ~RGLRU_MERGE_GELU_TANH) return fail(RGLRU_ERR_INVALID_ARG, "unknown merge flags 0x%x", flags);
  const size_t as = act_size(shape);
  if (pos < 0) return fail(RGLRU_ERR_INVALID_ARG, "pos must be >= 0");
  CHECK(check_ptr(u_t, "u_t", as, true));
  CHECK(check_ptr(branch_t, "branch_t", as, true));
  CHECK(check_ptr(h, "h", 4, true));
  CHECK(check_ptr(conv_state, "conv_state", as, shape->conv_width != 0));
  CHECK(check_ptr(out_t, "out_t", as, true));
  if (out_t == branch_t || out_t == u_t)
    return fail(RGLRU_ERR_INVALID_ARG, "out_t must not alias branch_t or u_t");

  Problem q;
  memset(&q, 0, sizeof(q));
  fill_params(q, shape, params);
  q.T = 1; q.pos0 = pos; q.u = u_t; q.hT = h; q.state_in = conv_state;
  q.state_out = conv_state; q.y = out_t;
  if (shape->conv_width == 0) q.state_in = q.state_out = nullptr;
  const bool bf = shape->act_dtype == RGLRU_BF16;
  const bool tanh_form = (flags & RGLRU_MERGE_GELU_TANH) != 0;
  hipStream_t s = (hipStream_t)stream;
  q.merge = tanh_form ? 2 : 1; q.branch = branch_t;
  hipError_t e;
  if (decode_mfma_supported(q, bf)) {
    e = launch_decode_mfma(q, s);
    if (e != hipSuccess) return hip_fail(e, "decode launch");
  } else if (decode_wide_supported(q, bf)) {
    e = launch_decode_wide(q, s);
    if (e != hipSuccess) return hip_fail(e, "decode launch");
  } else {
    q.merge = 0;
    e = launch_decode_generic(q, bf, s);
    if (e != hipSuccess) return hip_fail(e, "decode launch");
    e = launch_merge_forward(out_t, branch_t, out_t, (size_t)shape->B * shape->D, bf, tanh_form, s);
    if (e != hipSuccess) return hip_fail(e, "merge launch");
  }
  g_err[0] = 0;
  return RGLRU_OK;
}

int rglru_backward_merge(const rglru_shape *shape, const rglru_params *params, const void *u,
                         const void *branch, const float *h0, const void *conv_state_in,
                         int64_t pos0, unsigned flags, const void *y, const void *dout,
                         const float *dhT, void *du, void *dbranch, float *dh0,
                         const rglru_param_grads *grads, void *workspace,
                         size_t workspace_bytes, void *stream) {
  CHECK(check_shape(shape, true, true, 1));
  if (flags & ~RGLRU_MERGE_GELU_TANH) return fail(RGLRU_ERR_INVALID_ARG, "unknown merge flags 0x%x", flags);
  const size_t as = act_size(shape);
  CHECK(check_ptr(branch, "branch", as, true));
  CHECK(check_ptr(y, "y", as, true));
  CHECK(check_ptr(dout, "dout", as, true));
  CHECK(check_ptr(dbranch, "dbranch", as, true));
  CHECK(check_workspace(workspace, workspace_bytes, workspace_need(shape, RGLRU_OP_BACKWARD_MERGE)));
  if (dbranch == y || dbranch == u || dbranch == du)
    return fail(RGLRU_ERR_INVALID_ARG, "dbranch must not alias y, u or du");
  // the rest of the arguments are checked by rglru_backward before anything is launched:
  // a dry run of its checks first, so that a bad argument leaves every output untouched
  const size_t dyb = merge_dy_bytes(shape);
  const bool bf = shape->act_dtype == RGLRU_BF16;
  void *dy = workspace;
  void *dy_lo = bf ? (char *)workspace + merge_dy_part(shape) : nullptr;
  void *rest = (char *)workspace + dyb;
  CHECK(backward_checks(shape, params, u, h0, conv_state_in, pos0, y, dy, dhT, du, dh0, grads, rest,
                        workspace_bytes - dyb));
  hipError_t e = launch_merge_backward(y, branch, dout, dy, dy_lo, dbranch,
                                       (size_t)shape->B * shape->T * shape->D, bf,
                                       (flags & RGLRU_MERGE_GELU_TANH) != 0, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "merge launch");
  return backward_run(shape, params, u, h0, conv_state_in, pos0, y, dy, dy_lo, dhT, du, dh0, grads, rest,
                      workspace_bytes - dyb, stream);
}

int rglru_cg_forward(const rglru_shape *shape, const rglru_cg_params *params, const void *u,
                     const float *h0, const void *conv_state_in, int64_t pos0, void *y, float *hT,
                     void *conv_state_out, void *workspace, size_t workspace_bytes, void *stream) {
  CHECK(check_shape(shape, true, true, 0));
  CHECK(check_cg_shape(shape));
  if (workspace && !aligned(workspace, 256)) return fail(RGLRU_ERR_INVALID_ARG, "workspace is not 256-byte aligned");
  CHECK(check_cg_params(shape, params));
  const size_t as = act_size(shape);
  if (pos0 < 0) return fail(RGLRU_ERR_INVALID_ARG, "pos0 must be >= 0");
  CHECK(check_ptr(u, "u", as, shape->T > 0));
  CHECK(check_ptr(y, "y", as, shape->T > 0));
  CHECK(check_ptr(h0, "h0", 4, false));
  CHECK(check_ptr(hT, "hT", 4, false));
  CHECK(check_ptr(conv_state_in, "conv_state_in", as, false));
  CHECK(check_ptr(conv_state_out, "conv_state_out", as, false));
  Problem q;
  memset(&q, 0, sizeof(q));
  fill_cg_params(q, shape, params);
  q.pos0 = pos0; q.u = u; q.h0 = h0; q.state_in = conv_state_in;
  q.y = y; q.hT = hT; q.state_out = conv_state_out;
  if (shape->conv_width == 0) q.state_in = q.state_out = nullptr;
  q.ws = workspace; q.ws_bytes = workspace ? workspace_bytes : 0;
  const bool bf = shape->act_dtype == RGLRU_BF16;
  hipError_t e = launch_cg_forward(q, bf, (hipStream_t)stream);
  // the new ring state is written after the last read of the incoming one (they may alias)
  if (e == hipSuccess) e = launch_state_update(q, bf, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "forward launch");
  g_err[0] = 0;
  return RGLRU_OK;
}

int rglru_cg_decode_step(const rglru_shape *shape, const rglru_cg_params *params, const void *u_t,
                         float *h, void *conv_state, int64_t pos, void *y_t, void *stream) {
  CHECK(check_shape(shape, true, false, 0));
  CHECK(check_cg_shape(shape));
  CHECK(check_cg_params(shape, params));
  const size_t as = act_size(shape);
  if (pos < 0) return fail(RGLRU_ERR_INVALID_ARG, "pos must be >= 0");
  CHECK(check_ptr(u_t, "u_t", as, true));
  CHECK(check_ptr(h, "h", 4, true));
  CHECK(check_ptr(conv_state, "conv_state", as, shape->conv_width != 0));
  CHECK(check_ptr(y_t, "y_t", as, true));
  Problem q;
  memset(&q, 0, sizeof(q));
  fill_cg_params(q, shape, params);
  q.T = 1;
  q.pos0 = pos; q.u = u_t; q.hT = h; q.y = y_t;
  q.state_in = q.state_out = shape->conv_width == 0 ? nullptr : conv_state;
  const hipError_t e = launch_cg_decode(q, shape->act_dtype == RGLRU_BF16, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "decode launch");
  g_err[0] = 0;
  return RGLRU_OK;
}

int rglru_cg_backward(const rglru_shape *shape, const rglru_cg_params *params, const void *u,
                      const float *h0, const void *conv_state_in, int64_t pos0, const void *dy,
                      const float *dhT, void *du, float *dh0, const rglru_cg_param_grads *grads,
                      void *workspace, size_t workspace_bytes, void *stream) {
  CHECK(check_shape(shape, true, true, 1));
  CHECK(check_cg_shape(shape));
  CHECK(check_cg_params(shape, params));
  const size_t as = act_size(shape);
  if (pos0 < 0) return fail(RGLRU_ERR_INVALID_ARG, "pos0 must be >= 0");
  CHECK(check_ptr(u, "u", as, true));
  CHECK(check_ptr(dy, "dy", as, true));
  CHECK(check_ptr(du, "du", as, true));
  CHECK(check_ptr(h0, "h0", 4, false));
  CHECK(check_ptr(dhT, "dhT", 4, false));
  CHECK(check_ptr(dh0, "dh0", 4, false));
  CHECK(check_ptr(conv_state_in, "conv_state_in", as, false));
  if (!grads) return fail(RGLRU_ERR_INVALID_ARG, "grads is NULL");
  CHECK(check_ptr(grads->dW_a, "grads.dW_a", 4, true));
  CHECK(check_ptr(grads->dW_x, "grads.dW_x", 4, true));
  CHECK(check_ptr(grads->db_a, "grads.db_a", 4, true));
  CHECK(check_ptr(grads->db_x, "grads.db_x", 4, true));
  CHECK(check_ptr(grads->dLambda, "grads.dLambda", 4, true));
  CHECK(check_ptr(grads->dtheta, "grads.dtheta", 4, true));
  CHECK(check_ptr(grads->dconv_w, "grads.dconv_w", 4, shape->conv_width != 0));
  CHECK(check_ptr(grads->dconv_b, "grads.dconv_b", 4, false));
  CHECK(check_workspace(workspace, workspace_bytes, workspace_need(shape, RGLRU_OP_CG_BACKWARD)));
  Problem q;
  memset(&q, 0, sizeof(q));
  fill_cg_params(q, shape, params);
  q.pos0 = pos0; q.u = u; q.h0 = h0; q.state_in = conv_state_in;
  q.dy = dy; q.dhT = dhT; q.du = du; q.dh0 = dh0;
  q.g.dW_a = grads->dW_a; q.g.dW_x = grads->dW_x; q.g.db_a = grads->db_a; q.g.db_x = grads->db_x;
  q.g.dLambda = grads->dLambda; q.dtheta = grads->dtheta;
  q.g.dconv_w = grads->dconv_w; q.g.dconv_b = grads->dconv_b;
  if (shape->conv_width == 0) {
    q.state_in = nullptr;
    q.g.dconv_w = q.g.dconv_b = nullptr;
  }
  q.ws = workspace; q.ws_bytes = workspace_bytes;
  const hipError_t e = launch_cg_backward(q, shape->act_dtype == RGLRU_BF16, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "backward launch");
  g_err[0] = 0;
  return RGLRU_OK;
}

}  // extern "C"
