// Internal declarations shared by the translation units of librglru (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "rglru.h"

namespace rglru {

// bfloat16 storage type: raw bits; arithmetic always happens in fp32.
struct bf16 {
  unsigned short v;
};

__device__ __forceinline__ float ldf(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float ldf(const bf16 *p, size_t i) {
  return __uint_as_float(((unsigned)p[i].v) << 16);
}
// round-to-nearest-even, NaN kept quiet
__device__ __forceinline__ unsigned short f32_to_bf16_bits(float f) {
  unsigned u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;
  u += 0x7fffu + ((u >> 16) & 1u);
  return (unsigned short)(u >> 16);
}
// four consecutive elements from a 16-byte (fp32) / 8-byte (bf16) aligned position
__device__ __forceinline__ void ldf4(const float *p, size_t i, float (&o)[4]) {
  const float4 v = *(const float4 *)(p + i);
  o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
}
__device__ __forceinline__ void ldf4(const bf16 *p, size_t i, float (&o)[4]) {
  const uint2 v = *(const uint2 *)(p + i);
  o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
  o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
}
__device__ __forceinline__ void stf(float *p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void stf(bf16 *p, size_t i, float v) { p[i].v = f32_to_bf16_bits(v); }

// mathematical n mod 3 for the conv ring buffer (n may be negative)
__host__ __device__ __forceinline__ int ring_slot(long long n) {
  int r = (int)(n % 3);
  return r < 0 ? r + 3 : r;
}

// Everything a kernel needs to know about one call. Pointers are device pointers.
struct Problem {
  int B, T, D, nb, bs;
  float c;
  long long pos0;
  const long long *pos_rows;   // decode only: position per sequence (device, [B]) instead of pos0
  const void *u;
  const void *W_a, *W_x;
  const float *b_a, *b_x, *Lambda, *conv_w, *conv_b;   // conv_w null: no Conv1D, x_t = u_t (identity tap)
  const float *theta;   // complex-gated variant only: [D/2] phases of the recurrence weight
  float *dtheta;        //   and their gradient (backward)
  const float *h0;
  const void *state_in;
  const unsigned char *reset;  // [B][T] or null: non-zero where a new document starts (packed sequences):
                               // h_{t-1} := 0 and the Conv1D sees zeros before that step
  void *y;
  float *hT;
  void *state_out;
  // backward only
  const void *y_in, *dy;
  const void *dy_lo;    // bf16 storage only, may be null: dy is the sum of two bf16 tensors, dy + dy_lo
                        // (an upstream gradient the library formed itself and must not round to 8 bits)
  const float *dhT;
  void *du;
  float *dh0;
  rglru_param_grads g;
  void *ws;
  size_t ws_bytes;
  // merge epilogue (forward): out = y * GeLU(branch) goes to `out`, y itself to `y` if not null
  int merge;            // 0 none, 1 GeLU = z Phi(z), 2 tanh form
  const void *branch;
  void *out;
};

// internal scan flag (never accepted from the C ABI): g is stored in IEEE half precision; goes
// with RGLRU_SCAN_LOG_A | RGLRU_SCAN_NO_INPUT_SCALE and the tiled kernel only
constexpr unsigned SCAN_G_FP16 = 0x100u;
// internal: the adjoint scan writes delta in IEEE half precision (tiled kernel, log-decay form)
constexpr unsigned SCAN_OUT_FP16 = 0x200u;

// One rglru_scan call.
struct ScanProblem {
  int B, T, D;
  unsigned flags;
  const void *a, *g;
  const float *h0;
  void *h;
  float *hT;
  void *ws;
  size_t ws_bytes;
};

// sets the calling thread's error string (printf-style)
void set_last_error(const char *fmt, ...);

// Benchmark timing: brackets a kernel launch with HIP events when timing is enabled on this
// thread (see rglru_timing_enable in rglru.h). Usage: { KernelTimer t("name", stream); launch; }
struct KernelTimer {
  hipStream_t s;
  int slot;
  KernelTimer(const char *name, hipStream_t stream);
  ~KernelTimer();
};

// Launchers. Each returns hipSuccess or the launch error. `bf` selects bf16 act+weights.
hipError_t launch_conv1d_generic(const Problem &p, bool bf, void *x_out, hipStream_t s);
hipError_t launch_state_update(const Problem &p, bool bf, hipStream_t s);
hipError_t launch_forward_generic(const Problem &p, bool bf, hipStream_t s);   // (two passes, parallel over time, if p.ws holds forward_generic_ws_bytes)
size_t forward_generic_ws_bytes(int B, int T, int D);
hipError_t launch_decode_generic(const Problem &p, bool bf, hipStream_t s);
hipError_t launch_backward_generic(const Problem &p, bool bf, hipStream_t s);
size_t backward_generic_ws_bytes(int B, int T, int D, int nb);
// without the pointwise pass (and without the dgrad pass if the caller has added W^T dp + W^T dq to dx)
hipError_t launch_backward_generic_tail(const Problem &p, bool bf, hipStream_t s, bool with_dgrad = true,
                                        bool with_wgrad = true, bool with_du = true);
void backward_generic_arrays(const Problem &p, float **x, float **dp, float **dq, float **dx, float **partA);
// du from an fp32 dx [B][T][D] by a streaming kernel (bf16 storage, no document boundaries, aligned)
bool conv_adjoint_rows_applies(const Problem &p, bool bf);
hipError_t launch_conv_adjoint_rows(const Problem &p, const float *dx, hipStream_t s);
size_t generic_lds_bytes(int bs);

// Complex-gated variant (Appendix B): D real channels as D / 2 complex ones, Problem.bs = complex
// channels per gate block, W [nb][bs][2 bs]; shape-generic kernels. The backward's workspace is
// the real layer's generic one for the same B, T, D followed by the recomputed states in fp32.
size_t cg_backward_ws_bytes(int B, int T, int D, int nb);
hipError_t launch_cg_forward(const Problem &p, bool bf, hipStream_t s);
hipError_t launch_cg_decode(const Problem &p, bool bf, hipStream_t s);
hipError_t launch_cg_backward(const Problem &p, bool bf, hipStream_t s);

// MFMA forward (bf16 storage, gate blocks of 256)
bool forward_mfma_supported(const Problem &p, bool bf);
bool forward_mfma_block(int bs);   // gate block sizes the forward kernel takes
size_t forward_mfma_ws_bytes(int B, int T, int D, int nb);
size_t forward_mfma_mask_bytes(int B, int T);   // appended for packed sequences (Problem.reset)
hipError_t launch_forward_mfma(const Problem &p, hipStream_t s);
bool forward_mfma_merge_fused(const Problem &p);   // merge as epilogue (else: a kernel of its own)

// Forward for the other block sizes in bf16 (any multiple of 16): Conv1D, gate products + gates,
// scan as separate passes through the workspace
bool forward_wide_block(int bs);
bool forward_wide_supported(const Problem &p, bool bf);
size_t forward_wide_ws_bytes(int B, int T, int D, int nb);
hipError_t launch_forward_wide(const Problem &p, hipStream_t s);
bool backward_wide_supported(const Problem &p, bool bf);
size_t backward_wide_ws_bytes(int B, int T, int D, int nb);
size_t backward_wide_flag_offset(int B, int T, int D, int nb);
hipError_t launch_backward_wide(const Problem &p, hipStream_t s);
bool decode_wide_supported(const Problem &p, bool bf);
hipError_t launch_decode_wide(const Problem &p, hipStream_t s);

// MFMA decode step (bf16 storage, gate blocks of 256)
bool decode_mfma_supported(const Problem &p, bool bf);
hipError_t launch_decode_mfma(const Problem &p, hipStream_t s);

// MFMA backward (bf16 storage, gate blocks of 256)
bool backward_mfma_supported(const Problem &p, bool bf);
size_t backward_mfma_ws_bytes(int B, int T, int D, int nb);
size_t backward_mfma_packed_ws_bytes(int B, int T, int D, int nb);   // with the boundary masks of packed sequences (Problem.reset)
size_t backward_mfma_flag_offset(int B, int T, int D, int nb);   // byte offset of the timeout flag
hipError_t launch_backward_mfma(const Problem &p, hipStream_t s);

// Backward for narrower gate blocks: the problem widened to 256-channel blocks in the workspace
bool backward_padded_block(int bs);
bool backward_padded_supported(const Problem &p, bool bf);
size_t backward_padded_ws_bytes(int B, int T, int D, int nb);
size_t backward_padded_flag_offset(int B, int T, int D, int nb);
hipError_t launch_backward_padded(const Problem &p, hipStream_t s);

// sc (256 bytes of scratch) <- sc[1] = S, sc[2] = 1 / S with S the power of two that brings
// max(|dy|, |dhT|) into [2^shift, 2^(shift+1)); dy bf16 [n], dhT fp32 [nd] or null. Gradients are
// linear in dy: kernels that keep adjoints in half precision work on S dy and undo it at the end.
hipError_t launch_grad_scale(const void *dy, size_t n, const float *dhT, size_t nd, float *sc, int shift,
                             hipStream_t s);

// clears `bytes` (% 16 == 0) at a 16-byte aligned address with a fill kernel
hipError_t launch_clear(void *at, size_t bytes, hipStream_t s);

// Linear scan of eq. (4): any shape and storage type / bf16 storage with D % 256 == 0
hipError_t launch_scan_generic(const ScanProblem &p, bool bf, hipStream_t s);
bool scan_tiled_supported(const ScanProblem &p, bool bf);
size_t scan_tiled_ws_bytes(int B, int T, int D);
hipError_t launch_scan_tiled(const ScanProblem &p, hipStream_t s);


// The recurrent block's merge as kernels of its own (any shape and storage type)
//   forward:  out = y * GeLU(branch), n elements; out may alias y or branch
//   backward: dy = dout * GeLU(branch), dbranch = dout * y * GeLU'(branch)
hipError_t launch_merge_forward(const void *y, const void *branch, void *out, size_t n, bool bf,
                                bool tanh_form, hipStream_t s);
//   dy_lo (bf16 storage, may be null): dy - bf16(dy), so that dy + dy_lo carries 16 significant bits
hipError_t launch_merge_backward(const void *y, const void *branch, const void *dout, void *dy, void *dy_lo,
                                 void *dbranch, size_t n, bool bf, bool tanh_form, hipStream_t s);

}  // namespace rglru
