// Backward for gate blocks narrower than 256 channels (Section 4.1: 16 blocks; 160 channels at
// width 2560): the tuned backward kernels are built for 256-wide blocks, so the problem is
// widened to nb blocks of 256 channels - activations, states and parameters are copied into
// zero-padded buffers in the workspace, the tuned kernels run on those, and du and the
// parameter gradients are copied back. A padded channel has zero input, zero weights, zero
// state and zero upstream gradient: its state stays zero and every gradient it contributes is
// zero, so the existing channels see exactly the arithmetic of the narrow problem.
// Pure data movement, 16 bytes per lane; costs four streaming passes on top of a backward
// over 256 / bs times the channels.
#include "rglru_internal.h"

namespace rglru {
namespace {

constexpr int PBS = 256;
constexpr int PTHR = 256;

inline size_t al256(size_t n) { return (n + 255) & ~(size_t)255; }

struct ActPair {
  const uint4 *src;
  uint4 *dst;
};
struct ActArgs {
  ActPair t[3];
  int n;          // tensors
  size_t rows;    // B * T (or B * 3, B)
  int nb, cb;     // blocks, 16-byte chunks per narrow block (bs * esz / 16)
  int cp;         // chunks per padded block
};

// narrow [rows][nb][cb] chunks -> padded [rows][nb][cp] chunks, zero fill
__global__ void __launch_bounds__(PTHR) pad_rows_kernel(ActArgs a) {
  const size_t total = a.rows * a.nb * a.cp;
  for (size_t i = (size_t)blockIdx.x * PTHR + threadIdx.x; i < total; i += (size_t)gridDim.x * PTHR) {
    const int c = (int)(i % a.cp);
    const size_t rb = i / a.cp;   // row * nb + block
    for (int k = 0; k < a.n; ++k)
      a.t[k].dst[i] = c < a.cb ? a.t[k].src[rb * a.cb + c] : uint4{0, 0, 0, 0};
  }
}
// padded -> narrow
__global__ void __launch_bounds__(PTHR) unpad_rows_kernel(ActArgs a) {
  const size_t total = a.rows * a.nb * a.cb;
  for (size_t i = (size_t)blockIdx.x * PTHR + threadIdx.x; i < total; i += (size_t)gridDim.x * PTHR) {
    const int c = (int)(i % a.cb);
    const size_t rb = i / a.cb;
    for (int k = 0; k < a.n; ++k) a.t[k].dst[i] = a.t[k].src[rb * a.cp + c];
  }
}

struct MatArgs {
  const uint4 *src[2];
  uint4 *dst[2];
  int nb, bs, esz;   // esz: bytes per element (2 = bf16 weights in, 4 = fp32 gradients out)
};
// [nb][bs][bs] -> [nb][256][256], zero fill (rows and columns)
__global__ void __launch_bounds__(PTHR) pad_mats_kernel(MatArgs a) {
  const int cpr = PBS * a.esz / 16, cbr = a.bs * a.esz / 16;   // chunks per padded / narrow row
  const size_t total = (size_t)a.nb * PBS * cpr;
  for (size_t i = (size_t)blockIdx.x * PTHR + threadIdx.x; i < total; i += (size_t)gridDim.x * PTHR) {
    const int c = (int)(i % cpr);
    const int r = (int)((i / cpr) % PBS);
    const size_t g = i / ((size_t)cpr * PBS);
    const bool ok = c < cbr && r < a.bs;
    for (int k = 0; k < 2; ++k)
      a.dst[k][i] = ok ? a.src[k][(g * a.bs + r) * cbr + c] : uint4{0, 0, 0, 0};
  }
}
__global__ void __launch_bounds__(PTHR) unpad_mats_kernel(MatArgs a) {
  const int cpr = PBS * a.esz / 16, cbr = a.bs * a.esz / 16;
  const size_t total = (size_t)a.nb * a.bs * cbr;
  for (size_t i = (size_t)blockIdx.x * PTHR + threadIdx.x; i < total; i += (size_t)gridDim.x * PTHR) {
    const int c = (int)(i % cbr);
    const int r = (int)((i / cbr) % a.bs);
    const size_t g = i / ((size_t)cbr * a.bs);
    for (int k = 0; k < 2; ++k) a.dst[k][i] = a.src[k][(g * PBS + r) * cpr + c];
  }
}

constexpr int MAXV = 12;
struct VecArgs {
  const float *src[MAXV];   // nullptr: the destination row is zero filled / the row is skipped
  float *dst[MAXV];
  int n, nb, bs;
};
// fp32 rows [nb * bs] -> [nb * 256] (pad) or back (unpad), one element per thread
__global__ void __launch_bounds__(PTHR) pad_vecs_kernel(VecArgs a) {
  const int i = blockIdx.x * PTHR + threadIdx.x;
  if (i >= a.nb * PBS) return;
  const int g = i / PBS, c = i % PBS;
  for (int k = 0; k < a.n; ++k)
    a.dst[k][i] = (a.src[k] && c < a.bs) ? a.src[k][g * a.bs + c] : 0.f;
}
__global__ void __launch_bounds__(PTHR) unpad_vecs_kernel(VecArgs a) {
  const int i = blockIdx.x * PTHR + threadIdx.x;
  if (i >= a.nb * a.bs) return;
  const int g = i / a.bs, c = i % a.bs;
  for (int k = 0; k < a.n; ++k)
    if (a.dst[k]) a.dst[k][i] = a.src[k][g * PBS + c];
}

int grid_of(size_t total) {
  const size_t b = (total + PTHR - 1) / PTHR;
  return (int)(b < 1 ? 1 : (b > 256 * 32 ? 256 * 32 : b));
}

struct PadPlan {
  int Dp;
  size_t act, off_u, off_y, off_dy, off_dylo, off_du, off_wa, off_wx, off_vec, off_h0, off_dhT, off_dh0, off_state,
      off_dwa, off_dwx, off_gvec, off_inner, total;
};

PadPlan plan(int B, int T, int D, int nb) {
  PadPlan q;
  q.Dp = nb * PBS;
  q.act = al256((size_t)B * T * q.Dp * 2);
  size_t off = 0;
  q.off_u = off; off += q.act;
  q.off_y = off; off += q.act;
  q.off_dy = off; off += q.act;
  q.off_dylo = off; off += q.act;   // second half of an upstream gradient given as a sum of two tensors
  q.off_du = off; off += q.act;
  q.off_wa = off; off += al256((size_t)nb * PBS * PBS * 2);
  q.off_wx = off; off += al256((size_t)nb * PBS * PBS * 2);
  q.off_vec = off; off += al256((size_t)8 * q.Dp * 4);      // b_a, b_x, Lambda, conv_w[4], conv_b
  q.off_h0 = off; off += al256((size_t)B * q.Dp * 4);
  q.off_dhT = off; off += al256((size_t)B * q.Dp * 4);
  q.off_dh0 = off; off += al256((size_t)B * q.Dp * 4);
  q.off_state = off; off += al256((size_t)B * 3 * q.Dp * 2);
  q.off_dwa = off; off += al256((size_t)nb * PBS * PBS * 4);
  q.off_dwx = off; off += al256((size_t)nb * PBS * PBS * 4);
  q.off_gvec = off; off += al256((size_t)8 * q.Dp * 4);     // db_a, db_x, dLambda, dconv_w[4], dconv_b
  q.off_inner = off; off += backward_mfma_ws_bytes(B, T, q.Dp, nb);
  q.total = off;
  return q;
}

}  // namespace

bool backward_padded_block(int bs) { return bs % 16 == 0 && bs >= PBS / 2 && bs < PBS; }

bool backward_padded_supported(const Problem &p, bool bf) {
  auto al = [](const void *q) { return ((uintptr_t)q % 16) == 0; };
  return bf && backward_padded_block(p.bs) && p.T >= 1 &&
         (size_t)p.T * p.nb * PBS * 4 < ((size_t)1 << 32) && al(p.W_a) && al(p.W_x) && al(p.u) &&
         al(p.y_in) && al(p.dy) && al(p.dy_lo) && al(p.du) && (!p.state_in || al(p.state_in)) && al(p.g.dW_a) &&
         al(p.g.dW_x) && al(p.h0) && al(p.dhT) && al(p.dh0);
}

size_t backward_padded_ws_bytes(int B, int T, int D, int nb) { return plan(B, T, D, nb).total; }

size_t backward_padded_flag_offset(int B, int T, int D, int nb) {
  const PadPlan q = plan(B, T, D, nb);
  return q.off_inner + backward_mfma_flag_offset(B, T, q.Dp, nb);
}

hipError_t launch_backward_padded(const Problem &p, hipStream_t s) {
  const PadPlan q = plan(p.B, p.T, p.D, p.nb);
  char *ws = (char *)p.ws;
  const int Dp = q.Dp, nb = p.nb, bs = p.bs;
  float *vec = (float *)(ws + q.off_vec), *gvec = (float *)(ws + q.off_gvec);

  // ---- widen the inputs
  {
    KernelTimer kt("pad_kernel", s);
    ActArgs a;
    a.n = 3; a.rows = (size_t)p.B * p.T; a.nb = nb; a.cb = bs * 2 / 16; a.cp = PBS * 2 / 16;
    a.t[0] = {(const uint4 *)p.u, (uint4 *)(ws + q.off_u)};
    a.t[1] = {(const uint4 *)p.y_in, (uint4 *)(ws + q.off_y)};
    a.t[2] = {(const uint4 *)p.dy, (uint4 *)(ws + q.off_dy)};
    hipLaunchKernelGGL(pad_rows_kernel, dim3(grid_of(a.rows * nb * a.cp)), dim3(PTHR), 0, s, a);
    if (p.dy_lo) {
      ActArgs b = a;
      b.n = 1;
      b.t[0] = {(const uint4 *)p.dy_lo, (uint4 *)(ws + q.off_dylo)};
      hipLaunchKernelGGL(pad_rows_kernel, dim3(grid_of(b.rows * nb * b.cp)), dim3(PTHR), 0, s, b);
    }
    if (p.state_in) {
      ActArgs b = a;
      b.n = 1; b.rows = (size_t)p.B * 3;
      b.t[0] = {(const uint4 *)p.state_in, (uint4 *)(ws + q.off_state)};
      hipLaunchKernelGGL(pad_rows_kernel, dim3(grid_of(b.rows * nb * b.cp)), dim3(PTHR), 0, s, b);
    }
    if (p.h0 || p.dhT) {   // fp32 rows: 4 channels per chunk
      ActArgs b;
      b.n = 0; b.rows = (size_t)p.B; b.nb = nb; b.cb = bs * 4 / 16; b.cp = PBS * 4 / 16;
      if (p.h0) b.t[b.n++] = {(const uint4 *)p.h0, (uint4 *)(ws + q.off_h0)};
      if (p.dhT) b.t[b.n++] = {(const uint4 *)p.dhT, (uint4 *)(ws + q.off_dhT)};
      hipLaunchKernelGGL(pad_rows_kernel, dim3(grid_of(b.rows * nb * b.cp)), dim3(PTHR), 0, s, b);
    }
    MatArgs m;
    m.src[0] = (const uint4 *)p.W_a; m.src[1] = (const uint4 *)p.W_x;
    m.dst[0] = (uint4 *)(ws + q.off_wa); m.dst[1] = (uint4 *)(ws + q.off_wx);
    m.nb = nb; m.bs = bs; m.esz = 2;
    hipLaunchKernelGGL(pad_mats_kernel, dim3(grid_of((size_t)nb * PBS * PBS * 2 / 16)), dim3(PTHR), 0, s, m);
    VecArgs v;
    v.n = 8; v.nb = nb; v.bs = bs;
    const float *cw = p.conv_w;   // null (no Conv1D) stays null for the tuned kernels
    const float *rows[8] = {p.b_a, p.b_x, p.Lambda, cw, cw ? cw + p.D : nullptr, cw ? cw + 2 * (size_t)p.D : nullptr,
                            cw ? cw + 3 * (size_t)p.D : nullptr, p.conv_b};
    for (int k = 0; k < 8; ++k) {
      v.src[k] = rows[k];
      v.dst[k] = vec + (size_t)k * Dp;
    }
    hipLaunchKernelGGL(pad_vecs_kernel, dim3((Dp + PTHR - 1) / PTHR), dim3(PTHR), 0, s, v);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }

  // ---- the tuned backward on the widened problem
  Problem w = p;
  w.D = Dp; w.bs = PBS;
  w.u = ws + q.off_u; w.y_in = ws + q.off_y; w.dy = ws + q.off_dy; w.du = ws + q.off_du;
  w.dy_lo = p.dy_lo ? ws + q.off_dylo : nullptr;
  w.W_a = ws + q.off_wa; w.W_x = ws + q.off_wx;
  w.b_a = vec; w.b_x = vec + Dp; w.Lambda = vec + 2 * (size_t)Dp;
  w.conv_w = p.conv_w ? vec + 3 * (size_t)Dp : nullptr;
  w.conv_b = p.conv_b ? vec + 7 * (size_t)Dp : nullptr;
  w.h0 = p.h0 ? (const float *)(ws + q.off_h0) : nullptr;
  w.dhT = p.dhT ? (const float *)(ws + q.off_dhT) : nullptr;
  w.dh0 = p.dh0 ? (float *)(ws + q.off_dh0) : nullptr;
  w.state_in = p.state_in ? ws + q.off_state : nullptr;
  w.g.dW_a = (float *)(ws + q.off_dwa); w.g.dW_x = (float *)(ws + q.off_dwx);
  w.g.db_a = gvec; w.g.db_x = gvec + Dp; w.g.dLambda = gvec + 2 * (size_t)Dp;
  w.g.dconv_w = p.g.dconv_w ? gvec + 3 * (size_t)Dp : nullptr;
  w.g.dconv_b = p.g.dconv_b ? gvec + 7 * (size_t)Dp : nullptr;
  w.ws = ws + q.off_inner;
  w.ws_bytes = q.total - q.off_inner;
  if (!backward_mfma_supported(w, true)) return hipErrorInvalidValue;
  hipError_t e = launch_backward_mfma(w, s);
  if (e != hipSuccess) return e;

  // ---- narrow the results
  {
    KernelTimer kt("unpad_kernel", s);
    ActArgs a;
    a.n = 1; a.rows = (size_t)p.B * p.T; a.nb = nb; a.cb = bs * 2 / 16; a.cp = PBS * 2 / 16;
    a.t[0] = {(const uint4 *)(ws + q.off_du), (uint4 *)p.du};
    hipLaunchKernelGGL(unpad_rows_kernel, dim3(grid_of(a.rows * nb * a.cb)), dim3(PTHR), 0, s, a);
    MatArgs m;
    m.src[0] = (const uint4 *)(ws + q.off_dwa); m.src[1] = (const uint4 *)(ws + q.off_dwx);
    m.dst[0] = (uint4 *)p.g.dW_a; m.dst[1] = (uint4 *)p.g.dW_x;
    m.nb = nb; m.bs = bs; m.esz = 4;
    hipLaunchKernelGGL(unpad_mats_kernel, dim3(grid_of((size_t)nb * bs * bs * 4 / 16)), dim3(PTHR), 0, s, m);
    VecArgs v;
    v.n = 8; v.nb = nb; v.bs = bs;
    float *dcw = p.g.dconv_w;
    float *rows[8] = {p.g.db_a, p.g.db_x, p.g.dLambda, dcw, dcw ? dcw + p.D : nullptr,
                      dcw ? dcw + 2 * (size_t)p.D : nullptr, dcw ? dcw + 3 * (size_t)p.D : nullptr, p.g.dconv_b};
    for (int k = 0; k < 8; ++k) {
      v.src[k] = gvec + (size_t)k * Dp;
      v.dst[k] = rows[k];
    }
    hipLaunchKernelGGL(unpad_vecs_kernel, dim3((nb * bs + PTHR - 1) / PTHR), dim3(PTHR), 0, s, v);
    if (p.dh0) {
      ActArgs b;
      b.n = 1; b.rows = (size_t)p.B; b.nb = nb; b.cb = bs * 4 / 16; b.cp = PBS * 4 / 16;
      b.t[0] = {(const uint4 *)(ws + q.off_dh0), (uint4 *)p.dh0};
      hipLaunchKernelGGL(unpad_rows_kernel, dim3(grid_of(b.rows * nb * b.cb)), dim3(PTHR), 0, s, b);
    }
    e = hipGetLastError();
  }
  return e;
}

}  // namespace rglru
