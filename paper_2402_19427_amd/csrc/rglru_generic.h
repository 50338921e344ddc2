// Device helpers shared by the shape-generic kernels of the real layer and of the complex-gated
// variant: tile constants, accurate scalar math, compensated sums, the Conv1D on the fly
// (Section 2.3, with the ring state of Appendix F and document boundaries), and the layout of
// the backward's scratch arrays.
#pragma once
#include "rglru_internal.h"

namespace rglru {

constexpr int GT = 8;        // rows (time steps or sequences) per tile
constexpr int NTHREADS = 256;

__device__ __forceinline__ float softplus_f(float z) {
  return z > 0.f ? z + log1pf(expf(-z)) : log1pf(expf(z));
}
__device__ __forceinline__ float sigmoid_f(float z) { return 1.f / (1.f + expf(-z)); }

// total += v with the rounding error of the addition carried in `comp` (compensated summation:
// the parameter gradients are sums over every (sequence, step) and have to stay inside the
// fp32 contract however long they are)
__device__ __forceinline__ void comp_add(float &total, float &comp, float v) {
  const float y = v - comp;
  const float t = total + y;
  comp = (t - total) - y;
  total = t;
}

struct Gates {
  float r, i, a, m;
  float rc, ic;   // 1 - r, 1 - i as sigmoid(-p), sigmoid(-q): no cancellation when a gate saturates open
};
// eqs. (1)-(3): neg_cs = -c * softplus(-Lambda) = c * log sigmoid(Lambda)
__device__ __forceinline__ Gates gate_math(float p, float q, float neg_cs) {
  Gates g;
  g.r = sigmoid_f(p);
  g.i = sigmoid_f(q);
  g.rc = sigmoid_f(-p);
  g.ic = sigmoid_f(-q);
  const float la = neg_cs * g.r;
  g.a = expf(la);
  g.m = sqrtf(-expm1f(2.f * la));  // sqrt(1 - a^2) without cancellation
  return g;
}

// input of sequence b at time t (t may be negative: carried state, else zero padding)
template <typename AT>
__device__ __forceinline__ float input_at(const Problem &p, int b, int t, int d) {
  if (t >= 0) return ldf((const AT *)p.u, ((size_t)b * p.T + t) * p.D + d);
  if (!p.state_in) return 0.f;
  return ldf((const AT *)p.state_in, ((size_t)b * 3 + ring_slot(p.pos0 + t)) * p.D + d);
}

// true where step t of sequence b starts a new document (packed sequences)
__device__ __forceinline__ bool starts_document(const Problem &p, int b, int t) {
  return p.reset && p.reset[(size_t)b * p.T + t] != 0;
}

// the largest lag (0..3) the Conv1D may reach back from step t without crossing the first step
// of a document: inputs in front of a document's start count as zeros
__device__ __forceinline__ int lags_at(const Problem &p, int b, int t) {
  if (!p.reset) return 3;
  int n = 0;
#pragma unroll
  for (int k = 1; k < 4; ++k) {
    const int tb = t - k + 1;   // lag k crosses the starts at steps tb .. t
    if (tb >= 0 && p.reset[(size_t)b * p.T + tb]) break;
    n = k;
  }
  return n;
}

// Conv1D output x[b,t,d] (Section 2.3), lag-indexed taps
template <typename AT>
__device__ __forceinline__ float conv_at(const Problem &p, int b, int t, int d) {
  if (!p.conv_w) return input_at<AT>(p, b, t, d);   // no Conv1D: x_t = u_t
  float acc = p.conv_b ? p.conv_b[d] : 0.f;
  const int n = lags_at(p, b, t);
#pragma unroll
  for (int k = 0; k < 4; ++k)
    if (k <= n) acc = fmaf(p.conv_w[(size_t)k * p.D + d], input_at<AT>(p, b, t - k, d), acc);
  return acc;
}

// Workspace layout (floats): x[N] dp[N] dq[N] dx[N] | partA[B][3][D] | partC[nchunk][5][D]
struct BwdWs {
  float *x, *dp, *dq, *dx, *partA, *partC;
  int tchunk, nchunk;
};
constexpr int CONV_TCHUNK = 256;

static inline size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

static inline BwdWs carve_bwd_ws(void *ws, int B, int T, int D) {
  BwdWs w;
  const size_t N = (size_t)B * T * D;
  char *base = (char *)ws;
  size_t off = 0;
  w.x = (float *)(base + off); off += align256(N * 4);
  w.dp = (float *)(base + off); off += align256(N * 4);
  w.dq = (float *)(base + off); off += align256(N * 4);
  w.dx = (float *)(base + off); off += align256(N * 4);
  w.partA = (float *)(base + off); off += align256((size_t)B * 3 * D * 4);
  w.tchunk = CONV_TCHUNK;
  w.nchunk = B * ((T + CONV_TCHUNK - 1) / CONV_TCHUNK);
  w.partC = (float *)(base + off);
  return w;
}

// out.p[r][d] = sum_q part[q][r][d] for r < rows, in a fixed order (deterministic)
struct RowOuts {
  float *p[5];
};
hipError_t launch_reduce_parts(const float *part, int nparts, int rows, int D, const RowOuts &out, hipStream_t s);

}  // namespace rglru
