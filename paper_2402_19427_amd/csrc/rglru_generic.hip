// Shape-generic kernels for the Conv1D -> RG-LRU path: any block size, fp32 or bf16 storage,
// fp32 arithmetic with accurate math (expf / expm1f / log1pf). They serve the fp32 contract
// (relative error 1e-5) and every shape the MFMA kernels do not cover.
//
// Equations: Conv1D - Section 2.3 of the Griffin/Hawk paper; gates, decay, recurrence -
// Section 2.4 eqs. (1)-(4); log-space decay - Appendix A (with the sign that matches
// a = sigmoid(Lambda)); decode state - Appendix F.
#include "rglru_generic.h"

namespace rglru {

// largest dynamic LDS any generic kernel asks for: two [GT][bs] tiles (dgrad)
size_t generic_lds_bytes(int bs) { return (size_t)(2 * GT) * bs * sizeof(float); }

// p[tt], q[tt] = b + W[g][j][:] . xs[tt][:] for the ROWS rows of an LDS tile xs[ROWS][bs]
template <typename AT, int ROWS = GT>
__device__ __forceinline__ void gate_rows(const Problem &p, int g, int j, const float *xs,
                                          float *pa, float *qa) {
  const int bs = p.bs, d = g * bs + j;
  const AT *wa = (const AT *)p.W_a + ((size_t)g * bs + j) * bs;
  const AT *wx = (const AT *)p.W_x + ((size_t)g * bs + j) * bs;
#pragma unroll
  for (int tt = 0; tt < ROWS; ++tt) {
    pa[tt] = p.b_a[d];
    qa[tt] = p.b_x[d];
  }
  int k = 0;
  // four inputs at a time where the rows allow it: one 16-byte LDS read per row and four inputs,
  // the weights as one vector load (the same products in the same order as one by one)
  if ((bs & 3) == 0 && (((uintptr_t)p.W_a | (uintptr_t)p.W_x) & 15) == 0) {
#pragma unroll 4   // (the loads of four steps in flight)
    for (; k < bs; k += 4) {
      float a4[4], x4[4];
      ldf4(wa, k, a4);
      ldf4(wx, k, x4);
#pragma unroll
      for (int tt = 0; tt < ROWS; ++tt) {
        const float4 v = *(const float4 *)(xs + tt * bs + k);
        pa[tt] = fmaf(a4[3], v.w, fmaf(a4[2], v.z, fmaf(a4[1], v.y, fmaf(a4[0], v.x, pa[tt]))));
        qa[tt] = fmaf(x4[3], v.w, fmaf(x4[2], v.z, fmaf(x4[1], v.y, fmaf(x4[0], v.x, qa[tt]))));
      }
    }
  }
  for (; k < bs; ++k) {
    const float a = ldf(wa, k), x = ldf(wx, k);
#pragma unroll
    for (int tt = 0; tt < ROWS; ++tt) {
      const float v = xs[tt * bs + k];
      pa[tt] = fmaf(a, v, pa[tt]);
      qa[tt] = fmaf(x, v, qa[tt]);
    }
  }
}

// ------------------------------------------------------------------------ Conv1D alone
template <typename AT>
__global__ void __launch_bounds__(NTHREADS) conv1d_kernel(Problem p, AT *x_out) {
  const size_t n = (size_t)p.B * p.T * p.D;
  for (size_t idx = (size_t)blockIdx.x * NTHREADS + threadIdx.x; idx < n;
       idx += (size_t)gridDim.x * NTHREADS) {
    const int d = (int)(idx % p.D);
    const size_t bt = idx / p.D;
    const int t = (int)(bt % p.T), b = (int)(bt / p.T);
    stf(x_out, idx, conv_at<AT>(p, b, t, d));
  }
}

// Ring state after the T inputs: slots of the new inputs are overwritten, the others are
// carried from state_in (or zero). One thread per (b, slot, d).
template <typename AT>
__global__ void __launch_bounds__(NTHREADS) state_update_kernel(Problem p) {
  const size_t n = (size_t)p.B * 3 * p.D;
  for (size_t idx = (size_t)blockIdx.x * NTHREADS + threadIdx.x; idx < n;
       idx += (size_t)gridDim.x * NTHREADS) {
    const int d = (int)(idx % p.D);
    const int slot = (int)((idx / p.D) % 3), b = (int)(idx / ((size_t)3 * p.D));
    // newest position that maps to this slot among pos0+T-3 .. pos0+T-1
    const long long end = p.pos0 + p.T;
    long long npos = end - 1 - ring_slot(end - 1 - slot);
    float v;
    if (npos >= p.pos0)
      v = ldf((const AT *)p.u, ((size_t)b * p.T + (size_t)(npos - p.pos0)) * p.D + d);
    else
      v = p.state_in ? ldf((const AT *)p.state_in, idx) : 0.f;
    if (p.reset) {   // an input in front of the last document's first step is not part of its history
      const long long first = npos - p.pos0 + 1;   // (at least T - 2: at most three steps to look at)
      for (int t = first > 0 ? (int)first : 0; t < p.T; ++t)
        if (p.reset[(size_t)b * p.T + t]) v = 0.f;
    }
    stf((AT *)p.state_out, idx, v);
  }
}

// --------------------------------------------------------------------------- forward
// One workgroup per (gate block, sequence), walking the sequence in tiles of GT steps:
// Conv1D into LDS, gate dot products per output channel, then the recurrence with the state
// kept per channel in LDS.
template <typename AT>
__global__ void __launch_bounds__(NTHREADS) forward_kernel(Problem p) {
  extern __shared__ __attribute__((aligned(16))) float smem[];
  const int g = blockIdx.x, b = blockIdx.y, bs = p.bs, tid = threadIdx.x;
  float *xs = smem, *hc = smem + GT * bs;
  for (int j = tid; j < bs; j += NTHREADS)
    hc[j] = p.h0 ? p.h0[(size_t)b * p.D + g * bs + j] : 0.f;
  for (int t0 = 0; t0 < p.T; t0 += GT) {
    const int nt = min(GT, p.T - t0);
    __syncthreads();
    for (int idx = tid; idx < GT * bs; idx += NTHREADS) {
      const int tt = idx / bs, j = idx - tt * bs;
      xs[idx] = tt < nt ? conv_at<AT>(p, b, t0 + tt, g * bs + j) : 0.f;
    }
    __syncthreads();
    for (int j = tid; j < bs; j += NTHREADS) {
      const int d = g * bs + j;
      float pa[GT], qa[GT];
      gate_rows<AT>(p, g, j, xs, pa, qa);
      const float neg_cs = -p.c * softplus_f(-p.Lambda[d]);
      float h = hc[j];
#pragma unroll
      for (int tt = 0; tt < GT; ++tt) {
        if (tt < nt) {
          const Gates gt = gate_math(pa[tt], qa[tt], neg_cs);
          if (starts_document(p, b, t0 + tt)) h = 0.f;
          h = fmaf(gt.a, h, gt.m * (gt.i * xs[tt * bs + j]));  // eq. (4)
          stf((AT *)p.y, ((size_t)b * p.T + t0 + tt) * p.D + d, h);
        }
      }
      hc[j] = h;
    }
  }
  __syncthreads();
  if (p.hT)
    for (int j = tid; j < bs; j += NTHREADS) p.hT[(size_t)b * p.D + g * bs + j] = hc[j];
}

// The same forward in two passes, parallel over time, for callers that bring scratch memory:
// (1) one workgroup per (gate block, sequence, tile of TG steps) forms the scan's coefficients
//     a_t (zero at a document's first step) and b_t = sqrt(1 - a_t^2) i_t x_t for a chunk of the
//     time axis; (2) one thread per (sequence, channel) runs eq. (4) over the chunk. The chunks
//     follow each other on the stream, the state travels in `hstate`.
constexpr int TG = 16;
template <typename AT>
__global__ void __launch_bounds__(NTHREADS) fwd_coeff_kernel(Problem p, int t_lo, int t_hi, float *A, float *Bv) {
  extern __shared__ __attribute__((aligned(16))) float smem[];
  const int g = blockIdx.x, b = blockIdx.y, t0 = t_lo + blockIdx.z * TG, bs = p.bs, tid = threadIdx.x;
  const int nt = min(TG, t_hi - t0), tc = t_hi - t_lo;
  float *xs = smem;
  for (int idx = tid; idx < TG * bs; idx += NTHREADS) {
    const int tt = idx / bs, j = idx - tt * bs;
    xs[idx] = tt < nt ? conv_at<AT>(p, b, t0 + tt, g * bs + j) : 0.f;
  }
  __syncthreads();
  for (int j = tid; j < bs; j += NTHREADS) {
    const int d = g * bs + j;
    float pa[TG], qa[TG];
    gate_rows<AT, TG>(p, g, j, xs, pa, qa);
    const float neg_cs = -p.c * softplus_f(-p.Lambda[d]);
#pragma unroll
    for (int tt = 0; tt < TG; ++tt) {
      if (tt < nt) {
        const Gates gt = gate_math(pa[tt], qa[tt], neg_cs);
        const size_t o = ((size_t)b * tc + (t0 - t_lo) + tt) * p.D + d;
        A[o] = starts_document(p, b, t0 + tt) ? 0.f : gt.a;
        Bv[o] = gt.m * (gt.i * xs[tt * bs + j]);
      }
    }
  }
}
template <typename AT>
__global__ void __launch_bounds__(NTHREADS) fwd_scan_kernel(Problem p, int t_lo, int t_hi, const float *A,
                                                            const float *Bv, const float *h_in, float *h_out) {
  const size_t n = (size_t)p.B * p.D, idx = (size_t)blockIdx.x * NTHREADS + threadIdx.x;
  if (idx >= n) return;
  const int b = (int)(idx / p.D), d = (int)(idx - (size_t)b * p.D), tc = t_hi - t_lo;
  float h = h_in ? h_in[idx] : 0.f;
  const float *a = A + (size_t)b * tc * p.D + d, *bv = Bv + (size_t)b * tc * p.D + d;
  AT *y = (AT *)p.y + ((size_t)b * p.T + t_lo) * p.D + d;
  // (the loads do not depend on the state: 32 steps of them are in flight at a time)
  int t = 0;
  for (; t + 32 <= tc; t += 32) {
    float av[32], bb[32];
#pragma unroll
    for (int k = 0; k < 32; ++k) {
      av[k] = a[(size_t)(t + k) * p.D];
      bb[k] = bv[(size_t)(t + k) * p.D];
    }
#pragma unroll
    for (int k = 0; k < 32; ++k) {
      h = fmaf(av[k], h, bb[k]);   // eq. (4)
      stf(y, (size_t)(t + k) * p.D, h);
    }
  }
  for (; t < tc; ++t) {
    h = fmaf(a[(size_t)t * p.D], h, bv[(size_t)t * p.D]);
    stf(y, (size_t)t * p.D, h);
  }
  if (h_out) h_out[idx] = h;
}

// ---------------------------------------------------------------------------- decode
// One workgroup per (gate block, tile of GT sequences); T == 1, states updated in place.
// The ring slot of the new token is written by the workgroup that owns the channels, after
// all of its reads of the state.
template <typename AT>
__global__ void __launch_bounds__(NTHREADS) decode_kernel(Problem p) {
  extern __shared__ __attribute__((aligned(16))) float smem[];
  const int g = blockIdx.x, b0 = blockIdx.y * GT, bs = p.bs, tid = threadIdx.x;
  const int nbat = min(GT, p.B - b0);
  float *xs = smem;
  AT *state = (AT *)p.state_out;  // in-place ring
  for (int idx = tid; idx < GT * bs; idx += NTHREADS) {
    const int tt = idx / bs, j = idx - tt * bs, d = g * bs + j;
    float acc = 0.f;
    if (tt < nbat) {
      const int b = b0 + tt;
      if (!p.conv_w) {   // no Conv1D (and no ring): x_t = u_t
        acc = ldf((const AT *)p.u, (size_t)b * p.D + d);
      } else {
        acc = p.conv_b ? p.conv_b[d] : 0.f;
        acc = fmaf(p.conv_w[d], ldf((const AT *)p.u, (size_t)b * p.D + d), acc);
        const long long posb = p.pos_rows ? p.pos_rows[b] : p.pos0;
#pragma unroll
        for (int k = 1; k < 4; ++k)
          acc = fmaf(p.conv_w[(size_t)k * p.D + d],
                     ldf(state, ((size_t)b * 3 + ring_slot(posb - k)) * p.D + d), acc);
      }
    }
    xs[idx] = acc;
  }
  __syncthreads();
  for (int j = tid; j < bs; j += NTHREADS) {
    const int d = g * bs + j;
    float pa[GT], qa[GT];
    gate_rows<AT>(p, g, j, xs, pa, qa);
    const float neg_cs = -p.c * softplus_f(-p.Lambda[d]);
#pragma unroll
    for (int tt = 0; tt < GT; ++tt) {
      if (tt < nbat) {
        const size_t o = (size_t)(b0 + tt) * p.D + d;
        const Gates gt = gate_math(pa[tt], qa[tt], neg_cs);
        const float h = fmaf(gt.a, p.hT[o], gt.m * (gt.i * xs[tt * bs + j]));
        p.hT[o] = h;
        stf((AT *)p.y, o, h);
        if (state) {
          const int wslot = ring_slot(p.pos_rows ? p.pos_rows[b0 + tt] : p.pos0);
          state[((size_t)(b0 + tt) * 3 + wslot) * p.D + d] = ((const AT *)p.u)[o];
        }
      }
    }
  }
}

// --------------------------------------------------------------------------- backward
size_t backward_generic_ws_bytes(int B, int T, int D, int nb) {
  (void)nb;
  const size_t N = (size_t)B * T * D;
  const size_t nchunk = (size_t)B * ((T + CONV_TCHUNK - 1) / CONV_TCHUNK);
  return 4 * align256(N * 4) + align256((size_t)B * 3 * D * 4) + align256(nchunk * 5 * D * 4);
}

// Pass 1a, parallel over time: one workgroup per (gate block, sequence, tile of TG steps) recomputes
// the Conv1D and the gate pre-activations and parks x, p, q (fp32) where the later passes expect
// x, dp, dq.
template <typename AT>
__global__ void __launch_bounds__(NTHREADS) bwd_preact_kernel(Problem p, BwdWs w) {
  extern __shared__ __attribute__((aligned(16))) float smem[];
  const int g = blockIdx.x, b = blockIdx.y, t0 = blockIdx.z * TG, bs = p.bs, tid = threadIdx.x;
  const int nt = min(TG, p.T - t0);
  float *xs = smem;
  for (int idx = tid; idx < TG * bs; idx += NTHREADS) {
    const int tt = idx / bs, j = idx - tt * bs;
    xs[idx] = tt < nt ? conv_at<AT>(p, b, t0 + tt, g * bs + j) : 0.f;
  }
  __syncthreads();
  for (int j = tid; j < bs; j += NTHREADS) {
    const int d = g * bs + j;
    float pa[TG], qa[TG];
    gate_rows<AT, TG>(p, g, j, xs, pa, qa);
#pragma unroll
    for (int tt = 0; tt < TG; ++tt) {
      if (tt < nt) {
        const size_t o = ((size_t)b * p.T + t0 + tt) * p.D + d;
        w.x[o] = xs[tt * bs + j];
        w.dp[o] = pa[tt];
        w.dq[o] = qa[tt];
      }
    }
  }
}

// Pass 1b: one thread per (sequence, channel) walks the sequence backwards: gates from the parked
// pre-activations, delta_t = dy_t + a_{t+1} delta_{t+1}, the pointwise adjoints; dp, dq replace
// the pre-activations in place, the direct part of dx goes to its array, and the per-sequence
// sums for db_a, db_x, dLambda are kept with compensation (eight steps as plain sums at a time).
template <typename AT>
__global__ void __launch_bounds__(NTHREADS) bwd_chain_kernel(Problem p, BwdWs w) {
  const size_t n = (size_t)p.B * p.D, idx = (size_t)blockIdx.x * NTHREADS + threadIdx.x;
  if (idx >= n) return;
  const int b = (int)(idx / p.D), d = (int)(idx - (size_t)b * p.D);
  const float neg_cs = -p.c * softplus_f(-p.Lambda[d]);
  const float lam_scale = p.c * sigmoid_f(-p.Lambda[d]);   // 1 - sigmoid(Lambda) without cancellation
  float cy = p.dhT ? p.dhT[idx] : 0.f;
  float sum[3] = {0.f, 0.f, 0.f}, comp[3] = {0.f, 0.f, 0.f};
  const size_t base = (size_t)b * p.T * p.D + d;
  for (int t1 = p.T; t1 > 0; t1 -= 8) {   // steps t1-1 down to max(t1-8, 0)
    const int t_lo = t1 > 8 ? t1 - 8 : 0, cnt = t1 - t_lo;
    float pv[8], qv[8], xv[8], dyv[8], hp[8];
    // the loads of a group do not depend on the chain: all in flight at once. (No load under a
    // condition - the compiler waits for such a load on the spot: steps in front of the sequence
    // re-read step 0, step 0 reads its own y in place of the one before and takes h0 afterwards.)
    const AT *dyl = (const AT *)(p.dy_lo ? p.dy_lo : p.dy);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int t = k < cnt ? t1 - 1 - k : t_lo;
      const size_t o = base + (size_t)t * p.D;
      pv[k] = w.dp[o];
      qv[k] = w.dq[o];
      xv[k] = w.x[o];
      const float lo = ldf(dyl, o);
      dyv[k] = ldf((const AT *)p.dy, o) + (p.dy_lo ? lo : 0.f);
      hp[k] = ldf((const AT *)p.y_in, t > 0 ? o - p.D : o);
    }
    if (t_lo == 0) {
      const float h0v = p.h0 ? p.h0[idx] : 0.f;
#pragma unroll
      for (int k = 0; k < 8; ++k)   // (a dynamic index would put the array in scratch memory)
        if (k == cnt - 1) hp[k] = h0v;
    }
    float s_ba = 0.f, s_bx = 0.f, s_lam = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      if (k < cnt) {
        const int t = t1 - 1 - k;
        const size_t o = base + (size_t)t * p.D;
        const bool fresh = starts_document(p, b, t);   // h_{t-1} := 0, nothing flows further back
        const Gates gt = gate_math(pv[k], qv[k], neg_cs);
        const float delta = dyv[k] + cy;
        const float hprev = fresh ? 0.f : hp[k];
        const float gin = gt.i * xv[k];
        // d m / d a = -a / m; the term vanishes with the gate in the limit m -> 0
        const float corr = gt.m > 0.f ? gt.a * gin / gt.m : 0.f;
        const float dla = delta * gt.a * (hprev - corr);
        const float dg = delta * gt.m;
        const float dpv = neg_cs * dla * gt.r * gt.rc;
        const float dqv = dg * xv[k] * gt.i * gt.ic;
        s_lam = fmaf(dla * gt.r, lam_scale, s_lam);
        s_ba += dpv;
        s_bx += dqv;
        w.dp[o] = dpv;
        w.dq[o] = dqv;
        w.dx[o] = dg * gt.i;
        cy = fresh ? 0.f : gt.a * delta;
      }
    }
    comp_add(sum[0], comp[0], s_ba);
    comp_add(sum[1], comp[1], s_bx);
    comp_add(sum[2], comp[2], s_lam);
  }
  if (p.dh0) p.dh0[idx] = cy;
  w.partA[((size_t)b * 3 + 0) * p.D + d] = sum[0];
  w.partA[((size_t)b * 3 + 1) * p.D + d] = sum[1];
  w.partA[((size_t)b * 3 + 2) * p.D + d] = sum[2];
}

// Pass 2: dx[t][k] += sum_j W_a[g][j][k] dp[t][j] + W_x[g][j][k] dq[t][j]
template <typename AT, int ROWS>
__global__ void __launch_bounds__(NTHREADS) bwd_dgrad_kernel(Problem p, BwdWs w) {
  constexpr int TR = ROWS;   // steps per workgroup: 16, or 8 for blocks whose two tiles of 16 would not fit LDS
  extern __shared__ __attribute__((aligned(16))) float smem[];
  const int g = blockIdx.x, b = blockIdx.y, t0 = blockIdx.z * TR, bs = p.bs, tid = threadIdx.x;
  const int nt = min(TR, p.T - t0);
  float *dps = smem, *dqs = smem + TR * bs;  // [TR][bs] each
  for (int idx = tid; idx < TR * bs; idx += NTHREADS) {
    const int tt = idx / bs, j = idx - tt * bs;
    const size_t o = ((size_t)b * p.T + t0 + tt) * p.D + g * bs + j;
    dps[idx] = tt < nt ? w.dp[o] : 0.f;
    dqs[idx] = tt < nt ? w.dq[o] : 0.f;
  }
  __syncthreads();
  const AT *Wa = (const AT *)p.W_a + (size_t)g * bs * bs;
  const AT *Wx = (const AT *)p.W_x + (size_t)g * bs * bs;
  for (int k = tid; k < bs; k += NTHREADS) {
    float acc[TR];
#pragma unroll
    for (int tt = 0; tt < TR; ++tt)
      acc[tt] = tt < nt ? w.dx[((size_t)b * p.T + t0 + tt) * p.D + g * bs + k] : 0.f;
    int j = 0;
    // four gate outputs at a time where the rows allow it: one 16-byte LDS read per row and array
    // (the same products in the same order as one by one)
    if ((bs & 3) == 0) {
      for (; j < bs; j += 4) {
        float wa[4], wx[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          wa[e] = ldf(Wa, (size_t)(j + e) * bs + k);
          wx[e] = ldf(Wx, (size_t)(j + e) * bs + k);
        }
#pragma unroll
        for (int tt = 0; tt < TR; ++tt) {
          const float4 dp4 = *(const float4 *)(dps + tt * bs + j), dq4 = *(const float4 *)(dqs + tt * bs + j);
          float a = acc[tt];
          a = fmaf(wa[0], dp4.x, fmaf(wx[0], dq4.x, a));
          a = fmaf(wa[1], dp4.y, fmaf(wx[1], dq4.y, a));
          a = fmaf(wa[2], dp4.z, fmaf(wx[2], dq4.z, a));
          a = fmaf(wa[3], dp4.w, fmaf(wx[3], dq4.w, a));
          acc[tt] = a;
        }
      }
    }
    for (; j < bs; ++j) {
      const float wa = ldf(Wa, (size_t)j * bs + k), wx = ldf(Wx, (size_t)j * bs + k);
#pragma unroll
      for (int tt = 0; tt < TR; ++tt)
        acc[tt] = fmaf(wa, dps[tt * bs + j], fmaf(wx, dqs[tt * bs + j], acc[tt]));
    }
#pragma unroll
    for (int tt = 0; tt < TR; ++tt)
      if (tt < nt) w.dx[((size_t)b * p.T + t0 + tt) * p.D + g * bs + k] = acc[tt];
  }
}

// Pass 3a: du[b,t,d] = sum_k conv_w[k][d] dx[b,t+k,d]
template <typename AT>
__global__ void __launch_bounds__(NTHREADS) bwd_conv_input_kernel(Problem p, BwdWs w) {
  const size_t n = (size_t)p.B * p.T * p.D;
  for (size_t idx = (size_t)blockIdx.x * NTHREADS + threadIdx.x; idx < n;
       idx += (size_t)gridDim.x * NTHREADS) {
    const int d = (int)(idx % p.D);
    const int t = (int)((idx / p.D) % p.T), b = (int)(idx / ((size_t)p.T * p.D));
    float acc = 0.f;
    if (!p.conv_w) {
      acc = w.dx[idx];   // no Conv1D: du = dx
    } else {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if (t + k >= p.T || (k > 0 && starts_document(p, b, t + k))) break;   // x of a later document does not see u_t
        acc = fmaf(p.conv_w[(size_t)k * p.D + d], w.dx[idx + (size_t)k * p.D], acc);
      }
    }
    stf((AT *)p.du, idx, acc);
  }
}

// Pass 3b: per (sequence, time chunk) partial sums of dconv_w[k][d] = sum dx_t u_{t-k} and
// dconv_b[d] = sum dx_t
template <typename AT>
__global__ void __launch_bounds__(NTHREADS) bwd_conv_weight_kernel(Problem p, BwdWs w) {
  const int d = blockIdx.x * NTHREADS + threadIdx.x;
  if (d >= p.D) return;
  const int nct = (p.T + w.tchunk - 1) / w.tchunk;
  const int b = blockIdx.y / nct, c = blockIdx.y % nct;
  const int t0 = c * w.tchunk, t1 = min(p.T, t0 + w.tchunk);
  float s[5] = {0.f, 0.f, 0.f, 0.f, 0.f}, sc[5] = {0.f, 0.f, 0.f, 0.f, 0.f};
  const int n0 = t0 < t1 ? lags_at(p, b, t0) : 3;   // history in front of a document's start is zero
  float u1 = n0 >= 1 ? input_at<AT>(p, b, t0 - 1, d) : 0.f, u2 = n0 >= 2 ? input_at<AT>(p, b, t0 - 2, d) : 0.f,
        u3 = n0 >= 3 ? input_at<AT>(p, b, t0 - 3, d) : 0.f;
  for (int tc = t0; tc < t1; tc += 16) {   // short plain sums, added up with compensation
    float l[5] = {0.f, 0.f, 0.f, 0.f, 0.f};
    const int te = min(t1, tc + 16);
    for (int t = tc; t < te; ++t) {
      const size_t o = ((size_t)b * p.T + t) * p.D + d;
      const float dx = w.dx[o], u0 = ldf((const AT *)p.u, o);
      if (starts_document(p, b, t)) u1 = u2 = u3 = 0.f;
      l[0] = fmaf(dx, u0, l[0]);
      l[1] = fmaf(dx, u1, l[1]);
      l[2] = fmaf(dx, u2, l[2]);
      l[3] = fmaf(dx, u3, l[3]);
      l[4] += dx;
      u3 = u2; u2 = u1; u1 = u0;
    }
#pragma unroll
    for (int k = 0; k < 5; ++k) comp_add(s[k], sc[k], l[k]);
  }
#pragma unroll
  for (int k = 0; k < 5; ++k) w.partC[((size_t)blockIdx.y * 5 + k) * p.D + d] = s[k];
}

__global__ void __launch_bounds__(NTHREADS) reduce_parts_kernel(const float *part, int nparts,
                                                                int rows, int D, RowOuts out) {
  const int d = blockIdx.x * NTHREADS + threadIdx.x, r = blockIdx.y;
  if (d >= D || !out.p[r]) return;
  float s = 0.f, c = 0.f;
  for (int q = 0; q < nparts; ++q) comp_add(s, c, part[((size_t)q * rows + r) * D + d]);
  out.p[r][d] = s;
}

// Pass 4: dW_a[g][j][k] = sum_{b,t} dp[b,t,j] x[b,t,k], dW_x likewise with dq. One workgroup per
// 64x64 output tile of one block and slice of the B*T rows, 16x16 threads with 4x4 outputs each
// (12 LDS reads per 32 products), rows streamed through LDS 32 at a time; the chunks of 32 rows
// are added up with compensation. With one slice the sums go straight to dW; otherwise to
// part[slice][gate][nb][bs][bs], which wgrad_reduce_kernel adds up in a fixed order.
__global__ void __launch_bounds__(NTHREADS) bwd_wgrad_kernel(Problem p, BwdWs w, float *part, int rows_per, int tiles) {
  __shared__ float xs[32][65], ps[32][65], qs[32][65];
  const int g = blockIdx.x, j0 = (blockIdx.y / tiles) * 64, k0 = (blockIdx.y % tiles) * 64, bs = p.bs;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float aa[4][4], ax[4][4], ca[4][4], cx[4][4];   // sums and their compensation terms
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int c = 0; c < 4; ++c) aa[a][c] = ax[a][c] = ca[a][c] = cx[a][c] = 0.f;
  const size_t rows = (size_t)p.B * p.T;
  const size_t r_lo = (size_t)blockIdx.z * rows_per, r_hi = r_lo + rows_per < rows ? r_lo + rows_per : rows;
  for (size_t r0 = r_lo; r0 < r_hi; r0 += 32) {
    __syncthreads();
    for (int idx = threadIdx.x; idx < 32 * 64; idx += NTHREADS) {
      const int rr = idx >> 6, cc = idx & 63;
      const size_t row = r0 + rr;
      const bool okr = row < r_hi;
      const size_t base = row * p.D + (size_t)g * bs;
      xs[rr][cc] = (okr && k0 + cc < bs) ? w.x[base + k0 + cc] : 0.f;
      ps[rr][cc] = (okr && j0 + cc < bs) ? w.dp[base + j0 + cc] : 0.f;
      qs[rr][cc] = (okr && j0 + cc < bs) ? w.dq[base + j0 + cc] : 0.f;
    }
    __syncthreads();
    float la[4][4], lx[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int c = 0; c < 4; ++c) la[a][c] = lx[a][c] = 0.f;
#pragma unroll 4
    for (int rr = 0; rr < 32; ++rr) {
      float xv[4], pv[4], qv[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        xv[e] = xs[rr][tx + 16 * e];
        pv[e] = ps[rr][ty + 16 * e];
        qv[e] = qs[rr][ty + 16 * e];
      }
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          la[a][c] = fmaf(pv[a], xv[c], la[a][c]);
          lx[a][c] = fmaf(qv[a], xv[c], lx[a][c]);
        }
    }
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        comp_add(aa[a][c], ca[a][c], la[a][c]);
        comp_add(ax[a][c], cx[a][c], lx[a][c]);
      }
  }
  const size_t per_gate = (size_t)p.nb * bs * bs;
  float *oa = part ? part + (size_t)blockIdx.z * 2 * per_gate : p.g.dW_a;
  float *ox = part ? oa + per_gate : p.g.dW_x;
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int j = j0 + ty + 16 * a, k = k0 + tx + 16 * c;
      if (j < bs && k < bs) {
        oa[((size_t)g * bs + j) * bs + k] = aa[a][c];
        ox[((size_t)g * bs + j) * bs + k] = ax[a][c];
      }
    }
}
__global__ void __launch_bounds__(NTHREADS) wgrad_reduce_kernel(Problem p, const float *part, int S) {
  const size_t per_gate = (size_t)p.nb * p.bs * p.bs, i = (size_t)blockIdx.x * NTHREADS + threadIdx.x;
  if (i >= 2 * per_gate) return;
  float sum = 0.f, comp = 0.f;
  for (int s = 0; s < S; ++s) comp_add(sum, comp, part[(size_t)s * 2 * per_gate + i]);
  if (i < per_gate) p.g.dW_a[i] = sum;
  else p.g.dW_x[i - per_gate] = sum;
}

// ------------------------------------------------------------------------- launchers
hipError_t launch_reduce_parts(const float *part, int nparts, int rows, int D, const RowOuts &out, hipStream_t s) {
  hipLaunchKernelGGL(reduce_parts_kernel, dim3((D + NTHREADS - 1) / NTHREADS, rows), dim3(NTHREADS), 0, s, part,
                     nparts, rows, D, out);
  return hipGetLastError();
}

static int grid_1d(size_t n) {
  size_t blocks = (n + NTHREADS - 1) / NTHREADS;
  return (int)(blocks < 1 ? 1 : (blocks > 65536 ? 65536 : blocks));
}

template <typename K>
static hipError_t allow_lds(K kernel, size_t bytes) {
  if (bytes <= 48 * 1024) return hipSuccess;
  return hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)bytes);
}

hipError_t launch_conv1d_generic(const Problem &p, bool bf, void *x_out, hipStream_t s) {
  const size_t n = (size_t)p.B * p.T * p.D;
  if (n == 0) return hipSuccess;
  if (bf)
    hipLaunchKernelGGL(conv1d_kernel<bf16>, dim3(grid_1d(n)), dim3(NTHREADS), 0, s, p, (bf16 *)x_out);
  else
    hipLaunchKernelGGL(conv1d_kernel<float>, dim3(grid_1d(n)), dim3(NTHREADS), 0, s, p, (float *)x_out);
  return hipGetLastError();
}

hipError_t launch_state_update(const Problem &p, bool bf, hipStream_t s) {
  if (!p.state_out) return hipSuccess;
  const size_t n = (size_t)p.B * 3 * p.D;
  if (bf)
    hipLaunchKernelGGL(state_update_kernel<bf16>, dim3(grid_1d(n)), dim3(NTHREADS), 0, s, p);
  else
    hipLaunchKernelGGL(state_update_kernel<float>, dim3(grid_1d(n)), dim3(NTHREADS), 0, s, p);
  return hipGetLastError();
}

// scratch of the two-pass forward: a 256-byte cell (left alone: the fused kernels keep their status
// word there), the state between chunks, a_t and b_t of one chunk of steps (at most 64 MB each)
static int fwd_chunk_steps(int B, int T, int D) {
  long long tc = ((long long)64 << 20) / ((long long)4 * B * D);
  tc = tc / TG * TG;
  if (tc < TG) tc = TG;
  return (int)(tc < T ? tc : T);
}
size_t forward_generic_ws_bytes(int B, int T, int D) {
  if (T < 1) return 0;
  const size_t chunk = align256((size_t)4 * B * D * fwd_chunk_steps(B, T, D));
  return 256 + align256((size_t)4 * B * D) + 2 * chunk;
}

template <typename AT>
static hipError_t forward_two_pass(const Problem &p, hipStream_t s) {
  const int tcmax = fwd_chunk_steps(p.B, p.T, p.D);
  const size_t chunk = align256((size_t)4 * p.B * p.D * tcmax), lds = (size_t)TG * p.bs * sizeof(float);
  float *hstate = (float *)((char *)p.ws + 256);
  float *A = (float *)((char *)p.ws + 256 + align256((size_t)4 * p.B * p.D)), *Bv = (float *)((char *)A + chunk);
  hipError_t e = allow_lds(fwd_coeff_kernel<AT>, lds);
  if (e != hipSuccess) return e;
  const int sblocks = (int)(((size_t)p.B * p.D + NTHREADS - 1) / NTHREADS);
  for (int t_lo = 0; t_lo < p.T; t_lo += tcmax) {
    const int t_hi = t_lo + tcmax < p.T ? t_lo + tcmax : p.T, ntile = (t_hi - t_lo + TG - 1) / TG;
    if (ntile > 65535) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(fwd_coeff_kernel<AT>, dim3(p.nb, p.B, ntile), dim3(NTHREADS), lds, s, p, t_lo, t_hi, A, Bv);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const bool last = t_hi == p.T;
    hipLaunchKernelGGL(fwd_scan_kernel<AT>, dim3(sblocks), dim3(NTHREADS), 0, s, p, t_lo, t_hi, A, Bv,
                       t_lo == 0 ? p.h0 : hstate, last ? p.hT : hstate);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_forward_generic(const Problem &p, bool bf, hipStream_t s) {
  // with enough scratch and more than one tile of steps: the two-pass version, parallel over time
  if (p.ws && p.T > GT && p.ws_bytes >= forward_generic_ws_bytes(p.B, p.T, p.D) && ((uintptr_t)p.ws % 256) == 0)
    return bf ? forward_two_pass<bf16>(p, s) : forward_two_pass<float>(p, s);
  const size_t lds = generic_lds_bytes(p.bs);
  hipError_t e = bf ? allow_lds(forward_kernel<bf16>, lds) : allow_lds(forward_kernel<float>, lds);
  if (e != hipSuccess) return e;
  const dim3 grid(p.nb, p.B);
  if (bf)
    hipLaunchKernelGGL(forward_kernel<bf16>, grid, dim3(NTHREADS), lds, s, p);
  else
    hipLaunchKernelGGL(forward_kernel<float>, grid, dim3(NTHREADS), lds, s, p);
  return hipGetLastError();
}

hipError_t launch_decode_generic(const Problem &p, bool bf, hipStream_t s) {
  const size_t lds = generic_lds_bytes(p.bs);
  hipError_t e = bf ? allow_lds(decode_kernel<bf16>, lds) : allow_lds(decode_kernel<float>, lds);
  if (e != hipSuccess) return e;
  const dim3 grid(p.nb, (p.B + GT - 1) / GT);
  if (bf)
    hipLaunchKernelGGL(decode_kernel<bf16>, grid, dim3(NTHREADS), lds, s, p);
  else
    hipLaunchKernelGGL(decode_kernel<float>, grid, dim3(NTHREADS), lds, s, p);
  return hipGetLastError();
}

template <typename AT>
static hipError_t backward_generic_t(const Problem &p, hipStream_t s, bool with_pointwise = true,
                                     bool with_dgrad = true, bool with_wgrad = true, bool with_du = true) {
  const BwdWs w = carve_bwd_ws(p.ws, p.B, p.T, p.D);
  const size_t lds = generic_lds_bytes(p.bs);
  hipError_t e = allow_lds(bwd_preact_kernel<AT>, (size_t)TG * p.bs * sizeof(float));
  if (e != hipSuccess) return e;
  const int dg_rows = p.bs <= 1024 ? TG : GT;
  const size_t lds_dg = (size_t)2 * dg_rows * p.bs * sizeof(float);
  e = dg_rows == TG ? allow_lds(bwd_dgrad_kernel<AT, TG>, lds_dg) : allow_lds(bwd_dgrad_kernel<AT, GT>, lds_dg);
  if (e != hipSuccess) return e;
  const size_t n = (size_t)p.B * p.T * p.D;
  const int dblocks = (p.D + NTHREADS - 1) / NTHREADS;

  if (with_pointwise) {
    const int nt16 = (p.T + TG - 1) / TG;
    if (nt16 > 65535 || p.B > 65535) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(bwd_preact_kernel<AT>, dim3(p.nb, p.B, nt16), dim3(NTHREADS), (size_t)TG * p.bs * sizeof(float), s,
                       p, w);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(bwd_chain_kernel<AT>, dim3((unsigned)(((size_t)p.B * p.D + NTHREADS - 1) / NTHREADS)),
                       dim3(NTHREADS), 0, s, p, w);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  const RowOuts gate_outs = {{p.g.db_a, p.g.db_x, p.g.dLambda, nullptr, nullptr}};
  hipLaunchKernelGGL(reduce_parts_kernel, dim3(dblocks, 3), dim3(NTHREADS), 0, s, w.partA, p.B, 3,
                     p.D, gate_outs);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  // dgrad: time tiles in gridDim.z (<= 65535), sequences in y
  const int ntile = (p.T + dg_rows - 1) / dg_rows;
  if (ntile > 65535 || p.B > 65535) return hipErrorInvalidConfiguration;
  if (with_dgrad) {
    if (dg_rows == TG)
      hipLaunchKernelGGL((bwd_dgrad_kernel<AT, TG>), dim3(p.nb, p.B, ntile), dim3(NTHREADS), lds_dg, s, p, w);
    else
      hipLaunchKernelGGL((bwd_dgrad_kernel<AT, GT>), dim3(p.nb, p.B, ntile), dim3(NTHREADS), lds_dg, s, p, w);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (with_du) {
    if (conv_adjoint_rows_applies(p, sizeof(AT) == 2)) {   // 4 channels x 8 steps per thread, vector accesses
      if ((e = launch_conv_adjoint_rows(p, w.dx, s)) != hipSuccess) return e;
    } else {
      hipLaunchKernelGGL(bwd_conv_input_kernel<AT>, dim3(grid_1d(n)), dim3(NTHREADS), 0, s, p, w);
      if ((e = hipGetLastError()) != hipSuccess) return e;
    }
  }
  if (p.g.dconv_w) {   // (absent without a Conv1D)
    if (w.nchunk > 65535) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(bwd_conv_weight_kernel<AT>, dim3(dblocks, w.nchunk), dim3(NTHREADS), 0, s, p, w);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const RowOuts conv_outs = {{p.g.dconv_w, p.g.dconv_w + p.D, p.g.dconv_w + 2 * (size_t)p.D,
                                p.g.dconv_w + 3 * (size_t)p.D, p.g.dconv_b}};
    hipLaunchKernelGGL(reduce_parts_kernel, dim3(dblocks, 5), dim3(NTHREADS), 0, s, w.partC, w.nchunk,
                       5, p.D, conv_outs);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (!with_wgrad) return hipSuccess;
  // slices of the rows: enough workgroups for the chip, none shorter than 128 rows; their partial
  // sums go where dx was (every reader of dx has run by now) as far as that array reaches
  const int tiles = (p.bs + 63) / 64;
  const size_t rows = (size_t)p.B * p.T, wg1 = (size_t)p.nb * tiles * tiles;
  size_t S = (1024 + wg1 - 1) / wg1;
  if (S > rows / 128) S = rows / 128;
  if (S > n / (2 * (size_t)p.D * p.bs)) S = n / (2 * (size_t)p.D * p.bs);   // S partial copies of dW_a, dW_x in n floats
  if (S < 1) S = 1;
  if (S > 65535 || (size_t)tiles * tiles > 65535) return hipErrorInvalidConfiguration;
  const int rows_per = (int)(((rows + S - 1) / S + 31) / 32 * 32);
  float *part = S > 1 ? w.dx : nullptr;
  hipLaunchKernelGGL(bwd_wgrad_kernel, dim3(p.nb, tiles * tiles, (unsigned)S), dim3(NTHREADS), 0, s, p, w, part, rows_per,
                     tiles);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (S > 1) {
    const size_t cnt = 2 * (size_t)p.nb * p.bs * p.bs;
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)((cnt + NTHREADS - 1) / NTHREADS)), dim3(NTHREADS), 0, s, p,
                       (const float *)part, (int)S);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_backward_generic(const Problem &p, bool bf, hipStream_t s) {
  return bf ? backward_generic_t<bf16>(p, s) : backward_generic_t<float>(p, s);
}

// everything after the pointwise pass: the caller has filled x, dp, dq, dx and partA itself
hipError_t launch_backward_generic_tail(const Problem &p, bool bf, hipStream_t s, bool with_dgrad, bool with_wgrad,
                                        bool with_du) {
  return bf ? backward_generic_t<bf16>(p, s, false, with_dgrad, with_wgrad, with_du)
            : backward_generic_t<float>(p, s, false, with_dgrad, with_wgrad, with_du);
}

void backward_generic_arrays(const Problem &p, float **x, float **dp, float **dq, float **dx, float **partA) {
  const BwdWs w = carve_bwd_ws(p.ws, p.B, p.T, p.D);
  *x = w.x; *dp = w.dp; *dq = w.dq; *dx = w.dx; *partA = w.partA;
}

}  // namespace rglru
