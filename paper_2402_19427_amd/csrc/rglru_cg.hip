// Complex-gated LRU (Appendix B of the Griffin/Hawk paper): the RG-LRU with a complex diagonal
// recurrence weight a~ = sigmoid(Lambda) e^{i theta}. The D real channels of x_t are read as
// H = D / 2 complex ones (first half real parts, second half imaginary parts); the gates, the
// decay and the state have H entries:
//     r_t = sigmoid(W_a x_t + b_a),  i_t = sigmoid(W_x x_t + b_x)
//     a~_t = a~^(c r_t) = exp(c r_t (log sigmoid(Lambda) + i theta))
//     h~_t = a~_t h~_{t-1} + sqrt(1 - |a~_t|^2) (i_t x~_t),   y_t = [Re h~_t ; Im h~_t]
// Gate block g (of nb) owns the complex channels g*hs .. (g+1)*hs-1 (hs = H / nb) and sees the
// real and the imaginary parts of exactly those channels: W[g] is [hs][2 hs].
//
// Shape-generic kernels (any block size, fp32 or bf16 storage, fp32 arithmetic with accurate
// math), built like the real layer's general kernels: one workgroup per (gate block, sequence)
// walks the sequence in tiles of GT steps. In Problem, bs = hs and D is the real width.
#include "rglru_generic.h"
#include "rglru_mfma.h"

namespace rglru {

namespace {

// real channel of input k (0 .. 2 hs - 1) of gate block g
__device__ __forceinline__ int cg_channel(int g, int hs, int H, int k) {
  return k < hs ? g * hs + k : H + g * hs + (k - hs);
}

struct CGates {
  float r, i, rc, ic;   // gates and their complements sigmoid(-p), sigmoid(-q)
  float ar, ai;         // a~_t
  float m;              // sqrt(1 - |a~_t|^2)
  float mod2;           // |a~_t|^2
};
// neg_cs = c log sigmoid(Lambda) = log|a~| * c, c_theta = c * theta
__device__ __forceinline__ CGates cg_gate_math(float p, float q, float neg_cs, float c_theta) {
  CGates g;
  g.r = sigmoid_f(p);
  g.i = sigmoid_f(q);
  g.rc = sigmoid_f(-p);
  g.ic = sigmoid_f(-q);
  const float lm = neg_cs * g.r;   // log |a~_t| <= 0
  const float mod = expf(lm);
  float sn, cs;
  sincosf(c_theta * g.r, &sn, &cs);
  g.ar = mod * cs;
  g.ai = mod * sn;
  g.mod2 = expf(2.f * lm);
  g.m = sqrtf(-expm1f(2.f * lm));   // no cancellation as |a~_t| -> 1
  return g;
}

// the x tile of gate block g: xs[tt][k] for the GT steps from t0 (zero past the sequence's end)
template <typename AT, int ROWS = GT>
__device__ __forceinline__ void cg_load_tile(const Problem &p, int g, int b, int t0, int nt, float *xs) {
  const int hs = p.bs, H = p.D / 2;
  for (int idx = threadIdx.x; idx < ROWS * 2 * hs; idx += NTHREADS) {
    const int tt = idx / (2 * hs), k = idx - tt * 2 * hs;
    xs[idx] = tt < nt ? conv_at<AT>(p, b, t0 + tt, cg_channel(g, hs, H, k)) : 0.f;
  }
}

// pre-activations of output j of block g for the GT rows of the tile: b + W[g][j][:] . xs[tt][:]
template <typename AT, int ROWS = GT>
__device__ __forceinline__ void cg_gate_rows(const Problem &p, int g, int j, const float *xs, float *pa,
                                             float *qa) {
  const int hs = p.bs, nin = 2 * hs, h = g * hs + j;
  const AT *wa = (const AT *)p.W_a + (size_t)h * nin;
  const AT *wx = (const AT *)p.W_x + (size_t)h * nin;
#pragma unroll
  for (int tt = 0; tt < ROWS; ++tt) {
    pa[tt] = p.b_a[h];
    qa[tt] = p.b_x[h];
  }
  int k = 0;
  // four inputs at a time where the rows allow it (the same products in the same order)
  if ((nin & 3) == 0 && (((uintptr_t)p.W_a | (uintptr_t)p.W_x) & 15) == 0) {
#pragma unroll 4   // (the loads of four steps in flight: 40 % on the decode step, whose few threads hide no latency)
    for (; k < nin; k += 4) {
      float a4[4], x4[4];
      ldf4(wa, k, a4);
      ldf4(wx, k, x4);
#pragma unroll
      for (int tt = 0; tt < ROWS; ++tt) {
        const float4 v = *(const float4 *)(xs + tt * nin + k);
        pa[tt] = fmaf(a4[3], v.w, fmaf(a4[2], v.z, fmaf(a4[1], v.y, fmaf(a4[0], v.x, pa[tt]))));
        qa[tt] = fmaf(x4[3], v.w, fmaf(x4[2], v.z, fmaf(x4[1], v.y, fmaf(x4[0], v.x, qa[tt]))));
      }
    }
  }
  for (; k < nin; ++k) {
    const float a = ldf(wa, k), x = ldf(wx, k);
#pragma unroll
    for (int tt = 0; tt < ROWS; ++tt) {
      const float v = xs[tt * nin + k];
      pa[tt] = fmaf(a, v, pa[tt]);
      qa[tt] = fmaf(x, v, qa[tt]);
    }
  }
}

// --------------------------------------------------------------------------- forward
// OT: storage type of y (the backward recomputes the states into an fp32 array)
template <typename AT, typename OT = AT>
__global__ void __launch_bounds__(NTHREADS) cg_forward_kernel(Problem p) {
  extern __shared__ __attribute__((aligned(16))) float smem[];
  const int g = blockIdx.x, b = blockIdx.y, hs = p.bs, H = p.D / 2, tid = threadIdx.x;
  float *xs = smem, *hc = smem + GT * 2 * hs;   // state: [hs] real parts, [hs] imaginary parts
  for (int j = tid; j < hs; j += NTHREADS) {
    hc[j] = p.h0 ? p.h0[(size_t)b * p.D + g * hs + j] : 0.f;
    hc[hs + j] = p.h0 ? p.h0[(size_t)b * p.D + H + g * hs + j] : 0.f;
  }
  for (int t0 = 0; t0 < p.T; t0 += GT) {
    const int nt = min(GT, p.T - t0);
    __syncthreads();
    cg_load_tile<AT>(p, g, b, t0, nt, xs);
    __syncthreads();
    for (int j = tid; j < hs; j += NTHREADS) {
      const int h = g * hs + j;
      float pa[GT], qa[GT];
      cg_gate_rows<AT>(p, g, j, xs, pa, qa);
      const float neg_cs = -p.c * softplus_f(-p.Lambda[h]), c_theta = p.c * p.theta[h];
      float hr = hc[j], hi = hc[hs + j];
#pragma unroll
      for (int tt = 0; tt < GT; ++tt) {
        if (tt < nt) {
          const CGates gt = cg_gate_math(pa[tt], qa[tt], neg_cs, c_theta);
          const float gain = gt.m * gt.i;
          const float nr = fmaf(gt.ar, hr, fmaf(-gt.ai, hi, gain * xs[tt * 2 * hs + j]));
          const float ni = fmaf(gt.ar, hi, fmaf(gt.ai, hr, gain * xs[tt * 2 * hs + hs + j]));
          hr = nr;
          hi = ni;
          const size_t o = ((size_t)b * p.T + t0 + tt) * p.D;
          stf((OT *)p.y, o + h, hr);
          stf((OT *)p.y, o + H + h, hi);
        }
      }
      hc[j] = hr;
      hc[hs + j] = hi;
    }
  }
  __syncthreads();
  if (p.hT)
    for (int j = tid; j < hs; j += NTHREADS) {
      p.hT[(size_t)b * p.D + g * hs + j] = hc[j];
      p.hT[(size_t)b * p.D + H + g * hs + j] = hc[hs + j];
    }
}

// The forward in two passes, parallel over time, where scratch is at hand: (1) a workgroup per
// (gate block, sequence, 16 steps) writes the scan's coefficients a~_t and b~_t = sqrt(1 - |a~_t|^2)
// i_t x~_t for a chunk of steps as (re, im) pairs [B][steps][H]; (2) a thread per (sequence,
// complex channel) runs the recurrence over the chunk. OT: storage type of y.
// KEEP (the backward's recomputation): x goes to `xk` [B][T][D] and the gate pre-activations to
// `pq` ([B*T][H] of p, then [B*T][H] of q) as well.
constexpr int CTG = 16;
template <typename AT, bool KEEP = false>
__global__ void __launch_bounds__(NTHREADS) cg_coeff_kernel(Problem p, int t_lo, int t_hi, float2 *A, float2 *Bv,
                                                            float *xk = nullptr, float *pq = nullptr) {
  extern __shared__ __attribute__((aligned(16))) float smem[];
  const int g = blockIdx.x, b = blockIdx.y, t0 = t_lo + blockIdx.z * CTG, hs = p.bs, H = p.D / 2;
  const int nt = min(CTG, t_hi - t0), tc = t_hi - t_lo;
  float *xs = smem;
  cg_load_tile<AT, CTG>(p, g, b, t0, nt, xs);
  __syncthreads();
  for (int j = threadIdx.x; j < hs; j += NTHREADS) {
    const int h = g * hs + j;
    float pa[CTG], qa[CTG];
    cg_gate_rows<AT, CTG>(p, g, j, xs, pa, qa);
    const float neg_cs = -p.c * softplus_f(-p.Lambda[h]), c_theta = p.c * p.theta[h];
#pragma unroll
    for (int tt = 0; tt < CTG; ++tt) {
      if (tt < nt) {
        const CGates gt = cg_gate_math(pa[tt], qa[tt], neg_cs, c_theta);
        const float gain = gt.m * gt.i;
        const size_t o = ((size_t)b * tc + (t0 - t_lo) + tt) * H + h;
        A[o] = make_float2(gt.ar, gt.ai);
        Bv[o] = make_float2(gain * xs[tt * 2 * hs + j], gain * xs[tt * 2 * hs + hs + j]);
        if (KEEP) {
          const size_t row = (size_t)b * p.T + t0 + tt;
          xk[row * p.D + h] = xs[tt * 2 * hs + j];
          xk[row * p.D + H + h] = xs[tt * 2 * hs + hs + j];
          pq[row * H + h] = pa[tt];
          pq[((size_t)p.B * p.T + row) * H + h] = qa[tt];
        }
      }
    }
  }
}
// The same pass with the gate products on the matrix cores (bf16 storage, hs a multiple of 16):
// a workgroup of four waves takes 32 steps of one (gate block, sequence); the x tile sits in LDS
// in fp32 (for b~_t and the parked copy) and as a half-precision high part + low part (the
// products' row operand, two products per fragment: with the high part alone, 11 significant bits,
// the phase errors of a~_t added up over 2048 steps to 3e-2 in dW_a and du at width 2560; the
// bf16 weights convert to half precision exactly from 6.1e-5 up); a wave
// owns 32 complex channels at a time and multiplies the tile by those channels' rows of W_a and
// of W_x, fetched as 16-byte fragments straight from the matrices (v_mfma_f32_32x32x16_f16), so
// that a lane ends up with both pre-activations of one channel for 16 steps.
constexpr int MT = 32;   // steps per tile of the matrix-core passes
// row of the x tile that lane column j feeds, so that accumulator register r of lane half hf is step 16 hf + r
__device__ __forceinline__ int mfma_arow(int j) { return ((j >> 2) & 1) * 16 + (j >> 3) * 4 + (j & 3); }
template <bool KEEP = false>
__global__ void __launch_bounds__(NTHREADS) cg_coeff_mfma_kernel(Problem p, int t_lo, int t_hi, float2 *A, float2 *Bv,
                                                                 float *xk = nullptr, float *pq = nullptr) {
  extern __shared__ __attribute__((aligned(16))) float smem[];
  const int g = blockIdx.x, b = blockIdx.y, t0 = t_lo + blockIdx.z * MT, hs = p.bs, H = p.D / 2, nin = 2 * hs;
  const int nt = min(MT, t_hi - t0), tc = t_hi - t_lo, xsh = nin + 8;
  float *xf = smem;                                    // [MT][nin] fp32
  _Float16 *xh = (_Float16 *)(smem + MT * nin);        // [MT][nin + 8] half precision, high part
  _Float16 *xl = xh + MT * xsh;                        // ... and low part (x = high + low to 22 bits)
  for (int k = threadIdx.x; k < nin; k += NTHREADS) {   // a thread walks one input column down the tile's steps
    const int d = cg_channel(g, hs, H, k);
    const bool conv = p.conv_w != nullptr;
    const float w0 = conv ? p.conv_w[d] : 1.f, w1 = conv ? p.conv_w[(size_t)p.D + d] : 0.f;
    const float w2 = conv ? p.conv_w[(size_t)2 * p.D + d] : 0.f, w3 = conv ? p.conv_w[(size_t)3 * p.D + d] : 0.f;
    const float cb = (conv && p.conv_b) ? p.conv_b[d] : 0.f;
    float u1 = conv ? input_at<bf16>(p, b, t0 - 1, d) : 0.f, u2 = conv ? input_at<bf16>(p, b, t0 - 2, d) : 0.f;
    float u3 = conv ? input_at<bf16>(p, b, t0 - 3, d) : 0.f;
    // (no load under a condition - the compiler waits for such a load on the spot: steps past the
    // end re-read the last row and are dropped below)
    const bf16 *ucol = (const bf16 *)p.u + (size_t)b * p.T * p.D + d;
    float un[MT];
#pragma unroll
    for (int tt = 0; tt < MT; ++tt) un[tt] = ldf(ucol, (size_t)(t0 + tt < p.T ? t0 + tt : p.T - 1) * p.D);
#pragma unroll
    for (int tt = 0; tt < MT; ++tt) {
      const float u0 = un[tt];
      const float v = tt < nt ? fmaf(w0, u0, fmaf(w1, u1, fmaf(w2, u2, fmaf(w3, u3, cb)))) : 0.f;
      xf[tt * nin + k] = v;
      const _Float16 vh = (_Float16)v;
      xh[tt * xsh + k] = vh;
      xl[tt * xsh + k] = (_Float16)(v - (float)vh);
      u3 = u2;
      u2 = u1;
      u1 = u0;
    }
  }
  __syncthreads();
  const int lane = threadIdx.x & 63, hf = lane >> 5, j = lane & 31, wv = threadIdx.x >> 6;
  const _Float16 *arow = xh + mfma_arow(j) * xsh + hf * 8;
  for (int cb = wv; cb * 32 < hs; cb += NTHREADS / 64) {
    const int jj = cb * 32 + j;
    const bool ok = jj < hs;
    const int h = g * hs + (ok ? jj : hs - 1);
    const mfma::bf16x8 *wa = (const mfma::bf16x8 *)((const unsigned short *)p.W_a + (size_t)h * nin + hf * 8);
    const mfma::bf16x8 *wx = (const mfma::bf16x8 *)((const unsigned short *)p.W_x + (size_t)h * nin + hf * 8);
    mfma::f32x16 accp, accq;
    const float bp = p.b_a[h], bq = p.b_x[h];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      accp[r] = bp;
      accq[r] = bq;
    }
    for (int ks = 0; ks < nin / 16; ++ks) {
      const mfma::f16x8 a = *(const mfma::f16x8 *)(arow + ks * 16), al = *(const mfma::f16x8 *)(arow + MT * xsh + ks * 16);
      const mfma::f16x8 fa = mfma::w_to_f16(wa[ks * 2]), fx = mfma::w_to_f16(wx[ks * 2]);
      accp = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, fa, accp, 0, 0, 0);
      accq = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, fx, accq, 0, 0, 0);
      accp = __builtin_amdgcn_mfma_f32_32x32x16_f16(al, fa, accp, 0, 0, 0);
      accq = __builtin_amdgcn_mfma_f32_32x32x16_f16(al, fx, accq, 0, 0, 0);
    }
    if (!ok) continue;
    // (base-2 exponentials and the hardware's sine / cosine of an angle in revolutions)
    const float l2cs = -p.c * softplus_f(-p.Lambda[h]) * mfma::LOG2E, rev = p.c * p.theta[h] * 0.15915494309189535f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int tt = hf * 16 + r;
      if (tt < nt) {
        const float gr = __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-accp[r] * mfma::LOG2E));
        const float gi = __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-accq[r] * mfma::LOG2E));
        const float l2 = l2cs * gr, mod = __builtin_amdgcn_exp2f(l2);   // |a~_t| and its base-2 logarithm
        const float ar = mod * __builtin_amdgcn_cosf(rev * gr), ai = mod * __builtin_amdgcn_sinf(rev * gr);
        const float gain = __builtin_amdgcn_sqrtf(mfma::one_minus_sq(mod, l2)) * gi;
        const float xr = xf[tt * nin + jj], xi = xf[tt * nin + hs + jj];
        const size_t o = ((size_t)b * tc + (t0 - t_lo) + tt) * H + h;
        A[o] = make_float2(ar, ai);
        Bv[o] = make_float2(gain * xr, gain * xi);
      }
    }
    if (KEEP) {   // (a loop of its own: fused with the one above it took 300 registers)
      const size_t row0 = (size_t)b * p.T + t0 + hf * 16;
      float *xo = xk + row0 * p.D + h, *po = pq + row0 * H + h, *qo = po + (size_t)p.B * p.T * H;
      const float *xr = xf + (hf * 16) * nin + jj;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        if (hf * 16 + r < nt) {
          xo[(size_t)r * p.D] = xr[r * nin];
          xo[(size_t)r * p.D + H] = xr[r * nin + hs];
          po[(size_t)r * H] = accp[r];
          qo[(size_t)r * H] = accq[r];
        }
      }
    }
  }
}
// whether the matrix-core passes take this problem (bf16 storage is the caller's to check)
static bool cg_mfma_ok(const Problem &p) {
  return p.bs % 16 == 0 && p.bs <= 256 && ((uintptr_t)p.W_a % 16) == 0 && ((uintptr_t)p.W_x % 16) == 0;
}
// Fused forward (bf16 storage, hs = 32, 64, 96 or 128; needs no scratch): one workgroup of four
// waves per (gate block, sequence) walks the sequence in tiles of 32 steps and never parks the scan's
// coefficients. Per tile: the thread of input column k turns 32 prefetched inputs into Conv1D
// outputs (its last three inputs stay in registers from tile to tile); the gate products as in
// cg_coeff_mfma_kernel, a wave owning 32 complex channels; then every lane has a~_t, b~_t of one
// channel for 16 consecutive steps and runs the complex recurrence twice - from zero for its run's
// aggregate (product of a~_t, end state), which the two lane halves exchange, then from the true
// incoming state, writing y. The state stays in registers between tiles.
// KEEP (the backward's recomputation): y is the fp32 state array, and x, the pre-activations and
// a~_t are parked as cg_coeff_mfma_kernel<true> parks them - each stored where it is produced, so
// that nothing more stays live.
template <typename OT, bool KEEP>
__global__ void __launch_bounds__(NTHREADS) cg_fused_kernel(Problem p, float *xk, float *pq, float2 *A) {
  extern __shared__ __attribute__((aligned(16))) float smem[];
  const int g = blockIdx.x, b = blockIdx.y, hs = p.bs, H = p.D / 2, nin = 2 * hs, xsh = nin + 8;
  float *xf = smem;
  _Float16 *xh = (_Float16 *)(smem + MT * nin), *xl = xh + MT * xsh;
  const int T = p.T, ntile = (T + MT - 1) / MT;
  // ---- this thread's input column
  const int k = threadIdx.x;
  const bool col = k < nin, conv = p.conv_w != nullptr;
  const int dcol = cg_channel(g, hs, H, col ? k : 0);
  const float w0 = conv ? p.conv_w[dcol] : 1.f, w1 = conv ? p.conv_w[(size_t)p.D + dcol] : 0.f;
  const float w2 = conv ? p.conv_w[(size_t)2 * p.D + dcol] : 0.f, w3 = conv ? p.conv_w[(size_t)3 * p.D + dcol] : 0.f;
  const float cbias = (conv && p.conv_b) ? p.conv_b[dcol] : 0.f;
  float u1 = (conv && col) ? input_at<bf16>(p, b, -1, dcol) : 0.f, u2 = (conv && col) ? input_at<bf16>(p, b, -2, dcol) : 0.f;
  float u3 = (conv && col) ? input_at<bf16>(p, b, -3, dcol) : 0.f;
  const bf16 *ucol = (const bf16 *)p.u + (size_t)b * T * p.D + dcol;
  float un[MT];
  auto fetch = [&](int t0) __attribute__((always_inline)) {
#pragma unroll
    for (int tt = 0; tt < MT; ++tt) {   // (no load under a condition: the compiler would wait for each on the spot;
                                        // steps past the end re-read the last row and are dropped by the Conv1D below)
      const int t = t0 + tt < T ? t0 + tt : T - 1;
      un[tt] = ldf(ucol, (size_t)t * p.D);
    }
  };
  // ---- this lane's complex channel
  const int lane = threadIdx.x & 63, hf = lane >> 5, j = lane & 31, wv = threadIdx.x >> 6;
  const bool active = wv * 32 < hs;
  const int jj = wv * 32 + j, h = g * hs + (active ? jj : 0);
  const _Float16 *arow = xh + mfma_arow(j) * xsh + hf * 8;
  // this channel's rows of W_a and W_x stay in registers for the whole sequence (a wave runs alone
  // on its SIMD here, so it has the whole register file, and nothing would hide the latency of
  // fetching them per tile)
  const int nks = nin / 16;
  constexpr int RES = 16;   // K-steps of the weights kept in registers (all: 0 / 8 / 12 measured 50 / 18 / 10 % slower)
  mfma::f16x8 wra[RES > 0 ? RES : 1], wrx[RES > 0 ? RES : 1];
  const mfma::bf16x8 *wa = (const mfma::bf16x8 *)((const unsigned short *)p.W_a + (size_t)h * nin + hf * 8);
  const mfma::bf16x8 *wx = (const mfma::bf16x8 *)((const unsigned short *)p.W_x + (size_t)h * nin + hf * 8);
#pragma unroll
  for (int ks = 0; ks < RES; ++ks) {
    wra[ks] = mfma::w_to_f16(wa[(ks < nks ? ks : 0) * 2]);
    wrx[ks] = mfma::w_to_f16(wx[(ks < nks ? ks : 0) * 2]);
  }
  const float bp = p.b_a[h], bq = p.b_x[h];
  const float l2cs = -p.c * softplus_f(-p.Lambda[h]) * mfma::LOG2E, rev = p.c * p.theta[h] * 0.15915494309189535f;
  float sr = p.h0 ? p.h0[(size_t)b * p.D + h] : 0.f, si = p.h0 ? p.h0[(size_t)b * p.D + H + h] : 0.f;   // state entering the tile

  // parked arrays of this sequence as buffers (KEEP): per-lane offset = (first step of the lane's run, channel)
  const unsigned seq_elems = (unsigned)T * (unsigned)H;
  const __amdgpu_buffer_rsrc_t p_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      mfma::uniform_ptr(KEEP ? (void *)(pq + (size_t)b * seq_elems) : (void *)p.y), 0, KEEP ? seq_elems * 4u : 0u, 0x00020000);
  const __amdgpu_buffer_rsrc_t q_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      mfma::uniform_ptr(KEEP ? (void *)(pq + ((size_t)p.B + b) * seq_elems) : (void *)p.y), 0, KEEP ? seq_elems * 4u : 0u, 0x00020000);
  const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      mfma::uniform_ptr(KEEP ? (void *)(A + (size_t)b * seq_elems) : (void *)p.y), 0, KEEP ? seq_elems * 8u : 0u, 0x00020000);
  const unsigned k_voff = ((unsigned)(hf * 16) * (unsigned)H + (unsigned)h) * 4u;
  const unsigned row_elems = (unsigned)T * (unsigned)p.D;
  const __amdgpu_buffer_rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      mfma::uniform_ptr(KEEP ? (void *)(xk + (size_t)b * row_elems) : (void *)p.y), 0, KEEP ? row_elems * 4u : 0u, 0x00020000);
  const __amdgpu_buffer_rsrc_t y_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      mfma::uniform_ptr((OT *)p.y + (size_t)b * row_elems), 0, row_elems * (unsigned)sizeof(OT), 0x00020000);
  const unsigned y_voff = ((unsigned)(hf * 16) * (unsigned)p.D + (unsigned)h) * (unsigned)sizeof(OT);
  if (ntile > 0) fetch(0);
  for (int tile = 0; tile < ntile; ++tile) {
    const int t0 = tile * MT, nt = min(MT, T - t0);
    if (col) {
#pragma unroll
      for (int tt = 0; tt < MT; ++tt) {
        const float u0 = un[tt];
        const float v = tt < nt ? fmaf(w0, u0, fmaf(w1, u1, fmaf(w2, u2, fmaf(w3, u3, cbias)))) : 0.f;
        xf[tt * nin + k] = v;
        const _Float16 vh = (_Float16)v;
        xh[tt * xsh + k] = vh;
        xl[tt * xsh + k] = (_Float16)(v - (float)vh);
        if (KEEP && tt < nt)
          __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), x_rsrc, (unsigned)dcol * 4u, (unsigned)(t0 + tt) * (unsigned)p.D * 4u, 0);
        u3 = u2;
        u2 = u1;
        u1 = u0;
      }
    }
    __syncthreads();
    if (tile + 1 < ntile) fetch(t0 + MT);   // lands during the products and the recurrence
    if (active) {
      mfma::f32x16 accp, accq;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        accp[r] = bp;
        accq[r] = bq;
      }
      // (the K-steps that are not resident: all fragments of the tile requested up front)
      mfma::bf16x8 sa[RES < 16 ? 16 - RES : 1], sx[RES < 16 ? 16 - RES : 1];
#pragma unroll
      for (int ks = RES; ks < 16; ++ks) {
        sa[ks - RES] = wa[(ks < nks ? ks : 0) * 2];
        sx[ks - RES] = wx[(ks < nks ? ks : 0) * 2];
      }
#pragma unroll
      for (int ks = 0; ks < 16; ++ks) {
        if (ks < nks) {
          const mfma::f16x8 a = *(const mfma::f16x8 *)(arow + ks * 16), al = *(const mfma::f16x8 *)(arow + MT * xsh + ks * 16);
          const mfma::f16x8 fa = ks < RES ? wra[ks < RES ? ks : 0] : mfma::w_to_f16(sa[ks >= RES ? ks - RES : 0]);
          const mfma::f16x8 fx = ks < RES ? wrx[ks < RES ? ks : 0] : mfma::w_to_f16(sx[ks >= RES ? ks - RES : 0]);
          accp = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, fa, accp, 0, 0, 0);
          accq = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, fx, accq, 0, 0, 0);
          accp = __builtin_amdgcn_mfma_f32_32x32x16_f16(al, fa, accp, 0, 0, 0);
          accq = __builtin_amdgcn_mfma_f32_32x32x16_f16(al, fx, accq, 0, 0, 0);
        }
      }
      // gates, coefficients of this lane's 16 steps, and their aggregate from a zero state
      // (kept in registers between the two runs: parked in LDS instead they cost 10 % more time than
      // the spills they avoid)
      float car[16], cai[16], cbr[16], cbi[16];
      float Pr = 1.f, Pi = 0.f, Hr = 0.f, Hi = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int tt = hf * 16 + r;
        if (KEEP && tt < nt) {   // (scalar row offsets: no address registers per step)
          __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(accp[r]), p_rsrc, k_voff, (unsigned)(t0 + r) * (unsigned)H * 4u, 0);
          __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(accq[r]), q_rsrc, k_voff, (unsigned)(t0 + r) * (unsigned)H * 4u, 0);
        }
        const float gr = __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-accp[r] * mfma::LOG2E));
        const float gi = __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-accq[r] * mfma::LOG2E));
        const float l2 = l2cs * gr, mod = __builtin_amdgcn_exp2f(l2);
        float ar = mod * __builtin_amdgcn_cosf(rev * gr), ai = mod * __builtin_amdgcn_sinf(rev * gr);
        const float gain = __builtin_amdgcn_sqrtf(mfma::one_minus_sq(mod, l2)) * gi;
        float br = gain * xf[tt * nin + jj], bi = gain * xf[tt * nin + hs + jj];
        if (tt >= nt) {   // past the end of the sequence: the state passes through
          ar = 1.f; ai = 0.f; br = 0.f; bi = 0.f;
        } else if (KEEP) {
          typedef unsigned u32x2k __attribute__((ext_vector_type(2)));
          const u32x2k av = {__float_as_uint(ar), __float_as_uint(ai)};
          __builtin_amdgcn_raw_buffer_store_b64(av, a_rsrc, 2 * k_voff, (unsigned)(t0 + r) * (unsigned)H * 8u, 0);
        }
        car[r] = ar; cai[r] = ai; cbr[r] = br; cbi[r] = bi;
        const float nHr = fmaf(ar, Hr, fmaf(-ai, Hi, br)), nHi = fmaf(ar, Hi, fmaf(ai, Hr, bi));
        const float nPr = fmaf(ar, Pr, -ai * Pi), nPi = fmaf(ar, Pi, ai * Pr);
        Hr = nHr; Hi = nHi; Pr = nPr; Pi = nPi;
      }
      // lane halves: lower = steps 0..15, upper = 16..31
      const float oPr = __shfl_xor(Pr, 32), oPi = __shfl_xor(Pi, 32), oHr = __shfl_xor(Hr, 32), oHi = __shfl_xor(Hi, 32);
      const float Plr = hf ? oPr : Pr, Pli = hf ? oPi : Pi, Hlr = hf ? oHr : Hr, Hli = hf ? oHi : Hi;   // lower half's
      const float Pur = hf ? Pr : oPr, Pui = hf ? Pi : oPi, Hur = hf ? Hr : oHr, Hui = hf ? Hi : oHi;   // upper half's
      // state after the lower half's steps, then after the tile
      const float mr = fmaf(Plr, sr, fmaf(-Pli, si, Hlr)), mi = fmaf(Plr, si, fmaf(Pli, sr, Hli));
      const float er = fmaf(Pur, mr, fmaf(-Pui, mi, Hur)), ei = fmaf(Pur, mi, fmaf(Pui, mr, Hui));
      float hr = hf ? mr : sr, hi = hf ? mi : si;   // state entering this lane's run
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float nr = fmaf(car[r], hr, fmaf(-cai[r], hi, cbr[r])), ni = fmaf(car[r], hi, fmaf(cai[r], hr, cbi[r]));
        hr = nr;
        hi = ni;
        if (hf * 16 + r < nt && jj < hs) {
          const unsigned so = (unsigned)(t0 + r) * (unsigned)p.D * (unsigned)sizeof(OT);
          if (sizeof(OT) == 4) {
            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(hr), y_rsrc, y_voff, so, 0);
            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(hi), y_rsrc, y_voff + (unsigned)H * 4u, so, 0);
          } else {
            __builtin_amdgcn_raw_buffer_store_b16((short)f32_to_bf16_bits(hr), y_rsrc, y_voff, so, 0);
            __builtin_amdgcn_raw_buffer_store_b16((short)f32_to_bf16_bits(hi), y_rsrc, y_voff + (unsigned)H * 2u, so, 0);
          }
        }
      }
      sr = er;
      si = ei;
    }
    __syncthreads();   // the tile is consumed before the next Conv1D outputs overwrite it
  }
  if (p.hT && active && hf == 0 && jj < hs) {
    p.hT[(size_t)b * p.D + h] = sr;
    p.hT[(size_t)b * p.D + H + h] = si;
  }
}
// whether the fused forward takes this problem (bf16 storage is the caller's to check)
static bool cg_fused_ok(const Problem &p) {
  return p.bs % 32 == 0 && p.bs <= 128 && ((uintptr_t)p.W_a % 16) == 0 && ((uintptr_t)p.W_x % 16) == 0 && p.B <= 65535;
}
template <typename OT, bool KEEP>
static hipError_t launch_cg_fused(const Problem &p, float *xk, float *pq, float2 *A, hipStream_t s) {
  const size_t lds = (size_t)MT * 2 * p.bs * 4 + (size_t)2 * MT * (2 * p.bs + 8) * 2;
  if (lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute((const void *)cg_fused_kernel<OT, KEEP>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((cg_fused_kernel<OT, KEEP>), dim3(p.nb, p.B), dim3(NTHREADS), lds, s, p, xk, pq, A);
  return hipGetLastError();
}
template <typename OT>
__global__ void __launch_bounds__(NTHREADS) cg_scan_kernel(Problem p, int t_lo, int t_hi, const float2 *A,
                                                           const float2 *Bv, const float *h_in, float *h_out) {
  const int H = p.D / 2;
  const size_t n = (size_t)p.B * H, idx = (size_t)blockIdx.x * NTHREADS + threadIdx.x;
  if (idx >= n) return;
  const int b = (int)(idx / H), h = (int)(idx - (size_t)b * H), tc = t_hi - t_lo;
  float hr = h_in ? h_in[(size_t)b * p.D + h] : 0.f, hi = h_in ? h_in[(size_t)b * p.D + H + h] : 0.f;
  const float2 *a = A + (size_t)b * tc * H + h, *bv = Bv + (size_t)b * tc * H + h;
  OT *y = (OT *)p.y + ((size_t)b * p.T + t_lo) * p.D + h;
  int t = 0;
  for (; t + 16 <= tc; t += 16) {   // (the loads do not depend on the state: 16 steps of them in flight)
    float2 av[16], bb[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      av[k] = a[(size_t)(t + k) * H];
      bb[k] = bv[(size_t)(t + k) * H];
    }
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      const float nr = fmaf(av[k].x, hr, fmaf(-av[k].y, hi, bb[k].x));
      const float ni = fmaf(av[k].x, hi, fmaf(av[k].y, hr, bb[k].y));
      hr = nr;
      hi = ni;
      stf(y, (size_t)(t + k) * p.D, hr);
      stf(y, (size_t)(t + k) * p.D + H, hi);
    }
  }
  for (; t < tc; ++t) {
    const float2 av = a[(size_t)t * H], bb = bv[(size_t)t * H];
    const float nr = fmaf(av.x, hr, fmaf(-av.y, hi, bb.x));
    const float ni = fmaf(av.x, hi, fmaf(av.y, hr, bb.y));
    hr = nr;
    hi = ni;
    stf(y, (size_t)t * p.D, hr);
    stf(y, (size_t)t * p.D + H, hi);
  }
  if (h_out) {
    h_out[(size_t)b * p.D + h] = hr;
    h_out[(size_t)b * p.D + H + h] = hi;
  }
}

// ---------------------------------------------------------------------------- decode
// One workgroup per (gate block, tile of GT sequences); states updated in place. The ring slot
// of the new token is written by the workgroup that owns the channels, after all its reads.
template <typename AT>
__global__ void __launch_bounds__(NTHREADS) cg_decode_kernel(Problem p) {
  extern __shared__ __attribute__((aligned(16))) float smem[];
  const int g = blockIdx.x, b0 = blockIdx.y * GT, hs = p.bs, H = p.D / 2, tid = threadIdx.x;
  const int nbat = min(GT, p.B - b0);
  float *xs = smem;
  AT *state = (AT *)p.state_out;  // in-place ring
  for (int idx = tid; idx < GT * 2 * hs; idx += NTHREADS) {
    const int tt = idx / (2 * hs), k = idx - tt * 2 * hs, d = cg_channel(g, hs, H, k);
    float acc = 0.f;
    if (tt < nbat) {
      const int b = b0 + tt;
      if (!p.conv_w) {
        acc = ldf((const AT *)p.u, (size_t)b * p.D + d);
      } else {
        acc = p.conv_b ? p.conv_b[d] : 0.f;
        acc = fmaf(p.conv_w[d], ldf((const AT *)p.u, (size_t)b * p.D + d), acc);
#pragma unroll
        for (int l = 1; l < 4; ++l)
          acc = fmaf(p.conv_w[(size_t)l * p.D + d],
                     ldf(state, ((size_t)b * 3 + ring_slot(p.pos0 - l)) * p.D + d), acc);
      }
    }
    xs[idx] = acc;
  }
  __syncthreads();
  for (int j = tid; j < hs; j += NTHREADS) {
    const int h = g * hs + j;
    float pa[GT], qa[GT];
    cg_gate_rows<AT>(p, g, j, xs, pa, qa);
    const float neg_cs = -p.c * softplus_f(-p.Lambda[h]), c_theta = p.c * p.theta[h];
#pragma unroll
    for (int tt = 0; tt < GT; ++tt) {
      if (tt < nbat) {
        const size_t o = (size_t)(b0 + tt) * p.D;
        const CGates gt = cg_gate_math(pa[tt], qa[tt], neg_cs, c_theta);
        const float gain = gt.m * gt.i, hr = p.hT[o + h], hi = p.hT[o + H + h];
        const float nr = fmaf(gt.ar, hr, fmaf(-gt.ai, hi, gain * xs[tt * 2 * hs + j]));
        const float ni = fmaf(gt.ar, hi, fmaf(gt.ai, hr, gain * xs[tt * 2 * hs + hs + j]));
        p.hT[o + h] = nr;
        p.hT[o + H + h] = ni;
        stf((AT *)p.y, o + h, nr);
        stf((AT *)p.y, o + H + h, ni);
        if (state) {
          const size_t so = ((size_t)(b0 + tt) * 3 + ring_slot(p.pos0)) * p.D;
          state[so + h] = ((const AT *)p.u)[o + h];
          state[so + H + h] = ((const AT *)p.u)[o + H + h];
        }
      }
    }
  }
}

// --------------------------------------------------------------------------- backward
// Pass 0 is the forward once more (two passes, parallel over time), writing the states h~_t in
// fp32 into the workspace (`hs32`): the gradient of the decay multiplies delta~_t by
// conj(h~_{t-1}), and with the phases in play the 8 bits of a bf16 y would leave dW_a some 3e-2
// off. It parks x, the pre-activations and the coefficients a~_t as well.
// Pass 1a: the adjoint of the state is complex, delta~_t = dy~_t + conj(a~_{t+1}) delta~_{t+1} (a
// complex number standing for the pair of derivatives with respect to the real and the imaginary
// part): a linear recurrence backwards in time over the parked a~_t, one thread per (sequence,
// complex channel) with the loads of 16 steps in flight; delta~_t goes where pass 0 had the
// b~_t. Nothing else is serial in time.
template <typename AT>
__global__ void __launch_bounds__(NTHREADS) cg_adj_scan_kernel(Problem p, const float2 *A, float2 *delta) {
  const int H = p.D / 2;
  const size_t n = (size_t)p.B * H, idx = (size_t)blockIdx.x * NTHREADS + threadIdx.x;
  if (idx >= n) return;
  const int b = (int)(idx / H), h = (int)(idx - (size_t)b * H);
  float cr = p.dhT ? p.dhT[(size_t)b * p.D + h] : 0.f, ci = p.dhT ? p.dhT[(size_t)b * p.D + H + h] : 0.f;
  const float2 *a = A + (size_t)b * p.T * H + h;
  float2 *dl = delta + (size_t)b * p.T * H + h;
  const AT *dy = (const AT *)p.dy + (size_t)b * p.T * p.D + h;
  int t = p.T;
  for (; t >= 16; t -= 16) {   // steps t-1 down to t-16
    float2 av[16];
    float yr[16], yi[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      const size_t tt = (size_t)(t - 1 - k);
      av[k] = a[tt * H];
      yr[k] = ldf(dy, tt * p.D);
      yi[k] = ldf(dy, tt * p.D + H);
    }
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      const float dr_ = yr[k] + cr, di_ = yi[k] + ci;
      dl[(size_t)(t - 1 - k) * H] = make_float2(dr_, di_);
      cr = fmaf(av[k].x, dr_, av[k].y * di_);    // conj(a~_t) delta~_t
      ci = fmaf(av[k].x, di_, -av[k].y * dr_);
    }
  }
  for (; t > 0; --t) {
    const size_t tt = (size_t)(t - 1);
    const float2 av = a[tt * H];
    const float dr_ = ldf(dy, tt * p.D) + cr, di_ = ldf(dy, tt * p.D + H) + ci;
    dl[tt * H] = make_float2(dr_, di_);
    cr = fmaf(av.x, dr_, av.y * di_);
    ci = fmaf(av.x, di_, -av.y * dr_);
  }
  if (p.dh0) {
    p.dh0[(size_t)b * p.D + h] = cr;
    p.dh0[(size_t)b * p.D + H + h] = ci;
  }
}

// Pass 1b, parallel over time: a thread takes PCH consecutive steps of one complex channel and
// forms, from delta~_t and what pass 0 parked, the gate adjoints (dp, dq) - written as a pair over
// the a~_t it has just read - and the direct part of dx; a workgroup is 64 channels x 4 such runs,
// whose sums for db_a, db_x, dLambda, dtheta it adds up in a fixed order into one row of `parts`
// ([B * gridDim.z][4][H]; four steps as plain sums at a time, compensated beyond).
constexpr int PCH = 64;
template <typename AT>
__global__ void __launch_bounds__(NTHREADS) cg_bwd_point_kernel(Problem p, BwdWs w, const float *hs32, const float *pq,
                                                                float2 *adpq, const float2 *delta, float *parts) {
  __shared__ float red[4][4][64];
  const int H = p.D / 2, hl = threadIdx.x & 63, cq = threadIdx.x >> 6;
  const int h = blockIdx.x * 64 + hl, b = blockIdx.y;
  const int t_lo = (blockIdx.z * 4 + cq) * PCH, t_hi = min(p.T, t_lo + PCH);
  float sum[4] = {0.f, 0.f, 0.f, 0.f}, comp[4] = {0.f, 0.f, 0.f, 0.f};
  if (h < H && t_lo < t_hi) {
    const float theta = p.theta[h];
    const float log_sig = -softplus_f(-p.Lambda[h]);         // log sigmoid(Lambda)
    const float neg_cs = p.c * log_sig;
    const float lam_scale = p.c * sigmoid_f(-p.Lambda[h]);   // c d log sigmoid(Lambda) / d Lambda
    const size_t rows = (size_t)p.B * p.T;
    for (int t0 = t_lo; t0 < t_hi; t0 += 4) {
      const int cnt = min(4, t_hi - t0);
      float pv[4], qv[4], xr[4], xi[4], pr[4], pi[4];
      float2 av[4], dv[4];
      // (no load under a condition - the compiler would wait for each on the spot: steps past the
      // run re-read its last step, step 0 reads the state of step 0 in place of the one before it
      // and takes h0 afterwards)
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int t = k < cnt ? t0 + k : t_hi - 1;
        const size_t row = (size_t)b * p.T + t, o = row * p.D, op = t > 0 ? o - p.D : o;
        pv[k] = pq[row * H + h];
        qv[k] = pq[(rows + row) * H + h];
        xr[k] = w.x[o + h];
        xi[k] = w.x[o + H + h];
        av[k] = adpq[row * H + h];
        dv[k] = delta[row * H + h];
        pr[k] = hs32[op + h];
        pi[k] = hs32[op + H + h];
      }
      if (t0 == 0) {
        pr[0] = p.h0 ? p.h0[(size_t)b * p.D + h] : 0.f;
        pi[0] = p.h0 ? p.h0[(size_t)b * p.D + H + h] : 0.f;
      }
      float s_ba = 0.f, s_bx = 0.f, s_lam = 0.f, s_th = 0.f;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if (k < cnt) {
          const size_t row = (size_t)b * p.T + t0 + k, o = row * p.D;
          const float r = sigmoid_f(pv[k]), rc = sigmoid_f(-pv[k]), gi = sigmoid_f(qv[k]), ic = sigmoid_f(-qv[k]);
          const float lm2 = 2.f * neg_cs * r;              // log |a~_t|^2 <= 0
          const float mod2 = expf(lm2), m = sqrtf(-expm1f(lm2));
          const float dr_ = dv[k].x, di_ = dv[k].y, ar = av[k].x, ai = av[k].y;
          // G = delta~ conj(h~_{t-1}) = (dL/dRe a~_t, dL/dIm a~_t)
          const float Gr = fmaf(dr_, pr[k], di_ * pi[k]), Gi = fmaf(di_, pr[k], -dr_ * pi[k]);
          const float s = fmaf(dr_, xr[k], di_ * xi[k]);   // dL/d(m_t i_t)
          // a~_t = exp(lm + i ph): d/d lm = a~_t, d/d ph = i a~_t;  m_t = sqrt(1 - e^{2 lm})
          float dlm = fmaf(Gr, ar, Gi * ai);
          const float dph = fmaf(Gi, ar, -Gr * ai);
          if (m > 0.f) dlm -= s * gi * mod2 / m;
          const float dgate_r = p.c * fmaf(dlm, log_sig, dph * theta);
          const float dpv = dgate_r * r * rc;
          const float dqv = s * m * gi * ic;
          s_lam = fmaf(dlm * r, lam_scale, s_lam);
          s_th = fmaf(dph * r, p.c, s_th);
          s_ba += dpv;
          s_bx += dqv;
          adpq[row * H + h] = make_float2(dpv, dqv);
          const float gain = m * gi;
          w.dx[o + h] = dr_ * gain;
          w.dx[o + H + h] = di_ * gain;
        }
      }
      comp_add(sum[0], comp[0], s_ba);
      comp_add(sum[1], comp[1], s_bx);
      comp_add(sum[2], comp[2], s_lam);
      comp_add(sum[3], comp[3], s_th);
    }
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) red[cq][q][hl] = sum[q];
  __syncthreads();
  if (cq == 0 && h < H) {
#pragma unroll
    for (int q = 0; q < 4; ++q)
      parts[(((size_t)b * gridDim.z + blockIdx.z) * 4 + q) * H + h] =
          ((red[0][q][hl] + red[1][q][hl]) + red[2][q][hl]) + red[3][q][hl];
  }
}

// Pass 2: dx[t][chan(k)] += sum_j W_a[g][j][k] dp[t][j] + W_x[g][j][k] dq[t][j]   (dpq: the (dp, dq) pairs [B*T][H])
template <typename AT>
__global__ void __launch_bounds__(NTHREADS) cg_bwd_dgrad_kernel(Problem p, BwdWs w, const float2 *dpq) {
  extern __shared__ __attribute__((aligned(16))) float smem[];
  const int g = blockIdx.x, b = blockIdx.y, t0 = blockIdx.z * GT, hs = p.bs, H = p.D / 2, tid = threadIdx.x;
  const int nt = min(GT, p.T - t0), nin = 2 * hs;
  float *dps = smem, *dqs = smem + GT * hs;   // [GT][hs] each
  for (int idx = tid; idx < GT * hs; idx += NTHREADS) {
    const int tt = idx / hs, j = idx - tt * hs;
    const size_t o = ((size_t)b * p.T + t0 + tt) * H + g * hs + j;
    const float2 v = tt < nt ? dpq[o] : make_float2(0.f, 0.f);
    dps[idx] = v.x;
    dqs[idx] = v.y;
  }
  __syncthreads();
  const AT *Wa = (const AT *)p.W_a + (size_t)g * hs * nin;
  const AT *Wx = (const AT *)p.W_x + (size_t)g * hs * nin;
  for (int k = tid; k < nin; k += NTHREADS) {
    const int d = cg_channel(g, hs, H, k);
    float acc[GT];
#pragma unroll
    for (int tt = 0; tt < GT; ++tt) acc[tt] = tt < nt ? w.dx[((size_t)b * p.T + t0 + tt) * p.D + d] : 0.f;
    for (int j = 0; j < hs; ++j) {
      const float wa = ldf(Wa, (size_t)j * nin + k), wx = ldf(Wx, (size_t)j * nin + k);
#pragma unroll
      for (int tt = 0; tt < GT; ++tt)
        acc[tt] = fmaf(wa, dps[tt * hs + j], fmaf(wx, dqs[tt * hs + j], acc[tt]));
    }
#pragma unroll
    for (int tt = 0; tt < GT; ++tt)
      if (tt < nt) w.dx[((size_t)b * p.T + t0 + tt) * p.D + d] = acc[tt];
  }
}

// Pass 2 on the matrix cores (bf16 storage, hs a multiple of 16 up to 256). The contraction runs
// over a block's 2 hs gate outputs (dp against W_a, dq against W_x), so the weights are needed
// transposed: cg_wt_kernel writes wt[g][k][jj] = W_a[g][jj][k] for jj < hs, W_x[g][jj - hs][k] beyond
// (bf16, exact) into the workspace. A workgroup of four waves takes 32 steps of one (gate block,
// sequence): the (dp, dq) tile in LDS as bf16 high + low parts (16 significant bits at the full
// fp32 exponent range), a wave owns 32 of the 2 hs inputs at a time and adds its products to dx.
__global__ void __launch_bounds__(NTHREADS) cg_wt_kernel(Problem p, unsigned short *wt) {
  const int hs = p.bs, nin = 2 * hs;
  const size_t n = (size_t)p.nb * nin * nin, i = (size_t)blockIdx.x * NTHREADS + threadIdx.x;
  if (i >= n) return;
  const int g = (int)(i / ((size_t)nin * nin)), rem = (int)(i - (size_t)g * nin * nin), k = rem / nin, jj = rem - k * nin;
  const unsigned short *src = (const unsigned short *)(jj < hs ? p.W_a : p.W_x);
  wt[i] = src[((size_t)g * hs + (jj < hs ? jj : jj - hs)) * nin + k];
}
__global__ void __launch_bounds__(NTHREADS) cg_dgrad_mfma_kernel(Problem p, BwdWs w, const float2 *dpq,
                                                                 const unsigned short *wt) {
  extern __shared__ __attribute__((aligned(16))) unsigned short dsm[];
  const int g = blockIdx.x, b = blockIdx.y, t0 = blockIdx.z * MT, hs = p.bs, H = p.D / 2, nin = 2 * hs;
  const int nt = min(MT, p.T - t0), xs = nin + 8;
  unsigned short *a_hi = dsm, *a_lo = dsm + MT * xs;   // [MT][nin + 8] each: dp of the hs outputs, then dq
  for (int jc = threadIdx.x; jc < hs; jc += NTHREADS) {   // a thread walks one output column down the tile
    const float2 *src = dpq + ((size_t)b * p.T + t0) * H + (size_t)g * hs + jc;
#pragma unroll 8
    for (int tt = 0; tt < MT; ++tt) {
      float2 v = src[(size_t)(tt < nt ? tt : nt - 1) * H];   // (no load under a condition)
      if (tt >= nt) v = make_float2(0.f, 0.f);
      unsigned hi, lo;
      mfma::split_bf16(v.x, v.y, hi, lo);
      a_hi[tt * xs + jc] = (unsigned short)(hi & 0xffff);
      a_hi[tt * xs + hs + jc] = (unsigned short)(hi >> 16);
      a_lo[tt * xs + jc] = (unsigned short)(lo & 0xffff);
      a_lo[tt * xs + hs + jc] = (unsigned short)(lo >> 16);
    }
  }
  __syncthreads();
  const int lane = threadIdx.x & 63, hf = lane >> 5, j = lane & 31, wv = threadIdx.x >> 6;
  const int aoff = mfma_arow(j) * xs + hf * 8;
  for (int cb = wv; cb * 32 < nin; cb += NTHREADS / 64) {
    const int k = cb * 32 + j;   // (nin is a multiple of 32)
    const mfma::bf16x8 *wk = (const mfma::bf16x8 *)(wt + ((size_t)g * nin + k) * nin + hf * 8);
    mfma::f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    for (int ks = 0; ks < nin / 16; ++ks) {
      const mfma::bf16x8 bw = wk[ks * 2];
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const mfma::bf16x8 *)(a_hi + aoff + ks * 16), bw, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const mfma::bf16x8 *)(a_lo + aoff + ks * 16), bw, acc, 0, 0, 0);
    }
    float *dst = w.dx + ((size_t)b * p.T + t0 + hf * 16) * p.D + cg_channel(g, hs, H, k);
#pragma unroll
    for (int r = 0; r < 16; ++r)
      if (hf * 16 + r < nt) dst[(size_t)r * p.D] += acc[r];
  }
}

// Pass 4: dW_a[g][j][k] = sum_{b,t} dp[b,t,j] x[b,t,chan(k)], dW_x likewise with dq. One
// workgroup per 32x32 output tile of one block, 16x16 threads with 2x2 outputs each, rows
// streamed through LDS 32 at a time; the chunks of 32 rows are added up with compensation.
__global__ void __launch_bounds__(NTHREADS) cg_bwd_wgrad_kernel(Problem p, BwdWs w, const float2 *dpq) {
  __shared__ float xs[32][33], ps[32][33], qs[32][33];
  const int g = blockIdx.x, j0 = blockIdx.y * 32, k0 = blockIdx.z * 32, hs = p.bs, H = p.D / 2, nin = 2 * hs;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float aa[2][2] = {{0.f, 0.f}, {0.f, 0.f}}, ax[2][2] = {{0.f, 0.f}, {0.f, 0.f}};
  float ca[2][2] = {{0.f, 0.f}, {0.f, 0.f}}, cx[2][2] = {{0.f, 0.f}, {0.f, 0.f}};
  const size_t rows = (size_t)p.B * p.T;
  for (size_t r0 = 0; r0 < rows; r0 += 32) {
    __syncthreads();
    for (int idx = threadIdx.x; idx < 32 * 32; idx += NTHREADS) {
      const int rr = idx >> 5, cc = idx & 31;
      const size_t row = r0 + rr;
      const bool okr = row < rows;
      xs[rr][cc] = (okr && k0 + cc < nin) ? w.x[row * p.D + cg_channel(g, hs, H, k0 + cc)] : 0.f;
      const float2 v = (okr && j0 + cc < hs) ? dpq[row * H + g * hs + j0 + cc] : make_float2(0.f, 0.f);
      ps[rr][cc] = v.x;
      qs[rr][cc] = v.y;
    }
    __syncthreads();
    float la[2][2] = {{0.f, 0.f}, {0.f, 0.f}}, lx[2][2] = {{0.f, 0.f}, {0.f, 0.f}};
#pragma unroll 8
    for (int rr = 0; rr < 32; ++rr) {
      const float x0 = xs[rr][tx], x1 = xs[rr][tx + 16];
      const float p0 = ps[rr][ty], p1 = ps[rr][ty + 16];
      const float q0 = qs[rr][ty], q1 = qs[rr][ty + 16];
      la[0][0] = fmaf(p0, x0, la[0][0]); la[0][1] = fmaf(p0, x1, la[0][1]);
      la[1][0] = fmaf(p1, x0, la[1][0]); la[1][1] = fmaf(p1, x1, la[1][1]);
      lx[0][0] = fmaf(q0, x0, lx[0][0]); lx[0][1] = fmaf(q0, x1, lx[0][1]);
      lx[1][0] = fmaf(q1, x0, lx[1][0]); lx[1][1] = fmaf(q1, x1, lx[1][1]);
    }
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        comp_add(aa[a][c], ca[a][c], la[a][c]);
        comp_add(ax[a][c], cx[a][c], lx[a][c]);
      }
  }
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      const int j = j0 + ty + 16 * a, k = k0 + tx + 16 * c;
      if (j < hs && k < nin) {
        p.g.dW_a[((size_t)g * hs + j) * nin + k] = aa[a][c];
        p.g.dW_x[((size_t)g * hs + j) * nin + k] = ax[a][c];
      }
    }
}

// The same contraction on the matrix cores (bf16 storage, hs a multiple of 16 up to 128). Time
// is the contraction index, so both operands are staged transposed - [output j][step] for the
// (dp, dq) pairs, [input k][step] for x - each as a bf16 high part + low part (16 significant
// bits at the full fp32 exponent range: gradients may be arbitrarily small or large), and a
// product is hi*hi + hi*lo + lo*hi. A workgroup of eight waves accumulates one gate block's
// [2 hs][2 hs] gradient (rows: W_a's outputs, then W_x's) over a slice of the B*T rows, 32 rows at a
// time: wave w owns output rows 32 w .. 32 w + 31 against every column block. The next 32 rows are
// fetched into registers while the products run. The slices' partial sums ([S][nb][2 hs][2 hs])
// are added up in a fixed order by cg_wgrad_reduce_kernel.
constexpr int WRS = MT + 8;   // row stride of the transposed tiles (bf16 elements)
__global__ void __launch_bounds__(512) cg_wgrad_mfma_kernel(Problem p, BwdWs w, const float2 *dpq, float *part,
                                                            int rows_per) {
  extern __shared__ __attribute__((aligned(16))) unsigned short wsm[];
  const int g = blockIdx.x, sl = blockIdx.y, hs = p.bs, H = p.D / 2, nin = 2 * hs, ncb = nin / 32;
  unsigned short *d_hi = wsm, *d_lo = wsm + nin * WRS, *x_hi = wsm + 2 * nin * WRS, *x_lo = wsm + 3 * nin * WRS;
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5, j = lane & 31, wv = tid >> 6;
  const size_t rows = (size_t)p.B * p.T;
  const size_t r_lo = (size_t)sl * rows_per, r_hi = r_lo + rows_per < rows ? r_lo + rows_per : rows;
  // a thread stages 8 consecutive rows of one output's (dp, dq) and 16 consecutive rows of one
  // input's x: eight (sixteen) steps of a channel are one (two) 16-byte pieces of a transposed row
  const int jc = tid & 127, rg = tid >> 7;    // (dp, dq): complex channel jc of the block, rows 8 rg ..
  const int kx = tid & 255, rg2 = tid >> 8;   // x: input kx of the block, rows 16 rg2 ..
  const bool d_ok = jc < hs, x_ok = kx < nin;
  const float2 *dsrc = dpq + (size_t)g * hs + (d_ok ? jc : 0);
  const float *xsrc = w.x + cg_channel(g, hs, H, x_ok ? kx : 0);
  float2 dv[8];
  float xv[16];
  auto fetch = [&](size_t r0) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const size_t row = r0 + 8 * rg + i;   // (no load under a condition: rows past the slice re-read its last row)
      dv[i] = dsrc[(row < r_hi ? row : r_hi - 1) * H];
      if (!d_ok || row >= r_hi) dv[i] = make_float2(0.f, 0.f);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const size_t row = r0 + 16 * rg2 + i;
      xv[i] = xsrc[(row < r_hi ? row : r_hi - 1) * p.D];
      if (!x_ok || row >= r_hi) xv[i] = 0.f;
    }
  };
  typedef unsigned u32x4w __attribute__((ext_vector_type(4)));
  auto park = [&]() __attribute__((always_inline)) {
    if (d_ok) {
      u32x4w ph, pl, qh, ql;   // dp: high, low; dq: high, low
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        unsigned hi, lo;
        mfma::split_bf16(dv[2 * i].x, dv[2 * i + 1].x, hi, lo);
        ph[i] = hi;
        pl[i] = lo;
        mfma::split_bf16(dv[2 * i].y, dv[2 * i + 1].y, hi, lo);
        qh[i] = hi;
        ql[i] = lo;
      }
      *(u32x4w *)(d_hi + jc * WRS + 8 * rg) = ph;
      *(u32x4w *)(d_lo + jc * WRS + 8 * rg) = pl;
      *(u32x4w *)(d_hi + (hs + jc) * WRS + 8 * rg) = qh;
      *(u32x4w *)(d_lo + (hs + jc) * WRS + 8 * rg) = ql;
    }
    if (x_ok) {
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        u32x4w xh4, xl4;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          unsigned hi, lo;
          mfma::split_bf16(xv[8 * half + 2 * i], xv[8 * half + 2 * i + 1], hi, lo);
          xh4[i] = hi;
          xl4[i] = lo;
        }
        *(u32x4w *)(x_hi + kx * WRS + 16 * rg2 + 8 * half) = xh4;
        *(u32x4w *)(x_lo + kx * WRS + 16 * rg2 + 8 * half) = xl4;
      }
    }
  };
  mfma::f32x16 acc[8];
#pragma unroll
  for (int cb = 0; cb < 8; ++cb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[cb][r] = 0.f;
  const bool active = wv * 32 < nin;
  if (r_lo < r_hi) fetch(r_lo);
  for (size_t r0 = r_lo; r0 < r_hi; r0 += MT) {
    __syncthreads();   // the previous tile's products are done with the buffers
    park();
    __syncthreads();
    if (r0 + MT < r_hi) fetch(r0 + MT);
    if (active) {
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const int off = (wv * 32 + j) * WRS + 16 * q + 8 * hf;
        const mfma::bf16x8 a_hi = *(const mfma::bf16x8 *)(d_hi + off), a_lo = *(const mfma::bf16x8 *)(d_lo + off);
#pragma unroll
        for (int cb = 0; cb < 8; ++cb) {
          if (cb < ncb) {
            const int bo = (cb * 32 + j) * WRS + 16 * q + 8 * hf;
            const mfma::bf16x8 b_hi = *(const mfma::bf16x8 *)(x_hi + bo), b_lo = *(const mfma::bf16x8 *)(x_lo + bo);
            acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi, b_hi, acc[cb], 0, 0, 0);
            acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi, b_lo, acc[cb], 0, 0, 0);
            acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_lo, b_hi, acc[cb], 0, 0, 0);
          }
          if (cb & 1) __builtin_amdgcn_sched_barrier(0);   // (two column blocks' fragments in flight, not all eight)
        }
      }
    }
  }
  if (active) {
    float *out = part + ((size_t)sl * p.nb + g) * nin * nin;
#pragma unroll
    for (int cb = 0; cb < 8; ++cb) {
      if (cb < ncb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = wv * 32 + 8 * (r >> 2) + 4 * hf + (r & 3), col = cb * 32 + j;
          out[(size_t)row * nin + col] = acc[cb][r];
        }
      }
    }
  }
}
// dW_a[g][j][k], dW_x[g][j][k] from the S partial [2 hs][2 hs] sums of every block, in a fixed order
__global__ void __launch_bounds__(NTHREADS) cg_wgrad_reduce_kernel(Problem p, const float *part, int S) {
  const int hs = p.bs, nin = 2 * hs;
  const size_t per = (size_t)p.nb * nin * nin, i = (size_t)blockIdx.x * NTHREADS + threadIdx.x;
  if (i >= per) return;
  float sum = 0.f, comp = 0.f;
  for (int s = 0; s < S; ++s) comp_add(sum, comp, part[(size_t)s * per + i]);
  const int g = (int)(i / ((size_t)nin * nin)), rem = (int)(i - (size_t)g * nin * nin), jj = rem / nin, k = rem - jj * nin;
  float *dst = jj < hs ? p.g.dW_a : p.g.dW_x;
  dst[((size_t)g * hs + (jj < hs ? jj : jj - hs)) * nin + k] = sum;
}
static bool cg_wgrad_mfma_ok(int hs) { return hs % 16 == 0 && hs <= 128; }
// slices of the B*T rows that the matrix-core wgrad pass runs in: enough workgroups for the chip,
// no slice shorter than 256 rows
static int cg_wgrad_slices(size_t rows, int nb) {
  int S = (256 + nb - 1) / nb;
  const size_t most = (rows + 255) / 256;
  if ((size_t)S > most) S = (int)most;
  return S < 1 ? 1 : S;
}
// workspace of the matrix-core passes behind the partial sums of pass 1b: the wgrad pass's partial
// sums, then the transposed weights of the dgrad pass (sized whatever the storage type turns out to be)
static size_t cg_wgrad_part_bytes(size_t rows, int nb, int hs) {
  return cg_wgrad_mfma_ok(hs) ? align256((size_t)cg_wgrad_slices(rows, nb) * nb * 4 * hs * hs * sizeof(float)) : 0;
}
static size_t cg_wt_bytes(int nb, int hs) { return (hs % 16 == 0 && hs <= 256) ? align256((size_t)nb * 4 * hs * hs * 2) : 0; }

template <typename K>
hipError_t allow_lds(K kernel, size_t bytes) {
  if (bytes <= 48 * 1024) return hipSuccess;
  return hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

// the forward over steps [0, T) in chunks of at most `tcmax` steps: coefficients into A / Bv, then the
// recurrence; `hstate` carries the state between chunks; y of storage type OT
template <typename AT, typename OT, bool KEEP = false>
hipError_t cg_forward_two_pass(const Problem &p, int tcmax, float2 *A, float2 *Bv, float *hstate, hipStream_t s,
                               float *xk = nullptr, float *pq = nullptr) {
  const int hs = p.bs, H = p.D / 2;
  const bool on_mfma = sizeof(AT) == 2 && cg_mfma_ok(p);
  const size_t lds = on_mfma ? (size_t)MT * 2 * hs * 4 + (size_t)2 * MT * (2 * hs + 8) * 2 : (size_t)CTG * 2 * hs * sizeof(float);
  hipError_t e = on_mfma ? allow_lds(cg_coeff_mfma_kernel<KEEP>, lds) : allow_lds(cg_coeff_kernel<AT, KEEP>, lds);
  if (e != hipSuccess) return e;
  const int sblocks = (int)(((size_t)p.B * H + NTHREADS - 1) / NTHREADS), steps = on_mfma ? MT : CTG;
  for (int t_lo = 0; t_lo < p.T; t_lo += tcmax) {
    const int t_hi = t_lo + tcmax < p.T ? t_lo + tcmax : p.T, ntile = (t_hi - t_lo + steps - 1) / steps;
    if (ntile > 65535) return hipErrorInvalidConfiguration;
    if (on_mfma)
      hipLaunchKernelGGL((cg_coeff_mfma_kernel<KEEP>), dim3(p.nb, p.B, ntile), dim3(NTHREADS), lds, s, p, t_lo, t_hi, A,
                         Bv, xk, pq);
    else
      hipLaunchKernelGGL((cg_coeff_kernel<AT, KEEP>), dim3(p.nb, p.B, ntile), dim3(NTHREADS), lds, s, p, t_lo, t_hi, A,
                         Bv, xk, pq);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const bool last = t_hi == p.T;
    hipLaunchKernelGGL(cg_scan_kernel<OT>, dim3(sblocks), dim3(NTHREADS), 0, s, p, t_lo, t_hi, A, Bv,
                       t_lo == 0 ? p.h0 : hstate, last ? p.hT : hstate);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  return hipSuccess;
}

// rows of partial sums per sequence that pass 1b leaves: one per 4 runs of PCH steps
static int cg_point_rows(int T) { return ((T + PCH - 1) / PCH + 3) / 4; }

template <typename AT>
hipError_t cg_backward_t(const Problem &p, hipStream_t s) {
  const BwdWs w = carve_bwd_ws(p.ws, p.B, p.T, p.D);
  const int hs = p.bs, H = p.D / 2;
  const size_t lds2 = (size_t)(2 * GT * hs) * sizeof(float);
  hipError_t e;
  const int ntile = (p.T + GT - 1) / GT;
  if (ntile > 65535 || p.B > 65535) return hipErrorInvalidConfiguration;
  const size_t nbytes = ((size_t)p.B * p.T * p.D * sizeof(float) + 255) & ~(size_t)255;
  float *hs32 = (float *)((char *)p.ws + backward_generic_ws_bytes(p.B, p.T, p.D, p.nb));
  float *pq = (float *)((char *)hs32 + nbytes);
  float *parts = (float *)((char *)pq + nbytes);
  float2 *adpq = (float2 *)w.dp, *delta = (float2 *)w.dq;   // a~_t, then (dp, dq); b~_t, then delta~_t
  {   // pass 0: the forward once more, in two passes (the dp and dq arrays, not yet in use, hold the scan's
      // coefficients of the whole sequence); it parks x and the pre-activations for pass 1
    Problem f = p;
    f.y = hs32;
    f.hT = nullptr;
    // (with enough (gate block, sequence) pairs for the chip the fused kernel does it in one pass:
    // 6.9 -> 6.15 ms for the whole backward at 256 pairs; at 80 pairs the two passes, which are
    // parallel over time, are 2 % ahead. It parks a~_t but no b~_t: nothing reads them.)
    if (sizeof(AT) == 2 && cg_fused_ok(p) && p.B * p.nb >= 160)
      e = launch_cg_fused<float, true>(f, w.x, pq, (float2 *)w.dp, s);
    else
      e = cg_forward_two_pass<AT, float, true>(f, p.T, (float2 *)w.dp, (float2 *)w.dq, nullptr, s, w.x, pq);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(cg_adj_scan_kernel<AT>, dim3((unsigned)(((size_t)p.B * H + NTHREADS - 1) / NTHREADS)),
                     dim3(NTHREADS), 0, s, p, adpq, delta);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  const int nz = cg_point_rows(p.T);
  hipLaunchKernelGGL(cg_bwd_point_kernel<AT>, dim3((H + 63) / 64, p.B, nz), dim3(NTHREADS), 0, s, p, w, hs32, pq,
                     adpq, delta, parts);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  const RowOuts outs = {{p.g.db_a, p.g.db_x, p.g.dLambda, p.dtheta, nullptr}};
  if ((e = launch_reduce_parts(parts, p.B * nz, 4, H, outs, s)) != hipSuccess) return e;
  float *wpart = (float *)((char *)parts + align256((size_t)p.B * nz * 4 * H * sizeof(float)));
  if (sizeof(AT) == 2 && cg_mfma_ok(p)) {
    const int nin = 2 * hs, mtile = (p.T + MT - 1) / MT;
    unsigned short *wt = (unsigned short *)((char *)wpart + cg_wgrad_part_bytes((size_t)p.B * p.T, p.nb, hs));
    const size_t nw = (size_t)p.nb * nin * nin, ldsd = (size_t)2 * MT * (nin + 8) * 2;
    hipLaunchKernelGGL(cg_wt_kernel, dim3((unsigned)((nw + NTHREADS - 1) / NTHREADS)), dim3(NTHREADS), 0, s, p, wt);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if ((e = allow_lds(cg_dgrad_mfma_kernel, ldsd)) != hipSuccess) return e;
    hipLaunchKernelGGL(cg_dgrad_mfma_kernel, dim3(p.nb, p.B, mtile), dim3(NTHREADS), ldsd, s, p, w, adpq, wt);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  } else {
    if ((e = allow_lds(cg_bwd_dgrad_kernel<AT>, lds2)) != hipSuccess) return e;
    hipLaunchKernelGGL(cg_bwd_dgrad_kernel<AT>, dim3(p.nb, p.B, ntile), dim3(NTHREADS), lds2, s, p, w, adpq);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (sizeof(AT) == 2 && cg_wgrad_mfma_ok(hs)) {
    const size_t rows = (size_t)p.B * p.T;
    const int S = cg_wgrad_slices(rows, p.nb), nin = 2 * hs;
    const int rows_per = (int)(((rows + S - 1) / S + MT - 1) / MT * MT);
    const size_t ldsw = (size_t)4 * nin * WRS * 2;
    if ((e = allow_lds(cg_wgrad_mfma_kernel, ldsw)) != hipSuccess) return e;
    hipLaunchKernelGGL(cg_wgrad_mfma_kernel, dim3(p.nb, S), dim3(512), ldsw, s, p, w, adpq, wpart, rows_per);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const size_t per = (size_t)p.nb * nin * nin;
    hipLaunchKernelGGL(cg_wgrad_reduce_kernel, dim3((unsigned)((per + NTHREADS - 1) / NTHREADS)), dim3(NTHREADS), 0, s, p,
                       wpart, S);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  } else {
    const int tj = (hs + 31) / 32, tk = (2 * hs + 31) / 32;
    hipLaunchKernelGGL(cg_bwd_wgrad_kernel, dim3(p.nb, tj, tk), dim3(NTHREADS), 0, s, p, w, adpq);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  // the Conv1D's adjoint is the real layer's: du from dx, tap and bias gradients
  Problem q = p;
  q.g.db_a = q.g.db_x = q.g.dLambda = nullptr;
  return launch_backward_generic_tail(q, sizeof(AT) == 2, s, false, false, true);
}

}  // namespace

size_t cg_backward_ws_bytes(int B, int T, int D, int nb) {   // ... + the recomputed states, the parked
                                                             // pre-activations and the partial sums of pass 1b
  const size_t n = (size_t)B * T * D * sizeof(float);
  const size_t parts = (size_t)B * cg_point_rows(T) * 4 * (D / 2) * sizeof(float);
  const int hs = D / 2 / nb;
  return backward_generic_ws_bytes(B, T, D, nb) + 2 * ((n + 255) & ~(size_t)255) + ((parts + 255) & ~(size_t)255) +
         cg_wgrad_part_bytes((size_t)B * T, nb, hs) + cg_wt_bytes(nb, hs);
}

hipError_t launch_cg_forward(const Problem &p, bool bf, hipStream_t s) {
  if (bf && cg_fused_ok(p)) return launch_cg_fused<bf16, false>(p, nullptr, nullptr, nullptr, s);
  // with the optional scratch (the real layer's layout: a 256-byte cell, the state between chunks,
  // two coefficient arrays for a chunk of steps) and more than one tile of steps: two passes
  if (p.ws && p.T > GT && ((uintptr_t)p.ws % 256) == 0 && p.ws_bytes >= forward_generic_ws_bytes(p.B, p.T, p.D)) {
    const size_t state = ((size_t)4 * p.B * p.D + 255) & ~(size_t)255;
    const size_t chunk = (p.ws_bytes - 256 - state) / 2 & ~(size_t)255;
    int tcmax = (int)(chunk / ((size_t)4 * p.B * p.D)) / CTG * CTG;
    if (tcmax > p.T) tcmax = p.T;
    if (tcmax >= CTG || tcmax == p.T) {
      float *hstate = (float *)((char *)p.ws + 256);
      float2 *A = (float2 *)((char *)p.ws + 256 + state), *Bv = (float2 *)((char *)A + chunk);
      return bf ? cg_forward_two_pass<bf16, bf16>(p, tcmax, A, Bv, hstate, s)
                : cg_forward_two_pass<float, float>(p, tcmax, A, Bv, hstate, s);
    }
  }
  const size_t lds = (size_t)(GT * 2 * p.bs + 2 * p.bs) * sizeof(float);
  hipError_t e = bf ? allow_lds(cg_forward_kernel<bf16>, lds) : allow_lds(cg_forward_kernel<float>, lds);
  if (e != hipSuccess) return e;
  const dim3 grid(p.nb, p.B);
  if (bf)
    hipLaunchKernelGGL(cg_forward_kernel<bf16>, grid, dim3(NTHREADS), lds, s, p);
  else
    hipLaunchKernelGGL(cg_forward_kernel<float>, grid, dim3(NTHREADS), lds, s, p);
  return hipGetLastError();
}

hipError_t launch_cg_decode(const Problem &p, bool bf, hipStream_t s) {
  const size_t lds = (size_t)(GT * 2 * p.bs) * sizeof(float);
  hipError_t e = bf ? allow_lds(cg_decode_kernel<bf16>, lds) : allow_lds(cg_decode_kernel<float>, lds);
  if (e != hipSuccess) return e;
  const dim3 grid(p.nb, (p.B + GT - 1) / GT);
  if (bf)
    hipLaunchKernelGGL(cg_decode_kernel<bf16>, grid, dim3(NTHREADS), lds, s, p);
  else
    hipLaunchKernelGGL(cg_decode_kernel<float>, grid, dim3(NTHREADS), lds, s, p);
  return hipGetLastError();
}

hipError_t launch_cg_backward(const Problem &p, bool bf, hipStream_t s) {
  return bf ? cg_backward_t<bf16>(p, s) : cg_backward_t<float>(p, s);
}

}  // namespace rglru
