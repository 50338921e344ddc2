// Fused forward for bf16 storage and gate blocks of 256 channels (gfx950).
//
// One workgroup of 8 waves owns one (sequence, gate block) pair - or one of G interleaved
// time slices of it - and walks it in tiles of 32 steps:
//   Conv1D (Section 2.3) in fp32 -> bf16 tile in LDS
//   gate pre-activations W_a x, W_x x (eqs. 1-2) with v_mfma_f32_32x32x16_bf16; each wave keeps
//     its 32 output channels of both gate matrices in registers for the whole kernel
//   gates, a_t, sqrt(1-a_t^2) (eqs. 1-3, Appendix A) and the scan (eq. 4) in registers: every
//     lane runs 16 consecutive steps of one channel, the two lane halves are combined with
//     the affine composition (a2,b2)o(a1,b1) = (a2 a1, a2 b1 + b2)
//   carries between the time slices of one sequence travel through 8-byte records in global
//     memory (value + tag in one atomic word): each tile first publishes its own aggregate,
//     then looks back over its predecessors until it meets an inclusive state.
//
// Scaling trick: the Conv1D taps are multiplied by log2(e), so the MFMA delivers
// log2(e)*(Wx+b) and v_exp_f32 (a base-2 exponential) needs no extra multiply; the input gate
// is evaluated as ln(2)*sigmoid, which cancels the factor carried by x.
#include "rglru_internal.h"

namespace rglru {

namespace {

constexpr int BS = 256;          // gate block size this kernel is built for
constexpr int NWAVE = 8;         // waves per workgroup, 32 output channels each
constexpr int NTHR = NWAVE * 64;
constexpr int TT = 32;           // time steps per tile
constexpr int XS = BS + 8;       // LDS row stride in bf16 elements (528 B: conflict-free b128 reads)
constexpr float LOG2E = 1.4426950408889634f;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned long long u64;

constexpr unsigned TAG_AGG = 1, TAG_INCL = 2;
constexpr int SPIN_LIMIT = 1 << 22;

struct FwdArgs {
  Problem p;
  int G;         // time slices (workgroups) per (sequence, block)
  int ntile;     // tiles per sequence
  int R;         // record ring depth per unit (multiple of G)
  u64 *rec;      // [unit][R][2][256] records (A then H), zeroed before launch; NULL if G == 1
  int *err;      // set to 1 if a bounded wait expired
  int swizzle;   // remap block ids so that neighbouring time slices share an XCD
};

__device__ __forceinline__ float bf_lo(unsigned v) { return __uint_as_float(v << 16); }
__device__ __forceinline__ float bf_hi(unsigned v) { return __uint_as_float(v & 0xffff0000u); }
__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
  return (unsigned)f32_to_bf16_bits(lo) | ((unsigned)f32_to_bf16_bits(hi) << 16);
}

__device__ __forceinline__ u64 make_rec(float v, unsigned tag) {
  return ((u64)tag << 32) | (u64)__float_as_uint(v);
}
__device__ __forceinline__ void publish(u64 *slot, float v, unsigned tag) {
  __hip_atomic_store(slot, make_rec(v, tag), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ u64 peek(const u64 *slot) {
  return __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// eqs. (1)-(3) with base-2 exponentials; pp, qq, xx carry a factor log2(e).
// Returns a_t and b_t = sqrt(1-a_t^2) * i_t * x_t.
__device__ __forceinline__ void gate_fast(float pp, float qq, float xx, float kd, float &a,
                                          float &b) {
  const float ep = __builtin_amdgcn_exp2f(-pp);
  const float r = __builtin_amdgcn_rcpf(1.f + ep);
  a = __builtin_amdgcn_exp2f(kd * r);
  const float m = __builtin_amdgcn_sqrtf(fmaf(-a, a, 1.f));
  const float eq = __builtin_amdgcn_exp2f(-qq);
  const float il = __builtin_amdgcn_rcpf(fmaf(eq, LOG2E, LOG2E));  // ln2 * sigmoid(q)
  b = (m * il) * xx;
}

__global__ void __launch_bounds__(256) zero_words_kernel(u64 *p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256)
    p[i] = 0;
}

template <bool MULTI>
__global__ void __launch_bounds__(NTHR) __attribute__((amdgpu_waves_per_eu(2, 2)))
fwd_mfma_kernel(FwdArgs a) {
  __shared__ __attribute__((aligned(16))) unsigned short xs[2][TT * XS];
  const Problem &p = a.p;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, hf = lane >> 5, j = lane & 31;

  int bid = blockIdx.x;
  if (a.swizzle) {  // consecutive logical ids on the same XCD (ids are dealt round-robin to 8)
    const int per = gridDim.x >> 3;
    bid = (bid & 7) * per + (bid >> 3);
  }
  const int unit = bid / a.G, w = bid - unit * a.G;
  const int b = unit / p.nb, g = unit - b * p.nb;
  const int D = p.D, T = p.T;
  const int ch = wv * 32 + j;            // channel inside the block owned by this lane
  const int d = g * BS + ch;

  // ---- gate weights of this wave's 32 output channels, resident in registers
  bf16x8 wa[16], wx[16];
  {
    const bf16x8 *pa = (const bf16x8 *)((const unsigned short *)p.W_a + ((size_t)g * BS + ch) * BS + hf * 8);
    const bf16x8 *px = (const bf16x8 *)((const unsigned short *)p.W_x + ((size_t)g * BS + ch) * BS + hf * 8);
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) {
      wa[ks] = pa[ks * 2];
      wx[ks] = px[ks * 2];
    }
  }
  // selection matrices that copy this wave's 32 columns of the tile into accumulator layout
  bf16x8 sel0, sel1;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    sel0[e] = (__bf16)((hf * 8 + e == j) ? 1.0f : 0.0f);
    sel1[e] = (__bf16)((hf * 8 + e + 16 == j) ? 1.0f : 0.0f);
  }
  const float bias_p = p.b_a[d] * LOG2E, bias_q = p.b_x[d] * LOG2E;
  float kd;  // -c * softplus(-Lambda) * log2(e)
  {
    const float z = -p.Lambda[d];
    const float sp = z > 0.f ? z + log1pf(expf(-z)) : log1pf(expf(z));
    kd = -p.c * sp * LOG2E;
  }

  // ---- Conv1D assignment: channel pair c2, rows 8*rg .. 8*rg+7 of the tile
  const int c2 = tid & 127, rg = tid >> 7;
  const int dc = g * BS + 2 * c2;
  float cw[4][2], cb[2];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    cw[k][0] = p.conv_w[(size_t)k * D + dc] * LOG2E;
    cw[k][1] = p.conv_w[(size_t)k * D + dc + 1] * LOG2E;
  }
  cb[0] = p.conv_b ? p.conv_b[dc] * LOG2E : 0.f;
  cb[1] = p.conv_b ? p.conv_b[dc + 1] * LOG2E : 0.f;
  const unsigned *u32 = (const unsigned *)((const unsigned short *)p.u + (size_t)b * T * D + dc);
  const unsigned *st32 =
      p.state_in ? (const unsigned *)((const unsigned short *)p.state_in + (size_t)b * 3 * D + dc) : nullptr;

  auto conv_tile = [&](int t0, int buf) {
    // inputs t0+8rg-3 .. t0+8rg+7 of the channel pair
    unsigned raw[11];
#pragma unroll
    for (int n = 0; n < 11; ++n) {
      const int t = t0 + 8 * rg - 3 + n;
      unsigned v = 0;
      if (t >= 0) {
        if (t < T) v = u32[(size_t)t * (D / 2)];
      } else if (st32) {
        v = st32[(size_t)ring_slot(p.pos0 + t) * (D / 2)];
      }
      raw[n] = v;
    }
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      float x0 = cb[0], x1 = cb[1];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        x0 = fmaf(cw[k][0], bf_lo(raw[r + 3 - k]), x0);
        x1 = fmaf(cw[k][1], bf_hi(raw[r + 3 - k]), x1);
      }
      const int t = t0 + 8 * rg + r;
      const unsigned packed = t < T ? pack_bf16(x0, x1) : 0u;
      *(unsigned *)&xs[buf][(8 * rg + r) * XS + 2 * c2] = packed;
    }
  };

  // A-operand row of this lane: accumulator register r of lane half hf must be time hf*16+r
  const int arow = ((j >> 2) & 1) * 16 + (j >> 3) * 4 + (j & 3);

  float carry = (!MULTI && p.h0) ? p.h0[(size_t)b * D + d] : 0.f;  // state entering the next tile
  unsigned short *yb = (unsigned short *)p.y + (size_t)b * T * D + d;

  int tile = w;
  if (tile < a.ntile) conv_tile(tile * TT, 0);
  __syncthreads();

  for (int it = 0; tile < a.ntile; tile += a.G, ++it) {
    const int buf = it & 1, t0 = tile * TT;
    // ---- gate pre-activations on the matrix cores
    f32x16 accp, accq, accx;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      accp[r] = bias_p;
      accq[r] = bias_q;
      accx[r] = 0.f;
    }
    const unsigned short *arow_ptr = &xs[buf][arow * XS + hf * 8];
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) {
      const bf16x8 av = *(const bf16x8 *)(arow_ptr + ks * 16);
      accp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, wa[ks], accp, 0, 0, 0);
      accq = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, wx[ks], accq, 0, 0, 0);
    }
    {
      const bf16x8 a0 = *(const bf16x8 *)(arow_ptr + (2 * wv) * 16);
      const bf16x8 a1 = *(const bf16x8 *)(arow_ptr + (2 * wv + 1) * 16);
      accx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, sel0, accx, 0, 0, 0);
      accx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, sel1, accx, 0, 0, 0);
    }

    // ---- gates and the 16-step scan of this lane (zero incoming state)
    const int nvalid = min(TT, T - t0) - hf * 16;  // valid steps of this lane's run (may be <= 0)
    float hl[16], pr[16];
    float hrun = 0.f, prun = 1.f;
    if (T - t0 >= TT) {  // full tile (uniform over the workgroup)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float av, bv;
        gate_fast(accp[r], accq[r], accx[r], kd, av, bv);
        hrun = fmaf(av, hrun, bv);
        prun *= av;
        hl[r] = hrun;
        pr[r] = prun;
      }
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float av, bv;
        gate_fast(accp[r], accq[r], accx[r], kd, av, bv);
        if (r >= nvalid) {  // steps past the end of the sequence leave the state untouched
          av = 1.f;
          bv = 0.f;
        }
        hrun = fmaf(av, hrun, bv);
        prun *= av;
        hl[r] = hrun;
        pr[r] = prun;
      }
    }
    // ---- combine the two lane halves: lower half = steps 0..15, upper = 16..31
    const float oA = __shfl_xor(prun, 32), oH = __shfl_xor(hrun, 32);
    const float A_lo = hf ? oA : prun, H_lo = hf ? oH : hrun;
    const float A_up = hf ? prun : oA, H_up = hf ? hrun : oH;
    const float A_tile = A_lo * A_up, H_tile = fmaf(A_up, H_lo, H_up);

    float h_in;
    if (MULTI) {
      u64 *ring = a.rec + (size_t)unit * a.R * 2 * BS;
      u64 *mine = ring + (size_t)(tile % a.R) * 2 * BS;
      const unsigned tagbase = (unsigned)(tile + 1) << 2;
      // publish the aggregate: lower half writes A, upper half writes H
      publish(mine + hf * BS + ch, hf ? H_tile : A_tile, tagbase | TAG_AGG);
      // look back
      float accA = 1.f, accH = 0.f;
      int k = tile - 1;
      int spins = 0;
      bool found = false;
      while (k >= 0 && !found) {
        const u64 *slot = ring + (size_t)(k % a.R) * 2 * BS;
        const unsigned want = (unsigned)(k + 1) << 2;
        u64 rh = peek(slot + BS + ch);
        while (((unsigned)(rh >> 32) & ~3u) != want) {
          if (++spins > SPIN_LIMIT) break;
          __builtin_amdgcn_s_sleep(2);
          rh = peek(slot + BS + ch);
        }
        if (spins > SPIN_LIMIT) break;
        const float hv = __uint_as_float((unsigned)rh);
        if (((unsigned)(rh >> 32) & 3u) == TAG_INCL) {
          accH = fmaf(accA, hv, accH);
          found = true;
        } else {
          u64 ra = peek(slot + ch);
          while (((unsigned)(ra >> 32) & ~3u) != want) {
            if (++spins > SPIN_LIMIT) break;
            __builtin_amdgcn_s_sleep(2);
            ra = peek(slot + ch);
          }
          if (spins > SPIN_LIMIT) break;
          accH = fmaf(accA, hv, accH);
          accA *= __uint_as_float((unsigned)ra);
          --k;
        }
      }
      if (spins > SPIN_LIMIT) *a.err = 1;
      if (!found) {  // reached the start of the sequence
        const float h0v = p.h0 ? p.h0[(size_t)b * D + d] : 0.f;
        accH = fmaf(accA, h0v, accH);
      }
      h_in = accH;
      const float h_end = fmaf(A_tile, h_in, H_tile);
      if (hf) publish(mine + BS + ch, h_end, tagbase | TAG_INCL);
      carry = h_end;
    } else {
      h_in = carry;
      carry = fmaf(A_tile, h_in, H_tile);
    }

    // ---- outputs: y_t = local state + (product of a up to t) * state entering the run
    const float hin_seg = hf ? fmaf(A_lo, h_in, H_lo) : h_in;
    unsigned short *yrow = yb + (size_t)(t0 + hf * 16) * D;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      if (r < nvalid) yrow[(size_t)r * D] = f32_to_bf16_bits(fmaf(pr[r], hin_seg, hl[r]));
    }

    // ---- next tile of this workgroup into the other LDS buffer
    const int next = tile + a.G;
    if (next < a.ntile) conv_tile(next * TT, buf ^ 1);
    __syncthreads();
  }

  // the workgroup that ran the last tile owns the final state
  if (p.hT && (a.ntile - 1) % a.G == w && hf == 0) p.hT[(size_t)b * D + d] = carry;
}

}  // namespace

// ------------------------------------------------------------------------------ host side
static int g_num_cu = 0;

static int num_cu() {
  if (g_num_cu == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
      g_num_cu = n;
    else
      g_num_cu = 256;
  }
  return g_num_cu;
}

bool forward_mfma_supported(const Problem &p, bool bf) {
  return bf && p.bs == BS && p.T >= 1 && ((uintptr_t)p.W_a % 16 == 0) &&
         ((uintptr_t)p.W_x % 16 == 0) && ((uintptr_t)p.u % 4 == 0) &&
         (!p.state_in || (uintptr_t)p.state_in % 4 == 0);
}

// time slices per (sequence, block): as many as keep every workgroup resident at once
static int pick_slices(int units, int ntile, int ncu) {
  int G = ncu / units;
  if (G < 1) G = 1;
  if (G > ntile) G = ntile;
  if (G > 32) G = 32;
  return G;
}

// Workspace: one record ring per unit when the sequence is sliced in time. Sized for the
// worst case of 256 compute units so that it does not depend on the device.
size_t forward_mfma_ws_bytes(int B, int T, int D, int nb) {
  const int units = B * nb, ntile = (T + TT - 1) / TT;
  const int G = pick_slices(units, ntile, 256);
  if (G == 1) return 0;
  const size_t R = 4 * (size_t)G;
  return 256 + (size_t)units * R * 2 * BS * sizeof(u64);
}

hipError_t launch_forward_mfma(const Problem &p, hipStream_t s) {
  FwdArgs a;
  a.p = p;
  const int units = p.B * p.nb;
  a.ntile = (p.T + TT - 1) / TT;
  int ncu = num_cu();
  if (ncu > 256) ncu = 256;  // the workspace is sized for at most 256 resident workgroups
  a.G = pick_slices(units, a.ntile, ncu);
  a.R = 4 * a.G;
  const int grid = units * a.G;
  a.swizzle = (a.G > 1 && grid % 8 == 0) ? 1 : 0;
  if (a.G == 1) {
    a.rec = nullptr;
    a.err = nullptr;
    hipLaunchKernelGGL(fwd_mfma_kernel<false>, dim3(grid), dim3(NTHR), 0, s, a);
    return hipGetLastError();
  }
  a.err = (int *)p.ws;
  a.rec = (u64 *)((char *)p.ws + 256);
  const size_t nwords = 32 + (size_t)units * a.R * 2 * BS;
  hipLaunchKernelGGL(zero_words_kernel, dim3(256), dim3(256), 0, s, (u64 *)p.ws, nwords);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(fwd_mfma_kernel<true>, dim3(grid), dim3(NTHR), 0, s, a);
  return hipGetLastError();
}

}  // namespace rglru
