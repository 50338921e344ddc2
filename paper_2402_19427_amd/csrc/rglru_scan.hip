// rglru_scan: eq. (4) alone as a linear scan over given decays and gated inputs
// (Section 4.2, "A custom linear scan"; the operation timed in Appendix A.3).
//
//   h_t = a_t h_{t-1} + m_t g_t,  m_t = sqrt(1 - a_t^2) (or 1),  a_t given directly or as log a_t
//
// Generic kernel: one thread per (sequence, channel) walking the time axis; any shape, fp32 or
// bf16 storage, accurate math. It carries the fp32 contract and the shapes the tiled kernel
// does not cover.
//
// Tiled kernel (bf16 storage, D % 256 == 0): the recurrence part of the forward kernel without
// its Conv1D and gate products. A workgroup (8 waves) owns 256 channels of one sequence, or one
// of G <= 16 interleaved time slices of them, and walks tiles of 32 steps. Rows of a_t and g_t
// are loaded 16 bytes per thread two tiles ahead (into registers, written to LDS one tile
// ahead), two selection MFMAs per tensor bring the wave's 32 columns into the layout where a
// lane owns 16 consecutive steps of one channel (exact: the inputs are bf16), the lane scans
// its run, the two lane halves and the time slices combine by the affine composition
// (a2, b2) o (a1, b1) = (a2 a1, a2 b1 + b2) on tagged records, and h leaves through a staging
// tile as 16-byte stores. The per-step pairs (a_t, b_t) of a tile stay in registers until the
// tile's incoming state is known, one iteration later. Traffic: 6 bytes per element.
#include "rglru_mfma.h"

#include <type_traits>

namespace rglru {
namespace {

constexpr int SCAN_THREADS = 256;

// a_t and m_t from the stored value, in fp32 with accurate library math
__device__ __forceinline__ void decay_terms(float v, unsigned flags, float &a, float &m) {
  if (flags & RGLRU_SCAN_LOG_A) {
    a = expf(v);
    m = (flags & RGLRU_SCAN_NO_INPUT_SCALE) ? 1.f : sqrtf(-expm1f(2.f * v));
  } else {
    a = v;
    m = (flags & RGLRU_SCAN_NO_INPUT_SCALE) ? 1.f : sqrtf(fmaxf(1.f - v * v, 0.f));
  }
}

template <typename AT>
__global__ void __launch_bounds__(SCAN_THREADS) scan_generic_kernel(ScanProblem p) {
  const int d = blockIdx.x * SCAN_THREADS + threadIdx.x, b = blockIdx.y;
  if (d >= p.D) return;
  float h = p.h0 ? p.h0[(size_t)b * p.D + d] : 0.f;
  const AT *a = (const AT *)p.a, *g = (const AT *)p.g;
  AT *out = (AT *)p.h;
  if (p.flags & RGLRU_SCAN_ADJOINT) {   // delta_t = g_t + a_{t+1} delta_{t+1}, backwards in time
    float s = h;                         // a_{t+1} delta_{t+1}; starts as the gradient of the final state
    for (int t = p.T - 1; t >= 0; --t) {
      const size_t o = ((size_t)b * p.T + t) * p.D + d;
      float av, mv;
      decay_terms(ldf(a, o), p.flags, av, mv);
      const float dl = ldf(g, o) + s;
      stf(out, o, dl);
      s = av * dl;
    }
    if (p.hT) p.hT[(size_t)b * p.D + d] = s;
    return;
  }
  for (int t = 0; t < p.T; ++t) {
    const size_t o = ((size_t)b * p.T + t) * p.D + d;
    float av, mv;
    decay_terms(ldf(a, o), p.flags, av, mv);
    h = fmaf(av, h, mv * ldf(g, o));
    stf(out, o, h);
  }
  if (p.hT) p.hT[(size_t)b * p.D + d] = h;
}

}  // namespace

hipError_t launch_scan_generic(const ScanProblem &p, bool bf, hipStream_t s) {
  const dim3 grid((p.D + SCAN_THREADS - 1) / SCAN_THREADS, p.B);
  KernelTimer kt("scan_generic_kernel", s);
  if (bf)
    hipLaunchKernelGGL(scan_generic_kernel<bf16>, grid, dim3(SCAN_THREADS), 0, s, p);
  else
    hipLaunchKernelGGL(scan_generic_kernel<float>, grid, dim3(SCAN_THREADS), 0, s, p);
  return hipGetLastError();
}

// ------------------------------------------------------------------------- tiled kernel
namespace {
using namespace mfma;

constexpr int SC_TILE = TT * XS * 2;                 // one [32][264] bf16 tile
constexpr int SC_BUF = 2 * SC_TILE;                  // a_t rows | g_t rows
constexpr int SC_OFF_SEL = 2 * SC_BUF;               // two buffers, then the selection operands
constexpr int SC_OFF_OT = SC_OFF_SEL + 64 * 32;      // per-wave output staging tiles
constexpr int SC_LDS = SC_OFF_OT + NWAVE * OTILE_BYTES;
constexpr int SCAN_MAX_SLICES = 16;
constexpr float LN2_F = 0.6931471805599453f;

struct ScanArgs {
  ScanProblem p;
  int G, ntile, R, ncg;   // time slices, tiles per sequence, record ring depth, channel groups
  u64 *rec;               // [unit][R][2][256] records (A then H), zeroed before launch
  int *err;
  int swizzle;
};

// a_t and b_t = m_t g_t from the stored values (fp32 copies of bf16); fast math: the results
// are rounded to bf16 on the way out
template <bool LOGA, bool SCALE>
__device__ __forceinline__ void scan_terms(float av, float gv, float &a, float &b) {
  if (LOGA) {
    a = __builtin_amdgcn_exp2f(av * LOG2E);
    if (SCALE) {
      // 1 - a^2 = -expm1(2 log a): the series where the subtraction would cancel
      const float x = 2.f * av;
      const float ser = -x * fmaf(x, fmaf(x, 1.f / 6.f, 0.5f), 1.f);
      const float m2 = x > -0.125f ? ser : fmaf(-a, a, 1.f);
      b = __builtin_amdgcn_sqrtf(fmaxf(m2, 0.f)) * gv;
    } else {
      b = gv;
    }
  } else {
    a = av;
    b = SCALE ? __builtin_amdgcn_sqrtf(fmaxf(fmaf(-av, av, 1.f), 0.f)) * gv : gv;
  }
}

// GF16: g_t is stored in IEEE half precision (the library's own intermediate of the forward in
// separate passes); its columns are moved with the f16 form of the same selection product.
// REV: the adjoint recurrence. The kernel runs in logical time tau = T-1-t: rows are read and
// written at their mirrored positions, the decay of logical step tau is a_{t+1} (one row further
// on; the first logical step has none: it reads as log a = 0, or is set to 1), and the state
// after the last step, times a_0, is the gradient of the initial state.
template <int GMAX, bool LOGA, bool SCALE, bool GF16, bool REV>
__global__ void __launch_bounds__(NTHR) __attribute__((amdgpu_waves_per_eu(2, 2)))
scan_tiled_kernel(ScanArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16x8 *sel_lds = (bf16x8 *)(smem + SC_OFF_SEL);
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  const ScanProblem &p = a.p;
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5, j = lane & 31;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  unsigned short *otile = (unsigned short *)(smem + SC_OFF_OT) + wv * (OTILE_BYTES / 2);
  const int G = GMAX == 1 ? 1 : a.G;
  int bid = blockIdx.x;
  if (GMAX > 1 && a.swizzle) {  // consecutive logical ids on one XCD (ids are dealt round-robin to 8)
    const int per = gridDim.x >> 3;
    bid = (bid & 7) * per + (bid >> 3);
  }
  const int unit = bid / G, w = bid - unit * G;
  const int b = unit / a.ncg, cg = unit - b * a.ncg;
  const int D = p.D, T = p.T;
  const int ch = wv * 32 + j, d = cg * BS + ch;

  if (tid < 64) {  // selection matrices: the wave's 32 columns of a tile into accumulator layout
    bf16x8 sel0, sel1;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      sel0[e] = (__bf16)((hf * 8 + e == j) ? 1.0f : 0.0f);
      sel1[e] = (__bf16)((hf * 8 + e + 16 == j) ? 1.0f : 0.0f);
    }
    sel_lds[lane] = sel0;
    sel_lds[64 + lane] = sel1;
  }
  typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
  f16x8 sh0, sh1;   // the same selection operands in half precision
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    sh0[e] = (_Float16)((hf * 8 + e == j) ? 1.0f : 0.0f);
    sh1[e] = (_Float16)((hf * 8 + e + 16 == j) ? 1.0f : 0.0f);
  }

  const unsigned seq_bytes = (unsigned)((size_t)T * D * 2), row_bytes = (unsigned)D * 2;
  auto rsrc = [&](const void *base) {
    return __builtin_amdgcn_make_buffer_rsrc(uniform_ptr((const unsigned short *)base + (size_t)b * T * D), 0,
                                             seq_bytes, 0x00020000);
  };
  const __amdgpu_buffer_rsrc_t a_rsrc = rsrc(p.a), g_rsrc = rsrc(p.g), h_rsrc = rsrc(p.h);

  // rows lr and lr + 16 of a tile, 16 bytes (8 channels) per thread; rows past the end of the
  // sequence get an out-of-range offset and read as zero (no branch around a load)
  const int lc = tid & 31, lr = tid >> 5;
  const unsigned in_voff = (unsigned)(cg * BS + 8 * lc) * 2;
  u32x4 ra[2][2], rg[2][2];   // [tile parity][row half]
  auto load_tile = [&](int t0, u32x4 (&xa)[2], u32x4 (&xg)[2]) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int row = t0 + lr + 16 * i;
      if (REV) {
        const unsigned vg = row < T ? in_voff + (unsigned)(T - 1 - row) * row_bytes : 0x80000000u;
        const unsigned va = (row >= 1 && row < T) ? in_voff + (unsigned)(T - row) * row_bytes : 0x80000000u;
        xa[i] = __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, va, 0, RGLRU_NT);
        xg[i] = __builtin_amdgcn_raw_buffer_load_b128(g_rsrc, vg, 0, RGLRU_NT);
        if (!LOGA && row == 0) xa[i] = u32x4{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};   // a = 1
        continue;
      }
      const unsigned vo = row < T ? in_voff + (unsigned)(lr + 16 * i) * row_bytes : 0x80000000u;
      xa[i] = __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, vo, (unsigned)t0 * row_bytes, RGLRU_NT);
      xg[i] = __builtin_amdgcn_raw_buffer_load_b128(g_rsrc, vo, (unsigned)t0 * row_bytes, RGLRU_NT);
    }
  };
  auto park_tile = [&](int buf, const u32x4 (&xa)[2], const u32x4 (&xg)[2]) __attribute__((always_inline)) {
    unsigned short *ta = (unsigned short *)(smem + buf * SC_BUF) + lr * XS + 8 * lc;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      *(u32x4 *)(ta + 16 * i * XS) = xa[i];
      *(u32x4 *)(ta + SC_TILE / 2 + 16 * i * XS) = xg[i];
    }
  };

  // A-operand row of this lane: accumulator register r of lane half hf must be time hf*16+r
  const int arow = ((j >> 2) & 1) * 16 + (j >> 3) * 4 + (j & 3);
  const int a_off = arow * XS + hf * 8 + (2 * wv) * 16;   // the wave's own two K-steps

  u64 *ring = GMAX > 1 ? a.rec + (size_t)unit * a.R * 2 * BS + ch : nullptr;
  float carry = p.h0 ? p.h0[(size_t)b * D + d] : 0.f;  // state after this workgroup's previous tile
  // (a workspace that still reports an expired wait of an earlier call: no waiting, NaN throughout)
  int spins = (GMAX > 1 && expired_before(a.err)) ? SPIN_LIMIT : 0;

  unsigned short *ot_mine = otile + (hf * 16) * OT + j;
  const unsigned hw_voff = (unsigned)(cg * BS + wv * 32 + (lane & 3) * 8) * 2 + (unsigned)(lane >> 2) * row_bytes;

  // The tile whose local scan is complete but whose incoming state is not known yet keeps its
  // (a_t, b_t) pairs and aggregates in registers for one iteration, while the next tile's are
  // computed into the other set: [parity of the iteration]
  int held = -1;
  float ha[2][16], hb[2][16];
  float agg[2][4];   // A and H of the lower lane half's run, A and H of the whole tile
  u64 rec[GMAX > 1 ? GMAX - 1 : 1];   // one record per lane half (A below, H above)

  auto fetch_records = [&](int t) __attribute__((always_inline)) {
#pragma unroll
    for (int s = 0; s < GMAX - 1; ++s) {
      const int k = t - (G - 1) + s;
      if (s < G - 1 && k >= 0) rec[s] = peek(ring + (size_t)(k % a.R) * 2 * BS + hf * BS);
    }
  };
  // finish tile t (register set P): carry the state across the tiles of the other slices, write h
  auto resolve = [&](int t, auto par_c) __attribute__((always_inline)) {
    constexpr int P = decltype(par_c)::value;
    float h = carry;
#pragma unroll
    for (int s = 0; s < GMAX - 1; ++s) {
      const int k = t - (G - 1) + s;
      if (s < G - 1 && k >= 0) {
        const u64 *slot = ring + (size_t)(k % a.R) * 2 * BS + hf * BS;
        const unsigned want = (unsigned)(k + 1);
        while ((unsigned)(rec[s] >> 32) != want && spins < SPIN_LIMIT) {
          ++spins;
          __builtin_amdgcn_s_sleep(1);
          rec[s] = peek(slot);
        }
        if (spins < SPIN_LIMIT) spins = 0;   // the limit is per wait; an expired wait stays expired
        const float mine = __uint_as_float((unsigned)rec[s]), other = __shfl_xor(mine, 32);
        h = fmaf(hf ? other : mine, h, hf ? mine : other);
      }
    }
    // a wait that expired: this channel's outputs are NaN from here on, visibly invalid
    if (GMAX > 1 && (spins >= SPIN_LIMIT || __shfl_xor(spins, 32) >= SPIN_LIMIT)) h = __builtin_nanf("");
    float hrun = hf ? fmaf(agg[P][0], h, agg[P][1]) : h;  // state entering this lane's run
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float h0v = fmaf(ha[P][4 * q], hrun, hb[P][4 * q]), h1v = fmaf(ha[P][4 * q + 1], h0v, hb[P][4 * q + 1]);
      const float h2v = fmaf(ha[P][4 * q + 2], h1v, hb[P][4 * q + 2]), h3v = fmaf(ha[P][4 * q + 3], h2v, hb[P][4 * q + 3]);
      hrun = h3v;
      unsigned p0, p1;
      if (REV && (p.flags & SCAN_OUT_FP16)) {   // the library's own intermediate: half precision
        typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
        const f16x2 q0 = {(_Float16)h0v, (_Float16)h1v}, q1 = {(_Float16)h2v, (_Float16)h3v};
        p0 = *(const unsigned *)&q0;
        p1 = *(const unsigned *)&q1;
      } else {
        p0 = pack_bf16(h0v, h1v);
        p1 = pack_bf16(h2v, h3v);
      }
      unsigned short *o = ot_mine + (4 * q) * OT;
      o[0] = (unsigned short)(p0 & 0xffff);
      o[OT] = (unsigned short)(p0 >> 16);
      o[2 * OT] = (unsigned short)(p1 & 0xffff);
      o[3 * OT] = (unsigned short)(p1 >> 16);
    }
    wave_lds_fence();
    // (inputs are read non-temporally, outputs written through the cache: measured best)
    if (REV) {   // rows at their mirrored positions
      const int row = t * TT + (lane >> 2);
      const unsigned cvo = (unsigned)(cg * BS + wv * 32 + (lane & 3) * 8) * 2;
      const u32x4 v0 = *(const u32x4 *)(otile + (lane >> 2) * OT + (lane & 3) * 8);
      const u32x4 v1 = *(const u32x4 *)(otile + ((lane >> 2) + 16) * OT + (lane & 3) * 8);
      if (row < T) __builtin_amdgcn_raw_buffer_store_b128(v0, h_rsrc, cvo + (unsigned)(T - 1 - row) * row_bytes, 0, 0);
      if (row + 16 < T) __builtin_amdgcn_raw_buffer_store_b128(v1, h_rsrc, cvo + (unsigned)(T - 17 - row) * row_bytes, 0, 0);
    } else {
      store_staged_tile_s<OT, 0>(otile, lane, h_rsrc, hw_voff, (unsigned)(t * TT) * row_bytes, row_bytes,
                                 T - t * TT);
    }
    wave_lds_fence();
    carry = fmaf(agg[P][2], h, agg[P][3]);
  };

  // one tile: PAR is the parity of the iteration (register sets and LDS buffer of the tile)
  auto step = [&](int tile, auto par_c) __attribute__((always_inline)) {
    constexpr int PAR = decltype(par_c)::value;
    const int t0 = tile * TT;
    // rows two tiles ahead into the register set this tile has left; records of the held tile
    // (they land while this tile is scanned)
    if (tile + 2 * G < a.ntile) load_tile((tile + 2 * G) * TT, ra[PAR], rg[PAR]);
    if (GMAX > 1 && held >= 0) fetch_records(held);
    // the wave's 32 columns of a_t and g_t into accumulator layout
    f32x16 acca, accg;
#pragma unroll
    for (int r = 0; r < 16; ++r) acca[r] = accg[r] = 0.f;
    {
      const unsigned short *ta = (const unsigned short *)(smem + PAR * SC_BUF) + a_off;
      const bf16x8 s0 = sel_lds[lane], s1 = sel_lds[64 + lane];
      acca = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(ta), s0, acca, 0, 0, 0);
      if (GF16) accg = __builtin_amdgcn_mfma_f32_32x32x16_f16(*(const f16x8 *)(ta + SC_TILE / 2), sh0, accg, 0, 0, 0);
      else accg = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(ta + SC_TILE / 2), s0, accg, 0, 0, 0);
      acca = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(ta + 16), s1, acca, 0, 0, 0);
      if (GF16) accg = __builtin_amdgcn_mfma_f32_32x32x16_f16(*(const f16x8 *)(ta + SC_TILE / 2 + 16), sh1, accg, 0, 0, 0);
      else accg = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(ta + SC_TILE / 2 + 16), s1, accg, 0, 0, 0);
    }
    // local scan of this lane's 16-step run: prun = prod a, hrun = end state from zero
    float hrun = 0.f, prun = 1.f;
    const int nvalid = T - t0 - hf * 16;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float av, bv;
      scan_terms<LOGA, SCALE>(acca[r], accg[r], av, bv);
      if (r >= nvalid) {   // steps past the end of the sequence leave the state untouched
        av = 1.f;
        bv = 0.f;
      }
      hrun = fmaf(av, hrun, bv);
      prun *= av;
      ha[PAR][r] = av;
      hb[PAR][r] = bv;
    }
    {  // combine the two lane halves: lower half = steps 0..15, upper = 16..31
      const float oA = __shfl_xor(prun, 32), oH = __shfl_xor(hrun, 32);
      agg[PAR][0] = hf ? oA : prun;
      agg[PAR][1] = hf ? oH : hrun;
      const float A_up = hf ? prun : oA, H_up = hf ? hrun : oH;
      agg[PAR][2] = agg[PAR][0] * A_up;
      agg[PAR][3] = fmaf(A_up, agg[PAR][1], H_up);
    }
    if (GMAX > 1) {
      // the other slices wait for this aggregate, not for the outputs: publish first, then
      // finish the tile parked one iteration ago
      publish(ring + (size_t)(tile % a.R) * 2 * BS + hf * BS, hf ? agg[PAR][3] : agg[PAR][2], (unsigned)(tile + 1));
      if (held >= 0) resolve(held, std::integral_constant<int, PAR ^ 1>{});
      held = tile;
    } else {
      resolve(tile, par_c);
    }
    // rows of the next tile (requested one iteration ago) into the other LDS buffer
    if (tile + G < a.ntile) park_tile(PAR ^ 1, ra[PAR ^ 1], rg[PAR ^ 1]);
    __syncthreads();
  };

  int tile = w;
  if (tile < a.ntile) load_tile(tile * TT, ra[0], rg[0]);
  if (tile + G < a.ntile) load_tile((tile + G) * TT, ra[1], rg[1]);
  if (tile < a.ntile) park_tile(0, ra[0], rg[0]);
  __syncthreads();
  int last_par = 0;
  for (; tile < a.ntile; tile += 2 * G) {
    step(tile, std::integral_constant<int, 0>{});
    last_par = 0;
    if (tile + G < a.ntile) {
      step(tile + G, std::integral_constant<int, 1>{});
      last_par = 1;
    }
  }
  if (GMAX > 1 && held >= 0) {
    fetch_records(held);
    if (last_par) resolve(held, std::integral_constant<int, 1>{});
    else resolve(held, std::integral_constant<int, 0>{});
    if (spins >= SPIN_LIMIT) mark_expired(a.err);
  }
  // the workgroup that ran the last tile owns the final state
  if ((a.ntile - 1) % G == w && p.hT && hf == 0) {
    float fin = carry;
    if (REV) {   // times a_0: the gradient reaching the state before the first step
      const float v0 = bf_lo((unsigned)((const unsigned short *)p.a)[(size_t)b * T * D + d]);
      fin *= LOGA ? __builtin_amdgcn_exp2f(v0 * LOG2E) : v0;
    }
    p.hT[(size_t)b * D + d] = fin;
  }
}

template <int GMAX, bool LOGA, bool SCALE, bool GF16 = false, bool REV = false>
hipError_t launch_scan_t(const ScanArgs &a, int grid, hipStream_t s) {
  static bool configured = false;  // the kernel asks for more than the default LDS limit
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void *)scan_tiled_kernel<GMAX, LOGA, SCALE, GF16, REV>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, SC_LDS);
    if (e != hipSuccess) return e;
    configured = true;
  }
  KernelTimer kt("scan_tiled_kernel", s);
  hipLaunchKernelGGL((scan_tiled_kernel<GMAX, LOGA, SCALE, GF16, REV>), dim3(grid), dim3(NTHR), SC_LDS, s, a);
  return hipGetLastError();
}

template <int GMAX>
hipError_t launch_scan_flags(const ScanArgs &a, int grid, hipStream_t s) {
  const bool loga = a.p.flags & RGLRU_SCAN_LOG_A, scale = !(a.p.flags & RGLRU_SCAN_NO_INPUT_SCALE);
  if (a.p.flags & SCAN_G_FP16)   // internal use: the log-decay form without the input scale only
    return (a.p.flags & RGLRU_SCAN_ADJOINT) ? launch_scan_t<GMAX, true, false, true, true>(a, grid, s)
                                            : launch_scan_t<GMAX, true, false, true>(a, grid, s);
  if (a.p.flags & RGLRU_SCAN_ADJOINT)   // (always without the input scale)
    return loga ? launch_scan_t<GMAX, true, false, false, true>(a, grid, s)
                : launch_scan_t<GMAX, false, false, false, true>(a, grid, s);
  if (loga) return scale ? launch_scan_t<GMAX, true, true>(a, grid, s) : launch_scan_t<GMAX, true, false>(a, grid, s);
  return scale ? launch_scan_t<GMAX, false, true>(a, grid, s) : launch_scan_t<GMAX, false, false>(a, grid, s);
}

}  // namespace

bool scan_tiled_supported(const ScanProblem &p, bool bf) {
  const uintptr_t all = (uintptr_t)p.a | (uintptr_t)p.g | (uintptr_t)p.h;
  return bf && p.T >= 1 && p.D % BS == 0 && all % 16 == 0 && (size_t)p.T * p.D * 2 < ((size_t)1 << 31);
}

// Workspace: one record ring per unit when the sequences are sliced in time. Sized for the
// worst case of 256 compute units so that it does not depend on the device.
size_t scan_tiled_ws_bytes(int B, int T, int D) {
  const int units = B * (D / BS), ntile = (T + TT - 1) / TT;
  const int G = pick_slices(units, ntile, 256, SCAN_MAX_SLICES);
  if (G == 1) return 0;
  return 256 + (size_t)units * 8 * G * 2 * BS * sizeof(u64);
}

hipError_t launch_scan_tiled(const ScanProblem &p, hipStream_t s) {
  ScanArgs a;
  a.p = p;
  a.ncg = p.D / BS;
  const int units = p.B * a.ncg;
  a.ntile = (p.T + TT - 1) / TT;
  int ncu = num_cu();
  if (ncu > 256) ncu = 256;  // the workspace is sized for at most 256 resident workgroups
  a.G = pick_slices(units, a.ntile, ncu, SCAN_MAX_SLICES);
  a.R = 8 * a.G;
  const int grid = units * a.G;
  a.swizzle = (a.G > 1 && grid % 8 == 0) ? 1 : 0;
  if (a.G == 1) {
    a.rec = nullptr;
    a.err = nullptr;
    if (p.ws && p.ws_bytes >= 256) {   // workspace sized for a larger device: clear its status word
      hipError_t e = launch_prep(p.ws, 256, s);
      if (e != hipSuccess) return e;
    }
    return launch_scan_flags<1>(a, grid, s);
  }
  a.err = (int *)p.ws;
  a.rec = (u64 *)((char *)p.ws + 256);
  hipError_t e = launch_prep(p.ws, 256 + (size_t)units * a.R * 2 * BS * sizeof(u64), s, true);
  if (e != hipSuccess) return e;
  return launch_scan_flags<16>(a, grid, s);
}

}  // namespace rglru
