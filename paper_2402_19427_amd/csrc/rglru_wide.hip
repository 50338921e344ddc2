// Forward for the gate block sizes the fused kernel does not take (bf16 storage, any multiple of
// 16 channels: Section 4.1's 16 blocks give 352 and 512 channels at widths 5632 and 8192), as
// three passes over kernels that exist plus one that is new here:
//   1. Conv1D (Section 2.3) into x in the workspace, as bf16 (operand of the gate products) and
//      in half precision (the x_t of i_t x_t: bf16 is too coarse there)   conv_rows_kernel
//   2. gates_wide_kernel: the gate products of eqs. (1)-(2) on the matrix cores over the whole
//      K = bs of a block in chunks of 256 input channels, then eqs. (1)-(3) per element; it
//      writes log a_t (bf16) and b_t = sqrt(1 - a_t^2) i_t x_t (half precision) to the workspace
//   3. eq. (4) as a linear scan over (log a_t, b_t)                the scan-only kernels
// and the Conv1D ring update. About 20 bytes per element through memory instead of the fused
// kernel's 4, and the gate weights come from L2 for every 64 rows; the generic kernels these
// shapes ran on before are ~30 times slower.
#include "rglru_gelu.h"
#include "rglru_mfma.h"

#include <math.h>

namespace rglru {
using namespace mfma;

namespace {

constexpr int WM = 64;                       // rows (sequence, step) per workgroup: two MFMA row tiles
constexpr int W_XT = WM * XS;                // one [64][264] bf16 tile, in elements
constexpr int W_OFF_SEL = 2 * W_XT * 2;      // two buffers
constexpr int W_OFF_OT = W_OFF_SEL + 64 * 32;
// per wave and gate: 4 K-steps (128 bytes) of the wave's 32 weight rows, turned into MFMA fragment
// order through LDS; the row stride keeps 16-byte reads down a column free of bank conflicts
constexpr int W_WROW = 128 + 16;
constexpr int W_WPH = 32 * W_WROW;
constexpr int W_OFF_W = W_OFF_OT + NWAVE * OTILE_BYTES;
constexpr int W_LDS = W_OFF_W + NWAVE * 2 * W_WPH;
constexpr unsigned OOB = 0x80000000u;        // buffer offset past every range

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

struct WideArgs {
  Problem p;
  const unsigned short *x;     // [M][D] Conv1D output in half precision: operand of the gate products and
                               // the x_t of i_t x_t (bf16 is too coarse for that term)
  const unsigned short *xh;    // unused
  unsigned short *la, *gb;     // [M][D] log a_t (bf16), b_t (half precision)
  unsigned short *rv;          // backward only: [M][D] the recurrence gate r_t (half precision)
  int nob;                     // groups of 256 output channels per block
  int nkc;                     // chunks of 256 input channels (K) per block
  int kdim;                    // input channels per block: bs, or 2 bs for the dgrad product
  unsigned x_row_bytes;        // bytes of a row of x
  float *dx;                   // dgrad: [M][D] fp32, accumulated into
  size_t w_block_elems;        // elements between the weight rows of consecutive blocks
  float *dWa, *dWx;            // wgrad: [nb][bs][bs] fp32, written
  unsigned M;                  // B * T
  unsigned ntiles;             // row tiles a workgroup column walks (persistent workgroups)
};
constexpr int MODE_FWD = 0, MODE_BWD = 1, MODE_DGRAD = 2, MODE_WGRAD = 3;

// MODE_BWD: for the backward in passes the second result is the input gate i_t itself (half
// precision) instead of b_t, plus r_t, and x_t is not needed here.
// MODE_DGRAD: the same product machinery as the plain matrix pass dx += [dp | dq] [W_a | W_x]^T:
// "x" holds dp and dq of a block side by side (K = 2 bs, half precision), the weights are the
// transposed gate matrices side by side (converted to half precision), one accumulator on the
// f16 form of the MFMA, and the result is added to the fp32 dx.
// MODE_WGRAD: dW[j][k] = sum over (sequence, step) of dp[.][j] x[.][k] with the roles turned: the
// rows of "x" are the channels k of a block (x transposed, half precision, K = B T), the "weights"
// are dp and dq transposed (rows j), the products run on the f16 form of the MFMA (x in bf16 is
// too coarse for the weight gradients), and the accumulators are dW_a and dW_x themselves.
template <int MODE>
__global__ void __launch_bounds__(NTHR) __attribute__((amdgpu_waves_per_eu(2, 2)))
gates_wide_kernel(WideArgs a) {
  constexpr bool BWD = MODE == MODE_BWD, WG = MODE == MODE_WGRAD;
  constexpr bool DG = MODE == MODE_DGRAD;          // one product, no parameters
  constexpr bool NOPAR = DG || WG;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned short *xs = (unsigned short *)smem;                     // [2][WM][XS]
  const Problem &p = a.p;
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5, j = lane & 31;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  unsigned short *otile = (unsigned short *)(smem + W_OFF_OT) + wv * (OTILE_BYTES / 2);
  const int D = p.D, bs = p.bs;
  const int g = blockIdx.y / a.nob, ob = blockIdx.y - g * a.nob;
  // (wgrad: the row tiles lie inside block g's rows of the transposed x)
  const unsigned m_base = WG ? (unsigned)(g * bs) : 0u;
  const unsigned m_end = WG ? (unsigned)(g * bs + bs) : a.M;
  unsigned m0 = m_base + blockIdx.x * WM;   // first row of the tile in hand
  const unsigned row_bytes = (unsigned)D * 2, xrow = a.x_row_bytes;
  const int kdim = a.kdim;

  // this lane's output channel; a channel past the block is computed from an existing one's
  // parameters and never stored
  const int och = ob * BS + wv * 32 + j;
  const int ochc = och < bs ? och : bs - 1;
  const int d = g * bs + ochc;
  const float bias_p = NOPAR ? 0.f : p.b_a[d], bias_q = NOPAR ? 0.f : p.b_x[d];
  float kdn = 0.f;  // -c * softplus(-Lambda) = log of the fully open decay, eq. (3)
  if (!NOPAR) {
    const float z = -p.Lambda[d];
    const float sp = z > 0.f ? z + log1pf(expf(-z)) : log1pf(expf(z));
    kdn = -p.c * sp;
  }
  // ---- gate weights: a fragment read straight from the row-major matrix touches 32 cache lines
  // per instruction; instead the wave reads whole 128-byte lines of its 32 rows (8 lanes per
  // row, 4 K-steps of both gates per phase) and turns them into fragment order through its own
  // LDS buffers. Rows and columns past the block are read from existing ones (they end in
  // outputs that are dropped, or meet zeros in x).
  const unsigned char *wbase_a = (const unsigned char *)p.W_a + (size_t)g * a.w_block_elems * 2;
  const unsigned char *wbase_x = (const unsigned char *)p.W_x + (size_t)g * a.w_block_elems * 2;
  unsigned w_row[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = ob * BS + wv * 32 + i * 8 + (lane >> 3);
    w_row[i] = (unsigned)(r < bs ? r : bs - 1) * (unsigned)(kdim * 2);
  }
  unsigned char *wl = smem + W_OFF_W + wv * 2 * W_WPH;
  const unsigned wl_wr = (unsigned)(lane >> 3) * W_WROW + (unsigned)(lane & 7) * 16;
  const unsigned wl_rd = (unsigned)j * W_WROW + (unsigned)hf * 16;
  u32x4 stg[2][8];
  auto load_phase = [&](int P, u32x4 (&dst)[8]) __attribute__((always_inline)) {   // phase P: K-steps 4P .. 4P+3 of the block
    const int c = P * 8 + (lane & 7);   // 16-byte chunk of the row
    const unsigned w_col = (unsigned)(c < (kdim >> 3) ? c : (kdim >> 3) - 1) * 16;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      dst[i] = *(const u32x4 *)(wbase_a + w_row[i] + w_col);
      if (!DG) dst[4 + i] = *(const u32x4 *)(wbase_x + w_row[i] + w_col);
    }
  };
  auto write_phase = [&](const u32x4 (&src)[8]) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      *(u32x4 *)(wl + i * 8 * W_WROW + wl_wr) = src[i];
      if (!DG) *(u32x4 *)(wl + W_WPH + i * 8 * W_WROW + wl_wr) = src[4 + i];
    }
  };

  // ---- x tile loader: thread -> 16 bytes (8 channels) of rows r0, r0 + 16, r0 + 32, r0 + 48
  const __amdgpu_buffer_rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      uniform_ptr(a.x), 0, (WG ? (unsigned)p.D : a.M) * xrow, 0x00020000);
  const int lc = tid & 31, r0 = tid >> 5;
  u32x4 nx[4];
  auto load_chunk = [&](unsigned mt, int kc) __attribute__((always_inline)) {   // chunk kc of the input channels, tile at row mt
    const int col = kc * BS + lc * 8;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const unsigned m = mt + r0 + 16 * i;
      const bool ok = m < m_end && col < kdim;   // (kc past the last chunk: col >= kdim)
      nx[i] = __builtin_amdgcn_raw_buffer_load_b128(
          x_rsrc, ok ? m * xrow + (unsigned)((WG ? 0 : g * kdim) + col) * 2 : OOB, 0, 0);
    }
  };
  auto park_chunk = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 4; ++i) *(u32x4 *)(xs + buf * W_XT + (r0 + 16 * i) * XS + lc * 8) = nx[i];
  };

  const int arow = ((j >> 2) & 1) * 16 + (j >> 3) * 4 + (j & 3);   // row of this lane's A operand
  // ---- persistent over row tiles: the weights of this workgroup are the same for every tile, so
  // their phase pipeline simply wraps around, and the first chunk of the next tile is requested
  // during the last chunk of this one - loads, products and epilogue of consecutive tiles overlap
  // instead of forming one dependent chain per workgroup
  const int nph = a.nkc * 4;
  int bufp = 0;   // LDS buffer that holds the chunk to be multiplied next
  load_phase(0, stg[0]);
  load_phase(1 % nph, stg[1]);
  load_chunk(m0, 0);
  park_chunk(0);
  write_phase(stg[0]);
  __syncthreads();

  for (unsigned tile = blockIdx.x; tile < a.ntiles; tile += gridDim.x) {
  m0 = m_base + tile * WM;
  const unsigned m0_next = m0 + gridDim.x * WM;   // (past the rows if this was the last tile: reads as zero)
  f32x16 accp[2], accq[2], accx[2];
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      accp[mi][r] = bias_p;
      accq[mi][r] = bias_q;
      accx[mi][r] = 0.f;
    }

  for (int kc = 0; kc < a.nkc; ++kc) {
    const int buf = bufp;
    const bool last = kc + 1 == a.nkc;
    load_chunk(last ? m0_next : m0, last ? 0 : kc + 1);   // lands during the products
    const unsigned short *ap = xs + buf * W_XT + arow * XS + hf * 8;
#pragma unroll
    for (int ph = 0; ph < 4; ++ph) {
      const int P = kc * 4 + ph;
      int P2 = P + 2;
      if (P2 >= nph) P2 -= nph;
      // two phases ahead, into the registers whose contents are in LDS already
      load_phase(P2, stg[ph & 1]);
      wave_lds_fence();   // the fragments come from other lanes of this wave
      bf16x8 fa[4], fx[4];
#pragma unroll
      for (int k2 = 0; k2 < 4; ++k2) {
        fa[k2] = *(const bf16x8 *)(wl + wl_rd + k2 * 32);
        if (!DG) fx[k2] = *(const bf16x8 *)(wl + W_WPH + wl_rd + k2 * 32);
      }
      wave_lds_fence();
      write_phase(stg[(ph + 1) & 1]);   // LDS serves a wave's accesses in order: queued behind the reads
#pragma unroll
      for (int k2 = 0; k2 < 4; ++k2) {
        const int ks = ph * 4 + k2;
        const bf16x8 a0 = *(const bf16x8 *)(ap + ks * 16), a1 = *(const bf16x8 *)(ap + 32 * XS + ks * 16);
        {   // half-precision operands in every mode
          typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
          const f16x8 h0 = __builtin_bit_cast(f16x8, a0), h1 = __builtin_bit_cast(f16x8, a1);
          const f16x8 ha = __builtin_bit_cast(f16x8, fa[k2]);
          accp[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(h0, ha, accp[0], 0, 0, 0);
          accp[1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(h1, ha, accp[1], 0, 0, 0);
          if (!DG) {
            const f16x8 hx = __builtin_bit_cast(f16x8, fx[k2]);
            accq[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(h0, hx, accq[0], 0, 0, 0);
            accq[1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(h1, hx, accq[1], 0, 0, 0);
          }
        }
      }
    }
    if (MODE == MODE_FWD && kc == ob) {   // this chunk holds the wave's own channels: x_t into accumulator layout
      typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
      f16x8 sh0, sh1;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        sh0[e] = (_Float16)((hf * 8 + e == j) ? 1.0f : 0.0f);
        sh1[e] = (_Float16)((hf * 8 + e + 16 == j) ? 1.0f : 0.0f);
      }
#pragma unroll
      for (int mi = 0; mi < 2; ++mi) {
        const unsigned short *sp = ap + mi * 32 * XS;
        accx[mi] = __builtin_amdgcn_mfma_f32_32x32x16_f16(*(const f16x8 *)(sp + (2 * wv) * 16), sh0, accx[mi], 0, 0, 0);
        accx[mi] = __builtin_amdgcn_mfma_f32_32x32x16_f16(*(const f16x8 *)(sp + (2 * wv + 1) * 16), sh1, accx[mi], 0, 0, 0);
      }
    }
    park_chunk(buf ^ 1);
    __syncthreads();
    bufp = buf ^ 1;
  }

  if (WG) {   // lane (j, hf) holds dW[och][k] for the 16 rows k = tile row 16 hf .. 16 hf + 15
    if (och < bs) {
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const unsigned m = m0 + mi * 32 + hf * 16 + r;
          if (m < m_end) {
            const size_t o = ((size_t)g * bs + och) * bs + (m - (unsigned)(g * bs));
            a.dWa[o] = accp[mi][r];
            a.dWx[o] = accq[mi][r];
          }
        }
    }
    continue;
  }
  if (DG) {   // dx += the products: lane (j, hf) holds channel och of rows 16 hf .. 16 hf + 15
    if (och < bs) {
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const unsigned m = m0 + mi * 32 + hf * 16 + r;
          if (m < a.M) a.dx[(size_t)m * D + g * bs + och] += accp[mi][r];
        }
    }
    continue;
  }
  // ---- eqs. (1)-(3) per element; the two results leave through the wave's staging tile as
  // 16-byte rows
  const __amdgpu_buffer_rsrc_t la_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      uniform_ptr(a.la), 0, a.M * row_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t gb_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      uniform_ptr(a.gb), 0, a.M * row_bytes, 0x00020000);
  const bool chunk_ok = ob * BS + wv * 32 + (lane & 3) * 8 < bs;
  const unsigned o_voff =
      chunk_ok ? (unsigned)(g * bs + ob * BS + wv * 32 + (lane & 3) * 8) * 2 + (unsigned)(lane >> 2) * row_bytes : OOB;
  unsigned short *ot_mine = otile + (hf * 16) * OT + j;
#pragma unroll
  for (int mi = 0; mi < 2; ++mi) {
    const unsigned mrow = m0 + mi * 32;
    const int nrows = (int)a.M - (int)mrow;
    float bv[16], rr[BWD ? 16 : 1];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float rg = __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-LOG2E * accp[mi][r]));
      // (the backward keeps the pre-activation, not r_t: half precision has no relative
      // accuracy left for r_t below 6e-5, a recurrence gate closed that far still decides
      // sqrt(1 - a_t^2), and the logit is as accurate as r_t everywhere else)
      if (BWD) rr[r] = fminf(fmaxf(accp[mi][r], -60000.f), 60000.f);
      const float la = kdn * rg;
      const float av = __builtin_amdgcn_exp2f(LOG2E * la);
      const float mm = __builtin_amdgcn_sqrtf(one_minus_sq(av, LOG2E * la));
      const float ig = __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-LOG2E * accq[mi][r]));
      // (the backward keeps the logit of i_t as well: 1 - i_t of an open input gate is not
      // representable next to i_t in half precision)
      bv[r] = BWD ? fminf(fmaxf(accq[mi][r], -60000.f), 60000.f) : mm * ig * accx[mi][r];
      ot_mine[r * OT] = (unsigned short)(pack_bf16(la, 0.f) & 0xffff);
    }
    store_staged_tile_s<OT, 0>(otile, lane, la_rsrc, o_voff, mrow * row_bytes, row_bytes, nrows);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const _Float16 hv = (_Float16)bv[r];
      ot_mine[r * OT] = *(const unsigned short *)&hv;
    }
    store_staged_tile_s<OT, 0>(otile, lane, gb_rsrc, o_voff, mrow * row_bytes, row_bytes, nrows);
    if (BWD) {   // r_t in half precision too: log a_t in bf16 is too coarse for the adjoints
      const __amdgpu_buffer_rsrc_t rv_rsrc = __builtin_amdgcn_make_buffer_rsrc(
          uniform_ptr(a.rv), 0, a.M * row_bytes, 0x00020000);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const _Float16 hv = (_Float16)rr[r];
        ot_mine[r * OT] = *(const unsigned short *)&hv;
      }
      store_staged_tile_s<OT, 0>(otile, lane, rv_rsrc, o_voff, mrow * row_bytes, row_bytes, nrows);
    }
  }
  }   // row tiles
}

// ------------------------------------------------------------------------------ decode
// One decode step (Section 5; states of Appendix F) for the same block sizes: a workgroup takes
// 32 sequences and 256 output channels of one gate block and walks the block's input channels
// in chunks of 256: Conv1D over the ring for the chunk into an LDS tile (high + low bf16 part,
// scaled by log2 e), then its 16 K-steps with the weights read as whole lines and turned into
// fragment order through wave-private LDS. The Conv1D inputs and taps of the next chunk are
// requested as soon as those of the current one are used up, so they land during the products.
// Every workgroup of a block reads the whole ring of the block, so the new token cannot replace
// the oldest slot in place here: a second kernel writes it once this one has finished.
constexpr int DW_OFF_W = 2 * XT_ELEMS * 2;                 // x tile (high, low) first
constexpr int DW_OFF_H = DW_OFF_W + NWAVE * 2 * W_WPH;     // per wave: h / y staging, 32 rows
constexpr int DW_MAXCH = 3;                                // chunks of input channels: blocks up to 768
constexpr int DW_OFF_CW = DW_OFF_H + NWAVE * W_WPH;        // Conv1D taps and bias: [chunk][5][256] f32
constexpr int DW_LDS = DW_OFF_CW + DW_MAXCH * 5 * BS * 4;
constexpr int DW_YROW = 64 + 16;

struct DecWideArgs {
  Problem p;   // u = u_t [B][D], hT = h [B][D] (in place), state_out = ring (read), y = y_t / out_t
  int nob;
};

template <int MERGE, bool PERSEQ = false>
__global__ void __launch_bounds__(NTHR) __attribute__((amdgpu_waves_per_eu(2, 2)))
decode_wide_kernel(DecWideArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned short *xs = (unsigned short *)smem;   // [high, low][32][XS]
  const Problem &p = a.p;
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5, j = lane & 31;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = blockIdx.x / a.nob, ob = blockIdx.x - g * a.nob, b0 = blockIdx.y * TT;
  const int D = p.D, B = p.B, bs = p.bs;
  const unsigned row2 = (unsigned)D * 2;

  const int och = ob * BS + wv * 32 + j;
  const int d = g * bs + (och < bs ? och : bs - 1);
  const float bias_p = p.b_a[d] * LOG2E, bias_q = p.b_x[d] * LOG2E, lam = p.Lambda[d];

  const __amdgpu_buffer_rsrc_t u_rsrc = __builtin_amdgcn_make_buffer_rsrc(uniform_ptr(p.u), 0, (unsigned)B * row2, 0x00020000);
  const __amdgpu_buffer_rsrc_t ring_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(uniform_ptr(p.state_out), 0, 3u * (unsigned)B * row2, 0x00020000);
  const __amdgpu_buffer_rsrc_t h_rsrc = __builtin_amdgcn_make_buffer_rsrc(uniform_ptr(p.hT), 0, 2u * (unsigned)B * row2, 0x00020000);
  const __amdgpu_buffer_rsrc_t y_rsrc = __builtin_amdgcn_make_buffer_rsrc(uniform_ptr(p.y), 0, (unsigned)B * row2, 0x00020000);

  // ---- Conv1D inputs and taps of chunk kc: 8 channels (16 bytes) of rows lr and lr + 16
  const int lc = tid & 31, lr = tid >> 5;
  const int s1 = ring_slot(p.pos0 - 1), s2 = ring_slot(p.pos0 - 2), s3 = ring_slot(p.pos0 - 3);
  u32x4 ru[2][4];
  unsigned rq[2][3] = {};
  if constexpr (PERSEQ) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int b = b0 + lr + 16 * i;
      const long long pb = p.pos_rows[b < B ? b : B - 1];
#pragma unroll
      for (int k = 0; k < 3; ++k) rq[i][k] = (unsigned)ring_slot(pb - 1 - k);
    }
  }
  // taps and bias of every chunk parked in LDS once (missing channels: zero bias, any taps -
  // their inputs read as zero), so that only the inputs are in flight during the products
  float *cw_lds = (float *)(smem + DW_OFF_CW);
  if (lr < a.nob) {
    const int col = lr * BS + lc * 8;
    const bool cok = col < bs;
    const int dcc = g * bs + (cok ? col : 0);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      *(f32x4 *)(cw_lds + (lr * 5 + k) * BS + lc * 8) = *(const f32x4 *)(p.conv_w + (size_t)k * D + dcc);
      *(f32x4 *)(cw_lds + (lr * 5 + k) * BS + lc * 8 + 4) = *(const f32x4 *)(p.conv_w + (size_t)k * D + dcc + 4);
    }
    const f32x4 z = {0.f, 0.f, 0.f, 0.f};
    const bool bon = p.conv_b && cok;
    *(f32x4 *)(cw_lds + (lr * 5 + 4) * BS + lc * 8) = bon ? *(const f32x4 *)(p.conv_b + dcc) : z;
    *(f32x4 *)(cw_lds + (lr * 5 + 4) * BS + lc * 8 + 4) = bon ? *(const f32x4 *)(p.conv_b + dcc + 4) : z;
  }
  auto load_conv = [&](int kc) __attribute__((always_inline)) {
    const int col = kc * BS + lc * 8;
    const bool cok = col < bs;                       // (also false for every chunk past the block)
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int b = b0 + lr + 16 * i;
      const bool ok = b < B && cok;
      const unsigned uvo = ok ? (unsigned)b * row2 + (unsigned)(g * bs + col) * 2 : OOB;
      const unsigned rvo = ok ? (unsigned)(b * 3) * row2 + (unsigned)(g * bs + col) * 2 : OOB;
      ru[i][0] = __builtin_amdgcn_raw_buffer_load_b128(u_rsrc, uvo, 0, 0);
      if constexpr (PERSEQ) {   // slots of this row's own position, carried in the lane offset
        ru[i][1] = __builtin_amdgcn_raw_buffer_load_b128(ring_rsrc, ok ? rvo + rq[i][0] * row2 : OOB, 0, 0);
        ru[i][2] = __builtin_amdgcn_raw_buffer_load_b128(ring_rsrc, ok ? rvo + rq[i][1] * row2 : OOB, 0, 0);
        ru[i][3] = __builtin_amdgcn_raw_buffer_load_b128(ring_rsrc, ok ? rvo + rq[i][2] * row2 : OOB, 0, 0);
      } else {
        ru[i][1] = __builtin_amdgcn_raw_buffer_load_b128(ring_rsrc, rvo, (unsigned)s1 * row2, 0);
        ru[i][2] = __builtin_amdgcn_raw_buffer_load_b128(ring_rsrc, rvo, (unsigned)s2 * row2, 0);
        ru[i][3] = __builtin_amdgcn_raw_buffer_load_b128(ring_rsrc, rvo, (unsigned)s3 * row2, 0);
      }
    }
  };
  auto conv_chunk = [&](int kc) __attribute__((always_inline)) {   // x tile of the chunk whose inputs are in ru
    f32x4 cw[4][2], cb[2];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      cw[k][0] = *(const f32x4 *)(cw_lds + (kc * 5 + k) * BS + lc * 8);
      cw[k][1] = *(const f32x4 *)(cw_lds + (kc * 5 + k) * BS + lc * 8 + 4);
    }
    cb[0] = *(const f32x4 *)(cw_lds + (kc * 5 + 4) * BS + lc * 8);
    cb[1] = *(const f32x4 *)(cw_lds + (kc * 5 + 4) * BS + lc * 8 + 4);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      u32x4 hi4, lo4;
#pragma unroll
      for (int e = 0; e < 4; ++e) {   // channels 2e, 2e+1 of the 8
        const int v = e >> 1, c0 = (2 * e) & 3;
        const unsigned u0 = ru[i][0][e], u1 = ru[i][1][e], u2 = ru[i][2][e], u3 = ru[i][3][e];
        float x0 = cb[v][c0], x1 = cb[v][c0 + 1];
        x0 = fmaf(cw[0][v][c0], bf_lo(u0), x0); x1 = fmaf(cw[0][v][c0 + 1], bf_hi(u0), x1);
        x0 = fmaf(cw[1][v][c0], bf_lo(u1), x0); x1 = fmaf(cw[1][v][c0 + 1], bf_hi(u1), x1);
        x0 = fmaf(cw[2][v][c0], bf_lo(u2), x0); x1 = fmaf(cw[2][v][c0 + 1], bf_hi(u2), x1);
        x0 = fmaf(cw[3][v][c0], bf_lo(u3), x0); x1 = fmaf(cw[3][v][c0 + 1], bf_hi(u3), x1);
        unsigned hi_pk, lo_pk;
        split_bf16(x0 * LOG2E, x1 * LOG2E, hi_pk, lo_pk);   // missing rows and channels: all inputs read as zero
        hi4[e] = hi_pk;
        lo4[e] = lo_pk;
      }
      *(u32x4 *)(xs + (lr + 16 * i) * XS + 8 * lc) = hi4;
      *(u32x4 *)(xs + XT_ELEMS + (lr + 16 * i) * XS + 8 * lc) = lo4;
    }
  };
  load_conv(0);

  // ---- gate weights, as in gates_wide_kernel
  const unsigned char *wbase_a = (const unsigned char *)p.W_a + (size_t)g * bs * bs * 2;
  const unsigned char *wbase_x = (const unsigned char *)p.W_x + (size_t)g * bs * bs * 2;
  unsigned w_row[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = ob * BS + wv * 32 + i * 8 + (lane >> 3);
    w_row[i] = (unsigned)(r < bs ? r : bs - 1) * (unsigned)(bs * 2);
  }
  unsigned char *wl = smem + DW_OFF_W + wv * 2 * W_WPH;
  const unsigned wl_wr = (unsigned)(lane >> 3) * W_WROW + (unsigned)(lane & 7) * 16;
  const unsigned wl_rd = (unsigned)j * W_WROW + (unsigned)hf * 16;
  u32x4 stg[2][8];
  auto load_phase = [&](int P, u32x4 (&dst)[8]) __attribute__((always_inline)) {
    const int c = P * 8 + (lane & 7);
    const unsigned w_col = (unsigned)(c < (bs >> 3) ? c : (bs >> 3) - 1) * 16;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      dst[i] = *(const u32x4 *)(wbase_a + w_row[i] + w_col);
      dst[4 + i] = *(const u32x4 *)(wbase_x + w_row[i] + w_col);
    }
  };
  auto write_phase = [&](const u32x4 (&src)[8]) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      *(u32x4 *)(wl + i * 8 * W_WROW + wl_wr) = src[i];
      *(u32x4 *)(wl + W_WPH + i * 8 * W_WROW + wl_wr) = src[4 + i];
    }
  };
  load_phase(0, stg[0]);

  // ---- recurrent state of this wave's 32 x 32 tile, and where its outputs go
  unsigned char *hl = smem + DW_OFF_H + wv * W_WPH;
  const unsigned hl_wide = (unsigned)(lane >> 3) * W_WROW + (unsigned)(lane & 7) * 16;
  unsigned h_vo[4];
  u32x4 hin[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int b = b0 + (lane >> 3) + 8 * i;
    const int c = ob * BS + wv * 32 + (lane & 7) * 4;
    h_vo[i] = (b < B && c < bs) ? ((unsigned)b * (unsigned)D + (unsigned)(g * bs + c)) * 4 : OOB;
    hin[i] = __builtin_amdgcn_raw_buffer_load_b128(h_rsrc, h_vo[i], 0, 0);
  }
  unsigned y_vo[2];
  u32x4 brq[2];
  const __amdgpu_buffer_rsrc_t br_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(uniform_ptr(MERGE ? p.branch : p.u), 0, (unsigned)B * row2, 0x00020000);
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int b = b0 + (lane >> 2) + 16 * i;
    const int c = ob * BS + wv * 32 + (lane & 3) * 8;
    y_vo[i] = (b < B && c < bs) ? ((unsigned)b * (unsigned)D + (unsigned)(g * bs + c)) * 2 : OOB;
    if (MERGE) brq[i] = __builtin_amdgcn_raw_buffer_load_b128(br_rsrc, y_vo[i], 0, 0);
  }
  load_phase(1, stg[1]);

  typedef bf16x8 frag_t;
  bf16x8 sel0, sel1;   // selection operands, in registers (nothing else is resident here)
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    sel0[e] = (__bf16)((hf * 8 + e == j) ? 1.0f : 0.0f);
    sel1[e] = (__bf16)((hf * 8 + e + 16 == j) ? 1.0f : 0.0f);
  }
  float kd;
  {
    const float z = -lam;
    const float sp = z > 0.f ? z + log1pf(expf(-z)) : log1pf(expf(z));
    kd = -p.c * sp * LOG2E;
  }

  const int arow = ((j >> 2) & 1) * 16 + (j >> 3) * 4 + (j & 3);
  const unsigned short *ap = xs + arow * XS + hf * 8;
  f32x16 accp, accq, accx;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    accp[r] = bias_p;
    accq[r] = bias_q;
    accx[r] = 0.f;
  }
  write_phase(stg[0]);
  float gl[2][8];
  __syncthreads();   // the taps parked in LDS are visible
  for (int kc = 0; kc < a.nob; ++kc) {
    conv_chunk(kc);
    load_conv(kc + 1);   // inputs and taps of the next chunk (nothing is read past the block)
    if (MERGE && kc == 0) {   // GeLU of the other branch while the weights are on their way
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          gl[i][2 * k] = gelu<MERGE == 2, true>(bf_lo(brq[i][k]));
          gl[i][2 * k + 1] = gelu<MERGE == 2, true>(bf_hi(brq[i][k]));
        }
    }
    __syncthreads();
#pragma unroll
    for (int ph = 0; ph < 4; ++ph) {
      const int P = kc * 4 + ph;
      load_phase(P + 2, stg[ph & 1]);
      wave_lds_fence();
      frag_t av[4], fa[4], fx[4];
#pragma unroll
      for (int k2 = 0; k2 < 4; ++k2) {
        av[k2] = *(const bf16x8 *)(ap + (ph * 4 + k2) * 16);
        fa[k2] = *(const bf16x8 *)(wl + wl_rd + k2 * 32);
        fx[k2] = *(const bf16x8 *)(wl + W_WPH + wl_rd + k2 * 32);
      }
      wave_lds_fence();
      write_phase(stg[(ph + 1) & 1]);
#pragma unroll
      for (int k2 = 0; k2 < 4; ++k2) {
        accp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[k2], fa[k2], accp, 0, 0, 0);
        accq = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[k2], fx[k2], accq, 0, 0, 0);
      }
    }
    if (kc == ob) {   // the chunk with this workgroup's own channels: x_t (high + low part)
      accx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(ap + (2 * wv) * 16), sel0, accx, 0, 0, 0);
      accx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(ap + (2 * wv + 1) * 16), sel1, accx, 0, 0, 0);
      accx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(ap + XT_ELEMS + (2 * wv) * 16), sel0, accx, 0, 0, 0);
      accx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(ap + XT_ELEMS + (2 * wv + 1) * 16), sel1, accx, 0, 0, 0);
    }
    __syncthreads();   // the x tile is free for the next chunk
  }

  // ---- h into accumulator layout: lane (j, hf) owns channel j of rows 16 hf .. 16 hf + 15
#pragma unroll
  for (int i = 0; i < 4; ++i) *(u32x4 *)(hl + i * 8 * W_WROW + hl_wide) = hin[i];
  wave_lds_fence();
  float rh[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) rh[r] = *(const float *)(hl + (hf * 16 + r) * W_WROW + j * 4);
  wave_lds_fence();

  // ---- eqs. (1)-(4) with base-2 exponentials (the pre-activations and x carry log2 e)
  unsigned char *yl = wl;   // weight buffer 0 of this wave is free again
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const float rg = __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-accp[r]));
    const float av_ = __builtin_amdgcn_exp2f(kd * rg);
    const float mm = __builtin_amdgcn_sqrtf(one_minus_sq(av_, kd * rg));
    const float eq = __builtin_amdgcn_exp2f(-accq[r]);
    const float il = __builtin_amdgcn_rcpf(fmaf(eq, LOG2E, LOG2E));   // sigmoid(q) / log2 e
    const float hn = fmaf(av_, rh[r], (mm * il) * accx[r]);
    *(float *)(hl + (hf * 16 + r) * W_WROW + j * 4) = hn;
    *(unsigned short *)(yl + (hf * 16 + r) * DW_YROW + j * 2) = (unsigned short)(pack_bf16(hn, 0.f) & 0xffff);
  }
  wave_lds_fence();
#pragma unroll
  for (int i = 0; i < 4; ++i)
    __builtin_amdgcn_raw_buffer_store_b128(*(const u32x4 *)(hl + i * 8 * W_WROW + hl_wide), h_rsrc, h_vo[i], 0, 0);
#pragma unroll
  for (int i = 0; i < 2; ++i) {   // lane l: 16 bytes of rows l/4 + 16 i
    const int row = (lane >> 2) + 16 * i;
    u32x4 yv = *(const u32x4 *)(yl + row * DW_YROW + (lane & 3) * 16);
    if (MERGE) {
#pragma unroll
      for (int k = 0; k < 4; ++k)
        yv[k] = pack_bf16(bf_lo(yv[k]) * gl[i][2 * k], bf_hi(yv[k]) * gl[i][2 * k + 1]);
    }
    __builtin_amdgcn_raw_buffer_store_b128(yv, y_rsrc, y_vo[i], 0, 0);
  }
}

// the new token into ring slot pos mod 3, 16 bytes per thread
__global__ void __launch_bounds__(256) ring_store_kernel(const uint4 *u, uint4 *ring, int B, int chunks, int slot,
                                                         const long long *pos_rows) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= B * chunks) return;
  const int b = i / chunks, c = i - b * chunks;
  if (pos_rows) slot = ring_slot(pos_rows[b]);
  ring[((size_t)b * 3 + slot) * chunks + c] = u[i];
}

inline size_t al256(size_t n) { return (n + 255) & ~(size_t)255; }

// workgroups along the row tiles: each walks a few tiles (enough to overlap their loads, products
// and epilogues), and there stay many more workgroups than CUs so that the hardware balances them
#ifndef WIDE_TILES_PER_WG
#define WIDE_TILES_PER_WG 4
#endif
inline unsigned wide_grid_x(unsigned ntiles, int gy) {
  (void)gy;
  const unsigned gx = (ntiles + WIDE_TILES_PER_WG - 1) / WIDE_TILES_PER_WG;
  return gx < 1 ? 1 : gx;
}

// ---- Conv1D (Section 2.3) as a streaming pass: a thread produces 8 channels (16 bytes) of CR
// consecutive steps from CR + 3 input rows; steps before the sequence start read the carried
// ring state (slot = position mod 3) or zero.
constexpr int CR = 8;
struct ConvArgs {
  Problem p;
  unsigned short *x;    // bf16
  unsigned short *xh;   // half precision
};
__global__ void __launch_bounds__(256) conv_rows_kernel(ConvArgs a) {
  const Problem &p = a.p;
  const int D = p.D, T = p.T, nch = D / 8, ntr = (T + CR - 1) / CR;
  const size_t total = (size_t)p.B * ntr * nch;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % nch);
  const int tr = (int)((i / nch) % ntr);
  const int b = (int)(i / ((size_t)nch * ntr));
  const int t0 = tr * CR, d0 = c * 8;
  float w[4][8], bias[8];
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int e = 0; e < 8; ++e) w[k][e] = p.conv_w ? p.conv_w[(size_t)k * D + d0 + e] : (k == 0 ? 1.f : 0.f);
#pragma unroll
  for (int e = 0; e < 8; ++e) bias[e] = p.conv_b ? p.conv_b[d0 + e] : 0.f;
  const unsigned short *u = (const unsigned short *)p.u + (size_t)b * T * D + d0;
  const unsigned short *st = p.state_in ? (const unsigned short *)p.state_in + (size_t)b * 3 * D + d0 : nullptr;
  u32x4 in[CR + 3];
#pragma unroll
  for (int n = 0; n < CR + 3; ++n) {
    const int t = t0 - 3 + n;
    u32x4 v = {0, 0, 0, 0};
    if (t >= 0) {
      if (t < T) v = *(const u32x4 *)(u + (size_t)t * D);
    } else if (st) {
      v = *(const u32x4 *)(st + (size_t)ring_slot(p.pos0 + t) * D);
    }
    in[n] = v;
  }
#pragma unroll
  for (int r = 0; r < CR; ++r) {
    if (t0 + r >= T) break;
    u32x4 o, oh;
    typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      float x0 = bias[2 * e2], x1 = bias[2 * e2 + 1];
#pragma unroll
      for (int k = 0; k < 4; ++k) {   // lag k multiplies the input k steps back
        const unsigned v = in[r + 3 - k][e2];
        x0 = fmaf(w[k][2 * e2], bf_lo(v), x0);
        x1 = fmaf(w[k][2 * e2 + 1], bf_hi(v), x1);
      }
      o[e2] = pack_bf16(x0, x1);
      const f16x2 h2 = {(_Float16)x0, (_Float16)x1};
      oh[e2] = *(const unsigned *)&h2;
    }
    if (a.x) *(u32x4 *)(a.x + ((size_t)b * T + t0 + r) * D + d0) = o;
    *(u32x4 *)(a.xh + ((size_t)b * T + t0 + r) * D + d0) = oh;
  }
}

// ---- backward in passes, pointwise part: with delta_t from the adjoint scan, log a_t and i_t
// from the gates pass, x_t and h_{t-1}, the adjoints of eqs. (1)-(4) per element
//   dL/d(log a_t) = delta_t a_t (h_{t-1} - a_t i_t x_t / m_t),   dL/d(i_t x_t) = delta_t m_t
// (r_t, i_t from the gates pass: a_t = exp(-c softplus(-Lambda) r_t), m_t = sqrt(1 - a_t^2))
// written as fp32 x, dp, dq and the direct part of dx where the contraction passes expect them,
// plus the sums over a chunk of steps of dp, dq and of the Lambda term per (sequence, channel).
constexpr int PT_STEPS = 128;   // steps per thread
struct PointArgs {
  Problem p;
  const unsigned short *xh, *rv, *iv, *delta;   // x_t, the logits of r_t and i_t, delta_t in half precision, all [B][T][D]
  float *x, *dp, *dq, *dx;                      // [B][T][D] fp32
  float *part;                                  // [chunk][B][3][D]
  unsigned short *dpqh;                         // [B][T][nb][2][bs] half precision: dp and dq of a block side by
                                                // side (operand of both contractions)
  int fp32_operands;                            // also write fp32 x, dp, dq (the generic wgrad pass reads them)
};
__device__ __forceinline__ float half_bits(unsigned short v) { return (float)__builtin_bit_cast(_Float16, v); }

__global__ void __launch_bounds__(256) point_adjoint_kernel(PointArgs a) {
  const Problem &p = a.p;
  const int d = blockIdx.x * 256 + threadIdx.x, b = blockIdx.y, ch = blockIdx.z;
  if (d >= p.D) return;
  const int t0 = ch * PT_STEPS, t1 = min(t0 + PT_STEPS, p.T);
  const float lam = p.Lambda[d];
  const float z = -lam;
  const float neg_cs = -p.c * (z > 0.f ? z + log1pf(expf(-z)) : log1pf(expf(z)));   // -c softplus(-Lambda)
  const float lam_scale = p.c / (1.f + expf(lam));                                   // c sigmoid(-Lambda)
  float s_ba = 0.f, s_bx = 0.f, s_lam = 0.f;
  const int gb_ = d / p.bs, cb_ = d - gb_ * p.bs;
  for (int t = t0; t < t1; ++t) {
    const size_t o = ((size_t)b * p.T + t) * p.D + d;
    const float pl = half_bits(a.rv[o]);   // the logit of r_t
    const float r = 1.f / (1.f + expf(-pl)), rc = 1.f / (1.f + expf(pl)), la = neg_cs * r;
    const float av = expf(la), mv = sqrtf(-expm1f(2.f * la));
    const float ql = half_bits(a.iv[o]);   // the logit of i_t
    const float iv = 1.f / (1.f + expf(-ql)), ic = 1.f / (1.f + expf(ql));
    const float x = half_bits(a.xh[o]), delta = half_bits(a.delta[o]);
    const float hprev = t > 0 ? bf_lo((unsigned)((const unsigned short *)p.y_in)[o - p.D])
                              : (p.h0 ? p.h0[(size_t)b * p.D + d] : 0.f);
    const float gin = iv * x;
    const float corr = mv > 0.f ? av * gin / mv : 0.f;   // the term vanishes with the gate as m -> 0
    const float dla = delta * av * (hprev - corr);
    const float dg = delta * mv;
    const float dpv = neg_cs * dla * r * rc;
    const float dqv = dg * x * iv * ic;
    s_lam = fmaf(dla * r, lam_scale, s_lam);
    s_ba += dpv;
    s_bx += dqv;
    if (a.fp32_operands) {
      a.x[o] = x;
      a.dp[o] = dpv;
      a.dq[o] = dqv;
    }
    a.dx[o] = dg * iv;
    {
      const size_t oq = (((size_t)b * p.T + t) * p.nb + gb_) * 2 * p.bs + cb_;
      a.dpqh[oq] = __builtin_bit_cast(unsigned short, (_Float16)dpv);
      a.dpqh[oq + p.bs] = __builtin_bit_cast(unsigned short, (_Float16)dqv);
    }
  }
  float *out = a.part + ((size_t)ch * p.B + b) * 3 * p.D + d;
  out[0] = s_ba;
  out[p.D] = s_bx;
  out[2 * (size_t)p.D] = s_lam;
}

// du[b,t,d] = sum_k conv_w[k][d] dx[b,t+k,d] (adjoint of the Conv1D with respect to its input): a
// thread makes 4 channels of CR consecutive steps from CR + 3 rows of the fp32 dx
struct ConvAdjArgs {
  const float *dx, *conv_w;
  unsigned short *du;
  int B, T, D;
};
__global__ void __launch_bounds__(256) conv_adjoint_rows_kernel(ConvAdjArgs a) {
  const int D = a.D, T = a.T, nch = D / 4, ntr = (T + CR - 1) / CR;
  const size_t total = (size_t)a.B * ntr * nch;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % nch);
  const int tr = (int)((i / nch) % ntr);
  const int b = (int)(i / ((size_t)nch * ntr));
  const int t0 = tr * CR, d0 = c * 4;
  f32x4 w[4], in[CR + 3];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const float id = k == 0 ? 1.f : 0.f;   // no Conv1D: du = dx
    w[k] = a.conv_w ? *(const f32x4 *)(a.conv_w + (size_t)k * D + d0) : f32x4{id, id, id, id};
  }
  const float *dx = a.dx + (size_t)b * T * D + d0;
#pragma unroll
  for (int n = 0; n < CR + 3; ++n) {   // (no load under a condition: rows past the end re-read the last row)
    const int t = t0 + n;
    in[n] = *(const f32x4 *)(dx + (size_t)(t < T ? t : T - 1) * D);
    if (t >= T) in[n] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
#pragma unroll
  for (int r = 0; r < CR; ++r) {
    if (t0 + r >= T) break;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[e] = fmaf(w[k][e], in[r + k][e], acc[e]);
    uint2 o;
    o.x = pack_bf16(acc[0], acc[1]);
    o.y = pack_bf16(acc[2], acc[3]);
    *(uint2 *)(a.du + ((size_t)b * T + t0 + r) * D + d0) = o;
  }
}
}  // namespace
// du from the fp32 dx with the streaming kernel above: bf16 storage, rows that hold one document each,
// a width that is a multiple of 4 and 8-byte / 16-byte aligned du / taps; false if it does not apply
bool conv_adjoint_rows_applies(const Problem &p, bool bf) {
  return bf && !p.reset && p.D % 4 == 0 && p.T >= 1 && (uintptr_t)p.du % 8 == 0 && (uintptr_t)p.conv_w % 16 == 0;
}
hipError_t launch_conv_adjoint_rows(const Problem &p, const float *dx, hipStream_t s) {
  KernelTimer kt("conv_adjoint_rows_kernel", s);
  ConvAdjArgs ca;
  ca.dx = dx; ca.conv_w = p.conv_w; ca.du = (unsigned short *)p.du;
  ca.B = p.B; ca.T = p.T; ca.D = p.D;
  const size_t total = (size_t)p.B * ((p.T + CR - 1) / CR) * (p.D / 4);
  hipLaunchKernelGGL(conv_adjoint_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, ca);
  return hipGetLastError();
}
namespace {

// bf16 -> half precision, n elements (gate weights: the products run on the f16 form of the MFMA
// with x in half precision; exact for weights from 6.1e-5 up to 65504, smaller ones round with
// an absolute error below 3e-8)
__global__ void __launch_bounds__(256) to_f16_kernel(const unsigned short *src, unsigned short *dst, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = __builtin_bit_cast(unsigned short, (_Float16)__uint_as_float((unsigned)src[i] << 16));
}

// W'[g][k][gate * bs + j] = W_gate[g][j][k]: the transposed gate matrices of a block side by side,
// in half precision
__global__ void __launch_bounds__(256) wt_concat_kernel(const unsigned short *Wa, const unsigned short *Wx,
                                                        unsigned short *out, int nb, int bs) {
  const size_t total = (size_t)nb * bs * 2 * bs;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int jj = (int)(i % (2 * bs));
  const int k = (int)((i / (2 * bs)) % bs);
  const int g = (int)(i / ((size_t)2 * bs * bs));
  const int gate = jj >= bs, j = jj - gate * bs;
  // (bf16 -> half precision is exact from 6.1e-5 up to 65504; smaller weights round with an
  // absolute error below 3e-8)
  const float w = __uint_as_float((unsigned)(gate ? Wx : Wa)[((size_t)g * bs + j) * bs + k] << 16);
  out[i] = __builtin_bit_cast(unsigned short, (_Float16)w);
}

// dst[c][r] = src[r][c] for 16-bit elements, 64 x 64 tiles through LDS, two elements per access
// on both sides (R and C even)
__global__ void __launch_bounds__(256) transpose16_kernel(const unsigned short *src, unsigned short *dst,
                                                          unsigned R, unsigned C) {
  __shared__ unsigned short tile[64][66];
  const unsigned r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const unsigned tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 pairs across, 8 lines down
  for (unsigned i = ty; i < 64; i += 8) {
    unsigned v = 0;
    if (r0 + i < R && c0 + 2 * tx < C) v = *(const unsigned *)(src + (size_t)(r0 + i) * C + c0 + 2 * tx);
    tile[i][2 * tx] = (unsigned short)(v & 0xffffu);
    tile[i][2 * tx + 1] = (unsigned short)(v >> 16);
  }
  __syncthreads();
  for (unsigned i = ty; i < 64; i += 8)
    if (c0 + i < C && r0 + 2 * tx < R)
      *(unsigned *)(dst + (size_t)(c0 + i) * R + r0 + 2 * tx) =
          (unsigned)tile[2 * tx][i] | ((unsigned)tile[2 * tx + 1][i] << 16);
}

// ---- range of the upstream gradient. The backward in passes keeps delta_t, dp_t and dq_t in IEEE
// half precision (operands of the f16 matrix-core products), whose exponent range is narrow,
// while gradients are linear in dy and arrive at any scale (a mean-reduced loss gives 1e-5 ..
// 1e-7 per element). The passes therefore run on dy * S and dhT * S with S the power of two that
// brings max(|dy|, |dhT|) into [16, 32) - exact in bf16 and fp32 - and every result is multiplied
// by 1 / S at the end.
// bits of max |v| over n bf16 values (the bit patterns of non-negative floats order like integers)
__global__ void __launch_bounds__(256) absmax_bf16_kernel(const unsigned short *v, size_t n, unsigned *out) {
  unsigned m = 0;
  auto take = [&](unsigned bits16) {
    const unsigned b = (bits16 & 0x7fffu) << 16;
    if (b <= 0x7f800000u) m = max(m, b);   // NaNs are left out of the range estimate
  };
  // 16 bytes per thread where the address allows it (always, for tensors the matrix-core paths take)
  const size_t n8 = (((uintptr_t)v & 15) == 0) ? n / 8 : 0;
  const uint4 *v8 = (const uint4 *)v;
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  auto take8 = [&](const uint4 &w) {
    take(w.x); take(w.x >> 16); take(w.y); take(w.y >> 16);
    take(w.z); take(w.z >> 16); take(w.w); take(w.w >> 16);
  };
  for (; i + 3 * stride < n8; i += 4 * stride) {   // four loads in flight per thread
    const uint4 w0 = v8[i], w1 = v8[i + stride], w2 = v8[i + 2 * stride], w3 = v8[i + 3 * stride];
    take8(w0); take8(w1); take8(w2); take8(w3);
  }
  for (; i < n8; i += stride) take8(v8[i]);
  for (size_t k = n8 * 8 + (size_t)blockIdx.x * 256 + threadIdx.x; k < n; k += stride) take(v[k]);
  for (int o = 32; o > 0; o >>= 1) m = max(m, (unsigned)__shfl_xor((int)m, o));
  // one atomic per workgroup: thousands of them on one address would cost more than the pass itself
  __shared__ unsigned wm[4];
  if ((threadIdx.x & 63) == 0) wm[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    m = max(max(wm[0], wm[1]), max(wm[2], wm[3]));
    if (m) atomicMax(out, m);
  }
}
__global__ void __launch_bounds__(256) absmax_f32_kernel(const float *v, size_t n, unsigned *out) {
  unsigned m = 0;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    const unsigned b = __float_as_uint(v[i]) & 0x7fffffffu;
    if (b <= 0x7f800000u) m = max(m, b);
  }
  for (int o = 32; o > 0; o >>= 1) m = max(m, (unsigned)__shfl_xor((int)m, o));
  if ((threadIdx.x & 63) == 0 && m) atomicMax(out, m);
}
// sc[0] = bits of the maximum (in), sc[1] = S, sc[2] = 1 / S (out); the scaled maximum lands in
// [2^shift, 2^(shift+1))
__global__ void scale_setup_kernel(float *sc, int shift) {
  const unsigned bits = __float_as_uint(sc[0]);
  int e = (int)(bits >> 23) - 127 - shift;        // max in [2^(e+shift), 2^(e+shift+1))
  if (bits == 0 || bits >= 0x7f800000u) e = 0;   // all zero, or infinite: leave the values alone
  if (e > 126) e = 126;
  if (e < -126) e = -126;
  sc[1] = __uint_as_float((unsigned)(127 - e) << 23);
  sc[2] = __uint_as_float((unsigned)(127 + e) << 23);
}
// dst = src * sc[which] for bf16 values (a power of two: exact unless the result leaves the range)
__global__ void __launch_bounds__(256) scale_bf16_kernel(const unsigned short *src, unsigned short *dst, size_t n,
                                                         const float *sc, int which) {
  const float f = sc[which];
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256)
    dst[i] = (unsigned short)(pack_bf16(bf_lo((unsigned)src[i]) * f, 0.f) & 0xffffu);
}
// dst (half precision) = (hi + lo) * sc[1] for an upstream gradient given as two bf16 tensors
__global__ void __launch_bounds__(256) scale_sum_f16_kernel(const unsigned short *hi, const unsigned short *lo,
                                                            unsigned short *dst, size_t n, const float *sc) {
  const float f = sc[1];
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    const _Float16 h = (_Float16)((bf_lo((unsigned)hi[i]) + bf_lo((unsigned)lo[i])) * f);
    dst[i] = __builtin_bit_cast(unsigned short, h);
  }
}
__global__ void __launch_bounds__(256) scale_f32_kernel(const float *src, float *dst, size_t n, const float *sc,
                                                        int which) {
  const float f = sc[which];
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i] * f;
}

// partA[b][r][d] = sum over chunks, in a fixed order
__global__ void __launch_bounds__(256) sum_chunks_kernel(const float *part, float *partA, int nch, size_t per_chunk) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= per_chunk) return;
  float s = 0.f;
  for (int c = 0; c < nch; ++c) s += part[(size_t)c * per_chunk + i];
  partA[i] = s;
}

}  // namespace

bool forward_wide_block(int bs) { return bs % 16 == 0 && bs >= 16 && !forward_mfma_block(bs); }

// (the scan pass needs a width that is a multiple of 256; 16-byte accesses throughout)
bool forward_wide_supported(const Problem &p, bool bf) {
  const uintptr_t all = (uintptr_t)p.W_a | (uintptr_t)p.W_x | (uintptr_t)p.y | (uintptr_t)p.u |
                        (uintptr_t)p.state_in | (uintptr_t)p.conv_w | (uintptr_t)p.conv_b;
  return bf && forward_wide_block(p.bs) && p.D % BS == 0 && p.T >= 1 && all % 16 == 0 &&
         (size_t)p.B * p.T * p.D * 2 < ((size_t)1 << 31);
}

size_t forward_wide_ws_bytes(int B, int T, int D, int nb) {
  const size_t n = al256((size_t)B * T * D * 2);
  const size_t wf = al256((size_t)nb * (D / nb) * (D / nb) * 2);   // a gate's weights in half precision
  return 4 * n + 2 * wf + scan_tiled_ws_bytes(B, T, D);
}

hipError_t launch_forward_wide(const Problem &p, hipStream_t s) {
  const size_t n = al256((size_t)p.B * p.T * p.D * 2);
  char *ws = (char *)p.ws;
  void *la = ws + n, *gb = ws + 2 * n, *xh = ws + 3 * n;
  const size_t wf = al256((size_t)p.nb * p.bs * p.bs * 2);
  unsigned short *wfa = (unsigned short *)(ws + 4 * n), *wfx = (unsigned short *)(ws + 4 * n + wf);
  const size_t scan_off = 4 * n + 2 * wf;
  {
    KernelTimer kt("to_f16_kernel", s);
    const size_t nw = (size_t)p.nb * p.bs * p.bs;
    hipLaunchKernelGGL(to_f16_kernel, dim3((unsigned)((nw + 255) / 256)), dim3(256), 0, s, (const unsigned short *)p.W_a, wfa, nw);
    hipLaunchKernelGGL(to_f16_kernel, dim3((unsigned)((nw + 255) / 256)), dim3(256), 0, s, (const unsigned short *)p.W_x, wfx, nw);
    hipError_t e0 = hipGetLastError();
    if (e0 != hipSuccess) return e0;
  }
  hipError_t e;
  {
    KernelTimer kt("conv_rows_kernel", s);
    ConvArgs c;
    c.p = p;
    c.x = nullptr;
    c.xh = (unsigned short *)xh;
    const size_t total = (size_t)p.B * ((p.T + CR - 1) / CR) * (p.D / 8);
    hipLaunchKernelGGL(conv_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, c);
    e = hipGetLastError();
  }
  if (e != hipSuccess) return e;
  WideArgs a;
  a.p = p;
  a.p.W_a = wfa;
  a.p.W_x = wfx;
  a.x = (const unsigned short *)xh;
  a.xh = nullptr;
  a.la = (unsigned short *)la;
  a.gb = (unsigned short *)gb;
  a.rv = nullptr;
  a.nob = (p.bs + BS - 1) / BS;
  a.nkc = a.nob;
  a.kdim = p.bs;
  a.x_row_bytes = (unsigned)p.D * 2;
  a.dx = nullptr;
  a.w_block_elems = (size_t)p.bs * p.bs;
  a.dWa = a.dWx = nullptr;
  a.ntiles = (unsigned)(((size_t)p.B * p.T + WM - 1) / WM);
  a.M = (unsigned)((size_t)p.B * p.T);
  static bool configured = false;
  if (!configured) {
    e = hipFuncSetAttribute((const void *)gates_wide_kernel<MODE_FWD>, hipFuncAttributeMaxDynamicSharedMemorySize, W_LDS);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void *)gates_wide_kernel<MODE_BWD>, hipFuncAttributeMaxDynamicSharedMemorySize, W_LDS);
    if (e != hipSuccess) return e;
    configured = true;
  }
  {
    KernelTimer kt("gates_wide_kernel", s);
    hipLaunchKernelGGL(gates_wide_kernel<MODE_FWD>, dim3(wide_grid_x(a.ntiles, p.nb * a.nob), p.nb * a.nob), dim3(NTHR), W_LDS, s, a);
    e = hipGetLastError();
  }
  if (e != hipSuccess) return e;
  ScanProblem q;
  q.B = p.B; q.T = p.T; q.D = p.D;
  q.flags = RGLRU_SCAN_LOG_A | RGLRU_SCAN_NO_INPUT_SCALE | SCAN_G_FP16;   // b_t carries sqrt(1 - a_t^2)
  q.a = la; q.g = gb; q.h0 = p.h0; q.h = p.y; q.hT = p.hT;
  q.ws = ws + scan_off;
  q.ws_bytes = p.ws_bytes > scan_off ? p.ws_bytes - scan_off : 0;
  if (!scan_tiled_supported(q, true)) return hipErrorInvalidValue;
  e = launch_scan_tiled(q, s);
  if (e != hipSuccess) return e;
  return launch_state_update(p, true, s);
}

}  // namespace rglru

namespace rglru {

// ---- backward for these block sizes: the pointwise pass of the generic kernels (sequential in
// time, with the gate products on the vector unit: 80 % of their time) replaced by passes -
// Conv1D rows, gate products on the matrix cores, the adjoint scan, the pointwise adjoints - that
// leave x, dp, dq and the direct part of dx where the generic contraction passes expect them.
namespace {
struct BwdWidePlan {
  size_t generic, n2, off_x, off_xh, off_la, off_iv, off_rv, off_delta, off_part, off_dpqh, off_xT, off_wf, wf,
      off_dpqT, off_wt, off_dys, off_dhTs, off_scale, off_scan, total;
  int nch;
};
BwdWidePlan plan_bwd_wide(int B, int T, int D, int nb) {
  BwdWidePlan q;
  q.generic = al256(backward_generic_ws_bytes(B, T, D, nb));
  q.n2 = al256((size_t)B * T * D * 2);
  q.nch = (T + PT_STEPS - 1) / PT_STEPS;
  size_t off = q.generic;
  q.off_x = off; off += q.n2;
  q.off_xh = off; off += q.n2;
  q.off_la = off; off += q.n2;
  q.off_iv = off; off += q.n2;
  q.off_rv = off; off += q.n2;
  q.off_delta = off; off += q.n2;
  q.off_part = off; off += al256((size_t)q.nch * B * 3 * D * 4);
  q.off_dpqh = off; off += 2 * q.n2;
  q.wf = al256((size_t)nb * (D / nb) * (D / nb) * 2);
  q.off_wf = off; off += 2 * q.wf;
  q.off_xT = off; off += q.n2;
  q.off_dpqT = off; off += 2 * q.n2;
  q.off_wt = off; off += al256((size_t)nb * (D / nb) * 2 * (D / nb) * 2);
  q.off_dys = off; off += q.n2;                               // dy * S
  q.off_dhTs = off; off += al256((size_t)B * D * 4);          // dhT * S
  q.off_scale = off; off += 256;                              // max bits, S, 1 / S
  q.off_scan = off; off += scan_tiled_ws_bytes(B, T, D);
  q.total = off;
  return q;
}
}  // namespace

bool backward_wide_supported(const Problem &p, bool bf) {
  const uintptr_t all = (uintptr_t)p.W_a | (uintptr_t)p.W_x | (uintptr_t)p.u | (uintptr_t)p.dy |
                        (uintptr_t)p.state_in | (uintptr_t)p.conv_w | (uintptr_t)p.conv_b;
  return bf && forward_wide_block(p.bs) && p.D % BS == 0 && p.T >= 1 && all % 16 == 0 &&
         (size_t)p.B * p.T * p.D * 4 < ((size_t)1 << 31) && (p.T + PT_STEPS - 1) / PT_STEPS <= 65535 &&
         p.B <= 65535;
}

size_t backward_wide_ws_bytes(int B, int T, int D, int nb) { return plan_bwd_wide(B, T, D, nb).total; }

size_t backward_wide_flag_offset(int B, int T, int D, int nb) {   // 0 if the scan does not slice
  return scan_tiled_ws_bytes(B, T, D) ? plan_bwd_wide(B, T, D, nb).off_scan : 0;
}

static unsigned stream_grid(size_t n) { return (unsigned)((n + 255) / 256 < 2048 ? (n + 255) / 256 : 2048); }

// sc (256 bytes of scratch, 16-byte aligned) <- the power of two S that brings max(|dy|, |dhT|)
// into [2^shift, 2^(shift+1)) and 1 / S, as sc[1] and sc[2]; dy bf16 [n], dhT fp32 [nd] or null
hipError_t launch_grad_scale(const void *dy, size_t n, const float *dhT, size_t nd, float *sc, int shift,
                             hipStream_t s) {
  KernelTimer kt("grad_scale_kernels", s);
  hipError_t e = launch_clear(sc, 256, s);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(absmax_bf16_kernel, dim3(stream_grid((n + 7) / 8)), dim3(256), 0, s, (const unsigned short *)dy, n,
                     (unsigned *)sc);
  if (dhT) hipLaunchKernelGGL(absmax_f32_kernel, dim3(stream_grid(nd)), dim3(256), 0, s, dhT, nd, (unsigned *)sc);
  hipLaunchKernelGGL(scale_setup_kernel, dim3(1), dim3(1), 0, s, sc, shift);
  return hipGetLastError();
}

hipError_t launch_backward_wide(const Problem &p_in, hipStream_t s) {
  const BwdWidePlan q = plan_bwd_wide(p_in.B, p_in.T, p_in.D, p_in.nb);
  char *ws = (char *)p_in.ws;
  hipError_t e;
  // the passes run on dy * S and dhT * S (see absmax_bf16_kernel); results are unscaled at the end
  Problem p = p_in;
  float *sc = (float *)(ws + q.off_scale);
  const size_t N = (size_t)p.B * p.T * p.D, BD = (size_t)p.B * p.D;
  {
    // the scaled maximum lands in [16, 32): the adjoints stay below a few thousand times that,
    // inside half precision's 65504, and the small ones (channels whose gates are nearly shut)
    // keep four more bits above its subnormal range
    if ((e = launch_grad_scale(p_in.dy, N, p_in.dhT, BD, sc, 4, s)) != hipSuccess) return e;
    KernelTimer kt("grad_scale_kernels", s);
    if (p_in.dy_lo)   // dy + dy_lo: 16 significant bits, kept as far as half precision holds them
      hipLaunchKernelGGL(scale_sum_f16_kernel, dim3(stream_grid(N)), dim3(256), 0, s, (const unsigned short *)p_in.dy,
                         (const unsigned short *)p_in.dy_lo, (unsigned short *)(ws + q.off_dys), N, (const float *)sc);
    else
      hipLaunchKernelGGL(scale_bf16_kernel, dim3(stream_grid(N)), dim3(256), 0, s, (const unsigned short *)p_in.dy,
                         (unsigned short *)(ws + q.off_dys), N, (const float *)sc, 1);
    p.dy = ws + q.off_dys;
    if (p_in.dhT) {
      hipLaunchKernelGGL(scale_f32_kernel, dim3(stream_grid(BD)), dim3(256), 0, s, p_in.dhT,
                         (float *)(ws + q.off_dhTs), BD, (const float *)sc, 1);
      p.dhT = (const float *)(ws + q.off_dhTs);
    }
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  {
    KernelTimer kt("conv_rows_kernel", s);
    ConvArgs c;
    c.p = p;
    c.x = nullptr;
    c.xh = (unsigned short *)(ws + q.off_xh);
    const size_t total = (size_t)p.B * ((p.T + CR - 1) / CR) * (p.D / 8);
    hipLaunchKernelGGL(conv_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, c);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  WideArgs a;
  a.p = p;
  {
    KernelTimer kt("to_f16_kernel", s);
    const size_t nw = (size_t)p.nb * p.bs * p.bs;
    hipLaunchKernelGGL(to_f16_kernel, dim3((unsigned)((nw + 255) / 256)), dim3(256), 0, s, (const unsigned short *)p.W_a,
                       (unsigned short *)(ws + q.off_wf), nw);
    hipLaunchKernelGGL(to_f16_kernel, dim3((unsigned)((nw + 255) / 256)), dim3(256), 0, s, (const unsigned short *)p.W_x,
                       (unsigned short *)(ws + q.off_wf + q.wf), nw);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  a.p.W_a = ws + q.off_wf;
  a.p.W_x = ws + q.off_wf + q.wf;
  a.x = (const unsigned short *)(ws + q.off_xh);
  a.xh = nullptr;
  a.la = (unsigned short *)(ws + q.off_la);
  a.gb = (unsigned short *)(ws + q.off_iv);
  a.rv = (unsigned short *)(ws + q.off_rv);
  a.nob = (p.bs + BS - 1) / BS;
  a.nkc = a.nob;
  a.kdim = p.bs;
  a.x_row_bytes = (unsigned)p.D * 2;
  a.dx = nullptr;
  a.w_block_elems = (size_t)p.bs * p.bs;
  a.dWa = a.dWx = nullptr;
  a.ntiles = (unsigned)(((size_t)p.B * p.T + WM - 1) / WM);
  a.M = (unsigned)((size_t)p.B * p.T);
  static bool configured = false;
  if (!configured) {
    e = hipFuncSetAttribute((const void *)gates_wide_kernel<MODE_BWD>, hipFuncAttributeMaxDynamicSharedMemorySize, W_LDS);
    if (e != hipSuccess) return e;
    configured = true;
  }
  {
    KernelTimer kt("gates_wide_kernel", s);
    hipLaunchKernelGGL(gates_wide_kernel<MODE_BWD>, dim3(wide_grid_x(a.ntiles, p.nb * a.nob), p.nb * a.nob), dim3(NTHR), W_LDS, s, a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  // delta_t = dy_t + a_{t+1} delta_{t+1}; its last value times a_0 is dh0
  ScanProblem sp;
  sp.B = p.B; sp.T = p.T; sp.D = p.D;
  sp.flags = RGLRU_SCAN_LOG_A | RGLRU_SCAN_NO_INPUT_SCALE | RGLRU_SCAN_ADJOINT | SCAN_OUT_FP16 |
             (p_in.dy_lo ? SCAN_G_FP16 : 0u);
  sp.a = ws + q.off_la; sp.g = p.dy; sp.h0 = p.dhT; sp.h = ws + q.off_delta; sp.hT = p.dh0;
  sp.ws = ws + q.off_scan;
  sp.ws_bytes = q.total - q.off_scan;
  if (!scan_tiled_supported(sp, true)) return hipErrorInvalidValue;
  if ((e = launch_scan_tiled(sp, s)) != hipSuccess) return e;
  {
    KernelTimer kt("point_adjoint_kernel", s);
    PointArgs pa;
    pa.p = p;
    pa.xh = (const unsigned short *)(ws + q.off_xh);
    pa.rv = (const unsigned short *)(ws + q.off_rv);
    pa.iv = (const unsigned short *)(ws + q.off_iv);
    pa.delta = (const unsigned short *)(ws + q.off_delta);
    float *gx, *gdp, *gdq, *gdx, *gpartA;
    backward_generic_arrays(p, &gx, &gdp, &gdq, &gdx, &gpartA);
    pa.x = gx; pa.dp = gdp; pa.dq = gdq; pa.dx = gdx;
    pa.part = (float *)(ws + q.off_part);
    pa.dpqh = (unsigned short *)(ws + q.off_dpqh);
    pa.fp32_operands = ((size_t)p.B * p.T) % 8 != 0;   // (else both contractions run on the matrix cores)
    hipLaunchKernelGGL(point_adjoint_kernel, dim3((p.D + 255) / 256, p.B, q.nch), dim3(256), 0, s, pa);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const size_t per_chunk = (size_t)p.B * 3 * p.D;
    hipLaunchKernelGGL(sum_chunks_kernel, dim3((unsigned)((per_chunk + 255) / 256)), dim3(256), 0, s,
                       (const float *)(ws + q.off_part), gpartA, q.nch, per_chunk);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  // dx += [dp | dq] [W_a | W_x]^T on the matrix cores (the product machinery of the gates pass)
  {
    KernelTimer kt("wt_concat_kernel", s);
    const size_t total = (size_t)p.nb * p.bs * 2 * p.bs;
    hipLaunchKernelGGL(wt_concat_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                       (const unsigned short *)p.W_a, (const unsigned short *)p.W_x,
                       (unsigned short *)(ws + q.off_wt), p.nb, p.bs);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  {
    WideArgs dg;
    dg.p = p;
    dg.p.W_a = ws + q.off_wt;
    dg.p.W_x = ws + q.off_wt;
    dg.x = (const unsigned short *)(ws + q.off_dpqh);
    dg.xh = nullptr; dg.la = dg.gb = dg.rv = nullptr;
    dg.nob = (p.bs + BS - 1) / BS;
    dg.kdim = 2 * p.bs;
    dg.nkc = (dg.kdim + BS - 1) / BS;
    dg.x_row_bytes = (unsigned)p.D * 4;
    dg.w_block_elems = (size_t)p.bs * 2 * p.bs;
    dg.dWa = dg.dWx = nullptr;
    dg.M = (unsigned)((size_t)p.B * p.T);
    dg.ntiles = (dg.M + WM - 1) / WM;
    float *gx, *gdp, *gdq, *gdx, *gpartA;
    backward_generic_arrays(p, &gx, &gdp, &gdq, &gdx, &gpartA);
    dg.dx = gdx;
    static bool configured_dg = false;
    if (!configured_dg) {
      e = hipFuncSetAttribute((const void *)gates_wide_kernel<MODE_DGRAD>, hipFuncAttributeMaxDynamicSharedMemorySize, W_LDS);
      if (e != hipSuccess) return e;
      configured_dg = true;
    }
    KernelTimer kt("dgrad_wide_kernel", s);
    hipLaunchKernelGGL(gates_wide_kernel<MODE_DGRAD>, dim3(wide_grid_x(dg.ntiles, p.nb * dg.nob), p.nb * dg.nob), dim3(NTHR), W_LDS, s, dg);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  // dW_a, dW_x on the matrix cores: transposed half-precision copies of x and of dp | dq, then the
  // product machinery with the roles turned (the sum over all (sequence, step) rows is one
  // workgroup's K loop: no partial sums, a fixed order)
  const unsigned M = (unsigned)((size_t)p.B * p.T);
  const bool mfma_wgrad = M % 8 == 0;
  if (mfma_wgrad) {
    {
      KernelTimer kt("transpose16_kernel", s);
      hipLaunchKernelGGL(transpose16_kernel, dim3((p.D + 63) / 64, (M + 63) / 64), dim3(256), 0, s,
                         (const unsigned short *)(ws + q.off_xh), (unsigned short *)(ws + q.off_xT), M, (unsigned)p.D);
      hipLaunchKernelGGL(transpose16_kernel, dim3((2 * p.D + 63) / 64, (M + 63) / 64), dim3(256), 0, s,
                         (const unsigned short *)(ws + q.off_dpqh), (unsigned short *)(ws + q.off_dpqT), M,
                         2u * (unsigned)p.D);
      if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    WideArgs wg;
    wg.p = p;
    wg.p.W_a = ws + q.off_dpqT;
    wg.p.W_x = ws + q.off_dpqT + (size_t)p.bs * M * 2;
    wg.x = (const unsigned short *)(ws + q.off_xT);
    wg.xh = nullptr; wg.la = wg.gb = wg.rv = nullptr; wg.dx = nullptr;
    wg.nob = (p.bs + BS - 1) / BS;
    wg.kdim = (int)M;
    wg.nkc = (int)((M + BS - 1) / BS);
    wg.x_row_bytes = M * 2;
    wg.w_block_elems = (size_t)2 * p.bs * M;
    wg.M = M;
    wg.ntiles = (unsigned)((p.bs + WM - 1) / WM);   // few row tiles with a very long K: one per workgroup
    wg.dWa = p.g.dW_a;
    wg.dWx = p.g.dW_x;
    static bool configured_wg = false;
    if (!configured_wg) {
      e = hipFuncSetAttribute((const void *)gates_wide_kernel<MODE_WGRAD>, hipFuncAttributeMaxDynamicSharedMemorySize, W_LDS);
      if (e != hipSuccess) return e;
      configured_wg = true;
    }
    KernelTimer kt("wgrad_wide_kernel", s);
    hipLaunchKernelGGL(gates_wide_kernel<MODE_WGRAD>, dim3(wg.ntiles, p.nb * wg.nob), dim3(NTHR), W_LDS, s, wg);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  // (du: the tail takes the streaming kernel below where it applies)
  if ((e = launch_backward_generic_tail(p, true, s, false, !mfma_wgrad, true)) != hipSuccess) return e;
  {
    KernelTimer kt("grad_scale_kernels", s);
    hipLaunchKernelGGL(scale_bf16_kernel, dim3(stream_grid(N)), dim3(256), 0, s, (const unsigned short *)p.du,
                       (unsigned short *)p.du, N, (const float *)sc, 2);
    const size_t nw = (size_t)p.nb * p.bs * p.bs, D = (size_t)p.D;
    float *outs[8] = {p.g.dW_a, p.g.dW_x, p.g.db_a, p.g.db_x, p.g.dLambda, p.g.dconv_w, p.g.dconv_b, p.dh0};
    const size_t ns[8] = {nw, nw, D, D, D, 4 * D, D, BD};
    for (int i = 0; i < 8; ++i)
      if (outs[i])
        hipLaunchKernelGGL(scale_f32_kernel, dim3(stream_grid(ns[i])), dim3(256), 0, s, (const float *)outs[i],
                           outs[i], ns[i], (const float *)sc, 2);
    e = hipGetLastError();
  }
  return e;
}

bool decode_wide_supported(const Problem &p, bool bf) {
  const uintptr_t all = (uintptr_t)p.W_a | (uintptr_t)p.W_x | (uintptr_t)p.u | (uintptr_t)p.state_out |
                        (uintptr_t)p.hT | (uintptr_t)p.y | (uintptr_t)p.conv_w | (uintptr_t)p.conv_b |
                        (uintptr_t)(p.merge ? p.branch : nullptr);
  return bf && p.conv_w && forward_wide_block(p.bs) && p.bs <= DW_MAXCH * BS && all % 16 == 0 &&
         (size_t)(p.B + TT) * 3 * p.D * 2 < ((size_t)1 << 31);
}

hipError_t launch_decode_wide(const Problem &p, hipStream_t s) {
  DecWideArgs a;
  a.p = p;
  a.nob = (p.bs + BS - 1) / BS;
  static bool configured = false;
  hipError_t e;
  if (!configured) {
    if ((e = hipFuncSetAttribute((const void *)decode_wide_kernel<0>, hipFuncAttributeMaxDynamicSharedMemorySize, DW_LDS)) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute((const void *)decode_wide_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, DW_LDS)) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute((const void *)decode_wide_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize, DW_LDS)) != hipSuccess) return e;
    if ((e = hipFuncSetAttribute((const void *)decode_wide_kernel<0, true>, hipFuncAttributeMaxDynamicSharedMemorySize, DW_LDS)) != hipSuccess) return e;
    configured = true;
  }
  const dim3 grid(p.nb * a.nob, (p.B + TT - 1) / TT);
  {
    KernelTimer kt("decode_wide_kernel", s);
    if (p.pos_rows) hipLaunchKernelGGL((decode_wide_kernel<0, true>), grid, dim3(NTHR), DW_LDS, s, a);
    else if (p.merge == 0) hipLaunchKernelGGL(decode_wide_kernel<0>, grid, dim3(NTHR), DW_LDS, s, a);
    else if (p.merge == 1) hipLaunchKernelGGL(decode_wide_kernel<1>, grid, dim3(NTHR), DW_LDS, s, a);
    else hipLaunchKernelGGL(decode_wide_kernel<2>, grid, dim3(NTHR), DW_LDS, s, a);
    e = hipGetLastError();
  }
  if (e != hipSuccess) return e;
  const int chunks = p.D / 8;
  hipLaunchKernelGGL(ring_store_kernel, dim3((p.B * chunks + 255) / 256), dim3(256), 0, s, (const uint4 *)p.u,
                     (uint4 *)p.state_out, p.B, chunks, ring_slot(p.pos0), p.pos_rows);
  return hipGetLastError();
}

}  // namespace rglru
