// Backward for bf16 storage and gate blocks of 256 channels (gfx950), in three kernels:
//
//  1. bwd_gates_kernel - walks each (sequence, gate block) backwards in tiles of 32 steps:
//     recomputes the Conv1D and the gates (same MFMA layout as the forward kernel), runs the
//     reverse scan eps_t = a_t (dy_t + eps_{t+1}) (so that delta_t = dy_t + eps_{t+1}) and forms
//     the pointwise adjoints of Section 2.4 eqs. (1)-(4):
//        dla_t = delta_t a_t (h_{t-1} - a_t g_t / m_t)      g = i x, m = sqrt(1 - a^2)
//                (h_{t-1} is the stored y_{t-1}, or h0 at the first step. The algebraically
//                 equal delta (h_t - g / m) would need y_t only, but it cancels: for small a_t
//                 the state h_{t-1} has left no trace in the rounded y_t)
//        dp_t  = -c softplus(-Lambda) dla_t r_t (1 - r_t)
//        dq_t  = delta_t m_t g_t (1 - i_t)
//        dxd_t = delta_t m_t i_t                 (the part of dx that bypasses the gates)
//     and writes S dp, S dq, S dxd in half precision (S: the power of two that brings max |dy| into
//     [32, 64), found by a pass over dy beforehand; the dgrad and wgrad kernels undo it; four
//     steps of a channel of dxd packed in 8 bytes) plus per-channel sums for db_a, db_x, dLambda.
//     Time slices of one sequence exchange tile aggregates (prod a, local eps) as tagged 8-byte
//     records; a first sweep over the tile computes a_t and the aggregate, a second sweep the
//     adjoints once the incoming eps is known.
//  2. bwd_dgrad_kernel - dx = dxd + dp W_a + dq W_x, the products on the matrix cores (transposed weights
//     resident in registers), then the Conv1D adjoint: du_t = sum_k w_k dx_{t+k},
//     dconv_w[k] = sum dx_t u_{t-k}, dconv_b = sum dx_t.
//  3. bwd_wgrad_kernel - dW_a = dp^T x, dW_x = dq^T x with the time axis as the contraction.
#include "rglru_mfma.h"

namespace rglru {

using namespace mfma;

namespace {

typedef unsigned u32x3 __attribute__((ext_vector_type(3)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
constexpr int TS = TT + 8;                       // row stride (bf16) of the [channel][time] tiles
constexpr int TR_BYTES = BS * TS * 2;            // one transposed tile
// LDS of the gates kernel: x tile (high, low) | constants | dy^T | y^T | r_t of the tile |
// W_x fragments
constexpr int G_NRES = 4;                        // K-steps of W_x resident in registers (5 without time slices)
// further K-steps of W_x resident in LDS (an upstream gradient given as two bf16 tensors needs
// a second transposed tile, which takes the room of two of them)
constexpr int g_nlds(bool dylo) { return dylo ? 3 : 5; }
constexpr int G_OFF_CONST = XS_BYTES / 2;        // one x buffer: the kernel has two barriers per tile
constexpr int G_OFF_DYT = G_OFF_CONST + CONST_BYTES;
constexpr int G_OFF_YT = G_OFF_DYT + TR_BYTES;
constexpr int G_OFF_DYLO = G_OFF_YT + TR_BYTES;   // only with dy_lo
constexpr int g_off_hold(bool dylo) { return G_OFF_YT + TR_BYTES + (dylo ? TR_BYTES : 0); }
constexpr int g_off_wx(bool dylo) { return g_off_hold(dylo) + HOLD_BYTES / 2; }
constexpr int g_lds(bool dylo) { return g_off_wx(dylo) + g_nlds(dylo) * NWAVE * 64 * 16; }
static_assert(g_lds(false) <= 160 * 1024 && g_lds(true) <= 160 * 1024, "LDS of the gates kernel");


struct BwdArgs {
  Problem p;
  int G, ntile, R;
  u64 *rec;
  int *err;
  int swizzle;
  const unsigned short *wxf;              // W_x in fragment order (bwd_prep_kernel)
  unsigned short *dpo, *dqo;              // half precision [B][T][D]: S dp, S dq
  const float *sc;                        // sc[1] = S, sc[2] = 1 / S (launch_grad_scale)
  unsigned char *dxo;                     // S dxd, half precision, [B][ceil(T/4)][D][4 steps] (bf16 would break du:
                                          // it sums four taps of it with cancellation)
  float *part;                            // [B*G][3][D]: sums for db_a, db_x, dLambda
  const uint4 *rmask;                     // packed sequences: boundary bit masks per (sequence, tile), or NULL
};

// packs the low halves (sel = 0) or high halves (sel = 1) of two dwords of bf16 pairs
__device__ __forceinline__ unsigned pick_halves(unsigned lo_src, unsigned hi_src, int sel) {
  return sel ? __builtin_amdgcn_perm(hi_src, lo_src, 0x07060302u)   // hi16(hi_src) : hi16(lo_src)
             : __builtin_amdgcn_perm(hi_src, lo_src, 0x05040100u);  // lo16(hi_src) : lo16(lo_src)
}

// DYLO: the upstream gradient is dy + dy_lo, two bf16 tensors (16 significant bits)
// PACKED: the sequences hold several documents (BwdArgs.rmask): nothing crosses a document's
// first step - its h_{t-1} is zero, a_t delta_t does not reach the step before it, and the
// Conv1D takes the inputs in front of it as zeros. An instance of its own, so that the plain
// kernel keeps its register allocation.
template <int GMAX, bool DYLO = false, bool PACKED = false>
__global__ void __launch_bounds__(NTHR) __attribute__((amdgpu_waves_per_eu(2, 2)))
bwd_gates_kernel(BwdArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned short *xs = (unsigned short *)smem;
  f16x8 *sel_lds = (f16x8 *)(smem + G_OFF_CONST);
  f32x4 *cw_lds = (f32x4 *)(smem + G_OFF_CONST + 64 * 32);
  unsigned short *dyT = (unsigned short *)(smem + G_OFF_DYT);
  unsigned short *yT = (unsigned short *)(smem + G_OFF_YT);
  unsigned short *dyTlo = (unsigned short *)(smem + G_OFF_DYLO);
  float *hold = (float *)(smem + g_off_hold(DYLO));
  const Problem &p = a.p;
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5, j = lane & 31;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int G = GMAX == 1 ? 1 : a.G;

  int bid = blockIdx.x;
  if (GMAX > 1 && a.swizzle) {
    const int per = gridDim.x >> 3;
    bid = (bid & 7) * per + (bid >> 3);
  }
  const int unit = bid / G, w = bid - unit * G;
  const int b = unit / p.nb, g = unit - b * p.nb;
  const int D = p.D, T = p.T;
  const int ch = wv * 32 + j;
  const int d = g * BS + ch;

  // gate weights of this wave's 32 output channels: all of W_a and the first NRES K-steps of W_x
  // stay in registers, the next NLDS K-steps of W_x in LDS, and the rest is re-read from L2
  // every tile as contiguous 1 KB fragments (the register file cannot hold everything this
  // kernel needs, and L2 is a far better spill space than scratch)
  constexpr int NRES = (GMAX == 1 ? G_NRES + 1 : G_NRES) - (PACKED ? 2 : 0), NLDS = g_nlds(DYLO);   // (the masks of packed sequences take registers of their own)
  // (the products run in half precision, see w_to_f16; the streamed copy is already converted)
  f16x8 wa[16], wx[NRES];
  // fragment ks of this lane when streamed: pxs[ks * 64] (W_x in fragment order)
  const f16x8 *pxs = (const f16x8 *)a.wxf + (size_t)(g * NWAVE + wv) * 16 * 64 + lane;
  f16x8 *wxl = (f16x8 *)(smem + g_off_wx(DYLO)) + (size_t)wv * NLDS * 64 + lane;   // [K-step][lane]
  {
    const bf16x8 *pa = (const bf16x8 *)((const unsigned short *)p.W_a + ((size_t)g * BS + ch) * BS + hf * 8);
    const bf16x8 *px = (const bf16x8 *)((const unsigned short *)p.W_x + ((size_t)g * BS + ch) * BS + hf * 8);
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) wa[ks] = w_to_f16(pa[ks * 2]);
#pragma unroll
    for (int ks = 0; ks < NRES; ++ks) wx[ks] = w_to_f16(px[ks * 2]);
#pragma unroll
    for (int i = 0; i < NLDS; ++i) wxl[i * 64] = w_to_f16(px[(NRES + i) * 2]);   // read back by the same lane only
  }
  if (tid < 64) {
    f16x8 sel0, sel1;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      sel0[e] = (_Float16)((hf * 8 + e == j) ? 1.0f : 0.0f);
      sel1[e] = (_Float16)((hf * 8 + e + 16 == j) ? 1.0f : 0.0f);
    }
    sel_lds[lane] = sel0;
    sel_lds[64 + lane] = sel1;
  }
  const float bias_p = p.b_a[d] * LOG2E, bias_q = p.b_x[d] * LOG2E;
  const float S = a.sc[1], invS = a.sc[2];
  float kd, kd_ln, lam_scale;
  {
    const float z = -p.Lambda[d];
    const float sp = z > 0.f ? z + log1pf(expf(-z)) : log1pf(expf(z));  // softplus(-Lambda)
    kd_ln = -p.c * sp;
    kd = kd_ln * LOG2E;
    lam_scale = p.c / (1.f + expf(-z));  // c * sigmoid(-Lambda) = c * (1 - sigmoid(Lambda))
  }

  const int c2 = tid & 127;
  const int rg = __builtin_amdgcn_readfirstlane(tid >> 7);
  const int dc = g * BS + 2 * c2;
  if (tid < 128 && !p.conv_w) {   // no Conv1D: x_t = u_t
    cw_lds[c2] = f32x4{LOG2E, LOG2E, 0.f, 0.f};
    cw_lds[128 + c2] = f32x4{0.f, 0.f, 0.f, 0.f};
    cw_lds[256 + c2] = f32x4{0.f, 0.f, 0.f, 0.f};
  } else if (tid < 128) {
    f32x4 t0v, t1v, t2v;
    t0v[0] = p.conv_w[dc] * LOG2E;                  t0v[1] = p.conv_w[dc + 1] * LOG2E;
    t0v[2] = p.conv_w[(size_t)D + dc] * LOG2E;      t0v[3] = p.conv_w[(size_t)D + dc + 1] * LOG2E;
    t1v[0] = p.conv_w[(size_t)2 * D + dc] * LOG2E;  t1v[1] = p.conv_w[(size_t)2 * D + dc + 1] * LOG2E;
    t1v[2] = p.conv_w[(size_t)3 * D + dc] * LOG2E;  t1v[3] = p.conv_w[(size_t)3 * D + dc + 1] * LOG2E;
    t2v[0] = p.conv_b ? p.conv_b[dc] * LOG2E : 0.f;
    t2v[1] = p.conv_b ? p.conv_b[dc + 1] * LOG2E : 0.f;
    t2v[2] = t2v[3] = 0.f;
    cw_lds[c2] = t0v;
    cw_lds[128 + c2] = t1v;
    cw_lds[256 + c2] = t2v;
  }

  const unsigned seq_bytes = (unsigned)((size_t)T * D * 2);
  const unsigned row_bytes = (unsigned)D * 2;
  const size_t seq_off = (size_t)b * T * D;
  auto rsrc = [&](const void *base) {
    return __builtin_amdgcn_make_buffer_rsrc(uniform_ptr((const unsigned short *)base + seq_off), 0,
                                             seq_bytes, 0x00020000);
  };
  const __amdgpu_buffer_rsrc_t u_rsrc = rsrc(p.u), y_rsrc = rsrc(p.y_in), dy_rsrc = rsrc(p.dy);
  const __amdgpu_buffer_rsrc_t dyl_rsrc = rsrc(DYLO ? p.dy_lo : p.dy);
  const __amdgpu_buffer_rsrc_t dp_rsrc = rsrc(a.dpo), dq_rsrc = rsrc(a.dqo);
  // S dxd: [group of 4 steps][channel][8 bytes], four half-precision values
  const unsigned grp_bytes = (unsigned)D * 8, ngrp = (unsigned)(T + 3) / 4;
  const __amdgpu_buffer_rsrc_t dx_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      uniform_ptr(a.dxo + (size_t)b * ngrp * grp_bytes), 0, ngrp * grp_bytes, 0x00020000);
  const unsigned dx_voff = (unsigned)d * 8 + (unsigned)hf * 4 * grp_bytes;  // channel, lane half
  const unsigned c_voff = (unsigned)dc * 2;                                   // channel pair
  const unsigned o_voff = (unsigned)d * 2 + (unsigned)hf * 16 * row_bytes;    // channel, lane half
  const unsigned *st32 =
      p.state_in ? (const unsigned *)((const unsigned short *)p.state_in + (size_t)b * 3 * D + dc) : nullptr;

  unsigned raw[11];
  auto load_rows = [&](int t0) {
    const int tb = t0 + 8 * rg - 3;
    if (tb >= 0 && tb + 11 <= T) {
#pragma unroll
      for (int n = 0; n < 11; ++n)
        raw[n] = __builtin_amdgcn_raw_buffer_load_b32(u_rsrc, c_voff, (unsigned)(tb + n) * row_bytes, RGLRU_NT);
    } else {
#pragma unroll
      for (int n = 0; n < 11; ++n) {
        const int t = tb + n;
        unsigned v = 0;
        if (t >= 0) {
          if (t < T) v = __builtin_amdgcn_raw_buffer_load_b32(u_rsrc, c_voff, (unsigned)t * row_bytes, RGLRU_NT);
        } else if (st32) {
          v = st32[(size_t)ring_slot(p.pos0 + t) * (D / 2)];
        }
        raw[n] = v;
      }
    }
  };
  unsigned short *xw = xs + (8 * rg) * XS + 2 * c2;
  // Conv1D rows of this workgroup's next tile into the x tile (mk: the tile's mask word; packed
  // sequences drop the lags that reach in front of a row's document, a select per lag on a
  // scalar condition)
  auto conv_rows = [&](const u32x4 &mk) {
    const f32x4 w01 = cw_lds[c2], w23 = cw_lds[128 + c2], bb = cw_lds[256 + c2];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const int bit = 8 * rg + r;
      const unsigned v1 = (!PACKED || ((mk[1] >> bit) & 1u)) ? raw[r + 2] : 0u;
      const unsigned v2 = (!PACKED || ((mk[2] >> bit) & 1u)) ? raw[r + 1] : 0u;
      const unsigned v3 = (!PACKED || ((mk[3] >> bit) & 1u)) ? raw[r] : 0u;
      float x0 = bb[0], x1 = bb[1];
      x0 = fmaf(w01[0], bf_lo(raw[r + 3]), x0); x1 = fmaf(w01[1], bf_hi(raw[r + 3]), x1);
      x0 = fmaf(w01[2], bf_lo(v1), x0);         x1 = fmaf(w01[3], bf_hi(v1), x1);
      x0 = fmaf(w23[0], bf_lo(v2), x0);         x1 = fmaf(w23[1], bf_hi(v2), x1);
      x0 = fmaf(w23[2], bf_lo(v3), x0);         x1 = fmaf(w23[3], bf_hi(v3), x1);
      unsigned hi_pk, lo_pk;
      split_f16(x0, x1, hi_pk, lo_pk);
      *(unsigned *)(xw + r * XS) = hi_pk;
      *(unsigned *)(xw + XT_ELEMS + r * XS) = lo_pk;
    }
  };
  // dy and y rows 8*rg..8*rg+7 of tile t0 for the channel pair (zero past the sequence end)
  unsigned rdy[8], ry[8], ryh;   // ryh: the row before the tile (h_{t-1} of its first step)
  unsigned rdl[DYLO ? 8 : 1];
  // (no branch around the loads: rows past the end of the sequence are out of the descriptors'
  // range and read as zero; a conditional load would make the compiler wait for it on the spot)
  auto load_dy_y = [&](int t0) {
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const unsigned so = (unsigned)(t0 + 8 * rg + r) * row_bytes;
      rdy[r] = __builtin_amdgcn_raw_buffer_load_b32(dy_rsrc, c_voff, so, RGLRU_NT);
      ry[r] = __builtin_amdgcn_raw_buffer_load_b32(y_rsrc, c_voff, so, RGLRU_NT);
      if (DYLO) rdl[r] = __builtin_amdgcn_raw_buffer_load_b32(dyl_rsrc, c_voff, so, RGLRU_NT);
    }
    // (t0 = 0: the offset wraps to the top of the 32-bit range, far outside the descriptor,
    // and reads as zero; the lanes take h0 there instead)
    ryh = __builtin_amdgcn_raw_buffer_load_b32(y_rsrc, c_voff, (unsigned)(t0 - 1) * row_bytes, RGLRU_NT);
  };
  // transposed [channel][time] copies: 8 consecutive steps of one channel are 16 contiguous bytes
  auto park_dy_y = [&]() {
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      uint4 vd, vy;
      vd.x = pick_halves(rdy[0], rdy[1], c); vd.y = pick_halves(rdy[2], rdy[3], c);
      vd.z = pick_halves(rdy[4], rdy[5], c); vd.w = pick_halves(rdy[6], rdy[7], c);
      vy.x = pick_halves(ry[0], ry[1], c);   vy.y = pick_halves(ry[2], ry[3], c);
      vy.z = pick_halves(ry[4], ry[5], c);   vy.w = pick_halves(ry[6], ry[7], c);
      *(uint4 *)(dyT + (2 * c2 + c) * TS + 8 * rg) = vd;
      *(uint4 *)(yT + (2 * c2 + c) * TS + 8 * rg) = vy;
      if (DYLO) {
        uint4 vl;
        vl.x = pick_halves(rdl[0], rdl[1], c); vl.y = pick_halves(rdl[2], rdl[3], c);
        vl.z = pick_halves(rdl[4], rdl[5], c); vl.w = pick_halves(rdl[6], rdl[7], c);
        *(uint4 *)(dyTlo + (2 * c2 + c) * TS + 8 * rg) = vl;
      }
    }
    if (rg == 0) {   // the row before the tile goes to the spare column TS - 1 of the y tile
      yT[(2 * c2) * TS + TS - 1] = (unsigned short)(ryh & 0xffffu);
      yT[(2 * c2 + 1) * TS + TS - 1] = (unsigned short)(ryh >> 16);
    }
  };

  const float kdS = kd_ln * S;
  const int arow = ((j >> 2) & 1) * 16 + (j >> 3) * 4 + (j & 3);
  const unsigned short *arow_base = xs + arow * XS + hf * 8;
  f32x4 *hold_mine = (f32x4 *)hold + (size_t)wv * 4 * 64 + lane;
  const uint4 *dyT_mine = (const uint4 *)(dyT + ch * TS + hf * 16);
  const uint4 *yT_mine = (const uint4 *)(yT + ch * TS + hf * 16);
  const uint4 *dyTlo_mine = (const uint4 *)(dyTlo + ch * TS + hf * 16);

  u64 *ring = GMAX > 1 ? a.rec + (size_t)unit * a.R * 2 * BS + ch : nullptr;
  float carry = p.dhT ? p.dhT[(size_t)b * D + d] : 0.f;  // eps entering this workgroup's next tile
  const float h_first = p.h0 ? p.h0[(size_t)b * D + d] : 0.f;   // h_{-1}
  float s_ba = 0.f, s_bx = 0.f, s_lam = 0.f;
  // (a workspace that still reports an expired wait of an earlier call: no waiting, NaN throughout)
  int spins = (GMAX > 1 && expired_before(a.err)) ? SPIN_LIMIT : 0;

  // tiles are walked from the end of the sequence: this workgroup owns ntile-1-w, -G, ...
  int tile = a.ntile - 1 - w;
  // Mask words of packed sequences: lanes 0..3 fetch the four dwords of a tile's word two tiles
  // ahead, as the first load of an iteration, and the word reaches the scalar registers by lane
  // reads where the tile's rows are waited for anyway. Tiles outside the sequence read as zero.
  const __amdgpu_buffer_rsrc_t mk_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      uniform_ptr(PACKED ? (const void *)(a.rmask + (size_t)b * a.ntile) : (const void *)p.u), 0,
      PACKED ? (unsigned)a.ntile * 16u : 0u, 0x00020000);
  auto mask_fetch = [&](int tl) __attribute__((always_inline)) {
    return __builtin_amdgcn_raw_buffer_load_b32(mk_rsrc, (unsigned)(lane & 3) * 4u, (unsigned)tl * 16u, 0);
  };
  auto mask_word = [&](unsigned v) __attribute__((always_inline)) {
    u32x4 m;
    m[0] = __builtin_amdgcn_readlane(v, 0); m[1] = __builtin_amdgcn_readlane(v, 1);
    m[2] = __builtin_amdgcn_readlane(v, 2); m[3] = __builtin_amdgcn_readlane(v, 3);
    return m;
  };
  u32x4 mk0 = {0u, 0u, 0u, 0u};
  unsigned mv_next = 0u;
  if (PACKED && tile >= 0) {
    mk0 = mask_word(mask_fetch(tile));
    mv_next = mask_fetch(tile - G);
  }
  unsigned starts = mk0[0];   // steps of this iteration's tile that start a document
  if (tile >= 0) load_rows(tile * TT);
  __syncthreads();
  if (tile >= 0) conv_rows(mk0);
  if (tile >= 0) load_dy_y(tile * TT);
  __syncthreads();

  for (int it = 0; tile >= 0; tile -= G, ++it) {
    const int t0 = tile * TT;
    const int next = tile - G;
    unsigned mv_after = 0u;
    if (PACKED) mv_after = mask_fetch(next - G);
    const unsigned st16 = hf ? starts >> 16 : starts;   // this lane's 16 steps

    // ---- gate pre-activations on the matrix cores
    f32x16 accp, accq, accx;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      accp[r] = bias_p;
      accq[r] = bias_q;
      accx[r] = 0.f;
    }
    const unsigned short *ap = arow_base;
    {
      f16x8 a0 = *(const f16x8 *)(ap), a1 = *(const f16x8 *)(ap + 16);
      constexpr int NS = NRES + NLDS;                            // first streamed K-step
      f16x8 s0 = pxs[NS * 64], s1 = pxs[(NS + 1) * 64];          // streamed W_x fragments, two in flight
      f16x8 l0 = wxl[0];                                         // LDS-resident fragment, one ahead
#pragma unroll
      for (int ks = 0; ks < 16; ++ks) {
        const f16x8 a2 = *(const f16x8 *)(ap + ((ks + 2) & 15) * 16);
        accp = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, wa[ks], accp, 0, 0, 0);
        if (ks < NRES) {
          accq = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, wx[ks], accq, 0, 0, 0);
        } else if (ks < NS) {
          accq = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, l0, accq, 0, 0, 0);
          if (ks + 1 < NS) l0 = wxl[(ks + 1 - NRES) * 64];
        } else {
          accq = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, s0, accq, 0, 0, 0);
          s0 = s1;
          if (ks + 2 < 16) s1 = pxs[(ks + 2) * 64];
        }
        __builtin_amdgcn_sched_barrier(0);
        a0 = a1;
        a1 = a2;
      }
    }
    {
      const f16x8 s0 = *(const f16x8 *)(ap + (2 * wv) * 16);
      const f16x8 s1 = *(const f16x8 *)(ap + (2 * wv + 1) * 16);
      const f16x8 l0 = *(const f16x8 *)(ap + XT_ELEMS + (2 * wv) * 16);
      const f16x8 l1 = *(const f16x8 *)(ap + XT_ELEMS + (2 * wv + 1) * 16);
      accx = __builtin_amdgcn_mfma_f32_32x32x16_f16(s0, sel_lds[lane], accx, 0, 0, 0);
      accx = __builtin_amdgcn_mfma_f32_32x32x16_f16(s1, sel_lds[64 + lane], accx, 0, 0, 0);
      accx = __builtin_amdgcn_mfma_f32_32x32x16_f16(l0, sel_lds[lane], accx, 0, 0, 0);
      accx = __builtin_amdgcn_mfma_f32_32x32x16_f16(l1, sel_lds[64 + lane], accx, 0, 0, 0);
    }
    park_dy_y();
    if (next >= 0) load_rows(next * TT);  // consumed by conv_rows at the end of the iteration
    __syncthreads();

    // ---- first sweep (latest step first): r_t, a_t into LDS, aggregate of this lane's run:
    // eps_out = prun * eps_in + erun
    const int nvalid = T - t0 - hf * 16;  // steps of this lane's run inside the sequence
    float erun = 0.f, prun = 1.f;
#pragma unroll
    for (int q = 3; q >= 0; --q) {
      const uint4 dq4 = dyT_mine[q >> 1];
      const unsigned d01 = (q & 1) ? dq4.z : dq4.x, d23 = (q & 1) ? dq4.w : dq4.y;
      float dyv[4] = {bf_lo(d01), bf_hi(d01), bf_lo(d23), bf_hi(d23)};
      if (DYLO) {
        const uint4 dl4 = dyTlo_mine[q >> 1];
        const unsigned l01 = (q & 1) ? dl4.z : dl4.x, l23 = (q & 1) ? dl4.w : dl4.y;
        dyv[0] += bf_lo(l01); dyv[1] += bf_hi(l01); dyv[2] += bf_lo(l23); dyv[3] += bf_hi(l23);
      }
      f32x4 rq;
#pragma unroll
      for (int e = 3; e >= 0; --e) {
        const float ep = __builtin_amdgcn_exp2f(-accp[4 * q + e]);
        const float rv = __builtin_amdgcn_rcpf(1.f + ep);
        float av = __builtin_amdgcn_exp2f(kd * rv);
        if (4 * q + e >= nvalid) av = 1.f;  // past the end: eps passes through (dy is zero there)
        if (PACKED && ((st16 >> (4 * q + e)) & 1u)) av = 0.f;   // nothing flows out of a document's first step
        erun = av * (dyv[e] + erun);
        prun *= av;
        rq[e] = rv;
      }
      hold_mine[q * 64] = rq;
    }
    // ---- combine the lane halves; the upper half (later steps) is applied first
    const float oA = __shfl_xor(prun, 32), oE = __shfl_xor(erun, 32);
    const float A_up = hf ? prun : oA, E_up = hf ? erun : oE;
    const float A_lo = hf ? oA : prun, E_lo = hf ? oE : erun;
    const float A_t = A_lo * A_up, E_t = fmaf(A_lo, E_up, E_lo);

    float e_in = carry;
    if (GMAX > 1) {
      publish(ring + (size_t)(tile % a.R) * 2 * BS + hf * BS, hf ? E_t : A_t, (unsigned)(tile + 1));
      // eps entering this tile: own state after tile+G carried across tiles tile+G-1 .. tile+1.
      // Each lane half fetches one of a tile's two records (A below, E above; the halves swap
      // them afterwards), four tiles per round trip; a tag that is not there yet is simply
      // read again.
      constexpr int NB = 4;
#pragma unroll
      for (int s0 = GMAX - 2; s0 >= 0; s0 -= NB) {
        u64 rec[NB];
#pragma unroll
        for (int i = 0; i < NB; ++i) {
          const int s = s0 - i, k = tile + 1 + s;
          if (s >= 0 && s < G - 1 && k < a.ntile) rec[i] = peek(ring + (size_t)(k % a.R) * 2 * BS + hf * BS);
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
          const int s = s0 - i, k = tile + 1 + s;
          if (s >= 0 && s < G - 1 && k < a.ntile) {
            const u64 *slot = ring + (size_t)(k % a.R) * 2 * BS + hf * BS;
            const unsigned want = (unsigned)(k + 1);
            while ((unsigned)(rec[i] >> 32) != want && spins < SPIN_LIMIT) {
              ++spins;
              __builtin_amdgcn_s_sleep(2);
              rec[i] = peek(slot);
            }
            if (spins < SPIN_LIMIT) spins = 0;   // the limit is per wait; an expired wait stays expired
            const float mine = __uint_as_float((unsigned)rec[i]), other = __shfl_xor(mine, 32);
            e_in = fmaf(hf ? other : mine, e_in, hf ? mine : other);
          }
        }
      }
    }
    // a wait that expired: this channel's results are NaN from here on, visibly invalid
    if (GMAX > 1 && (spins >= SPIN_LIMIT || __shfl_xor(spins, 32) >= SPIN_LIMIT)) e_in = __builtin_nanf("");
    carry = fmaf(A_t, e_in, E_t);

    // ---- second sweep: adjoints with the true eps, latest step first
    float erev = hf ? e_in : fmaf(A_up, e_in, E_up);  // eps_{t+1} for the last step of this run
    const unsigned so = (unsigned)t0 * row_bytes;
#pragma unroll
    for (int q = 3; q >= 0; --q) {
      const uint4 dq4 = dyT_mine[q >> 1], yq4 = yT_mine[q >> 1];
      const unsigned d01 = (q & 1) ? dq4.z : dq4.x, d23 = (q & 1) ? dq4.w : dq4.y;
      const unsigned y01 = (q & 1) ? yq4.z : yq4.x, y23 = (q & 1) ? yq4.w : yq4.y;
      float dyv[4] = {bf_lo(d01), bf_hi(d01), bf_lo(d23), bf_hi(d23)};
      if (DYLO) {
        const uint4 dl4 = dyTlo_mine[q >> 1];
        const unsigned l01 = (q & 1) ? dl4.z : dl4.x, l23 = (q & 1) ? dl4.w : dl4.y;
        dyv[0] += bf_lo(l01); dyv[1] += bf_hi(l01); dyv[2] += bf_lo(l23); dyv[3] += bf_hi(l23);
      }
      const float yv[4] = {bf_lo(y01), bf_hi(y01), bf_lo(y23), bf_hi(y23)};
      const f32x4 rq = hold_mine[q * 64];
      // h_{t-1} of the quad's first step: the step before it in the y tile (the spare column
      // for the first step of the tile, h0 for the first step of the sequence)
      const int pcol = q == 0 ? (hf ? 15 : TS - 1) : hf * 16 + 4 * q - 1;
      float hfirst = bf_lo((unsigned)yT[ch * TS + pcol]);
      if (q == 0 && hf == 0 && tile == 0) hfirst = h_first;
      float dpv[4], dqv[4], dxv[4];
#pragma unroll
      for (int e = 3; e >= 0; --e) {
        const float rv = rq[e];
        const float l2 = kd * rv;
        const float av = __builtin_amdgcn_exp2f(l2);
        const bool ok = 4 * q + e < nvalid;
        const float delta = ok ? dyv[e] + erev : 0.f;
        // (a gate closed so far that r_t = 0 in fp32 gives m = 0: the floor keeps 1/m finite,
        // and the terms it scales carry the factor r_t (1 - r_t) = 0)
        const float m2 = fmaxf(one_minus_sq(av, l2), 1e-30f);
        const float rs = __builtin_amdgcn_rsqf(m2);       // 1 / m
        const float m = m2 * rs;
        const float eq = __builtin_amdgcn_exp2f(-accq[4 * q + e]);
        const float iv = __builtin_amdgcn_rcpf(1.f + eq);
        const float gin = iv * (accx[4 * q + e] * LN2);   // i_t x_t
        const bool fresh = PACKED && ((st16 >> (4 * q + e)) & 1u);   // a document's first step: h_{t-1} = 0
        const float hprev = fresh ? 0.f : (e > 0 ? yv[e - 1] : hfirst);
        const float dla = (delta * av) * fmaf(-av * gin, rs, hprev);   // delta a (h_{t-1} - a g/m)
        const float dg = delta * m;
        const float dxu = dg * iv;
        dxv[e] = dxu * S;
        const float dqu = dg * gin * (1.f - iv);
        dqv[e] = dqu * S;
        dpv[e] = (kdS * dla) * fmaf(-rv, rv, rv);   // S dp
        s_lam = fmaf(dla, rv, s_lam);
        s_ba += dpv[e];                             // (unscaled at the end)
        s_bx += dqu;
        erev = ok ? (fresh ? 0.f : av * delta) : erev;
      }
      // S dp, S dq (half precision): one 64-byte piece of a row per lane half and step
      {
        const unsigned p0 = pack_f16(dpv[0], dpv[1]), p1 = pack_f16(dpv[2], dpv[3]);
        const unsigned q0 = pack_f16(dqv[0], dqv[1]), q1 = pack_f16(dqv[2], dqv[3]);
        const unsigned soq = so + (unsigned)(4 * q) * row_bytes;
        const int nv = nvalid - 4 * q;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (e < nv) {
            const unsigned pp = e < 2 ? p0 : p1, qq = e < 2 ? q0 : q1;
            const short sp = (short)((e & 1) ? (pp >> 16) : (pp & 0xffff));
            const short sq = (short)((e & 1) ? (qq >> 16) : (qq & 0xffff));
            __builtin_amdgcn_raw_buffer_store_b16(sp, dp_rsrc, o_voff, soq + e * row_bytes, RGLRU_NT);
            __builtin_amdgcn_raw_buffer_store_b16(sq, dq_rsrc, o_voff, soq + e * row_bytes, RGLRU_NT);
          }
        }
      }
      // S dxd: the four steps in half precision (zero past the end of the sequence), 8 bytes per
      // lane, 256 contiguous bytes per lane half
      if (4 * q < nvalid) {
        typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
        u32x2 w;
        w[0] = pack_f16(dxv[0], dxv[1]);
        w[1] = pack_f16(dxv[2], dxv[3]);
        __builtin_amdgcn_raw_buffer_store_b64(w, dx_rsrc, dx_voff, (unsigned)(t0 / 4 + q) * grp_bytes, RGLRU_NT);
      }
    }

    u32x4 mkn = {0u, 0u, 0u, 0u};
    if (PACKED) mkn = mask_word(mv_next);
    starts = mkn[0];
    mv_next = mv_after;
    if (next >= 0) {
      conv_rows(mkn);
      // dy and y of the next tile: requested before the barrier, so that part of the trip to HBM
      // is over when the streamed weight fragments of the next product queue up behind it
      load_dy_y(next * TT);
    }
    __syncthreads();
  }
  if (GMAX > 1 && spins >= SPIN_LIMIT) mark_expired(a.err);

  // per-channel sums of this workgroup (both lane halves hold the same channel)
  s_ba += __shfl_xor(s_ba, 32);
  s_bx += __shfl_xor(s_bx, 32);
  s_lam += __shfl_xor(s_lam, 32);
  if (hf == 0) {
    float *pp = a.part + ((size_t)(b * G + w) * 3) * D + d;
    pp[0] = s_ba * invS;
    pp[D] = s_bx;
    pp[2 * (size_t)D] = s_lam * lam_scale;
    // the workgroup that ran tile 0 holds eps_0 = dL/dh0
    if (p.dh0 && (a.ntile - 1 - w) % G == 0) p.dh0[(size_t)b * D + d] = carry;
  }
}


// ------------------------------------------------------------------------------ dgrad
// A tile: 32 steps x (S dp 256 | S dq 256) half precision, filled by direct-to-LDS loads (layout below);
// two of them, two u tiles of 35 rows, the selection fragments, and a staging tile per wave that
// turns the du columns into 16-byte stores. Few, wide memory instructions matter here: a
// compute unit issues roughly one vector memory instruction per 8 cycles, whatever its width
// (as long as the lanes of one instruction touch few cache lines).
constexpr int AS = 2 * BS + 8;                       // slot stride in elements (1040 B)
constexpr int D_A_TILE = TT * AS * 2;                // one A tile: 16 dp slots, then 16 dq slots
constexpr int D_A_BYTES = 2 * D_A_TILE;              // two A tiles
constexpr int US_ROWS = TT + 3;                      // u rows t0-3 .. t0+31
constexpr int D_OFF_SEL = D_A_BYTES;
constexpr int D_OFF_U = D_OFF_SEL + 64 * 32;
constexpr int D_U_TILE = US_ROWS * XS * 2;
constexpr int D_OFF_OT = D_OFF_U + 2 * D_U_TILE;     // per wave: du staging tile [32][OT] bf16
constexpr int D_LDS = D_OFF_OT + NWAVE * OTILE_BYTES;

struct DgradArgs {
  Problem p;
  int C, ntile;                            // contiguous time chunks per unit, tiles per sequence
  const unsigned short *dpo, *dqo;         // half precision [B][T][D]: S dp, S dq
  const float *sc;                         // sc[2] = 1 / S
  const unsigned char *dxo;                // S dxd, half precision [B][ceil(T/4)][D][4 steps]
  const unsigned short *wta, *wtx;         // transposed gate weights [nb][in k][out j], half precision
  float *part;                             // [B*C][5][D]: dconv_w[0..3], dconv_b partial sums
  const uint4 *rmask;                      // packed sequences: boundary bit masks per (sequence, tile), or NULL
};

// Preparation pass of the backward: the first 128 nb blocks transpose W_a and W_x in 32 x 32
// tiles for the dgrad kernel; the others clear the record rings and copy W_x into MFMA
// fragment order, [block][wave][K-step][lane][8], so that the gates kernel re-reads the K-steps
// it cannot keep in registers as contiguous 1 KB pieces.
struct PrepArgs {
  const unsigned short *Wa, *Wx;
  unsigned short *WTa, *WTx;
  uint4 *wxf;
  uint4 *zero;
  size_t n16;   // 16-byte words to clear
  int nb;
};
__global__ void __launch_bounds__(256) bwd_prep_kernel(PrepArgs a) {
  __shared__ unsigned short tile[32][33];
  const int nT = 128 * a.nb;
  if ((int)blockIdx.x < nT) {
    const int t = blockIdx.x & 63, mz = blockIdx.x >> 6;
    const int m = mz % a.nb, which = mz / a.nb;
    const int bx = (t & 7) * 32, by = (t >> 3) * 32;
    const unsigned short *src = (which ? a.Wx : a.Wa) + (size_t)m * BS * BS;
    unsigned short *dst = (which ? a.WTx : a.WTa) + (size_t)m * BS * BS;
    for (int i = threadIdx.x; i < 32 * 32; i += 256) {
      const int r = i >> 5, c = i & 31;
      tile[r][c] = src[(size_t)(by + r) * BS + bx + c];
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 32 * 32; i += 256) {
      const int r = i >> 5, c = i & 31;
      // (in half precision: exact for bf16 weights from 6.1e-5 up)
      const float wv_ = __uint_as_float((unsigned)tile[c][r] << 16);
      dst[(size_t)(bx + r) * BS + by + c] = (unsigned short)(pack_f16(wv_, 0.f) & 0xffffu);
    }
    return;
  }
  const size_t i = (size_t)(blockIdx.x - nT) * 256 + threadIdx.x;
  if (i < a.n16) a.zero[i] = cleared_word(a.zero, i, true);
  if (i < (size_t)a.nb * BS * BS / 8) {
    const int lane = (int)(i & 63), ks = (int)((i >> 6) & 15), wv = (int)((i >> 10) & 7), g = (int)(i >> 13);
    const int hf = lane >> 5, j = lane & 31;
    // (in half precision: the gates kernel's products run on the f16 form of the MFMA)
    const uint4 w = ((const uint4 *)a.Wx)[((size_t)g * BS + wv * 32 + j) * (BS / 8) + ks * 2 + hf];
    a.wxf[i] = make_uint4(pack_f16(bf_lo(w.x), bf_hi(w.x)), pack_f16(bf_lo(w.y), bf_hi(w.y)),
                          pack_f16(bf_lo(w.z), bf_hi(w.z)), pack_f16(bf_lo(w.w), bf_hi(w.w)));
  }
}

// PACKED: the sequences hold several documents (DgradArgs.rmask): lag k of step t counts only
// while step t - k belongs to t's document, in du and in the tap gradients alike.
template <bool PACKED = false>
__global__ void __launch_bounds__(NTHR) __attribute__((amdgpu_waves_per_eu(2, 2)))
bwd_dgrad_kernel(DgradArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned short *as = (unsigned short *)smem;                       // [2] A tiles
  bf16x8 *sel_lds = (bf16x8 *)(smem + D_OFF_SEL);
  unsigned short *us = (unsigned short *)(smem + D_OFF_U);           // [2][35][XS]
  const Problem &p = a.p;
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5, j = lane & 31;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int unit = blockIdx.x / a.C, c = blockIdx.x - unit * a.C;
  const int b = unit / p.nb, g = unit - b * p.nb;
  const int D = p.D, T = p.T;
  const int ch = wv * 32 + j;   // input channel (column of the gate matrices) owned by this lane
  const int d = g * BS + ch;

  // transposed weights of this wave's 32 columns: B operand rows are output channels
  const float invS = a.sc[2];
  f16x8 wa[16], wx[16];
  {
    const f16x8 *pa = (const f16x8 *)(a.wta + ((size_t)g * BS + ch) * BS + hf * 8);
    const f16x8 *px = (const f16x8 *)(a.wtx + ((size_t)g * BS + ch) * BS + hf * 8);
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) {
      wa[ks] = pa[ks * 2];
      wx[ks] = px[ks * 2];
    }
  }
  if (tid < 64) {
    bf16x8 sel0, sel1;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      sel0[e] = (__bf16)((hf * 8 + e == j) ? 1.0f : 0.0f);
      sel1[e] = (__bf16)((hf * 8 + e + 16 == j) ? 1.0f : 0.0f);
    }
    sel_lds[lane] = sel0;
    sel_lds[64 + lane] = sel1;
  }
  float cw[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) cw[k] = p.conv_w ? p.conv_w[(size_t)k * D + d] : (k == 0 ? 1.f : 0.f);

  const unsigned seq_bytes = (unsigned)((size_t)T * D * 2);
  const unsigned row_bytes = (unsigned)D * 2;
  const size_t seq_off = (size_t)b * T * D;
  auto rsrc = [&](const void *base) {
    return __builtin_amdgcn_make_buffer_rsrc(uniform_ptr((const unsigned short *)base + seq_off), 0,
                                             seq_bytes, 0x00020000);
  };
  const __amdgpu_buffer_rsrc_t u_rsrc = rsrc(p.u), du_rsrc = rsrc(p.du);
  const __amdgpu_buffer_rsrc_t dp_rsrc = rsrc(a.dpo), dq_rsrc = rsrc(a.dqo);
  // this wave's du staging tile; lane l stores 8 channels of rows l/4 and l/4 + 16
  unsigned short *otile = (unsigned short *)(smem + D_OFF_OT) + wv * (OTILE_BYTES / 2);
  unsigned short *ot_mine = otile + (hf * 16) * OT + j;
  const unsigned du_voff = (unsigned)(g * BS + wv * 32 + (lane & 3) * 8) * 2 + (unsigned)(lane >> 2) * row_bytes;

  // A tiles go from global memory straight into LDS, 16 bytes per lane: one instruction lays
  // 1024 contiguous bytes, the 256 channels of row r (lanes 0-31) and of row r+8 (lanes 32-63)
  // of one array. Slot s = (r & 7) + 8 (r >> 4) holds that pair; rows r and r+8 never meet in
  // one 16-lane group of the fragment reads, so the 1040-byte slot stride keeps them apart in
  // the banks. Rows past the end of the sequence are out of the buffer's range and read as zero.
  const unsigned a_voff = (unsigned)(g * BS + 8 * (lane & 31)) * 2 + (unsigned)(lane >> 5) * 8 * row_bytes;
  auto load_a = [&](int buf, int t0) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int sl = wv * 2 + i, r0 = (sl & 7) + (sl >> 3) * 16;
      const unsigned so = (unsigned)(t0 + r0) * row_bytes;
      unsigned char *dst = smem + buf * D_A_TILE + sl * (AS * 2);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(dp_rsrc, (__attribute__((address_space(3))) void *)dst, 16, a_voff, so, 0, RGLRU_NT);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(dq_rsrc, (__attribute__((address_space(3))) void *)(dst + D_A_TILE / 2), 16, a_voff, so, 0, RGLRU_NT);
    }
  };
  // S dxd of this lane's run (channel d, 16 consecutive steps): four groups of four half-precision
  // values, 8 bytes each; groups past the end of the sequence are out of range and read as zero
  const unsigned grp_bytes = (unsigned)D * 8, ngrp = (unsigned)(T + 3) / 4;
  const __amdgpu_buffer_rsrc_t dx_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      uniform_ptr(a.dxo + (size_t)b * ngrp * grp_bytes), 0, ngrp * grp_bytes, 0x00020000);
  const unsigned dx_voff = (unsigned)d * 8 + (unsigned)hf * 4 * grp_bytes;
  typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
  u32x2 dxw[4];
  // (no branches around these loads, see load_u below; `ok` false pushes them all out of range)
  auto load_dxd = [&](int t0, bool ok) {
    const unsigned vo = ok ? dx_voff : 0x80000000u;
    const unsigned so = ok ? (unsigned)(t0 / 4) * grp_bytes : 0u;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      dxw[q] = __builtin_amdgcn_raw_buffer_load_b64(dx_rsrc, vo, so + (unsigned)q * grp_bytes, RGLRU_NT);
  };
  auto dxd_at = [&](int r) __attribute__((always_inline)) {   // S dxd at step r of the run, in fp32
    const unsigned pair = dxw[r >> 2][(r >> 1) & 1];
    return (r & 1) ? f16_hi(pair) : f16_lo(pair);
  };
  // u rows t0-3 .. t0+31 (35 rows), 16 bytes (8 channels) per thread: rows lr, lr+16 and
  // (for lr < 3) lr+32
  const int lc = tid & 31, lr = tid >> 5;
  const unsigned u_voff = (unsigned)(g * BS + 8 * lc) * 2;
  const unsigned *st32 =
      p.state_in ? (const unsigned *)((const unsigned short *)p.state_in + (size_t)b * 3 * D + g * BS + 8 * lc)
                 : nullptr;
  uint4 ru[3];
  // No branches around the loads: a loaded value that meets a zero in a phi makes the compiler
  // wait for it on the spot, and that wait drains every outstanding load (a trip to HBM, three
  // times per tile). Rows past the end of the sequence and the row slots past 35 are pushed
  // out of the descriptor's range instead and read as zero; only the tile at t = 0, whose first
  // three rows come from the carried-in state, takes the branchy path.
  auto load_u = [&](int t0, bool ok) {
    if (t0 > 0 || !ok) {
      const unsigned so = ok ? (unsigned)(t0 - 3) * row_bytes : 0u;
#pragma unroll
      for (int h = 0; h < 3; ++h) {
        const int rho = lr + 16 * h;
        const unsigned vo = (ok && rho < US_ROWS) ? u_voff + (unsigned)rho * row_bytes : 0x80000000u;
        ru[h] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(u_rsrc, vo, so, RGLRU_NT));
      }
    } else {
#pragma unroll
      for (int h = 0; h < 3; ++h) {
        const int rho = lr + 16 * h, t = t0 - 3 + rho;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (rho < US_ROWS) {
          if (t >= 0) {
            if (t < T) v = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(u_rsrc, u_voff, (unsigned)t * row_bytes, RGLRU_NT));
          } else if (st32) {
            v = *(const uint4 *)(st32 + (size_t)ring_slot(p.pos0 + t) * (D / 2));
          }
        }
        ru[h] = v;
      }
    }
  };
  auto park_u = [&](int ub) {
#pragma unroll
    for (int h = 0; h < 3; ++h) {
      const int rho = lr + 16 * h;
      if (rho < US_ROWS) *(uint4 *)(us + ub * (D_U_TILE / 2) + rho * XS + 8 * lc) = ru[h];
    }
  };

  const int arow = ((j >> 2) & 1) * 16 + (j >> 3) * 4 + (j & 3);
  const unsigned short *arow_base = as + ((arow & 7) + (arow >> 4) * 8) * AS + ((arow >> 3) & 1) * BS + hf * 8;
  const unsigned short *urow_base = us + (arow + 3) * XS + (2 * wv) * 16 + hf * 8;

  // this workgroup's tiles [lo, hi), walked backwards; tile hi (if any) only supplies the
  // three dx rows that the Conv1D adjoint of tile hi-1 reaches into
  const int per = (a.ntile + a.C - 1) / a.C;
  const int lo = c * per, hi = min(a.ntile, lo + per);
  float sw[4] = {0.f, 0.f, 0.f, 0.f}, sb = 0.f;
  float nx0 = 0.f, nx1 = 0.f, nx2 = 0.f;  // dx at the first three steps of the next tile (upper half lanes)
  if (lo < hi) {
    // One barrier per tile. Everything a tile needs from memory is requested a whole iteration
    // ahead, right after the barrier of the tile before it: the A tile two tiles on (into the
    // buffer whose last readers have just passed that barrier), dxd and u of the next tile (into
    // the registers just consumed). The barrier's wait for outstanding loads therefore finds
    // them done. The u tile is double-buffered so that the taps' sums of one tile may still read
    // it while the next tile is parked.
    int tile = hi < a.ntile ? hi : hi - 1;
    // mask words of packed sequences (lag masks y, z, w of a tile's word): fetched by lanes 0..3 an
    // iteration ahead with the other loads, read into scalar registers at the top of the next one
    const __amdgpu_buffer_rsrc_t mk_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        uniform_ptr(PACKED ? (const void *)(a.rmask + (size_t)b * a.ntile) : (const void *)p.u), 0,
        PACKED ? (unsigned)a.ntile * 16u : 0u, 0x00020000);
    auto mask_fetch = [&](int tl) __attribute__((always_inline)) {
      return __builtin_amdgcn_raw_buffer_load_b32(mk_rsrc, (unsigned)(lane & 3) * 4u, (unsigned)tl * 16u, 0);
    };
    unsigned mv = 0u, lnext[4] = {0u, 0u, 0u, 0u};   // word of this iteration's tile (lanes 0..3); the tile after it
    if (PACKED) {
      const unsigned v = mask_fetch(tile + 1);
#pragma unroll
      for (int k = 1; k < 4; ++k) lnext[k] = __builtin_amdgcn_readlane(v, k);
      mv = mask_fetch(tile);
    }
    load_a(0, tile * TT);
    if (tile > lo) load_a(1, (tile - 1) * TT);
    load_dxd(tile * TT, true);
    load_u(tile * TT, tile != hi);
    __syncthreads();
    for (int it = 0; tile >= lo; --tile, ++it) {
      const int buf = it & 1, t0 = tile * TT;
      const bool halo = tile == hi;
      unsigned lcur[4] = {0u, ~0u, ~0u, ~0u};
      if (PACKED) {
#pragma unroll
        for (int k = 1; k < 4; ++k) lcur[k] = __builtin_amdgcn_readlane(mv, k);
      }

      f32x16 acc0, acc1;
#pragma unroll
      for (int r = 0; r < 16; ++r) acc0[r] = acc1[r] = 0.f;
      const unsigned short *ap = arow_base + buf * (D_A_TILE / 2);
      {
        constexpr int DQ = D_A_TILE / 4;   // dq slots, in elements
        f16x8 a0 = *(const f16x8 *)(ap), a1 = *(const f16x8 *)(ap + DQ);
#pragma unroll
        for (int ks = 0; ks < 16; ++ks) {
          const f16x8 n0 = *(const f16x8 *)(ap + ((ks + 1) & 15) * 16);
          const f16x8 n1 = *(const f16x8 *)(ap + DQ + ((ks + 1) & 15) * 16);
          acc0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, wa[ks], acc0, 0, 0, 0);
          acc1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, wx[ks], acc1, 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          a0 = n0;
          a1 = n1;
        }
      }
      float dx[19];
#pragma unroll
      for (int r = 0; r < 16; ++r) dx[r] = (acc0[r] + acc1[r] + dxd_at(r)) * invS;
      // steps 16..18 of this lane's run: the other half's first three (lower lanes) or the
      // next tile's first three (upper lanes)
      const float s0v = __shfl_xor(dx[0], 32), s1v = __shfl_xor(dx[1], 32), s2v = __shfl_xor(dx[2], 32);
      dx[16] = hf ? nx0 : s0v;
      dx[17] = hf ? nx1 : s1v;
      dx[18] = hf ? nx2 : s2v;
      nx0 = s0v; nx1 = s1v; nx2 = s2v;
      if (!halo) park_u(buf);
      __syncthreads();
      if (tile - 2 >= lo) load_a(buf, t0 - 2 * TT);
      load_dxd(t0 - TT, tile > lo);   // (nothing left to fetch after the last tile: out of range, zeros)
      load_u(t0 - TT, tile > lo);
      if (PACKED) mv = mask_fetch(tile - 1);
      // lag masks of the 19 steps from this lane's first: bit i = step 16 hf + i (the steps past
      // the tile are the next tile's first three)
      unsigned wk[4] = {0u, 0u, 0u, 0u};
      // (the packed instance masks every tile: the selects are cheap next to this kernel's memory
      // traffic, and a second copy of the sums for tiles without a boundary costs registers)
      constexpr bool plain = !PACKED;
      if (PACKED) {
#pragma unroll
        for (int k = 1; k < 4; ++k) wk[k] = hf ? ((lcur[k] >> 16) | (lnext[k] << 16)) : lcur[k];
      }
      if (!halo) {
        // Conv1D adjoint towards the input; the wave's [32 steps][32 channels] results leave
        // through its staging tile as 16-byte stores
        if (plain) {
#pragma unroll
          for (int r = 0; r < 16; r += 2) {
            float v0 = cw[0] * dx[r], v1 = cw[0] * dx[r + 1];
#pragma unroll
            for (int k = 1; k < 4; ++k) {
              v0 = fmaf(cw[k], dx[r + k], v0);
              v1 = fmaf(cw[k], dx[r + 1 + k], v1);
            }
            const unsigned pk = pack_bf16(v0, v1);
            ot_mine[r * OT] = (unsigned short)(pk & 0xffff);
            ot_mine[(r + 1) * OT] = (unsigned short)(pk >> 16);
          }
        } else {   // x_{t+k} sees u_t only while t lies in its document
#pragma unroll
          for (int r = 0; r < 16; r += 2) {
            float v0 = cw[0] * dx[r], v1 = cw[0] * dx[r + 1];
#pragma unroll
            for (int k = 1; k < 4; ++k) {
              v0 = fmaf(cw[k], ((wk[k] >> (r + k)) & 1u) ? dx[r + k] : 0.f, v0);
              v1 = fmaf(cw[k], ((wk[k] >> (r + 1 + k)) & 1u) ? dx[r + 1 + k] : 0.f, v1);
            }
            const unsigned pk = pack_bf16(v0, v1);
            ot_mine[r * OT] = (unsigned short)(pk & 0xffff);
            ot_mine[(r + 1) * OT] = (unsigned short)(pk >> 16);
          }
        }
        // (cached normally: two waves' 64-byte pieces make up a line, and as non-temporal stores they
        // reached memory separately - 35 % more bytes written than du has, 3 % of this kernel's time)
        store_staged_tile_s<OT, 0>(otile, lane, du_rsrc, du_voff, (unsigned)t0 * row_bytes, row_bytes, T - t0);
        // Conv1D adjoint towards the taps: u_{t-k} in accumulator layout by selection
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          f32x16 au;
#pragma unroll
          for (int r = 0; r < 16; ++r) au[r] = 0.f;
          const unsigned short *up = urow_base + buf * (D_U_TILE / 2) - k * XS;
          au = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(up), sel_lds[lane], au, 0, 0, 0);
          au = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(up + 16), sel_lds[64 + lane], au, 0, 0, 0);
          if (k == 0 || plain) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sw[k] = fmaf(dx[r], au[r], sw[k]);
          } else {
#pragma unroll
            for (int r = 0; r < 16; ++r) sw[k] = fmaf(((wk[k] >> r) & 1u) ? dx[r] : 0.f, au[r], sw[k]);
          }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) sb += dx[r];
      }
      if (PACKED) {
#pragma unroll
        for (int k = 1; k < 4; ++k) lnext[k] = lcur[k];
      }
    }
  }
  // partial sums of this workgroup
#pragma unroll
  for (int k = 0; k < 4; ++k) sw[k] += __shfl_xor(sw[k], 32);
  sb += __shfl_xor(sb, 32);
  if (hf == 0) {
    float *pp = a.part + ((size_t)(b * a.C + c) * 5) * D + d;
#pragma unroll
    for (int k = 0; k < 4; ++k) pp[(size_t)k * D] = sw[k];
    pp[(size_t)4 * D] = sb;
  }
}


// ------------------------------------------------------------------------------ wgrad
// One workgroup accumulates a 256 x 256 block dW[gate][g] over a slice of the B*T rows.
// Wave (mw, nw) owns output rows 64*mw.. (2 blocks of 32) and columns 128*nw.. (4 blocks).
// The product contracts over time, so a fragment is 8 consecutive steps of one channel.
// x is rebuilt here from u with the Conv1D of Section 2.3 (cheaper than a round trip of x
// through HBM): a thread produces 8 consecutive steps of a channel pair in half precision and
// lays them into a [channel][time] tile, where a fragment is one 16-byte read. S dp (or S dq)
// arrives as the [time][channel] half-precision rows the gates kernel wrote; a selection MFMA
// turns a 32-channel column block of it into (channel, 16 consecutive steps) registers, which
// packed to half precision again (exactly) are the fragments of the other operand. Both
// operands carry 11 significant bits; the factor S is taken out by the finishing pass.
constexpr int W_TILE = TT * XS * 2;          // dp or dq: one [32 steps][264] 16-bit tile
constexpr int W_XT = BS * TS * 2;            // x: one [256 channels][40] half-precision tile, time fastest
constexpr int W_BUF = W_TILE + W_XT;         // one buffer: dp|dq tile, x tile
constexpr int W_OFF_SEL = 2 * W_BUF;
constexpr int W_OFF_CW = W_OFF_SEL + 64 * 32;
constexpr int W_LDS = W_OFF_CW + 128 * 48;   // Conv1D taps and bias per channel pair

struct WgradArgs {
  int nb, S, D, T;
  long long rows;                           // B*T
  long long pos0;
  const unsigned short *dpo, *dqo;          // half precision [rows][D]: S dp, S dq
  const unsigned short *u;                  // bf16 [rows][D]
  const unsigned short *state_in;           // bf16 [B][3][D] ring, or NULL
  const float *conv_w, *conv_b;             // [4][D], [D] or NULL
  float *part;                              // [S][2][nb][256][256]
  const unsigned char *nlag;                // packed sequences: [rows] largest Conv1D lag inside the row's document, or NULL
};

// PACKED: the sequences hold several documents (WgradArgs.nlag): x is rebuilt with the lags that
// reach in front of a row's document dropped.
template <bool PACKED = false>
__global__ void __launch_bounds__(NTHR) __attribute__((amdgpu_waves_per_eu(2, 2)))
bwd_wgrad_kernel(WgradArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  f16x8 *sel_lds = (f16x8 *)(smem + W_OFF_SEL);
  f32x4 *cw_lds = (f32x4 *)(smem + W_OFF_CW);
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5, j = lane & 31;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int mw = wv >> 1, nw = wv & 1;
  // block id -> (slice s, gate, block g). Consecutive ids are dealt to the 8 XCDs in turn, so
  // the two gates of a (g, s) pair get ids 8 apart: same XCD, started together, and the u rows
  // one of them fetches are found in that XCD's L2 by the other.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int gate = slot & 1, pair = (slot >> 1) * 8 + xcd;
  if (pair >= a.S * a.nb) return;
  const int s = pair / a.nb, g = pair - s * a.nb;
  const unsigned short *src = gate ? a.dqo : a.dpo;
  const int D = a.D, T = a.T;

  if (tid < 64) {
    f16x8 sel0, sel1;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      sel0[e] = (_Float16)((hf * 8 + e == j) ? 1.0f : 0.0f);
      sel1[e] = (_Float16)((hf * 8 + e + 16 == j) ? 1.0f : 0.0f);
    }
    sel_lds[lane] = sel0;
    sel_lds[64 + lane] = sel1;
  }
  // Conv1D assignment: channel pair c2, rows 8*rg .. 8*rg+7 of the tile
  const int c2 = tid & 127;
  const int rg = __builtin_amdgcn_readfirstlane(tid >> 7);
  const int dc = g * BS + 2 * c2;
  if (tid < 128 && !a.conv_w) {   // no Conv1D: x_t = u_t
    cw_lds[c2] = f32x4{1.f, 1.f, 0.f, 0.f};
    cw_lds[128 + c2] = f32x4{0.f, 0.f, 0.f, 0.f};
    cw_lds[256 + c2] = f32x4{0.f, 0.f, 0.f, 0.f};
  } else if (tid < 128) {
    f32x4 t0v, t1v, t2v;
    t0v[0] = a.conv_w[dc];                  t0v[1] = a.conv_w[dc + 1];
    t0v[2] = a.conv_w[(size_t)D + dc];      t0v[3] = a.conv_w[(size_t)D + dc + 1];
    t1v[0] = a.conv_w[(size_t)2 * D + dc];  t1v[1] = a.conv_w[(size_t)2 * D + dc + 1];
    t1v[2] = a.conv_w[(size_t)3 * D + dc];  t1v[3] = a.conv_w[(size_t)3 * D + dc + 1];
    t2v[0] = a.conv_b ? a.conv_b[dc] : 0.f;
    t2v[1] = a.conv_b ? a.conv_b[dc + 1] : 0.f;
    t2v[2] = t2v[3] = 0.f;
    cw_lds[c2] = t0v;
    cw_lds[128 + c2] = t1v;
    cw_lds[256 + c2] = t2v;
  }

  // rows of this slice, in steps of 32
  const long long nstep_all = (a.rows + TT - 1) / TT;
  const long long per = (nstep_all + a.S - 1) / a.S;
  const long long st_lo = (long long)s * per, st_hi = st_lo + per < nstep_all ? st_lo + per : nstep_all;

  // dp / dq loader: 16 bytes per thread, rows lr and lr+16 of the tile
  const int lc = tid & 31, lr = tid >> 5;
  const unsigned short *gsrc = src + (size_t)g * BS + 8 * lc;
  uint4 rl[2];
  // u rows of the channel pair. A tile of the flattened [B*T] rows may straddle sequences, so
  // every input is addressed through its own (sequence, step): in(row, lag) is u[row - lag]
  // while that stays inside the row's sequence, else the carried-in Conv1D state or zero.
  const unsigned *u32 = (const unsigned *)(a.u + dc);
  const unsigned *st32 = a.state_in ? (const unsigned *)(a.state_in + dc) : nullptr;
  auto input_at = [&](long long b, int t) -> unsigned {   // pair of inputs at step t (may be < 0)
    if (t >= 0) return u32[(size_t)(b * T + t) * (D / 2)];
    if (st32) return st32[((size_t)b * 3 + ring_slot(a.pos0 + t)) * (D / 2)];
    return 0u;
  };
  unsigned raw[11];   // inputs of rows r0-3 .. r0+7, r0 = first of this thread's 8 rows
  unsigned nl0 = 0x03030303u, nl1 = 0x03030303u;   // largest lag of rows r0 .. r0+3 and r0+4 .. r0+7, a byte each
  int slow = 0;       // this thread's rows of the tile being prepared are not one plain window
  // (sequence, step) of this thread's first row in the tile the next load_tiles call fetches;
  // the calls walk consecutive tiles, so it advances without a division
  long long nb_ = (st_lo * TT + 8 * rg) / T;
  int nt_ = (int)(st_lo * TT + 8 * rg - nb_ * T);
  // Both fetches go through buffer descriptors made per tile (the flattened row index does not
  // fit a 32-bit byte offset for large batches): scalar row offsets, one per-lane column offset,
  // rows past the end of the tensor read as zero.
  const unsigned row_bytes = (unsigned)D * 2;
  const unsigned t_voff = (unsigned)(g * BS + 8 * lc) * 2 + (unsigned)lr * row_bytes;   // dp / dq rows lr, lr+16
  const unsigned u_voff = (unsigned)dc * 2;                                           // channel pair
  auto load_tiles = [&](long long step) __attribute__((always_inline)) {
    const long long r0 = step * TT + 8 * rg;
    {
      const long long first = step * TT, left = a.rows - first;
      const unsigned nrows = left < TT ? (unsigned)left : (unsigned)TT;
      const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
          uniform_ptr(src + (size_t)first * D), 0, nrows * row_bytes, 0x00020000);
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, t_voff, (unsigned)(16 * h) * row_bytes, RGLRU_NT);
        rl[h] = make_uint4(v[0], v[1], v[2], v[3]);
      }
    }
    slow = !(nt_ >= 3 && nt_ + 8 <= T && r0 + 8 <= a.rows);
    if (PACKED) {   // (no branch on `slow` around the load; r0 is a multiple of 8, and the array is
                    // padded by a tile beyond the last row: one aligned 8-byte read)
      const uint2 v = *(const uint2 *)(a.nlag + r0);
      nl0 = v.x;
      nl1 = v.y;
    }
    if (!slow) {
      // (cached normally: the other gate's workgroup of this slice finds these rows in L2)
      const __amdgpu_buffer_rsrc_t ru = __builtin_amdgcn_make_buffer_rsrc(
          uniform_ptr(a.u + (size_t)(r0 - 3) * D), 0, 11 * row_bytes, 0x00020000);
#pragma unroll
      for (int n = 0; n < 11; ++n) raw[n] = __builtin_amdgcn_raw_buffer_load_b32(ru, u_voff, (unsigned)n * row_bytes, 0);
    }
    nt_ += TT;
    while (nt_ >= T) {
      nt_ -= T;
      ++nb_;
    }
  };
  // dp / dq rows and the rebuilt x of the requested tile into LDS buffer `buf`
  auto park_tiles = [&](long long step, int buf) __attribute__((always_inline)) {
    unsigned short *t0p = (unsigned short *)(smem + (size_t)buf * W_BUF);
#pragma unroll
    for (int h = 0; h < 2; ++h) *(uint4 *)(t0p + (lr + 16 * h) * XS + 8 * lc) = rl[h];
    const f32x4 w01 = cw_lds[c2], w23 = cw_lds[128 + c2], bb = cw_lds[256 + c2];
    float xa[8], xb[8];   // 8 consecutive steps of the two channels
    if (!slow) {
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const unsigned n = PACKED ? (((r < 4 ? nl0 : nl1) >> (8 * (r & 3))) & 3u) : 3u;
        const unsigned v1 = n >= 1u ? raw[r + 2] : 0u, v2 = n >= 2u ? raw[r + 1] : 0u, v3 = n >= 3u ? raw[r] : 0u;
        float x0 = bb[0], x1 = bb[1];
        x0 = fmaf(w01[0], bf_lo(raw[r + 3]), x0); x1 = fmaf(w01[1], bf_hi(raw[r + 3]), x1);
        x0 = fmaf(w01[2], bf_lo(v1), x0);         x1 = fmaf(w01[3], bf_hi(v1), x1);
        x0 = fmaf(w23[0], bf_lo(v2), x0);         x1 = fmaf(w23[1], bf_hi(v2), x1);
        x0 = fmaf(w23[2], bf_lo(v3), x0);         x1 = fmaf(w23[3], bf_hi(v3), x1);
        xa[r] = x0;
        xb[r] = x1;
      }
    } else {  // first rows of a sequence, a tile across two sequences, or the ragged end
      const long long r0 = step * TT + 8 * rg;
#pragma unroll 1
      for (int r = 0; r < 8; ++r) {
        const long long row = r0 + r;
        float x0 = 0.f, x1 = 0.f;
        if (row < a.rows) {
          const long long b = row / T;
          const int t = (int)(row - b * T);
          const unsigned n = PACKED ? a.nlag[row] : 3u;
          const unsigned i0 = input_at(b, t), i1 = n >= 1u ? input_at(b, t - 1) : 0u,
                         i2 = n >= 2u ? input_at(b, t - 2) : 0u, i3 = n >= 3u ? input_at(b, t - 3) : 0u;
          x0 = bb[0]; x1 = bb[1];
          x0 = fmaf(w01[0], bf_lo(i0), x0); x1 = fmaf(w01[1], bf_hi(i0), x1);
          x0 = fmaf(w01[2], bf_lo(i1), x0); x1 = fmaf(w01[3], bf_hi(i1), x1);
          x0 = fmaf(w23[0], bf_lo(i2), x0); x1 = fmaf(w23[1], bf_hi(i2), x1);
          x0 = fmaf(w23[2], bf_lo(i3), x0); x1 = fmaf(w23[3], bf_hi(i3), x1);
        }
        // (a dynamic index into xa / xb would put them in scratch memory)
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          if (q == r) {
            xa[q] = x0;
            xb[q] = x1;
          }
        }
      }
    }
    uint4 ah, bh;
    ah.x = pack_f16(xa[0], xa[1]); ah.y = pack_f16(xa[2], xa[3]);
    ah.z = pack_f16(xa[4], xa[5]); ah.w = pack_f16(xa[6], xa[7]);
    bh.x = pack_f16(xb[0], xb[1]); bh.y = pack_f16(xb[2], xb[3]);
    bh.z = pack_f16(xb[4], xb[5]); bh.w = pack_f16(xb[6], xb[7]);
    unsigned short *xh = (unsigned short *)(smem + (size_t)buf * W_BUF + W_TILE) + (2 * c2) * TS + 8 * rg;
    *(uint4 *)(xh) = ah;
    *(uint4 *)(xh + TS) = bh;
  };

  const int arow = ((j >> 2) & 1) * 16 + (j >> 3) * 4 + (j & 3);
  const int a_off = arow * XS + hf * 8;

  f32x16 acc[2][4];
#pragma unroll
  for (int m = 0; m < 2; ++m)
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[m][n][r] = 0.f;

  // products of the tile in LDS buffer `buf`
  auto products = [&](int buf) __attribute__((always_inline)) {
    const unsigned short *tg = (const unsigned short *)(smem + (size_t)buf * W_BUF) + a_off;
    const unsigned short *xh = (const unsigned short *)(smem + (size_t)buf * W_BUF + W_TILE) +
                               (4 * nw * 32 + j) * TS + 16 * hf;
    const f16x8 sl0 = sel_lds[lane], sl1 = sel_lds[64 + lane];
    // x fragments (as in the dp / dq fragments, lane half hf holds steps 16 hf .. 16 hf + 7 in
    // the first K-step and the following 8 in the second), in the order of their use: f = 4 r +
    // 2 q + i is column block 2 r + i, K-step q. LDS latency is several products long, so the
    // reads run ahead of the products: the first four are requested before the dp / dq fragments
    // are built.
    auto xfrag = [&](int f) __attribute__((always_inline)) {
      const int r = f >> 2, q = (f >> 1) & 1, i = f & 1;
      return *(const f16x8 *)(xh + (2 * r + i) * 32 * TS + q * 8);
    };
    f16x8 w[8];
#pragma unroll
    for (int f = 0; f < 4; ++f) w[f] = xfrag(f);
    __builtin_amdgcn_sched_barrier(0);
    // dp / dq fragments: column block c of the tile -> two K-steps of 8 consecutive steps per lane
    f16x8 fa[2][2];
#pragma unroll
    for (int m = 0; m < 2; ++m) {
      const unsigned short *tile = tg + (2 * mw + m) * 32;
      f32x16 t;
#pragma unroll
      for (int r = 0; r < 16; ++r) t[r] = 0.f;
      t = __builtin_amdgcn_mfma_f32_32x32x16_f16(*(const f16x8 *)(tile), sl0, t, 0, 0, 0);
      t = __builtin_amdgcn_mfma_f32_32x32x16_f16(*(const f16x8 *)(tile + 16), sl1, t, 0, 0, 0);
      unsigned pk[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) pk[e] = pack_f16(t[2 * e], t[2 * e + 1]);   // exact: the values are half precision
      uint4 lo4 = make_uint4(pk[0], pk[1], pk[2], pk[3]), hi4 = make_uint4(pk[4], pk[5], pk[6], pk[7]);
      fa[m][0] = __builtin_bit_cast(f16x8, lo4);
      fa[m][1] = __builtin_bit_cast(f16x8, hi4);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int f = 4; f < 8; ++f) w[f] = xfrag(f);
#pragma unroll
    for (int pr = 0; pr < 4; ++pr) {   // four independent accumulators per round: no product waits for its predecessor
      const int r = pr >> 1, q = pr & 1;
      acc[0][2 * r] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[0][q], w[2 * pr], acc[0][2 * r], 0, 0, 0);
      acc[1][2 * r] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[1][q], w[2 * pr], acc[1][2 * r], 0, 0, 0);
      acc[0][2 * r + 1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[0][q], w[2 * pr + 1], acc[0][2 * r + 1], 0, 0, 0);
      acc[1][2 * r + 1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[1][q], w[2 * pr + 1], acc[1][2 * r + 1], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
  };

  // The two waves that share a SIMD work half a step apart: waves 4-7 multiply and then
  // prepare the next tile, waves 0-3 prepare first and multiply afterwards (their inputs are
  // requested one step earlier), so that matrix and vector phases of the pair overlap. Both
  // orders read buffer `buf` and write the other one between the same two barriers. (The SIMD
  // serves its older wave first; the late order is the longer chain, so waves 0-3 get it.)
  const bool late = wv < NWAVE / 2;
  if (st_lo < st_hi) {
    load_tiles(st_lo);
    __syncthreads();   // the taps parked in LDS are visible
    park_tiles(st_lo, 0);
    if (late && st_lo + 1 < st_hi) load_tiles(st_lo + 1);
    __syncthreads();
    int it = 0;
    if (!late) {
      for (long long step = st_lo; step < st_hi; ++step, ++it) {
        const int buf = it & 1;
        if (step + 1 < st_hi) load_tiles(step + 1);
        products(buf);
        if (step + 1 < st_hi) park_tiles(step + 1, buf ^ 1);
        __syncthreads();
      }
    } else {
      for (long long step = st_lo; step < st_hi; ++step, ++it) {
        const int buf = it & 1;
        if (step + 1 < st_hi) park_tiles(step + 1, buf ^ 1);
        if (step + 2 < st_hi) load_tiles(step + 2);
        products(buf);
        __syncthreads();
      }
    }
  }
  // rows of the accumulator are output channels j, columns are input channels k
  float *out = a.part + (((size_t)s * 2 + gate) * a.nb + g) * BS * BS;
#pragma unroll
  for (int m = 0; m < 2; ++m)
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = 64 * mw + 32 * m + 8 * (r >> 2) + 4 * hf + (r & 3);
        const int col = 128 * nw + 32 * n + j;
        out[(size_t)row * BS + col] = acc[m][n][r];
      }
}

// Final pass: every partial sum of the three kernels is added up in a fixed order.
//   blocks [0, nW):  dW[gate][g][j][k] = sum over the S slices of the wgrad kernel
//   then 3 rows x D: db_a, db_x, dLambda from the gates kernel's B*G partial rows
//   then 5 rows x D: dconv_w[0..3], dconv_b from the dgrad kernel's B*C partial rows
struct FinishArgs {
  const float *partW, *partA, *partC;
  const float *sc;   // sc[2] = 1 / S: the wgrad partial sums carry the factor S of dp, dq
  int S, nA, nC, D;
  size_t per_gate;
  float *dWa, *dWx;
  float *rowsA[3];
  float *rowsC[5];
};
__global__ void __launch_bounds__(256) bwd_finish_kernel(FinishArgs a) {
  const int nW = (int)((2 * a.per_gate + 255) / 256), dblocks = (a.D + 255) / 256;
  int blk = blockIdx.x;
  if (blk < nW) {
    const size_t i = (size_t)blk * 256 + threadIdx.x;
    if (i >= 2 * a.per_gate) return;
    float sum = 0.f;
    for (int s = 0; s < a.S; ++s) sum += a.partW[(size_t)s * 2 * a.per_gate + i];
    sum *= a.sc[2];
    if (i < a.per_gate)
      a.dWa[i] = sum;
    else
      a.dWx[i - a.per_gate] = sum;
    return;
  }
  blk -= nW;
  const int r = blk / dblocks, d = (blk - r * dblocks) * 256 + threadIdx.x;
  if (d >= a.D) return;
  const bool gates = r < 3;
  const int rr = gates ? r : r - 3, rows = gates ? 3 : 5, n = gates ? a.nA : a.nC;
  const float *part = gates ? a.partA : a.partC;
  float *out = gates ? a.rowsA[rr] : a.rowsC[rr];
  if (!out) return;
  float s = 0.f;
  for (int q = 0; q < n; ++q) s += part[((size_t)q * rows + rr) * a.D + d];
  out[d] = s;
}

}  // namespace

// ------------------------------------------------------------------------------ host side
namespace {

size_t al256(size_t n) { return (n + 255) & ~(size_t)255; }

struct BwdPlan {
  int units, ntile, G, R, C, S;
  size_t off_dp, off_dq, off_dx, off_wta, off_wtx, off_wxf, off_sc, off_rec, off_partA, off_partC, off_partW, total;
  size_t off_masks, off_nlag;   // packed sequences only, behind everything else
};

BwdPlan plan_backward(int B, int T, int D, int nb, int ncu, bool packed = false) {
  BwdPlan q;
  q.units = B * nb;
  q.ntile = (T + TT - 1) / TT;
  q.G = pick_slices(q.units, q.ntile, ncu, 16);
  q.R = 8 * q.G;
  q.C = ncu / q.units;
  if (q.C < 1) q.C = 1;
  if (q.C > q.ntile) q.C = q.ntile;
  // wgrad: 2*nb blocks per slice; enough slices to cover the device, each at least 8 steps
  const long long steps = ((long long)B * T + TT - 1) / TT;
  long long S = ncu / (2 * nb);
  if (S < 1) S = 1;
  if (S > steps / 8) S = steps / 8 > 0 ? steps / 8 : 1;
  q.S = (int)S;
  const size_t N2 = al256((size_t)B * T * D * 2), wbytes = al256((size_t)nb * BS * BS * 2);
  size_t off = 0;
  q.off_dp = off; off += N2;
  q.off_dq = off; off += N2;
  q.off_dx = off; off += al256((size_t)B * ((T + 3) / 4) * D * 8);
  q.off_wta = off; off += wbytes;
  q.off_wtx = off; off += wbytes;
  q.off_wxf = off; off += wbytes;
  q.off_sc = off; off += 256;
  q.off_rec = off; off += al256(256 + (size_t)q.units * q.R * 2 * BS * sizeof(u64));
  q.off_partA = off; off += al256((size_t)B * q.G * 3 * D * 4);
  q.off_partC = off; off += al256((size_t)B * q.C * 5 * D * 4);
  q.off_partW = off; off += al256((size_t)q.S * 2 * nb * BS * BS * 4);
  q.off_masks = q.off_nlag = off;
  if (packed) {
    q.off_masks = off; off += al256((size_t)B * q.ntile * sizeof(uint4));
    q.off_nlag = off; off += al256((size_t)B * T + TT);   // (read in 8-byte pieces up to a tile past the end)
  }
  q.total = off;
  return q;
}

}  // namespace

bool backward_mfma_supported(const Problem &p, bool bf) {
  auto al = [](const void *q, size_t n) { return ((uintptr_t)q % n) == 0; };
  return bf && p.bs == BS && p.T >= 1 && (size_t)p.T * p.D * 4 < ((size_t)1 << 32) &&
         al(p.W_a, 16) && al(p.W_x, 16) && al(p.u, 16) && al(p.y_in, 4) && al(p.dy, 4) && al(p.dy_lo, 4) &&
         al(p.du, 2) && (!p.state_in || al(p.state_in, 16));
}

size_t backward_mfma_ws_bytes(int B, int T, int D, int nb) {
  // sized for 256 compute units so that the answer does not depend on the device
  return plan_backward(B, T, D, nb, 256).total;
}

size_t backward_mfma_packed_ws_bytes(int B, int T, int D, int nb) {
  return plan_backward(B, T, D, nb, 256, true).total;
}

size_t backward_mfma_flag_offset(int B, int T, int D, int nb) {
  int ncu = num_cu();
  if (ncu > 256) ncu = 256;
  return plan_backward(B, T, D, nb, ncu).off_rec;   // the plan the launch uses
}

template <typename K>
static hipError_t big_lds(K kernel, int bytes) {
  return hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

hipError_t launch_backward_mfma(const Problem &p, hipStream_t s) {
  int ncu = num_cu();
  if (ncu > 256) ncu = 256;
  const bool packed = p.reset != nullptr;
  const BwdPlan q = plan_backward(p.B, p.T, p.D, p.nb, ncu, packed);
  char *ws = (char *)p.ws;
  hipError_t e;
  static bool configured = false;
  if (!configured) {
    if ((e = big_lds(bwd_gates_kernel<1, false, true>, g_lds(false))) != hipSuccess) return e;
    if ((e = big_lds(bwd_gates_kernel<4, false, true>, g_lds(false))) != hipSuccess) return e;
    if ((e = big_lds(bwd_gates_kernel<8, false, true>, g_lds(false))) != hipSuccess) return e;
    if ((e = big_lds(bwd_gates_kernel<16, false, true>, g_lds(false))) != hipSuccess) return e;
    if ((e = big_lds(bwd_dgrad_kernel<true>, D_LDS)) != hipSuccess) return e;
    if ((e = big_lds(bwd_wgrad_kernel<true>, W_LDS)) != hipSuccess) return e;
    if ((e = big_lds(bwd_gates_kernel<1>, g_lds(false))) != hipSuccess) return e;
    if ((e = big_lds(bwd_gates_kernel<4>, g_lds(false))) != hipSuccess) return e;
    if ((e = big_lds(bwd_gates_kernel<8>, g_lds(false))) != hipSuccess) return e;
    if ((e = big_lds(bwd_gates_kernel<16>, g_lds(false))) != hipSuccess) return e;
    if ((e = big_lds(bwd_gates_kernel<1, true>, g_lds(true))) != hipSuccess) return e;
    if ((e = big_lds(bwd_gates_kernel<4, true>, g_lds(true))) != hipSuccess) return e;
    if ((e = big_lds(bwd_gates_kernel<8, true>, g_lds(true))) != hipSuccess) return e;
    if ((e = big_lds(bwd_gates_kernel<16, true>, g_lds(true))) != hipSuccess) return e;
    if ((e = big_lds(bwd_dgrad_kernel<false>, D_LDS)) != hipSuccess) return e;
    if ((e = big_lds(bwd_wgrad_kernel<false>, W_LDS)) != hipSuccess) return e;
    configured = true;
  }
  unsigned short *wta = (unsigned short *)(ws + q.off_wta), *wtx = (unsigned short *)(ws + q.off_wtx);
  // 0. the scale of the upstream gradient: dp and dq travel between the kernels in half
  // precision as S dp, S dq with max(|dy|, |dhT|) S in [32, 64). delta sums dy over the memory
  // of the recurrence and the adjoints are a small multiple of it: they stay inside half
  // precision's 65504 unless thousands of steps of dy at its maximum and of one sign pile up
  // (the conversion then saturates, it does not overflow to infinity), and keep 11 bits down
  // to 2e-6 of that maximum.
  float *sc = (float *)(ws + q.off_sc);
  if ((e = launch_grad_scale(p.dy, (size_t)p.B * p.T * p.D, p.dhT, (size_t)p.B * p.D, sc, 5, s)) != hipSuccess)
    return e;

  // (packed sequences: the document boundaries as bit masks per tile and as lag counts per step)
  uint4 *masks = (uint4 *)(ws + q.off_masks);
  unsigned char *nlag = (unsigned char *)(ws + q.off_nlag);
  if (packed && (e = launch_reset_masks(p.reset, masks, nlag, p.B, p.T, s)) != hipSuccess) return e;

  // 1. gates, reverse scan, pointwise adjoints
  BwdArgs a;
  a.p = p;
  a.rmask = packed ? masks : nullptr;
  a.G = q.G; a.ntile = q.ntile; a.R = q.R;
  a.err = (int *)(ws + q.off_rec);
  a.rec = (u64 *)(ws + q.off_rec + 256);
  a.dpo = (unsigned short *)(ws + q.off_dp);
  a.dqo = (unsigned short *)(ws + q.off_dq);
  a.dxo = (unsigned char *)(ws + q.off_dx);
  a.sc = sc;
  a.part = (float *)(ws + q.off_partA);
  const int grid = q.units * q.G;
  a.swizzle = (q.G > 1 && grid % 8 == 0) ? 1 : 0;
  a.wxf = (const unsigned short *)(ws + q.off_wxf);
  // the records only exist (and need clearing) when sequences are sliced in time; the status
  // word in front of them is cleared in any case (a later health check reads it)
  const size_t clear = q.G > 1 ? 256 + (size_t)q.units * q.R * 2 * BS * sizeof(u64) : 256;
  {
    PrepArgs pa;
    pa.Wa = (const unsigned short *)p.W_a; pa.Wx = (const unsigned short *)p.W_x;
    pa.WTa = wta; pa.WTx = wtx;
    pa.wxf = (uint4 *)(ws + q.off_wxf);
    pa.zero = (uint4 *)(ws + q.off_rec);
    pa.n16 = clear / 16;
    pa.nb = p.nb;
    const size_t nfrag = (size_t)p.nb * BS * BS / 8, n = pa.n16 > nfrag ? pa.n16 : nfrag;
    KernelTimer kt("bwd_prep_kernel", s);
    hipLaunchKernelGGL(bwd_prep_kernel, dim3((unsigned)(128 * p.nb + (n + 255) / 256)), dim3(256), 0, s, pa);
  }
  if ((e = hipGetLastError()) != hipSuccess) return e;
  {
    KernelTimer kt(packed ? "bwd_gates_packed_kernel" : "bwd_gates_kernel", s);
    if (packed) {   // (the packed entry point takes dy as one tensor)
      if (q.G == 1)
        hipLaunchKernelGGL((bwd_gates_kernel<1, false, true>), dim3(grid), dim3(NTHR), g_lds(false), s, a);
      else if (q.G <= 4)
        hipLaunchKernelGGL((bwd_gates_kernel<4, false, true>), dim3(grid), dim3(NTHR), g_lds(false), s, a);
      else if (q.G <= 8)
        hipLaunchKernelGGL((bwd_gates_kernel<8, false, true>), dim3(grid), dim3(NTHR), g_lds(false), s, a);
      else
        hipLaunchKernelGGL((bwd_gates_kernel<16, false, true>), dim3(grid), dim3(NTHR), g_lds(false), s, a);
    } else if (p.dy_lo) {
      if (q.G == 1)
        hipLaunchKernelGGL((bwd_gates_kernel<1, true>), dim3(grid), dim3(NTHR), g_lds(true), s, a);
      else if (q.G <= 4)
        hipLaunchKernelGGL((bwd_gates_kernel<4, true>), dim3(grid), dim3(NTHR), g_lds(true), s, a);
      else if (q.G <= 8)
        hipLaunchKernelGGL((bwd_gates_kernel<8, true>), dim3(grid), dim3(NTHR), g_lds(true), s, a);
      else
        hipLaunchKernelGGL((bwd_gates_kernel<16, true>), dim3(grid), dim3(NTHR), g_lds(true), s, a);
    } else if (q.G == 1)
      hipLaunchKernelGGL(bwd_gates_kernel<1>, dim3(grid), dim3(NTHR), g_lds(false), s, a);
    else if (q.G <= 4)
      hipLaunchKernelGGL(bwd_gates_kernel<4>, dim3(grid), dim3(NTHR), g_lds(false), s, a);
    else if (q.G <= 8)
      hipLaunchKernelGGL(bwd_gates_kernel<8>, dim3(grid), dim3(NTHR), g_lds(false), s, a);
    else
      hipLaunchKernelGGL(bwd_gates_kernel<16>, dim3(grid), dim3(NTHR), g_lds(false), s, a);
  }
  if ((e = hipGetLastError()) != hipSuccess) return e;

  // 2. dgrad and Conv1D adjoint
  DgradArgs dg;
  dg.p = p;
  dg.C = q.C; dg.ntile = q.ntile;
  dg.dpo = a.dpo; dg.dqo = a.dqo; dg.dxo = a.dxo;
  dg.sc = sc;
  dg.wta = wta; dg.wtx = wtx;
  dg.part = (float *)(ws + q.off_partC);
  dg.rmask = packed ? masks : nullptr;
  {
    KernelTimer kt(packed ? "bwd_dgrad_packed_kernel" : "bwd_dgrad_kernel", s);
    if (packed)
      hipLaunchKernelGGL(bwd_dgrad_kernel<true>, dim3(q.units * q.C), dim3(NTHR), D_LDS, s, dg);
    else
      hipLaunchKernelGGL(bwd_dgrad_kernel<false>, dim3(q.units * q.C), dim3(NTHR), D_LDS, s, dg);
  }
  if ((e = hipGetLastError()) != hipSuccess) return e;

  // 3. wgrad
  WgradArgs wg;
  wg.nb = p.nb; wg.S = q.S; wg.D = p.D; wg.T = p.T;
  wg.rows = (long long)p.B * p.T;
  wg.pos0 = p.pos0;
  wg.dpo = a.dpo; wg.dqo = a.dqo;
  wg.u = (const unsigned short *)p.u;
  wg.state_in = (const unsigned short *)p.state_in;
  wg.conv_w = p.conv_w; wg.conv_b = p.conv_b;
  wg.part = (float *)(ws + q.off_partW);
  wg.nlag = packed ? nlag : nullptr;
  {
    KernelTimer kt(packed ? "bwd_wgrad_packed_kernel" : "bwd_wgrad_kernel", s);
    if (packed)
      hipLaunchKernelGGL(bwd_wgrad_kernel<true>, dim3((q.S * 2 * p.nb + 15) / 16 * 16), dim3(NTHR), W_LDS, s, wg);
    else
      hipLaunchKernelGGL(bwd_wgrad_kernel<false>, dim3((q.S * 2 * p.nb + 15) / 16 * 16), dim3(NTHR), W_LDS, s, wg);
  }
  if ((e = hipGetLastError()) != hipSuccess) return e;
  // 4. all partial sums
  FinishArgs fa;
  fa.partW = wg.part; fa.partA = a.part; fa.partC = dg.part;
  fa.sc = sc;
  fa.S = q.S; fa.nA = p.B * q.G; fa.nC = p.B * q.C; fa.D = p.D;
  fa.per_gate = (size_t)p.nb * BS * BS;
  fa.dWa = p.g.dW_a; fa.dWx = p.g.dW_x;
  fa.rowsA[0] = p.g.db_a; fa.rowsA[1] = p.g.db_x; fa.rowsA[2] = p.g.dLambda;
  for (int k = 0; k < 4; ++k) fa.rowsC[k] = p.g.dconv_w ? p.g.dconv_w + (size_t)k * p.D : nullptr;
  fa.rowsC[4] = p.g.dconv_b;
  {
    const unsigned nW = (unsigned)((2 * fa.per_gate + 255) / 256), dblocks = (unsigned)((p.D + 255) / 256);
    KernelTimer kt("bwd_finish_kernel", s);
    hipLaunchKernelGGL(bwd_finish_kernel, dim3(nW + 8 * dblocks), dim3(256), 0, s, fa);
  }
  return hipGetLastError();
}


}  // namespace rglru
