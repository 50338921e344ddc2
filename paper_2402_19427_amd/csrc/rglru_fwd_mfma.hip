// Fused forward for bf16 storage and gate blocks of 256 channels (gfx950).
//
// One workgroup of 8 waves owns one (sequence, gate block) pair - or one of G interleaved
// time slices of it - and walks it in tiles of 32 steps:
//   Conv1D (Section 2.3) in fp32 -> tile in LDS as a high part + a low part in half precision;
//     the gate products read the high part, the recurrence input x_t is rebuilt from both
//   gate pre-activations W_a x, W_x x (eqs. 1-2) with v_mfma_f32_32x32x16_f16; each wave keeps
//     its 32 output channels of both gate matrices in registers for the whole kernel
//   gates, a_t, sqrt(1-a_t^2) (eqs. 1-3, Appendix A) and the scan (eq. 4) in registers: every
//     lane runs 16 consecutive steps of one channel, the two lane halves are combined with
//     the affine composition (a2,b2)o(a1,b1) = (a2 a1, a2 b1 + b2)
//   when a sequence is sliced in time (tile t belongs to workgroup t mod G), every tile
//     publishes its aggregate (prod a, local end state) as tagged 8-byte records; a workgroup
//     carries its own state from its previous tile across the G-1 tiles in between by reading
//     their aggregates. Aggregates do not depend on incoming states, so no workgroup ever
//     waits on a chain; the outputs of a tile are finished one iteration late, from the (a_t, b_t)
//     pairs parked in LDS, so that the records it needs are long since visible.
//
// Scaling trick: the Conv1D taps are multiplied by log2(e), so the MFMA delivers
// log2(e)*(Wx+b) and v_exp_f32 (a base-2 exponential) needs no extra multiply; the input gate
// is evaluated as ln(2)*sigmoid, which cancels the factor carried by x.
#include "rglru_gelu.h"
#include "rglru_mfma.h"

#include <atomic>
#include <type_traits>

namespace rglru {

using namespace mfma;

namespace {

constexpr int FWD_LDS = XS_BYTES + CONST_BYTES + HOLD_BYTES + NWAVE * OTILE_BYTES;


struct FwdArgs {
  Problem p;
  int G;         // time slices (workgroups) per (sequence, block)
  int ntile;     // tiles per sequence
  int R;         // record ring depth per unit
  u64 *rec;      // [unit][R][2][256] records (A then H), zeroed before launch; NULL if G == 1
  int *err;      // set to 1 if a bounded wait expired
  int swizzle;   // remap block ids so that neighbouring time slices share an XCD
  const unsigned short *wx16;   // W_x in half precision, same layout (fwd_prep_kernel)
  const uint4 *rmask;           // packed sequences: per (sequence, tile) bit masks of the document
                                // boundaries (reset_mask_kernel), or NULL
  // Contiguous time slices (G == 1 only): S > 1 cuts every sequence into S windows of Ts steps
  // (the last one shorter), each a workgroup's own; h0, state_in (and hT, aprod of the
  // aggregate pass) are then [B*S] arrays with one entry per window.
  int S, Ts;
  float *aprod;                 // aggregate pass: [B*S][D] product of a_t over the window
};

// eqs. (1)-(3) with base-2 exponentials; pp, qq, xx carry a factor log2(e).
// Returns a_t and b_t = sqrt(1-a_t^2) * i_t * x_t.
__device__ __forceinline__ void gate_fast(float pp, float qq, float xx, float kd, float &a,
                                          float &b) {
  const float ep = __builtin_amdgcn_exp2f(-pp);
  const float r = __builtin_amdgcn_rcpf(1.f + ep);
  const float l2 = kd * r;
  a = __builtin_amdgcn_exp2f(l2);
  const float m = __builtin_amdgcn_sqrtf(one_minus_sq(a, l2));
  const float eq = __builtin_amdgcn_exp2f(-qq);
  const float il = __builtin_amdgcn_rcpf(fmaf(eq, LOG2E, LOG2E));  // ln2 * sigmoid(q)
  b = (m * il) * xx;
}

// Preparation pass of the sliced forward kernel: clears the record rings (a fill kernel rather
// than a memset, so that a caller may capture the call in a HIP graph).
__global__ void __launch_bounds__(256) prep_kernel(uint4 *zero, size_t n16, bool keep_status) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n16) zero[i] = cleared_word(zero, i, keep_status);
}
// The forward kernel's own preparation: the same clearing, and W_x once in half precision (its
// K-steps that do not fit the registers are re-read every tile; converting them there would
// cost more than this pass; n8 = groups of eight weights).
__global__ void __launch_bounds__(256) fwd_prep_kernel(uint4 *zero, size_t n16, const uint4 *wx, uint4 *wx16,
                                                       size_t n8) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n16) zero[i] = cleared_word(zero, i, true);
  if (i < n8) {
    const uint4 w = wx[i];
    wx16[i] = make_uint4(pack_f16(bf_lo(w.x), bf_hi(w.x)), pack_f16(bf_lo(w.y), bf_hi(w.y)),
                         pack_f16(bf_lo(w.z), bf_hi(w.z)), pack_f16(bf_lo(w.w), bf_hi(w.w)));
  }
}

typedef unsigned u32x4m __attribute__((ext_vector_type(4)));

// Document boundaries of packed sequences as bit masks, one uint4 per (sequence, tile of 32
// steps), bit i = step 32 tile + i:
//   x: a document starts at this step (the recurrence takes h_{t-1} = 0)
//   y, z, w: the Conv1D's lag 1, 2, 3 of this step stays inside the step's document (no start at
//            steps t .. t-lag+1; inputs in front of a document count as zeros)
// Steps past the end of the sequence count as inside a document (their inputs are zero anyway),
// so that a ragged last tile without a boundary looks like any other tile without one.
// nlag (may be null): per step the largest lag (0..3) that stays inside the step's document,
// [B * T] bytes, for kernels that walk the flattened rows.
__global__ void __launch_bounds__(256) reset_mask_kernel(const unsigned char *reset, uint4 *out,
                                                         unsigned char *nlag, int B, int T, int ntile) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= B * ntile) return;
  const int b = i / ntile, t0 = (i - b * ntile) * TT;
  const unsigned char *m = reset + (size_t)b * T;
  unsigned r = 0, l1 = 0, l2 = 0, l3 = 0;
  for (int k = 0; k < TT; ++k) {
    const int t = t0 + k;
    if (t >= T) {
      l1 |= 1u << k; l2 |= 1u << k; l3 |= 1u << k;
      continue;
    }
    const bool s0 = m[t] != 0, s1 = t >= 1 && m[t - 1] != 0, s2 = t >= 2 && m[t - 2] != 0;
    r |= (unsigned)s0 << k;
    l1 |= (unsigned)(!s0) << k;
    l2 |= (unsigned)(!s0 && !s1) << k;
    l3 |= (unsigned)(!s0 && !s1 && !s2) << k;
    if (nlag) nlag[(size_t)b * T + t] = (unsigned char)(s0 ? 0 : s1 ? 1 : s2 ? 2 : 3);
  }
  out[i] = make_uint4(r, l1, l2, l3);
}

constexpr int FWD_MAX_SLICES = 16;

// Contiguous time slices ("windows") of a sequence, first helper: the Conv1D ring each window
// starts from - the caller's ring for a sequence's first window (zeros without one), the three
// inputs in front of it for every other window, in the slots their positions select.
struct WinArgs {
  const unsigned short *u, *state_in;
  unsigned short *rings;   // [B*S][3][D]
  int B, S, Ts, T, D;
  long long pos0;
};
__global__ void __launch_bounds__(256) window_ring_kernel(WinArgs a) {
  const int D2 = a.D / 2;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)a.B * a.S * 3 * D2) return;
  const int c = (int)(i % D2), slot = (int)((i / D2) % 3);
  const int bw = (int)(i / ((size_t)3 * D2)), seq = bw / a.S, win = bw - seq * a.S;
  unsigned v = 0;
  if (win == 0) {
    if (a.state_in) v = ((const unsigned *)a.state_in)[((size_t)seq * 3 + slot) * D2 + c];
  } else {
    const long long pw = a.pos0 + (long long)win * a.Ts;   // position of the window's first step
    for (int k = 1; k <= 3; ++k)
      if (ring_slot(pw - k) == slot)
        v = ((const unsigned *)a.u)[((size_t)seq * a.T + (size_t)win * a.Ts - k) * D2 + c];
  }
  ((unsigned *)a.rings)[i] = v;
}
// Second helper: the state every window starts from, out of the windows' aggregates
// (h_end = A h_in + H for a window with decay product A and zero-state end value H; eq. (4)).
__global__ void __launch_bounds__(256) window_chain_kernel(const float *h0, const float *A, const float *H,
                                                           float *hin, int B, int S, int D) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)B * D) return;
  const int seq = (int)(i / D), d = (int)(i - (size_t)seq * D);
  float h = h0 ? h0[i] : 0.f;
  for (int w0 = 0; w0 < S; w0 += 8) {   // eight windows' aggregates in flight ahead of the chain
    float av[8], hv[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const size_t k = ((size_t)seq * S + (w0 + e < S ? w0 + e : S - 1)) * D + d;
      av[e] = A[k];
      hv[e] = H[k];
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      if (w0 + e < S) {
        hin[((size_t)seq * S + w0 + e) * D + d] = h;
        h = fmaf(av[e], h, hv[e]);
      }
    }
  }
}

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

// eight values of y (bf16 pairs) times GeLU of eight values of the block's other branch
template <int MERGE>
__device__ __forceinline__ u32x4 merge8(const u32x4 yv, const u32x4 bv) {
  u32x4 o;
#pragma unroll
  for (int k = 0; k < 4; ++k)
    o[k] = pack_bf16(bf_lo(yv[k]) * gelu<MERGE == 2, true>(bf_lo(bv[k])),
                     bf_hi(yv[k]) * gelu<MERGE == 2, true>(bf_hi(bv[k])));
  return o;
}

// GMAX = 1: one workgroup per (sequence, block); GMAX = 4 / 8 / 16: 2..4 / 5..8 / 9..16 time slices
// MERGE = 0: y is the output; 1 / 2: the recurrent block's merge (Section 2.3) as epilogue,
// out = y * GeLU(branch) with GeLU = z Phi(z) / its tanh form, y itself written only if asked for
// PAD: gate blocks narrower than 256 channels (a multiple of 16, Section 4.1's 16 blocks at
// width 2560 give 160) run in the 256-wide tile: parameter reads of the missing channels and
// K-steps are clamped to existing ones (whatever they hold meets zeros: the Conv1D lanes of
// missing channels write x = 0), their loads of u read nothing and their stores are dropped.
// PACKED: the sequences hold several documents (FwdArgs.rmask); a variant of its own, so that
// the plain kernel keeps its register allocation
// AGG: aggregate pass over contiguous time slices: nothing of y is formed or written, every
// window leaves its end state for a zero incoming state (hT) and the product of its a_t (aprod)
template <int GMAX, int MERGE, bool PAD, bool PACKED = false, bool AGG = false>
__global__ void __launch_bounds__(NTHR) __attribute__((amdgpu_waves_per_eu(2, 2)))
fwd_mfma_kernel(FwdArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned short *xs = (unsigned short *)smem;                   // [2 buffers][high, low][TT][XS]
  f16x8 *sel_lds = (f16x8 *)(smem + XS_BYTES);                   // [2][64] selection operands
  f32x4 *cw_lds = (f32x4 *)(smem + XS_BYTES + 64 * 32);          // [3][128] Conv1D taps and bias
  float *hold = (float *)(smem + XS_BYTES + CONST_BYTES);        // [wave][8][64] float4
  const Problem &p = a.p;
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5, j = lane & 31;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  // this wave's staging tile for the y rows it produces
  unsigned short *otile = (unsigned short *)(smem + XS_BYTES + CONST_BYTES + HOLD_BYTES) + wv * (OTILE_BYTES / 2);
  const int G = GMAX == 1 ? 1 : a.G;

  int bid = blockIdx.x;
  if (GMAX > 1 && a.swizzle) {  // consecutive logical ids on one XCD (ids are dealt round-robin to 8)
    const int per = gridDim.x >> 3;
    bid = (bid & 7) * per + (bid >> 3);
  }
  const int unit = bid / G, w = bid - unit * G;
  // b: entry of the per-sequence arrays (h0, states); with contiguous time slices that is the
  // window, which covers rows row0 .. row0 + T - 1 of the [B*T] rows and starts at position pos0
  const int b = unit / p.nb, g = unit - b * p.nb;
  const int D = p.D;
  int T = p.T, ntile = a.ntile, win = 0, nwin = 1, ob = b;   // ob: entry of the final states
  size_t row0 = (size_t)b * p.T;
  long long pos0 = p.pos0;
  if (GMAX == 1 && !PACKED && a.S > 1) {
    const int seq = b / a.S;
    nwin = a.S;
    ob = seq;
    win = b - seq * a.S;
    row0 = (size_t)seq * p.T + (size_t)win * a.Ts;
    T = p.T - win * a.Ts < a.Ts ? p.T - win * a.Ts : a.Ts;
    ntile = (T + TT - 1) / TT;
    pos0 += (long long)win * a.Ts;
  }
  const int ch = wv * 32 + j;  // channel inside the block owned by this lane
  constexpr unsigned OOB = 0x80000000u;   // buffer offset past every range: loads give 0, stores are dropped
  const int bs = PAD ? p.bs : BS;         // channels of a gate block in memory
  const int nk = bs >> 4;                 // its K-steps
  const bool ch_ok = !PAD || ch < bs;
  const int chc = ch_ok ? ch : bs - 1;    // an existing channel to read parameters of
  const int d = g * bs + chc;
  auto kc = [&](int ks) __attribute__((always_inline)) { return PAD ? (ks < nk ? ks : nk - 1) : ks; };

  // ---- gate weights of this wave's 32 output channels, resident in registers
  // (the late waves keep their accumulators across the barrier, and a sequence sliced in time
  // needs registers for the carry exchange as well: the last K-steps of W_x are re-read from L2
  // every tile - a far better spill space than scratch memory)
  // (the merge epilogue holds eight more registers: the tile's rows of the other branch)
  constexpr int NRES_PLAIN = GMAX == 1 ? 13 : (GMAX == 4 ? 9 : (GMAX == 8 ? 6 : 2));   // measured best
  constexpr int NRES_M = MERGE == 0 ? NRES_PLAIN : (NRES_PLAIN >= 2 ? NRES_PLAIN - 2 : 0);
  // (a narrower block has fewer K-steps that matter, and its clamped addresses cost registers;
  // measured best at 160 channels)
  constexpr int NRES_P = GMAX == 1 ? 11 : (GMAX == 4 ? 2 : (GMAX == 8 ? 0 : 2));
  constexpr int NRES_U = !PAD ? NRES_M : (MERGE == 0 ? NRES_P : (NRES_P >= 2 ? NRES_P - 2 : 0));
  // (the masks of packed sequences take registers of their own)
  // (the aggregate pass stages no outputs)
  constexpr int NRES = AGG ? (PAD ? 11 : 14) : !PACKED ? NRES_U : (NRES_U >= 1 ? NRES_U - 1 : 0);
  constexpr int PF = 2;   // streamed fragments in flight (deeper rings measured no better)
  f16x8 wa[16], wx[NRES > 0 ? NRES : 1];   // (half precision, see w_to_f16)
  const f16x8 *pxs = (const f16x8 *)(a.wx16 + ((size_t)g * bs + chc) * bs + hf * 8);
  {
    const bf16x8 *pa = (const bf16x8 *)((const unsigned short *)p.W_a + ((size_t)g * bs + chc) * bs + hf * 8);
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) wa[ks] = w_to_f16(pa[kc(ks) * 2]);
#pragma unroll
    for (int ks = 0; ks < NRES; ++ks) wx[ks] = pxs[kc(ks) * 2];
  }
  // selection matrices that copy this wave's 32 columns of the tile into accumulator layout
  // (the same for every wave; parked in LDS to keep registers for the weights)
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
  float kd;  // -c * softplus(-Lambda) * log2(e)
  {
    const float z = -p.Lambda[d];
    const float sp = z > 0.f ? z + log1pf(expf(-z)) : log1pf(expf(z));
    kd = -p.c * sp * LOG2E;
  }

  // ---- Conv1D assignment: channel pair c2, rows 8*rg .. 8*rg+7 of the tile
  const int c2 = tid & 127;
  const int rg = __builtin_amdgcn_readfirstlane(tid >> 7);
  const bool pair_ok = !PAD || 2 * c2 < bs;
  const int dc = g * bs + (pair_ok ? 2 * c2 : 0);
  if (tid < 128 && !p.conv_w) {   // no Conv1D: x_t = u_t, the identity tap
    cw_lds[c2] = pair_ok ? f32x4{LOG2E, LOG2E, 0.f, 0.f} : f32x4{0.f, 0.f, 0.f, 0.f};
    cw_lds[128 + c2] = f32x4{0.f, 0.f, 0.f, 0.f};
    cw_lds[256 + c2] = f32x4{0.f, 0.f, 0.f, 0.f};
  } else if (tid < 128) {  // taps (scaled by log2 e) and bias of the channel pair, parked in LDS
    f32x4 t0v, t1v, t2v;
    t0v[0] = p.conv_w[dc] * LOG2E;                  t0v[1] = p.conv_w[dc + 1] * LOG2E;
    t0v[2] = p.conv_w[(size_t)D + dc] * LOG2E;      t0v[3] = p.conv_w[(size_t)D + dc + 1] * LOG2E;
    t1v[0] = p.conv_w[(size_t)2 * D + dc] * LOG2E;  t1v[1] = p.conv_w[(size_t)2 * D + dc + 1] * LOG2E;
    t1v[2] = p.conv_w[(size_t)3 * D + dc] * LOG2E;  t1v[3] = p.conv_w[(size_t)3 * D + dc + 1] * LOG2E;
    t2v[0] = p.conv_b ? p.conv_b[dc] * LOG2E : 0.f;
    t2v[1] = p.conv_b ? p.conv_b[dc + 1] * LOG2E : 0.f;
    t2v[2] = t2v[3] = 0.f;
    if (!pair_ok) t0v = t1v = t2v = f32x4{0.f, 0.f, 0.f, 0.f};
    cw_lds[c2] = t0v;
    cw_lds[128 + c2] = t1v;
    cw_lds[256 + c2] = t2v;
  }

  // buffer descriptors over this sequence: scalar row offsets, per-lane channel offsets
  const unsigned seq_bytes = (unsigned)((size_t)T * D * 2);
  const unsigned row_bytes = (unsigned)D * 2;
  const __amdgpu_buffer_rsrc_t u_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      uniform_ptr((const unsigned short *)p.u + row0 * D), 0, seq_bytes, 0x00020000);
  // (a y that is not asked for gets an empty range: its stores are dropped)
  const __amdgpu_buffer_rsrc_t y_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      uniform_ptr((unsigned short *)p.y + row0 * D), 0, p.y ? seq_bytes : 0u, 0x00020000);
  const __amdgpu_buffer_rsrc_t br_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      uniform_ptr((const unsigned short *)(MERGE ? p.branch : p.u) + row0 * D), 0, seq_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t out_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      uniform_ptr((unsigned short *)(MERGE ? p.out : p.y) + row0 * D), 0, seq_bytes, 0x00020000);
  const unsigned u_voff = pair_ok ? (unsigned)dc * 2 : OOB;
  const unsigned *st32 = (p.state_in && pair_ok)
      ? (const unsigned *)((const unsigned short *)p.state_in + (size_t)b * 3 * D + dc) : nullptr;

  unsigned raw[11];  // inputs t0+8rg-3 .. t0+8rg+7 of the channel pair
  auto load_rows = [&](int t0) __attribute__((always_inline)) {
    const int tb = t0 + 8 * rg - 3;
    if (tb >= 0 && tb + 11 <= T) {
#pragma unroll
      for (int n = 0; n < 11; ++n)
        raw[n] = __builtin_amdgcn_raw_buffer_load_b32(u_rsrc, u_voff, (unsigned)(tb + n) * row_bytes, 0);
    } else {  // first or last rows of the sequence (uniform over the wave)
#pragma unroll
      for (int n = 0; n < 11; ++n) {
        const int t = tb + n;
        unsigned v = 0;
        if (t >= 0) {
          if (t < T) v = __builtin_amdgcn_raw_buffer_load_b32(u_rsrc, u_voff, (unsigned)t * row_bytes, 0);
        } else if (st32) {
          v = st32[(size_t)ring_slot(pos0 + t) * (D / 2)];
        }
        raw[n] = v;
      }
    }
  };
  // the same for a tile after the first, free of branches (a load under a branch makes every
  // later wait on an older load a wait for all loads): no row lies before the sequence start,
  // and the row offset is part of the per-lane offset, which the descriptor's range check
  // covers - rows past the end of the sequence read as zero
  auto load_rows_inner = [&](int t0) __attribute__((always_inline)) {
    const unsigned base = u_voff + (unsigned)(t0 + 8 * rg - 3) * row_bytes;
#pragma unroll
    for (int n = 0; n < 11; ++n)
      raw[n] = __builtin_amdgcn_raw_buffer_load_b32(u_rsrc, pair_ok ? base + (unsigned)n * row_bytes : OOB, 0, 0);
  };
  // (without the epilogue nothing waits on an older load in between, and the version that
  // skips the loads of a tile that does not exist measured 3-4 % faster)
  auto next_rows = [&](int next) __attribute__((always_inline)) {
    if (MERGE == 0) {
      if (next < ntile) load_rows(next * TT);
    } else {
      load_rows_inner(next * TT);
    }
  };
  unsigned short *xw = xs + (8 * rg) * XS + 2 * c2;
  // (tl: the tile whose rows `raw` holds, mk: its mask word)
  auto conv_rows = [&](int buf, int tl, const u32x4m &mk) __attribute__((always_inline)) {
    const f32x4 w01 = cw_lds[c2], w23 = cw_lds[128 + c2], bb = cw_lds[256 + c2];
    // packed sequences: lags that reach in front of the row's document drop out (uniform over
    // the workgroup; tiles without a boundary nearby take the plain path)
    unsigned l1 = ~0u, l2 = ~0u, l3 = ~0u;
    if (PACKED) {
      l1 = mk[1]; l2 = mk[2]; l3 = mk[3];   // (rows past the end of the sequence: zero inputs either way)
    }
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      // (packed sequences: a select per lag on a scalar condition, no branch around the rows)
      const int bit = 8 * rg + r;
      const unsigned v1 = (!PACKED || ((l1 >> bit) & 1u)) ? raw[r + 2] : 0u;
      const unsigned v2 = (!PACKED || ((l2 >> bit) & 1u)) ? raw[r + 1] : 0u;
      const unsigned v3 = (!PACKED || ((l3 >> bit) & 1u)) ? raw[r] : 0u;
      float x0 = bb[0], x1 = bb[1];
      x0 = fmaf(w01[0], bf_lo(raw[r + 3]), x0); x1 = fmaf(w01[1], bf_hi(raw[r + 3]), x1);
      x0 = fmaf(w01[2], bf_lo(v1), x0);         x1 = fmaf(w01[3], bf_hi(v1), x1);
      x0 = fmaf(w23[0], bf_lo(v2), x0);         x1 = fmaf(w23[1], bf_hi(v2), x1);
      x0 = fmaf(w23[2], bf_lo(v3), x0);         x1 = fmaf(w23[3], bf_hi(v3), x1);
      unsigned hi_pk, lo_pk;
      split_f16(x0, x1, hi_pk, lo_pk);
      *(unsigned *)(xw + buf * (2 * XT_ELEMS) + r * XS) = hi_pk;
      *(unsigned *)(xw + buf * (2 * XT_ELEMS) + XT_ELEMS + r * XS) = lo_pk;
    }
  };

  // A-operand row of this lane: accumulator register r of lane half hf must be time hf*16+r
  const int arow = ((j >> 2) & 1) * 16 + (j >> 3) * 4 + (j & 3);
  const unsigned short *arow_base = xs + arow * XS + hf * 8;
  f32x4 *hold_mine = (f32x4 *)hold + (size_t)wv * 8 * 64 + lane;

  u64 *ring = GMAX > 1 ? a.rec + (size_t)unit * a.R * 2 * BS + ch : nullptr;
  float carry = p.h0 ? p.h0[(size_t)b * D + d] : 0.f;  // state after this workgroup's previous tile
  float aprod = 1.f;                                    // (aggregate pass) product of a_t so far
  // (a workspace that still reports an expired wait of an earlier call: no waiting, NaN throughout)
  int spins = (GMAX > 1 && expired_before(a.err)) ? SPIN_LIMIT : 0;

  // four consecutive steps (quarter q) of this lane's run: h <- a h + b, y = h (eq. 4); the
  // bf16 results go to the wave's staging tile at (row = step, column = channel)
  unsigned short *ot_mine = otile + (hf * 16) * OT + j;
  auto run_quarter = [&](int q, const f32x4 &av, const f32x4 &bv, float &h) __attribute__((always_inline)) {
    const float h0v = fmaf(av[0], h, bv[0]), h1v = fmaf(av[1], h0v, bv[1]);
    const float h2v = fmaf(av[2], h1v, bv[2]), h3v = fmaf(av[3], h2v, bv[3]);
    h = h3v;
    const unsigned p0 = pack_bf16(h0v, h1v), p1 = pack_bf16(h2v, h3v);
    unsigned short *o = ot_mine + (4 * q) * OT;
    o[0] = (unsigned short)(p0 & 0xffff);
    o[OT] = (unsigned short)(p0 >> 16);
    o[2 * OT] = (unsigned short)(p1 & 0xffff);
    o[3 * OT] = (unsigned short)(p1 >> 16);
  };
  // 16-byte stores of the staged tile: lane l owns 8 channels of rows l/4 and l/4+16
  const bool chunk_ok = !PAD || wv * 32 + (lane & 3) * 8 < bs;
  const unsigned yw_voff =
      chunk_ok ? (unsigned)(g * bs + wv * 32 + (lane & 3) * 8) * 2 + (unsigned)(lane >> 2) * row_bytes : OOB;

  // state of the held tile (its local scan sits in LDS until the next iteration)
  int held = -1;
  float hA_lo = 1.f, hH_lo = 0.f, hA_t = 1.f, hH_t = 0.f;  // aggregates of the tile parked in LDS
  // (each lane half fetches one of the two records of a tile, A below and H above, and the
  // halves swap them when the state is carried across: half the loads and registers)
  u64 rec[GMAX > 1 ? GMAX - 1 : 1];

  auto fetch_records = [&](int t) __attribute__((always_inline)) {  // aggregates of the G-1 tiles before tile t
#pragma unroll
    for (int s = 0; s < GMAX - 1; ++s) {
      const int k = t - (G - 1) + s;
      if (s < G - 1 && k >= 0) {
        rec[s] = peek(ring + (size_t)(k % a.R) * 2 * BS + hf * BS);
      }
    }
  };
  // finish tile t: carry the state across the tiles of the other slices, write y
  // the rows of the other branch that this lane merges into tile t: requested a whole step
  // before the tile is finished (rows outside the sequence are outside the descriptor's range
  // and read as zero, so any t may be asked for)
  u32x4 bq0 = {0, 0, 0, 0}, bq1 = {0, 0, 0, 0};
  auto fetch_branch = [&](int t) __attribute__((always_inline)) {
    if (MERGE) {
      const unsigned vo = yw_voff + (unsigned)(t * TT) * row_bytes;
      bq0 = __builtin_amdgcn_raw_buffer_load_b128(br_rsrc, chunk_ok ? vo : OOB, 0, RGLRU_NT);
      bq1 = __builtin_amdgcn_raw_buffer_load_b128(br_rsrc, chunk_ok ? vo + 16 * row_bytes : OOB, 0, RGLRU_NT);
    }
  };
  auto resolve = [&](int t) __attribute__((always_inline)) {
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
    float hrun = hf ? fmaf(hA_lo, h, hH_lo) : h;  // state entering this lane's run
#pragma unroll
    for (int q = 0; q < 4; ++q) run_quarter(q, hold_mine[q * 64], hold_mine[(q + 4) * 64], hrun);
    if (MERGE) {
      const int row = lane >> 2, chunk = lane & 3, nrows = T - t * TT;
      const unsigned soff = (unsigned)(t * TT) * row_bytes;
      const u32x4 v0 = *(const u32x4 *)(otile + row * OT + chunk * 8);
      const u32x4 v1 = *(const u32x4 *)(otile + (row + 16) * OT + chunk * 8);
      const u32x4 o0 = merge8<MERGE>(v0, bq0), o1 = merge8<MERGE>(v1, bq1);
      if (row < nrows) {
        __builtin_amdgcn_raw_buffer_store_b128(v0, y_rsrc, yw_voff, soff, 0);
        __builtin_amdgcn_raw_buffer_store_b128(o0, out_rsrc, yw_voff, soff, 0);
      }
      if (row + 16 < nrows) {
        __builtin_amdgcn_raw_buffer_store_b128(v1, y_rsrc, yw_voff, soff + 16 * row_bytes, 0);
        __builtin_amdgcn_raw_buffer_store_b128(o1, out_rsrc, yw_voff, soff + 16 * row_bytes, 0);
      }
    } else {
      store_staged_tile(otile, lane, y_rsrc, yw_voff, (unsigned)(t * TT) * row_bytes, row_bytes, T - t * TT);
    }
    carry = fmaf(hA_t, h, hH_t);
  };

  // ---- gate pre-activations of the tile in LDS buffer `buf` on the matrix cores, and the
  // tile's own columns (high + low part) moved into accumulator layout by selection
  f32x16 accp, accq, accx;
  auto gemm = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      accp[r] = bias_p;
      accq[r] = bias_q;
      accx[r] = 0.f;
    }
    const unsigned short *ap = arow_base + buf * (2 * XT_ELEMS);
    {
      f16x8 a0 = *(const f16x8 *)(ap), a1 = *(const f16x8 *)(ap + 16);
      // streamed W_x fragments: a ring of PF, all requested up front (the resident K-steps
      // come first, so the ring has that long to fill)
      f16x8 st[PF];
      if (NRES < 16) {
#pragma unroll
        for (int i = 0; i < PF; ++i) st[i] = pxs[kc(NRES + i < 16 ? NRES + i : 15) * 2];
      }
#pragma unroll
      for (int ks = 0; ks < 16; ++ks) {
        const f16x8 a2 = *(const f16x8 *)(ap + ((ks + 2) & 15) * 16);  // two steps ahead
        accp = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, wa[ks], accp, 0, 0, 0);
        if (ks < NRES) {
          accq = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, wx[ks], accq, 0, 0, 0);
        } else {
          accq = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, st[(ks - NRES) % PF], accq, 0, 0, 0);
          if (ks + PF < 16) st[(ks - NRES) % PF] = pxs[kc(ks + PF) * 2];
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
  };

  // ---- everything after the products for tile `tl`, whose pre-activations sit in the
  // accumulators: finish the tile parked one step earlier, gates, aggregates, publication
  auto pointwise = [&](int tl, unsigned starts) __attribute__((always_inline)) {
    const int t0 = tl * TT;
    if (GMAX > 1 && held >= 0) resolve(held);

    // gates (eqs. 1-3); the (a_t, b_t) pairs go to LDS, the lane keeps the aggregate of
    // its 16-step run: prun = prod a, hrun = end state for a zero incoming state
    float hrun = 0.f, prun = 1.f;
    // (starts: the steps of this tile that start a document, packed sequences only)
    if (T - t0 >= TT && starts == 0u) {  // full tile without a boundary (uniform over the workgroup)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        f32x4 aq, bq;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float av, bv;
          gate_fast(accp[4 * q + e], accq[4 * q + e], accx[4 * q + e], kd, av, bv);
          hrun = fmaf(av, hrun, bv);
          prun *= av;
          aq[e] = av;
          bq[e] = bv;
        }
        if (!AGG) {
          hold_mine[q * 64] = aq;
          hold_mine[(q + 4) * 64] = bq;
        }
      }
    } else {
      const int nvalid = T - t0 - hf * 16;
      const unsigned st16 = hf ? starts >> 16 : starts;   // this lane's 16 steps
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        f32x4 aq, bq;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float av, bv;
          gate_fast(accp[4 * q + e], accq[4 * q + e], accx[4 * q + e], kd, av, bv);
          if (4 * q + e >= nvalid) {  // steps past the end of the sequence leave the state untouched
            av = 1.f;
            bv = 0.f;
          }
          // a document's first step starts from h_{t-1} = 0: nothing is carried into it (its
          // own input still enters with sqrt(1 - a_t^2) of the true a_t)
          if (PACKED && ((st16 >> (4 * q + e)) & 1u)) av = 0.f;
          hrun = fmaf(av, hrun, bv);
          prun *= av;
          aq[e] = av;
          bq[e] = bv;
        }
        if (!AGG) {
          hold_mine[q * 64] = aq;
          hold_mine[(q + 4) * 64] = bq;
        }
      }
    }
    // combine the two lane halves: lower half = steps 0..15, upper = 16..31
    {
      const float oA = __shfl_xor(prun, 32), oH = __shfl_xor(hrun, 32);
      hA_lo = hf ? oA : prun;
      hH_lo = hf ? oH : hrun;
      const float A_up = hf ? prun : oA, H_up = hf ? hrun : oH;
      hA_t = hA_lo * A_up;
      hH_t = fmaf(A_up, hH_lo, H_up);
    }
    if (GMAX > 1) {
      // publish the aggregate: lower half writes A, upper half writes H
      publish(ring + (size_t)(tl % a.R) * 2 * BS + hf * BS, hf ? hH_t : hA_t, (unsigned)(tl + 1));
      held = tl;
    } else if (AGG) {   // only the window's aggregate is wanted
      carry = fmaf(hA_t, carry, hH_t);
      aprod *= hA_t;
    } else {
      resolve(tl);
    }
  };

  // The two waves that share a SIMD run half a step apart: waves 4-7 multiply first and then do
  // the pointwise work of the same tile, waves 0-3 do the pointwise work of their previous tile
  // first and multiply afterwards, keeping the accumulators across the barrier. Matrix and
  // vector phases of the pair then overlap instead of colliding. (The SIMD serves its older
  // wave first; the late order is the longer chain, so waves 0-3 get it.)
  const bool late = wv < NWAVE / 2;

  int tile = w;
  if (tile < ntile) load_rows(tile * TT);
  __syncthreads();  // the constants parked in LDS are visible to every wave
  // Mask words of packed sequences: lanes 0..3 of a wave fetch the four dwords of a tile's word two
  // tiles ahead, as the first load of an iteration (a load consumed any sooner would make its
  // wait a wait for the prefetched rows and weight fragments behind it as well); the word reaches
  // the scalar registers by lane reads one iteration later. Tiles past the end read as zero.
  const __amdgpu_buffer_rsrc_t mk_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      uniform_ptr(PACKED ? (const void *)(a.rmask + (size_t)b * a.ntile) : (const void *)p.u), 0,
      PACKED ? (unsigned)a.ntile * 16u : 0u, 0x00020000);
  auto mask_fetch = [&](int tl) __attribute__((always_inline)) {
    return __builtin_amdgcn_raw_buffer_load_b32(mk_rsrc, (unsigned)(lane & 3) * 4u, (unsigned)tl * 16u, 0);
  };
  auto mask_word = [&](unsigned v) __attribute__((always_inline)) {
    u32x4m m;
    m[0] = __builtin_amdgcn_readlane(v, 0); m[1] = __builtin_amdgcn_readlane(v, 1);
    m[2] = __builtin_amdgcn_readlane(v, 2); m[3] = __builtin_amdgcn_readlane(v, 3);
    return m;
  };
  u32x4m mk0 = {0u, 0u, 0u, 0u};
  unsigned mv_next = 0u;   // (lanes 0..3) word of the tile after this iteration's
  if (PACKED) {
    mk0 = mask_word(mask_fetch(tile));
    mv_next = mask_fetch(tile + G);
  }
  if (tile < ntile) conv_rows(0, tile, mk0);
  unsigned st_cur = mk0[0], st_prev = 0u;   // starts of this iteration's tile and of the one before
  __syncthreads();

  // (two copies of the loop, one per order, so that the accumulators are live across the
  // barrier only where they have to be; both execute the same number of barriers)
  auto run = [&](auto late_c) __attribute__((always_inline)) {
    constexpr bool LATE = decltype(late_c)::value;
    int it = 0;
    for (; tile < ntile; tile += G, ++it) {
      const int buf = it & 1;
      const int next = tile + G;
      u32x4m mkn = {0u, 0u, 0u, 0u};
      unsigned mv_after = 0u;
      if (PACKED) mv_after = mask_fetch(next + G);
      if (!LATE) {
        // rows of the next tile: after the streamed W_x fragments (loads return in order, and
        // these are trips to HBM); they land during the pointwise work
        gemm(buf);
        next_rows(next);
        pointwise(tile, st_cur);
        fetch_branch(GMAX > 1 ? held : next);   // for the tile that is finished next
      } else {
        if (it > 0) pointwise(tile - G, st_prev);
        fetch_branch(GMAX > 1 ? held : tile);
        next_rows(next);                              // lands during the products
        gemm(buf);
      }
      // next tile of this workgroup into the other LDS buffer
      // (the word of the next tile is read where the tile's rows are waited for anyway)
      if (PACKED) mkn = mask_word(mv_next);
      if (next < ntile) conv_rows(buf ^ 1, next, mkn);
      st_prev = st_cur;
      st_cur = mkn[0];
      mv_next = mv_after;
      // aggregates the parked tile will need: requested here, a whole step before their use and
      // clear of the streamed weight fragments (loads return in order); the other slices
      // published them earlier in this step
      if (GMAX > 1 && held >= 0) fetch_records(held);
      __syncthreads();
    }
    if (LATE && it > 0) {
      pointwise(tile - G, st_prev);
      if (GMAX > 1) fetch_branch(held);
    }
  };
  if (GMAX == 1 && !late) fetch_branch(tile);
  if (late) run(std::true_type{});
  else run(std::false_type{});
  if (GMAX > 1 && held >= 0) {
    fetch_records(held);
    resolve(held);
    if (spins >= SPIN_LIMIT) mark_expired(a.err);
  }

  // the workgroup that ran the last tile owns the final states
  if (AGG) {
    if (hf == 0 && ch_ok) {
      p.hT[(size_t)b * D + d] = carry;
      a.aprod[(size_t)b * D + d] = aprod;
    }
  } else if ((ntile - 1) % G == w && win == nwin - 1) {   // (of contiguous windows, the sequence's last)
    if (p.hT && hf == 0 && ch_ok) p.hT[(size_t)ob * D + d] = carry;
    if (p.state_out && tid < 128 && pair_ok) {
      // ring slots of the last three inputs; older slots are carried over (Appendix F state)
      unsigned *so32 = (unsigned *)((unsigned short *)p.state_out + (size_t)ob * 3 * D + dc);
      const long long end = pos0 + T;
#pragma unroll
      for (int slot = 0; slot < 3; ++slot) {
        const long long npos = end - 1 - ring_slot(end - 1 - slot);
        unsigned v = 0;
        if (npos >= pos0)
          v = __builtin_amdgcn_raw_buffer_load_b32(u_rsrc, u_voff, (unsigned)(npos - pos0) * row_bytes, 0);
        else if (st32)
          v = st32[(size_t)slot * (D / 2)];
        if (PACKED) {   // an input in front of the last document's first step is not part of its history
          const long long first = npos - pos0 + 1;   // (at least T - 2)
          for (int t = first > 0 ? (int)first : 0; t < T; ++t)
            if (p.reset[(size_t)b * T + t]) v = 0;
        }
        so32[(size_t)slot * (D / 2)] = v;
      }
    }
  }
}


// ------------------------------------------------------------------------------ decode
// One decode step (Section 5; states of Appendix F) for a tile of 32 sequences and one gate
// block: the rows of the MFMA tile are sequences instead of time steps. The ring slot of the
// new token is the slot of the lag-3 input, which the same thread has just read.
// LDS of the decode kernel: x tile (high, low) | selection operands | per wave: two buffers
// (W_a, W_x) in which a quarter (4 K-steps) of the wave's 32 weight rows is turned into MFMA
// fragment order, and one staging tile through which h (in, then out) and y move between 16-byte-per-lane
// global accesses and the accumulator layout
constexpr int DEC_WROW = 128 + 16;               // row stride: conflict-free 16-byte reads down a column
constexpr int DEC_WPH = 32 * DEC_WROW;           // 32 rows x (4 K-steps of weights | 32 fp32 of h)
constexpr int DEC_OFF_W = 2 * XT_ELEMS * 2 + 64 * 32;
constexpr int DEC_OFF_H = DEC_OFF_W + NWAVE * 2 * DEC_WPH;
constexpr int DEC_LDS = DEC_OFF_H + NWAVE * DEC_WPH;
constexpr int DEC_YROW = 64 + 16;                // y staging rows (32 bf16), in weight buffer 0

struct DecArgs {
  Problem p;   // u = u_t [B][D], hT = h [B][D] (in place), state_out = ring (in place), y = y_t
};

// One decode step (eqs. (1)-(4) at T = 1 on top of the Conv1D ring): a workgroup takes 32
// sequences of one gate block. The step is latency-bound, so the kernel is built around the
// memory pipeline: every access is 16 bytes per lane (a CU issues about one vector-memory
// instruction per 8 cycles whatever its width, and moves 64 bytes per cycle), loads are
// requested as early as registers allow, and nothing is loaded under a branch (that would make the compiler drain all
// outstanding loads on the spot) - rows past the batch get an out-of-range buffer offset
// instead: they read as zero and their stores are dropped.
// MERGE = 1 / 2: the block's merge as epilogue, y_t * GeLU(branch_t) is what is written.
// PAD: gate blocks narrower than 256 channels in the 256-wide tile, as in the forward kernel.
// PERSEQ: a position per sequence; the ring slots then differ from row to row and travel in the
// per-lane offsets.
template <int MERGE, bool PAD, bool PERSEQ = false>
__global__ void __launch_bounds__(NTHR) __attribute__((amdgpu_waves_per_eu(2, 2)))
decode_mfma_kernel(DecArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned short *xs = (unsigned short *)smem;                       // [high, low][32][XS]
  bf16x8 *sel_lds = (bf16x8 *)(smem + 2 * XT_ELEMS * 2);
  using u32x4 = unsigned __attribute__((ext_vector_type(4)));
  const Problem &p = a.p;
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5, j = lane & 31;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = blockIdx.x, b0 = blockIdx.y * TT;
  const int D = p.D, B = p.B;
  const int bs = PAD ? p.bs : BS;
  const int ch = wv * 32 + j, d = g * bs + ((!PAD || ch < bs) ? ch : bs - 1);

  constexpr unsigned OOB = 0x80000000u;
  const unsigned row2 = (unsigned)D * 2;
  const __amdgpu_buffer_rsrc_t u_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      uniform_ptr(p.u), 0, (unsigned)B * row2, 0x00020000);
  const __amdgpu_buffer_rsrc_t ring_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      uniform_ptr(p.state_out), 0, 3u * (unsigned)B * row2, 0x00020000);
  const __amdgpu_buffer_rsrc_t h_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      uniform_ptr(p.hT), 0, 2u * (unsigned)B * row2, 0x00020000);
  const __amdgpu_buffer_rsrc_t y_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      uniform_ptr(p.y), 0, (unsigned)B * row2, 0x00020000);

  // ---- Conv1D assignment: 8 channels (16 bytes) of rows (sequences) lr and lr + 16 of the tile
  const int lc = tid & 31, lr = tid >> 5;
  const bool lc_ok = !PAD || 8 * lc < bs;           // missing channels: no input, x = 0
  const int dc = g * bs + (lc_ok ? 8 * lc : 0);
  // per-channel vectors first (loads return in order, and these are needed first)
  f32x4 cw[4][2], cb[2];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    cw[k][0] = *(const f32x4 *)(p.conv_w + (size_t)k * D + dc);
    cw[k][1] = *(const f32x4 *)(p.conv_w + (size_t)k * D + dc + 4);
  }
  {
    const float *cbp = (p.conv_b ? p.conv_b : p.conv_w) + dc;
    cb[0] = *(const f32x4 *)cbp;
    cb[1] = *(const f32x4 *)(cbp + 4);
  }
  const float cb_on = (p.conv_b && lc_ok) ? 1.f : 0.f;
  const float bias_p = p.b_a[d] * LOG2E, bias_q = p.b_x[d] * LOG2E, lam = p.Lambda[d];

  const int s1 = ring_slot(p.pos0 - 1), s2 = ring_slot(p.pos0 - 2), s3 = ring_slot(p.pos0 - 3);
  u32x4 ru[2][4];
  unsigned ring_vo[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int b = b0 + lr + 16 * i;
    const bool ok = b < B && lc_ok;
    const unsigned uvo = ok ? (unsigned)b * row2 + (unsigned)dc * 2 : OOB;
    const unsigned rvo = ok ? (unsigned)(b * 3) * row2 + (unsigned)dc * 2 : OOB;
    ru[i][0] = __builtin_amdgcn_raw_buffer_load_b128(u_rsrc, uvo, 0, 0);
    if (PERSEQ) {
      const long long pb = p.pos_rows[b < B ? b : B - 1];
      const unsigned q1 = ring_slot(pb - 1), q2 = ring_slot(pb - 2), q3 = ring_slot(pb - 3);
      ring_vo[i] = ok ? rvo + q3 * row2 : OOB;   // where the new token goes
      ru[i][1] = __builtin_amdgcn_raw_buffer_load_b128(ring_rsrc, ok ? rvo + q1 * row2 : OOB, 0, 0);
      ru[i][2] = __builtin_amdgcn_raw_buffer_load_b128(ring_rsrc, ok ? rvo + q2 * row2 : OOB, 0, 0);
      ru[i][3] = __builtin_amdgcn_raw_buffer_load_b128(ring_rsrc, ring_vo[i], 0, 0);
      continue;
    }
    ring_vo[i] = rvo;
    ru[i][1] = __builtin_amdgcn_raw_buffer_load_b128(ring_rsrc, rvo, (unsigned)s1 * row2, 0);
    ru[i][2] = __builtin_amdgcn_raw_buffer_load_b128(ring_rsrc, rvo, (unsigned)s2 * row2, 0);
    ru[i][3] = __builtin_amdgcn_raw_buffer_load_b128(ring_rsrc, rvo, (unsigned)s3 * row2, 0);
  }

  // ---- gate weights of this wave's 32 output channels. A fragment read straight from the
  // row-major matrix touches 64 cache lines per instruction; instead the wave reads its rows
  // (16 KB contiguous per gate) in four phases of four K-steps of both gates, whole 128-byte
  // lines per 8 lanes, and turns each phase into fragment order through its own LDS buffers
  // (one per gate; LDS serves a wave's accesses in order, so a phase may be written while the
  // reads of the previous one are still queued). One phase is requested here, the next once
  // the Conv1D inputs are in (more would only delay those, queued behind).
  // (missing rows and K-steps of a narrower block are read from existing ones: they meet
  // zeros in x or end in outputs that are dropped)
  const unsigned char *wrow_a = (const unsigned char *)p.W_a + (size_t)g * bs * bs * 2;
  const unsigned char *wrow_x = (const unsigned char *)p.W_x + (size_t)g * bs * bs * 2;
  unsigned w_row[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = wv * 32 + i * 8 + (lane >> 3);
    w_row[i] = (unsigned)((!PAD || r < bs) ? r : bs - 1) * (unsigned)(bs * 2);
  }
  unsigned char *wl = smem + DEC_OFF_W + wv * 2 * DEC_WPH;
  const unsigned wl_wr = (unsigned)(lane >> 3) * DEC_WROW + (unsigned)(lane & 7) * 16;
  const unsigned wl_rd = (unsigned)j * DEC_WROW + (unsigned)hf * 16;
  u32x4 stg[2][8];
  auto load_phase = [&](int ph, u32x4 (&dst)[8]) __attribute__((always_inline)) {
    const int c = ph * 8 + (lane & 7);   // 16-byte chunk of the row
    const unsigned w_col = (unsigned)((!PAD || c < (bs >> 3)) ? c : (bs >> 3) - 1) * 16;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      dst[i] = *(const u32x4 *)(wrow_a + w_row[i] + w_col);
      dst[4 + i] = *(const u32x4 *)(wrow_x + w_row[i] + w_col);
    }
  };
  auto write_phase = [&](const u32x4 (&src)[8]) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      *(u32x4 *)(wl + i * 8 * DEC_WROW + wl_wr) = src[i];
      *(u32x4 *)(wl + DEC_WPH + i * 8 * DEC_WROW + wl_wr) = src[4 + i];
    }
  };
  load_phase(0, stg[0]);

  // ---- recurrent state of this wave's 32 x 32 tile: lane l takes 16 bytes of rows l/8 + 8i
  unsigned char *hl = smem + DEC_OFF_H + wv * DEC_WPH;
  const unsigned hl_wide = (unsigned)(lane >> 3) * DEC_WROW + (unsigned)(lane & 7) * 16;
  unsigned h_vo[4];
  u32x4 hin[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int b = b0 + (lane >> 3) + 8 * i;
    const bool ok = b < B && (!PAD || wv * 32 + (lane & 7) * 4 < bs);
    h_vo[i] = ok ? ((unsigned)b * (unsigned)D + (unsigned)(g * bs + wv * 32 + (lane & 7) * 4)) * 4 : OOB;
    hin[i] = __builtin_amdgcn_raw_buffer_load_b128(h_rsrc, h_vo[i], 0, 0);
  }
  // where this lane's 16 bytes of y (rows l/4 and l/4 + 16) go; the other branch is read there
  unsigned y_vo[2];
  u32x4 brq[2];
  const __amdgpu_buffer_rsrc_t br_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      uniform_ptr(MERGE ? p.branch : p.u), 0, (unsigned)B * row2, 0x00020000);
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int b = b0 + (lane >> 2) + 16 * i;
    const bool ok = b < B && (!PAD || wv * 32 + (lane & 3) * 8 < bs);
    y_vo[i] = ok ? ((unsigned)b * (unsigned)D + (unsigned)(g * bs + wv * 32 + (lane & 3) * 8)) * 2 : OOB;
    if (MERGE) brq[i] = __builtin_amdgcn_raw_buffer_load_b128(br_rsrc, y_vo[i], 0, 0);
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
  float kd;
  {
    const float z = -lam;
    const float sp = z > 0.f ? z + log1pf(expf(-z)) : log1pf(expf(z));
    kd = -p.c * sp * LOG2E;
  }

  // ---- Conv1D over the ring; the new token replaces the oldest slot
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    u32x4 hi4, lo4;
#pragma unroll
    for (int e = 0; e < 4; ++e) {   // channels 2e, 2e+1 of the 8
      const int v = e >> 1, c0 = (2 * e) & 3;
      const unsigned u0 = ru[i][0][e], u1 = ru[i][1][e], u2 = ru[i][2][e], u3 = ru[i][3][e];
      float x0 = cb[v][c0] * cb_on, x1 = cb[v][c0 + 1] * cb_on;
      x0 = fmaf(cw[0][v][c0], bf_lo(u0), x0); x1 = fmaf(cw[0][v][c0 + 1], bf_hi(u0), x1);
      x0 = fmaf(cw[1][v][c0], bf_lo(u1), x0); x1 = fmaf(cw[1][v][c0 + 1], bf_hi(u1), x1);
      x0 = fmaf(cw[2][v][c0], bf_lo(u2), x0); x1 = fmaf(cw[2][v][c0 + 1], bf_hi(u2), x1);
      x0 = fmaf(cw[3][v][c0], bf_lo(u3), x0); x1 = fmaf(cw[3][v][c0 + 1], bf_hi(u3), x1);
      unsigned hi_pk, lo_pk;
      split_bf16(x0 * LOG2E, x1 * LOG2E, hi_pk, lo_pk);   // rows past the batch: all inputs read as zero
      hi4[e] = hi_pk;
      lo4[e] = lo_pk;
    }
    // slot pos mod 3 == slot (pos-3) mod 3
    __builtin_amdgcn_raw_buffer_store_b128(ru[i][0], ring_rsrc, ring_vo[i], PERSEQ ? 0u : (unsigned)s3 * row2, 0);
    *(u32x4 *)(xs + (lr + 16 * i) * XS + 8 * lc) = hi4;
    *(u32x4 *)(xs + XT_ELEMS + (lr + 16 * i) * XS + 8 * lc) = lo4;
  }
  load_phase(1, stg[1]);
  // GeLU of the other branch now, while the weights are on their way: the step is
  // latency-bound and the vector unit idle here, at the end it would be on the critical path
  float gl[2][8];
  if (MERGE) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        gl[i][2 * k] = gelu<MERGE == 2, true>(bf_lo(brq[i][k]));
        gl[i][2 * k + 1] = gelu<MERGE == 2, true>(bf_hi(brq[i][k]));
      }
  }
  __syncthreads();

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
#pragma unroll
  for (int ph = 0; ph < 4; ++ph) {
    if (ph + 2 < 4) load_phase(ph + 2, stg[ph & 1]);
    // the fragments come from other lanes of this wave
    wave_lds_fence();
    bf16x8 av[4], fa[4], fx[4];
#pragma unroll
    for (int k2 = 0; k2 < 4; ++k2) {
      av[k2] = *(const bf16x8 *)(ap + (ph * 4 + k2) * 16);
      fa[k2] = *(const bf16x8 *)(wl + wl_rd + k2 * 32);
      fx[k2] = *(const bf16x8 *)(wl + DEC_WPH + wl_rd + k2 * 32);
    }
    wave_lds_fence();
    if (ph + 1 < 4) write_phase(stg[(ph + 1) & 1]);
#pragma unroll
    for (int k2 = 0; k2 < 4; ++k2) {   // two independent accumulation chains
      accp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[k2], fa[k2], accp, 0, 0, 0);
      accq = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[k2], fx[k2], accq, 0, 0, 0);
    }
  }
  accx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(ap + (2 * wv) * 16), sel_lds[lane], accx, 0, 0, 0);
  accx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(ap + (2 * wv + 1) * 16), sel_lds[64 + lane], accx, 0, 0, 0);
  accx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(ap + XT_ELEMS + (2 * wv) * 16), sel_lds[lane], accx, 0, 0, 0);
  accx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(ap + XT_ELEMS + (2 * wv + 1) * 16), sel_lds[64 + lane], accx, 0, 0, 0);

  // ---- h into accumulator layout: lane (j, hf) owns channel j of rows 16 hf .. 16 hf + 15
#pragma unroll
  for (int i = 0; i < 4; ++i) *(u32x4 *)(hl + i * 8 * DEC_WROW + hl_wide) = hin[i];
  wave_lds_fence();
  float rh[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) rh[r] = *(const float *)(hl + (hf * 16 + r) * DEC_WROW + j * 4);
  wave_lds_fence();

  // ---- eq. (4) for the 16 sequences of this lane's run; results back through the staging tiles
  unsigned char *yl = wl;   // weight buffer 0 of this wave is free again
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    float av_, bv;
    gate_fast(accp[r], accq[r], accx[r], kd, av_, bv);
    const float hn = fmaf(av_, rh[r], bv);
    *(float *)(hl + (hf * 16 + r) * DEC_WROW + j * 4) = hn;
    *(unsigned short *)(yl + (hf * 16 + r) * DEC_YROW + j * 2) = (unsigned short)(pack_bf16(hn, 0.f) & 0xffff);
  }
  wave_lds_fence();
#pragma unroll
  for (int i = 0; i < 4; ++i)
    __builtin_amdgcn_raw_buffer_store_b128(*(const u32x4 *)(hl + i * 8 * DEC_WROW + hl_wide), h_rsrc, h_vo[i], 0, 0);
#pragma unroll
  for (int i = 0; i < 2; ++i) {   // lane l: 16 bytes of rows l/4 + 16 i
    const int row = (lane >> 2) + 16 * i;
    u32x4 yv = *(const u32x4 *)(yl + row * DEC_YROW + (lane & 3) * 16);
    if (MERGE) {
#pragma unroll
      for (int k = 0; k < 4; ++k)
        yv[k] = pack_bf16(bf_lo(yv[k]) * gl[i][2 * k], bf_hi(yv[k]) * gl[i][2 * k + 1]);
    }
    __builtin_amdgcn_raw_buffer_store_b128(yv, y_rsrc, y_vo[i], 0, 0);
  }
}

}  // namespace

// ------------------------------------------------------------------------------ host side
static int g_num_cu = 0;

int mfma::num_cu() {
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

hipError_t mfma::launch_prep(void *zero, size_t zero_bytes, hipStream_t s, bool keep_status) {
  const size_t n16 = zero_bytes / 16;
  KernelTimer kt("prep_kernel", s);
  hipLaunchKernelGGL(prep_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, s, (uint4 *)zero, n16, keep_status);
  return hipGetLastError();
}

// gate block sizes the forward kernel takes: 256 channels, or narrower blocks (a multiple of 16,
// at least half the tile: below that the padding costs more than the generic kernels)
hipError_t launch_clear(void *at, size_t bytes, hipStream_t s) { return launch_prep(at, bytes, s); }

bool forward_mfma_block(int bs) { return bs == BS || (bs % 16 == 0 && bs >= BS / 2 && bs < BS); }

bool forward_mfma_supported(const Problem &p, bool bf) {
  // (the narrower blocks mark dropped accesses with an offset of 2^31)
  const bool block_ok = forward_mfma_block(p.bs) && (p.bs == BS || (size_t)p.T * p.D * 2 < ((size_t)1 << 31));
  return bf && block_ok && p.T >= 1 && (size_t)p.T * p.D * 2 < ((size_t)1 << 32) &&
         ((uintptr_t)p.W_a % 16 == 0) && ((uintptr_t)p.W_x % 16 == 0) && ((uintptr_t)p.u % 4 == 0) &&
         ((uintptr_t)p.y % 16 == 0) &&
         (!p.merge || ((uintptr_t)p.branch % 16 == 0 && (uintptr_t)p.out % 16 == 0)) &&
         (!p.state_in || (uintptr_t)p.state_in % 4 == 0) &&
         (!p.state_out || (uintptr_t)p.state_out % 4 == 0);
}

// Whether the merge runs as the forward kernel's epilogue. With more than 8 time slices per
// sequence the kernel has no registers left for it (every W_x fragment is then re-read per
// tile) and the merge as a streaming kernel of its own measured faster.
static int contiguous_windows(int units, int ntile, int ncu, bool packed, int *tiles_per);
bool forward_mfma_merge_fused(const Problem &p) {
  int ncu = num_cu();
  if (ncu > 256) ncu = 256;
  // (contiguous windows run the kernel of unsliced sequences, which has the epilogue)
  if (contiguous_windows(p.B * p.nb, (p.T + TT - 1) / TT, ncu, p.reset != nullptr, nullptr)) return true;
  return pick_slices(p.B * p.nb, (p.T + TT - 1) / TT, ncu, FWD_MAX_SLICES) <= 8;
}

// time slices per (sequence, block): as many as keep every workgroup resident at once, at
// most 8 (every tile reads the aggregates of the G-1 tiles before it)
static std::atomic<int> g_slice_cap{0};
void mfma::set_slice_cap(int cap) { g_slice_cap.store(cap); }

int mfma::pick_slices(int units, int ntile, int ncu, int cap) {
  int G = ncu / units;
  if (G < 1) G = 1;
  if (G > ntile) G = ntile;
  if (G > cap) G = cap;
  const int user = g_slice_cap.load();
  if (user > 0 && G > user) G = user;
  return G;
}

// Long sequences of very few units (a single prompt: B * nb of 12 or less) are cut into
// contiguous windows instead, as many as there are compute units, and run in two passes - the
// windows' aggregates (decay product, end state from zero) first, then, once a short chain has
// turned them into every window's incoming state, the forward proper. That doubles the
// arithmetic but nothing is exchanged between running workgroups. Interleaved slices read G - 1
// records per tile and stop at 16 slices (7.2 us per workgroup and tile there, against 3.5 + 4.3 us
// for the two passes of a window's tile on a full chip), so the two passes win where they put
// 21 or more compute units on a sequence's block instead of 16 and the sequence is long enough to
// pay for three more launches (measured: B = 1, T = 32768, 10 blocks 467 -> 344 us; 16 or 20
// units: 5-8 % slower, left to the interleaved scheme). Returns the number of windows, or 0.
constexpr int WIN_MAX_UNITS = 12, WIN_MIN_TILES = 384;
static int contiguous_windows(int units, int ntile, int ncu, bool packed, int *tiles_per) {
  if (packed || units > WIN_MAX_UNITS || ntile < WIN_MIN_TILES) return 0;
  int S = ncu / units;
  if (S > ntile / 4) S = ntile / 4;
  const int user = g_slice_cap.load();
  if (user > 0 && S > user) S = user;
  if (S < 2) return 0;
  const int per = (ntile + S - 1) / S;
  S = (ntile + per - 1) / per;    // no empty window
  if (tiles_per) *tiles_per = per;
  return S >= 2 ? S : 0;
}
static size_t al256(size_t n) { return (n + 255) & ~(size_t)255; }

// Workspace: one record ring per unit when the sequence is sliced in time, or the windows'
// rings, incoming states and aggregates. Sized for the worst case of 256 compute units so that
// it does not depend on the device.
static size_t fwd_rec_bytes(int B, int T, int D, int nb) {   // status word + the above, 256-byte granules
  const int units = B * nb, ntile = (T + TT - 1) / TT;
  const int G = pick_slices(units, ntile, 256, FWD_MAX_SLICES);
  const size_t R = 8 * (size_t)G;
  size_t n = G == 1 ? 0 : (size_t)units * R * 2 * BS * sizeof(u64);
  // (whatever the user's cap on the slices is when the size is asked for: the largest count)
  int S = 256 / units;
  if (S > ntile / 4) S = ntile / 4;
  if (units <= WIN_MAX_UNITS && ntile >= WIN_MIN_TILES && S >= 2) {
    const size_t w = al256((size_t)B * S * 3 * D * 2) + 3 * al256((size_t)B * S * D * 4);
    if (w > n) n = w;
  }
  return 256 + n;
}
// ... followed by W_x in half precision
size_t forward_mfma_ws_bytes(int B, int T, int D, int nb) {
  const size_t w = (size_t)D * (D / nb) * 2;
  return fwd_rec_bytes(B, T, D, nb) + ((w + 255) & ~(size_t)255);
}

hipError_t mfma::launch_reset_masks(const unsigned char *reset, uint4 *masks, unsigned char *nlag, int B, int T,
                                    hipStream_t s) {
  const int ntile = (T + TT - 1) / TT, n = B * ntile;
  hipLaunchKernelGGL(reset_mask_kernel, dim3((n + 255) / 256), dim3(256), 0, s, reset, masks, nlag, B, T, ntile);
  return hipGetLastError();
}

// ... and, for packed sequences, by the boundary masks
size_t forward_mfma_mask_bytes(int B, int T) {
  const size_t n = (size_t)B * ((T + TT - 1) / TT) * sizeof(uint4);
  return (n + 255) & ~(size_t)255;
}

template <int GMAX, int MERGE, bool PAD>
static hipError_t launch_tmp(const FwdArgs &a, int grid, size_t lds, hipStream_t s) {
  static bool configured = false;  // the kernel asks for more than the default LDS limit
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void *)fwd_mfma_kernel<GMAX, MERGE, PAD>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       FWD_LDS);
    if (e != hipSuccess) return e;
    configured = true;
  }
  KernelTimer kt(MERGE ? "fwd_merge_mfma_kernel" : "fwd_mfma_kernel", s);
  hipLaunchKernelGGL((fwd_mfma_kernel<GMAX, MERGE, PAD>), dim3(grid), dim3(NTHR), lds, s, a);
  return hipGetLastError();
}
template <int GMAX, bool PAD>
static hipError_t launch_packed_tp(const FwdArgs &a, int grid, size_t lds, hipStream_t s) {
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void *)fwd_mfma_kernel<GMAX, 0, PAD, true>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, FWD_LDS);
    if (e != hipSuccess) return e;
    configured = true;
  }
  KernelTimer kt("fwd_packed_mfma_kernel", s);
  hipLaunchKernelGGL((fwd_mfma_kernel<GMAX, 0, PAD, true>), dim3(grid), dim3(NTHR), lds, s, a);
  return hipGetLastError();
}
template <bool PAD>
static hipError_t launch_agg_tp(const FwdArgs &a, int grid, size_t lds, hipStream_t s) {
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void *)fwd_mfma_kernel<1, 0, PAD, false, true>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, FWD_LDS);
    if (e != hipSuccess) return e;
    configured = true;
  }
  KernelTimer kt("fwd_agg_mfma_kernel", s);
  hipLaunchKernelGGL((fwd_mfma_kernel<1, 0, PAD, false, true>), dim3(grid), dim3(NTHR), lds, s, a);
  return hipGetLastError();
}
template <int GMAX, int MERGE>
static hipError_t launch_tm(const FwdArgs &a, int grid, size_t lds, hipStream_t s) {
  return a.p.bs == BS ? launch_tmp<GMAX, MERGE, false>(a, grid, lds, s)
                      : launch_tmp<GMAX, MERGE, true>(a, grid, lds, s);
}
template <int GMAX>
static hipError_t launch_t(const FwdArgs &a, int grid, size_t lds, hipStream_t s) {
  if (a.rmask)   // (the packed entry point has no merge epilogue)
    return a.p.bs == BS ? launch_packed_tp<GMAX, false>(a, grid, lds, s) : launch_packed_tp<GMAX, true>(a, grid, lds, s);
  return a.p.merge == 0 ? launch_tm<GMAX, 0>(a, grid, lds, s)
       : a.p.merge == 1 ? launch_tm<GMAX, 1>(a, grid, lds, s)
                        : launch_tm<GMAX, 2>(a, grid, lds, s);
}

hipError_t launch_forward_mfma(const Problem &p, hipStream_t s) {
  FwdArgs a;
  a.p = p;
  const int units = p.B * p.nb;
  a.ntile = (p.T + TT - 1) / TT;
  int ncu = num_cu();
  if (ncu > 256) ncu = 256;  // the workspace is sized for at most 256 resident workgroups
  int tiles_per = 0;
  const int S = contiguous_windows(units, a.ntile, ncu, p.reset != nullptr, &tiles_per);
  a.S = 1;
  a.Ts = p.T;
  a.aprod = nullptr;
  a.G = S ? 1 : pick_slices(units, a.ntile, ncu, FWD_MAX_SLICES);
  a.R = 8 * a.G;
  const int grid = units * a.G;
  a.swizzle = (a.G > 1 && grid % 8 == 0) ? 1 : 0;
  // workspace: status word, record rings (sized for 256 compute units), W_x in half precision
  unsigned short *wx16 = (unsigned short *)((char *)p.ws + fwd_rec_bytes(p.B, p.T, p.D, p.nb));
  a.wx16 = wx16;
  const size_t n8 = (size_t)p.D * p.bs / 8;
  const size_t n16 = (a.G == 1 ? 256 : 256 + (size_t)units * a.R * 2 * BS * sizeof(u64)) / 16;
  {
    const size_t n = n8 > n16 ? n8 : n16;
    KernelTimer kt("prep_kernel", s);
    hipLaunchKernelGGL(fwd_prep_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (uint4 *)p.ws, n16,
                       (const uint4 *)p.W_x, (uint4 *)wx16, n8);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  a.rmask = nullptr;
  if (p.reset) {
    uint4 *masks = (uint4 *)((char *)p.ws + forward_mfma_ws_bytes(p.B, p.T, p.D, p.nb));
    hipError_t e = launch_reset_masks(p.reset, masks, nullptr, p.B, p.T, s);
    if (e != hipSuccess) return e;
    a.rmask = masks;
  }
  if (S) {   // contiguous windows in two passes (contiguous_windows)
    a.rec = nullptr;
    a.err = nullptr;
    a.S = S;
    a.Ts = tiles_per * TT;
    const size_t nw = (size_t)p.B * S;
    char *at = (char *)p.ws + 256;
    unsigned short *rings = (unsigned short *)at;
    at += al256(nw * 3 * p.D * 2);
    float *hin = (float *)at;
    at += al256(nw * p.D * 4);
    float *Hs = (float *)at;
    at += al256(nw * p.D * 4);
    float *As = (float *)at;
    WinArgs wa;
    wa.u = (const unsigned short *)p.u;
    wa.state_in = (const unsigned short *)p.state_in;
    wa.rings = rings;
    wa.B = p.B; wa.S = S; wa.Ts = a.Ts; wa.T = p.T; wa.D = p.D;
    wa.pos0 = p.pos0;
    hipError_t e;
    {
      KernelTimer kt("window_ring_kernel", s);
      const size_t n = nw * 3 * (p.D / 2);
      hipLaunchKernelGGL(window_ring_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, wa);
      if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    FwdArgs g = a;   // pass 1: aggregates of every window
    g.p.y = nullptr; g.p.out = nullptr; g.p.branch = nullptr; g.p.merge = 0;
    g.p.h0 = nullptr; g.p.state_in = rings; g.p.state_out = nullptr;
    g.p.hT = Hs;
    g.aprod = As;
    e = p.bs == BS ? launch_agg_tp<false>(g, units * S, FWD_LDS, s) : launch_agg_tp<true>(g, units * S, FWD_LDS, s);
    if (e != hipSuccess) return e;
    {
      KernelTimer kt("window_chain_kernel", s);
      const size_t n = (size_t)p.B * p.D;
      hipLaunchKernelGGL(window_chain_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                         (const float *)p.h0, (const float *)As, (const float *)Hs, hin, p.B, S, p.D);
      if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    a.p.h0 = hin;        // pass 2: the forward proper, every window from its own state
    a.p.state_in = rings;
    return launch_t<1>(a, units * S, FWD_LDS, s);
  }
  if (a.G == 1) {
    a.rec = nullptr;
    a.err = nullptr;
    return launch_t<1>(a, grid, FWD_LDS, s);
  }
  a.err = (int *)p.ws;
  a.rec = (u64 *)((char *)p.ws + 256);
  return a.G <= 4 ? launch_t<4>(a, grid, FWD_LDS, s)
       : a.G <= 8 ? launch_t<8>(a, grid, FWD_LDS, s)
                  : launch_t<16>(a, grid, FWD_LDS, s);
}

bool decode_mfma_supported(const Problem &p, bool bf) {
  // 16-byte accesses throughout; 32-bit byte offsets into the ring
  const uintptr_t all = (uintptr_t)p.W_a | (uintptr_t)p.W_x | (uintptr_t)p.u | (uintptr_t)p.state_out |
                        (uintptr_t)p.hT | (uintptr_t)p.y | (uintptr_t)p.conv_w | (uintptr_t)p.conv_b |
                        (uintptr_t)(p.merge ? p.branch : nullptr);
  // (a step without the Conv1D and its ring runs on the generic kernel)
  return bf && p.conv_w && forward_mfma_block(p.bs) && all % 16 == 0 &&
         (size_t)(p.B + TT) * 3 * p.D * 2 < ((size_t)1 << 31);
}

hipError_t launch_decode_mfma(const Problem &p, hipStream_t s) {
  DecArgs a;
  a.p = p;
  static bool configured = false;  // the kernel asks for more than the default LDS limit
  if (!configured) {
    hipError_t e;
    auto big = [](const void *k) { return hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, DEC_LDS); };
    if ((e = big((const void *)decode_mfma_kernel<0, false>)) != hipSuccess) return e;
    if ((e = big((const void *)decode_mfma_kernel<1, false>)) != hipSuccess) return e;
    if ((e = big((const void *)decode_mfma_kernel<2, false>)) != hipSuccess) return e;
    if ((e = big((const void *)decode_mfma_kernel<0, true>)) != hipSuccess) return e;
    if ((e = big((const void *)decode_mfma_kernel<1, true>)) != hipSuccess) return e;
    if ((e = big((const void *)decode_mfma_kernel<2, true>)) != hipSuccess) return e;
    if ((e = big((const void *)decode_mfma_kernel<0, false, true>)) != hipSuccess) return e;
    if ((e = big((const void *)decode_mfma_kernel<0, true, true>)) != hipSuccess) return e;
    configured = true;
  }
  KernelTimer kt("decode_mfma_kernel", s);
  const dim3 grid(p.nb, (p.B + TT - 1) / TT);
  if (p.pos_rows) {   // (callers pass no merge here)
    if (p.bs == BS) hipLaunchKernelGGL((decode_mfma_kernel<0, false, true>), grid, dim3(NTHR), DEC_LDS, s, a);
    else hipLaunchKernelGGL((decode_mfma_kernel<0, true, true>), grid, dim3(NTHR), DEC_LDS, s, a);
  } else if (p.bs == BS) {
    if (p.merge == 0) hipLaunchKernelGGL((decode_mfma_kernel<0, false>), grid, dim3(NTHR), DEC_LDS, s, a);
    else if (p.merge == 1) hipLaunchKernelGGL((decode_mfma_kernel<1, false>), grid, dim3(NTHR), DEC_LDS, s, a);
    else hipLaunchKernelGGL((decode_mfma_kernel<2, false>), grid, dim3(NTHR), DEC_LDS, s, a);
  } else {
    if (p.merge == 0) hipLaunchKernelGGL((decode_mfma_kernel<0, true>), grid, dim3(NTHR), DEC_LDS, s, a);
    else if (p.merge == 1) hipLaunchKernelGGL((decode_mfma_kernel<1, true>), grid, dim3(NTHR), DEC_LDS, s, a);
    else hipLaunchKernelGGL((decode_mfma_kernel<2, true>), grid, dim3(NTHR), DEC_LDS, s, a);
  }
  return hipGetLastError();
}


}  // namespace rglru
