// Device helpers shared by the MFMA kernels (bf16 storage, gate blocks of 256 channels).
#pragma once
#include "rglru_internal.h"

namespace rglru {
namespace mfma {

constexpr int BS = 256;          // gate block size this kernel is built for
constexpr int NWAVE = 8;         // waves per workgroup, 32 output channels each
constexpr int NTHR = NWAVE * 64;
constexpr int TT = 32;           // time steps per tile
constexpr int XS = BS + 8;       // LDS row stride in bf16 elements (528 B: conflict-free b128 reads)
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr int XT_ELEMS = TT * XS;                   // one [32][264] bf16 tile
constexpr int XS_BYTES = 4 * XT_ELEMS * 2;          // two buffers x (high part, low part) of the x tile
constexpr int CONST_BYTES = 64 * 32 + 128 * 48;      // selection operands + Conv1D taps per lane
constexpr int HOLD_BYTES = NWAVE * 64 * 32 * 4;     // local scan of one tile, per lane 32 floats
constexpr int OT = 40;                              // row stride (bf16) of a wave's output staging tile
constexpr int OTILE_BYTES = TT * OT * 2;            // [32 steps][32 channels] bf16 per wave
constexpr int SPIN_LIMIT = 1 << 22;
// Status word of a workspace whose kernels wait on each other (its first 16 bytes). A wait that
// expires writes this pattern; the outputs of that call are then filled with NaN from the point
// of the failure on, and so are those of every later call on the workspace (the preparation pass
// of a call keeps the word if and only if it holds exactly this pattern - whatever else an
// uninitialised workspace contains is cleared) until rglru_workspace_status has reported it.
#define RGLRU_EXPIRED_WORDS 0x4c474c52u, 0x58452d55u, 0x45524950u, 0xb3d3b3adu
__device__ __forceinline__ void mark_expired(int *status) {
  *(uint4 *)status = make_uint4(RGLRU_EXPIRED_WORDS);
}
__device__ __forceinline__ bool is_expired(const uint4 &w) {
  const uint4 m = make_uint4(RGLRU_EXPIRED_WORDS);
  return w.x == m.x && w.y == m.y && w.z == m.z && w.w == m.w;
}
// the status word at the start of a launch (uniform over the grid: nothing has written it yet)
__device__ __forceinline__ bool expired_before(const int *status) {
  return is_expired(*(const uint4 *)status);
}
// what the preparation pass leaves in 16-byte word i of a region whose first word is the status
__device__ __forceinline__ uint4 cleared_word(const uint4 *region, size_t i, bool keep_status) {
  if (keep_status && i == 0 && is_expired(region[0])) return region[0];
  return make_uint4(0, 0, 0, 0);
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned long long u64;

__device__ __forceinline__ float bf_lo(unsigned v) { return __uint_as_float(v << 16); }
__device__ __forceinline__ float bf_hi(unsigned v) { return __uint_as_float(v & 0xffff0000u); }
__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {  // v_cvt_pk_bf16_f32
  const f32x2 v = {lo, hi};
  const bf16x2 b = __builtin_convertvector(v, bf16x2);
  return *(const unsigned *)&b;
}
// x = high + low with both parts in bf16 (16 mantissa bits in total): packs two values
__device__ __forceinline__ void split_bf16(float x0, float x1, unsigned &hi_pk, unsigned &lo_pk) {
  hi_pk = pack_bf16(x0, x1);
  lo_pk = pack_bf16(x0 - bf_lo(hi_pk), x1 - bf_hi(hi_pk));
}

// ---- half-precision operands of the gate products. The activations are bf16 in memory, but
// x_t (the Conv1D output, fp32 in registers) enters the matrix cores as IEEE half precision:
// 11 significant bits instead of 8 at the same MFMA rate. log a_t = c log(sigma(Lambda)) r_t
// and the closed side of a sigmoid amplify the rounding of the pre-activations, and with bf16
// x_t that rounding was the largest single error of the path. The bf16 gate weights convert
// exactly (7-bit significands; below 6.1e-5 they land on half precision's subnormal grid with
// an absolute error under 3e-8).
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ unsigned pack_f16(float lo, float hi) {   // v_cvt_pkrtz_f16_f32
  const auto h = __builtin_amdgcn_cvt_pkrtz(lo, hi);
  return __builtin_bit_cast(unsigned, h);
}
__device__ __forceinline__ float f16_lo(unsigned v) {
  return (float)__builtin_bit_cast(f16x2, v)[0];
}
__device__ __forceinline__ float f16_hi(unsigned v) {
  return (float)__builtin_bit_cast(f16x2, v)[1];
}
// x = high + low with both parts in half precision (21 bits or more in total; values beyond
// +-65504 saturate): the gate products read the high part, x itself is rebuilt from both
__device__ __forceinline__ void split_f16(float x0, float x1, unsigned &hi_pk, unsigned &lo_pk) {
  hi_pk = pack_f16(x0, x1);
  lo_pk = pack_f16(x0 - f16_lo(hi_pk), x1 - f16_hi(hi_pk));
}
// eight bf16 weights (an MFMA fragment as it lies in memory) as half precision
__device__ __forceinline__ f16x8 w_to_f16(bf16x8 w) {
  const u32x4_t v = __builtin_bit_cast(u32x4_t, w);
  u32x4_t o;
#pragma unroll
  for (int k = 0; k < 4; ++k) o[k] = pack_f16(bf_lo(v[k]), bf_hi(v[k]));
  return __builtin_bit_cast(f16x8, o);
}

// 1 - a^2 for a decay a = exp2(l2) <= 1 given with its base-2 logarithm l2 <= 0, without the
// cancellation of 1 - a*a as a -> 1 (the reason Appendix A evaluates eq. (3) in log space):
// 1 - a^2 = -expm1(z) with z = 2 ln2 l2. The series -z - z^2/2 never exceeds the true value
// (it falls short by |z|^3/6); 1 - a*a carries the rounding of a, up to 1.2e-7 either way, and
// is therefore lowered by 2^-22 = 2.4e-7 so that it never exceeds the true value either. The
// larger of the two is then the series for |z| < 9e-3 (relative error < 1.4e-5) and 1 - a*a
// beyond |z| = 1.1e-2 (absolute error < 3.6e-7, relative < 3.3e-5): three instructions more
// than the cancelling form.
__device__ __forceinline__ float one_minus_sq(float a, float l2) {
  constexpr float C = 2.f * LN2;
  const float ser = l2 * fmaf(l2, -0.5f * C * C, -C);
  return __builtin_fmaxf(ser, fmaf(-a, a, 1.f - 0x1p-22f));
}

// 64-bit address made provably wave-uniform (kept in scalar registers), for buffer descriptors
__device__ __forceinline__ void *uniform_ptr(const void *q) {
  const u64 v = (u64)q;
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
  const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return (void *)(((u64)hi << 32) | lo);
}

__device__ __forceinline__ void publish(u64 *slot, float v, unsigned tag) {
  const u64 r = ((u64)tag << 32) | (u64)__float_as_uint(v);
  __hip_atomic_store(slot, r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ u64 peek(const u64 *slot) {
  return __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// A wave's [32 steps][32 channels] bf16 tile, staged in LDS by the lanes that own (channel,
// 16 consecutive steps), leaves as 16-byte stores: lane l writes 8 channels of row l/4 (and of
// row l/4 + 16), so 4 lanes cover the wave's 64 contiguous bytes of a row.
//   ot      this wave's staging tile
//   voff    byte offset of (row l/4, channel group l%4) of this lane inside the sequence
//   soff    byte offset of the tile's first row
//   nrows   rows of the tile inside the sequence (>= 32 for a full tile)
// Cache policy of the big once-through streams (bit 1 of a buffer instruction's auxiliary
// operand = non-temporal): they should not push the re-read weight fragments out of L2.
#ifndef RGLRU_NT
#define RGLRU_NT 2
#endif

// Orders a wave's own LDS accesses where lanes exchange data through a wave-private buffer:
// LDS serves the accesses of one wave in order, so no instruction is needed, only the
// compiler must not move them across this point.
__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int STRIDE, int AUX = 0>
__device__ __forceinline__ void store_staged_tile_s(const unsigned short *ot, int lane,
                                                    __amdgpu_buffer_rsrc_t rsrc, unsigned voff,
                                                    unsigned soff, unsigned row_bytes, int nrows) {
  const int row = lane >> 2, chunk = lane & 3;
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v0 = *(const u32x4 *)(ot + row * STRIDE + chunk * 8);
  const u32x4 v1 = *(const u32x4 *)(ot + (row + 16) * STRIDE + chunk * 8);
  if (row < nrows) __builtin_amdgcn_raw_buffer_store_b128(v0, rsrc, voff, soff, AUX);
  if (row + 16 < nrows) __builtin_amdgcn_raw_buffer_store_b128(v1, rsrc, voff, soff + 16 * row_bytes, AUX);
}
__device__ __forceinline__ void store_staged_tile(const unsigned short *ot, int lane,
                                                  __amdgpu_buffer_rsrc_t rsrc, unsigned voff,
                                                  unsigned soff, unsigned row_bytes, int nrows) {
  store_staged_tile_s<OT>(ot, lane, rsrc, voff, soff, row_bytes, nrows);
}

// host side (defined with the forward kernel)
int num_cu();                                    // compute units of the current device
int pick_slices(int units, int ntile, int ncu, int cap);  // time slices per (sequence, block), at most cap
void set_slice_cap(int cap);                              // process-wide upper bound on that (0 = none)
// clears zero_bytes (% 16 == 0) at `zero` with a fill kernel
//   keep_status: the region starts with a status word, which stays if it reports an expired wait
hipError_t launch_prep(void *zero, size_t zero_bytes, hipStream_t s, bool keep_status = false);
// packed sequences: the document boundaries reset[B][T] as one uint4 of bit masks per (sequence,
// tile of TT steps) - x: a document starts at the step, y / z / w: lag 1 / 2 / 3 of the step's
// Conv1D stays inside its document - and, if nlag is not null, the largest such lag per step
hipError_t launch_reset_masks(const unsigned char *reset, uint4 *masks, unsigned char *nlag, int B, int T,
                              hipStream_t s);

}  // namespace mfma
}  // namespace rglru
