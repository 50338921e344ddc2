// The recurrent block's merge as kernels of its own (Section 2.3, "Recurrent block"):
// out = y * GeLU(branch) and its adjoint. Pure streaming work: every element is read and
// written once, 16 bytes per lane where size and alignment allow.
#include "rglru_gelu.h"
#include "rglru_internal.h"

namespace rglru {
namespace {

constexpr int MTHR = 256;

template <typename AT> struct Vec;              // elements per 16-byte access
template <> struct Vec<float> { static constexpr int N = 4; };
template <> struct Vec<bf16> { static constexpr int N = 8; };

// V elements as one naturally aligned access: requested first (raw), unpacked to fp32 later,
// so that all requests of a trip are in flight together
template <typename AT, int V>
struct __attribute__((aligned(sizeof(AT) * V))) Pack {
  AT e[V];
};

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

template <typename AT, int V>
__device__ __forceinline__ Pack<AT, V> load_raw(const AT *p, size_t i) {
  return *(const Pack<AT, V> *)(p + i);
}
template <typename AT, int V>
__device__ __forceinline__ void unpack(const Pack<AT, V> &v, float (&f)[V]) {
#pragma unroll
  for (int k = 0; k < V; ++k) f[k] = ldf(v.e, k);
}
template <typename AT, int V>
__device__ __forceinline__ void store_pack(AT *p, size_t i, const float (&f)[V]) {
  Pack<AT, V> v;
  if constexpr (sizeof(AT) == 2 && V % 2 == 0) {   // v_cvt_pk_bf16_f32: two values per instruction
#pragma unroll
    for (int k = 0; k < V; k += 2) {
      const f32x2_t two = {f[k], f[k + 1]};
      const bf16x2_t b = __builtin_convertvector(two, bf16x2_t);
      const unsigned bits = *(const unsigned *)&b;
      v.e[k].v = (unsigned short)(bits & 0xffffu);
      v.e[k + 1].v = (unsigned short)(bits >> 16);
    }
  } else {
#pragma unroll
    for (int k = 0; k < V; ++k) stf(v.e, k, f[k]);
  }
  *(Pack<AT, V> *)(p + i) = v;
}

constexpr int NP = 2;   // packs per thread and trip

template <typename AT, int V, bool TANH>
__global__ void __launch_bounds__(MTHR)
merge_fwd_kernel(const AT *y, const AT *br, AT *out, size_t n) {
  constexpr bool FAST = sizeof(AT) == 2;
  const size_t stride = (size_t)gridDim.x * MTHR * V;
  size_t i = ((size_t)blockIdx.x * MTHR + threadIdx.x) * V;
  for (; i + (NP - 1) * stride < n; i += NP * stride) {
    Pack<AT, V> ry[NP], rb[NP];
#pragma unroll
    for (int h = 0; h < NP; ++h) {
      ry[h] = load_raw<AT, V>(y, i + h * stride);
      rb[h] = load_raw<AT, V>(br, i + h * stride);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int h = 0; h < NP; ++h) {
      float fy[V], fb[V], fo[V];
      unpack<AT, V>(ry[h], fy);
      unpack<AT, V>(rb[h], fb);
#pragma unroll
      for (int k = 0; k < V; ++k) fo[k] = fy[k] * gelu<TANH, FAST>(fb[k]);
      store_pack<AT, V>(out, i + h * stride, fo);
    }
  }
  for (; i < n; i += stride) {
    float fy[V], fb[V], fo[V];
    unpack<AT, V>(load_raw<AT, V>(y, i), fy);
    unpack<AT, V>(load_raw<AT, V>(br, i), fb);
#pragma unroll
    for (int k = 0; k < V; ++k) fo[k] = fy[k] * gelu<TANH, FAST>(fb[k]);
    store_pack<AT, V>(out, i, fo);
  }
}

template <typename AT, int V, bool TANH>
__global__ void __launch_bounds__(MTHR)
merge_bwd_kernel(const AT *y, const AT *br, const AT *dout, AT *dy, AT *dy_lo, AT *dbr, size_t n) {
  constexpr bool FAST = sizeof(AT) == 2;
  const size_t stride = (size_t)gridDim.x * MTHR * V;
  size_t i = ((size_t)blockIdx.x * MTHR + threadIdx.x) * V;
  auto one = [&](const Pack<AT, V> &ry, const Pack<AT, V> &rb, const Pack<AT, V> &rd, size_t at)
      __attribute__((always_inline)) {
    float fy[V], fb[V], fd[V], gy[V], gb[V];
    unpack<AT, V>(ry, fy);
    unpack<AT, V>(rb, fb);
    unpack<AT, V>(rd, fd);
#pragma unroll
    for (int k = 0; k < V; ++k) {
      float val, grad;
      gelu_and_grad<TANH, FAST>(fb[k], val, grad);
      gy[k] = fd[k] * val;
      gb[k] = fd[k] * fy[k] * grad;
    }
    store_pack<AT, V>(dy, at, gy);
    store_pack<AT, V>(dbr, at, gb);
    if (FAST && dy_lo) {   // what the bf16 rounding of dy took away, as a second bf16 tensor
      float gl[V];
#pragma unroll
      for (int k = 0; k < V; ++k)
        gl[k] = gy[k] - __uint_as_float((unsigned)f32_to_bf16_bits(gy[k]) << 16);
      store_pack<AT, V>(dy_lo, at, gl);
    }
  };
  for (; i + (NP - 1) * stride < n; i += NP * stride) {
    Pack<AT, V> ry[NP], rb[NP], rd[NP];
#pragma unroll
    for (int h = 0; h < NP; ++h) {
      ry[h] = load_raw<AT, V>(y, i + h * stride);
      rb[h] = load_raw<AT, V>(br, i + h * stride);
      rd[h] = load_raw<AT, V>(dout, i + h * stride);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int h = 0; h < NP; ++h) one(ry[h], rb[h], rd[h], i + h * stride);
  }
  for (; i < n; i += stride) one(load_raw<AT, V>(y, i), load_raw<AT, V>(br, i), load_raw<AT, V>(dout, i), i);
}

bool all_aligned16(std::initializer_list<const void *> ps) {
  for (const void *p : ps)
    if (((uintptr_t)p & 15) != 0) return false;
  return true;
}

int grid_for(size_t n, int v) {
  const size_t blocks = (n + (size_t)MTHR * v - 1) / ((size_t)MTHR * v);
  const size_t cap = 256 * 16;   // a few waves per SIMD on every CU, then grid-stride
  return (int)(blocks < cap ? (blocks ? blocks : 1) : cap);
}

template <typename AT, bool TANH>
hipError_t fwd_typed(const void *y, const void *br, void *out, size_t n, hipStream_t s) {
  constexpr int V = Vec<AT>::N;
  KernelTimer t("merge_fwd_kernel", s);
  if (n % V == 0 && all_aligned16({y, br, out}))
    hipLaunchKernelGGL((merge_fwd_kernel<AT, V, TANH>), dim3(grid_for(n, V)), dim3(MTHR), 0, s,
                       (const AT *)y, (const AT *)br, (AT *)out, n);
  else
    hipLaunchKernelGGL((merge_fwd_kernel<AT, 1, TANH>), dim3(grid_for(n, 1)), dim3(MTHR), 0, s,
                       (const AT *)y, (const AT *)br, (AT *)out, n);
  return hipGetLastError();
}

template <typename AT, bool TANH>
hipError_t bwd_typed(const void *y, const void *br, const void *dout, void *dy, void *dy_lo, void *dbr, size_t n,
                     hipStream_t s) {
  constexpr int V = Vec<AT>::N;
  KernelTimer t("merge_bwd_kernel", s);
  if (n % V == 0 && all_aligned16({y, br, dout, dy, dy_lo, dbr}))
    hipLaunchKernelGGL((merge_bwd_kernel<AT, V, TANH>), dim3(grid_for(n, V)), dim3(MTHR), 0, s,
                       (const AT *)y, (const AT *)br, (const AT *)dout, (AT *)dy, (AT *)dy_lo, (AT *)dbr, n);
  else
    hipLaunchKernelGGL((merge_bwd_kernel<AT, 1, TANH>), dim3(grid_for(n, 1)), dim3(MTHR), 0, s,
                       (const AT *)y, (const AT *)br, (const AT *)dout, (AT *)dy, (AT *)dy_lo, (AT *)dbr, n);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_merge_forward(const void *y, const void *branch, void *out, size_t n, bool bf,
                                bool tanh_form, hipStream_t s) {
  if (n == 0) return hipSuccess;
  if (bf) return tanh_form ? fwd_typed<bf16, true>(y, branch, out, n, s) : fwd_typed<bf16, false>(y, branch, out, n, s);
  return tanh_form ? fwd_typed<float, true>(y, branch, out, n, s) : fwd_typed<float, false>(y, branch, out, n, s);
}

hipError_t launch_merge_backward(const void *y, const void *branch, const void *dout, void *dy, void *dy_lo,
                                 void *dbranch, size_t n, bool bf, bool tanh_form, hipStream_t s) {
  if (n == 0) return hipSuccess;
  if (bf)
    return tanh_form ? bwd_typed<bf16, true>(y, branch, dout, dy, dy_lo, dbranch, n, s)
                     : bwd_typed<bf16, false>(y, branch, dout, dy, dy_lo, dbranch, n, s);
  return tanh_form ? bwd_typed<float, true>(y, branch, dout, dy, nullptr, dbranch, n, s)
                   : bwd_typed<float, false>(y, branch, dout, dy, nullptr, dbranch, n, s);
}

}  // namespace rglru
