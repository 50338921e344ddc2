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

template <typename AT, int V>
struct Pack {
  AT e[V];
};

template <typename AT, int V>
__device__ __forceinline__ void load_pack(const AT *p, size_t i, float (&f)[V]) {
  typedef Pack<AT, V> __attribute__((aligned(sizeof(AT) * V))) P;
  const P v = *(const P *)(p + i);
#pragma unroll
  for (int k = 0; k < V; ++k) f[k] = ldf(v.e, k);
}
template <typename AT, int V>
__device__ __forceinline__ void store_pack(AT *p, size_t i, const float (&f)[V]) {
  typedef Pack<AT, V> __attribute__((aligned(sizeof(AT) * V))) P;
  P v;
#pragma unroll
  for (int k = 0; k < V; ++k) stf(v.e, k, f[k]);
  *(P *)(p + i) = v;
}

template <typename AT, int V, bool TANH>
__global__ void __launch_bounds__(MTHR)
merge_fwd_kernel(const AT *y, const AT *br, AT *out, size_t n) {
  constexpr bool FAST = sizeof(AT) == 2;
  const size_t stride = (size_t)gridDim.x * MTHR * V;
  for (size_t i = ((size_t)blockIdx.x * MTHR + threadIdx.x) * V; i < n; i += stride) {
    float fy[V], fb[V], fo[V];
    load_pack<AT, V>(y, i, fy);
    load_pack<AT, V>(br, i, fb);
#pragma unroll
    for (int k = 0; k < V; ++k) fo[k] = fy[k] * gelu<TANH, FAST>(fb[k]);
    store_pack<AT, V>(out, i, fo);
  }
}

template <typename AT, int V, bool TANH>
__global__ void __launch_bounds__(MTHR)
merge_bwd_kernel(const AT *y, const AT *br, const AT *dout, AT *dy, AT *dbr, size_t n) {
  constexpr bool FAST = sizeof(AT) == 2;
  const size_t stride = (size_t)gridDim.x * MTHR * V;
  for (size_t i = ((size_t)blockIdx.x * MTHR + threadIdx.x) * V; i < n; i += stride) {
    float fy[V], fb[V], fd[V], gy[V], gb[V];
    load_pack<AT, V>(y, i, fy);
    load_pack<AT, V>(br, i, fb);
    load_pack<AT, V>(dout, i, fd);
#pragma unroll
    for (int k = 0; k < V; ++k) {
      float val, grad;
      gelu_and_grad<TANH, FAST>(fb[k], val, grad);
      gy[k] = fd[k] * val;
      gb[k] = fd[k] * fy[k] * grad;
    }
    store_pack<AT, V>(dy, i, gy);
    store_pack<AT, V>(dbr, i, gb);
  }
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
hipError_t bwd_typed(const void *y, const void *br, const void *dout, void *dy, void *dbr, size_t n,
                     hipStream_t s) {
  constexpr int V = Vec<AT>::N;
  KernelTimer t("merge_bwd_kernel", s);
  if (n % V == 0 && all_aligned16({y, br, dout, dy, dbr}))
    hipLaunchKernelGGL((merge_bwd_kernel<AT, V, TANH>), dim3(grid_for(n, V)), dim3(MTHR), 0, s,
                       (const AT *)y, (const AT *)br, (const AT *)dout, (AT *)dy, (AT *)dbr, n);
  else
    hipLaunchKernelGGL((merge_bwd_kernel<AT, 1, TANH>), dim3(grid_for(n, 1)), dim3(MTHR), 0, s,
                       (const AT *)y, (const AT *)br, (const AT *)dout, (AT *)dy, (AT *)dbr, n);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_merge_forward(const void *y, const void *branch, void *out, size_t n, bool bf,
                                bool tanh_form, hipStream_t s) {
  if (n == 0) return hipSuccess;
  if (bf) return tanh_form ? fwd_typed<bf16, true>(y, branch, out, n, s) : fwd_typed<bf16, false>(y, branch, out, n, s);
  return tanh_form ? fwd_typed<float, true>(y, branch, out, n, s) : fwd_typed<float, false>(y, branch, out, n, s);
}

hipError_t launch_merge_backward(const void *y, const void *branch, const void *dout, void *dy,
                                 void *dbranch, size_t n, bool bf, bool tanh_form, hipStream_t s) {
  if (n == 0) return hipSuccess;
  if (bf)
    return tanh_form ? bwd_typed<bf16, true>(y, branch, dout, dy, dbranch, n, s)
                     : bwd_typed<bf16, false>(y, branch, dout, dy, dbranch, n, s);
  return tanh_form ? bwd_typed<float, true>(y, branch, dout, dy, dbranch, n, s)
                   : bwd_typed<float, false>(y, branch, dout, dy, dbranch, n, s);
}

}  // namespace rglru
