// rglru_scan: eq. (4) alone as a linear scan over given decays and gated inputs
// (Section 4.2, "A custom linear scan"; the operation timed in Appendix A.3).
//
//   h_t = a_t h_{t-1} + m_t g_t,  m_t = sqrt(1 - a_t^2) (or 1),  a_t given directly or as log a_t
//
// Generic kernel: one thread per (sequence, channel) walking the time axis; any shape, fp32 or
// bf16 storage, accurate math. It carries the fp32 contract and the shapes the tiled kernel
// does not cover.
#include "rglru_internal.h"

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

bool scan_tiled_supported(const ScanProblem &, bool) { return false; }
size_t scan_tiled_ws_bytes(int, int, int) { return 0; }
hipError_t launch_scan_tiled(const ScanProblem &, hipStream_t) { return hipErrorNotSupported; }

}  // namespace rglru
