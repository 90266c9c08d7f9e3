// 2x2 max pooling (stride 2, no padding, a trailing odd row or column is
// dropped) of an NHWC tensor: the second step of the pooled entry point for
// the variants that cannot reduce the window in their epilogue.  Section 3 of
// the paper names pooling among the layers that sit between the convolutions.
//
// One lane per pooled element, features fastest: the four reads and the store
// of a wavefront are 64 consecutive elements each.  Memory-bound: reads the
// unpooled tensor once, writes a quarter of it.
#include "conv2d_internal.h"

namespace conv2d {
namespace {

__device__ __forceinline__ float load_as_float(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_as_float(const unsigned short* p, size_t i) {
  return __uint_as_float(static_cast<unsigned>(p[i]) << 16);
}
__device__ __forceinline__ void store_from_float(float* p, size_t i, float v) { p[i] = v; }
// (the maximum of bf16 values is one of them: the conversion back is exact)
__device__ __forceinline__ void store_from_float(unsigned short* p, size_t i, float v) {
  p[i] = static_cast<unsigned short>(__float_as_uint(v) >> 16);
}

template <class E>
__global__ __launch_bounds__(256) void max_pool_2x2_kernel(const E* __restrict__ in,
                                                           E* __restrict__ out, int P, int Q,
                                                           int K, long long total) {
  const int P2 = P / 2, Q2 = Q / 2;
  for (long long idx = blockIdx.x * 256LL + threadIdx.x; idx < total;
       idx += 256LL * gridDim.x) {
    const int k = static_cast<int>(idx % K);
    long long t = idx / K;
    const int px = static_cast<int>(t % Q2);
    t /= Q2;
    const int py = static_cast<int>(t % P2);
    const long long n = t / P2;
    const size_t base = ((static_cast<size_t>(n) * P + 2 * py) * Q + 2 * px) * K + k;
    const size_t row = static_cast<size_t>(Q) * K;
    const float a = load_as_float(in, base), b = load_as_float(in, base + K);
    const float c = load_as_float(in, base + row), d = load_as_float(in, base + row + K);
    store_from_float(out, static_cast<size_t>(idx), fmaxf(fmaxf(a, b), fmaxf(c, d)));
  }
}

}  // namespace

hipError_t launch_max_pool_2x2(const void* in, void* out, int N, int P, int Q, int K, bool bf16,
                               hipStream_t stream) {
  const long long total = 1LL * N * (P / 2) * (Q / 2) * K;
  if (total == 0) return hipSuccess;
  const long long blocks = (total + 255) / 256;
  const int grid = static_cast<int>(blocks < 256 * 64 ? blocks : 256 * 64);
  if (bf16)
    hipLaunchKernelGGL(max_pool_2x2_kernel<unsigned short>, dim3(grid), dim3(256), 0, stream,
                       static_cast<const unsigned short*>(in), static_cast<unsigned short*>(out),
                       P, Q, K, total);
  else
    hipLaunchKernelGGL(max_pool_2x2_kernel<float>, dim3(grid), dim3(256), 0, stream,
                       static_cast<const float*>(in), static_cast<float*>(out), P, Q, K, total);
  return hipGetLastError();
}

}  // namespace conv2d
