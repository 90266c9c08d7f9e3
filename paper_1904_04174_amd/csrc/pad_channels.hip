// Small channel counts through the vector tiles.
//
// A first layer has 3 input channels (the 7x7 stem of ResNet-50 among the
// paper's shapes): no 16-byte vector along the channels, so only the
// element-wise tiles can gather it, one 2- or 4-byte load per element.  This
// path pads the channels with zeros to the vector width (4 fp32 / 8 bf16) in
// the workspace, input and filter alike, and runs a per-lane addressed
// direct-to-LDS tile on the padded tensors: more multiply-adds (the zeros),
// but 16-byte gathers and a pipelined kernel.  The result is unchanged: the
// added products are exact zeros.
#include "conv2d_internal.h"

namespace conv2d {
namespace {

// dst[pixel][c'] = c' < C ? src[pixel][c'] : 0 for `pixels` pixels (input:
// N*H*W, filter viewed as R*S pixels of C rows of K values: see pad_filter).
// One thread per padded vector of CP elements (16 bytes).
template <typename E, int CP>
__global__ __launch_bounds__(256) void pad_input_kernel(const E* __restrict__ src,
                                                        E* __restrict__ dst, long long vectors,
                                                        int C) {
  const long long i = static_cast<long long>(blockIdx.x) * 256 + threadIdx.x;
  if (i >= vectors) return;
  const int per_pixel = (C + CP - 1) / CP;        // vectors per pixel
  // (one vector per pixel, the usual case of 3 channels: no 64-bit division per thread)
  const long long pixel = per_pixel == 1 ? i : i / per_pixel;
  const int c0 = per_pixel == 1 ? 0 : static_cast<int>(i % per_pixel) * CP;
  E v[CP];
#pragma unroll
  for (int j = 0; j < CP; ++j) v[j] = (c0 + j < C) ? src[pixel * C + c0 + j] : E(0);
  E* out = dst + i * CP;
#pragma unroll
  for (int j = 0; j < CP; ++j) out[j] = v[j];
}

// Filter [taps][C][K] -> [taps][Cp][K], rows c >= C zero.  One thread per element.
template <typename E>
__global__ __launch_bounds__(256) void pad_filter_kernel(const E* __restrict__ src,
                                                         E* __restrict__ dst, int taps, int C,
                                                         int Cp, int K) {
  const long long i = static_cast<long long>(blockIdx.x) * 256 + threadIdx.x;
  const long long total = static_cast<long long>(taps) * Cp * K;
  if (i >= total) return;
  const int k = static_cast<int>(i % K);
  const int c = static_cast<int>((i / K) % Cp);
  const int t = static_cast<int>(i / (static_cast<long long>(K) * Cp));
  dst[i] = c < C ? src[(static_cast<long long>(t) * C + c) * K + k] : E(0);
}

size_t align256(size_t b) { return (b + 255) / 256 * 256; }

struct Plan {
  int Cp;
  size_t in_bytes, filt_bytes;
  Problem inner;
};

Plan make_plan(const Problem& p) {
  Plan pl;
  const int vec = p.in_bf16 ? 8 : 4, es = p.in_bf16 ? 2 : 4;
  pl.Cp = (p.C + vec - 1) / vec * vec;
  pl.in_bytes = align256(static_cast<size_t>(p.N) * p.H * p.W * pl.Cp * es);
  pl.filt_bytes = align256(static_cast<size_t>(p.R) * p.S * pl.Cp * p.K * es);
  pl.inner = p;
  pl.inner.C = pl.Cp;
  pl.inner.Kg = p.R * p.S * pl.Cp;
  return pl;
}

}  // namespace

bool padded_supports(const Problem& p, int gemm_tile) {
  const int vec = p.in_bf16 ? 8 : 4, es = p.in_bf16 ? 2 : 4;
  if (p.C % vec == 0 || p.C > 2 * vec || p.M == 0) return false;  // small, unaligned C only
  if (igemm_dma_tile_addressing(p.in_bf16, gemm_tile) != 1) return false;
  const Plan pl = make_plan(p);
  int bm, bn, bk;
  igemm_dma_tile_shape(p.in_bf16, gemm_tile, &bm, &bn, &bk);
  // the padded tensors must fit the 31-bit byte offsets of the gather kernel
  if (1LL * es * (1LL * p.N * p.H * p.W + 1LL * p.R * p.W + p.S) * pl.Cp >= (1LL << 31)) return false;
  if (1LL * es * (pl.inner.Kg + bk) * p.K >= (1LL << 31)) return false;
  return true;
}

size_t padded_workspace_bytes(const Problem& p, int gemm_tile) {
  const Plan pl = make_plan(p);
  return pl.in_bytes + pl.filt_bytes + igemm_dma_workspace_bytes(pl.inner, p.in_bf16, gemm_tile, 1);
}

namespace {

hipError_t pad_filter(const Problem& p, const Plan& pl, void* filt_p, hipStream_t stream) {
  const long long felems = static_cast<long long>(p.R) * p.S * pl.Cp * p.K;
  const dim3 fgrid(static_cast<unsigned>((felems + 255) / 256));
  if (p.in_bf16)
    hipLaunchKernelGGL((pad_filter_kernel<unsigned short>), fgrid, dim3(256), 0, stream,
                       static_cast<const unsigned short*>(p.filt),
                       static_cast<unsigned short*>(filt_p), p.R * p.S, p.C, pl.Cp, p.K);
  else
    hipLaunchKernelGGL((pad_filter_kernel<float>), fgrid, dim3(256), 0, stream,
                       static_cast<const float*>(p.filt), static_cast<float*>(filt_p), p.R * p.S,
                       p.C, pl.Cp, p.K);
  return hipGetLastError();
}

}  // namespace

// The filter packed ahead of time: the zero-padded filter, then that repacked for the tile.
// Only the second part is read by a launch.
size_t padded_packed_filter_bytes(const Problem& p, int gemm_tile) {
  const Plan pl = make_plan(p);
  return pl.filt_bytes + igemm_dma_packed_filter_bytes(pl.inner, p.in_bf16, gemm_tile);
}

hipError_t padded_pack_filter(const Problem& p, int gemm_tile, void* packed, hipStream_t stream) {
  Plan pl = make_plan(p);
  hipError_t e = pad_filter(p, pl, packed, stream);
  if (e != hipSuccess) return e;
  pl.inner.filt = packed;
  return igemm_dma_pack_filter(pl.inner, p.in_bf16, gemm_tile,
                               static_cast<unsigned char*>(packed) + pl.filt_bytes, stream);
}

hipError_t launch_padded(const Problem& p, int gemm_tile, hipStream_t stream) {
  Plan pl = make_plan(p);
  unsigned char* ws = static_cast<unsigned char*>(p.workspace);
  void* in_p = ws;
  void* filt_p = ws + pl.in_bytes;
  const int vec = p.in_bf16 ? 8 : 4;
  const long long vectors = static_cast<long long>(p.N) * p.H * p.W * (pl.Cp / vec);
  const dim3 igrid(static_cast<unsigned>((vectors + 255) / 256));
  if (p.in_bf16)
    hipLaunchKernelGGL((pad_input_kernel<unsigned short, 8>), igrid, dim3(256), 0, stream,
                       static_cast<const unsigned short*>(p.in),
                       static_cast<unsigned short*>(in_p), vectors, p.C);
  else
    hipLaunchKernelGGL((pad_input_kernel<float, 4>), igrid, dim3(256), 0, stream,
                       static_cast<const float*>(p.in), static_cast<float*>(in_p), vectors, p.C);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (p.packed_filt) {
    pl.inner.packed_filt = static_cast<const unsigned char*>(p.packed_filt) + pl.filt_bytes;
  } else {
    e = pad_filter(p, pl, filt_p, stream);
    if (e != hipSuccess) return e;
  }
  pl.inner.in = in_p;
  pl.inner.filt = filt_p;
  pl.inner.workspace = ws + pl.in_bytes + pl.filt_bytes;
  return launch_igemm_dma(pl.inner, p.in_bf16, gemm_tile, 1, stream);
}

}  // namespace conv2d
