// Winograd F(2x2, 3x3) forward convolution, fp32, stride 1: the transform
// algorithm that section 3 of the paper lists beside its direct kernels (and
// that its Figure 1 shows ahead on the 3x3 layers).  2.25 times fewer
// multiplications than the direct sum, paid for with transform passes.
//
// For every 2x2 block of output pixels the 4x4 input patch d and the 3x3
// filter g are transformed, multiplied point by point and transformed back:
//
//   Y = A^T [ (G g G^T) .* (B^T d B) ] A          (summed over the channels)
//
//   B^T = | 1  0 -1  0 |   G = | 1    0    0  |   A^T = | 1 1  1  0 |
//         | 0  1  1  0 |       | 1/2  1/2  1/2|         | 0 1 -1 -1 |
//         | 0 -1  1  0 |       | 1/2 -1/2  1/2|
//         | 0  1  0 -1 |       | 0    0    1  |
//
// The sum over channels of the 16 point-wise products is 16 independent
// matrix products  Mt[t] = V[t] (tiles x C)  *  U[t] (C x K):  2.25 times
// fewer multiplications than the direct sum.  Four kernels:
//
//   1. filter_transform_kernel   f[3][3][C][K]      -> U[16][C][K]
//   2. input_transform_kernel    in[N][H][W][C]     -> V[16][tiles][C]
//   3. the 16 products as ONE batched launch of the direct-to-LDS gather
//      kernel (a 1x1 convolution over a 1 x tiles "image" per point)
//   4. output_transform_kernel   Mt[16][tiles][K]   -> out[N][P][Q][K]
//
// "Fused" variants replace 3 and 4 by one launch of the gather kernel in its
// Winograd mode: a workgroup runs the 16 products of its block of tiles one
// after the other and folds each into the four output pixels with the signs
// of A^T (x) A^T, so Mt (4x the output) never goes through memory.
//
// All transform entries are 0, +-1 or +-1/2, so the transforms add no
// rounding error beyond a few ulp of their inputs; the measured error against
// the fp64 oracle stays within the fp32 tolerance of the direct kernels
// (F(4x4, 3x3), which would save 4x, measured 2.8e-4 at C = 512 with the
// standard interpolation points and is therefore not offered).
//
// Workspace: U, V, Mt and the batched product's repacked filters.  Needs C
// and K multiples of 4 (16-byte vectors along the channels / features).
#include "conv2d_internal.h"

namespace conv2d {
namespace {

constexpr int kPoints = 16;

__device__ __forceinline__ float4 add4(float4 a, float4 b) {
  return float4{a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w};
}
__device__ __forceinline__ float4 sub4(float4 a, float4 b) {
  return float4{a.x - b.x, a.y - b.y, a.z - b.z, a.w - b.w};
}
__device__ __forceinline__ float4 half4(float4 a) {
  return float4{0.5f * a.x, 0.5f * a.y, 0.5f * a.z, 0.5f * a.w};
}

// U[t = a*4 + b][c][k] = sum_{r,s} G[a][r] G[b][s] f[r][s][c][k].
// One thread per (c, 4 consecutive k).
__global__ __launch_bounds__(256) void filter_transform_kernel(const float* __restrict__ f,
                                                               float* __restrict__ u, int C,
                                                               int K) {
  const int kv = K / 4;
  const long long idx = static_cast<long long>(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= static_cast<long long>(C) * kv) return;
  const int c = static_cast<int>(idx / kv), k = static_cast<int>(idx % kv) * 4;
  const size_t ck = static_cast<size_t>(C) * K;
  float4 g[3][3];
#pragma unroll
  for (int r = 0; r < 3; ++r)
#pragma unroll
    for (int s = 0; s < 3; ++s)
      g[r][s] = *reinterpret_cast<const float4*>(f + (r * 3 + s) * ck + static_cast<size_t>(c) * K + k);
  // rows: t[a][s] = sum_r G[a][r] g[r][s]
  float4 t[4][3];
#pragma unroll
  for (int s = 0; s < 3; ++s) {
    const float4 sum02 = add4(g[0][s], g[2][s]);
    t[0][s] = g[0][s];
    t[1][s] = half4(add4(sum02, g[1][s]));
    t[2][s] = half4(sub4(sum02, g[1][s]));
    t[3][s] = g[2][s];
  }
  // columns: U[a][b] = sum_s t[a][s] G[b][s]
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const float4 sum02 = add4(t[a][0], t[a][2]);
    const float4 o[4] = {t[a][0], half4(add4(sum02, t[a][1])), half4(sub4(sum02, t[a][1])),
                         t[a][2]};
#pragma unroll
    for (int b = 0; b < 4; ++b)
      *reinterpret_cast<float4*>(u + (a * 4 + b) * ck + static_cast<size_t>(c) * K + k) = o[b];
  }
}

// V[t = a*4 + b][tile][c] = (B^T d B)[a][b] for the 4x4 input patch d of tile
// (n, th, tw): rows 2*th - pt .. + 3, columns 2*tw - pl .. + 3, zero outside
// the image.  One thread per (tile, 4 consecutive c).
__global__ __launch_bounds__(256) void input_transform_kernel(const float* __restrict__ in,
                                                              float* __restrict__ v, int N, int H,
                                                              int W, int C, int pt, int pl, int TH,
                                                              int TW) {
  const int cv = C / 4;
  const long long tiles = static_cast<long long>(N) * TH * TW;
  const long long idx = static_cast<long long>(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= tiles * cv) return;
  const long long tile = idx / cv;
  const int c = static_cast<int>(idx % cv) * 4;
  const int tw = static_cast<int>(tile % TW);
  const int th = static_cast<int>((tile / TW) % TH);
  const int n = static_cast<int>(tile / (static_cast<long long>(TW) * TH));
  const int h0 = 2 * th - pt, w0 = 2 * tw - pl;
  float4 d[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int h = h0 + i, w = w0 + j;
      const bool ok = static_cast<unsigned>(h) < static_cast<unsigned>(H) &&
                      static_cast<unsigned>(w) < static_cast<unsigned>(W);
      d[i][j] = ok ? *reinterpret_cast<const float4*>(
                         in + ((static_cast<size_t>(n) * H + h) * W + w) * C + c)
                   : float4{0.f, 0.f, 0.f, 0.f};
    }
  // rows: t[a][j] = sum_i B^T[a][i] d[i][j]
  float4 t[4][4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    t[0][j] = sub4(d[0][j], d[2][j]);
    t[1][j] = add4(d[1][j], d[2][j]);
    t[2][j] = sub4(d[2][j], d[1][j]);
    t[3][j] = sub4(d[1][j], d[3][j]);
  }
  const size_t plane = static_cast<size_t>(tiles) * C;
  float* dst = v + static_cast<size_t>(tile) * C + c;
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const float4 o[4] = {sub4(t[a][0], t[a][2]), add4(t[a][1], t[a][2]), sub4(t[a][2], t[a][1]),
                         sub4(t[a][1], t[a][3])};
#pragma unroll
    for (int b = 0; b < 4; ++b) *reinterpret_cast<float4*>(dst + (a * 4 + b) * plane) = o[b];
  }
}

// out[n][2*th + i][2*tw + j][k] = (A^T m A)[i][j], m[a][b] = Mt[a*4 + b][tile][k].
// One thread per (tile, 4 consecutive k); outputs past P or Q are dropped.
__global__ __launch_bounds__(256) void output_transform_kernel(const float* __restrict__ mt,
                                                               float* __restrict__ out, int N,
                                                               int P, int Q, int K, int TH,
                                                               int TW,
                                                               const float* __restrict__ bias,
                                                               int relu, int pool) {
  const int kv = K / 4;
  const long long tiles = static_cast<long long>(N) * TH * TW;
  const long long idx = static_cast<long long>(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= tiles * kv) return;
  const long long tile = idx / kv;
  const int k = static_cast<int>(idx % kv) * 4;
  const int tw = static_cast<int>(tile % TW);
  const int th = static_cast<int>((tile / TW) % TH);
  const int n = static_cast<int>(tile / (static_cast<long long>(TW) * TH));
  const size_t plane = static_cast<size_t>(tiles) * K;
  const float* src = mt + static_cast<size_t>(tile) * K + k;
  float4 m[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) m[a][b] = *reinterpret_cast<const float4*>(src + (a * 4 + b) * plane);
  // rows: t[i][b] = sum_a A^T[i][a] m[a][b]
  float4 t[2][4];
#pragma unroll
  for (int b = 0; b < 4; ++b) {
    t[0][b] = add4(add4(m[0][b], m[1][b]), m[2][b]);
    t[1][b] = sub4(sub4(m[1][b], m[2][b]), m[3][b]);
  }
  const float4 b = bias ? float4{bias[k], bias[k + 1], bias[k + 2], bias[k + 3]}
                        : float4{0.f, 0.f, 0.f, 0.f};
  if (pool) {
    // 2x2 max pooling: the four outputs of a Winograd tile are one pooling window; bias and
    // activation after the maximum (both monotone); windows past P/2 or Q/2 are dropped
    if (th >= P / 2 || tw >= Q / 2) return;
    float4 best;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const float4 y0 = add4(add4(t[i][0], t[i][1]), t[i][2]);
      const float4 y1 = sub4(sub4(t[i][1], t[i][2]), t[i][3]);
      const float4 m = float4{fmaxf(y0.x, y1.x), fmaxf(y0.y, y1.y), fmaxf(y0.z, y1.z),
                              fmaxf(y0.w, y1.w)};
      best = i == 0 ? m : float4{fmaxf(best.x, m.x), fmaxf(best.y, m.y), fmaxf(best.z, m.z),
                                 fmaxf(best.w, m.w)};
    }
    best = float4{finish(best.x, b.x, relu), finish(best.y, b.y, relu), finish(best.z, b.z, relu),
                  finish(best.w, b.w, relu)};
    *reinterpret_cast<float4*>(out + ((static_cast<size_t>(n) * (P / 2) + th) * (Q / 2) + tw) * K +
                               k) = best;
    return;
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int op = 2 * th + i;
    if (op >= P) continue;
    float4 y0 = add4(add4(t[i][0], t[i][1]), t[i][2]);
    float4 y1 = sub4(sub4(t[i][1], t[i][2]), t[i][3]);
    y0 = float4{finish(y0.x, b.x, relu), finish(y0.y, b.y, relu), finish(y0.z, b.z, relu),
                finish(y0.w, b.w, relu)};
    y1 = float4{finish(y1.x, b.x, relu), finish(y1.y, b.y, relu), finish(y1.z, b.z, relu),
                finish(y1.w, b.w, relu)};
    float* row = out + ((static_cast<size_t>(n) * P + op) * Q) * K + k;
    const int oq = 2 * tw;
    *reinterpret_cast<float4*>(row + static_cast<size_t>(oq) * K) = y0;
    if (oq + 1 < Q) *reinterpret_cast<float4*>(row + static_cast<size_t>(oq + 1) * K) = y1;
  }
}

size_t align256(size_t b) { return (b + 255) / 256 * 256; }

struct Plan {
  int TH, TW;
  long long tiles;
  size_t u_bytes, v_bytes, m_bytes;
  Problem gemm;  // the point products as a problem of the direct-to-LDS gather kernel
};

// `fused`: the products run point after point inside one workgroup per tile
// block, which folds each into the output pixels (no Mt): V is then an image
// of 16 rows (points) x tiles columns and U a 16x1 window.  Otherwise: 16
// batched 1x1 convolutions over a 1 x tiles image that write Mt.
Plan make_plan(const Problem& p, bool fused) {
  Plan pl;
  pl.TH = (p.P + 1) / 2;
  pl.TW = (p.Q + 1) / 2;
  pl.tiles = static_cast<long long>(p.N) * pl.TH * pl.TW;
  pl.u_bytes = align256(sizeof(float) * kPoints * static_cast<size_t>(p.C) * p.K);
  pl.v_bytes = align256(sizeof(float) * kPoints * static_cast<size_t>(pl.tiles) * p.C);
  pl.m_bytes = fused ? 0 : align256(sizeof(float) * kPoints * static_cast<size_t>(pl.tiles) * p.K);
  Problem g = {};
  g.N = 1; g.W = static_cast<int>(pl.tiles); g.C = p.C; g.K = p.K;
  g.sr = 1; g.sc = 1; g.pt = 0; g.pl = 0;
  g.P = 1; g.Q = g.W; g.M = g.W;
  g.in_bf16 = 0; g.out_bf16 = 0;
  if (fused) {
    g.H = kPoints; g.R = kPoints; g.S = 1; g.Kg = kPoints * p.C;
    g.wino_th = pl.TH; g.wino_tw = pl.TW; g.wino_p = p.P; g.wino_q = p.Q;
    g.bias = p.bias; g.relu = p.relu;
  } else {
    g.H = 1; g.R = 1; g.S = 1; g.Kg = p.C;
    g.batches = kPoints;
    g.in_stride = pl.tiles * p.C;
    g.filt_stride = static_cast<long long>(p.C) * p.K;
    g.out_stride = pl.tiles * p.K;
  }
  pl.gemm = g;
  return pl;
}

}  // namespace

bool winograd_supports(const Problem& p, int gemm_tile, bool fused) {
  if (p.in_bf16 || p.out_bf16) return false;
  if (p.R != 3 || p.S != 3 || p.sr != 1 || p.sc != 1) return false;
  if (p.C % 4 != 0 || p.K % 4 != 0 || p.M == 0) return false;
  const Plan pl = make_plan(p, fused);
  const int addressing = igemm_dma_tile_addressing(0, gemm_tile);
  int bm, bn, bk;
  igemm_dma_tile_shape(0, gemm_tile, &bm, &bn, &bk);
  // the products' operands must fit the 31-bit byte offsets of the gather kernel
  const long long points = fused ? kPoints : 1;
  if (points * pl.tiles * p.C * 4 >= (1LL << 31) || pl.tiles * p.K * 4 >= (1LL << 31)) return false;
  if (4LL * (points * p.C + bk) * p.K >= (1LL << 31)) return false;
  if (fused) return igemm_dma_tile_has_wino(0, gemm_tile) && p.C % bk == 0;
  if (addressing == 0) return p.C % bk == 0;
  return addressing == 1;
}

size_t winograd_workspace_bytes(const Problem& p, int gemm_tile, bool fused) {
  const Plan pl = make_plan(p, fused);
  return pl.u_bytes + pl.v_bytes + pl.m_bytes + igemm_dma_workspace_bytes(pl.gemm, 0, gemm_tile, 1);
}

// The filter packed ahead of time: the transformed filter U, then U repacked for the products'
// tile (one per point, or the 16-point-long one of the fused variant).  Only the second part is
// read by a launch; U is the packing's intermediate.
size_t winograd_packed_filter_bytes(const Problem& p, int gemm_tile, bool fused) {
  const Plan pl = make_plan(p, fused);
  return pl.u_bytes + igemm_dma_packed_filter_bytes(pl.gemm, 0, gemm_tile);
}

hipError_t winograd_pack_filter(const Problem& p, int gemm_tile, bool fused, void* packed,
                                hipStream_t stream) {
  Plan pl = make_plan(p, fused);
  float* u = static_cast<float*>(packed);
  const long long fthreads = static_cast<long long>(p.C) * (p.K / 4);
  hipLaunchKernelGGL(filter_transform_kernel, dim3(static_cast<unsigned>((fthreads + 255) / 256)),
                     dim3(256), 0, stream, static_cast<const float*>(p.filt), u, p.C, p.K);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  pl.gemm.filt = u;
  return igemm_dma_pack_filter(pl.gemm, 0, gemm_tile, static_cast<unsigned char*>(packed) + pl.u_bytes,
                               stream);
}

hipError_t launch_winograd(const Problem& p, int gemm_tile, bool fused, hipStream_t stream) {
  Plan pl = make_plan(p, fused);
  unsigned char* ws = static_cast<unsigned char*>(p.workspace);
  float* u = reinterpret_cast<float*>(ws);
  float* v = reinterpret_cast<float*>(ws + pl.u_bytes);
  float* mt = reinterpret_cast<float*>(ws + pl.u_bytes + pl.v_bytes);
  void* gemm_ws = ws + pl.u_bytes + pl.v_bytes + pl.m_bytes;

  hipError_t e = hipSuccess;
  if (p.packed_filt) {
    pl.gemm.packed_filt = static_cast<const unsigned char*>(p.packed_filt) + pl.u_bytes;
  } else {
    const long long fthreads = static_cast<long long>(p.C) * (p.K / 4);
    hipLaunchKernelGGL(filter_transform_kernel,
                       dim3(static_cast<unsigned>((fthreads + 255) / 256)), dim3(256), 0, stream,
                       static_cast<const float*>(p.filt), u, p.C, p.K);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }

  const long long ithreads = pl.tiles * (p.C / 4);
  hipLaunchKernelGGL(input_transform_kernel, dim3(static_cast<unsigned>((ithreads + 255) / 256)),
                     dim3(256), 0, stream, static_cast<const float*>(p.in), v, p.N, p.H, p.W, p.C,
                     p.pt, p.pl, pl.TH, pl.TW);
  e = hipGetLastError();
  if (e != hipSuccess) return e;

  pl.gemm.in = v;
  pl.gemm.filt = u;
  pl.gemm.workspace = gemm_ws;
  if (fused) {
    pl.gemm.out = p.out;
    pl.gemm.pool = p.pool;
    return launch_igemm_dma_wino(pl.gemm, 0, gemm_tile, stream);
  }
  pl.gemm.out = mt;
  e = launch_igemm_dma(pl.gemm, 0, gemm_tile, 1, stream);
  if (e != hipSuccess) return e;

  const long long othreads = pl.tiles * (p.K / 4);
  hipLaunchKernelGGL(output_transform_kernel, dim3(static_cast<unsigned>((othreads + 255) / 256)),
                     dim3(256), 0, stream, mt, static_cast<float*>(p.out), p.N, p.P, p.Q, p.K,
                     pl.TH, pl.TW, p.bias, p.relu, p.pool);
  return hipGetLastError();
}

}  // namespace conv2d
