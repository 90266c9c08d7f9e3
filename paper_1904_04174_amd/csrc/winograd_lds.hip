// Winograd F(2x2, 3x3) forward convolution, fp32, stride 1, in ONE launch: the transform
// algorithm that section 3 of the paper lists beside its direct kernels, with the input
// transform, the 16 point-wise products and the output transform all inside one workgroup, so
// that neither the transformed input (4x the input) nor the products (4x the output) ever
// reach memory.  Only the filter is transformed ahead (U, 16/9 of the filter; it can be packed
// once and reused).
//
//   Y = A^T [ sum_c (G g G^T) .* (B^T d B) ] A      per 2x2 block of output pixels ("tile")
//
// A workgroup (4 wavefronts) owns 32 consecutive tiles (in (image, tile row, tile column)
// order) x 64 output features and walks the channels 4 at a time ("slice").  Per slice:
//
//   1. direct global->LDS loads bring the 16 input pixels x 4 channels of each tile (16 bytes
//      per pixel; pixels outside the image arrive as zeros through out-of-range offsets) and
//      the slice of U for the 64 features: U'[feature tile][slice][row a][64 features][4 k]
//      [column b] (point 4a + b), 16 KB that lie contiguously in memory, written that way by
//      winograd_lds_pack_kernel;
//   2. every thread transforms one (tile, channel) patch in registers (B^T d B), two of the
//      four rows of the transformed patch each (wavefronts 0, 1 the upper, 2, 3 the lower
//      rows), and writes V[row a][tile][4 k][column b] in LDS, 16 bytes per row;
//   3. per point, v_mfma_f32_16x16x4_f32 multiplies U (16 features x 4 k) by V (4 k x 16
//      tiles): a wavefront owns 16 tiles x 32 features, i.e. 16 points x 2 blocks of
//      accumulators (128 registers), and one 16-byte LDS read per operand block gives a lane
//      its values for the four points of a row a.
//
// U, the input pixels and V are double buffered (64 KB of LDS, two workgroups per compute
// unit): loads run one slice ahead (U) or two (input), the transform one slice ahead; one
// barrier per slice, placed before the slice's last four points so that their MFMAs cover the
// barrier and the first fragment reads of the next slice.  After the last slice each lane
// holds, for one tile and 2 x 4 consecutive features, all 16 points: it applies A^T . A in
// registers, then bias, activation and, when asked, the 2x2 maximum (a tile is one pooling
// window), and stores 16 bytes per pixel.
//
// All transform entries are 0, +-1 or +-1/2: integer-valued tensors give exact results, as with
// the separate-pass Winograd variants.
#include <type_traits>

#include "buffer_lds.h"
#include "conv2d_internal.h"

namespace conv2d {
namespace wlds {  // named namespace: the kernels' host stubs need external linkage

using namespace buf;

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kXcds = 8;
constexpr int kTiles = 32;     // tiles of a workgroup
constexpr int kFeatures = 64;  // features of a workgroup
constexpr int kBK = 4;         // channels of a slice
constexpr int kPoints = 16;
constexpr int kUBytes = kPoints * kFeatures * kBK * 4;  // a slice of U: 16 KB
constexpr int kRawBytes = 16 * kTiles * kBK * 4;        // the tiles' input pixels: 8 KB
constexpr int kVBytes = kPoints * kTiles * kBK * 4;     // their transform: 8 KB
constexpr int kU0 = 0, kRaw0 = 2 * kUBytes, kV0 = kRaw0 + 2 * kRawBytes;  // all double buffered
constexpr int kLdsBytes = kV0 + 2 * kVBytes;  // 64 KB
// s_waitcnt immediate (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8)
constexpr int kWaitLoadsAndLds = 0x0070;  // vmcnt(0) lgkmcnt(0)

// U'[nt][s][a][f][j][b] = sum_{r,q} G[a][r] G[b][q] filt[r][q][4s + j][64 nt + f] (0 for
// features past K): point t = 4a + b of the transformed filter; the four points of a row a lie
// together, and the 16-byte chunk j of feature f sits at position j ^ ((f >> 1) & 3) of the
// feature's 64 bytes (the bank swizzle of the fragment reads).  One thread per (feature, slice).
__global__ __launch_bounds__(256) void winograd_lds_pack_kernel(const float* __restrict__ filt,
                                                                float* __restrict__ u, int C,
                                                                int K, int nslices) {
  const int kpad = (K + kFeatures - 1) / kFeatures * kFeatures;
  const long long idx = static_cast<long long>(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= static_cast<long long>(kpad) * nslices) return;
  const int k = static_cast<int>(idx % kpad), s = static_cast<int>(idx / kpad);
  const size_t ck = static_cast<size_t>(C) * K;
  floatx4 out[4][kBK];  // [row a][channel j] -> the four columns b
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int j = 0; j < kBK; ++j) out[a][j] = floatx4{0.f, 0.f, 0.f, 0.f};
  if (k < K) {
#pragma unroll
    for (int j = 0; j < kBK; ++j) {
      const int c = s * kBK + j;
      float g[3][3];
#pragma unroll
      for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int q = 0; q < 3; ++q) g[r][q] = filt[(r * 3 + q) * ck + static_cast<size_t>(c) * K + k];
      // rows: t[a][q] = sum_r G[a][r] g[r][q]
      float t[4][3];
#pragma unroll
      for (int q = 0; q < 3; ++q) {
        const float sum02 = g[0][q] + g[2][q];
        t[0][q] = g[0][q];
        t[1][q] = 0.5f * (sum02 + g[1][q]);
        t[2][q] = 0.5f * (sum02 - g[1][q]);
        t[3][q] = g[2][q];
      }
      // columns: U[a][b] = sum_q t[a][q] G[b][q]
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const float sum02 = t[a][0] + t[a][2];
        out[a][j] = floatx4{t[a][0], 0.5f * (sum02 + t[a][1]), 0.5f * (sum02 - t[a][1]), t[a][2]};
      }
    }
  }
  const int nt = k / kFeatures, f = k % kFeatures;
  float* dst = u + (static_cast<size_t>(nt) * nslices + s) * (kUBytes / 4) + f * 16;
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int j = 0; j < kBK; ++j)
      *reinterpret_cast<floatx4*>(dst + a * (kFeatures * 16) + (j ^ ((f >> 1) & 3)) * 4) = out[a][j];
}

__global__ __launch_bounds__(256, 2) void winograd_lds_kernel(const Problem p,
                                                              const float* __restrict__ u,
                                                              const int TH, const int TW,
                                                              const int tiles, const int nslices,
                                                              const int tiles_n,
                                                              const int ntiles) {
  __shared__ __align__(1024) unsigned char lds[kLdsBytes];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int tg = wave >> 1;  // tile group of this wavefront: tiles 16 tg .. 16 tg + 15
  const int fg = wave & 1;   // feature group: features 32 fg .. 32 fg + 31
  const int lr = lane & 15;  // MFMA row / column of the lane
  const int lk = lane >> 4;  // its k

  // Workgroup i runs on XCD i % 8: every XCD gets a contiguous range of workgroup tiles, feature
  // tiles fastest, so that the workgroups that share input pixels share an L2.
  const int xcd = blockIdx.x % kXcds, local = blockIdx.x / kXcds;
  const int per = ntiles / kXcds, rem = ntiles % kXcds;
  const int tile = xcd * per + (xcd < rem ? xcd : rem) + local;
  const int t0 = (tile / tiles_n) * kTiles;
  const int nt = tile % tiles_n;
  const int n0 = nt * kFeatures;

  const uintx4 in_rsrc = make_rsrc(p.in, 4LL * p.N * p.H * p.W * p.C);
  const uintx4 u_rsrc =
      make_rsrc(u, 1LL * tiles_n * nslices * kUBytes);
  const unsigned lds_base = __builtin_amdgcn_readfirstlane(static_cast<unsigned>(
      reinterpret_cast<size_t>(lds)));

  // ---- loader role.  Input: wavefront w loads patch row w (4 pixels) of all 32 tiles, two
  // instructions of 64 (tile, pixel) entries per pixel column pair; lane -> entry.
  // LDS: raw[pixel 16][tile 32][4 channels].
  int raw_voff[2];
  {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      // instruction i covers pixels (row = wave, column 2 i + lane / 32), tile lane % 32
      const int t = t0 + (lane & 31);
      const bool t_ok = t < tiles;
      const int tt = t_ok ? t : 0;
      const int tw = tt % TW, th = (tt / TW) % TH, n = tt / (TW * TH);
      const int h = 2 * th - p.pt + wave, w = 2 * tw - p.pl + 2 * i + (lane >> 5);
      const bool ok = t_ok && static_cast<unsigned>(h) < static_cast<unsigned>(p.H) &&
                      static_cast<unsigned>(w) < static_cast<unsigned>(p.W);
      raw_voff[i] = ok ? ((n * p.H + h) * p.W + w) * p.C * 4 : kOutOfRange;
    }
  }
  auto load_raw = [&](int s, int buf) {
    const int soff = min(s, nslices - 1) * kBK * 4;  // (past the end: the last slice again)
#pragma unroll
    for (int i = 0; i < 2; ++i)
      dma16(in_rsrc, lds_base + kRaw0 + buf * kRawBytes + (wave * 4 + 2 * i) * (kTiles * 16),
            raw_voff[i], soff);
  };
  // U: the slice is 16 KB contiguous; wavefront w copies KB 4 w .. 4 w + 3
  const int u_voff = lane * 16;
  auto load_u = [&](int s, int buf) {
    const int soff = (nt * nslices + min(s, nslices - 1)) * kUBytes;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      dma16(u_rsrc, lds_base + kU0 + buf * kUBytes + (wave * 4 + i) * 1024, u_voff,
            soff + (wave * 4 + i) * 1024);
  };

  // ---- transform role: thread -> patch (tile, channel) = tid % 128; wavefronts 0 and 1 compute
  // rows 0, 1 of the transformed patch (from pixel rows 0..2), wavefronts 2 and 3 rows 2, 3 (from
  // pixel rows 1..3).  V[row a = group of 4 points][tile][channel][column b]: a thread writes
  // the four points of a row with one 16-byte store, the multipliers read them with one load.
  const int item = tid & 127;
  const bool lower = wave >= 2;  // (wave-uniform)
  // B^T rows: (1,0,-1,0), (0,1,1,0) need pixel rows 0..2; (0,-1,1,0), (0,1,0,-1) rows 1..3.  With
  // x0, x1, x2 = pixel rows 0, 1, 2 (upper) or 2, 3, 1 (lower) both pairs are
  // x0 - x2 and sign * x1 + x2 with sign = +1 (upper), -1 (lower): no per-lane selects.
  const int x_row0 = lower ? 2 : 0, x_row1 = lower ? 3 : 1, x_row2 = lower ? 1 : 2;
  const float x_sign = lower ? -1.f : 1.f;
  const unsigned char* raw_item = lds + kRaw0 + item * 4;
  float d[3][4], tr[2][4];
  auto raw_read = [&](int buf, int e) {  // e = 0..11: x(e / 4), column e % 4
    const int row = (e >> 2) == 0 ? x_row0 : (e >> 2) == 1 ? x_row1 : x_row2;
    d[e >> 2][e & 3] = *reinterpret_cast<const float*>(raw_item + buf * kRawBytes +
                                                       (row * 4 + (e & 3)) * (kTiles * 16));
  };
  auto row_transform = [&](int j) {
    tr[0][j] = d[0][j] - d[2][j];
    tr[1][j] = x_sign * d[1][j] + d[2][j];
  };
  // (16-byte chunk `channel` of a tile's 64-byte row sits at position channel ^ swizzle(tile),
  // see the fragment reads)
  const int v_write_off = (item >> 2) * 64 + (((item & 3) ^ ((item >> 3) & 3)) * 16);
  auto row_write = [&](int buf, int a) {
    const floatx4 o = {tr[a][0] - tr[a][2], tr[a][1] + tr[a][2], tr[a][2] - tr[a][1],
                       tr[a][1] - tr[a][3]};
    *reinterpret_cast<floatx4*>(lds + kV0 + buf * kVBytes + ((lower ? 2 : 0) + a) * (kTiles * 64) +
                                v_write_off) = o;
  };

  // ---- multiplier role
  floatx4 acc[kPoints][2];
#pragma unroll
  for (int t = 0; t < kPoints; ++t)
#pragma unroll
    for (int b = 0; b < 2; ++b) acc[t][b] = floatx4{0.f, 0.f, 0.f, 0.f};
  // U[group][feature][k][4 points], V[group][tile][k][4 points]: 64 bytes per row
  // A wavefront's 16-byte reads (row = lane % 16, chunk k = lane / 16) hit all banks only if the
  // chunks of a row are permuted: chunk k of row r sits at position k ^ ((r >> 1) & 3).
  const int frag_pos = (lk ^ ((lr >> 1) & 3)) * 16;
  const int a_off = (32 * fg + lr) * 64 + frag_pos;  // + group * 4096 + block * 1024
  const int b_off = (16 * tg + lr) * 64 + frag_pos;  // + group * 2048
  // fragments of a group of 4 points, two sets (one being used, one being read)
  floatx4 fa[2][2], fb[2];
  auto read_group = [&](int set, int buf, int group) {
    const unsigned char* ub = lds + kU0 + buf * kUBytes + group * (kFeatures * 64) + a_off;
    fa[set][0] = *reinterpret_cast<const floatx4*>(ub);
    fa[set][1] = *reinterpret_cast<const floatx4*>(ub + 1024);
    fb[set] = *reinterpret_cast<const floatx4*>(lds + kV0 + buf * kVBytes + group * (kTiles * 64) + b_off);
  };
  // the 8 MFMAs of a group with `side(m)` after MFMA m, pinned in that order
  auto multiply_group = [&](int set, int group, auto side) {
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      const int i = m >> 1, b = m & 1, point = 4 * group + i;
      acc[point][b] =
          __builtin_amdgcn_mfma_f32_16x16x4f32(fa[set][b][i], fb[set][i], acc[point][b], 0, 0, 0);
      side(m);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // ---- prologue: U(0), input(0) and input(1) in flight; transform(0); fragments of group 0
  load_u(0, 0);
  load_raw(0, 0);
  load_raw(1, 1);
  __builtin_amdgcn_s_waitcnt(kWaitLoadsAndLds);
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
#pragma unroll
  for (int e = 0; e < 12; ++e) raw_read(0, e);
#pragma unroll
  for (int j = 0; j < 4; ++j) row_transform(j);
  row_write(0, 0);
  row_write(0, 1);
  __builtin_amdgcn_s_waitcnt(kWaitLds);
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  read_group(0, 0, 0);
  __builtin_amdgcn_sched_barrier(0);

  // The lane's output tile and bias values, worked out here (the divisions and loads overlap the
  // first slice's waits; at the end they would delay the stores).
  const int t = t0 + 16 * tg + lr;
  const int tw = t % TW, th = (t / TW) % TH, n = t / (TW * TH);
  floatx4 bias2[2];
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int v = 0; v < 4; ++v) bias2[b][v] = bias_of(p.bias, n0 + 32 * fg + 16 * b + 4 * lk + v, p.K);

  // Slice s: U, V and its input pixels in buffer s % 2 (`cur`, a compile-time constant: the
  // loop body is a pair of slices).
  auto slice = [&](int s, auto cur_c) {
    constexpr int cur = decltype(cur_c)::value, nxt = cur ^ 1;
    // U(s + 1) into the buffer that slice s - 1 read; input(s + 2) into the buffer that the
    // transform read during slice s - 1
    // (nothing past the last slice: the epilogue would wait for those loads)
    if (s + 1 < nslices) load_u(s + 1, nxt);
    if (s + 2 < nslices) load_raw(s + 2, cur);
    // groups 0..2: the next group's fragments, then 8 MFMAs with the transform of input(s + 1)
    // into V(s + 1) between them: 12 reads, 4 row steps, 2 writes
    read_group(1, cur, 1);
    __builtin_amdgcn_sched_barrier(0);
    multiply_group(0, 0, [&](int m) {
      raw_read(nxt, m);
      if (m >= 4) raw_read(nxt, m + 4);
    });
    read_group(0, cur, 2);
    __builtin_amdgcn_sched_barrier(0);
    multiply_group(1, 1, [&](int m) {
      if (m & 1) row_transform(m >> 1);
    });
    read_group(1, cur, 3);
    __builtin_amdgcn_sched_barrier(0);
    multiply_group(0, 2, [&](int m) {
      if (m == 2) row_write(nxt, 0);
      if (m == 5) row_write(nxt, 1);
    });
    // U(s + 1) and input(s + 2) have landed, this wavefront's part of V(s + 1) is written and
    // its reads of slice s are done
    __builtin_amdgcn_s_waitcnt(kWaitLoadsAndLds);
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    // the last group runs from registers while the next slice's first fragments arrive
    read_group(0, nxt, 0);
    __builtin_amdgcn_sched_barrier(0);
    multiply_group(1, 3, [&](int) {});
  };
  int s = 0;
  for (; s + 1 < nslices; s += 2) {
    slice(s, std::integral_constant<int, 0>{});
    slice(s + 1, std::integral_constant<int, 1>{});
  }
  if (s < nslices) slice(s, std::integral_constant<int, 0>{});
  __builtin_amdgcn_s_waitcnt(kWaitLoadsAndLds);

  // ---- output transform and stores: lane = tile 16 tg + lr, features 4 lk .. 4 lk + 3 of the
  // two 16-feature blocks
  if (t >= tiles) return;
  float* out = static_cast<float*>(p.out);
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    const int k = n0 + 32 * fg + 16 * b + 4 * lk;
    if (k >= p.K) continue;  // (K is a multiple of 4)
    const floatx4 bias = bias2[b];
    // rows: r[i][c] = sum_a A^T[i][a] m[a][c], A^T = (1,1,1,0), (0,1,-1,-1)
    floatx4 r[2][4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      r[0][c] = acc[0 + c][b] + acc[4 + c][b] + acc[8 + c][b];
      r[1][c] = acc[4 + c][b] - acc[8 + c][b] - acc[12 + c][b];
    }
    floatx4 y[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      y[i][0] = r[i][0] + r[i][1] + r[i][2];
      y[i][1] = r[i][1] - r[i][2] - r[i][3];
    }
    if (p.pool) {
      // a tile is one 2x2 pooling window; bias and activation after the maximum (both monotone)
      if (th >= p.P / 2 || tw >= p.Q / 2) continue;
      floatx4 best;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const float m = fmaxf(fmaxf(y[0][0][v], y[0][1][v]), fmaxf(y[1][0][v], y[1][1][v]));
        best[v] = finish(m, bias[v], p.relu);
      }
      *reinterpret_cast<floatx4*>(
          out + ((static_cast<size_t>(n) * (p.P / 2) + th) * (p.Q / 2) + tw) * p.K + k) = best;
      continue;
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int op = 2 * th + i, oq = 2 * tw + j;
        if (op >= p.P || oq >= p.Q) continue;
        floatx4 o;
#pragma unroll
        for (int v = 0; v < 4; ++v) o[v] = finish(y[i][j][v], bias[v], p.relu);
        *reinterpret_cast<floatx4*>(out + ((static_cast<size_t>(n) * p.P + op) * p.Q + oq) * p.K + k) = o;
      }
  }
}

size_t u_bytes(const Problem& p) {
  const size_t tiles_n = (p.K + kFeatures - 1) / kFeatures;
  return tiles_n * (p.C / kBK) * kUBytes;
}

}  // namespace wlds
using namespace wlds;

bool winograd_lds_supports(const Problem& p) {
  if (p.in_bf16 || p.out_bf16) return false;
  if (p.R != 3 || p.S != 3 || p.sr != 1 || p.sc != 1) return false;
  if (p.C % kBK != 0 || p.K % 4 != 0 || p.M == 0 || p.batches > 1) return false;
  // 31-bit byte offsets into the input and into U'
  if (4LL * p.N * p.H * p.W * p.C >= (1LL << 31)) return false;
  if (u_bytes(p) >= (1ULL << 31)) return false;
  return true;
}

size_t winograd_lds_packed_filter_bytes(const Problem& p) { return (u_bytes(p) + 255) / 256 * 256; }
size_t winograd_lds_workspace_bytes(const Problem& p) { return winograd_lds_packed_filter_bytes(p); }

hipError_t winograd_lds_pack_filter(const Problem& p, void* packed, hipStream_t stream) {
  const int nslices = p.C / kBK;
  const long long threads = 1LL * ((p.K + kFeatures - 1) / kFeatures * kFeatures) * nslices;
  hipLaunchKernelGGL(winograd_lds_pack_kernel, dim3(static_cast<unsigned>((threads + 255) / 256)),
                     dim3(256), 0, stream, static_cast<const float*>(p.filt),
                     static_cast<float*>(packed), p.C, p.K, nslices);
  return hipGetLastError();
}

hipError_t launch_winograd_lds(const Problem& p, hipStream_t stream) {
  if (!winograd_lds_supports(p)) return hipErrorInvalidValue;
  const float* u = static_cast<const float*>(p.packed_filt);
  if (!u) {
    hipError_t e = winograd_lds_pack_filter(p, p.workspace, stream);
    if (e != hipSuccess) return e;
    u = static_cast<const float*>(p.workspace);
  }
  const int TH = (p.P + 1) / 2, TW = (p.Q + 1) / 2;
  const long long tiles = 1LL * p.N * TH * TW;
  const int tiles_n = (p.K + kFeatures - 1) / kFeatures;
  const long long ntiles = (tiles + kTiles - 1) / kTiles * tiles_n;
  if (tiles >= (1LL << 31) - kTiles || ntiles >= (1LL << 31)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(winograd_lds_kernel, dim3(static_cast<unsigned>(ntiles)), dim3(256), 0, stream,
                     p, u, TH, TW, static_cast<int>(tiles), p.C / kBK, tiles_n,
                     static_cast<int>(ntiles));
  return hipGetLastError();
}

}  // namespace conv2d
