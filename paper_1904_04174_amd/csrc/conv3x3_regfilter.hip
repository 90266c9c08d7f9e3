// 3x3, stride-1 convolution of bf16 layers with 64 channels and 64 features, for gfx950: the
// whole filter lives in registers.
//
// Such a layer (the first 3x3 stages of the VGG- and ResNet-style networks that the paper's
// section 3 benchmarks) has a short reduction, Kg = 576, and a large image: per output pixel it
// reads 128 bytes, writes 256 (fp32) and multiplies for 576 x 64 products, which puts it on the
// memory side of the MFMA ridge.  The tiled kernels spend its time elsewhere: a barrier and a
// filter slice from L2 for every 32 reduction indices (128 clocks of MFMA work per wave), and
// the filter, 72 KB, fetched again for every 32 KB of input.  Here
//
//  * a workgroup of 8 waves is persistent and owns the whole filter: wave (wm, wn) keeps the
//    MFMA operands of its 32 features for all 576 reduction indices in 144 registers per lane
//    (36 steps of 16 indices x 4 registers), loaded once from the HWCF filter as it lies;
//  * a tile is a 16 x 16 block of output pixels of one image; its 18 x 18 x 64 input patch is
//    fetched by direct global->LDS loads into one of two buffers (8 planes of 16-byte channel
//    chunks, so that a fragment read is conflict free), the next tile's while the current
//    tile's 72 MFMAs per wave run: the loop reads only the pixel operand from LDS;
//  * one barrier per tile.  A wave waits for its share of the next patch (issued a tile ago),
//    then issues its stores, then meets the others: the stores drain while the next tile is
//    multiplied, and no wave waits for a store it has just issued;
//  * workgroup i runs on XCD i % 8; every XCD walks a contiguous range of tiles, its 32
//    workgroups on neighbouring blocks, so that the halo rows of a block come from its L2.
//
// Requirements (checked on the host): bf16 input and filter, 3x3 window, stride 1, C = 64,
// K = 64, 16-byte aligned input, tensors below 2^31 bytes.  No workspace.
#include "buffer_lds.h"
#include "conv2d_internal.h"

namespace conv2d {
namespace rf {  // named namespace: the kernel's host stub needs external linkage

using namespace buf;

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kXcds = 8;
constexpr int kComputeUnits = 256;
constexpr int kC = 64, kK = 64;          // channels and features of the layers this kernel takes
constexpr int kBH = 16, kBW = 16;        // output pixels of a tile
constexpr int kPW = kBW + 2;             // patch row width
constexpr int kEntries = (kBH + 2) * kPW;          // 324 patch entries (pixels) of 128 bytes
constexpr int kChunks = (kEntries + 63) / 64;      // 6 loads of 64 entries per plane
constexpr int kPlanes = kC * 2 / 16;               // 8 planes: 16-byte chunk c of every entry
constexpr int kPlaneBytes = kChunks * 64 * 16;     // 6 KiB
constexpr int kPatchBytes = kPlanes * kPlaneBytes; // 48 KiB
constexpr int kSteps = 9 * kC / 16;                // 36 steps of 16 reduction indices
constexpr int kWaves = 8, kThreads = 64 * kWaves;
constexpr int kFilterBytes = 9 * kC * kK * 2;     // 72 KiB
static_assert(kFilterBytes >= kPatchBytes && kFilterBytes % (kThreads * 16) == 0, "staging copy");
static_assert(kPlanes == kWaves, "one plane per wave");

__device__ __forceinline__ unsigned short to_bf16_bits(float x) {
  unsigned int u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<unsigned short>((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<unsigned short>(u >> 16);
}

// gridDim.x workgroups; `tiles` = N * blocks per image.
template <bool OUT_BF16>
__global__ __launch_bounds__(kThreads) void conv3x3_regfilter_kernel(const Problem p,
                                                                     const int tiles,
                                                                     const int blocks_x,
                                                                     const int blocks_y) {
  // [patch buffer 0 | patch buffer 1]; the filter's staging copy overlies buffer 1 and beyond
  __shared__ __align__(1024) unsigned char lds[kPatchBytes + kFilterBytes];
  unsigned char* const patch = lds;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;   // 64 pixels x 32 features per wave
  const int lr = lane & 31, lk = lane >> 5;

  // ---- tiles of this workgroup: XCD x owns a contiguous range, walked with the stride of the
  // XCD's workgroup count
  const int nwg = gridDim.x;
  const int xcd = blockIdx.x % kXcds, local = blockIdx.x / kXcds;
  const int per = tiles / kXcds, rem = tiles % kXcds;
  const int range_first = xcd * per + (xcd < rem ? xcd : rem);
  const int range_end = range_first + per + (xcd < rem ? 1 : 0);
  const int tile_step = nwg / kXcds + (xcd < nwg % kXcds ? 1 : 0);
  int tile = range_first + local;
  if (tile >= range_end) return;

  const uintx4 in_rsrc = make_rsrc(p.in, 1LL * p.N * p.H * p.W * kC * 2);
  const unsigned lds_base = __builtin_amdgcn_readfirstlane(lds_address(patch));

  // ---- patch loader role: this wave loads plane `wave` (channels 8 wave .. 8 wave + 7) of all
  // entries, 64 entries per load; entry e is pixel (e / 18, e % 18) of the input block
  int ent_dy[kChunks], ent_dx[kChunks];
#pragma unroll
  for (int c = 0; c < kChunks; ++c) {
    const int e = c * 64 + lane;
    ent_dy[c] = e < kEntries ? e / kPW : 1 << 20;   // past the patch: never inside an image
    ent_dx[c] = e % kPW;
  }
  // (image, top row, left column) of a tile's output block
  auto block_of = [&](int t, int& bn, int& bp, int& bq) {
    bq = (t % blocks_x) * kBW;
    const int r = t / blocks_x;
    bp = (r % blocks_y) * kBH;
    bn = r / blocks_y;
  };
  // load number c of the patch of block (bn, bp, bq) into buffer `buf`
  auto load_chunk = [&](int buf, int c, int bn, int bp, int bq) {
    const int h = bp - p.pt + ent_dy[c], w = bq - p.pl + ent_dx[c];
    const bool ok = static_cast<unsigned>(h) < static_cast<unsigned>(p.H) &&
                    static_cast<unsigned>(w) < static_cast<unsigned>(p.W);
    const int voff = ok ? ((bn * p.H + h) * p.W + w) * (kC * 2) + wave * 16 : kOutOfRange;
    dma16(in_rsrc, lds_base + buf * kPatchBytes + wave * kPlaneBytes + c * 1024, voff, 0);
  };

  int bn, bp, bq;
  block_of(tile, bn, bp, bq);
#pragma unroll
  for (int c = 0; c < kChunks; ++c) load_chunk(0, c, bn, bp, bq);

  // ---- the filter operands of this wave: step s covers reduction indices 16 s + 8 lk + j,
  // j = 0 .. 7 (tap s / 4, channels 16 (s % 4) + 8 lk + j), of feature 32 wn + lr.  The filter
  // (576 rows of 64 features, 72 KiB) is copied to LDS as it lies, behind the first patch
  // buffer (over the second one, which nobody loads before the first tile's loop), and every
  // lane picks its 288 values from there.
  uintx4 breg[kSteps];
  {
    // 16-byte chunk q of the staging copy: filter row q / 8, position q % 8, which holds the 8
    // features of chunk (q % 8) ^ swizzle(row) (pairs of 32-byte pieces swapped by bit 1 of the
    // row: the transposing reads below then spread over the banks)
    const uintx4 f_rsrc = make_rsrc(p.filt, kFilterBytes);
#pragma unroll
    for (int i = 0; i < kFilterBytes / (kThreads * 16); ++i) {
      const int q = i * kThreads + tid;
      const int k = q / 8, c = (q % 8) ^ (((k >> 1) & 1) << 2);
      dma16(f_rsrc, lds_base + kPatchBytes + (i * kThreads + wave * 64) * 16, k * 128 + c * 16, 0);
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));   // this wave's part of the first patch and the filter
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    // ds_read_b64_tr_b16: the 16 lanes of a group hand in 4 rows x 16 features (lane a: row
    // a / 4, features 4 (a % 4) .. + 3) and lane i gets the 4 rows of feature i.  Lane l of
    // the MFMA operand (feature l % 32, reduction indices 8 (l / 32) .. + 7 of the step) reads
    // rows 8 lk + a / 4 and + 4 of the 16-feature piece 2 wn + (l / 16) % 2.
    typedef short shortx4 __attribute__((ext_vector_type(4)));
    typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));
    typedef __attribute__((address_space(3))) shortx4* lds_ptr;
    const int a = lane & 15, k = 8 * lk + a / 4;
    const unsigned char* src = lds + kPatchBytes + k * 128 + 8 * (a % 4) +
                               32 * ((2 * wn + ((lane >> 4) & 1)) ^ (((k >> 1) & 1) << 1));
#pragma unroll
    for (int s = 0; s < kSteps; ++s) {
      const uintx2 lo = __builtin_bit_cast(
          uintx2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(src + 16 * s * 128)));
      const uintx2 hi = __builtin_bit_cast(
          uintx2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(src + (16 * s + 4) * 128)));
      breg[s] = uintx4{lo.x, lo.y, hi.x, hi.y};
    }
    // every wave has its operands before anybody loads the second patch over the filter
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  }
  const float bias_col = bias_of(p.bias, wn * 32 + lr, kK);

  // ---- pixel operand addressing: block i of the wave covers pixels 64 wm + 32 i + lr of the
  // tile (row-major in the 16 x 16 block); plane 2 cb + lk of step (tap, cb)
  int a_frag[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int pm = wm * 64 + i * 32 + lr;
    a_frag[i] = ((pm / kBW) * kPW + pm % kBW) * 16 + lk * kPlaneBytes;
  }
  auto read_a = [&](int buf, int s, int i) {
    const int tap = s / 4, cb = s % 4;
    return *reinterpret_cast<const uintx4*>(patch + buf * kPatchBytes + a_frag[i] +
                                            2 * cb * kPlaneBytes +
                                            ((tap / 3) * kPW + tap % 3) * 16);
  };

  int buf = 0;
  for (;;) {
    const int tile_next = tile + tile_step;
    const bool has_next = tile_next < range_end;
    int nn = 0, np = 0, nq = 0;
    if (has_next) block_of(tile_next, nn, np, nq);

    floatx16 acc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;

    uintx4 af[2][2];
    af[0][0] = read_a(buf, 0, 0);
    af[0][1] = read_a(buf, 0, 1);
#pragma unroll
    for (int s = 0; s < kSteps; ++s) {
      if (s + 1 < kSteps) {
        af[(s + 1) & 1][0] = read_a(buf, s + 1, 0);
        af[(s + 1) & 1][1] = read_a(buf, s + 1, 1);
      }
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af[s & 1][0]),
                                                       __builtin_bit_cast(bf16x8, breg[s]),
                                                       acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af[s & 1][1]),
                                                       __builtin_bit_cast(bf16x8, breg[s]),
                                                       acc[1], 0, 0, 0);
      // the next tile's patch, one load every fourth step from step 2 on (every wave passed
      // the barrier before this tile, so nobody still reads the other buffer)
      if (s % 4 == 2 && s / 4 < kChunks) {
        if (has_next) load_chunk(buf ^ 1, s / 4, nn, np, nq);
      }
    }

    // this wave's loads of the next patch have landed (they are older than the stores below)
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));

    // ---- stores: lane l, register v -> pixel 8 (v / 4) + 4 (l / 32) + v % 4 of the block of
    // 32, feature l % 32
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int pm = wm * 64 + i * 32 + 8 * (v / 4) + 4 * lk + (v % 4);
        const int op = bp + pm / kBW, oq = bq + pm % kBW;
        if (op < p.P && oq < p.Q) {
          const size_t idx = (static_cast<size_t>(bn * p.P + op) * p.Q + oq) * kK + wn * 32 + lr;
          const float r = finish(acc[i][v], bias_col, p.relu);
          if (OUT_BF16)
            __builtin_nontemporal_store(to_bf16_bits(r), static_cast<unsigned short*>(p.out) + idx);
          else
            __builtin_nontemporal_store(r, static_cast<float*>(p.out) + idx);
        }
      }
    }
    if (!has_next) break;
    __builtin_amdgcn_s_barrier();   // the next patch is whole; this buffer is free
    asm volatile("" ::: "memory");
    tile = tile_next;
    bn = nn;
    bp = np;
    bq = nq;
    buf ^= 1;
  }
}

bool supports(const Problem& p) {
  if (!p.in_bf16 || p.R != 3 || p.S != 3 || p.sr != 1 || p.sc != 1) return false;
  if (p.C != kC || p.K != kK || p.batches > 1 || p.pool) return false;
  if (1LL * p.N * p.H * p.W * kC * 2 >= (1LL << 31)) return false;
  if (1LL * p.M * kK >= (1LL << 31)) return false;
  return true;
}

template <bool OUT_BF16>
hipError_t launch_one(const Problem& p, hipStream_t stream) {
  const int blocks_x = (p.Q + kBW - 1) / kBW, blocks_y = (p.P + kBH - 1) / kBH;
  const long long tiles = 1LL * p.N * blocks_x * blocks_y;
  if (tiles >= (1LL << 31)) return hipErrorInvalidValue;
  const int grid = tiles < kComputeUnits ? static_cast<int>(tiles) : kComputeUnits;
  hipLaunchKernelGGL((conv3x3_regfilter_kernel<OUT_BF16>), dim3(grid), dim3(kThreads), 0, stream,
                     p, static_cast<int>(tiles), blocks_x, blocks_y);
  return hipGetLastError();
}

}  // namespace rf

bool conv3x3_regfilter_supports(const Problem& p) { return rf::supports(p); }
hipError_t launch_conv3x3_regfilter(const Problem& p, hipStream_t stream) {
  if (!rf::supports(p)) return hipErrorInvalidValue;
  if (p.out_bf16) return rf::launch_one<true>(p, stream);
  return rf::launch_one<false>(p, stream);
}

}  // namespace conv2d
