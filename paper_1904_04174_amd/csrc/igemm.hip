// Forward convolution as an implicit GEMM on the CDNA4 matrix cores, for
// gfx950: fp32 on v_mfma_f32_32x32x2_f32, bf16 on v_mfma_f32_32x32x16_bf16
// (fp32 accumulation in both).
//
// GEMM view of the convolution of the paper's section 3:
//   D[M][K] = A[M][Kg] * B[Kg][K],  M = N*P*Q, Kg = R*S*C ordered (r,s,c).
//   B is the HWCF filter as it lies in memory, D is the NHWC output as it
//   lies in memory, and row m of A is gathered on the fly from the NHWC
//   input: R*S runs of C contiguous elements, or zeros where the window
//   hangs over the border.
//
// One workgroup owns a BM x BN tile of D.  Per BK-wide slice of Kg it stages
// the A and B tiles in LDS, both with k contiguous per row, so that one
// 16-byte LDS read gives a lane the consecutive k of its row that the MFMA
// wants (fp32: four k for four 32x32x2 MFMAs; bf16: the eight k of one
// 32x32x16 MFMA).  B arrives feature-contiguous from memory and is
// transposed in registers (VEC x VEC blocks) on its way to LDS.
//
// Global loads are raw buffer loads: a tap outside the image (or a row past
// M, or a k past Kg) gets an offset beyond the buffer and the hardware
// returns zeros, so the gather has no branches and no selects.  Loads run one
// slice ahead of the MFMAs through staging registers, LDS is double
// buffered, one barrier per slice.
//
// Two further features of the template:
//  * SCALAR tiles gather single elements instead of 16-byte vectors,
//    so they take any channel and feature count (C = 3 first layers, odd K)
//    and pointers aligned to one element.
//  * Split reduction: gridDim.y workgroups share one output tile, each takes
//    a contiguous range of k slices and writes an fp32 partial tile to the
//    workspace; split_reduce_kernel adds the partials in a fixed order (so
//    results do not depend on timing).  This is what fills the machine when
//    M*K is small (batch-1 layers deep in a network).
//
// Requirements (checked by the host before launch): vector tiles need C and K
// multiples of the 16-byte vector (4 fp32 / 8 bf16) and 16-byte aligned
// in/filt; all tiles need input and filter each below 2^31 bytes and the
// output below 2^31 elements.
#include <type_traits>

#include "conv2d_internal.h"
#include "split_in_launch.h"

namespace conv2d {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kXcds = 8;                      // workgroups are dealt round-robin over the 8 XCDs
constexpr unsigned kRsrcFlags = 0x00020000u;  // raw buffer, 32-bit data format
// byte offset 2^31: past the end of any buffer this kernel accepts, reads as zero
constexpr int kOutOfRange = static_cast<int>(0x80000000u);

template <bool BF16_, int BM_, int BN_, int BK_, int WAVES_M_, int WAVES_N_, bool TWO_LEVEL_,
          int OCC_, bool SCALAR_, int WAVES_K_ = 1>
struct Tile {
  static constexpr bool BF16 = BF16_;
  static constexpr int BM = BM_, BN = BN_, BK = BK_;
  // Two-level summation (fp32 tiles): the MFMA accumulators are added into a
  // second set of fp32 registers every `flush_slices` slices and restarted
  // from zero.  A chain of n fp32 additions has a rounding error that grows
  // like n; the split keeps both chains near sqrt(n), which is what holds the
  // 1e-4 tolerance at Kg = 4608 (a single chain measured 7e-5 at Kg = 2304
  // and 1.0e-4 at Kg = 4608).  Costs one extra register per accumulator.
  static constexpr bool TWO_LEVEL = TWO_LEVEL_;
  static constexpr int OCC = OCC_;  // wavefronts per SIMD the register allocation must allow
  static constexpr bool SCALAR = SCALAR_;  // element-wise global loads (any C, K)
  static constexpr int ES = BF16 ? 2 : 4;   // element size in bytes
  static constexpr int VEC = 16 / ES;       // elements per 16-byte vector
  static constexpr int KSTEP = 2 * VEC;     // k consumed per fragment read (two lane halves)
  static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
  // WAVES_K > 1: that many groups of waves share an output tile, each group
  // multiplies its own part of every slice's k range, and the groups' sums
  // are added through LDS in group order at the end (a split of the
  // reduction inside the workgroup: small tiles for small layers without a
  // second launch for the reduce)
  static constexpr int WAVES_K = WAVES_K_;
  static constexpr int NT = 64 * WAVES_M * WAVES_N * WAVES_K;
  static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  static constexpr int TM = WM / 32, TN = WN / 32;
  static constexpr int LD = BK + VEC;  // LDS row stride in elements: 16 bytes of padding keep
                                       // the 16-byte fragment reads free of bank conflicts
  static constexpr int AV = SCALAR ? 1 : VEC;  // elements per global load of A
  static constexpr int KV = BK / AV;           // global loads per A row
  static constexpr int A_ROWS_PER_PASS = NT / KV;
  static constexpr int A_ITERS = BM / A_ROWS_PER_PASS;
  // B work items: VEC(k) x VEC(n) blocks, or single elements for SCALAR tiles
  static constexpr int B_BLOCKS = SCALAR ? BK * BN : (BK / VEC) * (BN / VEC);
  static constexpr int B_ITERS = (B_BLOCKS + NT - 1) / NT;
  static constexpr int LDS_BYTES = 2 * (BM + BN) * LD * ES;
  static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile must be a multiple of 32x32");
  static_assert(BK % KSTEP == 0, "BK must be a multiple of the fragment step");
  static_assert((BK / KSTEP) % WAVES_K == 0, "fragment steps must divide over the k groups");
  static_assert((WAVES_K - 1) * (BM / WAVES_M / 32) * (BN / WAVES_N / 32) * 4096 * WAVES_M *
                        WAVES_N <= 2 * (BM + BN) * (BK + 16 / (BF16_ ? 2 : 4)) * (BF16_ ? 2 : 4),
                "the k groups' sums must fit the tile buffers");
  static_assert(NT % KV == 0 && BM % A_ROWS_PER_PASS == 0, "A tile must divide over the threads");
  static_assert(!(BF16 && TWO_LEVEL), "two-level summation is an fp32 feature");
  static_assert(LDS_BYTES <= 160 * 1024, "tile does not fit LDS");
};

// fp32 -> bf16 bits, round to nearest even (NaN stays NaN).
__device__ __forceinline__ unsigned short to_bf16_bits(float x) {
  unsigned int u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<unsigned short>((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<unsigned short>(u >> 16);
}

// Sum of the `splits` fp32 partial tiles of a split reduction, in a fixed
// order.  A workgroup covers 256 / groups vectors of 4 consecutive outputs;
// thread (vector o, group g) adds the partials g, g + groups, g + 2 groups ...
// in that order, and group 0 then adds the group sums in group order from LDS.
// `groups` is a power of two up to 16: with few outputs and many splits it
// spreads the otherwise serial chain of dependent loads over more threads.
template <bool OUT_BF16>
__global__ __launch_bounds__(256) void split_reduce_kernel(const float* __restrict__ partial,
                                                           void* __restrict__ out, int total,
                                                           int splits, int groups,
                                                           const float* __restrict__ bias, int relu,
                                                           int K) {
  __shared__ float4 sums[256];
  const int per_wg = 256 / groups;
  const int o = threadIdx.x % per_wg, g = threadIdx.x / per_wg;
  const int i0 = (blockIdx.x * per_wg + o) * 4;
  const bool vec = (total & 3) == 0;  // then every partial vector is 16-byte aligned and whole
  float4 acc = {0.f, 0.f, 0.f, 0.f};
  if (i0 < total) {
    for (int s = g; s < splits; s += groups) {
      const float* src = partial + static_cast<size_t>(s) * total + i0;
      float4 v = {0.f, 0.f, 0.f, 0.f};
      if (vec) {
        v = *reinterpret_cast<const float4*>(src);
      } else {
        v.x = src[0];
        if (i0 + 1 < total) v.y = src[1];
        if (i0 + 2 < total) v.z = src[2];
        if (i0 + 3 < total) v.w = src[3];
      }
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
  }
  sums[threadIdx.x] = acc;
  __syncthreads();
  if (g != 0 || i0 >= total) return;
  for (int j = 1; j < groups; ++j) {
    const float4 v = sums[j * per_wg + o];
    acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
  }
  // fused epilogue: the feature of flat output index i is i % K
  const int col = i0 % K;
  float a[4] = {acc.x, acc.y, acc.z, acc.w};
#pragma unroll
  for (int c = 0; c < 4; ++c) a[c] = finish(a[c], bias_of(bias, (col + c) % K, K), relu);
  acc = float4{a[0], a[1], a[2], a[3]};
  if (vec) {
    if (OUT_BF16) {
      ushort4 r = {to_bf16_bits(a[0]), to_bf16_bits(a[1]), to_bf16_bits(a[2]), to_bf16_bits(a[3])};
      *reinterpret_cast<ushort4*>(static_cast<unsigned short*>(out) + i0) = r;
    } else {
      *reinterpret_cast<float4*>(static_cast<float*>(out) + i0) = acc;
    }
  } else {
    for (int c = 0; c < 4 && i0 + c < total; ++c) {
      if (OUT_BF16)
        static_cast<unsigned short*>(out)[i0 + c] = to_bf16_bits(a[c]);
      else
        static_cast<float*>(out)[i0 + c] = a[c];
    }
  }
}

// gridDim.x = output tiles, gridDim.y = splits of the reduction.  With
// gridDim.y > 1 workgroup (x, y) multiplies slices [y*slices_per_split,
// (y+1)*slices_per_split) and stores an fp32 partial tile at
// p.workspace + y*M*K floats; otherwise it stores the result to p.out.
template <class T, bool OUT_BF16>
__global__ __launch_bounds__(T::NT, T::OCC) void igemm_kernel(const Problem p,
                                                              const int slices_per_split,
                                                              const int flush_slices,
                                                              unsigned* split_counters,
                                                              const int reduce_groups) {
  constexpr int BM = T::BM, BN = T::BN, BK = T::BK, LD = T::LD, NT = T::NT;
  constexpr int ES = T::ES, VEC = T::VEC, AV = T::AV;
  constexpr bool SCALAR = T::SCALAR;
  extern __shared__ __align__(16) unsigned char lds[];
  unsigned char* As = lds;                          // [2][BM][LD] elements
  unsigned char* Bs = lds + 2 * BM * LD * ES;       // [2][BN][LD] elements

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wk = wave / (T::WAVES_M * T::WAVES_N);           // k group of this wave
  const int wmn = wave % (T::WAVES_M * T::WAVES_N);
  const int wm = wmn / T::WAVES_N;
  const int wn = wmn % T::WAVES_N;
  const int lr = lane & 31;   // row (A) / column (B, D) inside a 32x32 MFMA tile
  const int lk = lane >> 5;   // which half of the k group this lane feeds

  // Tile of this workgroup.  Workgroup i runs on XCD i % 8; give each XCD a
  // contiguous range of tiles so that neighbours share input rows in its L2,
  // and walk feature tiles fastest so that an A tile is reused while hot.
  const int tiles_n = (p.K + BN - 1) / BN;
  const int nwg = gridDim.x;
  const int xcd = blockIdx.x % kXcds;
  const int local = blockIdx.x / kXcds;
  const int per = nwg / kXcds, rem = nwg % kXcds;
  const int tile = xcd * per + (xcd < rem ? xcd : rem) + local;
  const int m0 = (tile / tiles_n) * BM;
  const int n0 = (tile % tiles_n) * BN;

  // k slices of this workgroup
  const int nslices_all = (p.Kg + BK - 1) / BK;
  const int slice_begin = blockIdx.y * slices_per_split;
  const int nslices = min(slices_per_split, nslices_all - slice_begin);

  const __amdgpu_buffer_rsrc_t in_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<void*>(p.in), 0, p.N * p.H * p.W * p.C * ES, kRsrcFlags);
  const __amdgpu_buffer_rsrc_t filt_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<void*>(p.filt), 0, p.Kg * p.K * ES, kRsrcFlags);

  // ---- per-thread description of the A rows it gathers
  const int a_kv = tid % T::KV;
  const int a_row0 = tid / T::KV;
  int a_off[T::A_ITERS];  // element offset of tap (0,0), channel 0 of the row's window
  int a_h0[T::A_ITERS], a_w0[T::A_ITERS];
#pragma unroll
  for (int i = 0; i < T::A_ITERS; ++i) {
    const int m = m0 + a_row0 + i * T::A_ROWS_PER_PASS;
    if (m < p.M) {
      const int q = m % p.Q;
      const int t = m / p.Q;
      const int op = t % p.P;
      const int n = t / p.P;
      a_h0[i] = op * p.sr - p.pt;
      a_w0[i] = q * p.sc - p.pl;
      a_off[i] = ((n * p.H + a_h0[i]) * p.W + a_w0[i]) * p.C;
    } else {
      a_h0[i] = -(1 << 28);  // every tap fails the bounds test
      a_w0[i] = 0;
      a_off[i] = 0;
    }
  }
  // (r, s, c) of this thread's k (vector) in the next slice to load, and the
  // per-slice advance of BK channels split into whole taps and a channel
  // remainder so that stepping needs no division and no branch
  int k_next = slice_begin * BK;  // first k of the next slice to load
  int kc, ks, kr;
  {
    const int kg = k_next + a_kv * AV;
    kc = kg % p.C;
    const int t = kg / p.C;
    ks = t % p.S;
    kr = t / p.S;
  }
  const int step_c = BK % p.C;
  const int step_s = (BK / p.C) % p.S;
  const int step_r = (BK / p.C) / p.S;
  // B, vector tiles: VEC(k) x VEC(n) blocks, first k row and column fixed per
  // thread.  SCALAR tiles: single elements, columns fastest over the threads.
  int b_col[T::B_ITERS], b_krow[T::B_ITERS];
#pragma unroll
  for (int i = 0; i < T::B_ITERS; ++i) {
    const int b = tid + i * NT;
    const int per_row = SCALAR ? BN : BN / VEC;
    const int col = n0 + (b % per_row) * (SCALAR ? 1 : VEC);
    const int kb = b / per_row;
    b_krow[i] = (b < T::B_BLOCKS && col < p.K) ? kb * (SCALAR ? 1 : VEC) : (1 << 30);
    b_col[i] = col;
  }

  // staging registers (only the set that matches the tile kind is live)
  uintx4 a_vec[SCALAR ? 1 : T::A_ITERS];
  uintx4 b_vec[SCALAR ? 1 : T::B_ITERS][VEC];
  unsigned a_elt[SCALAR ? T::A_ITERS : 1];
  unsigned b_elt[SCALAR ? T::B_ITERS : 1];

  auto issue_loads = [&]() {
    const int tap = (kr * p.W + ks) * p.C + kc;
    // past the last window row (k >= Kg) the row test below must fail
    const int kr_t = (kr < p.R) ? kr : (1 << 30);
#pragma unroll
    for (int i = 0; i < T::A_ITERS; ++i) {
      const bool ok = (static_cast<unsigned>(a_h0[i] + kr_t) < static_cast<unsigned>(p.H)) &
                      (static_cast<unsigned>(a_w0[i] + ks) < static_cast<unsigned>(p.W));
      const int off = ok ? (a_off[i] + tap) * ES : kOutOfRange;
      if constexpr (SCALAR && T::BF16)
        a_elt[i] = static_cast<unsigned short>(__builtin_amdgcn_raw_buffer_load_b16(in_rsrc, off, 0, 0));
      else if constexpr (SCALAR)
        a_elt[i] = __builtin_amdgcn_raw_buffer_load_b32(in_rsrc, off, 0, 0);
      else
        a_vec[i] = __builtin_amdgcn_raw_buffer_load_b128(in_rsrc, off, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < T::B_ITERS; ++i) {
      if constexpr (SCALAR) {
        const int kg = k_next + b_krow[i];
        const int off = (kg < p.Kg) ? (kg * p.K + b_col[i]) * ES : kOutOfRange;
        if constexpr (T::BF16)
          b_elt[i] = static_cast<unsigned short>(
              __builtin_amdgcn_raw_buffer_load_b16(filt_rsrc, off, 0, 0));
        else
          b_elt[i] = __builtin_amdgcn_raw_buffer_load_b32(filt_rsrc, off, 0, 0);
      } else {
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
          const int kg = k_next + b_krow[i] + j;
          const int off = (kg < p.Kg) ? (kg * p.K + b_col[i]) * ES : kOutOfRange;
          b_vec[i][j] = __builtin_amdgcn_raw_buffer_load_b128(filt_rsrc, off, 0, 0);
        }
      }
    }
    // advance to the following slice
    k_next += BK;
    kc += step_c;
    const int carry_c = kc >= p.C;
    kc -= carry_c ? p.C : 0;
    ks += step_s + carry_c;
    const int carry_s = ks >= p.S;
    ks -= carry_s ? p.S : 0;
    kr += step_r + carry_s;
  };
  auto store_tiles = [&](int buf) {
    unsigned char* as = As + buf * BM * LD * ES;
    unsigned char* bs = Bs + buf * BN * LD * ES;
#pragma unroll
    for (int i = 0; i < T::A_ITERS; ++i) {
      unsigned char* dst = as + ((a_row0 + i * T::A_ROWS_PER_PASS) * LD + a_kv * AV) * ES;
      if constexpr (SCALAR && T::BF16)
        *reinterpret_cast<unsigned short*>(dst) = static_cast<unsigned short>(a_elt[i]);
      else if constexpr (SCALAR)
        *reinterpret_cast<unsigned*>(dst) = a_elt[i];
      else
        *reinterpret_cast<uintx4*>(dst) = a_vec[i];
    }
#pragma unroll
    for (int i = 0; i < T::B_ITERS; ++i) {
      const int b = tid + i * NT;
      if (b < T::B_BLOCKS) {
        if constexpr (SCALAR) {
          // LDS keeps B as [n][k], k contiguous
          unsigned char* dst = bs + ((b % BN) * LD + b / BN) * ES;
          if constexpr (T::BF16)
            *reinterpret_cast<unsigned short*>(dst) = static_cast<unsigned short>(b_elt[i]);
          else
            *reinterpret_cast<unsigned*>(dst) = b_elt[i];
        } else {
          const int nbv = b % (BN / VEC);
          const int kb = b / (BN / VEC);
          // VEC x VEC transpose in registers
          unsigned char* dst = bs + ((nbv * VEC) * LD + kb * VEC) * ES;
          if constexpr (T::BF16) {
#pragma unroll
            for (int n = 0; n < 8; ++n) {
              const unsigned sel = (n & 1) ? 0x07060302u : 0x05040100u;  // high / low halves
              uintx4 v;
#pragma unroll
              for (int j = 0; j < 4; ++j)
                v[j] = __builtin_amdgcn_perm(b_vec[i][2 * j + 1][n >> 1], b_vec[i][2 * j][n >> 1],
                                             sel);
              *reinterpret_cast<uintx4*>(dst + n * LD * ES) = v;
            }
          } else {
#pragma unroll
            for (int n = 0; n < 4; ++n)
              *reinterpret_cast<uintx4*>(dst + n * LD * ES) =
                  uintx4{b_vec[i][0][n], b_vec[i][1][n], b_vec[i][2][n], b_vec[i][3][n]};
          }
        }
      }
    }
  };

  floatx16 acc[T::TM][T::TN];
#pragma unroll
  for (int i = 0; i < T::TM; ++i)
#pragma unroll
    for (int j = 0; j < T::TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  floatx16 total[T::TWO_LEVEL ? T::TM : 1][T::TWO_LEVEL ? T::TN : 1];
  if (T::TWO_LEVEL) {
#pragma unroll
    for (int i = 0; i < T::TM; ++i)
#pragma unroll
      for (int j = 0; j < T::TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) total[i][j][v] = 0.f;
  }
  int until_flush = flush_slices;

  auto multiply = [&](int buf) {
    const unsigned char* as = As + (buf * BM * LD + (wm * T::WM + lr) * LD + lk * VEC) * ES;
    const unsigned char* bs = Bs + (buf * BN * LD + (wn * T::WN + lr) * LD + lk * VEC) * ES;
    constexpr int KK = BK / T::KSTEP / T::WAVES_K;  // fragment steps of one k group
#pragma unroll
    for (int k0 = 0; k0 < KK; ++k0) {
      const int kk = wk * KK + k0;
      uintx4 af[T::TM], bf[T::TN];
#pragma unroll
      for (int i = 0; i < T::TM; ++i)
        af[i] = *reinterpret_cast<const uintx4*>(as + (i * 32 * LD + kk * T::KSTEP) * ES);
#pragma unroll
      for (int j = 0; j < T::TN; ++j)
        bf[j] = *reinterpret_cast<const uintx4*>(bs + (j * 32 * LD + kk * T::KSTEP) * ES);
#pragma unroll
      for (int i = 0; i < T::TM; ++i)
#pragma unroll
        for (int j = 0; j < T::TN; ++j) {
          if (T::BF16) {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                __builtin_bit_cast(bf16x8, af[i]), __builtin_bit_cast(bf16x8, bf[j]), acc[i][j], 0,
                0, 0);
          } else {
#pragma unroll
            for (int t = 0; t < 4; ++t)
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                  __uint_as_float(af[i][t]), __uint_as_float(bf[j][t]), acc[i][j], 0, 0, 0);
          }
        }
    }
    if (T::TWO_LEVEL) {
      if (--until_flush == 0) {
        until_flush = flush_slices;
#pragma unroll
        for (int i = 0; i < T::TM; ++i)
#pragma unroll
          for (int j = 0; j < T::TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              total[i][j][v] += acc[i][j][v];
              acc[i][j][v] = 0.f;
            }
      }
    }
  };

  // The slice loaded after the last one of this workgroup is multiplied by
  // nobody, so the pipeline needs no tail special case (past Kg it reads as
  // zeros: its offsets are out of range).
  issue_loads();
  store_tiles(0);
  __syncthreads();

  for (int slice = 0; slice < nslices; slice += 2) {
    // even slice: its data is in LDS buffer 0 and the staging registers are
    // free.  The scheduling fences keep the loads ahead of the MFMAs: if the
    // compiler sinks them, their destination registers get shared with the
    // LDS fragments and every LDS read then waits for all loads in flight.
    issue_loads();
    __builtin_amdgcn_sched_barrier(0);
    multiply(0);
    __builtin_amdgcn_sched_barrier(0);
    store_tiles(1);
    __syncthreads();
    if (slice + 1 >= nslices) break;
    issue_loads();
    __builtin_amdgcn_sched_barrier(0);
    multiply(1);
    __builtin_amdgcn_sched_barrier(0);
    store_tiles(0);
    __syncthreads();
  }
  if (T::TWO_LEVEL) {
#pragma unroll
    for (int i = 0; i < T::TM; ++i)
#pragma unroll
      for (int j = 0; j < T::TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] += total[i][j][v];
  }

  if constexpr (T::WAVES_K > 1) {
    // sum of the k groups, in group order, through LDS (the tile buffers are free now)
    float* red = reinterpret_cast<float*>(lds);
    const int slot = wmn * 64 + lane;  // one float per (wave position, lane) and accumulator register
    constexpr int PER_GROUP = T::WAVES_M * T::WAVES_N * 64 * T::TM * T::TN * 16;
    __syncthreads();
    if (wk > 0) {
#pragma unroll
      for (int i = 0; i < T::TM; ++i)
#pragma unroll
        for (int j = 0; j < T::TN; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            red[(wk - 1) * PER_GROUP + ((i * T::TN + j) * 16 + v) * (T::WAVES_M * T::WAVES_N * 64) +
                slot] = acc[i][j][v];
    }
    __syncthreads();
    // (with the sum of the splits inside the launch, the other groups' waves come back for it)
    if (wk > 0 && split_counters == nullptr) return;
    if (wk == 0) {
#pragma unroll
      for (int g = 0; g < T::WAVES_K - 1; ++g)
#pragma unroll
        for (int i = 0; i < T::TM; ++i)
#pragma unroll
          for (int j = 0; j < T::TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v)
              acc[i][j][v] += red[g * PER_GROUP + ((i * T::TN + j) * 16 + v) *
                                                      (T::WAVES_M * T::WAVES_N * 64) + slot];
    }
  }

  // ---- epilogue: D tile -> NHWC output (or the fp32 partial of this split).
  // In a 32x32 accumulator, lane l register v holds row 8*(v/4) + 4*(l/32) +
  // v%4, column l%32, so each store instruction writes two contiguous
  // 32-element row segments.
  // The bias of this lane's columns, fetched before the first store.  The empty asm makes the
  // values "arrive" here, in uniform control flow: left to itself the compiler waits for the
  // loads inside every bounds-checked store block, and that wait (the counter covers loads
  // and stores alike) drains all earlier stores each time, one round trip per store.
  float bias_col[T::TN];
#pragma unroll
  for (int j = 0; j < T::TN; ++j)
    bias_col[j] = bias_of(p.bias, n0 + wn * T::WN + j * 32 + lr, p.K);
#pragma unroll
  for (int j = 0; j < T::TN; ++j) asm volatile("" : "+v"(bias_col[j]));
  const bool to_partial = gridDim.y > 1;
  const bool in_launch = split_counters != nullptr;
  float* part = static_cast<float*>(p.workspace) +
                static_cast<size_t>(blockIdx.y) * static_cast<size_t>(p.M) * p.K;
  if (wk == 0) {
#pragma unroll
  for (int i = 0; i < T::TM; ++i) {
#pragma unroll
    for (int j = 0; j < T::TN; ++j) {
      const int col = n0 + wn * T::WN + j * 32 + lr;
      const int rbase = m0 + wm * T::WM + i * 32 + lk * 4;
      const float bcol = bias_col[j];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = rbase + 8 * (v / 4) + (v % 4);
        if (row < p.M && col < p.K) {
          const size_t idx = static_cast<size_t>(row) * p.K + col;
          if (in_launch)
            splitk::split_store(part + idx, acc[i][j][v]);
          else if (to_partial)
            part[idx] = acc[i][j][v];
          else if (OUT_BF16)
            static_cast<unsigned short*>(p.out)[idx] =
                to_bf16_bits(finish(acc[i][j][v], bcol, p.relu));
          else
            static_cast<float*>(p.out)[idx] = finish(acc[i][j][v], bcol, p.relu);
        }
      }
    }
  }
  }  // waves of k group 0
  if (!in_launch) return;

  // ---- split reduction inside the launch (split_in_launch.h), by all waves of the workgroup;
  // the tile buffers are free (the call's first step is a barrier)
  if constexpr (BM * BN <= 128 * 64 && BM * BN / 4 % NT == 0) {
    // (loads in flight per thread: up to 8 vectors of 16 bytes, the chain of dependent round
    // trips to the other XCDs' data is what the last workgroup spends its time on)
    constexpr int PER = BM * BN / 4 / NT;
    constexpr int AHEAD = PER == 1 ? 8 : PER == 2 ? 4 : PER <= 4 ? 3 : 2;
    splitk::split_reduce_in_launch<BM, BN, NT, OUT_BF16, AHEAD>(
        p, static_cast<const float*>(p.workspace), split_counters + tile, gridDim.y,
        reduce_groups, m0, n0, reinterpret_cast<unsigned*>(lds), tid);
  }
}

template <class T, bool OUT_BF16>
hipError_t launch_one(const Problem& p, int splits, hipStream_t stream) {
  const int tiles_m = (p.M + T::BM - 1) / T::BM;
  const int tiles_n = (p.K + T::BN - 1) / T::BN;
  const size_t lds_bytes = T::LDS_BYTES;
  if (lds_bytes > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&igemm_kernel<T, OUT_BF16>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       static_cast<int>(lds_bytes));
    if (e != hipSuccess) return e;
  }
  const int nslices = (p.Kg + T::BK - 1) / T::BK;
  if (splits < 1) splits = 1;
  if (splits > nslices) splits = nslices;
  const int per_split = (nslices + splits - 1) / splits;
  splits = (nslices + per_split - 1) / per_split;  // no empty split
  // flush interval of the two-level summation: about sqrt(#slices)
  int flush = 1;
  while (flush * flush < per_split) ++flush;
  // A split adds its partial sums inside the launch where it can and where it pays
  // (split_in_launch.h), given a counter bank for the stream.
  unsigned* counters = nullptr;
  if (T::BM * T::BN / 4 % T::NT == 0 &&
      splitk::split_in_launch_pays(p, T::BM, T::BN, splits, OUT_BF16))
    counters = split_counters_for_stream(stream, tiles_m * tiles_n);
  hipLaunchKernelGGL((igemm_kernel<T, OUT_BF16>), dim3(tiles_m * tiles_n, splits), dim3(T::NT),
                     lds_bytes, stream, p, per_split, flush, counters,
                     split_reduce_groups(p.M * p.K, splits));
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || splits == 1 || counters) return e;
  return launch_split_reduce(static_cast<const float*>(p.workspace), p.out, p.M * p.K, splits,
                             OUT_BF16, p.bias, p.relu, p.K, stream);
}

template <class T>
hipError_t launch(const Problem& p, int splits, hipStream_t stream) {
  if (T::BF16 && p.out_bf16) return launch_one<T, T::BF16>(p, splits, stream);
  return launch_one<T, false>(p, splits, stream);
}

struct TileEntry {
  const char* name;
  int bm, bn, bk, occ;
  bool scalar;
  hipError_t (*fn)(const Problem&, int, hipStream_t);
  int waves_k;
};

#define CONV2D_TILE(dt, isbf, bm, bn, bk, wm, wn, two, occ, scalar, tag) \
  { "igemm_" dt "_" #bm "x" #bn "x" #bk tag, bm, bn, bk, occ, scalar, \
    &launch<Tile<isbf, bm, bn, bk, wm, wn, two, occ, scalar>>, 1 }
// tiles whose waves also split the k range of a slice (see Tile::WAVES_K)
#define CONV2D_TILE_K(dt, isbf, bm, bn, bk, wm, wn, wk, two, occ)     \
  { "igemm_" dt "_" #bm "x" #bn "x" #bk "_k" #wk, bm, bn, bk, occ, false, \
    &launch<Tile<isbf, bm, bn, bk, wm, wn, two, occ, false, wk>>, wk }

const TileEntry kTilesF32[] = {
    CONV2D_TILE("f32", false, 256, 128, 16, 4, 2, true, 2, false, ""),
    CONV2D_TILE("f32", false, 128, 128, 16, 2, 2, true, 2, false, ""),
    CONV2D_TILE("f32", false, 256, 64, 16, 4, 1, true, 2, false, ""),
    CONV2D_TILE("f32", false, 128, 64, 16, 2, 2, true, 3, false, ""),
    CONV2D_TILE("f32", false, 64, 64, 16, 2, 2, true, 4, false, ""),
    CONV2D_TILE("f32", false, 128, 32, 16, 4, 1, true, 4, false, ""),
    CONV2D_TILE("f32", false, 128, 128, 32, 2, 2, true, 2, false, ""),
    CONV2D_TILE("f32", false, 128, 64, 32, 2, 2, true, 3, false, ""),
    CONV2D_TILE("f32", false, 256, 128, 32, 4, 2, true, 2, false, ""),
    CONV2D_TILE_K("f32", false, 32, 32, 64, 1, 1, 4, true, 4),
    CONV2D_TILE_K("f32", false, 64, 32, 32, 2, 1, 2, true, 4),
    CONV2D_TILE("f32", false, 128, 64, 16, 2, 2, true, 3, true, "_scalar"),
    CONV2D_TILE("f32", false, 64, 64, 16, 2, 2, true, 4, true, "_scalar"),
    CONV2D_TILE("f32", false, 128, 32, 16, 4, 1, true, 4, true, "_scalar"),
};
const TileEntry kTilesBf16[] = {
    CONV2D_TILE("bf16", true, 128, 128, 64, 2, 2, false, 2, false, ""),
    CONV2D_TILE("bf16", true, 128, 128, 32, 2, 2, false, 2, false, ""),
    CONV2D_TILE("bf16", true, 128, 64, 64, 2, 2, false, 3, false, ""),
    CONV2D_TILE("bf16", true, 128, 64, 32, 2, 2, false, 3, false, ""),
    CONV2D_TILE("bf16", true, 64, 64, 32, 2, 2, false, 4, false, ""),
    CONV2D_TILE_K("bf16", true, 32, 32, 128, 1, 1, 4, false, 4),
    CONV2D_TILE_K("bf16", true, 64, 32, 64, 2, 1, 2, false, 4),
    // element-wise gathers: any C and K (a 3-channel stem in bf16), 2-byte alignment
    CONV2D_TILE("bf16", true, 128, 64, 32, 2, 2, false, 3, true, "_scalar"),
    CONV2D_TILE("bf16", true, 64, 64, 32, 2, 2, false, 4, true, "_scalar"),
};
constexpr int kNumF32 = sizeof(kTilesF32) / sizeof(kTilesF32[0]);
constexpr int kNumBf16 = sizeof(kTilesBf16) / sizeof(kTilesBf16[0]);

}  // namespace

// more groups while the grid would stay under two workgroups per compute unit
int split_reduce_groups(int total, int splits) {
  const int vecs = (total + 3) / 4;
  int groups = 1;
  while (groups < 16 && groups * 2 <= splits && (vecs + 256 / groups - 1) / (256 / groups) < 512)
    groups *= 2;
  return groups;
}

hipError_t launch_split_reduce(const float* partial, void* out, int total, int splits,
                               bool out_bf16, const float* bias, int relu, int K,
                               hipStream_t stream) {
  const int vecs = (total + 3) / 4;
  const int groups = split_reduce_groups(total, splits);
  const int per_wg = 256 / groups;
  const dim3 grid((vecs + per_wg - 1) / per_wg), block(256);
  if (out_bf16)
    hipLaunchKernelGGL((split_reduce_kernel<true>), grid, block, 0, stream, partial, out, total,
                       splits, groups, bias, relu, K);
  else
    hipLaunchKernelGGL((split_reduce_kernel<false>), grid, block, 0, stream, partial, out, total,
                       splits, groups, bias, relu, K);
  return hipGetLastError();
}

int igemm_num_tiles(int bf16) { return bf16 ? kNumBf16 : kNumF32; }
static const TileEntry& entry(int bf16, int tile) { return bf16 ? kTilesBf16[tile] : kTilesF32[tile]; }
const char* igemm_tile_name(int bf16, int tile) { return entry(bf16, tile).name; }
void igemm_tile_shape(int bf16, int tile, int* bm, int* bn, int* bk) {
  const TileEntry& t = entry(bf16, tile);
  *bm = t.bm;
  *bn = t.bn;
  *bk = t.bk;
}
int igemm_tile_occupancy(int bf16, int tile) { return entry(bf16, tile).occ; }
bool igemm_tile_is_scalar(int bf16, int tile) { return entry(bf16, tile).scalar; }
int igemm_tile_waves_k(int bf16, int tile) { return entry(bf16, tile).waves_k; }
hipError_t launch_igemm(const Problem& p, int bf16, int tile, int splits, hipStream_t stream) {
  return entry(bf16, tile).fn(p, splits, stream);
}

}  // namespace conv2d
