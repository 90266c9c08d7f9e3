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
// returns zeros, so the gather has no branches and no selects.  Loads run PF
// slices ahead of the MFMAs through PF register sets, LDS is double
// buffered, one barrier per slice.
//
// Requirements (checked by the host before launch): C and K multiples of the
// 16-byte vector (4 fp32 / 8 bf16), 16-byte aligned in/filt, input and
// filter each below 2^31 bytes, output below 2^31 elements.
#include <type_traits>

#include "conv2d_internal.h"

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
          int OCC_, int PF_>
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
  static constexpr int PF = PF_;    // slices of global-load lookahead (register sets)
  static constexpr int ES = BF16 ? 2 : 4;   // element size in bytes
  static constexpr int VEC = 16 / ES;       // elements per 16-byte vector
  static constexpr int KSTEP = 2 * VEC;     // k consumed per fragment read (two lane halves)
  static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
  static constexpr int NT = 64 * WAVES_M * WAVES_N;
  static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  static constexpr int TM = WM / 32, TN = WN / 32;
  static constexpr int LD = BK + VEC;  // LDS row stride in elements: 16 bytes of padding keep
                                       // the 16-byte fragment reads free of bank conflicts
  static constexpr int KV = BK / VEC;  // 16-byte vectors per A row
  static constexpr int A_ROWS_PER_PASS = NT / KV;
  static constexpr int A_ITERS = BM / A_ROWS_PER_PASS;
  static constexpr int B_BLOCKS = (BK / VEC) * (BN / VEC);  // VEC(k) x VEC(n) blocks
  static constexpr int B_ITERS = (B_BLOCKS + NT - 1) / NT;
  static constexpr int LDS_BYTES = 2 * (BM + BN) * LD * ES;
  static_assert(PF == 1 || PF == 2, "one or two register sets");
  static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile must be a multiple of 32x32");
  static_assert(BK % KSTEP == 0, "BK must be a multiple of the fragment step");
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

template <class T, bool OUT_BF16>
__global__ __launch_bounds__(T::NT, T::OCC) void igemm_kernel(const Problem p,
                                                              const int flush_slices) {
  constexpr int BM = T::BM, BN = T::BN, BK = T::BK, LD = T::LD, NT = T::NT, PF = T::PF;
  constexpr int ES = T::ES, VEC = T::VEC;
  extern __shared__ __align__(16) unsigned char lds[];
  unsigned char* As = lds;                          // [2][BM][LD] elements
  unsigned char* Bs = lds + 2 * BM * LD * ES;       // [2][BN][LD] elements

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave / T::WAVES_N;
  const int wn = wave % T::WAVES_N;
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
  // (r, s, c) of this thread's k vector in the next slice to load, and the
  // per-slice advance of BK channels split into whole taps and a channel
  // remainder so that stepping needs no division and no branch
  int kc, ks, kr;
  {
    const int kg = a_kv * VEC;
    kc = kg % p.C;
    const int t = kg / p.C;
    ks = t % p.S;
    kr = t / p.S;
  }
  const int step_c = BK % p.C;
  const int step_s = (BK / p.C) % p.S;
  const int step_r = (BK / p.C) / p.S;
  // B: VEC(k) x VEC(n) blocks; the column part of the offset is fixed per thread
  int b_col[T::B_ITERS], b_krow[T::B_ITERS];
#pragma unroll
  for (int i = 0; i < T::B_ITERS; ++i) {
    const int b = tid + i * NT;
    const int nbv = b % (BN / VEC);
    const int kb = b / (BN / VEC);
    const int col = n0 + nbv * VEC;
    b_krow[i] = (b < T::B_BLOCKS && col < p.K) ? kb * VEC : (1 << 30);  // first k row of the block
    b_col[i] = col;
  }
  int k_next = 0;  // first k of the next slice to load

  uintx4 a_reg[PF][T::A_ITERS];
  uintx4 b_reg[PF][T::B_ITERS][VEC];

  auto issue_loads = [&](auto set_c) {
    constexpr int set = decltype(set_c)::value;
    const int tap = (kr * p.W + ks) * p.C + kc;
    // past the last window row (k >= Kg) the row test below must fail
    const int kr_t = (kr < p.R) ? kr : (1 << 30);
#pragma unroll
    for (int i = 0; i < T::A_ITERS; ++i) {
      const bool ok = (static_cast<unsigned>(a_h0[i] + kr_t) < static_cast<unsigned>(p.H)) &
                      (static_cast<unsigned>(a_w0[i] + ks) < static_cast<unsigned>(p.W));
      const int off = ok ? (a_off[i] + tap) * ES : kOutOfRange;
      a_reg[set][i] = __builtin_amdgcn_raw_buffer_load_b128(in_rsrc, off, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < T::B_ITERS; ++i) {
#pragma unroll
      for (int j = 0; j < VEC; ++j) {
        const int kg = k_next + b_krow[i] + j;
        const int off = (kg < p.Kg) ? (kg * p.K + b_col[i]) * ES : kOutOfRange;
        b_reg[set][i][j] = __builtin_amdgcn_raw_buffer_load_b128(filt_rsrc, off, 0, 0);
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
  auto store_tiles = [&](auto set_c, int buf) {
    constexpr int set = decltype(set_c)::value;
    unsigned char* as = As + buf * BM * LD * ES;
    unsigned char* bs = Bs + buf * BN * LD * ES;
#pragma unroll
    for (int i = 0; i < T::A_ITERS; ++i)
      *reinterpret_cast<uintx4*>(as + ((a_row0 + i * T::A_ROWS_PER_PASS) * LD + a_kv * VEC) * ES) =
          a_reg[set][i];
#pragma unroll
    for (int i = 0; i < T::B_ITERS; ++i) {
      const int b = tid + i * NT;
      if (b < T::B_BLOCKS) {
        const int nbv = b % (BN / VEC);
        const int kb = b / (BN / VEC);
        // VEC x VEC transpose in registers: LDS keeps B as [n][k], k contiguous
        unsigned char* dst = bs + ((nbv * VEC) * LD + kb * VEC) * ES;
        if (T::BF16) {
#pragma unroll
          for (int n = 0; n < 8; ++n) {
            const unsigned sel = (n & 1) ? 0x07060302u : 0x05040100u;  // high / low halves
            uintx4 v;
#pragma unroll
            for (int j = 0; j < 4; ++j)
              v[j] = __builtin_amdgcn_perm(b_reg[set][i][2 * j + 1][n >> 1],
                                           b_reg[set][i][2 * j][n >> 1], sel);
            *reinterpret_cast<uintx4*>(dst + n * LD * ES) = v;
          }
        } else {
#pragma unroll
          for (int n = 0; n < 4; ++n)
            *reinterpret_cast<uintx4*>(dst + n * LD * ES) =
                uintx4{b_reg[set][i][0][n], b_reg[set][i][1][n], b_reg[set][i][2][n],
                       b_reg[set][i][3][n]};
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
#pragma unroll
    for (int kk = 0; kk < BK / T::KSTEP; ++kk) {
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

  using Set0 = std::integral_constant<int, 0>;
  using Set1 = std::integral_constant<int, PF - 1>;  // the same set as Set0 when PF == 1

  // Slices past the end are loaded as zeros (their offsets are out of range)
  // and multiplied by nobody, so the pipeline needs no tail special cases.
  const int nslices = (p.Kg + BK - 1) / BK;
  issue_loads(Set0{});
  if (PF == 2) issue_loads(Set1{});
  store_tiles(Set0{}, 0);
  __syncthreads();

  for (int slice = 0; slice < nslices; slice += 2) {
    // even slice: its data is in LDS buffer 0 and register set 0 is free.
    // The scheduling fences keep the loads ahead of the MFMAs: if the
    // compiler sinks them, their destination registers get shared with the
    // LDS fragments and every LDS read then waits for all loads in flight.
    issue_loads(Set0{});
    __builtin_amdgcn_sched_barrier(0);
    multiply(0);
    __builtin_amdgcn_sched_barrier(0);
    store_tiles(Set1{}, 1);  // PF == 1: the set just loaded; PF == 2: the one loaded a slice ago
    __syncthreads();
    if (slice + 1 >= nslices) break;
    // odd slice: LDS buffer 1, register set 1 (PF == 2) is free
    issue_loads(Set1{});
    __builtin_amdgcn_sched_barrier(0);
    multiply(1);
    __builtin_amdgcn_sched_barrier(0);
    store_tiles(Set0{}, 0);
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

  // ---- epilogue: D tile -> NHWC output.  In a 32x32 accumulator, lane l
  // register v holds row 8*(v/4) + 4*(l/32) + v%4, column l%32, so each
  // store instruction writes two contiguous 32-element row segments.
#pragma unroll
  for (int i = 0; i < T::TM; ++i) {
#pragma unroll
    for (int j = 0; j < T::TN; ++j) {
      const int col = n0 + wn * T::WN + j * 32 + lr;
      const int rbase = m0 + wm * T::WM + i * 32 + lk * 4;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = rbase + 8 * (v / 4) + (v % 4);
        if (row < p.M && col < p.K) {
          const size_t idx = static_cast<size_t>(row) * p.K + col;
          if (OUT_BF16)
            static_cast<unsigned short*>(p.out)[idx] = to_bf16_bits(acc[i][j][v]);
          else
            static_cast<float*>(p.out)[idx] = acc[i][j][v];
        }
      }
    }
  }
}

template <class T, bool OUT_BF16>
hipError_t launch_one(const Problem& p, hipStream_t stream) {
  const int tiles_m = (p.M + T::BM - 1) / T::BM;
  const int tiles_n = (p.K + T::BN - 1) / T::BN;
  const size_t lds_bytes = T::LDS_BYTES;
  if (lds_bytes > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&igemm_kernel<T, OUT_BF16>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       static_cast<int>(lds_bytes));
    if (e != hipSuccess) return e;
  }
  // flush interval of the two-level summation: about sqrt(#slices)
  const int nslices = (p.Kg + T::BK - 1) / T::BK;
  int flush = 1;
  while (flush * flush < nslices) ++flush;
  hipLaunchKernelGGL((igemm_kernel<T, OUT_BF16>), dim3(tiles_m * tiles_n), dim3(T::NT), lds_bytes,
                     stream, p, flush);
  return hipGetLastError();
}

template <class T>
hipError_t launch(const Problem& p, hipStream_t stream) {
  if (T::BF16 && p.out_bf16) return launch_one<T, T::BF16>(p, stream);
  return launch_one<T, false>(p, stream);
}

struct TileEntry {
  const char* name;
  int bm, bn, bk;
  hipError_t (*fn)(const Problem&, hipStream_t);
};

#define CONV2D_TILE(dt, isbf, bm, bn, bk, wm, wn, two, occ, pf, tag) \
  { "igemm_" dt "_" #bm "x" #bn "x" #bk tag, bm, bn, bk, \
    &launch<Tile<isbf, bm, bn, bk, wm, wn, two, occ, pf>> }

const TileEntry kTilesF32[] = {
    CONV2D_TILE("f32", false, 256, 128, 16, 4, 2, true, 2, 1, ""),
    CONV2D_TILE("f32", false, 128, 128, 16, 2, 2, true, 2, 1, ""),
    CONV2D_TILE("f32", false, 256, 64, 16, 4, 1, true, 2, 1, ""),
    CONV2D_TILE("f32", false, 128, 64, 16, 2, 2, true, 3, 1, ""),
    CONV2D_TILE("f32", false, 64, 64, 16, 2, 2, true, 4, 1, ""),
    CONV2D_TILE("f32", false, 128, 32, 16, 4, 1, true, 4, 1, ""),
    CONV2D_TILE("f32", false, 128, 128, 32, 2, 2, true, 2, 1, ""),
    CONV2D_TILE("f32", false, 128, 64, 32, 2, 2, true, 3, 1, ""),
    CONV2D_TILE("f32", false, 256, 128, 32, 4, 2, true, 2, 1, ""),
};
const TileEntry kTilesBf16[] = {
    CONV2D_TILE("bf16", true, 128, 128, 64, 2, 2, false, 2, 1, ""),
    CONV2D_TILE("bf16", true, 128, 128, 32, 2, 2, false, 2, 1, ""),
    CONV2D_TILE("bf16", true, 128, 64, 64, 2, 2, false, 3, 1, ""),
    CONV2D_TILE("bf16", true, 128, 64, 32, 2, 2, false, 3, 1, ""),
    CONV2D_TILE("bf16", true, 64, 64, 32, 2, 2, false, 4, 1, ""),
};
constexpr int kNumF32 = sizeof(kTilesF32) / sizeof(kTilesF32[0]);
constexpr int kNumBf16 = sizeof(kTilesBf16) / sizeof(kTilesBf16[0]);

}  // namespace

int igemm_f32_num_tiles() { return kNumF32; }
const char* igemm_f32_tile_name(int tile) { return kTilesF32[tile].name; }
void igemm_f32_tile_shape(int tile, int* bm, int* bn, int* bk) {
  *bm = kTilesF32[tile].bm;
  *bn = kTilesF32[tile].bn;
  *bk = kTilesF32[tile].bk;
}
hipError_t launch_igemm_f32(const Problem& p, int tile, hipStream_t stream) {
  return kTilesF32[tile].fn(p, stream);
}

int igemm_bf16_num_tiles() { return kNumBf16; }
const char* igemm_bf16_tile_name(int tile) { return kTilesBf16[tile].name; }
void igemm_bf16_tile_shape(int tile, int* bm, int* bn, int* bk) {
  *bm = kTilesBf16[tile].bm;
  *bn = kTilesBf16[tile].bn;
  *bk = kTilesBf16[tile].bk;
}
hipError_t launch_igemm_bf16(const Problem& p, int tile, hipStream_t stream) {
  return kTilesBf16[tile].fn(p, stream);
}

}  // namespace conv2d
