// Implicit-GEMM forward convolution with a multi-stage LDS ring fed by direct
// global->LDS loads (buffer_load ... lds, 16 bytes per lane), for gfx950.
// Same GEMM view as igemm.hip (paper section 3: the convolution as the
// routine to accelerate; D[M][K] = A[M][Kg] * B[Kg][K], Kg ordered (r,s,c)):
// A rows are gathered from the NHWC input, D is the NHWC output.
//
// Differences from the register-staged kernel:
//  * The filter is first repacked into the workspace as Bt[K][Kg_p] (k
//    contiguous, Kg_p = Kg rounded up to the slice width, zero filled), so
//    that A and B tiles are both "rows of ROWB contiguous bytes" and both can
//    be written to LDS by the load instruction itself: no staging registers,
//    no transposes, and as many slices in flight as LDS has room for.
//  * A slice is ROWB = 64 or 128 bytes of k per row.  One load instruction
//    of a wavefront fills 1 KiB of LDS: lane l -> row l / CPR, 16-byte chunk
//    position l % CPR (CPR = ROWB/16 chunks per row).  LDS cannot be padded
//    under this scheme, so bank conflicts are avoided by an XOR swizzle: the
//    chunk stored at position p of row r is chunk p ^ ((r >> 1) & (CPR-1)).
//    The lane simply fetches that chunk from memory; the MFMA fragment reads
//    apply the same XOR (measured: full LDS read rate, 100 B/clk/CU).
//  * Padding taps / rows past M / k past Kg use an out-of-range buffer
//    offset: the hardware then writes zeros to LDS.
//  * STAGES (>= 3) LDS buffers form a ring and the whole thing is software
//    pipelined.  The MFMA fragments are double buffered in registers: while
//    the MFMAs of step t run, the fragments of step t+1 are read from LDS.
//    In the last step of slice i each wave waits for its own loads of slice
//    i+1 (s_waitcnt vmcnt(N), younger slices stay in flight), passes the one
//    barrier of the slice, issues the loads of slice i+STAGES-1 into the
//    stage of slice i-1 (which every wave has left), and reads the first
//    fragments of slice i+1: the MFMA stream never drains at a slice border.
//  * The loads are issued from inline assembly, so the compiler's automatic
//    wait insertion does not see them (it would make LDS reads of one stage
//    wait for loads into the others); ordering is explicit as described.
#include <type_traits>

#include "conv2d_internal.h"

namespace conv2d {
namespace dma {  // named namespace: the kernels' host stubs need external linkage

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kXcds = 8;
constexpr unsigned kRsrcFlags = 0x00020000u;
constexpr int kOutOfRange = static_cast<int>(0x80000000u);

// s_waitcnt immediate that waits for vmcnt <= n only (gfx9 encoding:
// vmcnt in bits 3:0 and 15:14, expcnt 6:4 and lgkmcnt 11:8 left at "no wait").
constexpr int vmcnt_imm(int n) { return (n & 0xf) | ((n >> 4) << 14) | (0x7 << 4) | (0xf << 8); }

// Raw buffer descriptor (base, stride 0, bytes, flags) as four scalars.
__device__ __forceinline__ uintx4 make_rsrc(const void* base, int bytes) {
  const size_t a = reinterpret_cast<size_t>(base);
  uintx4 r;
  r[0] = static_cast<unsigned>(a);
  r[1] = static_cast<unsigned>(a >> 32) & 0xffffu;
  r[2] = static_cast<unsigned>(bytes);
  r[3] = kRsrcFlags;
  return r;
}

// LDS byte address of a pointer into a __shared__ array (the low half of its flat address).
__device__ __forceinline__ unsigned lds_address(const void* p) {
  return static_cast<unsigned>(reinterpret_cast<size_t>(p));
}

// One wavefront-wide 16-byte-per-lane load from a buffer straight into LDS:
// lane l's 16 bytes land at lds_base + 16*l (lds_base is wave-uniform and goes
// through M0); an out-of-range voffset writes zeros.
__device__ __forceinline__ void dma16(const uintx4& rsrc, unsigned lds_base, int voffset,
                                      int soffset) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :
               : "s"(lds_base), "v"(voffset), "s"(rsrc), "s"(soffset)
               : "memory", "m0");
}

template <bool BF16_, int BM_, int BN_, int ROWB_, int WAVES_M_, int WAVES_N_, int STAGES_,
          bool TWO_LEVEL_, int OCC_>
struct DmaTile {
  static constexpr bool BF16 = BF16_;
  static constexpr int BM = BM_, BN = BN_;
  static constexpr int ROWB = ROWB_;             // bytes of k per LDS row = one slice
  static constexpr int CPR = ROWB / 16;          // 16-byte chunks per row
  static constexpr int ES = BF16 ? 2 : 4;
  static constexpr int VEC = 16 / ES;
  static constexpr int BK = ROWB / ES;
  static constexpr int KSTEPS = CPR / 2;         // a fragment step eats two chunks (two lane halves)
  static constexpr int STAGES = STAGES_;
  static constexpr bool TWO_LEVEL = TWO_LEVEL_;  // see igemm.hip: two-level fp32 summation
  static constexpr int OCC = OCC_;
  static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
  static constexpr int NW = WAVES_M * WAVES_N;
  static constexpr int NT = 64 * NW;
  static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  static constexpr int TM = WM / 32, TN = WN / 32;
  static constexpr int ROWS_PER_INSTR = 64 / CPR;
  static constexpr int ROWS_PER_PASS = NT / CPR;
  static constexpr int A_ITERS = BM / ROWS_PER_PASS;
  static constexpr int B_ITERS = BN / ROWS_PER_PASS;
  static constexpr int LOADS = A_ITERS + B_ITERS;  // load instructions per slice per lane
  static constexpr int STAGE_BYTES = (BM + BN) * ROWB;
  static constexpr int WAIT_STEADY = (STAGES - 3) * LOADS;  // loads that may stay in flight
  static constexpr int WAIT_FIRST = (STAGES - 2) * LOADS;
  static_assert(ROWB == 64 || ROWB == 128, "64 or 128 bytes per row");
  static_assert(KSTEPS % 2 == 0, "fragment double buffering needs an even step count");
  static_assert(STAGES >= 3 && STAGES <= 5, "3 to 5 stages");
  static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile must be a multiple of 32x32");
  static_assert(BM % ROWS_PER_PASS == 0 && BN % ROWS_PER_PASS == 0, "tile rows must divide");
  static_assert(ROWS_PER_PASS % 16 == 0, "the swizzle must be the same for all rows of a lane");
  static_assert(WAIT_FIRST <= 63, "vmcnt has 6 bits");
  static_assert(STAGES * STAGE_BYTES <= 160 * 1024, "stages do not fit LDS");
  static_assert(!(BF16 && TWO_LEVEL), "two-level summation is an fp32 feature");
};

__device__ __forceinline__ unsigned short to_bf16_bits(float x) {
  unsigned int u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<unsigned short>((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<unsigned short>(u >> 16);
}

// Bt[n][k] = filt[k][n] for k < Kg, 0 for Kg <= k < Kg_p.  32x32 tiles through LDS.
template <typename E>
__global__ __launch_bounds__(256) void repack_filter_kernel(const E* __restrict__ filt,
                                                            E* __restrict__ bt, int Kg, int K,
                                                            int Kg_p) {
  __shared__ E tile[32][33];
  const int k0 = blockIdx.x * 32, n0 = blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int k = k0 + ty + 8 * j, n = n0 + tx;
    tile[ty + 8 * j][tx] = (k < Kg && n < K) ? filt[static_cast<size_t>(k) * K + n] : E(0);
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int n = n0 + ty + 8 * j, k = k0 + tx;
    if (n < K && k < Kg_p) bt[static_cast<size_t>(n) * Kg_p + k] = tile[tx][ty + 8 * j];
  }
}

template <class T, bool OUT_BF16>
__global__ __launch_bounds__(T::NT, T::OCC) void igemm_dma_kernel(const Problem p, const int Kg_p,
                                                                  const int flush_slices) {
  constexpr int BM = T::BM, BN = T::BN, BK = T::BK, S = T::STAGES, ROWB = T::ROWB, CPR = T::CPR;
  constexpr int ES = T::ES, VEC = T::VEC, KSTEPS = T::KSTEPS;
  // one array per stage: [BM rows of A | BN rows of B], ROWB bytes per row
  __shared__ __align__(1024) unsigned char stage0[T::STAGE_BYTES];
  __shared__ __align__(1024) unsigned char stage1[T::STAGE_BYTES];
  __shared__ __align__(1024) unsigned char stage2[T::STAGE_BYTES];
  __shared__ __align__(1024) unsigned char stage3[S > 3 ? T::STAGE_BYTES : 16];
  __shared__ __align__(1024) unsigned char stage4[S > 4 ? T::STAGE_BYTES : 16];
  unsigned char* const stages[5] = {stage0, stage1, stage2, stage3, stage4};

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave / T::WAVES_N;
  const int wn = wave % T::WAVES_N;
  const int lr = lane & 31;
  const int lk = lane >> 5;

  const int tiles_n = (p.K + BN - 1) / BN;
  const int nwg = gridDim.x;
  const int xcd = blockIdx.x % kXcds;
  const int local = blockIdx.x / kXcds;
  const int per = nwg / kXcds, rem = nwg % kXcds;
  const int tile = xcd * per + (xcd < rem ? xcd : rem) + local;
  const int m0 = (tile / tiles_n) * BM;
  const int n0 = (tile % tiles_n) * BN;

  const uintx4 in_rsrc = make_rsrc(p.in, p.N * p.H * p.W * p.C * ES);
  const uintx4 bt_rsrc = make_rsrc(p.workspace, p.K * Kg_p * ES);

  // ---- loader role of this lane: row tid / CPR (+ passes of ROWS_PER_PASS),
  // LDS chunk position tid % CPR, memory chunk = position ^ swizzle(row);
  // passes step by a multiple of 16 rows, so the swizzle is the same in all
  const int ld_row0 = tid / CPR;
  const int ld_pos = tid % CPR;
  const int ld_chunk = ld_pos ^ ((ld_row0 >> 1) & (CPR - 1));
  int a_off[T::A_ITERS], a_h0[T::A_ITERS], a_w0[T::A_ITERS];
#pragma unroll
  for (int i = 0; i < T::A_ITERS; ++i) {
    const int m = m0 + ld_row0 + i * T::ROWS_PER_PASS;
    if (m < p.M) {
      const int q = m % p.Q;
      const int t = m / p.Q;
      const int op = t % p.P;
      const int n = t / p.P;
      a_h0[i] = op * p.sr - p.pt;
      a_w0[i] = q * p.sc - p.pl;
      a_off[i] = ((n * p.H + a_h0[i]) * p.W + a_w0[i]) * p.C;
    } else {
      a_h0[i] = -(1 << 28);
      a_w0[i] = 0;
      a_off[i] = 0;
    }
  }
  int b_voff[T::B_ITERS];
#pragma unroll
  for (int i = 0; i < T::B_ITERS; ++i) {
    const int n = n0 + ld_row0 + i * T::ROWS_PER_PASS;
    b_voff[i] = (n < p.K) ? (n * Kg_p + ld_chunk * VEC) * ES : kOutOfRange;
  }
  // (r, s, c) of this lane's chunk in the next slice to load; branch-free stepping
  int kc, ks, kr;
  {
    const int kg = ld_chunk * VEC;
    kc = kg % p.C;
    const int t = kg / p.C;
    ks = t % p.S;
    kr = t / p.S;
  }
  const int step_c = BK % p.C;
  const int step_s = (BK / p.C) % p.S;
  const int step_r = (BK / p.C) / p.S;
  int k_next_bytes = 0;
  const int k_last_bytes = (Kg_p - BK) * ES;

  auto issue_slice = [&](unsigned char* stage) {
    const int tap = (kr * p.W + ks) * p.C + kc;
    const int kr_t = (kr < p.R) ? kr : (1 << 30);
    const unsigned dst = __builtin_amdgcn_readfirstlane(lds_address(stage) + wave * 1024);
#pragma unroll
    for (int i = 0; i < T::A_ITERS; ++i) {
      const bool ok = (static_cast<unsigned>(a_h0[i] + kr_t) < static_cast<unsigned>(p.H)) &
                      (static_cast<unsigned>(a_w0[i] + ks) < static_cast<unsigned>(p.W));
      const int off = ok ? (a_off[i] + tap) * ES : kOutOfRange;
      dma16(in_rsrc, dst + i * T::ROWS_PER_PASS * ROWB, off, 0);
    }
    const unsigned dstb = dst + BM * ROWB;
#pragma unroll
    for (int i = 0; i < T::B_ITERS; ++i)
      dma16(bt_rsrc, dstb + i * T::ROWS_PER_PASS * ROWB, b_voff[i], k_next_bytes);
    // the scalar offset is not range checked: slices issued past the end
    // re-read the last slice (into a stage nobody reads) instead of running
    // off the end of the repacked filter
    k_next_bytes = min(k_next_bytes + ROWB, k_last_bytes);
    kc += step_c;
    const int carry_c = kc >= p.C;
    kc -= carry_c ? p.C : 0;
    ks += step_s + carry_c;
    const int carry_s = ks >= p.S;
    ks -= carry_s ? p.S : 0;
    kr += step_r + carry_s;
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

  // fragment addressing: row lr of each 32-row block, chunk (2*kk + lk) ^ swizzle
  const int frag_swz = (lr >> 1) & (CPR - 1);
  const int a_row_bytes = (wm * T::WM + lr) * ROWB;
  const int b_row_bytes = (BM + wn * T::WN + lr) * ROWB;
  int chunk_bytes[KSTEPS];
#pragma unroll
  for (int kk = 0; kk < KSTEPS; ++kk) chunk_bytes[kk] = ((2 * kk + lk) ^ frag_swz) * 16;

  uintx4 af[2][T::TM], bf[2][T::TN];  // double-buffered MFMA fragments

  auto read_frags = [&](auto buf_c, const unsigned char* stage, int kk) {
    constexpr int buf = decltype(buf_c)::value;
#pragma unroll
    for (int i = 0; i < T::TM; ++i)
      af[buf][i] =
          *reinterpret_cast<const uintx4*>(stage + a_row_bytes + i * 32 * ROWB + chunk_bytes[kk]);
#pragma unroll
    for (int j = 0; j < T::TN; ++j)
      bf[buf][j] =
          *reinterpret_cast<const uintx4*>(stage + b_row_bytes + j * 32 * ROWB + chunk_bytes[kk]);
  };
  auto mfmas = [&](auto buf_c) {
    constexpr int buf = decltype(buf_c)::value;
#pragma unroll
    for (int i = 0; i < T::TM; ++i)
#pragma unroll
      for (int j = 0; j < T::TN; ++j) {
        if (T::BF16) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              __builtin_bit_cast(bf16x8, af[buf][i]), __builtin_bit_cast(bf16x8, bf[buf][j]),
              acc[i][j], 0, 0, 0);
        } else {
#pragma unroll
          for (int t = 0; t < 4; ++t)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(af[buf][i][t]),
                                                             __uint_as_float(bf[buf][j][t]),
                                                             acc[i][j], 0, 0, 0);
        }
      }
  };
  using Buf0 = std::integral_constant<int, 0>;
  using Buf1 = std::integral_constant<int, 1>;

  const int nslices = Kg_p / BK;
  // prologue: slices 0 .. S-2 in flight, slice 0 landed, its first fragments read
#pragma unroll
  for (int s = 0; s < S - 1; ++s) issue_slice(stages[s]);
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(T::WAIT_FIRST));
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  read_frags(Buf0{}, stages[0], 0);

  for (int slice = 0; slice < nslices; slice += S) {
#pragma unroll
    for (int u = 0; u < S; ++u) {
      if (slice + u < nslices) {
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
          // 1. fragments of the next step into the other register buffer
          if (kk == KSTEPS - 1) {
            // next step belongs to the next slice: its loads must have landed
            // (this lane's: vmcnt; everyone's: barrier), and the barrier also
            // says that every wave has left the previous slice's stage
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(T::WAIT_STEADY));
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");  // LDS changed behind the compiler's back
            issue_slice(stages[(u + S - 1) % S]);
            read_frags(Buf0{}, stages[(u + 1) % S], 0);  // KSTEPS is even: next step uses buffer 0
          } else if (kk % 2 == 0) {
            read_frags(Buf1{}, stages[u], kk + 1);
          } else {
            read_frags(Buf0{}, stages[u], kk + 1);
          }
          __builtin_amdgcn_sched_barrier(0);
          // 2. MFMAs of this step
          if (kk % 2 == 0) mfmas(Buf0{}); else mfmas(Buf1{});
          __builtin_amdgcn_sched_barrier(0);
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
      }
    }
  }
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // drain the slices issued past the end
  if (T::TWO_LEVEL) {
#pragma unroll
    for (int i = 0; i < T::TM; ++i)
#pragma unroll
      for (int j = 0; j < T::TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] += total[i][j][v];
  }

  // ---- epilogue (accumulator layout: lane l reg v -> row 8*(v/4) + 4*(l/32) + v%4, col l%32)
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
  const int Kg_p = (p.Kg + T::BK - 1) / T::BK * T::BK;
  // 1. filter -> Bt[K][Kg_p] in the workspace
  dim3 rgrid((Kg_p + 31) / 32, (p.K + 31) / 32);
  if (T::BF16)
    hipLaunchKernelGGL((repack_filter_kernel<unsigned short>), rgrid, dim3(256), 0, stream,
                       static_cast<const unsigned short*>(p.filt),
                       static_cast<unsigned short*>(p.workspace), p.Kg, p.K, Kg_p);
  else
    hipLaunchKernelGGL((repack_filter_kernel<float>), rgrid, dim3(256), 0, stream,
                       static_cast<const float*>(p.filt), static_cast<float*>(p.workspace), p.Kg,
                       p.K, Kg_p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  // 2. the convolution
  const int tiles_m = (p.M + T::BM - 1) / T::BM;
  const int tiles_n = (p.K + T::BN - 1) / T::BN;
  const int nslices = Kg_p / T::BK;
  int flush = 1;
  while (flush * flush < nslices) ++flush;
  hipLaunchKernelGGL((igemm_dma_kernel<T, OUT_BF16>), dim3(tiles_m * tiles_n), dim3(T::NT), 0,
                     stream, p, Kg_p, flush);
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

#define CONV2D_DMA_TILE(dt, isbf, bm, bn, rowb, wm, wn, st, two, occ)                     \
  { "igemm_dma_" dt "_" #bm "x" #bn "_r" #rowb "_w" #wm "x" #wn "_s" #st, bm, bn,          \
    DmaTile<isbf, bm, bn, rowb, wm, wn, st, two, occ>::BK,                                 \
    &launch<DmaTile<isbf, bm, bn, rowb, wm, wn, st, two, occ>> }

const TileEntry kTilesF32[] = {
    CONV2D_DMA_TILE("f32", false, 128, 128, 64, 2, 2, 4, true, 2),
    CONV2D_DMA_TILE("f32", false, 128, 64, 64, 2, 2, 4, true, 3),
    CONV2D_DMA_TILE("f32", false, 256, 128, 64, 4, 2, 4, true, 2),
    CONV2D_DMA_TILE("f32", false, 128, 128, 128, 2, 2, 3, true, 1),
};
const TileEntry kTilesBf16[] = {
    CONV2D_DMA_TILE("bf16", true, 256, 256, 64, 4, 2, 4, false, 2),
    CONV2D_DMA_TILE("bf16", true, 256, 128, 64, 4, 2, 4, false, 2),
    CONV2D_DMA_TILE("bf16", true, 128, 128, 64, 2, 2, 4, false, 2),
    CONV2D_DMA_TILE("bf16", true, 128, 64, 64, 2, 2, 4, false, 3),
    CONV2D_DMA_TILE("bf16", true, 256, 128, 128, 2, 2, 3, false, 1),
    CONV2D_DMA_TILE("bf16", true, 128, 128, 128, 2, 2, 4, false, 1),
};
constexpr int kNumF32 = sizeof(kTilesF32) / sizeof(kTilesF32[0]);
constexpr int kNumBf16 = sizeof(kTilesBf16) / sizeof(kTilesBf16[0]);

}  // namespace dma
using namespace dma;

int igemm_dma_num_tiles(int bf16) { return bf16 ? kNumBf16 : kNumF32; }
const char* igemm_dma_tile_name(int bf16, int tile) {
  return bf16 ? kTilesBf16[tile].name : kTilesF32[tile].name;
}
void igemm_dma_tile_shape(int bf16, int tile, int* bm, int* bn, int* bk) {
  const TileEntry& t = bf16 ? kTilesBf16[tile] : kTilesF32[tile];
  *bm = t.bm;
  *bn = t.bn;
  *bk = t.bk;
}
size_t igemm_dma_workspace_bytes(const Problem& p, int bf16, int tile) {
  const TileEntry& t = bf16 ? kTilesBf16[tile] : kTilesF32[tile];
  const size_t kg_p = static_cast<size_t>((p.Kg + t.bk - 1) / t.bk) * t.bk;
  return kg_p * p.K * (bf16 ? 2 : 4);
}
hipError_t launch_igemm_dma(const Problem& p, int bf16, int tile, hipStream_t stream) {
  return (bf16 ? kTilesBf16[tile] : kTilesF32[tile]).fn(p, stream);
}

}  // namespace conv2d
