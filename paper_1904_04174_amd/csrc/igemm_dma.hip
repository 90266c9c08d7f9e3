// Implicit-GEMM forward convolution with a multi-stage LDS ring fed by direct
// global->LDS loads (buffer_load ... lds, 16 bytes per lane) and a hand-placed
// instruction schedule, for gfx950.  Same GEMM view as igemm.hip (paper
// section 3: the convolution as the routine to accelerate;
// D[M][K] = A[M][Kg] * B[Kg][K], Kg ordered (r,s,c)): A rows are gathered from
// the NHWC input, D is the NHWC output.
//
//  * The filter is first repacked into the workspace as Bt[slice][K][BK]
//    (k contiguous within a slice of BK, Kg rounded up to whole slices, zero
//    filled), so that A and B tiles are both "rows of ROWB contiguous bytes"
//    and both can be written to LDS by the load instruction itself: no
//    staging registers, no transposes, and as many slices in flight as LDS
//    has room for.  A slice's B tile is one contiguous block of memory.
//  * A slice is ROWB = 64 or 128 bytes of k per row.  One load instruction
//    of a wavefront fills 1 KiB of LDS: lane l -> row l / CPR, 16-byte chunk
//    position l % CPR (CPR = ROWB/16 chunks per row).  LDS cannot be padded
//    under this scheme, so bank conflicts are avoided by an XOR swizzle: the
//    chunk stored at position p of row r is chunk p ^ ((r >> SWZ_SHIFT) & (CPR-1)).
//    The lane simply fetches that chunk from memory; the MFMA fragment reads
//    apply the same XOR (measured: full LDS read rate).
//  * Padding taps / rows past M / k past Kg use an out-of-range buffer
//    offset: the hardware then writes zeros to LDS.
//  * STAGES (>= 2) LDS buffers form a ring.  The MFMA fragments are double
//    buffered in registers: while the MFMAs of step t run, the fragments of
//    step t+1 are read from LDS, so during the last step of slice i nothing
//    of its stage is needed any more.  In that step each wave waits for its
//    own loads of slice i+1 (s_waitcnt vmcnt(N), younger slices stay in
//    flight) and for its own LDS reads, passes the one barrier of the slice,
//    issues the loads of slice i+STAGES into the stage of slice i (which
//    every wave has now read completely), and reads the first fragments of
//    slice i+1: loads run STAGES-1 slices ahead of the MFMAs.
//  * Everything that is not an MFMA (fragment reads, address arithmetic, load
//    issue, the barrier) is dealt out one piece at a time between consecutive
//    MFMAs and pinned there with scheduling fences: an MFMA occupies the
//    matrix core for 32 (bf16) or 64 (fp32) cycles during which the wave can
//    issue a handful of other instructions for free, whereas a block of them
//    between two blocks of MFMAs leaves the matrix core idle.
//  * UNIFORM tiles (C a multiple of the slice width, window of at most 31
//    taps) know that a slice lies inside one tap: the tap offset is a scalar
//    and each row keeps a bit mask of its valid taps, three vector
//    instructions per gathered row.  Other shapes step (r,s,c) per lane.
//  * The loads are issued from inline assembly, so the compiler's automatic
//    wait insertion does not see them (it would make LDS reads of one stage
//    wait for loads into the others); ordering is explicit as described.
//  * gridDim.y > 1 splits the reduction: each workgroup takes a range of
//    slices and writes an fp32 partial tile behind the repacked filter in the
//    workspace; a reduce pass adds the partials in a fixed order.
//  * Tail balancing ("stream-K tail"): output tiles rarely divide evenly over
//    the 256 compute units (every M here is 49 * 2^k).  The first n_main
//    tiles, a multiple of 256, run as whole tiles; the slices of the remaining
//    tiles are laid end to end and cut into equal contiguous ranges, one per
//    tail workgroup, so that every compute unit gets the same amount of work.
//    A range covers pieces of at most two tiles; each piece is one workgroup
//    that stores an fp32 partial tile, and tail_reduce_kernel adds the pieces
//    of a tile in slice order.
//  * Final outputs are stored non-temporally (store_out); partial tiles and
//    the batched launches' outputs, which another kernel reads next, are not.
//  * A filter packed ahead of time (Problem::packed_filt) is the repacked
//    Bt as a tensor of its own; the launch then skips the repack.
//
// The second half of the file is the LDS-resident patch kernel for 3x3,
// stride-1 layers (consecutive-pixel and blocked tiles, persistent launch of
// the blocked tiles, 16-row MFMA tiles, pooling epilogue); see there.
#include <atomic>
#include <mutex>
#include <type_traits>

#include "buffer_lds.h"
#include "conv2d_internal.h"
#include "split_in_launch.h"

namespace conv2d {
namespace dma {  // named namespace: the kernels' host stubs need external linkage

using namespace buf;

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kXcds = 8;
constexpr int kComputeUnits = 256;
// ADDR: how the gathered A rows are addressed.
//   kUniform  a slice lies inside one tap (C a multiple of the slice width, at
//             most 31 taps): scalar tap offset + per-row tap masks, 16-byte loads
//   kVector   any C that is a multiple of the 16-byte vector: (r,s,c) per lane
//   kElement  any C (fp32 only): 4-byte loads, (r,s,c) per lane and element
constexpr int kUniform = 0, kVector = 1, kElement = 2;

// NATIVE (bf16 uniform tiles): the filter slice is loaded as it lies in memory, BK rows (one
// per k) of BN consecutive features, and the B fragments are formed by transposing LDS reads
// (see the patch tiles below): no repacked filter, no launch before the convolution.
template <bool BF16_, int BM_, int BN_, int ROWB_, int WAVES_M_, int WAVES_N_, int STAGES_,
          bool TWO_LEVEL_, int OCC_, int ADDR_, bool NATIVE_ = false>
struct DmaTile {
  static constexpr bool NATIVE = NATIVE_;
  static_assert(!NATIVE_ || (ADDR_ == 0 && BN_ % 64 == 0), "native filter: uniform tiles");
  static constexpr int B_ROW_BYTES = BN_ * (BF16_ ? 2 : 4);   // NATIVE: a filter row (one k) in LDS
  // NATIVE, bf16: XOR of the 32-byte piece index of filter row k.  A 32-row block's read takes,
  // per half wavefront, 4 rows x 2 adjacent pieces: the XOR moves pairs of pieces (bit 0 clear).
  // NATIVE, fp32 (a lane reads single values, 32 consecutive features of row k per lane half,
  // the other half 4 rows on): XOR of the 128-byte half index, so that the two halves of a
  // wavefront read different banks.
  static constexpr int native_swizzle(int k) {
    if (!BF16_) return (k >> 2) & 1;
    return BN_ >= 128 ? ((k & 3) << 1) : (((k >> 1) & 1) << 1);
  }
  static constexpr bool BF16 = BF16_;
  static constexpr int BM = BM_, BN = BN_;
  static constexpr int ROWB = ROWB_;             // bytes of k per LDS row = one slice
  static constexpr int CPR = ROWB / 16;          // 16-byte chunks per row
  static constexpr int ES = BF16 ? 2 : 4;
  static constexpr int VEC = 16 / ES;
  static constexpr int BK = ROWB / ES;
  static constexpr int KSTEPS = CPR / 2;         // a fragment step eats two chunks (two lane halves)
  // XOR swizzle of the chunk position: (row >> SWZ_SHIFT) & (CPR - 1).  A fragment read of a
  // 32-row block must spread over all 64 banks: with 64-byte rows four rows share a quarter of
  // the banks, so rows r, r+4, r+8, r+12 need four different positions (shift 2; measured
  // 246 bytes per clock and compute unit against 127 with shift 1); 128-byte rows: shift 1.
  static constexpr int SWZ_SHIFT = CPR == 4 ? 2 : 1;
  static constexpr int STAGES = STAGES_;
  static constexpr bool TWO_LEVEL = TWO_LEVEL_;  // see igemm.hip: two-level fp32 summation
  static constexpr int OCC = OCC_;
  static constexpr int ADDR = ADDR_;
  static constexpr bool UNIFORM = ADDR_ == kUniform;  // a slice never straddles two taps
  static constexpr bool ELEMENT = ADDR_ == kElement;  // A gathered element by element
  static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
  static constexpr int NW = WAVES_M * WAVES_N;
  static constexpr int NT = 64 * NW;
  static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  static constexpr int TM = WM / 32, TN = WN / 32;
  static constexpr int MPF = BF16 ? 1 : 4;       // MFMAs per pair of 16-byte fragments
  static constexpr int NM = TM * TN * MPF;       // MFMAs per fragment step
  static constexpr int NR = TM + TN;             // fragment reads per step
  static constexpr int ROWS_PER_INSTR = 64 / CPR;
  static constexpr int ROWS_PER_PASS = NT / CPR;
  static constexpr int A_VEC = ELEMENT ? 1 : VEC;          // elements per A load
  static constexpr int A_LPR = (ROWB / ES) / A_VEC;        // A loads per row
  static constexpr int A_ROWS_PER_PASS = NT / A_LPR;
  static constexpr int A_ITERS = BM / A_ROWS_PER_PASS;
  static constexpr int B_ITERS = BN / ROWS_PER_PASS;
  static constexpr int LOADS = A_ITERS + B_ITERS;  // load instructions per slice per lane
  static constexpr int STAGE_BYTES = (BM + BN) * ROWB;
  static constexpr int WAIT_STEADY = (STAGES - 2) * LOADS;  // loads that may stay in flight
  // after the prologue: slices 1 .. S-2 and the first share of slice S-1
  static constexpr int WAIT_FIRST = (STAGES - 2) * LOADS + LOADS / KSTEPS;
  static_assert(ROWB == 64 || ROWB == 128, "64 or 128 bytes per row");
  static_assert(KSTEPS % 2 == 0, "fragment double buffering needs an even step count");
  static_assert(STAGES >= 2 && STAGES <= 8, "2 to 8 stages");
  static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile must be a multiple of 32x32");
  static_assert(BM % A_ROWS_PER_PASS == 0 && BN % ROWS_PER_PASS == 0, "tile rows must divide");
  static_assert(A_ROWS_PER_PASS % 16 == 0, "the swizzle must be the same for all rows of a lane");
  static_assert(!(ELEMENT && BF16), "element-wise gathers are fp32 only");
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

// Final outputs are stored non-temporally: nothing in the call reads them back, and as ordinary
// stores they take L2 lines from the input rows that neighbouring tiles are about to re-use
// (measured on a 224x224x64 bf16 layer, persistent patch tile: 189.5 MB fetched from beyond L2
// with ordinary stores, 103.6 MB with the stores switched off; the input is 102.8 MB).
template <class V>
__device__ __forceinline__ void store_out(V* ptr, V value) {
  __builtin_nontemporal_store(value, ptr);
}


// Bt[k' / bk][n][k' % bk] = filt[k][n], 0 for Kg <= k' < Kg_p: one slice of bk
// consecutive k' for all features is contiguous, so a B tile of a slice is
// one contiguous block and its loads fetch whole cache lines.  With
// block == 0, k' = k (the (r,s,c) order).  With block > 0 (a divisor of C)
// the reduction is reordered channel block by channel block:
// k' = ((c / block) * taps + tap) * block + c % block for k = tap * C + c.
// One workgroup transposes one slice x 64 features through LDS: 16-byte
// loads along the features, 16-byte stores along k (a contiguous 64*bk block).
template <typename E>
__global__ __launch_bounds__(256) void repack_filter_kernel(const E* __restrict__ filt,
                                                            E* __restrict__ bt, int Kg, int K,
                                                            int Kg_p, int C, int taps, int block,
                                                            int bk, long long filt_stride,
                                                            long long bt_stride) {
  constexpr int V = 16 / sizeof(E);          // elements per 16-byte vector
  filt += blockIdx.z * filt_stride;          // batched: one filter per blockIdx.z
  bt += blockIdx.z * bt_stride;
  __shared__ __align__(16) E tile[64][128 + V];  // [n][k of the slice], bk <= 128
  const int slice = blockIdx.x, n0 = blockIdx.y * 64;
  const bool vec_ok = (K % V == 0) && ((reinterpret_cast<size_t>(filt) & 15) == 0);
  // load: thread -> (k of the slice, vector of V features)
  for (int idx = threadIdx.x; idx < bk * (64 / V); idx += 256) {
    const int kk = idx / (64 / V), nv = (idx % (64 / V)) * V;
    const int kp = slice * bk + kk;
    int k = kp;
    if (block > 0 && kp < Kg) {
      const int per = taps * block;
      const int rem = kp % per;
      k = (rem / block) * C + (kp / per) * block + rem % block;
    }
    E v[V];
    const int n = n0 + nv;
    if (kp < Kg && vec_ok && n + V <= K) {
      *reinterpret_cast<uint4*>(v) =
          *reinterpret_cast<const uint4*>(filt + static_cast<size_t>(k) * K + n);
    } else {
#pragma unroll
      for (int j = 0; j < V; ++j)
        v[j] = (kp < Kg && n + j < K) ? filt[static_cast<size_t>(k) * K + n + j] : E(0);
    }
#pragma unroll
    for (int j = 0; j < V; ++j) tile[nv + j][kk] = v[j];
  }
  __syncthreads();
  // store: thread -> (feature, vector of V consecutive k)
  for (int idx = threadIdx.x; idx < 64 * (bk / V); idx += 256) {
    const int n = idx / (bk / V), kv = (idx % (bk / V)) * V;
    if (n0 + n < K)
      *reinterpret_cast<uint4*>(bt + (static_cast<size_t>(slice) * K + n0 + n) * bk + kv) =
          *reinterpret_cast<const uint4*>(&tile[n][kv]);
  }
}

// How the tail tiles' slices are dealt to the tail workgroups: `units` slices
// in all, workgroup g takes base (+1 for the first `extra` workgroups).
struct TailPlan {
  int n_main;   // tiles [0, n_main) are computed whole, one workgroup each
  int wgs;      // ranges the tail is cut into (0 = no tail); two workgroups per range
  int base, extra;
  // Order in which the workgroups of an XCD take the whole tiles of the XCD's range (a block of
  // pixel-tile rows x all feature tiles): feature tiles fastest (0), or pixel tiles fastest (1).
  // Workgroups that run at the same time then share input rows, or filter slabs; the second is
  // better where the filter is the larger stream (measured, fp32 64x64 tiles at batch 16, bytes
  // fetched from beyond L2: 28x28, 512 -> 512: 385 MB / 164 MB; 56x56, 256 -> 256: 80 MB / 231
  // MB; the kernel times do not differ, both layers are MFMA-bound).
  int pixel_tiles_first;
  __host__ __device__ long long first_unit(int g) const {
    return 1LL * g * base + (g < extra ? g : extra);
  }
  __host__ __device__ int owner(long long u) const {  // workgroup that holds unit u
    const long long head = 1LL * extra * (base + 1);
    return u < head ? static_cast<int>(u / (base + 1)) : extra + static_cast<int>((u - head) / base);
  }
};

// gridDim.x = tail.n_main + 2 * tail.wgs workgroups, gridDim.y = splits of the
// reduction (1 when there is a tail).  `bt` is the repacked filter, `partial`
// the fp32 partial outputs: [split][M][K] for a split reduction, or one
// [BM][BN] tile per tail workgroup.
// Signs of A^T (x) A^T for Winograd F(2x2, 3x3): contribution of point
// t = 4a + b to output pixel 2i + j of a tile is A^T[i][a] * A^T[j][b] with
// A^T = [[1, 1, 1, 0], [0, 1, -1, -1]].
__constant__ float kWinoFold[16][4] = {
    {1, 0, 0, 0},  {1, 1, 0, 0},   {1, -1, 0, 0},  {0, -1, 0, 0},
    {1, 0, 1, 0},  {1, 1, 1, 1},   {1, -1, 1, -1}, {0, -1, 0, -1},
    {1, 0, -1, 0}, {1, 1, -1, -1}, {1, -1, -1, 1}, {0, -1, 0, 1},
    {0, 0, -1, 0}, {0, 0, -1, -1}, {0, 0, -1, 1},  {0, 0, 0, 1}};

// WINO: the reduction is the 16 Winograd point products laid end to end
// (flush_slices slices each); each finished product is folded into the four
// output pixels of the tile's rows and the epilogue stores those.
template <class T, bool OUT_BF16, bool WINO = false>
__global__ __launch_bounds__(T::NT, T::OCC) void igemm_dma_kernel(const Problem p, const int Kg_p,
                                                                  const int slices_per_split,
                                                                  const int flush_slices,
                                                                  const void* bt,
                                                                  float* partial,
                                                                  const TailPlan tail,
                                                                  unsigned* split_counters,
                                                                  const int reduce_groups) {
  constexpr int BM = T::BM, BN = T::BN, BK = T::BK, S = T::STAGES, ROWB = T::ROWB, CPR = T::CPR;
  constexpr int ES = T::ES, VEC = T::VEC, KSTEPS = T::KSTEPS;
  constexpr int TM = T::TM, TN = T::TN, NM = T::NM, NR = T::NR, MPF = T::MPF;
  constexpr bool UNIFORM = T::UNIFORM, ELEMENT = T::ELEMENT;
  // stage s: [BM rows of A | BN rows of B], ROWB bytes per row
  __shared__ __align__(1024) unsigned char ring[S * T::STAGE_BYTES];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave / T::WAVES_N;
  const int wn = wave % T::WAVES_N;
  const int lr = lane & 31;
  const int lk = lane >> 5;

  const int tiles_n = (p.K + BN - 1) / BN;
  const int nslices_all = Kg_p / BK;
  const bool is_tail = static_cast<int>(blockIdx.x) >= tail.n_main;
  const unsigned ring_base = __builtin_amdgcn_readfirstlane(lds_address(ring) + wave * 1024);
  const unsigned ring_base_elt = __builtin_amdgcn_readfirstlane(lds_address(ring) + wave * 256);

  int tile, slice_begin, nslices;
  int piece = 0;  // tail: index of this workgroup's piece (two per range)
  if (!is_tail) {
    // Workgroup i runs on XCD i % 8; give each XCD a contiguous range of
    // tiles so that neighbours share input rows in its L2
    const int nwg = tail.n_main;
    const int xcd = blockIdx.x % kXcds;
    const int local = blockIdx.x / kXcds;
    const int per = nwg / kXcds, rem = nwg % kXcds;
    const int first = xcd * per + (xcd < rem ? xcd : rem), count = per + (xcd < rem ? 1 : 0);
    tile = first + local;
    if (tail.pixel_tiles_first && count % tiles_n == 0 && first % tiles_n == 0) {
      const int rows = count / tiles_n;
      tile = first + (local % rows) * tiles_n + local / rows;
    }
    slice_begin = blockIdx.y * slices_per_split;
    nslices = min(slices_per_split, nslices_all - slice_begin);
  } else {
    // tail workgroups 2g and 2g+1 take the two pieces of range g of the tail
    // tiles' slice units: the part in the range's first tile and the rest
    // (n_main is a multiple of 8, so tail workgroup j also runs on XCD j % 8;
    // as above each XCD takes a contiguous run of pieces)
    const int j = blockIdx.x - tail.n_main;
    const int nwg = 2 * tail.wgs;
    const int per = nwg / kXcds, rem = nwg % kXcds;
    const int xcd = j % kXcds;
    const int w = xcd * per + (xcd < rem ? xcd : rem) + j / kXcds;
    piece = w;
    const long long u0 = tail.first_unit(w >> 1), u1 = tail.first_unit((w >> 1) + 1);
    const int t0 = static_cast<int>(u0 / nslices_all);
    const long long cut = min(u1, 1LL * (t0 + 1) * nslices_all);
    const long long b = (w & 1) ? cut : u0, e = (w & 1) ? u1 : cut;
    if (b >= e) return;  // the range lies in one tile: no second piece
    tile = tail.n_main + t0 + (w & 1);
    slice_begin = static_cast<int>(b - 1LL * (t0 + (w & 1)) * nslices_all);
    nslices = static_cast<int>(e - b);
  }
  const int m0 = (tile / tiles_n) * BM;
  const int n0 = (tile % tiles_n) * BN;

  // UNIFORM tiles address a row by the (possibly negative) offset of its
  // window origin plus a scalar tap offset; the descriptor base is moved
  // back by `shift` bytes so that the vector part is never negative.
  const int shift = UNIFORM ? (p.pt * p.W + p.pl) * p.C * ES : 0;
  // batched launch: problem blockIdx.z of p.batches
  const size_t bz = blockIdx.z;
  const size_t bt_bytes = (static_cast<size_t>(Kg_p) * p.K * ES + 255) / 256 * 256;
  const uintx4 in_rsrc =
      make_rsrc(static_cast<const unsigned char*>(p.in) + bz * p.in_stride * ES, shift,
                p.N * p.H * p.W * p.C * ES + shift);
  const uintx4 bt_rsrc =
      make_rsrc(static_cast<const unsigned char*>(bt) + bz * bt_bytes, 0, p.K * Kg_p * ES);

  // ---- loader role of this lane: row tid / CPR (+ passes of ROWS_PER_PASS),
  // LDS chunk position tid % CPR, memory chunk = position ^ swizzle(row);
  // passes step by a multiple of 16 rows, so the swizzle is the same in all
  const int ld_row0 = tid / CPR;
  const int ld_pos = tid % CPR;
  const int ld_chunk = ld_pos ^ ((ld_row0 >> T::SWZ_SHIFT) & (CPR - 1));
  // A loads of ELEMENT tiles move one element per lane: row tid / A_LPR,
  // element position tid % A_LPR inside the LDS row, memory element =
  // (chunk position ^ swizzle) * VEC + element within the chunk
  const int a_row0 = ELEMENT ? tid / T::A_LPR : ld_row0;
  const int a_k0 = ELEMENT ? ((((tid % T::A_LPR) / VEC) ^ ((a_row0 >> T::SWZ_SHIFT) & (CPR - 1))) * VEC +
                              (tid % T::A_LPR) % VEC)
                           : ld_chunk * VEC;
  // UNIFORM: byte offset of the row's window origin (+ shift, + this lane's
  // chunk); otherwise the element offset of the window origin
  int a_off[T::A_ITERS];
  int a_h0[UNIFORM ? 1 : T::A_ITERS], a_w0[UNIFORM ? 1 : T::A_ITERS];
  unsigned a_mask[UNIFORM ? T::A_ITERS : 1];  // bit r*S+s: tap (r,s) of the row lies inside the image
#pragma unroll
  for (int i = 0; i < T::A_ITERS; ++i) {
    const int m = m0 + a_row0 + i * T::A_ROWS_PER_PASS;
    const bool row_ok = m < p.M;
    const int mm = row_ok ? m : 0;
    const int q = mm % p.Q;
    const int t = mm / p.Q;
    const int op = t % p.P;
    const int n = t / p.P;
    const int h0 = op * p.sr - p.pt;
    const int w0 = q * p.sc - p.pl;
    const int off = ((n * p.H + h0) * p.W + w0) * p.C;
    if constexpr (UNIFORM) {
      unsigned mask = 0;
      for (int r = 0; r < p.R; ++r)
        for (int s = 0; s < p.S; ++s)
          if (static_cast<unsigned>(h0 + r) < static_cast<unsigned>(p.H) &&
              static_cast<unsigned>(w0 + s) < static_cast<unsigned>(p.W))
            mask |= 1u << (r * p.S + s);
      a_mask[i] = row_ok ? mask : 0u;
      a_off[i] = (off + ld_chunk * VEC) * ES + shift;
    } else {
      a_h0[i] = row_ok ? h0 : -(1 << 28);
      a_w0[i] = w0;
      a_off[i] = off;
    }
  }
  int b_voff[T::B_ITERS];
#pragma unroll
  for (int i = 0; i < T::B_ITERS; ++i) {
    if constexpr (T::NATIVE) {
      // 16-byte chunk q of the stage's filter part: row k = q / chunks per row; its position
      // q % chunks per row holds the features [8c, 8c + 8) with c = position ^ swizzle
      constexpr int CH = BN / VEC;
      const int q = i * T::NT + tid;
      const int k = q / CH;
      // (bf16: pieces of 2 chunks; fp32: halves of 8 chunks)
      const int c = (q % CH) ^ (T::native_swizzle(k) << (T::BF16 ? 1 : 3));
      const int n = n0 + VEC * c;
      b_voff[i] = (n + VEC <= p.K) ? (k * p.K + n) * ES : kOutOfRange;
    } else {
      const int n = n0 + ld_row0 + i * T::ROWS_PER_PASS;
      b_voff[i] = (n < p.K) ? (n * BK + ld_chunk * VEC) * ES : kOutOfRange;
    }
  }
  // Position of the next slice to load.  UNIFORM: scalar tap index and channel
  // offset.  Otherwise (r, s, c) of this lane's chunk, stepped without division.
  int kc, ks, kr;
  int tap_bit = 0, tap_idx = 0, tap_c = 0, tap_s = 0, tap_rowoff = 0;  // UNIFORM
  {
    const int kg = slice_begin * BK + (UNIFORM ? 0 : a_k0);
    kc = kg % p.C;
    const int t = kg / p.C;
    ks = t % p.S;
    kr = t / p.S;
    if constexpr (UNIFORM) {
      // UNIFORM tiles walk the reduction channel block by channel block, all
      // taps of a block of BK channels before the next block: the taps of
      // one block re-read the same input pixels within a few slices, while
      // they are still in L2 (the filter is repacked in the same order)
      const int taps = p.R * p.S;
      const int tap = slice_begin % taps;
      tap_c = (slice_begin / taps) * BK;
      tap_s = tap % p.S;
      tap_rowoff = (tap / p.S) * p.W * p.C;
      tap_idx = tap;
      tap_bit = tap_c < p.C ? tap : 31;
    }
  }
  const int step_c = BK % p.C;
  const int step_s = (BK / p.C) % p.S;
  const int step_r = (BK / p.C) / p.S;
  // byte offset of a slice of the repacked filter: slices of K rows of ROWB bytes
  const int k_slice_bytes = p.K * ROWB;
  const int k_last_bytes = (nslices_all - 1) * k_slice_bytes;
  int k_next_bytes = min(slice_begin * k_slice_bytes, k_last_bytes);
  // NATIVE: slice (channel block, tap) starts at filter row tap * C + channel offset
  if constexpr (T::NATIVE)
    k_next_bytes = tap_c < p.C ? (tap_idx * p.C + tap_c) * p.K * ES : 0;

  // One A load (row pass i) of the slice at the current position into `stage`.
  auto load_a = [&](int stage, int i) {
    // a wave's load fills 1 KiB (16-byte loads) or 256 bytes (4-byte loads) of the stage
    const unsigned dst = (ELEMENT ? ring_base_elt : ring_base) + stage * T::STAGE_BYTES +
                         i * T::A_ROWS_PER_PASS * ROWB;
    if constexpr (UNIFORM) {
      const bool ok = (a_mask[i] >> tap_bit) & 1u;
      const int soff = (tap_rowoff + tap_s * p.C + tap_c) * ES;
      dma16(in_rsrc, dst, ok ? a_off[i] : kOutOfRange, soff);
    } else {
      const int tap = (kr * p.W + ks) * p.C + kc;
      const int kr_t = (kr < p.R) ? kr : (1 << 30);
      const bool ok = (static_cast<unsigned>(a_h0[i] + kr_t) < static_cast<unsigned>(p.H)) &
                      (static_cast<unsigned>(a_w0[i] + ks) < static_cast<unsigned>(p.W));
      if constexpr (T::ELEMENT)
        dma4(in_rsrc, dst, ok ? (a_off[i] + tap) * ES : kOutOfRange, 0);
      else
        dma16(in_rsrc, dst, ok ? (a_off[i] + tap) * ES : kOutOfRange, 0);
    }
  };
  auto load_b = [&](int stage, int i) {
    const unsigned dst = ring_base + stage * T::STAGE_BYTES + (BM + i * T::ROWS_PER_PASS) * ROWB;
    dma16(bt_rsrc, dst, b_voff[i],
          T::NATIVE ? __builtin_amdgcn_readfirstlane(k_next_bytes) : k_next_bytes);
  };
  // Moves the load position one slice on.
  auto advance = [&]() {
    // the scalar offset is not range checked: slices issued past the end
    // re-read the last slice (into a stage nobody reads) instead of running
    // off the end of the repacked filter
    k_next_bytes = min(k_next_bytes + k_slice_bytes, k_last_bytes);
    if constexpr (UNIFORM) {
      ++tap_idx;
      if (++tap_s >= p.S) {
        tap_s = 0;
        tap_rowoff += p.W * p.C;
      }
      if (tap_idx >= p.R * p.S) {
        tap_idx = 0;
        tap_rowoff = 0;
        tap_c += BK;
      }
      // windows have at most 31 taps here, so bit 31 is clear in every mask:
      // past the last channel block every row reads as out of range
      tap_bit = tap_c < p.C ? tap_idx : 31;
      // (past the end: the first slice again, into a stage nobody reads)
      if constexpr (T::NATIVE)
        k_next_bytes = tap_c < p.C ? (tap_idx * p.C + tap_c) * p.K * ES : 0;
    } else {
      kc += step_c;
      const int carry_c = kc >= p.C;
      kc -= carry_c ? p.C : 0;
      ks += step_s + carry_c;
      const int carry_s = ks >= p.S;
      ks -= carry_s ? p.S : 0;
      kr += step_r + carry_s;
    }
  };

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  constexpr bool TWO_LEVEL = T::TWO_LEVEL && !WINO;
  floatx16 total[TWO_LEVEL ? TM : 1][TWO_LEVEL ? TN : 1];
  if (TWO_LEVEL) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) total[i][j][v] = 0.f;
  }
  floatx16 pixel[WINO ? 4 : 1][WINO ? TM : 1][WINO ? TN : 1];  // WINO: the 2x2 outputs of a tile row
  if (WINO) {
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v) pixel[q][i][j][v] = 0.f;
  }
  int wino_point = 0;
  int until_flush = flush_slices;

  // fragment addressing: row lr of each 32-row block, chunk (2*kk + lk) ^ swizzle
  const int frag_swz = (lr >> T::SWZ_SHIFT) & (CPR - 1);
  const unsigned char* a_frag = ring + (wm * T::WM + lr) * ROWB;
  const unsigned char* b_frag = ring + (BM + wn * T::WN + lr) * ROWB;
  int chunk_bytes[KSTEPS];
#pragma unroll
  for (int kk = 0; kk < KSTEPS; ++kk) chunk_bytes[kk] = ((2 * kk + lk) ^ frag_swz) * 16;

  uintx4 af[2][TM], bf[2][TN];  // double-buffered MFMA fragments
  // NATIVE: lane (feature lane % 16 of half block (lane / 16) % 2, k group lk) hands in the
  // address of row 16 * kk + 8 * lk + (lane % 16) / 4 (+ 4 for the second read), features
  // 4 * (lane % 4) ... of its 16-feature piece
  int nat_row_off = 0, nat_piece_off[T::NATIVE ? TN : 1] = {};
  if constexpr (T::NATIVE && T::BF16) {
    const int a = lane & 15, k = 8 * lk + a / 4;
    nat_row_off = BM * ROWB + k * T::B_ROW_BYTES + 8 * (a % 4);
#pragma unroll
    for (int j = 0; j < TN; ++j)
      nat_piece_off[j] = 32 * ((2 * (wn * TN + j) + ((lane >> 4) & 1)) ^ T::native_swizzle(k));
  }
  // NATIVE, fp32: lane (feature lr of a block, half lk) reads rows 8 * kk + 4 * lk + t, t = 0..3
  // (the four MFMAs of a step), feature lr of the block's 128-byte half
  if constexpr (T::NATIVE && !T::BF16) {
    nat_row_off = BM * ROWB + 4 * lk * T::B_ROW_BYTES + 4 * lr;
#pragma unroll
    for (int j = 0; j < TN; ++j) nat_piece_off[j] = 128 * ((wn * TN + j) ^ lk);
  }

  // Fragment read number r (A blocks first, then B blocks) of step kk of `stage`.
  auto read_frag = [&](auto buf_c, int stage, int kk, int r) {
    constexpr int buf = decltype(buf_c)::value;
    if (r < TM) {
      af[buf][r] = *reinterpret_cast<const uintx4*>(a_frag + stage * T::STAGE_BYTES +
                                                    r * 32 * ROWB + chunk_bytes[kk]);
    } else if constexpr (T::NATIVE && !T::BF16) {
      const unsigned char* src = ring + stage * T::STAGE_BYTES + nat_row_off +
                                 nat_piece_off[r - TM] + 8 * kk * T::B_ROW_BYTES;
      uintx4 v;
#pragma unroll
      for (int t = 0; t < 4; ++t)
        v[t] = *reinterpret_cast<const unsigned*>(src + t * T::B_ROW_BYTES);
      bf[buf][r - TM] = v;
    } else if constexpr (T::NATIVE) {
      typedef short shortx4 __attribute__((ext_vector_type(4)));
      typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));
      typedef __attribute__((address_space(3))) shortx4* lds_ptr;
      const unsigned char* src = ring + stage * T::STAGE_BYTES + nat_row_off +
                                 nat_piece_off[r - TM] + 16 * kk * T::B_ROW_BYTES;
      const uintx2 lo = __builtin_bit_cast(
          uintx2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(src)));
      const uintx2 hi = __builtin_bit_cast(
          uintx2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(src + 4 * T::B_ROW_BYTES)));
      bf[buf][r - TM] = uintx4{lo.x, lo.y, hi.x, hi.y};
    } else {
      bf[buf][r - TM] = *reinterpret_cast<const uintx4*>(b_frag + stage * T::STAGE_BYTES +
                                                         (r - TM) * 32 * ROWB + chunk_bytes[kk]);
    }
  };
  // MFMA number m of a step.
  auto mfma = [&](auto buf_c, int m) {
    constexpr int buf = decltype(buf_c)::value;
    const int i = m / (TN * MPF), j = (m / MPF) % TN, t = m % MPF;
    if constexpr (T::BF16) {
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
          __builtin_bit_cast(bf16x8, af[buf][i]), __builtin_bit_cast(bf16x8, bf[buf][j]), acc[i][j],
          0, 0, 0);
    } else {
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(af[buf][i][t]),
                                                       __uint_as_float(bf[buf][j][t]), acc[i][j],
                                                       0, 0, 0);
    }
  };
  using Buf0 = std::integral_constant<int, 0>;
  using Buf1 = std::integral_constant<int, 1>;

  // One fragment step: NM MFMAs with the side work dealt out between them.
  // The loads of slice i+S may start once the barrier in the last step of
  // slice i has released that slice's stage, and must all be out before the
  // barrier of slice i+1: they are dealt over the KSTEPS steps in between
  // (load number l in step l * KSTEPS / LOADS of that period), because a
  // burst of them right after the barrier backs up the load unit and stalls
  // the wave's MFMA issue behind it.
  // Side work of the last step of a slice: wait + barrier, the NR reads of
  // the next slice's first step, the first share of the loads of slice i+S.
  // Side work of any other step kk of slice i+1: the NR reads of its next
  // step and share kk+1 of those loads (into the stage of slice i); the
  // load position advances after the last share.
  auto load_one = [&](int stage, int l) {
    if (l < T::A_ITERS) load_a(stage, l); else load_b(stage, l - T::A_ITERS);
  };
  auto step = [&](auto cur_c, auto nxt_c, int stage, int kk, int stage_next, int stage_prev) {
    const bool last = kk == KSTEPS - 1;
    const int share = last ? 0 : kk + 1;                      // which share of the loads
    const int l0 = share * T::LOADS / KSTEPS, l1 = (share + 1) * T::LOADS / KSTEPS;
    const bool adv = share == KSTEPS - 1;
    const int nside = (last ? 1 : 0) + NR + (l1 - l0) + (adv ? 1 : 0);
    const int room = NM > 3 ? NM - 2 : NM;           // MFMA gaps that take side work
    const int per_gap = (nside + room - 1) / room;   // side items per gap
    int item = 0;
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      mfma(cur_c, m);
#pragma unroll
      for (int g = 0; g < per_gap; ++g, ++item) {
        const int it = last ? item - 1 : item;       // item number after the barrier
        if (item >= nside) {
          // nothing left for this gap
        } else if (last && item == 0) {
          // next step belongs to the next slice: its loads must have landed
          // (this lane's: vmcnt; everyone's: barrier), and the barrier also
          // says that every wave's reads of this slice's stage are complete
          // (lgkmcnt), so the loads that follow may overwrite it
          __builtin_amdgcn_s_waitcnt(vmcnt_lds_imm(T::WAIT_STEADY));
          __builtin_amdgcn_s_barrier();
          asm volatile("" ::: "memory");  // LDS changed behind the compiler's back
        } else if (it < NR) {
          if (last) read_frag(nxt_c, stage_next, 0, it); else read_frag(nxt_c, stage, kk + 1, it);
        } else if (it < NR + (l1 - l0)) {
          load_one(last ? stage : stage_prev, l0 + it - NR);
        } else {
          advance();
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // prologue: slices 0 .. S-2 and the first share of slice S-1 in flight
  // (the steps of slice 0 issue its other shares), slice 0 landed, its first
  // fragments read
#pragma unroll
  for (int s = 0; s < S; ++s) {
#pragma unroll
    for (int l = 0; l < (s < S - 1 ? T::LOADS : T::LOADS / KSTEPS); ++l) load_one(s, l);
    if (s < S - 1) advance();
  }
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(T::WAIT_FIRST));
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
#pragma unroll
  for (int r = 0; r < NR; ++r) read_frag(Buf0{}, 0, 0, r);
  __builtin_amdgcn_sched_barrier(0);

  for (int slice = 0; slice < nslices; slice += S) {
#pragma unroll
    for (int u = 0; u < S; ++u) {
      if (slice + u < nslices) {
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
          // KSTEPS is even: step kk uses fragment buffer kk % 2, and the first
          // step of the next slice uses buffer 0 again
          if (kk % 2 == 0)
            step(Buf0{}, Buf1{}, u, kk, (u + 1) % S, (u + S - 1) % S);
          else
            step(Buf1{}, Buf0{}, u, kk, (u + 1) % S, (u + S - 1) % S);
        }
        if (WINO) {
          if (--until_flush == 0) {
            until_flush = flush_slices;
            const int pt = min(wino_point, 15);
            ++wino_point;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const float sign = kWinoFold[pt][q];
#pragma unroll
              for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                  for (int v = 0; v < 16; ++v)
                    pixel[q][i][j][v] = fmaf(sign, acc[i][j][v], pixel[q][i][j][v]);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
              for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
          }
        }
        if (TWO_LEVEL) {
          if (--until_flush == 0) {
            until_flush = flush_slices;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
              for (int j = 0; j < TN; ++j)
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
  // The bias of this lane's columns, fetched before the first store.  The empty asm makes the
  // values "arrive" here, in uniform control flow: left to itself the compiler waits for the
  // loads inside every bounds-checked store block, and that wait (the counter covers loads
  // and stores alike) drains all earlier stores each time, one round trip per store.
  float bias_col[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j)
    bias_col[j] = bias_of(p.bias, n0 + wn * T::WN + j * 32 + lr, p.K);
#pragma unroll
  for (int j = 0; j < TN; ++j) asm volatile("" : "+v"(bias_col[j]));
  if (WINO) {
    // the tile's rows are Winograd tiles (n, th, tw): four output pixels each
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = n0 + wn * T::WN + j * 32 + lr;
        const int rbase = m0 + wm * T::WM + i * 32 + lk * 4;
        const float bcol = bias_col[j];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = rbase + 8 * (v / 4) + (v % 4);
          if (row < p.M && col < p.K) {
            const int tw = row % p.wino_tw;
            const int tr = row / p.wino_tw;
            const int th = tr % p.wino_th;
            const int n = tr / p.wino_th;
            if (p.pool) {
              // the four outputs of a Winograd tile are one 2x2 pooling window
              const int P2 = p.wino_p / 2, Q2 = p.wino_q / 2;
              if (th < P2 && tw < Q2) {
                const float m = fmaxf(fmaxf(pixel[0][i][j][v], pixel[1][i][j][v]),
                                      fmaxf(pixel[2][i][j][v], pixel[3][i][j][v]));
                store_out(static_cast<float*>(p.out) +
                              ((static_cast<size_t>(n) * P2 + th) * Q2 + tw) * p.K + col,
                          finish(m, bcol, p.relu));
              }
              continue;
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const int op = 2 * th + (q >> 1), oq = 2 * tw + (q & 1);
              if (op < p.wino_p && oq < p.wino_q)
                store_out(static_cast<float*>(p.out) +
                              ((static_cast<size_t>(n) * p.wino_p + op) * p.wino_q + oq) * p.K + col,
                          finish(pixel[q][i][j][v], bcol, p.relu));
            }
          }
        }
      }
    }
    return;
  }
  if (TWO_LEVEL) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] += total[i][j][v];
  }

  // ---- epilogue (accumulator layout: lane l reg v -> row 8*(v/4) + 4*(l/32) + v%4, col l%32)
  if (is_tail) {
    // piece of a tail tile: a whole [BM][BN] fp32 tile, no bounds
    float* part = partial + static_cast<size_t>(piece) * (BM * BN);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          part[(wm * T::WM + i * 32 + lk * 4 + 8 * (v / 4) + (v % 4)) * BN + wn * T::WN + j * 32 +
               lr] = acc[i][j][v];
    return;
  }
  const bool to_partial = gridDim.y > 1;
  // split_counters: the workgroup of a tile that stores its partial sums last adds them all
  // (below); the partial sums then go through memory with device-coherent stores and loads.
  const bool in_launch = to_partial && split_counters != nullptr;
  float* part = partial + static_cast<size_t>(blockIdx.y) * static_cast<size_t>(p.M) * p.K;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
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
            store_out(static_cast<unsigned short*>(p.out) + bz * p.out_stride + idx,
                      to_bf16_bits(finish(acc[i][j][v], bcol, p.relu)));
          else if (p.batches > 1)  // an intermediate that the next kernel reads: keep it cached
            static_cast<float*>(p.out)[bz * p.out_stride + idx] =
                finish(acc[i][j][v], bcol, p.relu);
          else
            store_out(static_cast<float*>(p.out) + bz * p.out_stride + idx,
                      finish(acc[i][j][v], bcol, p.relu));
        }
      }
    }
  }
  if (!in_launch) return;

  // ---- split reduction inside the launch (split_in_launch.h): the ring is free from here on
  // (the call's first step is a wait for this wave's loads past the end and a barrier)
  constexpr int AHEAD = BM * BN / 4 / T::NT <= 4 && T::OCC <= 4 ? 3 : 2;
  if constexpr (BM * BN <= 128 * 64)
    splitk::split_reduce_in_launch<BM, BN, T::NT, OUT_BF16, AHEAD>(
        p, partial, split_counters + tile, gridDim.y, reduce_groups, m0, n0,
        reinterpret_cast<unsigned*>(ring), tid);
}

// Sum of the pieces of each tail tile, in slice order, to the output.
// gridDim.x = tail tiles, gridDim.y * 1024 = BM * BN: a thread adds 4
// consecutive columns of one row.
template <int BM, int BN, bool OUT_BF16>
__global__ __launch_bounds__(256) void tail_reduce_kernel(const float* __restrict__ partial,
                                                          void* __restrict__ out, int M, int K,
                                                          int nslices, const TailPlan tail,
                                                          const float* __restrict__ bias,
                                                          int relu) {
  const int t = blockIdx.x;  // tail tile
  const int tiles_n = (K + BN - 1) / BN;
  const int tile = tail.n_main + t;
  const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;
  const long long first = 1LL * t * nslices;
  const int g_lo = tail.owner(first);
  const int g_hi = tail.owner(first + nslices - 1);
  const int e = (blockIdx.y * 256 + threadIdx.x) * 4;
  const int row = e / BN, col = e % BN;
  // range g_lo holds the tile's first slice: as its first piece if the range
  // starts there, else as its second; every later range starts inside the tile
  const float* src = partial + (static_cast<size_t>(g_lo) * 2 +
                                (tail.first_unit(g_lo) == first ? 0 : 1)) * (BM * BN) + e;
  float4 acc = *reinterpret_cast<const float4*>(src);
  for (int g = g_lo + 1; g <= g_hi; ++g) {
    const float4 v =
        *reinterpret_cast<const float4*>(partial + static_cast<size_t>(g) * 2 * (BM * BN) + e);
    acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
  }
  const int m = m0 + row, n = n0 + col;
  if (m >= M) return;
  const float a[4] = {acc.x, acc.y, acc.z, acc.w};
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    if (n + c < K) {
      const size_t idx = static_cast<size_t>(m) * K + n + c;
      const float r = finish(a[c], bias_of(bias, n + c, K), relu);
      if (OUT_BF16)
        static_cast<unsigned short*>(out)[idx] = to_bf16_bits(r);
      else
        static_cast<float*>(out)[idx] = r;
    }
  }
}

// ---- counters of the split reduction inside the launch.  One counter per output tile, in banks;
// a stream gets a bank of its own the first time it runs such a launch (launches of one stream
// never overlap, and every launch leaves its counters at zero, which is also how the array
// starts), so launches that run at the same time on different streams never share a counter.
// A stream that is being captured into a graph gets none (the graph may be replayed on any
// stream), nor does a stream that comes when all banks are taken: those launches add their
// partial sums in a second launch, as do outputs of more tiles than a bank has counters.
constexpr int kCounterBanks = 32;
constexpr int kCountersPerBank = 4096;
constexpr int kCounterDevices = 64;
}  // namespace dma
}  // namespace conv2d
static __device__ unsigned split_counter_array[conv2d::dma::kCounterBanks *
                                               conv2d::dma::kCountersPerBank];
namespace conv2d {
namespace dma {
std::mutex counter_mutex;
unsigned* counter_base[kCounterDevices] = {};
struct BankOwner {
  int device;
  hipStream_t stream;
};
BankOwner bank_owner[kCounterBanks];
int banks_taken = 0;
std::atomic<int> split_reduce_separate{0};  // 1: always add the partial sums in a second launch

}  // namespace dma
// The stream's counter bank on the current device, or null.
unsigned* split_counters_for_stream(hipStream_t stream, int tiles) {
  using namespace dma;
  if (split_reduce_separate.load(std::memory_order_relaxed) || tiles > kCountersPerBank)
    return nullptr;
  hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(stream, &capture) != hipSuccess) {
    (void)hipGetLastError();
    return nullptr;
  }
  if (capture != hipStreamCaptureStatusNone) return nullptr;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kCounterDevices) return nullptr;
  std::lock_guard<std::mutex> lock(counter_mutex);
  if (!counter_base[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(split_counter_array)) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
    counter_base[dev] = static_cast<unsigned*>(ptr);
  }
  int bank = -1;
  for (int b = 0; b < banks_taken; ++b)
    if (bank_owner[b].device == dev && bank_owner[b].stream == stream) bank = b;
  if (bank < 0) {
    if (banks_taken == kCounterBanks) return nullptr;
    bank = banks_taken++;
    bank_owner[bank] = BankOwner{dev, stream};
  }
  return counter_base[dev] + bank * kCountersPerBank;
}
namespace dma {

// Bytes of the repacked filter at the head of the workspace (a multiple of 256).
template <class T>
size_t filter_bytes(const Problem& p) {
  if (T::NATIVE) return 0;  // no repacked copy
  const size_t kg_p = static_cast<size_t>((p.Kg + T::BK - 1) / T::BK) * T::BK;
  return (kg_p * p.K * T::ES + 255) / 256 * 256;
}

template <class T>
int clamp_splits(const Problem& p, int splits, int* per_split) {
  const int nslices = (p.Kg + T::BK - 1) / T::BK;
  if (splits < 1) splits = 1;
  if (splits > nslices) splits = nslices;
  *per_split = (nslices + splits - 1) / splits;
  return (nslices + *per_split - 1) / *per_split;  // no empty split
}

// Tail plan for a problem.  Whole rounds of 256 tiles (one per compute unit)
// run as they are; the slices of the remaining tiles are dealt evenly to up
// to 256 ranges (never more than two pieces each, no piece shorter than about
// 4 slices).  The dispatcher fills all workgroup slots of a compute unit
// before it moves to the next, so fewer whole tiles than one workgroup per
// slot would leave units idle while others hold two tiles: then every tile
// goes to the tail.
template <class T>
TailPlan plan_tail(const Problem& p, bool want_tail) {
  const int tiles = ((p.M + T::BM - 1) / T::BM) * ((p.K + T::BN - 1) / T::BN);
  const int nslices = (p.Kg + T::BK - 1) / T::BK;
  TailPlan t = {tiles, 0, 0, 0, 0};
  // pixel tiles first where an XCD's share of the input is smaller than the filter
  const double in_bytes = 1.0 * p.N * p.H * p.W * p.C, filt_bytes = 1.0 * p.Kg * p.K;
  t.pixel_tiles_first = (p.batches <= 1 && filt_bytes > in_bytes / kXcds) ? 1 : 0;
  int rest = tiles % 256;
  if (!want_tail || rest == 0) return t;
  if (tiles - rest < 256 * T::OCC) rest = tiles;
  const long long units = 1LL * rest * nslices;
  const long long most = rest > 256 ? 256LL * ((rest + 255) / 256) : 256;
  long long wgs = units / 4 < most ? units / 4 : most;
  if (wgs < rest) wgs = rest;
  t.n_main = tiles - rest;
  t.wgs = static_cast<int>(wgs);
  t.base = static_cast<int>(units / wgs);
  t.extra = static_cast<int>(units % wgs);
  return t;
}

// `splits` > 1: uniform split of the reduction; `splits` == kTailBalanced:
// whole tiles plus a balanced tail; otherwise one workgroup per tile.
template <class T, bool OUT_BF16>
hipError_t launch_one(const Problem& p, int splits, hipStream_t stream) {
  const int Kg_p = (p.Kg + T::BK - 1) / T::BK * T::BK;
  const int batches = p.batches > 1 ? p.batches : 1;
  if (batches > 1 && splits != 1) return hipErrorInvalidValue;  // batched: whole tiles only
  // 1. filter -> Bt[K][Kg_p] in the workspace (one per batch), unless the caller packed it before
  // (native tiles read the filter as it is; their "packed" filter is a plain copy)
  if (T::NATIVE && (p.K % T::VEC != 0 || batches > 1)) return hipErrorInvalidValue;
  const void* bt = p.packed_filt ? p.packed_filt : (T::NATIVE ? p.filt : p.workspace);
  hipError_t e = hipSuccess;
  if (!p.packed_filt && !T::NATIVE) {
    dim3 rgrid(Kg_p / T::BK, (p.K + 63) / 64, batches);
    const long long bt_stride = static_cast<long long>(filter_bytes<T>(p) / T::ES);
    if (T::BF16)
      hipLaunchKernelGGL((repack_filter_kernel<unsigned short>), rgrid, dim3(256), 0, stream,
                         static_cast<const unsigned short*>(p.filt),
                         static_cast<unsigned short*>(p.workspace), p.Kg, p.K, Kg_p, p.C,
                         p.R * p.S, T::UNIFORM ? T::BK : 0, T::BK, p.filt_stride, bt_stride);
    else
      hipLaunchKernelGGL((repack_filter_kernel<float>), rgrid, dim3(256), 0, stream,
                         static_cast<const float*>(p.filt), static_cast<float*>(p.workspace),
                         p.Kg, p.K, Kg_p, p.C, p.R * p.S, T::UNIFORM ? T::BK : 0, T::BK,
                         p.filt_stride, bt_stride);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  // 2. the convolution
  const TailPlan tail = plan_tail<T>(p, splits == kTailBalanced);
  int per_split;
  splits = clamp_splits<T>(p, splits, &per_split);
  int flush = 1;
  while (flush * flush < per_split) ++flush;
  float* partial = reinterpret_cast<float*>(static_cast<unsigned char*>(p.workspace) +
                                            filter_bytes<T>(p));
  // A uniform split adds its partial sums inside the launch where it can and where it pays
  // (split_in_launch.h; a 56x56x256 -> 256 layer at batch 1 with 6 splits of 64x64 tiles: 45.2 ->
  // 42.3 us; 14x14x512 -> 512 at batch 1 with 18 splits: 22.0 -> 25.3 us, so that one keeps the
  // second launch), given a counter bank for the stream.
  unsigned* counters = nullptr;
  if (tail.wgs == 0 && splitk::split_in_launch_pays(p, T::BM, T::BN, splits, OUT_BF16))
    counters = split_counters_for_stream(stream, tail.n_main);
  hipLaunchKernelGGL((igemm_dma_kernel<T, OUT_BF16>),
                     dim3(tail.n_main + 2 * tail.wgs, splits, batches), dim3(T::NT), 0, stream, p,
                     Kg_p, per_split, flush, bt, partial, tail, counters,
                     split_reduce_groups(p.M * p.K, splits));
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (counters) return hipSuccess;
  // 3. sum of the partial outputs
  if (tail.wgs > 0) {
    const int rest = ((p.M + T::BM - 1) / T::BM) * ((p.K + T::BN - 1) / T::BN) - tail.n_main;
    hipLaunchKernelGGL((tail_reduce_kernel<T::BM, T::BN, OUT_BF16>),
                       dim3(rest, T::BM * T::BN / 1024), dim3(256), 0, stream, partial, p.out, p.M,
                       p.K, Kg_p / T::BK, tail, p.bias, p.relu);
    return hipGetLastError();
  }
  if (splits > 1)
    return launch_split_reduce(partial, p.out, p.M * p.K, splits, OUT_BF16, p.bias, p.relu, p.K,
                               stream);
  return hipSuccess;
}

template <class T>
hipError_t launch(const Problem& p, int splits, hipStream_t stream) {
  if (T::BF16 && p.out_bf16) return launch_one<T, T::BF16>(p, splits, stream);
  return launch_one<T, false>(p, splits, stream);
}

// Winograd point products with the output transform folded in: repack of U,
// then one workgroup per (BM Winograd tiles) x (BN features).
template <class T>
hipError_t launch_wino(const Problem& p, hipStream_t stream) {
  if (p.C % T::BK != 0 || p.R != 16 || p.S != 1 || p.out_bf16) return hipErrorInvalidValue;
  const int Kg_p = p.Kg;
  const void* bt = p.packed_filt ? p.packed_filt : p.workspace;
  hipError_t e = hipSuccess;
  if (!p.packed_filt) {
    dim3 rgrid(Kg_p / T::BK, (p.K + 63) / 64, 1);
    hipLaunchKernelGGL((repack_filter_kernel<float>), rgrid, dim3(256), 0, stream,
                       static_cast<const float*>(p.filt), static_cast<float*>(p.workspace), p.Kg,
                       p.K, Kg_p, p.C, p.R * p.S, 0, T::BK, 0LL, 0LL);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const int tiles = ((p.M + T::BM - 1) / T::BM) * ((p.K + T::BN - 1) / T::BN);
  const TailPlan none = {tiles, 0, 0, 0, 0};
  hipLaunchKernelGGL((igemm_dma_kernel<T, false, true>), dim3(tiles, 1, 1), dim3(T::NT), 0, stream,
                     p, Kg_p, Kg_p / T::BK, p.C / T::BK, bt, static_cast<float*>(nullptr), none,
                     static_cast<unsigned*>(nullptr), 1);
  return hipGetLastError();
}

template <class T>
size_t workspace_bytes(const Problem& p, int splits) {
  if (p.batches > 1) return filter_bytes<T>(p) * p.batches;
  const TailPlan tail = plan_tail<T>(p, splits == kTailBalanced);
  if (tail.wgs > 0)
    return filter_bytes<T>(p) + static_cast<size_t>(tail.wgs) * 2 * T::BM * T::BN * sizeof(float);
  int per_split;
  splits = clamp_splits<T>(p, splits, &per_split);
  return filter_bytes<T>(p) +
         (splits > 1 ? static_cast<size_t>(splits) * p.M * p.K * sizeof(float) : 0);
}

// ---------------------------------------------------------------------------
// LDS-resident input patch for 3x3 (any R x S), stride-1 layers.
//
// The gather kernel above fetches every input element once per tap: nine
// times for a 3x3 window, and at 64 bytes per pixel row per slice that
// request stream, not the matrix cores, is what bounds the bf16 tiles (the L2
// of an XCD is ~83 % busy).  Here a workgroup loads, per block of BK
// channels, the whole patch of input pixels that its BM consecutive output
// pixels touch, once, and the MFMA fragment reads of all R*S taps address
// into it: with the input laid out as a zero-padded image of width
// Wp = W + pad_left + pad_right, output pixel m with window origin index
// base(m) = (n*Hp + p)*Wp + q reads, for tap (r,s), patch entry
// base(m) + r*Wp + s.  The patch of a tile is the contiguous range of such
// indices from base(m0) on; entries that fall into the padding frame (or
// past the last image) are loaded with an out-of-range offset and read zero.
//
// LDS layout of a patch: CPR planes of PATCH_ROWS x 16 bytes (plane c holds
// 16-byte chunk c of every entry), so one load instruction fills 64
// consecutive entries of a plane and a fragment read (32 consecutive entries
// of one plane per lane half) is conflict free without a swizzle.  Two patch
// buffers alternate between channel blocks; the filter slices go through a
// three-stage ring exactly as above (same repacked, channel-block-major
// filter).  The nine taps of a 3x3 window are unrolled, one barrier per tap
// slice; the patch of the next channel block is loaded during the first six
// tap slices of the current one.
//
// Blocked tiles (BW > 0) take a BH x BW block of output pixels of one image
// (BH = BM / BW) instead of BM consecutive ones: their patch is the
// (BH + 2) x (BW + 2) block of input pixels around it, stored row by row with
// its own width, so wide images, whose consecutive-pixel patch would span
// several whole image rows, fit as well.
//
// 16-row tiles (MF16, bf16): 16x16x32 MFMA blocks, one per 64-byte row (a
// single step per slice), so that a wave tile can be 112 rows high: the
// output pixel counts of these workloads are 49 * 2^k, which tiles of 224 or
// 448 rows divide and tiles of 128 or 256 rows do not (a last round that is
// 77 % full against 87.5 %).  The blocks are computed transposed (filter
// fragment as the first operand), so a lane ends up with four consecutive
// features of one pixel and stores them as one 16-byte vector.
//
// Native filter (NATIVE, bf16 16-row tiles): the filter slice is loaded as it lies in memory,
// BK rows (one per k) of BN consecutive features, and the MFMA operand (8 consecutive k of one
// feature per lane) is formed by two transposing LDS reads (ds_read_b64_tr_b16: the 16 lanes of
// a group hand in 4 rows x 16 features and each gets the 4 rows of its feature).  No repacked
// copy of the filter, no workspace and no launch before the convolution.  A group's read
// touches 4 rows at one feature offset, 16 row pieces of 32 bytes per wavefront, which would all
// start at the same bank (the rows are a multiple of 256 bytes apart), so the 32-byte piece j
// of row k is stored at piece position j ^ native_swizzle(k): measured 200 bytes per clock and
// compute unit against 32 unswizzled.
template <bool BF16_, int BM_, int BN_, int WAVES_M_, int WAVES_N_, int PATCH_ROWS_,
          bool TWO_LEVEL_, int OCC_, int BW_ = 0, bool MF16_ = false, bool NATIVE_ = false>
struct PatchTile {
  static constexpr bool NATIVE = NATIVE_;
  static_assert(!NATIVE_ || BN_ % 64 == 0, "native filter: whole 64-feature groups");
  static constexpr int B_ROW_BYTES = BN_ * (BF16_ ? 2 : 4);   // NATIVE: a filter row (one k) in LDS
  // NATIVE, bf16 16-row blocks: XOR of the 32-byte piece index of filter row k (rows of at
  // least 8 pieces: the 4 rows of a lane group and the group 8 rows on get 8 different
  // positions; 4 pieces: 2 bits).  32-row blocks (bf16 and fp32): as DmaTile::native_swizzle.
  static constexpr int native_swizzle(int k) {
    if (!BF16_) return (k >> 2) & 1;
    if (!MF16_) return BN_ >= 128 ? ((k & 3) << 1) : (((k >> 1) & 1) << 1);
    return BN_ >= 128 ? ((k & 3) | (((k >> 3) & 1) << 2)) : (((k >> 1) & 1) | (((k >> 3) & 1) << 1));
  }
  static constexpr bool BF16 = BF16_;
  static constexpr int BM = BM_, BN = BN_;
  static constexpr int BW = BW_;                       // 0: BM consecutive output pixels
  static constexpr int BH = BW_ > 0 ? BM_ / BW_ : 0;
  static constexpr int PW = BW_ + 2;                   // patch width of a blocked tile
  static_assert(BW_ == 0 || (BM_ % BW_ == 0 && (BM_ / BW_ + 2) * (BW_ + 2) <= PATCH_ROWS_),
                "blocked tile: BM = BH * BW and its patch must fit");
  static constexpr bool MF16 = MF16_;
  static_assert(!MF16_ || BF16_, "16-row blocks are a bf16 feature");
  static constexpr int BLK = MF16 ? 16 : 32;        // rows / columns of an MFMA block
  static constexpr int ACC = MF16 ? 4 : 16;         // accumulator registers of a block
  static constexpr int ROWB = 64, CPR = 4, KSTEPS = MF16 ? 1 : 2;
  // swizzle of the filter rows (see DmaTile): a 16-row block's read (row = lane % 16, chunk =
  // lane / 16) is conflict free with shift 1, a 32-row block's with shift 2
  static constexpr int SWZ_SHIFT = MF16 ? 1 : 2;
  static constexpr int ES = BF16 ? 2 : 4;
  static constexpr int VEC = 16 / ES;
  static constexpr int BK = ROWB / ES;
  static constexpr int SB = 3;                   // filter ring stages
  static constexpr bool TWO_LEVEL = TWO_LEVEL_;
  static constexpr int OCC = OCC_;
  static constexpr int ADDR = 3;
  // blocked tiles of 32-row blocks: a workgroup takes several tiles, one after the other (the
  // 16-row tiles were slower that way: 71.9 -> 81.0 us on a 112x112x128 layer at batch 16)
  static constexpr bool PERSIST = BW_ > 0 && !MF16_;
  // A split reduction over the channel blocks (several workgroups per tile, fp32 partial sums):
  // for tiles of one tile per workgroup whose wave tiles leave registers for it
  static constexpr bool SPLITS = !PERSIST && (BM_ / WAVES_M_) * (BN_ / WAVES_N_) <= 128 * 64;
  // 2x2 pooling in the epilogue: blocks of 16 columns and an even number of rows, 32-row blocks
  static constexpr bool POOLS = BW_ == 16 && !MF16_ && (BM_ / 16) % 2 == 0;
  static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
  static constexpr int NW = WAVES_M * WAVES_N;
  static constexpr int NT = 64 * NW;
  static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  static constexpr int TM = WM / BLK, TN = WN / BLK;
  static constexpr int MPF = BF16 ? 1 : 4;
  static constexpr int NM = TM * TN * MPF;
  static constexpr int NR = TM + TN;
  static constexpr int PATCH_ROWS = PATCH_ROWS_;
  static constexpr int PLANE_BYTES = PATCH_ROWS * 16;
  static constexpr int PATCH_BYTES = CPR * PLANE_BYTES;
  // Patch loads: a wave takes 64 consecutive entries of every plane per pass
  // (A_PASSES passes); a patch that is no multiple of 64 * NW entries is dealt
  // by plane instead (BY_PLANE: wave w loads plane w of every 64-entry chunk).
  static constexpr bool BY_PLANE = PATCH_ROWS % (64 * NW) != 0;
  static_assert(!BY_PLANE || (NW == CPR && PATCH_ROWS % 64 == 0), "patch rows over the waves");
  static constexpr int A_PASSES = BY_PLANE ? PATCH_ROWS / 64 : PATCH_ROWS / (64 * NW);
  static constexpr int A_LOADS = BY_PLANE ? A_PASSES : A_PASSES * CPR;  // per lane and block
  static constexpr int A_SLICES = 6;              // dealt over the first 6 tap slices of a block
  static constexpr int B_ROWS_PER_PASS = NT / CPR;
  static constexpr int B_ITERS = BN / B_ROWS_PER_PASS;
  static constexpr int B_STAGE_BYTES = BN * ROWB;
  static constexpr int LDS_BYTES = 2 * PATCH_BYTES + SB * B_STAGE_BYTES;
  static_assert(BN % B_ROWS_PER_PASS == 0 && B_ROWS_PER_PASS % 16 == 0, "filter tile rows");
  static_assert(LDS_BYTES <= 160 * 1024, "does not fit LDS");
  static_assert(WM % BLK == 0 && WN % BLK == 0, "wave tile must be a multiple of the MFMA block");
  static_assert(!(BF16 && TWO_LEVEL), "two-level summation is an fp32 feature");
  // patch loads issued at the end of tap slice t of a block
  static constexpr int a_first(int t) { return t >= A_SLICES ? A_LOADS : t * A_LOADS / A_SLICES; }
  static constexpr int a_count(int t) { return t < 0 ? 0 : a_first(t + 1) - a_first(t); }
};

// Patch entries that the tile starting at output pixel m0 needs.
__host__ __device__ inline long long patch_base(const Problem& p, int Hp, int Wp, int m) {
  const int q = m % p.Q, t = m / p.Q;
  return (1LL * (t / p.P) * Hp + t % p.P) * Wp + q;
}

template <class T, bool OUT_BF16>
__global__ __launch_bounds__(T::NT, T::OCC) void igemm_patch_kernel(const Problem p, const int Hp,
                                                                    const int Wp,
                                                                    const int flush_slices,
                                                                    const void* bt,
                                                                    const int ntiles,
                                                                    const int blocks_per_split,
                                                                    float* partial) {
  constexpr int BM = T::BM, BN = T::BN, BK = T::BK, ROWB = T::ROWB, CPR = T::CPR, SB = T::SB;
  constexpr int ES = T::ES, VEC = T::VEC, KSTEPS = T::KSTEPS;
  constexpr int TM = T::TM, TN = T::TN, NM = T::NM, NR = T::NR, MPF = T::MPF;
  constexpr int BLK = T::BLK, ACC = T::ACC;
  using Acc = std::conditional_t<T::MF16, floatx4, floatx16>;
  __shared__ __align__(1024) unsigned char ring[T::LDS_BYTES];
  constexpr int B_REGION = 2 * T::PATCH_BYTES;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave / T::WAVES_N;
  const int wn = wave % T::WAVES_N;
  const int lr = lane & (BLK - 1);   // row / column of the lane inside an MFMA block
  const int lk = lane / BLK;         // its group of 8 (bf16) / 4 (fp32) k values

  // Tiles of this workgroup.  Each XCD owns a contiguous range of tiles (feature tiles
  // fastest); workgroup i runs on XCD i % 8.  Persistent tiles (blocked, 32-row blocks) are
  // launched with at most OCC workgroups per compute unit, and a workgroup walks its XCD's
  // range with the stride of that XCD's workgroup count, loading the next tile's patch and
  // first filter slices while it finishes the current one; all others get one tile each.
  constexpr bool PERSIST = T::PERSIST;
  const int tiles_n = (p.K + BN - 1) / BN;
  const int nwg = gridDim.x;
  const int xcd = blockIdx.x % kXcds;
  const int local = blockIdx.x / kXcds;
  const int per = ntiles / kXcds, rem = ntiles % kXcds;
  const int tile_end = xcd * per + (xcd < rem ? xcd : rem) + per + (xcd < rem ? 1 : 0);
  const int tile_step = nwg / kXcds + (xcd < nwg % kXcds ? 1 : 0);
  int tile = tile_end - (per + (xcd < rem ? 1 : 0)) + local;
  int m0 = (tile / tiles_n) * BM;   // consecutive-pixel tiles: first output pixel
  int n0 = (tile % tiles_n) * BN;
  // blocked tiles: image and top-left output pixel of the block
  int blk_n = 0, blk_p = 0, blk_q = 0;
  auto block_of = [&](int t, int& bn, int& bp, int& bq) {
    if constexpr (T::BW > 0) {
      const int nbx = (p.Q + T::BW - 1) / T::BW, nby = (p.P + T::BH - 1) / T::BH;
      const int tm = t / tiles_n;
      bq = (tm % nbx) * T::BW;
      bp = ((tm / nbx) % nby) * T::BH;
      bn = tm / (nbx * nby);
    }
  };
  if constexpr (T::BW > 0) block_of(tile, blk_n, blk_p, blk_q);
  constexpr int taps = 9;
  const int Kg_p = p.Kg;             // C is a multiple of BK
  // Channel blocks of this workgroup: all of them, or (gridDim.y > 1: a split reduction over
  // the channels) those from blockIdx.y * blocks_per_split on, whose sum goes to plane
  // blockIdx.y of `partial`.  Input and filter are then seen from the first of these channels
  // on (channel c of a pixel is c * ES bytes into the pixel, filter row (tap, c) c rows into the
  // tap, repacked slice (block, tap) 9 * block + tap slices in), so that nothing below changes.
  const int first_block = T::SPLITS ? blockIdx.y * blocks_per_split : 0;
  const int nblocks = T::SPLITS ? min(blocks_per_split, p.C / BK - first_block) : p.C / BK;
  const bool to_partial = T::SPLITS && gridDim.y > 1;
  const long long in_shift = 1LL * first_block * ROWB;
  const long long bt_shift =
      T::NATIVE ? 1LL * first_block * BK * p.K * ES : 1LL * first_block * taps * p.K * ROWB;
  const uintx4 in_rsrc = make_rsrc(static_cast<const unsigned char*>(p.in) + in_shift, 0,
                                   1LL * p.N * p.H * p.W * p.C * ES - in_shift);
  const uintx4 bt_rsrc = make_rsrc(static_cast<const unsigned char*>(bt) + bt_shift, 0,
                                   1LL * p.K * Kg_p * ES - bt_shift);
  const unsigned ring_base = __builtin_amdgcn_readfirstlane(lds_address(ring) + wave * 1024);

  // ---- patch loader role: entries (pass*NW + wave)*64 + lane of the patch
  const long long v0 = T::BW > 0 ? 0 : patch_base(p, Hp, Wp, m0);
  int a_voff[T::A_PASSES];
  // blocked tiles: the patch offsets of the block at (bn, bp, bq)
  auto block_patch_offsets = [&](int bn, int bp, int bq, int (&voff)[T::A_PASSES]) {
#pragma unroll
    for (int i = 0; i < T::A_PASSES; ++i) {
      // entry e of the patch: row e / PW, column e % PW of the input block
      const int e = (T::BY_PLANE ? i : i * T::NW + wave) * 64 + lane;
      const int dy = e / T::PW, dx = e % T::PW;
      const int h = bp - p.pt + dy, w = bq - p.pl + dx;
      const bool ok = dy < T::BH + 2 && static_cast<unsigned>(h) < static_cast<unsigned>(p.H) &&
                      static_cast<unsigned>(w) < static_cast<unsigned>(p.W);
      voff[i] = ok ? ((bn * p.H + h) * p.W + w) * p.C * ES : kOutOfRange;
    }
  };
  if constexpr (T::BW > 0) block_patch_offsets(blk_n, blk_p, blk_q, a_voff);
#pragma unroll
  for (int i = 0; i < T::A_PASSES; ++i) {
    if constexpr (T::BW == 0) {
      // (32-bit arithmetic: padded pixel indices stay far below 2^31 for tensors that the
      // host accepts, and 64-bit divisions here were a third of a workgroup's start-up time)
      const unsigned v = static_cast<unsigned>(v0) + (T::BY_PLANE ? i : i * T::NW + wave) * 64 + lane;
      const unsigned t = v / static_cast<unsigned>(Wp);
      const int w = static_cast<int>(v - t * Wp) - p.pl;
      const unsigned n = t / static_cast<unsigned>(Hp);
      const int h = static_cast<int>(t - n * Hp) - p.pt;
      const bool ok = n < static_cast<unsigned>(p.N) &&
                      static_cast<unsigned>(h) < static_cast<unsigned>(p.H) &&
                      static_cast<unsigned>(w) < static_cast<unsigned>(p.W);
      a_voff[i] = ok ? static_cast<int>(((n * p.H + h) * p.W + w) * p.C * ES) : kOutOfRange;
    }
  }
  // ---- filter loader role (as in the gather kernel)
  const int ld_row0 = tid / CPR;
  const int ld_chunk = (tid % CPR) ^ ((ld_row0 >> T::SWZ_SHIFT) & (CPR - 1));
  int b_voff[T::B_ITERS];
  auto filter_offsets = [&](int col0, int (&voff)[T::B_ITERS]) {
#pragma unroll
    for (int i = 0; i < T::B_ITERS; ++i) {
      if constexpr (T::NATIVE) {
        // 16-byte chunk q of the stage: row k = q / chunks per row, position q % chunks per
        // row, which holds the chunk of features [8c, 8c + 8) with c = position ^ swizzle
        constexpr int CH = BN / VEC;
        const int q = i * T::NT + tid;
        const int k = q / CH;
        // (bf16: pieces of 2 chunks; fp32: halves of 8 chunks)
        const int c = (q % CH) ^ (T::native_swizzle(k) << (T::BF16 ? 1 : 3));
        const int n = col0 + VEC * c;
        voff[i] = (n + VEC <= p.K) ? (k * p.K + n) * ES : kOutOfRange;
      } else {
        const int n = col0 + ld_row0 + i * T::B_ROWS_PER_PASS;
        voff[i] = (n < p.K) ? (n * BK + ld_chunk * VEC) * ES : kOutOfRange;
      }
    }
  };
  filter_offsets(n0, b_voff);
  const int k_slice_bytes = p.K * ROWB;
  const int k_last_bytes = (nblocks * taps - 1) * k_slice_bytes;
  int k_next_bytes = 0;         // filter slice to load next; wraps into the next tile's
  // NATIVE: the slices are visited channel block by channel block, all taps of a block; slice
  // (block, tap) starts at filter row tap * C + block * BK
  int nat_tap = 0, nat_block_bytes = 0;
  const int nat_tap_bytes = p.C * p.K * ES;
  const int nat_blocks_bytes = nblocks * BK * p.K * ES;  // this workgroup's channels of a tap
  // Moves the filter load position one slice on (past the last slice: to the first again).
  auto next_filter_slice = [&]() {
    if constexpr (T::NATIVE) {
      // (selects, not branches: the position stays in scalar registers)
      const bool wrap = ++nat_tap == taps;
      nat_tap = wrap ? 0 : nat_tap;
      const int next_block = nat_block_bytes + BK * p.K * ES;
      nat_block_bytes = wrap ? (next_block >= nat_blocks_bytes ? 0 : next_block) : nat_block_bytes;
      k_next_bytes = wrap ? nat_block_bytes : k_next_bytes + nat_tap_bytes;
    } else {
      k_next_bytes = k_next_bytes >= k_last_bytes ? 0 : k_next_bytes + k_slice_bytes;
    }
  };
  int a_next_block_bytes = 0;   // channel offset (bytes) of the patch being loaded
  // Persistent tiles: the loads of a tile's last channel block (patch) and last SB slices
  // (filter) fetch the workgroup's next tile's (or nothing: out-of-range offsets); the loader
  // offsets are switched at those points.
  bool last_block = false;
  int tile_next = 0, n0_next = 0, next_n = 0, next_p = 0, next_q = 0;
  bool has_next = false;

  auto load_b = [&](int stage, int i) {
    dma16(bt_rsrc, ring_base + B_REGION + stage * T::B_STAGE_BYTES + i * T::B_ROWS_PER_PASS * ROWB,
          b_voff[i], T::NATIVE ? __builtin_amdgcn_readfirstlane(k_next_bytes) : k_next_bytes);
  };
  // patch load number j (pass j / CPR, plane j % CPR) into patch buffer `buf`
  auto load_a = [&](int buf, int j) {
    if constexpr (T::BY_PLANE) {
      // chunk j of plane `wave` (ring_base - wave * 1024 is the start of the ring)
      const int w = __builtin_amdgcn_readfirstlane(wave);
      dma16(in_rsrc, ring_base + buf * T::PATCH_BYTES + w * (T::PLANE_BYTES - 1024) + j * 1024,
            a_voff[j], a_next_block_bytes + w * 16);
    } else {
      const int i = j / CPR, c = j % CPR;
      dma16(in_rsrc, ring_base + buf * T::PATCH_BYTES + c * T::PLANE_BYTES + i * T::NW * 1024,
            a_voff[i], a_next_block_bytes + c * 16);
    }
  };

  Acc acc[TM][TN];
  Acc total[T::TWO_LEVEL ? TM : 1][T::TWO_LEVEL ? TN : 1];
  int until_flush = flush_slices;

  // ---- fragment addressing.  A: patch entry of the lane's output pixel in
  // each 32-row block (pixels past M repeat the last one; they are not
  // stored), plane lk (+2 per step).  B: as in the gather kernel.
  int a_frag[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    if constexpr (T::BW > 0) {
      const int ml = wm * T::WM + i * BLK + lr;  // pixel (ml / BW, ml % BW) of the block
      a_frag[i] = ((ml / T::BW) * T::PW + ml % T::BW) * 16 + lk * T::PLANE_BYTES;
    } else {
      const int m = min(m0 + wm * T::WM + i * BLK + lr, p.M - 1);
      a_frag[i] = static_cast<int>(patch_base(p, Hp, Wp, m) - v0) * 16 + lk * T::PLANE_BYTES;
    }
  }
  const int frag_swz = (lr >> T::SWZ_SHIFT) & (CPR - 1);
  const unsigned char* b_frag = ring + B_REGION + (wn * T::WN + lr) * ROWB;
  int chunk_bytes[KSTEPS];
#pragma unroll
  for (int kk = 0; kk < KSTEPS; ++kk) chunk_bytes[kk] = ((2 * kk + lk) ^ frag_swz) * 16;

  // NATIVE: lane (feature lr of a block, k group lk) hands in the address of row
  // 8 * lk + lr / 4 (+ 4 for the second read), features 4 * (lr % 4) ... of the block
  int nat_row_off = 0, nat_piece_off[T::NATIVE ? TN : 1] = {};
  if constexpr (T::NATIVE && T::MF16) {
    const int k = 8 * lk + lr / 4;
    nat_row_off = k * T::B_ROW_BYTES + 8 * (lr % 4);
#pragma unroll
    for (int j = 0; j < TN; ++j)
      nat_piece_off[j] = 32 * ((wn * TN + j) ^ T::native_swizzle(k));
  }
  // 32-row blocks (as in the gather kernel): bf16 lanes hand in row 16 kk + 8 lk +
  // (lane % 16) / 4 of their half block; fp32 lanes read rows 8 kk + 4 lk + t of their feature
  if constexpr (T::NATIVE && !T::MF16 && T::BF16) {
    const int a = lane & 15, k = 8 * lk + a / 4;
    nat_row_off = k * T::B_ROW_BYTES + 8 * (a % 4);
#pragma unroll
    for (int j = 0; j < TN; ++j)
      nat_piece_off[j] = 32 * ((2 * (wn * TN + j) + ((lane >> 4) & 1)) ^ T::native_swizzle(k));
  }
  if constexpr (T::NATIVE && !T::BF16) {
    nat_row_off = 4 * lk * T::B_ROW_BYTES + 4 * lr;
#pragma unroll
    for (int j = 0; j < TN; ++j) nat_piece_off[j] = 128 * ((wn * TN + j) ^ lk);
  }

  uintx4 af[2][TM], bf[2][TN];
  int a_buf_off = 0;  // byte offset of the patch buffer being read (0 or PATCH_BYTES)

  // Fragment read r (A blocks, then B blocks) of step kk; A from the patch at
  // byte offset a_off (buffer + tap), B from filter stage `bstage`.
  auto read_frag = [&](auto buf_c, int a_off, int bstage, int kk, int r) {
    constexpr int buf = decltype(buf_c)::value;
    // (16-row blocks: one buffer for the A fragments, two only for the last)
    if (r < TM) {
      af[T::MF16 && r < TM - 1 ? 0 : buf][r] = *reinterpret_cast<const uintx4*>(
          ring + a_frag[r] + a_off + 2 * kk * T::PLANE_BYTES);
    } else if constexpr (T::NATIVE && !T::BF16) {
      const unsigned char* src = ring + B_REGION + bstage * T::B_STAGE_BYTES + nat_row_off +
                                 nat_piece_off[r - TM] + 8 * kk * T::B_ROW_BYTES;
      uintx4 v;
#pragma unroll
      for (int t = 0; t < 4; ++t)
        v[t] = *reinterpret_cast<const unsigned*>(src + t * T::B_ROW_BYTES);
      bf[buf][r - TM] = v;
    } else if constexpr (T::NATIVE) {
      typedef short shortx4 __attribute__((ext_vector_type(4)));
      typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));
      typedef __attribute__((address_space(3))) shortx4* lds_ptr;
      // (16-row blocks have one step per slice: kk = 0)
      const unsigned char* src = ring + B_REGION + bstage * T::B_STAGE_BYTES + nat_row_off +
                                 nat_piece_off[r - TM] + 16 * kk * T::B_ROW_BYTES;
      const uintx2 lo = __builtin_bit_cast(
          uintx2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(src)));
      const uintx2 hi = __builtin_bit_cast(
          uintx2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(src + 4 * T::B_ROW_BYTES)));
      bf[buf][r - TM] = uintx4{lo.x, lo.y, hi.x, hi.y};
    } else {
      bf[buf][r - TM] = *reinterpret_cast<const uintx4*>(
          b_frag + bstage * T::B_STAGE_BYTES + (r - TM) * BLK * ROWB + chunk_bytes[kk]);
    }
  };
  auto mfma = [&](auto buf_c, int m) {
    constexpr int buf = decltype(buf_c)::value;
    const int i = m / (TN * MPF), j = (m / MPF) % TN, t = m % MPF;
    if constexpr (T::MF16) {
      // transposed block: features x pixels
      acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
          __builtin_bit_cast(bf16x8, bf[buf][j]),
          __builtin_bit_cast(bf16x8, af[i < TM - 1 ? 0 : buf][i]), acc[i][j], 0, 0, 0);
    } else if constexpr (T::BF16) {
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
          __builtin_bit_cast(bf16x8, af[buf][i]), __builtin_bit_cast(bf16x8, bf[buf][j]), acc[i][j],
          0, 0, 0);
    } else {
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(af[buf][i][t]),
                                                       __uint_as_float(bf[buf][j][t]), acc[i][j],
                                                       0, 0, 0);
    }
  };
  using Buf0 = std::integral_constant<int, 0>;
  using Buf1 = std::integral_constant<int, 1>;
  // NM MFMAs of one step with `nside` side items dealt out between them
  // (pinned by scheduling fences, none after the last two MFMAs).
  auto run_step = [&](auto cur_c, int nside, auto side) {
    const int room = NM > 3 ? NM - 2 : NM;
    const int per_gap = (nside + room - 1) / room;
    int item = 0;
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      mfma(cur_c, m);
#pragma unroll
      for (int g = 0; g < per_gap; ++g, ++item)
        if (item < nside) side(item);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // Tap slice t of a channel block: filter stage t % SB.  Step 0 reads the
  // fragments of step 1.  Step 1: wait for the next slice's filter tile (and
  // this wave's LDS reads), barrier, read the next slice's first fragments,
  // load the filter slice SB ahead into the stage just released, and this
  // slice's share of the next block's patch.
  // The same for 16-row blocks, where the A fragments have a single buffer (registers): the
  // next slice's A fragment i is read right after the last MFMA that uses this slice's
  // (MFMAs run A block by A block), everything else fills the other gaps in order.  The last
  // A fragment would be read after the slice's last MFMA, right before the next slice's wait
  // for all LDS reads; it has two buffers and is read early, as one of the other items.
  auto run_step16 = [&](auto cur_c, int nside, auto side, auto read_a) {
    int item = 0;
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      mfma(cur_c, m);
      if (m % TN == TN - 1 && m / TN < TM - 1) {
        read_a(m / TN);
      } else if (item < nside) {
        side(item);
        ++item;
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  static_assert(!T::MF16 || 3 + TN + T::B_ITERS + T::A_LOADS <= NM - TM, "side items need gaps");

  // With one step per slice (16-row blocks) the B fragment buffers alternate per slice: `par`
  // is the buffer that holds this slice's.
  auto tap_slice = [&](auto t_c, auto par_c) {
    constexpr int t = decltype(t_c)::value;
    constexpr int par = decltype(par_c)::value;
    using Cur = std::integral_constant<int, KSTEPS == 2 ? 1 : par>;
    using Nxt = std::integral_constant<int, KSTEPS == 2 ? 0 : (par ^ 1)>;
    constexpr int bstage = t % SB;
    constexpr int tn = (t + 1) % taps;
    const int a_cur = a_buf_off + ((t / 3) * Wp + t % 3) * 16;
    const int a_nxt = (t == taps - 1 ? (a_buf_off ^ T::PATCH_BYTES) : a_buf_off) +
                      ((tn / 3) * Wp + tn % 3) * 16;
    const int a_load_buf = (a_buf_off ^ T::PATCH_BYTES) / T::PATCH_BYTES;
    constexpr int a_from = T::a_first(t), a_n = T::a_count(t);
    // loads younger than the next slice's filter tile: the filter tile after
    // it and the patch loads of the two slices before this one
    constexpr int wait_n = T::B_ITERS + T::a_count(t - 2) + T::a_count(t - 1);
    // the filter loads of a tile's last SB slices fetch the next tile's first slices
    // (a tile without a successor loads its own first slices again, into stages nobody reads)
    if constexpr (PERSIST && t == taps - SB) {
      if (last_block) {
        filter_offsets(n0_next, b_voff);
        if (!has_next) {
#pragma unroll
          for (int i = 0; i < T::B_ITERS; ++i) b_voff[i] = kOutOfRange;
        }
      }
    }
    if constexpr (T::MF16) {
      run_step16(
          Cur{}, 2 + TN + T::B_ITERS + a_n + 1,
          [&](int item) {
            if (item == 0) {
              __builtin_amdgcn_s_waitcnt(vmcnt_lds_imm(wait_n));
              __builtin_amdgcn_s_barrier();
              asm volatile("" ::: "memory");  // LDS changed behind the compiler's back
            } else if (item <= TN) {
              read_frag(Nxt{}, a_nxt, (bstage + 1) % SB, 0, TM + item - 1);
            } else if (item == TN + 1) {
              read_frag(Nxt{}, a_nxt, (bstage + 1) % SB, 0, TM - 1);
            } else if (item <= 1 + TN + T::B_ITERS) {
              load_b(bstage, item - TN - 2);
            } else if (item <= 1 + TN + T::B_ITERS + a_n) {
              load_a(a_load_buf, a_from + item - TN - T::B_ITERS - 2);
            } else {
              next_filter_slice();
            }
          },
          [&](int i) { read_frag(Nxt{}, a_nxt, (bstage + 1) % SB, 0, i); });
    } else {
    if constexpr (KSTEPS == 2)
      run_step(Buf0{}, NR, [&](int item) { read_frag(Buf1{}, a_cur, bstage, 1, item); });
    run_step(Cur{}, 1 + NR + T::B_ITERS + a_n + 1, [&](int item) {
      if (item == 0) {
        __builtin_amdgcn_s_waitcnt(vmcnt_lds_imm(wait_n));
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");  // LDS changed behind the compiler's back
      } else if (item <= NR) {
        read_frag(Nxt{}, a_nxt, (bstage + 1) % SB, 0, item - 1);
      } else if (item <= NR + T::B_ITERS) {
        load_b(bstage, item - NR - 1);
      } else if (item <= NR + T::B_ITERS + a_n) {
        load_a(a_load_buf, a_from + item - NR - T::B_ITERS - 1);
      } else {
        next_filter_slice();
      }
    });
    }
    if (T::TWO_LEVEL) {
      if (--until_flush == 0) {
        until_flush = flush_slices;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < ACC; ++v) {
              total[i][j][v] += acc[i][j][v];
              acc[i][j][v] = 0.f;
            }
      }
    }
  };
  // the nine tap slices of a channel block whose first slice's fragments are in buffer `bp`
  auto channel_block = [&](auto bp_c) {
    constexpr int bp = decltype(bp_c)::value;
    tap_slice(std::integral_constant<int, 0>{}, std::integral_constant<int, bp>{});
    tap_slice(std::integral_constant<int, 1>{}, std::integral_constant<int, bp ^ 1>{});
    tap_slice(std::integral_constant<int, 2>{}, std::integral_constant<int, bp>{});
    tap_slice(std::integral_constant<int, 3>{}, std::integral_constant<int, bp ^ 1>{});
    tap_slice(std::integral_constant<int, 4>{}, std::integral_constant<int, bp>{});
    tap_slice(std::integral_constant<int, 5>{}, std::integral_constant<int, bp ^ 1>{});
    tap_slice(std::integral_constant<int, 6>{}, std::integral_constant<int, bp>{});
    tap_slice(std::integral_constant<int, 7>{}, std::integral_constant<int, bp ^ 1>{});
    tap_slice(std::integral_constant<int, 8>{}, std::integral_constant<int, bp>{});
  };

  // prologue: the first block's patch and the first SB filter slices in
  // flight; patch and slice 0 landed; first fragments read
#pragma unroll
  for (int j = 0; j < T::A_LOADS; ++j) load_a(0, j);
#pragma unroll
  for (int s = 0; s < SB; ++s) {
#pragma unroll
    for (int i = 0; i < T::B_ITERS; ++i) load_b(s, i);
    next_filter_slice();
  }
  __builtin_amdgcn_s_waitcnt(vmcnt_imm((SB - 1) * T::B_ITERS));
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
#pragma unroll
  for (int r = 0; r < NR; ++r) read_frag(Buf0{}, 0, 0, 0, r);
  __builtin_amdgcn_sched_barrier(0);

  // The patch loaded during a channel block is the next block's; during a tile's last block it
  // is the first block of the workgroup's next tile (or nothing).
  auto begin_block = [&](int block) {
    if constexpr (PERSIST) {
      last_block = block == nblocks - 1;
      a_next_block_bytes = last_block ? 0 : (block + 1) * ROWB;
      if (last_block) {
        block_patch_offsets(next_n, next_p, next_q, a_voff);
        if (!has_next) {
#pragma unroll
          for (int i = 0; i < T::A_PASSES; ++i) a_voff[i] = kOutOfRange;
        }
      }
    } else {
      // (past the end: the last block again, into the buffer nobody reads)
      a_next_block_bytes = min(block + 1, nblocks - 1) * ROWB;
    }
  };

  for (;;) {
  // ---- the workgroup's next tile, if any
  tile_next = tile + tile_step;
  has_next = PERSIST && tile_next < tile_end;
  if constexpr (PERSIST) {
    if (has_next) {
      block_of(tile_next, next_n, next_p, next_q);
      n0_next = (tile_next % tiles_n) * BN;
    }
  }
  // The bias of this lane's columns (32-row blocks), fetched before the tile's loop.  The empty
  // asm makes the values "arrive" here, in uniform control flow: left to itself the compiler
  // waits for the loads inside every bounds-checked store block, and that wait (the counter
  // covers loads and stores alike) drains all earlier stores each time, one round trip per
  // store.  At this point it only waits for loads that the first slice needs anyway.
  float bias_col[TN];
  if constexpr (!T::MF16) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
      bias_col[j] = bias_of(p.bias, n0 + wn * T::WN + j * 32 + lr, p.K);
#pragma unroll
    for (int j = 0; j < TN; ++j) asm volatile("" : "+v"(bias_col[j]));
  }
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < ACC; ++v) acc[i][j][v] = 0.f;
  if (T::TWO_LEVEL) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < ACC; ++v) total[i][j][v] = 0.f;
    until_flush = flush_slices;
  }

  if constexpr (KSTEPS == 2) {
    for (int block = 0; block < nblocks; ++block) {
      begin_block(block);
      channel_block(Buf0{});
      a_buf_off ^= T::PATCH_BYTES;
    }
  } else {
    // nine slices per block and one step per slice: the fragment buffer parity flips from
    // block to block, so the loop body is a pair of blocks
    int block = 0;
    for (; block + 1 < nblocks; block += 2) {
      begin_block(block);
      channel_block(Buf0{});
      a_buf_off ^= T::PATCH_BYTES;
      begin_block(block + 1);
      channel_block(Buf1{});
      a_buf_off ^= T::PATCH_BYTES;
    }
    if (block < nblocks) {
      begin_block(block);
      channel_block(Buf0{});
      a_buf_off ^= T::PATCH_BYTES;
    }
  }
  if (T::TWO_LEVEL) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < ACC; ++v) acc[i][j][v] += total[i][j][v];
  }

  if constexpr (T::MF16) {
    // ---- epilogue of the transposed 16x16 blocks: lane l, register v -> pixel l % 16,
    // feature 4 * (l / 16) + v of the block: four consecutive features per lane
    float bias4[TN][4];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v)
        bias4[j][v] = bias_of(p.bias, n0 + wn * T::WN + j * BLK + lk * 4 + v, p.K);
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) asm volatile("" : "+v"(bias4[j][v]));
    const bool vec_ok = (p.K & 3) == 0;
    // output row of pixel `px` of 16-row block i, or -1 if it is not stored
    auto out_row = [&](int i, int px) {
      int row = m0 + wm * T::WM + i * BLK + px;
      bool row_ok = row < p.M;
      if constexpr (T::BW > 0) {
        const int ml = row - m0;  // position in the block
        const int op = blk_p + ml / T::BW, oq = blk_q + ml % T::BW;
        row_ok = op < p.P && oq < p.Q;
        row = (blk_n * p.P + op) * p.Q + oq;
      }
      return row_ok ? row : -1;
    };
    // fp32 output with whole 32-feature groups: two feature blocks are stored together so that
    // one store instruction writes whole 128-byte lines (8 pixels x 32 features) instead of
    // 64-byte halves (16 pixels x 16 features), which as non-temporal stores cost ~1.45x the
    // write traffic.  Lanes px and px ^ 8 swap one of their two quads (a rotate by 8 inside
    // the row of 16 lanes); then the first store covers the pixels with px & 8 == 0, the second
    // the others.
    constexpr int kStageRow = T::WN * 2 + 16;  // bytes of a staged pixel: its features + a pad
    if (to_partial) {
      // a split over the channels: the sums as they are, to this split's plane of `partial`
      // (ordinary stores: the kernel that adds the planes reads them next)
      float* part = partial + static_cast<size_t>(blockIdx.y) * p.M * p.K;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row = out_row(i, lr);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const int col = n0 + wn * T::WN + j * BLK + lk * 4;
          if (row < 0) continue;
          const size_t idx = static_cast<size_t>(row) * p.K + col;
          if (vec_ok && col + 3 < p.K) {
            *reinterpret_cast<floatx4*>(part + idx) = acc[i][j];
          } else {
#pragma unroll
            for (int v = 0; v < 4; ++v)
              if (col + v < p.K) part[idx + v] = acc[i][j][v];
          }
        }
      }
    } else if (OUT_BF16 && T::WN == 64 && (p.K & 7) == 0 &&
        T::NW * T::WM * kStageRow <= T::LDS_BYTES) {
      // bf16 output: a lane's 8-byte pieces (four features of a pixel) are gathered through LDS
      // into whole 128-byte lines (64 features of a pixel), 8 pixels per store instruction.  The
      // ring is free: every wave has its last fragments in registers (the reads issued during
      // the last slice are the dummy ones past the end), once the loads that every wave issued
      // past the end have landed (they write all over the ring).  Each wave stages its own rows.
      typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      unsigned char* stage = ring + wave * (T::WM * kStageRow);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          float r[4];
#pragma unroll
          for (int v = 0; v < 4; ++v) r[v] = finish(acc[i][j][v], bias4[j][v], p.relu);
          uintx2 packed;
          packed.x = to_bf16_bits(r[0]) | (static_cast<unsigned>(to_bf16_bits(r[1])) << 16);
          packed.y = to_bf16_bits(r[2]) | (static_cast<unsigned>(to_bf16_bits(r[3])) << 16);
          *reinterpret_cast<uintx2*>(stage + (i * BLK + lr) * kStageRow + (j * BLK + lk * 4) * 2) =
              packed;
        }
      __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): this wave's staged rows are written
      asm volatile("" ::: "memory");
      const int chunk = lane & 7;           // 16 bytes = 8 features
      const int col = n0 + wn * T::WN + chunk * 8;
#pragma unroll
      for (int t = 0; t < T::WM / 8; ++t) {
        const int pw = t * 8 + (lane >> 3);  // pixel of the wave's rows
        const uintx4 line = *reinterpret_cast<const uintx4*>(stage + pw * kStageRow + chunk * 16);
        const int row = out_row(pw / BLK, pw % BLK);
        if (row >= 0 && col + 7 < p.K)
          store_out(reinterpret_cast<uintx4*>(static_cast<unsigned short*>(p.out) +
                                              static_cast<size_t>(row) * p.K + col),
                    line);
      }
    } else if (!OUT_BF16 && TN % 2 == 0 && (p.K & 31) == 0) {
      const bool hi = (lr & 8) != 0;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row_own = out_row(i, lr), row_other = out_row(i, lr ^ 8);
#pragma unroll
        for (int j = 0; j < TN; j += 2) {
          const int col = n0 + wn * T::WN + (hi ? j + 1 : j) * BLK + lk * 4;
          floatx4 lo, up, sent, got;
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            lo[v] = finish(acc[i][j][v], bias4[j][v], p.relu);
            up[v] = finish(acc[i][j + 1][v], bias4[j + 1][v], p.relu);
          }
          sent = hi ? lo : up;
#pragma unroll
          for (int v = 0; v < 4; ++v)
            got[v] = __int_as_float(__builtin_amdgcn_update_dpp(
                0, __float_as_int(sent[v]), 0x128 /* row_ror:8 */, 0xf, 0xf, false));
          // pixels with px & 8 == 0: their own lower quad, the partner's upper quad
          const int row_a = hi ? row_other : row_own;
          if (row_a >= 0 && col + 3 < p.K)
            store_out(reinterpret_cast<floatx4*>(static_cast<float*>(p.out) +
                                                 static_cast<size_t>(row_a) * p.K + col),
                      hi ? got : lo);
          const int row_b = hi ? row_own : row_other;
          if (row_b >= 0 && col + 3 < p.K)
            store_out(reinterpret_cast<floatx4*>(static_cast<float*>(p.out) +
                                                 static_cast<size_t>(row_b) * p.K + col),
                      hi ? up : got);
        }
      }
    } else {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int row = out_row(i, lr);
      const bool row_ok = row >= 0;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = n0 + wn * T::WN + j * BLK + lk * 4;
        float r[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) r[v] = finish(acc[i][j][v], bias4[j][v], p.relu);
        if (row_ok) {
          const size_t idx = static_cast<size_t>(row) * p.K + col;
          if (vec_ok && col + 3 < p.K) {
            if (OUT_BF16) {
              typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));
              uintx2 packed;
              packed.x = to_bf16_bits(r[0]) | (static_cast<unsigned>(to_bf16_bits(r[1])) << 16);
              packed.y = to_bf16_bits(r[2]) | (static_cast<unsigned>(to_bf16_bits(r[3])) << 16);
              // (32 bytes per pixel and instruction: as non-temporal stores such pieces cost more
              // write traffic than they save in L2; ordinary stores, which L2 merges.  Only for
              // shapes that the staged path above does not take.)
              *reinterpret_cast<uintx2*>(static_cast<unsigned short*>(p.out) + idx) = packed;
            } else {
              floatx4 quad = {r[0], r[1], r[2], r[3]};
              store_out(reinterpret_cast<floatx4*>(static_cast<float*>(p.out) + idx), quad);
            }
          } else {
#pragma unroll
            for (int v = 0; v < 4; ++v)
              if (col + v < p.K) {
                if (OUT_BF16)
                  static_cast<unsigned short*>(p.out)[idx + v] = to_bf16_bits(r[v]);
                else
                  static_cast<float*>(p.out)[idx + v] = r[v];
              }
          }
        }
      }
    }
    }  // one feature block per store
  } else {
  bool pooled = false;
  if constexpr (T::POOLS) {
    if (p.pool) {
      // ---- pooled epilogue.  A 32-row block is two rows of the 16-pixel-wide tile; with the
      // accumulator layout below, the 2x2 window of pooled column x of that row pair is
      // registers v, v + 1 (pixel pair along the row) and v + 8, v + 9 (the row below) of one
      // lane, v = 0, 2, 4, 6.
      const int P2 = p.P / 2, Q2 = p.Q / 2;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int py = (blk_p + (wm * T::WM + i * 32) / T::BW) / 2;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const int col = n0 + wn * T::WN + j * 32 + lr;
          const float bcol = bias_col[j];
#pragma unroll
          for (int v = 0; v < 8; v += 2) {
            const int px = (blk_q + 8 * (v / 4) + 4 * lk + v % 4) / 2;
            const float m = fmaxf(fmaxf(acc[i][j][v], acc[i][j][v + 1]),
                                  fmaxf(acc[i][j][v + 8], acc[i][j][v + 9]));
            if (py < P2 && px < Q2 && col < p.K) {
              const size_t idx = (static_cast<size_t>(blk_n * P2 + py) * Q2 + px) * p.K + col;
              if (OUT_BF16)
                store_out(static_cast<unsigned short*>(p.out) + idx,
                          to_bf16_bits(finish(m, bcol, p.relu)));
              else
                store_out(static_cast<float*>(p.out) + idx, finish(m, bcol, p.relu));
            }
          }
        }
      }
      pooled = true;
    }
  }
  if (!pooled) {
  // ---- epilogue (accumulator layout: lane l reg v -> row 8*(v/4) + 4*(l/32) + v%4, col l%32)
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = n0 + wn * T::WN + j * 32 + lr;
      const int rbase = m0 + wm * T::WM + i * 32 + lk * 4;
      const float bcol = bias_col[j];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        int row = rbase + 8 * (v / 4) + (v % 4);
        bool row_ok = row < p.M;
        if constexpr (T::BW > 0) {
          const int ml = row - m0;  // position in the block
          const int op = blk_p + ml / T::BW, oq = blk_q + ml % T::BW;
          row_ok = op < p.P && oq < p.Q;
          row = (blk_n * p.P + op) * p.Q + oq;
        }
        if (row_ok && col < p.K) {
          const size_t idx = static_cast<size_t>(row) * p.K + col;
          if (to_partial)  // a split over the channels: the sum as it is, to its plane
            partial[static_cast<size_t>(blockIdx.y) * p.M * p.K + idx] = acc[i][j][v];
          else if (OUT_BF16)
            store_out(static_cast<unsigned short*>(p.out) + idx,
                      to_bf16_bits(finish(acc[i][j][v], bcol, p.relu)));
          else
            store_out(static_cast<float*>(p.out) + idx, finish(acc[i][j][v], bcol, p.relu));
        }
      }
    }
  }
  }  // unpooled
  }  // 32-row blocks

  if (!has_next) break;
  // on to the next tile: its patch and first filter slices are in flight or landed, its first
  // fragments are in registers, the loader offsets were switched during the last block
  tile = tile_next;
  n0 = n0_next;
  m0 = (tile / tiles_n) * BM;
  blk_n = next_n;
  blk_p = next_p;
  blk_q = next_q;
  }  // tiles of this workgroup
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // drain the loads issued past the end
}

// Largest number of patch entries any tile of the problem needs.
template <class T>
long long patch_rows_needed(const Problem& p) {
  const int Hp = p.P + p.R - 1, Wp = p.Q + p.S - 1;  // stride 1: padded extent
  long long worst = 0;
  for (int m0 = 0; m0 < p.M; m0 += T::BM) {
    const int m1 = (m0 + T::BM - 1 < p.M - 1) ? m0 + T::BM - 1 : p.M - 1;
    const long long span = patch_base(p, Hp, Wp, m1) - patch_base(p, Hp, Wp, m0);
    if (span > worst) worst = span;
  }
  return worst + 1LL * (p.R - 1) * Wp + (p.S - 1) + 1;
}

template <class T>
bool patch_fits(const Problem& p) {
  if (!(p.R == 3 && p.S == 3 && p.sr == 1 && p.sc == 1 && p.C % T::BK == 0)) return false;
  if (T::NATIVE && p.K % T::VEC != 0) return false;  // 16-byte chunks of a filter row
  if (T::BW > 0) return true;  // a block's patch always fits
  // (the kernel indexes the padded images' pixels with 32 bits)
  if (1LL * p.N * (p.P + p.R - 1) * (p.Q + p.S - 1) + T::PATCH_ROWS >= (1LL << 31)) return false;
  return patch_rows_needed<T>(p) <= T::PATCH_ROWS;
}

// Output tiles along M: blocks of BH x BW pixels per image, or runs of BM pixels.
template <class T>
int patch_tiles_m(const Problem& p) {
  if (T::BW > 0) return p.N * ((p.P + T::BH - 1) / T::BH) * ((p.Q + T::BW - 1) / T::BW);
  return (p.M + T::BM - 1) / T::BM;
}

// Repacked filter (none for native tiles), then the partial sums of a split over the channels.
template <class T>
size_t workspace_bytes_patch(const Problem& p, int splits) {
  const size_t filter =
      T::NATIVE ? 0 : (static_cast<size_t>(p.Kg) * p.K * T::ES + 255) / 256 * 256;
  if (splits <= 1 || !T::SPLITS) return filter;
  return filter + static_cast<size_t>(splits) * p.M * p.K * sizeof(float);
}

// Split of the channel blocks of a patch tile over `splits` workgroups per tile: blocks per
// split, and the number of splits that leaves none empty (1 for tiles that do not split).
template <class T>
int patch_blocks_per_split(const Problem& p, int* splits) {
  const int nblocks = p.C / T::BK;
  int s = !T::SPLITS || *splits < 1 ? 1 : *splits;
  if (s > nblocks) s = nblocks;
  const int per = (nblocks + s - 1) / s;
  *splits = (nblocks + per - 1) / per;
  return per;
}

template <class T, bool OUT_BF16>
hipError_t launch_patch_one(const Problem& p, int splits, hipStream_t stream) {
  // 1. filter -> Bt[slice][K][BK], channel block by channel block, unless packed before
  // (native tiles read the filter as it is; their "packed" filter is a plain copy)
  const void* bt = p.packed_filt ? p.packed_filt : (T::NATIVE ? p.filt : p.workspace);
  hipError_t e = hipSuccess;
  if (!p.packed_filt && !T::NATIVE) {
    dim3 rgrid(p.Kg / T::BK, (p.K + 63) / 64);
    if (T::BF16)
      hipLaunchKernelGGL((repack_filter_kernel<unsigned short>), rgrid, dim3(256), 0, stream,
                         static_cast<const unsigned short*>(p.filt),
                         static_cast<unsigned short*>(p.workspace), p.Kg, p.K, p.Kg, p.C,
                         p.R * p.S, T::BK, T::BK, 0LL, 0LL);
    else
      hipLaunchKernelGGL((repack_filter_kernel<float>), rgrid, dim3(256), 0, stream,
                         static_cast<const float*>(p.filt), static_cast<float*>(p.workspace),
                         p.Kg, p.K, p.Kg, p.C, p.R * p.S, T::BK, T::BK, 0LL, 0LL);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  // 2. the convolution
  const int tiles = patch_tiles_m<T>(p) * ((p.K + T::BN - 1) / T::BN);
  const int nslices = p.Kg / T::BK;
  int flush = 1;
  while (flush * flush < nslices) ++flush;
  // width of the patch rows: the padded image's, or the block's own
  const int patch_width = T::BW > 0 ? T::PW : p.Q + p.S - 1;
  const int resident = kComputeUnits * T::OCC;
  const int grid = T::PERSIST && tiles > resident ? resident : tiles;
  // 3. with a split over the channels: fp32 partial sums behind the repacked filter, added by
  // split_reduce_kernel
  const int per_split = patch_blocks_per_split<T>(p, &splits);
  float* partial = reinterpret_cast<float*>(static_cast<unsigned char*>(p.workspace) +
                                            workspace_bytes_patch<T>(p, 1));
  hipLaunchKernelGGL((igemm_patch_kernel<T, OUT_BF16>), dim3(grid, splits), dim3(T::NT), 0, stream,
                     p, p.P + p.R - 1, patch_width, flush, bt, tiles, per_split, partial);
  e = hipGetLastError();
  if (e != hipSuccess || splits == 1) return e;
  return launch_split_reduce(partial, p.out, p.M * p.K, splits, OUT_BF16, p.bias, p.relu, p.K,
                             stream);
}

template <class T>
hipError_t launch_patch(const Problem& p, int splits, hipStream_t stream) {
  if (!patch_fits<T>(p)) return hipErrorInvalidValue;
  if (T::BF16 && p.out_bf16) return launch_patch_one<T, T::BF16>(p, splits, stream);
  return launch_patch_one<T, false>(p, splits, stream);
}

// Extra shape condition of the native gather tiles: 16-byte chunks of a filter row.
bool native_fits(const Problem& p) { return p.K % (p.in_bf16 ? 8 : 4) == 0 && p.batches <= 1; }

struct TileEntry {
  const char* name;
  int bm, bn, bk, occ;
  int addr;
  hipError_t (*fn)(const Problem&, int, hipStream_t);
  size_t (*ws)(const Problem&, int);
  bool (*fits)(const Problem&);  // extra shape condition of a tile, or null
  hipError_t (*wino)(const Problem&, hipStream_t);  // fused Winograd products, or null
  bool pools = false;                               // 2x2 pooling in the epilogue
  bool native = false;                              // reads the filter as it lies: no repack
  bool splits_channels = false;                     // patch tiles: PatchTile::SPLITS
};

#define CONV2D_PATCH_TILE(dt, isbf, bm, bn, wm, wn, rows, two, occ)                              \
  { "igemm_patch_" dt "_" #bm "x" #bn "_w" #wm "x" #wn "_p" #rows, bm, bn,                       \
    PatchTile<isbf, bm, bn, wm, wn, rows, two, occ>::BK, occ, 3,                                 \
    &launch_patch<PatchTile<isbf, bm, bn, wm, wn, rows, two, occ>>,                              \
    &workspace_bytes_patch<PatchTile<isbf, bm, bn, wm, wn, rows, two, occ>>,                     \
    &patch_fits<PatchTile<isbf, bm, bn, wm, wn, rows, two, occ>>, nullptr, false, false,         \
    PatchTile<isbf, bm, bn, wm, wn, rows, two, occ>::SPLITS }

// 16-row MFMA blocks (tile heights that are multiples of 7 * 32)
#define CONV2D_PATCH_TILE_M16(dt, isbf, bm, bn, wm, wn, rows, occ)                               \
  { "igemm_patch_" dt "_" #bm "x" #bn "_w" #wm "x" #wn "_p" #rows "_m16", bm, bn,               \
    PatchTile<isbf, bm, bn, wm, wn, rows, false, occ, 0, true>::BK, occ, 3,                      \
    &launch_patch<PatchTile<isbf, bm, bn, wm, wn, rows, false, occ, 0, true>>,                   \
    &workspace_bytes_patch<PatchTile<isbf, bm, bn, wm, wn, rows, false, occ, 0, true>>,          \
    &patch_fits<PatchTile<isbf, bm, bn, wm, wn, rows, false, occ, 0, true>>, nullptr, false,     \
    false, PatchTile<isbf, bm, bn, wm, wn, rows, false, occ, 0, true>::SPLITS }

#define CONV2D_PATCH_TILE_M16B(dt, isbf, bm, bn, wm, wn, rows, occ, bw)                          \
  { "igemm_patch_" dt "_" #bm "x" #bn "_w" #wm "x" #wn "_p" #rows "_b" #bw "_m16", bm, bn,      \
    PatchTile<isbf, bm, bn, wm, wn, rows, false, occ, bw, true>::BK, occ, 3,                     \
    &launch_patch<PatchTile<isbf, bm, bn, wm, wn, rows, false, occ, bw, true>>,                  \
    &workspace_bytes_patch<PatchTile<isbf, bm, bn, wm, wn, rows, false, occ, bw, true>>,         \
    &patch_fits<PatchTile<isbf, bm, bn, wm, wn, rows, false, occ, bw, true>>, nullptr, false,    \
    false, PatchTile<isbf, bm, bn, wm, wn, rows, false, occ, bw, true>::SPLITS }

// 16-row tiles that read the filter as it lies in memory (transposing LDS reads): bw = 0 for
// consecutive pixels
#define CONV2D_PATCH_TILE_M16N(dt, isbf, bm, bn, wm, wn, rows, occ, bw, tag)                     \
  { "igemm_patch_" dt "_" #bm "x" #bn "_w" #wm "x" #wn "_p" #rows tag "_m16_nat", bm, bn,        \
    PatchTile<isbf, bm, bn, wm, wn, rows, false, occ, bw, true, true>::BK, occ, 3,               \
    &launch_patch<PatchTile<isbf, bm, bn, wm, wn, rows, false, occ, bw, true, true>>,            \
    &workspace_bytes_patch<PatchTile<isbf, bm, bn, wm, wn, rows, false, occ, bw, true, true>>,   \
    &patch_fits<PatchTile<isbf, bm, bn, wm, wn, rows, false, occ, bw, true, true>>, nullptr,     \
    false, true, PatchTile<isbf, bm, bn, wm, wn, rows, false, occ, bw, true, true>::SPLITS }

// blocked patch tiles of 32-row blocks that read the filter as it lies in memory
#define CONV2D_PATCH_TILE_BN(dt, isbf, bm, bn, wm, wn, rows, two, occ, bw)                       \
  { "igemm_patch_" dt "_" #bm "x" #bn "_w" #wm "x" #wn "_p" #rows "_b" #bw "_nat", bm, bn,       \
    PatchTile<isbf, bm, bn, wm, wn, rows, two, occ, bw, false, true>::BK, occ, 3,                \
    &launch_patch<PatchTile<isbf, bm, bn, wm, wn, rows, two, occ, bw, false, true>>,             \
    &workspace_bytes_patch<PatchTile<isbf, bm, bn, wm, wn, rows, two, occ, bw, false, true>>,    \
    &patch_fits<PatchTile<isbf, bm, bn, wm, wn, rows, two, occ, bw, false, true>>, nullptr,      \
    PatchTile<isbf, bm, bn, wm, wn, rows, two, occ, bw, false, true>::POOLS, true }

// blocked patch tiles: bm / bw x bw output pixels of one image
#define CONV2D_PATCH_TILE_B(dt, isbf, bm, bn, wm, wn, rows, two, occ, bw)                        \
  { "igemm_patch_" dt "_" #bm "x" #bn "_w" #wm "x" #wn "_p" #rows "_b" #bw, bm, bn,              \
    PatchTile<isbf, bm, bn, wm, wn, rows, two, occ, bw>::BK, occ, 3,                             \
    &launch_patch<PatchTile<isbf, bm, bn, wm, wn, rows, two, occ, bw>>,                          \
    &workspace_bytes_patch<PatchTile<isbf, bm, bn, wm, wn, rows, two, occ, bw>>,                 \
    &patch_fits<PatchTile<isbf, bm, bn, wm, wn, rows, two, occ, bw>>, nullptr,                   \
    PatchTile<isbf, bm, bn, wm, wn, rows, two, occ, bw>::POOLS }

// uniform tiles that read the filter as it lies in memory
#define CONV2D_DMA_TILE_N(dt, isbf, bm, bn, rowb, wm, wn, st, two, occ)                         \
  { "igemm_dma_" dt "_" #bm "x" #bn "_r" #rowb "_w" #wm "x" #wn "_s" #st "_nat", bm, bn,        \
    DmaTile<isbf, bm, bn, rowb, wm, wn, st, two, occ, kUniform, true>::BK, occ, kUniform,       \
    &launch<DmaTile<isbf, bm, bn, rowb, wm, wn, st, two, occ, kUniform, true>>,                 \
    &workspace_bytes<DmaTile<isbf, bm, bn, rowb, wm, wn, st, two, occ, kUniform, true>>,        \
    &native_fits, nullptr, false, true }

#define CONV2D_DMA_TILE(dt, isbf, bm, bn, rowb, wm, wn, st, two, occ, addr, tag)                \
  { "igemm_dma_" dt "_" #bm "x" #bn "_r" #rowb "_w" #wm "x" #wn "_s" #st tag, bm, bn,           \
    DmaTile<isbf, bm, bn, rowb, wm, wn, st, two, occ, addr>::BK, occ, addr,                     \
    &launch<DmaTile<isbf, bm, bn, rowb, wm, wn, st, two, occ, addr>>,                           \
    &workspace_bytes<DmaTile<isbf, bm, bn, rowb, wm, wn, st, two, occ, addr>>, nullptr, nullptr }

// the same with an instantiation for the fused Winograd products
#define CONV2D_DMA_TILE_W(dt, isbf, bm, bn, rowb, wm, wn, st, two, occ, addr, tag)              \
  { "igemm_dma_" dt "_" #bm "x" #bn "_r" #rowb "_w" #wm "x" #wn "_s" #st tag, bm, bn,           \
    DmaTile<isbf, bm, bn, rowb, wm, wn, st, two, occ, addr>::BK, occ, addr,                     \
    &launch<DmaTile<isbf, bm, bn, rowb, wm, wn, st, two, occ, addr>>,                           \
    &workspace_bytes<DmaTile<isbf, bm, bn, rowb, wm, wn, st, two, occ, addr>>, nullptr,         \
    &launch_wino<DmaTile<isbf, bm, bn, rowb, wm, wn, st, two, occ, addr>> }

const TileEntry kTilesF32[] = {
    CONV2D_PATCH_TILE("f32", false, 128, 128, 2, 2, 512, true, 1),
    CONV2D_PATCH_TILE_B("f32", false, 128, 128, 2, 2, 256, true, 2, 16),
    CONV2D_PATCH_TILE_B("f32", false, 128, 64, 2, 2, 256, true, 3, 16),
    CONV2D_PATCH_TILE_BN("f32", false, 128, 128, 2, 2, 256, true, 2, 16),
    CONV2D_PATCH_TILE_BN("f32", false, 128, 64, 2, 2, 256, true, 3, 16),
    CONV2D_DMA_TILE("f32", false, 128, 128, 64, 2, 2, 4, true, 2, kUniform, ""),
    CONV2D_DMA_TILE("f32", false, 128, 64, 64, 2, 2, 4, true, 3, kUniform, ""),
    CONV2D_DMA_TILE("f32", false, 256, 128, 64, 4, 2, 4, true, 2, kUniform, ""),
    CONV2D_DMA_TILE("f32", false, 64, 64, 64, 2, 2, 4, true, 4, kUniform, ""),
    CONV2D_DMA_TILE("f32", false, 64, 64, 64, 2, 2, 3, true, 6, kUniform, ""),
    CONV2D_DMA_TILE_N("f32", false, 128, 128, 64, 2, 2, 4, true, 2),
    CONV2D_DMA_TILE_N("f32", false, 128, 64, 64, 2, 2, 4, true, 3),
    CONV2D_DMA_TILE_N("f32", false, 64, 64, 64, 2, 2, 4, true, 4),
    CONV2D_DMA_TILE_N("f32", false, 64, 64, 64, 2, 2, 3, true, 6),
    // (an 8-stage ring for split reductions of few workgroups per compute unit, whose slices
    // are bound by the latency of their loads: 14x14x512 -> 512 at batch 1, 20.6 us against 22.9)
    CONV2D_DMA_TILE_N("f32", false, 64, 64, 64, 2, 2, 8, true, 2),
    CONV2D_DMA_TILE("f32", false, 128, 128, 64, 2, 2, 4, true, 2, kVector, "_g"),
    CONV2D_DMA_TILE("f32", false, 128, 64, 64, 2, 2, 4, true, 3, kVector, "_g"),
    CONV2D_DMA_TILE_W("f32", false, 64, 64, 64, 2, 2, 4, true, 4, kVector, "_g"),
    CONV2D_DMA_TILE("f32", false, 128, 64, 64, 2, 2, 4, true, 3, kElement, "_e"),
    CONV2D_DMA_TILE("f32", false, 64, 64, 64, 2, 2, 4, true, 4, kElement, "_e"),
};
const TileEntry kTilesBf16[] = {
    CONV2D_PATCH_TILE("bf16", true, 256, 256, 4, 2, 512, false, 1),
    CONV2D_PATCH_TILE("bf16", true, 256, 256, 2, 2, 512, false, 1),
    CONV2D_PATCH_TILE("bf16", true, 256, 128, 4, 2, 512, false, 1),
    CONV2D_PATCH_TILE("bf16", true, 224, 256, 1, 4, 512, false, 1),
    CONV2D_PATCH_TILE_M16("bf16", true, 224, 128, 2, 2, 384, 2),
    CONV2D_PATCH_TILE_M16B("bf16", true, 224, 128, 2, 2, 384, 2, 16),
    CONV2D_PATCH_TILE_M16N("bf16", true, 224, 128, 2, 2, 384, 2, 0, ""),
    CONV2D_PATCH_TILE_M16N("bf16", true, 224, 128, 2, 2, 384, 2, 16, "_b16"),
    CONV2D_PATCH_TILE_B("bf16", true, 256, 256, 4, 2, 512, false, 1, 16),
    CONV2D_PATCH_TILE_B("bf16", true, 256, 128, 4, 2, 512, false, 1, 16),
    CONV2D_PATCH_TILE_B("bf16", true, 256, 64, 4, 1, 512, false, 2, 16),
    CONV2D_PATCH_TILE_B("bf16", true, 128, 64, 2, 2, 256, false, 3, 16),
    CONV2D_PATCH_TILE_B("bf16", true, 128, 128, 2, 2, 256, false, 2, 16),
    CONV2D_PATCH_TILE_BN("bf16", true, 256, 64, 4, 1, 512, false, 2, 16),
    CONV2D_PATCH_TILE_BN("bf16", true, 128, 64, 2, 2, 256, false, 3, 16),
    CONV2D_PATCH_TILE_BN("bf16", true, 128, 128, 2, 2, 256, false, 2, 16),
    CONV2D_DMA_TILE("bf16", true, 256, 256, 64, 4, 2, 4, false, 1, kUniform, ""),
    CONV2D_DMA_TILE("bf16", true, 256, 256, 128, 4, 2, 2, false, 1, kUniform, ""),
    CONV2D_DMA_TILE("bf16", true, 256, 128, 64, 4, 2, 4, false, 1, kUniform, ""),
    CONV2D_DMA_TILE("bf16", true, 256, 128, 64, 4, 2, 3, false, 2, kUniform, ""),
    CONV2D_DMA_TILE("bf16", true, 128, 128, 64, 2, 2, 4, false, 2, kUniform, ""),
    CONV2D_DMA_TILE("bf16", true, 128, 64, 64, 2, 2, 4, false, 3, kUniform, ""),
    CONV2D_DMA_TILE("bf16", true, 64, 64, 64, 2, 2, 4, false, 4, kUniform, ""),
    CONV2D_DMA_TILE("bf16", true, 64, 64, 64, 2, 2, 3, false, 6, kUniform, ""),
    CONV2D_DMA_TILE("bf16", true, 64, 64, 128, 2, 2, 4, false, 2, kUniform, ""),
    CONV2D_DMA_TILE_N("bf16", true, 256, 128, 64, 4, 2, 3, false, 2),
    CONV2D_DMA_TILE_N("bf16", true, 128, 128, 64, 2, 2, 4, false, 2),
    CONV2D_DMA_TILE_N("bf16", true, 128, 64, 64, 2, 2, 4, false, 3),
    CONV2D_DMA_TILE_N("bf16", true, 64, 64, 64, 2, 2, 4, false, 4),
    CONV2D_DMA_TILE_N("bf16", true, 64, 64, 64, 2, 2, 3, false, 6),
    CONV2D_DMA_TILE_N("bf16", true, 64, 64, 128, 2, 2, 4, false, 2),
    CONV2D_DMA_TILE("bf16", true, 128, 128, 64, 2, 2, 4, false, 2, kVector, "_g"),
    CONV2D_DMA_TILE("bf16", true, 128, 64, 64, 2, 2, 4, false, 3, kVector, "_g"),
    CONV2D_DMA_TILE("bf16", true, 64, 64, 64, 2, 2, 4, false, 4, kVector, "_g"),
};
constexpr int kNumF32 = sizeof(kTilesF32) / sizeof(kTilesF32[0]);
constexpr int kNumBf16 = sizeof(kTilesBf16) / sizeof(kTilesBf16[0]);

const TileEntry& entry(int bf16, int tile) { return bf16 ? kTilesBf16[tile] : kTilesF32[tile]; }

}  // namespace dma
using namespace dma;

int igemm_dma_num_tiles(int bf16) { return bf16 ? kNumBf16 : kNumF32; }
const char* igemm_dma_tile_name(int bf16, int tile) { return entry(bf16, tile).name; }
void igemm_dma_tile_shape(int bf16, int tile, int* bm, int* bn, int* bk) {
  const TileEntry& t = entry(bf16, tile);
  *bm = t.bm;
  *bn = t.bn;
  *bk = t.bk;
}
int igemm_dma_tile_occupancy(int bf16, int tile) { return entry(bf16, tile).occ; }
int igemm_dma_tile_addressing(int bf16, int tile) { return entry(bf16, tile).addr; }
bool igemm_dma_tile_fits(const Problem& p, int bf16, int tile) {
  const TileEntry& t = entry(bf16, tile);
  return t.fits == nullptr || t.fits(p);
}
bool igemm_dma_tile_has_wino(int bf16, int tile) { return entry(bf16, tile).wino != nullptr; }
bool igemm_dma_tile_pools(int bf16, int tile) { return entry(bf16, tile).pools; }
bool igemm_dma_tile_native(int bf16, int tile) { return entry(bf16, tile).native; }
bool igemm_dma_tile_splits_channels(int bf16, int tile) {
  return entry(bf16, tile).splits_channels;
}
size_t igemm_dma_packed_filter_bytes(const Problem& p, int bf16, int tile) {
  const TileEntry& t = entry(bf16, tile);
  if (t.native)  // a plain copy of the filter
    return (static_cast<size_t>(p.Kg) * p.K * (bf16 ? 2 : 4) + 255) / 256 * 256;
  const size_t kg_p = static_cast<size_t>((p.Kg + t.bk - 1) / t.bk) * t.bk;
  return (kg_p * p.K * (bf16 ? 2 : 4) + 255) / 256 * 256 * (p.batches > 1 ? p.batches : 1);
}
hipError_t igemm_dma_pack_filter(const Problem& p, int bf16, int tile, void* packed,
                                 hipStream_t stream) {
  const TileEntry& t = entry(bf16, tile);
  if (t.native)
    return hipMemcpyAsync(packed, p.filt, static_cast<size_t>(p.Kg) * p.K * (bf16 ? 2 : 4),
                          hipMemcpyDeviceToDevice, stream);
  const int Kg_p = (p.Kg + t.bk - 1) / t.bk * t.bk;
  // uniform and patch tiles walk the reduction channel block by channel block
  const int block = (t.addr == kUniform || t.addr == 3) ? t.bk : 0;
  // (a batched problem: one packed filter per batch, one after the other)
  const int batches = p.batches > 1 ? p.batches : 1;
  const long long bt_stride = static_cast<long long>(
      igemm_dma_packed_filter_bytes(p, bf16, tile) / batches / (bf16 ? 2 : 4));
  dim3 rgrid(Kg_p / t.bk, (p.K + 63) / 64, batches);
  if (bf16)
    hipLaunchKernelGGL((repack_filter_kernel<unsigned short>), rgrid, dim3(256), 0, stream,
                       static_cast<const unsigned short*>(p.filt),
                       static_cast<unsigned short*>(packed), p.Kg, p.K, Kg_p, p.C, p.R * p.S,
                       block, t.bk, p.filt_stride, bt_stride);
  else
    hipLaunchKernelGGL((repack_filter_kernel<float>), rgrid, dim3(256), 0, stream,
                       static_cast<const float*>(p.filt), static_cast<float*>(packed), p.Kg, p.K,
                       Kg_p, p.C, p.R * p.S, block, t.bk, p.filt_stride, bt_stride);
  return hipGetLastError();
}
hipError_t launch_igemm_dma_wino(const Problem& p, int bf16, int tile, hipStream_t stream) {
  const TileEntry& t = entry(bf16, tile);
  return t.wino ? t.wino(p, stream) : hipErrorInvalidValue;
}
size_t igemm_dma_workspace_bytes(const Problem& p, int bf16, int tile, int splits) {
  return entry(bf16, tile).ws(p, splits);
}
hipError_t launch_igemm_dma(const Problem& p, int bf16, int tile, int splits, hipStream_t stream) {
  return entry(bf16, tile).fn(p, splits, stream);
}
void igemm_dma_split_reduce_separate(bool on) {
  split_reduce_separate.store(on ? 1 : 0, std::memory_order_relaxed);
}

}  // namespace conv2d
