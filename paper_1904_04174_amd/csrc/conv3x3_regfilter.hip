// 3x3, stride-1 convolution of bf16 layers whose whole filter fits the registers of one compute
// unit (64 channels -> 64 features), for gfx950.
//
// Such a layer (the first 3x3 stages of the VGG- and ResNet-style networks that the paper's
// section 3 benchmarks) has a short reduction, Kg = 576, and a large image: per output pixel it
// reads 128 bytes, writes 256 (fp32) and multiplies for 576 x 64 products, which puts it on the
// memory side of the MFMA ridge.  The tiled kernels spend its time away from the memory system:
// a new workgroup per tile that fetches the filter again (72 KB for every 32 KB of input), a
// barrier and a filter slice from L2 for every 32 reduction indices, a burst of stores that
// nothing overlaps.  Here
//
//  * a workgroup (8 waves: 4 along the pixels x 2 along the features) is persistent and owns
//    the whole filter: every wave keeps the MFMA operands of its 32 features for all Kg
//    reduction indices in Kg / 4 = 144 registers per lane (steps of 16 indices x 4 registers),
//    read once from the HWCF filter as it lies (through LDS and transposing reads);
//  * a tile is a block of 16 x 16 output pixels of one image; its 18 x 18 x 64 input patch is
//    fetched by direct global->LDS loads, whole pixels per load instruction, into one of two
//    buffers (entry by entry, the 16-byte chunks XOR-swizzled so that a fragment read is
//    conflict free), the next tile's during the current tile's first steps: the loop reads only
//    the pixel operand from LDS;
//  * a finished pass's sums are held in registers and stored one by one during the next pass's
//    steps, at the rate the memory system takes them, never in a burst; the wait for the next
//    patch at a tile's end counts the stores issued since its loads and leaves them in flight;
//  * one barrier per tile;
//  * workgroup i runs on XCD i % 8; every XCD walks a contiguous range of tiles, its 32
//    workgroups on neighbouring blocks, so that the halo rows of a block come from its L2.
//
// Requirements (checked on the host): bf16 input and filter, 3x3 window, stride 1, C = K = 64,
// 16-byte aligned input and filter, tensors below 2^31 bytes.  No workspace.
#include "buffer_lds.h"
#include "conv2d_internal.h"

namespace conv2d {
namespace rf {  // named namespace: the kernels' host stubs need external linkage

using namespace buf;

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kXcds = 8;
constexpr int kComputeUnits = 256;
constexpr int kBW = 16;                  // columns of a tile
constexpr int kPW = kBW + 2;             // patch row width

// C channels = K features; BH rows of a tile; WM x WN waves (pixels x features).
template <int C_, int BH_, int WM_, int WN_, int PASSES_, int PF_>
struct Cfg {
  static constexpr int C = C_, K = 32 * WN_, BH = BH_, WM = WM_, WN = WN_;
  static constexpr int NW = WM * WN, NT = 64 * NW;
  static constexpr int PXW = BH * kBW / WM;          // pixels per wave
  static constexpr int TM = PXW / 32;                // 32-pixel MFMA blocks per wave
  // A wave works through a tile in PASSES passes over the reduction, TMU blocks each, so that
  // only TMU accumulator blocks (and as many held ones) are live beside the filter; the pixel
  // operand is read PF steps ahead of its MFMA.
  static constexpr int PASSES = PASSES_, TMU = TM / PASSES_, PF = PF_;
  static_assert(TM % PASSES_ == 0, "blocks over the passes");
  static constexpr int ENTRIES = (BH + 2) * kPW;     // patch entries (pixels) of 2 C bytes
  // A patch lies in LDS entry by entry, the 16-byte chunks of an entry XOR-swizzled by the
  // entry's index so that the fragment read of 16 consecutive entries at one channel chunk
  // spreads over all banks.  One load instruction moves 64 chunks = EPI whole entries: the
  // lanes of a pixel fetch one contiguous piece of memory (the first build of this kernel
  // kept planes of chunks, 64 pixels per load instruction, one 16-byte piece of each: eight
  // times the requests, and a fifth of the layer's time).
  static constexpr int ENTRY_BYTES = C * 2;
  static constexpr int CPE = ENTRY_BYTES / 16;       // chunks per entry (8 or 16)
  static constexpr int EPI = 64 / CPE;               // entries per load instruction
  static constexpr int LOADS = ((ENTRIES + EPI - 1) / EPI + NW - 1) / NW;   // per wave and tile
  static constexpr int PATCH_BYTES = LOADS * NW * 1024;
  static constexpr int swizzle_of_entry(int e) { return CPE == 8 ? (e >> 1) & 7 : e & 15; }
  static constexpr int CB = C / 16;                  // steps per tap
  static constexpr int STEPS = 9 * CB;               // steps of 16 reduction indices
  static constexpr int ROW_BYTES = K * 2;            // a filter row (one reduction index)
  // the filter goes through LDS in passes of PASS_ROWS rows (at most 96 KiB), behind the
  // first patch buffer
  static constexpr int KG = 9 * C;
  static constexpr int PASS_ROWS = KG * ROW_BYTES <= 96 * 1024 ? KG : 96 * 1024 / ROW_BYTES;
  static constexpr int FPASSES = KG / PASS_ROWS;
  static constexpr int PASS_BYTES = PASS_ROWS * ROW_BYTES;
  // two patch buffers; the staging copy overlies the second and what lies behind it
  static constexpr int LDS_BYTES = PATCH_BYTES + (PASS_BYTES > PATCH_BYTES ? PASS_BYTES : PATCH_BYTES);
  // bank swizzle of the staged filter rows, in 32-byte pieces (as the native gather tiles)
  static constexpr int swizzle(int k) { return K >= 128 ? ((k & 3) << 1) : (((k >> 1) & 1) << 1); }
  // bf16 output only where the registers allow it: with 128 channels the conversion's
  // temporaries on top of 288 operand, 64 accumulator and 64 held registers do not fit, and
  // the compiler moves the operand array to scratch memory
  static constexpr bool BF16_OUT = C <= 64;
  static_assert(PXW % 32 == 0 && (CPE == 8 || CPE == 16), "tile over the waves, entry sizes");
  static_assert(STEPS % LOADS == 0, "patch loads dealt evenly over the steps");
  static_assert(KG % PASS_ROWS == 0 && PASS_ROWS % 16 == 0 && PASS_BYTES % (NT * 16) == 0, "passes");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS");
};

__device__ __forceinline__ unsigned short to_bf16_bits(float x) {
  unsigned int u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<unsigned short>((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<unsigned short>(u >> 16);
}

// gridDim.x workgroups; `tiles` = N * blocks per image.
template <class T, bool OUT_BF16>
__global__ __launch_bounds__(T::NT) void conv3x3_regfilter_kernel(const Problem p, const int tiles,
                                                                  const int blocks_x,
                                                                  const int blocks_y) {
  constexpr int C = T::C, K = T::K, BH = T::BH, TM = T::TM;
  // [patch buffer 0 | 1]; the filter's staging copy overlies buffer 1 and beyond
  __shared__ __align__(1024) unsigned char lds[T::LDS_BYTES];
  unsigned char* const patch = lds;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / T::WN, wn = wave % T::WN;   // PXW pixels x 32 features per wave
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

  const uintx4 in_rsrc = make_rsrc(p.in, 1LL * p.N * p.H * p.W * C * 2);
  const unsigned lds_base = __builtin_amdgcn_readfirstlane(lds_address(patch));

  // ---- patch loader role: load j of this wave is instruction I = j * NW + wave of the patch:
  // lane l fetches chunk (l % CPE) ^ swizzle(e) of entry e = I * EPI + l / CPE, which is pixel
  // (e / 18, e % 18) of the input block
  // (worked out for every load: 12 more live registers do not fit beside the filter)
  auto entry_of = [&](int j, int& dy, int& dx, int& chunk) {
    const int e = (j * T::NW + wave) * T::EPI + lane / T::CPE;
    chunk = (lane % T::CPE) ^ T::swizzle_of_entry(e);
    dy = e < T::ENTRIES ? e / kPW : 1 << 20;   // past the patch: never inside an image
    dx = e % kPW;
  };
  // (image, top row, left column) of a tile's output block
  auto block_of = [&](int t, int& bn, int& bp, int& bq) {
    bq = (t % blocks_x) * kBW;
    const int r = t / blocks_x;
    bp = (r % blocks_y) * BH;
    bn = r / blocks_y;
  };
  // load number j of the patch of block (bn, bp, bq) into buffer `buf`
  auto load_chunk = [&](int buf, int j, int bn, int bp, int bq) {
    int dy, dx, chunk;
    entry_of(j, dy, dx, chunk);
    const int h = bp - p.pt + dy, w = bq - p.pl + dx;
    const bool ok = static_cast<unsigned>(h) < static_cast<unsigned>(p.H) &&
                    static_cast<unsigned>(w) < static_cast<unsigned>(p.W);
    const int voff = ok ? ((bn * p.H + h) * p.W + w) * T::ENTRY_BYTES + chunk * 16 : kOutOfRange;
    dma16(in_rsrc, lds_base + buf * T::PATCH_BYTES + (j * T::NW + wave) * 1024, voff, 0);
  };

  int bn, bp, bq;
  block_of(tile, bn, bp, bq);
#pragma unroll
  for (int i = 0; i < T::LOADS; ++i) load_chunk(0, i, bn, bp, bq);

  // ---- the filter operands of this wave: step s covers reduction indices 16 s + 8 lk + j,
  // j = 0 .. 7 (tap s / CB, channels 16 (s % CB) + 8 lk + j), of feature 32 wn + lr.  The
  // filter (Kg rows of K features) is copied to LDS as it lies, PASS_ROWS rows at a time,
  // behind the first patch buffer (over the second one, which nobody loads before the first
  // tile's loop), and every lane picks its values from there.
  uintx4 breg[T::STEPS];
  {
    typedef short shortx4 __attribute__((ext_vector_type(4)));
    typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));
    typedef __attribute__((address_space(3))) shortx4* lds_ptr;
    constexpr int CH = T::ROW_BYTES / 16;   // 16-byte chunks of a filter row
    const uintx4 f_rsrc = make_rsrc(p.filt, T::KG * T::ROW_BYTES);
    // ds_read_b64_tr_b16: the 16 lanes of a group hand in 4 rows x 16 features (lane a: row
    // a / 4, features 4 (a % 4) .. + 3) and lane i gets the 4 rows of feature i.  Lane l of
    // the MFMA operand (feature l % 32, reduction indices 8 (l / 32) .. + 7 of the step) reads
    // rows 8 lk + a / 4 and + 4 of the 16-feature piece 2 wn + (l / 16) % 2.
    const int a = lane & 15, k = 8 * lk + a / 4;
    const unsigned char* src = lds + T::PATCH_BYTES + k * T::ROW_BYTES + 8 * (a % 4) +
                               32 * ((2 * wn + ((lane >> 4) & 1)) ^ T::swizzle(k));
#pragma unroll
    for (int ps = 0; ps < T::FPASSES; ++ps) {
      // 16-byte chunk q of the staging copy: row q / CH of the pass, position q % CH, which
      // holds the 8 features of chunk (q % CH) ^ swizzle(row): the transposing reads then
      // spread over the banks
#pragma unroll
      for (int i = 0; i < T::PASS_BYTES / (T::NT * 16); ++i) {
        const int q = i * T::NT + tid;
        const int row = q / CH, c = (q % CH) ^ (T::swizzle(row) << 1);
        dma16(f_rsrc, lds_base + T::PATCH_BYTES + (i * T::NT + wave * 64) * 16,
              (ps * T::PASS_ROWS + row) * T::ROW_BYTES + c * 16, 0);
      }
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));   // this wave's part of the pass (and the patch)
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
#pragma unroll
      for (int s = 0; s < T::PASS_ROWS / 16; ++s) {
        const uintx2 lo = __builtin_bit_cast(
            uintx2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(src + 16 * s * T::ROW_BYTES)));
        const uintx2 hi = __builtin_bit_cast(
            uintx2,
            __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(src + (16 * s + 4) * T::ROW_BYTES)));
        breg[ps * (T::PASS_ROWS / 16) + s] = uintx4{lo.x, lo.y, hi.x, hi.y};
      }
      // every wave has its operands before the next pass, or the second patch, overwrites them
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_waitcnt(kWaitLds);
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
    }
  }
  const float bias_col = bias_of(p.bias, wn * 32 + lr, K);

  // ---- pixel operand addressing: block b of the wave covers pixels PXW wm + 32 b + lr of the
  // tile (row-major in the BH x 16 block).  Step (tap, cb) reads chunk c = 2 cb + lk of entry
  // e = entry(pixel) + tap offset, which lies at e * ENTRY_BYTES + 16 (c ^ swizzle(e)); with
  // g = (e * ENTRY_BYTES | 16 (lk ^ swizzle(e))) + buffer, worked out once per tap, that is
  // g ^ 32 cb.
  constexpr int TMU = T::TMU, PF = T::PF, UNIT_STEPS = T::STEPS, TILE_STEPS = T::PASSES * T::STEPS;
  const int e00 = ((wm * T::PXW + lr) / kBW) * kPW + (wm * T::PXW + lr) % kBW;   // block 0
  auto tap_base = [&](int b, int tap, int buf_off) {
    // (a block is two rows of the tile on)
    const int e = e00 + b * 2 * kPW + (tap / 3) * kPW + tap % 3;
    return (e * T::ENTRY_BYTES | ((lk ^ T::swizzle_of_entry(e)) << 4)) + buf_off;
  };
  auto read_a = [&](int g, int cb) {
    return *reinterpret_cast<const uintx4*>(patch + (g ^ (cb << 5)));
  };

  // ---- the sums of a finished pass are kept in `hold` and stored during the next pass's
  // steps, one store every other step, instead of in one burst.  A compute unit's share of the
  // chip's store rate is about 8 bytes per clock; a tile's output at that rate takes nearly as
  // long as its products, so the two must overlap, and they only do if the store queue never
  // fills: a wave that issues a store into a full queue sits there, its MFMAs behind it.
  // Store k of a pass: block k / 16 of the pass, register v = k % 16 -> pixel 8 (v / 4) +
  // 4 (l / 32) + v % 4 of the block of 32, feature l % 32.  A buffer store with the tile's
  // origin in the descriptor, the store's pixel as the scalar offset and the lane's part (4 lk
  // pixels on, its feature) as the vector offset, which is out of range for a column past the
  // image.
  constexpr int OES = OUT_BF16 ? 2 : 4;
  floatx16 hold[TMU];
  __amdgpu_buffer_rsrc_t out_rsrc = __builtin_amdgcn_make_buffer_rsrc(p.out, 0, 0, kRsrcFlags);
  int held_rows = 0, held_cols = 0;   // rows (from the pass's first) and columns inside the image
  int held_row0 = 0;                  // first row of the held pass in its tile
  bool have_hold = false;
  const int lane_off = (4 * lk * K + wn * 32 + lr) * OES;
  auto hold_pass = [&](const floatx16 (&acc)[TMU], int pass, int n, int pr, int pq) {
#pragma unroll
    for (int i = 0; i < TMU; ++i) hold[i] = acc[i];
    const long long origin = (static_cast<long long>(n * p.P + pr) * p.Q + pq) * K * OES;
    const long long left = static_cast<long long>(p.M) * K * OES - origin;
    out_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        static_cast<unsigned char*>(p.out) + origin, 0,
        static_cast<int>(left < 0x7fffffffLL ? left : 0x7fffffffLL), kRsrcFlags);
    held_row0 = wm * (T::PXW / kBW) + pass * TMU * 2;
    held_rows = p.P - pr - held_row0;
    held_cols = p.Q - pq - 4 * lk;
    have_hold = true;
  };
  auto store_held = [&](int k) {
    const int i = k / 16, v = k % 16;
    const int r = i * 32 + 8 * (v / 4) + (v % 4);   // pixel of the pass's, without 4 lk
    const int py = r / kBW, px = r % kBW;
    // (always issued: a pixel outside the image has an out-of-range vector offset, and a scalar
    // offset of zero so that the sum of the two is out of range as well)
    const bool row_ok = py < held_rows;
    const int voff = (row_ok && px < held_cols) ? lane_off : kOutOfRange;
    const int soff = row_ok ? ((held_row0 + py) * p.Q + px) * K * OES : 0;
    const float x = finish(hold[i][v], bias_col, p.relu);
    if (OUT_BF16)
      __builtin_amdgcn_raw_buffer_store_b16(to_bf16_bits(x), out_rsrc, voff, soff, 2 /* nt */);
    else
      __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(x), out_rsrc, voff, soff, 2);
  };
  constexpr int STORES = TMU * 16;
  constexpr int STORE_EVERY = UNIT_STEPS / STORES >= 2 ? 2 : 1;
  static_assert(T::LOADS + STORES <= UNIT_STEPS && STORES * STORE_EVERY <= UNIT_STEPS,
                "loads, then stores, over a pass");

  // Two patch buffers.  During a tile's first steps the wave issues its loads of the next
  // tile's patch (one per step), then the held stores, one per step or every other step; at the
  // tile's end it waits until no more operations are outstanding than it has issued since the
  // last of those loads (a wave's memory operations retire in the order issued, loads and
  // stores alike: what the compiler's own wait counts rely on), so the patch has landed and the
  // stores just issued are not waited for.  Every store of a tile is issued, those outside the
  // image with an out-of-range offset, so that the count is known.
  constexpr int AFTER_LOADS = T::PASSES * STORES < 63 ? T::PASSES * STORES : 63;
  constexpr int AFTER_LOADS_FIRST = (T::PASSES - 1) * STORES < 63 ? (T::PASSES - 1) * STORES : 63;
  int next_tile = tile + tile_step;
  int buf = 0;
  for (;;) {
    const bool has_next = next_tile < range_end;
    int nn = 0, np = 0, nq = 0;
    if (has_next) block_of(next_tile, nn, np, nq);
    const int buf_off = buf * T::PATCH_BYTES;
    const bool first_tile = !have_hold;

    floatx16 acc[TMU];
#pragma unroll
    for (int i = 0; i < TMU; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;

    // Step S of the tile: pass S / UNIT_STEPS, reduction step S % UNIT_STEPS.  The operand of
    // step S + PF is read right after the MFMA of step S on the same block, pinned there by
    // scheduling fences: the read is issued while the matrix core is busy and has PF steps to
    // arrive.  (Left to itself the compiler reads every operand right before its MFMA,
    // through one register quadruple, and each MFMA waits for LDS.)
    int g[TMU];
    uintx4 af[PF + 1][TMU];
#pragma unroll
    for (int S = 0; S < PF; ++S) {
#pragma unroll
      for (int i = 0; i < TMU; ++i) {
        if (S % T::CB == 0) g[i] = tap_base(i, S / T::CB, buf_off);
        af[S][i] = read_a(g[i], S % T::CB);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma clang loop unroll(full)
    for (int S = 0; S < TILE_STEPS; ++S) {
      const int pass = S / UNIT_STEPS, s = S % UNIT_STEPS;
      const int Sn = S + PF, pass_n = Sn / UNIT_STEPS, s_n = Sn % UNIT_STEPS;
#pragma unroll
      for (int i = 0; i < TMU; ++i) {
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            __builtin_bit_cast(bf16x8, af[S % (PF + 1)][i]), __builtin_bit_cast(bf16x8, breg[s]),
            acc[i], 0, 0, 0);
        if (Sn < TILE_STEPS) {
          if (s_n % T::CB == 0) g[i] = tap_base(pass_n * TMU + i, s_n / T::CB, buf_off);
          af[Sn % (PF + 1)][i] = read_a(g[i], s_n % T::CB);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      if (S < T::LOADS) {
        // (every wave passed the barrier before this tile, so nobody still reads that buffer)
        if (has_next) load_chunk(buf ^ 1, S, nn, np, nq);
        __builtin_amdgcn_sched_barrier(0);
      }
      const int ks = pass == 0 ? s - T::LOADS : (s % STORE_EVERY == 0 ? s / STORE_EVERY : -1);
      if (ks >= 0 && ks < STORES) {
        if (have_hold) store_held(ks);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (s == UNIT_STEPS - 1) {
        if (pass == T::PASSES - 1 && has_next) {
          if (first_tile)
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(AFTER_LOADS_FIRST));
          else
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(AFTER_LOADS));
        }
        hold_pass(acc, pass, bn, bp, bq);
#pragma unroll
        for (int i = 0; i < TMU; ++i)
#pragma unroll
          for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if (!has_next) break;
    __builtin_amdgcn_s_barrier();   // the next patch is whole; this tile's buffer is free
    asm volatile("" ::: "memory");
    tile = next_tile;
    next_tile = tile + tile_step;
    bn = nn;
    bp = np;
    bq = nq;
    buf ^= 1;
  }
  // the last pass's sums
#pragma unroll
  for (int k = 0; k < STORES; ++k) store_held(k);
}

template <class T>
bool supports(const Problem& p) {
  if (!p.in_bf16 || p.R != 3 || p.S != 3 || p.sr != 1 || p.sc != 1) return false;
  if (p.C != T::C || p.K != T::K || p.batches > 1 || p.pool) return false;
  if (!T::BF16_OUT && p.out_bf16) return false;
  if (1LL * p.N * p.H * p.W * T::C * 2 >= (1LL << 31)) return false;
  if (1LL * p.M * T::K >= (1LL << 31)) return false;
  return true;
}

template <class T, bool OUT_BF16>
hipError_t launch_one(const Problem& p, hipStream_t stream) {
  const int blocks_x = (p.Q + kBW - 1) / kBW, blocks_y = (p.P + T::BH - 1) / T::BH;
  const long long tiles = 1LL * p.N * blocks_x * blocks_y;
  if (tiles >= (1LL << 31)) return hipErrorInvalidValue;
  const int grid = tiles < kComputeUnits ? static_cast<int>(tiles) : kComputeUnits;
  hipLaunchKernelGGL((conv3x3_regfilter_kernel<T, OUT_BF16>), dim3(grid), dim3(T::NT), 0, stream,
                     p, static_cast<int>(tiles), blocks_x, blocks_y);
  return hipGetLastError();
}

template <class T>
hipError_t launch(const Problem& p, hipStream_t stream) {
  if (!supports<T>(p)) return hipErrorInvalidValue;
  if constexpr (T::BF16_OUT) {
    if (p.out_bf16) return launch_one<T, true>(p, stream);
  }
  return launch_one<T, false>(p, stream);
}

struct Entry {
  const char* name;
  int rows;   // rows of a tile (16 columns)
  bool (*supports)(const Problem&);
  hipError_t (*launch)(const Problem&, hipStream_t);
};
using Cfg64 = Cfg<64, 16, 4, 2, 2, 1>;
// (Cfg<128, 8, 1, 4, 2, 2>, 128 channels -> 128 features on 8 x 16 tiles with 4 waves of 288
// operand registers each, passes the same tests and is not compiled in: a 112x112 layer at batch
// 16 takes it 67-68 us against 56-59 us on the 16-row patch tile, 30 us with its stores and loads
// switched off: four waves do not keep enough stores in flight to fill the chip's store rate.)
const Entry kEntries[] = {
    {"conv3x3_bf16_regfilter_256x64", 16, &supports<Cfg64>, &launch<Cfg64>},
};
constexpr int kNumEntries = sizeof(kEntries) / sizeof(kEntries[0]);

}  // namespace rf

int conv3x3_regfilter_num_tiles() { return rf::kNumEntries; }
const char* conv3x3_regfilter_tile_name(int tile) { return rf::kEntries[tile].name; }
int conv3x3_regfilter_tile_rows(int tile) { return rf::kEntries[tile].rows; }
bool conv3x3_regfilter_supports(const Problem& p, int tile) { return rf::kEntries[tile].supports(p); }
hipError_t launch_conv3x3_regfilter(const Problem& p, int tile, hipStream_t stream) {
  return rf::kEntries[tile].launch(p, stream);
}

}  // namespace conv2d
