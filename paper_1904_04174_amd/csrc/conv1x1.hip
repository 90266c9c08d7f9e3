// Streaming kernel for window-1 (1x1) convolutions, any stride, for gfx950.
//
// The paper's Figure 1 shows the layers with a window of 1 as a regime of
// their own (its tiled kernel wins them); here they are the memory-bound end
// of the workload: out[m][k] = sum_c in[pixel(m)][c] * filt[c][k] with a
// short reduction (C = 64 ... 256) and an output that is most of the bytes.
// The generic gather tiles spend such a layer's time on everything but the
// products: a new workgroup per 64x64 tile that works out its addresses,
// fetches its filter slices again, waits for the first loads and ends in a
// burst of stores.  This kernel keeps what does not change and streams the
// rest:
//
//  * Persistent workgroups.  A workgroup owns a slab of BN features and
//    walks the tiles of 64 output pixels with the stride of its slab's
//    workgroup count.
//  * The filter slab [C][BN] stays in LDS for the whole launch, as it lies in
//    memory (one row per channel, features contiguous): loaded once per
//    workgroup, no repacked copy, no workspace.  The B fragments are read
//    with single-value reads (fp32: lane = feature, the four MFMAs of a step
//    take four rows) or transposing reads (bf16: ds_read_b64_tr_b16, see
//    igemm_dma.hip), with the same bank swizzles as the native gather tiles.
//  * The input rows go through a ring of NST (6 or 12) stages of 64 pixels x 64 bytes,
//    filled by direct global->LDS loads that run NST-1 slices ahead, across
//    tile boundaries.
//  * Loads and stores are issued by different wavefronts.  A wavefront has
//    one counter for its outstanding loads and stores, so a wavefront that
//    stores a tile and then waits for a load waits for its stores as well: a
//    tile's store burst stalls the pipeline once per tile (measured on the
//    window-row gather kernel: the output's time at the store rate was not
//    hidden).  Here wavefront 4 of the workgroup only loads (and waits for
//    loads) and wavefronts 0-3 only multiply and store (and never wait for
//    memory): one barrier per slice hands a landed stage from the loader to
//    the multipliers and a drained stage back.
//
// Requirements (checked on the host): window 1x1, C a multiple of the slice
// (16 fp32 / 32 bf16 values), K a multiple of the 16-byte vector, 16-byte
// aligned pointers, the filter slab C x BN within 64 KiB, tensors below 2^31
// bytes.
#include "buffer_lds.h"
#include "conv2d_internal.h"

namespace conv2d {
namespace c1 {  // named namespace: the kernels' host stubs need external linkage

using namespace buf;

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kComputeUnits = 256;
constexpr int kBM = 64;            // output pixels per tile
constexpr int kRowB = 64;          // bytes of k per ring row = one slice
constexpr int kMaxSlabBytes = 64 * 1024;

__device__ __forceinline__ unsigned short to_bf16_bits(float x) {
  unsigned int u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<unsigned short>((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<unsigned short>(u >> 16);
}

template <bool BF16_, int BN_>
struct Tile {
  static constexpr bool BF16 = BF16_;
  static constexpr int BN = BN_;
  static constexpr int ES = BF16 ? 2 : 4;
  static constexpr int VEC = 16 / ES;
  static constexpr int BK = kRowB / ES;          // k per slice
  static constexpr int TN = BN / 64;             // 32-feature blocks per wave (2 x 2 waves)
  static constexpr int ROW_BYTES = BN * ES;      // a filter row (one channel) in LDS
  static constexpr int CH = BN / VEC;            // 16-byte chunks per filter row
  // ring stages: the bf16 layers are pure streams and want many slices in flight (12 against 8:
  // 23 against 27 us on a 56x56x64 -> 256 layer at batch 32); the fp32 layers are bound by
  // their products and gain more from a fourth resident workgroup than from a deeper ring
  static constexpr int NST = BF16 ? 12 : 6;
  static constexpr int RING_BYTES = NST * kBM * kRowB;
  // bank swizzle of the filter rows (as the native gather tiles): bf16 moves pairs of 32-byte
  // pieces, fp32 swaps 128-byte halves
  static constexpr int swizzle(int k) {
    if (!BF16) return (k >> 2) & 1;
    return BN >= 128 ? ((k & 3) << 1) : (((k >> 1) & 1) << 1);
  }
};

// gridDim.x = workgroups; workgroup w owns slab w % slabs and the tiles (w / slabs) + i *
// (gridDim.x / slabs).  320 threads: wavefronts 0-3 multiply and store, wavefront 4 loads.
template <class T, bool OUT_BF16>
__global__ __launch_bounds__(320) void conv1x1_kernel(const Problem p, const int slabs,
                                                      const int tiles_m) {
  constexpr int BN = T::BN, ES = T::ES, VEC = T::VEC, BK = T::BK, TN = T::TN;
  constexpr int kNST = T::NST;
  extern __shared__ __align__(1024) unsigned char lds[];   // [ring | filter slab]
  unsigned char* const ring = lds;
  unsigned char* const slab = lds + T::RING_BYTES;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nsl = p.C / BK;                       // slices per tile
  const int n0 = (blockIdx.x % slabs) * BN;
  const int tile_first = blockIdx.x / slabs;
  const int tile_step = gridDim.x / slabs;
  const int my_tiles = tile_first < tiles_m ? (tiles_m - tile_first + tile_step - 1) / tile_step : 0;
  const int total = my_tiles * nsl;               // slices this workgroup walks
  if (total == 0) return;

  if (wave == 4) {
    // ------------------------------------------------------------- the loader wavefront
    // (its few instructions per slice go first: the multipliers' MFMAs would otherwise keep
    // it from issuing, and every multiplier then waits for it at the next barrier)
    __builtin_amdgcn_s_setprio(3);
    const uintx4 in_rsrc = make_rsrc(p.in, 1LL * p.N * p.H * p.W * p.C * ES);
    const uintx4 f_rsrc = make_rsrc(p.filt, 1LL * p.C * p.K * ES);
    const unsigned ring_base = __builtin_amdgcn_readfirstlane(static_cast<unsigned>(
        reinterpret_cast<size_t>(ring)));
    const unsigned slab_base = __builtin_amdgcn_readfirstlane(static_cast<unsigned>(
        reinterpret_cast<size_t>(slab)));
    // the filter slab: chunk q -> row k = q / CH, position q % CH holds the features
    // [VEC * c, VEC * c + VEC) of the slab with c = position ^ swizzle
    const int slab_chunks = p.C * T::CH;
    for (int q0 = 0; q0 < slab_chunks; q0 += 64) {
      const int q = q0 + lane;
      const int k = q / T::CH;
      const int c = (q % T::CH) ^ (T::swizzle(k) << (T::BF16 ? 1 : 3));
      const int n = n0 + VEC * c;
      const bool ok = q < slab_chunks && n + VEC <= p.K;
      dma16(f_rsrc, slab_base + q0 * 16, ok ? (k * p.K + n) * ES : kOutOfRange, 0);
    }
    // a stage: 64 pixels x 4 chunks; load number i of a slice covers rows 16 i ... 16 i + 15
    // (lane -> row 16 i + lane / 4, position lane % 4 holds chunk position ^ ((row >> 2) & 3))
    int row_off[4];        // byte offset of this lane's pixel in the current tile, or out of range
    auto tile_rows = [&](int tile) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = 16 * i + lane / 4;
        const int chunk = (lane % 4) ^ ((row >> 2) & 3);
        const int m = tile * kBM + row;
        int pix = m;   // stride 1: the output pixels are the input pixels
        if (p.sr != 1 || p.sc != 1) {
          const int mm = m < p.M ? m : 0;
          const int q = mm % p.Q, t = mm / p.Q;
          const int op = t % p.P, n = t / p.P;
          pix = (n * p.H + op * p.sr) * p.W + q * p.sc;
        }
        row_off[i] = m < p.M ? (pix * p.C + chunk * VEC) * ES : kOutOfRange;
      }
    };
    int ld_tile = tile_first, ld_slice = 0, ld_stage = 0;
    tile_rows(ld_tile);
    auto load_slice = [&]() {
      // (past the workgroup's last slice: out-of-range loads, zeros into a stage nobody reads)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        dma16(in_rsrc, ring_base + ld_stage * (kBM * kRowB) + i * 1024, row_off[i],
              ld_slice * kRowB);
      ld_stage = ld_stage + 1 == kNST ? 0 : ld_stage + 1;
      if (++ld_slice == nsl) {
        ld_slice = 0;
        ld_tile += tile_step;
        if (ld_tile < tiles_m) {
          tile_rows(ld_tile);
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i) row_off[i] = kOutOfRange;
        }
      }
    };
    for (int s = 0; s < kNST - 1; ++s) load_slice();
    for (int g = 0; g < total; ++g) {
      // slice g (and the filter slab, issued before it) has landed; slices g+1 ... g+NST-2
      // may still be in flight
      __builtin_amdgcn_s_waitcnt(vmcnt_imm((kNST - 2) * 4));
      __builtin_amdgcn_s_barrier();   // hands slice g over; every multiplier has left slice g-1
      load_slice();                   // slice g+NST-1 into the stage of slice g-1
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    return;
  }

  // ------------------------------------------------------------- the multiplying wavefronts
  const int wm = wave >> 1, wn = wave & 1;
  const int lr = lane & 31, lk = lane >> 5;
  // A fragment: row lr of the wave's 32 rows, chunk (2 kk + lk) ^ swizzle
  const unsigned char* a_frag = ring + (wm * 32 + lr) * kRowB;
  const int a_swz = (lr >> 2) & 3;
  // B fragment addressing inside the slab (without the slice's row offset)
  int b_row_off, b_piece_off[TN];
  if constexpr (T::BF16) {
    const int a = lane & 15, k = 8 * lk + a / 4;
    b_row_off = k * T::ROW_BYTES + 8 * (a % 4);
#pragma unroll
    for (int j = 0; j < TN; ++j)
      b_piece_off[j] = 32 * ((2 * (wn * TN + j) + ((lane >> 4) & 1)) ^ T::swizzle(k));
  } else {
    b_row_off = 4 * lk * T::ROW_BYTES + 4 * lr;
#pragma unroll
    for (int j = 0; j < TN; ++j) b_piece_off[j] = 128 * ((wn * TN + j) ^ lk);
  }
  float bias_col[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) bias_col[j] = bias_of(p.bias, n0 + (wn * TN + j) * 32 + lr, p.K);
#pragma unroll
  for (int j = 0; j < TN; ++j) asm volatile("" : "+v"(bias_col[j]));

  floatx16 acc[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;

  // Fragments of both steps of a slice: A from the slice's stage, B from the resident slab.
  struct Frags {
    uintx4 a[2];
    uintx4 b[2][TN];
  };
  auto read_frags = [&](Frags& f, int stage, int slice) {
    const unsigned char* a_src = a_frag + stage * (kBM * kRowB);
    const unsigned char* b_src = slab + slice * (BK * T::ROW_BYTES) + b_row_off;
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      f.a[kk] = *reinterpret_cast<const uintx4*>(a_src + (((2 * kk + lk) ^ a_swz) * 16));
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        if constexpr (T::BF16) {
          typedef __attribute__((address_space(3))) shortx4* lds_ptr;
          const unsigned char* src = b_src + b_piece_off[j] + 16 * kk * T::ROW_BYTES;
          const uintx2 lo = __builtin_bit_cast(
              uintx2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(src)));
          const uintx2 hi = __builtin_bit_cast(
              uintx2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(src + 4 * T::ROW_BYTES)));
          f.b[kk][j] = uintx4{lo.x, lo.y, hi.x, hi.y};
        } else {
          const unsigned char* src = b_src + b_piece_off[j] + 8 * kk * T::ROW_BYTES;
#pragma unroll
          for (int t = 0; t < 4; ++t)
            f.b[kk][j][t] = *reinterpret_cast<const unsigned*>(src + t * T::ROW_BYTES);
        }
      }
    }
  };
  auto multiply = [&](const Frags& f) {
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        if constexpr (T::BF16) {
          acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f.a[kk]),
                                                           __builtin_bit_cast(bf16x8, f.b[kk][j]),
                                                           acc[j], 0, 0, 0);
        } else {
          // (the four MFMAs of a block back to back, pinned: a dependent MFMA that follows its
          // predecessor directly takes the accumulator from it without a bubble; the compiler's
          // own order interleaves the blocks)
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(f.a[kk][t]),
                                                          __uint_as_float(f.b[kk][j][t]), acc[j],
                                                          0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
  };
  // the tile's sums: lane l, register v -> row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32.
  // 32-bit element offsets from the output's base (the host checks the size), no test per row
  // except in the ragged last tile.
  auto store_tile = [&](int tile) {
    const int row0 = tile * kBM + wm * 32 + lk * 4;
    const bool whole = tile * kBM + kBM <= p.M;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = n0 + (wn * TN + j) * 32 + lr;
      const unsigned base = static_cast<unsigned>(row0) * static_cast<unsigned>(p.K) +
                            static_cast<unsigned>(col);
      if (col < p.K) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int dr = 8 * (v / 4) + (v % 4);
          if (whole || row0 + dr < p.M) {
            const unsigned idx = base + static_cast<unsigned>(dr) * static_cast<unsigned>(p.K);
            const float r = finish(acc[j][v], bias_col[j], p.relu);
            if (OUT_BF16)
              __builtin_nontemporal_store(to_bf16_bits(r),
                                          static_cast<unsigned short*>(p.out) + idx);
            else
              __builtin_nontemporal_store(r, static_cast<float*>(p.out) + idx);
          }
        }
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
    }
  };

  // Software pipeline: while the MFMAs of slice g run, the fragments of slice g+1 are read
  // (two fragment sets that swap roles from slice to slice).  Barrier number g hands slice g
  // over (the loader counts the same barriers); a multiplier reaches it only after its own
  // reads of slice g-1 have completed, so the loader may then refill that stage.
  int tile = tile_first, slice = 0, stage = 0;
  Frags f0, f1;
  __builtin_amdgcn_s_barrier();   // slice 0 (and the filter slab) is in LDS
  asm volatile("" ::: "memory");
  read_frags(f0, 0, 0);
  auto one_slice = [&](Frags& cur, Frags& nxt, int g) {
    const int stage_n = stage + 1 == kNST ? 0 : stage + 1;
    const int slice_n = slice + 1 == nsl ? 0 : slice + 1;
    if (g + 1 < total) {
      __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): this wave's reads of slice g are done
      __builtin_amdgcn_s_barrier();         // slice g+1 is in its stage
      asm volatile("" ::: "memory");
      read_frags(nxt, stage_n, slice_n);
    }
    multiply(cur);
    if (slice_n == 0) {
      store_tile(tile);
      tile += tile_step;
    }
    stage = stage_n;
    slice = slice_n;
  };
  for (int g = 0; g < total; g += 2) {
    one_slice(f0, f1, g);
    if (g + 1 < total) one_slice(f1, f0, g + 1);
  }
}

template <class T>
size_t lds_bytes(const Problem& p) {
  return T::RING_BYTES + static_cast<size_t>(p.C) * T::ROW_BYTES;
}

template <class T>
bool supports(const Problem& p) {
  if (p.R != 1 || p.S != 1 || p.in_bf16 != (T::BF16 ? 1 : 0)) return false;
  if (p.C % T::BK != 0 || p.K % T::VEC != 0) return false;
  if (static_cast<size_t>(p.C) * T::ROW_BYTES > static_cast<size_t>(kMaxSlabBytes)) return false;
  if (1LL * p.N * p.H * p.W * p.C * T::ES >= (1LL << 31)) return false;
  if (1LL * p.C * p.K * T::ES >= (1LL << 31)) return false;
  if (1LL * p.M * p.K >= (1LL << 30)) return false;   // 32-bit byte offsets into the output
  return p.batches <= 1;
}

template <class T, bool OUT_BF16>
hipError_t launch_one(const Problem& p, hipStream_t stream) {
  const int slabs = (p.K + T::BN - 1) / T::BN;
  const int tiles_m = (p.M + kBM - 1) / kBM;
  const size_t lds = lds_bytes<T>(p);
  // as many workgroups as fit at once (by LDS; five wavefronts each), a multiple of the slabs
  int per_cu = static_cast<int>((160 * 1024) / lds);
  if (per_cu > 4) per_cu = 4;
  if (per_cu < 1) return hipErrorInvalidValue;
  long long grid = 1LL * kComputeUnits * per_cu / slabs * slabs;
  if (grid < slabs) grid = slabs;
  if (grid > 1LL * tiles_m * slabs) grid = 1LL * tiles_m * slabs;
  auto kernel = conv1x1_kernel<T, OUT_BF16>;
  if (lds > 64 * 1024) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize,
                                             static_cast<int>(lds));
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kernel, dim3(static_cast<unsigned>(grid)), dim3(320), lds, stream, p, slabs,
                     tiles_m);
  return hipGetLastError();
}

template <class T>
hipError_t launch(const Problem& p, hipStream_t stream) {
  if (!supports<T>(p)) return hipErrorInvalidValue;
  if (T::BF16 && p.out_bf16) return launch_one<T, T::BF16>(p, stream);
  return launch_one<T, false>(p, stream);
}

struct Entry {
  const char* name;
  int bf16, bn;
  bool (*supports)(const Problem&);
  hipError_t (*launch)(const Problem&, hipStream_t);
};
const Entry kEntries[] = {
    {"conv1x1_f32_64x64", 0, 64, &supports<Tile<false, 64>>, &launch<Tile<false, 64>>},
    {"conv1x1_f32_64x128", 0, 128, &supports<Tile<false, 128>>, &launch<Tile<false, 128>>},
    {"conv1x1_bf16_64x64", 1, 64, &supports<Tile<true, 64>>, &launch<Tile<true, 64>>},
    {"conv1x1_bf16_64x128", 1, 128, &supports<Tile<true, 128>>, &launch<Tile<true, 128>>},
};
constexpr int kNumEntries = sizeof(kEntries) / sizeof(kEntries[0]);

}  // namespace c1

int conv1x1_num_tiles() { return c1::kNumEntries; }
const char* conv1x1_tile_name(int tile) { return c1::kEntries[tile].name; }
int conv1x1_tile_bf16(int tile) { return c1::kEntries[tile].bf16; }
int conv1x1_tile_features(int tile) { return c1::kEntries[tile].bn; }
bool conv1x1_supports(const Problem& p, int tile) { return c1::kEntries[tile].supports(p); }
hipError_t launch_conv1x1(const Problem& p, int tile, hipStream_t stream) {
  return c1::kEntries[tile].launch(p, stream);
}

}  // namespace conv2d
