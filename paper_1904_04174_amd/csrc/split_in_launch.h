// The sum of a split reduction's partial tiles inside the convolution launch, shared by the
// implicit-GEMM kernels (igemm_dma.hip, igemm.hip).  Internal, device side only.
//
// Every workgroup of an output tile writes its partial tile ([split][M][K] fp32 planes, with
// device-scope coherent stores: split_store) and then calls split_reduce_in_launch: it counts
// itself in on the tile's counter after its stores have been acknowledged; the workgroup that
// finds all others counted adds the tile's partial sums, applies the epilogue and stores the
// output.  Nobody waits for anybody.  The workgroups of a tile run on different XCDs, whose L2
// caches do not see each other's lines: the partial sums are written and read with device-scope
// coherent accesses (sc1).  The counter is left at zero for the next launch.
#pragma once

#include <hip/hip_runtime.h>

#include "conv2d_internal.h"

namespace conv2d {
namespace splitk {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));

constexpr int kOutOfRange = static_cast<int>(0x80000000u);
constexpr unsigned kRsrcFlags = 0x00020000u;

__device__ __forceinline__ unsigned short bf16_bits(float x) {
  unsigned int u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<unsigned short>((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<unsigned short>(u >> 16);
}

// One value of a partial tile.
__device__ __forceinline__ void split_store(float* dst, float value) {
  __hip_atomic_store(dst, value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Tiles of up to 128x64 only (the host keeps larger ones on the second launch: one workgroup
// would read too much), so the registers used here stay under what the main loops need.
// `scratch_word`: a word of LDS that no wave uses any more; `ahead`: splits whose loads are in
// flight together.  Returns after the tile's output is stored, or at once in every workgroup
// but the last to arrive.
template <int BM, int BN, int NT, bool OUT_BF16, int AHEAD>
__device__ __forceinline__ void split_reduce_in_launch(const Problem& p, const float* partial,
                                                       unsigned* counter, unsigned nsplits,
                                                       int reduce_groups, int m0, int n0,
                                                       unsigned* scratch_word, int tid) {
  // s_waitcnt vmcnt(0): this wave's partial sums (and any loads still in flight)
  __builtin_amdgcn_s_waitcnt((0x7 << 4) | (0xf << 8));
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  if (tid == 0) {
    const unsigned before =
        __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (before == nsplits - 1)
      __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *scratch_word = before;
  }
  __syncthreads();
  if (*scratch_word != nsplits - 1) return;

  if constexpr (BM * BN <= 128 * 64) {
  // 16-byte pieces of the tile, row by row: piece f = row * (BN / 4) + column quad
  constexpr int PER = BM * BN / 4 / NT;  // pieces per thread
  static_assert(BM * BN / 4 % NT == 0 && PER >= 1, "tile pieces over the threads");
  const __amdgpu_buffer_rsrc_t part_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<float*>(partial), 0,
      static_cast<int>(nsplits * static_cast<unsigned>(p.M) * p.K * 4u), kRsrcFlags);
  const int plane_bytes = p.M * p.K * 4;
  int piece_off[PER];
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    const int f = e * NT + tid;
    const int row = m0 + f / (BN / 4), col = n0 + 4 * (f % (BN / 4));
    piece_off[e] = (row < p.M && col < p.K) ? (row * p.K + col) * 4 : kOutOfRange;
  }
  // The order of the additions is split_reduce_kernel's, so that both ways give the same bits:
  // `reduce_groups` sums, group g over the splits g, g + groups, ... from zero, then group 0's
  // sum + group 1's + ...  The splits are visited in that order, AHEAD loads at a time.
  floatx4 acc[PER], total[PER];
#pragma unroll
  for (int e = 0; e < PER; ++e) acc[e] = total[e] = floatx4{0.f, 0.f, 0.f, 0.f};
  bool have_total = false;
  int next_group = 0, next_split = 0;
  for (unsigned done = 0; done < nsplits; done += AHEAD) {
    uintx4 got[AHEAD][PER];
    unsigned starts_group = 0;
#pragma unroll
    for (int a = 0; a < AHEAD; ++a) {
      // (a visit past the last, like a piece outside the output, reads out of range: zeros;
      // the range check covers the vector offset only, so the split's plane is part of it)
      const bool live = done + a < nsplits;
      const int plane = next_split * plane_bytes;
      if (live) {
        if (next_split == next_group) starts_group |= 1u << a;
        next_split += reduce_groups;
        if (next_split >= static_cast<int>(nsplits)) next_split = ++next_group;
      }
#pragma unroll
      for (int e = 0; e < PER; ++e)
        got[a][e] = __builtin_amdgcn_raw_buffer_load_b128(
            part_rsrc, (live && piece_off[e] != kOutOfRange) ? piece_off[e] + plane : kOutOfRange,
            0, 16 /* sc1 */);
    }
#pragma unroll
    for (int a = 0; a < AHEAD; ++a) {
      if (done + a >= nsplits) break;
      if (((starts_group >> a) & 1u) && done + a > 0) {
        // a group's sum is complete: fold it into the total
#pragma unroll
        for (int e = 0; e < PER; ++e) {
          total[e] = have_total ? total[e] + acc[e] : acc[e];
          acc[e] = floatx4{0.f, 0.f, 0.f, 0.f};
        }
        have_total = true;
      }
#pragma unroll
      for (int e = 0; e < PER; ++e)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[e][c] += __uint_as_float(got[a][e][c]);
    }
  }
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    if (piece_off[e] == kOutOfRange) continue;
    const floatx4 sum = have_total ? total[e] + acc[e] : acc[e];
    const int f = e * NT + tid;
    const int col = n0 + 4 * (f % (BN / 4));
    const size_t idx = static_cast<size_t>(piece_off[e]) / 4;
    floatx4 r;
#pragma unroll
    for (int c = 0; c < 4; ++c) r[c] = finish(sum[c], bias_of(p.bias, col + c, p.K), p.relu);
    // (non-temporal: nothing in the call reads the output back)
    if (OUT_BF16) {
      uintx2 packed;
      packed.x = bf16_bits(r[0]) | (static_cast<unsigned>(bf16_bits(r[1])) << 16);
      packed.y = bf16_bits(r[2]) | (static_cast<unsigned>(bf16_bits(r[3])) << 16);
      __builtin_nontemporal_store(
          packed, reinterpret_cast<uintx2*>(static_cast<unsigned short*>(p.out) + idx));
    } else {
      __builtin_nontemporal_store(r, reinterpret_cast<floatx4*>(static_cast<float*>(p.out) + idx));
    }
  }
  }  // tiles of up to 128x64
}

// The host's rule for using it: whole 16-byte pieces of output rows (K a multiple of 4, an
// aligned output), partial sums within 2^31 bytes, and little enough to add that one workgroup
// does it faster than a second launch (it reads at ~36 GB/s: up to 96 KiB per tile).
inline bool split_in_launch_pays(const Problem& p, int bm, int bn, int splits, bool out_bf16) {
  return splits > 1 && p.K % 4 == 0 && bm * bn <= 128 * 64 &&
         static_cast<long long>(splits) * bm * bn * 4 <= 96 * 1024 &&
         reinterpret_cast<uintptr_t>(p.out) % (out_bf16 ? 8 : 16) == 0 &&
         static_cast<unsigned long long>(splits) * p.M * p.K * 4ull < (1ull << 31);
}

}  // namespace splitk
}  // namespace conv2d
