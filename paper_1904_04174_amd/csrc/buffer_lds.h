// Helpers shared by the kernels that load straight from a buffer into LDS (igemm_dma.hip,
// conv1x1.hip, winograd_lds.hip): raw buffer descriptors, the wavefront-wide global->LDS load,
// s_waitcnt immediates.  Internal, device side only.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>

namespace conv2d {
namespace buf {

typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

constexpr unsigned kRsrcFlags = 0x00020000u;  // raw buffer, 32-bit data format
// A voffset that is out of range for every descriptor here (tensors stay below 2^31 bytes): the
// load returns zeros and touches no memory.
constexpr int kOutOfRange = static_cast<int>(0x80000000u);

// s_waitcnt immediate that waits for vmcnt <= n only (gfx9 encoding: vmcnt in bits 3:0 and
// 15:14, expcnt 6:4 and lgkmcnt 11:8 left at "no wait").
constexpr int vmcnt_imm(int n) { return (n & 0xf) | ((n >> 4) << 14) | (0x7 << 4) | (0xf << 8); }
// the same, and all of this wave's LDS accesses complete as well (lgkmcnt == 0)
constexpr int vmcnt_lds_imm(int n) { return (n & 0xf) | ((n >> 4) << 14) | (0x7 << 4); }
constexpr int kWaitLds = 0xc07f;  // lgkmcnt(0) only

// Raw buffer descriptor (base moved back by shift_back bytes, stride 0, `bytes` records, flags)
// as four scalars.
__device__ __forceinline__ uintx4 make_rsrc(const void* base, int shift_back, long long bytes) {
  const size_t a = reinterpret_cast<size_t>(base) - static_cast<size_t>(shift_back);
  uintx4 r;
  r[0] = static_cast<unsigned>(a);
  r[1] = static_cast<unsigned>(a >> 32) & 0xffffu;
  r[2] = static_cast<unsigned>(bytes);
  r[3] = kRsrcFlags;
  return r;
}
__device__ __forceinline__ uintx4 make_rsrc(const void* base, long long bytes) {
  return make_rsrc(base, 0, bytes);
}

// LDS byte address of a pointer into a __shared__ array (the low half of its flat address).
__device__ __forceinline__ unsigned lds_address(const void* p) {
  return static_cast<unsigned>(reinterpret_cast<size_t>(p));
}

// One wavefront-wide 16-byte-per-lane load from a buffer straight into LDS: lane l's 16 bytes
// land at lds_base + 16 * l (lds_base is wave-uniform and goes through M0); an out-of-range
// voffset writes zeros.
__device__ __forceinline__ void dma16(const uintx4& rsrc, unsigned lds_base, int voffset,
                                      int soffset) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :
               : "s"(lds_base), "v"(voffset), "s"(rsrc), "s"(soffset)
               : "memory", "m0");
}

// The same with 4 bytes per lane: lane l's dword lands at lds_base + 4 * l.
__device__ __forceinline__ void dma4(const uintx4& rsrc, unsigned lds_base, int voffset,
                                     int soffset) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, %3 offen lds"
               :
               : "s"(lds_base), "v"(voffset), "s"(rsrc), "s"(soffset)
               : "memory", "m0");
}

}  // namespace buf
}  // namespace conv2d
