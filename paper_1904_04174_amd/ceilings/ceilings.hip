// Reachable ceilings of one MI355X, measured with loops that do nothing else:
// matrix-core issue from registers, LDS fragment reads, and streaming copies.
// Not part of the convolution library and not part of its C ABI: a helper
// that bench.py --ceilings loads to report "achievable peak" next to the
// published peaks (the convolution kernels are priced against the published
// ones; these say how much of the gap any kernel could close at all).
//
// Every loop also reads the shader clock counter (clock64) and the
// constant-rate counter (wall_clock64) at its start and end in one lane, so
// per-clock figures use the clock the chip actually ran at during the loop,
// not the nominal 2.4 GHz.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct Clocks {
  unsigned long long core0, core1, wall0, wall1;
};

__device__ __forceinline__ void clocks_begin(Clocks* c) {
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    c->core0 = clock64();
    c->wall0 = wall_clock64();
  }
}
__device__ __forceinline__ void clocks_end(Clocks* c) {
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    c->core1 = clock64();
    c->wall1 = wall_clock64();
  }
}

// ---- matrix cores, operands and accumulators in registers
template <int KIND, int NACC>
__global__ __launch_bounds__(256) void mfma_loop(float* out, int iters, Clocks* c) {
  clocks_begin(c);
  float s = 0.f;
  if constexpr (KIND == 0) {
    floatx16 acc[NACC];
    for (int i = 0; i < NACC; ++i)
      for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    const float a = 1.f + threadIdx.x, b = 0.5f;
    for (int it = 0; it < iters; ++it)
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int i = 0; i < NACC; ++i)
          acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[i], 0, 0, 0);
    for (int i = 0; i < NACC; ++i)
      for (int v = 0; v < 16; ++v) s += acc[i][v];
  } else if constexpr (KIND == 1) {
    floatx16 acc[NACC];
    for (int i = 0; i < NACC; ++i)
      for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    bf16x8 a, b;
    for (int v = 0; v < 8; ++v) {
      a[v] = (__bf16)(1.f + v);
      b[v] = (__bf16)(0.5f);
    }
    for (int it = 0; it < iters; ++it)
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int i = 0; i < NACC; ++i)
          acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
    for (int i = 0; i < NACC; ++i)
      for (int v = 0; v < 16; ++v) s += acc[i][v];
  } else if constexpr (KIND == 3) {
    floatx4 acc[NACC];
    for (int i = 0; i < NACC; ++i)
      for (int v = 0; v < 4; ++v) acc[i][v] = 0.f;
    const float a = 1.f + threadIdx.x, b = 0.5f;
    for (int it = 0; it < iters; ++it)
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int i = 0; i < NACC; ++i)
          acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[i], 0, 0, 0);
    for (int i = 0; i < NACC; ++i)
      for (int v = 0; v < 4; ++v) s += acc[i][v];
  } else {
    floatx4 acc[NACC];
    for (int i = 0; i < NACC; ++i)
      for (int v = 0; v < 4; ++v) acc[i][v] = 0.f;
    bf16x8 a, b;
    for (int v = 0; v < 8; ++v) {
      a[v] = (__bf16)(1.f + v);
      b[v] = (__bf16)(0.5f);
    }
    for (int it = 0; it < iters; ++it)
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int i = 0; i < NACC; ++i)
          acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[i], 0, 0, 0);
    for (int i = 0; i < NACC; ++i)
      for (int v = 0; v < 4; ++v) s += acc[i][v];
  }
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
  clocks_end(c);
}

// ---- LDS reads in the shapes the convolution kernels use.
//  KIND 0: 16 bytes per lane, rows of 64 bytes, 32 rows per lane half, chunk
//          XOR-swizzled with (row >> 1) & 3 (the fragment read of the
//          direct-to-LDS tiles)
//  KIND 1: 16 bytes per lane, 64 consecutive chunks (the patch planes)
//  KIND 2: 8 bytes per lane, consecutive
//  KIND 3: transposing 8-byte read (ds_read_b64_tr_b16), consecutive
template <int KIND>
__global__ __launch_bounds__(256) void lds_loop(unsigned* out, int iters, Clocks* c) {
  __shared__ __align__(16) unsigned char buf[65536];
  for (int i = threadIdx.x; i < 16384; i += 256) reinterpret_cast<unsigned*>(buf)[i] = i;
  __syncthreads();
  clocks_begin(c);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lr = lane & 31, lk = lane >> 5;
  unsigned acc = 0;
  if constexpr (KIND == 0 || KIND == 1) {
    const unsigned char* base =
        KIND == 0 ? buf + wave * 16384 + lr * 64 + ((lk ^ ((lr >> 1) & 3)) * 16)
                  : buf + wave * 16384 + lane * 16;
    for (int it = 0; it < iters; ++it) {
      uintx4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const uintx4*>(base + u * 2048);
      // (one consumer after all eight reads, so that they are all in flight together)
      asm volatile("" ::"v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]), "v"(v[4]), "v"(v[5]),
                   "v"(v[6]), "v"(v[7]));
      acc += v[0].x;
    }
  } else if constexpr (KIND == 2) {
    const unsigned char* base = buf + wave * 8192 + lane * 8;
    for (int it = 0; it < iters; ++it) {
      uintx2 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const uintx2*>(base + (u & 7) * 512);
      asm volatile("" ::"v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]), "v"(v[4]), "v"(v[5]),
                   "v"(v[6]), "v"(v[7]));
      acc += v[0].x;
    }
  } else {
    typedef __attribute__((address_space(3))) shortx4* lds_ptr;
    const unsigned char* base = buf + wave * 8192 + lane * 8;
    for (int it = 0; it < iters; ++it) {
      shortx4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        v[u] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(base + (u & 7) * 512));
      asm volatile("" ::"v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]), "v"(v[4]), "v"(v[5]),
                   "v"(v[6]), "v"(v[7]));
      acc += static_cast<unsigned>(v[0].x);
    }
  }
  out[blockIdx.x * 256 + threadIdx.x] = acc;
  clocks_end(c);
}

// 16-byte reads at host-given per-lane byte offsets (within 2 KiB), eight in
// flight per wave: to compare fragment-read address patterns.
__global__ __launch_bounds__(256) void lds_pattern_loop(unsigned* out, int iters, Clocks* c,
                                                        const int* lane_offset) {
  __shared__ __align__(16) unsigned char buf[65536];
  for (int i = threadIdx.x; i < 16384; i += 256) reinterpret_cast<unsigned*>(buf)[i] = i;
  __syncthreads();
  clocks_begin(c);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const unsigned char* base = buf + wave * 16384 + lane_offset[lane];
  unsigned acc = 0;
  for (int it = 0; it < iters; ++it) {
    uintx4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const uintx4*>(base + u * 2048);
    asm volatile("" ::"v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]), "v"(v[4]), "v"(v[5]),
                 "v"(v[6]), "v"(v[7]));
    acc += v[0].x;
  }
  out[blockIdx.x * 256 + threadIdx.x] = acc;
  clocks_end(c);
}

// Transposing 8-byte reads (ds_read_b64_tr_b16) at host-given per-lane byte offsets, eight in
// flight per wave: offsets of read u are lane_offset[(u % 2) * 64 + lane] (the two reads that
// make up one MFMA operand) plus (u / 2) * `step` bytes.
__global__ __launch_bounds__(256) void lds_tr_pattern_loop(unsigned* out, int iters, Clocks* c,
                                                           const int* lane_offset, int step) {
  __shared__ __align__(16) unsigned char buf[65536];
  for (int i = threadIdx.x; i < 16384; i += 256) reinterpret_cast<unsigned*>(buf)[i] = i;
  __syncthreads();
  clocks_begin(c);
  typedef __attribute__((address_space(3))) shortx4* lds_ptr;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const unsigned char* b0 = buf + wave * 16384 + lane_offset[lane];
  const unsigned char* b1 = buf + wave * 16384 + lane_offset[64 + lane];
  unsigned acc = 0;
  for (int it = 0; it < iters; ++it) {
    shortx4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u)
      v[u] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)((u % 2 ? b1 : b0) + (u / 2) * step));
    asm volatile("" ::"v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]), "v"(v[4]), "v"(v[5]),
                 "v"(v[6]), "v"(v[7]));
    acc += static_cast<unsigned>(v[0].x);
  }
  out[blockIdx.x * 256 + threadIdx.x] = acc;
  clocks_end(c);
}

// ---- streaming: 16 bytes per lane, grid-stride
template <int KIND>  // 0 copy, 1 read, 2 write, 3 copy with non-temporal stores
__global__ __launch_bounds__(256) void stream_loop(const uintx4* __restrict__ a,
                                                   uintx4* __restrict__ b, size_t n) {
  uintx4 s = {1, 2, 3, 4};
  for (size_t i = blockIdx.x * 256ull + threadIdx.x; i < n; i += gridDim.x * 256ull) {
    if (KIND == 0) b[i] = a[i];
    if (KIND == 1) { const uintx4 v = a[i]; s.x += v.x; s.y ^= v.y; s.z += v.z; s.w ^= v.w; }
    if (KIND == 2) b[i] = s;
    if (KIND == 3) __builtin_nontemporal_store(a[i], b + i);
  }
  if (KIND == 1 && s.x == 0x12345678u && s.y == 0x9abcdef0u) b[0] = s;
}

struct Result {
  char name[64];
  double value;
  char unit[16];
};

struct Collector {
  Result* out;
  int max, n;
  void add(const char* name, double value, const char* unit) {
    if (n >= max) return;
    std::snprintf(out[n].name, sizeof(out[n].name), "%s", name);
    std::snprintf(out[n].unit, sizeof(out[n].unit), "%s", unit);
    out[n].value = value;
    ++n;
  }
};

#define CHECK(x)                          \
  do {                                    \
    if ((x) != hipSuccess) return -1;     \
  } while (0)

// MHz of the shader clock over the span the kernel recorded (wall counter: 100 MHz).
double core_mhz(const Clocks& c) {
  const double wall = static_cast<double>(c.wall1 - c.wall0);
  return wall > 0 ? static_cast<double>(c.core1 - c.core0) / wall * 100.0 : 0.0;
}

template <class Launch>
int timed(Launch launch, float* ms) {
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  CHECK(hipEventRecord(e0, nullptr));
  launch();
  CHECK(hipEventRecord(e1, nullptr));
  CHECK(hipEventSynchronize(e1));
  CHECK(hipEventElapsedTime(ms, e0, e1));
  CHECK(hipEventDestroy(e0));
  CHECK(hipEventDestroy(e1));
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace

extern "C" {

// Fills `out` (room for `max` records of {char name[64]; double value; char unit[16]})
// and returns the number written, or -1 on a runtime error.  Allocates and
// frees its own buffers on the current device; synchronises.
__attribute__((visibility("default"))) int conv2d_ceilings_measure(void* out, int max) {
  Collector col = {static_cast<Result*>(out), max, 0};
  int cus = 0;
  CHECK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, 0));
  col.add("compute_units", cus, "");
  float* fout = nullptr;
  Clocks* clk = nullptr;
  CHECK(hipMalloc(&fout, 4096 * 256 * sizeof(float)));
  CHECK(hipMalloc(&clk, sizeof(Clocks)));
  Clocks h;
  float ms;
  char name[64];

  // matrix cores: 1, 2 and 4 workgroups of 4 waves per compute unit (1, 2, 4 waves per SIMD);
  // the best of the three is the reachable rate
  const int iters = 2000;
  struct M { const char* name; double flop; void (*k)(float*, int, Clocks*); int nacc; };
  const M ms_[] = {
      {"mfma_f32_32x32x2 x4acc", 4096, mfma_loop<0, 4>, 4},
      {"mfma_bf16_32x32x16 x4acc", 32768, mfma_loop<1, 4>, 4},
      {"mfma_bf16_16x16x32 x8acc", 16384, mfma_loop<2, 8>, 8},
      {"mfma_f32_16x16x4 x8acc", 2048, mfma_loop<3, 8>, 8},
  };
  for (const M& m : ms_) {
    double best = 0.0, best_mhz = 0.0;
    int best_per_cu = 0;
    for (int per_cu = 1; per_cu <= 4; per_cu *= 2) {
      const int wgs = cus * per_cu;
      m.k<<<wgs, 256>>>(fout, 200, clk);  // warm-up: lets the clocks settle under this load
      CHECK(hipDeviceSynchronize());
      if (timed([&] { m.k<<<wgs, 256>>>(fout, iters, clk); }, &ms)) return -1;
      CHECK(hipMemcpy(&h, clk, sizeof(h), hipMemcpyDeviceToHost));
      const double rate = 1.0 * wgs * 4 * iters * 8 * m.nacc * m.flop / ms / 1e9;
      if (rate > best) { best = rate; best_mhz = core_mhz(h); best_per_cu = per_cu; }
    }
    col.add(m.name, best, "TFLOP/s");
    std::snprintf(name, sizeof(name), "%s clock", m.name);
    col.add(name, best_mhz, "MHz");
    std::snprintf(name, sizeof(name), "%s waves/SIMD", m.name);
    col.add(name, best_per_cu, "");
  }

  // LDS reads: 2 workgroups of 4 waves per compute unit (64 KiB each)
  struct L { const char* name; int bytes; void (*k)(unsigned*, int, Clocks*); };
  const L ls[] = {
      {"lds_read_b128 swizzled rows", 16, lds_loop<0>},
      {"lds_read_b128 consecutive", 16, lds_loop<1>},
      {"lds_read_b64 consecutive", 8, lds_loop<2>},
      {"lds_read_b64_tr_b16 consecutive", 8, lds_loop<3>},
  };
  for (const L& l : ls) {
    const int lw = cus * 2, li = 4000;
    l.k<<<lw, 256>>>(reinterpret_cast<unsigned*>(fout), 10, clk);
    CHECK(hipDeviceSynchronize());
    if (timed([&] { l.k<<<lw, 256>>>(reinterpret_cast<unsigned*>(fout), li, clk); }, &ms)) return -1;
    CHECK(hipMemcpy(&h, clk, sizeof(h), hipMemcpyDeviceToHost));
    const double bytes = 1.0 * lw * 256 * li * 8 * l.bytes;
    const double mhz = core_mhz(h);
    std::snprintf(name, sizeof(name), "%s", l.name);
    col.add(name, mhz > 0 ? bytes / (ms * 1e-3) / cus / (mhz * 1e6) : 0.0, "B/clk/CU");
    std::snprintf(name, sizeof(name), "%s clock", l.name);
    col.add(name, mhz, "MHz");
  }
  // fragment-read patterns: lane -> (row, 16-byte chunk) of rows of 64 or 128 bytes.
  // 32-row MFMA blocks: row = lane % 32, k chunk = lane / 32; 16-row blocks: row = lane % 16,
  // k chunk = lane / 16.  Position of a chunk in its row = chunk ^ swizzle(row).
  {
    struct P { const char* name; int rowb, rows, shift; };
    const P ps[] = {
        {"lds frag 64B rows, 32-row blk, swz (r>>1)&3", 64, 32, 1},
        {"lds frag 64B rows, 32-row blk, swz (r>>2)&3", 64, 32, 2},
        {"lds frag 64B rows, 32-row blk, swz r&3", 64, 32, 0},
        {"lds frag 64B rows, 16-row blk, swz (r>>1)&3", 64, 16, 1},
        {"lds frag 64B rows, 16-row blk, swz (r>>2)&3", 64, 16, 2},
        {"lds frag 128B rows, 32-row blk, swz (r>>1)&7", 128, 32, 1},
        {"lds frag 128B rows, 32-row blk, swz r&7", 128, 32, 0},
        {"lds frag 128B rows, 16-row blk, swz (r>>1)&7", 128, 16, 1},
        {"lds frag 128B rows, 16-row blk, swz r&7", 128, 16, 0},
        {"lds frag planes, 32-row blk, plane stride 1024", 0, 32, 1024},
        {"lds frag planes, 32-row blk, plane stride 1024+256", 0, 32, 1024 + 256},
        {"lds frag planes, 16-row blk, plane stride 512", 0, 16, 512},
        {"lds frag planes, 16-row blk, plane stride 512+64", 0, 16, 512 + 64},
        {"lds frag planes, 16-row blk, plane stride 512+128", 0, 16, 512 + 128},
    };
    // (rowb == 0: "planes": consecutive 16-byte entries per k chunk, chunk c of every entry
    // `shift` bytes after chunk c - 1: the patch layout of the 3x3 kernels, where the plane
    // stride is a multiple of 256 bytes, or that plus a pad)
    int* d_off = nullptr;
    CHECK(hipMalloc(&d_off, 64 * sizeof(int)));
    for (const P& q : ps) {
      int off[64];
      const int cpr = q.rowb / 16;
      for (int l = 0; l < 64; ++l) {
        const int row = l % q.rows, chunk = l / q.rows;
        if (q.rowb == 0)
          off[l] = row * 16 + chunk * q.shift;
        else
          off[l] = (row * q.rowb + ((chunk ^ ((row >> q.shift) & (cpr - 1))) * 16)) % 2048;
      }
      CHECK(hipMemcpy(d_off, off, sizeof(off), hipMemcpyHostToDevice));
      const int lw = cus * 2, li = 4000;
      lds_pattern_loop<<<lw, 256>>>(reinterpret_cast<unsigned*>(fout), 10, clk, d_off);
      CHECK(hipDeviceSynchronize());
      if (timed([&] { lds_pattern_loop<<<lw, 256>>>(reinterpret_cast<unsigned*>(fout), li, clk, d_off); }, &ms))
        return -1;
      CHECK(hipMemcpy(&h, clk, sizeof(h), hipMemcpyDeviceToHost));
      const double bytes = 1.0 * lw * 256 * li * 8 * 16;
      const double mhz = core_mhz(h);
      col.add(q.name, mhz > 0 ? bytes / (ms * 1e-3) / cus / (mhz * 1e6) : 0.0, "B/clk/CU");
    }
    CHECK(hipFree(d_off));
  }
  // transposing reads of an MFMA operand whose 8 k values per lane lie in 8 different LDS rows
  // (the filter as it lies in memory: a row = one k, features contiguous).  A 16-lane group
  // reads 4 rows x 32 bytes; piece j of row k is stored at piece position j ^ swizzle(k).
  {
    struct Q { const char* name; int row_bytes, blk, swz; };
    const Q qs[] = {
        {"lds tr-read, 256B rows, 16-row blk, no swizzle", 256, 16, 0},
        {"lds tr-read, 256B rows, 16-row blk, swz k&3|k>>3&1<<2", 256, 16, 1},
        {"lds tr-read, 128B rows, 16-row blk, swz k>>1&1|k>>3&1<<1", 128, 16, 2},
        {"lds tr-read, 512B rows, 16-row blk, swz k&3|k>>3&1<<2", 512, 16, 1},
        {"lds tr-read, 256B rows, 32-row blk, swz (k&3)<<1", 256, 32, 3},
        {"lds tr-read, 512B rows, 32-row blk, swz (k&3)<<1", 512, 32, 3},
        {"lds tr-read, 128B rows, 32-row blk, swz (k>>1&1)<<1", 128, 32, 4},
    };
    int* d_off = nullptr;
    CHECK(hipMalloc(&d_off, 128 * sizeof(int)));
    for (const Q& q : qs) {
      int off[128];
      for (int r = 0; r < 2; ++r)
        for (int l = 0; l < 64; ++l) {
          const int a = l % 16;
          int k, piece;
          if (q.blk == 16) { k = 8 * (l / 16) + 4 * r + a / 4; piece = 0; }
          else { k = 8 * (l / 32) + 4 * r + a / 4; piece = (l / 16) % 2; }
          int sw = 0;
          if (q.swz == 1) sw = (k & 3) | (((k >> 3) & 1) << 2);
          if (q.swz == 2) sw = ((k >> 1) & 1) | (((k >> 3) & 1) << 1);
          if (q.swz == 3) sw = (k & 3) << 1;
          if (q.swz == 4) sw = ((k >> 1) & 1) << 1;
          off[r * 64 + l] = k * q.row_bytes + 32 * (piece ^ sw) + 8 * (a % 4);
        }
      CHECK(hipMemcpy(d_off, off, sizeof(off), hipMemcpyHostToDevice));
      // (further reads of the loop: the next feature block, 2 pieces on for 32-row blocks)
      const int step = q.row_bytes >= 256 ? 64 : 0;
      const int lw = cus * 2, li = 4000;
      lds_tr_pattern_loop<<<lw, 256>>>(reinterpret_cast<unsigned*>(fout), 10, clk, d_off, step);
      CHECK(hipDeviceSynchronize());
      if (timed([&] { lds_tr_pattern_loop<<<lw, 256>>>(reinterpret_cast<unsigned*>(fout), li, clk, d_off, step); }, &ms))
        return -1;
      CHECK(hipMemcpy(&h, clk, sizeof(h), hipMemcpyDeviceToHost));
      const double bytes = 1.0 * lw * 256 * li * 8 * 8;
      const double mhz = core_mhz(h);
      col.add(q.name, mhz > 0 ? bytes / (ms * 1e-3) / cus / (mhz * 1e6) : 0.0, "B/clk/CU");
    }
    CHECK(hipFree(d_off));
  }
  CHECK(hipFree(clk));
  CHECK(hipFree(fout));

  // streaming over 1 GiB (beyond the 256 MB last-level cache)
  const size_t n = (1ull << 30) / 16;
  uintx4 *a = nullptr, *b = nullptr;
  CHECK(hipMalloc(&a, n * 16));
  CHECK(hipMalloc(&b, n * 16));
  CHECK(hipMemset(a, 1, n * 16));
  CHECK(hipMemset(b, 2, n * 16));
  struct S { const char* name; double bytes; void (*k)(const uintx4*, uintx4*, size_t); };
  const S ss[] = {
      {"hbm_copy (read+write)", 32, stream_loop<0>},
      {"hbm_read", 16, stream_loop<1>},
      {"hbm_write", 16, stream_loop<2>},
      {"hbm_copy nontemporal stores", 32, stream_loop<3>},
  };
  for (const S& s : ss) {
    const int grid = cus * 32;
    s.k<<<grid, 256>>>(a, b, n);
    CHECK(hipDeviceSynchronize());
    if (timed([&] { for (int i = 0; i < 5; ++i) s.k<<<grid, 256>>>(a, b, n); }, &ms)) return -1;
    col.add(s.name, n * s.bytes * 5 / ms / 1e6, "GB/s");
  }
  CHECK(hipFree(a));
  CHECK(hipFree(b));
  return col.n;
}

}  // extern "C"
