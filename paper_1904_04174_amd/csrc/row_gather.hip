// Window-row gather kernels for layers with very few input channels (fp32, and a bf16 twin
// further down), such as the 7x7 stride-2 first layer of a ResNet on a 3-channel image
// (Figure 1's caption gives the parameter tuple; section 3 asks for a choice
// of algorithm per layer).
//
// With C <= 4 a 16-byte gather vector covers a pixel and a quarter, so the
// vector tiles cannot run and the element-wise tiles issue one load per
// multiply operand.  Here the reduction index k = (r, s, c) is read as
// (r, j) with j = s * C + c: the S * C values of one window row are
// consecutive in the NHWC input, and k itself is the row index of the HWCF
// filter, so nothing is repacked and only a window row of odd length is
// padded by one value (7x7x3: 154 reduction indices instead of 196 with the
// channels padded to 4).
//
// A workgroup (4 waves) computes an 8 x 16 block of output pixels of one
// image times 64 features.  It keeps the filter tile in LDS (loaded once:
// workgroups are persistent and walk the tiles with the grid's stride) and
// loads the block's input patch, (7 * sr + R) rows of (15 * sc + S) * C
// consecutive values, zero outside the image (fetched into registers while the
// previous tile is computed, stored to LDS before that tile's output stores).  Wave w owns block rows 2w and
// 2w + 1 (32 pixels) and all 64 features: two 32x32x2 fp32 MFMA accumulators.
// Per step of two reduction indices (both in one window row) a lane reads one
// patch value (its pixel, value 2 * jj + lane / 32 of the row) and two filter
// values; fragments are fetched two steps ahead.  The patch's row pitch is chosen so that the 32 pixels of a wave
// fall into distinct LDS banks.
#include "conv2d_internal.h"

namespace conv2d {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kBH = 8, kBW = 16, kBN = 64, kThreads = 256;
constexpr int kMaxLds = 64 * 1024;
constexpr int kFilterLoads = 16; // filter values per thread and pass
constexpr int kPatchLoads = 12;  // patch values per thread: patches of up to 12 * 256 values

struct RowPlan {
  int PH, PWE, pitch;   // patch rows, values per row, LDS row pitch (floats)
  int steps;            // pairs of reduction indices
  int frows;            // filter rows kept in LDS (2 * steps + 2, zero past Kg)
  int tiles_x, tiles_y, tiles_n;
  int tiles_m;          // N * tiles_y * tiles_x
  long long tiles;
  int lds_bytes;
  int grid;
};

RowPlan make_plan(const Problem& p) {
  RowPlan pl;
  pl.PH = (kBH - 1) * p.sr + p.R;
  pl.PWE = ((kBW - 1) * p.sc + p.S) * p.C;
  // a wave's second block row lies sr * pitch floats after the first: half a turn of the 64
  // banks apart when the pixels of a row are an even number of floats apart (else any pitch)
  pl.pitch = pl.PWE;
  if ((p.sc * p.C) % 2 == 0)
    while ((1LL * p.sr * pl.pitch) % 64 != 32 && pl.pitch < pl.PWE + 64) ++pl.pitch;
  if ((1LL * p.sr * pl.pitch) % 64 != 32) pl.pitch = pl.PWE | 1;
  pl.steps = p.R * ((p.S * p.C + 1) / 2);  // window rows padded to an even length
  pl.frows = 2 * pl.steps + 4;   // fragments are fetched up to two steps past the end
  pl.tiles_x = (p.Q + kBW - 1) / kBW;
  pl.tiles_y = (p.P + kBH - 1) / kBH;
  pl.tiles_n = (p.K + kBN - 1) / kBN;
  pl.tiles_m = p.N * pl.tiles_y * pl.tiles_x;
  pl.tiles = 1LL * pl.tiles_m * pl.tiles_n;
  // (three more patch rows: the fragments fetched after the last step lie in the rows after the
  // window; +4: the pad value of an odd window row may lie one past the last value of a row)
  const long long lds = 4LL * (1LL * pl.frows * kBN + 1LL * (pl.PH + 3) * pl.pitch + 4);
  pl.lds_bytes = lds > (1LL << 30) ? (1 << 30) : static_cast<int>(lds);
  int occ = pl.lds_bytes > 0 ? (160 * 1024) / pl.lds_bytes : 1;
  occ = occ < 1 ? 1 : (occ > 3 ? 3 : occ);
  const long long resident = 256LL * occ;
  pl.grid = static_cast<int>(pl.tiles < resident ? pl.tiles : resident);
  return pl;
}

// LDS position of filter value (k, col) of the tile: the two reduction indices of a step side
// by side, so that the lanes of both halves of a wave read distinct banks.
__device__ __forceinline__ int filter_slot(int k, int col) {
  return (k >> 1) * 128 + (k & 1) * 32 + (col & 31) + (col >> 5) * 64;
}

// Workgroup barrier that orders LDS accesses only.  (__syncthreads also waits for the wave's
// global stores: every tile would then wait for its own output stores to be acknowledged.)
__device__ __forceinline__ void lds_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

__global__ __launch_bounds__(kThreads, 2) void row_gather_kernel(const Problem p,
                                                                 const RowPlan pl) {
  extern __shared__ __align__(16) float lds[];
  float* lds_f = lds;
  float* lds_p = lds + pl.frows * kBN;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int l32 = lane & 31;
  const int kh = lane >> 5;

  const float* __restrict__ in = static_cast<const float*>(p.in);
  const float* __restrict__ filt = static_cast<const float*>(p.filt);
  float* __restrict__ out = static_cast<float*>(p.out);

  const int row_len = p.S * p.C;
  // the lane's pixel of the block: wave's rows 2w, 2w + 1
  const int py = 2 * wave + (l32 >> 4), px = l32 & 15;
  const int a_lane = py * p.sr * pl.pitch + px * p.sc * p.C + kh;
  const int row_steps = (row_len + 1) / 2;
  const bool odd_pad = (row_len & 1) && kh == 1;
  const int b_base = kh * 32 + l32;

  // ---- patch loader role: values tid + i * 256 of the patch (row y, value e of the row); the
  // same for every tile, so the positions are worked out once.  A tile's values are fetched
  // into registers while the previous tile is computed and stored to LDS after it.  (All of
  // this in 32-bit integer arithmetic with as few instructions per tile as possible: they are
  // issued by the same SIMDs that issue the products.)
  int ye[kPatchLoads], p_slot[kPatchLoads], g_rel[kPatchLoads];
#pragma unroll
  for (int i = 0; i < kPatchLoads; ++i) {
    const int idx = tid + i * kThreads;
    const int y = idx / pl.PWE, e = idx - y * pl.PWE;
    ye[i] = y < pl.PH ? (y << 16 | e) : -1;
    p_slot[i] = y * pl.pitch + e;
    g_rel[i] = y * p.W * p.C + e;   // input offset relative to the patch's first value
  }
  float pv[kPatchLoads];
  unsigned pmask = 0;               // bit i: value i lies inside the image
  // tile t -> feature tile, image, block row and column
  auto tile_of = [&](unsigned t, int& tn, int& n, int& by, int& bx) {
    const unsigned tiles_m = static_cast<unsigned>(pl.tiles_m);
    tn = static_cast<int>(t / tiles_m);
    const unsigned tm = t - static_cast<unsigned>(tn) * tiles_m;
    const unsigned per_image = static_cast<unsigned>(pl.tiles_x * pl.tiles_y);
    n = static_cast<int>(tm / per_image);
    const unsigned tb = tm - static_cast<unsigned>(n) * per_image;
    by = static_cast<int>(tb / static_cast<unsigned>(pl.tiles_x));
    bx = static_cast<int>(tb) - by * pl.tiles_x;
  };
  auto fetch_patch = [&](int n, int by, int bx) {
    // rows from h0, values from column w0 on; zero outside the image
    const int h0 = by * kBH * p.sr - p.pt;
    const int w0 = bx * kBW * p.sc - p.pl;
    const int lo_e = (w0 < 0 ? -w0 : 0) * p.C;
    const int hi_w = p.W - w0;  // columns of the image from w0 on
    const int hi_e = hi_w <= 0 ? 0 : (1LL * hi_w * p.C < pl.PWE ? hi_w * p.C : pl.PWE);
    const int src0 = ((n * p.H + h0) * p.W + w0) * p.C;
    pmask = 0;
#pragma unroll
    for (int i = 0; i < kPatchLoads; ++i) {
      const int y = ye[i] >> 16, e = ye[i] & 0xffff;
      const bool ok = ye[i] >= 0 && static_cast<unsigned>(h0 + y) < static_cast<unsigned>(p.H) &&
                      e >= lo_e && e < hi_e;
      // (an unconditional load from a safe address, the select when the value is stored to LDS:
      // loads under a branch would each be waited for, one after the other)
      pv[i] = in[ok ? src0 + g_rel[i] : 0];
      pmask |= ok ? 1u << i : 0u;
    }
  };

  // ---- filter loader role: column tid % 64 of rows tid / 64 + 4 * i of the padded filter
  const int f_col = tid & 63;
  const int row2 = 2 * row_steps;   // padded window row
  const int row_skip = pl.pitch - row2;  // from the end of a window row to the start of the next

  auto load_filter = [&](int n0) {
    // padded row kp = (fr, fj) with rows of row2 values; zero for the pads and past the end.
    // Sixteen loads in flight per thread: one at a time their latencies would add up to more
    // than a tile's products.
    int kp = tid >> 6, fr = 0, fj = kp;
    if (fj >= row2) { fj -= row2; ++fr; }
    if (fj >= row2) { fj -= row2; ++fr; }
    const bool col_ok = n0 + f_col < p.K;
    for (int base = 0; base < pl.frows; base += 4 * kFilterLoads) {
      float fv[kFilterLoads];
      unsigned fmask = 0;
      int slot[kFilterLoads];
#pragma unroll
      for (int u = 0; u < kFilterLoads; ++u) {
        const bool ok = kp < pl.frows && fr < p.R && fj < row_len && col_ok;
        fv[u] = filt[ok ? (fr * row_len + fj) * p.K + n0 + f_col : 0];
        fmask |= ok ? 1u << u : 0u;
        slot[u] = kp < pl.frows ? filter_slot(kp, f_col) : -1;
        kp += 4; fj += 4;
        if (fj >= row2) { fj -= row2; ++fr; }
        if (fj >= row2) { fj -= row2; ++fr; }
      }
#pragma unroll
      for (int u = 0; u < kFilterLoads; ++u)
        if (slot[u] >= 0) lds_f[slot[u]] = (fmask >> u & 1) ? fv[u] : 0.f;
    }
  };
  auto stash_patch = [&]() {
#pragma unroll
    for (int i = 0; i < kPatchLoads; ++i)
      if (ye[i] >= 0) lds_p[p_slot[i]] = (pmask >> i & 1) ? pv[i] : 0.f;
  };

  // Order of a tile's phases: products; barrier; the NEXT tile's patch from registers to LDS;
  // this tile's output stores; barrier; loads of the tile after next.  The wait for the patch
  // loads thus comes a whole tile of products after the previous stores were issued: the one
  // counter of outstanding memory operations covers stores too, and straight after the stores
  // it would wait for all of them to be acknowledged.
  const unsigned ntiles = static_cast<unsigned>(pl.tiles);
  unsigned t = blockIdx.x;
  if (t >= ntiles) return;
  int tn = 0, n = 0, by = 0, bx = 0;
  tile_of(t, tn, n, by, bx);
  fetch_patch(n, by, bx);
  load_filter(tn * kBN);
  float bias0 = bias_of(p.bias, tn * kBN + l32, p.K);
  float bias1 = bias_of(p.bias, tn * kBN + 32 + l32, p.K);
  stash_patch();
  lds_barrier();
  for (;;) {
    const int n0 = tn * kBN;
    const bool col0_ok = n0 + l32 < p.K, col1_ok = n0 + 32 + l32 < p.K;
    // this tile's output position; then the next tile's patch, in flight during the products
    const int op0 = by * kBH + 2 * wave, oq0 = bx * kBW + 4 * kh;
    float* tile_out = out + ((static_cast<size_t>(n) * p.P + op0) * p.Q + oq0) * p.K + n0 + l32;
    const unsigned t_next = t + gridDim.x;
    const bool has_next = t_next < ntiles;
    int tn_next = tn;
    if (has_next) {
      tile_of(t_next, tn_next, n, by, bx);
      fetch_patch(n, by, bx);
    }

    floatx16 acc0 = {}, acc1 = {};
    // Step (r, jj) multiplies values j = 2 * jj + kh of window row r (both halves of the wave in
    // the same row, so the patch offset of a step is the same for all lanes); with an odd row
    // length the upper half's last value of a row is a pad: zero filter row, value forced to 0.
    // (The scalar bookkeeping of a step is kept to a few dependent instructions: a wave issues
    // them one after the other between its products.)
    // Fragments are fetched two steps ahead, into three sets of registers that take turns (X, Y,
    // Z: the step loop is unrolled by three, so no set is copied): with a single step ahead, or
    // with copies from set to set, the reads' latency lies on a wave's path from one step to
    // the next.  A pad value is forced to zero when its set is multiplied, a step or two after
    // it was read.  The fragments read past the last step are never multiplied.
    int jj = 0, off = 0;
    struct Frag { float a, b0, b1; bool pad; };
    auto read_frag = [&](int step, Frag& f) {
      f.pad = odd_pad && jj == row_steps - 1;
      f.a = lds_p[a_lane + off];
      f.b0 = lds_f[b_base + step * 128];
      f.b1 = lds_f[b_base + step * 128 + 64];
      ++jj; off += 2;
      if (jj == row_steps) { jj = 0; off += row_skip; }
    };
    auto multiply = [&](const Frag& f) {
      const float a = f.pad ? 0.f : f.a;
      __builtin_amdgcn_sched_barrier(0);  // the reads before are issued ahead of the products
      acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, f.b0, acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, f.b1, acc1, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    };
    Frag X, Y, Z;
    read_frag(0, X);
    read_frag(1, Y);
    const int whole = pl.steps / 3 * 3;
    for (int s = 0; s < whole; s += 3) {
      read_frag(s + 2, Z);
      multiply(X);
      read_frag(s + 3, X);
      multiply(Y);
      read_frag(s + 4, Y);
      multiply(Z);
    }
    if (pl.steps - whole >= 1) multiply(X);
    if (pl.steps - whole == 2) multiply(Y);

    lds_barrier();  // every wave has read this tile's patch and filter
    if (has_next) {
      if (tn_next != tn) load_filter(tn_next * kBN);
      stash_patch();
    }

    // ---- epilogue: register v of a lane is row 8 * (v / 4) + 4 * kh + v % 4 of the wave's 32
    // pixels (block row v / 8, column 8 * (v / 4 % 2) + 4 * kh + v % 4), column l32 of the
    // feature block: a store instruction writes two pixels' 32 consecutive features (whole
    // 128-byte lines; non-temporal: the output is not read again).  The bias values are in
    // registers before the first store (a wait for them between the stores would also wait for
    // the stores before it, one after the other).
    asm volatile("" : "+v"(bias0), "+v"(bias1));
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int dy = v >> 3, dx = 8 * ((v >> 2) & 1) + (v & 3);
      if (op0 + dy < p.P && oq0 + dx < p.Q) {
        float* dst = tile_out + (dy * p.Q + dx) * p.K;
        if (col0_ok) __builtin_nontemporal_store(finish(acc0[v], bias0, p.relu), dst);
        if (col1_ok) __builtin_nontemporal_store(finish(acc1[v], bias1, p.relu), dst + 32);
      }
    }
    if (!has_next) break;
    if (tn_next != tn) {
      bias0 = bias_of(p.bias, tn_next * kBN + l32, p.K);
      bias1 = bias_of(p.bias, tn_next * kBN + 32 + l32, p.K);
    }
    lds_barrier();  // the next tile's patch (and filter) are in LDS
    t = t_next;
    tn = tn_next;
  }
}


// ---------------------------------------------------------------------------------------------
// The same kernel for bf16 input and filter (fp32 accumulation, fp32 or bf16 output) on
// v_mfma_f32_32x32x8_bf16_1k: a lane supplies 4 consecutive reduction indices of its k group, so a
// step covers 8 values of a window row and a row of S * C values is padded to a multiple of 8
// (7x7x3: 21 -> 24, 21 steps instead of 77).  Differences from the fp32 kernel:
//   * the patch lies in LDS as bf16; a lane's 4 values are two 4-byte reads, which needs the
//     pixels of a row an even number of values apart (sc * C even; the 3-channel stride-2 stem);
//     values past the end of a window row belong to the neighbouring pixels and are masked to
//     zero (their filter rows are zero too, but a NaN there must not reach this pixel);
//   * the filter tile lies in LDS feature-major with the reduction index contiguous (transposed
//     while it is loaded, once per workgroup and feature tile): a lane's 4 values are one 8-byte
//     read; a feature's row is 2 (mod 32) words long, so the 32 lanes of a half wave read
//     distinct banks.
typedef short shortx4 __attribute__((ext_vector_type(4)));

struct RowPlanB {
  int PH, PWE, pitch;   // patch rows, values per row, LDS row pitch (bf16 values, even)
  int row2, row_steps;  // padded window row, its steps of 8
  int steps;            // steps of 8 reduction indices
  int kpad;             // filter values per feature kept in LDS (zero past the window)
  int wrow;             // words per feature in LDS
  int tiles_x, tiles_y, tiles_n, tiles_m;
  long long tiles;
  int lds_bytes;
  int grid;
};

RowPlanB make_plan_b(const Problem& p) {
  RowPlanB pl;
  pl.PH = (kBH - 1) * p.sr + p.R;
  pl.PWE = ((kBW - 1) * p.sc + p.S) * p.C;
  // a wave's second block row lies sr * pitch values = sr * pitch / 2 words after the first: half
  // a turn of the 64 banks apart where that can be had
  pl.pitch = (pl.PWE + 1) / 2 * 2;
  const int first = pl.pitch;
  while ((1LL * p.sr * pl.pitch / 2) % 64 != 32 && pl.pitch < first + 128) pl.pitch += 2;
  if ((1LL * p.sr * pl.pitch / 2) % 64 != 32) pl.pitch = first;
  const int row_len = p.S * p.C;
  pl.row2 = (row_len + 7) / 8 * 8;
  pl.row_steps = pl.row2 / 8;
  pl.steps = p.R * pl.row_steps;
  pl.kpad = p.R * pl.row2 + 16;  // (+ the two steps fetched after the last one)
  pl.wrow = pl.kpad / 2;
  while (pl.wrow % 32 != 2) ++pl.wrow;
  pl.tiles_x = (p.Q + kBW - 1) / kBW;
  pl.tiles_y = (p.P + kBH - 1) / kBH;
  pl.tiles_n = (p.K + kBN - 1) / kBN;
  pl.tiles_m = p.N * pl.tiles_y * pl.tiles_x;
  pl.tiles = 1LL * pl.tiles_m * pl.tiles_n;
  // (one more patch row and 16 values: the fragment fetched after the last step lies in the row
  // after the window, a padded window row may reach past the end of a patch row)
  const long long lds = 4LL * kBN * pl.wrow + 2LL * ((pl.PH + 3LL) * pl.pitch + 16);
  pl.lds_bytes = lds > (1LL << 30) ? (1 << 30) : static_cast<int>((lds + 15) / 16 * 16);
  int occ = pl.lds_bytes > 0 ? (160 * 1024) / pl.lds_bytes : 1;
  occ = occ < 1 ? 1 : (occ > 3 ? 3 : occ);
  const long long resident = 256LL * occ;
  pl.grid = static_cast<int>(pl.tiles < resident ? pl.tiles : resident);
  return pl;
}

__device__ __forceinline__ unsigned short bf16_bits(float x) {
  unsigned int u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<unsigned short>((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<unsigned short>(u >> 16);
}

template <bool OUT_BF16>
__global__ __launch_bounds__(kThreads, 2) void row_gather_bf16_kernel(const Problem p,
                                                                      const RowPlanB pl) {
  extern __shared__ __align__(16) unsigned lds_w[];
  unsigned* lds_f = lds_w;  // [64 features][wrow words]
  unsigned short* lds_p = reinterpret_cast<unsigned short*>(lds_w + kBN * pl.wrow);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int l32 = lane & 31;
  const int kh = lane >> 5;

  const unsigned short* __restrict__ in = static_cast<const unsigned short*>(p.in);
  const unsigned short* __restrict__ filt = static_cast<const unsigned short*>(p.filt);

  const int row_len = p.S * p.C;
  const int py = 2 * wave + (l32 >> 4), px = l32 & 15;
  // (values; even, so that the two reads of a fragment are 4-byte aligned)
  const int a_lane = py * p.sr * pl.pitch + px * p.sc * p.C + 4 * kh;
  const int row_steps = pl.row_steps;
  // the lane's values of a window row's last step that lie inside the row
  int inside = row_len - (8 * (row_steps - 1) + 4 * kh);
  inside = inside < 0 ? 0 : (inside > 4 ? 4 : inside);
  const unsigned mask0 = inside >= 2 ? 0xffffffffu : inside == 1 ? 0xffffu : 0u;
  const unsigned mask1 = inside >= 4 ? 0xffffffffu : inside == 3 ? 0xffffu : 0u;
  const int b_base0 = l32 * pl.wrow + 2 * kh, b_base1 = (32 + l32) * pl.wrow + 2 * kh;

  // ---- patch loader role (as in the fp32 kernel, 2-byte values)
  int ye[kPatchLoads], p_slot[kPatchLoads], g_rel[kPatchLoads];
#pragma unroll
  for (int i = 0; i < kPatchLoads; ++i) {
    const int idx = tid + i * kThreads;
    const int y = idx / pl.PWE, e = idx - y * pl.PWE;
    ye[i] = y < pl.PH ? (y << 16 | e) : -1;
    p_slot[i] = y * pl.pitch + e;
    g_rel[i] = y * p.W * p.C + e;
  }
  unsigned short pv[kPatchLoads];
  unsigned pmask = 0;
  auto tile_of = [&](unsigned t, int& tn, int& n, int& by, int& bx) {
    const unsigned tiles_m = static_cast<unsigned>(pl.tiles_m);
    tn = static_cast<int>(t / tiles_m);
    const unsigned tm = t - static_cast<unsigned>(tn) * tiles_m;
    const unsigned per_image = static_cast<unsigned>(pl.tiles_x * pl.tiles_y);
    n = static_cast<int>(tm / per_image);
    const unsigned tb = tm - static_cast<unsigned>(n) * per_image;
    by = static_cast<int>(tb / static_cast<unsigned>(pl.tiles_x));
    bx = static_cast<int>(tb) - by * pl.tiles_x;
  };
  auto fetch_patch = [&](int n, int by, int bx) {
    const int h0 = by * kBH * p.sr - p.pt;
    const int w0 = bx * kBW * p.sc - p.pl;
    const int lo_e = (w0 < 0 ? -w0 : 0) * p.C;
    const int hi_w = p.W - w0;
    const int hi_e = hi_w <= 0 ? 0 : (1LL * hi_w * p.C < pl.PWE ? hi_w * p.C : pl.PWE);
    const int src0 = ((n * p.H + h0) * p.W + w0) * p.C;
    pmask = 0;
#pragma unroll
    for (int i = 0; i < kPatchLoads; ++i) {
      const int y = ye[i] >> 16, e = ye[i] & 0xffff;
      const bool ok = ye[i] >= 0 && static_cast<unsigned>(h0 + y) < static_cast<unsigned>(p.H) &&
                      e >= lo_e && e < hi_e;
      pv[i] = in[ok ? src0 + g_rel[i] : 0];
      pmask |= ok ? 1u << i : 0u;
    }
  };
  auto stash_patch = [&]() {
#pragma unroll
    for (int i = 0; i < kPatchLoads; ++i)
      if (ye[i] >= 0) lds_p[p_slot[i]] = (pmask >> i & 1) ? pv[i] : static_cast<unsigned short>(0);
  };

  // ---- filter loader role: feature tid % 64, padded reduction indices tid / 64 + 4 * i; the
  // value goes to [feature][index]: the transpose that the k-contiguous fragment read needs
  const int f_col = tid & 63;
  const int row2 = pl.row2;
  unsigned short* lds_f16 = reinterpret_cast<unsigned short*>(lds_f);
  auto load_filter = [&](int n0) {
    int kp = tid >> 6, fr = 0, fj = kp;
    while (fj >= row2) { fj -= row2; ++fr; }
    const bool col_ok = n0 + f_col < p.K;
    for (int base = 0; base < pl.kpad; base += 4 * kFilterLoads) {
      unsigned short fv[kFilterLoads];
      unsigned fmask = 0;
      int slot[kFilterLoads];
#pragma unroll
      for (int u = 0; u < kFilterLoads; ++u) {
        const bool ok = kp < pl.kpad && fr < p.R && fj < row_len && col_ok;
        fv[u] = filt[ok ? (fr * row_len + fj) * p.K + n0 + f_col : 0];
        fmask |= ok ? 1u << u : 0u;
        slot[u] = kp < pl.kpad ? f_col * (2 * pl.wrow) + kp : -1;
        kp += 4; fj += 4;
        while (fj >= row2) { fj -= row2; ++fr; }
      }
#pragma unroll
      for (int u = 0; u < kFilterLoads; ++u)
        if (slot[u] >= 0) lds_f16[slot[u]] = (fmask >> u & 1) ? fv[u] : static_cast<unsigned short>(0);
    }
  };

  typedef unsigned uintx2 __attribute__((ext_vector_type(2)));
  auto read_a = [&](int off) {
    const unsigned* src = reinterpret_cast<const unsigned*>(lds_p + a_lane + off);
    return uintx2{src[0], src[1]};
  };
  auto read_b = [&](int base, int s) {
    return *reinterpret_cast<const uintx2*>(lds_f + base + 4 * s);
  };

  const unsigned ntiles = static_cast<unsigned>(pl.tiles);
  unsigned t = blockIdx.x;
  if (t >= ntiles) return;
  int tn = 0, n = 0, by = 0, bx = 0;
  tile_of(t, tn, n, by, bx);
  fetch_patch(n, by, bx);
  load_filter(tn * kBN);
  float bias0 = bias_of(p.bias, tn * kBN + l32, p.K);
  float bias1 = bias_of(p.bias, tn * kBN + 32 + l32, p.K);
  stash_patch();
  lds_barrier();
  for (;;) {
    const int n0 = tn * kBN;
    const bool col0_ok = n0 + l32 < p.K, col1_ok = n0 + 32 + l32 < p.K;
    const int op0 = by * kBH + 2 * wave, oq0 = bx * kBW + 4 * kh;
    const size_t out_first = ((static_cast<size_t>(n) * p.P + op0) * p.Q + oq0) * p.K + n0 + l32;
    const unsigned t_next = t + gridDim.x;
    const bool has_next = t_next < ntiles;
    int tn_next = tn;
    if (has_next) {
      tile_of(t_next, tn_next, n, by, bx);
      fetch_patch(n, by, bx);
    }

    floatx16 acc0 = {}, acc1 = {};
    // Fragments two steps ahead in three sets of registers that take turns, as in the fp32
    // kernel; the values past the end of a window row are masked when the set is multiplied.
    int jj = 0, off = 0;
    struct Frag { uintx2 a, b0, b1; bool last; };
    auto read_frag = [&](int step, Frag& f) {
      f.last = jj == row_steps - 1;
      f.a = read_a(off);
      f.b0 = read_b(b_base0, step);
      f.b1 = read_b(b_base1, step);
      ++jj; off += 8;
      if (jj == row_steps) { jj = 0; off += pl.pitch - row2; }
    };
    auto multiply = [&](const Frag& f) {
      uintx2 a = f.a;
      a.x &= f.last ? mask0 : 0xffffffffu;
      a.y &= f.last ? mask1 : 0xffffffffu;
      __builtin_amdgcn_sched_barrier(0);
      acc0 = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(__builtin_bit_cast(shortx4, a),
                                                      __builtin_bit_cast(shortx4, f.b0), acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(__builtin_bit_cast(shortx4, a),
                                                      __builtin_bit_cast(shortx4, f.b1), acc1, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    };
    Frag X, Y, Z;
    read_frag(0, X);
    read_frag(1, Y);
    const int whole = pl.steps / 3 * 3;
    for (int s = 0; s < whole; s += 3) {
      read_frag(s + 2, Z);
      multiply(X);
      read_frag(s + 3, X);
      multiply(Y);
      read_frag(s + 4, Y);
      multiply(Z);
    }
    if (pl.steps - whole >= 1) multiply(X);
    if (pl.steps - whole == 2) multiply(Y);

    lds_barrier();
    if (has_next) {
      if (tn_next != tn) load_filter(tn_next * kBN);
      stash_patch();
    }

    asm volatile("" : "+v"(bias0), "+v"(bias1));
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int dy = v >> 3, dx = 8 * ((v >> 2) & 1) + (v & 3);
      if (op0 + dy < p.P && oq0 + dx < p.Q) {
        const size_t idx = out_first + static_cast<size_t>(dy * p.Q + dx) * p.K;
        const float r0 = finish(acc0[v], bias0, p.relu), r1 = finish(acc1[v], bias1, p.relu);
        if (OUT_BF16) {
          unsigned short* dst = static_cast<unsigned short*>(p.out) + idx;
          if (col0_ok) dst[0] = bf16_bits(r0);
          if (col1_ok) dst[32] = bf16_bits(r1);
        } else {
          float* dst = static_cast<float*>(p.out) + idx;
          if (col0_ok) __builtin_nontemporal_store(r0, dst);
          if (col1_ok) __builtin_nontemporal_store(r1, dst + 32);
        }
      }
    }
    if (!has_next) break;
    if (tn_next != tn) {
      bias0 = bias_of(p.bias, tn_next * kBN + l32, p.K);
      bias1 = bias_of(p.bias, tn_next * kBN + 32 + l32, p.K);
    }
    lds_barrier();
    t = t_next;
    tn = tn_next;
  }
}

bool supports_bf16(const Problem& p) {
  if (!p.in_bf16 || p.M == 0) return false;
  if (p.C > 4 || (p.sc * p.C) % 2 != 0) return false;
  if (p.R > 16 || p.S > 16 || p.sr > 4 || p.sc > 4) return false;
  const RowPlanB pl = make_plan_b(p);
  if (pl.PWE >= (1 << 16) || 1LL * pl.PH * pl.PWE > kPatchLoads * kThreads) return false;
  if (pl.tiles >= (1LL << 31) || 1LL * p.Kg * p.K >= (1LL << 31)) return false;
  return pl.lds_bytes <= kMaxLds;
}

}  // namespace

bool row_gather_supports(const Problem& p) {
  if (p.in_bf16) return supports_bf16(p);
  if (p.out_bf16 || p.M == 0) return false;
  if (p.C > 4) return false;   // wider pixels: the 16-byte gather tiles
  if (p.R > 16 || p.S > 16 || p.sr > 4 || p.sc > 4) return false;
  const RowPlan pl = make_plan(p);
  if (pl.PWE >= (1 << 16) || 1LL * pl.PH * pl.PWE > kPatchLoads * kThreads) return false;
  if (pl.tiles >= (1LL << 31) || 1LL * p.Kg * p.K >= (1LL << 31)) return false;
  return pl.lds_bytes <= kMaxLds;
}

// Modelled cost in clock cycles (for the selector), from measurements on 224x224x3 -> 64
// layers with 1x1 to 7x7 windows at stride 2: a workgroup alone on its compute unit takes about
// 390 cycles per step (the fragment reads' latency is exposed), three resident ones about 170
// each; the fixed part is the output stream or, for a few tiles, about 15000 cycles of launch,
// filter and patch loads.  Priced 15 % up: chosen only where it wins clearly.
double row_gather_cost(const Problem& p) {
  if (p.in_bf16) {
    // the same form with the bf16 kernel's steps of 8 reduction indices (two small MFMAs and
    // three LDS reads each) and half the input bytes
    const RowPlanB pb = make_plan_b(p);
    int occ_b = (160 * 1024) / pb.lds_bytes;
    occ_b = occ_b < 1 ? 1 : (occ_b > 3 ? 3 : occ_b);
    const double per_unit_b = static_cast<double>((pb.tiles + 255) / 256);
    const double resident_b = per_unit_b < occ_b ? per_unit_b : occ_b;
    const double rounds_b = static_cast<double>((pb.tiles + 256LL * occ_b - 1) / (256LL * occ_b));
    const double step_b = 70.0 * resident_b > 200.0 ? 70.0 * resident_b : 200.0;
    const double stream_b =
        (2.0 * p.N * p.H * p.W * p.C + (p.out_bf16 ? 2.0 : 4.0) * p.M * p.K) / 2083.3;
    return 1.15 * (rounds_b * (pb.steps * step_b + 3000.0) + (stream_b > 15000.0 ? stream_b : 15000.0));
  }
  const RowPlan pl = make_plan(p);
  int occ = (160 * 1024) / pl.lds_bytes;
  occ = occ < 1 ? 1 : (occ > 3 ? 3 : occ);
  const double per_unit = static_cast<double>((pl.tiles + 255) / 256);
  const double resident = per_unit < occ ? per_unit : occ;
  const double rounds = static_cast<double>((pl.tiles + 256LL * occ - 1) / (256LL * occ));
  const double step = 170.0 * resident > 390.0 ? 170.0 * resident : 390.0;
  const double stream = (4.0 * p.N * p.H * p.W * p.C + 4.0 * p.M * p.K) / 2083.3;
  return 1.15 * (rounds * pl.steps * step + (stream > 15000.0 ? stream : 15000.0));
}

hipError_t launch_row_gather(const Problem& p, hipStream_t stream) {
  if (p.in_bf16) {
    const RowPlanB pb = make_plan_b(p);
    if (!supports_bf16(p) || pb.grid <= 0) return hipErrorInvalidValue;
    if (p.out_bf16)
      hipLaunchKernelGGL(row_gather_bf16_kernel<true>, dim3(pb.grid), dim3(kThreads), pb.lds_bytes,
                         stream, p, pb);
    else
      hipLaunchKernelGGL(row_gather_bf16_kernel<false>, dim3(pb.grid), dim3(kThreads), pb.lds_bytes,
                         stream, p, pb);
    return hipGetLastError();
  }
  const RowPlan pl = make_plan(p);
  if (!row_gather_supports(p) || pl.grid <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(row_gather_kernel, dim3(pl.grid), dim3(kThreads), pl.lds_bytes, stream, p, pl);
  return hipGetLastError();
}

}  // namespace conv2d
