// Host side of the C ABI declared in include/conv2d.h: parameter validation,
// output geometry, the variant table, the shape-keyed selector and dispatch.
//
// The paper (section 3) describes a library that holds several algorithms
// with the same numeric result and picks an algorithm and its parameters per
// device and layer shape by hand tuning; Figure 1's caption adds that not
// every algorithm supports every parameter set.  Here a "variant" is a kernel
// family plus a tile configuration, each with a supports() predicate, and the
// selector is a hand-tuned rule for one device (MI355X).
#include "../../include/conv2d.h"

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "conv2d_internal.h"

namespace conv2d {
namespace {

constexpr long long kMaxElems = (1LL << 31) - 1;

enum Family { kDirect = 0, kIgemm = 1, kDma = 2, kWinograd = 3, kPadded = 4, kRowGather = 5, kConv1x1 = 6,
              kWinogradLds = 7, kRegFilter = 8 };
// (kWinograd: transform passes around the products; kWinogradLds: everything in one launch)
inline bool is_winograd(int family) { return family == kWinograd || family == kWinogradLds; }
enum Split { kWhole = 0, kSplit = 1, kTail = 2, kFused = 3 };

struct Variant {
  Family family;
  int bf16;    // element type of input and filter the variant is compiled for
  int tile;    // index into the family's tile table
  int split;   // kWhole, kSplit (reduction split uniformly over workgroups) or kTail (balanced tail)
  char name[80];
};

// Variant table: id 0 is the direct kernel (supports everything), then the
// register-staged implicit-GEMM tiles (fp32, then bf16), each followed by its
// split-reduction twin where the tile is small enough for that to make sense,
// then the direct-to-LDS tiles, then the Winograd variants, then the window-row gather kernel
// for very few channels.
struct Table {
  Variant v[256];
  int n;
  void add(Family f, int bf16, int tile, int split, const char* base) {
    Variant& x = v[n++];
    x.family = f; x.bf16 = bf16; x.tile = tile; x.split = split;
    std::snprintf(x.name, sizeof(x.name), "%s%s", base,
                  split == kSplit ? "_splitk" : split == kTail ? "_tail" : "");
  }
  Table() : n(0) {
    add(kDirect, 0, 0, kWhole, "direct");
    for (int bf = 0; bf < 2; ++bf)
      for (int t = 0; t < igemm_num_tiles(bf); ++t) {
        add(kIgemm, bf, t, kWhole, igemm_tile_name(bf, t));
        int bm, bn, bk;
        igemm_tile_shape(bf, t, &bm, &bn, &bk);
        if (bm <= 128) add(kIgemm, bf, t, kSplit, igemm_tile_name(bf, t));
      }
    for (int bf = 0; bf < 2; ++bf)
      for (int t = 0; t < igemm_dma_num_tiles(bf); ++t) {
        add(kDma, bf, t, kWhole, igemm_dma_tile_name(bf, t));
        add(kDma, bf, t, kSplit, igemm_dma_tile_name(bf, t));
        add(kDma, bf, t, kTail, igemm_dma_tile_name(bf, t));
      }
    // zero-padded channels for small C: one variant per per-lane addressed gather tile
    for (int bf = 0; bf < 2; ++bf)
      for (int t = 0; t < igemm_dma_num_tiles(bf); ++t) {
        if (igemm_dma_tile_addressing(bf, t) != 1) continue;
        char base[80];
        // "igemm_dma_bf16_64x64_..._g" -> "padc_bf16_64x64_..._g"
        std::snprintf(base, sizeof(base), "padc_%s", igemm_dma_tile_name(bf, t) + 10);
        add(kPadded, bf, t, kWhole, base);
      }
    // Winograd F(2x2, 3x3), fp32: one variant per gather tile that can run its products
    for (int t = 0; t < igemm_dma_num_tiles(0); ++t) {
      const int addressing = igemm_dma_tile_addressing(0, t);
      if (addressing != 0 && addressing != 1) continue;
      if (igemm_dma_tile_native(0, t)) continue;  // the batched products repack per point
      char base[80];
      // "igemm_dma_f32_64x64_..." -> "winograd2x2_f32_64x64_..."
      std::snprintf(base, sizeof(base), "winograd2x2_%s", igemm_dma_tile_name(0, t) + 10);
      add(kWinograd, 0, t, kWhole, base);
      if (igemm_dma_tile_has_wino(0, t)) {
        // products and output transform fused in one launch (the split field marks it)
        std::snprintf(base, sizeof(base), "winograd2x2_fused_%s", igemm_dma_tile_name(0, t) + 10);
        add(kWinograd, 0, t, kWhole, base);
        v[n - 1].split = kFused;
      }
    }
    add(kWinogradLds, 0, 0, kWhole, "winograd2x2_lds_f32_32x64");
    add(kRowGather, 0, 0, kWhole, "rowgather_f32_128x64");
    add(kRowGather, 1, 0, kWhole, "rowgather_bf16_128x64");
    // the streaming kernel for 1x1 windows
    for (int t = 0; t < conv1x1_num_tiles(); ++t)
      add(kConv1x1, conv1x1_tile_bf16(t), t, kWhole, conv1x1_tile_name(t));
    // 3x3 bf16 layers of 64 channels and features: the filter in registers
    for (int t = 0; t < conv3x3_regfilter_num_tiles(); ++t)
      add(kRegFilter, 1, t, kWhole, conv3x3_regfilter_tile_name(t));
  }
};
const Table& table() {
  static const Table t;
  return t;
}

long long ceil_div_ll(long long a, long long b) { return (a + b - 1) / b; }

int axis(int padding, int extent, int window, int stride, int32_t* out, int32_t* before,
         int32_t* after) {
  long long o, total = 0;
  if (padding == CONV2D_PAD_VALID) {
    if (window > extent) return CONV2D_STATUS_INVALID_ARGUMENT;
    o = ceil_div_ll(static_cast<long long>(extent) - window + 1, stride);
  } else {
    o = ceil_div_ll(extent, stride);
    total = (o - 1) * stride + window - extent;
    if (total < 0) total = 0;
  }
  if (o <= 0 || o > kMaxElems || total > kMaxElems) return CONV2D_STATUS_INVALID_ARGUMENT;
  *out = static_cast<int32_t>(o);
  *before = static_cast<int32_t>(total / 2);
  *after = static_cast<int32_t>(total - total / 2);
  return CONV2D_STATUS_OK;
}

int validate(const conv2d_params* p, conv2d_geometry* g) {
  if (!p || !g) return CONV2D_STATUS_INVALID_ARGUMENT;
  if (p->batch < 0 || p->in_rows <= 0 || p->in_cols <= 0 || p->channels <= 0 || p->features <= 0 ||
      p->window_rows <= 0 || p->window_cols <= 0 || p->stride_rows <= 0 || p->stride_cols <= 0)
    return CONV2D_STATUS_INVALID_ARGUMENT;
  if (p->padding != CONV2D_PAD_VALID && p->padding != CONV2D_PAD_SAME)
    return CONV2D_STATUS_INVALID_ARGUMENT;
  if ((p->in_dtype != CONV2D_F32 && p->in_dtype != CONV2D_BF16) ||
      (p->out_dtype != CONV2D_F32 && p->out_dtype != CONV2D_BF16))
    return CONV2D_STATUS_INVALID_ARGUMENT;
  int rc = axis(p->padding, p->in_rows, p->window_rows, p->stride_rows, &g->out_rows, &g->pad_top,
                &g->pad_bottom);
  if (rc) return rc;
  rc = axis(p->padding, p->in_cols, p->window_cols, p->stride_cols, &g->out_cols, &g->pad_left,
            &g->pad_right);
  if (rc) return rc;
  if (p->in_dtype == CONV2D_F32 && p->out_dtype == CONV2D_BF16) return CONV2D_STATUS_UNSUPPORTED;
  return CONV2D_STATUS_OK;
}

// Fills the derived problem (without pointers).  TOO_LARGE if a tensor or the
// reduction length does not fit 31-bit element indices.
int derive(const conv2d_params* p, Problem* q) {
  conv2d_geometry g;
  int rc = validate(p, &g);
  if (rc) return rc;
  const long long in_elems = 1LL * p->batch * p->in_rows * p->in_cols * p->channels;
  const long long m = 1LL * p->batch * g.out_rows * g.out_cols;
  const long long kg = 1LL * p->window_rows * p->window_cols * p->channels;
  if (1LL * p->in_rows * p->in_cols > kMaxElems || in_elems > kMaxElems || m > kMaxElems ||
      kg > kMaxElems || kg * p->features > kMaxElems || m * p->features > kMaxElems)
    return CONV2D_STATUS_TOO_LARGE;
  std::memset(q, 0, sizeof(*q));
  q->N = p->batch; q->H = p->in_rows; q->W = p->in_cols; q->C = p->channels; q->K = p->features;
  q->R = p->window_rows; q->S = p->window_cols; q->sr = p->stride_rows; q->sc = p->stride_cols;
  q->pt = g.pad_top; q->pl = g.pad_left; q->P = g.out_rows; q->Q = g.out_cols;
  q->M = static_cast<int>(m);
  q->Kg = static_cast<int>(kg);
  q->in_bf16 = p->in_dtype == CONV2D_BF16;
  q->out_bf16 = p->out_dtype == CONV2D_BF16;
  return CONV2D_STATUS_OK;
}

void tile_shape(const Variant& v, int* bm, int* bn, int* bk) {
  if (v.family == kIgemm) igemm_tile_shape(v.bf16, v.tile, bm, bn, bk);
  else igemm_dma_tile_shape(v.bf16, v.tile, bm, bn, bk);
}

int occupancy(const Variant& v) {
  return v.family == kIgemm ? igemm_tile_occupancy(v.bf16, v.tile)
                            : igemm_dma_tile_occupancy(v.bf16, v.tile);
}

// Element-wise tiles: any C and K, pointers only 4-byte aligned.
bool is_scalar(const Variant& v) {
  if (v.family == kRowGather) return true;
  if (v.family == kIgemm) return igemm_tile_is_scalar(v.bf16, v.tile);
  return v.family == kDma && igemm_dma_tile_addressing(v.bf16, v.tile) == 2;
}

bool supports(const Variant& v, const Problem& q) {
  if (v.family == kDirect) return true;
  const int es = q.in_bf16 ? 2 : 4, vec = 16 / es;
  if (v.bf16 != q.in_bf16) return false;
  if (!q.in_bf16 && q.out_bf16) return false;
  // buffer addressing needs input and filter below 2^31 bytes
  if (1LL * es * q.N * q.H * q.W * q.C >= (1LL << 31)) return false;
  if (v.family == kWinograd) return winograd_supports(q, v.tile, v.split == kFused);
  if (v.family == kRowGather) return row_gather_supports(q);
  if (v.family == kWinogradLds) return winograd_lds_supports(q);
  if (v.family == kConv1x1) return conv1x1_supports(q, v.tile);
  if (v.family == kRegFilter) return conv3x3_regfilter_supports(q, v.tile);
  if (v.family == kPadded) {
    if (v.bf16 != q.in_bf16 || (!q.in_bf16 && q.out_bf16)) return false;
    return padded_supports(q, v.tile);
  }
  int bm, bn, bk;
  tile_shape(v, &bm, &bn, &bk);
  if (v.family == kIgemm) {
    if (1LL * es * q.Kg * q.K >= (1LL << 31)) return false;
    // 16-byte gathers need C and K in multiples of the vector
    if (!is_scalar(v) && (q.C % vec != 0 || q.K % vec != 0)) return false;
    if (v.split == kSplit && (q.Kg + bk - 1) / bk < 2) return false;  // nothing to split
    return true;
  }
  // direct-to-LDS tiles: filter rows in the workspace are padded to the slice
  // width; the input descriptor is extended by up to a window of bytes
  if ((!is_scalar(v) && q.C % vec != 0) || 1LL * es * (q.Kg + bk) * q.K >= (1LL << 31)) return false;
  if (1LL * es * (1LL * q.N * q.H * q.W + 1LL * q.R * q.W + q.S) * q.C >= (1LL << 31)) return false;
  if (igemm_dma_tile_addressing(v.bf16, v.tile) == 0 && (q.C % bk != 0 || q.R * q.S > 31)) return false;
  if (igemm_dma_tile_addressing(v.bf16, v.tile) == 3) {
    // patch tiles: whole tiles, or a split over the channel blocks where there are several
    if (!igemm_dma_tile_fits(q, v.bf16, v.tile) || v.split == kTail) return false;
    if (v.split == kSplit) return igemm_dma_tile_splits_channels(v.bf16, v.tile) && q.C / bk >= 2;
    return true;
  }
  if (igemm_dma_tile_native(v.bf16, v.tile) && !igemm_dma_tile_fits(q, v.bf16, v.tile)) return false;
  if (v.split == kSplit && (q.Kg + bk - 1) / bk < 2) return false;
  if (v.split == kTail) {
    // A balanced tail needs tiles left over after whole rounds of the 256
    // compute units.  With fewer whole tiles than resident workgroups every
    // tile would go to the tail: fine for a handful of tiles (the tail then
    // spreads their slices over the chip), but from one round of tiles on the
    // uneven pieces land on the units unbalanced and a uniform split is faster.
    const long long tiles = ceil_div_ll(q.M, bm) * ceil_div_ll(q.K, bn);
    const long long rest = tiles % 256;
    if (rest == 0) return false;
    if (tiles >= 256 && tiles - rest < 256LL * occupancy(v)) return false;
  }
  return true;
}

// Number of workgroups that share one output tile in a split-reduction
// variant: enough to give every compute unit its full set of resident
// workgroups, at least 2, and no split shorter than 4 slices unless the
// whole reduction is.
int split_factor(const Variant& v, const Problem& q) {
  if (v.split == kTail) return kTailBalanced;
  if (v.split != kSplit) return 1;
  int bm, bn, bk;
  tile_shape(v, &bm, &bn, &bk);
  const long long tiles = ceil_div_ll(q.M, bm) * ceil_div_ll(q.K, bn);
  if (tiles == 0) return 1;  // empty batch
  if (v.family == kDma && igemm_dma_tile_addressing(v.bf16, v.tile) == 3) {
    // Patch tiles split their channel blocks (nine slices each): one workgroup per compute
    // unit, no split shorter than four blocks unless that leaves a single one (a workgroup's
    // start and its burst of partial sums cost about two blocks' time).
    const int nblocks = q.C / bk;
    long long s = ceil_div_ll(256, tiles);
    const long long cap = nblocks / 4 > 2 ? nblocks / 4 : 2;
    if (s > cap) s = cap;
    if (s < 2) s = 2;
    if (s > nblocks) s = nblocks;
    return static_cast<int>(s);
  }
  const int nslices = (q.Kg + bk - 1) / bk;
  const long long target = 256LL * occupancy(v);
  long long s = ceil_div_ll(target, tiles);
  const long long cap = nslices / 4 > 2 ? nslices / 4 : 2;
  if (s > cap) s = cap;
  if (s < 2) s = 2;
  if (s > nslices) s = nslices;
  return static_cast<int>(s);
}

// Cost model of a variant on this device, in clock cycles of a compute unit
// (256 units; per unit and clock 128 fp32 or 2048 bf16 multiply-adds on the
// matrix cores).  The busiest unit works through its share of the K-slices;
// a slice costs the larger of its MFMA time at the family's sustained
// efficiency and the time to bring its operands into the unit, plus the load
// latency that the resident workgroups cannot hide between them (large for
// the register-staged family, which prefetches one slice, small for the
// direct-to-LDS pipeline).  On top come a start-up and drain time per round
// of resident workgroups, the filter repack of the direct-to-LDS family, the
// partial tiles of a split reduction or a balanced tail going through memory
// twice, and a fixed time per kernel launched.  The constants are a fit to
// the measured times of every variant on 210 random layer shapes in each
// element type on one MI355X (all families, Winograd included); with them
// the selector's pick is 3 percent slower than the best variant in the
// geometric mean.
struct ModelGroup {
  double eff;     // sustained fraction of the MFMA peak
  double bwcu;    // operand bytes per clock into one compute unit
  double lat;     // exposed load latency per slice, cycles, shared by the resident workgroups
  double pro;     // start-up and drain per round of workgroups, cycles
  double epi;     // epilogue cycles per output element of the tile
  double single;  // efficiency factor when a workgroup has its compute unit to itself
};
constexpr ModelGroup kModelDma[2] = {{0.8883, 137.8, 3.797, 2796.1, 0.3092, 0.7661},
                                     {0.5598, 41.55, 29.93, 8874.6, 0.03176, 1}};
constexpr ModelGroup kModelIgemm[2] = {{0.8179, 41.48, 537.2, 6614.4, 0.5328, 0.9163},
                                       {0.2657, 82.96, 529.2, 13765, 0.02623, 0.9554}};
constexpr double kLaunchCycles = 8605.2;       // per kernel launched
constexpr double kRepackPerByte = 0.0003335;     // filter repack, cycles per byte of filter
constexpr double kChipBytesPerClock = 12892;  // whole-chip streaming rate (cache-resident sizes)
constexpr double kPartialFactor = 6.942;      // partial tiles: cost relative to that rate
constexpr double kVectorGatherFactor = 0.8502;  // efficiency of the per-lane addressed tiles
constexpr double kElementFactor = 0.75;        // ... of the element-wise tiles
constexpr double kKSplitFactor = 0.9858;          // ... of the tiles whose waves split the k range
constexpr double kKSplitLatency = 0.3428;        // extra exposed latency per further k group (their slices are deeper)
constexpr double kWinogradLdsEff = 0.70;       // MFMA rate of the one-launch Winograd kernel's loop
constexpr double kPatchFactor = 1.246;         // ... of the LDS-resident patch tiles

// The balanced tail's plan as the launcher makes it: tiles computed whole,
// tail tiles, ranges the tail is cut into.
void tail_plan(const Variant& v, const Problem& q, long long* n_main, long long* rest,
               long long* ranges) {
  int bm, bn, bk;
  tile_shape(v, &bm, &bn, &bk);
  const long long tiles = ceil_div_ll(q.M, bm) * ceil_div_ll(q.K, bn);
  const long long nslices = (q.Kg + bk - 1) / bk;
  long long r = tiles % 256;
  if (tiles - r < 256LL * occupancy(v)) r = tiles;
  const long long units = r * nslices;
  const long long most = r > 256 ? 256 * ceil_div_ll(r, 256) : 256;
  long long w = units / 4 < most ? units / 4 : most;
  if (w < r) w = r;
  *n_main = tiles - r; *rest = r; *ranges = w;
}

double model_cost(const Variant& v, const Problem& q);

// Winograd F(2x2, 3x3): the 16 point-wise products cost what the gather tile
// costs on a 1x1 convolution over all 16 * tiles rows (at least the time to
// stream the transformed input and the products through memory, which do not
// fit the caches), plus the transform kernels' traffic and three more launches.
double winograd_cost(const Variant& v, const Problem& q) {
  const long long tiles = 1LL * q.N * ((q.P + 1) / 2) * ((q.Q + 1) / 2);
  const bool fused = v.split == kFused;  // products folded into the output: no Mt
  Problem g = {};
  g.N = 1; g.C = q.C; g.K = q.K; g.S = 1; g.sr = 1; g.sc = 1; g.P = 1;
  if (fused) {
    // one workgroup per block of tiles runs the 16 products one after the other
    g.H = 16; g.R = 16; g.W = static_cast<int>(tiles); g.Kg = 16 * q.C;
  } else {
    g.H = 1; g.R = 1; g.W = static_cast<int>(16 * tiles < 0x7fffffff ? 16 * tiles : 0x7fffffff);
    g.Kg = q.C;
  }
  g.Q = g.W; g.M = g.W;
  Variant inner = v;
  inner.family = kDma;
  inner.split = kWhole;
  const double memory_rate = 2083.3;  // bytes per clock from HBM (fitted)
  const double v_bytes = 4.0 * 16 * tiles * q.C;
  const double m_bytes = fused ? 0.0 : 4.0 * 16 * tiles * q.K;
  double product = model_cost(inner, g);
  const double product_stream = (v_bytes + m_bytes) / memory_rate;
  if (product < product_stream) product = product_stream;
  const double transforms =
      (4.0 * q.N * q.H * q.W * q.C + v_bytes + m_bytes + 4.0 * q.M * q.K) / memory_rate;
  return product + transforms + (fused ? 2 : 3) * kLaunchCycles;
}

double model_cost(const Variant& v, const Problem& q) {
  if (v.family == kWinograd) return winograd_cost(v, q);
  if (v.family == kRowGather) return row_gather_cost(q);
  if (v.family == kWinogradLds) {
    // 16 point products per 2x2 outputs on the matrix cores (16 / 36 of the direct sum's
    // multiplications) at the kernel's sustained rate, whole workgroups of 32 tiles x 64
    // features in rounds of two per compute unit; the filter transform is a launch of its own
    const long long tiles = 1LL * q.N * ((q.P + 1) / 2) * ((q.Q + 1) / 2);
    const long long wgs = ceil_div_ll(tiles, 32) * ceil_div_ll(q.K, 64);
    const double per_wg = 16.0 * 32 * 64 * q.C / 128.0 / kWinogradLdsEff + 6000.0;
    const double rounds = static_cast<double>(ceil_div_ll(wgs, 256));
    const double filter = 4.0 * q.C * q.K * (9.0 + 16.0) / kChipBytesPerClock;
    return rounds * per_wg + filter + 2 * kLaunchCycles;
  }
  if (v.family == kConv1x1) {
    // a stream: the larger of the products' time and the tensors' bytes at the chip's streaming
    // rate (the input is read once per slab of features), one launch, a persistent pipeline
    const double es = q.in_bf16 ? 2.0 : 4.0;
    const int bn = conv1x1_tile_features(v.tile);
    const double slabs = static_cast<double>(ceil_div_ll(q.K, bn));
    const double mfma = 1.0 * q.M * q.K * q.C / ((q.in_bf16 ? 2048.0 : 128.0) * 256.0) /
                        (q.in_bf16 ? 0.5 : 0.8);
    const double bytes = es * q.M * q.C * (slabs > 1 ? 1.3 : 1.0) + es * q.C * q.K * 256.0 +
                         (q.out_bf16 ? 2.0 : 4.0) * q.M * q.K;
    const double stream = bytes / 1900.0;
    return (mfma > stream ? mfma : stream) * 1.1 + 4000.0 + kLaunchCycles;
  }
  if (v.family == kRegFilter) {
    // a stream like the 1x1 kernel: the products at about half the MFMA rate or the tensors'
    // bytes at the chip's streaming rate, whichever is larger, one launch, tiles of 16x16
    // pixels (ragged blocks at the image edge are computed whole), 256 persistent workgroups
    const int rows = conv3x3_regfilter_tile_rows(v.tile);
    const double blocks = 1.0 * q.N * ceil_div_ll(q.P, rows) * ceil_div_ll(q.Q, 16);
    const double rounds = static_cast<double>(ceil_div_ll(static_cast<long long>(blocks), 256));
    const double mfma = rounds * rows * 16.0 * q.K * q.Kg / 2048.0 / 0.6;
    const double halo = (rows + 2.0) * 18.0 / (rows * 16.0);
    const double bytes = 2.0 * q.N * q.H * q.W * q.C * halo + (q.out_bf16 ? 2.0 : 4.0) * q.M * q.K;
    const double stream = bytes / 1900.0;
    // (the start: the filter through LDS into the registers of every workgroup)
    return (mfma > stream ? mfma : stream) * 1.05 + 4000.0 + 2.0 * q.Kg * q.K / 64.0 +
           kLaunchCycles;
  }
  if (v.family == kPadded) {
    // the gather tile on the padded problem, the padding passes' traffic, two more launches
    const int vec = q.in_bf16 ? 8 : 4;
    Problem g = q;
    g.C = (q.C + vec - 1) / vec * vec;
    g.Kg = q.R * q.S * g.C;
    Variant inner = v;
    inner.family = kDma;
    const double es = q.in_bf16 ? 2.0 : 4.0;
    const double pad_bytes = es * q.N * q.H * q.W * (q.C + g.C);
    return model_cost(inner, g) + pad_bytes / 2083.3 + 2 * kLaunchCycles;
  }
  int bm, bn, bk;
  tile_shape(v, &bm, &bn, &bk);
  const ModelGroup& g = v.family == kDma ? kModelDma[q.in_bf16] : kModelIgemm[q.in_bf16];
  const int addressing = v.family == kDma ? igemm_dma_tile_addressing(v.bf16, v.tile)
                                          : (is_scalar(v) ? 2 : 1);
  const long long tiles = ceil_div_ll(q.M, bm) * ceil_div_ll(q.K, bn);
  const long long nslices = (q.Kg + bk - 1) / bk;
  const double mac_rate = q.in_bf16 ? 2048.0 : 128.0;
  const double es = q.in_bf16 ? 2.0 : 4.0;
  const double area = 1.0 * bm * bn;
  double eff = g.eff;
  double slice_bytes = 1.0 * (bm + bn) * bk * es;
  double exposed_latency = g.lat;
  if (v.family == kIgemm && igemm_tile_waves_k(v.bf16, v.tile) > 1) {
    // small tiles whose waves split the slice: every MFMA reads both its fragments from LDS,
    // and a slice is waves_k times deeper than a plain tile's
    eff *= kKSplitFactor;
    exposed_latency *= 1.0 + kKSplitLatency * (igemm_tile_waves_k(v.bf16, v.tile) - 1);
  }
  if (addressing == 1 && v.family == kDma) eff *= kVectorGatherFactor;
  if (addressing == 2) eff *= kElementFactor;
  if (addressing == 3) {
    eff *= kPatchFactor;
    slice_bytes = (bm / 3.0 + bn) * bk * es;  // a 3x3 patch is loaded once for its taps
  }
  double slices_on_unit, extra = 0.0;
  long long wgs;
  int kernels = 1;
  if (v.split == kTail) {
    long long n_main, rest, ranges;
    tail_plan(v, q, &n_main, &rest, &ranges);
    slices_on_unit = (n_main / 256.0) * nslices + (1.0 * rest * nslices) / 256.0;
    if (n_main == 0) {  // two pieces of different ranges may share a unit
      const double two = 2.0 * rest * nslices / (ranges > 0 ? ranges : 1);
      if (two > slices_on_unit) slices_on_unit = two;
    }
    wgs = n_main + ranges;
    extra = kPartialFactor * 8.0 * (ranges + rest) * area / kChipBytesPerClock;
    ++kernels;
  } else {
    const int splits = split_factor(v, q);
    const long long per_split = ceil_div_ll(nslices, splits);
    wgs = tiles * splits;
    slices_on_unit = 1.0 * ceil_div_ll(wgs, 256) * per_split;
    if (splits > 1) {
      extra = kPartialFactor * 4.0 * q.M * q.K * (2 * splits + 1) / kChipBytesPerClock;
      ++kernels;
    }
  }
  const long long per_unit = ceil_div_ll(wgs, 256);
  const int occ = occupancy(v);
  const double resident = per_unit < occ ? static_cast<double>(per_unit) : occ;
  const long long rounds = ceil_div_ll(per_unit, occ);
  const double mfma = bm * bn * bk / mac_rate / (eff * (resident == 1 ? g.single : 1.0));
  const double feed = slice_bytes / g.bwcu;
  const double slice = (mfma > feed ? mfma : feed) + exposed_latency / resident;
  const double compute = slices_on_unit * slice;
  const double stream =
      (es * (1.0 * q.N * q.H * q.W * q.C + 1.0 * q.Kg * q.K) + 4.0 * q.M * q.K) / kChipBytesPerClock;
  double cost = (compute > stream ? compute : stream) + rounds * (g.pro + g.epi * area) + extra;
  if (v.family == kDma && !igemm_dma_tile_native(v.bf16, v.tile)) {
    ++kernels;
    cost += kRepackPerByte * es * q.Kg * q.K;
  }
  return cost + kernels * kLaunchCycles;
}

// Hand-tuned choices for known layer shapes (section 3: per-device manual
// tuning of algorithm and parameters), written by the tuning script.
struct Tuned {
  int bf16, n, h, w, c, k, r, s, sr, sc, padding;
  const char* variant;
};
const Tuned kTuned[] = {
#include "tuned_table.inc"
};

bool usable(const Variant& v, const Problem& q, bool aligned) {
  if (!supports(v, q)) return false;
  return aligned || v.family == kDirect || is_scalar(v);
}

// `direct_sum_only` leaves out the variants that reach the result through a
// transform (Winograd): fewer multiplications, a large workspace.  A shape
// may have two rows in the tuned table, the transform variant first.
// What a selection is for: any algorithm, the direct-sum variants only, or the pooled entry
// point (see select_uncached).
enum SelectMode { kAny = 0, kDirectSumOnly = 1, kForPooling = 2 };
int select_uncached(const Problem& q, int padding, bool aligned, int mode);
bool pools_in_epilogue(const Variant& v);

// The model path evaluates every variant (about 10 us of host time), which a
// layer of a few microseconds cannot afford on every call: each thread keeps
// its last selections in a small direct-mapped cache keyed on the parameters.
int select(const Problem& q, int padding, bool aligned, int mode) {
  struct Entry {
    int key[14];
    int variant;
    bool valid;
  };
  constexpr int kEntries = 64;
  thread_local Entry cache[kEntries] = {};
  const int key[14] = {q.N, q.H, q.W, q.C, q.K, q.R, q.S, q.sr, q.sc, padding, q.in_bf16,
                       q.out_bf16, aligned ? 1 : 0, mode};
  unsigned h = 2166136261u;
  for (int v : key) h = (h ^ static_cast<unsigned>(v)) * 16777619u;
  Entry& e = cache[h % kEntries];
  if (e.valid && std::memcmp(e.key, key, sizeof(key)) == 0) return e.variant;
  const int id = select_uncached(q, padding, aligned, mode);
  std::memcpy(e.key, key, sizeof(key));
  e.variant = id;
  e.valid = true;
  return id;
}

int select_uncached(const Problem& q, int padding, bool aligned, int mode) {
  const Table& tb = table();
  if (q.M == 0) return 0;  // empty batch: nothing is launched
  if (mode == kForPooling) {
    // The unrestricted pick, unless that is a patch tile that cannot pool (the 16-row tiles)
    // while a blocked patch tile that can is priced within 30 % of it and the layer is short
    // enough in the reduction for the second kernel to matter: measured on 3x3 layers at batch
    // 16 in bf16, 128 -> 128 channels 84.7 us with the second kernel against 64.5 us on a
    // pooling tile, 256 -> 256 69.2 against 60.7, but 512 -> 512 64.3 against 68.8 (the
    // unpooled tensor is small there and the 16-row tile is that much faster).  Other picks
    // (Winograd, gather tiles) keep the two-kernel path: the model is not sharp enough to
    // trade them against the pooling epilogue.
    const int any = select_uncached(q, padding, aligned, kAny);
    const Variant& a = tb.v[any];
    if (pools_in_epilogue(a) || a.family != kDma || igemm_dma_tile_addressing(a.bf16, a.tile) != 3)
      return any;
    if (q.Kg > 3000) return any;
    int best = any;
    double best_cost = 1.3 * model_cost(a, q);
    for (int i = 1; i < tb.n; ++i) {
      if (!usable(tb.v[i], q, aligned) || !pools_in_epilogue(tb.v[i])) continue;
      const double c = model_cost(tb.v[i], q);
      if (c < best_cost) { best = i; best_cost = c; }
    }
    return best;
  }
  const bool direct_sum_only = mode == kDirectSumOnly;
  for (const Tuned& t : kTuned) {
    if (t.bf16 == q.in_bf16 && t.n == q.N && t.h == q.H && t.w == q.W && t.c == q.C &&
        t.k == q.K && t.r == q.R && t.s == q.S && t.sr == q.sr && t.sc == q.sc &&
        t.padding == padding) {
      for (int i = 0; i < tb.n; ++i)
        if (std::strcmp(tb.v[i].name, t.variant) == 0 && usable(tb.v[i], q, aligned) &&
            !(direct_sum_only && is_winograd(tb.v[i].family)))
          return i;
    }
  }
  int best = 0;
  double best_cost = 0;
  const int vec = q.in_bf16 ? 8 : 4;
  for (int i = 1; i < tb.n; ++i) {
    const Variant& v = tb.v[i];
    if (!usable(v, q, aligned)) continue;
    if (direct_sum_only && is_winograd(v.family)) continue;
    // element-wise tiles only where the vector tiles cannot run
    if (v.family == kRowGather && q.C % vec == 0) continue;
    if (is_scalar(v) && aligned && q.C % vec == 0 && q.K % vec == 0) continue;
    const double c = model_cost(v, q);
    if (best == 0 || c < best_cost) { best = i; best_cost = c; }
  }
  return best;
}

size_t workspace_bytes_for(const Variant& v, const Problem& q) {
  if (v.family == kWinograd) return winograd_workspace_bytes(q, v.tile, v.split == kFused);
  if (v.family == kWinogradLds) return winograd_lds_workspace_bytes(q);
  if (v.family == kPadded) return padded_workspace_bytes(q, v.tile);
  if (v.family == kDma) return igemm_dma_workspace_bytes(q, v.bf16, v.tile, split_factor(v, q));
  if (v.family == kIgemm && v.split)
    return static_cast<size_t>(split_factor(v, q)) * q.M * q.K * sizeof(float);
  return 0;
}

size_t align256(size_t bytes) { return (bytes + 255) / 256 * 256; }

// Bytes of variant `v`'s packed filter (every family has one; *ok stays for a family without).
size_t packed_filter_bytes_for(const Variant& v, const Problem& q, bool* ok) {
  *ok = true;
  if (v.family == kPadded) return padded_packed_filter_bytes(q, v.tile);
  if (v.family == kDma) return igemm_dma_packed_filter_bytes(q, v.bf16, v.tile);
  if (v.family == kDirect || v.family == kIgemm || v.family == kRowGather ||
      v.family == kConv1x1 || v.family == kRegFilter)  // these read the filter as it is: a copy
    return align256(static_cast<size_t>(q.Kg) * q.K * (q.in_bf16 ? 2 : 4));
  if (v.family == kWinograd) return winograd_packed_filter_bytes(q, v.tile, v.split == kFused);
  if (v.family == kWinogradLds) return winograd_lds_packed_filter_bytes(q);
  *ok = false;
  return 0;
}

// The runtime's error code behind this thread's last LAUNCH_FAILED status.
thread_local hipError_t last_launch_error = hipSuccess;

// 2x2 pooling in the epilogue: whole blocked patch tiles.
bool pools_in_epilogue(const Variant& v) {
  // (the four outputs of a Winograd F(2x2, 3x3) tile are one pooling window: the output
  // transform, or the fused variant's epilogue, takes their maximum)
  if (is_winograd(v.family)) return true;
  return v.family == kDma && v.split == kWhole && igemm_dma_tile_pools(v.bf16, v.tile);
}


// Workspace of the pooled entry point with variant `v`: the variant's own, then (unless the
// variant pools in its epilogue) the unpooled output tensor.
size_t pooled_workspace_bytes_for(const Variant& v, const Problem& q) {
  const size_t own = workspace_bytes_for(v, q);
  if (pools_in_epilogue(v)) return own;
  return align256(own) + static_cast<size_t>(q.M) * q.K * (q.out_bf16 ? 2 : 4);
}

bool aligned16(const void* a, const void* b, const void* c) {
  return ((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b) |
           reinterpret_cast<uintptr_t>(c)) & 15u) == 0;
}

// Variant that the selecting entry points of the calling thread are told to run, or -1
// (conv2d_debug_force_variant).  The thread's first call takes the CONV2D_FORCE_VARIANT
// environment variable (a variant id) as its initial value, read once per process.
int& forced_variant_of_thread() {
  static const int from_environment = [] {
    const char* env = std::getenv("CONV2D_FORCE_VARIANT");
    return (env && *env) ? std::atoi(env) : -1;
  }();
  thread_local int forced = from_environment;
  return forced;
}
int forced_variant_from_environment() { return forced_variant_of_thread(); }

// The variant a selecting entry point runs for pointers of the given alignment.
int pick(const Problem& q, int padding, bool aligned, int mode) {
  const Table& tb = table();
  int id = select(q, padding, aligned, mode);
  const int forced = forced_variant_from_environment();
  if (forced >= 0 && forced < tb.n && usable(tb.v[forced], q, aligned)) id = forced;
  return id;
}

int run(const conv2d_params* params, const void* in, const void* filt, void* out, void* workspace,
        size_t workspace_bytes, void* hip_stream, int variant_id, const float* bias = nullptr,
        int activation = CONV2D_ACT_NONE, bool pool = false, bool filt_is_packed = false,
        int select_mode_override = -1) {
  Problem q;
  int rc = derive(params, &q);
  if (rc) return rc;
  const Table& tb = table();
  if (variant_id >= tb.n) return CONV2D_STATUS_INVALID_ARGUMENT;
  if (q.N == 0) return CONV2D_STATUS_OK;
  if (pool && (q.P < 2 || q.Q < 2)) return CONV2D_STATUS_OK;  // empty pooled tensor: nothing to do
  if (!in || !filt || !out) return CONV2D_STATUS_INVALID_ARGUMENT;
  const bool al = aligned16(in, filt, out);
  int id = variant_id;
  if (id < 0) {
    const int mode = select_mode_override >= 0 ? select_mode_override : (pool ? kForPooling : kAny);
    id = pick(q, params->padding, al, mode);
    if (!al) {
      // The size queries see no pointers and answer for 16-byte-aligned ones.  Pointers that are
      // only element-aligned get another pick, which may need more scratch than the caller was
      // told: then the cheapest usable variant that fits what the caller brought (the direct
      // kernel needs none).
      const size_t need0 = pool ? pooled_workspace_bytes_for(tb.v[id], q) : workspace_bytes_for(tb.v[id], q);
      if (need0 > 0 && (!workspace || workspace_bytes < need0)) {
        int best = -1;
        double best_cost = 0;
        for (int i = 0; i < tb.n; ++i) {
          if (!usable(tb.v[i], q, false)) continue;
          if (mode == kDirectSumOnly && is_winograd(tb.v[i].family)) continue;
          const size_t n = pool ? pooled_workspace_bytes_for(tb.v[i], q) : workspace_bytes_for(tb.v[i], q);
          if (n > 0 && (!workspace || workspace_bytes < n)) continue;
          const double c = tb.v[i].family == kDirect ? 1e300 : model_cost(tb.v[i], q);
          if (best < 0 || c < best_cost) { best = i; best_cost = c; }
        }
        if (best >= 0) id = best;
      }
    }
  } else {
    if (!supports(tb.v[id], q)) return CONV2D_STATUS_UNSUPPORTED;
    if (!al && tb.v[id].family != kDirect && !is_scalar(tb.v[id]))
      return CONV2D_STATUS_UNSUPPORTED;
  }
  const bool fused_pool = pool && pools_in_epilogue(tb.v[id]);
  const size_t need = pool ? pooled_workspace_bytes_for(tb.v[id], q) : workspace_bytes_for(tb.v[id], q);
  if (need > 0) {
    if (!workspace || workspace_bytes < need) return CONV2D_STATUS_WORKSPACE_TOO_SMALL;
    if (reinterpret_cast<uintptr_t>(workspace) & 15u) return CONV2D_STATUS_INVALID_ARGUMENT;
  }
  q.in = in; q.filt = filt; q.out = out; q.workspace = workspace;
  // (a packed filter of the direct and register-staged variants is a plain copy)
  if (filt_is_packed && (tb.v[id].family == kDma || is_winograd(tb.v[id].family) ||
                         tb.v[id].family == kPadded))
    q.packed_filt = filt;
  q.bias = bias;
  q.relu = activation == CONV2D_ACT_RELU;
  q.pool = fused_pool ? 1 : 0;
  // (a variant that cannot pool writes the unpooled tensor behind its own workspace)
  void* unpooled = nullptr;
  if (pool && !fused_pool) {
    unpooled = static_cast<char*>(workspace) + align256(workspace_bytes_for(tb.v[id], q));
    q.out = unpooled;
  }
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  // (an error that some earlier, unrelated runtime call of the process left behind is not
  // this call's: the launchers below report through hipGetLastError)
  (void)hipGetLastError();
  hipError_t e = hipSuccess;
  switch (tb.v[id].family) {
    case kDirect: e = launch_direct(q, stream); break;
    case kIgemm:
      e = launch_igemm(q, tb.v[id].bf16, tb.v[id].tile, split_factor(tb.v[id], q), stream);
      break;
    case kDma:
      e = launch_igemm_dma(q, tb.v[id].bf16, tb.v[id].tile, split_factor(tb.v[id], q), stream);
      break;
    case kPadded: e = launch_padded(q, tb.v[id].tile, stream); break;
    case kRowGather: e = launch_row_gather(q, stream); break;
    case kConv1x1: e = launch_conv1x1(q, tb.v[id].tile, stream); break;
    case kRegFilter: e = launch_conv3x3_regfilter(q, tb.v[id].tile, stream); break;
    case kWinograd:
      e = launch_winograd(q, tb.v[id].tile, tb.v[id].split == kFused, stream);
      break;
    case kWinogradLds: e = launch_winograd_lds(q, stream); break;
  }
  if (e == hipSuccess && unpooled)
    e = launch_max_pool_2x2(unpooled, out, q.N, q.P, q.Q, q.K, q.out_bf16 != 0, stream);
  if (e != hipSuccess) last_launch_error = e;
  return e == hipSuccess ? CONV2D_STATUS_OK : CONV2D_STATUS_LAUNCH_FAILED;
}

}  // namespace
}  // namespace conv2d

using namespace conv2d;

// ---- scratch memory of the entry point that allocates nothing -------------------------------
// conv2d_forward_static_scratch runs conv2d_forward's kernels with the repacked filter and the
// partial sums of a split reduction in this array instead of a caller's workspace.  Every GPU
// that loads the library holds its own copy until the process ends.  In host code the array's
// name is only a handle for hipGetSymbolAddress; the device address is looked up once per
// device and that pointer is what the kernels get.
namespace {
constexpr size_t kStaticScratchBytes = CONV2D_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
}  // namespace
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
namespace {
std::mutex scratch_mutex;
void* scratch_ptr[kMaxDevices] = {};

// The current device's copy of `scratch`; null (and *err set) if the runtime refuses.
void* static_scratch_of_current_device(hipError_t* err) {
  int dev = 0;
  *err = hipGetDevice(&dev);
  if (*err != hipSuccess) return nullptr;
  if (dev < 0 || dev >= kMaxDevices) {
    *err = hipErrorInvalidDevice;
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_ptr[dev]) {
    void* ptr = nullptr;
    *err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (*err != hipSuccess) return nullptr;
    scratch_ptr[dev] = ptr;
  }
  return scratch_ptr[dev];
}
}  // namespace

extern "C" {

int conv2d_get_geometry(const conv2d_params* params, conv2d_geometry* geometry) {
  if (!geometry) return CONV2D_STATUS_INVALID_ARGUMENT;
  conv2d_geometry g;
  const int rc = validate(params, &g);
  // an unsupported dtype pair still has a geometry
  if (rc == CONV2D_STATUS_OK || rc == CONV2D_STATUS_UNSUPPORTED) *geometry = g;
  return rc;
}

int conv2d_workspace_size(const conv2d_params* params, size_t* bytes) {
  Problem q;
  if (!bytes) return CONV2D_STATUS_INVALID_ARGUMENT;
  int rc = derive(params, &q);
  if (rc) return rc;
  *bytes = workspace_bytes_for(table().v[pick(q, params->padding, true, kAny)], q);
  return CONV2D_STATUS_OK;
}

int conv2d_workspace_size_variant(const conv2d_params* params, int variant_id, size_t* bytes) {
  Problem q;
  if (!bytes) return CONV2D_STATUS_INVALID_ARGUMENT;
  int rc = derive(params, &q);
  if (rc) return rc;
  const Table& tb = table();
  if (variant_id < 0 || variant_id >= tb.n) return CONV2D_STATUS_INVALID_ARGUMENT;
  if (!supports(tb.v[variant_id], q)) return CONV2D_STATUS_UNSUPPORTED;
  *bytes = workspace_bytes_for(tb.v[variant_id], q);
  return CONV2D_STATUS_OK;
}

int conv2d_forward(const conv2d_params* params, const void* in, const void* filt, void* out,
                   void* workspace, size_t workspace_bytes, void* hip_stream) {
  return run(params, in, filt, out, workspace, workspace_bytes, hip_stream, -1);
}

int conv2d_forward_static_scratch(const conv2d_params* params, const void* in, const void* filt,
                                  void* out, void* hip_stream) {
  Problem q;
  int rc = derive(params, &q);
  if (rc) return rc;
  if (q.N == 0) return CONV2D_STATUS_OK;
  if (!in || !filt || !out) return CONV2D_STATUS_INVALID_ARGUMENT;
  // conv2d_forward's pick among the direct-sum variants (the transform variants need several
  // times the input as scratch), then the same kernels on the library's own array
  const int id = pick(q, params->padding, aligned16(in, filt, out), kDirectSumOnly);
  const size_t need = workspace_bytes_for(table().v[id], q);
  if (need > kStaticScratchBytes) return CONV2D_STATUS_SCRATCH_EXCEEDED;
  void* ws = nullptr;
  if (need > 0) {
    hipError_t e = hipSuccess;
    ws = static_scratch_of_current_device(&e);
    if (!ws) {
      last_launch_error = e;
      return CONV2D_STATUS_LAUNCH_FAILED;
    }
  }
  return run(params, in, filt, out, ws, need, hip_stream, id);
}

int conv2d_forward_variant(const conv2d_params* params, const void* in, const void* filt, void* out,
                           void* workspace, size_t workspace_bytes, void* hip_stream,
                           int variant_id) {
  if (variant_id < 0) return CONV2D_STATUS_INVALID_ARGUMENT;
  return run(params, in, filt, out, workspace, workspace_bytes, hip_stream, variant_id);
}

int conv2d_forward_bias_act(const conv2d_params* params, const void* in, const void* filt,
                            const float* bias, int activation, void* out, void* workspace,
                            size_t workspace_bytes, void* hip_stream) {
  if (activation != CONV2D_ACT_NONE && activation != CONV2D_ACT_RELU)
    return CONV2D_STATUS_INVALID_ARGUMENT;
  if (bias && (reinterpret_cast<uintptr_t>(bias) & 3u)) return CONV2D_STATUS_INVALID_ARGUMENT;
  return run(params, in, filt, out, workspace, workspace_bytes, hip_stream, -1, bias, activation);
}

int conv2d_pool_workspace_size(const conv2d_params* params, size_t* bytes) {
  Problem q;
  if (!bytes) return CONV2D_STATUS_INVALID_ARGUMENT;
  int rc = derive(params, &q);
  if (rc) return rc;
  *bytes = pooled_workspace_bytes_for(table().v[pick(q, params->padding, true, kForPooling)], q);
  return CONV2D_STATUS_OK;
}

int conv2d_pool_workspace_size_variant(const conv2d_params* params, int variant_id,
                                       size_t* bytes) {
  Problem q;
  if (!bytes) return CONV2D_STATUS_INVALID_ARGUMENT;
  int rc = derive(params, &q);
  if (rc) return rc;
  const Table& tb = table();
  if (variant_id < 0 || variant_id >= tb.n) return CONV2D_STATUS_INVALID_ARGUMENT;
  if (!supports(tb.v[variant_id], q)) return CONV2D_STATUS_UNSUPPORTED;
  *bytes = pooled_workspace_bytes_for(tb.v[variant_id], q);
  return CONV2D_STATUS_OK;
}

int conv2d_forward_bias_act_pool(const conv2d_params* params, const void* in, const void* filt,
                                 const float* bias, int activation, void* out, void* workspace,
                                 size_t workspace_bytes, void* hip_stream) {
  if (activation != CONV2D_ACT_NONE && activation != CONV2D_ACT_RELU)
    return CONV2D_STATUS_INVALID_ARGUMENT;
  if (bias && (reinterpret_cast<uintptr_t>(bias) & 3u)) return CONV2D_STATUS_INVALID_ARGUMENT;
  return run(params, in, filt, out, workspace, workspace_bytes, hip_stream, -1, bias, activation,
             true);
}

int conv2d_packed_filter_size(const conv2d_params* params, int variant_id, size_t* bytes) {
  Problem q;
  if (!bytes) return CONV2D_STATUS_INVALID_ARGUMENT;
  int rc = derive(params, &q);
  if (rc) return rc;
  const Table& tb = table();
  if (variant_id < 0 || variant_id >= tb.n) return CONV2D_STATUS_INVALID_ARGUMENT;
  if (!supports(tb.v[variant_id], q)) return CONV2D_STATUS_UNSUPPORTED;
  bool ok;
  *bytes = packed_filter_bytes_for(tb.v[variant_id], q, &ok);
  return ok ? CONV2D_STATUS_OK : CONV2D_STATUS_UNSUPPORTED;
}

int conv2d_pack_filter(const conv2d_params* params, int variant_id, const void* filt, void* packed,
                       size_t packed_bytes, void* hip_stream) {
  Problem q;
  int rc = derive(params, &q);
  if (rc) return rc;
  const Table& tb = table();
  if (variant_id < 0 || variant_id >= tb.n) return CONV2D_STATUS_INVALID_ARGUMENT;
  const Variant& v = tb.v[variant_id];
  if (!supports(v, q)) return CONV2D_STATUS_UNSUPPORTED;
  bool ok;
  const size_t need = packed_filter_bytes_for(v, q, &ok);
  if (!ok) return CONV2D_STATUS_UNSUPPORTED;
  if (!filt || !packed) return CONV2D_STATUS_INVALID_ARGUMENT;
  if (packed_bytes < need) return CONV2D_STATUS_WORKSPACE_TOO_SMALL;
  if (!is_scalar(v) && v.family != kDirect &&
      ((reinterpret_cast<uintptr_t>(filt) | reinterpret_cast<uintptr_t>(packed)) & 15u))
    return CONV2D_STATUS_UNSUPPORTED;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  (void)hipGetLastError();  // not this call's
  hipError_t e;
  if (v.family == kDma) {
    q.filt = filt;
    e = igemm_dma_pack_filter(q, v.bf16, v.tile, packed, stream);
  } else if (v.family == kWinograd) {
    q.filt = filt;
    e = winograd_pack_filter(q, v.tile, v.split == kFused, packed, stream);
  } else if (v.family == kWinogradLds) {
    q.filt = filt;
    e = winograd_lds_pack_filter(q, packed, stream);
  } else if (v.family == kPadded) {
    q.filt = filt;
    e = padded_pack_filter(q, v.tile, packed, stream);
  } else {
    e = hipMemcpyAsync(packed, filt, static_cast<size_t>(q.Kg) * q.K * (q.in_bf16 ? 2 : 4),
                       hipMemcpyDeviceToDevice, stream);
  }
  if (e != hipSuccess) last_launch_error = e;
  return e == hipSuccess ? CONV2D_STATUS_OK : CONV2D_STATUS_LAUNCH_FAILED;
}

int conv2d_forward_packed(const conv2d_params* params, int variant_id, const void* in,
                          const void* packed_filt, const float* bias, int activation, void* out,
                          void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (variant_id < 0) return CONV2D_STATUS_INVALID_ARGUMENT;
  if (activation != CONV2D_ACT_NONE && activation != CONV2D_ACT_RELU)
    return CONV2D_STATUS_INVALID_ARGUMENT;
  if (bias && (reinterpret_cast<uintptr_t>(bias) & 3u)) return CONV2D_STATUS_INVALID_ARGUMENT;
  {
    Problem q;
    int rc = derive(params, &q);
    if (rc) return rc;
    const Table& tb = table();
    if (variant_id >= tb.n) return CONV2D_STATUS_INVALID_ARGUMENT;
    bool ok;
    packed_filter_bytes_for(tb.v[variant_id], q, &ok);
    if (!ok) return CONV2D_STATUS_UNSUPPORTED;
  }
  return run(params, in, packed_filt, out, workspace, workspace_bytes, hip_stream, variant_id, bias,
             activation, false, true);
}

int conv2d_debug_force_variant(int variant_id) {
  if (variant_id < -1 || variant_id >= table().n) return CONV2D_STATUS_INVALID_ARGUMENT;
  forced_variant_of_thread() = variant_id;
  return CONV2D_STATUS_OK;
}

int conv2d_debug_split_reduce_separate(int on) {
  if (on != 0 && on != 1) return CONV2D_STATUS_INVALID_ARGUMENT;
  igemm_dma_split_reduce_separate(on != 0);
  return CONV2D_STATUS_OK;
}

int conv2d_num_variants(void) { return table().n; }

const char* conv2d_variant_name(int variant_id) {
  const Table& tb = table();
  return (variant_id >= 0 && variant_id < tb.n) ? tb.v[variant_id].name : nullptr;
}

int conv2d_variant_supports(const conv2d_params* params, int variant_id) {
  Problem q;
  int rc = derive(params, &q);
  if (rc) return rc;
  const Table& tb = table();
  if (variant_id < 0 || variant_id >= tb.n) return CONV2D_STATUS_INVALID_ARGUMENT;
  return supports(tb.v[variant_id], q) ? 1 : 0;
}

int conv2d_selected_variant(const conv2d_params* params, int* variant_id) {
  Problem q;
  if (!variant_id) return CONV2D_STATUS_INVALID_ARGUMENT;
  int rc = derive(params, &q);
  if (rc) return rc;
  *variant_id = select(q, params->padding, true, kAny);
  return CONV2D_STATUS_OK;
}

int conv2d_select_variant(const conv2d_params* params, uint32_t flags, int* variant_id) {
  Problem q;
  if (!variant_id || (flags & ~static_cast<uint32_t>(CONV2D_SELECT_DIRECT_SUM_ONLY)))
    return CONV2D_STATUS_INVALID_ARGUMENT;
  int rc = derive(params, &q);
  if (rc) return rc;
  *variant_id = select(q, params->padding, true,
                       (flags & CONV2D_SELECT_DIRECT_SUM_ONLY) ? kDirectSumOnly : kAny);
  return CONV2D_STATUS_OK;
}

const char* conv2d_status_string(int status) {
  switch (status) {
    case CONV2D_STATUS_OK: return "ok";
    case CONV2D_STATUS_INVALID_ARGUMENT: return "invalid argument";
    case CONV2D_STATUS_UNSUPPORTED: return "unsupported by this variant";
    case CONV2D_STATUS_WORKSPACE_TOO_SMALL: return "workspace too small";
    case CONV2D_STATUS_LAUNCH_FAILED: return "kernel launch failed";
    case CONV2D_STATUS_TOO_LARGE: return "tensor too large for 31-bit indexing";
    case CONV2D_STATUS_SCRATCH_EXCEEDED:
      return "layer needs more scratch than the library's static array holds";
  }
  return "unknown status";
}

const char* conv2d_last_launch_error(void) {
  return last_launch_error == hipSuccess ? "" : hipGetErrorString(last_launch_error);
}

int conv2d_version(void) { return 100; }

}  // extern "C"
