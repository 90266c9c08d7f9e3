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

#include <cstdlib>
#include <cstring>

#include "conv2d_internal.h"

namespace conv2d {
namespace {

constexpr long long kMaxElems = (1LL << 31) - 1;

enum Family { kDirect = 0, kIgemmF32 = 1, kIgemmBf16 = 2, kDmaF32 = 3, kDmaBf16 = 4 };

struct Variant {
  Family family;
  int tile;
  const char* name;
};

// Variant table: id 0 is the direct kernel (supports everything), then the
// fp32 implicit-GEMM tiles, then the bf16 ones.
struct Table {
  Variant v[64];
  int n;
  Table() : n(0) {
    v[n++] = {kDirect, 0, "direct"};
    for (int t = 0; t < igemm_f32_num_tiles(); ++t) v[n++] = {kIgemmF32, t, igemm_f32_tile_name(t)};
    for (int t = 0; t < igemm_bf16_num_tiles(); ++t)
      v[n++] = {kIgemmBf16, t, igemm_bf16_tile_name(t)};
    for (int t = 0; t < igemm_dma_num_tiles(0); ++t) v[n++] = {kDmaF32, t, igemm_dma_tile_name(0, t)};
    for (int t = 0; t < igemm_dma_num_tiles(1); ++t) v[n++] = {kDmaBf16, t, igemm_dma_tile_name(1, t)};
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

bool supports(const Variant& v, const Problem& q) {
  switch (v.family) {
    case kDirect:
      return true;
    case kIgemmF32:
      // 16-byte gathers need C and K in multiples of 4; buffer addressing
      // needs input and filter below 2^31 bytes
      return !q.in_bf16 && !q.out_bf16 && q.C % 4 == 0 && q.K % 4 == 0 &&
             4LL * q.N * q.H * q.W * q.C < (1LL << 31) && 4LL * q.Kg * q.K < (1LL << 31);
    case kIgemmBf16:
      return q.in_bf16 && q.C % 8 == 0 && q.K % 8 == 0 &&
             2LL * q.N * q.H * q.W * q.C < (1LL << 31) && 2LL * q.Kg * q.K < (1LL << 31);
    case kDmaF32:  // the repacked filter rows are padded to 32 (fp32) / 64 (bf16) k
      return !q.in_bf16 && !q.out_bf16 && q.C % 4 == 0 &&
             4LL * q.N * q.H * q.W * q.C < (1LL << 31) && 4LL * (q.Kg + 32) * q.K < (1LL << 31);
    case kDmaBf16:
      return q.in_bf16 && q.C % 8 == 0 &&
             2LL * q.N * q.H * q.W * q.C < (1LL << 31) && 2LL * (q.Kg + 64) * q.K < (1LL << 31);
  }
  return false;
}

// Hand-tuned choice of tile for one device (MI355X: 256 compute units, two
// 256-thread workgroups of these kernels resident per unit).
int pick_tile(const Problem& q, Family family, int ntiles, void (*shape)(int, int*, int*, int*)) {
  // Widest feature tile that K fills, then the tallest pixel tile that still
  // gives every compute unit about two workgroups.
  const long long slots = 512;
  int best = -1;
  long long best_score = -1;
  for (int t = 0; t < ntiles; ++t) {
    int bm, bn, bk;
    const Variant cand = {family, t, ""};
    if (!supports(cand, q)) continue;
    shape(t, &bm, &bn, &bk);
    const long long tm = ceil_div_ll(q.M, bm), tn = ceil_div_ll(q.K, bn);
    const long long wgs = tm * tn;
    // useful fraction of the launched tile area, times a machine-fill factor
    const double useful = (1.0 * q.M * q.K) / (1.0 * tm * bm * tn * bn);
    const long long waves = ceil_div_ll(wgs, slots);
    const double fill = 1.0 * wgs / (1.0 * waves * slots);
    // larger tiles reuse LDS operands better
    const double reuse = 1.0 - 0.5 * (32.0 / bm + 32.0 / bn) * 0.5;
    const long long score = static_cast<long long>(1e6 * useful * fill * reuse);
    if (score > best_score) { best_score = score; best = t; }
  }
  return best;
}

int select(const Problem& q, bool aligned) {
  const Table& tb = table();
  if (aligned) {
    if (!q.in_bf16 && igemm_f32_num_tiles() > 0) {
      {
        const int t = pick_tile(q, kIgemmF32, igemm_f32_num_tiles(), igemm_f32_tile_shape);
        for (int i = 0; i < tb.n; ++i)
          if (tb.v[i].family == kIgemmF32 && tb.v[i].tile == t) return i;
      }
    }
    if (q.in_bf16 && igemm_bf16_num_tiles() > 0) {
      {
        const int t = pick_tile(q, kIgemmBf16, igemm_bf16_num_tiles(), igemm_bf16_tile_shape);
        for (int i = 0; i < tb.n; ++i)
          if (tb.v[i].family == kIgemmBf16 && tb.v[i].tile == t) return i;
      }
    }
  }
  return 0;
}

size_t workspace_bytes_for(const Variant& v, const Problem& q) {
  if (v.family == kDmaF32) return igemm_dma_workspace_bytes(q, 0, v.tile);
  if (v.family == kDmaBf16) return igemm_dma_workspace_bytes(q, 1, v.tile);
  return 0;
}

bool aligned16(const void* a, const void* b, const void* c) {
  return ((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b) |
           reinterpret_cast<uintptr_t>(c)) & 15u) == 0;
}

int run(const conv2d_params* params, const void* in, const void* filt, void* out, void* workspace,
        size_t workspace_bytes, void* hip_stream, int variant_id) {
  Problem q;
  int rc = derive(params, &q);
  if (rc) return rc;
  const Table& tb = table();
  if (variant_id >= tb.n) return CONV2D_STATUS_INVALID_ARGUMENT;
  if (q.N == 0) return CONV2D_STATUS_OK;
  if (!in || !filt || !out) return CONV2D_STATUS_INVALID_ARGUMENT;
  const bool al = aligned16(in, filt, out);
  int id = variant_id;
  if (id < 0) {
    id = select(q, al);
    const char* env = std::getenv("CONV2D_FORCE_VARIANT");
    if (env && *env) {
      const int forced = std::atoi(env);
      if (forced >= 0 && forced < tb.n && supports(tb.v[forced], q) &&
          (al || tb.v[forced].family == kDirect))
        id = forced;
    }
  } else {
    if (!supports(tb.v[id], q)) return CONV2D_STATUS_UNSUPPORTED;
    if (!al && tb.v[id].family != kDirect) return CONV2D_STATUS_UNSUPPORTED;
  }
  const size_t need = workspace_bytes_for(tb.v[id], q);
  if (need > 0) {
    if (!workspace || workspace_bytes < need) return CONV2D_STATUS_WORKSPACE_TOO_SMALL;
    if (reinterpret_cast<uintptr_t>(workspace) & 15u) return CONV2D_STATUS_INVALID_ARGUMENT;
  }
  q.in = in; q.filt = filt; q.out = out; q.workspace = workspace;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  hipError_t e = hipSuccess;
  switch (tb.v[id].family) {
    case kDirect: e = launch_direct(q, stream); break;
    case kIgemmF32: e = launch_igemm_f32(q, tb.v[id].tile, stream); break;
    case kIgemmBf16: e = launch_igemm_bf16(q, tb.v[id].tile, stream); break;
    case kDmaF32: e = launch_igemm_dma(q, 0, tb.v[id].tile, stream); break;
    case kDmaBf16: e = launch_igemm_dma(q, 1, tb.v[id].tile, stream); break;
  }
  return e == hipSuccess ? CONV2D_STATUS_OK : CONV2D_STATUS_LAUNCH_FAILED;
}

}  // namespace
}  // namespace conv2d

using namespace conv2d;

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
  *bytes = workspace_bytes_for(table().v[select(q, true)], q);
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

int conv2d_forward_variant(const conv2d_params* params, const void* in, const void* filt, void* out,
                           void* workspace, size_t workspace_bytes, void* hip_stream,
                           int variant_id) {
  if (variant_id < 0) return CONV2D_STATUS_INVALID_ARGUMENT;
  return run(params, in, filt, out, workspace, workspace_bytes, hip_stream, variant_id);
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
  *variant_id = select(q, true);
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
  }
  return "unknown status";
}

int conv2d_version(void) { return 100; }

}  // extern "C"
