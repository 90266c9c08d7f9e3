// Internal declarations shared by the host API and the HIP kernels of the
// forward convolution library.  Not part of the public C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace conv2d {

// A fully derived problem: the public parameter tuple (Figure 1's caption in
// the paper) plus output size and leading pads.  Implicit-GEMM view:
//   M = N*P*Q output pixels, K output features, Kg = R*S*C reduction length
//   ordered (r, s, c) so that the HWCF filter is the row-major [Kg][K] matrix
//   and the NHWC output is the row-major [M][K] matrix.
struct Problem {
  int N, H, W, C, K;
  int R, S, sr, sc;
  int pt, pl;
  int P, Q;
  int M;        // N*P*Q
  int Kg;       // R*S*C
  int in_bf16;  // 0: fp32 input/filter, 1: bf16
  int out_bf16; // 0: fp32 output, 1: bf16
  const void* in;
  const void* filt;
  void* out;
  void* workspace;
  // The filter already in the repacked form of the direct-to-LDS tile that runs (written by
  // igemm_dma_pack_filter / winograd_pack_filter for the same tile and parameters), or null:
  // the launch transforms and repacks `filt` into the workspace first.
  const void* packed_filt;
  // Fused epilogue: out = act(sum + bias[k]).  bias: K fp32 values on the
  // device, or null; relu: 0 or 1.
  const float* bias;
  int relu;
  // Fused 2x2 max pooling (stride 2, trailing odd row / column dropped): only
  // for tiles with igemm_dma_tile_pools and for the Winograd variants (a tile's
  // four outputs are one window); `out` is then [N][P/2][Q/2][K].
  int pool;
  // Batched launch of the direct-to-LDS gather kernels (used by the Winograd
  // path for its per-point matrix products): `batches` > 1 problems of this
  // shape whose input, filter and output start `*_stride` elements apart.
  int batches;
  long long in_stride, filt_stride, out_stride;
  // Winograd product with fused output transform (see launch_igemm_dma_wino):
  // tiles per image column and row, and the real output size.
  int wino_th, wino_tw, wino_p, wino_q;
};

// The fused epilogue on one finished sum of feature `col`.  A NaN sum stays
// NaN.  Tile epilogues fetch the bias of their column once (bias_of) and
// apply it to all rows (finish with the value): the output stores in between
// may alias the bias as far as the compiler knows, so a load per element
// would not be hoisted.
__device__ __forceinline__ float bias_of(const float* __restrict__ bias, int col, int K) {
  return (bias && col < K) ? bias[col] : 0.f;
}
__device__ __forceinline__ float finish(float v, float bias_value, int relu) {
  v += bias_value;
  if (relu) v = v < 0.f ? 0.f : v;
  return v;
}

// Window-row gather kernels for layers of at most 4 channels (row_gather.hip; fp32, and bf16
// where the pixels of a row are an even number of values apart): supported
// problems, modelled cost in clock cycles, launch.  No workspace; reads the filter as it is.
bool row_gather_supports(const Problem& p);
double row_gather_cost(const Problem& p);
hipError_t launch_row_gather(const Problem& p, hipStream_t stream);

// Streaming kernel for 1x1 windows (conv1x1.hip): persistent workgroups, the filter slab of
// `features` output features resident in LDS as it lies in memory, loads and stores issued by
// different wavefronts.  No workspace.
int conv1x1_num_tiles();
const char* conv1x1_tile_name(int tile);
int conv1x1_tile_bf16(int tile);
int conv1x1_tile_features(int tile);
bool conv1x1_supports(const Problem& p, int tile);
hipError_t launch_conv1x1(const Problem& p, int tile, hipStream_t stream);

// 3x3, stride-1 bf16 layers with 64 channels and 64 features, or 128 and 128
// (conv3x3_regfilter.hip): persistent workgroups that keep the whole filter in registers and
// stream tiles of `rows` x 16 pixels through a double-buffered LDS patch.  No workspace; reads
// the filter as it is.
int conv3x3_regfilter_num_tiles();
const char* conv3x3_regfilter_tile_name(int tile);
int conv3x3_regfilter_tile_rows(int tile);
bool conv3x3_regfilter_supports(const Problem& p, int tile);
hipError_t launch_conv3x3_regfilter(const Problem& p, int tile, hipStream_t stream);

// Launchers (one per kernel family).  Each returns hipSuccess or the launch
// error; none synchronises.  `tile` selects a compiled tile configuration.
hipError_t launch_direct(const Problem& p, hipStream_t stream);

// Register-staged implicit GEMM (fp32 on v_mfma_f32_32x32x2_f32, bf16 on
// v_mfma_f32_32x32x16_bf16).  `splits` > 1 splits the reduction over that many
// workgroups per output tile and needs splits*M*K floats of workspace.
int igemm_num_tiles(int bf16);
const char* igemm_tile_name(int bf16, int tile);
void igemm_tile_shape(int bf16, int tile, int* bm, int* bn, int* bk);
int igemm_tile_occupancy(int bf16, int tile);   // workgroups per compute unit
bool igemm_tile_is_scalar(int bf16, int tile);  // element-wise loads: any C, K, alignment
int igemm_tile_waves_k(int bf16, int tile);     // wave groups that split a slice's k range (1 = none)
hipError_t launch_igemm(const Problem& p, int bf16, int tile, int splits, hipStream_t stream);

// Adds `splits` fp32 partial outputs of `total` elements each (laid out one
// after the other at `partial`) in a fixed order, applies the fused epilogue
// (feature = index % K) and stores the result to `out` as fp32 or bf16.
hipError_t launch_split_reduce(const float* partial, void* out, int total, int splits,
                               bool out_bf16, const float* bias, int relu, int K,
                               hipStream_t stream);
// The order of its additions: `groups` sums, group g over the splits g, g + groups, ... from
// zero, then group 0's sum + group 1's + ...  (The reduction inside a launch adds in the same
// order, so both give the same bits.)
int split_reduce_groups(int total, int splits);

// Value of `splits` that asks the direct-to-LDS kernels for whole tiles plus
// a balanced tail instead of a uniform split.
constexpr int kTailBalanced = -1;

// Implicit GEMM with a multi-stage LDS ring fed by direct global->LDS loads.
// The workspace holds the repacked (k-contiguous) filter and, for splits > 1,
// the fp32 partial outputs.  Addressing kinds of a tile: 0 = "uniform" (C a
// multiple of the tile's bk and a window of at most 31 taps), 1 = vector (C a
// multiple of the 16-byte vector), 2 = element-wise (fp32, any C and K, any
// 4-byte alignment of input, filter and output), 3 = LDS-resident input
// patch (3x3 window, stride 1, C a multiple of bk, tiles whose patch fits;
// whole tiles only).
int igemm_dma_num_tiles(int bf16);
const char* igemm_dma_tile_name(int bf16, int tile);
void igemm_dma_tile_shape(int bf16, int tile, int* bm, int* bn, int* bk);
int igemm_dma_tile_occupancy(int bf16, int tile);
int igemm_dma_tile_addressing(int bf16, int tile);
bool igemm_dma_tile_fits(const Problem& p, int bf16, int tile);  // extra shape condition (kind 3)
// Tiles that are blocks of output pixels of one image with an even number of
// rows and columns: a 2x2 pooling window never leaves the tile, and with
// Problem::pool the epilogue reduces the four sums in registers (bias and
// activation after the maximum: both are monotone) and stores the pooled
// tensor only.
bool igemm_dma_tile_pools(int bf16, int tile);
// Tiles that read the filter as it lies in memory (no repacked copy, no launch before the
// convolution); their packed filter is a plain copy.
bool igemm_dma_tile_native(int bf16, int tile);
// Patch tiles (kind 3) that can split the channel blocks of a tile over several workgroups (a
// split reduction: splits * M * K fp32 partial sums in the workspace behind the repacked
// filter): one tile per workgroup, wave tiles of up to 128 x 64.
bool igemm_dma_tile_splits_channels(int bf16, int tile);
// The repacked filter of a tile (slice-major, k contiguous, zero padded to whole slices) as a
// tensor of its own: its size and the kernel that writes it from p.filt.  A launch with
// Problem::packed_filt set to it skips its own repack.
size_t igemm_dma_packed_filter_bytes(const Problem& p, int bf16, int tile);
hipError_t igemm_dma_pack_filter(const Problem& p, int bf16, int tile, void* packed,
                                 hipStream_t stream);
// (a batched problem holds one repacked filter per batch and takes whole tiles only)
size_t igemm_dma_workspace_bytes(const Problem& p, int bf16, int tile, int splits);
hipError_t launch_igemm_dma(const Problem& p, int bf16, int tile, int splits, hipStream_t stream);
// A uniform split of the reduction (splits > 1) adds its partial sums inside the convolution
// launch where it can (the last workgroup of a tile to arrive adds them; counters in a device
// array of the library, one bank per stream).  `on`: always use the second launch instead
// (split_reduce_kernel), as streams under graph capture and outputs of too many tiles do anyway.
void igemm_dma_split_reduce_separate(bool on);
// The calling stream's bank of per-tile arrival counters for a split reduction inside the
// launch (one counter per output tile, all zero between launches), or null: a stream under
// graph capture, more tiles than a bank has counters, all banks taken, or the switch above.
unsigned* split_counters_for_stream(hipStream_t stream, int tiles);

// The Winograd F(2x2, 3x3) point products with the output transform folded
// in, on a direct-to-LDS tile that has such an instantiation
// (igemm_dma_tile_has_wino).  `p` describes the transformed input V as an
// image of 16 rows (the points) by `tiles` columns and the transformed
// filter U as a 16x1 window (VALID, stride 1), so that the reduction runs
// point by point over the channels; every C / bk slices the kernel folds the
// finished point product into the four output pixels of each tile with the
// signs of A^T (x) A^T, and the epilogue stores those (p.wino_* give the
// tiling and the real output size, p.out the NHWC output).  Needs C a
// multiple of bk.  Workspace: the repacked U (igemm_dma_workspace_bytes(p, ..., 1)).
bool igemm_dma_tile_has_wino(int bf16, int tile);
hipError_t launch_igemm_dma_wino(const Problem& p, int bf16, int tile, hipStream_t stream);

// Winograd F(2x2, 3x3), fp32, stride 1: filter, input and output transforms
// around one batched launch of direct-to-LDS tile `gemm_tile` (addressing kind
// 0 or 1) for the 16 point-wise matrix products.  The workspace holds the
// transformed filter, input and products and the batched launch's own
// workspace.
// `fused`: products and output transform in one launch (no Mt); needs a tile
// with igemm_dma_tile_has_wino and C a multiple of its bk.
bool winograd_supports(const Problem& p, int gemm_tile, bool fused);
size_t winograd_workspace_bytes(const Problem& p, int gemm_tile, bool fused);
hipError_t launch_winograd(const Problem& p, int gemm_tile, bool fused, hipStream_t stream);
// The filter transformed and repacked ahead of time (Problem::packed_filt of a later launch).
size_t winograd_packed_filter_bytes(const Problem& p, int gemm_tile, bool fused);
hipError_t winograd_pack_filter(const Problem& p, int gemm_tile, bool fused, void* packed,
                                hipStream_t stream);

// Winograd F(2x2, 3x3), fp32, stride 1, in one launch (winograd_lds.hip): input transform,
// point products and output transform inside one workgroup; only the transformed filter goes
// through memory (the workspace, or a filter packed ahead of time).  Pools in its epilogue.
bool winograd_lds_supports(const Problem& p);
size_t winograd_lds_workspace_bytes(const Problem& p);
size_t winograd_lds_packed_filter_bytes(const Problem& p);
hipError_t winograd_lds_pack_filter(const Problem& p, void* packed, hipStream_t stream);
hipError_t launch_winograd_lds(const Problem& p, hipStream_t stream);

// 2x2 max pooling, stride 2, of the NHWC tensor `in` [N][P][Q][K] (fp32 or bf16)
// into `out` [N][P/2][Q/2][K] of the same type: the second step of the pooled
// entry point for variants that cannot pool in their epilogue.
hipError_t launch_max_pool_2x2(const void* in, void* out, int N, int P, int Q, int K, bool bf16,
                               hipStream_t stream);

// Small channel counts that are no multiple of the 16-byte vector (a 3-channel
// first layer): input and filter are zero-padded to the vector width in the
// workspace and per-lane addressed direct-to-LDS tile `gemm_tile` runs on the
// padded tensors.  The workspace holds the padded input and filter and the
// tile's own workspace.
bool padded_supports(const Problem& p, int gemm_tile);
size_t padded_workspace_bytes(const Problem& p, int gemm_tile);
hipError_t launch_padded(const Problem& p, int gemm_tile, hipStream_t stream);
// The filter padded and repacked ahead of time (Problem::packed_filt of a later launch).
size_t padded_packed_filter_bytes(const Problem& p, int gemm_tile);
hipError_t padded_pack_filter(const Problem& p, int gemm_tile, void* packed, hipStream_t stream);

}  // namespace conv2d
