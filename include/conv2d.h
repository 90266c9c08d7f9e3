/*
 * conv2d.h -- C ABI of the MI355X (gfx950) forward 2-D convolution library.
 *
 * The routine is the forward convolution that the paper (section 3,
 * "SYCL-DNN") names as its primary optimisation target; the parameter tuple
 * is the one in the caption of its Figure 1 (window, stride, image rows,
 * image columns, input features, output features) plus the batch size.  The
 * paper gives no formula, layout, padding rule or data type; the conventions
 * below are this library's:
 *
 *   out[n,p,q,k] = sum_{r,s,c} X(n, p*stride_rows + r - pad_top,
 *                                  q*stride_cols + s - pad_left, c) * filt[r,s,c,k]
 *   X(n,h,w,c) = in[n,h,w,c] inside the image, 0 outside      (cross-correlation)
 *
 *   in   : [batch][in_rows][in_cols][channels]            NHWC, dense
 *   filt : [window_rows][window_cols][channels][features] HWCF, dense
 *   out  : [batch][out_rows][out_cols][features]          NHWC, dense
 *
 *   VALID: out_rows = ceil((in_rows - window_rows + 1) / stride_rows), no padding.
 *   SAME : out_rows = ceil(in_rows / stride_rows); total padding
 *          max((out_rows-1)*stride_rows + window_rows - in_rows, 0), of which
 *          floor(total/2) goes before (top/left) and the rest after.
 *   Columns alike.  Dilation 1, one group; bias and activation only through
 *   conv2d_forward_bias_act.
 *
 * Section 3 also says the library offers several algorithms that give the
 * same numeric result and chooses among them (and among their parameters)
 * per device and shape, and Figure 1's caption notes that not every
 * algorithm supports every parameter set.  Here that is the "variant": a
 * kernel + tile configuration.  conv2d_forward picks one from the layer
 * shape; conv2d_forward_variant forces one and reports CONV2D_STATUS_UNSUPPORTED
 * when it cannot run the given parameters.
 *
 * General rules for every call:
 *   - All data pointers are DEVICE pointers owned by the caller; the library
 *     never allocates, frees or keeps them.  `in` and `filt` are only read;
 *     every element of `out` is written; `out` must not overlap the others.
 *   - `params` and the small out-parameters are HOST pointers.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = default stream).
 *     Calls only enqueue work on it and never synchronise.
 *   - Return value: CONV2D_STATUS_OK (0) or a negative conv2d_status_t.
 *     Parameter validation happens before any HIP call, so it also works on a
 *     host without a GPU.
 *   - Element type CONV2D_F32 is IEEE binary32, CONV2D_BF16 is bfloat16
 *     (upper 16 bits of binary32).  Accumulation is always fp32.
 */
#ifndef CONV2D_MI355X_H_
#define CONV2D_MI355X_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The library is built with hidden visibility; these are its only exports. */
#define CONV2D_API __attribute__((visibility("default")))

typedef enum { CONV2D_PAD_VALID = 0, CONV2D_PAD_SAME = 1 } conv2d_padding_t;
typedef enum { CONV2D_F32 = 0, CONV2D_BF16 = 1 } conv2d_dtype_t;

typedef enum {
  CONV2D_STATUS_OK = 0,
  CONV2D_STATUS_INVALID_ARGUMENT = -1,   /* null pointer, size <= 0, unknown enum, VALID window > image */
  CONV2D_STATUS_UNSUPPORTED = -2,        /* forced variant / dtype pair cannot run these parameters   */
  CONV2D_STATUS_WORKSPACE_TOO_SMALL = -3,
  CONV2D_STATUS_LAUNCH_FAILED = -4,      /* the HIP runtime rejected a launch                          */
  CONV2D_STATUS_TOO_LARGE = -5,          /* a tensor has 2^31 or more elements                         */
  CONV2D_STATUS_SCRATCH_EXCEEDED = -6    /* conv2d_forward_static_scratch: layer needs more scratch
                                            than CONV2D_STATIC_SCRATCH_BYTES                           */
} conv2d_status_t;

/* The parameter tuple of Figure 1's caption, plus batch, padding mode and
 * element types.  All sizes are element counts. */
typedef struct {
  int32_t batch;        /* N >= 0 (0 = no-op) */
  int32_t in_rows;      /* H > 0 */
  int32_t in_cols;      /* W > 0 */
  int32_t channels;     /* C > 0, input features  */
  int32_t features;     /* K > 0, output features */
  int32_t window_rows;  /* R > 0 */
  int32_t window_cols;  /* S > 0 */
  int32_t stride_rows;  /* > 0 */
  int32_t stride_cols;  /* > 0 */
  int32_t padding;      /* conv2d_padding_t */
  int32_t in_dtype;     /* conv2d_dtype_t of `in` AND `filt` */
  int32_t out_dtype;    /* conv2d_dtype_t of `out`; CONV2D_BF16 only with in_dtype == CONV2D_BF16 */
} conv2d_params;

typedef struct {
  int32_t out_rows, out_cols, pad_top, pad_bottom, pad_left, pad_right;
} conv2d_geometry;

/* Output size and padding for `params` (host only, touches no GPU): the
 * parameter tuple is the one of Figure 1's caption; the paper gives no padding
 * rule, the output size and padding follow the conventions at the top of this
 * file.  INVALID_ARGUMENT if the tuple has no valid output. */
CONV2D_API int conv2d_get_geometry(const conv2d_params* params, conv2d_geometry* geometry);

/* Bytes of device scratch that conv2d_forward may use for `params` (section 3:
 * the library chooses the algorithm, so it also says what that algorithm
 * needs) with the variant it selects for 16-byte-aligned pointers (0 for some
 * layers; non-zero when the filter is repacked or the reduction over window
 * and channels is split across workgroups).  The query sees no pointers; with
 * pointers that are only element-aligned conv2d_forward selects among the
 * element-wise variants, and if its pick there needs more than the workspace
 * it is given, it runs the cheapest variant that fits (the direct kernel
 * needs none), so a workspace of this size is always enough.  Host only. */
CONV2D_API int conv2d_workspace_size(const conv2d_params* params, size_t* bytes);

/* Same, for a forced variant (Figure 1's caption: not every algorithm supports
 * every parameter set).  UNSUPPORTED if the variant cannot run `params`. */
CONV2D_API int conv2d_workspace_size_variant(const conv2d_params* params, int variant_id, size_t* bytes);

/* Forward convolution with the variant the selector picks for the layer
 * shape (section 3: algorithm and parameter choice per shape).
 *   in, filt, out : device pointers, layouts above, element-aligned; the
 *                   vectorised variants are only selected when the bases are
 *                   16-byte aligned.
 *   workspace     : device scratch of at least conv2d_workspace_size() bytes,
 *                   16-byte aligned, or NULL when that size is 0.  Contents
 *                   are undefined afterwards.
 * Enqueues on hip_stream and returns.  batch == 0 returns OK without a launch. */
CONV2D_API int conv2d_forward(const conv2d_params* params, const void* in, const void* filt, void* out,
                   void* workspace, size_t workspace_bytes, void* hip_stream);

/* conv2d_forward for callers that cannot allocate or pass scratch memory: code
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  (It follows no passage of the paper; it exists for those callers.)
 * It runs the variant that conv2d_select_variant(params,
 * CONV2D_SELECT_DIRECT_SUM_ONLY) names for pointers of this alignment, with
 * that variant's scratch (repacked filter, partial sums of a split reduction)
 * in an array of CONV2D_STATIC_SCRATCH_BYTES that the library itself holds in
 * device memory, one copy on every GPU that loads the library, until the
 * process ends.  The result is bit-identical to conv2d_forward_variant with
 * that variant.  The call allocates and frees nothing and calls no allocating
 * routine; it looks the array's address up once per device, at its first call
 * on that device (make that call outside a stream capture).
 *   - A layer whose variant needs more than CONV2D_STATIC_SCRATCH_BYTES
 *     returns CONV2D_STATUS_SCRATCH_EXCEEDED and launches nothing (use
 *     conv2d_forward with a workspace).  Every layer of this library's
 *     workloads up to 3x3x512x512 filters fits.
 *   - All calls on one GPU share that GPU's array, which keeps the previous
 *     call's contents; no kernel relies on its initial contents.  Two calls
 *     that may overlap on one GPU (different streams, or different threads
 *     without ordering between their streams) race on it: order them.
 *   - in, filt, out, hip_stream and the return value: as conv2d_forward. */
#define CONV2D_STATIC_SCRATCH_BYTES (32u << 20)
CONV2D_API int conv2d_forward_static_scratch(const conv2d_params* params, const void* in,
                                             const void* filt, void* out, void* hip_stream);

/* Same, with the variant forced (0 <= variant_id < conv2d_num_variants()).
 * Section 3: the library's algorithms all give the same numeric result; here:
 * every variant that supports `params` produces the same result up to the
 * order of floating-point summation (the Winograd variants: up to the
 * rounding of their transforms, within the same tolerance).  UNSUPPORTED if it cannot run them. */
CONV2D_API int conv2d_forward_variant(const conv2d_params* params, const void* in, const void* filt,
                           void* out, void* workspace, size_t workspace_bytes, void* hip_stream,
                           int variant_id);

/* Forward convolution with a fused epilogue:
 *   out[n,p,q,k] = act( conv(in, filt)[n,p,q,k] + bias[k] )
 * Section 3 of the paper names the layers that sit between the convolutions
 * of a network only in passing; folding the bias and the activation into the
 * store of the convolution saves one round trip of the output through memory
 * (on the 1x1 layers the output is most of the traffic).
 *   bias       : device pointer to `features` fp32 values, or NULL for none
 *   activation : CONV2D_ACT_NONE or CONV2D_ACT_RELU (max(x, 0); NaN stays NaN)
 * The sum is formed in fp32 exactly as by conv2d_forward, the bias is added
 * in fp32 and the result is rounded once to out_dtype.  Same variant
 * selection, workspace and other rules as conv2d_forward; INVALID_ARGUMENT
 * for an unknown activation or a misaligned bias pointer. */
typedef enum { CONV2D_ACT_NONE = 0, CONV2D_ACT_RELU = 1 } conv2d_activation_t;
CONV2D_API int conv2d_forward_bias_act(const conv2d_params* params, const void* in, const void* filt,
                            const float* bias, int activation, void* out, void* workspace,
                            size_t workspace_bytes, void* hip_stream);

/* Convolution + bias + activation + 2x2 max pooling (stride 2, no padding) in
 * one call:
 *   out[n,i,j,k] = max over a, b in {0,1} of
 *                  act( conv(in, filt)[n, 2i+a, 2j+b, k] + bias[k] )
 *   out : [batch][out_rows/2][out_cols/2][features], NHWC, dense, out_dtype;
 *         a trailing odd row or column of the convolution's output is dropped
 *         (nothing is written if out_rows or out_cols is below 2).
 * Section 3 of the paper names pooling among the layers that sit between the
 * convolutions; the 3x3 layers of a VGG-style network that precede a pooling
 * layer are exactly the ones whose output traffic this removes (a quarter of
 * the unpooled tensor is written and nothing of it is read back).
 * Variants whose tiles are even-sized blocks of output pixels of one image
 * (the blocked patch tiles: 3x3 window, stride 1) take the maximum of the
 * four sums in registers and write only the pooled tensor; so do the Winograd
 * variants, whose tiles of 2x2 outputs are exactly the pooling windows.  Every other
 * variant writes the unpooled tensor into the workspace, behind its own
 * scratch, and a second kernel pools it; the result is the same.
 * The maximum is taken with fmaxf: a NaN among the four is dropped unless all
 * four are NaN.  conv2d_pool_workspace_size (host only) gives the bytes this
 * entry point needs for the variant it would select for 16-byte-aligned
 * pointers, the _variant form for a given variant (UNSUPPORTED if that variant
 * cannot run the parameters).  With pointers that are only element-aligned no
 * variant pools in its epilogue, so the workspace must also hold the unpooled
 * tensor: conv2d_pool_workspace_size_variant(params, 0, ...) (the direct
 * kernel's size) is then enough, less is WORKSPACE_TOO_SMALL.  All other
 * rules are those of conv2d_forward_bias_act. */
CONV2D_API int conv2d_pool_workspace_size(const conv2d_params* params, size_t* bytes);
CONV2D_API int conv2d_pool_workspace_size_variant(const conv2d_params* params, int variant_id,
                                       size_t* bytes);
CONV2D_API int conv2d_forward_bias_act_pool(const conv2d_params* params, const void* in,
                                 const void* filt, const float* bias, int activation, void* out,
                                 void* workspace, size_t workspace_bytes, void* hip_stream);

/* Filters packed ahead of time.  (These three calls follow no passage of the
 * paper: they serve inference loops whose filters do not change.  The tiles
 * whose names end in "_nat" and the conv1x1_* variants read the filter as it
 * lies in memory and need none of this: their packed filter is a plain copy.)
 * The other matrix-core kernels read the filter in a
 * layout of their own (reduction index contiguous, cut into the tile's
 * slices), which conv2d_forward writes into the workspace on every call: a
 * small kernel of its own, ~5 us, a tenth to a third of a whole call on the
 * small layers of a network at batch 1-4.  A caller whose filters do not
 * change (inference) packs them once:
 *   conv2d_packed_filter_size  bytes of the packed filter of `variant_id` for
 *                              these parameters (host only)
 *   conv2d_pack_filter         writes it (device to device, on the stream)
 *   conv2d_forward_packed      conv2d_forward_bias_act with that variant on
 *                              the packed filter; same workspace as
 *                              conv2d_workspace_size_variant gives
 * The packed filter belongs to the variant and the parameters it was packed
 * for (take the id from conv2d_select_variant or conv2d_selected_variant);
 * using it with others gives wrong results, not an error.  For the Winograd
 * variants it holds the transformed filter (16 points, 16/9 of the filter's
 * size, twice: transformed and repacked); for the zero-padded-channel
 * variants (padc_*) the padded and repacked filter (their input is still
 * padded in every call); for the direct, the register-staged and the
 * window-row gather (rowgather_*) variants it is a plain copy.
 * Results are bit-identical to conv2d_forward_variant / _bias_act with the
 * same variant.  Pointer alignment rules as for conv2d_forward. */
CONV2D_API int conv2d_packed_filter_size(const conv2d_params* params, int variant_id,
                                         size_t* bytes);
CONV2D_API int conv2d_pack_filter(const conv2d_params* params, int variant_id, const void* filt,
                                  void* packed, size_t packed_bytes, void* hip_stream);
CONV2D_API int conv2d_forward_packed(const conv2d_params* params, int variant_id, const void* in,
                                     const void* packed_filt, const float* bias, int activation,
                                     void* out, void* workspace, size_t workspace_bytes,
                                     void* hip_stream);

/* The runtime's description of the error behind the calling thread's last
 * CONV2D_STATUS_LAUNCH_FAILED ("" if there was none).  The string is the
 * runtime's and stays valid.  (Follows no passage of the paper.) */
CONV2D_API const char* conv2d_last_launch_error(void);

/* Variant introspection (host only): the "algorithms and their parameters" of
 * section 3 by number and name, and Figure 1's compatibility rule as a
 * predicate. */
CONV2D_API int conv2d_num_variants(void);
CONV2D_API const char* conv2d_variant_name(int variant_id);            /* NULL if out of range */
CONV2D_API int conv2d_variant_supports(const conv2d_params* params, int variant_id); /* 1, 0, or <0 status */
/* Debugging aid for the entry points that select a variant themselves and have
 * no forced-variant form (conv2d_forward_bias_act, conv2d_forward_bias_act_pool,
 * conv2d_forward_static_scratch, and conv2d_forward): from now on the calling
 * thread's calls run `variant_id` wherever it supports the parameters and the
 * pointers' alignment, and their own pick elsewhere; -1 switches it off.  The
 * size queries of the same thread follow.  A thread starts with the value of
 * the CONV2D_FORCE_VARIANT environment variable (read once per process), -1
 * without it.  It is how the tests check section 3's statement that every
 * algorithm gives the same result through these entry points too.
 * INVALID_ARGUMENT for an id outside [-1, conv2d_num_variants()). */
CONV2D_API int conv2d_debug_force_variant(int variant_id);
/* Debugging aid for the "_splitk" variants of the direct-to-LDS gather tiles (the reduction of
 * an output tile split over several workgroups, for layers with few output pixels).  They add a
 * tile's partial sums inside the convolution launch, by the last of the tile's workgroups to
 * finish, wherever they can: an output of at most 4096 tiles with a feature count that is a
 * multiple of 4, a stream that is not being captured into a graph, one of the 32 streams per
 * process that such launches have been seen on.  Everything else takes a second launch that adds
 * the partial sums.  on = 1 makes every launch of the process take the second launch, 0 (the
 * start value) returns to the rule above; both give the sum of the partial sums in split order.
 * It is how the tests run both paths.  INVALID_ARGUMENT for other values.  (Follows no passage
 * of the paper.) */
CONV2D_API int conv2d_debug_split_reduce_separate(int on);
/* The variant conv2d_forward would use, assuming 16-byte-aligned pointers. */
CONV2D_API int conv2d_selected_variant(const conv2d_params* params, int* variant_id);

/* Selection with a restriction.  The paper's library holds, next to the
 * algorithms that sum the window directly, a Winograd algorithm that reaches
 * the same result through data transforms with fewer multiplications
 * (section 3); here those are the "winograd2x2_*" variants (fp32, 3x3 window,
 * stride 1; they need a workspace several times the size of the input).
 * flags = 0 selects among all variants, exactly as conv2d_selected_variant;
 * CONV2D_SELECT_DIRECT_SUM_ONLY leaves the transform variants out, for a
 * caller that wants a small workspace or counts the executed multiplications.
 * INVALID_ARGUMENT for unknown flag bits.  Host only. */
#define CONV2D_SELECT_DIRECT_SUM_ONLY 1u
CONV2D_API int conv2d_select_variant(const conv2d_params* params, uint32_t flags, int* variant_id);

/* Text of a status code; the library's version (100 * major + minor).  (Follow
 * no passage of the paper.) */
CONV2D_API const char* conv2d_status_string(int status);
CONV2D_API int conv2d_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CONV2D_MI355X_H_ */
