/*
 * sparse_conv.h -- C ABI of the MI355X (gfx950) masked-convolution library.
 *
 * The operation (paper Sec. 3, Fig. 1-2; Sec. 3.2; App. A, Alg. 2): a convolution is the
 * product of a lowered activation matrix A[M x K] (one row per output position
 * r = (n*Ho + oy)*Wo + ox, K = kh*kw*Cin window entries) with the filter matrix
 * B[K x Cout].  A fixed binary mask over output positions removes whole rows of A; the
 * contraction runs over the surviving rows only and the results are placed back into the
 * dense output layout, with zeros at the removed positions.
 *
 * Conventions
 *   - mask byte != 0 keeps the row, 0 drops it (Alg. 1 getMask; Alg. 2 both functions);
 *   - a dropped position holds +0.0 (all bits zero) in every output channel: no bias, no
 *     activation (Alg. 2, post-process);  bias and ReLU act on kept rows only;
 *   - zero padding, cross-correlation, Ho = floor((H + 2*pad - dil*(kh-1) - 1)/stride) + 1;
 *   - SC_NHWC: x[N,H,W,Cin], w[Cout,kh,kw,Cin], y[N,Ho,Wo,Cout]   (fast path)
 *     SC_NCHW: x[N,Cin,H,W], w[Cout,Cin,kh,kw], y[N,Cout,Ho,Wo]   (element-wise gather path)
 *   - x, w and y share one element type; bias is always float; accumulation is float.
 *
 * Memory and ownership
 *   Every pointer named *_dev is DEVICE memory allocated and owned by the caller; the
 *   library never allocates, frees or keeps device memory of its own.  Derived data (row
 *   index list, packed filters, gather table) lives in the caller's workspace, which must
 *   stay alive and untouched for as long as the plan is used.  The plan object itself is
 *   host memory owned by the library until sparse_conv_plan_destroy.
 *   `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).
 *
 * Errors
 *   Every entry point returns a status code and never throws or aborts.  All argument
 *   checks happen on the host before the first HIP call.  sparse_conv_plan synchronises the
 *   stream once (it needs the kept-row count on the host); the *_run calls only enqueue
 *   work: no allocation, no host synchronisation.
 */
#ifndef SPARSE_CONV_H_
#define SPARSE_CONV_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SC_OK = 0,
  SC_ERR_NULL = 1,        /* a required pointer is NULL */
  SC_ERR_BAD_SHAPE = 2,   /* non-positive extent, empty output, or a tensor too large for 32-bit element offsets */
  SC_ERR_UNSUPPORTED = 3, /* groups other than 1 or depthwise, unknown dtype/layout/mode/format */
  SC_ERR_MASK_COUNT = 4,  /* popcount(mask) differs from the count the sparsity ratio demands */
  SC_ERR_WORKSPACE = 5,   /* workspace smaller than sparse_conv_workspace_bytes() */
  SC_ERR_ALIGN = 6,       /* a device pointer is not aligned to 16 bytes */
  SC_ERR_HIP = 7          /* a HIP call failed; sc_last_hip_error() holds its code */
} sc_status;

typedef enum { SC_F32 = 0, SC_F16 = 1, SC_BF16 = 2 } sc_dtype;
typedef enum { SC_NHWC = 0, SC_NCHW = 1 } sc_layout;

/* Scope of the mask over the batch.  The paper trains one 2-D mask per layer that every
 * image shares (Sec. 3.1; Alg. 2 indexes the mask by output y/x only) = SC_MASK_SPATIAL.
 * SC_MASK_ROW carries one byte per row of the lowered matrix of the whole batch. */
typedef enum { SC_MASK_ROW = 0, SC_MASK_SPATIAL = 1 } sc_mask_mode;

/* SC_OUT_ZERO_FILL: the run writes every element of y (zeros at dropped positions), as
 * Alg. 2's post-processing does.  SC_OUT_SCATTER_ONLY: the run writes kept rows only; the
 * caller guarantees the dropped positions of y already hold zeros (the mask is frozen after
 * training, Sec. 3.1, so a buffer zeroed once keeps them). */
typedef enum { SC_OUT_ZERO_FILL = 0, SC_OUT_SCATTER_ONLY = 1 } sc_out_mode;

typedef struct {
  int32_t n, c_in, h, w, c_out;
  int32_t kh, kw, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
  int32_t groups;      /* 1; or c_in == c_out == groups with SC_NHWC: depthwise, every channel filtered by its
                          own kh x kw window (filters [C][kh][kw][1]); the mask removes output pixels as for
                          ordinary layers (Sec. 3), compact formats work alike */
  int32_t dtype;       /* sc_dtype of x, w, y */
  int32_t layout;      /* sc_layout of x, w, y */
  int32_t has_bias;    /* 0/1 */
  int32_t relu;        /* 0/1, applied after bias on kept rows */
  int32_t mask_mode;   /* sc_mask_mode */
  int32_t out_mode;    /* sc_out_mode */
  float sparsity;      /* s in [0,1): plan fails with SC_ERR_MASK_COUNT unless
                          popcount(mask) == floor((1-s)*len + 0.5) (Sec. 3.2: the GEMM range is
                          output_size - sparsity*output_size);  s < 0 disables the check.
                          Where (1-s)*len falls on a half within the rounding interval of this float
                          (0.9 of 135 positions), both neighbouring counts pass.
                          The mask, never this number, decides which rows run. */
} sc_conv_desc;

typedef struct sc_plan sc_plan; /* opaque, host memory */

/* Output extents and row count M = N*Ho*Wo of a descriptor (host only). */
sc_status sparse_conv_output_shape(const sc_conv_desc* desc, int32_t* ho, int32_t* wo, int64_t* m);

/* Bytes of device workspace sparse_conv_plan needs for this descriptor (host only). */
sc_status sparse_conv_workspace_bytes(const sc_conv_desc* desc, size_t* bytes);

/*
 * Build a plan (Alg. 2, indirection init, done once per layer because the mask is frozen):
 *   - compacts the mask into the ascending list of kept rows (device, wavefront ballot scan);
 *   - packs the filters into the K-major layout the GEMM reads;
 *   - builds the per-K gather table; chooses tile shapes for the reduced and the full M.
 * mask_dev: uint8[N*Ho*Wo] (SC_MASK_ROW) or uint8[Ho*Wo] (SC_MASK_SPATIAL), device.
 * w_dev:    filters in the descriptor's layout and dtype, device; read during this call only.
 * workspace_dev: at least sparse_conv_workspace_bytes() bytes, 256-byte aligned, device.
 * Synchronises `hip_stream` before returning.  On failure *out is NULL.
 */
sc_status sparse_conv_plan(const sc_conv_desc* desc, const uint8_t* mask_dev, const void* w_dev,
                           void* workspace_dev, size_t workspace_bytes, void* hip_stream, sc_plan** out);

/*
 * Training-side refresh of a plan (Alg. 1: getMask draws a new mask whenever updateMask says so, and the
 * weights change with every optimiser step).  Same layer, same workspace, no new plan:
 *   sparse_conv_plan_set_mask     the indirection init of Alg. 2 again for a new mask (compaction, band
 *                                 tables); the kept-row count is checked against the descriptor's sparsity as
 *                                 in sparse_conv_plan.  Synchronises `hip_stream`.  After an error the plan must
 *                                 not be run until a later call has succeeded (its tables describe the rejected mask).
 *   sparse_conv_plan_set_filters  repacks the filters (same layout and dtype as at plan time); enqueues only.
 * Runs that are still in flight on another stream must have finished before either call.
 */
sc_status sparse_conv_plan_set_mask(sc_plan* plan, const uint8_t* mask_dev, void* hip_stream);
sc_status sparse_conv_plan_set_filters(sc_plan* plan, const void* w_dev, void* hip_stream);

/*
 * Masked convolution (Sec. 3.2 stages i-iii fused into one launch): gather the kept rows'
 * receptive fields, contract with the filters on the matrix cores, add bias / apply ReLU,
 * and store each result at its dense position; dropped positions receive zeros (or are
 * left alone in SC_OUT_SCATTER_ONLY mode).
 * x_dev: activations; bias_dev: float[Cout] or NULL when has_bias == 0; y_dev: output, fully
 * overwritten in SC_OUT_ZERO_FILL mode.  x_dev and y_dev must not overlap.
 * Enqueues on `hip_stream` only: no allocation, no synchronisation.  Runs of ONE plan may overlap in time (on
 * different streams) only when the launch keeps no state in the plan's workspace.  Two kinds of launch do:
 * launches that divide K among workgroups -- chosen automatically on deep layers, and by SC_OPT_SPLIT_K /
 * SC_OPT_STREAM_K; sparse_conv_plan_kernel reports "tile_split_k", "tile_stream_k", or "tile_slab" with more
 * workgroups than output tiles -- keep partial sums and arrival counters there; and plans of 16-bit NHWC layers
 * with few input channels whose launch is "tile_row_segments" (forced tiles, compact operands or fused shortcuts on,
 * e.g., a 3-channel stem; "band_row_segments" keeps no such state) rewrite a zero-margined copy of x there in
 * every run.  Overlapping runs of such a plan race and give wrong results without an error: use one plan per stream.
 */
sc_status sparse_conv_run(const sc_plan* plan, const void* x_dev, const float* bias_dev, void* y_dev,
                          void* hip_stream);

/*
 * The masked convolution with compact operands (NHWC layers): between two layers that share one mask
 * -- propagated masks are the same for every layer of one resolution, Sec. 3.1 -- the zeros of stage
 * (iii) of Sec. 3.2 and the gather of stage (i) cancel, so a pointwise consumer can take the GEMM
 * result of its producer as it is.
 *   y_rows = SC_ROWS_COMPACT: y_dev is [kept][Cout]; row i is the result of lowered row row_idx[i]
 *            (ascending, see sparse_conv_plan_info).  Nothing else is written: no zeros, no scatter.
 *   x_rows = SC_ROWS_COMPACT: x_dev is [kept][Cin]; row i is input pixel row_idx[i] of THIS layer's
 *            mask.  For 1x1 windows with stride 1 and no padding (the window is the pixel itself,
 *            so a kept row never reads a dropped pixel).  A depthwise layer with larger windows takes a
 *            compact input after sparse_conv_plan_set_input_mask (below): x_dev then holds the pixels that
 *            the INPUT's mask keeps, and the dropped ones read as the +0.0 Alg. 2 would have written.
 *            SC_ERR_UNSUPPORTED otherwise, also for NCHW plans and for formats other than the two below.
 *   SC_ROWS_DENSE for both is sparse_conv_run.  The out_mode of the plan applies to dense outputs only.
 * Pointer and alignment rules as for sparse_conv_run; no allocation, no synchronisation.
 */
typedef enum { SC_ROWS_DENSE = 0, SC_ROWS_COMPACT = 1 } sc_rows_format;
sc_status sparse_conv_run_rows(const sc_plan* plan, const void* x_dev, int32_t x_rows, const float* bias_dev,
                               void* y_dev, int32_t y_rows, void* hip_stream);

/*
 * The masked convolution fused with the shortcut sum that follows it in a residual block:
 *
 *     y = post( act(conv(x) + bias) + residual )        post = ReLU if residual_relu != 0, else identity
 *
 * `act` is the plan's own activation.  Alg. 2 makes a dropped row of the convolution +0.0, so a dropped row of a
 * dense-layout y receives post(residual) (in SC_OUT_SCATTER_ONLY mode it is left alone, as always).  residual_dev
 * has the dtype and the row format of y (dense map, or [kept][Cout] with y_rows = SC_ROWS_COMPACT), is 16-byte
 * aligned and must not overlap y.  The sum is formed in float before the one rounding to the layer dtype.
 * Runs in the tiled kernels, the alternating-group or the tap-pipelined band kernel (never the other band kernels, the row-panel or
 * the depthwise kernels, whatever the plan would pick for the plain run): SC_ERR_UNSUPPORTED for depthwise plans;
 * x_rows / y_rows as in sparse_conv_run_rows.
 * dense_conv_run_residual: the same with the identity row map (every row kept).
 */
sc_status sparse_conv_run_residual(const sc_plan* plan, const void* x_dev, int32_t x_rows, const float* bias_dev,
                                   const void* residual_dev, int32_t residual_relu, void* y_dev, int32_t y_rows,
                                   void* hip_stream);
sc_status dense_conv_run_residual(const sc_plan* plan, const void* x_dev, const float* bias_dev,
                                  const void* residual_dev, int32_t residual_relu, void* y_dev, void* hip_stream);

/*
 * Row list of a compact input for a depthwise layer with windows larger than one pixel (its producer's
 * mask, which under Alg. 1's propagation differs from the layer's own when the layer is strided):
 * mask_in_dev is uint8[N*H*W] (SC_MASK_ROW plans) or uint8[H*W] (SC_MASK_SPATIAL plans) over the INPUT
 * pixels, 1 = present in x.  Builds, inside the workspace, the map from input pixel to row of x that the
 * kernels consult for every tap; *kept_in (may be NULL) receives the number of rows x must hold.
 * Synchronises `hip_stream`.  SC_ERR_UNSUPPORTED for other plans; may be called again for a new mask.
 */
sc_status sparse_conv_plan_set_input_mask(sc_plan* plan, const uint8_t* mask_in_dev, int64_t* kept_in,
                                          void* hip_stream);

/* The same kernels with the identity row map: the ordinary dense convolution (the paper's
 * baseline; its GEMM is unchanged, App. A).  Ignores the mask. */
sc_status dense_conv_run(const sc_plan* plan, const void* x_dev, const float* bias_dev, void* y_dev,
                         void* hip_stream);

/* Plan facts.  Any output pointer may be NULL.  *row_idx_dev points into the workspace:
 * int32[kept], ascending. */
sc_status sparse_conv_plan_info(const sc_plan* plan, int64_t* m, int64_t* kept, int32_t* ho, int32_t* wo,
                                const int32_t** row_idx_dev);

/* The plan's private copy of the mask (device memory inside the workspace; uint8[N*Ho*Wo] or [Ho*Wo] as
 * the descriptor's mask_mode says).  NULL for a NULL plan. */
const uint8_t* sparse_conv_plan_mask(const sc_plan* plan);

/* Tile shape chosen for the sparse (which = 0) or dense (which = 1) launch: rows x couts per
 * workgroup, and the number of workgroups.  The library has two kernels: the tiled gather kernel
 * (tile_m > 0 kept rows per workgroup) and the band kernel, which stages a band of input rows of
 * one image in LDS (reported as tile_m = -BH, BH = output rows per band). */
sc_status sparse_conv_plan_tiles(const sc_plan* plan, int32_t which, int32_t* tile_m, int32_t* tile_n,
                                 int64_t* workgroups);

/* Name of the kernel the sparse (which = 0) or dense (which = 1) launch uses: "band",
 * "band_alternating", "band_tap", "band_stream", "band_row_segments", "tile_row_panel", "tile_slab", "tile_split_k", "tile_masked_store", "tile_stream_k", "tile_lds_direct",
 * "tile_registers", "tile_row_segments", "tile_elements" or "depthwise".
 * A static string; NULL for a NULL plan or an unknown `which`. */
const char* sparse_conv_plan_kernel(const sc_plan* plan, int32_t which);
/* The same for a launch fused with a shortcut sum (sparse_conv_run_residual / dense_conv_run_residual with dense
 * operands): "band_alternating" or one of the "tile_..." names; NULL also for depthwise plans (no fused form). */
const char* sparse_conv_plan_fused_kernel(const sc_plan* plan, int32_t which);

/* Tuning hook: force the kernel of later runs.  (0,0) restores the automatic choice; tile_m > 0
 * selects the tiled gather kernel of that shape; tile_m < 0 selects the band kernel (band height
 * stays automatic).  Returns SC_ERR_UNSUPPORTED when the library has no such kernel for the layer. */
sc_status sparse_conv_plan_set_tiles(sc_plan* plan, int32_t which, int32_t tile_m, int32_t tile_n);

/*
 * Measured kernel choice.  sparse_conv_plan prices its candidate launches (tile shape, K splits, band or tiled
 * kernel, and for small layers the variant that contracts every row and lets the mask decide at the store) with a
 * model of the device; this call times the serious candidates of the sparse and of the dense run on the caller's
 * real buffers and keeps the fastest of each.  x_dev, bias_dev, y_dev as for sparse_conv_run; y_dev is overwritten
 * many times and holds the masked convolution of x when the call returns.  Candidates are timed as captured graphs
 * of back-to-back launches on a stream the call creates and destroys (with two events; default priority), so that
 * layers of a few microseconds are not measured at the host's launch rate; `hip_stream` is synchronised first and
 * last; no device memory is allocated.  Choices forced with
 * sparse_conv_plan_set_tiles stay as they are; sparse_conv_plan_set_mask returns the sparse run to the model's choice.
 */
sc_status sparse_conv_plan_tune(sc_plan* plan, const void* x_dev, const float* bias_dev, void* y_dev, void* hip_stream);

/* Environment (read by sparse_conv_plan; tuning and tests only):
 *   SPARSE_CONV_BAND_HEIGHT=<rows>               fixes the band height of the streaming and of the
 *                                                alternating-group band kernels (automatic otherwise)
 *   SPARSE_CONV_BAND_KERNEL=single|alternating|tap|no-tap
 *                                                band kernel with one band per workgroup; the persistent one
 *                                                whose two wavefront groups alternate between transfer and
 *                                                matrix work; the one whose filters arrive window row by
 *                                                window row under the matrix work (both: 3x3 windows, 16-bit
 *                                                types, 32 or 64 input channels); the automatic choice
 *                                                without the last; automatic otherwise */

/* Tuning hook: SC_OPT_GATHER_PIPELINE selects how the tiled gather kernel moves its K tiles:
 * 0 = automatic, 1 = global -> registers -> LDS, 2 = global -> LDS directly (NHWC with 16-byte
 * channel groups only; other layers ignore it).  Unknown options return SC_ERR_UNSUPPORTED. */
/* SC_OPT_SPLIT_K: 0 = automatic, 1 = never split K, n >= 2 = divide K among n workgroups per output
 * tile wherever the split-K kernel applies (16-bit NHWC layers with >= 128 output channels and a
 * deep K); n is at most 64 and is clamped so that the partial sums fit their 16 MiB buffer and every
 * split has at least four K tiles.  Partial sums are added in a fixed order: results do not depend on scheduling. */
/* SC_OPT_ROW_PANEL: 0 = automatic, 1 = never, 2 = always where it applies.  The row-panel kernel
 * (16-bit NHWC layers with K <= 2 K tiles, i.e. pointwise layers with up to 128 input channels, and
 * at most 1024 output channels) gathers 128 kept rows once and walks all channel tiles with them. */
/* SC_OPT_STREAM_K: 0 = automatic, 1 = never, n >= 2 = run the tiled kernel as n persistent workgroups
 * (rounded up to a multiple of 8, at most 1024) that share the K steps of all output tiles evenly, wherever
 * that kernel applies (the layers SC_OPT_SPLIT_K names whose input channels are a multiple of 64); tiles
 * whose K walk is shared are completed from float partial sums added in a fixed order.  n is clamped so that
 * two partial-sum slots per workgroup fit the 16 MiB buffer and every workgroup has at least four K steps.
 * Measured slower than the ordinary launch on every benchmark layer (the partial sums cross the fabric
 * between the XCDs' caches), so automatic means off. */
/* SC_OPT_MASKED_STORE: 0 = automatic, 1 = never, 2 = always where it applies.  A sparse run of dense NHWC operands
 * (no shortcut tensor, not the row-segment gather) may contract EVERY row with the identity row map and let the mask
 * decide at the store -- zeros for a dropped row, or nothing in scatter-only mode: the results are those of Alg. 2,
 * the work is the dense layer's.  Taken where the kept-row list costs more (a dependent round trip to memory before
 * the first transfer) than the rows it removes: layers of a few microseconds. */
/* SC_OPT_SLAB: 0 = automatic, 1 = never, 2 = always where it applies, 128 / 256 = always, with tiles of that many kept
 * rows.  The slab form of the tiled kernel serves 3x3 layers with stride 1, no dilation, 16-bit NHWC tensors, input
 * channels a multiple of 32 and output channels a multiple of 16 (at least 96): per chunk of 32 input channels a
 * workgroup keeps the input pixels under the windows of its kept rows (Sec. 3.2: only those rows are lowered) in LDS and
 * reads them once per window tap, instead of fetching the nine-fold lowered rows.  A K split (SC_OPT_SPLIT_K) divides
 * the chunks; the split-K note on overlapping runs applies. */
enum { SC_OPT_GATHER_PIPELINE = 0, SC_OPT_SPLIT_K = 1, SC_OPT_ROW_PANEL = 2, SC_OPT_STREAM_K = 3, SC_OPT_MASKED_STORE = 4,
       SC_OPT_SLAB = 5 };
sc_status sparse_conv_plan_set_option(sc_plan* plan, int32_t option, int32_t value);

void sparse_conv_plan_destroy(sc_plan* plan);

const char* sc_status_string(sc_status s);
int32_t sc_last_hip_error(void); /* hipError_t of the last failed HIP call on this thread */

/*
 * Backward pass of the masked convolution (Alg. 1: backward(model) follows maskedForward(model, mask)).
 * With g[r, co] = dy[r, co] where mask[r] == 1 and (no ReLU or y[r, co] > 0), and 0 elsewhere:
 *     db[co] = sum_r g[r, co]      dw[co, k] = sum_r g[r, co] * A[r, k]      dx = transposed convolution of g
 * (A = lowered activations, Sec. 3).  The contraction for dw runs over the kept rows only, like the
 * forward GEMM (Sec. 3.2).  NHWC layers with one group, bf16, fp16 or float (the paper's own arithmetic:
 * a plainer kernel on the 32 x 32 x 2 float MFMA), Cin and Cout multiples of 8; SC_ERR_UNSUPPORTED otherwise.
 *   sparse_conv_backward_plan   `fwd` is the layer's forward plan (it supplies the mask and the row list and must
 *                         outlive the backward plan; after sparse_conv_plan_set_mask the backward plan follows);
 *                         `desc` the descriptor the forward plan was made from; w_dev the filters.  workspace_dev:
 *                         at least sparse_conv_backward_workspace_bytes() bytes, 256-byte aligned, device, owned
 *                         by the caller, used by every run (g map, partial sums, rotated filters).  Synchronises.
 *   sparse_conv_backward_run    x_dev: the forward input; y_dev: the forward output (its sign gates the ReLU; may be
 *                         NULL for layers without ReLU); dy_dev: upstream gradient, layout and dtype of y.
 *                         dx_dev (layout and dtype of x), dw_dev (float [Cout][kh][kw][Cin]) and db_dev
 *                         (float [Cout]) are each optional (NULL = not wanted).  dx is the ordinary convolution of g (with
 *                         zeros interleaved for strided layers) with the rotated filters and runs through the
 *                         forward kernels; SC_ERR_UNSUPPORTED only when the layer's padding exceeds
 *                         dil * (k - 1).  Additions happen in a fixed order: results do not depend on
 *                         scheduling, and dw and db are the same bits whether or not dx is asked for (without dx no g
 *                         map is written: the filter-gradient kernel gates dy by y itself).  Enqueues only; no
 *                         allocation, no synchronisation.
 *   sparse_conv_backward_set_filters   new filter values (after an optimiser step) for the input gradient.
 */
typedef struct sc_bwd_plan sc_bwd_plan;
sc_status sparse_conv_backward_workspace_bytes(const sc_conv_desc* desc, size_t* bytes);
sc_status sparse_conv_backward_plan(const sc_plan* fwd, const sc_conv_desc* desc, const void* w_dev, void* workspace_dev,
                                    size_t workspace_bytes, void* hip_stream, sc_bwd_plan** out);
sc_status sparse_conv_backward_set_filters(sc_bwd_plan* plan, const void* w_dev, void* hip_stream);
sc_status sparse_conv_backward_run(const sc_bwd_plan* plan, const void* x_dev, const void* y_dev, const void* dy_dev,
                                   void* dx_dev, float* dw_dev, float* db_dev, void* hip_stream);
void sparse_conv_backward_destroy(sc_bwd_plan* plan);

/*
 * Mask generator of the training pipeline (Alg. 1, function getMask; Sec. 3.1): the mask of one layer
 * from a 2-D random score at the resolution of the network input.  Call it once per layer resolution
 * with the same score: the masks of all layers then show the same pattern (the propagation of Sec. 3.1).
 *   score_dev   float[in_h * in_w], row-major, device.  The random numbers are the caller's.
 *               Not-a-number scores are not supported.
 *   ho, wo      resolution of the layer's output map, 1 <= ho <= in_h, 1 <= wo <= in_w.  The score is
 *               average-pooled with window = stride = (in_h / ho, in_w / wo) (integer division); when
 *               the pooled map is larger than ho x wo its top-left corner is used.
 *   sparsity    in [0, 1]: ho*wo - floor((1 - sparsity) * ho*wo + 0.5) pixels are dropped, those with
 *               the lowest pooled score; equal scores are dropped in ascending pixel index.  Pixels are
 *               compared by the double-precision sum of their window, added in row-major order.
 *   mask_dev    uint8[ho * wo], device: 1 = keep, 0 = drop (the SC_MASK_SPATIAL mask of sparse_conv_plan).
 *   workspace_dev  at least sparse_mask_workspace_bytes(ho, wo) bytes, 8-byte aligned, device; scratch,
 *               owned by the caller, free for reuse once the stream has passed the call.
 *               (one 64-bit key per layer pixel and about 130 KiB of selection state.)
 * Enqueues two kernels on `hip_stream` (four for maps of more than 16 384 pixels, whose ranking is spread over many
 * workgroups) and returns; no allocation, no synchronisation.
 * Errors: SC_ERR_NULL, SC_ERR_BAD_SHAPE (extents, sparsity outside [0, 1], more than 2^26 pixels),
 * SC_ERR_WORKSPACE, SC_ERR_ALIGN, SC_ERR_HIP.
 */
sc_status sparse_mask_workspace_bytes(int32_t ho, int32_t wo, size_t* bytes);
sc_status sparse_mask_generate(const float* score_dev, int32_t in_h, int32_t in_w, int32_t ho, int32_t wo,
                               float sparsity, uint8_t* mask_dev, void* workspace_dev, size_t workspace_bytes,
                               void* hip_stream);

/*
 * sparse_mask_generate for callers that cannot allocate device memory and so have no workspace to hand over: code
 * under HIP graph capture, tight serving or training loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and bit-identical masks; the scratch (one 64-bit key per layer pixel, then the selection state) is a fixed
 * array inside the library's code object instead of the caller's workspace.
 *   - at most SC_STATIC_MASK_PIXELS layer pixels (ho * wo); a larger map returns SC_ERR_WORKSPACE and launches nothing;
 *   - the array (2 MiB + 128 KiB) exists once per GPU the library runs on and is held until the process ends; the first call
 *     on a device asks the runtime for its address (no allocation), so make that call outside a graph capture;
 *   - calls no hipMalloc / hipFree or other allocating routine and never synchronises;
 *   - every call on one GPU uses that GPU's one array: calls whose work overlaps on a GPU (two streams, two threads)
 *     race on it and give wrong masks -- order them on one stream or with events.  Nothing needs clearing between
 *     calls: the first kernel overwrites every key the later ones read and clears the counters they add to.
 * Errors otherwise as for sparse_mask_generate (SC_ERR_NULL, SC_ERR_BAD_SHAPE, SC_ERR_HIP).
 */
#define SC_STATIC_MASK_PIXELS (1 << 18)
sc_status sparse_mask_generate_static(const float* score_dev, int32_t in_h, int32_t in_w, int32_t ho, int32_t wo,
                                      float sparsity, uint8_t* mask_dev, void* hip_stream);

/*
 * Glue operators of the test networks (ResNet- and MobileNet-style stacks), NHWC device tensors of `dtype`.
 * They are not part of the paper's method; they only connect conv layers in network runs.
 *   sc_maxpool2d_nhwc: window k, stride s, zero-free padding p (padded taps never win).
 *   sc_add_relu:       y = max(a + b, 0), element-wise over `count` elements; y may alias a or b.
 *   sc_add:            y = a + b, likewise (the linear shortcut of inverted-residual blocks).  Both work on
 *                      compact [kept x C] matrices as well: an element-wise operator keeps the row format.
 * Errors: SC_ERR_NULL, SC_ERR_UNSUPPORTED (dtype), SC_ERR_BAD_SHAPE (negative count), SC_ERR_HIP.
 */
sc_status sc_maxpool2d_nhwc(const void* x_dev, void* y_dev, int32_t dtype, int32_t n, int32_t h, int32_t w,
                            int32_t c, int32_t k, int32_t s, int32_t p, void* hip_stream);
sc_status sc_add_relu(const void* a_dev, const void* b_dev, void* y_dev, int32_t dtype, int64_t count,
                      void* hip_stream);
sc_status sc_add(const void* a_dev, const void* b_dev, void* y_dev, int32_t dtype, int64_t count, void* hip_stream);

/*
 * Measurement probes (not part of the method): what the device sustains on the two roofs the kernels are priced against.
 *   sc_probe_stream_copy  enqueues a plain copy of `bytes` (a multiple of 16; both pointers 16-byte aligned, device, not
 *                         overlapping): read + write bandwidth of the memory system is 2 * bytes / time.
 *   sc_probe_mfma_bf16    enqueues `workgroups` workgroups of four wavefronts that each issue `iterations` x 4 independent
 *                         32x32x16 bf16 MFMAs on register operands; out_dev: float[workgroups * 256], written so that the
 *                         loop is live; *flops (host, may be NULL) receives the FLOP count of the launch.
 * Enqueue only.  Errors: SC_ERR_NULL, SC_ERR_ALIGN, SC_ERR_BAD_SHAPE, SC_ERR_HIP.
 */
sc_status sc_probe_stream_copy(void* dst_dev, const void* src_dev, size_t bytes, void* hip_stream);
sc_status sc_probe_mfma_bf16(int32_t iterations, int32_t workgroups, float* out_dev, double* flops, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SPARSE_CONV_H_ */
