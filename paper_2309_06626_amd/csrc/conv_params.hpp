// Kernel-side description of one masked-convolution launch (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace sc {

// One entry of the gather table: where a group of consecutive K entries of the lowered
// matrix sits relative to the top-left tap of a window (paper Sec. 3, Fig. 1: each row of
// the lowered matrix lists the kh*kw*Cin entries of one sliding window).
struct KEntry {
  int32_t off;   // element offset  dy*xs_h + dx*xs_w + ci*xs_c
  int32_t dydx;  // dy | (dx << 16); dy = ky*dil_h, dx = kx*dil_w; 0x7fff marks padding of K
};

struct ConvParams {
  const void* x;
  const void* wp;          // packed filters [cout_pad][k_pad], K contiguous
  const float* bias;       // may be null
  void* y;
  const int32_t* row_idx;  // ascending kept rows; null = identity (dense run)
  const uint8_t* mask;     // used for the zero fill only
  const KEntry* ktab;      // per K element (element gather only)
  const void* zeros;       // 256 bytes of zeros (source of padded window entries for direct-to-LDS gathers)
  int32_t rows;            // rows of the (compacted) GEMM: kept, or M for a dense run
  int32_t m_total;         // M = N*Ho*Wo
  int32_t h, w, ho_wo, wo;
  int32_t sh, sw, ph, pw;
  int32_t c_in, kh, kw, dil_h, dil_w;
  int32_t c_out;
  int32_t k_pad;           // K rounded up to the K tile
  int32_t k_tiles;
  int64_t xs_n;            // element strides of x
  int32_t xs_h, xs_w;
  int64_t ys_n;            // element strides of y: batch, position within image, channel
  int32_t ys_p, ys_c;
  int32_t relu;
  int32_t zero_fill;       // write zeros at dropped rows
  int32_t mask_spatial;    // mask has ho_wo entries shared by the batch
  int32_t vec_out;         // 0: element stores; 1: y rows are whole 16-byte groups and c_out % 16 == 0; 2: whole groups only
  // compact row formats (NHWC): x holds only the kept rows of the input map, row i = pixel row_idx[i]
  // (pointwise stride-1 layers); y receives only the kept rows, row i = result of row_idx[i]
  int32_t x_compact, y_compact;
  // fused shortcut sum: y = post(act(conv + bias) + residual), residual in the layout of y (may alias it);
  // a dropped row of a dense-layout output receives post(residual) instead of zeros
  const void* residual;    // null: none
  int32_t residual_relu;
  // 1 / 2: the run contracts every row (identity row map, rows = M) and the mask decides at the store: the result of a
  // dropped row is replaced by zeros (1: zero-fill mode) or not stored (2: scatter-only mode).  For layers so small
  // that the kept-row indirection costs more than the rows it saves.  Not with compact operands or a shortcut tensor.
  int32_t masked_store;
  int32_t m_tiles, n_tiles;
  // n / ho_wo and n / wo for 0 <= n < 2^31 as (n * mul) >> shift in 64 bits (exact; host-computed)
  uint32_t div_howo_mul, div_howo_shift, div_wo_mul, div_wo_shift;
  int32_t seg_gpk, seg_gpk_inv, seg_tail;   // row-segment gather: 16-byte groups per window row, entries of the last one inside the window
  uint32_t x_bytes, w_bytes;   // sizes of x and of the packed filters (buffer-load kernels; 0 = too large)
  // split-K launches only: the K tiles of an output tile are divided among `splits` workgroups
  int32_t splits;
  float* partial;          // [m_tiles * n_tiles][splits][BM * BN] float partial sums
  int32_t* counters;       // [m_tiles * n_tiles] arrival counters, zero between launches
  // stream-K launches only: persistent workgroups (a multiple of 8), each with two partial-sum slots in `partial`
  int32_t stream_wgs;
  // slab launches only (igemm_slab_kernel): bytes of one slab buffer in LDS, height and width of the virtual
  // zero-padded image (H + 2 * pad_h, W + 2 * pad_w) and their multiply-shift divisors
  int32_t slab_bytes, slab_hp, slab_wp;
  uint32_t div_hp_mul, div_hp_shift, div_wp_mul, div_wp_shift;
#ifdef SC_TIMING
  long long* dbg;          // development builds only: per-workgroup phase time stamps
#endif
};

// depthwise layers (groups == Cin == Cout, NHWC)
struct DepthwiseParams {
  const void* x;
  const void* wp;          // filters repacked to [kh*kw][C]
  const float* bias;       // may be null
  void* y;
  const int32_t* row_idx;  // items are kept rows (scatter-only and compact output); null: items are dense rows
  const uint8_t* mask;     // non-null: items are dense rows and a lane whose pixel is dropped stores zeros
  int64_t items;
  int32_t c, h, w, ho_wo, wo;
  int32_t kh, kw, sh, sw, ph, pw, dil_h, dil_w;
  int32_t relu, mask_spatial, x_compact, y_compact;
  uint32_t div_howo_mul, div_howo_shift, div_wo_mul, div_wo_shift;
  // LDS-tiled kernel (3x3 windows)
  const int32_t* rank;     // [M]: position of a kept row in the row list (compact output); else null
  int32_t n, ho;           // images, output rows
  int32_t zero_fill;       // dropped pixels of a dense-layout output receive zeros (else they are left alone)
  // compact input of a layer with windows: row of every input pixel in x, -1 for a pixel its producer dropped
  // (such a pixel reads as +0.0); null: a compact input holds the layer's own kept pixels (1x1 windows)
  const int32_t* x_rank;   // [N * H * W]
};

// Bands of output pixels of one image.  Without `split` band i holds the output rows [i*bh, (i+1)*bh) (the
// last band of an image may be shorter).  With `split` every such run of bh rows is cut into two bands of
// half its pixels each (the cut may fall inside a row): a way to give persistent workgroups two equal steps
// where one band per workgroup is all there is (56 rows: 8 x 7 rows -> 16 bands of 196 pixels).
__host__ __device__ inline void band_pixel_range(int band_in_image, int bh, int split, int ho, int wo, int* first,
                                                 int* end) {
  const int run = split ? band_in_image >> 1 : band_in_image;
  const int p0 = run * bh * wo;
  const int px = (ho - run * bh < bh ? ho - run * bh : bh) * wo;
  if (!split) { *first = p0; *end = p0 + px; return; }
  const int half = (px + 1) >> 1;
  *first = (band_in_image & 1) ? p0 + half : p0;
  *end = (band_in_image & 1) ? p0 + px : p0 + half;
}
__host__ __device__ inline int band_of_pixel(int pixel_in_image, int bh, int split, int ho, int wo) {
  const int run = (pixel_in_image / wo) / bh;
  if (!split) return run;
  const int p0 = run * bh * wo;
  const int px = (ho - run * bh < bh ? ho - run * bh : bh) * wo;
  return 2 * run + (pixel_in_image - p0 >= ((px + 1) >> 1) ? 1 : 0);
}
__host__ __device__ inline int bands_in_image(int ho, int bh, int split) {
  return (ho + bh - 1) / bh * (split ? 2 : 1);
}

// Division of 0 <= n < 2^31 by d >= 1 as (n * mul) >> shift in 64-bit arithmetic: with l = ceil(log2 d)
// and shift = 31 + l, mul = floor(2^shift / d) + 1 fits 32 bits and the quotient is exact.
inline void magic_div(uint32_t d, uint32_t* mul, uint32_t* shift) {
  uint32_t l = 0;
  while (((uint64_t)1 << l) < d) ++l;
  *shift = 31 + l;
  *mul = (uint32_t)((((uint64_t)1 << *shift) / d) + 1);
}

__device__ __forceinline__ int fast_div(int n, uint32_t mul, uint32_t shift) {
  return (int)(uint32_t)(((uint64_t)(uint32_t)n * mul) >> shift);
}

enum Dtype { kF32 = 0, kF16 = 1, kBF16 = 2 };

constexpr int kThreads = 256;
constexpr int kRowBytes = 128;  // bytes of K per LDS tile row (K tile = 128 B / element size)

struct TileShape { int bm, bn; };

// launcher signature shared by every instantiation
using LaunchFn = hipError_t (*)(const ConvParams&, hipStream_t);

struct KernelEntry {
  int bm, bn;
  LaunchFn vec;   // 16-byte gather through registers (NHWC, Cin*eb % 16 == 0)
  LaunchFn elem;  // element gather (any layout)
  LaunchFn dma;   // 16-byte gather straight into LDS (additionally needs channel-contiguous stores)
  LaunchFn dma2;  // the same with a two-tile ring: less LDS, more workgroups per CU (shallow K)
  LaunchFn splitk; // direct-to-LDS gather, deep ring, K divided among several workgroups (null: no such shape)
  size_t lds_bytes;
};

// the stream-K form of tile bm x bn for a 16-bit dtype, or null (igemm_streamk.hip)
LaunchFn streamk_kernel(int dtype, int bm, int bn);

// the row-segment-gather form of tile bm x bn for a 16-bit dtype, or null (igemm_rowseg.hip)
LaunchFn rowseg_kernel(int dtype, int bm, int bn);

// per-dtype kernel tables (defined in igemm_<dtype>.hip)
const KernelEntry* kernels_bf16(int* count);
const KernelEntry* kernels_f16(int* count);
const KernelEntry* kernels_f32(int* count);

// depthwise.hip
hipError_t depthwise_launch(int dtype, const DepthwiseParams& p, hipStream_t stream);
hipError_t depthwise_pack(int dtype, const void* w, void* wp, int c, int taps, hipStream_t stream);
hipError_t depthwise_rank(const int32_t* row_idx, const int32_t* kept_dev, int32_t* rank, int64_t m, hipStream_t stream);

}  // namespace sc
