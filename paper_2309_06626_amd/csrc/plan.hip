// Host side of the C ABI (validation, workspace carving, tile choice, launches) and the small
// plan-time kernels: mask -> row-index compaction, filter packing, gather-table build, and
// the glue operators of the test networks.
#include "../../include/sparse_conv.h"

#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>

#include "band_kernel.hpp"
#include "bandpp_kernel.hpp"
#include "bandrow_kernel.hpp"
#include "bandstream_kernel.hpp"
#include "bandtap_kernel.hpp"
#include "conv_params.hpp"
#include "igemm_buf_kernel.hpp"
#include "igemm_slab_kernel.hpp"
#include "igemm_streamk_kernel.hpp"
#include "igemm_panel_kernel.hpp"

namespace sc {

static thread_local int32_t g_last_hip = 0;
#ifdef SC_TIMING
static long long* g_dbg = nullptr;   // development builds only
#endif

static inline bool hip_failed(hipError_t e) {
  if (e != hipSuccess) { g_last_hip = (int32_t)e; return true; }
  return false;
}
#define SC_HIP(expr) do { if (hip_failed((expr))) return SC_ERR_HIP; } while (0)

// the other translation units of the library report their HIP failures through this
void note_hip_error(int32_t code) { g_last_hip = code; }

// ------------------------------------------------------------------------------------------------
// Mask -> ascending list of kept rows (Alg. 2, indirection init: positions are visited in
// ascending order and appended only where the mask is set).  Two passes, no inter-workgroup
// waiting: each wavefront owns a segment of kSeg rows; pass 1 counts with ballots, pass 2 sums
// the counts of the earlier segments and scatters with ballot + lane rank.
// ------------------------------------------------------------------------------------------------
constexpr int kSeg = 1024;

__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// (copy, may be null: the plan's private copy of the mask, mask_len bytes, written on the way -- the first mask_len
// rows read exactly those bytes)
__global__ __launch_bounds__(256) void mask_count_kernel(const uint8_t* __restrict__ mask, int m, int period,
                                                         int nseg, int32_t* __restrict__ counts,
                                                         uint8_t* __restrict__ copy, int mask_len) {
  const int lane = threadIdx.x & 63;
  const int seg = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (seg >= nseg) return;
  const int r0 = seg * kSeg;
  int cnt = 0;
  for (int it = 0; it < kSeg / 64; ++it) {
    int r = r0 + it * 64 + lane;
    const uint8_t v = r < m ? mask[period ? r % period : r] : (uint8_t)0;
    if (copy && r < mask_len) copy[r] = v;
    bool keep = v != 0;
    cnt += __popcll(__ballot(keep));
  }
  if (lane == 0) counts[seg] = cnt;
}

__global__ __launch_bounds__(256) void mask_scatter_kernel(const uint8_t* __restrict__ mask, int m, int period,
                                                           int nseg, const int32_t* __restrict__ counts,
                                                           int32_t* __restrict__ row_idx,
                                                           int32_t* __restrict__ kept_out) {
  const int lane = threadIdx.x & 63;
  const int seg = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (seg >= nseg) return;
  int part = 0;
  for (int i = lane; i < seg; i += 64) part += counts[i];
  int base = wave_sum(part);
  const int r0 = seg * kSeg;
  for (int it = 0; it < kSeg / 64; ++it) {
    int r = r0 + it * 64 + lane;
    bool keep = r < m && mask[period ? r % period : r] != 0;
    unsigned long long b = __ballot(keep);
    int rank = __popcll(b & ((1ull << lane) - 1ull));
    if (keep) row_idx[base + rank] = r;
    base += __popcll(b);
  }
  if (seg == nseg - 1 && lane == 0) {
    kept_out[0] = base;
    kept_out[1] = 0;      // the per-band maximum, raised by band_rows_kernel
    kept_out[2] = 0;      // the widest slab of a 128-row / 256-row tile, raised by slab_span_kernel
    kept_out[3] = 0;
  }
}

// Slab kernel (igemm_slab_kernel.hpp): virtual rows between the window corner of the first and of the last kept row of
// every tile of 128 and of 256 kept rows, plus the window height; the maximum over the tiles sizes the LDS slab.
__global__ __launch_bounds__(256) void slab_span_kernel(const int32_t* __restrict__ row_idx, const int32_t* __restrict__ kept_dev,
                                                        int ho_wo, int wo, int hp, int kh, int32_t* __restrict__ span_out) {
  const int kept = kept_dev[0];
  const int tile = blockIdx.x * 256 + threadIdx.x;
  auto vrow = [&](int r) { return (r / ho_wo) * hp + (r % ho_wo) / wo; };
  for (int b = 0; b < 2; ++b) {
    const int bm = 128 << b;
    const int64_t m0 = (int64_t)tile * bm;
    if (m0 >= kept) continue;
    const int last = (int)min((int64_t)kept, m0 + bm) - 1;
    atomicMax(span_out + b, vrow(row_idx[last]) + kh - vrow(row_idx[m0]));
  }
}

// The inverse map for a compact tensor: rank[r] = position of row r among the kept rows, -1 for a dropped
// row.  Same two passes (counts from mask_count_kernel).
__global__ __launch_bounds__(256) void mask_rank_kernel(const uint8_t* __restrict__ mask, int m, int period,
                                                        int nseg, const int32_t* __restrict__ counts,
                                                        int32_t* __restrict__ rank_out,
                                                        int32_t* __restrict__ kept_out) {
  const int lane = threadIdx.x & 63;
  const int seg = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (seg >= nseg) return;
  int part = 0;
  for (int i = lane; i < seg; i += 64) part += counts[i];
  int base = wave_sum(part);
  const int r0 = seg * kSeg;
  for (int it = 0; it < kSeg / 64; ++it) {
    int r = r0 + it * 64 + lane;
    bool keep = r < m && mask[period ? r % period : r] != 0;
    unsigned long long b = __ballot(keep);
    int rank = __popcll(b & ((1ull << lane) - 1ull));
    if (r < m) rank_out[r] = keep ? base + rank : -1;
    base += __popcll(b);
  }
  if (seg == nseg - 1 && lane == 0) *kept_out = base;
}

// ------------------------------------------------------------------------------------------------
// Filter packing: [cout_pad][k_pad] with K = (ky, kx, ci) contiguous, zero padded.  Inside every
// group of 32 output channels the rows are permuted so that MFMA output row 8j + 4h + i holds
// channel 16h + 4j + i: a lane of the result then owns 16 consecutive channels.
// ------------------------------------------------------------------------------------------------
// epad > 0 selects the row-segment K order of the small-channel gather: K' = (ky, e) with e = kx*c_in + ci
// padded to epad entries per window row (the padding holds zeros).
template <typename T>
__global__ void pack_filters_kernel(const T* __restrict__ w, T* __restrict__ wp, int c_out, int c_in, int kh, int kw,
                                    int k, int k_pad, int cout_pad, int nchw, int epad) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)cout_pad * k_pad) return;
  int prow = (int)(idx / k_pad), kk = (int)(idx % k_pad);
  int rho = prow & 31;
  int co = (prow & ~31) + 16 * ((rho >> 2) & 1) + 4 * (rho >> 3) + (rho & 3);
  T v = (T)0.0f;
  bool real = co < c_out && kk < k;
  if (epad > 0 && real) {
    int ky = kk / epad, e = kk % epad;
    real = e < kw * c_in;
    kk = ky * kw * c_in + e;   // position in the plain (ky, kx, ci) order
  }
  if (real) {
    int tap = kk / c_in, ci = kk % c_in;
    int ky = tap / kw, kx = tap % kw;
    int64_t src = nchw ? (((int64_t)co * c_in + ci) * kh + ky) * kw + kx
                       : (((int64_t)co * kh + ky) * kw + kx) * c_in + ci;
    v = w[src];
  }
  wp[idx] = v;
}

// Gather table: entry g covers K entries [g*vec, (g+1)*vec) (vec = 1 for the element gather).
__global__ void build_ktab_kernel(KEntry* __restrict__ tab, int entries, int vec, int k, int c_in, int kw, int dil_h,
                                  int dil_w, int xs_h, int xs_w, int xs_c) {
  int g = blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= entries) return;
  int kk = g * vec;
  KEntry e;
  if (kk < k) {
    int tap = kk / c_in, ci = kk % c_in;
    int dy = (tap / kw) * dil_h, dx = (tap % kw) * dil_w;
    e.off = dy * xs_h + dx * xs_w + ci * xs_c;
    e.dydx = dy | (dx << 16);
  } else {
    e.off = 0;
    e.dydx = 0x7fff;  // row offset no image reaches: the padded K entries read as zero
  }
  tab[g] = e;
}

// Small-channel gather: copy x [N][H][W][C] into the interior of the zero-margined buffer
// [N][Hp][Wp][C] (margins are zeroed once at plan time), 16 bytes per thread; rows of W*C elements are
// a multiple of 8 elements here.
template <typename T>
__global__ void pad_input_kernel(const T* __restrict__ x, T* __restrict__ xp, int n, int h, int row_elems, int hp,
                                 int prow_elems, int top, int left_elems) {
  typedef T vec8 __attribute__((ext_vector_type(8)));
  const int gpr = row_elems >> 3;
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t total = (int64_t)n * h * gpr;
  if (idx >= total) return;
  int g = (int)(idx % gpr);
  int64_t r = idx / gpr;
  int iy = (int)(r % h), b = (int)(r / h);
  const vec8 v = *reinterpret_cast<const vec8*>(x + r * row_elems + g * 8);
  T* dst = xp + ((int64_t)b * hp + iy + top) * prow_elems + left_elems + g * 8;
  __builtin_memcpy(dst, &v, 16);   // destination is only element-aligned
}

__global__ void fill_zero_kernel(uint4* __restrict__ dst, int64_t n16, unsigned char* tail, int ntail) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n16; i += stride) dst[i] = make_uint4(0, 0, 0, 0);
  if (blockIdx.x == 0 && (int)threadIdx.x < ntail) tail[threadIdx.x] = 0;
}

// First compacted row of every band: lower bound of the band's first dense row in the kept-row list.
__global__ void band_start_kernel(const int32_t* __restrict__ row_idx, const int32_t* __restrict__ kept_dev,
                                  int32_t* __restrict__ band_i0, int n_bands, int bands_per_image, int bh, int split,
                                  int ho, int wo) {
  int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b > n_bands) return;
  const int kept = *kept_dev;
  int target;
  if (b == n_bands) {
    target = 0x7fffffff;
  } else {
    int img = b / bands_per_image, first, end;
    band_pixel_range(b - img * bands_per_image, bh, split, ho, wo, &first, &end);
    target = img * ho * wo + first;
  }
  int lo = 0, hi = kept;
  while (lo < hi) {
    int mid = (lo + hi) >> 1;
    if (row_idx[mid] < target) lo = mid + 1; else hi = mid;
  }
  band_i0[b] = lo;
}

// Band-ordered copy of the kept-row list: the kept rows of band b, ascending, stored from index
// r_lo(b) (the band's first dense row) on, so the band kernel finds them without knowing counts.
// The first kept row of every band also raises band_max to the band's kept-row count (it sizes the accumulator blocks of
// the streaming kernel and picks the MFMA block shape of the others: the fullest band is the one a launch waits for).
__global__ void band_rows_kernel(const int32_t* __restrict__ row_idx, const int32_t* __restrict__ kept_dev,
                                 const int32_t* __restrict__ band_i0, int32_t* __restrict__ band_rows,
                                 int bands_per_image, int bh, int split, int ho, int wo, int32_t* __restrict__ band_max) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= *kept_dev) return;
  const int r = row_idx[i];
  const int ho_wo = ho * wo;
  const int img = r / ho_wo;
  const int bi = band_of_pixel(r - img * ho_wo, bh, split, ho, wo);
  const int band = img * bands_per_image + bi;
  int first, end;
  band_pixel_range(bi, bh, split, ho, wo, &first, &end);
  const int i0 = band_i0[band];
  band_rows[img * ho_wo + first + (i - i0)] = r;
  if (i == i0) atomicMax(band_max, band_i0[band + 1] - i0);
}

// ------------------------------------------------------------------------------------------------
// Glue operators for network runs
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ void maxpool_nhwc_kernel(const T* __restrict__ x, T* __restrict__ y, int n, int h, int w, int c, int k,
                                    int s, int p, int ho, int wo) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t total = (int64_t)n * ho * wo * c;
  if (idx >= total) return;
  int ch = (int)(idx % c);
  int64_t pos = idx / c;
  int ox = (int)(pos % wo);
  int oy = (int)((pos / wo) % ho);
  int b = (int)(pos / ((int64_t)wo * ho));
  float best = -INFINITY;
  for (int ky = 0; ky < k; ++ky) {
    int iy = oy * s - p + ky;
    if (iy < 0 || iy >= h) continue;
    for (int kx = 0; kx < k; ++kx) {
      int ix = ox * s - p + kx;
      if (ix < 0 || ix >= w) continue;
      float v = (float)x[(((int64_t)b * h + iy) * w + ix) * c + ch];
      best = fmaxf(best, v);
    }
  }
  y[idx] = (T)best;
}

// 16-bit types, channel count a multiple of 8: a thread owns 8 consecutive channels of one output
// position (16-byte loads and stores; the scalar kernel above moves 2 bytes per thread and access)
template <typename T>
__global__ void maxpool_nhwc_vec8_kernel(const T* __restrict__ x, T* __restrict__ y, int n, int h, int w, int c, int k,
                                         int s, int p, int ho, int wo) {
  typedef T vec8 __attribute__((ext_vector_type(8)));
  const int cg = c >> 3;
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t total = (int64_t)n * ho * wo * cg;
  if (idx >= total) return;
  int g = (int)(idx % cg);
  int64_t pos = idx / cg;
  int ox = (int)(pos % wo);
  int oy = (int)((pos / wo) % ho);
  int b = (int)(pos / ((int64_t)wo * ho));
  float best[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) best[e] = -INFINITY;
  for (int ky = 0; ky < k; ++ky) {
    int iy = oy * s - p + ky;
    if (iy < 0 || iy >= h) continue;
    for (int kx = 0; kx < k; ++kx) {
      int ix = ox * s - p + kx;
      if (ix < 0 || ix >= w) continue;
      const vec8 v = *reinterpret_cast<const vec8*>(x + (((int64_t)b * h + iy) * w + ix) * c + g * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) best[e] = fmaxf(best[e], (float)v[e]);
    }
  }
  vec8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = (T)best[e];
  *reinterpret_cast<vec8*>(y + pos * c + g * 8) = o;
}

// The same for the 3x3 window: the nine loads are unconditional (clamped coordinates; a padded tap is replaced by
// minus infinity afterwards), so they are all in flight at once.
template <typename T>
__global__ void maxpool3_nhwc_vec8_kernel(const T* __restrict__ x, T* __restrict__ y, int n, int h, int w, int c, int s,
                                          int p, int ho, int wo, uint32_t cg_mul, uint32_t cg_shift, uint32_t wo_mul,
                                          uint32_t wo_shift, uint32_t ho_mul, uint32_t ho_shift) {
  typedef T vec8 __attribute__((ext_vector_type(8)));
  const int cg = c >> 3;
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;          // (the launcher keeps n * ho * wo * cg below 2^31)
  if (idx >= n * ho * wo * cg) return;
  const int pos = fast_div(idx, cg_mul, cg_shift), g = idx - pos * cg;
  const int row = fast_div(pos, wo_mul, wo_shift), ox = pos - row * wo;
  const int b = fast_div(row, ho_mul, ho_shift), oy = row - b * ho;
  const int iy0 = oy * s - p, ix0 = ox * s - p;
  vec8 v[9];
  bool ok[9];
#pragma unroll
  for (int ky = 0; ky < 3; ++ky)
#pragma unroll
    for (int kx = 0; kx < 3; ++kx) {
      const int iy = iy0 + ky, ix = ix0 + kx;
      ok[ky * 3 + kx] = (unsigned)iy < (unsigned)h && (unsigned)ix < (unsigned)w;
      const int cy = min(max(iy, 0), h - 1), cx = min(max(ix, 0), w - 1);
      v[ky * 3 + kx] = *reinterpret_cast<const vec8*>(x + (((int64_t)b * h + cy) * w + cx) * c + g * 8);
    }
  float best[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) best[e] = -INFINITY;
#pragma unroll
  for (int tap = 0; tap < 9; ++tap)
#pragma unroll
    for (int e = 0; e < 8; ++e) best[e] = fmaxf(best[e], ok[tap] ? (float)v[tap][e] : -INFINITY);
  vec8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = (T)best[e];
  *reinterpret_cast<vec8*>(y + (int64_t)pos * c + g * 8) = o;
}

template <typename T, bool RELU>
__global__ void add_vec8_kernel(const T* a, const T* b, T* y, int64_t groups) {   // y may alias a or b
  typedef T vec8 __attribute__((ext_vector_type(8)));
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < groups; i += stride) {
    const vec8 va = reinterpret_cast<const vec8*>(a)[i], vb = reinterpret_cast<const vec8*>(b)[i];
    vec8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float v = (float)va[e] + (float)vb[e];
      o[e] = (T)(RELU ? fmaxf(v, 0.0f) : v);
    }
    reinterpret_cast<vec8*>(y)[i] = o;
  }
}

template <typename T, bool RELU>
__global__ void add_kernel(const T* a, const T* b, T* y, int64_t count) {   // y may alias a or b
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < count; i += stride) {
    const float v = (float)a[i] + (float)b[i];
    y[i] = (T)(RELU ? fmaxf(v, 0.0f) : v);
  }
}

// y = post(0 + shortcut): what a fused launch leaves when the mask keeps no row at all
template <typename T>
__global__ void shortcut_only_kernel(const T* __restrict__ res, T* __restrict__ y, int64_t count, int relu) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < count; i += stride) {
    float v = 0.0f + (float)res[i];
    if (relu) v = fmaxf(v, 0.0f);
    y[i] = (T)v;
  }
}

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline int elem_bytes(int dtype) { return dtype == SC_F32 ? 4 : 2; }

// float partial sums of a split-K launch at most (one BM x BN block per workgroup)
constexpr size_t kSplitKPartialBytes = (size_t)48 << 20;
constexpr int kStreamKMostWgs = 1024;   // persistent workgroups of a stream-K launch at most
constexpr int kSplitKMost = 64;   // splits per output tile at most

struct Geometry {
  int32_t ho, wo;
  int64_t m;
  int32_t k, k_pad, k_stride, k_tiles, vec, cout_pad;
  bool vec_gather, vec_out, vec_out8;
  int64_t x_elems, y_elems, mask_len;
  int32_t nseg;
  // workspace carve (byte offsets)
  size_t off_rows, off_counts, off_kept, off_zeros, off_mask, off_wp, off_ktab, off_band, off_band_rows, off_counters, off_partial, total;
  bool splitk_ok;          // the layer may run the split-K kernel (workspace reserved for it)
  // small-channel gather (NHWC, 16-bit, Cin*eb not a multiple of 16 bytes, e.g. the 3-channel stem): a
  // window row of kw*Cin contiguous elements is fetched as ceil(kw*Cin/8) unaligned 16-byte groups
  // from a zero-margined copy of the input, so no tap needs a bounds check
  bool depthwise;          // groups == Cin == Cout: its own kernel, no lowering
  bool rowseg;
  int32_t epad, hp, wp_cols;   // K entries per window row (padded to 8), padded input height and width
  size_t off_xpad;
  size_t off_xrank, off_xcounts;   // depthwise layers with windows: rank map of a compact input, its segment counts
};

static int out_extent(int in, int k, int stride, int pad, int dil) {
  int64_t eff = (int64_t)in + 2 * (int64_t)pad - (int64_t)dil * (k - 1) - 1;
  if (eff < 0) return 0;
  return (int)(eff / stride) + 1;
}

static sc_status check_desc(const sc_conv_desc* d, Geometry* g) {
  if (!d) return SC_ERR_NULL;
  // one group (the paper's lowering) or one channel per group (depthwise, NHWC)
  const bool depthwise = d->groups != 1;
  if (depthwise && !(d->groups == d->c_in && d->c_in == d->c_out && d->layout == SC_NHWC)) return SC_ERR_UNSUPPORTED;
  if (d->dtype != SC_F32 && d->dtype != SC_F16 && d->dtype != SC_BF16) return SC_ERR_UNSUPPORTED;
  if (d->layout != SC_NHWC && d->layout != SC_NCHW) return SC_ERR_UNSUPPORTED;
  if (d->mask_mode != SC_MASK_ROW && d->mask_mode != SC_MASK_SPATIAL) return SC_ERR_UNSUPPORTED;
  if (d->out_mode != SC_OUT_ZERO_FILL && d->out_mode != SC_OUT_SCATTER_ONLY) return SC_ERR_UNSUPPORTED;
  if (d->n < 1 || d->c_in < 1 || d->h < 1 || d->w < 1 || d->c_out < 1 || d->kh < 1 || d->kw < 1 ||
      d->stride_h < 1 || d->stride_w < 1 || d->pad_h < 0 || d->pad_w < 0 || d->dil_h < 1 || d->dil_w < 1)
    return SC_ERR_BAD_SHAPE;
  if (!(d->sparsity < 1.0f)) return SC_ERR_BAD_SHAPE;  // also rejects NaN
  // the gather table packs window offsets into 15 bits
  if (d->h > 16000 || d->w > 16000 || d->pad_h > 16000 || d->pad_w > 16000 ||
      (int64_t)(d->kh - 1) * d->dil_h > 16000 || (int64_t)(d->kw - 1) * d->dil_w > 16000)
    return SC_ERR_BAD_SHAPE;
  g->ho = out_extent(d->h, d->kh, d->stride_h, d->pad_h, d->dil_h);
  g->wo = out_extent(d->w, d->kw, d->stride_w, d->pad_w, d->dil_w);
  if (g->ho < 1 || g->wo < 1) return SC_ERR_BAD_SHAPE;
  const int64_t lim = (int64_t)1 << 31;
  g->m = (int64_t)d->n * g->ho * g->wo;
  g->x_elems = (int64_t)d->n * d->h * d->w * d->c_in;
  g->y_elems = g->m * d->c_out;
  int64_t k = (int64_t)d->kh * d->kw * (depthwise ? 1 : d->c_in);
  g->depthwise = depthwise;
  if (g->m >= lim || g->x_elems >= lim - (1 << 20) || g->y_elems >= lim || k >= (1 << 24) || d->c_out >= (1 << 24))
    return SC_ERR_BAD_SHAPE;
  const int eb = elem_bytes(d->dtype);
  g->vec = 16 / eb;
  g->rowseg = false;
  g->epad = g->hp = g->wp_cols = 0;
  // (window-row gather; not for pointwise layers, whose window row is one pixel and which may be handed
  // the kept rows of their input only)
  if (d->layout == SC_NHWC && d->dtype != SC_F32 && d->c_in % g->vec != 0 && d->dil_w == 1 && d->kw * d->c_in <= 64 &&
      (d->w * d->c_in) % 8 == 0 && d->kh * d->kw > 1 && !depthwise) {
    const int epad = (d->kw * d->c_in + 7) / 8 * 8;
    const int over = (epad - d->kw * d->c_in + d->c_in - 1) / d->c_in;      // pixels the last group reads past the window
    const int max_iy = (g->ho - 1) * d->stride_h - d->pad_h + (d->kh - 1) * d->dil_h;
    const int max_ix = (g->wo - 1) * d->stride_w - d->pad_w + d->kw - 1 + over;
    const int64_t hp = d->pad_h + std::max<int64_t>(d->h, max_iy + 1), wpc = d->pad_w + std::max<int64_t>(d->w, max_ix + 1);
    if ((int64_t)d->n * hp * wpc * d->c_in + 64 < lim - (1 << 20)) {
      g->rowseg = true;
      g->epad = epad;
      g->hp = (int32_t)hp;
      g->wp_cols = (int32_t)wpc;
      k = (int64_t)d->kh * epad;
    }
  }
  g->k = (int32_t)k;
  const int bk = 8 * g->vec;
  g->k_pad = (int32_t)((k + bk - 1) / bk * bk);
  g->k_tiles = g->k_pad / bk;
  // filter rows are spaced by an odd number of K tiles: the band kernel's LDS swizzle relies on it
  g->k_stride = (g->k_tiles & 1) ? g->k_pad : g->k_pad + bk;
  g->cout_pad = (d->c_out + 255) / 256 * 256;
  g->vec_gather = d->layout == SC_NHWC && d->c_in % g->vec == 0;
  g->vec_out = d->layout == SC_NHWC && d->c_out % 16 == 0;
  // output rows that are whole 16-byte groups but no multiple of 16 channels (e.g. 40, 56, 104): vectorised
  // stores in the register-staged tiled kernel only
  g->vec_out8 = d->layout == SC_NHWC && !g->vec_out && d->c_out % g->vec == 0;
  g->mask_len = d->mask_mode == SC_MASK_ROW ? g->m : (int64_t)g->ho * g->wo;
  g->nseg = (int32_t)((g->m + kSeg - 1) / kSeg);
  size_t off = 0;
  g->off_rows = off;   off = align_up(off + (size_t)g->m * 4, 256);
  g->off_counts = off; off = align_up(off + (size_t)g->nseg * 4, 256);
  g->off_kept = off;   off += 256;
  g->off_zeros = off;  off += 256;
  g->off_mask = off;   off = align_up(off + (size_t)g->mask_len, 256);
  g->off_wp = off;     off = align_up(off + (size_t)g->cout_pad * g->k_stride * eb, 256);
  g->off_ktab = off;   off = align_up(off + (size_t)g->k_pad * sizeof(KEntry), 256);
  g->off_band = off;   off = align_up(off + ((size_t)d->n * g->ho + 1) * 4, 256);
  g->off_band_rows = off; off = align_up(off + (size_t)g->m * 4, 256);
  g->off_xpad = off;
  if (g->rowseg) off = align_up(off + ((size_t)d->n * g->hp * g->wp_cols * d->c_in + 64) * eb, 256);
  g->off_xrank = g->off_xcounts = off;
  if (depthwise && d->kh * d->kw > 1) {
    const size_t pixels = (size_t)d->n * d->h * d->w;
    g->off_xrank = off;   off = align_up(off + pixels * 4, 256);
    g->off_xcounts = off; off = align_up(off + ((pixels + kSeg - 1) / kSeg + 1) * 4, 256);
  }
  // split-K (16-bit operands, direct-to-LDS gather, 128-channel tiles, deep K): arrival counters for
  // every output tile (64 x 64 is the smallest split-K tile) and the float partial sums
  g->splitk_ok = d->dtype != SC_F32 && g->vec_gather && g->vec_out && d->c_out >= 128 && g->k_tiles >= 16 && !depthwise;
  g->off_counters = g->off_partial = off;
  if (g->splitk_ok) {
    const size_t tiles = (size_t)((g->m + 63) / 64) * ((d->c_out + 63) / 64);
    g->off_counters = off; off = align_up(off + tiles * 4, 256);
    g->off_partial = off;  off = align_up(off + kSplitKPartialBytes, 256);
  }
  g->total = off;
  return SC_OK;
}

// Band kernel applicability and band height.
struct BandPlan {
  bool ok;
  bool stream;       // filters streamed through an LDS ring instead of resident
  bool pp;           // persistent workgroups, two wavefront groups alternating between transfer and MFMA
  bool tap;          // one band per workgroup of eight wavefronts, filters arriving tap by tap under the MFMAs
  int pp_grid;       // workgroups of that kernel
  int max_kept;      // most kept rows in one band
  int bh, bands_per_image, n_bands, n_tiles, ni_idx, ni;
  int split;         // alternating-group kernel only: every run of bh rows is two bands of half its pixels
  size_t b_bytes, x_bytes, lds;
  bool rowband;      // small-channel layers: window rows read from a zero-margined slab (row-segment K order)
  int rb_pitch, rb_left, rb_in_rows, rb_gpw, rb_tail;
};

constexpr size_t kLdsLimit = 160 * 1024;
// behind the band kernel's slabs: a zeroed KiB and 128 bias floats
constexpr size_t kBandExtraLds = 1024 + 128 * 4;

// 32-row MFMA units the busiest of four wavefronts runs for a band with `cnt` rows, with 32-row (MI = 1) or
// 64-row (MI = 2) blocks dealt round robin; `mi_idx` receives the better shape (at a tie the 64-row block, whose
// two row blocks share every filter fragment read from LDS).
static double band_units(double cnt, int* mi_idx) {
  const double units1 = std::ceil(std::ceil(cnt / 32.0) / 4.0), units2 = 2.0 * std::ceil(std::ceil(cnt / 64.0) / 4.0);
  if (mi_idx) *mi_idx = units1 < units2 ? 0 : 1;
  return std::min(units1, units2);
}

static bool tap_is_automatic(const sc_conv_desc& d, const Geometry& g, const BandPlan& tp, int64_t rows);
static int device_cus();

// Band kernel of the small-channel layers (row-segment K order): window starts must be 4-byte aligned in the slab, K
// at most 24 groups of 16 bytes, 64 output channels per workgroup, bands of at most 512 output pixels.  The tallest
// such band that still leaves a workgroup per compute unit.  SPARSE_CONV_BAND_KERNEL=none keeps such a layer on the
// tiled row-segment kernel, SPARSE_CONV_BAND_HEIGHT=<bh> fixes the band height (tuning and tests).
static BandPlan plan_rowband(const sc_conv_desc& d, const Geometry& g) {
  BandPlan bp;
  std::memset(&bp, 0, sizeof(bp));
  const int eb = elem_bytes(d.dtype);
  const char* variant = std::getenv("SPARSE_CONV_BAND_KERNEL");
  if (variant && std::strcmp(variant, "none") == 0) return bp;
  if (eb != 2 || !g.vec_out || d.dil_w != 1 || (d.stride_w * d.c_in * eb) % 4 != 0) return bp;
  const int gpw = g.epad / 8;
  if (d.kh * gpw > kRowBandMostGroups || (int64_t)d.kh * g.epad > g.k_stride) return bp;
  if (g.wo > kRowBandMaxRows) return bp;
  const int64_t reach = (int64_t)(g.wo - 1) * d.stride_w * d.c_in * eb + (int64_t)gpw * 16;   // end of the last window row
  const int64_t pitch = (int64_t)align_up((size_t)std::max<int64_t>((int64_t)(d.pad_w + d.w) * d.c_in * eb, reach), 16);
  const char* env = std::getenv("SPARSE_CONV_BAND_HEIGHT");
  const int forced_bh = env ? std::atoi(env) : 0;
  auto fits = [&](int bh) {
    const int64_t in_rows = (int64_t)(bh - 1) * d.stride_h + (int64_t)(d.kh - 1) * d.dil_h + 1;
    return (int64_t)bh * g.wo <= kRowBandMaxRows && rowband_slab_at(d.kh * gpw) + in_rows * pitch <= (int64_t)kLdsLimit;
  };
  if (!fits(1)) return bp;
  int bh = 1;
  while (bh < g.ho && fits(bh + 1)) ++bh;
  const int n_tiles = (d.c_out + 63) / 64;
  // (measured on the 7x7 stem at batch 4 .. 64: halving pays only while the bands do not cover the compute units once)
  while (bh > 1 && (int64_t)d.n * ((g.ho + bh - 1) / bh) * n_tiles < (int64_t)device_cus()) bh = (bh + 1) / 2;
  if (forced_bh > 0) { if (!fits(forced_bh)) return bp; bh = forced_bh; }
  bp.ok = bp.rowband = true;
  bp.ni = 2; bp.ni_idx = 1;
  bp.n_tiles = n_tiles;
  bp.bh = bh;
  bp.bands_per_image = (g.ho + bh - 1) / bh;
  bp.n_bands = d.n * bp.bands_per_image;
  bp.rb_pitch = (int)pitch;
  bp.rb_left = d.pad_w;
  bp.rb_in_rows = (bh - 1) * d.stride_h + (d.kh - 1) * d.dil_h + 1;
  bp.rb_gpw = gpw;
  bp.rb_tail = d.kw * d.c_in - (gpw - 1) * 8;
  bp.b_bytes = (size_t)64 * rowband_filter_pitch(d.kh * gpw);
  bp.x_bytes = (size_t)bp.rb_in_rows * pitch;
  bp.lds = rowband_slab_at(d.kh * gpw) + bp.x_bytes;
  return bp;
}

// `rows`: the rows the run is expected to contract (the kept rows of a sparse run, M of a dense one).
static BandPlan plan_band(const sc_conv_desc& d, const Geometry& g, int64_t rows) {
  BandPlan bp;
  std::memset(&bp, 0, sizeof(bp));
  const int eb = elem_bytes(d.dtype);
  if (g.depthwise) return bp;
  if (g.rowseg) return plan_rowband(d, g);
  if (d.layout != SC_NHWC || !g.vec_gather || !g.vec_out) return bp;
  if ((d.c_in / g.vec) % 2 != 0) return bp;      // a K step of two 16-byte groups must stay inside one tap
  if (d.kh * d.kw == 1) return bp;               // no window overlap to exploit: gather kept rows directly
  bp.ni = d.c_out <= 32 ? 1 : d.c_out <= 64 ? 2 : 4;
  bp.ni_idx = bp.ni == 1 ? 0 : bp.ni == 2 ? 1 : 2;
  bp.n_tiles = (d.c_out + 32 * bp.ni - 1) / (32 * bp.ni);
  bp.b_bytes = (size_t)32 * bp.ni * g.k_stride * eb;
  // Alternating-group kernel (persistent workgroups, filters resident, two input slabs): 3x3
  // windows of 16-bit operands with 4 or 8 channel groups per pixel.  It pays once a workgroup
  // walks several bands (measured on MI355X: from three steps on); with fewer, one band per
  // workgroup is faster.  SPARSE_CONV_BAND_KERNEL=single|alternating|tap|no-tap overrides (tuning and tests).
  const char* variant = std::getenv("SPARSE_CONV_BAND_KERNEL");
  const bool want_single = variant && std::strcmp(variant, "single") == 0;
  const bool want_pp = variant && std::strcmp(variant, "alternating") == 0;
  const bool want_tap = variant && std::strcmp(variant, "tap") == 0;
  const bool no_tap = variant && std::strcmp(variant, "no-tap") == 0;      // the automatic choice among the other kernels
  // Tap-pipelined kernel: 3x3 windows of 16-bit operands with 4 or 8 channel groups per pixel, one band per
  // workgroup; the tallest band that fits LDS and 512 rows and costs the fewest rounds of workgroups.
  if (!want_single && !want_pp && !no_tap && d.kh == 3 && d.kw == 3 && d.dtype != SC_F32 &&
      (d.c_in / g.vec == 8 || d.c_in / g.vec == 4)) {
    BandPlan tp = bp;
    tp.ni = d.c_out <= 32 ? 1 : 2;
    tp.ni_idx = tp.ni - 1;
    tp.n_tiles = (d.c_out + 32 * tp.ni - 1) / (32 * tp.ni);
    tp.b_bytes = (size_t)9 * 32 * tp.ni * (d.c_in / g.vec) * 16;
    const char* env = std::getenv("SPARSE_CONV_BAND_HEIGHT");
    const int forced_bh = env ? std::atoi(env) : 0;
    double best = 1e300;
    for (int bh = 1; bh <= g.ho; ++bh) {
      const int64_t ih = (int64_t)(bh - 1) * d.stride_h + (int64_t)2 * d.dil_h + 1;
      const size_t xbytes = align_up((size_t)ih * d.w * d.c_in * eb, 1024);
      if (tp.b_bytes + kTapFixedLds + xbytes > kLdsLimit) break;
      if ((int64_t)bh * g.wo > kTapMaxRows) break;
      const int bpi = (g.ho + bh - 1) / bh;
      const int64_t nb = (int64_t)d.n * bpi * tp.n_tiles;
      const double rounds = std::ceil((double)nb / (double)device_cus());
      const double cost = rounds * ((double)xbytes + (double)tp.b_bytes + 64.0 * bh * g.wo);
      const bool take = forced_bh > 0 ? bh == forced_bh : cost <= best;
      if (take) {
        best = cost;
        tp.ok = true;
        tp.tap = true;
        tp.bh = bh;
        tp.bands_per_image = bpi;
        tp.n_bands = d.n * bpi;
        tp.x_bytes = xbytes;
        tp.lds = tp.b_bytes + kTapFixedLds + xbytes;
      }
    }
    if (tp.ok && (want_tap || tap_is_automatic(d, g, tp, rows))) return tp;
  }
  if (!want_single && d.kh == 3 && d.kw == 3 && d.dtype != SC_F32 &&
      (d.c_in / g.vec == 8 || d.c_in / g.vec == 4)) {
    BandPlan pp = bp;
    pp.ni = d.c_out <= 32 ? 1 : 2;
    pp.ni_idx = pp.ni - 1;
    pp.n_tiles = (d.c_out + 32 * pp.ni - 1) / (32 * pp.ni);
    pp.b_bytes = (size_t)32 * pp.ni * g.k_stride * eb;
    // SPARSE_CONV_BAND_HEIGHT=<bh> or <bh>,split overrides the search (tuning and tests)
    const char* env = std::getenv("SPARSE_CONV_BAND_HEIGHT");
    const int forced_bh = env ? std::atoi(env) : 0;
    const int forced_split = (env && std::strstr(env, ",split")) ? 1 : 0;
    const int lanes_max = std::max(1, 256 / pp.n_tiles);
    int best_steps = 0;
    double best = 1e300;
    // whole runs of bh rows, and runs cut into two bands of half their pixels
    for (int bh = 1; bh <= g.ho; ++bh) {
      for (int split = 0; split <= 1; ++split) {
        // rows of output a band touches: a half band of an odd run reaches into the middle row from either side
        const int rows_out = split ? bh / 2 + 1 : bh;
        if (split && bh < 2) continue;
        int64_t ih = (int64_t)(rows_out - 1) * d.stride_h + (int64_t)(d.kh - 1) * d.dil_h + 1;
        size_t xbytes = align_up((size_t)ih * d.w * d.c_in * eb, 1024);
        if (pp.b_bytes + 2 * xbytes + kPPFixedLds > kLdsLimit) continue;
        const int64_t band_px = split ? ((int64_t)bh * g.wo + 1) / 2 : (int64_t)bh * g.wo;
        if (band_px > kPPMaxRows) continue;
        int bpi = bands_in_image(g.ho, bh, split);
        int64_t nb = (int64_t)d.n * bpi;
        int lanes = (int)std::min<int64_t>(nb, lanes_max);
        int steps = (int)((nb + lanes - 1) / lanes);
        // a step costs its band plus a fixed part (halo rows, barrier, transfer latency)
        double cost = steps * ((split ? 0.5 * bh : (double)bh) + 1.5);
        const bool take = forced_bh > 0 ? (bh == forced_bh && split == forced_split) : cost <= best;
        if (take) {
          best = cost;
          best_steps = steps;
          pp.ok = true;
          pp.pp = true;
          pp.bh = bh;
          pp.split = split;
          pp.bands_per_image = bpi;
          pp.n_bands = (int)nb;
          pp.x_bytes = xbytes;
          pp.lds = pp.b_bytes + 2 * xbytes + kPPFixedLds;
          pp.pp_grid = lanes * pp.n_tiles;
        }
      }
    }
    // two channel tiles would transfer every band twice: measured slower than the tiled kernel
    if (pp.ok && (want_pp || (best_steps >= 3 && pp.n_tiles == 1))) return pp;
    // Exactly two equal steps per workgroup (split bands, as many runs of rows as workgroups): the second band's
    // transfer hides behind the first one's MFMAs and stores, which is worth 4-8 % on the stage-1 ResNet layer at
    // batch 32 -- unless halving the bands costs MFMA blocks (64-row blocks that a whole run fills well fall apart
    // into more 32-row blocks: s = 0.25 there, 3 units per run against 2 + 2 per pair of halves).
    // The slowest workgroup sets the kernel's time, so the counts are those of a band three standard deviations
    // above the mean of a random mask (at s = 0.4 a half band keeps 118 rows on average, but more than the 128 of
    // four blocks in some workgroup of nearly every launch).
    if (pp.ok && pp.split && best_steps == 2 && pp.n_tiles == 1 && pp.n_bands == 2 * pp.pp_grid && !want_single) {
      const double drop = 1.0 - (double)rows / (double)g.m;
      auto busiest = [&](double mean) { return mean + 3.0 * std::sqrt(std::max(mean * drop, 0.0)); };
      const double whole = band_units(busiest((double)rows / (pp.n_bands / 2)), nullptr);
      const double halves = 2.0 * band_units(busiest((double)rows / pp.n_bands), nullptr);
      if (halves <= std::max(whole, 2.0)) return pp;
    }
  }
  if (bp.b_bytes > 96 * 1024) {
    // Filters too large to stay resident: stream them (16-bit types, whole 128-byte K tiles per tap,
    // 64 or 128 channels per workgroup).  Taller bands amortise the filter traffic, which every
    // workgroup pays in full; rows are capped by the accumulator registers (128 rows per MI step).
    if (d.dtype == SC_F32 || (d.c_in / g.vec) % 8 != 0 || bp.ni < 2) return bp;
    bp.stream = true;
    bp.b_bytes = (size_t)kStreamStages * 32 * bp.ni * kRowBytes;
    const char* env = std::getenv("SPARSE_CONV_BAND_HEIGHT");
    const int forced_bh = env ? std::atoi(env) : 0;
    int best_bh = 0;
    int64_t best_wg = 0;
    for (int bh = 1; bh <= g.ho; ++bh) {
      int64_t ih = (int64_t)(bh - 1) * d.stride_h + (int64_t)(d.kh - 1) * d.dil_h + 1;
      size_t xbytes = align_up((size_t)ih * d.w * d.c_in * eb, 1024);
      if (bp.b_bytes + xbytes + kBandExtraLds > kLdsLimit) break;
      if ((int64_t)bh * g.wo > (bp.ni == 4 ? 384 : 512)) break;   // accumulator registers: 3 / 4 blocks of 128 rows
      int bpi = (g.ho + bh - 1) / bh;
      int64_t nwg = (int64_t)d.n * bpi * bp.n_tiles;
      // the tallest band that still gives every CU a workgroup; failing that, one output row per
      // band (the most workgroups); SPARSE_CONV_BAND_HEIGHT overrides (tuning and tests)
      const bool take = forced_bh > 0 ? bh == forced_bh : (nwg >= 256 || best_bh == 0);
      if (take) { best_bh = bh; best_wg = nwg; bp.x_bytes = xbytes; }
    }
    (void)best_wg;
    if (best_bh == 0) { bp.stream = false; return bp; }
    bp.ok = true;
    bp.bh = best_bh;
    bp.bands_per_image = (g.ho + best_bh - 1) / best_bh;
    bp.n_bands = d.n * bp.bands_per_image;
    bp.lds = bp.b_bytes + bp.x_bytes + kBandExtraLds;
    return bp;
  }
  double best = 1e300;
  for (int bh = 1; bh <= g.ho; ++bh) {
    int64_t ih = (int64_t)(bh - 1) * d.stride_h + (int64_t)(d.kh - 1) * d.dil_h + 1;
    size_t xbytes = align_up((size_t)ih * d.w * d.c_in * eb, 1024);
    if (bp.b_bytes + xbytes + kBandExtraLds > kLdsLimit) break;
    if ((int64_t)bh * g.wo > kBandMaxRows) break;
    int bpi = (g.ho + bh - 1) / bh;
    int64_t nb = (int64_t)d.n * bpi * bp.n_tiles;
    double rounds = std::ceil((double)nb / 256.0);
    double cost = rounds * ((double)xbytes + (double)bp.b_bytes + 64.0 * bh * g.wo);
    if (cost <= best) {
      best = cost;
      bp.ok = true;
      bp.bh = bh;
      bp.bands_per_image = bpi;
      bp.n_bands = d.n * bpi;
      bp.x_bytes = xbytes;
      bp.lds = bp.b_bytes + xbytes + kBandExtraLds;
    }
  }
  return bp;
}

// Compute units of the current device (256 on MI355X), asked once per process.
static int device_cus() {
  static std::atomic<int> cached{0};
  int v = cached.load();
  if (v > 0) return v;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) {
    (void)hipGetLastError();
    cus = 256;
  }
  cached.store(cus);
  return cus;
}

// When the tap-pipelined kernel is the automatic choice: one channel tile (two would transfer every band twice) and
// at most one workgroup per compute unit.  Measured on MI355X, sparse run / dense run in us: ResNet18 stage-1 layer
// at batch 32, s = 0.5: 8.7 / 11.4 against 10.9 / 13.9 with the alternating-group kernel (s = 0.25: 10.5 against
// 13.6 with one band per workgroup); detector y2: 10.5 / 11.6 against 17.4 / 17.2; at batch 64 (two rounds of
// workgroups, nothing to overlap the second round's transfers with) 17.8 against 16.6 for persistent workgroups.
static bool tap_is_automatic(const sc_conv_desc& d, const Geometry& g, const BandPlan& tp, int64_t rows) {
  (void)d; (void)g; (void)rows;
  return tp.n_tiles == 1 && (int64_t)tp.n_bands * tp.n_tiles <= device_cus();
}

}  // namespace sc

using namespace sc;

struct sc_plan {
  sc_conv_desc desc;
  Geometry geo;
  BandPlan band;                   // of the sparse run (the band tables in the workspace follow it)
  BandPlan band_dense;             // of the dense run, which needs no tables: it may cut the bands differently
  const BandTable* band_table;
  const BandStreamTable* stream_table;
  const BandPPTable* pp_table;
  const BandTapTable* tap_table;
  unsigned char* ws;
  int64_t kept;
  const KernelEntry* table;
  int table_count;
  struct Pick { int ti, splits; bool masked; };
  Pick pick[2];                    // tiled launch of the sparse / dense run when nothing is forced: tile, K splits, and
                                   // (sparse run) whether every row is contracted and the mask decides at the store
  bool prefer_tiled[2];            // measured by sparse_conv_plan_tune: the tiled launch beat the band / row-panel kernel
  bool tuned;                      // pick and prefer_tiled come from measurements on this device, not from the cost model
  LaunchFn panel;                  // row-panel kernel of the plan's dtype (null: none)
  int tile_splitk;                 // index of the 64 x 128 entry, the tile of automatic split-K launches (-1: none)
  int forced[2];                   // -1 = automatic, >= 0 generic tile index, kForceBand = band kernel
  int gather_pipeline;             // 0 = automatic, 1 = through registers, 2 = straight into LDS
  int split_k;                     // 0 = automatic, 1 = never, n >= 2 = n splits wherever the kernel applies
  int row_panel;                   // 0 = automatic, 1 = never, 2 = wherever the kernel applies
  int stream_k;                    // 0 = automatic, 1 = never, n >= 2 = n persistent workgroups wherever the kernel applies
  int masked_store;                // 0 = automatic, 1 = never, 2 = wherever it applies (sparse runs of dense NHWC operands)
  bool x_rank_set;                 // sparse_conv_plan_set_input_mask has filled the rank map of a compact input
  // slab form of the tiled kernel (deep 3x3 layers)
  struct Slab { int bm, splits; };
  bool slab_ok;                    // the layer's geometry admits it
  int slab;                        // 0 = automatic, 1 = never, 2 = wherever it applies, 128 / 256 = with tiles of that many rows
  int slab_span[2][2];             // [sparse, dense run][128-row, 256-row tiles]: virtual rows of the widest tile's slab
  Slab slab_auto[2];               // what an automatic launch of the sparse / dense run takes (bm == 0: another kernel)
};
constexpr int kForceBand = -2;

namespace sc {

// Tile choice for a GEMM of `rows` x c_out x K.  The row count is the compacted one, so a heavily masked layer
// gets other tiles than its dense twin (Sec. 3.2: the GEMM range shrinks with the sparsity).  Every candidate
// (tile shape x K splits, and for the sparse run the variant that contracts every row and masks at the store)
// is priced with a small model of one launch on this device and the cheapest wins.  The constants are
// measurements on MI355X, each of one quantity:
//   kLaunchUs     what a launch costs beyond the lifetime of its workgroups (dispatch ramp and drain)
//   kWgFixedUs    set-up and epilogue of a workgroup; kRowListUs more when rows come through the row list
//                 (a dependent round trip to memory before the first transfer, and the zero fill)
//   kIngestKBus   what a compute unit moves from L2 into LDS per microsecond with 1, 2, 3+ workgroups resident
//                 (the K loops of these kernels are bound by that path, not by the matrix pipes)
//   kMfmaShare    share of the matrix peak a K loop sustains when it is the bound
//   kExchangeKBus rate at which float partial sums of a split K walk travel between workgroups (device-scope
//                 stores and loads: across the fabric between the dies' L2 caches)
// The model is good to about 15 %; sparse_conv_plan_tune replaces its choice by a measured one.
constexpr double kLaunchUs = 3.0, kWgFixedUs = 1.0, kRowListUs = 0.6, kMfmaShare = 0.85, kExchangeKBus = 4000.0;
constexpr double kIngestKBus[3] = {62.0, 110.0, 120.0};
constexpr double kIngestEightWavesKBus = 76.0;      // one resident workgroup of eight wavefronts
constexpr double kClockPerUs = 2100.0;

// LDS bytes of the kernel form a tile of this layer runs (decides how many workgroups share a compute unit)
static size_t tile_lds_bytes(const sc_plan* pl, const KernelEntry& ke) {
  const Geometry& g = pl->geo;
  if (g.vec_gather && g.vec_out && pl->gather_pipeline != 1) {
    const int stages = g.k_tiles <= 2 ? 2 : 3;
    return (size_t)stages * (ke.bm + ke.bn) * kRowBytes + (ke.bm + 4) * 4 + (size_t)ke.bn * 4;
  }
  return 2 * (size_t)(ke.bm + ke.bn) * kRowBytes + (size_t)ke.bm * 4;
}

// predicted microseconds of one tiled launch: `rows` rows through tile ke with K cut into `splits`;
// `listed`: rows come through the kept-row list and dropped rows are zero-filled by their owners
static double predict_us(const sc_plan* pl, const KernelEntry& ke, int64_t rows, int splits, bool listed) {
  const Geometry& g = pl->geo;
  const sc_conv_desc& d = pl->desc;
  const int cus = device_cus();
  const int64_t tiles = ((rows + ke.bm - 1) / ke.bm) * ((d.c_out + ke.bn - 1) / ke.bn);
  const int64_t wgs = tiles * splits;
  const int n_kt = (g.k_tiles + splits - 1) / splits;
  const double kb_wg = (double)(ke.bm + ke.bn) * kRowBytes * n_kt / 1024.0;          // through the L1 path
  const double peak = d.dtype == SC_F32 ? 4096.0 * 157.3 / 2500.0 : 4096.0;          // FLOP per clock and compute unit
  const int bk = kRowBytes / elem_bytes(d.dtype);
  const double mfma_us = 2.0 * ke.bm * ke.bn * bk * n_kt / (peak * kMfmaShare * kClockPerUs);
  const bool eight_waves = ke.bm * ke.bn >= 128 * 128 && g.vec_gather && g.vec_out && d.dtype != SC_F32 && d.c_in % 64 == 0;
  int occ = (int)std::min<size_t>(kLdsLimit / std::max<size_t>(tile_lds_bytes(pl, ke), 1), eight_waves ? 2 : 4);
  occ = std::max(occ, 1);
  const int c = (int)std::max<int64_t>(1, std::min<int64_t>(occ, (wgs + cus - 1) / cus));   // resident per compute unit
  const double rounds = std::ceil((double)wgs / ((double)cus * c));
  const double ingest = c == 1 && eight_waves ? kIngestEightWavesKBus : kIngestKBus[std::min(c, 3) - 1];
  const double round_us = kWgFixedUs + (listed ? kRowListUs : 0.0) + std::max(c * kb_wg / ingest, c * mfma_us);
  double t = kLaunchUs + rounds * round_us;
  if (splits > 1)   // every split writes its tile of floats, the last arrival reads them all
    t += 2.0 * (double)tiles * splits * ke.bm * ke.bn * 4.0 / 1024.0 / kExchangeKBus;
  return t;
}

static int most_splits(const sc_plan* pl, const KernelEntry& ke, int64_t rows);
static LaunchFn splitk_launcher(const sc_plan* pl, const KernelEntry& ke);
static bool buf_applies(const sc_plan* pl, const KernelEntry& ke);

// K splits the automatic choice considers for a tile: up to four, and only the buffer-load form of the split kernel
// (the older form of the small tiles measured slower than their unsplit launches everywhere)
static int split_candidates(const sc_plan* pl, const KernelEntry& ke, int64_t rows) {
  if (pl->split_k == 1 || !buf_applies(pl, ke) || pl->geo.k_tiles <= 2) return 1;
  if (!buf_splitk_kernel(pl->desc.dtype == SC_BF16 ? kBF16 : kF16, ke.bm, ke.bn)) return 1;
  return std::min(4, most_splits(pl, ke, rows));
}

// the cheapest tiled launch by the model.  Layers the fast gathers do not serve keep their one measured shape.
static sc_plan::Pick model_pick(const sc_plan* pl, int which, int64_t rows) {
  const Geometry& g = pl->geo;
  const sc_conv_desc& d = pl->desc;
  sc_plan::Pick best = {0, 1, false};
  auto find = [&](int bm, int bn) {
    for (int i = 0; i < pl->table_count; ++i)
      if (pl->table[i].bm == bm && pl->table[i].bn == bn) return i;
    return 0;
  };
  if (g.rowseg) { best.ti = d.c_out <= 32 ? find(128, 32) : find(64, 64); return best; }   // window-row gather (stems)
  if (!g.vec_gather) { best.ti = find(128, 64); return best; }                              // element gather
  double best_us = 1e300;
  const bool can_mask = which == 0 && rows < g.m && rows > 0;
  for (int i = 0; i < pl->table_count; ++i) {
    const KernelEntry& ke = pl->table[i];
    if (tile_lds_bytes(pl, ke) > kLdsLimit) continue;
    if (ke.bn > 128 && d.c_out <= 128) continue;                      // more than half of such a tile would be padding
    const int most = split_candidates(pl, ke, rows);
    for (int sp = 1; sp <= most; ++sp) {
      const double t = predict_us(pl, ke, rows, sp, which == 0 && rows < g.m);
      if (t < best_us) { best_us = t; best = {i, sp, false}; }
    }
    if (can_mask && pl->masked_store != 1) {       // every row contracted, the mask decides at the store: the dense launch plus a mask byte per row
      const double t = predict_us(pl, ke, g.m, 1, false) + 0.1;
      if (t < best_us) { best_us = t; best = {i, 1, true}; }
    }
  }
  return best;
}

// Split K?  Layers deep in a network have few rows and a long K: large output tiles cannot fill
// 256 CUs, and with small tiles every workgroup walks the whole K, one L2 round trip after the other.
// Dividing K among workgroups shortens that walk and still gives every CU work.
struct TilePick { int ti, splits; bool masked; };

// Row-panel kernel: short K (pointwise layers), several 64-channel tiles, enough rows to fill the
// CUs with 128-row panels.  There the tiled kernels are bound by the instructions every
// (row tile, channel tile) workgroup repeats; the panel kernel pays them once per row tile.
static bool use_panel(const sc_plan* pl, int which, int64_t rows) {
  const Geometry& g = pl->geo;
  const sc_conv_desc& d = pl->desc;
  const bool applies = pl->panel && pl->forced[which] < 0 && !(pl->prefer_tiled[which] && pl->row_panel != 2) &&
                       pl->gather_pipeline != 1 && pl->row_panel != 1 &&
                       g.vec_gather && g.vec_out && g.k_tiles <= kPanelMaxKTiles && d.c_out <= 1024;
  // (from 96 channels on, i.e. more than one channel tile per panel: 16 -> 96 channels on a 112 x 112 map,
  // batch 64, measured 52 -> 44 us with dense and 38 -> 27 us with compact operands)
  return applies && (pl->row_panel == 2 || (d.c_out >= 96 && rows >= 128 * 256));
}

static bool buf_applies(const sc_plan* pl, const KernelEntry& ke);

// the split-K launcher of a tile: the buffer-load form where the layer admits it, else the direct-to-LDS form
static LaunchFn splitk_launcher(const sc_plan* pl, const KernelEntry& ke) {
  if (buf_applies(pl, ke) && pl->geo.k_tiles > 2) {
    LaunchFn fn = buf_splitk_kernel(pl->desc.dtype == SC_BF16 ? kBF16 : kF16, ke.bm, ke.bn);
    if (fn) return fn;
  }
  return ke.splitk;
}

static int most_splits(const sc_plan* pl, const KernelEntry& ke, int64_t rows) {
  const Geometry& g = pl->geo;
  if (!g.splitk_ok || !splitk_launcher(pl, ke) || pl->split_k == 1 || pl->gather_pipeline == 1) return 1;
  const int64_t tiles = ((rows + ke.bm - 1) / ke.bm) * ((pl->desc.c_out + ke.bn - 1) / ke.bn);
  const int64_t by_buffer = (int64_t)(kSplitKPartialBytes / ((size_t)ke.bm * ke.bn * sizeof(float))) / std::max<int64_t>(tiles, 1);
  return (int)std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(by_buffer, g.k_tiles / 4), kSplitKMost));
}

// Buffer-load form of the tiled kernel: Cin a multiple of the K tile (a K tile then lies inside one tap),
// windows up to 8 x 8, tensors below 2 GiB (the out-of-range marker is offset 2^31).
static bool buf_applies(const sc_plan* pl, const KernelEntry& ke) {
  const sc_conv_desc& d = pl->desc;
  const Geometry& g = pl->geo;
  if (d.dtype == SC_F32) return false;
  const int eb = 2;
  const uint64_t xb = (uint64_t)d.n * d.h * d.w * d.c_in * eb, wb = (uint64_t)g.cout_pad * g.k_stride * eb;
  return buf_kernel(d.dtype == SC_BF16 ? kBF16 : kF16, ke.bm, ke.bn, g.k_tiles <= 2) && g.vec_gather && g.vec_out &&
         pl->gather_pipeline == 0 && d.c_in % 64 == 0 && d.kh <= 8 && d.kw <= 8 && xb < ((uint64_t)1 << 31) &&
         wb < ((uint64_t)1 << 31) && !g.rowseg;
}

// Stream-K launch of the buffer-load tiled kernel: how many persistent workgroups (0: an ordinary launch).
// Needs the split-K workspace (counters per tile, two partial-sum slots per workgroup), at least four K
// steps per workgroup, and step counts the kernel's 32-bit arithmetic holds.
static int stream_k_workgroups(const sc_plan* pl, const KernelEntry& ke, int64_t rows) {
  const Geometry& g = pl->geo;
  if (!g.splitk_ok || pl->stream_k == 1 || g.k_tiles <= 2 || !buf_applies(pl, ke)) return 0;
  if (!streamk_kernel(pl->desc.dtype == SC_BF16 ? kBF16 : kF16, ke.bm, ke.bn)) return 0;
  int want = pl->stream_k >= 2 ? pl->stream_k : 0;      // automatic: off
  if (want == 0) return 0;
  want = std::min((want + 7) / 8 * 8, kStreamKMostWgs);
  const int64_t tiles = ((rows + ke.bm - 1) / ke.bm) * ((pl->desc.c_out + ke.bn - 1) / ke.bn);
  const int64_t total = tiles * g.k_tiles;
  const int64_t by_buffer = (int64_t)(kSplitKPartialBytes / (2 * (size_t)ke.bm * ke.bn * sizeof(float))) / 8 * 8;
  want = (int)std::min<int64_t>(want, by_buffer);
  want = (int)std::min<int64_t>(want, total / 4 / 8 * 8);
  if (want < 8 || total * (want + 1) >= ((int64_t)1 << 31)) return 0;
  return want;
}

// ---- slab form of the tiled kernel --------------------------------------------------------------------
// 3x3 windows, stride 1, no dilation, 16-bit NHWC, input channels in chunks of 32, tensors below 2 GiB.
static bool slab_geometry_ok(const sc_conv_desc& d, const Geometry& g) {
  if (g.depthwise || g.rowseg || d.dtype == SC_F32 || d.layout != SC_NHWC || !g.vec_out) return false;
  if (d.kh != 3 || d.kw != 3 || d.stride_h != 1 || d.stride_w != 1 || d.dil_h != 1 || d.dil_w != 1) return false;
  if (d.pad_h > 2 || d.pad_w > 2 || d.c_in % kSlabCh != 0 || d.c_out < 96) return false;
  const uint64_t xb = (uint64_t)d.n * d.h * d.w * d.c_in * 2, wb = (uint64_t)g.cout_pad * g.k_stride * 2;
  return xb < ((uint64_t)1 << 31) && wb < ((uint64_t)1 << 31) && (int64_t)d.n * (d.h + 2 * d.pad_h) < ((int64_t)1 << 30);
}
// bytes of one slab buffer for tiles of bm rows whose widest slab spans `span` virtual rows (0: it does not fit)
static int slab_buffer_bytes(const sc_conv_desc& d, int bm, int span) {
  const int round = (bm == 256 ? 512 : 256) * 16;      // what one transfer of the whole workgroup covers
  const int64_t bytes = ((int64_t)span * (d.w + 2 * d.pad_w) * kSlabPixelBytes + round - 1) / round * round;
  return span > 0 && bytes <= kSlabMostBytes ? (int)bytes : 0;
}
// dense run: tiles are runs of bm consecutive pixels
static int slab_dense_span(const sc_conv_desc& d, const Geometry& g, int bm) {
  const int hp = d.h + 2 * d.pad_h, ho_wo = g.ho * g.wo;
  auto vrow = [&](int64_t r) { return (int)(r / ho_wo) * hp + (int)(r % ho_wo) / g.wo; };
  int span = 0;
  for (int64_t m0 = 0; m0 < g.m; m0 += bm) span = std::max(span, vrow(std::min<int64_t>(g.m, m0 + bm) - 1) + d.kh - vrow(m0));
  return span;
}
// K splits (by chunks of input channels) of a slab launch with tiles of bm rows: one workgroup per compute unit
static int slab_splits(const sc_plan* pl, int bm, int64_t rows) {
  const Geometry& g = pl->geo;
  if (!g.splitk_ok || pl->split_k == 1) return 1;
  const int64_t tiles = ((rows + bm - 1) / bm) * ((pl->desc.c_out + kSlabBN - 1) / kSlabBN);
  int64_t want = pl->split_k >= 2 ? pl->split_k : std::max<int64_t>(1, device_cus() / std::max<int64_t>(tiles, 1));
  const int64_t by_buffer = (int64_t)(kSplitKPartialBytes / ((size_t)bm * kSlabBN * sizeof(float))) / std::max<int64_t>(tiles, 1);
  want = std::min<int64_t>(std::min<int64_t>(want, by_buffer), std::min<int64_t>(pl->desc.c_in / kSlabCh, kSplitKMost));
  return (int)std::max<int64_t>(want, 1);
}
// the slab launch the options ask for, or the automatic one (bm == 0: none)
static sc_plan::Slab slab_pick(const sc_plan* pl, int which, int64_t rows) {
  const sc_plan::Slab none = {0, 1};
  if (!pl->slab_ok || pl->slab == 1 || rows == 0 || pl->gather_pipeline == 1) return none;
  if (pl->slab == 0) {
    if (pl->forced[which] != -1 || pl->split_k != 0 || pl->stream_k >= 2 || pl->masked_store == 2) return none;
    return pl->slab_auto[which];
  }
  for (int bm = 256; bm >= 128; bm >>= 1) {
    if (pl->slab >= 128 && pl->slab != bm) continue;
    if (slab_buffer_bytes(pl->desc, bm, pl->slab_span[which][bm == 256])) return {bm, slab_splits(pl, bm, rows)};
  }
  return none;
}
static TilePick pick_tile(const sc_plan* pl, int which, int64_t rows) {
  TilePick tp;
  tp.masked = false;
  if (pl->forced[which] >= 0) {          // tuning: the forced tile, split as requested
    tp.ti = pl->forced[which];
    tp.splits = pl->split_k >= 2 ? std::min(pl->split_k, most_splits(pl, pl->table[tp.ti], rows)) : 1;
    tp.masked = pl->masked_store == 2 && which == 0;
    return tp;
  }
  tp.ti = pl->pick[which].ti;
  tp.splits = pl->split_k == 1 ? 1 : std::min(pl->pick[which].splits, most_splits(pl, pl->table[tp.ti], rows));
  tp.masked = pl->masked_store == 2 ? which == 0 : pl->masked_store == 1 ? false : pl->pick[which].masked;
  if (pl->split_k >= 2 && pl->tile_splitk >= 0) {      // on request: that many splits of the 64 x 128 tile
    const int want = std::min(pl->split_k, most_splits(pl, pl->table[pl->tile_splitk], rows));
    if (want >= 2) { tp.ti = pl->tile_splitk; tp.splits = want; tp.masked = false; }
  }
  return tp;
}


// residual (may be null): shortcut tensor in the format of y, fused into the epilogue of a tiled kernel:
// y = post(act(conv + bias) + residual); dropped rows of a dense-layout output receive post(residual).
static sc_status launch_conv(const sc_plan* pl, bool dense, const void* x, const float* bias, void* y,
                             hipStream_t stream, bool x_compact = false, bool y_compact = false,
                             const void* residual = nullptr, int residual_relu = 0) {
  const sc_conv_desc& d = pl->desc;
  const Geometry& g = pl->geo;
  const int which = dense ? 1 : 0;
  const int64_t rows = dense ? g.m : pl->kept;
  const bool zero_fill = !dense && !y_compact && d.out_mode == SC_OUT_ZERO_FILL && pl->kept < g.m;
  // a mask that keeps every row makes the row list the identity: skip the indirection; so does a run
  // whose input and output both hold the kept rows only (row i in, row i out)
  // (not for a depthwise layer with windows: its compact input follows the input's mask, not its own)
  const bool ranked_input = x_compact && g.depthwise && d.kh * d.kw > 1;
  const bool identity = dense || pl->kept == g.m || (x_compact && y_compact && !ranked_input);
  const bool compact = !identity && (x_compact || y_compact);
  const int eb = elem_bytes(d.dtype);
  if (rows == 0) {
    if (d.out_mode == SC_OUT_ZERO_FILL && !y_compact && residual) {
      const dim3 grid((unsigned)std::min<int64_t>((g.y_elems + 255) / 256, 65536)), block(256);
      if (d.dtype == SC_F32)
        hipLaunchKernelGGL(shortcut_only_kernel<float>, grid, block, 0, stream, (const float*)residual, (float*)y, g.y_elems, residual_relu);
      else if (d.dtype == SC_F16)
        hipLaunchKernelGGL(shortcut_only_kernel<_Float16>, grid, block, 0, stream, (const _Float16*)residual, (_Float16*)y, g.y_elems, residual_relu);
      else
        hipLaunchKernelGGL(shortcut_only_kernel<__bf16>, grid, block, 0, stream, (const __bf16*)residual, (__bf16*)y, g.y_elems, residual_relu);
      SC_HIP(hipGetLastError());
    } else if (d.out_mode == SC_OUT_ZERO_FILL && !y_compact) {
      int64_t bytes = g.y_elems * eb;
      int64_t n16 = bytes / 16;
      int ntail = (int)(bytes - n16 * 16);
      int grid = (int)std::min<int64_t>((n16 + 255) / 256 + 1, 4096);
      hipLaunchKernelGGL(fill_zero_kernel, dim3(grid), dim3(256), 0, stream, (uint4*)y, n16,
                         (unsigned char*)y + n16 * 16, ntail);
      SC_HIP(hipGetLastError());
    }
    return SC_OK;
  }
  // the streaming variant measured no faster than the tiled kernel on the benchmark layers, so the
  // automatic choice takes it only on request
  if (g.depthwise) {
    if (residual) return SC_ERR_UNSUPPORTED;
    DepthwiseParams q;
    std::memset(&q, 0, sizeof(q));
    q.x = x;
    q.wp = pl->ws + g.off_wp;
    q.bias = d.has_bias ? bias : nullptr;
    q.y = y;
    // zero-fill runs walk the dense rows and look at the mask; the others walk the kept rows
    q.row_idx = (identity || zero_fill) ? nullptr : reinterpret_cast<const int32_t*>(pl->ws + g.off_rows);
    q.mask = identity ? nullptr : pl->ws + g.off_mask;
    // Only the zero-fill walk visits all M dense rows.  Every other run visits `rows` items: M for a dense run or
    // a mask that keeps everything, the kept rows otherwise -- through the row list, or as the identity over the
    // kept rows when both operands are compact (x and y then hold kept * C elements, not M * C).
    q.items = zero_fill ? g.m : rows;
    q.zero_fill = zero_fill ? 1 : 0;
    q.rank = (compact && y_compact) ? reinterpret_cast<const int32_t*>(pl->ws + g.off_band_rows) : nullptr;
    q.n = d.n; q.ho = g.ho;
    q.c = d.c_in; q.h = d.h; q.w = d.w; q.ho_wo = g.ho * g.wo; q.wo = g.wo;
    q.kh = d.kh; q.kw = d.kw; q.sh = d.stride_h; q.sw = d.stride_w; q.ph = d.pad_h; q.pw = d.pad_w;
    q.dil_h = d.dil_h; q.dil_w = d.dil_w;
    q.relu = d.relu;
    q.mask_spatial = d.mask_mode == SC_MASK_SPATIAL;
    q.x_compact = (compact && x_compact) || ranked_input ? 1 : 0;
    q.y_compact = compact && y_compact ? 1 : 0;
    // A 1x1 layer whose compact input feeds a zero-filled dense output walks the dense rows, so the item number is
    // no longer the row of x: a kept pixel finds its row in the layer's own rank table (input and output pixels
    // coincide for such a window; dropped pixels leave before they read).
    const bool own_rank_input = compact && x_compact && !ranked_input && zero_fill;
    q.x_rank = ranked_input     ? reinterpret_cast<const int32_t*>(pl->ws + g.off_xrank)
               : own_rank_input ? reinterpret_cast<const int32_t*>(pl->ws + g.off_band_rows)
                                : nullptr;
    magic_div((uint32_t)q.ho_wo, &q.div_howo_mul, &q.div_howo_shift);
    magic_div((uint32_t)q.wo, &q.div_wo_mul, &q.div_wo_shift);
    SC_HIP(depthwise_launch(d.dtype == SC_BF16 ? kBF16 : d.dtype == SC_F16 ? kF16 : kF32, q, stream));
    return SC_OK;
  }
  // the band kernels address input and output by dense position: runs with a compact operand take a tiled kernel
  const BandPlan& band = dense ? pl->band_dense : pl->band;
  // (of the band and row-panel kernels only the alternating-group band kernel has a shortcut path: any other
  // fused launch takes a tiled kernel)
  const sc_plan::Slab slab = x_compact ? sc_plan::Slab{0, 1} : slab_pick(pl, which, rows);
  const bool use_band = band.ok && !x_compact && !y_compact && (!residual || ((band.pp || band.tap) && !band.stream)) &&
                        (pl->forced[which] == kForceBand || (pl->forced[which] == -1 && !band.stream && !pl->prefer_tiled[which])) &&
                        !(slab.bm && pl->slab >= 2);
  if (use_band) {
    const BandPlan& b = band;
    BandParams q;
    std::memset(&q, 0, sizeof(q));
    q.x = x;
    q.wp = pl->ws + g.off_wp;
    q.bias = d.has_bias ? bias : nullptr;
    q.y = y;
    q.row_idx = identity ? nullptr : reinterpret_cast<const int32_t*>(pl->ws + g.off_rows);
    q.mask = pl->ws + g.off_mask;
    q.band_i0 = reinterpret_cast<const int32_t*>(pl->ws + g.off_band);
    q.band_rows = reinterpret_cast<const int32_t*>(pl->ws + g.off_band_rows);
    q.h = d.h; q.w = d.w; q.c_in = d.c_in; q.ho = g.ho; q.wo = g.wo; q.c_out = d.c_out;
    q.kh = d.kh; q.kw = d.kw; q.sh = d.stride_h; q.sw = d.stride_w; q.ph = d.pad_h; q.pw = d.pad_w;
    q.dil_h = d.dil_h; q.dil_w = d.dil_w;
    q.k_stride = g.k_stride;
    q.bh = b.bh; q.split = b.split; q.bands_per_image = b.bands_per_image; q.n_bands = b.n_bands; q.n_tiles = b.n_tiles;
    q.b_bytes = (int32_t)b.b_bytes;
    q.x_groups = (int32_t)(b.x_bytes / 16);
    q.relu = d.relu;
    q.zero_fill = zero_fill ? 1 : 0;
    q.mask_spatial = d.mask_mode == SC_MASK_SPATIAL;
    magic_div((uint32_t)g.wo, &q.div_wo_mul, &q.div_wo_shift);
#ifdef SC_TIMING
    q.dbg = g_dbg;
#endif
    if (b.rowband) {
      RowBandParams rq;
      rq.b = q;
      rq.pitch = b.rb_pitch; rq.left = b.rb_left; rq.in_rows = b.rb_in_rows;
      rq.gpw = b.rb_gpw; rq.groups = d.kh * b.rb_gpw; rq.tail = b.rb_tail;
      rq.fpitch = rowband_filter_pitch(rq.groups);
      magic_div((uint32_t)(b.rb_pitch / 16), &rq.div_cpr_mul, &rq.div_cpr_shift);
      int mi_idx = 0;
      band_units(dense || identity ? (double)(std::min(b.bh, g.ho) * g.wo) : (double)b.max_kept, &mi_idx);
      if (4 * b.lds <= kLdsLimit) mi_idx = 0;      // four workgroups per compute unit: only the 32-row form has the registers
      RowBandLaunchFn fn = bandrow_kernel_for(d.dtype == SC_BF16 ? kBF16 : kF16, mi_idx + 1, d.kh, b.rb_gpw);
      if (!fn) return SC_ERR_UNSUPPORTED;
      SC_HIP(fn(rq, b.lds, stream));
      return SC_OK;
    }
    if (b.stream) {
      // every kept row of a band sits in accumulators: 128 rows per MI step
      const int most = dense ? b.bh * g.wo : b.max_kept;
      const int mi = std::max(1, (most + 127) / 128);
      if (mi > (b.ni == 4 ? 3 : 4)) return SC_ERR_UNSUPPORTED;   // cannot happen: the planner caps the band rows
      SC_HIP(pl->stream_table->fn[b.ni == 4 ? 1 : 0][mi - 1](q, b.lds, stream));
      return SC_OK;
    }
    // 32-row (MI = 1) or 64-row (MI = 2) MFMA blocks, dealt to the four wavefronts round robin: the
    // shape that leaves the busiest wavefront fewer 32-row units
    int mi_idx = 0;
    const int band_px = (std::min(b.bh, g.ho) * g.wo + (b.split ? 1 : 0)) / (b.split ? 2 : 1);
    band_units(dense || identity ? (double)band_px : (double)b.max_kept, &mi_idx);
    if (b.tap) {
      // 32-row blocks b = wave, wave + 8: one or two per wavefront, by the fullest band of the run
      const int most = dense || identity ? band_px : b.max_kept;
      if (most > kTapMaxRows) return SC_ERR_UNSUPPORTED;   // cannot happen: the planner caps the band rows
      q.residual = residual;
      q.residual_relu = residual_relu ? 1 : 0;
      const auto& table = residual ? pl->tap_table->fn_res : pl->tap_table->fn;
      SC_HIP(table[d.c_in / g.vec == 8 ? 0 : 1][b.ni - 1][most > 256 ? 1 : 0](q, b.lds, stream));
      return SC_OK;
    }
    if (b.pp) {
      q.residual = residual;
      q.residual_relu = residual_relu ? 1 : 0;
      const auto& table = residual ? pl->pp_table->fn_res : pl->pp_table->fn;
      SC_HIP(table[d.c_in / g.vec == 8 ? 0 : 1][b.ni - 1][mi_idx](q, b.lds, b.pp_grid, stream));
      return SC_OK;
    }
    const int cpp = d.c_in / g.vec;
    const int shape = (d.kh == 3 && d.kw == 3 && cpp == 8) ? 1 : (d.kh == 3 && d.kw == 3 && cpp == 4) ? 2 : 0;
    SC_HIP(pl->band_table->fn[shape][b.ni_idx][mi_idx](q, b.lds, stream));
    return SC_OK;
  }
  if (slab.bm) {
    ConvParams p;
    std::memset(&p, 0, sizeof(p));
    p.x = x;
    p.wp = pl->ws + g.off_wp;
    p.bias = d.has_bias ? bias : nullptr;
    p.y = y;
    p.row_idx = identity ? nullptr : reinterpret_cast<const int32_t*>(pl->ws + g.off_rows);
    p.mask = pl->ws + g.off_mask;
    p.rows = (int32_t)rows;
    p.m_total = (int32_t)g.m;
    p.h = d.h; p.w = d.w; p.ho_wo = g.ho * g.wo; p.wo = g.wo;
    magic_div((uint32_t)p.ho_wo, &p.div_howo_mul, &p.div_howo_shift);
    magic_div((uint32_t)p.wo, &p.div_wo_mul, &p.div_wo_shift);
    p.sh = 1; p.sw = 1; p.ph = d.pad_h; p.pw = d.pad_w;
    p.c_in = d.c_in; p.kh = d.kh; p.kw = d.kw; p.dil_h = 1; p.dil_w = 1;
    p.c_out = d.c_out;
    p.k_pad = g.k_stride; p.k_tiles = g.k_tiles;
    p.relu = d.relu;
    p.zero_fill = zero_fill ? 1 : 0;
    p.mask_spatial = d.mask_mode == SC_MASK_SPATIAL;
    p.vec_out = 1;
    p.y_compact = compact && y_compact ? 1 : 0;
    p.residual = residual;
    p.residual_relu = residual_relu ? 1 : 0;
    p.m_tiles = (int32_t)((rows + slab.bm - 1) / slab.bm);
    p.n_tiles = (d.c_out + kSlabBN - 1) / kSlabBN;
    p.x_bytes = (uint32_t)((uint64_t)d.n * d.h * d.w * d.c_in * eb);
    p.w_bytes = (uint32_t)((uint64_t)g.cout_pad * g.k_stride * eb);
    // (a mask that keeps every row runs over the identity map: its tiles are those of the dense run)
    p.slab_bytes = slab_buffer_bytes(d, slab.bm, std::max(pl->slab_span[which][slab.bm == 256],
                                                          identity ? pl->slab_span[1][slab.bm == 256] : 0));
    p.slab_hp = d.h + 2 * d.pad_h;
    p.slab_wp = d.w + 2 * d.pad_w;
    magic_div((uint32_t)p.slab_hp, &p.div_hp_mul, &p.div_hp_shift);
    magic_div((uint32_t)p.slab_wp, &p.div_wp_mul, &p.div_wp_shift);
    if (p.slab_bytes == 0) return SC_ERR_UNSUPPORTED;    // cannot happen: slab_pick checked the span
    const int splits = std::min(slab.splits, d.c_in / kSlabCh);
    if (splits > 1) {
      p.splits = splits;
      p.partial = reinterpret_cast<float*>(pl->ws + g.off_partial);
      p.counters = reinterpret_cast<int32_t*>(pl->ws + g.off_counters);
    }
    LaunchFn fn = slab_kernel(d.dtype == SC_BF16 ? kBF16 : kF16, slab.bm, splits > 1);
    if (!fn) return SC_ERR_UNSUPPORTED;
    SC_HIP(fn(p, stream));
    return SC_OK;
  }
  TilePick tp = pick_tile(pl, which, rows);
  // every row contracted, the mask looked at only at the store: plain sparse runs of dense operands without a shortcut
  const bool masked = tp.masked && !dense && !identity && !compact && !x_compact && !y_compact && !residual &&
                      d.layout == SC_NHWC && !g.rowseg;
  if (tp.masked && !masked) tp = {tp.ti, 1, false};
  const int ti = tp.ti, splits = masked ? 1 : tp.splits;
  const KernelEntry& ke = pl->table[ti];
  const bool panel = !residual && !masked && use_panel(pl, which, rows);
  ConvParams p;
  std::memset(&p, 0, sizeof(p));
  p.x = x;
  p.wp = pl->ws + g.off_wp;
  p.bias = d.has_bias ? bias : nullptr;
  p.y = y;
  p.row_idx = (identity || masked) ? nullptr : reinterpret_cast<const int32_t*>(pl->ws + g.off_rows);
  p.mask = pl->ws + g.off_mask;
  p.ktab = reinterpret_cast<const KEntry*>(pl->ws + g.off_ktab);
  p.zeros = pl->ws + g.off_zeros;
  p.rows = (int32_t)(masked ? g.m : rows);
  p.masked_store = masked ? (d.out_mode == SC_OUT_ZERO_FILL ? 1 : 2) : 0;
  p.m_total = (int32_t)g.m;
  p.h = d.h; p.w = d.w; p.ho_wo = g.ho * g.wo; p.wo = g.wo;
  magic_div((uint32_t)p.ho_wo, &p.div_howo_mul, &p.div_howo_shift);
  magic_div((uint32_t)p.wo, &p.div_wo_mul, &p.div_wo_shift);
  p.sh = d.stride_h; p.sw = d.stride_w; p.ph = d.pad_h; p.pw = d.pad_w;
  p.c_in = d.c_in; p.kh = d.kh; p.kw = d.kw; p.dil_h = d.dil_h; p.dil_w = d.dil_w;
  p.c_out = d.c_out;
  p.k_pad = g.k_stride; p.k_tiles = g.k_tiles;
  if (d.layout == SC_NHWC) {
    p.xs_n = (int64_t)d.h * d.w * d.c_in; p.xs_h = d.w * d.c_in; p.xs_w = d.c_in;
    p.ys_n = (int64_t)p.ho_wo * d.c_out; p.ys_p = d.c_out; p.ys_c = 1;
  } else {
    p.xs_n = (int64_t)d.c_in * d.h * d.w; p.xs_h = d.w; p.xs_w = 1;
    p.ys_n = (int64_t)d.c_out * p.ho_wo; p.ys_p = 1; p.ys_c = p.ho_wo;
  }
  p.relu = d.relu;
  p.zero_fill = zero_fill && !masked ? 1 : 0;
  p.mask_spatial = d.mask_mode == SC_MASK_SPATIAL;
  p.vec_out = g.vec_out ? 1 : g.vec_out8 ? 2 : 0;
  p.x_compact = compact && x_compact ? 1 : 0;
  p.y_compact = compact && y_compact ? 1 : 0;
  p.residual = residual;
  p.residual_relu = residual_relu ? 1 : 0;
#ifdef SC_TIMING
  p.dbg = g_dbg;
#endif
  p.m_tiles = (int32_t)(((masked ? g.m : rows) + ke.bm - 1) / ke.bm);
  p.n_tiles = (d.c_out + ke.bn - 1) / ke.bn;
  // shallow K (pointwise layers): the workgroup lives for one or two K tiles, so residency, not
  // read-ahead, hides the latency -- take the two-tile ring and fit more workgroups per CU
  LaunchFn fn = !g.vec_gather ? ke.elem
                : (g.vec_out && pl->gather_pipeline != 1) ? (g.k_tiles <= 2 ? ke.dma2 : ke.dma) : ke.vec;
  if (g.rowseg && x_compact) return SC_ERR_UNSUPPORTED;   // the zero-margined copy is built from a dense input
  if (g.rowseg) {
    // small-channel gather: refresh the interior of the zero-margined input copy, then gather window rows
    // from it (no padding in the copy's coordinates: the margins are the padding)
    const int dt = d.dtype == SC_BF16 ? kBF16 : kF16;
    LaunchFn rs = rowseg_kernel(dt, ke.bm, ke.bn);
    if (!rs) return SC_ERR_UNSUPPORTED;
    const int row_elems = d.w * d.c_in, prow_elems = g.wp_cols * d.c_in;
    const int64_t groups = (int64_t)d.n * d.h * (row_elems / 8);
    _Float16* xp = reinterpret_cast<_Float16*>(pl->ws + g.off_xpad);   // 16-bit patterns are moved verbatim
    hipLaunchKernelGGL(pad_input_kernel<_Float16>, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, stream,
                       static_cast<const _Float16*>(x), xp, d.n, d.h, row_elems, g.hp, prow_elems, d.pad_h,
                       d.pad_w * d.c_in);
    SC_HIP(hipGetLastError());
    p.x = xp;
    p.h = g.hp; p.w = g.wp_cols; p.ph = 0; p.pw = 0;
    p.xs_n = (int64_t)g.hp * prow_elems; p.xs_h = prow_elems; p.xs_w = d.c_in;
    p.seg_gpk = g.epad / 8;
    p.seg_gpk_inv = 65536 / p.seg_gpk + 1;   // (g * inv) >> 16 == g / gpk for g < 4096
    p.seg_tail = d.kw * d.c_in - (p.seg_gpk - 1) * 8;
    fn = rs;
  }
  bool fn_is_buf = false;
  if (buf_applies(pl, ke)) {
    const int dt = d.dtype == SC_BF16 ? kBF16 : kF16;
    p.x_bytes = (uint32_t)((uint64_t)d.n * d.h * d.w * d.c_in * eb);
    p.w_bytes = (uint32_t)((uint64_t)g.cout_pad * g.k_stride * eb);
    fn = buf_kernel(dt, ke.bm, ke.bn, g.k_tiles <= 2);
    fn_is_buf = true;
  }
  if (fn_is_buf && splits == 1 && !panel && !masked) {
    const int dt = d.dtype == SC_BF16 ? kBF16 : kF16;
    const int wgs = stream_k_workgroups(pl, ke, rows);
    LaunchFn sk = wgs ? streamk_kernel(dt, ke.bm, ke.bn) : nullptr;
    if (sk) {
      p.stream_wgs = wgs;
      p.partial = reinterpret_cast<float*>(pl->ws + g.off_partial);
      p.counters = reinterpret_cast<int32_t*>(pl->ws + g.off_counters);
      fn = sk;
    }
  }
  if (splits > 1) {
    p.splits = splits;
    p.partial = reinterpret_cast<float*>(pl->ws + g.off_partial);
    p.counters = reinterpret_cast<int32_t*>(pl->ws + g.off_counters);
    fn = splitk_launcher(pl, ke);
  }
  if (panel) {
    p.m_tiles = (int32_t)((rows + kPanelBM - 1) / kPanelBM);
    p.n_tiles = (d.c_out + kPanelBN - 1) / kPanelBN;
    fn = pl->panel;
  }
  SC_HIP(fn(p, stream));
  return SC_OK;
}

static sc_status check_run_args(const sc_plan* plan, const void* x, const float* bias, void* y) {
  if (!plan || !x || !y) return SC_ERR_NULL;
  if (plan->desc.has_bias && !bias) return SC_ERR_NULL;
  if (((uintptr_t)x & 15) || ((uintptr_t)y & 15) || (plan->desc.has_bias && ((uintptr_t)bias & 15)))
    return SC_ERR_ALIGN;
  return SC_OK;
}

// Everything of a plan that depends on the filters: the packed filter matrix (and, once, the gather table).
static sc_status pack_filters(const sc_conv_desc& d, const Geometry& g, unsigned char* ws, const void* w_dev,
                              hipStream_t stream) {
  if (g.depthwise) {
    const int dt = d.dtype == SC_BF16 ? kBF16 : d.dtype == SC_F16 ? kF16 : kF32;
    SC_HIP(depthwise_pack(dt, w_dev, ws + g.off_wp, d.c_in, d.kh * d.kw, stream));
    return SC_OK;
  }
  {
    int64_t total = (int64_t)g.cout_pad * g.k_stride;
    int grid = (int)((total + 255) / 256);
    const int nchw = d.layout == SC_NCHW;
    if (d.dtype == SC_F32)
      hipLaunchKernelGGL(pack_filters_kernel<float>, dim3(grid), dim3(256), 0, stream, (const float*)w_dev,
                         (float*)(ws + g.off_wp), d.c_out, d.c_in, d.kh, d.kw, g.k, g.k_stride, g.cout_pad, nchw, g.rowseg ? g.epad : 0);
    else  // 16-bit patterns are moved verbatim
      hipLaunchKernelGGL(pack_filters_kernel<_Float16>, dim3(grid), dim3(256), 0, stream, (const _Float16*)w_dev,
                         (_Float16*)(ws + g.off_wp), d.c_out, d.c_in, d.kh, d.kw, g.k, g.k_stride, g.cout_pad, nchw, g.rowseg ? g.epad : 0);
    SC_HIP(hipGetLastError());
  }
  // gather table (depends on the geometry only; rebuilt with the filters for simplicity, it is tiny)
  {
    const int vec = g.vec_gather ? g.vec : 1;
    const int entries = g.k_pad / vec;
    int xs_h, xs_w, xs_c;
    if (d.layout == SC_NHWC) { xs_h = d.w * d.c_in; xs_w = d.c_in; xs_c = 1; }
    else { xs_h = d.w; xs_w = 1; xs_c = d.h * d.w; }
    hipLaunchKernelGGL(build_ktab_kernel, dim3((entries + 255) / 256), dim3(256), 0, stream,
                       reinterpret_cast<KEntry*>(ws + g.off_ktab), entries, vec, g.k, d.c_in, d.kw, d.dil_h, d.dil_w,
                       xs_h, xs_w, xs_c);
    SC_HIP(hipGetLastError());
  }
  return SC_OK;
}

// Everything of a plan that depends on the mask (Alg. 2, indirection init): the private mask copy, the
// ascending list of kept rows and its length, the band tables, the rank table of depthwise layers.
// Synchronises the stream (the kept count decides the launch shapes) and checks the count against the
// descriptor's sparsity.
static sc_status build_row_tables(const sc_conv_desc& d, const Geometry& g, unsigned char* ws, const uint8_t* mask_dev,
                                  hipStream_t stream, BandPlan* bp_io, int32_t* kept_out, int32_t* slab_span_out) {
  BandPlan& bp = *bp_io;
  // compaction
  const int period = d.mask_mode == SC_MASK_SPATIAL ? g.ho * g.wo : 0;
  int32_t* counts = reinterpret_cast<int32_t*>(ws + g.off_counts);
  int32_t* rows = reinterpret_cast<int32_t*>(ws + g.off_rows);
  int32_t* kept_dev = reinterpret_cast<int32_t*>(ws + g.off_kept);
  const int cgrid = (g.nseg + 3) / 4;
  // pass 1 also leaves the plan's private copy of the mask (the zero fill of every run reads it)
  hipLaunchKernelGGL(mask_count_kernel, dim3(cgrid), dim3(256), 0, stream, mask_dev, (int)g.m, period,
                     g.nseg, counts, ws + g.off_mask, (int)g.mask_len);
  SC_HIP(hipGetLastError());
  hipLaunchKernelGGL(mask_scatter_kernel, dim3(cgrid), dim3(256), 0, stream, ws + g.off_mask, (int)g.m, period,
                     g.nseg, counts, rows, kept_dev);
  SC_HIP(hipGetLastError());
  if (g.depthwise)   // position of every kept row in the row list (compact output of the LDS-tiled kernels)
    SC_HIP(depthwise_rank(rows, kept_dev, reinterpret_cast<int32_t*>(ws + g.off_band_rows), g.m, stream));

  if (bp.ok) {
    hipLaunchKernelGGL(band_start_kernel, dim3((bp.n_bands + 1 + 255) / 256), dim3(256), 0, stream, rows, kept_dev,
                       reinterpret_cast<int32_t*>(ws + g.off_band), bp.n_bands, bp.bands_per_image, bp.bh, bp.split, g.ho, g.wo);
    SC_HIP(hipGetLastError());
    // kept_dev + 1 holds the per-band maximum (zeroed by the scatter pass, raised by band_rows_kernel)
    hipLaunchKernelGGL(band_rows_kernel, dim3((unsigned)((g.m + 255) / 256)), dim3(256), 0, stream, rows, kept_dev,
                       reinterpret_cast<const int32_t*>(ws + g.off_band),
                       reinterpret_cast<int32_t*>(ws + g.off_band_rows), bp.bands_per_image, bp.bh, bp.split, g.ho, g.wo,
                       kept_dev + 1);
    SC_HIP(hipGetLastError());
  }

  if (slab_geometry_ok(d, g)) {
    hipLaunchKernelGGL(slab_span_kernel, dim3((unsigned)((g.m + 127) / 128 + 255) / 256), dim3(256), 0, stream, rows, kept_dev,
                       g.ho * g.wo, g.wo, d.h + 2 * d.pad_h, d.kh, kept_dev + 2);
    SC_HIP(hipGetLastError());
  }

  int32_t host_vals[4] = {-1, 0, 0, 0};   // kept count, most kept rows in one band, widest slab of a 128-row / 256-row tile
  SC_HIP(hipMemcpyAsync(host_vals, kept_dev, 4 * sizeof(int32_t), hipMemcpyDeviceToHost, stream));
  SC_HIP(hipStreamSynchronize(stream));
  *kept_out = host_vals[0];
  bp.max_kept = host_vals[1];
  slab_span_out[0] = host_vals[2];
  slab_span_out[1] = host_vals[3];

  if (d.sparsity >= 0.0f) {
    // Sec. 3.2: rows in the GEMM = output_size - sparsity * output_size (rounded half up).  The descriptor carries
    // the ratio as a float: where the product falls on a half within that float's rounding interval (0.9 of 135
    // rows), either neighbour is the count the caller's own ratio demands, and both are accepted.
    const double sp = (double)d.sparsity, eps = std::ldexp(std::fabs(sp), -24) + 1e-12;
    const int64_t want_hi = (int64_t)std::floor((1.0 - (sp - eps)) * (double)g.mask_len + 0.5);
    const int64_t want_lo = (int64_t)std::floor((1.0 - (sp + eps)) * (double)g.mask_len + 0.5);
    int64_t have = d.mask_mode == SC_MASK_ROW ? host_vals[0] : host_vals[0] / d.n;
    if (have < want_lo || have > want_hi) return SC_ERR_MASK_COUNT;
  }
  return SC_OK;
}

}  // namespace sc

extern "C" {

sc_status sparse_conv_output_shape(const sc_conv_desc* desc, int32_t* ho, int32_t* wo, int64_t* m) {
  Geometry g;
  sc_status s = check_desc(desc, &g);
  if (s != SC_OK) return s;
  if (ho) *ho = g.ho;
  if (wo) *wo = g.wo;
  if (m) *m = g.m;
  return SC_OK;
}

sc_status sparse_conv_workspace_bytes(const sc_conv_desc* desc, size_t* bytes) {
  if (!bytes) return SC_ERR_NULL;
  Geometry g;
  sc_status s = check_desc(desc, &g);
  if (s != SC_OK) return s;
  *bytes = g.total;
  return SC_OK;
}

sc_status sparse_conv_plan(const sc_conv_desc* desc, const uint8_t* mask_dev, const void* w_dev,
                           void* workspace_dev, size_t workspace_bytes, void* hip_stream, sc_plan** out) {
  if (!out) return SC_ERR_NULL;
  *out = nullptr;
  Geometry g;
  sc_status s = check_desc(desc, &g);
  if (s != SC_OK) return s;
  if (!mask_dev || !w_dev || !workspace_dev) return SC_ERR_NULL;
  if (workspace_bytes < g.total) return SC_ERR_WORKSPACE;
  if (((uintptr_t)workspace_dev & 255) || ((uintptr_t)w_dev & 15)) return SC_ERR_ALIGN;

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  unsigned char* ws = static_cast<unsigned char*>(workspace_dev);
  const sc_conv_desc& d = *desc;
  const int eb = elem_bytes(d.dtype);

  SC_HIP(hipMemsetAsync(ws + g.off_zeros, 0, 256, stream));
  if (g.rowseg)      // margins of the padded input copy stay zero; every run rewrites the interior
    SC_HIP(hipMemsetAsync(ws + g.off_xpad, 0, ((size_t)d.n * g.hp * g.wp_cols * d.c_in + 64) * eb, stream));
  if (g.splitk_ok)   // arrival counters start at zero; every launch leaves them at zero again
    SC_HIP(hipMemsetAsync(ws + g.off_counters, 0, g.off_partial - g.off_counters, stream));
  // (the kept-row count is not known yet: the descriptor's sparsity says what to expect, half the rows if it is silent)
  const int64_t rows_hint = d.sparsity >= 0.0f ? (int64_t)((1.0 - (double)d.sparsity) * (double)g.m + 0.5) : g.m / 2;
  BandPlan bp = plan_band(d, g, rows_hint);
  int32_t kept_host = 0;
  s = pack_filters(d, g, ws, w_dev, stream);
  if (s != SC_OK) return s;
  int32_t slab_span[2] = {0, 0};
  s = build_row_tables(d, g, ws, mask_dev, stream, &bp, &kept_host, slab_span);   // synchronises the stream
  if (s != SC_OK) return s;

  sc_plan* pl = new (std::nothrow) sc_plan;
  if (!pl) return SC_ERR_NULL;
  pl->desc = d;
  pl->geo = g;
  pl->ws = ws;
  pl->kept = kept_host;
  pl->table = d.dtype == SC_BF16 ? kernels_bf16(&pl->table_count)
              : d.dtype == SC_F16 ? kernels_f16(&pl->table_count)
                                  : kernels_f32(&pl->table_count);
  pl->forced[0] = pl->forced[1] = -1;
  pl->prefer_tiled[0] = pl->prefer_tiled[1] = false;
  pl->tuned = false;
  pl->gather_pipeline = 0;
  pl->split_k = 0;
  pl->row_panel = 0;
  pl->stream_k = 0;
  pl->masked_store = 0;
  pl->x_rank_set = false;
  pl->tile_splitk = -1;
  for (int i = 0; i < pl->table_count; ++i)
    if (pl->table[i].splitk && pl->table[i].bm == 64 && pl->table[i].bn == 128) pl->tile_splitk = i;
  if (pl->tile_splitk < 0) pl->geo.splitk_ok = false;
  pl->pick[0] = model_pick(pl, 0, pl->kept);
  pl->pick[1] = model_pick(pl, 1, g.m);
  pl->band = bp;
  pl->band_dense = plan_band(d, g, g.m);
  pl->slab = 0;
  pl->slab_ok = slab_geometry_ok(d, g) && slab_kernel(d.dtype == SC_BF16 ? kBF16 : kF16, 128, false);
  pl->slab_span[0][0] = slab_span[0]; pl->slab_span[0][1] = slab_span[1];
  pl->slab_span[1][0] = pl->slab_ok ? slab_dense_span(d, g, 128) : 0;
  pl->slab_span[1][1] = pl->slab_ok ? slab_dense_span(d, g, 256) : 0;
  // (automatic launches take the slab form only where sparse_conv_plan_tune measured it faster: the cost model's
  // quantities -- bytes through the L1 path, matrix time -- do not rank it, its K loop is bound by LDS reads)
  pl->slab_auto[0] = pl->slab_auto[1] = sc_plan::Slab{0, 1};
  pl->band_table = d.dtype == SC_BF16 ? band_bf16() : d.dtype == SC_F16 ? band_f16() : band_f32();
  pl->stream_table = d.dtype == SC_BF16 ? bandstream_bf16() : d.dtype == SC_F16 ? bandstream_f16() : nullptr;
  pl->pp_table = d.dtype == SC_BF16 ? bandpp_bf16() : d.dtype == SC_F16 ? bandpp_f16() : nullptr;
  pl->tap_table = d.dtype == SC_BF16 ? bandtap_bf16() : d.dtype == SC_F16 ? bandtap_f16() : nullptr;
  pl->panel = d.dtype == SC_BF16 ? panel_bf16() : d.dtype == SC_F16 ? panel_f16() : nullptr;
  (void)eb;
  *out = pl;
  return SC_OK;
}

sc_status sparse_conv_plan_set_mask(sc_plan* plan, const uint8_t* mask_dev, void* hip_stream) {
  if (!plan || !mask_dev) return SC_ERR_NULL;
  const sc_conv_desc& d = plan->desc;
  const Geometry& g = plan->geo;
  BandPlan bp = plan->band;
  int32_t kept_host = 0;
  int32_t slab_span[2] = {0, 0};
  sc_status s = build_row_tables(d, g, plan->ws, mask_dev, static_cast<hipStream_t>(hip_stream), &bp, &kept_host, slab_span);
  if (s != SC_OK) return s;
  plan->kept = kept_host;
  plan->band = bp;
  plan->pick[0] = model_pick(plan, 0, plan->kept);      // (a measured choice belonged to the previous mask's row count)
  plan->prefer_tiled[0] = false;
  plan->slab_span[0][0] = slab_span[0]; plan->slab_span[0][1] = slab_span[1];
  plan->slab_auto[0] = sc_plan::Slab{0, 1};
  return SC_OK;
}

sc_status sparse_conv_plan_set_input_mask(sc_plan* plan, const uint8_t* mask_in_dev, int64_t* kept_in,
                                          void* hip_stream) {
  if (!plan || !mask_in_dev) return SC_ERR_NULL;
  const sc_conv_desc& d = plan->desc;
  const Geometry& g = plan->geo;
  if (!g.depthwise || d.kh * d.kw == 1) return SC_ERR_UNSUPPORTED;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const int64_t pixels = (int64_t)d.n * d.h * d.w;
  if (pixels >= ((int64_t)1 << 31)) return SC_ERR_BAD_SHAPE;
  const int period = d.mask_mode == SC_MASK_SPATIAL ? d.h * d.w : 0;
  const int nseg = (int)((pixels + kSeg - 1) / kSeg);
  int32_t* counts = reinterpret_cast<int32_t*>(plan->ws + g.off_xcounts);
  int32_t* kept_dev = counts + nseg;
  const int cgrid = (nseg + 3) / 4;
  hipLaunchKernelGGL(mask_count_kernel, dim3(cgrid), dim3(256), 0, stream, mask_in_dev, (int)pixels, period, nseg, counts, nullptr, 0);
  SC_HIP(hipGetLastError());
  hipLaunchKernelGGL(mask_rank_kernel, dim3(cgrid), dim3(256), 0, stream, mask_in_dev, (int)pixels, period, nseg, counts,
                     reinterpret_cast<int32_t*>(plan->ws + g.off_xrank), kept_dev);
  SC_HIP(hipGetLastError());
  int32_t kept_host = 0;
  SC_HIP(hipMemcpyAsync(&kept_host, kept_dev, sizeof(int32_t), hipMemcpyDeviceToHost, stream));
  SC_HIP(hipStreamSynchronize(stream));
  plan->x_rank_set = true;
  if (kept_in) *kept_in = kept_host;
  return SC_OK;
}

sc_status sparse_conv_plan_set_filters(sc_plan* plan, const void* w_dev, void* hip_stream) {
  if (!plan || !w_dev) return SC_ERR_NULL;
  if ((uintptr_t)w_dev & 15) return SC_ERR_ALIGN;
  return pack_filters(plan->desc, plan->geo, plan->ws, w_dev, static_cast<hipStream_t>(hip_stream));
}

sc_status sparse_conv_run(const sc_plan* plan, const void* x_dev, const float* bias_dev, void* y_dev,
                          void* hip_stream) {
  sc_status s = check_run_args(plan, x_dev, bias_dev, y_dev);
  if (s != SC_OK) return s;
  return launch_conv(plan, false, x_dev, bias_dev, y_dev, static_cast<hipStream_t>(hip_stream));
}

sc_status sparse_conv_run_rows(const sc_plan* plan, const void* x_dev, int32_t x_rows, const float* bias_dev,
                               void* y_dev, int32_t y_rows, void* hip_stream) {
  sc_status s = check_run_args(plan, x_dev, bias_dev, y_dev);
  if (s != SC_OK) return s;
  if ((x_rows != SC_ROWS_DENSE && x_rows != SC_ROWS_COMPACT) || (y_rows != SC_ROWS_DENSE && y_rows != SC_ROWS_COMPACT))
    return SC_ERR_UNSUPPORTED;
  const sc_conv_desc& d = plan->desc;
  const bool xc = x_rows == SC_ROWS_COMPACT, yc = y_rows == SC_ROWS_COMPACT;
  if ((xc || yc) && d.layout != SC_NHWC) return SC_ERR_UNSUPPORTED;
  const bool pixel_window = d.kh == 1 && d.kw == 1 && d.stride_h == 1 && d.stride_w == 1 && d.pad_h == 0 && d.pad_w == 0;
  // a window that is the pixel itself never reads a dropped pixel; a depthwise layer with larger windows looks
  // every pixel up in the rank map of its input
  if (xc && !pixel_window && !(plan->geo.depthwise && plan->x_rank_set)) return SC_ERR_UNSUPPORTED;
  return launch_conv(plan, false, x_dev, bias_dev, y_dev, static_cast<hipStream_t>(hip_stream), xc, yc);
}

sc_status sparse_conv_run_residual(const sc_plan* plan, const void* x_dev, int32_t x_rows, const float* bias_dev,
                                   const void* residual_dev, int32_t residual_relu, void* y_dev, int32_t y_rows,
                                   void* hip_stream) {
  sc_status s = check_run_args(plan, x_dev, bias_dev, y_dev);
  if (s != SC_OK) return s;
  if (!residual_dev) return SC_ERR_NULL;
  if ((uintptr_t)residual_dev & 15) return SC_ERR_ALIGN;
  if ((x_rows != SC_ROWS_DENSE && x_rows != SC_ROWS_COMPACT) || (y_rows != SC_ROWS_DENSE && y_rows != SC_ROWS_COMPACT))
    return SC_ERR_UNSUPPORTED;
  const sc_conv_desc& d = plan->desc;
  const bool xc = x_rows == SC_ROWS_COMPACT, yc = y_rows == SC_ROWS_COMPACT;
  if ((xc || yc) && d.layout != SC_NHWC) return SC_ERR_UNSUPPORTED;
  const bool pixel_window = d.kh == 1 && d.kw == 1 && d.stride_h == 1 && d.stride_w == 1 && d.pad_h == 0 && d.pad_w == 0;
  if (plan->geo.depthwise || (xc && !pixel_window)) return SC_ERR_UNSUPPORTED;
  return launch_conv(plan, false, x_dev, bias_dev, y_dev, static_cast<hipStream_t>(hip_stream), xc, yc, residual_dev,
                     residual_relu);
}

sc_status dense_conv_run_residual(const sc_plan* plan, const void* x_dev, const float* bias_dev,
                                  const void* residual_dev, int32_t residual_relu, void* y_dev, void* hip_stream) {
  sc_status s = check_run_args(plan, x_dev, bias_dev, y_dev);
  if (s != SC_OK) return s;
  if (!residual_dev) return SC_ERR_NULL;
  if ((uintptr_t)residual_dev & 15) return SC_ERR_ALIGN;
  if (plan->geo.depthwise) return SC_ERR_UNSUPPORTED;
  return launch_conv(plan, true, x_dev, bias_dev, y_dev, static_cast<hipStream_t>(hip_stream), false, false,
                     residual_dev, residual_relu);
}

sc_status dense_conv_run(const sc_plan* plan, const void* x_dev, const float* bias_dev, void* y_dev,
                         void* hip_stream) {
  sc_status s = check_run_args(plan, x_dev, bias_dev, y_dev);
  if (s != SC_OK) return s;
  return launch_conv(plan, true, x_dev, bias_dev, y_dev, static_cast<hipStream_t>(hip_stream));
}

sc_status sparse_conv_plan_tune(sc_plan* plan, const void* x_dev, const float* bias_dev, void* y_dev, void* hip_stream) {
  sc_status st = check_run_args(plan, x_dev, bias_dev, y_dev);
  if (st != SC_OK) return st;
  if (plan->geo.depthwise) return SC_OK;       // one kernel per window shape: nothing to choose
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  SC_HIP(hipStreamSynchronize(stream));
  // Candidates are timed as graphs of back-to-back launches on a stream of the library's own: launched one by one
  // from the host, layers of a few microseconds would all measure the host's launch rate.
  hipStream_t ts = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  SC_HIP(hipStreamCreateWithFlags(&ts, hipStreamNonBlocking));
  if (hip_failed(hipEventCreate(&e0))) { (void)hipStreamDestroy(ts); return SC_ERR_HIP; }
  if (hip_failed(hipEventCreate(&e1))) { (void)hipEventDestroy(e0); (void)hipStreamDestroy(ts); return SC_ERR_HIP; }
  // microseconds per launch of the run as the plan stands (negative: something failed)
  auto time_us = [&](bool dense, int launches, int replays) -> double {
    if (launch_conv(plan, dense, x_dev, bias_dev, y_dev, ts) != SC_OK) return -1.0;     // also sets kernel attributes
    if (hipStreamBeginCapture(ts, hipStreamCaptureModeThreadLocal) != hipSuccess) return -1.0;
    bool ok = true;
    for (int i = 0; i < launches && ok; ++i) ok = launch_conv(plan, dense, x_dev, bias_dev, y_dev, ts) == SC_OK;
    hipGraph_t graph = nullptr;
    if (hipStreamEndCapture(ts, &graph) != hipSuccess || !ok || !graph) {
      if (graph) (void)hipGraphDestroy(graph);
      (void)hipGetLastError();
      return -1.0;
    }
    hipGraphExec_t exec = nullptr;
    double best = -1.0;
    if (hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0) == hipSuccess) {
      for (int rep = 0; rep <= replays; ++rep) {       // replay 0 warms up
        float ms = 0.0f;
        if (hipEventRecord(e0, ts) != hipSuccess || hipGraphLaunch(exec, ts) != hipSuccess ||
            hipEventRecord(e1, ts) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
            hipEventElapsedTime(&ms, e0, e1) != hipSuccess) { best = -1.0; break; }
        const double us = (double)ms * 1e3 / launches;
        if (rep > 0 && (best < 0.0 || us < best)) best = us;
      }
      (void)hipGraphExecDestroy(exec);
    }
    (void)hipGraphDestroy(graph);
    return best;
  };
  sc_status result = SC_OK;
  for (int which = 0; which < 2 && result == SC_OK; ++which) {
    const bool dense = which == 1;
    const int64_t rows = dense ? plan->geo.m : plan->kept;
    if (plan->forced[which] != -1 || rows == 0) continue;
    plan->pick[which] = model_pick(plan, which, rows);
    plan->prefer_tiled[which] = false;
    if (time_us(dense, 100, 4) < 0.0) { result = SC_ERR_HIP; break; }     // clocks up before anything is compared
    sc_plan::Pick best_pick = plan->pick[which];
    bool best_tiled = false;
    double best_us = time_us(dense, 40, 3);
    if (best_us < 0.0) { result = SC_ERR_HIP; break; }
    if (!plan->geo.vec_gather || plan->geo.rowseg) {                   // one tile shape serves these gathers
      const BandPlan& rb = dense ? plan->band_dense : plan->band;
      if (rb.ok && rb.rowband) {                                       // band kernel of the small-channel layers or that tile
        plan->prefer_tiled[which] = true;
        const double us = time_us(dense, 40, 3);
        if (!(us > 0.0 && us < 0.985 * best_us)) plan->prefer_tiled[which] = false;
      }
      continue;
    }
    // candidates: every tile x split (and the masked-store variant) the model prices within 1.6 x of its best
    struct Cand { sc_plan::Pick pick; double predicted; };
    Cand cands[128];
    int n = 0;
    double best_pred = 1e300;
    const bool can_mask = which == 0 && rows < plan->geo.m;
    for (int i = 0; i < plan->table_count && n < 120; ++i) {
      const KernelEntry& ke = plan->table[i];
      if (tile_lds_bytes(plan, ke) > kLdsLimit) continue;
      const int most = split_candidates(plan, ke, rows);
      for (int sp = 1; sp <= most; ++sp) {
        cands[n] = {{i, sp, false}, predict_us(plan, ke, rows, sp, which == 0 && rows < plan->geo.m)};
        best_pred = std::min(best_pred, cands[n++].predicted);
      }
      if (can_mask && plan->masked_store != 1) {
        cands[n] = {{i, 1, true}, predict_us(plan, ke, plan->geo.m, 1, false) + 0.1};
        best_pred = std::min(best_pred, cands[n++].predicted);
      }
    }
    for (int c = 0; c < n; ++c) {
      if (cands[c].predicted > 1.6 * best_pred) continue;
      plan->pick[which] = cands[c].pick;
      plan->prefer_tiled[which] = true;
      const double us = time_us(dense, 40, 3);
      if (us > 0.0 && us < 0.985 * best_us) { best_us = us; best_pick = cands[c].pick; best_tiled = true; }
    }
    plan->pick[which] = best_pick;
    plan->prefer_tiled[which] = best_tiled;
    // the slab form of the tiled kernel (deep 3x3 layers): both tile heights, the K splits around one workgroup per
    // compute unit; it replaces the choice so far only where it measures faster
    plan->slab_auto[which] = sc_plan::Slab{0, 1};
    const BandPlan& bsel = dense ? plan->band_dense : plan->band;
    if (plan->slab_ok && plan->slab == 0 && plan->split_k == 0 && !(bsel.ok && !bsel.stream && !best_tiled)) {
      sc_plan::Slab best_slab = {0, 1};
      for (int bm = 256; bm >= 128; bm >>= 1) {
        if (!slab_buffer_bytes(plan->desc, bm, plan->slab_span[which][bm == 256])) continue;
        const int around = slab_splits(plan, bm, rows);
        int tried[4] = {0, 0, 0, 0}, n_tried = 0;
        for (int sp : {around, around - 1, around + 1, 1}) {
          if (sp < 1 || sp > plan->desc.c_in / kSlabCh || (sp > 1 && !plan->geo.splitk_ok)) continue;
          if ((int64_t)((rows + bm - 1) / bm) * ((plan->desc.c_out + kSlabBN - 1) / kSlabBN) * sp * bm * kSlabBN * 4 > (int64_t)kSplitKPartialBytes) continue;
          bool seen = false;
          for (int i = 0; i < n_tried; ++i) seen = seen || tried[i] == sp;
          if (seen) continue;
          tried[n_tried++] = sp;
          plan->slab_auto[which] = {bm, sp};
          const double us = time_us(dense, 40, 3);
          if (us > 0.0 && us < 0.985 * best_us) { best_us = us; best_slab = {bm, sp}; }
        }
      }
      plan->slab_auto[which] = best_slab;
    }
  }
  // A sparse run must not lose to the dense run of its own plan: where it still does, try the dense run's tile with
  // every row contracted and the mask applied at the store.
  if (result == SC_OK && plan->forced[0] == -1 && plan->forced[1] == -1 && plan->kept > 0 && plan->kept < plan->geo.m &&
      plan->masked_store != 1 && plan->geo.vec_gather && !plan->geo.rowseg && plan->desc.layout == SC_NHWC) {
    const double us_sparse = time_us(false, 40, 3), us_dense = time_us(true, 40, 3);
    // (where the dense run takes a band or row-panel kernel, the tile is the one the dense run would take as a tiled launch)
    if (us_sparse > 0.0 && us_dense > 0.0 && us_sparse > us_dense) {
      const sc_plan::Pick keep = plan->pick[0];
      const bool keep_tiled = plan->prefer_tiled[0];
      const sc_plan::Slab keep_slab = plan->slab_auto[0];
      plan->pick[0] = {plan->pick[1].ti, 1, true};
      plan->prefer_tiled[0] = true;
      plan->slab_auto[0] = sc_plan::Slab{0, 1};
      const double us = time_us(false, 40, 3);
      if (!(us > 0.0 && us < us_sparse)) { plan->pick[0] = keep; plan->prefer_tiled[0] = keep_tiled; plan->slab_auto[0] = keep_slab; }
    }
  }
  plan->tuned = result == SC_OK;
  if (hip_failed(hipStreamSynchronize(ts)) && result == SC_OK) result = SC_ERR_HIP;
  if (result == SC_OK) result = launch_conv(plan, false, x_dev, bias_dev, y_dev, stream);   // y = the masked convolution
  if (hip_failed(hipStreamSynchronize(stream)) && result == SC_OK) result = SC_ERR_HIP;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  (void)hipStreamDestroy(ts);
  return result;
}

sc_status sparse_conv_plan_info(const sc_plan* plan, int64_t* m, int64_t* kept, int32_t* ho, int32_t* wo,
                                const int32_t** row_idx_dev) {
  if (!plan) return SC_ERR_NULL;
  if (m) *m = plan->geo.m;
  if (kept) *kept = plan->kept;
  if (ho) *ho = plan->geo.ho;
  if (wo) *wo = plan->geo.wo;
  if (row_idx_dev) *row_idx_dev = reinterpret_cast<const int32_t*>(plan->ws + plan->geo.off_rows);
  return SC_OK;
}

const uint8_t* sparse_conv_plan_mask(const sc_plan* plan) {
  return plan ? plan->ws + plan->geo.off_mask : nullptr;
}

sc_status sparse_conv_plan_tiles(const sc_plan* plan, int32_t which, int32_t* tile_m, int32_t* tile_n,
                                 int64_t* workgroups) {
  if (!plan) return SC_ERR_NULL;
  if (which != 0 && which != 1) return SC_ERR_UNSUPPORTED;
  if (plan->geo.depthwise) {   // one lane per pixel and 16-byte channel group, 256 lanes per workgroup
    const int eb = elem_bytes(plan->desc.dtype);
    const int v = plan->desc.c_in % (16 / eb) == 0 ? 16 / eb : 1;
    const bool walk_dense = which == 1 || plan->desc.out_mode == SC_OUT_ZERO_FILL;
    if (tile_m) *tile_m = 1;
    if (tile_n) *tile_n = v;
    if (workgroups) *workgroups = ((walk_dense ? plan->geo.m : plan->kept) * (plan->desc.c_in / v) + 255) / 256;
    return SC_OK;
  }
  const BandPlan& band = which ? plan->band_dense : plan->band;
  if (band.ok && (plan->forced[which] == kForceBand || (plan->forced[which] == -1 && !band.stream && !plan->prefer_tiled[which])) &&
      !(plan->slab >= 2 && slab_pick(plan, which, which ? plan->geo.m : plan->kept).bm)) {
    if (tile_m) *tile_m = -band.bh;     // (rows per run; split bands hold half a run each)
    if (tile_n) *tile_n = 32 * band.ni;
    if (workgroups) *workgroups = band.pp && !band.tap ? band.pp_grid : (int64_t)band.n_bands * band.n_tiles;
    return SC_OK;
  }
  int64_t rows = which ? plan->geo.m : plan->kept;
  if (const sc_plan::Slab sl = slab_pick(plan, which, rows); sl.bm) {
    if (tile_m) *tile_m = sl.bm;
    if (tile_n) *tile_n = kSlabBN;
    if (workgroups) *workgroups = ((rows + sl.bm - 1) / sl.bm) * ((plan->desc.c_out + kSlabBN - 1) / kSlabBN) * std::min(sl.splits, plan->desc.c_in / kSlabCh);
    return SC_OK;
  }
  if (use_panel(plan, which, rows)) {
    if (tile_m) *tile_m = kPanelBM;
    if (tile_n) *tile_n = kPanelBN;
    if (workgroups) *workgroups = (rows + kPanelBM - 1) / kPanelBM;
    return SC_OK;
  }
  const TilePick tp = pick_tile(plan, which, rows);
  const int splits = tp.masked ? 1 : tp.splits;
  if (tp.masked && which == 0) rows = plan->geo.m;
  const KernelEntry& ke = plan->table[tp.ti];
  if (tile_m) *tile_m = ke.bm;
  if (tile_n) *tile_n = ke.bn;
  if (workgroups) *workgroups = ((rows + ke.bm - 1) / ke.bm) * ((plan->desc.c_out + ke.bn - 1) / ke.bn) * splits;
  const int sk = splits == 1 ? stream_k_workgroups(plan, ke, rows) : 0;
  if (sk && workgroups) *workgroups = sk;      // persistent workgroups of a stream-K launch
  return SC_OK;
}

// name of the tiled kernel a launch of this plan takes when no band or row-panel kernel applies
static const char* tiled_kernel_name(const sc_plan* plan, int32_t which) {
  const Geometry& g = plan->geo;
  const TilePick tp = pick_tile(plan, which, which ? g.m : plan->kept);
  if (tp.masked) return "tile_masked_store";
  if (tp.splits > 1) return "tile_split_k";
  if (stream_k_workgroups(plan, plan->table[tp.ti], which ? g.m : plan->kept)) return "tile_stream_k";
  if (g.rowseg) return "tile_row_segments";
  if (!g.vec_gather) return "tile_elements";
  return (g.vec_out && plan->gather_pipeline != 1) ? "tile_lds_direct" : "tile_registers";
}

const char* sparse_conv_plan_kernel(const sc_plan* plan, int32_t which) {
  if (!plan || (which != 0 && which != 1)) return nullptr;
  if (plan->geo.depthwise) return "depthwise";
  const BandPlan& band = which ? plan->band_dense : plan->band;
  if (band.ok && (plan->forced[which] == kForceBand || (plan->forced[which] == -1 && !band.stream && !plan->prefer_tiled[which])) &&
      !(plan->slab >= 2 && slab_pick(plan, which, which ? plan->geo.m : plan->kept).bm))
    return band.rowband ? "band_row_segments" : band.stream ? "band_stream" : band.tap ? "band_tap" : band.pp ? "band_alternating" : "band";
  const Geometry& g = plan->geo;
  if (slab_pick(plan, which, which ? g.m : plan->kept).bm) return "tile_slab";
  if (use_panel(plan, which, which ? g.m : plan->kept)) return "tile_row_panel";
  return tiled_kernel_name(plan, which);
}

const char* sparse_conv_plan_fused_kernel(const sc_plan* plan, int32_t which) {
  if (!plan || (which != 0 && which != 1) || plan->geo.depthwise) return nullptr;
  const BandPlan& band = which ? plan->band_dense : plan->band;
  if (band.ok && (band.pp || band.tap) && !band.stream &&
      (plan->forced[which] == kForceBand || (plan->forced[which] == -1 && !plan->prefer_tiled[which])) &&
      !(plan->slab >= 2 && slab_pick(plan, which, which ? plan->geo.m : plan->kept).bm))
    return band.tap ? "band_tap" : "band_alternating";
  if (slab_pick(plan, which, which ? plan->geo.m : plan->kept).bm) return "tile_slab";
  return tiled_kernel_name(plan, which);
}

sc_status sparse_conv_plan_set_tiles(sc_plan* plan, int32_t which, int32_t tile_m, int32_t tile_n) {
  if (!plan) return SC_ERR_NULL;
  if (which != 0 && which != 1) return SC_ERR_UNSUPPORTED;
  if (tile_m == 0 && tile_n == 0) { plan->forced[which] = -1; return SC_OK; }
  if (plan->geo.depthwise) return SC_ERR_UNSUPPORTED;   // one kernel, no tiles to choose
  if (tile_m < 0) {
    if (!(which ? plan->band_dense : plan->band).ok) return SC_ERR_UNSUPPORTED;
    plan->forced[which] = kForceBand;
    return SC_OK;
  }
  for (int i = 0; i < plan->table_count; ++i)
    if (plan->table[i].bm == tile_m && plan->table[i].bn == tile_n) { plan->forced[which] = i; return SC_OK; }
  return SC_ERR_UNSUPPORTED;
}

sc_status sparse_conv_plan_set_option(sc_plan* plan, int32_t option, int32_t value) {
  if (!plan) return SC_ERR_NULL;
  if (option == SC_OPT_GATHER_PIPELINE && value >= 0 && value <= 2) { plan->gather_pipeline = value; return SC_OK; }
  if (option == SC_OPT_ROW_PANEL && value >= 0 && value <= 2) { plan->row_panel = value; return SC_OK; }
  if (option == SC_OPT_SPLIT_K && value >= 0 && value <= kSplitKMost) { plan->split_k = value; return SC_OK; }
  if (option == SC_OPT_STREAM_K && value >= 0 && value <= kStreamKMostWgs) { plan->stream_k = value; return SC_OK; }
  if (option == SC_OPT_MASKED_STORE && value >= 0 && value <= 2) { plan->masked_store = value; return SC_OK; }
  if (option == SC_OPT_SLAB && ((value >= 0 && value <= 2) || value == 128 || value == 256)) { plan->slab = value; return SC_OK; }
  return SC_ERR_UNSUPPORTED;
}

void sparse_conv_plan_destroy(sc_plan* plan) { delete plan; }

const char* sc_status_string(sc_status s) {
  switch (s) {
    case SC_OK: return "ok";
    case SC_ERR_NULL: return "a required pointer is NULL";
    case SC_ERR_BAD_SHAPE: return "bad shape (non-positive extent, empty output or tensor too large)";
    case SC_ERR_UNSUPPORTED: return "unsupported (groups other than 1 or depthwise NHWC, or unknown dtype/layout/mode/tile/format)";
    case SC_ERR_MASK_COUNT: return "mask popcount differs from the count the sparsity ratio demands";
    case SC_ERR_WORKSPACE: return "workspace too small";
    case SC_ERR_ALIGN: return "device pointer not sufficiently aligned";
    case SC_ERR_HIP: return "a HIP call failed (see sc_last_hip_error)";
  }
  return "unknown status";
}

int32_t sc_last_hip_error(void) { return sc::g_last_hip; }

#ifdef SC_TIMING
void sc_debug_set_buffer(void* p) { sc::g_dbg = static_cast<long long*>(p); }
#endif

sc_status sc_maxpool2d_nhwc(const void* x_dev, void* y_dev, int32_t dtype, int32_t n, int32_t h, int32_t w,
                            int32_t c, int32_t k, int32_t s, int32_t p, void* hip_stream) {
  if (!x_dev || !y_dev) return SC_ERR_NULL;
  if (dtype != SC_F32 && dtype != SC_F16 && dtype != SC_BF16) return SC_ERR_UNSUPPORTED;
  if (n < 1 || h < 1 || w < 1 || c < 1 || k < 1 || s < 1 || p < 0 || 2 * p > k) return SC_ERR_BAD_SHAPE;
  int ho = out_extent(h, k, s, p, 1), wo = out_extent(w, k, s, p, 1);
  if (ho < 1 || wo < 1) return SC_ERR_BAD_SHAPE;
  int64_t total = (int64_t)n * ho * wo * c;
  if (total >= ((int64_t)1 << 31) * 256) return SC_ERR_BAD_SHAPE;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  dim3 grid((unsigned)((total + 255) / 256)), block(256);
  const bool vec8 = dtype != SC_F32 && c % 8 == 0 && (((uintptr_t)x_dev | (uintptr_t)y_dev) & 15) == 0;
  if (vec8 && k == 3 && total / 8 < ((int64_t)1 << 31)) {
    dim3 vgrid((unsigned)((total / 8 + 255) / 256));
    uint32_t cm, cs, wm, ws_, hm, hs;
    sc::magic_div((uint32_t)(c / 8), &cm, &cs);
    sc::magic_div((uint32_t)wo, &wm, &ws_);
    sc::magic_div((uint32_t)ho, &hm, &hs);
    if (dtype == SC_F16)
      hipLaunchKernelGGL(maxpool3_nhwc_vec8_kernel<_Float16>, vgrid, block, 0, stream, (const _Float16*)x_dev,
                         (_Float16*)y_dev, n, h, w, c, s, p, ho, wo, cm, cs, wm, ws_, hm, hs);
    else
      hipLaunchKernelGGL(maxpool3_nhwc_vec8_kernel<__bf16>, vgrid, block, 0, stream, (const __bf16*)x_dev,
                         (__bf16*)y_dev, n, h, w, c, s, p, ho, wo, cm, cs, wm, ws_, hm, hs);
  } else if (vec8) {
    dim3 vgrid((unsigned)((total / 8 + 255) / 256));
    if (dtype == SC_F16)
      hipLaunchKernelGGL(maxpool_nhwc_vec8_kernel<_Float16>, vgrid, block, 0, stream, (const _Float16*)x_dev,
                         (_Float16*)y_dev, n, h, w, c, k, s, p, ho, wo);
    else
      hipLaunchKernelGGL(maxpool_nhwc_vec8_kernel<__bf16>, vgrid, block, 0, stream, (const __bf16*)x_dev,
                         (__bf16*)y_dev, n, h, w, c, k, s, p, ho, wo);
  } else if (dtype == SC_F32)
    hipLaunchKernelGGL(maxpool_nhwc_kernel<float>, grid, block, 0, stream, (const float*)x_dev, (float*)y_dev, n, h,
                       w, c, k, s, p, ho, wo);
  else if (dtype == SC_F16)
    hipLaunchKernelGGL(maxpool_nhwc_kernel<_Float16>, grid, block, 0, stream, (const _Float16*)x_dev,
                       (_Float16*)y_dev, n, h, w, c, k, s, p, ho, wo);
  else
    hipLaunchKernelGGL(maxpool_nhwc_kernel<__bf16>, grid, block, 0, stream, (const __bf16*)x_dev, (__bf16*)y_dev, n,
                       h, w, c, k, s, p, ho, wo);
  SC_HIP(hipGetLastError());
  return SC_OK;
}

}  // extern "C"

template <bool RELU>
static sc_status add_launch(const void* a_dev, const void* b_dev, void* y_dev, int32_t dtype, int64_t count,
                            void* hip_stream) {
  if (!a_dev || !b_dev || !y_dev) return SC_ERR_NULL;
  if (dtype != SC_F32 && dtype != SC_F16 && dtype != SC_BF16) return SC_ERR_UNSUPPORTED;
  if (count < 0) return SC_ERR_BAD_SHAPE;
  if (count == 0) return SC_OK;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  dim3 grid((unsigned)std::min<int64_t>((count + 255) / 256, 65536)), block(256);
  const bool vec8 = dtype != SC_F32 && count % 8 == 0 &&
                    (((uintptr_t)a_dev | (uintptr_t)b_dev | (uintptr_t)y_dev) & 15) == 0;
  if (vec8) {
    dim3 vgrid((unsigned)std::min<int64_t>((count / 8 + 255) / 256, 65536));
    if (dtype == SC_F16)
      hipLaunchKernelGGL((add_vec8_kernel<_Float16, RELU>), vgrid, block, 0, stream, (const _Float16*)a_dev,
                         (const _Float16*)b_dev, (_Float16*)y_dev, count / 8);
    else
      hipLaunchKernelGGL((add_vec8_kernel<__bf16, RELU>), vgrid, block, 0, stream, (const __bf16*)a_dev,
                         (const __bf16*)b_dev, (__bf16*)y_dev, count / 8);
  } else if (dtype == SC_F32)
    hipLaunchKernelGGL((add_kernel<float, RELU>), grid, block, 0, stream, (const float*)a_dev, (const float*)b_dev,
                       (float*)y_dev, count);
  else if (dtype == SC_F16)
    hipLaunchKernelGGL((add_kernel<_Float16, RELU>), grid, block, 0, stream, (const _Float16*)a_dev,
                       (const _Float16*)b_dev, (_Float16*)y_dev, count);
  else
    hipLaunchKernelGGL((add_kernel<__bf16, RELU>), grid, block, 0, stream, (const __bf16*)a_dev, (const __bf16*)b_dev,
                       (__bf16*)y_dev, count);
  SC_HIP(hipGetLastError());
  return SC_OK;
}

extern "C" {

sc_status sc_add_relu(const void* a_dev, const void* b_dev, void* y_dev, int32_t dtype, int64_t count,
                      void* hip_stream) {
  return add_launch<true>(a_dev, b_dev, y_dev, dtype, count, hip_stream);
}

sc_status sc_add(const void* a_dev, const void* b_dev, void* y_dev, int32_t dtype, int64_t count, void* hip_stream) {
  return add_launch<false>(a_dev, b_dev, y_dev, dtype, count, hip_stream);
}

}  // extern "C"
