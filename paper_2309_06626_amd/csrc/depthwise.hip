// Masked depthwise convolution (groups == Cin == Cout, NHWC): every channel is filtered by its own
// kh x kw window and the mask removes output pixels exactly as for ordinary layers (Sec. 3: a dropped
// pixel is dropped in all channels; Alg. 2: its output is zero).  There is no contraction over channels,
// so nothing here is GEMM-shaped: the layer moves each input and output byte once and is bound by HBM.
//
//   lane      = one output pixel x one 16-byte group of channels (8 for the 16-bit types, 4 for float)
//               -- or one channel when the channel count is not a multiple of the group;
//               consecutive lanes take consecutive channel groups of a pixel, so every load and store
//               of a wavefront covers contiguous memory
//   items     = the dense rows (zero-fill mode: a lane whose pixel is dropped stores zeros) or the kept
//               rows through the row list (scatter-only and compact output: dropped pixels cost nothing)
//   filters   = repacked at plan time to [kh*kw][C], so the lanes of a pixel read contiguous filter
//               entries for each tap; they stay in L1/L2 (kh*kw*C entries in all)
#include "conv_params.hpp"
#include "mma_common.hpp"

namespace sc {

template <typename T> struct DwVec;
template <> struct DwVec<float> { static constexpr int V = 4; };
template <> struct DwVec<_Float16> { static constexpr int V = 8; };
template <> struct DwVec<__bf16> { static constexpr int V = 8; };

template <typename T, int V>
struct alignas(sizeof(T) * V) DwGroup { T v[V]; };

// filters [C][kh*kw] (the caller's layout, one input channel per group) -> [kh*kw][C]
template <typename T>
__global__ void depthwise_pack_kernel(const T* __restrict__ w, T* __restrict__ wp, int c, int taps) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= c * taps) return;
  const int tap = i / c, ch = i - tap * c;
  wp[i] = w[(size_t)ch * taps + tap];
}

template <typename T, int V>
__global__ __launch_bounds__(256) void depthwise_kernel(const DepthwiseParams p) {
  using G = DwGroup<T, V>;
  const int groups = p.c / V;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t item = idx / groups;
  if (item >= p.items) return;
  const int c0 = (int)(idx - item * groups) * V;
  // dense position of the item, and where its result goes
  const int r = p.row_idx ? p.row_idx[item] : (int)item;
  const int64_t out_row = p.y_compact ? item : (int64_t)r;
  T* __restrict__ y = static_cast<T*>(p.y) + out_row * p.c + c0;
  const int n = fast_div(r, p.div_howo_mul, p.div_howo_shift), rem = r - n * p.ho_wo;
  if (p.mask) {   // zero-fill mode walks every dense row: Alg. 2, mask == 0 branch
    if (p.mask[p.mask_spatial ? rem : r] == 0) {
      G z;
#pragma unroll
      for (int j = 0; j < V; ++j) z.v[j] = (T)0.0f;
      *reinterpret_cast<G*>(y) = z;
      return;
    }
  }
  const int oy = fast_div(rem, p.div_wo_mul, p.div_wo_shift), ox = rem - oy * p.wo;
  const int iy0 = oy * p.sh - p.ph, ix0 = ox * p.sw - p.pw;
  // a compact input (1x1 windows only: the window is the pixel itself) holds pixel r in row `item`
  const T* __restrict__ x = p.x_compact
                                ? static_cast<const T*>(p.x) + (item - ((int64_t)iy0 * p.w + ix0)) * p.c + c0
                                : static_cast<const T*>(p.x) + (int64_t)n * p.h * p.w * p.c + c0;
  const T* __restrict__ wp = static_cast<const T*>(p.wp) + c0;
  float acc[V];
#pragma unroll
  for (int j = 0; j < V; ++j) acc[j] = 0.0f;
  for (int ky = 0; ky < p.kh; ++ky) {
    const int iy = iy0 + ky * p.dil_h;
    if ((unsigned)iy >= (unsigned)p.h) continue;
    for (int kx = 0; kx < p.kw; ++kx) {
      const int ix = ix0 + kx * p.dil_w;
      if ((unsigned)ix >= (unsigned)p.w) continue;
      const G xv = *reinterpret_cast<const G*>(x + ((int64_t)iy * p.w + ix) * p.c);
      const G wv = *reinterpret_cast<const G*>(wp + (int64_t)(ky * p.kw + kx) * p.c);
#pragma unroll
      for (int j = 0; j < V; ++j) acc[j] += (float)xv.v[j] * (float)wv.v[j];
    }
  }
  G out;
#pragma unroll
  for (int j = 0; j < V; ++j) {
    float v = acc[j] + (p.bias ? p.bias[c0 + j] : 0.0f);
    if (p.relu) v = v > 0.0f ? v : 0.0f;
    out.v[j] = (T)v;
  }
  *reinterpret_cast<G*>(y) = out;
}

template <typename T>
static hipError_t launch_typed(const DepthwiseParams& p, hipStream_t stream) {
  constexpr int V = DwVec<T>::V;
  const bool vec = p.c % V == 0;
  const int64_t threads = p.items * (vec ? p.c / V : p.c);
  const unsigned grid = (unsigned)((threads + 255) / 256);
  if (vec)
    hipLaunchKernelGGL((depthwise_kernel<T, V>), dim3(grid), dim3(256), 0, stream, p);
  else
    hipLaunchKernelGGL((depthwise_kernel<T, 1>), dim3(grid), dim3(256), 0, stream, p);
  return hipGetLastError();
}

hipError_t depthwise_launch(int dtype, const DepthwiseParams& p, hipStream_t stream) {
  if (p.items <= 0) return hipSuccess;
  if (dtype == kF32) return launch_typed<float>(p, stream);
  if (dtype == kF16) return launch_typed<_Float16>(p, stream);
  return launch_typed<__bf16>(p, stream);
}

hipError_t depthwise_pack(int dtype, const void* w, void* wp, int c, int taps, hipStream_t stream) {
  const unsigned grid = (unsigned)(((int64_t)c * taps + 255) / 256);
  if (dtype == kF32)
    hipLaunchKernelGGL(depthwise_pack_kernel<float>, dim3(grid), dim3(256), 0, stream, (const float*)w, (float*)wp, c, taps);
  else   // 16-bit patterns are moved verbatim
    hipLaunchKernelGGL(depthwise_pack_kernel<_Float16>, dim3(grid), dim3(256), 0, stream, (const _Float16*)w,
                       (_Float16*)wp, c, taps);
  return hipGetLastError();
}

}  // namespace sc
