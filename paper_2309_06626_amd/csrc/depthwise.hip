// Masked depthwise convolution (groups == Cin == Cout, NHWC): every channel is filtered by its own
// kh x kw window and the mask removes output pixels exactly as for ordinary layers (Sec. 3: a dropped
// pixel is dropped in all channels; Alg. 2: its output is zero).  There is no contraction over channels,
// so nothing here is GEMM-shaped.  Three kernels: a general one (below), an LDS-tiled one for 3x3 windows
// (float), and its two-term-dot-product form for the 16-bit types.
//
// General kernel:
//   lane      = one output pixel x one 16-byte group of channels (8 for the 16-bit types, 4 for float)
//               -- or one channel when the channel count is not a multiple of the group;
//               consecutive lanes take consecutive channel groups of a pixel, so every load and store
//               of a wavefront covers contiguous memory
//   items     = the dense rows (zero-fill mode: a lane whose pixel is dropped stores zeros) or the kept
//               rows through the row list (scatter-only and compact output: dropped pixels cost nothing)
//   filters   = repacked at plan time to [kh*kw][C], so the lanes of a pixel read contiguous filter
//               entries for each tap; they stay in L1/L2 (kh*kw*C entries in all)
#include <algorithm>

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
  if (p.mask && !p.row_idx) {   // zero-fill mode walks every dense row: Alg. 2, mask == 0 branch
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
  // a compact input without a rank map (1x1 windows only: the window is the pixel itself) holds pixel r in
  // row `item`; with a rank map every tap looks its pixel up
  const bool ranked = p.x_compact && p.x_rank;
  const T* __restrict__ x = ranked ? static_cast<const T*>(p.x) + c0
                            : p.x_compact
                                ? static_cast<const T*>(p.x) + (item - ((int64_t)iy0 * p.w + ix0)) * p.c + c0
                                : static_cast<const T*>(p.x) + (int64_t)n * p.h * p.w * p.c + c0;
  const int32_t* __restrict__ xr = ranked ? p.x_rank + (int64_t)n * p.h * p.w : nullptr;
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
      int64_t pix = (int64_t)iy * p.w + ix;
      if (ranked) {
        pix = xr[pix];
        if (pix < 0) continue;            // dropped by the producer: +0.0
      }
      const G xv = *reinterpret_cast<const G*>(x + pix * p.c);
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

// 3x3 windows without dilation, stride S in both directions, 16-byte channel groups.  A workgroup owns a
// tile of TY x TX output pixels of one image and a chunk of CG channel groups.  It stages the input
// patch of the tile -- ((TY-1)*S+3) x ((TX-1)*S+3) pixels x CG groups, zeros outside the image -- in LDS
// with coalesced 16-byte loads (consecutive lanes: consecutive channel groups, then consecutive
// pixels), so every input byte is fetched from memory once per tile instead of once per window that
// contains it.  Then lane t keeps channel group t % CG (its nine filter groups stay in registers, as
// floats) and walks pairs of horizontally adjacent pixels of the tile: the kernel is bound by vector
// instructions (nine multiply-adds and, for the 16-bit types, up to nine conversions per output
// element), and a pair shares the conversions of the window columns its two pixels have in common.
// The mask bytes of the tile are staged in LDS as well; a pair with no kept pixel costs only its zeros.
struct DwTile {
  int32_t ty, tx, tiles_y, tiles_x;   // output tile, tiles per image
  int32_t txp;                        // tile width rounded up to an even number of columns
  int32_t cg, chunks;                 // channel groups per workgroup, chunks per pixel
  int32_t in_h, in_w;                 // input patch
  uint32_t div_cg_mul, div_cg_shift, div_inw_mul, div_inw_shift, div_txp_mul, div_txp_shift, div_pairs_mul, div_pairs_shift;
};

template <typename T, int V, int S>
__global__ __launch_bounds__(256) void depthwise3x3_kernel(const DepthwiseParams p, const DwTile q) {
  using G = DwGroup<T, V>;
  extern __shared__ __align__(16) unsigned char smem[];
  G* s_x = reinterpret_cast<G*>(smem);
  unsigned char* s_keep = smem + (size_t)q.in_h * q.in_w * q.cg * sizeof(G);

  const int t = threadIdx.x;
  int b = blockIdx.x;
  const int chunk = b % q.chunks; b /= q.chunks;
  const int tile_x = b % q.tiles_x; b /= q.tiles_x;
  const int tile_y = b % q.tiles_y;
  const int n = b / q.tiles_y;
  const int oy0 = tile_y * q.ty, ox0 = tile_x * q.tx;
  const int groups = p.c / V;
  const int g0 = chunk * q.cg;                       // first channel group of the chunk
  const int iy_first = oy0 * S - p.ph, ix_first = ox0 * S - p.pw;

  // ---- stage the input patch and the tile's mask bytes ---------------------------------------------
  const T* __restrict__ x = static_cast<const T*>(p.x) + (int64_t)n * p.h * p.w * p.c;
  const int elems = q.in_h * q.in_w * q.cg;
  constexpr int U = 4;
  for (int e0 = 0; e0 < elems; e0 += U * 256) {
    G v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int e = e0 + u * 256 + t;
      const int pix = fast_div(e, q.div_cg_mul, q.div_cg_shift), g = e - pix * q.cg;
      const int py = fast_div(pix, q.div_inw_mul, q.div_inw_shift), px = pix - py * q.in_w;
      const int iy = iy_first + py, ix = ix_first + px;
#pragma unroll
      for (int k = 0; k < V; ++k) v[u].v[k] = (T)0.0f;
      if (e < elems && (unsigned)iy < (unsigned)p.h && (unsigned)ix < (unsigned)p.w && g0 + g < groups)
        v[u] = *reinterpret_cast<const G*>(x + ((int64_t)iy * p.w + ix) * p.c + (g0 + g) * V);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int e = e0 + u * 256 + t;
      if (e < elems) s_x[e] = v[u];
    }
  }
  // mask bytes of the tile, padded to an even number of columns: 1 = kept, 2 = dropped, 0 = outside the map
  const int tile_pixels = q.ty * q.txp;
  for (int pix = t; pix < tile_pixels; pix += 256) {
    const int ty = fast_div(pix, q.div_txp_mul, q.div_txp_shift), tx = pix - ty * q.txp;
    const int oy = oy0 + ty, ox = ox0 + tx;
    unsigned char k = 0;
    if (tx < q.tx && oy < p.ho && ox < p.wo)
      k = p.mask ? (p.mask[(p.mask_spatial ? 0 : n * p.ho_wo) + oy * p.wo + ox] ? 1 : 2) : 1;
    s_keep[pix] = k;
  }

  // ---- this lane's channel group: filters and bias -----------------------------------------------------
  const int g = t % q.cg, slot = t / q.cg, per_pass = 256 / q.cg;
  const bool lane_on = slot < per_pass && g0 + g < groups;
  const int c0 = (g0 + (lane_on ? g : 0)) * V;
  float wf[9][V];
  const T* __restrict__ wp = static_cast<const T*>(p.wp) + c0;
#pragma unroll
  for (int tap = 0; tap < 9; ++tap) {
    const G wv = *reinterpret_cast<const G*>(wp + (int64_t)tap * p.c);
#pragma unroll
    for (int k = 0; k < V; ++k) wf[tap][k] = (float)wv.v[k];
  }
  float bias_v[V];
#pragma unroll
  for (int k = 0; k < V; ++k) bias_v[k] = p.bias ? p.bias[c0 + k] : 0.0f;
  const float floor_v = p.relu ? 0.0f : -__builtin_inff();      // max(f, floor) is the activation
  T* __restrict__ y = static_cast<T*>(p.y) + c0;
  __syncthreads();
  if (!lane_on) return;

  // Two horizontally adjacent output pixels per step: their windows share two of three columns, so
  // 3 x (2 + S) groups are read and converted for 18 taps' worth of multiply-adds.
  const int pairs_per_row = q.txp >> 1, tile_pairs = q.ty * pairs_per_row;
  for (int pp = slot; pp < tile_pairs; pp += per_pass) {
    const int ty = fast_div(pp, q.div_pairs_mul, q.div_pairs_shift), tx = (pp - ty * pairs_per_row) * 2;
    const unsigned k0 = s_keep[ty * q.txp + tx], k1 = s_keep[ty * q.txp + tx + 1];
    if ((k0 | k1) == 0) continue;
    const int r = n * p.ho_wo + (oy0 + ty) * p.wo + ox0 + tx;
    G o0, o1;
#pragma unroll
    for (int j = 0; j < V; ++j) { o0.v[j] = (T)0.0f; o1.v[j] = (T)0.0f; }      // Alg. 2, mask == 0 branch: zeros
    if (k0 == 1 || k1 == 1) {
      const G* win = s_x + ((ty * S) * q.in_w + tx * S) * q.cg + g;
      float a0[V], a1[V];
#pragma unroll
      for (int j = 0; j < V; ++j) { a0[j] = bias_v[j]; a1[j] = bias_v[j]; }
#pragma unroll
      for (int ky = 0; ky < 3; ++ky) {
#pragma unroll
        for (int col = 0; col < 3 + S; ++col) {
          const G xv = win[(ky * q.in_w + col) * q.cg];
          float xf[V];
#pragma unroll
          for (int j = 0; j < V; ++j) xf[j] = (float)xv.v[j];
          if (col < 3) {
#pragma unroll
            for (int j = 0; j < V; ++j) a0[j] += xf[j] * wf[ky * 3 + col][j];
          }
          if (col >= S) {
#pragma unroll
            for (int j = 0; j < V; ++j) a1[j] += xf[j] * wf[ky * 3 + col - S][j];
          }
        }
      }
#pragma unroll
      for (int j = 0; j < V; ++j) {
        if (k0 == 1) o0.v[j] = (T)__builtin_fmaxf(a0[j], floor_v);
        if (k1 == 1) o1.v[j] = (T)__builtin_fmaxf(a1[j], floor_v);
      }
    }
    if (k0 == 1) *reinterpret_cast<G*>(y + (p.rank ? (int64_t)p.rank[r] : (int64_t)r) * p.c) = o0;
    else if (k0 == 2 && p.zero_fill) *reinterpret_cast<G*>(y + (int64_t)r * p.c) = o0;
    if (k1 == 1) *reinterpret_cast<G*>(y + (p.rank ? (int64_t)p.rank[r + 1] : (int64_t)(r + 1)) * p.c) = o1;
    else if (k1 == 2 && p.zero_fill) *reinterpret_cast<G*>(y + (int64_t)(r + 1) * p.c) = o1;
  }
}

// ---- 16-bit types: the same tiling with two-term dot products ---------------------------------------
// The tiled kernel above is bound by vector instructions, and for a 16-bit type half of them only widen
// operands.  v_dot2c_f32_{bf16,f16} multiplies two pairs of 16-bit values and adds both products to a
// float accumulator, without a conversion.  The pairs have to lie along the sum, i.e. along the window:
// so the patch is staged with its rows interleaved two by two -- one dword holds channel c of patch rows
// 2i and 2i+1 at one pixel -- and the filter registers hold the matching pairs of window rows:
//   stride 1, output rows 2j and 2j+1 (window rows 2j..2j+2 and 2j+1..2j+3), row pairs P_j and P_j+1:
//     out[2j]   = P_j . (w0, w1) + P_j+1 . (w2, 0)        out[2j+1] = P_j . (0, w0) + P_j+1 . (w1, w2)
//   stride 2, output row t (window rows 2t..2t+2):  out[t] = P_t . (w0, w1) + P_t+1 . (w2, 0)
// per window column: six instead of nine multiply-add instructions per output element, and no widening.
// LDS holds the interleaved groups in two planes (channels 0..3 and 4..7 of a group, 16 bytes each) so
// that consecutive lanes read consecutive 16-byte words.
typedef __bf16 dw_bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 dw_f16x2 __attribute__((ext_vector_type(2)));
template <typename T> struct Dot2;
template <> struct Dot2<__bf16> {
  static __device__ __forceinline__ float run(unsigned a, unsigned b, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(dw_bf16x2, a), __builtin_bit_cast(dw_bf16x2, b), c, false);
  }
};
template <> struct Dot2<_Float16> {
  static __device__ __forceinline__ float run(unsigned a, unsigned b, float c) {
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(dw_f16x2, a), __builtin_bit_cast(dw_f16x2, b), c, false);
  }
};

// The workgroups are persistent: workgroup b of chunk c walks the tiles b, b + gridDim.x, ... of that
// chunk.  The loads of the next tile's patch are issued (into registers) before the current tile is
// computed and written to LDS after it, so their latency hides behind the dot products and the stores.
constexpr int kDwStageMost = 4;       // patch words a lane stages per tile: the patch has at most 4 * 256 of them

struct DwPairTile {
  int32_t ty, tx, tiles_y, tiles_x;   // output tile (ty even for stride 1), tiles per image
  int32_t cg;                         // channel groups per workgroup (blockIdx.y = chunk of the pixel)
  int32_t pairs_h, in_w;              // patch: row pairs and columns
  int32_t tiles;                      // tiles per chunk: n * tiles_y * tiles_x
  uint32_t div_cg_mul, div_cg_shift, div_inw_mul, div_inw_shift, div_tx_mul, div_tx_shift;
  uint32_t div_tilesx_mul, div_tilesx_shift, div_tilesy_mul, div_tilesy_shift;
};

// XC: the input is compact; p.x_rank maps every input pixel to its row (or -1).  The ranks of a tile's patch
// are requested one tile before its data, so that the data requests never wait for them.
template <typename T, int S, bool XC>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3))) void depthwise3x3_dot2_kernel(const DepthwiseParams p, const DwPairTile q) {
  constexpr int V = 8;
  typedef unsigned u4 __attribute__((ext_vector_type(4)));
  extern __shared__ __align__(16) unsigned char smem[];
  const int plane = q.pairs_h * q.in_w * q.cg;            // 16-byte words per plane
  u4* s_lo = reinterpret_cast<u4*>(smem);
  u4* s_hi = s_lo + plane;
  unsigned char* s_keep = smem + (size_t)plane * 32;        // [256] mask byte of every tile pixel
  int* s_rank = reinterpret_cast<int*>(s_keep + 256);       // [256] its row in a compact output

  const int t = threadIdx.x;
  const int groups = p.c / V;
  const int g0 = blockIdx.y * q.cg;
  const int tile_pixels = q.ty * q.tx;

  // ---- this lane's channel group: filter pairs and bias ----------------------------------------------------
  const int g = t % q.cg, slot = t / q.cg, per_pass = 256 / q.cg;
  const bool lane_on = slot < per_pass && g0 + g < groups;
  const int c0 = (g0 + (lane_on ? g : 0)) * V;
  unsigned short wbits[9][V];
  {
    const T* __restrict__ wp = static_cast<const T*>(p.wp) + c0;
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
      const u4 wv = *reinterpret_cast<const u4*>(wp + (int64_t)tap * p.c);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        wbits[tap][2 * k] = (unsigned short)(wv[k] & 0xffffu);
        wbits[tap][2 * k + 1] = (unsigned short)(wv[k] >> 16);
      }
    }
  }
  // (first window row of a pair in the low half, as in the staged data)
  // w01 = (w0, w1); wl = (w1, w2) for stride 1, (w2, 0) for stride 2.  The two pairs with a zero half that
  // stride 1 needs are shifts of these: (w2, 0) = wl >> 16 and (0, w0) = w01 << 16 (registers are scarcer
  // than shift instructions here).
  unsigned w01[3][V], wl[3][V];
#pragma unroll
  for (int kx = 0; kx < 3; ++kx)
#pragma unroll
    for (int c = 0; c < V; ++c) {
      w01[kx][c] = (unsigned)wbits[kx][c] | ((unsigned)wbits[3 + kx][c] << 16);
      wl[kx][c] = S == 1 ? ((unsigned)wbits[3 + kx][c] | ((unsigned)wbits[6 + kx][c] << 16)) : (unsigned)wbits[6 + kx][c];
    }
  float bias_v[V];
#pragma unroll
  for (int k = 0; k < V; ++k) bias_v[k] = p.bias ? p.bias[c0 + k] : 0.0f;
  const float floor_v = p.relu ? 0.0f : -__builtin_inff();
  T* __restrict__ y = static_cast<T*>(p.y) + c0;

  // ---- staging: request a tile's patch and mask bytes; later interleave the rows two by two into LDS ------
  u4 ra[kDwStageMost], rb[kDwStageMost];
  unsigned keep_r = 0;
  int rank_r = 0;
  struct Tile { int n, oy0, ox0; };
  auto tile_of = [&](int id) -> Tile {
    const int t1 = fast_div(id, q.div_tilesx_mul, q.div_tilesx_shift), tile_x = id - t1 * q.tiles_x;
    const int n = fast_div(t1, q.div_tilesy_mul, q.div_tilesy_shift), tile_y = t1 - n * q.tiles_y;
    return Tile{n, tile_y * q.ty, tile_x * q.tx};
  };
  int ia[XC ? kDwStageMost : 1], ib[XC ? kDwStageMost : 1];     // rows of the patch pixels in a compact input
  auto request_ranks = [&](const Tile& tl) {
    if constexpr (XC) {
      const int32_t* __restrict__ xr = p.x_rank + (int64_t)tl.n * p.h * p.w;
      const int iy_first = tl.oy0 * S - p.ph, ix_first = tl.ox0 * S - p.pw;
#pragma unroll
      for (int u = 0; u < kDwStageMost; ++u) {
        const int e = u * 256 + t;
        const int pix = fast_div(e, q.div_cg_mul, q.div_cg_shift);
        const int pr = fast_div(pix, q.div_inw_mul, q.div_inw_shift), px = pix - pr * q.in_w;
        const int iy = iy_first + 2 * pr, ix = ix_first + px;
        const bool ok = e < plane && (unsigned)ix < (unsigned)p.w;
        ia[u] = ib[u] = -1;
        if (ok && (unsigned)iy < (unsigned)p.h) ia[u] = xr[iy * p.w + ix];
        if (ok && (unsigned)(iy + 1) < (unsigned)p.h) ib[u] = xr[(iy + 1) * p.w + ix];
      }
    }
  };
  auto request = [&](const Tile& tl) {
    const T* __restrict__ x = static_cast<const T*>(p.x) + (XC ? (int64_t)0 : (int64_t)tl.n * p.h * p.w * p.c);
    const int iy_first = tl.oy0 * S - p.ph, ix_first = tl.ox0 * S - p.pw;
#pragma unroll
    for (int u = 0; u < kDwStageMost; ++u) {
      const int e = u * 256 + t;
      const int pix = fast_div(e, q.div_cg_mul, q.div_cg_shift), gg = e - pix * q.cg;
      const int pr = fast_div(pix, q.div_inw_mul, q.div_inw_shift), px = pix - pr * q.in_w;
      const int iy = iy_first + 2 * pr, ix = ix_first + px;
      ra[u] = u4{0, 0, 0, 0};
      rb[u] = u4{0, 0, 0, 0};
      if constexpr (XC) {
        // (ranks outside the patch, the image or the channel range were left at -1 or are masked here)
        const bool ok = g0 + gg < groups;
        if (ok && ia[u] >= 0) ra[u] = *reinterpret_cast<const u4*>(x + (int64_t)ia[u] * p.c + (g0 + gg) * V);
        if (ok && ib[u] >= 0) rb[u] = *reinterpret_cast<const u4*>(x + (int64_t)ib[u] * p.c + (g0 + gg) * V);
      } else {
        const bool ok = e < plane && (unsigned)ix < (unsigned)p.w && g0 + gg < groups;
        const T* src = x + ((int64_t)iy * p.w + ix) * p.c + (g0 + gg) * V;
        if (ok && (unsigned)iy < (unsigned)p.h) ra[u] = *reinterpret_cast<const u4*>(src);
        if (ok && (unsigned)(iy + 1) < (unsigned)p.h) rb[u] = *reinterpret_cast<const u4*>(src + (int64_t)p.w * p.c);
      }
    }
    // mask byte of the tile pixel this lane looks after (a tile has at most 256 pixels): 1 = kept,
    // 2 = dropped, 0 = outside the map
    // The row of the pixel in a compact output travels the same way: looked up at the store it would be a
    // dependent global load in the compute loop, whose wait also waits for the next tile's patch.
    keep_r = 0;
    rank_r = 0;
    if (t < tile_pixels) {
      const int ty = fast_div(t, q.div_tx_mul, q.div_tx_shift), tx = t - ty * q.tx;
      const int oy = tl.oy0 + ty, ox = tl.ox0 + tx;
      if (oy < p.ho && ox < p.wo) {
        keep_r = p.mask ? (p.mask[(p.mask_spatial ? 0 : tl.n * p.ho_wo) + oy * p.wo + ox] ? 1u : 2u) : 1u;
        if (p.rank) rank_r = p.rank[tl.n * p.ho_wo + oy * p.wo + ox];   // (meaningful for kept pixels only)
      }
    }
  };
  auto deposit = [&]() {
#pragma unroll
    for (int u = 0; u < kDwStageMost; ++u) {
      const int e = u * 256 + t;
      if (e < plane) {
        u4 lo, hi;   // dword k of a row holds channels 2k (low half) and 2k+1
        lo[0] = (ra[u][0] & 0xffffu) | (rb[u][0] << 16); lo[1] = (ra[u][0] >> 16) | (rb[u][0] & 0xffff0000u);
        lo[2] = (ra[u][1] & 0xffffu) | (rb[u][1] << 16); lo[3] = (ra[u][1] >> 16) | (rb[u][1] & 0xffff0000u);
        hi[0] = (ra[u][2] & 0xffffu) | (rb[u][2] << 16); hi[1] = (ra[u][2] >> 16) | (rb[u][2] & 0xffff0000u);
        hi[2] = (ra[u][3] & 0xffffu) | (rb[u][3] << 16); hi[3] = (ra[u][3] >> 16) | (rb[u][3] & 0xffff0000u);
        s_lo[e] = lo;
        s_hi[e] = hi;
      }
    }
    if (t < tile_pixels) {
      s_keep[t] = (unsigned char)keep_r;
      if (p.rank) s_rank[t] = rank_r;
    }
  };

  auto pack_out = [&](const float (&a)[V]) -> u4 {
    DwGroup<T, V> o;
#pragma unroll
    for (int j = 0; j < V; ++j) o.v[j] = (T)__builtin_fmaxf(a[j], floor_v);
    return __builtin_bit_cast(u4, o);
  };
  // pixel `pix` of the tile = dense row r
  auto put = [&](unsigned k, int pix, int r, u4 v) {
    if (k == 1) *reinterpret_cast<u4*>(y + (p.rank ? (int64_t)s_rank[pix] : (int64_t)r) * p.c) = v;
    else if (k == 2 && p.zero_fill) *reinterpret_cast<u4*>(y + (int64_t)r * p.c) = u4{0, 0, 0, 0};   // Alg. 2, mask == 0 branch
  };

  auto compute = [&](const Tile& tl) {
    if (!lane_on) return;
    if constexpr (S == 1) {
      const int items = (q.ty >> 1) * q.tx;                 // vertical pairs of output pixels
      for (int it = slot; it < items; it += per_pass) {
        const int j = fast_div(it, q.div_tx_mul, q.div_tx_shift), tx = it - j * q.tx;
        const unsigned k0 = s_keep[(2 * j) * q.tx + tx], k1 = s_keep[(2 * j + 1) * q.tx + tx];
        if ((k0 | k1) == 0) continue;
        const int r0 = tl.n * p.ho_wo + (tl.oy0 + 2 * j) * p.wo + tl.ox0 + tx;
        u4 o0 = u4{0, 0, 0, 0}, o1 = u4{0, 0, 0, 0};
        if (k0 == 1 || k1 == 1) {
          const int base = (j * q.in_w + tx) * q.cg + g, next = base + q.in_w * q.cg;
          float a0[V], a1[V];
#pragma unroll
          for (int c = 0; c < V; ++c) { a0[c] = bias_v[c]; a1[c] = bias_v[c]; }
#pragma unroll
          for (int kx = 0; kx < 3; ++kx) {
            const u4 pl = s_lo[base + kx * q.cg], ph = s_hi[base + kx * q.cg];
            const u4 ql = s_lo[next + kx * q.cg], qh = s_hi[next + kx * q.cg];
#pragma unroll
            for (int c = 0; c < V; ++c) {
              const unsigned xa = c < 4 ? pl[c & 3] : ph[c & 3], xb = c < 4 ? ql[c & 3] : qh[c & 3];
              // (the empty statements keep the compiler from hoisting the shifted pairs out of the loop
              // into 48 more registers)
              unsigned wa = w01[kx][c], wb = wl[kx][c];
              asm volatile("" : "+v"(wa), "+v"(wb));
              // the halves that meet a zero filter entry belong to rows outside the window: they are
              // cleared, so that a non-finite value there cannot turn 0 * x into a NaN
              a0[c] = Dot2<T>::run(xa, wa, a0[c]);
              a0[c] = Dot2<T>::run(xb & 0xffffu, wb >> 16, a0[c]);
              a1[c] = Dot2<T>::run(xa & 0xffff0000u, wa << 16, a1[c]);
              a1[c] = Dot2<T>::run(xb, wb, a1[c]);
            }
            __builtin_amdgcn_sched_barrier(0);   // one window column at a time: fewer patch words live at once
          }
          o0 = pack_out(a0);
          o1 = pack_out(a1);
        }
        put(k0, (2 * j) * q.tx + tx, r0, o0);
        put(k1, (2 * j + 1) * q.tx + tx, r0 + p.wo, o1);
      }
    } else {
      const int items = q.ty * q.tx;
      for (int it = slot; it < items; it += per_pass) {
        const unsigned k0 = s_keep[it];
        if (k0 == 0) continue;
        const int ty = fast_div(it, q.div_tx_mul, q.div_tx_shift), tx = it - ty * q.tx;
        const int r0 = tl.n * p.ho_wo + (tl.oy0 + ty) * p.wo + tl.ox0 + tx;
        u4 o0 = u4{0, 0, 0, 0};
        if (k0 == 1) {
          const int base = (ty * q.in_w + tx * 2) * q.cg + g, next = base + q.in_w * q.cg;
          float a0[V];
#pragma unroll
          for (int c = 0; c < V; ++c) a0[c] = bias_v[c];
#pragma unroll
          for (int kx = 0; kx < 3; ++kx) {
            const u4 pl = s_lo[base + kx * q.cg], ph = s_hi[base + kx * q.cg];
            const u4 ql = s_lo[next + kx * q.cg], qh = s_hi[next + kx * q.cg];
#pragma unroll
            for (int c = 0; c < V; ++c) {
              const unsigned xa = c < 4 ? pl[c & 3] : ph[c & 3], xb = c < 4 ? ql[c & 3] : qh[c & 3];
              a0[c] = Dot2<T>::run(xa, w01[kx][c], a0[c]);
              a0[c] = Dot2<T>::run(xb & 0xffffu, wl[kx][c], a0[c]);     // (the high half is a row below the window)
            }
          }
          o0 = pack_out(a0);
        }
        put(k0, it, r0, o0);
      }
    }
  };

  // ---- the tiles of this workgroup ------------------------------------------------------------------------
  int id = blockIdx.x;
  if (id >= q.tiles) return;
  Tile cur = tile_of(id);
  request_ranks(cur);
  request(cur);
  if (id + (int)gridDim.x < q.tiles) request_ranks(tile_of(id + gridDim.x));
  deposit();
  __syncthreads();
  for (;;) {
    const int next_id = id + gridDim.x;
    const bool more = next_id < q.tiles;
    Tile nxt = cur;
    if (more) {
      nxt = tile_of(next_id);
      request(nxt);            // in flight while this tile is computed
      if (next_id + (int)gridDim.x < q.tiles) request_ranks(tile_of(next_id + gridDim.x));
    }
    compute(cur);
    if (!more) break;
    __syncthreads();           // every lane has read the patch
    deposit();
    __syncthreads();
    cur = nxt;
    id = next_id;
  }
}

// position of every kept row in the row list: rank[row_idx[i]] = i
__global__ void depthwise_rank_kernel(const int32_t* __restrict__ row_idx, const int32_t* __restrict__ kept,
                                      int32_t* __restrict__ rank) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < *kept) rank[row_idx[i]] = i;
}

// Tile extent along one axis: the extent in [6, most] that wastes the fewest pixels at the edge of a map
// of `size` pixels, the larger one at a tie.
static int tile_extent(int size, int most) {
  if (size <= most) return size;
  int best = most;
  double best_waste = 1e30;
  for (int t = most; t >= 6 && t >= 1; --t) {
    const double waste = (double)((size + t - 1) / t * t) / size;
    if (waste < best_waste - 1e-9) { best_waste = waste; best = t; }
  }
  return best;
}

constexpr int kDwPatchBytes = 48 * 1024;   // most LDS one workgroup spends on its input patch

// Channel groups per workgroup.  Up to 32 groups (512 bytes per pixel) a workgroup takes whole pixels: a
// patch row is then one contiguous run of memory.  Beyond that the pixel is cut into chunks of 16 or 8
// groups, i.e. at multiples of a 128-byte line wherever the group count allows: a line that two
// workgroups share is fetched twice and written in two halves.
static void channel_chunks(int groups, int32_t* cg, int32_t* chunks) {
  if (groups <= 32) *cg = groups;
  else if (groups % 16 == 0) *cg = 16;
  else if (groups % 8 == 0) *cg = 8;
  else *cg = 16;
  *chunks = (groups + *cg - 1) / *cg;
}

// widest tile (output columns) whose patch leaves room for `rows` units of `unit_bytes` per patch column
static int widest_tile(int budget, int rows, int unit_bytes, int stride) {
  const int most_in_w = budget / (rows * unit_bytes);
  return std::max(4, std::min(16, (most_in_w - 3) / stride + 1));
}

template <typename T, int S>
static hipError_t launch_tiles(const DepthwiseParams& p, hipStream_t stream) {
  constexpr int V = DwVec<T>::V;
  const int groups = p.c / V;
  DwTile q;
  channel_chunks(groups, &q.cg, &q.chunks);
  q.tx = tile_extent(p.wo, widest_tile(kDwPatchBytes, 10, q.cg * 16, S));
  q.txp = (q.tx + 1) & ~1;
  q.in_w = (q.txp - 1) * S + 3;
  const int row_bytes = q.in_w * q.cg * 16;
  const int most_in_h = std::max(3, kDwPatchBytes / row_bytes);
  q.ty = tile_extent(p.ho, std::max(1, std::min(16, (most_in_h - 3) / S + 1)));
  q.in_h = (q.ty - 1) * S + 3;
  q.tiles_y = (p.ho + q.ty - 1) / q.ty;
  q.tiles_x = (p.wo + q.tx - 1) / q.tx;
  magic_div((uint32_t)q.cg, &q.div_cg_mul, &q.div_cg_shift);
  magic_div((uint32_t)q.in_w, &q.div_inw_mul, &q.div_inw_shift);
  magic_div((uint32_t)q.txp, &q.div_txp_mul, &q.div_txp_shift);
  magic_div((uint32_t)(q.txp / 2), &q.div_pairs_mul, &q.div_pairs_shift);
  const size_t lds = (size_t)q.in_h * row_bytes + (size_t)((q.ty * q.txp + 15) / 16 * 16);
  const int64_t wgs = (int64_t)p.n * q.tiles_y * q.tiles_x * q.chunks;
  hipLaunchKernelGGL((depthwise3x3_kernel<T, V, S>), dim3((unsigned)wgs), dim3(256), lds, stream, p, q);
  return hipGetLastError();
}

template <typename T, int S, bool XC>
static hipError_t launch_pair_tiles(const DepthwiseParams& p, hipStream_t stream) {
  const int groups = p.c / 8;
  DwPairTile q;
  int32_t chunks;
  channel_chunks(groups, &q.cg, &chunks);
  // the patch holds at most kDwStageMost * 256 interleaved words of 32 bytes
  const int budget = kDwStageMost * 256 * 32;
  q.tx = tile_extent(p.wo, widest_tile(budget, 4, q.cg * 32, S));
  q.in_w = (q.tx - 1) * S + 3;
  const int pair_bytes = q.in_w * q.cg * 32;                       // one pair of patch rows
  const int most_pairs = std::max(2, budget / pair_bytes);
  // stride 1: ty (even) output rows need ty/2 + 1 row pairs; stride 2: ty output rows need ty + 1;
  // a tile has at most 256 pixels (one mask byte per lane)
  int most_ty = S == 1 ? 2 * (most_pairs - 1) : most_pairs - 1;
  most_ty = std::max(1, std::min(most_ty, 256 / q.tx));
  if (S == 1) most_ty = std::max(2, most_ty & ~1);
  q.ty = tile_extent(p.ho, std::min(16, most_ty));
  if (S == 1) q.ty = std::min((q.ty + 1) & ~1, most_ty);
  q.pairs_h = S == 1 ? q.ty / 2 + 1 : q.ty + 1;
  if ((int64_t)q.pairs_h * q.in_w * q.cg > kDwStageMost * 256 || q.ty * q.tx > 256) return hipErrorInvalidValue;
  q.tiles_y = (p.ho + q.ty - 1) / q.ty;
  q.tiles_x = (p.wo + q.tx - 1) / q.tx;
  q.tiles = p.n * q.tiles_y * q.tiles_x;
  magic_div((uint32_t)q.cg, &q.div_cg_mul, &q.div_cg_shift);
  magic_div((uint32_t)q.in_w, &q.div_inw_mul, &q.div_inw_shift);
  magic_div((uint32_t)q.tx, &q.div_tx_mul, &q.div_tx_shift);
  magic_div((uint32_t)q.tiles_x, &q.div_tilesx_mul, &q.div_tilesx_shift);
  magic_div((uint32_t)q.tiles_y, &q.div_tilesy_mul, &q.div_tilesy_shift);
  const size_t lds = (size_t)q.pairs_h * pair_bytes + 256 + 256 * sizeof(int);   // patch, mask bytes, compact rows
  // persistent workgroups: about three per compute unit (LDS and registers allow that many), split over the chunks
  constexpr int per_cu = 3;
  const int wgs = std::max(1, std::min(q.tiles, (256 * per_cu + chunks - 1) / chunks));
  hipLaunchKernelGGL((depthwise3x3_dot2_kernel<T, S, XC>), dim3((unsigned)wgs, (unsigned)chunks), dim3(256), lds, stream, p, q);
  return hipGetLastError();
}

template <typename T>
static hipError_t launch_typed(const DepthwiseParams& p, hipStream_t stream) {
  constexpr int V = DwVec<T>::V;
  const bool vec = p.c % V == 0;
  // the LDS-tiled kernels: 3x3 windows, no dilation, stride 1 or 2; a compact input (with its rank map) only
  // in the 16-bit kernel
  if (vec && p.kh == 3 && p.kw == 3 && p.dil_h == 1 && p.dil_w == 1 && p.sh == p.sw && (p.sh == 1 || p.sh == 2)) {
    if constexpr (sizeof(T) == 2) {
      if (p.x_compact && p.x_rank)
        return p.sh == 1 ? launch_pair_tiles<T, 1, true>(p, stream) : launch_pair_tiles<T, 2, true>(p, stream);
      if (!p.x_compact)
        return p.sh == 1 ? launch_pair_tiles<T, 1, false>(p, stream) : launch_pair_tiles<T, 2, false>(p, stream);
    } else if (!p.x_compact) {
      return p.sh == 1 ? launch_tiles<T, 1>(p, stream) : launch_tiles<T, 2>(p, stream);
    }
  }
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

hipError_t depthwise_rank(const int32_t* row_idx, const int32_t* kept_dev, int32_t* rank, int64_t m, hipStream_t stream) {
  hipLaunchKernelGGL(depthwise_rank_kernel, dim3((unsigned)((m + 255) / 256)), dim3(256), 0, stream, row_idx, kept_dev, rank);
  return hipGetLastError();
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
