// Backward pass of the masked convolution (Alg. 1: backward(model) follows maskedForward(model, mask)).
//
// Forward: y[r, co] = mask[r] ? act(sum_k A[r, k] w[co, k] + bias[co]) : 0, A = lowered activations (Sec. 3).
// With the upstream gradient dy and  g[r, co] = dy[r, co] if mask[r] and (no ReLU or y[r, co] > 0), else 0:
//     db[co]    = sum_r g[r, co]
//     dw[co, k] = sum_r g[r, co] A[r, k]          -- a contraction over the kept rows only: it shrinks with
//                                                     the sparsity exactly like the forward GEMM (Sec. 3.2)
//     dx        = the transposed convolution of g  -- for stride 1 an ordinary convolution of the g map
//                                                     with the filters rotated by 180 degrees and
//                                                     transposed; it runs through the forward kernels
// Kernels here: g map with its column sums (db), the filter-gradient GEMM on the matrix cores with
// a deterministic two-pass reduction over row splits, and the filter rotation for the input gradient.
#include "../../include/sparse_conv.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <new>

#include "conv_params.hpp"
#include "mma_common.hpp"

namespace sc {

void note_hip_error(int32_t code);   // defined with the other host code of the library

// ---- g map and db ------------------------------------------------------------------------------------------------
// g = the gradient that actually flows through a row (zero rows for dropped positions); db = its column
// sums, in two passes with a fixed order of additions.  First pass, fused with the g map: a workgroup owns
// a slab of rows; a lane owns one 16-byte group of channels and every (256 / groups)-th row of the slab,
// writes g for them and keeps their sum; the row lanes of a group are then added in lane order through LDS.
constexpr int kSumRows = 512;   // most rows per workgroup
constexpr int kSumRowsLeast = 32;
// rows per workgroup: about 1024 workgroups, between kSumRowsLeast and kSumRows rows each
static inline int colsum_slab_rows(int64_t rows) {
  const int64_t want = (rows + 1023) / 1024;
  return (int)std::min<int64_t>(kSumRows, std::max<int64_t>(kSumRowsLeast, (want + 31) / 32 * 32));
}
template <typename T>
__global__ __launch_bounds__(256) void grad_map_kernel(const T* __restrict__ y, const T* __restrict__ dy,
                                                       const uint8_t* __restrict__ mask, T* __restrict__ g, int64_t rows,
                                                       int c, int slab_rows, int relu, int period,
                                                       float* __restrict__ partial) {
  __shared__ float s_acc[256][9];                       // (padded: the final adds walk a column of it)
  struct alignas(16) Grp { T v[8]; };
  const int groups = c / 8;
  const int64_t r0 = (int64_t)blockIdx.x * slab_rows, r1 = min(rows, r0 + slab_rows);
  for (int gbase = 0; gbase < groups; gbase += 256) {   // (more than 2048 channels: several sweeps)
    const int gcount = min(256, groups - gbase);
    const int lanes_per_group = 256 / gcount;            // row lanes that share a channel group
    const int gi = threadIdx.x % gcount, rl = threadIdx.x / gcount;
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.0f;
    if (rl < lanes_per_group)
      for (int64_t r = r0 + rl; r < r1; r += lanes_per_group) {
        const int64_t at = r * c + (int64_t)(gbase + gi) * 8;
        Grp out;
#pragma unroll
        for (int j = 0; j < 8; ++j) out.v[j] = (T)0.0f;
        if (mask[period ? r % period : r] != 0) {
          out = *reinterpret_cast<const Grp*>(dy + at);
          if (relu) {
            const Grp f = *reinterpret_cast<const Grp*>(y + at);
#pragma unroll
            for (int j = 0; j < 8; ++j) out.v[j] = (float)f.v[j] > 0.0f ? out.v[j] : (T)0.0f;
          }
        }
        *reinterpret_cast<Grp*>(g + at) = out;
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] += (float)out.v[j];
      }
#pragma unroll
    for (int j = 0; j < 8; ++j) s_acc[threadIdx.x][j] = acc[j];
    __syncthreads();
    if (threadIdx.x < gcount) {
      float tot[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) tot[j] = 0.0f;
      for (int l = 0; l < lanes_per_group; ++l)
#pragma unroll
        for (int j = 0; j < 8; ++j) tot[j] += s_acc[l * gcount + threadIdx.x][j];
#pragma unroll
      for (int j = 0; j < 8; ++j) partial[(int64_t)blockIdx.x * c + (int64_t)(gbase + threadIdx.x) * 8 + j] = tot[j];
    }
    __syncthreads();
  }
}
// Second pass: a workgroup owns four channels; 64 lanes per channel each add every 64th slab, then the 64
// sub-sums are added in lane order.
__global__ __launch_bounds__(256) void colsum_final_kernel(const float* __restrict__ partial, int slabs, int c,
                                                           float* __restrict__ out) {
  __shared__ float s_sub[64][5];
  const int e = threadIdx.x & 3, sl = threadIdx.x >> 2;
  const int col = blockIdx.x * 4 + e;
  float acc = 0.0f;
  if (col < c)
    for (int s = sl; s < slabs; s += 64) acc += partial[(int64_t)s * c + col];
  s_sub[sl][e] = acc;
  __syncthreads();
  if (threadIdx.x < 4 && col < c) {
    float tot = 0.0f;
    for (int l = 0; l < 64; ++l) tot += s_sub[l][threadIdx.x];
    out[col] = tot;
  }
}

// ---- filters for the input gradient: w'[ci][kh-1-ky][kw-1-kx][co] = w[co][ky][kx][ci] ---------------------------
template <typename T>
__global__ void rotate_filters_kernel(const T* __restrict__ w, T* __restrict__ wr, int c_out, int c_in, int kh, int kw) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t total = (int64_t)c_out * kh * kw * c_in;
  if (idx >= total) return;
  int64_t rest = idx;
  const int co = (int)(rest % c_out); rest /= c_out;
  const int kx = (int)(rest % kw); rest /= kw;
  const int ky = (int)(rest % kh);
  const int ci = (int)(rest / kh);
  wr[idx] = w[(((int64_t)co * kh + (kh - 1 - ky)) * kw + (kw - 1 - kx)) * c_in + ci];
}

__global__ void fill_bytes_kernel(uint8_t* __restrict__ p, int64_t n, uint8_t v) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = v;
}

// Strided layers: the transposed convolution is an ordinary stride-1 convolution of the g map with zeros
// interleaved -- row (oy, ox) of g lands at (oy * sh, ox * sw) of a map of hu x wu pixels that is zero
// everywhere else.  The zeros are written once (plan time) and stay: every run rewrites the same pixels.
template <int V16>
__global__ void upsample_rows_kernel(const v4i* __restrict__ g, v4i* __restrict__ gu, int64_t groups_total,
                                     int groups_per_row, int ho_wo, int wo, int sh, int sw, int hu, int wu) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= groups_total) return;
  const int64_t r = idx / groups_per_row;
  const int q = (int)(idx - r * groups_per_row);
  const int n = (int)(r / ho_wo), rem = (int)(r - (int64_t)n * ho_wo);
  const int oy = rem / wo, ox = rem - oy * wo;
  gu[(((int64_t)n * hu + (int64_t)oy * sh) * wu + (int64_t)ox * sw) * groups_per_row + q] = g[idx];
}

// ---- filter gradient -----------------------------------------------------------------------------------------
// dW[co][k] = sum over the kept rows i of g[row_i][co] * A[row_i][k]: a GEMM whose contraction runs over
// rows.  Both operands are row-major (a row of g is Cout contiguous values, a window tap of a row is Cin
// contiguous values), while an MFMA lane needs eight consecutive CONTRACTION entries of one column.  The
// tiles are therefore staged row-major in LDS (coalesced 16-byte gathers, as in the forward kernels) and
// read with the transposing LDS load of gfx950 (ds_read_b64_tr_b16): two loads give a lane the eight
// consecutive rows of its column.
//   workgroup = 128 output channels x 128 window entries x one split of the kept rows; 2 x 2 wavefronts,
//               each 64 x 64 (2 x 2 MFMA blocks of 32 x 32 x 16)
//   stage     = 64 kept rows, double buffered: the next stage's gathers are in flight during the MFMAs
//   result    = float partial sums per split; a second kernel adds the splits in order (deterministic)
struct WgradParams {
  const void* x;
  const void* g;             // g map [M][Cout]
  const int32_t* row_idx;    // kept rows, or null for the identity
  float* out;                // [splits][Cout][K]
  int32_t rows, rows_per_split, splits;
  int32_t h, w, c_in, ho_wo, wo, c_out;
  int32_t kh, kw, sh, sw, ph, pw, dil_h, dil_w;
  int32_t k;                 // kh * kw * c_in
  int32_t co_tiles, k_tiles;
  uint32_t div_howo_mul, div_howo_shift, div_wo_mul, div_wo_shift;
};

constexpr int kWgRows = 64;      // kept rows per stage

// BM output channels x BN window entries per workgroup, BM * BN = 128 * 128.  (A 64 x 256 shape for layers
// with at most 64 output channels measured slower than 128 x 128 with half of its channel rows idle: the
// kernel is bound by the instructions spent per staged row, not by the MFMAs.)
template <int DT, int BM, int BN>
__global__ __launch_bounds__(256) void wgrad_kernel(const WgradParams p) {
  using E = Elem<DT>;
  using T = typename E::T;
  constexpr int R = kWgRows;
  constexpr int WAVES_N = BN / 64;
  static_assert((BM / 64) * WAVES_N == 4, "four wavefronts of 64 x 64");
  // LDS row pitches in 16-bit elements: 64 bytes more than a multiple of 256, so that the 4 rows x 32 bytes
  // x 2 column blocks that 32 lanes of a transposing read touch fall into 64 different banks
  constexpr int PG = BM + 32, PA = BN + 32;
  constexpr int GQ = BM / 8, AQ = BN / 8;              // 16-byte groups per staged row
  constexpr int NG = GQ / 4, NA = AQ / 4;              // groups a lane stages per tile
  static_assert(R == 64, "one staged row per four lanes");
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned short* s_g = reinterpret_cast<unsigned short*>(smem);      // [2][R][PG]
  unsigned short* s_a = s_g + 2 * R * PG;                             // [2][R][PA]

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int fp = lane & 31, fh = lane >> 5;
  const int wm0 = (wave / WAVES_N) * 64, wn0 = (wave % WAVES_N) * 64;
  const int tiles = p.co_tiles * p.k_tiles;
  const int split = blockIdx.x / tiles, tile = blockIdx.x - split * tiles;
  const int co0 = (tile / p.k_tiles) * BM, k0 = (tile % p.k_tiles) * BN;
  const int i_begin = split * p.rows_per_split, i_end = min(p.rows, i_begin + p.rows_per_split);

  // Staging: four lanes share one row of a stage; lane `sub` of the four takes the 16-byte groups
  // sub, sub + 4, sub + 8, ... of that row in both tiles (adjacent lanes: adjacent groups, so a load
  // instruction covers 64 contiguous bytes per row).  The row is decoded once per lane and stage; what
  // depends on the group -- its window tap and channel -- is fixed for the whole kernel.
  const int srow = t >> 2, sub = t & 3;
  const T* __restrict__ xg = static_cast<const T*>(p.x);
  const T* __restrict__ gg = static_cast<const T*>(p.g);
  int g_col[NG];                                       // first output channel of group u, or -1 beyond Cout
#pragma unroll
  for (int u = 0; u < NG; ++u) {
    const int c = co0 + 8 * (4 * u + sub);
    g_col[u] = c < p.c_out ? c : -1;                   // (Cout is a multiple of 8)
  }
  int a_dy[NA], a_dx[NA], a_off[NA];                   // tap displacement and element offset of group u; a_off < 0 beyond K
#pragma unroll
  for (int u = 0; u < NA; ++u) {
    const int kk = k0 + 8 * (4 * u + sub);             // (Cin is a multiple of 8: a group lies inside one tap)
    const int tap = kk < p.k ? kk / p.c_in : 0, ci = kk - tap * p.c_in;
    const int ky = tap / p.kw, kx = tap - ky * p.kw;
    a_dy[u] = ky * p.dil_h;
    a_dx[u] = kx * p.dil_w;
    a_off[u] = kk < p.k ? (a_dy[u] * p.w + a_dx[u]) * p.c_in + ci : -1;
  }

  // row numbers are fetched one stage ahead of the data they address, so a stage costs one round trip
  v4i rg[NG], ra[NA];
  int r_next = -1;
  auto request_rows = [&](int i0) {
    const int i = i0 + srow;
    r_next = i < i_end ? (p.row_idx ? p.row_idx[i] : i) : -1;
  };
  auto request = [&]() {
    const int r = r_next;
#pragma unroll
    for (int u = 0; u < NG; ++u) rg[u] = v4i{0, 0, 0, 0};
#pragma unroll
    for (int u = 0; u < NA; ++u) ra[u] = v4i{0, 0, 0, 0};
    if (r >= 0) {
      const T* grow = gg + (int64_t)r * p.c_out;
#pragma unroll
      for (int u = 0; u < NG; ++u)
        if (g_col[u] >= 0) rg[u] = *reinterpret_cast<const v4i*>(grow + g_col[u]);
      const int n = fast_div(r, p.div_howo_mul, p.div_howo_shift), rem = r - n * p.ho_wo;
      const int oy = fast_div(rem, p.div_wo_mul, p.div_wo_shift), ox = rem - oy * p.wo;
      const int iy0 = oy * p.sh - p.ph, ix0 = ox * p.sw - p.pw;
      const T* xrow = xg + (((int64_t)n * p.h + iy0) * p.w + ix0) * p.c_in;     // may point before the tensor: used with in-range taps only
#pragma unroll
      for (int u = 0; u < NA; ++u)
        if (a_off[u] >= 0 && (unsigned)(iy0 + a_dy[u]) < (unsigned)p.h && (unsigned)(ix0 + a_dx[u]) < (unsigned)p.w)
          ra[u] = *reinterpret_cast<const v4i*>(xrow + a_off[u]);
    }
  };
  auto deposit = [&](int buf) {
#pragma unroll
    for (int u = 0; u < NG; ++u) *reinterpret_cast<v4i*>(s_g + (buf * R + srow) * PG + 8 * (4 * u + sub)) = rg[u];
#pragma unroll
    for (int u = 0; u < NA; ++u) *reinterpret_cast<v4i*>(s_a + (buf * R + srow) * PA + 8 * (4 * u + sub)) = ra[u];
  };

  floatx16 acc[2][2];
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

  // An MFMA operand: eight consecutive rows of one column of a staged tile.  ds_read_b64_tr_b16 transposes
  // within groups of 16 lanes -- result lane j, element t = source lane 4t + j/4, element j%4 (layout checked
  // on the device) -- so with source lane s of a group addressing row s/4, columns 4*(s%4) .. +3 of a
  // 4 x 16 block, result lane j holds rows 0..3 of column j of that block: two such reads (rows 0..3 and
  // 4..7) are the operand, in the order the MFMA wants, with no further instructions.
  typedef short tr_s16x4 __attribute__((ext_vector_type(4)));
  typedef __attribute__((address_space(3))) tr_s16x4 lds_s16x4;
  const int l16 = lane & 15;
  const int tr_g = (8 * fh + (l16 >> 2)) * PG + 16 * ((lane & 31) >> 4) + 4 * (l16 & 3);   // element offsets
  const int tr_a = (8 * fh + (l16 >> 2)) * PA + 16 * ((lane & 31) >> 4) + 4 * (l16 & 3);
  auto column = [&](const unsigned short* s, int pitch) -> v4i {
    const tr_s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(s));
    const tr_s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(s + 4 * pitch));
    struct { tr_s16x4 a, b; } both = {lo, hi};
    return __builtin_bit_cast(v4i, both);
  };

  if (i_begin < i_end) {
    request_rows(i_begin);
    request();
    request_rows(i_begin + R);
    deposit(0);
  }
  __syncthreads();
  int buf = 0;
  for (int i0 = i_begin; i0 < i_end; i0 += R) {
    const bool more = i0 + R < i_end;
    if (more) {
      request();                                   // in flight during the MFMAs below
      request_rows(i0 + 2 * R);
    }
    const unsigned short* tg = s_g + buf * R * PG;
    const unsigned short* ta = s_a + buf * R * PA;
#pragma unroll
    for (int ks = 0; ks < R / 16; ++ks) {
      v4i gf[2], af[2];
#pragma unroll
      for (int mi = 0; mi < 2; ++mi) gf[mi] = column(tg + 16 * ks * PG + wm0 + 32 * mi + tr_g, PG);
#pragma unroll
      for (int ni = 0; ni < 2; ++ni) af[ni] = column(ta + 16 * ks * PA + wn0 + 32 * ni + tr_a, PA);
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) E::mma(acc[mi][ni], gf[mi], af[ni]);
    }
    if (more) deposit(buf ^ 1);
    __syncthreads();
    buf ^= 1;
  }

  // MFMA result row 8j + 4h + i sits in register 4j + i of lane half h; column = lane % 32
  float* __restrict__ out = p.out + (int64_t)split * p.c_out * p.k;
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
      const int kcol = k0 + wn0 + 32 * ni + fp;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int co = co0 + wm0 + 32 * mi + 8 * (v >> 2) + 4 * fh + (v & 3);
        if (co < p.c_out && kcol < p.k) out[(int64_t)co * p.k + kcol] = acc[mi][ni][v];
      }
    }
}

template <int DT, int BM, int BN>
static hipError_t wgrad_launch(WgradParams p, hipStream_t stream) {
  constexpr size_t lds = (size_t)2 * kWgRows * (BM + 32 + BN + 32) * 2;
  p.co_tiles = (p.c_out + BM - 1) / BM;
  p.k_tiles = (p.k + BN - 1) / BN;
  const unsigned grid = (unsigned)(p.co_tiles * p.k_tiles * p.splits);
  static std::atomic<bool> attr_set{false};                       // (one flag per tile shape and type)
  if (lds > 64 * 1024 && !attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(wgrad_kernel<DT, BM, BN>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((wgrad_kernel<DT, BM, BN>), dim3(grid), dim3(256), lds, stream, p);
  return hipGetLastError();
}

// dw[i] = sum over the splits of partial[s][i].  A workgroup owns 64 consecutive elements (16 groups of
// four); 16 lanes per group each add every 16th split (independent 16-byte loads in flight), then the 16
// sub-sums are added in lane order: the order of additions is fixed.  (Cout * K is a multiple of 64.)
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const float* __restrict__ partial, int splits, int64_t count,
                                                           float* __restrict__ dw) {
  __shared__ v4f s_sub[16][17];
  const int e = threadIdx.x & 15, sl = threadIdx.x >> 4;
  const int64_t i = ((int64_t)blockIdx.x * 16 + e) * 4;
  v4f acc = {0.0f, 0.0f, 0.0f, 0.0f};
  if (i < count)
    for (int s = sl; s < splits; s += 16) {
      const v4f v = *reinterpret_cast<const v4f*>(partial + (int64_t)s * count + i);
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] += v[j];
    }
  s_sub[sl][e] = acc;
  __syncthreads();
  if (threadIdx.x < 16 && i < count) {
    v4f tot = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int l = 0; l < 16; ++l)
#pragma unroll
      for (int j = 0; j < 4; ++j) tot[j] += s_sub[l][threadIdx.x][j];
    *reinterpret_cast<v4f*>(dw + i) = tot;
  }
}

constexpr size_t kWgradPartialBytes = (size_t)64 << 20;   // most workspace the row splits may take

static int wgrad_splits(int64_t rows, int c_out, int k) {
  const int bm = 128, bn = 128;
  const int64_t tiles = (int64_t)((c_out + bm - 1) / bm) * ((k + bn - 1) / bn);
  int64_t want = (768 + tiles - 1) / tiles;                                        // about three workgroups per CU
  want = std::min<int64_t>(want, (rows + 8 * kWgRows - 1) / (8 * kWgRows));        // at least eight stages per split
  want = std::min<int64_t>(want, (int64_t)(kWgradPartialBytes / ((size_t)c_out * k * 4)));
  return (int)std::max<int64_t>(want, 1);
}

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace sc

struct sc_bwd_plan {
  const sc_plan* fwd;
  sc_conv_desc desc;
  int32_t ho, wo;
  int64_t m;
  unsigned char* ws;
  size_t off_g, off_ones, off_wrot, off_inner, off_partial, off_colsum, off_gup;
  int32_t hu, wu;            // zero-interleaved g map of strided layers (0: stride 1, the g map itself is used)
  sc_plan* inner;            // dense plan of the transposed convolution (null: no input gradient for this layer)
};

namespace sc {

static sc_status backward_layout(const sc_conv_desc* d, sc_bwd_plan* L, sc_conv_desc* inner, bool* has_inner,
                                 size_t* total) {
  if (!d) return SC_ERR_NULL;
  int32_t *ho = &L->ho, *wo = &L->wo, *hu = &L->hu, *wu = &L->wu;
  int64_t* m = &L->m;
  size_t *off_g = &L->off_g, *off_ones = &L->off_ones, *off_wrot = &L->off_wrot, *off_inner = &L->off_inner,
         *off_partial = &L->off_partial, *off_colsum = &L->off_colsum, *off_gup = &L->off_gup;
  sc_status s = sparse_conv_output_shape(d, ho, wo, m);
  if (s != SC_OK) return s;
  // the filter-gradient kernel gathers 16-byte channel groups of 16-bit values
  if (d->groups != 1 || d->layout != SC_NHWC || (d->dtype != SC_BF16 && d->dtype != SC_F16) || d->c_in % 8 != 0 ||
      d->c_out % 8 != 0)
    return SC_ERR_UNSUPPORTED;
  const size_t eb = 2;
  const int64_t k = (int64_t)d->kh * d->kw * d->c_in;
  // input gradient: an ordinary stride-1 convolution of the g map (zero-interleaved for strided layers) with
  // the rotated filters, padded by dil * (k - 1) - pad; the interleaved map gets as many extra zero rows /
  // columns at the end as the forward pass left input rows / columns unused
  const int pad_h = d->dil_h * (d->kh - 1) - d->pad_h, pad_w = d->dil_w * (d->kw - 1) - d->pad_w;
  *has_inner = pad_h >= 0 && pad_w >= 0;
  const bool strided = d->stride_h != 1 || d->stride_w != 1;
  const int eff_h = d->h + 2 * d->pad_h - d->dil_h * (d->kh - 1) - 1, eff_w = d->w + 2 * d->pad_w - d->dil_w * (d->kw - 1) - 1;
  *hu = strided ? (*ho - 1) * d->stride_h + 1 + eff_h % d->stride_h : 0;
  *wu = strided ? (*wo - 1) * d->stride_w + 1 + eff_w % d->stride_w : 0;
  size_t off = 0;
  *off_g = off;      off = align_up(off + (size_t)*m * d->c_out * eb, 256);
  *off_colsum = off; off = align_up(off + (size_t)((*m + kSumRowsLeast - 1) / kSumRowsLeast) * d->c_out * 4, 256);
  *off_partial = off;
  off = align_up(off + (size_t)wgrad_splits(*m, d->c_out, (int)k) * d->c_out * k * 4, 256);   // the dense row count bounds every mask
  *off_ones = *off_wrot = *off_inner = *off_gup = off;
  if (*has_inner) {
    std::memset(inner, 0, sizeof(*inner));
    inner->n = d->n; inner->c_in = d->c_out; inner->h = strided ? *hu : *ho; inner->w = strided ? *wu : *wo;
    inner->c_out = d->c_in;
    inner->kh = d->kh; inner->kw = d->kw; inner->stride_h = 1; inner->stride_w = 1;
    inner->pad_h = pad_h; inner->pad_w = pad_w; inner->dil_h = d->dil_h; inner->dil_w = d->dil_w;
    inner->groups = 1; inner->dtype = d->dtype; inner->layout = SC_NHWC; inner->has_bias = 0; inner->relu = 0;
    inner->mask_mode = SC_MASK_SPATIAL; inner->out_mode = SC_OUT_ZERO_FILL; inner->sparsity = -1.0f;
    size_t inner_bytes = 0;
    s = sparse_conv_workspace_bytes(inner, &inner_bytes);
    if (s != SC_OK) return s;
    int32_t iho = 0, iwo = 0; int64_t im = 0;
    s = sparse_conv_output_shape(inner, &iho, &iwo, &im);
    if (s != SC_OK) return s;
    if (iho != d->h || iwo != d->w) return SC_ERR_UNSUPPORTED;     // (cannot happen: the sizes above are made to fit)
    *off_ones = off;  off = align_up(off + (size_t)d->h * d->w, 256);
    *off_wrot = off;  off = align_up(off + (size_t)d->c_out * k * eb, 256);
    *off_inner = off; off = align_up(off + inner_bytes, 256);
    if (strided) { *off_gup = off; off = align_up(off + (size_t)d->n * *hu * *wu * d->c_out * eb, 256); }
  }
  *total = off;
  return SC_OK;
}

static sc_status rotate_filters(const sc_bwd_plan* bp, const void* w_dev, hipStream_t stream) {
  const sc_conv_desc& d = bp->desc;
  const int64_t total = (int64_t)d.c_out * d.kh * d.kw * d.c_in;
  hipLaunchKernelGGL(rotate_filters_kernel<_Float16>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                     (const _Float16*)w_dev, (_Float16*)(bp->ws + bp->off_wrot), d.c_out, d.c_in, d.kh, d.kw);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { note_hip_error((int32_t)e); return SC_ERR_HIP; }
  return SC_OK;
}

}  // namespace sc

extern "C" {

sc_status sparse_conv_backward_workspace_bytes(const sc_conv_desc* desc, size_t* bytes) {
  if (!bytes) return SC_ERR_NULL;
  *bytes = 0;
  sc_bwd_plan layout; sc_conv_desc inner; bool has_inner; size_t total;
  sc_status s = sc::backward_layout(desc, &layout, &inner, &has_inner, &total);
  if (s != SC_OK) return s;
  *bytes = total;
  return SC_OK;
}

sc_status sparse_conv_backward_plan(const sc_plan* fwd, const sc_conv_desc* desc, const void* w_dev, void* workspace_dev,
                                    size_t workspace_bytes, void* hip_stream, sc_bwd_plan** out) {
  if (!out) return SC_ERR_NULL;
  *out = nullptr;
  if (!fwd || !desc || !w_dev || !workspace_dev) return SC_ERR_NULL;
  sc_bwd_plan tmp;
  std::memset(&tmp, 0, sizeof(tmp));
  sc_conv_desc inner; bool has_inner; size_t total;
  sc_status s = sc::backward_layout(desc, &tmp, &inner, &has_inner, &total);
  if (s != SC_OK) return s;
  // the descriptor must be the forward plan's
  int64_t fm = 0, fkept = 0; int32_t fho = 0, fwo = 0;
  s = sparse_conv_plan_info(fwd, &fm, &fkept, &fho, &fwo, nullptr);
  if (s != SC_OK) return s;
  if (fm != tmp.m || fho != tmp.ho || fwo != tmp.wo) return SC_ERR_BAD_SHAPE;
  if (workspace_bytes < total) return SC_ERR_WORKSPACE;
  if (((uintptr_t)workspace_dev & 255) || ((uintptr_t)w_dev & 15)) return SC_ERR_ALIGN;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  tmp.fwd = fwd;
  tmp.desc = *desc;
  tmp.ws = static_cast<unsigned char*>(workspace_dev);
  if (has_inner) {
    const int64_t ones = (int64_t)desc->h * desc->w;
    hipLaunchKernelGGL(sc::fill_bytes_kernel, dim3((unsigned)((ones + 255) / 256)), dim3(256), 0, stream,
                       tmp.ws + tmp.off_ones, ones, (uint8_t)1);
    s = sc::rotate_filters(&tmp, w_dev, stream);
    if (s != SC_OK) return s;
    if (tmp.hu > 0) {   // the zeros between the rows of g: written once, never overwritten
      hipError_t e = hipMemsetAsync(tmp.ws + tmp.off_gup, 0, (size_t)desc->n * tmp.hu * tmp.wu * desc->c_out * 2, stream);
      if (e != hipSuccess) { sc::note_hip_error((int32_t)e); return SC_ERR_HIP; }
    }
    s = sparse_conv_plan(&inner, tmp.ws + tmp.off_ones, tmp.ws + tmp.off_wrot, tmp.ws + tmp.off_inner,
                         total - tmp.off_inner, hip_stream, &tmp.inner);
    if (s != SC_OK) return s;
  }
  sc_bwd_plan* bp = new (std::nothrow) sc_bwd_plan(tmp);
  if (!bp) { sparse_conv_plan_destroy(tmp.inner); return SC_ERR_NULL; }
  *out = bp;
  return SC_OK;
}

sc_status sparse_conv_backward_set_filters(sc_bwd_plan* plan, const void* w_dev, void* hip_stream) {
  if (!plan || !w_dev) return SC_ERR_NULL;
  if ((uintptr_t)w_dev & 15) return SC_ERR_ALIGN;
  if (!plan->inner) return SC_OK;            // only the input gradient uses the filters
  sc_status s = sc::rotate_filters(plan, w_dev, static_cast<hipStream_t>(hip_stream));
  if (s != SC_OK) return s;
  return sparse_conv_plan_set_filters(plan->inner, plan->ws + plan->off_wrot, hip_stream);
}

sc_status sparse_conv_backward_run(const sc_bwd_plan* plan, const void* x_dev, const void* y_dev, const void* dy_dev,
                                   void* dx_dev, float* dw_dev, float* db_dev, void* hip_stream) {
  if (!plan || !dy_dev) return SC_ERR_NULL;
  const sc_conv_desc& d = plan->desc;
  if (d.relu && !y_dev) return SC_ERR_NULL;
  if (dw_dev && !x_dev) return SC_ERR_NULL;
  if (((uintptr_t)dy_dev & 15) || ((uintptr_t)y_dev & 15) || ((uintptr_t)x_dev & 15) || ((uintptr_t)dx_dev & 15) ||
      ((uintptr_t)dw_dev & 15) || ((uintptr_t)db_dev & 3))
    return SC_ERR_ALIGN;
  if (dx_dev && !plan->inner) return SC_ERR_UNSUPPORTED;     // padding larger than the window reach: no input gradient
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  int64_t m = 0, kept = 0; const int32_t* rows_dev = nullptr;
  sc_status s = sparse_conv_plan_info(plan->fwd, &m, &kept, nullptr, nullptr, &rows_dev);
  if (s != SC_OK) return s;
  const uint8_t* mask = sparse_conv_plan_mask(plan->fwd);
  const int dt = d.dtype == SC_BF16 ? sc::kBF16 : sc::kF16;
  const int period = d.mask_mode == SC_MASK_SPATIAL ? plan->ho * plan->wo : 0;
  _Float16* g = reinterpret_cast<_Float16*>(plan->ws + plan->off_g);    // 16-bit patterns; compared as the real type below

  // g map, with the column sums of its slabs on the side
  const int slab_rows = sc::colsum_slab_rows(m);
  const int slabs = (int)((m + slab_rows - 1) / slab_rows);
  float* colsum = reinterpret_cast<float*>(plan->ws + plan->off_colsum);
  if (dt == sc::kBF16)
    hipLaunchKernelGGL(sc::grad_map_kernel<__bf16>, dim3(slabs), dim3(256), 0, stream, (const __bf16*)y_dev,
                       (const __bf16*)dy_dev, mask, (__bf16*)g, m, d.c_out, slab_rows, d.relu, period, colsum);
  else
    hipLaunchKernelGGL(sc::grad_map_kernel<_Float16>, dim3(slabs), dim3(256), 0, stream, (const _Float16*)y_dev,
                       (const _Float16*)dy_dev, mask, g, m, d.c_out, slab_rows, d.relu, period, colsum);
  // db
  if (db_dev)
    hipLaunchKernelGGL(sc::colsum_final_kernel, dim3((d.c_out + 3) / 4), dim3(256), 0, stream, colsum, slabs, d.c_out, db_dev);
  // dw
  if (dw_dev) {
    const int k = d.kh * d.kw * d.c_in;
    const int64_t count = (int64_t)d.c_out * k;
    if (kept == 0) {
      hipLaunchKernelGGL(sc::wgrad_reduce_kernel, dim3((unsigned)((count + 63) / 64)), dim3(256), 0, stream,
                         (const float*)nullptr, 0, count, dw_dev);
    } else {
      sc::WgradParams p;
      std::memset(&p, 0, sizeof(p));
      p.x = x_dev; p.g = g;
      p.row_idx = kept == m ? nullptr : rows_dev;
      p.splits = sc::wgrad_splits(kept, d.c_out, k);
      p.rows = (int32_t)kept;
      p.rows_per_split = (int32_t)(((kept + p.splits - 1) / p.splits + sc::kWgRows - 1) / sc::kWgRows * sc::kWgRows);
      p.splits = (int32_t)((kept + p.rows_per_split - 1) / p.rows_per_split);
      p.out = p.splits == 1 ? dw_dev : reinterpret_cast<float*>(plan->ws + plan->off_partial);
      p.h = d.h; p.w = d.w; p.c_in = d.c_in; p.ho_wo = plan->ho * plan->wo; p.wo = plan->wo; p.c_out = d.c_out;
      p.kh = d.kh; p.kw = d.kw; p.sh = d.stride_h; p.sw = d.stride_w; p.ph = d.pad_h; p.pw = d.pad_w;
      p.dil_h = d.dil_h; p.dil_w = d.dil_w;
      p.k = k;
      sc::magic_div((uint32_t)p.ho_wo, &p.div_howo_mul, &p.div_howo_shift);
      sc::magic_div((uint32_t)p.wo, &p.div_wo_mul, &p.div_wo_shift);
      hipError_t e;
      e = dt == sc::kBF16 ? sc::wgrad_launch<sc::kBF16, 128, 128>(p, stream) : sc::wgrad_launch<sc::kF16, 128, 128>(p, stream);
      if (e != hipSuccess) { sc::note_hip_error((int32_t)e); return SC_ERR_HIP; }
      if (p.splits > 1)
        hipLaunchKernelGGL(sc::wgrad_reduce_kernel, dim3((unsigned)((count + 63) / 64)), dim3(256), 0, stream,
                           (const float*)p.out, p.splits, count, dw_dev);
    }
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { sc::note_hip_error((int32_t)e); return SC_ERR_HIP; }
  // dx: the g map (zero-interleaved for strided layers) through the forward kernels with the rotated filters
  if (dx_dev) {
    const void* src = g;
    if (plan->hu > 0) {
      const int gpr = d.c_out / 8;
      const int64_t groups = m * gpr;
      sc::v4i* gu = reinterpret_cast<sc::v4i*>(plan->ws + plan->off_gup);
      hipLaunchKernelGGL(sc::upsample_rows_kernel<0>, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, stream,
                         reinterpret_cast<const sc::v4i*>(g), gu, groups, gpr, plan->ho * plan->wo, plan->wo, d.stride_h,
                         d.stride_w, plan->hu, plan->wu);
      hipError_t e2 = hipGetLastError();
      if (e2 != hipSuccess) { sc::note_hip_error((int32_t)e2); return SC_ERR_HIP; }
      src = gu;
    }
    return dense_conv_run(plan->inner, src, nullptr, dx_dev, hip_stream);
  }
  return SC_OK;
}

void sparse_conv_backward_destroy(sc_bwd_plan* plan) {
  if (!plan) return;
  sparse_conv_plan_destroy(plan->inner);
  delete plan;
}

}  // extern "C"
