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
// Kernels here: the filter-gradient GEMM on the matrix cores in two 16-bit forms -- operands straight into LDS, dy gated by
// y on the way and db summed from the same tiles (the form that runs wherever the tensors fit 32-bit offsets), and an
// older register-staged form that reads a g map -- and a float form, each with a deterministic second pass over its row splits; the g
// map with its column sums (written only when the input gradient, a convolution of the g map, is asked for); and the
// filter rotation for the input gradient.
#include "../../include/sparse_conv.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <new>

#include "conv_params.hpp"
#include "igemm_buf_kernel.hpp"
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

// ---- filter gradient, second form: operands straight into LDS ---------------------------------------------------
// The kernel above moves every staged row through registers, one stage ahead: a workgroup waits a memory round
// trip per 64 rows.  This form keeps several stages in flight without registers:
//   * a stage = 32 kept rows; its tiles lie in LDS as panels of 32 rows x 128 bytes (64 channels or window entries of
//     a 16-bit type), filled by `buffer_load ... lds` transfers: wavefront w fills rows 8w .. 8w+7 of every panel, lane
//     l the 16-byte group l % 8 of row 8w + l / 8 -- a lane decodes ONE row per stage (from the split's row list, which
//     sits in LDS) and derives every panel's offset from it; an offset past the end of the buffer makes the hardware
//     write zeros, which serves padded taps, absent rows and columns beyond Cout or K;
//   * the upstream gradient is gated on the fly: the tiles of dy and of y arrive side by side, and a lane keeps the
//     elements of its dy fragment whose y is positive (g of Alg. 1's backward, never written to memory); the column sums
//     of the gated fragments are db, accumulated by the wavefronts of the first K tile in a fixed order;
//   * 16-byte groups are placed at (group ^ 2 * (row % 4)), so the four rows x 32 bytes that 16 lanes of a
//     transposing read touch cover all banks once;
//   * ring of STAGES stages; a wavefront waits for "all but the newest STAGES-2 stages of MY transfers have landed",
//     then a barrier, then refills the slot the previous stage left.
//   workgroup = BM output channels x BN window entries x one split of the kept rows; four wavefronts
//   result    = float partial sums per split, [Cout x K] then [Cout] (db); wgrad_reduce_kernel adds the splits
struct Wgrad2Params {
  const void* x;
  const void* dy;            // upstream gradient [M][Cout] (or the g map, with y null)
  const void* y;             // forward output [M][Cout] when the layer has a ReLU, else null
  const int32_t* row_idx;    // kept rows, or null for the identity
  float* out;                // [splits][Cout * K + Cout]
  int64_t split_stride;      // Cout * K + Cout
  int32_t rows, rows_per_split, splits;
  int32_t h, w, c_in, ho_wo, wo, c_out;
  int32_t kh, kw, sh, sw, ph, pw, dil_h, dil_w;
  int32_t k;                 // kh * kw * c_in
  int32_t co_tiles, k_tiles;
  uint32_t div_howo_mul, div_howo_shift, div_wo_mul, div_wo_shift;
  uint32_t x_bytes, dy_bytes;
};

constexpr int kW2Rows = 32;               // kept rows per stage
constexpr int kW2PanelBytes = kW2Rows * 128;
constexpr int kW2MostSplitRows = 2048;    // rows of one split (its row list lies in LDS)

template <int I, int N, class Fn> __device__ __forceinline__ void for_constants(Fn&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    for_constants<I + 1, N>(f);
  }
}
typedef int v2i __attribute__((ext_vector_type(2)));
// An LDS word read the compiler does not see as one (it would wait for every transfer in flight before a read of
// LDS that transfers may write); the value is complete when this returns.
__device__ __forceinline__ int lds_word_now(unsigned addr) {
  int v;
  asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(addr));
  return v;
}
// ds_read_b64_tr_b16: within 16 lanes, result lane j, element t = source lane 4t + j/4, element j%4.  With source
// lane s addressing row s/4, columns 4(s%4) .. +3 of a 4 x 16 block, result lane j holds rows 0..3 of column j.
template <int OFF> __device__ __forceinline__ v2i lds_read_tr(unsigned addr) {
  v2i v;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}
// wait until at most N LDS operations are outstanding; the halves pass through so that no use moves above the wait
template <int N, int CNT> __device__ __forceinline__ void wait_halves(v2i (&h)[CNT]) {
  static_assert((CNT == 8 || CNT == 12 || CNT == 14) && N <= 15, "halves of 4, 6 or 7 fragments; the counter has four bits");
  if constexpr (CNT == 8)
    asm volatile("s_waitcnt lgkmcnt(%8)"
                 : "+v"(h[0]), "+v"(h[1]), "+v"(h[2]), "+v"(h[3]), "+v"(h[4]), "+v"(h[5]), "+v"(h[6]), "+v"(h[7])
                 : "n"(N));
  if constexpr (CNT == 12)
    asm volatile("s_waitcnt lgkmcnt(%12)"
                 : "+v"(h[0]), "+v"(h[1]), "+v"(h[2]), "+v"(h[3]), "+v"(h[4]), "+v"(h[5]), "+v"(h[6]), "+v"(h[7]),
                   "+v"(h[8]), "+v"(h[9]), "+v"(h[10]), "+v"(h[11])
                 : "n"(N));
  if constexpr (CNT == 14)
    asm volatile("s_waitcnt lgkmcnt(%14)"
                 : "+v"(h[0]), "+v"(h[1]), "+v"(h[2]), "+v"(h[3]), "+v"(h[4]), "+v"(h[5]), "+v"(h[6]), "+v"(h[7]),
                   "+v"(h[8]), "+v"(h[9]), "+v"(h[10]), "+v"(h[11]), "+v"(h[12]), "+v"(h[13])
                 : "n"(N));
}

#ifdef SC_TIMING
__device__ long long g_w2_stamps[1024 * 8];       // development builds: per workgroup, clock at the phase boundaries
#define SC_W2_STAMP(slot) do { if (threadIdx.x == 0 && blockIdx.x < 1024) g_w2_stamps[blockIdx.x * 8 + (slot)] = wall_clock64(); } while (0)
#else
#define SC_W2_STAMP(slot) do { } while (0)
#endif

__device__ __forceinline__ void lds_store16(unsigned addr, v4i v) {
  asm volatile("ds_write_b128 %0, %1" ::"v"(addr), "v"(v) : "memory");
}

template <int DT, int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, bool GATE>
__global__ __launch_bounds__(256) void wgrad2_kernel(const Wgrad2Params p) {
  using E = Elem<DT>;
  using T = typename E::T;
  constexpr int R = kW2Rows;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int MI = WM / 32, NI = WN / 32;
  constexpr int GP = BM / 64, AP = BN / 64;                 // panels of the dy (and y) tile, of the window tile
  constexpr int YP0 = GP, AP0 = GATE ? 2 * GP : GP;         // first panel of the y tile, of the window tile
  constexpr int LPT = AP0 + AP;                             // transfers per wavefront and stage
  constexpr int STAGE_BYTES = LPT * kW2PanelBytes;
  constexpr int F = MI + NI;                                // fragments per 16-row step
  static_assert(WAVES_M * WAVES_N == 4 && BM % 64 == 0 && BN % 64 == 0 && WM % 32 == 0 && WN % 32 == 0, "shape");
  static_assert(STAGES >= 3 && (STAGES - 2) * LPT <= 63, "vmcnt is a 6-bit counter");
  static_assert(STAGE_BYTES + 2048 + 512 < 65536, "fragment offsets are immediates");
  static_assert(2 * F <= 15, "LDS reads of one 16-row step in flight: the counter has four bits");
  static_assert(STAGES * STAGE_BYTES >= R * BM * 4, "the ring doubles as scratch of the db sums");
  extern __shared__ __align__(16) unsigned char smem[];
  int32_t* s_rows = reinterpret_cast<int32_t*>(smem + STAGES * STAGE_BYTES);      // [kW2MostSplitRows]

  const int t = threadIdx.x, lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int fp = lane & 31, fh = lane >> 5;
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
  // consecutive workgroup numbers go round the chip's eight dies: renumbered so that the tiles of one split, and
  // neighbouring splits, share a die -- each die's L2 then holds its own eighth of the rows instead of all of them
  const int tiles = p.co_tiles * p.k_tiles;
  const int nwg = tiles * p.splits;
  const int per_xcd = (nwg + 7) >> 3;
  const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (logical >= nwg) return;
  const int split = logical / tiles, tile = logical - split * tiles;
  const int co0 = (tile / p.k_tiles) * BM, k0 = (tile % p.k_tiles) * BN;
  const bool sums_db = tile % p.k_tiles == 0;               // the workgroups of the first K tile also sum db
  const int i_begin = split * p.rows_per_split, i_end = min(p.rows, i_begin + p.rows_per_split);
  const int n_st = (i_end - i_begin + R - 1) / R;
  SC_W2_STAMP(0);

  // the split's row numbers
  if (p.row_idx)
    for (int i = t; i < i_end - i_begin; i += 256) s_rows[i] = p.row_idx[i_begin + i];
  __syncthreads();

  // what this lane transfers: row slot 8 * wave + lane / 8 of every panel, the 16-byte group that lands at
  // position lane % 8 of that row
  const int slot = wave * 8 + (lane >> 3);
  const int lc = (lane & 7) ^ (2 * ((lane >> 3) & 3));      // logical group (8 elements) within a panel row
  int g_col[GP];                                            // element offset of that group in a row of dy, or -1 beyond Cout
#pragma unroll
  for (int q = 0; q < GP; ++q) {
    const int c = co0 + 64 * q + 8 * lc;
    g_col[q] = c < p.c_out ? c : -1;                        // (Cout is a multiple of 8)
  }
  int a_dy[AP], a_dx[AP], a_off[AP];                        // tap displacement and element offset of the group; a_off < 0 beyond K
#pragma unroll
  for (int q = 0; q < AP; ++q) {
    const int kk = k0 + 64 * q + 8 * lc;                    // (Cin is a multiple of 8: a group lies inside one tap)
    const int tap = kk < p.k ? kk / p.c_in : 0, ci = kk - tap * p.c_in;
    const int ky = tap / p.kw, kx = tap - ky * p.kw;
    a_dy[q] = ky * p.dil_h;
    a_dx[q] = kx * p.dil_w;
    a_off[q] = kk < p.k ? (a_dy[q] * p.w + a_dx[q]) * p.c_in + ci : -1;
  }
  const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.x), 0, (int)p.x_bytes, kBufferWord3);
  const __amdgpu_buffer_rsrc_t rdy = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.dy), 0, (int)p.dy_bytes, kBufferWord3);
  const __amdgpu_buffer_rsrc_t ry =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(GATE ? p.y : p.dy), 0, (int)p.dy_bytes, kBufferWord3);
  typedef __attribute__((address_space(3))) void lds_void;
  const unsigned lds0 = (unsigned)(unsigned long long)(__attribute__((address_space(3))) unsigned char*)smem;
  const unsigned rows_addr = lds0 + (unsigned)(STAGES * STAGE_BYTES);

  // the row this lane transfers in stage `st`: decoded once, then one transfer per panel
  bool t_present = false;
  uint32_t t_row_off = 0;
  int t_xrow = 0, t_iy0 = 0, t_ix0 = 0;
  auto prepare_stage = [&](int st) {
    const int i = i_begin + st * R + slot;
    t_present = i < i_end;
    const int r = t_present ? (p.row_idx ? lds_word_now(rows_addr + 4u * (unsigned)(i - i_begin)) : i) : 0;
    t_row_off = (uint32_t)r * (uint32_t)p.c_out;
    const int n = fast_div(r, p.div_howo_mul, p.div_howo_shift), rem = r - n * p.ho_wo;
    const int oy = fast_div(rem, p.div_wo_mul, p.div_wo_shift), ox = rem - oy * p.wo;
    t_iy0 = oy * p.sh - p.ph;
    t_ix0 = ox * p.sw - p.pw;
    t_xrow = ((n * p.h + t_iy0) * p.w + t_ix0) * p.c_in;              // may be negative: used with in-range taps only
  };
  // transfer `IDX` of the prepared stage into ring slot `ring`: the dy panels (each followed by its y panel), then the
  // window panels
  auto issue_one = [&](auto idx_c, int ring) {
    constexpr int IDX = decltype(idx_c)::value;
    unsigned char* base = smem + ring * STAGE_BYTES + wave * 1024;      // this wavefront's 8 rows of panel 0
    if constexpr (IDX < AP0) {
      constexpr int q = GATE ? IDX / 2 : IDX;
      constexpr bool is_y = GATE && (IDX & 1);
      const bool ok = t_present & (g_col[q] >= 0);          // (bitwise: one transfer instruction, no branch around it)
      const uint32_t voff = ok ? (t_row_off + (uint32_t)g_col[q]) * 2u : kOutOfRange;
      if constexpr (is_y) __builtin_amdgcn_raw_ptr_buffer_load_lds(ry, (lds_void*)(base + (YP0 + q) * kW2PanelBytes), 16, voff, 0, 0, 0);
      else __builtin_amdgcn_raw_ptr_buffer_load_lds(rdy, (lds_void*)(base + q * kW2PanelBytes), 16, voff, 0, 0, 0);
    } else {
      constexpr int q = IDX - AP0;
      const bool ok = t_present & (a_off[q] >= 0) & ((unsigned)(t_iy0 + a_dy[q]) < (unsigned)p.h) &
                      ((unsigned)(t_ix0 + a_dx[q]) < (unsigned)p.w);
      const uint32_t voff = ok ? (uint32_t)(t_xrow + a_off[q]) * 2u : kOutOfRange;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (lds_void*)(base + (AP0 + q) * kW2PanelBytes), 16, voff, 0, 0, 0);
    }
  };
  auto issue_stage = [&](int st, int ring) {
    prepare_stage(st);
    for_constants<0, LPT>([&](auto idx_c) { issue_one(idx_c, ring); });
  };

  floatx16 acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;
  float dbsum[GP][8];                   // this lane's groups of dy (one per panel), summed over its rows of every stage
#pragma unroll
  for (int q = 0; q < GP; ++q)
#pragma unroll
    for (int j = 0; j < 8; ++j) dbsum[q][j] = 0.0f;

  // A lane's own groups of a stage, once they have landed and before anybody reads fragments: the group of dy keeps
  // the elements whose y is positive (written back in place: the fragments below are fragments of g), and in the
  // workgroups of the first K tile the lane adds the group to its db sums.  No other lane touches these 16 bytes
  // before the barrier that follows.
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  constexpr int OWN = GATE ? 2 * GP : GP;
  static_assert(GP <= 2, "one or two panels of output channels");
  const bool owns = GATE || sums_db;
  v4i own[OWN];                        // the groups of dy, then those of y; the reads write these registers when they complete
  unsigned own_at = 0;
  auto own_read = [&](unsigned ring_off) {
    if (!owns) return;
    own_at = lds0 + ring_off + (unsigned)t * 16u;
    own[0] = lds_read16_at<0>(own_at);
    if constexpr (GP == 2) own[1] = lds_read16_at<kW2PanelBytes>(own_at);
    if constexpr (GATE) {
      own[GP] = lds_read16_at<YP0 * kW2PanelBytes>(own_at);
      if constexpr (GP == 2) own[GP + 1] = lds_read16_at<(YP0 + 1) * kW2PanelBytes>(own_at);
    }
  };
  auto own_finish = [&]() {
    if (!owns) return;
    wait_frags<0>(own);
#pragma unroll
    for (int q = 0; q < GP; ++q) {
      v4i gq = own[q];
      if constexpr (GATE) {
        const s16x8 keep = __builtin_bit_cast(s16x8, own[GP + q]) > (short)0;    // y > 0 for both 16-bit float types
        gq = __builtin_bit_cast(v4i, __builtin_bit_cast(s16x8, gq) & keep);
        lds_store16(own_at + q * kW2PanelBytes, gq);
      }
      if (sums_db) {
        struct alignas(16) Grp { T v[8]; };
        const Grp gr = __builtin_bit_cast(Grp, gq);
#pragma unroll
        for (int j = 0; j < 8; ++j) dbsum[q][j] += (float)gr.v[j];
      }
    }
  };

  // fragment addresses in ring slot 0, 16-row step 0: the lane addresses row 8 * fh + (lane % 16) / 4 (the second
  // read 4 rows further), columns 16 * ((lane % 32) / 16) + 4 * (lane % 4) .. +3 of its 32-column block
  const int l16 = lane & 15;
  const int frow = 8 * fh + (l16 >> 2), fswz = 2 * (l16 >> 2);
  auto frag_addr = [&](int col) -> unsigned {              // col: column within the tile (multiple of 4)
    const int panel = col >> 6, cin = col & 63;
    return lds0 + (unsigned)(panel * kW2PanelBytes + frow * 128 + (((cin >> 3) ^ fswz) << 4) + (cin & 7) * 2);
  };
  unsigned g_addr[MI], a_addr[NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) g_addr[mi] = frag_addr(wm0 + 32 * mi + 16 * ((lane & 31) >> 4) + 4 * (l16 & 3));
#pragma unroll
  for (int ni = 0; ni < NI; ++ni)
    a_addr[ni] = frag_addr(wn0 + 32 * ni + 16 * ((lane & 31) >> 4) + 4 * (l16 & 3)) + AP0 * kW2PanelBytes;

  auto read_step = [&](unsigned ring_off, auto ks_c, v2i (&h)[2 * F]) {
    constexpr int KO = decltype(ks_c)::value * 16 * 128;
    int at = 0;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      h[at++] = lds_read_tr<KO>(g_addr[mi] + ring_off);
      h[at++] = lds_read_tr<KO + 512>(g_addr[mi] + ring_off);
    }
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
      h[at++] = lds_read_tr<KO>(a_addr[ni] + ring_off);
      h[at++] = lds_read_tr<KO + 512>(a_addr[ni] + ring_off);
    }
  };
  // The MFMAs of one 16-row step with one side job issued behind each: the transfers of the stage that enters the
  // ring (a wavefront that issues them back to back sits in the issue stage while the address unit takes them; behind
  // an MFMA the slot is free), then the lane's own groups of the next stage.  JOB0 = number of the first side job.
  constexpr int JOBS = LPT + 2;
  static_assert(JOBS <= 2 * MI * NI, "a slot behind an MFMA for every side job");
  static_assert(LPT >= MI * NI || 2 * F + OWN <= 15, "own-group reads issued while a step's fragment reads are in flight");
  auto mma_step = [&](const v2i (&h)[2 * F], auto job0_c, int fill_ring, bool fill, unsigned next_off, bool next) {
    constexpr int JOB0 = decltype(job0_c)::value;
    v4i gf[MI], af[NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) gf[mi] = v4i{h[2 * mi][0], h[2 * mi][1], h[2 * mi + 1][0], h[2 * mi + 1][1]};
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
      af[ni] = v4i{h[2 * MI + 2 * ni][0], h[2 * MI + 2 * ni][1], h[2 * MI + 2 * ni + 1][0], h[2 * MI + 2 * ni + 1][1]};
    for_constants<0, MI * NI>([&](auto i_c) {
      constexpr int I = decltype(i_c)::value;
      constexpr int mi = I / NI, ni = I % NI;
      E::mma(acc[mi][ni], gf[mi], af[ni]);
      constexpr int JOB = JOB0 + I;
      if constexpr (JOB < JOBS) {
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (JOB < LPT) { if (fill) issue_one(std::integral_constant<int, JOB>{}, fill_ring); }
        if constexpr (JOB == LPT) { if (next) own_read(next_off); }
        if constexpr (JOB == LPT + 1) { if (next) own_finish(); }
        __builtin_amdgcn_sched_barrier(0);
      }
    });
  };

  SC_W2_STAMP(1);
#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s)
    if (s < n_st) issue_stage(s, s);
  // Step st: my transfers of stage st + 1 have landed (so have those of stage st); barrier -- stage st is complete
  // and gated for everybody, and everybody has left stage st - 1, whose slot the stage st + STAGES - 1 now takes;
  // fragments and MFMAs of stage st, with the side jobs behind them.
  if (n_st > 0) {
    if (STAGES - 2 < n_st) wait_vmcnt<(STAGES - 2) * LPT>();
    else wait_vmcnt<0>();
    own_read(0);
    own_finish();
  }
  int ring = 0;
  for (int st = 0; st < n_st; ++st) {
    if (st + STAGES - 2 < n_st) wait_vmcnt<(STAGES - 3) * LPT>();
    else wait_vmcnt<0>();
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // my gated groups of stage st are written
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    const unsigned ring_off = (unsigned)(ring * STAGE_BYTES);
    const int next_ring = ring + 1 == STAGES ? 0 : ring + 1;
    const bool fill = st + STAGES - 1 < n_st, next = st + 1 < n_st;
    if (fill) prepare_stage(st + STAGES - 1);
    v2i h0[2 * F], h1[2 * F];          // (one step's reads in flight at a time: two would overrun the counter)
    read_step(ring_off, std::integral_constant<int, 0>{}, h0);
    wait_halves<0>(h0);
    read_step(ring_off, std::integral_constant<int, 1>{}, h1);     // lands under the MFMAs of step 0
    mma_step(h0, std::integral_constant<int, 0>{}, ring == 0 ? STAGES - 1 : ring - 1, fill, (unsigned)(next_ring * STAGE_BYTES), next);
    wait_halves<0>(h1);
    mma_step(h1, std::integral_constant<int, MI * NI>{}, ring == 0 ? STAGES - 1 : ring - 1, fill, (unsigned)(next_ring * STAGE_BYTES), next);
    ring = next_ring;
  }

  SC_W2_STAMP(2);
  // MFMA result row 8j + 4h + i sits in register 4j + i of lane half h; column = lane % 32
  float* __restrict__ out = p.out + (int64_t)split * p.split_stride;
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
      const int kcol = k0 + wn0 + 32 * ni + fp;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int co = co0 + wm0 + 32 * mi + 8 * (v >> 2) + 4 * fh + (v & 3);
        if (co < p.c_out && kcol < p.k) out[(int64_t)co * p.k + kcol] = acc[mi][ni][v];
      }
    }
  if (sums_db) {      // the 32 row slots of every channel, added in slot order through LDS (the ring is free now)
    __syncthreads();
    float* s_db = reinterpret_cast<float*>(smem);          // [32 row slots][BM channels]
#pragma unroll
    for (int q = 0; q < GP; ++q)
#pragma unroll
      for (int j = 0; j < 8; ++j) s_db[slot * BM + 64 * q + 8 * lc + j] = dbsum[q][j];
    __syncthreads();
    if (t < BM && co0 + t < p.c_out) {
      float tot = 0.0f;
      for (int r = 0; r < R; ++r) tot += s_db[r * BM + t];
      out[(int64_t)p.c_out * p.k + co0 + t] = tot;
    }
  }
  SC_W2_STAMP(3);
}

template <int DT, int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, bool GATE>
static hipError_t wgrad2_launch(Wgrad2Params p, hipStream_t stream) {
  constexpr size_t lds = (size_t)STAGES * ((GATE ? 2 : 1) * (BM / 64) + BN / 64) * kW2PanelBytes + kW2MostSplitRows * 4;
  static_assert(lds <= 160 * 1024, "LDS of a compute unit");
  p.co_tiles = (p.c_out + BM - 1) / BM;
  p.k_tiles = (p.k + BN - 1) / BN;
  const unsigned grid = (unsigned)((p.co_tiles * p.k_tiles * p.splits + 7) / 8 * 8);
  static std::atomic<bool> attr_set{false};                       // (one flag per instantiation)
  if (lds > 64 * 1024 && !attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(wgrad2_kernel<DT, BM, BN, WAVES_M, WAVES_N, STAGES, GATE>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((wgrad2_kernel<DT, BM, BN, WAVES_M, WAVES_N, STAGES, GATE>), dim3(grid), dim3(256), lds, stream, p);
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

// The same for the partial results of wgrad2_kernel: per split Cout * K filter-gradient sums, then Cout bias-gradient
// sums (`stride` floats in all); dw and db may each be null.
__global__ __launch_bounds__(256) void wgrad2_reduce_kernel(const float* __restrict__ partial, int splits, int64_t stride,
                                                            int64_t count_dw, float* __restrict__ dw, float* __restrict__ db) {
  __shared__ v4f s_sub[16][17];
  const int e = threadIdx.x & 15, sl = threadIdx.x >> 4;
  const int64_t i = ((int64_t)blockIdx.x * 16 + e) * 4;
  v4f acc = {0.0f, 0.0f, 0.0f, 0.0f};
  if (i < stride)
    for (int s = sl; s < splits; s += 16) {
      const v4f v = *reinterpret_cast<const v4f*>(partial + (int64_t)s * stride + i);
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] += v[j];
    }
  s_sub[sl][e] = acc;
  __syncthreads();
  if (threadIdx.x < 16 && i < stride) {
    v4f tot = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int l = 0; l < 16; ++l)
#pragma unroll
      for (int j = 0; j < 4; ++j) tot[j] += s_sub[l][threadIdx.x][j];
    if (i < count_dw) {
      if (dw) *reinterpret_cast<v4f*>(dw + i) = tot;
    } else if (db) {
      *reinterpret_cast<v4f*>(db + (i - count_dw)) = tot;
    }
  }
}

// ---- filter gradient in float (the paper's arithmetic: App. A works on floats) -----------------------------------
// The 32 x 32 x 2 float MFMA takes, per lane, ONE element of each operand: row (lane % 32) of its 32-wide block and
// contraction entry lane / 32.  With the contraction over kept rows that is element [row 2s + lane / 32][column
// lane % 32] of a row-major tile -- no transposition, plain 4-byte LDS reads; rows lie 96 floats apart so that
// the two rows of a step fall into different halves of the banks.
//   workgroup = 64 output channels x 64 window entries x one split of the kept rows; 2 x 2 wavefronts of 32 x 32
//   stage     = 32 kept rows; a thread stages one column of both tiles for every fourth row, the next stage's values
//               are fetched into registers before the MFMAs of the current one
//   result    = float partial sums per split; wgrad_reduce_kernel adds the splits in order
constexpr int kWfRows = 32, kWfPitch = 96, kWfTile = 64;
__global__ __launch_bounds__(256) void wgrad_f32_kernel(const WgradParams p) {
  __shared__ float s_g[kWfRows * kWfPitch], s_a[kWfRows * kWfPitch];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int fp = lane & 31, fh = lane >> 5;
  const int wm0 = (wave >> 1) * 32, wn0 = (wave & 1) * 32;
  const int tiles = p.co_tiles * p.k_tiles;
  const int split = blockIdx.x / tiles, tile = blockIdx.x - split * tiles;
  const int co0 = (tile / p.k_tiles) * kWfTile, k0 = (tile % p.k_tiles) * kWfTile;
  const int i_begin = split * p.rows_per_split, i_end = min(p.rows, i_begin + p.rows_per_split);
  const int n_st = (i_end - i_begin + kWfRows - 1) / kWfRows;
  const float* __restrict__ xg = static_cast<const float*>(p.x);
  const float* __restrict__ gg = static_cast<const float*>(p.g);

  // this thread's column of both tiles: output channel co, window entry kcol = (tap, ci)
  const int col = t & 63, r0 = t >> 6;
  const int co = co0 + col, kcol = k0 + col;
  const bool co_ok = co < p.c_out, k_ok = kcol < p.k;
  const int tap = k_ok ? kcol / p.c_in : 0, ci = kcol - tap * p.c_in;
  const int ky = tap / p.kw, kx = tap - ky * p.kw;
  const int tdy = ky * p.dil_h, tdx = kx * p.dil_w;
  float gv[8], av[8];
  auto fetch = [&](int st) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int i = i_begin + st * kWfRows + r0 + 4 * j;
      gv[j] = 0.0f;
      av[j] = 0.0f;
      if (i < i_end) {
        const int r = p.row_idx ? p.row_idx[i] : i;
        if (co_ok) gv[j] = gg[(int64_t)r * p.c_out + co];
        const int n = fast_div(r, p.div_howo_mul, p.div_howo_shift), rem = r - n * p.ho_wo;
        const int oy = fast_div(rem, p.div_wo_mul, p.div_wo_shift), ox = rem - oy * p.wo;
        const int iy = oy * p.sh - p.ph + tdy, ix = ox * p.sw - p.pw + tdx;
        if (k_ok && (unsigned)iy < (unsigned)p.h && (unsigned)ix < (unsigned)p.w)
          av[j] = xg[(((int64_t)n * p.h + iy) * p.w + ix) * p.c_in + ci];
      }
    }
  };
  floatx16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
  if (n_st > 0) fetch(0);
  for (int st = 0; st < n_st; ++st) {
    __syncthreads();                                   // everybody has read the previous stage
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      s_g[(r0 + 4 * j) * kWfPitch + col] = gv[j];
      s_a[(r0 + 4 * j) * kWfPitch + col] = av[j];
    }
    __syncthreads();
    if (st + 1 < n_st) fetch(st + 1);                  // in flight under the MFMAs below
#pragma unroll
    for (int s2 = 0; s2 < kWfRows / 2; ++s2) {
      const float a = s_g[(2 * s2 + fh) * kWfPitch + wm0 + fp];
      const float b = s_a[(2 * s2 + fh) * kWfPitch + wn0 + fp];
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
    }
  }
  // MFMA result row 8j + 4h + i sits in register 4j + i of lane half h; column = lane % 32
  float* __restrict__ out = p.out + (int64_t)split * p.c_out * p.k;
  const int kc = k0 + wn0 + fp;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int c = co0 + wm0 + 8 * (v >> 2) + 4 * fh + (v & 3);
    if (c < p.c_out && kc < p.k) out[(int64_t)c * p.k + kc] = acc[v];
  }
}

// rows per split of the float kernel: about three workgroups per compute unit, at least eight stages per split
static int wgrad_f32_splits(int64_t rows, int c_out, int k) {
  const int64_t tiles = (int64_t)((c_out + kWfTile - 1) / kWfTile) * ((k + kWfTile - 1) / kWfTile);
  int64_t want = (768 + tiles - 1) / tiles;
  want = std::min<int64_t>(want, (rows + 8 * kWfRows - 1) / (8 * kWfRows));
  want = std::min<int64_t>(want, (int64_t)(((size_t)64 << 20) / ((size_t)c_out * k * 4)));
  return (int)std::max<int64_t>(want, 1);
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

// Row splits of wgrad2_kernel: one workgroup per compute unit for the 128-channel tile (its LDS admits no second one), two
// for the 64-channel tile (ring of three stages, 80 KB: the kernel spends its time issuing instructions -- row decode, gate,
// db sums -- with one wavefront per SIMD, and a second workgroup fills the gaps: benchmark layer 26.4 -> 22.8 us), every
// split's row list within kW2MostSplitRows, the partial sums within kWgradPartialBytes.  0 = the layer does not fit (the
// first form runs).
constexpr int kW2Workgroups = 256;
static int wgrad2_tile_m(int c_out) { return c_out <= 64 ? 64 : 128; }
static int wgrad2_tile_n(int, bool) { return 256; }
static int wgrad2_splits(int64_t rows, int c_out, int k, bool gate) {
  const int bm = wgrad2_tile_m(c_out), bn = wgrad2_tile_n(c_out, gate);
  const int64_t tiles = (int64_t)((c_out + bm - 1) / bm) * ((k + bn - 1) / bn);
  int64_t want = std::max<int64_t>((bm == 64 ? 2 : 1) * kW2Workgroups / tiles, 1);
  want = std::min<int64_t>(want, (rows + 4 * kW2Rows - 1) / (4 * kW2Rows));      // at least four stages per split
  want = std::max<int64_t>(want, (rows + kW2MostSplitRows - 1) / kW2MostSplitRows);
  want = std::max<int64_t>(want, 1);
  if ((size_t)want * ((size_t)c_out * k + c_out) * 4 > kWgradPartialBytes) return 0;
  return (int)want;
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
  // the 16-bit filter-gradient kernels gather 16-byte channel groups, and the g map is written in groups of eight channels
  if (d->groups != 1 || d->layout != SC_NHWC || (d->dtype != SC_BF16 && d->dtype != SC_F16 && d->dtype != SC_F32) ||
      d->c_in % 8 != 0 || d->c_out % 8 != 0)
    return SC_ERR_UNSUPPORTED;
  const size_t eb = d->dtype == SC_F32 ? 4 : 2;
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
  // (the dense row count bounds every mask's; both forms of the kernel fit)
  off = align_up(off + std::max(std::max((size_t)wgrad_splits(*m, d->c_out, (int)k), (size_t)wgrad_f32_splits(*m, d->c_out, (int)k)) * d->c_out * k * 4,
                                (size_t)wgrad2_splits(*m, d->c_out, (int)k, d->relu != 0) * ((size_t)d->c_out * k + d->c_out) * 4), 256);
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
  if (d.dtype == SC_F32)
    hipLaunchKernelGGL(rotate_filters_kernel<float>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                       (const float*)w_dev, (float*)(bp->ws + bp->off_wrot), d.c_out, d.c_in, d.kh, d.kw);
  else   // 16-bit patterns are moved verbatim
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
      hipError_t e = hipMemsetAsync(tmp.ws + tmp.off_gup, 0, (size_t)desc->n * tmp.hu * tmp.wu * desc->c_out * (desc->dtype == SC_F32 ? 4 : 2), stream);
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
  const int dt = d.dtype == SC_BF16 ? sc::kBF16 : d.dtype == SC_F16 ? sc::kF16 : sc::kF32;
  const int period = d.mask_mode == SC_MASK_SPATIAL ? plan->ho * plan->wo : 0;
  _Float16* g = reinterpret_cast<_Float16*>(plan->ws + plan->off_g);    // 16-bit patterns; compared as the real type below

  if (dt == sc::kF32) {
    // float layers: g map with its slab sums, column sums, the float filter-gradient kernel and its reduction
    float* gf = reinterpret_cast<float*>(plan->ws + plan->off_g);
    const int slab_rows = sc::colsum_slab_rows(m);
    const int slabs = (int)((m + slab_rows - 1) / slab_rows);
    float* colsum = reinterpret_cast<float*>(plan->ws + plan->off_colsum);
    hipLaunchKernelGGL(sc::grad_map_kernel<float>, dim3(slabs), dim3(256), 0, stream, (const float*)y_dev, (const float*)dy_dev,
                       mask, gf, m, d.c_out, slab_rows, d.relu, period, colsum);
    if (db_dev)
      hipLaunchKernelGGL(sc::colsum_final_kernel, dim3((d.c_out + 3) / 4), dim3(256), 0, stream, colsum, slabs, d.c_out, db_dev);
    if (dw_dev) {
      const int k = d.kh * d.kw * d.c_in;
      const int64_t count = (int64_t)d.c_out * k;
      sc::WgradParams p;
      std::memset(&p, 0, sizeof(p));
      p.x = x_dev; p.g = gf;
      p.row_idx = kept == m ? nullptr : rows_dev;
      p.rows = (int32_t)kept;
      p.splits = kept > 0 ? sc::wgrad_f32_splits(kept, d.c_out, k) : 0;
      if (p.splits > 0) {
        p.rows_per_split = (int32_t)(((kept + p.splits - 1) / p.splits + sc::kWfRows - 1) / sc::kWfRows * sc::kWfRows);
        p.splits = (int32_t)((kept + p.rows_per_split - 1) / p.rows_per_split);
        p.out = reinterpret_cast<float*>(plan->ws + plan->off_partial);
        p.h = d.h; p.w = d.w; p.c_in = d.c_in; p.ho_wo = plan->ho * plan->wo; p.wo = plan->wo; p.c_out = d.c_out;
        p.kh = d.kh; p.kw = d.kw; p.sh = d.stride_h; p.sw = d.stride_w; p.ph = d.pad_h; p.pw = d.pad_w;
        p.dil_h = d.dil_h; p.dil_w = d.dil_w;
        p.k = k;
        p.co_tiles = (d.c_out + sc::kWfTile - 1) / sc::kWfTile;
        p.k_tiles = (k + sc::kWfTile - 1) / sc::kWfTile;
        sc::magic_div((uint32_t)p.ho_wo, &p.div_howo_mul, &p.div_howo_shift);
        sc::magic_div((uint32_t)p.wo, &p.div_wo_mul, &p.div_wo_shift);
        hipLaunchKernelGGL(sc::wgrad_f32_kernel, dim3((unsigned)(p.co_tiles * p.k_tiles * p.splits)), dim3(256), 0, stream, p);
      }
      // (no kept row: zero splits, the reduction writes zeros)
      hipLaunchKernelGGL(sc::wgrad_reduce_kernel, dim3((unsigned)((count + 63) / 64)), dim3(256), 0, stream,
                         (const float*)p.out, p.splits, count, dw_dev);
    }
    hipError_t ef = hipGetLastError();
    if (ef != hipSuccess) { sc::note_hip_error((int32_t)ef); return SC_ERR_HIP; }
    if (dx_dev) {
      const void* src = gf;
      if (plan->hu > 0) {
        const int gpr = d.c_out / 4;
        const int64_t groups = m * gpr;
        sc::v4i* gu = reinterpret_cast<sc::v4i*>(plan->ws + plan->off_gup);
        hipLaunchKernelGGL(sc::upsample_rows_kernel<0>, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, stream,
                           reinterpret_cast<const sc::v4i*>(gf), gu, groups, gpr, plan->ho * plan->wo, plan->wo, d.stride_h,
                           d.stride_w, plan->hu, plan->wu);
        hipError_t e2 = hipGetLastError();
        if (e2 != hipSuccess) { sc::note_hip_error((int32_t)e2); return SC_ERR_HIP; }
        src = gu;
      }
      return dense_conv_run(plan->inner, src, nullptr, dx_dev, hip_stream);
    }
    return SC_OK;
  }

  // Which form of the filter-gradient kernel: the LDS-direct one wherever the tensors fit 32-bit buffer offsets and
  // the splits fit the workspace.  It gates dy itself and sums db on the way, so the g map is written only when the
  // input gradient (a convolution of the g map) is asked for.
  const int k = d.kh * d.kw * d.c_in;
  const int64_t count = (int64_t)d.c_out * k;
  const uint64_t x_bytes = (uint64_t)d.n * d.h * d.w * d.c_in * 2, dy_bytes = (uint64_t)m * d.c_out * 2;
  const bool fits = dw_dev && kept > 0 && x_bytes < (1ull << 31) && dy_bytes < (1ull << 31);
  // (the splits do not depend on whether dx is asked for: dw and db come out bit-identical either way)
  const int splits2 = fits ? sc::wgrad2_splits(kept, d.c_out, k, d.relu != 0) : 0;
  const bool direct = splits2 > 0;
  const bool want_g = dx_dev || !direct;

  // g map, with the column sums of its slabs on the side
  const int slab_rows = sc::colsum_slab_rows(m);
  const int slabs = (int)((m + slab_rows - 1) / slab_rows);
  float* colsum = reinterpret_cast<float*>(plan->ws + plan->off_colsum);
  if (want_g) {
    if (dt == sc::kBF16)
      hipLaunchKernelGGL(sc::grad_map_kernel<__bf16>, dim3(slabs), dim3(256), 0, stream, (const __bf16*)y_dev,
                         (const __bf16*)dy_dev, mask, (__bf16*)g, m, d.c_out, slab_rows, d.relu, period, colsum);
    else
      hipLaunchKernelGGL(sc::grad_map_kernel<_Float16>, dim3(slabs), dim3(256), 0, stream, (const _Float16*)y_dev,
                         (const _Float16*)dy_dev, mask, g, m, d.c_out, slab_rows, d.relu, period, colsum);
  }
  if (direct) {
    sc::Wgrad2Params p;
    std::memset(&p, 0, sizeof(p));
    p.x = x_dev;
    const bool gate = !want_g && d.relu;            // with a g map at hand the kernel reads that, ungated
    p.dy = want_g ? (const void*)g : dy_dev;
    p.y = gate ? y_dev : nullptr;
    p.row_idx = kept == m ? nullptr : rows_dev;
    p.rows = (int32_t)kept;
    p.rows_per_split = (int32_t)(((kept + splits2 - 1) / splits2 + sc::kW2Rows - 1) / sc::kW2Rows * sc::kW2Rows);
    p.splits = (int32_t)((kept + p.rows_per_split - 1) / p.rows_per_split);
    p.split_stride = count + d.c_out;
    p.out = reinterpret_cast<float*>(plan->ws + plan->off_partial);
    p.h = d.h; p.w = d.w; p.c_in = d.c_in; p.ho_wo = plan->ho * plan->wo; p.wo = plan->wo; p.c_out = d.c_out;
    p.kh = d.kh; p.kw = d.kw; p.sh = d.stride_h; p.sw = d.stride_w; p.ph = d.pad_h; p.pw = d.pad_w;
    p.dil_h = d.dil_h; p.dil_w = d.dil_w;
    p.k = k;
    p.x_bytes = (uint32_t)x_bytes; p.dy_bytes = (uint32_t)dy_bytes;
    sc::magic_div((uint32_t)p.ho_wo, &p.div_howo_mul, &p.div_howo_shift);
    sc::magic_div((uint32_t)p.wo, &p.div_wo_mul, &p.div_wo_shift);
    hipError_t e;
    const bool narrow = sc::wgrad2_tile_m(d.c_out) == 64;
    if (dt == sc::kBF16) {
      if (narrow) e = gate ? sc::wgrad2_launch<sc::kBF16, 64, 256, 1, 4, 3, true>(p, stream) : sc::wgrad2_launch<sc::kBF16, 64, 256, 1, 4, 3, false>(p, stream);
      else e = gate ? sc::wgrad2_launch<sc::kBF16, 128, 256, 2, 2, 4, true>(p, stream) : sc::wgrad2_launch<sc::kBF16, 128, 256, 2, 2, 5, false>(p, stream);
    } else {
      if (narrow) e = gate ? sc::wgrad2_launch<sc::kF16, 64, 256, 1, 4, 3, true>(p, stream) : sc::wgrad2_launch<sc::kF16, 64, 256, 1, 4, 3, false>(p, stream);
      else e = gate ? sc::wgrad2_launch<sc::kF16, 128, 256, 2, 2, 4, true>(p, stream) : sc::wgrad2_launch<sc::kF16, 128, 256, 2, 2, 5, false>(p, stream);
    }
    if (e != hipSuccess) { sc::note_hip_error((int32_t)e); return SC_ERR_HIP; }
    hipLaunchKernelGGL(sc::wgrad2_reduce_kernel, dim3((unsigned)((p.split_stride / 4 + 15) / 16)), dim3(256), 0, stream,
                       (const float*)p.out, p.splits, p.split_stride, count, dw_dev, db_dev);
  } else {
    // db
    if (db_dev)
      hipLaunchKernelGGL(sc::colsum_final_kernel, dim3((d.c_out + 3) / 4), dim3(256), 0, stream, colsum, slabs, d.c_out, db_dev);
    // dw
    if (dw_dev) {
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

#ifdef SC_TIMING
sc_status sc_debug_w2_stamps(long long* out_host) {
  return hipMemcpyFromSymbol(out_host, HIP_SYMBOL(sc::g_w2_stamps), sizeof(long long) * 1024 * 8) == hipSuccess ? SC_OK : SC_ERR_HIP;
}
#endif

void sparse_conv_backward_destroy(sc_bwd_plan* plan) {
  if (!plan) return;
  sparse_conv_plan_destroy(plan->inner);
  delete plan;
}

}  // extern "C"
