// Fused masked-convolution kernel for gfx950: implicit lowering of the kept rows
// (paper Sec. 3.2 stage i), matrix-core contraction on the compacted row dimension
// (stage ii) and placement into the dense output with zero fill (stage iii; App. A, Alg. 2),
// in one launch.
//
// Work decomposition
//   workgroup = BM kept rows x BN output channels, 256 threads = 4 wavefronts of 64 lanes
//   arranged WAVES_M x WAVES_N; every wavefront owns (BM/WAVES_M) x (BN/WAVES_N) outputs as
//   32x32 MFMA blocks.  K advances in tiles of 128 bytes per row.
//
// Operand orientation
//   The MFMA computes D = Wt * Xt with filters as the row operand and window entries as the
//   column operand, so a lane ends up holding 16 output channels of ONE output position.
//   Filter rows are stored pre-permuted (see pack kernel) such that those 16 channels are
//   consecutive: lane (p, h) register v  <->  position p, channel 16*h + v of the 32-block.
//   The store of a kept row is then 16 consecutive channels per lane.
//
// LDS layout
//   A tile [BM][128 B] and B tile [BN][128 B], double buffered; the eight 16-byte groups of
//   a row are XOR-swizzled with ((row >> 1) & 7): LDS has 64 banks, odd and even 128-byte rows
//   sit in different bank halves, so the 128-bit reads of sixteen consecutive rows hit sixteen
//   distinct 16-byte bank groups.
#pragma once
#include "conv_params.hpp"
#include "mma_common.hpp"
#include "igemm_dma_kernel.hpp"

namespace sc {

template <int BM, int BN>
constexpr size_t igemm_lds_bytes() { return 2 * (size_t)(BM + BN) * kRowBytes + BM * sizeof(int32_t); }

// GATHER: 0 = element by element (any layout), 1 = 16-byte channel groups (NHWC, Cin*eb % 16 == 0),
// 2 = window-row segments of a zero-margined NHWC copy of the input (small Cin, 16-bit types).
template <int DT, int BM, int BN, int WAVES_M, int WAVES_N, int GATHER, int DEPTH>
__global__ __launch_bounds__(kThreads) void igemm_kernel(const ConvParams p) {
  constexpr bool VEC = GATHER == 1;
  constexpr bool ROWSEG = GATHER == 2;
  using E = Elem<DT>;
  using T = typename E::T;
  constexpr int V = E::V;
  constexpr int EB = sizeof(T);
  constexpr int BK = 8 * V;  // K entries per tile (128 bytes)
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int MI = WM / 32, NI = WN / 32;
  constexpr int A_LOADS = BM / 32, B_LOADS = BN / 32;
  static_assert(WAVES_M * WAVES_N * 64 == kThreads, "four wavefronts");
  static_assert(WM % 32 == 0 && WN % 32 == 0, "32x32 MFMA blocks");

  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* s_a = smem;                              // [2][BM][128]
  unsigned char* s_b = smem + 2 * BM * kRowBytes;         // [2][BN][128]
  int32_t* s_rows = reinterpret_cast<int32_t*>(smem + 2 * (BM + BN) * kRowBytes);  // [BM]

  // Workgroup -> tile.  Consecutive workgroup ids land on different XCDs (8 per device); give
  // each XCD one contiguous run of tiles so neighbouring windows share that XCD's L2.
  const int nwg = p.m_tiles * p.n_tiles;
  const int per_xcd = (nwg + 7) >> 3;
  const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (logical >= nwg) return;
  const int tile_m = logical / p.n_tiles;
  const int tile_n = logical - tile_m * p.n_tiles;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;

  const T* __restrict__ x = static_cast<const T*>(p.x);
  T* __restrict__ y = static_cast<T*>(p.y);

  // ---- per-thread gather state: the rows this thread stages, fixed for the whole K loop -------
  const int c16 = t & 7;      // which 16-byte group of the 128-byte K tile
  const int lrow = t >> 3;    // 0..31
  int32_t a_base[A_LOADS], a_iy0[A_LOADS], a_ix0[A_LOADS];
#pragma unroll
  for (int j = 0; j < A_LOADS; ++j) {
    const int ic = m0 + lrow + 32 * j;
    int rr = -1;
    if (ic < p.rows) rr = p.row_idx ? p.row_idx[ic] : ic;
    int code = (rr >= 0 && p.y_compact) ? ic : rr;                // row the epilogue stores to
    if (p.masked_store && rr >= 0) {
      const int mr = p.mask_spatial ? rr - fast_div(rr, p.div_howo_mul, p.div_howo_shift) * p.ho_wo : rr;
      if (p.mask[mr] == 0) code = dropped_row_code(rr);
    }
    s_rows[lrow + 32 * j] = code;                                 // (eight threads write the same value)
    if (rr >= 0 && p.x_compact) rr = ic;                          // row the window is read from
    if (rr >= 0) {
      int n = fast_div(rr, p.div_howo_mul, p.div_howo_shift), rem = rr - n * p.ho_wo;
      int oy = fast_div(rem, p.div_wo_mul, p.div_wo_shift), ox = rem - oy * p.wo;
      a_iy0[j] = oy * p.sh - p.ph;
      a_ix0[j] = ox * p.sw - p.pw;
      a_base[j] = (int32_t)(n * p.xs_n + (int64_t)a_iy0[j] * p.xs_h + (int64_t)a_ix0[j] * p.xs_w);
    } else {
      a_iy0[j] = -(1 << 30);
      a_ix0[j] = 0;
      a_base[j] = 0;
    }
  }
  const T* __restrict__ wp = static_cast<const T*>(p.wp) + (int64_t)(n0 + lrow) * p.k_pad + c16 * V;

  // Position of this thread's 16-byte group inside the window, advanced by one K tile per load:
  // channel g_ci of tap (g_ky, g_kx).  Taps past the last one (K padding) read as zero.
  int g_ci = 0, g_kx = 0, g_ky = 0;
  if constexpr (VEC) {
    const int k0 = c16 * V;
    const int tap = k0 / p.c_in;
    g_ci = k0 - tap * p.c_in;
    g_ky = tap / p.kw;
    g_kx = tap - g_ky * p.kw;
  }

  // row-segment gather: dword masks that clear the entries of a window row's last 16-byte group which
  // lie beyond the window (their filter entries are zero, but a non-finite neighbour must not leak in)
  int seg_mask[4] = {-1, -1, -1, -1};
  if constexpr (ROWSEG) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      seg_mask[i] = p.seg_tail >= 2 * i + 2 ? -1 : p.seg_tail == 2 * i + 1 ? 0xffff : 0;
  }

  v4i ra[DEPTH][A_LOADS], rb[DEPTH][B_LOADS];

  auto load_tile = [&](int kt, v4i (&a)[A_LOADS], v4i (&b)[B_LOADS]) {
    if constexpr (ROWSEG) {
      // group g of K = (window row ky, 16-byte group gx of that row); the input copy has zero margins,
      // so every tap of every present row is in bounds
      const int g = kt * 8 + c16;
      const int ky = (g * p.seg_gpk_inv) >> 16, gx = g - ky * p.seg_gpk;   // g / gpk for g < 4096, gpk <= 8
      const bool row_ok = ky < p.kh;
      const int off = ky * p.dil_h * p.xs_h + gx * 8;
      const bool last = gx == p.seg_gpk - 1;
#pragma unroll
      for (int j = 0; j < A_LOADS; ++j) {
        v4i v = {0, 0, 0, 0};
        if (row_ok && a_iy0[j] >= 0) {
          __builtin_memcpy(&v, x + (a_base[j] + off), 16);   // element-aligned source
          if (last) {
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] &= seg_mask[i];
          }
        }
        a[j] = v;
      }
    } else if constexpr (VEC) {
      const int dy = g_ky * p.dil_h, dx = g_kx * p.dil_w;
      const int off = dy * p.xs_h + dx * p.xs_w + g_ci;
      const bool tap_ok = g_ky < p.kh;
#pragma unroll
      for (int j = 0; j < A_LOADS; ++j) {
        bool ok = tap_ok && (unsigned)(a_iy0[j] + dy) < (unsigned)p.h && (unsigned)(a_ix0[j] + dx) < (unsigned)p.w;
        v4i v = {0, 0, 0, 0};
        if (ok) v = *reinterpret_cast<const v4i*>(x + (a_base[j] + off));
        a[j] = v;
      }
      g_ci += BK;
      while (g_ci >= p.c_in) {
        g_ci -= p.c_in;
        if (++g_kx == p.kw) { g_kx = 0; ++g_ky; }
      }
    } else {
      const KEntry* kt_e = p.ktab + kt * BK + c16 * V;
#pragma unroll
      for (int j = 0; j < A_LOADS; ++j) {
        T tmp[V];
#pragma unroll
        for (int e = 0; e < V; ++e) {
          KEntry ke = kt_e[e];
          int dy = ke.dydx & 0xffff, dx = ke.dydx >> 16;
          bool ok = (unsigned)(a_iy0[j] + dy) < (unsigned)p.h && (unsigned)(a_ix0[j] + dx) < (unsigned)p.w;
          tmp[e] = ok ? x[a_base[j] + ke.off] : E::from_float(0.0f);
        }
        v4i v;
        __builtin_memcpy(&v, tmp, 16);
        a[j] = v;
      }
    }
#pragma unroll
    for (int j = 0; j < B_LOADS; ++j)
      b[j] = *reinterpret_cast<const v4i*>(wp + (int64_t)(32 * j) * p.k_pad + kt * BK);
  };

  // prefetch the first DEPTH K tiles before anything else so their latency overlaps the set-up
#pragma unroll
  for (int s = 0; s < DEPTH; ++s)
    if (s < p.k_tiles) load_tile(s, ra[s], rb[s]);

  __syncthreads();  // s_rows visible

  // ---- zero fill of the dropped rows this workgroup owns (Alg. 2, mask == 0 branch) ----------
  // Ownership: the dense rows from this tile's first kept row up to the next tile's first kept
  // row (first tile starts at row 0, last tile ends at M), restricted to this tile's channels.
  if (p.zero_fill) {
    const int lo = tile_m == 0 ? 0 : s_rows[0];
    const int hi = (m0 + BM >= p.rows) ? p.m_total : p.row_idx[m0 + BM];
    if (p.vec_out) {
      // thread (zr, zc) covers 16-byte group zc of rows lo + zr + u*RPI; mask bytes four passes at a time
      constexpr int CPR = BN * EB / 16;   // 16-byte groups per row slice
      constexpr int RPI = kThreads / CPR;
      const int valid = (min(BN, p.c_out - n0) * EB) >> 4;
      const int zc = t % CPR, zr = t / CPR;
      if (zc < valid) {
        unsigned char* ybase = reinterpret_cast<unsigned char*>(y) + (int64_t)n0 * EB + zc * 16;
        const int64_t res_at = (int64_t)n0 * EB + zc * 16;     // the same group of the shortcut tensor
        const v4i z = {0, 0, 0, 0};
        for (int r0 = lo + zr; r0 < hi; r0 += 4 * RPI) {
          unsigned char mk[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            int r = min(r0 + u * RPI, hi - 1);
            if (p.mask_spatial) r -= fast_div(r, p.div_howo_mul, p.div_howo_shift) * p.ho_wo;
            mk[u] = p.mask[r];
          }
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int r = r0 + u * RPI;
            if (r < hi && mk[u] == 0) {
              const int64_t at = (int64_t)r * p.c_out * EB;
              sc_store16(reinterpret_cast<v4i*>(ybase + at), p.residual ? dropped_row_group<DT>(p.residual, res_at + at, p.residual_relu) : z);
            }
          }
        }
      }
    } else {
      const int total = (hi - lo) * BN;
      for (int idx = t; idx < total; idx += kThreads) {
        int r = lo + idx / BN, c = n0 + idx % BN;
        int mr = p.mask_spatial ? r % p.ho_wo : r;
        if (c < p.c_out && p.mask[mr] == 0) {
          int n = r / p.ho_wo, rem = r - n * p.ho_wo;
          const int64_t at = n * p.ys_n + (int64_t)rem * p.ys_p + (int64_t)c * p.ys_c;
          float fill = 0.0f;
          if (p.residual) {
            fill += (float)static_cast<const T*>(p.residual)[at];
            if (p.residual_relu) fill = fmaxf(fill, 0.0f);
          }
          y[at] = E::from_float(fill);
        }
      }
    }
  }

  const int st_off = lrow * kRowBytes + ((c16 ^ ((lrow >> 1) & 7)) << 4);
  auto store_tile = [&](int buf, const v4i (&a)[A_LOADS], const v4i (&b)[B_LOADS]) {
    unsigned char* pa = s_a + buf * BM * kRowBytes + st_off;
    unsigned char* pb = s_b + buf * BN * kRowBytes + st_off;
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j) *reinterpret_cast<v4i*>(pa + j * 32 * kRowBytes) = a[j];
#pragma unroll
    for (int j = 0; j < B_LOADS; ++j) *reinterpret_cast<v4i*>(pb + j * 32 * kRowBytes) = b[j];
  };

  floatx16 acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

  const int fp = lane & 31, fh = lane >> 5;
  int frag_off[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) frag_off[ks] = fp * kRowBytes + (((2 * ks + fh) ^ ((fp >> 1) & 7)) << 4);

  auto compute_tile = [&](int buf) {
    const unsigned char* a = s_a + buf * BM * kRowBytes + wm0 * kRowBytes;
    const unsigned char* b = s_b + buf * BN * kRowBytes + wn0 * kRowBytes;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      v4i xf[MI], wf[NI];
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
        xf[mi] = *reinterpret_cast<const v4i*>(a + mi * 32 * kRowBytes + frag_off[ks]);
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
        wf[ni] = *reinterpret_cast<const v4i*>(b + ni * 32 * kRowBytes + frag_off[ks]);
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) E::mma(acc[mi][ni], wf[ni], xf[mi]);
    }
  };

  // ---- main loop: global -> registers (DEPTH K tiles in flight) -> LDS (double buffered) -> MFMA,
  // one barrier per K tile.  Tile kt sits in register slot kt % DEPTH; the loop is unrolled by
  // DEPTH so that every slot index is a compile-time constant.
  store_tile(0, ra[0], rb[0]);
  __syncthreads();
#pragma unroll 1
  for (int kt0 = 0; kt0 < p.k_tiles; kt0 += DEPTH) {
#pragma unroll
    for (int s = 0; s < DEPTH; ++s) {
      const int kt = kt0 + s;
      if (kt >= p.k_tiles) break;
      if (kt + DEPTH < p.k_tiles) load_tile(kt + DEPTH, ra[s], rb[s]);   // slot s was drained last iteration
      compute_tile(kt & 1);
      if (kt + 1 < p.k_tiles) store_tile((kt + 1) & 1, ra[(s + 1) % DEPTH], rb[(s + 1) % DEPTH]);
      __syncthreads();
    }
  }

  // ---- epilogue: bias, ReLU, convert, store every kept row at its dense position --------------
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    const int rr = s_rows[wm0 + mi * 32 + fp];
    if (rr == -1 || (rr < -1 && p.masked_store != 1)) continue;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
      const int c0 = n0 + wn0 + ni * 32 + 16 * fh;
      if (c0 >= p.c_out) continue;
      if (rr < 0) { store_zero_block<DT>(-2 - rr, c0, y, p.vec_out, p.c_out, p.ho_wo, p.ys_n, p.ys_p, p.ys_c); continue; }
      store_kept_block_res<DT>(acc[mi][ni], rr, c0, y, p.bias, c0, p.relu, p.vec_out, p.c_out, p.ho_wo, p.ys_n, p.ys_p,
                               p.ys_c, static_cast<const T*>(p.residual), p.residual_relu);
    }
  }
}

template <int DT, int BM, int BN, int WAVES_M, int WAVES_N, int GATHER, int DEPTH>
hipError_t igemm_launch(const ConvParams& p, hipStream_t stream) {
  constexpr size_t lds = igemm_lds_bytes<BM, BN>();
  auto kern = igemm_kernel<DT, BM, BN, WAVES_M, WAVES_N, GATHER, DEPTH>;
  static std::atomic<bool> attr_set{false};
  if (lds > 64 * 1024 && !attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int nwg = p.m_tiles * p.n_tiles;
  const int grid = ((nwg + 7) / 8) * 8;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), lds, stream, p);
  return hipGetLastError();
}

#define SC_KERNEL_ENTRY(DT, BM, BN, WM_, WN_, DEPTH, STAGES)                              \
  KernelEntry { BM, BN, igemm_launch<DT, BM, BN, WM_, WN_, 1, DEPTH>,                 \
                igemm_launch<DT, BM, BN, WM_, WN_, 0, 1>,                            \
                igemm_dma_launch<DT, BM, BN, WM_, WN_, STAGES>,                          \
                igemm_dma_launch<DT, BM, BN, WM_, WN_, 2>, nullptr, igemm_lds_bytes<BM, BN>() }

// the same plus the split-K form of the direct-to-LDS kernel with a ring of SK_STAGES tiles
#define SC_KERNEL_ENTRY_SPLITK(DT, BM, BN, WM_, WN_, DEPTH, STAGES, SK_STAGES)           \
  KernelEntry { BM, BN, igemm_launch<DT, BM, BN, WM_, WN_, 1, DEPTH>,                 \
                igemm_launch<DT, BM, BN, WM_, WN_, 0, 1>,                            \
                igemm_dma_launch<DT, BM, BN, WM_, WN_, STAGES>,                          \
                igemm_dma_launch<DT, BM, BN, WM_, WN_, 2>,                               \
                igemm_dma_launch<DT, BM, BN, WM_, WN_, SK_STAGES, true>, igemm_lds_bytes<BM, BN>() }

}  // namespace sc
