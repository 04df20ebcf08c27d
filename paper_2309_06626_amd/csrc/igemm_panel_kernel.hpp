// Row-panel masked-convolution kernel for layers with a short K (pointwise layers: K = Cin <= 128
// bytes * 2 per row) and many output channels.
//
// Same three fused stages as the tiled kernels (paper Sec. 3.2: lower the kept rows only, contract,
// put the results and the zeros back), but a workgroup owns BM kept rows for *all* output channels:
// the rows' K entries are gathered once (straight into LDS) and stay there while the workgroup
// walks the channel tiles, whose filter slices arrive through a two-slot ring one tile ahead.
//
// Why: on such layers the tiled kernels are bound by instruction issue, not by memory or the matrix
// cores -- every (row tile, channel tile) workgroup repeats the row decode, the gather set-up and
// the zero-fill bookkeeping (about 900 instructions per wavefront) for two K tiles of work.  Here
// that is paid once per row tile; a channel tile costs its transfers, 8 * MI * NI MFMAs and its
// stores.  The workgroup also writes whole output rows (its kept rows and the zeros of the dropped
// rows it owns, one contiguous range of the dense output).
//
// Waiting: the stores of channel tile n are issued after the transfers of tile n+1, and the memory
// counter retires in order, so "tile n+1 has landed" is vmcnt(<number of stores of tile n>) -- a
// compile-time number when the row tile and the channel tile are complete, vmcnt(0) otherwise.
#pragma once
#include "igemm_dma_kernel.hpp"

namespace sc {

constexpr int kPanelMaxKTiles = 2;

// LDS bytes: gathered rows [k_tiles][BM], filter ring [2][k_tiles][BN], row list, bias of all channels
template <int BM, int BN>
inline size_t igemm_panel_lds_bytes(int k_tiles, int c_out) {
  return (size_t)k_tiles * (BM + 2 * BN) * kRowBytes + BM * sizeof(int32_t) + (size_t)((c_out + 63) / 64) * 64 * sizeof(float);
}

template <int DT, int BM, int BN, int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(kThreads) void igemm_panel_kernel(const ConvParams p) {
  using E = Elem<DT>;
  using T = typename E::T;
  constexpr int V = E::V;
  constexpr int EB = sizeof(T);
  constexpr int BK = 8 * V;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int MI = WM / 32, NI = WN / 32;
  constexpr int A_LOADS = BM / 32, B_LOADS = BN / 32;
  constexpr int STORES = MI * NI * (16 * EB / 16);     // store instructions of one channel tile per wavefront
  static_assert(WAVES_M * WAVES_N * 64 == kThreads, "four wavefronts");
  static_assert(EB == 2, "16-bit operands");

  extern __shared__ __align__(16) unsigned char smem[];
  const int KT = p.k_tiles;
  const unsigned off_b = (unsigned)(KT * BM * kRowBytes);
  const unsigned off_rows = off_b + (unsigned)(2 * KT * BN * kRowBytes);
  int32_t* s_rows = reinterpret_cast<int32_t*>(smem + off_rows);      // [BM]
  float* s_bias = reinterpret_cast<float*>(s_rows + BM);              // [ceil(c_out / 64) * 64]

  const int per_xcd = (p.m_tiles + 7) >> 3;
  const int tile_m = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);   // each XCD: one contiguous run of row tiles
  if (tile_m >= p.m_tiles) return;
  const int m0 = tile_m * BM;

  const int t = threadIdx.x;
  const int lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
  const int fp = lane & 31, fh = lane >> 5;

  const T* __restrict__ x = static_cast<const T*>(p.x);
  T* __restrict__ y = static_cast<T*>(p.y);
  const T* __restrict__ zeros = static_cast<const T*>(p.zeros);

  // ---- one round trip: row numbers, bias, the dense row range this workgroup owns --------------------
  const int c16 = t & 7;                              // physical 16-byte group this lane fills
  const int lrow = t >> 3;                            // tile row (plus 32 per transfer)
  const int lc = c16 ^ ((lrow >> 1) & 7);             // logical group it fetches
  int32_t a_row[A_LOADS];
#pragma unroll
  for (int j = 0; j < A_LOADS; ++j) {
    const int icc = min(m0 + lrow + 32 * j, p.rows - 1);
    a_row[j] = p.row_idx ? p.row_idx[icc] : icc;
  }
  const int bias_n = ((p.c_out + 63) >> 6) << 6;
  float bias_v[4];                                    // up to 1024 channels
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = t + i * kThreads;
    bias_v[i] = (p.bias && c < p.c_out) ? p.bias[c] : 0.0f;
  }
  int z_lo = 0, z_hi = p.m_total;
  if (p.zero_fill) {
    if (tile_m != 0) z_lo = p.row_idx[m0];
    if (m0 + BM < p.rows) z_hi = p.row_idx[m0 + BM];
  }

  int32_t a_base[A_LOADS], a_iy0[A_LOADS], a_ix0[A_LOADS];
#pragma unroll
  for (int j = 0; j < A_LOADS; ++j) {
    const bool present = m0 + lrow + 32 * j < p.rows;
    const int ic = m0 + lrow + 32 * j;                       // position in the compacted GEMM
    const int rr = present ? (p.y_compact ? ic : a_row[j]) : -1;   // row the epilogue stores to
    s_rows[lrow + 32 * j] = rr;
    const int rc = present ? (p.x_compact ? ic : a_row[j]) : 0;    // row the window is read from
    const int n = fast_div(rc, p.div_howo_mul, p.div_howo_shift), rem = rc - n * p.ho_wo;
    const int oy = fast_div(rem, p.div_wo_mul, p.div_wo_shift), ox = rem - oy * p.wo;
    a_iy0[j] = present ? oy * p.sh - p.ph : -(1 << 30);
    a_ix0[j] = ox * p.sw - p.pw;
    a_base[j] = (int32_t)(n * p.xs_n + (int64_t)(oy * p.sh - p.ph) * p.xs_h + (int64_t)a_ix0[j] * p.xs_w);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = t + i * kThreads;
    if (c < bias_n) s_bias[c] = bias_v[i];
  }
  // Zero fill: the owned dense rows are dealt to the wavefronts in chunks of 64 (chunk c to wavefront
  // c & 3); a lane fetches the mask byte of one row of the chunk, a ballot turns the chunk into a
  // 64-bit set of dropped rows.  The first chunk of every wavefront is requested here.
  auto mask_of = [&](int r) -> unsigned {
    r = min(r, p.m_total - 1);
    if (p.mask_spatial) r -= fast_div(r, p.div_howo_mul, p.div_howo_shift) * p.ho_wo;
    return p.mask[r];
  };
  const unsigned mk0 = mask_of(z_lo + 64 * wave + lane);
  __syncthreads();   // s_rows, s_bias written; nothing is in flight yet

  const int64_t zoff = reinterpret_cast<const unsigned char*>(zeros) - reinterpret_cast<const unsigned char*>(x);
  auto dma16 = [](const void* src, unsigned char* lds_base) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                     (__attribute__((address_space(3))) void*)lds_base, 16, 0, 0);
  };
  // gathered rows, every K tile: the same lane-to-window mapping as the tiled kernel
  {
    int g_ci, g_kx, g_ky;
    const int k0 = lc * V;
    const int tap = k0 / p.c_in;
    g_ci = k0 - tap * p.c_in;
    g_ky = tap / p.kw;
    g_kx = tap - g_ky * p.kw;
    for (int kt = 0; kt < KT; ++kt) {
      unsigned char* sa = smem + kt * BM * kRowBytes + wave * 8 * kRowBytes;
      const int dy = g_ky * p.dil_h, dx = g_kx * p.dil_w;
      const int off = dy * p.xs_h + dx * p.xs_w + g_ci;
      const bool tap_ok = g_ky < p.kh;
#pragma unroll
      for (int j = 0; j < A_LOADS; ++j) {
        const bool ok = tap_ok && (unsigned)(a_iy0[j] + dy) < (unsigned)p.h && (unsigned)(a_ix0[j] + dx) < (unsigned)p.w;
        const int64_t boff = ok ? (int64_t)(a_base[j] + off) * EB : zoff;
        dma16(reinterpret_cast<const unsigned char*>(x) + boff, sa + j * 32 * kRowBytes);
      }
      g_ci += BK;
      while (g_ci >= p.c_in) {
        g_ci -= p.c_in;
        if (++g_kx == p.kw) { g_kx = 0; ++g_ky; }
      }
    }
  }
  // filter slice of channel tile n into ring slot `slot`
  const T* __restrict__ wp = static_cast<const T*>(p.wp) + (int64_t)lrow * p.k_pad + lc * V;
  auto issue_filters = [&](int n, int slot) {
    for (int kt = 0; kt < KT; ++kt) {
      unsigned char* sb = smem + off_b + (slot * KT + kt) * BN * kRowBytes + wave * 8 * kRowBytes;
#pragma unroll
      for (int j = 0; j < B_LOADS; ++j)
        dma16(wp + (int64_t)(n * BN + 32 * j) * p.k_pad + kt * BK, sb + j * 32 * kRowBytes);
    }
  };
  issue_filters(0, 0);

  const unsigned lds0 = (unsigned)(unsigned long long)(__attribute__((address_space(3))) unsigned char*)smem;
  unsigned frag_a[4], frag_b[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const unsigned o = (unsigned)(fp * kRowBytes + (((2 * ks + fh) ^ ((fp >> 1) & 7)) << 4));
    frag_a[ks] = lds0 + wm0 * kRowBytes + o;
    frag_b[ks] = lds0 + off_b + wn0 * kRowBytes + o;
  }
  auto read_step = [&](unsigned a_off, unsigned b_off, int ks, v4i (&f)[MI + NI]) {
    const unsigned aa = frag_a[ks] + a_off, ab = frag_b[ks] + b_off;
    if constexpr (MI >= 1) f[0] = lds_read16_at<0>(aa);
    if constexpr (MI >= 2) f[1] = lds_read16_at<32 * kRowBytes>(aa);
    if constexpr (MI >= 3) f[2] = lds_read16_at<64 * kRowBytes>(aa);
    if constexpr (MI >= 4) f[3] = lds_read16_at<96 * kRowBytes>(aa);
    if constexpr (NI >= 1) f[MI + 0] = lds_read16_at<0>(ab);
    if constexpr (NI >= 2) f[MI + 1] = lds_read16_at<32 * kRowBytes>(ab);
  };

  int rr[MI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) rr[mi] = s_rows[wm0 + mi * 32 + fp];
  const bool rows_full = m0 + BM <= p.rows;

  // ---- channel tiles ---------------------------------------------------------------------------------
  bool prev_full = false;
  for (int n = 0; n < p.n_tiles; ++n) {
    // filter slice n (and, at n = 0, the gathered rows) has landed once only the stores of tile n-1
    // are still in flight
    if (n > 0 && prev_full) wait_vmcnt<STORES>();
    else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();   // ... for every wavefront; and all have left ring slot (n+1) & 1
    asm volatile("" ::: "memory");
    if (n + 1 < p.n_tiles) issue_filters(n + 1, (n + 1) & 1);

    floatx16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;
    for (int kt = 0; kt < KT; ++kt) {
      const unsigned a_off = (unsigned)(kt * BM * kRowBytes);
      const unsigned b_off = (unsigned)((((n & 1) * KT) + kt) * BN * kRowBytes);
      v4i f0[MI + NI], f1[MI + NI], f2[MI + NI], f3[MI + NI];
      read_step(a_off, b_off, 0, f0);
      read_step(a_off, b_off, 1, f1);
      read_step(a_off, b_off, 2, f2);
      read_step(a_off, b_off, 3, f3);
      wait_frags<3 * (MI + NI)>(f0);
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) E::mma(acc[mi][ni], f0[MI + ni], f0[mi]);
      wait_frags<2 * (MI + NI)>(f1);
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) E::mma(acc[mi][ni], f1[MI + ni], f1[mi]);
      wait_frags<(MI + NI)>(f2);
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) E::mma(acc[mi][ni], f2[MI + ni], f2[mi]);
      wait_frags<0>(f3);
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) E::mma(acc[mi][ni], f3[MI + ni], f3[mi]);
    }

    // epilogue of the channel tile: bias, ReLU, conversion, kept rows to their dense slots
    const int n0 = n * BN;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      if (rr[mi] < 0) continue;
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) {
        const int c0 = n0 + wn0 + ni * 32 + 16 * fh;
        if (c0 >= p.c_out) continue;
        store_kept_block<DT>(acc[mi][ni], rr[mi], c0, y, p.bias ? s_bias + c0 : nullptr, 0, p.relu, 1, p.c_out,
                             p.ho_wo, 0, 0, 0);
      }
    }
    prev_full = rows_full && n0 + BN <= p.c_out;
  }

  // ---- zero fill of the dropped rows this workgroup owns (Alg. 2, mask == 0 branch): whole rows --------
  if (p.zero_fill) {
    const int gpr = (p.c_out * EB) >> 4;          // 16-byte groups per output row
    const v4i z = {0, 0, 0, 0};
    unsigned char* ybase = reinterpret_cast<unsigned char*>(y);
    for (int c0 = z_lo + 64 * wave; c0 < z_hi; c0 += 256) {
      const unsigned m = c0 == z_lo + 64 * wave ? mk0 : mask_of(c0 + lane);
      unsigned long long dropped = __ballot(m == 0 && c0 + lane < z_hi);
      while (dropped) {
        const int r = c0 + __builtin_ctzll(dropped);
        dropped &= dropped - 1;
        v4i* row = reinterpret_cast<v4i*>(ybase + (int64_t)r * p.c_out * EB);
        for (int gq = lane; gq < gpr; gq += 64) sc_store16(row + gq, z);
      }
    }
  }
}

template <int DT, int BM, int BN, int WAVES_M, int WAVES_N>
hipError_t igemm_panel_launch(const ConvParams& p, hipStream_t stream) {
  const size_t lds = igemm_panel_lds_bytes<BM, BN>(p.k_tiles, p.c_out);
  auto kern = igemm_panel_kernel<DT, BM, BN, WAVES_M, WAVES_N>;
  static std::atomic<size_t> attr_bytes{0};   // (plans may be run from several host threads)
  if (lds > 64 * 1024 && lds > attr_bytes) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_bytes = lds;
  }
  const int grid = ((p.m_tiles + 7) / 8) * 8;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), lds, stream, p);
  return hipGetLastError();
}

// row tile and channel tile of the panel kernel
constexpr int kPanelBM = 128, kPanelBN = 64;
LaunchFn panel_bf16();
LaunchFn panel_f16();

}  // namespace sc
