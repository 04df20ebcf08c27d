// Band kernel with streamed filters, for 3x3-like layers whose filter slab does not fit in LDS.
//
// A tiled GEMM reads every input pixel once per window tap: for a 3x3 layer the lowered matrix A
// (paper Sec. 3, Fig. 1) is nine times the size of the activation tensor, and on this GPU the L2 ->
// LDS traffic of A, not the matrix cores, bounds the tiled kernel.  Here the workgroup keeps the
// input slab of its band resident in LDS (read from L2 once, as in band_kernel.hpp) and streams
// only the filters: K tiles of 128 bytes per filter row go through a ring of STAGES LDS tiles by
// direct global-to-LDS transfers, STAGES-1 tiles ahead of the MFMAs.  All kept rows of the band
// stay in accumulators for the whole K loop: 32*MI rows per wavefront, 4 wavefronts, 32*NI channels.
//
// Waits are explicit (see igemm_dma_kernel.hpp): vmcnt for "K tile kt has landed", lgkmcnt for the
// inline ds_read_b128 fragment reads.
#pragma once
#include "band_kernel.hpp"
#include "conv_params.hpp"
#include "igemm_dma_kernel.hpp"
#include "mma_common.hpp"

namespace sc {

constexpr int kStreamStages = 4;

template <int DT, int NI, int MI>
__global__ __launch_bounds__(kThreads) void bandstream_kernel(const BandParams p) {
  using E = Elem<DT>;
  using T = typename E::T;
  constexpr int V = E::V;
  constexpr int EB = sizeof(T);
  constexpr int BK = 8 * V;
  constexpr int BN = 32 * NI;
  constexpr int B_LOADS = BN / 32;                 // transfers per K tile and wavefront
  constexpr int STAGES = kStreamStages;
  constexpr int STAGE_BYTES = BN * kRowBytes;
  constexpr int CPR = BN * EB / 16;
  constexpr int RPI = kThreads / CPR;

  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* s_w = smem;                                       // [STAGES][BN][128]
  v4i* s_x = reinterpret_cast<v4i*>(smem + STAGES * STAGE_BYTES);  // input slab, then 1 KiB of zeros

  SC_STAMP(0);
  const int nwg = p.n_bands * p.n_tiles;
  const int per_xcd = (nwg + 7) >> 3;
  const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (logical >= nwg) return;
  const int band = logical / p.n_tiles;
  const int n0 = (logical - band * p.n_tiles) * BN;

  const int t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int fp = lane & 31, fh = lane >> 5;

  const int img = band / p.bands_per_image;
  const int oy0 = (band - img * p.bands_per_image) * p.bh;
  const int oy1 = min(oy0 + p.bh, p.ho);
  const int ho_wo = p.ho * p.wo;
  const int r_lo = img * ho_wo + oy0 * p.wo, r_hi = img * ho_wo + oy1 * p.wo;
  const int band_rows_n = r_hi - r_lo;
  const int iy_base = oy0 * p.sh - p.ph;
  const int iy_lo = max(iy_base, 0);
  const int iy_hi = min((oy1 - 1) * p.sh - p.ph + (p.kh - 1) * p.dil_h + 1, p.h);
  const int cpp = p.c_in / V;            // 16-byte groups per pixel, a multiple of 8 here
  const int tiles_per_tap = cpp >> 3;
  const int k_tiles = p.kh * p.kw * tiles_per_tap;

  const T* __restrict__ x = static_cast<const T*>(p.x);
  T* __restrict__ y = static_cast<T*>(p.y);

  // ---- kept rows of the band: blocks of 32 rows dealt round robin, MI blocks per wavefront ----------
  int cnt = band_rows_n;
  if (p.row_idx) cnt = p.band_i0[band + 1] - p.band_i0[band];
  int r_pre[MI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    const int jc = min((mi * 4 + wave) * 32 + fp, band_rows_n - 1);   // clamped: unconditional load
    r_pre[mi] = p.row_idx ? p.band_rows[r_lo + jc] : r_lo + jc;
  }
  __builtin_amdgcn_sched_barrier(0);

  // ---- stage the input slab (contiguous in global memory), swizzle on the global side --------------
  auto dma16 = [](const void* src, void* lds_base) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                     (__attribute__((address_space(3))) void*)lds_base, 16, 0, 0);
  };
  {
    const v4i* gx = reinterpret_cast<const v4i*>(x + ((int64_t)(img * p.h + iy_lo) * p.w) * p.c_in);
    const int nx = max(iy_hi - iy_lo, 0) * p.w * cpp;
    const int qx0 = (iy_lo - iy_base) * p.w * cpp;
    for (int qb = (qx0 & ~63) + wave * 64; qb < qx0 + nx; qb += kThreads) {
      const int g = swz(qb + lane) - qx0;
      if (g >= 0 && g < nx) dma16(gx + g, s_x + qb);
    }
  }

  // ---- filter ring: lane (row, physical group c16) of a transfer fetches logical group c16 ^ key ----
  const int c16 = t & 7, lrow = t >> 3;
  const int lc = c16 ^ ((lrow >> 1) & 7);
  const T* __restrict__ wp = static_cast<const T*>(p.wp) + (int64_t)(n0 + lrow) * p.k_stride + lc * V;
  auto issue_tile = [&](int kt, int stage) {
    unsigned char* sb = s_w + stage * STAGE_BYTES + wave * 8 * kRowBytes;
#pragma unroll
    for (int j = 0; j < B_LOADS; ++j) dma16(wp + (int64_t)(32 * j) * p.k_stride + kt * BK, sb + j * 32 * kRowBytes);
  };
  // Workgroups of one channel tile stream the same filters; each starts at a different K tile so
  // that they do not all ask the same L2 lines at the same moment (the sum over K is order-free).
  const int k_rot = (int)(((unsigned)band * 5u) % (unsigned)k_tiles);
  auto tile_id = [&](int i) { int k = i + k_rot; return k >= k_tiles ? k - k_tiles : k; };
#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s)
    if (s < k_tiles) issue_tile(tile_id(s), s);

  // ---- per-lane window geometry of its MI rows -------------------------------------------------------
  int rr[MI], ly0[MI], lx0[MI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    const bool present = (mi * 4 + wave) * 32 + fp < cnt;
    rr[mi] = present ? r_pre[mi] : -1;
    const int rem = (present ? r_pre[mi] : r_lo) - img * ho_wo;
    const int oy = rem / p.wo, ox = rem - oy * p.wo;
    ly0[mi] = oy * p.sh - p.ph - iy_base;
    lx0[mi] = present ? ox * p.sw - p.pw : -(1 << 28);   // no tap of an absent row is ever in range
  }
  const unsigned lds0 = (unsigned)(unsigned long long)(__attribute__((address_space(3))) unsigned char*)smem;
  const unsigned xbase = lds0 + STAGES * STAGE_BYTES, zaddr = xbase + (unsigned)p.x_groups * 16u;
  if (t < 64) {
    const v4i z = {0, 0, 0, 0};
    s_x[p.x_groups + t] = z;
  }
  unsigned frag_w[4];   // LDS address of this lane's filter fragment of K step ks in ring stage 0
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
    frag_w[ks] = lds0 + (unsigned)(fp * kRowBytes + (((2 * ks + fh) ^ ((fp >> 1) & 7)) << 4));

  floatx16 acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

  // ---- K loop ------------------------------------------------------------------------------------------
  int stage = 0;
  int tap0 = k_rot / tiles_per_tap;
  int tt = k_rot - tap0 * tiles_per_tap, ky = tap0 / p.kw, kx = tap0 - (tap0 / p.kw) * p.kw;   // tile tt of tap (ky, kx)
  unsigned pix_q[MI];                               // LDS group of channel group 0 of the tap's pixel, or ~0u
  auto set_tap = [&]() {
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      const int ly = ly0[mi] + ky * p.dil_h, ix = lx0[mi] + kx * p.dil_w;
      const bool ok = (unsigned)(iy_base + ly) < (unsigned)p.h && (unsigned)ix < (unsigned)p.w;
      pix_q[mi] = ok ? (unsigned)((ly * p.w + ix) * cpp) : 0xffffffffu;
    }
  };
  set_tap();
  SC_STAMP(1);
  for (int kt = 0; kt < k_tiles; ++kt) {
    if (kt == 1) SC_STAMP(2);
    if (kt == k_tiles / 2) SC_STAMP(3);
    if (kt + STAGES - 2 < k_tiles) wait_vmcnt<(STAGES - 2) * B_LOADS>();
    else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();   // tile kt (and, the first time, the slab) is in LDS for everyone
    asm volatile("" ::: "memory");
    if (kt + STAGES - 1 < k_tiles) {
      int fill = stage + STAGES - 1;
      if (fill >= STAGES) fill -= STAGES;
      issue_tile(tile_id(kt + STAGES - 1), fill);
    }
    const unsigned stage_off = (unsigned)(stage * STAGE_BYTES);
    unsigned xa[MI];   // address of channel group (tt*8 + fh) of the tap's pixel; K step ks adds 2*ks groups
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      const unsigned q = pix_q[mi] + (unsigned)(tt * 8 + fh);
      xa[mi] = pix_q[mi] == 0xffffffffu ? zaddr : xbase + ((q ^ ((q >> 4) & 7u)) << 4);
    }
    // the swizzle XORs only the low three group bits and 2*ks + fh < 8 stays inside them:
    // group (q0 + 2*ks) -> address (base ^ (2*ks << 4)) with base built for ks = 0
    v4i f0[MI + NI], f1[MI + NI], f2[MI + NI], f3[MI + NI];
    auto read_step = [&](int ks, v4i (&f)[MI + NI]) {
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) f[mi] = lds_read16_at<0>(xa[mi] ^ ((unsigned)(2 * ks) << 4));
      const unsigned wa = frag_w[ks] + stage_off;
      if constexpr (NI >= 1) f[MI + 0] = lds_read16_at<0>(wa);
      if constexpr (NI >= 2) f[MI + 1] = lds_read16_at<32 * kRowBytes>(wa);
      if constexpr (NI >= 3) f[MI + 2] = lds_read16_at<64 * kRowBytes>(wa);
      if constexpr (NI >= 4) f[MI + 3] = lds_read16_at<96 * kRowBytes>(wa);
    };
    auto mma_step = [&](const v4i (&f)[MI + NI]) {
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) E::mma(acc[mi][ni], f[MI + ni], f[mi]);
    };
    read_step(0, f0);
    read_step(1, f1);
    wait_frags<MI + NI>(f0);
    mma_step(f0);
    read_step(2, f2);
    wait_frags<MI + NI>(f1);
    mma_step(f1);
    read_step(3, f3);
    wait_frags<MI + NI>(f2);
    mma_step(f2);
    wait_frags<0>(f3);
    mma_step(f3);

    if (++stage == STAGES) stage = 0;
    if (++tt == tiles_per_tap) {
      tt = 0;
      if (++kx == p.kw) { kx = 0; if (++ky == p.kh) ky = 0; }
      set_tap();
    }
  }

  SC_STAMP(5);
  // ---- zero fill of the band's dropped rows (Alg. 2, mask == 0 branch) --------------------------------
  if (p.zero_fill) {
    const int valid = (min(BN, p.c_out - n0) * EB) >> 4;
    const int zc = t % CPR, zr = t / CPR;
    if (zc < valid) {
      unsigned char* ybase = reinterpret_cast<unsigned char*>(y) + (int64_t)n0 * EB + zc * 16;
      const v4i z = {0, 0, 0, 0};
      for (int r0 = r_lo + zr; r0 < r_hi; r0 += 4 * RPI) {
        unsigned char mk[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int r = min(r0 + u * RPI, r_hi - 1);
          mk[u] = p.mask[p.mask_spatial ? r - img * ho_wo : r];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int r = r0 + u * RPI;
          if (r < r_hi && mk[u] == 0) sc_store16(reinterpret_cast<v4i*>(ybase + (int64_t)r * p.c_out * EB), z);
        }
      }
    }
  }

  SC_STAMP(6);
  // ---- epilogue ------------------------------------------------------------------------------------------
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    if (rr[mi] < 0) continue;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
      const int c0 = n0 + ni * 32 + 16 * fh;
      if (c0 >= p.c_out) continue;
      store_kept_block<DT>(acc[mi][ni], rr[mi], c0, y, p.bias, c0, p.relu, 1, p.c_out, ho_wo, 0, 0, 0);
    }
  }
  SC_STAMP(4);
}

template <int DT, int NI, int MI>
hipError_t bandstream_launch(const BandParams& p, size_t lds, hipStream_t stream) {
  auto kern = bandstream_kernel<DT, NI, MI>;
  static std::atomic<size_t> attr_bytes{0};   // (plans may be run from several host threads)
  if (lds > 64 * 1024 && lds > attr_bytes) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_bytes = lds;
  }
  const int nwg = p.n_bands * p.n_tiles;
  const int grid = ((nwg + 7) / 8) * 8;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), lds, stream, p);
  return hipGetLastError();
}

// fn[ni index 0..1 -> NI 2,4][MI - 1]
struct BandStreamTable { BandLaunchFn fn[2][4]; };
const BandStreamTable* bandstream_bf16();
const BandStreamTable* bandstream_f16();

#define SC_BANDSTREAM_TABLE(DT)                                                                       \
  { { { bandstream_launch<DT, 2, 1>, bandstream_launch<DT, 2, 2>, bandstream_launch<DT, 2, 3>,        \
        bandstream_launch<DT, 2, 4> },                                                                \
      { bandstream_launch<DT, 4, 1>, bandstream_launch<DT, 4, 2>, bandstream_launch<DT, 4, 3>,        \
        bandstream_launch<DT, 4, 4> } } }

}  // namespace sc
