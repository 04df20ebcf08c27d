// Band kernel with two alternating wavefront groups (3x3 windows, 16-bit types).
//
// Same decomposition as band_kernel.hpp (Sec. 3.2: lower only the kept windows of a band of output
// rows, inside LDS; GEMM on the kept rows; results and zeros written back by the band's owner), but
// a workgroup here is persistent and walks a list of bands:
//
//   workgroup  = 8 wavefronts in two groups of four; the filter slab [32*NI channels][K] is staged
//                once and stays in LDS; two input slabs sit behind it
//   step k     = group (k & 1) runs the MFMA loop and the stores of band k from slab (k & 1), while
//                the other group transfers band k+1 into the other slab (global -> LDS directly) and
//                fetches its kept-row numbers and mask bytes; one workgroup barrier between steps
//
// so the HBM read of the next band, the matrix work of this band and the draining stores of the
// previous one overlap inside one CU, which a single resident workgroup per CU (the filter slab
// leaves no room for a second one) cannot do on its own.  A group waits only for its own memory
// operations (each wavefront has its own counters): the stores of band k are waited for by the
// group that issued them, while the other group computes band k+1.
#pragma once
#include "band_kernel.hpp"

namespace sc {

constexpr int kPPThreads = 512;
constexpr int kPPGroup = 256;       // threads per wavefront group
constexpr int kPPMaxRows = 512;     // tallest band (output rows x width)
// LDS behind the filter slab: a zeroed KiB, 128 bias floats, then the two input slabs
constexpr int kPPFixedLds = 1024 + 512;

// RES: the run is fused with the shortcut sum that follows it (sparse_conv_run_residual): the epilogue adds the
// shortcut tensor in float before the one rounding, and the transferring group writes post(shortcut) instead of
// zeros at the dropped rows.  A separate instantiation, so the plain run keeps its registers and its code.
template <int DT, int NI, int MI, int KH, int KW, int CPP, bool RES = false>
__global__ __launch_bounds__(kPPThreads) void bandpp_kernel(const BandParams p) {
  using E = Elem<DT>;
  using T = typename E::T;
  constexpr int V = E::V;
  constexpr int EB = sizeof(T);
  constexpr int BN = 32 * NI;
  constexpr int CPR = BN * EB / 16;     // 16-byte groups per output row slice
  constexpr int RPI = kPPGroup / CPR;   // output rows covered by one zero-fill pass of a group
  constexpr int ZIT = 8;                // zero-fill passes whose mask bytes are fetched up front
  constexpr int RB = kPPMaxRows / (4 * 32 * MI);   // MFMA blocks per wavefront that cover the tallest band
  static_assert(KH > 0 && KW > 0 && (CPP & (CPP - 1)) == 0 && CPP >= 2 && CPP <= 8, "fixed window shapes only");
  static_assert(EB == 2, "16-bit operands");

  extern __shared__ __align__(16) unsigned char smem[];
  v4i* s_b = reinterpret_cast<v4i*>(smem);
  v4i* s_zero = reinterpret_cast<v4i*>(smem + p.b_bytes);
  float* s_bias = reinterpret_cast<float*>(smem + p.b_bytes + 1024);
  unsigned char* s_x_bytes = smem + p.b_bytes + kPPFixedLds;
  const int x_bytes = p.x_groups * 16;

  // workgroup -> (filter tile, band lane); consecutive lanes run on the same XCD so that the halo
  // rows shared by neighbouring bands are in that XCD's L2 when the second reader comes
  const int G = gridDim.x;
  const int logical = (G & 7) == 0 ? (int)(blockIdx.x & 7) * (G >> 3) + (int)(blockIdx.x >> 3) : (int)blockIdx.x;
  const int lanes = G / p.n_tiles;
  const int n0 = (logical % p.n_tiles) * BN;
  const int lane_id = logical / p.n_tiles;
  const int steps = lane_id < p.n_bands ? (p.n_bands - lane_id + lanes - 1) / lanes : 0;
  auto band_at = [&](int k) { return lane_id + k * lanes; };      // bands are dealt round robin

  const int t = threadIdx.x;
  const int grp = __builtin_amdgcn_readfirstlane(t >> 8);
  const int tl = t & (kPPGroup - 1);
  const int lane = t & 63, wave = tl >> 6;
  const int fp = lane & 31, fh = lane >> 5;
  const int ho_wo = p.ho * p.wo;
  const int kgr = p.k_stride / V;       // 16-byte groups per filter row

  const T* __restrict__ x = static_cast<const T*>(p.x);
  T* __restrict__ y = static_cast<T*>(p.y);

  auto dma16 = [](const v4i* src, v4i* lds_base) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                     (__attribute__((address_space(3))) void*)lds_base, 16, 0, 0);
  };

#ifdef SC_TIMING
  if (p.dbg && threadIdx.x == 0) p.dbg[(size_t)blockIdx.x * 128 + 120] = wall_clock64();
#endif
  // ---- once per workgroup: filter slab (all eight wavefronts), zero group, bias slice -------------
  {
    const v4i* gb = reinterpret_cast<const v4i*>(static_cast<const T*>(p.wp) + (int64_t)n0 * p.k_stride);
    const int nb = BN * kgr;
    for (int qb = (t >> 6) * 64; qb < nb; qb += kPPThreads) dma16(gb + swz(qb + lane), s_b + qb);
    if (t < 64) {
      const v4i z = {0, 0, 0, 0};
      s_zero[t] = z;
    }
    if (t < BN) s_bias[t] = (p.bias && n0 + t < p.c_out) ? p.bias[n0 + t] : 0.0f;
  }

#ifdef SC_TIMING
#define SC_PP_STAMP(k, slot) do { if (p.dbg && tl == 0 && (k) < 16) p.dbg[(size_t)blockIdx.x * 128 + (k) * 8 + (slot)] = clock64(); } while (0)
#else
#define SC_PP_STAMP(k, slot) do { } while (0)
#endif
  // band geometry (wavefront-uniform)
  struct Geo { int img, r_lo, r_hi, iy_base, iy_lo, iy_hi; };
  auto geo = [&](int band) {
    Geo g;
    g.img = band / p.bands_per_image;
    int first, end;       // the band's pixels; with split bands the range may begin and end inside a row
    band_pixel_range(band - g.img * p.bands_per_image, p.bh, p.split, p.ho, p.wo, &first, &end);
    const int oy0 = first / p.wo, oy1 = (end - 1) / p.wo + 1;
    g.r_lo = g.img * ho_wo + first;
    g.r_hi = g.img * ho_wo + end;
    g.iy_base = oy0 * p.sh - p.ph;
    g.iy_lo = max(g.iy_base, 0);
    g.iy_hi = min((oy1 - 1) * p.sh - p.ph + (KH - 1) * p.dil_h + 1, p.h);
    return g;
  };

  // carried from a group's transfer step to its compute step
  int r_pre[RB][MI];
  int cnt_v = 0;            // kept rows of the band (every lane holds the same value)
  const int zc = tl % CPR, zr = tl / CPR;   // zero fill: thread (zr, zc) covers 16-byte group zc of rows r_lo + zr + u*RPI

  auto transfer = [&](int band, v4i* s_x) {
    const Geo g = geo(band);
    // small loads first: kept-row numbers of this lane's MFMA columns, mask bytes of its zero-fill rows
    int i0 = 0, i1 = g.r_hi - g.r_lo;
    if (p.row_idx) { i0 = p.band_i0[band]; i1 = p.band_i0[band + 1]; }
#pragma unroll
    for (int b = 0; b < RB; ++b)
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        const int j = ((b * 4 + wave) * MI + mi) * 32 + fp;
        const int jc = min(j, g.r_hi - g.r_lo - 1);
        r_pre[b][mi] = p.row_idx ? p.band_rows[g.r_lo + jc] : g.r_lo + jc;
      }
    unsigned mk[ZIT];   // one register each: packing them would wait for the loads before the slab transfer
#pragma unroll
    for (int u = 0; u < ZIT; ++u) mk[u] = 1;
    if (p.zero_fill) {
#pragma unroll
      for (int u = 0; u < ZIT; ++u) {
        const int r = min(g.r_lo + zr + u * RPI, g.r_hi - 1);
        mk[u] = p.mask[p.mask_spatial ? r - g.img * ho_wo : r];
      }
    }
    __builtin_amdgcn_sched_barrier(0);   // the small loads are in flight before the slab transfer starts
    // the input slab: contiguous in global memory; the lane that owns LDS group q fetches global group swz(q)
    const v4i* gx = reinterpret_cast<const v4i*>(x + ((int64_t)(g.img * p.h + g.iy_lo) * p.w) * p.c_in);
    const int nx = max(g.iy_hi - g.iy_lo, 0) * p.w * CPP;
    const int qx0 = (g.iy_lo - g.iy_base) * p.w * CPP;
    const int q_end = qx0 + nx;
    for (int qb = (qx0 & ~63) + wave * 64; qb < q_end; qb += kPPGroup) {
      const int q = swz(qb + lane) - qx0;
      if (q >= 0 && q < nx) dma16(gx + q, s_x + qb);
    }
    __builtin_amdgcn_sched_barrier(0);   // nothing above waits for the small loads
    cnt_v = i1 - i0;
    // Alg. 2, mask == 0 branch: zeros for the dropped rows of the band, written by the transferring
    // group so that the computing group's store queue carries results only
    if (p.zero_fill) {
      const int valid = (min(BN, p.c_out - n0) * EB) >> 4;
      const v4i z = {0, 0, 0, 0};
      const int64_t col_at = (int64_t)n0 * EB + zc * 16;     // byte offset of this thread's group inside a row
      unsigned char* ybase = reinterpret_cast<unsigned char*>(y) + col_at;
      auto fill = [&](int r) {
        const int64_t at = (int64_t)r * p.c_out * EB;
        if constexpr (RES) sc_store16(reinterpret_cast<v4i*>(ybase + at), dropped_row_group<DT>(p.residual, col_at + at, p.residual_relu));
        else sc_store16(reinterpret_cast<v4i*>(ybase + at), z);
      };
      if (zc < valid) {
#pragma unroll
        for (int u = 0; u < ZIT; ++u) {
          const int r = g.r_lo + zr + u * RPI;
          if (r < g.r_hi && mk[u] == 0) fill(r);
        }
        for (int r = g.r_lo + zr + ZIT * RPI; r < g.r_hi; r += RPI)
          if (p.mask[p.mask_spatial ? r - g.img * ho_wo : r] == 0) fill(r);
      }
    }
  };

  auto compute = [&](int band, const v4i* s_x, int kk) {
    const Geo g = geo(band);
    const int cnt = __builtin_amdgcn_readfirstlane(cnt_v);
    const int nblk = (cnt + 32 * MI - 1) / (32 * MI);
    const unsigned xbase = lds_addr_of(s_x), zaddr = lds_addr_of(s_zero);
    const unsigned bbase = lds_addr_of(s_b);
#pragma unroll
    for (int bi = 0; bi < RB; ++bi) {
      const int blk = bi * 4 + wave;
      if (blk >= nblk) break;
      int rr[MI];
      unsigned tap_addr[MI][KH * KW];   // LDS address of channel group fh of every tap's pixel
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        const int j = (blk * MI + mi) * 32 + fp;
        const bool have = j < cnt;
        const int r = r_pre[bi][mi];
        const int rem = r - g.img * ho_wo;
        const int oy = rem / p.wo, ox = rem - oy * p.wo;
        rr[mi] = have ? r : -1;
        const int ly0 = oy * p.sh - p.ph - g.iy_base;
        const int lx0 = ox * p.sw - p.pw;
        const int pb = ly0 * p.w + lx0;
#pragma unroll
        for (int ky = 0; ky < KH; ++ky) {
          const bool oky = have && (unsigned)(g.iy_base + ly0 + ky * p.dil_h) < (unsigned)p.h;
#pragma unroll
          for (int kx = 0; kx < KW; ++kx) {
            const bool ok = oky && (unsigned)(lx0 + kx * p.dil_w) < (unsigned)p.w;
            const unsigned g0 = (unsigned)(pb + ky * p.dil_h * p.w + kx * p.dil_w) * CPP;
            const unsigned rel = ((g0 ^ ((g0 >> 4) & 7u)) << 4) ^ ((unsigned)fh << 4);
            tap_addr[mi][ky * KW + kx] = ok ? xbase + rel : zaddr;
          }
        }
      }
      floatx16 acc[MI][NI];
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
          for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

      // K steps of 32 bytes per row, in groups of GS; the fragments of group g+1 are read while the
      // MFMAs of group g run.  The swizzled byte address of channel group c of a pixel is
      // (pixel base) ^ (c << 4).
      constexpr int SPT = CPP / 2;            // steps per tap
      constexpr int S = KH * KW * SPT;
      constexpr int GS = MI * NI >= 4 ? 2 : 4;   // read-ahead depth, bounded by the register file (two wavefronts per SIMD)
      constexpr int NG = (S + GS - 1) / GS;
      unsigned w_q0[NI];
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) w_q0[ni] = (unsigned)((ni * 32 + fp) * kgr);
      v4i xb[2][GS][MI], wb[2][GS][NI];
      auto load_group = [&](int gi, v4i (&xd)[GS][MI], v4i (&wd)[GS][NI]) {
#pragma unroll
        for (int e = 0; e < GS; ++e) {
          const int st = gi * GS + e;
          if (st < S) {
            const int tp = st / SPT, j = (st % SPT) * 2;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) xd[e][mi] = lds_load16(tap_addr[mi][tp] ^ ((unsigned)j << 4));
            const unsigned kc = (unsigned)(tp * CPP + j) + (unsigned)fh;
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
              const unsigned q = w_q0[ni] + kc;
              wd[e][ni] = lds_load16(bbase + ((q ^ ((q >> 4) & 7u)) << 4));
            }
          }
        }
      };
      SC_PP_STAMP(kk, 3);
      load_group(0, xb[0], wb[0]);
#pragma unroll
      for (int gi = 0; gi < NG; ++gi) {
        __builtin_amdgcn_sched_barrier(0);
        if (gi + 1 < NG) load_group(gi + 1, xb[(gi + 1) & 1], wb[(gi + 1) & 1]);
#pragma unroll
        for (int e = 0; e < GS; ++e) {
          if (gi * GS + e < S) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
              for (int ni = 0; ni < NI; ++ni) E::mma(acc[mi][ni], wb[gi & 1][e][ni], xb[gi & 1][e][mi]);
          }
        }
        if (gi + 1 < NG) {
#pragma unroll
          for (int i = 0; i < GS * MI * NI; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      SC_PP_STAMP(kk, 7);

#pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        if (rr[mi] < 0) continue;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
          const int c0 = n0 + ni * 32 + 16 * fh;
          if (c0 >= p.c_out) continue;
          if constexpr (RES)
            store_kept_block_res<DT>(acc[mi][ni], rr[mi], c0, y, p.bias ? s_bias + (c0 - n0) : nullptr, 0, p.relu, 1,
                                     p.c_out, ho_wo, 0, 0, 0, static_cast<const T*>(p.residual), p.residual_relu);
          else
            store_kept_block<DT>(acc[mi][ni], rr[mi], c0, y, p.bias ? s_bias + (c0 - n0) : nullptr, 0, p.relu, 1,
                                 p.c_out, ho_wo, 0, 0, 0);
        }
      }
    }
  };

  // ---- steps: every thread passes steps + 1 barriers -------------------------------------------
  for (int k = 0; k <= steps; ++k) {
    v4i* slab_k = reinterpret_cast<v4i*>(s_x_bytes + (size_t)(k & 1) * x_bytes);
    if (grp == (k & 1)) {
      SC_PP_STAMP(k, 0);
      if (k < steps) transfer(band_at(k), slab_k);
      SC_PP_STAMP(k, 1);
      // everything this group has in flight: the slab (and, at k = 0, the filters), and the stores
      // of the band it computed in the previous step
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      SC_PP_STAMP(k, 2);
    } else {
      if (k == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this group's share of the filter slab
      SC_PP_STAMP(k, 4);
      if (k >= 1)
        compute(band_at(k - 1), reinterpret_cast<const v4i*>(s_x_bytes + (size_t)((k - 1) & 1) * x_bytes), k);
      SC_PP_STAMP(k, 5);
    }
    // LDS is the only memory the two groups share: wait for this wavefront's LDS operations, then
    // the barrier; no global-memory fence, so the stores of the band just computed keep draining
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    SC_PP_STAMP(k, 6);
  }
#ifdef SC_TIMING
  if (p.dbg && threadIdx.x == 0) p.dbg[(size_t)blockIdx.x * 128 + 121] = wall_clock64();
#endif
}

template <int DT, int NI, int MI, int KH, int KW, int CPP, bool RES = false>
hipError_t bandpp_launch(const BandParams& p, size_t lds, int grid, hipStream_t stream) {
  auto kern = bandpp_kernel<DT, NI, MI, KH, KW, CPP, RES>;
  static std::atomic<size_t> attr_bytes{0};   // (plans may be run from several host threads)
  if (lds > 64 * 1024 && lds > attr_bytes) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_bytes = lds;
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kPPThreads), lds, stream, p);
  return hipGetLastError();
}

using BandPPLaunchFn = hipError_t (*)(const BandParams&, size_t, int, hipStream_t);

// fn[shape 0: 3x3 window, 8 groups per pixel; 1: 3x3 window, 4 groups per pixel][NI - 1][MI - 1];
// fn_res: the same fused with a shortcut sum
struct BandPPTable { BandPPLaunchFn fn[2][2][2]; BandPPLaunchFn fn_res[2][2][2]; };
const BandPPTable* bandpp_bf16();
const BandPPTable* bandpp_f16();

#define SC_BANDPP_SHAPE(DT, CPP)                                                         \
  { { bandpp_launch<DT, 1, 1, 3, 3, CPP>, bandpp_launch<DT, 1, 2, 3, 3, CPP> },          \
    { bandpp_launch<DT, 2, 1, 3, 3, CPP>, bandpp_launch<DT, 2, 2, 3, 3, CPP> } }
#define SC_BANDPP_SHAPE_RES(DT, CPP)                                                                  \
  { { bandpp_launch<DT, 1, 1, 3, 3, CPP, true>, bandpp_launch<DT, 1, 2, 3, 3, CPP, true> },          \
    { bandpp_launch<DT, 2, 1, 3, 3, CPP, true>, bandpp_launch<DT, 2, 2, 3, 3, CPP, true> } }
#define SC_BANDPP_TABLE(DT) { { SC_BANDPP_SHAPE(DT, 8), SC_BANDPP_SHAPE(DT, 4) }, { SC_BANDPP_SHAPE_RES(DT, 8), SC_BANDPP_SHAPE_RES(DT, 4) } }

}  // namespace sc
