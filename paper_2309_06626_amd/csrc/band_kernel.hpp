// Band-staged masked convolution for layers whose filters fit in LDS next to a band of input.
//
// Paper Sec. 3.2: (i) lower only the kept windows, (ii) dense GEMM on fewer rows, (iii) put the
// results back with zeros in between.  Adjacent kept windows overlap (Fig. 2: a pixel masked for
// one window stays live for its neighbours), so a workgroup that owns a band of output rows of
// one image reads the union of its windows -- a contiguous slab of input rows -- from HBM exactly
// once, with fully coalesced 16-byte loads, into LDS.  The filter slab [32*NI channels][K] is
// staged once as well.  The lowering then happens inside LDS: each lane of an MFMA column operand
// fetches its own window entries with per-lane LDS addresses, only for kept rows.
//
//   workgroup  = one band (BH output rows x all Wo columns of one image) x 32*NI output channels
//   wavefront  = a contiguous quarter of the band's kept rows, 32*MI rows per MFMA block
//   LDS        = filter slab, then the input slab; 16-byte groups are XOR-swizzled
//                (q ^ ((q >> 4) & 7)) so that sixteen lanes reading the same channel group of
//                sixteen consecutive pixels / filter rows hit sixteen different bank groups
//   ownership  = the band's dense rows are exactly its output rows: the workgroup writes every
//                element of them once (results for kept rows, zeros for dropped rows).
#pragma once
#include "conv_params.hpp"
#include "mma_common.hpp"

namespace sc {

struct BandParams {
  const void* x;
  const void* wp;            // packed filters [cout_pad][k_stride]
  const float* bias;
  void* y;
  const int32_t* row_idx;    // ascending kept rows; null = dense run
  const uint8_t* mask;
  const int32_t* band_i0;    // [n_bands + 1]: first compacted row of every band (sparse runs)
  const int32_t* band_rows;  // [M]: the kept rows of band b, ascending, stored from index r_lo(b) on
  int32_t h, w, c_in, ho, wo, c_out;
  int32_t kh, kw, sh, sw, ph, pw, dil_h, dil_w;
  int32_t k_stride;          // elements between packed filter rows (odd multiple of the K tile)
  int32_t bh, bands_per_image, n_bands, n_tiles;
  int32_t split;             // alternating-group kernel: every run of bh rows is two bands of half its pixels
  int32_t b_bytes;           // LDS bytes of the filter slab
  int32_t x_groups;          // 16-byte groups reserved for the input slab (a zeroed KiB follows)
  int32_t relu, zero_fill, mask_spatial;
  // fused shortcut sum (alternating-group kernel, RES instantiations only): y = post(act(conv + bias) + residual),
  // residual in the dense layout of y; a dropped row receives post(residual)
  const void* residual;
  int32_t residual_relu;
  uint32_t div_wo_mul, div_wo_shift;   // n / wo as (n * mul) >> shift (tap-pipelined kernel)
#ifdef SC_TIMING
  long long* dbg;            // development builds only: per-workgroup phase time stamps
#endif
};

#ifdef SC_TIMING
#define SC_STAMP(slot) do { if (p.dbg && threadIdx.x == 0) p.dbg[(size_t)blockIdx.x * 8 + (slot)] = clock64(); } while (0)
#else
#define SC_STAMP(slot) do { } while (0)
#endif

// LDS has 64 banks of 4 bytes: a 128-bit read is conflict-free when 16 consecutive lanes cover 16
// different 16-byte bank groups.  Bit 3 of a group index already selects the bank half, so the low
// three bits are XORed with bits 4..6.
// tallest band (output rows x width) the band kernel accepts: its kept-row numbers are fetched up
// front into registers, kBandMaxRows / 256 per lane
constexpr int kBandMaxRows = 1024;

__device__ __forceinline__ int swz(int q) { return q ^ ((q >> 4) & 7); }

// 32-bit LDS addressing (keeps the per-fragment address arithmetic out of 64-bit registers)
typedef __attribute__((address_space(3))) unsigned char lds_byte;
__device__ __forceinline__ unsigned lds_addr_of(const void* generic_ptr) {
  return (unsigned)(unsigned long long)(lds_byte*)generic_ptr;
}
__device__ __forceinline__ v4i lds_load16(unsigned addr) {
  return *(const __attribute__((address_space(3))) v4i*)(lds_byte*)(unsigned long long)addr;
}

// KH/KW/CPP > 0 fix the window shape and the 16-byte groups per pixel at compile time so the whole
// K loop unrolls (LDS reads of later taps overlap the MFMAs of earlier ones); 0 = run-time shape.
template <int DT, int NI, int MI, int KH, int KW, int CPP>
__global__ __launch_bounds__(kThreads) void band_kernel(const BandParams p) {
  using E = Elem<DT>;
  using T = typename E::T;
  constexpr int V = E::V;
  constexpr int EB = sizeof(T);
  constexpr int BN = 32 * NI;
  constexpr int CPR = BN * EB / 16;     // 16-byte groups per output row slice
  constexpr int RPI = kThreads / CPR;   // output rows covered by one zero-fill pass of the workgroup
  constexpr int ZIT = 16;               // zero-fill passes whose mask bytes are fetched up front

  extern __shared__ __align__(16) unsigned char smem[];
  v4i* s_b = reinterpret_cast<v4i*>(smem);
  v4i* s_x = reinterpret_cast<v4i*>(smem + p.b_bytes);
  // behind the input slab: 1 KiB of zeros, then the bias slice
  float* s_bias = reinterpret_cast<float*>(smem + p.b_bytes + (size_t)p.x_groups * 16 + 1024);   // [BN]

  SC_STAMP(0);
#ifdef SC_TIMING
  const long long wall0 = wall_clock64();
#endif
  const int nwg = p.n_bands * p.n_tiles;
  const int per_xcd = (nwg + 7) >> 3;
  const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (logical >= nwg) return;
  const int band = logical / p.n_tiles;
  const int n0 = (logical - band * p.n_tiles) * BN;

  const int t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int fp = lane & 31, fh = lane >> 5;

  const int kh = KH ? KH : p.kh, kw = KW ? KW : p.kw;
  const int img = band / p.bands_per_image;
  const int oy0 = (band - img * p.bands_per_image) * p.bh;
  const int oy1 = min(oy0 + p.bh, p.ho);
  const int ho_wo = p.ho * p.wo;
  const int r_lo = img * ho_wo + oy0 * p.wo, r_hi = img * ho_wo + oy1 * p.wo;
  const int iy_base = oy0 * p.sh - p.ph;
  const int iy_lo = max(iy_base, 0);
  const int iy_hi = min((oy1 - 1) * p.sh - p.ph + (kh - 1) * p.dil_h + 1, p.h);
  const int cpp = CPP ? CPP : p.c_in / V;   // 16-byte groups per pixel
  const int kgr = p.k_stride / V;           // 16-byte groups per filter row

  const T* __restrict__ x = static_cast<const T*>(p.x);
  T* __restrict__ y = static_cast<T*>(p.y);

  // ---- small, latency-critical loads first, all independent of each other -----------------------
  // kept rows of the band: count from the band table, row numbers from the band-ordered list (its
  // address depends only on the band, not on the count); 64*MI rows per block, blocks dealt to the
  // wavefronts round robin; the first RB blocks of a wavefront are fetched here.
  constexpr int RB = kBandMaxRows / (4 * 32 * MI);   // blocks per wavefront that cover the tallest band
  int cnt = r_hi - r_lo;
  if (p.row_idx) cnt = p.band_i0[band + 1] - p.band_i0[band];
  int r_pre[RB][MI];
#pragma unroll
  for (int b = 0; b < RB; ++b)
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      const int j = ((b * 4 + wave) * MI + mi) * 32 + fp;     // position in the band's list (< band rows)
      const int jc = min(j, r_hi - r_lo - 1);
      r_pre[b][mi] = p.row_idx ? p.band_rows[r_lo + jc] : r_lo + jc;
    }
  // zero fill: thread (zr, zc) covers 16-byte group zc of rows r_lo + zr + u*RPI
  const int zc = t % CPR, zr = t / CPR;
  unsigned char mk[ZIT];

  float bias_v = 0.0f;
  if (t < BN && p.bias && n0 + t < p.c_out) bias_v = p.bias[n0 + t];

  // ---- stage the filter slab and the input slab: both are contiguous in global memory ----------
  const v4i* gb = reinterpret_cast<const v4i*>(static_cast<const T*>(p.wp) + (int64_t)n0 * p.k_stride);
  const int nb = BN * kgr;
  const v4i* gx = reinterpret_cast<const v4i*>(x + ((int64_t)(img * p.h + iy_lo) * p.w) * p.c_in);
  const int nx = max(iy_hi - iy_lo, 0) * p.w * cpp;
  const int qx0 = (iy_lo - iy_base) * p.w * cpp;   // LDS group of the first staged input group

  auto zero_fill = [&]() {
    // Alg. 2, mask == 0 branch: consecutive lanes write consecutive 16-byte groups of a dropped row
    const int valid = (min(BN, p.c_out - n0) * EB) >> 4;
    const v4i z = {0, 0, 0, 0};
    unsigned char* ybase = reinterpret_cast<unsigned char*>(y) + (int64_t)n0 * EB + zc * 16;
    if (zc < valid) {
#pragma unroll
      for (int u = 0; u < ZIT; ++u) {
        const int r = r_lo + zr + u * RPI;
        if (r < r_hi && mk[u] == 0) sc_store16(reinterpret_cast<v4i*>(ybase + (int64_t)r * p.c_out * EB), z);
      }
      for (int r = r_lo + zr + ZIT * RPI; r < r_hi; r += RPI)   // bands taller than ZIT passes
        if (p.mask[p.mask_spatial ? r - img * ho_wo : r] == 0)
          sc_store16(reinterpret_cast<v4i*>(ybase + (int64_t)r * p.c_out * EB), z);
    }
  };

  // Both slabs go straight from global memory into LDS (no register staging): one wavefront
  // instruction fills 64 consecutive 16-byte LDS groups, lane l the group base + l.  The swizzle is
  // an involution inside every aligned block of 64 groups, so the lane that owns LDS group q fetches
  // global group swz(q); the 64 fetches still cover one contiguous KiB.
  __builtin_amdgcn_sched_barrier(0);   // the small loads above stay ahead of the slab transfers
  auto dma16 = [](const v4i* src, v4i* lds_base) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                     (__attribute__((address_space(3))) void*)lds_base, 16, 0, 0);
  };
  for (int qb = wave * 64; qb < nb; qb += kThreads) dma16(gb + swz(qb + lane), s_b + qb);
  {
    const int q_end = qx0 + nx;
    for (int qb = (qx0 & ~63) + wave * 64; qb < q_end; qb += kThreads) {
      const int g = swz(qb + lane) - qx0;
      if (g >= 0 && g < nx) dma16(gx + g, s_x + qb);
    }
  }
  // the mask bytes of the zero fill, behind the transfers: the compiler packs them four to a register and waits for
  // them right here, which must not hold back the issue of the slabs
  if (p.zero_fill) {
#pragma unroll
    for (int u = 0; u < ZIT; ++u) {
      const int r = min(r_lo + zr + u * RPI, r_hi - 1);       // clamped: the loads stay unconditional
      mk[u] = p.mask[p.mask_spatial ? r - img * ho_wo : r];
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  if (t < 64) {
    const v4i z = {0, 0, 0, 0};
    s_x[p.x_groups + t] = z;
  }
  if (t < BN) s_bias[t] = bias_v;

  SC_STAMP(1);
#ifdef SC_TIMING
  if (p.dbg && threadIdx.x == 0) p.dbg[(size_t)blockIdx.x * 8 + 2] = wall0;
#endif
  __syncthreads();   // slabs staged
  SC_STAMP(3);
  // the zero stores are issued now and drain while the matrix cores work; nothing waits for them
  if (p.zero_fill) zero_fill();

  const int zq = p.x_groups;          // a zeroed 16-byte group behind the input slab
  const int nblk = (cnt + 32 * MI - 1) / (32 * MI);
#pragma unroll
  for (int bi = 0; bi < RB; ++bi) {
    const int blk = bi * 4 + wave;
    if (blk >= nblk) break;
    int rr[MI], ly0[MI], lx0[MI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      const int j = (blk * MI + mi) * 32 + fp;
      rr[mi] = -1;
      ly0[mi] = 0;
      lx0[mi] = -(1 << 28);   // no tap of an absent row is ever in range
      if (j < cnt) {
        const int r = r_pre[bi][mi];
        const int rem = r - img * ho_wo;
        const int oy = rem / p.wo, ox = rem - oy * p.wo;
        rr[mi] = r;
        ly0[mi] = oy * p.sh - p.ph - iy_base;
        lx0[mi] = ox * p.sw - p.pw;
      }
    }
    floatx16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;
    SC_STAMP(5);

    // LDS group of the window entry (ky, kx, channel group c) of this lane's rows; taps outside the
    // image (zero padding) and absent rows point at the zeroed group instead.
    auto xgroup = [&](int mi, int ky, int kx, int c) -> int {
      const int ly = ly0[mi] + ky * p.dil_h, ix = lx0[mi] + kx * p.dil_w;
      const bool ok = (unsigned)(iy_base + ly) < (unsigned)p.h && (unsigned)ix < (unsigned)p.w;
      return ok ? swz((ly * p.w + ix) * cpp + c) : zq;
    };
    auto wgroup = [&](int ni, int kc) -> int { return swz((ni * 32 + fp) * kgr + kc); };

    if constexpr (KH > 0) {
      // K steps of 32 bytes per row, in groups of G; the fragments of group g+1 are read while the
      // MFMAs of group g run.  CPP is a power of two here, so the swizzled byte address of channel
      // group c of a pixel is (pixel base) ^ (c << 4): one XOR per fragment read.
      static_assert((CPP & (CPP - 1)) == 0 && CPP <= 8, "power-of-two groups per pixel");
      constexpr int SPT = CPP / 2;            // steps per tap
      constexpr int S = KH * KW * SPT;
      constexpr int G = 4;
      constexpr int NG = (S + G - 1) / G;
      const unsigned xbase = lds_addr_of(s_x), zaddr = xbase + (unsigned)p.x_groups * 16u;
      const unsigned bbase = lds_addr_of(s_b);
      unsigned tap_addr[MI][KH * KW];         // address of channel group fh of every tap's pixel
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        const int pb = ly0[mi] * p.w + lx0[mi];
#pragma unroll
        for (int ky = 0; ky < KH; ++ky) {
          const bool oky = (unsigned)(iy_base + ly0[mi] + ky * p.dil_h) < (unsigned)p.h;
#pragma unroll
          for (int kx = 0; kx < KW; ++kx) {
            const bool ok = oky && (unsigned)(lx0[mi] + kx * p.dil_w) < (unsigned)p.w;
            const unsigned g0 = (unsigned)(pb + ky * p.dil_h * p.w + kx * p.dil_w) * CPP;
            const unsigned rel = ((g0 ^ ((g0 >> 4) & 7u)) << 4) ^ ((unsigned)fh << 4);
            tap_addr[mi][ky * KW + kx] = ok ? xbase + rel : zaddr;
          }
        }
      }
      unsigned w_q0[NI];                      // LDS group of K group 0 of this lane's filter rows
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) w_q0[ni] = (unsigned)((ni * 32 + fp) * kgr);
      v4i xb[2][G][MI], wb[2][G][NI];
      auto load_group = [&](int g, v4i (&xd)[G][MI], v4i (&wd)[G][NI]) {
#pragma unroll
        for (int e = 0; e < G; ++e) {
          const int st = g * G + e;
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
      load_group(0, xb[0], wb[0]);
#pragma unroll
      for (int g = 0; g < NG; ++g) {
        // One scheduling region per group: the read-ahead of group g+1 is interleaved with the MFMAs
        // of group g, one LDS read behind every MFMA, so neither the LDS queue nor the matrix pipe
        // waits for a burst of the other.
        __builtin_amdgcn_sched_barrier(0);
        if (g + 1 < NG) load_group(g + 1, xb[(g + 1) & 1], wb[(g + 1) & 1]);
#pragma unroll
        for (int e = 0; e < G; ++e) {
          if (g * G + e < S) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
              for (int ni = 0; ni < NI; ++ni) E::mma(acc[mi][ni], wb[g & 1][e][ni], xb[g & 1][e][mi]);
          }
        }
        if (g + 1 < NG) {
#pragma unroll
          for (int i = 0; i < G * MI * NI; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    } else {
      // run-time window: one K step at a time, the next step's fragments read ahead
      int ky = 0, kx = 0, j = 0;
      v4i xn[MI];
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) xn[mi] = s_x[xgroup(mi, 0, 0, fh)];
      const int steps = kh * kw * (cpp >> 1);
      for (int st = 0; st < steps; ++st) {
        v4i xf[MI], wf[NI];
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) xf[mi] = xn[mi];
        const int kc = (ky * kw + kx) * cpp + j + fh;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) wf[ni] = s_b[wgroup(ni, kc)];
        j += 2;
        if (j >= cpp) { j = 0; if (++kx == kw) { kx = 0; ++ky; } }
        if (st + 1 < steps) {
#pragma unroll
          for (int mi = 0; mi < MI; ++mi) xn[mi] = s_x[xgroup(mi, ky, kx, j + fh)];
        }
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
          for (int ni = 0; ni < NI; ++ni) E::mma(acc[mi][ni], wf[ni], xf[mi]);
      }
    }

    SC_STAMP(6);
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      if (rr[mi] < 0) continue;
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) {
        const int c0 = n0 + ni * 32 + 16 * fh;
        if (c0 >= p.c_out) continue;
        store_kept_block<DT>(acc[mi][ni], rr[mi], c0, y, p.bias ? s_bias + (c0 - n0) : nullptr, 0, p.relu, 1,
                             p.c_out, ho_wo, 0, 0, 0);
      }
    }
  }
  SC_STAMP(4);
#ifdef SC_TIMING
  if (p.dbg && threadIdx.x == 0) p.dbg[(size_t)blockIdx.x * 8 + 7] = wall_clock64();
#endif
}

template <int DT, int NI, int MI, int KH, int KW, int CPP>
hipError_t band_launch(const BandParams& p, size_t lds, hipStream_t stream) {
  auto kern = band_kernel<DT, NI, MI, KH, KW, CPP>;
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

using BandLaunchFn = hipError_t (*)(const BandParams&, size_t, hipStream_t);

// fn[shape][ni index 0..2 -> NI 1,2,4][mi index 0..1 -> MI 1,2]
// shape 0: run-time window; 1: 3x3 window, 8 groups per pixel; 2: 3x3 window, 4 groups per pixel
struct BandTable { BandLaunchFn fn[3][3][2]; };
const BandTable* band_bf16();
const BandTable* band_f16();
const BandTable* band_f32();

// Unrolled window shapes exist for one and two filter blocks; four filter blocks keep the run-time
// loops (the unrolled form exceeds the register file).
#define SC_BAND_SHAPE(DT, KH, KW, CPP)                                                        \
  { { band_launch<DT, 1, 1, KH, KW, CPP>, band_launch<DT, 1, 2, KH, KW, CPP> },               \
    { band_launch<DT, 2, 1, KH, KW, CPP>, band_launch<DT, 2, 2, KH, KW, CPP> },               \
    { band_launch<DT, 4, 1, 0, 0, 0>, band_launch<DT, 4, 2, 0, 0, 0> } }

#define SC_BAND_TABLE(DT) { { SC_BAND_SHAPE(DT, 0, 0, 0), SC_BAND_SHAPE(DT, 3, 3, 8), SC_BAND_SHAPE(DT, 3, 3, 4) } }

}  // namespace sc
