// Band kernel whose matrix work starts while most of its filters are still to come (3x3 windows, 16-bit types).
//
// Same decomposition as band_kernel.hpp (Sec. 3.2: the kept windows of a band of output rows are lowered
// inside LDS, the GEMM runs on the kept rows only, the band's owner writes results and zeros), but the
// phases that kernel runs one after the other -- all transfers, then all MFMAs, then all stores -- overlap:
//
//   * the filter slab lies tap-major in LDS ([tap][filter row][channel group]), so the filters of one window
//     row (three taps) are three contiguous blocks, one transfer instruction per wavefront and tap for
//     64 x 64 channels.  Up front a wavefront issues only what the first window row needs: the band's
//     kept-row list and count, the bias slice, the input slab and taps 0-2.  A wavefront that issues more than
//     the memory pipeline takes sits in the issue stage until it drains (measured: issuing everything up
//     front cost as long as the transfers themselves), so the taps of window row g+1 are issued one behind each
//     of the first MFMA steps of window row g and land under its matrix work;
//   * the K loop is tap-major over all of a wavefront's rows, three taps between barriers; fragments are read
//     from LDS two K steps ahead of the MFMAs that consume them;
//   * nothing a wavefront needs comes through a register or scalar load after the kernel arguments: row
//     numbers, the band's kept count, bias and the dropped-row map are read from LDS, where transfers put them --
//     a dependent round trip to memory before the first transfer (the count) cost more than a microsecond;
//   * every wait for transfers is "all of mine have landed" followed by a workgroup barrier: no assumption about
//     the order in which memory operations complete;
//   * the zeros of the dropped rows are issued once every transfer has landed (before the MFMAs of the last
//     window row) and drain under them.
//
//   workgroup  = 8 wavefronts, one band (BH output rows x all Wo columns of one image) x 32*NI channels
//   wavefront  = 32-row MFMA blocks b = wave, wave + 8 (RB of them) of the band's kept rows, all channels
//   LDS        = filters [9 taps][32*NI rows][CPP groups] | 1 KiB of zeros | bias, kept count | row list |
//                dropped-row map | input slab; 16-byte groups swizzled q ^ ((q >> 4) & 7) as in band_kernel.hpp
#pragma once
#include <type_traits>

#include "band_kernel.hpp"
#include "igemm_dma_kernel.hpp"

namespace sc {

constexpr int kTapThreads = 512;
constexpr int kTapWaves = kTapThreads / 64;
constexpr int kTapMaxRows = 512;                 // tallest band (output rows x width)
// LDS between the filter slab and the input slab: zeros, bias (then the band's first and last compact row), row
// list, dropped-row map
constexpr int kTapZeroAt = 0, kTapBiasAt = 1024, kTapCountAt = 1024 + 384, kTapListAt = 1536,
              kTapKeepAt = 1536 + 4 * kTapMaxRows;
constexpr int kTapFixedLds = kTapKeepAt + kTapMaxRows;

template <int I, int N, class F> __device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}
template <int OFF> __device__ __forceinline__ v4i lds_read16_far(unsigned addr) {   // the offset field holds 16 bits
  if constexpr (OFF < 65536) return lds_read16_at<OFF>(addr);
  else return lds_read16_at<0>(addr + (unsigned)OFF);
}
__device__ __forceinline__ int lds_read4(unsigned addr) {
  int v;
  asm volatile("ds_read_b32 %0, %1" : "=v"(v) : "v"(addr));
  return v;
}
__device__ __forceinline__ int lds_read1(unsigned addr) {
  int v;
  asm volatile("ds_read_u8 %0, %1" : "=v"(v) : "v"(addr));
  return v;
}
__device__ __forceinline__ void lds_write16(unsigned addr, v4i v) {
  asm volatile("ds_write_b128 %0, %1" ::"v"(addr), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_write1(unsigned addr, int v) {
  asm volatile("ds_write_b8 %0, %1" ::"v"(addr), "v"(v) : "memory");
}
// all LDS operations of this wavefront have completed; the values pass through so that no use moves above
__device__ __forceinline__ void wait_lds(int& a) { asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a)); }
__device__ __forceinline__ void wait_lds(int& a, int& b) { asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a), "+v"(b)); }
__device__ __forceinline__ void wait_lds() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

#ifdef SC_TIMING
#define SC_TAP_STAMP(slot) do { ts[slot] = clock64(); } while (0)
#else
#define SC_TAP_STAMP(slot) do { } while (0)
#endif

// RES: the run is fused with the shortcut sum that follows it (sparse_conv_run_residual): the epilogue adds the
// shortcut tensor in float before the one rounding, and dropped rows receive post(shortcut) instead of zeros.
template <int DT, int NI, int CPP, int RB, bool RES = false>
__global__ __launch_bounds__(kTapThreads) void bandtap_kernel(const BandParams p) {
#ifdef SC_TIMING
  long long ts[16] = {};            // development builds only: phase time stamps, kept in registers until the end
  const long long wall0 = wall_clock64();
  SC_TAP_STAMP(0);
#endif
  using E = Elem<DT>;
  using T = typename E::T;
  constexpr int V = E::V;
  constexpr int EB = sizeof(T);
  constexpr int BN = 32 * NI;
  constexpr int TAPS = 9;
  constexpr int SPT = CPP / 2;                      // K steps (two 16-byte groups) per tap
  constexpr int GST = 3 * SPT;                      // K steps per window row
  constexpr int TAP_GROUPS = BN * CPP;              // 16-byte groups of one tap's filter block
  constexpr int TAP_INSTR = TAP_GROUPS / 64;        // transfer instructions per tap: wavefronts 0 .. TAP_INSTR-1
  constexpr int CPR = BN * EB / 16;                 // 16-byte groups per output row slice
  constexpr int RPI = kTapThreads / CPR;            // output rows covered by one zero-fill pass
  static_assert(EB == 2 && (CPP == 4 || CPP == 8) && (NI == 1 || NI == 2) && (RB == 1 || RB == 2), "shapes");
  static_assert(TAP_GROUPS % 64 == 0 && TAP_INSTR <= kTapWaves, "one transfer per wavefront and tap at most");

  // every kernel argument a later address depends on, fetched in the first round trip
  asm volatile("" ::"s"(p.x), "s"(p.wp), "s"(p.bias), "s"(p.y), "s"(p.row_idx), "s"(p.band_i0), "s"(p.band_rows),
               "s"(p.n_bands), "s"(p.n_tiles), "s"(p.k_stride), "s"(p.bh), "s"(p.bands_per_image));

  extern __shared__ __align__(16) unsigned char smem[];
  const unsigned lds0 = lds_addr_of(smem);
  constexpr unsigned B_BYTES = TAPS * TAP_GROUPS * 16;
  const unsigned zaddr = lds0 + B_BYTES + kTapZeroAt;
  float* s_bias = reinterpret_cast<float*>(smem + B_BYTES + kTapBiasAt);      // filled by a transfer, read in the epilogue
  int32_t* s_count = reinterpret_cast<int32_t*>(smem + B_BYTES + kTapCountAt);
  int32_t* s_list = reinterpret_cast<int32_t*>(smem + B_BYTES + kTapListAt);
  const unsigned list_addr = lds0 + B_BYTES + kTapListAt, keep_addr = lds0 + B_BYTES + kTapKeepAt;
  v4i* s_x = reinterpret_cast<v4i*>(smem + B_BYTES + kTapFixedLds);
  const unsigned xbase = lds0 + B_BYTES + kTapFixedLds;

  const int nwg = p.n_bands * p.n_tiles;
  const int per_xcd = (nwg + 7) >> 3;
  const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (logical >= nwg) return;
  const int band = logical / p.n_tiles;
  const int n0 = (logical - band * p.n_tiles) * BN;

  const int t = threadIdx.x;
  const int lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int fp = lane & 31, fh = lane >> 5;

  const int img = band / p.bands_per_image;
  const int oy0 = (band - img * p.bands_per_image) * p.bh;
  const int oy1 = min(oy0 + p.bh, p.ho);
  const int ho_wo = p.ho * p.wo;
  const int r_lo = img * ho_wo + oy0 * p.wo, r_hi = img * ho_wo + oy1 * p.wo;
  const int npx = r_hi - r_lo;
  const int iy_base = oy0 * p.sh - p.ph;
  const int iy_lo = max(iy_base, 0);
  const int iy_hi = min((oy1 - 1) * p.sh - p.ph + 2 * p.dil_h + 1, p.h);

  const T* __restrict__ x = static_cast<const T*>(p.x);
  T* __restrict__ y = static_cast<T*>(p.y);
  const bool sparse = p.row_idx != nullptr;

  typedef __attribute__((address_space(1))) void gvoid;
  typedef __attribute__((address_space(3))) void lvoid;

  // ---- transfers of the first window row, smallest first -----------------------------------------------------
  if (wave == 1 && sparse && lane < 2)      // first compact row of this band and of the next: their difference is the count
    __builtin_amdgcn_global_load_lds((const gvoid*)(p.band_i0 + band + lane), (lvoid*)s_count, 4, 0, 0);
  if (wave == 0 && p.bias) {
    const int c = min(n0 + lane, p.c_out - 1);        // lanes past the last channel re-read it; never used
    __builtin_amdgcn_global_load_lds((const gvoid*)(p.bias + c), (lvoid*)s_bias, 4, 0, 0);
  }
  if (sparse) {
    // the band's kept rows, ascending, stored from index r_lo of the band-ordered list (entries past the
    // band's count belong to nobody; they stay inside the list and are never used)
    const int j = min(wave * 64 + lane, npx - 1);
    __builtin_amdgcn_global_load_lds((const gvoid*)(p.band_rows + r_lo + j), (lvoid*)(s_list + wave * 64), 4, 0, 0);
  }
  {
    const v4i* gx = reinterpret_cast<const v4i*>(x + ((int64_t)(img * p.h + iy_lo) * p.w) * p.c_in);
    const int nx = max(iy_hi - iy_lo, 0) * p.w * CPP;
    const int qx0 = (iy_lo - iy_base) * p.w * CPP;    // LDS group of the first staged input group
    const int q_end = qx0 + nx;
    for (int qb = (qx0 & ~63) + wave * 64; qb < q_end; qb += kTapThreads) {
      const int q = swz(qb + lane) - qx0;
      if (q >= 0 && q < nx)
        __builtin_amdgcn_global_load_lds((const gvoid*)(gx + q), (lvoid*)(s_x + qb), 16, 0, 0);
    }
  }
  __builtin_amdgcn_sched_barrier(0);
  // LDS group q of a tap block = (filter row q / CPP, physical group q % CPP); it receives logical group
  // swz(q) of the block, i.e. 16 bytes of filter row n0 + swz(q) / CPP at K group tap * CPP + swz(q) % CPP
  const int fg = swz((wave & (TAP_INSTR - 1)) * 64 + lane);
  const T* f_src = static_cast<const T*>(p.wp) + (int64_t)(n0 + fg / CPP) * p.k_stride + (fg % CPP) * V;
  unsigned char* f_dst = smem + (wave & (TAP_INSTR - 1)) * 1024;
  auto issue_tap = [&](auto tp_c) {
    constexpr int TP = decltype(tp_c)::value;
    if (wave < TAP_INSTR)
      __builtin_amdgcn_global_load_lds((const gvoid*)(f_src + TP * CPP * V), (lvoid*)(f_dst + TP * TAP_GROUPS * 16), 16, 0, 0);
  };
  issue_tap(std::integral_constant<int, 0>{});
  issue_tap(std::integral_constant<int, 1>{});
  issue_tap(std::integral_constant<int, 2>{});
  __builtin_amdgcn_sched_barrier(0);
  // LDS the transfers do not touch: the zeroed KiB (source of padded taps and absent rows) and the map of kept
  // pixels, cleared here and marked from the row list below
  {
    const v4i z = {0, 0, 0, 0};
    if (t < 64) lds_write16(zaddr + t * 16, z);
    if (t >= 64 && t < 64 + kTapMaxRows / 16) lds_write16(keep_addr + (t - 64) * 16, z);
  }
  // filter fragment of row ni*32 + fp: group q = row * CPP + c sits at q ^ ((q >> 4) & 7); the key does not
  // depend on c (c < CPP, the row part has zero low bits) nor on the tap (a tap block is a multiple of 64 groups)
  unsigned w_addr[NI];
#pragma unroll
  for (int ni = 0; ni < NI; ++ni) {
    const unsigned q = (unsigned)((ni * 32 + fp) * CPP) + (unsigned)fh;
    w_addr[ni] = lds0 + ((q ^ ((q >> 4) & 7u)) << 4);
  }
  floatx16 acc[RB][NI];
#pragma unroll
  for (int bi = 0; bi < RB; ++bi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[bi][ni][v] = 0.0f;

  SC_TAP_STAMP(1);
  // ---- count, bias, row list, slab and taps 0-2 have landed --------------------------------------------------
  wait_vmcnt<0>();
  wait_lds();
  SC_TAP_STAMP(2);
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  SC_TAP_STAMP(3);

  // this lane's rows: one per 32-row block; LDS address of channel group fh of every tap's pixel
  int cnt = npx;                                      // kept rows of the band
  int rr[RB];
  unsigned tap_addr[RB][TAPS];
  {
    int rj[RB];
    int i0 = 0, i1 = 0;
    if (sparse) {
      i0 = lds_read4(lds0 + B_BYTES + kTapCountAt);
      i1 = lds_read4(lds0 + B_BYTES + kTapCountAt + 4);
    }
#pragma unroll
    for (int bi = 0; bi < RB; ++bi) {
      const int j = (bi * kTapWaves + wave) * 32 + fp;
      rj[bi] = r_lo + min(j, npx - 1);
      if (sparse) rj[bi] = lds_read4(list_addr + 4 * min(j, kTapMaxRows - 1));
    }
    int rk = 0;
    if (sparse && p.zero_fill) rk = lds_read4(list_addr + 4 * t);
    if (sparse) {
      wait_lds(i0, i1);
      cnt = __builtin_amdgcn_readfirstlane(i1 - i0);
    }
    if (sparse && p.zero_fill) {
      // dropped-row map: one byte per band pixel, set for the kept ones (Alg. 2 zero-fills the others)
      wait_lds(rk);
      if (t < cnt) lds_write1(keep_addr + (rk - r_lo), 1);
    }
#pragma unroll
    for (int bi = 0; bi < RB; ++bi) {
      if (sparse) wait_lds(rj[bi]);
      const int j = (bi * kTapWaves + wave) * 32 + fp;
      const bool have = j < cnt;
      const int rem = rj[bi] - img * ho_wo;
      const int oy = have ? fast_div(rem, p.div_wo_mul, p.div_wo_shift) : 0, ox = rem - oy * p.wo;
      rr[bi] = have ? rj[bi] : -1;
      const int ly0 = oy * p.sh - p.ph - iy_base;
      const int lx0 = ox * p.sw - p.pw;
      const int pb = ly0 * p.w + lx0;
#pragma unroll
      for (int ky = 0; ky < 3; ++ky) {
        const bool oky = have && (unsigned)(iy_base + ly0 + ky * p.dil_h) < (unsigned)p.h;
#pragma unroll
        for (int kx = 0; kx < 3; ++kx) {
          const bool ok = oky && (unsigned)(lx0 + kx * p.dil_w) < (unsigned)p.w;
          const unsigned g0 = (unsigned)(pb + ky * p.dil_h * p.w + kx * p.dil_w) * CPP;
          const unsigned rel = ((g0 ^ ((g0 >> 4) & 7u)) << 4) ^ ((unsigned)fh << 4);
          tap_addr[bi][ky * 3 + kx] = ok ? xbase + rel : zaddr;
        }
      }
    }
    wait_lds();      // the map is complete before this wavefront passes the next barrier (zero_fill reads it after the last)
  }
  SC_TAP_STAMP(4);
  const int nblk = (cnt + 31) >> 5;
  const bool work0 = wave < nblk, work1 = RB > 1 && wave + kTapWaves < nblk;

  // fragments of K step S (tap S / SPT, groups 2 * (S % SPT) + fh) for the first NB blocks of this wavefront: the
  // window entries of this lane's rows, then the filter rows
  auto read_step = [&](auto s_c, auto nb_c, v4i* f) {
    constexpr int S = decltype(s_c)::value, NB = decltype(nb_c)::value;
    constexpr int TP = S / SPT;
    constexpr unsigned cx = (unsigned)(2 * (S % SPT)) << 4;
#pragma unroll
    for (int bi = 0; bi < NB; ++bi) f[bi] = lds_read16_at<0>(tap_addr[bi][TP] ^ cx);
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) f[NB + ni] = lds_read16_far<TP * TAP_GROUPS * 16>(w_addr[ni] ^ cx);
  };
  // Window row G for NB blocks: fragments are read two K steps ahead; behind each of the first three steps'
  // MFMAs one tap of the next window row is requested (the issue slot is free while the matrix pipeline works).
  // Alg. 2, mask == 0 branch: consecutive lanes write consecutive 16-byte groups of a dropped row.  Pass u covers
  // rows r_lo + zr + u * RPI; the passes ride behind the MFMA steps of the last window row, one store
  // instruction per step, so the store queue fills while the matrix pipeline works.
  constexpr int ZP = kTapMaxRows / RPI;
  const int zc = t % CPR, zr = t / CPR;
  const bool zvalid = zc < ((min(BN, p.c_out - n0) * EB) >> 4);
  int kp[ZP];
  auto zero_prepare = [&]() {
#pragma unroll
    for (int u = 0; u < ZP; ++u) kp[u] = lds_read1(keep_addr + min(zr + u * RPI, kTapMaxRows - 1));
#pragma unroll
    for (int u = 0; u < ZP; ++u) wait_lds(kp[u]);
  };
  auto zero_pass = [&](auto u_c) {
    constexpr int U = decltype(u_c)::value;
    if constexpr (U < ZP) {
      const int r = r_lo + zr + U * RPI;
      if (zvalid && r < r_hi && kp[U] == 0) {
        const int64_t col_at = (int64_t)n0 * EB + zc * 16;      // byte offset of this thread's group inside a row
        const int64_t at = (int64_t)r * p.c_out * EB;
        v4i* dst = reinterpret_cast<v4i*>(reinterpret_cast<unsigned char*>(y) + col_at + at);
        if constexpr (RES) sc_store16(dst, dropped_row_group<DT>(p.residual, col_at + at, p.residual_relu));
        else sc_store16(dst, v4i{0, 0, 0, 0});
      }
    }
  };

  constexpr int ZPS = (ZP + GST - 1) / GST;      // zero-fill passes per K step of the last window row
  const bool filling = sparse && p.zero_fill;
  auto row_mma = [&](auto g_c, auto nb_c) {
    constexpr int G = decltype(g_c)::value, NB = decltype(nb_c)::value;
    constexpr int S0 = G * GST;
    v4i f[3][NB + NI];
    read_step(std::integral_constant<int, S0>{}, nb_c, f[0]);
    if constexpr (GST > 1) read_step(std::integral_constant<int, S0 + 1>{}, nb_c, f[1]);
    static_for<0, GST>([&](auto i_c) {
      constexpr int I = decltype(i_c)::value;
      if constexpr (I + 2 < GST) read_step(std::integral_constant<int, S0 + I + 2>{}, nb_c, f[(I + 2) % 3]);
      constexpr int AHEAD = (I + 2 < GST ? 2 : GST - 1 - I) * (NB + NI);     // reads younger than those of step I
      wait_frags<AHEAD>(f[I % 3]);
#pragma unroll
      for (int bi = 0; bi < NB; ++bi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) E::mma(acc[bi][ni], f[I % 3][NB + ni], f[I % 3][bi]);
      if constexpr (G < 2 && I < 3) {
        __builtin_amdgcn_sched_barrier(0);
        issue_tap(std::integral_constant<int, 3 * (G + 1) + I>{});
        __builtin_amdgcn_sched_barrier(0);
      }
      if constexpr (G == 2 && I * ZPS < ZP) {
        __builtin_amdgcn_sched_barrier(0);
        if (filling) static_for<I * ZPS, (I + 1) * ZPS>(zero_pass);
        __builtin_amdgcn_sched_barrier(0);
      }
    });
  };

  // ---- K loop: three window rows ----------------------------------------------------------------------------------
  auto window_row = [&](auto g_c) {
    constexpr int G = decltype(g_c)::value;
    if constexpr (G > 0) {
      wait_vmcnt<0>();                   // this wavefront's taps of window row G have landed ...
      __builtin_amdgcn_s_barrier();      // ... and everybody else's
      asm volatile("" ::: "memory");
    }
    if constexpr (G == 2) {
      // every transfer has landed: whatever this wavefront stores from here on competes with nothing it waits for
      if (filling) zero_prepare();
    }
    if constexpr (RB == 2) {
      if (work1) row_mma(g_c, std::integral_constant<int, 2>{});
      else if (work0) row_mma(g_c, std::integral_constant<int, 1>{});
    } else {
      if (work0) row_mma(g_c, std::integral_constant<int, 1>{});
    }
    if constexpr (G < 2) {
      // wavefronts without rows still fetch their share of the next window row's filters
      if (!work0) static_for<0, 3>([&](auto i_c) { issue_tap(std::integral_constant<int, 3 * (G + 1) + decltype(i_c)::value>{}); });
    } else {
      if (!work0 && filling) static_for<0, ZP>(zero_pass);      // ... and write their share of the zeros
    }
    __builtin_amdgcn_sched_barrier(0);
    SC_TAP_STAMP(5 + G);
  };
  window_row(std::integral_constant<int, 0>{});
  window_row(std::integral_constant<int, 1>{});
  window_row(std::integral_constant<int, 2>{});

  // ---- epilogue -----------------------------------------------------------------------------------------------
  // (the bias slice comes out of LDS through explicit reads as well: a compiler-managed LDS read would first wait
  // for every outstanding vector-memory operation, i.e. for the zero stores that are meant to drain on their own)
#pragma unroll
  for (int ni = 0; ni < NI; ++ni) {
    const int c0 = n0 + ni * 32 + 16 * fh;
    float bl[16];
    if (p.bias) {
      v4i b4[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) b4[q] = lds_read16_at<0>(lds0 + B_BYTES + kTapBiasAt + (unsigned)(c0 - n0) * 4 + q * 16);
      wait_frags<0>(b4);
      __builtin_memcpy(bl, b4, 64);
    }
#pragma unroll
    for (int bi = 0; bi < RB; ++bi) {
      if (rr[bi] < 0 || c0 >= p.c_out) continue;
      if constexpr (RES)
        store_kept_block_res<DT>(acc[bi][ni], rr[bi], c0, y, p.bias ? bl : nullptr, 0, p.relu, 1, p.c_out, ho_wo, 0, 0, 0,
                                 static_cast<const T*>(p.residual), p.residual_relu);
      else
        store_kept_block<DT>(acc[bi][ni], rr[bi], c0, y, p.bias ? bl : nullptr, 0, p.relu, 1, p.c_out, ho_wo, 0, 0, 0);
    }
  }
#ifdef SC_TIMING
  SC_TAP_STAMP(8);
  if (p.dbg && (threadIdx.x & 63) == 0 && wave < 2) {
    long long* out = p.dbg + ((size_t)blockIdx.x * 2 + wave) * 32;
#pragma unroll
    for (int i = 0; i < 15; ++i) out[i] = ts[i];
    out[15] = wall0;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    out[16] = wall_clock64();
  }
#endif
}

template <int DT, int NI, int CPP, int RB, bool RES = false>
hipError_t bandtap_launch(const BandParams& p, size_t lds, hipStream_t stream) {
  auto kern = bandtap_kernel<DT, NI, CPP, RB, RES>;
  static std::atomic<size_t> attr_bytes{0};   // (plans may be run from several host threads)
  if (lds > 64 * 1024 && lds > attr_bytes) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_bytes = lds;
  }
  const int nwg = p.n_bands * p.n_tiles;
  const int grid = ((nwg + 7) / 8) * 8;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kTapThreads), lds, stream, p);
  return hipGetLastError();
}

// fn[0: 8 groups per pixel, 1: 4 groups per pixel][NI - 1][RB - 1]; fn_res: the same fused with a shortcut sum
struct BandTapTable { BandLaunchFn fn[2][2][2]; BandLaunchFn fn_res[2][2][2]; };
const BandTapTable* bandtap_bf16();
const BandTapTable* bandtap_f16();

#define SC_BANDTAP_SHAPE(DT, CPP)                                                    \
  { { bandtap_launch<DT, 1, CPP, 1>, bandtap_launch<DT, 1, CPP, 2> },                \
    { bandtap_launch<DT, 2, CPP, 1>, bandtap_launch<DT, 2, CPP, 2> } }
#define SC_BANDTAP_SHAPE_RES(DT, CPP)                                                            \
  { { bandtap_launch<DT, 1, CPP, 1, true>, bandtap_launch<DT, 1, CPP, 2, true> },                \
    { bandtap_launch<DT, 2, CPP, 1, true>, bandtap_launch<DT, 2, CPP, 2, true> } }
#define SC_BANDTAP_TABLE(DT) { { SC_BANDTAP_SHAPE(DT, 8), SC_BANDTAP_SHAPE(DT, 4) }, { SC_BANDTAP_SHAPE_RES(DT, 8), SC_BANDTAP_SHAPE_RES(DT, 4) } }

}  // namespace sc
