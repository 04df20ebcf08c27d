// Tiled masked-convolution kernel with direct global-to-LDS gathers (NHWC, 16-byte channel groups).
//
// Same decomposition as igemm_kernel (paper Sec. 3.2 stages i-iii fused; workgroup = BM kept rows x
// BN channels, 32x32 MFMA blocks, filters as the MFMA row operand), but the K tiles never pass
// through registers: every lane fetches its 16 bytes of a kept row's window (or of a filter row)
// with global_load_lds into a ring of STAGES LDS tiles, STAGES-1 tiles ahead of the MFMAs.
//
// A wavefront instruction fills 64 consecutive 16-byte LDS groups = 8 tile rows of 128 bytes, lane
// l the group l, so the bank swizzle (group ^ ((row >> 1) & 7)) is applied to the *global* address:
// the lane that owns physical group c of a row fetches logical group c ^ key.  Lanes whose window
// entry lies in the zero padding, past K, or in an absent row fetch from a page of zeros.
//
// The compiler cannot see which LDS tile a transfer fills and would wait for all of them before any
// LDS read, so the waits are explicit: vmcnt for "tile kt has landed" (transfers of later tiles may
// still be in flight), lgkmcnt for the fragment reads, which are issued as inline ds_read_b128.
#pragma once
#include "conv_params.hpp"
#include "mma_common.hpp"

namespace sc {

template <int N> __device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

template <int OFF> __device__ __forceinline__ v4i lds_read16_at(unsigned addr) {
  v4i v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}

// wait until at most N LDS reads are outstanding; the fragments pass through the statement so that
// no MFMA that consumes them can be scheduled above the wait
template <int N, int CNT> __device__ __forceinline__ void wait_frags(v4i (&f)[CNT]) {
  if constexpr (CNT == 1) asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(f[0]) : "n"(N));
  if constexpr (CNT == 2) asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(f[0]), "+v"(f[1]) : "n"(N));
  if constexpr (CNT == 3) asm volatile("s_waitcnt lgkmcnt(%3)" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]) : "n"(N));
  if constexpr (CNT == 4)
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]) : "n"(N));
  if constexpr (CNT == 5)
    asm volatile("s_waitcnt lgkmcnt(%5)" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(f[4]) : "n"(N));
  if constexpr (CNT == 7)
    asm volatile("s_waitcnt lgkmcnt(%7)"
                 : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(f[4]), "+v"(f[5]), "+v"(f[6])
                 : "n"(N));
  if constexpr (CNT == 6)
    asm volatile("s_waitcnt lgkmcnt(%6)"
                 : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(f[4]), "+v"(f[5])
                 : "n"(N));
  if constexpr (CNT == 8)
    asm volatile("s_waitcnt lgkmcnt(%8)"
                 : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(f[4]), "+v"(f[5]), "+v"(f[6]), "+v"(f[7])
                 : "n"(N));
  static_assert(CNT >= 1 && CNT <= 8, "fragment count");
}

#ifdef SC_TIMING
#define SC_DMA_STAMP(slot) do { if (p.dbg && threadIdx.x == 0) p.dbg[(size_t)blockIdx.x * 8 + (slot)] = wall_clock64(); } while (0)
#else
#define SC_DMA_STAMP(slot) do { } while (0)
#endif

template <int BM, int BN, int STAGES>
constexpr size_t igemm_dma_lds_bytes() {
  return (size_t)STAGES * (BM + BN) * kRowBytes + (BM + 4) * sizeof(int32_t) + BN * sizeof(float);
}

// SPLITK: grid = output tiles x p.splits; workgroup (tile, split) contracts its share of the K tiles
// and leaves float partial sums in p.partial; the workgroup that arrives last at the tile's counter
// adds the partial sums in split order (so the result does not depend on who was last) and runs
// the epilogue.  Nobody waits for anybody: a workgroup either finishes the tile or leaves.
template <int DT, int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, bool SPLITK = false>
__global__ __launch_bounds__(kThreads) void igemm_dma_kernel(const ConvParams p) {
  using E = Elem<DT>;
  using T = typename E::T;
  constexpr int V = E::V;
  constexpr int EB = sizeof(T);
  constexpr int BK = 8 * V;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int MI = WM / 32, NI = WN / 32;
  constexpr int A_LOADS = BM / 32, B_LOADS = BN / 32;
  constexpr int LPT = A_LOADS + B_LOADS;                    // transfers per K tile and wavefront
  constexpr int STAGE_BYTES = (BM + BN) * kRowBytes;
  static_assert(WAVES_M * WAVES_N * 64 == kThreads, "four wavefronts");
  static_assert(STAGES >= 2 && (STAGES - 2) * LPT <= 63, "vmcnt is a 6-bit counter");

  extern __shared__ __align__(16) unsigned char smem[];
  int32_t* s_rows = reinterpret_cast<int32_t*>(smem + STAGES * STAGE_BYTES);   // [BM], then one flag word
  float* s_bias = reinterpret_cast<float*>(s_rows + BM + 4);                   // [BN]
  SC_DMA_STAMP(0);

  const int splits = SPLITK ? p.splits : 1;
  const int nwg = p.m_tiles * p.n_tiles * splits;
  const int per_xcd = (nwg + 7) >> 3;
  const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (logical >= nwg) return;
  // the splits of one tile are neighbours: they run on one XCD and share the tile's rows in its L2
  const int tile = logical / splits;
  const int split = logical - tile * splits;
  const int tile_m = tile / p.n_tiles;
  const int tile_n = tile - tile_m * p.n_tiles;
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int kt_lo = SPLITK ? (int)((int64_t)split * p.k_tiles / splits) : 0;
  const int kt_hi = SPLITK ? (int)((int64_t)(split + 1) * p.k_tiles / splits) : p.k_tiles;
  const int n_kt = kt_hi - kt_lo;

  const int t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;

  const T* __restrict__ x = static_cast<const T*>(p.x);
  T* __restrict__ y = static_cast<T*>(p.y);
  const T* __restrict__ zeros = static_cast<const T*>(p.zeros);

  // ---- per-thread gather state ---------------------------------------------------------------------
  const int c16 = t & 7;                              // physical 16-byte group this lane fills
  const int lrow = t >> 3;                            // tile row (plus 32 per transfer)
  const int lc = c16 ^ ((lrow >> 1) & 7);             // logical group it fetches (the key ignores +32j)
  int32_t a_base[A_LOADS], a_iy0[A_LOADS], a_ix0[A_LOADS];
  int32_t a_row[A_LOADS];
#pragma unroll
  for (int j = 0; j < A_LOADS; ++j) {                        // all row numbers first: one round trip
    const int icc = min(m0 + lrow + 32 * j, p.rows - 1);     // clamped: the loads stay unconditional
    a_row[j] = p.row_idx ? p.row_idx[icc] : icc;
  }
  // Everything the end of the kernel needs from global memory is requested here, in the same round
  // trip, so that the epilogue and the zero fill start without one of their own: the bias slice and
  // the first and last dense row this workgroup owns (Alg. 2, mask == 0 branch: it writes the zeros
  // of the dense rows from its first kept row up to the next tile's first kept row).
  float bias_v = 0.0f;
  if (t < BN && p.bias && n0 + t < p.c_out) bias_v = p.bias[n0 + t];
  int z_lo = 0, z_hi = p.m_total;
  if (p.zero_fill) {
    if (tile_m != 0) z_lo = p.row_idx[m0];
    if (m0 + BM < p.rows) z_hi = p.row_idx[m0 + BM];
  }
  // a run that contracts every row and lets the mask decide at the store: the mask bytes of this lane's rows,
  // requested here, looked at after the K loop
  unsigned mkeep[A_LOADS];
#pragma unroll
  for (int j = 0; j < A_LOADS; ++j) {
    mkeep[j] = 1;
    if (p.masked_store) {
      const int r = min(m0 + lrow + 32 * j, p.rows - 1);
      mkeep[j] = p.mask[p.mask_spatial ? r - fast_div(r, p.div_howo_mul, p.div_howo_shift) * p.ho_wo : r];
    }
  }
#pragma unroll
  for (int j = 0; j < A_LOADS; ++j) {
    const bool present = m0 + lrow + 32 * j < p.rows;
    const int ic = m0 + lrow + 32 * j;                       // position in the compacted GEMM
    const int rr = present ? (p.y_compact ? ic : a_row[j]) : -1;   // row the epilogue stores to
    s_rows[lrow + 32 * j] = rr;
    const int rc = present ? (p.x_compact ? ic : a_row[j]) : 0;    // row the window is read from
    const int n = fast_div(rc, p.div_howo_mul, p.div_howo_shift), rem = rc - n * p.ho_wo;
    const int oy = fast_div(rem, p.div_wo_mul, p.div_wo_shift), ox = rem - oy * p.wo;
    a_iy0[j] = present ? oy * p.sh - p.ph : -(1 << 30);      // no tap of an absent row is in range
    a_ix0[j] = ox * p.sw - p.pw;
    a_base[j] = (int32_t)(n * p.xs_n + (int64_t)(oy * p.sh - p.ph) * p.xs_h + (int64_t)a_ix0[j] * p.xs_w);
  }
  const T* __restrict__ wp = static_cast<const T*>(p.wp) + (int64_t)(n0 + lrow) * p.k_pad + lc * V;

  int g_ci, g_kx, g_ky;   // window position of this lane's K group, advanced by one K tile per issue
  {
    const int k0 = kt_lo * BK + lc * V;
    const int tap = k0 / p.c_in;
    g_ci = k0 - tap * p.c_in;
    g_ky = tap / p.kw;
    g_kx = tap - g_ky * p.kw;
  }
  // mask bytes of the first zero-fill passes: requested before any K tile (they are older than the
  // transfers, so no wait in the K loop is delayed by them) and first looked at after the K loop
  constexpr int CPR = BN * EB / 16;        // 16-byte groups per output row slice
  constexpr int RPI = kThreads / CPR;      // dense rows per fill pass of the workgroup
  constexpr int ZB = 4;                    // passes whose mask bytes are fetched up front
  const int zc = t % CPR, zr = t / CPR;
  unsigned mk[ZB];
#pragma unroll
  for (int u = 0; u < ZB; ++u) {           // unconditional, clamped: dense runs read a few bytes they ignore
    int r = min(z_lo + zr + u * RPI, p.m_total - 1);
    if (p.mask_spatial) r -= fast_div(r, p.div_howo_mul, p.div_howo_shift) * p.ho_wo;
    mk[u] = p.mask[r];
  }
  __syncthreads();   // s_rows written (read again in the epilogue); nothing is in flight yet

  // byte offset of the zero page relative to x: one address select per transfer, no branch
  const int64_t zoff = reinterpret_cast<const unsigned char*>(zeros) - reinterpret_cast<const unsigned char*>(x);
  auto dma16 = [](const void* src, unsigned char* lds_base) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                     (__attribute__((address_space(3))) void*)lds_base, 16, 0, 0);
  };
  auto issue_tile = [&](int kt, int stage) {
    unsigned char* sa = smem + stage * STAGE_BYTES + wave * 8 * kRowBytes;      // this wavefront's 8 rows
    unsigned char* sb = sa + BM * kRowBytes;
    const int dy = g_ky * p.dil_h, dx = g_kx * p.dil_w;
    const int off = dy * p.xs_h + dx * p.xs_w + g_ci;
    const bool tap_ok = g_ky < p.kh;
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j) {
      const bool ok = tap_ok && (unsigned)(a_iy0[j] + dy) < (unsigned)p.h && (unsigned)(a_ix0[j] + dx) < (unsigned)p.w;
      const int64_t boff = ok ? (int64_t)(a_base[j] + off) * EB : zoff;
      dma16(reinterpret_cast<const unsigned char*>(x) + boff, sa + j * 32 * kRowBytes);
    }
#pragma unroll
    for (int j = 0; j < B_LOADS; ++j) dma16(wp + (int64_t)(32 * j) * p.k_pad + kt * BK, sb + j * 32 * kRowBytes);
    g_ci += BK;
    while (g_ci >= p.c_in) {
      g_ci -= p.c_in;
      if (++g_kx == p.kw) { g_kx = 0; ++g_ky; }
    }
  };

  floatx16 acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

  const int fp = lane & 31, fh = lane >> 5;
  const unsigned lds0 = (unsigned)(unsigned long long)(__attribute__((address_space(3))) unsigned char*)smem;
  unsigned frag_a[4], frag_b[4];   // LDS address of this lane's fragment of K step ks in stage 0
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const unsigned o = (unsigned)(fp * kRowBytes + (((2 * ks + fh) ^ ((fp >> 1) & 7)) << 4));
    frag_a[ks] = lds0 + wm0 * kRowBytes + o;
    frag_b[ks] = lds0 + (BM + wn0) * kRowBytes + o;
  }

  auto read_step = [&](unsigned stage_off, int ks, v4i (&f)[MI + NI]) {
    const unsigned aa = frag_a[ks] + stage_off, ab = frag_b[ks] + stage_off;
    if constexpr (MI >= 1) f[0] = lds_read16_at<0>(aa);
    if constexpr (MI >= 2) f[1] = lds_read16_at<32 * kRowBytes>(aa);
    if constexpr (MI >= 3) f[2] = lds_read16_at<64 * kRowBytes>(aa);
    if constexpr (MI >= 4) f[3] = lds_read16_at<96 * kRowBytes>(aa);
    if constexpr (NI >= 1) f[MI + 0] = lds_read16_at<0>(ab);
    if constexpr (NI >= 2) f[MI + 1] = lds_read16_at<32 * kRowBytes>(ab);
    if constexpr (NI >= 3) f[MI + 2] = lds_read16_at<64 * kRowBytes>(ab);
    if constexpr (NI >= 4) f[MI + 3] = lds_read16_at<96 * kRowBytes>(ab);
  };
  auto mma_step = [&](const v4i (&f)[MI + NI]) {
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) E::mma(acc[mi][ni], f[MI + ni], f[mi]);
  };

  // ---- main loop ---------------------------------------------------------------------------------------
#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s)
    if (s < n_kt) issue_tile(kt_lo + s, s);

  SC_DMA_STAMP(1);
  int stage = 0;   // kt % STAGES
  for (int kt = 0; kt < n_kt; ++kt) {
    if (kt == 1) SC_DMA_STAMP(2);
    // tile kt has landed once at most the transfers of the STAGES-2 later tiles are in flight
    if (kt + STAGES - 2 < n_kt) wait_vmcnt<(STAGES - 2) * LPT>();
    else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();   // ... for every wavefront; and all have left tile kt-1
    asm volatile("" ::: "memory");
    if (kt + STAGES - 1 < n_kt) {
      int fill = stage + STAGES - 1;
      if (fill >= STAGES) fill -= STAGES;
      issue_tile(kt_lo + kt + STAGES - 1, fill);   // into the stage tile kt-1 occupied
    }
    // four K steps per tile, each with its own fragment registers (no register is rewritten while
    // an MFMA that reads it may still be starting); the reads of step ks+1 are in flight during the
    // MFMAs of step ks
    const unsigned stage_off = (unsigned)(stage * STAGE_BYTES);
    v4i f0[MI + NI], f1[MI + NI], f2[MI + NI], f3[MI + NI];
    read_step(stage_off, 0, f0);
    read_step(stage_off, 1, f1);
    wait_frags<MI + NI>(f0);
    mma_step(f0);
    read_step(stage_off, 2, f2);
    wait_frags<MI + NI>(f1);
    mma_step(f1);
    read_step(stage_off, 3, f3);
    wait_frags<MI + NI>(f2);
    mma_step(f2);
    wait_frags<0>(f3);
    mma_step(f3);
    if (++stage == STAGES) stage = 0;
  }

  SC_DMA_STAMP(3);
  // ---- split K: leave the partial sums; the last workgroup of the tile adds them up ----------------------
  if constexpr (SPLITK) {
    if (splits > 1) {
      // Partial sums travel through device-scope relaxed atomic stores and loads of 8 bytes: those
      // write through to, and read from, the point where the XCDs' L2 caches agree, so no cache-wide
      // write-back / invalidate fence is needed (a device-scope fence flushes a whole L2: tens of
      // microseconds per launch here).  Order: stores acknowledged (vmcnt 0) -> workgroup barrier ->
      // arrival counter; the last arrival reads after it has seen every other arrival.
      constexpr int PER_WAVE = MI * NI * 8;     // 8-byte chunks per lane
      typedef unsigned long long u64;
      u64* part = reinterpret_cast<u64*>(p.partial) + ((int64_t)tile * splits * (kThreads / 64)) * PER_WAVE * 64;
      u64* mine = part + ((int64_t)split * (kThreads / 64) + wave) * PER_WAVE * 64 + lane;
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
          for (int q = 0; q < 8; ++q) {
            const u64 v = (u64)__float_as_uint(acc[mi][ni][2 * q]) | ((u64)__float_as_uint(acc[mi][ni][2 * q + 1]) << 32);
            __hip_atomic_store(mine + ((mi * NI + ni) * 8 + q) * 64, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      SC_DMA_STAMP(4);
      __syncthreads();
      int32_t* s_flag = s_rows + BM;             // one word behind the row list
      if (t == 0) {
        const int old = __hip_atomic_fetch_add(p.counters + tile, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // everybody has arrived: leave the counter at zero for the next launch
        if (old == splits - 1) __hip_atomic_store(p.counters + tile, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *s_flag = old;
      }
      __syncthreads();
      if (*s_flag != splits - 1) return;          // not the last one: done; the last one also writes the tile's zeros
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
          for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;
      for (int sp = 0; sp < splits; ++sp) {      // fixed order: the sum does not depend on who came last
        const u64* src = part + ((int64_t)sp * (kThreads / 64) + wave) * PER_WAVE * 64 + lane;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
          for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int q = 0; q < 8; ++q) {
              const u64 v = __hip_atomic_load(src + ((mi * NI + ni) * 8 + q) * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              acc[mi][ni][2 * q] += __uint_as_float((unsigned)v);
              acc[mi][ni][2 * q + 1] += __uint_as_float((unsigned)(v >> 32));
            }
      }
    }
  }

  SC_DMA_STAMP(5);
  if (p.masked_store) {
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j)
      if (c16 == 0 && mkeep[j] == 0 && m0 + lrow + 32 * j < p.rows) s_rows[lrow + 32 * j] = dropped_row_code(m0 + lrow + 32 * j);
  }
  // ---- zero fill of the dropped rows this workgroup owns (Alg. 2, mask == 0 branch) --------------------
  if (t < BN) s_bias[t] = bias_v;
  // LDS-only barrier (the bias slice): no global-memory wait, the zero stores below just drain
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
  if (p.zero_fill) {
    const int valid = (min(BN, p.c_out - n0) * EB) >> 4;
    if (zc < valid) {
      unsigned char* ybase = reinterpret_cast<unsigned char*>(y) + (int64_t)n0 * EB + zc * 16;
      const int64_t res_at = (int64_t)n0 * EB + zc * 16;     // the same group of the shortcut tensor
      const v4i z = {0, 0, 0, 0};
#pragma unroll
      for (int u = 0; u < ZB; ++u) {
        const int r = z_lo + zr + u * RPI;
        if (r < z_hi && mk[u] == 0) {
          const int64_t at = (int64_t)r * p.c_out * EB;
          sc_store16(reinterpret_cast<v4i*>(ybase + at), p.residual ? dropped_row_group<DT>(p.residual, res_at + at, p.residual_relu) : z);
        }
      }
      for (int r0 = z_lo + zr + ZB * RPI; r0 < z_hi; r0 += 4 * RPI) {   // tiles that own more rows
        unsigned char m4[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          int r = min(r0 + u * RPI, z_hi - 1);
          if (p.mask_spatial) r -= fast_div(r, p.div_howo_mul, p.div_howo_shift) * p.ho_wo;
          m4[u] = p.mask[r];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int r = r0 + u * RPI;
          if (r < z_hi && m4[u] == 0) {
            const int64_t at = (int64_t)r * p.c_out * EB;
            sc_store16(reinterpret_cast<v4i*>(ybase + at), p.residual ? dropped_row_group<DT>(p.residual, res_at + at, p.residual_relu) : z);
          }
        }
      }
    }
  }

  // ---- epilogue ----------------------------------------------------------------------------------------
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    const int rr = s_rows[wm0 + mi * 32 + fp];
    if (rr == -1 || (rr < -1 && p.masked_store != 1)) continue;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
      const int c0 = n0 + wn0 + ni * 32 + 16 * fh;
      if (c0 >= p.c_out) continue;
      if (rr < 0) { store_zero_block<DT>(-2 - rr, c0, y, 1, p.c_out, p.ho_wo, 0, 0, 0); continue; }
      store_kept_block_res<DT>(acc[mi][ni], rr, c0, y, p.bias ? s_bias + (c0 - n0) : nullptr, 0, p.relu, 1, p.c_out,
                               p.ho_wo, 0, 0, 0, static_cast<const T*>(p.residual), p.residual_relu);
    }
  }
  SC_DMA_STAMP(6);
}

template <int DT, int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, bool SPLITK = false>
hipError_t igemm_dma_launch(const ConvParams& p, hipStream_t stream) {
  constexpr size_t lds = igemm_dma_lds_bytes<BM, BN, STAGES>();
  auto kern = igemm_dma_kernel<DT, BM, BN, WAVES_M, WAVES_N, STAGES, SPLITK>;
  static std::atomic<bool> attr_set{false};
  if (lds > 64 * 1024 && !attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int nwg = p.m_tiles * p.n_tiles * (SPLITK ? p.splits : 1);
  const int grid = ((nwg + 7) / 8) * 8;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), lds, stream, p);
  return hipGetLastError();
}

// bytes of float partial sums one output tile and one split need
template <int BM, int BN>
constexpr size_t igemm_partial_bytes() { return (size_t)BM * BN * sizeof(float); }

}  // namespace sc
