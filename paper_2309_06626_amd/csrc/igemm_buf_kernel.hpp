// Tiled masked-convolution kernel, direct-to-LDS gathers through buffer loads, for layers whose input
// channel count is a multiple of the K tile (64 channels of a 16-bit type: every deep layer of the
// benchmark networks).
//
// Decomposition, LDS layout, zero-fill ownership and epilogue are those of igemm_dma_kernel (paper
// Sec. 3.2 stages i-iii fused; workgroup = BM kept rows x BN channels).  What differs is the cost of
// one K tile in instructions, which is what bounds that kernel once the matrix work is small:
//
//  * a K tile lies inside one window tap, the same for every lane, so the tap walk is scalar
//    arithmetic (no per-lane tap state, no multiplies, no divergent loop);
//  * transfers are `buffer_load_dwordx4 ... lds`: the buffer descriptor carries the base, the K-tile
//    part of the address is a scalar offset, a lane contributes one 32-bit offset per kept row; an
//    offset past the end of the buffer makes the hardware write zeros into LDS, which is how padded
//    taps and absent rows are served (one select per row, no page of zeros, no 64-bit address math);
//    filter rows need no per-lane work at all;
//  * the ring position is a compile-time constant (the loop is unrolled over the ring), so LDS read
//    addresses are immediates on top of eight registers set up once.
#pragma once
#include <type_traits>

#include "igemm_dma_kernel.hpp"

namespace sc {

constexpr unsigned kBufferWord3 = 0x00020000u;   // raw buffer, 32-bit data format (gfx9 family)
constexpr unsigned kOutOfRange = 0x80000000u;    // byte offset no buffer of this library reaches

template <int OFF> __device__ __forceinline__ v4i lds_read16_big(unsigned addr) {
  if constexpr (OFF < 65536) return lds_read16_at<OFF>(addr);
  else return lds_read16_at<0>(addr + (unsigned)OFF);
}

// 16-byte accesses at device scope (the partial sums of a split K walk): they write through to, and read from,
// the point where the L2 caches of the chip's dies agree, like the relaxed device-scope atomics of the other
// split kernels, but four floats at a time.  The caller orders them with s_waitcnt vmcnt(0).
__device__ __forceinline__ void store16_device_scope(void* dst, v4i v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(dst), "v"(v) : "memory");
}
__device__ __forceinline__ v4i load16_device_scope(const void* src) {
  v4i v;
  asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v) : "v"(src) : "memory");
  return v;
}

// SPLITK: grid = output tiles x p.splits; the workgroups of one tile are neighbours (one die, so the tile's rows
// are shared in its L2), each contracts its share of the K tiles and leaves float partial sums; the one that
// arrives last at the tile's counter adds them in split order (the result does not depend on who was last) and
// runs the epilogue.  Nobody waits for anybody.
template <int DT, int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, bool SPLITK = false>
__global__ __launch_bounds__(WAVES_M * WAVES_N * 64) void igemm_buf_kernel(const ConvParams p) {
  using E = Elem<DT>;
  using T = typename E::T;
  constexpr int V = E::V;
  constexpr int EB = sizeof(T);
  constexpr int BK = 8 * V;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int MI = WM / 32, NI = WN / 32;
  constexpr int NT = WAVES_M * WAVES_N * 64;   // threads: four wavefronts, or eight (two per SIMD) for the largest tile
  constexpr int RPR = NT / 8;                  // tile rows one transfer of the whole workgroup covers
  constexpr int A_LOADS = BM / RPR, B_LOADS = BN / RPR;
  constexpr int LPT = A_LOADS + B_LOADS;
  constexpr int STAGE_BYTES = (BM + BN) * kRowBytes;
  static_assert(NT == 256 || NT == 512, "four or eight wavefronts");
  static_assert(BM % RPR == 0 && BN % RPR == 0, "whole transfers");
  static_assert(STAGES >= 2 && (STAGES - 2) * LPT <= 63, "vmcnt is a 6-bit counter");
  static_assert(EB == 2, "16-bit operands");

  extern __shared__ __align__(16) unsigned char smem[];
  int32_t* s_rows = reinterpret_cast<int32_t*>(smem + STAGES * STAGE_BYTES);   // [BM], then one spare group
  float* s_bias = reinterpret_cast<float*>(s_rows + BM + 4);                   // [BN]

  const int splits = SPLITK ? p.splits : 1;
  const int nwg = p.m_tiles * p.n_tiles * splits;
  const int per_xcd = (nwg + 7) >> 3;
  const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (logical >= nwg) return;
  const int tile = logical / splits;
  const int split = logical - tile * splits;
  const int tile_m = tile / p.n_tiles;
  const int tile_n = tile - tile_m * p.n_tiles;
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int kt_lo = SPLITK ? (int)((int64_t)split * p.k_tiles / splits) : 0;
  const int kt_hi = SPLITK ? (int)((int64_t)(split + 1) * p.k_tiles / splits) : p.k_tiles;
  const int n_kt = kt_hi - kt_lo;

  const int t = threadIdx.x;
  const int lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
  const int fp = lane & 31, fh = lane >> 5;
  T* __restrict__ y = static_cast<T*>(p.y);

  // ---- one round trip: row numbers, bias slice, the dense row range this workgroup owns -------------
  const int c16 = lane & 7;                           // physical 16-byte group this lane fills
  const int lrow = wave * 8 + (lane >> 3);            // tile row (plus 32 per transfer)
  const int lc = c16 ^ ((lrow >> 1) & 7);             // logical group it fetches
  int32_t a_row[A_LOADS];
#pragma unroll
  for (int j = 0; j < A_LOADS; ++j) {
    const int icc = min(m0 + lrow + RPR * j, p.rows - 1);
    a_row[j] = p.row_idx ? p.row_idx[icc] : icc;
  }
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
      const int r = min(m0 + lrow + RPR * j, p.rows - 1);
      mkeep[j] = p.mask[p.mask_spatial ? r - fast_div(r, p.div_howo_mul, p.div_howo_shift) * p.ho_wo : r];
    }
  }

  // per kept row: byte offset of (n, iy0, ix0, this lane's channel group) -- possibly negative, valid
  // once a tap's offset is added -- and which taps fall inside the image: bit ky for the rows, bit
  // 8 + kx for the columns (kh, kw <= 8)
  int32_t a_voff[A_LOADS];
  uint32_t a_taps[A_LOADS];
#pragma unroll
  for (int j = 0; j < A_LOADS; ++j) {
    const bool present = m0 + lrow + RPR * j < p.rows;
    const int ic = m0 + lrow + RPR * j;                      // position in the compacted GEMM
    const int rr = present ? (p.y_compact ? ic : a_row[j]) : -1;   // row the epilogue stores to
    if (c16 == 0) s_rows[lrow + RPR * j] = rr;
    const int rc = present ? (p.x_compact ? ic : a_row[j]) : 0;    // row the window is read from
    const int n = fast_div(rc, p.div_howo_mul, p.div_howo_shift), rem = rc - n * p.ho_wo;
    const int oy = fast_div(rem, p.div_wo_mul, p.div_wo_shift), ox = rem - oy * p.wo;
    const int iy0 = oy * p.sh - p.ph, ix0 = ox * p.sw - p.pw;
    a_voff[j] = (int32_t)((n * p.xs_n + (int64_t)iy0 * p.xs_h + (int64_t)ix0 * p.xs_w + lc * V) * EB);
    uint32_t bits = 0;
    for (int ky = 0; ky < p.kh; ++ky) bits |= ((unsigned)(iy0 + ky * p.dil_h) < (unsigned)p.h ? 1u : 0u) << ky;
    for (int kx = 0; kx < p.kw; ++kx) bits |= ((unsigned)(ix0 + kx * p.dil_w) < (unsigned)p.w ? 1u : 0u) << (8 + kx);
    a_taps[j] = present ? bits : 0u;
  }
  const uint32_t b_voff = (uint32_t)((lrow * p.k_pad + lc * V) * EB);

  constexpr int CPR = BN * EB / 16;        // 16-byte groups per output row slice
  constexpr int RPI = NT / CPR;           // dense rows per fill pass of the workgroup
  constexpr int ZB = 4;                    // passes whose mask bytes are fetched up front
  const int zc = t % CPR, zr = t / CPR;
  unsigned mk[ZB];
#pragma unroll
  for (int u = 0; u < ZB; ++u) {
    int r = min(z_lo + zr + u * RPI, p.m_total - 1);
    if (p.mask_spatial) r -= fast_div(r, p.div_howo_mul, p.div_howo_shift) * p.ho_wo;
    mk[u] = p.mask[r];
  }
  __syncthreads();   // s_rows written; nothing is in flight yet

  const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.x), 0, (int)p.x_bytes, kBufferWord3);
  const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.wp), 0, (int)p.w_bytes, kBufferWord3);
  typedef __attribute__((address_space(3))) void lds_void;

  // scalar walk over the window, entered at K tile kt_lo: K tile kt lies in tap (s_ky, s_kx) at channel s_ci
  const int step_x = p.dil_w * p.xs_w * EB, step_y = p.dil_h * p.xs_h * EB;
  const int k_first = kt_lo * BK;
  const int tap_first = k_first / p.c_in;
  int s_ci = k_first - tap_first * p.c_in;
  int s_ky = tap_first / p.kw;
  int s_kx = tap_first - s_ky * p.kw;
  int s_off = s_ci * EB + s_kx * step_x + s_ky * step_y;     // byte offset of that tap and channel
  uint32_t s_bits = (1u << s_ky) | (1u << (8 + s_kx));        // its two validity bits
  int s_boff = (n0 * p.k_pad + k_first) * EB;                 // byte offset of filter row n0 at the current K tile
  // transfer `idx` of a K tile (the A rows first, then the filter rows); the last one steps the walk
  auto issue_one = [&](auto stage_c, auto idx_c) {
    constexpr int ST = decltype(stage_c)::value;
    constexpr int IDX = decltype(idx_c)::value;
    unsigned char* sa = smem + ST * STAGE_BYTES + wave * 8 * kRowBytes;      // this wavefront's 8 rows
    unsigned char* sb = sa + BM * kRowBytes;
    if constexpr (IDX < A_LOADS) {
      constexpr int j = IDX;
      const bool ok = (a_taps[j] & s_bits) == s_bits;
      const uint32_t voff = ok ? (uint32_t)(a_voff[j] + s_off) : kOutOfRange;   // out of range: LDS gets zeros
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (lds_void*)(sa + j * RPR * kRowBytes), 16, voff, 0, 0, 0);
    } else {
      constexpr int j = IDX - A_LOADS;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (lds_void*)(sb + j * RPR * kRowBytes), 16, b_voff,
                                               s_boff + j * RPR * p.k_pad * EB, 0, 0);
    }
    if constexpr (IDX == LPT - 1) {
      s_boff += BK * EB;
      s_ci += BK;
      s_off += BK * EB;
      if (s_ci == p.c_in) {                     // next tap (uniform: Cin is a multiple of the K tile)
        s_ci = 0;
        s_off += step_x - p.c_in * EB;
        if (++s_kx == p.kw) {
          s_kx = 0;
          ++s_ky;
          s_off += step_y - p.kw * step_x;
        }
        s_bits = (1u << s_ky) | (1u << (8 + s_kx));
      }
    }
  };
  auto issue_from = [&](auto stage_c, auto first_c) {      // transfers first .. LPT-1, back to back
    constexpr int FIRST = decltype(first_c)::value;
    if constexpr (FIRST < LPT) {
      issue_one(stage_c, first_c);
      if constexpr (FIRST + 1 < LPT) issue_one(stage_c, std::integral_constant<int, FIRST + 1>{});
      if constexpr (FIRST + 2 < LPT) issue_one(stage_c, std::integral_constant<int, FIRST + 2>{});
      if constexpr (FIRST + 3 < LPT) issue_one(stage_c, std::integral_constant<int, FIRST + 3>{});
      if constexpr (FIRST + 4 < LPT) issue_one(stage_c, std::integral_constant<int, FIRST + 4>{});
      if constexpr (FIRST + 5 < LPT) issue_one(stage_c, std::integral_constant<int, FIRST + 5>{});
      if constexpr (FIRST + 6 < LPT) issue_one(stage_c, std::integral_constant<int, FIRST + 6>{});
      if constexpr (FIRST + 7 < LPT) issue_one(stage_c, std::integral_constant<int, FIRST + 7>{});
      static_assert(LPT - FIRST <= 8, "at most eight transfers per wavefront and K tile");
    }
  };
  auto issue_tile = [&](auto stage_c) { issue_from(stage_c, std::integral_constant<int, 0>{}); };

  floatx16 acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

  const unsigned lds0 = (unsigned)(unsigned long long)(__attribute__((address_space(3))) unsigned char*)smem;
  unsigned frag_a[4], frag_b[4];   // LDS address of this lane's fragment of K step ks in ring slot 0
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const unsigned o = (unsigned)(fp * kRowBytes + (((2 * ks + fh) ^ ((fp >> 1) & 7)) << 4));
    frag_a[ks] = lds0 + wm0 * kRowBytes + o;
    frag_b[ks] = lds0 + (BM + wn0) * kRowBytes + o;
  }
  auto read_step = [&](auto stage_c, int ks, v4i (&f)[MI + NI]) {
    constexpr int SO = decltype(stage_c)::value * STAGE_BYTES;
    const unsigned aa = frag_a[ks], ab = frag_b[ks];
    if constexpr (MI >= 1) f[0] = lds_read16_big<SO>(aa);
    if constexpr (MI >= 2) f[1] = lds_read16_big<SO + 32 * kRowBytes>(aa);
    if constexpr (MI >= 3) f[2] = lds_read16_big<SO + 64 * kRowBytes>(aa);
    if constexpr (MI >= 4) f[3] = lds_read16_big<SO + 96 * kRowBytes>(aa);
    if constexpr (NI >= 1) f[MI + 0] = lds_read16_big<SO>(ab);
    if constexpr (NI >= 2) f[MI + 1] = lds_read16_big<SO + 32 * kRowBytes>(ab);
    if constexpr (NI >= 3) f[MI + 2] = lds_read16_big<SO + 64 * kRowBytes>(ab);
    if constexpr (NI >= 4) f[MI + 3] = lds_read16_big<SO + 96 * kRowBytes>(ab);
  };
  auto mma_step = [&](const v4i (&f)[MI + NI]) {
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) E::mma(acc[mi][ni], f[MI + ni], f[mi]);
  };
  // The same with one transfer of the next ring slot issued behind every MFMA.  A wavefront that issues its
  // transfers back to back sits in the issue stage until the address unit (shared by the CU) has taken them
  // all, and only then starts its matrix work: measured, a lone workgroup's K tile costs transfer time PLUS
  // matrix time.  Behind an MFMA the issue slot is free while the matrix pipeline works.
  auto mma_step_issuing = [&](const v4i (&f)[MI + NI], auto stage_c, auto ks_c, bool more) {
    constexpr int KS = decltype(ks_c)::value;
    auto one = [&](auto mi_c, auto ni_c) {
      constexpr int mi = decltype(mi_c)::value, ni = decltype(ni_c)::value;
      if constexpr (mi < MI && ni < NI) {
        E::mma(acc[mi][ni], f[MI + ni], f[mi]);
        constexpr int IDX = KS * MI * NI + mi * NI + ni;
        if constexpr (IDX < LPT) {
          __builtin_amdgcn_sched_barrier(0);
          if (more) issue_one(stage_c, std::integral_constant<int, IDX>{});
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    };
    using I0 = std::integral_constant<int, 0>; using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>; using I3 = std::integral_constant<int, 3>;
    one(I0{}, I0{}); one(I0{}, I1{}); one(I0{}, I2{}); one(I0{}, I3{});
    one(I1{}, I0{}); one(I1{}, I1{}); one(I1{}, I2{}); one(I1{}, I3{});
    one(I2{}, I0{}); one(I2{}, I1{}); one(I2{}, I2{}); one(I2{}, I3{});
    one(I3{}, I0{}); one(I3{}, I1{}); one(I3{}, I2{}); one(I3{}, I3{});
  };

  // one K tile: wait until it has landed, contract it, refilling the slot the previous tile occupied on the way
  // (interleaved where a wavefront has at least two MFMAs per K step: measured 5-13 % faster on the 64 x 128,
  // 128 x 64 and 128 x 128 tiles, 3-5 % slower on the tiles with one MFMA per step, which keep the plain order)
  constexpr bool INTERLEAVE = MI * NI >= 2;
  int issued = 0;
  auto k_tile = [&](auto stage_c, int kt) {
    constexpr int ST = decltype(stage_c)::value;
    using Refill = std::integral_constant<int, (ST + STAGES - 1) % STAGES>;
    if (kt + STAGES - 2 < n_kt) wait_vmcnt<(STAGES - 2) * LPT>();
    else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();   // landed for every wavefront; and all have left tile kt-1
    asm volatile("" ::: "memory");
    const bool more = issued < n_kt;
    if constexpr (!INTERLEAVE) {
      if (more) issue_tile(Refill{});
    }
    v4i f0[MI + NI], f1[MI + NI], f2[MI + NI], f3[MI + NI];
    read_step(stage_c, 0, f0);
    read_step(stage_c, 1, f1);
    wait_frags<MI + NI>(f0);
    if constexpr (INTERLEAVE) mma_step_issuing(f0, Refill{}, std::integral_constant<int, 0>{}, more); else mma_step(f0);
    read_step(stage_c, 2, f2);
    wait_frags<MI + NI>(f1);
    if constexpr (INTERLEAVE) mma_step_issuing(f1, Refill{}, std::integral_constant<int, 1>{}, more); else mma_step(f1);
    read_step(stage_c, 3, f3);
    wait_frags<MI + NI>(f2);
    if constexpr (INTERLEAVE) mma_step_issuing(f2, Refill{}, std::integral_constant<int, 2>{}, more); else mma_step(f2);
    wait_frags<0>(f3);
    if constexpr (INTERLEAVE) mma_step_issuing(f3, Refill{}, std::integral_constant<int, 3>{}, more); else mma_step(f3);
    if constexpr (INTERLEAVE) {
      if (more) issue_from(Refill{}, std::integral_constant<int, (4 * MI * NI < LPT ? 4 * MI * NI : LPT)>{});   // more transfers than MFMAs
    }
    if (more) ++issued;
  };

  // ---- main loop, unrolled over the ring --------------------------------------------------------------
  if (0 < n_kt) { issue_tile(std::integral_constant<int, 0>{}); ++issued; }
  if constexpr (STAGES >= 3) if (1 < n_kt) { issue_tile(std::integral_constant<int, 1>{}); ++issued; }
  if constexpr (STAGES >= 4) if (2 < n_kt) { issue_tile(std::integral_constant<int, 2>{}); ++issued; }
  static_assert(STAGES <= 4, "ring of at most four tiles");
  for (int kt = 0; kt < n_kt; kt += STAGES) {
    k_tile(std::integral_constant<int, 0>{}, kt);
    if (kt + 1 < n_kt) k_tile(std::integral_constant<int, 1 % STAGES>{}, kt + 1);
    if constexpr (STAGES >= 3) if (kt + 2 < n_kt) k_tile(std::integral_constant<int, 2 % STAGES>{}, kt + 2);
    if constexpr (STAGES >= 4) if (kt + 3 < n_kt) k_tile(std::integral_constant<int, 3 % STAGES>{}, kt + 3);
  }

  // ---- split K: leave the partial sums; the last workgroup of the tile adds them up ----------------------
  if constexpr (SPLITK) {
    if (splits > 1) {
      // Order: stores acknowledged (vmcnt 0) -> workgroup barrier -> arrival counter (device scope); the last
      // arrival reads after it has seen every other arrival.  No cache-wide fence anywhere.
      constexpr int CHUNKS = MI * NI * 4;                    // 16-byte chunks per lane
      constexpr int64_t SLOT = (int64_t)(NT / 64) * CHUNKS * 64;   // chunks per (tile, split)
      v4i* part = reinterpret_cast<v4i*>(p.partial) + (int64_t)tile * splits * SLOT;
      v4i* mine = part + (int64_t)split * SLOT + (int64_t)wave * CHUNKS * 64 + lane;
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            v4f v = {acc[mi][ni][4 * q], acc[mi][ni][4 * q + 1], acc[mi][ni][4 * q + 2], acc[mi][ni][4 * q + 3]};
            store16_device_scope(mine + ((mi * NI + ni) * 4 + q) * 64, __builtin_bit_cast(v4i, v));
          }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
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
      // fixed order: the sum does not depend on who came last.  The partial sums of split sp + 1 are requested
      // before those of split sp are added (each request is a round trip to the memory side of the L2s).
      constexpr int CH = MI * NI * 4;
      v4i got[2][CH];
      auto request = [&](int sp, v4i (&dst)[CH]) {
        const v4i* src = part + (int64_t)sp * SLOT + (int64_t)wave * CHUNKS * 64 + lane;
#pragma unroll
        for (int c = 0; c < CH; ++c) dst[c] = load16_device_scope(src + c * 64);
      };
      auto add = [&](v4i (&src)[CH]) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
          for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              asm volatile("" : "+v"(src[(mi * NI + ni) * 4 + q]));     // not before the wait that precedes
              const v4f v = __builtin_bit_cast(v4f, src[(mi * NI + ni) * 4 + q]);
#pragma unroll
              for (int e = 0; e < 4; ++e) acc[mi][ni][4 * q + e] += v[e];
            }
      };
      request(0, got[0]);
      for (int sp = 0; sp < splits; sp += 2) {
        if (sp + 1 < splits) { request(sp + 1, got[1]); wait_vmcnt<CH>(); } else wait_vmcnt<0>();
        add(got[0]);
        if (sp + 1 < splits) {
          if (sp + 2 < splits) { request(sp + 2, got[0]); wait_vmcnt<CH>(); } else wait_vmcnt<0>();
          add(got[1]);
        }
      }
    }
  }

  if (p.masked_store) {
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j)
      if (c16 == 0 && mkeep[j] == 0 && m0 + lrow + RPR * j < p.rows) s_rows[lrow + RPR * j] = dropped_row_code(m0 + lrow + RPR * j);
  }
  // ---- zero fill of the dropped rows this workgroup owns (Alg. 2, mask == 0 branch) --------------------
  if (t < BN) s_bias[t] = bias_v;
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // LDS only: the bias slice and the row codes
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
}

template <int DT, int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, bool SPLITK = false>
hipError_t igemm_buf_launch(const ConvParams& p, hipStream_t stream) {
  constexpr size_t lds = igemm_dma_lds_bytes<BM, BN, STAGES>();
  auto kern = igemm_buf_kernel<DT, BM, BN, WAVES_M, WAVES_N, STAGES, SPLITK>;
  static std::atomic<bool> attr_set{false};
  if (lds > 64 * 1024 && !attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int nwg = p.m_tiles * p.n_tiles * (SPLITK ? p.splits : 1);
  const int grid = ((nwg + 7) / 8) * 8;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(WAVES_M * WAVES_N * 64), lds, stream, p);
  return hipGetLastError();
}

// the buffer-load form of tile bm x bn for a 16-bit dtype (shallow: ring of two K tiles), or null
LaunchFn buf_kernel(int dtype, int bm, int bn, bool shallow);
// its split-K form, or null
LaunchFn buf_splitk_kernel(int dtype, int bm, int bn);

}  // namespace sc
