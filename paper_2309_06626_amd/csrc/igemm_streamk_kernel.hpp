// Tiled masked-convolution kernel with the K steps of all output tiles dealt evenly to a fixed number
// of persistent workgroups ("stream-K" scheduling of the compacted GEMM of paper Sec. 3.2).
//
// Why: the deep layers of the benchmark networks have few kept rows and a long K.  Their output tiles
// number a little more than the CUs (280 tiles of 64 x 128 on 256 CUs for a 4 480-row layer), so with
// one workgroup per tile some CUs carry two tiles and the others one, and the kernel lasts as long as
// the CUs with two -- while a CU with a single workgroup cannot even keep enough operand bytes in
// flight to use its share of the L2 bandwidth.  Here the (tile, K tile) steps, tile-major, are cut
// into gridDim.x equal contiguous ranges, two workgroups per CU; a workgroup walks its range tile by
// tile.  A tile whose K walk is shared leaves float partial sums (device-scope relaxed atomic stores,
// as in the split-K kernel) and counts arrivals; the workgroup that arrives last adds the partial sums
// in the order of the K ranges, so the result does not depend on who was last, and runs the epilogue
// (bias, ReLU, scatter, zero fill of the dropped rows the tile owns: Alg. 2's post-processing).  No
// workgroup ever waits for another one.
//
// The K loop, LDS layout and epilogue are those of igemm_buf_kernel.
#pragma once
#include "igemm_buf_kernel.hpp"

namespace sc {

// float partial sums of one (workgroup, unit): a workgroup leaves at most two (the tail of the tile its
// range starts in, the head of the tile it ends in)
template <int BM, int BN>
constexpr size_t streamk_slot_bytes() { return (size_t)BM * BN * sizeof(float); }

template <int DT, int BM, int BN, int WAVES_M, int WAVES_N, int STAGES>
__global__ __launch_bounds__(kThreads) void igemm_streamk_kernel(const ConvParams p) {
  using E = Elem<DT>;
  using T = typename E::T;
  constexpr int V = E::V;
  constexpr int EB = sizeof(T);
  constexpr int BK = 8 * V;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int MI = WM / 32, NI = WN / 32;
  constexpr int A_LOADS = BM / 32, B_LOADS = BN / 32;
  constexpr int LPT = A_LOADS + B_LOADS;
  constexpr int STAGE_BYTES = (BM + BN) * kRowBytes;
  static_assert(WAVES_M * WAVES_N * 64 == kThreads, "four wavefronts");
  static_assert(STAGES >= 2 && (STAGES - 2) * LPT <= 63, "vmcnt is a 6-bit counter");
  static_assert(EB == 2, "16-bit operands");

  extern __shared__ __align__(16) unsigned char smem[];
  int32_t* s_rows = reinterpret_cast<int32_t*>(smem + STAGES * STAGE_BYTES);   // [BM], then one spare group
  float* s_bias = reinterpret_cast<float*>(s_rows + BM + 4);                   // [BN]
  int32_t* s_flag = s_rows + BM;

  // consecutive ranges (the K ranges of one tile, tiles that share rows) run on one XCD
  const unsigned G = gridDim.x;                       // a multiple of 8
  const unsigned me = (blockIdx.x & 7) * (G >> 3) + (blockIdx.x >> 3);
  const unsigned n_kt = (unsigned)p.k_tiles;
  const unsigned total = (unsigned)(p.m_tiles * p.n_tiles) * n_kt;   // the host keeps (G + 1) * total below 2^31
  unsigned s_at = __builtin_amdgcn_readfirstlane(me * total / G);
  const unsigned s_end = __builtin_amdgcn_readfirstlane((me + 1) * total / G);

  const int t = threadIdx.x;
  const int lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
  const int fp = lane & 31, fh = lane >> 5;
  T* __restrict__ y = static_cast<T*>(p.y);

  const int c16 = lane & 7;                           // physical 16-byte group this lane fills
  const int lrow = wave * 8 + (lane >> 3);            // tile row (plus 32 per transfer)
  const int lc = c16 ^ ((lrow >> 1) & 7);             // logical group it fetches
  const uint32_t b_voff = (uint32_t)((lrow * p.k_pad + lc * V) * EB);

  constexpr int CPR = BN * EB / 16;        // 16-byte groups per output row slice
  constexpr int RPI = kThreads / CPR;      // dense rows per fill pass of the workgroup
  constexpr int ZB = 4;                    // passes whose mask bytes are fetched up front
  const int zc = t % CPR, zr = t / CPR;

  const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.x), 0, (int)p.x_bytes, kBufferWord3);
  const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.wp), 0, (int)p.w_bytes, kBufferWord3);
  typedef __attribute__((address_space(3))) void lds_void;
  const int step_x = p.dil_w * p.xs_w * EB, step_y = p.dil_h * p.xs_h * EB;

  const unsigned lds0 = (unsigned)(unsigned long long)(__attribute__((address_space(3))) unsigned char*)smem;
  unsigned frag_a[4], frag_b[4];   // LDS address of this lane's fragment of K step ks in ring slot 0
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const unsigned o = (unsigned)(fp * kRowBytes + (((2 * ks + fh) ^ ((fp >> 1) & 7)) << 4));
    frag_a[ks] = lds0 + wm0 * kRowBytes + o;
    frag_b[ks] = lds0 + (BM + wn0) * kRowBytes + o;
  }

  bool first_unit = true;
  while (s_at < s_end) {
    // ---- the unit: K tiles [kt_lo, kt_lo + n_steps) of one output tile ----------------------------------
    const unsigned tile = s_at / n_kt;
    const int kt_lo = (int)(s_at - tile * n_kt);
    const int n_steps = (int)min(n_kt - (unsigned)kt_lo, s_end - s_at);
    const int tile_m = (int)tile / p.n_tiles;
    const int tile_n = (int)tile - tile_m * p.n_tiles;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    // every wavefront has left the previous unit (ring, row list, bias slice, flag) and its stores have been
    // acknowledged, so that the ring's vmcnt arithmetic below counts the ring's transfers only
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    // ---- one round trip: row numbers, bias slice, the dense row range this tile owns -------------------
    int32_t a_row[A_LOADS];
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j) {
      const int icc = min(m0 + lrow + 32 * j, p.rows - 1);
      a_row[j] = p.row_idx ? p.row_idx[icc] : icc;
    }
    float bias_v = 0.0f;
    if (t < BN && p.bias && n0 + t < p.c_out) bias_v = p.bias[n0 + t];
    int z_lo = 0, z_hi = p.m_total;
    if (p.zero_fill) {
      if (tile_m != 0) z_lo = p.row_idx[m0];
      if (m0 + BM < p.rows) z_hi = p.row_idx[m0 + BM];
    }
    int32_t a_voff[A_LOADS];
    uint32_t a_taps[A_LOADS];
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j) {
      const bool present = m0 + lrow + 32 * j < p.rows;
      const int ic = m0 + lrow + 32 * j;                       // position in the compacted GEMM
      const int rr = present ? (p.y_compact ? ic : a_row[j]) : -1;   // row the epilogue stores to
      if (c16 == 0) s_rows[lrow + 32 * j] = rr;
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
    unsigned mk[ZB];
#pragma unroll
    for (int u = 0; u < ZB; ++u) {
      int r = min(z_lo + zr + u * RPI, p.m_total - 1);
      if (p.mask_spatial) r -= fast_div(r, p.div_howo_mul, p.div_howo_shift) * p.ho_wo;
      mk[u] = p.mask[r];
    }
    __syncthreads();   // s_rows written; nothing is in flight

    // scalar walk over the window, entered at K tile kt_lo: a K tile lies in tap (s_ky, s_kx) at channel s_ci
    const int k0 = kt_lo * BK;
    const int tap0 = k0 / p.c_in;
    int s_ci = k0 - tap0 * p.c_in;
    int s_ky = tap0 / p.kw;
    int s_kx = tap0 - s_ky * p.kw;
    int s_off = s_ci * EB + s_kx * step_x + s_ky * step_y;   // byte offset of that tap and channel
    uint32_t s_bits = (1u << s_ky) | (1u << (8 + s_kx));      // its two validity bits
    int s_boff = (n0 * p.k_pad + k0) * EB;                    // byte offset of filter row n0 at the current K tile
    auto issue_tile = [&](auto stage_c) {
      constexpr int ST = decltype(stage_c)::value;
      unsigned char* sa = smem + ST * STAGE_BYTES + wave * 8 * kRowBytes;      // this wavefront's 8 rows
      unsigned char* sb = sa + BM * kRowBytes;
#pragma unroll
      for (int j = 0; j < A_LOADS; ++j) {
        const bool ok = (a_taps[j] & s_bits) == s_bits;
        const uint32_t voff = ok ? (uint32_t)(a_voff[j] + s_off) : kOutOfRange;   // out of range: LDS gets zeros
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (lds_void*)(sa + j * 32 * kRowBytes), 16, voff, 0, 0, 0);
      }
#pragma unroll
      for (int j = 0; j < B_LOADS; ++j)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (lds_void*)(sb + j * 32 * kRowBytes), 16, b_voff,
                                                 s_boff + j * 32 * p.k_pad * EB, 0, 0);
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
    };

    floatx16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

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

    // one K tile: wait until it has landed, refill the slot the previous tile occupied, contract
    int issued = 0;
    auto k_tile = [&](auto stage_c, int kt) {
      constexpr int ST = decltype(stage_c)::value;
      if (kt + STAGES - 2 < n_steps) wait_vmcnt<(STAGES - 2) * LPT>();
      else wait_vmcnt<0>();
      __builtin_amdgcn_s_barrier();   // landed for every wavefront; and all have left tile kt-1
      asm volatile("" ::: "memory");
      if (issued < n_steps) {
        issue_tile(std::integral_constant<int, (ST + STAGES - 1) % STAGES>{});
        ++issued;
      }
      v4i f0[MI + NI], f1[MI + NI], f2[MI + NI], f3[MI + NI];
      read_step(stage_c, 0, f0);
      read_step(stage_c, 1, f1);
      wait_frags<MI + NI>(f0);
      mma_step(f0);
      read_step(stage_c, 2, f2);
      wait_frags<MI + NI>(f1);
      mma_step(f1);
      read_step(stage_c, 3, f3);
      wait_frags<MI + NI>(f2);
      mma_step(f2);
      wait_frags<0>(f3);
      mma_step(f3);
    };

    // ---- K loop of the unit, unrolled over the ring -----------------------------------------------------
    if (0 < n_steps) { issue_tile(std::integral_constant<int, 0>{}); ++issued; }
    if constexpr (STAGES >= 3) if (1 < n_steps) { issue_tile(std::integral_constant<int, 1>{}); ++issued; }
    if constexpr (STAGES >= 4) if (2 < n_steps) { issue_tile(std::integral_constant<int, 2>{}); ++issued; }
    static_assert(STAGES <= 4, "ring of at most four tiles");
    for (int kt = 0; kt < n_steps; kt += STAGES) {
      k_tile(std::integral_constant<int, 0>{}, kt);
      if (kt + 1 < n_steps) k_tile(std::integral_constant<int, 1 % STAGES>{}, kt + 1);
      if constexpr (STAGES >= 3) if (kt + 2 < n_steps) k_tile(std::integral_constant<int, 2 % STAGES>{}, kt + 2);
      if constexpr (STAGES >= 4) if (kt + 3 < n_steps) k_tile(std::integral_constant<int, 3 % STAGES>{}, kt + 3);
    }

    // ---- a shared tile: leave the partial sums; the last arrival adds them up --------------------------
    bool finish = true;
    if (n_steps != (int)n_kt) {
      // Partial sums travel through device-scope relaxed atomic stores and loads of 8 bytes (they write
      // through to, and read from, the point where the XCDs' L2 caches agree; no cache-wide fence).
      // Order: stores acknowledged (vmcnt 0) -> workgroup barrier -> arrival counter; the last arrival
      // reads after it has seen every other arrival.
      constexpr int PER_WAVE = MI * NI * 8;     // 8-byte chunks per lane
      constexpr int SLOT = (kThreads / 64) * PER_WAVE * 64;   // 8-byte chunks per slot
      typedef unsigned long long u64;
      u64* part = reinterpret_cast<u64*>(p.partial);
      u64* mine = part + (int64_t)(2 * me + (first_unit ? 0 : 1)) * SLOT + wave * PER_WAVE * 64 + lane;
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
      __syncthreads();
      // the workgroups whose ranges meet this tile: the owners of its first and of its last step, and all between
      const unsigned q0 = tile * n_kt, q1 = q0 + n_kt - 1;
      const unsigned w_first = ((q0 + 1) * G - 1) / total, w_last = ((q1 + 1) * G - 1) / total;
      if (t == 0) {
        const int last = (int)(w_last - w_first);
        const int old = __hip_atomic_fetch_add(p.counters + tile, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // everybody has arrived: leave the counter at zero for the next launch
        if (old == last) __hip_atomic_store(p.counters + tile, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *s_flag = old == last ? 1 : 0;
      }
      __syncthreads();
      finish = __builtin_amdgcn_readfirstlane(*s_flag) != 0;
      if (finish) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
          for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;
        for (unsigned w = w_first; w <= w_last; ++w) {      // ascending K ranges: the sum does not depend on who came last
          // a range that starts inside this tile has it as its first unit, else (only w_first) as its second
          const unsigned slot = 2 * w + ((w * total / G) >= q0 ? 0u : 1u);
          const u64* src = part + (int64_t)slot * SLOT + wave * PER_WAVE * 64 + lane;
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

    if (finish) {
      // ---- zero fill of the dropped rows this tile owns (Alg. 2, mask == 0 branch) -----------------------
      if (t < BN) s_bias[t] = bias_v;
      asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // LDS only: the bias slice
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

      // ---- epilogue ------------------------------------------------------------------------------------
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        const int rr = s_rows[wm0 + mi * 32 + fp];
        if (rr < 0) continue;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
          const int c0 = n0 + wn0 + ni * 32 + 16 * fh;
          if (c0 >= p.c_out) continue;
          store_kept_block_res<DT>(acc[mi][ni], rr, c0, y, p.bias ? s_bias + (c0 - n0) : nullptr, 0, p.relu, 1, p.c_out,
                                   p.ho_wo, 0, 0, 0, static_cast<const T*>(p.residual), p.residual_relu);
        }
      }
    }
    s_at += (unsigned)n_steps;
    first_unit = false;
  }
}

template <int DT, int BM, int BN, int WAVES_M, int WAVES_N, int STAGES>
hipError_t igemm_streamk_launch(const ConvParams& p, hipStream_t stream) {
  constexpr size_t lds = igemm_dma_lds_bytes<BM, BN, STAGES>();
  auto kern = igemm_streamk_kernel<DT, BM, BN, WAVES_M, WAVES_N, STAGES>;
  static std::atomic<bool> attr_set{false};
  if (lds > 64 * 1024 && !attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3(p.stream_wgs), dim3(kThreads), lds, stream, p);
  return hipGetLastError();
}

}  // namespace sc
