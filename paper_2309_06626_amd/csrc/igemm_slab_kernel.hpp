// Tiled masked-convolution kernel whose lowered rows come from a resident input slab, for deep 3x3 layers
// (stride 1, no dilation, 16-bit NHWC, input channels a multiple of 32, output channels a multiple of 16).
//
// The lowered matrix of a 3x3 layer (paper Sec. 3, Fig. 1) holds every input pixel nine times, and the tiled
// kernels fetch it that way: per K tile a workgroup moves BM x 128 bytes of window entries from L2 into LDS next
// to BN x 128 bytes of filters, and on this GPU that path (about 60-76 KB per microsecond and compute unit),
// not the matrix cores, bounds their K loop.  Here the K loop runs chunk-major: for every chunk of 32 input
// channels the workgroup holds, in LDS, the slab of input pixels that the windows of its BM kept rows touch
// (Sec. 3.2: only kept rows are lowered -- the slab spans from the first to the last kept row of the tile),
// fetched from L2 once and read nine times, once per tap, by the MFMA fragment reads; only the filters stream.
//
//   slab      virtual zero-padded rows: row n * Hp + iy + pad_h of width Wp = W + 2 * pad_w (Hp = H + 2 * pad_h);
//             the output pixel (n, oy, ox) has its window's top-left corner at virtual row n * Hp + oy, column ox,
//             and tap (ky, kx) lies Wp * ky + kx pixels further -- the same displacement for every row, so a
//             lane's fragment address for a tap is a constant computed once.  The tile's slab is the run of
//             virtual rows from the first kept row's window to the last kept row's; padding pixels are written
//             as zeros by the hardware (buffer loads with an offset past the end of the buffer).
//   LDS       64 bytes per pixel and chunk, 16-byte groups stored at (group ^ ((pixel >> 2) & 3)): sixteen lanes
//             that read consecutive pixels touch every bank once (kept rows are a random subset of the pixels, so
//             two of sixteen may still meet: measured, not assumed).  Two slab buffers: chunk c + 1 arrives under
//             the MFMAs of chunk c.
//   filters   one stage = the three taps of a window row for one chunk: 3 x 128 filter rows x 64 bytes, ring of
//             three stages, so the ring slot of a stage is its window row (a compile-time constant).
//   K order   (chunk, ky, kx, channel): any order of the K sum is a valid order; the oracle comparison bounds it.
//   waits     "all my transfers except the newest stage's have landed", then a workgroup barrier.  A window row's
//             stage issues the filter transfers of the stage two ahead and, in a chunk's first stage, the slab of
//             the next chunk in front of them -- one transfer behind each MFMA.
//
// Tile = BM kept rows x 128 channels, wavefronts of 64 x 64.  Zero-fill ownership, epilogue and the split-K
// exchange (K split by chunks) are those of igemm_buf_kernel.
//
// SC_SLAB_PROBE (development builds only; results are wrong on purpose, every access stays where the real kernel's
// is): 1 = every filter transfer fetches the first chunk's tile (always an L2 hit), 2 = so does every slab
// transfer, 3 = one K step of six issues MFMAs, 4 = no transfers at all -- what each part of a stage costs.
#pragma once
#include <type_traits>

#include "igemm_buf_kernel.hpp"

namespace sc {

constexpr int kSlabCh = 32;                              // input channels per chunk
constexpr int kSlabPixelBytes = kSlabCh * 2;             // 64
constexpr int kSlabBN = 128;
constexpr int kSlabTapBytes = kSlabBN * kSlabPixelBytes; // filter tile of one tap and chunk
constexpr int kSlabStageBytes = 3 * kSlabTapBytes;       // one window row
constexpr int kSlabRing = 3;
constexpr int kSlabMostBytes = 40960;                    // one slab buffer at most (two of them beside the ring)

template <int BM>
constexpr size_t igemm_slab_lds_bytes(int slab_bytes) {
  return (size_t)kSlabRing * kSlabStageBytes + 2 * (size_t)slab_bytes + (BM + 4) * sizeof(int32_t) + kSlabBN * sizeof(float);
}

template <int DT, int BM, int WAVES_M, int WAVES_N, bool SPLITK>
__global__ __launch_bounds__(WAVES_M * WAVES_N * 64) void igemm_slab_kernel(const ConvParams p) {
  using E = Elem<DT>;
  using T = typename E::T;
  constexpr int EB = sizeof(T);
  constexpr int BN = kSlabBN;
  constexpr int NT = WAVES_M * WAVES_N * 64;
  constexpr int NW = NT / 64;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int MI = WM / 32, NI = WN / 32;
  constexpr int PPR = NT / 4;                                  // slab pixels per transfer round of the workgroup
  constexpr int ROUND_BYTES = NT * 16;
  constexpr int J_MAX = kSlabMostBytes / ROUND_BYTES;          // slab transfers per wavefront and chunk at most
  constexpr int RPT = NW * 16;                                 // filter rows per transfer round
  constexpr int ROUNDS_PER_TAP = BN / RPT;                     // 1 (eight wavefronts) or 2
  constexpr int BPW = 3 * ROUNDS_PER_TAP;                      // filter transfers per wavefront and stage
  constexpr int RING_BYTES = kSlabRing * kSlabStageBytes;
  constexpr int MMAS = 6 * MI * NI;                            // MFMAs of a wavefront per stage
  static_assert(EB == 2, "16-bit operands");
  static_assert(NT == 256 || NT == 512, "four or eight wavefronts");
  static_assert(MI == 2 && NI == 2, "wavefront tiles of 64 x 64");
  static_assert(J_MAX + BPW <= MMAS, "a slot behind an MFMA for every transfer of a stage");
  static_assert(BPW <= 63, "vmcnt is a 6-bit counter");

  extern __shared__ __align__(16) unsigned char smem[];
  const int slab_bytes = p.slab_bytes;                         // one buffer; a multiple of ROUND_BYTES
  int32_t* s_rows = reinterpret_cast<int32_t*>(smem + RING_BYTES + 2 * slab_bytes);   // [BM], then one spare group
  float* s_bias = reinterpret_cast<float*>(s_rows + BM + 4);                          // [BN]

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
  const int n_chunks = p.c_in / kSlabCh;
  const int c_lo = SPLITK ? (int)((int64_t)split * n_chunks / splits) : 0;
  const int c_hi = SPLITK ? (int)((int64_t)(split + 1) * n_chunks / splits) : n_chunks;
  const int n_q = (c_hi - c_lo) * 3;                           // stages of this workgroup

  const int t = threadIdx.x;
  const int lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
  const int fp = lane & 31, fh = lane >> 5;
  T* __restrict__ y = static_cast<T*>(p.y);
  const int hp = p.slab_hp, wp = p.slab_wp;

  // ---- one round trip: row numbers, bias slice, the dense row range this workgroup owns -------------
  const int i_last = min(m0 + BM, p.rows) - 1;
  const int r_first = p.row_idx ? p.row_idx[m0] : m0;
  const int r_last = p.row_idx ? p.row_idx[i_last] : i_last;
  int my_row = -1, my_i = 0;                                    // tile row t (t < BM): the row the epilogue stores to
  if (t < BM) {
    my_i = min(m0 + t, p.rows - 1);
    my_row = p.row_idx ? p.row_idx[my_i] : my_i;
  }
  int f_row[MI];                                                // rows of this lane's fragments
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    const int ic = min(m0 + wm0 + mi * 32 + fp, p.rows - 1);
    f_row[mi] = p.row_idx ? p.row_idx[ic] : ic;
  }
  float bias_v = 0.0f;
  if (t < BN && p.bias && n0 + t < p.c_out) bias_v = p.bias[n0 + t];
  int z_lo = 0, z_hi = p.m_total;
  if (p.zero_fill) {
    if (tile_m != 0) z_lo = r_first;
    if (m0 + BM < p.rows) z_hi = p.row_idx[m0 + BM];
  }
  constexpr int CPR = BN * EB / 16;        // 16-byte groups per output row slice
  constexpr int RPI = NT / CPR;            // dense rows per fill pass of the workgroup
  constexpr int ZB = 4;                    // passes whose mask bytes are fetched up front
  const int zc = t % CPR, zr = t / CPR;
  unsigned mk[ZB];
#pragma unroll
  for (int u = 0; u < ZB; ++u) {
    int r = min(z_lo + zr + u * RPI, p.m_total - 1);
    if (p.mask_spatial) r -= fast_div(r, p.div_howo_mul, p.div_howo_shift) * p.ho_wo;
    mk[u] = p.mask[r];
  }

  // virtual row of a dense output row's window corner
  auto corner = [&](int r, int* vrow, int* col) {
    const int n = fast_div(r, p.div_howo_mul, p.div_howo_shift), rem = r - n * p.ho_wo;
    const int oy = fast_div(rem, p.div_wo_mul, p.div_wo_shift);
    *vrow = n * hp + oy;
    *col = rem - oy * p.wo;
  };
  int vr_lo, vr_last, col_unused;
  corner(r_first, &vr_lo, &col_unused);
  corner(r_last, &vr_last, &col_unused);
  const int slab_rows = vr_last + p.kh - vr_lo;                // virtual rows the tile's windows touch
  const int slab_px = slab_rows * wp;
  // transfer rounds of a chunk's slab; never past the buffer (the host sizes the buffer for the widest tile)
  const int j_tile = min((slab_px + PPR - 1) / PPR, slab_bytes / ROUND_BYTES);

  if (t < BM) s_rows[t] = m0 + t < p.rows ? (p.y_compact ? my_i : my_row) : -1;
  if (t < BN) s_bias[t] = bias_v;

  const unsigned lds0 = (unsigned)(unsigned long long)(__attribute__((address_space(3))) unsigned char*)smem;
  const unsigned slab0 = lds0 + RING_BYTES;

  // fragment addresses of the lowered rows: pixel P of the slab at 64 * P, group g at (g ^ ((P >> 2) & 3));
  // K step 0 of a tap reads group fh, K step 1 group 2 + fh = the same address with bit 5 flipped
  unsigned a_tap[MI][9];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    int vrow, col;
    corner(f_row[mi], &vrow, &col);
    const int p0 = (vrow - vr_lo) * wp + col;
#pragma unroll
    for (int ky = 0; ky < 3; ++ky)
#pragma unroll
      for (int kx = 0; kx < 3; ++kx) {
        const int px = p0 + ky * wp + kx;
        a_tap[mi][ky * 3 + kx] = slab0 + (unsigned)(px * kSlabPixelBytes + (((fh ^ (px >> 2)) & 3) << 4));
      }
  }
  // filter fragments: tile row at 64 * row, group g at (g ^ ((row >> 2) & 3))
  unsigned b_frag[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks)
    b_frag[ks] = lds0 + (unsigned)((wn0 + fp) * kSlabPixelBytes + ((((2 * ks + fh) ^ (fp >> 2)) & 3) << 4));

  // what this lane transfers of a slab: pixel j * PPR + t / 4, the group that lands at position t % 4
  uint32_t s_voff[J_MAX];
#pragma unroll
  for (int j = 0; j < J_MAX; ++j) {
    const int px = j * PPR + (t >> 2);
    const int grp = (t & 3) ^ ((px >> 2) & 3);
    const int sr = fast_div(px, p.div_wp_mul, p.div_wp_shift), vc = px - sr * wp;
    const int vr = vr_lo + sr;
    const int n = fast_div(vr, p.div_hp_mul, p.div_hp_shift);
    const int iy = vr - n * hp - p.ph, ix = vc - p.pw;
    const bool ok = sr < slab_rows && (unsigned)iy < (unsigned)p.h && (unsigned)ix < (unsigned)p.w;
    s_voff[j] = ok ? (uint32_t)((((n * p.h + iy) * p.w + ix) * p.c_in + grp * 8) * EB) : kOutOfRange;
  }
  // of a filter stage: rows wave * 16 + lane / 4 (+ RPT per further round), the group that lands at position lane % 4
  const uint32_t b_voff = (uint32_t)(((n0 + wave * 16 + (lane >> 2)) * p.k_pad + (((lane & 3) ^ ((lane >> 4) & 3)) * 8)) * EB);

  const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.x), 0, (int)p.x_bytes, kBufferWord3);
  const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p.wp), 0, (int)p.w_bytes, kBufferWord3);
  typedef __attribute__((address_space(3))) void lds_void;

  auto issue_slab = [&](auto j_c, int chunk, int buf) {
    constexpr int J = decltype(j_c)::value;
    unsigned char* dst = smem + RING_BYTES + buf * slab_bytes + J * ROUND_BYTES + wave * 1024;
    const uint32_t voff = s_voff[J];     // (a local: as a direct argument the host pass drops the kernel's stub)
#if defined(SC_SLAB_PROBE) && SC_SLAB_PROBE == 2
    chunk = 0;
#endif
#if defined(SC_SLAB_PROBE) && SC_SLAB_PROBE == 4
    return;
#endif
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (lds_void*)dst, 16, voff, chunk * kSlabPixelBytes, 0, 0);
  };
  // transfer B of the filter stage (chunk, window row KY): tap B / ROUNDS_PER_TAP, rows (B % ROUNDS_PER_TAP) * RPT ...
  auto issue_filters = [&](auto ky_c, auto b_c, int chunk) {
    constexpr int KY = decltype(ky_c)::value, B = decltype(b_c)::value;
    constexpr int KX = B / ROUNDS_PER_TAP, H = B % ROUNDS_PER_TAP;
    unsigned char* dst = smem + KY * kSlabStageBytes + KX * kSlabTapBytes + (H * RPT) * kSlabPixelBytes + wave * 1024;
#if defined(SC_SLAB_PROBE) && (SC_SLAB_PROBE == 1 || SC_SLAB_PROBE == 2)
    const int soff = (((KY * 3 + KX) * p.c_in + 0 * chunk) + H * RPT * p.k_pad) * EB;
#else
    const int soff = (((KY * 3 + KX) * p.c_in + chunk * kSlabCh) + H * RPT * p.k_pad) * EB;
#endif
#if defined(SC_SLAB_PROBE) && SC_SLAB_PROBE == 4
    return;
#endif
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (lds_void*)dst, 16, b_voff, soff, 0, 0);
  };
  auto issue_filter_stage = [&](auto ky_c, int chunk) {
    auto one = [&](auto b_c) {
      if constexpr (decltype(b_c)::value < BPW) issue_filters(ky_c, b_c, chunk);
    };
    one(std::integral_constant<int, 0>{}); one(std::integral_constant<int, 1>{}); one(std::integral_constant<int, 2>{});
    one(std::integral_constant<int, 3>{}); one(std::integral_constant<int, 4>{}); one(std::integral_constant<int, 5>{});
    static_assert(BPW <= 6, "at most six filter transfers per wavefront and stage");
  };

  floatx16 acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

  __syncthreads();   // s_rows and s_bias written; nothing is in flight yet

  // ---- prologue: the first chunk's slab, the first two filter stages -----------------------------------
  {
    auto slab_round = [&](auto j_c) {
      if constexpr (decltype(j_c)::value < J_MAX)
        if (decltype(j_c)::value < j_tile) issue_slab(j_c, c_lo, 0);
    };
    slab_round(std::integral_constant<int, 0>{}); slab_round(std::integral_constant<int, 1>{});
    slab_round(std::integral_constant<int, 2>{}); slab_round(std::integral_constant<int, 3>{});
    slab_round(std::integral_constant<int, 4>{}); slab_round(std::integral_constant<int, 5>{});
    slab_round(std::integral_constant<int, 6>{}); slab_round(std::integral_constant<int, 7>{});
    slab_round(std::integral_constant<int, 8>{}); slab_round(std::integral_constant<int, 9>{});
    static_assert(J_MAX <= 10, "at most ten slab transfers per wavefront and chunk");
    issue_filter_stage(std::integral_constant<int, 0>{}, c_lo);
    issue_filter_stage(std::integral_constant<int, 1>{}, c_lo);
  }

  // ---- one stage: window row KY of chunk `chunk`; q = its number within this workgroup ------------------
  auto stage = [&](auto ky_c, int q, int chunk, int buf) {
    constexpr int KY = decltype(ky_c)::value;
    if (q + 1 < n_q) wait_vmcnt<BPW>();      // everything but the newest filter stage has landed: this stage, and in a
    else wait_vmcnt<0>();                    // chunk's first stage its slab (issued three stages ago)
    __builtin_amdgcn_s_barrier();            // ... for every wavefront; and all have left the stage before
    asm volatile("" ::: "memory");
    // side jobs of this stage, one behind each of its first MFMAs: (first stage of a chunk) the next chunk's slab
    // into the other buffer, then the filters of the stage two ahead into the slot the previous stage left
    const bool more_slab = KY == 0 && chunk + 1 < c_hi;
    const bool more_filters = q + 2 < n_q;
    const int f_chunk = KY == 0 ? chunk : chunk + 1;
    using FKY = std::integral_constant<int, (KY + 2) % 3>;
    auto side_job = [&](auto m_c) {
      constexpr int M = decltype(m_c)::value;
      constexpr int FIRST_B = KY == 0 ? J_MAX : 0;
      if constexpr (KY == 0 && M < J_MAX) {
        __builtin_amdgcn_sched_barrier(0);
        if (more_slab && M < j_tile) issue_slab(m_c, chunk + 1, buf ^ 1);
        __builtin_amdgcn_sched_barrier(0);
      } else if constexpr (M >= FIRST_B && M < FIRST_B + BPW) {
        __builtin_amdgcn_sched_barrier(0);
        if (more_filters) issue_filters(FKY{}, std::integral_constant<int, M - FIRST_B>{}, f_chunk);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    auto read_step = [&](auto s_c, v4i (&f)[MI + NI]) {
      constexpr int S = decltype(s_c)::value, KX = S / 2, KS = S % 2;
      constexpr int BO = KY * kSlabStageBytes + KX * kSlabTapBytes;
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) f[mi] = lds_read16_at<0>(a_tap[mi][KY * 3 + KX] ^ (unsigned)(KS * 32));
      f[MI + 0] = lds_read16_big<BO>(b_frag[KS]);
      f[MI + 1] = lds_read16_big<BO + 32 * kSlabPixelBytes>(b_frag[KS]);
    };
    auto mma_step = [&](auto s_c, const v4i (&f)[MI + NI]) {
      constexpr int S = decltype(s_c)::value;
#if defined(SC_SLAB_PROBE) && SC_SLAB_PROBE == 3
      if (S == 0) { E::mma(acc[0][0], f[MI + 0], f[0]); E::mma(acc[0][1], f[MI + 1], f[0]); E::mma(acc[1][0], f[MI + 0], f[1]); E::mma(acc[1][1], f[MI + 1], f[1]); }
      side_job(std::integral_constant<int, S * 4 + 0>{}); side_job(std::integral_constant<int, S * 4 + 1>{});
      side_job(std::integral_constant<int, S * 4 + 2>{}); side_job(std::integral_constant<int, S * 4 + 3>{});
#else
      E::mma(acc[0][0], f[MI + 0], f[0]); side_job(std::integral_constant<int, S * 4 + 0>{});
      E::mma(acc[0][1], f[MI + 1], f[0]); side_job(std::integral_constant<int, S * 4 + 1>{});
      E::mma(acc[1][0], f[MI + 0], f[1]); side_job(std::integral_constant<int, S * 4 + 2>{});
      E::mma(acc[1][1], f[MI + 1], f[1]); side_job(std::integral_constant<int, S * 4 + 3>{});
#endif
    };
    using S0 = std::integral_constant<int, 0>; using S1 = std::integral_constant<int, 1>;
    using S2 = std::integral_constant<int, 2>; using S3 = std::integral_constant<int, 3>;
    using S4 = std::integral_constant<int, 4>; using S5 = std::integral_constant<int, 5>;
    v4i f0[MI + NI], f1[MI + NI], f2[MI + NI], f3[MI + NI], f4[MI + NI], f5[MI + NI];
    read_step(S0{}, f0);
    read_step(S1{}, f1);
    wait_frags<MI + NI>(f0); mma_step(S0{}, f0);
    read_step(S2{}, f2);
    wait_frags<MI + NI>(f1); mma_step(S1{}, f1);
    read_step(S3{}, f3);
    wait_frags<MI + NI>(f2); mma_step(S2{}, f2);
    read_step(S4{}, f4);
    wait_frags<MI + NI>(f3); mma_step(S3{}, f3);
    read_step(S5{}, f5);
    wait_frags<MI + NI>(f4); mma_step(S4{}, f4);
    wait_frags<0>(f5); mma_step(S5{}, f5);
  };

  // ---- main loop: three stages per chunk, the slab buffers alternate -------------------------------------
  {
    int q = 0, buf = 0;
    for (int chunk = c_lo; chunk < c_hi; ++chunk) {
      stage(std::integral_constant<int, 0>{}, q, chunk, buf);
      stage(std::integral_constant<int, 1>{}, q + 1, chunk, buf);
      stage(std::integral_constant<int, 2>{}, q + 2, chunk, buf);
      q += 3;
      const unsigned delta = buf ? (unsigned)(-slab_bytes) : (unsigned)slab_bytes;
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int tap = 0; tap < 9; ++tap) a_tap[mi][tap] += delta;
      buf ^= 1;
    }
  }

  // ---- split K: leave the partial sums; the last workgroup of the tile adds them up ----------------------
  if constexpr (SPLITK) {
    if (splits > 1) {
      // Order: stores acknowledged (vmcnt 0) -> workgroup barrier -> arrival counter (device scope); the last
      // arrival reads after it has seen every other arrival.  No cache-wide fence anywhere.
      constexpr int CHUNKS = MI * NI * 4;                    // 16-byte chunks per lane
      constexpr int64_t SLOT = (int64_t)NW * CHUNKS * 64;    // chunks per (tile, split)
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
      // fixed order: the sum does not depend on who came last; split sp + 1 is requested before sp is added
      v4i got[2][CHUNKS];
      auto request = [&](int sp, v4i (&dst)[CHUNKS]) {
        const v4i* src = part + (int64_t)sp * SLOT + (int64_t)wave * CHUNKS * 64 + lane;
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c) dst[c] = load16_device_scope(src + c * 64);
      };
      auto add = [&](v4i (&src)[CHUNKS]) {
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
        if (sp + 1 < splits) { request(sp + 1, got[1]); wait_vmcnt<CHUNKS>(); } else wait_vmcnt<0>();
        add(got[0]);
        if (sp + 1 < splits) {
          if (sp + 2 < splits) { request(sp + 2, got[0]); wait_vmcnt<CHUNKS>(); } else wait_vmcnt<0>();
          add(got[1]);
        }
      }
    }
  }

  // ---- zero fill of the dropped rows this workgroup owns (Alg. 2, mask == 0 branch) --------------------
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

template <int DT, int BM, int WAVES_M, int WAVES_N, bool SPLITK>
hipError_t igemm_slab_launch(const ConvParams& p, hipStream_t stream) {
  constexpr int NT = WAVES_M * WAVES_N * 64;
  if (p.slab_bytes <= 0 || p.slab_bytes % (NT * 16) != 0 || p.slab_bytes > kSlabMostBytes) return hipErrorInvalidValue;
  const size_t lds = igemm_slab_lds_bytes<BM>(p.slab_bytes);
  auto kern = igemm_slab_kernel<DT, BM, WAVES_M, WAVES_N, SPLITK>;
  static std::atomic<bool> attr_set{false};
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)igemm_slab_lds_bytes<BM>(kSlabMostBytes));
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int nwg = p.m_tiles * p.n_tiles * (SPLITK ? p.splits : 1);
  const int grid = ((nwg + 7) / 8) * 8;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(NT), lds, stream, p);
  return hipGetLastError();
}

// the slab form for tiles of bm x 128 of a 16-bit dtype (bm = 256: eight wavefronts; 128: four), or null
LaunchFn slab_kernel(int dtype, int bm, bool splitk);

}  // namespace sc
