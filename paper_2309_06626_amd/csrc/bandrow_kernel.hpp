// Band kernel for small-channel layers (the 3-channel 7x7 stem of a ResNet): 16-bit NHWC inputs whose pixels are
// no whole 16-byte groups, so that the lowered matrix (paper Sec. 3, Fig. 1) cannot be gathered in channel groups.
//
// K is ordered (window row ky, entry e = kx * Cin + c) with every window row padded to a multiple of eight entries (the
// packing the row-segment tiled kernel uses): a window row of an output pixel is then kw * Cin CONTIGUOUS elements of
// one input row, i.e. one, two ... 16-byte groups that start at the pixel's first tap.  The tiled kernel fetches those
// groups from a zero-margined copy of the input in global memory, row by kept row, and spends its time issuing
// instructions.  Here a workgroup owns a band of output rows of one image (Sec. 3.2: only the kept windows of the band
// are lowered) and
//   * stages the band's input rows once into LDS, each with zero margins left and right and zero rows above / below
//     the image, so that no window entry needs a bounds check: a lane's fragment of (ky, group) is the 16 bytes at
//     [its pixel's slab address] + ky * row pitch + 16 * group -- immediates on one register per 32-row block;
//   * keeps the 64 filter rows of its channel tile in LDS (an odd number of 16-byte groups apart: sixteen rows, sixteen
//     bank groups);
//   * masks the entries of a window row's last group that lie beyond the window (their filter entries are zero, but a
//     non-finite neighbour pixel must not meet them);
//   * writes the band's outputs once: results of kept rows, zeros of dropped rows (Alg. 2), as the other band kernels.
// Window starts are 4-byte aligned in the slab (Cin * stride_w even, left margin chosen accordingly): fragments are read
// with LDS reads of two dwords each (ds_read2_b32), which need no more than that.
//
//   workgroup  = one band (BH output rows x all Wo columns of one image) x 64 output channels, four wavefronts
//   wavefront  = 64-row MFMA block pairs b = wave, wave + 4, ... of the band's kept rows
//   LDS        = filters [64][fpitch] | 256 B zeros | bias [64] | slab [IH rows][pitch]
#pragma once
#include "band_kernel.hpp"
#include "igemm_dma_kernel.hpp"

namespace sc {

constexpr int kRowBandMostGroups = 24;                         // 16-byte groups of K at most
// LDS layout: 64 filter rows `fpitch` bytes apart, 256 bytes of zeros, 64 bias floats, the slab.  fpitch = 16 * (an odd
// number of groups >= K's): sixteen consecutive rows then start in sixteen different 16-byte bank groups.
constexpr int rowband_filter_pitch(int groups) { return 16 * (groups | 1); }
constexpr int rowband_slab_at(int groups) { return 64 * rowband_filter_pitch(groups) + 512; }
constexpr int kRowBandMaxRows = 512;                           // tallest band (output rows x width)

struct RowBandParams {
  BandParams b;              // tensors, tables, geometry; b.bh, b.bands_per_image, b.n_bands, b.n_tiles as for band_kernel
  int32_t pitch;             // bytes between slab rows (a multiple of 16)
  int32_t left;              // zero pixels in front of a slab row's first input pixel
  int32_t in_rows;           // slab rows of a full band: (bh - 1) * stride_h + (kh - 1) * dil_h + 1
  int32_t gpw;               // 16-byte groups per window row (ceil(kw * Cin / 8))
  int32_t groups;            // kh * gpw
  int32_t tail;              // entries of a window row's last group that lie inside the window (1 .. 8)
  int32_t fpitch;            // bytes between filter rows in LDS: rowband_filter_pitch(groups)
  uint32_t div_cpr_mul, div_cpr_shift;   // n / (pitch / 16) as (n * mul) >> shift
};

// sixteen bytes of LDS at a 4-byte aligned address (two ds_read2_b32)
__device__ __forceinline__ v4i lds_load_4dwords(unsigned addr) {
  const __attribute__((address_space(3))) int* q = (const __attribute__((address_space(3))) int*)(lds_byte*)(unsigned long long)addr;
  return v4i{q[0], q[1], q[2], q[3]};
}

// KH, GPW > 0 fix the window rows and the groups per window row at compile time (the K loop unrolls); 0 = run-time shape.
// (32-row blocks leave room for four wavefronts per SIMD, 64-row blocks for three)
template <int DT, int MI, int KH, int GPW>
__global__ __launch_bounds__(kThreads, MI == 1 ? 4 : 3) void bandrow_kernel(const RowBandParams q) {
  using E = Elem<DT>;
  using T = typename E::T;
  constexpr int EB = sizeof(T);
  constexpr int NI = 2, BN = 64;
  constexpr int CPR = BN * EB / 16;     // 16-byte groups per output row slice
  constexpr int RPI = kThreads / CPR;   // output rows covered by one zero-fill pass of the workgroup
  constexpr int ZIT = kRowBandMaxRows / RPI;
  constexpr int RB = kRowBandMaxRows / (4 * 32 * MI);     // block groups per wavefront that cover the tallest band
  constexpr int STEPS = (KH * GPW + 1) / 2;
  static_assert(EB == 2, "16-bit operands");
  static_assert((KH > 0) == (GPW > 0), "both or neither");
  const BandParams& p = q.b;
  const int gpw = GPW ? GPW : q.gpw, groups = KH ? KH * GPW : q.groups;

  extern __shared__ __align__(16) unsigned char smem[];
  const unsigned lds0 = lds_addr_of(smem);
  const int fpitch = KH ? rowband_filter_pitch(KH * GPW) : q.fpitch;
  const int zero_at = 64 * fpitch, bias_at = zero_at + 256, slab_at = bias_at + 256;
  float* s_bias = reinterpret_cast<float*>(smem + bias_at);

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
  const int iy_base = oy0 * p.sh - p.ph;

  const T* __restrict__ x = static_cast<const T*>(p.x);
  T* __restrict__ y = static_cast<T*>(p.y);

  // ---- small, latency-critical loads first ----------------------------------------------------------------------
  int cnt = r_hi - r_lo;
  if (p.row_idx) cnt = p.band_i0[band + 1] - p.band_i0[band];
  int r_pre[RB][MI];
#pragma unroll
  for (int b = 0; b < RB; ++b)
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      const int j = ((b * 4 + wave) * MI + mi) * 32 + fp;     // position in the band's list
      const int jc = min(j, r_hi - r_lo - 1);
      r_pre[b][mi] = p.row_idx ? p.band_rows[r_lo + jc] : r_lo + jc;
    }
  const int zc = t % CPR, zr = t / CPR;
  unsigned char mk[ZIT];
  if (p.zero_fill) {
#pragma unroll
    for (int u = 0; u < ZIT; ++u) {
      const int r = min(r_lo + zr + u * RPI, r_hi - 1);       // clamped: the loads stay unconditional
      mk[u] = p.mask[p.mask_spatial ? r - img * ho_wo : r];
    }
  }
  float bias_v = 0.0f;
  if (t < BN && p.bias && n0 + t < p.c_out) bias_v = p.bias[n0 + t];

  // ---- filters and slab: every load of a pass is issued before the first LDS write ---------------------------------
  // filters: 64 rows of `groups` 16-byte groups, fpitch bytes apart in LDS; four threads per row
  v4i wv[kRowBandMostGroups / 4];
  {
    const v4i* gw = reinterpret_cast<const v4i*>(static_cast<const T*>(p.wp) + (int64_t)(n0 + (t >> 2)) * p.k_stride);
#pragma unroll
    for (int u = 0; u < kRowBandMostGroups / 4; ++u) {
      const int g = (t & 3) + 4 * u;
      wv[u] = v4i{0, 0, 0, 0};
      if (g < groups) wv[u] = gw[g];
    }
  }
  // slab: 16-byte pieces of LDS, piece i = (slab row i / cpr, piece i % cpr of the row); a piece inside the input row
  // is one 16-byte load at a 2-byte aligned address, a piece across an end of the row is put together from halfwords
  // (by the thread that owns that end of that row), the others (margins, rows above and below the image) are zeros
  {
    constexpr int U = 6;
    const int row_bytes = p.w * p.c_in * EB;                  // an input row in global memory
    const int lead = q.left * p.c_in * EB;                    // zero bytes in front of it in LDS
    const int cpr = q.pitch >> 4;
    const int in_rows = min(q.in_rows, (oy1 - 1 - oy0) * p.sh + (p.kh - 1) * p.dil_h + 1);
    const int pieces = in_rows * cpr;
    const unsigned char* ximg = reinterpret_cast<const unsigned char*>(x) + (int64_t)img * p.h * row_bytes;
    const int e0 = (lead & 15) ? lead >> 4 : -1, e1 = ((lead + row_bytes) & 15) ? (lead + row_bytes) >> 4 : -1;
    // end piece e = (row e / 2, front or back end): its eight halfwords, those outside the row zero
    auto end_piece = [&](int e, v4i* v) -> int {
      const int r = e >> 1, c = (e & 1) ? e1 : e0;
      const int iy = iy_base + r;
      if (e >= 2 * in_rows || c < 0 || (unsigned)iy >= (unsigned)p.h) return -1;
      const unsigned char* src = ximg + (int64_t)iy * row_bytes;
      const int at = 16 * c - lead;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        unsigned short lo = 0, hi = 0;
        if (at + 4 * k >= 0 && at + 4 * k < row_bytes) lo = *reinterpret_cast<const unsigned short*>(src + at + 4 * k);
        if (at + 4 * k + 2 >= 0 && at + 4 * k + 2 < row_bytes) hi = *reinterpret_cast<const unsigned short*>(src + at + 4 * k + 2);
        (*v)[k] = (int)((unsigned)lo | ((unsigned)hi << 16));
      }
      return r * cpr + c;
    };
    for (int base = 0; base < pieces; base += kThreads * U) {
      v4i v[U], ev;
      bool whole[U];
      int end_at = -1;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int i = base + u * kThreads + t;
        const int r = fast_div(i, q.div_cpr_mul, q.div_cpr_shift);
        const int c = i - r * cpr;
        const int at = 16 * c - lead;                         // byte of the input row the piece starts at
        const int iy = iy_base + r;
        const bool row_ok = (unsigned)iy < (unsigned)p.h;
        const unsigned char* src = ximg + (int64_t)(row_ok ? iy : 0) * row_bytes;
        v[u] = v4i{0, 0, 0, 0};
        whole[u] = i < pieces && !(row_ok && (c == e0 || c == e1));      // (end pieces belong to end_piece)
        if (i < pieces && row_ok && at >= 0 && at + 16 <= row_bytes) __builtin_memcpy(&v[u], reinterpret_cast<const unsigned short*>(src + at), 16);
      }
      if (base == 0) end_at = end_piece(t, &ev);
      if (base == 0) {
        // zero fill of the band's dropped rows (Alg. 2, mask == 0 branch): issued behind the loads, drains under the
        // matrix work
        if (p.zero_fill) {
          const int valid = (min(BN, p.c_out - n0) * EB) >> 4;
          const v4i z = {0, 0, 0, 0};
          unsigned char* ybase = reinterpret_cast<unsigned char*>(y) + (int64_t)n0 * EB + zc * 16;
          if (zc < valid) {
#pragma unroll
            for (int u = 0; u < ZIT; ++u) {
              const int r = r_lo + zr + u * RPI;
              if (r < r_hi && mk[u] == 0) sc_store16(reinterpret_cast<v4i*>(ybase + (int64_t)r * p.c_out * EB), z);
            }
          }
        }
#pragma unroll
        for (int u = 0; u < kRowBandMostGroups / 4; ++u) {
          const int g = (t & 3) + 4 * u;
          if (g < groups) *reinterpret_cast<v4i*>(smem + (t >> 2) * fpitch + g * 16) = wv[u];
        }
        if (end_at >= 0) *reinterpret_cast<v4i*>(smem + slab_at + end_at * 16) = ev;
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int i = base + u * kThreads + t;
        if (whole[u]) *reinterpret_cast<v4i*>(smem + slab_at + i * 16) = v[u];
      }
    }
    for (int e = t + kThreads; e < 2 * in_rows; e += kThreads) {       // (slabs of more than 128 rows)
      v4i ev;
      const int end_at = end_piece(e, &ev);
      if (end_at >= 0) *reinterpret_cast<v4i*>(smem + slab_at + end_at * 16) = ev;
    }
    if (t < 16) *reinterpret_cast<v4i*>(smem + zero_at + t * 16) = v4i{0, 0, 0, 0};
    if (t < BN) s_bias[t] = bias_v;
  }
  SC_STAMP(1);
  __syncthreads();   // filters, bias, zeros and the slab are in place
  SC_STAMP(2);

  SC_STAMP(3);
  // which entries of a window row's last group lie inside the window: dword i holds entries 2i, 2i + 1
  v4i tail_mask;
#pragma unroll
  for (int i = 0; i < 4; ++i) tail_mask[i] = q.tail >= 2 * i + 2 ? -1 : q.tail == 2 * i + 1 ? 0xffff : 0;
  const unsigned zaddr = lds0 + zero_at;
  const unsigned slab = lds0 + slab_at;
  const int steps = (groups + 1) >> 1;
  const int ky_pitch = p.dil_h * q.pitch;     // bytes between window rows in the slab
  const int nblk = (cnt + 32 * MI - 1) / (32 * MI);
#pragma unroll
  for (int bi = 0; bi < RB; ++bi) {
    const int blk = bi * 4 + wave;
    if (blk >= nblk) break;
    int rr[MI];
    unsigned a_base[MI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      const int j = (blk * MI + mi) * 32 + fp;
      const int r = r_pre[bi][mi];
      const bool have = j < cnt;
      const int rem = r - img * ho_wo;
      const int oy = fast_div(rem, p.div_wo_mul, p.div_wo_shift), ox = rem - oy * p.wo;
      rr[mi] = have ? r : -1;
      // the window's first entry: slab row (oy - oy0) * sh, pixel left + ox * sw - pw (absent rows read pixel 0 of row 0)
      a_base[mi] = have ? slab + (unsigned)((oy - oy0) * p.sh * q.pitch + (q.left + ox * p.sw - p.pw) * p.c_in * EB) : slab;
    }
    floatx16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;
    if (bi == 0) SC_STAMP(5);

    // K steps of two groups: this lane's group g = 2 * step + fh lies in window row g / gpw, at 16 * (g % gpw) bytes.
    // The fragments of step st + 1 are read while the MFMAs of step st run.
    int ky = 0, part = fh;
    if (part >= gpw) { part -= gpw; ky = 1; }
    auto read_step = [&](int st, v4i (&xf)[MI], v4i (&wf)[NI], bool& last) {
      const int g = 2 * st + fh;
      const bool g_ok = g < groups;
      if constexpr (GPW > 0) { ky = g / GPW; part = g - ky * GPW; }
      const unsigned off = (unsigned)(ky * ky_pitch + part * 16);
      last = part == gpw - 1;
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) xf[mi] = lds_load_4dwords(g_ok ? a_base[mi] + off : zaddr);
      const unsigned wat = lds0 + (unsigned)(fp * fpitch + g * 16);   // (groups beyond K: zeros for both operands)
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) wf[ni] = lds_load16(g_ok ? wat + ni * 32 * fpitch : zaddr);
      if constexpr (GPW == 0) {          // next step's window row and group (gpw >= 1: at most two rows further)
        part += 2;
        if (part >= gpw) { part -= gpw; ++ky; }
        if (part >= gpw) { part -= gpw; ++ky; }
      }
    };
    auto mma_step = [&](v4i (&xf)[MI], v4i (&wf)[NI], bool last) {
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) xf[mi] = last ? xf[mi] & tail_mask : xf[mi];
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) E::mma(acc[mi][ni], wf[ni], xf[mi]);
    };
    v4i xa[MI], wa[NI], xb[MI], wb[NI];
    bool la = false, lb = false;
    read_step(0, xa, wa, la);
    if constexpr (KH > 0) {
#pragma unroll
      for (int st = 0; st < STEPS; st += 2) {
        if (st + 1 < STEPS) read_step(st + 1, xb, wb, lb);
        mma_step(xa, wa, la);
        if (st + 2 < STEPS) read_step(st + 2, xa, wa, la);
        if (st + 1 < STEPS) mma_step(xb, wb, lb);
      }
    } else {
      for (int st = 0; st < steps; st += 2) {
        if (st + 1 < steps) read_step(st + 1, xb, wb, lb);
        mma_step(xa, wa, la);
        if (st + 2 < steps) read_step(st + 2, xa, wa, la);
        if (st + 1 < steps) mma_step(xb, wb, lb);
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
        store_kept_block<DT>(acc[mi][ni], rr[mi], c0, y, p.bias ? s_bias + (c0 - n0) : nullptr, 0, p.relu, 1, p.c_out,
                             ho_wo, 0, 0, 0);
      }
    }
  }
  SC_STAMP(4);
#ifdef SC_TIMING
  if (p.dbg && threadIdx.x == 0) p.dbg[(size_t)blockIdx.x * 8 + 7] = wall_clock64();
#endif
}

template <int DT, int MI, int KH, int GPW>
hipError_t bandrow_launch(const RowBandParams& q, size_t lds, hipStream_t stream) {
  auto kern = bandrow_kernel<DT, MI, KH, GPW>;
  static std::atomic<size_t> attr_bytes{0};   // (plans may be run from several host threads)
  if (lds > 64 * 1024 && lds > attr_bytes) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_bytes = lds;
  }
  const int nwg = q.b.n_bands * q.b.n_tiles;
  const int grid = ((nwg + 7) / 8) * 8;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), lds, stream, q);
  return hipGetLastError();
}

using RowBandLaunchFn = hipError_t (*)(const RowBandParams&, size_t, hipStream_t);
// the kernel for blocks of 32 * mi rows (mi = 1, 2) of a 16-bit dtype and a window of kh rows of gpw groups, or null
RowBandLaunchFn bandrow_kernel_for(int dtype, int mi, int kh, int gpw);

}  // namespace sc
