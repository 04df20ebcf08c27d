// Mask generator of the sparse-training pipeline (Alg. 1, function getMask; described in Sec. 3.1):
// a 2-D score at the resolution of the network input is pooled down to the resolution of a layer,
// the layer's pixels are ranked by the pooled score and the lowest-ranked ones are dropped.
//
// Pooling: the sum of each pixel's window in double, equal bit for bit to the sum added in row-major order of the
// window from +0.0, turned into a 64-bit key whose unsigned order is the order of the sums.
//   one lane per layer pixel for windows below 64 values;
//   one wavefront per layer pixel for larger windows: lane-wise partial sums combined across the wavefront when no
//   addition can round (then the order cannot matter), else one chain of additions in window order from LDS.
// Ranking = selection of the n_drop-th smallest key; pixels whose key equals it are dropped in ascending pixel
// index until the count is exact.  Keys are compared after subtracting the smallest key of the map: the leading bits
// every key shares drop out and the digits of a radix pass spread over their bins however narrow the range of the
// scores is.
// Launches by size of the map (pooling always runs on many workgroups: one workgroup that pools a whole map, even a
// small one, waits for memory pixel after pixel and takes longer than a second launch costs):
//   at most 16 384 pixels: score_key[_wave]_kernel, then mask_select_lds_kernel, one workgroup with every key in
//     LDS -- two launches;
//   larger maps -- four launches, every sweep over the keys spread over the chip:
//     score_key[_wave]_kernel  keys, each workgroup's smallest and largest key, cleared counters
//     mask_hist_kernel    12-bit histogram of (key - smallest key) at the top bits of the keys' range
//     mask_gather_kernel  finds the bin that holds the wanted key, collects that bin's keys (with their pixel
//                         indices) in a list; the workgroup that arrives last selects among them in LDS
//     mask_write_kernel   every pixel compares its key (and index, among equals) with the selected one
#include "../../include/sparse_conv.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <mutex>

namespace sc {

void note_hip_error(int32_t code);   // defined with the other host code of the library

using u64 = unsigned long long;

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kLdsKeys = 16384;      // largest map the one-workgroup selection takes (128 KiB of keys in LDS)
constexpr int kSmallList = 64;       // a candidate set this small is ranked by one wavefront
constexpr int kHistBits = 12, kHistBins = 1 << kHistBits;
constexpr int kChunk = 4 * kSelThreads;          // keys per workgroup in the sweeps of the large-map path
constexpr int kCandCap = 8192;       // most keys the gather pass may collect (96 KiB of LDS in the last workgroup)
constexpr int kSlots = 1024;         // most workgroups of a pooling launch: each leaves its smallest / largest key
constexpr unsigned kNoIndex = 0xffffffffu;

// Device state of one large-map selection, behind the keys in the workspace.  The pooling kernel clears what the
// later kernels accumulate into; everything else is written before it is read.
struct SelState {
  u64 slot_lo[kSlots], slot_hi[kSlots];
  unsigned hist[kHistBins];
  unsigned cand_n, arrived, pad0, pad1;
  u64 threshold;            // the n_drop-th smallest key
  unsigned last_index;      // among the pixels whose key equals it, those up to this index are dropped
  unsigned pad2;
  u64 cand_key[kCandCap];
  unsigned cand_idx[kCandCap];
};

// unsigned order of the result == numeric order of the doubles (-0.0 sorts directly below +0.0; a
// sum that starts from +0.0 never is -0.0)
__device__ __forceinline__ u64 order_key(double v) {
  const u64 b = (u64)__double_as_longlong(v);
  return (b >> 63) ? ~b : (b | 0x8000000000000000ull);
}

__device__ __forceinline__ u64 shfl_xor64(u64 v, int d) {
  const int lo = __shfl_xor((int)(unsigned)v, d, 64), hi = __shfl_xor((int)(unsigned)(v >> 32), d, 64);
  return ((u64)(unsigned)hi << 32) | (unsigned)lo;
}

// smallest and largest of the threads' values, for every thread; `part` holds 2 * waves words of LDS
template <int WAVES> __device__ __forceinline__ void block_min_max(u64& lo, u64& hi, u64* part) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    const u64 ol = shfl_xor64(lo, d), oh = shfl_xor64(hi, d);
    lo = ol < lo ? ol : lo;
    hi = oh > hi ? oh : hi;
  }
  __syncthreads();                       // the previous use of `part` is over
  if (lane == 0) { part[wave] = lo; part[WAVES + wave] = hi; }
  __syncthreads();
#pragma unroll
  for (int w = 0; w < WAVES; ++w) {
    lo = part[w] < lo ? part[w] : lo;
    hi = part[WAVES + w] > hi ? part[WAVES + w] : hi;
  }
}

// What a pooling workgroup leaves for the large-map selection: its extremes, and (workgroup 0) cleared counters.
template <int WAVES> __device__ __forceinline__ void leave_extremes(SelState* st, u64 lo, u64 hi, u64* part) {
  if (!st) return;
  block_min_max<WAVES>(lo, hi, part);
  if (threadIdx.x == 0) { st->slot_lo[blockIdx.x] = lo; st->slot_hi[blockIdx.x] = hi; }
  if (blockIdx.x == 0) {
    for (int b = threadIdx.x; b < kHistBins; b += WAVES * 64) st->hist[b] = 0;
    if (threadIdx.x == 0) { st->cand_n = 0; st->arrived = 0; }
  }
}

__device__ __forceinline__ int bit_length(u64 v) { return v ? 64 - __clzll((long long)v) : 0; }

// Sum of one pooling window by one lane, in double, row-major from +0.0 (windows below 64 values).
__device__ __forceinline__ double lane_window_sum(const float* __restrict__ win, int in_w, int rh, int rw) {
  double acc = 0.0;
  for (int dy = 0; dy < rh; ++dy) {
    const float* row = win + (size_t)dy * in_w;
    for (int dx = 0; dx < rw; dx += 8) {      // eight loads in flight, then their additions in window order
      float v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = dx + j < rw ? row[dx + j] : 0.0f;
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (dx + j < rw) acc = acc + (double)v[j];
    }
  }
  return acc;
}

// Sum of one pooling window by one wavefront (larger windows); the result equals the sum in double, row-major from
// +0.0, bit for bit.  The 64 lanes fetch the window in pieces of PIECE values (neighbouring lanes read neighbouring
// values of a window row) into `piece`, this wavefront's LDS.
//   * A chain of a thousand dependent double additions (with their conversions) costs 12 us on this part, so the
//     chain is avoided whenever the order cannot matter: with every value so far a multiple of 2^q and below 2^E in
//     magnitude, every partial sum of `count` values, in any order, is a multiple of 2^q below 2^(E + ceil(log2 count))
//     and has an exact double when E + ceil(log2 count) - q <= 53 -- no addition rounds, so lane-wise partial sums
//     combined across the wavefront give the row-major result.  (q from the lowest set bit of each float, E from its
//     exponent; scores drawn as k * 2^-24, or any values within a factor 2^19 of each other for 1 024 of them, pass.)
//   * Otherwise (from the first piece that fails on): the piece is added up in window order from LDS, 16 values per
//     batch, the LDS reads of a batch issued while the batch before it is added.  Every lane computes the same sum.
template <int PIECE>
__device__ __forceinline__ double wave_window_sum(const float* __restrict__ win, int in_w, int rw, int count,
                                                  float* __restrict__ piece) {
  const int lane = threadIdx.x & 63;
  const int step_dy = 64 / rw, step_dx = 64 - step_dy * rw;     // 64 values further along the window
  const int log_count = bit_length((u64)(count - 1));
  int e_max = 0, q_min = 1 << 20;      // biased exponent of the largest magnitude, lowest set bit (+150) so far
  bool exact = true;
  double acc = 0.0;
  for (int e0 = 0; e0 < count; e0 += PIECE) {
    const int len = min(PIECE, count - e0);
    int dy = (e0 + lane) / rw, dx = (e0 + lane) - dy * rw;
    double mine = 0.0;
    for (int e = lane; e < len; e += 64 * 8) {          // eight loads in flight per lane
      float v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        v[j] = e + 64 * j < len ? win[(size_t)dy * in_w + dx] : 0.0f;
        dy += step_dy;
        dx += step_dx;
        if (dx >= rw) { dx -= rw; ++dy; }
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (e + 64 * j < len) piece[e + 64 * j] = v[j];
        const unsigned bits = __float_as_uint(v[j]);
        if (bits << 1) {                                       // zeros of either sign change no sum
          const int ex = (int)((bits >> 23) & 0xffu);
          const int eff = ex ? ex : 1;                         // subnormals share the exponent of the smallest normals
          const unsigned mant = (bits & 0x7fffffu) | (ex ? 0x800000u : 0u);
          e_max = max(e_max, ex == 255 ? (1 << 20) : eff);     // infinities never pass
          q_min = min(q_min, eff + (__ffs((int)mant) - 1));
        }
        mine = mine + (double)v[j];
      }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
      e_max = max(e_max, __shfl_xor(e_max, d, 64));
      q_min = min(q_min, __shfl_xor(q_min, d, 64));
    }
    exact = exact && (e_max - q_min + 24 + log_count <= 53);
    if (exact) {
#pragma unroll
      for (int d = 32; d >= 1; d >>= 1)
        mine = mine + __longlong_as_double((long long)shfl_xor64((u64)__double_as_longlong(mine), d));
      acc = acc + mine;
      continue;
    }
    // this wavefront's LDS writes above are visible to its own reads below (one wavefront, LDS in order)
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const float4* p4 = reinterpret_cast<const float4*>(piece);
    const int batches = len >> 4;
    float4 c0, c1, c2, c3;
    if (batches > 0) { c0 = p4[0]; c1 = p4[1]; c2 = p4[2]; c3 = p4[3]; }
    for (int b = 0; b < batches; ++b) {
      float4 n0 = c0, n1 = c1, n2 = c2, n3 = c3;
      if (b + 1 < batches) { n0 = p4[4 * b + 4]; n1 = p4[4 * b + 5]; n2 = p4[4 * b + 6]; n3 = p4[4 * b + 7]; }
      acc = acc + (double)c0.x; acc = acc + (double)c0.y; acc = acc + (double)c0.z; acc = acc + (double)c0.w;
      acc = acc + (double)c1.x; acc = acc + (double)c1.y; acc = acc + (double)c1.z; acc = acc + (double)c1.w;
      acc = acc + (double)c2.x; acc = acc + (double)c2.y; acc = acc + (double)c2.z; acc = acc + (double)c2.w;
      acc = acc + (double)c3.x; acc = acc + (double)c3.y; acc = acc + (double)c3.z; acc = acc + (double)c3.w;
      c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    for (int e = batches << 4; e < len; ++e) acc = acc + (double)piece[e];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
  return acc;
}

constexpr int kKeyThreads = 256;
__global__ __launch_bounds__(kKeyThreads) void score_key_kernel(const float* __restrict__ score, int in_w, int rh, int rw,
                                                                int ho, int wo, u64* __restrict__ keys, SelState* st) {
  __shared__ u64 part[2 * (kKeyThreads / 64)];
  const int n = ho * wo;
  u64 lo = ~0ull, hi = 0ull;
  for (int i = blockIdx.x * kKeyThreads + threadIdx.x; i < n; i += gridDim.x * kKeyThreads) {
    const int oy = i / wo, ox = i - oy * wo;
    const u64 k = order_key(lane_window_sum(score + (size_t)oy * rh * in_w + (size_t)ox * rw, in_w, rh, rw));
    keys[i] = k;
    lo = k < lo ? k : lo;
    hi = k > hi ? k : hi;
  }
  leave_extremes<kKeyThreads / 64>(st, lo, hi, part);
}

// Large pooling windows: one wavefront per layer pixel; lane 0 stores the key.
constexpr int kPoolPiece = 2048;
__global__ __launch_bounds__(kKeyThreads) void score_key_wave_kernel(const float* __restrict__ score, int in_w, int rh,
                                                                     int rw, int ho, int wo, u64* __restrict__ keys,
                                                                     SelState* st) {
  __shared__ __align__(16) float s_piece[kKeyThreads / 64][kPoolPiece];
  __shared__ u64 part[2 * (kKeyThreads / 64)];
  constexpr int WAVES = kKeyThreads / 64;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = ho * wo;
  u64 lo = ~0ull, hi = 0ull;
  for (int i = blockIdx.x * WAVES + wave; i < n; i += gridDim.x * WAVES) {
    const int oy = i / wo, ox = i - oy * wo;
    const u64 k = order_key(wave_window_sum<kPoolPiece>(score + (size_t)oy * rh * in_w + (size_t)ox * rw, in_w, rw, rh * rw,
                                                        s_piece[wave]));
    if (lane == 0) keys[i] = k;
    lo = k < lo ? k : lo;
    hi = k > hi ? k : hi;
  }
  leave_extremes<WAVES>(st, lo, hi, part);
}

__device__ __forceinline__ u64 high_bits(u64 k, int low) { return low >= 64 ? 0ull : k >> low; }

// LDS of a selection by one workgroup of kSelThreads threads
struct SelShared {
  unsigned hist[256];
  u64 small[kSmallList];
  u64 part[2 * kSelWaves];
  unsigned wave_cnt[kSelWaves];
  u64 prefix;
  unsigned remaining, bin_count, small_n;
};

// Selection by one workgroup: among the values get(i, v) yields for i in [0, c) (it returns false for an i that
// is not part of the set), the one of 1-based rank `rank` in ascending order.  Returns it in `value`, together with
// how many members equal it (`equal`) and how many of those belong to the `rank` smallest (`take`).  Radix passes of
// 8 bits over (v - smallest), from the top bit of the range down; once at most kSmallList members share the known
// bits, one wavefront ranks them by counting.  Every thread of the workgroup calls it and receives the result.
template <class Get>
__device__ void block_select(SelShared& sh, Get get, int c, unsigned rank, u64& value, unsigned& take, unsigned& equal) {
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  u64 lo = ~0ull, hi = 0ull;
  unsigned members = 0;
  for (int i = t; i < c; i += kSelThreads) {
    u64 v;
    if (get(i, v)) {
      lo = v < lo ? v : lo;
      hi = v > hi ? v : hi;
      ++members;
    }
  }
  block_min_max<kSelWaves>(lo, hi, sh.part);
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) members += __shfl_xor(members, d, 64);
  __syncthreads();
  if (lane == 0) sh.wave_cnt[wave] = members;
  __syncthreads();
  members = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) members += sh.wave_cnt[w];

  int low = bit_length(hi - lo);       // bits [0, low) of (v - lo) are still unknown, the bits above are `prefix`
  u64 prefix = 0;
  unsigned remaining = rank, bin_count = members;
  while (low > 0 && bin_count > (unsigned)kSmallList) {
    const int width = low < 8 ? low : 8;
    const int shift = low - width;
    const unsigned dmask = (1u << width) - 1u;
    const u64 want_high = high_bits(prefix, low);
    __syncthreads();
    if (t < 256) sh.hist[t] = 0;
    __syncthreads();
    for (int i = t; i < c; i += kSelThreads) {
      u64 v;
      if (get(i, v) && high_bits(v - lo, low) == want_high) atomicAdd(&sh.hist[(unsigned)((v - lo) >> shift) & dmask], 1u);
    }
    __syncthreads();
    if (wave == 0) {   // lane l owns bins 4l .. 4l+3: running count over the 256 bins
      unsigned h[4], sum = 0;
#pragma unroll
      for (int b = 0; b < 4; ++b) { h[b] = sh.hist[lane * 4 + b]; sum += h[b]; }
      unsigned incl = sum;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const unsigned up = __shfl_up(incl, d, 64);
        if (lane >= d) incl += up;
      }
      unsigned before = incl - sum;
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        if (before < remaining && remaining <= before + h[b]) {      // true for exactly one bin of one lane
          sh.prefix = prefix | ((u64)(lane * 4 + b) << shift);
          sh.remaining = remaining - before;
          sh.bin_count = h[b];
        }
        before += h[b];
      }
    }
    __syncthreads();
    prefix = sh.prefix;
    remaining = sh.remaining;
    bin_count = sh.bin_count;
    low = shift;
  }
  if (low == 0) {                      // every bit known: bin_count members equal lo + prefix
    value = lo + prefix;
    take = remaining;
    equal = bin_count;
    return;
  }
  // at most kSmallList members share the known bits: list them, and let one wavefront count, for each of them,
  // the listed members below it and up to it
  const u64 want_high = high_bits(prefix, low);
  __syncthreads();
  if (t == 0) sh.small_n = 0;
  __syncthreads();
  for (int i = t; i < c; i += kSelThreads) {
    u64 v;
    if (get(i, v) && high_bits(v - lo, low) == want_high) sh.small[atomicAdd(&sh.small_n, 1u)] = v - lo;
  }
  __syncthreads();
  if (wave == 0) {
    const unsigned cnt = sh.small_n;
    const u64 mine = lane < (int)cnt ? sh.small[lane] : ~0ull;
    unsigned below = 0, upto = 0;
    for (unsigned j = 0; j < cnt; ++j) {
      const u64 other = sh.small[j];
      below += other < mine ? 1u : 0u;
      upto += other <= mine ? 1u : 0u;
    }
    const bool hit = lane < (int)cnt && below < remaining && remaining <= upto;     // the lanes that hold the wanted value
    const u64 hits = __ballot(hit);
    if (hits && lane == __ffsll((long long)hits) - 1) {
      sh.prefix = mine;
      sh.remaining = remaining - below;
      sh.bin_count = upto - below;
    }
  }
  __syncthreads();
  value = lo + sh.prefix;
  take = sh.remaining;
  equal = sh.bin_count;
}

// The n_drop-th smallest of the c keys key_at(i) and the tie rule: pixels (index index_at(i)) whose key equals it are
// dropped in ascending index.  Returns the key and the largest index that is still dropped among the equal ones
// (kNoIndex when all of them are dropped).  One workgroup; every thread receives the result.
template <class KeyAt, class IndexAt>
__device__ void block_threshold(SelShared& sh, KeyAt key_at, IndexAt index_at, int c, unsigned n_drop, u64& threshold,
                                unsigned& last_index) {
  unsigned take, equal;
  block_select(sh, [&](int i, u64& v) { v = key_at(i); return true; }, c, n_drop, threshold, take, equal);
  last_index = kNoIndex;
  if (take == equal) return;
  u64 idx;
  unsigned t2, e2;
  const u64 th = threshold;
  block_select(sh, [&](int i, u64& v) { v = index_at(i); return key_at(i) == th; }, c, take, idx, t2, e2);
  last_index = (unsigned)idx;
}

__device__ __forceinline__ uint8_t keep_byte(u64 k, unsigned i, u64 threshold, unsigned last_index) {
  return (k < threshold || (k == threshold && i <= last_index)) ? 0 : 1;
}

// Maps of at most kLdsKeys pixels: one workgroup, the keys in LDS (dynamic: n * 8 bytes).
__global__ __launch_bounds__(kSelThreads) void mask_select_lds_kernel(const u64* __restrict__ keys, int n, int n_drop,
                                                                      uint8_t* __restrict__ mask) {
  extern __shared__ __align__(16) u64 s_keys[];
  __shared__ SelShared sh;
  const int t = threadIdx.x;
  if (n_drop <= 0 || n_drop >= n) {          // nothing or everything is dropped: no ranking needed
    const uint8_t v = n_drop <= 0 ? 1 : 0;
    for (int i = t; i < n; i += kSelThreads) mask[i] = v;
    return;
  }
  for (int i = t; i < n; i += kSelThreads) s_keys[i] = keys[i];
  __syncthreads();
  u64 threshold;
  unsigned last_index;
  block_threshold(sh, [&](int i) { return s_keys[i]; }, [&](int i) { return (u64)i; }, n, (unsigned)n_drop, threshold,
                  last_index);
  for (int i = t; i < n; i += kSelThreads) mask[i] = keep_byte(s_keys[i], (unsigned)i, threshold, last_index);
}

// ---- large maps -----------------------------------------------------------------------------------------------

// smallest and largest key of the map from what the pooling workgroups left (every thread receives them)
__device__ __forceinline__ void map_extremes(const SelState* st, int slots, u64* part, u64& lo, u64& hi) {
  lo = ~0ull;
  hi = 0ull;
  for (int s = threadIdx.x; s < slots; s += kSelThreads) {
    const u64 a = st->slot_lo[s], b = st->slot_hi[s];
    lo = a < lo ? a : lo;
    hi = b > hi ? b : hi;
  }
  block_min_max<kSelWaves>(lo, hi, part);
}

__global__ __launch_bounds__(kSelThreads) void mask_hist_kernel(const u64* __restrict__ keys, int n, int slots,
                                                                SelState* st) {
  __shared__ unsigned hist[kHistBins];
  __shared__ u64 part[2 * kSelWaves];
  const int t = threadIdx.x;
  u64 lo, hi;
  map_extremes(st, slots, part, lo, hi);
  const int low = bit_length(hi - lo);
  if (low == 0) return;                      // every key is the same: nothing to count
  const int shift = low > kHistBits ? low - kHistBits : 0;
  for (int b = t; b < kHistBins; b += kSelThreads) hist[b] = 0;
  __syncthreads();
  const int i0 = blockIdx.x * kChunk;
  u64 k[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int i = i0 + u * kSelThreads + t;
    k[u] = i < n ? keys[i] : 0ull;
  }
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (i0 + u * kSelThreads + t < n) atomicAdd(&hist[(unsigned)((k[u] - lo) >> shift)], 1u);
  __syncthreads();
  for (int b = t; b < kHistBins; b += kSelThreads)
    if (hist[b]) atomicAdd(&st->hist[b], hist[b]);
}

__global__ __launch_bounds__(kSelThreads) void mask_gather_kernel(const u64* __restrict__ keys, int n, int n_drop, int slots,
                                                                  SelState* st) {
  extern __shared__ __align__(16) unsigned char s_dyn[];      // the last workgroup: candidate keys, then their indices
  __shared__ SelShared sh;
  __shared__ unsigned s_scan[kSelWaves];
  __shared__ unsigned s_bin, s_before, s_count, s_base, s_last;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  u64 lo, hi;
  map_extremes(st, slots, sh.part, lo, hi);
  const int low = bit_length(hi - lo);
  const int shift = low > kHistBits ? low - kHistBits : 0;

  // the bin that holds the wanted key: thread t owns bins 4t .. 4t+3
  unsigned bin = 0, before_bin = 0, in_bin = (unsigned)n;
  if (low > 0) {
    unsigned h[4], sum = 0;
#pragma unroll
    for (int b = 0; b < 4; ++b) { h[b] = st->hist[t * 4 + b]; sum += h[b]; }
    unsigned incl = sum;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const unsigned up = __shfl_up(incl, d, 64);
      if (lane >= d) incl += up;
    }
    if (lane == 63) s_scan[wave] = incl;
    __syncthreads();
    unsigned before = incl - sum;
    for (int w = 0; w < wave; ++w) before += s_scan[w];
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      if (before < (unsigned)n_drop && (unsigned)n_drop <= before + h[b]) {
        s_bin = (unsigned)(t * 4 + b);
        s_before = before;
        s_count = h[b];
      }
      before += h[b];
    }
    __syncthreads();
    bin = s_bin;
    before_bin = s_before;
    in_bin = s_count;
  }
  const bool listed = low > 0 && in_bin <= (unsigned)kCandCap;

  if (listed) {        // this workgroup's keys of that bin join the list (in any order: indices travel with them)
    const int i0 = blockIdx.x * kChunk;
    u64 k[4];
    bool hit[4];
    unsigned mine = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = i0 + u * kSelThreads + t;
      k[u] = i < n ? keys[i] : 0ull;
      hit[u] = i < n && (unsigned)((k[u] - lo) >> shift) == bin;
      mine += hit[u] ? 1u : 0u;
    }
    unsigned incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const unsigned up = __shfl_up(incl, d, 64);
      if (lane >= d) incl += up;
    }
    __syncthreads();
    if (lane == 63) s_scan[wave] = incl;
    __syncthreads();
    unsigned at = incl - mine, total = 0;
    for (int w = 0; w < kSelWaves; ++w) {
      at += w < wave ? s_scan[w] : 0u;
      total += s_scan[w];
    }
    if (t == 0) s_base = total ? atomicAdd(&st->cand_n, total) : 0u;
    __syncthreads();
    at += s_base;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (hit[u]) {     // device-scope stores: the workgroup that reads them may run on another die
        __hip_atomic_store(&st->cand_key[at], k[u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&st->cand_idx[at], (unsigned)(i0 + u * kSelThreads + t), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ++at;
      }
    }
  }
  // arrival: the workgroup that finds every other one arrived finishes the selection
  __threadfence();
  __syncthreads();
  if (t == 0) s_last = __hip_atomic_fetch_add(&st->arrived, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT) == gridDim.x - 1 ? 1u : 0u;
  __syncthreads();
  if (!s_last) return;
  __threadfence();

  u64 threshold;
  unsigned last_index;
  if (low == 0) {                    // every key equal: the first n_drop pixels go
    threshold = lo;
    last_index = (unsigned)n_drop - 1u;
  } else if (listed) {
    u64* c_key = reinterpret_cast<u64*>(s_dyn);
    unsigned* c_idx = reinterpret_cast<unsigned*>(s_dyn + (size_t)kCandCap * sizeof(u64));
    const int c = (int)in_bin;
    for (int j = t; j < c; j += kSelThreads) {
      c_key[j] = __hip_atomic_load(&st->cand_key[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      c_idx[j] = __hip_atomic_load(&st->cand_idx[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    block_threshold(sh, [&](int j) { return c_key[j]; }, [&](int j) { return (u64)c_idx[j]; }, c,
                    (unsigned)n_drop - before_bin, threshold, last_index);
  } else {
    // more keys share the bin than the list holds (few distinct scores): this workgroup selects among all keys
    // of the map straight from memory -- slow, and only for such maps
    block_threshold(sh, [&](int i) { return keys[i]; }, [&](int i) { return (u64)i; }, n, (unsigned)n_drop, threshold,
                    last_index);
  }
  if (t == 0) {
    st->threshold = threshold;
    st->last_index = last_index;
  }
}

__global__ __launch_bounds__(256) void mask_write_kernel(const u64* __restrict__ keys, int n, const SelState* st,
                                                         uint8_t* __restrict__ mask) {
  const u64 threshold = st->threshold;
  const unsigned last_index = st->last_index;
  for (int i = blockIdx.x * 256 + threadIdx.x; i < n; i += gridDim.x * 256)
    mask[i] = keep_byte(keys[i], (unsigned)i, threshold, last_index);
}

__global__ __launch_bounds__(256) void mask_fill_kernel(uint8_t* __restrict__ mask, int n, uint8_t v) {
  for (int i = blockIdx.x * 256 + threadIdx.x; i < n; i += gridDim.x * 256) mask[i] = v;
}

static inline int64_t kept_of(double sparsity, int64_t n) {
  return (int64_t)std::floor((1.0 - sparsity) * (double)n + 0.5);
}

static inline size_t key_bytes(int64_t n) { return ((size_t)n * sizeof(u64) + 255) / 256 * 256; }

static sc_status check_mask_args(int32_t in_h, int32_t in_w, int32_t ho, int32_t wo, float sparsity) {
  if (in_h < 1 || in_w < 1 || ho < 1 || wo < 1 || ho > in_h || wo > in_w) return SC_ERR_BAD_SHAPE;
  if ((int64_t)in_h * in_w > (1 << 26)) return SC_ERR_BAD_SHAPE;
  if (!(sparsity >= 0.0f && sparsity <= 1.0f)) return SC_ERR_BAD_SHAPE;   // also rejects NaN
  return SC_OK;
}

constexpr int kMostDevices = 64;

// The two kernels with more than 64 KiB of dynamic LDS need their limit raised, once per device.
static sc_status lds_limits() {
  static std::mutex lock;
  static bool done[kMostDevices];
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { note_hip_error((int32_t)e); return SC_ERR_HIP; }
  if (dev < 0 || dev >= kMostDevices) return SC_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> hold(lock);
  if (done[dev]) return SC_OK;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(mask_select_lds_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                          kLdsKeys * (int)sizeof(u64));
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(mask_gather_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            kCandCap * (int)(sizeof(u64) + sizeof(unsigned)));
  if (e != hipSuccess) { note_hip_error((int32_t)e); return SC_ERR_HIP; }
  done[dev] = true;
  return SC_OK;
}

// The launches of one mask.  `scratch` is device memory of key_bytes(n) + sizeof(SelState) bytes: ho * wo keys, every one
// of which the pooling kernel writes before a later kernel reads it, then the state of the large-map selection, which
// the pooling kernel clears (nothing has to be cleared between calls).
static sc_status launch_mask(const float* score_dev, int32_t in_h, int32_t in_w, int32_t ho, int32_t wo, float sparsity,
                             uint8_t* mask_dev, void* scratch, hipStream_t stream) {
  const int n = ho * wo;
  const int n_drop = n - (int)kept_of((double)sparsity, n);
  if (n_drop <= 0 || n_drop >= n) {          // nothing or everything is dropped: no ranking needed
    hipLaunchKernelGGL(mask_fill_kernel, dim3((unsigned)std::min((n + 255) / 256, 1024)), dim3(256), 0, stream, mask_dev, n,
                       (uint8_t)(n_drop <= 0 ? 1 : 0));
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { note_hip_error((int32_t)e); return SC_ERR_HIP; }
    return SC_OK;
  }
  sc_status s = lds_limits();
  if (s != SC_OK) return s;
  u64* keys = static_cast<u64*>(scratch);
  const bool large = n > kLdsKeys;
  SelState* st = large ? reinterpret_cast<SelState*>(static_cast<unsigned char*>(scratch) + key_bytes(n)) : nullptr;
  const int rh = in_h / ho, rw = in_w / wo;
  int slots;
  if ((int64_t)rh * rw >= 64) {
    slots = std::min((n + 3) / 4, kSlots);
    hipLaunchKernelGGL(score_key_wave_kernel, dim3((unsigned)slots), dim3(kKeyThreads), 0, stream, score_dev, in_w, rh, rw,
                       ho, wo, keys, st);
  } else {
    slots = std::min((n + kKeyThreads - 1) / kKeyThreads, kSlots);
    hipLaunchKernelGGL(score_key_kernel, dim3((unsigned)slots), dim3(kKeyThreads), 0, stream, score_dev, in_w, rh, rw, ho,
                       wo, keys, st);
  }
  if (!large) {
    hipLaunchKernelGGL(mask_select_lds_kernel, dim3(1), dim3(kSelThreads), (size_t)n * sizeof(u64), stream,
                       (const u64*)keys, n, n_drop, mask_dev);
  } else {
    const unsigned chunks = (unsigned)((n + kChunk - 1) / kChunk);
    hipLaunchKernelGGL(mask_hist_kernel, dim3(chunks), dim3(kSelThreads), 0, stream, (const u64*)keys, n, slots, st);
    hipLaunchKernelGGL(mask_gather_kernel, dim3(chunks), dim3(kSelThreads), (size_t)kCandCap * (sizeof(u64) + sizeof(unsigned)),
                       stream, (const u64*)keys, n, n_drop, slots, st);
    hipLaunchKernelGGL(mask_write_kernel, dim3((unsigned)std::min((n + 255) / 256, 4096)), dim3(256), 0, stream,
                       (const u64*)keys, n, (const SelState*)st, mask_dev);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { note_hip_error((int32_t)e); return SC_ERR_HIP; }
  return SC_OK;
}

// Scratch of the entry point that allocates nothing: one array per GPU inside the library's code object, held
// until the process ends.  On the host the array's name is only a handle; the device address comes from
// hipGetSymbolAddress, asked once per device with that device current, and is what the kernels receive.
constexpr int kStaticMaskPixels = SC_STATIC_MASK_PIXELS;      // 512 x 512 layer pixels: 2 MiB of keys
constexpr size_t kStaticWords = (size_t)kStaticMaskPixels + (sizeof(SelState) + sizeof(u64) - 1) / sizeof(u64);
static __device__ __align__(256) u64 scratch[kStaticWords];
static u64* g_scratch_ptr[kMostDevices];   // per device, null until asked
static std::mutex g_scratch_lock;

static sc_status static_scratch(u64** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { note_hip_error((int32_t)e); return SC_ERR_HIP; }
  if (dev < 0 || dev >= kMostDevices) return SC_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> hold(g_scratch_lock);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) { note_hip_error((int32_t)e); return SC_ERR_HIP; }
    g_scratch_ptr[dev] = static_cast<u64*>(ptr);
  }
  *out = g_scratch_ptr[dev];
  return SC_OK;
}

}  // namespace sc

extern "C" {

sc_status sparse_mask_workspace_bytes(int32_t ho, int32_t wo, size_t* bytes) {
  if (!bytes) return SC_ERR_NULL;
  *bytes = 0;
  if (ho < 1 || wo < 1 || (int64_t)ho * wo > (1 << 26)) return SC_ERR_BAD_SHAPE;
  *bytes = sc::key_bytes((int64_t)ho * wo) + sizeof(sc::SelState);
  return SC_OK;
}

sc_status sparse_mask_generate(const float* score_dev, int32_t in_h, int32_t in_w, int32_t ho, int32_t wo,
                               float sparsity, uint8_t* mask_dev, void* workspace_dev, size_t workspace_bytes,
                               void* hip_stream) {
  if (!score_dev || !mask_dev || !workspace_dev) return SC_ERR_NULL;
  sc_status s = sc::check_mask_args(in_h, in_w, ho, wo, sparsity);
  if (s != SC_OK) return s;
  size_t need = 0;
  s = sparse_mask_workspace_bytes(ho, wo, &need);
  if (s != SC_OK) return s;
  if (workspace_bytes < need) return SC_ERR_WORKSPACE;
  if ((uintptr_t)workspace_dev & 7) return SC_ERR_ALIGN;
  return sc::launch_mask(score_dev, in_h, in_w, ho, wo, sparsity, mask_dev, workspace_dev,
                         static_cast<hipStream_t>(hip_stream));
}

sc_status sparse_mask_generate_static(const float* score_dev, int32_t in_h, int32_t in_w, int32_t ho, int32_t wo,
                                      float sparsity, uint8_t* mask_dev, void* hip_stream) {
  if (!score_dev || !mask_dev) return SC_ERR_NULL;
  sc_status s = sc::check_mask_args(in_h, in_w, ho, wo, sparsity);
  if (s != SC_OK) return s;
  if ((int64_t)ho * wo > sc::kStaticMaskPixels) return SC_ERR_WORKSPACE;   // the fixed scratch array is too small
  sc::u64* keys = nullptr;
  s = sc::static_scratch(&keys);
  if (s != SC_OK) return s;
  return sc::launch_mask(score_dev, in_h, in_w, ho, wo, sparsity, mask_dev, keys, static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
