// Mask generator of the sparse-training pipeline (Alg. 1, function getMask; described in Sec. 3.1):
// a 2-D score at the resolution of the network input is pooled down to the resolution of a layer,
// the layer's pixels are ranked by the pooled score and the lowest-ranked ones are dropped.
//
// Two launches per layer, nothing else on the stream:
//   score_key_kernel   one lane per layer pixel (one wavefront per pixel for windows of 64 values and
//                      more): sum of the pooling window in double, in row-major order of the window,
//                      turned into a 64-bit key whose unsigned order is the order of the sums
//   mask_select_kernel one workgroup: radix selection (8 bits per pass, starting at the first bit in
//                      which the keys differ) of the n_drop-th smallest key, then one sweep that
//                      writes the mask; pixels whose key equals the selected one are dropped in
//                      ascending pixel index until the count is exact
#include "../../include/sparse_conv.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <mutex>

namespace sc {

void note_hip_error(int32_t code);   // defined with the other host code of the library

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelUnroll = 8;        // independent key loads a lane keeps in flight during a sweep
constexpr int kSelListCap = 4096;    // candidate keys kept in LDS once a radix bin is this small

// unsigned order of the result == numeric order of the doubles (-0.0 sorts directly below +0.0; a
// sum that starts from +0.0 never is -0.0)
__device__ __forceinline__ unsigned long long order_key(double v) {
  const unsigned long long b = (unsigned long long)__double_as_longlong(v);
  return (b >> 63) ? ~b : (b | 0x8000000000000000ull);
}

__global__ __launch_bounds__(256) void score_key_kernel(const float* __restrict__ score, int in_w, int rh, int rw,
                                                        int ho, int wo, unsigned long long* __restrict__ keys) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= ho * wo) return;
  const int oy = i / wo, ox = i - oy * wo;
  const float* win = score + (size_t)oy * rh * in_w + (size_t)ox * rw;
  double acc = 0.0;
  for (int dy = 0; dy < rh; ++dy)
    for (int dx = 0; dx < rw; ++dx) acc = acc + (double)win[(size_t)dy * in_w + dx];
  keys[i] = order_key(acc);
}

// Large pooling windows: one wavefront per layer pixel.  The 64 lanes fetch the window in pieces of
// kPoolPiece values into LDS (neighbouring lanes read neighbouring values of a window row), then lane 0
// adds the piece up in window order -- the order of the sum is the same as in the kernel above.
constexpr int kPoolPiece = 2048;
__global__ __launch_bounds__(256) void score_key_wave_kernel(const float* __restrict__ score, int in_w, int rh,
                                                             int rw, int ho, int wo,
                                                             unsigned long long* __restrict__ keys) {
  __shared__ float s_piece[4][kPoolPiece];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i = blockIdx.x * 4 + wave;
  const bool live = i < ho * wo;
  const int oy = live ? i / wo : 0, ox = live ? i - oy * wo : 0;
  const float* win = score + (size_t)oy * rh * in_w + (size_t)ox * rw;
  const int count = rh * rw;        // < 2^26: the score itself is that small
  double acc = 0.0;
  for (int e0 = 0; e0 < count; e0 += kPoolPiece) {
    const int len = min(kPoolPiece, count - e0);
    for (int e = lane; e < len; e += 64) {
      const int dy = (e0 + e) / rw, dx = (e0 + e) - dy * rw;
      s_piece[wave][e] = win[(size_t)dy * in_w + dx];
    }
    __syncthreads();
    if (lane == 0)
      for (int e = 0; e < len; ++e) acc = acc + (double)s_piece[wave][e];
    __syncthreads();
  }
  if (live && lane == 0) keys[i] = order_key(acc);
}

__device__ __forceinline__ unsigned long long high_bits(unsigned long long k, int low) {
  return low >= 64 ? 0ull : k >> low;
}

__global__ __launch_bounds__(kSelThreads) void mask_select_kernel(const unsigned long long* __restrict__ keys, int n,
                                                                  int n_drop, uint8_t* __restrict__ mask) {
  __shared__ unsigned hist[256];
  __shared__ unsigned long long s_list[kSelListCap];
  __shared__ unsigned long long s_lo[kSelWaves], s_hi[kSelWaves];
  __shared__ unsigned long long s_prefix;
  __shared__ unsigned s_remaining, s_bin_count, s_list_n;
  __shared__ unsigned wave_cnt[kSelWaves];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;

  if (n_drop <= 0 || n_drop >= n) {          // nothing or everything is dropped: no ranking needed
    const uint8_t v = n_drop <= 0 ? 1 : 0;
    for (int i = t; i < n; i += kSelThreads) mask[i] = v;
    return;
  }

  // smallest and largest key: the leading bits they share are the leading bits of every key, and the
  // digit passes start at the first bit in which keys differ (scores of one map lie close together;
  // without this the first passes would put every key into one bin)
  unsigned long long lo = ~0ull, hi = 0ull;
  for (int i0 = 0; i0 < n; i0 += kSelUnroll * kSelThreads) {
    unsigned long long k[kSelUnroll];
#pragma unroll
    for (int u = 0; u < kSelUnroll; ++u) {
      const int i = i0 + u * kSelThreads + t;
      k[u] = keys[i < n ? i : 0];          // an index past the end re-reads key 0, which changes neither extreme
    }
#pragma unroll
    for (int u = 0; u < kSelUnroll; ++u) {
      lo = k[u] < lo ? k[u] : lo;
      hi = k[u] > hi ? k[u] : hi;
    }
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    const unsigned long long ol = __shfl_xor(lo, d, 64), oh = __shfl_xor(hi, d, 64);
    lo = ol < lo ? ol : lo;
    hi = oh > hi ? oh : hi;
  }
  if (lane == 0) { s_lo[wave] = lo; s_hi[wave] = hi; }
  if (t == 0) s_list_n = 0;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) {
    lo = s_lo[w] < lo ? s_lo[w] : lo;
    hi = s_hi[w] > hi ? s_hi[w] : hi;
  }
  int low = lo == hi ? 0 : 64 - __clzll((long long)(lo ^ hi));   // bits [0, low) are still unknown
  unsigned long long prefix = low >= 64 ? 0ull : (lo >> low) << low;   // the known bits of the wanted key
  unsigned remaining = n_drop;     // 1-based rank of the wanted key among the keys that share the known bits
  unsigned bin_count = n;          // how many keys share the known bits
  bool listed = false;             // those keys sit in s_list
  while (low > 0) {
    const int width = low < 8 ? low : 8;
    const int shift = low - width;
    const unsigned dmask = (1u << width) - 1u;
    const unsigned long long want_high = high_bits(prefix, low);
    if (t < 256) hist[t] = 0;
    __syncthreads();
    if (listed) {
      const int ln = (int)s_list_n;
      for (int i = t; i < ln; i += kSelThreads) {
        const unsigned long long k = s_list[i];
        if (high_bits(k, low) == want_high) atomicAdd(&hist[(unsigned)(k >> shift) & dmask], 1u);
      }
    } else {
      // sweep over all keys; when the bin chosen by the previous pass is small enough its keys are
      // copied into LDS on the way and the later passes never touch global memory again
      const bool gather = bin_count <= (unsigned)kSelListCap;
      for (int i0 = 0; i0 < n; i0 += kSelUnroll * kSelThreads) {
        unsigned long long k[kSelUnroll];
#pragma unroll
        for (int u = 0; u < kSelUnroll; ++u) {
          const int i = i0 + u * kSelThreads + t;
          k[u] = i < n ? keys[i] : 0ull;
        }
#pragma unroll
        for (int u = 0; u < kSelUnroll; ++u) {
          const int i = i0 + u * kSelThreads + t;
          if (i < n && high_bits(k[u], low) == want_high) {
            atomicAdd(&hist[(unsigned)(k[u] >> shift) & dmask], 1u);
            if (gather) s_list[atomicAdd(&s_list_n, 1u)] = k[u];
          }
        }
      }
      listed = gather;
    }
    __syncthreads();
    if (wave == 0) {   // lane l owns bins 4l .. 4l+3: running count over the 256 bins
      unsigned h[4], sum = 0;
#pragma unroll
      for (int b = 0; b < 4; ++b) { h[b] = hist[lane * 4 + b]; sum += h[b]; }
      unsigned incl = sum;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const unsigned up = __shfl_up(incl, d, 64);
        if (lane >= d) incl += up;
      }
      unsigned c = incl - sum;
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        if (c < remaining && remaining <= c + h[b]) {      // true for exactly one bin of one lane
          s_prefix = prefix | ((unsigned long long)(lane * 4 + b) << shift);
          s_remaining = remaining - c;
          s_bin_count = h[b];
        }
        c += h[b];
      }
    }
    __syncthreads();
    prefix = s_prefix;
    remaining = s_remaining;
    bin_count = s_bin_count;
    low = shift;
  }

  // prefix is the n_drop-th smallest key; bin_count pixels have exactly that key and `remaining` of
  // them are dropped, the ones with the lowest indices.
  if (bin_count == remaining) {      // no tie at the threshold (the usual case): every pixel decides alone
    for (int i0 = 0; i0 < n; i0 += kSelUnroll * kSelThreads) {
      unsigned long long k[kSelUnroll];
#pragma unroll
      for (int u = 0; u < kSelUnroll; ++u) {
        const int i = i0 + u * kSelThreads + t;
        k[u] = i < n ? keys[i] : 0ull;
      }
#pragma unroll
      for (int u = 0; u < kSelUnroll; ++u) {
        const int i = i0 + u * kSelThreads + t;
        if (i < n) mask[i] = k[u] <= prefix ? 0 : 1;
      }
    }
    return;
  }
  // ties at the threshold: sweep in index order with a running count of the equal keys
  unsigned base = 0;
  for (int i0 = 0; i0 < n; i0 += kSelThreads) {
    const int i = i0 + t;
    const unsigned long long k = i < n ? keys[i] : 0ull;
    const bool eq = i < n && k == prefix;
    const unsigned long long bal = __ballot(eq);
    if (lane == 0) wave_cnt[wave] = (unsigned)__popcll(bal);
    __syncthreads();
    unsigned earlier = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
      const unsigned c = wave_cnt[w];
      earlier += w < wave ? c : 0u;
      total += c;
    }
    const unsigned rank = base + earlier + (unsigned)__popcll(bal & ((1ull << lane) - 1ull));
    if (i < n) mask[i] = (k < prefix || (eq && rank < remaining)) ? 0 : 1;
    base += total;
    __syncthreads();
  }
}

static inline int64_t kept_of(double sparsity, int64_t n) {
  return (int64_t)std::floor((1.0 - sparsity) * (double)n + 0.5);
}

static sc_status check_mask_args(int32_t in_h, int32_t in_w, int32_t ho, int32_t wo, float sparsity) {
  if (in_h < 1 || in_w < 1 || ho < 1 || wo < 1 || ho > in_h || wo > in_w) return SC_ERR_BAD_SHAPE;
  if ((int64_t)in_h * in_w > (1 << 26)) return SC_ERR_BAD_SHAPE;
  if (!(sparsity >= 0.0f && sparsity <= 1.0f)) return SC_ERR_BAD_SHAPE;   // also rejects NaN
  return SC_OK;
}

// The two launches of one mask; `keys` is device scratch of ho * wo 64-bit words, every one of which the first
// kernel writes before the second reads it (nothing has to be cleared between calls).
static sc_status launch_mask(const float* score_dev, int32_t in_h, int32_t in_w, int32_t ho, int32_t wo, float sparsity,
                             uint8_t* mask_dev, unsigned long long* keys, hipStream_t stream) {
  const int n = ho * wo;
  const int n_drop = n - (int)kept_of((double)sparsity, n);
  const int rh = in_h / ho, rw = in_w / wo;
  if ((int64_t)rh * rw >= 64)
    hipLaunchKernelGGL(score_key_wave_kernel, dim3((unsigned)((n + 3) / 4)), dim3(256), 0, stream, score_dev, in_w,
                       rh, rw, ho, wo, keys);
  else
    hipLaunchKernelGGL(score_key_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, score_dev, in_w,
                       rh, rw, ho, wo, keys);
  hipLaunchKernelGGL(mask_select_kernel, dim3(1), dim3(kSelThreads), 0, stream, (const unsigned long long*)keys, n,
                     n_drop, mask_dev);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { note_hip_error((int32_t)e); return SC_ERR_HIP; }
  return SC_OK;
}

// Scratch of the entry point that allocates nothing: one array per GPU inside the library's code object, held
// until the process ends.  On the host the array's name is only a handle; the device address comes from
// hipGetSymbolAddress, asked once per device with that device current, and is what the kernels receive.
constexpr int kStaticMaskPixels = SC_STATIC_MASK_PIXELS;      // 512 x 512 layer pixels: 2 MiB of keys
constexpr int kMostDevices = 64;
static __device__ __align__(256) unsigned long long scratch[kStaticMaskPixels];
static unsigned long long* g_scratch_ptr[kMostDevices];   // per device, null until asked
static std::mutex g_scratch_lock;

static sc_status static_scratch(unsigned long long** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { note_hip_error((int32_t)e); return SC_ERR_HIP; }
  if (dev < 0 || dev >= kMostDevices) return SC_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> hold(g_scratch_lock);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) { note_hip_error((int32_t)e); return SC_ERR_HIP; }
    g_scratch_ptr[dev] = static_cast<unsigned long long*>(ptr);
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
  *bytes = (size_t)ho * wo * sizeof(unsigned long long);
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
  return sc::launch_mask(score_dev, in_h, in_w, ho, wo, sparsity, mask_dev,
                         static_cast<unsigned long long*>(workspace_dev), static_cast<hipStream_t>(hip_stream));
}

sc_status sparse_mask_generate_static(const float* score_dev, int32_t in_h, int32_t in_w, int32_t ho, int32_t wo,
                                      float sparsity, uint8_t* mask_dev, void* hip_stream) {
  if (!score_dev || !mask_dev) return SC_ERR_NULL;
  sc_status s = sc::check_mask_args(in_h, in_w, ho, wo, sparsity);
  if (s != SC_OK) return s;
  if ((int64_t)ho * wo > sc::kStaticMaskPixels) return SC_ERR_WORKSPACE;   // the fixed scratch array is too small
  unsigned long long* keys = nullptr;
  s = sc::static_scratch(&keys);
  if (s != SC_OK) return s;
  return sc::launch_mask(score_dev, in_h, in_w, ho, wo, sparsity, mask_dev, keys, static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
