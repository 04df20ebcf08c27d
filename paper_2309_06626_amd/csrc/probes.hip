// Measurement probes: what this GPU sustains on the two roofs the convolution kernels are priced against, measured with
// the simplest kernels that can reach them.  They are not part of the method; bench.py and the layer report quote
// their figures beside the nominal peaks.
//   sc_probe_stream_copy   a plain copy, 16 bytes per lane and access, one contiguous chunk per workgroup: HBM read + write bandwidth
//   sc_probe_mfma_bf16     a loop of independent 32x32x16 bf16 MFMAs on register operands: the matrix pipes alone
#include "../../include/sparse_conv.h"

#include <hip/hip_runtime.h>

#include "mma_common.hpp"

namespace sc {

void note_hip_error(int32_t code);

// every workgroup owns one contiguous chunk; four independent 16-byte loads in flight per lane; streaming
// (non-temporal) loads and stores: measured best of the plain shapes tried (6.3-6.4 TB/s for 512 MiB on MI355X against
// 4.3-5.0 TB/s for a grid-stride loop with cached accesses and 4.8 TB/s for the runtime's device-to-device copy)
__global__ __launch_bounds__(256) void stream_copy_kernel(const v4i* __restrict__ src, v4i* __restrict__ dst, size_t n16) {
  const size_t per = (n16 + gridDim.x - 1) / gridDim.x;
  const size_t lo = per * blockIdx.x, hi = lo + per < n16 ? lo + per : n16;
  for (size_t i = lo + threadIdx.x; i < hi; i += 256 * 4) {
    v4i v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (i + u * 256 < hi) v[u] = __builtin_nontemporal_load(src + i + u * 256);
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (i + u * 256 < hi) __builtin_nontemporal_store(v[u], dst + i + u * 256);
  }
}

constexpr int kProbeChains = 4;      // independent accumulators per wavefront: back-to-back issue without dependency stalls

__global__ __launch_bounds__(256) void mfma_loop_kernel(int iterations, float* __restrict__ out) {
  floatx16 acc[kProbeChains];
#pragma unroll
  for (int c = 0; c < kProbeChains; ++c)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[c][v] = 0.0f;
  // operands from the lane number: small values, nothing overflows in `iterations` additions
  v4i a, b;
  const int t = threadIdx.x;
  a = v4i{0x3c003c00 + (t & 3), 0x38003800, 0x3c003c00, 0x38003800};
  b = v4i{0x38003800, 0x3c003c00 + (t & 1), 0x38003800, 0x3c003c00};
  for (int i = 0; i < iterations; ++i) {
#pragma unroll
    for (int c = 0; c < kProbeChains; ++c) Elem<kBF16>::mma(acc[c], a, b);
  }
  float s = 0.0f;
#pragma unroll
  for (int c = 0; c < kProbeChains; ++c)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += acc[c][v];
  out[(size_t)blockIdx.x * 256 + t] = s;
}

}  // namespace sc

extern "C" {

sc_status sc_probe_stream_copy(void* dst_dev, const void* src_dev, size_t bytes, void* hip_stream) {
  if (!dst_dev || !src_dev) return SC_ERR_NULL;
  if (((uintptr_t)dst_dev | (uintptr_t)src_dev) & 15) return SC_ERR_ALIGN;
  if (bytes % 16 != 0) return SC_ERR_BAD_SHAPE;
  if (bytes == 0) return SC_OK;
  const size_t n16 = bytes / 16;
  const unsigned grid = (unsigned)std::max<size_t>(1, std::min<size_t>(n16 / 2048, 16384));   // chunks of 32 KiB and more
  hipLaunchKernelGGL(sc::stream_copy_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                     static_cast<const sc::v4i*>(src_dev), static_cast<sc::v4i*>(dst_dev), n16);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { sc::note_hip_error((int32_t)e); return SC_ERR_HIP; }
  return SC_OK;
}

sc_status sc_probe_mfma_bf16(int32_t iterations, int32_t workgroups, float* out_dev, double* flops, void* hip_stream) {
  if (!out_dev) return SC_ERR_NULL;
  if (iterations < 1 || workgroups < 1 || workgroups > (1 << 20)) return SC_ERR_BAD_SHAPE;
  hipLaunchKernelGGL(sc::mfma_loop_kernel, dim3((unsigned)workgroups), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                     iterations, out_dev);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { sc::note_hip_error((int32_t)e); return SC_ERR_HIP; }
  // 4 wavefronts per workgroup, kProbeChains MFMAs of 32 x 32 x 16 x 2 FLOP per iteration and wavefront
  if (flops) *flops = (double)workgroups * 4.0 * sc::kProbeChains * iterations * 32.0 * 32.0 * 16.0 * 2.0;
  return SC_OK;
}

}  // extern "C"
