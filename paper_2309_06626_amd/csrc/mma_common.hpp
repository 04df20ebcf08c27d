// Types, MFMA wrappers and the kept-row store shared by the masked-convolution kernels.
#pragma once
#include "conv_params.hpp"

namespace sc {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

template <int DT> struct Elem;
template <> struct Elem<kBF16> {
  using T = __bf16;
  static constexpr int V = 8;  // elements per 16 bytes
  static __device__ __forceinline__ void mma(floatx16& acc, v4i wf, v4i xf) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wf), __builtin_bit_cast(bf16x8, xf),
                                                  acc, 0, 0, 0);
  }
  static __device__ __forceinline__ T from_float(float f) { return (__bf16)f; }
};
template <> struct Elem<kF16> {
  using T = _Float16;
  static constexpr int V = 8;
  static __device__ __forceinline__ void mma(floatx16& acc, v4i wf, v4i xf) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, wf), __builtin_bit_cast(f16x8, xf),
                                                 acc, 0, 0, 0);
  }
  static __device__ __forceinline__ T from_float(float f) { return (_Float16)f; }
};
template <> struct Elem<kF32> {
  using T = float;
  static constexpr int V = 4;
  // A 16-byte group holds 4 consecutive K entries; the two lane halves hold two different
  // groups, so MFMA number e contracts entry e of both groups (any consistent pairing of K
  // entries between the two operands is a valid order of the sum).
  static __device__ __forceinline__ void mma(floatx16& acc, v4i wf, v4i xf) {
    v4f a = __builtin_bit_cast(v4f, wf), b = __builtin_bit_cast(v4f, xf);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[0], b[0], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[1], b[1], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[2], b[2], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[3], b[3], acc, 0, 0, 0);
  }
  static __device__ __forceinline__ T from_float(float f) { return f; }
};

// Output stores are ordinary cached stores: streaming (non-temporal) stores measured about 5 % faster
// for a layer timed on its own, but slower for a chain of layers, whose next layer then finds its
// input in HBM instead of in the L2 / memory-side cache.
__device__ __forceinline__ void sc_store16(v4i* dst, v4i v) { *dst = v; }

// Bias, ReLU, conversion and store of one 32x32 MFMA block for the lane's output position:
// `acc` holds 16 consecutive output channels c0..c0+15 of dense row rr (Alg. 2, copy branch: the
// result of a kept row goes to its dense slot).  bias[bias_at + v] belongs to channel c0 + v.
// vec_out: 0 = element stores with strides; 1 = 16-byte stores, c_out a multiple of 16 (every block lies inside
// c_out; the only mode the LDS-direct, band and row-panel kernels are launched with, as a literal, so their
// epilogue stays as lean as it was); 2 = 16-byte stores, c_out a multiple of the 16-byte group only (the
// register-staged tiled kernel).
//
// `res` (may be null): a shortcut tensor in the layout of y that is added after the layer's own activation, with
// `post_relu` applied to the sum -- y = post(act(conv + bias) + res), the fused form of a block's conv -> add.
template <int DT>
__device__ __forceinline__ void store_kept_block_res(const floatx16& acc, int rr, int c0, typename Elem<DT>::T* y,
                                                     const float* __restrict__ bias, int bias_at, int relu, int vec_out,
                                                     int c_out, int ho_wo, int64_t ys_n, int ys_p, int ys_c,
                                                     const typename Elem<DT>::T* res, int post_relu) {
  using E = Elem<DT>;
  using T = typename E::T;
  constexpr int EB = sizeof(T);
  float vals[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) vals[v] = acc[v];
  // the shortcut's 16 channels of this row (whole 16-byte groups), added after the layer's activation
  auto add_shortcut = [&](int groups_ok) {
    if (res) {
      constexpr int GC = 16 / EB;
      const v4i* src = reinterpret_cast<const v4i*>(res + ((int64_t)rr * c_out + c0));
#pragma unroll
      for (int q = 0; q < 16 * EB / 16; ++q) {
        if (q < groups_ok) {
          const v4i g = src[q];
          T e[GC];
          __builtin_memcpy(e, &g, 16);
#pragma unroll
          for (int i = 0; i < GC; ++i) vals[q * GC + i] += (float)e[i];
        }
      }
    }
    if (post_relu) {
#pragma unroll
      for (int v = 0; v < 16; ++v) vals[v] = fmaxf(vals[v], 0.0f);
    }
  };
  if (vec_out == 1) {
    // every 16-channel block lies inside c_out (c_out is a multiple of 16): the plain path
    if (bias) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        v4f b4 = *reinterpret_cast<const v4f*>(bias + bias_at + 4 * q);
#pragma unroll
        for (int e = 0; e < 4; ++e) vals[4 * q + e] += b4[e];
      }
    }
    if (relu) {
#pragma unroll
      for (int v = 0; v < 16; ++v) vals[v] = fmaxf(vals[v], 0.0f);
    }
    add_shortcut(16 * EB / 16);
    T outv[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) outv[v] = E::from_float(vals[v]);
    v4i* dst = reinterpret_cast<v4i*>(y + ((int64_t)rr * c_out + c0));
    v4i pk[16 * EB / 16];
    __builtin_memcpy(pk, outv, 16 * EB);
#pragma unroll
    for (int q = 0; q < 16 * EB / 16; ++q) sc_store16(dst + q, pk[q]);
  } else if (vec_out == 2) {
    // c_out is a multiple of the 16-byte group (8 channels of a 16-bit type, 4 floats) but not of 16: in
    // the block that straddles c_out, the groups beyond it are neither loaded (bias) nor stored
    constexpr int GC = 16 / EB;                 // channels per 16-byte group
    const int groups_ok = min(16, c_out - c0) / GC;
    if (bias) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (4 * q < groups_ok * GC) {
          v4f b4 = *reinterpret_cast<const v4f*>(bias + bias_at + 4 * q);
#pragma unroll
          for (int e = 0; e < 4; ++e) vals[4 * q + e] += b4[e];
        }
      }
    }
    if (relu) {
#pragma unroll
      for (int v = 0; v < 16; ++v) vals[v] = fmaxf(vals[v], 0.0f);
    }
    add_shortcut(groups_ok);
    T outv[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) outv[v] = E::from_float(vals[v]);
    v4i* dst = reinterpret_cast<v4i*>(y + ((int64_t)rr * c_out + c0));
    v4i pk[16 * EB / 16];
    __builtin_memcpy(pk, outv, 16 * EB);
#pragma unroll
    for (int q = 0; q < 16 * EB / 16; ++q)
      if (q < groups_ok) sc_store16(dst + q, pk[q]);
  } else {
    const int n = rr / ho_wo, rem = rr - n * ho_wo;
    const int64_t at = n * ys_n + (int64_t)rem * ys_p;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      int c = c0 + v;
      if (c < c_out) {
        float f = vals[v] + (bias ? bias[bias_at + v] : 0.0f);
        if (relu) f = fmaxf(f, 0.0f);
        if (res) f += (float)res[at + (int64_t)c * ys_c];
        if (post_relu) f = fmaxf(f, 0.0f);
        y[at + (int64_t)c * ys_c] = E::from_float(f);
      }
    }
  }
}

// Row code of a tile row in the kernels' row lists: >= 0 the dense row the result goes to, -1 no such row,
// <= -2 a row the mask drops in a run that contracts every row (masked_store): -2 - row.
__device__ __forceinline__ int dropped_row_code(int row) { return -2 - row; }

// the zeros of such a row (Alg. 2, mask == 0 branch) for the lane's 16 channels
template <int DT>
__device__ __forceinline__ void store_zero_block(int rr, int c0, typename Elem<DT>::T* y, int vec_out, int c_out, int ho_wo,
                                                 int64_t ys_n, int ys_p, int ys_c) {
  floatx16 z;
#pragma unroll
  for (int v = 0; v < 16; ++v) z[v] = 0.0f;
  store_kept_block_res<DT>(z, rr, c0, y, nullptr, 0, 0, vec_out, c_out, ho_wo, ys_n, ys_p, ys_c, nullptr, 0);
}

template <int DT>
__device__ __forceinline__ void store_kept_block(const floatx16& acc, int rr, int c0, typename Elem<DT>::T* __restrict__ y,
                                                 const float* __restrict__ bias, int bias_at, int relu, int vec_out,
                                                 int c_out, int ho_wo, int64_t ys_n, int ys_p, int ys_c) {
  store_kept_block_res<DT>(acc, rr, c0, y, bias, bias_at, relu, vec_out, c_out, ho_wo, ys_n, ys_p, ys_c, nullptr, 0);
}

// What a dropped row of a dense-layout output receives in place of its 16-byte group `at` (byte offset into y):
// zeros (Alg. 2, mask == 0 branch), or post(shortcut) when a shortcut tensor is fused into the launch -- the
// convolution contributes +0.0 there, added in float like everywhere else (so -0.0 of the shortcut becomes +0.0).
template <int DT>
__device__ __forceinline__ v4i dropped_row_group(const void* res, int64_t at, int post_relu) {
  using T = typename Elem<DT>::T;
  constexpr int GC = 16 / (int)sizeof(T);
  if (!res) return v4i{0, 0, 0, 0};
  const v4i g = *reinterpret_cast<const v4i*>(static_cast<const unsigned char*>(res) + at);
  T e[GC];
  __builtin_memcpy(e, &g, 16);
#pragma unroll
  for (int i = 0; i < GC; ++i) {
    float f = 0.0f + (float)e[i];
    if (post_relu) f = fmaxf(f, 0.0f);
    e[i] = Elem<DT>::from_float(f);
  }
  v4i out;
  __builtin_memcpy(&out, e, 16);
  return out;
}

}  // namespace sc
