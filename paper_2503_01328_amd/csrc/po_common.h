// Shared device/host helpers of the HIP path (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace po {

typedef __bf16 bf16;

constexpr int kWave = 64;

enum DType : int { kF32 = 0, kBF16 = 1 };

template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16>(bf16 v) { return (float)v; }

template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return (bf16)v; }

// 16-byte vector of T for coalesced global access.
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  float v[4];
};
template <> struct Vec16<bf16> {
  static constexpr int N = 8;
  bf16 v[8];
};

template <typename T> __device__ __forceinline__ Vec16<T> load16(const T* p) {
  Vec16<T> r;
  *reinterpret_cast<uint4*>(&r) = *reinterpret_cast<const uint4*>(p);
  return r;
}
template <typename T> __device__ __forceinline__ void store16(T* p, const Vec16<T>& r) {
  *reinterpret_cast<uint4*>(p) = *reinterpret_cast<const uint4*>(&r);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// GeLU in its tanh form, and its derivative, in terms of r = 1 / (1 + exp(2z)), z = c (u + 0.044715 u^3):
//   tanh(z) = 1 - 2r,  gelu(u) = 0.5 u (1 + tanh z) = u (1 - r),
//   gelu'(u) = 0.5 (1 + tanh z) + 0.5 u (1 - tanh^2 z) z'(u) = (1 - r) (1 + 2 u r z'(u)),  z' = c (1 + 3 * 0.044715 u^2).
// exp(2z) is one exp2 of a cubic in u with the constants folded, the reciprocal is the hardware's (1 ulp): about
// fourteen operations for both values, where a division and two separate tanh cost thirty.  u -> +inf gives
// r = 0 (gelu = u, slope 1), u -> -inf gives r = 1 (gelu = 0, slope 0).
__device__ __forceinline__ float gelu_gate(float u) {  // r(u)
  const float k1 = 2.0f * 0.7978845608028654f * 1.4426950408889634f;  // 2 c log2(e)
  const float k2 = k1 * 0.044715f;
  float e = __builtin_amdgcn_exp2f(u * (k1 + k2 * u * u));
  return __builtin_amdgcn_rcpf(1.0f + e);
}
__device__ __forceinline__ float gelu_f(float u) {
  float r = gelu_gate(u);
  return u - u * r;
}
__device__ __forceinline__ void gelu_and_grad_f(float u, float& g, float& dg) {
  const float c = 0.7978845608028654f;
  float r = gelu_gate(u);
  float keep = 1.0f - r;
  float dz = c + (3.0f * 0.044715f * c) * u * u;
  g = u * keep;
  dg = keep * (1.0f + 2.0f * u * r * dz);
}
__device__ __forceinline__ float gelu_grad_f(float u) {
  float g, dg;
  gelu_and_grad_f(u, g, dg);
  return dg;
}

// Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3", SC'11): a counter-
// based generator, so a dropout mask is a pure function of its position and can be regenerated in the backward
// pass instead of being stored.  Each round multiplies words 0 and 2 by fixed odd constants, swaps the high and
// low halves around while mixing in words 1 and 3 and the round key, and advances the key by Weyl constants.
struct PhiloxWords {
  uint32_t w[4];
};
__device__ __forceinline__ PhiloxWords philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                                     uint32_t k1) {
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    c0 = hi1 ^ c1 ^ k0;
    c1 = lo1;
    c2 = hi0 ^ c3 ^ k1;
    c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  PhiloxWords r;
  r.w[0] = c0;
  r.w[1] = c1;
  r.w[2] = c2;
  r.w[3] = c3;
  return r;
}

// One dropout site: element (row, col) of the [s, h] tensor is kept iff word col % 4 of the block with counter
// (col / 4, row, stream, unit) under key (k0, k1) is >= threshold; kept values are multiplied by scale = 1 / (1 - p).
// stream = 2 * layer + site (site 0: after the attention output projection, 1: after the MLP output projection),
// unit = microbatch index.  scale == 0 means "no dropout here".
struct DropoutSite {
  uint32_t threshold, k0, k1, stream, unit;
  float scale;
};
__device__ __forceinline__ PhiloxWords dropout_words(const DropoutSite& d, int row, int col4) {
  return philox4x32_10((uint32_t)col4, (uint32_t)row, d.stream, d.unit, d.k0, d.k1);
}

// What a GEMM does with its fp32 accumulators (all pointers may be null).
struct Epilogue {
  const void* bias;      // [N] of T
  const void* residual;  // [M, N] of T, leading dimension ldc
  void* out;             // [M, N] of T
  void* gelu_out;        // [M, N] of T: gelu(out) or gelu(gelu_u)
  const void* gelu_u;    // [M, N] of T: out = acc * gelu'(gelu_u)
  float* acc_f32;        // [M, N] fp32: += acc
  int ldc;               // leading dimension of all [M, N] operands above
};

// Applies the epilogue to one accumulator value at (m, n).
template <typename T>
__device__ __forceinline__ void epilogue_store(const Epilogue& e, int m, int n, float acc) {
  size_t idx = (size_t)m * e.ldc + n;
  if (e.acc_f32) {
    e.acc_f32[idx] += acc;
    return;
  }
  if (e.bias) acc += to_f32(static_cast<const T*>(e.bias)[n]);
  if (e.residual) acc += to_f32(static_cast<const T*>(e.residual)[idx]);
  if (e.gelu_u) {
    float u = to_f32(static_cast<const T*>(e.gelu_u)[idx]);
    float g, dg;
    gelu_and_grad_f(u, g, dg);
    if (e.gelu_out) static_cast<T*>(e.gelu_out)[idx] = from_f32<T>(g);
    acc *= dg;
    static_cast<T*>(e.out)[idx] = from_f32<T>(acc);
    return;
  }
  T o = from_f32<T>(acc);
  if (e.out) static_cast<T*>(e.out)[idx] = o;
  if (e.gelu_out) static_cast<T*>(e.gelu_out)[idx] = from_f32<T>(gelu_f(to_f32(o)));
}

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }

}  // namespace po
