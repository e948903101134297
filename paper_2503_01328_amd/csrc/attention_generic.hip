// Causal attention on the vector ALU for any dtype, sequence length and head
// size up to 256: the fp32 debug path and the home of shapes the MFMA kernels
// do not take.  One wave owns one (head, row): lanes split the keys of a
// 64-wide chunk for the scores (online softmax, running max and sum), then
// split the head dimension for the weighted sums, the per-key weights being
// broadcast with shuffles.  Backward is split into a dQ kernel (wave per query
// row) and a dK/dV kernel (wave per key row), each summing in a fixed order, so
// there are no atomics and results are reproducible.
//
// Grouped-query attention: the qkv matrix is [s, h + 2 hkv] (query block, key block, value block) with
// hkv = n_kv_heads * dh; query head t reads key/value head t / group, group = n_heads / n_kv_heads.  The dK/dV
// kernel runs per key/value head and walks its group's query heads in order.
#include <math.h>

#include "kernels.h"

namespace po {

constexpr int kMaxHeadDim = 256;
constexpr int kDimSlots = kMaxHeadDim / kWave;  // head-dim elements per lane

template <typename T>
__global__ __launch_bounds__(256) void attn_fwd_generic_kernel(const T* __restrict__ qkv, T* __restrict__ o,
                                                               float* __restrict__ lse, int s, int h, int dh,
                                                               int hkv, int group, float scale) {
  __shared__ float qs[4][kMaxHeadDim];
  int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int head = blockIdx.y;
  int i = blockIdx.x * 4 + wave;
  bool active = i < s;
  int ld = h + 2 * hkv;
  const T* kbase = qkv + h + (head / group) * dh;
  const T* vbase = qkv + h + hkv + (head / group) * dh;
  if (active)
    for (int e = lane; e < dh; e += kWave) qs[wave][e] = to_f32(qkv[(size_t)i * ld + head * dh + e]) * scale;
  __syncthreads();
  if (!active) return;
  float m = -INFINITY, l = 0.f;
  float acc[kDimSlots];
#pragma unroll
  for (int r = 0; r < kDimSlots; ++r) acc[r] = 0.f;
  for (int j0 = 0; j0 <= i; j0 += kWave) {
    int j = j0 + lane;
    float sc = -INFINITY;
    if (j <= i) {
      const T* kr = kbase + (size_t)j * ld;
      float d = 0.f;
      for (int e = 0; e < dh; ++e) d = fmaf(qs[wave][e], to_f32(kr[e]), d);
      sc = d;
    }
    float mnew = fmaxf(m, wave_max(sc));
    float p = (j <= i) ? __expf(sc - mnew) : 0.f;
    float alpha = __expf(m - mnew);
    l = l * alpha + wave_sum(p);
#pragma unroll
    for (int r = 0; r < kDimSlots; ++r) acc[r] *= alpha;
    int nj = min(kWave, i - j0 + 1);
    for (int jj = 0; jj < nj; ++jj) {
      float pj = __shfl(p, jj, kWave);
      const T* vr = vbase + (size_t)(j0 + jj) * ld;
#pragma unroll
      for (int r = 0; r < kDimSlots; ++r) {
        int e = lane + kWave * r;
        if (e < dh) acc[r] = fmaf(pj, to_f32(vr[e]), acc[r]);
      }
    }
    m = mnew;
  }
  float inv = 1.0f / l;
#pragma unroll
  for (int r = 0; r < kDimSlots; ++r) {
    int e = lane + kWave * r;
    if (e < dh) o[(size_t)i * h + head * dh + e] = from_f32<T>(acc[r] * inv);
  }
  if (lane == 0) lse[(size_t)head * s + i] = m + __logf(l);
}

// delta[head][i] = sum_e dO[i, head, e] * O[i, head, e]
template <typename T>
__global__ __launch_bounds__(256) void attn_delta_kernel(const T* __restrict__ o, const T* __restrict__ d_o,
                                                         float* __restrict__ delta, int s, int h, int dh) {
  int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int head = blockIdx.y;
  int i = blockIdx.x * 4 + wave;
  if (i >= s) return;
  float d = 0.f;
  for (int e = lane; e < dh; e += kWave) {
    size_t idx = (size_t)i * h + head * dh + e;
    d = fmaf(to_f32(o[idx]), to_f32(d_o[idx]), d);
  }
  d = wave_sum(d);
  if (lane == 0) delta[(size_t)head * s + i] = d;
}

template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dq_generic_kernel(const T* __restrict__ qkv,
                                                                  const float* __restrict__ lse,
                                                                  const float* __restrict__ delta,
                                                                  const T* __restrict__ d_o, T* __restrict__ dqkv,
                                                                  int s, int h, int dh, int hkv, int group,
                                                                  float scale) {
  __shared__ float qs[4][kMaxHeadDim];
  __shared__ float dos[4][kMaxHeadDim];
  int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int head = blockIdx.y;
  int i = blockIdx.x * 4 + wave;
  bool active = i < s;
  int ld = h + 2 * hkv;
  const T* kbase = qkv + h + (head / group) * dh;
  const T* vbase = qkv + h + hkv + (head / group) * dh;
  if (active)
    for (int e = lane; e < dh; e += kWave) {
      qs[wave][e] = to_f32(qkv[(size_t)i * ld + head * dh + e]) * scale;
      dos[wave][e] = to_f32(d_o[(size_t)i * h + head * dh + e]);
    }
  __syncthreads();
  if (!active) return;
  float lse_i = lse[(size_t)head * s + i], delta_i = delta[(size_t)head * s + i];
  float acc[kDimSlots];
#pragma unroll
  for (int r = 0; r < kDimSlots; ++r) acc[r] = 0.f;
  for (int j0 = 0; j0 <= i; j0 += kWave) {
    int j = j0 + lane;
    float ds = 0.f;
    if (j <= i) {
      const T* kr = kbase + (size_t)j * ld;
      const T* vr = vbase + (size_t)j * ld;
      float sc = 0.f, dp = 0.f;
      for (int e = 0; e < dh; ++e) {
        sc = fmaf(qs[wave][e], to_f32(kr[e]), sc);
        dp = fmaf(dos[wave][e], to_f32(vr[e]), dp);
      }
      ds = __expf(sc - lse_i) * (dp - delta_i);
    }
    int nj = min(kWave, i - j0 + 1);
    for (int jj = 0; jj < nj; ++jj) {
      float dsj = __shfl(ds, jj, kWave);
      const T* kr = kbase + (size_t)(j0 + jj) * ld;
#pragma unroll
      for (int r = 0; r < kDimSlots; ++r) {
        int e = lane + kWave * r;
        if (e < dh) acc[r] = fmaf(dsj, to_f32(kr[e]), acc[r]);
      }
    }
  }
#pragma unroll
  for (int r = 0; r < kDimSlots; ++r) {
    int e = lane + kWave * r;
    if (e < dh) dqkv[(size_t)i * ld + head * dh + e] = from_f32<T>(acc[r] * scale);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dkv_generic_kernel(const T* __restrict__ qkv,
                                                                   const float* __restrict__ lse,
                                                                   const float* __restrict__ delta,
                                                                   const T* __restrict__ d_o, T* __restrict__ dqkv,
                                                                   int s, int h, int dh, int hkv, int group,
                                                                   float scale) {
  __shared__ float ks[4][kMaxHeadDim];
  __shared__ float vs[4][kMaxHeadDim];
  int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int kv_head = blockIdx.y;
  int j = blockIdx.x * 4 + wave;
  bool active = j < s;
  int ld = h + 2 * hkv;
  if (active)
    for (int e = lane; e < dh; e += kWave) {
      ks[wave][e] = to_f32(qkv[(size_t)j * ld + h + kv_head * dh + e]) * scale;
      vs[wave][e] = to_f32(qkv[(size_t)j * ld + h + hkv + kv_head * dh + e]);
    }
  __syncthreads();
  if (!active) return;
  float dk[kDimSlots], dv[kDimSlots];
#pragma unroll
  for (int r = 0; r < kDimSlots; ++r) dk[r] = dv[r] = 0.f;
  for (int g = 0; g < group; ++g) {  // the query heads that read this key/value head, in head order
    int head = kv_head * group + g;
    const T* qbase = qkv + head * dh;
    const T* dobase = d_o + head * dh;
    for (int i0 = j - (j % kWave); i0 < s; i0 += kWave) {
      int i = i0 + lane;
      float p = 0.f, ds = 0.f;
      if (i >= j && i < s) {
        const T* qr = qbase + (size_t)i * ld;
        const T* dor = dobase + (size_t)i * h;
        float sc = 0.f, dp = 0.f;
        for (int e = 0; e < dh; ++e) {
          sc = fmaf(ks[wave][e], to_f32(qr[e]), sc);
          dp = fmaf(vs[wave][e], to_f32(dor[e]), dp);
        }
        p = __expf(sc - lse[(size_t)head * s + i]);
        ds = p * (dp - delta[(size_t)head * s + i]);
      }
      int ni = min(kWave, s - i0);
      for (int ii = 0; ii < ni; ++ii) {
        float pi = __shfl(p, ii, kWave), dsi = __shfl(ds, ii, kWave);
        const T* qr = qbase + (size_t)(i0 + ii) * ld;
        const T* dor = dobase + (size_t)(i0 + ii) * h;
#pragma unroll
        for (int r = 0; r < kDimSlots; ++r) {
          int e = lane + kWave * r;
          if (e < dh) {
            dv[r] = fmaf(pi, to_f32(dor[e]), dv[r]);
            dk[r] = fmaf(dsi, to_f32(qr[e]), dk[r]);
          }
        }
      }
    }
  }
#pragma unroll
  for (int r = 0; r < kDimSlots; ++r) {
    int e = lane + kWave * r;
    if (e < dh) {
      dqkv[(size_t)j * ld + h + kv_head * dh + e] = from_f32<T>(dk[r] * scale);
      dqkv[(size_t)j * ld + h + hkv + kv_head * dh + e] = from_f32<T>(dv[r]);
    }
  }
}

static bool check_attention_shape(const char* what, int s, int h, int n_heads, int n_kv_heads) {
  if (s <= 0 || h <= 0 || n_heads <= 0 || h % n_heads != 0 || h / n_heads > kMaxHeadDim || n_kv_heads <= 0 ||
      n_heads % n_kv_heads != 0) {
    set_error("%s: s=%d h=%d heads=%d kv_heads=%d (head size must divide h and be <= %d, kv_heads must divide heads)",
              what, s, h, n_heads, n_kv_heads, kMaxHeadDim);
    return false;
  }
  return true;
}

bool attention_forward_generic(int dtype, const void* qkv, void* o, float* lse, int s, int h, int n_heads,
                               int n_kv_heads, hipStream_t stream) {
  if (!check_attention_shape("attention_forward", s, h, n_heads, n_kv_heads)) return false;
  int dh = h / n_heads, hkv = n_kv_heads * dh, group = n_heads / n_kv_heads;
  float scale = 1.0f / sqrtf((float)dh);
  dim3 grid(ceil_div(s, 4), n_heads);
  if (dtype == kF32)
    attn_fwd_generic_kernel<float><<<grid, 256, 0, stream>>>((const float*)qkv, (float*)o, lse, s, h, dh, hkv, group,
                                                             scale);
  else
    attn_fwd_generic_kernel<bf16><<<grid, 256, 0, stream>>>((const bf16*)qkv, (bf16*)o, lse, s, h, dh, hkv, group,
                                                            scale);
  return launch_ok("attn_fwd_generic_kernel");
}

bool attention_backward_generic(int dtype, const void* qkv, const void* o, const float* lse, const void* d_o,
                                void* dqkv, float* delta, int s, int h, int n_heads, int n_kv_heads,
                                hipStream_t stream) {
  if (!check_attention_shape("attention_backward", s, h, n_heads, n_kv_heads)) return false;
  int dh = h / n_heads, hkv = n_kv_heads * dh, group = n_heads / n_kv_heads;
  float scale = 1.0f / sqrtf((float)dh);
  dim3 grid(ceil_div(s, 4), n_heads), grid_kv(ceil_div(s, 4), n_kv_heads);
  if (dtype == kF32) {
    attn_delta_kernel<float><<<grid, 256, 0, stream>>>((const float*)o, (const float*)d_o, delta, s, h, dh);
    attn_bwd_dq_generic_kernel<float><<<grid, 256, 0, stream>>>((const float*)qkv, lse, delta, (const float*)d_o,
                                                                (float*)dqkv, s, h, dh, hkv, group, scale);
    attn_bwd_dkv_generic_kernel<float><<<grid_kv, 256, 0, stream>>>((const float*)qkv, lse, delta,
                                                                    (const float*)d_o, (float*)dqkv, s, h, dh, hkv,
                                                                    group, scale);
  } else {
    attn_delta_kernel<bf16><<<grid, 256, 0, stream>>>((const bf16*)o, (const bf16*)d_o, delta, s, h, dh);
    attn_bwd_dq_generic_kernel<bf16><<<grid, 256, 0, stream>>>((const bf16*)qkv, lse, delta, (const bf16*)d_o,
                                                               (bf16*)dqkv, s, h, dh, hkv, group, scale);
    attn_bwd_dkv_generic_kernel<bf16><<<grid_kv, 256, 0, stream>>>((const bf16*)qkv, lse, delta, (const bf16*)d_o,
                                                                   (bf16*)dqkv, s, h, dh, hkv, group, scale);
  }
  return launch_ok("attention backward kernels");
}

bool attention_forward(int dtype, const void* qkv, void* o, float* lse, int s, int h, int n_heads, int n_kv_heads,
                       bool force_generic, hipStream_t stream) {
  if (dtype == kBF16 && !force_generic && attention_mfma_supported(s, h, n_heads, n_kv_heads))
    return attention_forward_mfma(qkv, o, lse, s, h, n_heads, n_kv_heads, stream);
  return attention_forward_generic(dtype, qkv, o, lse, s, h, n_heads, n_kv_heads, stream);
}

bool attention_backward(int dtype, const void* qkv, const void* o, const float* lse, const void* d_o, void* dqkv,
                        float* delta, void* partials, int s, int h, int n_heads, int n_kv_heads, bool force_generic,
                        hipStream_t stream) {
  if (dtype == kBF16 && !force_generic && attention_mfma_supported(s, h, n_heads, n_kv_heads))
    return attention_backward_mfma(qkv, o, lse, d_o, dqkv, delta, partials, s, h, n_heads, n_kv_heads, stream);
  return attention_backward_generic(dtype, qkv, o, lse, d_o, dqkv, delta, s, h, n_heads, n_kv_heads, stream);
}

}  // namespace po
