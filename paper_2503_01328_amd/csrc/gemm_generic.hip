// Shape-agnostic GEMM on the vector ALU: the fp32 debug path and the home of
// every shape the MFMA kernel does not take (ragged tiles).  64x64 block tile,
// 16-deep k slices staged through LDS as fp32, each thread owns a 4x4 micro-tile.
// All bounds are checked, so any M, N, K >= 1 and any leading dimension works.
#include "kernels.h"

namespace po {

template <typename T>
__global__ __launch_bounds__(256) void gemm_generic_kernel(int trans_a, int trans_b, int M, int N, int K,
                                                           const T* __restrict__ A, int lda,
                                                           const T* __restrict__ B, int ldb, Epilogue ep) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN + 4];
  int tid = threadIdx.x;
  int tx = tid & 15, ty = tid >> 4;  // micro-tile column / row index
  int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  for (int k0 = 0; k0 < K; k0 += BK) {
    // stage A: BK x BM values, 4 per thread
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      int e = tid + u * 256;
      int kk, mm;
      if (trans_a) {  // A is [K, M]: m fastest
        mm = e & 63;
        kk = e >> 6;
      } else {  // A is [M, K]: k fastest
        kk = e & 15;
        mm = e >> 4;
      }
      int m = m0 + mm, k = k0 + kk;
      float v = 0.f;
      if (m < M && k < K) v = to_f32(trans_a ? A[(size_t)k * lda + m] : A[(size_t)m * lda + k]);
      As[kk][mm] = v;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      int e = tid + u * 256;
      int kk, nn;
      if (trans_b) {  // B is [N, K]: k fastest
        kk = e & 15;
        nn = e >> 4;
      } else {  // B is [K, N]: n fastest
        nn = e & 63;
        kk = e >> 6;
      }
      int n = n0 + nn, k = k0 + kk;
      float v = 0.f;
      if (n < N && k < K) v = to_f32(trans_b ? B[(size_t)n * ldb + k] : B[(size_t)k * ldb + n]);
      Bs[kk][nn] = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int n = n0 + tx * 4 + j;
      if (n < N) epilogue_store<T>(ep, m, n, acc[i][j]);
    }
  }
}

bool gemm_generic(int dtype, int trans_a, int trans_b, int M, int N, int K, const void* A, int lda, const void* B,
                  int ldb, const Epilogue& ep, hipStream_t stream) {
  if (M <= 0 || N <= 0 || K <= 0 || !A || !B) {
    set_error("gemm: M=%d N=%d K=%d A=%p B=%p", M, N, K, A, B);
    return false;
  }
  int need_lda = trans_a ? M : K, need_ldb = trans_b ? K : N;
  if (lda < need_lda || ldb < need_ldb || ep.ldc < N) {
    set_error("gemm: leading dimensions lda=%d ldb=%d ldc=%d too small for M=%d N=%d K=%d", lda, ldb, ep.ldc, M, N,
              K);
    return false;
  }
  if (!ep.out && !ep.acc_f32) {
    set_error("gemm: no output");
    return false;
  }
  if (ep.gelu_u && !ep.out) {
    set_error("gemm: gelu_u needs out");
    return false;
  }
  dim3 grid(ceil_div(N, 64), ceil_div(M, 64)), block(256);
  if (dtype == kF32)
    gemm_generic_kernel<float><<<grid, block, 0, stream>>>(trans_a, trans_b, M, N, K, (const float*)A, lda,
                                                           (const float*)B, ldb, ep);
  else
    gemm_generic_kernel<bf16><<<grid, block, 0, stream>>>(trans_a, trans_b, M, N, K, (const bf16*)A, lda,
                                                          (const bf16*)B, ldb, ep);
  return launch_ok("gemm_generic_kernel");
}

bool gemm(int dtype, int trans_a, int trans_b, int M, int N, int K, const void* A, int lda, const void* B, int ldb,
          const Epilogue& ep, bool force_generic, hipStream_t stream) {
  if (dtype == kBF16 && !force_generic && gemm_mfma_supported(trans_a, trans_b, M, N, K, lda, ldb, ep.ldc))
    return gemm_mfma_bf16(trans_a, trans_b, M, N, K, A, lda, B, ldb, ep, stream);
  return gemm_generic(dtype, trans_a, trans_b, M, N, K, A, lda, B, ldb, ep, stream);
}

}  // namespace po
