// Host-side launchers of the HIP kernels.  Every launcher validates its shapes
// on the host, enqueues on `stream`, and returns false with po::set_error text
// when the arguments do not fit what the kernel assumes.
#pragma once

#include "po_common.h"

namespace po {

void set_error(const char* fmt, ...);
const char* get_error();

// ---- elementwise / normalisation (elementwise.hip) -------------------------
bool layernorm_forward(int dtype, const void* x, const void* gain, const void* shift, void* y, int rows, int h,
                       float eps, hipStream_t stream);
size_t layernorm_backward_workspace(int rows, int h);
// parts: kLnInputGrad writes dx (= dres + LayerNorm input gradient) and the row statistics into the workspace;
// kLnParamGrad adds the gain / shift gradients, reading the statistics an earlier or the same call left there.
// n_out (with shift, kLnInputGrad only): also writes LayerNorm(x), bit for bit what layernorm_forward writes, for a
// caller that needs the recomputed forward output next and would otherwise read x once more for it.
enum { kLnInputGrad = 1, kLnParamGrad = 2 };
bool layernorm_backward(int dtype, const void* dn, const void* x, const void* gain, const void* dres, void* dx,
                        float* dgain, float* dshift, float* workspace, int rows, int h, float eps, int parts,
                        hipStream_t stream, const void* shift = nullptr, void* n_out = nullptr);
size_t colsum_workspace(int rows, int n);
bool colsum_accumulate(int dtype, const void* x, float* acc, float* workspace, int rows, int n, hipStream_t stream);
// The same with the partials in a device array built into the library (no workspace, nothing allocated);
// n <= 32768.  Calls that overlap on one GPU share that array and race.
bool colsum_accumulate_static(int dtype, const void* x, float* acc, int rows, int n, hipStream_t stream);
// Several column reductions over the same number of rows in two launches (all partial sums, then all final
// sums) instead of two per tensor: the bias gradients and LayerNorm gain / shift gradients of one layer.
// Per job the arithmetic and its order are those of colsum_accumulate / layernorm_backward(kLnParamGrad).
struct ReduceJob {
  const void* a;       // [rows, n] of dtype: the tensor summed over rows, or dn of a LayerNorm
  const void* x;       // LayerNorm input [rows, n]; null: plain column sum
  const float* stats;  // LayerNorm row statistics [rows][2] (mean, 1/std) left by kLnInputGrad; null for a sum
  float* out0;         // [n] fp32, += column sum, or += gain gradient
  float* out1;         // [n] fp32, += shift gradient (LayerNorm only)
  float* partials;     // fp32 workspace: column_reductions_workspace(rows, n) floats, x2 for a LayerNorm job
  int n;               // columns, even
};
constexpr int kMaxReduceJobs = 8;
size_t column_reductions_workspace(int rows, int n);  // bytes per output plane
bool column_reductions(int dtype, const ReduceJob* jobs, int n_jobs, int rows, hipStream_t stream);
bool embedding_forward(int dtype, const int32_t* tok, const void* wte, const void* wpe, void* x, int s, int h,
                       int vocab, hipStream_t stream);
bool embedding_backward(int dtype, const int32_t* tok, const void* dx, float* dwte, float* dwpe, int s, int h,
                        int vocab, hipStream_t stream);
bool fill_u32(void* p, uint32_t pattern, size_t bytes, hipStream_t stream);
bool copy_bytes(void* dst, const void* src, size_t bytes, hipStream_t stream);

constexpr int kMaxPackSegments = 48;
bool pack_segments(const void* const* seg_ptrs, const uint64_t* seg_bytes, int n_seg, void* packed,
                   hipStream_t stream);
bool unpack_segments(void* const* seg_ptrs, const uint64_t* seg_bytes, int n_seg, const void* packed,
                     hipStream_t stream);

// ---- GEMM (gemm_generic.hip, gemm_mfma.hip) ---------------------------------
// C[M,N] = op(A) op(B): trans_a == 0: A [M,K] (lda >= K); 1: A [K,M] (lda >= M).
// trans_b == 0: B [K,N] (ldb >= N); 1: B [N,K] (ldb >= K).
bool gemm_generic(int dtype, int trans_a, int trans_b, int M, int N, int K, const void* A, int lda, const void* B,
                  int ldb, const Epilogue& ep, hipStream_t stream);
// bf16 MFMA path; returns false (with error text) if the shape is not supported.
bool gemm_mfma_supported(int trans_a, int trans_b, int M, int N, int K, int lda, int ldb, int ldc);
// Output tile (rows, columns) the bf16 MFMA path uses for an M x N result; 0, 0 if it has none for the shape.
void gemm_mfma_tile(int M, int N, int* bm, int* bn);
bool gemm_mfma_bf16(int trans_a, int trans_b, int M, int N, int K, const void* A, int lda, const void* B, int ldb,
                    const Epilogue& ep, hipStream_t stream);
// Several weight-gradient GEMMs in one launch, C_i [M_i, N_i] (fp32) += A_i^T B_i with A_i [K_i, M_i] and
// B_i [K_i, N_i] bf16: the form of the four parameter-gradient products of a layer.  Supported when every M_i and
// N_i is a multiple of 256 and every K_i of 64 (at most 4 problems); results equal the single launches bit for bit.
struct GemmProblem {
  int M, N, K;
  const void* A;
  int lda;
  const void* B;
  int ldb;
  float* acc_f32;
  int ldc;
};
bool gemm_mfma_grouped_supported(int n, const GemmProblem* p);
bool gemm_mfma_grouped_accumulate(int n, const GemmProblem* p, hipStream_t stream);
// Picks the MFMA kernel for bf16 when the shape allows it, else the generic one.
bool gemm(int dtype, int trans_a, int trans_b, int M, int N, int K, const void* A, int lda, const void* B, int ldb,
          const Epilogue& ep, bool force_generic, hipStream_t stream);

// ---- dropout with regenerated masks (elementwise.hip) --------------------------
// threshold = round(p 2^32) (an element is kept iff its random word is >= it), scale = 1 / (1 - p), key = seed.
DropoutSite make_dropout_site(float p, uint64_t seed, int layer, int site, int unit);
// out = (residual ? residual : 0) + dropout(x); x, residual, out are [rows, cols] of dtype.
bool dropout_apply(int dtype, const void* x, const void* residual, void* out, int rows, int cols,
                   const DropoutSite& d, hipStream_t stream);

// ---- attention (attention_generic.hip, attention_mfma.hip) -------------------
// qkv is [s, h + 2 hkv]: query block [h], key block [hkv], value block [hkv], hkv = n_kv_heads * (h / n_heads);
// query head t reads key/value head t / (n_heads / n_kv_heads).  n_kv_heads = n_heads is plain multi-head.
bool attention_forward_generic(int dtype, const void* qkv, void* o, float* lse, int s, int h, int n_heads,
                               int n_kv_heads, hipStream_t stream);
bool attention_backward_generic(int dtype, const void* qkv, const void* o, const float* lse, const void* d_o,
                                void* dqkv, float* delta, int s, int h, int n_heads, int n_kv_heads,
                                hipStream_t stream);
bool attention_mfma_supported(int s, int h, int n_heads, int n_kv_heads);
bool attention_forward_mfma(const void* qkv, void* o, float* lse, int s, int h, int n_heads, int n_kv_heads,
                            hipStream_t stream);
// partials: optional [s, 2h] workspace of the dtype; with it, grouped-query shapes with few key/value heads run
// dK/dV per query head and add the groups up afterwards.
bool attention_backward_mfma(const void* qkv, const void* o, const float* lse, const void* d_o, void* dqkv,
                             float* delta, void* partials, int s, int h, int n_heads, int n_kv_heads,
                             hipStream_t stream);
bool attention_forward(int dtype, const void* qkv, void* o, float* lse, int s, int h, int n_heads, int n_kv_heads,
                       bool force_generic, hipStream_t stream);
bool attention_backward(int dtype, const void* qkv, const void* o, const float* lse, const void* d_o, void* dqkv,
                        float* delta, void* partials, int s, int h, int n_heads, int n_kv_heads, bool force_generic,
                        hipStream_t stream);

#define PO_HIP_OK(expr)                                                                  \
  do {                                                                                   \
    hipError_t e__ = (expr);                                                             \
    if (e__ != hipSuccess) {                                                             \
      po::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e__), __FILE__, __LINE__); \
      return false;                                                                      \
    }                                                                                    \
  } while (0)

// hipGetLastError is sticky per thread: an error left behind by an earlier, unrelated HIP call
// (of this library or of the host program) must not be blamed on the next launch.
inline void begin_launch() { (void)hipGetLastError(); }

inline bool launch_ok(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    set_error("launch of %s failed: %s", what, hipGetErrorString(e));
    return false;
  }
  return true;
}

}  // namespace po
