// HBM-bound kernels of the stage: LayerNorm forward / recompute+backward,
// deterministic column reductions (bias and LayerNorm parameter gradients),
// embedding, activation pack/unpack, fills and copies.
//
// LayerNorm rows are reduced with wavefront (64-lane) shuffles: one wave owns
// one row, lanes read 16 bytes each, so a row of h elements is covered by
// coalesced 1 KiB wave accesses.  Column reductions never use atomics: rows are
// split into chunks, each chunk writes a partial, and a second kernel adds the
// partials in chunk order, so results do not depend on scheduling.
#include <atomic>
#include <stdarg.h>
#include <stdio.h>

#include "kernels.h"

namespace po {

static thread_local char g_error[512] = "";
void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
}
const char* get_error() { return g_error; }

// --------------------------------------------------------------------------
// LayerNorm forward: y = (x - mean) * rstd * gain + shift, one wave per row.
// --------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void row_stats(const T* xr, int h, int lane, float eps, float& mean, float& rstd) {
  constexpr int V = Vec16<T>::N;
  float sum = 0.f;
  for (int c = lane * V; c < h; c += kWave * V) {
    Vec16<T> v = load16(xr + c);
#pragma unroll
    for (int i = 0; i < V; ++i) sum += to_f32(v.v[i]);
  }
  mean = wave_sum(sum) / (float)h;
  float sq = 0.f;
  for (int c = lane * V; c < h; c += kWave * V) {
    Vec16<T> v = load16(xr + c);
#pragma unroll
    for (int i = 0; i < V; ++i) {
      float d = to_f32(v.v[i]) - mean;
      sq += d * d;
    }
  }
  rstd = 1.0f / sqrtf(wave_sum(sq) / (float)h + eps);
}

template <typename T>
__global__ __launch_bounds__(256) void ln_forward_kernel(const T* __restrict__ x, const T* __restrict__ gain,
                                                         const T* __restrict__ shift, T* __restrict__ y, int rows,
                                                         int h, float eps) {
  constexpr int V = Vec16<T>::N;
  int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  int lane = threadIdx.x & 63;
  if (row >= rows) return;
  const T* xr = x + (size_t)row * h;
  T* yr = y + (size_t)row * h;
  float mean, rstd;
  row_stats(xr, h, lane, eps, mean, rstd);
  for (int c = lane * V; c < h; c += kWave * V) {
    Vec16<T> v = load16(xr + c), g = load16(gain + c), b = load16(shift + c), o;
#pragma unroll
    for (int i = 0; i < V; ++i)
      o.v[i] = from_f32<T>((to_f32(v.v[i]) - mean) * rstd * to_f32(g.v[i]) + to_f32(b.v[i]));
    store16(yr + c, o);
  }
}

// Same arithmetic in the same order with the row held in registers: VPL 16-byte vectors per lane, one pass
// over memory.  Used when h is VPL * 64 vectors exactly.
template <typename T, int VPL>
__global__ __launch_bounds__(256) void ln_forward_cached_kernel(const T* __restrict__ x, const T* __restrict__ gain,
                                                                const T* __restrict__ shift, T* __restrict__ y,
                                                                int rows, int h, float eps) {
  constexpr int V = Vec16<T>::N;
  int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  int lane = threadIdx.x & 63;
  if (row >= rows) return;
  const T* xr = x + (size_t)row * h;
  T* yr = y + (size_t)row * h;
  Vec16<T> xv[VPL];
#pragma unroll
  for (int j = 0; j < VPL; ++j) xv[j] = load16(xr + (j * kWave + lane) * V);
  float sum = 0.f;
#pragma unroll
  for (int j = 0; j < VPL; ++j)
#pragma unroll
    for (int i = 0; i < V; ++i) sum += to_f32(xv[j].v[i]);
  float mean = wave_sum(sum) / (float)h;
  float sq = 0.f;
#pragma unroll
  for (int j = 0; j < VPL; ++j)
#pragma unroll
    for (int i = 0; i < V; ++i) {
      float d = to_f32(xv[j].v[i]) - mean;
      sq += d * d;
    }
  float rstd = 1.0f / sqrtf(wave_sum(sq) / (float)h + eps);
#pragma unroll
  for (int j = 0; j < VPL; ++j) {
    int c = (j * kWave + lane) * V;
    Vec16<T> g = load16(gain + c), b = load16(shift + c), o;
#pragma unroll
    for (int i = 0; i < V; ++i)
      o.v[i] = from_f32<T>((to_f32(xv[j].v[i]) - mean) * rstd * to_f32(g.v[i]) + to_f32(b.v[i]));
    store16(yr + c, o);
  }
}

// Vectors per lane of a row that fits the register-cached kernels, else 0.
template <typename T>
static int cached_vpl(int h) {
  int per_pass = kWave * Vec16<T>::N;
  if (h % per_pass != 0) return 0;
  int vpl = h / per_pass;
  return (vpl <= 6 || vpl == 8 || vpl == 10 || vpl == 12 || vpl == 16) ? vpl : 0;
}
#define PO_VPL_SWITCH(vpl, CALL) \
  switch (vpl) {                 \
    case 1: CALL(1); break;      \
    case 2: CALL(2); break;      \
    case 3: CALL(3); break;      \
    case 4: CALL(4); break;      \
    case 5: CALL(5); break;      \
    case 6: CALL(6); break;      \
    case 8: CALL(8); break;      \
    case 10: CALL(10); break;    \
    case 12: CALL(12); break;    \
    default: CALL(16); break;    \
  }

bool layernorm_forward(int dtype, const void* x, const void* gain, const void* shift, void* y, int rows, int h,
                       float eps, hipStream_t stream) {
  if (rows <= 0 || h <= 0 || h % 8 != 0) {
    set_error("layernorm_forward: rows=%d h=%d (h must be a positive multiple of 8)", rows, h);
    return false;
  }
  dim3 grid(ceil_div(rows, 4)), block(256);
  int vpl = dtype == kF32 ? cached_vpl<float>(h) : cached_vpl<bf16>(h);
  if (vpl) {
#define PO_LNF_F32(N) ln_forward_cached_kernel<float, N><<<grid, block, 0, stream>>>( \
      (const float*)x, (const float*)gain, (const float*)shift, (float*)y, rows, h, eps)
#define PO_LNF_BF16(N) ln_forward_cached_kernel<bf16, N><<<grid, block, 0, stream>>>( \
      (const bf16*)x, (const bf16*)gain, (const bf16*)shift, (bf16*)y, rows, h, eps)
    if (dtype == kF32) {
      PO_VPL_SWITCH(vpl, PO_LNF_F32)
    } else {
      PO_VPL_SWITCH(vpl, PO_LNF_BF16)
    }
#undef PO_LNF_F32
#undef PO_LNF_BF16
    return launch_ok("ln_forward_cached_kernel");
  }
  if (dtype == kF32)
    ln_forward_kernel<float><<<grid, block, 0, stream>>>((const float*)x, (const float*)gain, (const float*)shift,
                                                         (float*)y, rows, h, eps);
  else
    ln_forward_kernel<bf16><<<grid, block, 0, stream>>>((const bf16*)x, (const bf16*)gain, (const bf16*)shift,
                                                        (bf16*)y, rows, h, eps);
  return launch_ok("ln_forward_kernel");
}

// --------------------------------------------------------------------------
// LayerNorm backward with recomputed statistics.
//   xhat = (x - mean) rstd ; dxhat = dn * gain
//   dx = dres + rstd (dxhat - mean(dxhat) - xhat mean(dxhat xhat))
//   dgain += colsum(dn * xhat) ; dshift += colsum(dn)
// Kernel 1 (wave per row) writes dx and the row statistics; kernel 2 builds
// per-row-chunk column partials; kernel 3 adds them in a fixed tree.
// --------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void ln_backward_rows_kernel(const T* __restrict__ dn, const T* __restrict__ x,
                                                               const T* __restrict__ gain,
                                                               const T* __restrict__ dres, T* __restrict__ dx,
                                                               float* __restrict__ stats, int rows, int h,
                                                               float eps) {
  constexpr int V = Vec16<T>::N;
  int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  int lane = threadIdx.x & 63;
  if (row >= rows) return;
  const T* xr = x + (size_t)row * h;
  const T* dnr = dn + (size_t)row * h;
  float mean, rstd;
  row_stats(xr, h, lane, eps, mean, rstd);
  float s1 = 0.f, s2 = 0.f;
  for (int c = lane * V; c < h; c += kWave * V) {
    Vec16<T> v = load16(xr + c), d = load16(dnr + c), g = load16(gain + c);
#pragma unroll
    for (int i = 0; i < V; ++i) {
      float dxh = to_f32(d.v[i]) * to_f32(g.v[i]);
      s1 += dxh;
      s2 += dxh * (to_f32(v.v[i]) - mean) * rstd;
    }
  }
  float c1 = wave_sum(s1) / (float)h, c2 = wave_sum(s2) / (float)h;
  for (int c = lane * V; c < h; c += kWave * V) {
    Vec16<T> v = load16(xr + c), d = load16(dnr + c), g = load16(gain + c), r, o;
    if (dres) r = load16(dres + (size_t)row * h + c);
#pragma unroll
    for (int i = 0; i < V; ++i) {
      float xh = (to_f32(v.v[i]) - mean) * rstd;
      float dxh = to_f32(d.v[i]) * to_f32(g.v[i]);
      float val = rstd * (dxh - c1 - xh * c2);
      if (dres) val += to_f32(r.v[i]);
      o.v[i] = from_f32<T>(val);
    }
    store16(dx + (size_t)row * h + c, o);
  }
  if (lane == 0) {
    stats[2 * row] = mean;
    stats[2 * row + 1] = rstd;
  }
}

// ln_backward_rows_kernel with x and dn of the row held in registers (same arithmetic, same order).
template <typename T, int VPL>
__global__ __launch_bounds__(256) void ln_backward_rows_cached_kernel(const T* __restrict__ dn, const T* __restrict__ x,
                                                                      const T* __restrict__ gain,
                                                                      const T* __restrict__ dres, T* __restrict__ dx,
                                                                      float* __restrict__ stats,
                                                                      const T* __restrict__ shift,
                                                                      T* __restrict__ n_out, int rows, int h,
                                                                      float eps) {
  constexpr int V = Vec16<T>::N;
  int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  int lane = threadIdx.x & 63;
  if (row >= rows) return;
  const T* xr = x + (size_t)row * h;
  const T* dnr = dn + (size_t)row * h;
  Vec16<T> xv[VPL], dv[VPL];
#pragma unroll
  for (int j = 0; j < VPL; ++j) {
    xv[j] = load16(xr + (j * kWave + lane) * V);
    dv[j] = load16(dnr + (j * kWave + lane) * V);
  }
  float sum = 0.f;
#pragma unroll
  for (int j = 0; j < VPL; ++j)
#pragma unroll
    for (int i = 0; i < V; ++i) sum += to_f32(xv[j].v[i]);
  float mean = wave_sum(sum) / (float)h;
  float sq = 0.f;
#pragma unroll
  for (int j = 0; j < VPL; ++j)
#pragma unroll
    for (int i = 0; i < V; ++i) {
      float d = to_f32(xv[j].v[i]) - mean;
      sq += d * d;
    }
  float rstd = 1.0f / sqrtf(wave_sum(sq) / (float)h + eps);
  float s1 = 0.f, s2 = 0.f;
#pragma unroll
  for (int j = 0; j < VPL; ++j) {
    Vec16<T> g = load16(gain + (j * kWave + lane) * V);
#pragma unroll
    for (int i = 0; i < V; ++i) {
      float dxh = to_f32(dv[j].v[i]) * to_f32(g.v[i]);
      s1 += dxh;
      s2 += dxh * (to_f32(xv[j].v[i]) - mean) * rstd;
    }
  }
  float c1 = wave_sum(s1) / (float)h, c2 = wave_sum(s2) / (float)h;
#pragma unroll
  for (int j = 0; j < VPL; ++j) {
    int c = (j * kWave + lane) * V;
    Vec16<T> g = load16(gain + c), r, o;
    if (dres) r = load16(dres + (size_t)row * h + c);
#pragma unroll
    for (int i = 0; i < V; ++i) {
      float xh = (to_f32(xv[j].v[i]) - mean) * rstd;
      float dxh = to_f32(dv[j].v[i]) * to_f32(g.v[i]);
      float val = rstd * (dxh - c1 - xh * c2);
      if (dres) val += to_f32(r.v[i]);
      o.v[i] = from_f32<T>(val);
    }
    store16(dx + (size_t)row * h + c, o);
    if (n_out) {  // the forward output of the row as well, in ln_forward_cached_kernel's arithmetic
      Vec16<T> b = load16(shift + c), n;
#pragma unroll
      for (int i = 0; i < V; ++i)
        n.v[i] = from_f32<T>((to_f32(xv[j].v[i]) - mean) * rstd * to_f32(g.v[i]) + to_f32(b.v[i]));
      store16(n_out + (size_t)row * h + c, n);
    }
  }
  if (lane == 0) {
    stats[2 * row] = mean;
    stats[2 * row + 1] = rstd;
  }
}

// Block: 256 threads = 4 waves; a lane owns 2 adjacent columns of a 128-column
// tile; wave w walks rows chunk_start + w, + 4, ...  Partials: [chunk][2][h].
template <typename T>
__global__ __launch_bounds__(256) void ln_backward_cols_kernel(const T* __restrict__ dn, const T* __restrict__ x,
                                                               const float* __restrict__ stats,
                                                               float* __restrict__ partials, int rows, int h,
                                                               int rows_per_chunk) {
  __shared__ float red[4][128][2];
  int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int col = blockIdx.x * 128 + lane * 2;
  int r0 = blockIdx.y * rows_per_chunk;
  int r1 = min(rows, r0 + rows_per_chunk);
  float g0 = 0.f, g1 = 0.f, b0 = 0.f, b1 = 0.f;
  if (col < h) {
    for (int r = r0 + wave; r < r1; r += 4) {
      float mean = stats[2 * r], rstd = stats[2 * r + 1];
      float d0 = to_f32(dn[(size_t)r * h + col]), d1 = to_f32(dn[(size_t)r * h + col + 1]);
      float x0 = to_f32(x[(size_t)r * h + col]), x1 = to_f32(x[(size_t)r * h + col + 1]);
      g0 += d0 * (x0 - mean) * rstd;
      g1 += d1 * (x1 - mean) * rstd;
      b0 += d0;
      b1 += d1;
    }
  }
  red[wave][lane * 2][0] = g0;
  red[wave][lane * 2 + 1][0] = g1;
  red[wave][lane * 2][1] = b0;
  red[wave][lane * 2 + 1][1] = b1;
  __syncthreads();
  if (threadIdx.x < 128) {
    int c = blockIdx.x * 128 + threadIdx.x;
    if (c < h) {
      float sg = 0.f, sb = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        sg += red[w][threadIdx.x][0];
        sb += red[w][threadIdx.x][1];
      }
      partials[((size_t)blockIdx.y * 2 + 0) * h + c] = sg;
      partials[((size_t)blockIdx.y * 2 + 1) * h + c] = sb;
    }
  }
}

// Sums up to 64 chunk partials per column in a fixed tree: a block owns 64 columns, thread (part, c) adds the
// chunks part, part + 4, ... in that order (its loads are independent, so they are all in flight together), and
// thread c of part 0 adds the four parts in order.  Partials are laid out [chunk][N_OUT][n]; plane o is added
// into out0 (o = 0) or out1 (o = 1).
template <int N_OUT>
__global__ __launch_bounds__(256) void chunk_partials_final_kernel(const float* __restrict__ partials,
                                                                   float* __restrict__ out0,
                                                                   float* __restrict__ out1, int n, int n_chunks) {
  __shared__ float red[N_OUT][4][64];
  int part = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int c = blockIdx.x * 64 + lane;
  float acc[N_OUT];
#pragma unroll
  for (int o = 0; o < N_OUT; ++o) acc[o] = 0.f;
  if (c < n) {
    float v[N_OUT][16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      int k = part + 4 * i;
#pragma unroll
      for (int o = 0; o < N_OUT; ++o) v[o][i] = k < n_chunks ? partials[((size_t)k * N_OUT + o) * n + c] : 0.f;
    }
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
      for (int o = 0; o < N_OUT; ++o) acc[o] += v[o][i];
  }
#pragma unroll
  for (int o = 0; o < N_OUT; ++o) red[o][part][lane] = acc[o];
  __syncthreads();
  if (part == 0 && c < n) {
#pragma unroll
    for (int o = 0; o < N_OUT; ++o) {
      float s = ((red[o][0][lane] + red[o][1][lane]) + red[o][2][lane]) + red[o][3][lane];
      float* out = o == 0 ? out0 : out1;
      out[c] += s;
    }
  }
}

static int reduce_chunks(int rows) { return max(1, min(64, ceil_div(rows, 32))); }

size_t layernorm_backward_workspace(int rows, int h) {
  return ((size_t)rows * 2 + (size_t)reduce_chunks(rows) * 2 * h) * sizeof(float);
}

bool layernorm_backward(int dtype, const void* dn, const void* x, const void* gain, const void* dres, void* dx,
                        float* dgain, float* dshift, float* workspace, int rows, int h, float eps, int parts,
                        hipStream_t stream, const void* shift, void* n_out) {
  if (rows <= 0 || h <= 0 || h % 8 != 0 || !workspace || !(parts & (kLnInputGrad | kLnParamGrad)) ||
      (n_out && (!shift || !(parts & kLnInputGrad)))) {
    set_error("layernorm_backward: rows=%d h=%d workspace=%p parts=%d shift=%p n_out=%p", rows, h, (void*)workspace,
              parts, shift, n_out);
    return false;
  }
  float* stats = workspace;
  float* partials = workspace + (size_t)rows * 2;
  int n_chunks = reduce_chunks(rows);
  int rows_per_chunk = ceil_div(rows, n_chunks);
  dim3 g1(ceil_div(rows, 4)), g2(ceil_div(h, 128), n_chunks), g3(ceil_div(h, 64));
  int vpl = dtype == kF32 ? cached_vpl<float>(h) : cached_vpl<bf16>(h);
  if ((parts & kLnInputGrad) && vpl) {
#define PO_LNB_F32(N) ln_backward_rows_cached_kernel<float, N><<<g1, 256, 0, stream>>>( \
      (const float*)dn, (const float*)x, (const float*)gain, (const float*)dres, (float*)dx, stats,         \
      (const float*)shift, (float*)n_out, rows, h, eps)
#define PO_LNB_BF16(N) ln_backward_rows_cached_kernel<bf16, N><<<g1, 256, 0, stream>>>( \
      (const bf16*)dn, (const bf16*)x, (const bf16*)gain, (const bf16*)dres, (bf16*)dx, stats,            \
      (const bf16*)shift, (bf16*)n_out, rows, h, eps)
    if (dtype == kF32) {
      PO_VPL_SWITCH(vpl, PO_LNB_F32)
    } else {
      PO_VPL_SWITCH(vpl, PO_LNB_BF16)
    }
#undef PO_LNB_F32
#undef PO_LNB_BF16
  } else if (parts & kLnInputGrad) {  // dx and the row statistics (kept in the workspace for the parameter part)
    if (dtype == kF32)
      ln_backward_rows_kernel<float><<<g1, 256, 0, stream>>>((const float*)dn, (const float*)x, (const float*)gain,
                                                             (const float*)dres, (float*)dx, stats, rows, h, eps);
    else
      ln_backward_rows_kernel<bf16><<<g1, 256, 0, stream>>>((const bf16*)dn, (const bf16*)x, (const bf16*)gain,
                                                            (const bf16*)dres, (bf16*)dx, stats, rows, h, eps);
    // rows too long for the register-cached kernel: the forward output comes from the forward kernel
    if (n_out && !layernorm_forward(dtype, x, gain, shift, n_out, rows, h, eps, stream)) return false;
  }
  if (parts & kLnParamGrad) {  // dgain, dshift from (dn, x) and the statistics an input-gradient call left
    if (dtype == kF32)
      ln_backward_cols_kernel<float><<<g2, 256, 0, stream>>>((const float*)dn, (const float*)x, stats, partials,
                                                             rows, h, rows_per_chunk);
    else
      ln_backward_cols_kernel<bf16><<<g2, 256, 0, stream>>>((const bf16*)dn, (const bf16*)x, stats, partials, rows,
                                                            h, rows_per_chunk);
    chunk_partials_final_kernel<2><<<g3, 256, 0, stream>>>(partials, dgain, dshift, h, n_chunks);
  }
  return launch_ok("layernorm_backward kernels");
}

// --------------------------------------------------------------------------
// acc[n] += sum over rows of x[r, n]   (bias gradients)
// --------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void colsum_partial_kernel(const T* __restrict__ x, float* __restrict__ partials,
                                                             int rows, int n, int rows_per_chunk) {
  __shared__ float red[4][128];
  int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int col = blockIdx.x * 128 + lane * 2;
  int r0 = blockIdx.y * rows_per_chunk;
  int r1 = min(rows, r0 + rows_per_chunk);
  float a0 = 0.f, a1 = 0.f;
  if (col < n) {
    for (int r = r0 + wave; r < r1; r += 4) {
      a0 += to_f32(x[(size_t)r * n + col]);
      a1 += to_f32(x[(size_t)r * n + col + 1]);
    }
  }
  red[wave][lane * 2] = a0;
  red[wave][lane * 2 + 1] = a1;
  __syncthreads();
  if (threadIdx.x < 128) {
    int c = blockIdx.x * 128 + threadIdx.x;
    if (c < n)
      partials[(size_t)blockIdx.y * n + c] =
          red[0][threadIdx.x] + red[1][threadIdx.x] + red[2][threadIdx.x] + red[3][threadIdx.x];
  }
}

size_t colsum_workspace(int rows, int n) { return (size_t)reduce_chunks(rows) * n * sizeof(float); }

bool colsum_accumulate(int dtype, const void* x, float* acc, float* workspace, int rows, int n,
                       hipStream_t stream) {
  if (rows <= 0 || n <= 0 || n % 2 != 0 || !workspace) {
    set_error("colsum_accumulate: rows=%d n=%d workspace=%p (n must be even)", rows, n, (void*)workspace);
    return false;
  }
  int n_chunks = reduce_chunks(rows);
  int rows_per_chunk = ceil_div(rows, n_chunks);
  dim3 g(ceil_div(n, 128), n_chunks);
  if (dtype == kF32)
    colsum_partial_kernel<float><<<g, 256, 0, stream>>>((const float*)x, workspace, rows, n, rows_per_chunk);
  else
    colsum_partial_kernel<bf16><<<g, 256, 0, stream>>>((const bf16*)x, workspace, rows, n, rows_per_chunk);
  chunk_partials_final_kernel<1><<<ceil_div(n, 64), 256, 0, stream>>>(workspace, acc, nullptr, n, n_chunks);
  return launch_ok("colsum kernels");
}

// --------------------------------------------------------------------------
// The same column sums for callers that can neither allocate nor bring a workspace (code under HIP graph
// capture, tight serving loops): the chunk partials live in a file-scope device array.  Every GPU the library
// runs on holds its own copy of the array, at its own address, until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress; what kernels and copies take is the address that call
// returns for the device that is current, resolved once per device and kept.
// --------------------------------------------------------------------------
constexpr int kStaticColsumMaxCols = 32768;
constexpr size_t kStaticScratchFloats = (size_t)64 * kStaticColsumMaxCols;  // 64 row chunks at most: 8 MiB
static __device__ __align__(256) float scratch[kStaticScratchFloats];

constexpr int kMaxDevices = 64;
static std::atomic<float*> g_scratch_of_device[kMaxDevices];

// Device address of `scratch` on the current device; null (with error text) if it cannot be resolved.
static float* static_scratch() {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    set_error("static scratch: hipGetDevice failed or device %d out of range: %s", dev, hipGetErrorString(e));
    return nullptr;
  }
  float* p = g_scratch_of_device[dev].load(std::memory_order_acquire);
  if (p) return p;
  void* addr = nullptr;
  e = hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch));
  if (e != hipSuccess || !addr) {
    set_error("static scratch: hipGetSymbolAddress failed on device %d: %s", dev, hipGetErrorString(e));
    return nullptr;
  }
  g_scratch_of_device[dev].store(static_cast<float*>(addr), std::memory_order_release);
  return static_cast<float*>(addr);
}

bool colsum_accumulate_static(int dtype, const void* x, float* acc, int rows, int n, hipStream_t stream) {
  if (rows <= 0 || n <= 0 || n % 2 != 0 || !x || !acc) {
    set_error("colsum_accumulate_static: rows=%d n=%d x=%p acc=%p (n must be even)", rows, n, x, (void*)acc);
    return false;
  }
  if (n > kStaticColsumMaxCols || colsum_workspace(rows, n) > sizeof(float) * kStaticScratchFloats) {
    set_error("colsum_accumulate_static: n=%d exceeds the %d columns the built-in scratch holds; use "
              "colsum_accumulate with a workspace", n, kStaticColsumMaxCols);
    return false;
  }
  float* ws = static_scratch();
  if (!ws) return false;
  // every partial the final kernel reads is written by the partial kernel of the same call first: nothing in
  // the scratch has to start at zero, and what an earlier call left there is never read
  return colsum_accumulate(dtype, x, acc, ws, rows, n, stream);
}

// --------------------------------------------------------------------------
// Batched column reductions: the jobs' column blocks are laid end to end on grid.x
// --------------------------------------------------------------------------
struct ReduceBatch {
  ReduceJob job[kMaxReduceJobs];
  int first128[kMaxReduceJobs + 1];  // first 128-column block of job j on the partial kernel's grid.x
  int first64[kMaxReduceJobs + 1];   // first 64-column block of job j on the final kernel's grid.x
  int n_jobs;
};

template <typename T>
__global__ __launch_bounds__(256) void reduce_batch_partial_kernel(ReduceBatch b, int rows, int rows_per_chunk) {
  __shared__ float red[4][128][2];
  int j = 0;
  while (j + 1 < b.n_jobs && (int)blockIdx.x >= b.first128[j + 1]) ++j;
  const ReduceJob& job = b.job[j];
  int n = job.n;
  int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int col0 = ((int)blockIdx.x - b.first128[j]) * 128;
  int col = col0 + lane * 2;
  int r0 = blockIdx.y * rows_per_chunk;
  int r1 = min(rows, r0 + rows_per_chunk);
  const T* a = static_cast<const T*>(job.a);
  if (job.x == nullptr) {  // plain column sum, as colsum_partial_kernel
    float a0 = 0.f, a1 = 0.f;
    if (col < n) {
      for (int r = r0 + wave; r < r1; r += 4) {
        a0 += to_f32(a[(size_t)r * n + col]);
        a1 += to_f32(a[(size_t)r * n + col + 1]);
      }
    }
    red[wave][lane * 2][0] = a0;
    red[wave][lane * 2 + 1][0] = a1;
    __syncthreads();
    if (threadIdx.x < 128) {
      int c = col0 + threadIdx.x;
      if (c < n)
        job.partials[(size_t)blockIdx.y * n + c] =
            red[0][threadIdx.x][0] + red[1][threadIdx.x][0] + red[2][threadIdx.x][0] + red[3][threadIdx.x][0];
    }
  } else {  // LayerNorm gain / shift partials, as ln_backward_cols_kernel
    const T* x = static_cast<const T*>(job.x);
    const float* stats = job.stats;
    float g0 = 0.f, g1 = 0.f, b0 = 0.f, b1 = 0.f;
    if (col < n) {
      for (int r = r0 + wave; r < r1; r += 4) {
        float mean = stats[2 * r], rstd = stats[2 * r + 1];
        float d0 = to_f32(a[(size_t)r * n + col]), d1 = to_f32(a[(size_t)r * n + col + 1]);
        float x0 = to_f32(x[(size_t)r * n + col]), x1 = to_f32(x[(size_t)r * n + col + 1]);
        g0 += d0 * (x0 - mean) * rstd;
        g1 += d1 * (x1 - mean) * rstd;
        b0 += d0;
        b1 += d1;
      }
    }
    red[wave][lane * 2][0] = g0;
    red[wave][lane * 2 + 1][0] = g1;
    red[wave][lane * 2][1] = b0;
    red[wave][lane * 2 + 1][1] = b1;
    __syncthreads();
    if (threadIdx.x < 128) {
      int c = col0 + threadIdx.x;
      if (c < n) {
        float sg = 0.f, sb = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          sg += red[w][threadIdx.x][0];
          sb += red[w][threadIdx.x][1];
        }
        job.partials[((size_t)blockIdx.y * 2 + 0) * n + c] = sg;
        job.partials[((size_t)blockIdx.y * 2 + 1) * n + c] = sb;
      }
    }
  }
}

// The same partials with 16-byte loads: a block still owns 128 columns of one chunk of rows, but a lane reads
// 16 bytes (8 bf16 or 4 fp32 columns) of a row, so a wave covers 64 / LPR rows of the block's 256 or 512 bytes
// per load instead of one row, 4 bytes a lane.  Per column the rows are summed in a fixed order (by lane, then
// across the block's row slots in order): deterministic, though not the order of the kernel above.  Needs
// n % V == 0 and 16-byte aligned rows.
template <typename T>
__global__ __launch_bounds__(256) void reduce_batch_partial_vec_kernel(ReduceBatch b, int rows, int rows_per_chunk) {
  constexpr int V = Vec16<T>::N;   // columns per lane
  constexpr int LPR = 128 / V;     // lanes per row of the block's 128 columns
  constexpr int RPW = kWave / LPR;  // rows a wave reads at once
  constexpr int SLOTS = 4 * RPW;   // row slots of the block
  __shared__ float red[SLOTS][2][128];
  int j = 0;
  while (j + 1 < b.n_jobs && (int)blockIdx.x >= b.first128[j + 1]) ++j;
  const ReduceJob& job = b.job[j];
  const int n = job.n;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int col0 = ((int)blockIdx.x - b.first128[j]) * 128;
  const int cl = (lane % LPR) * V;  // first column of this lane within the block
  const int slot = wave * RPW + lane / LPR;
  const int r0 = blockIdx.y * rows_per_chunk;
  const int r1 = min(rows, r0 + rows_per_chunk);
  const T* a = static_cast<const T*>(job.a);
  const T* x = static_cast<const T*>(job.x);
  const bool ln = x != nullptr;
  float s0[V], s1[V];
#pragma unroll
  for (int i = 0; i < V; ++i) s0[i] = s1[i] = 0.f;
  if (col0 + cl < n) {
    if (!ln) {
      for (int r = r0 + slot; r < r1; r += SLOTS) {
        Vec16<T> v = load16(a + (size_t)r * n + col0 + cl);
#pragma unroll
        for (int i = 0; i < V; ++i) s0[i] += to_f32(v.v[i]);
      }
    } else {
      const float* stats = job.stats;
      for (int r = r0 + slot; r < r1; r += SLOTS) {
        float mean = stats[2 * r], rstd = stats[2 * r + 1];
        Vec16<T> d = load16(a + (size_t)r * n + col0 + cl);
        Vec16<T> xv = load16(x + (size_t)r * n + col0 + cl);
#pragma unroll
        for (int i = 0; i < V; ++i) {
          float dv = to_f32(d.v[i]);
          s0[i] += dv * (to_f32(xv.v[i]) - mean) * rstd;
          s1[i] += dv;
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < V; ++i) {
    red[slot][0][cl + i] = s0[i];
    red[slot][1][cl + i] = s1[i];
  }
  __syncthreads();
  const int c = threadIdx.x & 127, plane = threadIdx.x >> 7;
  if (col0 + c < n && (plane == 0 || ln)) {
    float sum = 0.f;
#pragma unroll
    for (int k = 0; k < SLOTS; ++k) sum += red[k][plane][c];
    const int n_out = ln ? 2 : 1;
    job.partials[((size_t)blockIdx.y * n_out + plane) * n + col0 + c] = sum;
  }
}

// The fixed tree of chunk_partials_final_kernel, per job with one or two output planes.
__global__ __launch_bounds__(256) void reduce_batch_final_kernel(ReduceBatch b, int n_chunks) {
  __shared__ float red[2][4][64];
  int j = 0;
  while (j + 1 < b.n_jobs && (int)blockIdx.x >= b.first64[j + 1]) ++j;
  const ReduceJob& job = b.job[j];
  int n = job.n;
  int n_out = job.x ? 2 : 1;
  int part = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int c = ((int)blockIdx.x - b.first64[j]) * 64 + lane;
  float acc[2] = {0.f, 0.f};
  if (c < n) {
#pragma unroll
    for (int o = 0; o < 2; ++o) {
      if (o < n_out) {
        float v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          int k = part + 4 * i;
          v[i] = k < n_chunks ? job.partials[((size_t)k * n_out + o) * n + c] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[o] += v[i];
      }
    }
  }
  red[0][part][lane] = acc[0];
  red[1][part][lane] = acc[1];
  __syncthreads();
  if (part == 0 && c < n) {
    job.out0[c] += ((red[0][0][lane] + red[0][1][lane]) + red[0][2][lane]) + red[0][3][lane];
    if (n_out == 2) job.out1[c] += ((red[1][0][lane] + red[1][1][lane]) + red[1][2][lane]) + red[1][3][lane];
  }
}

size_t column_reductions_workspace(int rows, int n) { return (size_t)reduce_chunks(rows) * n * sizeof(float); }

bool column_reductions(int dtype, const ReduceJob* jobs, int n_jobs, int rows, hipStream_t stream) {
  if (n_jobs < 1 || n_jobs > kMaxReduceJobs || rows <= 0 || !jobs) {
    set_error("column_reductions: n_jobs=%d rows=%d", n_jobs, rows);
    return false;
  }
  ReduceBatch b;
  b.n_jobs = n_jobs;
  b.first128[0] = b.first64[0] = 0;
  for (int j = 0; j < n_jobs; ++j) {
    const ReduceJob& job = jobs[j];
    if (job.n <= 0 || job.n % 2 != 0 || !job.a || !job.out0 || !job.partials ||
        (job.x && (!job.stats || !job.out1))) {
      set_error("column_reductions: job %d: n=%d a=%p out0=%p partials=%p x=%p stats=%p out1=%p", j, job.n, job.a,
                (void*)job.out0, (void*)job.partials, job.x, (const void*)job.stats, (void*)job.out1);
      return false;
    }
    b.job[j] = job;
    b.first128[j + 1] = b.first128[j] + ceil_div(job.n, 128);
    b.first64[j + 1] = b.first64[j] + ceil_div(job.n, 64);
  }
  for (int j = n_jobs; j < kMaxReduceJobs; ++j) {
    b.job[j] = ReduceJob{nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0};
    b.first128[j + 1] = b.first128[n_jobs];
    b.first64[j + 1] = b.first64[n_jobs];
  }
  int n_chunks = reduce_chunks(rows);
  int rows_per_chunk = ceil_div(rows, n_chunks);
  dim3 g(b.first128[n_jobs], n_chunks);
  const int v = dtype == kF32 ? 4 : 8;
  bool vec = true;  // 16-byte loads need whole vectors per row and aligned rows
  for (int j = 0; j < n_jobs; ++j)
    vec = vec && jobs[j].n % v == 0 && (uintptr_t)jobs[j].a % 16 == 0 && (uintptr_t)jobs[j].x % 16 == 0;
  if (vec && dtype == kF32)
    reduce_batch_partial_vec_kernel<float><<<g, 256, 0, stream>>>(b, rows, rows_per_chunk);
  else if (vec)
    reduce_batch_partial_vec_kernel<bf16><<<g, 256, 0, stream>>>(b, rows, rows_per_chunk);
  else if (dtype == kF32)
    reduce_batch_partial_kernel<float><<<g, 256, 0, stream>>>(b, rows, rows_per_chunk);
  else
    reduce_batch_partial_kernel<bf16><<<g, 256, 0, stream>>>(b, rows, rows_per_chunk);
  reduce_batch_final_kernel<<<b.first64[n_jobs], 256, 0, stream>>>(b, n_chunks);
  return launch_ok("column reduction kernels");
}

// --------------------------------------------------------------------------
// Embedding: x[p] = wte[tok[p]] + wpe[p]; backward adds dx into dwpe row by row
// and into dwte with one block per vocabulary row scanning positions in order
// (repeated tokens are summed in position order: deterministic, no atomics).
// --------------------------------------------------------------------------
template <typename T>
__global__ void embedding_forward_kernel(const int32_t* __restrict__ tok, const T* __restrict__ wte,
                                         const T* __restrict__ wpe, T* __restrict__ x, int s, int h, int vocab) {
  int p = blockIdx.x;
  int t = tok[p];
  t = min(max(t, 0), vocab - 1);
  for (int c = threadIdx.x; c < h; c += blockDim.x)
    x[(size_t)p * h + c] = from_f32<T>(to_f32(wte[(size_t)t * h + c]) + to_f32(wpe[(size_t)p * h + c]));
}

template <typename T>
__global__ void embedding_backward_kernel(const int32_t* __restrict__ tok, const T* __restrict__ dx,
                                          float* __restrict__ dwte, float* __restrict__ dwpe, int s, int h,
                                          int vocab) {
  int row = blockIdx.x;
  if (row < vocab) {
    for (int p = 0; p < s; ++p) {
      int t = min(max(tok[p], 0), vocab - 1);
      if (t != row) continue;  // uniform across the block
      for (int c = threadIdx.x; c < h; c += blockDim.x) dwte[(size_t)row * h + c] += to_f32(dx[(size_t)p * h + c]);
    }
  } else {
    int p = row - vocab;
    for (int c = threadIdx.x; c < h; c += blockDim.x) dwpe[(size_t)p * h + c] += to_f32(dx[(size_t)p * h + c]);
  }
}

bool embedding_forward(int dtype, const int32_t* tok, const void* wte, const void* wpe, void* x, int s, int h,
                       int vocab, hipStream_t stream) {
  if (s <= 0 || h <= 0 || vocab <= 0) {
    set_error("embedding_forward: s=%d h=%d vocab=%d", s, h, vocab);
    return false;
  }
  if (dtype == kF32)
    embedding_forward_kernel<float><<<s, 256, 0, stream>>>(tok, (const float*)wte, (const float*)wpe, (float*)x,
                                                           s, h, vocab);
  else
    embedding_forward_kernel<bf16><<<s, 256, 0, stream>>>(tok, (const bf16*)wte, (const bf16*)wpe, (bf16*)x, s, h,
                                                          vocab);
  return launch_ok("embedding_forward_kernel");
}

bool embedding_backward(int dtype, const int32_t* tok, const void* dx, float* dwte, float* dwpe, int s, int h,
                        int vocab, hipStream_t stream) {
  if (s <= 0 || h <= 0 || vocab <= 0) {
    set_error("embedding_backward: s=%d h=%d vocab=%d", s, h, vocab);
    return false;
  }
  if (dtype == kF32)
    embedding_backward_kernel<float><<<vocab + s, 256, 0, stream>>>(tok, (const float*)dx, dwte, dwpe, s, h, vocab);
  else
    embedding_backward_kernel<bf16><<<vocab + s, 256, 0, stream>>>(tok, (const bf16*)dx, dwte, dwpe, s, h, vocab);
  return launch_ok("embedding_backward_kernel");
}

// --------------------------------------------------------------------------
// Dropout with a regenerated mask: out[r, c] = x[r, c] * keep(r, c) * scale.  The backward of a dropout site is
// the same map applied to the incoming gradient.  One thread per four columns (one generator block).
// --------------------------------------------------------------------------
// `residual` (may be null) is added after the mask: out = residual + dropout(x), the forward of a projection
// whose output is dropped before it joins the residual stream.
template <typename T>
__global__ __launch_bounds__(256) void dropout_apply_kernel(const T* __restrict__ x, const T* __restrict__ residual,
                                                            T* __restrict__ out, int rows, int cols, DropoutSite d) {
  int per_row = (cols + 3) >> 2;
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)rows * per_row) return;
  int r = (int)(idx / per_row), c4 = (int)(idx % per_row);
  PhiloxWords w = dropout_words(d, r, c4);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int c = 4 * c4 + i;
    if (c < cols) {
      size_t at = (size_t)r * cols + c;
      float v = w.w[i] >= d.threshold ? to_f32(x[at]) * d.scale : 0.f;
      if (residual) v += to_f32(residual[at]);
      out[at] = from_f32<T>(v);
    }
  }
}

DropoutSite make_dropout_site(float p, uint64_t seed, int layer, int site, int unit) {
  DropoutSite d;
  double t = (double)p * 4294967296.0 + 0.5;
  d.threshold = t >= 4294967295.0 ? 4294967295u : (uint32_t)t;
  d.k0 = (uint32_t)seed;
  d.k1 = (uint32_t)(seed >> 32);
  d.stream = (uint32_t)(2 * layer + site);
  d.unit = (uint32_t)unit;
  d.scale = (float)(1.0 / (1.0 - (double)p));
  return d;
}

bool dropout_apply(int dtype, const void* x, const void* residual, void* out, int rows, int cols,
                   const DropoutSite& d, hipStream_t stream) {
  if (rows <= 0 || cols <= 0 || !x || !out || d.scale == 0.f) {
    set_error("dropout_apply: rows=%d cols=%d x=%p out=%p", rows, cols, x, out);
    return false;
  }
  size_t n = (size_t)rows * ((cols + 3) / 4);
  unsigned grid = (unsigned)((n + 255) / 256);
  if (dtype == kF32)
    dropout_apply_kernel<float><<<grid, 256, 0, stream>>>((const float*)x, (const float*)residual, (float*)out, rows,
                                                          cols, d);
  else
    dropout_apply_kernel<bf16><<<grid, 256, 0, stream>>>((const bf16*)x, (const bf16*)residual, (bf16*)out, rows,
                                                         cols, d);
  return launch_ok("dropout_apply_kernel");
}

// --------------------------------------------------------------------------
// Fill / copy
// --------------------------------------------------------------------------
__global__ void fill_u32_kernel(uint32_t* p, uint32_t pattern, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = pattern;
}

bool fill_u32(void* p, uint32_t pattern, size_t bytes, hipStream_t stream) {
  if (bytes % 4 != 0) {
    set_error("fill_u32: %zu bytes is not a multiple of 4", bytes);
    return false;
  }
  if (bytes == 0) return true;
  size_t n = bytes / 4;
  int grid = (int)min((size_t)4096, (n + 255) / 256);
  fill_u32_kernel<<<grid, 256, 0, stream>>>((uint32_t*)p, pattern, n);
  return launch_ok("fill_u32_kernel");
}

__global__ __launch_bounds__(256) void copy16_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src,
                                                     size_t n) {
  size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x;
  uint4 v[4];
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (i + u * 256 < n) v[u] = src[i + u * 256];
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (i + u * 256 < n) dst[i + u * 256] = v[u];
}

bool copy_bytes(void* dst, const void* src, size_t bytes, hipStream_t stream) {
  if (bytes % 16 != 0 || ((uintptr_t)dst | (uintptr_t)src) % 16 != 0) {
    set_error("copy_bytes: %zu bytes / pointers must be multiples of 16", bytes);
    return false;
  }
  if (bytes == 0) return true;
  size_t n = bytes / 16;
  copy16_kernel<<<(unsigned)((n + 1023) / 1024), 256, 0, stream>>>((uint4*)dst, (const uint4*)src, n);
  return launch_ok("copy16_kernel");
}

// --------------------------------------------------------------------------
// Pack / unpack: n_seg segments <-> one contiguous buffer, 16 bytes per lane,
// four loads in flight per lane.  The segment table travels as a kernel argument.
// --------------------------------------------------------------------------
struct SegTable {
  char* ptr[kMaxPackSegments];
  uint64_t first_chunk[kMaxPackSegments + 1];  // prefix sums in 16-byte chunks
  int n;
};

template <bool kPack>
__global__ __launch_bounds__(256) void pack_kernel(SegTable tab, uint4* __restrict__ packed) {
  uint64_t total = tab.first_chunk[tab.n];
  uint64_t base = (uint64_t)blockIdx.x * 1024 + threadIdx.x;
  // segment holding the block's first chunk; later chunks only move forward
  int seg = 0;
  {
    uint64_t b0 = (uint64_t)blockIdx.x * 1024;
    while (seg + 1 < tab.n && tab.first_chunk[seg + 1] <= b0) ++seg;
  }
  uint4 v[4];
  uint4* where[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    uint64_t i = base + (uint64_t)u * 256;
    where[u] = nullptr;
    if (i < total) {
      int sg = seg;
      while (tab.first_chunk[sg + 1] <= i) ++sg;
      where[u] = reinterpret_cast<uint4*>(tab.ptr[sg]) + (i - tab.first_chunk[sg]);
      v[u] = kPack ? *where[u] : packed[i];
    }
  }
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    uint64_t i = base + (uint64_t)u * 256;
    if (i < total) {
      if (kPack)
        packed[i] = v[u];
      else
        *where[u] = v[u];
    }
  }
}

static bool build_table(const void* const* seg_ptrs, const uint64_t* seg_bytes, int n_seg, const void* packed,
                        SegTable& tab) {
  if (n_seg < 0 || n_seg > kMaxPackSegments) {
    set_error("pack: %d segments (at most %d)", n_seg, kMaxPackSegments);
    return false;
  }
  if ((uintptr_t)packed % 16 != 0) {
    set_error("pack: packed buffer is not 16-byte aligned");
    return false;
  }
  tab.n = n_seg;
  tab.first_chunk[0] = 0;
  for (int i = 0; i < n_seg; ++i) {
    if (seg_bytes[i] % 16 != 0 || (uintptr_t)seg_ptrs[i] % 16 != 0 || (seg_bytes[i] && !seg_ptrs[i])) {
      set_error("pack: segment %d (%p, %llu bytes) must be 16-byte aligned and sized", i, seg_ptrs[i],
                (unsigned long long)seg_bytes[i]);
      return false;
    }
    tab.ptr[i] = (char*)seg_ptrs[i];
    tab.first_chunk[i + 1] = tab.first_chunk[i] + seg_bytes[i] / 16;
  }
  return true;
}

bool pack_segments(const void* const* seg_ptrs, const uint64_t* seg_bytes, int n_seg, void* packed,
                   hipStream_t stream) {
  SegTable tab;
  if (!build_table(seg_ptrs, seg_bytes, n_seg, packed, tab)) return false;
  uint64_t total = tab.first_chunk[n_seg];
  if (total == 0) return true;
  pack_kernel<true><<<(unsigned)((total + 1023) / 1024), 256, 0, stream>>>(tab, (uint4*)packed);
  return launch_ok("pack_kernel");
}

bool unpack_segments(void* const* seg_ptrs, const uint64_t* seg_bytes, int n_seg, const void* packed,
                     hipStream_t stream) {
  SegTable tab;
  if (!build_table((const void* const*)seg_ptrs, seg_bytes, n_seg, packed, tab)) return false;
  uint64_t total = tab.first_chunk[n_seg];
  if (total == 0) return true;
  pack_kernel<false><<<(unsigned)((total + 1023) / 1024), 256, 0, stream>>>(tab, (uint4*)const_cast<void*>(packed));
  return launch_ok("unpack_kernel");
}

}  // namespace po
