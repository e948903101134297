// bf16 GEMM on the CDNA4 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulate.
//
// One 256-thread block (4 waves, 2 x 2) owns a (64*WTM) x (64*WTN) tile of C; a
// wave owns WTM x WTN MFMA tiles of 32 x 32, i.e. up to 128 x 128 with 256 fp32
// accumulators per lane.  K is walked in slices of 64.  A slice of an operand is
// held in LDS as [rows][64] bf16 (128 bytes per row, eight 16-byte chunks whose
// position is XOR-swizzled with the row index so that fragment reads and slice
// writes spread over the banks).  Slices are double-buffered: while the matrix
// cores work on slice t from LDS, the global loads of slice t+1 are in flight
// into registers and are written to the other LDS buffer before one barrier.
//
// Operand forms (all three are needed by the stage):
//   forward   C = A[M,K]   B[K,N]      (B is n-contiguous -> transposed on the way to LDS)
//   dgrad     C = A[M,K]   B^T, B[N,K] (both k-contiguous -> straight copies)
//   wgrad     C = A^T B, A[K,M] B[K,N] (both transposed on the way to LDS)
// A transposed operand is read from HBM in 8 x 8 blocks along its contiguous
// dimension (still 16-byte coalesced loads) and transposed in registers, so that
// LDS always holds k-contiguous rows and every MFMA fragment is one ds_read_b128.
//
// The MFMA is issued with the B fragment in the first operand slot: a lane then
// holds four consecutive n of one row m per accumulator quad, which gives 8-byte
// (bf16) or 16-byte (fp32) vector accesses in the epilogue.
//
// Workgroup ids are remapped so that the blocks that land on one XCD (ids equal
// modulo 8) work on neighbouring tiles and share operand slices in that XCD's L2.
#include "kernels.h"

namespace po {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBK = 64;

__device__ __forceinline__ int swizzle_chunk(int chunk, int row) { return chunk ^ (row & 7) ^ ((row >> 3) & 7); }

// ---- global -> registers -> LDS staging of one operand slice ----------------
template <int R, bool TRANS>
struct Stager {
  // k-contiguous: R*8 chunks of 16 B, R/32 per thread.  Transposed: R blocks of 8x8, at most one per thread.
  static constexpr int NREG = TRANS ? 8 : R / 32;
  u32x4 reg[NREG];

  // base points at element (row 0 of the tile, k = 0 of the matrix); k0 = slice start.
  __device__ __forceinline__ void load(const bf16* __restrict__ base, int ld, int k0, int tid) {
    if (TRANS) {
      if (tid < R) {
        int rb = tid % (R / 8), kb = tid / (R / 8);
        const bf16* p = base + (size_t)(k0 + 8 * kb) * ld + 8 * rb;
#pragma unroll
        for (int i = 0; i < 8; ++i) reg[i] = *reinterpret_cast<const u32x4*>(p + (size_t)i * ld);
      }
    } else {
#pragma unroll
      for (int u = 0; u < NREG; ++u) {
        int e = tid + 256 * u;
        int row = e >> 3, c = e & 7;
        reg[u] = *reinterpret_cast<const u32x4*>(base + (size_t)row * ld + k0 + c * 8);
      }
    }
  }

  __device__ __forceinline__ void store(char* lds, int tid) const {
    if (TRANS) {
      if (tid < R) {
        int rb = tid % (R / 8), kb = tid / (R / 8);
        const uint32_t* in = reinterpret_cast<const uint32_t*>(reg);  // in[i*4 + d]: k = i, m = 2d, 2d+1
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          u32x4 o;
          uint32_t* od = reinterpret_cast<uint32_t*>(&o);
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            uint32_t a = in[(2 * q) * 4 + (j >> 1)], b = in[(2 * q + 1) * 4 + (j >> 1)];
            od[q] = (j & 1) ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0xffffu) | (b << 16));
          }
          int row = 8 * rb + j;
          *reinterpret_cast<u32x4*>(lds + row * 128 + (swizzle_chunk(kb, row) << 4)) = o;
        }
      }
    } else {
#pragma unroll
      for (int u = 0; u < NREG; ++u) {
        int e = tid + 256 * u;
        int row = e >> 3, c = e & 7;
        *reinterpret_cast<u32x4*>(lds + row * 128 + (swizzle_chunk(c, row) << 4)) = reg[u];
      }
    }
  }
};

__device__ __forceinline__ bf16x8 read_fragment(const char* lds, int row, int chunk) {
  return *reinterpret_cast<const bf16x8*>(lds + row * 128 + (swizzle_chunk(chunk, row) << 4));
}

// ---- epilogue on four consecutive n of one row --------------------------------
struct __attribute__((aligned(8))) bf16x4_t {
  bf16 v[4];
};

// Epilogue kinds are compile-time so that the fully unrolled accumulator walk stays small.
enum EpiKind : int { kEpiStore = 0, kEpiStoreGelu = 1, kEpiGeluBackward = 2, kEpiAccumulate = 3 };

template <int EPI>
__device__ __forceinline__ void epilogue_store4(const Epilogue& e, int m, int n, float a0, float a1, float a2,
                                                float a3) {
  size_t idx = (size_t)m * e.ldc + n;
  float a[4] = {a0, a1, a2, a3};
  if (EPI == kEpiAccumulate) {
    float4* p = reinterpret_cast<float4*>(e.acc_f32 + idx);
    float4 o = *p;
    o.x += a[0];
    o.y += a[1];
    o.z += a[2];
    o.w += a[3];
    *p = o;
    return;
  }
  if (EPI == kEpiGeluBackward) {
    bf16x4_t u = *reinterpret_cast<const bf16x4_t*>(static_cast<const bf16*>(e.gelu_u) + idx);
    bf16x4_t o, g;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float uf = (float)u.v[i];
      g.v[i] = (bf16)gelu_f(uf);
      o.v[i] = (bf16)(a[i] * gelu_grad_f(uf));
    }
    if (e.gelu_out) *reinterpret_cast<bf16x4_t*>(static_cast<bf16*>(e.gelu_out) + idx) = g;
    *reinterpret_cast<bf16x4_t*>(static_cast<bf16*>(e.out) + idx) = o;
    return;
  }
  if (e.bias) {
    bf16x4_t b = *reinterpret_cast<const bf16x4_t*>(static_cast<const bf16*>(e.bias) + n);
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] += (float)b.v[i];
  }
  if (e.residual) {
    bf16x4_t r = *reinterpret_cast<const bf16x4_t*>(static_cast<const bf16*>(e.residual) + idx);
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] += (float)r.v[i];
  }
  bf16x4_t o;
#pragma unroll
  for (int i = 0; i < 4; ++i) o.v[i] = (bf16)a[i];
  *reinterpret_cast<bf16x4_t*>(static_cast<bf16*>(e.out) + idx) = o;
  if (EPI == kEpiStoreGelu) {
    bf16x4_t g;
#pragma unroll
    for (int i = 0; i < 4; ++i) g.v[i] = (bf16)gelu_f((float)o.v[i]);
    *reinterpret_cast<bf16x4_t*>(static_cast<bf16*>(e.gelu_out) + idx) = g;
  }
}

// ---- the kernel ---------------------------------------------------------------
template <int WTM, int WTN, bool TA, bool TB, int EPI>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(int K, const bf16* __restrict__ A, int lda,
                                                        const bf16* __restrict__ B, int ldb, Epilogue ep,
                                                        int tiles_m, int tiles_n) {
  constexpr int BM = 64 * WTM, BN = 64 * WTN;
  constexpr int STAGE = (BM + BN) * 128;
  extern __shared__ __align__(16) char smem[];

  // XCD-aware remap: ids equal modulo 8 share an XCD; give each XCD a contiguous run of tiles,
  // and walk the tiles in groups of 4 tile rows so that a run is compact in both dimensions.
  int n_tiles = tiles_m * tiles_n;
  int pid = blockIdx.x;
  int lin = (n_tiles % 8 == 0) ? (pid % 8) * (n_tiles / 8) + pid / 8 : pid;
  constexpr int GROUP = 4;
  int width = GROUP * tiles_n;
  int group_id = lin / width;
  int first_m = group_id * GROUP;
  int gsize = min(tiles_m - first_m, GROUP);
  int tile_m = first_m + (lin % width) % gsize;
  int tile_n = (lin % width) / gsize;

  int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int wm = wave >> 1, wn = wave & 1;
  int m0 = tile_m * BM, n0 = tile_n * BN;

  // Operand bases at (first row of the tile, k = 0).
  const bf16* a_base = TA ? A + m0 : A + (size_t)m0 * lda;  // TA: A is [K, M]
  const bf16* b_base = TB ? B + n0 : B + (size_t)n0 * ldb;  // TB: B is [K, N] (n-contiguous)

  Stager<BM, TA> sa;
  Stager<BN, TB> sb;

  f32x16 acc[WTM][WTN];
#pragma unroll
  for (int i = 0; i < WTM; ++i)
#pragma unroll
    for (int j = 0; j < WTN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  int nk = K / kBK;
  sa.load(a_base, lda, 0, tid);
  sb.load(b_base, ldb, 0, tid);
  sa.store(smem, tid);
  sb.store(smem + BM * 128, tid);
  __syncthreads();

  // Fragments of k-step 0 of the first slice.
  bf16x8 fa[2][WTM], fb[2][WTN];
  auto load_fragments = [&](const char* stage, int kk, int buf) {
    int chunk = 2 * kk + (lane >> 5);
    const char* la = stage;
    const char* lb = stage + BM * 128;
#pragma unroll
    for (int i = 0; i < WTM; ++i) fa[buf][i] = read_fragment(la, wm * (WTM * 32) + i * 32 + (lane & 31), chunk);
#pragma unroll
    for (int j = 0; j < WTN; ++j) fb[buf][j] = read_fragment(lb, wn * (WTN * 32) + j * 32 + (lane & 31), chunk);
  };
  load_fragments(smem, 0, 0);

  for (int kt = 0; kt < nk; ++kt) {
    char* cur = smem + (kt & 1) * STAGE;
    char* nxt = smem + ((kt + 1) & 1) * STAGE;
    bool more = kt + 1 < nk;
    if (more) {
      sa.load(a_base, lda, (kt + 1) * kBK, tid);
      sb.load(b_base, ldb, (kt + 1) * kBK, tid);
    }
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      // fragments of the next k-step are fetched while the matrix cores work on this one
      if (kk < 3) load_fragments(cur, kk + 1, (kk + 1) & 1);
      // the next slice goes to the other LDS buffer under the last k-step's MFMAs
      if (kk == 3 && more) {
        sa.store(nxt, tid);
        sb.store(nxt + BM * 128, tid);
      }
#pragma unroll
      for (int i = 0; i < WTM; ++i)
#pragma unroll
        for (int j = 0; j < WTN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[kk & 1][j], fa[kk & 1][i], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
    if (more) load_fragments(nxt, 0, 0);
  }

  // Accumulator layout: acc[i][j][4q + r] = C[m][n] with m = ... + (lane & 31),
  // n = ... + 8q + 4 (lane >> 5) + r.
#pragma unroll
  for (int i = 0; i < WTM; ++i) {
    int m = m0 + wm * (WTM * 32) + i * 32 + (lane & 31);
#pragma unroll
    for (int j = 0; j < WTN; ++j) {
      int nb = n0 + wn * (WTN * 32) + j * 32 + 4 * (lane >> 5);
#pragma unroll
      for (int q = 0; q < 4; ++q)
        epilogue_store4<EPI>(ep, m, nb + 8 * q, acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2],
                        acc[i][j][4 * q + 3]);
    }
  }
}

// ---- host side ------------------------------------------------------------------
static void pick_tile(int M, int N, int& wtm, int& wtn) {
  wtm = wtn = 0;
  if (M % 256 == 0 && N % 256 == 0 && (int64_t)(M / 256) * (N / 256) >= 200) {
    wtm = wtn = 4;
  } else if (M % 128 == 0 && N % 128 == 0) {
    wtm = wtn = 2;
  }
}

bool gemm_mfma_supported(int trans_a, int trans_b, int M, int N, int K, int lda, int ldb, int ldc) {
  (void)trans_a;
  (void)trans_b;
  int wtm, wtn;
  pick_tile(M, N, wtm, wtn);
  return wtm != 0 && K > 0 && K % kBK == 0 && lda % 8 == 0 && ldb % 8 == 0 && ldc % 4 == 0;
}

template <int WTM, int WTN, bool TA, bool TB, int EPI>
static bool launch_mfma_epi(int M, int N, int K, const bf16* A, int lda, const bf16* B, int ldb, const Epilogue& ep,
                            hipStream_t stream) {
  constexpr int BM = 64 * WTM, BN = 64 * WTN;
  constexpr int smem = 2 * (BM + BN) * 128;
  auto kern = gemm_mfma_kernel<WTM, WTN, TA, TB, EPI>;
  static bool configured = false;  // per instantiation
  if (!configured) {
    PO_HIP_OK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  smem));
    configured = true;
  }
  int tiles_m = M / BM, tiles_n = N / BN;
  kern<<<tiles_m * tiles_n, 256, smem, stream>>>(K, A, lda, B, ldb, ep, tiles_m, tiles_n);
  return launch_ok("gemm_mfma_kernel");
}

template <int WTM, int WTN, bool TA, bool TB>
static bool launch_mfma(int M, int N, int K, const bf16* A, int lda, const bf16* B, int ldb, const Epilogue& ep,
                        hipStream_t stream) {
  if (ep.acc_f32) return launch_mfma_epi<WTM, WTN, TA, TB, kEpiAccumulate>(M, N, K, A, lda, B, ldb, ep, stream);
  if (ep.gelu_u) return launch_mfma_epi<WTM, WTN, TA, TB, kEpiGeluBackward>(M, N, K, A, lda, B, ldb, ep, stream);
  if (ep.gelu_out) return launch_mfma_epi<WTM, WTN, TA, TB, kEpiStoreGelu>(M, N, K, A, lda, B, ldb, ep, stream);
  return launch_mfma_epi<WTM, WTN, TA, TB, kEpiStore>(M, N, K, A, lda, B, ldb, ep, stream);
}

template <int WTM, int WTN>
static bool dispatch_trans(int ta, int tb, int M, int N, int K, const bf16* A, int lda, const bf16* B, int ldb,
                           const Epilogue& ep, hipStream_t stream) {
  // kernel flag TB means "B is n-contiguous", i.e. the API's trans_b == 0
  if (!ta && !tb) return launch_mfma<WTM, WTN, false, true>(M, N, K, A, lda, B, ldb, ep, stream);
  if (!ta && tb) return launch_mfma<WTM, WTN, false, false>(M, N, K, A, lda, B, ldb, ep, stream);
  if (ta && !tb) return launch_mfma<WTM, WTN, true, true>(M, N, K, A, lda, B, ldb, ep, stream);
  return launch_mfma<WTM, WTN, true, false>(M, N, K, A, lda, B, ldb, ep, stream);
}

bool gemm_mfma_bf16(int trans_a, int trans_b, int M, int N, int K, const void* A, int lda, const void* B, int ldb,
                    const Epilogue& ep, hipStream_t stream) {
  if (!gemm_mfma_supported(trans_a, trans_b, M, N, K, lda, ldb, ep.ldc)) {
    set_error("gemm_mfma: unsupported shape M=%d N=%d K=%d lda=%d ldb=%d ldc=%d", M, N, K, lda, ldb, ep.ldc);
    return false;
  }
  int need_lda = trans_a ? M : K, need_ldb = trans_b ? K : N;
  if (lda < need_lda || ldb < need_ldb || ep.ldc < N || !A || !B || (!ep.out && !ep.acc_f32) ||
      (ep.gelu_u && !ep.out)) {
    set_error("gemm_mfma: bad operands (lda=%d ldb=%d ldc=%d)", lda, ldb, ep.ldc);
    return false;
  }
  uintptr_t al = (uintptr_t)A | (uintptr_t)B | (uintptr_t)ep.out | (uintptr_t)ep.gelu_out | (uintptr_t)ep.gelu_u |
                 (uintptr_t)ep.residual | (uintptr_t)ep.acc_f32;
  if (al % 16 != 0 || (uintptr_t)ep.bias % 8 != 0) {
    set_error("gemm_mfma: operands must be 16-byte aligned");
    return false;
  }
  int wtm, wtn;
  pick_tile(M, N, wtm, wtn);
  const bf16* a = (const bf16*)A;
  const bf16* b = (const bf16*)B;
  if (wtm == 4) return dispatch_trans<4, 4>(trans_a, trans_b, M, N, K, a, lda, b, ldb, ep, stream);
  return dispatch_trans<2, 2>(trans_a, trans_b, M, N, K, a, lda, b, ldb, ep, stream);
}

}  // namespace po
