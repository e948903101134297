// bf16 GEMM on the CDNA4 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulate.
//
// One 256-thread block (4 waves, 2 x 2) owns a (64*WTM) x (64*WTN) tile of C; a
// wave owns WTM x WTN MFMA tiles of 32 x 32, i.e. up to 128 x 128 with 256 fp32
// accumulators per lane.  K is walked in slices of 64 through a ring of LDS stages: two for the
// 256 x 256 and 256 x 192 tiles, four for the 128 x 128 tile, whose slices are too short to cover a
// memory round trip.  The 256 x 192 tile exists for outputs whose 256 x 256 tiles would leave a
// quarter of the chip idle (192 of them where 256 of the narrower ones fit).
//
// A wave is alone on its SIMD, so its one instruction stream has to keep the matrix core fed: the
// HBM -> LDS loads of a later slice, the LDS reads of the fragments three k-steps ahead and the
// MFMAs of the current k-step are woven together by hand, one load (three instructions: M0, a
// wait state, the load with a scalar base and a 32-bit lane offset) and one fragment read per two
// MFMAs, with a single barrier per slice placed where no MFMA waits for what follows it.
//
// Operand slices travel HBM -> LDS directly (global_load_lds_dwordx4: lane L of
// a wave deposits its 16 bytes at LDS base + 16 L), so no registers and no
// ds_write instructions are spent on staging.  Because the LDS side of such a
// load is fixed, the bank-conflict swizzle is applied on the global side: each
// lane fetches the 16-byte chunk that belongs at its LDS position.
//
// Two LDS layouts, chosen by how the operand lies in memory:
//   k-contiguous operand (A of forward/dgrad, B of dgrad): "row tile"
//     [rows][64] bf16, 128 bytes per row, 16-byte chunk c stored at c ^ (row & 7);
//     an MFMA fragment is one ds_read_b128.
//   operand whose contiguous index is m or n (B of forward, both of wgrad):
//     "k-major tile" [64][rows] bf16, 32-byte unit u of a row stored at
//     u ^ (k & 7) (u ^ (k & 3) when a row has 12 units); an MFMA fragment is two transposing reads (ds_read_b64_tr_b16),
//     arranged so that a lane receives k = 16 kk + 8 half + 0..7 exactly as the
//     ds_read_b128 path does, which lets the two kinds be mixed in one MFMA.
// Nothing is transposed in registers.
//
// The MFMA is issued with the B fragment in the first operand slot, so a lane holds
// four consecutive n of one row m per accumulator quad.  The epilogue moves each
// 32-row strip of a wave through LDS and then touches global memory row-wise, 16
// bytes per lane, whole 128-byte lines per row: bias, residual, GeLU, GeLU-backward
// and the fp32 accumulate all happen on that coalesced side.
//
// Workgroup ids are remapped so that the blocks that land on one XCD (ids equal
// modulo 8) work on neighbouring tiles and share operand slices in that XCD's L2.
#include <type_traits>

#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include "kernels.h"

namespace po {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

#define PO_LDS3(p) ((void __attribute__((address_space(3)))*)(p))
#define PO_GLB1(p) ((const void __attribute__((address_space(1)))*)(p))
#define PO_LDS_S16X4(p) ((s16x4 __attribute__((address_space(3)))*)(p))

constexpr int kBK = 64;

enum EpiKind : int { kEpiStore = 0, kEpiStoreGelu = 1, kEpiGeluBackward = 2, kEpiAccumulate = 3 };

// ---- HBM -> LDS, one operand slice -----------------------------------------------
// KMAJOR == false: operand is [R rows][K], slice = R rows x 64 k, row tile in LDS.
// KMAJOR == true : operand is [K][R], slice = 64 k x R, k-major tile in LDS.
// Swizzle of the k-major tile: row k keeps unit u at position u ^ (k & mask).  The position must stay inside
// the row, so a row of 12 units (R = 192) swaps only within groups of four; the fragment reads of four
// consecutive k and two neighbouring units still fall into eight different 32-byte bank groups.
template <int R>
__device__ __forceinline__ int kmajor_unit(int u, int k) {
  static_assert(R % 64 == 0, "rows of the k-major tile are whole groups of four units");
  constexpr int MASK = (R % 128 == 0) ? 7 : 3;
  return u ^ (k & MASK);
}

// Byte address of a pointer into the block's LDS as the hardware counts it (the generic -> LDS conversion and
// its null check happen here, once, instead of at every load).
__device__ __forceinline__ unsigned lds_address(const void* p) { return (unsigned)(size_t)PO_LDS3(p); }

// The slice is R * 128 bytes = R / 8 wave-wide loads of 1 KiB; wave w issues pieces w, w + 4, w + 8, ...
// What a lane fetches for piece u never changes from slice to slice except for a step that is the same for every
// lane, so the lane keeps one 32-bit byte offset per piece and the wave one 64-bit slice pointer in scalar
// registers: a load costs its own instruction and the M0 set-up, no address arithmetic.
template <int R, bool KMAJOR>
struct SliceLoader {
  static constexpr int N_INST = R * 128 / 1024;
  static constexpr int PER_WAVE = N_INST / 4;
  static_assert(N_INST % 4 == 0 && PER_WAVE >= 4, "tile too small for four waves");
  unsigned voff[PER_WAVE];  // this lane's byte offset from the slice pointer, per piece
  const char* slice;        // first byte of the next slice to request (same in every lane)
  unsigned step;            // bytes from one slice to the next

  // `base` points at (first row of the tile, k = 0).
  __device__ __forceinline__ void init(const bf16* base, int ld, int wave, int lane) {
#pragma unroll
    for (int u = 0; u < PER_WAVE; ++u) {
      int g = u * 4 + wave;  // which 1 KiB piece of the tile
      unsigned elem;
      if (!KMAJOR) {
        int row = 8 * g + (lane >> 3);
        int c = (lane & 7) ^ (row & 7);
        elem = (unsigned)row * (unsigned)ld + c * 8;
      } else {
        constexpr int ROW_BYTES = 2 * R;
        int byte = g * 1024 + lane * 16;
        int k = byte / ROW_BYTES;
        int pos16 = (byte % ROW_BYTES) >> 4;
        int unit = kmajor_unit<R>(pos16 >> 1, k);
        elem = (unsigned)k * (unsigned)ld + (unit * 2 + (pos16 & 1)) * 8;
      }
      voff[u] = elem * 2;
    }
    slice = reinterpret_cast<const char*>(base);
    step = KMAJOR ? 128u * (unsigned)ld : 128u;
  }
  // Piece u of the slice at `slice` -> LDS at lds_wave + 4096 u (lds_wave: the LDS address of this wave's piece 0
  // in the target stage).  Issued as inline assembly on purpose: through the builtin the compiler treats every
  // later LDS read as dependent on the load and waits for it at once, which would undo the double buffering.
  // The caller waits (wait_slice_loads) before the barrier that publishes the slice.
  __device__ __forceinline__ void issue(int u, unsigned lds_wave) const {
    unsigned dst = lds_wave + 4096u * u;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(dst), "v"(voff[u]), "s"(slice)
                 : "memory");
  }
  __device__ __forceinline__ void advance() { slice += step; }
};

// Waits until at most N of this wave's loads are outstanding (they complete in issue order).
template <int N>
__device__ __forceinline__ void wait_slice_loads() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// ---- LDS -> MFMA fragment: 32 rows (row0 + lane % 32), k = 16 kk + 8 (lane / 32) + 0..7 ----
template <int R, bool KMAJOR>
__device__ __forceinline__ bf16x8 read_fragment(const char* lds, int row0, int kk, int lane) {
  if (!KMAJOR) {
    int row = row0 + (lane & 31);
    int c = (2 * kk + (lane >> 5)) ^ (row & 7);
    return *reinterpret_cast<const bf16x8*>(lds + row * 128 + (c << 4));
  } else {
    // Transposing read: within a group of 16 lanes, lane i receives element (i % 4) of the
    // addresses supplied by lanes i / 4, 4 + i / 4, 8 + i / 4, 12 + i / 4.  Lane r of the group
    // supplies row k = kbase + r / 4, columns m0 + 4 (r % 4) .. + 3; lane i then holds
    // k = kbase .. kbase + 3 of column m0 + i.
    constexpr int ROW_BYTES = 2 * R;
    int i = lane & 15, grp = lane >> 4;
    int m = row0 + 16 * (grp & 1) + 4 * (i & 3);
    int k = 16 * kk + 8 * (grp >> 1) + (i >> 2);
    int unit = m >> 4;
    int inner = (m & 15) * 2;
    const char* p0 = lds + k * ROW_BYTES + (kmajor_unit<R>(unit, k) << 5) + inner;
    const char* p1 = lds + (k + 4) * ROW_BYTES + (kmajor_unit<R>(unit, k + 4) << 5) + inner;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(PO_LDS_S16X4(p0));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(PO_LDS_S16X4(p1));
    union {
      struct {
        s16x4 a, b;
      } s;
      bf16x8 v;
    } u;
    u.s.a = lo;
    u.s.b = hi;
    return u.v;
  }
}

// ---- epilogue on one row-contiguous piece ----------------------------------------
// v[0..N) are consecutive n of row m starting at n.  bf16 kinds use N = 8 (16-byte accesses),
// the fp32 accumulate uses N = 4.
struct __attribute__((aligned(16))) bf16x8_t {
  bf16 v[8];
};

// `aux` is the piece of the auxiliary operand at the same place, loaded by the caller ahead of time:
// u for the GeLU backward kind, the residual (if any) for the store kinds.
template <int EPI>
__device__ __forceinline__ void epilogue_row_piece(const Epilogue& e, int m, int n, const float* v,
                                                   const bf16x8_t& aux) {
  size_t idx = (size_t)m * e.ldc + n;
  float a[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] = v[i];
  if (EPI == kEpiGeluBackward) {
    const bf16x8_t& u = aux;
    bf16x8_t o, g;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float gf, dgf;
      gelu_and_grad_f((float)u.v[i], gf, dgf);
      g.v[i] = (bf16)gf;
      o.v[i] = (bf16)(a[i] * dgf);
    }
    if (e.gelu_out) *reinterpret_cast<bf16x8_t*>(static_cast<bf16*>(e.gelu_out) + idx) = g;
    *reinterpret_cast<bf16x8_t*>(static_cast<bf16*>(e.out) + idx) = o;
    return;
  }
  if (e.bias) {
    bf16x8_t b = *reinterpret_cast<const bf16x8_t*>(static_cast<const bf16*>(e.bias) + n);
#pragma unroll
    for (int i = 0; i < 8; ++i) a[i] += (float)b.v[i];
  }
  if (e.residual) {
#pragma unroll
    for (int i = 0; i < 8; ++i) a[i] += (float)aux.v[i];
  }
  bf16x8_t o;
#pragma unroll
  for (int i = 0; i < 8; ++i) o.v[i] = (bf16)a[i];
  *reinterpret_cast<bf16x8_t*>(static_cast<bf16*>(e.out) + idx) = o;
  if (EPI == kEpiStoreGelu) {
    bf16x8_t g;
#pragma unroll
    for (int i = 0; i < 8; ++i) g.v[i] = (bf16)gelu_f((float)o.v[i]);
    *reinterpret_cast<bf16x8_t*>(static_cast<bf16*>(e.gelu_out) + idx) = g;
  }
}

// LDS stages of a tile: what fits into 160 KiB at (BM + BN) * 128 bytes per stage.
constexpr int stages_of(int wtm, int wtn) { return wtm * wtn >= 12 ? 2 : 4; }

// Tiles are walked in groups of 4 tile rows, so that a run of consecutive tile numbers is compact in both
// dimensions (the blocks of one XCD take such a run and share operand slices in that XCD's L2).
__device__ __forceinline__ void tile_of(int lin, int tiles_m, int tiles_n, int& tile_m, int& tile_n) {
  constexpr int GROUP = 4;
  int width = GROUP * tiles_n;
  int group_id = lin / width;
  int first_m = group_id * GROUP;
  int gsize = min(tiles_m - first_m, GROUP);
  tile_m = first_m + (lin % width) % gsize;
  tile_n = (lin % width) / gsize;
}

// Tells the compiler that a value is the same in every lane (it is: it derives from the block id and the kernel
// arguments only), so that it stays in scalar registers.
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ const bf16* uniform(const bf16* p) {
  uintptr_t v = reinterpret_cast<uintptr_t>(p);
  unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v), hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return reinterpret_cast<const bf16*>(((uintptr_t)hi << 32) | lo);
}

// ---- one output tile -----------------------------------------------------------
// TA: A is [K, M] (m-contiguous).  TB: B is [K, N] (n-contiguous).  All 256 threads of the block call it with
// the same arguments; `smem` is the block's dynamic LDS (stages, then reused by the epilogue strips).
template <int WTM, int WTN, bool TA, bool TB, int EPI>
__device__ __forceinline__ void gemm_tile(int K, const bf16* __restrict__ A, int lda, const bf16* __restrict__ B,
                                          int ldb, const Epilogue& ep, int tile_m, int tile_n, char* smem) {
  constexpr int BM = 64 * WTM, BN = 64 * WTN;
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128;
  constexpr int STAGE = A_BYTES + B_BYTES;

  int tid = threadIdx.x, lane = tid & 63;
  int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  int wm = wave >> 1, wn = wave & 1;
  int m0 = tile_m * BM, n0 = tile_n * BN;

  const bf16* a_base = TA ? A + m0 : A + (size_t)m0 * lda;
  const bf16* b_base = TB ? B + n0 : B + (size_t)n0 * ldb;

  f32x16 acc[WTM][WTN];
#pragma unroll
  for (int i = 0; i < WTM; ++i)
#pragma unroll
    for (int j = 0; j < WTN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // Pipeline.  Three streams feed the MFMAs, each running ahead of them by a fixed distance:
  //   HBM -> LDS   slice kt + NSTAGE is requested during slice kt, into the stage slice kt occupies, from the
  //                moment every wave is done reading it (the barrier below);
  //   LDS -> regs  the fragments of a k-step are read three k-steps (most of a slice) before their MFMAs, into a
  //                ring of four register buffers, so an LDS round trip is never waited for;
  //   barrier      one per slice, before k-step 1: it publishes slice kt + 1 (whose first fragments are read
  //                from k-step 1 on) and releases stage kt % NSTAGE (whose last fragments were read in k-step 0).
  // The big tiles have room for two stages, the small tile (a slice is four times shorter) gets four.
  constexpr int NSTAGE = stages_of(WTM, WTN);
  using LoaderA = SliceLoader<BM, TA>;
  using LoaderB = SliceLoader<BN, TB>;
  constexpr int PER_SLICE = LoaderA::PER_WAVE + LoaderB::PER_WAVE;  // load instructions of one wave per slice
  int nk = K / kBK;
  LoaderA la;
  LoaderB lb;
  la.init(a_base, lda, wave, lane);
  lb.init(b_base, ldb, wave, lane);
  const unsigned lds0 = uniform((int)lds_address(smem)) + 1024u * wave;  // this wave's piece 0 of stage 0, operand A
  // Load q (0 .. PER_SLICE - 1, A's pieces first) of the slice the loaders point at, into stage `st`.
  auto issue_load = [&](int q, unsigned st) {
    unsigned base = lds0 + st * STAGE;
    if (q < LoaderA::PER_WAVE) la.issue(q, base);
    else lb.issue(q - LoaderA::PER_WAVE, base + A_BYTES);
  };
  auto next_slice = [&]() {
    la.advance();
    lb.advance();
  };
#ifdef PO_PHASE_TIMING  // measurement build only (gemm_phases.py): cycle counts of the three phases of tile (0, 0)
  const long long tim0 = __builtin_readcyclecounter(), wal0 = wall_clock64();
#endif
  {
    int ahead = min(nk, NSTAGE);
    for (int t = 0; t < ahead; ++t) {
#pragma unroll
      for (int q = 0; q < PER_SLICE; ++q) issue_load(q, t);
      next_slice();
    }
    // slice 0 has landed when at most ahead - 1 slices are still in flight
    if (ahead >= 4) wait_slice_loads<3 * PER_SLICE>();
    else if (ahead == 3) wait_slice_loads<2 * PER_SLICE>();
    else if (ahead == 2) wait_slice_loads<PER_SLICE>();
    else wait_slice_loads<0>();
  }
  __syncthreads();
#ifdef PO_PHASE_TIMING
  const long long tim1 = __builtin_readcyclecounter();
#endif

  bf16x8 fa[4][WTM], fb[4][WTN];
  // Fragments are fetched in the order a0 b0 a1 b1 ... and the MFMAs of a k-step walk the
  // (i, j) grid as a growing square, so the first MFMAs need only the first fragments fetched
  // and the fragment fetched last is needed last.
  constexpr int NFRAG = WTM + WTN;
  auto load_fragment = [&](const char* stage, int kk, int r) {  // r-th fragment of k-step kk, into buffer kk
    // (with WTM != WTN the longer operand's surplus fragments come last)
    constexpr int PAIRS = WTM < WTN ? WTM : WTN;
    bool is_a;
    int t;
    if (r < 2 * PAIRS) {
      is_a = (r & 1) == 0;
      t = r >> 1;
    } else {
      is_a = WTM > WTN;
      t = PAIRS + (r - 2 * PAIRS);
    }
    if (is_a) fa[kk][t] = read_fragment<BM, TA>(stage, wm * (WTM * 32) + t * 32, kk, lane);
    else fb[kk][t] = read_fragment<BN, TB>(stage + A_BYTES, wn * (WTN * 32) + t * 32, kk, lane);
  };
#pragma unroll
  for (int kk = 0; kk < 3; ++kk)
#pragma unroll
    for (int r = 0; r < NFRAG; ++r) load_fragment(smem, kk, r);

  // One slice: MFMAs on the fragments of stage kt % NSTAGE.  ISSUE: slice kt + NSTAGE is requested meanwhile.
  // MORE: a slice follows.  The tail slices are peeled off so that the steady-state loop body has no branches.
  //
  // Inside a k-step the three instruction streams are woven by hand, and scheduling barriers keep the compiler
  // from undoing it: behind every few MFMAs one LDS fragment read and, in k-steps 1 .. kLoadSteps, one
  // HBM -> LDS load.  A wave has a single MFMA pipe to keep busy and no other wave on its SIMD to fill in, so
  // anything issued in a clump (sixteen loads with their scalar set-up back to back) is time the matrix core
  // stands still.
  constexpr int NMFMA = WTM * WTN;
  constexpr int kLoadSteps = NSTAGE == 4 ? 3 : 2;  // measured: the small tile's eight loads spread thinner
  constexpr int LOADS_PER_STEP = (PER_SLICE + kLoadSteps - 1) / kLoadSteps;
  auto slice = [&](int kt, auto issue_tag, auto more_tag) {
    constexpr bool ISSUE = decltype(issue_tag)::value;
    constexpr bool MORE = decltype(more_tag)::value;
    unsigned st_cur = (unsigned)(kt % NSTAGE);
    char* cur = smem + st_cur * STAGE;
    char* nxt = smem + ((kt + 1) % NSTAGE) * STAGE;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      if (MORE && kk == 1) {
        // slice kt + 1 complete (in steady state NSTAGE - 2 younger slices may stay in flight; the tail slices
        // simply wait for everything), own reads of stage kt % NSTAGE complete, then the barrier
        wait_slice_loads<(ISSUE ? NSTAGE - 2 : 0) * PER_SLICE>();
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
      }
      int n = 0;  // MFMAs issued in this k-step
      auto after_mfma = [&]() {
        ++n;
        // the share of the other two streams that belongs behind MFMA n of NMFMA
        bool any = false;
        if (kk == 0) {
          // the last reads of this stage: all in the first half of the k-step, so that they have come back
          // when the wave waits for them at the barrier
#pragma unroll
          for (int r = (n - 1) * NFRAG * 2 / NMFMA; r < n * NFRAG * 2 / NMFMA; ++r)
            if (r < NFRAG) {
              load_fragment(cur, 3, r);
              any = true;
            }
        } else if (MORE) {
#pragma unroll
          for (int r = (n - 1) * NFRAG / NMFMA; r < n * NFRAG / NMFMA; ++r) {
            load_fragment(nxt, kk - 1, r);
            any = true;
          }
        }
        if (ISSUE && kk >= 1 && kk <= kLoadSteps) {
#pragma unroll
          for (int q = (n - 1) * LOADS_PER_STEP / NMFMA; q < n * LOADS_PER_STEP / NMFMA; ++q) {
            int ql = (kk - 1) * LOADS_PER_STEP + q;
            if (ql < PER_SLICE) {
              issue_load(ql, st_cur);
              any = true;
            }
          }
        }
        if (any) __builtin_amdgcn_sched_barrier(0);
      };
#pragma unroll
      for (int t = 0; t < (WTM > WTN ? WTM : WTN); ++t) {  // ring t of the growing square
#pragma unroll
        for (int j = 0; j < t && j < WTN; ++j)
          if (t < WTM) {
            acc[t][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[kk][j], fa[kk][t], acc[t][j], 0, 0, 0);
            after_mfma();
          }
#pragma unroll
        for (int i = 0; i <= t && i < WTM; ++i)
          if (t < WTN) {
            acc[i][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[kk][t], fa[kk][i], acc[i][t], 0, 0, 0);
            after_mfma();
          }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if (ISSUE) next_slice();
  };
  {
    using T = std::true_type;
    using F = std::false_type;
    int kt = 0;
    for (; kt + NSTAGE < nk; ++kt) slice(kt, T{}, T{});
    for (; kt + 1 < nk; ++kt) slice(kt, F{}, T{});  // nothing left to request
    slice(nk - 1, F{}, F{});
  }
  __syncthreads();  // the epilogue strips reuse the operand stages
#ifdef PO_PHASE_TIMING
  const long long tim2 = __builtin_readcyclecounter();
#endif

  // Epilogue.  acc[i][j][4q + r] = C[m][n], m = strip row (lane & 31), n = 32 j + 8 q + 4 (lane >> 5) + r.
  // Each wave owns a private [32][WTN*32 + 4] fp32 strip in LDS (the operand buffers are free now).
  constexpr int STRIP_N = WTN * 32;
  constexpr int STRIP_LD = STRIP_N + 4;  // floats; the 16-byte pad staggers rows over the banks
  float* strip = reinterpret_cast<float*>(smem) + wave * (32 * STRIP_LD);
  int col = lane & 31, half = lane >> 5;
#pragma unroll
  for (int i = 0; i < WTM; ++i) {
#pragma unroll
    for (int j = 0; j < WTN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        f32x4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
        *reinterpret_cast<f32x4*>(strip + col * STRIP_LD + 32 * j + 8 * q + 4 * half) = v;
      }
    // (a wave reads back only what it wrote itself: program order is enough, no barrier)
    int mrow0 = m0 + wm * (WTM * 32) + i * 32;
    int ncol0 = n0 + wn * STRIP_N;
    if (EPI == kEpiAccumulate) {
      // fp32 read-modify-write of the strip: all loads of the old values are issued before the first
      // add, so that a wave keeps 16 KiB in flight instead of one access at a time.
      constexpr int LPR = STRIP_N / 4;       // lanes per row, 4 floats each
      constexpr int NIT = 32 * LPR / 64;     // wave-wide accesses per strip; piece it * 64 + lane of the strip
      static_assert(32 * LPR % 64 == 0, "strip is a whole number of wave-wide accesses");
      f32x4 old[NIT];
      float* cbase = ep.acc_f32 + (size_t)mrow0 * ep.ldc + ncol0;
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        int piece = it * 64 + lane;
        old[it] = *reinterpret_cast<const f32x4*>(cbase + (size_t)(piece / LPR) * ep.ldc + (piece % LPR) * 4);
      }
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        int piece = it * 64 + lane;
        int r = piece / LPR;
        int c = (piece % LPR) * 4;
        f32x4 v = *reinterpret_cast<const f32x4*>(strip + r * STRIP_LD + c);
        *reinterpret_cast<f32x4*>(cbase + (size_t)r * ep.ldc + c) = old[it] + v;
      }
    } else {
      constexpr int LPR = STRIP_N / 8;  // lanes per row, 8 values each
      constexpr int NIT = 32 * LPR / 64;
      static_assert(32 * LPR % 64 == 0, "strip is a whole number of wave-wide accesses");
      // the strip's pieces of u (GeLU backward) or of the residual are all requested before the first use
      bf16x8_t aux[NIT];
      const bf16* aux_src = EPI == kEpiGeluBackward ? static_cast<const bf16*>(ep.gelu_u)
                                                    : static_cast<const bf16*>(ep.residual);
      if (aux_src) {
        const bf16* abase = aux_src + (size_t)mrow0 * ep.ldc + ncol0;
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
          int piece = it * 64 + lane;
          aux[it] = *reinterpret_cast<const bf16x8_t*>(abase + (size_t)(piece / LPR) * ep.ldc + (piece % LPR) * 8);
        }
      }
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        int piece = it * 64 + lane;
        int r = piece / LPR;
        int c = (piece % LPR) * 8;
        f32x4 v0 = *reinterpret_cast<const f32x4*>(strip + r * STRIP_LD + c);
        f32x4 v1 = *reinterpret_cast<const f32x4*>(strip + r * STRIP_LD + c + 4);
        float vv[8] = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
        epilogue_row_piece<EPI>(ep, mrow0 + r, ncol0 + c, vv, aux[it]);
      }
    }
  }
#ifdef PO_PHASE_TIMING  // overwrites the first 16 bytes of the result: prologue, main loop, epilogue cycles, cycles per 10 ns
  __syncthreads();
  if (tile_m == 0 && tile_n == 0 && threadIdx.x == 0 && ep.out) {
    const long long tim3 = __builtin_readcyclecounter();
    float* dbg = reinterpret_cast<float*>(ep.out);
    dbg[0] = (float)(tim1 - tim0); dbg[1] = (float)(tim2 - tim1); dbg[2] = (float)(tim3 - tim2);
    dbg[3] = (float)(tim3 - tim0) / (float)(wall_clock64() - wal0);
  }
#endif
}

// ---- the kernels -----------------------------------------------------------------
// One tile per block.  XCD-aware remap: ids equal modulo 8 share an XCD; each XCD gets a contiguous run of tiles.
template <int WTM, int WTN, bool TA, bool TB, int EPI>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(int K, const bf16* __restrict__ A, int lda,
                                                        const bf16* __restrict__ B, int ldb, Epilogue ep,
                                                        int tiles_m, int tiles_n) {
  extern __shared__ __align__(16) char smem[];
  int n_tiles = tiles_m * tiles_n;
  int pid = blockIdx.x;
  int lin = (n_tiles % 8 == 0) ? (pid % 8) * (n_tiles / 8) + pid / 8 : pid;
  int tile_m, tile_n;
  tile_of(lin, tiles_m, tiles_n, tile_m, tile_n);
  gemm_tile<WTM, WTN, TA, TB, EPI>(K, A, lda, B, ldb, ep, tile_m, tile_n, smem);
}

// Several independent GEMMs of one form in one launch: the 256 x 256 tiles of all problems are numbered one
// problem after the other and the blocks (at most one per CU) take them round by round, so that a round is full
// as long as tiles are left, whatever the shape of a single problem (a 2048 x 2048 result alone has 64 tiles,
// a 2048 x 6144 one 192), and a block's epilogue no longer marks the end of a launch.
constexpr int kMaxGroupedGemms = 4;
struct GroupedProblem {
  const bf16* A;
  const bf16* B;
  Epilogue ep;
  int K, lda, ldb, tiles_m, tiles_n, first_tile;
};
struct GroupedArgs {
  GroupedProblem p[kMaxGroupedGemms];
  int n, total_tiles;
};

template <bool TA, bool TB, int EPI>
__global__ __launch_bounds__(256) void gemm_mfma_grouped_kernel(GroupedArgs g) {
  extern __shared__ __align__(16) char smem[];
  int pid = blockIdx.x, nb = gridDim.x;
  int slot = (nb % 8 == 0) ? (pid % 8) * (nb / 8) + pid / 8 : pid;  // an XCD's blocks take a run of tile numbers
  for (int base = 0; base < g.total_tiles; base += nb) {
    int lin = base + slot;
    if (lin < g.total_tiles) {  // the same for every thread of the block
      // The problem that owns tile `lin`, picked with constant indices only: a run-time index into the argument
      // block would send it through private memory and the compiler would no longer know that K, the strides
      // and the LDS addresses derived from them are the same in every lane.
      GroupedProblem P = g.p[0];
#pragma unroll
      for (int i = 1; i < kMaxGroupedGemms; ++i)
        if (i < g.n && lin >= g.p[i].first_tile) P = g.p[i];
      int tile_m, tile_n;
      tile_of(lin - P.first_tile, P.tiles_m, P.tiles_n, tile_m, tile_n);
      gemm_tile<4, 4, TA, TB, EPI>(uniform(P.K), uniform(P.A), uniform(P.lda), uniform(P.B), uniform(P.ldb), P.ep,
                                   uniform(tile_m), uniform(tile_n), smem);
    }
    __syncthreads();  // the next tile's operand loads overwrite the epilogue strips of every wave
  }
}

// ---- host side ------------------------------------------------------------------
// 256 x 256 tiles once they fill three quarters of the 256 CUs in one round (measured: 192 big tiles beat 768
// small ones, 58 against 63 us at M = 2048, N = 6144, K = 2048); below that the 128 x 128 tile.  Where N is a
// multiple of 192 the 256 x 192 tile takes over when its rounds cost less: a round is as long as its slowest
// block, so 256 narrower tiles in one round beat 192 big ones with a quarter of the CUs idle, and 512 in two
// rounds beat 384 big ones (a narrow tile's round takes about 0.8 of a big tile's: 3/4 of the flops at
// slightly more operand bytes per flop).
static int tile_threshold() { return 192; }
static int64_t rounds(int64_t tiles) { return (tiles + 255) / 256; }
static void pick_tile(int M, int N, int& wtm, int& wtn) {
  wtm = wtn = 0;
  if (M % 256 == 0 && N % 256 == 0 && (int64_t)(M / 256) * (N / 256) >= tile_threshold()) {
    wtm = wtn = 4;
  } else if (M % 128 == 0 && N % 128 == 0) {
    wtm = wtn = 2;
  }
  if (M % 256 == 0 && N % 192 == 0 && (int64_t)(M / 256) * (N / 192) >= tile_threshold()) {
    int64_t narrow = 8 * rounds((int64_t)(M / 256) * (N / 192));  // in tenths of a big tile's round
    int64_t other = wtm == 4 ? 10 * rounds((int64_t)(M / 256) * (N / 256))
                             : (wtm == 2 ? 4 * rounds((int64_t)(M / 128) * (N / 128)) : INT64_MAX);
    if (narrow < other) {
      wtm = 4;
      wtn = 3;
    }
  }
}

void gemm_mfma_tile(int M, int N, int* bm, int* bn) {
  int wtm = 0, wtn = 0;
  if (M > 0 && N > 0) pick_tile(M, N, wtm, wtn);
  *bm = 64 * wtm;
  *bn = 64 * wtn;
}

bool gemm_mfma_supported(int trans_a, int trans_b, int M, int N, int K, int lda, int ldb, int ldc) {
  (void)trans_a;
  (void)trans_b;
  int wtm, wtn;
  pick_tile(M, N, wtm, wtn);
  return wtm != 0 && K > 0 && K % kBK == 0 && lda % 8 == 0 && ldb % 8 == 0 && ldc % 8 == 0;
}

template <int WTM, int WTN, bool TA, bool TB, int EPI>
static bool launch_mfma_epi(int M, int N, int K, const bf16* A, int lda, const bf16* B, int ldb, const Epilogue& ep,
                            hipStream_t stream) {
  constexpr int BM = 64 * WTM, BN = 64 * WTN;
  constexpr int smem_ops = stages_of(WTM, WTN) * (BM + BN) * 128;
  constexpr int smem_epi = 4 * 32 * (WTN * 32 + 4) * 4;
  constexpr int smem = smem_ops > smem_epi ? smem_ops : smem_epi;
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
                 (uintptr_t)ep.residual | (uintptr_t)ep.acc_f32 | (uintptr_t)ep.bias;
  if (al % 16 != 0) {
    set_error("gemm_mfma: operands must be 16-byte aligned");
    return false;
  }
  int wtm, wtn;
  pick_tile(M, N, wtm, wtn);
  const bf16* a = (const bf16*)A;
  const bf16* b = (const bf16*)B;
  if (wtm == 4 && wtn == 3) return dispatch_trans<4, 3>(trans_a, trans_b, M, N, K, a, lda, b, ldb, ep, stream);
  if (wtm == 4) return dispatch_trans<4, 4>(trans_a, trans_b, M, N, K, a, lda, b, ldb, ep, stream);
  return dispatch_trans<2, 2>(trans_a, trans_b, M, N, K, a, lda, b, ldb, ep, stream);
}

// ---- grouped launch ---------------------------------------------------------------
bool gemm_mfma_grouped_supported(int n, const GemmProblem* p) {
  if (n < 1 || n > kMaxGroupedGemms || !p) return false;
  for (int i = 0; i < n; ++i) {
    const GemmProblem& q = p[i];
    if (q.M <= 0 || q.N <= 0 || q.K <= 0 || q.M % 256 != 0 || q.N % 256 != 0 || q.K % kBK != 0 || q.lda % 8 != 0 ||
        q.ldb % 8 != 0 || q.ldc % 8 != 0 || q.lda < q.M || q.ldb < q.N || q.ldc < q.N || !q.A || !q.B || !q.acc_f32 ||
        ((uintptr_t)q.A | (uintptr_t)q.B | (uintptr_t)q.acc_f32) % 16 != 0)
      return false;
  }
  return true;
}

bool gemm_mfma_grouped_accumulate(int n, const GemmProblem* p, hipStream_t stream) {
  if (!gemm_mfma_grouped_supported(n, p)) {
    set_error("gemm_mfma_grouped: %d problems, or a shape, stride or pointer the grouped kernel does not take", n);
    return false;
  }
  GroupedArgs g;
  memset(&g, 0, sizeof(g));
  g.n = n;
  int total = 0;
  for (int i = 0; i < n; ++i) {
    GroupedProblem& q = g.p[i];
    q.A = static_cast<const bf16*>(p[i].A);
    q.B = static_cast<const bf16*>(p[i].B);
    q.ep.acc_f32 = p[i].acc_f32;
    q.ep.ldc = p[i].ldc;
    q.K = p[i].K;
    q.lda = p[i].lda;
    q.ldb = p[i].ldb;
    q.tiles_m = p[i].M / 256;
    q.tiles_n = p[i].N / 256;
    q.first_tile = total;
    total += q.tiles_m * q.tiles_n;
  }
  g.total_tiles = total;
  constexpr int smem = stages_of(4, 4) * (256 + 256) * 128;
  auto kern = gemm_mfma_grouped_kernel<true, true, kEpiAccumulate>;
  static bool configured = false;
  if (!configured) {
    PO_HIP_OK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  smem));
    configured = true;
  }
  int blocks = total < 256 ? total : 256;  // one block per CU; more tiles mean more rounds per block
  kern<<<blocks, 256, smem, stream>>>(g);
  return launch_ok("gemm_mfma_grouped_kernel");
}

}  // namespace po
