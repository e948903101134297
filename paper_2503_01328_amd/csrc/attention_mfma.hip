// bf16 causal attention on the CDNA4 matrix cores, forward and backward, with
// online softmax (no s x s matrix is ever stored; the forward keeps the
// per-row log-sum-exp, the backward recomputes the probabilities from it).
//
// Layout idea shared by all three kernels.  A 32 x 32 MFMA leaves lane L with
// column (L % 32) of the result and 16 of its rows.  The kernels always put the
// index a wave OWNS (its query rows in forward and dQ, its key rows in dK/dV)
// on the MFMA column, so that
//   * softmax statistics of a query row live in one lane (plus its partner
//     L ^ 32): row max / row sum need no cross-lane tree,
//   * a probability tile converted to bf16 is already laid out as the B operand
//     of the next MFMA (k index = the 8 rows a lane holds per 16-deep step), so
//     P and dS never travel through LDS,
//   * the other operand of that next MFMA (V, dO, Q or K as [row][dh], i.e. with
//     the contraction index as the slow dimension) is fetched with the gfx950
//     transposing LDS read (ds_read_b64_tr_b16), two per fragment.
//
// Forward: a block is eight compute waves, each owning 32 query rows, plus one wave that only loads; K/V
// tiles of 64 keys are staged through LDS (loaded HBM -> LDS directly, rings of two or three stages).
// Blocks with the most key tiles are launched first, over all heads (causal work is triangular).
//
// Backward, deterministic without atomics: one kernel per key block accumulates
// dK and dV over the query tiles at or below the diagonal; one kernel per query
// block accumulates dQ over the key tiles up to the diagonal.  Both recompute
// S = Q K^T and dP = dO V^T.
#include <math.h>

#include <type_traits>

#include "kernels.h"

namespace po {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

#define LDS_AS3(p) ((s16x4 __attribute__((address_space(3)))*)(p))

constexpr int kKeysPerTile = 64;

// ---- LDS tile --------------------------------------------------------------------
// [64 rows][DH] bf16, unpadded: the 16-byte chunk c of row r sits at chunk position c ^ swz(r).
// One tile serves both kinds of MFMA operand reads without bank conflicts:
//  * ds_read_b128 "row" fragments (contraction over the head dimension): 16 lanes read the same
//    chunk of 16 consecutive rows; swz is a bijection of those rows onto the 16 chunk positions
//    of a 256-byte bank line (for DH = 64 two rows share a line and the row parity picks the half);
//  * transposing reads (contraction over the tile's rows): a half-wave reads 64 contiguous bytes
//    of four consecutive rows; swz sends them to the four different 64-byte quarters of a line.
template <int DH>
__device__ __forceinline__ int swz(int r) {
  if (DH == 128) return ((r & 3) << 2) | ((r >> 2) & 3);
  return (((r >> 1) & 1) << 2) | ((r >> 2) & 3);
}
template <int DH>
__device__ __forceinline__ int tile_offset(int row, int chunk) {
  return row * (DH * 2) + ((chunk ^ swz<DH>(row)) << 4);
}
template <int DH> constexpr int tile_bytes() { return kKeysPerTile * DH * 2; }

// HBM -> LDS without a register stop: a wave-level global_load_lds_dwordx4 writes 1 KiB of the tile
// (lane L fills bytes 16 L ..), so each lane fetches the chunk that belongs at its position.  The block's
// WAVES waves issue tile_bytes / (1024 WAVES) loads each; between two loads of a wave the source advances by a
// whole number of rows that is a multiple of 16, which leaves swz unchanged: the per-lane part of the
// address is one 32-bit byte offset (tile_lane_offset, computed once per kernel) and everything else
// is wave-uniform scalar arithmetic.  `base` points at (row 0, first element of the head), rows are
// `ld` elements apart; base, row0 and wave must be wave-uniform.
// Inline assembly on purpose: through the builtin the compiler waits for the load before every
// later LDS read, which would undo the double buffering.  Callers wait (wait_tile_loads) before
// the barrier that publishes the tile.
template <int DH>
__device__ __forceinline__ unsigned tile_lane_offset(int ld, int wave, int lane) {
  constexpr int ROW_BYTES = DH * 2;
  int byte = wave * 1024 + lane * 16;
  int row = byte / ROW_BYTES;
  int c = ((byte % ROW_BYTES) >> 4) ^ swz<DH>(row);
  return (unsigned)((row * ld + c * 8) * 2);
}
template <int DH, int WAVES = 4>
__device__ __forceinline__ void load_tile_async(const bf16* __restrict__ base, int ld, int row0, char* tile,
                                                int wave, unsigned lane_offset) {
  constexpr int PER_WAVE = tile_bytes<DH>() / (1024 * WAVES);
  constexpr int ROWS_PER_LOAD = 1024 * WAVES / (DH * 2);  // rows the WAVES waves cover with one load each
  static_assert(ROWS_PER_LOAD % 16 == 0, "swz must not change between the loads of a lane");
#pragma unroll
  for (int u = 0; u < PER_WAVE; ++u) {
    const bf16* src = base + (size_t)(row0 + u * ROWS_PER_LOAD) * ld;
    unsigned lds_addr =
        (unsigned)(size_t)((void __attribute__((address_space(3)))*)(tile + (u * WAVES + wave) * 1024));
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr),
                 "v"(lane_offset), "s"(src)
                 : "memory");
  }
}
// Through the builtin, not inline assembly: the compiler keeps its own count of outstanding loads and cannot see
// into assembly text.  Left believing that a kernel's early register loads (Q, K or V fragments) might still be
// in flight, it guards their every use inside the tile loop with s_waitcnt vmcnt(n), and since the counter is
// shared those waits really wait for the tile loads issued a moment before: the prefetch would be waited for
// at once.  A wait it can see resets its count.
__device__ __forceinline__ void wait_tile_loads() {
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0), the other counters left alone (expcnt 7, lgkmcnt 15)
  asm volatile("" ::: "memory");
}
// The same wait as text the compiler does not look into.  The dK/dV kernels use it: they sit at the register limit
// of two waves per SIMD, their extra waits cost nothing measurable, and the different schedule the visible wait
// gives the compiler makes it spill.
__device__ __forceinline__ void wait_tile_loads_opaque() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Fragment whose contraction index is the tile's row: lane (column c = lane % 32 of the
// 32-wide block starting at col0, half = lane / 32) receives rows
// {row0 + 4 half + 0..3} and {row0 + 4 half + 8 + 0..3} of column col0 + c.
// Within a group of 16 lanes, the transposing read hands lane i element (i % 4) of the
// four addresses supplied by lanes i / 4, 4 + i / 4, 8 + i / 4, 12 + i / 4 of the group.
template <int DH>
__device__ __forceinline__ bf16x8 read_tr_fragment(const char* tile, int row0, int col0, int lane) {
  int i = lane & 15;
  int grp = lane >> 4;
  int half = grp >> 1;
  int r = row0 + 4 * half + (i >> 2);
  int c = col0 + 16 * (grp & 1) + 4 * (i & 3);
  int inner = (c & 7) * 2;
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_AS3(tile + tile_offset<DH>(r, c >> 3) + inner));
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_AS3(tile + tile_offset<DH>(r + 8, c >> 3) + inner));
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

template <int DH>
__device__ __forceinline__ bf16x8 read_row_fragment(const char* tile, int row, int chunk) {
  return *reinterpret_cast<const bf16x8*>(tile + tile_offset<DH>(row, chunk));
}

// Eight consecutive accumulator values -> bf16 operand fragment.
__device__ __forceinline__ bf16x8 pack_bf16x8(const f32x16& a, int first) {
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (bf16)a[first + e];
  return r;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// ==================================================================================
// Forward: S^T = K Q^T, online softmax, O^T += V^T P^T per 64-key tile, a wave owning 32 query rows.
//
// Separate roles.  Eight compute waves never touch global memory inside the loop; a ninth wave does nothing but
// issue the K / V tile loads (HBM -> LDS direct) and wait for them.  A wave that issues such a load stalls until
// the memory pipeline has accepted it (about 25 cycles per KiB of tile and CU), and when every compute wave
// issues its share those stalls sit in front of MFMAs (measured: a tile pair of two waves took 4400 cycles, 2600
// with the loads taken out of the kernel); a loader wave stalls in nobody's way, and the compute waves' LDS reads
// and MFMAs run at the same speed beside it (probed: four MFMA waves fed by one fragment read per MFMA keep 82 %
// of the matrix peak with or without four loader waves streaming 120 GB/s into the same LDS).  To fit nine waves
// (three on one SIMD) a wave may use 168 registers, so only the first Q fragments stay in registers and the others
// are read from a Q tile in LDS again for every key tile.
// Opposite phases.  The compute waves work in two groups of four; block-wide barriers cut time into slots, and in
// every slot one group multiplies (P V of its tile j - 1, then the scores of its tile j: a matrix slot) while the
// other group, whose waves share the SIMDs of the first (waves w and w + 4), does the softmax of its tile.  Left
// alone, two waves of a SIMD are as often both in their softmax as one in each kind of work.
// ==================================================================================
template <int BEGIN, int END, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (BEGIN < END) {
    f(std::integral_constant<int, BEGIN>());
    static_for<BEGIN + 1, END>(f);
  }
}

// Per-lane LDS byte offsets of the fragment reads of a tile, such that every fragment of the tile is one of them
// XOR a constant (which moves the 16-byte chunk within the row: the swizzle only touches those bits) plus a
// constant number of rows (a multiple of 16 rows leaves the swizzle unchanged): three registers instead of an
// address per fragment.
template <int DH>
struct FragmentOffsets {
  unsigned v_lo, v_hi;  // transposing reads: rows 4 half + i / 4 (+ 8), output block 0
  unsigned k;           // row reads: row = lane % 32, head-dimension step 0
  __device__ __forceinline__ void init(int lane) {
    int i = lane & 15, grp = lane >> 4, half = grp >> 1;
    int r = 4 * half + (i >> 2);
    int c = 16 * (grp & 1) + 4 * (i & 3);
    v_lo = (unsigned)(tile_offset<DH>(r, c >> 3) + (c & 7) * 2);
    v_hi = (unsigned)(tile_offset<DH>(r + 8, c >> 3) + (c & 7) * 2);
    k = (unsigned)tile_offset<DH>(lane & 31, lane >> 5);
  }
};
__device__ __forceinline__ unsigned lds_address_of(const char* p) {
  return (unsigned)(size_t)((const __attribute__((address_space(3))) char*)p);
}
// V fragment (contraction over keys 16 js .. 16 js + 15, output block d) and row fragment (rows 32 j + lane % 32,
// head-dimension step kk) from the bases above; `vlo`, `vhi`, `kb` already include the tile's LDS address (tiles
// start at multiples of their size, so XOR and add commute with it).
template <int DH>
__device__ __forceinline__ bf16x8 read_v_fragment(unsigned vlo, unsigned vhi, int js, int d) {
  typedef __attribute__((address_space(3))) s16x4* lds_ptr;
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(size_t)((vlo ^ (unsigned)(d << 6)) + js * 16 * DH * 2));
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(size_t)((vhi ^ (unsigned)(d << 6)) + js * 16 * DH * 2));
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
template <int DH>
__device__ __forceinline__ bf16x8 read_k_fragment(unsigned kb, int j, int kk) {
  typedef const __attribute__((address_space(3))) bf16x8* lds_ptr;
  return *(lds_ptr)(size_t)((kb ^ (unsigned)(kk << 5)) + j * 32 * DH * 2);
}

// Softmax of one tile for the 32 rows of a wave: raw scores in, probabilities out as the P fragments of P V;
// running reference maximum and row sum updated, output accumulators rescaled when the reference moved.
template <int DH, bool MASK>
__device__ __forceinline__ void fwd_softmax(f32x16 (&sacc)[2], f32x16 (&oacc)[DH / 32], float& m_run, float& l_run,
                                            bf16x8 (&pf)[2][2], int key0, int q, int lane, float c) {
  constexpr int DT = DH / 32;
  const int half = lane >> 5;
  if (MASK) {
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e)
        if (key0 + 32 * j + 8 * (e >> 2) + 4 * half + (e & 3) > q) sacc[j][e] = -INFINITY;
  }
  float mx0 = -INFINITY, mx1 = -INFINITY;
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    mx0 = fmaxf(mx0, sacc[0][e]);
    mx1 = fmaxf(mx1, sacc[1][e]);
  }
  float mx = fmaxf(mx0, mx1);
  mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
  // m_run is a reference value, not necessarily the maximum seen so far: it only follows the true maximum when
  // some row of the wave has outgrown it by more than a factor 2^kLazyLog2.  Probabilities up to that factor
  // above one are as exact in bf16 and fp32 as those below one, the row sum is taken against the same reference,
  // and the final division by the row sum (and lse = m_run scale + log l) takes the factor out again.  With the
  // plain rule some row of the wave has a new maximum on almost every tile and all of them pay the rescale of the
  // output accumulators; with this one it happens on the first tiles only (+4 to +6 % on the kernel).  A row that
  // has seen no key yet keeps m_run = -inf; its probabilities come out as exp2(-inf) = 0.
  constexpr float kLazyLog2 = 8.0f;
  const bool outgrown = __builtin_amdgcn_ballot_w64((mx - m_run) * c > kLazyLog2) != 0;
  float m_new = outgrown ? fmaxf(m_run, mx) : m_run;
  float alpha = fast_exp2((m_run - m_new) * c);
  float mc = m_new * c;
  float sum = 0.f;
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      float pr = fast_exp2(sacc[j][e] * c - mc);
      sacc[j][e] = pr;
      sum += pr;
    }
  l_run = l_run * alpha + sum;
  bool moved = __builtin_amdgcn_ballot_w64(m_new > m_run) != 0;
  m_run = m_new;
  if (moved) {
#pragma unroll
    for (int d = 0; d < DT; ++d)
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[d][e] *= alpha;
  }
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    pf[j][0] = pack_bf16x8(sacc[j], 0);
    pf[j][1] = pack_bf16x8(sacc[j], 8);
  }
}

// A matrix slot: O^T += V^T P^T of the tile whose softmax just ended (PV), then the raw scores of the next tile
// (SC), as one stream of MFMAs fed by one ring of fragment registers read AHEAD fragments ahead of their use.
// The P V products go round the DH / 32 output blocks (consecutive MFMAs never wait for each other's
// accumulator); a step of the scores reads the Q fragment of this wave's rows and the two K fragments.
// Q fragments of the first q_in_regs head-dimension steps stay in registers (what 168 registers a wave leave room
// for: +1 to +2 % over reading all eight from LDS); the others are read from the Q tile in LDS for every key tile.
template <int DH>
constexpr int q_in_regs() {
  return 4;
}

template <int DH, bool PV, bool SC>
__device__ __forceinline__ void fwd_matrix_slot(const char* vtile, const char* ktile, unsigned q_addr,
                                                const bf16x8 (&qreg)[q_in_regs<DH>() > 0 ? q_in_regs<DH>() : 1],
                                                const FragmentOffsets<DH>& fo, const bf16x8 (&pf)[2][2],
                                                f32x16 (&oacc)[DH / 32], f32x16 (&sacc)[2]) {
  constexpr int KS = DH / 16, DT = DH / 32, QR = q_in_regs<DH>();
  constexpr int NPV = PV ? 4 * DT : 0;  // P V MFMAs, one V fragment each
  constexpr int NSC = SC ? 2 * KS : 0;  // score MFMAs; step kk reads K(0, kk), K(1, kk) and, from QR on, Q(kk) first
  constexpr int NFS = SC ? 2 * QR + 3 * (KS - QR) : 0;  // fragments of the scores
  // Two rings: the V fragments are read AV ahead of their MFMA; the fragments of the scores AS ahead, in
  // registers that the P fragments and the V ring no longer need by then.
  constexpr int AV = 3, RV = AV + 1;
  constexpr int AS = 5, RS = AS + 3;
  // The fragment addresses are cheap to rebuild (an XOR each); hiding the bases from the optimiser here keeps it
  // from carrying some twenty of them across the tile loop, which at 168 registers a wave would cost spills.
  unsigned off_lo = fo.v_lo, off_hi = fo.v_hi, off_k = fo.k;
  asm volatile("" : "+v"(off_lo), "+v"(off_hi), "+v"(off_k), "+v"(q_addr));
  const unsigned vlo = lds_address_of(vtile) + off_lo, vhi = lds_address_of(vtile) + off_hi;
  const unsigned kb = lds_address_of(ktile) + off_k;
  bf16x8 ring_v[RV], ring_s[RS];
  auto fetch_v = [&](auto fc) {
    constexpr int f = decltype(fc)::value;
    ring_v[f % RV] = read_v_fragment<DH>(vlo, vhi, f / DT, f % DT);  // f / DT = 2 (key sub-tile) + (16-key step)
  };
  // Score fragment f: steps kk < QR hold (K0, K1), the later ones (Q, K0, K1).
  struct Idx {
    static constexpr int step_of(int f) { return f < 2 * QR ? f / 2 : QR + (f - 2 * QR) / 3; }
    static constexpr int first_of(int kk) { return kk < QR ? 2 * kk : 2 * QR + 3 * (kk - QR); }
    // fragments of the scores that must have been requested before score MFMA m (counted from 0) is issued
    static constexpr int want(int m) {
      int kk = m / 2, j = m % 2;
      int need = first_of(kk) + (kk < QR ? 0 : 1) + j;
      return need + AS < NFS - 1 ? need + AS + 1 : NFS;
    }
  };
  auto fetch_s = [&](auto fc) {
    constexpr int f = decltype(fc)::value;
    constexpr int kk = Idx::step_of(f), w = f - Idx::first_of(kk) + (kk < QR ? 1 : 0);  // 0: Q, 1: K0, 2: K1
    if constexpr (w == 0)
      ring_s[f % RS] = read_k_fragment<DH>(q_addr, 0, kk);
    else
      ring_s[f % RS] = read_k_fragment<DH>(kb, w - 1, kk);
  };
  constexpr int PRE_S = SC ? (PV ? 3 : Idx::want(0)) : 0;  // requested during the last P V MFMAs
  static_for<0, (AV < NPV ? AV : NPV)>(fetch_v);
  if constexpr (!PV) static_for<0, PRE_S>(fetch_s);
  __builtin_amdgcn_sched_barrier(0);
  static_for<0, NPV>([&](auto mc) {
    constexpr int m = decltype(mc)::value;
    if constexpr (m + AV < NPV) fetch_v(std::integral_constant<int, m + AV>());
    if constexpr (m + AV >= NPV && m + AV < NPV + PRE_S) fetch_s(std::integral_constant<int, m + AV - NPV>());
    constexpr int js = m / DT, d = m % DT;
    oacc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring_v[m % RV], pf[js >> 1][js & 1], oacc[d], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
  });
  static_for<0, NSC>([&](auto mc) {
    constexpr int m = decltype(mc)::value;
    constexpr int lo = m == 0 ? PRE_S : Idx::want(m - 1), hi = Idx::want(m);
    static_for<(lo < hi ? lo : hi), hi>(fetch_s);
    constexpr int kk = m / 2, j = m % 2;
    constexpr int fk = Idx::first_of(kk) + (kk < QR ? 0 : 1) + j;
    bf16x8 qf;
    if constexpr (kk < QR) qf = qreg[kk];
    else qf = ring_s[Idx::first_of(kk) % RS];
    if constexpr (kk == 0) {
      f32x16 zero;
#pragma unroll
      for (int e = 0; e < 16; ++e) zero[e] = 0.f;
      sacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring_s[fk % RS], qf, zero, 0, 0, 0);
    } else {
      sacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring_s[fk % RS], qf, sacc[j], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
  });
}

template <int DH, int G>
__global__ __launch_bounds__(576, 1) void attn_fwd_roles_mfma_kernel(const bf16* __restrict__ qkv,
                                                                    bf16* __restrict__ o, float* __restrict__ lse,
                                                                    int s, int h, int hkv, int group, float scale) {
  // G = 1: 256 rows per block, group 0 owns rows 0-127 and group 1 rows 128-255, both walk the same tiles
  // through one ring of three stages.  G = 2 (launches that would not fill the chip with 256-row blocks): 128
  // rows per block, both groups own the same rows, group 0 takes the even tiles and group 1 the odd ones, each
  // through two stages of its own; the two partial results are merged through LDS at the end.
  constexpr int DT = DH / 32;
  constexpr int BQ = 256 / G;
  constexpr int TBYTES = tile_bytes<DH>();
  constexpr int STAGE = 2 * TBYTES;           // V tile, K tile
  constexpr int QBYTES = (BQ / 64) * TBYTES;  // the block's Q rows as tiles of 64 rows
  constexpr int PIECES = TBYTES / 1024;
  constexpr int ROWS_PER_4K = 4096 / (DH * 2);
  constexpr int NST = G == 1 ? 3 : 2;  // stages of a ring
  extern __shared__ __align__(16) char smem[];
  char* stages = smem + QBYTES;

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int head = blockIdx.x;
  const int q0 = (gridDim.y - 1 - blockIdx.y) * BQ;
  const int ld = h + 2 * hkv;
  const int nkv = (q0 + BQ) / kKeysPerTile;  // key tiles of the block
  const int n_it = nkv / G;                  // tiles of a group: its tile j is tile G j + group
  // A group's stage j (j = 0 .. n_it) is what its matrix slot j reads: V of its tile j - 1 and K of its tile j.
  // Slots are numbered 0 .. 2 n_it + 1, each ends with a barrier.  Group 0: matrix slot j in slot 2 j, softmax of
  // tile j in slot 2 j + 1.  Group 1: the same one slot later.

  if (wave == 8) {  // the loader
    const bf16* qbase = qkv + head * DH;
    const bf16* kbase = qkv + h + (head / group) * DH;
    const bf16* vbase = qkv + h + hkv + (head / group) * DH;
    unsigned lane_off[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) lane_off[i] = tile_lane_offset<DH>(ld, i, lane);
    auto load_tile = [&](const bf16* base, int row0, char* tile) {
#pragma unroll
      for (int q = 0; q < PIECES; ++q) {
        const bf16* src = base + (size_t)(row0 + (q >> 2) * ROWS_PER_4K) * ld;
        unsigned lds_addr = lds_address_of(tile + q * 1024);
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr),
                     "v"(lane_off[q & 3]), "s"(src)
                     : "memory");
      }
    };
    const int tile_last = nkv - 1;
    // A tile that does not exist is replaced by the nearest one that does, so that every stage is the same number
    // of loads and the waits below can count them.
    auto load_stage = [&](int g, int j) {
      char* st = stages + (G == 1 ? (j % NST) : g * NST + (j % NST)) * STAGE;
      int tv = G * (j - 1) + (G == 1 ? 0 : g), tk = G * j + (G == 1 ? 0 : g);
      load_tile(vbase, min(max(tv, 0), tile_last) * kKeysPerTile, st);
      load_tile(kbase, min(tk, tile_last) * kKeysPerTile, st + TBYTES);
    };
    auto wait_all_but_one_stage = [&]() {
      if (DH == 128) asm volatile("s_waitcnt vmcnt(32)" ::: "memory");
      else asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    };
#pragma unroll
    for (int t = 0; t < BQ / 64; ++t) load_tile(qbase, q0 + 64 * t, smem + t * TBYTES);
    if (G == 1) {
      // Stage j is read in slots 2 j and 2 j + 1; its buffer (j mod 3) takes stage j + 3 from slot 2 j + 2 on.
      load_stage(0, 0);
      load_stage(0, 1);
      wait_tile_loads_opaque();
      __syncthreads();
      for (int g = 0; g <= 2 * n_it + 1; ++g) {
        if ((g & 1) == 0) load_stage(0, g / 2 + 2);  // its buffer held stage g / 2 - 1, last read in slot g - 1
        else wait_all_but_one_stage();  // stage (g + 1) / 2 is read from the next slot on; one more may be on its way
        __syncthreads();
      }
    } else {
      // Group 0's stage j is read in slot 2 j, group 1's in slot 2 j + 1; a buffer (j mod 2 of its group) takes
      // the group's stage j + 2 in the slot after.  Every slot: what the next slot reads must have arrived (only
      // the stage issued in the slot before may still be on its way), then one stage is issued.
      load_stage(0, 0);
      load_stage(1, 0);
      load_stage(0, 1);
      load_stage(1, 1);
      wait_tile_loads_opaque();
      __syncthreads();
      for (int g = 0; g <= 2 * n_it + 1; ++g) {
        wait_all_but_one_stage();
        if (g >= 1) load_stage((g - 1) & 1, (g - 1) / 2 + 2);  // odd slots refill group 0's buffer, even ones group 1's
        __syncthreads();
      }
    }
    wait_tile_loads_opaque();  // nothing may still be on its way into LDS when the merge starts or the block ends
    if (G == 2) __syncthreads();
    return;
  }

  const int grp = wave >> 2;
  const int half = lane >> 5, col = lane & 31;
  const int wrow = G == 1 ? wave : (wave & 3);  // which 32 rows of the block
  const int qw0 = q0 + wrow * 32;
  const float c = scale * 1.4426950408889634f;
  FragmentOffsets<DH> fo;
  fo.init(lane);
  // this wave's Q rows: tile wrow / 2 of the Q area, rows 32 (wrow % 2) ..
  const unsigned q_addr = lds_address_of(smem + (wrow >> 1) * TBYTES) + fo.k + (wrow & 1) * 32 * DH * 2;
  f32x16 oacc[DT], sacc[2];
  bf16x8 pf[2][2];
  float m_run = -INFINITY, l_run = 0.f;
#pragma unroll
  for (int d = 0; d < DT; ++d)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[d][e] = 0.f;
  // The group's tiles 0 .. n_act - 1 hold keys this wave's rows may see; the last of them may reach the diagonal.
  const int t_last = (qw0 + 31) / kKeysPerTile;
  const int tg = G == 1 ? 0 : grp;
  const int n_act = t_last >= tg ? (t_last - tg) / G + 1 : 0;
  char* my_stages = stages + (G == 1 ? 0 : grp * NST) * STAGE;
  constexpr int QR = q_in_regs<DH>();
  bf16x8 qreg[QR > 0 ? QR : 1];

  __syncthreads();                // Q and the first stages are there
#pragma unroll
  for (int kk = 0; kk < QR; ++kk) qreg[kk] = read_k_fragment<DH>(q_addr, 0, kk);
  if (grp == 1) __syncthreads();  // slot 0: group 1 has nothing to do yet
  // Matrix slot j and the softmax of the group's tile j, two slots; PV: tile j - 1 is active, SC: tile j is.
  auto pair = [&](int j, auto pv, auto sc, auto mask, bool last_barrier) __attribute__((always_inline)) {
    const char* st = my_stages + (j % NST) * STAGE;
    __builtin_amdgcn_s_setprio(1);
    if constexpr (decltype(pv)::value || decltype(sc)::value)
      fwd_matrix_slot<DH, decltype(pv)::value, decltype(sc)::value>(st, st + TBYTES, q_addr, qreg, fo, pf, oacc,
                                                                      sacc);
    __builtin_amdgcn_s_setprio(0);
    __syncthreads();
    if constexpr (decltype(sc)::value)
      fwd_softmax<DH, decltype(mask)::value>(sacc, oacc, m_run, l_run, pf, (G * j + tg) * kKeysPerTile, qw0 + col,
                                             lane, c);
    if (last_barrier) __syncthreads();
  };
  const std::true_type yes;
  const std::false_type no;
  // pairs j = 0 .. n_it; group 1's very last slot (the softmax slot after its last matrix slot) does not exist
  int j = 0;
  if (n_act >= 2) {
    pair(0, no, yes, no, true);
    for (j = 1; j + 1 < n_act; ++j) pair(j, yes, yes, no, true);
    pair(j, yes, yes, yes, true);  // the group's last tile for this wave: masked against the diagonal
    j = n_act;
    pair(j, yes, no, no, !(grp == 1 && j == n_it));  // its P V
    ++j;
  } else if (n_act == 1) {
    pair(0, no, yes, yes, true);
    pair(1, yes, no, no, !(grp == 1 && 1 == n_it));
    j = 2;
  }
  for (; j <= n_it; ++j) pair(j, no, no, no, !(grp == 1 && j == n_it));

  if (G == 2) {
    // Merge: group 1 -> LDS -> group 0 (the stages are no longer read; the loader has drained its loads).
    __syncthreads();
    float* xch = reinterpret_cast<float*>(stages) + wrow * (64 * (DT * 16 + 2));
    if (grp == 1) {
#pragma unroll
      for (int d = 0; d < DT; ++d)
#pragma unroll
        for (int e = 0; e < 16; ++e) xch[(d * 16 + e) * 64 + lane] = oacc[d][e];
      xch[(DT * 16) * 64 + lane] = m_run;
      xch[(DT * 16 + 1) * 64 + lane] = l_run;
    }
    __syncthreads();
    if (grp == 1) return;
    float m1 = xch[(DT * 16) * 64 + lane], l1 = xch[(DT * 16 + 1) * 64 + lane];
    float m = fmaxf(m_run, m1);  // group 0 has seen key 0, so m is finite
    float a0 = fast_exp2((m_run - m) * c), a1 = fast_exp2((m1 - m) * c);
    l_run = l_run * a0 + l1 * a1;
    m_run = m;
#pragma unroll
    for (int d = 0; d < DT; ++d)
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[d][e] = oacc[d][e] * a0 + xch[(d * 16 + e) * 64 + lane] * a1;
  }
  const int q = qw0 + col;
  float l = l_run + __shfl_xor(l_run, 32, 64);
  float inv = 1.0f / l;
#pragma unroll
  for (int d = 0; d < DT; ++d)
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      bf16x4 v;
#pragma unroll
      for (int r = 0; r < 4; ++r) v[r] = (bf16)(oacc[d][4 * b + r] * inv);
      *reinterpret_cast<bf16x4*>(o + (size_t)q * h + head * DH + 32 * d + 8 * b + 4 * half) = v;
    }
  if (half == 0) lse[(size_t)head * s + q] = m_run * scale + __logf(l);
}

// ==================================================================================
// Backward, part 1: dK and dV.  Block = 128 keys (a wave owns 32), loop over the
// 64-row query tiles at or below the diagonal.  The Q and dO tiles in LDS serve both
// kinds of reads: ds_read_b128 fragments (contraction over the head dimension, for S
// and dP) and transposing fragments (contraction over the query rows, for dV and dK).
//   S[q][key]  = Q K^T          P = exp(S scale - lse[q])
//   dP[q][key] = dO V^T         dS = P (dP - delta[q])      (lse and delta are folded into the
//                                                            initial value of the two accumulators)
//   dV[key]   += P^T dO         dK[key] += dS^T Q   (times scale at the end)
// ==================================================================================
// The backward kernels are written as block functions: bx, by and gy stand for blockIdx.x, blockIdx.y and gridDim.y,
// so that a kernel of its own (the thin wrapper after each function) and the one-launch kernel further down, which
// numbers its blocks itself, run the same code.
template <int DH>
__device__ __forceinline__ void attn_bwd_dkv_mfma_block(const bf16* __restrict__ qkv, const bf16* __restrict__ d_o,
    const float* __restrict__ lse, const float* __restrict__ delta, bf16* __restrict__ out, int ld_out, int out_k0,
    int out_v_delta, int hpb, int s, int h, int hkv, int group, float scale, int bx, int by, int gy) {
  // Block b of the x dimension works on the hpb query heads b * hpb .. (all of them read key/value head
  // b * hpb / group) and writes dK to columns out_k0 + b * DH .., dV out_v_delta columns further, of `out`
  // (rows ld_out apart).  hpb = group: one block per key/value head writing straight into dqkv.  hpb = 1: one
  // block per query head writing per-head partial results that a second kernel adds up per group; that keeps
  // the launch as parallel as with plain multi-head attention when there are few key/value heads.
  constexpr int KS = DH / 16, DT = DH / 32;
  constexpr int TBYTES = tile_bytes<DH>();
  constexpr int STAGE = 2 * TBYTES + 512;  // Q tile, dO tile, lse[64], delta[64]
  extern __shared__ __align__(16) char smem[];

  int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  int half = lane >> 5, col = lane & 31;
  int head_first = bx * hpb;  // heads vary fastest in dispatch order: heaviest blocks of all heads first
  int kv_head = head_first / group;
  int kb0 = by * 128;   // first key of the block (the earliest blocks have the most query tiles)
  int kw0 = kb0 + wave * 32;    // first key of this wave
  int ld = h + 2 * hkv;
  const float LOG2E = 1.4426950408889634f;
  const float c = scale * LOG2E;

  // K and V fragments of this wave's keys: B operands, column = key, contraction over the head dimension.
  // With DH = 128 the last two V fragments live in LDS (a private 16-byte slot per lane and fragment)
  // instead of registers: at two waves per SIMD the register file cannot hold them without spilling.
  constexpr int V_IN_LDS = DH == 128 ? 2 : 0;
  constexpr int V_IN_REG = KS - V_IN_LDS;
  char* vslot = smem + 2 * STAGE + (wave * V_IN_LDS * 64 + lane) * 16;
  bf16x8 kf[KS], vf[V_IN_REG > 0 ? V_IN_REG : 1];
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) {
    const bf16* row = qkv + (size_t)(kw0 + col) * ld + h + kv_head * DH + 16 * kk + 8 * half;
    kf[kk] = *reinterpret_cast<const bf16x8*>(row);
    bf16x8 v = *reinterpret_cast<const bf16x8*>(row + hkv);
    if (kk < V_IN_REG)
      vf[kk] = v;
    else
      *reinterpret_cast<bf16x8*>(vslot + (kk - V_IN_REG) * 1024) = v;
  }
  f32x16 dk[DT], dv[DT];
#pragma unroll
  for (int d = 0; d < DT; ++d)
#pragma unroll
    for (int e = 0; e < 16; ++e) dk[d][e] = dv[d][e] = 0.f;

  // Query tiles [q_first, q_last) of every query head of this block, one head after the other:
  // iteration `it` works on head head_first + it / n_qt, tile q_first + it % n_qt.
  int q_first = kb0 / kKeysPerTile, q_last = s / kKeysPerTile;
  int n_qt = q_last - q_first, n_it = hpb * n_qt;
  // Row statistics enter as the initial value of the accumulators: S starts at -lse / scale, so that
  // exp2((S - lse / scale) * scale * log2 e) = P, and dP starts at -delta, so that dS = P * acc.
  // Threads 0..63 carry lse of a row, 64..127 delta of a row (128..255 repeat them and store nothing).  The
  // load is unconditional and its value is not touched until store_stats, after the tile's arithmetic:
  // any earlier use would wait for this load and with it for the tile loads issued just before it.
  const float* stat_src = ((tid & 64) ? delta - 64 : lse) + (tid & 127);
  const float stat_mul = (tid & 64) ? -1.0f : __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(
                                                   __builtin_bit_cast(int, -1.0f / scale)));
  float stat = 0.f;
  auto load_stats = [&](int head, int q0) { stat = stat_src[(size_t)head * s + q0]; };
  auto tile_of = [&](int it, int& head, int& qt) {
    int g = it / n_qt;
    head = head_first + g;
    qt = q_first + it - g * n_qt;
  };
  auto store_stats = [&](char* stage) {
    if (tid < 128) reinterpret_cast<float*>(stage + 2 * TBYTES)[tid] = stat * stat_mul;
  };
  const unsigned q_lane_off = tile_lane_offset<DH>(ld, wave, lane), do_lane_off = tile_lane_offset<DH>(h, wave, lane);
  {
    int head0 = head_first;
    load_tile_async<DH>(qkv + head0 * DH, ld, q_first * kKeysPerTile, smem, wave, q_lane_off);
    load_tile_async<DH>(d_o + head0 * DH, h, q_first * kKeysPerTile, smem + TBYTES, wave, do_lane_off);
    load_stats(head0, q_first * kKeysPerTile);
  }
  store_stats(smem);
  wait_tile_loads_opaque();
  __syncthreads();

  for (int it = 0; it < n_it; ++it) {
    int head, qt;
    tile_of(it, head, qt);
    (void)head;
    const char* qtile = smem + (it & 1) * STAGE;
    const char* dotile = qtile + TBYTES;
    const float* st_lse = reinterpret_cast<const float*>(qtile + 2 * TBYTES);
    const float* st_delta = st_lse + 64;
    char* nxt = smem + ((it + 1) & 1) * STAGE;
    bool more = it + 1 < n_it;
    // The swizzled LDS addresses are cheap to rebuild (a few XORs); hiding the lane id from the optimiser
    // here keeps it from carrying some twenty address registers across iterations and spilling
    // accumulators instead.
    int lane_l = lane;
    asm volatile("" : "+v"(lane_l));
    int col_l = lane_l & 31, half_l = lane_l >> 5;
    const char* vslot_l = smem + 2 * STAGE + (wave * V_IN_LDS * 64 + lane_l) * 16;
    if (more) {  // the other stage was last read before the barrier that ended the previous iteration
      int nhead, nqt;
      tile_of(it + 1, nhead, nqt);
      load_tile_async<DH>(qkv + nhead * DH, ld, nqt * kKeysPerTile, nxt, wave, q_lane_off);
      load_tile_async<DH>(d_o + nhead * DH, h, nqt * kKeysPerTile, nxt + TBYTES, wave, do_lane_off);
      load_stats(nhead, nqt * kKeysPerTile);
    }
    int q0 = qt * kKeysPerTile;
    int key = kw0 + col;
#pragma unroll
    for (int j = 0; j < 2; ++j) {  // 32-row halves of the query tile, one at a time (keeps registers low)
      int qs0 = q0 + 32 * j;
      if (qs0 + 31 < kw0) continue;  // every row of this half is above every key of this wave
      f32x16 sacc, pacc;
#pragma unroll
      for (int b = 0; b < 4; ++b) {  // accumulator row 8 b + 4 half + r is query row 32 j + that
        f32x4 l4 = *reinterpret_cast<const f32x4*>(st_lse + 32 * j + 8 * b + 4 * half_l);
        f32x4 d4 = *reinterpret_cast<const f32x4*>(st_delta + 32 * j + 8 * b + 4 * half_l);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          sacc[4 * b + r] = l4[r];
          pacc[4 * b + r] = d4[r];
        }
      }
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) {
        bf16x8 qa = read_row_fragment<DH>(qtile, 32 * j + col_l, 2 * kk + half_l);
        bf16x8 da = read_row_fragment<DH>(dotile, 32 * j + col_l, 2 * kk + half_l);
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, kf[kk], sacc, 0, 0, 0);
        bf16x8 vb;
        if (kk < V_IN_REG)
          vb = vf[kk];
        else
          vb = *reinterpret_cast<const bf16x8*>(vslot_l + (kk - V_IN_REG) * 1024);
        pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(da, vb, pacc, 0, 0, 0);
      }
      bool need_mask = qs0 < kw0 + 31;
#pragma unroll
      for (int e = 0; e < 16; ++e) sacc[e] = fast_exp2(sacc[e] * c);
      if (need_mask) {  // only tiles that straddle the diagonal pay for the mask
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (key > qs0 + 8 * (e >> 2) + 4 * half + (e & 3)) sacc[e] = 0.f;
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) pacc[e] *= sacc[e];
      bf16x8 pf[2] = {pack_bf16x8(sacc, 0), pack_bf16x8(sacc, 8)};
      bf16x8 dsf[2] = {pack_bf16x8(pacc, 0), pack_bf16x8(pacc, 8)};
#pragma unroll
      for (int d = 0; d < DT; ++d)
#pragma unroll
        for (int st = 0; st < 2; ++st) {
          bf16x8 dot = read_tr_fragment<DH>(dotile, 32 * j + 16 * st, 32 * d, lane_l);
          bf16x8 qtr = read_tr_fragment<DH>(qtile, 32 * j + 16 * st, 32 * d, lane_l);
          dv[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dot, pf[st], dv[d], 0, 0, 0);
          dk[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qtr, dsf[st], dk[d], 0, 0, 0);
        }
    }
    if (more) store_stats(nxt);
    wait_tile_loads_opaque();
    __syncthreads();
  }

  int key = kw0 + col;
#pragma unroll
  for (int d = 0; d < DT; ++d)
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      bf16x4 vk, vv;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        vk[r] = (bf16)(dk[d][4 * b + r] * scale);
        vv[r] = (bf16)dv[d][4 * b + r];
      }
      size_t off = (size_t)key * ld_out + out_k0 + bx * DH + 32 * d + 8 * b + 4 * half;
      *reinterpret_cast<bf16x4*>(out + off) = vk;
      *reinterpret_cast<bf16x4*>(out + off + out_v_delta) = vv;
    }
}

template <int DH>
__global__ __launch_bounds__(256, 2) void attn_bwd_dkv_mfma_kernel(const bf16* __restrict__ qkv,
    const bf16* __restrict__ d_o, const float* __restrict__ lse, const float* __restrict__ delta,
    bf16* __restrict__ out, int ld_out, int out_k0, int out_v_delta, int hpb, int s, int h, int hkv, int group,
    float scale) {
  attn_bwd_dkv_mfma_block<DH>(qkv, d_o, lse, delta, out, ld_out, out_k0, out_v_delta, hpb, s, h, hkv, group, scale,
      (int)blockIdx.x, (int)blockIdx.y, (int)gridDim.y);
}

// dK, dV for launches too small to give every CU two blocks: the kernel above with eight waves per block.
template <int DH>
__device__ __forceinline__ void attn_bwd_dkv_split_mfma_block(const bf16* __restrict__ qkv,
    const bf16* __restrict__ d_o, const float* __restrict__ lse, const float* __restrict__ delta,
    bf16* __restrict__ out, int ld_out, int out_k0, int out_v_delta, int hpb, int s, int h, int hkv, int group,
    float scale, int bx, int by, int gy) {
  // Block b of the x dimension works on the hpb query heads b * hpb .. (all of them read key/value head
  // b * hpb / group) and writes dK to columns out_k0 + b * DH .., dV out_v_delta columns further, of `out`
  // (rows ld_out apart).  hpb = group: one block per key/value head writing straight into dqkv.  hpb = 1: one
  // block per query head writing per-head partial results that a second kernel adds up per group; that keeps
  // the launch as parallel as with plain multi-head attention when there are few key/value heads.
  constexpr int KS = DH / 16, DT = DH / 32;
  constexpr int TBYTES = tile_bytes<DH>();
  constexpr int STAGE = 2 * TBYTES + 512;  // Q tile, dO tile, lse[64], delta[64]
  extern __shared__ __align__(16) char smem_all[];

  // Eight waves: waves w and w + 4 own the same 32 keys; group 0 takes the even iterations, group 1 the odd
  // ones, each with its own pair of stages, and group 1's dK, dV go to group 0 through LDS at the end.
  int lane = threadIdx.x & 63, wave8 = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
  int grp = wave8 >> 2, wave = wave8 & 3, tid = threadIdx.x & 255;
  char* smem = smem_all + grp * (2 * STAGE);
  char* vslots = smem_all + 4 * STAGE;
  int half = lane >> 5, col = lane & 31;
  int head_first = bx * hpb;  // heads vary fastest in dispatch order: heaviest blocks of all heads first
  int kv_head = head_first / group;
  int kb0 = by * 128;   // first key of the block (the earliest blocks have the most query tiles)
  int kw0 = kb0 + wave * 32;    // first key of this wave
  int ld = h + 2 * hkv;
  const float LOG2E = 1.4426950408889634f;
  const float c = scale * LOG2E;

  // K and V fragments of this wave's keys: B operands, column = key, contraction over the head dimension.
  // With DH = 128 the last two V fragments live in LDS (a private 16-byte slot per lane and fragment)
  // instead of registers: at two waves per SIMD the register file cannot hold them without spilling.
  constexpr int V_IN_LDS = DH == 128 ? 3 : 0;  // one more than the four-wave kernel: this one needs the slack
  constexpr int V_IN_REG = KS - V_IN_LDS;
  char* vslot = vslots + (wave8 * V_IN_LDS * 64 + lane) * 16;
  bf16x8 kf[KS], vf[V_IN_REG > 0 ? V_IN_REG : 1];
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) {
    const bf16* row = qkv + (size_t)(kw0 + col) * ld + h + kv_head * DH + 16 * kk + 8 * half;
    kf[kk] = *reinterpret_cast<const bf16x8*>(row);
    bf16x8 v = *reinterpret_cast<const bf16x8*>(row + hkv);
    if (kk < V_IN_REG)
      vf[kk] = v;
    else
      *reinterpret_cast<bf16x8*>(vslot + (kk - V_IN_REG) * 1024) = v;
  }
  f32x16 dk[DT], dv[DT];
#pragma unroll
  for (int d = 0; d < DT; ++d)
#pragma unroll
    for (int e = 0; e < 16; ++e) dk[d][e] = dv[d][e] = 0.f;

  // Query tiles [q_first, q_last) of every query head of this block, one head after the other:
  // iteration `it` works on head head_first + it / n_qt, tile q_first + it % n_qt.
  int q_first = kb0 / kKeysPerTile, q_last = s / kKeysPerTile;
  int n_qt = q_last - q_first, n_it = hpb * n_qt;
  // Row statistics enter as the initial value of the accumulators: S starts at -lse / scale, so that
  // exp2((S - lse / scale) * scale * log2 e) = P, and dP starts at -delta, so that dS = P * acc.
  // Threads 0..63 carry lse of a row, 64..127 delta of a row (128..255 repeat them and store nothing).  The
  // load is unconditional and its value is not touched until store_stats, after the tile's arithmetic:
  // any earlier use would wait for this load and with it for the tile loads issued just before it.
  const float* stat_src = ((tid & 64) ? delta - 64 : lse) + (tid & 127);
  const float stat_mul = (tid & 64) ? -1.0f : __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(
                                                   __builtin_bit_cast(int, -1.0f / scale)));
  float stat = 0.f;
  auto load_stats = [&](int head, int q0) { stat = stat_src[(size_t)head * s + q0]; };
  auto tile_of = [&](int it, int& head, int& qt) {
    int g = it / n_qt;
    head = head_first + g;
    qt = q_first + it - g * n_qt;
  };
  auto store_stats = [&](char* stage) {
    if (tid < 128) reinterpret_cast<float*>(stage + 2 * TBYTES)[tid] = stat * stat_mul;
  };
  const unsigned q_lane_off = tile_lane_offset<DH>(ld, wave, lane), do_lane_off = tile_lane_offset<DH>(h, wave, lane);
  {  // n_it >= 2 (a key block has at least two query tiles at or below it): both groups have a first tile
    int head0, qt0;
    tile_of(grp, head0, qt0);
    load_tile_async<DH>(qkv + head0 * DH, ld, qt0 * kKeysPerTile, smem, wave, q_lane_off);
    load_tile_async<DH>(d_o + head0 * DH, h, qt0 * kKeysPerTile, smem + TBYTES, wave, do_lane_off);
    load_stats(head0, qt0 * kKeysPerTile);
  }
  store_stats(smem);
  wait_tile_loads_opaque();
  __syncthreads();

  int n_round = (n_it + 1) / 2;
  for (int rnd = 0; rnd < n_round; ++rnd) {
    int it = 2 * rnd + grp;
    bool active = it < n_it;  // the last round of group 1 is empty when n_it is odd
    int head, qt;
    tile_of(active ? it : 0, head, qt);
    (void)head;
    const char* qtile = smem + (rnd & 1) * STAGE;
    const char* dotile = qtile + TBYTES;
    const float* st_lse = reinterpret_cast<const float*>(qtile + 2 * TBYTES);
    const float* st_delta = st_lse + 64;
    char* nxt = smem + ((rnd + 1) & 1) * STAGE;
    bool more = it + 2 < n_it;
    // The swizzled LDS addresses are cheap to rebuild (a few XORs); hiding the lane id from the optimiser
    // here keeps it from carrying some twenty address registers across iterations and spilling
    // accumulators instead.
    int lane_l = lane;
    asm volatile("" : "+v"(lane_l));
    int col_l = lane_l & 31, half_l = lane_l >> 5;
    const char* vslot_l = vslots + (wave8 * V_IN_LDS * 64 + lane_l) * 16;
    if (more) {  // the other stage was last read before the barrier that ended the previous iteration
      int nhead, nqt;
      tile_of(it + 2, nhead, nqt);
      load_tile_async<DH>(qkv + nhead * DH, ld, nqt * kKeysPerTile, nxt, wave, q_lane_off);
      load_tile_async<DH>(d_o + nhead * DH, h, nqt * kKeysPerTile, nxt + TBYTES, wave, do_lane_off);
      load_stats(nhead, nqt * kKeysPerTile);
    }
    int q0 = qt * kKeysPerTile;
    int key = kw0 + col;
#pragma unroll
    for (int j = 0; j < 2; ++j) {  // 32-row halves of the query tile, one at a time (keeps registers low)
      int qs0 = q0 + 32 * j;
      if (!active || qs0 + 31 < kw0) continue;  // nothing to do, or every row of this half is above every key
      f32x16 sacc, pacc;
#pragma unroll
      for (int b = 0; b < 4; ++b) {  // accumulator row 8 b + 4 half + r is query row 32 j + that
        f32x4 l4 = *reinterpret_cast<const f32x4*>(st_lse + 32 * j + 8 * b + 4 * half_l);
        f32x4 d4 = *reinterpret_cast<const f32x4*>(st_delta + 32 * j + 8 * b + 4 * half_l);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          sacc[4 * b + r] = l4[r];
          pacc[4 * b + r] = d4[r];
        }
      }
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) {
        bf16x8 qa = read_row_fragment<DH>(qtile, 32 * j + col_l, 2 * kk + half_l);
        bf16x8 da = read_row_fragment<DH>(dotile, 32 * j + col_l, 2 * kk + half_l);
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, kf[kk], sacc, 0, 0, 0);
        bf16x8 vb;
        if (kk < V_IN_REG)
          vb = vf[kk];
        else
          vb = *reinterpret_cast<const bf16x8*>(vslot_l + (kk - V_IN_REG) * 1024);
        pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(da, vb, pacc, 0, 0, 0);
      }
      bool need_mask = qs0 < kw0 + 31;
#pragma unroll
      for (int e = 0; e < 16; ++e) sacc[e] = fast_exp2(sacc[e] * c);
      if (need_mask) {  // only tiles that straddle the diagonal pay for the mask
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (key > qs0 + 8 * (e >> 2) + 4 * half + (e & 3)) sacc[e] = 0.f;
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) pacc[e] *= sacc[e];
      bf16x8 pf[2] = {pack_bf16x8(sacc, 0), pack_bf16x8(sacc, 8)};
      bf16x8 dsf[2] = {pack_bf16x8(pacc, 0), pack_bf16x8(pacc, 8)};
#pragma unroll
      for (int d = 0; d < DT; ++d)
#pragma unroll
        for (int st = 0; st < 2; ++st) {
          bf16x8 dot = read_tr_fragment<DH>(dotile, 32 * j + 16 * st, 32 * d, lane_l);
          bf16x8 qtr = read_tr_fragment<DH>(qtile, 32 * j + 16 * st, 32 * d, lane_l);
          dv[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dot, pf[st], dv[d], 0, 0, 0);
          dk[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qtr, dsf[st], dk[d], 0, 0, 0);
        }
    }
    if (more) store_stats(nxt);
    wait_tile_loads_opaque();
    __syncthreads();
  }

  // group 1 -> LDS -> group 0: 2 * DT * 16 floats per lane (the stages are free after the last barrier)
  // The lane id is rebuilt here (two mbcnt instructions) rather than kept in a register across the loop, where
  // every register is taken.
  int lane_e = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
  float* xch = reinterpret_cast<float*>(smem_all) + wave * (64 * 2 * DT * 16) + lane_e;
  if (grp == 1) {
#pragma unroll
    for (int d = 0; d < DT; ++d)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        xch[(d * 16 + e) * 64] = dk[d][e];
        xch[((DT + d) * 16 + e) * 64] = dv[d][e];
      }
  }
  __syncthreads();
  if (grp == 0) {
    int half = lane_e >> 5;
    int key = kw0 + (lane_e & 31);
#pragma unroll
    for (int d = 0; d < DT; ++d)
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        bf16x4 vk, vv;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          int e = 4 * b + r;
          vk[r] = (bf16)((dk[d][e] + xch[(d * 16 + e) * 64]) * scale);
          vv[r] = (bf16)(dv[d][e] + xch[((DT + d) * 16 + e) * 64]);
        }
        size_t off = (size_t)key * ld_out + out_k0 + bx * DH + 32 * d + 8 * b + 4 * half;
        *reinterpret_cast<bf16x4*>(out + off) = vk;
        *reinterpret_cast<bf16x4*>(out + off + out_v_delta) = vv;
      }
  }
}

template <int DH>
__global__ __launch_bounds__(512, 1) void attn_bwd_dkv_split_mfma_kernel(const bf16* __restrict__ qkv,
    const bf16* __restrict__ d_o, const float* __restrict__ lse, const float* __restrict__ delta,
    bf16* __restrict__ out, int ld_out, int out_k0, int out_v_delta, int hpb, int s, int h, int hkv, int group,
    float scale) {
  attn_bwd_dkv_split_mfma_block<DH>(qkv, d_o, lse, delta, out, ld_out, out_k0, out_v_delta, hpb, s, h, hkv, group,
      scale, (int)blockIdx.x, (int)blockIdx.y, (int)gridDim.y);
}

// ==================================================================================
// Backward, part 2: dQ.  Block = 128 QT query rows (a wave owns 32 QT), loop over the
// key tiles up to the diagonal.  The K tile is read both ways (row fragments for
// S^T = K Q^T, transposing fragments for dQ^T = K^T dS^T), the V tile as row fragments.
// ==================================================================================
template <int DH, int QT>
__device__ __forceinline__ void attn_bwd_dq_mfma_block(const bf16* __restrict__ qkv, const bf16* __restrict__ d_o,
    const float* __restrict__ lse, const float* __restrict__ delta, bf16* __restrict__ dqkv, int s, int h, int hkv,
    int group, float scale, int bx, int by, int gy) {
  constexpr int KS = DH / 16, DT = DH / 32;
  constexpr int BQ = 128 * QT;
  constexpr int KBYTES = tile_bytes<DH>();
  constexpr int STAGE = 2 * KBYTES;  // K tile, V tile
  extern __shared__ __align__(16) char smem[];

  int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  int half = lane >> 5, col = lane & 31;
  int head = bx;  // dispatch order as in the forward kernel
  int qblock = gy - 1 - by;
  int q0 = qblock * BQ;
  int qw0 = q0 + wave * (32 * QT);
  int ld = h + 2 * hkv;
  const bf16* kbase = qkv + h + (head / group) * DH;
  const bf16* vbase = qkv + h + hkv + (head / group) * DH;
  const float LOG2E = 1.4426950408889634f;
  const float c = scale * LOG2E;

  bf16x8 qf[QT][KS], dof[QT][KS];
  float lse_q[QT], delta_q[QT];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    int q = qw0 + 32 * t + col;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      qf[t][kk] = *reinterpret_cast<const bf16x8*>(qkv + (size_t)q * ld + head * DH + 16 * kk + 8 * half);
      dof[t][kk] = *reinterpret_cast<const bf16x8*>(d_o + (size_t)q * h + head * DH + 16 * kk + 8 * half);
    }
    lse_q[t] = lse[(size_t)head * s + q] * LOG2E;
    delta_q[t] = delta[(size_t)head * s + q];
  }
  f32x16 dq[QT][DT];
#pragma unroll
  for (int t = 0; t < QT; ++t)
#pragma unroll
    for (int d = 0; d < DT; ++d)
#pragma unroll
      for (int e = 0; e < 16; ++e) dq[t][d][e] = 0.f;

  int nkv = (q0 + BQ) / kKeysPerTile;
  const unsigned lane_off = tile_lane_offset<DH>(ld, wave, lane);
  load_tile_async<DH>(kbase, ld, 0, smem, wave, lane_off);
  load_tile_async<DH>(vbase, ld, 0, smem + KBYTES, wave, lane_off);
  wait_tile_loads();
  __syncthreads();

  for (int kt = 0; kt < nkv; ++kt) {
    const char* ktile = smem + (kt & 1) * STAGE;
    const char* vtile = ktile + KBYTES;
    char* nxt = smem + ((kt + 1) & 1) * STAGE;
    bool more = kt + 1 < nkv;
    if (more) {  // the other stage was last read before the barrier that ended the previous iteration
      load_tile_async<DH>(kbase, ld, (kt + 1) * kKeysPerTile, nxt, wave, lane_off);
      load_tile_async<DH>(vbase, ld, (kt + 1) * kKeysPerTile, nxt + KBYTES, wave, lane_off);
    }
    int key0 = kt * kKeysPerTile;
#pragma unroll
    for (int j = 0; j < 2; ++j) {  // 32-key halves of the tile, one at a time (keeps registers low)
      int ks0 = key0 + 32 * j;
      if (ks0 > qw0 + 32 * QT - 1) continue;  // every key of this half is beyond every row of this wave
      f32x16 sacc[QT], pacc[QT];
#pragma unroll
      for (int t = 0; t < QT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) sacc[t][e] = pacc[t][e] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) {
        bf16x8 ka = read_row_fragment<DH>(ktile, 32 * j + col, 2 * kk + half);
        bf16x8 va = read_row_fragment<DH>(vtile, 32 * j + col, 2 * kk + half);
#pragma unroll
        for (int t = 0; t < QT; ++t) {
          sacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[t][kk], sacc[t], 0, 0, 0);
          pacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, dof[t][kk], pacc[t], 0, 0, 0);
        }
      }
      bf16x8 dsf[QT][2];
#pragma unroll
      for (int t = 0; t < QT; ++t) {
        int q = qw0 + 32 * t + col;
        bool need_mask = ks0 + 31 > qw0 + 32 * t;
#pragma unroll
        for (int e = 0; e < 16; ++e) sacc[t][e] = fast_exp2(sacc[t][e] * c - lse_q[t]);
        if (need_mask) {  // only tiles that straddle the diagonal pay for the mask
#pragma unroll
          for (int e = 0; e < 16; ++e)
            if (ks0 + 8 * (e >> 2) + 4 * half + (e & 3) > q) sacc[t][e] = 0.f;
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) pacc[t][e] = sacc[t][e] * (pacc[t][e] - delta_q[t]);
        dsf[t][0] = pack_bf16x8(pacc[t], 0);
        dsf[t][1] = pack_bf16x8(pacc[t], 8);
      }
#pragma unroll
      for (int d = 0; d < DT; ++d)
#pragma unroll
        for (int st = 0; st < 2; ++st) {
          bf16x8 ktr = read_tr_fragment<DH>(ktile, 32 * j + 16 * st, 32 * d, lane);
#pragma unroll
          for (int t = 0; t < QT; ++t)
            dq[t][d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ktr, dsf[t][st], dq[t][d], 0, 0, 0);
        }
    }
    wait_tile_loads();
    __syncthreads();
  }

#pragma unroll
  for (int t = 0; t < QT; ++t) {
    int q = qw0 + 32 * t + col;
#pragma unroll
    for (int d = 0; d < DT; ++d)
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        bf16x4 v;
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = (bf16)(dq[t][d][4 * b + r] * scale);
        *reinterpret_cast<bf16x4*>(dqkv + (size_t)q * ld + head * DH + 32 * d + 8 * b + 4 * half) = v;
      }
  }
}

template <int DH, int QT>
__global__ __launch_bounds__(256, QT == 1 ? 2 : 1) void attn_bwd_dq_mfma_kernel(const bf16* __restrict__ qkv,
    const bf16* __restrict__ d_o, const float* __restrict__ lse, const float* __restrict__ delta,
    bf16* __restrict__ dqkv, int s, int h, int hkv, int group, float scale) {
  attn_bwd_dq_mfma_block<DH, QT>(qkv, d_o, lse, delta, dqkv, s, h, hkv, group, scale, (int)blockIdx.x,
      (int)blockIdx.y, (int)gridDim.y);
}

// dQ for launches too small to give every CU two blocks: eight waves, waves w and w + 4 own the same 32
// query rows and alternate key tiles, as the two groups of the forward kernel's 128-row form do; group 1's
// partial dQ goes to group 0 through LDS at the end (one addition per element, always in the same order).
template <int DH>
__device__ __forceinline__ void attn_bwd_dq_split_mfma_block(const bf16* __restrict__ qkv,
    const bf16* __restrict__ d_o, const float* __restrict__ lse, const float* __restrict__ delta,
    bf16* __restrict__ dqkv, int s, int h, int hkv, int group, float scale, int bx, int by, int gy) {
  constexpr int KS = DH / 16, DT = DH / 32;
  constexpr int BQ = 128;
  constexpr int KBYTES = tile_bytes<DH>();
  constexpr int STAGE = 2 * KBYTES;  // K tile, V tile
  extern __shared__ __align__(16) char smem_all[];

  int tid = threadIdx.x, lane = tid & 63;
  int wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);
  int grp = wave8 >> 2, wave = wave8 & 3;
  char* smem = smem_all + grp * (2 * STAGE);
  int half = lane >> 5, col = lane & 31;
  int head = bx;
  int qblock = gy - 1 - by;
  int q0 = qblock * BQ;
  int qw0 = q0 + wave * 32;
  int ld = h + 2 * hkv;
  const bf16* kbase = qkv + h + (head / group) * DH;
  const bf16* vbase = qkv + h + hkv + (head / group) * DH;
  const float LOG2E = 1.4426950408889634f;
  const float c = scale * LOG2E;

  bf16x8 qf[KS], dof[KS];
  int q = qw0 + col;
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) {
    qf[kk] = *reinterpret_cast<const bf16x8*>(qkv + (size_t)q * ld + head * DH + 16 * kk + 8 * half);
    dof[kk] = *reinterpret_cast<const bf16x8*>(d_o + (size_t)q * h + head * DH + 16 * kk + 8 * half);
  }
  float lse_q = lse[(size_t)head * s + q] * LOG2E;
  float delta_q = delta[(size_t)head * s + q];
  f32x16 dq[DT];
#pragma unroll
  for (int d = 0; d < DT; ++d)
#pragma unroll
    for (int e = 0; e < 16; ++e) dq[d][e] = 0.f;

  int n_it = (q0 + BQ) / kKeysPerTile / 2;  // tiles per group
  const unsigned lane_off = tile_lane_offset<DH>(ld, wave, lane);
  load_tile_async<DH>(kbase, ld, grp * kKeysPerTile, smem, wave, lane_off);
  load_tile_async<DH>(vbase, ld, grp * kKeysPerTile, smem + KBYTES, wave, lane_off);
  wait_tile_loads();
  __syncthreads();

  for (int it = 0; it < n_it; ++it) {
    int kt = 2 * it + grp;
    const char* ktile = smem + (it & 1) * STAGE;
    const char* vtile = ktile + KBYTES;
    char* nxt = smem + ((it + 1) & 1) * STAGE;
    if (it + 1 < n_it) {
      load_tile_async<DH>(kbase, ld, (kt + 2) * kKeysPerTile, nxt, wave, lane_off);
      load_tile_async<DH>(vbase, ld, (kt + 2) * kKeysPerTile, nxt + KBYTES, wave, lane_off);
    }
    int key0 = kt * kKeysPerTile;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      int ks0 = key0 + 32 * j;
      if (ks0 > qw0 + 31) continue;
      f32x16 sacc, pacc;
#pragma unroll
      for (int e = 0; e < 16; ++e) sacc[e] = pacc[e] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) {
        bf16x8 ka = read_row_fragment<DH>(ktile, 32 * j + col, 2 * kk + half);
        bf16x8 va = read_row_fragment<DH>(vtile, 32 * j + col, 2 * kk + half);
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[kk], sacc, 0, 0, 0);
        pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, dof[kk], pacc, 0, 0, 0);
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) sacc[e] = fast_exp2(sacc[e] * c - lse_q);
      if (ks0 + 31 > qw0) {
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (ks0 + 8 * (e >> 2) + 4 * half + (e & 3) > q) sacc[e] = 0.f;
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) pacc[e] = sacc[e] * (pacc[e] - delta_q);
      bf16x8 dsf[2] = {pack_bf16x8(pacc, 0), pack_bf16x8(pacc, 8)};
#pragma unroll
      for (int d = 0; d < DT; ++d)
#pragma unroll
        for (int st = 0; st < 2; ++st) {
          bf16x8 ktr = read_tr_fragment<DH>(ktile, 32 * j + 16 * st, 32 * d, lane);
          dq[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ktr, dsf[st], dq[d], 0, 0, 0);
        }
    }
    wait_tile_loads();
    __syncthreads();
  }

  float* xch = reinterpret_cast<float*>(smem_all) + wave * (64 * DT * 16);
  if (grp == 1) {
#pragma unroll
    for (int d = 0; d < DT; ++d)
#pragma unroll
      for (int e = 0; e < 16; ++e) xch[(d * 16 + e) * 64 + lane] = dq[d][e];
  }
  __syncthreads();
  if (grp == 0) {
#pragma unroll
    for (int d = 0; d < DT; ++d)
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        bf16x4 v;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          int e = 4 * b + r;
          v[r] = (bf16)((dq[d][e] + xch[(d * 16 + e) * 64 + lane]) * scale);
        }
        *reinterpret_cast<bf16x4*>(dqkv + (size_t)q * ld + head * DH + 32 * d + 8 * b + 4 * half) = v;
      }
  }
}

template <int DH>
__global__ __launch_bounds__(512, 1) void attn_bwd_dq_split_mfma_kernel(const bf16* __restrict__ qkv,
    const bf16* __restrict__ d_o, const float* __restrict__ lse, const float* __restrict__ delta,
    bf16* __restrict__ dqkv, int s, int h, int hkv, int group, float scale) {
  attn_bwd_dq_split_mfma_block<DH>(qkv, d_o, lse, delta, dqkv, s, h, hkv, group, scale, (int)blockIdx.x,
      (int)blockIdx.y, (int)gridDim.y);
}

// dK/dV and dQ in one launch.  Both kernels give their blocks very unequal work (the causal triangle) and both
// dispatch their heaviest blocks first; as two launches, the CUs that drew light blocks idle until the heaviest
// block of each launch ends.  As one launch whose first n_kv blocks are the dK/dV blocks and whose other blocks
// are the dQ blocks, the dQ blocks start on the CUs that the light dK/dV blocks leave early.  The two parts
// share nothing but their inputs (dQ, and dK/dV or their partials, are disjoint outputs), so a block runs
// exactly what it would run in its own kernel and the results are the same bit for bit.
template <int DH, bool EIGHT>
__global__ __launch_bounds__(EIGHT ? 512 : 256, EIGHT ? 1 : 2) void attn_bwd_fused_mfma_kernel(
    const bf16* __restrict__ qkv, const bf16* __restrict__ d_o, const float* __restrict__ lse,
    const float* __restrict__ delta, bf16* __restrict__ out, int ld_out, int out_k0, int out_v_delta, int hpb,
    bf16* __restrict__ dqkv, int s, int h, int hkv, int group, float scale, int x_kv, int x_q) {
  int gy = s / 128;
  int b = (int)blockIdx.x, n_kv = x_kv * gy;
  if (b < n_kv) {
    int by = b / x_kv, bx = b - by * x_kv;
    if constexpr (EIGHT)
      attn_bwd_dkv_split_mfma_block<DH>(qkv, d_o, lse, delta, out, ld_out, out_k0, out_v_delta, hpb, s, h, hkv, group,
                                        scale, bx, by, gy);
    else
      attn_bwd_dkv_mfma_block<DH>(qkv, d_o, lse, delta, out, ld_out, out_k0, out_v_delta, hpb, s, h, hkv, group,
          scale,
                                  bx, by, gy);
  } else {
    b -= n_kv;
    int by = b / x_q, bx = b - by * x_q;
    if constexpr (EIGHT)
      attn_bwd_dq_split_mfma_block<DH>(qkv, d_o, lse, delta, dqkv, s, h, hkv, group, scale, bx, by, gy);
    else
      attn_bwd_dq_mfma_block<DH, 1>(qkv, d_o, lse, delta, dqkv, s, h, hkv, group, scale, bx, by, gy);
  }
}

// Adds the per-query-head dK / dV partials [s, 2h] (dK of head t at columns t * DH, dV at h + t * DH) of every
// group in head order, in fp32, into the key and value blocks of dqkv [s, h + 2 hkv].  One thread per 8 columns.
template <int DH>
__global__ __launch_bounds__(256) void attn_group_sum_kernel(const bf16* __restrict__ part, bf16* __restrict__ dqkv,
                                                             int s, int h, int hkv, int group) {
  int per_row = 2 * hkv / 8;
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)s * per_row) return;
  int row = (int)(idx / per_row), c8 = (int)(idx % per_row) * 8;
  int is_v = c8 >= hkv;
  int c = c8 - is_v * hkv;           // column inside the key (or value) block
  int kv_head = c / DH, e = c % DH;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int g = 0; g < group; ++g) {
    bf16x8 v = *reinterpret_cast<const bf16x8*>(part + (size_t)row * (2 * h) + is_v * h + (kv_head * group + g) * DH + e);
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] += (float)v[i];
  }
  bf16x8 o;
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = (bf16)acc[i];
  *reinterpret_cast<bf16x8*>(dqkv + (size_t)row * (h + 2 * hkv) + h + c8) = o;
}

// delta[head][i] = sum_e dO[i, head, e] * O[i, head, e].  Thread t takes the t-th group of eight consecutive
// elements of the [s, h] tensors (16-byte loads, consecutive lanes read consecutive addresses); the DH / 8 lanes
// that share a (row, head) add their partial sums with a butterfly, so every one of them ends with the total.
template <int DH>
__global__ __launch_bounds__(256) void attn_delta_mfma_path_kernel(const bf16* __restrict__ o,
                                                                   const bf16* __restrict__ d_o,
                                                                   float* __restrict__ delta, int s, int h) {
  constexpr int LPR = DH / 8;  // lanes per (row, head)
  size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
  size_t total = (size_t)s * h / 8;  // a multiple of LPR: a lane group is inside or outside as a whole
  float d = 0.f;
  if (t < total) {
    bf16x8 a = *reinterpret_cast<const bf16x8*>(o + t * 8);
    bf16x8 b = *reinterpret_cast<const bf16x8*>(d_o + t * 8);
#pragma unroll
    for (int e = 0; e < 8; ++e) d += (float)a[e] * (float)b[e];
  }
#pragma unroll
  for (int m = 1; m < LPR; m <<= 1) d += __shfl_xor(d, m);
  if (t < total && threadIdx.x % LPR == 0) {
    size_t row = t * 8 / h;
    int head = (int)(t * 8 % h) / DH;
    delta[(size_t)head * s + row] = d;
  }
}

// ==================================================================================
// Host side
// ==================================================================================
bool attention_mfma_supported(int s, int h, int n_heads, int n_kv_heads) {
  if (n_heads <= 0 || h % n_heads != 0 || n_kv_heads <= 0 || n_heads % n_kv_heads != 0) return false;
  int dh = h / n_heads;
  return (dh == 64 || dh == 128) && s >= 128 && s % 128 == 0;
}

template <int DH>
static bool launch_fwd(const bf16* qkv, bf16* o, float* lse, int s, int h, int n_heads, int n_kv_heads,
                       hipStream_t stream) {
  constexpr int smem = 10 * tile_bytes<DH>();  // Q tiles and stage rings: 160 KiB for DH = 128 in either form
  // 256-row blocks where they still give every CU one; else 128-row blocks whose two groups split the key tiles.
  const bool big = s % 256 == 0 && (int64_t)n_heads * (s / 256) >= 256;
  auto k1 = attn_fwd_roles_mfma_kernel<DH, 1>;
  auto k2 = attn_fwd_roles_mfma_kernel<DH, 2>;
  static bool configured = false;
  if (!configured) {
    PO_HIP_OK(hipFuncSetAttribute(reinterpret_cast<const void*>(k1), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  smem));
    PO_HIP_OK(hipFuncSetAttribute(reinterpret_cast<const void*>(k2), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  smem));
    configured = true;
  }
  const float scale = 1.0f / sqrtf((float)DH);
  if (big)
    k1<<<dim3(n_heads, s / 256), 576, smem, stream>>>(qkv, o, lse, s, h, n_kv_heads * DH, n_heads / n_kv_heads, scale);
  else
    k2<<<dim3(n_heads, s / 128), 576, smem, stream>>>(qkv, o, lse, s, h, n_kv_heads * DH, n_heads / n_kv_heads, scale);
  return launch_ok("attn_fwd_roles_mfma_kernel");
}

bool attention_forward_mfma(const void* qkv, void* o, float* lse, int s, int h, int n_heads, int n_kv_heads,
                            hipStream_t stream) {
  if (!attention_mfma_supported(s, h, n_heads, n_kv_heads) || !qkv || !o || !lse ||
      ((uintptr_t)qkv | (uintptr_t)o) % 16 != 0) {
    set_error("attention_forward_mfma: unsupported s=%d h=%d heads=%d kv_heads=%d or bad pointers", s, h, n_heads,
              n_kv_heads);
    return false;
  }
  const bf16* q = (const bf16*)qkv;
  bf16* out = (bf16*)o;
  if (h / n_heads == 128) return launch_fwd<128>(q, out, lse, s, h, n_heads, n_kv_heads, stream);
  return launch_fwd<64>(q, out, lse, s, h, n_heads, n_kv_heads, stream);
}

template <int DH>
static bool launch_bwd(const bf16* qkv, const bf16* o, const float* lse, const bf16* d_o, bf16* dqkv, float* delta,
                       bf16* partials, int s, int h, int n_heads, int n_kv_heads, hipStream_t stream) {
  constexpr int smem_kv = 2 * (2 * tile_bytes<DH>() + 512) + (DH == 128 ? 8192 : 0);  // + V fragments kept in LDS
  constexpr int smem_q = 4 * tile_bytes<DH>();
  auto kkv = attn_bwd_dkv_mfma_kernel<DH>;
  auto kq1 = attn_bwd_dq_mfma_kernel<DH, 1>;
  static bool configured = false;
  if (!configured) {
    PO_HIP_OK(hipFuncSetAttribute(reinterpret_cast<const void*>(kkv), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  smem_kv));
    PO_HIP_OK(hipFuncSetAttribute(reinterpret_cast<const void*>(kq1), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  smem_q));
    configured = true;
  }
  float scale = 1.0f / sqrtf((float)DH);
  int hkv = n_kv_heads * DH, group = n_heads / n_kv_heads;
  attn_delta_mfma_path_kernel<DH><<<(unsigned)(((size_t)s * h / 8 + 255) / 256), 256, 0, stream>>>(o, d_o, delta, s, h);
  // Few key/value heads: one block per query head and a per-group sum afterwards (needs the [s, 2h] workspace),
  // once the direct launch would not fill the chip's 512 block slots.
  bool split = group > 1 && partials && (int64_t)n_kv_heads * (s / 128) < 512;
  // At most one block per CU: the eight-wave kernel, which halves a wave's chain of tiles.
  constexpr int smem_kv8 = 4 * (2 * tile_bytes<DH>() + 512) + (DH == 128 ? 24576 : 0);
  auto kkv8 = attn_bwd_dkv_split_mfma_kernel<DH>;
  bool eight = (int64_t)(split ? n_heads : n_kv_heads) * (s / 128) <= 256;
  static bool eight_configured = false;
  if (eight && !eight_configured) {
    PO_HIP_OK(hipFuncSetAttribute(reinterpret_cast<const void*>(kkv8), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  smem_kv8));
    eight_configured = true;
  }
  const bool dq_eight = (int64_t)n_heads * (s / 128) <= 256;  // one block per CU at most: the eight-wave kernel
  constexpr int smem_split = 8 * tile_bytes<DH>();
  // where dK/dV go: per-head partials [s, 2h] or dqkv itself
  bf16* kv_out = split ? partials : dqkv;
  const int kv_ld = split ? 2 * h : h + 2 * hkv, kv_k0 = split ? 0 : h, kv_vd = split ? h : hkv;
  const int kv_hpb = split ? 1 : group, x_kv = split ? n_heads : n_kv_heads;
  if (eight == dq_eight) {  // same block shape: one launch, the dQ blocks queued behind the dK/dV blocks
    unsigned n_blocks = (unsigned)((x_kv + n_heads) * (s / 128));
    if (eight) {
      constexpr int smem_f = smem_kv8 > smem_split ? smem_kv8 : smem_split;
      auto kf = attn_bwd_fused_mfma_kernel<DH, true>;
      static bool fused8_configured = false;
      if (!fused8_configured) {
        PO_HIP_OK(hipFuncSetAttribute(reinterpret_cast<const void*>(kf), hipFuncAttributeMaxDynamicSharedMemorySize,
                                      smem_f));
        fused8_configured = true;
      }
      kf<<<n_blocks, 512, smem_f, stream>>>(qkv, d_o, lse, delta, kv_out, kv_ld, kv_k0, kv_vd, kv_hpb, dqkv, s, h,
          hkv,
                                            group, scale, x_kv, n_heads);
    } else {
      constexpr int smem_f = smem_kv > smem_q ? smem_kv : smem_q;
      auto kf = attn_bwd_fused_mfma_kernel<DH, false>;
      static bool fused4_configured = false;
      if (!fused4_configured) {
        PO_HIP_OK(hipFuncSetAttribute(reinterpret_cast<const void*>(kf), hipFuncAttributeMaxDynamicSharedMemorySize,
                                      smem_f));
        fused4_configured = true;
      }
      kf<<<n_blocks, 256, smem_f, stream>>>(qkv, d_o, lse, delta, kv_out, kv_ld, kv_k0, kv_vd, kv_hpb, dqkv, s, h,
          hkv,
                                            group, scale, x_kv, n_heads);
    }
  } else {
    if (eight)
      kkv8<<<dim3(x_kv, s / 128), 512, smem_kv8, stream>>>(qkv, d_o, lse, delta, kv_out, kv_ld, kv_k0, kv_vd, kv_hpb,
          s,
                                                           h, hkv, group, scale);
    else
      kkv<<<dim3(x_kv, s / 128), 256, smem_kv, stream>>>(qkv, d_o, lse, delta, kv_out, kv_ld, kv_k0, kv_vd, kv_hpb, s,
          h,
                                                         hkv, group, scale);
    if (dq_eight) {
      auto kqs = attn_bwd_dq_split_mfma_kernel<DH>;
      static bool split_configured = false;
      if (!split_configured) {
        PO_HIP_OK(hipFuncSetAttribute(reinterpret_cast<const void*>(kqs), hipFuncAttributeMaxDynamicSharedMemorySize,
                                      smem_split));
        split_configured = true;
      }
      kqs<<<dim3(n_heads, s / 128), 512, smem_split, stream>>>(qkv, d_o, lse, delta, dqkv, s, h, hkv, group, scale);
    } else {
      kq1<<<dim3(n_heads, s / 128), 256, smem_q, stream>>>(qkv, d_o, lse, delta, dqkv, s, h, hkv, group, scale);
    }
  }
  if (split) {
    size_t n = (size_t)s * (2 * hkv / 8);
    attn_group_sum_kernel<DH><<<(unsigned)((n + 255) / 256), 256, 0, stream>>>(partials, dqkv, s, h, hkv, group);
  }
  return launch_ok("attention backward MFMA kernels");
}

bool attention_backward_mfma(const void* qkv, const void* o, const float* lse, const void* d_o, void* dqkv,
                             float* delta, void* partials, int s, int h, int n_heads, int n_kv_heads,
                             hipStream_t stream) {
  if (!attention_mfma_supported(s, h, n_heads, n_kv_heads) || !qkv || !o || !lse || !d_o || !dqkv || !delta ||
      ((uintptr_t)qkv | (uintptr_t)o | (uintptr_t)d_o | (uintptr_t)dqkv) % 16 != 0) {
    set_error("attention_backward_mfma: unsupported s=%d h=%d heads=%d kv_heads=%d or bad pointers", s, h, n_heads,
              n_kv_heads);
    return false;
  }
  if (h / n_heads == 128)
    return launch_bwd<128>((const bf16*)qkv, (const bf16*)o, lse, (const bf16*)d_o, (bf16*)dqkv, delta,
                           (bf16*)partials, s, h, n_heads, n_kv_heads, stream);
  return launch_bwd<64>((const bf16*)qkv, (const bf16*)o, lse, (const bf16*)d_o, (bf16*)dqkv, delta, (bf16*)partials,
                        s, h, n_heads, n_kv_heads, stream);
}

}  // namespace po
