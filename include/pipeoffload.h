/*
 * pipeoffload.h -- C ABI of the MI355X stage + activation-offload library.
 *
 * One pipeline rank's share of a GPT-style model (a "stage": L decoder layers,
 * split into v chunks) runs forward and backward over a stream of in-flight
 * microbatches.  After a unit's forward (a unit = one microbatch of one chunk)
 * its saved activations -- 10 s h elements per layer, the paper's 20 b s h
 * bytes at two bytes per element (Appendix C, selective recomputation), plus the
 * attention log-sum-exp -- can be offloaded to pinned host memory and are
 * reloaded before the unit's backward (Section 1; Section 4.2; Appendix A).
 *
 * Conventions
 *  - Every pointer argument says whether it is HOST or DEVICE memory.  Device
 *    pointers must be on the device that was current at po_stage_create.
 *  - Matrices are row-major.  b = 1: an activation is [s, h].
 *  - Calls enqueue work and return; results are valid after po_synchronize (or
 *    a synchronisation of the compute stream for forward/backward outputs).
 *  - The caller owns parameters, gradients, inputs, outputs and the compute
 *    stream.  The library owns activation slabs, pinned host buffers, its copy
 *    streams, events and workspaces; only the stage itself is ever freed by the
 *    caller (po_stage_destroy).
 *  - Return value 0 = success, negative = po_error; po_last_error() gives text.
 *    No exception crosses this boundary and nothing aborts.
 *  - A stage is not thread-safe; use it from one host thread.
 */
#ifndef PIPEOFFLOAD_H
#define PIPEOFFLOAD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct po_stage po_stage; /* opaque */

typedef enum { PO_F32 = 0, PO_BF16 = 1 } po_dtype;

/* Rank-local op order.  1F1B: Table 1 first row / Appendix A.  Interleaved 1F1B:
 * Section 3.1 (warm-up d(v-1) + 2(d-i) - 1 forwards on rank i). */
/* PO_SCHED_GIS: generalized interleaved schedule with split backward (Sections 3.1, 3.2): every input-gradient
 * pass B is directly followed by the unit's weight-gradient pass W, warm-up g(v-1) + d-i-1 forwards, inner loop
 * over g = po_config.group microbatches (g = d: the paper's GIS, g = ceil(d/2): GIS-H). */
/* PO_SCHED_PO: the uniformly repeated schedule (Section 2; PO in Section 3.2 and Table 1): every microbatch runs
 * the same building block (the steady state of the generalized interleaved schedule with group size g, default
 * ceil(d/2)), 3v unit passes after the previous one; split backward; any m.  With LONGEST_LIFESPAN selection a
 * ratio of 0.5 is the paper's PO-H and 1 its PO-F. */
typedef enum { PO_SCHED_1F1B = 0, PO_SCHED_1F1B_INTERLEAVED = 1, PO_SCHED_GIS = 2, PO_SCHED_PO = 3 } po_schedule;

/* How a whole-job offload ratio picks units.  ALTERNATE_MB: microbatch j is
 * offloaded iff floor((j+1) r) > floor(j r).  LONGEST_LIFESPAN (Section 2):
 * chunks 0 .. ceil(r v) - 1 of every microbatch; equals ALTERNATE_MB if v == 1. */
typedef enum { PO_SEL_ALTERNATE_MB = 0, PO_SEL_LONGEST_LIFESPAN = 1 } po_select;

typedef enum {
  PO_OK = 0,
  PO_E_INVAL = -1,      /* bad argument or unsupported shape */
  PO_E_STATE = -2,      /* call not legal in the unit's state (e.g. backward of a unit still on the host) */
  PO_E_DEVICE_OOM = -3, /* device slab pool cap reached, or hipMalloc failed */
  PO_E_HOST_OOM = -4,   /* pinned host pool cap reached, or hipHostMalloc failed */
  PO_E_HIP = -5         /* a HIP call failed; text in po_last_error() */
} po_error;

typedef struct po_config {
  int32_t n_layers;        /* L: decoder layers held by this rank */
  int32_t n_chunks;        /* v: virtual chunks; L % v == 0 */
  int32_t hidden;          /* h; h % 64 == 0 */
  int32_t n_heads;         /* a; h % a == 0; head size 64 or 128 in bf16 mode */
  int32_t ffn;             /* f; f % 64 == 0 */
  int32_t seq;             /* s */
  int32_t vocab;           /* > 0: chunk 0 starts with wte[token] + wpe[position] and takes int32 tokens */
  int32_t dtype;           /* po_dtype of parameters and activations; gradients are always fp32 */
  int32_t pipeline_degree; /* d of the simulated pipeline */
  int32_t rank;            /* i in [0, d): rank 0 holds the most units in flight */
  int32_t prefetch_passes; /* run_schedule issues a unit's reload this many forward / backward passes before its
                              backward (weight-gradient passes in between are not counted) */
  int32_t copy_streams;    /* 2: separate offload and reload streams; 1: one shared copy stream (Section 4.2) */
  int32_t select_policy;   /* po_select */
  int32_t staged_copies;   /* 0: copy slabs in place; 1: pack into a staging buffer before D2H, unpack after H2D */
  int32_t debug_poison;    /* 1: fill a slab with a NaN pattern whenever it is released */
  int32_t profile_kernels; /* k > 0: po_run_schedule brackets every k-th GEMM launch and every k-th attention
                              launch with HIP events (1 = all; an event pair idles the stream for a few
                              microseconds, so benchmarks sample with an odd k) */
  int32_t group;           /* g, ceil(d/2) <= g <= d; 0 = d for PO_SCHED_GIS, ceil(d/2) for PO_SCHED_PO */
  int32_t weight_stream;   /* 1: weight-gradient work (W passes, and the weight half of po_stage_backward) runs on a
                              stream of its own after the unit's input-gradient work, beside the compute stream;
                              results are bit-identical to 0; gradients are complete after po_synchronize */
  int32_t n_kv_heads;      /* key/value heads of grouped-query attention (Table 2's query groups), a divisor of
                              n_heads; 0 = n_heads (plain multi-head).  The QKV projection is [h, h + 2 hkv],
                              hkv = n_kv_heads * h / n_heads, and the saved k and v shrink accordingly */
  int32_t min_gap_passes;  /* run_schedule does not offload a unit with fewer than this many forward / backward
                              passes between its forward and its backward (Section 4.4); 0 = offload all */
  float ln_eps;            /* LayerNorm epsilon */
  float dropout_p;         /* 0 = none; else the outputs of the attention and MLP output projections are dropped
                              with this probability before the residual add, masks regenerated in backward from
                              (dropout_seed, layer, site, microbatch, position) instead of being stored (App. C) */
  float slot_k;            /* > 0 with PO_SCHED_PO: po_run_schedule places the copies with po_schedule_ops_slots(k =
                              slot_k) instead of the prefetch rule (Section 4.2); 0 = prefetch rule */
  uint64_t host_pool_cap_bytes;   /* 0 = unlimited; else PO_E_HOST_OOM beyond it */
  uint64_t device_pool_cap_bytes; /* 0 = unlimited; else PO_E_DEVICE_OOM beyond it */
  uint64_t dropout_seed;          /* key of the counter-based generator; change it between iterations with
                                     po_set_dropout_seed */
} po_config;

/* One tensor of the flat parameter (and gradient) buffer. */
typedef struct po_param_desc {
  char name[32];        /* "wte", "wpe", or per layer: ln1_g ln1_b w_qkv b_qkv w_o b_o ln2_g ln2_b w_fc1 b_fc1 w_fc2 b_fc2 */
  int32_t layer;        /* -1 for embeddings */
  int32_t reserved;
  int64_t offset_elems; /* offset into the flat buffer, in elements */
  int64_t rows, cols;   /* vectors have rows == 1 */
} po_param_desc;

/* kind: 0 forward, 1 backward (input-gradient pass B in a schedule with W passes), 2 offload, 3 reload,
 * 4 weight-gradient pass W. */
typedef struct po_op {
  int32_t kind, mb, chunk;
  float ratio; /* offload: fraction of the unit's layers (rounded up, lowest layers first) */
} po_op;

typedef struct po_stats {
  double wall_s;            /* host wall time of the last po_run_schedule, enqueue to drained */
  double tokens_per_s;      /* m * s / wall_s */
  double compute_busy_s;    /* sum of compute-pass durations (HIP events on the compute stream) */
  double d2h_busy_s;        /* sum of offload copy durations */
  double h2d_busy_s;        /* sum of reload copy durations */
  double pack_busy_s;       /* sum of pack + unpack kernel durations (staged copies only) */
  double compute_span_s;    /* first compute pass start to last compute pass end */
  double gemm_busy_s;       /* profile_kernels: sum of the timed GEMM launches' durations on the compute stream */
  double gemm_flops;        /* profile_kernels: 2 M N K summed over those launches */
  double attn_busy_s;       /* profile_kernels: sum of the timed attention forward/backward launches' durations */
  double attn_flops;        /* profile_kernels: causal model flops of those, 2 s^2 h forward, 4 s^2 h backward */
  double copy_hidden_s;     /* part of d2h_busy_s + h2d_busy_s during which a compute pass was running as well */
  uint64_t bytes_d2h, bytes_h2d;
  uint64_t peak_slab_bytes;      /* high-water mark of activation slab bytes in use (incl. staging) */
  uint64_t pool_bytes_allocated; /* device bytes the slab pool holds */
  uint64_t host_bytes_allocated; /* pinned bytes the host pool holds */
  uint64_t workspace_bytes;      /* temporaries: recompute buffers, gradient workspaces */
  int32_t peak_resident_units;   /* high-water mark of units with at least one layer resident */
  int32_t peak_in_flight_units;  /* forwarded and not yet backwarded */
  int32_t n_compute_passes, n_offloads, n_reloads, n_gemm_launches;
} po_stats;

/* Fills *cfg with defaults (1 chunk, fp32, d = 1, prefetch 2, two copy streams, eps 1e-5). HOST. */
void po_config_default(po_config* cfg);

/* Thread-local text of the last error. */
const char* po_last_error(void);

/* ---- parameter layout (pure host code; usable without a GPU) ------------- */
/* Total elements of the flat parameter buffer of this config. */
int po_param_count(const po_config* cfg, int64_t* n_elems);
/* Writes up to *n descriptors into out (HOST) and sets *n to the number of tensors.
 * Call with out == NULL to query the count. */
int po_param_layout(const po_config* cfg, po_param_desc* out, int32_t* n);
/* Bytes of saved activations per layer: 10 s h elements + 4 a s (fp32 log-sum-exp), each tensor 256-byte aligned. */
int po_saved_bytes_per_layer(const po_config* cfg, uint64_t* bytes);

/* ---- schedule (pure host code; usable without a GPU) --------------------- */
/* The op list one rank executes, offload and reload ops included (Section 4.2 on a
 * single rank: offload right after the forward, reload `prefetch` compute passes
 * ahead of the backward).  out may be NULL to query *n. */
int po_schedule_ops(int32_t schedule, int32_t d, int32_t rank, int32_t v, int32_t m, int32_t group, float ratio,
                    int32_t policy, int32_t prefetch, int32_t min_gap, po_op* out, int32_t* n);

/* Section 4.2 (Figure 7): op list of the uniformly repeated schedule (PO_SCHED_PO, group as there) with the copies
 * of chunks 0 .. n_offload_chunks-1 of every microbatch placed into the slots of one shared copy stream on the
 * schedule's unit-time timeline (F = B = W = 1, bubbles kept): slot pairs of 3k units, an offload slot followed
 * by a reload slot, k = a unit's round trip over its F + B + W time (Eq. 1).  Offloads take the earliest free
 * slot that starts after their forward has ended, reloads the latest free slot that ends before their backward
 * starts; a unit whose reload slot would start before its offload slot has ended is not offloaded (Section 4.4).
 * A copy op stands before the first pass that starts no earlier than its slot.  out may be NULL to query *n. HOST. */
int po_schedule_ops_slots(int32_t d, int32_t rank, int32_t v, int32_t m, int32_t group, int32_t n_offload_chunks,
                          double k, po_op* out, int32_t* n);

/* Eq. 1: k = 10 / (3 (6h + s)) * B_c / B_o, with B_c in flop/s and B_o in byte/s. */
double po_offload_k(int32_t h, int32_t s, double compute_flops_per_s, double link_bytes_per_s);

/* Largest offload ratio whose transfers still hide behind compute for a given k (Section 2: k = T_o / T_c is the
 * proportion indicator; everything can be offloaded when k <= 1, else a fraction 1 / k): min(1, 1 / k); 1 for k <= 0. */
double po_offload_ratio_for_k(double k);

/* ---- stage ---------------------------------------------------------------- */
/* compute_stream: a hipStream_t (as void*) on the current device, NULL = default
 * stream.  Creates copy streams, events and workspaces; slabs and pinned buffers
 * grow on demand and are kept until destroy. */
int po_stage_create(const po_config* cfg, void* compute_stream, po_stage** out);
void po_stage_destroy(po_stage* st);

/* params: DEVICE, po_param_count elements of cfg.dtype.  grads: DEVICE, the same
 * number of fp32 elements; backward ADDS into it, the caller zeroes it. */
int po_bind_params(po_stage* st, const void* params, float* grads);

/* Forward of unit (mb, chunk) on the compute stream (per layer: LN, QKV, causal
 * attention, out-proj + residual, LN, FC1 + GeLU, FC2 + residual).
 * x_in: DEVICE [s, h] of cfg.dtype, or int32 tokens [s] when vocab > 0 and chunk == 0.  A token array is read
 * again by the unit's backward (the embedding gradient scatters by token): it must stay valid and unchanged until
 * that backward (po_stage_backward, or po_stage_backward_weight under a split schedule) has run on the device.
 * Activation inputs are copied into the unit's slab and may be reused as soon as the forward has run.
 * y_out: DEVICE [s, h].  The unit becomes RESIDENT. */
int po_stage_forward(po_stage* st, int32_t mb, int32_t chunk, const void* x_in, void* y_out);

/* Backward of a RESIDENT unit (waits for an outstanding reload).  dy: DEVICE [s, h].
 * dx: DEVICE [s, h], may be NULL when the unit starts with the embedding.
 * LayerNorm and GeLU outputs are recomputed (Appendix C).  Frees the unit. */
int po_stage_backward(po_stage* st, int32_t mb, int32_t chunk, const void* dy, void* dx);

/* New dropout key for the following forward passes; PO_E_STATE while a unit is in flight. */
int po_set_dropout_seed(po_stage* st, uint64_t seed);

/* Split backward (Section 3.1, zero-bubble strategy).  po_stage_backward_input is the B pass: it computes the
 * activation gradients only (dx as in po_stage_backward) and keeps, in a library-owned buffer, what the W pass
 * needs; the unit keeps its activations.  po_stage_backward_weight is the W pass: it adds the unit's parameter
 * gradients (the same values, bit for bit, as the fused po_stage_backward) and frees the unit.  dy must stay
 * valid and unchanged until the W pass has run on the device.  A unit between its B and W pass can be neither
 * offloaded nor reloaded (PO_E_STATE). */
int po_stage_backward_input(po_stage* st, int32_t mb, int32_t chunk, const void* dy, void* dx);
int po_stage_backward_weight(po_stage* st, int32_t mb, int32_t chunk);

/* Asynchronously moves the ceil(ratio * Lu) lowest layers of a RESIDENT unit to pinned
 * host memory on the offload stream once its forward has finished, and releases their
 * device slabs (Section 4.2; Appendix C buffer management).  The copies are issued from
 * the highest of those layers down: the reload brings layers back in the same order, and
 * the layer the backward needs first should not be the one that leaves last. */
int po_offload(po_stage* st, int32_t mb, int32_t chunk, float ratio);

/* Asynchronously brings an offloaded unit back on the reload stream, top layer first;
 * a no-op for a unit with nothing offloaded.  The backward then waits for each layer's
 * copy right before it reads that layer, so the lower layers travel while the upper
 * ones are differentiated. */
int po_reload(po_stage* st, int32_t mb, int32_t chunk);

/* Runs a whole rank-local schedule: po_schedule_ops(schedule, d, rank, v, m, ratio, ...)
 * executed with the four calls above.  Arrays are HOST arrays of DEVICE pointers,
 * indexed [chunk * m + mb], length m * v.  dx entries may be NULL for embedding
 * units.  stats (HOST) may be NULL.  Returns after everything has drained.
 * If the environment variable PIPEOFFLOAD_TRACE names a file, every run appends
 * "# run" and one line per timed span, "kind start_ms stop_ms" measured from the
 * first span (kind 0 compute pass, 1 D2H copy, 2 H2D copy, 3 pack/unpack, 4 GEMM
 * launch, 5 attention launch; 4 and 5 only with profile_kernels). */
int po_run_schedule(po_stage* st, int32_t schedule, int32_t n_microbatches, float offload_ratio,
                    const void* const* x_in, void* const* y_out, const void* const* dy, void* const* dx,
                    po_stats* stats);

int po_synchronize(po_stage* st);
/* Abandons every unit that is still in flight: waits for all streams, then returns the units' device slabs, pinned
 * buffers and gradient buffers to the pools (nothing is freed, parameter gradients already added stay).  After a
 * call that failed half way (a pool cap, for example) this brings the stage back to a state in which
 * po_stage_forward and po_run_schedule are legal again. */
int po_stage_reset(po_stage* st);
int po_get_stats(const po_stage* st, po_stats* out);

/* ---- single operations (what the stage is built from; for tests and
 * micro-benchmarks).  All pointers DEVICE, stream = hipStream_t or NULL. ----- */

/* y = LN(x) * gain + shift, rows x h (either LayerNorm of a layer; recomputed in backward, Appendix C). */
int po_op_layernorm_forward(int32_t dtype, const void* x, const void* gain, const void* shift, void* y,
                            int32_t rows, int32_t h, float eps, void* stream);
/* dx = dres + LNbwd(dn; x, gain); dgain += ..., dshift += ... (fp32): backward of either LayerNorm of a layer.
 * partials: fp32 workspace of po_op_layernorm_backward_workspace(rows, h) bytes. */
int po_op_layernorm_backward(int32_t dtype, const void* dn, const void* x, const void* gain, const void* dres,
                             void* dx, float* dgain, float* dshift, float* partials, int32_t rows, int32_t h,
                             float eps, void* stream);
uint64_t po_op_layernorm_backward_workspace(int32_t rows, int32_t h);

/* C = op(A) op(B) with the epilogues of the stage (the four projections of a layer: forward, input gradient
 * and weight gradient).
 * trans_a == 0: A is [M, K]; 1: A is [K, M].  trans_b == 0: B is [K, N]; 1: B is [N, K].
 * bias [N] and residual [M, N] may be NULL.  out [M, N] of dtype may be NULL.
 * gelu_out: if not NULL receives gelu(out).  gelu_u: if not NULL, out = result * gelu'(gelu_u)
 * and gelu_out = gelu(gelu_u).  acc_f32: if not NULL, acc_f32 [M, N] += result. */
int po_op_gemm(int32_t dtype, int32_t trans_a, int32_t trans_b, int32_t M, int32_t N, int32_t K,
               const void* A, int32_t lda, const void* B, int32_t ldb, const void* bias, const void* residual,
               void* out, void* gelu_out, const void* gelu_u, float* acc_f32, int32_t force_generic, void* stream);

/* n <= 4 independent weight-gradient products in one launch (bf16 operands, the matrix-core kernel only):
 * acc_f32[i] [M[i], N[i]] += A[i]^T B[i] with A[i] DEVICE [K[i], M[i]] (row stride lda[i]) and B[i] DEVICE
 * [K[i], N[i]] (row stride ldb[i]); acc_f32[i] DEVICE fp32 with row stride ldc[i].  The arrays themselves are HOST
 * arrays of length n.  Every M[i], N[i] must be a multiple of 256 and every K[i] of 64, else PO_E_INVAL (use
 * po_op_gemm per product then).  Each product equals po_op_gemm(trans_a = 1, trans_b = 0, acc_f32) bit for bit;
 * the stage runs the four parameter-gradient products of a layer this way (Section 3.1's W pass). */
int po_op_gemm_grouped(int32_t n, const int32_t* M, const int32_t* N, const int32_t* K, const void* const* A,
                       const int32_t* lda, const void* const* B, const int32_t* ldb, float* const* acc_f32,
                       const int32_t* ldc, void* stream);

/* Pure host code: the output tile (rows, columns) of the bf16 matrix-core kernel that po_op_gemm and the stage
 * use for an M x N result whose K is a multiple of 64: 256 x 256, 256 x 192 or 128 x 128, chosen so that a round of
 * tiles fills the 256 compute units; 0, 0 when M, N fit none of them (the shape-generic kernel runs instead). */
int po_op_gemm_tile(int32_t M, int32_t N, int32_t* tile_rows, int32_t* tile_cols);

/* Causal attention forward: qkv [s, h + 2 hkv] (q | k | v blocks, hkv = n_kv_heads * h / n_heads;
 * n_kv_heads = 0 means n_heads, i.e. [s, 3h]), o [s, h], lse [a, s] fp32.  With n_kv_heads < n_heads query head t
 * reads key/value head t / (n_heads / n_kv_heads) (grouped-query attention, Table 2). */
int po_op_attention_forward(int32_t dtype, const void* qkv, void* o, float* lse, int32_t s, int32_t h,
                            int32_t n_heads, int32_t n_kv_heads, int32_t force_generic, void* stream);
/* Causal attention backward: dqkv laid out like qkv; delta: fp32 workspace [a, s]; partials: NULL, or
 * a [s, 2h] workspace of dtype that lets grouped-query shapes with few key/value heads compute dK/dV per query
 * head and add the groups up afterwards (same result up to the rounding of the per-head terms). */
int po_op_attention_backward(int32_t dtype, const void* qkv, const void* o, const float* lse, const void* d_o,
                             void* dqkv, float* delta, void* partials, int32_t s, int32_t h, int32_t n_heads,
                             int32_t n_kv_heads, int32_t force_generic, void* stream);

/* out[r, c] = x[r, c] * keep(r, c) / (1 - p): one dropout site (site 0: after the attention output projection,
 * 1: after the MLP output projection) of global layer `layer` for microbatch `mb`.  keep(r, c) is true iff word
 * c % 4 of Philox4x32-10 with counter (c / 4, r, 2 * layer + site, mb) and key (seed mod 2^32, seed div 2^32) is
 * >= round(p * 2^32).  The same map is the site's backward (Appendix C: dropout is recomputed, not stored). */
int po_op_dropout(int32_t dtype, const void* x, void* out, int32_t rows, int32_t cols, float p, uint64_t seed,
                  int32_t layer, int32_t site, int32_t mb, void* stream);

/* acc[N] += column sums of x [rows, N] (bias gradients), deterministic: row chunks
 * are reduced to partials in `workspace` (fp32, po_op_colsum_workspace bytes), then added in chunk order. */
uint64_t po_op_colsum_workspace(int32_t rows, int32_t n);
int po_op_colsum_accumulate(int32_t dtype, const void* x, float* acc, float* workspace, int32_t rows, int32_t n,
                            void* stream);

/* For callers that cannot allocate device memory or carry a workspace (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): po_op_colsum_accumulate with the chunk partials in an 8 MiB device array
 * built into the library instead of a caller workspace.  Allocates nothing and calls no allocating routine; x
 * [rows, n] and acc [n] are DEVICE memory of the caller as above; same arithmetic, same order, same result bit
 * for bit.  n must be even and at most 32768 (any rows), else PO_E_INVAL with text.  The first call on a device
 * resolves the array's address on that device (make that call outside a capture).  Every call on one GPU uses that
 * GPU's one array: calls that overlap there (two streams, two threads) race; calls in stream order do not, and
 * nothing in the array needs clearing between calls.  The array is held on each GPU the library runs on until the
 * process ends. */
int po_op_colsum_accumulate_static(int32_t dtype, const void* x, float* acc, int32_t rows, int32_t n, void* stream);

/* Gather n_seg segments into one contiguous buffer / scatter them back (a layer's saved set to and from a
 * staging buffer, Section 4.2).
 * seg_ptrs: HOST array of DEVICE pointers; seg_bytes: HOST array, each a multiple of 16.
 * Segments land back to back in `packed` in array order. */
int po_op_pack(const void* const* seg_ptrs, const uint64_t* seg_bytes, int32_t n_seg, void* packed, void* stream);
int po_op_unpack(void* const* seg_ptrs, const uint64_t* seg_bytes, int32_t n_seg, const void* packed, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PIPEOFFLOAD_H */
