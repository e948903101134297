// The stage runtime: parameter layout, activation slabs, pinned host slabs, the
// copy streams with their event dependencies, the per-layer forward / backward
// sequences and the schedule executor.
//
// Memory plan.  A layer's saved activations (Appendix C: layer input, q|k|v,
// attention output, second LayerNorm's input, MLP pre-activation; plus the
// attention log-sum-exp) live in one contiguous "layer slab" that the forward
// kernels write directly.  Slabs come from a pool that grows on demand and is
// never shrunk; a unit holds Lu of them.  Offload moves a slab to a pinned host
// slab of the same size and hands the device slab back to the pool at once (in
// host order); the pool remembers, per slab, the event after which it may be
// overwritten, and whoever takes the slab next makes its stream wait for that
// event (Appendix C, deterministic device memory management: buffers are
// handed out in host order and guarded by events, not by deferred frees).
//
// Streams.  Compute runs on the caller's stream.  D2H copies run on the offload
// stream after the unit's forward-done event; H2D copies run on the reload
// stream (the same stream when copy_streams == 1, Section 4.2) after an event
// recorded on the compute stream when po_reload is called, so a reload never
// starts earlier than the compute work enqueued before it.  A unit's layers are
// copied from the top layer down in both directions, and the backward waits for
// a layer's reload-done event only when it reaches that layer, so the lower
// layers travel while the upper ones are differentiated.
#include <algorithm>
#include <chrono>
#include <deque>
#include <map>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <vector>

#include "../../include/pipeoffload.h"
#include "kernels.h"

namespace po {

bool build_schedule(int schedule, int d, int rank, int v, int m, int group, float ratio, int policy, int prefetch,
                    int min_gap,
                    std::vector<po_op>& ops);
bool build_slot_schedule(int d, int rank, int v, int m, int g, int n_sel, double k, std::vector<po_op>& ops);

#define PO_HIP(expr)                                                                          \
  do {                                                                                        \
    hipError_t e__ = (expr);                                                                  \
    if (e__ != hipSuccess) {                                                                  \
      set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e__), __FILE__, __LINE__);  \
      return PO_E_HIP;                                                                        \
    }                                                                                         \
  } while (0)

#define PO_K(call)                   \
  do {                               \
    if (!(call)) return PO_E_HIP;    \
  } while (0)

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ------------------------------------------------------------------------------
// Parameter layout
// ------------------------------------------------------------------------------
struct ParamLayout {
  std::vector<po_param_desc> descs;
  int64_t total = 0;
  int64_t emb_wte = -1, emb_wpe = -1;
  int64_t layer_stride = 0, layer0 = 0;
  // per-layer offsets relative to the layer's base
  int64_t ln1_g, ln1_b, w_qkv, b_qkv, w_o, b_o, ln2_g, ln2_b, w_fc1, b_fc1, w_fc2, b_fc2;
};

// Key/value heads (0 in the config = as many as query heads) and the width of the QKV projection,
// h for the queries plus n_kv_heads * head_dim each for keys and values.
static int kv_heads_of(const po_config& c) { return c.n_kv_heads > 0 ? c.n_kv_heads : c.n_heads; }
static int qkv_width_of(const po_config& c) { return c.hidden + 2 * kv_heads_of(c) * (c.hidden / c.n_heads); }

int validate_config(const po_config* c) {
  if (!c) {
    set_error("config is NULL");
    return PO_E_INVAL;
  }
  if (c->n_layers < 1 || c->n_chunks < 1 || c->n_layers % c->n_chunks != 0 || c->hidden < 64 ||
      c->hidden % 64 != 0 || c->n_heads < 1 || c->hidden % c->n_heads != 0 || c->ffn < 64 || c->ffn % 64 != 0 ||
      c->seq < 1 || c->vocab < 0 || (c->dtype != PO_F32 && c->dtype != PO_BF16) || c->pipeline_degree < 1 ||
      c->rank < 0 || c->rank >= c->pipeline_degree || c->prefetch_passes < 0 ||
      (c->copy_streams != 1 && c->copy_streams != 2) || c->hidden / c->n_heads > 256 ||
      (c->hidden / c->n_heads) % 8 != 0 || !(c->ln_eps > 0.f) || c->group < 0 || c->group > c->pipeline_degree ||
      (c->group > 0 && 2 * c->group < c->pipeline_degree) || (c->weight_stream != 0 && c->weight_stream != 1) ||
      c->min_gap_passes < 0 || c->n_kv_heads < 0 || !(c->dropout_p >= 0.f && c->dropout_p < 1.f) ||
      !(c->slot_k >= 0.f) || (c->n_kv_heads > 0 && c->n_heads % c->n_kv_heads != 0)) {
    set_error(
        "invalid config: L=%d v=%d h=%d a=%d kv_heads=%d f=%d s=%d vocab=%d dtype=%d d=%d rank=%d prefetch=%d "
        "copy_streams=%d group=%d weight_stream=%d min_gap=%d dropout_p=%g slot_k=%g ln_eps=%g",
        c->n_layers, c->n_chunks, c->hidden, c->n_heads, c->n_kv_heads, c->ffn, c->seq, c->vocab, c->dtype,
        c->pipeline_degree, c->rank, c->prefetch_passes, c->copy_streams, c->group, c->weight_stream,
        c->min_gap_passes, (double)c->dropout_p, (double)c->slot_k, (double)c->ln_eps);
    return PO_E_INVAL;
  }
  return PO_OK;
}

static void add_desc(ParamLayout& pl, const char* name, int layer, int64_t rows, int64_t cols, int64_t* rel,
                     int64_t base) {
  po_param_desc d;
  memset(&d, 0, sizeof(d));
  strncpy(d.name, name, sizeof(d.name) - 1);
  d.layer = layer;
  d.offset_elems = pl.total;
  d.rows = rows;
  d.cols = cols;
  if (rel) *rel = pl.total - base;
  pl.total += rows * cols;
  pl.descs.push_back(d);
}

void build_param_layout(const po_config& c, ParamLayout& pl) {
  int64_t h = c.hidden, f = c.ffn;
  pl.descs.clear();
  pl.total = 0;
  if (c.vocab > 0) {
    pl.emb_wte = pl.total;
    add_desc(pl, "wte", -1, c.vocab, h, nullptr, 0);
    pl.emb_wpe = pl.total;
    add_desc(pl, "wpe", -1, c.seq, h, nullptr, 0);
  }
  pl.layer0 = pl.total;
  for (int l = 0; l < c.n_layers; ++l) {
    int64_t base = pl.total;
    int64_t dummy;
    bool first = l == 0;
    add_desc(pl, "ln1_g", l, 1, h, first ? &pl.ln1_g : &dummy, base);
    add_desc(pl, "ln1_b", l, 1, h, first ? &pl.ln1_b : &dummy, base);
    add_desc(pl, "w_qkv", l, h, qkv_width_of(c), first ? &pl.w_qkv : &dummy, base);
    add_desc(pl, "b_qkv", l, 1, qkv_width_of(c), first ? &pl.b_qkv : &dummy, base);
    add_desc(pl, "w_o", l, h, h, first ? &pl.w_o : &dummy, base);
    add_desc(pl, "b_o", l, 1, h, first ? &pl.b_o : &dummy, base);
    add_desc(pl, "ln2_g", l, 1, h, first ? &pl.ln2_g : &dummy, base);
    add_desc(pl, "ln2_b", l, 1, h, first ? &pl.ln2_b : &dummy, base);
    add_desc(pl, "w_fc1", l, h, f, first ? &pl.w_fc1 : &dummy, base);
    add_desc(pl, "b_fc1", l, 1, f, first ? &pl.b_fc1 : &dummy, base);
    add_desc(pl, "w_fc2", l, f, h, first ? &pl.w_fc2 : &dummy, base);
    add_desc(pl, "b_fc2", l, 1, h, first ? &pl.b_fc2 : &dummy, base);
    if (first) pl.layer_stride = pl.total - base;
  }
}

// ------------------------------------------------------------------------------
// Saved-activation layout of one layer slab
// ------------------------------------------------------------------------------
struct SlabLayout {
  size_t off_x, off_qkv, off_o, off_x1, off_u, off_lse, bytes;
  size_t sz_x, sz_qkv, sz_o, sz_x1, sz_u, sz_lse;
  size_t packed_bytes;  // segments back to back, no alignment padding
};

void build_slab_layout(const po_config& c, SlabLayout& sl) {
  size_t E = c.dtype == PO_BF16 ? 2 : 4;
  size_t s = c.seq, h = c.hidden, f = c.ffn, a = c.n_heads;
  sl.sz_x = s * h * E;
  sl.sz_qkv = s * (size_t)qkv_width_of(c) * E;
  sl.sz_o = s * h * E;
  sl.sz_x1 = s * h * E;
  sl.sz_u = s * f * E;
  sl.sz_lse = a * s * 4;
  size_t off = 0;
  sl.off_x = off;
  off = align_up(off + sl.sz_x, 256);
  sl.off_qkv = off;
  off = align_up(off + sl.sz_qkv, 256);
  sl.off_o = off;
  off = align_up(off + sl.sz_o, 256);
  sl.off_x1 = off;
  off = align_up(off + sl.sz_x1, 256);
  sl.off_u = off;
  off = align_up(off + sl.sz_u, 256);
  sl.off_lse = off;
  off = align_up(off + sl.sz_lse, 256);
  sl.bytes = off;
  sl.packed_bytes = align_up(sl.sz_x, 16) + align_up(sl.sz_qkv, 16) + align_up(sl.sz_o, 16) +
                    align_up(sl.sz_x1, 16) + align_up(sl.sz_u, 16) + align_up(sl.sz_lse, 16);
}

// ------------------------------------------------------------------------------
// Pools
// ------------------------------------------------------------------------------
struct PoolBuf {
  char* ptr = nullptr;
  hipEvent_t free_event = nullptr;  // work after which the buffer may be overwritten
  hipStream_t guard_stream = nullptr;  // stream that event was recorded on
  bool guarded = false;
};

struct Pool {
  bool host = false;
  size_t buf_bytes = 0;
  uint64_t cap = 0;
  std::vector<PoolBuf> bufs;
  std::deque<int> free_list;
  int in_use = 0;

  uint64_t allocated() const { return (uint64_t)bufs.size() * buf_bytes; }

  // Takes a buffer; `stream` (the first stream that will write it) waits for the guard event.
  int acquire(hipStream_t stream, int* out) {
    int idx;
    if (!free_list.empty()) {
      // Oldest buffer that needs no wait (never used, or handed back on the taker's own stream, where stream
      // order already protects it); else the oldest of all, whose guard event the taker's stream waits for.
      auto pick = free_list.begin();
      for (auto it = free_list.begin(); it != free_list.end(); ++it)
        if (!bufs[*it].guarded || bufs[*it].guard_stream == stream) {
          pick = it;
          break;
        }
      idx = *pick;
      free_list.erase(pick);
      if (bufs[idx].guarded && bufs[idx].guard_stream != stream)
        PO_HIP(hipStreamWaitEvent(stream, bufs[idx].free_event, 0));
    } else {
      if (cap && allocated() + buf_bytes > cap) {
        set_error("%s pool cap of %llu bytes reached (%zu buffers of %zu bytes in use)", host ? "host" : "device",
                  (unsigned long long)cap, bufs.size(), buf_bytes);
        return host ? PO_E_HOST_OOM : PO_E_DEVICE_OOM;
      }
      PoolBuf b;
      hipError_t e = host ? hipHostMalloc((void**)&b.ptr, buf_bytes, hipHostMallocDefault)
                          : hipMalloc((void**)&b.ptr, buf_bytes);
      if (e != hipSuccess) {
        (void)hipGetLastError();
        set_error("%s of %zu bytes failed: %s", host ? "hipHostMalloc" : "hipMalloc", buf_bytes,
                  hipGetErrorString(e));
        return host ? PO_E_HOST_OOM : PO_E_DEVICE_OOM;
      }
      if (hipEventCreateWithFlags(&b.free_event, hipEventDisableTiming) != hipSuccess) {
        (void)(host ? hipHostFree(b.ptr) : hipFree(b.ptr));
        set_error("creating a pool buffer's guard event failed");
        return PO_E_HIP;
      }
      bufs.push_back(b);
      idx = (int)bufs.size() - 1;
    }
    ++in_use;
    *out = idx;
    return PO_OK;
  }

  // Hands a buffer back; it may be overwritten once the work enqueued on `stream` so far is done.
  int release(int idx, hipStream_t stream) {
    PO_HIP(hipEventRecord(bufs[idx].free_event, stream));
    bufs[idx].guard_stream = stream;
    bufs[idx].guarded = true;
    free_list.push_back(idx);
    --in_use;
    return PO_OK;
  }

  void destroy() {
    for (PoolBuf& b : bufs) {
      if (b.free_event) (void)hipEventDestroy(b.free_event);
      if (b.ptr) (void)(host ? hipHostFree(b.ptr) : hipFree(b.ptr));
    }
    bufs.clear();
    free_list.clear();
    in_use = 0;
  }
};

// Reusable events (timing enabled where asked).
struct EventBank {
  std::vector<hipEvent_t> ev;
  size_t next = 0;
  unsigned flags = 0;
  int get(hipEvent_t* out) {
    if (next == ev.size()) {
      hipEvent_t e;
      PO_HIP(hipEventCreateWithFlags(&e, flags));
      ev.push_back(e);
    }
    *out = ev[next++];
    return PO_OK;
  }
  void reset() { next = 0; }
  void destroy() {
    for (hipEvent_t e : ev) (void)hipEventDestroy(e);
    ev.clear();
    next = 0;
  }
};

enum LayerState { L_EMPTY = 0, L_RESIDENT, L_HOST };

struct UnitLayer {
  int state = L_EMPTY;
  int dev = -1;              // device slab index
  int hostbuf = -1;          // host slab index
  hipEvent_t d2h_done = nullptr;
  hipEvent_t h2d_done = nullptr;  // non-null: backward must wait for it
};

struct Unit {
  bool live = false;
  std::vector<UnitLayer> layers;
  hipEvent_t fwd_done = nullptr;
  const void* x_in = nullptr;  // tokens pointer for embedding units (needed again in backward)
  // split backward: set by the input-gradient pass, consumed by the weight-gradient pass
  bool weight_pending = false;
  int grad_buf = -1;            // buffer of the gradient pool holding this unit's BwdBufs tensors
  const void* dy_top = nullptr;  // the caller's upstream gradient (read again by the weight-gradient pass)
  hipEvent_t b_done = nullptr;   // end of the input-gradient pass on the compute stream
};

struct TimedSpan {
  hipEvent_t start, stop;
  int kind;  // 0 compute pass, 1 d2h, 2 h2d, 3 pack/unpack, 4 gemm, 5 attention
  double flops;
};

}  // namespace po

using namespace po;

struct po_stage {
  po_config cfg;
  ParamLayout pl;
  SlabLayout sl;
  int Lu = 0;
  size_t E = 2;
  hipStream_t compute = nullptr, offload = nullptr, reload = nullptr;
  hipStream_t wstream = nullptr;  // weight-gradient passes run here when cfg.weight_stream is set
  bool own_reload_stream = false;
  const char* params = nullptr;
  float* grads = nullptr;
  Pool dev_pool, host_pool;
  Pool grad_pool;  // per-unit gradient tensors between a B pass and its W pass (split backward only)
  size_t gl_sh = 0, gl_sf = 0, gl_s3h = 0, gl_lnws = 0, gl_layer = 0;  // layout of one such buffer
  EventBank sync_events, time_events;
  std::map<int64_t, Unit> units;
  std::vector<TimedSpan> spans;
  // workspaces
  char* ws = nullptr;
  size_t ws_bytes = 0;
  char *w_n, *w_g, *w_du, *w_dqkv, *w_do, *w_dx1, *w_dn, *w_dn1, *w_dy[2], *w_x0;
  char* w_dkv_part = nullptr;  // [s, 2h] per-query-head dK/dV of grouped-query attention (null with multi-head)
  char* w_dz[2];  // dropout-masked gradients of the fused backward
  char* w_n_w;  // the two LayerNorm outputs recomputed by the weight-gradient half (own buffers: it may run on its own stream)
  float *w_delta, *w_lnws, *w_lnws1, *w_colws_w;
  // accounting
  int resident_units = 0, in_flight_units = 0;
  po_stats stats;
  bool collect_timing = false;
  uint64_t gemm_launch_counter = 0, attn_launch_counter = 0;  // for profile_kernels sampling

  void note_usage() {
    uint64_t b = (uint64_t)dev_pool.in_use * sl.bytes;
    if (b > stats.peak_slab_bytes) stats.peak_slab_bytes = b;
    if (resident_units > stats.peak_resident_units) stats.peak_resident_units = resident_units;
    if (in_flight_units > stats.peak_in_flight_units) stats.peak_in_flight_units = in_flight_units;
  }
  const char* P(int layer, int64_t rel) const {
    return params + (size_t)(pl.layer0 + (int64_t)layer * pl.layer_stride + rel) * E;
  }
  float* G(int layer, int64_t rel) const { return grads + pl.layer0 + (int64_t)layer * pl.layer_stride + rel; }
};

namespace po {

static int64_t unit_key(int mb, int chunk) { return ((int64_t)chunk << 32) | (uint32_t)mb; }

static int span_begin(po_stage* st, hipStream_t stream, int kind, size_t* idx) {
  if (!st->collect_timing) {
    *idx = (size_t)-1;
    return PO_OK;
  }
  TimedSpan sp;
  sp.kind = kind;
  sp.flops = 0.0;
  int rc = st->time_events.get(&sp.start);
  if (rc) return rc;
  rc = st->time_events.get(&sp.stop);
  if (rc) return rc;
  PO_HIP(hipEventRecord(sp.start, stream));
  st->spans.push_back(sp);
  *idx = st->spans.size() - 1;
  return PO_OK;
}
static int span_end(po_stage* st, hipStream_t stream, size_t idx) {
  if (idx == (size_t)-1) return PO_OK;
  PO_HIP(hipEventRecord(st->spans[idx].stop, stream));
  return PO_OK;
}

static bool unit_has_resident_layer(const Unit& u) {
  for (const UnitLayer& l : u.layers)
    if (l.state == L_RESIDENT) return true;
  return false;
}

// ------------------------------------------------------------------------------
// Layer forward / backward
// ------------------------------------------------------------------------------
static Epilogue make_ep(int ldc) {
  Epilogue e;
  memset(&e, 0, sizeof(e));
  e.ldc = ldc;
  return e;
}

// GEMM / attention launches of the stage.  profile_kernels = k > 0 brackets every k-th GEMM launch and every
// k-th attention launch of a run with events (k = 1: all).  An event pair costs a few microseconds of idle
// stream, so k > 1 samples; an odd k that is coprime to the 9 GEMM launches of a layer (12 where the weight
// gradients are not one grouped launch) and its 2 attention launches walks through all of their shapes.
static bool sample_launch(po_stage* st, uint64_t& counter) {
  int k = st->cfg.profile_kernels;
  if (!st->collect_timing || k <= 0) return false;
  return counter++ % (uint64_t)k == 0;
}

static int st_gemm(po_stage* st, int ta, int tb, int M, int N, int K, const void* A, int lda, const void* B, int ldb,
                   const Epilogue& e, hipStream_t q = nullptr) {
  if (!q) q = st->compute;
  bool prof = sample_launch(st, st->gemm_launch_counter);
  size_t span = (size_t)-1;
  if (prof) {
    int rc = span_begin(st, q, 4, &span);
    if (rc) return rc;
    st->spans[span].flops = 2.0 * M * N * K;
  }
  PO_K(gemm(st->cfg.dtype, ta, tb, M, N, K, A, lda, B, ldb, e, false, q));
  return span_end(st, q, span);
}

static int st_gemm_grouped(po_stage* st, int n, const GemmProblem* prob, hipStream_t q) {
  bool prof = sample_launch(st, st->gemm_launch_counter);
  size_t span = (size_t)-1;
  if (prof) {
    int rc = span_begin(st, q, 4, &span);
    if (rc) return rc;
    for (int i = 0; i < n; ++i) st->spans[span].flops += 2.0 * prob[i].M * prob[i].N * prob[i].K;
  }
  PO_K(gemm_mfma_grouped_accumulate(n, prob, q));
  return span_end(st, q, span);
}

static int st_attention(po_stage* st, bool backward, const void* qkv, void* o, float* lse, const void* d_o,
                        void* dqkv) {
  const po_config& c = st->cfg;
  bool prof = sample_launch(st, st->attn_launch_counter);
  size_t span = (size_t)-1;
  if (prof) {
    int rc = span_begin(st, st->compute, 5, &span);
    if (rc) return rc;
    st->spans[span].flops = (backward ? 4.0 : 2.0) * c.seq * (double)c.seq * c.hidden;
  }
  if (backward)
    PO_K(attention_backward(c.dtype, qkv, o, lse, d_o, dqkv, st->w_delta, st->w_dkv_part, c.seq, c.hidden, c.n_heads,
                            kv_heads_of(c), false,
                            st->compute));
  else
    PO_K(attention_forward(c.dtype, qkv, o, lse, c.seq, c.hidden, c.n_heads, kv_heads_of(c), false, st->compute));
  return span_end(st, st->compute, span);
}

#define PO_RC(call)          \
  do {                       \
    int rc__ = (call);       \
    if (rc__) return rc__;   \
  } while (0)

// Dropout site `site` of `layer` for microbatch `mb` (scale 0 = off) with the stage's probability and seed.
static DropoutSite site_of(const po_stage* st, int layer, int site, int mb) {
  if (st->cfg.dropout_p > 0.f) return make_dropout_site(st->cfg.dropout_p, st->cfg.dropout_seed, layer, site, mb);
  DropoutSite d;
  memset(&d, 0, sizeof(d));
  return d;
}

static int layer_forward(po_stage* st, int layer, int mb, char* slab, void* y_out) {
  const po_config& c = st->cfg;
  const ParamLayout& pl = st->pl;
  const SlabLayout& sl = st->sl;
  int s = c.seq, h = c.hidden, f = c.ffn, dt = c.dtype;
  hipStream_t q = st->compute;
  char* x = slab + sl.off_x;
  char* qkv = slab + sl.off_qkv;
  char* o = slab + sl.off_o;
  char* x1 = slab + sl.off_x1;
  char* u = slab + sl.off_u;
  float* lse = (float*)(slab + sl.off_lse);

  PO_K(layernorm_forward(dt, x, st->P(layer, pl.ln1_g), st->P(layer, pl.ln1_b), st->w_n, s, h, c.ln_eps, q));
  const int wq = qkv_width_of(c);  // h + 2 hkv
  Epilogue e = make_ep(wq);
  e.bias = st->P(layer, pl.b_qkv);
  e.out = qkv;
  PO_RC(st_gemm(st, 0, 0, s, wq, h, st->w_n, h, st->P(layer, pl.w_qkv), wq, e));
  PO_RC(st_attention(st, false, qkv, o, lse, nullptr, nullptr));
  e = make_ep(h);
  e.bias = st->P(layer, pl.b_o);
  // With dropout the projection (bias included) lands in a scratch tensor and one more kernel forms
  // x1 = x + dropout(projection); fusing the generator into the GEMM epilogue cost the GEMM its registers.
  const bool drop = c.dropout_p > 0.f;
  e.residual = drop ? nullptr : x;
  e.out = drop ? st->w_dz[0] : x1;
  PO_RC(st_gemm(st, 0, 0, s, h, h, o, h, st->P(layer, pl.w_o), h, e));
  if (drop) PO_K(dropout_apply(dt, st->w_dz[0], x, x1, s, h, site_of(st, layer, 0, mb), q));
  PO_K(layernorm_forward(dt, x1, st->P(layer, pl.ln2_g), st->P(layer, pl.ln2_b), st->w_n, s, h, c.ln_eps, q));
  e = make_ep(f);
  e.bias = st->P(layer, pl.b_fc1);
  e.out = u;
  e.gelu_out = st->w_g;
  PO_RC(st_gemm(st, 0, 0, s, f, h, st->w_n, h, st->P(layer, pl.w_fc1), f, e));
  e = make_ep(h);
  e.bias = st->P(layer, pl.b_fc2);
  e.residual = drop ? nullptr : x1;
  e.out = drop ? (void*)st->w_dz[0] : y_out;
  PO_RC(st_gemm(st, 0, 0, s, h, f, st->w_g, f, st->P(layer, pl.w_fc2), h, e));
  if (drop) PO_K(dropout_apply(dt, st->w_dz[0], x1, y_out, s, h, site_of(st, layer, 1, mb), q));
  return PO_OK;
}

// dy: gradient of the layer output; dx_out: where the gradient of the layer input goes.
// Gradient tensors of one layer that the input-gradient half of the backward produces and the
// weight-gradient half consumes.  The fused backward points them at the stage workspaces (one layer at a
// time); the split backward (B pass, later W pass) points them into a per-unit buffer that lives from B to W.
struct BwdBufs {
  char *g, *du, *dn2, *dx1, *dqkv, *dn1;
  char *dz2, *dz1;  // with dropout: the masked, rescaled gradients at the two output projections
  float *lnws2, *lnws1;
};

// Input-gradient half of one layer (activation gradients only):
//   du = (dy W2^T) * gelu'(u) with g = gelu(u) recomputed, dn2 = du W1^T, dx1 = dy + LNbwd(dn2; x1),
//   dO = dx1 Wo^T, (dq, dk, dv) = attention backward, dn1 = dqkv Wqkv^T, dx = dx1 + LNbwd(dn1; x).
// With dropout the two projections see dz = dropout(gradient) (mask regenerated), the residual branches do not.
// n_out: null, or where the recomputed LayerNorm outputs go (LN2(x1), then LN1(x) gl_sh bytes further) for a
// weight-gradient half that runs right after this call and is told so (n_ready).
static int layer_backward_input(po_stage* st, int layer, int mb, const char* slab, const void* dy, void* dx_out,
                                const BwdBufs& b, char* n_out = nullptr) {
  const po_config& c = st->cfg;
  const ParamLayout& pl = st->pl;
  const SlabLayout& sl = st->sl;
  int s = c.seq, h = c.hidden, f = c.ffn, dt = c.dtype;
  hipStream_t q = st->compute;
  const char* x = slab + sl.off_x;
  const char* qkv = slab + sl.off_qkv;
  const char* o = slab + sl.off_o;
  const char* x1 = slab + sl.off_x1;
  const char* u = slab + sl.off_u;
  const float* lse = (const float*)(slab + sl.off_lse);

  const bool drop = c.dropout_p > 0.f;
  const void* dz2 = dy;
  if (drop) {
    PO_K(dropout_apply(dt, dy, nullptr, b.dz2, s, h, site_of(st, layer, 1, mb), q));
    dz2 = b.dz2;
  }
  Epilogue e = make_ep(f);
  e.out = b.du;
  e.gelu_u = u;
  e.gelu_out = b.g;
  PO_RC(st_gemm(st, 0, 1, s, f, h, dz2, h, st->P(layer, pl.w_fc2), h, e));
  e = make_ep(h);
  e.out = b.dn2;
  PO_RC(st_gemm(st, 0, 1, s, h, f, b.du, f, st->P(layer, pl.w_fc1), f, e));
  PO_K(layernorm_backward(dt, b.dn2, x1, st->P(layer, pl.ln2_g), dy, b.dx1, nullptr, nullptr, b.lnws2, s, h,
                          c.ln_eps, kLnInputGrad, q, n_out ? st->P(layer, pl.ln2_b) : nullptr, n_out));
  const void* dz1 = b.dx1;
  if (drop) {
    PO_K(dropout_apply(dt, b.dx1, nullptr, b.dz1, s, h, site_of(st, layer, 0, mb), q));
    dz1 = b.dz1;
  }
  e = make_ep(h);
  e.out = st->w_do;
  PO_RC(st_gemm(st, 0, 1, s, h, h, dz1, h, st->P(layer, pl.w_o), h, e));
  PO_RC(st_attention(st, true, qkv, const_cast<char*>(o), const_cast<float*>(lse), st->w_do, b.dqkv));
  e = make_ep(h);
  e.out = b.dn1;
  const int wq = qkv_width_of(c);
  PO_RC(st_gemm(st, 0, 1, s, h, wq, b.dqkv, wq, st->P(layer, pl.w_qkv), wq, e));
  PO_K(layernorm_backward(dt, b.dn1, x, st->P(layer, pl.ln1_g), b.dx1, dx_out, nullptr, nullptr, b.lnws1, s, h,
                          c.ln_eps, kLnInputGrad, q, n_out ? st->P(layer, pl.ln1_b) : nullptr,
                          n_out ? n_out + st->gl_sh : nullptr));
  return PO_OK;
}

// Weight-gradient half of one layer (parameter gradients only, accumulated in fp32):
//   dW2 += g^T dy, db2 += colsum(dy); dW1 += n2^T du, db1 += colsum(du) with n2 = LN2(x1) recomputed;
//   dWo += O^T dx1, dbo += colsum(dx1); dWqkv += n1^T dqkv, dbqkv += colsum(dqkv) with n1 = LN1(x) recomputed;
//   LayerNorm gains and shifts from (dn2, x1) and (dn1, x) with the row statistics the input half left.
// Runs on stream q with the LayerNorm-output and column-sum scratch buffers n_out / colws (the weight stream has
// its own, so that it can run beside the compute stream).
static int layer_backward_weight(po_stage* st, int layer, const char* slab, const void* dy, const BwdBufs& b,
                                 hipStream_t q, char* n_out, float* colws, bool n_ready = false) {
  const po_config& c = st->cfg;
  const ParamLayout& pl = st->pl;
  const SlabLayout& sl = st->sl;
  int s = c.seq, h = c.hidden, f = c.ffn, dt = c.dtype;
  const char* x = slab + sl.off_x;
  const char* o = slab + sl.off_o;
  const char* x1 = slab + sl.off_x1;

  const bool drop = c.dropout_p > 0.f;
  const void* dz2 = drop ? (const void*)b.dz2 : dy;  // what the input-gradient half fed the MLP output projection
  const void* dz1 = drop ? (const void*)b.dz1 : (const void*)b.dx1;
  const int wq = qkv_width_of(c);
  // All six column reductions of the layer (four bias gradients, two LayerNorm gain / shift pairs) in two
  // launches; their inputs are complete once the input-gradient half has run.
  {
    const size_t plane = column_reductions_workspace(s, 1) / sizeof(float);  // floats per column
    float* ws = colws;
    ReduceJob jobs[6];
    auto sum_job = [&](const void* a, float* out, int n) {
      ReduceJob j{a, nullptr, nullptr, out, nullptr, ws, n};
      ws += plane * n;
      return j;
    };
    jobs[0] = sum_job(dz2, st->G(layer, pl.b_fc2), h);
    jobs[1] = sum_job(b.du, st->G(layer, pl.b_fc1), f);
    jobs[2] = sum_job(dz1, st->G(layer, pl.b_o), h);
    jobs[3] = sum_job(b.dqkv, st->G(layer, pl.b_qkv), wq);
    jobs[4] = ReduceJob{b.dn2, x1, b.lnws2, st->G(layer, pl.ln2_g), st->G(layer, pl.ln2_b), b.lnws2 + (size_t)s * 2, h};
    jobs[5] = ReduceJob{b.dn1, x, b.lnws1, st->G(layer, pl.ln1_g), st->G(layer, pl.ln1_b), b.lnws1 + (size_t)s * 2, h};
    PO_K(column_reductions(dt, jobs, 6, s, q));
  }
  // The four products dW = operand^T gradient.  They do not depend on each other, so where the matrix-core
  // kernel can take them as one grouped launch (both LayerNorm outputs recomputed first, into two buffers) the
  // chip works through the tiles of all four without a launch boundary in between; else one launch each.
  char* n2 = n_out;
  char* n1 = n_out + st->gl_sh;
  GemmProblem prob[4] = {
      {f, h, s, b.g, f, dz2, h, st->G(layer, pl.w_fc2), h},
      {h, f, s, n2, h, b.du, f, st->G(layer, pl.w_fc1), f},
      {h, h, s, o, h, dz1, h, st->G(layer, pl.w_o), h},
      {h, wq, s, n1, h, b.dqkv, wq, st->G(layer, pl.w_qkv), wq},
  };
  if (dt == PO_BF16 && gemm_mfma_grouped_supported(4, prob)) {
    if (!n_ready) {
      PO_K(layernorm_forward(dt, x1, st->P(layer, pl.ln2_g), st->P(layer, pl.ln2_b), n2, s, h, c.ln_eps, q));
      PO_K(layernorm_forward(dt, x, st->P(layer, pl.ln1_g), st->P(layer, pl.ln1_b), n1, s, h, c.ln_eps, q));
    }
    return st_gemm_grouped(st, 4, prob, q);
  }
  for (int i = 0; i < 4; ++i) {
    if (i == 1 && !n_ready)
      PO_K(layernorm_forward(dt, x1, st->P(layer, pl.ln2_g), st->P(layer, pl.ln2_b), n2, s, h, c.ln_eps, q));
    if (i == 3 && !n_ready)
      PO_K(layernorm_forward(dt, x, st->P(layer, pl.ln1_g), st->P(layer, pl.ln1_b), n1, s, h, c.ln_eps, q));
    Epilogue e = make_ep(prob[i].ldc);
    e.acc_f32 = prob[i].acc_f32;
    PO_RC(st_gemm(st, 1, 0, prob[i].M, prob[i].N, prob[i].K, prob[i].A, prob[i].lda, prob[i].B, prob[i].ldb, e, q));
  }
  return PO_OK;
}

// ------------------------------------------------------------------------------
// Unit-level operations
// ------------------------------------------------------------------------------
int stage_forward(po_stage* st, int mb, int chunk, const void* x_in, void* y_out) {
  const po_config& c = st->cfg;
  if (!st->params) {
    set_error("forward before po_bind_params");
    return PO_E_STATE;
  }
  if (mb < 0 || chunk < 0 || chunk >= c.n_chunks || !x_in || !y_out) {
    set_error("forward: mb=%d chunk=%d x_in=%p y_out=%p", mb, chunk, x_in, y_out);
    return PO_E_INVAL;
  }
  Unit& u = st->units[unit_key(mb, chunk)];
  if (u.live) {
    set_error("forward of unit (mb %d, chunk %d) that is still in flight", mb, chunk);
    return PO_E_STATE;
  }
  u.layers.assign(st->Lu, UnitLayer());
  for (int l = 0; l < st->Lu; ++l) {
    int rc = st->dev_pool.acquire(st->compute, &u.layers[l].dev);
    if (rc) {
      for (int k = 0; k < l; ++k) st->dev_pool.release(u.layers[k].dev, st->compute);
      st->units.erase(unit_key(mb, chunk));
      return rc;
    }
    u.layers[l].state = L_RESIDENT;
  }
  u.live = true;
  u.x_in = x_in;
  ++st->in_flight_units;
  ++st->resident_units;
  st->note_usage();

  size_t span;
  int rc = span_begin(st, st->compute, 0, &span);
  if (rc) return rc;
  bool embed = c.vocab > 0 && chunk == 0;
  char* slab0 = st->dev_pool.bufs[u.layers[0].dev].ptr;
  if (embed) {
    PO_K(embedding_forward(c.dtype, (const int32_t*)x_in, st->params + (size_t)st->pl.emb_wte * st->E,
                           st->params + (size_t)st->pl.emb_wpe * st->E, slab0 + st->sl.off_x, c.seq, c.hidden,
                           c.vocab, st->compute));
  } else {
    PO_K(copy_bytes(slab0 + st->sl.off_x, x_in, st->sl.sz_x, st->compute));
  }
  for (int l = 0; l < st->Lu; ++l) {
    char* slab = st->dev_pool.bufs[u.layers[l].dev].ptr;
    void* out = (l + 1 < st->Lu) ? (void*)(st->dev_pool.bufs[u.layers[l + 1].dev].ptr + st->sl.off_x) : y_out;
    rc = layer_forward(st, chunk * st->Lu + l, mb, slab, out);
    if (rc) return rc;
  }
  rc = span_end(st, st->compute, span);
  if (rc) return rc;
  rc = st->sync_events.get(&u.fwd_done);
  if (rc) return rc;
  PO_HIP(hipEventRecord(u.fwd_done, st->compute));
  ++st->stats.n_compute_passes;
  return PO_OK;
}

static Unit* find_live_unit(po_stage* st, int mb, int chunk, const char* what) {
  auto it = st->units.find(unit_key(mb, chunk));
  if (it == st->units.end() || !it->second.live) {
    set_error("%s of unit (mb %d, chunk %d) that was not forwarded", what, mb, chunk);
    return nullptr;
  }
  return &it->second;
}

static void slab_segments(const SlabLayout& sl, char* slab, void** ptrs, uint64_t* bytes) {
  size_t offs[6] = {sl.off_x, sl.off_qkv, sl.off_o, sl.off_x1, sl.off_u, sl.off_lse};
  size_t szs[6] = {sl.sz_x, sl.sz_qkv, sl.sz_o, sl.sz_x1, sl.sz_u, sl.sz_lse};
  for (int i = 0; i < 6; ++i) {
    ptrs[i] = slab + offs[i];
    bytes[i] = align_up(szs[i], 16);
  }
}

int stage_offload(po_stage* st, int mb, int chunk, float ratio) {
  if (!(ratio >= 0.f && ratio <= 1.f)) {
    set_error("offload: ratio %g outside [0, 1]", ratio);
    return PO_E_INVAL;
  }
  Unit* u = find_live_unit(st, mb, chunk, "offload");
  if (!u) return PO_E_STATE;
  if (u->weight_pending) {
    set_error("offload of unit (mb %d, chunk %d) between its input-gradient and weight-gradient pass", mb, chunk);
    return PO_E_STATE;
  }
  int n = (int)ceil((double)ratio * st->Lu - 1e-9);
  for (int l = 0; l < n; ++l)
    if (u->layers[l].state != L_RESIDENT) {
      set_error("offload of unit (mb %d, chunk %d): layer %d is not resident", mb, chunk, l);
      return PO_E_STATE;
    }
  bool was_resident = unit_has_resident_layer(*u);
  hipStream_t q = st->offload;
  if (n > 0) PO_HIP(hipStreamWaitEvent(q, u->fwd_done, 0));
  // The n lowest layers go, the top one of them first: the reload brings the layers back in that order too (the
  // backward starts at the top), and a layer can only come back once it has gone, so the layer that is needed
  // first must not be the one that leaves last.
  for (int l = n - 1; l >= 0; --l) {
    UnitLayer& L = u->layers[l];
    if (L.h2d_done) {  // reloaded and offloaded again without a backward in between
      PO_HIP(hipStreamWaitEvent(q, L.h2d_done, 0));
      L.h2d_done = nullptr;
    }
    int rc = st->host_pool.acquire(q, &L.hostbuf);
    if (rc) return rc;
    char* dev = st->dev_pool.bufs[L.dev].ptr;
    char* host = st->host_pool.bufs[L.hostbuf].ptr;
    size_t span;
    if (st->cfg.staged_copies) {
      int stg;
      rc = st->dev_pool.acquire(q, &stg);
      if (rc) {  // the layer stays resident; its host buffer goes back unused
        (void)st->host_pool.release(L.hostbuf, q);
        L.hostbuf = -1;
        return rc;
      }
      st->note_usage();
      char* staging = st->dev_pool.bufs[stg].ptr;
      void* ptrs[6];
      uint64_t bytes[6];
      slab_segments(st->sl, dev, ptrs, bytes);
      rc = span_begin(st, q, 3, &span);
      if (rc) return rc;
      PO_K(pack_segments(ptrs, bytes, 6, staging, q));
      rc = span_end(st, q, span);
      if (rc) return rc;
      if (st->cfg.debug_poison) PO_K(fill_u32(dev, 0x7fc07fc0u, st->sl.bytes, q));
      rc = st->dev_pool.release(L.dev, q);  // the slab is free as soon as it is packed
      if (rc) return rc;
      rc = span_begin(st, q, 1, &span);
      if (rc) return rc;
      PO_HIP(hipMemcpyAsync(host, staging, st->sl.packed_bytes, hipMemcpyDeviceToHost, q));
      rc = span_end(st, q, span);
      if (rc) return rc;
      rc = st->dev_pool.release(stg, q);
      if (rc) return rc;
      st->stats.bytes_d2h += st->sl.packed_bytes;
    } else {
      rc = span_begin(st, q, 1, &span);
      if (rc) return rc;
      PO_HIP(hipMemcpyAsync(host, dev, st->sl.bytes, hipMemcpyDeviceToHost, q));
      rc = span_end(st, q, span);
      if (rc) return rc;
      if (st->cfg.debug_poison) PO_K(fill_u32(dev, 0x7fc07fc0u, st->sl.bytes, q));
      rc = st->dev_pool.release(L.dev, q);
      if (rc) return rc;
      st->stats.bytes_d2h += st->sl.bytes;
    }
    rc = st->sync_events.get(&L.d2h_done);
    if (rc) return rc;
    PO_HIP(hipEventRecord(L.d2h_done, q));
    L.dev = -1;
    L.state = L_HOST;
    ++st->stats.n_offloads;
  }
  if (was_resident && !unit_has_resident_layer(*u)) --st->resident_units;
  return PO_OK;
}

int stage_reload(po_stage* st, int mb, int chunk) {
  Unit* u = find_live_unit(st, mb, chunk, "reload");
  if (!u) return PO_E_STATE;
  bool any = false;
  for (const UnitLayer& L : u->layers) any |= L.state == L_HOST;
  if (!any) return PO_OK;
  bool was_resident = unit_has_resident_layer(*u);
  hipStream_t q = st->reload;
  // The reload may start once the compute work enqueued so far has been reached.
  hipEvent_t gate;
  int rc = st->sync_events.get(&gate);
  if (rc) return rc;
  PO_HIP(hipEventRecord(gate, st->compute));
  PO_HIP(hipStreamWaitEvent(q, gate, 0));
  // Top layer first: the backward consumes the layers from the top down and waits for each on its own, so the
  // lower layers travel while the upper ones are already being differentiated.
  for (int l = st->Lu - 1; l >= 0; --l) {
    UnitLayer& L = u->layers[l];
    if (L.state != L_HOST) continue;
    if (q != st->offload) PO_HIP(hipStreamWaitEvent(q, L.d2h_done, 0));
    rc = st->dev_pool.acquire(q, &L.dev);
    if (rc) return rc;
    st->note_usage();
    char* dev = st->dev_pool.bufs[L.dev].ptr;
    char* host = st->host_pool.bufs[L.hostbuf].ptr;
    size_t span;
    if (st->cfg.staged_copies) {
      int stg;
      rc = st->dev_pool.acquire(q, &stg);
      if (rc) return rc;
      st->note_usage();
      char* staging = st->dev_pool.bufs[stg].ptr;
      rc = span_begin(st, q, 2, &span);
      if (rc) return rc;
      PO_HIP(hipMemcpyAsync(staging, host, st->sl.packed_bytes, hipMemcpyHostToDevice, q));
      rc = span_end(st, q, span);
      if (rc) return rc;
      void* ptrs[6];
      uint64_t bytes[6];
      slab_segments(st->sl, dev, ptrs, bytes);
      rc = span_begin(st, q, 3, &span);
      if (rc) return rc;
      PO_K(unpack_segments(ptrs, bytes, 6, staging, q));
      rc = span_end(st, q, span);
      if (rc) return rc;
      rc = st->dev_pool.release(stg, q);
      if (rc) return rc;
      st->stats.bytes_h2d += st->sl.packed_bytes;
    } else {
      rc = span_begin(st, q, 2, &span);
      if (rc) return rc;
      PO_HIP(hipMemcpyAsync(dev, host, st->sl.bytes, hipMemcpyHostToDevice, q));
      rc = span_end(st, q, span);
      if (rc) return rc;
      st->stats.bytes_h2d += st->sl.bytes;
    }
    rc = st->sync_events.get(&L.h2d_done);
    if (rc) return rc;
    PO_HIP(hipEventRecord(L.h2d_done, q));
    rc = st->host_pool.release(L.hostbuf, q);
    if (rc) return rc;
    L.hostbuf = -1;
    L.state = L_RESIDENT;
    ++st->stats.n_reloads;
  }
  if (!was_resident) ++st->resident_units;
  st->note_usage();
  return PO_OK;
}

// Checks shared by the three backward entry points.
static int backward_prologue(po_stage* st, int mb, int chunk, const void* dy, void* dx, const char* what,
                             Unit** out) {
  const po_config& c = st->cfg;
  if (!st->params || !st->grads) {
    set_error("%s before po_bind_params", what);
    return PO_E_STATE;
  }
  if (mb < 0 || chunk < 0 || chunk >= c.n_chunks) {
    set_error("%s: mb=%d chunk=%d", what, mb, chunk);
    return PO_E_INVAL;
  }
  Unit* u = find_live_unit(st, mb, chunk, what);
  if (!u) return PO_E_STATE;
  if (u->weight_pending) {
    set_error("%s of unit (mb %d, chunk %d) whose input-gradient pass already ran", what, mb, chunk);
    return PO_E_STATE;
  }
  bool embed = c.vocab > 0 && chunk == 0;
  if (!dy || (!dx && !embed)) {
    set_error("%s: dy=%p dx=%p", what, dy, dx);
    return PO_E_INVAL;
  }
  for (int l = 0; l < st->Lu; ++l)
    if (u->layers[l].state != L_RESIDENT) {
      set_error("%s of unit (mb %d, chunk %d): layer %d is on the host and no reload was issued", what, mb, chunk,
                l);
      return PO_E_STATE;
    }
  *out = u;
  return PO_OK;
}

// The compute stream waits for a layer's outstanding reload right before the first kernel that reads its slab.
// A wait in the middle of a pass closes the pass's timed span and opens a new one behind it, so that time spent
// waiting for a copy is not booked as compute (span == nullptr: no span is open yet).
static int await_layer(po_stage* st, UnitLayer& L, size_t* span) {
  if (!L.h2d_done) return PO_OK;
  if (span) PO_RC(span_end(st, st->compute, *span));
  PO_HIP(hipStreamWaitEvent(st->compute, L.h2d_done, 0));
  L.h2d_done = nullptr;
  if (span) PO_RC(span_begin(st, st->compute, 0, span));
  return PO_OK;
}

// Hands the unit's slabs back once its last pass has been enqueued.
static int retire_unit(po_stage* st, Unit* u, hipStream_t q) {
  for (UnitLayer& L : u->layers) {
    if (st->cfg.debug_poison) PO_K(fill_u32(st->dev_pool.bufs[L.dev].ptr, 0x7fc07fc0u, st->sl.bytes, q));
    int rc = st->dev_pool.release(L.dev, q);
    if (rc) return rc;
    L = UnitLayer();
  }
  u->live = false;
  u->weight_pending = false;
  --st->resident_units;
  return PO_OK;
}

static BwdBufs workspace_bufs(po_stage* st) {
  BwdBufs b;
  b.g = st->w_g;
  b.du = st->w_du;
  b.dn2 = st->w_dn;
  b.dx1 = st->w_dx1;
  b.dqkv = st->w_dqkv;
  b.dn1 = st->w_dn1;
  b.dz2 = st->w_dz[0];
  b.dz1 = st->w_dz[1];
  b.lnws2 = st->w_lnws;
  b.lnws1 = st->w_lnws1;
  return b;
}

// Layer l's tensors inside a unit's gradient buffer; *dy_in is where the gradient arriving at the layer's
// output is kept (written by layer l+1's input-gradient half).
static BwdBufs unit_bufs(const po_stage* st, char* buf, int l, char** dy_in) {
  char* p = buf + (size_t)l * st->gl_layer;
  BwdBufs b;
  b.g = p;
  b.du = b.g + st->gl_sf;
  b.dn2 = b.du + st->gl_sf;
  b.dx1 = b.dn2 + st->gl_sh;
  b.dn1 = b.dx1 + st->gl_sh;
  *dy_in = b.dn1 + st->gl_sh;
  b.dz2 = *dy_in + st->gl_sh;
  b.dz1 = b.dz2 + st->gl_sh;
  b.dqkv = b.dz1 + st->gl_sh;
  b.lnws2 = (float*)(b.dqkv + st->gl_s3h);
  b.lnws1 = (float*)((char*)b.lnws2 + st->gl_lnws);
  return b;
}

int stage_backward_input(po_stage* st, int mb, int chunk, const void* dy, void* dx);
static int backward_weight_impl(po_stage* st, int mb, int chunk, bool count_pass);

// Fused backward: per layer, the input-gradient half directly followed by the weight-gradient half on the stage
// workspaces.  With a weight stream it is the B pass on the compute stream and the W pass on the weight stream
// (same kernels, same inputs, same results), so that the next passes overlap the weight gradients.
int stage_backward(po_stage* st, int mb, int chunk, const void* dy, void* dx) {
  const po_config& c = st->cfg;
  if (st->wstream) {
    int rc = stage_backward_input(st, mb, chunk, dy, dx);
    if (rc) return rc;
    return backward_weight_impl(st, mb, chunk, false);
  }
  Unit* u;
  int rc = backward_prologue(st, mb, chunk, dy, dx, "backward", &u);
  if (rc) return rc;
  bool embed = c.vocab > 0 && chunk == 0;
  rc = await_layer(st, u->layers[st->Lu - 1], nullptr);
  if (rc) return rc;
  size_t span;
  rc = span_begin(st, st->compute, 0, &span);
  if (rc) return rc;
  BwdBufs bufs = workspace_bufs(st);
  const void* grad = dy;
  for (int l = st->Lu - 1; l >= 0; --l) {
    rc = await_layer(st, u->layers[l], &span);
    if (rc) return rc;
    const char* slab = st->dev_pool.bufs[u->layers[l].dev].ptr;
    void* out;
    if (l > 0)
      out = st->w_dy[l & 1];
    else
      out = embed ? (void*)st->w_dy[0] : dx;
    // the input-gradient half's LayerNorm backward kernels also leave the two LayerNorm outputs that the
    // weight-gradient half, which follows at once, would otherwise recompute
    rc = layer_backward_input(st, chunk * st->Lu + l, mb, slab, grad, out, bufs, st->w_n_w);
    if (rc) return rc;
    rc = layer_backward_weight(st, chunk * st->Lu + l, slab, grad, bufs, st->compute, st->w_n_w, st->w_colws_w, true);
    if (rc) return rc;
    grad = out;
  }
  if (embed)
    PO_K(embedding_backward(c.dtype, (const int32_t*)u->x_in, grad, st->grads + st->pl.emb_wte,
                            st->grads + st->pl.emb_wpe, c.seq, c.hidden, c.vocab, st->compute));
  rc = span_end(st, st->compute, span);
  if (rc) return rc;
  rc = retire_unit(st, u, st->compute);
  if (rc) return rc;
  st->units.erase(unit_key(mb, chunk));  // (u is gone) a long run with ever new microbatch numbers must not grow the map
  --st->in_flight_units;
  ++st->stats.n_compute_passes;
  return PO_OK;
}

// Split backward, B pass: activation gradients of every layer of the unit, top layer first; what the W pass
// needs is left in a buffer of the gradient pool.  The unit keeps its slabs until the W pass.
int stage_backward_input(po_stage* st, int mb, int chunk, const void* dy, void* dx) {
  const po_config& c = st->cfg;
  Unit* u;
  int rc = backward_prologue(st, mb, chunk, dy, dx, "input-gradient pass", &u);
  if (rc) return rc;
  bool embed = c.vocab > 0 && chunk == 0;
  rc = st->grad_pool.acquire(st->compute, &u->grad_buf);
  if (rc) return rc;
  char* buf = st->grad_pool.bufs[u->grad_buf].ptr;
  rc = await_layer(st, u->layers[st->Lu - 1], nullptr);
  if (rc) return rc;
  size_t span;
  rc = span_begin(st, st->compute, 0, &span);
  if (rc) return rc;
  const void* grad = dy;
  for (int l = st->Lu - 1; l >= 0; --l) {
    rc = await_layer(st, u->layers[l], &span);
    if (rc) return rc;
    const char* slab = st->dev_pool.bufs[u->layers[l].dev].ptr;
    char* dy_in;
    BwdBufs bufs = unit_bufs(st, buf, l, &dy_in);
    (void)dy_in;
    void* out;
    if (l > 0) {
      char* below;  // layer l-1 keeps its incoming gradient for its own weight-gradient half
      (void)unit_bufs(st, buf, l - 1, &below);
      out = below;
    } else {
      out = embed ? (void*)(buf + (size_t)st->Lu * st->gl_layer) : dx;
    }
    rc = layer_backward_input(st, chunk * st->Lu + l, mb, slab, grad, out, bufs);
    if (rc) return rc;
    grad = out;
  }
  rc = span_end(st, st->compute, span);
  if (rc) return rc;
  if (st->wstream) {
    rc = st->sync_events.get(&u->b_done);
    if (rc) return rc;
    PO_HIP(hipEventRecord(u->b_done, st->compute));
  }
  u->weight_pending = true;
  u->dy_top = dy;
  --st->in_flight_units;
  ++st->stats.n_compute_passes;
  return PO_OK;
}

// Split backward, W pass: parameter gradients of every layer of the unit; frees the unit.  Runs on the weight
// stream when there is one (after the unit's B pass), else on the compute stream.
static int backward_weight_impl(po_stage* st, int mb, int chunk, bool count_pass) {
  const po_config& c = st->cfg;
  if (mb < 0 || chunk < 0 || chunk >= c.n_chunks) {
    set_error("weight-gradient pass: mb=%d chunk=%d", mb, chunk);
    return PO_E_INVAL;
  }
  Unit* u = find_live_unit(st, mb, chunk, "weight-gradient pass");
  if (!u) return PO_E_STATE;
  if (!u->weight_pending) {
    set_error("weight-gradient pass of unit (mb %d, chunk %d) before its input-gradient pass", mb, chunk);
    return PO_E_STATE;
  }
  bool embed = c.vocab > 0 && chunk == 0;
  hipStream_t q = st->wstream ? st->wstream : st->compute;
  if (st->wstream) PO_HIP(hipStreamWaitEvent(q, u->b_done, 0));
  char* buf = st->grad_pool.bufs[u->grad_buf].ptr;
  size_t span;
  int rc = span_begin(st, q, 0, &span);
  if (rc) return rc;
  for (int l = st->Lu - 1; l >= 0; --l) {
    const char* slab = st->dev_pool.bufs[u->layers[l].dev].ptr;
    char* dy_in;
    BwdBufs bufs = unit_bufs(st, buf, l, &dy_in);
    const void* grad = l == st->Lu - 1 ? u->dy_top : (const void*)dy_in;
    rc = layer_backward_weight(st, chunk * st->Lu + l, slab, grad, bufs, q, st->w_n_w, st->w_colws_w);
    if (rc) return rc;
  }
  if (embed)
    PO_K(embedding_backward(c.dtype, (const int32_t*)u->x_in, buf + (size_t)st->Lu * st->gl_layer,
                            st->grads + st->pl.emb_wte, st->grads + st->pl.emb_wpe, c.seq, c.hidden, c.vocab, q));
  rc = span_end(st, q, span);
  if (rc) return rc;
  rc = st->grad_pool.release(u->grad_buf, q);
  if (rc) return rc;
  u->grad_buf = -1;
  u->dy_top = nullptr;
  u->b_done = nullptr;
  rc = retire_unit(st, u, q);
  if (rc) return rc;
  st->units.erase(unit_key(mb, chunk));  // (u is gone)
  if (count_pass) ++st->stats.n_compute_passes;
  return PO_OK;
}

int stage_backward_weight(po_stage* st, int mb, int chunk) { return backward_weight_impl(st, mb, chunk, true); }

// Drops every unit that is still in flight (after a failed call, or to abandon a step): waits for all streams,
// then hands the units' device slabs, host slabs and gradient buffers back to their pools.  Nothing is freed.
int stage_reset(po_stage* st);

int stage_synchronize(po_stage* st) {
  PO_HIP(hipStreamSynchronize(st->compute));
  if (st->wstream) PO_HIP(hipStreamSynchronize(st->wstream));
  PO_HIP(hipStreamSynchronize(st->offload));
  if (st->reload != st->offload) PO_HIP(hipStreamSynchronize(st->reload));
  return PO_OK;
}

int stage_reset(po_stage* st) {
  int rc = stage_synchronize(st);
  if (rc) return rc;
  for (auto& kv : st->units) {
    Unit& u = kv.second;
    if (!u.live) continue;
    for (UnitLayer& L : u.layers) {
      if (L.dev >= 0) PO_RC(st->dev_pool.release(L.dev, st->compute));
      if (L.hostbuf >= 0) PO_RC(st->host_pool.release(L.hostbuf, st->compute));
      L = UnitLayer();
    }
    if (u.grad_buf >= 0) PO_RC(st->grad_pool.release(u.grad_buf, st->compute));
  }
  st->units.clear();
  st->resident_units = 0;
  st->in_flight_units = 0;
  st->sync_events.reset();
  return stage_synchronize(st);
}

// Folds the recorded spans into the stats (all streams must be drained).
static int collect_spans(po_stage* st) {
  double busy[6] = {0, 0, 0, 0, 0, 0};
  double flops[6] = {0, 0, 0, 0, 0, 0};
  hipEvent_t first = nullptr, last = nullptr;
  for (const TimedSpan& sp : st->spans) {
    float ms = 0.f;
    PO_HIP(hipEventElapsedTime(&ms, sp.start, sp.stop));
    busy[sp.kind] += ms * 1e-3;
    flops[sp.kind] += sp.flops;
    if (sp.kind == 4) ++st->stats.n_gemm_launches;
    if (sp.kind == 0) {
      if (!first) first = sp.start;
      last = sp.stop;
    }
  }
  // PIPEOFFLOAD_TRACE=<file>: one line per span of the run, "kind start_ms stop_ms" from the first span's start
  // (kind as in TimedSpan), appended; a run separator line "# run" first.
  if (const char* path = getenv("PIPEOFFLOAD_TRACE")) {
    if (!st->spans.empty()) {
      if (FILE* f = fopen(path, "a")) {
        fprintf(f, "# run\n");
        hipEvent_t origin = st->spans[0].start;
        for (const TimedSpan& sp : st->spans) {
          float a = 0.f, b = 0.f;
          PO_HIP(hipEventElapsedTime(&a, origin, sp.start));
          PO_HIP(hipEventElapsedTime(&b, origin, sp.stop));
          fprintf(f, "%d %.4f %.4f\n", sp.kind, a, b);
        }
        fclose(f);
      }
    }
  }
  // Copy time hidden behind compute: every offload / reload span intersected with the union of the compute spans.
  if (!st->spans.empty()) {
    hipEvent_t origin = st->spans[0].start;
    std::vector<std::pair<float, float>> comp, copies;
    for (const TimedSpan& sp : st->spans) {
      if (sp.kind > 2) continue;
      float a = 0.f, b = 0.f;
      PO_HIP(hipEventElapsedTime(&a, origin, sp.start));
      PO_HIP(hipEventElapsedTime(&b, origin, sp.stop));
      (sp.kind == 0 ? comp : copies).push_back({a, b});
    }
    std::sort(comp.begin(), comp.end());
    std::vector<std::pair<float, float>> merged;
    for (const auto& iv : comp) {
      if (!merged.empty() && iv.first <= merged.back().second)
        merged.back().second = std::max(merged.back().second, iv.second);
      else
        merged.push_back(iv);
    }
    double hidden = 0.0;
    for (const auto& cp : copies)
      for (const auto& iv : merged) {
        float lo = std::max(cp.first, iv.first), hi = std::min(cp.second, iv.second);
        if (hi > lo) hidden += hi - lo;
      }
    st->stats.copy_hidden_s = hidden * 1e-3;
  }
  st->stats.compute_busy_s = busy[0];
  st->stats.d2h_busy_s = busy[1];
  st->stats.h2d_busy_s = busy[2];
  st->stats.pack_busy_s = busy[3];
  st->stats.gemm_busy_s = busy[4];
  st->stats.gemm_flops = flops[4];
  st->stats.attn_busy_s = busy[5];
  st->stats.attn_flops = flops[5];
  if (first && last) {
    float ms = 0.f;
    PO_HIP(hipEventElapsedTime(&ms, first, last));
    st->stats.compute_span_s = ms * 1e-3;
  }
  return PO_OK;
}

static void reset_run_stats(po_stage* st) {
  uint64_t pool = st->dev_pool.allocated(), host = st->host_pool.allocated();
  memset(&st->stats, 0, sizeof(st->stats));
  st->stats.pool_bytes_allocated = pool;
  st->stats.host_bytes_allocated = host;
  st->stats.workspace_bytes = st->ws_bytes + st->grad_pool.allocated();
  st->spans.clear();
  st->time_events.reset();
}

int stage_run_schedule(po_stage* st, int schedule, int m, float ratio, const void* const* x_in, void* const* y_out,
                       const void* const* dy, void* const* dx, po_stats* out) {
  const po_config& c = st->cfg;
  if (!x_in || !y_out || !dy || !dx) {
    set_error("run_schedule: NULL pointer array");
    return PO_E_INVAL;
  }
  std::vector<po_op> ops;
  if (schedule == PO_SCHED_PO && c.slot_k > 0.f) {  // Section 4.2's slot plan; whole chunks, longest-lived first
    if (!(ratio >= 0.f && ratio <= 1.f)) {
      set_error("run_schedule: ratio %g outside [0, 1]", ratio);
      return PO_E_INVAL;
    }
    int n_sel = (int)ceil((double)ratio * c.n_chunks - 1e-9);
    if (!build_slot_schedule(c.pipeline_degree, c.rank, c.n_chunks, m, c.group, n_sel, (double)c.slot_k, ops))
      return PO_E_INVAL;
  } else if (!build_schedule(schedule, c.pipeline_degree, c.rank, c.n_chunks, m, c.group, ratio, c.select_policy,
                             c.prefetch_passes, c.min_gap_passes, ops)) {
    return PO_E_INVAL;
  }
  for (auto& kv : st->units)
    if (kv.second.live) {
      set_error("run_schedule with units still in flight");
      return PO_E_STATE;
    }
  int rc = stage_synchronize(st);
  if (rc) return rc;
  st->sync_events.reset();
  reset_run_stats(st);
  st->collect_timing = true;
  auto t0 = std::chrono::steady_clock::now();
  for (const po_op& op : ops) {
    size_t i = (size_t)op.chunk * m + op.mb;
    switch (op.kind) {
      case 0: rc = stage_forward(st, op.mb, op.chunk, x_in[i], y_out[i]); break;
      case 1:  // a schedule with W passes runs its B passes as input-gradient passes
        rc = (schedule == PO_SCHED_GIS || schedule == PO_SCHED_PO) ? stage_backward_input(st, op.mb, op.chunk, dy[i], dx[i])
                                                                   : stage_backward(st, op.mb, op.chunk, dy[i], dx[i]);
        break;
      case 2: rc = stage_offload(st, op.mb, op.chunk, op.ratio); break;
      case 3: rc = stage_reload(st, op.mb, op.chunk); break;
      case 4: rc = stage_backward_weight(st, op.mb, op.chunk); break;
      default:
        set_error("run_schedule: op kind %d", op.kind);
        rc = PO_E_INVAL;
        break;
    }
    if (rc) break;
  }
  int rc2 = stage_synchronize(st);
  auto t1 = std::chrono::steady_clock::now();
  st->collect_timing = false;
  if (rc) return rc;
  if (rc2) return rc2;
  st->stats.wall_s = std::chrono::duration<double>(t1 - t0).count();
  st->stats.tokens_per_s = (double)m * c.seq / st->stats.wall_s;
  st->stats.pool_bytes_allocated = st->dev_pool.allocated();
  st->stats.host_bytes_allocated = st->host_pool.allocated();
  st->stats.workspace_bytes = st->ws_bytes + st->grad_pool.allocated();
  rc = collect_spans(st);
  if (rc) return rc;
  if (out) *out = st->stats;
  return PO_OK;
}

// ------------------------------------------------------------------------------
// Create / destroy
// ------------------------------------------------------------------------------
int stage_create(const po_config* cfg, void* compute_stream, po_stage** out) {
  int rc = validate_config(cfg);
  if (rc) return rc;
  if (!out) {
    set_error("stage_create: out is NULL");
    return PO_E_INVAL;
  }
  po_stage* st = new po_stage();
  st->cfg = *cfg;
  build_param_layout(st->cfg, st->pl);
  build_slab_layout(st->cfg, st->sl);
  st->Lu = cfg->n_layers / cfg->n_chunks;
  st->E = cfg->dtype == PO_BF16 ? 2 : 4;
  st->compute = (hipStream_t)compute_stream;
  memset(&st->stats, 0, sizeof(st->stats));
  st->sync_events.flags = hipEventDisableTiming;
  // Timing events only bracket launches on one stream; nothing the host or another device reads depends on them,
  // so they do without the system-scope release of the default event (a cache write-back per record that cost
  // the bracketed launches 2 % and the step 1 % when every fifth GEMM launch was timed).
  st->time_events.flags = hipEventDisableSystemFence;
  st->dev_pool.host = false;
  st->dev_pool.buf_bytes = st->sl.bytes;
  st->dev_pool.cap = cfg->device_pool_cap_bytes;
  st->host_pool.host = true;
  st->host_pool.buf_bytes = st->sl.bytes;
  st->host_pool.cap = cfg->host_pool_cap_bytes;
  auto fail = [&](int code) {
    po_stage_destroy(st);
    return code;
  };
  // Copy streams at the default priority.
  if (hipStreamCreateWithFlags(&st->offload, hipStreamNonBlocking) != hipSuccess) {
    set_error("creating the offload stream failed");
    st->offload = nullptr;
    return fail(PO_E_HIP);
  }
  if (cfg->copy_streams == 2) {
    if (hipStreamCreateWithFlags(&st->reload, hipStreamNonBlocking) != hipSuccess) {
      set_error("creating the reload stream failed");
      st->reload = nullptr;
      return fail(PO_E_HIP);
    }
    st->own_reload_stream = true;
  } else {
    st->reload = st->offload;
  }
  if (cfg->weight_stream) {
    if (hipStreamCreateWithFlags(&st->wstream, hipStreamNonBlocking) != hipSuccess) {
      set_error("creating the weight-gradient stream failed");
      st->wstream = nullptr;
      return fail(PO_E_HIP);
    }
  }
  // Workspaces: one allocation, carved up.
  size_t s = cfg->seq, h = cfg->hidden, f = cfg->ffn, E = st->E;
  size_t sh = align_up(s * h * E, 256), sf = align_up(s * f * E, 256), s3h = align_up(s * (size_t)qkv_width_of(*cfg) * E, 256);
  size_t delta = align_up((size_t)cfg->n_heads * s * 4, 256);
  size_t lnws = align_up(layernorm_backward_workspace((int)s, (int)h), 256);
  // partial sums of the four bias-gradient reductions of a layer, side by side
  size_t colws = align_up(column_reductions_workspace((int)s, (int)(2 * h + f + (size_t)qkv_width_of(*cfg))), 256);
  bool grouped = kv_heads_of(*cfg) < cfg->n_heads;
  size_t total = 12 * sh + 2 * sf + s3h + delta + 2 * lnws + colws + (grouped ? 2 * sh : 0);
  // one unit's gradient buffer for the split backward: per layer g, du [s,f]; dn2, dx1, dn1, incoming dy, and the
  // two dropout-masked gradients [s,h];
  // dqkv [s,3h]; two LayerNorm workspaces; plus one [s,h] tensor per unit (gradient at the embedding output)
  st->gl_sh = sh;
  st->gl_sf = sf;
  st->gl_s3h = s3h;
  st->gl_lnws = lnws;
  st->gl_layer = 2 * sf + 6 * sh + s3h + 2 * lnws;
  st->grad_pool.host = false;
  st->grad_pool.buf_bytes = (size_t)st->Lu * st->gl_layer + sh;
  st->grad_pool.cap = 0;
  if (hipMalloc((void**)&st->ws, total) != hipSuccess) {
    (void)hipGetLastError();
    set_error("workspace allocation of %zu bytes failed", total);
    st->ws = nullptr;
    return fail(PO_E_DEVICE_OOM);
  }
  st->ws_bytes = total;
  char* p = st->ws;
  auto take = [&](size_t n) {
    char* r = p;
    p += n;
    return r;
  };
  st->w_n = take(sh);
  st->w_do = take(sh);
  st->w_dx1 = take(sh);
  st->w_dn = take(sh);
  st->w_dn1 = take(sh);
  st->w_n_w = take(2 * sh);  // LN2 and LN1 outputs of the weight-gradient half, side by side
  st->w_dz[0] = take(sh);
  st->w_dz[1] = take(sh);
  st->w_dy[0] = take(sh);
  st->w_dy[1] = take(sh);
  st->w_x0 = take(sh);
  st->w_g = take(sf);
  st->w_du = take(sf);
  st->w_dqkv = take(s3h);
  st->w_delta = (float*)take(delta);
  st->w_lnws = (float*)take(lnws);
  st->w_lnws1 = (float*)take(lnws);
  st->w_colws_w = (float*)take(colws);
  if (grouped) st->w_dkv_part = take(2 * sh);
  reset_run_stats(st);
  *out = st;
  return PO_OK;
}

}  // namespace po

// ------------------------------------------------------------------------------
// C ABI
// ------------------------------------------------------------------------------
extern "C" {

void po_config_default(po_config* c) {
  if (!c) return;
  memset(c, 0, sizeof(*c));
  c->n_layers = 1;
  c->n_chunks = 1;
  c->hidden = 64;
  c->n_heads = 1;
  c->ffn = 256;
  c->seq = 1;
  c->dtype = PO_F32;
  c->pipeline_degree = 1;
  c->prefetch_passes = 2;
  c->copy_streams = 2;
  c->ln_eps = 1e-5f;
}

const char* po_last_error(void) { return po::get_error(); }

int po_param_count(const po_config* cfg, int64_t* n) {
  int rc = validate_config(cfg);
  if (rc) return rc;
  if (!n) {
    set_error("po_param_count: n is NULL");
    return PO_E_INVAL;
  }
  ParamLayout pl;
  build_param_layout(*cfg, pl);
  *n = pl.total;
  return PO_OK;
}

int po_param_layout(const po_config* cfg, po_param_desc* out, int32_t* n) {
  int rc = validate_config(cfg);
  if (rc) return rc;
  if (!n) {
    set_error("po_param_layout: n is NULL");
    return PO_E_INVAL;
  }
  ParamLayout pl;
  build_param_layout(*cfg, pl);
  int32_t have = (int32_t)pl.descs.size();
  if (out) {
    int32_t k = *n < have ? *n : have;
    for (int32_t i = 0; i < k; ++i) out[i] = pl.descs[i];
  }
  *n = have;
  return PO_OK;
}

int po_saved_bytes_per_layer(const po_config* cfg, uint64_t* bytes) {
  int rc = validate_config(cfg);
  if (rc) return rc;
  if (!bytes) {
    set_error("po_saved_bytes_per_layer: bytes is NULL");
    return PO_E_INVAL;
  }
  SlabLayout sl;
  build_slab_layout(*cfg, sl);
  *bytes = sl.bytes;
  return PO_OK;
}

int po_schedule_ops(int32_t schedule, int32_t d, int32_t rank, int32_t v, int32_t m, int32_t group, float ratio,
                    int32_t policy, int32_t prefetch, int32_t min_gap, po_op* out, int32_t* n) {
  if (!n) {
    set_error("po_schedule_ops: n is NULL");
    return PO_E_INVAL;
  }
  std::vector<po_op> ops;
  if (!build_schedule(schedule, d, rank, v, m, group, ratio, policy, prefetch, min_gap, ops)) return PO_E_INVAL;
  int32_t have = (int32_t)ops.size();
  if (out) {
    int32_t k = *n < have ? *n : have;
    for (int32_t i = 0; i < k; ++i) out[i] = ops[i];
  }
  *n = have;
  return PO_OK;
}

int po_schedule_ops_slots(int32_t d, int32_t rank, int32_t v, int32_t m, int32_t group, int32_t n_offload_chunks,
                          double k, po_op* out, int32_t* n) {
  if (!n) {
    set_error("po_schedule_ops_slots: n is NULL");
    return PO_E_INVAL;
  }
  std::vector<po_op> ops;
  if (!build_slot_schedule(d, rank, v, m, group, n_offload_chunks, k, ops)) return PO_E_INVAL;
  int32_t have = (int32_t)ops.size();
  if (out) {
    int32_t take = *n < have ? *n : have;
    for (int32_t i = 0; i < take; ++i) out[i] = ops[i];
  }
  *n = have;
  return PO_OK;
}

double po_offload_ratio_for_k(double k) { return k > 1.0 ? 1.0 / k : 1.0; }

double po_offload_k(int32_t h, int32_t s, double bc, double bo) {
  return 10.0 / (3.0 * (6.0 * (double)h + (double)s)) * bc / bo;
}

int po_stage_create(const po_config* cfg, void* compute_stream, po_stage** out) {
  return stage_create(cfg, compute_stream, out);
}

void po_stage_destroy(po_stage* st) {
  if (!st) return;
  if (st->compute || st->offload) (void)stage_synchronize(st);
  st->dev_pool.destroy();
  st->host_pool.destroy();
  st->grad_pool.destroy();
  st->sync_events.destroy();
  st->time_events.destroy();
  if (st->ws) (void)hipFree(st->ws);
  if (st->own_reload_stream && st->reload) (void)hipStreamDestroy(st->reload);
  if (st->offload) (void)hipStreamDestroy(st->offload);
  if (st->wstream) (void)hipStreamDestroy(st->wstream);
  delete st;
}

int po_bind_params(po_stage* st, const void* params, float* grads) {
  if (!st || !params || !grads) {
    set_error("po_bind_params: NULL argument");
    return PO_E_INVAL;
  }
  if (((uintptr_t)params | (uintptr_t)grads) % 16 != 0) {
    set_error("po_bind_params: buffers must be 16-byte aligned");
    return PO_E_INVAL;
  }
  st->params = (const char*)params;
  st->grads = grads;
  return PO_OK;
}

#define PO_NEED_STAGE(st)             \
  if (!(st)) {                        \
    set_error("stage is NULL");       \
    return PO_E_INVAL;                \
  }

int po_stage_forward(po_stage* st, int32_t mb, int32_t chunk, const void* x_in, void* y_out) {
  begin_launch();
  PO_NEED_STAGE(st);
  return stage_forward(st, mb, chunk, x_in, y_out);
}
int po_stage_backward(po_stage* st, int32_t mb, int32_t chunk, const void* dy, void* dx) {
  begin_launch();
  PO_NEED_STAGE(st);
  return stage_backward(st, mb, chunk, dy, dx);
}
int po_set_dropout_seed(po_stage* st, uint64_t seed) {
  PO_NEED_STAGE(st);
  for (auto& kv : st->units)
    if (kv.second.live) {
      set_error("po_set_dropout_seed with units in flight (their backward must regenerate the forward's masks)");
      return PO_E_STATE;
    }
  st->cfg.dropout_seed = seed;
  return PO_OK;
}
int po_stage_backward_input(po_stage* st, int32_t mb, int32_t chunk, const void* dy, void* dx) {
  begin_launch();
  PO_NEED_STAGE(st);
  return stage_backward_input(st, mb, chunk, dy, dx);
}
int po_stage_backward_weight(po_stage* st, int32_t mb, int32_t chunk) {
  begin_launch();
  PO_NEED_STAGE(st);
  return stage_backward_weight(st, mb, chunk);
}
int po_offload(po_stage* st, int32_t mb, int32_t chunk, float ratio) {
  begin_launch();
  PO_NEED_STAGE(st);
  return stage_offload(st, mb, chunk, ratio);
}
int po_reload(po_stage* st, int32_t mb, int32_t chunk) {
  begin_launch();
  PO_NEED_STAGE(st);
  return stage_reload(st, mb, chunk);
}
int po_run_schedule(po_stage* st, int32_t schedule, int32_t m, float ratio, const void* const* x_in,
                    void* const* y_out, const void* const* dy, void* const* dx, po_stats* stats) {
  begin_launch();
  PO_NEED_STAGE(st);
  return stage_run_schedule(st, schedule, m, ratio, x_in, y_out, dy, dx, stats);
}
int po_synchronize(po_stage* st) {
  PO_NEED_STAGE(st);
  int rc = stage_synchronize(st);
  if (rc != PO_OK) return rc;
  for (const auto& kv : st->units)
    if (kv.second.live) return PO_OK;  // a unit between passes still holds some of the events
  st->sync_events.reset();
  return PO_OK;
}
int po_stage_reset(po_stage* st) {
  PO_NEED_STAGE(st);
  return stage_reset(st);
}
int po_get_stats(const po_stage* st, po_stats* out) {
  PO_NEED_STAGE(st);
  if (!out) {
    set_error("po_get_stats: out is NULL");
    return PO_E_INVAL;
  }
  *out = st->stats;
  out->pool_bytes_allocated = st->dev_pool.allocated();
  out->host_bytes_allocated = st->host_pool.allocated();
  return PO_OK;
}

// ---- single operations -----------------------------------------------------------
static int ok(bool b) { return b ? PO_OK : PO_E_INVAL; }
static bool dtype_ok(int32_t dtype) {
  if (dtype == PO_F32 || dtype == PO_BF16) return true;
  set_error("unknown dtype %d", dtype);
  return false;
}

int po_op_layernorm_forward(int32_t dtype, const void* x, const void* gain, const void* shift, void* y, int32_t rows,
                            int32_t h, float eps, void* stream) {
  begin_launch();
  if (!dtype_ok(dtype)) return PO_E_INVAL;
  return ok(layernorm_forward(dtype, x, gain, shift, y, rows, h, eps, (hipStream_t)stream));
}
uint64_t po_op_layernorm_backward_workspace(int32_t rows, int32_t h) {
  return rows > 0 && h > 0 ? layernorm_backward_workspace(rows, h) : 0;
}
int po_op_layernorm_backward(int32_t dtype, const void* dn, const void* x, const void* gain, const void* dres,
                             void* dx, float* dgain, float* dshift, float* partials, int32_t rows, int32_t h,
                             float eps, void* stream) {
  begin_launch();
  if (!dtype_ok(dtype)) return PO_E_INVAL;
  return ok(layernorm_backward(dtype, dn, x, gain, dres, dx, dgain, dshift, partials, rows, h, eps,
                               kLnInputGrad | kLnParamGrad,
                               (hipStream_t)stream));
}
int po_op_gemm(int32_t dtype, int32_t trans_a, int32_t trans_b, int32_t M, int32_t N, int32_t K, const void* A,
               int32_t lda, const void* B, int32_t ldb, const void* bias, const void* residual, void* out,
               void* gelu_out, const void* gelu_u, float* acc_f32, int32_t force_generic, void* stream) {
  begin_launch();
  if (!dtype_ok(dtype)) return PO_E_INVAL;
  Epilogue e;
  memset(&e, 0, sizeof(e));
  e.bias = bias;
  e.residual = residual;
  e.out = out;
  e.gelu_out = gelu_out;
  e.gelu_u = gelu_u;
  e.acc_f32 = acc_f32;
  e.ldc = N;
  return ok(gemm(dtype, trans_a != 0, trans_b != 0, M, N, K, A, lda, B, ldb, e, force_generic != 0,
                 (hipStream_t)stream));
}
int po_op_gemm_grouped(int32_t n, const int32_t* M, const int32_t* N, const int32_t* K, const void* const* A,
                       const int32_t* lda, const void* const* B, const int32_t* ldb, float* const* acc_f32,
                       const int32_t* ldc, void* stream) {
  begin_launch();
  if (n < 1 || n > 4 || !M || !N || !K || !A || !lda || !B || !ldb || !acc_f32 || !ldc) {
    set_error("po_op_gemm_grouped: n=%d (1..4) or a NULL array", n);
    return PO_E_INVAL;
  }
  GemmProblem prob[4];
  for (int i = 0; i < n; ++i) prob[i] = GemmProblem{M[i], N[i], K[i], A[i], lda[i], B[i], ldb[i], acc_f32[i], ldc[i]};
  return ok(gemm_mfma_grouped_accumulate(n, prob, (hipStream_t)stream));
}
int po_op_gemm_tile(int32_t M, int32_t N, int32_t* tile_rows, int32_t* tile_cols) {
  if (!tile_rows || !tile_cols) {
    set_error("po_op_gemm_tile: NULL output");
    return PO_E_INVAL;
  }
  int bm, bn;
  gemm_mfma_tile(M, N, &bm, &bn);
  *tile_rows = bm;
  *tile_cols = bn;
  return PO_OK;
}
int po_op_attention_forward(int32_t dtype, const void* qkv, void* o, float* lse, int32_t s, int32_t h,
                            int32_t n_heads, int32_t n_kv_heads, int32_t force_generic, void* stream) {
  begin_launch();
  if (!dtype_ok(dtype)) return PO_E_INVAL;
  return ok(attention_forward(dtype, qkv, o, lse, s, h, n_heads, n_kv_heads > 0 ? n_kv_heads : n_heads,
                              force_generic != 0, (hipStream_t)stream));
}
int po_op_attention_backward(int32_t dtype, const void* qkv, const void* o, const float* lse, const void* d_o,
                             void* dqkv, float* delta, void* partials, int32_t s, int32_t h, int32_t n_heads,
                             int32_t n_kv_heads, int32_t force_generic, void* stream) {
  begin_launch();
  if (!dtype_ok(dtype)) return PO_E_INVAL;
  return ok(attention_backward(dtype, qkv, o, lse, d_o, dqkv, delta, partials, s, h, n_heads,
                               n_kv_heads > 0 ? n_kv_heads : n_heads, force_generic != 0, (hipStream_t)stream));
}
int po_op_dropout(int32_t dtype, const void* x, void* out, int32_t rows, int32_t cols, float p, uint64_t seed,
                  int32_t layer, int32_t site, int32_t mb, void* stream) {
  begin_launch();
  if (!dtype_ok(dtype)) return PO_E_INVAL;
  if (!(p >= 0.f && p < 1.f) || layer < 0 || (site != 0 && site != 1) || mb < 0) {
    set_error("po_op_dropout: p=%g layer=%d site=%d mb=%d", p, layer, site, mb);
    return PO_E_INVAL;
  }
  return ok(dropout_apply(dtype, x, nullptr, out, rows, cols, make_dropout_site(p, seed, layer, site, mb),
                          (hipStream_t)stream));
}
uint64_t po_op_colsum_workspace(int32_t rows, int32_t n) { return rows > 0 && n > 0 ? colsum_workspace(rows, n) : 0; }
int po_op_colsum_accumulate(int32_t dtype, const void* x, float* acc, float* workspace, int32_t rows, int32_t n,
                            void* stream) {
  begin_launch();
  if (!dtype_ok(dtype)) return PO_E_INVAL;
  return ok(colsum_accumulate(dtype, x, acc, workspace, rows, n, (hipStream_t)stream));
}
int po_op_colsum_accumulate_static(int32_t dtype, const void* x, float* acc, int32_t rows, int32_t n, void* stream) {
  begin_launch();
  if (!dtype_ok(dtype)) return PO_E_INVAL;
  return ok(colsum_accumulate_static(dtype, x, acc, rows, n, (hipStream_t)stream));
}
int po_op_pack(const void* const* seg_ptrs, const uint64_t* seg_bytes, int32_t n_seg, void* packed, void* stream) {
  begin_launch();
  return ok(pack_segments(seg_ptrs, seg_bytes, n_seg, packed, (hipStream_t)stream));
}
int po_op_unpack(void* const* seg_ptrs, const uint64_t* seg_bytes, int32_t n_seg, const void* packed, void* stream) {
  begin_launch();
  return ok(unpack_segments(seg_ptrs, seg_bytes, n_seg, packed, (hipStream_t)stream));
}

}  // extern "C"
