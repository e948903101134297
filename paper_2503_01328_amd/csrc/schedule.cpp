// Rank-local op order of the pipeline schedules and the placement of offload /
// reload ops around the compute passes.  Pure host code.
//
// 1F1B (Table 1, first row; Appendix A): rank i of d runs d-i-1 warm-up forwards,
// then one-forward-one-backward pairs, then drains the backwards.
// Interleaved 1F1B (Section 3.1): v chunks per rank; the n-th forward works on
// microbatch group n / (d v), chunk (n / d) % v, microbatch n % d within the
// group; backwards visit the chunks in reverse.  Warm-up is d(v-1) + 2(d-i-1)
// forwards, which gives the paper's d(v-1) + 2(d-i) - 1 forwards before the
// first backward and dv + d - 1 units in flight on rank 0.
// Generalized interleaved schedule with split backward (Sections 3.1 and 3.2): the
// inner loop repeats g microbatches (ceil(d/2) <= g <= d), rank i runs
// g(v-1) + d-i-1 warm-up forwards, and every input-gradient pass B is directly
// followed by the unit's weight-gradient pass W.  g = d is the paper's GIS (dv units
// in flight on rank 0), g = ceil(d/2) its GIS-H; in general the peak is g(v-1) + d.
// Uniformly repeated schedule (Section 2; the PO rows of Table 1, Section 3.2): every microbatch runs the same
// building block, shifted by the 3v unit-time passes a rank spends per microbatch.  The block is the steady state
// of the generalized interleaved schedule: forward one unit per rank and g slots (3g units) per chunk, backward two
// units per rank and g slots per chunk, W right after B.  A pass that would overlap the pass it depends on, or a
// pass of an earlier or later microbatch on its rank, is delayed by whole slots, which keeps each rank's F, B, W
// rhythm.  The rank's order is by start time.  (The paper leaves the collision rule to a cited work; delaying by
// whole slots in dependency order is the rule chosen here.)
// Offload placement (Section 4.2 collapsed to one rank with its own copy queues):
// OFFLOAD directly after the unit's forward; RELOAD `prefetch` compute passes
// before the unit's backward (W passes not counted: a B and its W together are one
// backward's worth of time), never before its OFFLOAD.  Units with fewer than min_gap
// forward / backward passes between their forward and backward are not offloaded
// (Section 4.4: their round trip cannot be hidden and they add nothing to the peak).
#include <math.h>

#include <algorithm>
#include <vector>

#include "../../include/pipeoffload.h"
#include "kernels.h"

namespace po {

struct Pass {
  int kind, mb, chunk;
};

// n-th forward (or backward) of a bi-level order whose inner loop repeats g microbatches
static void unit_of(int n, int g, int v, bool backward, int& mb, int& chunk) {
  int group = n / (g * v), within = n % (g * v);
  chunk = within / g;
  if (backward) chunk = v - 1 - chunk;
  mb = group * g + within % g;
}

// Start times (unit passes) of one microbatch's passes on `rank`: f, b, w indexed by chunk.
static void repeatable_block(int d, int rank, int v, int g, std::vector<long>& f, std::vector<long>& b,
                             std::vector<long>& w) {
  const long period = 3L * v, slot = 3;
  std::vector<char> taken((size_t)d * period, 0);
  auto settle = [&](int r, long t, long not_before) {
    while (t < not_before || taken[(size_t)r * period + t % period]) t += slot;
    taken[(size_t)r * period + t % period] = 1;
    return t;
  };
  f.assign(v, 0);
  b.assign(v, 0);
  w.assign(v, 0);
  long prev_end = 0;
  for (int c = 0; c < v; ++c)
    for (int r = 0; r < d; ++r) {
      long t = settle(r, 3L * g * c + r, prev_end);
      prev_end = t + 1;
      if (r == rank) f[c] = t;
    }
  const long turn = 3L * g * (v - 1) + d;  // the last forward has left the last rank
  for (int c = v - 1; c >= 0; --c)
    for (int r = d - 1; r >= 0; --r) {
      long t = settle(r, turn + 3L * g * (v - 1 - c) + 2L * (d - 1 - r), prev_end);
      prev_end = t + 1;
      long tw = settle(r, turn + 3L * g * (v - 1 - c) + 2L * (d - 1 - r) + 1, prev_end);
      if (r == rank) {
        b[c] = t;
        w[c] = tw;
      }
    }
}

static bool uniform_repeat_passes(int d, int rank, int v, int m, int g, std::vector<Pass>& out) {
  if (g <= 0) g = (d + 1) / 2;
  if (g > d || 2 * g < d) {
    set_error("schedule: group size %d outside [ceil(d/2), d] for d=%d", g, d);
    return false;
  }
  std::vector<long> f, b, w;
  repeatable_block(d, rank, v, g, f, b, w);
  struct Timed {
    long t;
    Pass p;
  };
  std::vector<Timed> all;
  all.reserve((size_t)3 * v * m);
  for (int n = 0; n < m; ++n)
    for (int c = 0; c < v; ++c) {
      long shift = 3L * v * n;
      all.push_back(Timed{f[c] + shift, Pass{0, n, c}});
      all.push_back(Timed{b[c] + shift, Pass{1, n, c}});
      all.push_back(Timed{w[c] + shift, Pass{4, n, c}});
    }
  std::sort(all.begin(), all.end(), [](const Timed& x, const Timed& y) { return x.t < y.t; });  // times are distinct
  for (const Timed& e : all) out.push_back(e.p);
  return true;
}

// Slot plan of Section 4.2 on the uniformly repeated timeline of `rank` (unit pass times, bubbles kept): one copy
// stream cut into slot pairs of 3k units, an offload slot followed by a reload slot of 1.5k units each
// (k = a unit's round trip over its F + B + W time, Eq. 1).  The units of chunks 0 .. n_sel-1 take, in the order
// their forwards end, the earliest free offload slot that starts no earlier, and, in the reverse order of their
// backwards, the latest free reload slot that ends no later; a unit whose reload would start before its offload
// has ended keeps its activations on the device (Section 4.4).  The op list holds the passes by start time and
// each copy at the start time of its slot (a copy that starts together with a pass comes first).
bool build_slot_schedule(int d, int rank, int v, int m, int g, int n_sel, double k, std::vector<po_op>& ops) {
  if (d < 1 || rank < 0 || rank >= d || v < 1 || m < 1 || n_sel < 0 || n_sel > v || !(k > 0.0)) {
    set_error("slot schedule: d=%d rank=%d v=%d m=%d chunks=%d k=%g", d, rank, v, m, n_sel, k);
    return false;
  }
  if (g <= 0) g = (d + 1) / 2;
  if (g > d || 2 * g < d) {
    set_error("schedule: group size %d outside [ceil(d/2), d] for d=%d", g, d);
    return false;
  }
  std::vector<long> f, b, w;
  repeatable_block(d, rank, v, g, f, b, w);
  const double pair = 3.0 * k, eps = 1e-9;
  struct UnitTime {
    long t;
    int mb, chunk;
  };
  std::vector<UnitTime> by_forward, by_backward;
  for (int n = 0; n < m; ++n)
    for (int c = 0; c < n_sel; ++c) {
      by_forward.push_back(UnitTime{f[c] + 3L * v * n + 1, n, c});  // end of the forward
      by_backward.push_back(UnitTime{b[c] + 3L * v * n, n, c});     // start of the backward
    }
  auto less_unit = [](const UnitTime& x, const UnitTime& y) {
    if (x.t != y.t) return x.t < y.t;
    if (x.mb != y.mb) return x.mb < y.mb;
    return x.chunk < y.chunk;
  };
  std::sort(by_forward.begin(), by_forward.end(), less_unit);
  std::sort(by_backward.begin(), by_backward.end(), [&](const UnitTime& x, const UnitTime& y) {
    if (x.t != y.t) return x.t > y.t;
    if (x.mb != y.mb) return x.mb < y.mb;
    return x.chunk < y.chunk;
  });
  std::vector<long> off_slot((size_t)m * v, -1), rel_slot((size_t)m * v, -1);
  std::vector<long> taken;  // kept sorted
  auto is_taken = [&](long i) { return std::binary_search(taken.begin(), taken.end(), i); };
  auto take = [&](long i) { taken.insert(std::upper_bound(taken.begin(), taken.end(), i), i); };
  for (const UnitTime& u : by_forward) {
    long i = (long)ceil((double)u.t / pair - eps);
    if (i < 0) i = 0;
    while (is_taken(i)) ++i;
    take(i);
    off_slot[(size_t)u.chunk * m + u.mb] = i;
  }
  taken.clear();
  for (const UnitTime& u : by_backward) {
    long j = (long)floor((double)u.t / pair + eps) - 1;  // reload slot j ends at pair (j + 1)
    while (is_taken(j)) --j;
    take(j);
    rel_slot[(size_t)u.chunk * m + u.mb] = j;
  }
  struct Event {
    double t;
    int is_pass, not_reload;
    po_op op;
  };
  std::vector<Event> ev;
  for (int n = 0; n < m; ++n)
    for (int c = 0; c < v; ++c) {
      long shift = 3L * v * n;
      ev.push_back(Event{(double)(f[c] + shift), 1, 1, po_op{0, n, c, 0.f}});
      ev.push_back(Event{(double)(b[c] + shift), 1, 1, po_op{1, n, c, 0.f}});
      ev.push_back(Event{(double)(w[c] + shift), 1, 1, po_op{4, n, c, 0.f}});
      if (c < n_sel) {
        long i = off_slot[(size_t)c * m + n], j = rel_slot[(size_t)c * m + n];
        if (j >= i) {
          ev.push_back(Event{pair * (double)i, 0, 1, po_op{2, n, c, 1.0f}});
          ev.push_back(Event{pair * (double)j + pair / 2, 0, 0, po_op{3, n, c, 1.0f}});
        }
      }
    }
  std::sort(ev.begin(), ev.end(), [](const Event& x, const Event& y) {
    if (x.t != y.t) return x.t < y.t;
    if (x.is_pass != y.is_pass) return x.is_pass < y.is_pass;
    if (x.not_reload != y.not_reload) return x.not_reload < y.not_reload;
    if (x.op.mb != y.op.mb) return x.op.mb < y.op.mb;
    return x.op.chunk < y.op.chunk;
  });
  ops.clear();
  for (const Event& e : ev) ops.push_back(e.op);
  return true;
}

static bool compute_passes(int schedule, int d, int rank, int v, int m, int g, std::vector<Pass>& out) {
  if (d < 1 || rank < 0 || rank >= d || v < 1 || m < 1) {
    set_error("schedule: d=%d rank=%d v=%d m=%d", d, rank, v, m);
    return false;
  }
  if (schedule == PO_SCHED_PO) return uniform_repeat_passes(d, rank, v, m, g, out);
  int total, warm;
  if (schedule == PO_SCHED_1F1B) {
    if (v != 1) {
      set_error("schedule: 1F1B runs one chunk per rank (v=%d)", v);
      return false;
    }
    total = m;
    warm = d - rank - 1;
  } else if (schedule == PO_SCHED_1F1B_INTERLEAVED) {
    if (m % d != 0) {
      set_error("schedule: interleaved 1F1B needs m (%d) to be a multiple of d (%d)", m, d);
      return false;
    }
    total = m * v;
    warm = (v - 1) * d + 2 * (d - rank - 1);
    g = d;
  } else if (schedule == PO_SCHED_GIS) {
    if (g <= 0) g = d;
    if (g > d || 2 * g < d) {
      set_error("schedule: group size %d outside [ceil(d/2), d] for d=%d", g, d);
      return false;
    }
    if (m % g != 0) {
      set_error("schedule: m (%d) must be a multiple of the group size (%d)", m, g);
      return false;
    }
    total = m * v;
    warm = g * (v - 1) + d - rank - 1;
  } else {
    set_error("schedule: unknown schedule %d", schedule);
    return false;
  }
  if (warm > total) warm = total;
  auto emit = [&](int kind, int n) {
    Pass p;
    p.kind = kind;
    if (schedule == PO_SCHED_1F1B) {
      p.mb = n;
      p.chunk = 0;
    } else {
      unit_of(n, g, v, kind != 0, p.mb, p.chunk);
    }
    out.push_back(p);
  };
  const bool split = schedule == PO_SCHED_GIS;
  for (int n = 0; n < warm; ++n) emit(0, n);
  for (int n = 0; n + warm < total; ++n) {
    emit(0, warm + n);
    emit(1, n);
    if (split) emit(4, n);
  }
  for (int n = total - warm; n < total; ++n) {
    emit(1, n);
    if (split) emit(4, n);
  }
  return true;
}

static bool unit_selected(int mb, int chunk, int v, float ratio, int policy) {
  const double eps = 1e-9;
  if (policy == PO_SEL_LONGEST_LIFESPAN && v > 1) return chunk < (int)ceil((double)ratio * v - eps);
  return floor((mb + 1) * (double)ratio + eps) > floor(mb * (double)ratio + eps);
}

bool build_schedule(int schedule, int d, int rank, int v, int m, int group, float ratio, int policy, int prefetch,
                    int min_gap, std::vector<po_op>& ops) {
  if (!(ratio >= 0.f && ratio <= 1.f) || prefetch < 0 || min_gap < 0 ||
      (policy != PO_SEL_ALTERNATE_MB && policy != PO_SEL_LONGEST_LIFESPAN)) {
    set_error("schedule: ratio=%g prefetch=%d min_gap=%d policy=%d", ratio, prefetch, min_gap, policy);
    return false;
  }
  std::vector<Pass> passes;
  if (!compute_passes(schedule, d, rank, v, m, group, passes)) return false;
  int np = (int)passes.size();
  // position of each unit's forward
  std::vector<int> fpos((size_t)m * v, -1);
  for (int n = 0; n < np; ++n)
    if (passes[n].kind == 0) fpos[(size_t)passes[n].chunk * m + passes[n].mb] = n;
  // units that are offloaded: selected by the ratio, and (Section 4.4) with at least min_gap forward / backward
  // passes between their forward and their backward
  std::vector<char> offloaded((size_t)m * v, 0);
  {
    std::vector<int> fb_index((size_t)m * v, 0);
    int count = 0;
    for (int n = 0; n < np; ++n) {
      const Pass& p = passes[n];
      if (p.kind == 4) continue;
      size_t u = (size_t)p.chunk * m + p.mb;
      if (p.kind == 0)
        fb_index[u] = count;
      else
        offloaded[u] = unit_selected(p.mb, p.chunk, v, ratio, policy) && count - fb_index[u] - 1 >= min_gap;
      ++count;
    }
  }
  // reloads to emit before pass n
  std::vector<std::vector<Pass>> before(np);
  for (int n = 0; n < np; ++n) {
    const Pass& p = passes[n];
    if (p.kind != 1 || !offloaded[(size_t)p.chunk * m + p.mb]) continue;
    int at = n;  // walk back over `prefetch` forward / backward passes; W passes ride along uncounted
    for (int counted = 0; counted < prefetch && at > 0;) {
      --at;
      if (passes[at].kind != 4) ++counted;
    }
    int lo = fpos[(size_t)p.chunk * m + p.mb] + 1;
    if (at < lo) at = lo;
    before[at].push_back(p);
  }
  ops.clear();
  for (int n = 0; n < np; ++n) {
    for (const Pass& r : before[n]) ops.push_back(po_op{3, r.mb, r.chunk, 1.0f});
    ops.push_back(po_op{passes[n].kind, passes[n].mb, passes[n].chunk, 0.f});
    if (passes[n].kind == 0 && offloaded[(size_t)passes[n].chunk * m + passes[n].mb])
      ops.push_back(po_op{2, passes[n].mb, passes[n].chunk, 1.0f});
  }
  return true;
}

}  // namespace po
