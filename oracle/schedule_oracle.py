"""CPU oracle for the per-rank pipeline op order, offload selection and residency.

TEST INFRASTRUCTURE ONLY: the product path never imports this module.  It is an
independent model, in plain Python integers, of what one pipeline rank executes:

* 1F1B: rank i of d runs d-i-1 warm-up forwards, then alternates one forward
  and one backward, then drains the remaining backwards (Table 1, first row;
  Appendix A).
* Interleaved 1F1B: v chunks per rank, bi-level order (Section 2: the outer
  loop walks the chunks, the inner loop repeats d microbatches), with
  d(v-1) + 2(d-i) - 1 forwards before the first backward on rank i and a peak
  of dv + d - 1 units in flight on rank 0 (Section 3.1, warm-up paragraph).
* Offload: a selected unit is offloaded right after its forward and reloaded
  ``prefetch`` compute passes ahead of its backward (Section 4.2: earliest
  slot after the forward, latest slot before the backward; on a single rank
  with a dedicated copy queue these collapse to these two rules).

* Generalized interleaved schedule (Section 3.1 "free lunch" and Section 3.2):
  the backward is split into an input-gradient pass B and a weight-gradient
  pass W that directly follows it; the inner loop repeats g microbatches
  (ceil(d/2) <= g <= d) instead of d; rank i forwards g(v-1) + d - i units
  before its first backward.  g = d is the schedule the paper calls GIS
  (warm-up d(v-1) + d - i, peak dv on rank 0), g = ceil(d/2) is GIS-H; in
  general the rank-0 peak is g(v-1) + d.
* pipeline_timeline runs the op lists of all d ranks against each other with
  given pass durations, which yields the bubble sizes of Table 1.
* Uniform repeating (Section 2; the schedule Section 3.2 calls PO): one
  microbatch's passes form a building block, here the steady state of the
  generalized interleaved schedule (a chunk every g slots going forward and
  coming back, d slots for the round trip through the last chunk, a slot being
  one F, one B and one W); microbatch n runs the block n periods later, a
  period being the 3v unit-time passes a rank spends on one microbatch.  A
  rank's op order is its passes sorted by time.  Passes whose times collide
  modulo the period on a rank are moved later by whole slots (the paper leaves
  the collision rule to a cited work; this greedy rule is this build's reading).
  Peak memory is then about the summed lifespans over the period, which gives
  the stage-level selective offload of Section 2 (longest lifespan first) its
  better-than-linear effect.
* Slot placement (Section 4.2): on the unsqueezed uniformly repeated timeline a
  single copy stream is cut into alternating offload and reload slots whose
  length follows from k; offloads take the earliest free slot after their
  forward, reloads the latest free slot before their backward.

Op tuples are (kind, mb, chunk) with kind in {"F", "B", "W", "OFFLOAD", "RELOAD"}.
"""
from __future__ import annotations

import math


def one_f_one_b(d, rank, m):
    """Compute passes of 1F1B on ``rank`` for m microbatches (one chunk)."""
    warm = min(d - rank - 1, m)
    ops = [("F", j, 0) for j in range(warm)]
    for j in range(m - warm):
        ops.append(("F", warm + j, 0))
        ops.append(("B", j, 0))
    for j in range(m - warm, m):
        ops.append(("B", j, 0))
    return ops


def _interleaved_unit(k, d, v, backward):
    group, within = divmod(k, d * v)
    chunk = within // d
    mb = group * d + within % d
    return (mb, v - 1 - chunk) if backward else (mb, chunk)


def interleaved_one_f_one_b(d, rank, v, m):
    """Compute passes of interleaved 1F1B on ``rank``: m microbatches (m % d == 0),
    v chunks.  The k-th forward handles microbatch group k // (d v), chunk
    (k // d) % v; backwards walk the chunks in reverse."""
    if m % d:
        raise ValueError("interleaved 1F1B needs m to be a multiple of d")
    total = m * v
    warm = min((v - 1) * d + 2 * (d - rank - 1), total)
    ops = []
    for k in range(warm):
        ops.append(("F",) + _interleaved_unit(k, d, v, False))
    for j in range(total - warm):
        ops.append(("F",) + _interleaved_unit(warm + j, d, v, False))
        ops.append(("B",) + _interleaved_unit(j, d, v, True))
    for j in range(total - warm, total):
        ops.append(("B",) + _interleaved_unit(j, d, v, True))
    return ops


def _grouped_unit(k, g, v, backward):
    group, within = divmod(k, g * v)
    chunk = within // g
    mb = group * g + within % g
    return (mb, v - 1 - chunk) if backward else (mb, chunk)


def generalized_interleaved(d, rank, v, m, g=None):
    """Compute passes of the generalized interleaved schedule with split backward
    on ``rank`` (Sections 3.1 and 3.2): the k-th forward handles microbatch group
    k // (g v), chunk (k // g) % v; the backward passes walk the chunks in reverse
    and each input-gradient pass B is directly followed by its weight-gradient
    pass W.  g defaults to d (GIS)."""
    g = d if g is None else g
    if not (math.ceil(d / 2) <= g <= d):
        raise ValueError("the group size must lie in [ceil(d/2), d]")
    if m % g:
        raise ValueError("the schedule needs m to be a multiple of the group size")
    total = m * v
    warm = min(g * (v - 1) + d - rank - 1, total)
    ops = [("F",) + _grouped_unit(k, g, v, False) for k in range(warm)]
    for j in range(total - warm):
        ops.append(("F",) + _grouped_unit(warm + j, g, v, False))
        ops.append(("B",) + _grouped_unit(j, g, v, True))
        ops.append(("W",) + _grouped_unit(j, g, v, True))
    for j in range(total - warm, total):
        ops.append(("B",) + _grouped_unit(j, g, v, True))
        ops.append(("W",) + _grouped_unit(j, g, v, True))
    return ops


def pipeline_timeline(rank_ops, d, v, t_f, t_b, t_w):
    """Runs the op lists of all d ranks (compute passes only) against each other.

    Model stage c d + i lives on rank i as chunk c.  F(mb, c) on rank i needs the
    same forward on rank i-1, or on rank d-1 for chunk c-1 when i = 0.  B(mb, c)
    needs its own forward and the same backward on rank i+1, or on rank 0 for chunk
    c+1 when i = d-1.  W needs its own B.  A rank whose list has no W passes runs
    fused backwards of duration t_b + t_w.  Returns (makespan, finished) where
    finished is False when the lists deadlock."""
    done = {}
    ptr = [0] * d
    free = [0.0] * d
    split = [any(op[0] == "W" for op in ops) for ops in rank_ops]
    progress = True
    while progress:
        progress = False
        for i in range(d):
            while ptr[i] < len(rank_ops[i]):
                kind, mb, c = rank_ops[i][ptr[i]]
                if kind == "F":
                    deps = [(i - 1, "F", mb, c)] if i > 0 else ([(d - 1, "F", mb, c - 1)] if c > 0 else [])
                    t = t_f
                elif kind == "B":
                    deps = [(i, "F", mb, c)]
                    if i < d - 1:
                        deps.append((i + 1, "B", mb, c))
                    elif c < v - 1:
                        deps.append((0, "B", mb, c + 1))
                    t = t_b if split[i] else t_b + t_w
                elif kind == "W":
                    deps = [(i, "B", mb, c)]
                    t = t_w
                else:
                    raise ValueError(kind)
                if any(dep not in done for dep in deps):
                    break
                start = max([free[i]] + [done[dep] for dep in deps])
                free[i] = start + t
                done[(i, kind, mb, c)] = free[i]
                ptr[i] += 1
                progress = True
    finished = all(ptr[i] == len(rank_ops[i]) for i in range(d))
    return max(free), finished


def building_block_template(d, v, g):
    """Unit-time (F = B = W = 1) start times of one microbatch's passes in the
    steady state of the generalized interleaved schedule with group size g
    (Section 3.2): the forward moves one unit per rank and 3g units (g slots) per
    chunk; the backward of the last chunk starts when its forward has left rank
    d-1, moves two units per rank (a rank in a one-forward-one-backward rhythm
    starts B one slot minus one forward after its successor) and 3g units per
    chunk; W directly follows B.  On rank 0 chunk c then lives for
    6g(v-1-c) + 3d units, and the lifespans of a rank's chunks divided by the
    period 3v add up to the g(v-1) + d units of Section 3.2.
    Keys are (kind, rank, chunk)."""
    t = {}
    turn = 3 * g * (v - 1) + d
    for c in range(v):
        for i in range(d):
            t[("F", i, c)] = 3 * g * c + i
            t[("B", i, c)] = turn + 3 * g * (v - 1 - c) + 2 * (d - 1 - i)
            t[("W", i, c)] = t[("B", i, c)] + 1
    return t


def building_block(d, v, g):
    """The template made repeatable with period 3v: passes are placed in dependency
    order (forwards up the model stages, then backwards down, each W right after
    its B); a pass that would start before the pass it depends on has ended, or
    whose time modulo 3v is taken on its rank, moves later by whole slots (3
    units).  The template puts rank i's F, B and W at times i, i+1 and i+2 modulo
    3, so whole-slot moves keep every rank in a steady F, B, W rhythm, which is
    what lets the resulting order run without stalls when the three pass times
    differ; each kind has v places in the period and v passes, so a place is
    always found."""
    want = building_block_template(d, v, g)
    period = 3 * v
    used = [set() for _ in range(d)]
    placed = {}

    def place(key, earliest):
        t = want[key]
        while t < earliest or t % period in used[key[1]]:
            t += 3
        used[key[1]].add(t % period)
        placed[key] = t
        return t

    last = -1
    for stage in range(d * v):
        c, i = divmod(stage, d)
        last = place(("F", i, c), last + 1)
    for stage in reversed(range(d * v)):
        c, i = divmod(stage, d)
        last = place(("B", i, c), last + 1)
        place(("W", i, c), last + 1)
    return placed


def uniform_repeat(d, rank, v, m, g=None):
    """Compute passes of the uniformly repeated schedule on ``rank``: microbatch n
    runs the building block 3v n units later; the rank's order is by start time.
    g defaults to ceil(d/2), the block of GIS-H that Section 3.2 repeats."""
    g = math.ceil(d / 2) if g is None else g
    if not (math.ceil(d / 2) <= g <= d):
        raise ValueError("the group size must lie in [ceil(d/2), d]")
    block = building_block(d, v, g)
    timed = []
    for (kind, i, c), t in block.items():
        if i == rank:
            for n in range(m):
                timed.append((t + 3 * v * n, kind, n, c))
    timed.sort()
    return [(kind, n, c) for _, kind, n, c in timed]


def uniform_repeat_times(d, rank, v, m, g=None):
    """The uniformly repeated schedule of ``rank`` with its unit-time start times (bubbles kept): a list of
    (start, kind, mb, chunk) sorted by start."""
    g = math.ceil(d / 2) if g is None else g
    block = building_block(d, v, g)
    timed = [(t + 3 * v * n, kind, n, c) for (kind, i, c), t in block.items() if i == rank for n in range(m)]
    timed.sort()
    return timed


def slot_placement(timed, offload_chunks, k):
    """Offload and reload slots on one shared copy stream (Section 4.2, Figure 7).

    ``timed``: a rank's passes with unit-time starts (F = B = W = 1).  k (Eq. 1): a unit's round trip over its
    F + B + W time, so an offload takes 1.5 k units and a reload the same.  The stream is cut into slots in a
    one-offload-one-reload pattern from time 0: offload slot i is [3 k i, 3 k i + 1.5 k), reload slot i follows
    it up to 3 k (i + 1).  The units of the chosen chunks are taken left to right by the end of their forward
    and get the earliest free offload slot that starts no earlier; then right to left by the start of their
    backward and get the latest free reload slot that ends no later.  A unit whose reload slot would start
    before its offload slot has ended is not offloaded at all (Section 4.4: its gap is shorter than the round
    trip); its slots stay empty, like every slot nobody claimed.
    Returns {(mb, chunk): (offload_slot, reload_slot)}."""
    if k <= 0:
        raise ValueError("k must be positive")
    pair = 3.0 * k
    f_end, b_start = {}, {}
    for start, kind, mb, c in timed:
        if c in offload_chunks:
            if kind == "F":
                f_end[(mb, c)] = start + 1
            elif kind == "B":
                b_start[(mb, c)] = start
    eps = 1e-9
    off_slot, used = {}, set()
    for u in sorted(f_end, key=lambda u: (f_end[u], u)):
        i = max(0, math.ceil(f_end[u] / pair - eps))
        while i in used:
            i += 1
        used.add(i)
        off_slot[u] = i
    rel_slot, used = {}, set()
    for u in sorted(b_start, key=lambda u: (-b_start[u], u)):
        i = math.floor(b_start[u] / pair + eps) - 1  # reload slot i ends at pair (i + 1)
        while i in used:
            i -= 1
        used.add(i)
        rel_slot[u] = i
    # reload slot i starts at pair i + pair / 2, offload slot j ends at pair j + pair / 2
    return {u: (off_slot[u], rel_slot[u]) for u in off_slot if rel_slot[u] >= off_slot[u]}


def with_slot_offload(timed, placement, k):
    """Op list of the slot plan: compute passes by start time, OFFLOAD / RELOAD ops at the start times of
    their slots (a copy that starts together with a pass is listed first)."""
    pair = 3.0 * k
    events = [(start, 1, (kind, mb, c)) for start, kind, mb, c in timed]
    for (mb, c), (i, j) in placement.items():
        events.append((pair * i, 0, ("OFFLOAD", mb, c)))
        events.append((pair * j + pair / 2, 0, ("RELOAD", mb, c)))
    events.sort(key=lambda e: (e[0], e[1], e[2][0] != "RELOAD", e[2][1:]))
    return [op for _, _, op in events]


def peak_units(passes, offloaded_chunks=()):
    """Largest number of units a rank holds at once when the chunks in
    ``offloaded_chunks`` cost nothing (the idealised stage-level offload of Section 2,
    Figure 4: copies are instantaneous and leave no transient).  A unit is held
    from its F to its W, or to its B when the backward is fused."""
    split = any(op[0] == "W" for op in passes)
    held = peak = 0
    for kind, _, c in passes:
        if c in offloaded_chunks:
            continue
        if kind == "F":
            held += 1
        elif kind == ("W" if split else "B"):
            held -= 1
        peak = max(peak, held)
    return peak


def chunks_by_lifespan(passes, v):
    """Chunks of a rank ordered for selective offload (Section 2): longest mean
    forward-to-backward gap first, ties by chunk index."""
    gap = forward_backward_gaps(passes)
    total, count = [0] * v, [0] * v
    for (_, c), n in gap.items():
        total[c] += n
        count[c] += 1
    return sorted(range(v), key=lambda c: (-total[c] / max(count[c], 1), c))


def compute_passes(schedule, d, rank, v, m, g=None):
    if schedule == "po":
        return uniform_repeat(d, rank, v, m, g)
    if schedule == "gis":
        return generalized_interleaved(d, rank, v, m, g)
    if schedule == "1f1b":
        if v != 1:
            raise ValueError("1F1B has one chunk per rank")
        return one_f_one_b(d, rank, m)
    if schedule == "1f1b-interleaved":
        return interleaved_one_f_one_b(d, rank, v, m)
    raise ValueError(schedule)


def selected_units(m, v, ratio, policy="alternate-mb"):
    """Which (mb, chunk) units are offloaded for a whole-job offload ratio.

    alternate-mb: microbatch j is offloaded iff floor((j+1) r) > floor(j r)
    (r = 1 all, r = 0.5 the odd ones, r = 0 none), all of its chunks.
    longest-lifespan (Section 2: prefer the chunks whose forward-to-backward gap
    is longest, i.e. the lowest chunk indices): chunks 0 .. ceil(r v) - 1 of
    every microbatch; with one chunk it degenerates to alternate-mb.
    """
    if not 0.0 <= ratio <= 1.0:
        raise ValueError("ratio must be in [0, 1]")
    sel = set()
    if policy == "longest-lifespan" and v > 1:
        n = math.ceil(ratio * v - 1e-9)
        for j in range(m):
            for c in range(n):
                sel.add((j, c))
        return sel
    for j in range(m):
        if math.floor((j + 1) * ratio + 1e-9) > math.floor(j * ratio + 1e-9):
            for c in range(v):
                sel.add((j, c))
    return sel


def forward_backward_gaps(passes):
    """For every unit, the number of forward / backward passes that run strictly
    between its forward and its backward (weight-gradient passes not counted)."""
    pos, gap = {}, {}
    n = 0
    for kind, mb, c in passes:
        if kind == "W":
            continue
        if kind == "F":
            pos[(mb, c)] = n
        else:
            gap[(mb, c)] = n - pos[(mb, c)] - 1
        n += 1
    return gap


def with_offload(passes, selected, prefetch=1, min_gap=0):
    """Insert OFFLOAD / RELOAD ops into a list of compute passes.

    OFFLOAD(u) directly follows F(u).  RELOAD(u) is placed directly before the
    compute pass that runs ``prefetch`` passes ahead of B(u) (prefetch = 0:
    directly before B(u) itself), but never before OFFLOAD(u).  Weight-gradient
    passes are not counted: a (B, W) pair is one backward's worth of time, so the
    same ``prefetch`` buys the same lead with fused and with split backwards.

    min_gap (Section 4.4, second caveat): a selected unit with fewer than min_gap
    forward / backward passes between its forward and its backward is not
    offloaded at all; its round trip could not be hidden and it adds next to
    nothing to the peak.
    """
    if min_gap > 0:
        gap = forward_backward_gaps(passes)
        selected = {u for u in selected if gap[u] >= min_gap}
    pos_f = {(mb, c): n for n, (kind, mb, c) in enumerate(passes) if kind == "F"}
    reload_before = {}
    for n, (kind, mb, c) in enumerate(passes):
        if kind == "B" and (mb, c) in selected:
            at, counted = n, 0
            while counted < prefetch and at > 0:
                at -= 1
                if passes[at][0] != "W":
                    counted += 1
            at = max(at, pos_f[(mb, c)] + 1)
            reload_before.setdefault(at, []).append((mb, c))
    ops = []
    for n, (kind, mb, c) in enumerate(passes):
        for u in reload_before.get(n, []):
            ops.append(("RELOAD",) + u)
        ops.append((kind, mb, c))
        if kind == "F" and (mb, c) in selected:
            ops.append(("OFFLOAD", mb, c))
    return ops


def simulate(ops):
    """Walk an op list with zero-time copies.  Returns a dict with the peak
    number of units in flight (forwarded, not yet backwarded), the peak number
    resident on the device, forwards before the first backward, and a list of
    violated invariants (empty when the list is a valid schedule).  With split
    backward passes a unit leaves the in-flight count at B (the paper's activation
    count) and leaves the device at W."""
    state = {}
    errors = []
    split = any(op[0] == "W" for op in ops)
    in_flight = resident = peak_in_flight = peak_resident = 0
    forwards_before_first_backward = None
    n_forward = 0
    for n, (kind, mb, c) in enumerate(ops):
        u = (mb, c)
        st = state.get(u, "EMPTY")
        if kind == "F":
            if st != "EMPTY":
                errors.append(f"op {n}: forward of live unit {u}")
            state[u] = "RESIDENT"
            in_flight += 1
            resident += 1
            n_forward += 1
        elif kind == "OFFLOAD":
            if st != "RESIDENT":
                errors.append(f"op {n}: offload of unit {u} in state {st}")
            state[u] = "HOST"
            resident -= 1
        elif kind == "RELOAD":
            if st != "HOST":
                errors.append(f"op {n}: reload of unit {u} in state {st}")
            state[u] = "RESIDENT"
            resident += 1
        elif kind == "B":
            if st != "RESIDENT":
                errors.append(f"op {n}: backward of unit {u} in state {st}")
            if forwards_before_first_backward is None:
                forwards_before_first_backward = n_forward
            in_flight -= 1
            if split:
                state[u] = "WEIGHT-PENDING"  # its activations stay on the device until W
            else:
                state[u] = "DONE"
                resident -= 1
        elif kind == "W":
            if st != "WEIGHT-PENDING":
                errors.append(f"op {n}: weight-gradient pass of unit {u} in state {st}")
            state[u] = "DONE"
            resident -= 1
        else:
            errors.append(f"op {n}: unknown kind {kind}")
        peak_in_flight = max(peak_in_flight, in_flight)
        peak_resident = max(peak_resident, resident)
    for u, st in state.items():
        if st != "DONE":
            errors.append(f"unit {u} ends in state {st}")
    return dict(peak_in_flight=peak_in_flight, peak_resident=peak_resident,
                forwards_before_first_backward=forwards_before_first_backward, errors=errors)


def check_dependencies(passes, v):
    """Within one microbatch a rank must forward chunk c before chunk c+1 and
    backward chunk c+1 before chunk c, forward a unit before its backward, and run
    a weight-gradient pass after the unit's input-gradient pass."""
    pos = {(kind, mb, c): n for n, (kind, mb, c) in enumerate(passes)}
    bad = []
    for (kind, mb, c), n in pos.items():
        if kind == "F" and c + 1 < v and pos[("F", mb, c + 1)] < n:
            bad.append(("F-order", mb, c))
        if kind == "B" and c + 1 < v and pos[("B", mb, c + 1)] > n:
            bad.append(("B-order", mb, c))
        if kind == "B" and pos[("F", mb, c)] > n:
            bad.append(("B-before-F", mb, c))
        if kind == "W" and pos[("B", mb, c)] > n:
            bad.append(("W-before-B", mb, c))
    return bad


def offload_ratio_k(h, s, compute_flops_per_s, link_bytes_per_s):
    """Eq. 1: round-trip offload time over forward+backward compute time of one
    layer, k = 10 / (3 (6h + s)) * B_c / B_o."""
    return 10.0 / (3.0 * (6.0 * h + s)) * compute_flops_per_s / link_bytes_per_s


def saved_bytes_per_layer(s, h, n_heads, elem_bytes, n_kv_heads=None):
    """Appendix C: 20 b s h bytes per layer at 2-byte elements once LayerNorm,
    GeLU and dropout outputs are recomputed, i.e. 10 s h elements: layer input,
    q, k, v, attention output, second LayerNorm's input and the 4h-wide MLP
    pre-activation.  With grouped-query attention k and v shrink to
    n_kv_heads / n_heads of h each.  This build also keeps the softmax
    log-sum-exp per head and row in fp32 (needed by a score-free attention backward)."""
    kv = h if n_kv_heads is None else h // n_heads * n_kv_heads
    return (8 * h + 2 * kv) * s * elem_bytes + 4 * n_heads * s
