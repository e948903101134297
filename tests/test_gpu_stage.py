"""Stage-level parity against the CPU oracle and the offload exactness checks.

Gradients, outputs and input gradients of the HIP path are compared per tensor
with max |got - ref| / max |ref| and with the relative L2 norm (both printed): 1e-4 in fp32, 2e-2 in bf16.  With offload the
HIP path must reproduce its own no-offload results bit for bit (offload is a copy)."""
import numpy as np
import pytest
import torch

from oracle import schedule_oracle as sch
from oracle import stage_oracle as so
from paper_2503_01328_amd import binding as po
from paper_2503_01328_amd import inputs as syn
from paper_2503_01328_amd.harness import StageRunner, check_parity, max_rel_err

pytestmark = pytest.mark.gpu


def _oracle(shape, runner, m):
    x = {(j, c): syn.unit_input(shape, j, c, runner.seed) for j in range(m) for c in range(shape.n_chunks)}
    dy = {(j, c): syn.unit_upstream_grad(shape, j, c, runner.seed) for j in range(m) for c in range(shape.n_chunks)}
    return so.run_stage(runner.params_np, shape.n_layers, shape.n_chunks, shape.n_heads, x, dy, vocab=shape.vocab)


def _compare(shape, got, ref, tol):
    """Every output, input gradient and parameter gradient tensor in both norms (max norm and relative L2, both
    printed and both held to `tol`); returns the worst max-norm figure of the layer gradients."""
    y, dx, g = got
    ry, rdx, rg = ref
    worst = 0.0
    for u in ry:
        check_parity(y[u], ry[u], tol, f"y {u}")
        if rdx[u] is not None:
            check_parity(dx[u], rdx[u], tol, f"dx {u}")
    for l in range(shape.n_layers):
        for k, a in rg["layers"][l].items():
            worst = max(worst, check_parity(g["layers"][l][k], a, tol, f"grad layer {l} {k}")[0])
    for k in ("wte", "wpe"):
        if k in rg:
            check_parity(g[k], rg[k], tol, f"grad {k}")
    return worst


def _snapshot(r):
    torch.cuda.synchronize()
    return ([t.clone() for t in r.y], [None if t is None else t.clone() for t in r.dx], r.grads.clone())


def _assert_bit_identical(a, b):
    for ta, tb in zip(a[0], b[0]):
        assert torch.equal(ta, tb)
    for ta, tb in zip(a[1], b[1]):
        assert (ta is None and tb is None) or torch.equal(ta, tb)
    assert torch.equal(a[2], b[2])


def test_config1_tiny_gpt_fp32_against_oracle_with_full_offload(gpu_device):
    shape = syn.CONFIGS["C1"]
    with StageRunner(shape) as r:
        r.make_inputs()
        stats = r.run(po.PO_SCHED_1F1B, 1.0)
        assert stats["n_offloads"] == 4 * 2 and stats["n_reloads"] == 4 * 2
        assert stats["peak_in_flight_units"] == 2
        got = r.results()
        _compare(shape, got, _oracle(shape, r, 4), 1e-4)
        with_offload = _snapshot(r)
        r.zero_grads()
        r.run(po.PO_SCHED_1F1B, 0.0)
        _assert_bit_identical(with_offload, _snapshot(r))


SMALL_BF16 = syn.StageShape(2, 1, 256, 2, 1024, 384, dtype="bf16", pipeline_degree=3, n_microbatches=5)
SMALL_BF16_RAGGED = syn.StageShape(1, 1, 192, 3, 320, 200, dtype="bf16", pipeline_degree=2, n_microbatches=3)


@pytest.mark.parametrize("shape", [SMALL_BF16, SMALL_BF16_RAGGED], ids=["mfma-tiles", "ragged-generic"])
def test_bf16_stage_against_oracle(gpu_device, shape):
    with StageRunner(shape) as r:
        r.make_inputs()
        r.run(po.PO_SCHED_1F1B, 0.5)
        _compare(shape, r.results(), _oracle(shape, r, shape.n_microbatches), 2e-2)


@pytest.mark.parametrize("shape", [SMALL_BF16, syn.StageShape(2, 1, 128, 2, 512, 96, vocab=50, dtype="f32",
                                                             pipeline_degree=4, n_microbatches=6)],
                         ids=["bf16", "f32-embed"])
def test_offload_is_bit_identical_in_every_mode(gpu_device, shape):
    base = None
    for kw in [dict(ratio=0.0), dict(ratio=0.5), dict(ratio=1.0), dict(ratio=1.0, copy_streams=1),
               dict(ratio=1.0, staged_copies=1), dict(ratio=0.5, staged_copies=1, copy_streams=1),
               dict(ratio=1.0, prefetch_passes=0), dict(ratio=1.0, prefetch_passes=3),
               dict(ratio=1.0, debug_poison=1), dict(ratio=1.0, debug_poison=1, staged_copies=1),
               dict(ratio=0.0, weight_stream=1), dict(ratio=1.0, weight_stream=1),
               dict(ratio=1.0, weight_stream=1, debug_poison=1, prefetch_passes=1)]:
        ratio = kw.pop("ratio")
        with StageRunner(shape, **kw) as r:
            r.make_inputs()
            stats = r.run(po.PO_SCHED_1F1B, ratio)
            snap = _snapshot(r)
            # second run on the same stage (pools warm, slabs reused) must agree as well
            r.zero_grads()
            stats2 = r.run(po.PO_SCHED_1F1B, ratio)
            _assert_bit_identical(snap, _snapshot(r))
            assert stats2["pool_bytes_allocated"] == stats["pool_bytes_allocated"]
            # copy time hidden behind compute: none without copies, never more than the copies took
            busy = stats2["d2h_busy_s"] + stats2["h2d_busy_s"]
            assert 0.0 <= stats2["copy_hidden_s"] <= busy * (1 + 1e-6) + 1e-9
            assert (busy == 0.0) == (ratio == 0.0)
        if base is None:
            base = snap
        else:
            _assert_bit_identical(base, snap)


def test_interleaved_schedule_chunks_and_residency(gpu_device):
    shape = syn.StageShape(4, 2, 128, 2, 512, 64, dtype="bf16", pipeline_degree=2, n_microbatches=4)
    results = {}
    for ratio, policy in [(0.0, 0), (0.5, 0), (0.5, 1), (1.0, 0)]:
        with StageRunner(shape, select_policy=policy) as r:
            r.make_inputs()
            stats = r.run(po.PO_SCHED_1F1B_INTERLEAVED, ratio)
            results[(ratio, policy)] = _snapshot(r)
            ops = sch.with_offload(sch.interleaved_one_f_one_b(2, 0, 2, 4),
                                   sch.selected_units(4, 2, ratio, "longest-lifespan" if policy else "alternate-mb"),
                                   r.cfg.prefetch_passes)
            model = sch.simulate(ops)
            assert stats["peak_in_flight_units"] == model["peak_in_flight"]
            assert stats["peak_resident_units"] == model["peak_resident"]
            assert stats["n_offloads"] == sum(o[0] == "OFFLOAD" for o in ops) * 2  # two layers per unit
            if ratio == 0.0:
                _compare(shape, r.results(), _oracle(shape, r, 4), 2e-2)
    base = results[(0.0, 0)]
    for k, v in results.items():
        _assert_bit_identical(base, v)


def test_manual_calls_partial_ratio_and_state_errors(gpu_device):
    shape = syn.StageShape(4, 1, 128, 2, 512, 64, dtype="f32", pipeline_degree=2, n_microbatches=2)
    with StageRunner(shape) as r:
        r.make_inputs()
        st = r.stage
        layer_bytes = po.po_saved_bytes_per_layer(r.cfg)
        po.po_stage_forward(st, 0, 0, r.x[0], r.y[0])
        with pytest.raises(po.PipeOffloadError) as e:
            po.po_stage_forward(st, 0, 0, r.x[0], r.y[0])  # still in flight
        assert e.value.code == po.PO_E_STATE
        with pytest.raises(po.PipeOffloadError) as e:
            po.po_stage_backward(st, 1, 0, r.dy[1], r.dx[1])  # never forwarded
        assert e.value.code == po.PO_E_STATE
        with pytest.raises(po.PipeOffloadError) as e:
            po.po_offload(st, 0, 0, 1.5)
        assert e.value.code == po.PO_E_INVAL
        po.po_offload(st, 0, 0, 0.3)  # ceil(0.3 * 4) = 2 layers, lowest first
        po.po_synchronize(st)
        s = po.po_get_stats(st)
        assert s["n_offloads"] == 2 and s["bytes_d2h"] == 2 * layer_bytes
        with pytest.raises(po.PipeOffloadError) as e:
            po.po_stage_backward(st, 0, 0, r.dy[0], r.dx[0])  # two layers are on the host
        assert e.value.code == po.PO_E_STATE
        assert "reload" in po.po_last_error()
        with pytest.raises(po.PipeOffloadError) as e:
            po.po_offload(st, 0, 0, 0.5)  # those layers are not resident any more
        assert e.value.code == po.PO_E_STATE
        po.po_reload(st, 0, 0)
        po.po_reload(st, 0, 0)  # nothing left on the host: no-op
        po.po_stage_backward(st, 0, 0, r.dy[0], r.dx[0])
        po.po_synchronize(st)
        assert po.po_get_stats(st)["n_reloads"] == 2
        partial = (r.dx[0].clone(), r.grads.clone(), r.y[0].clone())
        r.zero_grads()
        po.po_stage_forward(st, 0, 0, r.x[0], r.y[0])
        po.po_stage_backward(st, 0, 0, r.dy[0], r.dx[0])
        po.po_synchronize(st)
        assert torch.equal(partial[0], r.dx[0]) and torch.equal(partial[1], r.grads) and torch.equal(partial[2], r.y[0])


def test_manual_calls_in_a_long_loop_keep_pools_and_results_stable(gpu_device):
    """The four stage calls driven by hand for many microbatches (two units in flight, every unit offloaded and
    reloaded, a po_synchronize now and then): the pools stop growing after the first units and a repeated input
    gives the same output and input gradient, bit for bit, every time."""
    shape = syn.StageShape(2, 1, 128, 2, 512, 64, dtype="bf16", pipeline_degree=2, n_microbatches=2)
    with StageRunner(shape) as r:
        r.make_inputs()
        st = r.stage
        first = {}
        grown = None
        po.po_stage_forward(st, 0, 0, r.x[0], r.y[0])
        po.po_offload(st, 0, 0, 1.0)
        for n in range(1, 61):
            cur, prev = n % 2, (n - 1) % 2
            po.po_stage_forward(st, n, 0, r.x[cur], r.y[cur])
            po.po_offload(st, n, 0, 1.0)
            po.po_reload(st, n - 1, 0)
            po.po_stage_backward(st, n - 1, 0, r.dy[prev], r.dx[prev])
            if n % 7 == 0:
                po.po_synchronize(st)
                s = po.po_get_stats(st)
                sizes = (s["pool_bytes_allocated"], s["host_bytes_allocated"])
                assert grown is None or sizes == grown
                grown = sizes
                snap = (r.y[prev].clone(), r.dx[prev].clone())
                if prev in first:
                    assert torch.equal(first[prev][0], snap[0]) and torch.equal(first[prev][1], snap[1])
                else:
                    first[prev] = snap
        po.po_reload(st, 60, 0)
        po.po_stage_backward(st, 60, 0, r.dy[0], r.dx[0])
        po.po_synchronize(st)
        assert len(first) == 2 and torch.isfinite(r.grads).all()
        assert po.po_get_stats(st)["n_offloads"] == 61 * 2


def test_pool_caps_give_oom_codes(gpu_device):
    shape = syn.StageShape(2, 1, 128, 2, 512, 64, dtype="f32", pipeline_degree=4, n_microbatches=4)
    layer_bytes = po.po_saved_bytes_per_layer(po.po_config_default(
        n_layers=2, hidden=128, n_heads=2, ffn=512, seq=64))
    with StageRunner(shape, device_pool_cap_bytes=3 * layer_bytes) as r:
        r.make_inputs()
        with pytest.raises(po.PipeOffloadError) as e:
            r.run(po.PO_SCHED_1F1B, 0.0)  # four units of two layers in flight do not fit three slabs
        assert e.value.code == po.PO_E_DEVICE_OOM
    with StageRunner(shape, host_pool_cap_bytes=1 * layer_bytes) as r:
        r.make_inputs()
        with pytest.raises(po.PipeOffloadError) as e:
            r.run(po.PO_SCHED_1F1B, 1.0)
        assert e.value.code == po.PO_E_HOST_OOM


def test_reset_after_a_failed_run_makes_the_stage_usable_again(gpu_device):
    """A run that stops at the device pool cap leaves units in flight; po_stage_reset drops them, and the same stage
    then gives, with two microbatches (which fit the cap), exactly what a fresh stage gives."""
    shape = syn.StageShape(2, 1, 128, 2, 512, 64, dtype="f32", pipeline_degree=4, n_microbatches=4)
    layer_bytes = po.po_saved_bytes_per_layer(po.po_config_default(
        n_layers=2, hidden=128, n_heads=2, ffn=512, seq=64))
    small = syn.StageShape(2, 1, 128, 2, 512, 64, dtype="f32", pipeline_degree=1, n_microbatches=2)
    with StageRunner(small, n_microbatches=2) as ref:
        ref.make_inputs()
        ref.run(po.PO_SCHED_1F1B, 0.0)
        want = _snapshot(ref)
    with StageRunner(shape, device_pool_cap_bytes=3 * layer_bytes) as r:
        r.make_inputs()
        with pytest.raises(po.PipeOffloadError):
            r.run(po.PO_SCHED_1F1B, 0.0)
        with pytest.raises(po.PipeOffloadError) as e:
            po.po_stage_forward(r.stage, 0, 0, r.x[0], r.y[0])  # still in flight from the failed run
        assert e.value.code == po.PO_E_STATE
        po.po_stage_reset(r.stage)
        r.zero_grads()
        for j in range(2):
            po.po_stage_forward(r.stage, j, 0, r.x[j], r.y[j])
            po.po_stage_backward(r.stage, j, 0, r.dy[j], r.dx[j])
        po.po_synchronize(r.stage)
        got = _snapshot(r)
        for a, b in zip(want[0] + want[1], got[0][:2] + got[1][:2]):
            assert torch.equal(a, b)
        assert torch.equal(want[2], got[2])
        po.po_stage_reset(r.stage)  # nothing in flight: a no-op


def test_peak_slab_bytes_follow_the_schedule_model(gpu_device):
    shape = syn.StageShape(1, 1, 128, 2, 512, 64, dtype="bf16", pipeline_degree=6, n_microbatches=12)
    layer_bytes = None
    peaks = {}
    for ratio in (0.0, 0.5, 1.0):
        with StageRunner(shape) as r:
            layer_bytes = po.po_saved_bytes_per_layer(r.cfg)
            r.make_inputs()
            stats = r.run(po.PO_SCHED_1F1B, ratio)
            ops = sch.with_offload(sch.one_f_one_b(6, 0, 12), sch.selected_units(12, 1, ratio), r.cfg.prefetch_passes)
            model = sch.simulate(ops)
            assert stats["peak_in_flight_units"] == model["peak_in_flight"] == 6
            assert stats["peak_resident_units"] == model["peak_resident"]
            assert stats["peak_slab_bytes"] == model["peak_resident"] * layer_bytes
            peaks[ratio] = stats["peak_slab_bytes"]
    assert peaks[1.0] < peaks[0.5] < peaks[0.0]


# ---- split backward (B / W passes) and the generalized interleaved schedule (Sections 3.1, 3.2) ----------------
@pytest.mark.parametrize("shape", [syn.StageShape(2, 1, 128, 2, 512, 96, vocab=50, dtype="f32", pipeline_degree=2,
                                                  n_microbatches=3),
                                   syn.StageShape(3, 1, 256, 2, 1024, 256, dtype="bf16", pipeline_degree=2,
                                                  n_microbatches=3)], ids=["f32-embedding", "bf16-mfma"])
def test_split_backward_is_bit_identical_to_the_fused_backward(gpu_device, shape):
    m = shape.n_microbatches
    with StageRunner(shape) as r:
        r.make_inputs()
        st = r.stage
        for j in range(m):
            po.po_stage_forward(st, j, 0, r.x[j], r.y[j])
        for j in range(m):
            po.po_stage_backward(st, j, 0, r.dy[j], r.dx[j])
        fused = _snapshot(r)
        _compare(shape, r.results(), _oracle(shape, r, m), 1e-4 if shape.dtype == "f32" else 2e-2)
        # B directly followed by W
        r.zero_grads()
        for j in range(m):
            po.po_stage_forward(st, j, 0, r.x[j], r.y[j])
        for j in range(m):
            po.po_stage_backward_input(st, j, 0, r.dy[j], r.dx[j])
            po.po_stage_backward_weight(st, j, 0)
        _assert_bit_identical(fused, _snapshot(r))
        # all B passes first, W passes delayed (several units weight-pending at once)
        r.zero_grads()
        for j in range(m):
            po.po_stage_forward(st, j, 0, r.x[j], r.y[j])
        for j in range(m):
            po.po_stage_backward_input(st, j, 0, r.dy[j], r.dx[j])
        for j in range(m):
            po.po_stage_backward_weight(st, j, 0)
        _assert_bit_identical(fused, _snapshot(r))


def test_split_backward_state_errors(gpu_device):
    shape = syn.StageShape(2, 1, 128, 2, 512, 64, dtype="f32", pipeline_degree=2, n_microbatches=2)
    with StageRunner(shape) as r:
        r.make_inputs()
        st = r.stage
        po.po_stage_forward(st, 0, 0, r.x[0], r.y[0])
        with pytest.raises(po.PipeOffloadError) as e:
            po.po_stage_backward_weight(st, 0, 0)  # no input-gradient pass yet
        assert e.value.code == po.PO_E_STATE
        with pytest.raises(po.PipeOffloadError) as e:
            po.po_stage_backward_weight(st, 1, 0)  # never forwarded
        assert e.value.code == po.PO_E_STATE
        po.po_stage_backward_input(st, 0, 0, r.dy[0], r.dx[0])
        for call in (lambda: po.po_stage_backward_input(st, 0, 0, r.dy[0], r.dx[0]),
                     lambda: po.po_stage_backward(st, 0, 0, r.dy[0], r.dx[0]),
                     lambda: po.po_offload(st, 0, 0, 1.0),
                     lambda: po.po_stage_forward(st, 0, 0, r.x[0], r.y[0])):
            with pytest.raises(po.PipeOffloadError) as e:
                call()
            assert e.value.code == po.PO_E_STATE
        po.po_stage_backward_weight(st, 0, 0)
        with pytest.raises(po.PipeOffloadError) as e:
            po.po_stage_backward_weight(st, 0, 0)  # the unit is gone
        assert e.value.code == po.PO_E_STATE
        po.po_synchronize(st)


@pytest.mark.parametrize("group", [0, 2])
def test_gis_schedule_against_oracle_and_schedule_model(gpu_device, group):
    d, v, m = 4, 2, 8
    shape = syn.StageShape(4, v, 128, 2, 512, 64, dtype="bf16", pipeline_degree=d, n_microbatches=m)
    results = {}
    for ratio in (0.0, 0.5, 1.0):
        with StageRunner(shape, group=group) as r:
            r.make_inputs()
            stats = r.run(po.PO_SCHED_GIS, ratio)
            results[ratio] = _snapshot(r)
            ops = sch.with_offload(sch.generalized_interleaved(d, 0, v, m, group or None),
                                   sch.selected_units(m, v, ratio), r.cfg.prefetch_passes)
            model = sch.simulate(ops)
            assert model["errors"] == []
            assert stats["peak_in_flight_units"] == model["peak_in_flight"] == (group or d) * (v - 1) + d
            assert stats["peak_resident_units"] == model["peak_resident"]
            assert stats["n_compute_passes"] == 3 * m * v
            if ratio == 0.0:
                _compare(shape, r.results(), _oracle(shape, r, m), 2e-2)
    for ratio in (0.5, 1.0):
        _assert_bit_identical(results[0.0], results[ratio])
    with StageRunner(shape, group=group, weight_stream=1, debug_poison=1) as r:  # W passes on their own stream
        r.make_inputs()
        r.run(po.PO_SCHED_GIS, 1.0)
        _assert_bit_identical(results[0.0], _snapshot(r))
    # every chunk sees its microbatches in ascending order in all these schedules, so the interleaved 1F1B run
    # accumulates the same sums in the same order
    with StageRunner(shape) as r:
        r.make_inputs()
        r.run(po.PO_SCHED_1F1B_INTERLEAVED, 0.0)
        _assert_bit_identical(results[0.0], _snapshot(r))


@pytest.mark.parametrize("rank,m", [(0, 8), (0, 7), (3, 6)])
def test_uniform_repeat_schedule_against_oracle_and_schedule_model(gpu_device, rank, m):
    """The uniformly repeated schedule (Section 2; PO of Table 1) with stage-level selection: ratio 0.5 offloads
    chunk 0 of every microbatch (PO-H), ratio 1 both chunks (PO-F); any number of microbatches."""
    d, v = 4, 2
    shape = syn.StageShape(4, v, 128, 2, 512, 64, dtype="bf16", pipeline_degree=d, rank=rank, n_microbatches=m)
    results = {}
    for ratio in (0.0, 0.5, 1.0):
        with StageRunner(shape, select_policy=po.PO_SEL_LONGEST_LIFESPAN) as r:
            r.make_inputs()
            stats = r.run(po.PO_SCHED_PO, ratio)
            results[ratio] = _snapshot(r)
            passes = sch.uniform_repeat(d, rank, v, m)
            ops = sch.with_offload(passes, sch.selected_units(m, v, ratio, "longest-lifespan"), r.cfg.prefetch_passes)
            model = sch.simulate(ops)
            assert model["errors"] == []
            assert stats["peak_in_flight_units"] == model["peak_in_flight"]
            assert stats["peak_resident_units"] == model["peak_resident"]
            assert stats["n_compute_passes"] == 3 * m * v
            assert stats["n_offloads"] == stats["n_reloads"] == int(ratio * v) * m * shape.layers_per_chunk  # per layer slab
            if ratio == 0.0:
                _compare(shape, r.results(), _oracle(shape, r, m), 2e-2)
    for ratio in (0.5, 1.0):
        _assert_bit_identical(results[0.0], results[ratio])
    # each chunk still sees its microbatches in ascending order: same sums, same order as the fused interleaved run
    if m % d == 0:
        with StageRunner(shape) as r:
            r.make_inputs()
            r.run(po.PO_SCHED_1F1B_INTERLEAVED, 0.0)
            _assert_bit_identical(results[0.0], _snapshot(r))


@pytest.mark.parametrize("k,copy_streams", [(1.0, 1), (0.5, 1), (1.5, 2)])
def test_slot_placed_copies_on_the_uniformly_repeated_schedule(gpu_device, k, copy_streams):
    """Section 4.2's slot plan (one-offload-one-reload slots of a shared copy stream) drives the stage: same
    results as the resident run, and as many units move, and as many stay resident, as the schedule model says."""
    import numpy as np
    d, v, m = 4, 2, 8
    shape = syn.StageShape(4, v, 128, 2, 512, 64, dtype="bf16", pipeline_degree=d, n_microbatches=m)
    with StageRunner(shape) as r:
        r.make_inputs()
        r.run(po.PO_SCHED_PO, 0.0)
        base = _snapshot(r)
    kf = float(np.float32(k))  # the config holds k in single precision
    for ratio in (0.5, 1.0):
        with StageRunner(shape, slot_k=k, copy_streams=copy_streams, debug_poison=1) as r:
            r.make_inputs()
            stats = r.run(po.PO_SCHED_PO, ratio)
            _assert_bit_identical(base, _snapshot(r))
            timed = sch.uniform_repeat_times(d, 0, v, m)
            placement = sch.slot_placement(timed, set(range(int(ratio * v))), kf)
            model = sch.simulate(sch.with_slot_offload(timed, placement, kf))
            assert model["errors"] == []
            assert stats["n_offloads"] == stats["n_reloads"] == len(placement) * shape.layers_per_chunk
            assert stats["peak_resident_units"] == model["peak_resident"]
            assert len(placement) > 0 or k * ratio * v > v  # more copy time asked for than a period holds


def test_short_gap_units_are_not_offloaded(gpu_device):
    # last rank of 1F1B: every backward directly follows its forward; with min_gap_passes = 1 nothing moves
    shape = syn.StageShape(2, 1, 128, 2, 512, 64, dtype="bf16", pipeline_degree=4, rank=3, n_microbatches=6)
    snaps = {}
    for min_gap in (0, 1):
        with StageRunner(shape, min_gap_passes=min_gap) as r:
            r.make_inputs()
            stats = r.run(po.PO_SCHED_1F1B, 1.0)
            snaps[min_gap] = _snapshot(r)
            assert stats["n_offloads"] == (12 if min_gap == 0 else 0)
            assert stats["peak_resident_units"] == 1
    _assert_bit_identical(snaps[0], snaps[1])


# ---- grouped-query attention in the stage (Table 2's query groups) ---------------------------------------------
@pytest.mark.parametrize("shape,tol", [
    (syn.StageShape(2, 1, 128, 4, 512, 96, vocab=40, dtype="f32", pipeline_degree=2, n_microbatches=3, n_kv_heads=2), 1e-4),
    (syn.StageShape(2, 1, 512, 4, 1024, 256, dtype="bf16", pipeline_degree=3, n_microbatches=4, n_kv_heads=1), 2e-2),
    (syn.StageShape(2, 1, 256, 4, 1024, 384, dtype="bf16", pipeline_degree=2, n_microbatches=3, n_kv_heads=2), 2e-2)],
    ids=["f32-generic", "bf16-mfma-dh128", "bf16-mfma-dh64"])
def test_stage_with_grouped_query_attention(gpu_device, shape, tol):
    m = shape.n_microbatches
    snaps = {}
    for ratio in (0.0, 1.0):
        with StageRunner(shape) as r:
            if shape.ffn == 4 * shape.hidden:  # the slab is the saved set plus at most six 256-byte alignment gaps
                model = sch.saved_bytes_per_layer(shape.seq, shape.hidden, shape.n_heads,
                                                  4 if shape.dtype == "f32" else 2, shape.n_kv_heads)
                assert 0 <= po.po_saved_bytes_per_layer(r.cfg) - model < 6 * 256
            r.make_inputs()
            stats = r.run(po.PO_SCHED_1F1B, ratio)
            snaps[ratio] = _snapshot(r)
            if ratio == 0.0:
                _compare(shape, r.results(), _oracle(shape, r, m), tol)
            else:
                assert stats["bytes_d2h"] == m * shape.n_layers * po.po_saved_bytes_per_layer(r.cfg)
    _assert_bit_identical(snaps[0.0], snaps[1.0])


# ---- dropout with regenerated masks (Appendix C) ---------------------------------------------------------------
@pytest.mark.parametrize("shape,tol", [
    (syn.StageShape(2, 1, 128, 2, 512, 96, vocab=40, dtype="f32", pipeline_degree=2, n_microbatches=3), 1e-4),
    (syn.StageShape(2, 1, 256, 2, 1024, 256, dtype="bf16", pipeline_degree=3, n_microbatches=4), 2e-2),
    (syn.StageShape(1, 1, 192, 3, 320, 200, dtype="bf16", pipeline_degree=2, n_microbatches=2), 2e-2)],
    ids=["f32-generic", "bf16-mfma", "bf16-ragged"])
def test_stage_with_dropout_against_oracle_and_bitwise_invariants(gpu_device, shape, tol):
    m, p, seed = shape.n_microbatches, float(np.float32(0.2)), 4242  # the library holds p in fp32
    x = {(j, 0): syn.unit_input(shape, j, 0) for j in range(m)}
    dy = {(j, 0): syn.unit_upstream_grad(shape, j, 0) for j in range(m)}
    snaps = {}
    for name, kw, ratio in [("plain", {}, 0.0), ("offload", {}, 1.0), ("weight-stream", dict(weight_stream=1), 1.0)]:
        with StageRunner(shape, dropout_p=p, dropout_seed=seed, **kw) as r:
            r.make_inputs()
            r.run(po.PO_SCHED_1F1B, ratio)
            snaps[name] = _snapshot(r)
            if name == "plain":
                ref = so.run_stage(r.params_np, shape.n_layers, 1, shape.n_heads, x, dy, vocab=shape.vocab,
                                   dropout_p=p, seed=seed)
                _compare(shape, r.results(), ref, tol)
                # without the masks the oracle is far away: the parity above really exercises them
                nodrop = so.run_stage(r.params_np, shape.n_layers, 1, shape.n_heads, x, dy, vocab=shape.vocab)
                got_y = r.results()[0][(0, 0)]
                assert max_rel_err(got_y, nodrop[0][(0, 0)]) > 5 * max_rel_err(got_y, ref[0][(0, 0)])
                # split backward regenerates the same masks
                r.zero_grads()
                for j in range(m):
                    po.po_stage_forward(r.stage, j, 0, r.x[j], r.y[j])
                for j in range(m):
                    po.po_stage_backward_input(r.stage, j, 0, r.dy[j], r.dx[j])
                    po.po_stage_backward_weight(r.stage, j, 0)
                _assert_bit_identical(snaps["plain"], _snapshot(r))
                # another seed, other masks
                with pytest.raises(po.PipeOffloadError):
                    po.po_stage_forward(r.stage, 0, 0, r.x[0], r.y[0])
                    po.po_set_dropout_seed(r.stage, 1)  # a unit is in flight
                po.po_stage_backward(r.stage, 0, 0, r.dy[0], r.dx[0])
                po.po_set_dropout_seed(r.stage, seed + 1)
                r.zero_grads()
                r.run(po.PO_SCHED_1F1B, 0.0)
                assert not torch.equal(snaps["plain"][2], r.grads)
    _assert_bit_identical(snaps["plain"], snaps["offload"])
    _assert_bit_identical(snaps["plain"], snaps["weight-stream"])


def test_features_together_across_schedules_and_offload_policies(gpu_device):
    """Grouped key/value heads, hidden dropout, an embedding chunk and two chunks per rank at once: the oracle's
    result within the bf16 tolerance, and the same bits under interleaved 1F1B with full offload, the split-backward
    schedule with alternate microbatches offloaded, the uniformly repeated schedule with the longest-lived chunk
    offloaded (prefetch rule and slot plan), on one copy stream and on two."""
    shape = syn.StageShape(4, 2, 256, 4, 1024, 256, vocab=60, dtype="bf16", pipeline_degree=3, n_microbatches=6,
                           n_kv_heads=2)
    p, seed, m = float(np.float32(0.1)), 99, 6
    x = {(j, c): syn.unit_input(shape, j, c) for j in range(m) for c in range(2)}
    dy = {(j, c): syn.unit_upstream_grad(shape, j, c) for j in range(m) for c in range(2)}
    runs = [
        ("interleaved, resident", po.PO_SCHED_1F1B_INTERLEAVED, 0.0, {}),
        ("interleaved, full offload", po.PO_SCHED_1F1B_INTERLEAVED, 1.0, {}),
        ("interleaved, full offload, one stream, staged", po.PO_SCHED_1F1B_INTERLEAVED, 1.0,
         dict(copy_streams=1, staged_copies=1)),
        ("split backward, alternate microbatches", po.PO_SCHED_GIS, 0.5, dict(group=2)),
        ("uniform repeat, chunk 0 offloaded", po.PO_SCHED_PO, 0.5,
         dict(select_policy=po.PO_SEL_LONGEST_LIFESPAN, prefetch_passes=3)),
        ("uniform repeat, slot plan", po.PO_SCHED_PO, 0.5, dict(slot_k=1.0, copy_streams=1)),
        ("uniform repeat, weight stream", po.PO_SCHED_PO, 1.0,
         dict(select_policy=po.PO_SEL_LONGEST_LIFESPAN, weight_stream=1)),
    ]
    base = None
    for name, sched, ratio, kw in runs:
        with StageRunner(shape, dropout_p=p, dropout_seed=seed, **kw) as r:
            r.make_inputs()
            stats = r.run(sched, ratio)
            snap = _snapshot(r)
            assert (stats["n_offloads"] > 0) == (ratio > 0.0), name
            if base is None:
                base = snap
                ref = so.run_stage(r.params_np, shape.n_layers, 2, shape.n_heads, x, dy, vocab=shape.vocab,
                                   dropout_p=p, seed=seed)
                _compare(shape, r.results(), ref, 2e-2)
            else:
                for a, b in zip(base[0] + [base[2]], snap[0] + [snap[2]]):
                    assert torch.equal(a, b), name
                for a, b in zip(base[1], snap[1]):
                    assert (a is None and b is None) or torch.equal(a, b), name


@pytest.mark.parametrize("shape,tol", [
    (syn.StageShape(1, 1, 64, 1, 64, 1, dtype="f32", pipeline_degree=1, n_microbatches=1), 1e-4),
    (syn.StageShape(2, 2, 64, 2, 64, 3, vocab=5, dtype="f32", pipeline_degree=1, n_microbatches=2), 1e-4),
    (syn.StageShape(1, 1, 64, 1, 64, 1, dtype="bf16", pipeline_degree=1, n_microbatches=1), 2e-2),
    (syn.StageShape(3, 1, 128, 2, 64, 2, dtype="bf16", pipeline_degree=5, n_microbatches=2), 2e-2)],
    ids=["one-token-f32", "three-tokens-two-chunks-embedding", "one-token-bf16", "more-ranks-than-microbatches"])
def test_degenerate_stage_shapes(gpu_device, shape, tol):
    """The smallest stages the configuration allows (one token, one head, the narrowest widths, one microbatch, a
    pipeline degree above the microbatch count) with everything offloaded: oracle parity and the same bits as the
    resident run."""
    m, v = shape.n_microbatches, shape.n_chunks
    sched = po.PO_SCHED_1F1B_INTERLEAVED if v > 1 else po.PO_SCHED_1F1B
    snaps = []
    for ratio in (1.0, 0.0):
        with StageRunner(shape) as r:
            r.make_inputs()
            stats = r.run(sched, ratio)
            snaps.append(_snapshot(r))
            if ratio == 1.0:
                assert stats["n_offloads"] == m * shape.n_layers and stats["n_reloads"] == m * shape.n_layers
                _compare(shape, r.results(), _oracle(shape, r, m), tol)
    _assert_bit_identical(snaps[0], snaps[1])
