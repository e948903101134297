"""Host-only checks of the C ABI: the library loads, exports every declared
symbol, and its pure-host entry points (schedule, parameter layout, Eq. 1, config
validation) agree with the independent oracle models.  No GPU work is issued."""
import os
import re

import pytest

from oracle import schedule_oracle as sch
from paper_2503_01328_amd import binding as po
from paper_2503_01328_amd import inputs as syn
from paper_2503_01328_amd import harness

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported_and_bound():
    header = open(os.path.join(ROOT, "include", "pipeoffload.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(po_[a-z0-9_]+)\s*\(", header))
    assert len(declared) >= 25
    for name in declared:
        assert hasattr(po.lib, name), f"{name} declared in the header but not exported"
        assert name in po.EXPORTS, f"{name} has no binding"
        assert hasattr(po, name), f"binding lacks a Python function {name}"
    assert set(po.EXPORTS) == declared


SCHEDS = {"1f1b": po.PO_SCHED_1F1B, "1f1b-interleaved": po.PO_SCHED_1F1B_INTERLEAVED}


@pytest.mark.parametrize("name,d,v,m", [("1f1b", 2, 1, 4), ("1f1b", 4, 1, 8), ("1f1b", 8, 1, 16), ("1f1b", 16, 1, 16),
                                        ("1f1b", 4, 1, 3), ("1f1b-interleaved", 8, 2, 32),
                                        ("1f1b-interleaved", 4, 3, 8), ("1f1b-interleaved", 2, 2, 2)])
@pytest.mark.parametrize("ratio", [0.0, 0.25, 0.5, 1.0])
@pytest.mark.parametrize("prefetch", [0, 1, 3])
def test_schedule_ops_match_the_oracle_model(name, d, v, m, ratio, prefetch):
    for rank in sorted({0, d // 2, d - 1}):
        for policy, pname in ((po.PO_SEL_ALTERNATE_MB, "alternate-mb"), (po.PO_SEL_LONGEST_LIFESPAN, "longest-lifespan")):
            got = po.po_schedule_ops(SCHEDS[name], d, rank, v, m, ratio, policy, prefetch)
            passes = sch.compute_passes(name, d, rank, v, m)
            want = sch.with_offload(passes, sch.selected_units(m, v, ratio, pname), prefetch)
            assert got == want
            assert sch.simulate(got)["errors"] == []


@pytest.mark.parametrize("d,v,m,g", [(8, 2, 32, 8), (8, 2, 32, 4), (4, 3, 12, 2), (4, 3, 12, 3), (4, 2, 8, 0), (6, 2, 12, 3),
                                     (2, 1, 4, 1)])
@pytest.mark.parametrize("ratio", [0.0, 0.5, 1.0])
@pytest.mark.parametrize("prefetch", [0, 2, 3])
def test_gis_schedule_ops_match_the_oracle_model(d, v, m, g, ratio, prefetch):
    for rank in sorted({0, d // 2, d - 1}):
        for policy, pname in ((po.PO_SEL_ALTERNATE_MB, "alternate-mb"), (po.PO_SEL_LONGEST_LIFESPAN, "longest-lifespan")):
            got = po.po_schedule_ops(po.PO_SCHED_GIS, d, rank, v, m, ratio, policy, prefetch, group=g)
            passes = sch.compute_passes("gis", d, rank, v, m, g or None)
            want = sch.with_offload(passes, sch.selected_units(m, v, ratio, pname), prefetch)
            assert got == want
            assert sch.simulate(got)["errors"] == []


@pytest.mark.parametrize("name,d,v,m", [("1f1b", 8, 1, 16), ("1f1b-interleaved", 8, 2, 32), ("gis", 8, 2, 32)])
@pytest.mark.parametrize("min_gap", [1, 3, 9])
def test_short_gap_units_are_skipped_like_in_the_oracle_model(name, d, v, m, min_gap):
    code = {"gis": po.PO_SCHED_GIS, **SCHEDS}[name]
    for rank in range(d):
        for ratio in (0.5, 1.0):
            got = po.po_schedule_ops(code, d, rank, v, m, ratio, 0, 2, min_gap=min_gap)
            want = sch.with_offload(sch.compute_passes(name, d, rank, v, m), sch.selected_units(m, v, ratio), 2, min_gap)
            assert got == want


@pytest.mark.parametrize("d,v,m,g", [(8, 2, 32, 0), (8, 2, 11, 4), (8, 4, 16, 6), (4, 3, 7, 2), (4, 4, 16, 4), (6, 3, 18, 0),
                                     (5, 2, 9, 0), (2, 2, 5, 1), (4, 1, 8, 0), (8, 16, 24, 0), (16, 2, 16, 0)])
@pytest.mark.parametrize("ratio", [0.0, 0.5, 1.0])
def test_uniform_repeat_schedule_ops_match_the_oracle_model(d, v, m, g, ratio):
    for rank in sorted({0, d // 2, d - 1}):
        for policy, pname in ((po.PO_SEL_ALTERNATE_MB, "alternate-mb"), (po.PO_SEL_LONGEST_LIFESPAN, "longest-lifespan")):
            for prefetch in (0, 2):
                got = po.po_schedule_ops(po.PO_SCHED_PO, d, rank, v, m, ratio, policy, prefetch, group=g)
                passes = sch.compute_passes("po", d, rank, v, m, g or None)
                want = sch.with_offload(passes, sch.selected_units(m, v, ratio, pname), prefetch)
                assert got == want
                assert sch.simulate(got)["errors"] == []


@pytest.mark.parametrize("d,v,m,g", [(8, 2, 16, 0), (4, 2, 9, 0), (8, 4, 12, 6), (6, 3, 10, 0), (4, 1, 8, 0), (2, 2, 5, 1)])
@pytest.mark.parametrize("k", [0.25, 0.5, 0.9, 1.0, 1.7, 3.0, 40.0])
def test_slot_schedule_ops_match_the_oracle_model(d, v, m, g, k):
    for rank in sorted({0, d // 2, d - 1}):
        for n_sel in range(v + 1):
            got = po.po_schedule_ops_slots(d, rank, v, m, n_sel, k, group=g)
            timed = sch.uniform_repeat_times(d, rank, v, m, g or None)
            placement = sch.slot_placement(timed, set(range(n_sel)), k)
            assert got == sch.with_slot_offload(timed, placement, k)
            assert sch.simulate(got)["errors"] == []


def test_slot_schedule_rejects_bad_arguments():
    for args in [(4, 0, 2, 8, 3, 1.0), (4, 0, 2, 8, 1, 0.0), (4, 0, 2, 8, 1, -1.0), (4, 4, 2, 8, 1, 1.0), (4, 0, 2, 0, 1, 1.0)]:
        with pytest.raises(po.PipeOffloadError) as e:
            po.po_schedule_ops_slots(*args)
        assert e.value.code == po.PO_E_INVAL
    with pytest.raises(po.PipeOffloadError):
        po.po_schedule_ops_slots(8, 0, 2, 8, 1, 1.0, group=3)


def test_uniform_repeat_rejects_bad_groups():
    for g in (3, 9):
        with pytest.raises(po.PipeOffloadError) as e:
            po.po_schedule_ops(po.PO_SCHED_PO, 8, 0, 2, 32, 0.5, group=g)
        assert e.value.code == po.PO_E_INVAL


def test_gis_schedule_rejects_bad_groups():
    for g, m in [(3, 32), (9, 32), (8, 30)]:
        with pytest.raises(po.PipeOffloadError) as e:
            po.po_schedule_ops(po.PO_SCHED_GIS, 8, 0, 2, m, 0.5, group=g)
        assert e.value.code == po.PO_E_INVAL


def test_schedule_ops_reject_bad_arguments():
    for args in [(0, 4, 4, 1, 8, 0.5), (0, 4, 0, 2, 8, 0.5), (1, 4, 0, 2, 6, 0.5), (0, 4, 0, 1, 8, 1.5), (7, 4, 0, 1, 8, 0.5)]:
        with pytest.raises(po.PipeOffloadError) as e:
            po.po_schedule_ops(*args)
        assert e.value.code == po.PO_E_INVAL
        assert "schedule" in po.po_last_error()


def test_grouped_query_layout_and_saved_bytes():
    shape = syn.StageShape(2, 1, 4096, 32, 16384, 4096, dtype="bf16", n_kv_heads=8)
    cfg = harness.make_config(shape)
    layout = {(d["layer"], d["name"]): d for d in po.po_param_layout(cfg)}
    assert (layout[(0, "w_qkv")]["rows"], layout[(0, "w_qkv")]["cols"]) == (4096, 4096 + 2 * 8 * 128)
    assert layout[(1, "b_qkv")]["cols"] == 6144
    assert po.po_param_count(cfg) == 2 * (4096 * 6144 + 6144 + 4096 * 4096 + 2 * 4096 * 16384 + 4096 * 5 + 16384 + 4096)
    model = sch.saved_bytes_per_layer(4096, 4096, 32, 2, 8)
    assert model == (8 * 4096 + 2 * 1024) * 4096 * 2 + 4 * 32 * 4096  # k and v a quarter of the multi-head size
    assert 0 <= po.po_saved_bytes_per_layer(cfg) - model < 6 * 256
    with pytest.raises(po.PipeOffloadError):
        po.po_param_count(harness.make_config(syn.StageShape(2, 1, 4096, 32, 16384, 4096, n_kv_heads=5)))


def test_offload_ratio_for_k():
    assert po.po_offload_ratio_for_k(0.5) == 1.0 and po.po_offload_ratio_for_k(1.0) == 1.0
    assert po.po_offload_ratio_for_k(2.0) == 0.5 and abs(po.po_offload_ratio_for_k(1.6) - 0.625) < 1e-12
    assert po.po_offload_ratio_for_k(0.0) == 1.0 and po.po_offload_ratio_for_k(-1.0) == 1.0


def test_offload_k_is_eq1():
    for h, s in [(8192, 4096), (4096, 4096), (5120, 16384), (2048, 2048)]:
        assert abs(po.po_offload_k(h, s, 220e12, 15e9) - sch.offload_ratio_k(h, s, 220e12, 15e9)) < 1e-12
    assert abs(po.po_offload_k(8192, 4096, 220e12, 15e9) - 0.918) < 1e-3


@pytest.mark.parametrize("key", ["C1", "C2", "C3", "C5"])
def test_param_layout_and_saved_bytes(key):
    shape = syn.CONFIGS[key]
    cfg = harness.make_config(shape)
    layout = po.po_param_layout(cfg)
    h, f = shape.hidden, shape.ffn
    per_layer = 12 * h * h + 13 * h if f == 4 * h else None
    total = po.po_param_count(cfg)
    emb = (shape.vocab + shape.seq) * h if shape.vocab else 0
    assert total == emb + shape.n_layers * per_layer
    # tensors tile the buffer without gaps, in the documented order, 16-byte aligned for bf16
    off = 0
    for d in layout:
        assert d["offset"] == off and d["offset"] % 8 == 0
        off += d["rows"] * d["cols"]
    assert off == total
    names = [d["name"] for d in layout if d["layer"] == 0]
    assert names == [n for n, _ in syn.LAYER_PARAMS]
    # Appendix C: 20 s h bytes per layer at two bytes per element (+ fp32 log-sum-exp, + alignment)
    E = 2 if shape.dtype == "bf16" else 4
    want = sch.saved_bytes_per_layer(shape.seq, h, shape.n_heads, E)
    got = po.po_saved_bytes_per_layer(cfg)
    assert want <= got < want + 6 * 256


def test_invalid_configs_are_rejected_without_touching_the_gpu():
    good = harness.make_config(syn.CONFIGS["C1"])
    assert po.po_param_count(good) > 0
    for field, value in [("n_layers", 0), ("n_chunks", 3), ("hidden", 100), ("n_heads", 7), ("seq", 0),
                         ("dtype", 5), ("rank", 2), ("copy_streams", 3), ("ln_eps", 0.0), ("slot_k", -1.0), ("dropout_p", 1.0),
                         ("group", 5), ("min_gap_passes", -1), ("n_kv_heads", 3), ("weight_stream", 2)]:
        cfg = harness.make_config(syn.CONFIGS["C1"])
        setattr(cfg, field, value)
        with pytest.raises(po.PipeOffloadError) as e:
            po.po_param_count(cfg)
        assert e.value.code == po.PO_E_INVAL


def test_flatten_unflatten_roundtrip():
    shape = syn.StageShape(2, 1, 64, 2, 256, 8, vocab=16, dtype="f32")
    cfg = harness.make_config(shape)
    params = syn.stage_params(shape, 3)
    flat = harness.flatten_params(cfg, params)
    back = harness.unflatten(cfg, flat)
    for l in range(2):
        for k, a in params["layers"][l].items():
            assert (back["layers"][l][k] == a).all()
    assert (back["wte"] == params["wte"]).all() and (back["wpe"] == params["wpe"]).all()


def test_gemm_tile_choice_fills_the_chip():
    """Host logic of the bf16 GEMM: which output tile a shape gets.  The GEMM shapes of the five workloads, the
    grouped-query QKV projection, and shapes that fit no tile."""
    tile = po.po_op_gemm_tile
    # C2 (tokens 2048, h 2048, f 8192): 2048 x 2048 results have only 64 big tiles -> 128 x 128;
    # the QKV projection's 192 big tiles would leave 64 compute units idle -> 256 of the 256 x 192 tiles
    assert tile(2048, 2048) == (128, 128)
    assert tile(2048, 8192) == (256, 256) and tile(8192, 2048) == (256, 256)
    assert tile(2048, 6144) == (256, 192)
    # C3 / C5: whole rounds of big tiles
    assert tile(4096, 4096) == (256, 256) and tile(4096, 12288) == (256, 256) and tile(4096, 16384) == (256, 256)
    assert tile(16384, 15360) == (256, 256) and tile(16384, 5120) == (256, 256) and tile(5120, 15360) == (256, 256)
    # C3 with 8 key/value heads: 384 big tiles need two rounds, 512 narrower ones too, at 3/4 of the work each
    assert tile(4096, 6144) == (256, 192)
    # too few tiles for the big shapes; no 192-wide tile when the row count is no multiple of 256
    assert tile(256, 384) == (128, 128) and tile(128, 6144) == (128, 128) and tile(384, 128) == (128, 128)
    # nothing fits: the shape-generic kernel runs
    assert tile(200, 130) == (0, 0) and tile(64, 64) == (0, 0) and tile(0, 128) == (0, 0)
    for M in range(128, 4097, 128):
        for N in range(64, 6145, 64):
            bm, bn = tile(M, N)
            assert (bm, bn) in ((0, 0), (128, 128), (256, 192), (256, 256))
            assert bm == 0 or (M % bm == 0 and N % bn == 0)


def test_hot_kernels_keep_their_accumulators_in_registers():
    """The compiler's own resource report (written by the build): no MFMA kernel may use scratch memory - a GEMM
    whose 256 accumulators spill runs six times slower without failing any numerical test - and the attention
    kernels must still fit two waves per SIMD."""
    import json

    from paper_2503_01328_amd import build as b

    if not os.path.exists(b.RESOURCES):
        b.build(verbose=False)
    usage = json.load(open(b.RESOURCES))
    gemm = {k: v for k, v in usage.items() if "gemm_mfma_kernel" in k}
    grouped = {k: v for k, v in usage.items() if "gemm_mfma_grouped_kernel" in k}
    assert len(grouped) == 1
    attn = {k: v for k, v in usage.items() if "attn_" in k and "_mfma_kernel" in k and "delta" not in k}
    # GEMM: three tiles x four operand layouts x four epilogues; attention: the forward kernel in its two block
    # shapes, the two backward kernels, their eight-wave forms and the one-launch form of both, two head dimensions
    assert len(gemm) == 48 and len(attn) >= 16
    for name, v in {**gemm, **grouped, **attn}.items():
        assert v["ScratchSize"] == 0, (name, v)
    for name, v in attn.items():
        assert v["Occupancy"] >= 2, (name, v)
    for name, v in gemm.items():
        assert v["VGPRs"] + v["AGPRs"] <= 512


def test_trace_viewer_reads_the_span_file(tmp_path):
    """The span file format of PIPEOFFLOAD_TRACE ("# run" separators, "kind start_ms stop_ms" lines) and the viewer."""
    from paper_2503_01328_amd import trace

    f = tmp_path / "t.txt"
    f.write_text("# run\n0 0.0 1.0\n1 1.0 2.5\n# run\n0 0.0 2.0\n0 2.5 3.0\n2 1.0 4.0\n")
    runs = trace.read_runs(str(f))
    assert [len(r) for r in runs] == [2, 3]
    text = trace.render(runs[-1])
    assert "run of 4.00 ms, 3 spans" in text and "compute: 2 spans, busy 2.50 ms" in text
    assert "H2D: 1 spans, busy 3.00 ms" in text and "gap  0.50" in text
    assert trace.main(["trace", str(f), "0"]) == 0 and trace.main(["trace"]) == 2
