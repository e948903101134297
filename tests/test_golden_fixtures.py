"""The oracle against the values under tests/golden/: closed forms the paper states, evaluated by hand, and the
published known-answer vectors of the random generator the dropout masks use.  Every fixture line carries its
citation; nothing in those files was produced by this repository's code."""
import os

import pytest

from oracle import schedule_oracle as sch
from oracle import stage_oracle as so

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _rows(name):
    out = []
    for line in open(os.path.join(GOLDEN, name)):
        line = line.split("|")[0].strip()
        if line and not line.startswith("#"):
            out.append(line.split())
    return out


def _bubble(rank_ops, d, v, m):
    makespan, finished = sch.pipeline_timeline(rank_ops, d, v, 1.0, 1.0, 1.0)
    assert finished
    return makespan - 3.0 * m * v


@pytest.mark.parametrize("row", _rows("schedule_closed_forms.txt"), ids=lambda r: "-".join(r[:5]))
def test_schedule_closed_forms(row):
    what, (d, v, rank, g), expected, tol = row[0], map(int, row[1:5]), float(row[5]), float(row[6])
    m = 4 * d * (g if g and (4 * d) % g else 1)  # a multiple of d and of g
    if what == "interleaved_forwards_before_first_backward":
        got = sch.simulate(sch.interleaved_one_f_one_b(d, rank, v, m))["forwards_before_first_backward"]
    elif what == "gis_forwards_before_first_backward":
        got = sch.simulate(sch.generalized_interleaved(d, rank, v, m, g))["forwards_before_first_backward"]
    elif what == "interleaved_peak_units":
        got = sch.simulate(sch.interleaved_one_f_one_b(d, rank, v, m))["peak_in_flight"]
    elif what == "gis_peak_units":
        got = sch.simulate(sch.generalized_interleaved(d, rank, v, m, g))["peak_in_flight"]
    elif what == "bubble_1f1b":  # the v stages of a device merged into one pass
        makespan, finished = sch.pipeline_timeline([sch.one_f_one_b(d, i, m) for i in range(d)], d, 1, v, v, v)
        assert finished
        got = makespan - 3.0 * m * v
    elif what == "bubble_interleaved":
        got = _bubble([sch.interleaved_one_f_one_b(d, i, v, m) for i in range(d)], d, v, m)
    elif what == "bubble_gis":
        got = _bubble([sch.generalized_interleaved(d, i, v, m, g) for i in range(d)], d, v, m)
    elif what == "po_half_offloaded_peak_units":
        got = sch.peak_units(sch.uniform_repeat(d, rank, v, m, g), set(range(v // 2)))
    elif what == "po_half_offloaded_fraction_of_own_peak_x100":
        ops = sch.uniform_repeat(d, rank, v, m, g)
        got = 100.0 * sch.peak_units(ops, set(range(v // 2))) / sch.peak_units(ops)
    elif what == "po_bubble_below":
        assert _bubble([sch.uniform_repeat(d, i, v, m, g) for i in range(d)], d, v, m) < expected
        return
    else:
        raise AssertionError(f"unknown quantity {what}")
    assert abs(got - expected) <= tol, (what, got, expected)


def test_eq1_values():
    for h, s, k in _rows("eq1_k_values.txt"):
        assert abs(sch.offload_ratio_k(int(h), int(s), 220e12, 15e9) - float(k)) < 1e-3


def test_saved_bytes():
    for s, h, nbytes in _rows("saved_bytes.txt"):
        s, h = int(s), int(h)
        a = h // 128
        assert sch.saved_bytes_per_layer(s, h, a, 2) - 4 * a * s == int(nbytes)  # the log-sum-exp is this build's extra


def test_philox_known_answers():
    for row in _rows("philox4x32_10_kat.txt"):
        w = [int(x, 16) for x in row]
        assert tuple(int(x) for x in so.philox4x32_10(tuple(w[0:4]), tuple(w[4:6]))) == tuple(w[6:10])


def test_dropout_threshold_and_keep_direction():
    """Hand values of the keep threshold (rounding mode and clamp included) and hand-derived masks on the words of
    the generator's first known-answer vector: a flipped comparison, a wrong rounding or a shifted counter word
    fails one of them."""
    for row in _rows("dropout_threshold.txt"):
        if row[0] == "threshold":
            num, k, want = int(row[1]), int(row[2]), int(row[3])
            assert so.dropout_threshold(num / 2.0 ** k) == want, row
        elif row[0] == "decimal":
            assert so.dropout_threshold(float(row[1])) == int(row[2]), row
        elif row[0] == "mask":
            got = so.dropout_keep_mask(0, 0, 0, 0, 1, 4, float(row[1]))[0]
            assert [int(x) for x in got] == [int(x) for x in row[2:6]], row
        else:
            raise AssertionError(row)


def test_uniform_repeat_block_worked_by_hand():
    """d = 2, v = 2, g = 2: the start time of every pass of the building block as derived by hand in the fixture."""
    block = sch.building_block(2, 2, 2)
    rows = _rows("po_block_d2_v2_g2.txt")
    assert len(rows) == len(block) == 12
    for kind, rank, chunk, start in rows:
        assert block[(kind, int(rank), int(chunk))] == int(start), (kind, rank, chunk)

