"""The schedule simulator against the closed forms of the paper's Table 1 (equal forward / p1 / p2 times)."""
import os
from fractions import Fraction

import pytest

from paper_2405_18047_amd import schedule as sch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table1_n4.txt")


def test_simulator_reproduces_the_printed_table_at_n4():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) == 4
    for name, a, b, gain in rows:
        without = sch.simulate(name, 4, two_bp=False)
        with_ = sch.simulate(name, 4, two_bp=True)
        assert without.bubble_ratio == Fraction(a), name
        assert with_.bubble_ratio == Fraction(b), name
        assert sch.throughput_gain(name, 4) == Fraction(gain), name


@pytest.mark.parametrize("n", [2, 3, 4, 5, 8, 16])
def test_closed_forms_for_other_pipeline_depths(n):
    closed = sch.table1(n)
    for name in sch.SCHEDULES:
        a, b, gain = closed[name]
        assert sch.simulate(name, n, two_bp=False).bubble_ratio == a, (name, n)
        assert sch.simulate(name, n, two_bp=True).bubble_ratio == b, (name, n)
        assert sch.throughput_gain(name, n) == gain, (name, n)
        assert gain == (1 - b) / (1 - a)                    # the paper's (1 - b) / (1 - a)


def test_work_is_conserved_and_memory_claims_hold():
    n = 4
    for name in sch.SCHEDULES:
        r0 = sch.simulate(name, n, 2, 3, 5, two_bp=False)
        r1 = sch.simulate(name, n, 2, 3, 5, two_bp=True)
        assert r0.busy_per_stage == r1.busy_per_stage        # 2BP re-orders work, it never adds any
        assert r1.makespan <= r0.makespan
    # Section 4.2: under 1F1B-1 the first stage only ever holds one micro-batch of derivatives, the last holds N
    r = sch.simulate("1f1b-1", n, two_bp=True)
    assert r.peak_pending_p2[0] == 1 and r.peak_pending_p2[-1] == n
    # a stage with free weight gradients gains nothing from deferring them
    assert sch.throughput_gain("1f1b-1", n, 1, 1, 0) == 1


def test_bench_schedule_prediction_and_power_sampler_without_a_gpu():
    """The host-side legs of the benchmark: with equal times the prediction equals Table 1's closed forms; with a
    cheap p2 the gain shrinks towards 1; the power sampler reports nothing rather than failing where the GPU's sysfs
    files do not exist."""
    import bench
    eq = bench.schedule_prediction(5.0, 5.0, 5.0)
    assert eq["gain"] == eq["gain_equal_times_table1"]
    cheap = bench.schedule_prediction(5.0, 5.0, 0.05)
    for k, v in cheap["gain"].items():
        assert 1.0 <= v < 1.01 and v < eq["gain"][k], k
    with bench._PowerSampler() as smp:
        pass
    assert isinstance(smp.mhz, list) and isinstance(smp.watts, list)
