"""Host logic of bench.py that needs no GPU: how K steps are cut into graph launches,
the median helper, and the refusal of more than one GPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


class _Recorder:
    """Stands in for GraphSteps' graph capture: counts what a run would launch."""

    def __init__(self, n_sets):
        self.gs = bench.GraphSteps.__new__(bench.GraphSteps)
        self.gs.n_sets = n_sets

    def steps(self, n):
        total = 0
        for (kind, k), times in self.gs._parts(n):
            assert k > 0 and times > 0
            if kind == "rot":
                assert k <= self.gs.n_sets
            total += k * times
        return total


@pytest.mark.parametrize("n_sets", [1, 2, 5, 19, 32])
def test_a_run_launches_exactly_the_steps_asked_for(n_sets):
    rec = _Recorder(n_sets)
    for n in [0, 1, 2, 5, 19, 20, 37, 200, 255, 256, 257, 300, 1000, 4000, 4001]:
        assert rec.steps(n) == n, (n_sets, n)


def test_short_runs_are_one_graph_and_long_ones_whole_rotations():
    rec = _Recorder(19)
    assert rec.gs._parts(20) == [(("run", 20), 1)]
    assert rec.gs._parts(4000) == [(("rot", 19), 210), (("rot", 10), 1)]
    assert rec.gs._parts(0) == []


def test_median():
    assert bench.median([3.0, 1.0, 2.0]) == 2.0
    assert bench.median([4.0, 1.0, 2.0, 3.0]) == 2.5


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr
