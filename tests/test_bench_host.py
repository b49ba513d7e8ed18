"""Host-side logic of bench.py that needs no GPU."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_power_sampler_integrates_by_trapezoids():
    import bench
    ps = bench.PowerSampler.__new__(bench.PowerSampler)
    ps.samples = [(0.0, 100.0), (1.0, 100.0), (2.0, 300.0), (2.5, 300.0)]      # seconds, watts
    assert abs(ps.joules() - (100.0 + 200.0 + 150.0)) < 1e-9
    ps.samples = [(5.0, 42.0)]
    assert ps.joules() == 0.0
