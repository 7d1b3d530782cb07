"""The measurement build of the library (same sources, per-block phase stamps compiled into the transfer kernel) and
its report, `bench.py --phases`: eight launches per step, every block of every launch with five ordered stamps."""
import os
import subprocess
import sys

import pytest

from paper_1910_04732_amd import flop

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_phase_report_of_the_benchmark_step():
    if not os.path.exists(flop.LIB_PATH_PHASES):
        pytest.skip("measurement build not present (built by __graft_entry__.build())")
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--phases"], stdout=subprocess.PIPE,
                       stderr=subprocess.STDOUT, text=True, timeout=240, cwd=ROOT)
    assert p.returncode == 0, p.stdout[-2000:]
    rows = [l for l in p.stdout.splitlines() if "<" in l and "/" in l]
    assert len(rows) == 8, p.stdout[-2000:]
    for l in rows:
        f = l.split(">")[1].replace("/", " ").split()
        blocks, span, event = int(f[0]), float(f[1]), float(f[-1])
        phases = [float(v) for v in f[2:-1]]
        assert blocks >= 192 and len(phases) == 12 and all(v > 0.0 for v in phases)
        # a block's median phase times fit into the launch's span, and the span into about the launch's own
        # begin/end events (wide margins: the figures are timings)
        assert sum(phases[1::3]) <= span * 1.25 and span <= event * 2.0
