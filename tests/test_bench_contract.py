"""Host-side checks of bench.py that need no GPU: every workload can be named in the output line, profile
figures are read from the committed summaries, and a run on more than one GPU is refused with a message."""
import os
import subprocess
import sys

import bench

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_workload_descriptions_split_into_name_and_step():
    for name, spec in bench.WORKLOADS.items():
        head, sep, step = spec["what"].partition(": ")
        assert sep and head and step, name
    assert bench.HEADLINE in bench.WORKLOADS and set(bench.DEFAULT_SET) <= set(bench.WORKLOADS)


def test_profile_figures_are_read_from_the_committed_summaries():
    for wl, kind in (("cfg5", "parallel"), ("cfg5", "chunk"), ("cfg5", "serial"), ("cfg4", "parallel"), ("cfg4", "serial"),
                     ("cfg3", "parallel"), ("cfg2", "parallel")):
        v = bench.profile_figure(wl, kind)
        assert isinstance(v, int) and v > 0, (wl, kind)
    assert bench.profile_figure("cfg1", "parallel") is None


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one-GPU" in (r.stdout + r.stderr)
