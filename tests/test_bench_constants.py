"""The traffic constants bench.py carries are the totals of the rocprofv3 summaries under profiles/."""
import glob
import os
import re

import bench

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _profiled():
    stage, call = {}, {}
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*_hbm_traffic.txt"))):
        for line in open(path):
            m = re.match(r"bench constant \((\w+), (\w+)\) = (\d+)\s*$", line)
            if m:
                stage[(m.group(1), m.group(2))] = int(m.group(3))
            m = re.match(r"bench constant call\((\w+)\) = (\d+)\s*$", line)
            if m:
                call[m.group(1)] = int(m.group(2))
    return stage, call


def test_every_traffic_constant_of_the_benchmark_is_a_profiled_total():
    stage, call = _profiled()
    for key, value in bench.MEASURED_TRAFFIC.items():
        assert key in stage, "no profile line for %s" % (key,)
        assert stage[key] == value, "%s: bench.py has %d, profiles/ has %d" % (key, value, stage[key])
    for key, value in bench.MEASURED_CALL_TRAFFIC.items():
        assert key in call, "no profile line for call(%s)" % key
        assert call[key] == value, "call(%s): bench.py has %d, profiles/ has %d" % (key, value, call[key])


def test_profiled_workloads_are_used_by_the_benchmark():
    # a summary that bench.py ignores has gone stale unnoticed: every whole-call total must be carried
    _, call = _profiled()
    for key in call:
        assert key in bench.MEASURED_CALL_TRAFFIC, "profiles/ holds call(%s) but bench.py does not use it" % key
