"""bench.py takes the HBM traffic of its dominant kernel from the committed rocprofv3 counter summary instead of a
number typed into the script: the summary must be there, parse, and cover both time-loop launches, and the kernel
summary of the same workload must list the same kernels.  CPU only."""
import os
import re

import bench

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_traffic_of_both_time_loop_kernels_comes_from_the_profile():
    for symbol in ("lstm_pipe_fwd_kernel", "lstm_pipe_bwd_kernel"):
        t = bench.traffic_from_profile("max", symbol)
        assert t is not None and 0.2e9 < t < 5e9, (symbol, t)
    assert bench.traffic_from_profile("nav", "lstm_pipe_bwd_kernel") is None      # the summary covers `max` only
    assert bench.traffic_from_profile("max", "no_such_kernel") is None
    assert bench.traffic_from_profile("max", "lstm_pipe_bwd_kernel", root="/nonexistent") is None


def test_profiles_name_their_commands_and_kernels():
    text = open(os.path.join(ROOT, bench.TRAFFIC_PROFILE)).read()
    assert text.count("rocprofv3 --pmc") >= 4 and "FETCH_SIZE" in text and "WRITE_SIZE" in text
    kernels = open(os.path.join(ROOT, "profiles", "all_kernels_max_workload.md")).read()
    assert "rocprofv3 --kernel-trace --stats" in kernels
    for symbol in ("lstm_pipe_fwd_kernel", "lstm_pipe_bwd_kernel"):
        assert re.search(r"\| `" + symbol + r"[^|]*\| \d+ \| [\d.]+ \| [\d.]+ \|", kernels), symbol
