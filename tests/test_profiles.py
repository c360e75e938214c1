"""The benchmark's `roofline.traffic` comes from the rocprofv3 summaries under profiles/ (bench.measured_traffic
parses them at run time, there is no second copy of the numbers).  These checks keep the two in step:
every summary must parse, agree with the algorithmic bytes it quotes itself, and give the command that
made it; the headline workload must have one."""
import glob
import os
import re

import pytest

import bench

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FILES = sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md")))


def test_the_headline_profile_exists_and_is_what_bench_reads():
    path = bench.profile_name("rtopk_wave_kernel", "c1_maxk", 32)
    assert os.path.exists(os.path.join(ROOT, path)), path
    traffic = bench.measured_traffic(path)
    algo = (1 << 20) * 1280
    assert traffic is not None and 0.98 * algo <= traffic <= 1.05 * algo


@pytest.mark.parametrize("path", FILES, ids=[os.path.basename(f) for f in FILES])
def test_profile_summary_parses_and_is_self_consistent(path):
    text = open(path).read()
    rel = os.path.relpath(path, ROOT)
    assert "rocprofv3 --kernel-trace --stats" in text and "rocprofv3 --pmc FETCH_SIZE" in text, "the commands are part of the summary"
    assert "_work" not in text, "a summary's commands run committed files only"
    traffic = bench.measured_traffic(rel)
    assert traffic is not None, "no 'HBM read ... + write ... = ... B per launch' line bench.py can use"
    # every such line: the total is the sum of its parts and within a few percent of the algorithmic bytes it quotes
    lines = re.findall(r"HBM read ([\d,]+) B \+ write ([\d,]+) B = ([\d,]+) B per launch; algorithmic ([\d,]+) B \(ratio ([\d.]+)\)", text)
    assert lines
    for rd, wr, tot, algo, ratio in lines:
        rd, wr, tot, algo = (int(v.replace(",", "")) for v in (rd, wr, tot, algo))
        assert abs(rd + wr - tot) <= 2
        assert abs(tot / algo - float(ratio)) < 1e-3
        # (also for rows too wide to hold on chip: on this workload the streamed kernel finds its k pairs in
        # the pass that finds the row's minimum and maximum, so it too reads a row once)
        assert 0.9 < tot / algo < 1.15, "measured traffic far from the algorithmic bytes: re-reads or a stale summary"
    # no derived percentage above 100
    for pct in re.findall(r"\((\d+) %\)", text):
        assert int(pct) <= 100, "a utilisation above 100 % is a normalisation error"
