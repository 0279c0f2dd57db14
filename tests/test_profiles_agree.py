"""The committed rocprofv3 summaries and bench.py's own per-launch timing must tell the same story.

Every ``profiles/<workload>.md`` ends with an ``agreement:`` line written by the run that produced it: the
average duration of the dominant kernel family as bench.py measured it (device timestamps of each launch, the
same command run without the profiler) and as ``rocprofv3 --kernel-trace --stats`` reports it for that command.
The two must agree within 3 % (or 0.6 us where that is more: between two runs of the same command the average of
the 15 us launches of the ResNeXt workload moves by 0.5 us, 15.2 ... 15.7, while its step time stays at
0.828 - 0.830 ms), and the roofline fraction derived from either must match the bytes stated.
"""
import glob
import json
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SUMMARIES = sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md")))


def agreement(path):
    lines = [l for l in open(path) if l.startswith("agreement:")]
    assert len(lines) == 1, path
    return {k: v for k, v in re.findall(r"(\w+)=([\w.+-]+)", lines[0])}


def test_every_workload_has_a_summary():
    names = {os.path.basename(p)[:-3] for p in SUMMARIES}
    assert {"encoder12_m32_s128", "encoder12_m32_s512", "resnet50_m32", "resnext50_32x4d_m16"} <= names


@pytest.mark.parametrize("path", SUMMARIES, ids=[os.path.basename(p) for p in SUMMARIES])
def test_bench_and_rocprof_durations_agree(path):
    a = agreement(path)
    bench_us, prof_us = float(a["bench_avg_us"]), float(a["rocprof_avg_us"])
    assert abs(bench_us - prof_us) <= max(0.03 * prof_us, 0.6), (bench_us, prof_us)
    assert abs(float(a["ratio"]) - bench_us / prof_us) < 1e-3
    # the fractions are algorithmic bytes / duration / 8 TB/s, from either duration
    nbytes = float(a["bytes_per_launch"])
    assert abs(float(a["frac_from_rocprof"]) - nbytes / (prof_us * 1e-6) / 8e12) < 2e-4
    assert abs(float(a["frac_from_bench"]) - nbytes / (bench_us * 1e-6) / 8e12) < 2e-4


@pytest.mark.parametrize("path", SUMMARIES, ids=[os.path.basename(p) for p in SUMMARIES])
def test_summary_names_its_commands_and_traffic(path):
    text = open(path).read()
    name = os.path.basename(path)[:-3]
    assert "rocprofv3 --kernel-trace --stats" in text and "--workload " + name in text
    assert "--pmc FETCH_SIZE" in text and "--pmc WRITE_SIZE" in text
    traffic = json.load(open(os.path.join(ROOT, "profiles", "traffic.json")))
    assert name in traffic
    # measured HBM traffic of the dominant family: at least the algorithmic bytes less counter noise, and not
    # more than 1.5 times them (beyond that a kernel re-reads an operand from HBM)
    nbytes = float(agreement(path)["bytes_per_launch"])
    assert 0.9 * nbytes <= traffic[name] <= 1.5 * nbytes, (traffic[name], nbytes)
