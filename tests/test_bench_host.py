"""Host-side checks of bench.py (no GPU): the one-GPU rule, and that the HBM traffic it reports
is read from the committed profile summaries of the workloads it names."""

import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
from paper_2602_00269_amd import synth  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_traffic_comes_from_the_profile_summaries():
    names = [synth._PRESETS[c][0] for c in (2, 3, 4, 5)]
    names += [synth._MULTI_PRESETS[k][0] for k in synth.MULTI_NAMES]
    names += [f"{w}_{s}x{v}" for w, (s, v, _) in bench.SAMPLE_WORKLOADS.items()]
    for name in names:
        t = bench.measured_traffic(name)
        assert isinstance(t, int) and t > 0, name
    assert bench.measured_traffic("no_such_workload") is None
    # a prefix of a workload's name must not pick up another workload's summary
    assert bench.measured_traffic("cfg3") is None


def test_every_profile_names_its_command_and_kernel():
    pdir = os.path.join(ROOT, "profiles")
    files = sorted(f for f in os.listdir(pdir) if f.endswith(".txt"))
    assert len(files) >= 11
    for f in files:
        text = open(os.path.join(pdir, f)).read()
        assert "rocprofv3 --kernel-trace --stats" in text and "rocprofv3 --pmc FETCH_SIZE" in text, f
        assert "bench.py --workload" in text and "traffic =" in text, f
        assert len(text) < 8192, f  # short summaries only
