"""bench.py's command-line contract where it can be checked without a GPU."""

import os
import subprocess
import sys

from conftest import ROOT


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def _bench_module():
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench_under_test", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_traffic_comes_from_a_profile_record_of_the_same_sources(tmp_path):
    """roofline.traffic is a measurement that belongs to the library sources it
    was taken on: a record with the current digest counts and names its file
    and commit, one with another digest yields None and the reason."""
    bench = _bench_module()
    now = bench.csrc_digest()
    assert len(now) == 16 and int(now, 16) >= 0
    prof = tmp_path / "profiles"
    prof.mkdir()
    (prof / "a_kernel.md").write_text(
        "# summary\n\n"
        "traffic-record: workload=w_one kernel=k_one bytes=1.5e9 csrc=%s commit=abc1234\n"
        "traffic-record: workload=w_two kernel=k_one bytes=2.5e9 csrc=0123456789abcdef commit=abc1234\n"
        % now)
    (prof / "ignored.csv").write_text(
        "traffic-record: workload=w_two kernel=k_one bytes=9e9 csrc=%s commit=x\n" % now)
    bench.PROFILES_DIR = str(prof)
    value, source = bench.measured_traffic("w_one", "k_one")
    assert value == 1.5e9 and "a_kernel.md" in source and "abc1234" in source
    value, source = bench.measured_traffic("w_two", "k_one")
    assert value is None and "other sources" in source and "0123456789abcdef" in source
    value, source = bench.measured_traffic("w_one", "k_two")
    assert value is None and "no rocprofv3 counter summary" in source
    bench.PROFILES_DIR = str(tmp_path / "missing")
    assert bench.measured_traffic("w_one", "k_one")[0] is None


def test_digest_follows_the_library_sources(tmp_path):
    bench = _bench_module()
    src = tmp_path / "csrc"
    src.mkdir()
    (src / "a.hip").write_text("kernel")
    (src / "b.h").write_text("header")
    (src / "notes.txt").write_text("not a source")
    bench.CSRC_DIR = str(src)
    d0 = bench.csrc_digest()
    (src / "notes.txt").write_text("changed")
    assert bench.csrc_digest() == d0
    (src / "b.h").write_text("header changed")
    d1 = bench.csrc_digest()
    assert d1 != d0
    (src / "c.cpp").write_text("")
    assert bench.csrc_digest() != d1


def test_committed_traffic_records_are_well_formed():
    """Every traffic-record line under profiles/ parses and names a positive
    byte count (whether it is current is bench.py's business at run time)."""
    import re
    n = 0
    prof = os.path.join(ROOT, "profiles")
    for name in sorted(os.listdir(prof)):
        with open(os.path.join(prof, name)) as f:
            for line in f:
                if "traffic-record:" not in line:
                    continue
                m = re.match(r"\s*traffic-record:\s*workload=(\S+)\s+kernel=(\S+)\s+bytes=(\S+)"
                             r"\s+csrc=([0-9a-f]{16})\s+commit=([0-9a-f]{7,40})\s*$", line)
                assert m, (name, line)
                assert float(m.group(3)) > 0
                n += 1
    assert n >= 4
