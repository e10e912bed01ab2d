"""bench.py's command line, host side only (nothing touches a GPU)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    # this build runs on one GPU; the refusal comes before torch or the library is loaded
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=60)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and "--gpus 1" in r.stderr
    assert r.stdout.strip() == ""            # no JSON line that could be taken for a measurement


def test_help_lists_every_mode():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--help"], capture_output=True, text=True, timeout=60)
    assert r.returncode == 0
    for flag in ("--gpus", "--steps", "--warmup", "--workload", "--pipeline", "--all", "--verify", "--draft", "--ragged", "--stream", "--ablations"):
        assert flag in r.stdout


def test_roofline_traffic_is_read_from_the_tracked_counter_summaries():
    """bench.py holds no counter literal: the figure comes from profiles/ (FETCH/WRITE KiB per launch times the
    calibration factors stated there), and a kernel the summary does not list yields no figure."""
    import re
    sys.path.insert(0, ROOT)
    import bench
    text = open(os.path.join(ROOT, "profiles", bench.COUNTER_FILES["reduce5"])).read()
    rows = [ln for ln in text.splitlines() if re.match(r"^\S.*\s{2,}\d+\s+\d+\s+\d+\s", ln)]
    assert len(rows) >= 5
    name = rows[0].split("  ")[0].strip()
    nums = [int(x) for x in re.findall(r"\s(\d+)(?=\s)", rows[0][len(name):])][:3]
    got = bench.counter_traffic("reduce5", [name])
    assert got == nums[1] * 1024 * 2.0 + nums[2] * 1024 * 1.0        # the factors of the summary's calibration line
    assert bench.counter_traffic("reduce5", ["a_kernel_that_does_not_exist"]) is None
    assert bench.counter_traffic("vocab", ["draft_scan_kernel", "draft_merge_kernel"]) > 150e6
