"""The launch-table store keeps every table it handed out at its address with its
contents when it grows (queued kernels and captured HIP graphs keep reading
them): checked on the host with a malloc back end, no GPU involved."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_table_cache_growth_keeps_earlier_tables(tmp_path):
    exe = tmp_path / "table_cache_check"
    src = os.path.join(ROOT, "tests", "host", "table_cache_check.cpp")
    subprocess.run(["g++", "-std=c++17", "-O1", "-Wall", "-fsanitize=address,undefined", src, "-o", str(exe)], check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    sys.stdout.write(r.stdout)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout + r.stderr
