"""The planner of the streamed attention launch cuts the work items of a launch into
equal runs of key blocks: coverage, part numbering and balance are checked on the host
(plain C++, no GPU involved)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_attn_stream_plan_covers_every_block_once_and_balances(tmp_path):
    exe = tmp_path / "attn_plan_check"
    src = os.path.join(ROOT, "tests", "host", "attn_plan_check.cpp")
    subprocess.run(["g++", "-std=c++17", "-O1", "-Wall", "-fsanitize=address,undefined", src, "-o", str(exe)], check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    sys.stdout.write(r.stdout)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout + r.stderr
