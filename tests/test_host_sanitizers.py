"""Host code under the sanitizers (no GPU): the round planner and the prompt plan (C++, AddressSanitizer + UBSan,
native drivers with seeded random inputs) and the oracle (C, UBSan, its own pins run once more against the
instrumented build).  A finding aborts the instrumented program, which fails the test."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan"]


def test_prompt_plan_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "prompt_plan_fuzz")
    cmd = ["g++", "-std=c++17", "-O1", "-g", *SAN, "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "prompt_plan_fuzz.cpp"),
           os.path.join(ROOT, "paper_2604_03143_amd", "csrc", "tdk_prompt.cpp"), "-o", exe]
    subprocess.run(cmd, check=True)
    run = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "clean" in run.stdout


def test_round_planner_under_asan_and_ubsan(tmp_path):
    """tdk_round_create's validation and index arithmetic (block-table slices, row map, page table, rotation
    tables, work list, per-XCD queues) live in csrc/tdk_plan.cpp, which needs no HIP."""
    exe = str(tmp_path / "plan_fuzz")
    csrc = os.path.join(ROOT, "paper_2604_03143_amd", "csrc")
    cmd = ["g++", "-std=c++17", "-O1", "-g", *SAN, "-I", os.path.join(ROOT, "include"), "-I", csrc,
           os.path.join(ROOT, "tests", "plan_fuzz.cpp"), os.path.join(csrc, "tdk_plan.cpp"), "-o", exe]
    subprocess.run(cmd, check=True)
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "clean" in run.stdout


def test_oracle_pins_under_ubsan(tmp_path):
    so = str(tmp_path / "libtdo_ubsan.so")
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
           "-fsanitize=undefined", "-fno-sanitize-recover=all", "-o", so, os.path.join(ROOT, "oracle", "tdo.c"), "-lm"]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, TDO_LIBRARY=so)
    tests = [os.path.join(ROOT, "tests", t) for t in ("test_oracle_rotate.py", "test_oracle_round.py", "test_oracle_attend.py",
                                                       "test_oracle_check_layer.py", "test_oracle_accounting.py")]
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *tests],
                         capture_output=True, text=True, env=env, cwd=ROOT, timeout=900)
    assert run.returncode == 0, run.stdout[-3000:] + run.stderr[-3000:]
