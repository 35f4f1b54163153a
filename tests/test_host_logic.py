"""Host logic of the library that needs no GPU: the segment pools that hold the list data
and the choice of resident lists under a budget are plain C++ behind allocation callbacks,
so a C++ test (tests/cpp/pool_test.cpp) drives them over heap memory: random walks
against a block map, out-of-memory paths, hand-worked rankings.  Built with the host
compiler and its undefined-behaviour and address checks."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_pool_bookkeeping_and_residency_choice(tmp_path):
    exe = str(tmp_path / "pool_test")
    src = os.path.join(ROOT, "tests", "cpp", "pool_test.cpp")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-Wall", "-Wextra", "-Werror",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", src, "-o", exe]
    subprocess.run(cmd, check=True, cwd=ROOT)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout + r.stderr
