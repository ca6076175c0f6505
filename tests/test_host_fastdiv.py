"""The reciprocal divisions of the kernels (csrc/fastdiv.h) against integer division, on the host: the header
compiles as plain C++, so a small program sweeps divisors and the dividends where a wrong reciprocal shows first
(multiples of the divisor near the top of the range; the last columns of the largest planes of every height)."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_reciprocal_divisions_are_exact(tmp_path):
    exe = str(tmp_path / "fastdiv_check")
    subprocess.check_call(["g++", "-O2", "-std=c++17", "-Wall", "-I", os.path.join(ROOT, "paper_1412_4564_amd", "csrc"),
                           "-o", exe, os.path.join(ROOT, "tests", "fastdiv_check.cpp")])
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and r.stdout.startswith("OK"), r.stdout[-500:] + r.stderr[-500:]


def test_stream_k_piece_lists_match_a_simulation_of_the_blocks(tmp_path):
    """csrc/streamk.h compiles as plain C++: the pieces the fix-up pass adds for every left-over tile against the
    segments the main kernel's blocks write (tests/streamk_check.cpp)."""
    exe = str(tmp_path / "streamk_check")
    subprocess.check_call(["g++", "-O2", "-std=c++17", "-Wall", "-I", os.path.join(ROOT, "paper_1412_4564_amd", "csrc"),
                           "-o", exe, os.path.join(ROOT, "tests", "streamk_check.cpp")])
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and r.stdout.startswith("OK"), r.stdout[-500:] + r.stderr[-500:]
