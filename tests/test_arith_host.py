"""Host build of the GPU library's integer arithmetic against the % operator."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_device_arithmetic_matches_plain_modulo_on_the_host(tmp_path):
    exe = tmp_path / "arith_selftest"
    subprocess.check_call(["g++", "-O2", "-std=c++17", "-fsanitize=undefined", "-fno-sanitize-recover=all",
                           "-I", os.path.join(ROOT, "paper_1205_2958_amd", "csrc"),
                           os.path.join(ROOT, "tests", "arith_selftest.cpp"), "-o", str(exe)])
    out = subprocess.run([str(exe)], stdout=subprocess.PIPE, text=True, timeout=300)
    assert out.returncode == 0, out.stdout
    assert out.stdout.startswith("OK "), out.stdout
    assert int(out.stdout.split()[1]) > 10_000_000
