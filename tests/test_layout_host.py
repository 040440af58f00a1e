"""The payload address arithmetic of the decode kernels, compiled for the host from the very
header the kernels include, over every tensor length up to 6000 and b = 2, 3, 4: no load
reaches outside [0, tq_payload_bytes) -- in particular not for the ragged last group of a
3-bit payload that ends exactly on a 16-byte boundary -- and every code is read from its own
bits.  No GPU is involved."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_code_load_stays_inside_the_payload(tmp_path):
    exe = str(tmp_path / "layout_check")
    subprocess.check_call(["g++", "-O1", "-std=c++17", "-Wall", "-Wextra", "-Werror",
                           "-fsanitize=undefined", "-fno-sanitize-recover=all",
                           "-I", os.path.join(ROOT, "paper_2402_01798_amd", "csrc"),
                           os.path.join(ROOT, "tests", "layout_check.cpp"), "-o", exe])
    out = subprocess.run([exe, "6000"], capture_output=True, text=True)
    assert out.returncode == 0, out.stdout + out.stderr
    assert out.stdout.startswith("ok ")
