"""The kernels' index arithmetic on unchecked device contents (csrc/index_math.h) is plain C++:
a host program sweeps hostile values (INT_MIN .. INT_MAX lengths, offsets, page ids, parents, kept
indices, paths) through it and checks that every row it produces lies inside the buffers the host
arguments describe.  Built with AddressSanitizer and UBSan, so a signed overflow fails too.
The GPU test with the same hostile contents stays as the second line of defence."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_index_math_sweep_under_sanitizers(tmp_path):
    exe = str(tmp_path / "index_math_sweep")
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-I", os.path.join(ROOT, "paper_2503_14075_amd", "csrc"),
                           os.path.join(ROOT, "tests", "host", "index_math_sweep.cpp"), "-o", exe])
    out = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stderr[-2000:]
    assert "index_math sweep: ok" in out.stdout
