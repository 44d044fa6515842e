"""Host logic of the library that can run without a GPU: the device index map evaluated on the host."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_index_map_matches_plain_formulas(tmp_path):
    exe = str(tmp_path / "host_index_map_check")
    src = os.path.join(ROOT, "tests", "host_index_map_check.cpp")
    subprocess.check_call(["/opt/rocm/bin/hipcc", "-x", "hip", "--offload-arch=gfx950", "-O1", "-std=c++17",
                           "-Wno-unused-command-line-argument", "-o", exe, src])
    out = subprocess.run([exe], stdout=subprocess.PIPE, text=True)
    assert out.returncode == 0, out.stdout
    assert out.stdout.startswith("ok")
