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


def test_lds_tile_layout_is_consistent_and_conflict_free(tmp_path):
    """The swizzled LDS layout the attention kernels stage into: coverage, read addresses, bank conflicts (host check)."""
    exe = str(tmp_path / "host_lds_layout_check")
    src = os.path.join(ROOT, "tests", "host_lds_layout_check.cpp")
    subprocess.check_call(["/opt/rocm/bin/hipcc", "-x", "hip", "--offload-arch=gfx950", "-O1", "-std=c++17",
                           "-Wno-unused-command-line-argument", "-o", exe, src])
    out = subprocess.run([exe], stdout=subprocess.PIPE, text=True)
    assert out.returncode == 0, out.stdout
    assert out.stdout.startswith("ok")
