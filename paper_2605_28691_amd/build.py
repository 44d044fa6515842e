"""Compiles the HIP sources under csrc/ (gfx950 only), in-tree: libskiparse.so, the attention library, and
libskiparse_probe.so, the measurement micro-kernels the benchmark times."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libskiparse.so")
SOURCES = ["api.hip", "permute.hip", "attn_fwd.hip", "attn_bwd.hip", "quant_fp8.hip", "attn_fwd_fp8.hip"]
PROBE_LIB = os.path.join(HERE, "libskiparse_probe.so")
PROBE_SOURCES = ["mfma_probe.hip"]
FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-shared",
    # packed-fp32 instructions are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def build(verbose: bool = False, save_temps: bool = False) -> str:
    """Builds both libraries; returns the path of the attention library."""
    _build_one(PROBE_LIB, PROBE_SOURCES, verbose, False)
    return _build_one(LIB, SOURCES, verbose, save_temps)


def _build_one(lib: str, sources, verbose: bool, save_temps: bool) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + os.environ.get("SKIPARSE_EXTRA_FLAGS", "").split()
    if save_temps:
        tmp = os.path.join(HERE, "_build")
        os.makedirs(tmp, exist_ok=True)
        cmd += ["-save-temps=obj"]
        out = os.path.join(tmp, os.path.basename(lib))
    else:
        out = lib + ".tmp"
    cmd += ["-o", out] + [os.path.join(CSRC, s) for s in sources]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the packed-fp32 target feature and says so; that is harmless
    log = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + log)
    if verbose and log.strip():
        print(log)
    os.replace(out, lib)
    return lib


if __name__ == "__main__":
    print(build(verbose=True, save_temps=bool(os.environ.get("SAVE_TEMPS"))))
