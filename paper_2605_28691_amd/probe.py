"""Binding of the measurement library (``include/skiparse_probe.h``, libskiparse_probe.so): MFMA-only micro-kernels and the
device's compute-unit count and clock.  Loaded by the benchmark and by one GPU test only; no part of the attention path."""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libskiparse_probe.so")
BF16, FP8_E4M3 = 0, 2

_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: build it first (python -m paper_2605_28691_amd.build)")
        L = ctypes.CDLL(_LIB_PATH)
        i, vp, sz, pd = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_double)
        L.skiparse_mfma_probe.restype = i
        L.skiparse_mfma_probe.argtypes = [vp, sz, vp, sz, i, i, i, pd, vp]
        L.skiparse_mfma_lds_probe.restype = i
        L.skiparse_mfma_lds_probe.argtypes = [vp, sz, vp, sz, i, i, pd, vp]
        L.skiparse_mfma_valu_probe.restype = i
        L.skiparse_mfma_valu_probe.argtypes = [vp, sz, vp, sz, i, i, i, pd, vp]
        L.skiparse_mfma8_valu_probe.restype = i
        L.skiparse_mfma8_valu_probe.argtypes = [vp, sz, vp, sz, i, i, i, pd, vp]
        L.skiparse_mfma_chain_probe.restype = i
        L.skiparse_mfma_chain_probe.argtypes = [vp, sz, vp, sz, i, i, i, pd, vp]
        L.skiparse_lds_read_probe.restype = i
        L.skiparse_lds_read_probe.argtypes = [vp, sz, vp, sz, i, i, i, pd, vp]
        L.skiparse_probe_device_info.restype = i
        L.skiparse_probe_device_info.argtypes = [i, ctypes.POINTER(i), ctypes.POINTER(i)]
        L.skiparse_probe_last_hip_error.restype = i
        L.skiparse_probe_last_hip_error.argtypes = []
        _lib = L
    return _lib


def _check(code: int, what: str) -> None:
    if code != 0:
        raise RuntimeError(f"{what}: error code {code} (hipError {lib().skiparse_probe_last_hip_error()})")


def _args(operands: torch.Tensor, sink: torch.Tensor):
    for t, name in ((operands, "operands"), (sink, "sink")):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous device tensor")
    return (ctypes.c_void_p(operands.data_ptr()), operands.numel() * operands.element_size(), ctypes.c_void_p(sink.data_ptr()),
            sink.numel() * sink.element_size())


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def mfma_probe(operands: torch.Tensor, sink: torch.Tensor, fp8: bool, blocks: int, iters: int) -> float:
    """Enqueues the matrix-core-only kernel on the operand bytes; returns the FLOP of the launch."""
    flop = ctypes.c_double(0.0)
    _check(lib().skiparse_mfma_probe(*_args(operands, sink), FP8_E4M3 if fp8 else BF16, blocks, iters, ctypes.byref(flop), _stream()),
           "skiparse_mfma_probe")
    return flop.value


def mfma_lds_probe(operands: torch.Tensor, sink: torch.Tensor, blocks: int, iters: int) -> float:
    """bf16 MFMA loop whose A operand is read from LDS for every MFMA; returns the FLOP of the launch."""
    flop = ctypes.c_double(0.0)
    _check(lib().skiparse_mfma_lds_probe(*_args(operands, sink), blocks, iters, ctypes.byref(flop), _stream()), "skiparse_mfma_lds_probe")
    return flop.value


def mfma_valu_probe(operands: torch.Tensor, sink: torch.Tensor, valu_per_mfma: int, blocks: int, iters: int) -> float:
    """bf16 MFMA loop with `valu_per_mfma` independent FMAs after every MFMA; returns the FLOP of the launch."""
    flop = ctypes.c_double(0.0)
    _check(lib().skiparse_mfma_valu_probe(*_args(operands, sink), valu_per_mfma, blocks, iters, ctypes.byref(flop), _stream()),
           "skiparse_mfma_valu_probe")
    return flop.value


def mfma8_valu_probe(operands: torch.Tensor, sink: torch.Tensor, valu_per_mfma: int, blocks: int, iters: int) -> float:
    """fp8 MFMA loop with `valu_per_mfma` independent FMAs after every MFMA; returns the FLOP of the launch."""
    flop = ctypes.c_double(0.0)
    _check(lib().skiparse_mfma8_valu_probe(*_args(operands, sink), valu_per_mfma, blocks, iters, ctypes.byref(flop), _stream()),
           "skiparse_mfma8_valu_probe")
    return flop.value


def mfma_chain_probe(operands: torch.Tensor, sink: torch.Tensor, chain: int, blocks: int, iters: int) -> float:
    """bf16 MFMA loop with `chain` consecutive MFMAs on the same accumulator; returns the FLOP of the launch."""
    flop = ctypes.c_double(0.0)
    _check(lib().skiparse_mfma_chain_probe(*_args(operands, sink), chain, blocks, iters, ctypes.byref(flop), _stream()), "skiparse_mfma_chain_probe")
    return flop.value


def lds_read_probe(operands: torch.Tensor, sink: torch.Tensor, kind: int, blocks: int, iters: int) -> float:
    """LDS reads only (0: 16-byte fragment reads, 1: transposing reads, 2: plain 8-byte reads); returns the bytes read by the launch."""
    nbytes = ctypes.c_double(0.0)
    _check(lib().skiparse_lds_read_probe(*_args(operands, sink), kind, blocks, iters, ctypes.byref(nbytes), _stream()), "skiparse_lds_read_probe")
    return nbytes.value


def device_info(device: int = 0):
    """(compute units, nominal engine clock in kHz) as the HIP runtime reports them."""
    cu, khz = ctypes.c_int(0), ctypes.c_int(0)
    _check(lib().skiparse_probe_device_info(device, ctypes.byref(cu), ctypes.byref(khz)), "skiparse_probe_device_info")
    return cu.value, khz.value
