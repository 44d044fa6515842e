"""MI355X-native Skiparse-2D attention: thin Python binding over the C ABI in ``include/skiparse.h``.

Argument marshalling only.  Tensors are ``torch`` CUDA(HIP) tensors used purely as device memory; every step of
the path runs in the library's own kernels on the current torch stream.  There is no CPU fallback: without the
built library, or on a bad argument, a call raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libskiparse.so")

TOKEN, GROUP = 0, 1
BF16, FP32, FP8_E4M3 = 0, 1, 2
FUSED = 1
PAD = 2
PATTERNS = {"token": TOKEN, "group": GROUP}
OUT_LAYOUTS = {"same": 0, "other": 1, "original": 2}
_DTYPES = {torch.bfloat16: BF16, torch.float32: FP32, torch.uint8: FP8_E4M3, torch.float8_e4m3fn: FP8_E4M3}

_lib = None


class SkiparseError(RuntimeError):
    def __init__(self, code: int, what: str):
        msg = lib().skiparse_strerror(code).decode()
        extra = f" [hipError {lib().skiparse_last_hip_error()}]" if code == -5 else ""
        super().__init__(f"{what}: {msg} (code {code}){extra}")
        self.code = code


def lib() -> ctypes.CDLL:
    """Loads libskiparse.so (built by ``paper_2605_28691_amd.build.build()``); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(
                f"{_LIB_PATH} is missing: build it first (python -m paper_2605_28691_amd.build); there is no fallback path"
            )
        L = ctypes.CDLL(_LIB_PATH)
        i, vp, f, u, sz = ctypes.c_int, ctypes.c_void_p, ctypes.c_float, ctypes.c_uint, ctypes.c_size_t
        L.skiparse_permute.restype = i
        L.skiparse_permute.argtypes = [vp, vp] + [i] * 9 + [vp]
        L.skiparse_unpermute.restype = i
        L.skiparse_unpermute.argtypes = [vp, vp] + [i] * 9 + [vp]
        L.skiparse_switch_pattern.restype = i
        L.skiparse_switch_pattern.argtypes = [vp, vp] + [i] * 9 + [vp]
        L.skiparse_ssp_pack.restype = i
        L.skiparse_ssp_pack.argtypes = [vp, vp] + [i] * 9 + [vp]
        L.skiparse_ssp_unpack.restype = i
        L.skiparse_ssp_unpack.argtypes = [vp, vp] + [i] * 9 + [vp]
        L.dense_attn_fwd.restype = i
        L.dense_attn_fwd.argtypes = [vp] * 4 + [i] * 6 + [f, i, vp]
        L.skiparse_attn_fwd.restype = i
        L.skiparse_attn_fwd.argtypes = [vp] * 4 + [i] * 8 + [f, i, u, vp, sz, vp]
        L.skiparse_attn_fwd_sparse.restype = i
        L.skiparse_attn_fwd_sparse.argtypes = [vp] * 4 + [i] * 9 + [f, i, vp]
        L.skiparse_lse_bytes.restype = sz
        L.skiparse_lse_bytes.argtypes = [i] * 8 + [u]
        L.skiparse_attn_fwd_lse.restype = i
        L.skiparse_attn_fwd_lse.argtypes = [vp] * 5 + [i] * 8 + [f, i, u, vp]
        L.skiparse_bwd_workspace_bytes.restype = sz
        L.skiparse_bwd_workspace_bytes.argtypes = [i] * 8 + [u]
        L.skiparse_attn_bwd.restype = i
        L.skiparse_attn_bwd.argtypes = [vp] * 9 + [i] * 8 + [f, i, u, vp, sz, vp]
        L.skiparse_attn_bwd_static.restype = i
        L.skiparse_attn_bwd_static.argtypes = [vp] * 9 + [i] * 8 + [f, i, u, vp]
        L.skiparse_static_scratch_bytes.restype = sz
        L.skiparse_static_scratch_bytes.argtypes = []
        L.skiparse_workspace_bytes.restype = sz
        L.skiparse_workspace_bytes.argtypes = [i] * 8 + [u]
        L.skiparse_quantize_fp8_ex.restype = i
        L.skiparse_quantize_fp8_ex.argtypes = [vp, vp, vp] + [i] * 8 + [u, vp]
        L.skiparse_attn_fwd_fp8_ex.restype = i
        L.skiparse_attn_fwd_fp8_ex.argtypes = [vp] * 7 + [i] * 8 + [f, u, vp]
        L.skiparse_quantize_fp8.restype = i
        L.skiparse_quantize_fp8.argtypes = [vp, vp, vp] + [i] * 8 + [vp]
        L.skiparse_attn_fwd_fp8.restype = i
        L.skiparse_attn_fwd_fp8.argtypes = [vp] * 7 + [i] * 8 + [f, vp]
        L.skiparse_strerror.restype = ctypes.c_char_p
        L.skiparse_strerror.argtypes = [i]
        L.skiparse_last_hip_error.restype = i
        L.skiparse_last_hip_error.argtypes = []
        _lib = L
    return _lib


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t: torch.Tensor, name: str) -> ctypes.c_void_p:
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous device tensor")
    return ctypes.c_void_p(t.data_ptr())


def _check(code: int, what: str) -> None:
    if code != 0:
        raise SkiparseError(code, what)


def _dims(x: torch.Tensor, T: int, H: int, W: int):
    B, N, heads, D = x.shape
    if N != T * H * W:
        raise ValueError("token axis does not match T*H*W")
    return B, heads, D


def skiparse_permute(x: torch.Tensor, T: int, H: int, W: int, s: int, pattern: str, out: torch.Tensor | None = None):
    """[B][N][heads][D] -> [s*s*B][N/s^2][heads][D] (original -> sparse layout), bit-exact row gather."""
    B, heads, D = _dims(x, T, H, W)
    if out is None:
        out = torch.empty((s * s * B, (T * H * W) // (s * s), heads, D), dtype=x.dtype, device=x.device)
    _check(
        lib().skiparse_permute(_dev(x, "x"), _dev(out, "out"), B, heads, T, H, W, D, s, PATTERNS[pattern], _DTYPES[x.dtype], _stream()),
        "skiparse_permute",
    )
    return out


def skiparse_unpermute(y: torch.Tensor, T: int, H: int, W: int, s: int, pattern: str, out: torch.Tensor | None = None):
    """[s*s*B][N/s^2][heads][D] -> [B][N][heads][D] (sparse -> original layout)."""
    SB, Nsub, heads, D = y.shape
    B = SB // (s * s)
    if SB != B * s * s or Nsub * s * s != T * H * W:
        raise ValueError("sparse-layout shape does not match the grid")
    if out is None:
        out = torch.empty((B, T * H * W, heads, D), dtype=y.dtype, device=y.device)
    _check(
        lib().skiparse_unpermute(_dev(y, "y"), _dev(out, "out"), B, heads, T, H, W, D, s, PATTERNS[pattern], _DTYPES[y.dtype], _stream()),
        "skiparse_unpermute",
    )
    return out


def skiparse_switch_pattern(y: torch.Tensor, T: int, H: int, W: int, s: int, from_pattern: str, out: torch.Tensor | None = None):
    """Sparse layout of `from_pattern` -> sparse layout of the other pattern, one row move per token."""
    SB, Nsub, heads, D = y.shape
    B = SB // (s * s)
    if SB != B * s * s or Nsub * s * s != T * H * W:
        raise ValueError("sparse-layout shape does not match the grid")
    if out is None:
        out = torch.empty_like(y)
    _check(
        lib().skiparse_switch_pattern(_dev(y, "y"), _dev(out, "out"), B, heads, T, H, W, D, s, PATTERNS[from_pattern], _DTYPES[y.dtype], _stream()),
        "skiparse_switch_pattern",
    )
    return out


def skiparse_ssp_pack(x: torch.Tensor, T: int, H: int, W: int, s: int, group_size: int, out: torch.Tensor | None = None):
    """One rank's shard [G*b][T*(H/s)*(W/s)][heads][D] (G = s*s/group_size subsequences, batch fastest) -> the all-to-all send buffer
    [group_size][G][G*b][T*(H/s^2)*(W/s^2)][heads][D] of Sparse Sequence Parallelism (chunk r is for rank r)."""
    Bl, n_local, heads, D = x.shape
    G = (s * s) // group_size
    if G < 1 or G * group_size != s * s or Bl % G or n_local * s * s != T * H * W:
        raise ValueError("shard shape does not match the grid and the group")
    if out is None:
        out = torch.empty((group_size, G, Bl, n_local // (s * s), heads, D), dtype=x.dtype, device=x.device)
    _check(
        lib().skiparse_ssp_pack(_dev(x, "x"), _dev(out, "out"), Bl // G, heads, T, H, W, D, s, group_size, _DTYPES[x.dtype], _stream()),
        "skiparse_ssp_pack",
    )
    return out


def skiparse_ssp_unpack(recv: torch.Tensor, T: int, H: int, W: int, s: int, group_size: int, out: torch.Tensor | None = None):
    """The all-to-all receive buffer [group_size][G][G*b][base][heads][D] (chunk r came from rank r) -> the rank's shard
    [G*b][T*(H/s)*(W/s)][heads][D] in the other pattern's sparse layout."""
    gs, G, Bl, base, heads, D = recv.shape
    if gs != group_size or G * group_size != s * s or Bl % G or base * s * s * s * s != T * H * W:
        raise ValueError("receive-buffer shape does not match the grid and the group")
    if out is None:
        out = torch.empty((Bl, base * s * s, heads, D), dtype=recv.dtype, device=recv.device)
    _check(
        lib().skiparse_ssp_unpack(_dev(recv, "recv"), _dev(out, "out"), Bl // G, heads, T, H, W, D, s, group_size, _DTYPES[recv.dtype], _stream()),
        "skiparse_ssp_unpack",
    )
    return out


def dense_attn_fwd(q, k, v, T: int, H: int, W: int, scale: float = 0.0, out: torch.Tensor | None = None):
    """softmax(q k^T * scale) v over all T*H*W tokens for every (batch, head); bf16 in, bf16 out."""
    B, heads, D = _dims(q, T, H, W)
    if out is None:
        out = torch.empty_like(q)
    _check(
        lib().dense_attn_fwd(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), _dev(out, "out"), B, heads, T, H, W, D, float(scale),
                             _DTYPES[q.dtype], _stream()),
        "dense_attn_fwd",
    )
    return out


def skiparse_workspace_bytes(B, heads, T, H, W, D, s, fused: bool) -> int:
    return int(lib().skiparse_workspace_bytes(B, heads, T, H, W, D, s, BF16, FUSED if fused else 0))


def skiparse_attn_fwd(q, k, v, T: int, H: int, W: int, s: int, pattern: str, scale: float = 0.0, fused: bool = True,
                      out: torch.Tensor | None = None, workspace: torch.Tensor | None = None, pad: bool = False):
    """Skiparse-2D attention, q/k/v/out in the original layout.  The unfused path needs a uint8 device workspace of
    skiparse_workspace_bytes() bytes; one is allocated with torch if none is passed.  pad=True selects the any-resolution
    mode (fused only): H and W arbitrary, end padding to multiples of s*s masked."""
    B, heads, D = _dims(q, T, H, W)
    if out is None:
        out = torch.empty_like(q)
    ws_ptr, ws_bytes = ctypes.c_void_p(0), 0
    if not fused:
        need = skiparse_workspace_bytes(B, heads, T, H, W, D, s, False)
        if workspace is None:
            workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=q.device)
        ws_ptr, ws_bytes = _dev(workspace, "workspace"), workspace.numel() * workspace.element_size()
    _check(
        lib().skiparse_attn_fwd(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), _dev(out, "out"), B, heads, T, H, W, D, s,
                                PATTERNS[pattern], float(scale), _DTYPES[q.dtype], (FUSED if fused else 0) | (PAD if pad else 0), ws_ptr, ws_bytes,
                                _stream()),
        "skiparse_attn_fwd",
    )
    return out


def skiparse_attn_fwd_sparse(q, k, v, T: int, H: int, W: int, s: int, pattern: str, out_layout: str = "other", scale: float = 0.0,
                             out: torch.Tensor | None = None):
    """Attention on tensors already in the sparse layout of `pattern` ([s*s*B][N/s^2][heads][D]); the output goes to the
    same layout ("same"), the other pattern's sparse layout ("other") or the original layout ("original")."""
    SB, Nsub, heads, D = q.shape
    B = SB // (s * s)
    if SB != B * s * s or Nsub * s * s != T * H * W:
        raise ValueError("sparse-layout shape does not match the grid")
    if out is None:
        shape = (B, T * H * W, heads, D) if out_layout == "original" else tuple(q.shape)
        out = torch.empty(shape, dtype=q.dtype, device=q.device)
    _check(
        lib().skiparse_attn_fwd_sparse(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), _dev(out, "out"), B, heads, T, H, W, D, s,
                                       PATTERNS[pattern], OUT_LAYOUTS[out_layout], float(scale), _DTYPES[q.dtype], _stream()),
        "skiparse_attn_fwd_sparse",
    )
    return out


def skiparse_lse_shape(B, heads, T, H, W, D, s, pattern: str, pad: bool = False):
    """Shape of the log-sum-exp tensor: [s*s*B][heads][positions per subsequence] (positions of the padded grid with pad=True)."""
    n = int(lib().skiparse_lse_bytes(B, heads, T, H, W, D, s, PATTERNS[pattern], PAD if pad else 0)) // 4
    if n == 0:
        raise ValueError("grid does not fit the pattern (use pad=True for the any-resolution mode)")
    return (s * s * B, heads, n // (s * s * B * heads))


def skiparse_attn_fwd_lse(q, k, v, T: int, H: int, W: int, s: int, pattern: str, scale: float = 0.0,
                          out: torch.Tensor | None = None, lse: torch.Tensor | None = None, pad: bool = False):
    """Fused forward that also returns the log-sum-exp the backward pass needs: (out, lse), lse float32 in subsequence order."""
    B, heads, D = _dims(q, T, H, W)
    if out is None:
        out = torch.empty_like(q)
    if lse is None:
        lse = torch.empty(skiparse_lse_shape(B, heads, T, H, W, D, s, pattern, pad), dtype=torch.float32, device=q.device)
    _check(
        lib().skiparse_attn_fwd_lse(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), _dev(out, "out"), _dev(lse, "lse"), B, heads, T, H, W, D, s,
                                    PATTERNS[pattern], float(scale), _DTYPES[q.dtype], PAD if pad else 0, _stream()),
        "skiparse_attn_fwd_lse",
    )
    return out, lse


def skiparse_bwd_workspace_bytes(B, heads, T, H, W, D, s, pattern: str, pad: bool = False) -> int:
    return int(lib().skiparse_bwd_workspace_bytes(B, heads, T, H, W, D, s, PATTERNS[pattern], PAD if pad else 0))


def skiparse_attn_bwd(q, k, v, out, dout, lse, T: int, H: int, W: int, s: int, pattern: str, scale: float = 0.0,
                      dq=None, dk=None, dv=None, workspace: torch.Tensor | None = None, pad: bool = False):
    """Gradients (dq, dk, dv) of the Skiparse attention layer; out and lse come from skiparse_attn_fwd_lse (same pad flag).  A
    uint8 device workspace of skiparse_bwd_workspace_bytes() bytes is allocated with torch if none is passed."""
    B, heads, D = _dims(q, T, H, W)
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(q) if dk is None else dk
    dv = torch.empty_like(q) if dv is None else dv
    if workspace is None:
        workspace = torch.empty(max(skiparse_bwd_workspace_bytes(B, heads, T, H, W, D, s, pattern, pad), 1), dtype=torch.uint8, device=q.device)
    _check(
        lib().skiparse_attn_bwd(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), _dev(out, "out"), _dev(dout, "dout"), _dev(lse, "lse"),
                                _dev(dq, "dq"), _dev(dk, "dk"), _dev(dv, "dv"), B, heads, T, H, W, D, s, PATTERNS[pattern], float(scale),
                                _DTYPES[q.dtype], PAD if pad else 0, _dev(workspace, "workspace"),
                                workspace.numel() * workspace.element_size(), _stream()),
        "skiparse_attn_bwd",
    )
    return dq, dk, dv


def skiparse_attn_bwd_static(q, k, v, out, dout, lse, dq, dk, dv, T: int, H: int, W: int, s: int, pattern: str, scale: float = 0.0,
                             pad: bool = False):
    """skiparse_attn_bwd for callers that cannot allocate: the delta workspace is the library's static device array, and this
    wrapper allocates nothing either (dq, dk, dv must be passed).  Problems above the array's size raise (code -4)."""
    B, heads, D = _dims(q, T, H, W)
    _check(
        lib().skiparse_attn_bwd_static(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), _dev(out, "out"), _dev(dout, "dout"), _dev(lse, "lse"),
                                       _dev(dq, "dq"), _dev(dk, "dk"), _dev(dv, "dv"), B, heads, T, H, W, D, s, PATTERNS[pattern],
                                       float(scale), _DTYPES[q.dtype], PAD if pad else 0, _stream()),
        "skiparse_attn_bwd_static",
    )
    return dq, dk, dv


def skiparse_quantize_fp8(x: torch.Tensor, T: int, H: int, W: int, s: int, pattern: str, pad: bool = False):
    """bf16 [B][N][heads][D] (original layout) -> (uint8 E4M3 codes [s*s*B][positions][heads][D] in the sparse layout,
    float32 scales [s*s*B][heads][ceil(positions/128)]).  positions = N/s^2, or with pad=True (any-resolution mode) the positions
    of the grid padded to multiples of s*s, with zero codes at the padding."""
    B, heads, D = _dims(x, T, H, W)
    if x.dtype != torch.bfloat16:
        raise ValueError("skiparse_quantize_fp8 takes bf16 input")
    nsub = skiparse_lse_shape(B, heads, T, H, W, D, s, pattern, pad)[2]
    x8 = torch.empty((s * s * B, nsub, heads, D), dtype=torch.uint8, device=x.device)
    scales = torch.empty((s * s * B, heads, (nsub + 127) // 128), dtype=torch.float32, device=x.device)
    _check(
        lib().skiparse_quantize_fp8_ex(_dev(x, "x"), _dev(x8, "x8"), _dev(scales, "scales"), B, heads, T, H, W, D, s,
                                       PATTERNS[pattern], PAD if pad else 0, _stream()),
        "skiparse_quantize_fp8",
    )
    return x8, scales


def skiparse_attn_fwd_fp8(q8, k8, v8, sq, sk, sv, T: int, H: int, W: int, s: int, pattern: str, scale: float = 0.0,
                          out: torch.Tensor | None = None, pad: bool = False):
    """Attention on quantised sparse-layout tensors (from skiparse_quantize_fp8, same pad flag); bf16 output [B][N][heads][D] in the
    original layout."""
    SB, nsub, heads, D = q8.shape
    B = SB // (s * s)
    if SB != B * s * s or (not pad and nsub * s * s != T * H * W):
        raise ValueError("sparse-layout shape does not match the grid")
    if out is None:
        out = torch.empty((B, T * H * W, heads, D), dtype=torch.bfloat16, device=q8.device)
    _check(
        lib().skiparse_attn_fwd_fp8_ex(_dev(q8, "q8"), _dev(k8, "k8"), _dev(v8, "v8"), _dev(sq, "sq"), _dev(sk, "sk"), _dev(sv, "sv"),
                                       _dev(out, "out"), B, heads, T, H, W, D, s, PATTERNS[pattern], float(scale), PAD if pad else 0, _stream()),
        "skiparse_attn_fwd_fp8",
    )
    return out
