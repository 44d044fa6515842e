"""Float64 CPU oracle for Skiparse-2D attention.  TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper around ``skiparse_oracle.c`` (plain C, float64, OpenMP over independent query
rows).  Only the tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import this
package; the GPU library never does, and this package never imports the GPU library.

Array conventions: inputs are C-contiguous numpy arrays in the original layout ``[B][N][heads][D]``
with dtype ``uint16`` (bfloat16 bit patterns), ``float32`` or ``float64``; attention outputs are
``float64``.  Patterns: ``"token"`` (token-wise sparse attention) and ``"group"`` (group-wise sparse
attention), Sec. 3.1 and Algorithm 1 of the OSP-Next paper.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "skiparse_oracle.c")
_LIB = os.path.join(_HERE, "libskiparse_oracle.so")

PATTERNS = {"token": 0, "group": 1}
_DTYPES = {np.dtype(np.uint16): 0, np.dtype(np.float32): 1, np.dtype(np.float64): 2}


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (a second or two); returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i, i64, dbl, vp = ctypes.c_int, ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        lib.oracle_src_index.restype = i64
        lib.oracle_src_index.argtypes = [i, i, i, i, i, i, i, i64]
        lib.oracle_dst_index.restype = None
        lib.oracle_dst_index.argtypes = [i, i, i, i, i, i64, ctypes.POINTER(i), ctypes.POINTER(i), ctypes.POINTER(i64)]
        lib.oracle_permute.restype = i
        lib.oracle_permute.argtypes = [vp, vp, i, i, i, i, i64, i, i]
        lib.oracle_unpermute.restype = i
        lib.oracle_unpermute.argtypes = [vp, vp, i, i, i, i, i64, i, i]
        lib.oracle_attention_bwd.restype = i
        lib.oracle_attention_bwd.argtypes = [vp] * 7 + [i64, i64, i, i, dbl, i]
        lib.oracle_skiparse_attention_bwd.restype = i
        lib.oracle_skiparse_attention_bwd.argtypes = [vp] * 7 + [i] * 8 + [dbl, i]
        lib.oracle_skiparse_attention_bwd_padded.restype = i
        lib.oracle_skiparse_attention_bwd_padded.argtypes = [vp] * 7 + [i] * 8 + [dbl, i]
        lib.oracle_skiparse_attention_bwd_unit_padded.restype = i
        lib.oracle_skiparse_attention_bwd_unit_padded.argtypes = [vp] * 5 + [i64] + [vp] * 3 + [i, i] + [i] * 8 + [dbl, i]
        lib.oracle_skiparse_attention_bwd_unit.restype = i
        lib.oracle_skiparse_attention_bwd_unit.argtypes = [vp] * 5 + [i64] + [vp] * 3 + [i, i, i64] + [i] * 8 + [dbl, i]
        lib.oracle_switch_pattern.restype = i
        lib.oracle_switch_pattern.argtypes = [vp, vp, i, i, i, i, i64, i, i]
        lib.oracle_attention.restype = i
        lib.oracle_attention.argtypes = [vp, vp, vp, vp, i64, i64, i, i, dbl, i]
        lib.oracle_skiparse_attention.restype = i
        lib.oracle_skiparse_attention.argtypes = [vp, vp, vp, vp, i, i, i, i, i, i, i, i, dbl, i]
        lib.oracle_skiparse_attention_rows.restype = i
        lib.oracle_skiparse_attention_rows.argtypes = [vp, vp, vp, vp, i64, vp, i, i, i, i, i, i, i, i, dbl, i]
        lib.oracle_skiparse_attention_rows_padded.restype = i
        lib.oracle_skiparse_attention_rows_padded.argtypes = [vp, vp, vp, vp, i64, vp, i, i, i, i, i, i, i, i, dbl, i]
        lib.oracle_masked_dense_attention.restype = i
        lib.oracle_masked_dense_attention.argtypes = [vp, vp, vp, vp, i, i, i, i, i, i, i, i, dbl, i]
        lib.oracle_quantize_fp8.restype = i
        lib.oracle_quantize_fp8.argtypes = [vp, vp, vp, i, i, i, i, i, i, i, i]
        lib.oracle_e4m3_encode.restype = ctypes.c_uint8
        lib.oracle_e4m3_encode.argtypes = [ctypes.c_float]
        lib.oracle_e4m3_decode.restype = dbl
        lib.oracle_e4m3_decode.argtypes = [ctypes.c_uint8]
        lib.oracle_num_threads.restype = i
        lib.oracle_num_threads.argtypes = []
        _lib = lib
    return _lib


def _ptr(a: np.ndarray) -> ctypes.c_void_p:
    return ctypes.c_void_p(a.ctypes.data)


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError(f"oracle: {what} rejected its arguments or ran out of memory (code {rc})")


def _dtype_code(*arrays: np.ndarray) -> int:
    dt = arrays[0].dtype
    for a in arrays:
        if a.dtype != dt or not a.flags.c_contiguous:
            raise ValueError("oracle inputs must share one dtype and be C-contiguous")
    if dt not in _DTYPES:
        raise ValueError(f"oracle: unsupported dtype {dt} (use uint16 bf16 bits, float32 or float64)")
    return _DTYPES[dt]


def num_threads() -> int:
    """Threads the OpenMP loops of the oracle will use."""
    return int(_load().oracle_num_threads())


def src_index(pattern: str, s: int, T: int, H: int, W: int, p: int, q: int, j: int) -> int:
    """Token index n of element j of the subsequence with spatial class (p, q) (Algorithm 1)."""
    return int(_load().oracle_src_index(PATTERNS[pattern], s, T, H, W, p, q, j))


def dst_index(pattern: str, s: int, T: int, H: int, W: int, n: int):
    """(p, q, j) of token n: its spatial class and its position inside that subsequence."""
    p, q, j = ctypes.c_int(), ctypes.c_int(), ctypes.c_int64()
    _load().oracle_dst_index(PATTERNS[pattern], s, T, H, W, n, ctypes.byref(p), ctypes.byref(q), ctypes.byref(j))
    return p.value, q.value, j.value


def permute(x: np.ndarray, T: int, H: int, W: int, s: int, pattern: str) -> np.ndarray:
    """[B][N][...] -> [s*s*B][N/s^2][...], rows moved verbatim (any dtype)."""
    x = np.ascontiguousarray(x)
    B, N = x.shape[0], x.shape[1]
    if N != T * H * W:
        raise ValueError("token axis does not match T*H*W")
    row_bytes = x.strides[1]
    y = np.empty((s * s * B, N // (s * s)) + x.shape[2:], dtype=x.dtype)
    _check(_load().oracle_permute(_ptr(x), _ptr(y), B, T, H, W, row_bytes, s, PATTERNS[pattern]), "permute")
    return y


def unpermute(y: np.ndarray, T: int, H: int, W: int, s: int, pattern: str) -> np.ndarray:
    """Inverse of :func:`permute`."""
    y = np.ascontiguousarray(y)
    B = y.shape[0] // (s * s)
    N = T * H * W
    if y.shape[0] != B * s * s or y.shape[1] * s * s != N:
        raise ValueError("sparse-layout shape does not match the grid")
    row_bytes = y.strides[1]
    x = np.empty((B, N) + y.shape[2:], dtype=y.dtype)
    _check(_load().oracle_unpermute(_ptr(y), _ptr(x), B, T, H, W, row_bytes, s, PATTERNS[pattern]), "unpermute")
    return x


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float) -> np.ndarray:
    """softmax(Q K^T * scale) V for every (batch, head); q,k,v are [nb][n][heads][D]."""
    code = _dtype_code(q, k, v)
    nb, n, heads, D = q.shape
    out = np.empty(q.shape, dtype=np.float64)
    _check(_load().oracle_attention(_ptr(q), _ptr(k), _ptr(v), _ptr(out), nb, n, heads, D, float(scale), code), "attention")
    return out


def skiparse_attention(q, k, v, T: int, H: int, W: int, s: int, pattern: str, scale: float) -> np.ndarray:
    """unpermute(attention(permute(q), permute(k), permute(v))), original layout in and out."""
    code = _dtype_code(q, k, v)
    B, N, heads, D = q.shape
    if N != T * H * W:
        raise ValueError("token axis does not match T*H*W")
    out = np.empty(q.shape, dtype=np.float64)
    _check(
        _load().oracle_skiparse_attention(
            _ptr(q), _ptr(k), _ptr(v), _ptr(out), B, heads, T, H, W, D, s, PATTERNS[pattern], float(scale), code
        ),
        "skiparse_attention",
    )
    return out


def skiparse_attention_rows(q, k, v, rows, T: int, H: int, W: int, s: int, pattern: str, scale: float) -> np.ndarray:
    """Rows of :func:`skiparse_attention` for query positions rows[i] = (b, head, n) only -> [n_rows][D]."""
    code = _dtype_code(q, k, v)
    B, N, heads, D = q.shape
    if N != T * H * W:
        raise ValueError("token axis does not match T*H*W")
    rows = np.ascontiguousarray(np.asarray(rows, dtype=np.int64).reshape(-1, 3))
    out = np.empty((rows.shape[0], D), dtype=np.float64)
    _check(
        _load().oracle_skiparse_attention_rows(
            _ptr(q), _ptr(k), _ptr(v), _ptr(rows), rows.shape[0], _ptr(out), B, heads, T, H, W, D, s,
            PATTERNS[pattern], float(scale), code,
        ),
        "skiparse_attention_rows",
    )
    return out


def attention_bwd(q, k, v, dout, scale: float):
    """Gradients (dq, dk, dv) of :func:`attention` for dL/dout = dout; all [nb][n][heads][D], float64 results."""
    code = _dtype_code(q, k, v, dout)
    nb, n, heads, D = q.shape
    dq, dk, dv = (np.empty(q.shape, dtype=np.float64) for _ in range(3))
    _check(
        _load().oracle_attention_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(dout), _ptr(dq), _ptr(dk), _ptr(dv), nb, n, heads, D, float(scale), code),
        "attention_bwd",
    )
    return dq, dk, dv


def skiparse_attention_bwd(q, k, v, dout, T: int, H: int, W: int, s: int, pattern: str, scale: float):
    """Gradients (dq, dk, dv) of :func:`skiparse_attention`, original layout in and out."""
    code = _dtype_code(q, k, v, dout)
    B, N, heads, D = q.shape
    if N != T * H * W:
        raise ValueError("token axis does not match T*H*W")
    dq, dk, dv = (np.empty(q.shape, dtype=np.float64) for _ in range(3))
    _check(
        _load().oracle_skiparse_attention_bwd(
            _ptr(q), _ptr(k), _ptr(v), _ptr(dout), _ptr(dq), _ptr(dk), _ptr(dv), B, heads, T, H, W, D, s, PATTERNS[pattern], float(scale), code
        ),
        "skiparse_attention_bwd",
    )
    return dq, dk, dv


def skiparse_attention_bwd_unit(q, k, v, dout, b: int, head: int, toks, T: int, H: int, W: int, s: int, pattern: str, scale: float):
    """Gradient rows (dq, dk, dv), each [len(toks)][D], for tokens `toks` of ONE attention unit: batch element b, head `head`
    and the subsequence that holds toks[0] (every token listed must lie in it).  Walks the whole unit."""
    code = _dtype_code(q, k, v, dout)
    B, N, heads, D = q.shape
    if N != T * H * W:
        raise ValueError("token axis does not match T*H*W")
    toks = np.ascontiguousarray(np.asarray(toks, dtype=np.int64).reshape(-1))
    dq, dk, dv = (np.empty((toks.shape[0], D), dtype=np.float64) for _ in range(3))
    _check(
        _load().oracle_skiparse_attention_bwd_unit(
            _ptr(q), _ptr(k), _ptr(v), _ptr(dout), _ptr(toks), toks.shape[0], _ptr(dq), _ptr(dk), _ptr(dv), int(b), int(head),
            int(toks[0]), B, heads, T, H, W, D, s, PATTERNS[pattern], float(scale), code,
        ),
        "skiparse_attention_bwd_unit",
    )
    return dq, dk, dv


def skiparse_attention_bwd_padded(q, k, v, dout, T: int, H: int, W: int, s: int, pattern: str, scale: float):
    """Gradients (dq, dk, dv) in the any-resolution mode (mask form: real tokens of one class attend to each other; any H, W)."""
    code = _dtype_code(q, k, v, dout)
    B, N, heads, D = q.shape
    if N != T * H * W:
        raise ValueError("token axis does not match T*H*W")
    dq, dk, dv = (np.empty(q.shape, dtype=np.float64) for _ in range(3))
    _check(
        _load().oracle_skiparse_attention_bwd_padded(
            _ptr(q), _ptr(k), _ptr(v), _ptr(dout), _ptr(dq), _ptr(dk), _ptr(dv), B, heads, T, H, W, D, s, PATTERNS[pattern], float(scale), code
        ),
        "skiparse_attention_bwd_padded",
    )
    return dq, dk, dv


def skiparse_attention_bwd_unit_padded(q, k, v, dout, b: int, head: int, toks, T: int, H: int, W: int, s: int, pattern: str, scale: float):
    """Any-resolution mode: gradient rows (dq, dk, dv), each [len(toks)][D], for tokens of ONE class (that of toks[0]) of batch
    element b and head `head`; walks the whole unit."""
    code = _dtype_code(q, k, v, dout)
    B, N, heads, D = q.shape
    if N != T * H * W:
        raise ValueError("token axis does not match T*H*W")
    toks = np.ascontiguousarray(np.asarray(toks, dtype=np.int64).reshape(-1))
    dq, dk, dv = (np.empty((toks.shape[0], D), dtype=np.float64) for _ in range(3))
    _check(
        _load().oracle_skiparse_attention_bwd_unit_padded(
            _ptr(q), _ptr(k), _ptr(v), _ptr(dout), _ptr(toks), toks.shape[0], _ptr(dq), _ptr(dk), _ptr(dv), int(b), int(head),
            B, heads, T, H, W, D, s, PATTERNS[pattern], float(scale), code,
        ),
        "skiparse_attention_bwd_unit_padded",
    )
    return dq, dk, dv


def masked_dense_attention(q, k, v, T: int, H: int, W: int, s: int, pattern: str, scale: float) -> np.ndarray:
    """Brute force: N x N attention with pairs of different spatial class masked out (tiny grids only)."""
    code = _dtype_code(q, k, v)
    B, N, heads, D = q.shape
    if N != T * H * W:
        raise ValueError("token axis does not match T*H*W")
    out = np.empty(q.shape, dtype=np.float64)
    _check(
        _load().oracle_masked_dense_attention(
            _ptr(q), _ptr(k), _ptr(v), _ptr(out), B, heads, T, H, W, D, s, PATTERNS[pattern], float(scale), code
        ),
        "masked_dense_attention",
    )
    return out


def e4m3_encode(y: float) -> int:
    """E4M3 code of a float with |y| <= 448 (round to nearest even)."""
    return int(_load().oracle_e4m3_encode(float(y)))


def e4m3_decode(code: int) -> float:
    return float(_load().oracle_e4m3_decode(int(code)))


def e4m3_decode_array(codes: np.ndarray) -> np.ndarray:
    """Values of an array of E4M3 codes as float64 (through the 256-entry decode table)."""
    table = np.array([e4m3_decode(c) for c in range(256)], dtype=np.float64)
    table[[0x7F, 0xFF]] = np.nan
    return table[codes]


def quantize_fp8(x: np.ndarray, T: int, H: int, W: int, s: int, pattern: str):
    """bf16 bit patterns in the original layout -> (E4M3 codes in the sparse layout, float32 scales per
    (subsequence, head, 128-position block)); the 8-bit workload's recipe."""
    if x.dtype != np.uint16 or not x.flags.c_contiguous:
        raise ValueError("quantize_fp8 takes C-contiguous uint16 bf16 bit patterns")
    B, N, heads, D = x.shape
    if N != T * H * W:
        raise ValueError("token axis does not match T*H*W")
    nsub = N // (s * s)
    x8 = np.empty((s * s * B, nsub, heads, D), dtype=np.uint8)
    scales = np.empty((s * s * B, heads, (nsub + 127) // 128), dtype=np.float32)
    _check(_load().oracle_quantize_fp8(_ptr(x), _ptr(x8), _ptr(scales), B, heads, T, H, W, D, s, PATTERNS[pattern]), "quantize_fp8")
    return x8, scales


def skiparse_attention_rows_padded(q, k, v, rows, T: int, H: int, W: int, s: int, pattern: str, scale: float) -> np.ndarray:
    """Any-resolution Skiparse attention (end padding to multiples of s*s, padding masked), rows[i] = (b, head, n) only.
    H and W need not be divisible by anything; for divisible grids this equals skiparse_attention_rows."""
    code = _dtype_code(q, k, v)
    B, N, heads, D = q.shape
    if N != T * H * W:
        raise ValueError("token axis does not match T*H*W")
    rows = np.ascontiguousarray(np.asarray(rows, dtype=np.int64).reshape(-1, 3))
    out = np.empty((rows.shape[0], D), dtype=np.float64)
    _check(
        _load().oracle_skiparse_attention_rows_padded(
            _ptr(q), _ptr(k), _ptr(v), _ptr(rows), rows.shape[0], _ptr(out), B, heads, T, H, W, D, s,
            PATTERNS[pattern], float(scale), code,
        ),
        "skiparse_attention_rows_padded",
    )
    return out


def switch_pattern(y: np.ndarray, T: int, H: int, W: int, s: int, from_pattern: str) -> np.ndarray:
    """Sparse layout of `from_pattern` -> sparse layout of the other pattern (Alg. 1, tsa_to_gsa / gsa_to_tsa)."""
    y = np.ascontiguousarray(y)
    B = y.shape[0] // (s * s)
    if y.shape[0] != B * s * s or y.shape[1] * s * s != T * H * W:
        raise ValueError("sparse-layout shape does not match the grid")
    out = np.empty_like(y)
    _check(_load().oracle_switch_pattern(_ptr(y), _ptr(out), B, T, H, W, y.strides[1], s, PATTERNS[from_pattern]), "switch_pattern")
    return out


# ---- Sparse Sequence Parallelism (Sec. 3.3; Algorithm 1, sparse_sequence_parallel): the steps of ONE rank, in the paper's order.
# A rank's shard is [(g, bb)][positions of a subsequence][...]: its G = s*s/group_size subsequences in class order, batch fastest.
# Plain compositions of this package's permute / unpermute (on the reduced grid (T, H/s, W/s)) and numpy axis moves.


def ssp_pack(x: np.ndarray, T: int, H: int, W: int, s: int, group_size: int) -> np.ndarray:
    """Step 1 and the view of step 2: every held subsequence is split token-wise once more on its own grid (T, H/s, W/s);
    returns the send buffer [group_size][G][G*b][T*(H/s^2)*(W/s^2)][...] (chunk r goes to rank r)."""
    G = s * s // group_size
    if G * group_size != s * s or x.shape[0] % G or H % (s * s) or W % (s * s):
        raise ValueError("group_size must divide s*s, the shard must hold G subsequences, H and W must be multiples of s*s")
    y = permute(x, T, H // s, W // s, s, "token")  # [(p' q' B_local)][base][...]
    return y.reshape((group_size, G, x.shape[0]) + y.shape[1:])


def ssp_exchange(sends):
    """What all_to_all_single does to the ranks' send buffers: rank r receives chunk r of every rank, in rank order."""
    n = len(sends)
    return [np.stack([sends[src][dst] for src in range(n)], axis=0) for dst in range(n)]


def ssp_unpack(recv: np.ndarray, T: int, H: int, W: int, s: int, group_size: int) -> np.ndarray:
    """Steps 3 and 4: recv [group_size][G][G*b][base][...] -> view [src rank][g'][g][b], swap the two subsequence axes, flatten to
    (p q b') order and undo the token-wise split on the reduced grid: the rank's shard in the other pattern's layout."""
    G = s * s // group_size
    Bl = recv.shape[2]
    b = Bl // G
    r = recv.reshape((group_size, G, G, b) + recv.shape[3:])
    r = np.ascontiguousarray(np.swapaxes(r, 1, 2)).reshape((s * s * G * b,) + recv.shape[3:])
    return unpermute(r, T, H // s, W // s, s, "token")


def quantize_fp8_padded(x: np.ndarray, T: int, H: int, W: int, s: int, pattern: str):
    """The 8-bit workload's quantiser in the any-resolution mode (Sec. 3.2): the grid is padded with zero tokens at the END of H and W
    to the next multiples of s*s and the padded tensor is quantised as usual.  Zero rows do not move a block's maximum and encode to
    code 0, so padding positions hold zeros and every scale is that of the block's real rows (1 for a block of nothing but padding).
    Returns (codes [s*s*B][T*Hp*Wp/s^2][heads][D], scales [s*s*B][heads][ceil(Nsub_padded/128)])."""
    if x.dtype != np.uint16:
        raise ValueError("quantize_fp8_padded takes uint16 bf16 bit patterns")
    B, N, heads, D = x.shape
    if N != T * H * W:
        raise ValueError("token axis does not match T*H*W")
    u = s * s
    Hp, Wp = (H + u - 1) // u * u, (W + u - 1) // u * u
    g = x.reshape(B, T, H, W, heads, D)
    g = np.pad(g, ((0, 0), (0, 0), (0, Hp - H), (0, Wp - W), (0, 0), (0, 0)))  # bf16 bit pattern 0 is +0.0
    return quantize_fp8(np.ascontiguousarray(g.reshape(B, T * Hp * Wp, heads, D)), T, Hp, Wp, s, pattern)
