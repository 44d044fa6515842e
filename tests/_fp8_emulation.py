"""Test-side emulation of an IDEAL E4M3 attention pipeline (numpy float64).  TEST INFRASTRUCTURE ONLY.

What it is for.  The 8-bit variant (OCP FP8 E4M3 with one float32 scale per (subsequence, head, 128 positions),
motivated by Sec. 3.5's 8-bit attention MatMuls) is compared with the float64 oracle evaluated on the UNQUANTISED
inputs.  Most of that difference is the format's rounding, not the kernel's arithmetic.  This module evaluates the
workload's recipe with every operation exact except the E4M3 roundings the recipe prescribes:
    q8, k8, v8, scales        from the oracle's block quantiser
    S = scale * (q8 sq)(k8 sk)^T,  m = max over ALL keys of the row,  P = exp(S - m)          float64
    P8 = e4m3(P * sv_block / sv_max * 16)                                                      the only other rounding
    O  = (sum_keys P8 v8) * sv_max / 16 / sum_keys P
Its error against the exact oracle is the floor any implementation of the recipe sits on; the GPU tests bound the
kernel's error by a small multiple of it.  Nothing here comes from the GPU library, and the GPU library never sees it.
"""
import numpy as np

import oracle

P_GAIN = 16.0
BLOCK = 128


def e4m3_round(x: np.ndarray) -> np.ndarray:
    """Nearest E4M3 value (ties to the even mantissa), saturating at +-448: 3 mantissa bits, smallest normal 2^-6,
    subnormal step 2^-9.  Vectorised; pinned against the oracle's scalar encoder in the CPU tests."""
    x = np.asarray(x, dtype=np.float64)
    a = np.minimum(np.abs(x), 448.0)
    e = np.floor(np.log2(np.maximum(a, 2.0 ** -6)))  # exponent of the binade; everything below 2^-6 shares the subnormal step
    step = np.exp2(e - 3.0)
    r = np.round(a / step) * step  # numpy rounds halves to even; a/step is exact (power-of-two step)
    return np.copysign(np.minimum(r, 448.0), x)


def dequantised_unit(x8: np.ndarray, scales: np.ndarray, sb: int, head: int) -> np.ndarray:
    """[Nsub][D] float64 values of one (subsequence, head) of a quantised tensor in the sparse layout."""
    codes = x8[sb, :, head, :]
    blk = np.arange(codes.shape[0]) // BLOCK
    return oracle.e4m3_decode_array(codes) * scales[sb, head, blk].astype(np.float64)[:, None]


def ideal_unit(q8, sq, k8, sk, v8, sv, sb: int, head: int, scale: float, positions=None) -> np.ndarray:
    """Ideal-E4M3 attention output of one (subsequence, head): rows `positions` (all when None), [len][D] float64."""
    qd = dequantised_unit(q8, sq, sb, head)
    if positions is not None:
        qd = qd[np.asarray(positions)]
    kd = dequantised_unit(k8, sk, sb, head)
    vcodes = oracle.e4m3_decode_array(v8[sb, :, head, :])  # raw code values: the V scale rides on the probabilities
    svb = sv[sb, head, np.arange(v8.shape[1]) // BLOCK].astype(np.float64)
    sv_max = float(sv[sb, head].max())
    S = scale * (qd @ kd.T)
    P = np.exp(S - S.max(axis=1, keepdims=True))
    P8 = e4m3_round(P * (svb / sv_max * P_GAIN)[None, :])
    return (P8 @ vcodes) * (sv_max / P_GAIN) / P.sum(axis=1, keepdims=True)


def ideal_attention(q, k, v, T, H, W, s, pattern, scale):
    """Whole tensor, original layout in and out (q, k, v: bf16 bit patterns as the oracle takes them)."""
    (q8, sq), (k8, sk), (v8, sv) = (oracle.quantize_fp8(t, T, H, W, s, pattern) for t in (q, k, v))
    sbn, nsub, heads, D = q8.shape
    o = np.empty((sbn, nsub, heads, D), dtype=np.float64)
    for sb in range(sbn):
        for hd in range(heads):
            o[sb, :, hd, :] = ideal_unit(q8, sq, k8, sk, v8, sv, sb, hd, scale)
    return oracle.unpermute(o, T, H, W, s, pattern)


def ideal_attention_rows(q, k, v, rows, T, H, W, s, pattern, scale):
    """rows[i] = (b, head, n) -> [len(rows)][D]; rows of one (subsequence, head) are evaluated together."""
    (q8, sq), (k8, sk), (v8, sv) = (oracle.quantize_fp8(t, T, H, W, s, pattern) for t in (q, k, v))
    B = q.shape[0]
    rows = np.asarray(rows, dtype=np.int64).reshape(-1, 3)
    where = {}
    for i, (b, hd, n) in enumerate(rows):
        p, qq, j = oracle.dst_index(pattern, s, T, H, W, int(n))
        where.setdefault(((p * s + qq) * B + int(b), int(hd)), []).append((i, j))
    out = np.empty((rows.shape[0], q.shape[3]), dtype=np.float64)
    for (sb, hd), lst in where.items():
        idx = [i for i, _ in lst]
        out[idx] = ideal_unit(q8, sq, k8, sk, v8, sv, sb, hd, scale, positions=[j for _, j in lst])
    return out


# ---- any-resolution mode (Sec. 3.2): positions run over the grid padded to multiples of s*s; padding positions are zero codes, masked
# as keys and skipped as queries.


def padded_positions(B, T, H, W, s, pattern):
    """tok_at[sb][j] = token number (in the unpadded tensor) at position j of subsequence sb of the padded grid, -1 for padding;
    from the oracle's permute applied to the token numbers of the zero-padded grid."""
    u = s * s
    Hp, Wp = (H + u - 1) // u * u, (W + u - 1) // u * u
    ids = np.arange(T * H * W, dtype=np.int64).reshape(1, T, H, W)
    ids = np.pad(ids, ((0, 0), (0, 0), (0, Hp - H), (0, Wp - W)), constant_values=-1)
    ids = np.repeat(ids, B, axis=0).reshape(B, T * Hp * Wp, 1)
    return oracle.permute(ids, T, Hp, Wp, s, pattern)[:, :, 0]


def ideal_attention_rows_padded(q, k, v, rows, T, H, W, s, pattern, scale):
    """rows[i] = (b, head, n) of REAL tokens -> [len(rows)][D]: the ideal-E4M3 pipeline on the padded quantised tensors with the
    padding positions masked as keys."""
    (q8, sq), (k8, sk), (v8, sv) = (oracle.quantize_fp8_padded(t, T, H, W, s, pattern) for t in (q, k, v))
    B = q.shape[0]
    tok_at = padded_positions(B, T, H, W, s, pattern)     # [s*s*B][Nsub_padded]
    rows = np.asarray(rows, dtype=np.int64).reshape(-1, 3)
    # inverse map: (batch element, token) -> (subsequence, position); subsequence sb belongs to batch element sb % B
    inv = np.full((B, T * H * W, 2), -1, dtype=np.int64)
    for sb in range(tok_at.shape[0]):
        js = np.flatnonzero(tok_at[sb] >= 0)
        inv[sb % B, tok_at[sb, js], 0] = sb
        inv[sb % B, tok_at[sb, js], 1] = js
    assert (inv >= 0).all()  # every real token sits at exactly one position
    where = {}
    for i, (b, hd, n) in enumerate(rows):
        where.setdefault((int(inv[b, n, 0]), int(hd)), []).append((i, int(inv[b, n, 1])))
    out = np.empty((rows.shape[0], q.shape[3]), dtype=np.float64)
    for (sb, hd), lst in where.items():
        real = tok_at[sb] >= 0
        qd = dequantised_unit(q8, sq, sb, hd)[[j for _, j in lst]]
        kd = dequantised_unit(k8, sk, sb, hd)
        vcodes = oracle.e4m3_decode_array(v8[sb, :, hd, :])
        svb = sv[sb, hd, np.arange(v8.shape[1]) // BLOCK].astype(np.float64)
        sv_max = float(sv[sb, hd].max())
        S = scale * (qd @ kd.T)
        S[:, ~real] = -np.inf
        P = np.exp(S - S.max(axis=1, keepdims=True))
        P8 = e4m3_round(P * (svb / sv_max * P_GAIN)[None, :])
        out[[i for i, _ in lst]] = (P8 @ vcodes) * (sv_max / P_GAIN) / P.sum(axis=1, keepdims=True)
    return out
