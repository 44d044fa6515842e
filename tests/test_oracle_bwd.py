"""Pins of the oracle's backward pass (CPU only).

The gradient formulas in oracle/skiparse_oracle.c are checked against things other than themselves:
  * reverse-mode differentiation by torch.autograd of the plain float64 expression softmax(q k^T * scale) v,
  * central finite differences of the oracle's own FORWARD (pinned separately) along random directions,
  * closed forms (one key; identical keys) and invariants (rows of dS sum to zero, rows of P to one),
  * for the sparse layer: autograd through a dense N x N attention with the class mask written from the class
    formulas of Sec. 3.1 (no rearrangement involved), both patterns,
  * the one-unit sampled mode against the full gradient.
"""
import numpy as np
import pytest
import torch

import oracle

RNG = np.random.default_rng(7)


def _rand(*shape):
    return RNG.standard_normal(shape)


def _autograd_attention(q, k, v, dout, scale, mask=None):
    """(dq, dk, dv) of sum(out * dout), out = softmax(q k^T * scale [+ mask]) v per (batch, head); [nb][n][heads][D]."""
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    s = torch.einsum("bihd,bjhd->bhij", tq, tk) * scale
    if mask is not None:
        s = s + torch.tensor(mask, dtype=torch.float64)[None, None]
    out = torch.einsum("bhij,bjhd->bihd", torch.softmax(s, dim=-1), tv)
    (out * torch.tensor(dout, dtype=torch.float64)).sum().backward()
    return tq.grad.numpy(), tk.grad.numpy(), tv.grad.numpy()


@pytest.mark.parametrize("nb,n,heads,D,scale", [(2, 7, 3, 5, 0.37), (1, 33, 2, 16, 0.25), (3, 1, 1, 4, 1.0)])
def test_attention_bwd_matches_autograd(nb, n, heads, D, scale):
    q, k, v, dout = (_rand(nb, n, heads, D) for _ in range(4))
    got = oracle.attention_bwd(q, k, v, dout, scale)
    want = _autograd_attention(q, k, v, dout, scale)
    for g, w, name in zip(got, want, "qkv"):
        np.testing.assert_allclose(g, w, rtol=1e-9, atol=1e-11, err_msg=f"d{name}")


def test_attention_bwd_matches_finite_differences_of_the_forward():
    nb, n, heads, D, scale = 1, 9, 2, 6, 0.6
    q, k, v, dout = (_rand(nb, n, heads, D) for _ in range(4))
    dq, dk, dv = oracle.attention_bwd(q, k, v, dout, scale)
    loss = lambda a, b, c: float((oracle.attention(a, b, c, scale) * dout).sum())
    eps = 1e-5
    for which, grad in enumerate((dq, dk, dv)):
        for _ in range(3):
            u = _rand(nb, n, heads, D)
            args_p, args_m = [q, k, v], [q, k, v]
            args_p[which] = args_p[which] + eps * u
            args_m[which] = args_m[which] - eps * u
            fd = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            assert abs(fd - float((grad * u).sum())) <= 1e-7 * max(1.0, abs(fd)), which


def test_closed_forms():
    # one key: P = 1, so dv = dout and the logits do not matter
    q, k, v, dout = (_rand(2, 1, 2, 4) for _ in range(4))
    dq, dk, dv = oracle.attention_bwd(q, k, v, dout, 0.5)
    np.testing.assert_array_equal(dq, 0.0)
    np.testing.assert_array_equal(dk, 0.0)
    np.testing.assert_allclose(dv, dout, rtol=0, atol=1e-15)
    # identical keys: P = 1/n everywhere -> dv_j = mean_i dout_i, dq = 0 (all keys pull the same way),
    # dk_j = scale/n * sum_i (dP_ij - mean_j' dP_ij') q_i
    n, D, scale = 6, 3, 0.8
    q, v, dout = (_rand(1, n, 1, D) for _ in range(3))
    k = np.repeat(_rand(1, 1, 1, D), n, axis=1)
    dq, dk, dv = oracle.attention_bwd(q, k, v, dout, scale)
    np.testing.assert_allclose(dv[0, :, 0], np.repeat(dout[0, :, 0].mean(0, keepdims=True), n, 0), rtol=1e-12)
    dP = dout[0, :, 0] @ v[0, :, 0].T                   # [i][j]
    dS = (dP - dP.mean(1, keepdims=True)) / n
    np.testing.assert_allclose(dk[0, :, 0], scale * dS.T @ q[0, :, 0], rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(dq[0, :, 0], scale * dS @ k[0, :, 0], rtol=1e-10, atol=1e-13)
    assert np.abs(dq).max() < 1e-12                     # rows of dS sum to zero and all keys are equal


def test_invariants():
    nb, n, heads, D = 2, 11, 2, 8
    q, k, v, dout = (_rand(nb, n, heads, D) for _ in range(4))
    dq, dk, dv = oracle.attention_bwd(q, k, v, dout, 0.3)
    # rows of dS sum to zero, so sum_j dk_j = scale * sum_i (sum_j dS_ij) q_i = 0
    np.testing.assert_allclose(dk.sum(axis=1), 0.0, atol=1e-12)
    # rows of P sum to one: sum_j dv_j = sum_i dout_i
    np.testing.assert_allclose(dv.sum(axis=1), dout.sum(axis=1), rtol=1e-12, atol=1e-12)
    # shifting all values by a constant vector shifts every output row by it: dq and dk do not depend on it
    dq2, dk2, _ = oracle.attention_bwd(q, k, v + 3.0, dout, 0.3)
    np.testing.assert_allclose(dq2, dq, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(dk2, dk, rtol=1e-9, atol=1e-11)


def _class_mask(T, H, W, s, pattern):
    """0 where two tokens share a subsequence, -inf elsewhere, from the class formulas of Sec. 3.1."""
    n = np.arange(T * H * W)
    h, w = (n // W) % H, n % W
    cls = (h % s) * s + (w % s) if pattern == "token" else ((h // s) % s) * s + ((w // s) % s)
    return np.where(cls[:, None] == cls[None, :], 0.0, -np.inf)


@pytest.mark.parametrize("pattern", ["token", "group"])
@pytest.mark.parametrize("B,heads,D,T,H,W,s", [(2, 2, 4, 2, 4, 8, 2), (1, 1, 3, 1, 9, 9, 3)])
def test_skiparse_bwd_matches_autograd_through_masked_dense_attention(B, heads, D, T, H, W, s, pattern):
    N = T * H * W
    q, k, v, dout = (_rand(B, N, heads, D) for _ in range(4))
    got = oracle.skiparse_attention_bwd(q, k, v, dout, T, H, W, s, pattern, 0.45)
    want = _autograd_attention(q, k, v, dout, 0.45, mask=_class_mask(T, H, W, s, pattern))
    for g, w_, name in zip(got, want, "qkv"):
        np.testing.assert_allclose(g, w_, rtol=1e-9, atol=1e-11, err_msg=f"d{name}")


def test_skiparse_bwd_s1_is_dense_bwd_and_bf16_inputs_are_widened_exactly():
    B, heads, D, T, H, W = 1, 2, 8, 1, 3, 5
    q, k, v, dout = (torch.randn(B, T * H * W, heads, D, generator=torch.Generator().manual_seed(i)).to(torch.bfloat16) for i in range(4))
    bits = [t.view(torch.int16).numpy().view(np.uint16) for t in (q, k, v, dout)]
    wide = [t.to(torch.float64).numpy() for t in (q, k, v, dout)]
    a = oracle.skiparse_attention_bwd(*bits, T, H, W, 1, "token", 0.3)
    b = oracle.attention_bwd(*wide, 0.3)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)


@pytest.mark.parametrize("pattern", ["token", "group"])
def test_unit_mode_matches_full_gradient(pattern):
    B, heads, D, T, H, W, s = 2, 3, 4, 2, 8, 8, 2
    N = T * H * W
    q, k, v, dout = (_rand(B, N, heads, D) for _ in range(4))
    full = oracle.skiparse_attention_bwd(q, k, v, dout, T, H, W, s, pattern, 0.5)
    b, head = 1, 2
    n0 = 37
    p0, q0, _ = oracle.dst_index(pattern, s, T, H, W, n0)
    toks = [n0] + [oracle.src_index(pattern, s, T, H, W, p0, q0, j) for j in (0, 5, N // (s * s) - 1) if oracle.src_index(pattern, s, T, H, W, p0, q0, j) != n0]
    got = oracle.skiparse_attention_bwd_unit(q, k, v, dout, b, head, toks, T, H, W, s, pattern, 0.5)
    for g, f in zip(got, full):
        np.testing.assert_allclose(g, f[b, toks, head], rtol=1e-10, atol=1e-13)
    # a token of another subsequence is rejected
    other = oracle.src_index(pattern, s, T, H, W, (p0 + 1) % s, q0, 0)
    with pytest.raises(ValueError):
        oracle.skiparse_attention_bwd_unit(q, k, v, dout, b, head, [n0, other], T, H, W, s, pattern, 0.5)


@pytest.mark.parametrize("pattern", ["token", "group"])
@pytest.mark.parametrize("B,heads,D,T,H,W,s", [(2, 2, 4, 2, 5, 7, 2), (1, 1, 3, 1, 7, 10, 3), (1, 2, 4, 1, 1, 1, 2)])
def test_padded_bwd_matches_autograd_through_masked_dense_attention(B, heads, D, T, H, W, s, pattern):
    """Any-resolution mode: grids that are not multiples of s*s.  The class mask needs no divisibility."""
    N = T * H * W
    q, k, v, dout = (_rand(B, N, heads, D) for _ in range(4))
    got = oracle.skiparse_attention_bwd_padded(q, k, v, dout, T, H, W, s, pattern, 0.45)
    want = _autograd_attention(q, k, v, dout, 0.45, mask=_class_mask(T, H, W, s, pattern))
    for g, w_, name in zip(got, want, "qkv"):
        np.testing.assert_allclose(g, w_, rtol=1e-9, atol=1e-11, err_msg=f"d{name}")


@pytest.mark.parametrize("pattern", ["token", "group"])
def test_padded_bwd_equals_plain_bwd_on_divisible_grids_and_unit_mode(pattern):
    B, heads, D, T, H, W, s = 2, 2, 4, 2, 8, 4, 2
    N = T * H * W
    q, k, v, dout = (_rand(B, N, heads, D) for _ in range(4))
    a = oracle.skiparse_attention_bwd_padded(q, k, v, dout, T, H, W, s, pattern, 0.5)
    b = oracle.skiparse_attention_bwd(q, k, v, dout, T, H, W, s, pattern, 0.5)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y, rtol=1e-11, atol=1e-13)
    # one unit of a non-divisible grid against the full padded gradient
    T, H, W = 2, 7, 9
    N = T * H * W
    q, k, v, dout = (_rand(B, N, heads, D) for _ in range(4))
    full = oracle.skiparse_attention_bwd_padded(q, k, v, dout, T, H, W, s, pattern, 0.5)
    mask = _class_mask(T, H, W, s, pattern)
    n0 = 40
    members = [int(n) for n in np.nonzero(mask[n0] == 0.0)[0]]
    toks = [n0, members[0], members[-1]] if members[0] != n0 and members[-1] != n0 else [n0, members[1]]
    got = oracle.skiparse_attention_bwd_unit_padded(q, k, v, dout, 1, 0, toks, T, H, W, s, pattern, 0.5)
    for g, f in zip(got, full):
        np.testing.assert_allclose(g, f[1, toks, 0], rtol=1e-10, atol=1e-13)
    other = int(np.nonzero(mask[n0] != 0.0)[0][0])
    with pytest.raises(ValueError):
        oracle.skiparse_attention_bwd_unit_padded(q, k, v, dout, 1, 0, [n0, other], T, H, W, s, pattern, 0.5)
