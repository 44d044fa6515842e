"""Pins for the oracle's index maps and permute/unpermute (CPU only).

Every check here compares the oracle's closed-form index arithmetic with something that is not that
arithmetic: hand-worked tables, a reshape/transpose formulation of Algorithm 1's axis splits, a
library routine (pixel_unshuffle), or an invariant the paper states.
"""
import os

import numpy as np
import pytest
import torch

import oracle

SHAPES = [  # B, T, H, W, s
    (1, 2, 8, 8, 2),
    (2, 3, 8, 12, 2),
    (1, 2, 9, 18, 3),
    (2, 1, 16, 16, 2),
    (3, 2, 4, 8, 1),
    (1, 1, 16, 32, 4),
]


def _token_ids(B, T, H, W, extra=()):
    N = T * H * W
    x = np.arange(B * N, dtype=np.int64).reshape((B, N) + (1,) * len(extra))
    return x


def _parse_golden(path):
    rows = []
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            head, vals = line.split(":")
            rows.append((head.split(), [int(v) for v in vals.split()]))
    return rows


@pytest.mark.parametrize("fname,H", [("rearrange_4x4_s2.txt", 4), ("rearrange_8x8_s2.txt", 8)])
def test_golden_tables_s2(golden_dir, fname, H):
    """Alg. 1 worked by hand on 4x4 and 8x8 grids, P=2."""
    x = _token_ids(1, 1, H, H)
    for (pattern, p, q), want in _parse_golden(os.path.join(golden_dir, fname)):
        y = oracle.permute(x, 1, H, H, 2, pattern)
        sb = int(p) * 2 + int(q)
        assert y[sb, :].tolist() == want, (pattern, p, q)
        for j, n in enumerate(want):
            assert oracle.src_index(pattern, 2, 1, H, H, int(p), int(q), j) == n
            assert oracle.dst_index(pattern, 2, 1, H, H, n) == (int(p), int(q), j)


def test_golden_table_s3_batch2(golden_dir):
    """P=3, two frames, batch of two: checks the (p q b) batch order and the frame stride."""
    B, T, H, W, s = 2, 2, 9, 9, 3
    x = _token_ids(B, T, H, W)
    for (pattern, _, sb), want in _parse_golden(os.path.join(golden_dir, "rearrange_2x3x9x9_s3.txt")):
        y = oracle.permute(x, T, H, W, s, pattern)
        b = int(sb) % B
        assert (y[int(sb), :] - b * T * H * W).tolist() == want, (pattern, sb)


def _reshape_formulation(x, T, H, W, s, pattern):
    """Algorithm 1's axis splits done with reshape/transpose instead of index arithmetic.

    token-wise: h = (h_s, p), w = (w_s, q); group-wise: h = (h_o, p, h_i), w = (w_o, q, w_i);
    the (p, q) axes move in front of the batch axis, everything else keeps its order.
    """
    B, N, C = x.shape
    if pattern == "token":
        a = x.reshape(B, T, H // s, s, W // s, s, C)  # b t hs p ws q c
        a = a.transpose(3, 5, 0, 1, 2, 4, 6)  # p q b t hs ws c
    else:
        a = x.reshape(B, T, H // (s * s), s, s, W // (s * s), s, s, C)  # b t ho p hi wo q wi c
        a = a.transpose(3, 6, 0, 1, 2, 4, 5, 7, 8)  # p q b t ho hi wo wi c
    return np.ascontiguousarray(a).reshape(s * s * B, N // (s * s), C)


@pytest.mark.parametrize("B,T,H,W,s", SHAPES)
@pytest.mark.parametrize("pattern", ["token", "group"])
def test_permute_matches_reshape_formulation(B, T, H, W, s, pattern):
    if pattern == "group" and (H % (s * s) or W % (s * s)):
        pytest.skip("group-wise needs multiples of s^2")
    rng = np.random.default_rng(5)
    x = rng.standard_normal((B, T * H * W, 3)).astype(np.float32)
    y = oracle.permute(x, T, H, W, s, pattern)
    assert np.array_equal(y, _reshape_formulation(x, T, H, W, s, pattern))


@pytest.mark.parametrize("B,T,H,W,s", SHAPES)
def test_token_wise_is_pixel_unshuffle_into_batch(B, T, H, W, s):
    """Sec. 3.1: token-wise rearrange is pixel-unshuffle with the sub-figures stacked on the batch axis."""
    C = 5
    rng = np.random.default_rng(6)
    x = rng.standard_normal((B, T * H * W, C)).astype(np.float32)
    img = torch.from_numpy(x).reshape(B, T, H, W, C).permute(0, 1, 4, 2, 3).reshape(B * T * C, 1, H, W)
    un = torch.nn.functional.pixel_unshuffle(img, s)  # (B*T*C, s*s, H/s, W/s); channel = p*s + q
    un = un.reshape(B, T, C, s * s, H // s, W // s).permute(3, 0, 1, 4, 5, 2).reshape(s * s * B, -1, C)
    assert np.array_equal(oracle.permute(x, T, H, W, s, "token"), un.numpy())


@pytest.mark.parametrize("B,T,H,W,s", SHAPES)
@pytest.mark.parametrize("pattern", ["token", "group"])
def test_classes_in_raster_order(B, T, H, W, s, pattern):
    """A subsequence is exactly the set of tokens of one spatial class, kept in raster order, and all
    subsequences have the same length (Sec. 3.1 class ids; Sec. 3.3 equal lengths)."""
    if pattern == "group" and (H % (s * s) or W % (s * s)):
        pytest.skip("group-wise needs multiples of s^2")
    N = T * H * W
    y = oracle.permute(_token_ids(B, T, H, W), T, H, W, s, pattern)
    assert y.shape == (s * s * B, N // (s * s))
    n = np.arange(N)
    h, w = (n // W) % H, n % W
    cls = (h % s) * s + (w % s) if pattern == "token" else ((h // s) % s) * s + ((w // s) % s)
    for c in range(s * s):
        members = n[cls == c]  # already in raster order
        for b in range(B):
            assert np.array_equal(y[c * B + b], members + b * N)


@pytest.mark.parametrize("B,T,H,W,s", SHAPES)
@pytest.mark.parametrize("pattern", ["token", "group"])
def test_inverse_and_bijection(B, T, H, W, s, pattern):
    if pattern == "group" and (H % (s * s) or W % (s * s)):
        pytest.skip("group-wise needs multiples of s^2")
    rng = np.random.default_rng(7)
    x = rng.integers(0, 2**16, size=(B, T * H * W, 2, 4), dtype=np.uint16)
    y = oracle.permute(x, T, H, W, s, pattern)
    assert np.array_equal(oracle.unpermute(y, T, H, W, s, pattern), x)
    ids = oracle.permute(_token_ids(B, T, H, W), T, H, W, s, pattern)
    assert np.array_equal(np.sort(ids.ravel()), np.arange(B * T * H * W))
    N = T * H * W
    for n in rng.integers(0, N, size=50):
        p, q, j = oracle.dst_index(pattern, s, T, H, W, int(n))
        assert oracle.src_index(pattern, s, T, H, W, p, q, j) == n


@pytest.mark.parametrize("pattern", ["token", "group"])
@pytest.mark.parametrize("s", [2, 3])
def test_local_equivalence(pattern, s):
    """Sec. 3.2: rearranging the H x W figure equals rearranging every s^2 x s^2 tile on its own; the
    class of a token and its position among its tile's class members depend only on the tile-local coordinates."""
    u = s * s
    T, H, W = 2, 2 * u, 3 * u
    for n in range(T * H * W):
        t, h, w = n // (H * W), (n // W) % H, n % W
        p, q, j = oracle.dst_index(pattern, s, T, H, W, n)
        pl, ql, jl = oracle.dst_index(pattern, s, 1, u, u, (h % u) * u + (w % u))
        assert (p, q) == (pl, ql)
        hs, ws = (j // (W // s)) % (H // s), j % (W // s)
        assert (hs, ws) == ((h // u) * s + jl // s, (w // u) * s + jl % s)
        assert j // ((H // s) * (W // s)) == t


@pytest.mark.parametrize("s,H,W", [(2, 8, 8), (2, 4, 12), (3, 9, 18)])
def test_two_hop_connectivity_and_density(s, H, W):
    """Sec. 3.1 / Fig. 1: any two tokens are connected by one token-wise step followed by one group-wise step;
    each pattern's same-class mask has density 1/s^2."""
    N = H * W
    masks = {}
    for pattern in ("token", "group"):
        cls = np.array([oracle.dst_index(pattern, s, 1, H, W, n)[:2] for n in range(N)])
        cid = cls[:, 0] * s + cls[:, 1]
        masks[pattern] = cid[:, None] == cid[None, :]
        assert masks[pattern].mean() == pytest.approx(1.0 / (s * s))
    reach = (masks["token"].astype(np.int64) @ masks["group"].astype(np.int64)) > 0
    assert reach.all()


def test_s1_is_identity():
    x = np.random.default_rng(8).standard_normal((2, 24, 4)).astype(np.float32)
    for pattern in ("token", "group"):
        assert np.array_equal(oracle.permute(x, 2, 3, 4, 1, pattern), x)


def test_bad_shapes_rejected():
    x = np.zeros((1, 2 * 6 * 8, 1), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.permute(x, 2, 6, 8, 2, "group")  # 6 is not a multiple of 4
    with pytest.raises(ValueError):
        oracle.permute(np.zeros((1, 2 * 5 * 8, 1), dtype=np.float32), 2, 5, 8, 2, "token")
    oracle.permute(x, 2, 6, 8, 2, "token")  # multiples of s are enough for token-wise


@pytest.mark.parametrize("B,T,H,W,s", [(1, 2, 8, 8, 2), (2, 3, 8, 12, 2), (1, 2, 9, 18, 3), (2, 1, 16, 32, 4)])
def test_switch_pattern_matches_reshape_formulation(B, T, H, W, s):
    """Alg. 1, tsa_to_gsa / gsa_to_tsa as axis moves: in the token-wise layout the class is (h%s, w%s) = (p2, q2) and the
    position splits as (t, h_o, p1, w_o, q1); the group-wise layout has class (p1, q1) and position (t, h_o, p2, w_o, q2)."""
    rng = np.random.default_rng(9)
    N = T * H * W
    x = rng.standard_normal((B, N, 3)).astype(np.float32)
    tsa = oracle.permute(x, T, H, W, s, "token")
    gsa = oracle.permute(x, T, H, W, s, "group")
    u = s * s
    a = tsa.reshape(s, s, B, T, H // u, s, W // u, s, 3)           # p2 q2 b t ho p1 wo q1 c
    want_gsa = np.ascontiguousarray(a.transpose(5, 7, 2, 3, 4, 0, 6, 1, 8)).reshape(u * B, N // u, 3)  # p1 q1 b t ho p2 wo q2 c
    assert np.array_equal(want_gsa, gsa)
    assert np.array_equal(oracle.switch_pattern(tsa, T, H, W, s, "token"), gsa)
    assert np.array_equal(oracle.switch_pattern(gsa, T, H, W, s, "group"), tsa)
