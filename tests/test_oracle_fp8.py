"""Pins for the oracle's E4M3 encoder and block quantiser (CPU only)."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si


def test_e4m3_code_points_from_the_format_definition():
    """OCP FP8 E4M3: bias 7, 3 mantissa bits, max 448, subnormals in steps of 2^-9; ties go to the even mantissa."""
    cases = {0.0: 0x00, 1.0: 0x38, -1.0: 0xB8, 0.0625: 0x18, 448.0: 0x7E, 240.0: 0x77, 2.0**-9: 0x01, 2.0**-10: 0x00,
             0.0015: 0x01, 1.0625: 0x38, 1.125: 0x39, 1.1875: 0x3A, 17.0: 0x58, 18.0: 0x59, 19.0: 0x5A, -0.3: 0xAA,
             2.0**-6: 0x08, 7 * 2.0**-9: 0x07, 7.5 * 2.0**-9: 0x08, 0.9375 + 0.03125: 0x38, 416.0 + 16.0: 0x7E}
    for y, code in cases.items():
        assert oracle.e4m3_encode(y) == code, (y, hex(code), hex(oracle.e4m3_encode(y)))
    for c in range(256):
        if c & 0x7F == 0x7F:
            continue  # NaN codes
        v = oracle.e4m3_decode(c)
        assert abs(v) <= 448.0
        if c not in (0x80,):
            assert oracle.e4m3_encode(v) == c  # every finite value encodes to itself (-0 aside)


def test_e4m3_encoder_matches_torch_float8():
    """Library routine: torch's float32 -> float8_e4m3fn conversion (round to nearest even) on values inside +-448."""
    g = torch.Generator().manual_seed(0)
    vals = torch.cat([torch.randn(20000, generator=g) * 100, torch.randn(20000, generator=g), torch.randn(20000, generator=g) * 0.01,
                      torch.linspace(-448, 448, 10001)]).clamp(-448, 448).float()
    want = vals.to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle.e4m3_encode(float(v)) for v in vals.numpy()], dtype=np.uint8)
    same = (got == want) | ((got & 0x7F) == 0) & ((want & 0x7F) == 0)  # +0 / -0
    assert same.all(), np.flatnonzero(~same)[:10]


@pytest.mark.parametrize("pattern", ["token", "group"])
def test_quantize_blocks_scales_and_layout(pattern):
    B, heads, D, T, H, W, s = 2, 3, 16, 5, 8, 12, 2  # Nsub = 120 -> one partial block; use T = 11 for two blocks below
    w = si.make_shape("q", B, heads, D, T, H, W, s, seed=4)
    x = si.make_qkv(w)[2]
    xb = si.as_oracle_array(x)
    x8, scales = oracle.quantize_fp8(xb, T, H, W, s, pattern)
    xp = oracle.permute(x.float().numpy(), T, H, W, s, pattern)  # [sb][j][heads][D]
    nsub = T * H * W // (s * s)
    assert x8.shape == (s * s * B, nsub, heads, D) and scales.shape == (s * s * B, heads, (nsub + 127) // 128)
    for blk in range(scales.shape[2]):
        seg = xp[:, blk * 128 : (blk + 1) * 128]
        amax = np.abs(seg).max(axis=(1, 3))  # [sb][heads]
        assert np.array_equal(scales[:, :, blk], (amax / np.float32(448.0)).astype(np.float32))
        deq = oracle.e4m3_decode_array(x8[:, blk * 128 : (blk + 1) * 128]) * scales[:, None, :, blk, None]
        # half an E4M3 step at the top binade is 16/448 of amax; elements are within that of the original
        assert (np.abs(deq - seg) <= amax[:, None, :, None] * (16.0 / 448.0) * 1.001).all()
        # the block maximum itself maps to +-448
        assert (np.abs(oracle.e4m3_decode_array(x8[:, blk * 128 : (blk + 1) * 128])).max(axis=(1, 3)) == 448.0).all()


def test_quantize_two_blocks_and_zero_block():
    B, heads, D, T, H, W, s = 1, 1, 8, 9, 8, 8, 2  # Nsub = 144: blocks of 128 and 16
    x = torch.randn((B, T * H * W, heads, D), generator=torch.Generator().manual_seed(1)).to(torch.bfloat16)
    ids = oracle.permute(np.arange(T * H * W).reshape(1, -1, 1), T, H, W, s, "group")[0, :, 0]  # tokens of subsequence 0
    x[0, ids[128:], 0, :] = 0  # second block of subsequence 0 is all zero
    x8, scales = oracle.quantize_fp8(si.as_oracle_array(x), T, H, W, s, "group")
    assert scales.shape == (4, 1, 2)
    assert scales[0, 0, 1] == 1.0 and (x8[0, 128:, 0] & 0x7F == 0).all()
    assert scales[0, 0, 0] > 0 and scales[1, 0, 1] != 1.0


@pytest.mark.parametrize("pattern", ["token", "group"])
def test_padded_quantiser_places_zeros_at_padding_and_ignores_them_in_the_scales(pattern):
    """Any-resolution mode: a 3 x 3 grid with s = 2 is padded to 4 x 4.  In the hand-worked 4 x 4 table (tests/golden) the token-wise
    class (1, 1) holds (h, w) = (1,1), (1,3), (3,1), (3,3) and the group-wise class (1, 1) holds (2,2), (2,3), (3,2), (3,3): one real
    token followed by three padding positions in both."""
    B, heads, D, T, H, W, s = 1, 2, 8, 2, 3, 3, 2
    w = si.make_shape("qp", B, heads, D, T, H, W, s, seed=6)
    x = si.make_qkv(w)[0]
    x8, sc = oracle.quantize_fp8_padded(si.as_oracle_array(x), T, H, W, s, pattern)
    assert x8.shape == (4, T * 4, heads, D) and sc.shape == (4, heads, 1)
    real_hw = (1, 1) if pattern == "token" else (2, 2)
    xf = x.float().numpy().reshape(B, T, H, W, heads, D)
    for t in range(T):
        rows = x8[3, 4 * t:4 * t + 4]                       # class (1, 1), frame t: 4 positions
        assert not rows[1:].any()                           # padding positions: code 0
        amax = np.abs(xf[0, :, real_hw[0], real_hw[1]]).max(axis=(0, 2))   # over the class's real tokens (all frames) and channels
        for hd in range(heads):
            assert sc[3, hd, 0] == np.float32(amax[hd]) / np.float32(448.0)
            want = [oracle.e4m3_encode(float(np.float32(v) * (np.float32(448.0) / np.float32(amax[hd])))) for v in xf[0, t, real_hw[0], real_hw[1], hd]]
            assert [c & 0xFF for c in rows[0, hd]] == want or all((a & 0x7F) == 0 and (b & 0x7F) == 0 or a == b for a, b in zip(rows[0, hd], want))
    # a divisible grid: the padded quantiser is the plain one
    w2 = si.make_shape("qd", 2, 2, 16, 3, 8, 8, 2, seed=7)
    x2 = si.as_oracle_array(si.make_qkv(w2)[0])
    a8, a_s = oracle.quantize_fp8_padded(x2, 3, 8, 8, 2, pattern)
    b8, b_s = oracle.quantize_fp8(x2, 3, 8, 8, 2, pattern)
    assert np.array_equal(a8, b8) and np.array_equal(a_s, b_s)
    # H = 1 with s = 2, token-wise: the classes with p = 1 hold padding only: scale 1, all codes 0
    if pattern == "token":
        w3 = si.make_shape("q1", 1, 1, 8, 2, 1, 8, 2, seed=8)
        c8, c_s = oracle.quantize_fp8_padded(si.as_oracle_array(si.make_qkv(w3)[0]), 2, 1, 8, 2, "token")
        assert not c8[2:].any() and (c_s[2:] == 1.0).all()
