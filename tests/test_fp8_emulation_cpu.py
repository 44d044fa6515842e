"""Pins of the test-side ideal-E4M3 emulation (CPU only): it is what the GPU tests of the 8-bit variant derive their
bounds from, so it must itself rest on the oracle and on the format definition."""
import numpy as np
import pytest

import _fp8_emulation as emu
import oracle
import synth_inputs as si
from _util import errors, oracle_inputs


def test_vectorised_rounding_equals_the_oracle_codec():
    rng = np.random.default_rng(0)
    vals = np.concatenate([rng.normal(size=3000) * sc for sc in (100.0, 1.0, 0.01, 0.001)]
                          + [np.linspace(-448, 448, 2001), np.arange(64) * 2.0 ** -11, np.array([500.0, -1e6, 448.0, 464.0, 0.0])])
    want = np.array([oracle.e4m3_decode(oracle.e4m3_encode(float(np.clip(x, -448, 448)))) for x in vals])
    assert np.array_equal(emu.e4m3_round(vals), want)
    # ties go to the even mantissa: 17 lies halfway between 16 and 18, 19 between 18 and 20 (step 2 in [16, 32))
    assert list(emu.e4m3_round(np.array([17.0, 19.0, 2.0 ** -10, 3 * 2.0 ** -10]))) == [16.0, 20.0, 0.0, 2.0 ** -8]


@pytest.mark.parametrize("pattern", ["token", "group"])
def test_emulation_without_p_rounding_is_the_oracle_on_dequantised_inputs(pattern, monkeypatch):
    """With the rounding of the probabilities switched off, what is left of the recipe (block scales, the V scale folded
    into the probabilities, the gain of 16) must reproduce float64 attention on the dequantised tensors exactly."""
    B, heads, D, T, H, W, s = 2, 2, 32, 5, 8, 16, 2  # Nsub = 160: one full scale block and a partial one
    w = si.make_shape("e", B, heads, D, T, H, W, s, seed=9)
    q, k, v = si.make_qkv(w)
    v[:, ::5] *= 7.0  # uneven V scales between blocks
    arrs = oracle_inputs(q, k, v)
    qs = [oracle.quantize_fp8(a, T, H, W, s, pattern) for a in arrs]

    def deq(x8, sc):
        rep = np.repeat(sc, 128, axis=2)[:, :, : x8.shape[1]]
        return oracle.e4m3_decode_array(x8) * rep.transpose(0, 2, 1)[:, :, :, None]

    want = oracle.unpermute(oracle.attention(deq(*qs[0]), deq(*qs[1]), deq(*qs[2]), w.scale), T, H, W, s, pattern)
    with_rounding = emu.ideal_attention(*arrs, T, H, W, s, pattern, w.scale)
    monkeypatch.setattr(emu, "e4m3_round", lambda x: x)
    exact_p = emu.ideal_attention(*arrs, T, H, W, s, pattern, w.scale)
    assert np.abs(exact_p - want).max() <= 1e-12 * max(1.0, np.abs(want).max())
    # with it switched on, every probability moves by at most half an E4M3 step (2^-4 relative; far less in the sum)
    _, rl = errors(with_rounding, want)
    assert 1e-4 < rl < 3e-2
    # sampled-row mode equals the full evaluation (up to the summation order of the matrix products)
    monkeypatch.undo()
    rows = np.array([(b, hd, n) for b in range(B) for hd in range(heads) for n in (0, 77, T * H * W - 1)])
    got = emu.ideal_attention_rows(*arrs, rows, T, H, W, s, pattern, w.scale)
    assert np.allclose(got, with_rounding[rows[:, 0], rows[:, 2], rows[:, 1]], rtol=1e-9, atol=1e-12)


def test_format_floor_on_gaussian_inputs_and_with_channel_means():
    """The emulation's own error: ~5e-2 relative L2 on i.i.d. N(0,1) inputs (why the GPU tests are relative to it), far below
    2e-2 once V carries a mean."""
    B, heads, D, T, H, W, s = 1, 2, 128, 9, 16, 16, 2
    w = si.make_shape("f", B, heads, D, T, H, W, s, seed=33)
    q, k, v = si.make_qkv(w)
    exact = oracle.skiparse_attention(*oracle_inputs(q, k, v), T, H, W, s, "group", w.scale)
    _, rl = errors(emu.ideal_attention(*oracle_inputs(q, k, v), T, H, W, s, "group", w.scale), exact)
    assert 3.5e-2 < rl < 7e-2
    vm = (v.float() * 0.25 + 2.0).to(v.dtype)
    exact = oracle.skiparse_attention(*oracle_inputs(q, k, vm), T, H, W, s, "group", w.scale)
    ma, rl = errors(emu.ideal_attention(*oracle_inputs(q, k, vm), T, H, W, s, "group", w.scale), exact)
    assert rl < 1e-2 and ma < 6e-2


def test_padded_emulation_equals_the_plain_one_on_a_divisible_grid_and_masks_padding_elsewhere():
    w = si.make_shape("ep", 1, 2, 64, 3, 8, 8, 2, seed=36)
    q, k, v = si.make_qkv(w)
    rows = si.sample_rows(w, 10, seed=2)
    a = emu.ideal_attention_rows_padded(*oracle_inputs(q, k, v), rows, 3, 8, 8, 2, "group", w.scale)
    b = emu.ideal_attention_rows(*oracle_inputs(q, k, v), rows, 3, 8, 8, 2, "group", w.scale)
    assert np.array_equal(a, b)
    # a grid that needs padding: every real token sits at exactly one position, padding positions are -1
    tok = emu.padded_positions(2, 3, 5, 7, 2, "token")
    assert tok.shape == (8, 3 * 8 * 8 // 4)
    for b_ in range(2):
        real = np.sort(tok[b_::2][tok[b_::2] >= 0])
        assert np.array_equal(real, np.arange(3 * 5 * 7))
    # and the emulation stays on the format's floor there as well
    w2 = si.make_shape("ep2", 1, 2, 128, 9, 17, 21, 2, seed=35)
    q, k, v = si.make_qkv(w2)
    rows = si.sample_rows(w2, 40, seed=1)
    exact = oracle.skiparse_attention_rows_padded(*oracle_inputs(q, k, v), rows, 9, 17, 21, 2, "token", w2.scale)
    _, rl = errors(emu.ideal_attention_rows_padded(*oracle_inputs(q, k, v), rows, 9, 17, 21, 2, "token", w2.scale), exact)
    assert 3.5e-2 < rl < 7e-2
