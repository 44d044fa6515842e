"""GPU parity: skiparse_permute / skiparse_unpermute through the C ABI against the oracle, byte for byte."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si

pytestmark = pytest.mark.gpu

CASES = [  # B, heads, D, T, H, W, s, torch dtype
    (1, 2, 64, 2, 8, 8, 2, torch.float32),      # the tiny workload's grid, fp32 rows of 512 B
    (2, 3, 128, 3, 8, 12, 2, torch.bfloat16),
    (1, 5, 128, 2, 9, 18, 3, torch.bfloat16),   # s = 3
    (3, 1, 64, 1, 16, 32, 4, torch.bfloat16),   # s = 4, short rows (128 B)
    (2, 40, 128, 1, 4, 8, 2, torch.bfloat16),   # 10 KiB rows as at the 768P shape
    (2, 2, 64, 2, 3, 5, 1, torch.bfloat16),     # s = 1: plain copy
    (1, 7, 128, 2, 8, 8, 2, torch.uint8),       # one-byte elements, 896-byte rows (ragged tail of 16-byte chunks)
]


def _random_bits(shape, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    nbytes = int(np.prod(shape)) * torch.empty((), dtype=dtype).element_size()
    raw = torch.randint(0, 256, (nbytes,), generator=g, dtype=torch.uint8)
    return raw.view(dtype).reshape(shape)


@pytest.mark.parametrize("B,heads,D,T,H,W,s,dtype", CASES)
@pytest.mark.parametrize("pattern", ["token", "group"])
def test_permute_roundtrip_bit_exact(B, heads, D, T, H, W, s, dtype, pattern):
    import paper_2605_28691_amd as sk

    if pattern == "group" and (H % (s * s) or W % (s * s)):
        pytest.skip("group-wise needs multiples of s^2")
    x = _random_bits((B, T * H * W, heads, D), dtype, seed=B * 100 + s)
    xb = x.view(torch.uint8).reshape(B, T * H * W, -1).numpy()
    want = oracle.permute(xb, T, H, W, s, pattern)
    xd = x.cuda()
    yd = sk.skiparse_permute(xd, T, H, W, s, pattern)
    got = yd.cpu().view(torch.uint8).reshape(want.shape).numpy()
    assert np.array_equal(got, want)
    back = sk.skiparse_unpermute(yd, T, H, W, s, pattern)
    assert torch.equal(back.cpu().view(torch.uint8), x.view(torch.uint8))
    # unpermute on its own, from the oracle's permuted bytes
    yo = torch.from_numpy(want).view(dtype).reshape(yd.shape).cuda()
    assert torch.equal(sk.skiparse_unpermute(yo, T, H, W, s, pattern).cpu().view(torch.uint8), x.view(torch.uint8))


@pytest.mark.parametrize("name", ["480p", "768p"])
def test_permute_full_size(name):
    """The benchmark shapes in full, every byte compared (bf16 rows of 3 KiB / 10 KiB)."""
    import paper_2605_28691_amd as sk

    w = si.WORKLOADS[name]
    g = torch.Generator().manual_seed(w.seed)
    x = torch.randint(-32768, 32767, (w.B, w.N, w.heads, w.D), generator=g, dtype=torch.int16).view(torch.bfloat16)
    xd = x.cuda()
    for pattern in w.patterns:
        want = oracle.permute(x.view(torch.int16).numpy(), w.T, w.H, w.W, w.s, pattern)
        yd = sk.skiparse_permute(xd, w.T, w.H, w.W, w.s, pattern)
        assert torch.equal(yd.cpu().view(torch.int16), torch.from_numpy(want))
        back = sk.skiparse_unpermute(yd, w.T, w.H, w.W, w.s, pattern)
        assert torch.equal(back.view(torch.int16), xd.view(torch.int16))
        del yd, back, want


def test_permute_does_not_touch_neighbouring_memory():
    """Canary bytes around the destination stay intact."""
    import paper_2605_28691_amd as sk

    B, heads, D, T, H, W, s = 1, 3, 64, 2, 8, 8, 2
    n = B * T * H * W * heads * D
    x = torch.randn((B, T * H * W, heads, D)).to(torch.bfloat16).cuda()
    buf = torch.full((n + 4096,), 7.0, dtype=torch.bfloat16, device="cuda")
    out = buf[2048 : 2048 + n].view(s * s * B, T * H * W // (s * s), heads, D)
    sk.skiparse_permute(x, T, H, W, s, "group", out=out)
    torch.cuda.synchronize()
    assert (buf[:2048] == 7.0).all() and (buf[2048 + n :] == 7.0).all()


@pytest.mark.parametrize("B,heads,D,T,H,W,s,dtype", [
    (1, 2, 64, 2, 8, 8, 2, torch.float32),
    (2, 3, 128, 3, 8, 12, 2, torch.bfloat16),
    (1, 5, 128, 2, 9, 18, 3, torch.bfloat16),
    (3, 1, 64, 1, 16, 32, 4, torch.bfloat16),
    (1, 7, 128, 2, 8, 8, 2, torch.uint8),
    (2, 2, 64, 2, 3, 5, 1, torch.bfloat16),
])
@pytest.mark.parametrize("from_pattern", ["token", "group"])
def test_switch_pattern_bit_exact(B, heads, D, T, H, W, s, dtype, from_pattern):
    """skiparse_switch_pattern against the oracle's composition unpermute(from) -> permute(other), byte for byte."""
    import paper_2605_28691_amd as sk

    y = _random_bits((s * s * B, T * H * W // (s * s), heads, D), dtype, seed=7 * B + s)
    yb = y.view(torch.uint8).reshape(y.shape[0], y.shape[1], -1).numpy()
    want = oracle.switch_pattern(yb, T, H, W, s, from_pattern)
    got = sk.skiparse_switch_pattern(y.cuda(), T, H, W, s, from_pattern)
    assert np.array_equal(got.cpu().view(torch.uint8).reshape(want.shape).numpy(), want)


def test_switch_pattern_768p_equals_two_step():
    """At the 768P shape: the one-step switch equals unpermute + permute done by the library itself (both already checked
    against the oracle), in both directions."""
    import paper_2605_28691_amd as sk

    w = si.WORKLOADS["768p"]
    g = torch.Generator(device="cuda").manual_seed(3)
    x = torch.randint(-32768, 32767, (w.B, w.N, w.heads, w.D), generator=g, dtype=torch.int16, device="cuda").view(torch.bfloat16)
    tsa = sk.skiparse_permute(x, w.T, w.H, w.W, w.s, "token")
    gsa = sk.skiparse_permute(x, w.T, w.H, w.W, w.s, "group")
    assert torch.equal(sk.skiparse_switch_pattern(tsa, w.T, w.H, w.W, w.s, "token").view(torch.int16), gsa.view(torch.int16))
    assert torch.equal(sk.skiparse_switch_pattern(gsa, w.T, w.H, w.W, w.s, "group").view(torch.int16), tsa.view(torch.int16))
