"""GPU parity: dense_attn_fwd and skiparse_attn_fwd (fused and unfused) through the C ABI against the float64 oracle.

Tolerance (bf16 path): max |diff| <= 2e-2 and relative L2 error <= 5e-3 on the compared rows.
"""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from _util import assert_close_bf16, gather_rows, oracle_inputs, to_np64

pytestmark = pytest.mark.gpu

SMALL = [  # B, heads, D, T, H, W, s -- several query/key tiles and ragged tails (tiles are 128 queries x 64 keys)
    (1, 2, 64, 2, 8, 8, 2),      # the tiny workload's shape: 32 tokens per subsequence, a single partial tile
    (2, 3, 128, 3, 8, 12, 2),    # Nsub = 72: partial query tile, one full + one partial key tile
    (1, 2, 128, 5, 16, 20, 2),   # Nsub = 400: 4 query tiles, 7 key tiles, tail of 16
    (2, 2, 64, 5, 16, 20, 2),    # same with head_dim 64 and a batch of 2
    (1, 9, 128, 4, 9, 18, 3),    # s = 3, 9 heads (unit count not a multiple of 8)
    (1, 1, 128, 1, 16, 48, 4),   # s = 4: 16 subsequences of 48 tokens
    (1, 2, 128, 7, 16, 16, 2),   # Nsub = 448 = 7 * 64: no key tail
    (1, 1, 64, 9, 24, 28, 2),    # Nsub = 1512: 24 key tiles, more than the 16 slots of the row-offset ring, tail of 40
    (2, 2, 64, 1, 2, 2, 2),      # one token per subsequence (token-wise only): out = v
]


def _gpu(ts):
    return tuple(t.cuda() for t in ts)


@pytest.mark.parametrize("B,heads,D,T,H,W,s", SMALL)
@pytest.mark.parametrize("pattern", ["token", "group"])
@pytest.mark.parametrize("fused", [True, False])
def test_skiparse_attention_small(B, heads, D, T, H, W, s, pattern, fused):
    import paper_2605_28691_amd as sk

    if pattern == "group" and (H % (s * s) or W % (s * s)):
        pytest.skip("group-wise needs multiples of s^2")
    w = si.make_shape("small", B, heads, D, T, H, W, s, seed=11 + s)
    q, k, v = si.make_qkv(w)
    want = oracle.skiparse_attention(*oracle_inputs(q, k, v), T, H, W, s, pattern, w.scale)
    out = sk.skiparse_attn_fwd(*_gpu((q, k, v)), T, H, W, s, pattern, scale=w.scale, fused=fused)
    assert_close_bf16(to_np64(out), want, f"{pattern} fused={fused}")


@pytest.mark.parametrize("B,heads,D,N", [(1, 2, 128, 1000), (2, 3, 64, 333), (1, 1, 128, 64), (1, 1, 64, 1), (1, 8, 128, 130)])
def test_dense_attention_small(B, heads, D, N):
    import paper_2605_28691_amd as sk

    w = si.make_shape("dense", B, heads, D, 1, 1, N, 1, seed=N)
    q, k, v = si.make_qkv(w)
    want = oracle.attention(*oracle_inputs(q, k, v), w.scale)
    out = sk.dense_attn_fwd(*_gpu((q, k, v)), 1, 1, N, scale=0.0)  # scale <= 0 selects 1/sqrt(D)
    assert_close_bf16(to_np64(out), want, "dense")


def test_tiny_workload_both_patterns_and_s1():
    """BASELINE tiny case on the GPU (values rounded to bf16 once; the oracle sees the same rounded values):
    both patterns against the oracle, and s = 1 equals dense attention bit for bit (same kernel, same order)."""
    import paper_2605_28691_amd as sk

    w = si.WORKLOADS["tiny"]
    q, k, v = (t.to(torch.bfloat16) for t in si.make_qkv(w))
    qd, kd, vd = _gpu((q, k, v))
    for pattern in w.patterns:
        want = oracle.skiparse_attention(*oracle_inputs(q, k, v), w.T, w.H, w.W, w.s, pattern, w.scale)
        brute = oracle.masked_dense_attention(*oracle_inputs(q, k, v), w.T, w.H, w.W, w.s, pattern, w.scale)
        for fused in (True, False):
            out = to_np64(sk.skiparse_attn_fwd(qd, kd, vd, w.T, w.H, w.W, w.s, pattern, fused=fused))
            assert_close_bf16(out, want, f"tiny {pattern}")
            assert_close_bf16(out, brute, f"tiny {pattern} vs masked dense")
    dense = sk.dense_attn_fwd(qd, kd, vd, w.T, w.H, w.W)
    for pattern in w.patterns:
        assert torch.equal(sk.skiparse_attn_fwd(qd, kd, vd, w.T, w.H, w.W, 1, pattern, fused=True), dense)
    assert_close_bf16(to_np64(dense), oracle.attention(*oracle_inputs(q, k, v), w.scale), "tiny dense")


def test_peaky_and_shifted_logits():
    """Large logits with a large common offset: exercises the running-maximum updates (early keys small, late keys large)."""
    import paper_2605_28691_amd as sk

    B, heads, D, N = 1, 2, 128, 700
    g = torch.Generator().manual_seed(5)
    q = torch.randn((B, N, heads, D), generator=g)
    k = torch.randn((B, N, heads, D), generator=g)
    v = torch.randn((B, N, heads, D), generator=g)
    ramp = torch.linspace(0.2, 3.0, N).view(1, N, 1, 1)  # later keys have larger norm -> the maximum keeps growing
    k = k * ramp
    q, k, v = (t.to(torch.bfloat16) for t in (q, k, v))
    want = oracle.attention(*oracle_inputs(q, k, v), 1.0)  # scale 1: logits of order +-100
    out = sk.dense_attn_fwd(*_gpu((q, k, v)), 1, 1, N, scale=1.0)
    assert_close_bf16(to_np64(out), want, "peaky")


def test_run_to_run_determinism_and_canaries():
    import paper_2605_28691_amd as sk

    B, heads, D, T, H, W, s = 1, 3, 128, 3, 16, 16, 2
    w = si.make_shape("det", B, heads, D, T, H, W, s, seed=3)
    qd, kd, vd = _gpu(si.make_qkv(w))
    n = qd.numel()
    buf = torch.full((n + 8192,), 3.0, dtype=torch.bfloat16, device="cuda")
    out = buf[4096 : 4096 + n].view_as(qd)
    sk.skiparse_attn_fwd(qd, kd, vd, T, H, W, s, "group", fused=True, out=out)
    first = out.clone()
    for _ in range(3):
        sk.skiparse_attn_fwd(qd, kd, vd, T, H, W, s, "group", fused=True, out=out)
        assert torch.equal(out, first)
    assert (buf[:4096] == 3.0).all() and (buf[4096 + n :] == 3.0).all()


@pytest.mark.parametrize("name", ["480p", "768p"])
def test_benchmark_shapes_sampled_rows(name):
    """The benchmark shapes in the launch configuration bench.py times: sampled query rows in every (batch, head)
    against the oracle, fused and unfused, plus one contiguous block of rows that includes the ragged last tile."""
    import paper_2605_28691_amd as sk

    w = si.WORKLOADS[name]
    q, k, v = si.make_qkv(w)
    oq, ok_, ov = oracle_inputs(q, k, v)
    qd, kd, vd = _gpu((q, k, v))
    rows = si.sample_rows(w, 64, seed=w.seed)
    tail = np.array([(0, w.heads - 1, n) for n in range(w.N - 96, w.N)], dtype=np.int64)
    rows = np.concatenate([rows, tail])
    for pattern in w.patterns:
        want = oracle.skiparse_attention_rows(oq, ok_, ov, rows, w.T, w.H, w.W, w.s, pattern, w.scale)
        for fused in (True, False):
            out = sk.skiparse_attn_fwd(qd, kd, vd, w.T, w.H, w.W, w.s, pattern, scale=w.scale, fused=fused)
            torch.cuda.synchronize()
            assert_close_bf16(gather_rows(out, rows), want, f"{name} {pattern} fused={fused}")
            del out


def test_768p_no_leakage_full_tensor():
    """Property at full size: with V constant inside every subsequence the output equals that constant in every row
    (softmax rows sum to one and nothing crosses subsequences); checked over the whole 80,640 x 40 x 128 tensor."""
    import paper_2605_28691_amd as sk

    w = si.WORKLOADS["768p"]
    g = torch.Generator(device="cuda").manual_seed(1)
    shape = (w.B, w.N, w.heads, w.D)
    qd = torch.randn(shape, generator=g, device="cuda", dtype=torch.bfloat16)
    kd = torch.randn(shape, generator=g, device="cuda", dtype=torch.bfloat16)
    for pattern in w.patterns:
        marks = torch.empty((w.s * w.s * w.B, w.Nsub, w.heads, w.D), device="cuda", dtype=torch.bfloat16)
        for sb in range(marks.shape[0]):
            marks[sb] = float(sb + 1) * 0.25  # exactly representable, distinct per subsequence
        vd = sk.skiparse_unpermute(marks, w.T, w.H, w.W, w.s, pattern)
        out = sk.skiparse_attn_fwd(qd, kd, vd, w.T, w.H, w.W, w.s, pattern, fused=True)
        # a bf16-rounded ratio of fp32 sums of identical products: allow one bf16 ulp
        assert torch.allclose(out.float(), vd.float(), rtol=2 ** -7, atol=0)
        del marks, vd, out


def test_768p_dense_sampled_rows():
    """dense_attn_fwd at the hybrid comparison's shape (80,640 tokens, 40 heads): sampled rows against the oracle."""
    import paper_2605_28691_amd as sk

    w = si.WORKLOADS["hybrid"]
    q, k, v = si.make_qkv(w)
    rows = si.sample_rows(w, 1, seed=9)  # 3 rows per head; each costs 41 MFLOP on the CPU
    want = oracle.skiparse_attention_rows(*oracle_inputs(q, k, v), rows, w.T, w.H, w.W, 1, "token", w.scale)
    out = sk.dense_attn_fwd(*_gpu((q, k, v)), w.T, w.H, w.W, scale=w.scale)
    torch.cuda.synchronize()
    assert_close_bf16(gather_rows(out, rows), want, "dense 768p")


PAD_CASES = [  # B, heads, D, T, H, W, s -- H or W not a multiple of s*s
    (1, 2, 128, 3, 5, 7, 2),
    (2, 3, 128, 4, 10, 13, 2),
    (1, 2, 64, 5, 6, 30, 2),     # the 480P grid's H = 30 problem in small: 6 % 4 != 0
    (1, 4, 128, 2, 11, 20, 3),
    (1, 2, 128, 6, 8, 12, 2),    # divisible: the padded mode must agree with the plain one
    (1, 1, 128, 9, 1, 33, 2),    # H = 1: the classes with p = 1 are empty
    (1, 1, 64, 11, 21, 26, 2),   # padded grid 24 x 28: 1848 positions per class = 29 key tiles (ring wrap-around), rows of padding inside
]


@pytest.mark.parametrize("B,heads,D,T,H,W,s", PAD_CASES)
@pytest.mark.parametrize("pattern", ["token", "group"])
def test_any_resolution_padding_small(B, heads, D, T, H, W, s, pattern):
    """Any-resolution mode (end padding to multiples of s*s, padding masked) against the oracle's mask-form definition."""
    import paper_2605_28691_amd as sk

    w = si.make_shape("pad", B, heads, D, T, H, W, s, seed=41 + s)
    q, k, v = si.make_qkv(w)
    rows = np.array([(b, hd, n) for b in range(B) for hd in range(heads) for n in range(T * H * W)], dtype=np.int64)
    want = oracle.skiparse_attention_rows_padded(*oracle_inputs(q, k, v), rows, T, H, W, s, pattern, w.scale)
    n = q.numel()
    buf = torch.full((n + 4096,), 5.0, dtype=torch.bfloat16, device="cuda")
    out = buf[2048 : 2048 + n].view(q.shape)
    sk.skiparse_attn_fwd(*_gpu((q, k, v)), T, H, W, s, pattern, scale=w.scale, fused=True, pad=True, out=out)
    torch.cuda.synchronize()
    assert (buf[:2048] == 5.0).all() and (buf[2048 + n :] == 5.0).all()
    assert_close_bf16(gather_rows(out, rows), want, f"padded {pattern}")
    if H % (s * s) == 0 and W % (s * s) == 0:
        plain = sk.skiparse_attn_fwd(*_gpu((q, k, v)), T, H, W, s, pattern, scale=w.scale, fused=True)
        assert_close_bf16(to_np64(out), to_np64(plain), "padded vs plain")


def test_any_resolution_720p_sampled_rows():
    """The paper's padded workload: 81 x 720 x 1280 video, latent grid 21 x 45 x 80, padded to 21 x 48 x 80 (Tab. 2a),
    40 heads of 128 channels, s = 2, both patterns: sampled rows against the oracle."""
    import paper_2605_28691_amd as sk

    w = si.make_shape("720p", 1, 40, 128, 21, 45, 80, 2, seed=7)
    q, k, v = si.make_qkv(w)
    rows = si.sample_rows(w, 8, seed=7)
    qd, kd, vd = _gpu((q, k, v))
    for pattern in ("token", "group"):
        want = oracle.skiparse_attention_rows_padded(*oracle_inputs(q, k, v), rows, w.T, w.H, w.W, w.s, pattern, w.scale)
        out = sk.skiparse_attn_fwd(qd, kd, vd, w.T, w.H, w.W, w.s, pattern, scale=w.scale, fused=True, pad=True)
        torch.cuda.synchronize()
        assert_close_bf16(gather_rows(out, rows), want, f"720p {pattern}")
        del out


def test_fused_equals_unfused_bit_for_bit_on_random_shapes():
    """The fused call (index map in the kernel's addressing) and the unfused path (explicit permutes around the same kernel) run the
    same arithmetic in the same order, so they must agree bit for bit; seeded random shapes, both patterns, odd head counts."""
    import paper_2605_28691_amd as sk

    rng = np.random.default_rng(123)
    for case in range(12):
        s = int(rng.choice([2, 2, 2, 3, 4]))
        D = int(rng.choice([64, 128]))
        B, heads, T = int(rng.integers(1, 3)), int(rng.integers(1, 6)), int(rng.integers(1, 5))
        H, W = s * s * int(rng.integers(1, 5)), s * s * int(rng.integers(1, 7))
        pattern = "token" if case % 2 == 0 else "group"
        w = si.make_shape("rnd", B, heads, D, T, H, W, s, seed=500 + case)
        q, k, v = _gpu(si.make_qkv(w))
        a = sk.skiparse_attn_fwd(q, k, v, T, H, W, s, pattern, scale=w.scale, fused=True)
        b = sk.skiparse_attn_fwd(q, k, v, T, H, W, s, pattern, scale=w.scale, fused=False)
        assert torch.equal(a, b), (case, B, heads, D, T, H, W, s, pattern)
        assert bool(torch.isfinite(a.float()).all())


def test_largest_admitted_batch_element_sampled_rows():
    """Maximum size: one batch element just below the 4 GiB that the kernels' 32-bit row offsets can address (40 heads of 128,
    grid 21 x 120 x 166 = 418,320 tokens: 4,283,596,800 bytes per tensor, 99.7 % of the limit; subsequences of 104,580 tokens with a
    ragged last tile).  Sampled query rows against the oracle, among them the first and the very last token (the highest offset), and
    canaries behind the output.  One token row more per batch element is rejected by the size check."""
    import ctypes

    import paper_2605_28691_amd as sk

    B, heads, D, T, H, W, s = 1, 40, 128, 21, 120, 166, 2
    N = T * H * W
    assert N * heads * D * 2 < 2 ** 32 <= T * 120 * 168 * heads * D * 2
    g = torch.Generator(device="cuda").manual_seed(77)
    q, k, v = (torch.randn((B, N, heads, D), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16) for _ in range(3))
    buf = torch.full((q.numel() + 4096,), 3.0, dtype=torch.bfloat16, device="cuda")
    out = buf[:q.numel()].view_as(q)
    sk.skiparse_attn_fwd(q, k, v, T, H, W, s, "token", fused=True, out=out)
    torch.cuda.synchronize()
    assert bool((buf[q.numel():] == 3.0).all())
    rng = np.random.default_rng(5)
    rows = np.array([(0, int(h), int(n)) for h, n in zip(rng.integers(0, heads, 60), rng.integers(0, N, 60))]
                    + [(0, 0, 0), (0, heads - 1, N - 1), (0, 17, N - 1), (0, 3, N - 2)], dtype=np.int64)
    want = oracle.skiparse_attention_rows(*(si.as_oracle_array(t.cpu()) for t in (q, k, v)), rows, T, H, W, s, "token", 1.0 / np.sqrt(D))
    assert_close_bf16(gather_rows(out, rows), want, "largest batch element")
    # 21 x 120 x 167 tokens would pass 4 GiB: refused before anything is launched
    p = [ctypes.c_void_p(t.data_ptr()) for t in (q, k, v, out)]
    rc = sk.lib().skiparse_attn_fwd(*p, 1, heads, T, 120, 168, D, s, 0, ctypes.c_float(0.0), 0, 1, None, 0, None)
    assert rc == -2
