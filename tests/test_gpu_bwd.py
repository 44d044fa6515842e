"""GPU parity: skiparse_attn_fwd_lse + skiparse_attn_bwd through the C ABI against the float64 oracle's gradients.

Tolerance (bf16 path: P and dS rounded to bf16 for the matrix products, fp32 accumulation, bf16 results), per gradient:
relative L2 error <= 1e-2 and max |diff| <= 3e-2 * max |reference|.
"""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from _util import errors, oracle_inputs, to_np64

pytestmark = pytest.mark.gpu

BWD_REL_L2 = 1e-2
BWD_MAX_REL = 3e-2

SMALL = [  # B, heads, D, T, H, W, s
    (1, 2, 64, 2, 8, 8, 2),      # 32 tokens per subsequence: a single partial tile on both sides
    (2, 3, 128, 3, 8, 12, 2),    # Nsub = 72: one full + one partial streamed tile
    (1, 2, 128, 5, 16, 20, 2),   # Nsub = 400: two owner tiles (256 + 144), 7 streamed tiles with a tail of 16
    (2, 2, 64, 5, 16, 20, 2),    # head_dim 64, batch of 2
    (1, 9, 128, 4, 9, 18, 3),    # s = 3, 9 heads
    (1, 2, 128, 7, 16, 16, 2),   # Nsub = 448 = 7 * 64: no tail
    (1, 1, 64, 9, 24, 28, 2),    # Nsub = 1512: 24 streamed tiles, more than the 16 slots of the row-offset ring
    (1, 1, 128, 1, 16, 48, 4),   # s = 4: 16 subsequences of 48 tokens
    (2, 2, 64, 1, 2, 2, 2),      # one token per subsequence (token-wise only): P = 1, dv = dout, dq = dk = 0
]


def assert_grad_close(got, want, what):
    assert np.isfinite(got).all(), f"{what}: non-finite"
    max_abs, rel_l2 = errors(got, want)
    lim = BWD_MAX_REL * float(np.abs(want).max())
    assert rel_l2 <= BWD_REL_L2 and max_abs <= lim, f"{what}: rel-L2 {rel_l2:.3e}, max-abs {max_abs:.3e} (limit {lim:.3e})"
    return max_abs, rel_l2


def _run(sk, q, k, v, dout, T, H, W, s, pattern, scale):
    qg, kg, vg, dg = (t.cuda() for t in (q, k, v, dout))
    out, lse = sk.skiparse_attn_fwd_lse(qg, kg, vg, T, H, W, s, pattern, scale=scale)
    dq, dk, dv = sk.skiparse_attn_bwd(qg, kg, vg, out, dg, lse, T, H, W, s, pattern, scale=scale)
    return out, lse, dq, dk, dv


@pytest.mark.parametrize("B,heads,D,T,H,W,s", SMALL)
@pytest.mark.parametrize("pattern", ["token", "group"])
def test_backward_small(B, heads, D, T, H, W, s, pattern):
    import paper_2605_28691_amd as sk

    if pattern == "group" and (H % (s * s) or W % (s * s)):
        pytest.skip("group-wise needs multiples of s^2")
    w = si.make_shape("bwd", B, heads, D, T, H, W, s, seed=40 + s)
    q, k, v = si.make_qkv(w)
    dout = si.make_dout(w)
    want = oracle.skiparse_attention_bwd(*oracle_inputs(q, k, v), si.as_oracle_array(dout), T, H, W, s, pattern, w.scale)
    out, lse, dq, dk, dv = _run(sk, q, k, v, dout, T, H, W, s, pattern, w.scale)
    # the forward with the extra output is the same forward
    assert torch.equal(out, sk.skiparse_attn_fwd(q.cuda(), k.cuda(), v.cuda(), T, H, W, s, pattern, scale=w.scale))
    # log-sum-exp against its definition on the rearranged tensors (float64)
    qs, ks = (oracle.permute(to_np64(t), T, H, W, s, pattern) for t in (q, k))
    logits = np.einsum("bihd,bjhd->bhij", qs, ks) * w.scale
    m = logits.max(-1, keepdims=True)
    lse_ref = (m + np.log(np.exp(logits - m).sum(-1, keepdims=True)))[..., 0]
    assert np.abs(to_np64(lse) - lse_ref).max() <= 5e-3
    for g, wnt, name in zip((dq, dk, dv), want, ("dq", "dk", "dv")):
        if w.Nsub == 1:  # one key per subsequence: dv = dout exactly, dq = dk = 0 (a relative bound means nothing at zero)
            assert np.abs(to_np64(g) - wnt).max() <= 1e-6, name
        else:
            assert_grad_close(to_np64(g), wnt, f"{pattern} {name}")


@pytest.mark.parametrize("B,heads,D,N", [(1, 2, 128, 1000), (2, 3, 64, 333), (1, 1, 128, 64), (1, 1, 64, 1)])
def test_backward_dense_s1(B, heads, D, N):
    import paper_2605_28691_amd as sk

    w = si.make_shape("bwd_dense", B, heads, D, 1, 1, N, 1, seed=N + 1)
    q, k, v = si.make_qkv(w)
    dout = si.make_dout(w)
    want = oracle.attention_bwd(*oracle_inputs(q, k, v), si.as_oracle_array(dout), w.scale)
    _, _, dq, dk, dv = _run(sk, q, k, v, dout, 1, 1, N, 1, "token", w.scale)
    for g, wnt, name in zip((dq, dk, dv), want, ("dq", "dk", "dv")):
        if N == 1:  # one key: dv = dout exactly, dq = dk = 0
            assert np.abs(to_np64(g) - wnt).max() <= 1e-6, name
        else:
            assert_grad_close(to_np64(g), wnt, f"dense {name}")


def test_backward_peaky_logits():
    """Large logits (one dominant key per query): P is nearly one-hot and the log-sum-exp is large."""
    import paper_2605_28691_amd as sk

    w = si.make_shape("bwd_peaky", 1, 2, 128, 2, 8, 16, 2, seed=3)
    q, k, v = si.make_qkv(w)
    q, k = (q.float() * 4.0).to(torch.bfloat16), (k.float() * 4.0).to(torch.bfloat16)
    dout = si.make_dout(w)
    want = oracle.skiparse_attention_bwd(*oracle_inputs(q, k, v), si.as_oracle_array(dout), w.T, w.H, w.W, w.s, "token", w.scale)
    _, _, dq, dk, dv = _run(sk, q, k, v, dout, w.T, w.H, w.W, w.s, "token", w.scale)
    for g, wnt, name in zip((dq, dk, dv), want, ("dq", "dk", "dv")):
        assert_grad_close(to_np64(g), wnt, f"peaky {name}")


def test_backward_is_deterministic_and_stays_in_bounds():
    import paper_2605_28691_amd as sk

    w = si.make_shape("bwd_det", 1, 3, 128, 3, 8, 12, 2, seed=8)
    q, k, v = si.make_qkv(w)
    dout = si.make_dout(w)
    qg, kg, vg, dg = (t.cuda() for t in (q, k, v, dout))
    out, lse = sk.skiparse_attn_fwd_lse(qg, kg, vg, w.T, w.H, w.W, w.s, "group", scale=w.scale)
    n = q.numel()
    pad = 4096
    runs = []
    for _ in range(2):
        buf = torch.full((3, n + 2 * pad), 7.0, dtype=torch.bfloat16, device="cuda")  # canaries around every gradient
        views = [buf[i, pad : pad + n].view(q.shape) for i in range(3)]
        sk.skiparse_attn_bwd(qg, kg, vg, out, dg, lse, w.T, w.H, w.W, w.s, "group", scale=w.scale, dq=views[0], dk=views[1], dv=views[2])
        assert bool((buf[:, :pad] == 7.0).all()) and bool((buf[:, pad + n :] == 7.0).all())
        runs.append(buf)
    assert torch.equal(runs[0], runs[1])


def test_backward_480p_one_unit_and_invariants():
    """Benchmark-shaped grid: the gradients of sampled tokens of one attention unit against the oracle (which walks the whole
    unit), plus properties that hold at any size for every unit: sum_keys dk = 0 and sum_keys dv = sum_queries dout."""
    import paper_2605_28691_amd as sk

    w = si.WORKLOADS["480p"]
    q, k, v = si.make_qkv(w)
    dout = si.make_dout(w)
    T, H, W, s = w.T, w.H, w.W, w.s
    _, _, dq, dk, dv = _run(sk, q, k, v, dout, T, H, W, s, "token", w.scale)
    b, head, n0 = 0, 5, 12345
    p0, q0, _ = oracle.dst_index("token", s, T, H, W, n0)
    toks = [n0] + [oracle.src_index("token", s, T, H, W, p0, q0, j) for j in (0, 1, 4097, w.Nsub - 1)]
    want = oracle.skiparse_attention_bwd_unit(*oracle_inputs(q, k, v), si.as_oracle_array(dout), b, head, toks, T, H, W, s, "token", w.scale)
    for g, wnt, name in zip((dq, dk, dv), want, ("dq", "dk", "dv")):
        assert_grad_close(to_np64(g[b, toks, head]), wnt, f"480p {name}")
    # invariants per (batch, head, subsequence), in float64 on the bf16 results
    for pattern_class in range(s * s):
        p, qq = divmod(pattern_class, s)
        idx = torch.tensor([oracle.src_index("token", s, T, H, W, p, qq, j) for j in range(0, w.Nsub)], device="cuda")
        dk_sum = dk[0, idx].double().sum(0)                     # [heads][D]
        dv_sum = dv[0, idx].double().sum(0)
        do_sum = dout.cuda()[0, idx].double().sum(0)
        dk_abs = dk[0, idx].double().abs().sum(0)
        assert float((dk_sum.abs() / dk_abs).max()) <= 2e-2     # cancels up to the bf16 rounding of the rows
        assert float((dv_sum - do_sum).abs().max()) <= 2e-2 * float(do_sum.abs().max())


PAD_CASES = [  # B, heads, D, T, H, W, s -- any-resolution mode: H or W not a multiple of s*s
    (1, 2, 128, 3, 5, 7, 2),
    (2, 3, 128, 4, 10, 13, 2),   # padded grid 12 x 16: Nsub_pad = 192
    (1, 2, 64, 5, 6, 30, 2),
    (1, 4, 128, 2, 11, 20, 3),   # s = 3: padded to 18 x 27
    (1, 2, 128, 9, 17, 21, 2),   # Nsub_pad = 9 * 5 * 6 = 270: two owner tiles, padding rows inside and at the end of tiles
    (1, 1, 128, 9, 1, 33, 2),    # H = 1: the classes with p = 1 hold padding only
    (1, 2, 128, 6, 8, 12, 2),    # divisible: must agree bit for bit with the plain mode
    (1, 1, 64, 11, 21, 26, 2),   # padded grid 24 x 28: 29 streamed tiles (ring wrap-around), rows of padding inside
]


@pytest.mark.parametrize("B,heads,D,T,H,W,s", PAD_CASES)
@pytest.mark.parametrize("pattern", ["token", "group"])
def test_backward_any_resolution_small(B, heads, D, T, H, W, s, pattern):
    """Sec. 3.2's padding + mask in the backward pass, against the oracle's mask-form gradients."""
    import paper_2605_28691_amd as sk

    w = si.make_shape("bwd_pad", B, heads, D, T, H, W, s, seed=50 + s)
    q, k, v = si.make_qkv(w)
    dout = si.make_dout(w)
    want = oracle.skiparse_attention_bwd_padded(*oracle_inputs(q, k, v), si.as_oracle_array(dout), T, H, W, s, pattern, w.scale)
    qg, kg, vg, dg = (t.cuda() for t in (q, k, v, dout))
    out, lse = sk.skiparse_attn_fwd_lse(qg, kg, vg, T, H, W, s, pattern, scale=w.scale, pad=True)
    assert torch.equal(out, sk.skiparse_attn_fwd(qg, kg, vg, T, H, W, s, pattern, scale=w.scale, fused=True, pad=True))
    n = q.numel()
    guard = 4096
    buf = torch.full((3, n + 2 * guard), 7.0, dtype=torch.bfloat16, device="cuda")  # canaries around every gradient
    views = [buf[i, guard : guard + n].view(q.shape) for i in range(3)]
    sk.skiparse_attn_bwd(qg, kg, vg, out, dg, lse, T, H, W, s, pattern, scale=w.scale, dq=views[0], dk=views[1], dv=views[2], pad=True)
    assert bool((buf[:, :guard] == 7.0).all()) and bool((buf[:, guard + n :] == 7.0).all())
    for g, wnt, name in zip(views, want, ("dq", "dk", "dv")):
        assert_grad_close(to_np64(g), wnt, f"padded {pattern} {name}")
    if H % (s * s) == 0 and W % (s * s) == 0:
        _, lse0, *plain = _run(sk, q, k, v, dout, T, H, W, s, pattern, w.scale)
        assert torch.equal(lse, lse0)
        for g, p in zip(views, plain):
            assert torch.equal(g, p)


def test_backward_720p_one_unit():
    """The paper's training grid (Sec. 4.1: 720 x 1280, latent 21 x 45 x 80, padded to 21 x 48 x 80), 8 of the 40 heads:
    gradients of sampled tokens of one unit per pattern against the oracle, and the invariants over every unit."""
    import paper_2605_28691_amd as sk

    w = si.make_shape("720p_bwd", 1, 8, 128, 21, 45, 80, 2, seed=11)
    q, k, v = si.make_qkv(w)
    dout = si.make_dout(w)
    T, H, W, s = w.T, w.H, w.W, w.s
    qg, kg, vg, dg = (t.cuda() for t in (q, k, v, dout))
    n = np.arange(T * H * W)
    hh, ww = (n // W) % H, n % W
    for pattern in ("token", "group"):
        out, lse = sk.skiparse_attn_fwd_lse(qg, kg, vg, T, H, W, s, pattern, scale=w.scale, pad=True)
        dq, dk, dv = sk.skiparse_attn_bwd(qg, kg, vg, out, dg, lse, T, H, W, s, pattern, scale=w.scale, pad=True)
        cls = (hh % s) * s + (ww % s) if pattern == "token" else ((hh // s) % s) * s + ((ww // s) % s)  # Sec. 3.1
        b, head, n0 = 0, 3, 44 * W + 79 + 5 * H * W  # last row and column of a frame: next to the padding
        members = np.nonzero(cls == cls[n0])[0]
        toks = [int(n0)] + [int(members[i]) for i in (0, 1, len(members) // 2, len(members) - 1) if members[i] != n0]
        want = oracle.skiparse_attention_bwd_unit_padded(*oracle_inputs(q, k, v), si.as_oracle_array(dout), b, head, toks, T, H, W, s,
                                                         pattern, w.scale)
        for g, wnt, name in zip((dq, dk, dv), want, ("dq", "dk", "dv")):
            assert_grad_close(to_np64(g[b, toks, head]), wnt, f"720p {pattern} {name}")
        for c in range(s * s):
            idx = torch.tensor(np.nonzero(cls == c)[0], device="cuda")
            dk_sum, dv_sum, do_sum = (x[0, idx].double().sum(0) for x in (dk, dv, dg))
            dk_abs = dk[0, idx].double().abs().sum(0)
            assert float((dk_sum.abs() / dk_abs).max()) <= 2e-2
            assert float((dv_sum - do_sum).abs().max()) <= 2e-2 * float(do_sum.abs().max())
        del out, lse, dq, dk, dv


def test_backward_768p_one_unit_group():
    """The benchmark's shape (21 x 48 x 80, s = 2), group-wise, 4 of the 40 heads: gradients of sampled tokens of one attention unit
    (20,160 tokens) against the oracle, which walks the whole unit."""
    import paper_2605_28691_amd as sk

    w = si.make_shape("768p_bwd", 1, 4, 128, 21, 48, 80, 2, seed=12)
    q, k, v = si.make_qkv(w)
    dout = si.make_dout(w)
    T, H, W, s = w.T, w.H, w.W, w.s
    _, _, dq, dk, dv = _run(sk, q, k, v, dout, T, H, W, s, "group", w.scale)
    b, head, n0 = 0, 2, 54321
    p0, q0, _ = oracle.dst_index("group", s, T, H, W, n0)
    toks = [n0] + [oracle.src_index("group", s, T, H, W, p0, q0, j) for j in (0, 255, 256, 10007, w.Nsub - 1)]
    want = oracle.skiparse_attention_bwd_unit(*oracle_inputs(q, k, v), si.as_oracle_array(dout), b, head, toks, T, H, W, s, "group", w.scale)
    for g, wnt, name in zip((dq, dk, dv), want, ("dq", "dk", "dv")):
        assert_grad_close(to_np64(g[b, toks, head]), wnt, f"768p group {name}")


def test_backward_768p_one_unit_token_all_heads():
    """The call bench.py times: the 768P workload itself (40 heads, seed 2), token-wise.  Gradients of sampled tokens of one
    attention unit against the oracle, plus the any-size invariants for every head of one subsequence."""
    import paper_2605_28691_amd as sk

    w = si.WORKLOADS["768p"]
    q, k, v = si.make_qkv(w)
    dout = si.make_dout(w)
    T, H, W, s = w.T, w.H, w.W, w.s
    _, _, dq, dk, dv = _run(sk, q, k, v, dout, T, H, W, s, "token", w.scale)
    b, head, n0 = 0, 37, 70001
    p0, q0, _ = oracle.dst_index("token", s, T, H, W, n0)
    toks = [n0] + [oracle.src_index("token", s, T, H, W, p0, q0, j) for j in (0, 255, 256, 12345, w.Nsub - 1)]
    want = oracle.skiparse_attention_bwd_unit(*oracle_inputs(q, k, v), si.as_oracle_array(dout), b, head, toks, T, H, W, s, "token", w.scale)
    for g, wnt, name in zip((dq, dk, dv), want, ("dq", "dk", "dv")):
        ma, rl = assert_grad_close(to_np64(g[b, toks, head]), wnt, f"768p token {name}")
        print(f"768p token-wise {name}: max-abs {ma:.3e} rel-L2 {rl:.3e}")
    idx = torch.tensor([oracle.src_index("token", s, T, H, W, p0, q0, j) for j in range(w.Nsub)], device="cuda")
    dk_sum, dk_abs = dk[0, idx].double().sum(0), dk[0, idx].double().abs().sum(0)
    dv_sum, do_sum = dv[0, idx].double().sum(0), dout.cuda()[0, idx].double().sum(0)
    assert float((dk_sum.abs() / dk_abs).max()) <= 2e-2
    assert float((dv_sum - do_sum).abs().max()) <= 2e-2 * float(do_sum.abs().max())
