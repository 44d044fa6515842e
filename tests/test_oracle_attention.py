"""Pins for the oracle's attention (CPU only): library special cases, closed forms, invariants, brute force."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si


def _rand(shape, seed, dtype=np.float64):
    return np.random.default_rng(seed).standard_normal(shape).astype(dtype)


def _sdpa64(q, k, v, scale):
    """torch's float64 scaled_dot_product_attention on [nb][n][heads][D] arrays."""
    tq, tk, tv = (torch.from_numpy(a.astype(np.float64)).permute(0, 2, 1, 3) for a in (q, k, v))
    o = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=scale)
    return o.permute(0, 2, 1, 3).contiguous().numpy()


@pytest.mark.parametrize("nb,n,heads,D", [(1, 17, 1, 8), (3, 33, 2, 16), (2, 64, 3, 64)])
def test_attention_matches_sdpa_float64(nb, n, heads, D):
    q, k, v = (_rand((nb, n, heads, D), s) for s in (1, 2, 3))
    got = oracle.attention(q, k, v, 0.37)
    assert np.allclose(got, _sdpa64(q, k, v, 0.37), rtol=1e-12, atol=1e-13)


def test_attention_is_not_symmetric_in_q_and_k():
    """A transposed operand (K used as Q) must show: compare with an explicit numpy formula on a case
    where n_q side and n_k side differ in content."""
    q, k, v = (_rand((1, 9, 1, 4), s) for s in (4, 5, 6))
    S = 0.5 * q[0, :, 0] @ k[0, :, 0].T
    P = np.exp(S - S.max(axis=1, keepdims=True))
    want = (P / P.sum(axis=1, keepdims=True)) @ v[0, :, 0]
    assert np.allclose(oracle.attention(q, k, v, 0.5)[0, :, 0], want, rtol=1e-12, atol=1e-14)


def test_uniform_logits_give_mean_of_v():
    """Closed form: Q = 0 makes every logit equal, so every output row is the mean of V over the subsequence."""
    B, heads, D, T, H, W, s = 2, 2, 8, 2, 8, 8, 2
    N = T * H * W
    k, v = _rand((B, N, heads, D), 1), _rand((B, N, heads, D), 2)
    q = np.zeros_like(k)
    for pattern in ("token", "group"):
        out = oracle.skiparse_attention(q, k, v, T, H, W, s, pattern, 1.0)
        vp = oracle.permute(v, T, H, W, s, pattern)
        want = oracle.unpermute(np.broadcast_to(vp.mean(axis=1, keepdims=True), vp.shape).copy(), T, H, W, s, pattern)
        assert np.allclose(out, want, rtol=1e-12, atol=1e-14)


def test_one_hot_logits_select_a_value_row():
    """Closed form: with a very large scale the softmax is a hard arg-max over the keys of the own subsequence."""
    T, H, W, s, D = 1, 4, 4, 2, 4
    N = T * H * W
    rng = np.random.default_rng(3)
    k = rng.standard_normal((1, N, 1, D))
    k /= np.linalg.norm(k, axis=-1, keepdims=True)
    q = k.copy()  # each query matches its own key best (unit vectors)
    v = rng.standard_normal((1, N, 1, D))
    for pattern in ("token", "group"):
        out = oracle.skiparse_attention(q, k, v, T, H, W, s, pattern, 1e4)
        assert np.allclose(out, v, rtol=1e-9, atol=1e-9)


@pytest.mark.parametrize("pattern", ["token", "group"])
def test_tiny_config_equals_masked_dense_and_sampled_rows(pattern):
    """The tiny workload (B=1, 2 heads, D=64, grid 2x8x8, s=2, fp32, seed 0): per-subsequence attention equals
    brute-force N x N attention masked to same-class pairs, and the sampled-row entry point equals the full one."""
    w = si.WORKLOADS["tiny"]
    q, k, v = (si.as_oracle_array(t) for t in si.make_qkv(w))
    full = oracle.skiparse_attention(q, k, v, w.T, w.H, w.W, w.s, pattern, w.scale)
    brute = oracle.masked_dense_attention(q, k, v, w.T, w.H, w.W, w.s, pattern, w.scale)
    assert np.allclose(full, brute, rtol=1e-12, atol=1e-13)
    rows = si.sample_rows(w, 16, seed=1)
    got = oracle.skiparse_attention_rows(q, k, v, rows, w.T, w.H, w.W, w.s, pattern, w.scale)
    want = np.stack([full[b, n, h] for b, h, n in rows])
    assert np.array_equal(got, want)


@pytest.mark.parametrize("pattern", ["token", "group"])
def test_masked_dense_on_s3_batch2(pattern):
    B, heads, D, T, H, W, s = 2, 1, 8, 1, 9, 9, 3
    q, k, v = (_rand((B, T * H * W, heads, D), i, np.float32) for i in (7, 8, 9))
    a = oracle.skiparse_attention(q, k, v, T, H, W, s, pattern, 0.3)
    b = oracle.masked_dense_attention(q, k, v, T, H, W, s, pattern, 0.3)
    assert np.allclose(a, b, rtol=1e-12, atol=1e-13)


def test_s1_equals_full_attention():
    B, heads, D, T, H, W = 2, 2, 16, 2, 4, 6
    q, k, v = (_rand((B, T * H * W, heads, D), i) for i in (1, 2, 3))
    want = _sdpa64(q, k, v, 0.25)
    for pattern in ("token", "group"):
        assert np.allclose(oracle.skiparse_attention(q, k, v, T, H, W, 1, pattern, 0.25), want, rtol=1e-12, atol=1e-13)
    rows = [(1, 1, 5), (0, 0, 47)]
    got = oracle.skiparse_attention_rows(q, k, v, rows, T, H, W, 1, "token", 0.25)
    assert np.allclose(got, np.stack([want[b, n, h] for b, h, n in rows]), rtol=1e-12, atol=1e-13)


def test_skiparse_equals_sdpa_per_subsequence():
    """The composition permute -> library attention -> unpermute, with the library doing the middle step."""
    B, heads, D, T, H, W, s = 2, 3, 16, 2, 8, 12, 2
    q, k, v = (_rand((B, T * H * W, heads, D), i) for i in (11, 12, 13))
    for pattern in ("token", "group"):
        qp, kp, vp = (oracle.permute(a, T, H, W, s, pattern) for a in (q, k, v))
        want = oracle.unpermute(_sdpa64(qp, kp, vp, 0.2), T, H, W, s, pattern)
        assert np.allclose(oracle.skiparse_attention(q, k, v, T, H, W, s, pattern, 0.2), want, rtol=1e-12, atol=1e-13)


def test_rows_sum_to_one_and_no_leakage():
    """V = 1 gives O = 1; V constant per subsequence gives that constant back (nothing leaks across classes);
    outputs are convex combinations, so they stay inside [min V, max V] per channel."""
    B, heads, D, T, H, W, s = 1, 2, 8, 2, 8, 8, 2
    N = T * H * W
    q, k, v = (_rand((B, N, heads, D), i) for i in (21, 22, 23))
    for pattern in ("token", "group"):
        assert np.allclose(oracle.skiparse_attention(q, k, np.ones_like(v), T, H, W, s, pattern, 0.35), 1.0, atol=1e-14)
        marks = np.zeros((s * s * B, N // (s * s), heads, D))
        marks += np.arange(s * s * B).reshape(-1, 1, 1, 1) + 1.0
        vc = oracle.unpermute(marks, T, H, W, s, pattern)
        assert np.allclose(oracle.skiparse_attention(q, k, vc, T, H, W, s, pattern, 0.35), vc, rtol=1e-13)
        out = oracle.skiparse_attention(q, k, v, T, H, W, s, pattern, 0.35)
        assert (out <= v.max(axis=1, keepdims=True) + 1e-12).all() and (out >= v.min(axis=1, keepdims=True) - 1e-12).all()


def test_permutation_equivariance_inside_a_sequence():
    nb, n, heads, D = 1, 40, 2, 8
    q, k, v = (_rand((nb, n, heads, D), i) for i in (31, 32, 33))
    perm = np.random.default_rng(0).permutation(n)
    a = oracle.attention(q, k, v, 0.3)
    b = oracle.attention(q[:, perm].copy(), k[:, perm].copy(), v[:, perm].copy(), 0.3)
    assert np.allclose(a[:, perm], b, rtol=1e-12, atol=1e-14)


def test_dtype_widening_is_exact():
    """bf16 bit patterns and float32 inputs are widened exactly: same values in three storage types, same result."""
    B, heads, D, T, H, W, s = 1, 2, 16, 1, 8, 8, 2
    t = torch.randn((B, T * H * W, heads, D), generator=torch.Generator().manual_seed(1)).to(torch.bfloat16)
    qb, kb, vb = si.as_oracle_array(t), si.as_oracle_array(t.flip(1).contiguous()), si.as_oracle_array((t * 2).contiguous())
    f32 = [torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).float().numpy() for a in (qb, kb, vb)]
    f64 = [a.astype(np.float64) for a in f32]
    o16 = oracle.skiparse_attention(qb, kb, vb, T, H, W, s, "group", 0.25)
    o32 = oracle.skiparse_attention(*f32, T, H, W, s, "group", 0.25)
    o64 = oracle.skiparse_attention(*f64, T, H, W, s, "group", 0.25)
    assert np.array_equal(o16, o32) and np.array_equal(o32, o64)


def test_scale_enters_the_logits():
    """scale multiplies the logits (not the output): doubling the scale equals doubling q."""
    q, k, v = (_rand((1, 12, 1, 4), i) for i in (41, 42, 43))
    assert np.allclose(oracle.attention(q, k, v, 0.8), oracle.attention(2 * q, k, v, 0.4), rtol=1e-12, atol=1e-14)
    assert not np.allclose(oracle.attention(q, k, v, 0.8), oracle.attention(q, k, v, 0.4))


def _all_rows(B, heads, N):
    return np.array([(b, h, n) for b in range(B) for h in range(heads) for n in range(N)], dtype=np.int64)


@pytest.mark.parametrize("pattern", ["token", "group"])
def test_padded_variant_reduces_to_plain_on_divisible_grids(pattern):
    """Sec. 3.2: no mask is needed when H and W are multiples of s*s, so the padded variant must equal the plain one."""
    B, heads, D, T, H, W, s = 2, 2, 8, 2, 8, 12, 2
    q, k, v = (_rand((B, T * H * W, heads, D), i) for i in (51, 52, 53))
    rows = _all_rows(B, heads, T * H * W)
    a = oracle.skiparse_attention_rows_padded(q, k, v, rows, T, H, W, s, pattern, 0.3)
    b = oracle.skiparse_attention_rows(q, k, v, rows, T, H, W, s, pattern, 0.3)
    assert np.allclose(a, b, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("pattern", ["token", "group"])
@pytest.mark.parametrize("H,W,s", [(5, 7, 2), (3, 9, 2), (10, 11, 3), (1, 6, 2)])
def test_padded_variant_equals_explicit_padding(pattern, H, W, s):
    """Sec. 3.2 done literally: pad H and W at the end to multiples of s*s with zeros, run the divisible-grid attention on
    the padded figure with the padding keys removed from every softmax (here by giving them a logit of about -1e9 through
    an extra channel), and drop the padded queries.  Must equal the mask-form definition."""
    B, heads, D, T = 1, 2, 6, 2
    u = s * s
    Hp, Wp = -(-H // u) * u, -(-W // u) * u
    rng = np.random.default_rng(3)
    q, k, v = (rng.standard_normal((B, T * H * W, heads, D)) for _ in range(3))

    def pad(x, fill_extra):
        g = np.zeros((B, T, Hp, Wp, heads, D + 1))
        g[:, :, :H, :W, :, :D] = x.reshape(B, T, H, W, heads, D)
        g[..., D] = fill_extra(np.pad(np.ones((H, W)), ((0, Hp - H), (0, Wp - W)))[None, None, :, :, None])
        return g.reshape(B, T * Hp * Wp, heads, D + 1)

    big = 1e9
    qp = pad(q, lambda real: np.ones_like(real))          # extra channel of q is 1
    kp = pad(k, lambda real: (real - 1.0) * big)          # extra channel of k is 0 for real keys, -1e9 for padding
    vp = pad(v, lambda real: np.zeros_like(real))
    full = oracle.skiparse_attention(qp, kp, vp, T, Hp, Wp, s, pattern, 0.4)[..., :D]
    want = full.reshape(B, T, Hp, Wp, heads, D)[:, :, :H, :W].reshape(B, T * H * W, heads, D)
    rows = _all_rows(B, heads, T * H * W)
    got = oracle.skiparse_attention_rows_padded(q, k, v, rows, T, H, W, s, pattern, 0.4)
    assert np.allclose(got, np.stack([want[b, n, h] for b, h, n in rows]), rtol=1e-9, atol=1e-11)
    brute = oracle.masked_dense_attention(q, k, v, T, H, W, s, pattern, 0.4)
    assert np.allclose(got, np.stack([brute[b, n, h] for b, h, n in rows]), rtol=1e-12, atol=1e-14)
