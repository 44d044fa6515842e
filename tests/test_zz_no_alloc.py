"""GPU: skiparse_attn_bwd_static (the backward pass for callers that cannot allocate: delta workspace in a static device array of
the library) against skiparse_attn_bwd, through the C ABI.  Same kernels, same order: the gradients must agree bit for bit
(which is within the backward tolerance a fortiori).  Two calls in a row, the second on a smaller problem, so that stale
contents of the shared scratch would show; then the first problem again."""
import pytest
import torch

import synth_inputs as si

pytestmark = pytest.mark.gpu


def _both(sk, w, pattern, pad=False):
    q, k, v = (t.cuda() for t in si.make_qkv(w))
    dout = si.make_dout(w).cuda()
    T, H, W, s = w.T, w.H, w.W, w.s
    out, lse = sk.skiparse_attn_fwd_lse(q, k, v, T, H, W, s, pattern, scale=w.scale, pad=pad)
    want = sk.skiparse_attn_bwd(q, k, v, out, dout, lse, T, H, W, s, pattern, scale=w.scale, pad=pad)
    got = tuple(torch.full_like(q, float("nan")) for _ in range(3))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    sk.skiparse_attn_bwd_static(q, k, v, out, dout, lse, *got, T, H, W, s, pattern, scale=w.scale, pad=pad)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before  # the wrapper allocated nothing either
    for g, wnt, name in zip(got, want, ("dq", "dk", "dv")):
        assert torch.equal(g, wnt), f"{w.name} {pattern} {name}"


def test_static_scratch_backward_equals_the_workspace_one():
    import paper_2605_28691_amd as sk

    assert sk.lib().skiparse_static_scratch_bytes() == 16 * 1024 * 1024
    big = si.make_shape("na_big", 2, 3, 128, 5, 16, 20, 2, seed=51)    # Nsub = 400, 24 units
    small = si.make_shape("na_small", 1, 2, 64, 3, 8, 12, 2, seed=52)  # Nsub = 72, 8 units
    _both(sk, big, "group")
    _both(sk, small, "token")
    _both(sk, big, "token")
    padded = si.make_shape("na_pad", 1, 2, 128, 4, 10, 13, 2, seed=53)  # any-resolution mode: padded grid 12 x 16
    _both(sk, padded, "group", pad=True)


def test_forward_and_static_backward_replay_from_a_hip_graph():
    """What the entry point is for: a training step (forward with log-sum-exp, backward with the static scratch) captured ONCE into
    a HIP graph and replayed on new inputs.  Nothing in the captured region allocates.  Every replay is checked against the eager
    result on the same inputs; eager work and synchronisations lie between the replays."""
    import paper_2605_28691_amd as sk

    w = si.make_shape("graph", 1, 3, 128, 4, 16, 16, 2, seed=61)   # Nsub = 256
    T, H, W, s = w.T, w.H, w.W, w.s
    q, k, v = (t.cuda() for t in si.make_qkv(w))
    dout = si.make_dout(w).cuda()
    out = torch.empty_like(q)
    lse = torch.empty(sk.skiparse_lse_shape(w.B, w.heads, T, H, W, w.D, s, "group"), dtype=torch.float32, device="cuda")
    grads = tuple(torch.empty_like(q) for _ in range(3))

    def step():
        sk.skiparse_attn_fwd_lse(q, k, v, T, H, W, s, "group", scale=w.scale, out=out, lse=lse)
        sk.skiparse_attn_bwd_static(q, k, v, out, dout, lse, *grads, T, H, W, s, "group", scale=w.scale)

    step()  # first call on this device outside the capture: looks up the scratch's address
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for trial in range(3):
        gen = torch.Generator(device="cuda").manual_seed(100 + trial)
        for t in (q, k, v, dout):
            t.copy_(torch.randn(t.shape, generator=gen, device="cuda", dtype=torch.float32))
        for t in (out, *grads):
            t.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (out, *grads)]
        o2, l2 = sk.skiparse_attn_fwd_lse(q, k, v, T, H, W, s, "group", scale=w.scale)  # eager, fresh buffers
        want = sk.skiparse_attn_bwd(q, k, v, o2, dout, l2, T, H, W, s, "group", scale=w.scale)
        torch.cuda.synchronize()
        for g_, w_, name in zip(got, (o2, *want), ("out", "dq", "dk", "dv")):
            assert torch.equal(g_, w_), f"replay {trial}: {name}"
