"""GPU parity of the local halves of the pattern switch under Sparse Sequence Parallelism (Sec. 3.3; Alg. 1,
sparse_sequence_parallel) through the C ABI: byte for byte against the oracle's steps, and the whole switch with the ranks of a
group simulated on the one GPU (the all-to-all is an exchange of chunks done with torch indexing; the library communicates nothing)."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si

pytestmark = pytest.mark.gpu

CASES = [  # b, heads, D, T, H, W, s, group_size
    (1, 2, 64, 2, 8, 8, 2, 1),
    (1, 2, 64, 2, 8, 8, 2, 2),
    (2, 3, 128, 3, 8, 12, 2, 4),
    (2, 2, 64, 5, 16, 20, 2, 2),
    (1, 5, 128, 2, 9, 18, 3, 3),
    (2, 1, 128, 1, 9, 9, 3, 9),
    (1, 2, 64, 1, 16, 32, 4, 8),
    (1, 1, 64, 3, 4, 4, 1, 1),     # s = 1: a copy
]


def _bits(t: torch.Tensor) -> np.ndarray:
    return t.cpu().contiguous().view(torch.uint8).numpy()


@pytest.mark.parametrize("b,heads,D,T,H,W,s,group_size", CASES)
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32, torch.uint8])
def test_pack_and_unpack_equal_the_oracle_steps(b, heads, D, T, H, W, s, group_size, dtype):
    import paper_2605_28691_amd as sk

    G = s * s // group_size
    n_local = T * (H // s) * (W // s)
    g = torch.Generator().manual_seed(7 * s + group_size)
    x = torch.randint(0, 255, (G * b, n_local, heads, D * torch.empty((), dtype=dtype).element_size()), generator=g, dtype=torch.uint8).view(dtype)
    xo = x.view(torch.uint8).numpy()  # the oracle moves rows of bytes
    want_send = oracle.ssp_pack(xo, T, H, W, s, group_size)
    guard = torch.full((x.numel() + 4096,), 0, dtype=dtype).cuda()
    send = guard[2048:2048 + x.numel()].view(group_size, G, G * b, n_local // (s * s), heads, D)
    sk.skiparse_ssp_pack(x.cuda(), T, H, W, s, group_size, out=send)
    assert np.array_equal(_bits(send).reshape(want_send.shape), want_send)
    assert not guard[:2048].view(torch.uint8).any() and not guard[2048 + x.numel():].view(torch.uint8).any()
    # unpack of an arbitrary receive buffer (here: the send buffer itself) against the oracle's steps 3 and 4
    want_y = oracle.ssp_unpack(want_send, T, H, W, s, group_size)
    y = sk.skiparse_ssp_unpack(send.clone(), T, H, W, s, group_size)
    assert np.array_equal(_bits(y).reshape(want_y.shape), want_y)


@pytest.mark.parametrize("b,heads,D,T,H,W,s,group_size", [c for c in CASES if c[6] > 1])
@pytest.mark.parametrize("start", ["token", "group"])
def test_simulated_group_switches_pattern(b, heads, D, T, H, W, s, group_size, start):
    """All ranks of a group on one GPU, one after the other: pack, exchange chunks, unpack.  Every rank must end with its shard of
    the other pattern's layout (the library's own single-device permute of the whole tensor, itself checked against the oracle)."""
    import paper_2605_28691_amd as sk

    other = "group" if start == "token" else "token"
    w = si.make_shape("ssp", b, heads, D, T, H, W, s, seed=3)
    x = si.make_qkv(w)[0].cuda()
    G = s * s // group_size
    have = sk.skiparse_permute(x, T, H, W, s, start)
    want = sk.skiparse_permute(x, T, H, W, s, other)
    assert np.array_equal(_bits(want), oracle.permute(si.as_oracle_array(x.cpu()), T, H, W, s, other).view(np.uint8).reshape(_bits(want).shape))
    shards = [have[r * G * b:(r + 1) * G * b].contiguous() for r in range(group_size)]
    sends = [sk.skiparse_ssp_pack(sh, T, H, W, s, group_size) for sh in shards]
    for r in range(group_size):
        recv = torch.stack([sends[src][r] for src in range(group_size)], dim=0).contiguous()
        got = sk.skiparse_ssp_unpack(recv, T, H, W, s, group_size)
        assert torch.equal(got, want[r * G * b:(r + 1) * G * b]), f"rank {r}"


def test_768p_share_of_one_rank_of_four():
    """The benchmark shape, hidden-state rows of 40 x 128 bf16, four ranks (one subsequence each): rank 2's pack and unpack against
    the oracle on sampled rows of the buffers, plus the whole switch for that rank against the single-device permute."""
    import paper_2605_28691_amd as sk

    w = si.WORKLOADS["768p"]
    T, H, W, s, gsz = w.T, w.H, w.W, w.s, 4
    x = si.make_qkv(w)[0]
    tsa = sk.skiparse_permute(x.cuda(), T, H, W, s, "token")      # [4][20160][40][128]
    gsa = sk.skiparse_permute(x.cuda(), T, H, W, s, "group")
    sends = [sk.skiparse_ssp_pack(tsa[r:r + 1].contiguous(), T, H, W, s, gsz) for r in range(gsz)]
    want_send = oracle.ssp_pack(si.as_oracle_array(tsa[2:3].cpu().contiguous()), T, H, W, s, gsz)
    assert np.array_equal(sends[2].cpu().view(torch.int16).numpy().view(np.uint16), want_send)
    recv = torch.stack([sends[src][2] for src in range(gsz)], dim=0).contiguous()
    got = sk.skiparse_ssp_unpack(recv, T, H, W, s, gsz)
    assert torch.equal(got, gsa[2:3])
