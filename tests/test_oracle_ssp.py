"""Pins of the oracle's Sparse Sequence Parallelism steps (Sec. 3.3; Algorithm 1, sparse_sequence_parallel), CPU only.

What the paper fixes: the subsequences of a sparse layout are spread over the ranks of a group, and one local rearrangement, one
all-to-all and one local rearrangement turn every rank's shard of the token-wise layout into its shard of the group-wise layout
(and back), without an all-gather.  The ranks are simulated here in one process; the all-to-all is the exchange of array chunks.
Expected values come from the separately pinned single-device rearrangements: permute of the whole tensor, then sharding.
"""
import numpy as np
import pytest

import oracle


def _shards(sparse, group_size, s, B):
    """[(pq b)][Nsub][...] -> one array per rank: its G consecutive classes."""
    G = s * s // group_size
    return [np.ascontiguousarray(sparse[r * G * B:(r + 1) * G * B]) for r in range(group_size)]


def _switch_by_ssp(shards, T, H, W, s, group_size):
    sends = [oracle.ssp_pack(x, T, H, W, s, group_size) for x in shards]
    recvs = oracle.ssp_exchange(sends)
    return [oracle.ssp_unpack(r, T, H, W, s, group_size) for r in recvs]


@pytest.mark.parametrize("B,T,H,W,s,group_size", [
    (1, 2, 8, 8, 2, 1), (1, 2, 8, 8, 2, 2), (1, 2, 8, 8, 2, 4), (2, 3, 8, 12, 2, 2), (2, 1, 16, 8, 2, 4),
    (1, 2, 9, 18, 3, 1), (1, 2, 9, 18, 3, 3), (2, 1, 9, 9, 3, 9), (1, 1, 16, 32, 4, 8),
])
@pytest.mark.parametrize("start", ["token", "group"])
def test_ssp_switches_every_rank_shard_to_the_other_pattern(B, T, H, W, s, group_size, start):
    other = "group" if start == "token" else "token"
    N, C = T * H * W, 3
    x = np.arange(B * N * C, dtype=np.int32).reshape(B, N, C)  # every element distinct: a wrong row or a wrong order shows
    have = _shards(oracle.permute(x, T, H, W, s, start), group_size, s, B)
    want = _shards(oracle.permute(x, T, H, W, s, other), group_size, s, B)
    got = _switch_by_ssp(have, T, H, W, s, group_size)
    for r in range(group_size):
        assert np.array_equal(got[r], want[r]), f"rank {r}"
    # twice is the identity on every shard
    back = _switch_by_ssp(got, T, H, W, s, group_size)
    for r in range(group_size):
        assert np.array_equal(back[r], have[r])


def test_ssp_single_rank_is_the_single_device_switch():
    B, T, H, W, s = 2, 2, 8, 12, 2
    x = np.random.default_rng(0).integers(0, 1 << 15, size=(B, T * H * W, 5)).astype(np.uint16)
    tsa = oracle.permute(x, T, H, W, s, "token")
    got = _switch_by_ssp([tsa], T, H, W, s, 1)[0]
    assert np.array_equal(got, oracle.switch_pattern(tsa, T, H, W, s, "token"))


def test_ssp_message_sizes_and_what_stays_local():
    """Every rank sends group_size equal chunks of 1/group_size of its shard (Sec. 3.3: volume O(N S) instead of an all-gather's
    O(N^2 S)); the chunk addressed to itself never leaves the rank."""
    B, T, H, W, s, g = 1, 2, 8, 8, 2, 4
    x = np.arange(B * T * H * W * 2, dtype=np.int32).reshape(B, T * H * W, 2)
    have = _shards(oracle.permute(x, T, H, W, s, "token"), g, s, B)
    sends = [oracle.ssp_pack(h, T, H, W, s, g) for h in have]
    for r, snd in enumerate(sends):
        assert snd.shape[0] == g and snd.size == have[r].size
        assert sorted(snd.ravel()) == sorted(have[r].ravel())  # a permutation of the shard
    recvs = oracle.ssp_exchange(sends)
    for r in range(g):
        assert np.array_equal(recvs[r][r], sends[r][r])


def test_ssp_rejects_groups_that_split_a_subsequence():
    x = np.zeros((4, 2 * 4 * 4, 1), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.ssp_pack(x, 2, 8, 8, 2, 3)
