"""Pins for the oracle's sender-side sharding (Sec. 4.2: per-rank slice ranges on both sides,
"heterogeneous parallelism configurations"): a sender holds shard s of S of every tensor and emits
to D destination shards.  What fixes the result without any implementation to compare with:
the senders' outputs together are exactly the full-tensor encode (already pinned), each sender
only touches destinations its slice overlaps, and applying every sender's entries to the sliced
old weights gives the sliced new weights (slices taken with plain numpy)."""
import numpy as np
import pytest
import torch

from oracle import oracle
from oracle.oracle import REPLICATED, SPLIT_ROWS, SPLIT_COLS, FUSED_ROWS
from workloads import synth
from test_oracle_shard_map import numpy_shard


def bits(t):
    return t.view(torch.int16).numpy().view(np.uint16).copy()


CASES = [
    (REPLICATED, 1, 96, None), (SPLIT_ROWS, 32, 9, None), (SPLIT_COLS, 7, 64, None),
    (FUSED_ROWS, 64, 5, [32, 16, 16]), (FUSED_ROWS, 48, 3, [24, 24]),
]


def slices(o, n, rule, R, C, sec, S):
    return [(np.ascontiguousarray(numpy_shard(o.reshape(R, C), rule, sec, S, s)).ravel(),
             np.ascontiguousarray(numpy_shard(n.reshape(R, C), rule, sec, S, s)).ravel()) for s in range(S)]


@pytest.mark.parametrize("rule,R,C,sec", CASES)
@pytest.mark.parametrize("S,D", [(1, 4), (2, 2), (2, 4), (4, 2), (8, 4), (4, 1), (8, 8), (2, 8)])
@pytest.mark.parametrize("p", [0.1, 1.0])
def test_senders_together_equal_the_full_encode(rule, R, C, sec, S, D, p):
    old, new = synth.pair_bernoulli(R * C, p, seed=R * 7 + C + 13 * S + D)
    o, n = bits(old), bits(new)
    full = oracle.encode_tensor(o, n, R, C, rule, sec, D)
    owner = 3 % S                                           # which sender sends a replicated tensor
    per_sender = [oracle.encode_tensor_src(so, sn, R, C, rule, sec, D, S, s, sends_replicated=(s == owner))
                  for s, (so, sn) in enumerate(slices(o, n, rule, R, C, sec, S))]
    for d in range(D):
        idx = np.concatenate([ps[d][0] for ps in per_sender])
        val = np.concatenate([ps[d][1] for ps in per_sender])
        order = np.argsort(idx, kind="stable")
        assert np.array_equal(idx[order], full[d][0]), (d, "indices")       # disjoint and complete
        assert np.array_equal(val[order], full[d][1]), (d, "values")
        for ps in per_sender:
            assert (np.diff(ps[d][0].astype(np.int64)) > 0).all()           # each sender: ascending
        # apply in sender order onto the sliced old weights: the sliced new weights, bit for bit
        out = np.ascontiguousarray(numpy_shard(o.reshape(R, C), rule, sec, D, d)).ravel().copy()
        for ps in per_sender:
            oracle.apply_segment(ps[d][0], ps[d][1], out)
        assert np.array_equal(out, np.ascontiguousarray(numpy_shard(n.reshape(R, C), rule, sec, D, d)).ravel())


def test_a_sender_reaches_only_overlapping_destinations():
    """SPLIT_ROWS 32 rows, S = 4 senders, D = 2: senders 0, 1 overlap destination 0 only; with
    D = 8 sender 1 (rows 8..15) overlaps destinations 2 and 3 (rows 8..11, 12..15)."""
    R, C = 32, 4
    o = np.zeros(R * C, dtype=np.uint16)
    n = np.ones(R * C, dtype=np.uint16)                     # everything changes
    sl = slices(o, n, SPLIT_ROWS, R, C, None, 4)
    got = oracle.encode_tensor_src(sl[1][0], sl[1][1], R, C, SPLIT_ROWS, None, 2, 4, 1)
    assert [g[0].size for g in got] == [8 * C, 0]
    assert np.array_equal(got[0][0], np.arange(8 * C, 16 * C, dtype=np.int32))   # rows 8..15 of shard 0's 16 rows
    got = oracle.encode_tensor_src(sl[1][0], sl[1][1], R, C, SPLIT_ROWS, None, 8, 4, 1)
    assert [g[0].size for g in got] == [0, 0, 4 * C, 4 * C, 0, 0, 0, 0]
    assert np.array_equal(got[2][0], np.arange(4 * C, dtype=np.int32))


def test_column_blocks_interleave_in_the_destination():
    """SPLIT_COLS, 2 rows x 8 cols, S = 4 (2 cols each), D = 2 (4 cols each): sender 1 holds
    cols 2, 3 = the second half of each row of destination 0 -> local indices 2, 3, 6, 7."""
    R, C = 2, 8
    o = np.zeros(R * C, dtype=np.uint16)
    n = (np.arange(R * C) + 100).astype(np.uint16)
    sl = slices(o, n, SPLIT_COLS, R, C, None, 4)
    got = oracle.encode_tensor_src(sl[1][0], sl[1][1], R, C, SPLIT_COLS, None, 2, 4, 1)
    assert np.array_equal(got[0][0], np.array([2, 3, 6, 7], dtype=np.int32))
    assert np.array_equal(got[0][1], np.array([102, 103, 110, 111], dtype=np.uint16))
    assert got[1][0].size == 0


def test_replicated_tensor_is_sent_by_the_named_sender_only():
    o = np.zeros(40, dtype=np.uint16)
    n = np.ones(40, dtype=np.uint16)
    assert all(g[0].size == 0 for g in oracle.encode_tensor_src(o, n, 1, 40, REPLICATED, None, 4, 2, 0, False))
    got = oracle.encode_tensor_src(o, n, 1, 40, REPLICATED, None, 4, 2, 1, True)
    assert all(np.array_equal(g[0], np.arange(40, dtype=np.int32)) for g in got)


def test_bad_sender_arguments_are_refused():
    o = np.zeros(32, dtype=np.uint16)
    with pytest.raises(oracle.OracleError):
        oracle.encode_tensor_src(o, o, 8, 4, SPLIT_ROWS, None, 2, 3, 0)          # 8 rows over 3 senders
    with pytest.raises(oracle.OracleError):
        oracle.encode_tensor_src(o[:16], o[:16], 8, 4, SPLIT_ROWS, None, 2, 2, 2)  # rank out of range


def interleave_by_groups(x, sec, G):
    """[Q;K;V] stacking -> per group [q_g; k_g; v_g], with plain numpy slicing."""
    parts, first = [], []
    r0 = 0
    for sj in sec:
        first.append(r0)
        r0 += sj
    for g in range(G):
        for f, sj in zip(first, sec):
            per = sj // G
            parts.append(x[f + g * per:f + (g + 1) * per])
    return np.concatenate(parts, 0)


@pytest.mark.parametrize("sec,C,G", [([32, 8, 8], 5, 8), ([40, 8, 8], 3, 8), ([16, 16, 16], 4, 4), ([24, 24], 2, 4)])
@pytest.mark.parametrize("S,D", [(1, 1), (1, 4), (2, 4), (4, 2), (4, 4), (2, 1)])
def test_group_interleaved_sender_layout(sec, C, G, S, D):
    """The sender side keeps the fused tensor interleaved by head group and splits it in S row
    blocks (whole groups); built here with numpy slicing of the plain stacking.  The senders'
    outputs together must be the plain full-tensor encode."""
    if G % S or any(sj % D for sj in sec):
        pytest.skip("degree does not divide")
    R = sum(sec)
    old, new = synth.pair_bernoulli(R * C, 0.3, seed=R + C + G + 3 * S + D)
    o, n = bits(old).reshape(R, C), bits(new).reshape(R, C)
    full = oracle.encode_tensor(o, n, R, C, FUSED_ROWS, sec, D)
    oi, ni = interleave_by_groups(o, sec, G), interleave_by_groups(n, sec, G)
    per = R // S
    per_sender = [oracle.encode_tensor_src(oi[s * per:(s + 1) * per], ni[s * per:(s + 1) * per], R, C, FUSED_ROWS, sec,
                                           D, S, s, src_groups=G) for s in range(S)]
    for d in range(D):
        idx = np.concatenate([ps[d][0] for ps in per_sender])
        val = np.concatenate([ps[d][1] for ps in per_sender])
        order = np.argsort(idx, kind="stable")
        assert np.array_equal(idx[order], full[d][0]) and np.array_equal(val[order], full[d][1]), d


def test_group_interleaving_hand_case():
    """Sections (4, 2, 2), G = 2: plain rows q0 q1 q2 q3 k0 k1 v0 v1 are kept as q0 q1 k0 v0 | q2 q3 k1 v1.
    One column, everything changes, one destination: sender 1 of 2 holds q2 q3 k1 v1 = plain rows 2 3 5 7."""
    o = np.zeros(8, dtype=np.uint16)
    n = np.array([12, 13, 15, 17], dtype=np.uint16)             # the sender's slice, values name plain rows + 10
    got = oracle.encode_tensor_src(o[:4], n, 8, 1, FUSED_ROWS, [4, 2, 2], 1, 2, 1, src_groups=2)
    assert got[0][0].tolist() == [2, 3, 5, 7] and got[0][1].tolist() == [12, 13, 15, 17]
    with pytest.raises(oracle.OracleError):
        oracle.encode_tensor_src(o[:4], n, 8, 1, FUSED_ROWS, [4, 2, 2], 1, 2, 1, src_groups=3)
    with pytest.raises(oracle.OracleError):
        oracle.encode_tensor_src(o, o, 8, 1, SPLIT_ROWS, None, 1, 1, 0, src_groups=2)
