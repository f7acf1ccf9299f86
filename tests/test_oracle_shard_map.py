"""Pins for the oracle's shard map (Sec. 4.2 "Shard-aware Weight Transfer": sharded
dimension -> per-rank slice ranges).  Pinned against hand-worked cases and against plain
numpy slicing / concatenation of a tensor that holds its own global index."""
import os

import numpy as np
import pytest

from oracle import oracle
from oracle.oracle import REPLICATED, SPLIT_ROWS, SPLIT_COLS, FUSED_ROWS

GOLD = os.path.join(os.path.dirname(__file__), "golden", "shard_map_cases.txt")


def _cases():
    out = []
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        lhs, rhs = line.split("->")
        rule, R, C, sec, D, r, c = lhs.split()
        sec = None if sec == "-" else [int(s) for s in sec.split(";")]
        out.append((int(rule), int(R), int(C), sec, int(D), int(r), int(c),
                    tuple(int(x) for x in rhs.split())))
    return out


@pytest.mark.parametrize("rule,R,C,sec,D,r,c,want", _cases())
def test_hand_cases(rule, R, C, sec, D, r, c, want):
    assert oracle.shard_map(rule, R, C, sec, D, r, c) == want


def numpy_shard(x, rule, sec, D, d):
    """Shard d of full 2-D array x by plain slicing (the textbook definition)."""
    R, C = x.shape
    if rule == REPLICATED:
        return x
    if rule == SPLIT_ROWS:
        return x[d * (R // D):(d + 1) * (R // D)]
    if rule == SPLIT_COLS:
        return x[:, d * (C // D):(d + 1) * (C // D)]
    parts, row0 = [], 0
    for s in sec:
        part = x[row0:row0 + s]
        parts.append(part[d * (s // D):(d + 1) * (s // D)])
        row0 += s
    return np.concatenate(parts, axis=0)


SHAPES = [
    (REPLICATED, 1, 12, None), (REPLICATED, 3, 5, None),
    (SPLIT_ROWS, 8, 3, None), (SPLIT_ROWS, 16, 1, None), (SPLIT_ROWS, 24, 7, None),
    (SPLIT_COLS, 3, 8, None), (SPLIT_COLS, 1, 16, None), (SPLIT_COLS, 5, 24, None),
    (FUSED_ROWS, 32, 3, [16, 8, 8]), (FUSED_ROWS, 48, 2, [24, 24]),
    (FUSED_ROWS, 56, 5, [40, 8, 8]), (FUSED_ROWS, 8, 4, [8]),
    (FUSED_ROWS, 24, 2, [8, 0, 16]),
]


@pytest.mark.parametrize("rule,R,C,sec", SHAPES)
@pytest.mark.parametrize("D", [1, 2, 4, 8])
def test_map_equals_numpy_slicing_and_is_a_bijection(rule, R, C, sec, D):
    x = np.arange(R * C, dtype=np.int64).reshape(R, C)
    shards = [np.ascontiguousarray(numpy_shard(x, rule, sec, D, d)).ravel() for d in range(D)]
    seen = [np.zeros(s.size, dtype=np.int32) for s in shards]
    for r in range(R):
        for c in range(C):
            d0, nd, loc = oracle.shard_map(rule, R, C, sec, D, r, c)
            assert nd == (D if rule == REPLICATED else 1)
            for d in range(d0, d0 + nd):
                assert shards[d][loc] == r * C + c
                seen[d][loc] += 1
    for d in range(D):
        assert shards[d].size == oracle.local_numel(rule, R, C, D)
        assert (seen[d] == 1).all()          # every local slot hit exactly once


def test_shape_errors():
    with pytest.raises(oracle.OracleError):
        oracle.shard_map(SPLIT_ROWS, 6, 4, None, 4, 0, 0)
    with pytest.raises(oracle.OracleError):
        oracle.shard_map(SPLIT_COLS, 4, 6, None, 4, 0, 0)
    with pytest.raises(oracle.OracleError):
        oracle.shard_map(FUSED_ROWS, 12, 4, [8, 2, 2], 4, 0, 0)      # section not divisible
    with pytest.raises(oracle.OracleError):
        oracle.shard_map(FUSED_ROWS, 12, 4, [8, 8], 4, 0, 0)         # sections do not sum to R
    with pytest.raises(oracle.OracleError):
        oracle.shard_map(SPLIT_ROWS, 8, 4, None, 4, 8, 0)            # row out of range


def test_32b_gqa_layout_puts_one_kv_head_on_each_shard():
    # fused QKV of the 32B-style config: 40 query / 8 KV heads of 128 at TP = 8
    hd, R, C, sec = 128, 7168, 5120, [5120, 1024, 1024]
    for d in range(8):
        # first row of query head 5d, of key head d, of value head d
        for row, local_row in ((5 * d * hd, 0), (5120 + d * hd, 640), (6144 + d * hd, 768)):
            assert oracle.shard_map(FUSED_ROWS, R, C, sec, 8, row, 7) == (d, 1, local_row * C + 7)
    assert oracle.local_numel(FUSED_ROWS, R, C, 8) == 896 * C
