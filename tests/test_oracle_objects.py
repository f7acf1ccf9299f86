"""Pins for the oracle's transport objects (Sec. 4.2 "Asynchronous Weight Transfer": fixed-size,
self-describing buckets pushed to a relay and pulled independently): the byte layout against a
hand-worked example, and the property that matters: any cut of a destination stream into objects,
applied in any order, gives what applying the stream gives."""
import os

import numpy as np
import pytest
import torch

from oracle import oracle
from oracle.oracle import SPLIT_ROWS, SPLIT_COLS, REPLICATED, FUSED_ROWS
from workloads import synth

HERE = os.path.dirname(os.path.abspath(__file__))


def golden_bytes():
    rows = [l for l in open(os.path.join(HERE, "golden", "object_layout.txt")) if l.strip() and not l.startswith("#")]
    return np.array([int(x, 16) for l in rows for x in l.split()], dtype=np.uint8)


def test_layout_matches_the_hand_worked_example():
    bucket = {"seg_off": np.array([0, 2, 2, 5]), "idx": np.array([7, 9, 1, 4, 6], dtype=np.int32),
              "val": np.array([0x0101, 0x0202, 0x0303, 0x0404, 0x0505], dtype=np.uint16)}
    obj = oracle.pack_object(bucket, 2, 1, 3)
    want = golden_bytes()
    assert obj.size == want.size == 128 == oracle.object_bytes(3, 3)
    assert np.array_equal(obj, want)
    back = oracle.unpack_object(want, 3)
    assert back["shard"] == 2 and back["first_entry"] == 1
    assert back["seg_off"].tolist() == [0, 1, 1, 3]
    assert back["idx"].tolist() == [9, 1, 4] and back["val"].tolist() == [0x0202, 0x0303, 0x0404]


def model_bucket(seed, tp, d):
    ts = [dict(rows=16, cols=24, rule=SPLIT_ROWS, sections=None), dict(rows=1, cols=50, rule=REPLICATED, sections=None),
          dict(rows=8, cols=32, rule=SPLIT_COLS, sections=None), dict(rows=1, cols=7, rule=REPLICATED, sections=None),
          dict(rows=32, cols=5, rule=FUSED_ROWS, sections=[16, 8, 8])]
    recs = []
    for i, t in enumerate(ts):
        o, n = synth.pair_bernoulli(t["rows"] * t["cols"], 0.0 if i == 3 else 0.3, seed=seed + i)
        recs.append(dict(t, old=o.view(torch.int16).numpy().view(np.uint16).copy(),
                         new=n.view(torch.int16).numpy().view(np.uint16).copy()))
    bucket = oracle.encode_model(recs, tp)[d]
    olds = [oracle.dense_shard(r["old"], r["rows"], r["cols"], r["rule"], r["sections"], tp, d) for r in recs]
    news = [oracle.dense_shard(r["new"], r["rows"], r["cols"], r["rule"], r["sections"], tp, d) for r in recs]
    return bucket, olds, news, len(ts)


@pytest.mark.parametrize("chunk", [1, 3, 16, 1000])
def test_any_cut_applied_in_any_order_equals_the_stream(chunk):
    bucket, olds, news, nt = model_bucket(40, 2, 1)
    total = int(bucket["seg_off"][-1])
    assert total > 30
    objs = [oracle.pack_object(bucket, 1, e, min(chunk, total - e)) for e in range(0, total, chunk)]
    assert sum(oracle.unpack_object(o, nt)["idx"].size for o in objs) == total
    rng = np.random.default_rng(chunk)
    dst = [x.copy() for x in olds]
    for k in rng.permutation(len(objs)):
        oracle.apply_object(objs[k], nt, dst)
    for a, b in zip(dst, news):
        assert np.array_equal(a, b)
    # an object that starts inside one segment and ends inside another keeps both parts
    if chunk == 16:
        u = oracle.unpack_object(objs[1], nt)
        assert u["first_entry"] == 16 and (np.diff(u["seg_off"]) >= 0).all() and u["seg_off"][-1] == u["idx"].size


def test_empty_object_and_malformed_objects():
    bucket, olds, news, nt = model_bucket(41, 1, 0)
    empty = oracle.pack_object(bucket, 0, 5, 0)
    assert oracle.unpack_object(empty, nt)["idx"].size == 0
    good = oracle.pack_object(bucket, 0, 0, 10)
    for damage in ("magic", "version", "tensors", "short", "count"):
        bad = good.copy()
        if damage == "magic":
            bad[0] ^= 1
        elif damage == "version":
            bad[4] = 2
        elif damage == "tensors":
            bad[12] += 1
        elif damage == "short":
            bad = bad[:-16]
        else:
            bad[24] = 200                      # says 200 entries, holds 10
        with pytest.raises(oracle.OracleError):
            oracle.unpack_object(bad, nt)
    with pytest.raises(oracle.OracleError):
        oracle.pack_object(bucket, 0, 0, int(bucket["seg_off"][-1]) + 1)
