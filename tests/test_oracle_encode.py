"""Pins for the oracle's dense-to-sparse / sparse-to-dense (Sec. 4.2 "Sparsity-aware Weight
Transfer", App. F D2S / S2D): library reduction at TP = 1, the lossless round trip and the
counting invariants under every shard rule, and the degenerate cases."""
import numpy as np
import pytest
import torch

from oracle import oracle
from oracle.oracle import REPLICATED, SPLIT_ROWS, SPLIT_COLS, FUSED_ROWS
from workloads import synth
from test_oracle_shard_map import numpy_shard


def bits(t):
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def test_tp1_equals_numpy_flatnonzero():
    old, new = synth.pair_bernoulli(300 * 77, 0.03, seed=5)
    o, n = bits(old), bits(new)
    (idx, val), = oracle.encode_tensor(o, n, 300, 77, SPLIT_ROWS, None, 1)
    ref = np.flatnonzero(o != n)
    assert idx.dtype == np.int32 and val.dtype == np.uint16
    assert np.array_equal(idx, ref)
    assert np.array_equal(val, n[ref])
    out = o.copy()
    oracle.apply_segment(idx, val, out)
    ref_out = o.copy()
    ref_out[ref] = n[ref]
    assert np.array_equal(out, ref_out) and np.array_equal(out, n)


CASES = [
    (REPLICATED, 1, 100, None), (SPLIT_ROWS, 32, 9, None), (SPLIT_COLS, 7, 64, None),
    (FUSED_ROWS, 64, 5, [32, 16, 16]), (FUSED_ROWS, 48, 3, [24, 24]),
]


@pytest.mark.parametrize("rule,R,C,sec", CASES)
@pytest.mark.parametrize("D", [1, 2, 4, 8])
@pytest.mark.parametrize("p", [0.0, 0.1, 1.0])
def test_roundtrip_and_counts(rule, R, C, sec, D, p):
    old, new = synth.pair_bernoulli(R * C, p, seed=R * 31 + C + D)
    o, n = bits(old), bits(new)
    segs = oracle.encode_tensor(o, n, R, C, rule, sec, D)
    changed = int((o != n).sum())
    total = sum(idx.size for idx, _ in segs)
    assert total == changed * (D if rule == REPLICATED else 1)          # counts = popcount
    hits = np.zeros(R * C, dtype=np.int32)
    gidx = np.arange(R * C, dtype=np.int64).reshape(R, C)
    for d, (idx, val) in enumerate(segs):
        so = np.ascontiguousarray(numpy_shard(o.reshape(R, C), rule, sec, D, d)).ravel()
        sn = np.ascontiguousarray(numpy_shard(n.reshape(R, C), rule, sec, D, d)).ravel()
        sg = np.ascontiguousarray(numpy_shard(gidx, rule, sec, D, d)).ravel()
        assert (np.diff(idx.astype(np.int64)) > 0).all()                # ascending, no duplicates
        assert (idx >= 0).all() and (idx < so.size).all()
        assert (so[idx] != val).all()                                   # only real changes
        np.add.at(hits, sg[idx], 1)
        out = so.copy()
        oracle.apply_segment(idx, val, out)
        assert np.array_equal(out, sn)                                  # lossless round trip
    want = (o != n).astype(np.int32) * (D if rule == REPLICATED else 1)
    assert np.array_equal(hits, want)                                   # each change lands once per owner


def test_degenerate_cases():
    n_el = 64
    o = np.full(n_el, 0x3C00, dtype=np.uint16)
    assert oracle.encode_tensor(o, o.copy(), 8, 8, SPLIT_ROWS, None, 2)[0][0].size == 0
    n = o.copy(); n[0] ^= 1; n[-1] ^= 1                                  # first and last element
    s = oracle.encode_tensor(o, n, 8, 8, SPLIT_ROWS, None, 2)
    assert list(s[0][0]) == [0] and list(s[1][0]) == [31]
    n = o ^ np.uint16(0x8000)                                            # all changed (sign flip)
    (idx, val), = oracle.encode_tensor(o, n, 8, 8, SPLIT_COLS, None, 1)
    assert np.array_equal(idx, np.arange(64)) and np.array_equal(val, n)
    z = np.zeros(4, dtype=np.uint16); mz = z.copy(); mz[2] = 0x8000      # +0 -> -0 is a change
    (idx, val), = oracle.encode_tensor(z, mz, 1, 4, REPLICATED, None, 1)
    assert list(idx) == [2] and list(val) == [0x8000]
    nan = np.full(4, 0x7FC1, dtype=np.uint16)                            # identical NaN: no change
    assert oracle.encode_tensor(nan, nan.copy(), 1, 4, REPLICATED, None, 1)[0][0].size == 0
    e = np.empty(0, dtype=np.uint16)                                     # empty tensor
    assert oracle.encode_tensor(e, e, 0, 8, SPLIT_ROWS, None, 2)[1][0].size == 0


def test_fp32_master_input_rounds_before_comparing():
    old, new32 = synth.pair_clustered_f32(64, 40, seed=3)
    o = bits(old)
    n32 = new32.numpy().view(np.uint32)
    nb = new32.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)   # library cast as pin
    (idx, val), = oracle.encode_tensor(o, n32, 64, 40, SPLIT_ROWS, None, 1)
    ref = np.flatnonzero(o != nb)
    assert ref.size > 0 and ref.size < o.size
    assert np.array_equal(idx, ref) and np.array_equal(val, nb[ref])


def test_model_buckets_and_dense_path():
    from workloads import models
    ts = models.decoder(2, 64, 4, 2, 16, 96, 128, fused=True)
    recs = []
    for i, t, old, new in synth.model_pairs(ts, "bernoulli", seed=9, p=0.05):
        recs.append(dict(t, old=bits(old), new=bits(new)))
    D = 2
    buckets = oracle.encode_model(recs, D)
    for d in range(D):
        dsts = [np.ascontiguousarray(numpy_shard(r["old"].reshape(r["rows"], r["cols"]), r["rule"],
                                                 r["sections"], D, d)).ravel().copy() for r in recs]
        oracle.apply_bucket(buckets[d], dsts)
        for r, dst in zip(recs, dsts):
            want = np.ascontiguousarray(numpy_shard(r["new"].reshape(r["rows"], r["cols"]), r["rule"],
                                                    r["sections"], D, d)).ravel()
            assert np.array_equal(dst, want)
            assert np.array_equal(oracle.dense_shard(r["new"], r["rows"], r["cols"], r["rule"],
                                                     r["sections"], D, d), want)
        so = buckets[d]["seg_off"]
        assert so[0] == 0 and so[-1] == buckets[d]["idx"].size and (np.diff(so) >= 0).all()


def test_generator_statistics():
    n, p = 1 << 22, 0.01
    old, new = synth.pair_bernoulli(n, p, seed=0)
    nnz = int((bits(old) != bits(new)).sum())
    sigma = (n * p * (1 - p)) ** 0.5
    assert abs(nnz - n * p) < 6 * sigma
    assert abs(float(old.float().std()) - 0.02) < 1e-3
    # shifted elements moved by 1..3 units in the last place
    o, w = bits(old).astype(np.int64), bits(new).astype(np.int64)
    key = lambda b: np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)
    d = np.abs(key(w) - key(o))
    assert set(np.unique(d[d > 0])) <= {1, 2, 3}


def test_model_sizes():
    from workloads import models
    assert models.numel(models.decoder_7b()) == 6_738_415_616
    assert models.numel(models.decoder_7b(fused=False)) == 6_738_415_616
    assert models.numel(models.decoder_32b()) == 32_763_417_600
    assert len(models.decoder_32b()) == 387
