"""Pins for the oracle's pipeline-stage functions (Sec. 4.2 "Shard-aware Weight Transfer": TP and
PP on both sides).  `stage_of` is pinned by hand-written stage tables and by counting; the
model-level `encode_model_pp` by what must hold whatever the stage split is: with one stage on
either side it is the plain model encode; the senders of all stages together produce exactly the
plain encode's entries, each in the bucket of the stage that receives its tensor; and applying
every sender's buckets onto numpy-sliced old shards gives the numpy-sliced new shards."""
import os

import numpy as np
import pytest
import torch

from oracle import oracle
from test_oracle_shard_map import numpy_shard
from workloads import models, synth

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "stage_tables.txt")


def test_stage_of_hand_written_tables():
    rows = [tuple(int(x) for x in l.split()) for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 30
    for n_layers, pp, layer, stage in rows:
        assert oracle.stage_of(layer, n_layers, pp) == stage, (n_layers, pp, layer)


@pytest.mark.parametrize("n_layers,pp", [(4, 1), (4, 2), (4, 4), (6, 3), (36, 4), (64, 2), (64, 8)])
def test_stage_of_deals_equal_consecutive_groups(n_layers, pp):
    st = [oracle.stage_of(l, n_layers, pp) for l in range(n_layers)]
    assert st == sorted(st) and st[0] == 0 and st[-1] == pp - 1
    assert np.bincount(st, minlength=pp).tolist() == [n_layers // pp] * pp
    assert oracle.stage_of(oracle.LAYER_FIRST, n_layers, pp) == 0
    assert oracle.stage_of(oracle.LAYER_LAST, n_layers, pp) == pp - 1


def test_stage_of_rejects_what_the_reading_does_not_cover():
    for layer, n_layers, pp in [(0, 4, 3), (4, 4, 2), (-3, 4, 2), (0, 0, 1), (0, 4, 0)]:
        with pytest.raises(oracle.OracleError):
            oracle.stage_of(layer, n_layers, pp)


def small_model(layers=4, seed=3, p=0.1):
    ts = models.decoder(layers, 64, 4, 2, 16, 96, 128, fused=True)
    recs = []
    bits = lambda x: x.view(torch.int16).numpy().view(np.uint16).copy()
    for i, t, o, n in synth.model_pairs(ts, "bernoulli", seed, "cpu", p=p):
        recs.append(dict(t, old=bits(o), new=bits(n)))
    return ts, recs


def slices(recs, tp_src, s):
    """The sender's slices, cut with plain numpy slicing."""
    out = []
    for r in recs:
        cut = lambda x: np.ascontiguousarray(numpy_shard(x.reshape(r["rows"], r["cols"]), r["rule"], r["sections"],
                                                         tp_src, s)).ravel()
        out.append(dict(r, old=cut(r["old"]), new=cut(r["new"])))
    return out


def test_layers_named_by_the_workload_match_its_tensor_names():
    ts = models.decoder(4, 64, 4, 2, 16, 96, 128, fused=True)
    assert ts[0]["name"] == "embed" and ts[0]["layer"] == oracle.LAYER_FIRST
    assert [t["layer"] for t in ts[-2:]] == [oracle.LAYER_LAST] * 2
    for t in ts[1:-2]:
        assert t["name"].startswith("l%d." % t["layer"])


def test_one_stage_on_both_sides_is_the_plain_encode():
    ts, recs = small_model()
    for tp in (1, 2):
        want = oracle.encode_model(recs, tp)
        got = oracle.encode_model_pp(recs, tp, 1, 0, 4, 1, 0, 1)
        assert len(got) == tp
        for g, w in zip(got, want):
            assert np.array_equal(g["seg_off"], w["seg_off"])
            assert np.array_equal(g["idx"], w["idx"]) and np.array_equal(g["val"], w["val"])


@pytest.mark.parametrize("pp_src,pp_dst,tp_src,tp", [(2, 1, 1, 2), (1, 2, 1, 2), (2, 1, 2, 4), (4, 2, 2, 1), (2, 4, 1, 1)])
def test_all_senders_together_are_the_plain_encode_routed_by_stage(pp_src, pp_dst, tp_src, tp):
    n_layers = 4
    ts, recs = small_model(n_layers)
    plain = oracle.encode_model(recs, tp)              # what every destination shard must receive in total
    # hand table of the receiving stage per tensor for this model (embed, 6 tensors per layer, norm, head)
    per_layer = 6                                     # input norm, qkv, o, post norm, gate_up, down
    assert len(ts) == 1 + n_layers * per_layer + 2
    stage_dst = [0] + [l // (n_layers // pp_dst) for l in range(n_layers) for _ in range(per_layer)] + [pp_dst - 1] * 2
    stage_src = [0] + [l // (n_layers // pp_src) for l in range(n_layers) for _ in range(per_layer)] + [pp_src - 1] * 2
    merged = [[[] for _ in ts] for _ in range(pp_dst * tp)]          # bucket, tensor -> list of (idx, val)
    for st in range(pp_src):
        for s in range(tp_src):
            got = oracle.encode_model_pp(slices(recs, tp_src, s), tp, tp_src, s, n_layers, pp_src, st, pp_dst)
            assert len(got) == pp_dst * tp
            for b, bk in enumerate(got):
                so = bk["seg_off"]
                assert so[0] == 0 and so[-1] == bk["idx"].size and (np.diff(so) >= 0).all()
                for t in range(len(ts)):
                    a, e = int(so[t]), int(so[t + 1])
                    if e > a:
                        assert stage_src[t] == st and stage_dst[t] == b // tp, (st, s, b, t)
                        merged[b][t].append((bk["idx"][a:e], bk["val"][a:e]))
    for b in range(pp_dst * tp):
        d = b % tp
        for t in range(len(ts)):
            a, e = int(plain[d]["seg_off"][t]), int(plain[d]["seg_off"][t + 1])
            if stage_dst[t] != b // tp:
                assert not merged[b][t]
                continue
            idx = np.concatenate([x for x, _ in merged[b][t]]) if merged[b][t] else np.empty(0, np.int32)
            val = np.concatenate([v for _, v in merged[b][t]]) if merged[b][t] else np.empty(0, np.uint16)
            order = np.argsort(idx, kind="stable")     # the senders' parts of a segment interleave
            assert np.array_equal(idx[order], plain[d]["idx"][a:e]), (b, t)
            assert np.array_equal(val[order], plain[d]["val"][a:e]), (b, t)


def test_round_trip_through_different_stage_splits():
    """Training TP2 x PP2 feeds serving TP4 x PP1 (the paper's example, scaled down): every receiver
    shard, built by numpy slicing from the old weights, ends as the numpy slice of the new ones."""
    n_layers, tp_src, pp_src, tp, pp_dst = 4, 2, 2, 4, 1
    ts, recs = small_model(n_layers, seed=9, p=0.2)
    shards = [[np.ascontiguousarray(numpy_shard(r["old"].reshape(r["rows"], r["cols"]), r["rule"], r["sections"], tp, d)).ravel().copy()
               for r in recs] for d in range(tp)]
    for st in range(pp_src):
        for s in range(tp_src):
            for b, bk in enumerate(oracle.encode_model_pp(slices(recs, tp_src, s), tp, tp_src, s, n_layers, pp_src, st, pp_dst)):
                oracle.apply_bucket(bk, shards[b % tp])
    for d in range(tp):
        for r, got in zip(recs, shards[d]):
            want = np.ascontiguousarray(numpy_shard(r["new"].reshape(r["rows"], r["cols"]), r["rule"], r["sections"], tp, d)).ravel()
            assert np.array_equal(got, want), (d, r["name"])
