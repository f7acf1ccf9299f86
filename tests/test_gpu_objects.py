"""GPU parity for transport objects (Sec. 4.2 "Asynchronous Weight Transfer"): objects packed on
the device are byte-identical to the oracle's, and any cut of a destination's stream into objects,
applied in any order, gives the receiver the sliced new weights; malformed objects change nothing."""
import numpy as np
import pytest
import torch

import paper_2605_06534_amd as R
from oracle import oracle
from workloads import models
from gpu_harness import Case, bits
from test_gpu_parity import bern_case

pytestmark = pytest.mark.gpu


def encode_case(tp, p, seed):
    ts = models.decoder(2, 320, 8, 8, 40, 1376, 2048, fused=True)
    c = bern_case(ts, tp, p, seed)
    c.encode()
    want = oracle.encode_model(c.records(), tp)
    return ts, c, want


@pytest.mark.parametrize("chunk", [1000, 65536, 1 << 22])
def test_objects_equal_oracle_and_apply_in_any_order(chunk):
    print("case: transport objects chunk=%d" % chunk, flush=True)
    tp = 2
    ts, c, want = encode_case(tp, 0.05, seed=31)
    recs = c.records()
    for d in range(tp):
        total = R.bucket_check(c.plan, c.buckets[d])
        assert total == want[d]["seg_off"][-1]
        objs = []
        for first in range(0, total, chunk):
            n = min(chunk, total - first)
            obj = torch.full((R.object_bytes(c.plan, n),), 0xEE, dtype=torch.uint8, device="cuda")
            assert obj.numel() == oracle.object_bytes(len(ts), n)
            R.bucket_pack(c.plan, d, c.buckets[d], first, n, obj)
            objs.append(obj)
        torch.cuda.synchronize()
        for k, first in enumerate(range(0, total, chunk)):
            n = min(chunk, total - first)
            ref = oracle.pack_object(want[d], d, first, n)
            assert np.array_equal(objs[k].cpu().numpy(), ref), (d, k)
            assert R.object_check(c.plan, objs[k]) == (d, first, n)
            assert R.object_check(c.plan, objs[k], with_payload=True)[3] == R.PAYLOAD_NEW
        old_bits = [r["old"] for r in recs]
        dst = c.shard_init(d, old_bits)
        tab = R.ptr_table(dst)
        for k in np.random.default_rng(chunk + d).permutation(len(objs)):
            R.object_apply(c.plan, objs[k], tab)
        torch.cuda.synchronize()
        new_bits = [r["new"] for r in recs]
        for g, w in zip(dst, c.shard_init(d, new_bits)):
            assert torch.equal(g, w)


def test_malformed_objects_change_nothing_and_errors_are_reported():
    print("case: malformed transport objects", flush=True)
    ts, c, want = encode_case(1, 0.05, seed=32)
    recs = c.records()
    total = R.bucket_check(c.plan, c.buckets[0])
    n = min(total, 5000)
    good = torch.zeros(R.object_bytes(c.plan, n), dtype=torch.uint8, device="cuda")
    R.bucket_pack(c.plan, 0, c.buckets[0], 0, n, good)
    torch.cuda.synchronize()
    old_bits = [r["old"] for r in recs]
    ref = c.shard_init(0, old_bits)

    def unchanged_after(obj):
        dst = c.shard_init(0, old_bits)
        R.object_apply(c.plan, obj, R.ptr_table(dst))
        torch.cuda.synchronize()
        return all(torch.equal(a, b) for a, b in zip(dst, ref))

    assert not unchanged_after(good)                       # the good object does change something
    for damage in ("magic", "version", "tensors", "count", "short", "segtable"):
        bad = good.clone()
        if damage == "magic":
            bad[0] ^= 1
        elif damage == "version":
            bad[4] = 2
        elif damage == "tensors":
            bad[12] += 1
        elif damage == "count":
            bad[26] = 1                                     # n_entries + 65536: more than the object holds
        elif damage == "short":
            bad = bad[:bad.numel() - 64].clone()
        else:
            bad[64] = 1                                     # seg_off[0] != 0
        assert unchanged_after(bad), damage
        if damage != "segtable":
            with pytest.raises(R.RoseError):
                R.object_check(c.plan, bad)
    # a range beyond the stream: packed with a zero magic, applies to nothing
    beyond = torch.zeros(R.object_bytes(c.plan, 16), dtype=torch.uint8, device="cuda")
    R.bucket_pack(c.plan, 0, c.buckets[0], total - 8, 16, beyond)
    torch.cuda.synchronize()
    assert int(beyond[:4].view(torch.int32)[0]) == 0 and unchanged_after(beyond)
    # host-side errors
    small = torch.zeros(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(R.RoseError) as e:
        R.bucket_pack(c.plan, 0, c.buckets[0], 0, n, small)
    assert e.value.status == R.binding.ERR_CAPACITY
    with pytest.raises(R.RoseError):
        R.bucket_pack(c.plan, 1, c.buckets[0], 0, n, good)
    with pytest.raises(R.RoseError):
        R.bucket_pack(c.plan, 0, c.buckets[0], -1, n, good)


def test_object_with_indices_out_of_order_changes_nothing():
    """The apply kernel gives every 64-byte piece of a tensor to one wave on the strength of the
    entries' order; an object whose indices do not ascend inside a segment is turned away whole,
    like one with a bad header."""
    print("case: transport objects with shuffled indices", flush=True)
    ts, c, want = encode_case(1, 0.05, seed=33)
    recs = c.records()
    total = R.bucket_check(c.plan, c.buckets[0])
    n = min(total, 70000)
    good = torch.zeros(R.object_bytes(c.plan, n), dtype=torch.uint8, device="cuda")
    R.bucket_pack(c.plan, 0, c.buckets[0], 0, n, good)
    torch.cuda.synchronize()
    old_bits = [r["old"] for r in recs]
    ref = c.shard_init(0, old_bits)
    idx_off = oracle.object_bytes(len(ts), 0)            # where the index array starts
    seg = good[64:64 + 8 * (len(ts) + 1)].view(torch.int64).cpu().numpy()

    def unchanged_after(obj):
        dst = c.shard_init(0, old_bits)
        R.object_apply(c.plan, obj, R.ptr_table(dst))
        torch.cuda.synchronize()
        return all(torch.equal(a, b) for a, b in zip(dst, ref))

    assert not unchanged_after(good)
    t_big = int(np.argmax(np.diff(seg)))                 # a segment with many entries
    a, b = int(seg[t_big]), int(seg[t_big + 1])
    assert b - a > 300
    for kind in ("swap_neighbours", "swap_far", "duplicate", "last_two", "segment_table_decreases"):
        bad = good.clone()
        idx = bad[idx_off:idx_off + 4 * n].view(torch.int32)
        if kind == "swap_neighbours":
            i = a + 100
            idx[i], idx[i + 1] = int(idx[i + 1]), int(idx[i])
        elif kind == "swap_far":                         # two chunks of 64 entries apart
            i, j = a + 10, a + 200
            idx[i], idx[j] = int(idx[j]), int(idx[i])
        elif kind == "duplicate":
            idx[a + 65] = int(idx[a + 64])
        elif kind == "last_two":
            idx[b - 1] = int(idx[b - 2])
        else:
            st = bad[64:64 + 8 * (len(ts) + 1)].view(torch.int64)
            st[t_big + 1] = a - 1 if a > 0 else 0
            if a == 0:
                st[t_big + 1], st[t_big] = 0, 5
        assert unchanged_after(bad), kind
    # a drop at a segment start is what a well-formed object has: still applied
    assert not unchanged_after(good)


def test_objects_of_the_7b_workload_at_64_mb():
    """Full-size: shard 1's stream of the 7B workload at 5 % cut into 64 MB objects (the paper's
    push size), applied in reverse order; the result equals applying the bucket."""
    print("case: 7B shard 1 in 64 MB objects", flush=True)
    from workloads import synth
    ts = models.decoder_7b(layers=8)
    olds, news = [], []
    for _, _, o, n in synth.model_pairs(ts, "bernoulli", 2, "cuda", p=0.05):
        olds.append(o); news.append(n)
    tp, d = 4, 1
    plan = R.shard_plan(ts, tp)
    old_tab, new_tab = R.ptr_table(olds), R.ptr_table(news)
    buckets = [R.Bucket(int(plan.bucket_capacity(k) * 0.07) + 4096, len(ts)) for k in range(tp)]
    R.delta_encode(plan, old_tab, new_tab, R.BF16, buckets, R.workspace(plan))
    total = R.bucket_check(plan, buckets[d])
    per = (64 << 20) // 6
    objs = []
    for first in range(0, total, per):
        n = min(per, total - first)
        obj = torch.empty(R.object_bytes(plan, n), dtype=torch.uint8, device="cuda")
        R.bucket_pack(plan, d, buckets[d], first, n, obj)
        objs.append(obj)
    assert len(objs) >= 2
    a = [torch.empty(plan.local_numel(t, d), dtype=torch.bfloat16, device="cuda") for t in range(len(ts))]
    R.dense_copy(plan, d, old_tab, R.BF16, R.ptr_table(a))
    b = [x.clone() for x in a]
    for obj in reversed(objs):
        R.object_apply(plan, obj, R.ptr_table(a))
    R.delta_apply(plan, d, buckets[d], R.ptr_table(b))
    want = [torch.empty_like(x) for x in a]
    R.dense_copy(plan, d, new_tab, R.BF16, R.ptr_table(want))
    torch.cuda.synchronize()
    for x, y, w in zip(a, b, want):
        assert torch.equal(x.view(torch.int16), w.view(torch.int16)) and torch.equal(y.view(torch.int16), w.view(torch.int16))
