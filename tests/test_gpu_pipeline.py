"""GPU parity for pipeline-parallel plans (Sec. 4.2 "Shard-aware Weight Transfer": TP and PP on
both sides, e.g. training TP8 x PP2 feeding serving TP4).  Every sender (tensor-parallel rank in a
pipeline stage) encodes the slices it holds; the buckets must be the oracle's, entry by entry, and
the receivers, whose stage split differs from the senders', must end with the plainly sliced new
weights, through buckets and through transport objects."""
import numpy as np
import pytest
import torch

import paper_2605_06534_amd as R
from oracle import oracle
from workloads import models, synth
from gpu_harness import assert_buckets_equal, bits
from test_oracle_shard_map import numpy_shard

pytestmark = pytest.mark.gpu


def model(n_layers, seed, p):
    ts = models.decoder(n_layers, 256, 8, 4, 32, 704, 1024, fused=True)
    recs = []
    for _, t, o, n in synth.model_pairs(ts, "bernoulli", seed, "cpu", p=p):
        recs.append(dict(t, old=bits(o), new=bits(n)))
    return ts, recs


def cut(x, r, deg, k):
    return np.ascontiguousarray(numpy_shard(x.reshape(r["rows"], r["cols"]), r["rule"], r["sections"], deg, k)).ravel()


def dev(a):
    return torch.from_numpy(a.view(np.int16).copy()).cuda()


def sender_encode(ts, recs, tp, tp_src, s, n_layers, pp_src, st, pp_dst, dummy):
    """Plan and encode on the sender (s, st); -> plan, buckets, the oracle's buckets."""
    plan = R.shard_plan(ts, tp, tp_src, s, n_layers, pp_src, st, pp_dst)
    held = [plan.stage_of(i)[0] == st for i in range(len(ts))]
    sl = [dict(r, old=cut(r["old"], r, tp_src, s), new=cut(r["new"], r, tp_src, s)) for r in recs]
    # tensors of other stages are not on this sender: their table entries are never read (they
    # point at a few valid bytes here, which no test result depends on)
    olds = [dev(x["old"]) if h else dummy for x, h in zip(sl, held)]
    news = [dev(x["new"]) if h else dummy for x, h in zip(sl, held)]
    for i, h in enumerate(held):
        assert plan.src_numel(i) == (sl[i]["old"].size if h else 0)
        assert h or not plan.tensor_is_read(i, R.ENCODE_REFRESH)
    buckets = [R.Bucket(plan.bucket_capacity(b), len(ts)) for b in range(plan.n_buckets)]
    R.delta_encode(plan, R.ptr_table(olds), R.ptr_table(news), R.BF16, buckets, R.workspace(plan))
    torch.cuda.synchronize()
    want = oracle.encode_model_pp(sl, tp, tp_src, s, n_layers, pp_src, st, pp_dst)
    got = []
    for b in range(plan.n_buckets):
        n = R.bucket_check(plan, buckets[b])
        got.append({"idx": buckets[b].idx[:n].cpu().numpy(), "val": buckets[b].val[:n].cpu().numpy().view(np.uint16),
                    "seg_off": buckets[b].seg_off.cpu().numpy()})
        assert_buckets_equal(got[b], want[b], "sender (tp %d, stage %d) bucket %d" % (s, st, b))
    return plan, buckets, want


def receiver_shards(ts, recs, plan, tp, which, dummy):
    """Bucket b's resident copies: numpy slices of `which` for the tensors its stage holds."""
    out = []
    for b in range(plan.n_buckets):
        loc = []
        for i, r in enumerate(recs):
            if plan.local_numel(i, b) == 0:
                loc.append(dummy)
            else:
                x = cut(r[which], r, tp, b % tp)
                assert x.size == plan.local_numel(i, b)
                loc.append(dev(x))
        out.append(loc)
    return out


@pytest.mark.parametrize("n_layers,tp_src,pp_src,tp,pp_dst",
                         [(4, 2, 2, 4, 1), (4, 1, 1, 2, 2), (4, 2, 4, 2, 2), (4, 4, 1, 1, 4), (6, 1, 3, 2, 2), (6, 2, 2, 2, 3)])
def test_pipeline_senders_feed_receivers_with_another_stage_split(n_layers, tp_src, pp_src, tp, pp_dst, tile_order):
    print("case: pipeline %d layers tp_src=%d pp_src=%d -> tp=%d pp_dst=%d" % (n_layers, tp_src, pp_src, tp, pp_dst), flush=True)
    ts, recs = model(n_layers, seed=40 + pp_src, p=0.08)
    senders_feed_receivers(ts, recs, n_layers, tp_src, pp_src, tp, pp_dst)


def test_paper_example_at_full_width():
    """Sec. 4.2's example, training TP8 x PP2 -> serving TP4, on the 32B-style attention shapes at full
    width (hidden 5120, 40 query and 8 KV heads of 128: one KV head per sender; two layers, one per
    sending stage; the feed-forward width and the vocabulary cut to an eighth and a thirty-second to
    keep the host-side slicing short): every one of the 16 senders' buckets against the oracle, the
    receivers against numpy slices."""
    print("case: pipeline, 32B-style shapes, tp_src=8 pp_src=2 -> tp=4 pp_dst=1", flush=True)
    n_layers = 2
    ts = models.decoder(n_layers, 5120, 40, 8, 128, 27648 // 8, 152064 // 32, fused=True)
    recs = []
    for _, t, o, n in synth.model_pairs(ts, "bernoulli", 61, "cuda", p=0.02):       # drawn on the device, kept on the host
        recs.append(dict(t, old=bits(o), new=bits(n)))
        del o, n
    torch.cuda.empty_cache()
    senders_feed_receivers(ts, recs, n_layers, 8, 2, 4, 1)


def senders_feed_receivers(ts, recs, n_layers, tp_src, pp_src, tp, pp_dst):
    dummy = torch.zeros(64, dtype=torch.int16, device="cuda")
    # the receivers know nothing of the senders' split: their plan is made with one sending stage
    rplan = R.shard_plan(ts, tp, 1, 0, n_layers, 1, 0, pp_dst)
    by_bucket = receiver_shards(ts, recs, rplan, tp, "old", dummy)
    by_object = receiver_shards(ts, recs, rplan, tp, "old", dummy)
    tabs_b = [R.ptr_table(x) for x in by_bucket]
    tabs_o = [R.ptr_table(x) for x in by_object]
    keep = []
    for st in range(pp_src):
        for s in range(tp_src):
            plan, buckets, want = sender_encode(ts, recs, tp, tp_src, s, n_layers, pp_src, st, pp_dst, dummy)
            for b in range(plan.n_buckets):
                R.delta_apply(rplan, b, buckets[b], tabs_b[b])
                total = int(want[b]["seg_off"][-1])
                half = total // 2
                for first, n in ((half, total - half), (0, half)):          # two objects, second half first
                    obj = torch.empty(R.object_bytes(plan, n), dtype=torch.uint8, device="cuda")
                    R.bucket_pack(plan, b, buckets[b], first, n, obj)
                    assert R.object_check(rplan, obj) == (b, first, n)
                    R.object_apply(rplan, obj, tabs_o[b])
                    keep.append(obj)
            keep.append((plan, buckets))
    torch.cuda.synchronize()
    want_new = receiver_shards(ts, recs, rplan, tp, "new", dummy)
    for b in range(rplan.n_buckets):
        for i in range(len(ts)):
            if rplan.local_numel(i, b):
                assert torch.equal(by_bucket[b][i], want_new[b][i]), ("bucket", b, i, ts[i]["name"])
                assert torch.equal(by_object[b][i], want_new[b][i]), ("object", b, i, ts[i]["name"])
    assert torch.count_nonzero(dummy).item() == 0       # nothing was ever written through a stand-in pointer


def test_pipeline_object_for_a_bucket_the_receiver_does_not_have_is_turned_away():
    print("case: pipeline object with a shard word out of range", flush=True)
    n_layers = 4
    ts, recs = model(n_layers, seed=47, p=0.05)
    dummy = torch.zeros(64, dtype=torch.int16, device="cuda")
    plan, buckets, want = sender_encode(ts, recs, 2, 1, 0, n_layers, 1, 0, 2, dummy)      # 4 buckets
    b = 3
    n = int(want[b]["seg_off"][-1])
    obj = torch.empty(R.object_bytes(plan, n), dtype=torch.uint8, device="cuda")
    R.bucket_pack(plan, b, buckets[b], 0, n, obj)
    small = R.shard_plan(ts, 2, 1, 0, n_layers, 1, 0, 1)          # a receiving side with one stage: buckets 0, 1
    shards = receiver_shards(ts, recs, small, 2, "old", dummy)
    ref = [x.clone() for x in shards[1]]
    R.object_apply(small, obj, R.ptr_table(shards[1]))
    torch.cuda.synchronize()
    assert all(torch.equal(a, r) for a, r in zip(shards[1], ref))
    with pytest.raises(R.RoseError):
        R.object_check(small, obj)


def test_pipeline_sender_refresh_touches_only_its_stage():
    """Encode with sender refresh on a pipeline plan: the sender's own tensors (sent or only held, like
    the replicated ones another rank sends) end equal to the new ones, the stand-in buffer behind the
    other stages' table entries is never read or written, and the buckets are the oracle's."""
    print("case: pipeline refresh tp_src=2 pp_src=2 -> tp=4 pp_dst=1", flush=True)
    n_layers, tp, tp_src, pp_src, pp_dst = 4, 4, 2, 2, 1
    ts, recs = model(n_layers, seed=52, p=0.1)
    dummy = torch.zeros(64, dtype=torch.int16, device="cuda")
    for st in range(pp_src):
        for s in range(tp_src):
            plan = R.shard_plan(ts, tp, tp_src, s, n_layers, pp_src, st, pp_dst)
            held = [plan.stage_of(i)[0] == st for i in range(len(ts))]
            sl = [dict(r, old=cut(r["old"], r, tp_src, s), new=cut(r["new"], r, tp_src, s)) for r in recs]
            olds = [dev(x["old"]) if h else dummy for x, h in zip(sl, held)]
            news = [dev(x["new"]) if h else dummy for x, h in zip(sl, held)]
            buckets = [R.Bucket(plan.bucket_capacity(b), len(ts)) for b in range(plan.n_buckets)]
            R.delta_encode_refresh(plan, R.ptr_table(olds), R.ptr_table(news), R.BF16, buckets, R.workspace(plan))
            torch.cuda.synchronize()
            want = oracle.encode_model_pp(sl, tp, tp_src, s, n_layers, pp_src, st, pp_dst)
            for b in range(plan.n_buckets):
                n = R.bucket_check(plan, buckets[b])
                got = {"idx": buckets[b].idx[:n].cpu().numpy(), "val": buckets[b].val[:n].cpu().numpy().view(np.uint16),
                       "seg_off": buckets[b].seg_off.cpu().numpy()}
                assert_buckets_equal(got, want[b], "sender (tp %d, stage %d) bucket %d" % (s, st, b))
            for i, h in enumerate(held):
                if h:
                    assert torch.equal(olds[i], news[i]), ("not refreshed", st, s, ts[i]["name"])
                    assert plan.tensor_is_read(i, R.ENCODE_REFRESH)
    assert torch.count_nonzero(dummy).item() == 0
