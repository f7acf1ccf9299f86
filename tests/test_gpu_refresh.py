"""GPU tests of encode with sender refresh (Sec. 4.2: the sender keeps W_{t-1} resident): the
buckets are the oracle's, and afterwards the old tensors hold the new weights as bf16, bit for
bit (what "refreshed" means needs no oracle beyond the pinned round-to-nearest-even cast)."""
import numpy as np
import pytest
import torch

import paper_2605_06534_amd as R
from oracle import oracle
from workloads import models, synth
from gpu_harness import Case, assert_buckets_equal, bits, host_new
from test_gpu_parity import bern_case, T
from test_oracle_shard_map import numpy_shard

pytestmark = pytest.mark.gpu


def check_refresh(c):
    recs = c.records()
    want = oracle.encode_model(recs, c.tp)
    R.delta_encode_refresh(c.plan, c.old_tab, c.new_tab, c.new_dtype, c.buckets, c.ws)
    torch.cuda.synchronize()
    for d in range(c.tp):
        assert R.bucket_check(c.plan, c.buckets[d]) == want[d]["seg_off"][-1]
        assert_buckets_equal(c.host_bucket(d), want[d], "shard %d" % d)
    for i, (o, r) in enumerate(zip(c.old, recs)):
        nb = r["new"] if r["new"].dtype == np.uint16 else oracle.rne_bf16(r["new"])
        assert np.array_equal(bits(o), nb), ("old not refreshed", i, c.tensors[i]["name"])
    # a second step with the same new weights finds nothing
    R.delta_encode_refresh(c.plan, c.old_tab, c.new_tab, c.new_dtype, c.buckets, c.ws)
    torch.cuda.synchronize()
    assert all(R.bucket_check(c.plan, b) == 0 for b in c.buckets)


@pytest.mark.parametrize("tp", [1, 4])
@pytest.mark.parametrize("p", [0.01, 0.3])
def test_refresh_small_decoder(tp, p, tile_order):
    print("case: refresh small decoder tp=%d p=%g" % (tp, p), flush=True)
    ts = models.decoder(2, 320, 8, 8, 40, 1376, 2048, fused=True)
    check_refresh(bern_case(ts, tp, p, seed=50 + tp))


def test_refresh_odd_shapes_and_misaligned():
    print("case: refresh odd shapes", flush=True)
    ts = [T(1, 8191, R.REPLICATED), T(64, 37, R.SPLIT_ROWS), T(37, 64, R.SPLIT_COLS), T(1, 3 * 8192 + 5, R.REPLICATED),
          T(48, 129, R.FUSED_ROWS, [32, 16]), T(6, 8200, R.SPLIT_ROWS)]
    check_refresh(bern_case(ts, 2, 0.2, seed=60))
    # tensors at odd byte offsets
    olds, news = [], []
    for i, t, o, n in synth.model_pairs(ts, "bernoulli", 61, "cpu", p=0.2):
        olds.append(o); news.append(n)
    c = Case(ts, 2, olds, news)
    pool_o = torch.zeros(sum(x.numel() for x in olds) + 64, dtype=torch.bfloat16, device="cuda")
    pool_n = torch.zeros_like(pool_o)
    off, c.old, c.new = 1, [], []
    for o, n in zip(olds, news):
        a, b = pool_o[off:off + o.numel()], pool_n[off:off + n.numel()]
        a.copy_(o); b.copy_(n)
        c.old.append(a); c.new.append(b)
        off += o.numel() + 1
    c.old_tab, c.new_tab = R.ptr_table(c.old), R.ptr_table(c.new)
    check_refresh(c)


def test_refresh_fp32_master():
    print("case: refresh fp32 master", flush=True)
    ts = models.decoder(1, 256, 8, 4, 32, 704, 1024, fused=True)
    olds, news = [], []
    for i, t, o, n in synth.model_pairs(ts, "clustered_f32", 7, "cpu", vocab_active=200):
        olds.append(o); news.append(n)
    check_refresh(Case(ts, 4, olds, news))


def test_refresh_few_workers_dense(tile_order):
    """The regime where tiles are walked twice (two tickets of one group in a row): a tile must
    not be refreshed before its second walk."""
    print("case: refresh few workers", flush=True)
    ts = models.decoder(2, 1024, 16, 16, 64, 2816, 4096, fused=True)
    pairs = 0
    for workers, p in [(66, 0.6), (70, 0.9)]:
        c = bern_case(ts, 2, p, seed=workers)
        c.plan.set_worker_cap(workers)
        recs = c.records()
        want = oracle.encode_model(recs, 2)
        R.delta_encode_refresh(c.plan, c.old_tab, c.new_tab, c.new_dtype, c.buckets, c.ws)
        torch.cuda.synchronize()
        pairs += int(c.ws.view(torch.int32)[2])
        for d in range(2):
            assert_buckets_equal(c.host_bucket(d), want[d], "shard %d" % d)
        for o, r in zip(c.old, recs):
            assert np.array_equal(bits(o), r["new"])
    assert pairs > 0


def test_refresh_on_a_sender_side_plan():
    """Sender 1 of 2: its slices are refreshed, and so are the replicated tensors it holds but
    does not send."""
    print("case: refresh with sender-side sharding", flush=True)
    ts = models.decoder(2, 512, 8, 8, 64, 1408, 2048, fused=True)
    tp, tp_src, s = 4, 2, 1
    olds, news = [], []
    for _, _, o, n in synth.model_pairs(ts, "bernoulli", 70, "cpu", p=0.05):
        olds.append(bits(o)); news.append(bits(n))
    sl = lambda x, t: np.ascontiguousarray(numpy_shard(x.reshape(t["rows"], t["cols"]), t["rule"], t["sections"], tp_src, s)).ravel()
    so = [torch.from_numpy(sl(o, t).view(np.int16).copy()).cuda() for t, o in zip(ts, olds)]
    sn = [torch.from_numpy(sl(n, t).view(np.int16).copy()).cuda() for t, n in zip(ts, news)]
    plan = R.shard_plan(ts, tp, tp_src, s)
    buckets = [R.Bucket(plan.bucket_capacity(d), len(ts)) for d in range(tp)]
    R.delta_encode_refresh(plan, R.ptr_table(so), R.ptr_table(sn), R.BF16, buckets, R.workspace(plan))
    torch.cuda.synchronize()
    for i, t in enumerate(ts):
        want = oracle.encode_tensor_src(sl(olds[i], t), sl(news[i], t), t["rows"], t["cols"], t["rule"], t["sections"],
                                        tp, tp_src, s, sends_replicated=(i % tp_src == s))
        for d in range(tp):
            seg = buckets[d].seg_off.cpu().numpy()
            a, b = int(seg[i]), int(seg[i + 1])
            assert np.array_equal(buckets[d].idx[a:b].cpu().numpy(), want[d][0]), (i, d)
        assert torch.equal(so[i], sn[i]), ("not refreshed", i, t["name"])
