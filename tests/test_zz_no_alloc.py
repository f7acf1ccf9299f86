"""rose_delta_encode_static (the entry point for callers that cannot allocate: it works on the
library's built-in scratch array) against rose_delta_encode_ex with a caller's workspace, through
the C ABI: the buckets must come out byte-identical, on two calls in a row, the second with a
smaller input, so that what the first call left in the shared array is shown not to matter."""
import numpy as np
import pytest
import torch

import paper_2605_06534_amd as R
from workloads import models, synth

pytestmark = pytest.mark.gpu


def make(ts, tp, p, seed):
    olds, news = [], []
    for _, _, o, n in synth.model_pairs(ts, "bernoulli", seed, "cuda", p=p):
        olds.append(o)
        news.append(n)
    plan = R.shard_plan(ts, tp)
    return plan, olds, news


def encode_both(plan, olds, news, flags):
    tp, nt = plan.tp, plan.n_tensors
    old_tab, new_tab = R.ptr_table(olds), R.ptr_table(news)
    ref = [R.Bucket(plan.bucket_capacity(d), nt) for d in range(tp)]
    got = [R.Bucket(plan.bucket_capacity(d), nt) for d in range(tp)]
    for b in got:                                  # poison: whatever the call leaves untouched would show
        b.idx.fill_(-7)
        b.val.fill_(0x5A5A)
        b.seg_off.fill_(-3)
    R.delta_encode_ex(plan, old_tab, new_tab, R.BF16, flags, ref, R.workspace(plan))
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    R.delta_encode_static(plan, old_tab, new_tab, R.BF16, flags, got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before      # torch's allocator was not asked either
    for d in range(tp):
        n = R.bucket_check(plan, ref[d])
        assert R.bucket_check(plan, got[d]) == n
        assert torch.equal(got[d].seg_off, ref[d].seg_off), d
        assert torch.equal(got[d].idx[:n], ref[d].idx[:n]), d
        assert torch.equal(got[d].val[:n], ref[d].val[:n]), d
    return sum(R.bucket_check(plan, b) for b in ref)


def test_static_scratch_matches_workspace_twice_in_a_row():
    print("case: no-alloc encode, decoder tp=4 p=0.05 then a smaller decoder tp=2 p=0.3", flush=True)
    big = models.decoder(3, 1024, 16, 8, 64, 2816, 8192, fused=True)
    plan1, o1, n1 = make(big, 4, 0.05, seed=11)
    plan1.upload()
    assert plan1.workspace_bytes() <= R.binding.STATIC_SCRATCH_BYTES
    total1 = encode_both(plan1, o1, n1, 0)
    assert total1 > 0
    small = models.decoder(1, 256, 8, 4, 32, 704, 1024, fused=True)
    plan2, o2, n2 = make(small, 2, 0.3, seed=12)
    plan2.upload()
    assert plan2.n_tiles() < plan1.n_tiles()
    total2 = encode_both(plan2, o2, n2, R.ENCODE_ARITH)
    assert 0 < total2 < total1
    # and the first input again: the array now holds the smaller call's leftovers
    assert encode_both(plan1, o1, n1, 0) == total1


def test_static_scratch_rejects_what_it_cannot_hold():
    print("case: no-alloc encode, errors", flush=True)
    ts = models.decoder(1, 256, 8, 4, 32, 704, 1024, fused=True)
    plan, olds, news = make(ts, 2, 0.1, seed=13)
    buckets = [R.Bucket(plan.bucket_capacity(d), len(ts)) for d in range(2)]
    with pytest.raises(R.RoseError) as e:          # not resident yet: the call may not upload it itself
        R.delta_encode_static(plan, R.ptr_table(olds), R.ptr_table(news), R.BF16, 0, buckets)
    assert e.value.status == R.binding.ERR_SCRATCH
    # a plan whose descriptors do not fit the array: one (empty-run) tile per tensor is enough to count
    n_big = R.binding.STATIC_SCRATCH_BYTES // 8 + 1000
    huge = [dict(name="e%d" % i, rows=0, cols=8, rule=R.SPLIT_ROWS, sections=None) for i in range(n_big // 16 + 1)]
    plan_h = R.shard_plan(huge, 16)
    assert plan_h.workspace_bytes() > R.binding.STATIC_SCRATCH_BYTES
    plan_h.upload()
    hb = [R.Bucket(0, len(huge)) for _ in range(16)]
    tab = torch.zeros(len(huge), dtype=torch.int64, device="cuda")
    with pytest.raises(R.RoseError) as e:
        R.delta_encode_static(plan_h, tab, tab, R.BF16, 0, hb)
    assert e.value.status == R.binding.ERR_SCRATCH
