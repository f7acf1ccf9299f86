"""Full-size GPU checks, in the launch configuration bench.py times: the library runs on the
whole synthetic parameter set; the oracle is compared entry by entry on sampled tensors (it
computes any single tensor in well under a second), and properties that hold at any size are
checked on everything with plain torch ops: counts equal the popcount of the change mask,
indices ascend inside a segment, and applying every bucket turns the receiver's copy of the old
weights into the plainly sliced new weights, bit for bit."""
import gc

import numpy as np
import pytest
import torch

import paper_2605_06534_amd as R
from oracle import oracle
from workloads import models, synth

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def free_device_memory_first():
    """Every test here sizes itself by the free device memory: blocks that earlier tests left in
    torch's cache must not decide whether a configuration runs."""
    gc.collect()
    torch.cuda.empty_cache()
    yield
    gc.collect()
    torch.cuda.empty_cache()


def torch_shard(x, t, tp, d):
    """Shard d of the full 2-D tensor x by plain slicing (test-side statement of the layout)."""
    x = x.view(t["rows"], t["cols"])
    rule = t["rule"]
    if rule == R.REPLICATED:
        return x.reshape(-1)
    if rule == R.SPLIT_ROWS:
        n = t["rows"] // tp
        return x[d * n:(d + 1) * n].reshape(-1)
    if rule == R.SPLIT_COLS:
        n = t["cols"] // tp
        return x[:, d * n:(d + 1) * n].reshape(-1)
    parts, row0 = [], 0
    for s in t["sections"]:
        n = s // tp
        parts.append(x[row0 + d * n:row0 + (d + 1) * n])
        row0 += s
    return torch.cat(parts, 0).reshape(-1)


def host_bits(t):
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.float32:
        return t.view(torch.int32).numpy().view(np.uint32)
    return t.view(torch.int16).numpy().view(np.uint16)


def new_as_bf16(n):
    return n.to(torch.bfloat16) if n.dtype == torch.float32 else n


def run_and_check(tensors, tp, recipe, seed, sample, density=None, cap_frac=None, arith=False, window=None, **kw):
    dev = "cuda"
    olds, news = [], []
    for _, _, o, n in synth.model_pairs(tensors, recipe, seed, dev, **kw):
        olds.append(o)
        news.append(n)
    new_dtype = R.FP32_RNE if news[0].dtype == torch.float32 else R.BF16
    plan = R.shard_plan(tensors, tp)
    old_tab, new_tab = R.ptr_table(olds), R.ptr_table(news)
    ws = R.workspace(plan)
    if cap_frac is None:
        cap_frac = min(1.0, 1.3 * density + 0.002)
    buckets = [R.Bucket(int(plan.bucket_capacity(d) * cap_frac) + 4096, len(tensors)) for d in range(tp)]
    print("  encode", flush=True)
    if arith:
        R.delta_encode_ex(plan, old_tab, new_tab, new_dtype, R.ENCODE_ARITH, buckets, ws)
    else:
        R.delta_encode(plan, old_tab, new_tab, new_dtype, buckets, ws)
    torch.cuda.synchronize()
    totals = [R.bucket_check(plan, b) for b in buckets]
    seg = [b.seg_off.cpu().numpy() for b in buckets]

    # property: counts = popcount of the mask (times tp for replicated tensors)
    print("  counts", flush=True)
    grand = 0
    for i, (t, o, n) in enumerate(zip(tensors, olds, news)):
        changed = int((o.view(torch.int16) != new_as_bf16(n).view(torch.int16)).sum())
        got = sum(int(seg[d][i + 1] - seg[d][i]) for d in range(tp))
        assert got == changed * (tp if t["rule"] == R.REPLICATED else 1), (i, t["name"])
        grand += got
    assert grand == sum(totals)
    for d in range(tp):
        assert seg[d][0] == 0 and seg[d][-1] == totals[d] and (np.diff(seg[d]) >= 0).all()

    # property: indices ascend strictly inside every segment (checked on the whole bucket at once:
    # a drop in the index stream may only happen at a segment boundary)
    print("  order", flush=True)
    for d in range(tp):
        idx = buckets[d].idx[:totals[d]]
        if arith:
            idx = idx & 0x7FFFFFFF                      # bit 31 marks an escaped entry
        if totals[d] > 1:
            drops = torch.nonzero(idx[1:] <= idx[:-1]).flatten() + 1
            starts = set(int(x) for x in seg[d])
            assert all(int(x) in starts for x in drops.cpu()), "shard %d" % d

    # oracle parity on the sampled tensors, every shard
    print("  oracle on %d sampled tensors" % len(sample), flush=True)
    for i in sample:
        t = tensors[i]
        want = oracle.encode_tensor(host_bits(olds[i]), host_bits(news[i]), t["rows"], t["cols"], t["rule"],
                                    t["sections"], tp)
        for d in range(tp):
            a, b = int(seg[d][i]), int(seg[d][i + 1])
            if arith:
                old_local = oracle.dense_shard(host_bits(olds[i]), t["rows"], t["cols"], t["rule"], t["sections"], tp, d)
                ab = oracle.arith_bucket({"idx": want[d][0], "val": want[d][1],
                                          "seg_off": np.array([0, want[d][0].size], dtype=np.int64)}, [old_local])
                want[d] = (ab["idx"], ab["val"])
            assert b - a == want[d][0].size, (i, d)
            assert np.array_equal(buckets[d].idx[a:b].cpu().numpy(), want[d][0]), (i, d)
            assert np.array_equal(buckets[d].val[a:b].cpu().numpy().view(np.uint16), want[d][1]), (i, d)

    # oracle parity on a window of elements of a single flat tensor (tp = 1): the entries whose index
    # falls inside it are the oracle's entries of the window's elements, shifted by its start
    if window is not None:
        assert tp == 1 and len(tensors) == 1
        a, w = window
        print("  oracle on elements [%d, %d)" % (a, a + w), flush=True)
        o, n = olds[0].view(torch.int16), new_as_bf16(news[0]).view(torch.int16)
        lo = int((o[:a] != n[:a]).sum())
        idx_w, val_w = oracle.encode_tensor(host_bits(olds[0][a:a + w]), host_bits(news[0][a:a + w]), 1, w,
                                            R.REPLICATED, None, 1)[0]
        assert idx_w.size > 0
        assert np.array_equal(buckets[0].idx[lo:lo + idx_w.size].cpu().numpy(), idx_w + a)
        assert np.array_equal(buckets[0].val[lo:lo + idx_w.size].cpu().numpy().view(np.uint16), val_w)
        if lo + idx_w.size < totals[0]:
            assert int(buckets[0].idx[lo + idx_w.size]) >= a + w

    # property: apply(encode(old, new), slice(old)) == slice(new), all tensors, all shards
    print("  apply + round trip", flush=True)
    for d in range(tp):
        dst = [torch_shard(o, t, tp, d).clone() for t, o in zip(tensors, olds)]
        if arith:
            R.delta_apply_ex(plan, d, buckets[d], R.PAYLOAD_ARITH, R.ptr_table(dst))
        else:
            R.delta_apply(plan, d, buckets[d], R.ptr_table(dst))
        torch.cuda.synchronize()
        for i, (t, n) in enumerate(zip(tensors, news)):
            want = torch_shard(new_as_bf16(n), t, tp, d)
            assert torch.equal(dst[i].view(torch.int16), want.view(torch.int16)), (d, i, t["name"])
        if d == tp - 1:   # dense path against the same slicing, last shard
            R.dense_copy(plan, d, new_tab, new_dtype, R.ptr_table(dst))
            torch.cuda.synchronize()
            for i, (t, n) in enumerate(zip(tensors, news)):
                assert torch.equal(dst[i].view(torch.int16), torch_shard(new_as_bf16(n), t, tp, d).view(torch.int16))
        del dst
    del olds, news, buckets
    torch.cuda.empty_cache()
    return totals


def test_decoder7b_tp4_p05(tile_order):
    """7B-style decoder, TP=4, Bernoulli(0.05): the workload bench.py times."""
    print("case: decoder7b tp=4 p=0.05 seed=0", flush=True)
    ts = models.decoder_7b()
    # embed, a norm, fused qkv, o (column blocks), gate_up, down of the first layer; the last
    # layer's down, the final norm and lm_head
    sample = [0, 1, 2, 3, 5, 6, len(ts) - 3, len(ts) - 2, len(ts) - 1]
    totals = run_and_check(ts, 4, "bernoulli", 0, sample, density=0.05, p=0.05)
    n = models.numel(ts)
    assert abs(sum(totals) - 0.05 * n) < 6 * (n * 0.05 * 0.95) ** 0.5 + 0.05 * 4 * 65 * 4096


def test_decoder7b_tp4_p05_arithmetic_payload():
    """The same workload with arithmetic payloads (rounded differences, escapes where adding back
    would not be exact): sampled tensors against the oracle, round trip on everything."""
    print("case: decoder7b tp=4 p=0.05 seed=0 arith", flush=True)
    ts = models.decoder_7b()
    sample = [0, 1, 2, 3, 5, 6, len(ts) - 1]
    run_and_check(ts, 4, "bernoulli", 0, sample, density=0.05, arith=True, p=0.05)


@pytest.mark.parametrize("p", [0.001, 0.01, 0.1, 0.5])
def test_flat_2pow30_density_sweep(p, tile_order):
    """One flat 2^30-element tensor, TP=1, int32 indices up to 2^30 - 1."""
    print("case: flat 2^30 p=%g seed=0" % p, flush=True)
    # the oracle on the whole tensor at the low densities, on a window of 2^24 elements that starts in
    # the middle of a tile at the high ones
    totals = run_and_check(models.flat(1 << 30), 1, "bernoulli", 0, sample=[0] if p <= 0.01 else [], density=p, p=p,
                           window=None if p <= 0.01 else ((1 << 29) + 12345, 1 << 24))
    n = 1 << 30
    assert abs(totals[0] - p * n) < 6 * (n * p * (1 - p)) ** 0.5


def test_decoder32b_tp8_p02(tile_order):
    """32B-style GQA decoder, TP=8 (one KV head per shard), Bernoulli(0.02); old + new are 131 GB resident."""
    print("case: decoder32b tp=8 p=0.02 seed=0 tile order %d" % tile_order, flush=True)
    free, _ = torch.cuda.mem_get_info()
    if free < 165e9:
        pytest.skip("needs about 160 GB of free device memory")
    ts = models.decoder_32b()
    sample = [1, 2, 3, 5, 6, len(ts) - 2]          # norm, GQA qkv, o, gate_up, down, final norm
    run_and_check(ts, 8, "bernoulli", 0, sample, density=0.02, p=0.02)


@pytest.mark.parametrize("tp", [1, 4])
def test_decoder8b_shapes(tp, tile_order):
    """8B-style GQA decoder (the paper's smaller model), at the rollout side's TP=1 and the training
    side's TP=4; Bernoulli(0.02)."""
    print("case: decoder8b tp=%d p=0.02 seed=1 tile order %d" % (tp, tile_order), flush=True)
    ts = models.decoder_8b()
    sample = [0, 1, 2, 3, 5, 6, len(ts) - 2, len(ts) - 1]
    run_and_check(ts, tp, "bernoulli", 1, sample, density=0.02, p=0.02)


def test_decoder32b_tp8_fp32_master_clustered(tile_order):
    """fp32-master input with per-row Beta(0.5, 20) change rates on the whole 32B-style set: old
    (65.5 GB) and the fp32 new weights (131 GB) are resident, the receiver's shards are built and
    checked one shard at a time."""
    print("case: decoder32b tp=8 clustered fp32 seed=0 tile order %d" % tile_order, flush=True)
    free, _ = torch.cuda.mem_get_info()
    if free < 245e9:
        pytest.skip("needs about 240 GB of free device memory, %.0f GB are free" % (free / 1e9))
    ts = models.decoder_32b()
    sample = [0, 2, 3, 6, len(ts) - 1]
    run_and_check(ts, 8, "clustered_f32", 0, sample, cap_frac=0.03, vocab_active=20000)


def test_decoder32b_tp8_fp32_master_clustered_8_layers():
    """The same input recipe on 8 of the 64 layers (about 40 GB): runs on any box, whatever else holds memory."""
    print("case: decoder32b (8 layers) tp=8 clustered fp32 seed=0", flush=True)
    ts = models.decoder_32b(layers=8)
    sample = [0, 2, 3, 6, len(ts) - 1]
    run_and_check(ts, 8, "clustered_f32", 0, sample, cap_frac=0.03, vocab_active=20000)


def test_largest_local_tensor_two_shards():
    """The largest local tensor the int32 index admits (2^31 - 8 elements per shard), two shards, so
    that global element numbers pass 2^32: every entry against torch.nonzero on the shard's slice,
    with changes planted at the first and last element of each shard."""
    n = (1 << 31) - 8
    print("case: 2 x (2^31 - 8) split rows tp=2 p=0.001 seed=5", flush=True)
    free, _ = torch.cuda.mem_get_info()
    if free < 40e9:
        pytest.skip("needs about 35 GB of free device memory")
    ts = [dict(name="big", rows=2, cols=n, rule=R.SPLIT_ROWS, sections=None)]
    old, new = synth.pair_bernoulli(2 * n, 0.001, 5, "cuda")
    ob, nb = old.view(torch.int16), new.view(torch.int16)
    for g in (0, n - 1, n, 2 * n - 1):
        nb[g] = ob[g] ^ 0x0101
    plan = R.shard_plan(ts, 2)
    ws = R.workspace(plan)
    buckets = [R.Bucket(int(n * 0.0015), 1) for _ in range(2)]
    R.delta_encode(plan, R.ptr_table([old]), R.ptr_table([new]), R.BF16, buckets, ws)
    torch.cuda.synchronize()
    for d in range(2):
        o, w = ob[d * n:(d + 1) * n], nb[d * n:(d + 1) * n]
        want = torch.nonzero(o != w).ravel()
        total = R.bucket_check(plan, buckets[d])
        assert total == want.numel()
        assert int(want[0]) == 0 and int(want[-1]) == n - 1
        assert torch.equal(buckets[d].idx[:total].long(), want)
        assert torch.equal(buckets[d].val[:total].view(torch.int16), w[want])
        dst = o.clone()
        R.delta_apply(plan, d, buckets[d], R.ptr_table([dst]))
        torch.cuda.synchronize()
        assert torch.equal(dst, w)
        del dst, want
