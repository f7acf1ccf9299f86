"""GPU parity for sender-side sharding (Sec. 4.2: slice ranges on both sides, different degrees):
every sender encodes its own slices; its buckets must equal the oracle's entry by entry, and the
senders' buckets together, applied in any order, must turn the destination's sliced old weights
into the sliced new weights."""
import numpy as np
import pytest
import torch

import paper_2605_06534_amd as R
from oracle import oracle
from workloads import models, synth
from gpu_harness import bits
from test_oracle_shard_map import numpy_shard

pytestmark = pytest.mark.gpu


def np_slice(full_bits, t, tp, d):
    return np.ascontiguousarray(numpy_shard(full_bits.reshape(t["rows"], t["cols"]), t["rule"], t["sections"], tp, d)).ravel()


def run(tensors, tp, tp_src, p, seed, order=None):
    olds, news = [], []
    for _, _, o, n in synth.model_pairs(tensors, "bernoulli", seed, "cpu", p=p):
        olds.append(bits(o))
        news.append(bits(n))
    nt = len(tensors)
    dst = [[torch.from_numpy(np_slice(o, t, tp, d).view(np.int16).copy()).cuda() for t, o in zip(tensors, olds)]
           for d in range(tp)]
    dense = [[torch.full_like(x, 0x1111) for x in dst[d]] for d in range(tp)]
    total = [0] * tp
    for s in (order or range(tp_src)):
        plan = R.shard_plan(tensors, tp, tp_src, s)
        so = [torch.from_numpy(np_slice(o, t, tp_src, s).view(np.int16).copy()).cuda() for t, o in zip(tensors, olds)]
        sn = [torch.from_numpy(np_slice(n, t, tp_src, s).view(np.int16).copy()).cuda() for t, n in zip(tensors, news)]
        for i in range(nt):
            assert plan.src_numel(i) == so[i].numel()
        old_tab, new_tab = R.ptr_table(so), R.ptr_table(sn)
        ws = R.workspace(plan)
        buckets = [R.Bucket(plan.bucket_capacity(d), nt) for d in range(tp)]
        R.delta_encode(plan, old_tab, new_tab, R.BF16, buckets, ws)
        torch.cuda.synchronize()
        want = [oracle.encode_tensor_src(np_slice(o, t, tp_src, s), np_slice(n, t, tp_src, s), t["rows"], t["cols"],
                                         t["rule"], t["sections"], tp, tp_src, s,
                                         sends_replicated=(i % tp_src == s))
                for i, (t, o, n) in enumerate(zip(tensors, olds, news))]
        for d in range(tp):
            seg = buckets[d].seg_off.cpu().numpy()
            assert R.bucket_check(plan, buckets[d]) == seg[-1]
            total[d] += int(seg[-1])
            for i in range(nt):
                a, b = int(seg[i]), int(seg[i + 1])
                assert b - a == want[i][d][0].size, (s, d, i, tensors[i]["name"])
                assert np.array_equal(buckets[d].idx[a:b].cpu().numpy(), want[i][d][0]), (s, d, i)
                assert np.array_equal(buckets[d].val[a:b].cpu().numpy().view(np.uint16), want[i][d][1]), (s, d, i)
            R.delta_apply(plan, d, buckets[d], R.ptr_table(dst[d]))
            R.dense_copy(plan, d, new_tab, R.BF16, R.ptr_table(dense[d]))
        torch.cuda.synchronize()
    for d in range(tp):
        for i, (t, n) in enumerate(zip(tensors, news)):
            w = np_slice(n, t, tp, d)
            assert np.array_equal(dst[d][i].cpu().numpy().view(np.uint16), w), ("apply", d, i)
            assert np.array_equal(dense[d][i].cpu().numpy().view(np.uint16), w), ("dense", d, i)
    return total


@pytest.mark.parametrize("tp_src,tp", [(2, 4), (4, 2), (8, 4), (4, 1), (2, 2), (8, 8), (2, 8), (1, 4)])
def test_small_decoder_between_degrees(tp_src, tp):
    print("case: sender-side sharding tp_src=%d tp=%d" % (tp_src, tp), flush=True)
    ts = models.decoder(2, 512, 8, 8, 64, 1408, 2048, fused=True)
    run(ts, tp, tp_src, 0.05, seed=tp_src * 10 + tp)


def test_unfused_gqa_and_reverse_sender_order():
    print("case: sender-side sharding, separate q/k/v, senders applied in reverse", flush=True)
    ts = models.decoder(1, 1024, 16, 8, 64, 2816, 4096, fused=False)
    run(ts, 4, 8, 0.2, seed=3, order=[7, 6, 5, 4, 3, 2, 1, 0])


def test_odd_widths_take_the_element_path():
    """Column blocks that are not multiples of 8 elements: neither side can use 128-bit accesses."""
    print("case: sender-side sharding, odd widths", flush=True)
    T = lambda r, c, rule, sec=None: dict(name="t", rows=r, cols=c, rule=rule, sections=sec)
    ts = [T(12, 20, R.SPLIT_COLS), T(20, 3, R.SPLIT_ROWS), T(1, 37, R.REPLICATED), T(24, 5, R.FUSED_ROWS, [16, 8]),
          T(300, 44, R.SPLIT_COLS)]
    run(ts, 2, 4, 0.5, seed=9)
    run(ts, 4, 2, 0.5, seed=10)


def test_full_width_training_to_rollout_8b_layer():
    """The paper's 8B setup: training TP=4, rollout TP=1 (Sec. 5); two layers at full width."""
    print("case: 8B shapes, 2 layers, tp_src=4 -> tp=1", flush=True)
    ts = models.decoder_8b(layers=2)
    ts = [t for t in ts if t["name"] not in ("embed", "lm_head")] + [dict(name="embed", rows=151936 // 8, cols=4096,
                                                                       rule=R.SPLIT_ROWS, sections=None)]
    run(ts, 1, 4, 0.02, seed=4)


@pytest.mark.parametrize("tp_src,tp", [(3, 1), (6, 2), (6, 3), (2, 1), (1, 3)])
def test_pieces_of_a_single_column(tp_src, tp):
    """Column splits so fine that a sender (or a destination) holds one column per row: runs of one
    element, for which the kernel's index arithmetic has no magic divisor."""
    print("case: single-column pieces tp_src=%d tp=%d" % (tp_src, tp), flush=True)
    ts = [dict(name="c6", rows=25, cols=6, rule=R.SPLIT_COLS, sections=None),
          dict(name="c6b", rows=3000, cols=6, rule=R.SPLIT_COLS, sections=None),
          dict(name="r", rows=6, cols=5, rule=R.SPLIT_ROWS, sections=None),
          dict(name="n", rows=1, cols=77, rule=R.REPLICATED, sections=None)]
    run(ts, tp, tp_src, 0.3, seed=10 * tp_src + tp)


@pytest.mark.parametrize("tp_src,tp", [(1, 4), (4, 4), (8, 4), (2, 8), (4, 1)])
def test_group_interleaved_qkv_from_the_training_side(tp_src, tp):
    """Fused QKV kept interleaved by KV-head group on the sender side (built with numpy), plainly
    stacked on the destination side: GQA shapes with 8 groups of 5 query heads."""
    from test_oracle_src_sharding import interleave_by_groups
    print("case: group-interleaved qkv tp_src=%d tp=%d" % (tp_src, tp), flush=True)
    hd, G, qpg, H = 16, 8, 5, 256
    sec = [G * qpg * hd, G * hd, G * hd]
    rows = sum(sec)
    t = dict(name="qkv", rows=rows, cols=H, rule=R.FUSED_ROWS, sections=sec, src_groups=G)
    o, n = synth.pair_bernoulli(rows * H, 0.05, seed=tp_src * 100 + tp)
    o, n = bits(o).reshape(rows, H), bits(n).reshape(rows, H)
    oi, ni = interleave_by_groups(o, sec, G), interleave_by_groups(n, sec, G)
    per = rows // tp_src
    dst = [torch.from_numpy(np_slice(o.ravel(), t, tp, d).view(np.int16).copy()).cuda() for d in range(tp)]
    for s in range(tp_src):
        so = torch.from_numpy(np.ascontiguousarray(oi[s * per:(s + 1) * per]).view(np.int16).copy()).cuda()
        sn = torch.from_numpy(np.ascontiguousarray(ni[s * per:(s + 1) * per]).view(np.int16).copy()).cuda()
        plan = R.shard_plan([t], tp, tp_src, s)
        buckets = [R.Bucket(plan.bucket_capacity(d), 1) for d in range(tp)]
        R.delta_encode(plan, R.ptr_table([so]), R.ptr_table([sn]), R.BF16, buckets, R.workspace(plan))
        torch.cuda.synchronize()
        want = oracle.encode_tensor_src(oi[s * per:(s + 1) * per], ni[s * per:(s + 1) * per], rows, H, R.FUSED_ROWS, sec,
                                        tp, tp_src, s, src_groups=G)
        for d in range(tp):
            cnt = R.bucket_check(plan, buckets[d])
            assert cnt == want[d][0].size, (s, d)
            assert np.array_equal(buckets[d].idx[:cnt].cpu().numpy(), want[d][0]), (s, d)
            assert np.array_equal(buckets[d].val[:cnt].cpu().numpy().view(np.uint16), want[d][1]), (s, d)
            R.delta_apply(plan, d, buckets[d], R.ptr_table([dst[d]]))
        torch.cuda.synchronize()
    for d in range(tp):
        assert np.array_equal(dst[d].cpu().numpy().view(np.uint16), np_slice(n.ravel(), t, tp, d)), d
