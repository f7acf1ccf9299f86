"""GPU parity of the arithmetic payload (Sec. 4.2 states the update as W_t = W_{t-1} + dW_t):
buckets written with ENCODE_ARITH equal the oracle's arithmetic buckets entry by entry (index with
its escape bit, value), and applying them to the receiver's old shards gives the new shards bit
for bit: through the bucket, and through transport objects."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import paper_2605_06534_amd as R
from oracle import oracle
from workloads import models, synth
from gpu_harness import Case, assert_buckets_equal, bits
from test_gpu_parity import bern_case, T
from test_oracle_shard_map import numpy_shard

pytestmark = pytest.mark.gpu


def any_case(tensors, tp, p, seed, **kw):
    olds, news = [], []
    for i, t, o, n in synth.model_pairs(tensors, "any_patterns", seed, "cpu", p=p):
        olds.append(o); news.append(n)
    return Case(tensors, tp, olds, news, **kw)


def shard_of(c, bits_list, d):
    return [np.ascontiguousarray(numpy_shard(b.reshape(t["rows"], t["cols"]), t["rule"], t["sections"], c.tp, d)).ravel()
            for t, b in zip(c.tensors, bits_list)]


def check_arith(c, flags=R.ENCODE_ARITH, objects=False, min_escape=None):
    recs = c.records()
    old_bits = [r["old"] for r in recs]
    new_bits = [r["new"] if r["new"].dtype == np.uint16 else oracle.rne_bf16(r["new"]) for r in recs]
    plain = oracle.encode_model(recs, c.tp)
    R.delta_encode_ex(c.plan, c.old_tab, c.new_tab, c.new_dtype, flags, c.buckets, c.ws)
    torch.cuda.synchronize()
    n_esc = n_all = 0
    for d in range(c.tp):
        want = oracle.arith_bucket(plain[d], shard_of(c, old_bits, d))
        assert R.bucket_check(c.plan, c.buckets[d]) == want["seg_off"][-1]
        got = c.host_bucket(d)
        assert_buckets_equal(got, want, "shard %d" % d)
        n_esc += int((want["idx"] < 0).sum()); n_all += want["idx"].size
        # receiver: old shards + bucket -> new shards
        dst = c.shard_init(d, old_bits)
        tab = R.ptr_table(dst)
        if objects:
            total = int(want["seg_off"][-1])
            cuts = sorted({0, total // 3, min(total, total // 3 + 1), (2 * total) // 3, total})
            objs = []
            for a, b in zip(cuts[:-1], cuts[1:]):
                obj = torch.empty(R.object_bytes(c.plan, b - a), dtype=torch.uint8, device="cuda")
                R.bucket_pack_ex(c.plan, d, c.buckets[d], R.PAYLOAD_ARITH, a, b - a, obj)
                assert R.object_check(c.plan, obj, with_payload=True) == (d, a, b - a, R.PAYLOAD_ARITH)
                objs.append(obj)
            for obj in reversed(objs):                    # any order
                R.object_apply(c.plan, obj, tab)
        else:
            R.delta_apply_ex(c.plan, d, c.buckets[d], R.PAYLOAD_ARITH, tab)
        torch.cuda.synchronize()
        ref = [x.copy() for x in shard_of(c, old_bits, d)]
        oracle.apply_bucket_arith(want, ref)
        for t, (g, r, nb) in enumerate(zip(dst, ref, shard_of(c, new_bits, d))):
            gb = bits(g)
            assert np.array_equal(gb, r), "apply shard %d tensor %d" % (d, t)
            assert np.array_equal(gb, nb), "round trip shard %d tensor %d" % (d, t)
    if flags & R.ENCODE_REFRESH:
        for i, (o, nb) in enumerate(zip(c.old, new_bits)):
            assert np.array_equal(bits(o), nb), ("old not refreshed", i)
    if min_escape is not None:
        assert n_all > 0 and n_esc >= min_escape * n_all, (n_esc, n_all)
    return n_esc, n_all


@pytest.mark.parametrize("tp", [1, 4])
def test_arith_small_decoder_small_steps(tp):
    """steps of a few units in the last place: nearly every entry carries a true difference"""
    print("case: arith small decoder tp=%d" % tp, flush=True)
    ts = models.decoder(2, 320, 8, 8, 40, 1376, 2048, fused=True)
    n_esc, n_all = check_arith(bern_case(ts, tp, 0.05, seed=70 + tp))
    assert n_esc < 0.02 * n_all


@pytest.mark.parametrize("tp,p", [(2, 0.02), (4, 0.3)])
def test_arith_any_patterns(tp, p):
    """infinities, NaNs, subnormals, both zeros, large jumps: many escapes, still lossless"""
    print("case: arith any patterns tp=%d p=%g" % (tp, p), flush=True)
    ts = models.decoder(2, 320, 8, 8, 40, 1376, 2048, fused=True)
    check_arith(any_case(ts, tp, p, seed=80 + tp), min_escape=0.1)


def test_arith_odd_shapes_full_tiles_and_misaligned():
    print("case: arith odd shapes", flush=True)
    ts = [T(1, 8191, R.REPLICATED), T(64, 37, R.SPLIT_ROWS), T(37, 64, R.SPLIT_COLS), T(1, 3 * 8192 + 5, R.REPLICATED),
          T(48, 129, R.FUSED_ROWS, [32, 16]), T(6, 8200, R.SPLIT_ROWS)]
    check_arith(any_case(ts, 2, 0.2, seed=90))
    # every element changes: more entries per tile than the kernel can park
    check_arith(any_case(ts, 2, 1.0, seed=91))
    # tensors at odd byte offsets (no 128-bit loads, direct stores on apply)
    olds, news = [], []
    for i, t, o, n in synth.model_pairs(ts, "any_patterns", 92, "cpu", p=0.2):
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
    check_arith(c)


def test_arith_fp32_master():
    print("case: arith fp32 master", flush=True)
    ts = models.decoder(1, 256, 8, 4, 32, 704, 1024, fused=True)
    olds, news = [], []
    for i, t, o, n in synth.model_pairs(ts, "clustered_f32", 7, "cpu", vocab_active=200):
        olds.append(o); news.append(n)
    check_arith(Case(ts, 4, olds, news))


@pytest.mark.parametrize("f32", [False, True])
def test_arith_with_refresh(f32):
    print("case: arith with refresh f32=%s" % f32, flush=True)
    if f32:
        ts = models.decoder(1, 256, 8, 4, 32, 704, 1024, fused=True)
        olds, news = [], []
        for i, t, o, n in synth.model_pairs(ts, "clustered_f32", 8, "cpu", vocab_active=200):
            olds.append(o); news.append(n)
        c = Case(ts, 4, olds, news)
    else:
        ts = models.decoder(2, 320, 8, 8, 40, 1376, 2048, fused=True)
        c = any_case(ts, 4, 0.1, seed=95)
    check_arith(c, flags=R.ENCODE_ARITH | R.ENCODE_REFRESH)


def test_arith_objects_any_order():
    print("case: arith objects", flush=True)
    ts = models.decoder(2, 320, 8, 8, 40, 1376, 2048, fused=True)
    check_arith(any_case(ts, 2, 0.05, seed=97), objects=True)


def test_ex_with_no_flags_is_plain_encode_and_bad_arguments():
    print("case: encode_ex flags", flush=True)
    ts = models.decoder(1, 256, 8, 4, 32, 704, 1024, fused=True)
    c = bern_case(ts, 2, 0.05, seed=98)
    want = oracle.encode_model(c.records(), c.tp)
    R.delta_encode_ex(c.plan, c.old_tab, c.new_tab, c.new_dtype, 0, c.buckets, c.ws)
    torch.cuda.synchronize()
    for d in range(c.tp):
        assert_buckets_equal(c.host_bucket(d), want[d], "shard %d" % d)
    with pytest.raises(R.RoseError):
        R.delta_encode_ex(c.plan, c.old_tab, c.new_tab, c.new_dtype, 4, c.buckets, c.ws)
    dst = c.shard_init(0, [r["old"] for r in c.records()])
    with pytest.raises(R.RoseError):
        R.delta_apply_ex(c.plan, 0, c.buckets[0], 2, R.ptr_table(dst))
    obj = torch.empty(R.object_bytes(c.plan, 4), dtype=torch.uint8, device="cuda")
    with pytest.raises(R.RoseError):
        R.bucket_pack_ex(c.plan, 0, c.buckets[0], 7, 0, 4, obj)
    # a plain bucket applied through apply_ex(PAYLOAD_NEW) is rose_delta_apply
    R.delta_apply_ex(c.plan, 0, c.buckets[0], R.PAYLOAD_NEW, R.ptr_table(dst))
    torch.cuda.synchronize()
    new_bits = [r["new"] for r in c.records()]
    for g, nb in zip(dst, shard_of(c, new_bits, 0)):
        assert np.array_equal(bits(g), nb)


def test_arith_every_pattern_pair():
    """All 2^32 (old, new) pairs of 16-bit patterns: escape bit and value of every entry equal the
    oracle's, and applying gives back the new pattern.  Blocks of 8192 old patterns x all new ones;
    the oracle side runs on a thread pool (its C routine, one old pattern per call)."""
    B = 8192
    ts = [T(B, 65536, R.REPLICATED)]
    plan = R.shard_plan(ts, 1)
    ws = R.workspace(plan)
    bucket = [R.Bucket(B * 65536, 1)]
    lib = oracle._load()
    news = np.arange(65536, dtype=np.uint16)

    def oracle_block(o0):
        esc = np.empty((B, 65536), dtype=np.uint8)
        val = np.empty((B, 65536), dtype=np.uint16)

        def one(i):
            idx = np.arange(65536, dtype=np.int32)
            v = news.copy()
            old = np.full(65536, o0 + i, dtype=np.uint16)
            assert lib.orc_arith_from_overwrite(idx.ctypes.data, v.ctypes.data, 65536, old.ctypes.data, 65536) == 0
            esc[i] = idx < 0
            val[i] = v
        with ThreadPoolExecutor(16) as ex:
            list(ex.map(one, range(B)))
        return esc, val

    def as_bf16(x):
        return (((x + 0x8000) & 0xFFFF) - 0x8000).to(torch.int16).view(torch.bfloat16)

    new = as_bf16(torch.arange(65536, dtype=torch.int32, device="cuda").repeat(B))
    for o0 in range(0, 65536, B):
        print("case: arith all pairs, old patterns %04x..%04x" % (o0, o0 + B - 1), flush=True)
        esc, val = oracle_block(o0)
        old = as_bf16(torch.arange(o0, o0 + B, dtype=torch.int32, device="cuda").repeat_interleave(65536))
        R.delta_encode_ex(plan, R.ptr_table([old]), R.ptr_table([new]), R.BF16, R.ENCODE_ARITH, bucket, ws)
        torch.cuda.synchronize()
        n = R.bucket_check(plan, bucket[0])
        assert n == B * 65536 - B
        idx, v = bucket[0].idx[:n], bucket[0].val[:n]
        pos = (idx & 0x7FFFFFFF).long()
        assert torch.equal(pos, torch.nonzero(old.view(torch.int16) != new.view(torch.int16)).ravel())
        w_esc = torch.from_numpy(esc.ravel()).cuda()
        w_val = torch.from_numpy(val.ravel().view(np.int16)).cuda()
        assert torch.equal((idx < 0).to(torch.uint8), w_esc[pos]), "escape bits, block %04x" % o0
        assert torch.equal(v.view(torch.int16), w_val[pos]), "values, block %04x" % o0
        dst = old.clone()
        R.delta_apply_ex(plan, 0, bucket[0], R.PAYLOAD_ARITH, R.ptr_table([dst]))
        torch.cuda.synchronize()
        assert torch.equal(dst.view(torch.int16), new.view(torch.int16)), "apply, block %04x" % o0
        del old, dst, pos, w_esc, w_val


def test_arith_few_workers_dense_changes(tile_order):
    """Arithmetic payloads through the regime where tiles are counted first and walked again (two
    tickets of one group in a row) and where tiles are too dense to park, with and without refresh."""
    ts = models.decoder(2, 1024, 16, 16, 64, 2816, 4096, fused=True)
    pairs = 0
    for workers, p, flags in [(66, 0.6, R.ENCODE_ARITH), (70, 0.9, R.ENCODE_ARITH | R.ENCODE_REFRESH),
                              (97, 1.0, R.ENCODE_ARITH)]:
        print("case: arith few workers=%d p=%g flags=%d" % (workers, p, flags), flush=True)
        c = any_case(ts, 2, p, seed=workers)
        c.plan.set_worker_cap(workers)
        check_arith(c, flags=flags)
        pairs += int(c.ws.view(torch.int32)[2])
    assert pairs > 0, "the pair handling never ran: the test does not reach what it is for"


def test_arith_sender_side_sharding():
    """A sender that holds its own slice only (degree 2, interleaved fused QKV) towards 4 destinations."""
    print("case: arith sender-side sharding", flush=True)
    ts = models.decoder(1, 256, 8, 4, 32, 704, 1024, fused=True)
    for t in ts:
        t["src_groups"] = 4 if t["name"].endswith("qkv") else 0
    olds, news = [], []
    for i, t, o, n in synth.model_pairs(ts, "any_patterns", 99, "cpu", p=0.1):
        olds.append(o); news.append(n)
    tp, tp_src = 4, 2
    full_old, full_new = [bits(o) for o in olds], [bits(n) for n in news]
    recs = [dict(t, old=o, new=n) for t, o, n in zip(ts, full_old, full_new)]
    dst_old = [[oracle.dense_shard(r["old"], r["rows"], r["cols"], r["rule"], r["sections"], tp, d) for r in recs]
               for d in range(tp)]
    dst_new = [[oracle.dense_shard(r["new"], r["rows"], r["cols"], r["rule"], r["sections"], tp, d) for r in recs]
               for d in range(tp)]
    shards = [[torch.from_numpy(x.view(np.int16).copy()).cuda() for x in dst_old[d]] for d in range(tp)]
    for s in range(tp_src):
        plan = R.shard_plan(ts, tp, tp_src, s)
        cut = R.shard_plan(ts, tp_src)                     # cuts the sender's slices with the library's dense path
        so = [torch.empty(cut.local_numel(i, s), dtype=torch.bfloat16, device="cuda") for i in range(len(ts))]
        sn = [torch.empty_like(x) for x in so]
        # the sender's slices under its own (group-interleaved) layout come from the oracle
        for i, r in enumerate(recs):
            for src, dstt in ((r["old"], so[i]), (r["new"], sn[i])):
                sl = oracle_src_slice(r, src, tp_src, s)
                dstt.copy_(torch.from_numpy(sl.view(np.int16).copy()).view(torch.bfloat16))
        buckets = [R.Bucket(plan.bucket_capacity(d), len(ts)) for d in range(tp)]
        ws = R.workspace(plan)
        R.delta_encode_ex(plan, R.ptr_table(so), R.ptr_table(sn), R.BF16, R.ENCODE_ARITH, buckets, ws)
        torch.cuda.synchronize()
        for d in range(tp):
            per_t = [oracle.encode_tensor_src(bits(so[i]), bits(sn[i]), r["rows"], r["cols"], r["rule"], r["sections"],
                                              tp, tp_src, s, sends_replicated=(i % tp_src == s),
                                              src_groups=r.get("src_groups", 0))[d] for i, r in enumerate(recs)]
            seg = np.zeros(len(ts) + 1, dtype=np.int64)
            for i, (ix, _) in enumerate(per_t):
                seg[i + 1] = seg[i] + ix.size
            plain = {"idx": np.concatenate([x[0] for x in per_t]), "val": np.concatenate([x[1] for x in per_t]),
                     "seg_off": seg}
            want = oracle.arith_bucket(plain, dst_old[d])
            n = R.bucket_check(plan, buckets[d])
            got = {"idx": buckets[d].idx[:n].cpu().numpy(), "val": buckets[d].val[:n].cpu().numpy().view(np.uint16),
                   "seg_off": buckets[d].seg_off.cpu().numpy()}
            assert_buckets_equal(got, want, "sender %d shard %d" % (s, d))
            R.delta_apply_ex(plan, d, buckets[d], R.PAYLOAD_ARITH, R.ptr_table(shards[d]))
        torch.cuda.synchronize()
    for d in range(tp):
        for i in range(len(ts)):
            assert np.array_equal(bits(shards[d][i]), dst_new[d][i]), (d, i)


def oracle_src_slice(r, full_bits, tp_src, s):
    """The sender's slice of a full tensor under the sender-side layout (numpy, test side): the plain
    shard, or for a group-interleaved fused tensor an equal row block of the interleaved matrix."""
    from test_oracle_src_sharding import interleave_by_groups
    g = r.get("src_groups", 0)
    x = full_bits.reshape(r["rows"], r["cols"])
    if not g:
        return np.ascontiguousarray(numpy_shard(x, r["rule"], r["sections"], tp_src, s)).ravel()
    xi = interleave_by_groups(x, r["sections"], g)
    per = r["rows"] // tp_src
    return np.ascontiguousarray(xi[s * per:(s + 1) * per]).ravel()
