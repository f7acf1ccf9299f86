"""Shared plumbing of the GPU parity tests: move a seeded workload to the card, run the library
through its C ABI, bring the buckets back and compare them with the oracle entry by entry."""
import numpy as np
import torch

import paper_2605_06534_amd as R
from oracle import oracle
from test_oracle_shard_map import numpy_shard


def bits(t):
    """bf16 / int16 torch tensor (any device) -> numpy uint16 copy on the host."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16).copy()


def host_new(t):
    """new weights -> numpy uint16 (bf16) or uint32 (fp32 master) patterns on the host."""
    if t.dtype == torch.float32:
        return t.detach().cpu().contiguous().view(torch.int32).numpy().view(np.uint32).copy()
    return bits(t)


class Case:
    """A parameter set on the GPU with everything encode / apply need."""

    def __init__(self, tensors, tp, olds, news, capacity=None, slack=1.0):
        self.tensors, self.tp = tensors, tp
        self.old = [o.cuda() for o in olds]
        self.new = [n.cuda() for n in news]
        self.new_dtype = R.FP32_RNE if self.new and self.new[0].dtype == torch.float32 else R.BF16
        self.plan = R.shard_plan(tensors, tp)
        self.old_tab = R.ptr_table(self.old)
        self.new_tab = R.ptr_table(self.new)
        self.ws = R.workspace(self.plan)
        caps = [int(self.plan.bucket_capacity(d) * slack) if capacity is None else capacity for d in range(tp)]
        self.buckets = [R.Bucket(c, len(tensors)) for c in caps]

    def records(self):
        return [dict(t, old=bits(o), new=host_new(n)) for t, o, n in zip(self.tensors, self.old, self.new)]

    def encode(self):
        R.delta_encode(self.plan, self.old_tab, self.new_tab, self.new_dtype, self.buckets, self.ws)
        torch.cuda.synchronize()

    def host_bucket(self, d):
        b = self.buckets[d]
        so = b.seg_off.cpu().numpy()
        n = int(min(so[-1], b.capacity))
        return {"idx": b.idx[:n].cpu().numpy(), "val": b.val[:n].cpu().numpy().view(np.uint16), "seg_off": so}

    def shard_init(self, d, src_bits):
        """Receiver copies of shard d built by plain numpy slicing of the given full tensors."""
        out = []
        for t, fb in zip(self.tensors, src_bits):
            s = np.ascontiguousarray(numpy_shard(fb.reshape(t["rows"], t["cols"]), t["rule"],
                                                 t["sections"], self.tp, d)).ravel()
            out.append(torch.from_numpy(s.view(np.int16).copy()).cuda())
        return out


def assert_buckets_equal(got, want, what=""):
    assert np.array_equal(got["seg_off"], want["seg_off"]), what + " seg_off"
    assert got["idx"].size == want["idx"].size, what + " count"
    assert np.array_equal(got["idx"], want["idx"]), what + " idx"
    assert np.array_equal(got["val"], want["val"]), what + " val"


def full_parity(case, check_dense=True):
    """encode == oracle buckets, apply == oracle apply == sliced new, dense copy == oracle."""
    recs = case.records()
    want = oracle.encode_model(recs, case.tp)
    case.encode()
    for d in range(case.tp):
        got = case.host_bucket(d)
        assert R.bucket_check(case.plan, case.buckets[d]) == want[d]["seg_off"][-1]
        assert_buckets_equal(got, want[d], "shard %d" % d)
    old_bits = [r["old"] for r in recs]
    new_bits = [r["new"] if r["new"].dtype == np.uint16 else oracle.rne_bf16(r["new"]) for r in recs]
    for d in range(case.tp):
        dst = case.shard_init(d, old_bits)
        tab = R.ptr_table(dst)
        R.delta_apply(case.plan, d, case.buckets[d], tab)
        torch.cuda.synchronize()
        ref = [x.cpu().numpy().view(np.uint16).copy() for x in case.shard_init(d, old_bits)]
        oracle.apply_bucket(want[d], ref)
        for t, (g, r) in enumerate(zip(dst, ref)):
            gb = g.cpu().numpy().view(np.uint16)
            assert np.array_equal(gb, r), "apply shard %d tensor %d" % (d, t)
            s = np.ascontiguousarray(numpy_shard(new_bits[t].reshape(case.tensors[t]["rows"], case.tensors[t]["cols"]),
                                                 case.tensors[t]["rule"], case.tensors[t]["sections"], case.tp, d)).ravel()
            assert np.array_equal(gb, s), "round trip shard %d tensor %d" % (d, t)
        if check_dense:
            dd = [torch.full_like(x, 0x5A5A) for x in dst]
            R.dense_copy(case.plan, d, case.new_tab, case.new_dtype, R.ptr_table(dd))
            torch.cuda.synchronize()
            for t, g in enumerate(dd):
                tt = case.tensors[t]
                w = oracle.dense_shard(new_bits[t], tt["rows"], tt["cols"], tt["rule"], tt["sections"], case.tp, d)
                assert np.array_equal(g.cpu().numpy().view(np.uint16), w), "dense shard %d tensor %d" % (d, t)
    return want
