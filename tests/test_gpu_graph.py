"""The whole step (encode, then apply of every bucket) captured in a HIP graph and replayed: every
replay, with the program's own eager work and synchronisations in between, must give what the
eager calls give.  The library clears its workspace with a fill kernel (never a memset node) and
allocates nothing after a plan's first device call, so the calls are capturable."""
import numpy as np
import pytest
import torch

import paper_2605_06534_amd as R
from oracle import oracle
from workloads import models, synth
from gpu_harness import bits
from test_gpu_parity import bern_case

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("entry", ["workspace", "built_in_scratch"])
def test_step_in_a_graph_replays_exactly(entry, tile_order):
    print("case: graph capture of encode + apply, %s, tile order %d" % (entry, tile_order), flush=True)
    tp = 2
    ts = models.decoder(2, 320, 8, 8, 40, 1376, 2048, fused=True)
    c = bern_case(ts, tp, 0.05, seed=90)
    recs = c.records()
    want = oracle.encode_model(recs, tp)
    old_bits = [r["old"] for r in recs]
    dst = [c.shard_init(d, old_bits) for d in range(tp)]
    tabs = [R.ptr_table(x) for x in dst]
    new_shards = [c.shard_init(d, [r["new"] for r in recs]) for d in range(tp)]

    def step():
        if entry == "workspace":
            R.delta_encode(c.plan, c.old_tab, c.new_tab, c.new_dtype, c.buckets, c.ws)
        else:                                # the entry point for callers that cannot allocate, e.g. under capture
            R.delta_encode_static(c.plan, c.old_tab, c.new_tab, c.new_dtype, 0, c.buckets)
        for d in range(tp):
            R.delta_apply(c.plan, d, c.buckets[d], tabs[d])

    c.plan.upload()                          # the built-in-scratch entry never makes a plan resident by itself
    step()                                   # eager once: warms everything
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(4):
        # eager work between replays: new weights change, the receiver is reset to the old weights
        for k, n in enumerate(c.new):
            n.copy_(torch.roll(n, 1) if rep % 2 else c.new[k])
        if rep % 2:
            recs_now = [dict(r, new=bits(n)) for r, n in zip(recs, c.new)]
        else:
            recs_now = recs
        for d in range(tp):
            for x, o in zip(dst[d], c.shard_init(d, old_bits)):
                x.copy_(o)
        for b in c.buckets:
            b.idx.fill_(-7)
            b.seg_off.fill_(-1)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        want_now = oracle.encode_model(recs_now, tp)
        for d in range(tp):
            got = c.host_bucket(d)
            assert np.array_equal(got["seg_off"], want_now[d]["seg_off"]), (rep, d)
            assert np.array_equal(got["idx"], want_now[d]["idx"]) and np.array_equal(got["val"], want_now[d]["val"]), (rep, d)
            shard_new = c.shard_init(d, [r["new"] for r in recs_now])
            for x, w in zip(dst[d], shard_new):
                assert torch.equal(x, w), (rep, d)
        # restore the original new weights for the next round
        for k, r in enumerate(recs):
            c.new[k].copy_(torch.from_numpy(r["new"].view(np.int16)).cuda().view(torch.bfloat16))
