"""The library's own choice of tile order: from the density that rose_bucket_check read back for
the plan's last launch (timed below 4 %, neighbours below 7.5 %, spread above), whatever the buckets
could hold; the buckets are the oracle's in every case."""
import pytest
import torch

import paper_2605_06534_amd as R
from paper_2605_06534_amd import binding
from workloads import models
from gpu_harness import full_parity
from test_gpu_parity import bern_case

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("p,want", [(0.02, binding.TILE_ORDER_TIMED), (0.055, binding.TILE_ORDER_NEIGHBOURS),
                                    (0.12, binding.TILE_ORDER_SPREAD)])
def test_order_follows_the_density_read_back(p, want):
    print("case: auto tile order at p=%g" % p, flush=True)
    ts = models.decoder(2, 512, 8, 8, 64, 1408, 4096, fused=True)
    c = bern_case(ts, 4, p, seed=7)
    caps = [b.capacity for b in c.buckets]
    full = [c.plan.bucket_capacity(d) for d in range(4)]
    assert c.plan.pick_tile_order(full) == binding.TILE_ORDER_SPREAD          # nothing known, nothing bounded
    full_parity(c)                                                             # encodes, checks every bucket, applies
    assert c.plan.pick_tile_order(full) == want
    assert c.plan.pick_tile_order(caps) == want
    full_parity(c)                                                             # the launch in the picked order
    torch.cuda.synchronize()
