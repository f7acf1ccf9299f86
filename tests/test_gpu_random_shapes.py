"""Seeded sweep over random small parameter sets: random rules, shapes (odd widths, empty tensors,
tensors of several tiles), degrees and densities, each checked entry by entry against the oracle
(encode, apply, dense copy), with the default and with the arithmetic payload."""
import numpy as np
import pytest
import torch

import paper_2605_06534_amd as R
from gpu_harness import full_parity
from test_gpu_arith import any_case, check_arith
from test_gpu_parity import bern_case, T

pytestmark = pytest.mark.gpu


def random_tensors(rng, tp):
    ts = []
    for _ in range(int(rng.integers(1, 7))):
        kind = int(rng.integers(0, 4))
        wide = rng.random() < 0.3                              # some tensors span several 8192-element tiles
        if kind == 0:
            ts.append(T(int(rng.integers(1, 4)), int(rng.integers(1, 30000 if wide else 600)), R.REPLICATED))
        elif kind == 1:
            ts.append(T(tp * int(rng.integers(0, 40)), int(rng.integers(1, 2000 if wide else 300)), R.SPLIT_ROWS))
        elif kind == 2:
            ts.append(T(int(rng.integers(1, 300 if wide else 40)), tp * int(rng.integers(1, 200 if wide else 40)),
                        R.SPLIT_COLS))
        else:
            sec = [tp * int(rng.integers(0, 20)) for _ in range(int(rng.integers(1, 4)))]
            if sum(sec) == 0:
                sec[0] = tp
            ts.append(T(sum(sec), int(rng.integers(1, 1500 if wide else 200)), R.FUSED_ROWS, sec))
    return ts


@pytest.mark.parametrize("seed", range(40))
def test_random_parameter_sets(seed, tile_order):
    rng = np.random.default_rng(1000 + seed)
    tp = int(rng.choice([1, 2, 3, 4, 8]))
    p = [0.003, 0.05, 0.3, 1.0, 0.0][seed % 5]
    ts = random_tensors(rng, tp)
    print("case: random set seed=%d tp=%d p=%g shapes=%s" %
          (seed, tp, p, [(t["rows"], t["cols"], t["rule"], t["sections"]) for t in ts]), flush=True)
    full_parity(bern_case(ts, tp, p, seed=seed))
    flags = R.ENCODE_ARITH | (R.ENCODE_REFRESH if seed % 2 else 0)
    check_arith(any_case(ts, tp, p, seed=seed + 500), flags=flags, objects=(seed % 3 == 0))


@pytest.mark.parametrize("seed", [278] + list(range(24)))
def test_random_parameter_sets_from_sharded_senders(seed, tile_order):
    """The same kind of random sets, sent by every sender of a random degree to a random destination
    degree (seed 278: one column per sender and row, found by a longer run of this sweep)."""
    import math
    from test_gpu_src_sharding import run
    rng = np.random.default_rng(5000 + seed)
    tp = int(rng.choice([1, 2, 3, 4, 8]))
    tp_src = int(rng.choice([1, 2, 3, 4, 6, 8]))
    ts = random_tensors(rng, tp * tp_src // math.gcd(tp, tp_src))
    p = [0.003, 0.05, 0.3, 1.0][seed % 4]
    print("case: random set from senders seed=%d tp_src=%d tp=%d p=%g shapes=%s" %
          (seed, tp_src, tp, p, [(t["rows"], t["cols"], t["rule"], t["sections"]) for t in ts]), flush=True)
    run(ts, tp, tp_src, p, seed)
