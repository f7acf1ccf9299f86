"""Host-side checks of the C-ABI library that need no GPU: every declared symbol is exported,
the planner's tables agree with the oracle's shard map, argument errors are reported."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2605_06534_amd as R
from paper_2605_06534_amd import binding
from oracle import oracle
from workloads import models

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "rose_delta.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(rose_[a-z0-9_]+)\s*\(", header))
    assert {"rose_shard_plan_create", "rose_delta_encode", "rose_delta_apply"} <= declared
    lib = ctypes.CDLL(binding._LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(binding.EXPORTS)


SHAPES = [
    (R.REPLICATED, 1, 40, None), (R.REPLICATED, 3, 5, None),
    (R.SPLIT_ROWS, 16, 3, None), (R.SPLIT_ROWS, 8, 16, None),
    (R.SPLIT_COLS, 3, 16, None), (R.SPLIT_COLS, 5, 64, None), (R.SPLIT_COLS, 1, 32, None),
    (R.SPLIT_COLS, 7, 8, None),
    (R.FUSED_ROWS, 32, 8, [16, 8, 8]), (R.FUSED_ROWS, 24, 3, [8, 0, 16]), (R.FUSED_ROWS, 8, 4, [8]),
]


@pytest.mark.parametrize("tp", [1, 2, 4, 8])
def test_planner_tables_match_oracle_map(tp):
    ts = [dict(name="t%d" % i, rows=r, cols=c, rule=rule, sections=sec)
          for i, (rule, r, c, sec) in enumerate(SHAPES)]
    plan = R.shard_plan(ts, tp)
    assert plan.n_tensors == len(ts) and plan.tp == tp
    base = 0
    for i, t in enumerate(ts):
        assert plan.tensor_base(i) == base
        base += t["rows"] * t["cols"]
        for d in range(tp):
            assert plan.local_numel(i, d) == oracle.local_numel(t["rule"], t["rows"], t["cols"], tp)
        for g in range(t["rows"] * t["cols"]):
            want = oracle.shard_map(t["rule"], t["rows"], t["cols"], t["sections"], tp,
                                    g // t["cols"], g % t["cols"])
            assert plan.map_index(i, g) == want, (i, g)
    assert plan.tensor_base(len(ts)) == base
    assert plan.bucket_capacity(0) == sum(plan.local_numel(i, 0) for i in range(len(ts)))
    assert plan.workspace_bytes() >= 8 * plan.n_tiles()


@pytest.mark.parametrize("tp_src,tp", [(2, 4), (4, 2), (8, 4), (4, 1), (2, 2), (8, 8), (2, 8)])
def test_sender_side_plan_matches_oracle_maps(tp_src, tp):
    """Sender holds shard s of tp_src: element g of its slice is element (r, c) of the full tensor
    (found by inverting the oracle's map for degree tp_src by brute force) and goes where the
    oracle's map for degree tp sends (r, c)."""
    shapes = [s for s in SHAPES if s[0] == R.REPLICATED or
              (s[0] == R.SPLIT_ROWS and s[1] % 8 == 0) or (s[0] == R.SPLIT_COLS and s[2] % 8 == 0) or
              (s[0] == R.FUSED_ROWS and all(x % 8 == 0 for x in s[3]))]
    ts = [dict(name="t%d" % i, rows=r, cols=c, rule=rule, sections=sec) for i, (rule, r, c, sec) in enumerate(shapes)]
    for s in range(tp_src):
        plan = R.shard_plan(ts, tp, tp_src, s)
        cap = [0] * tp
        for i, t in enumerate(ts):
            assert plan.src_numel(i) == oracle.local_numel(t["rule"], t["rows"], t["cols"], tp_src)
            sends = t["rule"] != R.REPLICATED or i % tp_src == s
            for r in range(t["rows"]):
                for c in range(t["cols"]):
                    s_first, n_src, g = oracle.shard_map(t["rule"], t["rows"], t["cols"], t["sections"], tp_src, r, c)
                    if not (s_first <= s < s_first + n_src):
                        continue
                    want = oracle.shard_map(t["rule"], t["rows"], t["cols"], t["sections"], tp, r, c)
                    got = plan.map_index(i, g)
                    if sends:
                        assert got == want, (s, i, r, c)
                        for d in range(want[0], want[0] + want[1]):
                            cap[d] += 1
                    else:
                        assert got[1] == 0
        assert [plan.bucket_capacity(d) for d in range(tp)] == cap


@pytest.mark.parametrize("sec,C,G", [([32, 8, 8], 5, 8), ([16, 16, 16], 8, 4), ([24, 24], 2, 4)])
@pytest.mark.parametrize("tp_src,tp", [(1, 1), (1, 4), (2, 4), (4, 2), (4, 4), (2, 1)])
def test_group_interleaved_sender_plan(sec, C, G, tp_src, tp):
    """The sender's layout is built with numpy (a tensor holding its own plain index, interleaved by
    group, cut in row blocks); every element of a slice must go where the oracle's map sends the
    plain element it is."""
    import numpy as np
    from test_oracle_src_sharding import interleave_by_groups
    if G % tp_src or any(x % tp for x in sec):
        pytest.skip("degree does not divide")
    rows = sum(sec)
    t = dict(name="qkv", rows=rows, cols=C, rule=R.FUSED_ROWS, sections=sec, src_groups=G)
    plain = np.arange(rows * C, dtype=np.int64).reshape(rows, C)
    inter = interleave_by_groups(plain, sec, G)
    per = rows // tp_src
    for s in range(tp_src):
        plan = R.shard_plan([t], tp, tp_src, s)
        sl = inter[s * per:(s + 1) * per].ravel()
        for g_s, g in enumerate(sl):
            want = oracle.shard_map(R.FUSED_ROWS, rows, C, sec, tp, int(g) // C, int(g) % C)
            assert plan.map_index(0, g_s) == want, (s, g_s)


def test_group_interleaving_argument_errors():
    bad = [dict(rows=8, cols=4, rule=R.SPLIT_ROWS, sections=None, src_groups=2),
           dict(rows=12, cols=4, rule=R.FUSED_ROWS, sections=[8, 2, 2], src_groups=4)]
    for t in bad:
        with pytest.raises(R.RoseError):
            R.shard_plan([t], 1)
    with pytest.raises(R.RoseError):          # 4 groups cannot be split over 8 senders
        R.shard_plan([dict(rows=48, cols=4, rule=R.FUSED_ROWS, sections=[16, 16, 16], src_groups=4)], 1, 8, 0)


def test_sender_side_plan_argument_errors():
    t = [dict(rows=8, cols=8, rule=R.SPLIT_ROWS, sections=None)]
    for tp_src, rank, status in [(3, 0, binding.ERR_SHAPE), (2, 2, binding.ERR_ARG), (2, -1, binding.ERR_ARG),
                                 (0, 0, binding.ERR_ARG), (32, 0, binding.ERR_UNSUPPORTED)]:
        with pytest.raises(R.RoseError) as e:
            R.shard_plan(t, 2, tp_src, rank)
        assert e.value.status == status, (tp_src, rank)


def test_large_shapes_sampled_against_oracle():
    ts = models.decoder(1, 5120, 40, 8, 128, 27648, 152064)
    plan = R.shard_plan(ts, 8)
    import random
    rnd = random.Random(0)
    for i, t in enumerate(ts):
        n = t["rows"] * t["cols"]
        for g in [0, n - 1] + [rnd.randrange(n) for _ in range(20)]:
            want = oracle.shard_map(t["rule"], t["rows"], t["cols"], t["sections"], 8,
                                    g // t["cols"], g % t["cols"])
            assert plan.map_index(i, g) == want


def test_argument_errors():
    def plan(rows, cols, rule, tp, sections=None):
        return R.shard_plan([dict(rows=rows, cols=cols, rule=rule, sections=sections)], tp)

    for args, status in [
        ((6, 4, R.SPLIT_ROWS, 4), binding.ERR_SHAPE),
        ((4, 6, R.SPLIT_COLS, 4), binding.ERR_SHAPE),
        ((12, 4, R.FUSED_ROWS, 4, [8, 2, 2]), binding.ERR_SHAPE),
        ((12, 4, R.FUSED_ROWS, 4, [8, 8]), binding.ERR_SHAPE),
        ((12, 4, R.FUSED_ROWS, 4), binding.ERR_ARG),            # no sections
        ((4, 4, 7, 2), binding.ERR_ARG),                        # unknown rule
        ((-1, 4, R.SPLIT_ROWS, 1), binding.ERR_ARG),
        ((4, 4, R.SPLIT_ROWS, 0), binding.ERR_ARG),
        ((32, 4, R.SPLIT_ROWS, 32), binding.ERR_UNSUPPORTED),   # tp above ROSE_MAX_TP
        ((1, 1 << 31, R.REPLICATED, 1), binding.ERR_UNSUPPORTED),   # local numel >= 2^31
        ((1 << 20, 1 << 45, R.REPLICATED, 1), binding.ERR_UNSUPPORTED),
    ]:
        with pytest.raises(R.RoseError) as e:
            plan(*args)
        assert e.value.status == status, args
    with pytest.raises(R.RoseError):
        R.shard_plan([], 1)
    p = plan(8, 8, R.SPLIT_ROWS, 2)
    for bad in (lambda: p.local_numel(1, 0), lambda: p.local_numel(0, 2), lambda: p.map_index(0, 64),
                lambda: p.bucket_capacity(-1), lambda: p.tensor_base(2)):
        with pytest.raises(R.RoseError):
            bad()
    # a 2^31 - 8 element flat tensor at TP = 1 is the largest accepted local size class
    assert plan(1, (1 << 31) - 8, R.REPLICATED, 1).local_numel(0, 0) == (1 << 31) - 8
    # the bound is on the destination's local size: the sender's slice (here the whole tensor, past
    # 2^32 elements) is addressed with 64-bit offsets
    n = (1 << 31) - 8
    big = plan(2, n, R.SPLIT_ROWS, 2)
    assert big.local_numel(0, 1) == n and big.src_numel(0) == 2 * n
    assert big.map_index(0, 2 * n - 1) == (1, 1, n - 1) and big.map_index(0, n) == (1, 1, 0)
    assert big.map_index(0, n - 1) == (0, 1, n - 1)


def test_empty_tensor_gets_a_tile():
    p = R.shard_plan([dict(rows=0, cols=8, rule=R.SPLIT_ROWS, sections=None),
                      dict(rows=4, cols=8, rule=R.SPLIT_ROWS, sections=None)], 2)
    assert p.n_tiles() == 4 and p.local_numel(0, 1) == 0


def test_pp_stage_helper_partitions_the_model():
    from workloads import models
    ts = models.decoder_8b(layers=8)
    for pp in (1, 2, 4, 8):
        got = [i for st in range(pp) for i, _ in models.pp_stage(ts, 8, pp, st)]
        assert got == list(range(len(ts)))
    assert models.pp_stage(ts, 8, 4, 0)[0][1]["name"] == "embed"
    assert models.pp_stage(ts, 8, 4, 3)[-1][1]["name"] == "lm_head"
    assert models.numel(models.decoder_8b()) == 8190726144


def test_planner_matches_oracle_map_on_random_parameter_sets():
    """The parameter sets of the GPU sweep (random rules, odd widths, empty tensors, several tiles),
    on the host: every element's destination and local index from the planner's tables against the
    oracle's shard map, and the sizes the plan reports against the oracle's."""
    from test_gpu_random_shapes import random_tensors
    rng0 = np.random.default_rng(7)
    for seed in range(40):
        rng = np.random.default_rng(1000 + seed)
        tp = int(rng.choice([1, 2, 3, 4, 8]))
        ts = random_tensors(rng, tp)
        plan = R.shard_plan(ts, tp)
        cap = [0] * tp
        for i, t in enumerate(ts):
            n = t["rows"] * t["cols"]
            assert plan.src_numel(i) == n
            for d in range(tp):
                assert plan.local_numel(i, d) == oracle.local_numel(t["rule"], t["rows"], t["cols"], tp)
                cap[d] += oracle.local_numel(t["rule"], t["rows"], t["cols"], tp)
            if n == 0:
                continue
            picks = np.unique(np.concatenate([[0, n - 1], rng0.integers(0, n, 300)]))
            for g in picks:
                want = oracle.shard_map(t["rule"], t["rows"], t["cols"], t["sections"], tp, int(g) // t["cols"],
                                        int(g) % t["cols"])
                assert plan.map_index(i, int(g)) == want, (seed, i, int(g))
        for d in range(tp):
            assert plan.bucket_capacity(d) == cap[d]


def test_which_pointer_table_entries_a_launch_reads():
    """A replicated tensor is sent by one sender (ordinal mod tp_src); the others read its pointers
    only when they refresh their own copy.  Empty tensors are never read."""
    ts = [dict(name="n0", rows=1, cols=64, rule=R.REPLICATED, sections=None),
          dict(name="w", rows=16, cols=8, rule=R.SPLIT_ROWS, sections=None),
          dict(name="n1", rows=1, cols=64, rule=R.REPLICATED, sections=None),
          dict(name="empty", rows=0, cols=8, rule=R.SPLIT_ROWS, sections=None),
          dict(name="n2", rows=1, cols=64, rule=R.REPLICATED, sections=None)]
    for s in range(2):
        plan = R.shard_plan(ts, 4, 2, s)
        sent = [plan.tensor_is_read(t) for t in range(len(ts))]
        assert sent == [s == 0, True, s == 0, False, s == 0]
        assert [plan.tensor_is_read(t, R.ENCODE_REFRESH) for t in range(len(ts))] == [True, True, True, False, True]
        assert [plan.tensor_is_read(t, R.ENCODE_ARITH) for t in range(len(ts))] == sent
    with pytest.raises(R.RoseError):
        R.shard_plan(ts, 4).tensor_is_read(0, 8)
    with pytest.raises(R.RoseError):
        R.shard_plan(ts, 4).tensor_is_read(5)


@pytest.mark.parametrize("n_layers,pp_src,pp_dst,tp_src,tp",
                         [(4, 2, 1, 2, 4), (4, 1, 2, 1, 2), (4, 4, 2, 2, 1), (4, 2, 4, 1, 4), (4, 2, 2, 4, 2),
                          (6, 3, 2, 1, 2), (6, 6, 3, 2, 2), (6, 3, 1, 2, 1), (6, 2, 6, 4, 2)])
def test_pipeline_plan_matches_oracle_stages_and_maps(n_layers, pp_src, pp_dst, tp_src, tp):
    """The plan of a sender (tensor-parallel rank s in pipeline stage st) lists the whole model: its
    tables must hold, for every element of every tensor of the sender's stage, the oracle's
    destination under the receiving side's degree, in the bucket of the oracle's receiving stage,
    and nothing for the tensors of other stages."""
    ts = models.decoder(n_layers, 32, 4, 4, 8, 48, 64, fused=True)
    for st in range(pp_src):
        for s in range(tp_src):
            plan = R.shard_plan(ts, tp, tp_src, s, n_layers, pp_src, st, pp_dst)
            assert plan.n_buckets == tp * pp_dst and plan.tp == tp
            cap = [0] * plan.n_buckets
            for i, t in enumerate(ts):
                held = oracle.stage_of(t["layer"], n_layers, pp_src) == st
                to = oracle.stage_of(t["layer"], n_layers, pp_dst)
                assert plan.stage_of(i) == (oracle.stage_of(t["layer"], n_layers, pp_src), to)
                assert plan.src_numel(i) == (oracle.local_numel(t["rule"], t["rows"], t["cols"], tp_src) if held else 0)
                for b in range(plan.n_buckets):
                    want = oracle.local_numel(t["rule"], t["rows"], t["cols"], tp) if b // tp == to else 0
                    assert plan.local_numel(i, b) == want
                assert plan.tensor_is_read(i) == (held and (t["rule"] != R.REPLICATED or i % tp_src == s))
                if not held:
                    with pytest.raises(R.RoseError):
                        plan.map_index(i, 0)
                    continue
                sends = t["rule"] != R.REPLICATED or i % tp_src == s
                for r in range(0, t["rows"], 3):
                    for c in range(0, t["cols"], 5):
                        s_first, n_src, g = oracle.shard_map(t["rule"], t["rows"], t["cols"], t["sections"], tp_src, r, c)
                        if not (s_first <= s < s_first + n_src):
                            continue
                        d_first, n_dest, local = oracle.shard_map(t["rule"], t["rows"], t["cols"], t["sections"], tp, r, c)
                        got = plan.map_index(i, g)
                        if sends:
                            assert got == (to * tp + d_first, n_dest, local), (st, s, i, r, c)
                        else:
                            assert got[1] == 0
                if sends:
                    # everything of the tensor that this sender holds lands in the receiving stage's buckets
                    n = oracle.local_numel(t["rule"], t["rows"], t["cols"], tp_src)
                    per = n * (tp if t["rule"] == R.REPLICATED else 1)
                    cap[to * tp] += per       # compared with the sum over the stage's buckets below
            got_caps = [plan.bucket_capacity(b) for b in range(plan.n_buckets)]
            for stage in range(pp_dst):
                assert sum(got_caps[stage * tp:(stage + 1) * tp]) == cap[stage * tp]


def test_pipeline_plan_argument_errors():
    ts = models.decoder(4, 32, 4, 4, 8, 48, 64, fused=True)
    for tp, kw, status in [(4, dict(n_layers=4, pp_src=3), binding.ERR_SHAPE),
                           (4, dict(n_layers=4, pp_dst=3), binding.ERR_SHAPE),
                           (4, dict(n_layers=4, pp_src=2, stage_src=2), binding.ERR_ARG),
                           (4, dict(n_layers=2, pp_src=2), binding.ERR_ARG),        # layer 3 of a 2-layer model
                           (4, dict(n_layers=0, pp_src=2), binding.ERR_SHAPE),
                           (8, dict(n_layers=4, pp_dst=4), binding.ERR_UNSUPPORTED)]:   # 8 * 4 buckets
        with pytest.raises(R.RoseError) as e:
            R.shard_plan(ts, tp, **kw)
        assert e.value.status == status, kw
    # one stage on both sides ignores the layer field altogether
    R.shard_plan([dict(t, layer=99) for t in ts], 4)


def test_tile_order_setter_checks_its_argument():
    plan = R.shard_plan([dict(name="w", rows=8, cols=8, rule=R.SPLIT_ROWS, sections=None)], 2)
    for order in (binding.TILE_ORDER_AUTO, binding.TILE_ORDER_SPREAD, binding.TILE_ORDER_NEIGHBOURS, binding.TILE_ORDER_TIMED):
        plan.set_tile_order(order)
    for bad in (-1, 4):
        with pytest.raises(R.RoseError):
            plan.set_tile_order(bad)


def test_tile_order_is_picked_from_what_the_buckets_can_hold():
    """Before anything is read back the library bounds the density by the buckets' capacities:
    timed below 4 %, neighbours below 7.5 %, spread otherwise and when the buckets could hold
    everything; an order that was set is used as it is."""
    ts = models.decoder(2, 64, 4, 4, 16, 96, 128, fused=True)
    plan = R.shard_plan(ts, 4)
    full = [plan.bucket_capacity(d) for d in range(4)]
    share = lambda f: [int(c * f) for c in full]
    assert plan.pick_tile_order(share(0.02)) == binding.TILE_ORDER_TIMED
    assert plan.pick_tile_order(share(0.039)) == binding.TILE_ORDER_TIMED
    assert plan.pick_tile_order(share(0.05)) == binding.TILE_ORDER_NEIGHBOURS
    assert plan.pick_tile_order(share(0.074)) == binding.TILE_ORDER_NEIGHBOURS
    assert plan.pick_tile_order(share(0.08)) == binding.TILE_ORDER_SPREAD
    assert plan.pick_tile_order(full) == binding.TILE_ORDER_SPREAD
    assert plan.pick_tile_order([0, 0, 0, 0]) == binding.TILE_ORDER_TIMED
    for order in (binding.TILE_ORDER_SPREAD, binding.TILE_ORDER_NEIGHBOURS, binding.TILE_ORDER_TIMED):
        plan.set_tile_order(order)
        assert plan.pick_tile_order(share(0.02)) == order and plan.pick_tile_order(full) == order
