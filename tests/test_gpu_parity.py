"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle, bit for bit
(integer / index work, so the bar is exact equality).  Inputs are seeded and synthetic."""
import numpy as np
import pytest
import torch

import paper_2605_06534_amd as R
from oracle import oracle
from workloads import models, synth
from gpu_harness import Case, assert_buckets_equal, bits, full_parity

pytestmark = pytest.mark.gpu

TILE = 8192   # elements per encode tile (kThreads * kVec * kIters)


def bern_case(tensors, tp, p, seed, **kw):
    olds, news = [], []
    for i, t, o, n in synth.model_pairs(tensors, "bernoulli", seed, "cpu", p=p):
        olds.append(o); news.append(n)
    return Case(tensors, tp, olds, news, **kw)


def T(rows, cols, rule, sections=None, name="t"):
    return dict(name=name, rows=rows, cols=cols, rule=rule, sections=sections)


def test_config1_single_matrix():
    """4096 x 4096, Bernoulli(0.01) +-1..3 ulp, one shard, int32 indices."""
    print("case: config1 4096x4096 p=0.01 tp=1 seed=0", flush=True)
    c = bern_case(models.single_matrix(4096, 4096), 1, 0.01, seed=0)
    want = full_parity(c)
    nnz = want[0]["idx"].size
    assert abs(nnz - 167772) < 6 * 408


@pytest.mark.parametrize("tp", [1, 2, 4, 8])
@pytest.mark.parametrize("fused", [True, False])
def test_small_decoder_all_rules(tp, fused, tile_order):
    print("case: small decoder tp=%d fused=%s" % (tp, fused), flush=True)
    ts = models.decoder(2, 320, 8, 8 if not fused else 8, 40, 1376, 2048, fused=fused)
    full_parity(bern_case(ts, tp, 0.05, seed=11 + tp))


def test_gqa_decoder_tp8_one_kv_head_per_shard():
    print("case: gqa decoder tp=8", flush=True)
    ts = models.decoder(1, 640, 40, 8, 16, 3456, 1216, fused=True)
    full_parity(bern_case(ts, 8, 0.02, seed=4))


@pytest.mark.parametrize("p", [0.0, 0.001, 0.5, 1.0])
def test_densities(p, tile_order):
    print("case: densities p=%g" % p, flush=True)
    ts = [T(96, 1024, R.SPLIT_ROWS), T(64, 2048, R.SPLIT_COLS), T(1, 5000, R.REPLICATED)]
    full_parity(bern_case(ts, 4, p, seed=21))


@pytest.mark.parametrize("numel", [1, 7, 8, 9, 63, 511, 513, TILE - 1, TILE, TILE + 1, 3 * TILE + 17])
def test_ragged_flat_sizes(numel, tile_order):
    print("case: ragged flat numel=%d" % numel, flush=True)
    full_parity(bern_case([T(1, numel, R.REPLICATED)], 2, 0.3, seed=numel))


def test_odd_shapes_take_the_element_path():
    """Columns and row pieces that are not multiples of 8 elements."""
    print("case: odd shapes", flush=True)
    ts = [T(34, 5, R.SPLIT_ROWS), T(7, 12, R.SPLIT_COLS), T(129, 36, R.SPLIT_COLS),
          T(24, 3, R.FUSED_ROWS, [12, 6, 6]), T(6, 2, R.SPLIT_COLS), T(3, 1000, R.SPLIT_COLS),
          T(0, 16, R.SPLIT_ROWS), T(2, 20000, R.SPLIT_COLS)]
    full_parity(bern_case(ts, 2, 0.2, seed=3))
    ts3 = [T(33, 5, R.SPLIT_ROWS), T(7, 12, R.SPLIT_COLS), T(129, 36, R.SPLIT_COLS),
           T(5, 3, R.SPLIT_COLS), T(0, 16, R.SPLIT_ROWS), T(4, 30000, R.SPLIT_COLS),
           T(27, 7, R.FUSED_ROWS, [9, 18])]
    full_parity(bern_case(ts3, 3, 0.2, seed=5))


def test_single_changes_and_special_patterns():
    print("case: special patterns", flush=True)
    n = 2 * TILE + 40
    base = torch.full((n,), 0.0123, dtype=torch.bfloat16)
    ts = [T(1, n, R.REPLICATED)] * 4
    olds = [base.clone() for _ in range(4)]
    news = [base.clone() for _ in range(4)]
    news[0].view(torch.int16)[0] ^= 1                     # first element only
    news[1].view(torch.int16)[n - 1] ^= 1                 # last element only
    olds[2].view(torch.int16)[5] = 0x0000                 # +0 -> -0 is a change
    news[2].view(torch.int16)[5] = -0x8000
    olds[3].view(torch.int16)[9] = 0x7FC1                 # identical NaN is not a change
    news[3].view(torch.int16)[9] = 0x7FC1
    c = Case(ts, 1, olds, news)
    want = full_parity(c)
    assert list(np.diff(want[0]["seg_off"])) == [1, 1, 1, 0]


def test_misaligned_tensors_still_exact():
    print("case: misaligned pointers", flush=True)
    ts = [T(40, 256, R.SPLIT_ROWS), T(16, 512, R.SPLIT_COLS)]
    c = bern_case(ts, 2, 0.1, seed=8)
    # rebuild the pointer tables on storage shifted by one element (2 bytes)
    pad_old = [torch.empty(o.numel() + 8, dtype=o.dtype, device="cuda") for o in c.old]
    pad_new = [torch.empty(o.numel() + 8, dtype=o.dtype, device="cuda") for o in c.new]
    for po, pn, o, n in zip(pad_old, pad_new, c.old, c.new):
        po[1:1 + o.numel()] = o; pn[1:1 + n.numel()] = n
    c.old = [po[1:1 + o.numel()] for po, o in zip(pad_old, c.old)]
    c.new = [pn[1:1 + n.numel()] for pn, n in zip(pad_new, c.new)]
    c.old_tab, c.new_tab = R.ptr_table(c.old), R.ptr_table(c.new)
    assert c.old[0].data_ptr() % 16 == 2
    full_parity(c, check_dense=True)


def test_fp32_master_input():
    print("case: fp32 master clustered", flush=True)
    ts = models.decoder(1, 320, 8, 8, 40, 1376, 2048, fused=True)
    olds, news = [], []
    for i, t, o, n in synth.model_pairs(ts, "clustered_f32", 13, "cpu", vocab_active=300):
        olds.append(o); news.append(n)
    want = full_parity(Case(ts, 4, olds, news))
    assert sum(b["idx"].size for b in want) > 1000


def test_fp32_rounding_special_values():
    print("case: fp32 special values", flush=True)
    rng = np.random.default_rng(0)
    pats = [0x3F808000, 0x3F818000, 0x3F808001, 0x3F807FFF, 0x7F7FFFFF, 0xFF7FFFFF, 0x00000001, 0x80000001,
            0x00008000, 0x00018000, 0x007FFFFF, 0x7F800000, 0xFF800000, 0x7FC00000, 0x7F800001, 0xFFFFFFFF,
            0x80000000, 0x00000000, 0x7FA00000, 0xFF812345]
    u = np.concatenate([np.array(pats, dtype=np.uint32),
                        rng.integers(0, 1 << 32, size=3 * TILE, dtype=np.uint64).astype(np.uint32)])
    new = torch.from_numpy(u.view(np.int32).copy()).view(torch.float32)
    old = torch.zeros(u.size, dtype=torch.bfloat16)
    c = Case([T(1, u.size, R.REPLICATED)], 1, [old], [new])
    want = full_parity(c)
    # every pattern that does not round to +0 is an entry, and its value is the oracle's cast
    rb = oracle.rne_bf16(u)
    assert np.array_equal(want[0]["val"], rb[rb != 0])


def test_few_workers_dense_changes(tile_order):
    """Few workers and tiles that fill the LDS ring: workers wait often and take tickets at a low
    rate, so one worker gets two tickets of one group of blocks in a row; the kernel then
    publishes that pair's counts before it may wait again.  The result must not depend on any of
    it.  (Word 2 of the workspace header counts how often the pair handling ran.)"""
    ts = models.decoder(2, 1024, 16, 16, 64, 2816, 4096, fused=True)
    pairs = 0
    for workers, p in [(65, 0.9), (66, 0.6), (70, 0.9), (97, 1.0), (130, 0.3)]:
        print("case: few workers=%d p=%g seed=%d" % (workers, p, workers), flush=True)
        c = bern_case(ts, 2, p, seed=workers)
        c.plan.set_worker_cap(workers)
        full_parity(c, check_dense=False)
        n = int(c.ws.view(torch.int32)[2])
        print("  same-group ticket pairs handled: %d" % n, flush=True)
        pairs += n
    assert pairs > 0, "the pair handling never ran: the test does not reach what it is for"


@pytest.mark.parametrize("p", [0.45, 0.8, 1.0])
def test_dense_tiles_are_counted_ahead(p, tile_order):
    """More than a third of the elements change: the ring does not hold a ticket's three tiles, and a
    workgroup counts the rest of its ticket before it waits for room (word 3 of the workspace header
    counts how often).  Same buckets as ever."""
    print("case: dense tiles p=%g" % p, flush=True)
    ts = models.decoder(2, 1024, 16, 16, 64, 2816, 4096, fused=True)
    c = bern_case(ts, 4, p, seed=77)
    full_parity(c, check_dense=False)
    n = int(c.ws.view(torch.int32)[3])
    print("  tickets counted ahead: %d" % n, flush=True)
    assert n > 0, "the count-ahead path never ran: the test does not reach what it is for"


def test_capacity_overflow_is_reported_and_bounded():
    print("case: capacity overflow", flush=True)
    ts = [T(64, 512, R.SPLIT_ROWS), T(1, 3000, R.REPLICATED)]
    c = bern_case(ts, 2, 0.25, seed=2, capacity=1000)
    guard = 64
    for b in c.buckets:                                     # room behind the capacity to watch
        b.idx = torch.full((1000 + guard,), -7, dtype=torch.int32, device="cuda")
        b.val = torch.full((1000 + guard,), -7, dtype=torch.int16, device="cuda")
    want = oracle.encode_model(c.records(), 2)
    c.encode()
    for d in range(2):
        with pytest.raises(R.RoseError) as e:
            R.bucket_check(c.plan, c.buckets[d])
        assert e.value.status == 3 and e.value.required == want[d]["seg_off"][-1] > 1000
        assert np.array_equal(c.buckets[d].seg_off.cpu().numpy(), want[d]["seg_off"])     # exact counts
        assert np.array_equal(c.buckets[d].idx[:1000].cpu().numpy(), want[d]["idx"][:1000])
        assert (c.buckets[d].idx[1000:] == -7).all() and (c.buckets[d].val[1000:] == -7).all()


def test_encode_is_deterministic_and_reusable():
    print("case: determinism", flush=True)
    ts = models.decoder(1, 320, 8, 8, 40, 1376, 2048)
    c = bern_case(ts, 4, 0.05, seed=6)
    c.encode()
    first = [c.host_bucket(d) for d in range(4)]
    for b in c.buckets:
        b.idx.fill_(-1); b.val.fill_(-1); b.seg_off.fill_(-1)
    c.ws.fill_(-1)                                          # stale workspace contents must not matter
    c.encode()
    for d in range(4):
        assert_buckets_equal(c.host_bucket(d), first[d])


def test_identical_weights_give_empty_buckets():
    print("case: identical", flush=True)
    ts = models.decoder(1, 320, 8, 8, 40, 1376, 2048)
    c = bern_case(ts, 2, 0.0, seed=1)
    c.encode()
    for d in range(2):
        assert int(c.buckets[d].seg_off.abs().sum()) == 0


def test_argument_errors_on_device_calls():
    print("case: argument errors", flush=True)
    c = bern_case([T(8, 64, R.SPLIT_ROWS)], 2, 0.1, seed=1)
    small = torch.empty(8, dtype=torch.int64, device="cuda")
    with pytest.raises(R.RoseError) as e:
        R.delta_encode(c.plan, c.old_tab, c.new_tab, R.BF16, c.buckets, small)
    assert e.value.status == 1
    with pytest.raises(R.RoseError) as e:
        R.delta_encode(c.plan, c.old_tab, c.new_tab, 5, c.buckets, c.ws)
    assert e.value.status == 1
    b = c.buckets[0]
    keep = b.idx
    b.idx = keep[1:]                                       # 4-byte offset: not 16-byte aligned
    with pytest.raises(R.RoseError) as e:
        R.delta_encode(c.plan, c.old_tab, c.new_tab, R.BF16, c.buckets, c.ws)
    assert e.value.status == 4
    b.idx = keep
    with pytest.raises(R.RoseError) as e:
        R.delta_apply(c.plan, 2, c.buckets[0], c.old_tab)
    assert e.value.status == 1
    torch.cuda.synchronize()


def test_pipeline_stages_encode_independently():
    """PP-aware use (Sec. 4.2 supports TP and PP): each pipeline stage plans, encodes and applies
    only the tensors it holds; together the stages cover the model exactly once."""
    print("case: pipeline stages pp=2 tp=2", flush=True)
    ts = models.decoder(4, 256, 8, 4, 32, 704, 1024, fused=True)
    seen = []
    for stage in range(2):
        sub = models.pp_stage(ts, 4, 2, stage)
        seen += [i for i, _ in sub]
        full_parity(bern_case([t for _, t in sub], 2, 0.05, seed=20 + stage), check_dense=False)
    assert sorted(seen) == list(range(len(ts)))


def test_bandwidth_probes_move_what_they_say():
    """The probes are measurement aids; what can be checked: the copy probe copies, the mixed probe
    writes exactly the stated bytes per chunk and nothing beyond, bad sizes are refused."""
    print("case: bandwidth probes", flush=True)
    g = torch.Generator(device="cpu").manual_seed(5)
    a = torch.randint(0, 255, (4 * 16384,), dtype=torch.uint8, generator=g).cuda()
    b = torch.randint(0, 255, (4 * 16384,), dtype=torch.uint8, generator=g).cuda()
    out = torch.zeros_like(a)
    sink = torch.zeros(1, dtype=torch.int64, device="cuda")
    R.bw_probe(a, out, sink)
    torch.cuda.synchronize()
    assert torch.equal(a, out)
    per_chunk = 48
    dst = torch.full((4 * per_chunk + 64,), 0x5A, dtype=torch.uint8, device="cuda")
    R.bw_probe_mixed(a, b, dst, per_chunk, sink)
    torch.cuda.synchronize()
    assert bool((dst[4 * per_chunk:] == 0x5A).all()), "the mixed probe wrote past its output"
    # every 16-byte vector of a chunk's output is some thread's running XOR of what it has read so
    # far; thread 0 of the workgroup that handles chunk c (one chunk per workgroup here) has read
    # the vectors 0, 256, 512, 768 of both inputs
    av, bv = a.view(-1, 16).cpu().numpy(), b.view(-1, 16).cpu().numpy()
    for c in range(4):
        want = np.zeros(16, dtype=np.uint8)
        for j in range(4):
            want ^= av[c * 1024 + j * 256] ^ bv[c * 1024 + j * 256]
        assert np.array_equal(dst[c * per_chunk:c * per_chunk + 16].cpu().numpy(), want), c
    # the timed variant writes the same places (what it writes is whatever the thread has read by then)
    av0 = dst[:4 * per_chunk].clone()
    dst.fill_(0x5A)
    R.bw_probe_mixed(a, b, dst, per_chunk, sink, timed=True)
    torch.cuda.synchronize()
    assert bool((dst[4 * per_chunk:] == 0x5A).all()), "the timed mixed probe wrote past its output"
    assert torch.equal(dst[:4 * per_chunk], av0)       # one chunk per workgroup: due and written at once or at the end
    # the line probe changes whole 64-byte lines, about the stated share of them, first word of each
    # 16-byte part incremented, everything else as it was
    buf = torch.zeros(1 << 22, dtype=torch.int32, device="cuda")            # 16 MiB = 262,144 lines
    R.bw_probe_lines(buf, 0.3)
    torch.cuda.synchronize()
    parts = buf.view(-1, 4).cpu().numpy()
    assert (parts[:, 1:] == 0).all() and set(np.unique(parts[:, 0])) <= {0, 1}
    lines = parts[:, 0].reshape(-1, 4)
    assert ((lines.sum(1) == 0) | (lines.sum(1) == 4)).all()
    n = lines.shape[0]
    assert abs(int((lines.sum(1) == 4).sum()) - 0.3 * n) < 6 * (n * 0.3 * 0.7) ** 0.5
    R.bw_probe_lines(buf, 1.0)
    torch.cuda.synchronize()
    assert int(buf.view(-1, 4)[:, 0].min()) >= 1
    with pytest.raises(R.RoseError):
        R.bw_probe_lines(buf[:24], 0.5)                  # not a multiple of 64 bytes
    with pytest.raises(R.RoseError):
        R.bw_probe_mixed(a[:1000], b[:1000], dst, per_chunk, sink)
    with pytest.raises(R.RoseError):
        R.bw_probe_mixed(a, b, dst, 50, sink)
