#!/usr/bin/env python3
"""Benchmark of the sparse weight-delta hot path on one MI355X.

A step is one pass of the whole path over one synthetic parameter-set update: delta_encode of
all tensors into every destination bucket, then delta_apply of every bucket into the receiver's
shard copies.  Default workload: the 7B-style decoder re-sharded to TP = 4 at 5 % change density.
Prints one JSON line (metric: dense GB/s scanned = 4 bytes per element / step time).
"""
import argparse
import json
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="decoder7b_tp4",
                    choices=["matrix4096_tp1", "decoder7b_tp4", "flat1g_tp1", "decoder32b_tp8", "decoder32b_tp8_f32",
                             "decoder8b_tp1", "decoder8b_tp4"])
    ap.add_argument("--density", type=float, default=None, help="change density p (default: the workload's)")
    ap.add_argument("--layers", type=int, default=None, help="fewer decoder layers (debugging only)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--tp-src", type=int, default=1,
                    help="sender-side sharding: time the sender that holds shard --src-rank of this many")
    ap.add_argument("--src-rank", type=int, default=0)
    ap.add_argument("--payload", choices=("new", "arith"), default="new",
                    help="entry payload: the new pattern (default) or the arithmetic difference with escapes")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-elems", type=float, default=4.0e9)
    ap.add_argument("--graph", action="store_true",
                    help="replay the step from a HIP graph (for launch-bound small workloads); the per-kernel "
                         "times in `detail` are still taken from eager launches")
    ap.add_argument("--traffic-bytes", type=float, default=None,
                    help="HBM bytes per encode launch from rocprofv3 counters, to report as roofline.traffic")
    return ap.parse_args()


def workload(args):
    from workloads import models
    w = args.workload
    if w == "matrix4096_tp1":
        return models.single_matrix(), 1, "bernoulli", 0.01
    if w == "decoder7b_tp4":
        return models.decoder_7b(args.layers or 32), 4, "bernoulli", 0.05
    if w == "flat1g_tp1":
        return models.flat(1 << 30), 1, "bernoulli", 0.01
    if w == "decoder32b_tp8":
        return models.decoder_32b(args.layers or 64), 8, "bernoulli", 0.02
    if w in ("decoder8b_tp1", "decoder8b_tp4"):
        return models.decoder_8b(args.layers or 36), 1 if w.endswith("tp1") else 4, "bernoulli", 0.02
    return models.decoder_32b(args.layers or 64), 8, "clustered_f32", None


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (all destination buckets are produced and applied "
              "on the one device; there are no collectives). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback.", file=sys.stderr)
        sys.exit(2)

    import paper_2605_06534_amd as R
    from workloads import models, synth

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    tensors, tp, recipe, p = workload(args)
    if args.density is not None:
        p = args.density
    n_elems = models.numel(tensors)

    # ---- inputs resident in HBM: W_{t-1}, W_t, the receiver's shard copies, buckets ----
    olds, news = [], []
    kw = {"p": p} if recipe == "bernoulli" else {"vocab_active": 20000}
    for _, _, o, n in synth.model_pairs(tensors, recipe, args.seed, "cuda", **kw):
        olds.append(o)
        news.append(n)
    new_dtype = R.FP32_RNE if recipe == "clustered_f32" else R.BF16
    if args.tp_src > 1:
        # the sender's slices of W_{t-1} and W_t, cut with the library's own dense path
        if new_dtype != R.BF16:
            print("bench.py: --tp-src is for bf16 workloads", file=sys.stderr)
            sys.exit(2)
        cut = R.shard_plan(tensors, args.tp_src)
        full_old, full_new = R.ptr_table(olds), R.ptr_table(news)
        so = [torch.empty(cut.local_numel(t, args.src_rank), dtype=torch.bfloat16, device=dev) for t in range(len(tensors))]
        sn = [torch.empty_like(x) for x in so]
        R.dense_copy(cut, args.src_rank, full_old, R.BF16, R.ptr_table(so))
        R.dense_copy(cut, args.src_rank, full_new, R.BF16, R.ptr_table(sn))
        torch.cuda.synchronize()
        olds, news = so, sn
        del cut, full_old, full_new
        torch.cuda.empty_cache()
        n_elems = sum(x.numel() for x in olds)
    plan = R.shard_plan(tensors, tp, args.tp_src, args.src_rank)
    old_tab, new_tab = R.ptr_table(olds), R.ptr_table(news)
    ws = R.workspace(plan)
    frac = 0.03 if p is None else min(1.0, 1.3 * p + 0.002)    # the clustered recipe changes about 1.4 %
    buckets = [R.Bucket(int(plan.bucket_capacity(d) * frac) + 4096, len(tensors)) for d in range(tp)]
    shards, shard_tabs = [], []
    for d in range(tp):
        loc = [torch.zeros(plan.local_numel(t, d), dtype=torch.bfloat16, device=dev) for t in range(len(tensors))]
        tab = R.ptr_table(loc)
        R.dense_copy(plan, d, old_tab, R.BF16, tab)        # receiver starts from W_{t-1} (the part this sender covers)
        shards.append(loc)
        shard_tabs.append(tab)
    torch.cuda.synchronize()

    arith = args.payload == "arith"

    def step(ev=None):
        if ev:
            ev[0].record()
        if arith:
            R.delta_encode_ex(plan, old_tab, new_tab, new_dtype, R.ENCODE_ARITH, buckets, ws)
        else:
            R.delta_encode(plan, old_tab, new_tab, new_dtype, buckets, ws)
        if ev:
            ev[1].record()
        for d in range(tp):
            if arith:
                R.delta_apply_ex(plan, d, buckets[d], R.PAYLOAD_ARITH, shard_tabs[d])
            else:
                R.delta_apply(plan, d, buckets[d], shard_tabs[d])
        if ev:
            ev[2].record()

    for _ in range(max(args.warmup, 1)):
        step()
    torch.cuda.synchronize()
    nnz = [R.bucket_check(plan, buckets[d]) for d in range(tp)]    # raises if a bucket overflowed
    nnz_total = sum(nnz)

    if arith:
        # an arithmetic bucket may be applied once only: start the receivers from W_{t-1} again and
        # take one step before checking (the timed steps below keep adding; their values are not used)
        for d in range(tp):
            R.dense_copy(plan, d, old_tab, R.BF16, shard_tabs[d])
        step()
        torch.cuda.synchronize()
    # the receiver now holds W_t: check one shard tensor per rule class against a dense copy
    # (one tensor at a time: the largest workload leaves no room for a second copy of a whole shard)
    for t in range(len(tensors)):
        if t % 7 == 0 or t >= len(tensors) - 3:            # walks through every rule class; both ends of the model
            chk = shards[tp - 1][t].clone()
            only = R.shard_plan([tensors[t]], tp, args.tp_src, args.src_rank)
            R.dense_copy(only, tp - 1, R.ptr_table([news[t]]), new_dtype, R.ptr_table([chk]))
            torch.cuda.synchronize()
            if not torch.equal(shards[tp - 1][t].view(torch.int16), chk.view(torch.int16)):
                print("bench.py: applied shard differs from the dense copy of the new weights (tensor %d)" % t,
                      file=sys.stderr)
                sys.exit(1)
            del chk, only

    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(events[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    if args.graph:
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.synchronize()
        for _ in range(max(args.warmup, 1)):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    t_enc = sum(e[0].elapsed_time(e[1]) for e in events) / args.steps      # ms, HIP events on the launch stream
    t_app = sum(e[1].elapsed_time(e[2]) for e in events) / args.steps

    # dense path for comparison (Sec. 6.3 crossover): every shard's slice of the new weights copied
    ev_c = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for rep in range(3):
        if rep == 1:
            ev_c[0].record()
        for d in range(tp):
            R.dense_copy(plan, d, new_tab, new_dtype, shard_tabs[d])
    ev_c[1].record()
    torch.cuda.synchronize()
    t_copy = ev_c[0].elapsed_time(ev_c[1]) / 2

    in_bytes_per_elem = 6 if new_dtype == R.FP32_RNE else 4
    scanned = in_bytes_per_elem * n_elems
    enc_bytes = scanned + 6 * nnz_total            # algorithmic: read old + new once, write idx + val
    app_bytes = 8 * nnz_total                      # read idx + val, write val
    value = scanned / 1e9 / (ms_per_step / 1e3)

    # ---- bandwidth probe in the same run (1 GiB buffers) ----
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty_like(src)
    sink = torch.zeros(1, dtype=torch.int64, device=dev)
    probe = {}
    for name, d_, s_ in (("copy", dst, None), ("read", None, sink)):
        for _ in range(2):
            R.bw_probe(src, d_, s_)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(10):
            R.bw_probe(src, d_, s_)
        b.record()
        torch.cuda.synchronize()
        moved = (2 if name == "copy" else 1) * src.numel() * 10
        probe[name + "_GBs"] = round(moved / 1e9 / (a.elapsed_time(b) / 1e3), 1)
    # the same mix of reads and writes as the encode launch (two read streams, 6 * nnz / tiles bytes
    # written per 2 x 16 KB read), with no work attached: what HBM delivers for that traffic
    if new_dtype == R.BF16:
        per_chunk = min(16384, max(16, int(round(6 * nnz_total / max(plan.n_tiles(), 1) / 16)) * 16))
        del src, dst
        big = 4 << 30                                  # per stream: far beyond the 256 MB memory-side cache
        src_a = torch.empty(big, dtype=torch.uint8, device=dev).fill_(1)
        src_b = torch.empty(big, dtype=torch.uint8, device=dev).fill_(2)
        mix_dst = torch.empty((big // 16384) * per_chunk, dtype=torch.uint8, device=dev)
        for _ in range(2):
            R.bw_probe_mixed(src_a, src_b, mix_dst, per_chunk, sink)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(5):
            R.bw_probe_mixed(src_a, src_b, mix_dst, per_chunk, sink)
        b.record()
        torch.cuda.synchronize()
        moved = (2 * big + mix_dst.numel()) * 5
        probe["encode_mix_GBs"] = round(moved / 1e9 / (a.elapsed_time(b) / 1e3), 1)
        probe["encode_mix_write_bytes_per_16k_pair"] = per_chunk
        del mix_dst, src_a, src_b
    else:
        del src, dst

    # Modelled synchronisation time over a link of B Gbit/s (the paper's range): the sparse path sends
    # 6 bytes per entry, the dense path 2 bytes per element; kernel times are the measured ones.
    crossover = {}
    for gbps in (1, 5, 20, 200):
        bps = gbps * 1e9 / 8
        crossover["%dGbps" % gbps] = {"sparse_s": round((t_enc + t_app) / 1e3 + 6 * nnz_total / bps, 4),
                                      "dense_s": round(t_copy / 1e3 + 2 * n_elems / bps, 4)}
    # apply moves whole 64-byte lines: entries read + touched lines read and written
    local_elems = sum(plan.local_numel(t, d) for t in range(len(tensors)) for d in range(tp))
    dens = nnz_total / local_elems
    app_line_bytes = 6 * nnz_total + 2 * (1 - (1 - dens) ** 32) * 2 * local_elems

    # HBM bytes per encode launch as counted by rocprofv3 (FETCH_SIZE x 2.0 + WRITE_SIZE KiB, two --pmc runs,
    # scale factors from the copy probe): cannot be collected from inside this process, so the figure
    # recorded in profiles/encode_apply_decoder7b_tp4_hbm_traffic.txt is reported for the workload it was
    # taken on, and null for any other unless --traffic-bytes passes one in.
    traffic = args.traffic_bytes
    if (traffic is None and args.workload == "decoder7b_tp4" and args.density is None and args.layers is None
            and args.tp_src == 1 and args.payload == "new" and args.seed == 0):
        traffic = 29.70e9
    out = {
        "metric": "weight-delta encode+apply GB/s (bf16 scanned)",
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u16", "data": "synthetic",
        "config": {"workload": args.workload, "elements": n_elems, "tensors": len(tensors), "tp": tp,
                   "recipe": recipe, "density": p, "nnz": nnz_total, "seed": args.seed,
                   "tp_src": args.tp_src, "src_rank": args.src_rank, "hip_graph": bool(args.graph), "payload": args.payload,
                   "new_dtype": "fp32->bf16 RNE" if new_dtype == R.FP32_RNE else "bf16"},
        "roofline": {"bound": "hbm", "kernel": "encode_kernel",
                     "achieved": round(enc_bytes / 1e9 / (t_enc / 1e3), 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(enc_bytes / 1e9 / (t_enc / 1e3) / HBM_PEAK_GBS, 4),
                     "traffic": traffic,
                     "algorithmic_bytes": enc_bytes, "launch_ms": round(t_enc, 4)},
        "detail": {"t_encode_ms": round(t_enc, 4), "t_apply_ms": round(t_app, 4),
                   "encode_scanned_GBs": round(scanned / 1e9 / (t_enc / 1e3), 1),
                   "apply_algorithmic_GBs": round(app_bytes / 1e9 / (t_app / 1e3), 1) if t_app > 0 else None,
                   "encode_plus_apply_algorithmic_frac_of_peak":
                       round((enc_bytes + app_bytes) / 1e9 / ((t_enc + t_app) / 1e3) / HBM_PEAK_GBS, 4),
                   "apply_line_model_bytes": int(app_line_bytes),
                   "apply_line_model_frac_of_peak": round(app_line_bytes / 1e9 / (t_app / 1e3) / HBM_PEAK_GBS, 4)
                   if t_app > 0 else None,
                   "t_dense_copy_ms": round(t_copy, 4), "wire_bytes_sparse_over_dense": round(6 * nnz_total / (2 * n_elems), 4),
                   "modelled_sync": crossover,
                   "bw_probe": probe, "tiles": plan.n_tiles()},
    }

    if not args.no_cpu_baseline and args.tp_src == 1:
        out["cpu_baseline"] = cpu_baseline(tensors, tp, olds, news, args.cpu_sample_elems, in_bytes_per_elem)
    print(json.dumps(out), flush=True)


def cpu_baseline(tensors, tp, olds, news, sample_elems, in_bytes_per_elem):
    """The oracle as it stands on the first tensors of the same workload (copied from the device
    beforehand; copies are not timed): once on one thread, once with whole tensors dealt to a pool
    of threads (the oracle's C code runs outside the interpreter lock)."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor
    from oracle import oracle

    def host(t):
        t = t.detach().cpu().contiguous()
        if t.dtype == torch.float32:
            return t.view(torch.int32).numpy().view(np.uint32)
        return t.view(torch.int16).numpy().view(np.uint16)

    work, done = [], 0
    for t, o, n in zip(tensors, olds, news):
        if done >= sample_elems:
            break
        work.append((t, host(o), host(n)))
        done += work[-1][1].size

    def one(item):
        t, ho, hn = item
        dsts = [np.zeros(oracle.local_numel(t["rule"], t["rows"], t["cols"], tp), dtype=np.uint16) for _ in range(tp)]
        segs = oracle.encode_tensor(ho, hn, t["rows"], t["cols"], t["rule"], t["sections"], tp)
        for d, (idx, val) in enumerate(segs):
            oracle.apply_segment(idx, val, dsts[d])

    t0 = time.perf_counter()
    for item in work:
        one(item)
    secs1 = time.perf_counter() - t0
    threads = max(1, min(16, os.cpu_count() or 1, len(work)))
    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=threads) as pool:
        list(pool.map(one, work))
    secs_n = time.perf_counter() - t0
    rate = lambda s: round(in_bytes_per_elem * done / 1e9 / s, 3)
    return {"value": rate(secs_n), "unit": "GB/s", "cores": threads, "kind": "oracle", "value_1core": rate(secs1),
            "sample": "first %d tensors of the workload (%d elements), encode+apply, %.1f s on one thread, %.1f s on %d"
                      % (len(work), done, secs1, secs_n, threads)}


if __name__ == "__main__":
    main()
