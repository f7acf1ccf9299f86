#!/usr/bin/env python3
"""Benchmark of the sparse weight-delta hot path on one MI355X.

A step is one pass of the whole path over one synthetic parameter-set update: delta_encode of
all tensors into every destination bucket, then delta_apply of every bucket into the receiver's
shard copies.  Default workload: the 32B-style GQA decoder re-sharded to TP = 8 at 2 % change
density (the largest configuration that fits one GPU); the 7B-style decoder at TP = 4 is timed
afterwards in the same process at 1, 5 and 10 % and reported under `detail`.
Prints one JSON line (metric: dense GB/s scanned = 4 bytes per element / step time).
"""
import argparse
import gc
import hashlib
import json
import os
import re
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
WORKLOADS = ["matrix4096_tp1", "decoder7b_tp4", "flat1g_tp1", "decoder32b_tp8", "decoder32b_tp8_f32",
             "decoder8b_tp1", "decoder8b_tp4"]


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="decoder32b_tp8", choices=WORKLOADS)
    ap.add_argument("--density", type=float, default=None, help="change density p (default: the workload's)")
    ap.add_argument("--layers", type=int, default=None, help="fewer decoder layers (debugging only)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--tp", type=int, default=None, help="receiving side's tensor-parallel degree (default: the workload's)")
    ap.add_argument("--tp-src", type=int, default=1,
                    help="sender-side sharding: time the sender that holds shard --src-rank of this many")
    ap.add_argument("--src-rank", type=int, default=0)
    ap.add_argument("--pp-src", type=int, default=1, help="pipeline stages on the sending side (the step is "
                    "then one sender's share: the tensors of --stage-src)")
    ap.add_argument("--stage-src", type=int, default=0)
    ap.add_argument("--pp-dst", type=int, default=1, help="pipeline stages on the receiving side (tp * pp-dst buckets)")
    ap.add_argument("--payload", choices=("new", "arith"), default="new",
                    help="entry payload: the new pattern (default) or the arithmetic difference with escapes")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-elems", type=float, default=4.0e9)
    ap.add_argument("--no-extra", action="store_true",
                    help="skip the 7B-style decoder runs that follow the default workload")
    ap.add_argument("--no-probes", action="store_true", help="skip the bandwidth probes")
    ap.add_argument("--graph", action="store_true",
                    help="replay the step from a HIP graph (for launch-bound small workloads); the per-kernel "
                         "times in `detail` are still taken from eager launches")
    ap.add_argument("--traffic-bytes", type=float, default=None,
                    help="HBM bytes per encode launch from rocprofv3 counters, to report as roofline.traffic "
                         "instead of the figure in profiles/")
    return ap.parse_args()


def workload(name, layers=None):
    """-> tensors, tp, input recipe, default density"""
    from workloads import models
    if name == "matrix4096_tp1":
        return models.single_matrix(), 1, "bernoulli", 0.01
    if name == "decoder7b_tp4":
        return models.decoder_7b(layers or 32), 4, "bernoulli", 0.05
    if name == "flat1g_tp1":
        return models.flat(1 << 30), 1, "bernoulli", 0.01
    if name == "decoder32b_tp8":
        return models.decoder_32b(layers or 64), 8, "bernoulli", 0.02
    if name in ("decoder8b_tp1", "decoder8b_tp4"):
        return models.decoder_8b(layers or 36), 1 if name.endswith("tp1") else 4, "bernoulli", 0.02
    return models.decoder_32b(layers or 64), 8, "clustered_f32", None


def kernels_sha256():
    h = hashlib.sha256()
    for f in ("kernels.hip", "rose_internal.h"):
        with open(os.path.join(ROOT, "paper_2605_06534_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def profile_traffic(name, density, kernel):
    """HBM bytes per launch of `kernel` on this workload as rocprofv3 counted them (FETCH_SIZE and
    WRITE_SIZE in KiB per dispatch, each scaled by what the same counter reads for the copy probe),
    taken from the `TRAFFIC` line of the committed profiles/<...>_hbm_traffic.txt that names this
    workload, density and kernel.  Counters cannot be collected from inside this process.  The
    figure is reported only if the kernel sources still hash to what the profile was taken on.
    -> (bytes or None, description of the source)"""
    pdir = os.path.join(ROOT, "profiles")
    want = {"kernel": kernel, "workload": name, "density": "%g" % density if density is not None else "recipe"}
    for fn in sorted(os.listdir(pdir)) if os.path.isdir(pdir) else []:
        if not fn.endswith("_hbm_traffic.txt"):
            continue
        for line in open(os.path.join(pdir, fn)):
            if not line.startswith("TRAFFIC "):
                continue
            kv = dict(x.split("=", 1) for x in line.split()[1:] if "=" in x)
            if any(kv.get(k) != v for k, v in want.items()):
                continue
            src = {"file": "profiles/" + fn, "kernels_sha256": kv.get("kernels_sha256")}
            if kv.get("kernels_sha256") != kernels_sha256():
                src["note"] = "the kernel sources have changed since this profile was taken: not reported"
                return None, src
            nbytes = 1024.0 * (float(kv["fetch_KiB"]) * float(kv["fetch_scale"]) +
                               float(kv["write_KiB"]) * float(kv["write_scale"]))
            return nbytes, src
    src = {"note": "no TRAFFIC line for this workload, density and kernel under profiles/"}
    # counters taken on a part of the workload (same shapes, fewer layers) are named, never scaled up
    for fn in sorted(os.listdir(pdir)) if os.path.isdir(pdir) else []:
        if fn.endswith("_hbm_traffic.txt"):
            for line in open(os.path.join(pdir, fn)):
                kv = dict(x.split("=", 1) for x in line.split()[1:] if "=" in x) if line.startswith("TRAFFIC ") else {}
                if kv.get("kernel") == kernel and kv.get("workload", "").startswith(name + "_") and kv.get("density") == want["density"]:
                    src["related"] = {"file": "profiles/" + fn, "workload": kv["workload"],
                                      "bytes": round(1024.0 * (float(kv["fetch_KiB"]) * float(kv["fetch_scale"]) +
                                                               float(kv["write_KiB"]) * float(kv["write_scale"]))),
                                      "kernels_sha256_matches": kv.get("kernels_sha256") == kernels_sha256()}
    return None, src


def measure(R, name, tensors, tp, recipe, p, args, steps, warmup, probes, keep_host_sample):
    """Build the workload on the device, check one step, time `steps` steps.  -> dict of results."""
    from workloads import models, synth
    dev = torch.device("cuda:0")
    n_elems = models.numel(tensors)

    # ---- the plan: this sender's view of the whole model (host only so far) ----
    staged = args.pp_src > 1 or args.pp_dst > 1
    if staged:
        n_layers = max(t["layer"] for t in tensors) + 1
        plan = R.shard_plan(tensors, tp, args.tp_src, args.src_rank, n_layers, args.pp_src, args.stage_src, args.pp_dst)
    else:
        plan = R.shard_plan(tensors, tp, args.tp_src, args.src_rank)
    n_b = plan.n_buckets                                    # tp, or tp * pp_dst
    held = [plan.stage_of(t)[0] == args.stage_src for t in range(len(tensors))]

    # ---- inputs resident in HBM: W_{t-1}, W_t, the receiver's shard copies, buckets ----
    # (a tensor of another sending stage is not on this sender: its table entries are never read and
    # point at a few valid bytes)
    stand_in = torch.zeros(64, dtype=torch.bfloat16, device=dev)
    olds, news = [], []
    kw = {"p": p} if recipe == "bernoulli" else {"vocab_active": 20000}
    for _, _, o, n in synth.model_pairs(tensors, recipe, args.seed, "cuda", only=held, **kw):
        olds.append(stand_in if o is None else o)
        news.append(stand_in if n is None else n)
    new_dtype = R.FP32_RNE if recipe == "clustered_f32" else R.BF16
    if staged and new_dtype != R.BF16:
        print("bench.py: --pp-src / --pp-dst are for bf16 workloads", file=sys.stderr)
        sys.exit(2)
    if args.tp_src > 1:
        # the sender's slices of W_{t-1} and W_t, cut with the library's own dense path
        if new_dtype != R.BF16:
            print("bench.py: --tp-src is for bf16 workloads", file=sys.stderr)
            sys.exit(2)
        mine = [t for t in range(len(tensors)) if held[t]]
        cut = R.shard_plan([tensors[t] for t in mine], args.tp_src)
        full_old, full_new = R.ptr_table([olds[t] for t in mine]), R.ptr_table([news[t] for t in mine])
        so = [torch.empty(cut.local_numel(k, args.src_rank), dtype=torch.bfloat16, device=dev) for k in range(len(mine))]
        sn = [torch.empty_like(x) for x in so]
        R.dense_copy(cut, args.src_rank, full_old, R.BF16, R.ptr_table(so))
        R.dense_copy(cut, args.src_rank, full_new, R.BF16, R.ptr_table(sn))
        torch.cuda.synchronize()
        for k, t in enumerate(mine):
            olds[t], news[t] = so[k], sn[k]
        del cut, full_old, full_new, so, sn
        torch.cuda.empty_cache()
    if staged or args.tp_src > 1:
        n_elems = sum(olds[t].numel() for t in range(len(tensors)) if held[t])
    old_tab, new_tab = R.ptr_table(olds), R.ptr_table(news)
    ws = R.workspace(plan)
    frac = 0.03 if p is None else min(1.0, 1.3 * p + 0.002)    # the clustered recipe changes about 1.6 %
    buckets = [R.Bucket(int(plan.bucket_capacity(d) * frac) + 4096, len(tensors)) for d in range(n_b)]
    shards, shard_tabs = [], []
    for d in range(n_b):
        loc = [torch.zeros(plan.local_numel(t, d), dtype=torch.bfloat16, device=dev) if plan.local_numel(t, d) else stand_in
               for t in range(len(tensors))]
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
        for d in range(n_b):
            if arith:
                R.delta_apply_ex(plan, d, buckets[d], R.PAYLOAD_ARITH, shard_tabs[d])
            else:
                R.delta_apply(plan, d, buckets[d], shard_tabs[d])
        if ev:
            ev[2].record()

    for _ in range(max(warmup, 1)):
        step()
    torch.cuda.synchronize()
    nnz = [R.bucket_check(plan, buckets[d]) for d in range(n_b)]   # raises if a bucket overflowed
    nnz_total = sum(nnz)

    if arith:
        # an arithmetic bucket may be applied once only: start the receivers from W_{t-1} again and
        # take one step before checking (the timed steps below keep adding; their values are not used)
        for d in range(n_b):
            R.dense_copy(plan, d, old_tab, R.BF16, shard_tabs[d])
        step()
        torch.cuda.synchronize()
    # the receiver now holds W_t: check one shard tensor per rule class against a dense copy
    # (one tensor at a time: the largest workload leaves no room for a second copy of a whole shard)
    for t in range(len(tensors)):
        if held[t] and (t % 7 == 0 or t >= len(tensors) - 3):   # walks through every rule class; both ends of the model
            last = plan.stage_of(t)[1] * tp + tp - 1           # the last shard of the stage that receives the tensor
            chk = shards[last][t].clone()
            only = R.shard_plan([tensors[t]], tp, args.tp_src, args.src_rank)
            R.dense_copy(only, tp - 1, R.ptr_table([news[t]]), new_dtype, R.ptr_table([chk]))
            torch.cuda.synchronize()
            if not torch.equal(shards[last][t].view(torch.int16), chk.view(torch.int16)):
                print("bench.py: applied shard differs from the dense copy of the new weights (tensor %d)" % t,
                      file=sys.stderr)
                sys.exit(1)
            del chk, only

    # HIP events on the stream the kernels are launched on (torch's current stream: the binding passes it)
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        step(events[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / steps
    if args.graph:
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.synchronize()
        for _ in range(max(warmup, 1)):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    t_enc = sum(e[0].elapsed_time(e[1]) for e in events) / steps
    t_app = sum(e[1].elapsed_time(e[2]) for e in events) / steps

    # dense path for comparison (Sec. 6.3 crossover): every shard's slice of the new weights copied
    ev_c = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for rep in range(3):
        if rep == 1:
            ev_c[0].record()
        for d in range(n_b):
            R.dense_copy(plan, d, new_tab, new_dtype, shard_tabs[d])
    ev_c[1].record()
    torch.cuda.synchronize()
    t_copy = ev_c[0].elapsed_time(ev_c[1]) / 2

    in_bytes_per_elem = 6 if new_dtype == R.FP32_RNE else 4
    scanned = in_bytes_per_elem * n_elems
    enc_bytes = scanned + 6 * nnz_total            # algorithmic: read old + new once, write idx + val
    app_bytes = 8 * nnz_total                      # read idx + val, write val
    # apply moves whole 64-byte lines: entries read + touched lines read and written
    local_elems = sum(plan.local_numel(t, d) for t in range(len(tensors)) for d in range(n_b))
    dens = nnz_total / max(local_elems, 1)
    app_line_bytes = 6 * nnz_total + 2 * (1 - (1 - dens) ** 32) * 2 * local_elems
    # what the memory moves for it (counters): reads come in 128-byte units (both halves of an L2 line
    # are fetched when one is asked for), writes in the 64-byte lines the kernel stores
    app_mem_bytes = 6 * nnz_total + ((1 - (1 - dens) ** 64) + (1 - (1 - dens) ** 32)) * 2 * local_elems
    res = {
        "name": name, "n_elems": n_elems, "n_tensors": len(tensors), "tp": tp, "recipe": recipe, "density": p,
        "nnz": nnz_total, "new_dtype": "fp32->bf16 RNE" if new_dtype == R.FP32_RNE else "bf16",
        "in_bytes_per_elem": in_bytes_per_elem, "ms_per_step": ms_per_step, "t_enc": t_enc, "t_app": t_app,
        "t_copy": t_copy, "scanned": scanned, "enc_bytes": enc_bytes, "app_bytes": app_bytes,
        "app_line_bytes": app_line_bytes, "tiles": plan.n_tiles(),
        "enc_frac": enc_bytes / 1e9 / (t_enc / 1e3) / HBM_PEAK_GBS,
        "both_frac": (enc_bytes + app_bytes) / 1e9 / ((t_enc + t_app) / 1e3) / HBM_PEAK_GBS,
        "app_line_frac": app_line_bytes / 1e9 / (t_app / 1e3) / HBM_PEAK_GBS if t_app > 0 else None,
        "app_mem_bytes": app_mem_bytes,
        "app_mem_frac": app_mem_bytes / 1e9 / (t_app / 1e3) / HBM_PEAK_GBS if t_app > 0 else None,
    }
    if keep_host_sample:
        res["host_sample"] = host_sample(tensors, olds, news, args.cpu_sample_elems)
    n_tiles = plan.n_tiles()
    del shards, shard_tabs, buckets, ws, olds, news, old_tab, new_tab, plan
    gc.collect()
    torch.cuda.empty_cache()
    if probes:
        res["bw_probe"] = bw_probes(R, nnz_total, n_tiles, new_dtype == R.BF16, 1 - (1 - dens) ** 32)
    return res


def bw_probes(R, nnz_total, n_tiles, mixed, touched_lines):
    """What HBM delivers beside the kernels, in the same run: 1 GiB copy and read, a read-modify-write
    of the share of 64-byte lines that apply touches at this density (4 GiB, no other work), and
    (bf16 input) a stream with the encode launch's mix of reads and writes and none of its work."""
    dev = torch.device("cuda:0")
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
    del src, dst
    lines = torch.zeros(4 << 30, dtype=torch.uint8, device=dev)
    for _ in range(2):
        R.bw_probe_lines(lines, touched_lines)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(5):
        R.bw_probe_lines(lines, touched_lines)
    b.record()
    torch.cuda.synchronize()
    probe["lines_rmw_GBs"] = round(2 * touched_lines * lines.numel() * 5 / 1e9 / (a.elapsed_time(b) / 1e3), 1)
    probe["lines_rmw_touched_share"] = round(touched_lines, 4)
    del lines
    if mixed:
        # two read streams, 6 * nnz / tiles bytes written per 2 x 16 KB read
        per_chunk = min(16384, max(16, int(round(6 * nnz_total / max(n_tiles, 1) / 16)) * 16))
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
        # the same traffic with the writes held back and sent in the windows of the timed tile order
        for _ in range(2):
            R.bw_probe_mixed(src_a, src_b, mix_dst, per_chunk, sink, timed=True)
        a.record()
        for _ in range(5):
            R.bw_probe_mixed(src_a, src_b, mix_dst, per_chunk, sink, timed=True)
        b.record()
        torch.cuda.synchronize()
        probe["encode_mix_timed_writes_GBs"] = round(moved / 1e9 / (a.elapsed_time(b) / 1e3), 1)
        del mix_dst, src_a, src_b
    torch.cuda.empty_cache()
    return probe


def host_sample(tensors, olds, news, sample_elems):
    """Host copies of the first tensors of the workload (about sample_elems elements) for the CPU
    baseline; the copies are not timed."""
    import numpy as np

    def host(t):
        t = t.detach().cpu().contiguous()
        if t.dtype == torch.float32:
            return t.view(torch.int32).numpy().view(np.uint32)
        return t.view(torch.int16).numpy().view(np.uint16)

    work, done = [], 0
    for t, o, n in zip(tensors, olds, news):
        if done >= sample_elems:
            break
        if len(tensors) == 1 and o.numel() > sample_elems:    # a single large tensor: its leading part
            k = int(sample_elems)
            t = dict(t, rows=1, cols=k, rule=0, sections=None)
            o, n = o[:k], n[:k]
        work.append((t, host(o), host(n)))
        done += work[-1][1].size
    return work, done


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

    torch.cuda.set_device(0)
    tensors, tp, recipe, p = workload(args.workload, args.layers)
    if args.density is not None:
        p = args.density
    if args.tp is not None:
        tp = args.tp
    want_cpu = not args.no_cpu_baseline and args.tp_src == 1 and args.pp_src == 1 and args.pp_dst == 1
    m = measure(R, args.workload, tensors, tp, recipe, p, args, args.steps, args.warmup, not args.no_probes, want_cpu)

    # Modelled synchronisation time over a link of B Gbit/s (the paper's range): the sparse path sends
    # 6 bytes per entry, the dense path 2 bytes per element; kernel times are the measured ones.
    crossover = {}
    for gbps in (1, 5, 20, 200):
        bps = gbps * 1e9 / 8
        crossover["%dGbps" % gbps] = {"sparse_s": round((m["t_enc"] + m["t_app"]) / 1e3 + 6 * m["nnz"] / bps, 4),
                                      "dense_s": round(m["t_copy"] / 1e3 + 2 * m["n_elems"] / bps, 4)}

    kernel = "encode_kernel<%d, 0, %d>" % (1 if recipe == "clustered_f32" else 0, 1 if args.payload == "arith" else 0)
    traffic, traffic_src = None, {"note": "non-default run: no committed profile applies"}
    if args.traffic_bytes is not None:
        traffic, traffic_src = args.traffic_bytes, {"note": "--traffic-bytes"}
    elif args.layers is None and args.tp_src == 1 and args.seed == 0 and args.tp is None \
            and args.pp_src == 1 and args.pp_dst == 1:
        traffic, traffic_src = profile_traffic(args.workload, p, kernel.replace(" ", ""))
    value = m["scanned"] / 1e9 / (m["ms_per_step"] / 1e3)
    out = {
        "metric": "weight-delta encode+apply GB/s (bf16 scanned)",
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(m["ms_per_step"], 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u16", "data": "synthetic",
        "config": {"workload": args.workload, "elements": m["n_elems"], "tensors": m["n_tensors"], "tp": tp,
                   "recipe": recipe, "density": p, "nnz": m["nnz"], "seed": args.seed,
                   "tp_src": args.tp_src, "src_rank": args.src_rank, "pp_src": args.pp_src,
                   "stage_src": args.stage_src, "pp_dst": args.pp_dst, "hip_graph": bool(args.graph),
                   "payload": args.payload, "new_dtype": m["new_dtype"]},
        "roofline": {"bound": "hbm", "kernel": kernel,
                     "achieved": round(m["enc_bytes"] / 1e9 / (m["t_enc"] / 1e3), 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(m["enc_frac"], 4),
                     "traffic": traffic, "traffic_source": traffic_src,
                     "algorithmic_bytes": m["enc_bytes"], "launch_ms": round(m["t_enc"], 4)},
        "detail": {"t_encode_ms": round(m["t_enc"], 4), "t_apply_ms": round(m["t_app"], 4),
                   "encode_scanned_GBs": round(m["scanned"] / 1e9 / (m["t_enc"] / 1e3), 1),
                   "apply_algorithmic_GBs": round(m["app_bytes"] / 1e9 / (m["t_app"] / 1e3), 1) if m["t_app"] > 0 else None,
                   "encode_plus_apply_algorithmic_frac_of_peak": round(m["both_frac"], 4),
                   "apply_line_model_bytes": int(m["app_line_bytes"]),
                   "apply_line_model_frac_of_peak": round(m["app_line_frac"], 4) if m["app_line_frac"] else None,
                   "apply_memory_model_bytes": int(m["app_mem_bytes"]),
                   "apply_memory_model_frac_of_peak": round(m["app_mem_frac"], 4) if m["app_mem_frac"] else None,
                   "t_dense_copy_ms": round(m["t_copy"], 4),
                   "wire_bytes_sparse_over_dense": round(6 * m["nnz"] / (2 * m["n_elems"]), 4),
                   "modelled_sync": crossover,
                   "bw_probe": m.get("bw_probe"), "tiles": m["tiles"]},
    }

    # the other target configuration, in the same process: 7B-style decoder, TP = 4, at 1 / 5 / 10 %
    if args.workload == "decoder32b_tp8" and not args.no_extra and args.layers is None and args.tp_src == 1 \
            and args.pp_src == 1 and args.pp_dst == 1:
        extra = {}
        t7, tp7, rec7, _ = workload("decoder7b_tp4")
        for p7 in (0.01, 0.05, 0.1):
            e = measure(R, "decoder7b_tp4", t7, tp7, rec7, p7, args, max(5, args.steps // 2), 2, False, False)
            extra["p%g" % p7] = {"density": p7, "elements": e["n_elems"], "nnz": e["nnz"],
                                 "t_encode_ms": round(e["t_enc"], 4), "t_apply_ms": round(e["t_app"], 4),
                                 "ms_per_step": round(e["ms_per_step"], 4),
                                 "value_GBs_scanned": round(e["scanned"] / 1e9 / (e["ms_per_step"] / 1e3), 1),
                                 "encode_frac_of_peak": round(e["enc_frac"], 4),
                                 "encode_plus_apply_algorithmic_frac_of_peak": round(e["both_frac"], 4),
                                 "apply_line_model_frac_of_peak": round(e["app_line_frac"], 4),
                                 "apply_memory_model_frac_of_peak": round(e["app_mem_frac"], 4)}
        out["detail"]["decoder7b_tp4"] = extra

    if want_cpu:
        out["cpu_baseline"] = cpu_baseline(m["host_sample"], tp, m["in_bytes_per_elem"])
    print(json.dumps(out), flush=True)


def cpu_baseline(sample, tp, in_bytes_per_elem):
    """The oracle as it stands on a sample of the same workload: once on one thread, once with the
    work dealt to a pool of threads (the oracle's C code runs outside the interpreter lock).  Work
    items are whole tensors; a single-tensor workload is cut into chunks of 2^24 elements whose
    entry lists follow each other in order."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor
    from oracle import oracle

    work, done = sample
    if len(work) == 1 and tp == 1:
        t, ho, hn = work[0]
        chunk = 1 << 24
        work = [(dict(t, rows=1, cols=min(chunk, ho.size - a), rule=0, sections=None), ho[a:a + chunk], hn[a:a + chunk])
                for a in range(0, ho.size, chunk)]

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
    # every core this process may use: the scheduler's set, and never more workers than the box's
    # stated share of cores (it exports that as OMP_NUM_THREADS)
    found = os.cpu_count() or 1
    usable = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else found
    share = int(os.environ.get("OMP_NUM_THREADS", "0") or 0)
    threads = max(1, min(usable, share or usable, len(work)))
    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=threads) as pool:
        list(pool.map(one, work))
    secs_n = time.perf_counter() - t0
    rate = lambda s: round(in_bytes_per_elem * done / 1e9 / s, 3)
    return {"value": rate(secs_n), "unit": "GB/s", "cores": threads, "kind": "oracle", "value_1core": rate(secs1),
            "cores_found": found, "cores_usable": usable, "core_share": share or None,
            "sample": "%d work items (first tensors of the workload, %d elements), encode+apply, %.1f s on one thread, "
                      "%.1f s on %d" % (len(work), done, secs1, secs_n, threads)}


if __name__ == "__main__":
    main()
