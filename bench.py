#!/usr/bin/env python3
"""Benchmark of the blocked matrix-factorization SGD path on one MI355X.

A "step" is one epoch: for every stratum, localize the blocks, then pull / SGD
step / push for every entry of the stratum's blocks, then the barrier.  The
inputs (entries, factors, schedule) are resident in device memory before the
timed region starts.  Prints ONE JSON line on stdout; everything else goes to
stderr.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload wide|large|medium|tiny|complex] [--scale S]

The default workload is the largest configuration, wide (10M x 1M, 500M entries, rank 100); the large one
(480,189 x 17,770, 100M entries) is run in the same call and reported under "other_workloads".
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X HBM3E, published

# HBM bytes per launch of the SGD kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by what the same
# counters read for a plain 1 GiB copy; summaries under profiles/).  Only valid for the kernel sources they were
# taken with and for the default settings of the workload: bytes read, bytes written.
KERNEL_SOURCES = ("mf_sgd_chunk.hip", "mf_sgd.hip", "mf_device.h", "common.h")
TRAFFIC = {"kernel_sha256_16": "b7ddbd8b5d104008",
           "bytes_per_launch": {"large": (147068367.0, 125882961.0), "wide": (1324683903.0, 953180179.0)}}

# block boundaries per workload: a column of a block weighs this many entries on top of its own (see --col-cost)
COL_COST = {"wide": 3.0}


def kernel_sources_hash():
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        h.update(open(os.path.join(ROOT, "paper_2002_00655_amd", "csrc", name), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(args, name):
    """(bytes read, bytes written) per launch from the committed counter runs, or None when the kernel sources or
    the settings are not the ones the counters were taken with."""
    default = (args.scale == 1.0 and args.bounds == "balanced" and args.col_cost is None and args.waves == 0 and args.cache_rows == -1
               and args.heavy_len == 0 and args.team_max == 0 and not (args.entry_kernel or args.classic or args.handoff))
    rw = TRAFFIC["bytes_per_launch"].get(name)
    if default and rw and rw[0] > 0 and kernel_sources_hash() == TRAFFIC["kernel_sha256_16"]:
        return rw
    return None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(w, rb, cb, d, target_seconds=10.0):
    """The CPU oracle timed on a bounded sample of one epoch: the entries of the first K row blocks, i.e. K of the d
    workers in every one of the d subepochs, K sized to the time target.  Once on one core - the oracle as it stands -
    and once with the workers of a subepoch side by side on all cores (same result bit for bit: Sec. 2.2.2)."""
    from oracle.oracle import Oracle, mf_block_ratings
    from paper_2002_00655_amd import workloads as wl
    assumed_rate = 4e6                            # updates/s of one core, only used to size the sample
    cores = os.cpu_count() or 1
    K = int(round(assumed_rate * target_seconds / (w.nnz / d)))
    K = max(1, min(d, max(K, min(cores, 16))))
    hi = int(np.searchsorted(w.rows, rb[K], side="left"))      # the entries come sorted by (row, column)
    rows, cols, vals = w.rows[:hi], w.cols[:hi], w.vals[:hi]
    br, bc, bv, bp = mf_block_ratings(w.m, w.n, rows, cols, vals, rb, cb)
    sched = wl.cyclic_schedule(d)[:, :K]
    out = {}
    check = None
    for leg in ("one_core", "all_cores"):
        orc = Oracle("f32", w.m + w.n, w.rank, d)
        orc.push(np.arange(w.m), w.W0)
        orc.push(w.m + np.arange(w.n), w.H0)
        t0 = time.perf_counter()
        if leg == "one_core":
            orc.mf_sgd_epoch(w.m, w.n, br, bc, bv, rb, cb, bp, sched, w.lr, w.lam)
            used = 1
        else:
            used = orc.mf_sgd_epoch_workers(w.m, w.n, br, bc, bv, rb, cb, bp, sched, w.lr, w.lam)
        dt = time.perf_counter() - t0
        probe = orc.pull(np.arange(0, min(w.m, 4096)))
        if check is None:
            check = probe
        elif not np.array_equal(check, probe):
            raise RuntimeError("the all-core oracle run differs from the one-core run")
        out[leg] = {"value": rows.size / dt, "cores": used, "seconds": dt}
        del orc
    return {"value": out["one_core"]["value"], "unit": "updates/s", "cores": 1, "kind": "oracle",
            "sample": f"sample, not a full epoch: the first {K} of {d} row blocks (= {K} of the {d} workers) through all {d} subepochs "
                      f"of one epoch, {rows.size} updates, {out['one_core']['seconds']:.1f} s on one core, fp32 oracle, gcc -O2",
            "all_cores": {"value": out["all_cores"]["value"], "unit": "updates/s", "cores": out["all_cores"]["cores"],
                          "seconds": out["all_cores"]["seconds"],
                          "note": "same sample, the workers of a subepoch side by side (OpenMP), result identical to the one-core run"},
            "nproc": cores, "cpu_model": cpu_model()}


def chain_latency(P, torch, dev, rank, lr, lam):
    """Measured time per update along one dependency chain of the SGD kernel: all entries of one column (one after
    the other through that column's factor) and all entries of one row, each as a block of its own.  Every blocking
    of a matrix leaves these chains intact, so (largest column degree) x (column figure) and (largest row degree) x
    (row figure) bound an epoch from below whatever the bandwidth."""
    out = []
    for kind, nnz in (("column", 61440), ("row", 8000)):
        idx = torch.arange(nnz, dtype=torch.int32, device=dev)
        zero = torch.zeros(nnz, dtype=torch.int32, device=dev)
        rows, cols = (idx, zero) if kind == "column" else (zero, idx)
        m, n = (nnz, 1) if kind == "column" else (1, nnz)
        g = torch.Generator(device=dev); g.manual_seed(1)
        vals = torch.rand(nnz, device=dev, generator=g)
        rb, cb = np.array([0, m], np.int64), np.array([0, n], np.int64)
        br, bc, bv, bp = P.mf_block_ratings(m, n, rows, cols, vals, rb, cb)
        srv = P.ParameterServer(m + n, rank, 1)
        srv.push(torch.arange(m + n, device=dev), (torch.rand((m + n, rank), device=dev, generator=g) - 0.5) / rank ** 0.5)
        srv.mf_load_ratings(m, n, br, bc, bv, rb, cb, bp)
        sched = np.zeros((1, 1, 3), np.int32)
        srv.mf_sgd_epoch(sched, lr, lam)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(5):
            srv.mf_sgd_epoch(sched, lr, lam)
        torch.cuda.synchronize()
        out.append((time.perf_counter() - t0) / 5 / nnz * 1e9)
        srv.status()
        del srv
    return out[0], out[1]


def bench_kge(args, torch, dev) -> int:
    """One step = one mini-batch of the knowledge-graph-embedding workload: keys of the batch's positive triples
    and their negatives (one slot per key of a data point: subject, relation, object, each negative), pull, one
    AdaGrad update per slot on the gradient summed over the data point's triples, push.  Value: scored triples per
    second.  The mean loss per scored triple is reported for the first step, the last timed-size step, and for the
    first batch again after all the steps (the same data, so the fall is the training's)."""
    from paper_2002_00655_amd import workloads as wl
    from paper_2002_00655_amd import ps as P
    t0 = time.perf_counter()
    B = args.batch
    nsteps = args.warmup + args.steps
    s = args.scale
    w = wl.make_kge(num_entities=max(1000, int(500_000 * s)), num_relations=max(10, int(600 * s)), triples=max(B * nsteps, int(3_000_000 * s)))
    t_gen = time.perf_counter() - t0
    K, L = w.num_entities + w.num_relations, 4 * w.dim
    ns, no = w.neg_subj.shape[1], w.neg_obj.shape[1]
    per = 1 + ns + no
    slots = 3 + ns + no
    log(f"workload {w.name}: {w.num_entities} entities, {w.num_relations} relations, {w.subj.size} triples, dim {w.dim}, "
        f"{ns}+{no} negatives, batch {B}; generated in {t_gen:.1f} s")
    srv = P.ParameterServer(K, L, 4)
    init = torch.zeros((K, L), device=dev)
    init[:w.num_entities, :2 * w.dim] = torch.from_numpy(w.E0).to(dev)
    init[w.num_entities:, :2 * w.dim] = torch.from_numpy(w.R0).to(dev)
    for lo in range(0, K, 1 << 17):
        hi = min(K, lo + (1 << 17))
        srv.push(torch.arange(lo, hi, device=dev), init[lo:hi])
    del init
    nb = w.subj.size // B
    subj, rel, obj, negs, nego = (torch.from_numpy(np.ascontiguousarray(x[:nb * B])).to(dev) for x in (w.subj, w.rel, w.obj, w.neg_subj, w.neg_obj))

    def step(i, want_loss=False):
        sl = slice((i % nb) * B, (i % nb + 1) * B)
        return srv.kge_sgd_step(w.num_entities, w.dim, subj[sl], rel[sl], obj[sl], negs[sl], nego[sl], 0.1, 1e-10, 0, want_loss=want_loss)
    loss0 = step(0, True) / (B * per)
    for i in range(1, max(1, args.warmup)):
        step(i)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for i in range(args.steps):
        step(args.warmup + i)
    ev1.record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    srv.status()
    loss1 = step(args.warmup + args.steps, True) / (B * per)
    loss_again = step(0, True) / (B * per)
    ms_per_step = dt / args.steps * 1e3
    scored_per_s = B * per * args.steps / dt
    log(f"{args.steps} steps in {dt:.3f} s: {ms_per_step:.3f} ms/step (stream time {ev0.elapsed_time(ev1) / args.steps:.3f} ms), "
        f"{scored_per_s / 1e6:.2f} M scored triples/s; mean loss {loss0:.4f} (first step) -> {loss1:.4f} (step {args.warmup + args.steps}), "
        f"first batch again {loss_again:.4f}")
    # byte model per key slot: its value read once (pull) and the stored value read and written once (push),
    # plus its 8-byte key: 3 x 4 L + 8
    bytes_per_occ = 12 * L + 8
    model = B * slots * args.steps / dt * bytes_per_occ / 1e9
    result = {
        "metric": "scored triples/sec, ComplEx dim %d with AdaGrad through pull/push" % w.dim, "value": scored_per_s, "unit": "triples/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "complex_kge", "entities": w.num_entities, "relations": w.num_relations, "dim": w.dim,
                   "negatives": f"{ns}+{no}", "batch": B, "key_slots_per_step": B * slots, "lr": 0.1, "eps": 1e-10},
        "positive_triples_per_s": B * args.steps / dt,
        "roofline": {"bound": "hbm", "achieved": model, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": model / HBM_PEAK_GBS, "traffic": None,
                     "kernel": "whole step (keys, pull, updates, push)", "bytes_per_key_slot": bytes_per_occ,
                     "note": "algorithmic bytes (model: 12 L + 8 per key slot) over the step's wall time"},
        "mean_loss": {"first_step": loss0, "last_step": loss1, "first_batch_again": loss_again, "steps_between": args.warmup + args.steps},
    }
    if not args.no_cpu_baseline:
        from oracle.oracle import Oracle
        orc = Oracle("f32", K, L, 4)
        init_h = np.zeros((K, L), np.float32)
        init_h[:w.num_entities, :2 * w.dim] = w.E0
        init_h[w.num_entities:, :2 * w.dim] = w.R0
        orc.push(np.arange(K), init_h)
        del init_h
        t0 = time.perf_counter()
        done = 0
        while done < nb and time.perf_counter() - t0 < args.cpu_seconds:          # the same batches, in the same order
            sl = slice(done * B, (done + 1) * B)
            orc.kge_step(w.num_entities, w.dim, w.subj[sl], w.rel[sl], w.obj[sl], w.neg_subj[sl], w.neg_obj[sl], 0.1, 1e-10, 0)
            done += 1
        dtc = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": done * B * per / dtc, "unit": "triples/s", "cores": 1, "nproc": os.cpu_count(), "cpu_model": cpu_model(),
                                  "kind": "oracle",
                                  "sample": f"the first {done} steps of {B} positive triples ({done * B * per} scored, {dtc:.1f} s), fp32 oracle, gcc -O2, one core"}
        log(f"cpu oracle: {result['cpu_baseline']['value']:.0f} scored triples/s")
    print(json.dumps(result), flush=True)
    return 0


def bench_kge_epoch(args, torch, dev) -> int:
    """Epochs of the knowledge-graph workload over several workers with the data partitioned by relation and the next
    batch's entities localized ahead (kge_sgd_epoch): time per epoch and the share of accesses that are remote
    (localization conflicts), for 1, 2, 4, 8 workers with pre-localization and 8 workers without; the last two again
    with location caches, which change the number of messages that remote accesses cost."""
    from paper_2002_00655_amd import workloads as wl
    from paper_2002_00655_amd import ps as P
    s = args.scale
    w = wl.make_kge(num_entities=max(1000, int(500_000 * s)), num_relations=max(10, int(600 * s)), triples=max(args.batch, int(3_000_000 * s)))
    K, L = w.num_entities + w.num_relations, 4 * w.dim
    per = 1 + w.neg_subj.shape[1] + w.neg_obj.shape[1]
    rows = []
    for parts, lookahead, caches in ((1, 1, 0), (2, 1, 0), (4, 1, 0), (8, 1, 0), (8, 0, 0), (8, 1, 1), (8, 0, 1)):
        wp, part_ptr = wl.partition_by_relation(w, parts)
        srv = P.ParameterServer(K, L, 8)
        srv.set_option(P.OPT_LOCATION_CACHES, caches)
        init = torch.zeros((K, L), device=dev)
        init[:w.num_entities, :2 * w.dim] = torch.from_numpy(w.E0).to(dev)
        init[w.num_entities:, :2 * w.dim] = torch.from_numpy(w.R0).to(dev)
        for lo in range(0, K, 1 << 17):
            hi = min(K, lo + (1 << 17))
            srv.push(torch.arange(lo, hi, device=dev), init[lo:hi])
        del init
        data = [torch.from_numpy(np.ascontiguousarray(x)).to(dev) for x in (wp.subj, wp.rel, wp.obj, wp.neg_subj, wp.neg_obj)]
        srv.kge_sgd_epoch(w.num_entities, w.dim, *data, part_ptr, args.batch, lookahead, 0.1, 1e-10, want_loss=False)   # warm-up epoch
        torch.cuda.synchronize()
        st0 = srv.stats()
        t0 = time.perf_counter()
        loss = srv.kge_sgd_epoch(w.num_entities, w.dim, *data, part_ptr, args.batch, lookahead, 0.1, 1e-10)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        st = {k: v - st0[k] for k, v in srv.stats().items()}
        acc = st["pull_local"] + st["pull_remote"]
        msgs = st["msg_acc_req"] + st["msg_acc_fwd"] + st["msg_acc_reply"]
        res = {"workers": parts, "lookahead": lookahead, "location_caches": caches, "epoch_s": dt,
               "scored_triples_per_s": w.subj.size * per / dt, "remote_share": st["pull_remote"] / acc, "relocated": st["relocated"],
               "localize_keys": st["localize_keys"], "access_messages": msgs, "cache_hit": st["cache_hit"], "cache_stale": st["cache_stale"],
               "mean_loss": loss / (w.subj.size * per)}
        rows.append(res)
        log(f"workers {parts} lookahead {lookahead} location caches {caches}: epoch {dt * 1e3:.1f} ms, "
            f"{res['scored_triples_per_s'] / 1e6:.1f} M scored triples/s, remote accesses {100 * res['remote_share']:.2f} %, "
            f"relocations {st['relocated']}, messages of remote accesses {msgs} (entries correct {st['cache_hit']}, stale {st['cache_stale']}), "
            f"mean loss {res['mean_loss']:.4f}")
        del srv, data
    print(json.dumps({"metric": "knowledge-graph epoch over workers", "unit": "s", "n_gpus": 1, "dtype": "f32", "data": "synthetic",
                      "config": {"workload": "complex_kge_epoch", "entities": w.num_entities, "relations": w.num_relations,
                                 "triples": int(w.subj.size), "dim": w.dim, "batch": args.batch}, "results": rows}), flush=True)
    return 0


def bench_ps_micro(args, torch, dev) -> int:
    """Stand-alone primitives on a store of the large workload's size (value length 100): pull, push, localize
    for 2^20 .. 2^24 keys, uniform and Zipf(1.0); rows/s and GB/s by the byte model of each (pull: key + row read
    + row written = 8 + 8 L; push: key + update row + stored row read and written = 8 + 12 L; localize: key +
    owner read and written = 16)."""
    from paper_2002_00655_amd import ps as P
    K, L, W = 497_959, 100, 256
    srv = P.ParameterServer(K, L, W)
    g = torch.Generator(device=dev); g.manual_seed(0)
    zipf_w = (torch.arange(1, K + 1, device=dev, dtype=torch.float64) ** -1.0)
    zipf_cdf = torch.cumsum(zipf_w / zipf_w.sum(), 0)
    perm = torch.randperm(K, device=dev, generator=g)
    rows = []
    for logn in (20, 22, 24):
        n = 1 << logn
        for dist in ("uniform", "zipf"):
            if dist == "uniform":
                keys = torch.randint(0, K, (n,), device=dev, generator=g)
            else:
                u = torch.rand(n, device=dev, dtype=torch.float64, generator=g)
                keys = perm[torch.searchsorted(zipf_cdf, u).clamp_(max=K - 1)]
            buf = torch.zeros((n, L), device=dev)
            res = {"n": n, "keys": dist}
            for name, fn, nbytes in (("pull", lambda: srv.pull(keys, 0, out=buf), 8 + 8 * L),
                                     ("push", lambda: srv.push(keys, buf, 0), 8 + 12 * L),
                                     ("localize", lambda: srv.localize(keys, 1), 16)):
                fn(); torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(3):
                    fn()
                torch.cuda.synchronize()
                dt = (time.perf_counter() - t0) / 3
                res[name] = {"rows_per_s": n / dt, "model_gbs": n * nbytes / dt / 1e9}
            del buf
            srv.status()
            rows.append(res)
            log(f"n=2^{logn} {dist:8s}: " + ", ".join(f"{k} {res[k]['rows_per_s'] / 1e9:.2f} G rows/s ({res[k]['model_gbs']:.0f} GB/s)"
                                                        for k in ("pull", "push", "localize")))
    print(json.dumps({"metric": "parameter-server primitives, rows/s", "unit": "rows/s", "n_gpus": 1, "dtype": "f32", "data": "synthetic",
                      "config": {"workload": "ps_micro", "num_keys": K, "value_len": L, "workers": W}, "results": rows}), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="wide", choices=["tiny", "medium", "large", "wide", "complex"])
    ap.add_argument("--no-also-large", dest="also_large", action="store_false",
                    help="with the default workload (wide): do not also run the large one")
    ap.add_argument("--batch", type=int, default=8192, help="positive triples per step (complex only)")
    ap.add_argument("--scale", type=float, default=1.0)
    ap.add_argument("--bounds", default="balanced", choices=["equal", "balanced"],
                    help="block boundaries: ranges with equal numbers of entries (default; see --col-cost) or of equal length")
    ap.add_argument("--col-cost", type=float, default=None,
                    help="balanced bounds: a column of a block weighs this many entries on top of its own (0: entries only; "
                         "default: 8, wide 4)")
    ap.add_argument("--waves", type=int, default=0, help="wavefronts per workgroup of the SGD kernel (0: library default)")
    ap.add_argument("--cache-rows", type=int, default=-1)
    ap.add_argument("--heavy-len", type=int, default=0, help="column runs at least this long are processed in groups (0: library default)")
    ap.add_argument("--team-max", type=int, default=0, help="most wavefronts per long column run (0: library default)")
    ap.add_argument("--classic", type=int, default=0, choices=[0, 1, 2],
                    help="the epoch as on a classic parameter server (1: values copied out and back, 2: updated in place)")
    ap.add_argument("--handoff", action="store_true",
                    help="epochs without barriers: column blocks handed from worker to worker (mf_sgd_epoch_handoff), one launch per epoch")
    ap.add_argument("--col-blocks", type=int, default=0, help="column blocks (0: as many as row blocks; other values need --handoff)")
    ap.add_argument("--entry-kernel", action="store_true", help="use the entry-by-entry SGD kernel instead of the grouped one")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="size of the CPU oracle's sample, in seconds of one core")
    ap.add_argument("--kge-epoch", action="store_true", help="only time knowledge-graph epochs over 1..8 workers (kge_sgd_epoch)")
    ap.add_argument("--ps-micro", action="store_true", help="only time the stand-alone pull / push / localize primitives")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain device copy of 1 GiB five times (reference for the HBM traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path runs on one GPU; --gpus must be 1 (no multi-GPU figure is produced)", file=sys.stderr)
        return 2

    import torch
    from paper_2002_00655_amd import workloads as wl
    from paper_2002_00655_amd import ps as P

    torch.cuda.set_device(0)
    dev = torch.device("cuda")
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)        # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": src.numel() * 4, "copy_bytes_written": dst.numel() * 4, "copies": 5}))
        return 0
    props = torch.cuda.get_device_properties(0)
    log(f"device: {props.name} {props.gcnArchName}, {props.multi_processor_count} CUs, host cores {os.cpu_count()}")
    if args.ps_micro:
        return bench_ps_micro(args, torch, dev)
    if args.kge_epoch:
        return bench_kge_epoch(args, torch, dev)
    if args.workload == "complex":
        return bench_kge(args, torch, dev)

    primary = run_mf(args, args.workload, torch, dev, full=True)
    if primary is None:
        return 2
    if args.workload == "wide" and args.also_large and args.scale == 1.0 and not (args.handoff or args.classic or args.entry_kernel):
        # the other rank-100 configuration, in the same call (boundaries and kernel settings: its own defaults)
        other = run_mf(args, "large", torch, dev, full=False)
        if other is not None:
            keep = ("value", "unit", "ms_per_step", "config", "model_frac_of_hbm_peak", "train_rmse", "roofline", "critical_path")
            primary["other_workloads"] = {"large_mf": {k: other[k] for k in keep if k in other}}
    print(json.dumps(primary), flush=True)
    return 0


def run_mf(args, name, torch, dev, full):
    """One matrix-factorization workload: set-up, warm-up, the timed epochs, the roofline entry; with `full` also the
    pull / push figure, the dependency-chain bound and the CPU oracle.  Returns the result (a dict), or None."""
    from paper_2002_00655_amd import workloads as wl
    from paper_2002_00655_amd import ps as P
    t0 = time.perf_counter()
    w = wl.make_mf(name, scale=args.scale)
    d = w.d_row
    d_col = args.col_blocks if args.col_blocks > 0 else d
    if d_col != d and not args.handoff:
        print("bench.py: --col-blocks needs --handoff (the rotating schedule has as many column blocks as workers)", file=sys.stderr)
        return None
    col_cost = args.col_cost if args.col_cost is not None else COL_COST.get(name, 8.0)
    if args.bounds == "balanced":
        rb, cb = wl.balanced_bounds(w.rows, w.m, d), wl.balanced_bounds(w.cols, w.n, d_col, per_id=col_cost * d)
    else:
        rb, cb = wl.equal_bounds(w.m, d), wl.equal_bounds(w.n, d_col)
    max_col_deg = int(np.bincount(w.cols, minlength=w.n).max())
    max_row_deg = int(np.bincount(w.rows, minlength=w.m).max())
    t_gen = time.perf_counter() - t0
    log(f"workload {w.name}: {w.m} x {w.n}, nnz {w.nnz}, rank {w.rank}, {d} x {d_col} blocks ({args.bounds}); generated in {t_gen:.1f} s")

    # data layout on the device (set-up, reported but not part of updates/s)
    rows_d, cols_d, vals_d = (torch.from_numpy(x).to(dev) for x in (w.rows, w.cols, w.vals))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    br, bc, bv, bp = P.mf_block_ratings(w.m, w.n, rows_d, cols_d, vals_d, rb, cb)
    torch.cuda.synchronize()
    t_block = time.perf_counter() - t0
    del rows_d, cols_d, vals_d

    srv = P.ParameterServer(w.m + w.n, w.rank, d)
    if args.waves > 0:
        srv.set_option(P.OPT_MF_WAVES, args.waves)
    srv.set_option(P.OPT_MF_CACHE_ROWS, args.cache_rows)
    if args.heavy_len > 0:
        srv.set_option(P.OPT_MF_HEAVY_LEN, args.heavy_len)
    if args.team_max > 0:
        srv.set_option(P.OPT_MF_TEAM_MAX, args.team_max)
    if args.entry_kernel:
        srv.set_option(P.OPT_MF_GROUPED, 0)
    if args.classic:
        srv.set_option(P.OPT_MF_CLASSIC, args.classic)
    kernel_name = "k_mf_sgd_classic" if args.classic else ("k_mf_sgd" if (args.entry_kernel or w.rank > 128) else "k_mf_sgd_chunk")
    if args.handoff:
        kernel_name = "k_mf_sgd_handoff"
    srv.push(torch.arange(w.m, device=dev), torch.from_numpy(w.W0).to(dev))
    srv.push(w.m + torch.arange(w.n, device=dev), torch.from_numpy(w.H0).to(dev))
    t0 = time.perf_counter()
    srv.mf_load_ratings(w.m, w.n, br, bc, bv, rb, cb, bp)
    torch.cuda.synchronize()
    t_load = time.perf_counter() - t0
    del br, bc, bv
    log(f"set-up on device: block {t_block * 1e3:.1f} ms, load {t_load * 1e3:.1f} ms")

    from paper_2002_00655_amd.ps import _flatten_schedule
    tasks, sptr, _ = _flatten_schedule(wl.cyclic_schedule(d))
    rmse0 = float(np.sqrt(srv.mf_train_sse() / w.nnz))

    def epoch():
        if args.handoff:
            srv.mf_sgd_epoch_handoff(w.lr, w.lam, want_order=False)
        else:
            srv.mf_sgd_epoch_raw(tasks, sptr, w.lr, w.lam)

    for _ in range(args.warmup):
        epoch()
    # The timed region, between a synchronize on each side; an event at each end on the stream the kernels are
    # launched on gives the stream's own time for the same region (no per-launch events: they cost a few
    # microseconds each and would be timing themselves).
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        epoch()
    ev1.record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    stream_s = ev0.elapsed_time(ev1) * 1e-3
    srv.status()
    ms_per_step = dt / args.steps * 1e3
    updates_per_s = w.nnz * args.steps / dt
    rmse1 = float(np.sqrt(srv.mf_train_sse() / w.nnz))
    log(f"{args.steps} epochs in {dt:.3f} s: {ms_per_step:.2f} ms/epoch, {updates_per_s / 1e9:.3f} G updates/s; "
        f"train rmse {rmse0:.4f} -> {rmse1:.4f}")

    # The dominant kernel: one launch per subepoch (per epoch with hand-over), nothing else on the stream in the timed
    # region, so its average duration is the stream time of the region over the launches (it includes the gap
    # between two launches, a microsecond or two: an upper bound of what a kernel trace shows).
    launches = args.steps * (1 if args.handoff else d)
    bytes_per_update = 16 * w.rank + 12            # two rank-r fp32 rows read and written + the 12-byte entry
    units_per_launch = w.nnz * args.steps / launches
    avg_launch_s = stream_s / launches
    achieved = bytes_per_update * units_per_launch / avg_launch_s / 1e9
    rw = measured_traffic(args, name)
    roofline = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                "traffic": None if rw is None else rw[0] + rw[1], "traffic_unit": "bytes per launch", "kernel": kernel_name,
                "avg_launch_us": avg_launch_s * 1e6, "launches": launches, "bytes_per_update": bytes_per_update,
                "updates_per_launch": units_per_launch,
                "model": "achieved = algorithmic bytes (16 r + 12 per update: two rank-r fp32 rows read and written, the 12-byte entry) "
                         "per launch over the launch's duration; traffic = bytes the memory bus really moved per launch (rocprofv3 "
                         "FETCH_SIZE + WRITE_SIZE), less than the algorithmic bytes where factors stay in LDS or in cache"}
    if rw is not None:
        roofline["traffic_read_write"] = list(rw)
        roofline["measured_bus_gbs"] = (rw[0] + rw[1]) / avg_launch_s / 1e9
        roofline["measured_bus_frac"] = roofline["measured_bus_gbs"] / HBM_PEAK_GBS
    log(f"{kernel_name}: {launches} launches, avg {avg_launch_s * 1e6:.1f} us, model {achieved:.0f} GB/s ({100 * achieved / HBM_PEAK_GBS:.1f}% of peak)"
        + ("" if rw is None else f", memory bus {roofline['measured_bus_gbs']:.0f} GB/s ({100 * roofline['measured_bus_frac']:.1f}%)"))

    result = {
        "metric": "SGD updates/sec, MF rank %d" % w.rank, "value": updates_per_s, "unit": "updates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}_mf", "m": w.m, "n": w.n, "nnz": w.nnz, "rank": w.rank, "blocks": f"{d}x{d_col}",
                   "bounds": args.bounds, "col_cost": col_cost, "lr": w.lr, "lambda": w.lam, "waves": args.waves, "kernel": kernel_name},
        "model_gbs": updates_per_s * bytes_per_update / 1e9,
        "model_frac_of_hbm_peak": updates_per_s * bytes_per_update / 1e9 / HBM_PEAK_GBS,
        "setup_ms": {"generate_host": t_gen * 1e3, "block_ratings": t_block * 1e3, "load_ratings": t_load * 1e3},
        "train_rmse": [rmse0, rmse1],
        "roofline": roofline,
    }

    if not (args.classic or args.entry_kernel) and w.rank <= 128:
        # the dependency-chain bound: every entry of a column goes through that column's factor, one after the other,
        # whatever the blocking, and likewise for a row
        col_ns, row_ns = chain_latency(P, torch, dev, w.rank, w.lr, w.lam)
        bound_s = max(max_col_deg * col_ns, max_row_deg * row_ns) * 1e-9
        result["critical_path"] = {"max_col_degree": max_col_deg, "max_row_degree": max_row_deg, "ns_per_update_along_a_column": col_ns,
                                   "ns_per_update_along_a_row": row_ns, "bound_ms_per_epoch": bound_s * 1e3,
                                   "bound_updates_per_s": w.nnz / bound_s, "epoch_over_bound": ms_per_step / (bound_s * 1e3)}
        log(f"dependency chains: busiest column {max_col_deg} entries x {col_ns:.1f} ns, busiest row {max_row_deg} x {row_ns:.1f} ns: "
            f"an epoch takes at least {bound_s * 1e3:.1f} ms ({w.nnz / bound_s / 1e9:.2f} G updates/s); measured {ms_per_step:.1f} ms")

    if full:
        # pull + push rows per second through the C ABI (uniform random keys, value_len = rank)
        n_keys = 1 << 22
        g = torch.Generator(device=dev); g.manual_seed(0)
        keys = torch.randint(0, w.m + w.n, (n_keys,), device=dev, generator=g)
        deltas = torch.zeros((n_keys, w.rank), device=dev)
        out = torch.empty((n_keys, w.rank), device=dev)
        for rep in range(2):
            torch.cuda.synchronize(); t0 = time.perf_counter()
            for _ in range(5):
                srv.pull(keys, 0, out=out)
                srv.push(keys, deltas, 0)
            torch.cuda.synchronize(); t_pp = (time.perf_counter() - t0) / 5
        result["pull_push_rows_per_s"] = 2 * n_keys / t_pp
        result["pull_push_keys_per_call"] = n_keys
        del keys, deltas, out
    del srv
    torch.cuda.empty_cache()
    if full and not args.no_cpu_baseline:
        log("timing the CPU oracle on a sample ...")
        result["cpu_baseline"] = cpu_baseline(w, rb, cb, d, args.cpu_seconds)
        cbl = result["cpu_baseline"]
        log(f"cpu oracle: {cbl['value'] / 1e6:.2f} M updates/s on one core, {cbl['all_cores']['value'] / 1e6:.2f} M on {cbl['all_cores']['cores']} "
            f"({cbl['cpu_model']}, {cbl['nproc']} cores; {cbl['sample']})")
    return result


if __name__ == "__main__":
    sys.exit(main())
