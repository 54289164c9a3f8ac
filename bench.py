#!/usr/bin/env python3
"""Benchmark of the IVF hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2]

A step is one pass of the whole hot path over one batch of the workload: coarse search,
work-list build, list scan, top-k merge for the query batch, plus the insert batch the
config interleaves (assign + append).  All inputs are resident in HBM before the timed
region.  Prints ONE JSON line (see the design doc for the fields).
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

HBM_PEAK_GBS = 8000.0  # MI355X datasheet HBM3E bandwidth


def log(msg):
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


class SingleIndexWorkload:
    """Configs with one index: c1 (tiny), c2 (single agent), c4 (large static fp16), c5 (skewed dynamic)."""

    def __init__(self, cfg, steps_total, threads):
        import torch
        from paper_2602_21477_amd import binding as B
        from paper_2602_21477_amd import workload as W
        self.cfg, self.W, self.B, self.torch = cfg, W, B, torch
        self.threads = threads
        self.insert_m = {1: 1, 2: 8, 4: 0, 5: 1}[cfg.index]
        self.n_query_batches = 16
        self.steps_total = steps_total

    def setup(self):
        cfg, W, B, torch = self.cfg, self.W, self.B, self.torch
        t0 = time.time()
        if cfg.train == "component_means":
            self.x, comp = W.vectors(cfg, 0, cfg.n, threads=self.threads, with_components=True)
            self.cent = W.train_centroids(cfg, self.x, comp=comp)
        else:
            self.x = W.vectors(cfg, 0, cfg.n, threads=self.threads)
            log(f"generated {cfg.n} x {cfg.d} in {time.time() - t0:.1f}s")
            t1 = time.time()
            self.cent = W.train_centroids(cfg, self.x)
            log(f"trained {cfg.nlist} centroids in {time.time() - t1:.1f}s")
        t1 = time.time()
        xd = torch.empty((cfg.n, cfg.d), dtype=torch.float32, device="cuda")
        step = 1 << 20
        for s in range(0, cfg.n, step):
            xd[s:s + step].copy_(torch.from_numpy(self.x[s:s + step]))
        reserve = self.insert_m * self.steps_total
        self.index = B.Index(torch.from_numpy(self.cent).cuda(), xd, metric=cfg.metric, storage=cfg.storage,
                             insert_reserve=reserve + 1024)
        del xd
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        log(f"uploaded and built the index in {time.time() - t1:.1f}s")
        self.q_host = [W.queries(cfg, b) for b in range(self.n_query_batches)]
        self.q = [torch.from_numpy(q).cuda() for q in self.q_host]
        self.out_ids = torch.empty((cfg.nq, cfg.k), dtype=torch.int64, device="cuda")
        self.out_dist = torch.empty((cfg.nq, cfg.k), dtype=torch.float32, device="cuda")
        if self.insert_m:
            ins = np.concatenate([W.inserts(cfg, b, 256) for b in range((reserve + 255) // 256)])
            self.ins = torch.from_numpy(ins).cuda()
        self.step_no = 0
        torch.cuda.synchronize()

    @property
    def handle(self):
        return self.index.handle

    def step(self):
        B, cfg, i = self.B, self.cfg, self.step_no
        if cfg.index == 5 and self.insert_m:  # skewed dynamic: insert first, then search
            B.pk_insert(self.handle, self.ins[i:i + 1])
        B.pk_search(self.handle, self.q[i % self.n_query_batches], cfg.k, cfg.nprobe, self.out_ids, self.out_dist)
        if cfg.index != 5 and self.insert_m:
            m = self.insert_m
            B.pk_insert(self.handle, self.ins[i * m:(i + 1) * m])
        self.step_no += 1

    def queries_per_step(self):
        return self.cfg.nq

    def row_bytes(self):
        return self.cfg.d * (2 if self.cfg.storage == self.B.PK_F16 else 4)

    def recall(self, nsample):
        """recall@10 of the GPU search against the oracle's exact search on a few queries."""
        import oracle
        q = self.q_host[0][:nsample]
        ids, _ = self.index.search(self.q[0][:nsample].contiguous(), max(10, self.cfg.k), self.cfg.nprobe)
        bi, _ = oracle.bruteforce(self.x, q, 10, self.cfg.metric)
        got = ids.cpu().numpy()
        return float(np.mean([len(set(a[:10].tolist()) & set(b.tolist())) / 10.0 for a, b in zip(got, bi)]))

    def cpu_baseline(self, budget_s=12.0):
        """The oracle as it stands, on a bounded sample: an index over the first n/f rows with nlist/f
        lists (same list length, same nprobe and k, so the same number of vectors scanned per query)."""
        import oracle
        cfg, W = self.cfg, self.W
        f = 1
        while cfg.n // f * (cfg.nlist // f) * cfg.d > 2.5e10 and cfg.nlist // (f * 2) >= cfg.nprobe:
            f *= 2
        n_s, nlist_s = cfg.n // f, cfg.nlist // f
        xs = self.x[:n_s]
        if f == 1:
            cent = self.cent
        elif cfg.train == "component_means":
            cent = self.cent[:nlist_s]
        else:
            sub = W.scaled(cfg, nlist=nlist_s)
            rows = W.train_rows(sub, n_s)
            cent = W.lloyd(xs[rows], W.init_rows(sub, len(rows)), 4)
        t0 = time.time()
        ix = oracle.Index(cent, cfg.metric)
        ix.build(xs)
        build_s = time.time() - t0
        q = self.q_host[1][:min(cfg.nq, 64)]
        done, t0 = 0, time.time()
        while True:
            ix.search(q, cfg.k, cfg.nprobe)
            done += len(q)
            if time.time() - t0 > max(1.0, budget_s - build_s) / 2:
                break
        dt = time.time() - t0
        scanned = float(np.sort(ix.list_lengths())[::-1][:cfg.nprobe].sum())
        return {"value": done / dt, "unit": "queries/s", "cores": oracle.num_threads(), "kind": "oracle",
                "sample": f"{done} queries (nprobe={cfg.nprobe}, k={cfg.k}) on an oracle index over the first "
                          f"{n_s} rows with {nlist_s} lists (1/{f} of the workload, same list length, so the same "
                          f"vectors scanned per query; <= {scanned:.0f} per query); oracle build {build_s:.1f}s not "
                          f"included"}


def run(args):
    import torch
    from paper_2602_21477_amd import binding as B
    from paper_2602_21477_amd import workload as W

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU (the HIP path has no CPU fallback)")
    torch.cuda.set_device(0)
    B.lib()
    cfg = {"c1": W.C1, "c2": W.C2, "c4": W.C4, "c4ip": W.scaled(W.C4, metric=W.METRIC_IP), "c5": W.C5}[args.workload]
    steps_total = args.warmup + 2 * args.steps + 8
    threads = min(16, len(os.sched_getaffinity(0)))
    wl = SingleIndexWorkload(cfg, steps_total, threads)
    wl.setup()

    for _ in range(args.warmup):
        wl.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        wl.step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    qps = wl.queries_per_step() * args.steps / dt
    log(f"{args.steps} steps in {dt:.3f}s -> {qps:.0f} queries/s")

    # same steps again with HIP events around the stages of every search (on the search's stream)
    B.pk_profile_begin(wl.handle)
    for _ in range(args.steps):
        wl.step()
    pr = B.pk_profile_end(wl.handle)
    n = max(pr.launches, 1)
    scan_ms = pr.scan_ms / n
    alg_bytes = pr.scanned_rows / n * wl.row_bytes()
    achieved = alg_bytes / (scan_ms * 1e-3) / 1e9 if scan_ms > 0 else 0.0
    stages = {"coarse_ms": pr.coarse_ms / n, "worklist_ms": pr.worklist_ms / n, "scan_ms": scan_ms,
              "select_ms": pr.select_ms / n, "tiles": pr.tiles / n, "candidates": pr.candidates / n,
              "emitted": pr.emitted / n}
    log(f"stages per search: {stages}")
    st = wl.index.stats()
    if st.device_error:
        raise SystemExit(f"device error flag {st.device_error}")

    out = {
        "metric": "search queries/sec at recall@10>=0.9 (1 GPU); list-scan HBM GB/s vs peak",
        "value": qps, "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16" if cfg.storage == B.PK_F16 else "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "n": int(st.n_total), "d": cfg.d, "nlist": cfg.nlist, "nprobe": cfg.nprobe,
                   "k": cfg.k, "queries_per_step": cfg.nq, "inserts_per_step": wl.insert_m,
                   "metric": "ip" if cfg.metric == W.METRIC_IP else "l2"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None, "kernel": "scan_kernel (list scan)",
                     "algorithmic_bytes_per_launch": alg_bytes, "kernel_ms": scan_ms},
        "stages_ms": stages,
    }
    if not args.no_recall:
        out["recall_at_10"] = wl.recall(args.recall_queries)
        log(f"recall@10 = {out['recall_at_10']:.4f}")
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = wl.cpu_baseline()
        log(f"cpu baseline: {out['cpu_baseline']['value']:.1f} queries/s on {out['cpu_baseline']['cores']} threads")
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c4", "c4ip", "c5"])
    ap.add_argument("--recall-queries", type=int, default=8)
    ap.add_argument("--no-recall", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); run with --gpus 1. "
              "DESIGN.md describes how the path would shard.", file=sys.stderr)
        raise SystemExit(2)
    run(args)


if __name__ == "__main__":
    main()
