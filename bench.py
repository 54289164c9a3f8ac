#!/usr/bin/env python3
"""Benchmark of the IVF hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4]

A step is one pass of the whole hot path over one batch of the workload: coarse search
(centroid scoring + top-nprobe), threshold sampling, work-list build, list scan, top-k
merge for the query batch, plus the insert batch the config interleaves (assign +
append).  All inputs are resident in HBM before the timed region.  Prints ONE JSON line.

Workloads (the five benchmark configs): c1 tiny, c2 single agent, c3 multi agent, c4 large
static fp16 index under both metrics (c4l2 / c4ip: one of them), c5 skewed dynamic.  The
default, c4, is the 10 M-vector config the HBM target is quoted on; its headline value is
the slower of its two metric variants.
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
sys.path.insert(0, os.path.join(ROOT, "tests"))  # the harness's index training (centroids are an input)
import training  # noqa: E402

HBM_PEAK_GBS = 8000.0  # MI355X datasheet HBM3E bandwidth
METRIC_NAME = "search queries/sec at recall@10>=0.9 (1 GPU); list-scan HBM GB/s vs peak"


MEASURED_STREAM_GBS = 6000.0  # what a bare copy of the scan's load pattern reads on this chip (profiles/scan_kernel_c4_ip.md, section 3)
MEASURED_STREAM_SOURCE = "profiles/scan_kernel_c4_ip.md section 3 (scan load pattern, random data, 6.0-6.3 TB/s)"


def kernel_sources_sha():
    """Hash of the library's sources: a profile's counter figures only describe the kernels they were taken from."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2602_21477_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def profiled_traffic(workload, metric):
    """HBM bytes per scan launch from the committed rocprofv3 counter summary (FETCH_SIZE + WRITE_SIZE,
    calibrated against a plain copy), if there is one for this workload variant AND it was taken from
    the kernels as they are now (the summary records the hash of the sources it was taken from).
    Returns (bytes or None, source description)."""
    import re
    text = None
    # summaries are named for the kernel that scans most of the workload's rows
    for name in (f"scan_kernel_{workload}_{metric}.md", f"scan_ks_kernel_{workload}.md"):
        rel = os.path.join("profiles", name)
        try:
            text = open(os.path.join(ROOT, rel)).read()
            break
        except OSError:
            continue
    if text is None:
        return None, f"profiles/: no summary for {workload} ({metric})"
    m = re.search(r"^traffic_bytes_per_launch:\s*(\d+)", text, re.M)
    k = re.search(r"^kernel_sources_sha:\s*([0-9a-f]+)", text, re.M)
    if not m:
        return None, f"{rel}: no traffic figure"
    if not k or k.group(1) != kernel_sources_sha():
        return None, f"{rel}: taken from other kernel sources ({k.group(1) if k else 'unrecorded'}), now {kernel_sources_sha()}"
    return float(m.group(1)), f"{rel} (kernel sources {k.group(1)})"


def log(msg):
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def host_threads():
    return min(16, len(os.sched_getaffinity(0)))


class Data:
    """Host-side inputs of one agent's memory: rows, centroids (and mixture components)."""

    def __init__(self, cfg, n=None, agent=0):
        from paper_2602_21477_amd import workload as W
        n = cfg.n if n is None else n
        t0 = time.time()
        if cfg.train == "component_means":
            self.x, comp = W.vectors(cfg, 0, n, agent=agent, threads=host_threads(), with_components=True)
            self.cent = training.train_centroids(cfg, self.x, agent=agent, comp=comp)
        else:
            self.x = W.vectors(cfg, 0, n, agent=agent, threads=host_threads())
            self.cent = training.train_centroids(cfg, self.x, agent=agent)
        self.n, self.agent = n, agent
        log(f"agent {agent}: generated {n} x {cfg.d} and trained {cfg.nlist} centroids in {time.time() - t0:.1f}s")

    def upload(self):
        import torch
        xd = torch.empty(self.x.shape, dtype=torch.float32, device="cuda")
        step = 1 << 20
        for s in range(0, self.n, step):
            xd[s:s + step].copy_(torch.from_numpy(self.x[s:s + step]))
        return xd


class Scenario:
    """One timed configuration: indexes on the GPU, query / insert batches resident in HBM."""

    INSERTS = {1: 1, 2: 8, 3: 16, 4: 0, 5: 1}  # insert batch per step (c3: up to 16 per agent)
    N_QUERY_BATCHES = 16

    def __init__(self, cfg, datas, steps_total, xd=None, reserve=None):
        import torch
        from paper_2602_21477_amd import binding as B
        from paper_2602_21477_amd import workload as W
        self.cfg, self.B, self.W, self.torch = cfg, B, W, torch
        self.datas = datas
        self.insert_m = self.INSERTS[cfg.index]
        t0 = time.time()
        self.indexes = []
        for a, dat in enumerate(datas):
            xa = xd if xd is not None else dat.upload()
            self.indexes.append(B.Index(torch.from_numpy(dat.cent).cuda(), xa, metric=cfg.metric, storage=cfg.storage,
                                        insert_reserve=(self.insert_m * steps_total + 1024) if reserve is None
                                        else reserve))
            del xa
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        log(f"built {len(datas)} index(es) ({'ip' if cfg.metric == W.METRIC_IP else 'l2'}) in {time.time() - t0:.1f}s")
        na = len(datas)
        self.q_host = [np.concatenate([W.queries(cfg, b, agent=a) for a in range(na)])
                       for b in range(self.N_QUERY_BATCHES)]
        self.q = [torch.from_numpy(q).cuda() for q in self.q_host]
        self.q_offsets = [a * cfg.nq for a in range(na + 1)]
        nq = na * cfg.nq
        self.out_ids = torch.empty((nq, cfg.k), dtype=torch.int64, device="cuda")
        self.out_dist = torch.empty((nq, cfg.k), dtype=torch.float32, device="cuda")
        self.ins, self.ins_sizes = [], []
        if self.insert_m:
            for a in range(na):
                total = self.insert_m * steps_total
                ins = np.concatenate([W.inserts(cfg, b, 256, agent=a) for b in range((total + 255) // 256)])
                self.ins.append(torch.from_numpy(ins).cuda())
                if cfg.index == 3:
                    self.ins_sizes.append(W.insert_batch_sizes(cfg, steps_total, agent=a))
        self.ins_pos = [0] * na
        self.step_no = 0
        self.reserved = None
        torch.cuda.synchronize()

    @property
    def handle(self):
        return self.indexes[0].handle

    def _insert(self, a, m):
        lo = self.ins_pos[a]
        self.B.pk_insert(self.indexes[a].handle, self.ins[a][lo:lo + m])
        self.ins_pos[a] = lo + m

    def step(self):
        B, cfg, i, torch = self.B, self.cfg, self.step_no, self.torch
        q = self.q[i % self.N_QUERY_BATCHES]
        if cfg.index == 5:  # skewed dynamic: 1:1 interleave, the insert comes first
            self._insert(0, 1)
        if len(self.indexes) == 1:
            B.pk_search(self.handle, q, cfg.k, cfg.nprobe, self.out_ids, self.out_dist)
        else:
            B.pk_search_multi([ix.handle for ix in self.indexes], self.q_offsets, q, cfg.k, cfg.nprobe,
                              self.out_ids, self.out_dist)
        if cfg.index == 3:  # the agents' insert batches of this round, one call
            sizes = [int(self.ins_sizes[a][i]) for a in range(len(self.indexes))]
            rows = torch.cat([self.ins[a][self.ins_pos[a]:self.ins_pos[a] + m] for a, m in enumerate(sizes)])
            B.pk_insert_multi([ix.handle for ix in self.indexes], np.concatenate([[0], np.cumsum(sizes)]), rows)
            for a, m in enumerate(sizes):
                self.ins_pos[a] += m
        elif cfg.index != 5 and self.insert_m:
            self._insert(0, self.insert_m)
        self.step_no += 1

    def reserve(self, steps):
        """One workspace reservation for everything the run will call (Section 5: no operation blocks the caller)."""
        cfg = self.cfg
        ahead = max(self.insert_m, 16) * steps + 1024
        nq = max(self.queries_per_step(), 64)
        self.B.pk_workspace_reserve([ix.handle for ix in self.indexes], nq, max(cfg.k, 10), cfg.nprobe, ahead)
        self.reserved = {"nq_max": nq, "k_max": max(cfg.k, 10), "nprobe_max": cfg.nprobe, "inserts_ahead": ahead}

    def queries_per_step(self):
        return self.cfg.nq * len(self.indexes)

    def row_bytes(self):
        return self.cfg.d * (2 if self.cfg.storage == self.B.PK_F16 else 4)

    def n_total(self):
        return int(sum(ix.stats().n_total for ix in self.indexes))

    def check_errors(self):
        for ix in self.indexes:
            st = ix.stats()
            if st.device_error:
                raise SystemExit(f"device error flag {st.device_error}")

    def recall(self, nsample):
        """recall@10 of the GPU search against the oracle's exact search on a few queries of agent 0
        (base rows only: called before the timed steps insert anything)."""
        import oracle
        nq0 = self.cfg.nq  # agent 0's queries lead every batch
        q = np.concatenate([b[:nq0] for b in self.q_host])[:nsample]
        ids, _ = self.indexes[0].search(self.torch.from_numpy(q).cuda(), max(10, self.cfg.k), self.cfg.nprobe)
        bi, _ = oracle.bruteforce(self.datas[0].x, q, 10, self.cfg.metric)
        got = ids.cpu().numpy()
        return float(np.mean([len(set(a[:10].tolist()) & set(b.tolist())) / 10.0 for a, b in zip(got, bi)]))

    def cpu_baseline(self, budget_s=12.0):
        """The oracle as it stands, on a bounded sample: an index over the first n/f rows of agent 0 with
        nlist/f lists (same list length, same nprobe and k, so the same number of vectors scanned per
        query as in the full workload)."""
        import oracle
        cfg, W, dat = self.cfg, self.W, self.datas[0]
        f = 1
        while dat.n // f * (cfg.nlist // f) * cfg.d > 2.5e10 and cfg.nlist // (f * 2) >= cfg.nprobe:
            f *= 2
        n_s, nlist_s = dat.n // f, cfg.nlist // f
        xs = dat.x[:n_s]
        if f == 1:
            cent = dat.cent
        elif cfg.train == "component_means":
            cent = dat.cent[:nlist_s]
        else:
            sub = W.scaled(cfg, nlist=nlist_s)
            rows = W.train_rows(sub, n_s)
            cent = training.lloyd(xs[rows], W.init_rows(sub, len(rows)), 4)
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
                "omp_max_threads": oracle.num_threads(), "affinity_cpus": len(os.sched_getaffinity(0)),
                "os_cpu_count": os.cpu_count(),
                "sample": f"{done} queries (nprobe={cfg.nprobe}, k={cfg.k}) on an oracle index over the first "
                          f"{n_s} rows with {nlist_s} lists (1/{f} of the workload, same list length, so the same "
                          f"vectors scanned per query; <= {scanned:.0f} per query); oracle build {build_s:.1f}s not "
                          f"included"}

    def stream(self, rounds, window):
        """Config 5 as the paper's One-Search-One-Insert pattern (Section 6.1): `rounds` rounds of {insert one
        vector; search one batch}, every insert a call of its own, so that the lists' delta-page tables
        grow one vector at a time over the whole stream.  Timed: three windows of `window` rounds at the
        start, the middle and the end, every round of a window with its search; between the windows every
        insert still happens and every 64th round searches (what is skipped there is only the waiting for
        searches nobody times).  After each window 64 more rounds run with the library's stage events on."""
        torch, B, W, cfg = self.torch, self.B, self.W, self.cfg
        ix = self.indexes[0]
        t0 = time.time()
        nb = (rounds + 255) // 256
        rows = np.concatenate([W.inserts(cfg, 1000 + b, 256) for b in range(nb)])[:rounds]
        dev_rows = torch.from_numpy(rows).cuda()
        log(f"{rounds} insert vectors generated in {time.time() - t0:.1f}s")
        B.pk_workspace_reserve([ix.handle], max(cfg.nq, 64), max(cfg.k, 10), cfg.nprobe, rounds + 1024)
        grows0 = ix.stats().workspace_grows
        starts = sorted({0, max(0, rounds // 2 - window // 2), max(0, rounds - window - 64)})
        windows, r, nsearch = [], 0, 0

        last_say = [time.time()]

        def one_round(search):
            nonlocal r, nsearch
            if time.time() - last_say[0] > 20:
                log(f"stream: round {r} of {rounds}")
                last_say[0] = time.time()
            B.pk_insert(ix.handle, dev_rows[r:r + 1])
            if search:
                B.pk_search(ix.handle, self.q[r % self.N_QUERY_BATCHES], cfg.k, cfg.nprobe, self.out_ids, self.out_dist)
                nsearch += 1
            r += 1

        for w0 in starts:
            while r < w0:
                one_round(r % 64 == 0)
            n = min(window, rounds - r)
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ev[0].record()
            for i in range(n):
                one_round(True)
                ev[i + 1].record()
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            per = [ev[i].elapsed_time(ev[i + 1]) for i in range(n)]
            B.pk_profile_begin(ix.handle)
            for _ in range(min(64, rounds - r)):
                one_round(True)
            pr = B.pk_profile_end(ix.handle)
            m = max(pr.launches, 1)
            scan_ms = pr.scan_ms / m
            alg = pr.scanned_rows / m * self.row_bytes()
            st = ix.stats()
            windows.append({"first_round": w0, "rounds": n, "ms_per_round": dt / n * 1e3, "round_ms": percentiles(per),
                            "queries_per_s": cfg.nq * n / dt, "inserted_so_far": int(st.n_inserted),
                            "pages_used": int(st.pages_used), "max_list_len": int(st.max_list_len),
                            "scan_ms": scan_ms, "scan_GBps": alg / (scan_ms * 1e-3) / 1e9 if scan_ms > 0 else 0.0,
                            "scan_frac_of_peak": alg / (scan_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if scan_ms > 0 else 0.0,
                            "algorithmic_bytes_per_search": alg,
                            "stages_ms": {"coarse": pr.coarse_ms / m, "sample_and_worklist": pr.worklist_ms / m,
                                          "scan": scan_ms, "select": pr.select_ms / m}})
            log(f"window at round {w0}: {windows[-1]['ms_per_round']:.3f} ms/round, scan {scan_ms:.3f} ms = "
                f"{windows[-1]['scan_GBps']:.0f} GB/s, {st.n_inserted} inserted, {st.pages_used} pages")
        while r < rounds:
            one_round(r % 64 == 0)
        torch.cuda.synchronize()
        self.check_errors()
        st = ix.stats()
        return {"rounds": rounds, "single_vector_insert_calls": rounds, "searches": nsearch, "windows": windows,
                "inserted": int(st.n_inserted), "workspace_bytes": int(st.workspace_bytes),
                "workspace_grows_after_the_reservation": int(st.workspace_grows - grows0)}

    def maintenance(self, extra_inserts, steps=20):
        """Grow agent 0's lists by `extra_inserts` vectors (batches of 1024: delta pages open all over the
        arena), then fold everything into contiguous extents in a fresh arena (pk_index_compact) and report
        what the copy cost and what a search step costs before and after."""
        torch, B, W, cfg = self.torch, self.B, self.W, self.cfg
        ix = self.indexes[0]
        done = 0
        ins_s, ins_n = 0.0, 0
        while done < extra_inserts:
            m = min(1024, extra_inserts - done)
            rows = np.concatenate([W.inserts(cfg, 100000 + (done + j) // 256, 256) for j in range(0, m, 256)])[:m]
            dev_rows = torch.from_numpy(rows).cuda()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            try:
                ix.insert(dev_rows)
            except B.PancakeError as e:
                if e.status != B.PK_ERR_NOMEM:
                    raise
                ix.add_arena(B.pk_arena_bytes(ix.cfg, 0, max(extra_inserts - done, 1024)))
                continue
            torch.cuda.synchronize()
            if m == 1024 and done > 0:  # the first batch warms the path up
                ins_s += time.perf_counter() - t0
                ins_n += m
            done += m
        # single-vector inserts, back to back on the stream (rows already resident)
        singles = torch.from_numpy(W.inserts(cfg, 200000, 256)).cuda()
        single_us = None
        for attempt in range(2):
            try:
                ix.insert(singles[:1])
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for j in range(1, 201):
                    ix.insert(singles[j:j + 1])
                torch.cuda.synchronize()
                single_us = (time.perf_counter() - t0) / 200 * 1e6
                break
            except B.PancakeError as e:
                if e.status != B.PK_ERR_NOMEM or attempt:
                    raise
                ix.add_arena(B.pk_arena_bytes(ix.cfg, 0, 1024))

        def ms_per_step():
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                self.step()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / steps * 1e3

        # deletes: 4096 ids drawn over the whole id range (build rows carry ids 0 .. n-1)
        gone = torch.from_numpy(np.random.default_rng(7).choice(self.datas[0].n, 4096, replace=False)).cuda()
        ix.delete(gone[:8])  # warm-up
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        n_del = ix.delete(gone[8:])
        del_ms = (time.perf_counter() - t0) * 1e3
        before = ms_per_step()
        st = ix.stats()
        nbytes = B.pk_arena_bytes(ix.cfg, int(st.n_total), self.insert_m * (steps + 8) + 1024)
        new_arena = torch.empty(nbytes, dtype=torch.uint8, device="cuda")  # allocated outside the timed call
        page_bytes = (128 if ix.cfg.page_vecs == 0 else ix.cfg.page_vecs) * (self.row_bytes() + 12)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        B.pk_index_compact(ix.handle, new_arena)
        dt = time.perf_counter() - t0
        ix.arenas = [new_arena]
        after = ms_per_step()
        self.check_errors()
        # IVF-Split: lists over 8 x the mean length are split by a 2-means on the device
        thr = int(8 * st.n_total / cfg.nlist)
        arena2 = torch.empty(nbytes + (64 << 20), dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        n_split = B.pk_index_split(ix.handle, arena2, thr, 4)
        split_ms = (time.perf_counter() - t0) * 1e3
        ix.arenas = [arena2]
        ix.nlist += n_split
        ix.cfg.nlist = ix.nlist
        del new_arena
        after_split = ms_per_step()
        self.check_errors()
        copied = int(st.pages_used) * page_bytes
        return {"extra_inserts": extra_inserts,
                "insert_vectors_per_s_batches_of_1024": (ins_n / ins_s) if ins_s > 0 else None,
                "insert_us_per_single_vector_call": single_us, "deleted": n_del, "delete_ms_per_4088_ids": del_ms,
                "ids_scanned_per_s": float(st.n_total + n_del) / (del_ms * 1e-3), "n_total": int(st.n_total), "arenas_before": int(st.n_arenas),
                "compaction_ms": dt * 1e3, "bytes_copied": copied,
                "copy_GBps_read_plus_write": 2 * copied / dt / 1e9, "ms_per_step_before": before,
                "ms_per_step_after": after, "split_threshold": thr, "lists_split": n_split, "split_ms": split_ms,
                "ms_per_step_after_split": after_split}

    def graph_replay(self, steps=50):
        """The search of a step (no insert: an insert also advances host-side counters) captured into
        a HIP graph and replayed: what the launches themselves cost on small batches."""
        torch, B, cfg = self.torch, self.B, self.cfg
        q = self.q[0]

        def search():
            if len(self.indexes) == 1:
                B.pk_search(self.handle, q, cfg.k, cfg.nprobe, self.out_ids, self.out_dist)
            else:
                B.pk_search_multi([ix.handle for ix in self.indexes], self.q_offsets, q, cfg.k, cfg.nprobe,
                                  self.out_ids, self.out_dist)

        def timed(fn):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / steps * 1e3

        search()
        torch.cuda.synchronize()
        want_ids, want_dist = self.out_ids.clone(), self.out_dist.clone()
        eager = timed(search)
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                search()
        torch.cuda.synchronize()
        self.out_ids.fill_(-7)
        graph.replay()
        torch.cuda.synchronize()
        same = bool(torch.equal(self.out_ids, want_ids) and torch.equal(self.out_dist, want_dist))
        replay = timed(graph.replay)
        self.check_errors()
        return {"eager_ms_per_search": eager, "graph_ms_per_search": replay, "replay_equals_eager": same,
                "queries_per_s_graph": self.queries_per_step() / (replay * 1e-3)}

    def levels(self, steps=30):
        """Early termination over two levels (pk_search_levels).  The top level is what the paper's L1
        cache holds: the top-k' neighbours (k' = 4k) of the agent's recent queries (query batches 8..15),
        as an IVF index of its own trained by pk_kmeans.  The measured batch is half recent queries
        asked again with a little noise, half fresh ones.  On these synthetic mixtures every query's
        top-k distances are alike, so the paper's alpha_et * d_agent with alpha_et = 0.6..0.8 ends no
        search; the thresholds here are set to end a chosen share of the batch at the top level, which
        shows what the mechanism costs and saves: 0 (none ends), 0.5, 1 (all end)."""
        torch, B, W, cfg, dat = self.torch, self.B, self.W, self.cfg, self.datas[0]
        full = self.indexes[0]
        k, kp = cfg.k, min(4 * cfg.k, 1024)
        recent = np.concatenate(self.q_host[8:16])[:8 * cfg.nq]
        rq = torch.from_numpy(recent).cuda()
        ids, vals = full.search(rq, kp, cfg.nprobe)
        ids = ids.cpu().numpy().ravel()
        top_ids = np.unique(ids[(ids >= 0) & (ids < dat.n)])
        mean_topk = float(vals[:, :k].mean())
        x_top = torch.from_numpy(np.ascontiguousarray(dat.x[top_ids])).cuda()
        nlist_top = int(max(4, min(cfg.nlist, len(top_ids) // 256)))
        rng = np.random.default_rng(11)
        cent = x_top[torch.from_numpy(rng.choice(len(top_ids), nlist_top, replace=False)).cuda()].contiguous()
        B.pk_kmeans(x_top, cent, 5)
        top = B.Index(cent, x_top, metric=cfg.metric, storage=cfg.storage, ids=torch.from_numpy(top_ids).cuda())
        half = cfg.nq // 2
        again = recent[rng.choice(len(recent), half, replace=False)]
        again = again + rng.normal(0.0, 0.01 / np.sqrt(cfg.d), again.shape).astype(np.float32)
        q = torch.from_numpy(np.concatenate([again, self.q_host[0][:cfg.nq - half]]).astype(np.float32)).cuda()
        nprobes = [min(cfg.nprobe, nlist_top), cfg.nprobe]
        level = torch.empty(cfg.nq, dtype=torch.int32, device="cuda")
        oi, od = self.out_ids[:cfg.nq], self.out_dist[:cfg.nq]

        def timed(fn):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / steps * 1e3

        plain = timed(lambda: B.pk_search(full.handle, q, k, cfg.nprobe, oi, od))
        want = oi.clone()
        top_only = timed(lambda: B.pk_search(top.handle, q, k, nprobes[0], oi, od))
        kth = od[:, k - 1].clone()  # the top level's k-th value of every query
        ip = cfg.metric == W.METRIC_IP
        runs = []
        for share in (0.0, 0.5, 1.0):
            if share == 0.0:
                stop = torch.full_like(kth, float("inf") if ip else float("-inf"))
            elif share == 1.0:
                stop = torch.full_like(kth, float("-inf") if ip else float("inf"))
            else:
                stop = torch.full_like(kth, float(torch.quantile(kth, (1.0 - share) if ip else share)))
            ms = timed(lambda: B.pk_search_levels([top.handle, full.handle], nprobes, q, k, stop, level, oi, od))
            ended = level == 0
            same = (oi == want).float().mean(dim=1)
            runs.append({"share_wanted": share, "ended_at_top": float(ended.float().mean()),
                         "ended_at_top_among_repeated": float(ended[:half].float().mean()),
                         "ended_at_top_among_fresh": float(ended[half:].float().mean()),
                         "ms_per_call": ms,
                         "ids_equal_to_full_search_where_ended_at_top":
                             float(same[ended].mean()) if bool(ended.any()) else None})
        out = {"top_level_vectors": int(len(top_ids)), "top_level_lists": nlist_top, "queries": cfg.nq,
               "mean_top_k_value_of_recent_queries": mean_topk, "ms_full_index_search": plain,
               "ms_top_level_search": top_only, "runs": runs}
        self.check_errors()
        top.close()
        return out

    def scope_union(self, steps=30):
        """One agent's query batch searched across the memories of ALL agents of the workload
        (pk_search_union): the same number of (query, index) searches as one multi-agent step."""
        torch, B, cfg = self.torch, self.B, self.cfg
        q = self.q[0][:cfg.nq].contiguous()
        src = torch.empty((cfg.nq, cfg.k), dtype=torch.int32, device="cuda")
        hs = [ix.handle for ix in self.indexes]
        for _ in range(3):
            B.pk_search_union(hs, q, cfg.k, cfg.nprobe, src, self.out_ids[:cfg.nq], self.out_dist[:cfg.nq])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            B.pk_search_union(hs, q, cfg.k, cfg.nprobe, src, self.out_ids[:cfg.nq], self.out_dist[:cfg.nq])
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        return {"handles": len(hs), "queries": cfg.nq, "ms_per_call": dt * 1e3,
                "index_searches_per_s": cfg.nq * len(hs) / dt, "queries_per_s": cfg.nq / dt}

    def training(self, iters):
        """pk_kmeans on the workload's own training sample (the rows and initial centroids its index was
        trained from on the host): time per Lloyd iteration and the rate of the assignment GEMM."""
        torch, B, W, cfg, dat = self.torch, self.B, self.W, self.cfg, self.datas[0]
        rows = W.train_rows(cfg, dat.n)
        xs = torch.from_numpy(np.ascontiguousarray(dat.x[rows])).cuda()
        init = W.init_rows(cfg, len(rows))
        c0 = xs[torch.from_numpy(init).cuda()].contiguous()
        c = c0.clone()
        B.pk_kmeans(xs, c, 1)  # warm-up: workspace, code objects
        c = c0.clone()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        inertia = B.pk_kmeans(xs, c, iters)
        dt = time.perf_counter() - t0
        flops = 2.0 * len(rows) * cfg.nlist * cfg.d
        return {"n": int(len(rows)), "d": cfg.d, "nlist": cfg.nlist, "iters": iters, "ms_per_iter": dt / iters * 1e3,
                "assignment_TFLOPs_incl_update": flops * iters / dt / 1e12,
                "frac_of_fp32_mfma_peak": flops * iters / dt / 1e12 / 157.3,
                "inertia_first": inertia[0], "inertia_last": inertia[-1]}

    def close(self):
        for ix in self.indexes:
            ix.close()
        self.indexes = []
        self.torch.cuda.empty_cache()


def percentiles(ms):
    a = np.sort(np.asarray(ms, dtype=np.float64))
    return {"median": float(np.median(a)), "p10": float(np.percentile(a, 10)), "p90": float(np.percentile(a, 90)),
            "min": float(a[0]), "max": float(a[-1])}


def timed_steps(sc, steps):
    """K steps: wall clock around all of them (the headline rate) and one HIP event pair per step on the
    stream the library enqueues on (torch's current stream), for the spread."""
    import torch
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(steps):
        sc.step()
        ev[i + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    return dt, [ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]


def measure(sc, steps, warmup, recall_queries):
    """Warm-up, K timed steps, the same K steps again with stage events; returns the result dict."""
    import torch
    B = sc.B
    rec = sc.recall(recall_queries) if recall_queries else None
    sc.reserve(warmup + 2 * steps + 8)
    for _ in range(warmup):
        sc.step()
    grows0 = sc.indexes[0].stats().workspace_grows
    dt, per_step = timed_steps(sc, steps)
    qps = sc.queries_per_step() * steps / dt
    # stage timing: HIP events recorded by the library on the search's own stream
    B.pk_profile_begin(sc.handle)
    for _ in range(steps):
        sc.step()
    pr = B.pk_profile_end(sc.handle)
    sc.check_errors()
    st = sc.indexes[0].stats()
    n = max(pr.launches, 1)
    scan_ms = pr.scan_ms / n
    alg_bytes = pr.scanned_rows / n * sc.row_bytes()
    achieved = alg_bytes / (scan_ms * 1e-3) / 1e9 if scan_ms > 0 else 0.0
    res = {
        "qps": qps, "ms_per_step": dt / steps * 1e3, "step_ms": percentiles(per_step), "recall_at_10": rec,
        "recall_queries": recall_queries,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None, "traffic_source": None,
                     "measured_stream": MEASURED_STREAM_GBS, "frac_of_measured_stream": achieved / MEASURED_STREAM_GBS,
                     "measured_stream_source": MEASURED_STREAM_SOURCE,
                     "kernel": "pk::scan_kernel + pk::scan_rr_kernel (gated list scan)",
                     "algorithmic_bytes_per_launch": alg_bytes, "kernel_ms": scan_ms,
                     "kernel_ms_lists_probed_by_many_queries": pr.scan_hot_ms / n},
        "stages_ms": {"coarse": pr.coarse_ms / n, "sample_and_worklist": pr.worklist_ms / n, "scan": scan_ms,
                      "select": pr.select_ms / n},
        "per_search": {"tiles": pr.tiles / n, "candidates": pr.candidates / n, "emitted": pr.emitted / n,
                       "scanned_rows": pr.scanned_rows / n, "max_emitted_by_one_query": pr.max_emitted,
                       "queries_rescored_after_overflow": pr.overflowed},
        "workspace": {"bytes": int(st.workspace_bytes), "grows_during_timed_steps": int(st.workspace_grows - grows0),
                      "reserved_for": sc.reserved},
    }
    log(f"{qps:.0f} queries/s, {res['ms_per_step']:.3f} ms/step (median {res['step_ms']['median']:.3f}, p10 "
        f"{res['step_ms']['p10']:.3f}, p90 {res['step_ms']['p90']:.3f}), scan {scan_ms:.3f} ms = {achieved:.0f} GB/s "
        f"({achieved / HBM_PEAK_GBS:.3f} of peak), recall@10 {rec}, stages {res['stages_ms']}, workspace "
        f"{st.workspace_bytes / 2**20:.1f} MiB")
    return res


def run(args):
    import torch
    from paper_2602_21477_amd import binding as B
    from paper_2602_21477_amd import workload as W

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU (the HIP path has no CPU fallback)")
    torch.cuda.set_device(0)
    B.lib()
    name = args.workload
    base = {"c1": W.C1, "c2": W.C2, "c3": W.C3, "c4": W.C4, "c4l2": W.C4, "c4ip": W.C4, "c5": W.C5}[name]
    metrics = {"c4": [W.METRIC_L2, W.METRIC_IP], "c4l2": [W.METRIC_L2], "c4ip": [W.METRIC_IP]}.get(name, [base.metric])
    steps_total = args.warmup + 2 * args.steps + 8
    if base.n_agents > 1:
        sizes = W.agent_sizes(base)
        datas = [Data(base, int(sizes[a]), a) for a in range(base.n_agents)]
    else:
        datas = [Data(base)]
    xd = datas[0].upload() if len(metrics) > 1 else None  # shared by the variants' builds

    results = {}
    stream = None
    for metric in metrics:
        cfg = W.scaled(base, metric=metric)
        full_stream = name == "c5" and args.c5_rounds > 0
        sc = Scenario(cfg, datas, steps_total, xd=xd,
                      reserve=(args.c5_rounds + steps_total + 4096) if full_stream else None)
        res = measure(sc, args.steps, args.warmup, 0 if args.no_recall else args.recall_queries)
        if full_stream:
            stream = sc.stream(args.c5_rounds, args.c5_window)
        res["n"] = sc.n_total()
        results["ip" if metric == W.METRIC_IP else "l2"] = (res, sc, cfg)
        if metric != metrics[-1]:
            sc.close()
    del xd
    # headline: the slower variant
    head = min(results, key=lambda m: results[m][0]["qps"])
    res, sc, cfg = results[head]
    out = {
        "metric": METRIC_NAME, "value": res["qps"], "unit": "queries/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16" if cfg.storage == B.PK_F16 else "f32", "data": "synthetic",
        "config": {"workload": base.name, "n": res["n"], "d": cfg.d, "nlist": cfg.nlist, "nprobe": cfg.nprobe,
                   "k": cfg.k, "agents": len(datas), "queries_per_step": sc.queries_per_step(),
                   "inserts_per_step": sc.insert_m, "metric": head},
        "step_ms": res["step_ms"], "roofline": res["roofline"], "stages_ms": res["stages_ms"],
        "per_search": res["per_search"], "workspace": res["workspace"], "recall_at_10": res["recall_at_10"],
        "recall_queries": res["recall_queries"], "kernel_sources_sha": kernel_sources_sha(),
    }
    for m, r in results.items():
        r[0]["roofline"]["traffic"], r[0]["roofline"]["traffic_source"] = profiled_traffic(base.name.split("_")[0], m)
    if len(results) > 1:
        out["variants"] = {m: {k: v for k, v in r[0].items()} for m, r in results.items()}
    if stream is not None:
        # the headline of the skewed dynamic config is the 1:1 stream itself: all rounds of the three windows
        ws = stream["windows"]
        tot_rounds = sum(w["rounds"] for w in ws)
        tot_ms = sum(w["rounds"] * w["ms_per_round"] for w in ws)
        out["value"] = cfg.nq * tot_rounds / (tot_ms * 1e-3)
        out["ms_per_step"] = tot_ms / tot_rounds
        out["steps"] = tot_rounds
        last = ws[-1]
        out["roofline"].update({"achieved": last["scan_GBps"], "frac": last["scan_frac_of_peak"],
                                "frac_of_measured_stream": last["scan_GBps"] / MEASURED_STREAM_GBS,
                                "algorithmic_bytes_per_launch": last["algorithmic_bytes_per_search"],
                                "kernel_ms": last["scan_ms"], "window": "last"})
        out["stream"] = stream
        out["short_run_before_the_stream"] = {"qps": res["qps"], "ms_per_step": res["ms_per_step"],
                                              "step_ms": res["step_ms"], "stages_ms": res["stages_ms"]}
    if not args.no_cpu_baseline:
        # the headline scenario is the last one still open only if it ran last; rebuild nothing: the
        # baseline needs host data only
        out["cpu_baseline"] = sc.cpu_baseline()
        log(f"cpu baseline: {out['cpu_baseline']['value']:.1f} queries/s on {out['cpu_baseline']['cores']} threads")
    if args.graph:
        out["hip_graph"] = sc.graph_replay()
        log(f"hip graph: {out['hip_graph']}")
    if args.levels:
        out["levels"] = sc.levels()
        log(f"levels: {out['levels']}")
    if args.union:
        out["scope_union"] = sc.scope_union()
        log(f"scope union: {out['scope_union']}")
    if args.train:
        out["training"] = sc.training(args.train)
        log(f"training: {out['training']}")
    if args.maintenance:
        out["maintenance"] = sc.maintenance(args.maintenance)
        log(f"maintenance: {out['maintenance']}")
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c4", choices=["c1", "c2", "c3", "c4", "c4l2", "c4ip", "c5"])
    ap.add_argument("--recall-queries", type=int, default=64)
    ap.add_argument("--no-recall", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="also capture one search into a HIP graph and time its replays (extra field)")
    ap.add_argument("--levels", action="store_true",
                    help="also time pk_search_levels over a two-level stack (cache of recent neighbours above the "
                         "index) with early termination (extra field)")
    ap.add_argument("--union", action="store_true",
                    help="also time pk_search_union: one agent's batch searched across all agents' memories (extra field)")
    ap.add_argument("--train", type=int, default=0, metavar="ITERS",
                    help="also run ITERS Lloyd iterations of pk_kmeans on the workload's training sample and report "
                         "the time per iteration (extra field)")
    ap.add_argument("--maintenance", type=int, default=0, metavar="N",
                    help="after the timed steps: insert N more vectors, compact the index into a fresh arena "
                         "(pk_index_compact) and report the cost (extra field, the headline is unchanged)")
    ap.add_argument("--c5-rounds", type=int, default=200000,
                    help="workload c5: rounds of the 1:1 insert/search stream (Section 6.1 One-Search-One-Insert); "
                         "0 = only the short run of --steps steps")
    ap.add_argument("--c5-window", type=int, default=2000, help="workload c5: rounds per timed window (start, middle, end)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="counter calibration only: four plain 1 GiB device-to-device copies (a copy kernel of known "
                         "size for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE), then exit")
    args = ap.parse_args()
    if args.calib_copy:
        import torch
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(3)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calib_copy_bytes_each_way": 1 << 30, "copies": 4}))
        return
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); run with --gpus 1.", file=sys.stderr)
        raise SystemExit(2)
    run(args)


if __name__ == "__main__":
    main()
