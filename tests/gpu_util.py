"""Shared helpers of the GPU parity tests: one workload -> (HIP index, oracle index)."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from compare import check_probes, check_results
from paper_2602_21477_amd import binding as B
from paper_2602_21477_amd import workload as W
import training

TOL = {B.PK_F32: 1e-4, B.PK_F16: 1e-2}  # spec: relative tolerance for fp32 / fp16-stored vectors
KX = 48  # extra oracle results past k (fp32), so the comparator can look near-tied candidates up
KX_F16 = 1500  # the 1e-2 tolerance of fp16 storage makes near-tie runs that long


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


class Pair:
    """The same index on both sides."""

    def __init__(self, x, cent, metric, storage=B.PK_F32, ids=None, **kw):
        if storage == B.PK_F16:
            x = x.astype(np.float16).astype(np.float32)  # round once; both sides get these bits
        self.x, self.cent, self.metric, self.storage = x, cent, metric, storage
        self.tol = TOL[storage]
        self.kx = KX if storage == B.PK_F32 else KX_F16
        self.orc = oracle.Index(cent, metric)
        self.orc.build(x, ids)
        self.gpu = B.Index(dev(cent), dev(x) if len(x) else None, metric=metric, storage=storage,
                           ids=None if ids is None else dev(ids), **kw)
        self.xmax2 = float((x.astype(np.float64) ** 2).sum(1).max()) if len(x) else 1.0

    def scale(self, q):
        qn2 = (q.astype(np.float64) ** 2).sum(1)
        if self.metric == B.PK_METRIC_IP:
            return np.sqrt(qn2 * self.xmax2)
        return qn2 + self.xmax2

    def note_inserted(self, x):
        self.xmax2 = max(self.xmax2, float((x.astype(np.float64) ** 2).sum(1).max()))

    def check_scan(self, q, k, probes, where=""):
        """Fine search with the probe lists forced to the oracle's."""
        gi, gv = self.gpu.scan_probes(dev(q), k, dev(probes))
        oi, ov = self.orc.scan_probes(q, k + self.kx, probes)
        return check_results(gi.cpu().numpy(), gv.cpu().numpy(), oi, ov, k, self.tol, self.scale(q), self.metric,
                             where=where)

    def check_coarse(self, q, nprobe, where=""):
        gp = self.gpu.coarse(dev(q), nprobe).cpu().numpy()
        op, sc = self.orc.coarse(q, self.orc.nlist, with_scores=True)
        # centroid scores: the tolerance of fp32 storage (the coarse step always runs in fp32)
        cn2 = float((self.cent.astype(np.float64) ** 2).sum(1).max())
        qn2 = (q.astype(np.float64) ** 2).sum(1)
        for i in range(len(q)):
            s = np.sqrt(qn2[i] * cn2) if self.metric == B.PK_METRIC_IP else qn2[i] + cn2
            check_probes(gp[i:i + 1], op[i:i + 1], sc[i:i + 1], nprobe, TOL[B.PK_F32], float(s),
                         where=f"{where} query {i}")
        return gp

    def check_search(self, q, k, nprobe, where=""):
        """End to end.  The GPU's probe lists are validated against the oracle's ranking
        (exact outside near-ties) and then handed to the oracle, so a legitimate flip at
        the nprobe boundary does not masquerade as a scan error."""
        gp = self.check_coarse(q, nprobe, where=where)
        gi, gv = self.gpu.search(dev(q), k, nprobe)
        oi, ov = self.orc.scan_probes(q, k + self.kx, gp)
        check_results(gi.cpu().numpy(), gv.cpu().numpy(), oi, ov, k, self.tol, self.scale(q), self.metric, where=where)
        # how often the unforced oracle agrees outright (reported, near-ties may differ)
        ui, _ = self.orc.search(q, k, nprobe)
        return float(np.mean(ui == gi.cpu().numpy()))

    def insert_both(self, x, ids=None, where=""):
        """Insert on the GPU, compare the chosen lists with the oracle's rule, allow a flip
        only between near-tied centroids, and mirror the GPU's choice into the oracle."""
        if self.storage == B.PK_F16:
            x = x.astype(np.float16).astype(np.float32)
        lists = self.gpu.insert(dev(x), None if ids is None else dev(ids), want_lists=True).cpu().numpy()
        return self.accept_inserted(x, lists, ids, where)

    def accept_inserted(self, x, lists, ids=None, where=""):
        """The GPU put the (already rounded) rows x into `lists`: check them against the oracle's rule
        and mirror them into the oracle."""
        op, sc = self.orc.coarse(x, min(2, self.orc.nlist), with_scores=True)
        cn2 = float((self.cent.astype(np.float64) ** 2).sum(1).max())
        for i in range(len(x)):
            if lists[i] != op[i, 0]:
                xn2 = float((x[i].astype(np.float64) ** 2).sum())
                s = np.sqrt(xn2 * cn2) if self.metric == B.PK_METRIC_IP else xn2 + cn2
                gap = abs(sc[i, lists[i]] - sc[i, op[i, 0]])
                assert gap <= TOL[B.PK_F32] * max(abs(sc[i, op[i, 0]]), s), (
                    f"{where} insert {i}: list {lists[i]} vs oracle {op[i, 0]} with score gap {gap}")
        self.orc.insert(x, ids, forced_lists=lists)
        self.note_inserted(x)
        return lists

    def close(self):
        self.gpu.close()


def make_pair(cfg, n=None, metric=None, storage=None, agent=0, **kw):
    n = cfg.n if n is None else n
    cfg = W.scaled(cfg, n=n)
    if cfg.train == "component_means":
        x, comp = W.vectors(cfg, 0, n, agent=agent, with_components=True)
        cent = training.train_centroids(cfg, x, agent=agent, comp=comp)
    else:
        x = W.vectors(cfg, 0, n, agent=agent)
        cent = training.train_centroids(cfg, x, agent=agent)
    metric = cfg.metric if metric is None else metric
    storage = cfg.storage if storage is None else storage
    return Pair(x, cent, metric, storage, **kw), cfg
