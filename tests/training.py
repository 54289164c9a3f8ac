"""Index training for the tests and the benchmark: produces the centroid table that is an
INPUT to both the HIP path and the CPU oracle.

Harness code: the product package holds no k-means on the host, and the oracle's plain
``orc_kmeans`` would take hours on the large configs.  ``lloyd`` is the same algorithm with
BLAS-backed distance blocks; tests/test_oracle_pins.py checks it against ``orc_kmeans`` on the
tiny config.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor

import numpy as np

from paper_2602_21477_amd.workload import Config, init_rows, train_rows


def lloyd(x: np.ndarray, init: np.ndarray, iters: int, block: int = 16384, threads: int = 8) -> np.ndarray:
    """Lloyd's k-means under L2 with BLAS-backed distance blocks: assign each row to
    its nearest centroid (ties to the lower index), move each non-empty centroid to
    the mean of its members, keep empty ones.  Same algorithm as the oracle's plain
    ``orc_kmeans``; used where that one would take hours."""
    from scipy import sparse
    c = x[init].astype(np.float64)
    n, d = x.shape
    nlist = c.shape[0]
    for _ in range(iters):
        c32 = c.astype(np.float32)
        cn = np.einsum("ij,ij->i", c32, c32)
        def part(s, c32=c32, cn=cn):
            xb = x[s:s + block]
            a = np.argmin(cn[None, :] - 2.0 * (xb @ c32.T), axis=1)
            m = len(a)
            onehot = sparse.csr_matrix((np.ones(m), (a, np.arange(m))), shape=(nlist, m))
            return onehot @ xb.astype(np.float64), np.bincount(a, minlength=nlist)

        sums = np.zeros((nlist, d), dtype=np.float64)
        cnt = np.zeros(nlist, dtype=np.int64)
        with ThreadPoolExecutor(max_workers=threads) as ex:
            for ps, pc in ex.map(part, range(0, n, block)):  # summed in block order: deterministic
                sums += ps
                cnt += pc
        nz = cnt > 0
        c[nz] = sums[nz] / cnt[nz][:, None]
    return c.astype(np.float32)


def component_means(x: np.ndarray, comp: np.ndarray, ncomp: int) -> np.ndarray:
    """Per-component sample means (the skewed config: keeps list sizes Zipf-like,
    which k-means would equalise).  Components without a sample get a zero row."""
    order = np.argsort(comp, kind="stable")
    cnt = np.bincount(comp, minlength=ncomp)
    starts = np.concatenate(([0], np.cumsum(cnt)[:-1]))
    nz = cnt > 0
    out = np.zeros((ncomp, x.shape[1]), dtype=np.float64)
    out[nz] = np.add.reduceat(x[order].astype(np.float64), starts[nz], axis=0) / cnt[nz][:, None]
    return out.astype(np.float32)


def train_centroids(cfg: Config, x: np.ndarray, agent: int = 0, comp: np.ndarray | None = None) -> np.ndarray:
    """Centroid table [nlist, d] fp32 for one agent's rows ``x``."""
    if cfg.train == "component_means":
        assert comp is not None and cfg.nlist == cfg.ncomp
        return component_means(x, comp, cfg.ncomp)
    rows = train_rows(cfg, x.shape[0], agent)
    xt = x if rows.shape[0] == x.shape[0] else x[rows]
    return lloyd(xt, init_rows(cfg, xt.shape[0], agent), cfg.train_iters)
