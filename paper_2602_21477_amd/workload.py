"""Seeded synthetic inputs shaped like the paper's workloads.

This module only *generates inputs* (vectors, queries, insert streams, index
sizes, the seeded choice of training rows).  It holds none of the search / assignment / insert
arithmetic and is the single piece shared by the HIP path's tests, the CPU
oracle's tests and the benchmark, so both sides always see the same bits.

The paper evaluates on E5 embeddings (d = 1024) of 8 M MS MARCO passages and on
agent traces (Section 6.1, "Workloads"); none of that data exists here, so
Gaussian-mixture stand-ins of the same shapes are used: d = 128 .. 1536,
20 k .. 10 M rows, query batches of 16 .. 1024, search/insert interleaved 1:1,
up to 16 agents.

Recipe (everything is drawn in the un-normalised space, where coordinates are
O(1), and normalised afterwards):

    centre   mu_c ~ N(0, I_d)                              c = 0 .. ncomp-1
    vector   x = normalise(mu_c + sigma * g),  g ~ N(0, I), sigma = 0.3
    query    q = normalise(mu_c + sigma * g' + 0.05 * h),  fresh g', h ~ N(0, I)

Random streams are numpy ``Generator(PCG64(SeedSequence([BASE, config, agent,
stream, chunk])))``; data rows come in chunks of 65 536 so that any row range
can be regenerated independently and in parallel.
"""
from __future__ import annotations

import dataclasses
import functools
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

BASE_SEED = 260221477
CHUNK = 65536

S_CENTRES, S_COMPONENT, S_NOISE, S_QUERY, S_INSERT, S_TRAIN, S_SIZES = range(7)

METRIC_IP, METRIC_L2 = 0, 1
STORE_F32, STORE_F16 = 0, 1


@dataclass(frozen=True)
class Config:
    """One workload.  ``index`` is the position in the baseline's config list (1-based)."""
    name: str
    index: int
    n: int
    d: int
    ncomp: int
    nlist: int
    nprobe: int
    k: int
    nq: int
    metric: int = METRIC_IP
    storage: int = STORE_F32
    n_agents: int = 1
    n_lo: int = 0            # multi-agent: per-agent size drawn uniformly in [n_lo, n_hi]
    n_hi: int = 0
    insert_batch: int = 1
    sigma: float = 0.3
    qnoise: float = 0.05
    zipf_s: float = 0.0      # > 0: component weights proportional to rank^-s
    train: str = "lloyd"     # "lloyd" (k-means, 10 iterations) or "component_means"
    train_iters: int = 10
    train_rows_per_list: int = 256


C1 = Config("c1_tiny", 1, n=20_000, d=128, ncomp=64, nlist=64, nprobe=8, k=10, nq=256)
C2 = Config("c2_single_agent", 2, n=1_000_000, d=768, ncomp=1024, nlist=1024, nprobe=32, k=10, nq=64,
            insert_batch=8)
C3 = Config("c3_multi_agent", 3, n=0, d=1024, ncomp=256, nlist=512, nprobe=16, k=20, nq=32,
            n_agents=16, n_lo=100_000, n_hi=500_000, insert_batch=16)
C4 = Config("c4_large_static_f16", 4, n=10_000_000, d=768, ncomp=4096, nlist=4096, nprobe=64, k=100,
            nq=1024, metric=METRIC_L2, storage=STORE_F16, train_rows_per_list=64)
C5 = Config("c5_skewed_dynamic", 5, n=2_000_000, d=1536, ncomp=2048, nlist=2048, nprobe=48, k=10, nq=16,
            zipf_s=1.2, train="component_means")

CONFIGS = {c.name: c for c in (C1, C2, C3, C4, C5)}


def scaled(cfg: Config, **kw) -> Config:
    """A smaller (or otherwise altered) copy of a config; the seeds stay those of ``cfg.index``."""
    return dataclasses.replace(cfg, **kw)


def _rng(cfg: Config, agent: int, stream: int, chunk: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(
        [BASE_SEED, cfg.index, agent, stream, chunk])))


def _normalise(x: np.ndarray) -> np.ndarray:
    nrm = np.sqrt(np.einsum("ij,ij->i", x, x, dtype=np.float64)).astype(np.float32)
    x /= np.maximum(nrm, np.float32(1e-30))[:, None]
    return x


def _to_storage(cfg: Config, x: np.ndarray) -> np.ndarray:
    """fp16-stored configs: round ONCE here (round-to-nearest-even) and hand the
    rounded values, held as fp32, to both the oracle and the GPU build."""
    if cfg.storage == STORE_F16:
        return x.astype(np.float16).astype(np.float32)
    return x


@functools.lru_cache(maxsize=32)
def centres(cfg: Config, agent: int = 0) -> np.ndarray:
    """Mixture centres [ncomp, d]; cached, treat as read-only."""
    return _rng(cfg, agent, S_CENTRES).standard_normal((cfg.ncomp, cfg.d), dtype=np.float32)


def component_weights(cfg: Config) -> np.ndarray:
    if cfg.zipf_s > 0:
        w = np.arange(1, cfg.ncomp + 1, dtype=np.float64) ** (-cfg.zipf_s)
    else:
        w = np.ones(cfg.ncomp, dtype=np.float64)
    return w / w.sum()


def agent_sizes(cfg: Config) -> np.ndarray:
    """Rows per agent.  Single-agent configs: [n]."""
    if cfg.n_agents == 1:
        return np.array([cfg.n], dtype=np.int64)
    return _rng(cfg, 0, S_SIZES).integers(cfg.n_lo, cfg.n_hi + 1, size=cfg.n_agents).astype(np.int64)


def _chunk_rows(cfg: Config, agent: int, mu: np.ndarray, cdf: np.ndarray, chunk: int, lo: int, hi: int):
    """Rows [lo, hi) of chunk ``chunk`` (positions relative to the chunk start)."""
    # the generators fill row-major, so drawing only the first `hi` rows of the
    # chunk gives the same values as drawing the whole chunk
    comp = np.searchsorted(cdf, _rng(cfg, agent, S_COMPONENT, chunk).random(hi), side="right")
    comp = np.minimum(comp, cfg.ncomp - 1).astype(np.int32)
    g = _rng(cfg, agent, S_NOISE, chunk).standard_normal((hi, cfg.d), dtype=np.float32)
    comp, g = comp[lo:hi], g[lo:hi]
    x = mu[comp] + np.float32(cfg.sigma) * g
    return _to_storage(cfg, _normalise(x)), comp


def vectors(cfg: Config, lo: int, hi: int, agent: int = 0, threads: int = 1, out: np.ndarray | None = None,
            with_components: bool = False):
    """Base rows [lo, hi) of one agent's memory, fp32 [hi-lo, d] (fp16-representable
    values when the config stores fp16)."""
    mu = centres(cfg, agent)
    cdf = np.cumsum(component_weights(cfg))
    n = hi - lo
    x = out if out is not None else np.empty((n, cfg.d), dtype=np.float32)
    comp_all = np.empty(n, dtype=np.int32) if with_components else None
    jobs = []
    c0, c1 = lo // CHUNK, (hi - 1) // CHUNK if hi > lo else lo // CHUNK - 1
    for c in range(c0, c1 + 1):
        a, b = max(lo, c * CHUNK), min(hi, (c + 1) * CHUNK)
        jobs.append((c, a, b))

    def run(job):
        c, a, b = job
        rows, comp = _chunk_rows(cfg, agent, mu, cdf, c, a - c * CHUNK, b - c * CHUNK)
        x[a - lo:b - lo] = rows
        if comp_all is not None:
            comp_all[a - lo:b - lo] = comp

    if threads > 1 and len(jobs) > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(run, jobs))
    else:
        for j in jobs:
            run(j)
    return (x, comp_all) if with_components else x


def _mixture_samples(cfg: Config, agent: int, stream: int, batch: int, m: int, comp_weights: np.ndarray,
                     extra_noise: float) -> np.ndarray:
    rng = _rng(cfg, agent, stream, batch)
    mu = centres(cfg, agent)
    comp = rng.choice(cfg.ncomp, size=m, p=comp_weights)
    x = mu[comp] + np.float32(cfg.sigma) * rng.standard_normal((m, cfg.d), dtype=np.float32)
    if extra_noise > 0:
        x = x + np.float32(extra_noise) * rng.standard_normal((m, cfg.d), dtype=np.float32)
    return _normalise(x.astype(np.float32))


def queries(cfg: Config, batch: int = 0, nq: int | None = None, agent: int = 0) -> np.ndarray:
    """Query batch number ``batch``: fresh mixture samples plus N(0, 0.05) noise, normalised."""
    return _mixture_samples(cfg, agent, S_QUERY, batch, cfg.nq if nq is None else nq,
                            component_weights(cfg), cfg.qnoise)


def inserts(cfg: Config, batch: int = 0, m: int | None = None, agent: int = 0) -> np.ndarray:
    """Insert batch number ``batch``: fresh mixture samples.  With Zipf weights the
    component is drawn uniformly from the 5 % largest components."""
    w = component_weights(cfg)
    if cfg.zipf_s > 0:
        top = max(1, int(round(0.05 * cfg.ncomp)))
        w = np.zeros(cfg.ncomp)
        w[:top] = 1.0 / top
    x = _mixture_samples(cfg, agent, S_INSERT, batch, cfg.insert_batch if m is None else m, w, 0.0)
    return _to_storage(cfg, x)


def insert_batch_sizes(cfg: Config, rounds: int, agent: int = 0) -> np.ndarray:
    """Multi-agent config: each agent inserts U{1..insert_batch} vectors per round."""
    return _rng(cfg, agent, S_SIZES, 1).integers(1, cfg.insert_batch + 1, size=rounds)


# --------------------------------------------------------------------------
# Which rows an index is trained on (seeded choices only; the training itself
# is the harness's business, not this module's)
# --------------------------------------------------------------------------

def train_rows(cfg: Config, n: int, agent: int = 0) -> np.ndarray:
    """Rows used for training: all of them, or a seeded subsample of
    ``train_rows_per_list * nlist`` rows when the index is larger than that."""
    want = cfg.train_rows_per_list * cfg.nlist
    if n <= want:
        return np.arange(n, dtype=np.int64)
    return np.sort(_rng(cfg, agent, S_TRAIN, 1).choice(n, size=want, replace=False)).astype(np.int64)


def init_rows(cfg: Config, ntrain: int, agent: int = 0) -> np.ndarray:
    """Initial centroids: the first nlist entries of a seeded permutation of the training rows."""
    return _rng(cfg, agent, S_TRAIN, 0).permutation(ntrain)[:cfg.nlist].astype(np.int64)
