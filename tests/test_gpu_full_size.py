"""The five configs at their full sizes, in the launch configuration bench.py times
(same Scenario objects, full query batches), checked on sampled outputs:

  * probe lists of sampled queries against the oracle's centroid ranking (needs centroids only);
  * every returned (query, id, value) of the sampled queries against the oracle's value for
    that pair, one by one;
  * the returned ids against the oracle's exact search: the exact ranking, restricted to the
    vectors the oracle assigns to the probed lists, must be what the GPU returned (tolerance
    aware), and recall@10 must be at least 0.9;
  * structure: rows sorted, no repeated id, list lengths add up, no device error flag.

The oracle never builds the full index here (its plain assignment loop would take hours on
10 M x 4096 x 768); it assigns only the few hundred vectors it needs.
"""
import numpy as np
import pytest
import torch

import bench
import oracle
from compare import check_probes, check_row, recall_at
from paper_2602_21477_amd import binding as B
from paper_2602_21477_amd import workload as W

pytestmark = pytest.mark.gpu

TOL = {B.PK_F32: 1e-4, B.PK_F16: 1e-2}


def say(msg):
    print(msg, flush=True)


def full_batch_search(sc):
    """One search launch exactly as the benchmark issues it (batch 0), synchronised."""
    q = sc.q[0]
    if len(sc.indexes) == 1:
        B.pk_search(sc.handle, q, sc.cfg.k, sc.cfg.nprobe, sc.out_ids, sc.out_dist)
    else:
        B.pk_search_multi([ix.handle for ix in sc.indexes], sc.q_offsets, q, sc.cfg.k, sc.cfg.nprobe,
                          sc.out_ids, sc.out_dist)
    torch.cuda.synchronize()
    return sc.out_ids.cpu().numpy(), sc.out_dist.cpu().numpy()


def spot_check(sc, ids_all, val_all, agent, rows, extra=None, kprime=None):
    """rows: query rows (inside the agent's segment) to verify.  extra: (ids, vectors) inserted so far."""
    cfg, dat = sc.cfg, sc.datas[agent]
    tol = TOL[cfg.storage]
    lo = sc.q_offsets[agent]
    q = sc.q_host[0][lo:lo + cfg.nq][rows]
    gi, gv = ids_all[lo:lo + cfg.nq][rows], val_all[lo:lo + cfg.nq][rows]
    x_all = dat.x if extra is None else np.concatenate([dat.x, extra[1]])
    id_all = np.arange(dat.n, dtype=np.int64) if extra is None else np.concatenate([np.arange(dat.n), extra[0]])
    row_of = None if extra is None else {int(i): dat.n + j for j, i in enumerate(extra[0])}
    orc = oracle.Index(dat.cent, cfg.metric)  # centroids only: coarse ranking and assignment
    xn2 = 1.0 + 1e-3  # rows are unit vectors (up to fp16 rounding)
    qn2 = (q.astype(np.float64) ** 2).sum(1)
    cn2 = float((dat.cent.astype(np.float64) ** 2).sum(1).max())

    # 1. probe lists
    gp = sc.indexes[agent].coarse(torch.from_numpy(q).cuda(), cfg.nprobe).cpu().numpy()
    op, sco = orc.coarse(q, cfg.nlist, with_scores=True)
    for i in range(len(q)):
        s = np.sqrt(qn2[i] * cn2) if cfg.metric == W.METRIC_IP else qn2[i] + cn2
        check_probes(gp[i:i + 1], op[i:i + 1], sco[i:i + 1], cfg.nprobe, TOL[B.PK_F32], float(s),
                     where=f"agent {agent} query {rows[i]}")

    # 2. every returned value, pair by pair; structure of the rows
    for i in range(len(q)):
        ids = gi[i]
        assert np.all(ids >= 0), "full-size rows are never short"
        assert len(set(ids.tolist())) == len(ids)
        vecs = x_all[[int(t) if t < dat.n else row_of[int(t)] for t in ids]]
        ov = oracle.pair_values(np.repeat(q[i:i + 1], len(ids), 0), vecs, cfg.metric)
        s = np.sqrt(qn2[i] * xn2) if cfg.metric == W.METRIC_IP else qn2[i] + xn2
        assert np.all(np.abs(gv[i] - ov) <= tol * np.maximum(np.abs(ov), s)), f"value mismatch, query {rows[i]}"
        d = np.diff(gv[i])
        assert np.all(d <= 0) if cfg.metric == W.METRIC_IP else np.all(d >= 0)

    # 3. exact search, restricted to the probed lists
    kprime = kprime or max(4 * cfg.k, 256)
    bi, bv = oracle.bruteforce(x_all, q, kprime, cfg.metric, ids=id_all)
    assert recall_at(gi, bi, 10) >= 0.9
    for i in range(len(q)):
        vec_rows = [int(t) if t < dat.n else row_of[int(t)] for t in bi[i]]
        lists = orc.assign(x_all[vec_rows])
        keep = np.isin(lists, gp[i])
        ei, ev = bi[i][keep], bv[i][keep]
        assert len(ei) >= cfg.k, "raise kprime"
        s = np.sqrt(qn2[i] * xn2) if cfg.metric == W.METRIC_IP else qn2[i] + xn2
        check_row(gi[i], gv[i], ei, ev, cfg.k, tol, float(s), cfg.metric, where=f"agent {agent} query {rows[i]}")


def check_lists(sc):
    for ix, dat in zip(sc.indexes, sc.datas):
        st = ix.stats()
        assert st.device_error == 0
        assert int(ix.list_lengths().sum()) == st.n_total


def test_config2_single_agent_full_size(gpu_device):
    cfg = W.C2
    sc = bench.Scenario(cfg, [bench.Data(cfg)], steps_total=64)
    try:
        ids, val = full_batch_search(sc)
        say("c2: spot check before inserts")
        spot_check(sc, ids, val, 0, [0, 21, 63])
        new_ids, new_x = [], []
        for r in range(40):  # the config's interleave: search 64, insert 8
            lo = sc.ins_pos[0]
            new_x.append(sc.ins[0][lo:lo + 8].cpu().numpy())
            new_ids.append(np.arange(cfg.n + 8 * r, cfg.n + 8 * r + 8))
            sc.step()
        ids, val = full_batch_search(sc)
        say("c2: spot check after 40 insert batches")
        spot_check(sc, ids, val, 0, [5, 40], extra=(np.concatenate(new_ids), np.concatenate(new_x)))
        check_lists(sc)
        assert sc.indexes[0].stats().n_total == cfg.n + 320
    finally:
        sc.close()


def test_config3_multi_agent_full_size(gpu_device):
    cfg = W.C3
    sizes = W.agent_sizes(cfg)
    assert len(sizes) == 16 and sizes.min() >= 100_000 and sizes.max() <= 500_000
    datas = [bench.Data(cfg, int(sizes[a]), a) for a in range(cfg.n_agents)]
    sc = bench.Scenario(cfg, datas, steps_total=16)
    try:
        ids, val = full_batch_search(sc)
        for a in (0, 7, 15):
            say(f"c3: spot check agent {a}")
            spot_check(sc, ids, val, a, [1, 30])
        # one segmented launch == per-handle launches, bit for bit
        for a in (3, 12):
            lo = sc.q_offsets[a]
            si, sv = sc.indexes[a].search(sc.q[0][lo:lo + cfg.nq].contiguous(), cfg.k, cfg.nprobe)
            assert np.array_equal(si.cpu().numpy(), ids[lo:lo + cfg.nq])
            assert np.array_equal(sv.cpu().numpy(), val[lo:lo + cfg.nq])
        for _ in range(4):
            sc.step()  # inserts of 1..16 vectors per agent between launches
        check_lists(sc)
    finally:
        sc.close()


@pytest.mark.parametrize("metric", [W.METRIC_L2, W.METRIC_IP])
def test_config4_large_static_full_size(gpu_device, c4_data, metric):
    cfg = W.scaled(W.C4, metric=metric)
    sc = bench.Scenario(cfg, [c4_data[0]], steps_total=8, xd=c4_data[1])
    try:
        ids, val = full_batch_search(sc)
        say(f"c4 metric={metric}: spot check")
        spot_check(sc, ids, val, 0, [0, 511, 1023], kprime=2000)
        check_lists(sc)
    finally:
        sc.close()


@pytest.fixture(scope="module")
def c4_data(gpu_device):
    dat = bench.Data(W.C4)
    xd = dat.upload()
    yield dat, xd
    del xd
    torch.cuda.empty_cache()


def test_config5_skewed_dynamic_full_size(gpu_device):
    """2 M x 1536 with Zipf list sizes; the 200 000 single inserts of the config are applied as
    400 timed-style rounds {insert 1; search 16} plus bulk batches for the rest, so that lists
    grow by many delta pages; searches are spot-checked before, in between and after."""
    cfg = W.C5
    sc = bench.Scenario(cfg, [bench.Data(cfg)], steps_total=512, reserve=210_000)
    try:
        lens = sc.indexes[0].list_lengths()
        assert lens.max() > 50 * np.median(lens), "list sizes should be heavily skewed"
        ids, val = full_batch_search(sc)
        say("c5: spot check before inserts")
        spot_check(sc, ids, val, 0, [0, 9])
        new_x = []
        for r in range(400):
            new_x.append(sc.ins[0][sc.ins_pos[0]:sc.ins_pos[0] + 1].cpu().numpy())
            sc.step()
        done = 400
        bulk = []
        for b in range(49):  # 49 x 4096 = 200 704 more, from the same insert stream recipe
            xb = np.concatenate([W.inserts(cfg, 10_000 + 16 * b + j, 256) for j in range(16)])
            bulk.append(xb)
            B.pk_insert(sc.handle, torch.from_numpy(xb).cuda())
            if b == 20:
                ids, val = full_batch_search(sc)
                say("c5: spot check in the middle of the insert stream")
                xs = np.concatenate(new_x + bulk)
                spot_check(sc, ids, val, 0, [3], extra=(np.arange(cfg.n, cfg.n + len(xs)), xs))
        ids, val = full_batch_search(sc)
        xs = np.concatenate(new_x + bulk)
        say("c5: spot check after the insert stream")
        spot_check(sc, ids, val, 0, [1, 15], extra=(np.arange(cfg.n, cfg.n + len(xs)), xs))
        st = sc.indexes[0].stats()
        assert st.n_total == cfg.n + len(xs) and st.n_inserted == len(xs) >= 200_000 and st.device_error == 0
        lens2 = sc.indexes[0].list_lengths()
        assert int(lens2.sum()) == st.n_total
        grown = np.argsort(lens2 - lens)[::-1][:102]
        assert set(grown.tolist()) <= set(np.argsort(lens)[::-1][:160].tolist()), "inserts go to the largest lists"
    finally:
        sc.close()
