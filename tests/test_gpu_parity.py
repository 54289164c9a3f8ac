"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element.

Sizes are chosen so the oracle finishes in seconds while the scan still crosses several
pages per list, several query groups and ragged tails.  Bar: ids exact outside near-ties,
values within 1e-4 relative (fp32 storage) / 1e-2 (fp16 storage); see tests/compare.py.
"""
import numpy as np
import pytest
import torch

import oracle
from compare import check_results, recall_at
from gpu_util import KX, Pair, dev, make_pair
from paper_2602_21477_amd import binding as B
from paper_2602_21477_amd import workload as W
import training

pytestmark = pytest.mark.gpu

IP, L2 = B.PK_METRIC_IP, B.PK_METRIC_L2
F32, F16 = B.PK_F32, B.PK_F16


def say(msg):
    print(msg, flush=True)


@pytest.fixture(scope="module")
def tiny(gpu_device):
    """Config 1: 20 000 x 128, 64 lists from 10 Lloyd iterations; built once per variant."""
    cache = {}

    def get(metric, storage):
        key = (metric, storage)
        if key not in cache:
            say(f"build tiny index metric={metric} storage={storage}")
            cache[key] = make_pair(W.C1, metric=metric, storage=storage)[0]
        return cache[key]

    yield get
    for p in cache.values():
        p.close()


@pytest.mark.parametrize("storage", [F32, F16])
@pytest.mark.parametrize("metric", [IP, L2])
def test_build_lists_match_oracle(tiny, metric, storage):
    p = tiny(metric, storage)
    glen = p.gpu.list_lengths()
    olen = p.orc.list_lengths()
    st = p.gpu.stats()
    assert st.n_total == 20000 and st.device_error == 0
    assert glen.sum() == 20000
    # assignment flips need a centroid near-tie; on this mixture none is expected
    assert np.array_equal(glen, olen)


@pytest.mark.parametrize("storage", [F32, F16])
@pytest.mark.parametrize("metric", [IP, L2])
def test_scan_with_oracle_probes(tiny, metric, storage):
    p = tiny(metric, storage)
    q = W.queries(W.C1, 0)
    probes = p.orc.coarse(q, 8)
    say(f"scan parity metric={metric} storage={storage} nq={len(q)}")
    exact = p.check_scan(q, 10, probes)
    assert exact >= 0.5 * q.shape[0] * 10  # positions that are not part of any near-tie group


@pytest.mark.parametrize("metric", [IP, L2])
def test_coarse_probe_lists(tiny, metric):
    p = tiny(metric, F32)
    q = W.queries(W.C1, 1)
    for nprobe in (1, 8, 64):
        say(f"coarse parity metric={metric} nprobe={nprobe}")
        p.check_coarse(q, nprobe)


@pytest.mark.parametrize("storage", [F32, F16])
@pytest.mark.parametrize("metric", [IP, L2])
def test_search_end_to_end_and_recall(tiny, metric, storage):
    p = tiny(metric, storage)
    q = W.queries(W.C1, 2)
    say(f"search parity metric={metric} storage={storage}")
    agree = p.check_search(q, 10, 8)
    assert agree > 0.98
    gi, _ = p.gpu.search(dev(q), 10, 8)
    bi, _ = oracle.bruteforce(p.x, q, 10, metric)
    assert recall_at(gi.cpu().numpy(), bi, 10) >= 0.9


@pytest.mark.parametrize("metric", [IP, L2])
def test_full_probe_equals_exact_search(tiny, metric):
    p = tiny(metric, F32)
    q = W.queries(W.C1, 3, nq=32)
    gi, gv = p.gpu.search(dev(q), 20, 64)
    bi, bv = oracle.bruteforce(p.x, q, 20 + KX, metric)
    check_results(gi.cpu().numpy(), gv.cpu().numpy(), bi, bv, 20, p.tol, p.scale(q), metric, where="nprobe=nlist")


@pytest.mark.parametrize("storage", [F32, F16])
@pytest.mark.parametrize("metric", [IP, L2])
def test_interleaved_inserts_and_searches(gpu_device, metric, storage):
    """Config 1 stream: 32 rounds of {insert one fresh vector; search 8 queries + the vector itself}."""
    p, cfg = make_pair(W.C1, metric=metric, storage=storage, insert_reserve=4096)
    n0 = cfg.n
    try:
        for r in range(32):
            x = W.inserts(cfg, r, 1)
            say(f"insert round {r} metric={metric} storage={storage}")
            p.insert_both(x, where=f"round {r}")
            xs = x.astype(np.float16).astype(np.float32) if storage == F16 else x
            q = np.concatenate([W.queries(cfg, 100 + r, 8), xs])
            p.check_search(q, 10, 8, where=f"round {r}")
            gi, gv = p.gpu.search(dev(xs), 1, 1)
            assert int(gi[0, 0]) == n0 + r  # the vector's list is the rank-1 probe of itself
            v = float(gv[0, 0])
            if metric == L2:
                assert abs(v) <= p.tol * float(p.scale(xs)[0])
            else:
                assert abs(v - float((xs.astype(np.float64) ** 2).sum())) <= p.tol
        st = p.gpu.stats()
        assert st.n_total == n0 + 32 and st.n_inserted == 32 and st.device_error == 0
        assert np.array_equal(p.gpu.list_lengths(), p.orc.list_lengths())
    finally:
        p.close()


def test_batch_inserts_grow_delta_pages_and_match_rebuild(gpu_device):
    """Small pages so lists open many delta pages; build(n) + inserts == build(n + m) (same results)."""
    cfg = W.scaled(W.C1, n=6000)
    x = W.vectors(cfg, 0, cfg.n)
    cent = training.train_centroids(cfg, x)
    extra = np.concatenate([W.inserts(cfg, b, 37) for b in range(40)])  # 1480 vectors
    a = Pair(x, cent, IP, F32, page_vecs=32, insert_reserve=4000)
    b = Pair(np.concatenate([x, extra]), cent, IP, F32, page_vecs=32)
    try:
        for s in range(0, len(extra), 37):
            a.insert_both(extra[s:s + 37], where=f"batch {s // 37}")
        q = W.queries(cfg, 7, 64)
        ai, av = a.gpu.search(dev(q), 10, 8)
        bi, bv = b.gpu.search(dev(q), 10, 8)
        assert torch.equal(ai, bi) and torch.equal(av, bv)
        a.check_search(q, 10, 8, where="after inserts")
        st = a.gpu.stats()
        lens = a.gpu.list_lengths()
        assert st.device_error == 0 and np.array_equal(lens, b.gpu.list_lengths())
        assert st.pages_used == int(np.sum((lens + 31) // 32))
    finally:
        a.close()
        b.close()


@pytest.mark.parametrize("storage,metric", [(F32, IP), (F16, L2)])
def test_compaction_keeps_results_and_inserts_go_on(gpu_device, storage, metric):
    """Delta pages folded into contiguous extents in a new arena: identical search output before
    and after (positions inside a list do not move), oracle parity, then more inserts and another
    compaction into a third arena."""
    cfg = W.scaled(W.C1, n=5000)
    x = W.vectors(cfg, 0, cfg.n)
    cent = training.train_centroids(cfg, x)
    extra = np.concatenate([W.inserts(cfg, b, 61) for b in range(30)])  # 1830 vectors
    p = Pair(x, cent, metric, storage, page_vecs=32, insert_reserve=3000)
    try:
        for s in range(0, 20 * 61, 61):
            p.insert_both(extra[s:s + 61], where=f"batch {s // 61}")
        q = W.queries(cfg, 9, 96)
        i0, v0 = p.gpu.search(dev(q), 10, 8)
        before = p.gpu.stats()
        lens = p.gpu.list_lengths()
        assert before.pages_used == int(np.sum((lens + 31) // 32))
        nbytes = B.pk_arena_bytes(p.gpu.cfg, int(before.n_total), 2000)
        p.gpu.compact(nbytes)
        after = p.gpu.stats()
        assert after.n_arenas == 1 and after.n_total == before.n_total and after.n_inserted == before.n_inserted
        assert after.pages_used == before.pages_used and after.device_error == 0 and after.arena_bytes == nbytes
        assert np.array_equal(p.gpu.list_lengths(), lens)
        i1, v1 = p.gpu.search(dev(q), 10, 8)
        assert torch.equal(i0, i1) and torch.equal(v0, v1)
        p.check_search(q, 10, 8, where="after compaction")
        for s in range(20 * 61, 30 * 61, 61):
            p.insert_both(extra[s:s + 61], where=f"batch {s // 61} after compaction")
        p.check_search(q, 10, 8, where="inserts after compaction")
        assert np.array_equal(p.gpu.list_lengths(), p.orc.list_lengths())
        i2, v2 = p.gpu.search(dev(q), 10, 8)
        p.gpu.compact(B.pk_arena_bytes(p.gpu.cfg, int(p.gpu.stats().n_total), 0))
        i3, v3 = p.gpu.search(dev(q), 10, 8)
        assert torch.equal(i2, i3) and torch.equal(v2, v3)
        # too small an arena: refused, index untouched
        small = torch.empty(1 << 16, dtype=torch.uint8, device="cuda")
        with pytest.raises(B.PancakeError) as e:
            B.pk_index_compact(p.gpu.handle, small)
        assert e.value.status == B.PK_ERR_NOMEM
        i4, _ = p.gpu.search(dev(q), 10, 8)
        assert torch.equal(i3, i4)
    finally:
        p.close()


def _sq_dists(x, c):
    x64, c64 = x.astype(np.float64), c.astype(np.float64)
    return (x64 ** 2).sum(1)[:, None] - 2.0 * x64 @ c64.T + (c64 ** 2).sum(1)[None, :]


def test_kmeans_one_iteration_matches_oracle(gpu_device):
    """Lloyd step by step: the assignment is the oracle's argmin outside near-ties, the new centroids are
    the float64 means of the members the GPU chose, the objective is the float64 sum over that assignment,
    a cluster without members keeps its centroid."""
    cfg = W.scaled(W.C1, n=20000)  # 20000 x 128: two assignment chunks, the second one ragged
    x = W.vectors(cfg, 0, cfg.n)
    rows = W.init_rows(cfg, cfg.n)[:64].copy()
    rows[63] = rows[5]  # a duplicate initial centroid: ties go to the lower number, cluster 63 stays empty
    c0 = x[rows]
    oc, oin, oas = oracle.kmeans(x, 64, 1, rows)
    cg = dev(c0)
    ag = torch.empty(cfg.n, dtype=torch.int32, device="cuda")
    inertia = B.pk_kmeans(dev(x), cg, 1, ag)
    a, c1 = ag.cpu().numpy(), cg.cpu().numpy()
    d0 = _sq_dists(x, c0)
    diff = np.nonzero(a != oas)[0]
    assert len(diff) <= 0.001 * cfg.n
    for i in diff:  # a flip is legitimate only between near-tied centroids
        assert abs(d0[i, a[i]] - d0[i, oas[i]]) <= 1e-4 * (d0[i, oas[i]] + 2.0), (i, a[i], oas[i])
    assert not np.any(a == 63) and np.array_equal(c1[63], c0[63])
    for l in range(64):
        m = x[a == l].astype(np.float64)
        want = m.mean(0) if len(m) else c0[l].astype(np.float64)
        np.testing.assert_allclose(c1[l], want, rtol=2e-6, atol=1e-7, err_msg=f"cluster {l}")
    np.testing.assert_allclose(inertia[0], d0[np.arange(cfg.n), a].sum(), rtol=1e-9)
    if len(diff) == 0:
        np.testing.assert_allclose(c1, oc, rtol=2e-6, atol=1e-7)
        np.testing.assert_allclose(inertia[0], oin[0], rtol=1e-9)


def test_kmeans_training_run_tracks_oracle(gpu_device):
    """Ten iterations: the objective never goes up, ends where the oracle's ends (a flipped near-tie
    moves single points, not the solution), and an index built on the trained centroids searches like
    one built on the oracle's."""
    cfg = W.scaled(W.C1, n=12000)
    x = W.vectors(cfg, 0, cfg.n)
    rows = W.init_rows(cfg, cfg.n)[:64]
    oc, oin, _ = oracle.kmeans(x, 64, 10, rows)
    cg = dev(x[rows])
    inertia = B.pk_kmeans(dev(x), cg, 10)
    assert all(b <= a * (1 + 1e-12) for a, b in zip(inertia, inertia[1:]))
    np.testing.assert_allclose(inertia[0], oin[0], rtol=1e-6)
    np.testing.assert_allclose(inertia[-1], oin[-1], rtol=5e-3)
    c = cg.cpu().numpy()
    close = np.isclose(c, oc, rtol=1e-3, atol=1e-4).all(1)
    assert close.mean() >= 0.8, close.mean()
    p = Pair(x, c, IP, F32)
    try:
        p.check_search(W.queries(cfg, 3, 64), 10, 8, where="index on GPU-trained centroids")
    finally:
        p.close()


def test_ragged_shapes_padding_and_user_ids(gpu_device):
    """d not a multiple of the load width, nlist not a multiple of the coarse tile, empty lists,
    fewer candidates than k, arbitrary int64 ids."""
    rng = np.random.default_rng(5)
    n, d, nlist = 700, 100, 50
    x = rng.standard_normal((n, d)).astype(np.float32)
    cent = np.concatenate([x[rng.permutation(n)[:nlist - 3]], 50 + rng.standard_normal((3, d)).astype(np.float32)])
    ids = (rng.permutation(10 ** 6)[:n] + 2 ** 40).astype(np.int64)
    q = rng.standard_normal((37, d)).astype(np.float32)
    for metric in (L2, IP):
        for storage in (F32, F16):
            say(f"ragged metric={metric} storage={storage}")
            p = Pair(x, cent, metric, storage, ids=ids)
            try:
                if metric == L2:
                    assert (p.gpu.list_lengths()[-3:] == 0).all()  # far-away centroids own nothing
                p.check_search(q, 60, 2)       # most rows shorter than k -> padding
                p.check_search(q, 7, nlist)    # every list probed
                p.check_search(q[:1], 1, 1)
            finally:
                p.close()


def test_duplicates_across_the_k_boundary(gpu_device):
    """Nine exact copies of one vector with scrambled ids, k cuts through them: the lowest ids win."""
    rng = np.random.default_rng(6)
    n, d = 3000, 64
    x = rng.standard_normal((n, d)).astype(np.float32)
    x /= np.linalg.norm(x, axis=1, keepdims=True)
    dup_rows = [11, 500, 501, 777, 1200, 1999, 2500, 2501, 2999]
    x[dup_rows] = x[11]
    ids = rng.permutation(n).astype(np.int64)
    cent = x[rng.permutation(n)[:16]].copy()
    q = np.stack([x[11], x[42]])
    for metric in (IP, L2):
        p = Pair(x, cent, metric, F32, ids=ids)
        try:
            for k in (1, 4, 9, 12):
                p.check_search(q, k, 4, where=f"dup k={k}")
                gi, _ = p.gpu.search(dev(q), k, 4)
                want = sorted(ids[dup_rows].tolist())[:min(k, 9)]
                assert gi[0, :min(k, 9)].cpu().tolist() == want
        finally:
            p.close()


def test_one_id_carried_by_equal_rows_across_the_k_boundary(gpu_device):
    """Several rows may carry one id.  Seven exact copies of one vector carry only three distinct
    ids (5, 5, 5, 9, 9, 30, 30), and k cuts through the runs: every carrier is a candidate of its own,
    so the row is the multiset of the lowest (value, id) pairs, as in the oracle's sort."""
    rng = np.random.default_rng(16)
    n, d = 3000, 64
    x = rng.standard_normal((n, d)).astype(np.float32)
    x /= np.linalg.norm(x, axis=1, keepdims=True)
    dup_rows = [11, 500, 501, 777, 1200, 1999, 2500]
    x[dup_rows] = x[11]
    ids = (np.arange(n) + 1000).astype(np.int64)
    ids[dup_rows] = [5, 9, 5, 30, 5, 9, 30]
    cent = x[rng.permutation(n)[:16]].copy()
    q = np.stack([x[11], x[42]])
    carried = sorted(ids[dup_rows].tolist())
    for metric in (IP, L2):
        p = Pair(x, cent, metric, F32, ids=ids)
        try:
            for k in (1, 2, 3, 4, 5, 6, 7, 10):
                say(f"shared ids metric={metric} k={k}")
                gi, gv = p.gpu.search(dev(q), k, 16)
                gi, gv = gi.cpu().numpy(), gv.cpu().numpy()
                oi, ov = p.orc.search(q, k, 16)
                m = min(k, 7)
                assert gi[0, :m].tolist() == carried[:m], (k, gi[0].tolist())
                assert np.array_equal(gi, oi[:, :k]), (k, gi.tolist(), oi[:, :k].tolist())
                np.testing.assert_allclose(gv, ov[:, :k], rtol=1e-4, atol=1e-5)
        finally:
            p.close()


def test_multi_agent_equals_per_handle_calls(gpu_device):
    """Config 3 shape, scaled: several independent indexes, one segmented call."""
    cfg = W.scaled(W.C3, d=256, ncomp=32, nlist=48, n_agents=5)
    sizes = [2500, 4000, 1500, 3000, 2000]
    pairs, qs, offs = [], [], [0]
    try:
        for a, n in enumerate(sizes):
            p, _ = make_pair(cfg, n=n, agent=a, insert_reserve=256)
            pairs.append(p)
            nq = [32, 5, 0, 17, 32][a]
            qs.append(W.queries(cfg, 0, nq, agent=a) if nq else np.zeros((0, cfg.d), np.float32))
            offs.append(offs[-1] + nq)
        q = np.concatenate(qs)
        say("multi-agent launch")
        mi, mv = B.search_multi([p.gpu for p in pairs], offs, dev(q), 20, 16)
        for a, p in enumerate(pairs):
            if offs[a + 1] == offs[a]:
                continue
            si, sv = p.gpu.search(dev(qs[a]), 20, 16)
            assert torch.equal(mi[offs[a]:offs[a + 1]], si) and torch.equal(mv[offs[a]:offs[a + 1]], sv)
            p.check_search(qs[a], 20, 16, where=f"agent {a}")
        # inserts between launches, then again
        for a, p in enumerate(pairs):
            p.insert_both(W.inserts(cfg, 0, 1 + 3 * a, agent=a))
        mi2, mv2 = B.search_multi([p.gpu for p in pairs], offs, dev(q), 20, 16)
        oi, ov = oracle.search_multi([p.orc for p in pairs], offs, q, 20, 16)
        for a, p in enumerate(pairs):
            if offs[a + 1] == offs[a]:
                continue
            si, sv = p.gpu.search(dev(qs[a]), 20, 16)
            assert torch.equal(mi2[offs[a]:offs[a + 1]], si) and torch.equal(mv2[offs[a]:offs[a + 1]], sv)
        assert np.mean(oi == mi2.cpu().numpy()) > 0.98
    finally:
        for p in pairs:
            p.close()


def test_limits_128_handles_and_k_1024(gpu_device):
    """The documented maxima in one place: 128 handles in one multi-agent search, one multi-agent insert
    and one scope-union search with k = 1024 (more than any single memory holds)."""
    cfg = W.scaled(W.C1, n=300, d=32, ncomp=8, nlist=4)
    pairs = []
    try:
        for a in range(128):
            x = W.vectors(cfg, 0, 150 + a, agent=a)
            pairs.append(Pair(x, x[:4].copy(), L2, F32, insert_reserve=64))
        gpus, orcs = [p.gpu for p in pairs], [p.orc for p in pairs]
        q = W.queries(cfg, 1, 128)  # one query per agent
        offs = list(range(129))
        gi, gv = B.search_multi(gpus, offs, dev(q), 5, 4)
        oi, ov = oracle.search_multi(orcs, offs, q, 5 + KX, 4)
        check_results(gi.cpu().numpy(), gv.cpu().numpy(), oi, ov, 5, 1e-4, np.max([p.scale(q) for p in pairs], axis=0),
                      L2, where="128-handle search")
        sizes = [(a % 3) for a in range(128)]  # 0, 1 or 2 rows per agent
        xs = [W.inserts(cfg, 9, 2, agent=a)[:m] for a, m in enumerate(sizes)]
        out = torch.empty(sum(sizes), dtype=torch.int32, device="cuda")
        voffs = np.concatenate([[0], np.cumsum(sizes)])
        B.pk_insert_multi([g.handle for g in gpus], voffs, dev(np.concatenate(xs)), None, out)
        lists = out.cpu().numpy()
        for a, p in enumerate(pairs):
            if sizes[a]:
                p.accept_inserted(xs[a], lists[voffs[a]:voffs[a + 1]],
                                  150 + a + np.arange(sizes[a], dtype=np.int64), where=f"agent {a}")
        q8 = q[:8]
        gs, gi, gv = B.search_union(gpus, dev(q8), 1024, 4)
        os_, oi, ov = oracle.search_union(orcs, q8, 1024 + KX, 4)
        enc = lambda s_, i_: np.where(i_ < 0, -1, (s_.astype(np.int64) << 40) + i_)
        check_results(enc(gs.cpu().numpy(), gi.cpu().numpy()), gv.cpu().numpy(), enc(os_, oi), ov, 1024, 1e-4,
                      np.max([p.scale(q8) for p in pairs], axis=0), L2, where="128-handle union, k=1024")
        assert int((gi >= 0).sum()) == 8 * 1024  # 128 memories of 150+ rows: every slot is filled
    finally:
        for p in pairs:
            p.close()


@pytest.mark.parametrize("metric", [IP, L2])
def test_scope_union_search(gpu_device, metric):
    """One query batch searched across three memories of different sizes (one shorter than k, one row
    present in two of them): each handle's probe lists are validated against the oracle, then the
    oracle merges its own per-handle scans of those lists; sources and ids must agree."""
    cfg = W.scaled(W.C1, n=4000, nlist=16)
    pairs = []
    try:
        for a, n in enumerate((4000, 37, 2500)):
            x = W.vectors(cfg, 0, n, agent=a)
            if a == 2:
                x[5] = pairs[0].x[9]
            cent = training.train_centroids(W.scaled(cfg, n=n), x, agent=a) if n >= 16 * 4 else x[:16].copy()
            pairs.append(Pair(x, cent, metric, F32))
        q = np.concatenate([W.queries(cfg, 4, 40), pairs[0].x[9:10]])
        k, nprobe = 50, 6
        probes = np.stack([p.check_coarse(q, nprobe, where=f"memory {a}") for a, p in enumerate(pairs)])
        gs, gi, gv = B.search_union([p.gpu for p in pairs], dev(q), k, nprobe)
        os_, oi, ov = oracle.search_union([p.orc for p in pairs], q, k + KX, nprobe, probes=probes)
        enc = lambda s_, i_: np.where(i_ < 0, -1, (s_.astype(np.int64) << 40) + i_)
        scale = np.max([p.scale(q) for p in pairs], axis=0)
        check_results(enc(gs.cpu().numpy(), gi.cpu().numpy()), gv.cpu().numpy(), enc(os_, oi), ov, k, 1e-4, scale,
                      metric, where="union")
        g = gs.cpu().numpy()
        assert set(np.unique(g)) <= {-1, 0, 1, 2} and np.all((g == -1) == (gi.cpu().numpy() == -1))
        # the row stored in memories 0 and 2 is its own best match in both: memory 0 first
        assert (g[-1, 0], int(gi[-1, 0]), g[-1, 1], int(gi[-1, 1])) == (0, 9, 2, 5)
        # a scope of one memory is an ordinary search
        s1, i1, v1 = B.search_union([pairs[1].gpu], dev(q), k, nprobe)
        i2, v2 = pairs[1].gpu.search(dev(q), k, nprobe)
        assert torch.equal(i1, i2) and torch.equal(v1, v2) and bool(torch.all((s1 == 0) == (i1 >= 0)))
    finally:
        for p in pairs:
            p.close()


@pytest.mark.parametrize("storage,metric", [(F32, L2), (F16, IP)])
def test_delete_update_and_page_reuse(gpu_device, storage, metric):
    """Deletes by id (duplicated ids, ids nobody carries, a whole list, rows in delta pages), then
    inserts into the shrunken lists (their pages are reused) and an update (delete + insert under the
    old id); list lengths, counts and every search follow the oracle."""
    cfg = W.scaled(W.C1, n=5000)
    x = W.vectors(cfg, 0, cfg.n)
    cent = training.train_centroids(cfg, x)
    ids = np.arange(cfg.n, dtype=np.int64) * 7 + 3
    ids[1234] = ids[77]  # two rows under one id
    p = Pair(x, cent, metric, storage, ids=ids, page_vecs=32, insert_reserve=3000)
    try:
        extra = np.concatenate([W.inserts(cfg, b, 50) for b in range(12)])
        eids = 10 ** 9 + np.arange(len(extra), dtype=np.int64)
        for s in range(0, 400, 50):
            p.insert_both(extra[s:s + 50], eids[s:s + 50], where=f"batch {s // 50}")
        q = W.queries(cfg, 5, 64)
        rng = np.random.default_rng(5)
        big = int(np.argmax(p.orc.list_lengths()))
        gone = np.concatenate([ids[rng.permutation(cfg.n)[:700]], eids[:400:3], [ids[77], -5, 10 ** 15],
                               p.orc.list_ids(big)])  # the longest list goes entirely
        pages_before = p.gpu.stats().pages_used
        n_o = p.orc.delete(gone)
        n_g = p.gpu.delete(dev(gone))
        assert n_g == n_o > 700
        st = p.gpu.stats()
        assert st.n_total == p.orc.ntotal and st.device_error == 0 and st.pages_used == pages_before
        assert np.array_equal(p.gpu.list_lengths(), p.orc.list_lengths()) and p.gpu.list_lengths()[big] == 0
        assert p.gpu.delete(dev(gone)) == 0
        p.check_search(q, 10, 8, where="after delete")
        full = p.check_scan(q, 40, np.tile(np.arange(cfg.nlist, dtype=np.int32), (len(q), 1)), where="all lists")
        # growth after shrinking: the emptied list takes its old pages back, no new page is opened
        refill = extra[400:440] if storage == F32 else extra[400:440].astype(np.float16).astype(np.float32)
        forced = np.full(len(refill), big, dtype=np.int32)
        p.gpu.insert_assigned(dev(refill), dev(forced), dev(eids[400:440]))
        p.orc.insert(refill, eids[400:440], forced_lists=forced)
        p.note_inserted(refill)
        assert p.gpu.stats().pages_used == pages_before and p.gpu.list_lengths()[big] == 40
        for s in range(440, 600, 40):
            p.insert_both(extra[s:s + 40], eids[s:s + 40], where=f"batch {s // 40} after delete")
        assert np.array_equal(p.gpu.list_lengths(), p.orc.list_lengths())
        p.check_search(q, 10, 8, where="inserts after delete")
        # update: a surviving id gets a new vector
        keep = ids[~np.isin(ids, gone)][0]
        newv = q[3:4] if storage == F32 else q[3:4].astype(np.float16).astype(np.float32)
        assert p.gpu.delete(dev(np.array([keep]))) == 1 and p.orc.delete(np.array([keep])) == 1
        p.insert_both(newv, np.array([keep]), where="update")
        gi, gv = p.gpu.search(dev(q[3:4]), 1, 8)
        assert int(gi[0, 0]) == keep
        p.check_search(q, 10, 8, where="after update")
        # compaction after deletes drops the unused pages
        p.gpu.compact(B.pk_arena_bytes(p.gpu.cfg, int(p.gpu.stats().n_total), 100))
        lens = p.gpu.list_lengths()
        assert p.gpu.stats().pages_used == int(np.sum((lens + 31) // 32)) < pages_before
        p.check_search(q, 10, 8, where="compacted after deletes")
    finally:
        p.close()


def test_delete_from_a_very_long_list(gpu_device):
    """Deleting is parallel over the rows, not over the lists: 4096 ids out of a list of more than
    400 000 rows (most of them at its tail, so that rows to go and rows that stay meet beyond the list's
    new end), twice in a row, then ids that several rows carry (more rows than one pass takes).  List
    lengths and counts follow the oracle, searches over the shrunken list match it, and the call takes
    milliseconds, not the seconds a walk along the list would."""
    import time
    rng = np.random.default_rng(11)
    d, nlist, n_big, n_rest = 32, 8, 420000, 30000
    cent = rng.standard_normal((nlist, d)).astype(np.float32) * 4
    x = np.concatenate([cent[0] + 0.3 * rng.standard_normal((n_big, d)).astype(np.float32),
                        cent[rng.integers(1, nlist, n_rest)] + 0.3 * rng.standard_normal((n_rest, d)).astype(np.float32)])
    ids = np.arange(len(x), dtype=np.int64) * 3 + 1
    ids[200000:205000] = 77  # 5000 rows under one id
    p = Pair(x, cent, L2, F32, ids=ids, insert_reserve=1000)
    try:
        assert p.orc.list_lengths()[0] >= 400000
        q = (cent[0] + 0.3 * rng.standard_normal((32, d))).astype(np.float32)
        tail = ids[n_big - 3000:n_big]  # the list's last rows in build order
        free = np.concatenate([np.arange(0, 200000), np.arange(205000, n_big - 3000)])  # not the shared id, not the tail
        gone = np.concatenate([tail[::2], ids[rng.choice(free, 4096 - 1500, replace=False)]])
        for rep in range(2):
            say(f"delete of {len(gone)} ids, call {rep}")
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            n_g = p.gpu.delete(dev(gone))
            ms = (time.perf_counter() - t0) * 1e3
            n_o = p.orc.delete(gone)
            print(f"[delete] {len(gone)} ids, {n_g} rows removed from a {int(p.orc.list_lengths()[0]) + n_g}-row list "
                  f"in {ms:.2f} ms", flush=True)
            assert n_g == n_o and (n_g > 4000 if rep == 0 else n_g == 0)
            assert ms < 50, f"delete took {ms:.1f} ms"
            assert np.array_equal(p.gpu.list_lengths(), p.orc.list_lengths())
        p.check_search(q, 10, 2, where="after the delete")
        say("delete of an id that 5000 rows carry")
        assert p.gpu.delete(dev(np.array([77, ids[5]]))) == p.orc.delete(np.array([77, ids[5]])) == 5001
        assert np.array_equal(p.gpu.list_lengths(), p.orc.list_lengths())
        st = p.gpu.stats()
        assert st.n_total == p.orc.ntotal and st.device_error == 0
        p.check_search(q, 10, 2, where="after the second delete")
        full = np.tile(np.arange(nlist, dtype=np.int32), (len(q), 1))
        p.check_scan(q, 20, full, where="all lists after the deletes")
    finally:
        p.close()


@pytest.mark.parametrize("storage,metric", [(F32, L2), (F16, IP)])
def test_ivf_split(gpu_device, storage, metric):
    """Lists over the threshold are split by a 2-means on the device.  Against the oracle's own split:
    the same lists split, near-identical sides (a near-tie may move single members).  Exactly: the other
    lists and centroids are untouched, nothing is lost, each new centroid is the float64 mean of the
    members its side ended with; and an oracle index mirrored from the GPU's state (its centroids, its
    membership) agrees with every search and with inserts that follow."""
    cfg = W.scaled(W.C1, n=6000, nlist=16)
    x = W.vectors(cfg, 0, cfg.n)
    cent = training.train_centroids(cfg, x)
    ids = np.random.default_rng(11).permutation(cfg.n).astype(np.int64) * 5 + 2
    p = Pair(x, cent, metric, storage, ids=ids, page_vecs=32, insert_reserve=2000)
    try:
        extra = np.concatenate([W.inserts(cfg, b, 64) for b in range(8)])
        eids = 10 ** 8 + np.arange(len(extra), dtype=np.int64)
        for s in range(0, 384, 64):
            p.insert_both(extra[s:s + 64], eids[s:s + 64], where=f"batch {s // 64}")
        rows = {int(i): v for i, v in zip(ids, p.x)}
        ex = extra if storage == F32 else extra.astype(np.float16).astype(np.float32)
        rows.update({int(i): v for i, v in zip(eids, ex)})
        lens0 = p.gpu.list_lengths()
        thr = int(np.sort(lens0)[-5]) - 1  # the five longest lists split
        todo = [l for l in range(16) if lens0[l] > thr]
        old_ids = [np.sort(p.gpu.list_ids(l).cpu().numpy()) for l in range(16)]
        old_cent = p.gpu.centroids().cpu().numpy()
        n = p.gpu.split(thr, 8, B.pk_arena_bytes(p.gpu.cfg, int(lens0.sum()), 1500) + (1 << 20))
        assert n == len(todo) == 5 and p.orc.split(thr, 8) == n and p.gpu.nlist == p.orc.nlist == 21
        st = p.gpu.stats()
        lens1 = p.gpu.list_lengths()
        assert st.device_error == 0 and st.n_arenas == 1 and lens1.sum() == lens0.sum() == st.n_total
        c1 = p.gpu.centroids().cpu().numpy()
        got = [p.gpu.list_ids(l).cpu().numpy() for l in range(21)]
        for l in range(16):
            if l not in todo:
                assert np.array_equal(np.sort(got[l]), old_ids[l]) and np.array_equal(c1[l], old_cent[l])
        for t, l in enumerate(todo):
            a, b = set(got[l].tolist()), set(got[16 + t].tolist())
            assert not (a & b) and sorted(a | b) == old_ids[l].tolist()
            oa, ob = set(p.orc.list_ids(l).tolist()), set(p.orc.list_ids(16 + t).tolist())
            assert len(a & oa) + len(b & ob) >= 0.97 * len(old_ids[l]), (l, len(a), len(oa))
            for lst, members in ((l, a), (16 + t, b)):
                if members:
                    want = np.mean([rows[i].astype(np.float64) for i in members], axis=0)
                    np.testing.assert_allclose(c1[lst], want, rtol=1e-5, atol=1e-6)
        # mirror: an oracle index with the GPU's centroids and membership
        mirror = oracle.Index(c1, metric)
        for l in range(21):
            if len(got[l]):
                mirror.insert(np.stack([rows[int(i)] for i in got[l]]), got[l], forced_lists=np.full(len(got[l]), l, np.int32))
        p.orc, p.cent = mirror, c1
        q = W.queries(cfg, 6, 64)
        p.check_search(q, 10, 6, where="after split")
        p.check_scan(q, 30, np.tile(np.arange(21, dtype=np.int32), (len(q), 1)), where="all lists after split")
        for s in range(384, 512, 64):
            p.insert_both(extra[s:s + 64], eids[s:s + 64], where=f"batch {s // 64} after split")
        p.check_search(q, 10, 6, where="inserts after split")
        assert np.array_equal(p.gpu.list_lengths(), p.orc.list_lengths())
    finally:
        p.close()


def test_insert_multi_across_agents(gpu_device):
    """Insert batches of several agents in one call: per agent the same lists as its own centroids
    dictate (oracle rule), running ids per agent, an agent without rows, and a segment over 1024
    rows (handled agent by agent); searches follow the oracle afterwards."""
    cfg = W.scaled(W.C1, n=3000)
    pairs = []
    try:
        for a in range(3):
            x = W.vectors(cfg, 0, 3000 - 500 * a, agent=a)
            pairs.append(Pair(x, training.train_centroids(W.scaled(cfg, n=len(x)), x, agent=a), IP, F32, insert_reserve=4000))
        hs = [p.gpu.handle for p in pairs]
        for sizes, with_ids in (((5, 0, 17), True), ((64, 1, 9), False), ((3, 1500, 2), False)):
            xs = [W.inserts(cfg, 50 + a, max(n, 1), agent=a)[:n] for a, n in enumerate(sizes)]
            offs = np.concatenate([[0], np.cumsum(sizes)])
            ids = (10 ** 6 * (1 + np.arange(offs[-1], dtype=np.int64))) if with_ids else None
            out = torch.empty(int(offs[-1]), dtype=torch.int32, device="cuda")
            n_before = [p.gpu.stats().n_total for p in pairs]
            next_id = [p.orc.ntotal for p in pairs]
            B.pk_insert_multi(hs, offs, dev(np.concatenate(xs)), None if ids is None else dev(ids), out)
            lists = out.cpu().numpy()
            for a, p in enumerate(pairs):
                lo, hi = int(offs[a]), int(offs[a + 1])
                if hi > lo:
                    # without ids the library continues the agent's own counter of vectors ever added
                    mirror_ids = ids[lo:hi] if ids is not None else next_id[a] + np.arange(hi - lo, dtype=np.int64)
                    p.accept_inserted(xs[a], lists[lo:hi], mirror_ids, where=f"agent {a}")
                assert p.gpu.stats().n_total == n_before[a] + sizes[a]
                assert np.array_equal(p.gpu.list_lengths(), p.orc.list_lengths())
                if ids is None and hi > lo:  # running ids: the agent's own counter
                    got, _ = p.gpu.search(dev(xs[a][:1]), 1, p.gpu.nlist)
                    assert int(got[0, 0]) == next_id[a]
        for a, p in enumerate(pairs):
            p.check_search(W.queries(cfg, 8, 32, agent=a), 10, 8, where=f"agent {a} after multi inserts")
    finally:
        for p in pairs:
            p.close()


def test_wide_rows_many_queries_per_list(gpu_device):
    """d = 1536 (config 5 width) with few lists, so lists see more queries than one group holds."""
    cfg = W.scaled(W.C5, n=5000, ncomp=24, nlist=24, zipf_s=1.2)
    for storage in (F32, F16):
        p, _ = make_pair(cfg, storage=storage)
        try:
            q = W.queries(cfg, 0, 80)
            say(f"wide rows storage={storage}")
            p.check_search(q, 10, 6)
            p.check_search(q, 100, 24)
        finally:
            p.close()


def test_hot_lists_rows_stationary_kernel(gpu_device):
    """Batches of >= 512 queries over few lists: every list is probed by hundreds of queries and goes
    to the rows-stationary kernel (64-row tiles against all slots of the list), next to regular lists;
    ragged list tails, delta pages, more than 1024 queries on one list (two slot groups)."""
    cfg = W.scaled(W.C1, n=9000, ncomp=12, nlist=12)
    for storage, metric in ((F32, IP), (F16, L2), (F32, L2)):
        p, _ = make_pair(cfg, metric=metric, storage=storage, insert_reserve=2048)
        try:
            q = W.queries(cfg, 30, 640)
            say(f"hot lists storage={storage} metric={metric}: 640 queries, nprobe 6")
            p.check_search(q, 10, 6)
            p.insert_both(W.inserts(cfg, 0, 700), where="hot lists")
            say("hot lists: after 700 inserts, k 100")
            p.check_search(q, 100, 5)
            q2 = W.queries(cfg, 31, 1300)
            say("hot lists: 1300 queries on every list")
            p.check_search(q2, 10, 12)
        finally:
            p.close()
    # wide-ish fp16 rows (d = 768: the widest rows the kernel takes), lists of uneven length
    cfg = W.scaled(W.C4, n=6000, ncomp=40, nlist=40)
    p, _ = make_pair(cfg, metric=L2, storage=F16)
    try:
        q = W.queries(cfg, 32, 768)
        say("hot lists: d=768 fp16, 768 queries, nprobe 16")
        p.check_search(q, 20, 16)
    finally:
        p.close()


def test_two_tile_classes_side_by_side_on_two_streams(gpu_device):
    """A batch of 512 queries or more whose lists fall into both tile classes has the kernel for the lists
    many queries probe and the scan of the other lists run side by side (the second on a stream of the
    handle's own, forked from and joined to the caller's by events).  The call must stay stream-ordered for
    the caller: searches issued back to back on a stream other than the default one, with an insert between
    them, give bit for bit the rows of the same searches run one at a time between device-wide waits; those
    match the oracle; and a captured graph (under capture the two kernels run one after the other) replays
    to the same rows."""
    cfg = W.scaled(W.C1, n=30000, ncomp=96, nlist=96)
    p, _ = make_pair(cfg, metric=L2, storage=F16, insert_reserve=4096)
    try:
        k, nprobe, nq = 10, 6, 768
        qs = [dev(W.queries(cfg, 40 + b, nq)) for b in range(3)]
        new = W.inserts(cfg, 5, 300).astype(np.float16).astype(np.float32)
        say("one search at a time")
        alone = []
        for b in range(3):
            i, v = p.gpu.search(qs[b], k, nprobe)
            torch.cuda.synchronize()
            alone.append((i.cpu().numpy(), v.cpu().numpy()))
        B.pk_profile_begin(p.gpu.handle)
        p.gpu.search(qs[0], k, nprobe)
        pr = B.pk_profile_end(p.gpu.handle)
        assert pr.scan_hot_ms > 0 and pr.scan_ms >= pr.scan_hot_ms, "the batch has lists of both tile classes"
        say("back to back on a second stream")
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            outs = [p.gpu.search(qs[b], k, nprobe) for b in (0, 1, 2, 0)]
            lists = p.gpu.insert(dev(new), want_lists=True)
            after = p.gpu.search(qs[1], k, nprobe)
        torch.cuda.synchronize()
        for n, b in enumerate((0, 1, 2, 0)):
            assert np.array_equal(outs[n][0].cpu().numpy(), alone[b][0]), f"ids of back-to-back search {n} differ"
            assert np.array_equal(outs[n][1].cpu().numpy(), alone[b][1]), f"values of back-to-back search {n} differ"
        p.accept_inserted(new, lists.cpu().numpy(), where="insert between searches")
        say("after the insert: the oracle's rows, and the search issued right behind the insert")
        p.check_search(qs[1].cpu().numpy(), k, nprobe, where="after the insert")
        i2, v2 = p.gpu.search(qs[1], k, nprobe)
        torch.cuda.synchronize()
        assert np.array_equal(after[0].cpu().numpy(), i2.cpu().numpy()) and np.array_equal(after[1].cpu().numpy(), v2.cpu().numpy())
        say("graph capture")
        ids = torch.empty((nq, k), dtype=torch.int64, device="cuda")
        dist = torch.empty((nq, k), dtype=torch.float32, device="cuda")
        graph = torch.cuda.CUDAGraph()
        cap = torch.cuda.Stream()
        with torch.cuda.stream(cap):
            with torch.cuda.graph(graph, stream=cap):
                B.pk_search(p.gpu.handle, qs[1], k, nprobe, ids, dist)
        torch.cuda.synchronize()
        for rep in range(2):
            ids.fill_(-7)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert np.array_equal(ids.cpu().numpy(), i2.cpu().numpy()) and np.array_equal(dist.cpu().numpy(), v2.cpu().numpy())
        st = p.gpu.stats()
        assert st.device_error == 0
    finally:
        p.close()


def test_hot_lists_across_agents_in_one_call(gpu_device):
    """Two agents, hundreds of queries each over few lists, one segmented call: the rows-stationary tiles
    of both indexes share a launch.  Same results as the per-handle calls (which, 400 queries each, stay
    below the batch size that enables that kernel: the two paths must agree bit for bit) and parity with
    the oracle."""
    cfg = W.scaled(W.C3, d=128, ncomp=10, nlist=10, n_agents=2)
    pairs, qs, offs = [], [], [0]
    try:
        for a, n in enumerate((5000, 3500)):
            p, _ = make_pair(cfg, n=n, agent=a, insert_reserve=256)
            pairs.append(p)
            qs.append(W.queries(cfg, 3, 400, agent=a))
            offs.append(offs[-1] + 400)
        q = np.concatenate(qs)
        say("hot lists, two agents, one launch")
        mi, mv = B.search_multi([p.gpu for p in pairs], offs, dev(q), 10, 8)
        for a, p in enumerate(pairs):
            si, sv = p.gpu.search(dev(qs[a]), 10, 8)
            assert torch.equal(mi[offs[a]:offs[a + 1]], si) and torch.equal(mv[offs[a]:offs[a + 1]], sv)
            p.check_search(qs[a], 10, 8, where=f"agent {a}")
    finally:
        for p in pairs:
            p.close()


def test_very_large_query_batch(gpu_device):
    """More queries than one launch sequence takes (32768): the call is cut into batches; every list
    is probed by thousands of queries (many slot groups per rows-stationary tile)."""
    cfg = W.scaled(W.C1, n=2000, d=64, ncomp=8, nlist=8)
    p, _ = make_pair(cfg, metric=L2)
    try:
        q = np.concatenate([W.queries(cfg, 40 + b, 3000) for b in range(11)])  # 33 000 queries
        say("33 000 queries in one call")
        gi, gv = p.gpu.search(dev(q), 5, 2)
        gp = p.gpu.coarse(dev(q), 2).cpu().numpy()
        oi, ov = p.orc.scan_probes(q, 5 + KX, gp)
        check_results(gi.cpu().numpy(), gv.cpu().numpy(), oi, ov, 5, p.tol, p.scale(q), L2, where="large batch")
        assert p.gpu.stats().device_error == 0
        # the first and the last queries alone give the same rows
        for lo, hi in ((0, 100), (32900, 33000)):
            si, sv = p.gpu.search(dev(q[lo:hi]), 5, 2)
            assert torch.equal(si, gi[lo:hi]) and torch.equal(sv, gv[lo:hi])
    finally:
        p.close()


@pytest.mark.parametrize("storage,metric", [(F32, L2), (F16, IP)])
def test_level_cascade_with_early_termination(gpu_device, storage, metric):
    """Section 4.2: three levels (every upper level a subset of the one below), per-query thresholds.
    The level each query ends at must be the oracle's, its row that level's row (oracle parity with the
    GPU's own probe lists, as for a plain search).  Thresholds sit between the k-th values the levels
    give, far from any of them, so rounding cannot flip a decision."""
    cfg = W.scaled(W.C1, n=8000)
    x = W.vectors(cfg, 0, cfg.n)
    if storage == F16:
        x = x.astype(np.float16).astype(np.float32)
    cent = training.train_centroids(cfg, x)
    ids_all = np.arange(cfg.n, dtype=np.int64)
    subsets = [ids_all[::16], ids_all[::4], ids_all]  # top level first
    cents = [cent[:8].copy(), cent[:32].copy(), cent]
    nprobes = [4, 6, 8]
    k = 10
    pairs = [Pair(x[sub], c, metric, storage, ids=sub) for sub, c in zip(subsets, cents)]
    try:
        q = W.queries(cfg, 50, 96)
        kth = [p.orc.search(q, k, npb)[1][:, k - 1] for p, npb in zip(pairs, nprobes)]
        # a third of the queries end at each level: threshold just past the level's own k-th value
        # (and the upper levels' k-th values, sparser subsets, are farther than that)
        want = np.arange(len(q)) % 3
        worse = 1.0 if metric == L2 else -1.0
        stop = np.empty(len(q), np.float32)
        for i in range(len(q)):
            span = abs(kth[0][i] - kth[2][i]) + 1e-3
            if want[i] == 2:
                stop[i] = kth[2][i] - worse * 10 * span  # nothing beats it: the search runs to the last level
            else:
                stop[i] = kth[want[i]][i] + worse * 0.3 * span
        olevel, _, _ = oracle.search_levels([p.orc for p in pairs], q, k, nprobes, stop)
        say(f"level cascade storage={storage} metric={metric}: oracle levels {np.bincount(olevel, minlength=3)}")
        glevel, gi, gv = B.search_levels([p.gpu for p in pairs], nprobes, dev(q), k, dev(stop))
        glevel = glevel.cpu().numpy()
        # decisions whose margin is inside the tolerance may differ; the thresholds above keep clear of that
        margin = np.minimum.reduce([np.abs(kv - stop) for kv in kth])
        safe = margin > 20 * pairs[0].tol * pairs[0].scale(q)
        assert safe.mean() > 0.6
        assert np.array_equal(glevel[safe], olevel[safe])
        assert len(set(glevel.tolist())) == 3
        gi, gv = gi.cpu().numpy(), gv.cpu().numpy()
        for l, (p, npb) in enumerate(zip(pairs, nprobes)):
            rows = np.nonzero(glevel == l)[0]
            if rows.size == 0:
                continue
            gp = p.gpu.coarse(dev(q[rows]), npb).cpu().numpy()
            oi, ov = p.orc.scan_probes(q[rows], k + p.kx, gp)
            check_results(gi[rows], gv[rows], oi, ov, k, p.tol, p.scale(q[rows]), metric, where=f"level {l}")
            si, sv = p.gpu.search(dev(q[rows]), k, npb)  # and bit for bit the plain search of that level
            assert np.array_equal(si.cpu().numpy(), gi[rows]) and np.array_equal(sv.cpu().numpy(), gv[rows])
        for p in pairs:
            assert p.gpu.stats().device_error == 0
    finally:
        for p in pairs:
            p.close()


def test_search_replays_from_a_hip_graph(gpu_device):
    """A search enqueues kernels only (no allocation, no host synchronisation once the handle's workspace
    has been sized by an earlier call of the same shape), so it can be captured into a HIP graph.  Every
    replay, with eager work between the replays, must give exactly what the eager call gives on the
    queries then in the input buffer; the eager call itself is checked against the oracle."""
    cfg = W.scaled(W.C1, n=6000)
    for storage, metric in ((F32, IP), (F16, L2)):
        p, _ = make_pair(cfg, metric=metric, storage=storage)
        try:
            k, nprobe, nq = 10, 8, 48
            qbuf = torch.empty((nq, cfg.d), dtype=torch.float32, device="cuda")
            ids = torch.empty((nq, k), dtype=torch.int64, device="cuda")
            dist = torch.empty((nq, k), dtype=torch.float32, device="cuda")
            qbuf.copy_(dev(W.queries(cfg, 20, nq)))
            B.pk_search(p.gpu.handle, qbuf, k, nprobe, ids, dist)  # sizes the workspace
            torch.cuda.synchronize()
            side = torch.cuda.Stream()
            graph = torch.cuda.CUDAGraph()
            say(f"graph capture storage={storage} metric={metric}")
            with torch.cuda.stream(side):
                with torch.cuda.graph(graph, stream=side):
                    B.pk_search(p.gpu.handle, qbuf, k, nprobe, ids, dist)
            torch.cuda.synchronize()
            for rep in range(3):
                q = W.queries(cfg, 21 + rep, nq)
                qbuf.copy_(dev(q))
                ids.fill_(-7)
                dist.fill_(0)
                torch.cuda.synchronize()
                say(f"graph replay {rep}")
                graph.replay()
                torch.cuda.synchronize()
                gi, gv = ids.cpu().numpy().copy(), dist.cpu().numpy().copy()
                ei, ev = p.gpu.search(qbuf, k, nprobe)  # eager, between the replays
                torch.cuda.synchronize()
                assert np.array_equal(gi, ei.cpu().numpy()), f"replay {rep}: ids differ from the eager call"
                assert np.array_equal(gv, ev.cpu().numpy()), f"replay {rep}: values differ from the eager call"
                p.check_search(q, k, nprobe, where=f"eager after replay {rep}")
        finally:
            p.close()


def test_small_batches_take_fewer_launches_and_give_the_same_results(gpu_device):
    """Batches of few queries build their work list inside the coarse selection and the threshold kernel
    (no launches of its own), and a few single inserts are assigned by the centroid kernel itself.  Which
    launch sequence a query goes through must not show in its result: the rows of a small call are
    bit-identical to the same queries' rows in a batch large enough for the separate work-list kernels (and,
    with 512 queries or more, the rows-in-registers kernel for the lists many queries probe); single inserts
    and inserts of a few vectors land in the lists the oracle's rule picks."""
    cfg = W.scaled(W.C1, n=24000, nlist=96)
    for storage, metric in ((F32, IP), (F32, L2), (F16, L2)):
        p, _ = make_pair(cfg, metric=metric, storage=storage)
        try:
            k, nprobe, big = 10, 24, 1024  # 1024 x 24 pairs: beyond what the fused path takes
            q = np.concatenate([W.queries(cfg, 30 + b, 256) for b in range(big // 256)])
            say(f"large batch storage={storage} metric={metric}")
            bi, bv = p.gpu.search(dev(q), k, nprobe)
            bi, bv = bi.cpu().numpy(), bv.cpu().numpy()
            p.check_search(q[:64], k, nprobe, where="64 queries on their own")
            for lo, cnt in ((0, 1), (5, 16), (100, 48), (900, 64)):
                say(f"small batch [{lo}, {lo + cnt})")
                si, sv = p.gpu.search(dev(q[lo:lo + cnt]), k, nprobe)
                assert np.array_equal(si.cpu().numpy(), bi[lo:lo + cnt]), f"ids of queries {lo}..{lo + cnt} differ"
                assert np.array_equal(sv.cpu().numpy(), bv[lo:lo + cnt]), f"values of queries {lo}..{lo + cnt} differ"
            new = W.inserts(cfg, 3, 40)
            say("single inserts")
            for r in range(8):
                p.insert_both(new[r:r + 1], where=f"single insert {r}")
            p.insert_both(new[8:40], where="insert of 32")
            p.check_search(q[:32], k, nprobe, where="after the inserts")
        finally:
            p.close()


def test_small_batch_thresholds_from_one_tile_several_tiles_and_long_samples(gpu_device):
    """The one-launch sample of small batches has three ways to a query's threshold: one tile per query
    (values through LDS), several tiles (values through memory, the last workgroup to finish reads them
    back) with samples of up to 1024 rows, and longer samples (a very long list in a batch of one or two
    queries asks for many pages).  Each must give the rows the oracle gives, and the rows the same queries
    get inside a 1024-query batch, whose sample, thresholds and work list come from separate launches."""
    rng = np.random.default_rng(77)
    d, nlist = 32, 16
    cent = rng.standard_normal((nlist, d)).astype(np.float32)
    # list 3 takes 85 % of the rows: 60 000 of 70 000
    n = 70000
    comp = np.where(rng.random(n) < 0.85, 3, rng.integers(0, nlist, n))
    x = (cent[comp] + 0.35 * rng.standard_normal((n, d))).astype(np.float32)
    qc = np.where(rng.random(1024) < 0.5, 3, rng.integers(0, nlist, 1024))
    q = (cent[qc] + 0.35 * rng.standard_normal((1024, d))).astype(np.float32)
    for storage, metric, page_vecs in ((F32, L2, 128), (F16, IP, 128), (F32, IP, 32), (F16, L2, 1024)):
        p = Pair(x, cent, metric, storage, page_vecs=page_vecs)
        try:
            assert p.gpu.list_lengths()[3] > 50000
            for k, nprobe in ((10, 4), (100, 3), (300, 4)):
                say(f"large batch storage={storage} metric={metric} P={page_vecs} k={k}")
                bi, bv = p.gpu.search(dev(q), k, nprobe)
                bi, bv = bi.cpu().numpy(), bv.cpu().numpy()
                for lo, cnt in ((0, 1), (1, 2), (8, 8), (100, 64)):
                    say(f"small batch [{lo}, {lo + cnt}) k={k}")
                    si, sv = p.gpu.search(dev(q[lo:lo + cnt]), k, nprobe)
                    assert np.array_equal(si.cpu().numpy(), bi[lo:lo + cnt]), f"ids of queries {lo}..{lo + cnt} differ (k={k})"
                    assert np.array_equal(sv.cpu().numpy(), bv[lo:lo + cnt]), f"values of queries {lo}..{lo + cnt} differ (k={k})"
                p.check_search(q[:2], k, nprobe, where=f"two queries k={k}")
                p.check_search(q[100:132], k, nprobe, where=f"32 queries k={k}")
            assert p.gpu.stats().device_error == 0
        finally:
            p.close()


def _captured_kernel_launches(call):
    """Kernel nodes (and all nodes) of the HIP graph that capturing `call` on a stream of its own records.
    Nothing of the graph is run.  The HIP runtime is the one the process has loaded already (torch's)."""
    import ctypes as C
    path = None
    with open("/proc/self/maps") as f:
        for line in f:
            if "libamdhip64" in line:
                path = line.split()[-1]
                break
    assert path, "no HIP runtime in this process"
    hip = C.CDLL(path)
    hip.hipStreamBeginCapture.argtypes = [C.c_void_p, C.c_int]
    hip.hipStreamEndCapture.argtypes = [C.c_void_p, C.POINTER(C.c_void_p)]
    hip.hipGraphGetNodes.argtypes = [C.c_void_p, C.POINTER(C.c_void_p), C.POINTER(C.c_size_t)]
    hip.hipGraphNodeGetType.argtypes = [C.c_void_p, C.POINTER(C.c_int)]
    hip.hipGraphDestroy.argtypes = [C.c_void_p]
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    graph = C.c_void_p()
    with torch.cuda.stream(side):
        assert hip.hipStreamBeginCapture(side.cuda_stream, 2) == 0  # relaxed mode: other threads are not affected
        try:
            call()
        finally:
            rc = hip.hipStreamEndCapture(side.cuda_stream, C.byref(graph))
    assert rc == 0 and graph.value
    n = C.c_size_t(0)
    assert hip.hipGraphGetNodes(graph, None, C.byref(n)) == 0
    nodes = (C.c_void_p * max(1, n.value))()
    assert hip.hipGraphGetNodes(graph, nodes, C.byref(n)) == 0
    kernels = 0
    for i in range(n.value):
        kind = C.c_int(-1)
        assert hip.hipGraphNodeGetType(nodes[i], C.byref(kind)) == 0
        kernels += kind.value == 0  # hipGraphNodeTypeKernel
    hip.hipGraphDestroy(graph)
    torch.cuda.synchronize()
    return kernels, n.value


def test_a_small_search_is_five_kernel_launches(gpu_device):
    """Section 3.3: small batches are bound by launches, not by arithmetic.  A search of up to 64 queries
    over fp32 rows (inner product) is five kernels: centroid scores, top-nprobe with the pair counts,
    threshold sample with thresholds and work list, gated scan, final selection; the other storage and
    metric combinations add the preparation of the queries.  Counted as the kernel nodes of the HIP graph
    a capture of the call records (the graph is not run; the eager call before it is checked against the
    oracle, and so is the one after it)."""
    cfg = W.scaled(W.C1, n=6000)
    for storage, metric, most in ((F32, IP, 5), (F32, L2, 6), (F16, IP, 6), (F16, L2, 7)):
        p, _ = make_pair(cfg, metric=metric, storage=storage)
        try:
            k, nprobe = 10, 8
            for nq in (1, 16, 64):
                q = W.queries(cfg, 40, nq)
                qbuf = dev(q)
                ids = torch.empty((nq, k), dtype=torch.int64, device="cuda")
                dist = torch.empty((nq, k), dtype=torch.float32, device="cuda")
                p.check_search(q, k, nprobe, where=f"before the capture, {nq} queries")  # also sizes the workspace
                say(f"capture storage={storage} metric={metric} nq={nq}")
                kernels, nodes = _captured_kernel_launches(lambda: B.pk_search(p.gpu.handle, qbuf, k, nprobe, ids, dist))
                say(f"storage={storage} metric={metric} nq={nq}: {kernels} kernel launches ({nodes} graph nodes)")
                assert kernels == nodes, "a search records kernels only"
                assert kernels <= most, f"{kernels} launches for {nq} queries (storage {storage}, metric {metric})"
                p.check_search(q, k, nprobe, where=f"after the capture, {nq} queries")
        finally:
            p.close()


def test_reserved_workspace_never_grows_and_capture_refuses_growth(gpu_device):
    """Section 5: operations must not block the caller.  After one pk_workspace_reserve a config-5
    style stream of {insert 1; search 16} (and a batch insert, and a larger search within the
    limits) never reallocates the workspace; without the reservation the first call grows it; a
    call that would have to grow it while its stream is capturing is refused."""
    cfg = W.scaled(W.C5, n=30000, d=256, ncomp=64, nlist=64, nprobe=12)
    p, _ = make_pair(cfg, insert_reserve=5000)
    try:
        h = p.gpu.handle
        assert p.gpu.stats().workspace_bytes == 0  # the build's scratch is gone
        B.pk_workspace_reserve([h], 64, 20, 12, inserts_ahead=3000)
        st = p.gpu.stats()
        assert st.workspace_grows == 1 and 0 < st.workspace_bytes < 64 << 20
        say("reserved stream")
        new = W.inserts(cfg, 0, 600)
        q = W.queries(cfg, 0, 16)
        lists = []
        for r in range(600):
            lists.append(p.gpu.insert(dev(new[r:r + 1]), want_lists=True))
            if r % 40 == 0:
                p.gpu.search(dev(q), 10, 12)
        lists.append(p.gpu.insert(dev(W.inserts(cfg, 1, 64)), want_lists=True))
        p.gpu.search(dev(W.queries(cfg, 1, 64)), 20, 12)
        p.gpu.coarse(dev(q), 12)
        st = p.gpu.stats()
        assert st.workspace_grows == 1 and st.device_error == 0 and st.n_inserted == 664
        # the oracle agrees after the stream (the inserts checked and mirrored in one go)
        p.accept_inserted(np.concatenate([new, W.inserts(cfg, 1, 64)]), torch.cat(lists).cpu().numpy(),
                          where="reserved stream")
        p.check_scan(q, 10, p.orc.coarse(q, 12), where="after the reserved stream")
        # beyond the limits the workspace grows (eagerly) ...
        p.gpu.search(dev(W.queries(cfg, 2, 256)), 20, 12)
        assert p.gpu.stats().workspace_grows == 2
        # ... but not under capture: the call is refused and nothing is recorded
        big = dev(W.queries(cfg, 3, 2048))
        ids = torch.empty((2048, 20), dtype=torch.int64, device="cuda")
        dist = torch.empty((2048, 20), dtype=torch.float32, device="cuda")
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        refused = None
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                try:
                    B.pk_search(h, big, 20, 12, ids, dist)
                except B.PancakeError as e:
                    refused = e.status
        torch.cuda.synchronize()
        assert refused == B.PK_ERR_WORKSPACE
        assert p.gpu.stats().workspace_grows == 2
    finally:
        p.close()


def test_overflowing_emission_regions_are_rescored(gpu_device):
    """A query that emits more candidates than its region holds is selected by rescoring its rows.
    Forced with a tiny region (every query overflows): rows must equal the default path's bit for
    bit, multi-handle and level calls included, and match the oracle."""
    cfg = W.scaled(W.C1, n=9000)
    for storage, metric in ((F32, IP), (F16, L2), (F32, L2)):
        p, _ = make_pair(cfg, metric=metric, storage=storage, insert_reserve=512)
        try:
            p.insert_both(W.inserts(cfg, 0, 200), where="overflow setup")
            q = W.queries(cfg, 30, 40)
            for k, nprobe in ((10, 8), (1, 3), (100, 16)):
                want_i, want_v = p.gpu.search(dev(q), k, nprobe)
                B.pk_profile_begin(p.gpu.handle)
                B.pk_index_set_emit_cap(p.gpu.handle, 16)
                say(f"rescoring storage={storage} metric={metric} k={k} nprobe={nprobe}")
                got_i, got_v = p.gpu.search(dev(q), k, nprobe)
                pr = B.pk_profile_end(p.gpu.handle)
                B.pk_index_set_emit_cap(p.gpu.handle, 0)
                if k >= 10:  # k = 1 draws so tight a threshold that 16 entries can be enough
                    assert pr.overflowed > 0 and pr.max_emitted > 16
                assert torch.equal(got_i, want_i) and torch.equal(got_v, want_v)
            B.pk_index_set_emit_cap(p.gpu.handle, 16)
            p.check_search(q, 10, 8, where="rescored rows against the oracle")
            B.pk_index_set_emit_cap(p.gpu.handle, 0)
            assert p.gpu.stats().device_error == 0
        finally:
            p.close()


def test_tie_group_larger_than_the_emission_region(gpu_device):
    """3000 exact copies of one vector (scrambled ids, some ids carried twice) in one list: every copy
    passes any threshold, a region of 2048 entries (what a large batch gets for k = 10; set by hand here,
    a batch of three queries would get more) overflows by itself, and the k lowest ids of the tie group
    must come back, as in the oracle's sort."""
    rng = np.random.default_rng(26)
    n, d = 12000, 64
    x = rng.standard_normal((n, d)).astype(np.float32)
    x /= np.linalg.norm(x, axis=1, keepdims=True)
    dup = rng.permutation(n)[:3000]
    x[dup] = x[dup[0]]
    ids = rng.permutation(n).astype(np.int64) + 50
    ids[dup[1]] = ids[dup[2]] = 7   # one id carried by two members of the group
    cent = x[rng.permutation(n)[:8]].copy()
    q = np.stack([x[dup[0]], x[5], x[dup[0]] * 0.5])
    for metric in (IP, L2):
        p = Pair(x, cent, metric, F32, ids=ids)
        B.pk_index_set_emit_cap(p.gpu.handle, 2048)
        try:
            for k in (1, 10, 64):
                say(f"tie group metric={metric} k={k}")
                B.pk_profile_begin(p.gpu.handle)
                gi, gv = p.gpu.search(dev(q), k, 8)
                pr = B.pk_profile_end(p.gpu.handle)
                assert pr.overflowed >= 2, pr.overflowed
                gi, gv = gi.cpu().numpy(), gv.cpu().numpy()
                oi, ov = p.orc.search(q, k, 8)
                want = sorted(ids[dup].tolist())[:k]
                assert gi[0].tolist() == want and gi[2].tolist() == want
                assert np.array_equal(gi, oi[:, :k])
                np.testing.assert_allclose(gv, ov[:, :k], rtol=1e-4, atol=2e-6)
        finally:
            p.close()


def test_large_k_no_threshold_and_chunked_selection(gpu_device):
    """k larger than the first probed list: the threshold sample runs on into the next probed lists;
    with k = 1000 a query still emits more than its region holds (32768 entries) and is rescored."""
    cfg = W.scaled(W.C1, n=45000)
    p, _ = make_pair(cfg, metric=L2)
    try:
        q = W.queries(cfg, 9, 6)
        say("large k")
        p.check_search(q, 1000, 64)
        p.check_search(q, 1024, 64)
        p.check_search(q, 300, 20)
    finally:
        p.close()


def test_arena_exhaustion_is_reported_and_recoverable(gpu_device):
    cfg = W.scaled(W.C1, n=3000)
    x = W.vectors(cfg, 0, cfg.n)
    cent = training.train_centroids(cfg, x)
    c = B.pk_config(cfg.d, cfg.nlist, IP, F32, 32, 0)
    with pytest.raises(B.PancakeError) as e:
        B.Index(dev(cent), dev(x), page_vecs=32, arena_bytes=B.pk_arena_bytes(c, 100, 0))
    assert e.value.status == B.PK_ERR_NOMEM
    ix = B.Index(dev(cent), dev(x), page_vecs=32, arena_bytes=B.pk_arena_bytes(c, cfg.n, 0))
    try:
        free = ix.stats().pages_total - ix.stats().pages_used
        new = dev(W.inserts(cfg, 0, (int(free) + 2) * 32 + 64 * 32))  # cannot fit whatever the assignment
        with pytest.raises(B.PancakeError) as e:
            ix.insert(new)
        assert e.value.status == B.PK_ERR_NOMEM and ix.stats().n_total == cfg.n
        ix.add_arena(B.pk_arena_bytes(c, 0, 4096))
        ix.insert(new)
        st = ix.stats()
        assert st.n_total == cfg.n + new.shape[0] and st.device_error == 0 and st.n_arenas == 2
        ids, dist = ix.search(new[:16], 1, 1)
        assert ids[:, 0].cpu().tolist() == list(range(cfg.n, cfg.n + 16))
    finally:
        ix.close()


def test_argument_errors_on_device(gpu_device):
    cfg = W.scaled(W.C1, n=500)
    x = W.vectors(cfg, 0, cfg.n)
    ix = B.Index(dev(x[:8].copy()), dev(x))
    try:
        q = dev(x[:4].copy())
        for k, nprobe in ((0, 1), (1025, 1), (1, 0), (1, 9)):
            with pytest.raises(B.PancakeError) as e:
                ix.search(q, k, nprobe)
            assert e.value.status == B.PK_ERR_INVALID_ARG
        ids, dist = ix.search(q[:0], 3, 2)  # empty batch is a no-op
        assert ids.shape == (0, 3)
    finally:
        ix.close()
