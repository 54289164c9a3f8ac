"""Pins for the CPU oracle: what the paper's definitions and the mathematics fix.

The paper prints no worked IVF example, so the pins are (a) a hand-computed 2-D
example of the Section 2.2 / 3.1 definitions (tests/golden), (b) reduction of
exact search to a matmul + lexicographic sort, (c) invariants that any IVF index
obeys: nprobe = nlist equals exact search, insert-then-search returns the vector
itself at distance 0, unit-norm closed form, nestedness in nprobe, the partition
property, order-independence of storage, (d) textbook k-means properties.
"""
import json
import os

import numpy as np
import pytest

import oracle
from paper_2602_21477_amd import workload as W
import training

GOLD = os.path.join(os.path.dirname(__file__), "golden", "toy_ivf_2d.json")
METRICS = {"IP": oracle.IP, "L2": oracle.L2}


def _val(v):
    return float(v)  # "-inf" / "inf" strings parse too


def _numpy_exact(x, ids, q, k, metric):
    """Exact kNN by a library routine: float64 matmul + lexsort (value, then id)."""
    x64, q64 = x.astype(np.float64), q.astype(np.float64)
    if metric == oracle.IP:
        v = q64 @ x64.T
        key = -v
    else:
        v = ((q64[:, None, :] - x64[None, :, :]) ** 2).sum(-1)
        key = v
    out_i = np.empty((q.shape[0], k), dtype=np.int64)
    out_v = np.empty((q.shape[0], k))
    for i in range(q.shape[0]):
        order = np.lexsort((ids, key[i]))[:k]
        out_i[i], out_v[i] = ids[order], v[i][order]
    return out_i, out_v


def _small(seed, n=1500, d=16, nlist=12, normalise=True):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n, d)).astype(np.float32)
    q = rng.standard_normal((40, d)).astype(np.float32)
    if normalise:
        x /= np.linalg.norm(x, axis=1, keepdims=True)
        q /= np.linalg.norm(q, axis=1, keepdims=True)
    c = x[rng.permutation(n)[:nlist]].copy()
    return x, q, c, rng


# ----------------------------------------------------------------- golden toy

def test_golden_toy_example():
    g = json.load(open(GOLD))
    cent = np.array(g["centroids"], dtype=np.float32)
    x = np.array(g["vectors"], dtype=np.float32)
    for case in g["cases"]:
        m = METRICS[case["metric"]]
        ix = oracle.Index(cent, m)
        ix.build(x)
        for j, want in enumerate(case["lists"]):
            assert ix.list_ids(j).tolist() == want
        for s in case["searches"]:
            q = np.array([s["query"]], dtype=np.float32)
            assert ix.coarse(q, s["nprobe"])[0].tolist() == s["probes"]
            ids, val = ix.search(q, s["k"], s["nprobe"])
            assert ids[0].tolist() == s["ids"]
            assert val[0].tolist() == [_val(v) for v in s["values"]]
        for b in case["bruteforce"]:
            ids, val = oracle.bruteforce(x, np.array([b["query"]], dtype=np.float32), b["k"], m)
            assert ids[0].tolist() == b["ids"] and val[0].tolist() == [_val(v) for v in b["values"]]
        if "insert" in case:
            ins = case["insert"]
            a = ix.insert(np.array([ins["vector"]], dtype=np.float32), ids=[ins["id"]])
            assert a.tolist() == [ins["list"]]
            s = ins["then_search"]
            ids, val = ix.search(np.array([s["query"]], dtype=np.float32), s["k"], s["nprobe"])
            assert ids[0].tolist() == s["ids"] and val[0].tolist() == [_val(v) for v in s["values"]]


# ------------------------------------------------------- I1 library reduction

@pytest.mark.parametrize("metric", [oracle.IP, oracle.L2])
def test_bruteforce_equals_matmul_lexsort(metric):
    x, q, _, rng = _small(1, n=2000, d=16, normalise=False)
    x[100:110] = x[5]            # exact duplicates: order must follow the id
    ids = rng.permutation(10 * x.shape[0])[:x.shape[0]].astype(np.int64)  # arbitrary, non-monotone ids
    got_i, got_v = oracle.bruteforce(x, q, 25, metric, ids=ids)
    want_i, want_v = _numpy_exact(x, ids, q, 25, metric)
    assert np.array_equal(got_i, want_i)
    np.testing.assert_allclose(got_v, want_v, rtol=1e-12, atol=1e-12)


def test_pair_values_match_numpy():
    x, q, _, _ = _small(2, n=40, d=16, normalise=False)
    for metric in (oracle.IP, oracle.L2):
        v = oracle.pair_values(q, x, metric)
        w = (q.astype(np.float64) * x).sum(1) if metric == oracle.IP else ((q.astype(np.float64) - x) ** 2).sum(1)
        np.testing.assert_allclose(v, w, rtol=1e-13, atol=1e-13)


# --------------------------------------------- I2 nprobe = nlist is exact kNN

@pytest.mark.parametrize("metric", [oracle.IP, oracle.L2])
def test_full_probe_equals_bruteforce(metric):
    x, q, c, _ = _small(3)
    ix = oracle.Index(c, metric)
    ix.build(x)
    ids, val = ix.search(q, 20, ix.nlist)
    bi, bv = oracle.bruteforce(x, q, 20, metric)
    assert np.array_equal(ids, bi)
    assert np.array_equal(val, bv)


# ------------------------------------------------ I3 insert-then-search match

@pytest.mark.parametrize("metric", [oracle.IP, oracle.L2])
@pytest.mark.parametrize("nprobe", [1, 4])
def test_insert_then_search_returns_self(metric, nprobe):
    x, _, c, rng = _small(4)
    ix = oracle.Index(c, metric)
    ix.build(x)
    new = rng.standard_normal((8, x.shape[1])).astype(np.float32)
    if metric == oracle.IP:
        # under inner product the self match is only the best match for unit vectors
        new /= np.linalg.norm(new, axis=1, keepdims=True)
    first_id = ix.ntotal
    a = ix.insert(new)
    assert ix.ntotal == first_id + 8
    ids, val = ix.search(new, 3, nprobe)
    assert ids[:, 0].tolist() == list(range(first_id, first_id + 8))
    if metric == oracle.L2:
        assert np.all(val[:, 0] == 0.0)
    else:
        np.testing.assert_allclose(val[:, 0], (new.astype(np.float64) ** 2).sum(1), rtol=1e-14)
    # the assigned list is the rank-1 probe of the same vector
    assert np.array_equal(a, ix.coarse(new, 1)[:, 0])


# ----------------------------------------------------- I4 unit-norm closed form

def test_unit_norm_l2_is_two_minus_two_ip():
    x, q, c, _ = _small(5)
    # renormalise in double and keep only directions whose fp32 norm is 1 to ~1e-7
    ids_ip, v_ip = oracle.bruteforce(x, q, 30, oracle.IP)
    ids_l2, v_l2 = oracle.bruteforce(x, q, 30, oracle.L2)
    nx = (x.astype(np.float64) ** 2).sum(1)
    nq = (q.astype(np.float64) ** 2).sum(1)
    # general identity ||q-x||^2 = ||q||^2 + ||x||^2 - 2<q,x>, exact in double to 1e-12
    for i in range(q.shape[0]):
        np.testing.assert_allclose(v_l2[i], nq[i] + nx[ids_l2[i]] - 2 * oracle.pair_values(
            np.repeat(q[i:i + 1], 30, 0), x[ids_l2[i]], oracle.IP), atol=1e-12)
    # with unit norms (to fp32 rounding) the rankings coincide and L2 = 2 - 2 IP
    np.testing.assert_allclose(v_l2, 2.0 - 2.0 * v_ip, atol=5e-7)
    assert np.mean(ids_ip == ids_l2) > 0.97  # fp32 norm rounding may swap near-ties only


# ------------------------------------------------------- I5 nested in nprobe

@pytest.mark.parametrize("metric", [oracle.IP, oracle.L2])
def test_probe_sets_nested_and_quality_monotone(metric):
    x, q, c, _ = _small(6)
    ix = oracle.Index(c, metric)
    ix.build(x)
    bi, _ = oracle.bruteforce(x, q, 10, metric)
    prev_p, prev_kth, prev_rec = None, None, -1.0
    for nprobe in (1, 2, 3, 6, 12):
        p = ix.coarse(q, nprobe)
        if prev_p is not None:
            assert np.array_equal(p[:, :prev_p.shape[1]], prev_p)
        ids, val = ix.search(q, 10, nprobe)
        kth = val[:, -1]
        if prev_kth is not None:
            assert np.all(kth >= prev_kth) if metric == oracle.IP else np.all(kth <= prev_kth)
        rec = np.mean([len(set(a.tolist()) & set(b.tolist())) for a, b in zip(ids, bi)]) / 10
        assert rec >= prev_rec
        prev_p, prev_kth, prev_rec = p, kth, rec
    assert prev_rec == 1.0


# ---------------------------------------------------------- I6 partition

@pytest.mark.parametrize("metric", [oracle.IP, oracle.L2])
def test_lists_partition_the_ids(metric):
    x, _, c, rng = _small(7)
    ix = oracle.Index(c, metric)
    ix.build(x)
    new = rng.standard_normal((50, x.shape[1])).astype(np.float32)
    ix.insert(new)
    allx = np.concatenate([x, new])
    lens = ix.list_lengths()
    assert lens.sum() == allx.shape[0] == ix.ntotal
    seen = np.concatenate([ix.list_ids(j) for j in range(ix.nlist)])
    assert np.array_equal(np.sort(seen), np.arange(allx.shape[0]))
    # stored list = recomputed best centroid (float64 numpy, ties to the lower index)
    x64, c64 = allx.astype(np.float64), c.astype(np.float64)
    if metric == oracle.IP:
        best = np.argmax(x64 @ c64.T, axis=1)
    else:
        best = np.argmin(((x64[:, None, :] - c64[None]) ** 2).sum(-1), axis=1)
    for j in range(ix.nlist):
        assert np.all(best[ix.list_ids(j)] == j)
    assert np.array_equal(ix.assign(allx), best.astype(np.int32))


# ----------------------------------------------------- I7 k-means properties

def test_kmeans_inertia_monotone_and_centroids_are_means():
    x = W.vectors(W.scaled(W.C1, n=4000), 0, 4000)
    init = W.init_rows(W.C1, 4000)[:32]
    cent, inertia, assign = oracle.kmeans(x, 32, 8, init)
    assert np.all(np.diff(inertia) <= 1e-9)
    for j in range(32):
        members = x[assign == j]
        if len(members):
            np.testing.assert_allclose(cent[j], members.astype(np.float64).mean(0), rtol=0, atol=1e-6)
    # one more assignment step under the oracle's own L2 rule reproduces a lower inertia
    ix = oracle.Index(cent, oracle.L2)
    a2 = ix.assign(x)
    inertia_next = ((x.astype(np.float64) - cent[a2]) ** 2).sum()
    assert inertia_next <= inertia[-1] + 1e-6


def test_kmeans_recovers_separated_components():
    rng = np.random.default_rng(8)
    mu = rng.standard_normal((6, 8)) * 10.0
    comp = np.repeat(np.arange(6), 200)
    x = (mu[comp] + 0.01 * rng.standard_normal((1200, 8))).astype(np.float32)
    init = np.array([c * 200 for c in range(6)])  # one starting point per component
    cent, _, assign = oracle.kmeans(x, 6, 5, init)
    assert np.array_equal(assign, comp)
    np.testing.assert_allclose(cent, mu, atol=5e-3)


def test_kmeans_empty_cluster_keeps_centroid():
    x = np.array([[0, 0], [0, 0], [10, 10], [10, 11]], dtype=np.float32)
    # centroids 0 and 1 start identical: ties go to the lower index, so cluster 1 never
    # gets a member and must keep its starting centroid
    cent, _, assign = oracle.kmeans(x, 3, 3, np.array([0, 1, 2]))
    assert assign.tolist() == [0, 0, 2, 2]
    np.testing.assert_allclose(cent, [[0, 0], [0, 0], [10, 10.5]])


def test_blas_lloyd_matches_plain_kmeans_on_tiny_config():
    cfg = W.scaled(W.C1, n=6000)
    x = W.vectors(cfg, 0, cfg.n)
    init = W.init_rows(cfg, cfg.n)
    c_plain, inertia, _ = oracle.kmeans(x, cfg.nlist, cfg.train_iters, init)
    c_blas = training.lloyd(x, init, cfg.train_iters)
    close = np.all(np.abs(c_plain - c_blas) < 1e-5, axis=1)
    assert close.mean() >= 0.9  # fp32 BLAS distances may flip a near-tie in a few clusters
    ix = oracle.Index(c_blas, oracle.L2)
    inertia_blas = ((x.astype(np.float64) - c_blas[ix.assign(x)]) ** 2).sum()
    assert abs(inertia_blas - inertia[-1]) / inertia[-1] < 2e-2


# ------------------------------------- I8 duplicates and storage-order freedom

@pytest.mark.parametrize("metric", [oracle.IP, oracle.L2])
def test_duplicates_ascending_and_storage_order_irrelevant(metric):
    x, q, c, rng = _small(9)
    x[200:206] = x[17]
    q[0] = x[17]
    ids = np.arange(x.shape[0], dtype=np.int64)
    ix = oracle.Index(c, metric)
    ix.build(x, ids)
    r_ids, r_val = ix.search(q, 12, 5)
    dup = sorted([17] + list(range(200, 206)))
    assert r_ids[0, :7].tolist() == dup
    perm = rng.permutation(x.shape[0])
    ix2 = oracle.Index(c, metric)
    ix2.build(x[perm], ids[perm])
    p_ids, p_val = ix2.search(q, 12, 5)
    assert np.array_equal(r_ids, p_ids) and np.array_equal(r_val, p_val)


# --------------------------------- rebuild equivalence, multi-agent, padding

@pytest.mark.parametrize("metric", [oracle.IP, oracle.L2])
def test_build_plus_insert_equals_build_of_all(metric):
    x, q, c, _ = _small(10)
    a = oracle.Index(c, metric)
    a.build(x[:1000])
    for s in range(1000, 1500, 37):
        a.insert(x[s:s + 37])
    b = oracle.Index(c, metric)
    b.build(x)
    assert np.array_equal(a.list_lengths(), b.list_lengths())
    ra, rb = a.search(q, 15, 4), b.search(q, 15, 4)
    assert np.array_equal(ra[0], rb[0]) and np.array_equal(ra[1], rb[1])


def test_search_multi_is_a_loop_over_indexes():
    idx, qs, offs = [], [], [0]
    for s in range(3):
        x, q, c, _ = _small(20 + s, n=600 + 100 * s)
        ix = oracle.Index(c, oracle.IP)
        ix.build(x)
        idx.append(ix)
        qs.append(q[:5 + s])
        offs.append(offs[-1] + 5 + s)
    ids, val = oracle.search_multi(idx, offs, np.concatenate(qs), 7, 3)
    for s in range(3):
        i1, v1 = idx[s].search(qs[s], 7, 3)
        assert np.array_equal(ids[offs[s]:offs[s + 1]], i1) and np.array_equal(val[offs[s]:offs[s + 1]], v1)


@pytest.mark.parametrize("metric", [oracle.IP, oracle.L2])
def test_scope_union_with_full_probe_is_exact_knn_over_all_memories(metric):
    """Section 3.2 scope search: with nprobe = nlist in every index the union search must equal exact kNN
    over the concatenated memories (a separate code path: float64 matmul + lexsort), with the source
    index as the first tie-breaker; one row sits in two memories and one memory is shorter than k."""
    parts, idx = [], []
    for s, n in enumerate((500, 23, 800)):
        x, q, c, _ = _small(40 + s, n=n, nlist=5)
        if s == 2:
            x[7] = parts[0][11]  # the same vector in memories 0 and 2: equal values, source 0 first
        ix = oracle.Index(c, metric)
        ix.build(x)
        parts.append(x)
        idx.append(ix)
    _, q, _, _ = _small(50)
    k = 30
    src, ids, val = oracle.search_union(idx, q, k, 5)
    allx = np.concatenate(parts)
    code = np.concatenate([np.arange(len(x), dtype=np.int64) + (s << 32) for s, x in enumerate(parts)])
    bi, bv = _numpy_exact(allx, code, q, k, metric)
    assert np.array_equal((src.astype(np.int64) << 32) + ids, bi)
    np.testing.assert_allclose(val, bv, rtol=1e-12, atol=1e-12)
    # the duplicated row: found in both memories by its own query, memory 0 listed first
    s1, i1, v1 = oracle.search_union(idx, parts[0][11:12], 2, 5)
    assert list(zip(s1[0], i1[0])) == [(0, 11), (2, 7)] and v1[0, 0] == v1[0, 1]
    # a scope of one memory is an ordinary search; a scope smaller than k is padded
    s2, i2, v2 = oracle.search_union(idx[1:2], q, k, 5)
    i3, v3 = idx[1].search(q, k, 5)
    assert np.array_equal(i2, i3) and np.array_equal(v2, v3)
    assert np.all(s2[:, 23:] == -1) and np.all(i2[:, 23:] == -1) and np.all(s2[:, :23] == 0)
    # forced probe lists: the oracle's own probes reproduce the unforced call
    probes = np.stack([ix.coarse(q, 2) for ix in idx])
    a = oracle.search_union(idx, q, k, 2)
    b = oracle.search_union(idx, q, k, 2, probes=probes)
    assert all(np.array_equal(u, v) for u, v in zip(a, b))


@pytest.mark.parametrize("metric", [oracle.IP, oracle.L2])
def test_delete_then_search_is_exact_knn_over_what_is_left(metric):
    """Delete removes every carrier of an id and nothing else: with nprobe = nlist the search equals
    exact kNN (float64 matmul + lexsort) over the remaining rows; an update is delete + insert."""
    x, q, c, rng = _small(60)
    ids = np.arange(len(x), dtype=np.int64) * 3 + 1
    ids[100] = ids[7]  # one id carried by two rows: both go
    ix = oracle.Index(c, metric)
    ix.build(x, ids)
    gone = np.concatenate([ids[rng.permutation(len(x))[:200]], [ids[7], 10 ** 12]])  # + an id nobody has
    keep = ~np.isin(ids, gone)
    before = ix.list_lengths().sum()
    assert ix.delete(gone) == int((~keep).sum()) and ix.ntotal == int(keep.sum())
    assert ix.list_lengths().sum() == before - int((~keep).sum())
    assert ix.delete(gone) == 0
    got_i, got_v = ix.search(q, 25, ix.nlist)
    want_i, want_v = _numpy_exact(x[keep], ids[keep], q, 25, metric)
    assert np.array_equal(got_i, want_i)
    np.testing.assert_allclose(got_v, want_v, rtol=1e-12, atol=1e-12)
    # update: the deleted row comes back under its old id with a new vector
    new = q[:1].copy()
    ix.insert(new, np.array([ids[7]]))
    i2, v2 = ix.search(new, 1, ix.nlist)
    assert i2[0, 0] == ids[7]
    # deleting everything leaves empty lists and padded results
    assert ix.delete(ids) + ix.delete(np.array([ids[7]])) >= int(keep.sum())
    i3, _ = ix.search(q, 3, ix.nlist)
    assert ix.ntotal == 0 and np.all(i3 == -1)


def test_split_separates_two_blobs_and_leaves_the_rest_alone():
    """IVF-Split on a list that holds two well-separated blobs: the closed-form outcome is the blobs
    themselves, centroids their means; short lists are untouched; nothing is lost; exact search over
    all lists is unchanged."""
    rng = np.random.default_rng(70)
    d = 8
    a = rng.normal(0.0, 0.05, (300, d)).astype(np.float32) + 5.0
    b = rng.normal(0.0, 0.05, (200, d)).astype(np.float32) - 5.0
    far = rng.normal(0.0, 0.05, (40, d)).astype(np.float32) + np.float32(40.0)
    x = np.concatenate([a, b, far])
    order = rng.permutation(len(x))
    x, tag = x[order], np.concatenate([np.zeros(300), np.ones(200), np.full(40, 2)])[order]
    cent = np.stack([np.zeros(d, np.float32), np.full(d, 40.0, np.float32)])  # list 0 gets both blobs
    ix = oracle.Index(cent, oracle.L2)
    ix.build(x)
    assert list(ix.list_lengths()) == [500, 40]
    q = rng.normal(0.0, 3.0, (20, d)).astype(np.float32)
    before = ix.search(q, 15, 2)
    assert ix.split(100, 5) == 1 and ix.nlist == 3 and ix.ntotal == 540
    ids0, ids2 = set(ix.list_ids(0).tolist()), set(ix.list_ids(2).tolist())
    blob_a, blob_b = set(np.nonzero(tag == 0)[0].tolist()), set(np.nonzero(tag == 1)[0].tolist())
    assert {frozenset(ids0), frozenset(ids2)} == {frozenset(blob_a), frozenset(blob_b)}
    assert set(ix.list_ids(1).tolist()) == set(np.nonzero(tag == 2)[0].tolist())
    c = ix.centroids()
    for l, members in ((0, ids0), (2, ids2)):
        np.testing.assert_allclose(c[l], x[sorted(members)].astype(np.float64).mean(0), rtol=1e-6)
    np.testing.assert_array_equal(c[1], cent[1])
    # the side that holds the smallest id stays in the old list; storage order is kept
    assert min(ids0) == 0 and list(ix.list_ids(0)) == sorted(ids0) and list(ix.list_ids(2)) == sorted(ids2)
    after = ix.search(q, 15, 3)
    assert np.array_equal(before[0], after[0]) and np.array_equal(before[1], after[1])
    assert ix.split(100, 5) == 2 and ix.nlist == 5  # both blobs are still over the threshold and split again
    assert ix.split(1000, 5) == 0 and ix.nlist == 5 and ix.ntotal == 540


@pytest.mark.parametrize("metric", [oracle.IP, oracle.L2])
def test_short_rows_are_padded(metric):
    x, q, c, _ = _small(11, n=30, nlist=6)
    ix = oracle.Index(c, metric)
    ix.build(x)
    ids, val = ix.search(q, 50, 2)
    lens = ix.list_lengths()
    probes = ix.coarse(q, 2)
    pad = -np.inf if metric == oracle.IP else np.inf
    for i in range(q.shape[0]):
        n = int(lens[probes[i]].sum())
        assert np.all(ids[i, :n] >= 0) and np.all(ids[i, n:] == -1) and np.all(val[i, n:] == pad)
        members = np.concatenate([ix.list_ids(j) for j in probes[i]])
        assert set(ids[i, :n].tolist()) == set(members.tolist())  # every hit lies in a probed list


def test_scan_probes_with_forced_lists_matches_search():
    x, q, c, _ = _small(12)
    ix = oracle.Index(c, oracle.L2)
    ix.build(x)
    p = ix.coarse(q, 3)
    a, b = ix.scan_probes(q, 9, p), ix.search(q, 9, 3)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    # probe order is irrelevant to the result
    a2 = ix.scan_probes(q, 9, p[:, ::-1].copy())
    assert np.array_equal(a2[0], b[0]) and np.array_equal(a2[1], b[1])


def test_recall_on_tiny_config_is_high():
    """Config 1 recipe end to end on the oracle: recall@10 at nprobe = 8 of 64."""
    cfg = W.scaled(W.C1, n=8000)
    x = W.vectors(cfg, 0, cfg.n)
    cent = training.train_centroids(cfg, x)
    ix = oracle.Index(cent, oracle.IP)
    ix.build(x)
    q = W.queries(cfg, 0, 64)
    ids, _ = ix.search(q, 10, cfg.nprobe)
    bi, _ = oracle.bruteforce(x, q, 10, oracle.IP)
    rec = np.mean([len(set(a.tolist()) & set(b.tolist())) for a, b in zip(ids, bi)]) / 10
    assert rec >= 0.9


def test_level_cascade_worked_example_on_a_line():
    """Early termination (Section 4.2) on numbers one can check by hand.  Points on a line, L2 metric,
    one list per index.  Top level: {0, 1, 2}; bottom level: {0, 1, 2, 10, 11, 12, 2.4}.  k = 2."""
    def index(points, ids):
        ix = oracle.Index(np.zeros((1, 1), np.float32), oracle.L2)
        ix.build(np.asarray(points, np.float32).reshape(-1, 1), np.asarray(ids, np.int64))
        return ix
    top = index([0, 1, 2], [0, 1, 2])
    bottom = index([0, 1, 2, 10, 11, 12, 2.4], [0, 1, 2, 10, 11, 12, 24])
    q = np.asarray([[0.5], [2.2], [10.5], [0.5]], np.float32)
    # squared distances to the top level's best two: 0.25, 0.25 | 0.04, 1.44 | 72.25, 90.25 | 0.25, 0.25
    stop = np.asarray([1.0, 1.0, 1.0, 0.25])
    level, ids, val = oracle.search_levels([top, bottom], q, 2, [1, 1], stop)
    # query 0: both under 1.0 -> stops at the top.  Query 1: the second (1.44) is not under 1.0 -> bottom
    # level, where 2.4 (id 24) beats 1.  Query 2: far from the top level -> bottom.  Query 3: 0.25 is
    # not smaller than 0.25 -> bottom (same two points there).
    assert level.tolist() == [0, 1, 1, 1]
    assert ids.tolist() == [[0, 1], [2, 24], [10, 11], [0, 1]]
    np.testing.assert_allclose(val, [[0.25, 0.25], [0.04, 0.04], [0.25, 0.25], [0.25, 0.25]], atol=1e-6)
    # a top level with fewer than k points never ends a search
    tiny = index([0.5], [7])
    level, ids, _ = oracle.search_levels([tiny, bottom], q[:1], 2, [1, 1], [100.0])
    assert level.tolist() == [1] and ids.tolist() == [[0, 1]]


@pytest.mark.parametrize("metric", [oracle.IP, oracle.L2])
def test_level_cascade_limits_reduce_to_plain_searches(metric):
    """A threshold nothing passes -> the bottom level's search; a threshold everything passes -> the top
    level's; in between every query carries the result of the level it stopped at, and a query stops at
    the top exactly when its k-th value there beats the threshold."""
    x, q, c, _ = _small(21, n=600, nlist=8)
    bottom = oracle.Index(c, metric)
    bottom.build(x)
    sub = np.arange(0, 600, 3)
    top = oracle.Index(c[:4].copy(), metric)
    top.build(x[sub], sub.astype(np.int64))
    k = 5
    ti, tv = top.search(q, k, 2)
    bi, bv = bottom.search(q, k, 3)
    never = np.full(len(q), np.inf if metric == oracle.IP else -np.inf)
    always = -never
    lv, ids, val = oracle.search_levels([top, bottom], q, k, [2, 3], never)
    assert np.all(lv == 1) and np.array_equal(ids, bi) and np.array_equal(val, bv)
    lv, ids, val = oracle.search_levels([top, bottom], q, k, [2, 3], always)
    assert np.all(lv == 0) and np.array_equal(ids, ti) and np.array_equal(val, tv)
    stop = np.full(len(q), np.median(tv[:, k - 1]))
    lv, ids, val = oracle.search_levels([top, bottom], q, k, [2, 3], stop)
    beats = tv[:, k - 1] > stop if metric == oracle.IP else tv[:, k - 1] < stop
    assert np.array_equal(lv == 0, beats) and 0 < beats.sum() < len(q)
    for i in range(len(q)):
        ref = (ti, tv) if lv[i] == 0 else (bi, bv)
        assert np.array_equal(ids[i], ref[0][i]) and np.array_equal(val[i], ref[1][i])

