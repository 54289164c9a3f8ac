"""Comparator for search results: HIP path against the CPU oracle.

Rule:
  * values: |g - r| <= tol * max(|r|, scale) position by position, where scale is
    ||q||*||x|| for inner product and ||q||^2 + ||x||^2 for squared L2 (a purely
    relative test is meaningless at the self-match value 0);
  * ids: position j must hold the oracle's j-th id, unless another candidate's
    oracle value lies within the tolerance of the oracle's j-th value -- then that
    candidate is accepted too (the oracle row is extended past k so that such
    candidates can be looked up); no id may repeat.  So ids are exact wherever
    the value gap exceeds the tolerance, at position k and everywhere else;
  * candidates with exactly equal GPU values must come in ascending id order;
  * padding (id -1, value -inf / +inf) must agree exactly.
"""
from __future__ import annotations

import numpy as np

IP, L2 = 0, 1


def _tol_at(v, tol, scale):
    return tol * max(abs(v), scale)


def check_row(ids_g, val_g, ids_o, val_o, k, tol, scale, metric, where=""):
    """ids_o/val_o: oracle row of length kx >= k, best first.  Raises AssertionError."""
    ids_g = np.asarray(ids_g)
    val_g = np.asarray(val_g, dtype=np.float64)
    ids_o = np.asarray(ids_o)
    val_o = np.asarray(val_o, dtype=np.float64)
    kx = len(ids_o)
    assert len(ids_g) == k and kx >= k
    n_valid = int(np.sum(ids_o >= 0))  # oracle pads at the end only
    pad_val = -np.inf if metric == IP else np.inf
    exact = 0
    # padding
    for j in range(min(k, kx)):
        if ids_o[j] < 0:
            assert ids_g[j] == -1, f"{where} pos {j}: expected padding id -1, got {ids_g[j]}"
            assert val_g[j] == pad_val, f"{where} pos {j}: expected padding value {pad_val}, got {val_g[j]}"
    kk = min(k, n_valid)
    # values, position by position
    for j in range(kk):
        assert ids_g[j] >= 0, f"{where} pos {j}: GPU padded but oracle has id {ids_o[j]}"
        err = abs(val_g[j] - val_o[j])
        assert err <= _tol_at(val_o[j], tol, scale), (
            f"{where} pos {j}: value {val_g[j]!r} vs oracle {val_o[j]!r} (err {err:.3e}, tol {tol})")
    # order of GPU row: non-worsening, equal values by ascending id, no repeats
    for j in range(1, kk):
        if metric == IP:
            assert val_g[j] <= val_g[j - 1], f"{where} pos {j}: GPU row not sorted"
        else:
            assert val_g[j] >= val_g[j - 1], f"{where} pos {j}: GPU row not sorted"
        if val_g[j] == val_g[j - 1]:
            assert ids_g[j] > ids_g[j - 1], f"{where} pos {j}: equal values not in ascending id order"
    assert len(set(ids_g[:kk].tolist())) == kk, f"{where}: repeated id in GPU row"
    # ids: exact, or a candidate whose oracle value is within tolerance of the j-th oracle value
    where_o = {int(v): i for i, v in enumerate(ids_o[:n_valid].tolist())}
    for j in range(kk):
        if ids_g[j] == ids_o[j]:
            exact += 1
            continue
        tolj = _tol_at(val_o[j], tol, scale)
        pos = where_o.get(int(ids_g[j]))
        if pos is None:
            assert n_valid == kx and abs(val_o[kx - 1] - val_o[j]) <= tolj, (
                f"{where} pos {j}: id {ids_g[j]} is not among the oracle's {n_valid} best "
                f"(oracle has {ids_o[j]} with value {val_o[j]!r})")
            raise AssertionError(f"{where} pos {j}: near-tie run reaches past the oracle's extended row; raise kx")
        assert abs(val_o[pos] - val_o[j]) <= tolj, (
            f"{where} pos {j}: id {ids_g[j]} (oracle value {val_o[pos]!r}, oracle rank {pos}) where the oracle "
            f"has id {ids_o[j]} (value {val_o[j]!r}); gap exceeds the tolerance")
    return exact


def check_results(ids_g, val_g, ids_o, val_o, k, tol, scale, metric, where=""):
    """Row-wise check_row over a batch.  scale: scalar or per-query array."""
    nq = len(ids_g)
    scale = np.broadcast_to(np.asarray(scale, dtype=np.float64), (nq,))
    exact = 0
    for i in range(nq):
        exact += check_row(ids_g[i], val_g[i], ids_o[i], val_o[i], k, tol, float(scale[i]), metric,
                           where=f"{where} query {i}")
    return exact


def check_probes(probes_g, probes_o_ext, scores_o, nprobe, tol, scale, where=""):
    """Coarse step: probe lists exact wherever the score gaps exceed the tolerance.
    probes_o_ext: oracle ranking of lists (length >= nprobe, ideally all nlist);
    scores_o: oracle scores indexed by list number."""
    for i in range(len(probes_g)):
        ids_o = probes_o_ext[i]
        check_row_ids_only(probes_g[i], ids_o, scores_o[i][ids_o], nprobe, tol, scale, where=f"{where} query {i}")


def check_row_ids_only(ids_g, ids_o, val_o, k, tol, scale, where=""):
    """The id rule of check_row without GPU values (probe lists, assignments).  ids_o / val_o: the
    oracle's full ranking and the values in that order."""
    ids_g = np.asarray(ids_g)
    assert len(set(ids_g.tolist())) == len(ids_g), f"{where}: repeated id"
    where_o = {int(v): i for i, v in enumerate(np.asarray(ids_o).tolist())}
    for j in range(k):
        if ids_g[j] == ids_o[j]:
            continue
        pos = where_o.get(int(ids_g[j]))
        assert pos is not None, f"{where} pos {j}: id {ids_g[j]} unknown to the oracle"
        assert abs(val_o[pos] - val_o[j]) <= _tol_at(val_o[j], tol, scale), (
            f"{where} pos {j}: {ids_g[j]} (oracle value {val_o[pos]!r}, rank {pos}) vs oracle {ids_o[j]} "
            f"(value {val_o[j]!r}); gap exceeds the tolerance")


def recall_at(ids_found, ids_true, k):
    hit = 0
    for f, t in zip(ids_found, ids_true):
        hit += len(set(f[:k].tolist()) & set(t[:k].tolist()))
    return hit / (k * len(ids_found))
