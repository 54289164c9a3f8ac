"""Comparator for search results: HIP path against the CPU oracle.

Rule (north star + the readings listed in the design doc):
  * values: |g - r| <= tol * max(|r|, scale) position by position, where scale is
    ||q||*||x|| for inner product and ||q||^2 + ||x||^2 for squared L2 (a purely
    relative test is meaningless at the self-match value 0);
  * ids: the oracle row (extended past k) is cut into tie groups -- runs whose
    adjacent values differ by no more than the tolerance.  Inside a group that
    lies wholly in the top k the GPU ids must be a permutation of the oracle's;
    the group straddling position k may contribute any of its members; every
    other position is exact;
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
    # tie groups over the oracle's valid entries
    a = 0
    while a < kk:
        b = a + 1
        while b < n_valid and abs(val_o[b] - val_o[b - 1]) <= _tol_at(val_o[b - 1], tol, scale):
            b += 1
        group = set(ids_o[a:b].tolist())
        if b <= kk:
            got = set(ids_g[a:b].tolist())
            assert got == group, f"{where} pos [{a},{b}): ids {sorted(got)} != oracle group {sorted(group)}"
            if b - a == 1:
                exact += 1
        else:
            # straddles position k: the oracle row must show the whole group
            assert b < kx or n_valid < kx, (
                f"{where}: tie group at the k boundary runs past the oracle's extended row; raise kx")
            got = set(ids_g[a:kk].tolist())
            assert got <= group, f"{where} pos [{a},{kk}): ids {sorted(got - group)} not in boundary tie group"
        a = b
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
    """Tie-group id check without GPU values (used for probe lists and assignments)."""
    ids_g = np.asarray(ids_g)
    n_valid = len(ids_o)
    assert len(set(ids_g.tolist())) == len(ids_g), f"{where}: repeated id"
    a = 0
    while a < k:
        b = a + 1
        while b < n_valid and abs(val_o[b] - val_o[b - 1]) <= _tol_at(val_o[b - 1], tol, scale):
            b += 1
        group = set(np.asarray(ids_o[a:b]).tolist())
        if b <= k:
            got = set(ids_g[a:b].tolist())
            assert got == group, f"{where} pos [{a},{b}): {sorted(got)} != oracle group {sorted(group)}"
        else:
            got = set(ids_g[a:k].tolist())
            assert got <= group, f"{where} pos [{a},{k}): {sorted(got - group)} not in boundary tie group"
        a = b


def recall_at(ids_found, ids_true, k):
    hit = 0
    for f, t in zip(ids_found, ids_true):
        hit += len(set(f[:k].tolist()) & set(t[:k].tolist()))
    return hit / (k * len(ids_found))
