"""Pins the oracle's neighbour table (Algorithm 2, precompute part) to brute
force, to exact lattice cases with ties, and to structural properties."""
import numpy as np
import pytest


def _brute(cb, k):
    """All-pairs squared distances with a full sort; self forced first, ties by index."""
    cb = cb.astype(np.float64)
    V = cb.shape[0]
    out = np.empty((V, k), dtype=np.int32)
    for i in range(V):
        D = np.zeros(V)
        for c in range(cb.shape[1]):  # coordinate order, one rounded add at a time
            diff = cb[i, c] - cb[:, c]
            D = D + diff * diff
        idx = np.arange(V)
        order = np.lexsort((idx, D))
        order = order[order != i]
        out[i] = np.concatenate([[i], order[: k - 1]])
    return out


@pytest.mark.parametrize("V,d,k", [(1, 3, 1), (2, 1, 2), (17, 2, 5), (64, 8, 64), (50, 33, 7)])
def test_against_brute_force(oracle_mod, V, d, k):
    rng = np.random.default_rng(V * 100 + d)
    cb = rng.standard_normal((V, d)).astype(np.float32)
    got = oracle_mod.build_knn(cb, k)
    np.testing.assert_array_equal(got, _brute(cb, k))


def test_lattice_ties_and_duplicates(oracle_mod):
    # integer lattice: distances are exact, many exact ties -> lower index first
    xs, ys = np.meshgrid(np.arange(5), np.arange(5), indexing="ij")
    cb = np.stack([xs.ravel(), ys.ravel()], axis=1).astype(np.float32)  # token = 5*x + y
    got = oracle_mod.build_knn(cb, 9)
    np.testing.assert_array_equal(got, _brute(cb, 9))
    centre = 12  # (2,2): four neighbours at distance 1, then four at sqrt(2)
    assert list(got[centre]) == [12, 7, 11, 13, 17, 6, 8, 16, 18]
    # duplicates of a code: self stays first even when a lower-index twin exists
    cb = np.array([[0, 0], [1, 0], [0, 0], [3, 0], [0, 0]], dtype=np.float32)
    got = oracle_mod.build_knn(cb, 5)
    assert list(got[2]) == [2, 0, 4, 1, 3]
    assert list(got[0]) == [0, 2, 4, 1, 3]
    assert list(got[3]) == [3, 1, 0, 2, 4]


def test_structure(oracle_mod):
    rng = np.random.default_rng(11)
    V, d = 200, 8
    cb = rng.standard_normal((V, d)).astype(np.float32)
    cb /= np.linalg.norm(cb, axis=1, keepdims=True)
    big = oracle_mod.build_knn(cb, 60)
    small = oracle_mod.build_knn(cb, 13)
    np.testing.assert_array_equal(big[:, :13], small)            # B_k is a prefix of B_k'
    np.testing.assert_array_equal(big[:, 0], np.arange(V))        # self first
    for i in range(V):
        assert len(set(big[i])) == 60                             # distinct tokens
        D = ((cb[i].astype(np.float64) - cb[big[i]].astype(np.float64)) ** 2).sum(1)
        assert np.all(np.diff(D[1:]) >= 0)                        # increasing distance
        # nothing outside the row is nearer than the row's last entry
        rest = np.setdiff1d(np.arange(V), big[i])
        Dr = ((cb[i].astype(np.float64) - cb[rest].astype(np.float64)) ** 2).sum(1)
        assert Dr.min() >= D[-1]
    # on (nearly) unit-norm codes l2 order is descending dot product: a second, independent route
    dots = cb.astype(np.float64) @ cb.astype(np.float64).T
    agree = 0
    for i in range(V):
        order = np.argsort(-dots[i], kind="stable")
        order = order[order != i][:59]
        agree += int(np.array_equal(order, big[i, 1:]))
    assert agree >= V - 3  # norms are 1 only to fp32 rounding, so a rare near-tie may swap
    # rows can be computed in slices and by several threads with identical results
    part = oracle_mod.build_knn(cb, 60, rows=(50, 90), threads=3)
    np.testing.assert_array_equal(part, big[50:90])


def test_cosine_metric(oracle_mod):
    rng = np.random.default_rng(12)
    V, d = 80, 6
    cb = rng.standard_normal((V, d)).astype(np.float32) * rng.uniform(0.2, 5, (V, 1)).astype(np.float32)
    got = oracle_mod.build_knn(cb, 10, metric="cosine")
    c64 = cb.astype(np.float64)
    cosm = (c64 @ c64.T) / np.outer(np.linalg.norm(c64, axis=1), np.linalg.norm(c64, axis=1))
    for i in range(V):
        order = np.argsort(-cosm[i], kind="stable")
        order = order[order != i][:9]
        assert got[i, 0] == i
        np.testing.assert_array_equal(got[i, 1:], order)
    # unit-norm codebook: cosine and l2 give the same table (Section 5.3.1 compares them)
    unit = cb / np.linalg.norm(cb, axis=1, keepdims=True)
    a = oracle_mod.build_knn(unit, 10, metric="cosine")
    b = oracle_mod.build_knn(unit, 10, metric="l2")
    assert (a == b).mean() > 0.98


def test_cosine_with_codes_of_zero_norm(oracle_mod):
    """The cosine with a code of zero norm does not exist (0/0).  The reading taken: such a pair is the
    farthest possible (key +infinity), equal keys by the lower index (Section 5.3.1 does not treat it).
    Checked against a ranking built here from the finite similarities alone."""
    rng = np.random.default_rng(31)
    V, d = 40, 3
    cb = rng.standard_normal((V, d)).astype(np.float32)
    zeros = [5, 17, 39]
    cb[zeros] = 0.0
    got = oracle_mod.build_knn(cb, V, metric="cosine", threads=3)
    c64 = cb.astype(np.float64)
    nrm = np.linalg.norm(c64, axis=1)
    for i in range(V):
        assert got[i, 0] == i
        if i in zeros:   # no similarity to anything: every other token, by index
            want = [j for j in range(V) if j != i]
        else:
            live = [j for j in range(V) if j != i and j not in zeros]
            cos = {j: float(c64[i] @ c64[j]) / (nrm[i] * nrm[j]) for j in live}
            want = sorted(live, key=lambda j: (-cos[j], j)) + [j for j in zeros]
        np.testing.assert_array_equal(got[i, 1:], want)
    # the same reading for a key that is not a number under squared l2 (an infinite coordinate: inf - inf)
    cb2 = rng.standard_normal((12, 2)).astype(np.float32)
    cb2[4, 0] = np.inf
    cb2[9, 0] = np.inf
    got2 = oracle_mod.build_knn(cb2, 12, metric="l2")
    for i in range(12):
        if i in (4, 9):
            np.testing.assert_array_equal(got2[i, 1:], [j for j in range(12) if j != i])   # all keys inf or NaN
        else:
            np.testing.assert_array_equal(sorted(got2[i, -2:]), [4, 9])                      # the two at infinity last
            assert list(got2[i, -2:]) == [4, 9]


def test_bad_arguments(oracle_mod):
    cb = np.zeros((4, 2), dtype=np.float32)
    for k in (0, 5):
        with pytest.raises(ValueError):
            oracle_mod.build_knn(cb, k)
