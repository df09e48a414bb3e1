"""Pins the oracle's walk of a drafted chain (Algorithm 1: keep drafts while accepted, exit at the
first rejection with its resampled token, extra token when all were accepted)."""
import numpy as np


def test_hand_cases(oracle_mod):
    L = 4
    accept = np.array([[1, 1, 1, 1],      # all kept -> extra token needed
                       [1, 1, 0, 1],      # two kept, third rejected (a later acceptance is ignored)
                       [0, 1, 1, 1],      # nothing kept
                       [1, -1, 1, 1],     # unusable row ends the chain
                       [1, 1, 1, 0]], dtype=np.int32)
    resample = np.array([[-1, -1, -1, -1],
                         [-1, -1, 77, -1],
                         [5, -1, -1, -1],
                         [-1, -1, -1, -1],
                         [-1, -1, -1, 9]], dtype=np.int32)
    n, nxt = oracle_mod.accept_chains(accept, resample, L)
    assert list(n) == [4, 2, 0, 1, 3]
    assert list(nxt) == [-1, 77, 5, -2, 9]


def test_against_numpy(oracle_mod):
    rng = np.random.default_rng(31)
    for L in (1, 5, 60):
        B = 200
        accept = (rng.random((B, L)) < 0.8).astype(np.int32)
        resample = np.where(accept == 1, -1, rng.integers(0, 1000, (B, L))).astype(np.int32)
        n, nxt = oracle_mod.accept_chains(accept, resample, L)
        first = np.where((accept != 1).any(axis=1), (accept != 1).argmax(axis=1), L)
        np.testing.assert_array_equal(n, first)
        want = np.where(first < L, resample[np.arange(B), np.minimum(first, L - 1)], -1)
        np.testing.assert_array_equal(nxt, want)
        # mean accepted length of an i.i.d. chain: sum_{t=1..L} p^t
        p = 0.8
        assert abs(n.mean() - sum(p ** t for t in range(1, L + 1))) < 0.5
