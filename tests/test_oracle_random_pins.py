"""Pins the oracle's random neighbourhood table (Section 5.3.1 / Table 3, random selection): its
generator against published vectors and an independent implementation, the table against an
independent ordering of the same keys, and the sample against what uniformity implies."""
import numpy as np

from synth import philox


def test_philox_known_answers(oracle_mod):
    # Random123 known-answer vectors for philox4x32-10
    out = oracle_mod.philox4x32_10([0, 0, 0, 0], [0, 0])
    assert [hex(v) for v in out] == ["0x6627e8d5", "0xe169c58d", "0xbc57ac4c", "0x9b00dbd8"]
    out = oracle_mod.philox4x32_10([0xFFFFFFFF] * 4, [0xFFFFFFFF] * 2)
    assert [hex(v) for v in out] == ["0x408f276d", "0x41c83b0e", "0xa20bc7c6", "0x6d5451fd"]


def test_philox_against_numpy_implementation(oracle_mod):
    rng = np.random.default_rng(0)
    for _ in range(50):
        ctr = rng.integers(0, 2 ** 32, 4, dtype=np.uint64).astype(np.uint32)
        key = rng.integers(0, 2 ** 32, 2, dtype=np.uint64).astype(np.uint32)
        want = philox.philox4x32_10(ctr[None, :], (int(key[0]), int(key[1])))[0]
        np.testing.assert_array_equal(oracle_mod.philox4x32_10(ctr, key), want)


def _keys_numpy(V, x, seed):
    ctr = np.zeros(((V + 3) // 4, 4), dtype=np.uint32)
    ctr[:, 0] = np.arange((V + 3) // 4, dtype=np.uint32)
    ctr[:, 1] = x
    return philox.philox4x32_10(ctr, (seed & 0xFFFFFFFF, seed >> 32)).reshape(-1)[:V]


def test_rows_follow_the_key_order(oracle_mod):
    """Row x = x, then the other tokens by increasing (key, token), keys from the numpy generator."""
    seed = 0x1234567890ABCDEF
    for V, k in ((5, 5), (17, 4), (1000, 100), (4099, 1000)):
        table = oracle_mod.build_random(V, k, seed)
        for x in (0, 1, V // 2, V - 1):
            keys = _keys_numpy(V, x, seed).astype(np.int64)
            order = np.lexsort((np.arange(V), keys))
            order = order[order != x][: k - 1]
            assert table[x, 0] == x
            np.testing.assert_array_equal(table[x, 1:], order)


def test_structure_and_prefix_property(oracle_mod):
    V, seed = 2048, 77
    big = oracle_mod.build_random(V, 300, seed)
    assert (big[:, 0] == np.arange(V)).all()
    assert all(len(set(r.tolist())) == 300 for r in big)             # no token twice, none equal to x again
    assert big.min() >= 0 and big.max() < V
    small = oracle_mod.build_random(V, 40, seed)
    np.testing.assert_array_equal(small, big[:, :40])                # same keys: a prefix
    np.testing.assert_array_equal(oracle_mod.build_random(V, 300, seed, rows=(100, 140)), big[100:140])
    other = oracle_mod.build_random(V, 300, seed + 1)
    assert (other[:, 1:] != big[:, 1:]).mean() > 0.99                # another seed, another table
    full = oracle_mod.build_random(64, 64, 3)
    assert all(sorted(r.tolist()) == list(range(64)) for r in full)  # k = V: a permutation of all tokens


def test_sample_is_uniform(oracle_mod):
    """Each other token appears in a row with probability (k-1)/(V-1), at a uniform position."""
    V, k = 512, 65
    table = oracle_mod.build_random(V, k, seed=2024)
    member = np.zeros((V, V), dtype=np.int64)
    member[np.repeat(np.arange(V), k - 1), table[:, 1:].reshape(-1)] = 1
    per_token = member.sum(axis=0)                                   # rows that list token y
    p = (k - 1) / (V - 1)
    expect, sd = (V - 1) * p, np.sqrt((V - 1) * p * (1 - p))
    assert abs(per_token.mean() - expect) < 1e-9                     # V*(k-1) entries in all
    assert np.abs(per_token - expect).max() < 5.5 * sd
    chi2 = (((per_token - expect) ** 2) / (expect * (1 - p))).sum()  # ~ chi-square with about V degrees
    assert abs(chi2 - V) < 5 * np.sqrt(2 * V)
    # neighbour identities carry no information about the token: mean circular offset is flat
    offset = (table[:, 1:] - table[:, :1]) % V
    hist = np.bincount(offset.reshape(-1) * 8 // V, minlength=8)
    assert np.abs(hist / hist.sum() - 0.125).max() < 0.01
    # position in the row is independent of the token value: first and second half look alike
    first, second = table[:, 1:33].mean(), table[:, 33:].mean()
    assert abs(first - second) < 6 * (V / np.sqrt(12)) / np.sqrt(V * 32) * np.sqrt(2)
