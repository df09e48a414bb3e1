"""Pins the oracle's greedy-decoding variant (Section 4.3, last sentence: accept the
draft token iff it is the arg-max of the distorted target)."""
import numpy as np
import scipy.special


def _table_rows(V, k, rng):
    rows = np.empty((V, k), dtype=np.int32)
    for x in range(V):
        others = rng.permutation(np.delete(np.arange(V), x))[: k - 1]
        rows[x] = np.concatenate([[x], others])
    return rows


def test_hand_derived(oracle_mod):
    # t = [.4,.3,.2,.1], xt = 1, neighbourhood [1,2,0]:
    #  delta=.25: A={1,2}, t_A=[.4,.5,0,.1] -> arg-max is 1 = xt -> accept
    #  delta=0  : A={1},   t_A=t            -> arg-max is 0      -> reject, emit 0
    #  delta=2  : A={1,2,0}, t_A=[0,.9,0,.1] -> accept
    l = np.log(np.array([[.4, .3, .2, .1]])).astype(np.float32)
    table = np.array([[0, 1, 2], [1, 2, 0], [2, 1, 0], [3, 0, 1]], dtype=np.int32)
    for delta, want in ((.25, (1, -1, 2)), (0.0, (0, 0, 1)), (2.0, (1, -1, 3))):
        acc, tok, diag = oracle_mod.verify_greedy(l, [1], table, 3, delta)
        assert (acc[0], tok[0], int(diag["a_size"][0])) == want
    # the walk stops at the first neighbour that does not fit: xt=3 (t=.1), neighbourhood [3,0,1], delta=.35:
    # token 0 (t=.4) does not fit, token 1 (t=.3) is never reached -> t_A = t -> emit 0
    acc, tok, diag = oracle_mod.verify_greedy(l, [3], table, 3, 0.35)
    assert (acc[0], tok[0], int(diag["a_size"][0])) == (0, 0, 1)


def test_equal_logits_take_the_lowest_index(oracle_mod):
    l = np.zeros((4, 4), dtype=np.float32)            # uniform target: every token ties
    table = np.arange(4, dtype=np.int32).reshape(4, 1)
    acc, tok, _ = oracle_mod.verify_greedy(l, [0, 1, 2, 3], table, 1, 0.1)
    assert list(acc) == [1, 0, 0, 0] and list(tok) == [-1, 0, 0, 0]
    # a tie between the draft token and a later token is won by the draft token
    l = np.array([[0.0, 2.0, 1.0, 2.0]], dtype=np.float32)
    acc, tok, _ = oracle_mod.verify_greedy(l, [1], table, 1, 0.1)
    assert (acc[0], tok[0]) == (1, -1)
    acc, tok, _ = oracle_mod.verify_greedy(l, [3], table, 1, 0.1)
    assert (acc[0], tok[0]) == (0, 1)


def test_k1_and_delta0_are_plain_greedy_verification(oracle_mod):
    rng = np.random.default_rng(21)
    N, V = 200, 40
    l = (rng.standard_normal((N, V)) * 2).astype(np.float32)
    tokens = rng.integers(0, V, N).astype(np.int32)
    tokens[::3] = np.argmax(l[::3], axis=1)            # make a third of the drafts correct
    best = np.argmax(l, axis=1)
    for table, k, delta in ((np.arange(V, dtype=np.int32).reshape(V, 1), 1, 0.3),
                            (_table_rows(V, 6, rng), 6, 0.0)):
        acc, tok, diag = oracle_mod.verify_greedy(l, tokens, table, k, delta)
        np.testing.assert_array_equal(acc, (best == tokens).astype(np.int32))
        np.testing.assert_array_equal(tok, np.where(best == tokens, -1, best))
        assert np.all(diag["a_size"] == 1)


def test_agrees_with_the_distorted_target_of_the_sampling_path(oracle_mod):
    """Independent route: the distorted target returned by verify_probs, arg-max by numpy."""
    rng = np.random.default_rng(22)
    V, k = 64, 9
    table = _table_rows(V, k, rng)
    n_acc = 0
    for trial in range(300):
        l = (rng.standard_normal(V) * rng.choice([0.5, 1.5, 3.0])).astype(np.float32)
        xt = int(rng.integers(V)) if trial % 2 else int(np.argsort(-l)[rng.integers(0, 3)])
        delta = float(rng.choice([0.02, 0.1, 0.3, 0.8]))
        t = scipy.special.softmax(l.astype(np.float64))
        ref = oracle_mod.verify_probs(t, t, xt, table[xt], delta, 0.5, 0.5, want_dists=True)
        ta = ref["distorted_target"]
        best = int(np.argmax(ta))
        acc, tok, diag = oracle_mod.verify_greedy(l[None, :], [xt], table, k, delta)
        assert acc[0] == int(best == xt) and tok[0] == (-1 if best == xt else best)
        assert int(diag["a_size"][0]) == ref["a_size"]
        assert abs(diag["mass"][0] - ref["mass"]) < 1e-14
        # the emitted token is never a member of A other than xt
        A = set(int(x) for x in table[xt][: ref["a_size"]]) - {xt}
        assert tok[0] not in A
        n_acc += acc[0]
    assert 20 < n_acc < 280


def test_acceptance_grows_with_k_and_delta(oracle_mod):
    rng = np.random.default_rng(23)
    V = 96
    full = _table_rows(V, V, rng)
    for trial in range(40):
        l = (rng.standard_normal(V) * 1.5).astype(np.float32)[None, :]
        xt = int(np.argsort(-l[0])[rng.integers(0, 5)])
        prev = None
        for delta in (0.0, 0.05, 0.1, 0.2, 0.4, 0.8):
            accs = []
            for k in (1, 2, 5, 17, 64, 96):
                acc, _, _ = oracle_mod.verify_greedy(l, [xt], full[:, :k].copy(), k, delta)
                accs.append(int(acc[0]))
            assert all(b >= a for a, b in zip(accs, accs[1:]))
            if prev is not None:
                assert all(b >= a for a, b in zip(prev, accs))
            prev = accs


def test_unusable_rows(oracle_mod):
    V, k = 16, 4
    rng = np.random.default_rng(24)
    l = rng.standard_normal((4, V)).astype(np.float32)
    table = _table_rows(V, k, rng)
    tokens = np.array([1, V, 2, 3], dtype=np.int32)
    l[2, 5] = np.nan
    l[3, :] = -np.inf
    acc, tok, _ = oracle_mod.verify_greedy(l, tokens, table, k, 0.1)
    assert acc[0] in (0, 1)
    assert list(acc[1:]) == [-1, -1, -1] and list(tok[1:]) == [-1, -1, -1]
