"""Pins of the sequential-residual sibling rule (each sibling of a draft tree is verified against
the residual left by the siblings before it): exact enumeration of the emitted law, reductions to
the single-candidate verification and to the chain walk, hand-worked groups, and the law of the
default rule (every sibling against the undistorted target) for contrast."""
import itertools

import numpy as np
import pytest

from synth import philox


def _self_rows(tokens, V, k):
    """Table rows with the token first and then the next k-1 tokens cyclically."""
    return np.stack([(int(x) + np.arange(k)) % V for x in tokens]).astype(np.int32)


def _emitted_law_sequential(oracle, t, g, m, k, delta):
    """Law of the token that follows a node whose m children were drawn independently from g:
    sum over all child tuples of prod g(x_i) * [ sum_j prod_{i<j}(1 - a_i) a_j 1{y = x_j}
    + prod_i (1 - a_i) t_{m+1}(y) ], with a_j and t_{m+1} from the oracle."""
    V = len(t)
    law = np.zeros(V)
    for xs in itertools.product(range(V), repeat=m):
        w = float(np.prod([g[x] for x in xs]))
        if w == 0.0:
            continue
        r = oracle.sibling_group_probs(t, g, xs, _self_rows(xs, V, k), delta, [0.0] * m, [0.0] * m)
        stay = 1.0
        for j, x in enumerate(xs):
            law[x] += w * stay * r["accept_prob"][j]
            stay *= 1.0 - r["accept_prob"][j]
        law += w * stay * r["final_dist"]
    return law


def _emitted_law_independent(oracle, t, g, m):
    """The same for the default tree rule at k = 1: every sibling is tested against the undistorted
    target; when all fail the token is drawn from the first child's residual."""
    V = len(t)
    law = np.zeros(V)
    for xs in itertools.product(range(V), repeat=m):
        w = float(np.prod([g[x] for x in xs]))
        stay = 1.0
        first = oracle.verify_probs(t, g, xs[0], [xs[0]], 0.0, 0.0, 0.0, want_dists=True)
        for x in xs:
            a = min(1.0, t[x] / g[x])
            law[x] += w * stay * a
            stay *= 1.0 - a
        law += w * stay * first["residual"]
    return law


@pytest.mark.parametrize("V,m", [(3, 2), (4, 2), (4, 3), (5, 3), (4, 4)])
def test_emitted_law_equals_target_at_k1(oracle_mod, V, m):
    """Standard speculative sampling keeps the target law (Section 2); with k = 1 the relaxed rule is
    the standard one, and the sequential-residual rule must keep the law for any number of siblings."""
    rng = np.random.default_rng(100 * V + m)
    t = rng.dirichlet(np.ones(V) * 0.7)
    g = rng.dirichlet(np.ones(V) * 0.7)
    law = _emitted_law_sequential(oracle_mod, t, g, m, k=1, delta=0.3)
    np.testing.assert_allclose(law, t, atol=1e-12)
    law0 = _emitted_law_sequential(oracle_mod, t, g, m, k=min(3, V), delta=0.0)   # delta = 0: A is the token alone
    np.testing.assert_allclose(law0, t, atol=1e-12)


def test_default_rule_does_not_keep_the_law_with_siblings(oracle_mod):
    """The contrast that the header states: with two children per node the default rule's emitted law
    differs from t even at k = 1 (with one child it is t)."""
    rng = np.random.default_rng(7)
    t = rng.dirichlet(np.ones(4))
    g = rng.dirichlet(np.ones(4))
    np.testing.assert_allclose(_emitted_law_independent(oracle_mod, t, g, 1), t, atol=1e-12)
    assert np.abs(_emitted_law_independent(oracle_mod, t, g, 2) - t).max() > 1e-3
    np.testing.assert_allclose(_emitted_law_sequential(oracle_mod, t, g, 2, 1, 0.0), t, atol=1e-12)


def test_relaxed_law_is_a_distribution_and_moves_mass_only_within_neighbourhoods(oracle_mod):
    """k > 1, delta > 0: the emitted law still sums to one; it is no longer t (that is the method)."""
    rng = np.random.default_rng(3)
    V = 5
    t = rng.dirichlet(np.ones(V))
    g = rng.dirichlet(np.ones(V))
    law = _emitted_law_sequential(oracle_mod, t, g, 2, k=3, delta=0.2)
    assert law.min() >= 0 and law.sum() == pytest.approx(1.0, abs=1e-12)
    assert np.abs(law - t).max() > 1e-6


def test_hand_worked_group(oracle_mod):
    """t = [.5,.3,.2], g = [.2,.2,.6], siblings 2 then 0, k = 1.
    Sibling 2: accept prob min(1, .2/.6) = 1/3; residual max(0, t - g) = [.3,.1,0] / .4 = [.75,.25,0].
    Sibling 0 against [.75,.25,0]: accept prob min(1, .75/.2) = 1; its residual would be
    max(0, [.75,.25,0] - g) = [.55,.05,0] / .6."""
    t, g = [0.5, 0.3, 0.2], [0.2, 0.2, 0.6]
    rows = np.array([[2], [0]], dtype=np.int32)
    r = oracle_mod.sibling_group_probs(t, g, [2, 0], rows, 0.0, [0.9, 0.99], [0.5, 0.5])
    np.testing.assert_allclose(r["accept_prob"], [1 / 3, 1.0], atol=1e-15)
    assert r["taken"] == 1 and r["next"] == -1
    np.testing.assert_allclose(r["final_dist"], [0.55 / 0.6, 0.05 / 0.6, 0.0], atol=1e-15)
    r = oracle_mod.sibling_group_probs(t, g, [2, 0], rows, 0.0, [0.2, 0.99], [0.5, 0.5])
    assert r["taken"] == 0                                       # 0.2 * 0.6 < 0.2
    # both rejected is impossible here (second accept prob 1); with siblings 2, 2 it is not:
    rows22 = np.array([[2], [2]], dtype=np.int32)
    r = oracle_mod.sibling_group_probs(t, g, [2, 2], rows22, 0.0, [0.9, 0.5], [0.5, 0.8])
    np.testing.assert_allclose(r["accept_prob"], [1 / 3, 0.0], atol=1e-15)   # the residual gives token 2 no mass
    assert r["taken"] == -1
    # second residual: max(0, [.75,.25,0] - [.2,.2,.6]) = [.55,.05,0]/.6; u_res = .8 -> .48 of .6 -> token 0
    assert r["next"] == 0
    np.testing.assert_allclose(r["final_dist"], [0.55 / 0.6, 0.05 / 0.6, 0.0], atol=1e-15)
    r = oracle_mod.sibling_group_probs(t, g, [2, 2], rows22, 0.0, [0.9, 0.5], [0.5, 0.95])
    assert r["next"] == 1                                        # .57 of .6 lies beyond .55


def test_single_sibling_is_the_plain_verification(oracle_mod):
    rng = np.random.default_rng(11)
    V, k = 12, 4
    for _ in range(30):
        t = rng.dirichlet(np.ones(V) * 0.5)
        g = rng.dirichlet(np.ones(V) * 0.5)
        x = int(rng.integers(0, V))
        row = np.concatenate([[x], (x + 1 + rng.permutation(V - 1)[: k - 1]) % V]).astype(np.int32)
        ua, ur = float(rng.random()), float(rng.random())
        one = oracle_mod.verify_probs(t, g, x, row, 0.15, ua, ur, want_dists=True)
        grp = oracle_mod.sibling_group_probs(t, g, [x], row[None, :], 0.15, [ua], [ur])
        assert grp["accept_prob"][0] == one["accept_prob"]
        assert (grp["taken"] == 0) == (one["accept"] == 1)
        assert grp["next"] == one["resample"]
        np.testing.assert_array_equal(grp["final_dist"], one["residual"])


def _random_tree_inputs(rng, B, M, V, k, max_children=3):
    from synth.trees import random_trees
    parent = random_trees(rng, B, M, max_children=max_children)
    R = B * (M + 1)
    tl = (rng.standard_normal((R, V)) * 2.0).astype(np.float32)
    dl = (tl + rng.standard_normal((R, V))).astype(np.float32)
    row_index = (np.arange(B)[:, None] * (M + 1) + parent + 1).astype(np.int32).reshape(-1)
    tokens = rng.integers(0, V, B * M).astype(np.int32)
    table = np.stack([np.concatenate([[x], (x + 1 + rng.permutation(V - 1)[: k - 1]) % V]) for x in range(V)]).astype(np.int32)
    un = philox.uniforms(int(rng.integers(1, 1 << 30)), B * M)
    return parent, tl, dl, row_index, tokens, table, un


def test_tree_walk_matches_group_by_group_evaluation(oracle_mod):
    """The logits-level walk against a re-derivation in Python from the probability-level group
    function, and its invariants: the path is a branch, chains reduce to the chain walk."""
    rng = np.random.default_rng(5)
    B, M, V, k = 12, 14, 40, 5
    parent, tl, dl, row_index, tokens, table, un = _random_tree_inputs(rng, B, M, V, k)
    delta = 0.1
    n, path, nxt = oracle_mod.verify_trees_sequential(tl, dl, row_index, parent, M, tokens, table, k, delta, un, threads=2)
    d32 = float(np.float32(delta))
    for b in range(B):
        node, want_path = -1, []
        while True:
            kids = [i for i in range(M) if parent[b, i] == node]
            if not kids:
                want_next = -1
                break
            c = [b * M + i for i in kids]
            r = row_index[c[0]]
            grp = oracle_mod.sibling_group_probs(oracle_mod.softmax(tl[r]), oracle_mod.softmax(dl[r]), tokens[c],
                                                 table[tokens[c]], d32, un[c, 0], un[c, 1], want_final=False)
            if grp["taken"] >= 0:
                node = kids[grp["taken"]]
                want_path.append(node)
                continue
            want_next = grp["next"]
            break
        assert n[b] == len(want_path) and list(path[b, : n[b]]) == want_path and np.all(path[b, n[b]:] == -1)
        assert nxt[b] == want_next
        for a, c in zip([-1] + want_path[:-1], want_path):
            assert parent[b, c] == a


def test_chains_reduce_to_the_chain_walk(oracle_mod):
    """One child per node: the sequential rule is Algorithm 1's loop, the same as the default rule."""
    rng = np.random.default_rng(9)
    B, M, V, k = 10, 6, 30, 4
    parent = np.tile(np.arange(-1, M - 1, dtype=np.int32), (B, 1))
    _, tl, dl, row_index, tokens, table, un = _random_tree_inputs(rng, B, M, V, k)
    row_index = (np.arange(B)[:, None] * (M + 1) + parent + 1).astype(np.int32).reshape(-1)
    n, path, nxt = oracle_mod.verify_trees_sequential(tl, dl, row_index, parent, M, tokens, table, k, 0.05, un)
    acc, res, _ = oracle_mod.verify_rows(tl, dl, row_index, tokens, table, k, 0.05, un)
    n2, path2, nxt2 = oracle_mod.accept_trees(acc, res, parent, M)
    np.testing.assert_array_equal(n, n2)
    np.testing.assert_array_equal(path, path2)
    np.testing.assert_array_equal(nxt, nxt2)


def test_unusable_and_malformed(oracle_mod):
    rng = np.random.default_rng(13)
    B, M, V, k = 4, 5, 20, 3
    parent = np.array([[-1, -1, 0, 0, 2]] * B, dtype=np.int32)
    _, tl, dl, row_index, tokens, table, un = _random_tree_inputs(rng, B, M, V, k)
    row_index = (np.arange(B)[:, None] * (M + 1) + parent + 1).astype(np.int32).reshape(-1)
    un[:, 0] = np.float32(1 - 2.0 ** -24)
    for b in (0, 1):                              # the first root child is certainly rejected: the second gets tried
        r, x = row_index[b * M], tokens[b * M]
        dl[r, x] += 20.0
        tl[r, x] -= 5.0
    tokens[0 * M + 1] = V                         # tree 0: second root child unusable
    row_index[1 * M + 1] = row_index[1 * M + 0] + 1   # tree 1: sibling on other rows
    parent[2, 3] = 4                              # tree 2: malformed
    tl[row_index[3 * M + 0], 3] = np.nan          # tree 3: unusable logits
    n, path, nxt = oracle_mod.verify_trees_sequential(tl, dl, row_index, parent, M, tokens, table, k, 0.0, un)
    assert list(nxt) == [-2, -2, -3, -2] and list(n) == [0, 0, 0, 0]
