"""Pins the oracle's Jensen-Shannon-bounded neighbourhood (ablation of Section 5.3.2: the bound on
the divergence between the distorted target and the target, with JSD in place of TVD)."""
import numpy as np
import pytest
import scipy.spatial.distance
import scipy.special


def _nbrs(rng, V, k, xt):
    others = rng.permutation(np.delete(np.arange(V), xt))[: k - 1]
    return np.concatenate([[xt], others]).astype(np.int32)


def test_prefix_divergence_equals_the_full_vector_definition(oracle_mod):
    """For the prefix the oracle takes, the JSD of the distorted target it returns against the target,
    computed by scipy over the whole vocabulary, is below delta; adding the next neighbour would not be."""
    rng = np.random.default_rng(41)
    V = 80
    seen_cut = 0
    for trial in range(150):
        t = scipy.special.softmax(rng.standard_normal(V) * rng.choice([0.5, 2.0, 4.0]))
        g = scipy.special.softmax(rng.standard_normal(V))
        xt = int(rng.integers(V))
        k = int(rng.integers(1, V + 1))
        nb = _nbrs(rng, V, k, xt)
        delta = float(rng.choice([0.005, 0.02, 0.08, 0.2, 0.6]))
        r = oracle_mod.verify_probs(t, g, xt, nb, delta, 0.5, 0.5, want_dists=True, divergence="jsd")
        a = r["a_size"]
        ta = r["distorted_target"]
        jsd = scipy.spatial.distance.jensenshannon(ta, t) ** 2      # scipy returns the square root, base e
        assert jsd < delta
        assert abs(ta.sum() - 1) < 1e-12
        if a < k:
            seen_cut += 1
            bigger = t.copy()
            A = nb[: a + 1]
            bigger[A] = 0.0
            bigger[xt] = t[A].sum()
            assert scipy.spatial.distance.jensenshannon(bigger, t) ** 2 >= delta - 1e-12
    assert seen_cut > 30


def test_hand_value(oracle_mod):
    # t = [1/2, 1/4, 1/4], xt = 0, neighbourhood [0, 1]: moving 1/4 onto xt gives t_A = [3/4, 0, 1/4];
    # JSD = 1/2 [ 3/4 ln(3/4 / 5/8) + 1/2 ln(1/2 / 5/8) + 1/4 ln 2 ] = 0.0492160...
    want = 0.5 * (0.75 * np.log(0.75 / 0.625) + 0.5 * np.log(0.5 / 0.625) + 0.25 * np.log(2.0))
    t = [0.5, 0.25, 0.25]
    g = [0.2, 0.4, 0.4]
    for delta, a_size in ((want + 1e-9, 2), (want, 1), (want - 1e-9, 1)):   # strict bound
        r = oracle_mod.verify_probs(t, g, 0, [0, 1], delta, 0.5, 0.5, divergence="jsd")
        assert r["a_size"] == a_size


def test_jsd_is_looser_than_tvd_at_equal_delta_and_monotone(oracle_mod):
    """JSD <= ln2 * TVD for this pair of distributions, so at equal delta the JSD neighbourhood is at
    least as large as the TVD one; both grow with delta."""
    rng = np.random.default_rng(42)
    V = 64
    for trial in range(60):
        t = scipy.special.softmax(rng.standard_normal(V) * 2)
        g = scipy.special.softmax(rng.standard_normal(V))
        xt = int(rng.integers(V))
        nb = _nbrs(rng, V, 40, xt)
        prev = 0
        for delta in (0.0, 0.01, 0.05, 0.1, 0.3, 0.69, 0.7):
            a_j = oracle_mod.verify_probs(t, g, xt, nb, delta, 0.5, 0.5, divergence="jsd")["a_size"]
            a_t = oracle_mod.verify_probs(t, g, xt, nb, delta, 0.5, 0.5, divergence="tvd")["a_size"]
            assert a_j >= a_t and a_j >= prev
            prev = a_j
        assert prev == 40    # JSD never exceeds ln 2 < 0.7


def test_logits_path(oracle_mod):
    from synth import philox
    rng = np.random.default_rng(43)
    V, N, k = 120, 40, 15
    tl = (rng.standard_normal((N, V)) * 2).astype(np.float32)
    gl = (tl + rng.standard_normal((N, V))).astype(np.float32)
    tokens = rng.integers(0, V, N).astype(np.int32)
    table = np.stack([_nbrs(rng, V, k, x) for x in range(V)])
    un = philox.uniforms(9, N)
    acc, res, diag = oracle_mod.verify(tl, gl, tokens, table, k, 0.03, un, divergence="jsd")
    for i in range(N):
        t = scipy.special.softmax(tl[i].astype(np.float64))
        g = scipy.special.softmax(gl[i].astype(np.float64))
        r = oracle_mod.verify_probs(t, g, tokens[i], table[tokens[i]], 0.03, un[i, 0], un[i, 1], divergence="jsd")
        assert diag["a_size"][i] == r["a_size"]
        assert diag["accept_prob"][i] == pytest.approx(r["accept_prob"], rel=1e-12)


def test_a_bound_of_zero_takes_no_neighbour(oracle_mod):
    """The divergence is positive as soon as any mass moves, so under a bound of zero the neighbourhood is the
    token alone and the rule is standard speculative acceptance (Section 5.3.2 with Section 2).  When the moved
    mass is around one unit in the last place of t(xt), the two logarithmic terms at xt cancel to their rounding
    errors and the plain sum comes out negative (checked here with the same formula in numpy, for the first
    case); the oracle must not take that for 'below zero'."""
    t0, mv = 0.5348999931723383, 1.658202316445049e-16
    mass = t0 + mv
    mid = 0.5 * (mass + t0)
    plain = 0.5 * mass * np.log(mass / mid) + 0.5 * (t0 * np.log(t0 / mid) + mv * np.log(2.0))
    assert plain < 0.0          # the case is one where rounding alone would decide
    rng = np.random.default_rng(3)
    cases = [(t0, mv)] + [(float(a), float(a * b * 1.1e-16)) for a, b in
                          zip(rng.uniform(0.1, 0.9, 3000), rng.uniform(0.2, 3.0, 3000))]
    g = np.full(4, 0.25)
    for t0, mv in cases:
        t = np.array([t0, mv, 1.0 - t0 - mv, 0.0])
        for u in (0.1, 0.9):
            out = oracle_mod.verify_probs(t, g, 0, np.array([0, 1, 2], dtype=np.int32), 0.0, u, 0.5, divergence="jsd")
            assert out["a_size"] == 1
            assert out["accept"] == int(u * 0.25 < t0)      # u < min(1, t(xt) / g(xt))
            assert out["mass"] == t0
