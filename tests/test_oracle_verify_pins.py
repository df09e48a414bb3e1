"""Pins the CPU oracle's verification to things other than itself: hand-derived
rows (tests/golden), library softmax, the reduction to standard speculative
acceptance, the TVD invariant, monotonicity, residuals that sum to one, exact
enumeration of the output law and Monte-Carlo recovery of the target law."""
import json
import os

import numpy as np
import pytest
import scipy.special

from synth import philox

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_rows.json")


def _cases():
    with open(GOLDEN) as f:
        return json.load(f)["cases"]


@pytest.mark.parametrize("case", _cases(), ids=lambda c: c["name"])
def test_hand_derived_rows(oracle_mod, case):
    e = case["expect"]
    r = oracle_mod.verify_probs(case["t"], case["g"], case["xt"], case["nbrs"], case["delta"],
                                0.0, 0.0, want_dists=True)
    assert r["a_size"] == e["a_size"]
    assert r["mass"] == pytest.approx(e["mass"], abs=1e-15)
    assert r["accept_prob"] == pytest.approx(e["accept_prob"], abs=1e-15)
    assert r["tvd_walk"] == pytest.approx(e["tvd"], abs=1e-15)
    assert r["tvd_direct"] == pytest.approx(e["tvd"], abs=1e-15)
    np.testing.assert_allclose(r["distorted_target"], e["distorted_target"], atol=1e-15)
    if "residual" in e:
        np.testing.assert_allclose(r["residual"], e["residual"], atol=1e-15)
    for d in case["draws"]:
        r = oracle_mod.verify_probs(case["t"], case["g"], case["xt"], case["nbrs"], case["delta"],
                                    d["u_acc"], d["u_res"])
        assert (r["accept"], r["resample"]) == (d["accept"], d["resample"])


def test_softmax_against_library_and_invariants(oracle_mod):
    rng = np.random.default_rng(1)
    for scale in (0.1, 1.2, 3.0, 30.0):
        l = (rng.standard_normal(777) * scale).astype(np.float32)
        p = oracle_mod.softmax(l)
        np.testing.assert_allclose(p, scipy.special.softmax(l.astype(np.float64)), rtol=1e-13, atol=0)
        assert abs(p.sum() - 1.0) < 1e-12
        # adding a constant that is exact in fp32 leaves the row unchanged
        l2 = (l.astype(np.float64) + 8.0).astype(np.float32)
        exact = np.all(l2.astype(np.float64) == l.astype(np.float64) + 8.0)
        if exact:
            np.testing.assert_allclose(oracle_mod.softmax(l2), p, rtol=1e-13)
    l = np.array([0.0, -np.inf, 1.0, -np.inf], dtype=np.float32)
    p = oracle_mod.softmax(l)
    assert p[1] == 0.0 and p[3] == 0.0
    np.testing.assert_allclose(p[[0, 2]], [1 / (1 + np.e), np.e / (1 + np.e)], rtol=1e-15)
    # large offsets must not overflow: closed form 1/(1+e), e/(1+e)
    for off in (1000.0, -1000.0, 3.0e4):
        p = oracle_mod.softmax(np.array([off, off + 1.0], dtype=np.float32))
        np.testing.assert_allclose(p, [1 / (1 + np.e), np.e / (1 + np.e)], rtol=1e-15)
    for bad in ([np.nan, 0.0], [np.inf, 0.0], [-np.inf, -np.inf]):
        with pytest.raises(ValueError):
            oracle_mod.softmax(np.array(bad, dtype=np.float32))


def _random_row(rng, V, scale=2.0, noise=1.0):
    tl = rng.standard_normal(V) * scale
    gl = tl + rng.standard_normal(V) * noise
    t = scipy.special.softmax(tl)
    g = scipy.special.softmax(gl)
    return t, g


def _random_nbrs(rng, V, k, xt):
    others = rng.permutation(np.delete(np.arange(V), xt))[: k - 1]
    return np.concatenate([[xt], others]).astype(np.int32)


def test_reduces_to_standard_speculative_acceptance(oracle_mod):
    """k = 1 or delta = 0: acceptance min(1, t/g) and residual [t-g]_+ (Section 2)."""
    rng = np.random.default_rng(2)
    V = 50
    for trial in range(40):
        t, g = _random_row(rng, V)
        xt = int(rng.integers(V))
        want_prob = min(1.0, t[xt] / g[xt])
        want_res = np.maximum(t - g, 0.0)
        want_res = want_res / want_res.sum()
        for nbrs, delta in ((np.array([xt]), 0.3), (_random_nbrs(rng, V, 9, xt), 0.0)):
            r = oracle_mod.verify_probs(t, g, xt, nbrs, delta, 0.5, 0.5, want_dists=True)
            assert r["a_size"] == 1
            assert r["accept_prob"] == pytest.approx(want_prob, rel=1e-14)
            np.testing.assert_allclose(r["distorted_target"], t, rtol=0, atol=0)
            np.testing.assert_allclose(r["residual"], want_res, rtol=1e-13, atol=1e-16)
            for u in (0.0, 0.25, 0.75, 1 - 2.0 ** -24):
                r = oracle_mod.verify_probs(t, g, xt, nbrs, delta, u, 0.4)
                assert r["accept"] == int(u < want_prob)
                if not r["accept"]:
                    cdf = np.cumsum(want_res)
                    assert r["resample"] == int(np.searchsorted(cdf, 0.4, side="right"))


def test_tvd_invariant_prefix_and_maximality(oracle_mod):
    """TVD(t_A, t) < delta strictly, equals the walked sum, and the walk is maximal."""
    rng = np.random.default_rng(3)
    V = 64
    for trial in range(200):
        t, g = _random_row(rng, V, scale=rng.choice([0.5, 2.0, 4.0]))
        xt = int(rng.integers(V))
        k = int(rng.integers(1, V + 1))
        nbrs = _random_nbrs(rng, V, k, xt)
        delta = float(rng.choice([0.01, 0.05, 0.1, 0.2, 0.4, 0.9]))
        r = oracle_mod.verify_probs(t, g, xt, nbrs, delta, 0.5, 0.5, want_dists=True)
        a = r["a_size"]
        ta = r["distorted_target"]
        assert 1 <= a <= k
        assert r["tvd_direct"] == pytest.approx(r["tvd_walk"], abs=1e-14)
        assert r["tvd_walk"] < delta
        # independent evaluation of the definition of t_A for the prefix the oracle chose
        A = nbrs[:a]
        ref = t.copy()
        ref[A] = 0.0
        ref[xt] = t[A].sum()
        np.testing.assert_allclose(ta, ref, atol=1e-15)
        assert abs(ta.sum() - 1.0) < 1e-12 and ta.min() >= 0.0
        assert r["mass"] == pytest.approx(t[A].sum(), abs=1e-15)
        assert r["mass"] <= t[xt] + delta
        # accept probability never below the unrelaxed one (Section 4.2)
        assert r["accept_prob"] >= min(1.0, t[xt] / g[xt]) - 1e-15
        if a < k:  # the next neighbour would have broken the bound
            assert t[nbrs[1:a + 1]].sum() >= delta - 1e-15


def test_monotone_in_k_and_delta(oracle_mod):
    """Trend of Table 1: acceptance probability grows with k and with delta."""
    rng = np.random.default_rng(4)
    V = 128
    for trial in range(30):
        t, g = _random_row(rng, V)
        xt = int(rng.integers(V))
        full = _random_nbrs(rng, V, V, xt)
        prev_by_delta = None
        for delta in (0.0, 0.05, 0.1, 0.2, 0.4, 0.8, 1.5):
            probs, sizes = [], []
            for k in (1, 2, 5, 17, 64, 128):
                r = oracle_mod.verify_probs(t, g, xt, full[:k], delta, 0.5, 0.5)
                probs.append(r["accept_prob"])
                sizes.append(r["a_size"])
            assert all(b >= a for a, b in zip(probs, probs[1:]))
            assert all(b >= a for a, b in zip(sizes, sizes[1:]))
            if prev_by_delta is not None:
                assert all(b >= a for a, b in zip(prev_by_delta, probs))
            prev_by_delta = probs
        r = oracle_mod.verify_probs(t, g, xt, full[:40], 1.5, 0.5, 0.5)
        assert r["a_size"] == 40  # a bound above one never binds (eq. 1)
        assert r["mass"] == pytest.approx(t[full[:40]].sum(), abs=1e-14)


def test_residual_properties(oracle_mod):
    rng = np.random.default_rng(5)
    V = 96
    seen_reject = 0
    for trial in range(200):
        t, g = _random_row(rng, V, scale=1.0, noise=1.5)
        xt = int(np.argmax(g))  # drafter's favourite: often over-proposed, so rejections occur
        k = int(rng.integers(1, 20))
        nbrs = _random_nbrs(rng, V, k, xt)
        delta = float(rng.choice([0.02, 0.1, 0.3]))
        r = oracle_mod.verify_probs(t, g, xt, nbrs, delta, 1 - 2.0 ** -24, rng.random(), want_dists=True)
        rho = r["residual"]
        assert abs(rho.sum() - 1.0) < 1e-12 and rho.min() >= 0.0
        A = nbrs[: r["a_size"]]
        assert np.all(rho[A[A != xt]] == 0.0)
        if not r["accept"]:
            seen_reject += 1
            assert rho[xt] == 0.0  # rejected means g(xt) > mass
            assert rho[r["resample"]] > 0.0
            # independent numpy evaluation of the residual and the bucket rule
            ref = np.maximum(r["distorted_target"] - g, 0.0)
            assert r["resid_z"] == pytest.approx(ref.sum(), rel=1e-13)
    assert seen_reject > 50


def _output_law(oracle_mod, t, g, table, delta):
    """Closed-form law of the emitted token when xt ~ g: sum over xt of
    g(xt) * [ a(xt) 1{x = xt} + (1 - a(xt)) residual_xt(x) ]."""
    V = len(t)
    law = np.zeros(V)
    for xt in range(V):
        r = oracle_mod.verify_probs(t, g, xt, table[xt], delta, 0.5, 0.5, want_dists=True)
        law[xt] += g[xt] * r["accept_prob"]
        law += g[xt] * (1.0 - r["accept_prob"]) * r["residual"]
    return law


def test_exact_enumeration_recovers_target_at_k1(oracle_mod):
    """Standard speculative decoding emits exactly the target law (Section 2)."""
    rng = np.random.default_rng(6)
    for V in (3, 8, 33):
        t, g = _random_row(rng, V)
        table = np.arange(V, dtype=np.int32).reshape(V, 1)
        law = _output_law(oracle_mod, t, g, table, 0.3)
        np.testing.assert_allclose(law, t, atol=1e-14)
        # relaxed (k > 1) keeps total mass one but is no longer the target law
        table = np.stack([_random_nbrs(rng, V, 3, x) for x in range(V)])
        law = _output_law(oracle_mod, t, g, table, 0.5)
        assert abs(law.sum() - 1.0) < 1e-12


def _logits_for(p):
    return np.log(p).astype(np.float32)


@pytest.mark.parametrize("k,delta", [(1, 0.2), (3, 0.25)])
def test_monte_carlo_matches_closed_form_law(oracle_mod, k, delta):
    """Draw xt ~ g and run the full logits path with Philox uniforms: the
    frequencies of the emitted token match the closed-form law, which at k = 1
    is the target distribution itself."""
    rng = np.random.default_rng(7)
    V, n = 8, 200_000
    tl = (rng.standard_normal(V) * 1.5).astype(np.float32)
    gl = (tl + rng.standard_normal(V)).astype(np.float32)
    t = oracle_mod.softmax(tl)
    g = oracle_mod.softmax(gl)
    table = np.stack([_random_nbrs(rng, V, k, x) for x in range(V)]).astype(np.int32)
    u_tok = philox.uniform_block(99, n, stream=5)
    tokens = np.minimum(np.searchsorted(np.cumsum(g), u_tok, side="right"), V - 1).astype(np.int32)
    un = philox.uniforms(1234, n, stream=1)
    acc, res, _ = oracle_mod.verify(np.tile(tl, (n, 1)), np.tile(gl, (n, 1)), tokens, table, k, delta,
                                    un, threads=4, want_diag=False)
    emitted = np.where(acc == 1, tokens, res)
    freq = np.bincount(emitted, minlength=V) / n
    law = _output_law(oracle_mod, t, g, table, delta)
    if k == 1:
        np.testing.assert_allclose(law, t, atol=1e-14)
    sigma = np.sqrt(law * (1 - law) / n)
    assert np.all(np.abs(freq - law) < 5 * sigma + 1e-9)


def test_logits_path_matches_probability_path(oracle_mod):
    rng = np.random.default_rng(8)
    V, N, k = 200, 30, 12
    tl = (rng.standard_normal((N, V)) * 2).astype(np.float32)
    gl = (tl + rng.standard_normal((N, V))).astype(np.float32)
    tl[3, 5:40] = -np.inf  # filtered tokens
    tokens = rng.integers(0, V, N).astype(np.int32)
    tokens[3] = 100
    table = np.stack([_random_nbrs(rng, V, k, x) for x in range(V)]).astype(np.int32)
    un = philox.uniforms(5, N)
    acc, res, diag = oracle_mod.verify(tl, gl, tokens, table, k, 0.15, un)
    for i in range(N):
        t = scipy.special.softmax(tl[i].astype(np.float64))
        g = scipy.special.softmax(gl[i].astype(np.float64))
        r = oracle_mod.verify_probs(t, g, tokens[i], table[tokens[i]], 0.15, un[i, 0], un[i, 1])
        assert diag["accept_prob"][i] == pytest.approx(r["accept_prob"], rel=1e-12)
        assert diag["a_size"][i] == r["a_size"]
        if min(diag["margin_accept"][i], diag["margin_cdf"][i]) > 1e-12:
            assert (acc[i], res[i]) == (r["accept"], r["resample"])


def test_unusable_rows_get_sentinels(oracle_mod):
    V, k = 16, 4
    rng = np.random.default_rng(9)
    tl = rng.standard_normal((5, V)).astype(np.float32)
    gl = rng.standard_normal((5, V)).astype(np.float32)
    table = np.stack([_random_nbrs(rng, V, k, x) for x in range(V)]).astype(np.int32)
    tokens = np.array([0, V, -1, 3, 4], dtype=np.int32)
    tl[3, 2] = np.nan
    gl[4, :] = -np.inf
    un = philox.uniforms(1, 5)
    acc, res, _ = oracle_mod.verify(tl, gl, tokens, table, k, 0.1, un)
    assert acc[0] in (0, 1)
    assert list(acc[1:]) == [-1] * 4 and list(res[1:]) == [-1] * 4


def test_philox_known_answers():
    """Known-answer vectors of Philox4x32-10 from the Random123 distribution."""
    def run(c, k):
        return [int(x) for x in philox.philox4x32_10(np.array([c], dtype=np.uint32), k)[0]]
    assert run([0, 0, 0, 0], (0, 0)) == [0x6627E8D5, 0xE169C58D, 0xBC57AC4C, 0x9B00DBD8]
    assert run([0x243F6A88, 0x85A308D3, 0x13198A2E, 0x03707344], (0xA4093822, 0x299F31D0)) == \
        [0xD16CFE09, 0x94FDCCEB, 0x5001E420, 0x24126EA1]
    u = philox.uniforms(7, 1000)
    assert u.dtype == np.float32 and u.min() >= 0.0 and u.max() < 1.0
    assert np.all(u * 2.0 ** 24 == np.round(u * 2.0 ** 24))


def test_delta_is_the_binary32_value_of_the_abi(oracle_mod):
    """The logits-level oracle reads the bound as the binary32 number the C ABI carries: a prefix
    whose TVD lies between the double 0.4 and float32(0.4) is inside the bound; on explicit
    probabilities (fp64 interface) the same prefix is refused at the double 0.4."""
    from parity_utils import delta_window_row
    target, draft, tokens, table, un = delta_window_row()
    acc, res, diag = oracle_mod.verify(target, draft, tokens, table, 2, 0.4, un)
    assert diag["a_size"][0] == 2 and diag["mass"][0] == pytest.approx(1.0, abs=1e-15)
    t = oracle_mod.softmax(target[0])
    r = oracle_mod.verify_probs(t, [0.5, 0.5], 0, [0, 1], 0.4, 0.75, 0.5)
    assert r["a_size"] == 1
    r = oracle_mod.verify_probs(t, [0.5, 0.5], 0, [0, 1], float(np.float32(0.4)), 0.75, 0.5)
    assert r["a_size"] == 2
