"""The CPU side under AddressSanitizer and UndefinedBehaviorSanitizer: the oracle (through a small
C driver, tests/oracle_sanitize_main.c) on the hand-derived rows, brute-force neighbour cases with
ties and duplicates, unusable rows, the greedy variant, chain and tree walks and the random table;
and the host build of the device's fp64 exponential.  A sanitizer report aborts the process."""
import json
import os
import struct
import subprocess

import numpy as np
import pytest

from synth import philox

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=1", UBSAN_OPTIONS="print_stacktrace=1")


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("san") / "oracle_sanitize")
    subprocess.run(["gcc", "-std=c11", *SAN, "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
                    os.path.join(ROOT, "tests", "oracle_sanitize_main.c"), "-o", exe, "-lm"], check=True)
    return exe


class Stream:
    """Builds the driver's input file and remembers how to parse its output."""

    def __init__(self):
        self.buf = bytearray()
        self.readers = []

    def i32(self, *vals):
        self.buf += struct.pack(f"<{len(vals)}i", *[int(v) for v in vals])

    def f64(self, *vals):
        self.buf += struct.pack(f"<{len(vals)}d", *[float(v) for v in vals])

    def arr(self, a, dtype):
        self.buf += np.ascontiguousarray(a, dtype=dtype).tobytes()

    def run(self, exe, tmp_path):
        fin, fout = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
        with open(fin, "wb") as f:
            f.write(self.buf)
        r = subprocess.run([exe, fin, fout], env=ENV, capture_output=True, text=True)
        assert r.returncode == 0, f"driver failed ({r.returncode}):\n{r.stderr[-4000:]}"
        data = open(fout, "rb").read()
        pos, results = 0, []
        for reader in self.readers:
            rc = struct.unpack_from("<i", data, pos)[0]
            pos += 4
            out = []
            if rc == 0:
                for dtype, count in reader:
                    a = np.frombuffer(data, dtype=dtype, count=count, offset=pos)
                    pos += a.nbytes
                    out.append(a)
            results.append((rc, out))
        assert pos == len(data)
        return results


def _add_probs(s, t, g, xt, nbrs, delta, u_acc, u_res, divergence=0):
    V, k = len(t), len(nbrs)
    s.i32(1, V, k, xt, divergence)
    s.f64(delta, u_acc, u_res)
    s.arr(t, np.float64); s.arr(g, np.float64); s.arr(nbrs, np.int32)
    s.readers.append([(np.int32, 2), (np.float64, 12), (np.float64, V), (np.float64, V)])


def test_hand_rows_under_sanitizers(driver, oracle_mod, tmp_path):
    with open(os.path.join(ROOT, "tests", "golden", "hand_rows.json")) as f:
        cases = json.load(f)["cases"]
    s = Stream()
    expect = []
    for case in cases:
        for d in case["draws"]:
            for divergence in (0, 1):
                _add_probs(s, case["t"], case["g"], case["xt"], case["nbrs"], case["delta"], d["u_acc"], d["u_res"],
                           divergence)
                expect.append((case, d, divergence))
    for (rc, out), (case, d, divergence) in zip(s.run(driver, tmp_path), expect):
        assert rc == 0
        if divergence == 0:
            assert tuple(out[0]) == (d["accept"], d["resample"]), case["name"]
            assert int(out[1][7]) == case["expect"]["a_size"]
        else:   # same code path as the shared library: identical results
            r = oracle_mod.verify_probs(case["t"], case["g"], case["xt"], case["nbrs"], case["delta"], d["u_acc"],
                                        d["u_res"], divergence="jsd")
            assert tuple(out[0]) == (r["accept"], r["resample"])


def test_neighbour_tables_under_sanitizers(driver, oracle_mod, tmp_path):
    rng = np.random.default_rng(3)
    xs, ys = np.meshgrid(np.arange(6), np.arange(6), indexing="ij")
    lattice = np.stack([xs.ravel(), ys.ravel()], axis=1).astype(np.float32)      # exact ties
    base = rng.standard_normal((7, 5)).astype(np.float32)
    dup = base[rng.integers(0, 7, 50)]                                             # duplicates
    cases = [(lattice, 36, 0), (lattice, 9, 0), (dup, 20, 0), (dup, 50, 1),
             (rng.standard_normal((64, 3)).astype(np.float32), 64, 0), (np.ones((1, 4), np.float32), 1, 0)]
    s = Stream()
    for cb, k, metric in cases:
        V, d = cb.shape
        s.i32(2, V, d, k, metric, 0, V, 3)
        s.arr(cb, np.float32)
        s.readers.append([(np.int32, V * k)])
    s.i32(2, 8, 2, 9, 0, 0, 8, 1)          # k > V: refused, nothing written
    s.arr(np.zeros((8, 2)), np.float32)
    s.readers.append([])
    res = s.run(driver, tmp_path)
    for (rc, out), (cb, k, metric) in zip(res, cases):
        assert rc == 0
        want = oracle_mod.build_knn(cb, k, metric=("l2", "cosine")[metric], threads=2)
        np.testing.assert_array_equal(out[0].reshape(cb.shape[0], k), want)
    assert res[-1][0] != 0


def test_rows_from_logits_under_sanitizers(driver, oracle_mod, tmp_path):
    """Verification from logits, with every kind of unusable row, the greedy variant, and the walks."""
    rng = np.random.default_rng(9)
    N, V, k = 24, 61, 9
    t = (rng.standard_normal((N, V)) * 2.5).astype(np.float32)
    g = (t + rng.standard_normal((N, V))).astype(np.float32)
    tok = rng.integers(0, V, N).astype(np.int32)
    table = np.stack([np.concatenate([[x], (x + 1 + rng.permutation(V - 1)[: k - 1]) % V]) for x in range(V)]).astype(np.int32)
    un = philox.uniforms(4, N)
    t[1, 5] = np.nan
    g[2, 0] = np.inf
    t[3, :] = -np.inf
    tok[4] = V
    tok[5] = -1
    table[tok[6], k - 1] = V + 3
    t[7, 1:20] = -np.inf
    s = Stream()
    for divergence, delta in ((0, 0.2), (1, 0.05), (0, 0.0)):
        s.i32(3, N, V, k, divergence, 3)
        s.f64(float(np.float32(delta)))    # the front end hands the C routine the binary32 value
        s.arr(t, np.float32); s.arr(g, np.float32); s.arr(tok, np.int32); s.arr(table, np.int32); s.arr(un, np.float32)
        s.readers.append([(np.int32, N), (np.int32, N), (np.float64, N * 12)])
    s.i32(4, N, V, k, 2)
    s.f64(float(np.float32(0.2)))
    s.arr(t, np.float32); s.arr(tok, np.int32); s.arr(table, np.int32)
    s.readers.append([(np.int32, N), (np.int32, N)])
    acc_c = rng.integers(-1, 2, 40).astype(np.int32)
    res_c = rng.integers(0, V, 40).astype(np.int32)
    s.i32(5, 8, 5); s.arr(acc_c, np.int32); s.arr(res_c, np.int32)
    s.readers.append([(np.int32, 8), (np.int32, 8)])
    parent = np.concatenate([[-1] + [int(rng.integers(-1, i)) for i in range(1, 10)] for _ in range(4)]).astype(np.int32)
    parent[35] = 37                                                                  # malformed tree
    s.i32(6, 4, 10); s.arr(acc_c, np.int32); s.arr(res_c, np.int32); s.arr(parent, np.int32)
    s.readers.append([(np.int32, 4), (np.int32, 40), (np.int32, 4)])
    s.i32(7, 97, 13, 0, 97, 3)
    s.buf += struct.pack("<Q", 0xDEADBEEF12345678)
    s.readers.append([(np.int32, 97 * 13)])
    out = s.run(driver, tmp_path)
    for (rc, o), (divergence, delta) in zip(out[:3], (("tvd", 0.2), ("jsd", 0.05), ("tvd", 0.0))):
        assert rc == 0
        acc, res, _ = oracle_mod.verify(t, g, tok, table, k, delta, un, threads=2, divergence=divergence)
        np.testing.assert_array_equal(o[0], acc)
        np.testing.assert_array_equal(o[1], res)
        assert list(o[0][1:7]) == [-1] * 6 and o[0][7] >= 0
    rc, o = out[3]
    acc, tk, _ = oracle_mod.verify_greedy(t, tok, table, k, 0.2, threads=2)
    assert rc == 0 and o[0][1] == -1 and list(o[0][3:7]) == [-1] * 4    # row 2's bad value is in the draft row
    np.testing.assert_array_equal(o[0], acc)
    np.testing.assert_array_equal(o[1], tk)
    rc, o = out[4]
    n, nxt = oracle_mod.accept_chains(acc_c, res_c, 5)
    np.testing.assert_array_equal(o[0], n); np.testing.assert_array_equal(o[1], nxt)
    rc, o = out[5]
    n, path, nxt = oracle_mod.accept_trees(acc_c, res_c, parent, 10)
    np.testing.assert_array_equal(o[0], n); np.testing.assert_array_equal(o[1].reshape(4, 10), path)
    np.testing.assert_array_equal(o[2], nxt)
    assert o[2][3] == -3
    rc, o = out[6]
    np.testing.assert_array_equal(o[0].reshape(97, 13), oracle_mod.build_random(97, 13, 0xDEADBEEF12345678, threads=2))


def test_sequential_sibling_walk_under_sanitizers(driver, oracle_mod, tmp_path):
    from test_oracle_sibling_pins import _random_tree_inputs
    rng = np.random.default_rng(21)
    B, M, V, k = 6, 9, 25, 4
    parent, tl, dl, row_index, tokens, table, un = _random_tree_inputs(rng, B, M, V, k)
    tokens[3] = V + 2                                 # an unusable candidate
    tl[row_index[2 * M], 1] = np.inf
    s = Stream()
    for divergence, delta in ((0, 0.1), (1, 0.02)):
        s.i32(8, B * (M + 1), V, B, M, k, divergence, 3)
        s.f64(float(np.float32(delta)))
        s.arr(tl, np.float32); s.arr(dl, np.float32); s.arr(row_index, np.int32); s.arr(parent, np.int32)
        s.arr(tokens, np.int32); s.arr(table, np.int32); s.arr(un, np.float32)
        s.readers.append([(np.int32, B), (np.int32, B * M), (np.int32, B)])
    for (rc, o), (divergence, delta) in zip(s.run(driver, tmp_path), (("tvd", 0.1), ("jsd", 0.02))):
        assert rc == 0
        n, path, nxt = oracle_mod.verify_trees_sequential(tl, dl, row_index, parent, M, tokens, table, k, delta, un,
                                                          threads=2, divergence=divergence)
        np.testing.assert_array_equal(o[0], n)
        np.testing.assert_array_equal(o[1].reshape(B, M), path)
        np.testing.assert_array_equal(o[2], nxt)


def test_exp64_host_build_under_sanitizers(tmp_path):
    exe = str(tmp_path / "exp64_check_san")
    subprocess.run(["g++", *SAN, "-ffp-contract=off", "-I", os.path.join(ROOT, "paper_2410_03355_amd", "csrc"),
                    os.path.join(ROOT, "tests", "exp64_check.cpp"), "-o", exe, "-lm"], check=True)
    r = subprocess.run([exe], env=ENV, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    worst, n_diff, n, specials, worst_tab, n_diff_tab, specials_tab = (int(x) for x in r.stdout.split())
    assert worst <= 1 and specials == 1 and worst_tab <= 1 and specials_tab == 1
