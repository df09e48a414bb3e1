"""Pins the oracle's walk of a drafted tree (Algorithm 1 applied along the branches, siblings tried
in index order) and its verification over shared logit rows."""
import numpy as np
import torch

from synth import workloads
from parity_utils import random_trees


def test_hand_trees(oracle_mod):
    # one tree of 7 nodes:        prefix
    #                            /      \
    #                           0        1
    #                         / | \      |
    #                        2  3  4     5
    #                           |
    #                           6
    parent = np.array([-1, -1, 0, 0, 0, 1, 3], dtype=np.int32)
    res = np.array([10, 11, 12, 13, 14, 15, 16], dtype=np.int32)
    cases = [
        # accept flags                      len path        next
        ([1, 1, 0, 1, 1, 1, 1], 3, [0, 3, 6], -1),   # 0, then 3 (2 rejected), then leaf 6: extra token
        ([1, 1, 0, 1, 1, 1, 0], 2, [0, 3], 16),      # 6 rejected: its resampled token
        ([1, 1, 0, 0, 0, 1, 1], 1, [0], 12),         # all children of 0 rejected: first child's token
        ([0, 1, 1, 1, 1, 0, 1], 1, [1], 15),         # second root child taken, then 5 rejected
        ([0, 0, 1, 1, 1, 1, 1], 0, [], 10),          # nothing accepted: first root child's token
        ([0, 1, 1, 1, 1, 1, 1], 2, [1, 5], -1),
        ([1, 1, -1, 1, 1, 1, 1], 1, [0], -2),        # unusable child met before an accepted one
        ([1, 1, 0, 1, -1, 1, 1], 3, [0, 3, 6], -1),  # unusable child after the accepted one: not reached
        ([-1, 1, 1, 1, 1, 1, 1], 0, [], -2),
    ]
    for acc, want_len, want_path, want_next in cases:
        n, path, nxt = oracle_mod.accept_trees(np.array(acc, dtype=np.int32), res, parent, 7)
        assert n[0] == want_len and nxt[0] == want_next, (acc, n, nxt)
        assert list(path[0][:want_len]) == want_path and (path[0][want_len:] == -1).all()


def test_malformed_parent(oracle_mod):
    acc = np.ones(4, dtype=np.int32)
    res = np.full(4, -1, dtype=np.int32)
    for parent in ([-1, 0, 2, 1], [-1, 0, 5, 1], [-2, 0, 1, 2], [0, 0, 1, 2]):
        n, path, nxt = oracle_mod.accept_trees(acc, res, np.array(parent, dtype=np.int32), 4)
        assert n[0] == 0 and nxt[0] == -3 and (path == -1).all()


def test_chain_is_the_one_child_case(oracle_mod):
    rng = np.random.default_rng(5)
    B, L = 300, 12
    accept = rng.choice([1, 1, 1, 0, -1], size=(B, L), p=[0.3, 0.3, 0.25, 0.13, 0.02]).astype(np.int32)
    resample = np.where(accept == 0, rng.integers(0, 1000, (B, L)), -1).astype(np.int32)
    parent = np.tile(np.arange(-1, L - 1, dtype=np.int32), (B, 1))
    n_c, next_c = oracle_mod.accept_chains(accept, resample, L)
    n_t, path, next_t = oracle_mod.accept_trees(accept, resample, parent, L)
    np.testing.assert_array_equal(n_t, n_c)
    np.testing.assert_array_equal(next_t, next_c)
    for b in range(B):
        assert list(path[b][: n_t[b]]) == list(range(n_t[b]))


def test_properties_on_random_trees(oracle_mod):
    """What the rule fixes, checked from the outputs alone: the path is a branch from the prefix,
    every node on it is accepted, every earlier sibling of a path node was rejected, and the end of
    the walk matches the state of the last node's children."""
    rng = np.random.default_rng(17)
    for M, p_acc in ((1, 0.5), (7, 0.6), (60, 0.7), (60, 0.2), (200, 0.9)):
        B = 150
        parent = random_trees(rng, B, M)
        accept = rng.choice([1, 0, -1], size=(B, M), p=[p_acc, 1 - p_acc - 0.01, 0.01]).astype(np.int32)
        resample = np.where(accept == 0, rng.integers(0, 16384, (B, M)), -1).astype(np.int32)
        n, path, nxt = oracle_mod.accept_trees(accept, resample, parent, M)
        for b in range(B):
            kids = lambda v: [i for i in range(M) if parent[b, i] == v]
            cur = -1
            for j in range(n[b]):
                node = path[b, j]
                assert parent[b, node] == cur and accept[b, node] == 1
                assert all(accept[b, s] == 0 for s in kids(cur) if s < node)
                cur = node
            assert (path[b, n[b]:] == -1).all()
            ch = kids(cur)
            flags = [accept[b, c] for c in ch]
            if not ch:
                assert nxt[b] == -1
            elif all(f == 0 for f in flags):
                assert nxt[b] == resample[b, ch[0]] and nxt[b] >= 0
            else:
                first_nonzero = next(f for f in flags if f != 0)
                assert first_nonzero == -1 and nxt[b] == -2


def test_sibling_order_decides(oracle_mod):
    """Swapping two accepted siblings changes which of them is taken: the lower index wins."""
    parent = np.array([-1, -1, 0, 1], dtype=np.int32)
    res = np.full(4, -1, dtype=np.int32)
    n, path, nxt = oracle_mod.accept_trees(np.array([1, 1, 1, 1], dtype=np.int32), res, parent, 4)
    assert list(path[0][:2]) == [0, 2]
    n, path, nxt = oracle_mod.accept_trees(np.array([0, 1, 1, 1], dtype=np.int32), res, parent, 4)
    assert list(path[0][:2]) == [1, 3]


def test_verify_rows_is_verify_on_gathered_rows(oracle_mod):
    """Shared logit rows: the outcome of verification i depends on row row_index[i] only, so
    duplicating the rows by hand and verifying them one by one gives the same result."""
    cfg = workloads.CONFIGS["tiny"]
    cb = workloads.make_codebook(cfg)
    table = oracle_mod.build_knn(cb.numpy(), cfg.k, threads=4)
    st = workloads.make_step(cfg, step=2, rows=6)
    rng = np.random.default_rng(3)
    N = 20
    row_index = rng.integers(0, 6, N).astype(np.int32)
    row_index[4] = 6          # one past the end
    row_index[9] = -1
    tokens = rng.integers(0, cfg.V, N).astype(np.int32)
    un = torch.from_numpy(rng.random((N, 2)).astype(np.float32))
    acc, res, _ = oracle_mod.verify_rows(st.target_logits, st.draft_logits, row_index, tokens, table, cfg.k,
                                         cfg.delta, un)
    for i in range(N):
        if row_index[i] < 0 or row_index[i] >= 6:
            assert acc[i] == -1 and res[i] == -1
            continue
        r = int(row_index[i])
        a1, r1, _ = oracle_mod.verify(st.target_logits[r:r + 1], st.draft_logits[r:r + 1], tokens[i:i + 1], table,
                                      cfg.k, cfg.delta, un[i:i + 1])
        assert (acc[i], res[i]) == (a1[0], r1[0])
    accg, tokg, _ = oracle_mod.verify_greedy_rows(st.target_logits, row_index, tokens, table, cfg.k, cfg.delta)
    for i in range(N):
        if row_index[i] < 0 or row_index[i] >= 6:
            assert accg[i] == -1 and tokg[i] == -1
            continue
        r = int(row_index[i])
        a1, t1, _ = oracle_mod.verify_greedy(st.target_logits[r:r + 1], tokens[i:i + 1], table, cfg.k, cfg.delta)
        assert (accg[i], tokg[i]) == (a1[0], t1[0])
