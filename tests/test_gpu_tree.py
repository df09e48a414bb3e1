"""GPU parity of lantern_accept_trees, lantern_verify_rows and lantern_verify_greedy_rows against
the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from synth import workloads
from parity_utils import random_table, random_trees, sparse_table_from_oracle, tree_step

pytestmark = pytest.mark.gpu


def _walk_both(oracle, lantern, accept, resample, parent, M):
    n_o, path_o, next_o = oracle.accept_trees(accept, resample, parent, M)
    n, path, nxt = lantern.accept_trees(torch.from_numpy(accept).cuda().reshape(-1),
                                        torch.from_numpy(resample).cuda().reshape(-1),
                                        torch.from_numpy(parent).cuda().reshape(-1), M)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(n.cpu().numpy(), n_o)
    np.testing.assert_array_equal(path.cpu().numpy(), path_o)
    np.testing.assert_array_equal(nxt.cpu().numpy(), next_o)
    return n_o, path_o, next_o


@pytest.mark.parametrize("M,B,p_acc", [(1, 9, 0.5), (7, 130, 0.6), (60, 64, 0.7), (60, 257, 0.15),
                                       (64, 33, 0.9), (65, 33, 0.9), (200, 40, 0.95), (1000, 5, 0.99)])
def test_walk_random_trees(oracle_mod, lantern_gpu, M, B, p_acc):
    rng = np.random.default_rng(M * 7 + B)
    parent = random_trees(rng, B, M, max_children=3)
    accept = rng.choice([1, 0, -1], size=(B, M), p=[p_acc, 1 - p_acc - 0.004, 0.004]).astype(np.int32)
    resample = np.where(accept == 0, rng.integers(0, 16384, (B, M)), -1).astype(np.int32)
    n, path, nxt = _walk_both(oracle_mod, lantern_gpu, accept, resample, parent, M)
    if M >= 60:
        assert n.max() > 2


def test_walk_chains_and_malformed(oracle_mod, lantern_gpu):
    rng = np.random.default_rng(8)
    B, L = 100, 70                                 # chains longer than a wavefront
    accept = (rng.random((B, L)) < 0.97).astype(np.int32)
    resample = np.where(accept == 0, rng.integers(0, 999, (B, L)), -1).astype(np.int32)
    parent = np.tile(np.arange(-1, L - 1, dtype=np.int32), (B, 1))
    parent[3, 10] = 10                             # own parent
    parent[4, 0] = -2
    parent[5, 69] = 200
    n, path, nxt = _walk_both(oracle_mod, lantern_gpu, accept, resample, parent, L)
    assert list(nxt[3:6]) == [-3, -3, -3] and list(n[3:6]) == [0, 0, 0]
    kept, nxt_c = lantern_gpu.accept_chains(torch.from_numpy(accept).cuda().reshape(-1),
                                            torch.from_numpy(resample).cuda().reshape(-1), L)
    ok = np.ones(B, dtype=bool)
    ok[3:6] = False
    np.testing.assert_array_equal(kept.cpu().numpy()[ok], n[ok])
    np.testing.assert_array_equal(nxt_c.cpu().numpy()[ok], nxt[ok])


def _verify_rows_both(oracle, lantern, st, row_index, tokens, un, table, delta, divergence="tvd", threads=8):
    k = table.shape[1]
    acc_o, res_o, diag = oracle.verify_rows(st.target_logits, st.draft_logits, row_index, tokens, table, k, delta,
                                            un, threads=threads, divergence=divergence)
    acc, res = lantern.verify_rows(st.target_logits.cuda(), st.draft_logits.cuda(),
                                   torch.from_numpy(row_index).cuda(), torch.from_numpy(tokens).cuda(),
                                   torch.from_numpy(np.ascontiguousarray(table)).cuda(), delta, un.cuda(),
                                   divergence=divergence)
    torch.cuda.synchronize()
    acc, res = acc.cpu().numpy(), res.cpu().numpy()
    bad = np.nonzero((acc != acc_o) | (res != res_o))[0]
    assert bad.size == 0, (f"{bad.size} rows differ; first {bad[0]}: gpu {acc[bad[0]]}/{res[bad[0]]} "
                           f"oracle {acc_o[bad[0]]}/{res_o[bad[0]]}")
    return acc_o, res_o


@pytest.mark.parametrize("divergence", ["tvd", "jsd"])
def test_tiny_trees_end_to_end(oracle_mod, lantern_gpu, divergence):
    cfg = workloads.CONFIGS["tiny"]
    cb = workloads.make_codebook(cfg)
    table = oracle_mod.build_knn(cb.numpy(), cfg.k, threads=8)
    rng = np.random.default_rng(2)
    B, M = 12, 9
    parent = random_trees(rng, B, M, max_children=3)
    st, row_index, tokens, un = tree_step(cfg, parent, step=4)
    row_index[5] = B * (M + 1)                     # one past the last row
    row_index[17] = -4
    acc, res = _verify_rows_both(oracle_mod, lantern_gpu, st, row_index, tokens, un, table, cfg.delta, divergence)
    assert acc[5] == -1 and acc[17] == -1 and (acc == 1).any() and (acc == 0).any()
    _walk_both(oracle_mod, lantern_gpu, acc.reshape(B, M), res.reshape(B, M), parent, M)


@pytest.mark.parametrize("variant,delta", [("plain", 0.4), ("plain", 0.01), ("reject", 0.05)])
def test_llamagen_trees_of_60(oracle_mod, lantern_gpu, variant, delta):
    """60 candidates per tree as in the paper's set-up; V=16384, k=1000, bf16 logits."""
    cfg = workloads.CONFIGS["llamagen_step"]
    rng = np.random.default_rng(6)
    B, M = 4, 60
    parent = random_trees(rng, B, M, max_children=4)
    st, row_index, tokens, un = tree_step(cfg, parent, step=1, variant=variant)
    cb = workloads.make_codebook(cfg)
    table = sparse_table_from_oracle(oracle_mod, cb.numpy(), cfg.k, tokens)
    acc, res = _verify_rows_both(oracle_mod, lantern_gpu, st, row_index, tokens, un, table, delta)
    n, path, nxt = _walk_both(oracle_mod, lantern_gpu, acc.reshape(B, M), res.reshape(B, M), parent, M)
    # siblings share rows: fewer distinct logit rows than verifications
    assert len(set(row_index.tolist())) < B * M


def test_stress_trees_full_step(oracle_mod, lantern_gpu):
    """64 trees of 60 candidates: the 3840 verifications of the stress step, over shared rows."""
    cfg = workloads.CONFIGS["stress"]
    rng = np.random.default_rng(9)
    B, M = 64, 60
    parent = random_trees(rng, B, M, max_children=4)
    st, row_index, tokens, un = tree_step(cfg, parent, step=2)
    table = random_table(cfg.V, cfg.k, seed=8)
    for delta in (cfg.delta, 0.002):
        acc, res = _verify_rows_both(oracle_mod, lantern_gpu, st, row_index, tokens, un, table, delta, threads=16)
        n, path, nxt = _walk_both(oracle_mod, lantern_gpu, acc.reshape(B, M), res.reshape(B, M), parent, M)
    assert (acc == 0).sum() > 100 and (acc == 1).sum() > 100


def test_greedy_rows(oracle_mod, lantern_gpu):
    cfg = workloads.CONFIGS["llamagen_step"]
    rng = np.random.default_rng(12)
    B, M = 3, 60
    parent = random_trees(rng, B, M, max_children=4)
    st, row_index, tokens, un = tree_step(cfg, parent, step=7, variant="peaked")
    # greedy acceptance needs drafts near the top of the target row
    order = torch.argsort(st.target_logits.float(), dim=1, descending=True)[:, :3].numpy()
    tokens = order[row_index, rng.integers(0, 3, B * M)].astype(np.int32)
    row_index[7] = -1
    table = random_table(cfg.V, cfg.k, seed=3)
    for delta in (0.0, 0.01, 0.3):
        acc_o, tok_o, _ = oracle_mod.verify_greedy_rows(st.target_logits, row_index, tokens, table, cfg.k, delta,
                                                        threads=8)
        acc, tok = lantern_gpu.verify_greedy_rows(st.target_logits.cuda(), torch.from_numpy(row_index).cuda(),
                                                  torch.from_numpy(tokens).cuda(),
                                                  torch.from_numpy(table).cuda(), delta)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(acc.cpu().numpy(), acc_o)
        np.testing.assert_array_equal(tok.cpu().numpy(), tok_o)
        assert acc_o[7] == -1
        _walk_both(oracle_mod, lantern_gpu, acc_o.reshape(B, M), tok_o.reshape(B, M), parent, M)


def test_row_index_errors(lantern_gpu):
    t = torch.zeros((2, 16), device="cuda")
    tok = torch.zeros(3, dtype=torch.int32, device="cuda")
    knn = torch.arange(16, dtype=torch.int32, device="cuda").reshape(16, 1)
    un = torch.zeros((3, 2), device="cuda")
    with pytest.raises(ValueError):
        lantern_gpu.verify_rows(t, t, torch.zeros(2, dtype=torch.int32, device="cuda"), tok, knn, 0.1, un)
    lib = lantern_gpu.load()
    rc = lib.lantern_verify_rows(t.data_ptr(), t.data_ptr(), 0, 2, 16, 16, None, 3, tok.data_ptr(), knn.data_ptr(), 1,
                                 0, 0.1, un.data_ptr(), tok.data_ptr(), tok.data_ptr(), None)
    assert rc == -1
    rc = lib.lantern_verify_rows(t.data_ptr(), t.data_ptr(), 0, 0, 16, 16, tok.data_ptr(), 3, tok.data_ptr(),
                                 knn.data_ptr(), 1, 0, 0.1, un.data_ptr(), tok.data_ptr(), tok.data_ptr(), None)
    assert rc == -2
    rc = lib.lantern_accept_trees(tok.data_ptr(), tok.data_ptr(), tok.data_ptr(), 1, 0, tok.data_ptr(), tok.data_ptr(),
                                  tok.data_ptr(), None)
    assert rc == -2


def test_greedy_tree_step(oracle_mod, lantern_gpu):
    """lantern_verify_trees_greedy against the oracle's greedy verification over shared rows and its walk."""
    from parity_utils import level_order
    cfg = workloads.CONFIGS["llamagen_step"]
    rng = np.random.default_rng(41)
    B, M = 6, 60
    parent = level_order(random_trees(rng, B, M, max_children=5))
    st, row_index, tokens, un = tree_step(cfg, parent, step=9, variant="peaked")
    order = torch.argsort(st.target_logits.float(), dim=1, descending=True)[:, :3].numpy()
    tokens = order[row_index, rng.integers(0, 3, B * M)].astype(np.int32)     # drafts near the top of the target
    table = random_table(cfg.V, cfg.k, seed=13)
    for delta in (0.0, 0.02, 0.3):
        acc_o, tok_o, _ = oracle_mod.verify_greedy_rows(st.target_logits, row_index, tokens, table, cfg.k, delta,
                                                        threads=8)
        n_o, path_o, next_o = oracle_mod.accept_trees(acc_o, tok_o, parent, M)
        acc, tok, n, path, nxt = lantern_gpu.verify_trees_greedy(
            st.target_logits.cuda(), torch.from_numpy(row_index).cuda(), torch.from_numpy(parent).cuda().reshape(-1), M,
            torch.from_numpy(tokens).cuda(), torch.from_numpy(table).cuda(), delta)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(acc.cpu().numpy(), acc_o)
        np.testing.assert_array_equal(tok.cpu().numpy(), tok_o)
        np.testing.assert_array_equal(n.cpu().numpy(), n_o)
        np.testing.assert_array_equal(path.cpu().numpy(), path_o)
        np.testing.assert_array_equal(nxt.cpu().numpy(), next_o)
    assert n_o.max() >= 1
