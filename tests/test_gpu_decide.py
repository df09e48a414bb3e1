"""GPU parity of the split verification (lantern_decide_rows, lantern_resample_selected) and of the
fused tree step (lantern_verify_trees) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from synth import workloads
from parity_utils import random_table, random_trees, sparse_table_from_oracle, tree_step

pytestmark = pytest.mark.gpu


def _decide_and_select(oracle, lantern, target, draft, tokens, table, delta, uniforms, divergence="tvd",
                       threads=8, row_index=None):
    """decide_rows must give the oracle's decisions; resample_selected on every rejected row (plus
    an accepted one, a negative code and an index past the end) the oracle's tokens."""
    k = table.shape[1]
    if row_index is None:
        acc_o, res_o, _ = oracle.verify(target, draft, tokens, table, k, delta, uniforms, threads=threads,
                                        divergence=divergence)
    else:
        acc_o, res_o, _ = oracle.verify_rows(target, draft, row_index, tokens, table, k, delta, uniforms,
                                             threads=threads, divergence=divergence)
    dev = "cuda"
    args = (target.to(dev), draft.to(dev), None if row_index is None else torch.from_numpy(row_index).to(dev),
            torch.as_tensor(tokens).to(dev), torch.from_numpy(np.ascontiguousarray(table)).to(dev), delta,
            uniforms.to(dev))
    acc = lantern.decide_rows(*args, divergence=divergence)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(acc.cpu().numpy(), acc_o)
    N = len(acc_o)
    sel = list(np.nonzero(acc_o == 0)[0][:200]) + list(np.nonzero(acc_o == 1)[0][:3]) + \
        list(np.nonzero(acc_o == -1)[0][:3]) + [-1, -2, -3, N, N + 5]
    sel = np.array(sel, dtype=np.int32)
    got = lantern.resample_selected(*args, torch.from_numpy(sel).to(dev), divergence=divergence).cpu().numpy()
    want = np.array([s if s < 0 else (-2 if s >= N else (res_o[s] if acc_o[s] == 0 else (-1 if acc_o[s] == 1 else -2)))
                     for s in sel], dtype=np.int32)
    np.testing.assert_array_equal(got, want)
    return acc_o, res_o


@pytest.mark.parametrize("divergence", ["tvd", "jsd"])
@pytest.mark.parametrize("delta", [0.0, 0.1, 0.5])
def test_tiny(oracle_mod, lantern_gpu, divergence, delta):
    cfg = workloads.CONFIGS["tiny"]
    table = oracle_mod.build_knn(workloads.make_codebook(cfg).numpy(), cfg.k, threads=8)
    st = workloads.make_step(cfg, step=9)
    acc, res = _decide_and_select(oracle_mod, lantern_gpu, st.target_logits, st.draft_logits,
                                  st.draft_tokens.numpy(), table, delta, st.uniforms, divergence)
    assert (acc == 0).any() and (acc == 1).any()


@pytest.mark.parametrize("variant,delta", [("plain", 0.4), ("plain", 0.002), ("reject", 0.0), ("peaked", 0.01),
                                           ("peaked", 0.3)])
def test_llamagen_shape(oracle_mod, lantern_gpu, variant, delta):
    cfg = workloads.CONFIGS["llamagen_step"]
    st = workloads.make_step(cfg, step=4, rows=300, variant=variant)
    table = sparse_table_from_oracle(oracle_mod, workloads.make_codebook(cfg).numpy(), cfg.k,
                                     st.draft_tokens.numpy())
    _decide_and_select(oracle_mod, lantern_gpu, st.target_logits, st.draft_logits, st.draft_tokens.numpy(), table,
                       delta, st.uniforms)


def test_stress_reject_mix_full_step(oracle_mod, lantern_gpu):
    """3840 rows of which most are rejected: the fp32 pass settles the rejections too."""
    cfg = workloads.CONFIGS["stress"]
    st = workloads.make_step(cfg, step=3, variant="reject")
    table = random_table(cfg.V, cfg.k, seed=8)
    acc, res = _decide_and_select(oracle_mod, lantern_gpu, st.target_logits, st.draft_logits,
                                  st.draft_tokens.numpy(), table, 0.0, st.uniforms, threads=16)
    assert (acc == 0).mean() > 0.3
    # the rejections are settled by the fp32 pass, not handed to the fp64 path
    acc2, path = lantern_gpu.decide_rows(st.target_logits.cuda(), st.draft_logits.cuda(), None,
                                         st.draft_tokens.cuda(), torch.from_numpy(table).cuda(), 0.0,
                                         st.uniforms.cuda(), want_path=True)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(acc2.cpu().numpy(), acc)
    assert (path.cpu().numpy() == 0).mean() > 0.99


def test_wide_latent_fp32_and_unusable_rows(oracle_mod, lantern_gpu):
    cfg = workloads.CONFIGS["wide_latent"]
    st = workloads.make_step(cfg, step=2, rows=256, variant="reject")
    table = random_table(cfg.V, cfg.k, seed=4)
    t = st.target_logits.clone()
    g = st.draft_logits.clone()
    tok = st.draft_tokens.numpy().copy()
    t[3, 100] = float("nan")
    g[5, :] = float("-inf")
    tok[7] = -1
    tok[9] = cfg.V
    acc, res = _decide_and_select(oracle_mod, lantern_gpu, t, g, tok, table, 0.05, st.uniforms)
    assert list(acc[[3, 5, 7, 9]]) == [-1] * 4


@pytest.mark.parametrize("V,k,N,dtype", [(7, 7, 5, torch.float32), (1003, 50, 40, torch.bfloat16),
                                         (4096, 2500, 9, torch.bfloat16), (40000, 100, 6, torch.float32)])
def test_shapes_off_the_fast_path(oracle_mod, lantern_gpu, V, k, N, dtype):
    rng = np.random.default_rng(V + k)
    t = torch.from_numpy((rng.standard_normal((N, V)) * 2).astype(np.float32)).to(dtype)
    g = (t.float() + torch.from_numpy(rng.standard_normal((N, V)).astype(np.float32))).to(dtype)
    tok = rng.integers(0, V, N).astype(np.int32)
    un = torch.from_numpy(rng.random((N, 2)).astype(np.float32))
    table = random_table(V, k, seed=V)
    for delta in (0.0, 0.2):
        _decide_and_select(oracle_mod, lantern_gpu, t, g, tok, table, delta, un)


def _expected_tree_outputs(oracle, acc_o, res_o, parent, M):
    n_o, path_o, next_o = oracle.accept_trees(acc_o.reshape(-1, M), res_o.reshape(-1, M), parent, M)
    # the verification whose token follows: the first child of the last accepted node
    stop = next_o.copy()
    for b in range(parent.shape[0]):
        if next_o[b] >= 0:
            cur = path_o[b, n_o[b] - 1] if n_o[b] else -1
            stop[b] = b * M + int(np.flatnonzero(parent[b] == cur)[0])
    return n_o, path_o, next_o, stop


@pytest.mark.parametrize("cfg_name,B,variant,delta", [("tiny", 12, "plain", 0.3), ("llamagen_step", 4, "plain", 0.4),
                                                      ("llamagen_step", 4, "reject", 0.05),
                                                      ("llamagen_step", 3, "peaked", 0.01)])
def test_verify_trees(oracle_mod, lantern_gpu, cfg_name, B, variant, delta):
    cfg = workloads.CONFIGS[cfg_name]
    M = 9 if cfg_name == "tiny" else 60
    rng = np.random.default_rng(B + M)
    parent = random_trees(rng, B, M, max_children=4)
    st, row_index, tokens, un = tree_step(cfg, parent, step=5, variant=variant)
    if cfg_name == "tiny":
        table = oracle_mod.build_knn(workloads.make_codebook(cfg).numpy(), cfg.k, threads=8)
        row_index[11] = -1                                  # an unusable verification inside a tree
    else:
        table = sparse_table_from_oracle(oracle_mod, workloads.make_codebook(cfg).numpy(), cfg.k, tokens)
    acc_o, res_o, _ = oracle_mod.verify_rows(st.target_logits, st.draft_logits, row_index, tokens, table, cfg.k,
                                             delta, un, threads=8)
    n_o, path_o, next_o, stop = _expected_tree_outputs(oracle_mod, acc_o, res_o, parent, M)
    dev = "cuda"
    par_d = torch.from_numpy(parent).to(dev).reshape(-1)
    args = (st.target_logits.to(dev), st.draft_logits.to(dev), torch.from_numpy(row_index).to(dev))
    tail = (torch.from_numpy(tokens).to(dev), torch.from_numpy(np.ascontiguousarray(table)).to(dev), delta,
            un.to(dev))
    acc, n, path, nxt = lantern_gpu.verify_trees(*args, par_d, M, *tail)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(acc.cpu().numpy(), acc_o)
    np.testing.assert_array_equal(n.cpu().numpy(), n_o)
    np.testing.assert_array_equal(path.cpu().numpy(), path_o)
    np.testing.assert_array_equal(nxt.cpu().numpy(), next_o)
    # the walk without resampled tokens names the verification to resample
    n2, path2, stop2 = lantern_gpu.accept_trees(acc, None, par_d, M)
    np.testing.assert_array_equal(stop2.cpu().numpy(), stop)
    np.testing.assert_array_equal(n2.cpu().numpy(), n_o)


def test_stress_trees_fused_step(oracle_mod, lantern_gpu):
    """64 trees of 60 candidates, mostly rejected candidates as under the paper's acceptance rates."""
    cfg = workloads.CONFIGS["stress"]
    rng = np.random.default_rng(21)
    B, M = 64, 60
    parent = random_trees(rng, B, M, max_children=4)
    st, row_index, tokens, un = tree_step(cfg, parent, step=8, variant="reject")
    table = random_table(cfg.V, cfg.k, seed=8)
    delta = 0.0
    acc_o, res_o, _ = oracle_mod.verify_rows(st.target_logits, st.draft_logits, row_index, tokens, table, cfg.k,
                                             delta, un, threads=16)
    n_o, path_o, next_o, _ = _expected_tree_outputs(oracle_mod, acc_o, res_o, parent, M)
    dev = "cuda"
    acc, n, path, nxt = lantern_gpu.verify_trees(st.target_logits.to(dev), st.draft_logits.to(dev),
                                                 torch.from_numpy(row_index).to(dev),
                                                 torch.from_numpy(parent).to(dev).reshape(-1), M,
                                                 torch.from_numpy(tokens).to(dev), torch.from_numpy(table).to(dev),
                                                 delta, un.to(dev))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(acc.cpu().numpy(), acc_o)
    np.testing.assert_array_equal(n.cpu().numpy(), n_o)
    np.testing.assert_array_equal(path.cpu().numpy(), path_o)
    np.testing.assert_array_equal(nxt.cpu().numpy(), next_o)
    assert (acc_o == 0).mean() > 0.3 and (next_o >= 0).sum() > 10


def test_argument_errors(lantern_gpu):
    lib = lantern_gpu.load()
    t = torch.zeros((2, 16), device="cuda")
    tok = torch.zeros(3, dtype=torch.int32, device="cuda")
    knn = torch.arange(16, dtype=torch.int32, device="cuda").reshape(16, 1)
    un = torch.zeros((3, 2), device="cuda")
    # no row_index although R != N
    rc = lib.lantern_decide_rows(t.data_ptr(), t.data_ptr(), 0, 2, 16, 16, None, 3, tok.data_ptr(), knn.data_ptr(), 1,
                                 0, 0.1, un.data_ptr(), tok.data_ptr(), None, None)
    assert rc == -2
    rc = lib.lantern_resample_selected(t.data_ptr(), t.data_ptr(), 0, 3, 16, 16, None, 3, tok.data_ptr(),
                                       knn.data_ptr(), 1, 0, 0.1, un.data_ptr(), None, 2, tok.data_ptr(), None)
    assert rc == -1
    rc = lib.lantern_resample_selected(t.data_ptr(), t.data_ptr(), 0, 3, 16, 16, None, 3, tok.data_ptr(),
                                       knn.data_ptr(), 1, 0, 0.1, un.data_ptr(), tok.data_ptr(), -1, tok.data_ptr(),
                                       None)
    assert rc == -2


# ---- runs of consecutive verifications that share a pair of logit rows (siblings listed together) ----

def _rows_all_modes(oracle, lantern, st, row_index, tokens, un, table, delta, divergence="tvd", threads=8):
    k = table.shape[1]
    acc_o, res_o, _ = oracle.verify_rows(st.target_logits, st.draft_logits, row_index, tokens, table, k, delta, un,
                                         threads=threads, divergence=divergence)
    dev = "cuda"
    args = (st.target_logits.to(dev), st.draft_logits.to(dev), torch.from_numpy(row_index).to(dev),
            torch.from_numpy(tokens).to(dev), torch.from_numpy(np.ascontiguousarray(table)).to(dev), delta,
            un.to(dev))
    acc, res = lantern.verify_rows(*args, divergence=divergence)
    dacc = lantern.decide_rows(*args, divergence=divergence)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(acc.cpu().numpy(), acc_o)
    np.testing.assert_array_equal(res.cpu().numpy(), res_o)
    np.testing.assert_array_equal(dacc.cpu().numpy(), acc_o)
    return acc_o, res_o


@pytest.mark.parametrize("variant,delta", [("plain", 0.4), ("reject", 0.0), ("peaked", 0.01)])
def test_level_ordered_trees(oracle_mod, lantern_gpu, variant, delta):
    """Siblings next to each other, as a drafter that expands a level at a time lists them."""
    from parity_utils import level_order
    cfg = workloads.CONFIGS["llamagen_step"]
    rng = np.random.default_rng(31)
    B, M = 5, 60
    parent = level_order(random_trees(rng, B, M, max_children=6))
    st, row_index, tokens, un = tree_step(cfg, parent, step=11, variant=variant)
    assert (np.diff(row_index) == 0).sum() > B * M // 3          # many runs
    table = sparse_table_from_oracle(oracle_mod, workloads.make_codebook(cfg).numpy(), cfg.k, tokens)
    acc_o, res_o = _rows_all_modes(oracle_mod, lantern_gpu, st, row_index, tokens, un, table, delta)
    n_o, path_o, next_o, _ = _expected_tree_outputs(oracle_mod, acc_o, res_o, parent, M)
    dev = "cuda"
    acc, n, path, nxt = lantern_gpu.verify_trees(st.target_logits.to(dev), st.draft_logits.to(dev),
                                                 torch.from_numpy(row_index).to(dev),
                                                 torch.from_numpy(parent).to(dev).reshape(-1), M,
                                                 torch.from_numpy(tokens).to(dev), torch.from_numpy(table).to(dev),
                                                 delta, un.to(dev))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(acc.cpu().numpy(), acc_o)
    np.testing.assert_array_equal(n.cpu().numpy(), n_o)
    np.testing.assert_array_equal(path.cpu().numpy(), path_o)
    np.testing.assert_array_equal(nxt.cpu().numpy(), next_o)


@pytest.mark.parametrize("cfg_name,divergence", [("tiny", "tvd"), ("tiny", "jsd"), ("llamagen_step", "tvd")])
def test_long_and_odd_runs(oracle_mod, lantern_gpu, cfg_name, divergence):
    """Runs longer than 64, runs across multiples of 64, runs of invalid indices, single members."""
    cfg = workloads.CONFIGS[cfg_name]
    R = 7
    st = workloads.make_step(cfg, step=13, rows=R, variant="reject" if cfg_name == "tiny" else "plain")
    rng = np.random.default_rng(5)
    pieces = [np.full(150, 2), np.full(3, -1), np.array([0, 1, 0, 1]), np.full(70, 5), np.full(2, R), np.full(61, 6),
              np.arange(R), np.full(5, R + 100), np.full(66, 3)]
    row_index = np.concatenate(pieces).astype(np.int32)
    N = len(row_index)
    if cfg_name == "tiny":
        tokens = rng.integers(0, cfg.V, N).astype(np.int32)
        table = oracle_mod.build_knn(workloads.make_codebook(cfg).numpy(), cfg.k, threads=8)
    else:
        top = torch.topk(st.draft_logits.float(), 40, dim=1).indices.numpy()
        safe = np.clip(row_index, 0, R - 1)
        tokens = top[safe, rng.integers(0, 40, N)].astype(np.int32)
        table = sparse_table_from_oracle(oracle_mod, workloads.make_codebook(cfg).numpy(), cfg.k, tokens)
    tokens[20] = -3                                               # an unusable member inside a run
    tokens[160] = cfg.V
    un = torch.from_numpy(rng.random((N, 2)).astype(np.float32))
    un[::2, 0] = 1.0 - 2.0 ** -24                                 # every other member is hard to accept
    for delta in (0.0, cfg.delta):
        acc_o, res_o = _rows_all_modes(oracle_mod, lantern_gpu, st, row_index, tokens, un, table, delta, divergence)
        assert acc_o[20] == -1 and acc_o[150] == -1 and (acc_o == 1).any()
        assert delta > 0 or (acc_o == 0).any()


def test_empty_inputs(lantern_gpu):
    """N = 0, n_sel = 0 and B = 0 launch nothing and report success."""
    dev = "cuda"
    t = torch.zeros((0, 16), device=dev)
    knn = torch.arange(16, dtype=torch.int32, device=dev).reshape(16, 1)
    none_i = torch.zeros(0, dtype=torch.int32, device=dev)
    none_u = torch.zeros((0, 2), device=dev)
    assert lantern_gpu.decide_rows(t, t, None, none_i, knn, 0.1, none_u).numel() == 0
    assert lantern_gpu.verify_rows(t, t, none_i, none_i, knn, 0.1, none_u)[0].numel() == 0
    assert lantern_gpu.verify_greedy_rows(t, none_i, none_i, knn, 0.1)[0].numel() == 0
    acc, n, path, nxt = lantern_gpu.verify_trees(t, t, none_i, none_i, 5, none_i, knn, 0.1, none_u)
    assert acc.numel() == 0 and n.numel() == 0 and path.numel() == 0 and nxt.numel() == 0
    n, path, nxt = lantern_gpu.accept_trees(none_i, none_i, none_i, 7)
    assert n.numel() == 0
    # nothing selected, with verifications present
    t3 = torch.zeros((3, 16), device=dev)
    tok = torch.zeros(3, dtype=torch.int32, device=dev)
    un = torch.zeros((3, 2), device=dev)
    assert lantern_gpu.resample_selected(t3, t3, None, tok, knn, 0.1, un, none_i).numel() == 0
    torch.cuda.synchronize()


def test_chains_through_the_tree_step(oracle_mod, lantern_gpu):
    """A drafted chain is a tree with one child per node and a pair of rows per candidate: the
    fused step without an index array against the oracle's verification and chain walk."""
    cfg = workloads.CONFIGS["llamagen_step"]
    B, L = 12, 8
    st = workloads.make_step(cfg, step=21, rows=B * L, variant="peaked")
    table = sparse_table_from_oracle(oracle_mod, workloads.make_codebook(cfg).numpy(), cfg.k,
                                     st.draft_tokens.numpy())
    delta = 0.05
    acc_o, res_o, _ = oracle_mod.verify(st.target_logits, st.draft_logits, st.draft_tokens, table, cfg.k, delta,
                                        st.uniforms, threads=8)
    kept_o, next_o = oracle_mod.accept_chains(acc_o, res_o, L)
    parent = torch.arange(-1, L - 1, dtype=torch.int32).repeat(B).cuda()
    acc, n, path, nxt = lantern_gpu.verify_trees(st.target_logits.cuda(), st.draft_logits.cuda(), None, parent, L,
                                                 st.draft_tokens.cuda(), torch.from_numpy(table).cuda(), delta,
                                                 st.uniforms.cuda())
    torch.cuda.synchronize()
    np.testing.assert_array_equal(acc.cpu().numpy(), acc_o)
    np.testing.assert_array_equal(n.cpu().numpy(), kept_o)
    np.testing.assert_array_equal(nxt.cpu().numpy(), next_o)
    assert 0 < kept_o.mean() < L


@pytest.mark.parametrize("V,k,dtype", [(1003, 50, torch.bfloat16), (7, 7, torch.float32), (40000, 64, torch.float32)])
def test_shared_rows_off_the_fast_path(oracle_mod, lantern_gpu, V, k, dtype):
    """Shapes that only the fp64 kernels take (odd vocabulary, rows beyond the register budget), with an
    index array, in all three modes and through the tree step."""
    rng = np.random.default_rng(V)
    R, B, M = 5, 3, 6
    t = torch.from_numpy((rng.standard_normal((R, V)) * 2).astype(np.float32)).to(dtype)
    g = (t.float() + torch.from_numpy(rng.standard_normal((R, V)).astype(np.float32))).to(dtype)
    st = workloads.Step(target_logits=t, draft_logits=g, draft_tokens=None, uniforms=None)
    parent = random_trees(rng, B, M, max_children=3)
    N = B * M
    row_index = rng.integers(0, R, N).astype(np.int32)
    row_index[4] = R
    tokens = rng.integers(0, V, N).astype(np.int32)
    un = torch.from_numpy(rng.random((N, 2)).astype(np.float32))
    table = random_table(V, k, seed=V + 1)
    for delta in (0.0, 0.2):
        acc_o, res_o = _rows_all_modes(oracle_mod, lantern_gpu, st, row_index, tokens, un, table, delta)
        n_o, path_o, next_o, _ = _expected_tree_outputs(oracle_mod, acc_o, res_o, parent, M)
        acc, n, path, nxt = lantern_gpu.verify_trees(t.cuda(), g.cuda(), torch.from_numpy(row_index).cuda(),
                                                     torch.from_numpy(parent).cuda().reshape(-1), M,
                                                     torch.from_numpy(tokens).cuda(), torch.from_numpy(table).cuda(),
                                                     delta, un.cuda())
        torch.cuda.synchronize()
        np.testing.assert_array_equal(acc.cpu().numpy(), acc_o)
        np.testing.assert_array_equal(n.cpu().numpy(), n_o)
        np.testing.assert_array_equal(path.cpu().numpy(), path_o)
        np.testing.assert_array_equal(nxt.cpu().numpy(), next_o)
