"""GPU parity of lantern_verify_trees_sequential (siblings verified one after the other against
the residual of those before) against the CPU oracle's walk of the same rule, through the C ABI:
lengths, paths and the token that follows, element by element."""
import numpy as np
import pytest
import torch

from synth import workloads
from parity_utils import level_order, random_table, random_trees, tree_step

pytestmark = pytest.mark.gpu


def _both(oracle, lantern, st, row_index, parent, M, tokens, un, table, delta, divergence="tvd", threads=8):
    k = table.shape[1]
    n_o, path_o, next_o = oracle.verify_trees_sequential(st.target_logits, st.draft_logits, row_index, parent, M,
                                                         tokens, table, k, delta, un, threads=threads,
                                                         divergence=divergence)
    n, path, nxt = lantern.verify_trees_sequential(
        st.target_logits.cuda(), st.draft_logits.cuda(), torch.from_numpy(np.ascontiguousarray(row_index)).cuda(),
        torch.from_numpy(np.ascontiguousarray(parent)).cuda().reshape(-1), M,
        torch.from_numpy(np.ascontiguousarray(tokens)).cuda(), torch.from_numpy(np.ascontiguousarray(table)).cuda(),
        delta, un.cuda(), divergence=divergence)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(n.cpu().numpy(), n_o)
    np.testing.assert_array_equal(path.cpu().numpy(), path_o)
    np.testing.assert_array_equal(nxt.cpu().numpy(), next_o)
    return n_o, path_o, next_o


@pytest.mark.parametrize("divergence", ["tvd", "jsd"])
@pytest.mark.parametrize("variant", ["plain", "reject", "peaked"])
def test_tiny_trees(oracle_mod, lantern_gpu, variant, divergence):
    cfg = workloads.CONFIGS["tiny"]
    cb = workloads.make_codebook(cfg)
    table = oracle_mod.build_knn(cb.numpy(), cfg.k, threads=8)
    rng = np.random.default_rng(21)
    B, M = 40, 11
    parent = random_trees(rng, B, M, max_children=3)
    rejected_then_taken = 0
    for step in range(3):
        st, row_index, tokens, un = tree_step(cfg, parent, step=step, variant=variant)
        delta = 0.02 if divergence == "jsd" else cfg.delta
        n, path, nxt = _both(oracle_mod, lantern_gpu, st, row_index, parent, M, tokens, un, table, delta, divergence)
        # a later sibling taken: the residual target was in play
        for b in range(B):
            for j in range(n[b]):
                node = path[b, j]
                sibs = np.nonzero(parent[b] == parent[b, node])[0]
                rejected_then_taken += int(node != sibs[0])
    if variant != "plain":
        assert rejected_then_taken > 0


@pytest.mark.parametrize("name,B,M", [("llamagen_step", 6, 60), ("stress", 8, 60), ("wide_latent", 5, 60),
                                      ("image_batch", 4, 24)])
def test_configured_shapes(oracle_mod, lantern_gpu, name, B, M):
    """The paper's step shape (60 candidates per tree) on the configured vocabularies, table widths and
    logit types (bf16 and, for wide_latent, fp32), trees in level order and in drafting order, a mix that
    accepts often and one that rejects often."""
    cfg = workloads.CONFIGS[name]
    table = random_table(cfg.V, cfg.k, seed=17)
    rng = np.random.default_rng(5)
    parent = random_trees(rng, B, M, max_children=4)
    longest = 0
    for step, (variant, par) in enumerate((("plain", parent), ("reject", level_order(parent)), ("peaked", parent))):
        st, row_index, tokens, un = tree_step(cfg, par, step=30 + step, variant=variant)
        delta = 0.05 if variant == "reject" else cfg.delta
        n, _, nxt = _both(oracle_mod, lantern_gpu, st, row_index, par, M, tokens, un, table, delta)
        longest = max(longest, int(n.max()))
        assert (nxt >= -1).all()
    assert longest >= 2


def test_k1_is_plain_speculative_sampling(oracle_mod, lantern_gpu):
    """k = 1: the neighbourhood is the token itself, every residual is max(0, t_j - g) / Z."""
    cfg = workloads.CONFIGS["tiny"]
    table = np.arange(cfg.V, dtype=np.int32).reshape(cfg.V, 1)
    rng = np.random.default_rng(3)
    B, M = 64, 6
    parent = np.full((B, M), -1, dtype=np.int32)          # six candidates for the first position
    st, row_index, tokens, un = tree_step(cfg, parent, step=9, variant="reject")
    n, path, nxt = _both(oracle_mod, lantern_gpu, st, row_index, parent, M, tokens, un, table, 0.0)
    assert (n <= 1).all() and (nxt[n == 0] >= 0).all() and (nxt[n == 1] == -1).all()
    assert (n == 0).any() and (path[n == 1, 0] > 0).any()


def test_chains_without_row_index(oracle_mod, lantern_gpu):
    """One child per node and a pair of rows per candidate: the rule is Algorithm 1 on a chain."""
    cfg = workloads.CONFIGS["tiny"]
    cb = workloads.make_codebook(cfg)
    table = oracle_mod.build_knn(cb.numpy(), cfg.k, threads=8)
    B, L = 30, 7
    st = workloads.make_step(cfg, step=12, rows=B * L, variant="peaked")
    parent = np.tile(np.arange(-1, L - 1, dtype=np.int32), (B, 1))
    row_index = np.arange(B * L, dtype=np.int32)
    n_o, path_o, next_o = oracle_mod.verify_trees_sequential(st.target_logits, st.draft_logits, row_index, parent, L,
                                                             st.draft_tokens.numpy(), table, cfg.k, cfg.delta,
                                                             st.uniforms, threads=8)
    n, path, nxt = lantern_gpu.verify_trees_sequential(st.target_logits.cuda(), st.draft_logits.cuda(), None,
                                                       torch.from_numpy(parent).cuda().reshape(-1), L,
                                                       st.draft_tokens.cuda(), torch.from_numpy(table).cuda(),
                                                       cfg.delta, st.uniforms.cuda())
    torch.cuda.synchronize()
    np.testing.assert_array_equal(n.cpu().numpy(), n_o)
    np.testing.assert_array_equal(path.cpu().numpy(), path_o)
    np.testing.assert_array_equal(nxt.cpu().numpy(), next_o)
    # the same chains through the row-parallel path and the chain walk
    acc, res, _ = oracle_mod.verify(st.target_logits, st.draft_logits, st.draft_tokens, table, cfg.k, cfg.delta,
                                    st.uniforms, threads=8)
    kept, nxt_c = oracle_mod.accept_chains(acc, res, L)
    np.testing.assert_array_equal(n_o, kept)
    np.testing.assert_array_equal(next_o, nxt_c)


def test_unusable_and_malformed(oracle_mod, lantern_gpu):
    cfg = workloads.CONFIGS["tiny"]
    table = random_table(cfg.V, cfg.k, seed=4).copy()
    rng = np.random.default_rng(11)
    B, M = 16, 8
    parent = random_trees(rng, B, M, max_children=3)
    st, row_index, tokens, un = tree_step(cfg, parent, step=2, variant="reject")
    row_index = row_index.copy()
    tokens = tokens.copy()
    tl = st.target_logits.clone()
    dl = st.draft_logits.clone()
    roots = [np.nonzero(parent[b] == -1)[0] for b in range(B)]
    parent = parent.copy()
    parent[0, 3] = 3                                        # malformed: own parent
    parent[1, 0] = -2
    row_index[2 * M + roots[2][0]] = -1                     # first child's row out of range
    row_index[3 * M + roots[3][0]] = B * (M + 1)
    tokens[4 * M + roots[4][0]] = cfg.V                     # token out of range
    tokens[5 * M + roots[5][0]] = -1
    tl[row_index[6 * M + roots[6][0]], 5] = float("nan")    # unusable target row
    dl[row_index[7 * M + roots[7][0]], 9] = float("inf")    # unusable drafter row
    tl[row_index[8 * M + roots[8][0]], :] = float("-inf")   # no finite logit
    if roots[9].size > 1:
        row_index[9 * M + roots[9][1]] += 1                 # a sibling on another row
    table[tokens[10 * M + roots[10][0]], cfg.k - 1] = cfg.V  # table entry out of range
    table[tokens[11 * M + roots[11][0]], 0] = -1
    k = cfg.k
    n_o, path_o, next_o = oracle_mod.verify_trees_sequential(tl, dl, row_index, parent, M, tokens, table, k, 0.0, un,
                                                             threads=4)
    n, path, nxt = lantern_gpu.verify_trees_sequential(tl.cuda(), dl.cuda(), torch.from_numpy(row_index).cuda(),
                                                       torch.from_numpy(parent).cuda().reshape(-1), M,
                                                       torch.from_numpy(tokens).cuda(), torch.from_numpy(table).cuda(),
                                                       0.0, un.cuda())
    torch.cuda.synchronize()
    np.testing.assert_array_equal(n.cpu().numpy(), n_o)
    np.testing.assert_array_equal(path.cpu().numpy(), path_o)
    np.testing.assert_array_equal(nxt.cpu().numpy(), next_o)
    assert list(next_o[:2]) == [-3, -3]
    assert (next_o[2:9] == -2).all() and (next_o[10:12] == -2).all()


def test_single_candidate_large_vocabulary_and_empty(oracle_mod, lantern_gpu):
    """M = 1, a vocabulary that is no multiple of the wavefront size, k above one scan block; B = 0."""
    V, k, B = 5003, 1500, 7
    rng = np.random.default_rng(8)
    table = random_table(V, k, seed=9)
    tl = torch.from_numpy(rng.normal(0, 3, (B, V)).astype(np.float32))
    dl = torch.from_numpy((tl.numpy() + rng.normal(0, 1.5, (B, V))).astype(np.float32))
    tokens = dl.argmax(dim=1).to(torch.int32).numpy()
    parent = np.full((B, 1), -1, dtype=np.int32)
    un = torch.from_numpy(rng.random((B, 2)).astype(np.float32))
    un[:4, 0] = 0.999                                       # rejected unless the mass is nearly g(xt)
    row_index = np.arange(B, dtype=np.int32)
    for delta in (0.0, 0.02, 0.3):
        n_o, path_o, next_o = oracle_mod.verify_trees_sequential(tl, dl, row_index, parent, 1, tokens, table, k, delta,
                                                                 un, threads=4)
        n, path, nxt = lantern_gpu.verify_trees_sequential(tl.cuda(), dl.cuda(), torch.from_numpy(row_index).cuda(),
                                                           torch.from_numpy(parent).cuda().reshape(-1), 1,
                                                           torch.from_numpy(tokens).cuda(),
                                                           torch.from_numpy(table).cuda(), delta, un.cuda())
        torch.cuda.synchronize()
        np.testing.assert_array_equal(n.cpu().numpy(), n_o)
        np.testing.assert_array_equal(path.cpu().numpy(), path_o)
        np.testing.assert_array_equal(nxt.cpu().numpy(), next_o)
    empty = torch.empty(0, dtype=torch.int32, device="cuda")
    n, path, nxt = lantern_gpu.verify_trees_sequential(tl.cuda(), dl.cuda(), empty, empty, 1, empty,
                                                       torch.from_numpy(table).cuda(), 0.1,
                                                       torch.empty((0, 2), dtype=torch.float32, device="cuda"))
    assert n.numel() == 0 and path.numel() == 0 and nxt.numel() == 0


def test_bench_step_size(oracle_mod, lantern_gpu):
    """The step bench.py times in mode tree_seq: 64 trees of 60 candidates listed level by level on the
    stress shape, the table built from the workload's own codebook, the reject and peaked mixes."""
    cfg = workloads.CONFIGS["stress"]
    cb = workloads.make_codebook(cfg, device="cuda:0")
    knn = lantern_gpu.build_knn(cb, cfg.k)
    table = knn.cpu().numpy()
    B, M = 64, 60
    parent = level_order(random_trees(np.random.default_rng(workloads.BASE_SEED), B, M))
    for variant, delta in (("reject", 0.0), ("peaked", cfg.delta), ("plain", cfg.delta)):
        st, row_index, tokens, un = tree_step(cfg, parent, step=0, variant=variant)
        n, path, nxt = _both(oracle_mod, lantern_gpu, st, row_index, parent, M, tokens, un, table, delta, threads=16)
        if variant == "plain":
            assert n.mean() > 3


def test_capture_and_replay(oracle_mod, lantern_gpu):
    """The call only enqueues kernels on the caller's stream: captured into a HIP graph and replayed on
    new inputs, every replay equals the oracle."""
    cfg = workloads.CONFIGS["tiny"]
    table = random_table(cfg.V, cfg.k, seed=12)
    tb = torch.from_numpy(table).cuda()
    B, M = 24, 9
    parent = random_trees(np.random.default_rng(4), B, M, max_children=3)
    par_d = torch.from_numpy(parent).cuda().reshape(-1)
    steps = [tree_step(cfg, parent, step=s, variant=v) for s, v in ((1, "reject"), (2, "peaked"), (3, "plain"))]
    R = B * (M + 1)
    tl = torch.empty((R, cfg.V), dtype=steps[0][0].target_logits.dtype, device="cuda")
    dl = torch.empty_like(tl)
    ri = torch.empty(B * M, dtype=torch.int32, device="cuda")
    tok = torch.empty(B * M, dtype=torch.int32, device="cuda")
    un = torch.empty((B * M, 2), dtype=torch.float32, device="cuda")
    work = torch.empty(lantern_gpu.trees_sequential_workspace_bytes(B, M, cfg.V), dtype=torch.uint8, device="cuda")

    def load(step):
        st, row_index, tokens, uniforms = step
        tl.copy_(st.target_logits); dl.copy_(st.draft_logits)
        ri.copy_(torch.from_numpy(row_index)); tok.copy_(torch.from_numpy(tokens)); un.copy_(uniforms)

    delta = 0.05
    load(steps[0])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm up outside the capture
        lantern_gpu.verify_trees_sequential(tl, dl, ri, par_d, M, tok, tb, delta, un, workspace=work, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        n, path, nxt = lantern_gpu.verify_trees_sequential(tl, dl, ri, par_d, M, tok, tb, delta, un, workspace=work,
                                                           stream=torch.cuda.current_stream())
    for step in (steps[1], steps[2], steps[0], steps[1]):
        load(step)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        st, row_index, tokens, uniforms = step
        n_o, path_o, next_o = oracle_mod.verify_trees_sequential(st.target_logits, st.draft_logits, row_index, parent,
                                                                 M, tokens, table, cfg.k, delta, uniforms, threads=8)
        np.testing.assert_array_equal(n.cpu().numpy(), n_o)
        np.testing.assert_array_equal(path.cpu().numpy(), path_o)
        np.testing.assert_array_equal(nxt.cpu().numpy(), next_o)


@pytest.mark.parametrize("V,k,dtype", [(24001, 700, torch.float32), (1 << 19, 64, torch.bfloat16)])
def test_vocabularies_beyond_the_lds_copy(oracle_mod, lantern_gpu, V, k, dtype):
    """Beyond 19200 tokens the current target no longer fits in LDS and lives in the workspace; up to the
    largest vocabulary the library takes.  Children drafted as the drafter's most likely tokens, draws
    that reject often."""
    rng = np.random.default_rng(V)
    B, M = 3, 7
    parent = random_trees(rng, B, M, max_children=3)
    R = B * (M + 1)
    tl = torch.from_numpy(rng.normal(0, 2.5, (R, V)).astype(np.float32)).to(dtype)
    dl = torch.from_numpy((tl.float().numpy() + rng.normal(0, 1.0, (R, V))).astype(np.float32)).to(dtype)
    row_index = (np.arange(B, dtype=np.int64)[:, None] * (M + 1) + parent + 1).astype(np.int32).reshape(-1)
    rank = np.zeros((B, M), dtype=np.int64)
    for b in range(B):
        seen = {}
        for i in range(M):
            rank[b, i] = seen.get(parent[b, i], 0)
            seen[parent[b, i]] = rank[b, i] + 1
    top = torch.topk(dl.float(), int(rank.max()) + 1, dim=1).indices.numpy()
    tokens = top[row_index, rank.reshape(-1)].astype(np.int32)
    # every row valid (the token itself, then its successors); the rows of the drafted tokens random
    table = ((np.arange(V, dtype=np.int64)[:, None] + np.arange(k, dtype=np.int64)[None, :]) % V).astype(np.int32)
    for x in set(int(t) for t in tokens):
        others = rng.choice(V - 1, size=k - 1, replace=False)
        table[x, 1:] = others + (others >= x)
    un = torch.from_numpy(rng.random((B * M, 2)).astype(np.float32))
    un[::2, 0] = 0.9999
    resampled = 0
    for delta in (0.0, 0.1):
        n_o, path_o, next_o = oracle_mod.verify_trees_sequential(tl, dl, row_index, parent, M, tokens, table, k, delta,
                                                                 un, threads=8)
        n, path, nxt = lantern_gpu.verify_trees_sequential(tl.cuda(), dl.cuda(), torch.from_numpy(row_index).cuda(),
                                                           torch.from_numpy(parent).cuda().reshape(-1), M,
                                                           torch.from_numpy(tokens).cuda(),
                                                           torch.from_numpy(table).cuda(), delta, un.cuda())
        torch.cuda.synchronize()
        np.testing.assert_array_equal(n.cpu().numpy(), n_o)
        np.testing.assert_array_equal(path.cpu().numpy(), path_o)
        np.testing.assert_array_equal(nxt.cpu().numpy(), next_o)
        resampled += int((next_o >= 0).sum())
    assert resampled > 0
