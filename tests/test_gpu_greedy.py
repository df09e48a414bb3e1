"""GPU parity of lantern_verify_greedy against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from synth import workloads
from parity_utils import random_table, sparse_table_from_oracle

pytestmark = pytest.mark.gpu


def _compare(oracle, lantern, target, tokens, table, delta, label="", threads=8):
    k = table.shape[1]
    acc_o, tok_o, diag = oracle.verify_greedy(target, tokens, table, k, delta, threads=threads)
    acc, tok, path = lantern.verify_greedy(target.cuda(), tokens.cuda(),
                                           torch.from_numpy(np.ascontiguousarray(table)).cuda(), delta,
                                           want_path=True)
    torch.cuda.synchronize()
    acc, tok, path = acc.cpu().numpy(), tok.cpu().numpy(), path.cpu().numpy()
    bad = np.nonzero((acc != acc_o) | (tok != tok_o))[0]
    if bad.size:
        i = int(bad[0])
        raise AssertionError(f"{label}: {bad.size} rows differ; first row {i}: gpu {acc[i]}/{tok[i]} "
                             f"oracle {acc_o[i]}/{tok_o[i]} mass={diag['mass'][i]:.6e} "
                             f"other={diag['other'][i]:.6e} path={path[i]}")
    return acc_o, tok_o, diag, path


def _drafts_near_the_top(target, rng, spread=4):
    """Draft tokens among the few most likely target tokens, so acceptances occur."""
    order = torch.argsort(target.float(), dim=1, descending=True)[:, :spread].numpy()
    pick = rng.integers(0, spread, order.shape[0])
    return torch.from_numpy(order[np.arange(order.shape[0]), pick].astype(np.int32))


@pytest.mark.parametrize("delta,k_use", [(0.0, 16), (0.1, 1), (0.1, 16), (0.5, 16), (2.0, 16)])
def test_tiny(oracle_mod, lantern_gpu, delta, k_use):
    cfg = workloads.CONFIGS["tiny"]
    cb = workloads.make_codebook(cfg)
    table = oracle_mod.build_knn(cb.numpy(), k_use, threads=8)
    st = workloads.make_step(cfg, step=5)
    rng = np.random.default_rng(1)
    tokens = _drafts_near_the_top(st.target_logits, rng)
    acc, tok, diag, path = _compare(oracle_mod, lantern_gpu, st.target_logits, tokens, table, delta, "tiny")
    assert (acc == 1).sum() > 0 and (acc == 0).sum() > 0
    if delta == 0.0 or k_use == 1:   # plain greedy verification
        best = st.target_logits.argmax(dim=1).numpy()
        np.testing.assert_array_equal(acc, (best == tokens.numpy()).astype(np.int32))


@pytest.mark.parametrize("variant,delta", [("plain", 0.4), ("plain", 0.002), ("peaked", 0.01), ("peaked", 0.3)])
def test_llamagen_shape(oracle_mod, lantern_gpu, variant, delta):
    """V=16384, k=1000, bf16 logits (many exactly equal logits: ties are exercised)."""
    cfg = workloads.CONFIGS["llamagen_step"]
    st = workloads.make_step(cfg, step=3, rows=240, variant=variant)
    rng = np.random.default_rng(2)
    tokens = _drafts_near_the_top(st.target_logits, rng, spread=3)
    tokens[::5] = st.draft_tokens[::5]                     # some arbitrary drafts as well
    cb = workloads.make_codebook(cfg)
    table = sparse_table_from_oracle(oracle_mod, cb.numpy(), cfg.k, tokens.numpy())
    acc, tok, diag, path = _compare(oracle_mod, lantern_gpu, st.target_logits, tokens, table, delta,
                                    f"llamagen {variant} {delta}")
    assert (path == 0).mean() > 0.5                        # the fp32 path settles most rows


def test_stress_full_step(oracle_mod, lantern_gpu):
    cfg = workloads.CONFIGS["stress"]
    st = workloads.make_step(cfg, step=11)
    rng = np.random.default_rng(3)
    tokens = _drafts_near_the_top(st.target_logits, rng, spread=2)
    table = random_table(cfg.V, cfg.k, seed=8)
    # at delta = 0.4 a random 1000-token neighbourhood outweighs any single token: everything is accepted
    acc, tok, diag, path = _compare(oracle_mod, lantern_gpu, st.target_logits, tokens, table, cfg.delta,
                                    "stress", threads=16)
    assert len(acc) == 3840 and (acc == 1).all()
    # a bound of the size of the top probabilities gives a mix of both outcomes
    acc, tok, diag, path = _compare(oracle_mod, lantern_gpu, st.target_logits, tokens, table, 0.003,
                                    "stress small delta", threads=16)
    assert (acc == 1).sum() > 100 and (acc == 0).sum() > 100


def test_wide_latent_fp32(oracle_mod, lantern_gpu):
    cfg = workloads.CONFIGS["wide_latent"]
    st = workloads.make_step(cfg, step=1, rows=512)
    rng = np.random.default_rng(4)
    tokens = _drafts_near_the_top(st.target_logits, rng)
    table = random_table(cfg.V, cfg.k, seed=9)
    for delta in (0.0, 0.05, cfg.delta):
        _compare(oracle_mod, lantern_gpu, st.target_logits, tokens, table, delta, f"wide {delta}")


@pytest.mark.parametrize("V,k,N,dtype", [
    (1, 1, 3, torch.float32),
    (7, 7, 5, torch.float32),
    (1000, 33, 37, torch.float32),
    (1003, 50, 20, torch.bfloat16),
    (4096, 2500, 9, torch.bfloat16),
    (2048, 2048, 4, torch.float32),    # k = V: nothing is left outside A
    (32768, 64, 6, torch.bfloat16),
    (40000, 100, 5, torch.float32),
])
def test_shapes(oracle_mod, lantern_gpu, V, k, N, dtype):
    rng = np.random.default_rng(V * 3 + k)
    t = torch.from_numpy((rng.standard_normal((N, V)) * 2.5).astype(np.float32)).to(dtype)
    tokens = _drafts_near_the_top(t, rng, spread=min(3, V))
    table = random_table(V, k, seed=V + k)
    for delta in (0.05, 0.3, 1.5):
        _compare(oracle_mod, lantern_gpu, t, tokens, table, delta, f"V={V} k={k} d={delta}")


def test_ties_and_unusable_rows(oracle_mod, lantern_gpu):
    rng = np.random.default_rng(6)
    N, V, k = 12, 4096, 32
    t = np.clip(np.round(rng.standard_normal((N, V)) * 2), -5, 5).astype(np.float32)  # many tied maxima
    tied = [np.flatnonzero(t[i] == t[i].max()) for i in range(N)]
    tokens = np.array([int(m[rng.integers(0, min(3, len(m)))]) for m in tied], dtype=np.int32)
    table = random_table(V, k, seed=12)
    t[8, 17] = np.nan
    t[9, :] = -np.inf
    tokens[10] = V + 3
    table[tokens[11], 3] = -7
    acc, tok, diag, path = _compare(oracle_mod, lantern_gpu, torch.from_numpy(t), torch.from_numpy(tokens),
                                    table, 0.0, "ties")
    assert list(acc[8:]) == [-1] * 4 and list(tok[8:]) == [-1] * 4
    assert set(acc[:8]) <= {0, 1}
