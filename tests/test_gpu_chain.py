"""GPU parity of lantern_accept_chains (the loop of Algorithm 1 over a drafted chain)."""
import numpy as np
import pytest
import torch

from synth import workloads
from parity_utils import random_table

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("B,L", [(1, 1), (7, 5), (64, 60), (300, 64), (33, 130)])
def test_random_patterns(oracle_mod, lantern_gpu, B, L):
    rng = np.random.default_rng(B * 1000 + L)
    accept = (rng.random((B, L)) < 0.85).astype(np.int32)
    accept[rng.random((B, L)) < 0.02] = -1                       # a few unusable rows
    resample = np.where(accept == 0, rng.integers(0, 16384, (B, L)), -1).astype(np.int32)
    want_n, want_next = oracle_mod.accept_chains(accept, resample, L)
    n, nxt = lantern_gpu.accept_chains(torch.from_numpy(accept).cuda().reshape(-1),
                                       torch.from_numpy(resample).cuda().reshape(-1), L)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(n.cpu().numpy(), want_n)
    np.testing.assert_array_equal(nxt.cpu().numpy(), want_next)


def test_chain_of_verifications(oracle_mod, lantern_gpu):
    """64 chains of 6 drafted candidates verified on the device, then walked on the device."""
    cfg = workloads.CONFIGS["tiny"]
    L, B = 6, 64
    st = workloads.make_step(cfg, step=21, rows=B * L)
    table = random_table(cfg.V, cfg.k, seed=4)
    tb = torch.from_numpy(table).cuda()
    acc, res = lantern_gpu.verify(st.target_logits.cuda(), st.draft_logits.cuda(), st.draft_tokens.cuda(), tb,
                                  cfg.delta, st.uniforms.cuda())
    n, nxt = lantern_gpu.accept_chains(acc, res, L)
    torch.cuda.synchronize()
    acc_o, res_o, _ = oracle_mod.verify(st.target_logits, st.draft_logits, st.draft_tokens, table, cfg.k,
                                        cfg.delta, st.uniforms, threads=8)
    want_n, want_next = oracle_mod.accept_chains(acc_o, res_o, L)
    np.testing.assert_array_equal(n.cpu().numpy(), want_n)
    np.testing.assert_array_equal(nxt.cpu().numpy(), want_next)
    assert want_n.min() < L and want_n.max() > 0


def test_empty(lantern_gpu):
    e = torch.empty(0, dtype=torch.int32, device="cuda")
    n, nxt = lantern_gpu.accept_chains(e, e, 4)
    assert n.numel() == 0 and nxt.numel() == 0
