"""GPU parity of the Jensen-Shannon-bounded neighbourhood (lantern_verify_divergence) against the oracle."""
import numpy as np
import pytest
import torch

from synth import philox, workloads
from parity_utils import compare_verify, random_table

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("delta", [0.0, 0.002, 0.02, 0.1, 0.5, 0.7])
def test_tiny(oracle_mod, lantern_gpu, delta):
    cfg = workloads.CONFIGS["tiny"]
    cb = workloads.make_codebook(cfg)
    table = oracle_mod.build_knn(cb.numpy(), cfg.k, threads=8)
    st = workloads.make_step(cfg, step=31)
    acc, res, diag, g = compare_verify(oracle_mod, lantern_gpu, st.target_logits, st.draft_logits, st.draft_tokens,
                                       table, delta, st.uniforms, label=f"tiny jsd {delta}", divergence="jsd")
    if delta == 0.0:
        assert np.all(diag["a_size"] == 1)
    if delta == 0.7:                       # JSD never reaches ln 2
        assert np.all(diag["a_size"] == cfg.k)


@pytest.mark.parametrize("name,variant,delta", [
    ("llamagen_step", "plain", 0.2),       # the bound the paper uses with JSD
    ("llamagen_step", "plain", 0.01),
    ("llamagen_step", "peaked", 0.005),
    ("llamagen_step", "reject", 0.0),
    ("wide_latent", "plain", 0.003),
    ("wide_latent", "peaked", 0.02),
])
def test_full_width_rows(oracle_mod, lantern_gpu, name, variant, delta):
    cfg = workloads.CONFIGS[name]
    st = workloads.make_step(cfg, step=5, rows=384, variant=variant)
    table = random_table(cfg.V, cfg.k, seed=21)
    acc, res, diag, g = compare_verify(oracle_mod, lantern_gpu, st.target_logits, st.draft_logits, st.draft_tokens,
                                       table, delta, st.uniforms, threads=16, label=f"{name} {variant} jsd {delta}",
                                       divergence="jsd")
    if delta in (0.01, 0.005, 0.003, 0.02):
        assert (diag["a_size"] < cfg.k).sum() > 0      # the bound cuts some neighbourhoods
        assert (diag["a_size"] > 1).sum() > 0


@pytest.mark.parametrize("V,k,N,dtype", [(7, 7, 5, torch.float32), (1003, 50, 20, torch.bfloat16),
                                         (4096, 2500, 9, torch.bfloat16), (40000, 100, 5, torch.float32)])
def test_shapes(oracle_mod, lantern_gpu, V, k, N, dtype):
    rng = np.random.default_rng(V + k)
    t = torch.from_numpy((rng.standard_normal((N, V)) * 2.5).astype(np.float32))
    g = (t + torch.from_numpy(rng.standard_normal((N, V)).astype(np.float32))).to(dtype)
    t = t.to(dtype)
    tokens = torch.from_numpy(rng.integers(0, V, N).astype(np.int32))
    table = random_table(V, k, seed=V)
    un = torch.from_numpy(philox.uniforms(V, N))
    for delta in (0.01, 0.15):
        compare_verify(oracle_mod, lantern_gpu, t, g, tokens, table, delta, un, label=f"V={V} jsd",
                       divergence="jsd")


def test_unknown_divergence_is_rejected(lantern_gpu):
    import ctypes
    lib = lantern_gpu.load()
    p = ctypes.c_void_p(4096)
    rc = lib.lantern_verify_divergence(p, p, 0, 4, 16, 16, p, p, 4, 7, 0.1, p, p, p, None, None, None, None, None,
                                       None)
    assert rc == lantern_gpu.binding.E_SHAPE


@pytest.mark.parametrize("divergence,delta", [("tvd", 0.3), ("jsd", 0.15), ("tvd", 0.9), ("jsd", 0.6)])
def test_cut_beyond_the_first_1024_slots(oracle_mod, lantern_gpu, divergence, delta):
    """Long neighbourhoods: the walk passes the 1024 slots the workgroup scans together and ends (or
    does not end) in the part one wavefront walks alone."""
    V, k, N = 8192, 4000, 24
    rng = np.random.default_rng(11)
    t = torch.from_numpy((rng.standard_normal((N, V)) * 1.0).astype(np.float32)).to(torch.bfloat16)
    g = (t.float() + torch.from_numpy(rng.standard_normal((N, V)).astype(np.float32) * 0.5)).to(torch.bfloat16)
    tokens = torch.from_numpy(rng.integers(0, V, N).astype(np.int32))
    table = random_table(V, k, seed=21)
    un = torch.from_numpy(philox.uniforms(5, N))
    acc, res, diag, gout = compare_verify(oracle_mod, lantern_gpu, t, g, tokens, table, delta, un,
                                          label=f"long walk {divergence}", divergence=divergence)
    sizes = diag["a_size"]
    assert (sizes > 1024).any()
    if delta < 0.5:
        assert (sizes < k).any()          # the cut itself lies beyond slot 1024
    assert (gout["path"] == 0).any()      # and the fp32 pass settles such rows


@pytest.mark.parametrize("V,k,N,dtype,scale", [(2174, 255, 513, torch.float32, 30.0), (8, 8, 513, torch.float32, 8.0),
                                               (20496, 1025, 512, torch.float32, 30.0),
                                               (16384, 2019, 512, torch.bfloat16, 30.0)])
def test_a_bound_of_zero_takes_no_neighbour(oracle_mod, lantern_gpu, V, k, N, dtype, scale):
    """Widely spread logits put neighbours at 1e-17 of t(xt) and below, where the evaluated divergence is all
    rounding error; with a bound of zero neither side may take one."""
    g = torch.Generator().manual_seed(V + k)
    tl = torch.randn(N, V, generator=g) * scale
    dl = tl + torch.randn(N, V, generator=g) * scale
    tok = tl.argmax(dim=1).to(torch.int32)          # t(xt) large: the neighbours' terms are far below its last place
    tok[::3] = torch.randint(0, V, (len(tok[::3]),), generator=g, dtype=torch.int32)
    table = random_table(V, k, seed=5)
    un = torch.from_numpy(philox.uniforms(77, N, stream=3))
    acc, res, diag, out = compare_verify(oracle_mod, lantern_gpu, tl.to(dtype), dl.to(dtype), tok, table, 0.0, un,
                                         threads=16, label=f"jsd zero bound V={V}", divergence="jsd")
    assert np.all(diag["a_size"] == 1) and np.all(out["a_size"] == 1)
