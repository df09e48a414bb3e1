"""Shared helpers of the GPU parity tests: run the oracle and the HIP library on
the same seeded inputs and compare element by element."""
from __future__ import annotations

import numpy as np
import torch

from synth.trees import level_order, random_trees, tree_step  # noqa: F401  (used by the tree tests)

# tolerance on probabilities and acceptance ratios: 1e-5 relative for fp32
# logits, 2e-3 for bf16 logits (decisions and indices are compared exactly)
PROB_TOL = {torch.float32: 1e-5, torch.bfloat16: 2e-3}


def sparse_table_from_oracle(oracle, codebook, k, tokens, fill_rows=None, threads=8):
    """[V, k] table whose rows for `tokens` come from the oracle's neighbour
    search; the other rows (never read by verification of these tokens) hold the
    token itself followed by the next k-1 tokens cyclically."""
    V = codebook.shape[0]
    base = (np.arange(V, dtype=np.int64)[:, None] + np.arange(k, dtype=np.int64)[None, :]) % V
    table = base.astype(np.int32)
    for x in sorted(set(int(t) for t in tokens if 0 <= int(t) < V)):
        table[x] = oracle.build_knn(codebook, k, rows=(x, x + 1), threads=1)[0]
    return table


def random_table(V, k, seed):
    """Self first, then k-1 distinct other tokens in random order."""
    rng = np.random.default_rng(seed)
    table = np.empty((V, k), dtype=np.int32)
    for x in range(V):
        others = rng.permutation(V - 1)[: k - 1]
        others = others + (others >= x)
        table[x, 0] = x
        table[x, 1:] = others
    return table


def compare_verify(oracle, lantern, target, draft, tokens, table, delta, uniforms, threads=8,
                   label="", divergence="tvd"):
    """Runs both sides; asserts exact decisions / tokens / set sizes and
    tolerance-level probabilities.  Returns (oracle diag, gpu outputs)."""
    k = table.shape[1]
    acc_o, res_o, diag = oracle.verify(target, draft, tokens, table, k, delta, uniforms, threads=threads,
                                       divergence=divergence)
    dev = "cuda"
    out = lantern.verify_ex(target.to(dev), draft.to(dev), tokens.to(dev),
                            torch.from_numpy(np.ascontiguousarray(table)).to(dev), delta,
                            uniforms.to(dev), divergence=divergence)
    torch.cuda.synchronize()
    g = {n: v.cpu().numpy() for n, v in out.items()}
    if divergence == "tvd":
        # the plain entry point must agree with the diagnostic one
        acc2, res2 = lantern.verify(target.to(dev), draft.to(dev), tokens.to(dev),
                                    torch.from_numpy(np.ascontiguousarray(table)).to(dev), delta,
                                    uniforms.to(dev))
        torch.cuda.synchronize()
        np.testing.assert_array_equal(acc2.cpu().numpy(), g["accept"], err_msg=label)
        np.testing.assert_array_equal(res2.cpu().numpy(), g["resample"], err_msg=label)

    bad = np.nonzero((g["accept"] != acc_o) | (g["resample"] != res_o))[0]
    if bad.size:
        i = int(bad[0])
        raise AssertionError(
            f"{label}: {bad.size} rows differ; first row {i}: gpu accept/resample="
            f"{g['accept'][i]}/{g['resample'][i]} oracle={acc_o[i]}/{res_o[i]} "
            f"margins accept={diag['margin_accept'][i]:.3e} cut={diag['margin_cut'][i]:.3e} "
            f"cdf={diag['margin_cdf'][i]:.3e} path={g['path'][i]}")
    ok = acc_o >= 0
    np.testing.assert_array_equal(g["a_size"][ok], diag["a_size"][ok].astype(np.int32), err_msg=label)
    tol = PROB_TOL[target.dtype]
    for name, ref in (("accept_prob", diag["accept_prob"]), ("mass", diag["mass"]), ("g_tok", diag["g_tok"])):
        np.testing.assert_allclose(g[name][ok], ref[ok], rtol=tol, atol=1e-30, err_msg=f"{label} {name}")
    assert np.all(np.isnan(g["accept_prob"][~ok]))
    return acc_o, res_o, diag, g


def delta_window_row():
    """A two-token row whose only neighbour carries t = 0.40000000285: at or above the double 0.4
    and below the binary32 number nearest to 0.4 (0.4000000059604645), the value the C ABI's
    `float delta` carries.  Returns (target logits [1,2] fp32, draft logits, tokens, table, uniforms);
    with delta = 0.4 the neighbour is taken (|A| = 2) exactly when the bound is read as binary32."""
    target = torch.tensor([[0.0, -0.40546509623527527]], dtype=torch.float32)
    p1 = float(np.exp(np.float64(target[0, 1].item())) / (1.0 + np.exp(np.float64(target[0, 1].item()))))
    assert 0.4 < p1 < float(np.float32(0.4))
    draft = torch.tensor([[0.0, 0.0]], dtype=torch.float32)
    tokens = torch.tensor([0], dtype=torch.int32)
    table = np.array([[0, 1], [1, 0]], dtype=np.int32)
    uniforms = torch.tensor([[0.75, 0.5]], dtype=torch.float32)
    return target, draft, tokens, table, uniforms
