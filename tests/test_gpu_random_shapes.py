"""GPU parity on seeded random shapes: vocabulary sizes on and off the vector width, table widths around the
walk's block sizes, both logit types, bounds from zero to beyond one, masked tokens, unusable rows and
out-of-range tokens and table entries (Algorithm 1 and Algorithm 2, inference part; Section 4.3; Section 5.3.2),
and random draft trees under both sibling rules."""
import numpy as np
import pytest
import torch

from synth import philox, trees, workloads
from parity_utils import compare_verify

pytestmark = pytest.mark.gpu


def _table(V, k, rng):
    """Row x: x first, then k-1 distinct other tokens (a stretch of one permutation, x left out)."""
    P = rng.permutation(V).astype(np.int64)
    start = rng.integers(0, V, size=V)
    T = P[(start[:, None] + np.arange(k)[None, :]) % V]
    x = np.arange(V)
    hit = T == x[:, None]
    if k == V:                                   # every token listed: x changes places with slot 0
        pos = hit.argmax(axis=1)
        T[x, pos] = T[:, 0]
        T[:, 0] = x
    else:                                        # x, if present, gives way to the next token of the stretch
        T = np.where(hit, P[(start + k) % V][:, None], T)
        T = np.concatenate([x[:, None], T[:, : k - 1]], axis=1)
    return np.ascontiguousarray(T.astype(np.int32))


def _case(rng):
    V = int(rng.choice([int(rng.integers(2, 300)), int(rng.integers(300, 9000)), 8 * int(rng.integers(40, 4100)),
                        int(rng.choice([1024, 16384, 32768, 32776, 40000]))]))
    k = int(min(V, rng.choice([1, 2, 3, 17, 64, 255, 256, 257, 1000, 1024, 1025, 2000, 3000, int(rng.integers(1, 9000))])))
    return V, k


@pytest.mark.parametrize("seed", range(6))
def test_verification_on_random_shapes(oracle_mod, lantern_gpu, seed):
    rng = np.random.default_rng(4100 + seed)
    for case in range(8):
        V, k = _case(rng)
        rows = int(rng.choice([1, 7, 64, 200, 513]))
        dtype = torch.bfloat16 if rng.random() < 0.5 else torch.float32
        # delta = 1 with every token listed is left out: with t(xt) = 0 the prefix sum equals the bound exactly
        delta = float(rng.choice([0.0, 1e-4, 0.01, 0.1, 0.4, 0.9, 1.5]))
        scale = float(rng.choice([0.05, 1.0, 3.0, 8.0]))
        offset = float(rng.choice([0.0, -50.0, 200.0]))
        div = "jsd" if rng.random() < 0.3 else "tvd"
        g = torch.Generator().manual_seed(int(rng.integers(1 << 30)))
        tl = torch.randn(rows, V, generator=g) * scale + offset
        dl = tl + torch.randn(rows, V, generator=g) * float(rng.choice([0.1, 0.5, 1.0, 3.0])) * scale
        if rng.random() < 0.3:                   # tokens removed upstream
            m = torch.rand(rows, V, generator=g) < 0.3
            tl[m] = -float("inf")
            if rng.random() < 0.5:
                dl[m] = -float("inf")
        if rows > 2 and rng.random() < 0.2:      # unusable rows
            tl[1, int(rng.integers(V))] = float("nan")
            dl[2, int(rng.integers(V))] = float("inf")
        tl, dl = tl.to(dtype), dl.to(dtype)
        tok = torch.randint(0, V, (rows,), generator=g, dtype=torch.int32)
        if rng.random() < 0.2:
            tok[0] = V                           # out of range
        table = _table(V, k, rng)
        if k > 2 and rng.random() < 0.2:
            table[int(tok[-1]) % V, k - 1] = V + 5   # a table entry out of range, possibly beyond the cut
        un = torch.from_numpy(philox.uniforms(int(rng.integers(1 << 30)), rows, stream=3))
        if rng.random() < 0.3:
            un[:, 0] = 1 - 2.0 ** -24
        label = f"seed {seed} case {case}: V={V} k={k} rows={rows} {dtype} delta={delta} scale={scale} offset={offset} {div}"
        acc_o, res_o, diag, out = compare_verify(oracle_mod, lantern_gpu, tl, dl, tok, table, delta, un, threads=16,
                                                 label=label, divergence=div)
        tb = torch.from_numpy(table).cuda()
        dec = lantern_gpu.decide_rows(tl.cuda(), dl.cuda(), None, tok.cuda(), tb, delta, un.cuda(), divergence=div)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(dec.cpu().numpy(), acc_o, err_msg=label + " decide_rows")
        if div == "tvd":
            gacc, gtok = lantern_gpu.verify_greedy(tl.cuda(), tok.cuda(), tb, delta)
            torch.cuda.synchronize()
            ga_o, gt_o, _ = oracle_mod.verify_greedy(tl.float().numpy(), tok.numpy(), table, k, delta, threads=16)
            np.testing.assert_array_equal(gacc.cpu().numpy(), ga_o, err_msg=label + " greedy accept")
            np.testing.assert_array_equal(gtok.cpu().numpy(), gt_o, err_msg=label + " greedy token")


@pytest.mark.parametrize("seed", range(4))
def test_tree_steps_on_random_shapes(oracle_mod, lantern_gpu, seed):
    rng = np.random.default_rng(5200 + seed)
    base = workloads.CONFIGS["tiny"]
    for case in range(8):
        V = int(rng.choice([int(rng.integers(8, 400)), 8 * int(rng.integers(8, 1200)), int(rng.integers(400, 9000)), 16384, 20000]))
        k = int(min(V, rng.choice([1, 2, 5, 64, 100, 300, 1000, 1025, int(rng.integers(1, 2500))])))
        M = int(rng.choice([1, 2, 6, 17, 60]))
        B = int(rng.choice([1, 3, 16, 40]))
        cfg = workloads.with_overrides(base, V=V, k=k, logit_dtype=str(rng.choice(["f32", "bf16"])),
                                       logit_scale=float(rng.choice([0.3, 1.0, 2.0, 6.0])),
                                       draft_noise=float(rng.choice([0.2, 0.5, 1.5])))
        table = _table(V, k, rng)
        tb = torch.from_numpy(table).cuda()
        parent = trees.random_trees(rng, B, M, max_children=int(rng.integers(1, 7)))
        if rng.random() < 0.5:
            parent = trees.level_order(parent)
        delta = float(rng.choice([0.0, 0.01, 0.1, 0.4, 0.9]))
        div = "jsd" if rng.random() < 0.3 else "tvd"
        variant = str(rng.choice(["plain", "reject", "peaked"]))
        label = f"seed {seed} case {case}: V={V} k={k} B={B} M={M} {cfg.logit_dtype} delta={delta} {div} {variant}"
        st, ri, tok, un = trees.tree_step(cfg, parent, step=int(rng.integers(1 << 20)), variant=variant)
        pt = torch.from_numpy(parent).cuda().reshape(-1)
        dev = (st.target_logits.cuda(), st.draft_logits.cuda(), torch.from_numpy(ri).cuda(), pt, M,
               torch.from_numpy(tok).cuda(), tb, delta, un.cuda())
        acc_o, res_o, _ = oracle_mod.verify_rows(st.target_logits, st.draft_logits, ri, tok, table, k, delta, un,
                                                 threads=16, divergence=div)
        n_o, path_o, next_o = oracle_mod.accept_trees(acc_o, res_o, parent, M)
        acc, n, path, nxt = lantern_gpu.verify_trees(*dev, divergence=div)
        torch.cuda.synchronize()
        for got, want, what in ((acc, acc_o, "accept"), (n, n_o, "length"), (path, path_o, "path"), (nxt, next_o, "next")):
            np.testing.assert_array_equal(got.cpu().numpy(), want, err_msg=f"{label}: default rule, {what}")
        sn_o, spath_o, snext_o = oracle_mod.verify_trees_sequential(st.target_logits, st.draft_logits, ri, parent, M, tok,
                                                                    table, k, delta, un, threads=16, divergence=div)
        sn, spath, snxt = lantern_gpu.verify_trees_sequential(*dev, divergence=div)
        torch.cuda.synchronize()
        for got, want, what in ((sn, sn_o, "length"), (spath, spath_o, "path"), (snxt, snext_o, "next")):
            np.testing.assert_array_equal(got.cpu().numpy(), want, err_msg=f"{label}: sequential rule, {what}")


@pytest.mark.parametrize("seed", range(4))
def test_tables_on_random_shapes(oracle_mod, lantern_gpu, seed):
    """Neighbour tables (Algorithm 2, precompute part; Section 5.3.1 for the cosine key) of random shape and
    structure: Gaussian, clustered, sorted along an axis, heavy-tailed norms; half of them with codes of zero norm
    (cosine) or with an infinite or NaN coordinate (squared l2), which rank last on both sides."""
    rng = np.random.default_rng(6300 + seed)
    for case in range(7):
        if case < 6:
            V = int(rng.integers(1, 4200))
            d = int(rng.choice([1, 3, 4, 5, 8, 12, 16, 32, 100, 256]))
            k = int(rng.integers(1, min(V, 1500) + 1))
        else:                                    # sampled thresholds and candidate lists
            V = int(rng.integers(4096, 14000))
            d = int(rng.choice([4, 8, 16, 64]))
            k = int(rng.integers(40, 1010))
        dtype = torch.bfloat16 if rng.random() < 0.4 else torch.float32
        metric = "cosine" if rng.random() < 0.3 else "l2"
        kind = int(rng.integers(0, 4))
        g = torch.Generator().manual_seed(int(rng.integers(1 << 30)))
        cb = torch.randn(V, d, generator=g)
        if kind == 1:
            centres = torch.randn(32, d, generator=g) * 3
            cb = centres[(torch.arange(V) * 32 // V).clamp(max=31)] + 0.3 * cb
        elif kind == 2:
            cb = cb[torch.argsort(cb[:, 0])].contiguous()
        elif kind == 3:
            cb = cb * torch.exp(torch.randn(V, 1, generator=g))
        what = ""
        if rng.random() < 0.5:
            rows = rng.integers(0, V, size=int(rng.integers(1, 6)))
            if metric == "cosine":
                cb[rows] = 0.0
                what = f" zero rows {rows.tolist()}"
            else:
                val = float(rng.choice([np.inf, -np.inf, np.nan]))
                cb[rows, int(rng.integers(d))] = val
                what = f" {val} in rows {rows.tolist()}"
        cb = cb.to(dtype).contiguous()
        got = lantern_gpu.build_knn(cb.cuda(), k, metric=metric)
        torch.cuda.synchronize()
        want = oracle_mod.build_knn(cb.float().numpy(), k, metric=metric, threads=16)
        np.testing.assert_array_equal(got.cpu().numpy(), want,
                                      err_msg=f"seed {seed} case {case}: V={V} d={d} k={k} {dtype} {metric} kind={kind}{what}")
