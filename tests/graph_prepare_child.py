"""Run in a fresh process by tests/test_gpu_graph.py: after lantern_prepare, the very first call of a
shape on the device may sit inside a stream capture.  Captures a verification whose kernel needs more
than 64 KiB of LDS (V=32768, bf16) and a fused tree step (V=16384, bf16: the walk-and-draw kernel
stages both rows in LDS), replays the graph on fresh inputs and compares every replay with the
oracle.  Prints "ok" on success."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

import numpy as np
import torch

import oracle
import paper_2410_03355_amd as lantern
from parity_utils import random_table, random_trees, tree_step
from synth import philox, workloads


def main():
    lantern.load()
    oracle.build()
    V, k, N = 32768, 64, 12
    rng = np.random.default_rng(5)
    table = random_table(V, k, seed=3)
    tb = torch.from_numpy(table).cuda()
    tl = torch.empty((N, V), dtype=torch.bfloat16, device="cuda")
    dl = torch.empty_like(tl)
    tok = torch.empty(N, dtype=torch.int32, device="cuda")
    un = torch.empty((N, 2), dtype=torch.float32, device="cuda")
    acc = torch.empty(N, dtype=torch.int32, device="cuda")
    res = torch.empty(N, dtype=torch.int32, device="cuda")

    cfg = workloads.CONFIGS["llamagen_step"]
    B, M = 2, 60
    parent = random_trees(np.random.default_rng(8), B, M, max_children=4)
    table2 = random_table(cfg.V, cfg.k, seed=6)
    tb2 = torch.from_numpy(table2).cuda()
    par_d = torch.from_numpy(parent).cuda().reshape(-1)
    R = B * (M + 1)
    tl2 = torch.empty((R, cfg.V), dtype=torch.bfloat16, device="cuda")
    dl2 = torch.empty_like(tl2)
    ri = torch.empty(B * M, dtype=torch.int32, device="cuda")
    tok2 = torch.empty(B * M, dtype=torch.int32, device="cuda")
    un2 = torch.empty((B * M, 2), dtype=torch.float32, device="cuda")

    def inputs(seed):
        r = np.random.default_rng(seed)
        t = torch.from_numpy((r.standard_normal((N, V)) * 2.0).astype(np.float32))
        g = (t + torch.from_numpy(r.standard_normal((N, V)).astype(np.float32))).to(torch.bfloat16)
        t = t.to(torch.bfloat16)
        tokens = torch.from_numpy(r.integers(0, V, N).astype(np.int32))
        u = torch.from_numpy(philox.uniforms(seed, N))
        return t, g, tokens, u

    lantern.prepare(torch.bfloat16, V, k)
    lantern.prepare(torch.bfloat16, cfg.V, cfg.k)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):          # no call of either shape has happened in this process
        s = torch.cuda.current_stream()
        lantern.verify(tl, dl, tok, tb, 0.05, un, out_accept=acc, out_resample=res, stream=s)
        acc2, n2, path2, nxt2 = lantern.verify_trees(tl2, dl2, ri, par_d, M, tok2, tb2, 0.05, un2, stream=s)
    for seed, variant in ((1, "reject"), (2, "plain"), (3, "peaked")):
        t, g, tokens, u = inputs(seed)
        tl.copy_(t); dl.copy_(g); tok.copy_(tokens); un.copy_(u)
        st, row_index, tokens2, uniforms2 = tree_step(cfg, parent, step=seed, variant=variant)
        tl2.copy_(st.target_logits); dl2.copy_(st.draft_logits)
        ri.copy_(torch.from_numpy(row_index)); tok2.copy_(torch.from_numpy(tokens2)); un2.copy_(uniforms2)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        acc_o, res_o, _ = oracle.verify(t, g, tokens, table, k, 0.05, u, threads=8)
        np.testing.assert_array_equal(acc.cpu().numpy(), acc_o)
        np.testing.assert_array_equal(res.cpu().numpy(), res_o)
        a_o, r_o, _ = oracle.verify_rows(st.target_logits, st.draft_logits, row_index, tokens2, table2, cfg.k,
                                         0.05, uniforms2, threads=8)
        n_o, path_o, next_o = oracle.accept_trees(a_o, r_o, parent, M)
        np.testing.assert_array_equal(acc2.cpu().numpy(), a_o)
        np.testing.assert_array_equal(n2.cpu().numpy(), n_o)
        np.testing.assert_array_equal(path2.cpu().numpy(), path_o)
        np.testing.assert_array_equal(nxt2.cpu().numpy(), next_o)
    print("ok", flush=True)


if __name__ == "__main__":
    main()
