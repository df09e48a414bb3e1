"""The library only enqueues kernels on the caller's stream, so its calls can be captured into a HIP
graph and replayed; every replay must equal the eager result on the buffers' current contents."""
import numpy as np
import pytest
import torch

from synth import workloads
from parity_utils import random_table

pytestmark = pytest.mark.gpu


def test_capture_and_replay(oracle_mod, lantern_gpu):
    cfg = workloads.CONFIGS["tiny"]
    L, B = 4, 64
    rows = L * B
    table = random_table(cfg.V, cfg.k, seed=33)
    tb = torch.from_numpy(table).cuda()
    steps = [workloads.make_step(cfg, step=s, rows=rows) for s in (40, 41, 42)]
    # static buffers the captured calls read and write
    tl = torch.empty_like(steps[0].target_logits, device="cuda")
    dl = torch.empty_like(steps[0].draft_logits, device="cuda")
    tok = torch.empty(rows, dtype=torch.int32, device="cuda")
    un = torch.empty((rows, 2), dtype=torch.float32, device="cuda")
    acc = torch.empty(rows, dtype=torch.int32, device="cuda")
    res = torch.empty(rows, dtype=torch.int32, device="cuda")

    def load(st):
        tl.copy_(st.target_logits); dl.copy_(st.draft_logits); tok.copy_(st.draft_tokens); un.copy_(st.uniforms)

    load(steps[0])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm up outside the capture
        lantern_gpu.verify(tl, dl, tok, tb, cfg.delta, un, out_accept=acc, out_resample=res, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        s = torch.cuda.current_stream()
        lantern_gpu.verify(tl, dl, tok, tb, cfg.delta, un, out_accept=acc, out_resample=res, stream=s)
        kept, nxt = lantern_gpu.accept_chains(acc, res, L, stream=s)
        gacc, gtok = lantern_gpu.verify_greedy(tl, tok, tb, cfg.delta, stream=s)

    for st in (steps[1], steps[2], steps[0], steps[2]):
        load(st)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        acc_o, res_o, _ = oracle_mod.verify(st.target_logits, st.draft_logits, st.draft_tokens, table, cfg.k,
                                            cfg.delta, st.uniforms, threads=8)
        np.testing.assert_array_equal(acc.cpu().numpy(), acc_o)
        np.testing.assert_array_equal(res.cpu().numpy(), res_o)
        n_o, next_o = oracle_mod.accept_chains(acc_o, res_o, L)
        np.testing.assert_array_equal(kept.cpu().numpy(), n_o)
        np.testing.assert_array_equal(nxt.cpu().numpy(), next_o)
        ga_o, gt_o, _ = oracle_mod.verify_greedy(st.target_logits, st.draft_tokens, table, cfg.k, cfg.delta,
                                                 threads=8)
        np.testing.assert_array_equal(gacc.cpu().numpy(), ga_o)
        np.testing.assert_array_equal(gtok.cpu().numpy(), gt_o)


def test_capture_tree_step(oracle_mod, lantern_gpu):
    """The fused tree step (three launches, the last with more than 64 KiB of LDS) in a graph."""
    from parity_utils import random_trees, tree_step
    cfg = workloads.CONFIGS["llamagen_step"]
    B, M = 3, 60
    rng = np.random.default_rng(77)
    parent = random_trees(rng, B, M, max_children=4)
    table = random_table(cfg.V, cfg.k, seed=5)
    tb = torch.from_numpy(table).cuda()
    par_d = torch.from_numpy(parent).cuda().reshape(-1)
    steps = [tree_step(cfg, parent, step=s, variant=v) for s, v in ((1, "reject"), (2, "plain"), (3, "peaked"))]
    R = B * (M + 1)
    tl = torch.empty((R, cfg.V), dtype=torch.bfloat16, device="cuda")
    dl = torch.empty_like(tl)
    ri = torch.empty(B * M, dtype=torch.int32, device="cuda")
    tok = torch.empty(B * M, dtype=torch.int32, device="cuda")
    un = torch.empty((B * M, 2), dtype=torch.float32, device="cuda")

    def load(step):
        st, row_index, tokens, uniforms = step
        tl.copy_(st.target_logits); dl.copy_(st.draft_logits)
        ri.copy_(torch.from_numpy(row_index)); tok.copy_(torch.from_numpy(tokens)); un.copy_(uniforms)

    delta = 0.05
    load(steps[0])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm up outside the capture
        lantern_gpu.verify_trees(tl, dl, ri, par_d, M, tok, tb, delta, un, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        acc, n, path, nxt = lantern_gpu.verify_trees(tl, dl, ri, par_d, M, tok, tb, delta, un,
                                                     stream=torch.cuda.current_stream())

    for step in (steps[1], steps[2], steps[0], steps[1]):
        load(step)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        st, row_index, tokens, uniforms = step
        acc_o, res_o, _ = oracle_mod.verify_rows(st.target_logits, st.draft_logits, row_index, tokens, table, cfg.k,
                                                 delta, uniforms, threads=8)
        n_o, path_o, next_o = oracle_mod.accept_trees(acc_o, res_o, parent, M)
        np.testing.assert_array_equal(acc.cpu().numpy(), acc_o)
        np.testing.assert_array_equal(n.cpu().numpy(), n_o)
        np.testing.assert_array_equal(path.cpu().numpy(), path_o)
        np.testing.assert_array_equal(nxt.cpu().numpy(), next_o)


def test_first_call_inside_a_capture_after_prepare(lantern_gpu):
    """lantern_prepare raises the LDS limits ahead of time, so the first call of a shape in a process
    may be recorded into a graph: checked in a fresh process (tests/graph_prepare_child.py)."""
    import os
    import subprocess
    import sys
    child = os.path.join(os.path.dirname(os.path.abspath(__file__)), "graph_prepare_child.py")
    r = subprocess.run([sys.executable, "-u", child], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout[-2000:] + r.stderr[-4000:]
