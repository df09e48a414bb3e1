#!/usr/bin/env python3
"""Throughput of LANTERN's relaxed verification on one MI355X.

A step is one lantern_verify call over one batch of synthetic rows of the
stress workload (V=16384 codebook, k=1000 neighbours, delta=0.4, 3840 draft
candidates per step, bf16 logits, neighbour table resident in HBM).  Inputs
are generated on the device before the timed region; several distinct step
buffers are rotated so that reads come from HBM rather than from the 256 MB
last-level cache.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--variant plain|reject|peaked]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "relaxed verifications/sec at V=16384,k=1000 (bf16 logits); % HBM peak"
HBM_PEAK_GBS = 8000.0
# HBM bytes per launch of verify_fast on the stress/plain workload, from the rocprofv3 FETCH_SIZE and
# WRITE_SIZE runs summarised under profiles/ (one file per mode; FETCH_SIZE scaled by the factor a
# plain 256 MiB copy gives in the same run).  Other workloads have no counter run: traffic is null.
MEASURED_TRAFFIC_BYTES = {("stress", "plain", "sample"): 131140.3 * 1.99972 * 1024 + 240.1 * 1024,
                          ("stress", "plain", "greedy"): 69196.9 * 1.99973 * 1024 + 240.0 * 1024,
                          ("stress", "plain", "tree"): 75298.4 * 1.99973 * 1024 + 240.0 * 1024}


def algorithmic_bytes_per_verification(V: int, k: int, logit_bytes: int) -> int:
    """Both logit rows once, one table row, token, two uniforms, two outputs."""
    return 2 * V * logit_bytes + 4 * k + 20


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=576)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="stress", choices=["stress", "image_batch", "wide_latent", "llamagen_step", "tiny"],
                    help="stress is the headline; llamagen_step (one tree's 60 candidates per call) and tiny are "
                         "in the launch-latency regime: read ms_per_step")
    ap.add_argument("--variant", default="plain", choices=["plain", "reject", "peaked"])
    ap.add_argument("--mode", default="sample", choices=["sample", "greedy", "tree", "decide"],
                    help="sample: lantern_verify (the headline); greedy: lantern_verify_greedy, target rows only; "
                         "decide: lantern_decide_rows, the decisions without resampled tokens (rejections settle in "
                         "the fp32 pass too); tree: rows_per_step/60 random draft trees of 60 candidates, siblings sharing logit rows "
                         "(lantern_verify_trees: decisions, walk, one residual draw per tree)")
    ap.add_argument("--divergence", default="tvd", choices=["tvd", "jsd"],
                    help="bound on the neighbourhood: total variation (the headline) or Jensen-Shannon")
    ap.add_argument("--tree-order", default="level", choices=["level", "random"],
                    help="tree mode: candidates listed level by level with siblings next to each other (as a "
                         "drafter that expands one level at a time lists them), or in random drafting order")
    ap.add_argument("--buffers", type=int, default=6, help="distinct step inputs rotated through")
    ap.add_argument("--rows", type=int, default=None,
                    help="verifications per step, when not the workload's own (a sweep aid: the headline uses the default)")
    ap.add_argument("--cpu-seconds", type=float, default=10.0,
                    help="the CPU oracle is timed on whole steps of the workload until this much time has passed")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy, so that a counter run has a kernel of "
                         "known traffic to scale FETCH_SIZE / WRITE_SIZE by")
    ap.add_argument("--traffic-bytes", type=float, default=None,
                    help="HBM bytes per launch from rocprofv3 counters, if known")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (verifications are independent, so more GPUs "
              "would each take a share of the rows with the table replicated); run with --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    import paper_2410_03355_amd as lantern
    from synth import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the library has no CPU fallback", file=sys.stderr)
        return 2
    lantern.load()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = workloads.CONFIGS[args.workload]
    if args.rows is not None:
        cfg = workloads.with_overrides(cfg, rows=args.rows)
    delta = 0.0 if args.variant == "reject" else cfg.delta
    stream = torch.cuda.current_stream()

    # ---- neighbour table: built once on the device, stays resident ----
    codebook = workloads.make_codebook(cfg, device=dev)
    lantern.build_knn(codebook, cfg.k)  # warm-up (module load)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    knn = lantern.build_knn(codebook, cfg.k)
    e1.record()
    torch.cuda.synchronize()
    knn_build_ms = e0.elapsed_time(e1)

    # ---- step inputs, resident in HBM before the timed region ----
    nbuf = max(1, args.buffers)
    bufs = [workloads.make_step(cfg, step=s, device=dev, variant=args.variant) for s in range(nbuf)]
    out_acc = [torch.empty(cfg.rows, dtype=torch.int32, device=dev) for _ in range(nbuf)]
    out_res = [torch.empty(cfg.rows, dtype=torch.int32, device=dev) for _ in range(nbuf)]
    torch.cuda.synchronize()

    greedy = args.mode == "greedy"
    tree = args.mode == "tree"
    lib = lantern.load()
    dcode = lantern.BF16 if cfg.logit_dtype == "bf16" else lantern.F32

    if tree:
        import numpy as np
        from synth import trees
        M = 60
        B = cfg.rows // M
        rows_per_step = B * M
        parent_host = trees.random_trees(np.random.default_rng(workloads.BASE_SEED), B, M)
        if args.tree_order == "level":
            parent_host = trees.level_order(parent_host)
        parent = torch.from_numpy(parent_host).to(dev).reshape(-1)
        tbufs = []
        for s_ in range(nbuf):
            st_, ri, tok, un = trees.tree_step(cfg, parent_host, step=s_, variant=args.variant, device=dev)
            tbufs.append((st_, torch.from_numpy(ri).to(dev), torch.from_numpy(tok).to(dev), un))
        distinct_rows = len(set(tbufs[0][1].cpu().tolist()))
        t_len = torch.empty(B, dtype=torch.int32, device=dev)
        t_path = torch.empty(B * M, dtype=torch.int32, device=dev)
        t_next = torch.empty(B, dtype=torch.int32, device=dev)
        del bufs
        torch.cuda.synchronize()

    def step(i: int):
        if tree:
            st_, ri, tok, un = tbufs[i % nbuf]
            acc, res = out_acc[i % nbuf], out_res[i % nbuf]
            rc = lib.lantern_verify_trees(st_.target_logits.data_ptr(), st_.draft_logits.data_ptr(), dcode,
                                          B * (M + 1), cfg.V, cfg.V, ri.data_ptr(), parent.data_ptr(), B, M,
                                          tok.data_ptr(), knn.data_ptr(), cfg.k, 0, float(delta), un.data_ptr(),
                                          acc.data_ptr(), t_len.data_ptr(), t_path.data_ptr(), t_next.data_ptr(),
                                          stream.cuda_stream)
            assert rc == 0, rc
            return
        b = bufs[i % nbuf]
        if greedy:
            rc = lib.lantern_verify_greedy(b.target_logits.data_ptr(), dcode, cfg.rows, cfg.V, cfg.V,
                                           b.draft_tokens.data_ptr(), knn.data_ptr(), cfg.k, float(delta),
                                           out_acc[i % nbuf].data_ptr(), out_res[i % nbuf].data_ptr(), None,
                                           stream.cuda_stream)
            assert rc == 0, rc
        elif args.mode == "decide":
            rc = lib.lantern_decide_rows(b.target_logits.data_ptr(), b.draft_logits.data_ptr(), dcode, cfg.rows,
                                         cfg.V, cfg.V, None, cfg.rows, b.draft_tokens.data_ptr(), knn.data_ptr(),
                                         cfg.k, 1 if args.divergence == "jsd" else 0, float(delta),
                                         b.uniforms.data_ptr(), out_acc[i % nbuf].data_ptr(), None, stream.cuda_stream)
            assert rc == 0, rc
        elif args.divergence == "jsd":
            rc = lib.lantern_verify_divergence(b.target_logits.data_ptr(), b.draft_logits.data_ptr(), dcode,
                                               cfg.rows, cfg.V, cfg.V, b.draft_tokens.data_ptr(), knn.data_ptr(),
                                               cfg.k, 1, float(delta), b.uniforms.data_ptr(),
                                               out_acc[i % nbuf].data_ptr(), out_res[i % nbuf].data_ptr(),
                                               None, None, None, None, None, stream.cuda_stream)
            assert rc == 0, rc
        else:
            lantern.verify(b.target_logits, b.draft_logits, b.draft_tokens, knn, delta, b.uniforms,
                           out_accept=out_acc[i % nbuf], out_resample=out_res[i % nbuf], stream=stream)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        dst.copy_(src)  # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    # one pair of HIP events on the launch stream brackets the K launches of the timed region
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record(stream)
    for i in range(args.steps):
        step(i)
    ev1.record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    wall = t1 - t0
    # average launch duration: includes the gap between consecutive launches on the stream
    kernel_ms_avg = ev0.elapsed_time(ev1) / args.steps

    # the device's read rate for a plain stream of the same shape (same buffers, same rotation)
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    probe_src = [(b.target_logits, None if greedy else b.draft_logits) for b in bufs] if not tree else \
        [(t_[0].target_logits, t_[0].draft_logits) for t_ in tbufs]
    probe_bytes = probe_src[0][0].numel() * probe_src[0][0].element_size() // 65536 * 65536
    probe_total = probe_bytes * (1 if greedy else 2)
    for i in range(4):
        pa, pb = probe_src[i % nbuf]
        lib.lantern_probe_stream_read(pa.data_ptr(), None if pb is None else pb.data_ptr(), probe_bytes,
                                      sink.data_ptr(), stream.cuda_stream)
    pv0, pv1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    pv0.record(stream)
    n_probe = 100
    for i in range(n_probe):
        pa, pb = probe_src[i % nbuf]
        lib.lantern_probe_stream_read(pa.data_ptr(), None if pb is None else pb.data_ptr(), probe_bytes,
                                      sink.data_ptr(), stream.cuda_stream)
    pv1.record(stream)
    torch.cuda.synchronize()
    stream_read_gbs = probe_total * n_probe / (pv0.elapsed_time(pv1) * 1e-3) / 1e9

    rows = rows_per_step if tree else cfg.rows
    logit_bytes = 2 if cfg.logit_dtype == "bf16" else 4
    bytes_per_launch = algorithmic_bytes_per_verification(cfg.V, cfg.k, logit_bytes) * rows
    if tree:  # every distinct pair of logit rows once; per verification the table row and the small items
        bytes_per_launch = 2 * cfg.V * logit_bytes * distinct_rows + (4 * cfg.k + 24) * rows
    if greedy:  # one logit row, the table row, token, two outputs
        bytes_per_launch = (cfg.V * logit_bytes + 4 * cfg.k + 12) * rows
    achieved_gbs = bytes_per_launch / (kernel_ms_avg * 1e-3) / 1e9
    value = rows * args.steps / wall

    acc_all = torch.stack(out_acc[: min(nbuf, args.steps)])[:, :rows]
    accept_frac = float((acc_all == 1).float().mean().item())

    result = {
        "metric": METRIC,
        "value": value,
        "unit": "verifications/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": f"{cfg.name}/{args.variant}/{args.mode}/{args.divergence}: V={cfg.V} d={cfg.d} k={cfg.k} delta={delta} "
                        f"rows_per_step={rows} logits={cfg.logit_dtype}",
            "rows_per_step": rows,
            "distinct_step_buffers": nbuf,
            "accepted_fraction": accept_frac,
            **({"trees": B, "candidates_per_tree": M, "tree_order": args.tree_order, "distinct_logit_rows": distinct_rows,
                "mean_accepted_length": float(t_len.float().mean().item())} if tree else {}),
        },
        "roofline": {
            "bound": "hbm",
            "kernel": "greedy_fast" if greedy else "verify_fast",
            **({"note": "per step: verify_fast over shared rows, the tree walk, one fp64 residual draw per tree"}
               if tree else {}),
            "achieved": achieved_gbs,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved_gbs / HBM_PEAK_GBS,
            "traffic": args.traffic_bytes if args.traffic_bytes is not None
            else (None if args.divergence != "tvd"
                  else MEASURED_TRAFFIC_BYTES.get((args.workload, args.variant, args.mode))),
            "algorithmic_bytes_per_launch": bytes_per_launch,
            "kernel_ms_avg": kernel_ms_avg,
            "stream_read_gbs": stream_read_gbs,
            "stream_read_note": f"plain read of {probe_total >> 20} MiB per launch from the same rotating buffers, one "
                                "workgroup per 64 KiB: what a kernel with this access pattern reaches on this device",
        },
        "knn_build_ms": knn_build_ms,
    }

    if not args.no_cpu_baseline and args.mode == "sample" and args.divergence == "tvd":
        import numpy as np
        import oracle  # CPU baseline leg only
        threads = min(os.cpu_count() or 1, 16, oracle.max_threads())
        knn_host = knn.cpu().numpy()
        host = [(b.target_logits.float().cpu().numpy(), b.draft_logits.float().cpu().numpy(),
                 b.draft_tokens.cpu().numpy(), b.uniforms.cpu().numpy()) for b in bufs]
        # untimed: the GPU's outputs of the timed region against the oracle, buffer by buffer
        mism = 0
        for i, (tl, dl, tok, un) in enumerate(host[: min(nbuf, args.steps, 2)]):
            acc, res, _ = oracle.verify(tl, dl, tok, knn_host, cfg.k, delta, un, threads=threads,
                                        want_diag=False)
            mism += int((acc != out_acc[i].cpu().numpy()).sum() + (res != out_res[i].cpu().numpy()).sum())
        # timed: the oracle alone, whole steps of the same workload until the time is up
        n_cpu = 0
        c0 = time.perf_counter()
        while True:
            tl, dl, tok, un = host[n_cpu % nbuf]
            oracle.verify(tl, dl, tok, knn_host, cfg.k, delta, un, threads=threads, want_diag=False)
            n_cpu += 1
            c1 = time.perf_counter()
            if c1 - c0 >= args.cpu_seconds:
                break
        # one thread, one step; and the table build of a sample of query rows on all threads
        s0 = time.perf_counter()
        tl, dl, tok, un = host[0]
        n_single = min(rows, 512)
        oracle.verify(tl[:n_single], dl[:n_single], tok[:n_single], knn_host, cfg.k, delta, un[:n_single], threads=1,
                      want_diag=False)
        s1 = time.perf_counter()
        cb_host = codebook.float().cpu().numpy()
        n_knn = min(cfg.V, 256)
        k0 = time.perf_counter()
        oracle.build_knn(cb_host, cfg.k, rows=(0, n_knn), threads=threads)
        k1 = time.perf_counter()
        result["cpu_baseline"] = {
            "single_thread_value": n_single / (s1 - s0),
            "knn_build_ms_extrapolated": (k1 - k0) / n_knn * cfg.V * 1e3,
            "knn_sample": f"{n_knn} of {cfg.V} query rows on {threads} threads, scaled to the whole table",
            "value": n_cpu * rows / (c1 - c0),
            "unit": "verifications/s",
            "cores": threads,
            "kind": "oracle",
            "sample": f"{n_cpu} step(s) of {rows} rows of the same workload ({c1 - c0:.1f} s), rows split over "
                      f"{threads} threads",
            "mismatches_vs_gpu": mism,
        }

    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
