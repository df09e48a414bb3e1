"""GPU parity of lantern_verify / lantern_verify_ex against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from synth import philox, workloads
from parity_utils import compare_verify, random_table, sparse_table_from_oracle

pytestmark = pytest.mark.gpu


def _step_and_table(oracle, cfg, rows, variant="plain", step=0):
    st = workloads.make_step(cfg, step=step, rows=rows, variant=variant)
    cb = workloads.make_codebook(cfg)
    table = sparse_table_from_oracle(oracle, cb.float().numpy(), cfg.k, st.draft_tokens.numpy())
    return st, table


def test_tiny_config(oracle_mod, lantern_gpu):
    """V=1024, k=16, delta=0.1, fp32 logits, 64 rows: cut and rejections occur naturally."""
    cfg = workloads.CONFIGS["tiny"]
    cb = workloads.make_codebook(cfg)
    table = oracle_mod.build_knn(cb.numpy(), cfg.k, threads=8)
    st = workloads.make_step(cfg)
    acc, res, diag, g = compare_verify(oracle_mod, lantern_gpu, st.target_logits, st.draft_logits,
                                       st.draft_tokens, table, cfg.delta, st.uniforms, label="tiny")
    assert (acc == 0).sum() > 0 and (acc == 1).sum() > 0
    assert (diag["a_size"] < cfg.k).sum() > 0          # the TVD bound cuts some neighbourhoods


@pytest.mark.parametrize("delta,k_use", [(0.0, 16), (0.1, 1), (0.02, 16), (0.5, 16), (2.0, 16)])
def test_tiny_special_cases(oracle_mod, lantern_gpu, delta, k_use):
    """delta=0 and k=1 reduce to standard speculative acceptance; delta>1 never binds."""
    cfg = workloads.CONFIGS["tiny"]
    cb = workloads.make_codebook(cfg)
    table = oracle_mod.build_knn(cb.numpy(), k_use, threads=8)
    st = workloads.make_step(cfg, step=3)
    acc, res, diag, g = compare_verify(oracle_mod, lantern_gpu, st.target_logits, st.draft_logits,
                                       st.draft_tokens, table, delta, st.uniforms,
                                       label=f"tiny d={delta} k={k_use}")
    if delta == 0.0 or k_use == 1:
        assert np.all(diag["a_size"] == 1)
        t_over_g = np.minimum(1.0, diag["t_tok"] / diag["g_tok"])
        np.testing.assert_allclose(g["accept_prob"], t_over_g, rtol=1e-5)
    if delta == 2.0:
        assert np.all(diag["a_size"] == k_use)


@pytest.mark.parametrize("variant", ["plain", "peaked", "reject"])
def test_llamagen_step(oracle_mod, lantern_gpu, variant):
    """V=16384, k=1000, bf16 logits, one 60-candidate draft tree."""
    cfg = workloads.CONFIGS["llamagen_step"]
    st, table = _step_and_table(oracle_mod, cfg, cfg.rows, variant)
    # peaked rows put ~1000/16384 of the mass into a random neighbourhood: a small bound cuts it
    delta = {"plain": cfg.delta, "reject": 0.0, "peaked": 0.01}[variant]
    acc, res, diag, g = compare_verify(oracle_mod, lantern_gpu, st.target_logits, st.draft_logits,
                                       st.draft_tokens, table, delta, st.uniforms,
                                       label=f"llamagen {variant}")
    if variant == "plain":
        assert (acc == 1).mean() > 0.9 and np.all(g["path"][acc == 1] == 0)
    if variant == "reject":
        assert (acc == 0).mean() > 0.3
    if variant == "peaked":
        assert (diag["a_size"] < cfg.k).sum() > 0


def test_image_batch_rows(oracle_mod, lantern_gpu):
    """V=16384, k=300, delta=0.2, bf16: two steps of 960 rows of the 256-step job."""
    cfg = workloads.CONFIGS["image_batch"]
    for step in (0, 255):
        st, table = _step_and_table(oracle_mod, cfg, 240, step=step)
        compare_verify(oracle_mod, lantern_gpu, st.target_logits, st.draft_logits, st.draft_tokens,
                       table, cfg.delta, st.uniforms, label=f"image_batch step {step}")


def test_wide_latent_rows(oracle_mod, lantern_gpu):
    """V=8192, k=100, delta=0.3, fp32 logits (table rows from a d=256 bf16 codebook)."""
    cfg = workloads.CONFIGS["wide_latent"]
    for variant, delta in (("plain", cfg.delta), ("peaked", 0.01)):
        st, table = _step_and_table(oracle_mod, cfg, 256, variant)
        compare_verify(oracle_mod, lantern_gpu, st.target_logits, st.draft_logits, st.draft_tokens,
                       table, delta, st.uniforms, label=f"wide_latent {variant}")


def test_image_batch_full_step(oracle_mod, lantern_gpu):
    """image_batch at its own launch size: all 960 rows of a step in one call."""
    cfg = workloads.CONFIGS["image_batch"]
    st, table = _step_and_table(oracle_mod, cfg, cfg.rows, step=101)
    acc, res, diag, g = compare_verify(oracle_mod, lantern_gpu, st.target_logits, st.draft_logits, st.draft_tokens,
                                       table, cfg.delta, st.uniforms, threads=16, label="image_batch full step")
    assert len(acc) == 960


@pytest.mark.parametrize("variant,delta", [("plain", None), ("peaked", 0.01), ("reject", 0.0)])
def test_wide_latent_full_step(oracle_mod, lantern_gpu, variant, delta):
    """wide_latent at its own launch size: 3840 rows of fp32 logits (V=8192, k=100) in one call."""
    cfg = workloads.CONFIGS["wide_latent"]
    st = workloads.make_step(cfg, step=9, variant=variant)
    table = random_table(cfg.V, cfg.k, seed=31)
    acc, res, diag, g = compare_verify(oracle_mod, lantern_gpu, st.target_logits, st.draft_logits, st.draft_tokens,
                                       table, cfg.delta if delta is None else delta, st.uniforms, threads=16,
                                       label=f"wide_latent full step {variant}")
    assert len(acc) == 3840
    if variant == "reject":
        assert (acc == 0).mean() > 0.3


def test_delta_is_the_binary32_value(oracle_mod, lantern_gpu):
    """A prefix whose TVD lies between the double 0.4 and float32(0.4): inside the bound on both sides."""
    from parity_utils import delta_window_row
    target, draft, tokens, table, un = delta_window_row()
    acc, res, diag, g = compare_verify(oracle_mod, lantern_gpu, target, draft, tokens, table, 0.4, un,
                                       label="delta window")
    assert g["a_size"][0] == 2 and g["path"][0] == 1


def test_stress_full_step(oracle_mod, lantern_gpu):
    """One full 3840-row step of the stress configuration, in the bench's launch
    configuration (V=16384, k=1000, bf16, all rows in one call), every row compared."""
    cfg = workloads.CONFIGS["stress"]
    st = workloads.make_step(cfg, step=17)
    table = random_table(cfg.V, cfg.k, seed=5)  # any table with distinct rows is a valid input
    acc, res, diag, g = compare_verify(oracle_mod, lantern_gpu, st.target_logits, st.draft_logits,
                                       st.draft_tokens, table, cfg.delta, st.uniforms, threads=16,
                                       label="stress step")
    assert len(acc) == 3840


def test_stress_reject_heavy(oracle_mod, lantern_gpu):
    """Reject-heavy mix at full width: delta=0, acceptance draw just below one."""
    cfg = workloads.CONFIGS["stress"]
    st = workloads.make_step(cfg, step=2, rows=512, variant="reject")
    table = random_table(cfg.V, cfg.k, seed=6)
    acc, res, diag, g = compare_verify(oracle_mod, lantern_gpu, st.target_logits, st.draft_logits,
                                       st.draft_tokens, table, 0.0, st.uniforms, threads=16,
                                       label="stress reject")
    assert (acc == 0).mean() > 0.3
    rej = acc == 0
    assert np.all(res[rej] >= 0) and np.all(res[~rej] == -1)


@pytest.mark.parametrize("shift_t,shift_g", [(250.0, -180.0), (-600.0, 650.0)])
def test_large_logit_offsets(oracle_mod, lantern_gpu, shift_t, shift_g):
    """Rows whose logits sit far from zero (a softmax does not care): the reference of the fp32 pass
    is then a large number, whose rounding the fp64 sign test of the rejected rows has to account for."""
    V, k, N = 8192, 100, 384                                # fp32 logits: the offsets keep their resolution
    rng = np.random.default_rng(31)
    base = rng.normal(0.0, 1.5, (N, V))
    tl = torch.from_numpy((base + shift_t).astype(np.float32))
    dl = torch.from_numpy((base + rng.normal(0.0, 0.8, (N, V)) + shift_g).astype(np.float32))
    tokens = dl.argmax(dim=1).to(torch.int32)               # the drafter's favourite: g(xt) > t(xt) mostly
    un = torch.from_numpy(philox.uniforms(77, N, stream=1))
    un[:, 0] = 1.0 - 2.0 ** -24                             # acceptance draw just below one
    table = random_table(V, k, seed=9)
    for delta in (0.0, 0.05):
        acc, res, diag, g = compare_verify(oracle_mod, lantern_gpu, tl, dl, tokens, table, delta,
                                           un, threads=16, label="offset logits")
        assert (acc == 0).mean() > 0.2 and np.all(res[acc == 0] >= 0)
        assert (g["path"][acc == 0] == 1).all()


@pytest.mark.parametrize("V,k,N,dtype", [
    (1, 1, 3, torch.float32),          # degenerate vocabulary
    (7, 7, 5, torch.float32),          # ragged, k = V
    (1000, 33, 37, torch.float32),     # V not a multiple of the vector width
    (1003, 50, 20, torch.bfloat16),    # odd V, rows not 16-byte aligned
    (4096, 2500, 9, torch.bfloat16),   # k spans several scan chunks
    (2048, 2048, 4, torch.float32),    # k = V
    (32768, 64, 6, torch.bfloat16),    # largest register-resident bf16 row
    (16384, 128, 6, torch.float32),    # largest register-resident fp32 row
    (40000, 100, 5, torch.float32),    # beyond the fast pass: fp64 pass only
])
def test_shapes(oracle_mod, lantern_gpu, V, k, N, dtype):
    rng = np.random.default_rng(V * 7 + k)
    scale = 2.5
    t = torch.from_numpy((rng.standard_normal((N, V)) * scale).astype(np.float32))
    g = t + torch.from_numpy(rng.standard_normal((N, V)).astype(np.float32))
    t, g = t.to(dtype), g.to(dtype)
    tokens = torch.from_numpy(rng.integers(0, V, N).astype(np.int32))
    table = random_table(V, k, seed=V + k)
    un = torch.from_numpy(philox.uniforms(V, N))
    for delta in (0.05, 0.3):
        compare_verify(oracle_mod, lantern_gpu, t, g, tokens, table, delta, un, label=f"V={V} k={k}")


def test_strided_rows(oracle_mod, lantern_gpu):
    """Rows taken from a wider buffer: row stride larger than V."""
    rng = np.random.default_rng(3)
    N, V, k, pitch = 12, 2048, 40, 2304
    tb = torch.from_numpy((rng.standard_normal((N, pitch)) * 3).astype(np.float32)).to(torch.bfloat16)
    gb = (tb.float() + torch.from_numpy(rng.standard_normal((N, pitch)).astype(np.float32))).to(torch.bfloat16)
    tokens = torch.from_numpy(rng.integers(0, V, N).astype(np.int32))
    table = random_table(V, k, seed=9)
    un = torch.from_numpy(philox.uniforms(77, N))
    acc_o, res_o, _ = oracle_mod.verify(tb[:, :V].contiguous(), gb[:, :V].contiguous(), tokens, table, k,
                                        0.1, un)
    td, gd = tb.cuda()[:, :V], gb.cuda()[:, :V]
    assert td.stride(0) == pitch
    acc, res = lantern_gpu.verify(td, gd, tokens.cuda(), torch.from_numpy(table).cuda(), 0.1, un.cuda())
    torch.cuda.synchronize()
    np.testing.assert_array_equal(acc.cpu().numpy(), acc_o)
    np.testing.assert_array_equal(res.cpu().numpy(), res_o)


def test_filtered_and_unusable_rows(oracle_mod, lantern_gpu):
    """-inf logits (top-k / top-p filtering upstream) work; NaN, +inf, all -inf rows,
    tokens and table entries out of range give the -1 sentinels."""
    rng = np.random.default_rng(4)
    N, V, k = 16, 4096, 64
    t = (rng.standard_normal((N, V)) * 2).astype(np.float32)
    g = (t + rng.standard_normal((N, V))).astype(np.float32)
    tokens = rng.integers(0, V - 8, N).astype(np.int32)
    table = random_table(V, k, seed=10)
    keep = np.argsort(-t[0])[:50]                  # row 0: only 50 target tokens survive filtering
    mask = np.ones(V, bool); mask[keep] = False
    t[0, mask] = -np.inf
    tokens[0] = keep[3]
    g[1, : V // 2] = -np.inf                        # row 1: half of the draft row filtered
    tokens[1] = V // 2 + 5
    t[2, 100] = np.nan
    g[3, 7] = np.inf
    t[4, :] = -np.inf
    tokens[5] = V
    tokens[6] = -3
    table[tokens[7], 5] = V + 1                     # bad table entry in the row that row 7 reads
    t[8, tokens[8]] = -np.inf                       # draft token the target gives zero mass
    g[9, tokens[9]] = -np.inf                       # draft token the drafter gives zero mass
    un = torch.from_numpy(philox.uniforms(11, N))
    acc, res, diag, gg = compare_verify(oracle_mod, lantern_gpu, torch.from_numpy(t), torch.from_numpy(g),
                                        torch.from_numpy(tokens), table, 0.2, un, label="unusable")
    assert list(acc[2:8]) == [-1] * 6 and list(res[2:8]) == [-1] * 6
    assert acc[0] in (0, 1) and acc[1] in (0, 1)
    assert acc[9] == 1


def test_bad_table_entry_beyond_the_cut(oracle_mod, lantern_gpu):
    """All k entries of a table row are range-checked, also those after the cut and beyond the
    first 1024 slots: such rows are unusable on every path (sampling, decisions only, greedy)."""
    V, k, N = 8192, 4000, 12
    rng = np.random.default_rng(21)
    t = torch.from_numpy((rng.standard_normal((N, V)) * 6.0).astype(np.float32)).to(torch.bfloat16)   # peaked: early cut
    g = (t.float() + torch.from_numpy(rng.standard_normal((N, V)).astype(np.float32))).to(torch.bfloat16)
    tokens = torch.from_numpy(rng.permutation(V)[:N].astype(np.int32))
    table = random_table(V, k, seed=22)
    un = torch.from_numpy(philox.uniforms(23, N))
    _, _, clean = oracle_mod.verify(t, g, tokens, table, k, 0.02, un, threads=8)
    bad_rows = [int(i) for i in np.nonzero(clean["a_size"] < 1000)[0][:3]]   # rows whose walk ends early
    assert len(bad_rows) == 3
    for i, slot in zip(bad_rows, (1030, 2999, 3999)):
        table[int(tokens[i]), slot] = V + i
    acc, res, diag, gg = compare_verify(oracle_mod, lantern_gpu, t, g, tokens, table, 0.02, un, label="late bad entry")
    assert all(acc[i] == -1 for i in bad_rows) and (acc >= 0).sum() == N - len(bad_rows)
    tb = torch.from_numpy(table).cuda()
    dec = lantern_gpu.decide_rows(t.cuda(), g.cuda(), None, tokens.cuda(), tb, 0.02, un.cuda())
    ga, gt = lantern_gpu.verify_greedy(t.cuda(), tokens.cuda(), tb, 0.02)
    torch.cuda.synchronize()
    dec = dec[0] if isinstance(dec, tuple) else dec
    np.testing.assert_array_equal(dec.cpu().numpy(), acc)
    ga_o, gt_o, _ = oracle_mod.verify_greedy(t, tokens, table, k, 0.02, threads=8)
    np.testing.assert_array_equal(ga.cpu().numpy(), ga_o)
    np.testing.assert_array_equal(gt.cpu().numpy(), gt_o)
    assert all(ga_o[i] == -1 for i in bad_rows)


def test_empty_batch_and_determinism(oracle_mod, lantern_gpu):
    V, k = 512, 8
    table = torch.from_numpy(random_table(V, k, seed=1)).cuda()
    empty = torch.empty((0, V), device="cuda")
    acc, res = lantern_gpu.verify(empty, empty, torch.empty(0, dtype=torch.int32, device="cuda"), table, 0.1,
                                  torch.empty((0, 2), device="cuda"))
    assert acc.numel() == 0 and res.numel() == 0
    cfg = workloads.CONFIGS["tiny"]
    st = workloads.make_step(cfg, step=9, variant="peaked")
    tb = torch.from_numpy(random_table(cfg.V, cfg.k, seed=2)).cuda()
    args = (st.target_logits.cuda(), st.draft_logits.cuda(), st.draft_tokens.cuda(), tb, cfg.delta,
            st.uniforms.cuda())
    a1 = lantern_gpu.verify_ex(*args)
    a2 = lantern_gpu.verify_ex(*args)
    torch.cuda.synchronize()
    for name in a1:
        assert torch.equal(a1[name], a2[name]) or name in ("accept_prob", "mass", "g_tok") and \
            torch.equal(torch.nan_to_num(a1[name]), torch.nan_to_num(a2[name]))


def test_side_stream(oracle_mod, lantern_gpu):
    """Work is enqueued on the stream that is passed in."""
    cfg = workloads.CONFIGS["tiny"]
    st = workloads.make_step(cfg, step=1)
    table = random_table(cfg.V, cfg.k, seed=3)
    acc_o, res_o, _ = oracle_mod.verify(st.target_logits, st.draft_logits, st.draft_tokens, table, cfg.k,
                                        cfg.delta, st.uniforms)
    s = torch.cuda.Stream()
    args = [x.cuda() for x in (st.target_logits, st.draft_logits, st.draft_tokens)]
    tb, un = torch.from_numpy(table).cuda(), st.uniforms.cuda()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        acc, res = lantern_gpu.verify(args[0], args[1], args[2], tb, cfg.delta, un, stream=s)
    s.synchronize()
    np.testing.assert_array_equal(acc.cpu().numpy(), acc_o)
    np.testing.assert_array_equal(res.cpu().numpy(), res_o)


def test_maximum_vocabulary(oracle_mod, lantern_gpu):
    """V = LANTERN_MAX_VOCAB (2^19), the largest row the library takes, in both logit types; all
    entry points of the sampling path and the greedy one."""
    V = lantern_gpu.MAX_VOCAB
    N, k = 3, 40
    rng = np.random.default_rng(19)
    base = (rng.standard_normal((N, V)) * 2.0).astype(np.float32)
    tokens = rng.integers(0, V, N).astype(np.int32)
    tokens[0] = V - 1                                            # the last token of the vocabulary
    table = np.empty((V, k), dtype=np.int32)
    table[:, 0] = np.arange(V)
    table[:, 1:] = (np.arange(V)[:, None] + rng.integers(1, V, k - 1)[None, :]) % V   # distinct shifts, never 0
    un = torch.from_numpy(rng.random((N, 2)).astype(np.float32))
    un[1, 0] = 1.0 - 2.0 ** -24                                  # a rejection: the residual over 2^19 tokens
    for dtype in (torch.float32, torch.bfloat16):
        t = torch.from_numpy(base).to(dtype)
        gl = base + rng.standard_normal((N, V)).astype(np.float32)
        gl[1, tokens[1]] = 14.0                                  # the drafter is far too sure of this token
        g = torch.from_numpy(gl).to(dtype)
        acc, res, diag, gout = compare_verify(oracle_mod, lantern_gpu, t, g, torch.from_numpy(tokens), table, 0.05,
                                              un, label=f"max vocabulary {dtype}")
        assert (acc == 0).any()
        dacc = lantern_gpu.decide_rows(t.cuda(), g.cuda(), None, torch.from_numpy(tokens).cuda(),
                                       torch.from_numpy(table).cuda(), 0.05, un.cuda())
        np.testing.assert_array_equal(dacc.cpu().numpy(), acc)
        ga_o, gt_o, _ = oracle_mod.verify_greedy(t, tokens, table, k, 0.05)
        ga, gt = lantern_gpu.verify_greedy(t.cuda(), torch.from_numpy(tokens).cuda(), torch.from_numpy(table).cuda(),
                                           0.05)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(ga.cpu().numpy(), ga_o)
        np.testing.assert_array_equal(gt.cpu().numpy(), gt_o)


def test_stream_read_probe(lantern_gpu):
    """The measurement aid only reads: it must run, reject bad arguments and leave its source untouched."""
    lib = lantern_gpu.load()
    src = torch.arange(3 * 65536 // 4, dtype=torch.int32, device="cuda")
    keep = src.clone()
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    assert lib.lantern_probe_stream_read(src.data_ptr(), None, src.numel() * 4, sink.data_ptr(), None) == 0
    assert lib.lantern_probe_stream_read(src.data_ptr(), src.data_ptr(), src.numel() * 4, sink.data_ptr(), None) == 0
    assert lib.lantern_probe_stream_read(src.data_ptr(), None, 100, sink.data_ptr(), None) == 0      # no whole chunk
    assert lib.lantern_probe_stream_read(None, None, 65536, sink.data_ptr(), None) == -1
    assert lib.lantern_probe_stream_read(src.data_ptr() + 4, None, 65536, sink.data_ptr(), None) == -2
    torch.cuda.synchronize()
    assert torch.equal(src, keep)


def test_concurrent_host_threads(oracle_mod, lantern_gpu):
    """Several host threads, each on a stream of its own, call the library at once (ctypes drops the
    interpreter lock during a call); every result must equal the oracle's."""
    import threading
    cfg = workloads.CONFIGS["llamagen_step"]
    table = random_table(cfg.V, cfg.k, seed=77)
    tb = torch.from_numpy(table).cuda()
    steps = [workloads.make_step(cfg, step=60 + i, rows=64, variant=("plain", "reject", "peaked")[i % 3])
             for i in range(4)]
    deltas = [0.4, 0.0, 0.01, 0.2]
    want = [oracle_mod.verify(s.target_logits, s.draft_logits, s.draft_tokens, table, cfg.k, d, s.uniforms,
                              threads=4, want_diag=False)[:2] for s, d in zip(steps, deltas)]
    dev = [(s.target_logits.cuda(), s.draft_logits.cuda(), s.draft_tokens.cuda(), s.uniforms.cuda()) for s in steps]
    torch.cuda.synchronize()
    errors = []

    def worker(i):
        try:
            stream = torch.cuda.Stream()
            t, g, tok, un = dev[i]
            for _ in range(15):
                acc, res = lantern_gpu.verify(t, g, tok, tb, deltas[i], un, stream=stream)
                dacc = lantern_gpu.decide_rows(t, g, None, tok, tb, deltas[i], un, stream=stream)
                stream.synchronize()
                if not (np.array_equal(acc.cpu().numpy(), want[i][0]) and np.array_equal(res.cpu().numpy(), want[i][1])
                        and np.array_equal(dacc.cpu().numpy(), want[i][0])):
                    errors.append(i)
        except Exception as exc:   # noqa: BLE001
            errors.append(repr(exc))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(4)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert not errors, errors


def test_checked_mode_raises_on_unusable_rows(lantern_gpu):
    """The binding's checked mode: the calls themselves are asynchronous and mark an unusable row with
    -1; checked=True waits for the stream and raises E_TOKEN naming the rows."""
    cfg = workloads.CONFIGS["tiny"]
    st = workloads.make_step(cfg, step=3, rows=32)
    table = torch.from_numpy(random_table(cfg.V, cfg.k, seed=2)).cuda()
    tokens = st.draft_tokens.clone()
    tokens[5] = cfg.V
    tokens[17] = -3
    args = (st.target_logits.cuda(), st.draft_logits.cuda())
    acc, res = lantern_gpu.verify(*args, tokens.cuda(), table, cfg.delta, st.uniforms.cuda())
    torch.cuda.synchronize()
    assert acc[5].item() == -1 and acc[17].item() == -1 and res[5].item() == -1
    with pytest.raises(lantern_gpu.LanternError) as info:
        lantern_gpu.verify(*args, tokens.cuda(), table, cfg.delta, st.uniforms.cuda(), checked=True)
    assert info.value.status == lantern_gpu.binding.E_TOKEN and info.value.rows == [5, 17]
    lantern_gpu.verify(*args, st.draft_tokens.cuda(), table, cfg.delta, st.uniforms.cuda(), checked=True)
