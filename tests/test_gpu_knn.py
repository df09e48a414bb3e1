"""GPU parity of lantern_build_knn against the CPU oracle: indices must be identical."""
import numpy as np
import pytest
import torch

from synth import workloads

pytestmark = pytest.mark.gpu


def _gpu_table(lantern, cb, k, metric="l2", max_exact_rows=None):
    out, exact_rows = lantern.build_knn(cb.cuda(), k, metric=metric, return_stats=True)
    torch.cuda.synchronize()
    if max_exact_rows is not None:  # the matrix-core pre-selection must settle (nearly) every row itself
        assert int(exact_rows.item()) <= max_exact_rows, f"{int(exact_rows.item())} rows took the all-pairs pass"
    return out.cpu().numpy()


def _check_structure(table, V, k):
    np.testing.assert_array_equal(table[:, 0], np.arange(V, dtype=np.int32))
    assert table.min() >= 0 and table.max() < V
    srt = np.sort(table, axis=1)
    assert np.all(srt[:, 1:] != srt[:, :-1]), "a row repeats a token"


def test_tiny_full_table(oracle_mod, lantern_gpu):
    cfg = workloads.CONFIGS["tiny"]
    cb = workloads.make_codebook(cfg)
    got = _gpu_table(lantern_gpu, cb, cfg.k, max_exact_rows=0)
    want = oracle_mod.build_knn(cb.numpy(), cfg.k, threads=8)
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("name", ["llamagen_step", "image_batch", "wide_latent", "stress"])
def test_full_size_tables(oracle_mod, lantern_gpu, name):
    """Full-size build on the GPU, every row of the table compared with the oracle's (each
    configuration has a codebook of its own seed)."""
    cfg = workloads.CONFIGS[name]
    cb = workloads.make_codebook(cfg)
    got = _gpu_table(lantern_gpu, cb, cfg.k, max_exact_rows=0)
    _check_structure(got, cfg.V, cfg.k)
    want = oracle_mod.build_knn(cb.float().numpy(), cfg.k, threads=16)
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("name", ["stress", "wide_latent"])
def test_full_size_cosine_tables(oracle_mod, lantern_gpu, name):
    """Cosine metric at full size: V=16384, d=8 fp32, k=1000 (codes scaled to unequal norms, so the
    order differs from the l2 one) and V=8192, d=256 bf16, k=100; whole tables compared."""
    cfg = workloads.CONFIGS[name]
    cb = workloads.make_codebook(cfg)
    if cfg.normalise:
        g = torch.Generator().manual_seed(cfg.index)
        cb = (cb * (torch.rand(cfg.V, 1, generator=g) * 3 + 0.25)).contiguous()
    got = _gpu_table(lantern_gpu, cb, cfg.k, metric="cosine")
    _check_structure(got, cfg.V, cfg.k)
    want = oracle_mod.build_knn(cb.float().numpy(), cfg.k, metric="cosine", threads=16)
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("V,d,k,dtype", [
    (1, 4, 1, torch.float32),
    (2, 1, 2, torch.float32),
    (17, 3, 17, torch.float32),      # k = V, odd width
    (300, 5, 40, torch.bfloat16),    # width not a multiple of the vector size
    (513, 64, 100, torch.bfloat16),
    (2500, 16, 700, torch.float32),  # more than one block of query rows, ragged tail
])
def test_shapes(oracle_mod, lantern_gpu, V, d, k, dtype):
    g = torch.Generator().manual_seed(V * 31 + d)
    cb = torch.randn(V, d, generator=g).to(dtype)
    got = _gpu_table(lantern_gpu, cb, k)
    want = oracle_mod.build_knn(cb.float().numpy(), k, threads=8)
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("V,d,k,dtype", [(20001, 8, 300, torch.float32), (32768, 16, 64, torch.bfloat16),
                                         (33000, 4, 20, torch.float32)])
def test_large_vocabularies(oracle_mod, lantern_gpu, V, d, k, dtype):
    """Vocabularies beyond 16384: 512 threads per row with the keys in registers up to 32768 tokens
    (ragged and full), and beyond that the variant that re-reads the keys; whole tables compared."""
    g = torch.Generator().manual_seed(V + d)
    cb = torch.randn(V, d, generator=g).to(dtype)
    got = _gpu_table(lantern_gpu, cb, k)
    _check_structure(got, V, k)
    want = oracle_mod.build_knn(cb.float().numpy(), k, threads=16)
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("V,d,k,dtype,metric", [
    (8192, 256, 300, torch.bfloat16, "l2"),      # matrix cores on bf16 codes, 16 steps of 16 coordinates
    (5000, 12, 260, torch.float32, "l2"),        # ragged last tile of rows and of columns
    (4100, 16, 58, torch.bfloat16, "l2"),        # smallest k of the path (65 candidates wanted), lists of 1024
    (4096, 8, 1009, torch.float32, "cosine"),    # smallest vocabulary and largest k of the path
    (40000, 8, 400, torch.float32, "l2"),        # beyond what the whole-row selection holds in registers
    # cosine with a ragged last strip of rows: the rows beyond the block have norm 0, and their keys
    # -g / sqrt(0) = -inf must not count as candidates (they once did, and their counters ran into row 0's list)
    (5000, 12, 260, torch.float32, "cosine"),
    (8328, 4, 736, torch.float32, "cosine"),
])
def test_sampled_threshold_path(oracle_mod, lantern_gpu, V, d, k, dtype, metric):
    """Shapes that take the sampled thresholds and the filtering contraction (4096 tokens or more,
    k - 1 + pad between 65 and 1024): whole tables compared, and no row may have needed the
    all-pairs pass (every list came out between what the selection wants and its capacity)."""
    g = torch.Generator().manual_seed(V * 7 + k)
    cb = torch.randn(V, d, generator=g).to(dtype)
    if metric == "cosine":
        cb = (cb * (torch.rand(V, 1, generator=g) * 3 + 0.25)).to(dtype).contiguous()
    got = _gpu_table(lantern_gpu, cb, k, metric=metric, max_exact_rows=0)
    _check_structure(got, V, k)
    want = oracle_mod.build_knn(cb.float().numpy(), k, metric=metric, threads=16)
    np.testing.assert_array_equal(got, want)


def test_heavy_tailed_norms_stay_on_the_fast_path(oracle_mod, lantern_gpu):
    """Codes whose norms spread over orders of magnitude: the error bound of the approximate keys
    grows with the norms, but a code of very large norm is far from a row of ordinary norm whatever
    its key's error, so the proof may leave such codes out of the bound; without that nearly every
    row went to the all-pairs pass."""
    g = torch.Generator().manual_seed(31)
    V, d, k = 6000, 12, 300
    cb = (torch.randn(V, d, generator=g) * torch.exp(torch.randn(V, 1, generator=g))).contiguous()
    got = _gpu_table(lantern_gpu, cb, k, max_exact_rows=16)
    np.testing.assert_array_equal(got, oracle_mod.build_knn(cb.numpy(), k, threads=16))
    small = cb[:1500].contiguous()                       # the whole-row path (V < 4096)
    got = _gpu_table(lantern_gpu, small, 200, max_exact_rows=16)
    np.testing.assert_array_equal(got, oracle_mod.build_knn(small.numpy(), 200, threads=16))


def test_sampled_threshold_path_falls_back(oracle_mod, lantern_gpu):
    """The same shapes when the sample misleads or the lists overflow.  (a) 64 distinct codes, each
    64 times: whole shells of equal keys sit at every threshold, lists come out too long or too
    short, and the rows must be ranked by the all-pairs pass, not guessed.  (b) A codebook whose
    first byte is not 16-byte aligned cannot use the matrix cores: it takes whole key blocks in a
    workspace that was sized for the lists."""
    rng = np.random.default_rng(11)
    base = rng.standard_normal((64, 8)).astype(np.float32)
    dup = np.repeat(base, 64, axis=0)[rng.permutation(4096)]
    got, exact_rows = lantern_gpu.build_knn(torch.from_numpy(dup).cuda(), 300, return_stats=True)
    torch.cuda.synchronize()
    assert int(exact_rows.item()) > 0
    np.testing.assert_array_equal(got.cpu().numpy(), oracle_mod.build_knn(dup, 300, threads=16))

    g = torch.Generator().manual_seed(12)
    V, d, k = 6000, 8, 300
    holder = torch.randn(V * d + 1, generator=g).cuda()
    cb = holder[1:].view(V, d)                       # 4 bytes past an aligned address
    assert cb.data_ptr() % 16 != 0 and cb.is_contiguous()
    got = lantern_gpu.build_knn(cb, k)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(got.cpu().numpy(), oracle_mod.build_knn(cb.cpu().numpy(), k, threads=16))


def test_exact_ties_and_duplicates(oracle_mod, lantern_gpu):
    """Integer lattice (many exactly equal distances) and repeated codes: the
    lower index wins and the token itself stays in slot 0."""
    xs, ys, zs = np.meshgrid(np.arange(8), np.arange(8), np.arange(8), indexing="ij")
    lattice = np.stack([xs.ravel(), ys.ravel(), zs.ravel()], axis=1).astype(np.float32)
    for k in (7, 27, 200):
        got = _gpu_table(lantern_gpu, torch.from_numpy(lattice), k)
        want = oracle_mod.build_knn(lattice, k, threads=8)
        np.testing.assert_array_equal(got, want)
    # more equal keys than the candidate buffer holds: the rows must go to the all-pairs pass
    # (and be counted), not be guessed
    same = torch.ones(3000, 4)
    got, exact_rows = lantern_gpu.build_knn(same.cuda(), 5, return_stats=True)
    torch.cuda.synchronize()
    assert int(exact_rows.item()) == 3000
    np.testing.assert_array_equal(got.cpu().numpy(), oracle_mod.build_knn(same.numpy(), 5, threads=8))
    rng = np.random.default_rng(5)
    base = rng.standard_normal((40, 8)).astype(np.float32)
    dup = base[rng.integers(0, 40, 600)]           # 600 codes, only 40 distinct
    got = _gpu_table(lantern_gpu, torch.from_numpy(dup), 50)
    want = oracle_mod.build_knn(dup, 50, threads=8)
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("V,d,k,dtype,metric", [
    (2166, 1, 1475, torch.float32, "cosine"),    # every key is -1, +1 or missing: all rows through the all-pairs pass
    (500, 3, 500, torch.float32, "cosine"),      # direct keys, every token listed
    (2048, 8, 100, torch.float32, "cosine"),     # contraction, whole rows
    (2048, 8, 2048, torch.float32, "cosine"),
    (8192, 8, 300, torch.float32, "cosine"),     # sampled thresholds and candidate lists
    (4100, 16, 58, torch.bfloat16, "cosine"),
    (1000, 4, 50, torch.float32, "l2"),          # infinite coordinates under squared l2 (inf - inf)
])
def test_keys_that_are_not_numbers(oracle_mod, lantern_gpu, V, d, k, dtype, metric):
    """Codes of zero norm under the cosine key (0/0) and infinite coordinates under squared l2: such a pair
    counts as the farthest possible, equal keys by the lower index, on both sides."""
    g = torch.Generator().manual_seed(V + 13 * d + k)
    cb = torch.randn(V, d, generator=g)
    where = torch.randint(0, V, (5,), generator=g)
    where[0], where[1] = 0, V - 1
    if metric == "cosine":
        cb[where] = 0.0
        cb[8 * (V // 16)] = 0.0   # a stratum boundary of the token sample
    else:
        cb[where, 0] = float("inf")
    cb = cb.to(dtype).contiguous()
    got = _gpu_table(lantern_gpu, cb, k, metric=metric)
    want = oracle_mod.build_knn(cb.float().numpy(), k, metric=metric, threads=16)
    np.testing.assert_array_equal(got, want)


def test_cosine_metric(oracle_mod, lantern_gpu):
    g = torch.Generator().manual_seed(77)
    cb = torch.randn(700, 12, generator=g) * (torch.rand(700, 1, generator=g) * 4 + 0.2)
    got = _gpu_table(lantern_gpu, cb, 60, metric="cosine")
    want = oracle_mod.build_knn(cb.numpy(), 60, metric="cosine", threads=8)
    np.testing.assert_array_equal(got, want)


def test_table_feeds_verify(oracle_mod, lantern_gpu):
    """End to end on the device: the table built by the library drives verification."""
    from parity_utils import compare_verify
    cfg = workloads.CONFIGS["tiny"]
    cb = workloads.make_codebook(cfg)
    table = _gpu_table(lantern_gpu, cb, cfg.k)
    st = workloads.make_step(cfg, step=4)
    compare_verify(oracle_mod, lantern_gpu, st.target_logits, st.draft_logits, st.draft_tokens, table,
                   cfg.delta, st.uniforms, label="gpu table")
