"""lantern_build_knn_static, the entry point that allocates nothing (its workspace is a static
device array inside the library), through the C ABI: same table, bit for bit, as
lantern_build_knn_metric, on two calls in a row of which the second has the smaller input."""
import ctypes
import gc

import numpy as np
import pytest
import torch

from synth import workloads

pytestmark = pytest.mark.gpu


def _static_table(lib, L, cb, k, metric):
    V, d = cb.shape
    out = torch.full((V, k), -7, dtype=torch.int32, device="cuda")
    stats = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    code = L.F32 if cb.dtype == torch.float32 else L.BF16

    def call():
        rc = lib.lantern_build_knn_static(ctypes.c_void_p(cb.data_ptr()), code, V, d, k, metric,
                                          ctypes.c_void_p(out.data_ptr()), ctypes.c_void_p(stats.data_ptr()),
                                          ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert rc == L.binding.OK, L.status_string(rc)
        torch.cuda.synchronize()

    # The runtime loads a code object, and with it the library's static device array, when one of its
    # kernels is first launched in the process: that is not the call allocating.  The readings are
    # taken around a second call of the same shape.
    call()
    out.fill_(-7)
    stats.fill_(-7)
    gc.collect()                       # nothing of an earlier test is freed between the two readings
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    free_before = torch.cuda.mem_get_info()[0]
    call()
    assert torch.cuda.memory_allocated() <= before        # nothing through torch's allocator
    assert torch.cuda.mem_get_info()[0] >= free_before    # nothing from the device directly
    return out.cpu().numpy(), int(stats.item())


def _workspace_table(lib, L, cb, k, metric):
    V, d = cb.shape
    code = L.F32 if cb.dtype == torch.float32 else L.BF16
    nbytes = lib.lantern_build_knn_workspace_bytes(code, V, d, k)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    out = torch.full((V, k), -9, dtype=torch.int32, device="cuda")
    rc = lib.lantern_build_knn_metric(ctypes.c_void_p(cb.data_ptr()), code, V, d, k, metric,
                                      ctypes.c_void_p(out.data_ptr()), ctypes.c_void_p(ws.data_ptr()), nbytes,
                                      ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == L.binding.OK, L.status_string(rc)
    torch.cuda.synchronize()
    return out.cpu().numpy(), int(ws[:4].view(torch.int32).item())


def test_static_scratch_build_matches_workspace_build(oracle_mod, lantern_gpu):
    L = lantern_gpu
    lib = L.load()
    cfg = workloads.CONFIGS["stress"]                       # V=16384, d=8 fp32, k=1000: several passes of 512 rows
    big = workloads.make_codebook(cfg).cuda()
    g = torch.Generator().manual_seed(3)
    small = torch.randn(2500, 16, generator=g).cuda()      # ragged tail, fewer rows than the first call
    same = torch.ones(300, 4).cuda()                        # every row goes to the all-pairs pass (uses its buffers)
    wide = workloads.make_codebook(workloads.CONFIGS["wide_latent"]).cuda()   # bf16, d=256
    for cb, k, metric in ((big, cfg.k, 0), (small, 700, 0), (same, 5, 0), (wide, 100, 1), (small, 60, 1)):
        got, got_exact = _static_table(lib, L, cb, k, metric)
        want, want_exact = _workspace_table(lib, L, cb, k, metric)
        np.testing.assert_array_equal(got, want)
        assert got_exact == want_exact
    # and against the oracle, for the smaller table
    got, _ = _static_table(lib, L, small, 700, 0)
    np.testing.assert_array_equal(got, oracle_mod.build_knn(small.cpu().numpy(), 700, threads=16))


def test_static_scratch_limit(lantern_gpu):
    L = lantern_gpu
    lib = L.load()
    V = L.binding.STATIC_MAX_V + 128
    cb = torch.zeros((V, 4), device="cuda")
    out = torch.full((V, 2), -7, dtype=torch.int32, device="cuda")
    rc = lib.lantern_build_knn_static(ctypes.c_void_p(cb.data_ptr()), L.F32, V, 4, 2, 0, ctypes.c_void_p(out.data_ptr()),
                                      None, None)
    assert rc == L.binding.E_WORKSPACE
    torch.cuda.synchronize()
    assert int((out != -7).sum()) == 0                      # nothing was launched
    # the largest size it serves
    V = L.binding.STATIC_MAX_V
    g = torch.Generator().manual_seed(5)
    cb = torch.randn(V, 4, generator=g).cuda()
    got, _ = _static_table(lib, L, cb, 8, 0)
    want, _ = _workspace_table(lib, L, cb, 8, 0)
    np.testing.assert_array_equal(got, want)
