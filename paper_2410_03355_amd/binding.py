"""Thin ctypes binding of liblantern.so: argument marshalling only.

PyTorch supplies device memory and the current HIP stream; every step of the
verification path runs in the library's kernels.  There is no CPU fallback: if
the library is missing, load() raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

from .build import LIB_PATH

F32, BF16 = 0, 1
METRIC_L2, METRIC_COSINE = 0, 1
MAX_VOCAB = 1 << 19

OK = 0
E_NULL, E_SHAPE, E_DTYPE, E_DELTA, E_TOKEN, E_WORKSPACE, E_DEVICE = -1, -2, -3, -4, -5, -6, -7

EXPORTS = (
    "lantern_build_knn_workspace_bytes", "lantern_build_knn", "lantern_build_knn_metric",
    "lantern_verify", "lantern_verify_ex", "lantern_verify_divergence", "lantern_verify_greedy",
    "lantern_accept_chains", "lantern_verify_rows", "lantern_verify_greedy_rows", "lantern_accept_trees",
    "lantern_build_random", "lantern_decide_rows", "lantern_resample_selected", "lantern_verify_trees",
    "lantern_verify_trees_greedy", "lantern_verify_trees_sequential_workspace_bytes",
    "lantern_verify_trees_sequential", "lantern_probe_stream_read", "lantern_prepare", "lantern_build_knn_static",
    "lantern_status_string",
    "lantern_version",
)

_lib = None


class LanternError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def load() -> ctypes.CDLL:
    """Loads the built library.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not found: build it with `python -m paper_2410_03355_amd.build` "
            "(there is no fallback implementation)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, f32, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
    lib.lantern_build_knn_workspace_bytes.argtypes = [i32, i32, i32, i32]
    lib.lantern_build_knn_workspace_bytes.restype = sz
    lib.lantern_build_knn.argtypes = [vp, i32, i32, i32, i32, vp, vp, sz, vp]
    lib.lantern_build_knn.restype = i32
    lib.lantern_build_knn_metric.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, sz, vp]
    lib.lantern_build_knn_metric.restype = i32
    lib.lantern_verify.argtypes = [vp, vp, i32, i32, i32, i64, vp, vp, i32, f32, vp, vp, vp, vp]
    lib.lantern_verify.restype = i32
    lib.lantern_verify_ex.argtypes = [vp, vp, i32, i32, i32, i64, vp, vp, i32, f32, vp, vp, vp,
                                      vp, vp, vp, vp, vp, vp]
    lib.lantern_verify_ex.restype = i32
    lib.lantern_verify_divergence.argtypes = [vp, vp, i32, i32, i32, i64, vp, vp, i32, i32, f32, vp, vp, vp,
                                              vp, vp, vp, vp, vp, vp]
    lib.lantern_verify_divergence.restype = i32
    lib.lantern_verify_greedy.argtypes = [vp, i32, i32, i32, i64, vp, vp, i32, f32, vp, vp, vp, vp]
    lib.lantern_verify_greedy.restype = i32
    lib.lantern_accept_chains.argtypes = [vp, vp, i32, i32, vp, vp, vp]
    lib.lantern_accept_chains.restype = i32
    lib.lantern_verify_rows.argtypes = [vp, vp, i32, i32, i32, i64, vp, i32, vp, vp, i32, i32, f32, vp, vp, vp, vp]
    lib.lantern_verify_rows.restype = i32
    lib.lantern_verify_greedy_rows.argtypes = [vp, i32, i32, i32, i64, vp, i32, vp, vp, i32, f32, vp, vp, vp]
    lib.lantern_verify_greedy_rows.restype = i32
    lib.lantern_accept_trees.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp, vp]
    lib.lantern_accept_trees.restype = i32
    lib.lantern_decide_rows.argtypes = [vp, vp, i32, i32, i32, i64, vp, i32, vp, vp, i32, i32, f32, vp, vp, vp, vp]
    lib.lantern_decide_rows.restype = i32
    lib.lantern_resample_selected.argtypes = [vp, vp, i32, i32, i32, i64, vp, i32, vp, vp, i32, i32, f32, vp, vp,
                                              i32, vp, vp]
    lib.lantern_resample_selected.restype = i32
    lib.lantern_verify_trees.argtypes = [vp, vp, i32, i32, i32, i64, vp, vp, i32, i32, vp, vp, i32, i32, f32, vp,
                                         vp, vp, vp, vp, vp]
    lib.lantern_verify_trees.restype = i32
    lib.lantern_verify_trees_greedy.argtypes = [vp, i32, i32, i32, i64, vp, vp, i32, i32, vp, vp, i32, f32, vp, vp, vp,
                                                vp, vp, vp]
    lib.lantern_verify_trees_greedy.restype = i32
    lib.lantern_verify_trees_sequential_workspace_bytes.argtypes = [i32, i32, i32]
    lib.lantern_verify_trees_sequential_workspace_bytes.restype = sz
    lib.lantern_verify_trees_sequential.argtypes = [vp, vp, i32, i32, i32, i64, vp, vp, i32, i32, vp, vp, i32, i32, f32,
                                                    vp, vp, vp, vp, vp, sz, vp]
    lib.lantern_verify_trees_sequential.restype = i32
    lib.lantern_probe_stream_read.argtypes = [vp, vp, sz, vp, vp]
    lib.lantern_probe_stream_read.restype = i32
    lib.lantern_build_random.argtypes = [i32, i32, ctypes.c_uint64, vp, vp]
    lib.lantern_build_random.restype = i32
    lib.lantern_build_knn_static.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, vp]
    lib.lantern_build_knn_static.restype = i32
    lib.lantern_prepare.argtypes = [i32, i32, i32]
    lib.lantern_prepare.restype = i32
    lib.lantern_status_string.argtypes = [i32]
    lib.lantern_status_string.restype = ctypes.c_char_p
    lib.lantern_version.argtypes = []
    lib.lantern_version.restype = i32
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().lantern_status_string(int(status)).decode()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}: float32 or bfloat16 expected")


def prepare(logits_dtype, V: int, k: int) -> None:
    """lantern_prepare: raises the LDS limits of every verification kernel for this logit dtype
    (torch.float32 / torch.bfloat16), vocabulary size and table width on the current device, so that
    later calls make no runtime call besides their launches (needed before stream capture)."""
    code = {torch.float32: F32, torch.bfloat16: BF16}[logits_dtype]
    rc = load().lantern_prepare(code, int(V), int(k))
    if rc != OK:
        raise LanternError(rc, "lantern_prepare")


def _stream_ptr(stream) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def _need_cuda(*tensors):
    for t in tensors:
        if t is not None and not t.is_cuda:
            raise ValueError("all tensors must live in device memory")


def knn_workspace_bytes(cb_dtype: int, V: int, d: int, k: int) -> int:
    return int(load().lantern_build_knn_workspace_bytes(cb_dtype, V, d, k))


def build_knn(codebook: torch.Tensor, k: int, metric: str = "l2", stream=None, return_stats: bool = False,
              workspace: torch.Tensor = None, out: torch.Tensor = None):
    """lantern_build_knn on a [V, d] device tensor; returns int32 [V, k] on the device.
    With return_stats also a device int32 scalar tensor: rows ranked by the exact all-pairs pass.
    workspace (uint8, at least knn_workspace_bytes, 256-byte aligned) and out ([V, k] int32) may be
    brought by the caller, who then builds several tables without allocating in between."""
    lib = load()
    _need_cuda(codebook)
    if codebook.dim() != 2 or not codebook.is_contiguous():
        raise ValueError("codebook must be a contiguous [V, d] tensor")
    V, d = codebook.shape
    code = _dtype_code(codebook)
    nbytes = knn_workspace_bytes(code, V, d, k)
    if nbytes == 0:
        raise LanternError(E_SHAPE, "lantern_build_knn_workspace_bytes")
    if workspace is None:
        ws = torch.empty(nbytes, dtype=torch.uint8, device=codebook.device)
    else:
        _need_cuda(workspace)
        if workspace.dtype != torch.uint8 or not workspace.is_contiguous() or workspace.numel() < nbytes:
            raise ValueError("workspace must be a contiguous uint8 tensor of at least knn_workspace_bytes")
        ws = workspace
    if out is None:
        out = torch.empty((V, k), dtype=torch.int32, device=codebook.device)
    else:
        _need_cuda(out)
        if out.dtype != torch.int32 or tuple(out.shape) != (V, k) or not out.is_contiguous():
            raise ValueError("out must be a contiguous int32 [V, k] tensor")
    rc = lib.lantern_build_knn_metric(codebook.data_ptr(), code, V, d, k,
                                      {"l2": METRIC_L2, "cosine": METRIC_COSINE}[metric],
                                      out.data_ptr(), ws.data_ptr(), ws.numel(), _stream_ptr(stream))
    if rc != OK:
        raise LanternError(rc, "lantern_build_knn")
    if workspace is None:
        ws.record_stream(torch.cuda.current_stream() if stream is None else stream)
    if return_stats:
        return out, ws[:4].view(torch.int32)[0]
    return out


STATIC_MAX_V = 32768


def build_knn_static(codebook: torch.Tensor, k: int, out: torch.Tensor, metric: str = "l2", exact_rows=None,
                     stream=None) -> None:
    """lantern_build_knn_static: the table into the caller's `out` ([V, k] int32, device) using the
    library's static scratch; this wrapper allocates nothing either.  exact_rows: device int32
    tensor of one element, or None."""
    lib = load()
    _need_cuda(codebook, out, exact_rows)
    if codebook.dim() != 2 or not codebook.is_contiguous():
        raise ValueError("codebook must be a contiguous [V, d] tensor")
    V, d = codebook.shape
    if out.dtype != torch.int32 or tuple(out.shape) != (V, k) or not out.is_contiguous():
        raise ValueError("out must be a contiguous int32 [V, k] tensor")
    rc = lib.lantern_build_knn_static(codebook.data_ptr(), _dtype_code(codebook), V, d, k,
                                      {"l2": METRIC_L2, "cosine": METRIC_COSINE}[metric], out.data_ptr(),
                                      None if exact_rows is None else exact_rows.data_ptr(), _stream_ptr(stream))
    if rc != OK:
        raise LanternError(rc, "lantern_build_knn_static")


def _check_verify_args(target_logits, draft_logits, draft_tokens, knn, uniforms):
    _need_cuda(target_logits, draft_logits, draft_tokens, knn, uniforms)
    if target_logits.dim() != 2 or target_logits.shape != draft_logits.shape:
        raise ValueError("logits must be two [N, V] tensors of equal shape")
    if target_logits.dtype != draft_logits.dtype:
        raise TypeError("target and draft logits must share a dtype")
    if target_logits.stride(1) != 1 or draft_logits.stride(1) != 1 or \
            target_logits.stride(0) != draft_logits.stride(0):
        raise ValueError("logit rows must be dense and both tensors must share the row stride")
    N, V = target_logits.shape
    if draft_tokens.dtype != torch.int32 or knn.dtype != torch.int32 or uniforms.dtype != torch.float32:
        raise TypeError("draft_tokens and knn must be int32, uniforms float32")
    if draft_tokens.numel() != N or uniforms.numel() != 2 * N or knn.dim() != 2 or knn.shape[0] != V:
        raise ValueError("shape mismatch between logits, tokens, uniforms and the table")
    if not (draft_tokens.is_contiguous() and knn.is_contiguous() and uniforms.is_contiguous()):
        raise ValueError("draft_tokens, knn and uniforms must be contiguous")
    return N, V, int(knn.shape[1])


def _raise_if_unusable(acc, stream, where: str):
    """Checked mode: waits for the call's stream and raises E_TOKEN if any verification came back unusable."""
    (torch.cuda.current_stream(acc.device) if stream is None else stream).synchronize()
    bad = torch.nonzero(acc < 0).flatten()
    if bad.numel():
        err = LanternError(E_TOKEN, where)
        err.rows = bad.cpu().tolist()
        raise err


def verify(target_logits, draft_logits, draft_tokens, knn, delta: float, uniforms,
           out_accept=None, out_resample=None, stream=None, checked: bool = False):
    """lantern_verify; returns (accept int32[N], resample int32[N]) device tensors.
    checked: synchronise and raise LanternError(E_TOKEN) (with .rows) if a verification was unusable; by
    default the call is asynchronous and such rows carry -1 in both outputs."""
    lib = load()
    N, V, k = _check_verify_args(target_logits, draft_logits, draft_tokens, knn, uniforms)
    dev = target_logits.device
    acc = torch.empty(N, dtype=torch.int32, device=dev) if out_accept is None else out_accept
    res = torch.empty(N, dtype=torch.int32, device=dev) if out_resample is None else out_resample
    rc = lib.lantern_verify(target_logits.data_ptr(), draft_logits.data_ptr(),
                            _dtype_code(target_logits), N, V, target_logits.stride(0) if N > 1 else V,
                            draft_tokens.data_ptr(), knn.data_ptr(), k, float(delta),
                            uniforms.data_ptr(), acc.data_ptr(), res.data_ptr(), _stream_ptr(stream))
    if rc != OK:
        raise LanternError(rc, "lantern_verify")
    if checked:
        _raise_if_unusable(acc, stream, "lantern_verify")
    return acc, res


DIV_TVD, DIV_JSD = 0, 1


def verify_ex(target_logits, draft_logits, draft_tokens, knn, delta: float, uniforms, stream=None,
              divergence: str = "tvd"):
    """lantern_verify_ex (divergence "tvd") or lantern_verify_divergence ("jsd"); returns a dict of
    device tensors with all diagnostics."""
    lib = load()
    N, V, k = _check_verify_args(target_logits, draft_logits, draft_tokens, knn, uniforms)
    dev = target_logits.device
    out = {
        "accept": torch.empty(N, dtype=torch.int32, device=dev),
        "resample": torch.empty(N, dtype=torch.int32, device=dev),
        "accept_prob": torch.empty(N, dtype=torch.float32, device=dev),
        "mass": torch.empty(N, dtype=torch.float32, device=dev),
        "g_tok": torch.empty(N, dtype=torch.float32, device=dev),
        "a_size": torch.empty(N, dtype=torch.int32, device=dev),
        "path": torch.empty(N, dtype=torch.int32, device=dev),
    }
    common_in = (target_logits.data_ptr(), draft_logits.data_ptr(), _dtype_code(target_logits), N, V,
                 target_logits.stride(0) if N > 1 else V, draft_tokens.data_ptr(), knn.data_ptr(), k)
    common_out = (uniforms.data_ptr(), out["accept"].data_ptr(), out["resample"].data_ptr(),
                  out["accept_prob"].data_ptr(), out["mass"].data_ptr(), out["g_tok"].data_ptr(),
                  out["a_size"].data_ptr(), out["path"].data_ptr(), _stream_ptr(stream))
    if divergence == "tvd":
        rc = lib.lantern_verify_ex(*common_in, float(delta), *common_out)
    else:
        rc = lib.lantern_verify_divergence(*common_in, {"jsd": DIV_JSD}[divergence], float(delta), *common_out)
    if rc != OK:
        raise LanternError(rc, "lantern_verify_ex")
    return out


def verify_greedy(target_logits, draft_tokens, knn, delta: float, stream=None, want_path: bool = False):
    """lantern_verify_greedy; returns (accept int32[N], token int32[N]) device tensors
    (and the per-row path tensor when want_path)."""
    lib = load()
    _need_cuda(target_logits, draft_tokens, knn)
    if target_logits.dim() != 2 or target_logits.stride(1) != 1:
        raise ValueError("logits must be a [N, V] tensor with dense rows")
    N, V = target_logits.shape
    if draft_tokens.dtype != torch.int32 or knn.dtype != torch.int32:
        raise TypeError("draft_tokens and knn must be int32")
    if draft_tokens.numel() != N or knn.dim() != 2 or knn.shape[0] != V:
        raise ValueError("shape mismatch between logits, tokens and the table")
    if not (draft_tokens.is_contiguous() and knn.is_contiguous()):
        raise ValueError("draft_tokens and knn must be contiguous")
    dev = target_logits.device
    acc = torch.empty(N, dtype=torch.int32, device=dev)
    tok = torch.empty(N, dtype=torch.int32, device=dev)
    path = torch.empty(N, dtype=torch.int32, device=dev) if want_path else None
    rc = lib.lantern_verify_greedy(target_logits.data_ptr(), _dtype_code(target_logits), N, V,
                                   target_logits.stride(0) if N > 1 else V, draft_tokens.data_ptr(),
                                   knn.data_ptr(), int(knn.shape[1]), float(delta), acc.data_ptr(),
                                   tok.data_ptr(), path.data_ptr() if want_path else None,
                                   _stream_ptr(stream))
    if rc != OK:
        raise LanternError(rc, "lantern_verify_greedy")
    return (acc, tok, path) if want_path else (acc, tok)


def accept_chains(accept, resample, L: int, stream=None):
    """lantern_accept_chains; accept / resample are int32 device tensors of B*L rows.
    Returns (kept int32[B], next_token int32[B])."""
    lib = load()
    _need_cuda(accept, resample)
    if accept.dtype != torch.int32 or resample.dtype != torch.int32:
        raise TypeError("accept and resample must be int32")
    if accept.numel() != resample.numel() or L < 1 or accept.numel() % L:
        raise ValueError("accept and resample must hold B*L rows")
    if not (accept.is_contiguous() and resample.is_contiguous()):
        raise ValueError("accept and resample must be contiguous")
    B = accept.numel() // L
    kept = torch.empty(B, dtype=torch.int32, device=accept.device)
    nxt = torch.empty(B, dtype=torch.int32, device=accept.device)
    rc = lib.lantern_accept_chains(accept.data_ptr(), resample.data_ptr(), B, int(L), kept.data_ptr(),
                                   nxt.data_ptr(), _stream_ptr(stream))
    if rc != OK:
        raise LanternError(rc, "lantern_accept_chains")
    return kept, nxt


def _check_row_index(row_index, N):
    if row_index.dtype != torch.int32 or not row_index.is_contiguous() or row_index.numel() != N:
        raise ValueError("row_index must be a contiguous int32 tensor with one entry per verification")


def verify_rows(target_logits, draft_logits, row_index, draft_tokens, knn, delta: float, uniforms,
                divergence: str = "tvd", stream=None):
    """lantern_verify_rows: verification i reads logit row row_index[i].
    Returns (accept int32[N], resample int32[N]) device tensors."""
    lib = load()
    _need_cuda(target_logits, draft_logits, row_index, draft_tokens, knn, uniforms)
    if target_logits.dim() != 2 or target_logits.shape != draft_logits.shape or \
            target_logits.dtype != draft_logits.dtype:
        raise ValueError("logits must be two [R, V] tensors of equal shape and dtype")
    if target_logits.stride(1) != 1 or draft_logits.stride(1) != 1 or \
            target_logits.stride(0) != draft_logits.stride(0):
        raise ValueError("logit rows must be dense and both tensors must share the row stride")
    R, V = target_logits.shape
    N = draft_tokens.numel()
    _check_row_index(row_index, N)
    if draft_tokens.dtype != torch.int32 or knn.dtype != torch.int32 or uniforms.dtype != torch.float32:
        raise TypeError("draft_tokens and knn must be int32, uniforms float32")
    if uniforms.numel() != 2 * N or knn.dim() != 2 or knn.shape[0] != V:
        raise ValueError("shape mismatch between tokens, uniforms and the table")
    if not (draft_tokens.is_contiguous() and knn.is_contiguous() and uniforms.is_contiguous()):
        raise ValueError("draft_tokens, knn and uniforms must be contiguous")
    dev = target_logits.device
    acc = torch.empty(N, dtype=torch.int32, device=dev)
    res = torch.empty(N, dtype=torch.int32, device=dev)
    rc = lib.lantern_verify_rows(target_logits.data_ptr(), draft_logits.data_ptr(), _dtype_code(target_logits),
                                 R, V, target_logits.stride(0) if R > 1 else V, row_index.data_ptr(), N,
                                 draft_tokens.data_ptr(), knn.data_ptr(), int(knn.shape[1]),
                                 {"tvd": DIV_TVD, "jsd": DIV_JSD}[divergence], float(delta),
                                 uniforms.data_ptr(), acc.data_ptr(), res.data_ptr(), _stream_ptr(stream))
    if rc != OK:
        raise LanternError(rc, "lantern_verify_rows")
    return acc, res


def verify_greedy_rows(target_logits, row_index, draft_tokens, knn, delta: float, stream=None):
    """lantern_verify_greedy_rows; returns (accept int32[N], token int32[N]) device tensors."""
    lib = load()
    _need_cuda(target_logits, row_index, draft_tokens, knn)
    if target_logits.dim() != 2 or target_logits.stride(1) != 1:
        raise ValueError("logits must be a [R, V] tensor with dense rows")
    R, V = target_logits.shape
    N = draft_tokens.numel()
    _check_row_index(row_index, N)
    if draft_tokens.dtype != torch.int32 or knn.dtype != torch.int32:
        raise TypeError("draft_tokens and knn must be int32")
    if knn.dim() != 2 or knn.shape[0] != V or not (draft_tokens.is_contiguous() and knn.is_contiguous()):
        raise ValueError("the table must be a contiguous [V, k] tensor, the tokens contiguous")
    dev = target_logits.device
    acc = torch.empty(N, dtype=torch.int32, device=dev)
    tok = torch.empty(N, dtype=torch.int32, device=dev)
    rc = lib.lantern_verify_greedy_rows(target_logits.data_ptr(), _dtype_code(target_logits), R, V,
                                        target_logits.stride(0) if R > 1 else V, row_index.data_ptr(), N,
                                        draft_tokens.data_ptr(), knn.data_ptr(), int(knn.shape[1]), float(delta),
                                        acc.data_ptr(), tok.data_ptr(), _stream_ptr(stream))
    if rc != OK:
        raise LanternError(rc, "lantern_verify_greedy_rows")
    return acc, tok


def accept_trees(accept, resample, parent, M: int, stream=None):
    """lantern_accept_trees; accept / resample / parent are int32 device tensors of B*M rows.
    Returns (len int32[B], path int32[B, M], next_token int32[B])."""
    lib = load()
    given = [t for t in (accept, resample, parent) if t is not None]
    _need_cuda(*given)
    for t in given:
        if t.dtype != torch.int32 or not t.is_contiguous():
            raise TypeError("accept, resample and parent must be contiguous int32 tensors")
    if any(t.numel() != accept.numel() for t in given) or M < 1 or accept.numel() % M:
        raise ValueError("accept, resample and parent must hold B*M rows")
    B = accept.numel() // M
    dev = accept.device
    n = torch.empty(B, dtype=torch.int32, device=dev)
    path = torch.empty((B, M), dtype=torch.int32, device=dev)
    nxt = torch.empty(B, dtype=torch.int32, device=dev)
    rc = lib.lantern_accept_trees(accept.data_ptr(), None if resample is None else resample.data_ptr(),
                                  parent.data_ptr(), B, int(M),
                                  n.data_ptr(), path.data_ptr(), nxt.data_ptr(), _stream_ptr(stream))
    if rc != OK:
        raise LanternError(rc, "lantern_accept_trees")
    return n, path, nxt


RANDOM_MAX_K = 4096


def build_random(V: int, k: int, seed: int, device="cuda", stream=None):
    """lantern_build_random; returns the [V, k] int32 table on the device."""
    lib = load()
    out = torch.empty((V, k), dtype=torch.int32, device=device)
    rc = lib.lantern_build_random(int(V), int(k), int(seed) & 0xFFFFFFFFFFFFFFFF, out.data_ptr(),
                                  _stream_ptr(stream))
    if rc != OK:
        raise LanternError(rc, "lantern_build_random")
    return out


def _rows_args(target_logits, draft_logits, row_index, draft_tokens, knn, uniforms):
    _need_cuda(target_logits, draft_logits, draft_tokens, knn, uniforms)
    if target_logits.dim() != 2 or target_logits.shape != draft_logits.shape or \
            target_logits.dtype != draft_logits.dtype:
        raise ValueError("logits must be two [R, V] tensors of equal shape and dtype")
    if target_logits.stride(1) != 1 or draft_logits.stride(1) != 1 or \
            target_logits.stride(0) != draft_logits.stride(0):
        raise ValueError("logit rows must be dense and both tensors must share the row stride")
    R, V = target_logits.shape
    N = draft_tokens.numel()
    if row_index is not None:
        _need_cuda(row_index)
        _check_row_index(row_index, N)
    elif R != N:
        raise ValueError("without row_index there must be one logit row per verification")
    if draft_tokens.dtype != torch.int32 or knn.dtype != torch.int32 or uniforms.dtype != torch.float32:
        raise TypeError("draft_tokens and knn must be int32, uniforms float32")
    if uniforms.numel() != 2 * N or knn.dim() != 2 or knn.shape[0] != V:
        raise ValueError("shape mismatch between tokens, uniforms and the table")
    if not (draft_tokens.is_contiguous() and knn.is_contiguous() and uniforms.is_contiguous()):
        raise ValueError("draft_tokens, knn and uniforms must be contiguous")
    return R, V, N, target_logits.stride(0) if R > 1 else V


def decide_rows(target_logits, draft_logits, row_index, draft_tokens, knn, delta: float, uniforms,
                divergence: str = "tvd", stream=None, want_path: bool = False):
    """lantern_decide_rows; returns accept int32[N] (device), and the per-row path tensor when want_path."""
    lib = load()
    R, V, N, stride = _rows_args(target_logits, draft_logits, row_index, draft_tokens, knn, uniforms)
    acc = torch.empty(N, dtype=torch.int32, device=target_logits.device)
    path = torch.empty(N, dtype=torch.int32, device=target_logits.device) if want_path else None
    rc = lib.lantern_decide_rows(target_logits.data_ptr(), draft_logits.data_ptr(), _dtype_code(target_logits),
                                 R, V, stride, None if row_index is None else row_index.data_ptr(), N,
                                 draft_tokens.data_ptr(), knn.data_ptr(), int(knn.shape[1]),
                                 {"tvd": DIV_TVD, "jsd": DIV_JSD}[divergence], float(delta),
                                 uniforms.data_ptr(), acc.data_ptr(),
                                 path.data_ptr() if want_path else None, _stream_ptr(stream))
    if rc != OK:
        raise LanternError(rc, "lantern_decide_rows")
    return (acc, path) if want_path else acc


def resample_selected(target_logits, draft_logits, row_index, draft_tokens, knn, delta: float, uniforms,
                      select, divergence: str = "tvd", stream=None):
    """lantern_resample_selected; returns token int32[len(select)] (device)."""
    lib = load()
    R, V, N, stride = _rows_args(target_logits, draft_logits, row_index, draft_tokens, knn, uniforms)
    _need_cuda(select)
    if select.dtype != torch.int32 or not select.is_contiguous():
        raise TypeError("select must be a contiguous int32 tensor")
    out = torch.empty(select.numel(), dtype=torch.int32, device=target_logits.device)
    rc = lib.lantern_resample_selected(target_logits.data_ptr(), draft_logits.data_ptr(),
                                       _dtype_code(target_logits), R, V, stride,
                                       None if row_index is None else row_index.data_ptr(), N,
                                       draft_tokens.data_ptr(), knn.data_ptr(), int(knn.shape[1]),
                                       {"tvd": DIV_TVD, "jsd": DIV_JSD}[divergence], float(delta),
                                       uniforms.data_ptr(), select.data_ptr(), select.numel(), out.data_ptr(),
                                       _stream_ptr(stream))
    if rc != OK:
        raise LanternError(rc, "lantern_resample_selected")
    return out


def verify_trees(target_logits, draft_logits, row_index, parent, M: int, draft_tokens, knn, delta: float,
                 uniforms, divergence: str = "tvd", stream=None):
    """lantern_verify_trees; returns (accept int32[B*M], len int32[B], path int32[B, M], next int32[B])."""
    lib = load()
    R, V, N, stride = _rows_args(target_logits, draft_logits, row_index, draft_tokens, knn, uniforms)
    _need_cuda(parent)
    if parent.dtype != torch.int32 or not parent.is_contiguous() or parent.numel() != N or M < 1 or N % M:
        raise ValueError("parent must be a contiguous int32 tensor of B*M entries")
    B = N // M
    dev = target_logits.device
    acc = torch.empty(N, dtype=torch.int32, device=dev)
    n = torch.empty(B, dtype=torch.int32, device=dev)
    path = torch.empty((B, M), dtype=torch.int32, device=dev)
    nxt = torch.empty(B, dtype=torch.int32, device=dev)
    rc = lib.lantern_verify_trees(target_logits.data_ptr(), draft_logits.data_ptr(), _dtype_code(target_logits),
                                  R, V, stride, None if row_index is None else row_index.data_ptr(),
                                  parent.data_ptr(), B, int(M),
                                  draft_tokens.data_ptr(), knn.data_ptr(), int(knn.shape[1]),
                                  {"tvd": DIV_TVD, "jsd": DIV_JSD}[divergence], float(delta), uniforms.data_ptr(),
                                  acc.data_ptr(), n.data_ptr(), path.data_ptr(), nxt.data_ptr(), _stream_ptr(stream))
    if rc != OK:
        raise LanternError(rc, "lantern_verify_trees")
    return acc, n, path, nxt


def verify_trees_sequential(target_logits, draft_logits, row_index, parent, M: int, draft_tokens, knn, delta: float,
                            uniforms, divergence: str = "tvd", workspace=None, stream=None):
    """lantern_verify_trees_sequential; returns (len int32[B], path int32[B, M], next int32[B]).
    workspace: a uint8 device tensor of at least trees_sequential_workspace_bytes(B, M, V) bytes, or None
    to allocate one."""
    lib = load()
    R, V, N, stride = _rows_args(target_logits, draft_logits, row_index, draft_tokens, knn, uniforms)
    _need_cuda(parent)
    if parent.dtype != torch.int32 or not parent.is_contiguous() or parent.numel() != N or M < 1 or N % M:
        raise ValueError("parent must be a contiguous int32 tensor of B*M entries")
    B = N // M
    dev = target_logits.device
    need = int(lib.lantern_verify_trees_sequential_workspace_bytes(B, int(M), V))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    _need_cuda(workspace)
    n = torch.empty(B, dtype=torch.int32, device=dev)
    path = torch.empty((B, M), dtype=torch.int32, device=dev)
    nxt = torch.empty(B, dtype=torch.int32, device=dev)
    rc = lib.lantern_verify_trees_sequential(target_logits.data_ptr(), draft_logits.data_ptr(),
                                             _dtype_code(target_logits), R, V, stride,
                                             None if row_index is None else row_index.data_ptr(),
                                             parent.data_ptr(), B, int(M), draft_tokens.data_ptr(), knn.data_ptr(),
                                             int(knn.shape[1]), {"tvd": DIV_TVD, "jsd": DIV_JSD}[divergence],
                                             float(delta), uniforms.data_ptr(), n.data_ptr(), path.data_ptr(),
                                             nxt.data_ptr(), workspace.data_ptr(),
                                             workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    if rc != OK:
        raise LanternError(rc, "lantern_verify_trees_sequential")
    return n, path, nxt


def trees_sequential_workspace_bytes(B: int, M: int, V: int) -> int:
    return int(load().lantern_verify_trees_sequential_workspace_bytes(int(B), int(M), int(V)))


def verify_trees_greedy(target_logits, row_index, parent, M: int, draft_tokens, knn, delta: float, stream=None):
    """lantern_verify_trees_greedy; returns (accept int32[B*M], token int32[B*M], len int32[B],
    path int32[B, M], next int32[B])."""
    lib = load()
    given = [t for t in (target_logits, row_index, parent, draft_tokens, knn) if t is not None]
    _need_cuda(*given)
    if target_logits.dim() != 2 or target_logits.stride(1) != 1:
        raise ValueError("logits must be a [R, V] tensor with dense rows")
    R, V = target_logits.shape
    N = draft_tokens.numel()
    if row_index is not None:
        _check_row_index(row_index, N)
    elif R != N:
        raise ValueError("without row_index there must be one logit row per candidate")
    for t in (parent, draft_tokens, knn):
        if t.dtype != torch.int32 or not t.is_contiguous():
            raise TypeError("parent, draft_tokens and knn must be contiguous int32 tensors")
    if parent.numel() != N or M < 1 or N % M or knn.dim() != 2 or knn.shape[0] != V:
        raise ValueError("shape mismatch between parent, tokens and the table")
    B = N // M
    dev = target_logits.device
    acc = torch.empty(N, dtype=torch.int32, device=dev)
    tok = torch.empty(N, dtype=torch.int32, device=dev)
    n = torch.empty(B, dtype=torch.int32, device=dev)
    path = torch.empty((B, M), dtype=torch.int32, device=dev)
    nxt = torch.empty(B, dtype=torch.int32, device=dev)
    rc = lib.lantern_verify_trees_greedy(target_logits.data_ptr(), _dtype_code(target_logits), R, V,
                                         target_logits.stride(0) if R > 1 else V,
                                         None if row_index is None else row_index.data_ptr(), parent.data_ptr(), B,
                                         int(M), draft_tokens.data_ptr(), knn.data_ptr(), int(knn.shape[1]),
                                         float(delta), acc.data_ptr(), tok.data_ptr(), n.data_ptr(), path.data_ptr(),
                                         nxt.data_ptr(), _stream_ptr(stream))
    if rc != OK:
        raise LanternError(rc, "lantern_verify_trees_greedy")
    return acc, tok, n, path, nxt
