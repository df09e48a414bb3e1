"""ctypes front end of the CPU oracle (oracle/lantern_oracle.c).

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by the smoke check and by the
bench's CPU-baseline leg; never by the product package.  All arithmetic lives
in the C file; this module widens inputs to fp32 storage (exact for bf16 and
fp32 values), calls the C routines and names the diagnostic columns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lantern_oracle.c")
_LIB = os.path.join(_HERE, "liblantern_oracle.so")

DIAG_NAMES = (
    "accept_prob", "mass", "g_tok", "t_tok", "tvd_walk", "tvd_direct", "resid_z",
    "a_size", "margin_accept", "margin_cut", "margin_cdf", "zero_resid",
)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  FP contraction is off so that the table's
    squared distances are separately rounded fp64 operations."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i32p = ctypes.POINTER(ctypes.c_int32)
        f32p = ctypes.POINTER(ctypes.c_float)
        f64p = ctypes.POINTER(ctypes.c_double)
        lib.oracle_build_knn_rows.argtypes = [f32p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                              ctypes.c_int, ctypes.c_int, ctypes.c_int, i32p,
                                              ctypes.c_int]
        lib.oracle_build_knn_rows.restype = ctypes.c_int
        lib.oracle_softmax.argtypes = [f32p, ctypes.c_int, f64p]
        lib.oracle_softmax.restype = ctypes.c_int
        lib.oracle_verify_probs.argtypes = [f64p, f64p, ctypes.c_int, ctypes.c_int, i32p,
                                            ctypes.c_int, ctypes.c_double, ctypes.c_double,
                                            ctypes.c_double, i32p, i32p, f64p, f64p, f64p]
        lib.oracle_verify_probs.restype = ctypes.c_int
        lib.oracle_verify.argtypes = [f32p, f32p, ctypes.c_int, ctypes.c_int, ctypes.c_int64,
                                      i32p, i32p, ctypes.c_int, ctypes.c_double, f32p, i32p, i32p,
                                      f64p, ctypes.c_int]
        lib.oracle_verify.restype = ctypes.c_int
        lib.oracle_verify_probs_div.argtypes = [f64p, f64p, ctypes.c_int, ctypes.c_int, i32p,
                                                ctypes.c_int, ctypes.c_int, ctypes.c_double, ctypes.c_double,
                                                ctypes.c_double, i32p, i32p, f64p, f64p, f64p]
        lib.oracle_verify_probs_div.restype = ctypes.c_int
        lib.oracle_verify_div.argtypes = [f32p, f32p, ctypes.c_int, ctypes.c_int, ctypes.c_int64,
                                          i32p, i32p, ctypes.c_int, ctypes.c_int, ctypes.c_double, f32p, i32p,
                                          i32p, f64p, ctypes.c_int]
        lib.oracle_verify_div.restype = ctypes.c_int
        lib.oracle_verify_greedy.argtypes = [f32p, ctypes.c_int, ctypes.c_int, ctypes.c_int64, i32p, i32p,
                                             ctypes.c_int, ctypes.c_double, i32p, i32p, f64p, ctypes.c_int]
        lib.oracle_verify_greedy.restype = ctypes.c_int
        lib.oracle_diag_count.restype = ctypes.c_int
        lib.oracle_max_threads.restype = ctypes.c_int
        assert lib.oracle_diag_count() == len(DIAG_NAMES)
        _lib = lib
    return _lib


def _as_f32(a) -> np.ndarray:
    """fp32 or bf16 values (numpy array or torch tensor) -> C-contiguous fp32 array."""
    if hasattr(a, "detach"):  # torch tensor; bf16 -> fp32 is exact
        a = a.detach().to("cpu").float().numpy()
    return np.ascontiguousarray(a, dtype=np.float32)


def _as_i32(a) -> np.ndarray:
    if hasattr(a, "detach"):
        a = a.detach().to("cpu").numpy()
    return np.ascontiguousarray(a, dtype=np.int32)


def _abi_delta(delta) -> float:
    """The bound as the library's C ABI carries it: a binary32 number.  The logits-level
    entry points below take their inputs in the ABI's types (fp32 / bf16 logits, fp32
    uniforms, a binary32 delta) and widen each of them exactly to fp64; the decision rule is
    then evaluated on that value, so 0.4 means 0.4000000059604645, on both sides."""
    return float(np.float32(delta))


def _p(a: np.ndarray, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def build_knn(codebook, k: int, rows=None, metric: str = "l2", threads: int = 1) -> np.ndarray:
    """Rows [rows[0], rows[1]) (default all) of the neighbour table, int32 [R, k]."""
    lib = _load()
    cb = _as_f32(codebook)
    V, d = cb.shape
    r0, r1 = (0, V) if rows is None else rows
    out = np.empty((r1 - r0, k), dtype=np.int32)
    rc = lib.oracle_build_knn_rows(_p(cb, ctypes.c_float), V, d, k, {"l2": 0, "cosine": 1}[metric],
                                   r0, r1, _p(out, ctypes.c_int32), threads)
    if rc != 0:
        raise ValueError("oracle_build_knn_rows: bad arguments")
    return out


def softmax(logits) -> np.ndarray:
    lib = _load()
    l = _as_f32(logits).reshape(-1)
    out = np.empty(l.shape[0], dtype=np.float64)
    rc = lib.oracle_softmax(_p(l, ctypes.c_float), l.shape[0], _p(out, ctypes.c_double))
    if rc != 0:
        raise ValueError("oracle_softmax: unusable row")
    return out


DIVERGENCES = {"tvd": 0, "jsd": 1}


def verify_probs(t, g, xt: int, nbrs, delta: float, u_acc: float, u_res: float,
                 want_dists: bool = False, divergence: str = "tvd") -> dict:
    """One verification on explicit probability vectors."""
    lib = _load()
    t = np.ascontiguousarray(t, dtype=np.float64)
    g = np.ascontiguousarray(g, dtype=np.float64)
    nb = _as_i32(nbrs)
    V = t.shape[0]
    acc = np.zeros(1, dtype=np.int32)
    res = np.zeros(1, dtype=np.int32)
    diag = np.empty(len(DIAG_NAMES), dtype=np.float64)
    rho = np.empty(V, dtype=np.float64) if want_dists else None
    ta = np.empty(V, dtype=np.float64) if want_dists else None
    rc = lib.oracle_verify_probs_div(_p(t, ctypes.c_double), _p(g, ctypes.c_double), V, int(xt),
                                 _p(nb, ctypes.c_int32), nb.shape[0], DIVERGENCES[divergence], float(delta),
                                 float(u_acc),
                                 float(u_res), _p(acc, ctypes.c_int32), _p(res, ctypes.c_int32),
                                 _p(diag, ctypes.c_double),
                                 _p(rho, ctypes.c_double) if want_dists else None,
                                 _p(ta, ctypes.c_double) if want_dists else None)
    if rc != 0:
        raise ValueError("oracle_verify_probs: bad arguments")
    out = {"accept": int(acc[0]), "resample": int(res[0])}
    out.update({n: float(v) for n, v in zip(DIAG_NAMES, diag)})
    out["a_size"] = int(out["a_size"])
    if want_dists:
        out["residual"] = rho
        out["distorted_target"] = ta
    return out


def verify(target_logits, draft_logits, draft_tokens, knn, k: int, delta: float, uniforms,
           threads: int = 1, want_diag: bool = True, divergence: str = "tvd"):
    """N verifications from logits.  Returns (accept int32[N], resample int32[N], diag dict|None)."""
    lib = _load()
    tl = _as_f32(target_logits)
    dl = _as_f32(draft_logits)
    if tl.ndim != 2 or tl.shape != dl.shape:
        raise ValueError("logits must be two [N, V] arrays of equal shape")
    N, V = tl.shape
    tok = _as_i32(draft_tokens).reshape(-1)
    tab = _as_i32(knn)
    un = _as_f32(uniforms).reshape(-1)
    if tok.shape[0] != N or un.shape[0] != 2 * N or tab.size != V * k:
        raise ValueError("shape mismatch")
    acc = np.empty(N, dtype=np.int32)
    res = np.empty(N, dtype=np.int32)
    diag = np.empty((N, len(DIAG_NAMES)), dtype=np.float64) if want_diag else None
    rc = lib.oracle_verify_div(_p(tl, ctypes.c_float), _p(dl, ctypes.c_float), N, V, V,
                           _p(tok, ctypes.c_int32), _p(tab, ctypes.c_int32), int(k), DIVERGENCES[divergence],
                           _abi_delta(delta),
                           _p(un, ctypes.c_float), _p(acc, ctypes.c_int32), _p(res, ctypes.c_int32),
                           _p(diag, ctypes.c_double) if want_diag else None, int(threads))
    if rc != 0:
        raise ValueError("oracle_verify: bad arguments")
    d = {n: diag[:, i] for i, n in enumerate(DIAG_NAMES)} if want_diag else None
    return acc, res, d


def verify_greedy(target_logits, draft_tokens, knn, k: int, delta: float, threads: int = 1):
    """Greedy-decoding variant.  Returns (accept int32[N], token int32[N], diag dict) where
    diag has mass, other (largest distorted-target value outside the draft token) and a_size."""
    lib = _load()
    tl = _as_f32(target_logits)
    if tl.ndim != 2:
        raise ValueError("logits must be [N, V]")
    N, V = tl.shape
    tok = _as_i32(draft_tokens).reshape(-1)
    tab = _as_i32(knn)
    if tok.shape[0] != N or tab.size != V * k:
        raise ValueError("shape mismatch")
    acc = np.empty(N, dtype=np.int32)
    out = np.empty(N, dtype=np.int32)
    diag = np.empty((N, 3), dtype=np.float64)
    rc = lib.oracle_verify_greedy(_p(tl, ctypes.c_float), N, V, V, _p(tok, ctypes.c_int32),
                                  _p(tab, ctypes.c_int32), int(k), _abi_delta(delta), _p(acc, ctypes.c_int32),
                                  _p(out, ctypes.c_int32), _p(diag, ctypes.c_double), int(threads))
    if rc != 0:
        raise ValueError("oracle_verify_greedy: bad arguments")
    return acc, out, {"mass": diag[:, 0], "other": diag[:, 1], "a_size": diag[:, 2]}


def accept_chains(accept, resample, L: int):
    """Walk of B drafted chains of L candidates; returns (kept int32[B], next_token int32[B])."""
    lib = _load()
    lib.oracle_accept_chains.argtypes = [ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32),
                                         ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_int32),
                                         ctypes.POINTER(ctypes.c_int32)]
    lib.oracle_accept_chains.restype = ctypes.c_int
    acc = _as_i32(accept).reshape(-1)
    res = _as_i32(resample).reshape(-1)
    if acc.shape != res.shape or acc.shape[0] % L:
        raise ValueError("shape mismatch")
    B = acc.shape[0] // L
    n = np.empty(B, dtype=np.int32)
    nxt = np.empty(B, dtype=np.int32)
    if lib.oracle_accept_chains(_p(acc, ctypes.c_int32), _p(res, ctypes.c_int32), B, L,
                                _p(n, ctypes.c_int32), _p(nxt, ctypes.c_int32)) != 0:
        raise ValueError("oracle_accept_chains: bad arguments")
    return n, nxt


def accept_trees(accept, resample, parent, M: int):
    """Walk of B drafted trees of M nodes; returns (len int32[B], path int32[B, M], next int32[B])."""
    lib = _load()
    P = ctypes.POINTER(ctypes.c_int32)
    lib.oracle_accept_trees.argtypes = [P, P, P, ctypes.c_int, ctypes.c_int, P, P, P]
    lib.oracle_accept_trees.restype = ctypes.c_int
    acc = _as_i32(accept).reshape(-1)
    res = _as_i32(resample).reshape(-1)
    par = _as_i32(parent).reshape(-1)
    if acc.shape != res.shape or acc.shape != par.shape or acc.shape[0] % M:
        raise ValueError("shape mismatch")
    B = acc.shape[0] // M
    n = np.empty(B, dtype=np.int32)
    path = np.empty((B, M), dtype=np.int32)
    nxt = np.empty(B, dtype=np.int32)
    if lib.oracle_accept_trees(_p(acc, ctypes.c_int32), _p(res, ctypes.c_int32), _p(par, ctypes.c_int32), B, M,
                               _p(n, ctypes.c_int32), _p(path, ctypes.c_int32), _p(nxt, ctypes.c_int32)) != 0:
        raise ValueError("oracle_accept_trees: bad arguments")
    return n, path, nxt


def verify_rows(target_logits, draft_logits, row_index, draft_tokens, knn, k: int, delta: float, uniforms,
                threads: int = 1, divergence: str = "tvd"):
    """N verifications over R shared logit rows: verification i reads row row_index[i] of both
    logit matrices (the siblings of a draft tree share the rows computed after their parent's
    prefix).  An index outside [0, R) makes that verification unusable (-1, -1).
    Returns (accept int32[N], resample int32[N], diag dict)."""
    tl = _as_f32(target_logits)
    dl = _as_f32(draft_logits)
    idx = np.asarray(row_index, dtype=np.int64).reshape(-1)
    ok = (idx >= 0) & (idx < tl.shape[0])
    safe = np.where(ok, idx, 0)
    acc, res, diag = verify(tl[safe], dl[safe], draft_tokens, knn, k, delta, uniforms, threads=threads,
                            divergence=divergence)
    acc[~ok] = -1
    res[~ok] = -1
    return acc, res, diag


def verify_greedy_rows(target_logits, row_index, draft_tokens, knn, k: int, delta: float, threads: int = 1):
    """Greedy-decoding variant over shared logit rows, as verify_rows."""
    tl = _as_f32(target_logits)
    idx = np.asarray(row_index, dtype=np.int64).reshape(-1)
    ok = (idx >= 0) & (idx < tl.shape[0])
    safe = np.where(ok, idx, 0)
    acc, tok, diag = verify_greedy(tl[safe], draft_tokens, knn, k, delta, threads=threads)
    acc[~ok] = -1
    tok[~ok] = -1
    return acc, tok, diag


def philox4x32_10(counter, key):
    """One Philox4x32-10 block: counter 4 words, key 2 words -> 4 words (uint32)."""
    lib = _load()
    U = ctypes.POINTER(ctypes.c_uint32)
    lib.oracle_philox4x32_10.argtypes = [U, U, U]
    lib.oracle_philox4x32_10.restype = None
    c = np.ascontiguousarray(np.asarray(counter, dtype=np.uint32).reshape(4))
    kk = np.ascontiguousarray(np.asarray(key, dtype=np.uint32).reshape(2))
    out = np.empty(4, dtype=np.uint32)
    lib.oracle_philox4x32_10(_p(c, ctypes.c_uint32), _p(kk, ctypes.c_uint32), _p(out, ctypes.c_uint32))
    return out


def build_random(V: int, k: int, seed: int, rows=None, threads: int = 8) -> np.ndarray:
    """Random neighbourhood table: token itself, then k-1 other tokens in random order.
    Returns int32 [r1-r0, k] for rows=(r0, r1), the whole table by default."""
    lib = _load()
    lib.oracle_build_random_rows.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_uint64, ctypes.c_int,
                                             ctypes.c_int, ctypes.POINTER(ctypes.c_int32), ctypes.c_int]
    lib.oracle_build_random_rows.restype = ctypes.c_int
    r0, r1 = (0, V) if rows is None else rows
    out = np.empty((r1 - r0, k), dtype=np.int32)
    if lib.oracle_build_random_rows(int(V), int(k), int(seed) & 0xFFFFFFFFFFFFFFFF, r0, r1,
                                    _p(out, ctypes.c_int32), int(threads)) != 0:
        raise ValueError("oracle_build_random_rows: bad arguments")
    return out


def sibling_group_probs(t, g, tokens, knn_rows, delta: float, u_acc, u_res, divergence: str = "tvd",
                        want_final: bool = True) -> dict:
    """One sibling group under the sequential-residual rule, on explicit probabilities (fp64
    interface: delta is taken as given).  tokens: the siblings' tokens in the order they are tried;
    knn_rows: [m, k] their table rows.  Returns taken (index or -1), next (token or -1),
    accept_prob [m] (NaN where not reached) and, with want_final, final_dist [V] = the
    distribution the following token is drawn from when every sibling is rejected."""
    lib = _load()
    D = ctypes.POINTER(ctypes.c_double)
    I = ctypes.POINTER(ctypes.c_int32)
    lib.oracle_sibling_group_probs.argtypes = [D, D, ctypes.c_int, ctypes.c_int, I, I, ctypes.c_int, ctypes.c_int,
                                               ctypes.c_double, D, D, I, I, D, D]
    lib.oracle_sibling_group_probs.restype = ctypes.c_int
    t = np.ascontiguousarray(t, dtype=np.float64)
    g = np.ascontiguousarray(g, dtype=np.float64)
    xs = _as_i32(tokens).reshape(-1)
    rows = _as_i32(knn_rows)
    m = xs.shape[0]
    if rows.ndim != 2 or rows.shape[0] != m:
        raise ValueError("knn_rows must be [m, k]")
    ua = np.ascontiguousarray(u_acc, dtype=np.float64).reshape(-1)
    ur = np.ascontiguousarray(u_res, dtype=np.float64).reshape(-1)
    taken = np.zeros(1, dtype=np.int32)
    nxt = np.zeros(1, dtype=np.int32)
    ap = np.empty(m, dtype=np.float64)
    fin = np.empty(t.shape[0], dtype=np.float64) if want_final else None
    rc = lib.oracle_sibling_group_probs(_p(t, ctypes.c_double), _p(g, ctypes.c_double), t.shape[0], m,
                                        _p(xs, ctypes.c_int32), _p(rows, ctypes.c_int32), rows.shape[1],
                                        DIVERGENCES[divergence], float(delta), _p(ua, ctypes.c_double),
                                        _p(ur, ctypes.c_double), _p(taken, ctypes.c_int32), _p(nxt, ctypes.c_int32),
                                        _p(ap, ctypes.c_double), _p(fin, ctypes.c_double) if want_final else None)
    if rc != 0:
        raise ValueError("oracle_sibling_group_probs: bad arguments")
    return {"taken": int(taken[0]), "next": int(nxt[0]), "accept_prob": ap, "final_dist": fin}


def verify_trees_sequential(target_logits, draft_logits, row_index, parent, M: int, draft_tokens, knn, k: int,
                            delta: float, uniforms, threads: int = 1, divergence: str = "tvd"):
    """Walk of B draft trees of M candidates under the sequential-residual sibling rule, from logits.
    Returns (len int32[B], path int32[B, M], next int32[B])."""
    lib = _load()
    F = ctypes.POINTER(ctypes.c_float)
    I = ctypes.POINTER(ctypes.c_int32)
    lib.oracle_verify_trees_sequential.argtypes = [F, F, ctypes.c_int, ctypes.c_int, ctypes.c_int64, I, I,
                                                   ctypes.c_int, ctypes.c_int, I, I, ctypes.c_int, ctypes.c_int,
                                                   ctypes.c_double, F, I, I, I, ctypes.c_int]
    lib.oracle_verify_trees_sequential.restype = ctypes.c_int
    tl = _as_f32(target_logits)
    dl = _as_f32(draft_logits)
    if tl.ndim != 2 or tl.shape != dl.shape:
        raise ValueError("logits must be two [R, V] arrays of equal shape")
    R, V = tl.shape
    ri = _as_i32(row_index).reshape(-1)
    par = _as_i32(parent).reshape(-1)
    tok = _as_i32(draft_tokens).reshape(-1)
    tab = _as_i32(knn)
    un = _as_f32(uniforms).reshape(-1)
    N = ri.shape[0]
    if N % M or par.shape[0] != N or tok.shape[0] != N or un.shape[0] != 2 * N or tab.size != V * k:
        raise ValueError("shape mismatch")
    B = N // M
    n = np.empty(B, dtype=np.int32)
    path = np.empty((B, M), dtype=np.int32)
    nxt = np.empty(B, dtype=np.int32)
    rc = lib.oracle_verify_trees_sequential(_p(tl, ctypes.c_float), _p(dl, ctypes.c_float), R, V, V,
                                            _p(ri, ctypes.c_int32), _p(par, ctypes.c_int32), B, M,
                                            _p(tok, ctypes.c_int32), _p(tab, ctypes.c_int32), int(k),
                                            DIVERGENCES[divergence], _abi_delta(delta), _p(un, ctypes.c_float),
                                            _p(n, ctypes.c_int32), _p(path, ctypes.c_int32), _p(nxt, ctypes.c_int32),
                                            int(threads))
    if rc != 0:
        raise ValueError("oracle_verify_trees_sequential: bad arguments")
    return n, path, nxt
