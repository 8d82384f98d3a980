"""ctypes front end of the C oracle (``nmf_mu_oracle.c``) plus two tiny
pure-Python routines used only to cross-check it on very small shapes.

TEST INFRASTRUCTURE ONLY.  Imported by ``tests/``, by the smoke check and by
the ``cpu_baseline`` leg of the benchmark; never by the GPU library or its
Python binding.  All arithmetic is IEEE double.  The iteration order is the
one of the paper's Algorithm 3 run on a single unit: H update, then W update
with the new H.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nmf_mu_oracle.c")
_LIB = os.path.join(_HERE, "libnmf_mu_oracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP, baseline x86-64) if needed."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(
            ["gcc", "-O3", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(_LIB)
    i64, i32, f64 = ctypes.c_int64, ctypes.c_int32, ctypes.c_double
    vp = ctypes.c_void_p
    lib.oracle_num_threads.restype = ctypes.c_int
    lib.oracle_get_mac_count.restype = ctypes.c_longlong
    lib.oracle_gram_w.argtypes = [vp, i64, i32, vp]
    lib.oracle_gram_h.argtypes = [vp, i32, i64, vp]
    lib.oracle_wta_dense.argtypes = [vp, i64, i64, vp, i32, vp]
    lib.oracle_aht_dense.argtypes = [vp, i64, i64, vp, i32, vp]
    lib.oracle_wta_csr.argtypes = [vp, vp, vp, i64, i64, vp, i32, vp]
    lib.oracle_aht_csr.argtypes = [vp, vp, vp, i64, i64, vp, i32, vp]
    lib.oracle_h_update.argtypes = [vp, vp, vp, i32, i64, f64]
    lib.oracle_w_update.argtypes = [vp, vp, vp, i64, i32, f64]
    lib.oracle_mu_dense.argtypes = [vp, i64, i64, i32, vp, vp, i32, f64]
    lib.oracle_mu_dense.restype = ctypes.c_int
    lib.oracle_mu_csr.argtypes = [vp, vp, vp, i64, i64, i32, vp, vp, i32, f64]
    lib.oracle_mu_csr.restype = ctypes.c_int
    lib.oracle_h_step_dense.argtypes = [vp, i64, i64, i32, vp, vp, f64]
    lib.oracle_h_step_dense.restype = ctypes.c_int
    lib.oracle_w_step_dense.argtypes = [vp, i64, i64, i32, vp, vp, f64]
    lib.oracle_w_step_dense.restype = ctypes.c_int
    lib.oracle_residual_dense.argtypes = [vp, i64, i64, i32, vp, vp]
    lib.oracle_residual_dense.restype = f64
    _lib = lib
    return lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _f32(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.float32)
    if shape is not None:
        assert a.shape == shape, (a.shape, shape)
    return a


def _f64(a, shape=None):
    a = np.array(a, dtype=np.float64, order="C", copy=True)
    if shape is not None:
        assert a.shape == shape, (a.shape, shape)
    return a


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def reset_mac_count() -> None:
    _load().oracle_reset_mac_count()


def mac_count() -> int:
    return int(_load().oracle_get_mac_count())


# ---- single products (Algorithm 3, one line each) -------------------------

def gram_w(W):
    W = _f64(W)
    m, k = W.shape
    G = np.empty((k, k))
    _load().oracle_gram_w(_p(W), m, k, _p(G))
    return G


def gram_h(H):
    H = _f64(H)
    k, n = H.shape
    G = np.empty((k, k))
    _load().oracle_gram_h(_p(H), k, n, _p(G))
    return G


def wta_dense(A, W):
    A = _f32(A)
    W = _f64(W)
    m, n = A.shape
    k = W.shape[1]
    assert W.shape[0] == m
    P = np.empty((k, n))
    _load().oracle_wta_dense(_p(A), m, n, _p(W), k, _p(P))
    return P


def aht_dense(A, H):
    A = _f32(A)
    H = _f64(H)
    m, n = A.shape
    k = H.shape[0]
    assert H.shape[1] == n
    Q = np.empty((m, k))
    _load().oracle_aht_dense(_p(A), m, n, _p(H), k, _p(Q))
    return Q


def _csr(rowptr, colidx, vals):
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    assert rowptr[0] == 0 and rowptr[-1] == colidx.size == vals.size
    return rowptr, colidx, vals


def wta_csr(rowptr, colidx, vals, n, W):
    rowptr, colidx, vals = _csr(rowptr, colidx, vals)
    W = _f64(W)
    m, k = W.shape
    assert rowptr.size == m + 1
    P = np.empty((k, n))
    _load().oracle_wta_csr(_p(rowptr), _p(colidx), _p(vals), m, n, _p(W), k, _p(P))
    return P


def aht_csr(rowptr, colidx, vals, H):
    rowptr, colidx, vals = _csr(rowptr, colidx, vals)
    H = _f64(H)
    k, n = H.shape
    m = rowptr.size - 1
    Q = np.empty((m, k))
    _load().oracle_aht_csr(_p(rowptr), _p(colidx), _p(vals), m, n, _p(H), k, _p(Q))
    return Q


def h_update(H, P, G, eps):
    H = _f64(H)
    k, n = H.shape
    P = _f64(P, (k, n))
    G = _f64(G, (k, k))
    _load().oracle_h_update(_p(H), _p(P), _p(G), k, n, float(eps))
    return H


def w_update(W, Q, G, eps):
    W = _f64(W)
    m, k = W.shape
    Q = _f64(Q, (m, k))
    G = _f64(G, (k, k))
    _load().oracle_w_update(_p(W), _p(Q), _p(G), m, k, float(eps))
    return W


# ---- whole iterations ------------------------------------------------------

def mu_dense(A, W0, H0, iters, eps):
    """`iters` MU iterations (H then W) on dense A; returns (W, H) in double."""
    A = _f32(A)
    m, n = A.shape
    W = _f64(W0)
    H = _f64(H0)
    k = W.shape[1]
    assert W.shape == (m, k) and H.shape == (k, n)
    rc = _load().oracle_mu_dense(_p(A), m, n, k, _p(W), _p(H), int(iters), float(eps))
    if rc != 0:
        raise MemoryError("oracle_mu_dense")
    return W, H


def mu_csr(rowptr, colidx, vals, m, n, W0, H0, iters, eps):
    rowptr, colidx, vals = _csr(rowptr, colidx, vals)
    W = _f64(W0)
    H = _f64(H0)
    k = W.shape[1]
    assert rowptr.size == m + 1 and W.shape == (m, k) and H.shape == (k, n)
    rc = _load().oracle_mu_csr(_p(rowptr), _p(colidx), _p(vals), m, n, k,
                               _p(W), _p(H), int(iters), float(eps))
    if rc != 0:
        raise MemoryError("oracle_mu_csr")
    return W, H


def h_step_dense(A, W, H, eps):
    A = _f32(A)
    m, n = A.shape
    W = _f64(W)
    H = _f64(H)
    _load().oracle_h_step_dense(_p(A), m, n, W.shape[1], _p(W), _p(H), float(eps))
    return W, H


def w_step_dense(A, W, H, eps):
    A = _f32(A)
    m, n = A.shape
    W = _f64(W)
    H = _f64(H)
    _load().oracle_w_step_dense(_p(A), m, n, W.shape[1], _p(W), _p(H), float(eps))
    return W, H


def residual_dense(A, W, H) -> float:
    """||A - W H||_F (paper, section 2.1)."""
    A = _f32(A)
    m, n = A.shape
    W = _f64(W)
    H = _f64(H)
    return float(_load().oracle_residual_dense(_p(A), m, n, W.shape[1], _p(W), _p(H)))


def residual_csr(rowptr, colidx, vals, m, n, W, H) -> float:
    """||A - W H||_F over all m n entries for a CSR matrix without repeated
    (row, column) pairs, without forming W H: the square is
    ||A||^2 - 2 <A H^T, W> + <W^T W, H H^T> (expand the norm of section 2.1 and use
    <A, W H> = trace(A^T W H) = <A H^T, W>, <W H, W H> = trace(H^T W^T W H)
    = <W^T W, H H^T>).  All in double, from the oracle's own products."""
    W = _f64(W)
    H = _f64(H)
    v = np.asarray(vals, dtype=np.float64)
    a2 = float(np.dot(v, v))
    cross = float(np.sum(aht_csr(rowptr, colidx, vals, H) * W))
    gg = float(np.sum(gram_w(W) * gram_h(H)))
    return float(np.sqrt(max(a2 - 2.0 * cross + gg, 0.0)))


def mu_dense_tol(A, W0, H0, max_iters, eps, tol, check_every=1):
    """Algorithm 1's loop: iterate (H then W) until ||A - W H||_F <= tol or
    max_iters iterations have run; the objective is looked at before the first
    iteration and after every `check_every` iterations.  Returns (W, H,
    iterations applied, final objective)."""
    W = _f64(W0)
    H = _f64(H0)
    done = 0
    res = residual_dense(A, W, H)
    while done < max_iters and res > tol:
        chunk = min(check_every, max_iters - done)
        W, H = mu_dense(A, W, H, chunk, eps)
        done += chunk
        res = residual_dense(A, W, H)
    return W, H, done, res


def mu_csr_tol(rowptr, colidx, vals, m, n, W0, H0, max_iters, eps, tol, check_every=1):
    """Algorithm 1's loop on a CSR matrix, as mu_dense_tol: the objective (over all
    m n entries, residual_csr) is looked at before the first iteration and after
    every `check_every` iterations.  Returns (W, H, iterations applied, final objective)."""
    W = _f64(W0)
    H = _f64(H0)
    done = 0
    res = residual_csr(rowptr, colidx, vals, m, n, W, H)
    while done < max_iters and res > tol:
        chunk = min(check_every, max_iters - done)
        W, H = mu_csr(rowptr, colidx, vals, m, n, W, H, chunk, eps)
        done += chunk
        res = residual_csr(rowptr, colidx, vals, m, n, W, H)
    return W, H, done, res


def mu_ensemble(As, W0s, H0s, iters, eps):
    """Independent runs, one after another (NMFk-style ensemble)."""
    return [mu_dense(A, W0, H0, iters, eps) for A, W0, H0 in zip(As, W0s, H0s)]


def rel_fro(X, Xref) -> float:
    """||X - Xref||_F / ||Xref||_F in double; the parity metric."""
    X = np.asarray(X, dtype=np.float64)
    Xref = np.asarray(Xref, dtype=np.float64)
    den = np.linalg.norm(Xref)
    return float(np.linalg.norm(X - Xref) / den) if den > 0 else float(np.linalg.norm(X))


# ---- the same iteration with library matrix products as the steps -----------
#
# Cross-checks of the loop oracle, not replacements for it: the six lines of
# Algorithm 3 taken literally as numpy / scipy.sparse float64 products.  Dense
# A is widened to double one row block at a time (the co-linear row batches of
# Algorithm 5), which only bounds memory: every product is still a plain sum
# over all rows.  (They are slower than the C loops at the shapes of interest:
# thin products are a poor fit for the BLAS.)

def mu_dense_blas(A, W0, H0, iters, eps, row_block=8192):
    """`iters` MU iterations (H then W) with float64 library matmuls."""
    m, n = A.shape
    W = _f64(W0)
    H = _f64(H0)
    eps = float(eps)
    for _ in range(int(iters)):
        WTW = W.T @ W
        WTA = np.zeros((W.shape[1], n))
        for i0 in range(0, m, row_block):
            Ab = np.asarray(A[i0:i0 + row_block], dtype=np.float64)
            WTA += W[i0:i0 + row_block].T @ Ab
        H = H * WTA / (WTW @ H + eps)
        HHT = H @ H.T
        for i0 in range(0, m, row_block):
            Ab = np.asarray(A[i0:i0 + row_block], dtype=np.float64)
            Wb = W[i0:i0 + row_block]
            W[i0:i0 + row_block] = Wb * (Ab @ H.T) / (Wb @ HHT + eps)
    return W, H


def mu_csr_scipy(rowptr, colidx, vals, m, n, W0, H0, iters, eps):
    """The CSR iteration with scipy.sparse float64 products (repeated entries
    of the CSR arrays add up, as in the loop oracle)."""
    import scipy.sparse as sp
    A = sp.csr_matrix((np.asarray(vals, dtype=np.float64), np.asarray(colidx), np.asarray(rowptr)),
                      shape=(m, n))
    At = A.T.tocsr()
    W = _f64(W0)
    H = _f64(H0)
    eps = float(eps)
    for _ in range(int(iters)):
        WTW = W.T @ W
        WTA = np.ascontiguousarray((At @ W).T)
        H = H * WTA / (WTW @ H + eps)
        HHT = H @ H.T
        AHT = A @ np.ascontiguousarray(H.T)
        W = W * AHT / (W @ HHT + eps)
    return W, H
