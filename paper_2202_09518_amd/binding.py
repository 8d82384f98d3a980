"""Thin ctypes binding of libnmfmu.so: argument marshalling only.

Every function has the name and argument order of its C entry point in
``include/nmfmu.h``; tensors are torch tensors whose ``data_ptr()`` is handed
over.  Nothing is computed here and there is no fallback: if the HIP library
has not been built, importing the symbols raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnmfmu.so")

EXPORTS = [
    "nmf_status_string", "nmf_last_error",
    "nmf_mu_dense", "nmf_mu_dense_noalloc", "nmf_mu_dense_profile", "nmf_residual_dense", "nmf_mu_dense_tol", "nmf_mu_dense_monitor", "nmf_mu_csr", "nmf_mu_csr_monitor", "nmf_mu_csr_tol", "nmf_mu_ooc", "nmf_mu_ooc_monitor", "nmf_mu_ooc_hostw", "nmf_mu_csr_ooc", "nmf_mu_dense_batched",
    "nmf_mu_workspace_bytes", "nmf_mu_set_workspace", "nmf_mu_release",
    "nmf_csr_partition", "nmf_split_planes", "nmf_csr_to_csc", "nmf_gram_w", "nmf_wta_dense", "nmf_h_update", "nmf_aht_w_update_dense",
]

NMF_OK, NMF_EINVAL, NMF_ENOMEM, NMF_EHIP, NMF_EUNSUPPORTED = range(5)
NMF_MU_MAX_K = 64
NMF_MU_MAX_K_SLICED = 1024

_lib = None


class NmfError(RuntimeError):
    def __init__(self, status: int, name: str, detail: str):
        super().__init__(f"{name}: {detail}" if detail else name)
        self.status = status


def lib() -> ctypes.CDLL:
    """Load libnmfmu.so (built by ``paper_2202_09518_amd.build``); no fallback."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -m paper_2202_09518_amd.build); "
            "there is no CPU or PyTorch fallback")
    L = ctypes.CDLL(LIB_PATH)
    vp, i64, i32, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_float
    L.nmf_status_string.restype = ctypes.c_char_p
    L.nmf_status_string.argtypes = [ctypes.c_int]
    L.nmf_last_error.restype = ctypes.c_char_p
    L.nmf_mu_dense.argtypes = [vp, i64, i64, i32, vp, vp, i32, f32, vp]
    L.nmf_mu_dense_noalloc.argtypes = [vp, i64, i64, i32, vp, vp, i32, f32, vp]
    L.nmf_mu_dense_profile.argtypes = [vp, i64, i64, i32, vp, vp, i32, f32, vp, vp]
    L.nmf_residual_dense.argtypes = [vp, i64, i64, i32, vp, vp, vp, vp]
    L.nmf_mu_dense_tol.argtypes = [vp, i64, i64, i32, vp, vp, i32, f32, ctypes.c_double, i32, vp, vp, vp]
    L.nmf_mu_csr.argtypes = [vp, vp, vp, i64, i64, i64, i32, vp, vp, i32, f32, vp]
    L.nmf_mu_csr_monitor.argtypes = [vp, vp, vp, i64, i64, i64, i32, vp, vp, i32, f32, vp, vp]
    L.nmf_mu_csr_tol.argtypes = [vp, vp, vp, i64, i64, i64, i32, vp, vp, i32, f32, ctypes.c_double, i32, vp, vp, vp]
    L.nmf_mu_ooc.argtypes = [vp, i64, i64, i32, vp, vp, i32, f32, i64, i64, vp]
    L.nmf_mu_ooc_monitor.argtypes = [vp, i64, i64, i32, vp, vp, i32, f32, i64, i64, vp, vp]
    L.nmf_mu_dense_monitor.argtypes = [vp, i64, i64, i32, vp, vp, i32, f32, vp, vp]
    L.nmf_mu_csr_ooc.argtypes = [vp, vp, vp, i64, i64, i64, i32, vp, vp, i32, f32, i64, i64, vp]
    L.nmf_mu_ooc_hostw.argtypes = [vp, vp, i64, i64, i32, vp, i32, f32, i64, i32, vp, vp]
    L.nmf_mu_dense_batched.argtypes = [i32, vp, i64, i64, vp, vp, vp, i32, f32, vp]
    L.nmf_mu_workspace_bytes.restype = ctypes.c_size_t
    L.nmf_mu_workspace_bytes.argtypes = [ctypes.c_int, i64, i64, i64, i32, i64]
    L.nmf_mu_set_workspace.argtypes = [vp, ctypes.c_size_t]
    L.nmf_mu_release.argtypes = []
    L.nmf_csr_partition.argtypes = [vp, i64, i32, vp, vp]
    L.nmf_split_planes.argtypes = [vp, i64, i32, vp, vp]
    L.nmf_csr_to_csc.argtypes = [vp, vp, vp, i64, i64, i64, vp, vp, vp, vp]
    L.nmf_gram_w.argtypes = [vp, i64, i32, vp, vp]
    L.nmf_wta_dense.argtypes = [vp, i64, i64, i32, vp, vp, vp]
    L.nmf_h_update.argtypes = [vp, vp, vp, i32, i64, f32, vp, vp]
    L.nmf_aht_w_update_dense.argtypes = [vp, i64, i64, i32, vp, vp, vp, f32, vp]
    for name in EXPORTS:
        fn = getattr(L, name)
        if fn.restype is ctypes.c_int and name not in ("nmf_status_string", "nmf_last_error"):
            fn.restype = ctypes.c_int
    _lib = L
    return L


def _check(status: int) -> None:
    if status != NMF_OK:
        L = lib()
        raise NmfError(status, L.nmf_status_string(status).decode(), L.nmf_last_error().decode())


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream
    return int(stream)


def _dev(t: torch.Tensor, dtype, what: str) -> int:
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise ValueError(f"{what}: need a contiguous {dtype} device tensor")
    return t.data_ptr()


def nmf_status_string(status: int) -> str:
    return lib().nmf_status_string(int(status)).decode()


def nmf_last_error() -> str:
    return lib().nmf_last_error().decode()


def nmf_mu_dense(A, m, n, k, W, H, iters, eps, stream=None) -> None:
    _check(lib().nmf_mu_dense(_dev(A, torch.float32, "A"), m, n, k, _dev(W, torch.float32, "W"),
                              _dev(H, torch.float32, "H"), iters, eps, _stream(stream)))


def nmf_mu_dense_noalloc(A, m, n, k, W, H, iters, eps, stream=None) -> None:
    _check(lib().nmf_mu_dense_noalloc(_dev(A, torch.float32, "A"), m, n, k, _dev(W, torch.float32, "W"),
                                      _dev(H, torch.float32, "H"), iters, eps, _stream(stream)))


def nmf_mu_dense_profile(A, m, n, k, W, H, iters, eps, stream=None):
    """Returns [six average kernel times in ms (launch order of one iteration), mirrored flag,
    ms per launch of the pass over A and of the pass over A^T launched back to back]."""
    ms = (ctypes.c_float * 9)()
    _check(lib().nmf_mu_dense_profile(_dev(A, torch.float32, "A"), m, n, k, _dev(W, torch.float32, "W"),
                                      _dev(H, torch.float32, "H"), iters, eps, _stream(stream), ms))
    return list(ms)


def nmf_residual_dense(A, m, n, k, W, H, stream=None) -> float:
    """||A - W H||_F (blocking)."""
    out = ctypes.c_double()
    _check(lib().nmf_residual_dense(_dev(A, torch.float32, "A"), m, n, k, _dev(W, torch.float32, "W"),
                                    _dev(H, torch.float32, "H"), ctypes.byref(out), _stream(stream)))
    return out.value


def nmf_mu_dense_tol(A, m, n, k, W, H, max_iters, eps, tol, check_every, stream=None):
    """Returns (iterations applied, ||A - W H||_F of the returned factors); blocking."""
    done = ctypes.c_int32()
    res = ctypes.c_double()
    _check(lib().nmf_mu_dense_tol(_dev(A, torch.float32, "A"), m, n, k, _dev(W, torch.float32, "W"),
                                  _dev(H, torch.float32, "H"), max_iters, eps, tol, check_every,
                                  ctypes.byref(done), ctypes.byref(res), _stream(stream)))
    return done.value, res.value


def nmf_mu_csr(rowptr, colidx, vals, m, n, nnz, k, W, H, iters, eps, stream=None) -> None:
    _check(lib().nmf_mu_csr(_dev(rowptr, torch.int64, "rowptr"), _dev(colidx, torch.int32, "colidx"),
                            _dev(vals, torch.float32, "vals"), m, n, nnz, k,
                            _dev(W, torch.float32, "W"), _dev(H, torch.float32, "H"),
                            iters, eps, _stream(stream)))


def nmf_mu_ooc_monitor(A_host, m, n, k, W, H, iters, eps, batch_rows, device_budget_bytes, stream=None):
    """nmf_mu_ooc that also returns the objective after each iteration (list of floats, blocking)."""
    if A_host.is_cuda or A_host.dtype != torch.float32 or not A_host.is_contiguous():
        raise ValueError("A_host: need a contiguous float32 host tensor (pinned for overlap)")
    out = (ctypes.c_double * max(iters, 1))()
    _check(lib().nmf_mu_ooc_monitor(A_host.data_ptr(), m, n, k, _dev(W, torch.float32, "W"),
                                    _dev(H, torch.float32, "H"), iters, eps, batch_rows,
                                    device_budget_bytes, out, _stream(stream)))
    return list(out)[:iters]


def nmf_mu_csr_monitor(rowptr, colidx, vals, m, n, nnz, k, W, H, iters, eps, stream=None):
    """Runs `iters` iterations on a CSR matrix; returns the objective after each (list of floats, blocking)."""
    out = (ctypes.c_double * max(iters, 1))()
    _check(lib().nmf_mu_csr_monitor(_dev(rowptr, torch.int64, "rowptr"), _dev(colidx, torch.int32, "colidx"),
                                    _dev(vals, torch.float32, "vals"), m, n, nnz, k,
                                    _dev(W, torch.float32, "W"), _dev(H, torch.float32, "H"),
                                    iters, eps, out, _stream(stream)))
    return list(out)[:iters]


def nmf_mu_csr_tol(rowptr, colidx, vals, m, n, nnz, k, W, H, max_iters, eps, tol, check_every=1, stream=None):
    """Algorithm 1's loop on a CSR matrix; returns (iterations applied, final objective).  Blocking."""
    done = ctypes.c_int32(0)
    res = ctypes.c_double(0.0)
    _check(lib().nmf_mu_csr_tol(_dev(rowptr, torch.int64, "rowptr"), _dev(colidx, torch.int32, "colidx"),
                                _dev(vals, torch.float32, "vals"), m, n, nnz, k,
                                _dev(W, torch.float32, "W"), _dev(H, torch.float32, "H"),
                                max_iters, eps, tol, check_every, ctypes.byref(done), ctypes.byref(res),
                                _stream(stream)))
    return done.value, res.value


def nmf_mu_ooc(A_host, m, n, k, W, H, iters, eps, batch_rows, device_budget_bytes, stream=None) -> None:
    if A_host.is_cuda or A_host.dtype != torch.float32 or not A_host.is_contiguous():
        raise ValueError("A_host: need a contiguous float32 host tensor (pinned for overlap)")
    _check(lib().nmf_mu_ooc(A_host.data_ptr(), m, n, k, _dev(W, torch.float32, "W"),
                            _dev(H, torch.float32, "H"), iters, eps, batch_rows,
                            device_budget_bytes, _stream(stream)))


def nmf_mu_ooc_hostw(A_host, W_host, m, n, k, H, iters, eps, batch_rows, slots, stream=None) -> int:
    """W_host is updated in place (valid after the stream is synchronised).  Returns the
    device bytes the call used (workspace + staging)."""
    for t, what in ((A_host, "A_host"), (W_host, "W_host")):
        if t.is_cuda or t.dtype != torch.float32 or not t.is_contiguous():
            raise ValueError(f"{what}: need a contiguous float32 host tensor (pinned for overlap)")
    used = ctypes.c_size_t(0)
    _check(lib().nmf_mu_ooc_hostw(A_host.data_ptr(), W_host.data_ptr(), m, n, k, _dev(H, torch.float32, "H"),
                                  iters, eps, batch_rows, slots, _stream(stream), ctypes.byref(used)))
    return int(used.value)


def nmf_mu_dense_monitor(A, m, n, k, W, H, iters, eps, stream=None):
    """Runs `iters` iterations; returns the objective after each (list of floats, blocking)."""
    out = (ctypes.c_double * max(iters, 1))()
    _check(lib().nmf_mu_dense_monitor(_dev(A, torch.float32, "A"), m, n, k, _dev(W, torch.float32, "W"),
                                      _dev(H, torch.float32, "H"), iters, eps, out, _stream(stream)))
    return list(out)[:iters]


def nmf_mu_csr_ooc(rowptr, colidx, vals, m, n, nnz, k, W, H, iters, eps, batch_nnz, device_budget_bytes,
                   stream=None) -> None:
    """rowptr (int64), colidx (int32), vals (float32): contiguous HOST tensors (pinned for overlap)."""
    for t, dt, what in ((rowptr, torch.int64, "rowptr"), (colidx, torch.int32, "colidx"), (vals, torch.float32, "vals")):
        if t.is_cuda or t.dtype != dt or not t.is_contiguous():
            raise ValueError(f"{what}: need a contiguous {dt} host tensor")
    _check(lib().nmf_mu_csr_ooc(rowptr.data_ptr(), colidx.data_ptr(), vals.data_ptr(), m, n, nnz, k,
                                _dev(W, torch.float32, "W"), _dev(H, torch.float32, "H"), iters, eps,
                                batch_nnz, device_budget_bytes, _stream(stream)))


def nmf_mu_dense_batched(n_runs, A, m, n, k, W, H, iters, eps, stream=None) -> None:
    """A, W, H: sequences of device tensors (A entries may repeat); k: sequence of ranks."""
    PtrArr = ctypes.c_void_p * n_runs
    a = PtrArr(*[_dev(t, torch.float32, "A[r]") for t in A])
    w = PtrArr(*[_dev(t, torch.float32, "W[r]") for t in W])
    h = PtrArr(*[_dev(t, torch.float32, "H[r]") for t in H])
    ks = (ctypes.c_int32 * n_runs)(*[int(x) for x in k])
    _check(lib().nmf_mu_dense_batched(n_runs, a, m, n, ks, w, h, iters, eps, _stream(stream)))


def nmf_mu_workspace_bytes(kind, m, n, nnz, k, batch_rows) -> int:
    return int(lib().nmf_mu_workspace_bytes(kind, m, n, nnz, k, batch_rows))


def nmf_mu_set_workspace(buf, nbytes=None) -> None:
    if buf is None:
        _check(lib().nmf_mu_set_workspace(None, 0))
    else:
        _check(lib().nmf_mu_set_workspace(buf.data_ptr(), buf.numel() * buf.element_size() if nbytes is None else nbytes))


def nmf_mu_release() -> None:
    _check(lib().nmf_mu_release())


def nmf_csr_partition(rowptr, m, nparts, part, stream=None) -> None:
    _check(lib().nmf_csr_partition(_dev(rowptr, torch.int64, "rowptr"), m, nparts,
                                   _dev(part, torch.int64, "part"), _stream(stream)))


def nmf_split_planes(X, rows, k, planes, stream=None) -> None:
    """planes: int16 device tensor of ceil(rows / 8) * 24 * KP elements (bf16 bit patterns),
    KP = 32 for k <= 32, else 64."""
    _check(lib().nmf_split_planes(_dev(X, torch.float32, "X"), rows, k, _dev(planes, torch.int16, "planes"),
                                  _stream(stream)))


def nmf_csr_to_csc(rowptr, colidx, vals, m, n, nnz, colptr, rowidx, cvals, stream=None) -> None:
    _check(lib().nmf_csr_to_csc(_dev(rowptr, torch.int64, "rowptr"), _dev(colidx, torch.int32, "colidx"),
                                _dev(vals, torch.float32, "vals"), m, n, nnz,
                                _dev(colptr, torch.int64, "colptr"), _dev(rowidx, torch.int32, "rowidx"),
                                _dev(cvals, torch.float32, "cvals"), _stream(stream)))


def nmf_gram_w(W, m, k, G, stream=None) -> None:
    _check(lib().nmf_gram_w(_dev(W, torch.float32, "W"), m, k, _dev(G, torch.float32, "G"), _stream(stream)))


def nmf_wta_dense(A, m, n, k, W, P, stream=None) -> None:
    _check(lib().nmf_wta_dense(_dev(A, torch.float32, "A"), m, n, k, _dev(W, torch.float32, "W"),
                               _dev(P, torch.float32, "P"), _stream(stream)))


def nmf_h_update(H, P, G, k, n, eps, GH=None, stream=None) -> None:
    _check(lib().nmf_h_update(_dev(H, torch.float32, "H"), _dev(P, torch.float32, "P"),
                              _dev(G, torch.float32, "G"), k, n, eps,
                              None if GH is None else _dev(GH, torch.float32, "GH"), _stream(stream)))


def nmf_aht_w_update_dense(A, m, n, k, H, GH, W, eps, stream=None) -> None:
    _check(lib().nmf_aht_w_update_dense(_dev(A, torch.float32, "A"), m, n, k,
                                        _dev(H, torch.float32, "H"), _dev(GH, torch.float32, "GH"),
                                        _dev(W, torch.float32, "W"), eps, _stream(stream)))
