"""The allocation-free entry point nmf_mu_dense_noalloc against nmf_mu_dense.

Through the C ABI, on two calls in a row, the second with a smaller input (the fixed
scratch array keeps the first call's contents).  Compared bit for bit with nmf_mu_dense
held to the same plan (a caller workspace too small for the transposed copy of A), and to
the parity bar (1e-5 after one iteration, 1e-3 after 100) with nmf_mu_dense as it runs by
default and with the oracle.
"""
import ctypes

import numpy as np
import pytest
import torch

import nmf_inputs
import paper_2202_09518_amd as nmf
from oracle import nmf_oracle as orc

pytestmark = pytest.mark.gpu

EPS = 1e-16


def problem(m, n, k, seed):
    A = nmf_inputs.dense_planted(m, n, min(k, 8), seed=seed, device="cuda")
    W, H = nmf_inputs.init_factors(m, n, k, seed=seed + 1, device="cuda")
    return A, W, H


def run(fn, A, W, H, iters):
    m, n = A.shape
    Wd, Hd = W.clone(), H.clone()
    fn(A, m, n, W.shape[1], Wd, Hd, iters, EPS)
    torch.cuda.synchronize()
    return Wd, Hd


def small_plan_dense(A, W, H, iters):
    """nmf_mu_dense with a caller workspace that only holds the small plan."""
    m, n = A.shape
    k = W.shape[1]
    buf = torch.empty(nmf.nmf_mu_workspace_bytes(4, m, n, 0, k, 0), dtype=torch.uint8, device="cuda")
    nmf.nmf_mu_set_workspace(buf)
    try:
        return run(nmf.nmf_mu_dense, A, W, H, iters)
    finally:
        torch.cuda.synchronize()
        nmf.nmf_mu_set_workspace(None)


def rel(x, ref):
    return orc.rel_fro(x.cpu().numpy(), ref.cpu().numpy() if torch.is_tensor(ref) else ref)


def test_noalloc_two_calls_in_a_row_second_one_smaller():
    big = problem(3000, 2100, 32, 500)        # several row splits and column slabs, ragged edges
    small = problem(257, 131, 17, 510)
    for A, W, H in (big, small):
        for iters in (1, 3):
            got = run(nmf.nmf_mu_dense_noalloc, A, W, H, iters)
            same_plan = small_plan_dense(A, W, H, iters)
            assert torch.equal(got[0], same_plan[0]) and torch.equal(got[1], same_plan[1])
            default = run(nmf.nmf_mu_dense, A, W, H, iters)
            assert max(rel(got[0], default[0]), rel(got[1], default[1])) < 1e-5 * iters
    # against the oracle: one iteration and the final count of the dense configurations
    A, W, H = small
    for iters, tol in ((1, 1e-5), (100, 1e-3)):
        got = run(nmf.nmf_mu_dense_noalloc, A, W, H, iters)
        Wr, Hr = orc.mu_dense(A.cpu().numpy(), W.cpu().numpy(), H.cpu().numpy(), iters, float(np.float32(EPS)))
        assert max(rel(got[0], Wr), rel(got[1], Hr)) < tol


def test_noalloc_k64_then_config1():
    A, W, H = problem(1000, 520, 64, 520)
    got = run(nmf.nmf_mu_dense_noalloc, A, W, H, 2)
    ref = small_plan_dense(A, W, H, 2)
    assert torch.equal(got[0], ref[0]) and torch.equal(got[1], ref[1])
    m, n, k = 256, 192, 4
    A = nmf_inputs.dense_planted(m, n, 4, seed=1001, noise="add", lo=0.0, hi=0.01).cuda()
    W, H = (t.cuda() for t in nmf_inputs.init_factors(m, n, k, seed=2001))
    got = run(nmf.nmf_mu_dense_noalloc, A, W, H, 100)
    Wr, Hr = orc.mu_dense(A.cpu().numpy(), W.cpu().numpy(), H.cpu().numpy(), 100, float(np.float32(EPS)))
    assert max(rel(got[0], Wr), rel(got[1], Hr)) < 1e-3


def test_noalloc_rejects_what_does_not_fit():
    L = nmf.lib()
    one = ctypes.c_void_p(256)
    # 32768 x 16384 at k = 64 needs 53.5 MiB of scratch: beyond the fixed array
    assert nmf.nmf_mu_workspace_bytes(4, 32768, 16384, 0, 64, 0) > 32 << 20
    assert L.nmf_mu_dense_noalloc(one, 32768, 16384, 64, one, one, 1, 1e-16, None) == nmf.NMF_ENOMEM
    assert "scratch" in nmf.nmf_last_error()
    assert L.nmf_mu_dense_noalloc(one, 64, 64, 65, one, one, 1, 1e-16, None) == nmf.NMF_EUNSUPPORTED
    assert L.nmf_mu_dense_noalloc(None, 64, 64, 4, one, one, 1, 1e-16, None) == nmf.NMF_EINVAL
    assert L.nmf_mu_dense_noalloc(one, 64, 64, 4, one, one, 0, 1e-16, None) == nmf.NMF_OK
    # config 2 at k = 32 fits
    assert nmf.nmf_mu_workspace_bytes(4, 32768, 16384, 0, 32, 0) <= 32 << 20
