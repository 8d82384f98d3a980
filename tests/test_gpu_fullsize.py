"""Parity at the full sizes of the benchmark configurations, through the same
entry points and launch configurations that bench.py times.

Whole results are compared, also for the 64 GiB out-of-memory configuration
(two oracle products over the matrix, about a minute each), together with the
objective that the monitored entry points report.
"""
import sys

import numpy as np
import pytest
import torch

import nmf_inputs
import paper_2202_09518_amd as nmf
from oracle import nmf_oracle as orc

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]

EPS = 1e-16
EPSD = float(np.float32(EPS))


@pytest.fixture(autouse=True)
def release_memory_between_tests():
    """The cases here hold tens of GiB of pinned host and device memory each: give the library's
    workspace and torch's cached blocks (device and pinned host) back after every test."""
    yield
    import gc
    gc.collect()
    torch.cuda.synchronize()
    nmf.nmf_mu_release()
    torch.cuda.empty_cache()
    if hasattr(torch._C, "_host_emptyCache"):
        torch._C._host_emptyCache()


def say(msg):
    print(msg, file=sys.stderr, flush=True)


def errs(Wd, Hd, Wr, Hr):
    torch.cuda.synchronize()
    return orc.rel_fro(Wd.cpu().numpy(), Wr), orc.rel_fro(Hd.cpu().numpy(), Hr)


def test_config2_full_size_1_and_100_iterations():
    m, n, k = 32768, 16384, 32
    A = nmf_inputs.dense_planted(m, n, 32, seed=1002, device="cuda")
    W, H = nmf_inputs.init_factors(m, n, k, seed=2002, device="cuda")
    Ah, W0, H0 = A.cpu().numpy(), W.cpu().numpy(), H.cpu().numpy()
    W1, H1 = W.clone(), H.clone()
    nmf.nmf_mu_dense(A, m, n, k, W1, H1, 1, EPS)
    Wr, Hr = orc.mu_dense(Ah, W0, H0, 1, EPSD)
    ew, eh = errs(W1, H1, Wr, Hr)
    say(f"config 2 full size, 1 iteration: rel err W {ew:.2e} H {eh:.2e}")
    assert max(ew, eh) < 1e-5
    nmf.nmf_mu_dense(A, m, n, k, W, H, 100, EPS)
    Wr, Hr = orc.mu_dense(Ah, W0, H0, 100, EPSD)
    ew, eh = errs(W, H, Wr, Hr)
    say(f"config 2 full size, 100 iterations: rel err W {ew:.2e} H {eh:.2e}")
    assert max(ew, eh) < 1e-3
    assert bool((W >= 0).all()) and bool((H >= 0).all())


def test_config2_size_misaligned_and_64_factors_without_a_transposed_copy():
    """The two plans that stand in for the row plan of config 2 at its size: an A whose rows are
    16382 floats long at an odd float offset (copied once into an aligned, zero-padded array), and
    64 factors with a workspace that has no room for a transposed copy (the row kernel with two
    32-factor tiles).  Two iterations each."""
    m, n, k = 32768, 16382, 32
    base = nmf_inputs.dense_planted(m, 16384, 32, seed=1002, device="cuda")
    buf = torch.empty(m * n + 8, dtype=torch.float32, device="cuda")
    A = buf[1:1 + m * n].view(m, n)
    A.copy_(base[:, :n])
    del base
    W, H = nmf_inputs.init_factors(m, n, k, seed=2002, device="cuda")
    Ah, W0, H0 = A.cpu().numpy(), W.cpu().numpy(), H.cpu().numpy()
    nmf.nmf_mu_dense(A, m, n, k, W, H, 2, EPS)
    Wr, Hr = orc.mu_dense(Ah, W0, H0, 2, EPSD)
    ew, eh = errs(W, H, Wr, Hr)
    say(f"32768 x 16382 at a 4-byte offset, 2 iterations: rel err W {ew:.2e} H {eh:.2e}")
    assert max(ew, eh) < 2e-5
    del A, buf, W, H
    m, n, k = 32768, 16384, 64
    A = nmf_inputs.dense_planted(m, n, 32, seed=1002, device="cuda")
    W, H = nmf_inputs.init_factors(m, n, k, seed=2012, device="cuda")
    Ah, W0, H0 = A.cpu().numpy(), W.cpu().numpy(), H.cpu().numpy()
    ws = torch.empty(nmf.nmf_mu_workspace_bytes(4, m, n, 0, k, 0), dtype=torch.uint8, device="cuda")
    nmf.nmf_mu_set_workspace(ws)
    try:
        nmf.nmf_mu_dense(A, m, n, k, W, H, 2, EPS)
        torch.cuda.synchronize()
    finally:
        nmf.nmf_mu_set_workspace(None)
    Wr, Hr = orc.mu_dense(Ah, W0, H0, 2, EPSD)
    ew, eh = errs(W, H, Wr, Hr)
    say(f"32768 x 16384, k = 64 on the row kernel, 2 iterations: rel err W {ew:.2e} H {eh:.2e}")
    assert max(ew, eh) < 2e-5


def test_streamed_batches_of_32768_rows_k32():
    """Streamed dense run whose batches take the row kernel with four row tiles per wave (128-row
    blocks: 24576 rows or more per batch), last batch ragged; with the objective of every iteration."""
    m, n, k, batch = 90000, 2048, 32, 32768
    A = nmf_inputs.dense_planted(m, n, 32, seed=1004)
    W, H = nmf_inputs.init_factors(m, n, k, seed=2004, device="cuda")
    W0, H0 = W.cpu().numpy(), H.cpu().numpy()
    Ap = A.pin_memory()
    obj = nmf.nmf_mu_ooc_monitor(Ap, m, n, k, W, H, 3, EPS, batch, 3 * batch * n * 4 + 4096)
    Ah = A.numpy()
    Wr, Hr = orc.mu_dense(Ah, W0, H0, 3, EPSD)
    ew, eh = errs(W, H, Wr, Hr)
    want = orc.residual_dense(Ah, Wr, Hr)
    say(f"streamed 90000 x 2048, k = 32, batches of 32768 rows, 3 iterations: rel err W {ew:.2e} H {eh:.2e}; "
        f"objective {obj[-1]:.6e} against {want:.6e}")
    assert max(ew, eh) < 3e-5
    assert abs(obj[-1] - want) < 1e-3 * float(np.linalg.norm(Ah.astype(np.float64)))


def test_config3_full_size_one_iteration():
    m, n, k = 4194304, 1048576, 32
    rowptr, colidx, vals = nmf_inputs.csr_uniform(m, n, 1e-4, seed=1003, device="cuda")
    nnz = int(vals.numel())
    W, H = nmf_inputs.init_factors(m, n, k, seed=2003, device="cuda")
    rp0, ci0, va0 = rowptr.clone(), colidx.clone(), vals.clone()
    W0, H0 = W.cpu().numpy(), H.cpu().numpy()
    obj = nmf.nmf_mu_csr_monitor(rowptr, colidx, vals, m, n, nnz, k, W, H, 1, EPS)[0]   # W, H as nmf_mu_csr gives them
    torch.cuda.synchronize()
    assert torch.equal(rowptr, rp0) and torch.equal(colidx, ci0) and torch.equal(vals, va0)
    del rp0, ci0, va0
    say(f"config 3: nnz = {nnz}; running the oracle (about a minute)")
    rph, cih, vah = rowptr.cpu().numpy(), colidx.cpu().numpy(), vals.cpu().numpy()
    Wr, Hr = orc.mu_csr(rph, cih, vah, m, n, W0, H0, 1, EPSD)
    ew, eh = errs(W, H, Wr, Hr)
    want = orc.residual_csr(rph, cih, vah, m, n, Wr, Hr)
    say(f"config 3 full size, 1 iteration: rel err W {ew:.2e} H {eh:.2e}; objective {obj:.8g} against {want:.8g}")
    assert max(ew, eh) < 1e-5
    assert abs(obj - want) <= 1e-5 * want
    del rph, cih, vah
    # the same matrix streamed from pinned host memory in batches of 32 Mi stored entries
    # (the launch configuration of bench.py --workload c3ooc), against the same oracle result
    rp, ci, va = rowptr.cpu().pin_memory(), colidx.cpu().pin_memory(), vals.cpu().pin_memory()
    del rowptr, colidx, vals
    W2, H2 = torch.from_numpy(W0).cuda(), torch.from_numpy(H0).cuda()
    nmf.nmf_mu_csr_ooc(rp, ci, va, m, n, nnz, k, W2, H2, 1, EPS, 32 << 20, 2 << 30)
    ew, eh = errs(W2, H2, Wr, Hr)
    say(f"config 3 full size streamed from host memory, 1 iteration: rel err W {ew:.2e} H {eh:.2e}")
    assert max(ew, eh) < 1e-5


def test_config4_full_size_one_iteration_with_objective():
    m, n, k, batch = 262144, 65536, 64, 8192
    Ah = torch.empty((m, n), dtype=torch.float32, pin_memory=True)
    nmf_inputs.dense_planted(m, n, 64, seed=1004, device="cuda", out=Ah, row_block=batch)
    torch.cuda.synchronize()
    W, H = nmf_inputs.init_factors(m, n, k, seed=2004, device="cuda")
    W0, H0 = W.cpu().numpy(), H.cpu().numpy()
    obj = nmf.nmf_mu_ooc_monitor(Ah, m, n, k, W, H, 1, EPS, batch, 8 << 30)[0]     # W, H as nmf_mu_ooc gives them
    torch.cuda.synchronize()
    nmf.nmf_mu_release()          # give the 6 GiB of staging back
    An = Ah.numpy()
    say("config 4: oracle W^T A and A H^T over 64 GiB (about a minute each)")
    Hr = orc.h_update(H0, orc.wta_dense(An, W0), orc.gram_w(W0), EPSD)
    eh = orc.rel_fro(H.cpu().numpy(), Hr)
    Q = orc.aht_dense(An, Hr)
    Wr = orc.w_update(W0, Q, orc.gram_h(Hr), EPSD)
    ew = orc.rel_fro(W.cpu().numpy(), Wr)
    # objective of the oracle's factors from its own products (the definition would be a third pass with
    # m n k multiplications): ||A||^2 - 2 <A H^T, W> + <W^T W, H H^T>, the identity test_oracle_pins holds
    # against the definition for the sparse oracle
    a2 = 0.0
    for i0 in range(0, m, batch):
        blk = An[i0:i0 + batch].astype(np.float64)
        a2 += float(np.vdot(blk, blk))
    want = float(np.sqrt(a2 - 2.0 * float(np.sum(Q * Wr)) + float(np.sum(orc.gram_w(Wr) * orc.gram_h(Hr)))))
    say(f"config 4 full size, 1 iteration: rel err H {eh:.2e}, W {ew:.2e}; objective {obj:.8g} against {want:.8g}")
    assert max(ew, eh) < 1e-5
    assert abs(obj - want) <= 1e-5 * want + 3e-7 * a2 / want
    assert bool(torch.isfinite(W).all()) and bool((W >= 0).all())


@pytest.mark.parametrize("k", [2, 16])
def test_config5_shape_one_copy_1_and_100_iterations(k):
    m, n = 16384, 8192
    base = nmf_inputs.dense_planted(m, n, 8, seed=1005, device="cuda")
    A = nmf_inputs.perturb(base, 3000)
    W, H = nmf_inputs.init_factors(m, n, k, seed=2005 + k, device="cuda")
    Ah, W0, H0 = A.cpu().numpy(), W.cpu().numpy(), H.cpu().numpy()
    for iters in (1, 100):
        Wd, Hd = W.clone(), H.clone()
        nmf.nmf_mu_dense_batched(1, [A], m, n, [k], [Wd], [Hd], iters, EPS)
        Wr, Hr = orc.mu_dense(Ah, W0, H0, iters, EPSD)
        ew, eh = errs(Wd, Hd, Wr, Hr)
        say(f"config 5 shape, k={k}, {iters} iterations: rel err W {ew:.2e} H {eh:.2e}")
        assert max(ew, eh) < (1e-5 if iters == 1 else 1e-3)


def test_oom1_shape_host_resident_w_rank_128_two_iterations():
    """The paper's out-of-memory benchmark shape (section 4.4): 524288 x 4096 in 32 batches, A and W
    in pinned host memory, through the entry point and slot count bench.py --workload oom1 times."""
    m, n, k, nbatch = 524288, 4096, 128, 32
    batch = m // nbatch
    Ah = torch.empty((m, n), dtype=torch.float32, pin_memory=True)
    nmf_inputs.dense_planted(m, n, 32, seed=1006, device="cuda", out=Ah, row_block=batch)
    W, H = nmf_inputs.init_factors(m, n, k, seed=2006, device="cuda")
    W0, H0 = W.cpu().numpy(), H.cpu().numpy()
    Wh = torch.empty((m, k), dtype=torch.float32, pin_memory=True)
    Wh.copy_(W)
    del W
    torch.cuda.synchronize()
    nmf.nmf_mu_ooc_hostw(Ah, Wh, m, n, k, H, 2, EPS, batch, 3)
    torch.cuda.synchronize()
    say("oom1 shape: running the oracle (2 iterations, k = 128)")
    Wr, Hr = orc.mu_dense(Ah.numpy(), W0, H0, 2, EPSD)
    ew, eh = orc.rel_fro(Wh.numpy(), Wr), orc.rel_fro(H.cpu().numpy(), Hr)
    say(f"oom1 shape, host-resident W, k = 128, 2 iterations: rel err W {ew:.2e} H {eh:.2e}")
    assert max(ew, eh) < 2e-5


def test_rank_1024_resident_one_iteration():
    """The largest supported rank on a matrix the oracle finishes in well under a minute."""
    m, n, k = 16384, 4096, 1024
    A = nmf_inputs.dense_planted(m, n, 32, seed=1007, device="cuda")
    W, H = nmf_inputs.init_factors(m, n, k, seed=2007, device="cuda")
    Ah, W0, H0 = A.cpu().numpy(), W.cpu().numpy(), H.cpu().numpy()
    nmf.nmf_mu_dense(A, m, n, k, W, H, 1, EPS)
    Wr, Hr = orc.mu_dense(Ah, W0, H0, 1, EPSD)
    ew, eh = errs(W, H, Wr, Hr)
    say(f"rank 1024 resident, 1 iteration: rel err W {ew:.2e} H {eh:.2e}")
    assert max(ew, eh) < 1e-5


def test_config5_one_copy_all_ranks_stacked_one_and_three_iterations():
    """One perturbed copy with its 15 runs (k = 2..16) in one batched call, as bench.py --workload c5
    issues them: the library stacks them 54 + 50 + 31 wide, so the 64-wide and the 32-wide pass
    kernels both run at the full 16384 x 8192 shape.  Every run against its own oracle run."""
    m, n = 16384, 8192
    base = nmf_inputs.dense_planted(m, n, 8, seed=1005, device="cuda")
    A = nmf_inputs.perturb(base, 3000)
    Ah = A.cpu().numpy()
    ks = list(range(2, 17))
    for iters, tol in ((1, 1e-5), (3, 1e-4)):
        Ws, Hs, W0s, H0s = [], [], [], []
        for i, k in enumerate(ks):
            W, H = nmf_inputs.init_factors(m, n, k, seed=2005 + i, device="cuda")
            Ws.append(W); Hs.append(H); W0s.append(W.cpu().numpy()); H0s.append(H.cpu().numpy())
        nmf.nmf_mu_dense_batched(len(ks), [A] * len(ks), m, n, ks, Ws, Hs, iters, EPS)
        torch.cuda.synchronize()
        worst = 0.0
        for i, k in enumerate(ks):
            Wr, Hr = orc.mu_dense(Ah, W0s[i], H0s[i], iters, EPSD)
            worst = max(worst, *errs(Ws[i], Hs[i], Wr, Hr))
        say(f"config 5 shape, 15 stacked runs, {iters} iteration(s): worst rel err {worst:.2e}")
        assert worst < tol


def test_rank_64_resident_config2_matrix_one_iteration():
    m, n, k = 32768, 16384, 64
    A = nmf_inputs.dense_planted(m, n, 32, seed=1002, device="cuda")
    W, H = nmf_inputs.init_factors(m, n, k, seed=2002, device="cuda")
    Ah, W0, H0 = A.cpu().numpy(), W.cpu().numpy(), H.cpu().numpy()
    nmf.nmf_mu_dense(A, m, n, k, W, H, 1, EPS)
    Wr, Hr = orc.mu_dense(Ah, W0, H0, 1, EPSD)
    ew, eh = errs(W, H, Wr, Hr)
    say(f"rank 64 on config 2's matrix, 1 iteration: rel err W {ew:.2e} H {eh:.2e}")
    assert max(ew, eh) < 1e-5


@pytest.mark.parametrize("m,k", [(32, 16), (16, 40)])
def test_more_than_2_to_25_columns(m, k):
    """Past 2^25 columns a 16-row step of A no longer fits a buffer descriptor's 32-bit
    extent: the pass over A takes the kernels with plain 64-bit addressing, the pass over
    the transpose walks 2^25 rows per column slab, and the factor update sees 2^25 columns."""
    n = (1 << 25) + 64
    A = nmf_inputs.uniform((m, n), 1025, device="cuda")
    W, H = nmf_inputs.init_factors(m, n, k, seed=2025, device="cuda")
    Ah, W0, H0 = A.cpu().numpy(), W.cpu().numpy(), H.cpu().numpy()
    P = torch.empty((k, n), device="cuda")
    nmf.nmf_wta_dense(A, m, n, k, W, P)
    ep = orc.rel_fro(P.cpu().numpy(), orc.wta_dense(Ah, W0))
    del P
    got = nmf.nmf_residual_dense(A, m, n, k, W, H)
    want = orc.residual_dense(Ah, W0, H0)
    nmf.nmf_mu_dense(A, m, n, k, W, H, 1, EPS)
    Wr, Hr = orc.mu_dense(Ah, W0, H0, 1, EPSD)
    ew, eh = errs(W, H, Wr, Hr)
    say(f"{m} x 2^25+64, k = {k}: rel err W^T A {ep:.2e}, objective {abs(got - want) / want:.2e}, 1 iteration W {ew:.2e} H {eh:.2e}")
    assert ep < 1e-5 and abs(got - want) <= 1e-5 * want and max(ew, eh) < 1e-5
