"""Parity at each configuration's FINAL iteration count on every path other than the
resident dense one (which tests/test_gpu_fullsize.py and tests/test_gpu_parity.py cover):
the sparse gather, the streamed sparse and dense paths, the host-resident-W pipeline, the
rank-sliced engine and the stacked ensemble, each on the recipe of its benchmark
configuration at a size the float64 oracle finishes in seconds.

Bars, from the target statement: relative Frobenius error max over W and H of 1e-5 after
one iteration and 1e-3 after the final count (50 sparse, 20 streamed, 500 ensemble, 100
otherwise); the objectives of the two results must agree to 1e-3 of ||A||_F as well.
"""
import sys

import numpy as np
import pytest
import torch

import nmf_inputs
import paper_2202_09518_amd as nmf
from oracle import nmf_oracle as orc

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(600)]

EPS = 1e-16
EPSD = float(np.float32(EPS))
TOL1 = 1e-5
TOLN = 1e-3


def say(msg):
    print(msg, file=sys.stderr, flush=True)


def dev(x, dtype=torch.float32):
    return torch.as_tensor(np.ascontiguousarray(x)).to(dtype).cuda().contiguous()


def host(t):
    torch.cuda.synchronize()
    return t.detach().cpu().numpy().astype(np.float64)


def worst(Wg, Hg, Wr, Hr):
    assert np.isfinite(Wg).all() and np.isfinite(Hg).all()
    assert (Wg >= 0).all() and (Hg >= 0).all()
    return max(orc.rel_fro(Wg, Wr), orc.rel_fro(Hg, Hr))


# ---- sparse: the recipe of config 3 (uniform positions, values in (0, 1], k = 32) -------------

def csr_case():
    m, n, k, density = 65536, 16384, 32, 1e-3
    rowptr, colidx, vals = (t.numpy() for t in nmf_inputs.csr_uniform(m, n, density, seed=1003))
    W, H = (t.numpy() for t in nmf_inputs.init_factors(m, n, k, seed=2003))
    return m, n, k, rowptr, colidx, vals, W, H


@pytest.fixture(scope="module")
def csr_oracle():
    """The oracle's factors after 1, 50 and 100 iterations (one run, continued)."""
    m, n, k, rowptr, colidx, vals, W, H = csr_case()
    out = {}
    Wr, Hr = orc.mu_csr(rowptr, colidx, vals, m, n, W, H, 1, EPSD)
    out[1] = (Wr, Hr)
    Wr, Hr = orc.mu_csr(rowptr, colidx, vals, m, n, Wr, Hr, 49, EPSD)
    out[50] = (Wr, Hr)
    Wr, Hr = orc.mu_csr(rowptr, colidx, vals, m, n, Wr, Hr, 50, EPSD)
    out[100] = (Wr, Hr)
    return out


def csr_objective_gap(rowptr, colidx, vals, m, n, Wg, Hg, Wr, Hr):
    norm_a = float(np.sqrt(np.sum(vals.astype(np.float64) ** 2)))
    fg = orc.residual_csr(rowptr, colidx, vals, m, n, Wg, Hg)
    fr = orc.residual_csr(rowptr, colidx, vals, m, n, Wr, Hr)
    return abs(fg - fr) / norm_a


@pytest.mark.parametrize("iters", [1, 50, 100])
def test_csr_resident_at_the_final_iteration_counts(csr_oracle, iters):
    m, n, k, rowptr, colidx, vals, W, H = csr_case()
    Wd, Hd = dev(W), dev(H)
    nmf.nmf_mu_csr(dev(rowptr, torch.int64), dev(colidx, torch.int32), dev(vals), m, n, int(vals.size), k,
                   Wd, Hd, iters, EPS)
    Wg, Hg = host(Wd), host(Hd)
    Wr, Hr = csr_oracle[iters]
    e = worst(Wg, Hg, Wr, Hr)
    gap = csr_objective_gap(rowptr, colidx, vals, m, n, Wg, Hg, Wr, Hr)
    say(f"csr resident {m}x{n} nnz={vals.size} k={k}, {iters} iterations: rel err {e:.2e}, objective gap {gap:.2e}")
    assert e < (TOL1 if iters == 1 else TOLN)
    assert gap < TOLN


@pytest.mark.parametrize("iters", [1, 50])
def test_csr_streamed_at_the_final_iteration_count(csr_oracle, iters):
    m, n, k, rowptr, colidx, vals, W, H = csr_case()
    rp = torch.from_numpy(rowptr).pin_memory()
    ci = torch.from_numpy(colidx).pin_memory()
    va = torch.from_numpy(vals).pin_memory()
    Wd, Hd = dev(W), dev(H)
    batch_nnz = 150001                      # 8 ragged batches of whole rows
    nmf.nmf_mu_csr_ooc(rp, ci, va, m, n, int(vals.size), k, Wd, Hd, iters, EPS, batch_nnz, 1 << 30)
    Wg, Hg = host(Wd), host(Hd)
    Wr, Hr = csr_oracle[iters]
    e = worst(Wg, Hg, Wr, Hr)
    gap = csr_objective_gap(rowptr, colidx, vals, m, n, Wg, Hg, Wr, Hr)
    say(f"csr streamed, {iters} iterations: rel err {e:.2e}, objective gap {gap:.2e}")
    assert e < (TOL1 if iters == 1 else TOLN)
    assert gap < TOLN


# ---- streamed dense: the recipe of config 4 (planted rank 64, k = 64, 8 ragged batches) --------

def ooc_case(k):
    m, n, batch = 4000, 2048, 512                   # 7 batches of 512 rows and one of 416
    A = nmf_inputs.dense_planted(m, n, 64, seed=1004).numpy()
    W, H = (t.numpy() for t in nmf_inputs.init_factors(m, n, k, seed=2004))
    return m, n, batch, A, W, H


_ooc_oracle_cache = {}


def ooc_oracle(k, iters):
    """The oracle's factors on ooc_case(k) after `iters` iterations; a longer run continues the
    longest shorter one already computed (the iteration has no memory besides W and H)."""
    m, n, batch, A, W, H = ooc_case(k)
    have = [i for (kk, i) in _ooc_oracle_cache if kk == k and i <= iters]
    done = max(have) if have else 0
    Wr, Hr = _ooc_oracle_cache[(k, done)] if have else (W, H)
    if iters > done:
        Wr, Hr = orc.mu_dense(A, Wr, Hr, iters - done, EPSD)
        _ooc_oracle_cache[(k, iters)] = (Wr, Hr)
    return Wr, Hr


def dense_objective_gap(A, Wg, Hg, Wr, Hr):
    norm_a = float(np.linalg.norm(A.astype(np.float64)))
    return abs(orc.residual_dense(A, Wg, Hg) - orc.residual_dense(A, Wr, Hr)) / norm_a


@pytest.mark.parametrize("iters", [1, 20])
def test_ooc_k64_at_the_final_iteration_count(iters):
    k = 64
    m, n, batch, A, W, H = ooc_case(k)
    Wd, Hd = dev(W), dev(H)
    nmf.nmf_mu_ooc(torch.from_numpy(A).pin_memory(), m, n, k, Wd, Hd, iters, EPS, batch, 3 * batch * n * 4 + 4096)
    Wg, Hg = host(Wd), host(Hd)
    Wr, Hr = ooc_oracle(k, iters)
    e = worst(Wg, Hg, Wr, Hr)
    gap = dense_objective_gap(A, Wg, Hg, Wr, Hr)
    say(f"ooc {m}x{n} k={k} batch {batch}, {iters} iterations: rel err {e:.2e}, objective gap {gap:.2e}")
    assert e < (TOL1 if iters == 1 else TOLN)
    assert gap < TOLN


@pytest.mark.parametrize("k,iters", [(64, 20), (128, 20), (128, 100)])
def test_ooc_hostw_at_the_final_iteration_counts(k, iters):
    """Algorithm 5 with W_b up and down per batch; k = 128 takes two 64-factor slices."""
    m, n, batch, A, W, H = ooc_case(k)
    Ah = torch.from_numpy(A).pin_memory()
    Wh = torch.from_numpy(W.copy()).pin_memory()
    Hd = dev(H)
    nmf.nmf_mu_ooc_hostw(Ah, Wh, m, n, k, Hd, iters, EPS, batch, 3)
    torch.cuda.synchronize()
    Wg, Hg = Wh.numpy().astype(np.float64), host(Hd)
    Wr, Hr = ooc_oracle(k, iters)
    e = worst(Wg, Hg, Wr, Hr)
    gap = dense_objective_gap(A, Wg, Hg, Wr, Hr)
    say(f"ooc hostw k={k}, {iters} iterations: rel err {e:.2e}, objective gap {gap:.2e}")
    assert e < TOLN
    assert gap < TOLN


def test_dense_rank_sliced_100_iterations():
    m, n, k = 1024, 768, 160                       # three slices: 64 + 64 + 32 factors
    A = nmf_inputs.dense_planted(m, n, 32, seed=1002).numpy()
    W, H = (t.numpy() for t in nmf_inputs.init_factors(m, n, k, seed=2002))
    Wd, Hd = dev(W), dev(H)
    nmf.nmf_mu_dense(dev(A), m, n, k, Wd, Hd, 100, EPS)
    Wg, Hg = host(Wd), host(Hd)
    Wr, Hr = orc.mu_dense(A, W, H, 100, EPSD)
    e = worst(Wg, Hg, Wr, Hr)
    gap = dense_objective_gap(A, Wg, Hg, Wr, Hr)
    say(f"dense rank-sliced {m}x{n} k={k}, 100 iterations: rel err {e:.2e}, objective gap {gap:.2e}")
    assert e < TOLN
    assert gap < TOLN


# ---- ensemble: the recipe of config 5 (planted rank 8, one perturbed copy, k = 2 .. 16 stacked) ----

def test_stacked_ensemble_k2_to_16_500_iterations():
    m, n = 1024, 512
    base = nmf_inputs.dense_planted(m, n, 8, seed=1005)
    Ap = nmf_inputs.perturb(base, 3000)
    ks = list(range(2, 17))                         # sum 135: stacks of 54 + 63 + 18 factors... as the library cuts them
    Ws, Hs = [], []
    for r, k in enumerate(ks):
        W, H = nmf_inputs.init_factors(m, n, k, seed=2005 + r)
        Ws.append(W)
        Hs.append(H)
    Ad = Ap.cuda()
    Wd = [w.cuda() for w in Ws]
    Hd = [h.cuda() for h in Hs]
    nmf.nmf_mu_dense_batched(len(ks), [Ad] * len(ks), m, n, ks, Wd, Hd, 500, EPS)
    An = Ap.numpy()
    ref = orc.mu_ensemble([An] * len(ks), [w.numpy() for w in Ws], [h.numpy() for h in Hs], 500, EPSD)
    norm_a = float(np.linalg.norm(An.astype(np.float64)))
    report = []
    for r, k in enumerate(ks):
        Wg, Hg = host(Wd[r]), host(Hd[r])
        Wr, Hr = ref[r]
        e = worst(Wg, Hg, Wr, Hr)
        gap = abs(orc.residual_dense(An, Wg, Hg) - orc.residual_dense(An, Wr, Hr)) / norm_a
        report.append((k, e, gap))
    say("stacked ensemble, 500 iterations: " + ", ".join(f"k={k}: {e:.1e}/{g:.1e}" for k, e, g in report))
    for k, e, gap in report:
        assert e < TOLN, (k, e)
        assert gap < TOLN, (k, gap)
