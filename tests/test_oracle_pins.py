"""Pins for the CPU oracle: facts fixed by the update equations and by
mathematics, none of which is the oracle's own formula retyped.

The paper (Algorithm 3: H update, then W update with the new H; Algorithm 1
for the meaning of eps; section 3.1 for the FLOP model) prints no numeric
example, so the pins are: a hand-worked fixture, exact rational arithmetic,
brute-force loops in a different loop order, closed forms, invariants of the
multiplicative update, and equivalences between the dense and CSR forms.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import nmf_oracle as orc
import nmf_inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
EPS = float(np.float32(1e-16))


def rng(seed):
    return np.random.default_rng(seed)


def small_case(m, n, k, seed, integer=False):
    r = rng(seed)
    if integer:
        A = r.integers(0, 6, size=(m, n)).astype(np.float32)
        W = r.integers(1, 5, size=(m, k)).astype(np.float64)
        H = r.integers(1, 5, size=(k, n)).astype(np.float64)
    else:
        A = r.random((m, n), dtype=np.float32)
        W = r.random((m, k), dtype=np.float32).astype(np.float64)
        H = r.random((k, n), dtype=np.float32).astype(np.float64)
    return A, W, H


# --- hand-worked fixture ---------------------------------------------------

def _read_golden(path):
    out = {}
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, r, c, *vals = line.split()
        out[name] = np.array([float(Fraction(v)) for v in vals]).reshape(int(r), int(c))
    return out


def test_golden_rank1_2x2():
    g = _read_golden(os.path.join(GOLDEN, "mu_rank1_2x2.txt"))
    W, H = orc.mu_dense(g["A"], g["W0"], g["H0"], 1, 0.0)
    np.testing.assert_allclose(H, g["H1"], rtol=1e-15)
    np.testing.assert_allclose(W, g["W1"], rtol=1e-15)


# --- exact rational arithmetic (brute force, tiny) ---------------------------

def _mu_fraction(A, W, H, iters):
    """MU iteration of Algorithm 3 in exact rationals, eps = 0, written with
    explicit index loops (i outermost) so that it shares nothing with the C code."""
    m, n = len(A), len(A[0])
    k = len(H)
    for _ in range(iters):
        P = [[Fraction(0)] * n for _ in range(k)]
        G = [[Fraction(0)] * k for _ in range(k)]
        for i in range(m):
            for c in range(k):
                for j in range(n):
                    P[c][j] += W[i][c] * A[i][j]
                for d in range(k):
                    G[c][d] += W[i][c] * W[i][d]
        Hn = [[None] * n for _ in range(k)]
        for j in range(n):
            for c in range(k):
                den = sum(G[c][d] * H[d][j] for d in range(k))
                Hn[c][j] = H[c][j] * P[c][j] / den
        H = Hn
        G = [[sum(H[c][j] * H[d][j] for j in range(n)) for d in range(k)] for c in range(k)]
        Wn = [[None] * k for _ in range(m)]
        for i in range(m):
            for c in range(k):
                q = sum(A[i][j] * H[c][j] for j in range(n))
                den = sum(W[i][d] * G[d][c] for d in range(k))
                Wn[i][c] = W[i][c] * q / den
        W = Wn
    return W, H


@pytest.mark.parametrize("m,n,k,iters,seed", [(3, 4, 2, 1, 1), (5, 3, 3, 2, 2), (4, 6, 1, 3, 3), (7, 5, 2, 2, 4)])
def test_against_exact_rationals(m, n, k, iters, seed):
    r = rng(seed)
    Ai = r.integers(1, 9, size=(m, n))
    Wi = r.integers(1, 6, size=(m, k))
    Hi = r.integers(1, 6, size=(k, n))
    Wf, Hf = _mu_fraction([[Fraction(int(x)) for x in row] for row in Ai],
                          [[Fraction(int(x)) for x in row] for row in Wi],
                          [[Fraction(int(x)) for x in row] for row in Hi], iters)
    W, H = orc.mu_dense(Ai.astype(np.float32), Wi, Hi, iters, 0.0)
    np.testing.assert_allclose(W, np.array([[float(x) for x in row] for row in Wf]), rtol=1e-13)
    np.testing.assert_allclose(H, np.array([[float(x) for x in row] for row in Hf]), rtol=1e-13)


# --- P1: every product against literal triple loops ---------------------------

@pytest.mark.parametrize("m,n,k,seed", [(8, 7, 3, 11), (1, 5, 2, 12), (6, 1, 1, 13), (5, 9, 4, 14)])
def test_products_brute_force(m, n, k, seed):
    A, W, H = small_case(m, n, k, seed)
    Ad = A.astype(np.float64)
    P = np.zeros((k, n)); Q = np.zeros((m, k)); GW = np.zeros((k, k)); GH = np.zeros((k, k))
    for j in range(n):              # loop order differs from the C code on purpose
        for c in range(k):
            for i in range(m):
                P[c, j] += W[i, c] * Ad[i, j]
    for c in range(k):
        for i in range(m):
            for j in range(n):
                Q[i, c] += Ad[i, j] * H[c, j]
    for i in range(m):
        for a in range(k):
            for b in range(k):
                GW[a, b] += W[i, a] * W[i, b]
    for j in range(n):
        for a in range(k):
            for b in range(k):
                GH[a, b] += H[a, j] * H[b, j]
    np.testing.assert_allclose(orc.wta_dense(A, W), P, rtol=1e-13)
    np.testing.assert_allclose(orc.aht_dense(A, H), Q, rtol=1e-13)
    np.testing.assert_allclose(orc.gram_w(W), GW, rtol=1e-13)
    np.testing.assert_allclose(orc.gram_h(H), GH, rtol=1e-13)
    # element-wise updates, denominators written out
    eps = 1e-3
    Hn = np.empty_like(H); Wn = np.empty_like(W)
    for c in range(k):
        for j in range(n):
            Hn[c, j] = H[c, j] * P[c, j] / (sum(GW[c, d] * H[d, j] for d in range(k)) + eps)
    for i in range(m):
        for c in range(k):
            Wn[i, c] = W[i, c] * Q[i, c] / (sum(W[i, d] * GH[d, c] for d in range(k)) + eps)
    np.testing.assert_allclose(orc.h_update(H, P, GW, eps), Hn, rtol=1e-13)
    np.testing.assert_allclose(orc.w_update(W, Q, GH, eps), Wn, rtol=1e-13)


def test_products_reduce_to_library_matmul():
    """On a moderate shape each product is a plain matrix product, so a
    library matmul in double must agree (catches transposed operands)."""
    A, W, H = small_case(97, 131, 5, 21)
    Ad = A.astype(np.float64)
    np.testing.assert_allclose(orc.wta_dense(A, W), W.T @ Ad, rtol=1e-12)
    np.testing.assert_allclose(orc.aht_dense(A, H), Ad @ H.T, rtol=1e-12)
    np.testing.assert_allclose(orc.gram_w(W), W.T @ W, rtol=1e-12)
    np.testing.assert_allclose(orc.gram_h(H), H @ H.T, rtol=1e-12)


def test_denominator_association():
    """(W^T W) H equals W^T (W H): the Gram-first form changes nothing."""
    A, W, H = small_case(9, 8, 3, 22)
    lhs = orc.gram_w(W) @ H
    rhs = W.T @ (W @ H)
    np.testing.assert_allclose(lhs, rhs, rtol=1e-12)


def test_eps_enters_once_in_the_denominator():
    """With A = 0 the numerator is 0 and with H = 0 the denominator is eps
    alone: W^T A / eps shows eps is added exactly once (Algorithm 1)."""
    A, W, H = small_case(4, 5, 2, 23)
    P = orc.wta_dense(A, W)
    G = orc.gram_w(W)
    tiny = 1e-30
    Hs = np.full_like(H, tiny)
    eps = 0.25
    out = orc.h_update(Hs, P, G, eps)
    np.testing.assert_allclose(out, tiny * P / eps, rtol=1e-12)


# --- P2: exact factorisation is a fixed point ---------------------------------

@pytest.mark.parametrize("seed", [31, 32, 33])
def test_fixed_point(seed):
    r = rng(seed)
    Ws = r.integers(1, 5, size=(6, 2)).astype(np.float64)
    Hs = r.integers(1, 5, size=(2, 7)).astype(np.float64)
    A = (Ws @ Hs).astype(np.float32)          # small integers: exact in fp32
    W, H = orc.mu_dense(A, Ws, Hs, 3, 0.0)
    np.testing.assert_allclose(W, Ws, rtol=1e-14)
    np.testing.assert_allclose(H, Hs, rtol=1e-14)


# --- P3: rank one closed form --------------------------------------------------

def test_rank_one_closed_form():
    A, W, H = small_case(7, 9, 1, 41)
    Ad = A.astype(np.float64)
    w = W[:, 0]
    h1 = (w @ Ad) / (w @ w)                   # independent of the initial H
    w1 = (Ad @ h1) / (h1 @ h1)
    Wo, Ho = orc.mu_dense(A, W, H, 1, 0.0)
    np.testing.assert_allclose(Ho[0], h1, rtol=1e-13)
    np.testing.assert_allclose(Wo[:, 0], w1, rtol=1e-13)
    Wo2, Ho2 = orc.mu_dense(A, W, 3.7 * H, 1, 0.0)
    np.testing.assert_allclose(Ho2, Ho, rtol=1e-13)


# --- P4: non-negativity and persistent zeros ------------------------------------

def test_nonnegative_and_zero_pattern():
    A, W, H = small_case(12, 10, 3, 51)
    A[4, :] = 0.0                              # a zero row of A
    W[2, 1] = 0.0
    H[0, 5] = 0.0
    Wo, Ho = orc.mu_dense(A, W, H, 5, EPS)
    assert np.isfinite(Wo).all() and np.isfinite(Ho).all()
    assert (Wo >= 0).all() and (Ho >= 0).all()
    assert Wo[2, 1] == 0.0 and Ho[0, 5] == 0.0
    assert (Wo[4, :] == 0.0).all()             # zero row of A drives its W row to zero


def test_all_zero_inputs_give_zero_not_nan():
    A = np.zeros((3, 4), dtype=np.float32)
    W = np.zeros((3, 2)); H = np.zeros((2, 4))
    Wo, Ho = orc.mu_dense(A, W, H, 2, EPS)
    assert (Wo == 0).all() and (Ho == 0).all()


# --- P5: the objective never increases ------------------------------------------

def config1():
    """256 x 192, planted rank 4 plus additive U[0, 0.01) noise, k = 4."""
    A = nmf_inputs.dense_planted(256, 192, 4, seed=1001, noise="add", lo=0.0, hi=0.01).numpy()
    W, H = nmf_inputs.init_factors(256, 192, 4, seed=2001)
    return A, W.numpy().astype(np.float64), H.numpy().astype(np.float64)


def test_monotone_objective_config1():
    A, W, H = config1()
    normA = float(np.linalg.norm(A.astype(np.float64)))
    prev = orc.residual_dense(A, W, H)
    first = prev
    for _ in range(100):
        W, H = orc.h_step_dense(A, W, H, EPS)
        r = orc.residual_dense(A, W, H)
        assert r <= prev + 1e-12 * normA
        prev = r
        W, H = orc.w_step_dense(A, W, H, EPS)
        r = orc.residual_dense(A, W, H)
        assert r <= prev + 1e-12 * normA
        prev = r
    assert prev < 0.1 * first                  # well below the starting error


@pytest.mark.parametrize("seed", [61, 62, 63, 64])
def test_monotone_objective_random(seed):
    r = rng(seed)
    m, n, k = int(r.integers(2, 12)), int(r.integers(2, 12)), int(r.integers(1, 4))
    A, W, H = small_case(m, n, k, seed)
    normA = float(np.linalg.norm(A))
    prev = orc.residual_dense(A, W, H)
    for _ in range(30):
        W, H = orc.h_step_dense(A, W, H, EPS)
        r1 = orc.residual_dense(A, W, H)
        W, H = orc.w_step_dense(A, W, H, EPS)
        r2 = orc.residual_dense(A, W, H)
        assert r1 <= prev + 1e-12 * normA and r2 <= r1 + 1e-12 * normA
        prev = r2


def test_residual_is_the_frobenius_norm():
    A, W, H = small_case(6, 5, 2, 65)
    want = np.sqrt(((A.astype(np.float64) - W @ H) ** 2).sum())
    assert abs(orc.residual_dense(A, W, H) - want) <= 1e-13 * want


@pytest.mark.parametrize("m,n,k,density,seed", [(7, 9, 2, 0.4, 1), (40, 30, 5, 0.1, 2), (30, 50, 3, 0.0, 3)])
def test_sparse_residual_is_the_frobenius_norm_over_all_entries(m, n, k, density, seed):
    """The expansion the sparse objective uses against the definition on the dense copy of A
    (zeros of A count: ||W H|| enters in full)."""
    r = np.random.default_rng(seed)
    Ad = (r.random((m, n)) * (r.random((m, n)) < density)).astype(np.float32)
    rowptr = np.zeros(m + 1, dtype=np.int64)
    cols, vals = [], []
    for i in range(m):
        nz = np.nonzero(Ad[i])[0]
        cols.append(nz.astype(np.int32))
        vals.append(Ad[i, nz])
        rowptr[i + 1] = rowptr[i] + nz.size
    colidx = np.concatenate(cols) if cols else np.zeros(0, np.int32)
    v = np.concatenate(vals).astype(np.float32) if vals else np.zeros(0, np.float32)
    W = r.random((m, k))
    H = r.random((k, n))
    want = np.sqrt(((Ad.astype(np.float64) - W @ H) ** 2).sum())
    got = orc.residual_csr(rowptr, colidx, v, m, n, W, H)
    assert abs(got - want) <= 1e-12 * want
    assert abs(got - orc.residual_dense(Ad, W, H)) <= 1e-12 * want


def test_half_steps_compose_to_one_iteration():
    A, W, H = small_case(9, 7, 3, 66)
    W1, H1 = orc.h_step_dense(A, W, H, EPS)
    np.testing.assert_array_equal(W1, W)       # the H step leaves W alone
    W2, H2 = orc.w_step_dense(A, W1, H1, EPS)
    np.testing.assert_array_equal(H2, H1)
    Wf, Hf = orc.mu_dense(A, W, H, 1, EPS)
    np.testing.assert_array_equal(Wf, W2)
    np.testing.assert_array_equal(Hf, H2)


# --- P6, P7: equivariances -------------------------------------------------------

def test_scale_equivariance():
    A, W, H = small_case(8, 9, 3, 71)
    d = np.array([0.5, 2.0, 4.0])              # powers of two: scaling is exact
    W1, H1 = orc.mu_dense(A, W, H, 1, 0.0)
    Ws, Hs = orc.mu_dense(A, W * d, H / d[:, None], 1, 0.0)
    np.testing.assert_allclose(Hs, H1 / d[:, None], rtol=1e-13)
    np.testing.assert_allclose(Ws, W1 * d, rtol=1e-13)


def test_permutation_equivariance():
    A, W, H = small_case(8, 9, 3, 72)
    r = rng(72)
    pr, pc, pk = r.permutation(8), r.permutation(9), r.permutation(3)
    W1, H1 = orc.mu_dense(A, W, H, 2, EPS)
    W2, H2 = orc.mu_dense(A[pr][:, pc], W[pr][:, pk], H[pk][:, pc], 2, EPS)
    np.testing.assert_allclose(W2, W1[pr][:, pk], rtol=1e-12)
    np.testing.assert_allclose(H2, H1[pk][:, pc], rtol=1e-12)


# --- P8: transpose duality ---------------------------------------------------------

def test_transpose_duality():
    """The W step on (A^T, H^T, W^T) is the transpose of the H step on
    (A, W, H), and vice versa: each half of the code checks the other."""
    A, W, H = small_case(7, 10, 3, 81)
    At = np.ascontiguousarray(A.T)
    _, H1 = orc.h_step_dense(A, W, H, EPS)
    Wp, _ = orc.w_step_dense(At, np.ascontiguousarray(H.T), np.ascontiguousarray(W.T), EPS)
    np.testing.assert_allclose(Wp.T, H1, rtol=1e-13)
    W1, _ = orc.w_step_dense(A, W, H, EPS)
    _, Hp = orc.h_step_dense(At, np.ascontiguousarray(H.T), np.ascontiguousarray(W.T), EPS)
    np.testing.assert_allclose(Hp.T, W1, rtol=1e-13)


# --- P9: composition -----------------------------------------------------------------

def test_composition_of_iteration_counts():
    A, W, H = small_case(10, 8, 2, 91)
    Wa, Ha = orc.mu_dense(A, W, H, 3, EPS)
    Wb, Hb = orc.mu_dense(A, Wa, Ha, 4, EPS)
    Wc, Hc = orc.mu_dense(A, W, H, 7, EPS)
    np.testing.assert_array_equal(Wb, Wc)
    np.testing.assert_array_equal(Hb, Hc)
    W0, H0 = orc.mu_dense(A, W, H, 0, EPS)
    np.testing.assert_array_equal(W0, W)
    np.testing.assert_array_equal(H0, H)


# --- P10: CSR stands for the dense matrix it sums to ----------------------------------

def _scrambled_csr(A, seed):
    """CSR of A with explicit zeros, shuffled columns within rows, and some
    entries split into two stored entries that add up to the original."""
    r = rng(seed)
    m, n = A.shape
    rows = []
    for i in range(m):
        ent = [(j, float(A[i, j])) for j in range(n) if A[i, j] != 0]
        for j in range(n):
            if A[i, j] == 0 and r.random() < 0.3:
                ent.append((j, 0.0))           # explicit stored zero
        extra = []
        for t, (j, v) in enumerate(ent):
            if v != 0 and r.random() < 0.3:
                half = float(np.float32(v * 0.5))
                rest = float(np.float32(v) - np.float32(half))
                if np.float32(half) + np.float32(rest) == np.float32(v):
                    ent[t] = (j, half)
                    extra.append((j, rest))
        ent += extra
        order = r.permutation(len(ent))
        rows.append([ent[t] for t in order])
    rowptr = np.zeros(m + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum([len(x) for x in rows])
    colidx = np.array([j for row in rows for j, _ in row], dtype=np.int32)
    vals = np.array([v for row in rows for _, v in row], dtype=np.float32)
    return rowptr, colidx, vals


@pytest.mark.parametrize("seed", [101, 102])
def test_csr_equals_dense(seed):
    r = rng(seed)
    m, n, k = 13, 11, 3
    A = r.random((m, n), dtype=np.float32)
    A[r.random((m, n)) < 0.6] = 0.0
    A[5, :] = 0.0                              # an empty row
    W = r.random((m, k)); H = r.random((k, n))
    rowptr, colidx, vals = _scrambled_csr(A, seed)
    np.testing.assert_allclose(orc.wta_csr(rowptr, colidx, vals, n, W), orc.wta_dense(A, W), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(orc.aht_csr(rowptr, colidx, vals, H), orc.aht_dense(A, H), rtol=1e-12, atol=1e-15)
    Wd, Hd = orc.mu_dense(A, W, H, 4, EPS)
    Ws, Hs = orc.mu_csr(rowptr, colidx, vals, m, n, W, H, 4, EPS)
    np.testing.assert_allclose(Ws, Wd, rtol=1e-11, atol=1e-300)
    np.testing.assert_allclose(Hs, Hd, rtol=1e-11, atol=1e-300)


def test_csr_generator_structure():
    rowptr, colidx, vals = nmf_inputs.csr_uniform(300, 500, 0.02, seed=7)
    rowptr, colidx, vals = rowptr.numpy(), colidx.numpy(), vals.numpy()
    assert rowptr.dtype == np.int64 and colidx.dtype == np.int32 and vals.dtype == np.float32
    assert rowptr[0] == 0 and rowptr[-1] == colidx.size == vals.size
    assert (np.diff(rowptr) >= 0).all()
    assert colidx.min() >= 0 and colidx.max() < 500
    for i in range(300):
        c = colidx[rowptr[i]:rowptr[i + 1]]
        assert (np.diff(c) > 0).all()
    assert (vals > 0).all() and (vals <= 1).all()
    assert abs(colidx.size - 300 * 500 * 0.02) < 5 * np.sqrt(300 * 500 * 0.02)


# --- P11: planted-rank recovery ------------------------------------------------------

@pytest.mark.parametrize("seed", [111, 112, 113])
def test_planted_rank_recovery(seed):
    r = rng(seed)
    W0 = r.random((24, 2)); H0 = r.random((2, 18))
    A = (W0 @ H0).astype(np.float32)
    W = r.random((24, 2)); H = r.random((2, 18))
    normA = float(np.linalg.norm(A))
    errs = [orc.residual_dense(A, W, H) / normA]
    for _ in range(5):
        W, H = orc.mu_dense(A, W, H, 1000, EPS)
        errs.append(orc.residual_dense(A, W, H) / normA)
    assert all(b <= a + 1e-12 for a, b in zip(errs, errs[1:]))
    assert errs[-1] < 1e-2, errs


# --- P12: operation count against the paper's FLOP model -------------------------------

def test_mac_count_matches_flop_model():
    """Section 3.1 lists five matrix products per iteration with I = m rows:
    W^T A (k I n), W^T W (k I k), H H^T (k n k), W HHT (I k k), A H^T (I n k).
    Its list leaves out the (W^T W) H product of the H update (k k n), which
    the update needs; the oracle executes the five listed ones plus that one."""
    m, n, k = 9, 7, 3
    A, W, H = small_case(m, n, k, 121)
    orc.reset_mac_count()
    orc.mu_dense(A, W, H, 2, EPS)
    listed = k * m * n + k * m * k + k * n * k + m * k * k + m * n * k
    assert orc.mac_count() == 2 * (listed + k * k * n)
    # the paper's total, 2*MACs minus one add per output element of each product
    flops_model = (2 * k * m * n + 2 * k * m * k + 2 * k * n + 2 * k * n * k + 2 * m * k * k
                   + 2 * m * n * k + 2 * m * k - k * n - k * k - k * k - m * k - m * k)
    products = 2 * listed - (k * n + k * k + k * k + m * k + m * k)
    elementwise = 2 * k * n + 2 * m * k
    assert flops_model == products + elementwise


# --- thread-count independence -----------------------------------------------------------

def test_reproducible_run_to_run():
    A, W, H = small_case(40, 33, 4, 131)
    W1, H1 = orc.mu_dense(A, W, H, 5, EPS)
    W2, H2 = orc.mu_dense(A, W, H, 5, EPS)
    np.testing.assert_array_equal(W1, W2)
    np.testing.assert_array_equal(H1, H2)


# --- the loop oracle against the same lines written as library products ---------------------

@pytest.mark.parametrize("m,n,k,block", [(40, 33, 4, 7), (129, 65, 9, 64), (64, 200, 17, 1000)])
def test_blas_variant_equals_loop_oracle(m, n, k, block):
    A, W, H = small_case(m, n, k, 141)
    W1, H1 = orc.mu_dense(A, W, H, 6, EPS)
    W2, H2 = orc.mu_dense_blas(A, W, H, 6, EPS, row_block=block)
    np.testing.assert_allclose(W2, W1, rtol=1e-11)
    np.testing.assert_allclose(H2, H1, rtol=1e-11)


def test_scipy_variant_equals_loop_oracle():
    r = rng(151)
    m, n, k = 60, 45, 5
    A = r.random((m, n), dtype=np.float32)
    A[r.random((m, n)) < 0.7] = 0.0
    A[7, :] = 0.0
    rowptr, colidx, vals = _scrambled_csr(A, 151)
    W = r.random((m, k)); H = r.random((k, n))
    W1, H1 = orc.mu_csr(rowptr, colidx, vals, m, n, W, H, 5, EPS)
    W2, H2 = orc.mu_csr_scipy(rowptr, colidx, vals, m, n, W, H, 5, EPS)
    np.testing.assert_allclose(W2, W1, rtol=1e-11, atol=1e-300)
    np.testing.assert_allclose(H2, H1, rtol=1e-11, atol=1e-300)


# --- Algorithm 1's loop with its stopping rule ------------------------------------------------

def test_tolerance_loop_stops_where_the_objective_says():
    A, W, H = config1()
    traj = [orc.residual_dense(A, W, H)]
    Wt, Ht = W, H
    for _ in range(12):
        Wt, Ht = orc.mu_dense(A, Wt, Ht, 5, EPS)
        traj.append(orc.residual_dense(A, Wt, Ht))
    tol = 0.5 * (traj[7] + traj[8])                   # first met after 8 checks = 40 iterations
    Wo, Ho, done, res = orc.mu_dense_tol(A, W, H, 1000, EPS, tol, check_every=5)
    assert done == 40 and res == traj[8] and res <= tol < traj[7]
    W40, H40 = orc.mu_dense(A, W, H, 40, EPS)
    np.testing.assert_array_equal(Wo, W40)
    np.testing.assert_array_equal(Ho, H40)
    # the iteration cap wins when the tolerance is out of reach; tol already met => no iteration
    _, _, done, _ = orc.mu_dense_tol(A, W, H, 7, EPS, 0.0, check_every=5)
    assert done == 7
    Wn, Hn, done, res = orc.mu_dense_tol(A, W, H, 7, EPS, 1e9, check_every=5)
    assert done == 0 and res == traj[0]
    np.testing.assert_array_equal(Wn, W)


def test_sparse_tolerance_loop_stops_where_the_objective_says():
    """mu_csr_tol against a hand-rolled loop over mu_csr and the objective of the dense copy."""
    import scipy.sparse as sp
    m, n, k = 40, 30, 3
    r = np.random.default_rng(12)
    Ad = (r.random((m, n)) * (r.random((m, n)) < 0.3)).astype(np.float32)
    S = sp.csr_matrix(Ad)
    S.sort_indices()
    rowptr, colidx, vals = S.indptr.astype(np.int64), S.indices.astype(np.int32), S.data.astype(np.float32)
    W, H = r.random((m, k)), r.random((k, n))
    traj = [orc.residual_dense(Ad, W, H)]
    Wt, Ht = W, H
    for _ in range(10):
        Wt, Ht = orc.mu_csr(rowptr, colidx, vals, m, n, Wt, Ht, 2, EPS)
        traj.append(orc.residual_dense(Ad, Wt, Ht))
    assert traj[5] < traj[4]
    tol = 0.5 * (traj[4] + traj[5])                   # first met after 5 checks = 10 iterations
    Wo, Ho, done, res = orc.mu_csr_tol(rowptr, colidx, vals, m, n, W, H, 1000, EPS, tol, check_every=2)
    assert done == 10 and abs(res - traj[5]) <= 1e-12 * traj[5] and res <= tol < traj[4]
    W10, H10 = orc.mu_csr(rowptr, colidx, vals, m, n, W, H, 10, EPS)
    np.testing.assert_array_equal(Wo, W10)
    np.testing.assert_array_equal(Ho, H10)
    _, _, done, _ = orc.mu_csr_tol(rowptr, colidx, vals, m, n, W, H, 7, EPS, 0.0, check_every=2)
    assert done == 7
    Wn, Hn, done, res = orc.mu_csr_tol(rowptr, colidx, vals, m, n, W, H, 7, EPS, 1e9, check_every=2)
    assert done == 0 and abs(res - traj[0]) <= 1e-12 * traj[0]
    np.testing.assert_array_equal(Wn, W)


def test_ensemble_is_the_block_diagonal_stacked_iteration():
    """mu_ensemble (independent runs, sections 1 and 4.5) against one stacked iteration written with
    library products: runs that share A are the factor blocks of a single W_all (m x sum k) and
    H_all (sum k x n) whose two Gram matrices are cut down to their diagonal blocks, so that no run
    sees another.  Also: a run's result does not change when another run's start does."""
    m, n = 37, 29
    r = np.random.default_rng(41)
    A = r.random((m, n)).astype(np.float32)
    ks = [1, 3, 2, 5]
    Ws = [r.random((m, k)) for k in ks]
    Hs = [r.random((k, n)) for k in ks]
    iters = 7
    got = orc.mu_ensemble([A] * len(ks), Ws, Hs, iters, EPS)
    assert len(got) == len(ks)
    ids = np.concatenate([np.full(k, i) for i, k in enumerate(ks)])
    mask = (ids[:, None] == ids[None, :]).astype(np.float64)
    Wall, Hall = np.concatenate(Ws, axis=1), np.concatenate(Hs, axis=0)
    Ad = A.astype(np.float64)
    for _ in range(iters):
        Hall = Hall * (Wall.T @ Ad) / (((Wall.T @ Wall) * mask) @ Hall + EPS)
        Wall = Wall * (Ad @ Hall.T) / (Wall @ ((Hall @ Hall.T) * mask) + EPS)
    off = 0
    for (Wg, Hg), k in zip(got, ks):
        assert Wg.shape == (m, k) and Hg.shape == (k, n)
        np.testing.assert_allclose(Wg, Wall[:, off:off + k], rtol=1e-11, atol=0)
        np.testing.assert_allclose(Hg, Hall[off:off + k], rtol=1e-11, atol=0)
        off += k
    # different matrices per run, and independence of the runs
    As = [A, (A * 1.5).astype(np.float32), A, A]
    base = orc.mu_ensemble(As, Ws, Hs, iters, EPS)
    Ws2 = [Ws[0], r.random((m, ks[1])), Ws[2], Ws[3]]
    other = orc.mu_ensemble(As, Ws2, Hs, iters, EPS)
    for i in (0, 2, 3):
        np.testing.assert_array_equal(base[i][0], other[i][0])
        np.testing.assert_array_equal(base[i][1], other[i][1])
    assert not np.array_equal(base[1][0], other[1][0])
    Wb, Hb = orc.mu_dense_blas(As[1], Ws[1], Hs[1], iters, EPS)
    np.testing.assert_allclose(base[1][0], Wb, rtol=1e-11, atol=0)
    np.testing.assert_allclose(base[1][1], Hb, rtol=1e-11, atol=0)
