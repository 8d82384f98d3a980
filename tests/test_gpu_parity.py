"""Parity of the HIP library (through its C ABI) against the CPU oracle.

Metric: relative Frobenius error max(||W-Wref||/||Wref||, ||H-Href||/||Href||)
with the fp32 result widened to double.  Bars (from the target statement):
1e-5 after one iteration, 1e-3 after the configuration's final iteration
count.  Single products are held to 1e-5 as well (fp32 accumulation over at
most a few thousand terms per chain, then tree sums).
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
TOL1 = 1e-5
TOLN = 1e-3


def dev(x, dtype=torch.float32):
    return torch.as_tensor(np.ascontiguousarray(x)).to(dtype).cuda().contiguous()


def host(t):
    torch.cuda.synchronize()
    return t.detach().cpu().numpy().astype(np.float64)


def rel(x, ref):
    return orc.rel_fro(x, ref)


def case(m, n, k, seed):
    A = nmf_inputs.uniform((m, n), seed).numpy()
    W, H = nmf_inputs.init_factors(m, n, k, seed + 1)
    return A, W.numpy(), H.numpy()


SHAPES = [
    (1, 5, 1), (2, 3, 2), (33, 31, 3), (64, 128, 4), (300, 200, 4), (257, 131, 17),
    (1000, 520, 32), (513, 260, 64), (130, 1027, 33), (2049, 96, 8), (70, 4100, 5),
]


@pytest.mark.parametrize("m,k", [(1, 1), (7, 3), (1000, 32), (4099, 64), (70000, 17), (513, 33)])
def test_gram_w(m, k):
    W = nmf_inputs.uniform((m, k), 5).numpy()
    G = torch.empty((k, k), device="cuda")
    nmf.nmf_gram_w(dev(W), m, k, G)
    assert rel(host(G), orc.gram_w(W)) < TOL1


@pytest.mark.parametrize("m,n,k", SHAPES)
def test_wta_dense(m, n, k):
    A, W, _ = case(m, n, k, 10)
    P = torch.empty((k, n), device="cuda")
    nmf.nmf_wta_dense(dev(A), m, n, k, dev(W), P)
    assert rel(host(P), orc.wta_dense(A, W)) < TOL1


# Few columns and many rows: a workgroup of the pass then walks 8192 rows.  The bf16 matrix
# instruction drops the bits of a product that fall below its accumulator's width without
# rounding, so a matrix accumulator kept over that many rows comes out low (1e-5 relative
# at 4096 rows on this data); the kernels bound its run and add the pieces up in rounded
# fp32.  n = 514 takes the kernels for unaligned rows (plain loads; fp32 instruction above
# 32 factors).
@pytest.mark.parametrize("m,n,k", [(262144, 512, 32), (262144, 512, 64), (262144, 514, 32), (262144, 514, 64),
                                   (100000, 1024, 48)])
def test_wta_dense_long_sums_keep_fp32_accuracy(m, n, k):
    A = nmf_inputs.uniform((m, n), 77).numpy()
    W = nmf_inputs.uniform((m, k), 78).numpy()
    P = torch.empty((k, n), device="cuda")
    nmf.nmf_wta_dense(dev(A), m, n, k, dev(W), P)
    want = orc.wta_dense(A, W)
    got = host(P).astype(np.float64)
    assert rel(got, want) < 3e-7
    assert abs(np.mean((got - want) / want)) < 1.5e-7


@pytest.mark.parametrize("n,k", [(5, 1), (131, 17), (1027, 33), (4100, 5), (20000, 32), (9999, 64)])
def test_h_update_and_gram_h(n, k):
    r = np.random.default_rng(n + k)
    H = r.random((k, n), dtype=np.float32)
    P = r.random((k, n), dtype=np.float32) * 7
    X = r.random((50, k), dtype=np.float32)
    G = (X.T @ X).astype(np.float32)
    Hd = dev(H)
    GH = torch.empty((k, k), device="cuda")
    nmf.nmf_h_update(Hd, dev(P), dev(G), k, n, 1e-3, GH)
    Href = orc.h_update(H, P, G, 1e-3)
    assert rel(host(Hd), Href) < TOL1
    assert rel(host(GH), orc.gram_h(host(Hd))) < TOL1


@pytest.mark.parametrize("m,n,k", SHAPES)
def test_aht_w_update(m, n, k):
    A, W, H = case(m, n, k, 20)
    GH = orc.gram_h(H).astype(np.float32)
    Wd = dev(W)
    nmf.nmf_aht_w_update_dense(dev(A), m, n, k, dev(H), dev(GH), Wd, EPS)
    Wref = orc.w_update(W, orc.aht_dense(A, H), GH, float(np.float32(EPS)))
    assert rel(host(Wd), Wref) < TOL1


def run_dense(A, W, H, iters, eps=EPS):
    m, n = A.shape
    k = W.shape[1]
    Wd, Hd = dev(W), dev(H)
    nmf.nmf_mu_dense(dev(A), m, n, k, Wd, Hd, iters, eps)
    return host(Wd), host(Hd)


def check(Wg, Hg, Wr, Hr, tol):
    assert np.isfinite(Wg).all() and np.isfinite(Hg).all()
    assert (Wg >= 0).all() and (Hg >= 0).all()
    e = max(rel(Wg, Wr), rel(Hg, Hr))
    assert e < tol, e
    return e


@pytest.mark.parametrize("m,n,k", SHAPES)
def test_mu_dense_one_iteration(m, n, k):
    A, W, H = case(m, n, k, 30)
    Wg, Hg = run_dense(A, W, H, 1)
    Wr, Hr = orc.mu_dense(A, W, H, 1, float(np.float32(EPS)))
    check(Wg, Hg, Wr, Hr, TOL1)


# The row plan (k <= 32, m >= 4096 or a small problem): ragged rows and columns, more row blocks
# than workgroups (the kernel then walks several blocks), 64-row and 128-row blocks, ranks off the
# tile sizes.
@pytest.mark.parametrize("m,n,k,iters", [
    (4100, 1028, 17, 2), (5000, 260, 32, 2), (40000, 128, 8, 2), (4097, 68, 1, 1), (33000, 1200, 32, 1),
    (24600, 4, 3, 2), (8192, 8256, 32, 1), (4100, 1028, 33, 1),
])
def test_row_plan_shapes(m, n, k, iters):
    """Run twice: as the library plans it (the row plan for 12288 rows and 512 columns or more and for
    small problems, a transposed copy otherwise), and with a workspace that has no room for a copy,
    which leaves every one of these shapes to the row kernel."""
    A, W, H = case(m, n, k, 300 + k)
    Wr, Hr = orc.mu_dense(A, W, H, iters, float(np.float32(EPS)))
    Wg, Hg = run_dense(A, W, H, iters)
    check(Wg, Hg, Wr, Hr, TOL1 * iters)
    buf = torch.empty(nmf.nmf_mu_workspace_bytes(4, m, n, 0, k, 0), dtype=torch.uint8, device="cuda")
    nmf.nmf_mu_set_workspace(buf)
    try:
        assert nmf.nmf_mu_dense_profile(dev(A), m, n, k, dev(W), dev(H), 1, EPS)[6] == 2.0
        Wg, Hg = run_dense(A, W, H, iters)
    finally:
        torch.cuda.synchronize()
        nmf.nmf_mu_set_workspace(None)
    check(Wg, Hg, Wr, Hr, TOL1 * iters)


@pytest.mark.parametrize("m,n,k,iters", [(4100, 1028, 33, 2), (5000, 260, 64, 2), (20000, 128, 48, 2), (640, 512, 64, 3)])
def test_row_plan_33_to_64_factors_without_room_for_a_transposed_copy(m, n, k, iters):
    """From 33 to 64 factors the transposed copy comes first; a workspace that cannot hold it leaves
    the run to the row plan (two 32-factor tiles per row tile, 64-row blocks)."""
    A, W, H = case(m, n, k, 320 + k)
    buf = torch.empty(nmf.nmf_mu_workspace_bytes(4, m, n, 0, k, 0), dtype=torch.uint8, device="cuda")
    nmf.nmf_mu_set_workspace(buf)
    try:
        Ad, Wd, Hd = dev(A), dev(W), dev(H)
        assert nmf.nmf_mu_dense_profile(Ad, m, n, k, dev(W), dev(H), 1, EPS)[6] == 2.0
        nmf.nmf_mu_dense(Ad, m, n, k, Wd, Hd, iters, EPS)
        Wg, Hg = host(Wd), host(Hd)
        # the same run cut into two calls: the seeding of W^T W and of the planes of W at call entry
        # adds up in the order of an updating launch, so the bits are the same
        W2, H2 = dev(W), dev(H)
        nmf.nmf_mu_dense(Ad, m, n, k, W2, H2, 1, EPS)
        nmf.nmf_mu_dense(Ad, m, n, k, W2, H2, iters - 1, EPS)
        np.testing.assert_array_equal(host(W2), Wg)
        np.testing.assert_array_equal(host(H2), Hg)
    finally:
        torch.cuda.synchronize()
        nmf.nmf_mu_set_workspace(None)
    Wr, Hr = orc.mu_dense(A, W, H, iters, float(np.float32(EPS)))
    check(Wg, Hg, Wr, Hr, TOL1 * iters)


@pytest.mark.parametrize("m,n,k,off,iters", [(5000, 1031, 32, 0, 2), (4100, 1028, 17, 1, 2), (6000, 514, 48, 3, 2),
                                             (300, 203, 8, 2, 3), (4097, 5, 3, 0, 2)])
def test_misaligned_a_runs_on_an_aligned_padded_copy(m, n, k, off, iters):
    """n % 4 != 0 or a base that is not 16-byte aligned: the call copies A and H into aligned arrays
    with zero columns appended and runs the row plan there; H comes back without the padding."""
    A, W, H = case(m, n, k, 330 + k)
    buf = torch.zeros(m * n + 8, dtype=torch.float32, device="cuda")
    Ad = buf[off:off + m * n].view(m, n)
    Ad.copy_(dev(A))
    hbuf = torch.full((k * n + 8,), -7.0, dtype=torch.float32, device="cuda")
    Hd = hbuf[off:off + k * n].view(k, n)
    Hd.copy_(dev(H))
    Wd = dev(W)
    nmf.nmf_mu_dense(Ad, m, n, k, Wd, Hd, iters, EPS)
    Wg, Hg = host(Wd), host(Hd)
    Wr, Hr = orc.mu_dense(A, W, H, iters, float(np.float32(EPS)))
    check(Wg, Hg, Wr, Hr, TOL1 * iters)
    torch.cuda.synchronize()
    guard = hbuf.cpu().numpy()
    assert (guard[:off] == -7.0).all() and (guard[off + k * n:] == -7.0).all()     # nothing written around H


def test_row_plan_zero_rows_and_columns():
    """All-zero rows and columns of A inside and at the edges of row blocks and column chunks."""
    A, W, H = case(4200, 520, 16, 310)
    A[0, :] = 0
    A[127:130, :] = 0
    A[4199, :] = 0
    A[:, 63:66] = 0
    A[:, 519] = 0
    Wg, Hg = run_dense(A, W, H, 3)
    Wr, Hr = orc.mu_dense(A, W, H, 3, float(np.float32(EPS)))
    check(Wg, Hg, Wr, Hr, 3 * TOL1)
    assert (Wg[0] == 0).all() and (Wg[128] == 0).all() and (Wg[4199] == 0).all()
    assert (Hg[:, 64] == 0).all() and (Hg[:, 519] == 0).all()


def config1():
    A = nmf_inputs.dense_planted(256, 192, 4, seed=1001, noise="add", lo=0.0, hi=0.01).numpy()
    W, H = nmf_inputs.init_factors(256, 192, 4, seed=2001)
    return A, W.numpy(), H.numpy()


def test_config1_dense_1_and_100_iterations():
    A, W, H = config1()
    eps = float(np.float32(EPS))
    check(*run_dense(A, W, H, 1), *orc.mu_dense(A, W, H, 1, eps), TOL1)
    Wg, Hg = run_dense(A, W, H, 100)
    Wr, Hr = orc.mu_dense(A, W, H, 100, eps)
    check(Wg, Hg, Wr, Hr, TOLN)
    normA = np.linalg.norm(A.astype(np.float64))
    assert abs(orc.residual_dense(A, Wg, Hg) - orc.residual_dense(A, Wr, Hr)) < 1e-4 * normA


def test_config2_shape_reduced_100_iterations():
    """Config 2 recipe (planted rank 32, multiplicative noise, k = 32) at
    4096 x 2048 so that the oracle finishes 100 iterations in seconds."""
    m, n, k = 4096, 2048, 32
    A = nmf_inputs.dense_planted(m, n, 32, seed=1002).numpy()
    W, H = (t.numpy() for t in nmf_inputs.init_factors(m, n, k, seed=2002))
    eps = float(np.float32(EPS))
    check(*run_dense(A, W, H, 1), *orc.mu_dense(A, W, H, 1, eps), TOL1)
    check(*run_dense(A, W, H, 100), *orc.mu_dense(A, W, H, 100, eps), TOLN)


def test_dense_composition_and_determinism():
    A, W, H = case(700, 900, 12, 40)
    W7, H7 = run_dense(A, W, H, 7)
    Wa, Ha = run_dense(A, W, H, 3)
    Wb, Hb = run_dense(A, Wa.astype(np.float32), Ha.astype(np.float32), 4)
    np.testing.assert_array_equal(W7, Wb)
    np.testing.assert_array_equal(H7, Hb)
    W7b, H7b = run_dense(A, W, H, 7)
    np.testing.assert_array_equal(W7, W7b)
    np.testing.assert_array_equal(H7, H7b)


def test_dense_zero_patterns():
    A, W, H = case(200, 300, 6, 50)
    A[17, :] = 0.0
    A[:, 5] = 0.0
    W[3, 2] = 0.0
    H[1, 9] = 0.0
    Wg, Hg = run_dense(A, W, H, 3)
    Wr, Hr = orc.mu_dense(A, W, H, 3, float(np.float32(EPS)))
    check(Wg, Hg, Wr, Hr, 1e-4)
    assert Wg[3, 2] == 0 and Hg[1, 9] == 0
    assert (Wg[17, :] == 0).all() and (Hg[:, 5] == 0).all()
    Z = np.zeros_like(A)
    Wz, Hz = run_dense(Z, np.zeros_like(W), np.zeros_like(H), 2)
    assert (Wz == 0).all() and (Hz == 0).all()


def test_dense_on_a_side_stream_and_unaligned_views():
    A, W, H = case(333, 444, 9, 60)
    m, n, k = 333, 444, 9
    # a base pointer that is 4-byte but not 16-byte aligned takes the scalar path
    buf = torch.empty(m * n + 1, device="cuda")
    Ad = buf[1:].view(m, n)
    Ad.copy_(torch.from_numpy(A))
    assert Ad.data_ptr() % 16 != 0
    Wd, Hd = dev(W), dev(H)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        nmf.nmf_mu_dense(Ad, m, n, k, Wd, Hd, 2, EPS, stream=s)
    s.synchronize()
    Wr, Hr = orc.mu_dense(A, W, H, 2, float(np.float32(EPS)))
    check(host(Wd), host(Hd), Wr, Hr, 2e-5)


def oracle_trajectory(A, W, H, iters):
    eps = float(np.float32(EPS))
    out = []
    for _ in range(iters):
        W, H = orc.mu_dense(A, W, H, 1, eps)
        out.append(orc.residual_dense(A, W, H))
    return np.array(out), W, H


@pytest.mark.parametrize("m,n,k,iters", [(256, 192, 4, 30), (1000, 520, 32, 6), (513, 260, 64, 4), (300, 200, 17, 5)])
def test_monitor_reports_the_objective_of_every_iteration(m, n, k, iters):
    if (m, n, k) == (256, 192, 4):
        A, W, H = config1()
    else:
        A, W, H = case(m, n, k, 44)
    want, Wr, Hr = oracle_trajectory(A, W, H, iters)
    Wd, Hd = dev(W), dev(H)
    got = np.array(nmf.nmf_mu_dense_monitor(dev(A), m, n, k, Wd, Hd, iters, EPS))
    normA2 = float(np.sum(A.astype(np.float64) ** 2))
    # fp32 sums in the three terms of the expansion: absolute error of f^2 about 3e-7 ||A||^2
    bound = np.maximum(1e-5 * want, 3e-7 * normA2 / want)
    assert (np.abs(got - want) <= bound).all(), (got, want)
    assert (np.diff(got) <= 1e-6 * got[:-1] + 2 * bound[1:]).all()        # non-increasing, as the method guarantees
    # the monitored run is the plain run, bit for bit
    Wg, Hg = run_dense(A, W, H, iters)
    np.testing.assert_array_equal(host(Wd), Wg)
    np.testing.assert_array_equal(host(Hd), Hg)


def test_monitor_small_plan_gives_the_exact_values():
    A, W, H = case(300, 200, 9, 45)
    want, _, _ = oracle_trajectory(A, W, H, 4)
    need = nmf.nmf_mu_workspace_bytes(4, 300, 200, 0, 9, 0) + (1 << 16)
    assert need < nmf.nmf_mu_workspace_bytes(0, 300, 200, 0, 9, 0)
    buf = torch.empty(need, dtype=torch.uint8, device="cuda")
    nmf.nmf_mu_set_workspace(buf)
    try:
        got = np.array(nmf.nmf_mu_dense_monitor(dev(A), 300, 200, 9, dev(W), dev(H), 4, EPS))
    finally:
        nmf.nmf_mu_set_workspace(None)
    assert (np.abs(got - want) <= 1e-5 * want).all()


# ---- operand encoding of the k <= 32 pass (bit-exact) ---------------------------------

def bf16_bits_to_f64(u16):
    return (u16.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


@pytest.mark.parametrize("rows,k", [(1, 1), (8, 32), (13, 5), (1000, 32), (4099, 17), (100, 33), (515, 64)])
def test_split_planes_encoding_is_exact(rows, k):
    """The three bf16 pieces of every factor entry add up to the entry bit for bit,
    each piece is the truncation the header states, the layout is the stated one
    and the padding is zero (host recomputation with integer masks)."""
    r = np.random.default_rng(rows * 100 + k)
    X = (r.random((rows, k), dtype=np.float32) * np.float32(10.0) ** r.integers(-20, 20, (rows, k))).astype(np.float32)
    X[0, 0] = 0.0
    X[rows // 2, k // 2] = np.float32(1.0)          # one piece only
    X[rows - 1, k - 1] = np.float32(3.0e38)
    groups = (rows + 7) // 8
    KP = 32 if k <= 32 else 64
    planes = torch.full((groups * 24 * KP,), -1, dtype=torch.int16, device="cuda")
    nmf.nmf_split_planes(dev(X), rows, k, planes)
    torch.cuda.synchronize()
    P = planes.cpu().numpy().view(np.uint16).reshape(groups, 3, KP, 8)
    # host: truncation by masking the low 16 bits, exact float32 subtractions
    Xp = np.zeros((groups * 8, KP), dtype=np.float32)
    Xp[:rows, :k] = X
    h = (Xp.view(np.uint32) & np.uint32(0xffff0000)).view(np.float32)
    r1 = Xp - h
    m = (r1.view(np.uint32) & np.uint32(0xffff0000)).view(np.float32)
    l = r1 - m
    assert ((l.view(np.uint32) & np.uint32(0xffff)) == 0).all()      # the last piece is a bf16 already
    want = np.stack([(x.view(np.uint32) >> 16).astype(np.uint16).reshape(groups, 8, KP).transpose(0, 2, 1)
                     for x in (h, m, l)], axis=1)
    np.testing.assert_array_equal(P, want)
    total = bf16_bits_to_f64(P[:, 0]) + bf16_bits_to_f64(P[:, 1]) + bf16_bits_to_f64(P[:, 2])
    np.testing.assert_array_equal(total.transpose(0, 2, 1).reshape(groups * 8, KP), Xp.astype(np.float64))


def random_shapes(count, seed):
    """Seeded shapes that mix the kernels' paths: row counts around the 16-row step and the
    32-row tile, column counts around the 64-, 128- and 256-column slabs (half of them
    multiples of 4, which the aligned kernels need), ranks around 32 and 64."""
    r = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        m = int(r.choice([r.integers(1, 40), r.integers(40, 700), 16 * r.integers(1, 40) + r.integers(-1, 2)]))
        n = int(r.choice([r.integers(1, 40), r.integers(40, 700), 64 * r.integers(1, 11) + r.integers(-1, 2)]))
        if r.random() < 0.5:
            n = max(4, n // 4 * 4)
        k = int(r.choice([r.integers(1, 65), r.choice([1, 15, 16, 17, 31, 32, 33, 48, 63, 64])]))
        out.append((max(m, 1), max(n, 1), k))
    return out


@pytest.mark.parametrize("m,n,k", random_shapes(40, 2024))
def test_dense_random_shapes_two_iterations(m, n, k):
    A, W, H = case(m, n, k, 1000 + m + 7 * n + 13 * k)
    Wg, Hg = run_dense(A, W, H, 2)
    Wr, Hr = orc.mu_dense(A, W, H, 2, float(np.float32(EPS)))
    check(Wg, Hg, Wr, Hr, 2 * TOL1)
    got = nmf.nmf_residual_dense(dev(A), m, n, k, dev(W), dev(H))
    want = orc.residual_dense(A, W, H)
    assert abs(got - want) <= 1e-5 * want


# ---- objective and tolerance-driven run --------------------------------------------

# the last ten take the streaming kernel: whole 32-row tiles (with up to 31 rows left to the
# general one), ragged and single column slabs, both factor step counts, fewer tiles than waves,
# and 5, 6, 7 and 9 tiles per row split (the kernel takes them in groups of four)
@pytest.mark.parametrize("m,n,k", SHAPES + [(4096, 2048, 32), (1000, 520, 16), (31, 64, 32), (32, 4, 16),
                                            (4128, 68, 16), (163, 8200, 32), (8192, 64, 32),
                                            (2591, 8200, 32), (4608, 8200, 16), (98304, 64, 16), (114705, 64, 32)])
def test_residual_dense(m, n, k):
    A, W, H = case(m, n, k, 32)
    got = nmf.nmf_residual_dense(dev(A), m, n, k, dev(W), dev(H))
    want = orc.residual_dense(A, W, H)
    assert abs(got - want) <= 1e-5 * want


def test_residual_dense_small_residual():
    """Near a good fit the objective is a small difference of large numbers:
    the fp32 tiles must still give it to 1e-4."""
    A, W, H = config1()
    Wr, Hr = orc.mu_dense(A, W, H, 100, float(np.float32(EPS)))
    Wf, Hf = Wr.astype(np.float32), Hr.astype(np.float32)
    got = nmf.nmf_residual_dense(dev(A), 256, 192, 4, dev(Wf), dev(Hf))
    want = orc.residual_dense(A, Wf, Hf)
    assert want < 0.1 * np.linalg.norm(A)
    assert abs(got - want) <= 1e-4 * want


def test_mu_dense_tol_matches_algorithm_1_loop():
    A, W, H = config1()
    eps = float(np.float32(EPS))
    traj = [orc.residual_dense(A, W, H)]
    Wt, Ht = W, H
    for _ in range(12):
        Wt, Ht = orc.mu_dense(A, Wt, Ht, 5, eps)
        traj.append(orc.residual_dense(A, Wt, Ht))
    tol = 0.5 * (traj[7] + traj[8])
    Wr, Hr, done_r, res_r = orc.mu_dense_tol(A, W, H, 1000, eps, tol, check_every=5)
    Wd, Hd = dev(W), dev(H)
    done, res = nmf.nmf_mu_dense_tol(dev(A), 256, 192, 4, Wd, Hd, 1000, EPS, tol, 5)
    assert done == done_r == 40
    assert abs(res - res_r) <= 1e-4 * res_r and res <= tol
    check(host(Wd), host(Hd), Wr, Hr, TOLN)
    # checked after every iteration (Algorithm 1 as printed): the cheap expansion decides far from
    # the tolerance, the exact evaluation near it; the stopping iteration is the oracle's
    want, _, _ = oracle_trajectory(A, W, H, 12)
    tol1 = 0.5 * (want[8] + want[9])
    Wd, Hd = dev(W), dev(H)
    done, res = nmf.nmf_mu_dense_tol(dev(A), 256, 192, 4, Wd, Hd, 1000, EPS, tol1, 1)
    assert done == 10 and abs(res - want[9]) <= 1e-4 * want[9]
    # cap reached / tolerance already met
    Wd, Hd = dev(W), dev(H)
    done, res = nmf.nmf_mu_dense_tol(dev(A), 256, 192, 4, Wd, Hd, 7, EPS, 0.0, 5)
    assert done == 7
    W7, H7 = orc.mu_dense(A, W, H, 7, eps)
    check(host(Wd), host(Hd), W7, H7, 1e-4)
    Wd, Hd = dev(W), dev(H)
    done, res = nmf.nmf_mu_dense_tol(dev(A), 256, 192, 4, Wd, Hd, 7, EPS, 1e9, 5)
    assert done == 0 and abs(res - traj[0]) <= 1e-5 * traj[0]
    np.testing.assert_array_equal(host(Wd), W.astype(np.float64))


# ---- out-of-memory path -------------------------------------------------------

@pytest.mark.parametrize("m,n,k,batch,slots,iters", [
    (1000, 520, 32, 256, 3, 3),     # ragged last batch
    (1000, 520, 32, 1000, 1, 2),    # one batch, one slot
    (777, 260, 64, 100, 2, 2),
    (300, 200, 4, 64, 3, 5),
    (129, 1027, 7, 1, 3, 2),        # one row per batch
    (500, 300, 16, 4096, 3, 2),     # batch larger than the matrix
])
def test_ooc_matches_oracle(m, n, k, batch, slots, iters):
    A, W, H = case(m, n, k, 70)
    Ah = torch.from_numpy(A).pin_memory()
    Wd, Hd = dev(W), dev(H)
    budget = slots * (((min(batch, m) * n * 4) + 255) // 256 * 256)
    nmf.nmf_mu_ooc(Ah, m, n, k, Wd, Hd, iters, EPS, batch, budget)
    Wr, Hr = orc.mu_dense(A, W, H, iters, float(np.float32(EPS)))
    check(host(Wd), host(Hd), Wr, Hr, TOL1 * iters)


@pytest.mark.parametrize("m,n,k,batch,slots,iters", [
    (1000, 520, 32, 256, 3, 5),     # ragged last batch: its workgroups leave a gap in the list of shares
    (777, 260, 64, 100, 2, 3),
    (256, 192, 4, 48, 3, 30),
    (640, 512, 17, 640, 1, 3),      # one batch
    (130, 70, 5, 1, 2, 2),          # one row per batch
])
def test_ooc_monitor_reports_the_objective_of_every_iteration(m, n, k, batch, slots, iters):
    if (m, n, k) == (256, 192, 4):
        A, W, H = config1()
    else:
        A, W, H = case(m, n, k, 71)
    want, Wr, Hr = oracle_trajectory(A, W, H, iters)
    Ah = torch.from_numpy(A).pin_memory()
    budget = slots * (((min(batch, m) * n * 4) + 255) // 256 * 256)
    Wd, Hd = dev(W), dev(H)
    got = np.array(nmf.nmf_mu_ooc_monitor(Ah, m, n, k, Wd, Hd, iters, EPS, batch, budget))
    normA2 = float(np.sum(A.astype(np.float64) ** 2))
    bound = np.maximum(1e-5 * want, 3e-7 * normA2 / want)
    assert (np.abs(got - want) <= bound).all(), (got, want)
    # the monitored run is the plain streamed run, bit for bit
    W2, H2 = dev(W), dev(H)
    nmf.nmf_mu_ooc(Ah, m, n, k, W2, H2, iters, EPS, batch, budget)
    np.testing.assert_array_equal(host(Wd), host(W2))
    np.testing.assert_array_equal(host(Hd), host(H2))


def test_ooc_monitor_argument_errors():
    A, W, H = case(64, 48, 70, 3)
    Ah = torch.from_numpy(A).pin_memory()
    with pytest.raises(nmf.NmfError) as e:
        nmf.nmf_mu_ooc_monitor(Ah, 64, 48, 70, dev(W), dev(H), 1, EPS, 16, 1 << 20)
    assert e.value.status == nmf.NMF_EUNSUPPORTED


def test_ooc_equals_small_plan_dense_bitwise_when_one_batch():
    """With one batch the out-of-memory path launches the same kernels as the
    resident path without the transposed copy of A (forced here by a caller
    workspace too small for that copy; n % 4 != 0 keeps both off the row plan)."""
    m, n, k = 640, 510, 48
    A, W, H = case(m, n, k, 80)
    buf = torch.empty(nmf.nmf_mu_workspace_bytes(4, m, n, 0, k, 0), dtype=torch.uint8, device="cuda")
    nmf.nmf_mu_set_workspace(buf)
    try:
        Wg, Hg = run_dense(A, W, H, 4)
        Ah = torch.from_numpy(A).pin_memory()
        Wd, Hd = dev(W), dev(H)
        nmf.nmf_mu_ooc(Ah, m, n, k, Wd, Hd, 4, EPS, m, 1 << 30)
        np.testing.assert_array_equal(host(Wd), Wg)
        np.testing.assert_array_equal(host(Hd), Hg)
    finally:
        nmf.nmf_mu_set_workspace(None)
    Wr, Hr = orc.mu_dense(A, W, H, 4, float(np.float32(EPS)))
    check(Wg, Hg, Wr, Hr, 4 * TOL1)


@pytest.mark.parametrize("m,n,k", SHAPES)
def test_small_plan_dense_one_iteration(m, n, k):
    """The direct A H^T kernel (no transposed copy of A) against the oracle."""
    A, W, H = case(m, n, k, 31)
    buf = torch.empty(nmf.nmf_mu_workspace_bytes(4, m, n, 0, k, 0), dtype=torch.uint8, device="cuda")
    nmf.nmf_mu_set_workspace(buf)
    try:
        Wg, Hg = run_dense(A, W, H, 1)
    finally:
        nmf.nmf_mu_set_workspace(None)
    Wr, Hr = orc.mu_dense(A, W, H, 1, float(np.float32(EPS)))
    check(Wg, Hg, Wr, Hr, TOL1)


def test_profile_entry_reports_plan_and_times():
    A, W, H = case(512, 384, 8, 33)
    Wd, Hd = dev(W), dev(H)
    ms = nmf.nmf_mu_dense_profile(dev(A), 512, 384, 8, Wd, Hd, 3, EPS)
    assert len(ms) == 9 and ms[6] == 2.0 and all(x >= 0 for x in ms[:6]) and ms[1] > 0 and ms[4] > 0
    assert ms[7] > 0 and ms[8] > 0
    # the timing launches leave the result alone: same bits as the plain entry point
    Wg, Hg = run_dense(A, W, H, 3)
    np.testing.assert_array_equal(host(Wd), Wg)
    np.testing.assert_array_equal(host(Hd), Hg)


def test_ooc_pageable_host_memory_and_config1():
    A, W, H = config1()
    Wd, Hd = dev(W), dev(H)
    nmf.nmf_mu_ooc(torch.from_numpy(A), 256, 192, 4, Wd, Hd, 100, EPS, 48, 3 * 48 * 192 * 4 + 1024)
    Wr, Hr = orc.mu_dense(A, W, H, 100, float(np.float32(EPS)))
    check(host(Wd), host(Hd), Wr, Hr, TOLN)


def random_ooc_cases(count, seed):
    r = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        m = int(r.integers(1, 900))
        n = int(r.choice([r.integers(1, 600), 4 * r.integers(1, 150)]))
        k = int(r.choice([r.integers(1, 65), r.integers(65, 140), r.choice([16, 32, 64])]))
        batch = int(r.choice([1, r.integers(1, m + 1), r.integers(1, m + 1), m, m + 5]))
        out.append((m, n, k, batch, int(r.integers(1, 4))))
    return out


@pytest.mark.parametrize("m,n,k,batch,slots", random_ooc_cases(16, 2026))
def test_ooc_random_cases_two_iterations(m, n, k, batch, slots):
    """Streamed dense runs with W on the device and with W in host memory, any batch size,
    against the oracle; for ranks up to 64 also the objective of both iterations."""
    A, W, H = case(m, n, k, 2000 + m + n + k)
    eps = float(np.float32(EPS))
    Wr, Hr = orc.mu_dense(A, W, H, 2, eps)
    Ah = torch.from_numpy(A).pin_memory()
    budget = slots * (((min(batch, m) * n * 4) + 255) // 256 * 256)
    Wd, Hd = dev(W), dev(H)
    if k <= 64:
        got = nmf.nmf_mu_ooc_monitor(Ah, m, n, k, Wd, Hd, 2, EPS, batch, budget)
        want = orc.residual_dense(A, Wr, Hr)
        normA2 = float(np.sum(A.astype(np.float64) ** 2))
        assert abs(got[1] - want) <= 1e-5 * want + 3e-7 * normA2 / want
    else:
        nmf.nmf_mu_ooc(Ah, m, n, k, Wd, Hd, 2, EPS, batch, budget)
    check(host(Wd), host(Hd), Wr, Hr, 2 * TOL1 if k <= 64 else 1e-4)
    Wg, Hg, _ = run_hostw(A, W, H, 2, batch, slots)
    check(Wg, Hg, Wr, Hr, 1e-4)


# ---- ranks above 64 (rank-sliced engine) and the host-resident-W pipeline ---------------

@pytest.mark.parametrize("m,n,k,iters", [(300, 200, 65, 1), (515, 260, 100, 1), (257, 1031, 96, 2),
                                         (130, 70, 130, 1), (1000, 520, 70, 5)])
def test_mu_dense_ranks_above_64(m, n, k, iters):
    A, W, H = case(m, n, k, 70)
    Wg, Hg = run_dense(A, W, H, iters)
    Wr, Hr = orc.mu_dense(A, W, H, iters, float(np.float32(EPS)))
    check(Wg, Hg, Wr, Hr, TOL1 if iters == 1 else 1e-4)


def test_mu_dense_rank_256_planted():
    """A larger rank on planted data, several iterations, and determinism."""
    m, n, k = 1536, 1024, 256
    A = nmf_inputs.dense_planted(m, n, 64, seed=1010).numpy()
    W, H = (t.numpy() for t in nmf_inputs.init_factors(m, n, k, seed=2010))
    Wg, Hg = run_dense(A, W, H, 3)
    Wr, Hr = orc.mu_dense(A, W, H, 3, float(np.float32(EPS)))
    check(Wg, Hg, Wr, Hr, 1e-4)
    Wg2, Hg2 = run_dense(A, W, H, 3)
    np.testing.assert_array_equal(Wg, Wg2)
    np.testing.assert_array_equal(Hg, Hg2)


def run_hostw(A, W, H, iters, batch_rows, slots, pinned=True):
    m, n = A.shape
    k = W.shape[1]
    Ah, Wh = torch.from_numpy(np.ascontiguousarray(A)), torch.from_numpy(np.ascontiguousarray(W)).clone()
    if pinned:
        Ah, Wh = Ah.pin_memory(), Wh.pin_memory()
    Hd = dev(H)
    used = nmf.nmf_mu_ooc_hostw(Ah, Wh, m, n, k, Hd, iters, EPS, batch_rows, slots)
    torch.cuda.synchronize()
    return Wh.numpy().astype(np.float64), host(Hd), used


@pytest.mark.parametrize("m,n,k,batch,slots,iters", [
    (256, 192, 4, 48, 3, 3), (300, 200, 40, 64, 1, 2), (300, 200, 40, 64, 2, 2), (300, 200, 40, 301, 4, 2),
    (515, 260, 100, 100, 16, 2), (257, 131, 17, 1, 3, 1), (130, 1027, 33, 50, 2, 1)])
def test_ooc_hostw_matches_oracle(m, n, k, batch, slots, iters):
    A, W, H = case(m, n, k, 80)
    Wg, Hg, used = run_hostw(A, W, H, iters, batch, slots)
    Wr, Hr = orc.mu_dense(A, W, H, iters, float(np.float32(EPS)))
    check(Wg, Hg, Wr, Hr, TOL1 if iters == 1 else 1e-4)
    nb = -(-m // min(batch, m))
    rows = min(batch, m)
    # staging: min(slots, batches) slots of a batch of A and of W; the rest is the workspace
    ws = nmf.nmf_mu_workspace_bytes(6, m, n, 0, k, batch)
    assert used >= ws + min(slots, nb) * rows * (n + k) * 4
    assert used <= ws + min(slots, nb) * (rows * (n + k) * 4 + 512)


def test_ooc_hostw_config1_100_iterations_pageable_memory():
    A, W, H = config1()
    Wg, Hg, _ = run_hostw(A, W, H, 100, 48, 3, pinned=False)
    Wr, Hr = orc.mu_dense(A, W, H, 100, float(np.float32(EPS)))
    check(Wg, Hg, Wr, Hr, TOLN)


def test_ooc_hostw_slot_count_does_not_change_the_result():
    A, W, H = case(700, 300, 48, 81)
    ref = run_hostw(A, W, H, 3, 96, 1)
    for slots in (2, 5, 16):
        got = run_hostw(A, W, H, 3, 96, slots)
        np.testing.assert_array_equal(ref[0], got[0])
        np.testing.assert_array_equal(ref[1], got[1])
        assert got[2] > ref[2] or slots > 8


def test_ooc_device_w_rank_above_64():
    A, W, H = case(515, 260, 100, 82)
    Wd, Hd = dev(W), dev(H)
    Ah = torch.from_numpy(A).pin_memory()
    nmf.nmf_mu_ooc(Ah, 515, 260, 100, Wd, Hd, 2, EPS, 128, 3 * 128 * 260 * 4 + 4096)
    Wr, Hr = orc.mu_dense(A, W, H, 2, float(np.float32(EPS)))
    check(host(Wd), host(Hd), Wr, Hr, 1e-4)
    # same engine, same batches: the host-W pipeline gives the same bits
    Wg, Hg, _ = run_hostw(A, W, H, 2, 128, 3)
    np.testing.assert_array_equal(host(Wd), Wg)
    np.testing.assert_array_equal(host(Hd), Hg)


# ---- CSR path --------------------------------------------------------------------

def run_csr(rowptr, colidx, vals, m, n, W, H, iters):
    k = W.shape[1]
    rp, ci, va = dev(rowptr, torch.int64), dev(colidx, torch.int32), dev(vals)
    rp0, ci0, va0 = rp.clone(), ci.clone(), va.clone()
    Wd, Hd = dev(W), dev(H)
    nmf.nmf_mu_csr(rp, ci, va, m, n, int(vals.size), k, Wd, Hd, iters, EPS)
    Wg, Hg = host(Wd), host(Hd)
    # the CSR structure is read-only: bit-exact after the call
    assert torch.equal(rp, rp0) and torch.equal(ci, ci0) and torch.equal(va, va0)
    return Wg, Hg


@pytest.mark.parametrize("m,n,k,density,iters", [
    (64, 48, 4, 0.3, 3), (500, 700, 32, 0.05, 3), (1000, 300, 17, 0.02, 2),
    (300, 1000, 64, 0.05, 2), (2000, 1500, 33, 0.01, 2), (50, 60, 1, 0.5, 3),
])
def test_csr_matches_oracle(m, n, k, density, iters):
    rowptr, colidx, vals = (t.numpy() for t in nmf_inputs.csr_uniform(m, n, density, seed=90))
    W, H = (t.numpy() for t in nmf_inputs.init_factors(m, n, k, seed=91))
    Wg, Hg = run_csr(rowptr, colidx, vals, m, n, W, H, iters)
    Wr, Hr = orc.mu_csr(rowptr, colidx, vals, m, n, W, H, iters, float(np.float32(EPS)))
    check(Wg, Hg, Wr, Hr, TOL1 * iters)


def test_csr_unsorted_duplicates_empty_rows_equal_dense():
    r = np.random.default_rng(95)
    m, n, k = 90, 70, 5
    A = r.random((m, n), dtype=np.float32)
    A[r.random((m, n)) < 0.7] = 0
    A[10, :] = 0
    A[m - 1, :] = 0
    rows = []
    for i in range(m):
        ent = [(j, float(A[i, j])) for j in range(n) if A[i, j] != 0]
        ent += [(int(j), 0.0) for j in r.integers(0, n, 2)]          # explicit zeros
        if ent and A[i].any():
            j, v = ent[0]
            half = float(np.float32(v * 0.5))
            ent[0] = (j, half)
            ent.append((j, float(np.float32(v) - np.float32(half))))  # duplicate that sums
        if i in (10, m - 1):
            ent = []
        order = r.permutation(len(ent))
        rows.append([ent[t] for t in order])
    rowptr = np.zeros(m + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum([len(x) for x in rows])
    colidx = np.array([j for row in rows for j, _ in row], dtype=np.int32)
    vals = np.array([v for row in rows for _, v in row], dtype=np.float32)
    Adense = np.zeros((m, n), dtype=np.float64)
    for i in range(m):
        for j, v in rows[i]:
            Adense[i, j] += v
    W, H = (t.numpy() for t in nmf_inputs.init_factors(m, n, k, seed=96))
    Wg, Hg = run_csr(rowptr, colidx, vals, m, n, W, H, 3)
    Wr, Hr = orc.mu_dense(Adense.astype(np.float32), W, H, 3, float(np.float32(EPS)))
    check(Wg, Hg, Wr, Hr, 5e-5)
    assert (Wg[10] == 0).all() and (Wg[m - 1] == 0).all()


@pytest.mark.parametrize("m,n,density,scramble", [(300, 500, 0.02, False), (64, 48, 0.3, True),
                                                  (5000, 3000, 0.004, True), (7, 2000, 0.01, False)])
def test_csc_structure_is_bit_exact(m, n, density, scramble):
    """The column-ordered copy (integer work): column pointers, row indices and
    values must equal a stable host sort of the stored entries by column,
    exactly, including unsorted rows, duplicates and empty columns."""
    rowptr, colidx, vals = (t.numpy() for t in nmf_inputs.csr_uniform(m, n, density, seed=93))
    if scramble:
        r = np.random.default_rng(94)
        colidx = colidx.copy(); vals = vals.copy()
        for i in range(m):
            a, b = rowptr[i], rowptr[i + 1]
            p = r.permutation(b - a)
            colidx[a:b] = colidx[a:b][p]
            vals[a:b] = vals[a:b][p]
            if b - a >= 2:
                colidx[a] = colidx[a + 1]          # a repeated (row, column) pair
    nnz = int(vals.size)
    rows = np.repeat(np.arange(m, dtype=np.int32), np.diff(rowptr))
    order = np.argsort(colidx, kind="stable")
    want_rowidx, want_vals = rows[order], vals[order]
    want_colptr = np.zeros(n + 1, dtype=np.int64)
    want_colptr[1:] = np.cumsum(np.bincount(colidx, minlength=n))
    colptr = torch.empty(n + 1, dtype=torch.int64, device="cuda")
    rowidx = torch.empty(nnz, dtype=torch.int32, device="cuda")
    cvals = torch.empty(nnz, dtype=torch.float32, device="cuda")
    nmf.nmf_csr_to_csc(dev(rowptr, torch.int64), dev(colidx, torch.int32), dev(vals), m, n, nnz,
                       colptr, rowidx, cvals)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(colptr.cpu().numpy(), want_colptr)
    np.testing.assert_array_equal(rowidx.cpu().numpy(), want_rowidx)
    np.testing.assert_array_equal(cvals.cpu().numpy(), want_vals)


@pytest.mark.parametrize("m,nparts,kind", [(5000, 64, "uniform"), (5000, 16384, "uniform"), (300, 7, "skewed"),
                                           (1, 4, "uniform"), (4000, 100, "empty")])
def test_csr_partition_table_is_bit_exact(m, nparts, kind):
    """Row ranges of equal work (integer work): the table must equal a host
    bisection of key(r) = rowptr[r] + 8 r exactly."""
    r = np.random.default_rng(m + nparts)
    if kind == "uniform":
        counts = r.poisson(20, m)
    elif kind == "skewed":
        counts = (r.pareto(1.0, m) * 5).astype(np.int64)
        counts[17] = 50000
    else:
        counts = np.zeros(m, dtype=np.int64)
    rowptr = np.zeros(m + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum(counts)
    key = rowptr + 8 * np.arange(m + 1)
    share = -(-int(key[m]) // nparts)
    want = np.searchsorted(key, np.arange(nparts + 1) * share, side="left").astype(np.int64)
    want = np.minimum(want, m)
    want[nparts] = m
    part = torch.empty(nparts + 1, dtype=torch.int64, device="cuda")
    nmf.nmf_csr_partition(dev(rowptr, torch.int64), m, nparts, part)
    torch.cuda.synchronize()
    got = part.cpu().numpy()
    np.testing.assert_array_equal(got, want)
    assert got[0] == 0 and got[-1] == m and (np.diff(got) >= 0).all()


def test_csr_skewed_rows_and_a_very_long_row():
    """Power-law row lengths plus rows above the long-row threshold (handled by
    a whole workgroup) and a long column, against the oracle."""
    r = np.random.default_rng(77)
    m, n, k = 400, 30000, 32
    counts = np.minimum((r.pareto(1.2, m) * 8).astype(np.int64), n)
    counts[5] = 20000            # long rows
    counts[123] = 17000
    counts[124] = 0
    rows = []
    for i in range(m):
        rows.append(np.sort(r.choice(n, int(counts[i]), replace=False)).astype(np.int32))
    rowptr = np.zeros(m + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum(counts)
    colidx = np.concatenate(rows)
    vals = (1.0 - r.random(colidx.size, dtype=np.float32)).astype(np.float32)
    W, H = (t.numpy() for t in nmf_inputs.init_factors(m, n, k, seed=78))
    Wg, Hg = run_csr(rowptr, colidx, vals, m, n, W, H, 2)
    Wr, Hr = orc.mu_csr(rowptr, colidx, vals, m, n, W, H, 2, float(np.float32(EPS)))
    check(Wg, Hg, Wr, Hr, 2 * TOL1)
    # transposed problem: long columns of A become long rows of the column-ordered copy
    import scipy.sparse as sp
    At = sp.csr_matrix((vals, colidx, rowptr), shape=(m, n)).T.tocsr()
    At.sort_indices()
    Wt, Ht = (t.numpy() for t in nmf_inputs.init_factors(n, m, k, seed=79))
    Wg, Hg = run_csr(At.indptr.astype(np.int64), At.indices.astype(np.int32), At.data.astype(np.float32), n, m, Wt, Ht, 2)
    Wr, Hr = orc.mu_csr(At.indptr.astype(np.int64), At.indices.astype(np.int32), At.data.astype(np.float32), n, m, Wt, Ht, 2, float(np.float32(EPS)))
    check(Wg, Hg, Wr, Hr, 2 * TOL1)


def run_csr_ooc(rowptr, colidx, vals, m, n, W, H, iters, batch_nnz, budget=1 << 30, pinned=True):
    k = W.shape[1]
    rp = torch.from_numpy(np.ascontiguousarray(rowptr, dtype=np.int64))
    ci = torch.from_numpy(np.ascontiguousarray(colidx, dtype=np.int32))
    va = torch.from_numpy(np.ascontiguousarray(vals, dtype=np.float32))
    if pinned:
        rp, ci, va = rp.pin_memory(), ci.pin_memory(), va.pin_memory()
    Wd, Hd = dev(W), dev(H)
    nmf.nmf_mu_csr_ooc(rp, ci, va, m, n, int(vals.size), k, Wd, Hd, iters, EPS, batch_nnz, budget)
    Wg, Hg = host(Wd), host(Hd)
    assert np.array_equal(rp.numpy(), rowptr) and np.array_equal(ci.numpy(), colidx) and np.array_equal(va.numpy(), vals)
    return Wg, Hg


@pytest.mark.parametrize("m,n,k,density,iters,batch_nnz", [
    (64, 48, 4, 0.3, 3, 100), (500, 700, 32, 0.05, 3, 3000), (1000, 300, 17, 0.02, 2, 1),
    (300, 1000, 64, 0.05, 2, 10 ** 9), (2000, 1500, 33, 0.01, 2, 7777), (50, 60, 1, 0.5, 3, 64),
])
def test_csr_ooc_matches_oracle(m, n, k, density, iters, batch_nnz):
    rowptr, colidx, vals = (t.numpy() for t in nmf_inputs.csr_uniform(m, n, density, seed=m + n))
    W, H = (t.numpy() for t in nmf_inputs.init_factors(m, n, k, seed=m + n + 1))
    Wg, Hg = run_csr_ooc(rowptr, colidx, vals, m, n, W, H, iters, batch_nnz)
    Wr, Hr = orc.mu_csr(rowptr, colidx, vals, m, n, W, H, iters, float(np.float32(EPS)))
    check(Wg, Hg, Wr, Hr, 1e-4 if iters > 1 else TOL1)


def test_csr_ooc_one_batch_equals_resident_csr_bitwise_and_slots_do_not_matter():
    rowptr, colidx, vals = (t.numpy() for t in nmf_inputs.csr_uniform(1500, 900, 0.02, seed=61))
    W, H = (t.numpy() for t in nmf_inputs.init_factors(1500, 900, 24, seed=62))
    # several batches: the staging budget (1, 2 or 3 slots) does not change a bit
    per_slot = 8 * 1501 + 8 * 5000 + 1024
    ref = run_csr_ooc(rowptr, colidx, vals, 1500, 900, W, H, 3, 4000, budget=per_slot)
    for slots in (2, 3):
        got = run_csr_ooc(rowptr, colidx, vals, 1500, 900, W, H, 3, 4000, budget=slots * per_slot, pinned=slots == 2)
        np.testing.assert_array_equal(ref[0], got[0])
        np.testing.assert_array_equal(ref[1], got[1])
    # one batch holding everything: the same sums in the same order as the resident CSR path
    one = run_csr_ooc(rowptr, colidx, vals, 1500, 900, W, H, 3, 10 ** 9)
    res = run_csr(rowptr, colidx, vals, 1500, 900, W, H, 3)
    np.testing.assert_array_equal(one[0], res[0])
    np.testing.assert_array_equal(one[1], res[1])


def test_csr_ooc_skewed_rows_long_row_empty_rows_and_duplicates():
    r = np.random.default_rng(91)
    m, n, k = 300, 30000, 32
    counts = np.minimum((r.pareto(1.2, m) * 8).astype(np.int64), n)
    counts[7] = 20000            # above the long-row threshold: a batch of its own at batch_nnz = 5000
    counts[8] = 0
    counts[299] = 0              # the matrix ends in an empty row
    rows = [np.sort(r.choice(n, int(c), replace=False)).astype(np.int32) for c in counts]
    rows[3] = np.concatenate([rows[3], rows[3][:2]]) if rows[3].size >= 2 else rows[3]      # repeated (row, column)
    counts[3] = rows[3].size
    rowptr = np.zeros(m + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum(counts)
    colidx = np.concatenate(rows).astype(np.int32)
    vals = (1.0 - r.random(colidx.size, dtype=np.float32)).astype(np.float32)
    W, H = (t.numpy() for t in nmf_inputs.init_factors(m, n, k, seed=92))
    Wg, Hg = run_csr_ooc(rowptr, colidx, vals, m, n, W, H, 2, 5000)
    Wr, Hr = orc.mu_csr(rowptr, colidx, vals, m, n, W, H, 2, float(np.float32(EPS)))
    check(Wg, Hg, Wr, Hr, 2 * TOL1)
    assert (Wg[8] == 0).all() and (Wg[299] == 0).all()


def test_csr_ooc_argument_errors():
    rp = torch.tensor([0, 1, 3], dtype=torch.int64)
    ci = torch.tensor([0, 1, 2], dtype=torch.int32)
    va = torch.ones(3)
    W, H = torch.ones((2, 2), device="cuda"), torch.ones((2, 3), device="cuda")
    with pytest.raises(nmf.NmfError) as e:
        nmf.nmf_mu_csr_ooc(rp, ci, va, 2, 3, 4, 2, W, H, 1, EPS, 10, 1 << 20)       # rowptr[m] != nnz
    assert e.value.status == nmf.NMF_EINVAL
    with pytest.raises(nmf.NmfError) as e:
        nmf.nmf_mu_csr_ooc(rp, ci, va, 2, 3, 3, 2, W, H, 1, EPS, 10, 8)             # budget below one batch
    assert e.value.status == nmf.NMF_ENOMEM


def test_csr_is_reproducible_run_to_run():
    rowptr, colidx, vals = (t.numpy() for t in nmf_inputs.csr_uniform(3000, 2000, 0.01, seed=98))
    W, H = (t.numpy() for t in nmf_inputs.init_factors(3000, 2000, 32, seed=99))
    W1, H1 = run_csr(rowptr, colidx, vals, 3000, 2000, W, H, 3)
    W2, H2 = run_csr(rowptr, colidx, vals, 3000, 2000, W, H, 3)
    np.testing.assert_array_equal(W1, W2)
    np.testing.assert_array_equal(H1, H2)


def test_csr_empty_matrix():
    m, n, k = 20, 30, 3
    rowptr = np.zeros(m + 1, dtype=np.int64)
    W, H = (t.numpy() for t in nmf_inputs.init_factors(m, n, k, seed=97))
    rp = dev(rowptr, torch.int64)
    ci = torch.empty(0, dtype=torch.int32, device="cuda")
    va = torch.empty(0, dtype=torch.float32, device="cuda")
    Wd, Hd = dev(W), dev(H)
    L = nmf.lib()
    rc = L.nmf_mu_csr(rp.data_ptr(), None, None, m, n, 0, k, Wd.data_ptr(), Hd.data_ptr(), 2, EPS, None)
    assert rc == 0
    assert (host(Wd) == 0).all() and (host(Hd) == 0).all()
    del ci, va


def random_csr_cases(count, seed):
    r = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        m = int(r.choice([r.integers(1, 50), r.integers(50, 3000)]))
        n = int(r.choice([r.integers(1, 50), r.integers(50, 3000)]))
        k = int(r.choice([r.integers(1, 65), r.choice([1, 3, 4, 5, 8, 16, 17, 32, 33, 64])]))
        density = float(r.choice([0.0005, 0.005, 0.05, 0.5]))
        out.append((m, n, k, density))
    return out


@pytest.mark.parametrize("m,n,k,density", random_csr_cases(16, 2025))
def test_csr_random_cases_two_iterations_with_objective(m, n, k, density):
    rowptr, colidx, vals = (t.numpy() for t in nmf_inputs.csr_uniform(m, n, density, seed=m + 3 * n + k))
    W, H = (t.numpy() for t in nmf_inputs.init_factors(m, n, k, seed=5 * m + n + k))
    eps = float(np.float32(EPS))
    Wr, Hr = orc.mu_csr(rowptr, colidx, vals, m, n, W, H, 2, eps)
    Wd, Hd = dev(W), dev(H)
    got = nmf.nmf_mu_csr_monitor(dev(rowptr, torch.int64), dev(colidx, torch.int32), dev(vals), m, n, int(vals.size),
                                 k, Wd, Hd, 2, EPS)
    check(host(Wd), host(Hd), Wr, Hr, 2 * TOL1)
    want = orc.residual_csr(rowptr, colidx, vals, m, n, Wr, Hr)
    normA2 = float(np.sum(vals.astype(np.float64) ** 2))
    if want > 0:
        assert abs(got[1] - want) <= 1e-5 * want + 3e-7 * normA2 / want
    else:
        assert got[1] == 0.0


def csr_monitor_case(rowptr, colidx, vals, m, n, W, H, iters):
    """Monitored sparse run against the oracle's trajectory (objective over all m n entries,
    from the dense copy of A) and against the plain run (same bits)."""
    import scipy.sparse as sp
    k = W.shape[1]
    Ad = np.asarray(sp.csr_matrix((vals, colidx, rowptr), shape=(m, n)).todense(), dtype=np.float32)
    eps = float(np.float32(EPS))
    want, Wr, Hr = [], W, H
    for _ in range(iters):
        Wr, Hr = orc.mu_csr(rowptr, colidx, vals, m, n, Wr, Hr, 1, eps)
        want.append(orc.residual_dense(Ad, Wr, Hr))
    want = np.array(want)
    Wd, Hd = dev(W), dev(H)
    got = np.array(nmf.nmf_mu_csr_monitor(dev(rowptr, torch.int64), dev(colidx, torch.int32), dev(vals), m, n,
                                          int(vals.size), k, Wd, Hd, iters, EPS))
    normA2 = float(np.sum(Ad.astype(np.float64) ** 2))
    bound = np.maximum(1e-5 * want, 3e-7 * normA2 / np.maximum(want, 1e-300))
    assert (np.abs(got - want) <= bound).all(), (got, want)
    Wg, Hg = run_csr(rowptr, colidx, vals, m, n, W, H, iters)
    np.testing.assert_array_equal(host(Wd), Wg)
    np.testing.assert_array_equal(host(Hd), Hg)


@pytest.mark.parametrize("m,n,k,density,iters", [
    (64, 48, 4, 0.3, 6), (500, 700, 32, 0.05, 4), (300, 1000, 64, 0.05, 3), (2000, 1500, 33, 0.01, 3),
])
def test_csr_monitor_reports_the_objective_of_every_iteration(m, n, k, density, iters):
    rowptr, colidx, vals = (t.numpy() for t in nmf_inputs.csr_uniform(m, n, density, seed=190))
    W, H = (t.numpy() for t in nmf_inputs.init_factors(m, n, k, seed=191))
    csr_monitor_case(rowptr, colidx, vals, m, n, W, H, iters)


def test_csr_monitor_with_long_rows_and_empty_rows():
    """Rows above the long-row threshold are finished by another kernel, which reports its own
    share of <A H^T, W>."""
    r = np.random.default_rng(177)
    m, n, k = 300, 30000, 16
    counts = np.minimum((r.pareto(1.2, m) * 8).astype(np.int64), n)
    counts[7] = 21000
    counts[200] = 16500
    counts[201] = 0
    rows = [np.sort(r.choice(n, int(c), replace=False)).astype(np.int32) for c in counts]
    rowptr = np.zeros(m + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum(counts)
    colidx = np.concatenate(rows)
    vals = (1.0 - r.random(colidx.size, dtype=np.float32)).astype(np.float32)
    W, H = (t.numpy() for t in nmf_inputs.init_factors(m, n, k, seed=178))
    csr_monitor_case(rowptr, colidx, vals, m, n, W, H, 3)


def csr_with_repeated_entries(m, n, density, seed):
    """A CSR matrix in which about a third of the stored positions appear two or three times
    (the parts add up to the entry), the entries of a row in shuffled order."""
    r = np.random.default_rng(seed)
    Ad = (r.random((m, n)) * (r.random((m, n)) < density)).astype(np.float32)
    rows = []
    for i in range(m):
        ent = []
        for j in np.nonzero(Ad[i])[0]:
            v = np.float32(Ad[i, j])
            parts = int(r.integers(1, 4)) if r.random() < 0.35 else 1
            cut = [np.float32(v * f) for f in r.dirichlet(np.ones(parts))] if parts > 1 else [v]
            ent += [(int(j), float(c)) for c in cut]
        order = r.permutation(len(ent))
        rows.append([ent[t] for t in order])
    rowptr = np.zeros(m + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum([len(x) for x in rows])
    colidx = np.array([j for row in rows for j, _ in row], dtype=np.int32)
    vals = np.array([v for row in rows for _, v in row], dtype=np.float32)
    return rowptr, colidx, vals


def test_csr_monitor_and_tol_with_repeated_entries():
    """Repeated (row, column) pairs stand for their sum: ||A||^2 in the objective's expansion is
    that of the summed matrix, not the sum of the squared stored values (which is smaller here by
    a tenth), in the reported objectives and in the stopping decision."""
    import scipy.sparse as sp
    m, n, k = 400, 300, 8
    rowptr, colidx, vals = csr_with_repeated_entries(m, n, 0.08, 77)
    Ad = np.asarray(sp.csr_matrix((vals, colidx, rowptr), shape=(m, n)).todense(), dtype=np.float32)
    assert np.sum(vals.astype(np.float64) ** 2) < 0.95 * np.sum(Ad.astype(np.float64) ** 2)
    W, H = (t.numpy() for t in nmf_inputs.init_factors(m, n, k, seed=78))
    csr_monitor_case(rowptr, colidx, vals, m, n, W, H, 5)
    eps = float(np.float32(EPS))
    traj, Wr, Hr = [orc.residual_dense(Ad, W, H)], W, H
    for _ in range(12):
        Wr, Hr = orc.mu_csr(rowptr, colidx, vals, m, n, Wr, Hr, 1, eps)
        traj.append(orc.residual_dense(Ad, Wr, Hr))
    assert traj[7] < traj[6]
    tol = 0.5 * (traj[6] + traj[7])
    Wd, Hd = dev(W), dev(H)
    done, res = nmf.nmf_mu_csr_tol(dev(rowptr, torch.int64), dev(colidx, torch.int32), dev(vals), m, n,
                                   int(vals.size), k, Wd, Hd, 100, EPS, tol, 1)
    assert done == 7
    assert abs(res - traj[7]) <= 1e-4 * traj[7]


@pytest.mark.parametrize("m,n,k,density,every", [(500, 700, 32, 0.05, 2), (300, 30000, 16, 0.002, 1)])
def test_csr_tol_matches_algorithm_1_loop(m, n, k, density, every):
    rowptr, colidx, vals = (t.numpy() for t in nmf_inputs.csr_uniform(m, n, density, seed=290))
    W, H = (t.numpy() for t in nmf_inputs.init_factors(m, n, k, seed=291))
    eps = float(np.float32(EPS))
    nnz = int(vals.size)
    traj = [orc.residual_csr(rowptr, colidx, vals, m, n, W, H)]
    Wt, Ht = W, H
    for _ in range(6):
        Wt, Ht = orc.mu_csr(rowptr, colidx, vals, m, n, Wt, Ht, every, eps)
        traj.append(orc.residual_csr(rowptr, colidx, vals, m, n, Wt, Ht))
    gap = traj[3] - traj[4]
    normA2 = float(np.sum(vals.astype(np.float64) ** 2))
    assert gap > 50 * 3e-7 * normA2 / traj[4]      # the two checks around the tolerance are far apart for the expansion
    tol = 0.5 * (traj[3] + traj[4])                # first met at the 4th check after the start
    Wr, Hr, done_r, res_r = orc.mu_csr_tol(rowptr, colidx, vals, m, n, W, H, 1000, eps, tol, check_every=every)
    rp, ci, va = dev(rowptr, torch.int64), dev(colidx, torch.int32), dev(vals)
    Wd, Hd = dev(W), dev(H)
    done, res = nmf.nmf_mu_csr_tol(rp, ci, va, m, n, nnz, k, Wd, Hd, 1000, EPS, tol, every)
    assert done == done_r == 4 * every
    assert abs(res - res_r) <= 1e-5 * res_r + 3e-7 * normA2 / res_r and res <= tol
    check(host(Wd), host(Hd), Wr, Hr, TOL1 * done)
    # the stopped run is the plain run of that many iterations, bit for bit
    Wg, Hg = run_csr(rowptr, colidx, vals, m, n, W, H, done)
    np.testing.assert_array_equal(host(Wd), Wg)
    np.testing.assert_array_equal(host(Hd), Hg)
    # cap reached / tolerance already met / no iterations allowed
    Wd, Hd = dev(W), dev(H)
    done, res = nmf.nmf_mu_csr_tol(rp, ci, va, m, n, nnz, k, Wd, Hd, 3, EPS, 0.0, 2)
    assert done == 3
    Wg, Hg = run_csr(rowptr, colidx, vals, m, n, W, H, 3)
    np.testing.assert_array_equal(host(Wd), Wg)
    Wd, Hd = dev(W), dev(H)
    done, res = nmf.nmf_mu_csr_tol(rp, ci, va, m, n, nnz, k, Wd, Hd, 7, EPS, 1e9, 2)
    assert done == 0 and abs(res - traj[0]) <= 1e-5 * traj[0]
    np.testing.assert_array_equal(host(Wd), W.astype(np.float64))
    np.testing.assert_array_equal(host(Hd), H.astype(np.float64))
    Wd, Hd = dev(W), dev(H)
    done, res = nmf.nmf_mu_csr_tol(rp, ci, va, m, n, nnz, k, Wd, Hd, 0, EPS, 0.0, 1)
    assert done == 0 and abs(res - traj[0]) <= 1e-5 * traj[0]


def test_csr_monitor_empty_matrix():
    m, n, k = 20, 30, 3
    W, H = (t.numpy() for t in nmf_inputs.init_factors(m, n, k, seed=97))
    Wd, Hd = dev(W), dev(H)
    out = (ctypes.c_double * 2)(7.0, 7.0)
    rc = nmf.lib().nmf_mu_csr_monitor(dev(np.zeros(m + 1, dtype=np.int64), torch.int64).data_ptr(), None, None, m, n, 0,
                                      k, Wd.data_ptr(), Hd.data_ptr(), 2, EPS, out, None)
    assert rc == 0 and list(out) == [0.0, 0.0]
    assert (host(Wd) == 0).all() and (host(Hd) == 0).all()


# ---- ensemble ----------------------------------------------------------------------

def test_batched_matches_loop_of_oracle_runs():
    m, n = 384, 256
    base = nmf_inputs.dense_planted(m, n, 8, seed=1005)
    copies = [nmf_inputs.perturb(base, 3000 + p) for p in range(2)]
    ks = [2, 3, 8, 16, 5]
    As, Ws, Hs = [], [], []
    for r, k in enumerate(ks):
        As.append(copies[r % 2])
        W, H = nmf_inputs.init_factors(m, n, k, seed=2005 + r)
        Ws.append(W)
        Hs.append(H)
    dA = [a.cuda() for a in copies]
    Ad = [dA[r % 2] for r in range(len(ks))]
    Wd = [w.cuda() for w in Ws]
    Hd = [h.cuda() for h in Hs]
    nmf.nmf_mu_dense_batched(len(ks), Ad, m, n, ks, Wd, Hd, 20, EPS)
    ref = orc.mu_ensemble([a.numpy() for a in As], [w.numpy() for w in Ws], [h.numpy() for h in Hs], 20,
                          float(np.float32(EPS)))
    for r in range(len(ks)):
        check(host(Wd[r]), host(Hd[r]), ref[r][0], ref[r][1], 2e-4)


def test_batched_stacks_runs_that_share_a():
    """Copies outer, ranks inner: consecutive runs share A and are stacked
    (34 = 2+3+8+16+5 in one stack, then 33 and 40 alone, per copy)."""
    m, n = 384, 256
    base = nmf_inputs.dense_planted(m, n, 8, seed=1005)
    copies = [nmf_inputs.perturb(base, 3100 + p) for p in range(2)]
    dA = [a.cuda() for a in copies]
    ks_one = [2, 3, 8, 16, 5, 33, 40]
    As, Ad, ks, Ws, Hs = [], [], [], [], []
    for p in range(2):
        for k in ks_one:
            W, H = nmf_inputs.init_factors(m, n, k, seed=2105 + len(ks))
            As.append(copies[p]); Ad.append(dA[p]); ks.append(k); Ws.append(W); Hs.append(H)
    Wd = [w.cuda() for w in Ws]
    Hd = [h.cuda() for h in Hs]
    nmf.nmf_mu_dense_batched(len(ks), Ad, m, n, ks, Wd, Hd, 20, EPS)
    worst = 0.0
    ref = orc.mu_ensemble([a.numpy() for a in As], [w.numpy() for w in Ws], [h.numpy() for h in Hs], 20,
                          float(np.float32(EPS)))
    for r in range(len(ks)):
        worst = max(worst, check(host(Wd[r]), host(Hd[r]), ref[r][0], ref[r][1], 2e-4))
    # one iteration, tight bar
    Wd = [w.cuda() for w in Ws]
    Hd = [h.cuda() for h in Hs]
    nmf.nmf_mu_dense_batched(len(ks), Ad, m, n, ks, Wd, Hd, 1, EPS)
    for r in range(len(ks)):
        Wr, Hr = orc.mu_dense(As[r].numpy(), Ws[r].numpy(), Hs[r].numpy(), 1, float(np.float32(EPS)))
        check(host(Wd[r]), host(Hd[r]), Wr, Hr, TOL1)


# ---- workspace handling -----------------------------------------------------------------

def test_caller_workspace_and_release():
    A, W, H = case(300, 200, 4, 100)
    Wref, Href = run_dense(A, W, H, 2)
    need = nmf.nmf_mu_workspace_bytes(0, 300, 200, 0, 4, 0)
    buf = torch.empty(need, dtype=torch.uint8, device="cuda")
    nmf.nmf_mu_set_workspace(buf)
    try:
        Wg, Hg = run_dense(A, W, H, 2)
        np.testing.assert_array_equal(Wg, Wref)
        np.testing.assert_array_equal(Hg, Href)
        with pytest.raises(nmf.NmfError) as ei:
            run_dense(*case(3000, 2000, 32, 101), 1)
        assert ei.value.status == nmf.NMF_ENOMEM
    finally:
        nmf.nmf_mu_set_workspace(None)
    nmf.nmf_mu_release()
    Wg, Hg = run_dense(A, W, H, 2)
    np.testing.assert_array_equal(Wg, Wref)
