"""Host-side checks that need no GPU: the shared library loads, exports every
symbol the public header declares, and the pure host helpers behave."""
import ctypes
import os
import re

import pytest

import paper_2202_09518_amd as nmf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    inc = os.path.join(ROOT, "include")
    for fn in os.listdir(inc):
        if fn.endswith(".h"):
            text = open(os.path.join(inc, fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(nmf_\w+)\s*\(", text))
    return sorted(names)


def symbols_of(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(nmf_\w+)\s*\(", text)))


def test_public_header_holds_the_boundary_and_nothing_else():
    """nmfmu.h: status reporting, the four method calls and the workspace calls of the boundary,
    the entry points of the next steps (objective and stopping rule, host-resident W, streamed
    CSR) and the allocation-free variant; the single steps that tests and profiling use live in
    nmfmu_test.h."""
    boundary = ["nmf_status_string", "nmf_last_error", "nmf_mu_dense", "nmf_mu_csr", "nmf_mu_ooc",
                "nmf_mu_dense_batched", "nmf_mu_workspace_bytes", "nmf_mu_set_workspace", "nmf_mu_release"]
    next_steps = ["nmf_residual_dense", "nmf_mu_dense_tol", "nmf_mu_dense_monitor", "nmf_mu_csr_monitor",
                  "nmf_mu_csr_tol", "nmf_mu_ooc_monitor", "nmf_mu_ooc_hostw", "nmf_mu_csr_ooc"]
    assert symbols_of("nmfmu.h") == sorted(boundary + next_steps + ["nmf_mu_dense_noalloc"])
    assert symbols_of("nmfmu_test.h") == sorted(
        ["nmf_mu_dense_profile", "nmf_gram_w", "nmf_wta_dense", "nmf_h_update", "nmf_aht_w_update_dense",
         "nmf_split_planes", "nmf_csr_partition", "nmf_csr_to_csc"])


def test_library_exports_every_declared_symbol():
    L = nmf.lib()
    decl = declared_symbols()
    assert len(decl) >= 13
    for name in decl:
        assert hasattr(L, name), name
    assert sorted(nmf.EXPORTS) == decl


def test_binding_has_the_same_names():
    for name in declared_symbols():
        assert callable(getattr(nmf, name)), name


def test_status_strings():
    assert nmf.nmf_status_string(0) == "NMF_OK"
    assert nmf.nmf_status_string(1) == "NMF_EINVAL"
    assert nmf.nmf_status_string(2) == "NMF_ENOMEM"
    assert nmf.nmf_status_string(3) == "NMF_EHIP"
    assert nmf.nmf_status_string(4) == "NMF_EUNSUPPORTED"
    assert nmf.nmf_status_string(99) == "NMF_UNKNOWN"


def test_max_k_matches_header():
    text = open(os.path.join(ROOT, "include", "nmfmu.h")).read()
    assert int(re.search(r"#define NMF_MU_MAX_K (\d+)", text).group(1)) == nmf.NMF_MU_MAX_K


def test_workspace_bytes():
    wb = nmf.nmf_mu_workspace_bytes
    assert wb(0, 0, 10, 0, 4, 0) == 0          # invalid m
    assert wb(0, 10, 10, 0, 65, 0) == 0        # k too large
    assert wb(7, 10, 10, 0, 4, 0) == 0         # unknown kind
    assert wb(2, 10, 10, 0, 4, 0) == 0         # ooc needs batch_rows
    d = wb(4, 32768, 16384, 0, 32, 0)
    # small plan: 4 row splits of a 32 x 16384 fp32 partial, the bf16 piece planes of W and of
    # H^T (3 pieces x 64 factor slots x 16 bytes per group of 8 rows) and the Gram scratch
    base = 4 * 32 * 16384 * 4 + ((32768 + 16384) // 8) * 3 * 64 * 16
    assert base <= d <= base + (4 << 20)
    # fast plan: additionally A^T, W^T and H^T
    extra = (32768 * 16384 + 32 * 32768 + 16384 * 32) * 4
    assert d + extra <= wb(0, 32768, 16384, 0, 32, 0) <= d + extra + (1 << 20)
    assert wb(1, 1000, 5000, 123, 8, 0) >= 2 * 5000 * 8 * 4
    assert wb(2, 262144, 65536, 0, 64, 8192) == wb(4, 8192, 65536, 0, 64, 0)
    # rank-sliced plans: A^T, W^T, H^T and two k x max(m, n) arrays at least / the batch versions
    assert wb(5, 1000, 600, 0, 1025, 0) == 0
    assert wb(5, 1000, 600, 0, 100, 0) >= (1000 * 600 + 2 * 100 * 1000 + 100 * 1000 + 600 * 100) * 4
    assert wb(6, 1000, 600, 0, 100, 0) == 0     # needs batch_rows
    assert wb(6, 1000, 600, 0, 100, 128) >= (600 * 128 + 3 * 100 * 128 + 2 * 100 * 600) * 4
    assert wb(6, 1000, 600, 0, 100, 128) < wb(5, 1000, 600, 0, 100, 0)


def test_argument_errors_need_no_device():
    """Argument validation happens before any HIP call."""
    L = nmf.lib()
    one = ctypes.c_void_p(16)
    null = ctypes.c_void_p(0)
    assert L.nmf_mu_dense(null, 4, 4, 2, one, one, 1, 1e-16, null) == nmf.NMF_EINVAL
    assert L.nmf_mu_dense(one, 0, 4, 2, one, one, 1, 1e-16, null) == nmf.NMF_EINVAL
    assert L.nmf_mu_dense(one, 4, 4, 0, one, one, 1, 1e-16, null) == nmf.NMF_EINVAL
    assert L.nmf_mu_dense(one, 4, 4, 1025, one, one, 1, 1e-16, null) == nmf.NMF_EUNSUPPORTED
    assert L.nmf_mu_csr(one, one, one, 4, 4, 3, 65, one, one, 1, 1e-16, null) == nmf.NMF_EUNSUPPORTED
    assert L.nmf_mu_ooc_hostw(one, one, 4, 4, 2, one, 1, 1e-16, 2, 0, null, null) == nmf.NMF_EINVAL
    assert L.nmf_mu_ooc_hostw(one, one, 4, 4, 2, one, 1, 1e-16, 2, 17, null, null) == nmf.NMF_EINVAL
    assert L.nmf_mu_ooc_hostw(one, null, 4, 4, 2, one, 1, 1e-16, 2, 2, null, null) == nmf.NMF_EINVAL
    assert L.nmf_mu_ooc_hostw(one, one, 4, 4, 2, one, 0, 1e-16, 2, 2, null, null) == nmf.NMF_OK
    assert L.nmf_mu_dense(one, 4, 4, 2, one, one, -1, 1e-16, null) == nmf.NMF_EINVAL
    assert L.nmf_mu_dense(one, 4, 4, 2, one, one, 1, -1.0, null) == nmf.NMF_EINVAL
    assert L.nmf_mu_dense(one, 4, 4, 2, one, one, 1, float("nan"), null) == nmf.NMF_EINVAL
    assert L.nmf_mu_dense(one, 4, 4, 2, one, one, 1, float("inf"), null) == nmf.NMF_EINVAL
    assert L.nmf_mu_dense(one, 4, 4, 2, one, one, 0, 1e-16, null) == nmf.NMF_OK   # iters = 0
    assert nmf.nmf_last_error() != ""
    assert L.nmf_mu_ooc(one, 4, 4, 2, one, one, 1, 1e-16, 0, 1 << 20, null) == nmf.NMF_EINVAL
    assert L.nmf_mu_ooc(one, 4, 4, 2, one, one, 1, 1e-16, 2, 0, null) == nmf.NMF_EINVAL
    assert L.nmf_mu_ooc(one, 4, 4, 2, one, one, 1, 1e-16, 2, 8, null) == nmf.NMF_ENOMEM
    assert L.nmf_mu_ooc_monitor(one, 4, 4, 2, one, one, 1, 1e-16, 2, 1 << 20, null, null) == nmf.NMF_EINVAL
    assert L.nmf_mu_ooc_monitor(one, 4, 4, 2, one, one, 1, 1e-16, 0, 1 << 20, one, null) == nmf.NMF_EINVAL
    assert L.nmf_mu_ooc_monitor(one, 4, 4, 70, one, one, 1, 1e-16, 2, 1 << 20, one, null) == nmf.NMF_EUNSUPPORTED
    assert L.nmf_mu_csr(null, one, one, 4, 4, 3, 2, one, one, 1, 1e-16, null) == nmf.NMF_EINVAL
    assert L.nmf_mu_csr(one, null, one, 4, 4, 3, 2, one, one, 1, 1e-16, null) == nmf.NMF_EINVAL
    assert L.nmf_mu_csr(one, one, one, 4, 4, -1, 2, one, one, 1, 1e-16, null) == nmf.NMF_EINVAL
    assert L.nmf_mu_csr_monitor(one, one, one, 4, 4, 3, 2, one, one, 1, 1e-16, null, null) == nmf.NMF_EINVAL
    assert L.nmf_mu_csr_monitor(null, one, one, 4, 4, 3, 2, one, one, 1, 1e-16, one, null) == nmf.NMF_EINVAL
    assert L.nmf_mu_csr_monitor(one, one, one, 4, 4, 3, 2, one, one, (1 << 20) + 1, 1e-16, one, null) == nmf.NMF_EINVAL
    assert L.nmf_mu_csr_tol(one, one, one, 4, 4, 3, 2, one, one, 5, 1e-16, 0.1, 1, null, one, null) == nmf.NMF_EINVAL
    assert L.nmf_mu_csr_tol(one, one, one, 4, 4, 3, 2, one, one, 5, 1e-16, 0.1, 0, one, one, null) == nmf.NMF_EINVAL
    assert L.nmf_mu_csr_tol(one, one, one, 4, 4, 3, 2, one, one, 5, 1e-16, -1.0, 1, one, one, null) == nmf.NMF_EINVAL
    assert L.nmf_mu_csr_tol(one, one, one, 4, 4, 3, 2, one, one, 5, 1e-16, float("nan"), 1, one, one, null) == nmf.NMF_EINVAL
    assert L.nmf_mu_dense_batched(-1, one, 4, 4, one, one, one, 1, 1e-16, null) == nmf.NMF_EINVAL
    assert L.nmf_mu_set_workspace(ctypes.c_void_p(8), 4096) == nmf.NMF_EINVAL   # misaligned


def test_missing_library_fails_loudly(monkeypatch):
    import paper_2202_09518_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "LIB_PATH", "/nonexistent/libnmfmu.so")
    with pytest.raises(ImportError):
        b.lib()
