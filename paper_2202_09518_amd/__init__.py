"""MI355X-native multiplicative-update NMF (dense, CSR, out-of-memory, ensemble).

The work is done by hand-written HIP kernels in ``libnmfmu.so`` (C ABI in
``include/nmfmu.h``); this package is the argument-marshalling layer only.
"""
from .binding import (  # noqa: F401
    EXPORTS, LIB_PATH, NMF_MU_MAX_K, NMF_MU_MAX_K_SLICED, NmfError, lib,
    NMF_OK, NMF_EINVAL, NMF_ENOMEM, NMF_EHIP, NMF_EUNSUPPORTED,
    nmf_status_string, nmf_last_error,
    nmf_mu_dense, nmf_mu_dense_noalloc, nmf_mu_dense_profile, nmf_residual_dense, nmf_mu_dense_tol, nmf_mu_dense_monitor, nmf_mu_csr, nmf_mu_csr_monitor, nmf_mu_csr_tol, nmf_mu_ooc, nmf_mu_ooc_monitor, nmf_mu_ooc_hostw, nmf_mu_csr_ooc, nmf_mu_dense_batched,
    nmf_mu_workspace_bytes, nmf_mu_set_workspace, nmf_mu_release,
    nmf_csr_partition, nmf_split_planes, nmf_csr_to_csc, nmf_gram_w, nmf_wta_dense, nmf_h_update, nmf_aht_w_update_dense,
)
