"""MI355X-native CSR SpMV/SpMM (fp32): four HIP kernels and a rule-based selector
behind the ``libdgsp`` C-ABI.  Importing the package loads nothing; the shared
library is opened on the first call into :mod:`paper_2106_16064_amd.binding`,
which raises if it has not been built (there is no CPU fallback)."""

__all__ = ["binding", "workloads"]
