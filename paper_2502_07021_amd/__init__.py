"""fsk: MI355X-native hot path of Federated Sinkhorn (dense, row-partitioned,
log-domain and batched Gibbs-kernel scaling iterations) behind a C ABI.

Importing the package does not load the GPU library; the first call of a
binding function in :mod:`paper_2502_07021_amd.api` does, and raises if the
library has not been built.
"""
__all__ = ["api", "workloads"]
