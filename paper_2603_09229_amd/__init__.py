"""MI355X-native exact Lloyd k-means iteration (fused assign + sort-inverse update).

The compute lives in hand-written HIP kernels behind the C-ABI library declared in
``include/flashkm.h``; :mod:`paper_2603_09229_amd.binding` marshals torch tensors into it.
Nothing is loaded at import time: the library is opened on first use and the call fails
loudly if it has not been built.
"""
__all__ = ["binding", "workloads"]
