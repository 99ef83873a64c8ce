"""Seeded synthetic inputs for the Lloyd k-means hot path.

This module only *draws data*: Gaussian-mixture point clouds and initial centroids picked
from the data rows.  It holds none of the method's arithmetic (no distances, no argmin, no
means) and is the one module both the GPU parity tests and the CPU oracle tests read, so
that both sides see identical stored bits.

The paper evaluates on synthetic shape sweeps only and names neither a dataset nor a value
distribution (its Section 5.1), so the five workload families below are the definition of
the inputs; their shapes echo the paper's regimes (tiny, mid-size, batched B = 32,
large-N / small-K, out-of-core large-K).
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import torch

_DT = {"fp32": torch.float32, "fp16": torch.float16, "bf16": torch.bfloat16}


@dataclass(frozen=True)
class Workload:
    """One synthetic k-means problem family (all sizes are per batch instance)."""
    name: str
    B: int            # independent instances solved together
    N: int            # points per instance
    d: int            # feature dimension
    K: int            # centroids per instance
    dtype: str        # storage type of X and of the low-precision centroid copy
    center_std: float  # true mixture centres ~ N(0, center_std^2 I)
    noise_std: float   # points = centre + N(0, noise_std^2 I)
    zipf_s: float      # 0 -> uniform cluster membership, else P(k) ~ (k+1)^-s
    iters: int         # Lloyd iterations the configuration calls for
    seed: int          # data seed; the init seed is seed + 1000

    @property
    def torch_dtype(self) -> torch.dtype:
        return _DT[self.dtype]

    def scaled(self, **kw) -> "Workload":
        """Same recipe at another size (used by tests that need an oracle-sized case)."""
        return replace(self, **kw)


# The five benchmark configurations (full sizes).
C1 = Workload("c1_tiny_fp32", 1, 16384, 64, 64, "fp32", 10.0, 1.0, 0.0, 10, 1001)
C2 = Workload("c2_mid_fp16", 1, 1 << 20, 128, 1024, "fp16", 4.0, 1.0, 0.0, 20, 1002)
C3 = Workload("c3_batched_bf16", 32, 32768, 128, 256, "bf16", 1.0, 0.5, 0.0, 10, 1003)
C4 = Workload("c4_skewed_fp16", 1, 1 << 24, 64, 16, "fp16", 8.0, 1.0, 1.2, 20, 1004)
C5 = Workload("c5_ooc_fp16", 1, 1 << 28, 128, 65536, "fp16", 4.0, 1.0, 0.0, 5, 1005)
# A shape the paper quotes for its large-N / large-K regime (Section 5.2: N = 1M, K = 64K,
# D = 512); not one of the five benchmark configurations, used to exercise the wide-feature
# kernels at scale.
P512 = Workload("paper_large_k_d512_fp16", 1, 1 << 20, 512, 65536, "fp16", 4.0, 1.0, 0.0, 3, 1006)
# The paper's large-N / small-K end-to-end shape (N = 8M, K = 1024; d = 128 assumed as in its
# kernel-level experiments) and the shape of its assignment-kernel comparison (N = 1M, K = 8192).
P8M = Workload("paper_large_n_k1024_fp16", 1, 1 << 23, 128, 1024, "fp16", 4.0, 1.0, 0.0, 5, 1007)
PK8K = Workload("paper_k8192_fp16", 1, 1 << 20, 128, 8192, "fp16", 4.0, 1.0, 0.0, 5, 1008)
CONFIGS = {w.name: w for w in (C1, C2, C3, C4, C5, P512, P8M, PK8K)}


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def membership_probs(K: int, zipf_s: float) -> torch.Tensor:
    """P(label = k): uniform, or proportional to (k+1)^-s (float64, sums to 1)."""
    if zipf_s == 0.0:
        return torch.full((K,), 1.0 / K, dtype=torch.float64)
    w = torch.arange(1, K + 1, dtype=torch.float64).pow(-zipf_s)
    return w / w.sum()


def make_points(w: Workload, device="cpu", rows_per_block: int = 1 << 22,
                out: torch.Tensor | None = None, return_labels: bool = False):
    """Draw X [B,N,d] in w's storage dtype (and optionally the true labels [B,N] int32).

    Values are drawn in float32 and rounded once to the storage dtype; what is returned is
    what every consumer reads.  Generation is blocked over rows so that the float32
    staging stays small next to a large X; `out` may be a preallocated tensor (for
    instance pinned host memory) of shape [B,N,d].
    """
    dev = torch.device(device)
    g = _gen(w.seed, dev)
    X = out if out is not None else torch.empty((w.B, w.N, w.d), dtype=w.torch_dtype, device=dev)
    if tuple(X.shape) != (w.B, w.N, w.d) or X.dtype != w.torch_dtype:
        raise ValueError("out has the wrong shape or dtype")
    labels = torch.empty((w.B, w.N), dtype=torch.int32, device=dev) if return_labels else None
    cum = membership_probs(w.K, w.zipf_s).cumsum(0).to(torch.float32).to(dev)
    cum[-1] = 1.0
    for b in range(w.B):
        centres = torch.randn((w.K, w.d), generator=g, device=dev, dtype=torch.float32) * w.center_std
        for r0 in range(0, w.N, rows_per_block):
            r1 = min(w.N, r0 + rows_per_block)
            u = torch.rand((r1 - r0,), generator=g, device=dev, dtype=torch.float32)
            lab = torch.searchsorted(cum, u, right=True).clamp_(max=w.K - 1)
            blk = torch.randn((r1 - r0, w.d), generator=g, device=dev, dtype=torch.float32)
            blk.mul_(w.noise_std).add_(centres[lab])
            X[b, r0:r1].copy_(blk.to(w.torch_dtype))
            if labels is not None:
                labels[b, r0:r1] = lab.to(torch.int32)
    return (X, labels) if return_labels else X


def init_rows(w: Workload, labels: torch.Tensor | None = None) -> torch.Tensor:
    """Indices [B,K] (int64, CPU) of the data rows that seed the centroids.

    K distinct rows per instance, seeded.  With `labels` given and a skewed membership
    (zipf_s > 0) one row is drawn from each true component instead, so that the skew of
    the mixture reaches the update step from the first iteration on.
    """
    g = _gen(w.seed + 1000, "cpu")
    idx = torch.empty((w.B, w.K), dtype=torch.int64)
    for b in range(w.B):
        if labels is not None and w.zipf_s > 0.0:
            lab = labels[b].cpu()
            for k in range(w.K):
                members = torch.nonzero(lab == k).flatten()
                if members.numel() == 0:
                    raise ValueError(f"component {k} drew no point")
                j = torch.randint(0, members.numel(), (1,), generator=g)
                idx[b, k] = members[j]
        else:
            if w.N >= (1 << 24):
                # a permutation of N is wasteful here: draw with replacement and redraw duplicates
                pick = torch.randint(0, w.N, (w.K,), generator=g)
                while pick.unique().numel() < w.K:
                    pick = torch.cat([pick.unique(),
                                      torch.randint(0, w.N, (w.K,), generator=g)])[: w.K]
                idx[b] = pick
            else:
                idx[b] = torch.randperm(w.N, generator=g)[: w.K]
    return idx


def gather_rows(X: torch.Tensor, idx: torch.Tensor) -> torch.Tensor:
    """X[b, idx[b]] -> [B,K,d] float32 (exact widening of the stored rows)."""
    B = X.shape[0]
    rows = [X[b].index_select(0, idx[b].to(X.device)).to(torch.float32) for b in range(B)]
    return torch.stack(rows, 0)
