"""GPU-assisted index construction for the large synthetic configurations (harness code).

Building a 10^7-vector index with 10^4 clusters is ~5e13 flop of nearest-centre search -- minutes
on host cores -- while it is not part of the search path this package is about.  This module does
the same build steps as `ivfpq_build_host` (Sec. I-C, first enumeration: k-means clusters,
residuals, per-sub-space codebooks, encoding, grouping by cluster) with plain torch matmuls on the
GPU and hands the resulting logical arrays to `ivfpq_index_from_arrays`.  Nothing here runs during
a search, and the search kernels never see torch.
"""
from __future__ import annotations

import numpy as np
import torch


def _assign(x: torch.Tensor, centres: torch.Tensor, chunk: int = 1 << 18) -> torch.Tensor:
    """Nearest centre of every row (ranking by |c|^2 - 2 x.c; ties to the lower index)."""
    cn = (centres * centres).sum(1)
    out = torch.empty(x.shape[0], dtype=torch.int64, device=x.device)
    step = max(1, min(chunk, (1 << 28) // max(centres.shape[0], 1)))
    for lo in range(0, x.shape[0], step):
        d = cn[None, :] - 2.0 * (x[lo:lo + step] @ centres.T)
        out[lo:lo + step] = torch.argmin(d, dim=1)
    return out


def _kmeans(x: torch.Tensor, k: int, iters: int, gen: torch.Generator) -> torch.Tensor:
    n = x.shape[0]
    if n >= k:
        start = torch.randperm(n, generator=gen, device=x.device)[:k].sort().values
    else:
        start = torch.arange(k, device=x.device) % max(n, 1)
    centres = x[start].clone()
    for _ in range(iters):
        lab = _assign(x, centres)
        sums = torch.zeros((k, x.shape[1]), dtype=torch.float64, device=x.device)
        sums.index_add_(0, lab, x.double())
        cnt = torch.bincount(lab, minlength=k)
        keep = cnt > 0
        centres[keep] = (sums[keep] / cnt[keep, None].double()).float()
    return centres


def _stride_rows(n: int, limit: int, device) -> torch.Tensor:
    if n <= limit:
        return torch.arange(n, device=device)
    return (torch.arange(limit, device=device, dtype=torch.int64) * n) // limit


def build_index_arrays(data: np.ndarray, n_lists: int, pq_dim: int, pq_bits: int, kmeans_iters: int = 10,
                       seed: int = 0):
    """-> (centroids, codebooks, list_offsets, codes, ids) as numpy arrays in the layout
    `ivfpq_index_from_arrays` takes."""
    dev = torch.device("cuda")
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    x = torch.from_numpy(data).to(dev)
    n, d = x.shape
    m, ksub = d // pq_dim, 1 << pq_bits
    centroids = _kmeans(x[_stride_rows(n, 256 * n_lists, dev)], n_lists, kmeans_iters, gen)
    labels = _assign(x, centroids)
    order = torch.argsort(labels, stable=True)                 # list order, ascending id inside a list
    counts = torch.bincount(labels, minlength=n_lists)
    offsets = torch.zeros(n_lists + 1, dtype=torch.int64, device=dev)
    offsets[1:] = torch.cumsum(counts, 0)
    # residuals in list order, in place and in slices (the 10^8-vector sets leave no room for copies)
    residual = x[order]
    del x
    lab_sorted = labels[order]
    for lo in range(0, n, 1 << 22):
        residual[lo:lo + (1 << 22)] -= centroids[lab_sorted[lo:lo + (1 << 22)]]
    del lab_sorted
    codebooks = torch.empty((pq_dim, ksub, m), dtype=torch.float32, device=dev)
    sub_codes = torch.empty((n, pq_dim), dtype=torch.uint8, device=dev)
    train_rows = _stride_rows(n, 262144, dev)
    for j in range(pq_dim):
        sub = residual[:, j * m:(j + 1) * m].contiguous()
        codebooks[j] = _kmeans(sub[train_rows], ksub, kmeans_iters, gen)
        sub_codes[:, j] = _assign(sub, codebooks[j]).to(torch.uint8)
    if pq_bits == 4:
        codes = sub_codes[:, 0::2] | (sub_codes[:, 1::2] << 4)
    else:
        codes = sub_codes
    return (centroids.cpu().numpy(), codebooks.cpu().numpy(), offsets.cpu().numpy(),
            np.ascontiguousarray(codes.cpu().numpy()), order.cpu().numpy())
