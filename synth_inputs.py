"""Seeded synthetic inputs for the sample / gather / train hot path.

This module only *makes data*: R-MAT edge lists, feature tables, labels, train
splits and initial weights, with the shapes of the paper's datasets (Table 4).
It holds none of the method's arithmetic (no sampling, no aggregation, no
Philox): both the CPU oracle's tests and the HIP path's tests draw their inputs
from here, and neither side's code is imported here.

All randomness comes from numpy's own generators, keyed by (seed, tag).
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional, Tuple

import numpy as np

# ----------------------------------------------------------------------------
# named workloads (shapes follow Table 4 of the paper; the graphs are synthetic)
# ----------------------------------------------------------------------------


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    n_vertices: int
    n_edges: int            # directed edges handed to the CSR builder
    symmetrise: bool        # emit n_edges/2 pairs in both directions
    rowptr_bits: int
    feat_dim: int
    feat_dtype: str         # "f32" | "bf16"
    n_classes: int
    hidden: int
    fanouts: Tuple[int, ...]  # hop order, counted from the seeds
    batch: int
    hot_fraction: float
    staleness: int
    seed: int = 0

    @property
    def n_layers(self) -> int:
        return len(self.fanouts)

    @property
    def dims(self) -> List[int]:
        return [self.feat_dim] + [self.hidden] * (self.n_layers - 1) + [self.n_classes]


WORKLOADS = {
    # tiny: the small case the oracle finishes in seconds
    "tiny": Workload("tiny", 10_000, 100_000, False, 32, 64, "f32", 16, 64, (10, 5), 256, 0.05, 0),
    # dense-neighbourhood graph (Reddit-shaped): the benchmark workload
    "dense": Workload("dense", 233_000, 114_000_000, False, 64, 602, "f32", 41, 256, (25, 10), 1024, 0.10, 1),
    # mid-size sparse graph (Products-shaped)
    "sparse": Workload("sparse", 2_400_000, 124_000_000, True, 32, 100, "f32", 47, 256, (15, 10, 5), 1024, 0.10, 2),
    # large graph (Papers100M-shaped), bf16 features
    "large": Workload("large", 111_000_000, 1_600_000_000, False, 64, 128, "bf16", 172, 256, (15, 10, 5), 1024, 0.10, 2),
    # hot-reuse sweep on the sparse graph with wider features
    "sweep": Workload("sweep", 2_400_000, 124_000_000, True, 32, 256, "f32", 47, 256, (15, 10, 5), 4096, 0.10, 2),
}


def scaled(w: Workload, factor: float, name: Optional[str] = None) -> Workload:
    """A shrunken copy of a workload (same degree, widths and fanouts; fewer vertices)."""
    v = max(64, int(w.n_vertices * factor))
    e = max(v, int(w.n_edges * factor))
    if w.symmetrise:
        e -= e % 2
    return dataclasses.replace(w, name=name or f"{w.name}@{factor:g}", n_vertices=v, n_edges=e)


def _rng(seed: int, tag: str) -> np.random.Generator:
    tag_words = [int.from_bytes(tag.encode()[i:i + 4].ljust(4, b"\0"), "little") for i in range(0, len(tag), 4)]
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed] + tag_words)))


# ----------------------------------------------------------------------------
# R-MAT
# ----------------------------------------------------------------------------

def _rmat_chunk(args):
    seed, chunk_index, quota, n_vertices, scale, ta, tb, tc = args
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 0x726D6174, chunk_index])))
    src = np.empty(quota, dtype=np.int32)
    dst = np.empty(quota, dtype=np.int32)
    filled = 0
    while filled < quota:
        m = int((quota - filled) * 1.35) + 1024
        u = rng.integers(0, 65536, size=(scale, m), dtype=np.uint16)
        s = np.zeros(m, dtype=np.int32)
        d = np.zeros(m, dtype=np.int32)
        for level in range(scale):
            ul = u[level]
            # quadrant a: neither bit, b: dst bit, c: src bit, d: both
            ge_tb = ul >= tb
            s <<= 1
            s |= ge_tb
            d <<= 1
            d |= ((ul >= ta) & ~ge_tb) | (ul >= tc)
        ok = (s < n_vertices) & (d < n_vertices)
        s = s[ok]
        d = d[ok]
        take = min(len(s), quota - filled)
        src[filled:filled + take] = s[:take]
        dst[filled:filled + take] = d[:take]
        filled += take
    return src, dst


def rmat_edges(n_vertices: int, n_edges: int, seed: int = 0, a: float = 0.57, b: float = 0.19,
               c: float = 0.19, symmetrise: bool = False, permute: bool = True,
               chunk: int = 1 << 22, workers: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Directed edge list (src, dst), int32, of an R-MAT graph.

    One quadrant choice per bit level (probabilities a, b, c, 1-a-b-c, 16 random bits
    per level); endpoints >= n_vertices are rejected and redrawn; vertex ids are then
    relabelled by a seeded permutation so that hubs are scattered over the id range.
    With ``symmetrise`` n_edges/2 pairs are drawn and emitted in both directions.
    Multi-edges and self-loops are kept, as R-MAT makes them. Edges are drawn in chunks
    with one generator per chunk, so the result does not depend on the worker count.
    """
    import concurrent.futures
    import os
    if n_vertices <= 0 or n_vertices >= 2 ** 31:
        raise ValueError("n_vertices out of range")
    scale = max(1, int(np.ceil(np.log2(n_vertices))))
    n_draw = n_edges // 2 if symmetrise else n_edges
    ta = int(round(a * 65536))
    tb = ta + int(round(b * 65536))
    tc = tb + int(round(c * 65536))
    jobs = [(seed, i, min(chunk, n_draw - lo), n_vertices, scale, ta, tb, tc)
            for i, lo in enumerate(range(0, n_draw, chunk))]
    if workers is None:
        workers = max(1, min(16, (os.cpu_count() or 1)))
    if len(jobs) <= 1 or workers == 1:
        parts = [_rmat_chunk(j) for j in jobs]
    else:
        with concurrent.futures.ThreadPoolExecutor(max_workers=workers) as ex:
            parts = list(ex.map(_rmat_chunk, jobs))
    if parts:
        src = np.concatenate([p[0] for p in parts])
        dst = np.concatenate([p[1] for p in parts])
    else:
        src = np.zeros(0, dtype=np.int32)
        dst = np.zeros(0, dtype=np.int32)
    if permute:
        perm = _rng(seed, "vperm").permutation(n_vertices).astype(np.int32)
        src = perm[src]
        dst = perm[dst]
    if symmetrise:
        src, dst = np.concatenate([src, dst]), np.concatenate([dst, src])
    return np.ascontiguousarray(src), np.ascontiguousarray(dst)


# ----------------------------------------------------------------------------
# features, labels, split, weights
# ----------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even conversion of float32 to bfloat16 bit patterns (uint16)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def features(n_vertices: int, dim: int, seed: int = 0, dtype: str = "f32") -> np.ndarray:
    """Feature table [V, dim], i.i.d. N(0,1); float32, or uint16 bf16 bit patterns."""
    rng = _rng(seed, "feat")
    x = rng.standard_normal((n_vertices, dim), dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(dtype)


def features_on_device(n_vertices: int, dim: int, seed: int = 0, dtype: str = "f32", device: str = "cuda",
                       chunk_rows: int = 1 << 22):
    """Feature table generated directly in device memory with torch's generator (for tables too large
    to make on the host in reasonable time, e.g. 111 M x 128). Returns a torch tensor: float32, or int16
    bf16 bit patterns (round-to-nearest-even). Rows are i.i.d. N(0,1); not the same values as features()."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(0x66656174 + 1000003 * seed)
    out = torch.empty((n_vertices, dim), dtype=torch.float32 if dtype == "f32" else torch.int16, device=device)
    for lo in range(0, n_vertices, chunk_rows):
        hi = min(n_vertices, lo + chunk_rows)
        x = torch.randn((hi - lo, dim), generator=gen, device=device, dtype=torch.float32)
        out[lo:hi] = x if dtype == "f32" else x.to(torch.bfloat16).view(torch.int16)
    return out


def labels(n_vertices: int, n_classes: int, seed: int = 0) -> np.ndarray:
    return _rng(seed, "label").integers(0, n_classes, size=n_vertices, dtype=np.int32)


def train_split(n_vertices: int, fraction: float = 0.65, seed: int = 0) -> np.ndarray:
    """Seeded permutation of the training vertices (unique ids, int32)."""
    perm = _rng(seed, "split").permutation(n_vertices).astype(np.int32)
    return np.ascontiguousarray(perm[: max(1, int(n_vertices * fraction))])


def batch_seeds(train_ids: np.ndarray, batch: int, step: int) -> np.ndarray:
    """Seeds of step t: slice [t*B, (t+1)*B) of the train permutation, wrapping by whole batches."""
    nb = max(1, len(train_ids) // batch)
    b = step % nb
    return np.ascontiguousarray(train_ids[b * batch:(b + 1) * batch])


def init_weights(dims: List[int], seed: int = 0):
    """Glorot-uniform W_self, W_neigh [d_in, d_out] and small random bias per layer (float32)."""
    rng = _rng(seed, "weights")
    out = []
    for d_in, d_out in zip(dims[:-1], dims[1:]):
        lim = float(np.sqrt(6.0 / (2 * d_in + d_out)))
        w_self = rng.uniform(-lim, lim, size=(d_in, d_out)).astype(np.float32)
        w_neigh = rng.uniform(-lim, lim, size=(d_in, d_out)).astype(np.float32)
        bias = rng.uniform(-0.1, 0.1, size=(d_out,)).astype(np.float32)
        out.append((w_self, w_neigh, bias))
    return out


def random_graph_small(n_vertices: int, n_edges: int, seed: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """Uniform random multigraph for tiny brute-force tests."""
    rng = _rng(seed, "gsmall")
    return (rng.integers(0, n_vertices, n_edges, dtype=np.int32),
            rng.integers(0, n_vertices, n_edges, dtype=np.int32))


def make_workload_arrays(w: Workload, with_features: bool = True):
    """(src, dst, feat, labels, train_ids, weights) for a workload."""
    src, dst = rmat_edges(w.n_vertices, w.n_edges, w.seed, symmetrise=w.symmetrise)
    feat = features(w.n_vertices, w.feat_dim, w.seed, w.feat_dtype) if with_features else None
    lab = labels(w.n_vertices, w.n_classes, w.seed)
    train = train_split(w.n_vertices, 0.65, w.seed)
    weights = init_weights(w.dims, w.seed)
    return src, dst, feat, lab, train, weights
