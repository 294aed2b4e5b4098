"""CPU oracle for one sample-based GNN training step with hot-embedding reuse.

THIS IS TEST INFRASTRUCTURE: a plain, slow, obviously-correct statement of what the hot path
computes. Only tests, the smoke check and the benchmark's CPU-baseline leg may use it; the
product path never does. It shares no code with the GPU library.

Integer work (Philox sampling, relabelling, transposition, hot counting, CSR build) lives in
``no_oracle.c`` (plain C, called through ctypes); floating point is numpy fp64 throughout.

What it follows in the paper:
  * Algorithm 1: per batch, sample L hops in reverse from the seeds, gather the input
    features, L forward layers, loss, L backward layers, one parameter update.
  * Eq. 1 / Eq. 2: AGGREGATE = average over sampled in-neighbours, UPDATE = dense layer.
    GraphSAGE-mean reading: h_v = act(W_self^T h_v + W_neigh^T mean_u h_u + b); ReLU between
    layers, none on the logits. GCN-style reading (arch "gcn"): Eq. 1 as printed, the average over
    N_in(v) U {v} of the sampled block, then h_v = act(W^T a_v + b).
  * Section 4.1.2: hot vertices by pre-sampling frequency; a hot vertex's layer-1 embedding
    computed at step t0 may be reused at steps t with t - t0 <= S (S = bound in batches);
    a reused embedding gets no aggregation and no backward pass.
  * Section 4.2 (Stage 2 and "Bounded Staleness"): n batches form a super-batch; while one
    super-batch trains, the embeddings of ALL hot vertices are recomputed for the next one
    (one-hop sample at the bottom fanout, layer-1 forward) and become the cache contents at the
    super-batch boundary, so a row made with parameter version k*n serves steps (k+1)*n ...
    (k+2)*n - 1: version gap at most 2n - 1 (`refresh_hot`, `train_superbatches`).
  * Section 4.3: the weight drift that stale rows may see is monitored against
    epsilon = (largest change of a weight in one update) x 2n (`weight_drift`, `drift_tolerance`).
"""
from __future__ import annotations

import ctypes
import dataclasses
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "no_oracle.c")
_LIB = os.path.join(_HERE, "libno_oracle.so")

DOMAIN_TRAIN = 0
DOMAIN_PRESAMPLE = 1
DOMAIN_REFRESH = 2


def build(force: bool = False) -> str:
    """Compile the C part with gcc (plain -O2)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        c = ctypes
        P = c.c_void_p
        L.ora_philox4x32_10.argtypes = [P, P, P]
        L.ora_philox4x32_10.restype = None
        L.ora_random64.argtypes = [c.c_uint64, c.c_uint32, c.c_uint32, c.c_uint64, c.c_uint32]
        L.ora_random64.restype = c.c_uint64
        L.ora_mulhi64.argtypes = [c.c_uint64, c.c_uint64]
        L.ora_mulhi64.restype = c.c_uint64
        L.ora_fisher_yates_prefix.argtypes = [c.c_int64, c.c_int32, P, P]
        L.ora_fisher_yates_prefix.restype = None
        L.ora_sample_row.argtypes = [c.c_uint64, c.c_uint32, c.c_uint32, c.c_uint64, c.c_int64, c.c_int32, P]
        L.ora_sample_row.restype = c.c_int32
        L.ora_build_csr.argtypes = [P, P, c.c_int64, c.c_int64, P, P]
        L.ora_build_csr.restype = None
        L.ora_sample_hop.argtypes = [P, P, P, c.c_int64, c.c_int32, c.c_uint64, c.c_uint32, c.c_uint32,
                                     P, P, P, P, P]
        L.ora_sample_hop.restype = c.c_int64
        L.ora_block_csc.argtypes = [P, P, c.c_int64, c.c_int64, P, P, P]
        L.ora_block_csc.restype = None
        L.ora_presample_counts.argtypes = [P, P, c.c_int64, P, c.c_int64, c.c_int32, P, c.c_int32, c.c_int32,
                                           c.c_uint64, P]
        L.ora_presample_counts.restype = None
        L.ora_gather_rows.argtypes = [P, c.c_int64, P, c.c_int64, P]
        L.ora_gather_rows.restype = None
        L.ora_mean_aggregate.argtypes = [P, c.c_int64, P, P, c.c_int64, P]
        L.ora_mean_aggregate.restype = None
        L.ora_mean_aggregate_adjoint.argtypes = [P, c.c_int64, P, P, c.c_int64, P]
        L.ora_mean_aggregate_adjoint.restype = None
        _lib = L
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _u64(x: int) -> int:
    return int(x) & 0xFFFFFFFFFFFFFFFF


# --------------------------------------------------------------------------- random source

def philox4x32_10(ctr: Sequence[int], key: Sequence[int]) -> Tuple[int, int, int, int]:
    c = np.array(ctr, dtype=np.uint32)
    k = np.array(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().ora_philox4x32_10(_p(c), _p(k), _p(out))
    return tuple(int(x) for x in out)


def random64(stream: int, domain: int, hop: int, v: int, slot: int) -> int:
    return int(lib().ora_random64(_u64(stream), domain, hop, v, slot))


def fisher_yates_prefix(d: int, k: int, r: Sequence[int]) -> List[int]:
    rr = np.array(r, dtype=np.int64)
    out = np.zeros(k, dtype=np.int64)
    lib().ora_fisher_yates_prefix(d, k, _p(rr), _p(out))
    return [int(x) for x in out]


def sample_row(stream: int, domain: int, hop: int, v: int, d: int, k: int) -> List[int]:
    out = np.zeros(max(k, 1), dtype=np.int64)
    n = lib().ora_sample_row(_u64(stream), domain, hop, v, d, k, _p(out))
    return [int(x) for x in out[:n]]


# --------------------------------------------------------------------------- graph

@dataclasses.dataclass
class Graph:
    n_vertices: int
    rowptr: np.ndarray   # int64 [V+1]
    col: np.ndarray      # int32 [E]

    @property
    def n_edges(self) -> int:
        return int(self.rowptr[-1])


def build_csr(src: np.ndarray, dst: np.ndarray, n_vertices: int, symmetrise: bool = False, dedup: bool = False) -> Graph:
    """In-neighbour CSR (Eq. 1 aggregates over N_in): row dst holds its sources, ascending; duplicates kept.
    symmetrise: every edge is also taken the other way round; dedup: of equal (src, dst) pairs one is kept."""
    src = np.asarray(src)
    dst = np.asarray(dst)
    if symmetrise:
        src, dst = np.concatenate([src, dst]), np.concatenate([dst, src])
    if dedup and len(src):
        pairs = np.unique(np.stack([np.asarray(dst, np.int64), np.asarray(src, np.int64)], axis=1), axis=0)
        dst, src = pairs[:, 0], pairs[:, 1]
    src = np.ascontiguousarray(src, dtype=np.int32)
    dst = np.ascontiguousarray(dst, dtype=np.int32)
    rowptr = np.zeros(n_vertices + 1, dtype=np.int64)
    col = np.zeros(max(len(src), 1), dtype=np.int32)
    lib().ora_build_csr(_p(src), _p(dst), len(src), n_vertices, _p(rowptr), _p(col))
    return Graph(n_vertices, rowptr, col[: len(src)])


# --------------------------------------------------------------------------- sampled blocks

@dataclasses.dataclass
class Block:
    """One sampled hop as a bipartite block: n_src sources (the first n_dst are the
    destinations themselves), rows = destinations."""
    dst_global: np.ndarray
    src_global: np.ndarray
    indptr: np.ndarray
    nbr_global: np.ndarray
    indices: np.ndarray
    csc_indptr: np.ndarray
    csc_dst: np.ndarray
    csc_eid: np.ndarray

    @property
    def n_dst(self) -> int:
        return len(self.dst_global)

    @property
    def n_src(self) -> int:
        return len(self.src_global)

    @property
    def nnz(self) -> int:
        return len(self.indices)


def sample_hop(g: Graph, dst_global: np.ndarray, fanout: int, stream: int, domain: int, hop: int,
               _map: Optional[np.ndarray] = None) -> Block:
    dst_global = np.ascontiguousarray(dst_global, dtype=np.int32)
    n_dst = len(dst_global)
    m = _map if _map is not None else np.full(g.n_vertices, -1, dtype=np.int32)
    cap_e = max(n_dst * fanout, 1)
    indptr = np.zeros(n_dst + 1, dtype=np.int32)
    nbr = np.zeros(cap_e, dtype=np.int32)
    idx = np.zeros(cap_e, dtype=np.int32)
    srcg = np.zeros(n_dst + cap_e, dtype=np.int32)
    n_src = lib().ora_sample_hop(_p(g.rowptr), _p(g.col), _p(dst_global), n_dst, fanout,
                                 _u64(stream), domain, hop, _p(m), _p(indptr), _p(nbr), _p(idx), _p(srcg))
    nnz = int(indptr[n_dst])
    idx = np.ascontiguousarray(idx[:nnz])
    csc_indptr = np.zeros(n_src + 1, dtype=np.int32)
    csc_dst = np.zeros(max(nnz, 1), dtype=np.int32)
    csc_eid = np.zeros(max(nnz, 1), dtype=np.int32)
    lib().ora_block_csc(_p(indptr), _p(idx), n_dst, n_src, _p(csc_indptr), _p(csc_dst), _p(csc_eid))
    return Block(dst_global, np.ascontiguousarray(srcg[:n_src]), indptr, np.ascontiguousarray(nbr[:nnz]), idx,
                 csc_indptr, csc_dst[:nnz], csc_eid[:nnz])


# --------------------------------------------------------------------------- hot set and cache

@dataclasses.dataclass
class Cache:
    """Hot set (Section 4.1.2) with its embedding store and version record."""
    hot_ids: np.ndarray          # int32 [n_hot], hotness order
    slot_of_vertex: np.ndarray   # int32 [V], -1 = cold
    version: np.ndarray          # int32 [n_hot], step whose weights made the row; -1 = empty
    emb: np.ndarray              # float64 [n_hot, emb_dim]
    staleness: int
    freq: Optional[np.ndarray] = None

    @property
    def n_hot(self) -> int:
        return len(self.hot_ids)

    def copy(self) -> "Cache":
        return Cache(self.hot_ids.copy(), self.slot_of_vertex.copy(), self.version.copy(), self.emb.copy(),
                     self.staleness, None if self.freq is None else self.freq.copy())


def presample_counts(g: Graph, train_ids: np.ndarray, batch: int, fanouts: Sequence[int], epochs: int,
                     seed: int) -> np.ndarray:
    train_ids = np.ascontiguousarray(train_ids, dtype=np.int32)
    fo = np.array(fanouts, dtype=np.int32)
    freq = np.zeros(g.n_vertices, dtype=np.int64)
    lib().ora_presample_counts(_p(g.rowptr), _p(g.col), g.n_vertices, _p(train_ids), len(train_ids), batch,
                               _p(fo), len(fo), epochs, _u64(seed), _p(freq))
    return freq


def select_hot(g: Graph, train_ids: np.ndarray, batch: int, fanouts: Sequence[int], presample_epochs: int,
               hot_fraction: float, staleness: int, emb_dim: int, seed: int) -> Cache:
    """Hot set = the floor(hot_fraction * V) most frequently pre-sampled vertices, ties by id."""
    freq = presample_counts(g, train_ids, batch, fanouts, presample_epochs, seed)
    n_hot = int(np.floor(hot_fraction * g.n_vertices))
    order = np.lexsort((np.arange(g.n_vertices), -freq))   # primary: freq descending; then id ascending
    hot = np.ascontiguousarray(order[:n_hot].astype(np.int32))
    slot = np.full(g.n_vertices, -1, dtype=np.int32)
    slot[hot] = np.arange(n_hot, dtype=np.int32)
    return Cache(hot, slot, np.full(n_hot, -1, dtype=np.int32), np.zeros((n_hot, emb_dim), dtype=np.float64),
                 staleness, freq)


def cache_lookup(cache: Cache, v1: np.ndarray, step: int):
    """Split V^1 (order kept) into reusable rows and rows to compute.
    A row is reusable iff the vertex is hot, its slot is filled, and step - version <= S."""
    slot = cache.slot_of_vertex[v1]
    ver = np.full(len(v1), -1, dtype=np.int64)
    ver[slot >= 0] = cache.version[slot[slot >= 0]]
    hit = (slot >= 0) & (ver >= 0) & (step - ver <= cache.staleness)
    hit_pos = np.nonzero(hit)[0].astype(np.int32)
    compute_pos = np.nonzero(~hit)[0].astype(np.int32)
    return compute_pos, hit_pos, slot[hit_pos].astype(np.int32)


@dataclasses.dataclass
class SampledBatch:
    blocks: List[Block]               # hop order from the seeds; blocks[-1] is the bottom hop
    compute_pos: Optional[np.ndarray]  # positions in V^1 of the bottom hop's destinations
    hit_pos: Optional[np.ndarray]
    hit_slot: Optional[np.ndarray]


def sample_blocks(g: Graph, seeds: np.ndarray, fanouts: Sequence[int], seed: int, step: int,
                  cache: Optional[Cache] = None, domain: int = DOMAIN_TRAIN) -> SampledBatch:
    """Reverse L-hop sampling from the seeds (Algorithm 1). The frontier of hop h+1 is the source
    set of hop h. With a cache, reusable hot vertices are left out of the bottom hop."""
    L = len(fanouts)
    stream = _u64(seed + step)
    m = np.full(g.n_vertices, -1, dtype=np.int32)
    blocks: List[Block] = []
    frontier = np.ascontiguousarray(seeds, dtype=np.int32)
    compute_pos = hit_pos = hit_slot = None
    for h in range(L):
        if h == L - 1 and cache is not None and L >= 2:
            compute_pos, hit_pos, hit_slot = cache_lookup(cache, frontier, step)
            frontier = np.ascontiguousarray(frontier[compute_pos])
        b = sample_hop(g, frontier, fanouts[h], stream, domain, h, m)
        blocks.append(b)
        frontier = b.src_global
    return SampledBatch(blocks, compute_pos, hit_pos, hit_slot)


# --------------------------------------------------------------------------- gather

def gather_features(table: np.ndarray, ids: np.ndarray) -> np.ndarray:
    """Feature collection: out[i,:] = table[ids[i],:], bit copy (any dtype)."""
    table = np.ascontiguousarray(table)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    out = np.empty((len(ids),) + table.shape[1:], dtype=table.dtype)
    lib().ora_gather_rows(_p(table), table.strides[0], _p(ids), len(ids), _p(out))
    return out


# --------------------------------------------------------------------------- layers (fp64)

def mean_aggregate(x_src: np.ndarray, indptr: np.ndarray, indices: np.ndarray, n_dst: int) -> np.ndarray:
    x = np.ascontiguousarray(x_src, dtype=np.float64)
    out = np.zeros((n_dst, x.shape[1]), dtype=np.float64)
    lib().ora_mean_aggregate(_p(x), x.shape[1], _p(np.ascontiguousarray(indptr, dtype=np.int32)),
                             _p(np.ascontiguousarray(indices, dtype=np.int32)), n_dst, _p(out))
    return out


def mean_aggregate_adjoint(grad_mean: np.ndarray, indptr: np.ndarray, indices: np.ndarray, n_dst: int,
                           n_src: int) -> np.ndarray:
    g = np.ascontiguousarray(grad_mean, dtype=np.float64)
    out = np.zeros((n_src, g.shape[1]), dtype=np.float64)
    lib().ora_mean_aggregate_adjoint(_p(g), g.shape[1], _p(np.ascontiguousarray(indptr, dtype=np.int32)),
                                     _p(np.ascontiguousarray(indices, dtype=np.int32)), n_dst, _p(out))
    return out


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Values rounded to bfloat16 (8 significant bits, fp32's exponent range), round-to-nearest-even, via fp32; returned
    as fp64. The precision the matrix units take the operands of a product in when the feature table is bf16."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000).astype(np.uint32)
    return r.view(np.float32).astype(np.float64)


def sage_layer_fwd_z(blk: Block, x_src: np.ndarray, w_self, w_neigh, bias, relu: bool, bf16_products: bool = False):
    """Eq. 1 (mean over the sampled row) then Eq. 2 (dense update). Returns (mean, z, h), z = pre-activation.
    bf16_products: the two products of Eq. 2 take their operands (features, mean, weights) rounded to bf16 and
    accumulate exactly: the arithmetic of a layer fed by a bf16 feature table ("bf16 with fp32 accumulate")."""
    x = np.asarray(x_src, dtype=np.float64)
    mean = mean_aggregate(x, blk.indptr, blk.indices, blk.n_dst)
    q = round_to_bf16 if bf16_products else (lambda a: np.asarray(a, np.float64))
    z = q(x[: blk.n_dst]) @ q(w_self) + q(mean) @ q(w_neigh) + np.asarray(bias, np.float64)
    h = np.maximum(z, 0.0) if relu else z
    return mean, z, h


def sage_layer_fwd(blk: Block, x_src: np.ndarray, w_self, w_neigh, bias, relu: bool):
    """Returns (mean, h) of one layer."""
    mean, _, h = sage_layer_fwd_z(blk, x_src, w_self, w_neigh, bias, relu)
    return mean, h


def sage_layer_bwd(blk: Block, x_src: np.ndarray, mean: np.ndarray, h: np.ndarray, grad_h: np.ndarray,
                   w_self, w_neigh, relu: bool, need_grad_x: bool, active: Optional[np.ndarray] = None,
                   bf16_products: bool = False):
    """Gradients of one layer. grad_x is None for the bottom layer (nothing below it learns).
    `active` (bool, shape of h) overrides the ReLU decision h > 0: a caller may supply decisions taken
    in another precision for pre-activations that are zero to within rounding, where either is valid.
    bf16_products: the two weight-gradient products take their operands (features, mean, gz) rounded to bf16; the bias
    gradient is the plain column sum."""
    x = np.asarray(x_src, dtype=np.float64)
    if relu:
        gz = np.asarray(grad_h, np.float64) * ((np.asarray(h) > 0) if active is None else active)
    else:
        gz = np.asarray(grad_h, np.float64)
    x_dst = x[: blk.n_dst]
    q = round_to_bf16 if bf16_products else (lambda a: np.asarray(a, np.float64))
    gw_self = q(x_dst).T @ q(gz)
    gw_neigh = q(mean).T @ q(gz)
    gb = gz.sum(axis=0)
    gx = None
    if need_grad_x:
        gmean = gz @ np.asarray(w_neigh, np.float64).T
        gx = mean_aggregate_adjoint(gmean, blk.indptr, blk.indices, blk.n_dst, blk.n_src)
        gx[: blk.n_dst] += gz @ np.asarray(w_self, np.float64).T
    return gw_self, gw_neigh, gb, gx


GCN_NORMS = ("mean", "sum", "sym")


def gcn_norm_of(arch: str) -> str:
    """Layer-form name -> normalisation of the GCN-style aggregate: "gcn" (average), "gcn_sum", "gcn_sym"."""
    return {"gcn": "mean", "gcn_sum": "sum", "gcn_sym": "sym"}[arch]


def gcn_scales(indptr: np.ndarray, indices: np.ndarray, n_dst: int, n_src: int, norm: str):
    """Row scale r_v and source scale s_u of the GCN-style aggregate a_v = r_v (s_v x_v + sum_{u in row v} s_u x_u)
    over the sampled block with self loops, A~ = A_i + I (destination v is source row v):
      "mean": r = 1 / (len + 1), s = 1            (AGGREGATE = average, Eq. 1)
      "sum":  r = 1, s = 1                        (AGGREGATE = sum, Eq. 1)
      "sym":  r = (len + 1)^-1/2, s_u = c_u^-1/2  (symmetric normalisation, Table 1: A^ = D_r^-1/2 A~ D_c^-1/2 with D_r the
              row sums of A~, len + 1, and D_c its column sums, c_u = number of sampled edges that leave u, plus one
              if u is a destination). A source no edge leaves and that is no destination has weight 0 (it is in no sum).
    """
    ln = np.diff(np.asarray(indptr[: n_dst + 1], dtype=np.int64)).astype(np.float64)
    nnz = int(indptr[n_dst])
    if norm == "mean":
        return 1.0 / (ln + 1.0), np.ones(n_src)
    if norm == "sum":
        return np.ones(n_dst), np.ones(n_src)
    if norm == "sym":
        c = np.bincount(np.asarray(indices[:nnz], dtype=np.int64), minlength=n_src).astype(np.float64)
        c[:n_dst] += 1.0
        s = np.zeros(n_src)
        s[c > 0] = c[c > 0] ** -0.5
        return (ln + 1.0) ** -0.5, s
    raise ValueError(norm)


def gcn_aggregate(x_src: np.ndarray, indptr: np.ndarray, indices: np.ndarray, n_dst: int, norm: str = "mean") -> np.ndarray:
    """Eq. 1 as printed, over N_in(v) U {v} of the sampled block: a_v = r_v (s_v x_v + sum over the sampled row of
    s_u x_u), with the scales of `gcn_scales`. Destination v is source row v of the block."""
    x = np.asarray(x_src, dtype=np.float64)
    r, s = gcn_scales(indptr, indices, n_dst, x.shape[0], norm)
    ln = np.diff(np.asarray(indptr[: n_dst + 1], dtype=np.int64))
    xs = x * s[:, None]
    out = xs[:n_dst].copy()
    rows = np.repeat(np.arange(n_dst), ln)
    np.add.at(out, rows, xs[np.asarray(indices[: ln.sum()], dtype=np.int64)])
    return out * r[:, None]


def gcn_aggregate_adjoint(grad_a: np.ndarray, indptr: np.ndarray, indices: np.ndarray, n_dst: int,
                          n_src: int, norm: str = "mean") -> np.ndarray:
    g = np.asarray(grad_a, dtype=np.float64)
    r, s = gcn_scales(indptr, indices, n_dst, n_src, norm)
    ln = np.diff(np.asarray(indptr[: n_dst + 1], dtype=np.int64))
    gs = g * r[:, None]
    out = np.zeros((n_src, g.shape[1]), dtype=np.float64)
    out[:n_dst] += gs
    rows = np.repeat(np.arange(n_dst), ln)
    np.add.at(out, np.asarray(indices[: ln.sum()], dtype=np.int64), gs[rows])
    return out * s[:, None]


def gcn_layer_fwd_z(blk: Block, x_src: np.ndarray, w, bias, relu: bool, norm: str = "mean"):
    """GCN-style layer: Eq. 1 over N_in(v) U {v} (average, sum or symmetric normalisation), Eq. 2 with one weight
    matrix. Returns (a, z, h)."""
    a = gcn_aggregate(x_src, blk.indptr, blk.indices, blk.n_dst, norm)
    z = a @ np.asarray(w, np.float64) + np.asarray(bias, np.float64)
    h = np.maximum(z, 0.0) if relu else z
    return a, z, h


def gcn_layer_fwd(blk: Block, x_src: np.ndarray, w, bias, relu: bool, norm: str = "mean"):
    a, _, h = gcn_layer_fwd_z(blk, x_src, w, bias, relu, norm)
    return a, h


def gcn_layer_bwd(blk: Block, a: np.ndarray, h: np.ndarray, grad_h: np.ndarray, w, relu: bool, need_grad_x: bool,
                  active: Optional[np.ndarray] = None, norm: str = "mean"):
    """Gradients of the GCN-style layer: (gw, gb, grad_x or None)."""
    if relu:
        gz = np.asarray(grad_h, np.float64) * ((np.asarray(h) > 0) if active is None else active)
    else:
        gz = np.asarray(grad_h, np.float64)
    gw = np.asarray(a, np.float64).T @ gz
    gb = gz.sum(axis=0)
    gx = None
    if need_grad_x:
        gx = gcn_aggregate_adjoint(gz @ np.asarray(w, np.float64).T, blk.indptr, blk.indices, blk.n_dst, blk.n_src, norm)
    return gw, gb, gx


def softmax_xent(logits: np.ndarray, labels: np.ndarray):
    """Mean softmax cross-entropy over the batch and its gradient w.r.t. the logits."""
    z = np.asarray(logits, np.float64)
    z = z - z.max(axis=1, keepdims=True)
    lse = np.log(np.exp(z).sum(axis=1, keepdims=True))
    logp = z - lse
    n = z.shape[0]
    loss = -logp[np.arange(n), labels].mean()
    g = np.exp(logp)
    g[np.arange(n), labels] -= 1.0
    return float(loss), g / n


# --------------------------------------------------------------------------- one training step

@dataclasses.dataclass
class StepResult:
    loss: float
    batch: SampledBatch
    x0: np.ndarray                       # gathered input features (table dtype)
    h: List[np.ndarray]                  # h[l-1] = output of layer l (h[0] holds all of V^1 with a cache)
    mean: List[np.ndarray]
    grads: List[Tuple[np.ndarray, np.ndarray, np.ndarray]]
    new_weights: List[Tuple[np.ndarray, np.ndarray, np.ndarray]]
    n_hit: int


def _to_f64(x: np.ndarray, feat_is_bf16: bool) -> np.ndarray:
    if feat_is_bf16:
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return x.astype(np.float64)


def train_step(g: Graph, feat: np.ndarray, labels: np.ndarray, seeds: np.ndarray, fanouts: Sequence[int],
               weights, lr: float, seed: int, step: int, cache: Optional[Cache] = None,
               feat_is_bf16: bool = False, relu_decisions=None, arch: str = "sage",
               bf16_products: Optional[bool] = None) -> StepResult:
    """One pass of Algorithm 1's loop body with plain SGD; updates `cache` in place.
    arch "sage": GraphSAGE-mean layers, weights[l] = (w_self, w_neigh, bias); arch "gcn" / "gcn_sum" / "gcn_sym":
    layers that aggregate over N_in(v) U {v} (average / sum / symmetric normalisation) with one matrix,
    weights[l] = (w, bias); `mean` then holds that aggregate.
    relu_decisions: optional callable(layer, z_layer) -> bool array or None, consulted in the backward
    pass for the ReLU decisions of layer `layer` given its pre-activations (rows of the computed vertices).
    bf16_products (default: on for a bf16 table with GraphSAGE-mean layers): layer 1's products, forward and weight
    gradients, take bf16 operands (`sage_layer_fwd_z`, `sage_layer_bwd`); the layers above work on fp32 activations."""
    L = len(fanouts)
    if bf16_products is None:
        bf16_products = feat_is_bf16 and arch == "sage"
    sb = sample_blocks(g, seeds, fanouts, seed, step, cache)
    bottom = sb.blocks[-1]
    x0 = gather_features(feat, bottom.src_global)
    x = _to_f64(x0, feat_is_bf16)
    hs, means, xs, zs = [], [], [], []
    use_cache = cache is not None and L >= 2
    for l in range(1, L + 1):
        blk = sb.blocks[L - l]
        xs.append(x)
        if arch != "sage":
            mean, z, h = gcn_layer_fwd_z(blk, x, weights[l - 1][0], weights[l - 1][1], relu=(l < L), norm=gcn_norm_of(arch))
        else:
            w_self, w_neigh, bias = weights[l - 1]
            mean, z, h = sage_layer_fwd_z(blk, x, w_self, w_neigh, bias, relu=(l < L), bf16_products=bf16_products and l == 1)
        means.append(mean)
        zs.append(z)
        if l == 1 and use_cache:
            n_v1 = len(sb.compute_pos) + len(sb.hit_pos)
            full = np.zeros((n_v1, h.shape[1]), dtype=np.float64)
            full[sb.compute_pos] = h
            full[sb.hit_pos] = cache.emb[sb.hit_slot]
            hs.append(full)
            x = full
        else:
            hs.append(h)
            x = h
    loss, gh = softmax_xent(hs[-1], np.asarray(labels)[np.asarray(seeds)])
    grads = [None] * L
    for l in range(L, 0, -1):
        blk = sb.blocks[L - l]
        h_l = hs[l - 1]
        if l == 1 and use_cache:
            h_l = h_l[sb.compute_pos]
            gh = gh[sb.compute_pos]        # reused rows take no gradient
        active = relu_decisions(l, zs[l - 1]) if (relu_decisions is not None and l < L) else None
        if arch != "sage":
            gw, gb, gx = gcn_layer_bwd(blk, means[l - 1], h_l, gh, weights[l - 1][0], relu=(l < L),
                                       need_grad_x=(l > 1), active=active, norm=gcn_norm_of(arch))
            grads[l - 1] = (gw, gb)
        else:
            w_self, w_neigh, _ = weights[l - 1]
            gws, gwn, gb, gx = sage_layer_bwd(blk, xs[l - 1], means[l - 1], h_l, gh, w_self, w_neigh,
                                              relu=(l < L), need_grad_x=(l > 1), active=active,
                                              bf16_products=bf16_products and l == 1)
            grads[l - 1] = (gws, gwn, gb)
        gh = gx
    new_w = [tuple(np.asarray(p, np.float64) - lr * q for p, q in zip(w, gr)) for w, gr in zip(weights, grads)]
    if use_cache:
        # every computed hot vertex refreshes its slot with the embedding made by step-t weights
        v1_computed = bottom.dst_global
        slots = cache.slot_of_vertex[v1_computed]
        sel = slots >= 0
        cache.emb[slots[sel]] = hs[0][sb.compute_pos][sel]
        cache.version[slots[sel]] = step
    return StepResult(loss, sb, x0, hs, means, grads, new_w, 0 if not use_cache else len(sb.hit_pos))


# --------------------------------------------------------------------------- bulk refresh (Section 4.2)

def refresh_hot(g: Graph, feat: np.ndarray, cache: Cache, layer1_weights, fanout: int, version: int, seed: int,
                feat_is_bf16: bool = False, norm: str = "mean"):
    """Stage 2 of Section 4.2 for one super-batch: the layer-1 embedding of EVERY hot vertex, from a one-hop
    sample at the bottom fanout and the given (snapshot of the) layer-1 parameters. Row i belongs to
    hot_ids[i]. Returns the pending cache contents (emb [n_hot, d1] fp64, version [n_hot] = `version`);
    they replace the cache at the next super-batch boundary (`commit_refresh`).
    Sampling stream: Philox key seed + version, domain DOMAIN_REFRESH, hop 0."""
    blk = sample_hop(g, cache.hot_ids, fanout, _u64(seed + version), DOMAIN_REFRESH, 0)
    x = _to_f64(gather_features(feat, blk.src_global), feat_is_bf16)
    if len(layer1_weights) == 2:          # GCN-style layer: (w, bias)
        _, h = gcn_layer_fwd(blk, x, layer1_weights[0], layer1_weights[1], relu=True, norm=norm)
    else:
        w_self, w_neigh, bias = layer1_weights
        _, h = sage_layer_fwd(blk, x, w_self, w_neigh, bias, relu=True)
    return h, np.full(cache.n_hot, version, dtype=np.int32)


def commit_refresh(cache: Cache, emb: np.ndarray, version: np.ndarray) -> None:
    """Super-batch boundary: the pending rows become the cache contents."""
    cache.emb[...] = emb
    cache.version[...] = version


def train_superbatches(g: Graph, feat: np.ndarray, labels: np.ndarray, batches: Sequence[np.ndarray],
                       fanouts: Sequence[int], weights, lr: float, seed: int, cache: Cache, n: int,
                       feat_is_bf16: bool = False, on_step=None, arch: str = "sage"):
    """The schedule of Section 4.2 in its sequential meaning. At every step t with t % n == 0 the rows
    computed during the previous super-batch are committed, then the refresh for the next super-batch is
    computed from the parameters as they stand before step t (version t). Steps are Algorithm 1 with reuse
    under the cache's bound S (S = 2n - 1 lets every committed row serve its whole super-batch).
    Returns the list of StepResult and the final weights."""
    pending = None
    out = []
    for t, seeds in enumerate(batches):
        if t % n == 0:
            if pending is not None:
                commit_refresh(cache, *pending)
            pending = refresh_hot(g, feat, cache, weights[0], fanouts[-1], t, seed, feat_is_bf16,
                                  norm="mean" if arch == "sage" else gcn_norm_of(arch))
        r = train_step(g, feat, labels, seeds, fanouts, weights, lr, seed, t, cache, feat_is_bf16, arch=arch)
        if on_step is not None:
            on_step(t, r, cache)
        weights = r.new_weights
        out.append(r)
    return out, weights


# --------------------------------------------------------------------------- weight-drift monitor (Section 4.3)

def max_weight_update(old_weights, new_weights) -> float:
    """Largest change of any entry of the given parameter arrays in one update (the paper's max delta ||W||)."""
    return max(float(np.abs(np.asarray(b, np.float64) - np.asarray(a, np.float64)).max())
               for a, b in zip(old_weights, new_weights))


def weight_drift(weights, snapshot) -> float:
    """max |W - W~| between the current parameters and the ones a set of stale embeddings was made with."""
    return max_weight_update(snapshot, weights)


def drift_tolerance(max_update: float, n: int) -> float:
    """The tolerated drift of Section 4.3: epsilon = (largest single-update change) x 2n."""
    return max_update * 2 * n
