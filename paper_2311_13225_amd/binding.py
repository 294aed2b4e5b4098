"""Thin ctypes binding of libneutronorch.so: argument marshalling only.

Function names follow the C ABI (include/neutronorch.h). PyTorch is used for device memory
(tensors in, tensor views of library-owned buffers out) and for the current HIP stream; every
step of the path runs in the library's kernels. There is no CPU fallback: a missing library or a
failing call raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libneutronorch.so")

NO_F32, NO_BF16 = 0, 1
NO_ARCH_SAGE_MEAN, NO_ARCH_GCN, NO_ARCH_GCN_SUM, NO_ARCH_GCN_SYM = 0, 1, 2, 3
ARCH_OF_NAME = {"sage": NO_ARCH_SAGE_MEAN, "gcn": NO_ARCH_GCN, "gcn_sum": NO_ARCH_GCN_SUM, "gcn_sym": NO_ARCH_GCN_SYM}
NO_CSR_INPUT_ON_DEVICE, NO_CSR_IDS_64, NO_CSR_SYMMETRISE, NO_CSR_DEDUP = 1, 2, 4, 8
NO_MAX_LAYERS = 8
ERROR_NAMES = {0: "NO_OK", -1: "NO_ERR_INVALID_ARG", -2: "NO_ERR_OUT_OF_RANGE", -3: "NO_ERR_CAPACITY",
               -4: "NO_ERR_OVERFLOW", -5: "NO_ERR_HIP", -6: "NO_ERR_UNSUPPORTED", -7: "NO_ERR_TIMEOUT"}


class NoError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("%s (%d): %s" % (ERROR_NAMES.get(code, "?"), code, msg))
        self.code = code


class no_block_view(C.Structure):
    _fields_ = [("n_dst_cap", C.c_int32), ("n_src_cap", C.c_int32), ("nnz_cap", C.c_int32),
                ("d_n_dst", C.c_void_p), ("d_n_src", C.c_void_p), ("d_nnz", C.c_void_p),
                ("d_dst_global", C.c_void_p), ("d_src_global", C.c_void_p), ("d_indptr", C.c_void_p),
                ("d_nbr_global", C.c_void_p), ("d_indices", C.c_void_p), ("d_csc_indptr", C.c_void_p),
                ("d_csc_dst", C.c_void_p), ("d_csc_eid", C.c_void_p), ("d_compute_pos", C.c_void_p),
                ("d_hit_pos", C.c_void_p), ("d_hit_slot", C.c_void_p), ("d_n_compute", C.c_void_p),
                ("d_n_hit", C.c_void_p)]


class no_step_stats(C.Structure):
    _fields_ = [("loss", C.c_float), ("n_dst", C.c_int32 * NO_MAX_LAYERS), ("n_src", C.c_int32 * NO_MAX_LAYERS),
                ("nnz", C.c_int32 * NO_MAX_LAYERS), ("n_hit", C.c_int32), ("n_refresh", C.c_int32),
                ("n_v1", C.c_int32), ("bad_seed", C.c_int32), ("n_miss_hot", C.c_int32), ("n_cold", C.c_int32),
                ("scan_timeout", C.c_int32), ("bad_label", C.c_int32), ("bytes_gathered_features", C.c_int64),
                ("bytes_gathered_embeddings", C.c_int64)]


_lib = None
_P, _I32, _I64, _U32, _U64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_uint64

_SIGNATURES = {
    "no_last_error": (C.c_char_p, []),
    "no_build_csr": (_I32, [_P, _P, _I64, _I64, _I32, _U32, _P, _P]),
    "no_graph_view": (_I32, [_P, _P, _P, _P, _P, _P]),
    "no_graph_destroy": (_I32, [_P]),
    "no_blocks_create": (_I32, [_P, _I32, _P, _I32, _P]),
    "no_sample_blocks": (_I32, [_P, _P, _I32, _U64, _I64, _P, _P, _P]),
    "no_blocks_view": (_I32, [_P, _I32, _P]),
    "no_blocks_sizes": (_I32, [_P, _P, _P]),
    "no_blocks_destroy": (_I32, [_P]),
    "no_select_hot": (_I32, [_P, _P, _I64, _I32, _P, _I32, _I32, C.c_double, _I32, _I32, _U64, _P, _P]),
    "no_cache_view": (_I32, [_P, _P, _P, _P, _P, _P, _P, _P, _P]),
    "no_cache_set_staleness": (_I32, [_P, _I32]),
    "no_cache_invalidate": (_I32, [_P, _P]),
    "no_cache_destroy": (_I32, [_P]),
    "no_refresh_hot_begin": (_I32, [_P, _P, _P, _I32, _I32, _P, _P, _P, _I32, _I64, _U64, _P]),
    "no_refresh_hot_commit": (_I32, [_P, _P]),
    "no_gather_features": (_I32, [_P, _I32, _I64, _I32, _I64, _P, _P, _I32, _P, _I64, _P]),
    "no_sage_layer_ws_bytes": (C.c_size_t, [_I32, _I32, _I32, _I32]),
    "no_sage_layer_fwd": (_I32, [_P, _P, _I32, _I32, _P, _P, _P, _I32, _I32, _P, _P, _P, C.c_size_t, _P]),
    "no_sage_layer_bwd": (_I32, [_P, _P, _I32, _I32, _P, _P, _P, _P, _P, _I32, _I32, _P, _P, _P, _P, _P,
                                 C.c_size_t, _P]),
    "no_sage_layer_bwd_static": (_I32, [_P, _P, _I32, _I32, _P, _P, _P, _P, _P, _I32, _I32, _P, _P, _P, _P, _P]),
    "no_model_create": (_I32, [_P, _I32, _P, _I32, _P, _I32, _P]),
    "no_model_params": (_I32, [_P, _I32, _P, _P, _P]),
    "no_model_grads": (_I32, [_P, _I32, _P, _P, _P]),
    "no_model_set_arch": (_I32, [_P, _I32]),
    "no_gcn_layer_fwd": (_I32, [_P, _I32, _P, _I32, _I32, _P, _P, _I32, _I32, _P, _P, _P, C.c_size_t, _P]),
    "no_gcn_layer_bwd": (_I32, [_P, _I32, _I32, _P, _P, _P, _P, _I32, _I32, _P, _P, _P, _P, C.c_size_t, _P]),
    "no_cache_set_layer_form": (_I32, [_P, _I32]),
    "no_model_activations": (_I32, [_P, _I32, _P, _P]),
    "no_model_blocks": (_I32, [_P, _P]),
    "no_model_gathered": (_I32, [_P, _P]),
    "no_train_step": (_I32, [_P, _P, _P, _P, _P, _I32, _P, _I64, _U64, C.c_float, _P, _P, _P]),
    "no_train_step_ahead": (_I32, [_P, _P, _P, _P, _P, _I32, _P, _I32, _I32, _P, _I64, _U64, C.c_float, _P, _P, _P]),
    "no_model_weight_drift": (_I32, [_P, _P, C.c_float, _P, _P, _P]),
    "no_model_destroy": (_I32, [_P]),
    "no_model_profile": (_I32, [_P, _I32]),
    "no_model_stage_ms": (_I32, [_P, _P, _P]),
    "no_stage_name": (C.c_char_p, [_I32]),
    "no_debug_scan_wait": (_I32, [_I32, _I32]),
}
NO_STAGE_COUNT = 12
EXPORTS = sorted(_SIGNATURES)


def lib():
    """Loads the HIP library; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libneutronorch.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def _check(code: int, stats=None):
    if code != 0:
        e = NoError(code, lib().no_last_error().decode())
        e.stats = stats          # a step that fails after its statistics were copied back still hands them over
        raise e


def _stream(stream=None) -> int:
    if stream is None:
        return int(torch.cuda.current_stream().cuda_stream)
    return int(getattr(stream, "cuda_stream", stream))


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


class _DevArray:
    def __init__(self, ptr: int, shape: Tuple[int, ...], typestr: str, owner):
        self.__cuda_array_interface__ = {"shape": tuple(shape), "typestr": typestr, "data": (int(ptr), False),
                                         "version": 2, "strides": None}
        self._owner = owner


def _view(ptr: Optional[int], shape, typestr: str, owner) -> Optional[torch.Tensor]:
    """Torch view of library-owned device memory (no copy)."""
    if not ptr:
        return None
    n = int(np.prod(shape))
    if n == 0:
        dt = {"<i4": torch.int32, "<i8": torch.int64, "<f4": torch.float32, "<u2": torch.int16}[typestr]
        return torch.empty(tuple(shape), dtype=dt, device="cuda")
    if typestr == "<u2":
        t = torch.as_tensor(_DevArray(ptr, shape, "<i2", owner), device="cuda")
    else:
        t = torch.as_tensor(_DevArray(ptr, shape, typestr, owner), device="cuda")
    t._no_owner = owner
    return t


def _i32_host(vals: Sequence[int]):
    return (C.c_int32 * len(vals))(*[int(v) for v in vals])


# ------------------------------------------------------------------------------------------ handles

class _Handle:
    _destroy = None

    def __init__(self, h):
        self.h = h

    def close(self):
        if self.h:
            getattr(lib(), self._destroy)(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Graph(_Handle):
    _destroy = "no_graph_destroy"


class Blocks(_Handle):
    _destroy = "no_blocks_destroy"
    n_layers = 0
    owned = True

    def close(self):
        if self.owned:
            super().close()
        self.h = None


class Cache(_Handle):
    _destroy = "no_cache_destroy"


class Model(_Handle):
    _destroy = "no_model_destroy"
    n_layers = 0
    dims: List[int] = []
    feat_dtype = NO_F32


# ------------------------------------------------------------------------------------------ graph

def no_build_csr(src, dst, n_vertices: int, rowptr_bits: int = 64, stream=None, symmetrise: bool = False,
                 dedup: bool = False) -> Graph:
    """src, dst: int32 or int64 numpy arrays (host) or CUDA tensors (device)."""
    on_device = isinstance(src, torch.Tensor) and src.is_cuda
    if on_device:
        assert src.dtype == dst.dtype and src.dtype in (torch.int32, torch.int64) and src.is_contiguous() and dst.is_contiguous()
        ids64 = src.dtype == torch.int64
        ps, pd, n = src.data_ptr(), dst.data_ptr(), src.numel()
    else:
        ids64 = np.asarray(src).dtype == np.int64
        src = np.ascontiguousarray(src, dtype=np.int64 if ids64 else np.int32)
        dst = np.ascontiguousarray(dst, dtype=np.int64 if ids64 else np.int32)
        ps, pd, n = src.ctypes.data, dst.ctypes.data, len(src)
    assert len(dst) == n
    torch.cuda.init()
    out = C.c_void_p()
    flags = (NO_CSR_INPUT_ON_DEVICE if on_device else 0) | (NO_CSR_IDS_64 if ids64 else 0) | \
            (NO_CSR_SYMMETRISE if symmetrise else 0) | (NO_CSR_DEDUP if dedup else 0)
    _check(lib().no_build_csr(ps, pd, n, n_vertices, rowptr_bits, flags, _stream(stream), C.byref(out)))
    return Graph(out)


def no_graph_view(g: Graph):
    """(V, E, rowptr_bits, rowptr tensor, col tensor) - tensors alias the graph's memory."""
    v, e, bits = C.c_int64(), C.c_int64(), C.c_int32()
    rp, col = C.c_void_p(), C.c_void_p()
    _check(lib().no_graph_view(g.h, C.byref(v), C.byref(e), C.byref(bits), C.byref(rp), C.byref(col)))
    rowptr = _view(rp.value, (v.value + 1,), "<i8" if bits.value == 64 else "<i4", g)
    return v.value, e.value, bits.value, rowptr, _view(col.value, (e.value,), "<i4", g)


# ------------------------------------------------------------------------------------------ blocks

def no_blocks_create(g: Graph, n_seeds_cap: int, fanouts: Sequence[int]) -> Blocks:
    out = C.c_void_p()
    _check(lib().no_blocks_create(g.h, n_seeds_cap, _i32_host(fanouts), len(fanouts), C.byref(out)))
    b = Blocks(out)
    b.n_layers = len(fanouts)
    return b


def no_sample_blocks(g: Graph, seeds: torch.Tensor, seed: int, step: int, cache: Optional[Cache], blocks: Blocks,
                     stream=None):
    assert seeds.is_cuda and seeds.dtype == torch.int32 and seeds.is_contiguous()
    _check(lib().no_sample_blocks(g.h, seeds.data_ptr(), seeds.numel(), seed & 0xFFFFFFFFFFFFFFFF, step,
                                  cache.h if cache is not None else None, blocks.h, _stream(stream)))


def no_blocks_view(blocks: Blocks, hop: int) -> no_block_view:
    v = no_block_view()
    _check(lib().no_blocks_view(blocks.h, hop, C.byref(v)))
    v._owner = blocks
    return v


def no_blocks_sizes(blocks: Blocks, stream=None) -> np.ndarray:
    """[n_layers, 4] int32: n_dst, n_src, nnz, n_hit per hop (synchronises)."""
    buf = (C.c_int32 * (4 * blocks.n_layers))()
    _check(lib().no_blocks_sizes(blocks.h, _stream(stream), buf))
    return np.array(buf, dtype=np.int32).reshape(blocks.n_layers, 4)


def block_arrays(blocks: Blocks, hop: int, sizes: np.ndarray) -> dict:
    """Host copies of one block's arrays, trimmed to their actual sizes."""
    v = no_blocks_view(blocks, hop)
    n_dst, n_src, nnz, n_hit = [int(x) for x in sizes[hop]]

    def get(ptr, n):
        t = _view(ptr, (n,), "<i4", blocks)
        return None if t is None else t.cpu().numpy()

    d = {"dst_global": get(v.d_dst_global, n_dst), "src_global": get(v.d_src_global, n_src),
         "indptr": get(v.d_indptr, n_dst + 1), "nbr_global": get(v.d_nbr_global, nnz),
         "indices": get(v.d_indices, nnz), "csc_indptr": get(v.d_csc_indptr, n_src + 1),
         "csc_dst": get(v.d_csc_dst, nnz), "csc_eid": get(v.d_csc_eid, nnz)}
    if v.d_compute_pos:
        d["compute_pos"] = get(v.d_compute_pos, n_dst)
        d["hit_pos"] = get(v.d_hit_pos, n_hit)
        d["hit_slot"] = get(v.d_hit_slot, n_hit)
    return d


def block_view_from_tensors(n_dst: torch.Tensor, n_src: torch.Tensor, indptr: torch.Tensor, indices: torch.Tensor,
                            n_dst_cap: int, n_src_cap: int, csc_indptr: Optional[torch.Tensor] = None,
                            csc_dst: Optional[torch.Tensor] = None) -> no_block_view:
    """A view over caller-owned int32 CUDA tensors (n_dst / n_src are 1-element tensors)."""
    v = no_block_view()
    v.n_dst_cap, v.n_src_cap, v.nnz_cap = n_dst_cap, n_src_cap, int(indices.numel())
    v.d_n_dst, v.d_n_src = n_dst.data_ptr(), n_src.data_ptr()
    v.d_indptr, v.d_indices = indptr.data_ptr(), indices.data_ptr()
    v.d_csc_indptr, v.d_csc_dst = _ptr(csc_indptr), _ptr(csc_dst)
    v._keep = (n_dst, n_src, indptr, indices, csc_indptr, csc_dst)
    return v


# ------------------------------------------------------------------------------------------ cache

def no_select_hot(g: Graph, train_ids: torch.Tensor, batch: int, fanouts: Sequence[int], presample_epochs: int,
                  hot_fraction: float, staleness: int, emb_dim: int, seed: int, stream=None) -> Cache:
    assert train_ids.is_cuda and train_ids.dtype == torch.int32 and train_ids.is_contiguous()
    out = C.c_void_p()
    _check(lib().no_select_hot(g.h, train_ids.data_ptr(), train_ids.numel(), batch, _i32_host(fanouts), len(fanouts),
                               presample_epochs, float(hot_fraction), staleness, emb_dim, seed & 0xFFFFFFFFFFFFFFFF,
                               _stream(stream), C.byref(out)))
    return Cache(out)


def no_cache_view(c: Cache, n_vertices: int) -> dict:
    """Tensor views of the cache: hot_ids, slot_of_vertex, version, emb, freq (aliases, no copies)."""
    n_hot, s, d = C.c_int64(), C.c_int32(), C.c_int32()
    p = [C.c_void_p() for _ in range(5)]
    _check(lib().no_cache_view(c.h, C.byref(n_hot), C.byref(s), C.byref(d), *[C.byref(x) for x in p]))
    nh, dim = n_hot.value, d.value
    return {"n_hot": nh, "staleness": s.value, "emb_dim": dim,
            "hot_ids": _view(p[0].value, (nh,), "<i4", c), "slot_of_vertex": _view(p[1].value, (n_vertices,), "<i4", c),
            "version": _view(p[2].value, (nh,), "<i4", c), "emb": _view(p[3].value, (nh, dim), "<f4", c),
            "freq": _view(p[4].value, (n_vertices,), "<i4", c)}


def no_cache_set_staleness(c: Cache, staleness: int):
    _check(lib().no_cache_set_staleness(c.h, staleness))


def no_cache_set_layer_form(c: Cache, form: int):
    _check(lib().no_cache_set_layer_form(c.h, form))


def no_cache_invalidate(c: Cache, stream=None):
    _check(lib().no_cache_invalidate(c.h, _stream(stream)))


def no_refresh_hot_begin(c: Cache, g: Graph, features: torch.Tensor, w_self: torch.Tensor, w_neigh: torch.Tensor,
                         bias: torch.Tensor, fanout: int, version: int, seed: int, stream=None):
    """Starts the bulk refresh of all hot embeddings into the pending copy of the cache (own stream)."""
    assert features.is_cuda and features.dim() == 2 and features.is_contiguous()
    for t in (w_self, w_neigh, bias):
        assert t is None or (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous())
    _check(lib().no_refresh_hot_begin(c.h, g.h, features.data_ptr(), _dtype_code(features), features.shape[1],
                                      w_self.data_ptr(), None if w_neigh is None else w_neigh.data_ptr(),
                                      bias.data_ptr(), fanout, version,
                                      seed & 0xFFFFFFFFFFFFFFFF, _stream(stream)))


def no_refresh_hot_commit(c: Cache, stream=None):
    """The pending rows become the cache contents (views from no_cache_view taken earlier name the other copy)."""
    _check(lib().no_refresh_hot_commit(c.h, _stream(stream)))


# ------------------------------------------------------------------------------------------ gather

def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return NO_F32
    if t.dtype in (torch.bfloat16, torch.int16, torch.uint16):
        return NO_BF16
    raise TypeError("features must be float32 or bfloat16 (or 16-bit integer bit patterns)")


def no_gather_features(table: torch.Tensor, ids: torch.Tensor, out: Optional[torch.Tensor] = None,
                       n_ids: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """out[i,:] = table[ids[i],:]; n_ids (1-element int32 CUDA tensor) limits the rows copied."""
    assert table.is_cuda and table.dim() == 2 and table.stride(1) == 1
    assert ids.is_cuda and ids.dtype == torch.int32 and ids.is_contiguous()
    if out is None:
        out = torch.empty((ids.numel(), table.shape[1]), dtype=table.dtype, device=table.device)
    assert out.stride(1) == 1 and out.dtype == table.dtype
    es = table.element_size()
    _check(lib().no_gather_features(table.data_ptr(), _dtype_code(table), table.shape[0], table.shape[1],
                                    table.stride(0) * es, ids.data_ptr(), _ptr(n_ids), ids.numel(), out.data_ptr(),
                                    out.stride(0) * es, _stream(stream)))
    return out


# ------------------------------------------------------------------------------------------ layers

def no_sage_layer_ws_bytes(n_dst_cap: int, n_src_cap: int, d_in: int, d_out: int) -> int:
    return int(lib().no_sage_layer_ws_bytes(n_dst_cap, n_src_cap, d_in, d_out))


def no_sage_layer_fwd(blk: no_block_view, x_src: torch.Tensor, w_self: torch.Tensor, w_neigh: torch.Tensor,
                      bias: torch.Tensor, relu: bool, mean: torch.Tensor, h: torch.Tensor, ws: torch.Tensor, stream=None):
    d_in, d_out = w_self.shape
    _check(lib().no_sage_layer_fwd(C.byref(blk), x_src.data_ptr(), _dtype_code(x_src), d_in, w_self.data_ptr(),
                                   w_neigh.data_ptr(), bias.data_ptr(), d_out, 1 if relu else 0, mean.data_ptr(),
                                   h.data_ptr(), ws.data_ptr(), ws.numel() * ws.element_size(), _stream(stream)))


def no_sage_layer_bwd(blk: no_block_view, x_src: torch.Tensor, mean: torch.Tensor, h: torch.Tensor,
                      grad_h: torch.Tensor, w_self: torch.Tensor, w_neigh: torch.Tensor, relu: bool,
                      gw_self: torch.Tensor, gw_neigh: torch.Tensor, gbias: torch.Tensor,
                      grad_x_src: Optional[torch.Tensor], ws: torch.Tensor, stream=None):
    d_in, d_out = w_self.shape
    _check(lib().no_sage_layer_bwd(C.byref(blk), x_src.data_ptr(), _dtype_code(x_src), d_in, mean.data_ptr(),
                                   h.data_ptr(), grad_h.data_ptr(), w_self.data_ptr(), w_neigh.data_ptr(), d_out,
                                   1 if relu else 0, gw_self.data_ptr(), gw_neigh.data_ptr(), gbias.data_ptr(),
                                   _ptr(grad_x_src), ws.data_ptr(), ws.numel() * ws.element_size(), _stream(stream)))


NO_LAYER_STATIC_WS_BYTES = 64 << 20


def no_sage_layer_bwd_static(blk: no_block_view, x_src: torch.Tensor, mean: torch.Tensor, h: torch.Tensor,
                             grad_h: torch.Tensor, w_self: torch.Tensor, w_neigh: torch.Tensor, relu: bool,
                             gw_self: torch.Tensor, gw_neigh: torch.Tensor, gbias: torch.Tensor,
                             grad_x_src: Optional[torch.Tensor], stream=None):
    """no_sage_layer_bwd with the workspace in the library's static device array (allocates nothing)."""
    d_in, d_out = w_self.shape
    _check(lib().no_sage_layer_bwd_static(C.byref(blk), x_src.data_ptr(), _dtype_code(x_src), d_in, mean.data_ptr(),
                                          h.data_ptr(), grad_h.data_ptr(), w_self.data_ptr(), w_neigh.data_ptr(), d_out,
                                          1 if relu else 0, gw_self.data_ptr(), gw_neigh.data_ptr(), gbias.data_ptr(),
                                          _ptr(grad_x_src), _stream(stream)))


def no_gcn_layer_fwd(blk: no_block_view, x_src: torch.Tensor, w: torch.Tensor, bias: torch.Tensor, relu: bool,
                     agg: torch.Tensor, h: torch.Tensor, ws: torch.Tensor, stream=None, form: int = NO_ARCH_GCN):
    d_in, d_out = w.shape
    _check(lib().no_gcn_layer_fwd(C.byref(blk), form, x_src.data_ptr(), _dtype_code(x_src), d_in, w.data_ptr(), bias.data_ptr(),
                                  d_out, 1 if relu else 0, agg.data_ptr(), h.data_ptr(), ws.data_ptr(),
                                  ws.numel() * ws.element_size(), _stream(stream)))


def no_gcn_layer_bwd(blk: no_block_view, agg: torch.Tensor, h: torch.Tensor, grad_h: torch.Tensor, w: torch.Tensor,
                     relu: bool, gw: torch.Tensor, gbias: torch.Tensor, grad_x_src: Optional[torch.Tensor],
                     ws: torch.Tensor, stream=None, form: int = NO_ARCH_GCN):
    d_in, d_out = w.shape
    _check(lib().no_gcn_layer_bwd(C.byref(blk), form, d_in, agg.data_ptr(), h.data_ptr(), grad_h.data_ptr(), w.data_ptr(), d_out,
                                  1 if relu else 0, gw.data_ptr(), gbias.data_ptr(), _ptr(grad_x_src), ws.data_ptr(),
                                  ws.numel() * ws.element_size(), _stream(stream)))


# ------------------------------------------------------------------------------------------ model / step

def no_model_create(g: Graph, dims: Sequence[int], n_seeds_cap: int, fanouts: Sequence[int],
                    feat_dtype: int = NO_F32) -> Model:
    out = C.c_void_p()
    _check(lib().no_model_create(g.h, len(fanouts), _i32_host(dims), n_seeds_cap, _i32_host(fanouts), feat_dtype,
                                 C.byref(out)))
    m = Model(out)
    m.n_layers, m.dims, m.feat_dtype = len(fanouts), [int(d) for d in dims], feat_dtype
    return m


def no_model_set_arch(m: Model, arch: int):
    """NO_ARCH_SAGE_MEAN (default) or NO_ARCH_GCN for every layer; call before the first step."""
    _check(lib().no_model_set_arch(m.h, arch))
    m.arch = arch


def _three(fn, m: Model, layer: int):
    a, b, c = C.c_void_p(), C.c_void_p(), C.c_void_p()
    _check(fn(m.h, layer, C.byref(a), C.byref(b), C.byref(c)))
    d_in, d_out = m.dims[layer - 1], m.dims[layer]
    return (_view(a.value, (d_in, d_out), "<f4", m), _view(b.value, (d_in, d_out), "<f4", m),
            _view(c.value, (d_out,), "<f4", m))


def no_model_params(m: Model, layer: int):
    """(w_self, w_neigh, bias) tensor views of layer `layer` (1-based); write initial values into them."""
    return _three(lib().no_model_params, m, layer)


def no_model_grads(m: Model, layer: int):
    return _three(lib().no_model_grads, m, layer)


def no_model_activations(m: Model, layer: int, n_rows: int, n_dst: int):
    a, b = C.c_void_p(), C.c_void_p()
    _check(lib().no_model_activations(m.h, layer, C.byref(a), C.byref(b)))
    return (_view(a.value, (n_rows, m.dims[layer]), "<f4", m), _view(b.value, (n_dst, m.dims[layer - 1]), "<f4", m))


def no_model_blocks(m: Model) -> Blocks:
    out = C.c_void_p()
    _check(lib().no_model_blocks(m.h, C.byref(out)))
    b = Blocks(out)
    b.owned = False
    b.n_layers = m.n_layers
    b._model = m
    return b


def no_model_gathered(m: Model, n_rows: int) -> torch.Tensor:
    out = C.c_void_p()
    _check(lib().no_model_gathered(m.h, C.byref(out)))
    return _view(out.value, (n_rows, m.dims[0]), "<f4" if m.feat_dtype == NO_F32 else "<u2", m)


def no_train_step(m: Model, g: Graph, features: torch.Tensor, labels: torch.Tensor, seeds: torch.Tensor,
                  cache: Optional[Cache], step: int, seed: int, lr: float, want_stats: bool = True,
                  stream=None) -> Optional[no_step_stats]:
    assert features.is_cuda and features.is_contiguous() and features.shape[1] == m.dims[0]
    assert _dtype_code(features) == m.feat_dtype
    assert labels.is_cuda and labels.dtype == torch.int32 and labels.is_contiguous()
    assert seeds.is_cuda and seeds.dtype == torch.int32 and seeds.is_contiguous()
    hs = no_step_stats() if want_stats else None
    _check(lib().no_train_step(m.h, g.h, features.data_ptr(), labels.data_ptr(), seeds.data_ptr(), seeds.numel(),
                               cache.h if cache is not None else None, step, seed & 0xFFFFFFFFFFFFFFFF, lr, None,
                               C.byref(hs) if want_stats else None, _stream(stream)), hs)
    return hs


def no_train_step_ahead(m: Model, g: Graph, features: torch.Tensor, labels: torch.Tensor, seeds: torch.Tensor,
                        next_seeds: Optional[torch.Tensor], commit_refresh_before_next: bool, cache: Optional[Cache],
                        step: int, seed: int, lr: float, want_stats: bool = True, stream=None) -> Optional[no_step_stats]:
    """no_train_step that also samples batch step + 1 (next_seeds) on the model's sampling stream while this batch
    trains. Pass the SAME tensor as `seeds` of the next call, or the sample is dropped."""
    assert features.is_cuda and features.is_contiguous() and features.shape[1] == m.dims[0]
    assert _dtype_code(features) == m.feat_dtype
    assert labels.is_cuda and labels.dtype == torch.int32 and labels.is_contiguous()
    for t in (seeds, next_seeds):
        assert t is None or (t.is_cuda and t.dtype == torch.int32 and t.is_contiguous())
    hs = no_step_stats() if want_stats else None
    _check(lib().no_train_step_ahead(m.h, g.h, features.data_ptr(), labels.data_ptr(), seeds.data_ptr(), seeds.numel(),
                                     None if next_seeds is None else next_seeds.data_ptr(),
                                     0 if next_seeds is None else next_seeds.numel(),
                                     1 if commit_refresh_before_next else 0,
                                     cache.h if cache is not None else None, step, seed & 0xFFFFFFFFFFFFFFFF, lr, None,
                                     C.byref(hs) if want_stats else None, _stream(stream)), hs)
    return hs


def no_model_weight_drift(m: Model, cache: Optional[Cache], lr: float, stream=None) -> Tuple[float, float]:
    """(largest change of a layer-1 parameter in the last update, drift from the snapshot behind the committed rows
    or -1): the two quantities of the weight-drift monitor. Synchronises the stream."""
    a, d = C.c_float(), C.c_float()
    _check(lib().no_model_weight_drift(m.h, cache.h if cache is not None else None, lr, C.byref(a), C.byref(d),
                                       _stream(stream)))
    return a.value, d.value


def no_model_profile(m: Model, enable: bool):
    _check(lib().no_model_profile(m.h, 1 if enable else 0))


def no_model_stage_ms(m: Model) -> Tuple[dict, int]:
    """({stage name: summed milliseconds}, steps accumulated) since profiling was enabled."""
    ms = (C.c_double * NO_STAGE_COUNT)()
    steps = C.c_int32()
    _check(lib().no_model_stage_ms(m.h, ms, C.byref(steps)))
    return {lib().no_stage_name(i).decode(): float(ms[i]) for i in range(NO_STAGE_COUNT)}, steps.value


def no_debug_scan_wait(spin_limit: int = 0, withhold_first_tile: bool = False):
    """Test aid: spin limit of the single-pass scans' bounded waits (0 = default) and whether tile 0 withholds its word."""
    _check(lib().no_debug_scan_wait(spin_limit, 1 if withhold_first_tile else 0))
