"""Thin ctypes layer over ``libgs.so``: same names as ``include/gs.h``.

Argument marshalling only.  Tensors are torch CUDA tensors used as plain
device buffers; each call passes ``data_ptr()`` values and the current torch
stream to the C entry point.  There is no CPU or torch fallback: if the shared
library is missing, or a tensor is not on the GPU, the call raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgs.so")

GS_OK, GS_EINVAL, GS_EWORKSPACE, GS_EOVERFLOW, GS_EHIP = 0, -1, -2, -3, -4
GS_SYMMETRIZE, GS_DROP_SELF_LOOPS, GS_DEDUPE = 1, 2, 4
GS_F32, GS_BF16, GS_F16 = 0, 1, 2

EXPORTS = (
    "gs_last_hip_error",
    "gs_csr_build_workspace_bytes", "gs_csr_build",
    "gs_alias_build_workspace_bytes", "gs_alias_build", "gs_alias_pack",
    "gs_random_walk", "gs_node2vec_walk",
    "gs_make_pairs_workspace_bytes", "gs_make_pairs",
    "gs_sample_negatives", "gs_sample_edges",
    "gs_sgns_step_workspace_bytes", "gs_sgns_step", "gs_sgns_step_static", "gs_sgns_momentum_step",
    "gs_sgns_adam_step",
    "gs_sgns_step_fused_workspace_bytes", "gs_sgns_step_fused",
    "gs_pair_offsets_workspace_bytes", "gs_pair_offsets",
    "gs_sgns_step_from_walks_workspace_bytes", "gs_sgns_step_from_walks",
    "gs_line1_step_workspace_bytes", "gs_line1_step",
    "gs_unique_ids_workspace_bytes", "gs_unique_ids", "gs_get_rows", "gs_put_rows",
    "gs_table_mult", "gs_table_mult_add", "gs_sort_pairs_workspace_bytes", "gs_sort_pairs",
)


class GsError(RuntimeError):
    def __init__(self, what: str, status: int, hip: int = 0):
        names = {-1: "GS_EINVAL", -2: "GS_EWORKSPACE", -3: "GS_EOVERFLOW", -4: "GS_EHIP"}
        msg = f"{what}: {names.get(status, status)}"
        if status == GS_EHIP:
            msg += f" (hip error {hip})"
        super().__init__(msg)
        self.status = status


class CsrStruct(C.Structure):
    _fields_ = [("num_nodes", C.c_int64), ("num_entries", C.c_int64),
                ("offsets", C.c_void_p), ("offset_bits", C.c_int32),
                ("nbrs", C.c_void_p), ("weights", C.c_void_p)]


class AliasStruct(C.Structure):
    _fields_ = [("prob", C.c_void_p), ("alias", C.c_void_p), ("packed", C.c_void_p)]


_lib = None


def lib() -> C.CDLL:
    """Opens libgs.so (built by ``paper_2407_15452_amd.build``); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2407_15452_amd.build`; "
                "there is no fallback path")
        l = C.CDLL(LIB_PATH)
        for name in EXPORTS:
            fn = getattr(l, name)
            fn.restype = C.c_size_t if name.endswith("_workspace_bytes") else C.c_int32
        _lib = l
    return _lib


def _dev(t, dtype=None, name="tensor"):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a CUDA tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must have dtype {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc, what):
    if rc != GS_OK:
        raise GsError(what, rc, lib().gs_last_hip_error() if rc == GS_EHIP else 0)


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


class Csr:
    """Device CSR (tensors + the host descriptor handed to the library)."""

    def __init__(self, offsets: torch.Tensor, nbrs: torch.Tensor, weights=None, num_entries=None):
        assert offsets.dtype in (torch.int32, torch.int64)
        self.offsets, self.nbrs, self.weights = offsets, nbrs, weights
        self.num_nodes = offsets.numel() - 1
        self.num_entries = int(nbrs.numel() if num_entries is None else num_entries)
        self.offset_bits = 64 if offsets.dtype == torch.int64 else 32
        self.struct = CsrStruct(self.num_nodes, self.num_entries, offsets.data_ptr(),
                                self.offset_bits, nbrs.data_ptr() if nbrs.numel() else None,
                                weights.data_ptr() if weights is not None else None)


class Alias:
    def __init__(self, prob: torch.Tensor, alias: torch.Tensor, packed=None):
        _dev(prob, torch.float32, "prob")
        _dev(alias, torch.int32, "alias")
        _dev(packed, torch.int64, "packed")
        self.prob, self.alias, self.packed = prob, alias, packed
        self.struct = AliasStruct(prob.data_ptr(), alias.data_ptr(),
                                  None if packed is None else packed.data_ptr())


def gs_csr_build(src, dst, w, num_nodes: int, flags: int, offset_bits: int = 32, ws=None) -> Csr:
    l = lib()
    m = int(src.numel())
    dev = src.device
    cap = max(1, m * (2 if flags & GS_SYMMETRIZE else 1))
    offsets = torch.empty(num_nodes + 1, dtype=torch.int64 if offset_bits == 64 else torch.int32,
                          device=dev)
    nbrs = torch.empty(cap, dtype=torch.int32, device=dev)
    w_out = torch.empty(cap, dtype=torch.float32, device=dev) if w is not None else None
    n_out = torch.zeros(1, dtype=torch.int64, device=dev)
    need = l.gs_csr_build_workspace_bytes(C.c_int64(m), C.c_int64(num_nodes), C.c_uint32(flags))
    if ws is None:
        ws = _workspace(need, dev)
    rc = l.gs_csr_build(_dev(src, torch.int32, "src"), _dev(dst, torch.int32, "dst"),
                        _dev(w, torch.float32, "w"), C.c_int64(m), C.c_int64(num_nodes),
                        C.c_uint32(flags), C.c_int32(offset_bits), _dev(offsets), _dev(nbrs),
                        _dev(w_out), _dev(n_out), _dev(ws), C.c_size_t(ws.numel()), _stream())
    _check(rc, "gs_csr_build")
    n = int(n_out.item())
    return Csr(offsets, nbrs[:n], None if w_out is None else w_out[:n], n)


def gs_alias_pack(prob, alias) -> torch.Tensor:
    """The table as one 8-byte word per entry (see gs.h)."""
    total = int(prob.numel())
    packed = torch.empty(max(1, total), dtype=torch.int64, device=prob.device)
    rc = lib().gs_alias_pack(_dev(prob, torch.float32, "prob"), _dev(alias, torch.int32, "alias"),
                             C.c_int64(total), _dev(packed), _stream())
    _check(rc, "gs_alias_pack")
    return packed[:total]


def gs_alias_build(seg_offsets, weights, ws=None, pack: bool = True) -> Alias:
    l = lib()
    dev = weights.device
    total = int(weights.numel())
    nseg = int(seg_offsets.numel()) - 1
    bits = 64 if seg_offsets.dtype == torch.int64 else 32
    prob = torch.empty(max(1, total), dtype=torch.float32, device=dev)
    alias = torch.empty(max(1, total), dtype=torch.int32, device=dev)
    need = l.gs_alias_build_workspace_bytes(C.c_int64(nseg), C.c_int64(total))
    if ws is None:
        ws = _workspace(need, dev)
    rc = l.gs_alias_build(_dev(seg_offsets, None, "seg_offsets"), C.c_int32(bits), C.c_int64(nseg),
                          C.c_int64(total), _dev(weights, torch.float32, "weights"), _dev(prob),
                          _dev(alias), _dev(ws), C.c_size_t(ws.numel()), _stream())
    _check(rc, "gs_alias_build")
    prob, alias = prob[:total], alias[:total]
    return Alias(prob, alias, gs_alias_pack(prob, alias) if pack and total > 0 else None)


def _alias_ref(a):
    return None if a is None else C.byref(a.struct)


def gs_random_walk(g: Csr, a, starts, walk_len: int, seed: int, walk_id_base: int = 0, out=None):
    nw = int(starts.numel())
    if out is None:
        out = torch.empty((nw, walk_len), dtype=torch.int32, device=starts.device)
    rc = lib().gs_random_walk(C.byref(g.struct), _alias_ref(a), _dev(starts, torch.int32, "starts"),
                              C.c_int64(nw), C.c_uint64(walk_id_base), C.c_int32(walk_len),
                              C.c_uint64(seed), _dev(out, torch.int32, "walks_out"), _stream())
    _check(rc, "gs_random_walk")
    return out


def gs_node2vec_walk(g: Csr, a, starts, walk_len: int, p: float, q: float, seed: int,
                     walk_id_base: int = 0, out=None):
    nw = int(starts.numel())
    if out is None:
        out = torch.empty((nw, walk_len), dtype=torch.int32, device=starts.device)
    rc = lib().gs_node2vec_walk(C.byref(g.struct), _alias_ref(a),
                                _dev(starts, torch.int32, "starts"), C.c_int64(nw),
                                C.c_uint64(walk_id_base), C.c_int32(walk_len), C.c_float(p),
                                C.c_float(q), C.c_uint64(seed), _dev(out, torch.int32, "walks_out"),
                                _stream())
    _check(rc, "gs_node2vec_walk")
    return out


def pair_capacity(num_walks: int, walk_len: int, window: int) -> int:
    """Capacity gs_make_pairs requires of its output arrays (see gs.h)."""
    if walk_len > window:
        return num_walks * (2 * window * walk_len - window * (window + 1))
    return num_walks * walk_len * (walk_len - 1)


def gs_make_pairs(walks, window: int, centers=None, contexts=None, num_pairs_out=None, ws=None,
                  sync: bool = True):
    """Returns (centers, contexts, num_pairs).  With sync=False num_pairs is the
    device scalar and the outputs are left at full capacity."""
    l = lib()
    nw, walk_len = int(walks.shape[0]), int(walks.shape[1])
    dev = walks.device
    cap = max(1, pair_capacity(nw, walk_len, window))
    if centers is None:
        centers = torch.empty(cap, dtype=torch.int32, device=dev)
    if contexts is None:
        contexts = torch.empty(cap, dtype=torch.int32, device=dev)
    if num_pairs_out is None:
        num_pairs_out = torch.zeros(1, dtype=torch.int64, device=dev)
    if ws is None:
        ws = _workspace(l.gs_make_pairs_workspace_bytes(C.c_int64(nw)), dev)
    rc = l.gs_make_pairs(_dev(walks, torch.int32, "walks"), C.c_int64(nw), C.c_int32(walk_len),
                         C.c_int32(window), _dev(centers, torch.int32), _dev(contexts, torch.int32),
                         _dev(num_pairs_out, torch.int64), _dev(ws), C.c_size_t(ws.numel()),
                         _stream())
    _check(rc, "gs_make_pairs")
    if not sync:
        return centers, contexts, num_pairs_out
    n = int(num_pairs_out.item())
    return centers[:n], contexts[:n], n


def gs_sample_negatives(noise, num_nodes: int, num_pairs: int, k: int, seed: int,
                        pair_index_base: int = 0, out=None, device=None):
    if out is None:
        dev = noise.prob.device if noise is not None else device
        out = torch.empty((num_pairs, k), dtype=torch.int32, device=dev)
    rc = lib().gs_sample_negatives(_alias_ref(noise), C.c_int64(num_nodes), C.c_int64(num_pairs),
                                   C.c_uint64(pair_index_base), C.c_int32(k), C.c_uint64(seed),
                                   _dev(out, torch.int32, "negs_out"), _stream())
    _check(rc, "gs_sample_negatives")
    return out


def gs_sample_edges(g: Csr, edge_alias, num_samples: int, seed: int, sample_index_base: int = 0,
                    centers_out=None, contexts_out=None):
    """LINE positive pairs: returns (centers, contexts), one CSR entry per sample."""
    dev = g.nbrs.device
    if centers_out is None:
        centers_out = torch.empty(max(num_samples, 0), dtype=torch.int32, device=dev)
    if contexts_out is None:
        contexts_out = torch.empty(max(num_samples, 0), dtype=torch.int32, device=dev)
    rc = lib().gs_sample_edges(C.byref(g.struct), _alias_ref(edge_alias), C.c_int64(num_samples),
                               C.c_uint64(sample_index_base), C.c_uint64(seed),
                               _dev(centers_out, torch.int32, "centers_out"),
                               _dev(contexts_out, torch.int32, "contexts_out"), _stream())
    _check(rc, "gs_sample_edges")
    return centers_out, contexts_out


def gs_sgns_step_workspace_bytes(num_pairs: int, num_nodes: int, k: int, dim: int,
                                 dtype: int = GS_F32) -> int:
    return int(lib().gs_sgns_step_workspace_bytes(C.c_int64(num_pairs), C.c_int64(num_nodes),
                                                  C.c_int32(k), C.c_int32(dim), C.c_int32(dtype)))


def gs_sgns_step(w_in, w_out, centers, contexts, negs, lr: float, loss_out=None, ws=None):
    """Updates w_in / w_out in place; returns the device scalar holding the summed loss."""
    dtype = _table_dtype(w_in)
    num_nodes, dim = int(w_in.shape[0]), int(w_in.shape[1])
    num_pairs = int(centers.numel())
    k = int(negs.shape[1]) if negs.dim() == 2 else 0
    dev = w_in.device
    if loss_out is None:
        loss_out = torch.zeros(1, dtype=torch.float64, device=dev)
    if ws is None:
        ws = _workspace(gs_sgns_step_workspace_bytes(num_pairs, num_nodes, k, dim, dtype), dev)
    rc = lib().gs_sgns_step(_dev(w_in, None, "w_in"), _dev(w_out, w_in.dtype, "w_out"),
                            C.c_int64(num_nodes), C.c_int32(dim), C.c_int32(dtype),
                            _dev(centers, torch.int32, "centers"),
                            _dev(contexts, torch.int32, "contexts"),
                            _dev(negs, torch.int32, "negs") if negs.numel() else None,
                            C.c_int64(num_pairs), C.c_int32(k), C.c_float(lr),
                            _dev(loss_out, torch.float64, "loss_sum_out"), _dev(ws),
                            C.c_size_t(ws.numel()), _stream())
    _check(rc, "gs_sgns_step")
    return loss_out


def gs_sgns_step_static(w_in, w_out, centers, contexts, negs, lr: float, loss_out=None):
    """gs_sgns_step on the library's own static scratch array (small batches; see gs.h)."""
    dtype = _table_dtype(w_in)
    num_nodes, dim = int(w_in.shape[0]), int(w_in.shape[1])
    num_pairs = int(centers.numel())
    k = int(negs.shape[1]) if negs.dim() == 2 else 0
    if loss_out is None:
        loss_out = torch.zeros(1, dtype=torch.float64, device=w_in.device)
    rc = lib().gs_sgns_step_static(_dev(w_in, None, "w_in"), _dev(w_out, w_in.dtype, "w_out"),
                                   C.c_int64(num_nodes), C.c_int32(dim), C.c_int32(dtype),
                                   _dev(centers, torch.int32, "centers"),
                                   _dev(contexts, torch.int32, "contexts"),
                                   _dev(negs, torch.int32, "negs") if negs.numel() else None,
                                   C.c_int64(num_pairs), C.c_int32(k), C.c_float(lr),
                                   _dev(loss_out, torch.float64, "loss_sum_out"), _stream())
    _check(rc, "gs_sgns_step_static")
    return loss_out


def gs_sgns_momentum_step(w_in, w_out, m_in, m_out, centers, contexts, negs, lr: float, mu: float,
                          loss_out=None, ws=None):
    """SGD-with-momentum iteration (see gs.h); the four tables are updated in place."""
    dtype = _table_dtype(w_in)
    num_nodes, dim = int(w_in.shape[0]), int(w_in.shape[1])
    num_pairs = int(centers.numel())
    k = int(negs.shape[1]) if negs.dim() == 2 else 0
    dev = w_in.device
    if loss_out is None:
        loss_out = torch.zeros(1, dtype=torch.float64, device=dev)
    if ws is None:
        ws = _workspace(gs_sgns_step_workspace_bytes(num_pairs, num_nodes, k, dim, dtype), dev)
    rc = lib().gs_sgns_momentum_step(
        _dev(w_in, None, "w_in"), _dev(w_out, w_in.dtype, "w_out"), _dev(m_in, w_in.dtype, "m_in"),
        _dev(m_out, w_in.dtype, "m_out"), C.c_int64(num_nodes), C.c_int32(dim), C.c_int32(dtype),
        _dev(centers, torch.int32, "centers"), _dev(contexts, torch.int32, "contexts"),
        _dev(negs, torch.int32, "negs") if negs.numel() else None, C.c_int64(num_pairs),
        C.c_int32(k), C.c_float(lr), C.c_float(mu), _dev(loss_out, torch.float64, "loss_sum_out"),
        _dev(ws), C.c_size_t(ws.numel()), _stream())
    _check(rc, "gs_sgns_momentum_step")
    return loss_out


def gs_unique_ids_workspace_bytes(n: int, num_nodes: int) -> int:
    return int(lib().gs_unique_ids_workspace_bytes(C.c_int64(n), C.c_int64(num_nodes)))


def gs_unique_ids(ids, num_nodes: int, want_inverse: bool = True, ws=None):
    """Returns (unique_out [n], num_unique device int64[1], inverse [n] or None); only the
    first num_unique entries of unique_out are meaningful."""
    n = int(ids.numel())
    dev = ids.device
    unique_out = torch.empty(max(n, 1), dtype=torch.int32, device=dev)
    count = torch.zeros(1, dtype=torch.int64, device=dev)
    inverse = torch.empty(max(n, 1), dtype=torch.int32, device=dev) if want_inverse else None
    if ws is None:
        ws = _workspace(gs_unique_ids_workspace_bytes(n, num_nodes), dev)
    rc = lib().gs_unique_ids(_dev(ids, torch.int32, "ids"), C.c_int64(n), C.c_int64(num_nodes),
                             _dev(unique_out, torch.int32), _dev(count, torch.int64),
                             _dev(inverse, torch.int32) if inverse is not None else None,
                             _dev(ws), C.c_size_t(ws.numel()), _stream())
    _check(rc, "gs_unique_ids")
    return unique_out[:n], count, (inverse[:n] if inverse is not None else None)


def _table_dtype(table):
    if table.dtype == torch.float32:
        return GS_F32
    if table.dtype == torch.bfloat16:
        return GS_BF16
    if table.dtype == torch.float16:
        return GS_F16
    raise TypeError(f"tables are float32, bfloat16 or float16, not {table.dtype}")


def gs_get_rows(table, ids, count=None, out=None):
    """out[i] = table[ids[i]] as float32; `count` (device int64[1]) limits the rows processed."""
    n, dim = int(ids.numel()), int(table.shape[1])
    if out is None:
        out = torch.empty((n, dim), dtype=torch.float32, device=table.device)
    rc = lib().gs_get_rows(_dev(table), C.c_int64(table.shape[0]), C.c_int32(dim),
                           C.c_int32(_table_dtype(table)), _dev(ids, torch.int32, "ids"), C.c_int64(n),
                           _dev(count, torch.int64) if count is not None else None,
                           _dev(out, torch.float32, "out"), _stream())
    _check(rc, "gs_get_rows")
    return out


def gs_put_rows(table, ids, rows, scale: float, count=None):
    """table[ids[i]] += scale * rows[i] in place; the ids must be distinct."""
    n, dim = int(ids.numel()), int(table.shape[1])
    rc = lib().gs_put_rows(_dev(table), C.c_int64(table.shape[0]), C.c_int32(dim),
                           C.c_int32(_table_dtype(table)), _dev(ids, torch.int32, "ids"), C.c_int64(n),
                           _dev(count, torch.int64) if count is not None else None,
                           _dev(rows, torch.float32, "rows"), C.c_float(scale), _stream())
    _check(rc, "gs_put_rows")


def gs_sgns_adam_step(w_in, w_out, m_in, m_out, v_in, v_out, centers, contexts, negs, lr: float,
                      beta1: float, beta2: float, eps: float, t: int, loss_out=None, ws=None):
    """Adam iteration number t on six float32 tables, in place; returns the device loss scalar."""
    num_nodes, dim = int(w_in.shape[0]), int(w_in.shape[1])
    num_pairs = int(centers.numel())
    k = int(negs.shape[1]) if negs.dim() == 2 else 0
    dev = w_in.device
    for tb in (w_in, w_out, m_in, m_out, v_in, v_out):
        if tb.dtype != torch.float32 or tuple(tb.shape) != (num_nodes, dim) or not tb.is_contiguous():
            raise TypeError("Adam tables must be contiguous float32 [num_nodes, dim]")
    if loss_out is None:
        loss_out = torch.zeros(1, dtype=torch.float64, device=dev)
    if ws is None:
        ws = _workspace(gs_sgns_step_workspace_bytes(num_pairs, num_nodes, k, dim, GS_F32), dev)
    rc = lib().gs_sgns_adam_step(
        _dev(w_in), _dev(w_out), _dev(m_in), _dev(m_out), _dev(v_in), _dev(v_out),
        C.c_int64(num_nodes), C.c_int32(dim), _dev(centers, torch.int32, "centers"),
        _dev(contexts, torch.int32, "contexts"), _dev(negs, torch.int32, "negs"),
        C.c_int64(num_pairs), C.c_int32(k), C.c_float(lr), C.c_float(beta1), C.c_float(beta2),
        C.c_float(eps), C.c_int64(t), _dev(loss_out, torch.float64), _dev(ws),
        C.c_size_t(ws.numel()), _stream())
    _check(rc, "gs_sgns_adam_step")
    return loss_out


def gs_sgns_step_fused_workspace_bytes(num_pairs: int, num_nodes: int, k: int, dim: int,
                                       dtype: int = GS_F32) -> int:
    return int(lib().gs_sgns_step_fused_workspace_bytes(C.c_int64(num_pairs), C.c_int64(num_nodes),
                                                        C.c_int32(k), C.c_int32(dim), C.c_int32(dtype)))


def gs_sgns_step_fused(w_in, w_out, centers, contexts, noise, k: int, neg_seed: int, lr: float,
                       pair_index_base: int = 0, loss_out=None, ws=None):
    """gs_sample_negatives + gs_sgns_step in one call; returns the device loss scalar."""
    dtype = _table_dtype(w_in)
    num_nodes, dim = int(w_in.shape[0]), int(w_in.shape[1])
    num_pairs = int(centers.numel())
    dev = w_in.device
    if loss_out is None:
        loss_out = torch.zeros(1, dtype=torch.float64, device=dev)
    if ws is None:
        ws = _workspace(gs_sgns_step_fused_workspace_bytes(num_pairs, num_nodes, k, dim, dtype), dev)
    rc = lib().gs_sgns_step_fused(
        _dev(w_in), _dev(w_out), C.c_int64(num_nodes), C.c_int32(dim), C.c_int32(dtype),
        _dev(centers, torch.int32, "centers"), _dev(contexts, torch.int32, "contexts"),
        C.c_int64(num_pairs), _alias_ref(noise), C.c_uint64(pair_index_base), C.c_uint64(neg_seed),
        C.c_int32(k), C.c_float(lr), _dev(loss_out, torch.float64), _dev(ws), C.c_size_t(ws.numel()),
        _stream())
    _check(rc, "gs_sgns_step_fused")
    return loss_out


def gs_pair_offsets(walks, window: int, out=None, ws=None):
    """int64[num_walks + 1]: pairs emitted for the walks before each walk, and for all of them."""
    num_walks, walk_len = int(walks.shape[0]), int(walks.shape[1])
    dev = walks.device
    if out is None:
        out = torch.empty(num_walks + 1, dtype=torch.int64, device=dev)
    if ws is None:
        ws = _workspace(int(lib().gs_pair_offsets_workspace_bytes(C.c_int64(num_walks))), dev)
    rc = lib().gs_pair_offsets(_dev(walks, torch.int32, "walks"), C.c_int64(num_walks), C.c_int32(walk_len),
                               C.c_int32(window), _dev(out, torch.int64, "offsets_out"), _dev(ws),
                               C.c_size_t(ws.numel()), _stream())
    _check(rc, "gs_pair_offsets")
    return out


def gs_sgns_step_from_walks_workspace_bytes(num_pairs: int, num_nodes: int, k: int, dim: int,
                                            dtype: int = GS_F32) -> int:
    return int(lib().gs_sgns_step_from_walks_workspace_bytes(
        C.c_int64(num_pairs), C.c_int64(num_nodes), C.c_int32(k), C.c_int32(dim), C.c_int32(dtype)))


def gs_sgns_step_from_walks(w_in, w_out, walks, window: int, pair_offsets, first_pair: int,
                            num_pairs: int, noise, k: int, neg_seed: int, lr: float,
                            pair_index_base: int = 0, loss_out=None, ws=None):
    """Pairs from the walk buffer, negatives from the counters, and the iteration, in one call."""
    dtype = _table_dtype(w_in)
    num_nodes, dim = int(w_in.shape[0]), int(w_in.shape[1])
    num_walks, walk_len = int(walks.shape[0]), int(walks.shape[1])
    dev = w_in.device
    if loss_out is None:
        loss_out = torch.zeros(1, dtype=torch.float64, device=dev)
    if ws is None:
        ws = _workspace(gs_sgns_step_from_walks_workspace_bytes(num_pairs, num_nodes, k, dim, dtype), dev)
    rc = lib().gs_sgns_step_from_walks(
        _dev(w_in), _dev(w_out), C.c_int64(num_nodes), C.c_int32(dim), C.c_int32(dtype),
        _dev(walks, torch.int32, "walks"), C.c_int64(num_walks), C.c_int32(walk_len), C.c_int32(window),
        _dev(pair_offsets, torch.int64, "pair_offsets"), C.c_int64(first_pair), C.c_int64(num_pairs),
        _alias_ref(noise), C.c_uint64(pair_index_base), C.c_uint64(neg_seed), C.c_int32(k),
        C.c_float(lr), _dev(loss_out, torch.float64), _dev(ws), C.c_size_t(ws.numel()), _stream())
    _check(rc, "gs_sgns_step_from_walks")
    return loss_out


def gs_line1_step_workspace_bytes(num_pairs: int, num_nodes: int, k: int, dim: int,
                                  dtype: int = GS_F32) -> int:
    return int(lib().gs_line1_step_workspace_bytes(C.c_int64(num_pairs), C.c_int64(num_nodes),
                                                   C.c_int32(k), C.c_int32(dim), C.c_int32(dtype)))


def gs_line1_step(w, sources, targets, negs, lr: float, loss_out=None, ws=None):
    """First-order LINE iteration on the single table w, in place; returns the device loss scalar."""
    dtype = _table_dtype(w)
    num_nodes, dim = int(w.shape[0]), int(w.shape[1])
    num_pairs = int(sources.numel())
    k = int(negs.shape[1]) if negs.dim() == 2 else 0
    dev = w.device
    if loss_out is None:
        loss_out = torch.zeros(1, dtype=torch.float64, device=dev)
    if ws is None:
        ws = _workspace(gs_line1_step_workspace_bytes(num_pairs, num_nodes, k, dim, dtype), dev)
    rc = lib().gs_line1_step(
        _dev(w), C.c_int64(num_nodes), C.c_int32(dim), C.c_int32(dtype),
        _dev(sources, torch.int32, "sources"), _dev(targets, torch.int32, "targets"),
        _dev(negs, torch.int32, "negs"), C.c_int64(num_pairs), C.c_int32(k), C.c_float(lr),
        _dev(loss_out, torch.float64), _dev(ws), C.c_size_t(ws.numel()), _stream())
    _check(rc, "gs_line1_step")
    return loss_out


def gs_table_mult(table, factor: float):
    """table *= factor in place, every row."""
    rc = lib().gs_table_mult(_dev(table), C.c_int64(table.shape[0]), C.c_int32(table.shape[1]),
                             C.c_int32(_table_dtype(table)), C.c_float(factor), _stream())
    _check(rc, "gs_table_mult")


def gs_table_mult_add(dst, src, factor: float):
    """dst += factor * src in place, every row (two tables of the same shape and dtype)."""
    if dst.shape != src.shape or dst.dtype != src.dtype:
        raise TypeError("gs_table_mult_add needs two tables of the same shape and dtype")
    rc = lib().gs_table_mult_add(_dev(dst), _dev(src), C.c_int64(dst.shape[0]),
                                 C.c_int32(dst.shape[1]), C.c_int32(_table_dtype(dst)),
                                 C.c_float(factor), _stream())
    _check(rc, "gs_table_mult_add")


def gs_sort_pairs_workspace_bytes(n: int) -> int:
    return int(lib().gs_sort_pairs_workspace_bytes(C.c_int64(n)))


def gs_sort_pairs(centers, contexts, num_nodes: int, centers_out=None, contexts_out=None, ws=None):
    """Pairs reordered by centre id (stable); returns (centers_out, contexts_out)."""
    n = int(centers.numel())
    dev = centers.device
    if centers_out is None:
        centers_out = torch.empty(max(n, 1), dtype=torch.int32, device=dev)[:n]
    if contexts_out is None:
        contexts_out = torch.empty(max(n, 1), dtype=torch.int32, device=dev)[:n]
    if ws is None:
        ws = _workspace(gs_sort_pairs_workspace_bytes(n), dev)
    rc = lib().gs_sort_pairs(_dev(centers, torch.int32, "centers"), _dev(contexts, torch.int32, "contexts"),
                             C.c_int64(n), C.c_int64(num_nodes), _dev(centers_out, torch.int32),
                             _dev(contexts_out, torch.int32), _dev(ws), C.c_size_t(ws.numel()), _stream())
    _check(rc, "gs_sort_pairs")
    return centers_out, contexts_out
