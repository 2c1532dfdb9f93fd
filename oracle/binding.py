"""ctypes/numpy wrapper around ``liboracle.so`` (built from ``gs_oracle.cpp``).

TEST INFRASTRUCTURE: marshals numpy arrays into the oracle's C entry points and
nothing else.  All arithmetic of the method lives in the C++ file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gs_oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")

F32, BF16, F16 = 0, 1, 2
SYMMETRIZE, DROP_SELF_LOOPS, DEDUPE = 1, 2, 4


class _Csr(C.Structure):
    _fields_ = [("num_nodes", C.c_int64), ("num_entries", C.c_int64),
                ("offsets", C.c_void_p), ("offset_bits", C.c_int32),
                ("nbrs", C.c_void_p), ("weights", C.c_void_p)]


class _Alias(C.Structure):
    _fields_ = [("prob", C.c_void_p), ("alias", C.c_void_p)]


SOURCE = _SRC
BASE_FLAGS = ["-std=c++17", "-ffp-contract=off", "-fPIC", "-shared", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (no fused multiply-add contraction).

    ``GS_ORACLE_LIB`` in the environment names a library built elsewhere from the same
    source (the sanitizer test builds one with -fsanitize=address,undefined and runs the
    pins in a child process against it); it is then loaded as it is."""
    other = os.environ.get("GS_ORACLE_LIB")
    if other:
        return other
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", *BASE_FLAGS, "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        for name in ("oracle_csr_build", "oracle_alias_build", "oracle_random_walk",
                     "oracle_node2vec_walk", "oracle_make_pairs", "oracle_sample_negatives",
                     "oracle_sgns_step", "oracle_sgns_momentum_step", "oracle_sample_edges", "oracle_unique_ids", "oracle_get_rows",
                     "oracle_put_rows", "oracle_sgns_adam_step", "oracle_line1_step", "oracle_table_mult",
                     "oracle_table_mult_add", "oracle_sort_pairs"):
            getattr(_lib, name).restype = C.c_int32
        _lib.oracle_philox4x32_10.restype = None
        _lib.oracle_f16_to_float.restype = None
        _lib.oracle_float_to_f16.restype = None
    return _lib


def _ptr(a):
    return None if a is None else C.c_void_p(a.ctypes.data)


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"{what} failed with status {rc}")


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def philox4x32_10(ctr, key):
    ctr = np.ascontiguousarray(ctr, dtype=np.uint32)
    key = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    _load().oracle_philox4x32_10(_ptr(ctr), _ptr(key), _ptr(out))
    return out


def csr_build(src, dst, w, num_nodes, flags, offset_bits=32):
    """Returns (offsets, nbrs, weights-or-None)."""
    src, dst = _i32(src), _i32(dst)
    m = int(src.shape[0])
    if w is not None:
        w = np.ascontiguousarray(w, dtype=np.float32)
    cap = max(1, m * (2 if flags & SYMMETRIZE else 1))
    offsets = np.zeros(num_nodes + 1, dtype=np.int64 if offset_bits == 64 else np.int32)
    nbrs = np.zeros(cap, dtype=np.int32)
    w_out = np.zeros(cap, dtype=np.float32) if w is not None else None
    ne = C.c_int64(0)
    rc = _load().oracle_csr_build(_ptr(src), _ptr(dst), _ptr(w), C.c_int64(m),
                                  C.c_int64(num_nodes), C.c_uint32(flags), C.c_int32(offset_bits),
                                  _ptr(offsets), _ptr(nbrs), _ptr(w_out), C.byref(ne))
    _check(rc, "oracle_csr_build")
    n = ne.value
    return offsets, nbrs[:n].copy(), (None if w_out is None else w_out[:n].copy())


def alias_build(seg_offsets, weights):
    """Returns (prob, alias) for the segments delimited by seg_offsets."""
    seg_offsets = np.ascontiguousarray(seg_offsets)
    assert seg_offsets.dtype in (np.int32, np.int64)
    bits = 64 if seg_offsets.dtype == np.int64 else 32
    weights = np.ascontiguousarray(weights, dtype=np.float32)
    prob = np.zeros(max(1, weights.shape[0]), dtype=np.float32)
    alias = np.zeros(max(1, weights.shape[0]), dtype=np.int32)
    rc = _load().oracle_alias_build(_ptr(seg_offsets), C.c_int32(bits),
                                    C.c_int64(seg_offsets.shape[0] - 1), _ptr(weights),
                                    _ptr(prob), _ptr(alias))
    _check(rc, "oracle_alias_build")
    return prob[:weights.shape[0]], alias[:weights.shape[0]]


def _csr_struct(offsets, nbrs, weights=None):
    offsets = np.ascontiguousarray(offsets)
    assert offsets.dtype in (np.int32, np.int64)
    nbrs = _i32(nbrs)
    keep = [offsets, nbrs, weights]
    s = _Csr(offsets.shape[0] - 1, nbrs.shape[0], offsets.ctypes.data,
             64 if offsets.dtype == np.int64 else 32, nbrs.ctypes.data,
             None if weights is None else weights.ctypes.data)
    return s, keep


def _alias_struct(alias):
    if alias is None:
        return None, []
    prob, al = alias
    prob = np.ascontiguousarray(prob, dtype=np.float32)
    al = _i32(al)
    return _Alias(prob.ctypes.data, al.ctypes.data), [prob, al]


def random_walk(offsets, nbrs, starts, walk_len, seed, alias=None, walk_id_base=0):
    g, keep = _csr_struct(offsets, nbrs)
    a, keep2 = _alias_struct(alias)
    starts = _i32(starts)
    nw = int(starts.shape[0])
    out = np.zeros((nw, walk_len), dtype=np.int32)
    rc = _load().oracle_random_walk(C.byref(g), None if a is None else C.byref(a), _ptr(starts),
                                    C.c_int64(nw), C.c_uint64(walk_id_base), C.c_int32(walk_len),
                                    C.c_uint64(seed), _ptr(out))
    _check(rc, "oracle_random_walk")
    del keep, keep2
    return out


def node2vec_walk(offsets, nbrs, starts, walk_len, p, q, seed, alias=None, walk_id_base=0):
    g, keep = _csr_struct(offsets, nbrs)
    a, keep2 = _alias_struct(alias)
    starts = _i32(starts)
    nw = int(starts.shape[0])
    out = np.zeros((nw, walk_len), dtype=np.int32)
    rc = _load().oracle_node2vec_walk(C.byref(g), None if a is None else C.byref(a), _ptr(starts),
                                      C.c_int64(nw), C.c_uint64(walk_id_base),
                                      C.c_int32(walk_len), C.c_float(p), C.c_float(q),
                                      C.c_uint64(seed), _ptr(out))
    _check(rc, "oracle_node2vec_walk")
    del keep, keep2
    return out


def make_pairs(walks, window):
    walks = _i32(walks)
    nw, walk_len = walks.shape
    cap = max(1, nw * walk_len * 2 * window)
    centers = np.zeros(cap, dtype=np.int32)
    contexts = np.zeros(cap, dtype=np.int32)
    n = C.c_int64(0)
    rc = _load().oracle_make_pairs(_ptr(walks), C.c_int64(nw), C.c_int32(walk_len),
                                   C.c_int32(window), _ptr(centers), _ptr(contexts), C.byref(n))
    _check(rc, "oracle_make_pairs")
    return centers[:n.value].copy(), contexts[:n.value].copy()


def sample_negatives(noise_alias, num_nodes, num_pairs, k, seed, pair_index_base=0):
    a, keep = _alias_struct(noise_alias)
    out = np.zeros((num_pairs, k), dtype=np.int32)
    rc = _load().oracle_sample_negatives(None if a is None else C.byref(a), C.c_int64(num_nodes),
                                         C.c_int64(num_pairs), C.c_uint64(pair_index_base),
                                         C.c_int32(k), C.c_uint64(seed), _ptr(out))
    _check(rc, "oracle_sample_negatives")
    del keep
    return out


def sample_edges(offsets, nbrs, num_samples, seed, edge_alias=None, sample_index_base=0):
    """LINE edge sampling: returns (centers, contexts), one CSR entry per sample."""
    g, keep = _csr_struct(offsets, nbrs)
    a, keep2 = _alias_struct(edge_alias)
    centers = np.zeros(max(1, num_samples), dtype=np.int32)
    contexts = np.zeros(max(1, num_samples), dtype=np.int32)
    rc = _load().oracle_sample_edges(C.byref(g), None if a is None else C.byref(a),
                                     C.c_int64(num_samples), C.c_uint64(sample_index_base),
                                     C.c_uint64(seed), _ptr(centers), _ptr(contexts))
    _check(rc, "oracle_sample_edges")
    del keep, keep2
    return centers[:num_samples], contexts[:num_samples]


def sgns_step(w_in, w_out, centers, contexts, negs, lr, dtype=F32):
    """Updates w_in / w_out (numpy, C-contiguous, float32 or uint16 bf16 bits) in place.

    Returns the summed loss of the batch.
    """
    want = np.float32 if dtype == F32 else np.uint16
    assert w_in.dtype == want and w_out.dtype == want
    assert w_in.flags.c_contiguous and w_out.flags.c_contiguous and w_in.shape == w_out.shape
    centers, contexts = _i32(centers), _i32(contexts)
    negs = _i32(negs)
    num_pairs = int(centers.shape[0])
    k = int(negs.shape[1]) if negs.ndim == 2 else 0
    loss = C.c_double(0.0)
    rc = _load().oracle_sgns_step(_ptr(w_in), _ptr(w_out), C.c_int64(w_in.shape[0]),
                                  C.c_int32(w_in.shape[1]), C.c_int32(dtype), _ptr(centers),
                                  _ptr(contexts), _ptr(negs), C.c_int64(num_pairs), C.c_int32(k),
                                  C.c_float(lr), C.byref(loss))
    _check(rc, "oracle_sgns_step")
    return loss.value


def sgns_momentum_step(w_in, w_out, m_in, m_out, centers, contexts, negs, lr, mu, dtype=F32):
    """SGD-with-momentum iteration; updates the four tables in place, returns the summed loss."""
    want = np.float32 if dtype == F32 else np.uint16
    for t in (w_in, w_out, m_in, m_out):
        assert t.dtype == want and t.flags.c_contiguous and t.shape == w_in.shape
    centers, contexts = _i32(centers), _i32(contexts)
    negs = _i32(negs)
    num_pairs = int(centers.shape[0])
    k = int(negs.shape[1]) if negs.ndim == 2 else 0
    loss = C.c_double(0.0)
    rc = _load().oracle_sgns_momentum_step(
        _ptr(w_in), _ptr(w_out), _ptr(m_in), _ptr(m_out), C.c_int64(w_in.shape[0]),
        C.c_int32(w_in.shape[1]), C.c_int32(dtype), _ptr(centers), _ptr(contexts), _ptr(negs),
        C.c_int64(num_pairs), C.c_int32(k), C.c_float(lr), C.c_float(mu), C.byref(loss))
    _check(rc, "oracle_sgns_momentum_step")
    return loss.value


def unique_ids(ids, num_nodes):
    """Returns (unique ascending, inverse): ids outside [0, num_nodes) are left out, inverse -1."""
    ids = _i32(ids)
    n = int(ids.shape[0])
    uniq = np.zeros(max(1, n), dtype=np.int32)
    inverse = np.zeros(max(1, n), dtype=np.int32)
    count = C.c_int64(0)
    rc = _load().oracle_unique_ids(_ptr(ids), C.c_int64(n), C.c_int64(num_nodes), _ptr(uniq),
                                   C.byref(count), _ptr(inverse))
    _check(rc, "oracle_unique_ids")
    return uniq[:count.value].copy(), inverse[:n].copy()


def get_rows(table, ids, dtype=F32):
    """table[ids] as float32 [n, dim] (zero rows for ids out of range)."""
    want = np.float32 if dtype == F32 else np.uint16
    assert table.dtype == want and table.flags.c_contiguous
    ids = _i32(ids)
    n = int(ids.shape[0])
    out = np.zeros((max(1, n), table.shape[1]), dtype=np.float32)
    rc = _load().oracle_get_rows(_ptr(table), C.c_int64(table.shape[0]), C.c_int32(table.shape[1]),
                                 C.c_int32(dtype), _ptr(ids), C.c_int64(n), _ptr(out))
    _check(rc, "oracle_get_rows")
    return out[:n]


def put_rows(table, ids, rows, scale, dtype=F32):
    """table[ids[i]] += scale * rows[i] in place (distinct ids)."""
    want = np.float32 if dtype == F32 else np.uint16
    assert table.dtype == want and table.flags.c_contiguous
    ids = _i32(ids)
    rows = np.ascontiguousarray(rows, dtype=np.float32)
    n = int(ids.shape[0])
    assert rows.shape == (n, table.shape[1])
    rc = _load().oracle_put_rows(_ptr(table), C.c_int64(table.shape[0]), C.c_int32(table.shape[1]),
                                 C.c_int32(dtype), _ptr(ids), C.c_int64(n), _ptr(rows),
                                 C.c_float(scale))
    _check(rc, "oracle_put_rows")


def sgns_adam_step(w_in, w_out, m_in, m_out, v_in, v_out, centers, contexts, negs, lr, beta1, beta2,
                   eps, t):
    """Adam iteration number t (>= 1) on float32 tables, in place; returns the summed loss."""
    for a in (w_in, w_out, m_in, m_out, v_in, v_out):
        assert a.dtype == np.float32 and a.flags.c_contiguous and a.shape == w_in.shape
    centers, contexts = _i32(centers), _i32(contexts)
    negs = _i32(negs)
    num_pairs = int(centers.shape[0])
    k = int(negs.shape[1]) if negs.ndim == 2 else 0
    loss = C.c_double(0.0)
    rc = _load().oracle_sgns_adam_step(
        _ptr(w_in), _ptr(w_out), _ptr(m_in), _ptr(m_out), _ptr(v_in), _ptr(v_out),
        C.c_int64(w_in.shape[0]), C.c_int32(w_in.shape[1]), _ptr(centers), _ptr(contexts), _ptr(negs),
        C.c_int64(num_pairs), C.c_int32(k), C.c_float(lr), C.c_float(beta1), C.c_float(beta2),
        C.c_float(eps), C.c_int64(t), C.byref(loss))
    _check(rc, "oracle_sgns_adam_step")
    return loss.value


def line1_step(w, sources, targets, negs, lr, dtype=F32):
    """First-order LINE iteration on the single table w, in place; returns the summed loss."""
    want = np.float32 if dtype == F32 else np.uint16
    assert w.dtype == want and w.flags.c_contiguous
    sources, targets = _i32(sources), _i32(targets)
    negs = _i32(negs)
    num_pairs = int(sources.shape[0])
    k = int(negs.shape[1]) if negs.ndim == 2 else 0
    loss = C.c_double(0.0)
    rc = _load().oracle_line1_step(_ptr(w), C.c_int64(w.shape[0]), C.c_int32(w.shape[1]),
                                   C.c_int32(dtype), _ptr(sources), _ptr(targets), _ptr(negs),
                                   C.c_int64(num_pairs), C.c_int32(k), C.c_float(lr), C.byref(loss))
    _check(rc, "oracle_line1_step")
    return loss.value


def table_mult(table, factor, dtype=F32):
    """table *= factor in place (one rounding per element)."""
    want = np.float32 if dtype == F32 else np.uint16
    assert table.dtype == want and table.flags.c_contiguous
    rc = _load().oracle_table_mult(_ptr(table), C.c_int64(table.shape[0]), C.c_int32(table.shape[1]),
                                   C.c_int32(dtype), C.c_float(factor))
    _check(rc, "oracle_table_mult")


def table_mult_add(dst, src, factor, dtype=F32):
    """dst += factor * src in place (one rounding per element)."""
    want = np.float32 if dtype == F32 else np.uint16
    assert dst.dtype == want and src.dtype == want and dst.shape == src.shape
    assert dst.flags.c_contiguous and src.flags.c_contiguous
    rc = _load().oracle_table_mult_add(_ptr(dst), _ptr(src), C.c_int64(dst.shape[0]),
                                       C.c_int32(dst.shape[1]), C.c_int32(dtype), C.c_float(factor))
    _check(rc, "oracle_table_mult_add")


def sort_pairs(centers, contexts, num_nodes):
    """Pairs reordered by centre id, stable; returns (centers, contexts)."""
    centers, contexts = _i32(centers), _i32(contexts)
    n = int(centers.shape[0])
    oc = np.zeros(max(1, n), dtype=np.int32)
    oo = np.zeros(max(1, n), dtype=np.int32)
    rc = _load().oracle_sort_pairs(_ptr(centers), _ptr(contexts), C.c_int64(n), C.c_int64(num_nodes),
                                   _ptr(oc), _ptr(oo))
    _check(rc, "oracle_sort_pairs")
    return oc[:n], oo[:n]


def f16_to_float(bits):
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.zeros(bits.shape, dtype=np.float32)
    _load().oracle_f16_to_float(_ptr(bits), C.c_int64(bits.size), _ptr(out))
    return out


def float_to_f16(values):
    values = np.ascontiguousarray(values, dtype=np.float32)
    out = np.zeros(values.shape, dtype=np.uint16)
    _load().oracle_float_to_f16(_ptr(values), C.c_int64(values.size), _ptr(out))
    return out
