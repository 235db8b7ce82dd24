"""ctypes front end of the C oracle in tree_attn_oracle.c (test infrastructure only).

The arithmetic lives in the C file: per (request, node, head) a textbook
max-subtracted softmax attention over the cached prefix followed by the node's
root-to-node path (paper section 3.1, "Tree attention"; cache addressing per
section 3.4, "Paged KV with tree attention").  This module only marshals numpy
arrays into the C struct.  Parity status: pinned (see the header of the C file).
"""
import ctypes
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tree_attn_oracle.c")
_LIB = os.path.join(_HERE, "libtreeattn_oracle.so")
_lib = None


class _Problem(ctypes.Structure):
    _fields_ = [
        ("q", ctypes.c_void_p),
        ("k_cache", ctypes.c_void_p),
        ("v_cache", ctypes.c_void_p),
        ("dtype", ctypes.c_int32),
        ("B", ctypes.c_int32),
        ("T", ctypes.c_int32),
        ("Hq", ctypes.c_int32),
        ("Hkv", ctypes.c_int32),
        ("D", ctypes.c_int32),
        ("q_stride", ctypes.c_int64 * 3),
        ("k_stride", ctypes.c_int64 * 3),
        ("v_stride", ctypes.c_int64 * 3),
        ("page_size", ctypes.c_int32),
        ("max_pages", ctypes.c_int32),
        ("page_table", ctypes.c_void_p),
        ("seq_lens", ctypes.c_void_p),
        ("tree_parent", ctypes.c_void_p),
        ("parent_stride_b", ctypes.c_int64),
        ("scale", ctypes.c_double),
        ("Tq", ctypes.c_int32),
        ("q_off", ctypes.c_int32),
        ("kv_start", ctypes.c_void_p),
    ]


def build_oracle(force=False):
    """Compile the C oracle with gcc (-O2 -fopenmp); returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c99", _SRC, "-o", tmp, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build_oracle())
        lib.tree_attn_oracle.restype = ctypes.c_int
        lib.tree_attn_oracle.argtypes = [ctypes.POINTER(_Problem), ctypes.c_void_p, ctypes.c_void_p]
        lib.tree_attn_oracle_sample.restype = ctypes.c_int
        lib.tree_attn_oracle_sample.argtypes = [
            ctypes.POINTER(_Problem), ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
        lib.tree_attn_oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def oracle_threads():
    """Number of OpenMP threads the oracle will use."""
    return int(_load().tree_attn_oracle_threads())


def _elem_strides(a, n):
    assert a.strides[-1] == a.itemsize, "innermost dimension must be contiguous"
    return [s // a.itemsize for s in a.strides[:n]]


def _marshal(q, k_cache, v_cache, page_table, seq_lens, tree_parent, scale, kv_start=None, q_node_offset=None):
    if q.dtype == np.float32:
        dtype = 0
    elif q.dtype == np.uint16:
        dtype = 1  # bf16 bit patterns
    else:
        raise TypeError("q must be float32 or uint16 (bf16 bits), got %s" % q.dtype)
    if k_cache.dtype != q.dtype or v_cache.dtype != q.dtype:
        raise TypeError("q, k_cache and v_cache must share a dtype")
    if q.ndim != 4 or k_cache.ndim != 4 or v_cache.ndim != 4:
        raise ValueError("q is [B,T,Hq,D]; caches are [num_pages,Hkv,page_size,D]")
    B, Tq, Hq, D = q.shape
    tree_parent = np.ascontiguousarray(tree_parent, dtype=np.int32)
    T = tree_parent.shape[-1]                  # nodes of the tree (keys); q holds Tq of them from q_node_offset on
    if q_node_offset is None:
        if Tq != T:
            raise ValueError("q has %d nodes, the tree %d: pass q_node_offset" % (Tq, T))
        q_node_offset = 0
    _, Hkv, ps, Dk = k_cache.shape
    if Dk != D or v_cache.shape != k_cache.shape:
        raise ValueError("cache shapes disagree with q")
    seq_lens = np.ascontiguousarray(seq_lens, dtype=np.int32)
    if tree_parent.ndim == 1:
        pstride = 0
    else:
        assert tree_parent.shape == (B, T)
        pstride = T
    keep = [seq_lens, tree_parent]
    p = _Problem()
    p.q, p.k_cache, p.v_cache = q.ctypes.data, k_cache.ctypes.data, v_cache.ctypes.data
    p.dtype = dtype
    p.B, p.T, p.Hq, p.Hkv, p.D = B, T, Hq, Hkv, D
    p.q_stride = (ctypes.c_int64 * 3)(*_elem_strides(q, 3))
    p.k_stride = (ctypes.c_int64 * 3)(*_elem_strides(k_cache, 3))
    p.v_stride = (ctypes.c_int64 * 3)(*_elem_strides(v_cache, 3))
    p.page_size = ps
    if page_table is None:
        p.page_table = None
        p.max_pages = 1
        if k_cache.shape[0] < B:
            raise ValueError("contiguous mode needs one cache page per request")
    else:
        page_table = np.ascontiguousarray(page_table, dtype=np.int32)
        assert page_table.ndim == 2 and page_table.shape[0] == B
        keep.append(page_table)
        p.page_table = page_table.ctypes.data
        p.max_pages = page_table.shape[1]
    p.seq_lens = seq_lens.ctypes.data
    p.tree_parent = tree_parent.ctypes.data
    p.parent_stride_b = pstride
    p.scale = (1.0 / math.sqrt(D)) if scale is None else float(scale)
    p.Tq, p.q_off = Tq, int(q_node_offset)
    if kv_start is None:
        p.kv_start = None
    else:
        kv_start = np.ascontiguousarray(kv_start, dtype=np.int32)
        assert kv_start.shape == (B,)
        keep.append(kv_start)
        p.kv_start = kv_start.ctypes.data
    return p, keep


def tree_attn_oracle(q, k_cache, v_cache, page_table, seq_lens, tree_parent, scale=None, kv_start=None,
                     q_node_offset=None):
    """All outputs in fp64: out [B,Tq,Hq,D], lse [B,Hq,Tq].  kv_start [B]: first prefix position still attended to.
    q_node_offset: q holds the nodes q_node_offset .. q_node_offset+Tq-1 of the tree (default: all of them)."""
    p, keep = _marshal(q, k_cache, v_cache, page_table, seq_lens, tree_parent, scale, kv_start, q_node_offset)
    out = np.empty((p.B, p.Tq, p.Hq, p.D), dtype=np.float64)
    lse = np.empty((p.B, p.Hq, p.Tq), dtype=np.float64)
    rc = _load().tree_attn_oracle(ctypes.byref(p), out.ctypes.data, lse.ctypes.data)
    if rc < 0:
        raise ValueError("oracle rejected the arguments")
    del keep
    return out, lse


def tree_attn_oracle_sample(q, k_cache, v_cache, page_table, seq_lens, tree_parent, triples, scale=None,
                            kv_start=None, q_node_offset=None):
    """Selected outputs: triples [n,3] of (request, row of q, head) -> out [n,D], lse [n] in fp64."""
    p, keep = _marshal(q, k_cache, v_cache, page_table, seq_lens, tree_parent, scale, kv_start, q_node_offset)
    triples = np.ascontiguousarray(triples, dtype=np.int32).reshape(-1, 3)
    n = triples.shape[0]
    out = np.empty((n, p.D), dtype=np.float64)
    lse = np.empty((n,), dtype=np.float64)
    rc = _load().tree_attn_oracle_sample(ctypes.byref(p), triples.ctypes.data, n, out.ctypes.data, lse.ctypes.data)
    if rc < 0:
        raise ValueError("oracle rejected the arguments")
    del keep
    return out, lse
