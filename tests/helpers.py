"""Test-side helpers: widen workloads to fp64 and flatten a request's cache (independent of oracle and HIP path)."""
import numpy as np

from paper_2508_08192_amd import workloads as W


def widen(a):
    """float64 view of a workload array (float32 values or bf16 bit patterns)."""
    if a.dtype == np.uint16:
        return W.bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


def logical_kv(w, b, n=None):
    """K and V of request b at logical positions 0..n-1 as fp64 arrays [Hkv, n, D]."""
    n = int(w.seq_lens[b]) + w.T if n is None else n
    ps = w.page_size
    K = np.empty((w.Hkv, n, w.D))
    V = np.empty((w.Hkv, n, w.D))
    for pos in range(n):
        if w.page_table is None:
            page, slot = b, pos
        else:
            page, slot = int(w.page_table[b, pos // ps]), pos % ps
        K[:, pos, :] = widen(w.k_cache[page, :, slot, :])
        V[:, pos, :] = widen(w.v_cache[page, :, slot, :])
    return K, V


def ancestors_inclusive(parent, i):
    out = []
    cur = int(i)
    while cur >= 0:
        out.append(cur)
        cur = int(parent[cur])
    return out[::-1]


def run_oracle(w, **kw):
    import oracle
    return oracle.tree_attn_oracle(w.q, w.k_cache, w.v_cache, w.page_table, w.seq_lens, w.tree_parent,
                                   scale=w.scale, **kw)
