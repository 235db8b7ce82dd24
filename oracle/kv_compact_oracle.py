"""CPU oracle for the cache bookkeeping after acceptance (test infrastructure only; byte work, plain loops).

What it computes (paper section 3, stage 6 "Bookkeeping": after sampling, the KV cache is rewound to the position the
accepted length gives; section 3.4, "Paged KV with tree attention": the tree tokens' keys and values sit behind the
prefix in the paged cache).  With a tree, node i of request b has its K/V at logical position L_b + i, so the accepted
root-to-leaf path is in general not contiguous.  Rewinding therefore means: the K/V rows of the accepted nodes
a_0, a_1, ..., a_{n-1} (root first) become positions L_b, L_b+1, ..., L_b+n-1, and the request's length becomes
L_b + n.  Everything else in the cache keeps its bytes.

All rows are read before any is written: a destination may be another accepted node's source.

Readings the paper leaves open: the accepted nodes are given as node ids in path order (any ids in [0, T), repeats
allowed); a request whose L_b, n or ids are out of range is left alone, its length unchanged, and reported.

Nothing here is shared with the HIP path.  Pins: tests/test_compact_oracle_pins.py (attention over the rewound cache
equals the tree attention of the path's nodes; a library gather on the contiguous layout; untouched bytes).
"""
import numpy as np


def _locate(page_table, page_size, b, pos):
    """(page, slot) of logical position pos of request b (section 3.4 addressing; no table: request b owns page b)."""
    if page_table is None:
        return b, pos
    return int(page_table[b, pos // page_size]), pos % page_size


def kv_compact_oracle(k_cache, v_cache, page_table, seq_lens, accepted, n_accepted, T):
    """k_cache, v_cache: arrays [num_pages, Hkv, page_size, D] of any dtype (raw 16-bit patterns for bf16).
    accepted [B, A] node ids, n_accepted [B].  Returns (k_out, v_out, new_lens, skipped) -- copies; `skipped` lists the
    requests left alone."""
    k_out, v_out = np.array(k_cache, copy=True), np.array(v_cache, copy=True)
    new_lens = np.array(seq_lens, dtype=np.int64, copy=True)
    B, A = accepted.shape
    assert len(seq_lens) == B and len(n_accepted) == B
    page_size = k_cache.shape[2]
    capacity = page_size if page_table is None else page_table.shape[1] * page_size
    skipped = []
    for b in range(B):
        L, n = int(seq_lens[b]), int(n_accepted[b])
        ids = [int(x) for x in accepted[b, :max(0, min(n, A))]]
        if L < 0 or L + T > capacity or n < 0 or n > A or any(i < 0 or i >= T for i in ids):
            skipped.append(b)
            continue
        rows = []
        for i in ids:                                   # read every source row first
            page, slot = _locate(page_table, page_size, b, L + i)
            rows.append((k_cache[page, :, slot, :].copy(), v_cache[page, :, slot, :].copy()))
        for j, (kr, vr) in enumerate(rows):             # then write them in path order behind the prefix
            page, slot = _locate(page_table, page_size, b, L + j)
            k_out[page, :, slot, :] = kr
            v_out[page, :, slot, :] = vr
        new_lens[b] = L + n
    return k_out, v_out, new_lens.astype(np.int32), skipped
