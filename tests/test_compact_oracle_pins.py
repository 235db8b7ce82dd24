"""Pins of the bookkeeping oracle (oracle/kv_compact_oracle.py) against things other than itself (CPU only).

Paper section 3, stage 6 (after acceptance the KV cache is rewound to the accepted length) read together with
section 3.1/3.4 (tree node i lives at cache position L_b + i): once the accepted path has been moved behind the
prefix, plain decoding over the rewound cache must see exactly what the path's nodes saw under tree attention.
"""
import importlib.util
import os

import numpy as np
import pytest

from oracle import kv_compact_oracle as KC
from paper_2508_08192_amd import workloads as W

from .helpers import ancestors_inclusive, run_oracle


def _problem(paged=True, ps=8, dtype="bf16", seed=3, T=11, lens=(37, 0, 16)):
    rng = np.random.default_rng(seed)
    tree = W.shuffle_tree(W.random_deep_tree(T, 4, rng), rng)[0]    # parents need not precede children
    return W.make_workload("compact", B=len(lens), T=T, Hq=4, Hkv=2, D=16, seq_lens=list(lens), trees=tree,
                           page_size=ps, dtype=dtype, seed=seed, paged=paged)


def _deepest_paths(w):
    """Per request: the root-to-node path of one deepest node (ids, root first)."""
    par = np.broadcast_to(w.tree_parent, (w.B, w.T)) if w.tree_parent.ndim == 1 else w.tree_parent
    paths = []
    for b in range(w.B):
        cand = [ancestors_inclusive(par[b], i) for i in range(w.T)]
        paths.append(max(cand, key=len))
    return paths


def _pack(paths, A):
    acc = np.full((len(paths), A), -7, dtype=np.int32)              # entries past n are never read
    n = np.zeros(len(paths), dtype=np.int32)
    for b, p in enumerate(paths):
        acc[b, :len(p)] = p
        n[b] = len(p)
    return acc, n


def _compact(w, acc, n, oracle_fn=None):
    fn = oracle_fn or KC.kv_compact_oracle
    return fn(w.k_cache, w.v_cache, w.page_table, w.seq_lens, acc, n, w.T)


@pytest.mark.parametrize("paged,ps", [(True, 8), (True, 4), (False, 64)])
def test_decoding_over_the_rewound_cache_sees_what_the_path_saw(paged, ps, oracle_fn=None):
    """For every depth d of the accepted path: one-token attention of that node's query over the rewound cache cut at
    L + d + 1 equals the node's tree-attention output over the original cache (attention oracle, itself pinned)."""
    w = _problem(paged=paged, ps=ps)
    ref, ref_lse = run_oracle(w)
    paths = _deepest_paths(w)
    assert max(len(p) for p in paths) >= 3
    acc, n = _pack(paths, w.T)
    k2, v2, new_lens, skipped = _compact(w, acc, n, oracle_fn)
    assert skipped == [] and (new_lens == w.seq_lens + n).all()
    import oracle
    for d in range(max(len(p) for p in paths)):
        rows = [b for b in range(w.B) if d < len(paths[b])]
        q1 = np.stack([w.q[b, paths[b][d]] for b in range(w.B) if b in rows])[:, None]     # [B', 1, Hq, D]
        lens1 = np.int32([w.seq_lens[b] + d for b in rows])                                  # the token itself is the tree
        pt = None if w.page_table is None else w.page_table[rows]
        kk, vv = (k2, v2) if pt is not None else (k2[rows], v2[rows])
        out1, lse1 = oracle.tree_attn_oracle(q1, kk, vv, pt, lens1, np.int32([-1]), scale=w.scale)
        for r, b in enumerate(rows):
            np.testing.assert_allclose(out1[r, 0], ref[b, paths[b][d]], rtol=0, atol=1e-12)
            np.testing.assert_allclose(lse1[r, :, 0], ref_lse[b, :, paths[b][d]], rtol=0, atol=1e-12)


def test_contiguous_layout_is_a_library_gather(oracle_fn=None):
    """Without a page table the cache is [B, Hkv, capacity, D]: the move is a fancy-indexed gather per request (the
    right-hand side is evaluated before the assignment, so overlapping sources and destinations are safe)."""
    w = _problem(paged=False, ps=64, dtype="f32", seed=9)
    acc = np.int32([[0, 2, 1, 5, 3, 4, 0], [3, 3, 3, 0, 0, 0, 0], [10, 9, 8, 7, 6, 5, 4]])   # swaps, repeats, reversal
    n = np.int32([6, 3, 7])
    k2, v2, new_lens, skipped = _compact(w, acc, n, oracle_fn)
    assert skipped == []
    for src, got in ((w.k_cache, k2), (w.v_cache, v2)):
        exp = src.copy()
        for b in range(w.B):
            L = int(w.seq_lens[b])
            exp[b][:, L:L + n[b]] = src[b][:, L + acc[b, :n[b]]]
        assert np.array_equal(exp, got)
    assert (new_lens == w.seq_lens + n).all()


def test_only_the_accepted_positions_change_and_bad_requests_are_left_alone(oracle_fn=None):
    w = _problem(paged=True, ps=4, seed=21, lens=(9, 30, 5, 12))
    acc = np.int32([[0, 4, 7, 0], [0, 11, 2, 3], [1, -1, 0, 0], [5, 6, 0, 0]])   # request 1: id == T, request 2: id < 0
    n = np.int32([3, 2, 2, 5])                                                    # request 3: n beyond the list
    k2, v2, new_lens, skipped = _compact(w, acc, n, oracle_fn)
    assert skipped == [1, 2, 3]
    assert list(new_lens) == [12, 30, 5, 12]
    changed = np.zeros(w.k_cache.shape[:1] + w.k_cache.shape[2:3], dtype=bool)    # [page, slot]
    for j in range(3):
        pos = 9 + j
        changed[w.page_table[0, pos // 4], pos % 4] = True
    for src, got in ((w.k_cache, k2), (w.v_cache, v2)):
        same = (src == got).all(axis=(1, 3))                                      # [page, slot]
        assert same[~changed].all()
    # zero accepted tokens: nothing moves, the length stays
    k3, v3, lens3, sk3 = _compact(w, acc, np.zeros(4, dtype=np.int32), oracle_fn)     # (ids past n are never looked at)
    assert np.array_equal(k3, w.k_cache) and np.array_equal(v3, w.v_cache) and sk3 == []
    assert list(lens3) == [9, 30, 5, 12]
    # a prefix that leaves no room for the tree is out of range as a whole
    w.seq_lens[0] = w.page_table.shape[1] * 4 - w.T + 1
    assert _compact(w, acc, np.int32([1, 0, 0, 0]), oracle_fn)[3] == [0]


# --- the pins must be able to see a mistake: each one planted in a copy of the oracle's source has to fail one of them
MUTATIONS = [
    ("rows written while later sources are still unread", "rows.append((k_cache[page, :, slot, :].copy(), v_cache[page, :, slot, :].copy()))",
     "rows.append((k_out[page, :, slot, :], v_out[page, :, slot, :]))"),
    ("source position without the prefix length", "_locate(page_table, page_size, b, L + i)", "_locate(page_table, page_size, b, i)"),
    ("destination is the node's own slot", "for j, (kr, vr) in enumerate(rows):", "for j, (kr, vr) in zip(ids, rows):"),
    ("path written leaf first", "for j, (kr, vr) in enumerate(rows):", "for j, (kr, vr) in enumerate(rows[::-1]):"),
    ("values not moved", "v_out[page, :, slot, :] = vr", "pass"),
    ("length not advanced", "new_lens[b] = L + n", "new_lens[b] = L"),
    ("slot without the page table", "return int(page_table[b, pos // page_size]), pos % page_size",
     "return int(page_table[b, 0]) + pos // page_size, pos % page_size"),
]


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(name, old, new, tmp_path):
    src = open(KC.__file__).read()
    assert src.count(old) == 1, "mutation anchor not unique: %r" % old
    path = tmp_path / "kv_compact_mutant.py"
    path.write_text(src.replace(old, new))
    spec = importlib.util.spec_from_file_location("kv_compact_mutant", os.fspath(path))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    failed = []
    for fn, kw in ((test_decoding_over_the_rewound_cache_sees_what_the_path_saw, dict(paged=True, ps=4)),
                   (test_contiguous_layout_is_a_library_gather, {}),
                   (test_only_the_accepted_positions_change_and_bad_requests_are_left_alone, {})):
        try:
            fn(oracle_fn=mod.kv_compact_oracle, **kw)
        except (AssertionError, IndexError):
            failed.append(fn.__name__)
    assert failed, "no pin noticed: " + name
