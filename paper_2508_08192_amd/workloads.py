"""Seeded synthetic inputs for tree attention: trees, prefix lengths, page tables, q/k/v values.

This module serves both the HIP path and the CPU oracle and therefore holds
none of the method's arithmetic: it only draws random inputs, rounds them once
to the storage type and lays them out in a paged cache.  The synthetic,
Llama-shaped workloads stand in for production traffic, which is not available.

Layouts
-------
q            [B, T, Hq, D]                      float32, or uint16 holding bf16 bit patterns
k/v cache    [num_pages, Hkv, page_size, D]     same element type as q
page_table   int32 [B, max_pages] (None = contiguous: request b owns page b)
seq_lens     int32 [B]   cached prefix length L_b (tree tokens not counted)
tree_parent  int32 [B, T] or [T]; parent of the root is -1; tree node i of
             request b has its K/V at logical cache position L_b + i.
"""
from dataclasses import dataclass, field
from typing import Optional

import numpy as np


def to_bf16_bits(x):
    """Round float32 values to bf16 (round to nearest, ties to even); returns uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    rounded = bits + np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    """Widen bf16 bit patterns (uint16) to float32 exactly."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------- trees

def chain_tree(T):
    return np.arange(-1, T - 1, dtype=np.int32)


def bfs_tree(T, branching, max_levels):
    """Level-by-level tree: a node on level l (root = level 1) gets branching[min(l, len) - 1]
    children, nodes are numbered in creation order; stop at T nodes or once level max_levels is full."""
    parent = [-1]
    level = [1]
    cur = 0
    while len(parent) < T and cur < len(parent):
        lv = level[cur]
        if lv < max_levels:
            for _ in range(branching[min(lv, len(branching)) - 1]):
                if len(parent) >= T:
                    break
                parent.append(cur)
                level.append(lv + 1)
        cur += 1
    if len(parent) != T:
        raise ValueError("tree budget %d cannot be reached with %r levels<=%d" % (T, branching, max_levels))
    return np.asarray(parent, dtype=np.int32)


def random_tree(T, max_levels, rng):
    """Parent of node i >= 1 uniform over 0..i-1, redrawn while the node would sit below max_levels."""
    parent = np.full(T, -1, dtype=np.int32)
    level = np.ones(T, dtype=np.int64)
    for i in range(1, T):
        while True:
            p = int(rng.integers(0, i))
            if level[p] + 1 <= max_levels:
                break
        parent[i] = p
        level[i] = level[p] + 1
    return parent


def random_deep_tree(T, depth, rng):
    """A spine of `depth` levels plus uniformly attached remaining nodes (no deeper than `depth`)."""
    depth = min(depth, T)
    parent = np.full(T, -1, dtype=np.int32)
    level = np.ones(T, dtype=np.int64)
    for i in range(1, depth):
        parent[i] = i - 1
        level[i] = i + 1
    for i in range(depth, T):
        while True:
            p = int(rng.integers(0, i))
            if level[p] + 1 <= depth:
                break
        parent[i] = p
        level[i] = level[p] + 1
    return parent


def shuffle_tree(parent, rng):
    """Relabel nodes with a random permutation (the result is in general NOT topologically ordered).
    Returns (new_parent, perm) with new id of old node i = perm[i]."""
    T = len(parent)
    perm = rng.permutation(T).astype(np.int32)
    new_parent = np.empty(T, dtype=np.int32)
    for i in range(T):
        new_parent[perm[i]] = -1 if parent[i] < 0 else perm[parent[i]]
    return new_parent, perm


def node_levels(parent):
    T = len(parent)
    out = np.zeros(T, dtype=np.int64)
    for i in range(T):
        n, cur = 0, i
        while cur >= 0:
            n += 1
            cur = int(parent[cur])
        out[i] = n
    return out


# ----------------------------------------------------------------------------- workloads

@dataclass
class Workload:
    name: str
    dtype: str                      # "f32" or "bf16"
    q: np.ndarray
    k_cache: np.ndarray
    v_cache: np.ndarray
    page_table: Optional[np.ndarray]
    seq_lens: np.ndarray
    tree_parent: np.ndarray
    scale: float
    meta: dict = field(default_factory=dict)
    kv_start: Optional[np.ndarray] = None     # int32 [B]: first prefix position still attended to (None: all of it)

    def window_lens(self):
        """Prefix tokens each request attends to."""
        L = self.seq_lens.astype(np.int64)
        return L if self.kv_start is None else L - self.kv_start.astype(np.int64)

    @property
    def B(self):
        return self.q.shape[0]

    @property
    def T(self):
        return self.q.shape[1]

    @property
    def Hq(self):
        return self.q.shape[2]

    @property
    def D(self):
        return self.q.shape[3]

    @property
    def Hkv(self):
        return self.k_cache.shape[1]

    @property
    def page_size(self):
        return self.k_cache.shape[2]

    def parents_2d(self):
        if self.tree_parent.ndim == 2:
            return self.tree_parent
        return np.broadcast_to(self.tree_parent, (self.B, self.T))

    def algorithmic_bytes(self):
        """Bytes the method itself must move for one verify step: every prefix and tree K and V
        element once, q in, out, lse, the page ids touched, lengths and parents."""
        es = 4 if self.dtype == "f32" else 2
        L = self.window_lens()
        kv = int((L + self.T).sum()) * self.Hkv * self.D * 2 * es
        qo = 2 * self.B * self.T * self.Hq * self.D * es
        lse = 4 * self.B * self.T * self.Hq
        pages = 0 if self.page_table is None else 4 * int(np.ceil((L + self.T) / self.page_size).sum())
        meta = 4 * self.B * (1 + self.T)
        return kv + qo + lse + pages + meta

    def useful_flops(self):
        """2 flops per multiply-add of the two contractions over every attended (query, key) pair."""
        L = self.window_lens()
        par = self.parents_2d()
        pairs = 0
        for b in range(self.B):
            pairs += self.T * int(L[b]) + int(node_levels(par[b]).sum())
        return 4 * self.D * self.Hq * pairs


_GARBAGE = 3.0e4   # large but finite: must never reach an output


def _draw_values(rng, shape, std, dtype):
    n = int(np.prod(shape))
    if dtype == "f32":
        out = rng.standard_normal(n, dtype=np.float32)
        if std != 1.0:
            out *= np.float32(std)
        return out.reshape(shape)
    out = np.empty(n, dtype=np.uint16)
    step = 1 << 24
    for s in range(0, n, step):
        chunk = rng.standard_normal(min(step, n - s), dtype=np.float32)
        if std != 1.0:
            chunk *= np.float32(std)
        out[s:s + step] = to_bf16_bits(chunk)
    return out.reshape(shape)


def make_workload(name, *, B, T, Hq, Hkv, D, seq_lens, trees, page_size, dtype="bf16", seed=0,
                  q_std=1.0, kv_std=1.0, paged=True, decoy_pages=3, permute=True, scale=None,
                  garbage=_GARBAGE):
    """Build one seeded workload.

    seq_lens: int or sequence of B prefix lengths.  trees: int32 [T] (one tree for the batch) or [B,T].
    paged=False gives the contiguous layout (page_table None, one cache row of max(L)+T slots per request).
    Cache slots that no request owns (decoy pages, the tail of each last page) hold `garbage`.
    """
    ss = np.random.SeedSequence(seed)
    s_q, s_k, s_v, s_perm = [np.random.default_rng(s) for s in ss.spawn(4)]
    seq_lens = np.broadcast_to(np.asarray(seq_lens, dtype=np.int32), (B,)).copy()
    trees = np.asarray(trees, dtype=np.int32)
    assert trees.shape in ((T,), (B, T))
    q = _draw_values(s_q, (B, T, Hq, D), q_std, dtype)
    total = seq_lens.astype(np.int64) + T
    if paged:
        pages_b = (total + page_size - 1) // page_size
        max_pages = int(pages_b.max())
        num_pages = int(pages_b.sum()) + decoy_pages
        ids = s_perm.permutation(num_pages).astype(np.int32) if permute else np.arange(num_pages, dtype=np.int32)
        page_table = np.zeros((B, max_pages), dtype=np.int32)   # unused entries point at page 0 (in range)
        cursor = 0
        for b in range(B):
            n = int(pages_b[b])
            page_table[b, :n] = ids[cursor:cursor + n]
            cursor += n
        ps = page_size
    else:
        num_pages, ps, page_table = B, int(total.max()), None
    shape = (num_pages, Hkv, ps, D)
    k_cache = _draw_values(s_k, shape, kv_std, dtype)
    v_cache = _draw_values(s_v, shape, kv_std, dtype)
    junk = np.float32(garbage) if dtype == "f32" else to_bf16_bits(np.float32([garbage]))[0]
    if paged:
        owned = np.zeros(num_pages, dtype=bool)
        for b in range(B):
            n = int(pages_b[b])
            owned[page_table[b, :n]] = True
            tail = int(total[b]) - (n - 1) * ps
            if tail < ps:
                last = page_table[b, n - 1]
                k_cache[last, :, tail:, :] = junk
                v_cache[last, :, tail:, :] = junk
        k_cache[~owned] = junk
        v_cache[~owned] = junk
    else:
        for b in range(B):
            k_cache[b, :, int(total[b]):, :] = junk
            v_cache[b, :, int(total[b]):, :] = junk
    return Workload(name=name, dtype=dtype, q=q, k_cache=k_cache, v_cache=v_cache, page_table=page_table,
                    seq_lens=seq_lens, tree_parent=trees,
                    scale=float(1.0 / np.sqrt(D)) if scale is None else float(scale),
                    meta=dict(seed=seed, q_std=q_std, kv_std=kv_std, paged=paged))


CONFIG_NAMES = ("c1_tiny_fp32", "c2_llama8b_gqa", "c3_batched_hetero", "c4_tp_share_70b", "c5_long_context")


def make_config(idx, seed=None, length_div=1):
    """The five benchmark configurations (idx 0..4).

    length_div > 1 divides every prefix length (same shapes, trees and paging) so that the CPU
    oracle can cover all outputs in seconds; length_div = 1 is the full size.
    """
    seed = 1000 + idx if seed is None else seed
    rng = np.random.default_rng(np.random.SeedSequence(seed).spawn(5)[4])
    name = CONFIG_NAMES[idx] + ("" if length_div == 1 else "_div%d" % length_div)
    if idx == 0:
        tree = np.asarray([-1, 0, 0, 1, 1, 2, 2], dtype=np.int32)       # full binary tree, 3 levels
        return make_workload(name, B=1, T=7, Hq=4, Hkv=1, D=64, seq_lens=max(128 // length_div, 1), trees=tree,
                             page_size=0, dtype="f32", seed=seed, paged=False)
    if idx == 1:
        tree = bfs_tree(64, [4], 6)
        return make_workload(name, B=1, T=64, Hq=32, Hkv=8, D=128, seq_lens=4096 // length_div, trees=tree,
                             page_size=64, seed=seed)
    if idx == 2:
        B = 32
        lens = rng.integers(512, 8192 + 1, size=B) // length_div
        trees = np.stack([random_tree(16, 5, rng) for _ in range(B)])
        return make_workload(name, B=B, T=16, Hq=32, Hkv=8, D=128, seq_lens=lens, trees=trees,
                             page_size=64, seed=seed)
    if idx == 3:
        B = 64
        lens = rng.integers(2048, 32768 + 1, size=B) // length_div
        tree = bfs_tree(32, [4, 2, 2, 1, 1], 5)
        return make_workload(name, B=B, T=32, Hq=8, Hkv=1, D=128, seq_lens=lens, trees=tree,
                             page_size=64, seed=seed)
    if idx == 4:
        tree = bfs_tree(64, [4, 2], 8)
        return make_workload(name, B=4, T=64, Hq=32, Hkv=8, D=128, seq_lens=131072 // length_div, trees=tree,
                             page_size=128, seed=seed, kv_std=0.5)
    raise IndexError(idx)


# Shapes of the regime the paper deploys (section 3.4: static pre-computed trees, a small tree at batch size 1 and a
# short chain above; N8 for the 70B model, N12 for Scout; one GPU's tensor-parallel share of the heads).  The paper
# does not print the topology of its pruned trees: these are plausible stand-ins of the same sizes.
PRODUCTION_NAMES = ("p1_70b_share_n8", "p2_70b_share_chain3", "p3_scout_share_n12", "p4_8b_n8_bs128",
                    "p5_scout_share_local", "p6_70b_share_n8_bs1", "p7_scout_share_n12_bs1_128k",
                    "u32_uniform_16k_rows32", "u64_uniform_16k_rows64", "u128_uniform_16k_rows128")
TREE_N8 = np.asarray([-1, 0, 0, 0, 1, 1, 2, 4], dtype=np.int32)                       # 8 nodes, 4 levels
TREE_N12 = np.asarray([-1, 0, 0, 0, 1, 1, 1, 2, 2, 4, 4, 9], dtype=np.int32)          # 12 nodes, 5 levels


def make_production(idx, seed=None, length_div=1):
    """Memory-bound shapes with few query rows per KV head (idx 0..9); synthetic like the five configurations.
    length_div > 1 divides every prefix length, for tests that compare all outputs with the oracle."""
    seed = 2000 + idx if seed is None else seed
    rng = np.random.default_rng(seed)
    name = PRODUCTION_NAMES[idx] + ("" if length_div == 1 else "_div%d" % length_div)
    if idx == 0:        # 70B-shaped, 8 of 64 query heads and 1 of 8 KV heads per GPU, batch 32, 8-node tree
        return make_workload(name, B=32, T=8, Hq=8, Hkv=1, D=128, seq_lens=rng.integers(1024, 16384 + 1, size=32) // length_div,
                             trees=TREE_N8, page_size=64, seed=seed)
    if idx == 1:        # the same share at batch 64 with a chain of 3 draft tokens behind the root
        return make_workload(name, B=64, T=4, Hq=8, Hkv=1, D=128, seq_lens=rng.integers(1024, 16384 + 1, size=64) // length_div,
                             trees=chain_tree(4), page_size=64, seed=seed)
    if idx == 2:        # Scout-shaped (40 query heads, 8 KV heads), one GPU of eight: 5 query heads on 1 KV head
        return make_workload(name, B=16, T=12, Hq=5, Hkv=1, D=128, seq_lens=rng.integers(8192, 65536 + 1, size=16) // length_div,
                             trees=TREE_N12, page_size=128, seed=seed)
    if idx == 3:        # 8B-shaped on one GPU, batch 128, short prefixes, 8-node tree
        return make_workload(name, B=128, T=8, Hq=32, Hkv=8, D=128, seq_lens=rng.integers(256, 4096 + 1, size=128) // length_div,
                             trees=TREE_N8, page_size=64, seed=seed)
    if idx == 4:        # p3's shape on a local-attention layer (section 3.4, iRoPE for Llama4): the prefix is the current 8192-token chunk
        w = make_workload(name, B=16, T=12, Hq=5, Hkv=1, D=128,
                          seq_lens=rng.integers(8192, 65536 + 1, size=16) // length_div,
                          trees=TREE_N12, page_size=128, seed=seed)
        chunk = max(8192 // length_div, 1)
        w.kv_start = (w.seq_lens // chunk * chunk).astype(np.int32)
        return w
    if idx == 5:        # batch size one, where the paper quotes its decoding latency: the 70B share, 8-node tree, 8k context
        return make_workload(name, B=1, T=8, Hq=8, Hkv=1, D=128, seq_lens=8192 // length_div, trees=TREE_N8,
                             page_size=64, seed=seed)
    if idx == 6:        # batch size one at a long context: the Scout share, 12-node tree, 128k tokens
        return make_workload(name, B=1, T=12, Hq=5, Hkv=1, D=128, seq_lens=131072 // length_div, trees=TREE_N12,
                             page_size=128, seed=seed)
    if idx in (7, 8, 9):  # uniform long prefixes, the purely memory-bound regime: 8B-shaped heads, batch 16, 16k context
        T = (8, 16, 32)[idx - 7]                       # 8-, 16- and 32-node trees on 4 query heads per KV head: 32/64/128 rows
        tree = TREE_N8 if T == 8 else bfs_tree(T, [3, 2], 5)
        return make_workload(name, B=16, T=T, Hq=32, Hkv=8, D=128, seq_lens=16384 // length_div, trees=tree,
                             page_size=64, seed=seed)
    raise IndexError(idx)
