"""Pure-Python brute force for tiny tree-attention inputs (test infrastructure only).

Independent of the C oracle: it shares no helper with it.  For each node it
materialises the explicit list of (key row, value row) pairs the node may see
-- the whole cached prefix, then every tree node that lies on the way from a
root down to the node (paper section 3.1: a node sees the context and its own
path, as if the path were unrolled into a sequence) -- and runs a few lines of
softmax over that list with Python floats.  The ancestor relation is found
top-down (children lists, depth-first from each root), not by walking parents.
"""
import math


def _visible_sets(parent):
    T = len(parent)
    children = [[] for _ in range(T)]
    roots = []
    for i, p in enumerate(parent):
        if p < 0:
            roots.append(i)
        else:
            children[p].append(i)
    seen = {}

    def descend(node, trail):
        trail = trail + [node]
        seen[node] = list(trail)
        for c in children[node]:
            descend(c, trail)

    for r in roots:
        descend(r, [])
    assert len(seen) == T, "parent array is not a forest"
    return seen


def _softmax_attend(qrow, pairs, scale):
    logits = [scale * sum(a * b for a, b in zip(qrow, k)) for k, _ in pairs]
    top = max(logits)
    weights = [math.exp(x - top) for x in logits]
    z = sum(weights)
    D = len(pairs[0][1])
    out = [sum(w * v[d] for w, (_, v) in zip(weights, pairs)) / z for d in range(D)]
    return out, top + math.log(z)


def brute_force_tree_attention(q, k_of, v_of, seq_lens, parents, G, scale):
    """q[b][i][h] -> list of D floats; k_of(b, g, pos) / v_of(b, g, pos) -> list of D floats for
    logical cache position pos; parents[b] -> list of T parent ids.
    Returns out[b][i][h] (list of D floats) and lse[b][h][i]."""
    B = len(q)
    out, lse = [], []
    for b in range(B):
        T, Hq = len(q[b]), len(q[b][0])
        vis = _visible_sets(list(parents[b]))
        ob = [[None] * Hq for _ in range(T)]
        lb = [[None] * T for _ in range(Hq)]
        for i in range(T):
            for h in range(Hq):
                g = h // G
                positions = list(range(seq_lens[b])) + [seq_lens[b] + j for j in vis[i]]
                pairs = [(k_of(b, g, pos), v_of(b, g, pos)) for pos in positions]
                ob[i][h], lb[h][i] = _softmax_attend(q[b][i][h], pairs, scale)
        out.append(ob)
        lse.append(lb)
    return out, lse
