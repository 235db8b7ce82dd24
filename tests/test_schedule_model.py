"""The rules by which the KV pass cuts the batch's tile lists into workgroup shares, restated on the host and checked
for the properties the kernels rely on: every tile belongs to exactly one workgroup, a list's owners are
consecutive workgroups (the merge pass reads the partials of all workgroups from the owner of the list's first tile to
the owner of its last one), no share is longer than ceil(total / n_wg) or the smallest share, and batches of equal
lists that divide evenly among the workgroups are cut at the lists' edges.

The device code lives in paper_2508_08192_amd/csrc/ta_common.h (ta_build_schedule, ta_share, ta_wg_range) and at the
top of the item loops of the KV kernels; the GPU parity tests exercise it directly.  This file pins the arithmetic
itself on many random batches, which needs no GPU."""
import numpy as np


def _units(lens, Hkv, pad):
    """Per list: (first unit, number of tiles, units incl. padding)."""
    out, u = [], 0
    for L in lens:
        n_b = (L + 63) // 64 + 1
        for _ in range(Hkv):
            out.append((u, n_b, n_b + pad))
            u += n_b + pad
    return out, u


def _cuts(total, n_wg, min_q):
    share = max(min_q, -(-total // n_wg))
    n_act = n_wg if n_wg * max(8, min_q) <= total else -(-total // share)
    return [total if k >= n_act else k * total // n_act for k in range(n_wg + 1)], share


def _check(lens, Hkv, pad, n_wg, min_q):
    lists, total = _units(lens, Hkv, pad)
    cuts, share = _cuts(total, n_wg, min_q)
    assert cuts[0] == 0 and cuts[-1] == total and all(0 <= b - a <= share for a, b in zip(cuts, cuts[1:]))
    owner_of_tile = {}
    for w in range(n_wg):
        t, t_end = cuts[w], cuts[w + 1]
        for i, (seg, n_b, n_u) in enumerate(lists):
            j0, j1 = max(t, seg) - seg, min(t_end, seg + n_b) - seg
            for j in range(max(j0, 0), max(j1, 0)):
                assert (i, j) not in owner_of_tile
                owner_of_tile[(i, j)] = w
    assert len(owner_of_tile) == sum(l[1] for l in lists), "a tile has no owner"
    for i, (seg, n_b, n_u) in enumerate(lists):
        owners = sorted({owner_of_tile[(i, j)] for j in range(n_b)})
        w_first, w_last = owner_of_tile[(i, 0)], owner_of_tile[(i, n_b - 1)]
        assert owners == list(range(w_first, w_last + 1)), (i, owners, w_first, w_last)
        # slots w + i of consecutive (workgroup, list) overlaps never collide and stay below n_wg + number of lists
        assert w_last + i < n_wg + len(lists)


def test_equal_lists_that_divide_evenly_are_cut_at_their_edges():
    """128 lists of 16384 tokens (256 prefix tiles, the tree tile, 8 units of padding) over 256 workgroups: two
    workgroups per list, no workgroup enters a second list."""
    for n_lists, n_wg, tiles, pad in ((128, 256, 257, 8), (128, 256, 257, 17), (64, 256, 129, 8), (512, 256, 33, 8)):
        total = n_lists * (tiles + pad)
        cuts, _ = _cuts(total, n_wg, 1)
        for w in range(n_wg):
            first, last = cuts[w] // (tiles + pad), (cuts[w + 1] - 1) // (tiles + pad)
            per_wg = max(1, n_lists // n_wg)
            assert last - first + 1 == per_wg, (n_lists, n_wg, w, first, last)


def test_shares_partition_the_tiles_and_the_merge_formula_finds_the_owners():
    rng = np.random.default_rng(2024)
    for case in range(400):
        B = int(rng.integers(1, 9))
        kind = case % 4
        if kind == 0:
            lens = rng.integers(0, 600, B)                      # many tiny lists, shorter than the padding
        elif kind == 1:
            lens = rng.integers(0, 20000, B)
        elif kind == 2:
            lens = np.full(B, int(rng.integers(1, 40)) * 64 * int(rng.integers(1, 9)))   # uniform, tile-aligned
        else:
            lens = rng.integers(0, 3, B) * int(rng.integers(1, 5000))
        Hkv = int(rng.integers(1, 4))
        pad = int(rng.choice([0, 1, 2, 8, 13, 40]))
        n_wg = int(rng.choice([1, 2, 3, 7, 64, 256, 1024]))
        min_q = int(rng.choice([1, 4]))
        _check([int(x) for x in lens], Hkv, pad, n_wg, min_q)
