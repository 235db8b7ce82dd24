"""The rules by which the KV pass cuts the batch's tile lists into workgroup shares, restated on the host and checked
for the properties the kernels rely on: every tile belongs to exactly one workgroup, a list's owners are
consecutive workgroups, and the merge pass's formula for them (first owner, number of owners) is right.

The device code lives in paper_2508_08192_amd/csrc/ta_common.h (ta_build_schedule, ta_share) and at the top of the
item loops of the KV kernels and of the merge kernels; the GPU parity tests exercise it directly.  This file pins the arithmetic itself on many random
batches, which needs no GPU."""
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


def _check(lens, Hkv, pad, n_wg, min_q):
    lists, total = _units(lens, Hkv, pad)
    share = max(min_q, -(-total // n_wg))
    owner_of_tile = {}
    for w in range(n_wg):
        t, t_end = w * share, min(total, (w + 1) * share)
        for i, (seg, n_b, n_u) in enumerate(lists):
            j0, j1 = max(t, seg) - seg, min(t_end, seg + n_b) - seg
            for j in range(max(j0, 0), max(j1, 0)):
                assert (i, j) not in owner_of_tile
                owner_of_tile[(i, j)] = w
    assert len(owner_of_tile) == sum(l[1] for l in lists), "a tile has no owner"
    for i, (seg, n_b, n_u) in enumerate(lists):
        owners = sorted({owner_of_tile[(i, j)] for j in range(n_b)})
        w_first = seg // share
        n_parts = (seg + n_b - 1) // share - w_first + 1
        assert owners == list(range(w_first, w_first + n_parts)), (i, owners, w_first, n_parts)
        # slots w + i of consecutive (workgroup, list) overlaps never collide and stay below n_wg + number of lists
        assert w_first + n_parts - 1 + i < n_wg + len(lists)


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
