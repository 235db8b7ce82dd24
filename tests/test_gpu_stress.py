"""Seeded random combinations of shape, window start, query range, folded write-back, forced splits and kernel family
against the oracles, each followed by a random bookkeeping call on the same cache.  One process, stops at the first
failure; every case prints what names it before it runs."""
import numpy as np
import pytest

from paper_2508_08192_amd import workloads as W

from .helpers import assert_parity, run_hip, run_oracle, to_device

pytestmark = pytest.mark.gpu

N_CASES = 200


def _case(seed):
    import torch
    from paper_2508_08192_amd import treeattn as ta
    from oracle import kv_compact_oracle as KC
    rng = np.random.default_rng(77000 + seed)
    T = int(rng.choice([1, 3, 4, 8, 12, 16, 31, 33, 64]))
    G = int(rng.choice([1, 2, 4, 5, 8]))
    Hkv = int(rng.choice([1, 2]))
    B = int(rng.integers(1, 4))
    ps = int(rng.choice([0, 4, 8, 16, 32, 64, 128]))
    Lmax = int(rng.choice([200, 3000, 20000]))
    lens = [int(rng.integers(0, Lmax + 1)) for _ in range(B)]
    trees = np.stack([W.random_tree(T, int(rng.integers(2, 8)), rng) for _ in range(B)])
    kernel = int(rng.choice([0, 0, 0, 1, 3])) if Lmax <= 3000 else 0
    w = W.make_workload("s%d" % seed, B=B, T=T, Hq=G * Hkv, Hkv=Hkv, D=128, seq_lens=lens, trees=trees,
                        page_size=ps if ps else 64, dtype="bf16", seed=78000 + seed, paged=ps > 0)
    use_win = rng.random() < 0.4
    if use_win:
        w.kv_start = np.int32([int(rng.integers(0, L + 1)) // 4 * 4 for L in lens])
    tq = int(rng.integers(1, T + 1))
    off = int(rng.integers(0, T - tq + 1))
    use_new = rng.random() < 0.5
    splits = int(rng.choice([0, 0, 0, 3, 40, 300]))
    print("\n[case] seed=%d T=%d G=%d Hkv=%d B=%d ps=%d L=%r kernel=%d win=%s q=%d+%d new=%s splits=%d" % (
        seed, T, G, Hkv, B, ps, lens, kernel, use_win, off, tq, use_new, splits), flush=True)
    ref, ref_lse = run_oracle(w)
    dev = to_device(w)
    opts = dict(kernel=kernel, num_splits=splits, q_node_offset=off)
    full_k, full_v = dev["k_cache"].clone(), dev["v_cache"].clone()
    if use_new:
        # the tree tokens leave the cache (their slots get a marker) and come back through the call's write-back
        k_new = torch.empty((B, T, Hkv, 128), dtype=torch.bfloat16, device="cuda")
        v_new = torch.empty_like(k_new)
        for b in range(B):
            for i in range(T):
                pos = lens[b] + i
                page, slot = (b, pos) if w.page_table is None else (int(w.page_table[b, pos // ps]), pos % ps)
                k_new[b, i] = full_k[page, :, slot, :]
                v_new[b, i] = full_v[page, :, slot, :]
                dev["k_cache"][page, :, slot, :] = 9.0
                dev["v_cache"][page, :, slot, :] = 9.0
        opts.update(k_new=k_new, v_new=v_new)
    dev["q"] = dev["q"][:, off:off + tq].contiguous()
    dev["out"] = torch.empty_like(dev["q"])
    dev["lse"] = torch.empty((B, w.Hq, tq), dtype=torch.float32, device="cuda")
    got, got_lse = run_hip(w, dev, **opts)
    assert_parity(got, got_lse, ref[:, off:off + tq], ref_lse[:, :, off:off + tq], "bf16", "seed %d" % seed)
    assert torch.equal(dev["k_cache"].view(torch.int16), full_k.view(torch.int16))
    assert torch.equal(dev["v_cache"].view(torch.int16), full_v.view(torch.int16))
    # bookkeeping on the same cache
    A = int(rng.integers(1, T + 1))
    acc = rng.integers(0, T, size=(B, A)).astype(np.int32)
    n = rng.integers(0, A + 1, size=B).astype(np.int32)
    k_ref, v_ref, lens_ref, skipped = KC.kv_compact_oracle(w.k_cache, w.v_cache, w.page_table, w.seq_lens, acc, n, T)
    ta.tree_attn_compact(dev["k_cache"], dev["v_cache"], dev["page_table"], dev["seq_lens"],
                         torch.from_numpy(acc).cuda(), torch.from_numpy(n).cuda(), T, seq_lens_out=dev["seq_lens"])
    torch.cuda.synchronize()
    assert skipped == [] and np.array_equal(dev["seq_lens"].cpu().numpy(), lens_ref)
    assert np.array_equal(dev["k_cache"].view(torch.int16).cpu().numpy(), k_ref.view(np.int16))
    assert np.array_equal(dev["v_cache"].view(torch.int16).cpu().numpy(), v_ref.view(np.int16))
    assert ta.tree_attn_last_status() == 0


def test_random_combinations_against_the_oracles():
    from paper_2508_08192_amd import treeattn as ta
    ta.tree_attn_last_status()
    for seed in range(N_CASES):
        _case(seed)
