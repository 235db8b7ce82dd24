"""GPU tests of what the library promises beyond the arithmetic: data-dependent mistakes end in NaN rows and a status
bit (never in a wild address), the caller's own status word, pages released before a window start are never read,
and the library-owned workspace outlives captured graphs."""
import numpy as np
import pytest

from paper_2508_08192_amd import workloads as W

from .helpers import assert_parity, run_hip, run_oracle, to_device

pytestmark = pytest.mark.gpu

GENERIC, MFMA, MFMA_BASIC = 1, 2, 3


def _announce(name):
    print("\n[case] %s" % name, flush=True)


def _with_decoy_pages(w, dev, extra=4):
    """The caches become views of the first pages of larger allocations whose extra pages hold NaN: a page id in
    [num_pages, num_pages + extra) is outside the cache the call was given, yet inside memory this process owns."""
    import torch
    out = {}
    for key in ("k_cache", "v_cache"):
        t = dev[key]
        full = torch.full((t.shape[0] + extra,) + tuple(t.shape[1:]), float("nan"), dtype=t.dtype, device=t.device)
        full[:t.shape[0]] = t
        out[key] = full[:t.shape[0]]
    dev.update(out)
    return dev


@pytest.mark.parametrize("kernel", [GENERIC, MFMA, MFMA_BASIC])
def test_page_ids_outside_the_cache_poison_the_request(kernel):
    import torch
    from paper_2508_08192_amd import treeattn as ta
    rng = np.random.default_rng(5)
    T = 12
    trees = np.stack([W.random_tree(T, 5, rng) for _ in range(4)])
    w = W.make_workload("badpage", B=4, T=T, Hq=8, Hkv=2, D=128, seq_lens=[900, 300, 1500, 64], trees=trees,
                        page_size=64, dtype="bf16", seed=1777)
    n_pages = w.k_cache.shape[0]
    ref, ref_lse = run_oracle(w)
    ta.tree_attn_last_status()
    for bad_id, where in ((n_pages, "first id past the cache"), (n_pages + 3, "a later one"), (-1, "negative")):
        dev = _with_decoy_pages(w, to_device(w))
        pt = w.page_table.copy()
        pt[1, 2] = bad_id                              # inside request 1's prefix
        pt[2, (1500 + T - 1) // 64] = bad_id           # the page of request 2's last tree tokens
        dev["page_table"] = torch.from_numpy(pt).cuda()
        own = torch.zeros(1, dtype=torch.int32, device="cuda")
        _announce("page id %d (%s), kernel %d" % (bad_id, where, kernel))
        got, got_lse = run_hip(w, dev, kernel=kernel, status=own)
        assert ta.tree_attn_last_status() == ta.TA_STATUS_BAD_PAGE
        assert int(own.item()) == ta.TA_STATUS_BAD_PAGE
        assert np.isnan(got[1]).all() and np.isnan(got[2]).all() and np.isnan(got_lse[1]).all()
        assert_parity(got[[0, 3]], got_lse[[0, 3]], ref[[0, 3]], ref_lse[[0, 3]], "bf16", "healthy requests")
    # ids past what a request uses are never looked at
    dev = _with_decoy_pages(w, to_device(w))
    pt = w.page_table.copy()
    pt[3, 2:] = n_pages + 1
    dev["page_table"] = torch.from_numpy(pt).cuda()
    got, got_lse = run_hip(w, dev, kernel=kernel)
    assert ta.tree_attn_last_status() == 0
    assert_parity(got, got_lse, ref, ref_lse, "bf16", "unused table entries")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_write_back_and_bookkeeping_skip_pages_outside_the_cache(dtype):
    import torch
    from paper_2508_08192_amd import treeattn as ta
    T, Hkv, D = 6, 2, 64 if dtype == "f32" else 128
    w = W.make_workload("badpage_wb", B=3, T=T, Hq=4, Hkv=Hkv, D=D, seq_lens=[30, 61, 10], trees=W.chain_tree(T),
                        page_size=16, dtype=dtype, seed=1888)
    n_pages = w.k_cache.shape[0]
    dev = _with_decoy_pages(w, to_device(w))
    pt = w.page_table.copy()
    pt[1, (61 + 3) // 16] = n_pages + 2                # the page of request 1's tree tokens 3..5
    dev["page_table"] = torch.from_numpy(pt).cuda()
    before_k, before_v = dev["k_cache"].clone(), dev["v_cache"].clone()
    k_new = torch.ones((3, T, Hkv, D), dtype=dev["k_cache"].dtype, device="cuda")
    v_new = torch.full_like(k_new, 2.0)
    ta.tree_attn_last_status()
    _announce("append with a page outside the cache, %s" % dtype)
    ta.tree_attn_append(k_new, v_new, dev["k_cache"], dev["v_cache"], dev["page_table"], dev["seq_lens"])
    assert ta.tree_attn_last_status() == ta.TA_STATUS_BAD_PAGE
    kc = dev["k_cache"].float().cpu().numpy()
    for b, L in enumerate([30, 61, 10]):
        for i in range(T):
            pos = L + i
            page, slot = int(pt[b, pos // 16]), pos % 16
            if page < n_pages:
                assert (kc[page, :, slot, :] == 1.0).all(), (b, i)
    # only those rows changed
    changed = (dev["k_cache"] != before_k).any(dim=3).any(dim=1).sum().item()
    assert changed == 3 * T - 3
    _announce("compact with a page outside the cache, %s" % dtype)
    acc = torch.tensor([[0, 1, 2], [0, 1, 2], [0, 2, 4]], dtype=torch.int32, device="cuda")
    n = torch.tensor([3, 3, 3], dtype=torch.int32, device="cuda")
    lens_out = torch.zeros(3, dtype=torch.int32, device="cuda")
    snap = dev["k_cache"].clone()
    ta.tree_attn_compact(dev["k_cache"], dev["v_cache"], dev["page_table"], dev["seq_lens"], acc, n, T,
                         seq_lens_out=lens_out)
    assert ta.tree_attn_last_status() == ta.TA_STATUS_BAD_PAGE
    assert lens_out.cpu().tolist() == [33, 61, 13]                     # request 1 is left alone
    pages1 = [int(x) for x in pt[1] if 0 <= x < n_pages]
    assert torch.equal(dev["k_cache"][pages1].view(torch.uint8), snap[pages1].view(torch.uint8))


@pytest.mark.parametrize("kernel", [GENERIC, MFMA, MFMA_BASIC])
def test_given_masks_of_a_malformed_tree_poison_the_request(kernel):
    """tree_attn_encode writes all-zero words for a malformed tree; a later call that takes those masks must treat
    the request as it treats a malformed parent array."""
    import torch
    from paper_2508_08192_amd import treeattn as ta
    T = 8
    trees = np.int32([[-1, 0, 1, 2, 3, 4, 5, 6], [-1, 0, 3, 2, 0, 0, 0, 0], [-1, 0, 0, 0, 1, 1, 2, 2]])   # a cycle in #1
    for lens in ([40, 40, 40], [0, 0, 0]):
        w = W.make_workload("badmask", B=3, T=T, Hq=4, Hkv=2, D=128, seq_lens=lens, trees=trees, page_size=16,
                            dtype="bf16", seed=1301)
        ref, ref_lse = run_oracle(w)
        dev = to_device(w)
        masks = torch.zeros((3, T), dtype=torch.int64, device="cuda")
        ta.tree_attn_encode(dev["tree_parent"], masks)
        assert ta.tree_attn_last_status() == ta.TA_STATUS_BAD_PARENT
        assert (masks[1] == 0).all().item()
        own = torch.zeros(1, dtype=torch.int32, device="cuda")
        _announce("given masks of a cyclic tree, L=%r, kernel %d" % (lens, kernel))
        got, got_lse = run_hip(w, dev, kernel=kernel, tree_masks=masks, status=own)
        assert ta.tree_attn_last_status() == ta.TA_STATUS_BAD_PARENT and int(own.item()) == ta.TA_STATUS_BAD_PARENT
        assert np.isnan(got[1]).all() and np.isnan(got_lse[1]).all()
        assert_parity(got[[0, 2]], got_lse[[0, 2]], ref[[0, 2]], ref_lse[[0, 2]], "bf16", "healthy requests")


def test_the_callers_status_word_collects_the_bits_and_is_left_alone_otherwise():
    import torch
    from paper_2508_08192_amd import treeattn as ta
    T = 8
    trees = np.int32([[-1, 0, 1, 2, 3, 4, 5, 6], [-1, 0, 9, 1, 1, 1, 1, 1]])
    w = W.make_workload("own_status", B=2, T=T, Hq=4, Hkv=2, D=128, seq_lens=[40, -2], trees=trees, page_size=16,
                        dtype="bf16", seed=1401)
    ta.tree_attn_last_status()
    own = torch.full((1,), 64, dtype=torch.int32, device="cuda")            # a bit of the caller's own stays
    run_hip(w, kernel=MFMA, status=own)
    assert int(own.item()) == 64 | ta.TA_STATUS_BAD_SEQLEN
    w.seq_lens[1] = 40
    run_hip(w, kernel=MFMA, status=own)
    assert int(own.item()) == 64 | ta.TA_STATUS_BAD_SEQLEN | ta.TA_STATUS_BAD_PARENT
    assert ta.tree_attn_last_status() == ta.TA_STATUS_BAD_SEQLEN | ta.TA_STATUS_BAD_PARENT
    w.tree_parent[1] = trees[0]
    own.zero_()
    run_hip(w, kernel=MFMA, status=own)
    assert int(own.item()) == 0 and ta.tree_attn_last_status() == 0


@pytest.mark.parametrize("kernel", [GENERIC, MFMA, MFMA_BASIC])
@pytest.mark.parametrize("ps", [4, 16, 64])
def test_pages_before_the_window_start_are_never_read(kernel, ps):
    """Local attention (section 3.4, iRoPE): a caller may already have released the pages before the window.  Their
    table entries name pages outside the cache here; the result must not notice."""
    import torch
    from paper_2508_08192_amd import treeattn as ta
    rng = np.random.default_rng(8)
    T = 8
    lens = [700, 333, 90, 1000]
    starts = np.int32([333, 200, 90, 7])               # mid-tile, mid-page, empty window, almost everything
    trees = np.stack([W.random_tree(T, 4, rng) for _ in range(4)])
    w = W.make_workload("released", B=4, T=T, Hq=8, Hkv=2, D=128, seq_lens=lens, trees=trees, page_size=ps,
                        dtype="bf16", seed=1501)
    w.kv_start = starts
    ref, ref_lse = run_oracle(w)
    dev = _with_decoy_pages(w, to_device(w))
    pt = w.page_table.copy()
    for b in range(4):
        pt[b, :int(starts[b]) // ps] = w.k_cache.shape[0] + 1          # whole pages before the window
    dev["page_table"] = torch.from_numpy(pt).cuda()
    ta.tree_attn_last_status()
    for splits in (0, 3):
        _announce("released pages, ps %d, kernel %d, splits %d" % (ps, kernel, splits))
        got, got_lse = run_hip(w, dev, kernel=kernel, num_splits=splits)
        assert ta.tree_attn_last_status() == 0
        assert_parity(got, got_lse, ref, ref_lse, "bf16", "released pages")


def test_library_workspace_outlives_a_captured_graph_and_never_grows_under_capture():
    """A graph captured with the library-owned workspace holds that buffer's address.  A later, larger eager call makes
    the library allocate a bigger buffer; the old one must stay valid, so the replay still gives the captured call's
    result.  Under capture a call that would have to allocate is refused instead."""
    import torch
    from paper_2508_08192_amd import treeattn as ta
    T = 16
    tree = W.bfs_tree(T, [3, 2], 4)
    small = W.make_workload("ws_small", B=2, T=T, Hq=4, Hkv=1, D=128, seq_lens=[600, 200], trees=tree, page_size=64,
                            dtype="bf16", seed=1601)
    big = W.make_workload("ws_big", B=24, T=64, Hq=32, Hkv=8, D=128, seq_lens=[300] * 24, trees=W.bfs_tree(64, [4], 6),
                          page_size=64, dtype="bf16", seed=1602)
    ref, ref_lse = run_oracle(small)
    ds, db = to_device(small), to_device(big)
    args = lambda d: (d["q"], d["k_cache"], d["v_cache"], d["page_table"], d["seq_lens"], d["tree_parent"], d["out"],
                      d["lse"])
    torch.cuda.synchronize()
    ta.tree_attn_release()
    side = torch.cuda.Stream()
    # nothing reserved: under capture the call must refuse to allocate and launch nothing
    _announce("growth refused under capture")
    graph0 = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph0, stream=side):
        rc = ta.tree_attn_fwd(*args(ds), stream=torch.cuda.current_stream(), check=False)
        ds["out"].zero_()                               # (an empty capture is not allowed everywhere)
    assert rc == ta.TA_ERR_WORKSPACE
    p_small = ta.tree_attn_plan(*args(ds), num_cus=torch.cuda.get_device_properties(0).multi_processor_count)
    p_big = ta.tree_attn_plan(*args(db), num_cus=torch.cuda.get_device_properties(0).multi_processor_count)
    assert p_big["workspace_bytes"] > ((p_small["workspace_bytes"] + (1 << 20) - 1) >> 20 << 20)
    ta.tree_attn_reserve(p_small["workspace_bytes"])
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        ta.tree_attn_fwd(*args(ds), stream=side)        # warm-up (kernel attributes)
    side.synchronize()
    _announce("capture with the small workspace")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        rc = ta.tree_attn_fwd(*args(ds), stream=torch.cuda.current_stream(), check=False)
    assert rc == ta.TA_OK
    for rep in range(3):
        _announce("bigger eager call, then replay %d" % rep)
        ta.tree_attn_fwd(*args(db))                     # needs more room: the library moves on to a larger buffer
        torch.cuda.synchronize()
        ds["out"].fill_(float("nan"))
        ds["lse"].fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = ds["out"].float().cpu().numpy().astype(np.float64)
        got_lse = ds["lse"].cpu().numpy().astype(np.float64)
        assert_parity(got, got_lse, ref, ref_lse, "bf16", "replay after the workspace grew")
    del graph, graph0
    torch.cuda.synchronize()
    ta.tree_attn_release()                              # and the library works on after a release
    got, got_lse = run_hip(small, ds)
    assert_parity(got, got_lse, ref, ref_lse, "bf16", "after release")


def test_measurement_probes_run():
    import torch
    from paper_2508_08192_amd import treeattn as ta
    buf = torch.ones(1 << 22, dtype=torch.float32, device="cuda")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    ta.tree_attn_stream_read(buf, sink)
    torch.cuda.synchronize()
    assert int(sink.item()) == 0
    fsink = torch.zeros(1, dtype=torch.float32, device="cuda")
    flop = ta.tree_attn_mfma_probe(10, fsink)
    torch.cuda.synchronize()
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert flop == cus * 8 * 32 * 10 * 32768 and float(fsink.item()) == 0.0


def test_the_binding_is_the_first_thing_a_process_uses():
    """A process whose first GPU call goes through the binding, before it has imported PyTorch itself: the binding has
    to bring PyTorch's HIP runtime in before the library (two runtimes in one process: every call fails)."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = ("from paper_2508_08192_amd import treeattn as ta\n"
            "print('status', ta.tree_attn_last_status())\n"
            "import torch\n"
            "x = torch.ones(1 << 20, device='cuda')\n"
            "s = torch.zeros(64, dtype=torch.float32, device='cuda')\n"
            "print('read', ta.tree_attn_stream_read(x, s))\n")
    out = subprocess.run([sys.executable, "-c", code], cwd=root, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                         text=True, timeout=300)
    assert out.returncode == 0 and "status 0" in out.stdout, out.stdout


def test_calls_on_two_streams_each_with_a_workspace_of_its_own():
    """Calls that overlap in time bring their own workspaces: two different batches launched alternately on two
    streams, twenty times each without a synchronisation in between, both against the oracle."""
    import torch
    from paper_2508_08192_amd import treeattn as ta
    rng = np.random.default_rng(99)
    wa = W.make_workload("two_a", B=4, T=64, Hq=8, Hkv=2, D=128, seq_lens=rng.integers(500, 6000, size=4),
                         trees=W.bfs_tree(64, [4, 2], 8), page_size=16, dtype="bf16", seed=9901)
    wb = W.make_workload("two_b", B=6, T=8, Hq=8, Hkv=2, D=128, seq_lens=rng.integers(100, 9000, size=6),
                         trees=W.random_tree(8, 4, rng), page_size=64, dtype="bf16", seed=9902)
    refs = [run_oracle(wa), run_oracle(wb)]
    devs = [to_device(wa), to_device(wb)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    wss, plans = [], []
    for w, d in zip((wa, wb), devs):
        plan = ta.tree_attn_plan(d["q"], d["k_cache"], d["v_cache"], d["page_table"], d["seq_lens"], d["tree_parent"],
                                 d["out"], d["lse"])
        plans.append(plan)
        wss.append(torch.empty(plan["workspace_bytes"], dtype=torch.uint8, device="cuda"))
    _announce("two streams, two workspaces")
    torch.cuda.synchronize()
    for rep in range(20):
        for d, st, ws in zip(devs, streams, wss):
            if rep == 19:
                with torch.cuda.stream(st):
                    d["out"].fill_(float("nan"))
            ta.tree_attn_fwd_ex(d["q"], d["k_cache"], d["v_cache"], d["page_table"], d["seq_lens"], d["tree_parent"],
                                d["out"], d["lse"], stream=st, workspace=ws)
    torch.cuda.synchronize()
    for (ref, ref_lse), d, w in zip(refs, devs, (wa, wb)):
        got = d["out"].float().cpu().numpy().astype(np.float64)
        got_lse = d["lse"].cpu().numpy().astype(np.float64)
        assert_parity(got, got_lse, ref, ref_lse, "bf16", w.name)
    assert ta.tree_attn_last_status() == 0


@pytest.mark.parametrize("kernel", [0, MFMA_BASIC, GENERIC])
def test_caches_beyond_four_gigabytes(kernel):
    """Page ids whose byte offsets need more than 32 bits: the requests' pages sit at the far end of caches of 5.2 GB
    each (40 000 pages of 64 tokens x 8 KV heads)."""
    import torch
    rng = np.random.default_rng(4321)
    B, T, ps = 3, 16, 64
    trees = np.stack([W.random_tree(T, 5, rng) for _ in range(B)])
    w = W.make_workload("big", B=B, T=T, Hq=32, Hkv=8, D=128, seq_lens=[3000, 64, 1500], trees=trees, page_size=ps,
                        dtype="bf16", seed=4322)
    ref, ref_lse = run_oracle(w)
    dev = to_device(w)
    n_small, n_big = dev["k_cache"].shape[0], 40000
    big_k = torch.empty((n_big,) + tuple(dev["k_cache"].shape[1:]), dtype=torch.bfloat16, device="cuda")
    big_v = torch.empty_like(big_k)
    remap = torch.from_numpy(rng.permutation(np.arange(n_big - 3000, n_big))[:n_small].astype(np.int64)).cuda()
    big_k[remap] = dev["k_cache"]
    big_v[remap] = dev["v_cache"]
    table = dev["page_table"].long()
    dev["page_table"] = torch.where((table >= 0) & (table < n_small), remap[table.clamp(0, n_small - 1)], table).int()
    dev["k_cache"], dev["v_cache"] = big_k, big_v
    _announce("caches of 5.2 GB, kernel=%d" % kernel)
    got, got_lse = run_hip(w, dev, kernel=kernel)
    assert_parity(got, got_lse, ref, ref_lse, "bf16", "caches beyond 4 GB")
    del big_k, big_v, dev
    torch.cuda.empty_cache()


def test_a_prefix_of_a_million_tokens():
    """One request with 1 000 000 cached tokens (positions and tile indices far beyond 16 bits), pages of 16 tokens."""
    rng = np.random.default_rng(1000000)
    w = W.make_workload("million", B=1, T=4, Hq=2, Hkv=1, D=128, seq_lens=[1000000], trees=W.chain_tree(4), page_size=16,
                        dtype="bf16", seed=1000001)
    _announce("one million tokens")
    ref, ref_lse = run_oracle(w)
    got, got_lse = run_hip(w)
    assert_parity(got, got_lse, ref, ref_lse, "bf16", "one million tokens")
