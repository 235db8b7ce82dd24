"""Parity of the HIP path (through the C-ABI) against the fp64 oracle on the same seeded inputs."""
import numpy as np
import pytest

from paper_2508_08192_amd import workloads as W

from .helpers import ancestors_inclusive, assert_parity, run_hip, run_oracle, to_device

pytestmark = pytest.mark.gpu

GENERIC, MFMA, MFMA_BASIC = 1, 2, 3


def _announce(name):
    print("\n[case] %s" % name, flush=True)


def _check(w, what=None, **opts):
    _announce(what or w.name)
    ref, ref_lse = run_oracle(w)
    got, got_lse = run_hip(w, **opts)
    assert_parity(got, got_lse, ref, ref_lse, w.dtype, what or w.name)
    return got, got_lse


def test_c1_tiny_fp32_exact_config():
    w = W.make_config(0)
    _check(w)
    _check(w, "c1 with 3 shares", num_splits=3)


@pytest.mark.parametrize("kernel", [GENERIC, MFMA])
@pytest.mark.parametrize("L", [0, 1, 63, 64, 65, 200, 777])
def test_bf16_prefix_length_sweep(kernel, L):
    rng = np.random.default_rng(L)
    B, T = 3, 16
    trees = np.stack([W.random_tree(T, 5, rng) for _ in range(B)])
    w = W.make_workload("sweep", B=B, T=T, Hq=8, Hkv=2, D=128, seq_lens=[L, L + 17, max(L - 1, 0)], trees=trees,
                        page_size=16, dtype="bf16", seed=200 + L)
    _check(w, "L=%d kernel=%d" % (L, kernel), kernel=kernel)


@pytest.mark.parametrize("kernel", [GENERIC, MFMA])
def test_tree_straddles_a_page_boundary(kernel):
    rng = np.random.default_rng(5)
    ps, T = 64, 32
    trees = np.stack([W.random_deep_tree(T, 9, rng) for _ in range(4)])
    w = W.make_workload("straddle", B=4, T=T, Hq=4, Hkv=1, D=128, seq_lens=[ps - 1, 2 * ps - 5, 3 * ps, 3 * ps - T],
                        trees=trees, page_size=ps, dtype="bf16", seed=301)
    _check(w, kernel=kernel)


@pytest.mark.parametrize("kernel", [GENERIC, MFMA])
@pytest.mark.parametrize("shape", [
    dict(T=1, Hq=4, Hkv=4),          # single node: decode attention, one row per KV head
    dict(T=3, Hq=8, Hkv=1),          # chain of three, 24 rows
    dict(T=8, Hq=8, Hkv=1),          # 64 rows
    dict(T=12, Hq=10, Hkv=2),        # 60 rows, ragged row block
    dict(T=64, Hq=8, Hkv=2),         # 256 rows
    dict(T=64, Hq=12, Hkv=1),        # 768 rows: three row groups
    dict(T=33, Hq=7, Hkv=1),         # 231 rows
])
def test_bf16_row_shapes(kernel, shape):
    rng = np.random.default_rng(shape["T"])
    T = shape["T"]
    B = 2
    trees = np.stack([W.random_tree(T, 6, rng) for _ in range(B)])
    w = W.make_workload("rows", B=B, T=T, D=128, seq_lens=[150, 333], trees=trees, page_size=32, dtype="bf16",
                        seed=400 + T, **{k: v for k, v in shape.items() if k != "T"})
    _check(w, "rows %r kernel=%d" % (shape, kernel), kernel=kernel)


@pytest.mark.parametrize("shape", [
    dict(T=1, Hq=4, Hkv=1),          # 4 rows: one wave computes, seven only move tiles
    dict(T=3, Hq=8, Hkv=1),          # 24 rows
    dict(T=12, Hq=10, Hkv=2),        # 60 rows: two waves, the second ragged
    dict(T=12, Hq=8, Hkv=1),         # 96 rows
    dict(T=33, Hq=7, Hkv=1),         # 231 rows: the eighth wave has 7 rows
])
@pytest.mark.parametrize("ps,splits", [(64, 1), (128, 0), (0, 2)])
def test_steady_state_loop_with_idle_waves(shape, ps, splits):
    """Prefixes long enough for the asm steady-state loop, row counts that leave waves without rows."""
    rng = np.random.default_rng(100 + shape["T"])
    T = shape["T"]
    trees = np.stack([W.random_tree(T, 6, rng) for _ in range(2)])
    w = W.make_workload("steady", B=2, T=T, D=128, seq_lens=[1500, 2117], trees=trees, page_size=ps, dtype="bf16",
                        seed=450 + T, paged=ps > 0, **{k: v for k, v in shape.items() if k != "T"})
    _check(w, "steady %r ps=%d splits=%d" % (shape, ps, splits), kernel=MFMA, num_splits=splits)


def test_steady_state_loop_over_two_page_id_spans():
    """One share longer than the page-id cache (2046 pages of 64 tokens): the loop restarts on a second span."""
    T = 16
    w = W.make_workload("two_spans", B=1, T=T, Hq=4, Hkv=1, D=128, seq_lens=[133000], trees=W.bfs_tree(T, [3, 2], 5),
                        page_size=64, dtype="bf16", seed=460)
    _check(w, kernel=MFMA, num_splits=1)


@pytest.mark.parametrize("kernel", [GENERIC, MFMA])
def test_contiguous_layout_and_chain_tree(kernel):
    w = W.make_workload("contig", B=3, T=24, Hq=4, Hkv=2, D=128, seq_lens=[90, 0, 301], trees=W.chain_tree(24),
                        page_size=0, dtype="bf16", seed=501, paged=False)
    _check(w, kernel=kernel)


@pytest.mark.parametrize("ps,L,splits", [(8, 20000, 1), (1, 700, 1), (2, 2500, 2), (4, 5000, 1), (16, 9000, 3),
                                          (256, 3000, 0)])
def test_256_row_kernel_page_sizes_and_long_shares(ps, L, splits):
    """256 rows take the pipelined kernel: tiny pages, shares longer than one page-id span, several spans."""
    rng = np.random.default_rng(ps)
    T = 32
    w = W.make_workload("pp_ps%d" % ps, B=2, T=T, Hq=8, Hkv=1, D=128, seq_lens=[L, L // 3 + 5],
                        trees=np.stack([W.random_tree(T, 6, rng), W.chain_tree(T)]), page_size=ps, dtype="bf16",
                        seed=1300 + ps)
    _check(w, "ps=%d L=%d splits=%d" % (ps, L, splits), kernel=MFMA, num_splits=splits)


def test_256_row_kernel_contiguous_layout():
    rng = np.random.default_rng(13)
    T = 64
    w = W.make_workload("pp_contig", B=2, T=T, Hq=4, Hkv=1, D=128, seq_lens=[1000, 63],
                        trees=np.stack([W.random_deep_tree(T, 10, rng), W.bfs_tree(T, [4, 2], 8)]), page_size=0,
                        dtype="bf16", seed=1400, paged=False)
    _check(w, kernel=MFMA)
    _check(w, "pp contiguous one share", kernel=MFMA, num_splits=1)


@pytest.mark.parametrize("splits", [0, 3])
def test_256_row_groups_on_the_register_staged_kernel(splits):
    """The fallback for 256-row groups (taken by itself when the pipelined kernel's LDS need is too large)."""
    rng = np.random.default_rng(14)
    T = 64
    w = W.make_workload("basic256", B=3, T=T, Hq=8, Hkv=2, D=128, seq_lens=[1500, 0, 777],
                        trees=np.stack([W.random_deep_tree(T, 9, rng), W.chain_tree(T), W.bfs_tree(T, [4, 2], 8)]),
                        page_size=32, dtype="bf16", seed=1500)
    _check(w, "basic splits=%d" % splits, kernel=MFMA_BASIC, num_splits=splits)


@pytest.mark.parametrize("T,Hq,Hkv", [(7, 4, 1), (16, 8, 2), (64, 8, 2), (33, 10, 2)])
def test_head_dim_64_on_the_matrix_cores(T, Hq, Hkv):
    """bf16 with head_dim 64 takes the register-staged matrix-core kernel (28, 64, 256 and 165 rows per KV head)."""
    import torch
    from paper_2508_08192_amd import treeattn as ta
    rng = np.random.default_rng(64 + T)
    for ps, lens in ((64, [0, 1, 65, 777]), (16, [63, 64, 200, 1500]), (0, [130, 5, 0, 64])):
        B = len(lens)
        trees = np.stack([W.random_tree(T, 5, rng) for _ in range(B)])
        w = W.make_workload("d64", B=B, T=T, Hq=Hq, Hkv=Hkv, D=64, seq_lens=lens, trees=trees,
                            page_size=ps if ps else 64, dtype="bf16", seed=6400 + T + ps, paged=ps > 0)
        dev = to_device(w)
        plan = ta.tree_attn_plan(dev["q"], dev["k_cache"], dev["v_cache"], dev["page_table"], dev["seq_lens"],
                                 dev["tree_parent"], dev["out"], dev["lse"])
        assert plan["kernel"] == MFMA
        _check(w, "D=64 T=%d rows=%d ps=%d" % (T, T * Hq // Hkv, ps))
        _check(w, "D=64 T=%d ps=%d, 5 shares" % (T, ps), num_splits=5)
    # window start and a range of query nodes
    w.kv_start = np.int32([64, 3, 0, 10])
    ref, ref_lse = run_oracle(w)
    tq, off = max(1, T // 2), T // 3
    dev = to_device(w)
    dev["q"] = dev["q"][:, off:off + tq].contiguous()
    dev["out"] = torch.empty_like(dev["q"])
    dev["lse"] = torch.empty((w.B, w.Hq, tq), dtype=torch.float32, device="cuda")
    _announce("D=64 window start and query range")
    got, got_lse = run_hip(w, dev, q_node_offset=off)
    assert_parity(got, got_lse, ref[:, off:off + tq], ref_lse[:, :, off:off + tq], "bf16", "D=64 options")


def test_generic_kernel_shapes_the_matrix_core_path_does_not_take():
    rng = np.random.default_rng(6)
    for D, ps, dtype in [(64, 48, "bf16"), (80, 48, "bf16"), (256, 8, "bf16"), (128, 48, "bf16"), (128, 16, "f32"),
                         (96, 10, "f32")]:
        T = 9
        w = W.make_workload("gen", B=2, T=T, Hq=6, Hkv=3, D=D, seq_lens=[70, 129], trees=W.random_tree(T, 4, rng),
                            page_size=ps, dtype=dtype, seed=600 + D)
        _check(w, "D=%d ps=%d %s" % (D, ps, dtype))


@pytest.mark.parametrize("kernel", [GENERIC, MFMA])
def test_result_does_not_depend_on_the_split(kernel):
    rng = np.random.default_rng(7)
    T = 16
    trees = np.stack([W.random_tree(T, 5, rng) for _ in range(4)])
    w = W.make_workload("splits", B=4, T=T, Hq=8, Hkv=2, D=128, seq_lens=[500, 64, 1030, 3], trees=trees,
                        page_size=64, dtype="bf16", seed=701)
    ref, ref_lse = run_oracle(w)
    dev = to_device(w)
    for n in (1, 2, 3, 7, 64, 0):
        _announce("num_splits=%d kernel=%d" % (n, kernel))
        got, got_lse = run_hip(w, dev, kernel=kernel, num_splits=n)
        assert_parity(got, got_lse, ref, ref_lse, "bf16", "num_splits=%d" % n)


@pytest.mark.parametrize("kernel", [GENERIC, MFMA, MFMA_BASIC])
def test_result_does_not_depend_on_the_per_list_cost_of_the_schedule(kernel):
    """Shares are cut over tiles plus a fixed number of units per list; shares that end inside a list's padding,
    lists shorter than the padding and shares longer than several lists all have to give the same result."""
    rng = np.random.default_rng(17)
    T = 12
    trees = np.stack([W.random_tree(T, 4, rng) for _ in range(6)])
    w = W.make_workload("item_cost", B=6, T=T, Hq=8, Hkv=2, D=128, seq_lens=[900, 0, 64, 2100, 5, 130], trees=trees,
                        page_size=64, dtype="bf16", seed=1701)
    ref, ref_lse = run_oracle(w)
    dev = to_device(w)
    for cost, n in [(1, 0), (2, 5), (4, 0), (9, 7), (9, 0), (40, 3), (40, 0), (300, 11), (4096, 0)]:
        _announce("item_cost=%d num_splits=%d kernel=%d" % (cost, n, kernel))
        got, got_lse = run_hip(w, dev, kernel=kernel, num_splits=n, item_cost=cost)
        assert_parity(got, got_lse, ref, ref_lse, "bf16", "item_cost=%d num_splits=%d" % (cost, n))


@pytest.mark.parametrize("kernel", [GENERIC, MFMA])
def test_non_topological_node_numbering_and_forest(kernel):
    rng = np.random.default_rng(8)
    T = 20
    base = W.random_tree(T, 6, rng)
    base[5] = -1                                   # a second root
    shuffled, _ = W.shuffle_tree(base, rng)
    w = W.make_workload("shuffled", B=2, T=T, Hq=4, Hkv=2, D=128, seq_lens=[100, 7], trees=np.stack([base, shuffled]),
                        page_size=16, dtype="bf16", seed=801)
    _check(w, kernel=kernel)


@pytest.mark.parametrize("kernel", [GENERIC, MFMA])
def test_mask_dominated_cases_short_prefix(kernel):
    """With L in {0,1,2} the tree tokens carry almost all the weight: a wrong ancestor mask cannot hide."""
    rng = np.random.default_rng(9)
    T = 64
    trees = np.stack([W.bfs_tree(T, [4], 6), W.random_deep_tree(T, 12, rng), W.chain_tree(T)])
    w = W.make_workload("maskdom", B=3, T=T, Hq=4, Hkv=1, D=128, seq_lens=[0, 1, 2], trees=trees, page_size=128,
                        dtype="bf16", seed=901)
    _check(w, kernel=kernel)


@pytest.mark.parametrize("kernel", [GENERIC, MFMA])
def test_nan_in_unowned_slots_does_not_leak(kernel):
    rng = np.random.default_rng(10)
    T = 8
    w = W.make_workload("nanjunk", B=2, T=T, Hq=8, Hkv=2, D=128, seq_lens=[70, 120], trees=W.random_tree(T, 4, rng),
                        page_size=64, dtype="bf16", seed=1001, garbage=float("nan"))
    _check(w, kernel=kernel)


def test_smallest_configuration_against_the_stored_oracle_outputs():
    """C1 (fp32) against tests/golden/c1_tiny_fp32_oracle.txt, which the oracle wrote and no GPU code ever touched."""
    from .test_oracle_pins import _read_c1_fixture
    w = W.make_config(0)
    ref, ref_lse = _read_c1_fixture()
    _announce("c1 against the stored oracle outputs")
    got, got_lse = run_hip(w)
    assert_parity(got, got_lse, ref, ref_lse, "f32", "c1 stored outputs")


@pytest.mark.parametrize("idx,div", [(1, 1), (2, 8), (3, 16), (4, 64)])
def test_benchmark_configs_reduced_lengths_all_outputs(idx, div):
    w = W.make_config(idx, length_div=div)
    _check(w)


@pytest.mark.parametrize("idx,div", [(0, 16), (1, 32), (2, 64), (3, 16), (4, 16), (5, 1), (6, 1)])
def test_production_shapes_reduced_lengths_all_outputs(idx, div):
    """Small static trees on one GPU's share of the heads (8 and 12 nodes, a chain of 3 behind the root; 5 or 8 query
    heads per KV head): every output against the oracle at reduced prefix lengths (the two batch-size-one shapes at
    full length)."""
    w = W.make_production(idx, length_div=div)
    _check(w)


@pytest.mark.parametrize("idx", [0, 1, 2, 3, 4])
def test_full_size_production_shapes_sampled_outputs(idx):
    """The deployment-like shapes at full size, in the launch configuration the bench times: sampled (request, node,
    head) outputs against the oracle, plus whole-output sanity."""
    import oracle
    w = W.make_production(idx)
    _announce(w.name)
    got, got_lse = run_hip(w)
    rng = np.random.default_rng(200 + idx)
    n = 200
    tri = np.stack([rng.integers(0, w.B, n), rng.integers(0, w.T, n), rng.integers(0, w.Hq, n)], axis=1)
    tri[:min(n, w.B), 0] = np.arange(min(n, w.B))      # (nearly) every request at least once
    ref, ref_lse = oracle.tree_attn_oracle_sample(w.q, w.k_cache, w.v_cache, w.page_table, w.seq_lens,
                                                  w.tree_parent, tri, scale=w.scale, kv_start=w.kv_start)
    g = got[tri[:, 0], tri[:, 1], tri[:, 2]]
    gl = got_lse[tri[:, 0], tri[:, 2], tri[:, 1]]
    assert_parity(g, gl, ref, ref_lse, "bf16", w.name)
    assert np.isfinite(got).all() and np.isfinite(got_lse).all()


@pytest.mark.parametrize("idx", [2, 3, 4])
def test_full_size_configs_all_outputs(idx):
    """The benchmark configurations at full size, in the launch configuration the bench times: every output and every
    log-sum-exp against the oracle (which needs seconds to a minute for these), plus whole-output sanity."""
    w = W.make_config(idx)
    _announce(w.name)
    got, got_lse = run_hip(w)
    ref, ref_lse = run_oracle(w)
    assert_parity(got, got_lse, ref, ref_lse, "bf16", w.name)
    # per request as well: the relative gate of a short request must not hide behind the scale of another
    for b in range(w.B):
        assert_parity(got[b], got_lse[b], ref[b], ref_lse[b], "bf16", "%s request %d" % (w.name, b))
    from .helpers import widen
    assert np.abs(got).max() <= np.abs(widen(w.v_cache[w.page_table[0, :4]])).max() * 4


def test_strided_views_token_major_cache():
    rng = np.random.default_rng(11)
    import torch
    T = 16
    _strided_case(W.make_workload("tokmajor", B=2, T=T, Hq=8, Hkv=2, D=128, seq_lens=[130, 64],
                                  trees=W.random_tree(T, 5, rng), page_size=32, dtype="bf16", seed=1101))
    T = 64                                             # 256 rows: the pipelined kernel
    _strided_case(W.make_workload("tokmajor256", B=2, T=T, Hq=8, Hkv=2, D=128, seq_lens=[700, 64],
                                  trees=W.random_tree(T, 7, rng), page_size=32, dtype="bf16", seed=1102))


def _strided_case(w):
    import torch
    T = w.T
    ref, ref_lse = run_oracle(w)
    dev = to_device(w)
    for key in ("k_cache", "v_cache"):
        dev[key] = dev[key].permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)    # [pages, ps, Hkv, D] storage
        assert not dev[key].is_contiguous()
    q_wide = torch.zeros((2, T, 8, 256), dtype=torch.bfloat16, device="cuda:0")      # q as a slice of a wider buffer
    q_wide[..., :128] = dev["q"]
    dev["q"] = q_wide[..., :128]
    for kernel in (GENERIC, MFMA):
        _announce("strided kernel=%d" % kernel)
        got, got_lse = run_hip(w, dev, kernel=kernel)
        assert_parity(got, got_lse, ref, ref_lse, "bf16", "strided kernel=%d" % kernel)


def test_merge_pass_variants():
    """More partial results than half a wave holds, an odd number of rows, and an output view whose rows are not
    16-byte aligned (which takes the general merge kernel) all have to agree with the oracle."""
    import torch
    rng = np.random.default_rng(23)
    T = 5
    w = W.make_workload("merge", B=2, T=T, Hq=3, Hkv=1, D=128, seq_lens=[4000, 90], trees=W.random_tree(T, 3, rng),
                        page_size=64, dtype="bf16", seed=2301)                      # 15 rows
    ref, ref_lse = run_oracle(w)
    dev = to_device(w)
    for kernel, n, cost in [(MFMA, 64, 1), (GENERIC, 64, 1), (MFMA, 0, 0), (MFMA, 7, 3)]:
        _announce("merge kernel=%d num_splits=%d item_cost=%d" % (kernel, n, cost))
        got, got_lse = run_hip(w, dev, kernel=kernel, num_splits=n, item_cost=cost)
        assert_parity(got, got_lse, ref, ref_lse, "bf16", "merge num_splits=%d" % n)
    wide = torch.zeros((2, T, 3, 130), dtype=torch.bfloat16, device="cuda:0")
    dev["out"] = wide[..., 1:129]                                                  # rows start 2 bytes off
    _announce("merge into an unaligned output view")
    got, got_lse = run_hip(w, dev, kernel=MFMA, num_splits=64, item_cost=1)
    assert_parity(got, got_lse, ref, ref_lse, "bf16", "unaligned out")
    wf = W.make_workload("merge32", B=1, T=T, Hq=3, Hkv=1, D=128, seq_lens=[3000], trees=W.random_tree(T, 3, rng),
                         page_size=64, dtype="f32", seed=2302)
    _check(wf, "merge fp32 many partials", num_splits=48, item_cost=1)


@pytest.mark.parametrize("idx,div", [(2, 16), (3, 16), (1, 1)])
def test_repeat_calls_are_bit_identical(idx, div):
    w = W.make_config(idx, length_div=div)
    dev = to_device(w)
    a, al = run_hip(w, dev)
    for _ in range(6):
        b, bl = run_hip(w, dev)
        assert np.array_equal(a, b) and np.array_equal(al, bl)


@pytest.mark.parametrize("kernel", [GENERIC, MFMA])
def test_malformed_requests_get_nan_and_a_status_bit(kernel):
    from paper_2508_08192_amd import treeattn as ta
    T = 8
    trees = np.int32([[-1, 0, 1, 2, 3, 4, 5, 6], [-1, 0, 3, 2, 0, 0, 0, 0], [-1, 0, 9, 1, 1, 1, 1, 1],
                      [-1, 0, 0, 0, 1, 1, 2, 2]])
    w = W.make_workload("bad", B=4, T=T, Hq=4, Hkv=2, D=128, seq_lens=[40, 40, 40, 40], trees=trees, page_size=16,
                        dtype="bf16", seed=1201)
    ta.tree_attn_last_status()
    ref, ref_lse = run_oracle(w)
    got, got_lse = run_hip(w, kernel=kernel)
    assert ta.tree_attn_last_status() == ta.TA_STATUS_BAD_PARENT
    assert np.isnan(got[1]).all() and np.isnan(got[2]).all() and np.isnan(got_lse[1]).all()
    assert_parity(got[[0, 3]], got_lse[[0, 3]], ref[[0, 3]], ref_lse[[0, 3]], "bf16", "healthy requests")
    w.seq_lens[0] = -3
    w.seq_lens[3] = w.page_table.shape[1] * 16 - T + 1
    w.tree_parent[1] = trees[0]
    w.tree_parent[2] = trees[0]
    ref, ref_lse = run_oracle(w)
    got, got_lse = run_hip(w, kernel=kernel)
    assert ta.tree_attn_last_status() == ta.TA_STATUS_BAD_SEQLEN
    assert np.isnan(got[0]).all() and np.isnan(got[3]).all()
    assert_parity(got[[1, 2]], got_lse[[1, 2]], ref[[1, 2]], ref_lse[[1, 2]], "bf16", "healthy requests")
    assert ta.tree_attn_last_status() == 0


def test_encoder_masks():
    import torch
    from paper_2508_08192_amd import treeattn as ta
    from .helpers import ancestors_inclusive
    rng = np.random.default_rng(12)
    T = 64
    trees = np.stack([W.random_tree(T, 9, rng), W.chain_tree(T), W.shuffle_tree(W.bfs_tree(T, [4, 2], 8), rng)[0]])
    par = torch.from_numpy(trees).cuda()
    masks = torch.zeros((3, T), dtype=torch.int64, device="cuda")
    ta.tree_attn_encode(par, masks)
    torch.cuda.synchronize()
    got = masks.cpu().numpy().view(np.uint64)
    for b in range(3):
        for i in range(T):
            want = 0
            for j in ancestors_inclusive(trees[b], i):
                want |= 1 << j
            assert int(got[b, i]) == want
    one = torch.zeros((T,), dtype=torch.int64, device="cuda")
    ta.tree_attn_encode(par[1], one)
    torch.cuda.synchronize()
    assert np.array_equal(one.cpu().numpy().view(np.uint64), got[1])


@pytest.mark.parametrize("kernel", [GENERIC, MFMA, MFMA_BASIC])
def test_masks_encoded_once_replace_the_walk_over_parents(kernel):
    """Static trees: tree_attn_encode runs once, later calls take its masks (ta_opts.tree_masks).  The parents passed
    along are deliberately different trees (all roots), so the call only agrees with the oracle if it reads the masks."""
    import torch
    from paper_2508_08192_amd import treeattn as ta
    rng = np.random.default_rng(31)
    T = 24
    trees = np.stack([W.random_tree(T, 6, rng) for _ in range(3)])
    w = W.make_workload("masks", B=3, T=T, Hq=8, Hkv=2, D=128, seq_lens=[700, 0, 130], trees=trees, page_size=64,
                        dtype="bf16", seed=3101)
    ref, ref_lse = run_oracle(w)
    dev = to_device(w)
    masks = torch.zeros((3, T), dtype=torch.int64, device="cuda")
    ta.tree_attn_encode(dev["tree_parent"], masks)
    masks |= (-1 << T)                                             # bits of nodes that do not exist are ignored
    dev["tree_parent"] = torch.full_like(dev["tree_parent"], -1)
    _announce("given masks, kernel=%d" % kernel)
    got, got_lse = run_hip(w, dev, kernel=kernel, tree_masks=masks)
    assert_parity(got, got_lse, ref, ref_lse, "bf16", "given masks")
    # one tree for the whole batch: masks [T], stride 0
    w1 = W.make_workload("masks1", B=3, T=T, Hq=8, Hkv=2, D=128, seq_lens=[64, 333, 1000], trees=trees[2], page_size=64,
                         dtype="bf16", seed=3102)
    ref, ref_lse = run_oracle(w1)
    dev = to_device(w1)
    one = torch.zeros((T,), dtype=torch.int64, device="cuda")
    ta.tree_attn_encode(torch.from_numpy(trees[2]).cuda(), one)
    dev["tree_parent"] = torch.full_like(dev["tree_parent"], -1)
    _announce("one mask set for the batch, kernel=%d" % kernel)
    got, got_lse = run_hip(w1, dev, kernel=kernel, tree_masks=one, num_splits=5)
    assert_parity(got, got_lse, ref, ref_lse, "bf16", "given masks, shared tree")


@pytest.mark.parametrize("kernel", [GENERIC, MFMA, MFMA_BASIC])
@pytest.mark.parametrize("T,Hq,Hkv", [(8, 8, 2), (64, 8, 2)])
def test_window_start_restricts_the_prefix(kernel, T, Hq, Hkv):
    """ta_opts.kv_start: windows that begin on and off tile and page edges, an empty window, one that leaves a
    single token, and long ones that run through the steady-state loop."""
    import torch
    rng = np.random.default_rng(41)
    lens = [700, 64, 130, 0, 1500, 9000, 9000, 3000, 65]
    start = [0, 64, 70, 0, 1000, 8192, 3001, 2999, 1]
    B = len(lens)
    trees = np.stack([W.random_tree(T, 5, rng) for _ in range(B)])
    w = W.make_workload("window", B=B, T=T, Hq=Hq, Hkv=Hkv, D=128, seq_lens=lens, trees=trees, page_size=64,
                        dtype="bf16", seed=4100 + T)
    ks = np.asarray(start, dtype=np.int32)
    ref, ref_lse = run_oracle(w, kv_start=ks)
    dev = to_device(w)
    dks = torch.from_numpy(ks).cuda()
    for n in (0, 3):
        _announce("kv_start kernel=%d T=%d num_splits=%d" % (kernel, T, n))
        got, got_lse = run_hip(w, dev, kernel=kernel, kv_start=dks, num_splits=n)
        assert_parity(got, got_lse, ref, ref_lse, "bf16", "kv_start num_splits=%d" % n)


@pytest.mark.parametrize("ps", [0, 8, 256])
def test_window_start_other_layouts(ps):
    """The window start with the contiguous cache, with pages smaller than a tile (several page-id spans) and with
    pages larger than one."""
    import torch
    rng = np.random.default_rng(43)
    T = 16
    lens = [20000, 777, 4100]
    start = [18000 if ps != 8 else 1000, 700, 4096]
    trees = np.stack([W.random_tree(T, 5, rng) for _ in range(3)])
    w = W.make_workload("window_ps%d" % ps, B=3, T=T, Hq=16, Hkv=1, D=128, seq_lens=lens, trees=trees, page_size=ps,
                        dtype="bf16", seed=4300 + ps, paged=ps > 0)
    w.kv_start = np.asarray(start, dtype=np.int32)
    _check(w, "window ps=%d one share" % ps, kernel=MFMA, num_splits=1)
    _check(w, "window ps=%d" % ps, kernel=MFMA)


def test_window_start_out_of_range_poisons_the_request():
    import torch
    from paper_2508_08192_amd import treeattn as ta
    rng = np.random.default_rng(42)
    T = 8
    w = W.make_workload("window_bad", B=3, T=T, Hq=4, Hkv=1, D=128, seq_lens=[100, 200, 300],
                        trees=W.random_tree(T, 3, rng), page_size=64, dtype="bf16", seed=4201)
    ks = np.asarray([101, 5, -1], dtype=np.int32)
    ref, ref_lse = run_oracle(w, kv_start=ks)
    ta.tree_attn_last_status()
    got, got_lse = run_hip(w, kernel=MFMA, kv_start=torch.from_numpy(ks).cuda())
    assert np.isnan(got[0]).all() and np.isnan(got[2]).all() and np.isnan(got_lse[0]).all()
    assert np.isnan(ref[0]).all() and np.isnan(ref[2]).all()
    assert np.abs(got[1] - ref[1]).max() <= 1e-2
    assert ta.tree_attn_last_status() & ta.TA_STATUS_BAD_SEQLEN


@pytest.mark.parametrize("dtype,ps", [("bf16", 64), ("bf16", 0), ("f32", 16)])
def test_write_back_of_tree_keys_and_values(dtype, ps):
    """tree_attn_append puts k_new/v_new at positions L_b .. L_b+T-1, bit for bit, and touches nothing else; the
    attention over the cache it completed agrees with the oracle."""
    import torch
    from paper_2508_08192_amd import treeattn as ta
    rng = np.random.default_rng(51)
    T, Hkv, D = 9, 2, 128 if dtype == "bf16" else 64
    w = W.make_workload("append", B=3, T=T, Hq=4, Hkv=Hkv, D=D, seq_lens=[130, 0, 63], trees=W.random_tree(T, 4, rng),
                        page_size=ps, dtype=dtype, seed=5100 + ps, paged=ps > 0)
    ref, ref_lse = run_oracle(w)
    dev = to_device(w)
    # pull the tree tokens out of the cache into dense tensors, then wipe them in the cache
    k_new = torch.empty((w.B, T, Hkv, D), dtype=dev["k_cache"].dtype, device="cuda")
    v_new = torch.empty_like(k_new)
    kc, vc = dev["k_cache"].clone(), dev["v_cache"].clone()
    for b in range(w.B):
        for i in range(T):
            pos = int(w.seq_lens[b]) + i
            page, slot = (b, pos) if w.page_table is None else (int(w.page_table[b, pos // ps]), pos % ps)
            k_new[b, i] = kc[page, :, slot, :]
            v_new[b, i] = vc[page, :, slot, :]
            dev["k_cache"][page, :, slot, :] = 7.0
            dev["v_cache"][page, :, slot, :] = 7.0
    _announce("append %s ps=%d" % (dtype, ps))
    ta.tree_attn_append(k_new, v_new, dev["k_cache"], dev["v_cache"], dev["page_table"], dev["seq_lens"])
    torch.cuda.synchronize()
    assert torch.equal(dev["k_cache"].view(torch.int16 if dtype == "bf16" else torch.int32),
                       kc.view(torch.int16 if dtype == "bf16" else torch.int32))
    assert torch.equal(dev["v_cache"].view(torch.int16 if dtype == "bf16" else torch.int32),
                       vc.view(torch.int16 if dtype == "bf16" else torch.int32))
    got, got_lse = run_hip(w, dev)
    assert_parity(got, got_lse, ref, ref_lse, dtype, "after write-back")


@pytest.mark.parametrize("dtype,ps,D,Hkv,T", [("bf16", 64, 128, 8, 12), ("bf16", 0, 128, 2, 9), ("f32", 4, 64, 3, 16),
                                              ("f32", 16, 256, 2, 64)])
def test_bookkeeping_moves_the_accepted_path_behind_the_prefix(dtype, ps, D, Hkv, T):
    """tree_attn_compact against the bookkeeping oracle, bit for bit over the whole cache (so nothing else may change),
    with lengths updated in place; then plain decoding over the rewound cache agrees with the attention oracle.
    Covers pages smaller than the path, the contiguous layout, sources that are also destinations, a unit larger
    than one staging phase (T 64, D 256, fp32), zero accepted nodes and the requests that must be left alone."""
    import torch
    from oracle import kv_compact_oracle as KC
    from paper_2508_08192_amd import treeattn as ta
    rng = np.random.default_rng(81)
    B = 6
    tree = W.shuffle_tree(W.random_deep_tree(T, min(T, 7), rng), rng)[0]
    lens = [130, 0, 63, 17, 5, 40]
    w = W.make_workload("compact", B=B, T=T, Hq=Hkv * 2, Hkv=Hkv, D=D, seq_lens=lens, trees=tree, page_size=ps if ps else 64,
                        dtype=dtype, seed=8100 + ps, paged=ps > 0)
    A = T
    acc = np.full((B, A), -3, dtype=np.int32)
    n = np.zeros(B, dtype=np.int32)
    paths = [max((ancestors_inclusive(tree, i) for i in range(T)), key=len)]
    paths.append(list(rng.permutation(T)[:A]))                     # not a path at all: a permutation, sources = destinations
    paths.append([])                                               # nothing accepted
    paths.append(paths[0][:2])
    paths.append([0, T])                                           # id out of range: left alone
    paths.append(paths[0])
    for b, p in enumerate(paths):
        acc[b, :len(p)] = p
        n[b] = len(p)
    n[5] = A + 1                                                   # accepted length beyond the list: left alone
    k_ref, v_ref, lens_ref, skipped = KC.kv_compact_oracle(w.k_cache, w.v_cache, w.page_table, w.seq_lens, acc, n, T)
    assert skipped == [4, 5]
    dev = to_device(w)
    _announce("compact %s ps=%d D=%d Hkv=%d T=%d" % (dtype, ps, D, Hkv, T))
    ta.tree_attn_last_status()
    ta.tree_attn_compact(dev["k_cache"], dev["v_cache"], dev["page_table"], dev["seq_lens"],
                         torch.from_numpy(acc).cuda(), torch.from_numpy(n).cuda(), T, seq_lens_out=dev["seq_lens"])
    torch.cuda.synchronize()
    bits = torch.int16 if dtype == "bf16" else torch.int32
    assert np.array_equal(dev["k_cache"].view(bits).cpu().numpy(), k_ref.view(np.int16 if dtype == "bf16" else np.int32))
    assert np.array_equal(dev["v_cache"].view(bits).cpu().numpy(), v_ref.view(np.int16 if dtype == "bf16" else np.int32))
    assert np.array_equal(dev["seq_lens"].cpu().numpy(), lens_ref)
    assert ta.tree_attn_last_status() == ta.TA_STATUS_BAD_PATH
    # the next step's attention over the rewound cache: the last accepted token is the single tree node
    keep = [0, 3]
    w1 = W.Workload(name="after", dtype=dtype, q=np.stack([w.q[b, paths[b][-1]] for b in keep])[:, None],
                    k_cache=k_ref if w.page_table is not None else k_ref[keep],
                    v_cache=v_ref if w.page_table is not None else v_ref[keep],
                    page_table=None if w.page_table is None else w.page_table[keep],
                    seq_lens=np.int32([lens_ref[b] - 1 for b in keep]), tree_parent=np.int32([-1]), scale=w.scale)
    ref, ref_lse = run_oracle(w1)
    full, full_lse = run_oracle(w)
    for r, b in enumerate(keep):                                    # (the pin of the oracle, repeated on this input)
        np.testing.assert_allclose(ref[r, 0], full[b, paths[b][-1]], rtol=0, atol=1e-12)
    got, got_lse = run_hip(w1)
    assert_parity(got, got_lse, ref, ref_lse, dtype, "decode after bookkeeping")


def test_bookkeeping_reports_a_prefix_without_room_and_writes_a_separate_length_array():
    import torch
    from oracle import kv_compact_oracle as KC
    from paper_2508_08192_amd import treeattn as ta
    T = 8
    w = W.make_workload("compact2", B=3, T=T, Hq=4, Hkv=2, D=128, seq_lens=[20, 9, 33], trees=W.chain_tree(T),
                        page_size=16, dtype="bf16", seed=8200)
    w.seq_lens[1] = w.page_table.shape[1] * 16 - T + 1             # the tree would not fit: left alone
    acc = np.int32([[0, 1, 2], [0, 1, 2], [0, 1, 2]])
    n = np.int32([3, 3, 1])
    k_ref, v_ref, lens_ref, skipped = KC.kv_compact_oracle(w.k_cache, w.v_cache, w.page_table, w.seq_lens, acc, n, T)
    assert skipped == [1]
    dev = to_device(w)
    new_lens = torch.full((3, 2), -1, dtype=torch.int32, device="cuda")
    _announce("compact: separate strided length array")
    ta.tree_attn_last_status()
    ta.tree_attn_compact(dev["k_cache"], dev["v_cache"], dev["page_table"], dev["seq_lens"],
                         torch.from_numpy(acc).cuda(), torch.from_numpy(n).cuda(), T, seq_lens_out=new_lens[:, 0])
    torch.cuda.synchronize()
    assert np.array_equal(dev["k_cache"].view(torch.int16).cpu().numpy(), k_ref.view(np.int16))
    assert np.array_equal(dev["v_cache"].view(torch.int16).cpu().numpy(), v_ref.view(np.int16))
    assert np.array_equal(new_lens[:, 0].cpu().numpy(), lens_ref) and (new_lens[:, 1] == -1).all()
    assert np.array_equal(dev["seq_lens"].cpu().numpy(), w.seq_lens)
    assert ta.tree_attn_last_status() == ta.TA_STATUS_BAD_SEQLEN


@pytest.mark.parametrize("kernel,dtype,ps,T", [(MFMA, "bf16", 64, 9), (MFMA, "bf16", 0, 64), (MFMA_BASIC, "bf16", 16, 33),
                                                (GENERIC, "bf16", 128, 12), (GENERIC, "f32", 16, 7), (MFMA, "bf16", 16, 64)])
def test_write_back_folded_into_the_call(kernel, dtype, ps, T):
    """ta_opts.k_new / v_new: the call takes the tree tokens' K/V from the dense tensors and stores them behind the
    prefix itself.  Its out and lse are bit for bit those of tree_attn_append followed by the plain call, the caches
    end up bit for bit the same, the oracle agrees, and a request with a bad length is neither computed nor written."""
    import torch
    from paper_2508_08192_amd import treeattn as ta
    rng = np.random.default_rng(52)
    Hkv, D = 2, 128 if dtype == "bf16" else 64
    lens = [130, 0, 63, 900]
    w = W.make_workload("fused", B=4, T=T, Hq=8, Hkv=Hkv, D=D, seq_lens=lens, trees=W.random_tree(T, 5, rng),
                        page_size=ps if ps else 64, dtype=dtype, seed=5200 + ps + T, paged=ps > 0)
    ref, ref_lse = run_oracle(w)
    dev = to_device(w)
    bits = torch.int16 if dtype == "bf16" else torch.int32
    k_new = torch.empty((w.B, T, Hkv, D), dtype=dev["k_cache"].dtype, device="cuda")
    v_new = torch.empty_like(k_new)
    full_k, full_v = dev["k_cache"].clone(), dev["v_cache"].clone()
    for b in range(w.B):                                           # tree tokens out of the cache, garbage in their place
        for i in range(T):
            pos = int(w.seq_lens[b]) + i
            page, slot = (b, pos) if w.page_table is None else (int(w.page_table[b, pos // ps]), pos % ps)
            k_new[b, i] = full_k[page, :, slot, :]
            v_new[b, i] = full_v[page, :, slot, :]
            dev["k_cache"][page, :, slot, :] = 7.0
            dev["v_cache"][page, :, slot, :] = 7.0
    wiped_k, wiped_v = dev["k_cache"].clone(), dev["v_cache"].clone()
    _announce("folded write-back kernel=%d %s ps=%d T=%d" % (kernel, dtype, ps, T))
    got, got_lse = run_hip(w, dev, kernel=kernel, k_new=k_new, v_new=v_new)
    assert_parity(got, got_lse, ref, ref_lse, dtype, "folded write-back")
    assert torch.equal(dev["k_cache"].view(bits), full_k.view(bits))
    assert torch.equal(dev["v_cache"].view(bits), full_v.view(bits))
    out_fused, lse_fused = dev["out"].clone(), dev["lse"].clone()
    # the two-call form on the wiped cache
    dev["k_cache"].copy_(wiped_k)
    dev["v_cache"].copy_(wiped_v)
    ta.tree_attn_append(k_new, v_new, dev["k_cache"], dev["v_cache"], dev["page_table"], dev["seq_lens"])
    run_hip(w, dev, kernel=kernel)
    assert torch.equal(dev["out"].view(bits), out_fused.view(bits)) and torch.equal(dev["lse"], lse_fused)
    # strided views of larger tensors serve as well; a request with a bad length is left alone
    big_k = torch.zeros((w.B, T + 3, Hkv + 1, D + 8), dtype=k_new.dtype, device="cuda")
    big_v = torch.zeros_like(big_k)
    big_k[:, 1:T + 1, 1:, :D] = k_new
    big_v[:, 1:T + 1, 1:, :D] = v_new
    dev["k_cache"].copy_(wiped_k)
    dev["v_cache"].copy_(wiped_v)
    dev["seq_lens"][2] = -1
    ta.tree_attn_last_status()
    got, got_lse = run_hip(w, dev, kernel=kernel, k_new=big_k[:, 1:T + 1, 1:, :D], v_new=big_v[:, 1:T + 1, 1:, :D])
    assert ta.tree_attn_last_status() & ta.TA_STATUS_BAD_SEQLEN
    keep = [0, 1, 3]                    # (the shares are cut differently now, so only the tolerance holds, not the bits)
    assert_parity(got[keep], got_lse[keep], ref[keep], ref_lse[keep], dtype, "beside a request with a bad length")
    assert np.isnan(got[2]).all() and np.isnan(got_lse[2]).all()
    exp_k, exp_v = full_k.clone(), full_v.clone()
    for i in range(T):                                             # request 2's tree positions keep the garbage
        pos = int(w.seq_lens[2]) + i
        page, slot = (2, pos) if w.page_table is None else (int(w.page_table[2, pos // ps]), pos % ps)
        exp_k[page, :, slot, :] = 7.0
        exp_v[page, :, slot, :] = 7.0
    assert torch.equal(dev["k_cache"].view(bits), exp_k.view(bits)) and torch.equal(dev["v_cache"].view(bits), exp_v.view(bits))
    if kernel == GENERIC:
        # rows that are not 16-byte aligned: element-wise copy, scalar kernel only
        odd_k = torch.zeros((w.B, T, Hkv, D + 3), dtype=k_new.dtype, device="cuda")
        odd_v = torch.zeros_like(odd_k)
        odd_k[..., 1:D + 1] = k_new
        odd_v[..., 1:D + 1] = v_new
        dev["k_cache"].copy_(wiped_k)
        dev["v_cache"].copy_(wiped_v)
        dev["seq_lens"][2] = int(w.seq_lens[2])
        run_hip(w, dev, kernel=kernel, k_new=odd_k[..., 1:D + 1], v_new=odd_v[..., 1:D + 1])
        assert torch.equal(dev["out"].view(bits), out_fused.view(bits))
        assert torch.equal(dev["k_cache"].view(bits), full_k.view(bits)) and torch.equal(dev["v_cache"].view(bits), full_v.view(bits))


@pytest.mark.parametrize("kernel", [GENERIC, MFMA, MFMA_BASIC])
def test_every_option_at_once(kernel):
    """A drafting-stage call on a local-attention layer of a static tree: window start, query range, masks encoded
    earlier, the write-back folded in, a caller workspace, a non-default scale, per-list cost and forced splits, all in
    one call -- against the oracle, and the caches against the plain write-back."""
    import torch
    from paper_2508_08192_amd import treeattn as ta
    rng = np.random.default_rng(131)
    T, off, tq = 21, 5, 8
    tree = W.bfs_tree(T, [4, 2, 1], 4)
    w = W.make_workload("all", B=3, T=T, Hq=8, Hkv=2, D=128, seq_lens=[900, 70, 4100], trees=tree, page_size=32,
                        dtype="bf16", seed=13100, scale=0.11)
    w.kv_start = np.int32([512, 70, 4096])                        # request 1: an empty window, the path alone
    ref, ref_lse = run_oracle(w)
    dev = to_device(w)
    k_new = torch.empty((w.B, T, w.Hkv, w.D), dtype=torch.bfloat16, device="cuda")
    v_new = torch.empty_like(k_new)
    full_k, full_v = dev["k_cache"].clone(), dev["v_cache"].clone()
    for b in range(w.B):
        for i in range(T):
            pos = int(w.seq_lens[b]) + i
            page, slot = int(w.page_table[b, pos // 32]), pos % 32
            k_new[b, i] = full_k[page, :, slot, :]
            v_new[b, i] = full_v[page, :, slot, :]
            dev["k_cache"][page, :, slot, :] = -3.0
            dev["v_cache"][page, :, slot, :] = -3.0
    masks = torch.zeros((T,), dtype=torch.int64, device="cuda")
    ta.tree_attn_encode(torch.from_numpy(tree).cuda(), masks)
    dev["tree_parent"] = torch.full_like(dev["tree_parent"], -1)  # only the masks describe the tree
    dev["q"] = dev["q"][:, off:off + tq].contiguous()
    dev["out"] = torch.empty_like(dev["q"])
    dev["lse"] = torch.empty((w.B, w.Hq, tq), dtype=torch.float32, device="cuda")
    ws = torch.empty(ta.tree_attn_workspace_bytes(w.B, tq, w.Hq, w.Hkv, w.D, ta.TA_BF16), dtype=torch.uint8, device="cuda")
    _announce("every option at once, kernel=%d" % kernel)
    got, got_lse = run_hip(w, dev, kernel=kernel, q_node_offset=off, tree_masks=masks, k_new=k_new, v_new=v_new,
                           workspace=ws, item_cost=3, num_splits=7)
    assert_parity(got, got_lse, ref[:, off:off + tq], ref_lse[:, :, off:off + tq], "bf16", "every option at once")
    assert torch.equal(dev["k_cache"].view(torch.int16), full_k.view(torch.int16))
    assert torch.equal(dev["v_cache"].view(torch.int16), full_v.view(torch.int16))
    assert ta.tree_attn_last_status() == 0


@pytest.mark.parametrize("kernel", [GENERIC, MFMA, MFMA_BASIC])
def test_queries_are_a_range_of_the_tree_nodes(kernel):
    """Drafting stage: the tree grows level by level; the newest nodes are the queries (ta_opts.q_node_offset), every
    node so far is a key.  Each level's outputs are the corresponding rows of the whole-tree result."""
    import torch
    rng = np.random.default_rng(61)
    T = 21
    tree = W.bfs_tree(T, [4, 2, 1], 4)                              # levels of 1, 4, 8, 8 nodes, numbered level by level
    w = W.make_workload("draft", B=3, T=T, Hq=8, Hkv=2, D=128, seq_lens=[900, 0, 131], trees=tree, page_size=64,
                        dtype="bf16", seed=6101)
    ref, ref_lse = run_oracle(w)
    dev = to_device(w)
    q_all = dev["q"]
    for off, tq in [(0, 1), (1, 4), (5, 8), (13, 8), (0, 21), (20, 1)]:
        dev["q"] = q_all[:, off:off + tq].contiguous()
        dev["out"] = torch.empty_like(dev["q"])
        dev["lse"] = torch.empty((w.B, w.Hq, tq), dtype=torch.float32, device="cuda")
        _announce("query nodes %d..%d kernel=%d" % (off, off + tq - 1, kernel))
        got, got_lse = run_hip(w, dev, kernel=kernel, q_node_offset=off)
        assert_parity(got, got_lse, ref[:, off:off + tq], ref_lse[:, :, off:off + tq], "bf16", "nodes from %d" % off)
    # a view into the full q works as well (strided rows)
    dev["q"] = q_all[:, 5:13]
    dev["out"] = torch.empty((w.B, 8, w.Hq, w.D), dtype=q_all.dtype, device="cuda")
    dev["lse"] = torch.empty((w.B, w.Hq, 8), dtype=torch.float32, device="cuda")
    got, got_lse = run_hip(w, dev, kernel=kernel, q_node_offset=5)
    assert_parity(got, got_lse, ref[:, 5:13], ref_lse[:, :, 5:13], "bf16", "q view")


def test_very_large_batch_falls_back_to_the_register_staged_kernel():
    """With more than about 1900 requests the schedule no longer fits beside the tile rings in LDS and the library
    takes the register-staged matrix-core kernel by itself (kernel = MFMA is still what the caller asked for)."""
    rng = np.random.default_rng(71)
    B, T = 2100, 4
    lens = rng.integers(0, 200, size=B)
    w = W.make_workload("big_batch", B=B, T=T, Hq=4, Hkv=1, D=128, seq_lens=lens, trees=W.chain_tree(T), page_size=64,
                        dtype="bf16", seed=7101)
    ks = (lens // 3).astype(np.int32)
    w.kv_start = ks
    _check(w, "B=2100 with window starts", kernel=MFMA)


@pytest.mark.parametrize("kernel", [GENERIC, MFMA, MFMA_BASIC])
@pytest.mark.parametrize("B", [64, 65, 129, 200])
def test_batches_around_multiples_of_a_wave_of_requests(kernel, B):
    """A workgroup finds the request of its first tile by counting, 64 requests at a time, the lists that end before
    it: batches of exactly one wave of requests, one more, and several waves with a ragged last one, with lengths that
    put list ends inside and between the workgroups' shares (some requests have no prefix at all)."""
    rng = np.random.default_rng(1000 + B)
    T = 4
    lens = rng.integers(0, 300, size=B)
    lens[rng.integers(0, B, size=B // 8)] = 0
    w = W.make_workload("waves_of_requests", B=B, T=T, Hq=4, Hkv=2, D=128, seq_lens=lens, trees=W.chain_tree(T),
                        page_size=64, dtype="bf16", seed=8800 + B)
    _check(w, "B=%d kernel=%d" % (B, kernel), kernel=kernel)


def test_empty_batch_and_no_lse():
    import torch
    from paper_2508_08192_amd import treeattn as ta
    w = W.make_config(2, length_div=64)
    dev = to_device(w)
    ref, _ = run_oracle(w)
    dev["out"].fill_(float("nan"))
    ta.tree_attn_fwd(dev["q"], dev["k_cache"], dev["v_cache"], dev["page_table"], dev["seq_lens"], dev["tree_parent"],
                     dev["out"], None)
    torch.cuda.synchronize()
    got = dev["out"].float().cpu().numpy().astype(np.float64)
    assert np.abs(got - ref).max() <= 1e-2
    e = {k: (v[:0] if v is not None and k != "k_cache" and k != "v_cache" else v) for k, v in dev.items()}
    assert ta.tree_attn_fwd(e["q"], e["k_cache"], e["v_cache"], e["page_table"], e["seq_lens"], e["tree_parent"],
                            e["out"], e["lse"]) == 0


def test_side_stream_and_graph_replay_follow_device_side_lengths():
    """The call neither synchronises nor allocates once the workspace is reserved, and every length it needs is read
    on the device: captured in a HIP graph on a side stream, replays must track seq_lens rewritten between them."""
    import torch
    from paper_2508_08192_amd import treeattn as ta
    rng = np.random.default_rng(77)
    T = 32
    trees = np.stack([W.random_tree(T, 6, rng), W.bfs_tree(T, [4, 2], 5)])
    lens = [[900, 2500], [64, 1], [1777, 640]]
    big = W.make_workload("graph_big", B=2, T=T, Hq=8, Hkv=1, D=128, seq_lens=[2500, 2500], trees=trees, page_size=64,
                          dtype="bf16", seed=4242)
    dev = to_device(big)
    ta.tree_attn_reserve(ta.tree_attn_workspace_bytes(big.B, big.T, big.Hq, big.Hkv, big.D, ta.TA_BF16))
    side = torch.cuda.Stream()
    args = (dev["q"], dev["k_cache"], dev["v_cache"], dev["page_table"], dev["seq_lens"], dev["tree_parent"], dev["out"],
            dev["lse"])
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        ta.tree_attn_fwd(*args, stream=side)               # warm-up on the side stream (sets kernel attributes)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        ta.tree_attn_fwd(*args, stream=torch.cuda.current_stream())
    for rep in range(2):
        for L in lens:
            # same caches and page table (capacity 2500 + T each), new prefix lengths: the oracle sees the same thing
            w = W.make_workload("graph_case", B=2, T=T, Hq=8, Hkv=1, D=128, seq_lens=[2500, 2500], trees=trees,
                                page_size=64, dtype="bf16", seed=4242)
            w.seq_lens[:] = np.asarray(L, dtype=w.seq_lens.dtype)
            ref, ref_lse = run_oracle(w)
            dev["seq_lens"].copy_(torch.from_numpy(w.seq_lens))
            dev["out"].fill_(float("nan"))
            dev["lse"].fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            got = dev["out"].float().cpu().numpy().astype(np.float64)
            got_lse = dev["lse"].cpu().numpy().astype(np.float64)
            assert_parity(got, got_lse, ref, ref_lse, "bf16", "graph replay %d L=%r" % (rep, L))


@pytest.mark.parametrize("splits", [0, 100, 300])
def test_one_long_list_cut_over_the_whole_chip(splits):
    """Batch size one (the paper's latency regime: one request, one GPU's share of the heads, a small static tree):
    the single list is cut into up to a few hundred shares, and the merge takes one workgroup per output row with its
    half-waves sharing the partials.  The second request of the second case is poisoned: its rows must be NaN, the
    other's untouched."""
    from paper_2508_08192_amd import treeattn as ta
    w = W.make_workload("b1", B=1, T=8, Hq=8, Hkv=1, D=128, seq_lens=[20000], trees=W.TREE_N8, page_size=64,
                        dtype="bf16", seed=9300)
    dev = to_device(w)
    plan = ta.tree_attn_plan(dev["q"], dev["k_cache"], dev["v_cache"], dev["page_table"], dev["seq_lens"],
                             dev["tree_parent"], dev["out"], dev["lse"], num_splits=splits)
    assert plan["merge_workgroups"] == 64                          # one per output row
    _check(w, "one list, %d splits" % splits, num_splits=splits)
    w2 = W.make_workload("b2", B=2, T=12, Hq=5, Hkv=1, D=128, seq_lens=[9000, 700], trees=W.TREE_N12, page_size=128,
                         dtype="bf16", seed=9301)
    w2.seq_lens[1] = -5
    ref, ref_lse = run_oracle(w2)
    _announce("two lists, one poisoned, %d splits" % splits)
    got, got_lse = run_hip(w2, num_splits=splits)
    assert np.isnan(got[1]).all() and np.isnan(got_lse[1]).all() and np.isnan(ref[1]).all()
    assert_parity(got[:1], got_lse[:1], ref[:1], ref_lse[:1], "bf16", "beside a poisoned request")
    assert ta.tree_attn_last_status() & ta.TA_STATUS_BAD_SEQLEN


@pytest.mark.parametrize("folded", [False, True])
def test_verify_loop_in_a_graph_write_back_attention_bookkeeping(folded):
    """Stages 4 and 6 of section 3 as the serving loop runs them: per step the tree tokens' K/V are written back,
    the tree is verified, and the accepted path is moved behind the prefix with the lengths advanced on the device.
    The three calls are captured once in a HIP graph; each replay is checked against the oracles run on a host mirror
    of the cache, and after the last step the caches agree bit for bit.  (Which nodes are accepted is the sampler's
    business and outside this library: seeded root-to-node paths stand in.)"""
    import torch
    from oracle import kv_compact_oracle as KC
    from paper_2508_08192_amd import treeattn as ta
    rng = np.random.default_rng(91)
    tree, T, B, Hq, Hkv, D, ps, steps = W.TREE_N8, 8, 3, 8, 2, 128, 16, 5
    lens0 = np.int32([40, 0, 250])
    w = W.make_workload("loop", B=B, T=T, Hq=Hq, Hkv=Hkv, D=D, seq_lens=list(lens0 + steps * 4), trees=tree, page_size=ps,
                        dtype="bf16", seed=9100)
    w.seq_lens[:] = lens0
    k_np, v_np, L = w.k_cache.copy(), w.v_cache.copy(), lens0.copy()
    dev = to_device(w)
    k_new = torch.zeros((B, T, Hkv, D), dtype=torch.bfloat16, device="cuda")
    v_new = torch.zeros_like(k_new)
    acc = torch.zeros((B, T), dtype=torch.int32, device="cuda")
    n_acc = torch.zeros((B,), dtype=torch.int32, device="cuda")
    ta.tree_attn_reserve(ta.tree_attn_workspace_bytes(B, T, Hq, Hkv, D, ta.TA_BF16))

    def step(kc, vc, sl, stream):
        args = (dev["q"], kc, vc, dev["page_table"], sl, dev["tree_parent"], dev["out"], dev["lse"])
        if folded:                                                 # the write-back as part of the attention call
            ta.tree_attn_fwd_ex(*args, stream=stream, k_new=k_new, v_new=v_new)
        else:
            ta.tree_attn_append(k_new, v_new, kc, vc, dev["page_table"], sl, stream=stream)
            ta.tree_attn_fwd(*args, stream=stream)
        ta.tree_attn_compact(kc, vc, dev["page_table"], sl, acc, n_acc, T, seq_lens_out=sl, stream=stream)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                                  # warm-up on copies: kernel attributes get set
        step(dev["k_cache"].clone(), dev["v_cache"].clone(), dev["seq_lens"].clone(), side)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(dev["k_cache"], dev["v_cache"], dev["seq_lens"], torch.cuda.current_stream())
    ta.tree_attn_last_status()

    def bits(x):
        return torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)

    for s in range(steps):
        q_s = W.to_bf16_bits(rng.standard_normal((B, T, Hq, D)).astype(np.float32))
        kn_s = W.to_bf16_bits(rng.standard_normal((B, T, Hkv, D)).astype(np.float32))
        vn_s = W.to_bf16_bits(rng.standard_normal((B, T, Hkv, D)).astype(np.float32))
        paths = [ancestors_inclusive(tree, int(rng.integers(0, T))) for _ in range(B)]
        acc_s = np.zeros((B, T), dtype=np.int32)
        n_s = np.int32([len(p) for p in paths])
        for b, p in enumerate(paths):
            acc_s[b, :len(p)] = p
        # host mirror: write-back, attention oracle, bookkeeping oracle
        for b in range(B):
            for i in range(T):
                pos = int(L[b]) + i
                page, slot = int(w.page_table[b, pos // ps]), pos % ps
                k_np[page, :, slot, :] = kn_s[b, i]
                v_np[page, :, slot, :] = vn_s[b, i]
        import oracle
        ref, ref_lse = oracle.tree_attn_oracle(q_s, k_np, v_np, w.page_table, L, tree, scale=w.scale)
        k_np, v_np, L, skipped = KC.kv_compact_oracle(k_np, v_np, w.page_table, L, acc_s, n_s, T)
        assert skipped == []
        # device: new inputs into the captured buffers, one replay
        dev["q"].copy_(bits(q_s))
        k_new.copy_(bits(kn_s))
        v_new.copy_(bits(vn_s))
        acc.copy_(torch.from_numpy(acc_s))
        n_acc.copy_(torch.from_numpy(n_s))
        dev["out"].fill_(float("nan"))
        dev["lse"].fill_(float("nan"))
        torch.cuda.synchronize()
        _announce("verify loop step %d lens %r accepted %r" % (s, list(L - n_s), list(n_s)))
        graph.replay()
        torch.cuda.synchronize()
        got = dev["out"].float().cpu().numpy().astype(np.float64)
        got_lse = dev["lse"].cpu().numpy().astype(np.float64)
        assert_parity(got, got_lse, ref, ref_lse, "bf16", "verify loop step %d" % s)
        assert np.array_equal(dev["seq_lens"].cpu().numpy(), L)
    assert np.array_equal(dev["k_cache"].view(torch.int16).cpu().numpy(), k_np.view(np.int16))
    assert np.array_equal(dev["v_cache"].view(torch.int16).cpu().numpy(), v_np.view(np.int16))
    assert ta.tree_attn_last_status() == 0


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes_against_oracle(seed):
    """Seeded random geometry: tree size, GQA group, page size, prefix lengths around tile and page edges, splits."""
    rng = np.random.default_rng(9000 + seed)
    T = int(rng.choice([1, 2, 5, 8, 16, 27, 32, 64]))
    G = int(rng.choice([1, 2, 4, 8]))
    Hkv = int(rng.choice([1, 2]))
    B = int(rng.integers(1, 4))
    ps = int(rng.choice([0, 16, 64, 128, 256]))
    edges = [0, 1, 63, 64, 65, 127, 128, 129, 191, 192, 193, 255, 256, 257, 320, 447, 448, 449, 511, 512, 513, 640,
             700, 1023, 1024, 1025, 1500]
    seq_lens = [int(rng.choice(edges)) for _ in range(B)]
    trees = np.stack([W.random_tree(T, int(rng.integers(2, 8)), rng) for _ in range(B)])
    splits = int(rng.choice([0, 0, 1, 2, 3, 5]))
    w = W.make_workload("rand%d" % seed, B=B, T=T, Hq=G * Hkv, Hkv=Hkv, D=128, seq_lens=seq_lens, trees=trees,
                        page_size=ps, dtype="bf16", seed=9100 + seed, paged=ps > 0)
    _check(w, "random seed=%d T=%d G=%d Hkv=%d B=%d ps=%d L=%r splits=%d" % (seed, T, G, Hkv, B, ps, seq_lens, splits),
           kernel=MFMA, num_splits=splits)


def _plan_of(w, **opts):
    from paper_2508_08192_amd import treeattn as ta
    d = to_device(w)
    return ta.tree_attn_plan(d["q"], d["k_cache"], d["v_cache"], d["page_table"], d["seq_lens"], d["tree_parent"],
                             d["out"], d["lse"], scale=w.scale, **opts)


@pytest.mark.parametrize("kernel", [0, MFMA_BASIC, GENERIC])
@pytest.mark.parametrize("rows", [32, 256])
def test_both_formats_of_the_partial_results(kernel, rows):
    """The matrix-core kernels hand their partial results to the merge pass as 16-bit fixed point with one scale per
    row, the scalar kernel as fp32.  Both against the oracle, with forced splits so that every list has several
    partials, and with one KV head's values 64 times smaller than the other's (the scale is per row)."""
    rng = np.random.default_rng(rows)
    T, Hq, Hkv = (8, 8, 2) if rows == 32 else (64, 8, 2)
    B = 5
    trees = np.stack([W.random_tree(T, 6, rng) for _ in range(B)])
    w = W.make_workload("fmt", B=B, T=T, Hq=Hq, Hkv=Hkv, D=128, seq_lens=rng.integers(100, 1500, size=B), trees=trees,
                        page_size=64, dtype="bf16", seed=900 + rows)
    v = w.v_cache.view(np.uint16)
    small = v[:, 1]                                      # KV head 1: exponent down by 6
    keep = (small & 0x7f80) > (6 << 7)
    v[:, 1] = np.where(keep, small - (6 << 7), small & 0x8000).astype(np.uint16)
    plan = _plan_of(w, kernel=kernel)
    assert plan["partials_q15"] == (0 if kernel == GENERIC else 1), plan
    _check(w, "partials rows=%d kernel=%d" % (rows, kernel), kernel=kernel)
    _check(w, "partials rows=%d kernel=%d, 37 shares" % (rows, kernel), kernel=kernel, num_splits=37)


@pytest.mark.parametrize("kernel", [GENERIC, MFMA, MFMA_BASIC])
@pytest.mark.parametrize("rows", [32, 256])
def test_a_nan_among_the_attended_values_reaches_the_output(kernel, rows):
    """A NaN in a value every node of a request attends to: the output column it belongs to is NaN for every row of
    that KV head (with 16-bit partials the whole row is: the row's scale carries the NaN); other KV heads and other
    requests stay finite and right."""
    rng = np.random.default_rng(7 + rows)
    T, Hq, Hkv = (8, 8, 2) if rows == 32 else (64, 8, 2)
    B, ps = 3, 64
    trees = np.stack([W.random_tree(T, 6, rng) for _ in range(B)])
    w = W.make_workload("nanv", B=B, T=T, Hq=Hq, Hkv=Hkv, D=128, seq_lens=[300, 700, 450], trees=trees,
                        page_size=ps, dtype="bf16", seed=950 + rows)
    ref, ref_lse = run_oracle(w)
    b, pos, g, col = 1, 133, 0, 3
    page = int(w.page_table[b, pos // ps])
    w.v_cache.view(np.uint16)[page, g, pos % ps, col] = 0x7fc0
    _announce("NaN value rows=%d kernel=%d" % (rows, kernel))
    got, got_lse = run_hip(w, kernel=kernel, num_splits=9)
    G = Hq // Hkv
    hit = np.zeros_like(got, dtype=bool)
    hit[b, :, g * G:(g + 1) * G, :] = True
    assert np.isnan(got[b, :, g * G:(g + 1) * G, col]).all()
    assert np.isfinite(got[~hit]).all()
    assert np.abs(got[~hit] - ref[~hit]).max() <= 1e-2
    rest = got[b, :, g * G:(g + 1) * G, :]
    ok = np.isnan(rest) | (np.abs(rest - ref[b, :, g * G:(g + 1) * G, :]) <= 1e-2)
    assert ok.all()
    assert np.abs(got_lse - ref_lse).max() <= 1e-3      # the log-sum-exps do not see the values
