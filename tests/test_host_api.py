"""Host-side checks that need no GPU: the library loads, exports what the header declares, rejects bad
descriptors before touching a device, and plans launches sensibly."""
import os
import re

import pytest

from paper_2508_08192_amd import treeattn as ta
from paper_2508_08192_amd.treeattn import Desc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def _built():
    if not os.path.exists(ta.LIB_PATH):
        from paper_2508_08192_amd.build import build_library
        build_library()


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "treeattn.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(tree_attn_\w+)\s*\(", header))
    assert declared == set(ta.EXPORTS)
    lib = ta.load_library()
    for name in declared:
        assert hasattr(lib, name), name
    assert ta.tree_attn_version() == 200
    assert ta.tree_attn_strerror(0) == "ok" and "NULL" in ta.tree_attn_strerror(ta.TA_ERR_NULL)


def _good(B=2, T=8, Hq=8, Hkv=2, D=128, ps=64, max_pages=5, dtype=ta.TA_BF16, pages=16):
    return dict(
        q=Desc((B, T, Hq, D), dtype), k_cache=Desc((pages, Hkv, ps, D), dtype), v_cache=Desc((pages, Hkv, ps, D), dtype),
        page_table=Desc((B, max_pages), ta.TA_I32), seq_lens=Desc((B,), ta.TA_I32),
        tree_parent=Desc((B, T), ta.TA_I32), out=Desc((B, T, Hq, D), dtype), lse=Desc((B, Hq, T), ta.TA_F32))


def _rc(**over):
    a = _good()
    a.update(over)
    # tree_attn_fwd must refuse these before any device call, so it is safe to call it without a GPU
    return ta.tree_attn_fwd(a["q"], a["k_cache"], a["v_cache"], a["page_table"], a["seq_lens"], a["tree_parent"],
                            a["out"], a["lse"], stream=0, check=False)


def test_descriptor_errors_are_reported_before_any_launch():
    assert _rc(q=None) == ta.TA_ERR_NULL
    assert _rc(out=None) == ta.TA_ERR_NULL
    assert _rc(q=Desc((2, 8, 8, 128), ta.TA_BF16, ptr=0)) == ta.TA_ERR_NULL
    assert _rc(q=Desc((2, 8, 8, 128), ta.TA_I32)) == ta.TA_ERR_DTYPE
    assert _rc(k_cache=Desc((16, 2, 64, 128), ta.TA_F32)) == ta.TA_ERR_DTYPE
    assert _rc(seq_lens=Desc((2,), ta.TA_F32)) == ta.TA_ERR_DTYPE
    assert _rc(lse=Desc((2, 8, 8), ta.TA_BF16)) == ta.TA_ERR_DTYPE
    assert _rc(q=Desc((2, 8, 1024), ta.TA_BF16)) == ta.TA_ERR_RANK
    assert _rc(page_table=Desc((10,), ta.TA_I32)) == ta.TA_ERR_RANK
    assert _rc(out=Desc((2, 8, 8, 64), ta.TA_BF16)) == ta.TA_ERR_SHAPE
    assert _rc(v_cache=Desc((16, 2, 32, 128), ta.TA_BF16)) == ta.TA_ERR_SHAPE
    assert _rc(seq_lens=Desc((3,), ta.TA_I32)) == ta.TA_ERR_SHAPE
    assert _rc(tree_parent=Desc((2, 7), ta.TA_I32)) == ta.TA_ERR_SHAPE
    assert _rc(lse=Desc((2, 8, 7), ta.TA_F32)) == ta.TA_ERR_SHAPE
    assert _rc(page_table=Desc((3, 5), ta.TA_I32)) == ta.TA_ERR_SHAPE
    assert _rc(q=Desc((2, 8, 8, 128), ta.TA_BF16, stride=(8192, 1024, 128, 2))) == ta.TA_ERR_STRIDE
    assert _rc(k_cache=Desc((16, 2, 64, 128), ta.TA_BF16, stride=(16384, 8192, -128, 1))) == ta.TA_ERR_STRIDE
    a = _good(Hq=6, Hkv=4)
    assert ta.tree_attn_fwd(*[a[k] for k in ("q", "k_cache", "v_cache", "page_table", "seq_lens", "tree_parent",
                                             "out", "lse")], stream=0, check=False) == ta.TA_ERR_HEADS
    a = _good(D=512)
    assert ta.tree_attn_fwd(*[a[k] for k in ("q", "k_cache", "v_cache", "page_table", "seq_lens", "tree_parent",
                                             "out", "lse")], stream=0, check=False) == ta.TA_ERR_HEAD_DIM
    a = _good(T=65)
    assert ta.tree_attn_fwd(*[a[k] for k in ("q", "k_cache", "v_cache", "page_table", "seq_lens", "tree_parent",
                                             "out", "lse")], stream=0, check=False) == ta.TA_ERR_TREE_SIZE
    a = _good(T=8, ps=4, max_pages=1)
    assert ta.tree_attn_fwd(*[a[k] for k in ("q", "k_cache", "v_cache", "page_table", "seq_lens", "tree_parent",
                                             "out", "lse")], stream=0, check=False) == ta.TA_ERR_PAGE_TABLE
    a = _good(B=5000)
    assert ta.tree_attn_fwd(*[a[k] for k in ("q", "k_cache", "v_cache", "page_table", "seq_lens", "tree_parent",
                                             "out", "lse")], stream=0, check=False) == ta.TA_ERR_BATCH
    # contiguous layout needs one cache row per request
    assert _rc(page_table=None, k_cache=Desc((1, 2, 64, 128), ta.TA_BF16),
               v_cache=Desc((1, 2, 64, 128), ta.TA_BF16)) == ta.TA_ERR_SHAPE


def _plan(a, **kw):
    return ta.tree_attn_plan(a["q"], a["k_cache"], a["v_cache"], a["page_table"], a["seq_lens"], a["tree_parent"],
                             a["out"], a["lse"], **kw)


def test_option_errors():
    a = _good()
    assert _plan(a, kernel=7, check=False) == ta.TA_ERR_OPTS
    assert _plan(a, num_splits=-1, check=False) == ta.TA_ERR_OPTS
    assert _plan(a, item_cost=-1, check=False) == ta.TA_ERR_OPTS
    assert _plan(a, item_cost=4097, check=False) == ta.TA_ERR_OPTS
    assert _plan(a, item_cost=4096)["kernel"] == ta.TA_KERNEL_MFMA
    # more than 256 query heads per KV head: outside the matrix-core kernels' row arithmetic
    assert _plan(_good(Hq=514, Hkv=2))["kernel"] == ta.TA_KERNEL_GENERIC
    # the matrix-core kernel is bf16, head_dim 128, power-of-two pages only
    assert _plan(_good(dtype=ta.TA_F32), kernel=ta.TA_KERNEL_MFMA, check=False) == ta.TA_ERR_OPTS
    assert _plan(_good(D=96), kernel=ta.TA_KERNEL_MFMA, check=False) == ta.TA_ERR_OPTS
    # head_dim 64 runs on the matrix cores too, on the register-staged kernel (its row of the dispatch table)
    p64 = _plan(_good(D=64))
    assert p64["kernel"] == ta.TA_KERNEL_MFMA and p64["merge_kernel"] == ta.TA_MERGE_GENERAL
    assert ta.tree_attn_dispatch_table()[p64["table_row"]]["family"] == ta.TA_KERNEL_MFMA_BASIC
    assert _plan(_good(ps=48), kernel=ta.TA_KERNEL_MFMA, check=False) == ta.TA_ERR_OPTS


def test_plan_picks_kernel_family_and_sizes():
    p = _plan(_good(B=1, T=64, Hq=32, Hkv=8, max_pages=65))
    assert p["kernel"] == ta.TA_KERNEL_MFMA and p["rows_per_group"] == 256 and p["row_groups"] == 1
    assert p["threads"] == 512 and p["tile"] == 64
    assert p["partial_slots"] == p["kv_workgroups"] + 8
    p = _plan(_good(B=32, T=16, Hq=32, Hkv=8, max_pages=129))
    assert p["kernel"] == ta.TA_KERNEL_MFMA and p["rows_per_group"] == 64 and p["threads"] == 512
    p = _plan(_good(B=1, T=64, Hq=64, Hkv=8, max_pages=65))       # 512 rows -> two row groups
    assert p["row_groups"] == 2 and p["rows_per_group"] == 256
    p = _plan(_good(B=1, T=7, Hq=4, Hkv=1, D=64, dtype=ta.TA_F32))
    assert p["kernel"] == ta.TA_KERNEL_GENERIC and p["rows_per_group"] == 28
    p = _plan(_good(ps=48))
    assert p["kernel"] == ta.TA_KERNEL_GENERIC
    p = _plan(_good(), num_splits=3)
    assert p["kv_workgroups"] == 3
    # never more workgroups than tiles that can exist: B*Hkv*(ceil((capacity-T)/64)+1)
    p = _plan(_good(B=1, T=8, Hq=8, Hkv=1, ps=64, max_pages=2))
    assert p["kv_workgroups"] <= 1 * 1 * (2 + 1)


def test_workspace_bound_covers_every_plan():
    for kw in (dict(B=1, T=64, Hq=32, Hkv=8, max_pages=65), dict(B=32, T=16, Hq=32, Hkv=8, max_pages=129),
               dict(B=64, T=32, Hq=8, Hkv=1, max_pages=513), dict(B=3, T=5, Hq=6, Hkv=3, D=64, dtype=ta.TA_F32)):
        a = _good(**kw)
        B, T, Hq, D = a["q"].shape
        Hkv = a["k_cache"].shape[1]
        bound = ta.tree_attn_workspace_bytes(B, T, Hq, Hkv, D, a["q"].dtype, 256)
        for kern in (ta.TA_KERNEL_AUTO, ta.TA_KERNEL_GENERIC):
            p = _plan(a, kernel=kern)
            need = p["partial_slots"] * p["row_groups"] * p["rows_per_group"] * (D + 1) * 4
            assert need <= bound
    assert ta.tree_attn_workspace_bytes(1, 65, 8, 8, 128, ta.TA_BF16, 256) == 0


def test_generated_asm_blocks_match_their_generator():
    """csrc/ta_sp_block.inc is committed next to the script that writes it; the two must not drift apart."""
    import importlib.util
    import os
    csrc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2508_08192_amd", "csrc")
    spec = importlib.util.spec_from_file_location("gen_sp_block", os.path.join(csrc, "gen_sp_block.py"))
    gen = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(gen)
    assert open(os.path.join(csrc, "ta_sp_block.inc")).read() == gen.generate()


def test_append_rejects_bad_arguments_before_any_launch():
    a = _good()
    kn = Desc((2, 8, 2, 128), ta.TA_BF16)
    ok = dict(k_new=kn, v_new=kn, k_cache=a["k_cache"], v_cache=a["v_cache"], page_table=a["page_table"],
              seq_lens=a["seq_lens"])

    def rc(**over):
        d = dict(ok)
        d.update(over)
        return ta.tree_attn_append(d["k_new"], d["v_new"], d["k_cache"], d["v_cache"], d["page_table"], d["seq_lens"],
                                   stream=0, check=False)
    assert rc(k_new=None) == ta.TA_ERR_NULL
    assert rc(v_new=Desc((2, 8, 2, 128), ta.TA_F32)) == ta.TA_ERR_DTYPE
    assert rc(v_new=Desc((2, 8, 2, 64), ta.TA_BF16)) == ta.TA_ERR_SHAPE
    assert rc(k_new=Desc((2, 8, 3, 128), ta.TA_BF16), v_new=Desc((2, 8, 3, 128), ta.TA_BF16)) == ta.TA_ERR_SHAPE
    assert rc(k_new=Desc((2, 65, 2, 128), ta.TA_BF16), v_new=Desc((2, 65, 2, 128), ta.TA_BF16)) == ta.TA_ERR_TREE_SIZE
    assert rc(seq_lens=Desc((3,), ta.TA_I32)) == ta.TA_ERR_SHAPE
    assert rc(page_table=Desc((3, 5), ta.TA_I32)) == ta.TA_ERR_PAGE_TABLE


def test_compact_rejects_bad_arguments_before_any_launch():
    a = _good()
    ok = dict(k_cache=a["k_cache"], v_cache=a["v_cache"], page_table=a["page_table"], seq_lens=a["seq_lens"],
              accepted=Desc((2, 6), ta.TA_I32), n_accepted=Desc((2,), ta.TA_I32), tree_size=8,
              seq_lens_out=Desc((2,), ta.TA_I32))

    def rc(**over):
        d = dict(ok)
        d.update(over)
        return ta.tree_attn_compact(d["k_cache"], d["v_cache"], d["page_table"], d["seq_lens"], d["accepted"],
                                    d["n_accepted"], d["tree_size"], d["seq_lens_out"], stream=0, check=False)
    assert rc(accepted=None) == ta.TA_ERR_NULL
    assert rc(k_cache=None) == ta.TA_ERR_NULL
    assert rc(accepted=Desc((2, 6), ta.TA_F32)) == ta.TA_ERR_DTYPE
    assert rc(v_cache=Desc((16, 2, 64, 128), ta.TA_F32)) == ta.TA_ERR_DTYPE
    assert rc(accepted=Desc((12,), ta.TA_I32)) == ta.TA_ERR_RANK
    assert rc(accepted=Desc((2, 65), ta.TA_I32)) == ta.TA_ERR_TREE_SIZE
    assert rc(tree_size=0) == ta.TA_ERR_TREE_SIZE
    assert rc(tree_size=65) == ta.TA_ERR_TREE_SIZE
    assert rc(n_accepted=Desc((3,), ta.TA_I32)) == ta.TA_ERR_SHAPE
    assert rc(seq_lens_out=Desc((3,), ta.TA_I32)) == ta.TA_ERR_SHAPE
    assert rc(v_cache=Desc((16, 2, 32, 128), ta.TA_BF16)) == ta.TA_ERR_SHAPE
    assert rc(page_table=Desc((3, 5), ta.TA_I32)) == ta.TA_ERR_PAGE_TABLE
    assert rc(accepted=Desc((2, 6), ta.TA_I32, stride=(6, 2))) == ta.TA_ERR_STRIDE
    # lengths may be updated in place, but a shifted overlap of the two arrays is refused
    sl = ok["seq_lens"]
    assert rc(seq_lens_out=Desc((2,), ta.TA_I32, ptr=sl.ptr + 4)) == ta.TA_ERR_STRIDE


def test_folded_write_back_arguments_are_checked_before_any_launch():
    a = _good()
    kn = Desc((2, 8, 2, 128), ta.TA_BF16)

    def rc(**kw):
        return ta.tree_attn_fwd_ex(a["q"], a["k_cache"], a["v_cache"], a["page_table"], a["seq_lens"], a["tree_parent"],
                                   a["out"], a["lse"], stream=0, check=False, **kw)
    assert rc(k_new=kn) == ta.TA_ERR_OPTS                                          # one without the other
    assert rc(k_new=kn, v_new=Desc((2, 8, 2, 128), ta.TA_F32)) == ta.TA_ERR_DTYPE
    assert rc(k_new=kn, v_new=Desc((2, 8, 2), ta.TA_BF16)) == ta.TA_ERR_RANK
    assert rc(k_new=kn, v_new=Desc((2, 7, 2, 128), ta.TA_BF16)) == ta.TA_ERR_SHAPE   # all T tree tokens are needed
    assert rc(k_new=Desc((2, 8, 4, 128), ta.TA_BF16), v_new=Desc((2, 8, 4, 128), ta.TA_BF16)) == ta.TA_ERR_SHAPE
    assert rc(k_new=kn, v_new=Desc((2, 8, 2, 128), ta.TA_BF16, stride=(4096, 512, 256, 2))) == ta.TA_ERR_STRIDE
    assert rc(k_new=kn, v_new=Desc((2, 8, 2, 128), ta.TA_BF16, ptr=0)) == ta.TA_ERR_NULL
    # rows that are not 16-byte aligned: the matrix-core kernel refuses, the automatic choice falls back
    odd = Desc((2, 8, 2, 128), ta.TA_BF16, stride=(8 * 2 * 132, 2 * 132, 132, 1))
    assert rc(k_new=odd, v_new=odd, kernel=ta.TA_KERNEL_MFMA) == ta.TA_ERR_OPTS


def test_dispatch_table_rows_and_the_plans_they_give():
    """Every row of the dispatch table is reachable, and a plan carries exactly its row's figures
    (section 3.4, "Attention kernel": the split is chosen by batch size, tree size and GPU)."""
    table = ta.tree_attn_dispatch_table()
    assert len(table) >= 7
    fam = {ta.TA_KERNEL_MFMA: ta.TA_KERNEL_MFMA, ta.TA_KERNEL_MFMA_BASIC: ta.TA_KERNEL_MFMA_BASIC,
           ta.TA_KERNEL_GENERIC: ta.TA_KERNEL_GENERIC}
    for f in fam:                                   # every family ends in a catch-all row
        last = [r for r in table if r["family"] == f][-1]
        assert last["rows_group_max"] >= 256 and last["lists_max"] == 2 ** 31 - 1
    seen = set()
    cus = 256
    for B, T, Hq, Hkv in [(1, 64, 32, 8), (1, 8, 8, 1), (4, 64, 32, 8), (32, 16, 32, 8), (64, 32, 8, 1), (128, 8, 32, 8),
                          (64, 4, 8, 1), (16, 12, 5, 1), (1, 12, 5, 1), (2, 64, 64, 8), (1, 3, 8, 1), (500, 4, 8, 2),
                          (16, 32, 32, 8), (2, 20, 10, 2)]:
        for kern in (ta.TA_KERNEL_AUTO, ta.TA_KERNEL_MFMA_BASIC, ta.TA_KERNEL_GENERIC):
            a = _good(B=B, T=T, Hq=Hq, Hkv=Hkv, max_pages=129, pages=B * 129)
            p = _plan(a, kernel=kern, num_cus=cus)
            row = table[p["table_row"]]
            seen.add(p["table_row"])
            want_family = ta.TA_KERNEL_MFMA if kern == ta.TA_KERNEL_AUTO else kern
            assert row["family"] == want_family
            assert p["rows_per_group"] <= row["rows_group_max"] and B * Hkv <= row["lists_max"]
            # the first matching row is the one taken
            for r in table[:p["table_row"]]:
                assert not (r["family"] == want_family and p["rows_per_group"] <= r["rows_group_max"]
                            and B * Hkv <= r["lists_max"])
            assert p["min_share"] == row["min_share"] and p["item_cost"] == row["item_cost"]
            per_rg = cus * row["wg_per_cu_x4"] // 4
            if want_family != ta.TA_KERNEL_GENERIC:
                per_rg = max(1, per_rg // p["row_groups"])
            tiles_cap = B * Hkv * ((129 * 64 - T + 63) // 64 + 1)
            assert p["kv_workgroups"] == min(per_rg, tiles_cap)
            parts = -(-p["kv_workgroups"] // (B * Hkv)) + 1
            wide = row["wide_from_parts"] > 0 and parts >= row["wide_from_parts"] and \
                B * Hkv * T * (Hq // Hkv) <= row["wide_max_rows"]
            assert p["merge_kernel"] == (ta.TA_MERGE_D128_WIDE if wide else ta.TA_MERGE_D128)
            assert p["workspace_bytes"] <= ta.tree_attn_workspace_bytes(B, T, Hq, Hkv, 128, ta.TA_BF16, cus)
            # 16-bit partial results from the matrix-core kernels, fp32 ones from the scalar kernel
            assert p["partials_q15"] == int(want_family != ta.TA_KERNEL_GENERIC), (B, T, Hq, Hkv, kern, p)
            # options override the row
            p2 = _plan(a, kernel=kern, num_cus=cus, num_splits=5, item_cost=3)
            assert p2["kv_workgroups"] == 5 and p2["min_share"] == 1 and p2["item_cost"] == 3
    assert seen == set(range(len(table))), "rows never taken: %r" % (set(range(len(table))) - seen)
    assert _plan(_good(D=64, dtype=ta.TA_F32))["merge_kernel"] == ta.TA_MERGE_GENERAL


def test_status_word_option_is_checked():
    a = _good()
    assert _plan(a, status=Desc((1,), ta.TA_I32, ptr=0x2002), check=False) == ta.TA_ERR_OPTS     # not 4-byte aligned
    assert _plan(a, status=Desc((1,), ta.TA_I32, ptr=0x2004))["kernel"] == ta.TA_KERNEL_MFMA


def test_random_descriptors_never_break_the_host_code():
    """Random ranks, shapes, strides and options through the planning and validation code: any answer is fine as
    long as it is a status code (the sanitizer build of the same code runs this test too)."""
    import numpy as np
    rng = np.random.default_rng(99)
    dtypes = [ta.TA_F32, ta.TA_BF16, ta.TA_I32, ta.TA_U64, 7]
    seen = set()
    for case in range(3000):
        B, T = int(rng.integers(0, 6)), int(rng.integers(0, 70))
        Hkv = int(rng.integers(1, 4))
        Hq = Hkv * int(rng.integers(1, 5)) + int(rng.random() < 0.1)
        D = int(rng.choice([0, 1, 64, 128, 128, 128, 256, 300]))
        ps = int(rng.choice([1, 3, 16, 64, 128]))
        dt = int(rng.choice([ta.TA_BF16, ta.TA_BF16, ta.TA_F32]))
        a = _good(B=B, T=T, Hq=Hq, Hkv=Hkv, D=D, ps=ps, max_pages=int(rng.integers(0, 40)), dtype=dt,
                  pages=int(rng.integers(0, 50)))
        if rng.random() < 0.5:                       # damage one descriptor
            key = str(rng.choice(sorted(a)))
            d = a[key]
            kind = int(rng.integers(0, 5))
            if kind == 0:
                a[key] = None
            elif kind == 1:
                a[key] = Desc(d.shape, int(rng.choice(dtypes)), d.stride, d.ptr)
            elif kind == 2:
                a[key] = Desc(d.shape[:-1] if rng.random() < 0.5 else d.shape + (2,), d.dtype)
            elif kind == 3:
                a[key] = Desc(d.shape, d.dtype, tuple(int(x) * int(rng.choice([-1, 1, 2, 3])) for x in d.stride), d.ptr)
            else:
                a[key] = Desc(tuple(int(rng.integers(0, 2 ** 33)) for _ in d.shape), d.dtype, d.stride,
                              int(rng.choice([0, 0x1000, 0x1002])))
        kw = dict(kernel=int(rng.integers(-1, 5)), num_splits=int(rng.integers(-1, 2000)),
                  item_cost=int(rng.integers(-1, 5000)), num_cus=int(rng.choice([0, 1, 256, 304])), check=False)
        r = _plan(a, **kw)
        if isinstance(r, dict):
            assert r["kv_workgroups"] >= 1 and r["partial_slots"] >= r["kv_workgroups"] and r["workspace_bytes"] > 0
            seen.add(0)
        else:
            assert -13 <= r < 0
            seen.add(r)
        n = ta.tree_attn_workspace_bytes(B, T, Hq, Hkv, D, dt, 256)
        assert n >= 0
    assert 0 in seen and len(seen) >= 8


def test_host_code_under_address_and_undefined_behaviour_sanitizers():
    """The same host tests against a g++ build of the host logic with -fsanitize=address,undefined (its launching
    entry points stop where the real library would touch a device).  A finding aborts the child process."""
    import subprocess
    import sys
    from paper_2508_08192_amd.build import build_host_checked
    lib, runtime = build_host_checked()
    assert os.path.exists(lib) and os.path.exists(runtime), (lib, runtime)
    env = dict(os.environ)
    env["TREEATTN_LIB"] = lib
    env["LD_PRELOAD"] = (runtime + " " + env.get("LD_PRELOAD", "")).strip()
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    proc = subprocess.run([sys.executable, "-m", "pytest", os.path.abspath(__file__), "-q", "-x", "-p", "no:cacheprovider",
                           "-k", "not sanitizers and not generated_asm"], cwd=ROOT, env=env, stdout=subprocess.PIPE,
                          stderr=subprocess.STDOUT, text=True, timeout=600)
    assert proc.returncode == 0, proc.stdout[-4000:]
    assert "passed" in proc.stdout
