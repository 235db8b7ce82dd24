"""The entry point that allocates nothing (tree_attn_fwd_static: partial results in a fixed scratch area of the
library image) against tree_attn_fwd_ex, through the C-ABI: bit for bit the same outputs, on calls in a row that
share the scratch area, the later ones smaller than the first."""
import numpy as np
import pytest

from paper_2508_08192_amd import workloads as W

from .helpers import assert_parity, run_oracle, to_device

pytestmark = pytest.mark.gpu


def _both(w, **opts):
    """(out, lse) of tree_attn_fwd_ex and of tree_attn_fwd_static on the same device tensors."""
    import torch
    from paper_2508_08192_amd import treeattn as ta
    dev = to_device(w)
    if w.kv_start is not None:
        opts = dict(opts, kv_start=torch.from_numpy(w.kv_start).cuda())
    args = (dev["q"], dev["k_cache"], dev["v_cache"], dev["page_table"], dev["seq_lens"], dev["tree_parent"])
    res = []
    for fn in (ta.tree_attn_fwd_ex, ta.tree_attn_fwd_static):
        out = torch.full_like(dev["q"], float("nan"))
        lse = torch.full((w.B, w.Hq, w.T), float("nan"), dtype=torch.float32, device="cuda")
        fn(*args, out, lse, scale=w.scale, **opts)
        torch.cuda.synchronize()
        res.append((out, lse))
    return res


def test_static_scratch_call_equals_the_allocating_call_on_calls_in_a_row():
    import torch
    from paper_2508_08192_amd import treeattn as ta
    rng = np.random.default_rng(21)
    big = W.make_config(3, length_div=16)                       # 64 lists x 256-row groups: tens of MB of partials
    mid = W.make_workload("static_mid", B=3, T=16, Hq=8, Hkv=2, D=128, seq_lens=[900, 64, 2000],
                          trees=np.stack([W.random_tree(16, 5, rng) for _ in range(3)]), page_size=64, dtype="bf16",
                          seed=2101)
    tiny = W.make_config(0)                                     # fp32, scalar kernels
    ta.tree_attn_last_status()
    for w, opts in ((big, {}), (mid, {}), (mid, dict(num_splits=7)), (tiny, {}), (mid, dict(kernel=1))):
        print("\n[case] static scratch, %s %r" % (w.name, opts), flush=True)
        (o_ex, l_ex), (o_st, l_st) = _both(w, **opts)
        bits = torch.int16 if w.dtype == "bf16" else torch.int32
        assert torch.equal(o_ex.view(bits), o_st.view(bits)), "outputs differ"
        assert torch.equal(l_ex.view(torch.int32), l_st.view(torch.int32)), "lse differs"
        ref, ref_lse = run_oracle(w)
        assert_parity(o_st.float().cpu().numpy().astype(np.float64), l_st.cpu().numpy().astype(np.float64), ref,
                      ref_lse, w.dtype, w.name)
    assert ta.tree_attn_last_status() == 0


def test_static_scratch_call_refuses_what_does_not_fit_and_a_caller_workspace():
    import torch
    from paper_2508_08192_amd import treeattn as ta
    w = W.make_workload("static_big", B=40, T=64, Hq=32, Hkv=8, D=128, seq_lens=[100] * 40,
                        trees=W.bfs_tree(64, [4], 6), page_size=64, dtype="bf16", seed=2201)
    dev = to_device(w)
    args = (dev["q"], dev["k_cache"], dev["v_cache"], dev["page_table"], dev["seq_lens"], dev["tree_parent"], dev["out"],
            dev["lse"])
    plan = ta.tree_attn_plan(*args, num_cus=torch.cuda.get_device_properties(0).multi_processor_count)
    assert plan["workspace_bytes"] > ta.TA_STATIC_SCRATCH_BYTES
    dev["out"].fill_(7.0)
    assert ta.tree_attn_fwd_static(*args, check=False) == ta.TA_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert (dev["out"] == 7.0).all().item()                     # nothing was launched
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    assert ta.tree_attn_fwd_static(*args, workspace=ws, check=False) == ta.TA_ERR_OPTS
