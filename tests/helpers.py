"""Test-side helpers: widen workloads to fp64 and flatten a request's cache (independent of oracle and HIP path)."""
import numpy as np

from paper_2508_08192_amd import workloads as W


def widen(a):
    """float64 view of a workload array (float32 values or bf16 bit patterns)."""
    if a.dtype == np.uint16:
        return W.bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


def logical_kv(w, b, n=None):
    """K and V of request b at logical positions 0..n-1 as fp64 arrays [Hkv, n, D]."""
    n = int(w.seq_lens[b]) + w.T if n is None else n
    ps = w.page_size
    K = np.empty((w.Hkv, n, w.D))
    V = np.empty((w.Hkv, n, w.D))
    for pos in range(n):
        if w.page_table is None:
            page, slot = b, pos
        else:
            page, slot = int(w.page_table[b, pos // ps]), pos % ps
        K[:, pos, :] = widen(w.k_cache[page, :, slot, :])
        V[:, pos, :] = widen(w.v_cache[page, :, slot, :])
    return K, V


def ancestors_inclusive(parent, i):
    out = []
    cur = int(i)
    while cur >= 0:
        out.append(cur)
        cur = int(parent[cur])
    return out[::-1]


def run_oracle(w, **kw):
    import oracle
    if w.kv_start is not None:
        kw.setdefault("kv_start", w.kv_start)
    return oracle.tree_attn_oracle(w.q, w.k_cache, w.v_cache, w.page_table, w.seq_lens, w.tree_parent,
                                   scale=w.scale, **kw)


# ----------------------------------------------------------------------------- GPU side

def to_device(w, device="cuda:0"):
    """Upload a workload: returns a dict of torch tensors holding exactly the workload's bits."""
    import torch

    def up(a):
        if a is None:
            return None
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
        return torch.from_numpy(a).to(device)

    d = dict(q=up(w.q), k_cache=up(w.k_cache), v_cache=up(w.v_cache), page_table=up(w.page_table),
             seq_lens=up(w.seq_lens), tree_parent=up(w.tree_parent))
    d["out"] = torch.empty_like(d["q"])
    d["lse"] = torch.empty((w.B, w.Hq, w.T), dtype=torch.float32, device=device)
    return d


def run_hip(w, dev=None, **opts):
    """One call through the C-ABI; returns (out, lse) as fp64 numpy arrays."""
    import torch
    from paper_2508_08192_amd import treeattn as ta
    d = to_device(w) if dev is None else dev
    d["out"].fill_(float("nan"))
    d["lse"].fill_(float("nan"))
    args = (d["q"], d["k_cache"], d["v_cache"], d["page_table"], d["seq_lens"], d["tree_parent"], d["out"], d["lse"])
    if w.kv_start is not None and "kv_start" not in opts:
        opts = dict(opts, kv_start=torch.from_numpy(w.kv_start).cuda())
    if opts or w.scale != float(1.0 / np.sqrt(w.D)):
        ta.tree_attn_fwd_ex(*args, scale=w.scale, **opts)
    else:
        ta.tree_attn_fwd(*args)
    torch.cuda.synchronize()
    return d["out"].float().cpu().numpy().astype(np.float64), d["lse"].cpu().numpy().astype(np.float64)


# Tolerances of the parity bar.  bf16 inputs with fp32 accumulation: max-abs <= 1e-2 and mean-abs <= 1e-3;
# fp32: <= 1e-5.  Outputs shrink like 1/sqrt(L) for long prefixes, so a relative gate rides along:
# max-abs error <= 2e-2 of the largest oracle magnitude (bf16) / 1e-4 (fp32).
def assert_parity(got, got_lse, ref, ref_lse, dtype, what=""):
    err = np.abs(got - ref)
    assert np.isfinite(got).all(), what + ": non-finite output"
    scale = np.abs(ref).max()
    if dtype == "f32":
        assert err.max() <= 1e-5, "%s: max-abs %.3g" % (what, err.max())
        assert err.max() <= 1e-4 * scale + 1e-30, "%s: relative %.3g" % (what, err.max() / scale)
        assert np.abs(got_lse - ref_lse).max() <= 1e-5, "%s: lse %.3g" % (what, np.abs(got_lse - ref_lse).max())
    else:
        assert err.max() <= 1e-2, "%s: max-abs %.3g" % (what, err.max())
        assert err.mean() <= 1e-3, "%s: mean-abs %.3g" % (what, err.mean())
        assert err.max() <= 2e-2 * scale + 1e-30, "%s: relative %.3g" % (what, err.max() / scale)
        assert np.abs(got_lse - ref_lse).max() <= 1e-3, "%s: lse %.3g" % (what, np.abs(got_lse - ref_lse).max())
