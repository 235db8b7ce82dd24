#!/usr/bin/env python3
"""Benchmark of the tree-attention verify step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5]

A step is one pass of the whole hot path -- tree_attn_fwd through the C-ABI: KV pass (prefix tiles +
masked tree tile, tree encoding fused in) and merge pass -- over one batch of seeded synthetic input
that is already resident in HBM.  Prints ONE JSON line: microseconds per verify step on the named
workload, the roofline of the dominant kernel (the KV pass; its duration is measured with HIP events
recorded inside the timed region on the launch stream), and the fp64 oracle timed on the host cores
over a bounded sample of the same workload.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix cores, published
WORKLOADS = {"c1": 0, "c2": 1, "c3": 2, "c4": 3, "c5": 4}
# shapes of the regime the paper deploys (few query rows per KV head, memory-bound): workloads.make_production
PRODUCTION = {"p1": 0, "p2": 1, "p3": 2, "p4": 3, "p5": 4, "p6": 5, "p7": 6, "u32": 7, "u64": 8, "u128": 9}


def make(name):
    from paper_2508_08192_amd import workloads as W
    return W.make_config(WORKLOADS[name]) if name in WORKLOADS else W.make_production(PRODUCTION[name])


class HipEvents:
    """hipEvent_t handles through libamdhip64 (torch.cuda.Event only sees torch's own recording)."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def create(self):
        ev = ctypes.c_void_p()
        assert self.hip.hipEventCreate(ctypes.byref(ev)) == 0
        return ev

    def elapsed_ms(self, a, b):
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
        assert rc == 0, "hipEventElapsedTime -> %d" % rc
        return float(ms.value)

    def destroy(self, ev):
        self.hip.hipEventDestroy(ev)


def upload(w, torch):
    import numpy as np

    def up(a):
        if a is None:
            return None
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(a).cuda()

    d = dict(q=up(w.q), k_cache=up(w.k_cache), v_cache=up(w.v_cache), page_table=up(w.page_table),
             seq_lens=up(w.seq_lens), tree_parent=up(w.tree_parent))
    d["out"] = torch.empty_like(d["q"])
    d["lse"] = torch.empty((w.B, w.Hq, w.T), dtype=torch.float32, device="cuda")
    d["kv_start"] = up(w.kv_start)
    return d


def cpu_baseline(w, budget_s, log):
    """The oracle as it stands, on the host cores, over a uniform sample of (request, node, head) outputs."""
    import numpy as np
    import oracle
    rng = np.random.default_rng(12345)
    total = w.B * w.T * w.Hq
    threads = oracle.oracle_threads()

    def run(n):
        tri = np.stack([rng.integers(0, w.B, n), rng.integers(0, w.T, n), rng.integers(0, w.Hq, n)], axis=1)
        t0 = time.perf_counter()
        oracle.tree_attn_oracle_sample(w.q, w.k_cache, w.v_cache, w.page_table, w.seq_lens, w.tree_parent, tri,
                                       scale=w.scale, kv_start=w.kv_start)
        return time.perf_counter() - t0

    probe_n = min(total, 4 * threads)
    probe = run(probe_n)
    n = int(max(probe_n, min(total, budget_s / max(probe / probe_n, 1e-9))))
    dt = run(n)
    log("cpu_baseline: %d of %d outputs in %.2f s on %d threads" % (n, total, dt, threads))
    est_us = dt / n * total * 1e6
    return {"value": est_us, "unit": "us/verify_step", "cores": threads, "kind": "oracle",
            "sample": "%d of %d (request,node,head) outputs drawn uniformly, %.1f s of wall time, "
                      "scaled by %d/%d" % (n, total, dt, total, n)}


SETTLE_SECONDS = 0.3           # untimed load before anything is timed: the shader clock needs ~0.1-0.2 s to settle
KERNEL_PASS_STEPS = 50          # least number of launches the per-kernel figures are taken over
IN_REGION_FROM_US = 100.0       # steps at least this long carry their kernel events inside the timed region itself


def _stats(xs):
    xs = sorted(xs)
    n = len(xs)
    med = xs[n // 2] if n % 2 else 0.5 * (xs[n // 2 - 1] + xs[n // 2])
    return {"mean": sum(xs) / n, "median": med, "min": xs[0], "max": xs[-1], "n": n}


def attainable_hbm(log):
    """Read rate a plain streaming kernel reaches on this device (GB/s): the library's tree_attn_stream_read over
    2 GiB, 20 launches between two events on the launch stream after 5 warm-up launches."""
    import torch
    from paper_2508_08192_amd import treeattn as ta
    n_bytes = 2 << 30
    buf = torch.empty(n_bytes // 4, dtype=torch.float32, device="cuda").fill_(1.0)
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    stream = torch.cuda.current_stream()
    t_end = time.perf_counter() + SETTLE_SECONDS
    while time.perf_counter() < t_end:
        for _ in range(5):
            ta.tree_attn_stream_read(buf, sink, stream=stream)
        torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)   # torch's own stream: fine here
    e0.record(stream)
    for _ in range(20):
        ta.tree_attn_stream_read(buf, sink, stream=stream)
    e1.record(stream)
    torch.cuda.synchronize()
    gbs = n_bytes * 20 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    log("attainable HBM read rate (plain streaming kernel, 2 GiB x 20): %.0f GB/s" % gbs)
    del buf
    torch.cuda.empty_cache()
    return gbs


def attainable_mfma(log):
    """bf16 matrix-core rate this device sustains (TFLOP/s): the library's tree_attn_mfma_probe, back to back for
    SETTLE_SECONDS so that the clock settles under the power limit, then 5 launches between two events."""
    import torch
    from paper_2508_08192_amd import treeattn as ta
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()
    iters = 2000                                  # about 1.3 ms per launch
    t_end = time.perf_counter() + 2 * SETTLE_SECONDS
    while time.perf_counter() < t_end:
        for _ in range(10):
            ta.tree_attn_mfma_probe(iters, sink, stream=stream)
        torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    flop = 0
    for _ in range(5):
        flop += ta.tree_attn_mfma_probe(iters, sink, stream=stream)
    e1.record(stream)
    torch.cuda.synchronize()
    tf = flop / (e0.elapsed_time(e1) * 1e-3) / 1e12
    log("attainable bf16 matrix-core rate (registers only, sustained): %.0f TFLOP/s" % tf)
    return tf


def prepare(w, log, rotate=0):
    """Uploads workload w and makes the copies of its KV pool the steps cycle through."""
    import numpy as np
    import torch
    dev = upload(w, torch)
    pool_bytes = dev["k_cache"].numel() * dev["k_cache"].element_size() * 2
    # Small workloads would be served from the 256 MB last-level cache on repeated calls; cycle through
    # enough copies of the KV pool that every step streams from HBM ("cold").  rotate=1 keeps one pool ("hot").
    if rotate > 0:
        n_pools = rotate
    elif pool_bytes >= 600e6:
        n_pools = 1
    else:
        n_pools = max(1, min(64, int(np.ceil(600e6 / max(pool_bytes, 1)))))
    pools = [(dev["k_cache"], dev["v_cache"])]
    for _ in range(n_pools - 1):
        pools.append((dev["k_cache"].clone(), dev["v_cache"].clone()))
    log("%s: KV pool %.1f MB x %d copies" % (w.name, pool_bytes / 1e6, n_pools))
    return dict(w=w, dev=dev, pools=pools)


def measure(ctx, steps, warmup, log, num_splits=0, kernel=0, check=False, item_cost=0, kernel_pass=True, hot=False):
    """Times `steps` verify steps of the prepared workload ctx (hot: on one KV pool only, so that a small
    workload is served from the last-level cache).  Protocol: `warmup` untimed steps, then untimed steps until
    SETTLE_SECONDS of load have passed (clock settle, independent of the command line), then EXACTLY `steps` steps
    between two synchronisations (wall clock -> the step time), then -- without a pause -- a kernel pass of at least
    KERNEL_PASS_STEPS steps that each carry the library's three HIP events on the launch stream (-> per-launch
    durations of the KV pass and the merge pass: mean, median, min).  When a step is long enough that three events do
    not matter (>= IN_REGION_FROM_US), the timed region itself carries the events on every step and its figures are
    reported as well."""
    import numpy as np
    import torch
    from paper_2508_08192_amd import treeattn as ta

    w, dev = ctx["w"], ctx["dev"]
    pools = ctx["pools"][:1] if hot else ctx["pools"]
    n_pools = len(pools)
    alg_bytes = w.algorithmic_bytes()
    flops = w.useful_flops()

    plan = ta.tree_attn_plan(dev["q"], dev["k_cache"], dev["v_cache"], dev["page_table"], dev["seq_lens"],
                             dev["tree_parent"], dev["out"], dev["lse"],
                             num_cus=torch.cuda.get_device_properties(0).multi_processor_count,
                             num_splits=num_splits, kernel=kernel, item_cost=item_cost)
    log("plan %r" % plan)
    ta.tree_attn_reserve(plan["workspace_bytes"])
    stream = torch.cuda.current_stream()

    def step(i, events=None):
        k, v = pools[i % n_pools]
        ta.tree_attn_fwd_ex(dev["q"], k, v, dev["page_table"], dev["seq_lens"], dev["tree_parent"], dev["out"],
                            dev["lse"], stream=stream, scale=w.scale, num_splits=num_splits, kernel=kernel,
                            events=events, item_cost=item_cost, kv_start=dev["kv_start"])

    if check:
        import oracle
        step(0)
        torch.cuda.synchronize()
        rng = np.random.default_rng(7)
        tri = np.stack([rng.integers(0, w.B, 64), rng.integers(0, w.T, 64), rng.integers(0, w.Hq, 64)], axis=1)
        ref, ref_lse = oracle.tree_attn_oracle_sample(w.q, w.k_cache, w.v_cache, w.page_table, w.seq_lens,
                                                      w.tree_parent, tri, scale=w.scale, kv_start=w.kv_start)
        got = dev["out"].float().cpu().numpy()[tri[:, 0], tri[:, 1], tri[:, 2]]
        log("check: max-abs err %.3g (oracle max %.3g)" % (np.abs(got - ref).max(), np.abs(ref).max()))

    it = 0
    for _ in range(warmup):
        step(it)
        it += 1
    torch.cuda.synchronize()
    # clock settle: untimed, at least SETTLE_SECONDS of back-to-back steps whatever --warmup was
    t_s = time.perf_counter()
    settle_steps = 0
    while time.perf_counter() - t_s < SETTLE_SECONDS:
        for _ in range(20):
            step(it)
            it += 1
        settle_steps += 20
        torch.cuda.synchronize()
    settle_s = time.perf_counter() - t_s
    est_us = settle_s / settle_steps * 1e6
    in_region = est_us >= IN_REGION_FROM_US

    hev = HipEvents()
    n_pass = max(KERNEL_PASS_STEPS, steps) if kernel_pass else 0
    evs = [[hev.create() for _ in range(3)] for _ in range(max(n_pass, steps if in_region else 0))]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(it + i, evs[i] if in_region else None)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    it += steps
    ms_per_step = elapsed / steps * 1e3
    region = None
    if in_region:
        region = {"kv_pass_us": _stats([hev.elapsed_ms(e[0], e[1]) * 1e3 for e in evs[:steps]]),
                  "merge_pass_us": _stats([hev.elapsed_ms(e[1], e[2]) * 1e3 for e in evs[:steps]])}
        # a kernel cannot take longer than the step that contains it
        assert region["kv_pass_us"]["mean"] + region["merge_pass_us"]["mean"] <= ms_per_step * 1e3 * 1.05, \
            (region, ms_per_step)
    kp = None
    if kernel_pass:
        for i in range(n_pass):
            step(it + i, evs[i])
        torch.cuda.synchronize()
        it += n_pass
        kp = {"kv_pass_us": _stats([hev.elapsed_ms(e[0], e[1]) * 1e3 for e in evs[:n_pass]]),
              "merge_pass_us": _stats([hev.elapsed_ms(e[1], e[2]) * 1e3 for e in evs[:n_pass]]),
              "step_us": _stats([hev.elapsed_ms(e[0], e[2]) * 1e3 for e in evs[:n_pass]])}
    for e in evs:
        for x in e:
            hev.destroy(x)
    src = region if in_region else kp
    kv_avg_us = src["kv_pass_us"]["mean"] if src else float("nan")
    mg_avg_us = src["merge_pass_us"]["mean"] if src else float("nan")
    log("%s: step %.1f us (wall, %d steps after %d warm-up + %d settle steps in %.2f s); KV pass mean %.1f median %.1f "
        "min %.1f us, merge pass mean %.1f us (%s)" %
        (w.name, ms_per_step * 1e3, steps, warmup, settle_steps, settle_s, kv_avg_us,
         src["kv_pass_us"]["median"] if src else float("nan"), src["kv_pass_us"]["min"] if src else float("nan"),
         mg_avg_us, "events inside the timed region" if in_region else "kernel pass after the timed region"))

    # Roofline of the dominant kernel (KV pass).  Its algorithmic bytes per launch: every K and V element
    # of prefix and tree once, plus q and the ids it reads (the output and lse belong to the merge pass).
    es = 4 if w.dtype == "f32" else 2
    kv_alg = alg_bytes - w.B * w.T * w.Hq * (w.D * es + 4)
    hbm_frac = kv_alg / (kv_avg_us * 1e-6) / 1e9 / HBM_PEAK_GBS
    mfma_frac = flops / (kv_avg_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS if w.dtype == "bf16" else 0.0
    return dict(w=w, plan=plan, n_pools=n_pools, ms_per_step=ms_per_step, kv_us=kv_avg_us, merge_us=mg_avg_us,
                alg_bytes=alg_bytes, kv_alg=kv_alg, flops=flops, hbm_frac=hbm_frac, mfma_frac=mfma_frac,
                in_region=in_region, region=region, kernel_pass=kp, settle_steps=settle_steps, settle_s=settle_s)


def dispatch_check(ctx, log, base):
    """The library's own pick (one row of its dispatch table) against forced alternatives (ta_opts.num_splits,
    ta_opts.item_cost) on one prepared workload: events from before the KV pass to after the merge pass, median over
    the kernel pass.  Returns the pick's time over the best one's."""
    import torch
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    auto_wg, auto_cost = base["plan"]["kv_workgroups"], base["plan"]["item_cost"]
    cands = []
    for wg in sorted({max(1, auto_wg // 2), auto_wg, min(auto_wg * 2, cus * 2)}):
        for cost in sorted({1, auto_cost, auto_cost * 2}):
            cands.append((wg, cost))

    def timed(wg, cost):
        m = measure(ctx, 20, 0, lambda msg: None, num_splits=wg, item_cost=cost)
        return m["kernel_pass"]["step_us"]["median"]

    # the pick is timed in the same loop as the alternatives, before and after them (the smaller counts): a figure
    # taken minutes earlier, at another clock, says nothing about the choice
    first = timed(0, 0)
    rows = [{"num_splits": wg, "item_cost": cost, "step_us_median": timed(wg, cost)} for wg, cost in cands]
    rows.insert(0, {"num_splits": 0, "item_cost": 0, "step_us_median": min(first, timed(0, 0))})
    best = min(rows, key=lambda r: r["step_us_median"])
    auto = rows[0]
    log("dispatch check %s: library pick (row %d: %d workgroups, item cost %d) %.1f us, best of %d forced %.1f us "
        "(%d workgroups, item cost %d)" %
        (ctx["w"].name, base["plan"]["table_row"], auto_wg, auto_cost, auto["step_us_median"], len(cands),
         best["step_us_median"], best["num_splits"], best["item_cost"]))
    return {"table_row": base["plan"]["table_row"], "auto_us": auto["step_us_median"], "best_us": best["step_us_median"],
            "best": {"num_splits": best["num_splits"], "item_cost": best["item_cost"]},
            "auto_over_best": auto["step_us_median"] / best["step_us_median"], "tried": len(cands),
            "forced_us": {"%dx%d" % (r["num_splits"], r["item_cost"]): round(r["step_us_median"], 1) for r in rows[1:]}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="c5", choices=sorted(WORKLOADS) + sorted(PRODUCTION))
    ap.add_argument("--num-splits", type=int, default=0)
    ap.add_argument("--kernel", type=int, default=0)
    ap.add_argument("--item-cost", type=int, default=0, help="ta_opts.item_cost (0 = the library's choice)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="wall-time budget of the oracle baseline (0 = skip)")
    ap.add_argument("--rotate", type=int, default=0,
                    help="distinct KV pools to cycle through (0 = enough to exceed the 256 MB last-level cache)")
    ap.add_argument("--check", action="store_true", help="compare sampled outputs with the oracle before timing")
    ap.add_argument("--others", type=int, default=1,
                    help="also time the other configurations briefly and list them under other_workloads (0 = no)")
    ap.add_argument("--dispatch-check", type=int, default=1,
                    help="with --others: time forced splits and per-list costs beside the library's own pick (0 = no)")
    ap.add_argument("--probes", type=int, default=1,
                    help="measure the attainable HBM read rate and matrix-core rate first (0 = skip, for profiler runs)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="instead of the benchmark, run a plain elementwise copy of 1 GiB (read 1 GiB, write 1 GiB) "
                         "five times: the known traffic against which HBM byte counters are scaled")
    args = ap.parse_args()
    if args.calibrate_copy:
        import torch
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": {"launches": 5, "read_bytes": 1 << 30, "write_bytes": 1 << 30}}))
        return 0
    if args.gpus != 1:
        print("bench.py measures one GPU: every box in this build has a single MI355X and the path needs no "
              "collective (it shards by KV head or by request without communication). Run with --gpus 1.",
              file=sys.stderr)
        return 2

    def log(msg):
        print("[bench] " + msg, file=sys.stderr, flush=True)

    import numpy as np
    import torch
    from paper_2508_08192_amd import treeattn as ta

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    ta.load_library()          # fails loudly if the HIP library is not built
    attainable = attainable_hbm(log) if args.probes else float("nan")
    attainable_tf = attainable_mfma(log) if args.probes else float("nan")
    t0 = time.time()
    w = make(args.workload)
    log("workload %s generated in %.1f s" % (w.name, time.time() - t0))
    ctx = prepare(w, log, args.rotate)
    m = measure(ctx, args.steps, args.warmup, log, args.num_splits, args.kernel, args.check, args.item_cost)
    ms_per_step, kv_us, plan = m["ms_per_step"], m["kv_us"], m["plan"]
    alg_bytes, kv_alg, flops = m["alg_bytes"], m["kv_alg"], m["flops"]

    traffic, traffic_at = None, None
    # HBM bytes per KV-pass launch as counted by rocprofv3 (FETCH_SIZE + WRITE_SIZE, scaled by a copy of
    # known size); the counter runs are separate, their summary sits under profiles/ and names the commit of the
    # sources it was collected with.
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if os.path.exists(tpath):
        body = json.loads("".join(l for l in open(tpath) if not l.startswith("#")))
        traffic = body.get(w.name, {}).get("kv_pass_bytes_per_launch")
        traffic_at = body.get("collected_at_commit")
    if m["hbm_frac"] >= m["mfma_frac"]:
        roof = {"bound": "hbm", "achieved": kv_alg / (kv_us * 1e-6) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": m["hbm_frac"], "traffic": traffic}
    else:
        roof = {"bound": "mfma", "achieved": flops / (kv_us * 1e-6) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": m["mfma_frac"], "traffic": traffic}
    src = m["region"] if m["in_region"] else m["kernel_pass"]
    med_us = src["kv_pass_us"]["median"]
    roof.update({"kernel": "ta_generic_kv_kernel" if plan["kernel"] != 2 else "ta_mfma_sp_kernel",
                 "avg_launch_us": kv_us, "median_launch_us": med_us, "min_launch_us": src["kv_pass_us"]["min"],
                 "launches_timed": src["kv_pass_us"]["n"],
                 "timed": "HIP events on the launch stream, every step of the timed region" if m["in_region"] else
                          "HIP events on the launch stream, every step of a kernel pass that follows the timed region "
                          "without a pause (three events per step would distort a step this short)",
                 "algorithmic_bytes_per_launch": kv_alg, "useful_flops_per_launch": flops,
                 "hbm_frac": m["hbm_frac"], "mfma_frac": m["mfma_frac"],
                 "hbm_frac_median": kv_alg / (med_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                 "attainable_GBps": attainable, "frac_of_attainable": kv_alg / (kv_us * 1e-6) / 1e9 / attainable,
                 "attainable_mfma_TFLOPs": attainable_tf,
                 "mfma_frac_of_attainable": flops / (kv_us * 1e-6) / 1e12 / attainable_tf if w.dtype == "bf16" else 0.0,
                 "ideal_us_at_attainable_rates": max(kv_alg / 1e9 / attainable, flops / 1e12 / attainable_tf) * 1e6,
                 "traffic_collected_at_commit": traffic_at})

    result = {
        "metric": "tree-attn us/verify step; achieved HBM GB/s & MFMA util vs MI355X peak",
        "value": ms_per_step * 1e3,
        "unit": "us/verify_step",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if w.dtype == "f32" else "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "T": w.T, "Hq": w.Hq, "Hkv": w.Hkv, "D": w.D,
                   "page_size": w.page_size if w.page_table is not None else 0,
                   "sum_prefix_tokens": int(w.seq_lens.astype(np.int64).sum()), "kv_pools_rotated": m["n_pools"],
                   "kv_std": w.meta["kv_std"], "plan": plan},
        "clock_settle": {"untimed_steps": m["settle_steps"], "seconds": m["settle_s"]},
        "tree_tokens_per_s": w.B * w.T / (ms_per_step * 1e-3),
        "kv_tokens_per_s": float(w.seq_lens.astype(np.int64).sum() + w.B * w.T) / (ms_per_step * 1e-3),
        "step_GBps": alg_bytes / (ms_per_step * 1e-3) / 1e9,
        "step_TFLOPs": flops / (ms_per_step * 1e-3) / 1e12,
        "step_frac_of_roofline": max(alg_bytes / 1e9 / HBM_PEAK_GBS, flops / 1e12 / MFMA_BF16_PEAK_TFLOPS) /
                                 (ms_per_step * 1e-3),
        "kernels_us": {"kv_pass": kv_us, "merge_pass": m["merge_us"],
                       "timed_region": m["region"], "kernel_pass": m["kernel_pass"]},
        "roofline": roof,
    }
    if args.cpu_seconds > 0:
        result["cpu_baseline"] = cpu_baseline(w, args.cpu_seconds, log)
    if args.others and args.dispatch_check:
        result["dispatch_check"] = {w.name: dispatch_check(ctx, log, m)}
    del m, w, ctx
    torch.cuda.empty_cache()
    if args.others:
        # the remaining configurations, briefly (context for the headline line; not separate bench lines)
        def brief(name):
            wo = make(name)
            cx = prepare(wo, log)
            mo = measure(cx, 50, 10, log)
            src = mo["region"] if mo["in_region"] else mo["kernel_pass"]
            row = {"us_per_step": mo["ms_per_step"] * 1e3, "kv_pass_us": mo["kv_us"],
                   "kv_pass_us_median": src["kv_pass_us"]["median"], "kv_pass_us_min": src["kv_pass_us"]["min"],
                   "merge_pass_us": mo["merge_us"], "hbm_frac": mo["hbm_frac"],
                   "mfma_frac": mo["mfma_frac"], "hbm_GBps": mo["kv_alg"] / (mo["kv_us"] * 1e-6) / 1e9,
                   "algorithmic_bytes": mo["alg_bytes"], "useful_flops": mo["flops"], "kv_pools": mo["n_pools"],
                   "table_row": mo["plan"]["table_row"], "partials_q15": mo["plan"]["partials_q15"]}
            if mo["n_pools"] > 1:
                # working set below the last-level cache: the figures above are "cold" (every step streams another
                # copy of the KV pool from HBM); "hot" repeats the step on one pool
                mh = measure(cx, 50, 10, lambda msg: None, hot=True)
                sh = mh["kernel_pass"]
                row["hot"] = {"us_per_step": mh["ms_per_step"] * 1e3, "kv_pass_us_median": sh["kv_pass_us"]["median"],
                              "kv_pass_us_min": sh["kv_pass_us"]["min"], "merge_pass_us": mh["merge_us"]}
            if args.dispatch_check:
                result["dispatch_check"][wo.name] = dispatch_check(cx, log, mo)
            del mo, cx
            torch.cuda.empty_cache()
            return wo.name, row
        result["other_workloads"] = dict(brief(n) for n in sorted(WORKLOADS) if n != args.workload)
        result["production_shapes"] = dict(brief(n) for n in PRODUCTION if n != args.workload)
        if args.dispatch_check:
            worst = max(result["dispatch_check"].values(), key=lambda r: r["auto_over_best"])
            result["dispatch_check"]["worst_auto_over_best"] = worst["auto_over_best"]
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
