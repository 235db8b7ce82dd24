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
PRODUCTION = {"p1": 0, "p2": 1, "p3": 2, "p4": 3, "p5": 4, "p6": 5, "p7": 6}


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


EVENT_EVERY = 8


def measure(w, steps, warmup, log, num_splits=0, kernel=0, rotate=0, check=False, item_cost=0):
    """Times `steps` verify steps of workload w (after `warmup` untimed ones).  Returns a dict with the step
    time, per-kernel times from HIP events recorded inside the timed region, and roofline figures."""
    import numpy as np
    import torch
    from paper_2508_08192_amd import treeattn as ta

    dev = upload(w, torch)
    alg_bytes = w.algorithmic_bytes()
    flops = w.useful_flops()
    pool_bytes = dev["k_cache"].numel() * dev["k_cache"].element_size() * 2
    # Small workloads would be served from the 256 MB last-level cache on repeated calls; cycle through
    # enough copies of the KV pool that every step streams from HBM.
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

    plan = ta.tree_attn_plan(dev["q"], dev["k_cache"], dev["v_cache"], dev["page_table"], dev["seq_lens"],
                             dev["tree_parent"], dev["out"], dev["lse"],
                             num_cus=torch.cuda.get_device_properties(0).multi_processor_count,
                             num_splits=num_splits, kernel=kernel)
    log("plan %r" % plan)
    ta.tree_attn_reserve(ta.tree_attn_workspace_bytes(w.B, w.T, w.Hq, w.Hkv, w.D,
                                                      ta.TA_F32 if w.dtype == "f32" else ta.TA_BF16))
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

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()

    # Per-kernel durations come from HIP events the library records on the launch stream inside the timed region.
    # Recording costs 2-3 us per event, which would inflate the step time of the small workloads by a quarter, so
    # only every EVENT_EVERY-th step of the timed region carries events.
    hev = HipEvents()
    evs = [[hev.create() for _ in range(3)] for _ in range((steps + EVENT_EVERY - 1) // EVENT_EVERY)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(warmup + i, evs[i // EVENT_EVERY] if i % EVENT_EVERY == 0 else None)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / steps * 1e3
    kv_ms = [hev.elapsed_ms(e[0], e[1]) for e in evs]
    mg_ms = [hev.elapsed_ms(e[1], e[2]) for e in evs]
    for e in evs:
        for x in e:
            hev.destroy(x)
    kv_avg = sum(kv_ms) / len(kv_ms)
    mg_avg = sum(mg_ms) / len(mg_ms)
    log("%s: KV pass avg %.1f us (min %.1f), merge pass avg %.1f us, step %.1f us" %
        (w.name, kv_avg * 1e3, min(kv_ms) * 1e3, mg_avg * 1e3, ms_per_step * 1e3))

    # Roofline of the dominant kernel (KV pass).  Its algorithmic bytes per launch: every K and V element
    # of prefix and tree once, plus q and the ids it reads (the output and lse belong to the merge pass).
    es = 4 if w.dtype == "f32" else 2
    kv_alg = alg_bytes - w.B * w.T * w.Hq * (w.D * es + 4)
    hbm_frac = kv_alg / (kv_avg * 1e-3) / 1e9 / HBM_PEAK_GBS
    mfma_frac = flops / (kv_avg * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS if w.dtype == "bf16" else 0.0
    return dict(w=w, plan=plan, n_pools=n_pools, ms_per_step=ms_per_step, kv_us=kv_avg * 1e3, merge_us=mg_avg * 1e3,
                alg_bytes=alg_bytes, kv_alg=kv_alg, flops=flops, hbm_frac=hbm_frac, mfma_frac=mfma_frac)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    # the GPU's clock needs about 0.1 s of uninterrupted load to settle: a short warm-up times a clock ramp instead
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
    from paper_2508_08192_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    ta.load_library()          # fails loudly if the HIP library is not built
    t0 = time.time()
    w = make(args.workload)
    log("workload %s generated in %.1f s" % (w.name, time.time() - t0))
    m = measure(w, args.steps, args.warmup, log, args.num_splits, args.kernel, args.rotate, args.check,
                args.item_cost)
    ms_per_step, kv_us, plan = m["ms_per_step"], m["kv_us"], m["plan"]
    alg_bytes, kv_alg, flops = m["alg_bytes"], m["kv_alg"], m["flops"]

    traffic = None
    # HBM bytes per KV-pass launch as counted by rocprofv3 (FETCH_SIZE + WRITE_SIZE, scaled by a copy of
    # known size); the counter runs are separate, their summary sits under profiles/.
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if os.path.exists(tpath):
        body = "".join(l for l in open(tpath) if not l.startswith("#"))
        traffic = json.loads(body).get(w.name, {}).get("kv_pass_bytes_per_launch")
    if m["hbm_frac"] >= m["mfma_frac"]:
        roof = {"bound": "hbm", "achieved": kv_alg / (kv_us * 1e-6) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": m["hbm_frac"], "traffic": traffic}
    else:
        roof = {"bound": "mfma", "achieved": flops / (kv_us * 1e-6) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": m["mfma_frac"], "traffic": traffic}
    roof.update({"kernel": "ta_generic_kv_kernel" if plan["kernel"] != 2 else "ta_mfma_sp_kernel",
                 "avg_launch_us": kv_us, "algorithmic_bytes_per_launch": kv_alg,
                 "useful_flops_per_launch": flops, "hbm_frac": m["hbm_frac"], "mfma_frac": m["mfma_frac"]})

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
        "tree_tokens_per_s": w.B * w.T / (ms_per_step * 1e-3),
        "kv_tokens_per_s": float(w.seq_lens.astype(np.int64).sum() + w.B * w.T) / (ms_per_step * 1e-3),
        "step_GBps": alg_bytes / (ms_per_step * 1e-3) / 1e9,
        "step_TFLOPs": flops / (ms_per_step * 1e-3) / 1e12,
        "step_frac_of_roofline": max(alg_bytes / 1e9 / HBM_PEAK_GBS, flops / 1e12 / MFMA_BF16_PEAK_TFLOPS) /
                                 (ms_per_step * 1e-3),
        "kernels_us": {"kv_pass": kv_us, "merge_pass": m["merge_us"]},
        "roofline": roof,
    }
    if args.cpu_seconds > 0:
        result["cpu_baseline"] = cpu_baseline(w, args.cpu_seconds, log)
    del m, w
    torch.cuda.empty_cache()
    if args.others:
        # the remaining configurations, briefly (context for the headline line; not separate bench lines)
        others = {}
        def brief(name):
            wo = make(name)
            mo = measure(wo, 100, 100, log)
            row = {"us_per_step": mo["ms_per_step"] * 1e3, "kv_pass_us": mo["kv_us"],
                   "merge_pass_us": mo["merge_us"], "hbm_frac": mo["hbm_frac"],
                   "mfma_frac": mo["mfma_frac"], "algorithmic_bytes": mo["alg_bytes"],
                   "useful_flops": mo["flops"]}
            del mo
            torch.cuda.empty_cache()
            return wo.name, row
        for name in sorted(WORKLOADS):
            if name != args.workload:
                k, v = brief(name)
                others[k] = v
        result["other_workloads"] = others
        result["production_shapes"] = dict(brief(name) for name in sorted(PRODUCTION) if name != args.workload)
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
