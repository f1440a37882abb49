#!/usr/bin/env python3
"""Benchmark of the whole verification path on one MI355X.

A step is one mpv_verify call (statistics, residual masses, walk, bonus sample)
over one batch of the benchmark workload, inputs resident in HBM.  Prints one
JSON line: nodes verified per second, plus the roofline of the dominant kernel
(measured with HIP events recorded by the library around each of its launches)
and the fp64 CPU oracle timed on a bounded sample of the same workload.
"""

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X published peak
METHOD_LABEL = {0: "SpecInfer", 1: "Traversal", 2: "NSS", 3: "Naive", 4: "SpecTr"}


def kernel_source_digest():
    """sha256 over the HIP sources the library is built from: a counter summary under
    profiles/ says which sources it was measured on."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2602_16994_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        with open(os.path.join(csrc, name), "rb") as f:
            h.update(name.encode())
            h.update(f.read())
    return h.hexdigest()[:16]


def parse_profile_traffic(path):
    """HBM bytes per launch of the dominant kernel from the committed counter summary
    (key = value lines): (bytes or None, provenance).  A summary measured on other kernel
    sources than the ones in the tree is stale: its figure is not reported."""
    prov = {"file": os.path.relpath(path, ROOT), "status": "missing"}
    try:
        vals = {}
        with open(path) as f:
            for line in f:
                if "=" in line and not line.lstrip().startswith("#"):
                    k, v = line.split("=", 1)
                    vals[k.strip()] = v.strip()
        traffic = float(vals["hbm_bytes_per_launch"])
    except Exception:
        return None, prov
    prov["measured_on_sources"] = vals.get("kernel_sources_sha256_16")
    prov["sources_now"] = kernel_source_digest()
    if prov["measured_on_sources"] != prov["sources_now"]:
        prov["status"] = "stale: the kernel sources have changed since the counters were read"
        return None, prov
    prov["status"] = "current"
    return traffic, prov


def cpu_baseline(cfg, inputs, method, budget_s=15.0):
    """The oracle, as it stands, on every host core this box gives a GPU job: one worker
    process per core (spawned; each imports numpy and the oracle only), each verifying one
    tree of the batch in sample mode over and over for `budget_s` seconds."""
    import multiprocessing as mp
    import bench_cpu_worker
    cores = max(1, min(16, os.cpu_count() or 1, cfg.B))       # a one-GPU machine's CPU share is 16 cores
    jobs = []
    for b in range(cores):
        jobs.append((method, list(inputs["parent"]),
                     inputs["tokens"][b].cpu().numpy(),
                     inputs["target"][b].float().cpu().numpy(),
                     inputs["draft"][b].float().cpu().numpy(),
                     cfg.T,
                     inputs["uniforms"][b].cpu().numpy(),
                     inputs["draw_uniforms"][b].cpu().numpy(),
                     budget_s))
    ctx = mp.get_context("spawn")
    t0 = time.perf_counter()
    with ctx.Pool(processes=cores) as pool:
        results = pool.map(bench_cpu_worker.verify_repeatedly, jobs, chunksize=1)
    wall = time.perf_counter() - t0
    trees = sum(r[0] for r in results)
    busy = max(r[1] for r in results)
    print(f"[bench] cpu baseline: {cores} worker processes, {trees} trees in {busy:.1f} s "
          f"({wall:.1f} s with start-up)", file=sys.stderr)
    return {
        "value": trees * cfg.N / busy,
        "unit": "nodes/s",
        "cores": cores,
        "kind": "oracle",
        "sample": f"{cores} worker processes (one per core), each verifying one tree of the same batch "
                  f"(trees 0..{cores - 1}) repeatedly in sample mode for {budget_s:.0f} s: {trees} trees in {busy:.1f} s",
    }


def other_configs(mpv, torch, workloads, skip, steps=10):
    """The remaining benchmark configurations, each with the rules it is quoted with: time per
    call, nodes per second, and the node-task kernel's algorithmic bytes over the whole call
    time (a lower bound of the kernel's own figure: the call also holds the set-up kernel)."""
    res = {}
    for name, cfg in workloads.CONFIGS.items():
        if name == skip:
            continue
        inp = workloads.make_inputs(cfg, "cuda:0")
        pair_bytes = 2 * cfg.V * cfg.elem_bytes
        entry = {"B": cfg.B, "N": cfg.N, "V": cfg.V, "logit_dtype": cfg.dtype, "methods": {}}
        for method in cfg.methods:
            def call(out=None):
                return mpv.mpv_verify(inp["parent"], inp["tokens"], inp["target"], inp["draft"], cfg.T,
                                      inp["uniforms"], method, debug=False, out=out,
                                      draw_uniforms=inp["draw_uniforms"])
            out = call()
            for _ in range(3):
                call(out)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                call(out)
            torch.cuda.synchronize()
            sec = (time.perf_counter() - t0) / steps
            counters = out.counters.tolist()
            if counters[4] != 0:
                raise RuntimeError(f"{name}/{METHOD_LABEL[method]}: {counters[4]} dependency timeouts")
            gbs = counters[5] * pair_bytes / sec / 1e9
            entry["methods"][METHOD_LABEL[method]] = {
                "ms_per_step": sec * 1e3, "nodes_per_s": cfg.B * cfg.N / sec, "node_tasks_run": counters[5],
                "algorithmic_GBps": gbs, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS,
                "mean_accept_len": float(out.accept_len.float().mean().item())}
        res[name] = entry
        del inp
        torch.cuda.empty_cache()
    return res


def merged_trees(mpv, torch, workloads, names=("v128k_delayed", "v152k_root"), steps=3):
    """mpv_verify_merged (draft trees whose nodes are distinct contexts, Def. 3.1) on batches whose
    rows are functions of the context: time per call with the trees as drafted and with trees of
    equal shape laid next to each other (one launch per run of equal shapes), next to the plain call
    on the same batch, and what merging does to the accepted length."""
    import numpy as np
    res = {}
    for name in names:
        cfg = workloads.CONFIGS[name]
        inp = workloads.make_context_inputs(cfg, "cuda:0")
        merged_parent, context_node = mpv.mpv_merge_duplicates(cfg.parent, inp["tokens"].cpu().numpy())
        order = sorted(range(cfg.B), key=lambda b: tuple(merged_parent[b]))
        entry = {"B": cfg.B, "N": cfg.N, "V": cfg.V,
                 "slots_that_repeat_a_context": int((context_node != np.arange(cfg.N)).sum()),
                 "distinct_shapes": len({tuple(r) for r in merged_parent.tolist()}), "methods": {}}

        def runs(rows):
            return 1 + sum(1 for b in range(1, len(rows)) if not np.array_equal(rows[b], rows[b - 1]))

        for method in cfg.methods:
            def timed(batch, rows):
                def call(out=None):
                    return mpv.mpv_verify(batch["parent"], batch["tokens"], batch["target"], batch["draft"], cfg.T,
                                          batch["uniforms"], method, debug=False, out=out,
                                          draw_uniforms=batch["draw_uniforms"], merged_parent=rows)
                out = call()
                call(out)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(steps):
                    call(out)
                torch.cuda.synchronize()
                sec = (time.perf_counter() - t0) / steps
                if out.counters.tolist()[4] != 0:
                    raise RuntimeError(f"merged {name}/{METHOD_LABEL[method]}: dependency timeouts")
                return sec, out
            sec_plain, out_plain = timed(inp, None)
            sec_drafted, out_merged = timed(inp, merged_parent)
            moved = workloads.reorder_trees(inp, order)
            sec_sorted, _ = timed(moved, merged_parent[order])
            del moved
            entry["methods"][METHOD_LABEL[method]] = {
                "plain_call_ms": sec_plain * 1e3,
                "merged_as_drafted": {"launches": runs(merged_parent), "ms_per_step": sec_drafted * 1e3},
                "merged_sorted_by_shape": {"launches": runs(merged_parent[order]), "ms_per_step": sec_sorted * 1e3},
                "mean_accept_len_plain": float(out_plain.accept_len.float().mean().item()),
                "mean_accept_len_merged": float(out_merged.accept_len.float().mean().item())}
        res[name] = entry
        del inp
        torch.cuda.empty_cache()
    return res


def side_measurements(mpv, torch, cfg, inputs, method, pair_bytes, steps=5):
    """Two reference points for the roofline, outside the timed region.
    every_node_task: the same call with the per-node test probabilities requested, which makes the
    library run the task of every internal node instead of only those the rule needs.
    acceptance_rates: mpv_acceptance_rates (App. C) for every internal node.
    nucleus_mask_top_p_0.9: mpv_nucleus_mask over every target row of the batch (out of place).
    block_efficiency_estimate: mpv_block_efficiency (expected accepted length + 1 of every tree, no sampling).
    softmax_statistics_only: step S2 alone (mpv_row_stats) over every target row of the batch."""
    def timed(fn):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    res = {}
    kw = dict(draw_uniforms=inputs["draw_uniforms"])
    out = mpv.mpv_verify(inputs["parent"], inputs["tokens"], inputs["target"], inputs["draft"],
                         cfg.T, inputs["uniforms"], method, debug=False, **kw)
    out.accept_prob = torch.empty(cfg.B, cfg.N, dtype=torch.float32, device=inputs["target"].device)
    s = timed(lambda: mpv.mpv_verify(inputs["parent"], inputs["tokens"], inputs["target"], inputs["draft"],
                                     cfg.T, inputs["uniforms"], method, debug=False, out=out, **kw))
    tasks = out.counters.tolist()[5]
    gbs = tasks * pair_bytes / s / 1e9
    res["every_node_task"] = {"ms_per_step": s * 1e3, "node_tasks_run": tasks,
                              "algorithmic_GBps": gbs, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS}
    be = mpv.mpv_block_efficiency(inputs["parent"], inputs["tokens"], inputs["target"], inputs["draft"], cfg.T, method)
    s = timed(lambda: mpv.mpv_block_efficiency(inputs["parent"], inputs["tokens"], inputs["target"],
                                               inputs["draft"], cfg.T, method, out=be))
    tasks = be.counters.tolist()[5]
    gbs = tasks * pair_bytes / s / 1e9
    res["block_efficiency_estimate"] = {"ms_per_step": s * 1e3, "node_tasks_run": tasks,
                                        "mean_expected_block_efficiency": float(be.expected.mean().item()),
                                        "algorithmic_GBps": gbs, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS}
    solver = method if method != 1 else 0               # Traversal is not an OTLP solver: time SpecInfer's rates
    s = timed(lambda: mpv.mpv_acceptance_rates(inputs["parent"], inputs["target"], inputs["draft"], cfg.T, solver))
    alpha, cnt = mpv.mpv_acceptance_rates(inputs["parent"], inputs["target"], inputs["draft"], cfg.T, solver)
    tasks = cnt.tolist()[5]
    gbs = tasks * pair_bytes / s / 1e9
    res["acceptance_rates"] = {"ms_per_step": s * 1e3, "solver": METHOD_LABEL[solver], "node_tasks_run": tasks,
                               "mean_rate_at_the_root": float(alpha[:, 0].mean().item()),
                               "algorithmic_GBps": gbs, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS}
    rows = inputs["target"].view(cfg.B * cfg.N, cfg.V)
    masked = torch.empty_like(rows)
    s = timed(lambda: mpv.mpv_nucleus_mask(rows, cfg.T, 0.9, out=masked))
    gbs = 2 * rows.numel() * rows.element_size() / s / 1e9          # read once, written once
    res["nucleus_mask_top_p_0.9"] = {"ms_per_step": s * 1e3, "rows": cfg.B * cfg.N,
                                     "algorithmic_GBps": gbs, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS}
    del masked
    st = mpv.mpv_row_stats(rows, cfg.T)
    s = timed(lambda: mpv.mpv_row_stats(rows, cfg.T, out=st))
    gbs = rows.numel() * rows.element_size() / s / 1e9
    res["softmax_statistics_only"] = {"ms_per_step": s * 1e3, "rows": cfg.B * cfg.N,
                                      "algorithmic_GBps": gbs, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS}
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="v152k_root")
    ap.add_argument("--method", default=None,
                    help="specinfer | traversal | nss | naive | spectr (default: the workload's)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-launch-timing", action="store_true",
                    help="do not bracket the library's launches with HIP events")
    ap.add_argument("--no-extra", action="store_true",
                    help="skip the two side measurements (every node task run; softmax statistics alone)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (a known-size kernel to scale profiler byte counters by)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (trees are independent: a batch shards by trees, with "
              "nothing to exchange); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2602_16994_amd as mpv
    import workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = workloads.CONFIGS[args.workload]
    if args.method is None:
        method = cfg.methods[-1]
    else:
        method = {"specinfer": 0, "traversal": 1, "nss": 2, "naive": 3, "spectr": 4}[args.method]
    inputs = workloads.make_inputs(cfg, "cuda:0")
    torch.cuda.synchronize()

    def step(out=None):
        return mpv.mpv_verify(inputs["parent"], inputs["tokens"], inputs["target"], inputs["draft"],
                              cfg.T, inputs["uniforms"], method, debug=False, out=out,
                              draw_uniforms=inputs["draw_uniforms"])

    if args.calibration_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)                     # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    out = step()
    for _ in range(args.warmup):
        step(out)
    torch.cuda.synchronize()

    launches_per_step = 8
    timing = not args.no_launch_timing
    if timing:
        mpv.mpv_timing_enable(launches_per_step * args.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(out)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    per_kernel = {}
    if timing:
        for kid, ms in mpv.mpv_timing_read(launches_per_step * args.steps):
            per_kernel.setdefault(mpv.MPV_KERNEL_NAMES[kid], []).append(ms)
        mpv.mpv_timing_enable(0)

    # ---- roofline of the dominant kernel (node tasks).  Algorithmic bytes: one read of the
    # target and the draft row of every (tree, internal node) whose rows the rule needs,
    # i.e. the tasks the kernel counted as run (Traversal proves the others irrelevant:
    # a node of weight 0 can neither be accepted nor pass weight on).
    n_internal = sum(1 for n in range(cfg.N) if n in set(cfg.parent[1:]))
    pair_bytes = 2 * cfg.V * cfg.elem_bytes                  # one target + one draft row
    counters = out.counters.tolist()
    tasks_run = counters[5]
    roofline = None
    kernels = {}
    if per_kernel:
        for name, v in per_kernel.items():
            kernels[name] = {"launches_per_step": len(v) / args.steps,
                             "avg_ms": sum(v) / len(v), "median_ms": sorted(v)[len(v) // 2], "min_ms": min(v),
                             "ms_per_step": sum(v) / args.steps}
        nt = per_kernel.get("node_task", [])
        if nt:
            launches = len(nt) / args.steps
            alg_bytes_per_launch = tasks_run * pair_bytes / launches
            avg_s = sum(nt) / len(nt) * 1e-3
            achieved = alg_bytes_per_launch / avg_s / 1e9
            traffic, traffic_provenance = parse_profile_traffic(os.path.join(
                ROOT, "profiles", f"node_task_{cfg.name}_pmc.txt"))
            roofline = {"bound": "hbm", "kernel": "node_task_kernel", "achieved": achieved,
                        "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                        "traffic": traffic,
                        # where the figure comes from (rocprofv3 counters, read in a run of their own)
                        "traffic_provenance": traffic_provenance,
                        # the counted bytes (profiles/) over the launch time measured here
                        "traffic_GBps": None if traffic is None else traffic / avg_s / 1e9,
                        "traffic_frac": None if traffic is None else traffic / avg_s / 1e9 / HBM_PEAK_GBS,
                        "algorithmic_bytes_per_launch": alg_bytes_per_launch,
                        "node_tasks_run": tasks_run, "node_tasks_total": cfg.B * n_internal,
                        "bytes_per_node_task": pair_bytes,
                        "avg_launch_ms": avg_s * 1e3, "launches_per_step": launches}

    if counters[4] != 0:
        # a wait inside the kernels ran into its time limit: the results of this run are invalid
        raise RuntimeError(f"bench.py: {counters[4]} dependency timeouts reported by the library")
    nodes_per_s = cfg.B * cfg.N / (ms_per_step * 1e-3)
    result = {
        "metric": "draft-tree nodes verified/sec",
        "value": nodes_per_s,
        "unit": "nodes/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B={cfg.B} trees, V={cfg.V}, "
                               f"{'root' if cfg.L1 == 0 else 'delayed'} expansion K={cfg.K} L1={cfg.L1} L2={cfg.L2} "
                               f"({cfg.N} nodes/tree), {cfg.dtype} logits, T={cfg.T}, "
                               f"{METHOD_LABEL[method]} verification",
                   "method": {0: "specinfer", 1: "traversal", 2: "nss", 3: "naive", 4: "spectr"}[method],
                   "logit_dtype": cfg.dtype},
        "trees_per_s": cfg.B / (ms_per_step * 1e-3),
        "mean_accept_len": float(out.accept_len.float().mean().item()),
        "counters": counters,
        "kernels": kernels,
        "roofline": roofline,
    }
    if not args.no_extra:
        result["also_measured"] = side_measurements(mpv, torch, cfg, inputs, method, pair_bytes)
        result["also_measured"]["configs"] = other_configs(mpv, torch, workloads, cfg.name)
        result["also_measured"]["merged_trees"] = merged_trees(mpv, torch, workloads)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, inputs, method)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
