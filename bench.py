#!/usr/bin/env python3
"""Benchmark of the prune-and-compact pass on one MI355X.

A step is one pass of the whole hot path over one synthetic network: one ranking call
for all K prune counts of the workload, then per variant: threshold-and-mask fused with
the zero-channel scan, the group plan, and the gather rebuild.  Inputs are resident in
HBM before the timed region starts.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5|c5p|c4|c2|c3|c1]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak

WORKLOADS = {
    # name: (config id, sparsities or None for the config's own schedule, description)
    "c5": (5, [0.95], "wide VGG-19 x4 (N=322,329,344), single sweep s=0.95"),
    "c5p": (5, None, "wide VGG-19 x4 (N=322,329,344), 10-variant portfolio s_k=1-0.8^k"),
    "c4": (4, None, "ResNet-50-shaped (N=25,502,912), 20-variant portfolio s_k=1-0.8^k"),
    "c3": (3, None, "ResNet-56-shaped (N=851,504), 15-variant portfolio"),
    "c2": (2, None, "VGG-16-shaped (N=14,715,584), 10-variant portfolio"),
    "c1": (1, None, "tiny CNN (N=24,112), s=0.9"),
}


def cpu_baseline_sample(spec, w, v, sparsity):
    """The oracle, as it stands, on a bounded sample of the workload: the leading layers
    of the network up to ~40 M weights (same values), one variant."""
    import copy
    import numpy as np
    from oracle import shifter_oracle as O
    from paper_2309_06973_amd import synth
    n_t, tot = 0, 0
    for t in spec.tensors:
        if tot + t.numel > 40_000_000 and n_t > 0:
            break
        tot += t.numel
        n_t += 1
    tensors = copy.deepcopy(spec.tensors[:n_t])
    groups_used = max(max(t.out_group, t.in_group) for t in tensors) + 1
    groups = copy.deepcopy(spec.groups[:groups_used])
    vecs = [d for d in spec.vecs if d.group < groups_used]
    p = synth.prune_count(tot, sparsity)
    t0 = time.perf_counter()
    r = O.prune_and_compact(w, v, tensors, vecs, groups, [p])[0]
    dt = time.perf_counter() - t0
    n2 = int(r.compacted.w.size)
    b_alg = 13 * tot + 8 * n2
    return {"value": round(b_alg / dt / 1e9, 4), "unit": "GB/s", "cores": 1,
            "kind": "oracle",
            "sample": f"first {n_t} weight tensors of the workload ({tot} weights), one "
                      f"variant at s={sparsity:.4f}; {dt:.2f} s; "
                      f"{1.0 / dt:.4f} variants/s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c5", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus must be 1 (the pass "
              "shards by variant or by arena range, see DESIGN.md, but no multi-GPU path "
              "is built)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2309_06973_amd import shifter as S
    from paper_2309_06973_amd import synth
    from paper_2309_06973_amd.pipeline import Pipeline

    if not torch.cuda.is_available():
        print("bench.py: no ROCm device visible", file=sys.stderr)
        sys.exit(1)
    if not os.path.exists(S._LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()

    c, sparsities, desc = WORKLOADS[args.workload]
    spec, w, v = synth.generate_config(c)
    sparsities = sparsities or synth.config_sparsities(c)
    n = spec.n_prunable
    n_prune = [synth.prune_count(n, s) for s in sparsities]
    k_var = len(n_prune)
    pl = Pipeline(spec, w, v, device=0)
    if k_var > 1:
        pl.enable_batch(k_var)

    def step(collect=None):
        if k_var == 1:
            # one prune count: ranking, mask and scan in a single read of the arena
            pl.prune_fused(n_prune[0])
            pl.propagate_groups(0, sync=False)
            out = pl.compact(sync=True)
            if collect is not None:
                collect.append(out[3])
            return
        # a portfolio: one ranking call for all counts, then one batched call per step
        _, out = pl.portfolio(n_prune, 0, with_in_alive=True, sync=True)
        if collect is not None:
            collect.extend(int(x) for x in out[3])

    # set-up: the HIP runtime finishes some one-time work (staging for device-to-host
    # copies among it) only after a few calls; keep that out of warm-up and timing
    kept = []
    for _ in range(6):
        step()
    # warm-up; the first one also records the (deterministic) compacted sizes
    step(kept)
    for _ in range(max(args.warmup - 1, 0)):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    # algorithmic bytes of one step: ranking reads the arena once per portfolio (4N);
    # each variant reads 4N, writes 4N sparse + N mask, and moves 4N' in and 4N' out
    b_alg = 4 * n + sum(9 * n + 8 * n2 for n2 in kept)
    gbs = b_alg / (dt / args.steps) / 1e9

    # dominant kernel (threshold-and-mask + scan): HIP events around each launch, on the
    # stream the kernels run on, over a second timed run of the same steps
    S.shifter_profile_enable(pl.ctx, True)
    for _ in range(args.steps):
        step()
    prof = S.shifter_profile_read(pl.ctx)
    S.shifter_profile_enable(pl.ctx, False)
    # the kernel that reads the arena and writes the sparse arena and the mask: it must move
    # 4N + 4N + N bytes whether or not the ranking is fused into it
    # (the batched kernel reads the arena once and writes K sparse arenas and K masks)
    if k_var == 1:
        dom = "spec_pass" if "spec_pass" in prof else "mask_scan"
        dom_bytes = 9 * n
    else:
        dom, dom_bytes = "mask_scan_batch", (4 + 5 * k_var) * n
    cnt, tot_ms = prof[dom]
    avg_ms = tot_ms / cnt
    achieved = dom_bytes / (avg_ms * 1e-3) / 1e9
    kernels = {name: {"launches_per_step": c_ // args.steps,
                      "avg_us": round(ms / c_ * 1e3, 2),
                      "us_per_step": round(ms / args.steps * 1e3, 2)}
               for name, (c_, ms) in sorted(prof.items(), key=lambda kv: -kv[1][1])}

    # plain copy kernel of the same arena: the bandwidth this chip sustains for a
    # read-once / write-once stream, and the known-size dispatch the memory-traffic
    # counters are calibrated against
    S.shifter_profile_enable(pl.ctx, True)
    for _ in range(5):
        S.shifter_copy_f32(pl.ctx, pl.d_w, pl.d_w_sparse, n)
    c_cnt, c_ms = S.shifter_profile_read(pl.ctx)["copy"]
    S.shifter_profile_enable(pl.ctx, False)
    copy_gbs = 8 * n / (c_ms / c_cnt * 1e-3) / 1e9

    out = {
        "metric": "prune+compact GB/s and % of HBM peak; variants/sec per portfolio",
        "value": round(gbs, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32",
        "data": "synthetic",
        "config": {"workload": desc, "variants_per_step": k_var,
                   "sparsities": [round(s, 5) for s in sparsities],
                   "kept_weights": kept, "algorithmic_bytes_per_step": b_alg},
        "pct_hbm_peak": round(100.0 * gbs / HBM_PEAK_GBS, 2),
        "variants_per_s": round(k_var / (dt / args.steps), 2),
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 2),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                     "bytes_per_launch": dom_bytes, "avg_launch_ms": round(avg_ms, 5)},
        "selection": S.shifter_get_select_stats(pl.ctx),
        "copy_kernel": {"bytes_per_launch": 8 * n, "gbs": round(copy_gbs, 1),
                        "frac_of_peak": round(copy_gbs / HBM_PEAK_GBS, 4)},
        "kernels": kernels,
    }
    pl.close()
    del pl
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_sample(spec, w, v, sparsities[-1])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
