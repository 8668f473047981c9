#!/usr/bin/env python3
"""Benchmark of the prune-and-compact pass on one MI355X.

A step is one pass of the whole hot path over one synthetic network: the ranking for all
K prune counts of the workload, the threshold-and-mask pass fused with the zero-channel
scan, the group plan, and the gather rebuild of every variant.  Inputs are resident in
HBM before the timed region starts.  Prints ONE JSON line: the headline workload on top,
the other full-size workloads of the target under "other_workloads".

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5|c5p|c4|c2|c3|c1]
                  [--others c4,c5p | --others none] [--no-cpu-baseline] [--cpu-sample]
                  [--no-lean] [--codec-profile REPS]
"""
import argparse
import functools
import gc
import hashlib
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

_generated = {}


def generated(c):
    from paper_2309_06973_amd import synth
    if c not in _generated:
        _generated.clear()          # one large arena on the host at a time
        _generated[c] = synth.generate_config(c)
    return _generated[c]


def kernel_source_digest():
    """Digest of the sources of the pass's kernels: measured counter figures are only quoted
    while the kernels are the ones they were taken on (api.hip holds host code only;
    codec.hip holds the codec's kernels, for which no counter figure is quoted)."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2309_06973_amd", "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".h")) and name not in ("api.hip", "codec.hip"):
            with open(os.path.join(d, name), "rb") as f:
                h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def recorded_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed counter summary of `workload`
    (FETCH_SIZE and WRITE_SIZE, calibrated on the copy kernel), or None when there is no
    summary or the kernel sources have changed since it was taken."""
    path = os.path.join(ROOT, "profiles", f"{workload}_hbm_counters.txt")
    if not os.path.exists(path):
        return None
    digest, value = None, None
    with open(path) as f:
        for line in f:
            parts = line.split()
            if len(parts) == 2 and parts[0] == "kernel_source_digest:":
                digest = parts[1]
            if len(parts) == 3 and parts[0] == "traffic_bytes_per_launch:" and parts[1] == kernel:
                value = int(parts[2])
    return value if digest == kernel_source_digest() else None


def cpu_baselines(spec, w, v, sparsity, whole=True):
    """The oracle, as it stands, on the host: the whole workload, one variant (or, with
    whole=False, the leading layers up to ~120 M weights).  Beside it the faster CPU program
    (selection instead of a sort), on one core and on the host's cores."""
    import copy
    from oracle import shifter_oracle as O
    from oracle import fast_baseline as FB
    from paper_2309_06973_amd import synth
    host_cores = os.cpu_count() or 1
    if whole:
        tensors, groups, vecs = spec.tensors, spec.groups, spec.vecs
        tot = sum(t.numel for t in tensors)
        what = f"whole workload ({tot} weights in {len(tensors)} tensors)"
    else:
        n_t, tot = 0, 0
        for t in spec.tensors:
            if tot + t.numel > 120_000_000 and n_t > 0:
                break
            tot += t.numel
            n_t += 1
        tensors = copy.deepcopy(spec.tensors[:n_t])
        groups_used = max(max(t.out_group, t.in_group) for t in tensors) + 1
        groups = copy.deepcopy(spec.groups[:groups_used])
        vecs = [d for d in spec.vecs if d.group < groups_used]
        what = (f"a sample: the first {n_t} weight tensors of the workload ({tot} of "
                f"{sum(t.numel for t in spec.tensors)} weights), pruned at its own threshold")
    n_pr = sum(t.numel for t in tensors if t.prunable)
    p = synth.prune_count(n_pr, sparsity)
    t0 = time.perf_counter()
    r = O.prune_and_compact(w, v, tensors, vecs, groups, [p])[0]
    dt = time.perf_counter() - t0
    n2 = int(r.compacted.w.size)
    del r
    # bytes credited to one variant by the metric: ranking 4N, mask pass 9N, rebuild 8N'
    b_alg = 13 * n_pr + 8 * n2
    base = {"value": round(b_alg / dt / 1e9, 4), "unit": "GB/s", "cores": 1, "host_cores": host_cores,
            "kind": "oracle", "seconds": round(dt, 2), "variants_per_s": round(1.0 / dt, 4),
            "sample": f"{what}, one variant at s={sparsity:.4f}"}
    # the same through a CPU program that selects instead of sorting (checked against the
    # oracle by the tests): the figure to compare a GPU speed-up with
    t0 = time.perf_counter()
    out = FB.prune_and_compact_fast(w, v, tensors, vecs, groups, p)
    dt1 = time.perf_counter() - t0
    assert int(out[3].size) == n2
    del out
    threads = min(16, host_cores)
    t0 = time.perf_counter()
    out = FB.prune_and_compact_fast_mt(w, v, tensors, vecs, groups, p, threads)
    dtm = time.perf_counter() - t0
    assert int(out[3].size) == n2
    del out
    fast = {"value": round(b_alg / dtm / 1e9, 4), "unit": "GB/s", "cores": threads, "host_cores": host_cores,
            "kind": "selection by counting and partition, vectorised masks and gathers (numpy), "
                    "a thread pool over slabs and tensors",
            "seconds": round(dtm, 2), "variants_per_s": round(1.0 / dtm, 4),
            "one_core": {"value": round(b_alg / dt1 / 1e9, 4), "seconds": round(dt1, 2),
                         "kind": "selection by partition, vectorised masks and gathers (numpy)"},
            "sample": "the same workload and variant"}
    return base, fast


def without_gc(fn):
    """Runs fn with the interpreter's cyclic garbage collector off, as timeit does: one
    collection is about a millisecond of host time (two c5 steps) and falls wherever the
    allocation counters put it, inside one run's timed steps and outside the next's."""
    @functools.wraps(fn)
    def wrapped(*a, **kw):
        gc.collect()
        gc.disable()
        try:
            return fn(*a, **kw)
        finally:
            gc.enable()
    return wrapped


@without_gc
def measure(name, steps, warmup, lean_run=True, cpu_leg=True):
    """Times `steps` steps of one workload; returns the fields of its report."""
    import torch
    from paper_2309_06973_amd import shifter as S
    from paper_2309_06973_amd import synth
    from paper_2309_06973_amd.pipeline import Pipeline

    c, sparsities, desc = WORKLOADS[name]
    spec, w, v = generated(c)
    sparsities = sparsities or synth.config_sparsities(c)
    n = spec.n_prunable
    n_prune = [synth.prune_count(n, s) for s in sparsities]
    k_var = len(n_prune)
    pl = Pipeline(spec, w, v, device=0)
    if k_var > 1:
        pl.enable_batch(k_var)

    def step(collect=None, sparse_arenas=True):
        # one pair of calls per step: the library enqueues ranking, masks, scan, plans and
        # rebuilds for all prune counts and waits once
        _, out = pl.step(n_prune, 0, with_in_alive=True, sparse_arenas=sparse_arenas)
        if collect is not None:
            collect.extend(int(x) for x in out[3])

    # set-up: the HIP runtime finishes some one-time work (staging for device-to-host
    # copies among it) only after a few calls; keep that out of warm-up and timing
    kept = []
    for _ in range(6):
        step()
    # warm-up; the first one also records the (deterministic) compacted sizes
    step(kept)
    for _ in range(max(warmup - 1, 0)):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / steps * 1e3

    # algorithmic bytes of one step: ranking reads the arena once per portfolio (4N);
    # each variant reads 4N, writes 4N sparse + N mask, and moves 4N' in and 4N' out
    b_alg = 4 * n + sum(9 * n + 8 * n2 for n2 in kept)
    gbs = b_alg / (dt / steps) / 1e9
    # what this path has to move at the least: one variant rides the ranking on the mask
    # pass (9N + 8N'); a portfolio reads the arena once per pass over it (ranking and
    # masks: one fused pass or two), writes K sparse arenas and masks, and the rebuild
    # reads the dense arena once more for all variants and writes the survivors
    if k_var == 1:
        b_moved = 9 * n + 8 * kept[0]
    else:
        fused_batch = pl.model.info.w_extent * 4 > (192 << 20)      # pipeline.portfolio's choice
        b_moved = (4 * n) * (1 if fused_batch else 2) + 5 * n * k_var + 4 * n + 4 * sum(kept)

    # dominant kernel: HIP events around each launch, on the stream the kernels run on,
    # over a second timed run of the same steps
    S.shifter_profile_enable(pl.ctx, True)
    for _ in range(steps):
        step()
    prof = S.shifter_profile_read(pl.ctx)
    S.shifter_profile_enable(pl.ctx, False)
    # the kernel that reads the arena and writes the sparse arena and the mask: it must
    # move 4N + 4N + N bytes whether or not the ranking is fused into it; the batched
    # kernel reads the arena once and writes K sparse arenas and K masks
    if k_var == 1:
        dom = "spec_pass" if "spec_pass" in prof else "mask_scan"
        dom_bytes = 9 * n
    else:
        dom, dom_bytes = "mask_scan_batch", (4 + 5 * k_var) * n
    cnt, tot_ms = prof[dom]
    avg_ms = tot_ms / cnt
    achieved = dom_bytes / (avg_ms * 1e-3) / 1e9
    kernels = {kn: {"launches_per_step": c_ // steps,
                    "avg_us": round(ms / c_ * 1e3, 2),
                    "us_per_step": round(ms / steps * 1e3, 2)}
               for kn, (c_, ms) in sorted(prof.items(), key=lambda kv: -kv[1][1])}

    # plain copy kernel of the same arena: the bandwidth this chip sustains for a
    # read-once / write-once stream, and the known-size dispatch the memory-traffic
    # counters are calibrated against
    S.shifter_profile_enable(pl.ctx, True)
    for _ in range(5):
        S.shifter_copy_f32(pl.ctx, pl.d_w, pl.d_w_sparse, n)
    c_cnt, c_ms = S.shifter_profile_read(pl.ctx)["copy"]
    S.shifter_profile_enable(pl.ctx, False)
    copy_gbs = 8 * n / (c_ms / c_cnt * 1e-3) / 1e9

    # the same portfolio without materialising the K sparse arenas (masks, flags, plans
    # and rebuilt variants only): ranking 4N, one more read of the arena 4N, K masks, and
    # 8N'_k per rebuilt variant
    lean = None
    if k_var > 1 and lean_run:
        for _ in range(3):
            step(sparse_arenas=False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step(sparse_arenas=False)
        torch.cuda.synchronize()
        dt2 = (time.perf_counter() - t0) / steps
        b2 = 8 * n + sum(n + 8 * n2 for n2 in kept)
        b2_moved = (4 * n) * (1 if fused_batch else 2) + n * k_var + 4 * n + 4 * sum(kept)
        lean = {"ms_per_step": round(dt2 * 1e3, 4), "variants_per_s": round(k_var / dt2, 2),
                "credited_bytes_per_step": b2, "credited_gbs": round(b2 / dt2 / 1e9, 2),
                "credited_pct_hbm_peak": round(100.0 * b2 / dt2 / 1e9 / HBM_PEAK_GBS, 2),
                "bytes_moved_per_step": b2_moved,
                "moved_pct_hbm_peak": round(100.0 * b2_moved / dt2 / 1e9 / HBM_PEAK_GBS, 2)}

    # arenas that fit the last-level cache: the same step with the caches evicted before it
    # (a 1.5 GB buffer is rewritten between steps); the headline figure is back-to-back
    cold = None
    if lean_run and pl.model.info.w_extent * 4 <= (256 << 20):
        scratch = torch.zeros(3 << 27, dtype=torch.float32, device=pl.dev)
        tot = 0.0
        for it in range(steps + 2):
            scratch.add_(1.0)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            step()
            torch.cuda.synchronize()
            if it >= 2:
                tot += time.perf_counter() - t0
        dtc = tot / steps
        cold = {"ms_per_step": round(dtc * 1e3, 4), "credited_gbs": round(b_alg / dtc / 1e9, 2),
                "credited_pct_hbm_peak": round(100.0 * b_alg / dtc / 1e9 / HBM_PEAK_GBS, 2),
                "moved_pct_hbm_peak": round(100.0 * b_moved / dtc / 1e9 / HBM_PEAK_GBS, 2),
                "variants_per_s": round(k_var / dtc, 2)}
        del scratch

    # the liveness-fixpoint plan (kernel-level index + rounds + rebuild) on the same sparse
    # arena, for the single-variant workloads: what it costs and what it removes on top
    fixpoint = None
    if k_var == 1 and lean_run:
        step()                      # the copy above overwrote the sparse arena
        pl.kernel_scan()
        pl.propagate_groups_fixpoint(0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            pl.kernel_scan()
            _, _, rounds = pl.propagate_groups_fixpoint(0)
            fout = pl.compact(sync=True)
        torch.cuda.synchronize()
        dt3 = (time.perf_counter() - t0) / steps
        fixpoint = {"ms_per_step_scan_plan_rebuild": round(dt3 * 1e3, 4), "rounds": rounds,
                    "kept_weights": int(fout[3]), "kept_weights_single_pass": int(kept[0])}
        # the same with nothing read back before the rebuild's own wait (four batches of four
        # rounds enqueued, those after the fixpoint return at once)
        for _ in range(3):                   # the runtime's one-time work stays out of the timing
            pl.kernel_scan()
            pl.propagate_groups_fixpoint(0, sync=False)
            pl.compact(sync=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            pl.kernel_scan()
            pl.propagate_groups_fixpoint(0, sync=False)
            fout2 = pl.compact(sync=True)
        torch.cuda.synchronize()
        fixpoint["ms_per_step_one_wait"] = round((time.perf_counter() - t0) / steps * 1e3, 4)
        fixpoint["one_wait_rounds_settled"] = list(S.shifter_fixpoint_status(pl.ctx, pl.model))
        fixpoint["one_wait_same_result"] = int(fout2[3]) == int(fout[3])
        S.shifter_profile_enable(pl.ctx, True)
        for _ in range(5):
            pl.kernel_scan()
        ks = S.shifter_profile_read(pl.ctx)
        S.shifter_profile_enable(pl.ctx, False)
        ks_ms = ks["kernel_scan"][1] / ks["kernel_scan"][0]
        fixpoint["kernel_scan_us"] = round(ks_ms * 1e3, 2)
        fixpoint["kernel_scan_read_gbs"] = round(4 * n / (ks_ms * 1e-3) / 1e9, 1)

    # Module 1's conv + BatchNorm fold of the sparse arena: one read and one write of every
    # weight (8 bytes per weight), a streaming kernel of its own
    fold = None
    if k_var == 1 and lean_run:
        step()
        fspec, folds = synth.fused_spec(spec)
        dst = torch.empty_like(pl.d_w_sparse)
        pl.fold_bn(folds, fspec.v_elems, 1e-5, dst=dst)
        S.shifter_profile_enable(pl.ctx, True)
        for _ in range(5):
            pl.fold_bn(folds, fspec.v_elems, 1e-5, dst=dst)
        fp = S.shifter_profile_read(pl.ctx)
        S.shifter_profile_enable(pl.ctx, False)
        fa_ms = fp["fold_apply"][1] / fp["fold_apply"][0]
        fs_ms = fp["fold_scale"][1] / fp["fold_scale"][0]
        fbytes = 8 * spec.w_elems
        fold = {"fold_apply_us": round(fa_ms * 1e3, 2), "fold_scale_us": round(fs_ms * 1e3, 2),
                "bytes_per_launch": fbytes,
                "gbs": round(fbytes / (fa_ms * 1e-3) / 1e9, 1),
                "frac_of_peak": round(fbytes / (fa_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        del dst

    # Phase 3 codec on the sparse arena: deflate (Module 7) and inflate (Module 8); the
    # stream is a DEFLATE stream, the ratio is raw bytes over stream bytes
    codec = None
    if k_var == 1 and lean_run:
        from paper_2309_06973_amd.pipeline import Codec
        step()
        cd = Codec(device=0, ctx=pl.ctx)
        raw = pl.d_w_sparse[:spec.w_elems]
        n_raw = 4 * spec.w_elems
        stream_buf = torch.empty(S.shifter_codec_layout(n_raw)[2], dtype=torch.uint8, device=pl.dev)
        pkg = cd.deflate(raw, stream=stream_buf)
        back = cd.inflate(pkg)
        S.shifter_profile_enable(pl.ctx, True)
        for _ in range(5):
            pkg = cd.deflate(raw, stream=stream_buf)
            cd.inflate(pkg, out=back)
        cp = S.shifter_profile_read(pl.ctx)
        S.shifter_profile_enable(pl.ctx, False)
        avg = lambda kn: cp[kn][1] / cp[kn][0]
        enc_ms = avg("deflate_chunk") + avg("codec_scan") + avg("codec_pack")
        dec_ms = avg("inflate_chunk")
        moved = n_raw + pkg.stream_bytes           # bytes either direction has to move
        codec = {"raw_bytes": n_raw, "stream_bytes": pkg.stream_bytes,
                 "side_information_bytes": pkg.sub_bits.numel() * 2 + pkg.sub_marks.numel() * 8
                 + pkg.seg_off.numel() * 8,
                 "ratio": round(n_raw / pkg.stream_bytes, 3),
                 "round_trip_equal": bool(torch.equal(back[:n_raw].view(torch.int32),
                                                      raw.view(torch.int32))),
                 "deflate_us": round(enc_ms * 1e3, 1), "inflate_us": round(dec_ms * 1e3, 1),
                 "deflate_chunk_us": round(avg("deflate_chunk") * 1e3, 1),
                 "deflate_gbs": round(moved / (enc_ms * 1e-3) / 1e9, 1),
                 "inflate_gbs": round(moved / (dec_ms * 1e-3) / 1e9, 1),
                 "inflate_frac_of_peak": round(moved / (dec_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        # the compacted (structurally pruned) variant of the same step: what is left after
        # the zero filters and channels are gone still holds the zeros inside the survivors
        step()
        n_c = int(kept[0])
        comp = pl.d_w_out[:n_c]
        cbuf = torch.empty(S.shifter_codec_layout(4 * n_c)[2], dtype=torch.uint8, device=pl.dev)
        cpkg = cd.deflate(comp, stream=cbuf)
        cback = cd.inflate(cpkg)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(10):
            cd.inflate(cpkg, out=cback)
        torch.cuda.synchronize()
        t_inf = (time.perf_counter() - t0) / 10
        t0 = time.perf_counter()
        for _ in range(10):
            cd.deflate(comp, stream=cbuf)
        torch.cuda.synchronize()
        t_def = (time.perf_counter() - t0) / 10
        codec["compacted_variant"] = {
            "raw_bytes": 4 * n_c, "stream_bytes": cpkg.stream_bytes,
            "ratio": round(4 * n_c / cpkg.stream_bytes, 3),
            "round_trip_equal": bool(torch.equal(cback[:4 * n_c].view(torch.int32), comp.view(torch.int32))),
            "deflate_call_us": round(t_def * 1e6, 1), "inflate_call_us": round(t_inf * 1e6, 1)}
        del cbuf, cback, cpkg
        # the zlib library on one host core, on the first 64 MiB of the same bytes
        if cpu_leg:
            import zlib
            sample = raw[:(64 << 20) // 4].cpu().numpy().tobytes()
            t0 = time.perf_counter()
            z = zlib.compress(sample, 6)
            t1 = time.perf_counter()
            zlib.decompress(z)
            t2 = time.perf_counter()
            codec["zlib_level6_one_core"] = {
                "sample_bytes": len(sample), "ratio": round(len(sample) / len(z), 3),
                "deflate_gbs": round(len(sample) / (t1 - t0) / 1e9, 3),
                "inflate_gbs": round(len(sample) / (t2 - t1) / 1e9, 3)}
        del stream_buf, back, pkg, cd

    out = {
        "value": round(gbs, 2),
        "unit": "GB/s",
        "ms_per_step": round(ms_per_step, 4),
        "steps": steps,
        "config": {"workload": desc, "variants_per_step": k_var,
                   "sparsities": [round(s, 5) for s in sparsities],
                   "kept_weights": kept, "algorithmic_bytes_per_step": b_alg},
        # `value` credits every variant with its own ranking read and its own read of the
        # weights (the metric's definition); the path moves fewer bytes than that, so the
        # credited percentage is not a bandwidth and may pass 100.  The achieved figure is
        # the bytes really moved over the same time.
        "value_kind": "credited bytes (the metric's definition) / time",
        "credited_pct_hbm_peak": round(100.0 * gbs / HBM_PEAK_GBS, 2),
        "achieved_frac_moved": round(b_moved / (dt / steps) / 1e9 / HBM_PEAK_GBS, 4),
        "bytes_moved_per_step": b_moved,
        "moved_gbs": round(b_moved / (dt / steps) / 1e9, 2),
        "moved_pct_hbm_peak": round(100.0 * b_moved / (dt / steps) / 1e9 / HBM_PEAK_GBS, 2),
        "us_per_variant": round(dt / steps / k_var * 1e6, 2),
        "variants_per_s": round(k_var / (dt / steps), 2),
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 2),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": recorded_traffic(name, dom),
                     "bytes_per_launch": dom_bytes, "avg_launch_ms": round(avg_ms, 5)},
        "selection": S.shifter_get_select_stats(pl.ctx),
        "copy_kernel": {"bytes_per_launch": 8 * n, "gbs": round(copy_gbs, 1),
                        "frac_of_peak": round(copy_gbs / HBM_PEAK_GBS, 4)},
        "kernels": kernels,
    }
    if cold is not None:
        out["cold_cache"] = cold
    if lean is not None:
        out["without_sparse_arenas"] = lean
    if fixpoint is not None:
        out["liveness_fixpoint"] = fixpoint
    if fold is not None:
        out["conv_bn_fold"] = fold
    if codec is not None:
        out["codec"] = codec
    pl.close()
    del pl
    torch.cuda.empty_cache()
    return out, (spec, w, v, sparsities)


def codec_profile(name, reps):
    """For a kernel trace of the codec alone: deflates and inflates ONE buffer, the sparse
    arena of the workload's first variant, `reps` times; prints its own JSON line."""
    import torch
    from paper_2309_06973_amd import shifter as S
    from paper_2309_06973_amd import synth
    from paper_2309_06973_amd.pipeline import Codec, Pipeline
    c, sparsities, desc = WORKLOADS[name]
    spec, w, v = generated(c)
    s0 = (sparsities or synth.config_sparsities(c))[0 if sparsities else -1]
    pl = Pipeline(spec, w, v, device=0)
    pl.step([synth.prune_count(spec.n_prunable, s0)])
    cd = Codec(device=0, ctx=pl.ctx)
    raw = pl.d_w_sparse[:spec.w_elems]
    n_raw = 4 * spec.w_elems
    buf = torch.empty(S.shifter_codec_layout(n_raw)[2], dtype=torch.uint8, device=pl.dev)
    pkg = cd.deflate(raw, stream=buf)
    back = cd.inflate(pkg)
    S.shifter_profile_enable(pl.ctx, True)
    for _ in range(reps):
        pkg = cd.deflate(raw, stream=buf)
        cd.inflate(pkg, out=back)
    cp = S.shifter_profile_read(pl.ctx)
    ok = bool(torch.equal(back[:n_raw].view(torch.int32), raw.view(torch.int32)))
    print(json.dumps({"workload": desc, "sparsity": s0, "raw_bytes": n_raw, "stream_bytes": pkg.stream_bytes,
                      "side_information_bytes": pkg.sub_bits.numel() * 2 + pkg.sub_marks.numel() * 8
                      + pkg.seg_off.numel() * 8, "round_trip_equal": ok, "reps": reps,
                      "avg_us": {k: round(ms / n * 1e3, 1) for k, (n, ms) in cp.items()}}))
    pl.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c5", choices=sorted(WORKLOADS))
    ap.add_argument("--others", default=None,
                    help="comma-separated workloads also measured (default: c5p,c4 with "
                         "the default workload, none otherwise)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", action="store_true",
                    help="time the CPU programs on the leading ~120 M weights instead of the "
                         "whole workload")
    ap.add_argument("--no-lean", action="store_true",
                    help="skip the extra timings (portfolio without sparse arenas, liveness "
                         "fixpoint): for profiling runs")
    ap.add_argument("--codec-profile", type=int, default=0, metavar="REPS",
                    help="only deflate and inflate the workload's sparse arena REPS times (one "
                         "input size; for a kernel trace of the codec)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU only; --gpus must be 1 (the pass "
              "shards by variant or by arena range, but no multi-GPU path is built)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2309_06973_amd import shifter as S

    if not torch.cuda.is_available():
        print("bench.py: no ROCm device visible", file=sys.stderr)
        sys.exit(1)
    if not os.path.exists(S._LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()

    if args.codec_profile:
        codec_profile(args.workload, args.codec_profile)
        return

    if args.others is None:
        others = ["c5p", "c4"] if args.workload == "c5" else []
    else:
        others = [o for o in args.others.split(",") if o and o != "none"]
    for o in others:
        if o not in WORKLOADS:
            ap.error(f"unknown workload {o!r}")

    main_out, (spec, w, v, sparsities) = measure(args.workload, args.steps, args.warmup,
                                                  not args.no_lean, not args.no_cpu_baseline)
    cpu = cpu_fast = None
    if not args.no_cpu_baseline:
        cpu, cpu_fast = cpu_baselines(spec, w, v, sparsities[-1], whole=not args.cpu_sample)
        moved_gbs = main_out["moved_gbs"]
        cpu["gpu_moved_gbs_over_this"] = round(moved_gbs / cpu["value"], 1)
        cpu_fast["gpu_moved_gbs_over_this"] = round(moved_gbs / cpu_fast["value"], 1)
    del spec, w, v

    out = {
        "metric": "prune+compact GB/s and % of HBM peak; variants/sec per portfolio",
        "value": main_out.pop("value"),
        "unit": main_out.pop("unit"),
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": main_out.pop("ms_per_step"),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "fp32",
        "data": "synthetic",
    }
    main_out.pop("steps")
    out.update(main_out)
    if cpu is not None:
        out["cpu_baseline"] = cpu
        out["cpu_fast_baseline"] = cpu_fast
    if others:
        # same measurement, same fields, for the other full-size workloads; keyed by name,
        # sorted so that workloads sharing an arena are generated once
        out["other_workloads"] = {}
        for o in sorted(others, key=lambda o: (WORKLOADS[o][0] != WORKLOADS[args.workload][0], o)):
            res, _ = measure(o, args.steps, args.warmup, not args.no_lean)
            out["other_workloads"][o] = res
    print(json.dumps(out))


if __name__ == "__main__":
    main()
