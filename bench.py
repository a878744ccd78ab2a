"""Benchmark of the GRAT attention hot path on one MI355X.

One step = build the per-group KV block lists + one grat_attention_fwd over the workload
(Q, K, V resident in HBM).  Prints ONE JSON line.

    python bench.py [--steps K] [--warmup W] [--workload img8192] [--pattern B3]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

BF16_MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak


def measured_traffic(workload, pattern):
    """HBM bytes per attention launch from the committed rocprofv3 counter summary, if there is one
    for this workload (profiles/attn_mfma_<workload>_<pattern>.md, line 'traffic_bytes_per_launch: N')."""
    path = os.path.join(ROOT, "profiles", f"attn_mfma_{workload}_{pattern}.md")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def kernel_name(w, n_g, n_glob, pattern, radius):
    """The instantiation the library launches for this workload (its rules, restated): template arguments
    = waves per workgroup, keys per LDS tile, mode (0 grouped, 2 joint, 3 grid the group does not divide),
    half?, head_dim."""
    import numpy as np
    import paper_2505_14687_amd as grat
    groups = int(np.prod([-(-t // g) for t, g in zip(w.grid, w.group)]))
    waves = 8 if n_g % 256 == 0 else (4 if n_g % 128 == 0 else 2)
    if waves == 8 and w.batch * w.heads * groups < 512:
        waves = 4
    ragged = any(t % g for t, g in zip(w.grid, w.group))
    mode = 2 if n_glob else (3 if ragged else 0)
    max_kv = grat.grat_block_list_shape(w.grid, w.group, pattern, radius)[1]
    keys = 32 if waves == 2 and mode != 2 and max_kv * n_g <= 4096 else 64
    return "grat::attn_mfma_kernel<%d, %d, %d, %s, %d>" % (waves, keys, mode, "true" if w.dtype == "f16" else "false", w.head_dim)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="img8192")
    ap.add_argument("--pattern", default="B3")
    ap.add_argument("--no-dense", action="store_true", help="skip the dense comparison launch")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-others", action="store_true", help="skip the workload's other patterns")
    ap.add_argument("--no-probe", action="store_true", help="skip the MFMA-only probe")
    ap.add_argument("--constant-data", action="store_true",
                    help="context run, not the benchmark: Q = K = V = 1.0 everywhere (same launches, same "
                         "traffic; shows how far the chip's clock under toggling data holds the kernel back); "
                         "implies --no-cpu")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--n-global", type=int, default=0,
                    help="prompt tokens ahead of the grid tokens (joint sequence, grat_attention_global_fwd)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build measures one GPU only (heads shard across GPUs with no "
                 "exchange inside attention, so the one-GPU figure is the per-GPU figure). Run with --gpus 1.")

    import numpy as np
    import torch

    import paper_2505_14687_amd as grat
    from paper_2505_14687_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    w = synth.WORKLOADS[args.workload]
    pattern, radius = w.patterns[args.pattern]
    n_g = int(np.prod(w.group))

    t0 = time.time()
    n_glob = args.n_global
    n_seq = n_glob + w.n_tokens
    host = synth.make_qkv(w.batch, w.heads, n_seq, w.head_dim, w.dtype, w.seed, threads=16)
    def dev(x):
        if x.dtype == np.uint16:
            return torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(x).cuda()
    Q, K, V = (dev(x) for x in host)
    if args.constant_data:
        args.no_cpu = True
        for t in (Q, K, V):
            t.fill_(1.0)
    O = torch.empty_like(Q)
    # one plain device copy of known size (Q -> O) ahead of everything: the reference against which
    # the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run of this script are scaled
    O.copy_(Q)
    torch.cuda.synchronize()
    log(f"inputs: {args.workload} {tuple(Q.shape)} {w.dtype} generated+uploaded in {time.time() - t0:.1f}s")

    def flops_of(kv_count):
        # grid query: its groups' tokens + every prompt token; prompt query: the whole sequence
        pairs = int(kv_count.sum().item()) * n_g * n_g + n_glob * w.n_tokens + n_glob * n_seq
        return 4.0 * w.head_dim * w.heads * w.batch * pairs, pairs

    def attention(count, index):
        if n_glob:
            grat.grat_attention_global_fwd(Q, K, V, w.scale, n_glob, True, w.grid, w.group, count, index, out=O)
        else:
            grat.grat_attention_fwd(Q, K, V, w.scale, w.grid, w.group, count, index, out=O)

    def step(pat, rad):
        count, index = grat.grat_build_block_lists(w.grid, w.group, pat, rad)
        return count, index

    def time_pattern(pat, rad, steps, warmup):
        """W warm-up steps, then exactly K timed steps between synchronisations; the attention
        launch of every timed step is also bracketed by events on the launch stream."""
        for _ in range(warmup):
            count, index = step(pat, rad)
            attention(count, index)
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        t0 = time.perf_counter()
        for i in range(steps):
            count, index = step(pat, rad)
            evs[i][0].record()
            attention(count, index)
            evs[i][1].record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / steps
        kern_ms = [a.elapsed_time(b) for a, b in evs]
        fl, pairs = flops_of(count)
        return {"ms_per_step": wall_ms, "attn_kernel_ms_avg": float(np.mean(kern_ms)),
                "attn_kernel_ms_min": float(np.min(kern_ms)), "attn_kernel_ms_median": float(np.median(kern_ms)),
                "flops": fl, "pairs": pairs}

    main_r = time_pattern(pattern, radius, args.steps, args.warmup)
    value = main_r["flops"] / (main_r["ms_per_step"] * 1e-3) / 1e12
    achieved = main_r["flops"] / (main_r["attn_kernel_ms_avg"] * 1e-3) / 1e12
    log(f"{args.pattern}: {main_r['ms_per_step']:.3f} ms/step, kernel {main_r['attn_kernel_ms_avg']:.3f} ms, "
        f"{achieved:.1f} TFLOP/s")

    extra = {}
    for label, (pat, rad) in w.patterns.items():
        if label == args.pattern or pat == "dense" or args.no_others:
            continue
        r = time_pattern(pat, rad, max(3, args.steps // 4), 2)
        extra[label] = {"ms_per_step": round(r["ms_per_step"], 4),
                        "attn_kernel_ms_avg": round(r["attn_kernel_ms_avg"], 4),
                        "tflops": round(r["flops"] / (r["attn_kernel_ms_avg"] * 1e-3) / 1e12, 2),
                        "frac_of_peak": round(r["flops"] / (r["attn_kernel_ms_avg"] * 1e-3) / 1e12 / BF16_MFMA_PEAK_TFLOPS, 4),
                        "attended_pairs": r["pairs"]}
        log(f"{label}: {extra[label]}")

    dense = None
    if not args.no_dense and w.dtype == "bf16":
        for _ in range(1):
            grat.grat_dense_attention_fwd(Q, K, V, w.scale, out=O)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 2
        a.record()
        for _ in range(reps):
            grat.grat_dense_attention_fwd(Q, K, V, w.scale, out=O)
        b.record()
        torch.cuda.synchronize()
        d_ms = a.elapsed_time(b) / reps
        d_fl = 4.0 * w.head_dim * w.heads * w.batch * float(n_seq) ** 2
        dense = {"kernel_ms": round(d_ms, 3), "tflops": round(d_fl / (d_ms * 1e-3) / 1e12, 2)}
        log(f"dense: {dense}")

    # what the MFMA instruction alone sustains on this machine (no memory traffic, no vector work)
    probe = probe_ones = None
    if not args.no_probe and w.dtype in ("bf16", "f16"):
        try:   # (an aid: a failure here must not cost the benchmark line)
            from paper_2505_14687_amd.probe import probe_wave_sum
            blocks, iters = 256 * 16, 4096
            sink = torch.empty(blocks * 256, dtype=torch.int64, device="cuda")
            rates = {}
            for kind in ("normal_like", "ones"):
                best = None
                for i in range(4):   # the first launch is a warm-up
                    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    a.record()
                    grat.grat_probe_mfma(Q.dtype, kind, blocks, iters, sink=sink)
                    b.record()
                    torch.cuda.synchronize()
                    if i:
                        best = a.elapsed_time(b) if best is None else min(best, a.elapsed_time(b))
                if bool(torch.all(sink.view(-1, 64).sum(1) == probe_wave_sum(kind, iters))):
                    rates[kind] = blocks * 4.0 * iters * 8 * 32768 / (best * 1e-3) / 1e12
                else:
                    log(f"MFMA-only probe ({kind}): wrong sums, not reported")
            probe, probe_ones = rates.get("normal_like"), rates.get("ones")
            log(f"MFMA-only probe: {rates}")
            del sink
        except Exception as e:   # noqa: BLE001
            log(f"MFMA-only probe failed: {e!r}")

    # the other benchmark configurations, one line each (attention launch only, lists prebuilt; inputs
    # N(0,1) rounded to bf16 like the main workload's, drawn on the device from a seeded generator)
    others_w = {}
    if not args.no_others and not args.constant_data and not n_glob and args.workload == "img8192":
        for name, labels in (("img1024", ("B3", "X")), ("img2048", ("B3", "B5", "X", "dense")), ("video", ("B3", "X")),
                             ("video_paper", ("B3", "X")), ("img8192_g8", ("B3", "B5"))):
            ww = synth.WORKLOADS[name]
            gen = torch.Generator(device="cuda")
            gen.manual_seed(ww.seed)
            shape = (ww.batch, ww.heads, ww.n_tokens, ww.head_dim)
            q, k, v = (torch.randn(shape, device="cuda", generator=gen, dtype=torch.bfloat16) for _ in range(3))
            o = torch.empty_like(q)
            n_gw = int(np.prod(ww.group))
            res = {}
            for label in labels:
                pat, rad = ww.patterns[label]
                if pat == "dense":
                    fn = lambda: grat.grat_dense_attention_fwd(q, k, v, ww.scale, out=o)
                    pairs_w = ww.n_tokens * ww.n_tokens
                else:
                    cnt, idx = grat.grat_build_block_lists(ww.grid, ww.group, pat, rad)
                    fn = lambda: grat.grat_attention_fwd(q, k, v, ww.scale, ww.grid, ww.group, cnt, idx, out=o)
                    pairs_w = int(cnt.sum().item()) * n_gw * n_gw
                for _ in range(3):
                    fn()
                torch.cuda.synchronize()
                # launches shorter than a millisecond are timed as they occur in a model: back to back
                # (20 per pair of events), not one at a time out of an idle GPU
                inner = 20 if name in ("img1024", "img2048") and pat != "dense" else 1
                times = []
                for _ in range(10):
                    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    a.record()
                    for _ in range(inner):
                        fn()
                    b.record()
                    torch.cuda.synchronize()
                    times.append(a.elapsed_time(b) / inner)
                ms = float(np.median(times))
                fl = 4.0 * ww.head_dim * ww.heads * ww.batch * pairs_w
                res[label] = {"kernel_ms": round(ms, 4), "tflops": round(fl / (ms * 1e-3) / 1e12, 1)}
            if "dense" in res:
                for label in labels:
                    if label != "dense":
                        res[label]["speedup_vs_dense"] = round(res["dense"]["kernel_ms"] / res[label]["kernel_ms"], 2)
            others_w[name] = res
            log(f"{name}: {res}")
            del q, k, v, o

    cpu = None
    if not args.no_cpu:
        import psutil
        from oracle import grat_oracle as orc
        # recompute the main pattern's output for the parity sample
        count, index = step(pattern, radius)
        attention(count, index)
        torch.cuda.synchronize()
        proc = psutil.Process()
        samples = synth.sample_rows(w.seed + 1000, 4096, w.batch, w.heads, n_seq)
        done, rows_out, t_cpu0, t0 = 0, [], sum(proc.cpu_times()[:2]), time.perf_counter()
        chunk = 32
        while done < len(samples) and time.perf_counter() - t0 < args.cpu_seconds:
            if n_glob:
                rows_out.append(orc.joint_attention_rows(*host, samples[done:done + chunk], n_glob, True,
                                                         w.grid, w.group, pattern, radius, w.scale))
            else:
                rows_out.append(orc.grat_attention_rows(*host, samples[done:done + chunk], w.grid, w.group,
                                                        pattern, radius, w.scale))
            done += chunk
        wall = time.perf_counter() - t0
        cores = max(1, round((sum(proc.cpu_times()[:2]) - t_cpu0) / wall))
        done = min(done, len(samples))
        want = np.concatenate(rows_out)[:done]
        s = torch.from_numpy(samples[:done]).cuda()
        got = O[s[:, 0], s[:, 1], s[:, 2]].double().cpu().numpy()
        pk = orc.token_group_coords(np.arange(w.n_tokens), w.grid, w.group)
        keys = np.empty(done)
        for i in range(done):
            row = int(samples[i, 2]) - n_glob
            if row < 0:
                keys[i] = n_seq
            else:
                pq = orc.token_group_coords(np.array([row]), w.grid, w.group)[0]
                keys[i] = n_glob + int(orc.attendable(pq, pk, pattern, radius).sum())
        cpu_flops = 4.0 * w.head_dim * float(keys.sum())
        diff = got - want
        cpu = {"value": cpu_flops / wall / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
               "sample": f"{done} seeded-random (head, query row) pairs of {args.workload} {args.pattern}, "
                         f"float64 numpy, {wall:.1f} s",
               "seconds_per_row": wall / done,
               "extrapolated_full_launch_s": main_r["flops"] / (cpu_flops / wall),
               "parity_max_abs": float(np.abs(diff).max()),
               "parity_rel_l2": float(np.linalg.norm(diff) / np.linalg.norm(want))}
        log(f"cpu oracle: {cpu}")

    traffic = None if n_glob or args.constant_data else measured_traffic(args.workload, args.pattern)
    all_patterns = None
    if extra:
        fl = main_r["flops"] + sum(4.0 * w.head_dim * w.heads * w.batch * e["attended_pairs"] for e in extra.values())
        ms = main_r["attn_kernel_ms_avg"] + sum(e["attn_kernel_ms_avg"] for e in extra.values())
        all_patterns = {"patterns": [args.pattern] + list(extra), "kernel_ms": round(ms, 4),
                        "tflops": round(fl / (ms * 1e-3) / 1e12, 2),
                        "frac_of_peak": round(fl / (ms * 1e-3) / 1e12 / BF16_MFMA_PEAK_TFLOPS, 4)}
    out = {
        "metric": "GRAT attn TFLOP/s (attended pairs) + speedup vs dense attn, 1 MI355X",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(main_r["ms_per_step"], 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "constant 1.0 (context run)" if args.constant_data else "synthetic",
        "config": {"workload": f"{args.workload}: token grid {'x'.join(map(str, w.grid))}, groups "
                               f"{'x'.join(map(str, w.group))}, batch {w.batch}, {w.heads} heads, head_dim "
                               f"{w.head_dim}, {w.dtype}, pattern {args.pattern} ({pattern}, radius {list(radius)})"
                               + (f", {n_glob} prompt tokens ahead of the grid tokens" if n_glob else ""),
                   "attended_pairs_per_head": main_r["pairs"], "seed": w.seed,
                   "step": "grat_build_block_lists + " + ("grat_attention_global_fwd" if n_glob else "grat_attention_fwd")},
        "roofline": {"bound": "mfma", "achieved": round(achieved, 2), "peak": BF16_MFMA_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(achieved / BF16_MFMA_PEAK_TFLOPS, 4),
                     "traffic": traffic,
                     "traffic_source": None if traffic is None else
                                       f"profiles/attn_mfma_{args.workload}_{args.pattern}.md: stored figure of a separate "
                                       "rocprofv3 --pmc run of this command, not measured in this run",
                     # template arguments: waves per workgroup, keys per LDS tile, mode (0 grouped, 2 joint), half?, head_dim
                     "kernel": kernel_name(w, n_g, n_glob, pattern, radius),
                     # the same matrix instruction in a register-resident loop on this machine (operands
                     # with full significands spread like N(0,1); then all ones), and `achieved` as a
                     # fraction of the former
                     "mfma_only_probe": round(probe, 1) if probe else None,
                     "mfma_only_probe_constant_operands": round(probe_ones, 1) if probe_ones else None,
                     "frac_of_probe": round(achieved / probe, 4) if probe else None,
                     "kernel_ms_avg": round(main_r["attn_kernel_ms_avg"], 4),
                     "kernel_ms_median": round(main_r["attn_kernel_ms_median"], 4),
                     "kernel_ms_min": round(main_r["attn_kernel_ms_min"], 4)},
        "cpu_baseline": cpu,
        "dense": dense,
        "speedup_vs_dense": round(dense["kernel_ms"] / main_r["attn_kernel_ms_avg"], 2) if dense else None,
        "paper_context": "paper: GRAT-B 35.8x over full attention at 8192x8192 on one NVIDIA A100",
        "other_patterns": extra,
        # the workload's patterns together (one launch each): total attended-pair work / total kernel time
        "all_patterns": all_patterns,
        "other_workloads": others_w,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
