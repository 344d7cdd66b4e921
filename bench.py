"""Benchmark: search + quantize + delta of one 7B-shaped fp32 checkpoint on one MI355X.

A "step" is one pass of the whole hot path over the current checkpoint (291 tensors, 6.74 G values,
27 GB): inshr_search over the 105-configuration grid, inshr_quantize with the chosen configuration
of every tensor, inshr_delta against the previous checkpoint's codes.  Inputs are resident in HBM
and the previous checkpoint's codes exist before the timed region starts.  One JSON line is printed.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth


def algorithmic_bytes_per_element(bits_cur: int, bits_prev: int) -> float:
    """Floor traffic of the path per element: two reads to find the order statistics, one to score,
    one to quantize (+ packed write), delta reads both symbol streams and writes one."""
    w = bits_cur + 1
    wp = bits_prev + 1
    wb = max(bits_cur, bits_prev) + 1
    return 16.0 + (2 * w + wp + wb) / 8.0


def cpu_baseline(sample, grid, eps, threads):
    """The oracle as it stands, one tensor per thread, on a bounded sample of the workload."""
    from concurrent.futures import ThreadPoolExecutor
    from oracle import ref

    def one(pair):
        prev, cur = pair
        bp, _, _ = ref.search(prev, grid, eps)
        bc, _, _ = ref.search(cur, grid, eps)
        qp = ref.quantize(prev, grid[bp])
        qc = ref.quantize(cur, grid[bc])
        ref.delta(qp["sym"], grid[bp][0], qc["sym"], grid[bc][0])
        return cur.size

    ref.lib()
    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=threads) as ex:
        n = sum(ex.map(one, sample))
    dt = time.perf_counter() - t0
    # each pair ran the path on two checkpoints; a step of the benchmark is one checkpoint
    return 2 * n * 4 / dt / 1e9, dt


TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "bench_llama7b_hbm_traffic.md")


def measured_traffic(kernel):
    """HBM bytes per launch (fetched + written) of `kernel` on the full workload, as the tracked
    summary of the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this bench states them (counters
    cannot be read from inside the process).  The summary carries one machine-readable line
    `traffic_bytes: {...}` with the commit its runs were made at.  (None, None) without it."""
    try:
        for line in open(TRAFFIC_PROFILE):
            if line.startswith("traffic_bytes:"):
                d = json.loads(line.split(":", 1)[1])
                return d.get(kernel), d.get("measured_at")
    except (OSError, ValueError):
        pass
    return None, None


def copy_yardstick():
    """A plain 1 GiB device-to-device copy: the kernel of known size that scales the FETCH_SIZE and
    WRITE_SIZE counters of `rocprofv3 --pmc` (run this mode under the profiler)."""
    import torch
    dev = torch.device("cuda:0")
    a = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
    b = torch.empty_like(a)
    torch.cuda.synchronize()
    for _ in range(3):
        b.copy_(a)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(20):
        b.copy_(a)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / 20
    t0 = time.perf_counter()
    for _ in range(20):
        s = a.sum()
    torch.cuda.synchronize()
    dr = (time.perf_counter() - t0) / 20
    # the same copy as an elementwise kernel (a dispatch of its own in every profiler's list)
    for _ in range(3):
        torch.mul(a, 1.0, out=b)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(20):
        torch.mul(a, 1.0, out=b)
    torch.cuda.synchronize()
    de = (time.perf_counter() - t0) / 20
    print(json.dumps({"copy_yardstick": "device copies of 1 GiB (1048576 KiB read, 1048576 KiB written each)",
                      "copy_GB/s_read_plus_write": round(2 * a.numel() * 4 / dt / 1e9, 1),
                      "elementwise_copy_GB/s_read_plus_write": round(2 * a.numel() * 4 / de / 1e9, 1),
                      "read_only_sum_GB/s": round(a.numel() * 4 / dr / 1e9, 1)}))


def checkpoint_hash(torch, qs, ds):
    """Order-sensitive 64-bit hash of all packed symbol words and delta stream words (wrapping
    integer arithmetic on the device)."""
    h = 0
    for k, t in enumerate([q.packed for q in qs] + [d.packed for d in ds]):
        w = torch.arange(1, t.numel() + 1, dtype=torch.int64, device=t.device) * 2654435761 + k
        h = (h * 1000003 + int((t * w).sum())) & 0xFFFFFFFFFFFFFFFF
    return h


def validate_batch(torch, ctx, cur, cfgs, grid, eps, q_prev, q_cur, d_out, step):
    """Untimed checks of the whole batch the timed steps worked on, on the device: class counts add
    up; the delta stream decodes (Algorithm 6) to the current symbols; every symbol is in range and
    the protected list holds exactly the elements with symbol 1 (the decoder checks both); every
    protected value is the input bit for bit; pruned values decode to +0.0; the squared error of
    the decoded checkpoint equals, per tensor, the score the search gave the chosen configuration;
    two more steps leave identical bytes."""
    res = {}
    res["class_counts_add_up"] = all(q.n_pruned + q.n_outlier + q.n_kept == q.n for q in q_cur)
    h1 = checkpoint_hash(torch, q_cur, d_out)
    step()
    h2 = checkpoint_hash(torch, q_cur, d_out)
    res["bytes_identical_across_steps"] = h1 == h2
    res["hash"] = f"{h2:016x}"
    rec = ctx.reconstruct(q_prev, d_out, [c[0] for c in cfgs])
    res["reconstructed_equals_current_codes"] = all(torch.equal(r, q.packed) for r, q in zip(rec, q_cur))
    del rec
    best, feas, scores = ctx.search(cur, grid, eps, want_scores=True)
    res["same_choice_with_scores"] = [grid[b] for b in best] == list(cfgs)
    buf = torch.empty(max(t.numel() for t in cur), dtype=torch.float32, device=cur[0].device)
    prot_ok = zero_ok = sse_ok = True
    worst = 0.0
    for i, (t, q) in enumerate(zip(cur, q_cur)):
        x = t.reshape(-1)
        y = buf[:x.numel()]
        ctx.dequantize([q], out=[y])  # raises on a symbol out of range or a wrong protected list
        idx = q.outlier_idx.to(torch.int64) & 0xFFFFFFFF
        prot_ok = prot_ok and torch.equal(x[idx].view(torch.int32), q.outlier_val.view(torch.int32)) \
            and torch.equal(y[idx].view(torch.int32), q.outlier_val.view(torch.int32))
        tau = q.tau_prune
        zero_ok = zero_ok and bool((y[x.abs() < tau].view(torch.int32) == 0).all())
        sse = float(((x.double() - y.double()) ** 2).sum())
        sc = scores[i * len(grid) + best[i]]
        err = abs(sc.sse - sse) / (1e-6 * sse + 1e-12 * sc.sumsq + 1e-300)
        worst = max(worst, err)
        sse_ok = sse_ok and err <= 1.0
    res["protected_values_bit_exact"] = prot_ok
    res["pruned_decode_to_zero"] = zero_ok
    res["decoded_error_equals_score"] = sse_ok
    res["decoded_error_vs_score_worst_over_tolerance"] = round(worst, 4)
    res["validated"] = all(v for k, v in res.items() if isinstance(v, bool))
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--layers", type=int, default=32, help="decoder layers of the 7B shape (32 = full)")
    ap.add_argument("--config", type=int, default=4, choices=[0, 1, 2, 3, 4],
                    help="benchmark configuration: 4 (default) is the metric's workload; 0-3 are the "
                         "smaller ones (config0 tensor, ResNet-50 / BERT-base / GPT-2-medium shapes "
                         "with Adam state), reported for reference")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-validate", action="store_true",
                    help="skip the untimed checks of the batch after the timed steps")
    ap.add_argument("--copy-yardstick", action="store_true",
                    help="run only a plain 1 GiB device copy (the kernel of known size that scales the "
                         "HBM traffic counters of rocprofv3 --pmc) and exit")
    ap.add_argument("--pooled", action="store_true",
                    help="also time search + quantize with thresholds shared per kind of layer (extra object)")
    ap.add_argument("--restore", action="store_true",
                    help="also time the restore side (reconstruct + dequantize of the checkpoint) after "
                         "the timed steps and report it as an extra object; needs 4 more bytes per value")
    ap.add_argument("--sketch", action="store_true",
                    help="also time the quantizer with the sketch + weighted K-Means bins on the chosen "
                         "configurations after the timed steps, and compare its squared error with the "
                         "equal-frequency bins (extra object; needs 4 more bytes per value)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)",
              file=sys.stderr)
        sys.exit(2)

    if args.copy_yardstick:
        copy_yardstick()
        return

    import numpy as np
    import torch
    from paper_2306_11800_amd import api, synth

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    grid = synth.grid_full() if args.config >= 2 else synth.grid_small()
    eps = synth.EPS_DEFAULT
    if args.config == 4:
        names, prev, cur = synth.llama7b_device_checkpoint(dev, seed=4000, n_layers=args.layers)
        what = (f"Llama-7B-shaped fp32 checkpoint, {args.layers} layers, Student-t(3)*0.015 with 0.1% "
                f"channels x20, next step = prev + N(0,1e-4)")
    else:  # host generators, uploaded once
        if args.config == 0:
            p0, c0 = synth.config0(seed=0)
            items, what = [("config0", p0, c0)], "one tensor 0.9 N(0,0.02) + 0.1 Laplace(0,0.08), next = prev + N(0,1e-4)"
        elif args.config == 1:
            items, what = list(synth.resnet50_checkpoint()), "ResNet-50-shaped weights + Adam m, v, one Adam step"
        elif args.config == 2:
            items, what = list(synth.bert_base_checkpoint()), "BERT-base-shaped weights + Adam m, v, sparse embedding update"
        else:
            items = [(n, st[0], st[1]) for n, st in synth.gpt2_medium_steps(n_steps=2)]
            what = "GPT-2-medium-shaped weights + Adam m, v, steps 0 -> 1"
        names = [n for n, _, _ in items]
        prev = [torch.from_numpy(a).to(dev) for _, a, _ in items]
        cur = [torch.from_numpy(b).to(dev) for _, _, b in items]
        del items
    n_total = sum(t.numel() for t in cur)
    ctx = api.Context(dev)
    mem0 = (torch.cuda.mem_get_info()[0], torch.cuda.memory_reserved())
    cur = ctx.batch(cur)  # the binding marshals the tensor list once, not in every step

    # previous checkpoint's codes (set-up, untimed)
    best_p, _, _ = ctx.search(prev, grid, eps, want_scores=False)
    q_prev = ctx.quantize(prev, [grid[b] for b in best_p], reuse_search=True)

    q_cur = None
    d_out = None

    def step():
        nonlocal q_cur, d_out
        best, feas, _ = ctx.search(cur, grid, eps, want_scores=False)
        cfgs = [grid[b] for b in best]
        q_cur = ctx.quantize(cur, cfgs, reuse_search=True, out=q_cur)
        d_out = ctx.delta(q_prev, q_cur, out=d_out)
        ctx.sync()
        return cfgs

    # the first call sizes the output buffers at full capacity (8-bit symbols, 0.1 % protected)
    full = [(8, 0, 1000)] * len(cur)
    q_cur = ctx.quantize(cur, full, reuse_search=False)
    d_out = ctx.delta(q_prev, q_cur)
    ctx.sync()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ctx.profile(True)
    t0 = time.perf_counter()
    marks = [t0]
    for _ in range(args.steps):
        cfgs = step()  # (ends with a synchronisation of the stream)
        marks.append(time.perf_counter())
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = ctx.profile_read()
    ctx.profile(False)
    step_ms = sorted((b - a) * 1e3 for a, b in zip(marks, marks[1:]))

    # device memory the library holds for its scratch (what left the device minus what torch reserved
    # for the inputs' neighbours: codes, delta streams)
    lib_scratch = (mem0[0] - torch.cuda.mem_get_info()[0]) - (torch.cuda.memory_reserved() - mem0[1])
    ms_per_step = dt / args.steps * 1e3
    value = n_total * 4 / (dt / args.steps) / 1e9

    # floor-traffic model of the whole path with the configurations actually chosen
    a_bytes = 0.0
    for t, c, bp in zip(cur, cfgs, best_p):
        a_bytes += t.numel() * algorithmic_bytes_per_element(c[0], grid[bp][0])
    path_gbs = a_bytes / (dt / args.steps) / 1e9

    # dominant kernel: algorithmic bytes per launch / average launch duration (HIP events)
    per_launch = {k: v[0] / max(v[1], 1) for k, v in prof.items()}
    dom = max(per_launch, key=per_launch.get)
    mean_w = sum(t.numel() * (c[0] + 1) for t, c in zip(cur, cfgs)) / n_total
    kernel_bytes = {
        "k_hist1": 4.0, "k_hist2": 4.0, "k_gather": 4.0, "k_score": 4.0,
        "k_quant": 4.0 + mean_w / 8.0,
        "k_dhist": mean_w / 8.0, "k_dscatter": 3.0 * mean_w / 8.0,
    }
    dom_bytes = kernel_bytes.get(dom, 4.0) * n_total
    achieved = dom_bytes / (per_launch[dom] * 1e-3) / 1e9
    traffic, traffic_at = measured_traffic(dom) if (args.layers == 32 and args.config == 4) else (None, None)
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": traffic, "traffic_measured_at": traffic_at,
                "avg_launch_ms": round(per_launch[dom], 4),
                "path_floor_bytes_per_elem": round(a_bytes / n_total, 3),
                "path_achieved": round(path_gbs, 1), "path_frac": round(path_gbs / HBM_PEAK_GBS, 4),
                "kernel_ms_per_step": {k: round(v[0] / args.steps, 4) for k, v in sorted(prof.items())}}

    validation = None
    if not args.no_validate:
        validation = validate_batch(torch, ctx, cur, cfgs, grid, eps, q_prev, q_cur, d_out, step)
        validation["lds_ordered"] = ctx.lds_ordered

    pooled = None
    if args.pooled and args.config == 4:
        # thresholds per layer type: the tensors of one kind in all layers share their thresholds
        # (the gate / up / down projections are kinds of their own: a group holds fewer than 2^32 values)
        kinds = {}
        groups = [kinds.setdefault(nm.split(".", 2)[2] if nm.startswith("layers.") else nm, len(kinds)) for nm in names]
        for it in range(3):
            if it == 1:
                torch.cuda.synchronize()
                ctx.profile(True)
                t0 = time.perf_counter()
            best_g, feas_g, sc_g = ctx.search(cur, grid, eps, want_scores=True, groups=groups)
            caps = [int(sc_g[i * len(grid) + b].n_outlier) + 1 for i, b in enumerate(best_g)]
            q_g = ctx.quantize(cur, [grid[b] for b in best_g], reuse_search=True, outlier_caps=caps)
            ctx.sync()
        torch.cuda.synchronize()
        pdt = (time.perf_counter() - t0) / 2
        pprof = ctx.profile_read()
        ctx.profile(False)
        pooled = {"groups": len(kinds), "ms_search_plus_quantize": round(pdt * 1e3, 3),
                  "kernel_ms": {k: round(v[0] / 2, 4) for k, v in sorted(pprof.items()) if v[0] / 2 > 0.3}}
        del q_g

    restore = None
    if args.restore:
        bits_cur = [c[0] for c in cfgs]
        xs = [torch.empty_like(t) for t in cur]
        for it in range(3):
            if it == 1:
                torch.cuda.synchronize()
                ctx.profile(True)
                t0 = time.perf_counter()
            rec = ctx.reconstruct(q_prev, d_out, bits_cur)
            ctx.dequantize(q_cur, out=xs)
        torch.cuda.synchronize()
        rdt = (time.perf_counter() - t0) / 2
        rprof = ctx.profile_read()
        ctx.profile(False)
        same = all(torch.equal(r, q.packed) for r, q in zip(rec, q_cur))
        restore = {"ms": round(rdt * 1e3, 3), "GB/s_of_fp32_restored": round(n_total * 4 / rdt / 1e9, 1),
                   "reconstructed_equals_current_codes": same,
                   "kernel_ms": {k: round(v[0] / 2, 4) for k, v in sorted(rprof.items())}}
        del xs, rec

    sketch = None
    if args.sketch:
        uni = np.random.default_rng(12345).uniform(size=(len(cur), 256))
        # stand-alone (one single-configuration search per distinct configuration inside), then on
        # top of the grid search of the step
        for it in range(2):
            if it == 1:
                torch.cuda.synchronize()
                t0 = time.perf_counter()
            q_sk, sk_info = ctx.quantize_sketch(cur, cfgs, uni, alpha=0.01, sigma=0.2, max_iter=100)
        torch.cuda.synchronize()
        sdt_alone = time.perf_counter() - t0
        ctx.search(cur, grid, eps, want_scores=False)
        for it in range(3):
            if it == 1:
                torch.cuda.synchronize()
                ctx.profile(True)
                t0 = time.perf_counter()
            q_sk, sk_info = ctx.quantize_sketch(cur, cfgs, uni, alpha=0.01, sigma=0.2, max_iter=100,
                                                reuse_search=True)
        torch.cuda.synchronize()
        sdt = (time.perf_counter() - t0) / 2
        sprof = ctx.profile_read()
        ctx.profile(False)
        q_eq = ctx.quantize(cur, cfgs, reuse_search=False)
        err_sk = err_eq = sumsq = 0.0
        buf = torch.empty(max(t.numel() for t in cur), dtype=torch.float32, device=dev)
        for t, a, b in zip(cur, q_sk, q_eq):
            y = buf[:t.numel()]
            ctx.dequantize([a], out=[y])
            err_sk += float(((t.reshape(-1).double() - y.double()) ** 2).sum())
            ctx.dequantize([b], out=[y])
            err_eq += float(((t.reshape(-1).double() - y.double()) ** 2).sum())
            sumsq += float((t.double() ** 2).sum())
        # fewer bits with the same prune / protect fractions: how many tensors still meet eps, and
        # the error of the whole checkpoint (Sec. 4.4: non-uniform bins need fewer of them)
        sq_t = [float((t.double() ** 2).sum()) for t in cur]
        fewer = {}
        ctx.search(cur, grid, eps, want_scores=False)
        for drop in (1, 2, 3, 4):
            c2 = [(max(2, c[0] - drop), c[1], c[2]) for c in cfgs]
            q2, _ = ctx.quantize_sketch(cur, c2, uni, alpha=0.01, sigma=0.2, max_iter=100,
                                        reuse_search=len(grid) == 105)
            ok, tot = 0, 0.0
            for t, a, sq in zip(cur, q2, sq_t):
                y = buf[:t.numel()]
                ctx.dequantize([a], out=[y])
                e = float(((t.reshape(-1).double() - y.double()) ** 2).sum())
                tot += e
                ok += 1 if e <= eps * sq else 0
            fewer[f"bits-{drop}"] = {"tensors_within_eps": ok, "rel_sq_error": tot / sumsq}
            del q2
        # the search over the bit width with the sketch bins, on top of the grid search of the step
        ctx.search(cur, grid, eps, want_scores=False)
        for it in range(3):
            if it == 1:
                torch.cuda.synchronize()
                ctx.profile(True)
                t0 = time.perf_counter()
            # (on top of the grid search when its grid holds every width of the fractions in use)
            q_ss, choices, _ = ctx.search_sketch(cur, cfgs, uni, eps, alpha=0.01, sigma=0.2, max_iter=100,
                                                 reuse_search=len(grid) == 105)
        torch.cuda.synchronize()
        ssdt = (time.perf_counter() - t0) / 2
        ssprof = ctx.profile_read()
        ctx.profile(False)
        bits_hist = {}
        for ch in choices:
            bits_hist[ch["best_bits"]] = bits_hist.get(ch["best_bits"], 0) + 1
        search_bits = {"ms_after_a_search": round(ssdt * 1e3, 3),
                       "kernel_ms": {k: round(v[0] / 2, 4) for k, v in sorted(ssprof.items())},
                       "k_sketch_score_GB/s": round(n_total * 4 / (ssprof["k_sketch_score"][0] / 2 * 1e-3) / 1e9, 1),
                       "chosen_bits": {str(b): bits_hist[b] for b in sorted(bits_hist)},
                       "infeasible": sum(1 for ch in choices if not ch["feasible"]),
                       "symbol_bits_per_value": round(sum(t.numel() * (ch["best_bits"] + 1) for t, ch in zip(cur, choices)) / n_total, 3),
                       "symbol_bits_per_value_equal_frequency": round(sum(t.numel() * (c[0] + 1) for t, c in zip(cur, cfgs)) / n_total, 3),
                       "rel_sq_error": sum(ch["sse"][ch["best_bits"] - 2] for ch in choices) / sum(ch["sumsq"] for ch in choices)}
        del q_ss
        # a whole step with the sketch bins and fixed fractions (those most tensors got): thresholds
        # only from the search kernels, sketch, clustering, scoring, quantize, then the delta
        common = max(set((c[1], c[2]) for c in cfgs), key=lambda pq: sum(1 for c in cfgs if (c[1], c[2]) == pq))
        fixed = [(0, common[0], common[1])] * len(cur)
        # (the previous checkpoint's codes come from the same kind of step, as in a chain)
        q_prev_alt, _, _ = ctx.search_sketch(prev, fixed, uni, eps, alpha=0.01, sigma=0.2, max_iter=100)
        q_alt = d_alt = None
        for it in range(3):
            if it == 1:
                torch.cuda.synchronize()
                ctx.profile(True)
                t0 = time.perf_counter()
            q_alt, alt_choices, _ = ctx.search_sketch(cur, fixed, uni, eps, alpha=0.01, sigma=0.2, max_iter=100,
                                                      out=q_alt)
            d_alt = ctx.delta(q_prev_alt, q_alt, out=d_alt)
            ctx.sync()
        torch.cuda.synchronize()
        adt = (time.perf_counter() - t0) / 2
        aprof = ctx.profile_read()
        ctx.profile(False)
        search_bits["whole_step_with_fixed_fractions"] = {
            "prune_ppm": common[0], "outlier_ppm": common[1], "ms": round(adt * 1e3, 3),
            "GB/s": round(n_total * 4 / adt / 1e9, 1),
            "kernel_ms": {k: round(v[0] / 2, 4) for k, v in sorted(aprof.items()) if v[0] / 2 >= 0.05},
            "symbol_bits_per_value": round(sum(t.numel() * (ch["best_bits"] + 1) for t, ch in zip(cur, alt_choices)) / n_total, 3)}
        del q_alt, d_alt, q_prev_alt
        hist_ms = sprof["k_sketch_hist"][0] / 2
        sketch = {"ms_after_a_search": round(sdt * 1e3, 3), "ms_stand_alone": round(sdt_alone * 1e3, 3),
                  "alpha": 0.01, "sigma": 0.2, "max_iter": 100,
                  "kernel_ms": {k: round(v[0] / 2, 4) for k, v in sorted(sprof.items())},
                  "k_sketch_hist_GB/s": round(n_total * 4 / (hist_ms * 1e-3) / 1e9, 1),
                  "buckets_mean": round(sum(i[0] for i in sk_info) / len(sk_info), 1),
                  "buckets_max": max(i[0] for i in sk_info),
                  "rounds_mean": round(sum(i[1] for i in sk_info) / len(sk_info), 1),
                  "rounds_max": max(i[1] for i in sk_info),
                  "rel_sq_error_sketch_bins": err_sk / sumsq,
                  "rel_sq_error_equal_frequency_bins": err_eq / sumsq,
                  "sketch_bins_with_fewer_bits": fewer,
                  "search_over_bits": search_bits}
        del q_sk, q_eq, buf

    cpu = None
    if not args.no_cpu_baseline:
        threads = min(16, os.cpu_count() or 1)
        rows = 1 << 20  # the first 2^20 values of the first `threads` 2-D weights ...
        picks = [i for i, t in enumerate(cur) if t.numel() >= rows][:threads]
        sample = [(prev[i].reshape(-1)[:rows].cpu().numpy(), cur[i].reshape(-1)[:rows].cpu().numpy()) for i in picks]
        # ... and every whole tensor the oracle finishes in seconds (a whole 4096 x 4096 weight takes
        # the sort-based oracle minutes on one core, more than this leg may spend)
        small = [i for i, t in enumerate(cur) if t.numel() <= 1 << 16]
        sample += [(prev[i].reshape(-1).cpu().numpy(), cur[i].reshape(-1).cpu().numpy()) for i in small]
        gbs, secs = cpu_baseline(sample, grid, eps, threads)
        cpu = {"value": round(gbs, 5), "unit": "GB/s", "cores": threads, "kind": "oracle",
               "sample": f"first {rows} values of {len(picks)} weight tensors ({', '.join(names[i] for i in picks[:3])}, ...) "
                         f"and {len(small)} whole tensors of at most 65536 values ({', '.join(names[i] for i in small[:2])}, ...), "
                         f"both checkpoints, same {len(grid)}-config grid, {secs:.1f} s wall"}

    out = {
        "metric": "GB/s fp32 checkpoint searched+quantized+delta-encoded; % of HBM roofline",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "ms_step_median": round(step_ms[len(step_ms) // 2], 3), "ms_step_min": round(step_ms[0], 3),
        "ms_step_max": round(step_ms[-1], 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{what}; {len(cur)} tensors, {n_total} values; grid of {len(grid)} "
                               f"configurations (" + ("bits 2..8 x prune {0,.05,.1,.2,.4} x protect {0,1e-4,1e-3}"
                                                      if len(grid) == 105 else
                                                      "bits {2,3,4,8} x prune {0,.1,.3} x protect {0,.001}")
                               + f"), eps {eps}",
                   "bytes_fp32": n_total * 4, "library_scratch_bytes": int(lib_scratch),
                   "chosen_configs": {f"b{b}_p{p}_o{o}": sum(1 for c in cfgs if tuple(c) == (b, p, o))
                                      for (b, p, o) in sorted(set(tuple(c) for c in cfgs))}},
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    if validation is not None:
        out["validation"] = validation
    if pooled is not None:
        out["pooled"] = pooled
    if restore is not None:
        out["restore"] = restore
    if sketch is not None:
        out["sketch"] = sketch
    print(json.dumps(out))


if __name__ == "__main__":
    main()
