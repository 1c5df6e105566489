"""Benchmark of the PyramidKV compression step on one MI355X.

A step = the whole hot path (budgets excluded: host, once) over one request batch: pkv_compress_layers over all L
layers of the workload -- window scoring, pooling, per-head top-k, K/V gather.  Inputs are resident in HBM.
Prints one JSON line (metric of the benchmark spec: compressed prefill tokens/s over all layers).

Order of the legs for a workload: (1) per-kernel HIP-event profile (also brings the device to its working
clocks), (2) W untimed warm-up steps, (3) K timed steps, every step bracketed by HIP events on the launch stream,
the whole region bracketed by synchronisations; `ms_per_step` is the MEDIAN of the K per-step event times
(`ms_per_step_mean_wall` is the wall-clock mean over the same K steps), (4) checks of the outputs the timed steps
left, (5) for the headline workload: the CPU oracle timed on a bounded sample of layers and compared with the
device's result on those layers.
"""
import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0         # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak, published
METRIC = "compressed prefill tokens/sec (all layers, select+gather); achieved HBM GB/s"


def layer_bytes(w, k_l, sum_n):
    """Algorithmic bytes of one layer: K once + Q_win + gathered K,V rows read and written + kept indices."""
    k_bytes = w.Hkv * sum_n * w.d * 2
    q_bytes = w.B * w.Hq * w.alpha * w.d * 2
    gather = 4 * w.B * w.Hkv * k_l * w.d * 2
    idx = w.B * w.Hkv * k_l * 4
    return k_bytes + q_bytes + gather + idx


def kernel_bytes(name, w, ks, sum_n):
    """Algorithmic bytes of ONE launch of a kernel (same accounting as layer_bytes, split per kernel)."""
    kq = w.Hkv * sum_n * w.d * 2 + w.B * w.Hq * w.alpha * w.d * 2          # K once + Q_win, one layer
    if name == "score_resident":                                             # one launch covers all layers
        return kq * w.L
    if name in ("score_stats", "score_accum"):                               # one launch per layer and sweep
        return kq
    if name == "gather":
        return sum(4 * w.B * w.Hkv * k * w.d * 2 for k in ks)
    if name == "pool_select":
        return sum(w.B * w.Hkv * k * 4 for k in ks)
    return 0


def score_flops(w, sum_n):
    """Matrix flops of the window logits of all layers, each logit formed once: 2 * (G alpha) * d per key and head."""
    return 2.0 * w.G * w.alpha * w.d * w.Hkv * sum_n * w.L


def tracked(table, kernel, workload, avg, cast):
    """A figure from a committed rocprofv3 counter summary (profiles/<table>), or None.
    Lines: kernel  workload  avg_budget  value."""
    path = os.path.join(ROOT, "profiles", table)
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if len(f) == 4 and not line.startswith("#") and f[0] == kernel and f[1] == workload and int(f[2]) == avg:
            return cast(f[3])
    return None


def cpu_baseline(w, ks, layers_host, lens, budget_s=12.0):
    """The oracle, as it stands, on the host cores, on a bounded sample of layers of the same workload."""
    from oracle import pkv_oracle
    sum_n = int(lens.sum()) if lens is not None else w.B * w.N
    t_used, done = 0.0, []
    order = [0, w.L - 1] + [l for l in range(1, w.L - 1)]
    for l in order:
        if l not in layers_host:
            continue
        Q, K, V = layers_host[l]
        t0 = time.perf_counter()
        pkv_oracle.compress_layer(Q, K, V, ks[l], w.alpha, w.pool, w.pool_w, seq_lens=lens, want_pooled=False)
        t_used += time.perf_counter() - t0
        done.append(l)
        if t_used > budget_s:
            break
    per_layer = t_used / len(done)
    threads = min(pkv_oracle.num_threads(), w.G * w.alpha)
    return {"value": sum_n / (per_layer * w.L), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"layers {sorted(done)} of {w.L} timed ({t_used:.1f} s), all-layer time extrapolated linearly"}


def verify_against_oracle(w, ks, Qs, Ks, Vs, lens, lens_dev, timed_outputs, verify_layers):
    """Outside the timed region: the device's result on sampled layers against the oracle (tests/parity.py's
    protocol), and the timed steps' own outputs against that verified result, bit for bit."""
    import torch
    from paper_2406_02069_amd import binding
    from tests.parity import compare_layer
    tot = {"layers": [], "units": 0, "near_tie_units": 0, "max_rel_err": 0.0}
    for l in verify_layers:
        Q, K, V = Qs[l], Ks[l], Vs[l]
        out = binding.compress_layer(Q, K, V, ks[l], w.pool, w.pool_w, seq_lens=lens_dev, want_scores=True)
        torch.cuda.synchronize()
        st = compare_layer(Q, K, V, ks[l], w.alpha, w.pool, w.pool_w, lens, out)
        for i in range(4):   # K_out, V_out, idx, count of the timed call
            if not torch.equal(out[i], timed_outputs[l][i]):
                raise RuntimeError(f"bench: layer {l}: output {i} of the timed steps differs from the verified call")
        tot["layers"].append(l)
        tot["units"] += st["units"]
        tot["near_tie_units"] += st["near_tie_units"]
        tot["max_rel_err"] = max(tot["max_rel_err"], st["max_rel_err"])
    return tot


def measure(w, avg, steps, warmup, dev, lse=False, page_size=0, host_layers=(), want_read_probe=True, graph=False):
    """Generates the workload on the device, runs the legs described at the top, returns (result dict, context)."""
    import numpy as np
    import torch
    from paper_2406_02069_amd import binding, synth

    ks = binding.budgets(w.L, avg, w.beta, w.alpha)
    lens = synth.seq_lens(w)
    sum_n = int(lens.sum()) if lens is not None else w.B * w.N
    lens_dev = None if lens is None else torch.from_numpy(lens).to(dev)
    Qs, Ks, Vs, layers_host = [], [], [], {}
    for l in range(w.L):
        Q, K, V, _ = synth.make_layer(w, l, dev)
        Qs.append(Q), Ks.append(K), Vs.append(V)
        if l in host_layers:
            layers_host[l] = (Q.cpu(), K.cpu(), V.cpu())
    lses = None
    if lse:  # what the prefill attention kernel would hand over; an input, prepared before timing
        from tests import prefill_stub
        lses = [prefill_stub.window_lse(Qs[l], Ks[l], lens) for l in range(w.L)]
    paged = None
    if page_size > 0:  # every layer its own pool and block table; pages handed out in a seeded random order
        P = page_size
        max_pages = max((min(k, w.N) + P - 1) // P for k in ks)
        num_pages = w.B * max_pages
        rs = np.random.RandomState(1234)
        Kp = [torch.zeros(num_pages, w.Hkv, P, w.d, dtype=torch.bfloat16, device=dev) for _ in range(w.L)]
        Vp = [torch.zeros(num_pages, w.Hkv, P, w.d, dtype=torch.bfloat16, device=dev) for _ in range(w.L)]
        tbs = [torch.from_numpy(rs.permutation(num_pages).astype(np.int32).reshape(w.B, max_pages)).to(dev)
               for _ in range(w.L)]
        paged = (Kp, Vp, tbs, P)
    call = binding.LayersCall(Qs, Ks, Vs, ks, w.pool, w.pool_w, seq_lens=lens_dev, lse=lses, paged=paged)
    torch.cuda.synchronize()

    # (1) Per-kernel device time, with HIP events around every kernel (recorded on the stream the kernels run on).
    # Kept apart from the timed region so that the event packets between the kernels do not slow `value`.
    n_prof, n_skip = max(steps, 10), 30   # the first n_skip profiled steps are this leg's own warm-up
    events = binding.HipEvents(5 * w.L + 1)
    per_kernel = {}
    for it in range(n_skip + n_prof):
        ids = binding.run_profiled(call, events)
        torch.cuda.synchronize()
        if it < n_skip:
            continue
        for i, kid in enumerate(ids):
            per_kernel.setdefault(kid, []).append(events.elapsed_ms(i, i + 1))
    events.close()
    avg_ms = {binding.KERNEL_NAMES[k]: float(np.mean(v)) for k, v in per_kernel.items()}
    sum_ms = {binding.KERNEL_NAMES[k]: float(np.sum(v)) / n_prof for k, v in per_kernel.items()}
    dominant = max(sum_ms, key=sum_ms.get)

    # (2) warm-up, (3) the timed steps
    step = call.run
    if graph:   # variant: the step recorded once into a HIP graph (on a side stream) and replayed
        side = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                call.run()
        step = g.replay
    for _ in range(warmup):
        step()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]   # torch's current stream = launch stream
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(steps):
        step()
        ev[i + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    step_ms = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(steps)])
    ms_per_step = float(np.median(step_ms))

    # (4) the outputs the timed steps left: a count of -1 means a scoring launch gave up a wait between its
    # workgroups (meaningless rows); such a run must not be reported as a measurement
    want_counts = [np.minimum(k, lens if lens is not None else np.full(w.B, w.N)).astype(np.int64) for k in ks]
    for l, out in enumerate(call.outputs):
        got = out[3].cpu().numpy().astype(np.int64)
        if not np.array_equal(got, want_counts[l]):
            raise RuntimeError(f"bench: layer {l}: count_out {got.tolist()} != {want_counts[l].tolist()}: "
                               "the timed steps did not produce valid results")

    total_bytes = sum(layer_bytes(w, k, sum_n) for k in ks)
    dom_bytes = kernel_bytes(dominant, w, ks, sum_n)
    achieved = dom_bytes / (avg_ms[dominant] * 1e-3) / 1e9
    kname = dominant + ("_lse" if lse else "")
    res = {
        "value": sum_n / (ms_per_step * 1e-3),
        "ms_per_step": ms_per_step,
        "ms_per_step_stat": f"median of {steps} per-step HIP-event times",
        "ms_per_step_mean_wall": dt / steps * 1e3,
        "ms_per_step_min": float(step_ms.min()), "ms_per_step_max": float(step_ms.max()),
        "config": {"workload": f"{w.name}: B{w.B} L{w.L} Hq{w.Hq} Hkv{w.Hkv} d{w.d} N{w.N} alpha{w.alpha} "
                               f"avg_budget{avg} beta{w.beta} pool{w.pool}/w{w.pool_w}" +
                               (" +lse" if lse else "") + (f" +pages{page_size}" if page_size > 0 else ""),
                   "tokens_per_step": sum_n, "algorithmic_bytes_per_step": total_bytes},
        "whole_path": {"achieved_GBps": total_bytes / (ms_per_step * 1e-3) / 1e9,
                       "frac_of_hbm_peak": total_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS},
        "roofline": {"kernel": dominant, "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": tracked("traffic_bytes.txt", kname, w.name, avg, int),
                     "algorithmic_bytes_per_launch": dom_bytes, "avg_launch_ms": avg_ms[dominant],
                     "launches_timed": len(per_kernel[binding.KERNEL_NAMES.index(dominant)]),
                     "mfma_busy_frac": tracked("pipe_busy.txt", kname + ":mfma", w.name, avg, float),
                     "valu_busy_frac": tracked("pipe_busy.txt", kname + ":valu", w.name, avg, float)},
        "kernel_ms_per_step": sum_ms,
    }
    # A workload whose window logits need more matrix work per byte of K than the chip's ridge is bound by the
    # matrix pipe, not by HBM: its roofline is stated in flops (each logit formed once; the two-sweep kernel
    # executes twice that, reported beside it).
    fl = score_flops(w, sum_n)
    launches_per_step = len(per_kernel[binding.KERNEL_NAMES.index(dominant)]) / n_prof
    if dominant.startswith("score") and fl / dom_bytes / max(launches_per_step, 1) > MFMA_BF16_PEAK_TFLOPS / HBM_PEAK_GBPS * 1e3:
        tf = fl / (sum_ms[dominant] * 1e-3) / 1e12
        sweeps = 1 if lse else 2
        res["roofline"].update({"bound": "mfma", "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                "frac": tf / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                                "executed_TFLOPs": tf * sweeps, "executed_frac": tf * sweeps / MFMA_BF16_PEAK_TFLOPS,
                                "hbm_frac": achieved / HBM_PEAK_GBPS})
    if want_read_probe:
        # Measured ceiling beside the published peak: one plain streaming read of every layer's K (the same bytes
        # the scoring kernel has to fetch), timed with events on the launch stream.
        sink = torch.zeros(1, dtype=torch.int32, device=dev)
        k_bytes_total = sum(K.numel() * K.element_size() for K in Ks)
        read_ms = []
        for rep in range(4):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for K in Ks:
                binding.probe_read(K, sink)
            e1.record()
            torch.cuda.synchronize()
            if rep > 0:
                read_ms.append(e0.elapsed_time(e1))
        read_gbps = k_bytes_total / (min(read_ms) * 1e-3) / 1e9
        if res["roofline"]["bound"] == "hbm":
            res["roofline"].update({"measured_read_GBps": read_gbps, "frac_of_measured_read": achieved / read_gbps})
    if total_bytes < (256 << 20):
        res["roofline"]["note"] = "inputs fit the memory-side cache: launch-bound, not an HBM figure"
    ctx = dict(call=call, ks=ks, lens=lens, lens_dev=lens_dev, layers_host=layers_host, Qs=Qs, Ks=Ks, Vs=Vs,
               lses=lses, paged=paged, sum_n=sum_n)
    return res, ctx


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2,
                    help="index into the workload list (default: the 32k config; 5: the multi-head long-context "
                         "measurement shape)")
    ap.add_argument("--avg-budget", type=int, default=None)
    ap.add_argument("--seq-len", type=int, default=None,
                    help="variant: the same workload at another context length (e.g. 131072); no cpu_baseline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-all-configs", action="store_true",
                    help="skip the short runs of the other four workloads (the all_configs array)")
    ap.add_argument("--lse", action="store_true",
                    help="variant: one-sweep scoring with the window queries' softmax denominators supplied "
                         "(computed beforehand, outside the timed region); not the headline configuration")
    ap.add_argument("--graph", action="store_true",
                    help="variant: the timed steps replay a HIP graph of the step instead of launching its kernels "
                         "one by one; not the headline configuration")
    ap.add_argument("--page-size", type=int, default=0,
                    help="variant: kept rows written into per-layer page pools of this page size through random "
                         "block tables (pkv_compress_layers_paged); not the headline configuration")
    ap.add_argument("--recall", action="store_true",
                    help="also report the attention recall rate of the kept sets (mean over layers, sequences and "
                         "KV heads) for the linear, geometric and uniform allocation of the same average budget, and "
                         "the time of the recall kernel; outside the timed region")
    ap.add_argument("--decode", action="store_true",
                    help="also time the step after the path: one decoding query per sequence attending over every "
                         "layer's compacted cache (pkv_decode_attention, one launch per layer, and "
                         "pkv_decode_attention_layers, one call for all layers); outside the timed region")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2406_02069_amd import binding, synth

    dev = "cuda:0"
    w = (synth.WORKLOADS + synth.EXTRA_WORKLOADS)[args.config]
    if args.seq_len is not None and args.seq_len != w.N:
        w = w.scaled(name=f"{w.name}@N{args.seq_len}", N=args.seq_len)
    else:
        args.seq_len = None
    avg = args.avg_budget or w.avg_budgets[0]
    variant = args.lse or args.page_size > 0 or args.seq_len is not None or args.graph
    if variant:
        args.no_cpu_baseline = True
        args.no_all_configs = True
    headline = args.config == 2 and not variant and args.avg_budget in (None, w.avg_budgets[0])
    if not headline:
        args.no_all_configs = True
    host_layers = () if args.no_cpu_baseline else tuple(range(w.L))[: 32]
    res, ctx = measure(w, avg, args.steps, args.warmup, dev, lse=args.lse, page_size=args.page_size,
                       host_layers=host_layers, graph=args.graph)
    call, ks, lens, lens_dev, paged = ctx["call"], ctx["ks"], ctx["lens"], ctx["lens_dev"], ctx["paged"]
    Qs, Ks, Vs, lses = ctx["Qs"], ctx["Ks"], ctx["Vs"], ctx["lses"]

    out = {
        "metric": METRIC +
                  (" [variant: softmax denominators supplied, one sweep]" if args.lse else "") +
                  (f" [variant: paged output, page size {args.page_size}]" if args.page_size > 0 else "") +
                  (f" [variant: context length {args.seq_len}]" if args.seq_len is not None else "") +
                  (" [variant: step replayed from a HIP graph]" if args.graph else ""),
        "value": res["value"],
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"],
        "ms_per_step_stat": res["ms_per_step_stat"],
        "ms_per_step_mean_wall": res["ms_per_step_mean_wall"],
        "ms_per_step_min": res["ms_per_step_min"], "ms_per_step_max": res["ms_per_step_max"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": res["config"],
        "whole_path": res["whole_path"],
        "roofline": res["roofline"],
        "kernel_ms_per_step": res["kernel_ms_per_step"],
    }
    if args.decode:
        import numpy as np
        outs = call.run()
        torch.cuda.synchronize()
        gq = torch.Generator(device=dev).manual_seed(99)
        qd = [torch.randn(w.B, w.Hq, w.d, generator=gq, device=dev).to(torch.bfloat16) for _ in range(w.L)]
        o_buf = torch.empty(w.B, w.Hq, w.d, dtype=torch.float32, device=dev)
        d_ws = torch.empty(64 << 20, dtype=torch.uint8, device=dev)   # ample for any shape here

        def decode_step():
            for l in range(w.L):
                if paged is not None:
                    binding.decode_attention(qd[l], outs[l][0], outs[l][1], outs[l][3], block_table=paged[2][l],
                                             k_cap=min(ks[l], w.N), out=o_buf, workspace=d_ws)
                else:
                    binding.decode_attention(qd[l], outs[l][0], outs[l][1], outs[l][3], out=o_buf, workspace=d_ws)

        for _ in range(20):
            decode_step()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            decode_step()
        e1.record()
        torch.cuda.synchronize()
        dms = e0.elapsed_time(e1) / args.steps
        rows = sum(int(o[3].clamp(min=0).sum()) for o in outs)          # kept rows over all layers and sequences
        dbytes = rows * w.Hkv * w.d * 2 * 2 + w.L * w.B * w.Hq * w.d * (2 + 4)
        out["decode_attention"] = {"ms_per_step": dms, "launches": w.L, "us_per_launch": dms * 1e3 / w.L,
                                   "algorithmic_bytes_per_step": dbytes,
                                   "achieved_GBps": dbytes / (dms * 1e-3) / 1e9,
                                   "frac_of_hbm_peak": dbytes / (dms * 1e-3) / 1e9 / HBM_PEAK_GBPS}
        # the same step through one call over all layers' caches (pkv_decode_attention_layers)
        if paged is not None:
            lc = binding.DecodeLayersCall(qd, [o[0] for o in outs], [o[1] for o in outs], [o[3] for o in outs],
                                          block_tables=list(paged[2]), k_caps=[min(k, w.N) for k in ks])
        else:
            lc = binding.DecodeLayersCall(qd, [o[0] for o in outs], [o[1] for o in outs], [o[3] for o in outs])
        for _ in range(20):
            lc.run()
        e0.record()
        for _ in range(args.steps):
            lc.run()
        e1.record()
        torch.cuda.synchronize()
        lms = e0.elapsed_time(e1) / args.steps
        out["decode_attention_layers"] = {"ms_per_step": lms, "calls": 1, "algorithmic_bytes_per_step": dbytes,
                                          "achieved_GBps": dbytes / (lms * 1e-3) / 1e9,
                                          "frac_of_hbm_peak": dbytes / (lms * 1e-3) / 1e9 / HBM_PEAK_GBPS}
    if args.recall:
        rec = {}
        for name, sched in (("linear", binding.SCHEDULE_LINEAR), ("geometric", binding.SCHEDULE_GEOMETRIC),
                            ("uniform", binding.SCHEDULE_UNIFORM)):
            ks_s = binding.budgets_schedule(w.L, avg, w.beta, w.alpha, sched)
            c = call if sched == binding.SCHEDULE_LINEAR else \
                binding.LayersCall(Qs, Ks, Vs, ks_s, w.pool, w.pool_w, seq_lens=lens_dev, lse=lses)
            c.run()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            r = binding.attention_recall(c)
            e1.record()
            torch.cuda.synchronize()
            rec[name] = float(torch.stack(r).mean())
            rec.setdefault("kernel_ms", e0.elapsed_time(e1))
            del c
        out["attention_recall"] = rec
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, ks, ctx["layers_host"], lens)
        # the same leg also checks the device's result on sampled layers against the oracle, outside any timing
        vl = sorted({0, w.L - 1, w.L // 2} & set(ctx["layers_host"]))
        out["verify"] = verify_against_oracle(w, ks, Qs, Ks, Vs, lens, lens_dev, call.outputs, vl)

    if not args.no_all_configs:
        # The other workloads of the configuration list, each measured the same way in a short run (they are
        # parity-test cases; the headline stays the line above), and the multi-head long-context shape (8 query
        # rows per head: what the padding of the rows to an MFMA tile costs per key).
        del call, Qs, Ks, Vs, lses, paged
        ctx.clear()
        gc.collect()
        torch.cuda.empty_cache()
        # The same workload through pkv_compress_layers_lse (denominators supplied by the caller's attention kernel;
        # here by tests/prefill_stub.py, outside any timing): a variant, reported beside the headline, never as it.
        r, c = measure(w, avg, 20, 10, dev, lse=True, want_read_probe=False)
        out["variant_supplied_denominators"] = {"ms_per_step": r["ms_per_step"], "value": r["value"], "unit": "tokens/s",
                                                "kernel_ms_per_step": r["kernel_ms_per_step"], "roofline": r["roofline"]}
        c.clear()
        del r, c
        gc.collect()
        torch.cuda.empty_cache()
        out["all_configs"] = []
        for ci in (0, 1, 3, 4, 5):
            wc = (synth.WORKLOADS + synth.EXTRA_WORKLOADS)[ci]
            r, c = measure(wc, wc.avg_budgets[0], 10, 5, dev, want_read_probe=False)
            out["all_configs"].append({"config": r["config"]["workload"], "ms_per_step": r["ms_per_step"],
                                       "value": r["value"], "unit": "tokens/s",
                                       "kernel_ms_per_step": r["kernel_ms_per_step"],
                                       "roofline": r["roofline"]})
            c.clear()
            del r, c
            gc.collect()
            torch.cuda.empty_cache()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
