"""Benchmark of the PyramidKV compression step on one MI355X.

A step = the whole hot path (budgets excluded: host, once) over one request batch: pkv_compress_layers over all L
layers of the workload -- window scoring, pooling, per-head top-k, K/V gather.  Inputs are resident in HBM.
Prints one JSON line (metric of the benchmark spec: compressed prefill tokens/s over all layers).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0       # MI355X HBM3E, published


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


def measured_traffic(kernel, workload, avg):
    """HBM bytes per launch from the committed rocprofv3 counter summary (profiles/traffic_bytes.txt), or None."""
    path = os.path.join(ROOT, "profiles", "traffic_bytes.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if len(f) == 4 and not line.startswith("#") and f[0] == kernel and f[1] == workload and int(f[2]) == avg:
            return int(f[3])
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", type=int, default=2, help="index into the workload list (default: the 32k config)")
    ap.add_argument("--avg-budget", type=int, default=None)
    ap.add_argument("--seq-len", type=int, default=None,
                    help="variant: the same workload at another context length (e.g. 131072); no cpu_baseline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--lse", action="store_true",
                    help="variant: one-sweep scoring with the window queries' softmax denominators supplied "
                         "(computed beforehand, outside the timed region); not the headline configuration")
    ap.add_argument("--page-size", type=int, default=0,
                    help="variant: kept rows written into per-layer page pools of this page size through random "
                         "block tables (pkv_compress_layers_paged); not the headline configuration")
    ap.add_argument("--recall", action="store_true",
                    help="also report the attention recall rate of the kept sets (mean over layers, sequences and "
                         "KV heads) for the linear, geometric and uniform allocation of the same average budget, and "
                         "the time of the recall kernel; outside the timed region")
    ap.add_argument("--decode", action="store_true",
                    help="also time the step after the path: one decoding query per sequence attending over every "
                         "layer's compacted cache (pkv_decode_attention, one launch per layer); outside the timed region")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2406_02069_amd import binding, synth

    dev = "cuda:0"
    w = synth.WORKLOADS[args.config]
    if args.seq_len is not None and args.seq_len != w.N:
        w = w.scaled(name=f"{w.name}@N{args.seq_len}", N=args.seq_len)
    else:
        args.seq_len = None
    avg = args.avg_budget or w.avg_budgets[0]
    ks = binding.budgets(w.L, avg, w.beta, w.alpha)
    lens = synth.seq_lens(w)
    sum_n = int(lens.sum()) if lens is not None else w.B * w.N
    lens_dev = None if lens is None else torch.from_numpy(lens).to(dev)

    # all layers resident in HBM; a bounded set of layers is also kept on the host for the oracle
    if args.lse or args.page_size > 0 or args.seq_len is not None:
        args.no_cpu_baseline = True
    n_host = 0 if args.no_cpu_baseline else min(w.L, 32)
    host_ids = sorted(set([0, w.L - 1] + list(range(1, w.L - 1))[: max(n_host - 2, 0)])) if n_host else []
    Qs, Ks, Vs, layers_host = [], [], [], {}
    for l in range(w.L):
        Q, K, V, _ = synth.make_layer(w, l, dev)
        Qs.append(Q), Ks.append(K), Vs.append(V)
        if l in host_ids:
            layers_host[l] = (Q.cpu(), K.cpu(), V.cpu())
    lses = None
    if args.lse:  # what the prefill attention kernel would hand over; an input, prepared before timing
        from tests import prefill_stub
        lses = [prefill_stub.window_lse(Qs[l], Ks[l], lens) for l in range(w.L)]
    paged = None
    if args.page_size > 0:  # every layer its own pool and block table; pages handed out in a seeded random order
        P = args.page_size
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

    for _ in range(args.warmup):
        call.run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        call.run()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    # Per-kernel device time: the same steps again, with HIP events around every kernel (recorded on the stream the
    # kernels run on).  Kept apart from the timed region above so that the event packets do not slow `value`.
    events = binding.HipEvents(5 * w.L + 1)
    per_kernel = {}
    for _ in range(args.steps):
        ids = binding.run_profiled(call, events)
        torch.cuda.synchronize()
        for i, kid in enumerate(ids):
            per_kernel.setdefault(kid, []).append(events.elapsed_ms(i, i + 1))
    events.close()
    avg_ms = {binding.KERNEL_NAMES[k]: float(np.mean(v)) for k, v in per_kernel.items()}
    sum_ms = {binding.KERNEL_NAMES[k]: float(np.sum(v)) / args.steps for k, v in per_kernel.items()}
    dominant = max(sum_ms, key=sum_ms.get)

    # Measured ceiling beside the published peak: one plain streaming read of every layer's K (the same bytes the
    # scoring kernel has to fetch), timed with events on the launch stream.
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

    total_bytes = sum(layer_bytes(w, k, sum_n) for k in ks)
    sweep_bytes = kernel_bytes(dominant, w, ks, sum_n)
    achieved = sweep_bytes / (avg_ms[dominant] * 1e-3) / 1e9
    out = {
        "metric": "compressed prefill tokens/sec (all layers, select+gather); achieved HBM GB/s" +
                  (" [variant: softmax denominators supplied, one sweep]" if args.lse else "") +
                  (f" [variant: paged output, page size {args.page_size}]" if args.page_size > 0 else "") +
                  (f" [variant: context length {args.seq_len}]" if args.seq_len is not None else ""),
        "value": sum_n / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: B{w.B} L{w.L} Hq{w.Hq} Hkv{w.Hkv} d{w.d} N{w.N} alpha{w.alpha} "
                               f"avg_budget{avg} beta{w.beta} pool{w.pool}/w{w.pool_w}" + (" +lse" if args.lse else "") + (f" +pages{args.page_size}" if args.page_size > 0 else ""),
                   "tokens_per_step": sum_n, "algorithmic_bytes_per_step": total_bytes},
        "whole_path": {"achieved_GBps": total_bytes / (ms_per_step * 1e-3) / 1e9,
                       "frac_of_hbm_peak": total_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS},
        "roofline": {"kernel": dominant, "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": measured_traffic(dominant + ("_lse" if args.lse else ""), w.name, avg),
                     "algorithmic_bytes_per_launch": sweep_bytes, "avg_launch_ms": avg_ms[dominant],
                     "measured_read_GBps": read_gbps, "frac_of_measured_read": achieved / read_gbps},
        "kernel_ms_per_step": sum_ms,
    }
    if args.decode:
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
        out["cpu_baseline"] = cpu_baseline(w, ks, layers_host, lens)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
