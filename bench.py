#!/usr/bin/env python3
"""Benchmark of the fused CD-SGD step on one MI355X.

A step is one pass of the whole hot path (quantise + pack own gradient, decode and
sum N packed streams, local and global update) over one batch of synthetic,
model-shaped gradients: one cdsgd_step_fused launch over the layer list.  The headline
workload is the VGG-16-shaped list (138 M fp32 parameters, N = 16 workers); the
ResNet-50-shaped list and the 4 GiB flat bucket are reported in "extra".

Prints ONE JSON line.  `value` is algorithmic GB/s = elements * (24 + N/4) bytes / step
time with every input already resident in HBM; compressed steps only (correction steps,
one in k, are timed separately and reported in "extra").
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM bytes per k_fused_compressed launch from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs of this
# file, scaled by the same counters' readings for a 1 GiB device copy (FETCH_SIZE x 2.0, WRITE_SIZE
# x 1.0 on this GPU); summaries in profiles/k_fused_compressed_<workload>.md.
MEASURED_TRAFFIC_BYTES = {"c4_vgg16": 3.8786e9, "c3_resnet50": 0.7170e9}


def _progress(msg):
    """Stage marker on stderr (stdout carries the one JSON line only)."""
    print("bench: " + msg, file=sys.stderr, flush=True)


def _compressed_steps(k, count, start=1):
    """`count` step numbers with step % k != 0."""
    out, s = [], start
    while len(out) < count:
        if s % k != 0:
            out.append(s)
        s += 1
    return out


def time_workload(name, steps, warmup, want_correction=True, want_unfused=False, grad_dtype=None):
    import torch
    from paper_2106_10796_amd import runner, synth
    cfg = synth.config(name)
    _progress("%s: building the workload and the peers' streams" % name)
    wl = runner.Workload(cfg, grad_dtype=grad_dtype or torch.float32)
    grad_bytes = 4 if grad_dtype in (None, torch.float32) else 2
    # inputs of a compressed step (own gradient, the peers' packed streams) and of a correction step
    if want_correction:
        wl.prepare_step(0)
    wl.prepare_step(1)
    wl.peer_residual = [None] * cfg.num_workers   # the peers are played; free their residuals
    wl._scratch = None
    torch.cuda.empty_cache()
    stream = torch.cuda.current_stream()

    def run(step_numbers, fn):
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for s in step_numbers:
            fn(s)
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / len(step_numbers)   # ms per step

    def per_step(step_numbers, fn):
        """One event pair per step: the median is robust against a stray slow step."""
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(len(step_numbers) + 1)]
        ev[0].record(stream)
        for i, s in enumerate(step_numbers):
            fn(s)
            ev[i + 1].record(stream)
        torch.cuda.synchronize()
        d = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(len(step_numbers)))
        return d[len(d) // 2], d[0]

    _progress("%s: timing %d fused steps" % (name, steps))
    run(_compressed_steps(cfg.k, max(warmup, 1)), wl.fused_step)
    ms = run(_compressed_steps(cfg.k, steps), wl.fused_step)
    med, best = per_step(_compressed_steps(cfg.k, max(10, min(steps, 40))), wl.fused_step)
    bpe = cfg.bytes_per_element - (4 - grad_bytes)        # 24 + N/4 with fp32 gradients, 22 + N/4 with 16-bit ones
    out = dict(workload=name, tensors=cfg.num_tensors, elements=cfg.elements, num_workers=cfg.num_workers,
               k=cfg.k, threshold=cfg.threshold, bytes_per_element=bpe,
               ms_per_step=ms, median_ms_per_step=med, min_ms_per_step=best,
               elems_per_s=cfg.elements / (ms * 1e-3),
               gbs=cfg.elements * bpe / (ms * 1e-3) / 1e9)
    out["frac_hbm_peak"] = out["gbs"] / HBM_PEAK_GBS
    if want_correction:
        run([0] * max(warmup, 1), wl.fused_step)
        ms_c = run([0] * max(3, steps // 4), wl.fused_step)
        out["correction_ms_per_step"] = ms_c
        out["correction_gbs"] = cfg.elements * (16.0 + grad_bytes) / (ms_c * 1e-3) / 1e9   # read W, g, agg; write W, Wloc
    if want_unfused:
        run(_compressed_steps(cfg.k, 1), wl.unfused_step)
        ms_u = run(_compressed_steps(cfg.k, max(2, steps // 4)), wl.unfused_step)
        out["threecall_ms_per_step"] = ms_u
        # delta of the paper's model: the worker-side compression alone (quantise + pack, one flat call)
        from paper_2106_10796_amd import binding
        qp = lambda s: binding.cdsgd_quantize_pack(wl.grad, wl.residual, wl.packed_self, cfg.threshold)
        run([1], qp)
        out["quantize_pack_ms"] = run([1] * max(3, steps // 4), qp)
    return out, wl


def time_small(name, steps=200):
    """Launch-bound workloads (everything fits in cache): microseconds per fused step, called
    eagerly and replayed from a HIP graph that holds one period of k steps."""
    import torch
    from paper_2106_10796_amd import runner, synth
    cfg = synth.config(name)
    wl = runner.Workload(cfg)
    wl.prepare_step(0)
    wl.prepare_step(1)
    period = list(range(cfg.k))
    reps = max(1, steps // cfg.k)

    def run_period():
        for s in period:
            wl.fused_step(s)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / (reps * cfg.k) * 1e6

    eager_us = timed(run_period)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run_period()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run_period()
    graph_us = timed(graph.replay)
    wl.destroy()
    return {"workload": name, "tensors": cfg.num_tensors, "elements": cfg.elements,
            "us_per_step_eager": eager_us, "us_per_step_hip_graph": graph_us,
            "note": "one period of k steps (1 correction + k-1 compressed) per graph; wall clock incl. launch"}


def time_correction_sum(name, steps, warmup):
    """Correction pass that sums the N workers' fp32 gradients in the kernel (Alg. 1, else-branch):
    reads W and N gradients, writes W and W_loc = 12 + 4N bytes per element."""
    import torch
    from paper_2106_10796_amd import runner, synth
    cfg = synth.config(name)
    wl = runner.Workload(cfg, peer_residuals=False, full_grads=True)
    wl.prepare_step(0)
    stream = torch.cuda.current_stream()
    for _ in range(max(warmup, 1)):
        wl.fused_step(0)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(steps):
        wl.fused_step(0)
    e1.record(stream)
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    bpe = 12.0 + 4.0 * cfg.num_workers
    wl.destroy()
    return {"ms_per_step": ms, "bytes_per_element": bpe, "gbs": cfg.elements * bpe / (ms * 1e-3) / 1e9,
            "frac_hbm_peak": cfg.elements * bpe / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}


def overlap_demo(name, iters=12):
    """Overhead hiding on one GPU (Sec. 3.2.2, Fig. 5): the next forward pass only needs the local
    weights.  Fused form: forward stand-in waits for the whole fused step.  Split form: stream L
    runs cdsgd_step_local and then the forward stand-in, stream G runs cdsgd_step_global behind an
    event; the next iteration's local update waits for G.  The stand-in is a compute-bound bf16
    matrix product; both streams have the default priority."""
    import torch
    from paper_2106_10796_amd import runner, synth
    cfg = synth.config(name)
    wl = runner.Workload(cfg)
    wl.prepare_step(1)
    wl.peer_residual = [None] * cfg.num_workers
    wl._scratch = None
    torch.cuda.empty_cache()
    M = 8192
    x = torch.randn(M, M, device="cuda", dtype=torch.bfloat16)
    y = torch.randn(M, M, device="cuda", dtype=torch.bfloat16)
    z = torch.empty(M, M, device="cuda", dtype=torch.bfloat16)
    main = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    steps = _compressed_steps(cfg.k, iters)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(main)
        fn()
        e1.record(main)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    def only(fn):
        return lambda: [fn(s) for s in steps]

    def fused_then_forward():
        for s in steps:
            wl.fused_step(s)
            torch.mm(x, y, out=z)

    def split_serial():
        for s in steps:
            wl.plan.step_local(cfg.lr)
            torch.mm(x, y, out=z)
            wl.plan.step_global(s, cfg.k, cfg.threshold, cfg.lr)

    def split_overlapped():
        g_done = None
        for s in steps:
            if g_done is not None:
                main.wait_event(g_done)            # next local update reads the new global weights
            wl.plan.step_local(cfg.lr)
            l_done = torch.cuda.Event()
            l_done.record(main)
            torch.mm(x, y, out=z)                  # forward stand-in, needs only w_local
            with torch.cuda.stream(side):
                side.wait_event(l_done)
                wl.plan.step_global(s, cfg.k, cfg.threshold, cfg.lr)
                g_done = torch.cuda.Event()
                g_done.record(side)
        main.wait_event(g_done)

    out = {
        "workload": name, "forward_stand_in": "bf16 %dx%dx%d matrix product" % (M, M, M),
        "ms_fused_step": timed(only(wl.fused_step)),
        "ms_step_local": timed(only(lambda s: wl.plan.step_local(cfg.lr))),
        "ms_step_global": timed(only(lambda s: wl.plan.step_global(s, cfg.k, cfg.threshold, cfg.lr))),
        "ms_forward_stand_in": timed(only(lambda s: torch.mm(x, y, out=z))),
        "ms_iter_fused_then_forward": timed(fused_then_forward),
        "ms_iter_split_one_stream": timed(split_serial),
        "ms_iter_split_two_streams": timed(split_overlapped),
    }
    out["forward_can_start_after_ms"] = {"fused": out["ms_fused_step"], "split": out["ms_step_local"]}
    wl.destroy()
    return out


def cpu_baseline(wl, target_seconds=40.0):
    """The oracle as it stands, timed on this host: worker 0's fused-equivalent work
    (quantise + pack own gradient, decode-and-sum N streams, both updates) on a bounded
    sample of the same workload, split over the host cores by element range (the work is
    elementwise, so the split changes nothing)."""
    import concurrent.futures as cf

    import numpy as np
    from oracle import cdsgd_oracle as O
    cfg = wl.cfg
    N, t = cfg.num_workers, cfg.threshold
    cores = max(1, min(int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)), os.cpu_count() or 1))
    big = max(range(cfg.num_tensors), key=lambda i: cfg.sizes[i])
    avail = cfg.sizes[big] // 16 * 16

    def sample(n):
        """Inputs of the sample, none of them produced by the HIP path: the own gradient and the
        weights are the synthetic buffers; each peer's packed words are made here by the oracle from
        a rotated copy of the same gradient values (same distribution, different alignment)."""
        sl = slice(0, n)
        g = wl.view(wl.grad, big)[sl].cpu().numpy()
        r = np.zeros(n, np.float32)
        W = wl.view(wl.w_global, big)[sl].cpu().numpy()
        peers = []
        for j in range(N):
            if j == wl.self_rank:
                peers.append(None)
                continue
            gj = np.ascontiguousarray(np.roll(g, 4099 * (j + 1)))
            peers.append(O.quantize_pack(gj, np.zeros(n, np.float32), t))
        return g, r, W, peers

    def work(g, r, W, peers, lo, hi):
        words = O.quantize_pack(g[lo:hi], r[lo:hi], t)
        streams = [words if p is None else np.ascontiguousarray(p[lo // 16: hi // 16]) for p in peers]
        agg = O.decode_sum(streams, hi - lo, t)
        Wl = np.empty(hi - lo, np.float32)
        O.update(W[lo:hi], Wl, g[lo:hi], agg, cfg.lr, cfg.lr, N)

    n_max = min(avail, 1 << 24)
    G, R0, W0, PEERS = sample(n_max)

    def timed(n, threads=None):
        threads = threads or cores
        n = max(16 * threads, min(n, n_max) // (16 * threads) * (16 * threads))
        r = R0[:n].copy()          # each pass starts from a zero residual
        W = W0[:n].copy()
        per = n // threads
        t0 = time.perf_counter()
        with cf.ThreadPoolExecutor(threads) as ex:
            futs = [ex.submit(work, G, r, W, PEERS, c * per, (c + 1) * per) for c in range(threads)]
            for f in futs:
                f.result()
        return n, time.perf_counter() - t0

    # about `target_seconds` of CPU work in total (all cores together), as repeated passes over the sample
    timed(1 << 20)                                              # warm the threads and the page cache
    n1, dt_first = timed(n_max)
    reps = max(1, int(round(target_seconds / (cores * max(dt_first, 1e-6)))))
    dt1 = 0.0
    for _ in range(reps):
        n1, dt = timed(n1)
        dt1 += dt
    dt1 /= reps
    gbs = n1 * cfg.bytes_per_element / dt1 / 1e9
    n_one, dt_one = timed(max(1 << 20, n1 // 4), threads=1)          # the same loop on one core
    return {"value": gbs, "unit": "GB/s", "cores": cores, "kind": "oracle",
            "elems_per_s": n1 / dt1,
            "one_core": {"value": n_one * cfg.bytes_per_element / dt_one / 1e9, "unit": "GB/s",
                         "elems_per_s": n_one / dt_one, "sample_elements": n_one},
            "sample": "first %d elements of tensor %d of %s, one compressed step of worker 0 "
                      "(quantise+pack, decode-sum of %d streams, both updates), mean of %d passes of %.2f s wall"
                      % (n1, big, cfg.name, N, reps, dt1)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c4_vgg16")
    ap.add_argument("--no-extra", action="store_true", help="skip the ResNet-50 and 4 GiB workloads")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run a plain device copy of known size (1 GiB read + 1 GiB written, 3 times): "
                         "under rocprofv3 --pmc its FETCH_SIZE / WRITE_SIZE readings give the counters' scale")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; the other workers' packed gradients are generated "
              "on the same device and nothing is sharded, so --gpus must be 1", file=sys.stderr)
        return 2
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    from paper_2106_10796_amd import binding, build as hip_build
    hip_build.ensure_built()
    binding.lib()   # the HIP library or nothing: there is no other path

    _progress("start")
    if args.calib_copy:
        src = torch.randn(1 << 28, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()
    head, wl = time_workload(args.workload, args.steps, args.warmup, want_correction=True,
                             want_unfused=not args.no_extra)
    cpu = None
    if not args.no_cpu_baseline:
        _progress("cpu baseline (oracle on the host cores)")
        cpu = cpu_baseline(wl)
    wl.destroy()
    del wl
    torch.cuda.empty_cache()
    extra = {"headline": head}
    if not args.no_extra:
        _progress("extras: correction with kernel sum, overlap, small workloads, bf16 gradients, other workloads")
        extra["correction_with_kernel_sum_" + args.workload] = time_correction_sum(
            args.workload, max(3, args.steps // 4), max(1, args.warmup // 2))
        torch.cuda.empty_cache()
        extra["overlap_demo"] = overlap_demo(args.workload)
        torch.cuda.empty_cache()
        for name in ("c1_single", "c2_resnet20"):
            extra[name] = time_small(name)
        r, w = time_workload(args.workload, max(5, args.steps // 2), max(2, args.warmup // 2),
                             want_correction=False, grad_dtype=torch.bfloat16)
        w.destroy()
        del w
        torch.cuda.empty_cache()
        extra["bf16_gradients_" + args.workload] = r
        # the paper's time model (Sec. 3.3) fed with the measured delta; tau and the wire are assumptions
        n_el, k = head["elements"], head["k"]
        wire = 56e9 / 8                                   # the paper's 56 Gbps InfiniBand, bytes/s
        assume = {"tau_ms": 100.0, "phi_ms": 2 * 4 * n_el / wire * 1e3,           # push fp32 + pull fp32
                  "psi_ms": (n_el / 4 + 4 * n_el) / wire * 1e3,                    # push 2-bit + pull fp32
                  "delta_ms": head["quantize_pack_ms"], "k": k}
        extra["time_model"] = {
            "assumptions": "tau = 100 ms (not measured: no FP/BP here); parameter-server wire at 56 Gbps: "
                           "phi = 8n B, psi = (n/4 + 4n) B; delta = measured cdsgd_quantize_pack time",
            "inputs": assume,
            "period_mean": binding.cdsgd_cost_period_mean(assume["tau_ms"], assume["phi_ms"], assume["psi_ms"],
                                                          assume["delta_ms"], k)}
        for name in ("c3_resnet50", "c5_flat4g"):
            if name == args.workload:
                continue
            r, w = time_workload(name, max(5, args.steps // 2), max(2, args.warmup // 2),
                                 want_correction=(name != "c5_flat4g"))
            w.destroy()
            del w
            torch.cuda.empty_cache()
            extra[name] = r

    bytes_per_launch = head["elements"] * head["bytes_per_element"]
    line = {
        "metric": "fused CD-SGD step GB/s and gradient elems/s on 1 MI355X; % of HBM peak",
        "value": head["gbs"], "unit": "GB/s",
        "elems_per_s": head["elems_per_s"],
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: VGG-16-shaped layer list" % head["workload"] if head["workload"] == "c4_vgg16"
                   else head["workload"],
                   "tensors": head["tensors"], "elements": head["elements"],
                   "num_workers": head["num_workers"], "k": head["k"], "threshold": head["threshold"],
                   "step": "compressed (step % k != 0), one cdsgd_step_fused launch"},
        "roofline": {"bound": "hbm", "kernel": "k_fused_compressed",
                     "achieved": bytes_per_launch / (head["ms_per_step"] * 1e-3) / 1e9,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": bytes_per_launch / (head["ms_per_step"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(head["workload"])},
        "cpu_baseline": cpu,
        "extra": extra,
        "paper_context": "end-to-end time 30% below 2-bit compression on a 16-GPU MXNet cluster at 56 Gbps "
                         "(abstract; another system, not comparable)",
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
