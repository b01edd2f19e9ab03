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

Timing: after --warmup untimed steps, blocks of exactly --steps fused steps run back to back on
the stream the kernels are launched on, with a HIP event between blocks and no host
synchronisation inside the run, until at least 10 blocks and at least one second of GPU time
have gone by.  `ms_per_step` is the MEDIAN block's time per step: a sustained figure.  The
first and the last block (a GPU that has just been idle clocks higher than one under sustained
load), the fastest and the slowest are in extra.headline.blocks.
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

# HBM bytes per k_fused_compressed launch.  NOT measured by this run: constants taken from earlier
# rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs of this file, scaled by the same counters' readings
# for a 1 GiB device copy (FETCH_SIZE x 2.0, WRITE_SIZE x 1.0 on this GPU); the summaries are
# profiles/k_fused_compressed_<workload>.md (c3_resnet50: read side from the current kernel, write
# side from an earlier build with the same stores).
PROFILED_TRAFFIC_BYTES = {"c4_vgg16": 3.8786e9, "c3_resnet50": 0.7169e9, "c5_flat4g": 30.098e9}
MIN_TIMED_SECONDS = 1.0     # sustained: the timed blocks of the headline cover at least this much GPU time
MIN_BLOCKS = 10


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


def timed_blocks(run_block, steps, stream, min_seconds=MIN_TIMED_SECONDS, min_blocks=MIN_BLOCKS, max_blocks=2000):
    """Blocks of `steps` launches back to back on `stream`, an event between blocks, one host
    synchronisation at the end.  The number of blocks is chosen from one untimed block so that the
    run covers min_seconds of GPU time and at least min_blocks blocks."""
    import torch
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    run_block()
    e1.record(stream)
    torch.cuda.synchronize()
    est_ms = max(e0.elapsed_time(e1), 1e-3)
    n = int(min(max_blocks, max(min_blocks, -(-min_seconds * 1e3 // est_ms))))
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
    ev[0].record(stream)
    for b in range(n):
        run_block()
        ev[b + 1].record(stream)
    torch.cuda.synchronize()
    per = [ev[b].elapsed_time(ev[b + 1]) / steps for b in range(n)]      # ms per step, block by block
    srt = sorted(per)
    return {"blocks": n, "steps_per_block": steps, "timed_seconds": sum(per) * steps * 1e-3,
            "median_ms_per_step": srt[n // 2] if n % 2 else 0.5 * (srt[n // 2 - 1] + srt[n // 2]),
            "first_block_ms_per_step": per[0], "last_block_ms_per_step": per[-1],
            "min_block_ms_per_step": srt[0], "max_block_ms_per_step": srt[-1],
            "mean_ms_per_step": sum(per) / n}


def time_workload(name, steps, warmup, want_correction=True, want_unfused=False, grad_dtype=None,
                  min_seconds=MIN_TIMED_SECONDS, sparse_peers=False, dense=False):
    import torch
    from paper_2106_10796_amd import runner, synth
    cfg = synth.config(name)
    _progress("%s: building the workload and the peers' streams" % name)
    wl = runner.Workload(cfg, grad_dtype=grad_dtype or torch.float32, sparse_peers=sparse_peers, dense=dense)
    grad_bytes = 4 if grad_dtype in (None, torch.float32) else 2
    # inputs of a compressed step (own gradient, the peers' packed streams) and of a correction step
    if want_correction:
        wl.prepare_step(0)
    wl.prepare_step(1)
    wl.peer_residual = [None] * cfg.num_workers   # the peers are played; free their residuals
    wl._scratch = None
    torch.cuda.empty_cache()
    stream = torch.cuda.current_stream()

    def run(step_numbers, fn, min_seconds=0.0):
        """ms per call of fn over the given step numbers, repeated back to back until min_seconds of
        GPU time have gone by (one event pair around everything)."""
        torch.cuda.synchronize()
        total_ms, calls = 0.0, 0
        while True:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for s in step_numbers:
                fn(s)
            e1.record(stream)
            torch.cuda.synchronize()
            total_ms += e0.elapsed_time(e1)
            calls += len(step_numbers)
            if total_ms >= min_seconds * 1e3:
                return total_ms / calls

    _progress("%s: timing blocks of %d fused steps" % (name, steps))
    block_steps = _compressed_steps(cfg.k, steps)
    run(_compressed_steps(cfg.k, max(warmup, 1)), wl.fused_step)
    blocks = timed_blocks(lambda: [wl.fused_step(s) for s in block_steps], steps, stream, min_seconds)
    ms = blocks["median_ms_per_step"]
    bpe = cfg.bytes_per_element - (4 - grad_bytes)        # 24 + N/4 with fp32 gradients, 22 + N/4 with 16-bit ones
    out = dict(workload=name, tensors=cfg.num_tensors, elements=cfg.elements, num_workers=cfg.num_workers,
               k=cfg.k, threshold=cfg.threshold, bytes_per_element=bpe,
               ms_per_step=ms, blocks=blocks,
               elems_per_s=cfg.elements / (ms * 1e-3),
               gbs=cfg.elements * bpe / (ms * 1e-3) / 1e9)
    out["frac_hbm_peak"] = out["gbs"] / HBM_PEAK_GBS
    if want_correction:
        run([0] * max(warmup, 1), wl.fused_step)
        ms_c = run([0] * max(3, steps // 4), wl.fused_step, min_seconds=0.3)
        out["correction_ms_per_step"] = ms_c
        out["correction_gbs"] = cfg.elements * (16.0 + grad_bytes) / (ms_c * 1e-3) / 1e9   # read W, g, agg; write W, Wloc
    if want_unfused:
        run(_compressed_steps(cfg.k, 1), wl.unfused_step)
        ms_u = run(_compressed_steps(cfg.k, max(2, steps // 4)), wl.unfused_step, min_seconds=0.3)
        out["threecall_ms_per_step"] = ms_u
        # delta of the paper's model: the worker-side compression alone (quantise + pack, one flat call)
        from paper_2106_10796_amd import binding
        qp = lambda s: binding.cdsgd_quantize_pack(wl.grad, wl.residual, wl.packed_self, cfg.threshold)
        run([1], qp)
        out["quantize_pack_ms"] = run([1] * max(3, steps // 4), qp, min_seconds=0.2)
    return out, wl


def stream_ceilings(wl, min_seconds=0.3):
    """What plain streaming kernels reach on this GPU, on the same arenas and in the same run, for
    comparison with the library's kernels.  Two families: the library's own bare streaming kernel
    (cdsgd_probe_streams: the loads, stores and launch shape of its passes on 32-bit gradients, no
    arithmetic) for several mixes of read and write streams, and torch's elementwise kernels (fill,
    sum, copy, add).  Harness, not product: nothing here is on the path that is being measured."""
    import torch
    from paper_2106_10796_amd import binding
    stream = torch.cuda.current_stream()
    n = wl.w_global.numel()
    a, b, g = wl.w_global, wl.residual, wl.grad                      # read only (the CPU baseline still needs them)
    c, d = wl.w_local, wl.agg_full                                   # free to overwrite now
    e = torch.empty_like(c)
    sink = torch.zeros(n // 256, dtype=torch.float32, device=c.device)
    fp32_grad = g.dtype == torch.float32
    ops = {"fill_write_only": (lambda: c.fill_(1.0), 4.0 * n),
           "sum_read_only": (lambda: torch.sum(a), 4.0 * n),
           "copy_1r_1w": (lambda: c.copy_(a), 8.0 * n),
           "add_2r_1w": (lambda: torch.add(a, b, out=c), 12.0 * n)}
    probe = {"probe_1r_0w": ([a], []), "probe_0r_1w": ([], [c]), "probe_1r_1w": ([a], [c]), "probe_2r_1w": ([a, b], [c])}
    if fp32_grad:
        probe.update({"probe_3r_0w": ([a, b, g], []), "probe_3r_2w": ([a, b, g], [c, d]),
                      "probe_3r_3w": ([a, b, g], [c, d, e])})
    for name, (rd, wr) in probe.items():
        ops[name] = ((lambda rd=rd, wr=wr: binding.cdsgd_probe_streams(rd, wr, sink)), 4.0 * n * (len(rd) + len(wr)))
    if fp32_grad:
        # the same mixes with the resident waves per compute unit bounded (LDS asked for and not used), the
        # knob the library's single-wave kernels are launched with: 20, 13 and 10 waves instead of 32
        for lds, waves in ((8192, 20), (12288, 13), (16384, 10)):
            for tag in ("probe_3r_2w", "probe_3r_3w"):
                rd, wr = probe[tag]
                ops["%s_%dwaves" % (tag, waves)] = (
                    (lambda rd=rd, wr=wr, lds=lds: binding.cdsgd_probe_streams(rd, wr, sink, lds_bytes=lds)),
                    4.0 * n * (len(rd) + len(wr)))
    out = {"elements": n,
           "note": "GB/s of bare streaming on the workload's own fp32 arenas, >= %.1f s each, after the headline (warm "
                   "GPU): probe_<R>r_<W>w = the library's streaming probe with R read and W write streams "
                   "(cdsgd_probe_streams), _<K>waves = at most K waves resident per compute unit; the others torch's "
                   "elementwise kernels" % min_seconds}
    for name, (fn, nbytes) in ops.items():
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        total_ms, calls = 0.0, 0
        while total_ms < min_seconds * 1e3:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(20):
                fn()
            e1.record(stream)
            torch.cuda.synchronize()
            total_ms += e0.elapsed_time(e1)
            calls += 20
        out[name + "_gbs"] = nbytes / (total_ms / calls * 1e-3) / 1e9
    del e, sink
    torch.cuda.empty_cache()
    return out


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


def layer_by_layer(name, steps, min_seconds=0.3):
    """The compressed pass enqueued layer by layer, last layer first, as back-propagation would deliver
    the gradients (Sec. 3.2.2), against the one-launch pass over the whole list: one range per tensor,
    and ranges grouped into buckets of at least 4 Mi elements.  ms per iteration of the whole list."""
    import torch
    from paper_2106_10796_amd import runner, synth
    cfg = synth.config(name)
    wl = runner.Workload(cfg)
    wl.prepare_step(1)
    wl.peer_residual = [None] * cfg.num_workers
    wl._scratch = None
    torch.cuda.empty_cache()
    stream = torch.cuda.current_stream()
    T, c = cfg.num_tensors, cfg
    buckets, hi, acc = [], T, 0
    for i in range(T - 1, -1, -1):
        acc += cfg.sizes[i]
        if acc >= (4 << 20) or i == 0:
            buckets.append((i, hi - i))
            hi, acc = i, 0
    forms = {"whole_list_one_launch": lambda: wl.plan.step(1, c.k, c.threshold, c.lr, c.lr),
             "one_range_per_tensor": lambda: [wl.plan.step_range(i, 1, 1, c.k, c.threshold, c.lr, c.lr)
                                              for i in range(T - 1, -1, -1)],
             "buckets_of_4Mi_elements": lambda: [wl.plan.step_range(lo, cnt, 1, c.k, c.threshold, c.lr, c.lr)
                                                 for lo, cnt in buckets]}
    out = {"workload": name, "tensors": T, "buckets": len(buckets)}
    for tag, fn in forms.items():
        fn()
        b = timed_blocks(lambda: [fn() for _ in range(steps)], steps, stream, min_seconds=min_seconds, min_blocks=5)
        out["ms_" + tag] = b["median_ms_per_step"]
    # the per-tensor launches again, replayed from a HIP graph (the launches cost the host nothing then)
    side = torch.cuda.Stream()
    side.wait_stream(stream)
    with torch.cuda.stream(side):
        forms["one_range_per_tensor"]()
    stream.wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        forms["one_range_per_tensor"]()
    graph.replay()
    b = timed_blocks(lambda: [graph.replay() for _ in range(steps)], steps, stream, min_seconds=min_seconds, min_blocks=5)
    out["ms_one_range_per_tensor_hip_graph"] = b["median_ms_per_step"]
    del graph
    wl.destroy()
    return out


def time_correction_sum(name, steps, warmup, min_seconds=0.5):
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
    blocks = timed_blocks(lambda: [wl.fused_step(0) for _ in range(steps)], steps, stream, min_seconds=min_seconds,
                          min_blocks=5)
    ms = blocks["median_ms_per_step"]
    bpe = 12.0 + 4.0 * cfg.num_workers
    out = {"ms_per_step": ms, "blocks": blocks, "bytes_per_element": bpe,
           "gbs": cfg.elements * bpe / (ms * 1e-3) / 1e9,
           "frac_hbm_peak": cfg.elements * bpe / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    # the same mix of streams moved by the bare streaming probe: N + 1 reads (W, N gradients), 2 writes
    if wl.grad.dtype == torch.float32 and cfg.num_workers + 1 <= 17:
        from paper_2106_10796_amd import binding
        reads = [wl.w_global, wl.grad] + [g for g in wl.peer_grad if g is not None]
        writes = [wl.w_local, wl.agg_full]
        probe = lambda: [binding.cdsgd_probe_streams(reads, writes) for _ in range(steps)]
        probe()
        pb = timed_blocks(probe, steps, stream, min_seconds=min_seconds, min_blocks=5)
        nbytes = 4.0 * wl.w_global.numel() * (len(reads) + len(writes))
        out["bare_streaming_same_mix"] = {"reads": len(reads), "writes": len(writes), "ms": pb["median_ms_per_step"],
                                          "gbs": nbytes / (pb["median_ms_per_step"] * 1e-3) / 1e9,
                                          "note": "cdsgd_probe_streams on the same arenas (pad included)"}
    wl.destroy()
    return out


def overlap_demo(name, iters=16):
    """Overhead hiding on one GPU (Sec. 3.2.2, Fig. 5): the next forward pass only needs the local
    weights.  Fused form: the forward stand-in waits for the whole fused step.  Split form: stream L
    runs cdsgd_step_local and then the forward stand-in, stream G runs cdsgd_step_global behind an
    event; the next iteration's local update waits for G.  Both streams have the default priority.
    cdsgd_step_global is run with one workgroup per chunk and with bounded grids
    (cdsgd_plan_set_max_workgroups), which leave compute units to the stand-in.  Two stand-ins:
    one bf16 matrix product that fills every compute unit, and a chain of small products that
    does not (a small-batch forward pass)."""
    import torch
    from paper_2106_10796_amd import runner, synth
    cfg = synth.config(name)
    wl = runner.Workload(cfg)
    wl.prepare_step(1)
    wl.peer_residual = [None] * cfg.num_workers
    wl._scratch = None
    torch.cuda.empty_cache()
    main = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    steps = _compressed_steps(cfg.k, iters)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        out = []
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(main)
            fn()
            e1.record(main)
            torch.cuda.synchronize()
            out.append(e0.elapsed_time(e1) / iters)
        return sorted(out)[1]

    def only(fn):
        return lambda: [fn(s) for s in steps]

    def make_stand_in(kind):
        if kind == "full_chip":
            M = 8192
            x = torch.randn(M, M, device="cuda", dtype=torch.bfloat16)
            y = torch.randn(M, M, device="cuda", dtype=torch.bfloat16)
            z = torch.empty(M, M, device="cuda", dtype=torch.bfloat16)
            return "one bf16 %dx%dx%d matrix product" % (M, M, M), lambda: torch.mm(x, y, out=z)
        # a forward pass that does NOT fill the chip: small products (at most 64 output tiles each), replayed
        # from a HIP graph so that the GPU, not the host's launch rate, sets their pace
        M, reps = 1024, 48
        x = torch.randn(M, M, device="cuda", dtype=torch.bfloat16)
        y = torch.randn(M, M, device="cuda", dtype=torch.bfloat16)
        z = torch.empty(M, M, device="cuda", dtype=torch.bfloat16)
        label = "%d bf16 %dx%dx%d matrix products in a row" % (reps, M, M, M)
        try:
            cap = torch.cuda.Stream()
            cap.wait_stream(main)
            with torch.cuda.stream(cap):
                for _ in range(3):
                    torch.mm(x, y, out=z)
            main.wait_stream(cap)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=cap):
                for _ in range(reps):
                    torch.mm(x, y, out=z)
            torch.cuda.synchronize()
            return label + ", replayed from a HIP graph", graph.replay
        except Exception as exc:                         # capture not possible: launch them one by one
            return label + " (eager: graph capture failed: %s)" % type(exc).__name__, \
                lambda: [torch.mm(x, y, out=z) for _ in range(reps)]

    def masked_stream(word):
        """A default-priority stream whose kernels may only run on the compute units named by a mask
        (hipExtStreamCreateWithCUMask): the same 32-bit word for each of 8 groups of 32 compute units."""
        import ctypes
        try:
            hip = ctypes.CDLL("libamdhip64.so")
            st = ctypes.c_void_p()
            arr = (ctypes.c_uint32 * 8)(*([word] * 8))
            if hip.hipExtStreamCreateWithCUMask(ctypes.byref(st), 8, arr) != 0 or not st.value:
                return None
            return torch.cuda.ExternalStream(st.value), (hip, st)
        except Exception:
            return None

    wl.plan.set_max_workgroups(0)
    out = {"workload": name,
           "ms_fused_step": timed(only(wl.fused_step)),
           "ms_step_local": timed(only(lambda s: wl.plan.step_local(cfg.lr))),
           "ms_step_global": timed(only(lambda s: wl.plan.step_global(s, cfg.k, cfg.threshold, cfg.lr))),
           "stand_ins": {}}
    out["forward_can_start_after_ms"] = {"fused": out["ms_fused_step"], "split": out["ms_step_local"]}
    limits = [0, 4096, 2048, 1024, 512, 256]
    for kind in ("full_chip", "partial_chip"):
        label, forward = make_stand_in(kind)

        def fused_then_forward():
            for s in steps:
                wl.fused_step(s)
                forward()

        def split_serial():
            for s in steps:
                wl.plan.step_local(cfg.lr)
                forward()
                wl.plan.step_global(s, cfg.k, cfg.threshold, cfg.lr)

        def split_overlapped(side=side):
            g_done = None
            for s in steps:
                if g_done is not None:
                    main.wait_event(g_done)            # next local update reads the new global weights
                wl.plan.step_local(cfg.lr)
                l_done = torch.cuda.Event()
                l_done.record(main)
                with torch.cuda.stream(side):
                    side.wait_event(l_done)
                    wl.plan.step_global(s, cfg.k, cfg.threshold, cfg.lr)
                    g_done = torch.cuda.Event()
                    g_done.record(side)
                forward()                              # forward stand-in, needs only w_local
            main.wait_event(g_done)

        r = {"forward_stand_in": label, "ms_forward_stand_in": timed(only(lambda s: forward()))}
        r["ms_iter_fused_then_forward"] = timed(fused_then_forward)
        r["ms_iter_split_one_stream"] = timed(split_serial)
        r["ms_iter_ideal_overlap"] = out["ms_step_local"] + max(r["ms_forward_stand_in"], out["ms_step_global"])
        two = {}
        for lim in limits:
            wl.plan.set_max_workgroups(lim)
            two["per_chunk" if lim == 0 else str(lim)] = {
                "ms_step_global_alone": timed(only(lambda s: wl.plan.step_global(s, cfg.k, cfg.threshold, cfg.lr))),
                "ms_iter_split_two_streams": timed(split_overlapped)}
        wl.plan.set_max_workgroups(0)
        r["two_streams_by_workgroup_limit_of_step_global"] = two
        # the same schedule with cdsgd_step_global on a stream confined to a share of the compute units
        masked = {}
        for share, word in (("64_of_256_cus", 0x000000FF), ("128_of_256_cus", 0x0000FFFF), ("192_of_256_cus", 0x00FFFFFF)):
            ms = masked_stream(word)
            if ms is None:
                masked[share] = None
                continue
            stream_m, (hip, handle) = ms

            def global_on_masked():
                with torch.cuda.stream(stream_m):
                    for s in steps:
                        wl.plan.step_global(s, cfg.k, cfg.threshold, cfg.lr)
                main.wait_stream(stream_m)
            stream_m.wait_stream(main)
            masked[share] = {"ms_step_global_alone": timed(global_on_masked),
                             "ms_iter_split_two_streams": timed(lambda: split_overlapped(stream_m))}
            torch.cuda.synchronize()
            hip.hipStreamDestroy(handle)
        r["two_streams_with_step_global_on_a_cu_masked_stream"] = masked
        cands = {("workgroup_limit", q): v["ms_iter_split_two_streams"] for q, v in two.items()}
        cands.update({("cu_mask", q): v["ms_iter_split_two_streams"] for q, v in masked.items() if v})
        best = min(cands, key=cands.get)
        r["best_two_streams"] = {best[0]: best[1], "ms_iter": cands[best],
                                 "vs_fused_then_forward": cands[best] / r["ms_iter_fused_then_forward"]}
        out["stand_ins"][kind] = r
    wl.destroy()
    return out


def cpu_baseline(wl, target_seconds=20.0):
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
    ap.add_argument("--min-seconds", type=float, default=MIN_TIMED_SECONDS,
                    help="GPU time the timed blocks of the headline must cover (default %(default)s; profiler runs "
                         "that collect counters per dispatch pass a small value to keep the dispatch count low)")
    ap.add_argument("--only-correction-sum", action="store_true",
                    help="time only the correction pass that sums the N gradients in the kernel (for profiling "
                         "k_fused_full<true, ...> on its own) and print its figures instead of the benchmark line")
    ap.add_argument("--only-layer-by-layer", action="store_true",
                    help="time only the compressed pass enqueued layer by layer (cdsgd_step_fused_range) against the "
                         "one-launch pass and print those figures instead of the benchmark line")
    ap.add_argument("--only-stream-ceilings", action="store_true",
                    help="time the headline workload and the bare streaming kernels on its arenas, nothing else (for "
                         "collecting the same counters on k_fused_compressed and on k_probe_streams in one profiler run)")
    ap.add_argument("--only-overlap", action="store_true",
                    help="run only the overlap demo (split step on two streams beside a forward stand-in) and print "
                         "its figures instead of the benchmark line")
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
    if args.only_overlap:
        print(json.dumps(overlap_demo(args.workload)))
        return 0
    if args.only_layer_by_layer:
        print(json.dumps(layer_by_layer(args.workload, max(5, args.steps // 4))))
        return 0
    if args.only_correction_sum:
        r = time_correction_sum(args.workload, args.steps, args.warmup, min_seconds=min(0.5, args.min_seconds))
        r["workload"] = args.workload
        print(json.dumps(r))
        return 0
    if args.only_stream_ceilings:
        head, wl = time_workload(args.workload, args.steps, args.warmup, want_correction=False,
                                 min_seconds=args.min_seconds)
        out = {"headline": {k: head[k] for k in ("workload", "ms_per_step", "gbs", "frac_hbm_peak")},
               "stream_ceilings": stream_ceilings(wl, min_seconds=min(0.3, args.min_seconds))}
        wl.destroy()
        print(json.dumps(out))
        return 0
    head, wl = time_workload(args.workload, args.steps, args.warmup, want_correction=True,
                             want_unfused=not args.no_extra, min_seconds=args.min_seconds)
    ceilings = None if args.no_extra else stream_ceilings(wl)
    cpu = None
    if not args.no_cpu_baseline:
        _progress("cpu baseline (oracle on the host cores)")
        cpu = cpu_baseline(wl)
    wl.destroy()
    del wl
    torch.cuda.empty_cache()
    extra = {"headline": head}
    if not args.no_extra:
        extra["stream_ceilings"] = ceilings
        _progress("extras: correction with kernel sum, overlap, small workloads, bf16 gradients, other workloads")
        extra["correction_with_kernel_sum_" + args.workload] = time_correction_sum(
            args.workload, max(3, args.steps // 4), max(1, args.warmup // 2))
        torch.cuda.empty_cache()
        extra["overlap_demo"] = overlap_demo(args.workload)
        torch.cuda.empty_cache()
        for name in ("c1_single", "c2_resnet20"):
            extra[name] = time_small(name)
        for name in ("c3_resnet50", "c4_vgg16"):
            extra["layer_by_layer_" + name] = layer_by_layer(name, max(5, args.steps // 4))
            torch.cuda.empty_cache()
        r, w = time_workload(args.workload, max(5, args.steps // 2), max(2, args.warmup // 2),
                             want_correction=False, grad_dtype=torch.bfloat16, min_seconds=0.5)
        w.destroy()
        del w
        torch.cuda.empty_cache()
        extra["bf16_gradients_" + args.workload] = r
        # the peers' streams in the sparse wire form (the library's own format, beyond the paper): on the
        # literal recipe nothing fires, so a peer costs 32 bytes of bitmap per chunk instead of 1 KiB; on the
        # dense parity recipe (a third of the codes fire) nearly every word travels.  GB/s here uses the
        # bytes this form really moves per element, stated next to the rate.
        for tag, dense in (("literal", False), ("dense", True)):
            r, w = time_workload(args.workload, max(5, args.steps // 2), max(2, args.warmup // 2),
                                 want_correction=False, min_seconds=0.5, sparse_peers=True, dense=dense)
            n_el, N = r["elements"], r["num_workers"]
            peer_bytes = 0.0
            for j in range(N):
                if w.peer_sparse[j] is not None:
                    for i, n in enumerate(w.cfg.sizes):
                        sv = w.sview(w.peer_sparse[j], i).view(-1, 264)[:, :8]
                        bits = sv.to(torch.int64) & 0xFFFFFFFF
                        nz = sum(int(((bits >> b) & 1).sum().item()) for b in range(32))
                        peer_bytes += 4.0 * (8 * sv.shape[0] + nz)
            bpe = 24.25 + peer_bytes / n_el
            r["bytes_per_element_sparse"] = bpe
            r["gbs_sparse_bytes"] = n_el * bpe / (r["ms_per_step"] * 1e-3) / 1e9
            r["note"] = "ms_per_step is the figure to compare with the packed form; gbs / frac_hbm_peak in this " \
                        "entry are still computed with the packed form's 24 + N/4 bytes"
            w.destroy()
            del w
            torch.cuda.empty_cache()
            extra["sparse_peers_%s_%s" % (tag, args.workload)] = r
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
                                 want_correction=(name != "c5_flat4g"), min_seconds=0.5)
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
        "timing": "median of %d back-to-back blocks of %d steps (%.2f s of GPU time); first block %.4f, last block "
                  "%.4f ms/step" % (head["blocks"]["blocks"], args.steps, head["blocks"]["timed_seconds"],
                                    head["blocks"]["first_block_ms_per_step"], head["blocks"]["last_block_ms_per_step"]),
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
                     "traffic": PROFILED_TRAFFIC_BYTES.get(head["workload"]),
                     "traffic_source": "constant from profiles/k_fused_compressed_%s.md (rocprofv3 --pmc FETCH_SIZE / "
                                       "WRITE_SIZE), not measured by this run" % head["workload"]},
        "cpu_baseline": cpu,
        "extra": extra,
        "paper_context": "end-to-end time 30% below 2-bit compression on a 16-GPU MXNet cluster at 56 Gbps "
                         "(abstract; another system, not comparable)",
    }
    # give everything back before the line goes out (the larger workloads hold over 100 GB of HBM), so that
    # the process is gone as soon as its result is
    import gc
    gc.collect()
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
