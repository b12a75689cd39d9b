#!/usr/bin/env python3
"""Benchmark of the batched tree-network forward pass on one MI355X.

One step = one tl_forward over one batch: structure pass, leaf cells, internal cells (scheduling
included) and root gather, with the batch and the parameters already resident in device memory.

Prints ONE JSON line.  `value` is trees/s of the whole step; `roofline` is about the dominant
kernel (the internal-node kernel) with its duration taken from HIP events recorded by the library on
the stream it launches on; `cpu_baseline` is the CPU checker timed on this host.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}      # MI355X dense matrix peaks
HBM_GBS = 8000.0
DEFAULT_SCHEDULER = "dataflow"


def measured_traffic(workload, scheduler, dtype):
    """HBM bytes per launch of the internal-node kernel from rocprofv3 counter passes (FETCH_SIZE, WRITE_SIZE, each
    scaled by a copy of known size), as written into profiles/traffic.json together with the counter summaries under
    profiles/.  A configuration whose counters have not been taken (or whose kernel has changed since) has no entry."""
    try:
        with open(os.path.join(ROOT, "profiles", "traffic.json")) as fh:
            table = json.load(fh)
    except (OSError, ValueError):
        return None
    return table.get("%s/%s/%s" % (workload, scheduler, dtype))


def algorithmic_work(w):
    """(flops of the internal cells, flops of the leaf cells, bytes) that the method must do:
    20 H^2 per internal TreeLSTM node (2 * 2H * 5H), 6 E H per leaf; bytes = every h/c row written once,
    every non-root row read once by its parent, one embedding row per leaf, the weights once, the indices."""
    from paper_1809_00832_amd import synth
    p, t = w.params, w.trees
    H, E = p.hidden, p.embed_dim
    n_int, n_leaf, N, B = t.n_internal, t.n_leaves, t.n_nodes, t.n_trees
    if p.cell == synth.CELL_TREELSTM:
        f_int, f_leaf, states = 20.0 * H * H * n_int, 6.0 * E * H * n_leaf, 2
        weights = (2 * H * 5 * H + E * 3 * H + 8 * H) * 4
    elif p.cell == synth.CELL_TREERNN:
        f_int, f_leaf, states = 4.0 * H * H * n_int, 0.0, 1
        weights = (2 * H * H + H) * 4
    else:
        f_int, f_leaf, states = (8.0 * H ** 3 + 4.0 * H * H) * n_int, 0.0, 1
        weights = (4 * H ** 3 + 2 * H * H + H) * 4
    bytes_ = states * N * H * 4 + states * (N - B) * H * 4 + n_leaf * E * 4 + weights + 3 * N * 4 + (B + 1) * 4
    return f_int, f_leaf, float(bytes_)


def heights_of(trees):
    """Height of every node (leaf 0, internal 1 + max of its children), by relaxation from the leaves."""
    import numpy as np
    left, right = np.asarray(trees.left), np.asarray(trees.right)
    inner = np.nonzero(left >= 0)[0]
    h = np.zeros(len(left), dtype=np.int64)
    while True:
        new = 1 + np.maximum(h[left[inner]], h[right[inner]])
        if np.array_equal(new, h[inner]):
            return h
        h[inner] = new


def span_bound_ms(w, peak_tflops, t_sync_us=2.0):
    """Critical-path lower bound of the internal stage: heights are evaluated one after the other, each at least
    its flops at the matrix peak or one grid-wide synchronisation (measured: about 2 us), whichever is longer."""
    import numpy as np
    h = heights_of(w.trees)
    counts = np.bincount(h)[1:]
    f_int, _, _ = algorithmic_work(w)
    per_node = f_int / max(1, w.trees.n_internal)
    return float(sum(max(c * per_node / (peak_tflops * 1e12) * 1e3, t_sync_us * 1e-3) for c in counts)), int(len(counts))


def time_steps(net, steps):
    import torch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        net.forward()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def time_graph_replays(net, steps):
    """The forward captured once in a HIP graph and replayed `steps` times (no host work per forward but the replay
    call): seconds per replay.  Device schedulers only: the host-driven one reads the number of heights back."""
    import torch
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        net.forward()
    for _ in range(3):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


PREHEAT_MS = 40.0


def preheat(net, ms):
    """Forwards of the same batch until the device has been busy for `ms` milliseconds, before the warm-up steps: a GPU
    that has been idle runs its first few milliseconds of work at a lower clock (measured: the first ten forwards of a
    process take up to 15 % longer), and a timed region of a few milliseconds would report that ramp instead of the
    sustained rate.  Not part of the warm-up or the timed steps; the figure is reported in the JSON line."""
    import torch
    if ms <= 0:
        return
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < ms:
        for _ in range(8):
            net.forward()
        torch.cuda.synchronize()


def run_scheduler(w, sched, precision, steps, warmup, graph=False):
    from paper_1809_00832_amd import binding
    net = binding.TreeNet(w.params, scheduler=sched, precision=precision)
    try:
        net.load(w.trees)
        preheat(net, PREHEAT_MS)
        for _ in range(warmup):
            net.forward()
        code = binding.tl_status(net.ctx)
        if code != 0:
            raise binding.TLError(code, "warm-up forward")
        sec = time_steps(net, steps)
        # same steps again with the library's stage events switched on
        binding.tl_set_profiling(net.ctx, True)
        k = min(steps, binding.TL_PROFILE_RING)
        sec_prof = time_steps(net, k)
        stages = [binding.tl_stage_ms(net.ctx, back) for back in range(k)]
        binding.tl_set_profiling(net.ctx, False)
        avg = {key: sum(s[key] for s in stages) / k for key in stages[0]}
        totals = sorted(s["total"] for s in stages)          # one forward each, first to last event on the stream
        latency = {"median": totals[len(totals) // 2], "min": totals[0], "max": totals[-1], "forwards": k}
        stats = binding.tl_last_stats(net.ctx)
        code = binding.tl_status(net.ctx)
        if code != 0:
            raise binding.TLError(code, "timed forward")
        out = dict(sec=sec, sec_profiled=sec_prof, stage_ms=avg, stats=stats, latency_ms=latency)
        if graph and sched != "level_host":
            out["sec_graph"] = time_graph_replays(net, steps)
            if binding.tl_status(net.ctx) != 0:
                raise binding.TLError(binding.tl_status(net.ctx), "graph replay")
        return out
    finally:
        net.close()


def head_stage(w, n_classes, reps=50):
    """The per-node classifier head on the h rows of one forward: mean kernel time from events on the launch stream
    (tl_classify is launched on torch's current stream), against the memory roofline (h read once, probabilities
    written once)."""
    import torch
    from paper_1809_00832_amd import binding
    net = binding.TreeNet(w.params, scheduler=DEFAULT_SCHEDULER)
    try:
        net.load(w.trees)
        net.forward()
        H, N = w.params.hidden, w.trees.n_nodes
        g = torch.Generator(device="cuda").manual_seed(1)
        ws = torch.randn((H, n_classes), device="cuda", generator=g) * (H ** -0.5)
        bs = torch.zeros(n_classes, device="cuda")
        probs = torch.empty((N, n_classes), device="cuda")
        for _ in range(5):
            binding.tl_classify(net.ctx, net.batch["h"], ws, bs, probs)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        ev[0].record()
        for i in range(reps):
            binding.tl_classify(net.ctx, net.batch["h"], ws, bs, probs)
            ev[i + 1].record()
        torch.cuda.synchronize()
        ms = sum(ev[i].elapsed_time(ev[i + 1]) for i in range(reps)) / reps
        bytes_ = (N * H + N * n_classes + H * n_classes + n_classes) * 4.0
        return {"classes": n_classes, "ms": ms, "bound": "hbm", "achieved": bytes_ / (ms * 1e-3) / 1e9, "peak": HBM_GBS,
                "unit": "GB/s", "frac": bytes_ / (ms * 1e-3) / 1e9 / HBM_GBS, "bytes_per_launch": bytes_}
    finally:
        net.close()


def length_sweep(steps, warmup):
    """Latency of ONE tree (no batching) against its number of leaves, parameters of the `sentence` workload: the
    experiment of Figure 11 (time per instance by sentence length; with enough parallel units a tree of N words takes
    O(log N) steps when it is balanced, O(N) when it is a chain)."""
    from paper_1809_00832_amd import binding, synth
    base = synth.workload("sentence")
    rows = []
    for shape in ("balanced", "random", "chain"):
        for leaves in (2, 4, 8, 16, 32, 64, 128, 256, 512, 1024):
            trees = synth.make_trees(100 + leaves, [leaves], [shape], base.params.vocab)
            row = {"shape": shape, "leaves": leaves, "height": int(heights_of(trees).max())}
            for sched in ("dataflow", "level_device", "ready"):
                net = binding.TreeNet(base.params, scheduler=sched)
                try:
                    net.load(trees)
                    for _ in range(warmup):
                        net.forward()
                    row[sched + "_ms"] = time_steps(net, steps) * 1e3
                    if binding.tl_status(net.ctx) != 0:
                        raise RuntimeError("forward failed")
                finally:
                    net.close()
            rows.append(row)
    print(json.dumps({"length_sweep": rows, "hidden": base.params.hidden, "embed_dim": base.params.embed_dim, "dtype": "f32",
                      "note": "one tree per forward, whole tl_forward (structure pass, leaves, internal nodes, roots)"}))


def backward_stage(w, n_classes, reps=10):
    """tl_backward on the states of one forward (TreeLSTM, fp32): mean wall time per call (the call waits for the
    structure pass itself), with its algorithmic flops: 60 H^2 per internal node (gates recomputed, operand
    gradient, weight gradient: 20 H^2 each) and 18 E H per leaf.  With a head (n_classes > 0) also the head's
    backward on its own and one training step without the parameter update: forward, head backward (which
    recomputes the head's forward), tree backward, back to back on one stream."""
    import torch
    from paper_1809_00832_amd import binding
    net = binding.TreeNet(w.params, scheduler=DEFAULT_SCHEDULER)
    try:
        b = net.load(w.trees)
        net.forward()
        H, E, N = w.params.hidden, w.params.embed_dim, w.trees.n_nodes
        g_h = torch.randn((N, H), device="cuda")

        def wall(fn, reps):
            for _ in range(2):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / reps * 1e3

        rntn = w.params.cell == 2
        ms = wall(lambda: binding.tl_backward(net.ctx, b, g_h, E, rntn=rntn), reps)
        if w.params.cell == 0:
            flops = 60.0 * H * H * w.trees.n_internal + 18.0 * E * H * w.trees.n_leaves
        elif w.params.cell == 1:    # TreeRNN: operand gradient and weight gradient, 4 H^2 each per internal node
            flops = 8.0 * H * H * w.trees.n_internal
        else:                       # RNTN: both contractions run over rows of d * 2d + d values, 2d outputs
            flops = 2.0 * 2.0 * (H * 2 * H + H) * 2 * H * w.trees.n_internal
        out = {"ms": ms, "flops": flops, "tflops": flops / (ms * 1e-3) / 1e12,
               "frac_mfma_peak": flops / (ms * 1e-3) / 1e12 / PEAK_TFLOPS["f32"]}
        # training mode: the forward keeps the gate activations, the backward does not recompute the contraction
        # (40 H^2 flops per internal node and 12 E H per leaf are left)
        if w.params.cell == 0:
            binding.tl_set_keep_gates(net.ctx, True)
            net.forward()
            out["ms_kept_gates"] = wall(lambda: binding.tl_backward(net.ctx, b, g_h, E), reps)
            out["forward_ms_keeping_gates"] = wall(net.forward, 50)
        if n_classes > 0:
            g = torch.Generator(device="cuda").manual_seed(2)
            ws = torch.randn((H, n_classes), device="cuda", generator=g) * (H ** -0.5)
            bs = torch.zeros(n_classes, device="cuda")
            label = torch.randint(0, n_classes, (N,), device="cuda", generator=g, dtype=torch.int32)
            out["head_backward_ms"] = wall(lambda: binding.tl_classify_backward(net.ctx, b["h"], ws, bs, label), 50)

            def train_step(lr=0.0):
                net.forward()
                hb = binding.tl_classify_backward(net.ctx, b["h"], ws, bs, label)
                grads = binding.tl_backward(net.ctx, b, hb["g_h"], E, rntn=rntn)
                binding.tl_sgd_update(net.ctx, lr, b, grads)           # lr = 0: all the work, parameters unchanged

            grads0 = binding.tl_backward(net.ctx, b, g_h, E, rntn=rntn)
            out["sgd_update_ms"] = wall(lambda: binding.tl_sgd_update(net.ctx, 0.0, b, grads0), reps)
            step_ms = wall(train_step, reps)
            out["train_step_ms"] = step_ms
            if w.params.cell != 2:
                # the same with a backward that does not wait for the device (all heights in one persistent kernel)
                binding.tl_set_async_backward(net.ctx, True)
                net.forward()                                          # (the update above has made the kept activations stale)
                out["ms_without_waiting"] = wall(lambda: binding.tl_backward(net.ctx, b, g_h, E), reps)
                out["train_step_ms_without_waiting"] = wall(train_step, reps)
                # and with launches per height whatever the number of heights (the default takes them up to 64 heights)
                binding.tl_set_async_backward(net.ctx, -1)
                net.forward()
                out["ms_launches_per_height"] = wall(lambda: binding.tl_backward(net.ctx, b, g_h, E), reps)
                binding.tl_set_async_backward(net.ctx, 0)
            out["train_trees_per_s"] = w.trees.n_trees / (step_ms * 1e-3)
            out["train_step_note"] = ("forward (a TreeLSTM keeps its gate activations) + head backward + tree backward + SGD update "
                                      "of all parameters (embedding rows included) and re-packing of the weights")
        return out
    finally:
        net.close()


def topdown_rows(steps, warmup, with_cpu):
    """Top-down generation of dynamically structured trees (the experiment of Table 3: batch sizes 1 and 64): instances
    per second of tl_td_generate with the root states resident, kernel time from events on the launch stream, the
    algorithmic flops (8 H^2 per generated child plus 2 H per scored node) and the dependent frontiers that bound it."""
    import torch
    from paper_1809_00832_amd import binding, synth
    rows = []
    for name in ("td64", "td1"):
        w = synth.topdown_workload(name)
        dev = lambda x: torch.from_numpy(x).cuda().contiguous()
        ctx = binding.tl_td_create(w.hidden, dev(w.u_td), dev(w.b_td), dev(w.w_stop), w.b_stop)
        try:
            out = binding.tl_td_generate(ctx, dev(w.h_root), dev(w.c_root), w.max_nodes, w.max_depth)
            B = w.h_root.shape[0]
            for _ in range(warmup):
                binding.tl_td_generate_into(ctx, B, w.max_depth, out)
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ev[0].record()
            for i in range(steps):
                binding.tl_td_generate_into(ctx, B, w.max_depth, out)
                ev[i + 1].record()
            torch.cuda.synchronize()
            sec = (time.perf_counter() - t0) / steps
            if binding.tl_td_status(ctx) != 0:
                raise RuntimeError("generation failed")
            counts = out["counts"].cpu().numpy()
            n, fronts = int(counts[0]), int(counts[2])
            kernel_ms = sum(ev[i].elapsed_time(ev[i + 1]) for i in range(steps)) / steps
            flops = 8.0 * w.hidden ** 2 * (n - B) + 2.0 * w.hidden * n
            row = {"workload": name, "instances": B, "hidden": w.hidden, "nodes": n, "frontiers": fronts,
                   "ms_per_batch": sec * 1e3, "instances_per_s": B / sec, "nodes_per_s": n / sec, "launch_ms": kernel_ms,
                   "tflops": flops / (kernel_ms * 1e-3) / 1e12, "frac_mfma_peak": flops / (kernel_ms * 1e-3) / 1e12 / PEAK_TFLOPS["f32"],
                   "us_per_frontier": kernel_ms * 1e3 / max(fronts, 1)}
            if with_cpu and name == "td1":
                import oracle
                t0 = time.perf_counter()
                r = oracle.td_generate(w.u_td, w.b_td, w.w_stop, w.b_stop, w.h_root, w.c_root, w.max_depth, w.max_nodes)
                dt = time.perf_counter() - t0
                row["cpu_baseline"] = {"value": 1.0 / dt, "unit": "instances/s", "cores": 1, "kind": "oracle",
                                       "sample": "the one tree of td1 (%d nodes)" % r["n_nodes"], "nodes_per_s": r["n_nodes"] / dt}
            rows.append(row)
        finally:
            binding.tl_td_destroy(ctx)
    return rows


TOPDOWN_NOTE = ("tl_td_generate, root states resident; td64: breadth first, two grid barriers per depth; td1 (batches of up to 32 "
                "roots): no frontiers, children computed while the parent is scored")


def topdown_bench(steps, warmup, with_cpu):
    print(json.dumps({"topdown": topdown_rows(steps, warmup, with_cpu), "dtype": "f32", "data": "synthetic", "note": TOPDOWN_NOTE}))


def other_configs(steps, warmup):
    """The evaluation workloads other than the headline one, a few steps each: ms per step, trees/s, nodes/s, the
    internal-node kernel's fraction of the matrix peak of its precision (algorithmic flops over its mean duration from
    the library's stage events) and the step's algorithmic bytes per second (the small and the TreeRNN workloads are
    bound by latency and memory, not by the matrix units), for the default scheduler, the
    ready-queue scheduler and the two level-wise ones (Section 4.1 against the depth-wise batching of Section 6.3)."""
    from paper_1809_00832_amd import binding, synth
    rows = []
    cases = [("tiny", "f32"), ("sentence", "f32"), ("throughput", "bf16"), ("treernn", "f32"), ("rntn", "f32"), ("stress", "f32"),
             ("sentence", "bf16"), ("stress", "bf16")]
    for name, dtype in cases:
        w = synth.workload(name)
        t = w.trees
        f_int, f_leaf, alg_bytes = algorithmic_work(w)
        prec = binding.TL_F32 if dtype == "f32" else binding.TL_BF16_IN
        heavy = name == "stress"
        k, wu = (min(steps, 5), min(warmup, 2)) if heavy else (min(steps, 20), min(warmup, 5))
        scheds = [DEFAULT_SCHEDULER, "ready", "level_device", "level_host"]
        row = {"workload": name, "dtype": dtype, "trees": t.n_trees, "nodes": t.n_nodes, "hidden": w.params.hidden, "schedulers": {}}
        for sched in scheds:
            r = run_scheduler(w, sched, prec, k, wu)
            kernel_ms = r["stage_ms"]["internal"]
            row["schedulers"][sched] = {
                "ms_per_step": r["sec"] * 1e3, "trees_per_sec": t.n_trees / r["sec"], "nodes_per_sec": t.n_nodes / r["sec"],
                "internal_ms": kernel_ms, "internal_frac_mfma_peak": f_int / (kernel_ms * 1e-3) / 1e12 / PEAK_TFLOPS[dtype],
                "step_frac_mfma_peak": (f_int + f_leaf) / r["sec"] / 1e12 / PEAK_TFLOPS[dtype],
                "step_algorithmic_gbs": alg_bytes / r["sec"] / 1e9, "step_frac_hbm_peak": alg_bytes / r["sec"] / 1e9 / HBM_GBS,
                "stage_ms": r["stage_ms"]}
        rows.append(row)
    return rows


def cpu_baseline(w, max_nodes=40000):
    """The CPU checker as it stands, one thread per host core (at most 16), on all trees of the workload, or, when
    the workload is large, on a sample of whole trees of about max_nodes nodes taken at even spacing over the batch."""
    import oracle
    from paper_1809_00832_amd import synth
    cores = min(16, os.cpu_count() or 1)
    trees, what = w.trees, "all %d trees of the workload" % w.trees.n_trees
    if trees.n_nodes > max_nodes:
        k = max(1, int(trees.n_trees * max_nodes / trees.n_nodes))
        pick = sorted(set(int(i * trees.n_trees / k) for i in range(k)))
        trees, _ = synth.subset(w.trees, pick)
        what = "%d of the %d trees (every %d-th), %d nodes" % (len(pick), w.trees.n_trees, w.trees.n_trees // k, trees.n_nodes)
    passes, dt_all = 0, 0.0
    while passes < 1 or (dt_all < 1.5 and passes < 20):      # about 25 core-seconds on the default workload
        t0 = time.perf_counter()
        oracle.forward_params(w.params, trees, n_threads=cores)
        dt_all += time.perf_counter() - t0
        passes += 1
    dt = dt_all / passes
    # and on one thread, on every eighth tree of that sample
    one, _ = synth.subset(trees, list(range(0, trees.n_trees, 8)))
    t0 = time.perf_counter()
    oracle.forward_params(w.params, one, n_threads=1)
    dt_one = time.perf_counter() - t0
    return {"value": trees.n_trees / dt, "unit": "trees/s", "cores": cores, "kind": "oracle",
            "nodes_per_sec": trees.n_nodes / dt, "seconds": dt_all + dt_one,
            "sample": "%s, %d passes (mean), trees spread over %d threads" % (what, passes, cores),
            "one_thread": {"value": one.n_trees / dt_one, "unit": "trees/s", "nodes_per_sec": one.n_nodes / dt_one,
                           "sample": "%d trees (%d nodes) of that sample, one pass" % (one.n_trees, one.n_nodes)}}


def copy_calibration(mib=1024, reps=3):
    """A plain copy of `mib` MiB, `reps` times: it reads and writes exactly that many bytes of HBM per launch, which
    gives the scale of the FETCH_SIZE / WRITE_SIZE counters when this command runs under rocprofv3 --pmc."""
    import torch
    src = torch.ones(mib << 18, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"copy_calibration": True, "bytes_read_per_launch": mib << 20, "bytes_written_per_launch": mib << 20,
                      "launches": reps}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="throughput")
    ap.add_argument("--scheduler", default=DEFAULT_SCHEDULER, choices=["ready", "level_device", "level_host", "ready_priority", "dataflow"])
    ap.add_argument("--precision", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--no-compare", action="store_true", help="skip the other two schedulers")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU baseline")
    ap.add_argument("--no-others", action="store_true", help="skip the short runs of the other workloads / precisions")
    ap.add_argument("--preheat-ms", type=float, default=PREHEAT_MS,
                    help="milliseconds of untimed forwards before the warm-up steps, so that the device has left its idle clock state (0: none)")
    ap.add_argument("--head", type=int, default=5, help="classes of the per-node classifier head timed as an extra stage (0: skip)")
    ap.add_argument("--backward", action="store_true", help="also time tl_backward on the same batch (TreeLSTM, fp32)")
    ap.add_argument("--length-sweep", action="store_true",
                    help="print only the latency of single trees of 2..1024 leaves (balanced, random, chain)")
    ap.add_argument("--graph", action="store_true",
                    help="also time the forward replayed from a HIP graph (device schedulers)")
    ap.add_argument("--topdown", action="store_true",
                    help="print only the throughput of top-down generation of dynamically structured trees (batches of 64 and 1)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a device-to-device copy of known size (reference reading for the HBM byte counters)")
    args = ap.parse_args()
    globals()["PREHEAT_MS"] = args.preheat_ms
    if args.gpus != 1:
        sys.exit("bench.py: the forward pass is evaluated on ONE GPU only (trees are independent: a batch shards by tree, "
                 "with no exchange between GPUs); run with --gpus 1")

    import torch
    from paper_1809_00832_amd import binding, synth
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    torch.cuda.set_device(0)
    if args.copy_calibration:
        copy_calibration()
        return
    if args.length_sweep:
        length_sweep(min(args.steps, 30), min(args.warmup, 5))
        return
    if args.topdown:
        topdown_bench(args.steps, args.warmup, not args.no_cpu)
        return
    precision = binding.TL_F32 if args.precision == "f32" else binding.TL_BF16_IN

    w = synth.workload(args.workload)
    t = w.trees
    f_int, f_leaf, bytes_ = algorithmic_work(w)

    main_run = run_scheduler(w, args.scheduler, precision, args.steps, args.warmup, graph=args.graph)
    sec = main_run["sec"]
    peak = PEAK_TFLOPS[args.precision]
    kernel_ms = main_run["stage_ms"]["internal"]
    achieved = f_int / (kernel_ms * 1e-3) / 1e12
    out = {
        "metric": "TreeLSTM forward trees/sec" if w.params.cell == 0 else "tree network forward trees/sec",
        "value": t.n_trees / sec,
        "unit": "trees/s",
        "nodes_per_sec": t.n_nodes / sec,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sec * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.precision, "data": "synthetic", "preheat_ms": args.preheat_ms,
        "config": {"workload": args.workload, "scheduler": args.scheduler, "trees": t.n_trees, "nodes": t.n_nodes,
                   "leaves": t.n_leaves, "hidden": w.params.hidden, "embed_dim": w.params.embed_dim,
                   "vocab": w.params.vocab},
        "step_tflops": (f_int + f_leaf) / sec / 1e12,
        "step_frac_mfma_peak": (f_int + f_leaf) / sec / 1e12 / peak,
        "step_algorithmic_gbs": bytes_ / sec / 1e9,
        "stage_ms": main_run["stage_ms"],
        "ms_per_step_with_stage_events": main_run["sec_profiled"] * 1e3,
        "forward_latency_ms": main_run["latency_ms"],
        **({"ms_per_step_graph_replay": main_run["sec_graph"] * 1e3} if "sec_graph" in main_run else {}),
        "tiles_formed": main_run["stats"]["n_tiles"],
        "roofline": {"bound": "mfma", "kernel": "internal-node kernel (%s scheduler)" % args.scheduler,
                     "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                     "flops_per_launch": f_int, "kernel_ms": kernel_ms, "traffic": None},
    }
    traffic = measured_traffic(args.workload, args.scheduler, args.precision)
    if traffic:
        out["roofline"]["traffic"] = traffic["read_bytes"] + traffic["write_bytes"]
        out["roofline"]["traffic_read"] = traffic["read_bytes"]
        out["roofline"]["traffic_write"] = traffic["write_bytes"]
        out["roofline"]["traffic_source"] = traffic.get("source")
    bound_ms, n_heights = span_bound_ms(w, peak)
    out["span_bound"] = {"internal_ms": bound_ms, "heights": n_heights,
                         "note": "sum over heights of max(flops at matrix peak, 2 us grid synchronisation)"}
    if args.head > 0:
        out["head"] = head_stage(w, args.head)
    if args.backward and args.precision == "f32":
        out["backward"] = backward_stage(w, args.head)
    if not args.no_compare:
        comp = {}
        for sched in ("dataflow", "ready", "ready_priority", "level_device", "level_host"):
            if sched == args.scheduler:
                continue
            r = run_scheduler(w, sched, precision, args.steps, args.warmup, graph=args.graph)
            comp[sched] = {"trees_per_sec": t.n_trees / r["sec"], "ms_per_step": r["sec"] * 1e3,
                           "stage_ms": r["stage_ms"], "forward_latency_ms": r["latency_ms"], "n_levels": r["stats"]["n_levels"]}
            if "sec_graph" in r:
                comp[sched]["ms_per_step_graph_replay"] = r["sec_graph"] * 1e3
        out["comparison"] = comp
    if not args.no_others and args.workload == "throughput" and args.precision == "f32":
        out["other_configs"] = other_configs(args.steps, args.warmup)
        if "backward" not in out:
            # the backward pass and a training step on the same batch (a few calls each: a fraction of a second)
            out["training"] = backward_stage(w, args.head if args.head > 0 else 5)
        # top-down generation of dynamically structured trees (batches of 64 roots and of one), a few calls each
        out["topdown"] = {"rows": topdown_rows(min(args.steps, 20), min(args.warmup, 5), False), "note": TOPDOWN_NOTE}
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
