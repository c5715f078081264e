#!/usr/bin/env python3
"""Benchmark of the per-rank multi-colour reduce + SGD update step on one MI355X.

A step is one pass of the whole path over one batch of synthetic gradients that are
already resident in HBM as per-layer tensors.  Two equivalent forms are timed:
  fused (default, the headline):  1 x mc_fused_step -- contributions read straight from the
      per-layer tensors, per-layer weights and momentum updated in place, flat g written;
  staged:  P x mc_pack (per-layer tensors -> flat colour-chunked payload)
           1 x mc_reduce_update (per-colour fixed-order sum fused with the SGD update, writes g)
           1 x mc_unpack (updated weights -> per-layer tensors)
The layout (a1) is built once per model, like the framework's flattening of its parameters;
its cost is reported separately as `layout_create_ms`.

Prints ONE JSON line.  `value` is algorithmic bytes of the whole step / wall time of the
step; `roofline` is for the dominant kernel (fused_step_kernel, or reduce_update_kernel with
--path staged), timed with events on the stream it is launched on, inside the timed region; `cpu_baseline` is the CPU oracle timed
on this machine's host cores on the same workload.
"""
import argparse
import json
import os
import sys
import threading
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0     # MI355X published HBM3E bandwidth
METRIC = "effective HBM GB/s (% of MI355X peak) and ms per ResNet-50-shaped reduce+update"


def measured_traffic(kernel, workload, P, k):
    """HBM-side bytes per launch of the dominant kernel, from the rocprofv3 counter runs whose
    summary is kept under profiles/ (None when there is none for this kernel and workload)."""
    path = os.path.join(ROOT, "profiles", f"{kernel.replace('_kernel', '')}_{workload}_P{P}_k{k}.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return int(line.split(":")[1])
    except OSError:
        pass
    return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="resnet50",
                    choices=["tiny", "resnet50", "resnet50_heavy", "vgg16", "googlenet"])
    ap.add_argument("--sets", type=int, default=0,
                    help="rotating sets of contribution tensors (0 = pick so that no step re-reads a cached set)")
    ap.add_argument("--order", default="rotation", choices=["identity", "rotation"])
    ap.add_argument("--path", default="fused", choices=["fused", "staged"],
                    help="fused: one mc_fused_step per step; staged: P packs + reduce_update + unpack")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--pipeline-packets", type=int, default=0,
                    help="also run the packet-pipelined experiment with this many packets per colour")
    ap.add_argument("--roles-nodes", type=int, default=0,
                    help="also time one rank's role-dependent step in a tree Allreduce over this many nodes")
    ap.add_argument("--unroll", type=int, default=0, choices=[0, 1, 2],
                    help="16-byte vectors per thread per tile (0 = the library picks from the size)")
    ap.add_argument("--state-store-sc1", type=int, default=-1, choices=[-1, 0, 1],
                    help="store policy of weights / momentum (-1 = the library's default)")
    ap.add_argument("--alternate-sweep", type=int, default=-1, choices=[-1, 0, 1],
                    help="alternate the sweep direction between steps (-1 = the library's default)")
    ap.add_argument("--xcd-run", type=int, default=-1,
                    help="consecutive tiles per die, 0..64 (-1 = the library's default)")
    ap.add_argument("--kernel-only", action="store_true",
                    help="time only mc_reduce_update launches (for profiler runs)")
    return ap.parse_args()


def cpu_baseline(cfg, order, host_sets, w_layers_host, seconds, parity_ref, step_bytes):
    """The oracle as it stands: whole step (P packs, reduce+update, unpack) on host cores.
    Its GB/s uses the same step_bytes as the GPU figure beside it, so that the ratio of the
    two values is the ratio of the step times."""
    import oracle
    O = oracle.Layout(cfg.sizes, cfg.k)
    N = O.N
    w = oracle.pack(O, w_layers_host)
    v = np.zeros(N, np.float32)

    def one_step(step):
        xs = [oracle.pack(O, ts) for ts in host_sets[step % len(host_sets)]]
        g = oracle.reduce_update(O, xs, w, v, cfg.lr, cfg.mu, cfg.wd, order=order)
        layers = oracle.unpack(O, w)
        return g, layers

    t0 = time.perf_counter()
    g, _ = one_step(0)
    first = time.perf_counter() - t0
    parity_ref.update(g=g, w=w.copy(), v=v.copy())
    n = max(1, min(200, int(seconds / max(first, 1e-4))))
    t0 = time.perf_counter()
    for s in range(1, n + 1):
        one_step(s)
    dt = (time.perf_counter() - t0) / n

    # colours are independent (and so are the P packs): one host thread per colour / pack
    ncpu = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    nthr = max(1, min(cfg.k, ncpu))
    w2 = oracle.pack(O, w_layers_host)
    v2 = np.zeros(N, np.float32)
    g2 = np.empty(N, np.float32)

    def threaded_step(step):
        tensors = host_sets[step % len(host_sets)]
        xs = [None] * cfg.P

        def do_pack(p):
            xs[p] = oracle.pack(O, tensors[p])
        th = [threading.Thread(target=do_pack, args=(p,)) for p in range(cfg.P)]
        [t.start() for t in th]
        [t.join() for t in th]
        seq = order if order is not None else np.tile(np.arange(cfg.P, dtype=np.int32), (cfg.k, 1))
        colours = list(range(cfg.k))

        def do_colours(tid):
            for c in colours[tid::nthr]:
                oracle.reduce_update_colour(O, c, xs, g2, w2, v2, cfg.lr, cfg.mu, cfg.wd, seq=seq[c])
        th = [threading.Thread(target=do_colours, args=(i,)) for i in range(nthr)]
        [t.start() for t in th]
        [t.join() for t in th]
        oracle.unpack(O, w2)

    threaded_step(0)
    n2 = max(1, min(200, int(0.5 * seconds / max(dt, 1e-4))))
    t0 = time.perf_counter()
    for s in range(1, n2 + 1):
        threaded_step(s)
    dt2 = (time.perf_counter() - t0) / n2
    return {
        "value": round(step_bytes / dt / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
        "ms_per_step": round(dt * 1e3, 3),
        "sample": f"{n} whole steps ({cfg.P} packs + reduce+update + unpack) of the full {cfg.name} "
                  f"workload, N={N}, single thread",
        "threaded": {"value": round(step_bytes / dt2 / 1e9, 3), "unit": "GB/s",
                     "cores": max(nthr, min(cfg.P, ncpu)), "ms_per_step": round(dt2 * 1e3, 3),
                     "sample": f"{n2} whole steps, one host thread per colour ({nthr}) / per pack ({cfg.P})"},
        "host_cpus": ncpu,
    }


def roles_experiment(torch, mc, L, cfg, flats, g, w, v, stream, n_nodes, reps):
    """One rank's real share in a k-colour tree Allreduce over n_nodes nodes (Section 4.2): it
    is inner node or root of at most one colour and a leaf of the others.  Phase 1: per colour,
    add the m local replicas (leaf) or those plus one buffer per child (inner node, root); only
    the root's colour is updated at once.  Phase 2: the other colours are updated from the
    broadcast sum (a single contribution).  m = the workload's P; child buffers are further
    flat buffers of the same size.  Times both phases for the rank with the most work (an inner
    node) and for a pure-leaf rank, with the algorithmic bytes of each."""
    N, m, k = cfg.total, cfg.P, cfg.k
    sh = int(stream.cuda_stream)
    bounds = [int(b) for b in L.colour_bounds()]
    lens = [bounds[c + 1] - bounds[c] for c in range(k)]
    child_bufs = [torch.randn(N, dtype=torch.float32, device="cuda") * 1e-3 for _ in range(k)]
    contrib = mc.ptr_table([f.data_ptr() for f in flats] + [c.data_ptr() for c in child_bufs])
    bcast = torch.randn(N, dtype=torch.float32, device="cuda") * 1e-3
    bcast_tab = mc.ptr_table([bcast.data_ptr()])
    scratch = torch.empty(N, dtype=torch.float32, device="cuda")

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        a = torch.cuda.Event(enable_timing=True)
        b = torch.cuda.Event(enable_timing=True)
        a.record(stream)
        for _ in range(reps):
            fn()
        b.record(stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    out = {"n_nodes": n_nodes, "colours": k, "local_replicas": m, "ranks": {}}
    picked = {}
    for rank in range(n_nodes):
        role, cnt, _children = mc.rank_roles(n_nodes, k, rank)
        kind = "root" if (role == mc.ROLE_ROOT).any() else "inner" if (role == mc.ROLE_INNER).any() else "leaf"
        picked.setdefault(kind, (rank, role, cnt))
    for kind, (rank, role, cnt) in picked.items():
        n_terms = [m + int(cnt[c]) for c in range(k)]
        upd = [1 if role[c] == mc.ROLE_ROOT else 0 for c in range(k)]
        later = [0 if role[c] == mc.ROLE_ROOT else 1 for c in range(k)]
        bytes1 = sum(4 * lens[c] * (n_terms[c] + 1 + (4 if upd[c] else 0)) for c in range(k))
        bytes2 = sum(4 * lens[c] * (1 + 4) for c in range(k) if later[c])
        t1 = timed(lambda: mc.reduce_update_roles(L, contrib, None, n_terms, upd, g.data_ptr(), w.data_ptr(),
                                                  v.data_ptr(), cfg.lr, cfg.mu, cfg.wd, sh))
        t2 = timed(lambda: mc.reduce_update_roles(L, bcast_tab, None, later, [1] * k, scratch.data_ptr(),
                                                  w.data_ptr(), v.data_ptr(), cfg.lr, cfg.mu, cfg.wd, sh)) \
            if any(later) else 0.0
        out["ranks"][kind] = {"rank": rank, "terms_per_colour": n_terms, "updates_at_once": upd,
                              "sum_ms": round(t1, 4), "sum_GBps": round(bytes1 / t1 / 1e6, 1),
                              "update_from_broadcast_ms": round(t2, 4),
                              "update_GBps": round(bytes2 / t2 / 1e6, 1) if t2 else None}
    return out


def pipeline_experiment(torch, mc, L, cfg, order, flats, flat_table, g, w, v, stream, packets, reps):
    """Section 4.2 pipelines the reductions packet by packet.  Here half of the P contributions
    are resident and the other half "arrive": staging copies on a second stream stand in for
    network buffers landing in the receive buffers.  Unpipelined: all copies, then one
    mc_reduce_update.  Pipelined: per packet (colours interleaved, as the colours progress
    concurrently), copy the packet of every arriving contribution, then mc_reduce_update_range
    on it as soon as its copies are done.  On one GPU copies and sum share the same HBM, so
    this measures latency hiding, not extra bandwidth."""
    N, P, k = cfg.total, cfg.P, cfg.k
    arriving = list(range(P // 2, P))
    src = [torch.randn(N, dtype=torch.float32, device="cuda") * 1e-3 for _ in arriving]
    copy_stream = torch.cuda.Stream()
    sh = int(stream.cuda_stream)
    bounds = [int(b) for b in L.colour_bounds()]
    pk = []
    for c in range(k):
        lo, hi = bounds[c], bounds[c + 1]
        if hi == lo:
            continue
        step = -(-(hi - lo) // packets)
        step = -(-step // 256) * 256
        pk.append([(b, min(hi, b + step)) for b in range(lo, hi, step)])
    order_of_packets = [p[j] for j in range(max(len(p) for p in pk)) for p in pk if j < len(p)]

    def pipelined(main=None):
        main = main or stream
        mh = int(main.cuda_stream)
        copy_stream.wait_stream(main)
        for (b, e) in order_of_packets:
            with torch.cuda.stream(copy_stream):
                for q, s_ in zip(arriving, src):
                    mc.copy(flats[q].data_ptr() + 4 * b, s_.data_ptr() + 4 * b, 4 * (e - b), int(copy_stream.cuda_stream))
                ev = torch.cuda.Event()
                ev.record(copy_stream)
            main.wait_event(ev)
            mc.reduce_update_range(L, flat_table, order, g.data_ptr(), w.data_ptr(), v.data_ptr(),
                                   cfg.lr, cfg.mu, cfg.wd, b, e, mh)
        main.wait_stream(copy_stream)

    def unpipelined_own_copy(main=None):
        main = main or stream
        copy_stream.wait_stream(main)
        with torch.cuda.stream(copy_stream):
            for q, s_ in zip(arriving, src):
                mc.copy(flats[q].data_ptr(), s_.data_ptr(), 4 * (N // 4) * 4, int(copy_stream.cuda_stream))
        main.wait_stream(copy_stream)
        mc.reduce_update(L, flat_table, order, g.data_ptr(), w.data_ptr(), v.data_ptr(),
                         cfg.lr, cfg.mu, cfg.wd, int(main.cuda_stream))

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        a = torch.cuda.Event(enable_timing=True)
        b = torch.cuda.Event(enable_timing=True)
        a.record(stream)
        for _ in range(reps):
            fn()
        b.record(stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    def captured(fn):
        """The same sequence captured once into a HIP graph (kernel nodes and event edges only)
        and replayed: removes the per-packet host cost of issuing launches and event waits."""
        cap = torch.cuda.Stream()
        cap.wait_stream(stream)
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=cap):
            fn(torch.cuda.current_stream())
        torch.cuda.synchronize()
        return timed(graph.replay)

    out = {"packets_per_colour": packets, "n_packets": len(order_of_packets),
           "arriving_contributions": len(arriving),
           "unpipelined_ms": round(timed(unpipelined_own_copy), 4),
           "pipelined_ms": round(timed(pipelined), 4)}
    out["unpipelined_graph_ms"] = round(captured(unpipelined_own_copy), 4)
    out["pipelined_graph_ms"] = round(captured(pipelined), 4)
    return out


def main():
    args = parse()
    world = int(os.environ.get("WORLD_SIZE", "1"))
    if args.gpus != 1 or world != 1:
        print("bench.py: this build measures one GPU's share of the step on ONE GPU; "
              "--gpus must be 1 (no collectives or multi-GPU paths are part of it).", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1711_00705_amd import mc, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback.", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    if args.unroll:
        mc.set_option(mc.OPT_RU_SHAPE, args.unroll)
    if args.alternate_sweep >= 0:
        mc.set_option(mc.OPT_ALTERNATE_SWEEP, args.alternate_sweep)
    if args.state_store_sc1 >= 0:
        mc.set_option(mc.OPT_STATE_STORE_SC1, args.state_store_sc1)
    if args.xcd_run >= 0:
        mc.set_option(mc.OPT_XCD_RUN, args.xcd_run)
    cfg = wl.workload(args.workload)
    N, P, k = cfg.total, cfg.P, cfg.k
    order = None if args.order == "identity" else wl.rotation_order(k, P)
    set_bytes = 4 * N * P
    # enough rotating sets that a step never finds its contributions in the 256 MB last-level cache
    n_sets = args.sets or (cfg.steps if cfg.steps > 1 else max(3, int(np.ceil(1.2e9 / set_bytes))))
    n_sets = min(n_sets, 100)

    t0 = time.perf_counter()
    L = mc.Layout(cfg.sizes, k)
    layout_ms = (time.perf_counter() - t0) * 1e3
    L.prepare()
    stream = torch.cuda.current_stream()
    sh = int(stream.cuda_stream)

    def upload(layers):
        return [torch.from_numpy(t).cuda() for t in layers]

    # ---- inputs: seeded, host-generated, uploaded as separate per-layer tensors ------------
    host_sets = []            # kept for the CPU baseline (first 3 sets only)
    dev_sets, tables, tsets = [], [], []
    for s in range(n_sets):
        per_p = [wl.contribution_tensors(cfg.sizes, p, step=s, heavy_tail=cfg.heavy_tail) for p in range(P)]
        if s < 3:
            host_sets.append(per_p)
        dev = [upload(ts) for ts in per_p]
        dev_sets.append(dev)
        tables.append([mc.ptr_table([t.data_ptr() for t in d]) for d in dev])
        tsets.append(mc.set_table([mc.TensorSet(L, [t.data_ptr() for t in d]) for d in dev]))
    w_layers_host = wl.weight_tensors(cfg.sizes)
    g = torch.empty(N, dtype=torch.float32, device="cuda")

    # staged path state: flat w, v (master), per-layer weights as the unpack destination
    w_layers = upload(w_layers_host)
    w_table = mc.ptr_table([t.data_ptr() for t in w_layers])
    flats = [torch.empty(N, dtype=torch.float32, device="cuda") for _ in range(P)]
    flat_table = mc.ptr_table([f.data_ptr() for f in flats])
    w = torch.empty(N, dtype=torch.float32, device="cuda")
    v = torch.zeros(N, dtype=torch.float32, device="cuda")
    mc.pack(L, w_table, w.data_ptr(), sh)

    # fused path state: per-layer weights and momentum, updated in place
    fw_layers = upload(w_layers_host)
    fv_layers = [torch.zeros_like(t) for t in fw_layers]
    fw_set = mc.TensorSet(L, [t.data_ptr() for t in fw_layers])
    fv_set = mc.TensorSet(L, [t.data_ptr() for t in fv_layers])
    torch.cuda.synchronize()

    def staged_step(i, ev=None):
        tabs = tables[i % n_sets]
        for p in range(P):
            mc.pack(L, tabs[p], flats[p].data_ptr(), sh)
        if ev is not None:
            ev[0].record(stream)
        mc.reduce_update(L, flat_table, order, g.data_ptr(), w.data_ptr(), v.data_ptr(),
                         cfg.lr, cfg.mu, cfg.wd, sh)
        if ev is not None:
            ev[1].record(stream)
        mc.unpack(L, w.data_ptr(), w_table, sh)

    def fused_step(i, ev=None):
        if ev:
            ev[0].record(stream)
        mc.fused_step(L, tsets[i % n_sets], order, g.data_ptr(), fw_set, fv_set, cfg.lr, cfg.mu, cfg.wd, sh)
        if ev:
            ev[1].record(stream)

    fused = args.path == "fused"
    step = fused_step if fused else staged_step
    kernel_name = "fused_step_kernel" if fused else "reduce_update_kernel"
    kernel_bytes = 4 * (P + 5) * N        # P reads + w, v read and written + g written: same for both kernels
    step_bytes = kernel_bytes if fused else (8 * P + 4 * (P + 5) + 8) * N

    # ---- parity of the very first step of BOTH paths against the oracle (same host bytes) ----
    parity_ref, cpu = {}, None
    staged_step(0)
    torch.cuda.synchronize()
    first = dict(g=g.cpu().numpy(), w=w.cpu().numpy(), v=v.cpu().numpy())
    fused_step(0)
    torch.cuda.synchronize()
    first_fused = dict(g=g.cpu().numpy(), w=[t.cpu().numpy() for t in fw_layers],
                       v=[t.cpu().numpy() for t in fv_layers])
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, order, host_sets, w_layers_host, args.cpu_seconds, parity_ref, step_bytes)
        import oracle
        O = oracle.Layout(cfg.sizes, k)
        ref_layers = dict(w=oracle.unpack(O, parity_ref["w"]), v=oracle.unpack(O, parity_ref["v"]))
        bad = [key for key in ("g", "w", "v")
               if not np.array_equal(first[key].view(np.uint32), parity_ref[key].view(np.uint32))]
        if not np.array_equal(first_fused["g"].view(np.uint32), parity_ref["g"].view(np.uint32)):
            bad.append("fused g")
        for key in ("w", "v"):
            for a, b in zip(first_fused[key], ref_layers[key]):
                if not np.array_equal(a.view(np.uint32), b.view(np.uint32)):
                    bad.append("fused " + key)
                    break
        if bad:
            print(f"bench.py: PARITY FAILURE against the oracle on {bad}", file=sys.stderr)
            sys.exit(4)
    host_sets = None

    def kernel_launch(i):
        if fused:
            mc.fused_step(L, tsets[i % n_sets], order, g.data_ptr(), fw_set, fv_set, cfg.lr, cfg.mu, cfg.wd, sh)
        else:
            mc.reduce_update(L, flat_table, order, g.data_ptr(), w.data_ptr(), v.data_ptr(),
                             cfg.lr, cfg.mu, cfg.wd, sh)

    if args.kernel_only:
        for i in range(args.warmup):
            kernel_launch(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            kernel_launch(args.warmup + i)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
        # known-size traffic for counter calibration: copy_kernel moves copy_bytes each way
        copy_bytes = (N // 4) * 16
        for i in range(3):
            mc.copy(flats[0].data_ptr(), g.data_ptr(), copy_bytes, sh)
        torch.cuda.synchronize()
        print(json.dumps({"kernel": kernel_name, "kernel_only_ms": ms, "GBps": kernel_bytes / ms / 1e6,
                          "kernel_bytes": kernel_bytes, "copy_bytes_each_way": copy_bytes}))
        return

    def timed_steps(fn, warmup, steps, per_step_events):
        """W untimed steps, then EXACTLY `steps` timed ones.  Returns (ms per step by the host
        clock, launch durations of the dominant kernel in ms by HIP events on the launch
        stream).  Staged path: one event pair around reduce_update in every step.  Fused
        path: the step IS the kernel, launched back to back, so one pair around the whole
        timed region gives its average duration (dispatch gaps included) without putting
        event packets between the launches."""
        for i in range(warmup):
            fn(i + 1)
        if per_step_events:
            events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                      for _ in range(steps)]
        else:
            span = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        if not per_step_events:
            span[0].record(stream)
        for i in range(steps):
            fn(warmup + 1 + i, events[i] if per_step_events else None)
        if not per_step_events:
            span[1].record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        if per_step_events:
            return wall * 1e3 / steps, np.array([a.elapsed_time(b) for a, b in events])
        return wall * 1e3 / steps, np.array([span[0].elapsed_time(span[1]) / steps])

    ms_per_step, k_ms = timed_steps(step, args.warmup, args.steps, per_step_events=not fused)
    other_ms, other_k_ms = timed_steps(staged_step if fused else fused_step, args.warmup, args.steps,
                                       per_step_events=fused)

    # Median and minimum of single launches of the fused kernel, from one event pair per launch in a
    # separate untimed pass (the event packets between launches add a few microseconds to each, which
    # is why the timed region above brackets all its launches with one pair instead).
    _, fused_each = timed_steps(fused_step, 2, max(10, min(args.steps, 100)), per_step_events=True)

    # ---- the pieces on their own (events around back-to-back launches), and the copy yardstick
    def timed(fn, reps):
        a = torch.cuda.Event(enable_timing=True)
        b = torch.cuda.Event(enable_timing=True)
        fn(0)
        torch.cuda.synchronize()
        a.record(stream)
        for r in range(reps):
            fn(r + 1)
        b.record(stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    reps = max(10, min(args.steps, 50))
    pack_ms = timed(lambda r: mc.pack(L, tables[r % n_sets][r % P], flats[r % P].data_ptr(), sh), reps)
    unpack_ms = timed(lambda r: mc.unpack(L, w.data_ptr(), w_table, sh), reps)
    copy_ms = timed(lambda r: mc.copy(flats[r % P].data_ptr(), flats[(r + 1) % P].data_ptr(), 4 * (N // 4) * 4, sh), reps)

    pipelined = None
    if args.pipeline_packets > 0:
        pipelined = pipeline_experiment(torch, mc, L, cfg, order, flats, flat_table, g, w, v, stream,
                                        args.pipeline_packets, reps=max(5, min(args.steps, 30)))

    roles = None
    if args.roles_nodes > 0:
        roles = roles_experiment(torch, mc, L, cfg, flats, g, w, v, stream, args.roles_nodes,
                                 reps=max(5, min(args.steps, 30)))

    k_avg = float(k_ms.mean())
    achieved = kernel_bytes / k_avg / 1e6
    staged_bytes = (8 * P + 4 * (P + 5) + 8) * N
    staged_ms, staged_k = (other_ms, other_k_ms) if fused else (ms_per_step, k_ms)
    fused_ms, fused_k = (ms_per_step, k_ms) if fused else (other_ms, other_k_ms)
    out = {
        "metric": METRIC,
        "value": round(step_bytes / ms_per_step / 1e6, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.n_tensors} tensors, N={N} fp32, P={P}, k={k}, "
                               f"lr={cfg.lr} mu={cfg.mu} wd={cfg.wd}, order={args.order}, "
                               f"{n_sets} rotating contribution sets",
                   "path": args.path,
                   "step": ("mc_fused_step: contributions read from per-layer tensors, per-layer weights and "
                            "momentum updated in place, flat grad_out written" if fused else
                            f"{P} x mc_pack + mc_reduce_update (writes grad_out) + mc_unpack(weights)"),
                   "step_bytes": step_bytes},
        "pct_of_hbm_peak": round(100 * step_bytes / ms_per_step / 1e6 / HBM_PEAK_GBPS, 2),
        "fused_step": {"ms_per_step": round(fused_ms, 4), "kernel_ms": round(float(fused_k.mean()), 4),
                       "GBps": round(kernel_bytes / float(fused_k.mean()) / 1e6, 1), "step_bytes": kernel_bytes,
                       "single_launch_ms_median": round(float(np.median(fused_each)), 4),
                       "single_launch_ms_min": round(float(fused_each.min()), 4)},
        "staged_step": {"ms_per_step": round(staged_ms, 4), "GBps": round(staged_bytes / staged_ms / 1e6, 1),
                        "step_bytes": staged_bytes,
                        "reduce_update_ms": round(float(staged_k.mean()), 4),
                        "reduce_update_ms_min": round(float(staged_k.min()), 4),
                        "reduce_update_GBps": round(kernel_bytes / float(staged_k.mean()) / 1e6, 1),
                        "pack_ms": round(pack_ms, 4), "pack_GBps": round(8 * N / pack_ms / 1e6, 1),
                        "unpack_ms": round(unpack_ms, 4), "unpack_GBps": round(8 * N / unpack_ms / 1e6, 1)},
        "copy_yardstick": {"ms": round(copy_ms, 4), "GBps": round(8 * (N // 4) * 4 / copy_ms / 1e6, 1)},
        "layout_create_ms": round(layout_ms, 3),
        "roofline": {"bound": "hbm", "kernel": kernel_name, "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": measured_traffic(kernel_name, cfg.name, P, k), "bytes_per_launch": kernel_bytes,
                     "kernel_ms": round(k_avg, 4)},
        "pipelined_packets": pipelined,
        "roles": roles,
        "cpu_baseline": cpu,
        "parity_checked_first_step": cpu is not None,
        "library": os.path.relpath(mc.LIBRARY_PATH, ROOT),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
