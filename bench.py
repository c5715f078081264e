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
step on the headline workload with steps launched back to back ("warm": weights and momentum
of a ResNet-50-sized model stay in the 256 MB memory-side cache between steps).
`roofline` is for the dominant kernel, timed with events on the stream it is launched on,
inside the timed region.  `roofline_cold` is the same step when nothing of the previous step is
still cached -- weights, momentum and g rotate over enough buffer sets to exceed the cache,
as after the forward / backward pass that separates two steps of real training.
`workloads` holds the other four configurations (fused step, first step checked against the
oracle).  `cpu_baseline` is the CPU oracle timed on this machine's host cores on the headline workload.
"""
import argparse
import hashlib
import json
import os
import sys
import threading
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0     # MI355X published HBM3E bandwidth
CACHE_BYTES = 256 << 20    # memory-side cache
METRIC = "effective HBM GB/s (% of MI355X peak) and ms per ResNet-50-shaped reduce+update"
WORKLOADS = ["tiny", "resnet50", "resnet50_heavy", "vgg16", "googlenet"]


def progress(msg):
    """One line per phase on stderr, so that a long default run is visibly alive."""
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def csrc_digest():
    """Hash of the kernel sources: a counter profile is only quoted while it matches them."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_1711_00705_amd", "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".h", ".cpp")):
            h.update(name.encode())
            h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()[:16]


def traffic_from_profile(kernel, workload, P, k, suffix=""):
    """HBM-side bytes per launch of the dominant kernel from the rocprofv3 counter runs whose
    summary is kept under profiles/ -- or None when there is no summary for this kernel and
    workload, or when the kernel sources have changed since it was taken."""
    path = os.path.join(ROOT, "profiles", f"{kernel.replace('_kernel', '')}_{workload}_P{P}_k{k}{suffix}.txt")
    traffic = digest = None
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = int(line.split(":")[1])
            if line.startswith("csrc_digest:"):
                digest = line.split(":")[1].strip()
    except OSError:
        return None, "no counter profile for this kernel and workload"
    if digest != csrc_digest():
        return None, f"{os.path.relpath(path, ROOT)} was taken with other kernel sources (digest {digest})"
    return traffic, os.path.relpath(path, ROOT)


def kernel_names(mc, L, P, k):
    """Which kernels the library launches for the uniform step under the current options."""
    how = mc.get_option(mc.OPT_DIRECT_TILES)
    plain = mc.get_option(mc.OPT_RU_SHAPE) != 2 and mc.get_option(mc.OPT_XCD_RUN) < 2 and P <= 8 and k <= 32
    if not plain or how == 0:
        return "fused_step_kernel", "reduce_update_kernel"
    fused = "fused_unit_kernel" if how == 1 and L.units()[0] > 0 else "fused_direct_kernel"
    return fused, "reduce_update_direct_kernel"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="resnet50", choices=WORKLOADS)
    ap.add_argument("--sets", type=int, default=0,
                    help="rotating sets of contribution tensors (0 = pick so that no step re-reads a cached set)")
    ap.add_argument("--order", default="rotation", choices=["identity", "rotation"])
    ap.add_argument("--path", default="fused", choices=["fused", "staged"],
                    help="fused: one mc_fused_step per step; staged: P packs + reduce_update + unpack")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--only-headline", action="store_true",
                    help="skip the cold pass, the roles figures and the other four workloads")
    ap.add_argument("--pipeline-packets", type=int, default=4,
                    help="packets per colour of the packet-pipelined experiment (0 = skip)")
    ap.add_argument("--packet-blocks", type=int, default=256,
                    help="packet pipeline: workgroups of the resident reducer")
    ap.add_argument("--arrival-gbps", type=float, default=50.0,
                    help="packet pipeline: rate at which arriving contributions land, GB/s (50 = four 100 Gb/s adapters)")
    ap.add_argument("--roles-nodes", type=int, default=8,
                    help="time one rank's role-dependent step in a tree Allreduce over this many nodes (0 = skip)")
    ap.add_argument("--shape", type=int, default=0,
                    help="workgroup shape of the update kernels (0 = the library picks)")
    ap.add_argument("--state-policy", type=int, default=0, choices=[0, 1, 2],
                    help="what the default state policy means (0 = the library's default, 1 resident, 2 streaming)")
    ap.add_argument("--state-store-sc1", type=int, default=-1, choices=[-1, 0, 1])
    ap.add_argument("--alternate-sweep", type=int, default=-1, choices=[-1, 0, 1])
    ap.add_argument("--direct-tiles", type=int, default=-1, choices=[-1, 0, 1, 2])
    ap.add_argument("--lds-cap-update", type=int, default=-2)
    ap.add_argument("--lds-cap-pack", type=int, default=-2)
    ap.add_argument("--xcd-run", type=int, default=-1)
    ap.add_argument("--xcd-run-pack", type=int, default=-2)
    ap.add_argument("--xcd-run-unpack", type=int, default=-2)
    ap.add_argument("--kernel-only", action="store_true",
                    help="time only the dominant kernel's launches (for profiler runs)")
    ap.add_argument("--cold", action="store_true",
                    help="with --kernel-only: launch the cold-state form (rotating state sets, streaming hint)")
    return ap.parse_args()


# ------------------------------------------------------------------------------------------
class Harness:
    """torch supplies device memory and the stream; everything timed is the library's."""

    def __init__(self, torch, mc, wl, args):
        self.torch, self.mc, self.wl, self.args = torch, mc, wl, args
        self.stream = torch.cuda.current_stream()
        self.sh = int(self.stream.cuda_stream)
        self.pool = ThreadPoolExecutor(max_workers=8)

    def upload(self, layers):
        return [self.torch.from_numpy(t).cuda() for t in layers]

    def host_set(self, cfg, step):
        """Contributions 0..P-1 of one step, generated on host threads (numpy releases the GIL)."""
        return list(self.pool.map(
            lambda p: self.wl.contribution_tensors(cfg.sizes, p, step=step, heavy_tail=cfg.heavy_tail), range(cfg.P)))

    def events(self):
        return self.torch.cuda.Event(enable_timing=True), self.torch.cuda.Event(enable_timing=True)

    def time_region(self, fn, warmup, steps):
        """W untimed calls, then EXACTLY `steps` timed ones bracketed by synchronisation.  Returns
        (ms per call by the host clock, ms per call by one HIP event pair around the region on the
        launch stream): back-to-back launches, no event packets between them."""
        torch = self.torch
        for i in range(warmup):
            fn(i)
        a, b = self.events()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        a.record(self.stream)
        for i in range(steps):
            fn(warmup + i)
        b.record(self.stream)
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3 / steps
        return wall, a.elapsed_time(b) / steps

    def time_each(self, fn, warmup, steps):
        """One event pair per call (adds a few microseconds to each): for medians and minima."""
        for i in range(warmup):
            fn(i)
        evs = [self.events() for _ in range(steps)]
        self.torch.cuda.synchronize()
        for i, (a, b) in enumerate(evs):
            a.record(self.stream)
            fn(warmup + i)
            b.record(self.stream)
        self.torch.cuda.synchronize()
        return np.array([a.elapsed_time(b) for a, b in evs])


class Inputs:
    """One workload resident in HBM: n_sets rotating contribution sets as per-layer tensors."""

    def __init__(self, H, cfg, n_sets, keep_host_sets):
        mc, wl = H.mc, H.wl
        self.cfg, self.n_sets = cfg, n_sets
        t0 = time.perf_counter()
        self.L = mc.Layout(cfg.sizes, cfg.k)
        self.layout_ms = (time.perf_counter() - t0) * 1e3
        self.L.prepare()
        self.host_sets, self.dev_sets, self.tables, self.tsets = [], [], [], []
        for s in range(n_sets):
            per_p = H.host_set(cfg, s)
            if s < keep_host_sets:
                self.host_sets.append(per_p)
            dev = [H.upload(ts) for ts in per_p]
            self.dev_sets.append(dev)
            self.tables.append([mc.ptr_table([t.data_ptr() for t in d]) for d in dev])
            self.tsets.append(mc.set_table([mc.TensorSet(self.L, [t.data_ptr() for t in d]) for d in dev]))
        self.w_host = wl.weight_tensors(cfg.sizes)

    def state_set(self, H):
        """Per-layer weights (seeded) and zero momentum, with their tensor sets."""
        w = H.upload(self.w_host)
        v = [H.torch.zeros_like(t) for t in w]
        return dict(w=w, v=v, wset=H.mc.TensorSet(self.L, [t.data_ptr() for t in w]),
                    vset=H.mc.TensorSet(self.L, [t.data_ptr() for t in v]))


def n_sets_for(cfg, args):
    set_bytes = 4 * cfg.total * cfg.P
    # enough rotating sets that a step never finds its contributions in the memory-side cache
    n = args.sets or (cfg.steps if cfg.steps > 1 else max(3, int(np.ceil(1.2e9 / set_bytes))))
    return min(n, 100)


def oracle_first_step(cfg, order, host_set, w_host):
    """The oracle's pack x P -> reduce_update -> unpack on the first contribution set."""
    import oracle
    O = oracle.Layout(cfg.sizes, cfg.k)
    w = oracle.pack(O, w_host)
    v = np.zeros(O.N, np.float32)
    xs = [oracle.pack(O, ts) for ts in host_set]
    g = oracle.reduce_update(O, xs, w, v, cfg.lr, cfg.mu, cfg.wd, order=order)
    return dict(g=g, w=w, v=v, w_layers=oracle.unpack(O, w), v_layers=oracle.unpack(O, v))


def same_bits(a, b):
    return np.array_equal(np.ascontiguousarray(a).view(np.uint32), np.ascontiguousarray(b).view(np.uint32))


def fused_parity(H, I, order, ref):
    """One mc_fused_step from the seeded initial state on set 0, compared bit for bit."""
    cfg, mc, torch = I.cfg, H.mc, H.torch
    st = I.state_set(H)
    g = torch.empty(cfg.total, dtype=torch.float32, device="cuda")
    mc.fused_step(I.L, I.tsets[0], order, g.data_ptr(), st["wset"], st["vset"], cfg.lr, cfg.mu, cfg.wd, H.sh)
    torch.cuda.synchronize()
    bad = []
    if not same_bits(g.cpu().numpy(), ref["g"]):
        bad.append("fused g")
    for key, layers in (("w", st["w"]), ("v", st["v"])):
        if not all(same_bits(a.cpu().numpy(), b) for a, b in zip(layers, ref[key + "_layers"])):
            bad.append("fused " + key)
    return bad


def cold_pass(H, I, order, steps, warmup):
    """The fused step with nothing left in the caches from the step before: weights, momentum and g
    rotate over enough sets to exceed three times the memory-side cache (contributions rotate anyway).
    Timed with the state policy a caller would pass when a forward / backward pass separates the
    steps (streaming) and, for comparison, with the policy that suits back-to-back steps (resident)."""
    cfg, mc, torch = I.cfg, H.mc, H.torch
    N, P = cfg.total, cfg.P
    n_state = max(4, int(np.ceil(3 * CACHE_BYTES / (8 * N))))
    n_g = max(4, int(np.ceil(3 * CACHE_BYTES / (4 * N))))
    states = [I.state_set(H) for _ in range(n_state)]
    gs = [torch.empty(N, dtype=torch.float32, device="cuda") for _ in range(n_g)]
    bytes_ = 4 * (P + 5) * N
    out = {"state_sets": n_state, "g_buffers": n_g, "contribution_sets": I.n_sets}
    for name, policy in (("streaming", mc.STATE_STREAMING), ("resident", mc.STATE_RESIDENT)):
        spec = mc.update_spec(cfg.lr, cfg.mu, cfg.wd, state_policy=policy, sweep=mc.SWEEP_FORWARD)

        def step(i):
            st = states[i % n_state]
            mc.fused_step_ex(I.L, I.tsets[i % I.n_sets], order, gs[i % n_g].data_ptr(), st["wset"], st["vset"],
                             spec, H.sh)
        wall, ev = H.time_region(step, warmup, steps)
        out[name] = {"ms_per_step": round(wall, 4), "kernel_ms": round(ev, 4),
                     "GBps": round(bytes_ / ev / 1e6, 1), "frac": round(bytes_ / ev / 1e6 / HBM_PEAK_GBPS, 4)}
    return out, states, gs


def replayed_pair(H, I, order, g, st, cfg, warmup, steps):
    """The same back-to-back steps from two captured graphs, one per contribution set and walking
    direction (a graph replays the direction it captured, so a caller whose state exceeds the cache
    captures one of each and alternates them)."""
    mc, torch = H.mc, H.torch
    graphs = []
    for j, sweep in enumerate((mc.SWEEP_FORWARD, mc.SWEEP_BACKWARD)):
        spec = mc.update_spec(cfg.lr, cfg.mu, cfg.wd, sweep=sweep)
        cap = torch.cuda.Stream()
        cap.wait_stream(H.stream)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=cap):
            mc.fused_step_ex(I.L, I.tsets[j], order, g.data_ptr(), st["wset"], st["vset"], spec,
                             int(torch.cuda.current_stream().cuda_stream))
        torch.cuda.synchronize()
        graphs.append(graph)
    for i in range(warmup):
        graphs[i % 2].replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        graphs[(warmup + i) % 2].replay()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    bytes_ = 4 * (cfg.P + 5) * cfg.total
    return {"ms_per_step": round(ms, 4), "GBps": round(bytes_ / ms / 1e6, 1),
            "what": "two captured graphs (forward sweep on set 0, backward sweep on set 1) replayed alternately"}


def replayed_chain(H, I, order, g, st, cfg, n_sets, chain=20, reps=10):
    """A launch-bound step (microseconds of work) as a caller would run it in a loop: `chain`
    consecutive steps over the rotating contribution sets captured into ONE graph, which is then
    replayed; per-step time of the replays against the same steps launched one by one."""
    mc, torch = H.mc, H.torch
    spec = mc.update_spec(cfg.lr, cfg.mu, cfg.wd, sweep=mc.SWEEP_FORWARD)
    cap = torch.cuda.Stream()
    cap.wait_stream(H.stream)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=cap):
        sh = int(torch.cuda.current_stream().cuda_stream)
        for j in range(chain):
            mc.fused_step_ex(I.L, I.tsets[j % n_sets], order, g.data_ptr(), st["wset"], st["vset"], spec, sh)
    torch.cuda.synchronize()
    for _ in range(2):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        graph.replay()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / (reps * chain)
    bytes_ = 4 * (cfg.P + 5) * cfg.total
    return {"ms_per_step": round(ms, 5), "GBps": round(bytes_ / ms / 1e6, 1),
            "what": f"{chain} consecutive steps captured into one graph, {reps} replays"}


def staggered_arenas(H, I, order, g, st, cfg, warmup, steps, apart_bytes=4096):
    """The same steps with every operand set (each contribution, weights, momentum) copied into one
    arena of its own, the arenas' first tensors 4 KB apart in address phase.  When nothing of the state
    fits the cache, all P + 2 streams of a tile come from HBM at once, and where they sit relative to
    one another decides how many of them meet in the same DRAM bank: tensors allocated one by one put
    every large tensor on a 2 MB boundary, i.e. all operands of a tile in the same phase."""
    mc, torch = H.mc, H.torch
    N, P = cfg.total, cfg.P
    pad = apart_bytes // 4
    keep = []

    def arena_copy(q, layers):
        arena = torch.empty(N + (P + 3) * pad, dtype=torch.float32, device="cuda")
        keep.append(arena)
        views, o = [], q * pad
        for t in layers:
            v = arena[o:o + t.numel()]
            v.copy_(t)
            views.append(v)
            o += t.numel()
        return mc.TensorSet(I.L, [v.data_ptr() if v.numel() else None for v in views])

    tsets = [mc.set_table([arena_copy(p, I.dev_sets[s][p]) for p in range(P)]) for s in range(I.n_sets)]
    wset, vset = arena_copy(P, st["w"]), arena_copy(P + 1, st["v"])

    def step(i):
        mc.fused_step(I.L, tsets[i % I.n_sets], order, g.data_ptr(), wset, vset, cfg.lr, cfg.mu, cfg.wd, H.sh)
    wall, ev = H.time_region(step, warmup, steps)
    bytes_ = 4 * (P + 5) * N
    del tsets, wset, vset, keep
    torch.cuda.empty_cache()
    return {"ms_per_step": round(wall, 4), "kernel_ms": round(ev, 4), "GBps": round(bytes_ / wall / 1e6, 1),
            "frac": round(bytes_ / ev / 1e6 / HBM_PEAK_GBPS, 4),
            "what": f"each operand set in one arena, arenas {apart_bytes} B apart in address phase"}


def flat_yardsticks(H, L, cfg, order, warmup, steps):
    """mc_reduce_update on flat buffers, launched back to back on its own: the step's arithmetic and
    access mix with no per-layer lookups at all (one fetch from the argument block per tile), i.e. what
    the fused step would reach if finding its tensors cost nothing.  Warm: one state set; cold: weights,
    momentum and g rotate over sets that exceed the memory-side cache, streaming state policy."""
    mc, torch = H.mc, H.torch
    N, P = cfg.total, cfg.P
    n_x = max(3, int(np.ceil(1.2e9 / (4 * N * P))))
    n_state = max(4, int(np.ceil(3 * CACHE_BYTES / (8 * N))))
    n_g = max(4, int(np.ceil(3 * CACHE_BYTES / (4 * N))))
    gen = torch.Generator(device="cuda")
    gen.manual_seed(wl_seed())
    xs = [[torch.randn(N, device="cuda", generator=gen) * 1e-3 for _ in range(P)] for _ in range(n_x)]
    ws = [torch.randn(N, device="cuda", generator=gen) * 0.05 for _ in range(n_state)]
    vs = [torch.zeros(N, device="cuda") for _ in range(n_state)]
    gs = [torch.empty(N, device="cuda") for _ in range(n_g)]
    tabs = [[t.data_ptr() for t in x] for x in xs]
    bytes_ = 4 * (P + 5) * N
    out = {"kernel": kernel_names(mc, L, P, cfg.k)[1], "bytes_per_launch": bytes_,
           "what": "mc_reduce_update alone on flat buffers (no per-layer lookups), random data"}
    for name, policy, rotate in (("back_to_back", mc.STATE_RESIDENT, False), ("cold", mc.STATE_STREAMING, True)):
        spec = mc.update_spec(cfg.lr, cfg.mu, cfg.wd, state_policy=policy, sweep=mc.SWEEP_FORWARD)

        def launch(i):
            s_ = i % n_state if rotate else 0
            mc.reduce_update_ex(L, tabs[i % n_x], order, gs[i % n_g if rotate else 0].data_ptr(),
                                ws[s_].data_ptr(), vs[s_].data_ptr(), spec, H.sh)
        _, ev = H.time_region(launch, warmup, steps)
        out[name] = {"kernel_ms": round(ev, 4), "GBps": round(bytes_ / ev / 1e6, 1),
                     "frac": round(bytes_ / ev / 1e6 / HBM_PEAK_GBPS, 4)}
    del xs, ws, vs, gs
    torch.cuda.empty_cache()
    return out


def wl_seed():
    return 171100705 + 424242


def run_other_workload(H, name, order_kind, check_parity):
    """Fused step of one of the non-headline configurations: first step against the oracle, then
    W warm-up + K timed back-to-back steps over rotating contribution sets."""
    mc, wl, torch = H.mc, H.wl, H.torch
    cfg = wl.workload(name)
    N, P, k = cfg.total, cfg.P, cfg.k
    order = None if order_kind == "identity" else wl.rotation_order(k, P)
    n_sets = n_sets_for(cfg, H.args)
    if name == "vgg16":
        n_sets = 2                      # 2.2 GB per set: two already exceed the cache many times over
    K, W = {"tiny": (200, 20), "resnet50": (50, 10), "resnet50_heavy": (50, 10), "vgg16": (20, 5),
            "googlenet": (100, 10)}[name]
    progress(f"{name}: generating and uploading {n_sets} contribution sets")
    t0 = time.perf_counter()
    I = Inputs(H, cfg, n_sets, keep_host_sets=1)
    setup_s = time.perf_counter() - t0
    progress(f"{name}: parity of the first step, then {W} + {K} steps")
    out = {"config": f"{cfg.n_tensors} tensors, N={N} fp32, P={P}, k={k}, lr={cfg.lr} mu={cfg.mu} wd={cfg.wd}, "
                     f"order={order_kind}, {n_sets} rotating contribution sets",
           "steps": K, "warmup": W}
    if check_parity:
        ref = oracle_first_step(cfg, order, I.host_sets[0], I.w_host)
        bad = fused_parity(H, I, order, ref)
        if bad:
            print(f"bench.py: PARITY FAILURE against the oracle on {name}: {bad}", file=sys.stderr)
            sys.exit(4)
        out["parity_first_step"] = True
    else:
        out["parity_first_step"] = None
    I.host_sets = None
    st = I.state_set(H)
    g = torch.empty(N, dtype=torch.float32, device="cuda")
    bytes_ = 4 * (P + 5) * N

    def step(i):
        mc.fused_step(I.L, I.tsets[i % n_sets], order, g.data_ptr(), st["wset"], st["vset"], cfg.lr, cfg.mu, cfg.wd, H.sh)
    wall, ev = H.time_region(step, W, K)
    state_bytes = 8 * N
    out.update({"ms_per_step": round(wall, 4), "kernel_ms": round(ev, 4), "step_bytes": bytes_,
                "GBps": round(bytes_ / wall / 1e6, 1), "frac": round(bytes_ / ev / 1e6 / HBM_PEAK_GBPS, 4),
                "state": ("weights + momentum (%d MB) exceed the memory-side cache: kept resident as far as they "
                          "fit, successive steps walk the payload in opposite directions" % (state_bytes >> 20))
                if state_bytes > CACHE_BYTES else
                ("weights + momentum (%d MB) stay cache-resident between back-to-back steps" % (state_bytes >> 20)),
                "setup_s": round(setup_s, 1)})
    if state_bytes > CACHE_BYTES and n_sets == 2:
        out["graph_replay"] = replayed_pair(H, I, order, g, st, cfg, W, K)
        out["operands_in_staggered_arenas"] = staggered_arenas(H, I, order, g, st, cfg, W, K)
    if name == "tiny":
        out["graph_replay"] = replayed_chain(H, I, order, g, st, cfg, n_sets)
    if name != "tiny":
        cold, states, gs = cold_pass(H, I, order, K, W)
        out["cold"] = cold
        del states, gs
    del I, st, g
    torch.cuda.empty_cache()
    return out


def cpu_baseline(cfg, order, host_sets, w_layers_host, seconds, parity_ref, gpu_step_ms):
    """The oracle as it stands: whole step (P packs, reduce+update, unpack) on host cores.  Its GB/s is
    over the bytes the oracle itself moves, (8P + 4(P+5) + 8) * N per step."""
    import oracle
    O = oracle.Layout(cfg.sizes, cfg.k)
    N = O.N
    moved = (8 * cfg.P + 4 * (cfg.P + 5) + 8) * N
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
        "value": round(moved / dt / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
        "ms_per_step": round(dt * 1e3, 3), "bytes_moved_per_step": moved,
        "step_time_ratio_vs_gpu": round(dt * 1e3 / gpu_step_ms, 1) if gpu_step_ms else None,
        "sample": f"{n} whole steps ({cfg.P} packs + reduce+update + unpack) of the full {cfg.name} "
                  f"workload, N={N}, single thread",
        "threaded": {"value": round(moved / dt2 / 1e9, 3), "unit": "GB/s",
                     "cores": max(nthr, min(cfg.P, ncpu)), "ms_per_step": round(dt2 * 1e3, 3),
                     "sample": f"{n2} whole steps, one host thread per colour ({nthr}) / per pack ({cfg.P})"},
        "host_cpus": ncpu,
    }


def roles_experiment(H, L, cfg, flats, g, w, v, n_nodes, reps, I=None, wset=None, vset=None):
    """One rank's real share in a k-colour tree Allreduce over n_nodes nodes (Section 4.2): it
    is inner node or root of at most one colour and a leaf of the others.  Phase 1: per colour,
    add the m local replicas (leaf) or those plus one buffer per child (inner node, root); only
    the root's colour is updated at once -- one launch whatever the mix.  Phase 2: the other colours
    are updated from the broadcast sum (a single contribution).  m = the workload's P; child
    buffers are further flat buffers of the same size.  Times both phases for one rank of each
    kind, with the algorithmic bytes of each -- on flat buffers (mc_reduce_update_roles) and, given the
    per-layer inputs, on per-layer tensors (mc_fused_step_ex with the same roles)."""
    torch, mc = H.torch, H.mc
    N, m, k = cfg.total, cfg.P, cfg.k
    fused_sets = fused_bcast = None
    if I is not None and I.n_sets >= 3 and k <= len(I.dev_sets[1]):
        def tset(layers):
            return mc.TensorSet(L, [t.data_ptr() if t.numel() else None for t in layers])
        keep_sets = [tset(I.dev_sets[0][p]) for p in range(m)] + [tset(I.dev_sets[1][c]) for c in range(k)]
        fused_sets = mc.set_table(keep_sets)
        keep_bcast = [tset(I.dev_sets[2][0])]
        fused_bcast = mc.set_table(keep_bcast)
        spec = mc.update_spec(cfg.lr, cfg.mu, cfg.wd)
    bounds = [int(b) for b in L.colour_bounds()]
    lens = [bounds[c + 1] - bounds[c] for c in range(k)]
    child_bufs = [torch.randn(N, dtype=torch.float32, device="cuda") * 1e-3 for _ in range(k)]
    contrib = mc.ptr_table([f.data_ptr() for f in flats] + [c.data_ptr() for c in child_bufs])
    bcast = torch.randn(N, dtype=torch.float32, device="cuda") * 1e-3
    bcast_tab = mc.ptr_table([bcast.data_ptr()])

    def timed(fn):
        _, ev = H.time_region(lambda i: fn(), 2, reps)
        return ev

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
                                                  v.data_ptr(), cfg.lr, cfg.mu, cfg.wd, H.sh))
        # every colour of this call updates, so no grad_out is needed
        t2 = timed(lambda: mc.reduce_update_roles(L, bcast_tab, None, later, [1] * k, None,
                                                  w.data_ptr(), v.data_ptr(), cfg.lr, cfg.mu, cfg.wd, H.sh)) \
            if any(later) else 0.0
        out["ranks"][kind] = {"rank": rank, "terms_per_colour": n_terms, "updates_at_once": upd,
                              "sum_ms": round(t1, 4), "sum_GBps": round(bytes1 / t1 / 1e6, 1),
                              "update_from_broadcast_ms": round(t2, 4),
                              "update_GBps": round(bytes2 / t2 / 1e6, 1) if t2 else None}
        if fused_sets is not None:
            f1 = timed(lambda: mc.fused_step_ex(L, fused_sets, None, g.data_ptr(), wset, vset, spec, H.sh,
                                                n_terms=n_terms, do_update=upd))
            f2 = timed(lambda: mc.fused_step_ex(L, fused_bcast, None, None, wset, vset, spec, H.sh,
                                                n_terms=later, do_update=[1] * k)) if any(later) else 0.0
            out["ranks"][kind].update({"per_layer_sum_ms": round(f1, 4), "per_layer_sum_GBps": round(bytes1 / f1 / 1e6, 1),
                                       "per_layer_update_from_broadcast_ms": round(f2, 4),
                                       "per_layer_update_GBps": round(bytes2 / f2 / 1e6, 1) if f2 else None})
    return out


def pipeline_experiment(H, L, cfg, order, flats, flat_table, g, w, v, packets, reps, arrival_gbps, blocks=256):
    """Section 4.2 pipelines the reductions packet by packet: a summing rank adds a packet when it
    arrives.  Here half of the P contributions are resident and the other half arrive: a producer
    stream delivers them packet by packet (colours interleaved, as the colours progress concurrently)
    into the receive buffers, paced with mc_delay to the rate of a network (`arrival_gbps` GB/s; a
    copy inside one GPU would "arrive" faster than anything can be summed).  Three ways to consume:
      unpipelined     wait for the last packet, then one mc_reduce_update over the whole payload;
      event-pipelined per packet an event wait on the compute stream, then mc_reduce_update_range;
      flag-pipelined  one resident mc_reduce_update_packets polling per-packet device flags that
                      mc_packet_deliver raises, plus the ordered second call that finishes the rest.
    What pipelining can win is the time from the LAST packet's arrival to the end of the step (the
    whole sum for the unpipelined form, one packet's worth for a pipelined one): `tail_ms`."""
    torch, mc, stream = H.torch, H.mc, H.stream
    N, P, k = cfg.total, cfg.P, cfg.k
    arriving = list(range(P // 2, P))
    src = [torch.randn(N, dtype=torch.float32, device="cuda") * 1e-3 for _ in arriving]
    prod = torch.cuda.Stream()
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
    n_pk = len(order_of_packets)
    n_blocks = min(blocks, 2 * torch.cuda.get_device_properties(0).multi_processor_count)   # the entry point's limit
    pk_dev = torch.tensor(np.array(order_of_packets, dtype=np.int64).reshape(-1), device="cuda")
    ready = torch.zeros(n_pk, dtype=torch.int32, device="cuda")
    progress_dev = torch.zeros(n_blocks + mc.PACKETS_STATUS_WORDS, dtype=torch.int32, device="cuda")
    spec = mc.update_spec(cfg.lr, cfg.mu, cfg.wd)
    mh, ph = int(stream.cuda_stream), int(prod.cuda_stream)

    def wire_us(b, e):
        return max(1, int(round(len(arriving) * 4 * (e - b) / (arrival_gbps * 1e3))))

    def deliver(j, b, e):
        """One packet lands: the wire time, then the data of every arriving contribution."""
        mc.delay(wire_us(b, e), ph)
        for q, s_ in zip(arriving, src):
            mc.packet_deliver(flats[q].data_ptr() + 4 * b, s_.data_ptr() + 4 * b, e - b, ready.data_ptr() + 4 * j, ph)

    def unpipelined(last):
        prod.wait_stream(stream)
        for j, (b, e) in enumerate(order_of_packets):
            deliver(j, b, e)
        last.record(prod)
        stream.wait_stream(prod)
        mc.reduce_update(L, flat_table, order, g.data_ptr(), w.data_ptr(), v.data_ptr(), cfg.lr, cfg.mu, cfg.wd, mh)

    def event_pipelined(last):
        prod.wait_stream(stream)
        for j, (b, e) in enumerate(order_of_packets):
            deliver(j, b, e)
            ev = torch.cuda.Event()
            ev.record(prod)
            stream.wait_event(ev)
            mc.reduce_update_range(L, flat_table, order, g.data_ptr(), w.data_ptr(), v.data_ptr(),
                                   cfg.lr, cfg.mu, cfg.wd, b, e, mh)
        last.record(prod)
        stream.wait_stream(prod)

    def flag_pipelined(last):
        mc.packets_reset(ready.data_ptr(), n_pk, progress_dev.data_ptr(), n_blocks, mh)
        prod.wait_stream(stream)

        def reducer():
            mc.reduce_update_packets(L, flat_table, order, g.data_ptr(), w.data_ptr(), v.data_ptr(), spec,
                                     pk_dev.data_ptr(), n_pk, ready.data_ptr(), len(arriving), 200000,
                                     progress_dev.data_ptr(), n_blocks, mh)
        reducer()
        for j, (b, e) in enumerate(order_of_packets):
            deliver(j, b, e)
        last.record(prod)
        stream.wait_stream(prod)
        reducer()

    def timed(fn):
        """Mean over reps of (whole step, time from the last packet's arrival to the end of the step)."""
        tot, tail = [], []
        for r in range(reps + 1):
            a, last, z = (torch.cuda.Event(enable_timing=True) for _ in range(3))
            torch.cuda.synchronize()
            a.record(stream)
            fn(last)
            z.record(stream)
            torch.cuda.synchronize()
            if r:                                   # the first pass warms up
                tot.append(a.elapsed_time(z))
                tail.append(last.elapsed_time(z))
        return round(float(np.mean(tot)), 4), round(float(np.mean(tail)), 4)

    wire_total = sum(wire_us(b, e) for b, e in order_of_packets) / 1e3
    out = {"packets_per_colour": packets, "n_packets": n_pk, "arriving_contributions": len(arriving),
           "reducer_workgroups": n_blocks, "arrival_GBps": arrival_gbps, "wire_ms_total": round(wire_total, 4)}
    for name, fn in (("unpipelined", unpipelined), ("event_pipelined", event_pipelined), ("flag_pipelined", flag_pipelined)):
        total, tail = timed(fn)
        out[name] = {"step_ms": total, "tail_ms": tail}
    pr = progress_dev.cpu().numpy()
    out["flag_pipelined"]["workgroups_that_gave_up_in_last_step"] = int(pr[n_blocks])
    out["flag_pipelined"]["complete"] = bool((pr[:n_blocks] == n_pk).all())
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
    if args.shape:
        mc.set_option(mc.OPT_RU_SHAPE, args.shape)
    if args.state_policy:
        mc.set_option(mc.OPT_STATE_POLICY, args.state_policy)
    if args.alternate_sweep >= 0:
        mc.set_option(mc.OPT_ALTERNATE_SWEEP, args.alternate_sweep)
    if args.state_store_sc1 >= 0:
        mc.set_option(mc.OPT_STATE_STORE_SC1, args.state_store_sc1)
    if args.lds_cap_update >= -1:
        mc.set_option(mc.OPT_LDS_CAP_UPDATE, args.lds_cap_update)
    if args.lds_cap_pack >= -1:
        mc.set_option(mc.OPT_LDS_CAP_PACK, args.lds_cap_pack)
    if args.direct_tiles >= 0:
        mc.set_option(mc.OPT_DIRECT_TILES, args.direct_tiles)
    if args.xcd_run >= 0:
        mc.set_option(mc.OPT_XCD_RUN, args.xcd_run)
    if args.xcd_run_pack >= -1:
        mc.set_option(mc.OPT_XCD_RUN_PACK, args.xcd_run_pack)
    if args.xcd_run_unpack >= -1:
        mc.set_option(mc.OPT_XCD_RUN_UNPACK, args.xcd_run_unpack)
    H = Harness(torch, mc, wl, args)
    stream, sh = H.stream, H.sh
    cfg = wl.workload(args.workload)
    N, P, k = cfg.total, cfg.P, cfg.k
    order = None if args.order == "identity" else wl.rotation_order(k, P)
    n_sets = n_sets_for(cfg, args)

    # ---- inputs: seeded, host-generated, uploaded as separate per-layer tensors ------------
    progress(f"{cfg.name}: generating and uploading {n_sets} contribution sets")
    I = Inputs(H, cfg, n_sets, keep_host_sets=3)
    L, tables, tsets = I.L, I.tables, I.tsets
    w_layers_host = I.w_host
    g = torch.empty(N, dtype=torch.float32, device="cuda")

    # staged path state: flat w, v (master), per-layer weights as the unpack destination
    w_layers = H.upload(w_layers_host)
    w_table = mc.ptr_table([t.data_ptr() for t in w_layers])
    flats = [torch.empty(N, dtype=torch.float32, device="cuda") for _ in range(P)]
    flat_table = mc.ptr_table([f.data_ptr() for f in flats])
    w = torch.empty(N, dtype=torch.float32, device="cuda")
    v = torch.zeros(N, dtype=torch.float32, device="cuda")
    mc.pack(L, w_table, w.data_ptr(), sh)

    # fused path state: per-layer weights and momentum, updated in place
    fst = I.state_set(H)
    fw_layers, fv_layers, fw_set, fv_set = fst["w"], fst["v"], fst["wset"], fst["vset"]
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

    def fused_step(i):
        mc.fused_step(L, tsets[i % n_sets], order, g.data_ptr(), fw_set, fv_set, cfg.lr, cfg.mu, cfg.wd, sh)

    fused = args.path == "fused"
    fused_kernel, staged_kernel = kernel_names(mc, L, P, k)
    kernel_name = fused_kernel if fused else staged_kernel
    kernel_bytes = 4 * (P + 5) * N        # P reads + w, v read and written + g written: same for both kernels
    staged_bytes = (8 * P + 4 * (P + 5) + 8) * N
    step_bytes = kernel_bytes if fused else staged_bytes

    if args.kernel_only:
        if args.cold:
            n_state = max(4, int(np.ceil(3 * CACHE_BYTES / (8 * N))))
            states = [I.state_set(H) for _ in range(n_state)]
            gs = [torch.empty(N, dtype=torch.float32, device="cuda") for _ in range(4)]
            spec = mc.update_spec(cfg.lr, cfg.mu, cfg.wd, state_policy=mc.STATE_STREAMING, sweep=mc.SWEEP_FORWARD)

            def kernel_launch(i):
                st = states[i % n_state]
                mc.fused_step_ex(L, tsets[i % n_sets], order, gs[i % 4].data_ptr(), st["wset"], st["vset"], spec, sh)
        elif fused:
            kernel_launch = fused_step
        else:
            def kernel_launch(i):
                mc.reduce_update(L, flat_table, order, g.data_ptr(), w.data_ptr(), v.data_ptr(),
                                 cfg.lr, cfg.mu, cfg.wd, sh)
        wall, ev = H.time_region(kernel_launch, args.warmup, args.steps)
        # known-size traffic for counter calibration: copy_kernel moves copy_bytes each way
        copy_bytes = (N // 4) * 16
        for i in range(3):
            mc.copy(flats[0].data_ptr(), g.data_ptr(), copy_bytes, sh)
        torch.cuda.synchronize()
        print(json.dumps({"kernel": kernel_name, "cold": bool(args.cold), "kernel_only_ms": ev,
                          "GBps": kernel_bytes / ev / 1e6, "kernel_bytes": kernel_bytes,
                          "copy_bytes_each_way": copy_bytes}))
        return

    progress(f"{cfg.name}: first steps, then {args.warmup} + {args.steps} timed steps of both forms")
    # ---- parity of the very first step of BOTH paths against the oracle (same host bytes) ----
    staged_step(0)
    torch.cuda.synchronize()
    first = dict(g=g.cpu().numpy(), w=w.cpu().numpy(), v=v.cpu().numpy())
    fused_step(0)
    torch.cuda.synchronize()
    first_fused = dict(g=g.cpu().numpy(), w=[t.cpu().numpy() for t in fw_layers],
                       v=[t.cpu().numpy() for t in fv_layers])

    # ---- timing of both forms of the step ---------------------------------------------------
    def timed_staged(warmup, steps):
        """Host clock around K whole staged steps after W untimed ones, one event pair around
        reduce_update in each."""
        for i in range(warmup):
            staged_step(i + 1)
        evs = [H.events() for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            staged_step(warmup + 1 + i, evs[i])
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3 / steps
        return wall, np.array([a.elapsed_time(b) for a, b in evs])

    fused_ms, fused_k = H.time_region(lambda i: fused_step(i + 1), args.warmup, args.steps)
    staged_ms, staged_k = timed_staged(args.warmup, args.steps)
    ms_per_step = fused_ms if fused else staged_ms
    k_avg = fused_k if fused else float(staged_k.mean())

    # Median and minimum of single launches of the fused kernel, from one event pair per launch in a
    # separate untimed pass (the event packets between launches add a few microseconds to each, which
    # is why the timed region above brackets all its launches with one pair instead).
    fused_each = H.time_each(lambda i: fused_step(i + 1), 2, max(10, min(args.steps, 100)))

    # ---- the pieces on their own (events around back-to-back launches), and the copy yardstick
    reps = max(10, min(args.steps, 50))
    _, pack_ms = H.time_region(lambda r: mc.pack(L, tables[r % n_sets][r % P], flats[r % P].data_ptr(), sh), 1, reps)
    _, unpack_ms = H.time_region(lambda r: mc.unpack(L, w.data_ptr(), w_table, sh), 1, reps)
    _, copy_ms = H.time_region(lambda r: mc.copy(flats[r % P].data_ptr(), flats[(r + 1) % P].data_ptr(),
                                                 4 * (N // 4) * 4, sh), 1, reps)

    # ---- CPU oracle: baseline and parity reference ---------------------------------------------
    parity_ref, cpu = {}, None
    if not args.no_cpu_baseline:
        progress(f"{cfg.name}: CPU oracle (baseline and parity reference), about {2 * args.cpu_seconds:.0f} s")
        cpu = cpu_baseline(cfg, order, I.host_sets, w_layers_host, args.cpu_seconds, parity_ref, ms_per_step)
        import oracle
        O = oracle.Layout(cfg.sizes, k)
        ref_layers = dict(w=oracle.unpack(O, parity_ref["w"]), v=oracle.unpack(O, parity_ref["v"]))
        bad = [key for key in ("g", "w", "v") if not same_bits(first[key], parity_ref[key])]
        if not same_bits(first_fused["g"], parity_ref["g"]):
            bad.append("fused g")
        for key in ("w", "v"):
            if not all(same_bits(a, b) for a, b in zip(first_fused[key], ref_layers[key])):
                bad.append("fused " + key)
        if bad:
            print(f"bench.py: PARITY FAILURE against the oracle on {bad}", file=sys.stderr)
            sys.exit(4)
    I.host_sets = None

    pipelined = None
    if args.pipeline_packets > 0 and not args.only_headline and k <= mc.PACKETS_MAX_COLOURS:
        progress(f"{cfg.name}: packet pipelines")
        pipelined = pipeline_experiment(H, L, cfg, order, flats, flat_table, g, w, v,
                                        args.pipeline_packets, reps=max(3, min(args.steps, 10)),
                                        arrival_gbps=args.arrival_gbps, blocks=args.packet_blocks)
    roles = cold = None
    others = {}
    if not args.only_headline:
        progress(f"{cfg.name}: roles and cold-state passes")
        if args.roles_nodes > 0 and k * ((args.roles_nodes - 1 + k - 1) // k) <= args.roles_nodes:
            roles = roles_experiment(H, L, cfg, flats, g, w, v, args.roles_nodes, reps=max(5, min(args.steps, 30)),
                                     I=I, wset=fw_set, vset=fv_set)
        if True:
            cold, states, gs = cold_pass(H, I, order, args.steps, args.warmup)
            del states, gs

    achieved = kernel_bytes / k_avg / 1e6
    traffic, traffic_src = traffic_from_profile(kernel_name, cfg.name, P, k)
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
                   "step_bytes": step_bytes,
                   "state": "warm: steps run back to back, so weights + momentum (%d MB) %s" % (
                       (8 * N) >> 20, "stay in the 256 MB memory-side cache between steps; see roofline_cold"
                       if 8 * N <= CACHE_BYTES else "exceed the memory-side cache; successive steps walk the payload "
                       "in opposite directions so that the part written last is read first")},
        "pct_of_hbm_peak": round(100 * step_bytes / ms_per_step / 1e6 / HBM_PEAK_GBPS, 2),
        "fused_step": {"ms_per_step": round(fused_ms, 4), "kernel_ms": round(fused_k, 4),
                       "GBps": round(kernel_bytes / fused_k / 1e6, 1), "step_bytes": kernel_bytes,
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
        "layout_create_ms": round(I.layout_ms, 3),
        "roofline": {"bound": "hbm", "kernel": kernel_name, "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": traffic, "traffic_source": traffic_src, "bytes_per_launch": kernel_bytes,
                     "kernel_ms": round(k_avg, 4), "state": "warm"},
        "roofline_cold": None,
        "pipelined_packets": pipelined,
        "roles": roles,
        "cpu_baseline": cpu,
        "parity_checked_first_step": cpu is not None,
        "library": os.path.relpath(mc.LIBRARY_PATH, ROOT),
    }
    if cold is not None:
        c = cold["streaming"]
        cold_traffic, cold_src = traffic_from_profile(fused_kernel, cfg.name, P, k, "_cold")
        out["roofline_cold"] = {"bound": "hbm", "kernel": fused_kernel, "achieved": c["GBps"],
                                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": c["frac"],
                                "traffic": cold_traffic, "traffic_source": cold_src,
                                "bytes_per_launch": kernel_bytes, "kernel_ms": c["kernel_ms"],
                                "ms_per_step": c["ms_per_step"], "state_policy": "streaming",
                                "resident_policy": cold["resident"],
                                "rotation": {key: cold[key] for key in ("state_sets", "g_buffers", "contribution_sets")}}

    if not args.only_headline:
        # free the headline's buffers before the large configurations
        del I, tables, tsets, flats, flat_table, w, v, g, fst, fw_layers, fv_layers, fw_set, fv_set, w_layers, w_table
        torch.cuda.empty_cache()
        progress(f"{cfg.name}: the flat kernel alone, back to back and cold")
        out["flat_kernel_yardstick"] = flat_yardsticks(H, L, cfg, order, args.warmup, args.steps)
        for name in WORKLOADS:
            if name != cfg.name:
                others[name] = run_other_workload(H, name, args.order, check_parity=not args.no_cpu_baseline)
    out["workloads"] = others or None
    print(json.dumps(out))


if __name__ == "__main__":
    main()
