#!/usr/bin/env python3
"""Benchmark of the IntSGD compression hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic gradients:
scale + round + clip + aggregate + decode + update + norm (one fused sweep kernel)
and the fixed-order final sums + next alpha (one small kernel behind it), through
a single library call.  Gradients, parameters and all state are resident in HBM
before the timed region; nothing is copied to the host inside it.  Prints ONE JSON
line.

  python bench.py [--gpus 1] [--steps K] [--warmup W]

With no --config the headline is the largest workload (5: d = 1.3e9, n = 8, randomized
rounding) and the line also carries `per_config`, one entry for each of the five
workloads.  With --config C only that workload runs (what the profiling commands use).
--copy-probe MiB runs a plain copy of known size instead (counter calibration).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E, published peak
# vector ALU: 256 compute units x 64 lanes x 2.4 GHz lane-instructions per second (one wavefront
# VALU instruction per CU and cycle); the chip sustains about 2.0 GHz under the randomized sweep
ALU_PEAK_LANE_OPS = 256 * 64 * 2.4e9
HEADLINE_CONFIG = 5
# State that the sweeps leave in the 256 MB memory-side cache from one step to the next (the
# library's policy: a state vector up to 192 MB whole, of a larger one the first 224 MB).
RESIDENT_BYTES = 192 << 20
KEEP_BYTES = 224 << 20
# default steps per timed region and workload (about 10-200 ms of GPU time each)
DEFAULT_STEPS = {1: 200, 2: 100, 3: 100, 4: 50, 5: 20}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="steps per timed region (0 = per workload)")
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--repeats", type=int, default=5,
                    help="timed regions per workload: the first is the reported one (with per-kernel "
                         "events), all of them give the median / min")
    ap.add_argument("--config", type=int, default=0,
                    help="workload 1..5 alone (0 = headline workload 5 plus per_config for all five)")
    ap.add_argument("--mode", default="fused", choices=["fused", "two_pass", "unfused"],
                    help="fused: one call; two_pass: F1, F2, a8; unfused: a1-a3, a4, a5-a6, a7, a8")
    ap.add_argument("--pool", type=int, default=0,
                    help="distinct gradient sets resident in HBM, cycled (0 = auto)")
    ap.add_argument("--tile", type=int, default=0)
    ap.add_argument("--grid", type=int, default=0)
    ap.add_argument("--wgs-per-cu", type=int, default=0)
    ap.add_argument("--two-phase", type=int, default=0, choices=[0, 1, 2],
                    help="form of the fused sweep: 0 automatic, 1 tile sweep, 2 two-phase sweep")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-threads", type=int, default=0,
                    help="threads of the all-cores oracle leg (0 = the box's CPU share)")
    ap.add_argument("--no-taps", action="store_true",
                    help="do not record per-kernel events (roofline numbers are then null)")
    ap.add_argument("--global-alpha", action="store_true", help="config 4 with one alpha")
    ap.add_argument("--rounding", default="config", choices=["config", "nearest", "stochastic"],
                    help="override the workload's rounding mode")
    ap.add_argument("--heuristic", action="store_true",
                    help="Heuristic IntSGD: a profiling pass (max |g|) sets alpha before every step")
    ap.add_argument("--diana", action="store_true",
                    help="IntDIANA step (Algorithm 3): n local shifts + a global shift in HBM")
    ap.add_argument("--momentum", action="store_true",
                    help="momentum 0.9 / weight decay 1e-4 form of the update (fused mode)")
    ap.add_argument("--row-skew", type=int, default=0, metavar="BYTES",
                    help="extra bytes (a multiple of 256) between the workers' gradient rows")
    ap.add_argument("--per-set", action="store_true",
                    help="also report the sweep kernel's mean time per resident gradient set")
    ap.add_argument("--no-placement", action="store_true",
                    help="leave every buffer wherever the allocator puts it instead of keeping "
                         "gradients and written state in different regions of one arena")
    ap.add_argument("--place", default="", metavar="FIELD=REGION,...",
                    help="move state fields (x, m, h, h_local, sum, q, x_old) to HBM region 0, 1 or 2 "
                         "of the arena (the gradient sets fill region 0, then 2)")
    ap.add_argument("--workers", type=int, default=0,
                    help="override the workload's worker count n (1 = the per-GPU shape of a real all-reduce)")
    ap.add_argument("--largest-sum", action="store_true",
                    help="also ask every step for the largest |S_j| per block (reported for the last step)")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MiB",
                    help="run five plain copies of this size and exit (calibrates FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


def host_threads():
    """Threads for the all-cores oracle leg: the CPUs this process may run on, at most 16
    (a one-GPU machine's share of its host)."""
    try:
        return max(1, min(16, len(os.sched_getaffinity(0))))
    except AttributeError:
        return max(1, min(16, os.cpu_count() or 1))


def cpu_baseline(w, rows, alpha_host, x_dev, *, threads, coords_per_thread, steps=1):
    """The oracle as it stands on a bounded sample of the same workload: `steps` consecutive
    steps on the leading `threads * coords_per_thread` coordinates (the whole vector when it is
    shorter), copied device -> host beforehand; reported in the metric's unit.  With
    threads > 1 the coordinate range is cut into that many slices and each thread calls the
    unchanged oracle on its slice (coordinates are independent, norms add)."""
    from concurrent.futures import ThreadPoolExecutor

    import numpy as np

    import oracle
    ln = min(w.d, max(4096, threads * coords_per_thread))
    off = None
    if w.block_offsets is not None:
        off = np.array(w.block_offsets, np.uint64)
    g = [r[:ln].cpu().numpy() for r in rows]
    x = x_dev[:ln].cpu().numpy()
    alpha = alpha_host
    r = np.zeros(w.num_blocks)
    threads = max(1, min(int(threads), ln // 4096))
    cuts = [(ln * i // threads) & ~3 for i in range(threads)] + [ln]

    def one_slice(i, k, xk, a):
        lo, hi = cuts[i], cuts[i + 1]
        return oracle.step([gi[lo:hi] for gi in g], a, xk[lo:hi], rounding=w.rounding, L=w.clip,
                           eta=w.eta, seed=w.philox_seed, step=k, j0=lo, offsets=off)

    pool = ThreadPoolExecutor(threads) if threads > 1 else None
    t0 = time.perf_counter()
    for k in range(1, steps + 1):
        if pool is None:
            outs = [one_slice(0, k, x, alpha)]
        else:
            outs = list(pool.map(lambda i: one_slice(i, k, x, alpha), range(threads)))
        x = outs[0]["x_new"] if threads == 1 else np.concatenate([o["x_new"] for o in outs])
        normsq = sum(o["normsq"] for o in outs)
        r, _, alpha, _ = oracle.next_alpha(normsq, r, d=w.d, n=w.n, beta=w.beta, eps=w.eps,
                                           eta=w.eta, offsets=off)
    dt = time.perf_counter() - t0
    if pool is not None:
        pool.shutdown()
    return {"value": 4.0 * w.n * ln * steps / dt / 1e9, "unit": "GB/s", "cores": threads,
            "kind": "oracle",
            "sample": "%d step(s) on the first %d of %d coordinates x %d workers, one chunk streamed "
                      "device -> host, %d slice(s) of %d coordinates (%.1f s)" % (
                          steps, ln, w.d, w.n, threads, ln // threads, dt)}


class HipEvents:
    """Raw HIP events from the runtime this process already has loaded (the library's
    launch options take hipEvent_t handles; the loop timer records on the launch stream)."""

    def __init__(self):
        import ctypes as C
        path = None
        with open("/proc/self/maps") as fh:
            for line in fh:
                if "libamdhip64" in line:
                    path = line.split()[-1]
                    break
        assert path, "HIP runtime not loaded"
        self.C = C
        self.hip = C.CDLL(path)
        self.hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.hip.hipEventDestroy.argtypes = [C.c_void_p]

    def create(self):
        ev = self.C.c_void_p()
        assert self.hip.hipEventCreate(self.C.byref(ev)) == 0
        return ev.value

    def record(self, ev, stream):
        rc = self.hip.hipEventRecord(ev, stream)
        assert rc == 0, "hipEventRecord -> %d" % rc

    def elapsed_ms(self, a, b):
        ms = self.C.c_float()
        rc = self.hip.hipEventElapsedTime(self.C.byref(ms), a, b)
        assert rc == 0, "hipEventElapsedTime -> %d" % rc
        return float(ms.value)

    def destroy(self, ev):
        self.hip.hipEventDestroy(ev)


def load_counters(name, form):
    """Committed rocprofv3 --pmc summary of the fused step's sweep kernel for this workload and
    form ("tile" or "two_phase"), from profiles/traffic.json: HBM bytes per launch and, where
    recorded, VALUBusy.  NOT measured in this run."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as fh:
            table = json.load(fh)
        return table.get("%s/%s" % (name, form), {})
    except (OSError, ValueError):
        return {}


def copy_probe(mib):
    import torch
    n = mib * 1024 * 1024 // 4
    src = torch.ones(n, dtype=torch.float32, device="cuda:0")
    dst = torch.empty_like(src)
    for _ in range(5):
        torch.mul(src, 1.0, out=dst)      # one elementwise kernel: reads n*4 B, writes n*4 B
    torch.cuda.synchronize()
    print(json.dumps({"copy_probe": {"launches": 5, "read_bytes_per_launch": n * 4,
                                     "write_bytes_per_launch": n * 4}}))


def device_state():
    """Clock and power mode as rocm-smi shows them (a child process; sampled right after the
    timed work, so sclk may already have dropped back), or None when the tool is not there."""
    import subprocess
    try:
        out = subprocess.run(["rocm-smi", "--showclocks", "--showperflevel", "--json"], timeout=20,
                             stdout=subprocess.PIPE, stderr=subprocess.DEVNULL).stdout.decode()
        card = json.loads(out[out.index("{"):])["card0"]
        return {"mclk": card.get("mclk clock speed:"), "sclk_after_run": card.get("sclk clock speed:"),
                "performance_level": card.get("Performance Level")}
    except Exception:        # noqa: BLE001 (reporting aid only)
        return None


def median(v):
    s = sorted(v)
    return s[len(s) // 2] if len(s) % 2 else 0.5 * (s[len(s) // 2 - 1] + s[len(s) // 2])


def run_workload(args, hip, cfg, *, cpu_legs, arena):
    """Times one workload; returns (top-level result dict, per_config entry)."""
    import torch

    import paper_2102_08374_amd as P
    from paper_2102_08374_amd import workloads as W
    from paper_2102_08374_amd.stepper import Stepper

    dev = "cuda:0"
    rounding = {"config": None, "nearest": 0, "stochastic": 1}[args.rounding]
    w = W.config(cfg, per_bucket=not args.global_alpha, rounding=rounding)
    if args.workers and args.workers != w.n:
        # the same recipe with another worker count; --workers 1 is the shape a GPU sees around a
        # real all-reduce (its own gradient only)
        import dataclasses
        w = dataclasses.replace(
            w, n=args.workers, name="%s-n%d" % (w.name, args.workers),
            clip=w.clip if w.wire == 8 else P.default_clip(args.workers),
            first_normsq=[v * w.n / args.workers for v in w.first_normsq])
    steps = args.steps or DEFAULT_STEPS[cfg]
    opts = P.LaunchOpts(args.tile, args.grid, args.wgs_per_cu, args.two_phase)
    desc = P.Desc(w.d, w.n, rounding=w.rounding, wire=w.wire, clip=w.clip, seed=w.philox_seed,
                  block_offsets=w.block_offsets, opts=opts)
    st = Stepper(desc, eta=w.eta, beta=w.beta, eps=w.eps, device=dev)
    largest = None
    if args.largest_sum:
        largest = torch.zeros(w.num_blocks, dtype=torch.int32, device=dev)
        desc.largest_sum = largest

    grad_bytes = 4 * w.n * w.d
    stride = W.row_stride(w.d, args.row_skew)
    set_bytes = 4 * w.n * stride
    settle_ms = 60.0
    stream = torch.cuda.current_stream().cuda_stream     # every library call below launches here

    # The written state of the step: x, the momentum buffer, IntDIANA's shifts, the integer
    # buffers of the unfused forms.
    fields = [("x", w.d, torch.float32)]
    if args.momentum:
        fields.append(("m", w.d, torch.float32))
    if args.diana:
        fields += [("h", w.d, torch.float32), ("h_local", w.n * stride, torch.float32)]
    if args.mode != "fused":
        fields.append(("sum", w.d, torch.int32))
    if args.mode == "unfused":
        fields += [("q", w.n * stride, torch.int8 if w.wire == 8 else torch.int32),
                   ("x_old", w.d, torch.float32)]
    if cpu_legs:
        fields.append(("x0", w.d, torch.float32))        # copy of x^0 for the CPU legs

    def nbytes(numel, dt):
        return numel * torch.empty(0, dtype=dt).element_size()

    # Placement in HBM (placement.py): the gradient sets, which the sweeps only read, fill
    # region 0 of the arena (then region 2); x goes into region 1, and a second written stream
    # (momentum buffer, local shifts) into a region other than x's: measured, two written
    # streams in one region cost 4-6 %, x in the gradients' region 3-6 %.  --place moves
    # single fields; --no-placement leaves it all to the allocator.
    # Resident gradient sets are cycled step by step so that nothing of a small set survives
    # in the 256 MB memory-side cache.
    default_region = {"x": 1, "m": 2, "h": 0, "h_local": 2, "sum": 1, "q": 2, "x_old": 2, "x0": 2}
    state_region = {name: default_region[name] for name, _, _ in fields}
    for item in (args.place.split(",") if args.place else []):
        name, region = item.split("=")
        assert name in state_region, "--place: no field %r in this mode" % name
        state_region[name] = int(region)
    want = args.pool or min(steps + args.warmup, 16)
    state, sets, set_regions = {}, [], []
    if arena is not None:
        arena.reset()
        for name, numel, dt in fields:      # the preferred region, or whichever has room
            need = nbytes(numel, dt)
            prefer = state_region[name]
            region = next((r for r in (prefer, *range(P.HBM_REGIONS)) if arena.free_in(r) >= need), None)
            assert region is not None, "the arena has no room for %s (%d bytes)" % (name, need)
            state_region[name] = region
            state[name] = arena.take(need, region).view(dt)
            state[name].zero_()
        for s_idx in range(want):
            region = next((r for r in (0, 2) if arena.free_in(r) >= set_bytes), None)
            if region is None and not sets:      # a small arena: anywhere rather than nowhere
                region = 1 if arena.free_in(1) >= set_bytes else None
            if region is None:
                break
            buf = arena.take(set_bytes, region).view(torch.float32).view(w.n, stride)
            sets.append(W.make_gradients(w, s_idx + 1, dev, out=buf, skew_bytes=args.row_skew))
            set_regions.append(region)
        assert sets, "the arena has no room for one gradient set"
    else:
        free_mem, _ = torch.cuda.mem_get_info()
        for name, numel, dt in fields:
            state[name] = torch.zeros(numel, dtype=dt, device=dev)
        for s_idx in range(max(1, min(want, int(0.45 * free_mem // set_bytes)))):
            sets.append(W.make_gradients(w, s_idx + 1, dev, skew_bytes=args.row_skew))
    pool = len(sets)

    def run_step(v, rows, k, tap=None):
        """One step on the written state `v` (views of an arena); `tap` = a pair of events to
        attach to the step's (first) sweep kernel."""
        x = v["x"]
        opts.set_events(None, None)
        if args.heuristic:
            nb = 7 if w.wire == 8 else 31
            P.intsgd_heuristic_alpha(desc, rows, nb, st.alpha, st.workspace)   # extra sweep
        if tap is not None:
            opts.set_events(*tap)
        desc.step = k
        if args.heuristic:
            st.step_fused(rows, x, k, chain_alpha=False)
        elif args.diana:
            hl = [v["h_local"][i * stride: i * stride + w.d] for i in range(w.n)]
            P.intsgd_diana_step(desc, rows, hl, st.alpha, st.eta, x, v["h"], st.r, st.beta,
                                st.eps, st.norm_sq, st.sat_count, st.workspace)
        elif args.momentum:
            st.step_momentum(rows, x, v["m"], k, 0.9, 1e-4)   # a1-a8 with the momentum update
        elif args.mode == "fused":
            st.step_fused(rows, x, k)                    # a1-a8, one call
        elif args.mode == "two_pass":                    # F1, F2, a8 (Stepper.step_two_pass)
            P.intsgd_compress_sum(desc, rows, st.alpha, v["sum"], st.sat_count, st.workspace)
            opts.set_events(None, None)
            P.intsgd_decode_update_norm(desc, v["sum"], st.alpha, st.eta, x, st.norm_sq, st.workspace)
            st.next_alpha()
        else:                                            # five calls + a copy of x (Stepper.step_unfused)
            q = [v["q"][i * stride: i * stride + w.d] for i in range(w.n)]
            P.intsgd_compress(desc, rows, st.alpha, q, st.sat_count, st.workspace)
            opts.set_events(None, None)
            P.intsgd_int_sum(desc, q, v["sum"])
            v["x_old"].copy_(x)
            P.intsgd_decode_update(desc, v["sum"], st.alpha, st.eta, x, None)
            P.intsgd_update_norm(desc, x, v["x_old"], st.norm_sq, st.workspace)
            st.next_alpha()

    # Evidence for the layout, taken at set-up (untimed): the same step with x moved into the
    # first gradient set's region.  Only for a plain fused step on a state the cache cannot hold.
    placement_check = None
    if (arena is not None and args.mode == "fused" and not (args.momentum or args.diana or args.heuristic)
            and 4 * w.d > (256 << 20) and state_region["x"] != set_regions[0]
            and arena.free_in(set_regions[0]) >= 4 * w.d):
        beside = dict(state)
        beside["x"] = arena.take(4 * w.d, set_regions[0]).view(torch.float32)
        beside["x"].zero_()
        st.start(w.first_normsq)
        e0, e1 = hip.create(), hip.create()
        placement_check = {}
        for label, v in (("x_apart_ms", state), ("x_beside_gradients_ms", beside),
                         ("x_apart_again_ms", state)):
            for _ in range(3):            # the cache-resident prefix of x has to settle first
                run_step(v, sets[0][1], 1)
            hip.record(e0, stream)
            for _ in range(3):
                run_step(v, sets[0][1], 1)
            hip.record(e1, stream)
            torch.cuda.synchronize()
            placement_check[label] = hip.elapsed_ms(e0, e1) / 3
        hip.destroy(e0)
        hip.destroy(e1)
        state["x"].zero_()
        del beside

    x = W.make_params(w, dev, out=state["x"])
    torch.cuda.synchronize()

    def one_step(k, tap=None):
        run_step(state, sets[(k - 1) % pool][1], k, tap)

    st.start(w.first_normsq)
    alpha0 = st.alpha.cpu().numpy().copy()
    x0 = state["x0"].copy_(x) if cpu_legs else None

    # Untimed: first enough steps for clocks and caches to settle after the set-up work (at
    # least settle_ms of them), then the W warm-up steps.
    k = 0
    t_settle = time.perf_counter()
    while (time.perf_counter() - t_settle) * 1e3 < settle_ms:
        for _ in range(4):
            k += 1
            one_step(k)
        torch.cuda.synchronize()
    settle_steps = k
    for _ in range(args.warmup):
        k += 1
        one_step(k)
    torch.cuda.synchronize()

    # Timed regions: exactly `steps` steps each, bracketed by a device synchronisation on both
    # sides (host clock) and by a pair of HIP events recorded on the launch stream.  In the
    # first region the library also attaches a pair of events to every sweep kernel's dispatch.
    taps = [] if args.no_taps else [(hip.create(), hip.create()) for _ in range(steps)]
    loop_ev = [(hip.create(), hip.create()) for _ in range(max(1, args.repeats))]
    host_ms, event_ms = [], []
    for rep, (e0, e1) in enumerate(loop_ev):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        hip.record(e0, stream)
        for i in range(steps):
            k += 1
            one_step(k, taps[i] if (rep == 0 and taps) else None)
        hip.record(e1, stream)
        torch.cuda.synchronize()
        host_ms.append((time.perf_counter() - t0) * 1e3 / steps)
        event_ms.append(hip.elapsed_ms(e0, e1) / steps)
    opts.set_events(None, None)

    per_set = None
    if taps and args.per_set:        # step k of the first region used set (settle + warmup + k) % pool
        raw = [hip.elapsed_ms(a, b) for a, b in taps]
        per_set = {}
        for i, ms in enumerate(raw):
            per_set.setdefault((settle_steps + args.warmup + i) % pool, []).append(ms)
        per_set = {str(s): sum(v) / len(v) for s, v in sorted(per_set.items())}
    kernel_ms = sorted(hip.elapsed_ms(a, b) for a, b in taps) if taps else None
    for a, b in taps + loop_ev:
        hip.destroy(a)
        hip.destroy(b)
    avg_kernel_ms = sum(kernel_ms) / len(kernel_ms) if kernel_ms else None
    per_coord = (4 * w.n + 8) if args.mode == "fused" else (4 * w.n + 4)
    state_vectors = 1
    if args.mode == "unfused":
        per_coord = (4 + w.wire // 8) * w.n
    if args.momentum:
        per_coord, state_vectors = 4 * w.n + 16, 2
    if args.diana:
        per_coord = 12 * w.n + 16
    algo_bytes = per_coord * w.d
    achieved = algo_bytes / (avg_kernel_ms * 1e-3) / 1e9 if kernel_ms else None
    form = P.intsgd_fused_step_form(desc)
    if args.diana:
        kernel_name = "k_diana<ROUND>: Algorithm 3 in one sweep"
    elif args.mode == "unfused":
        kernel_name = "k_compress<ROUND, WIRE>: a1-a3 for all n workers (first of the five calls)"
    elif args.mode != "fused":
        kernel_name = ("k_aggregate_phased<ROUND, sum only>" if form == 2
                       else "k_aggregate<ROUND, FUSED=false>") + ": a1-a4 (first of the two sweeps)"
    elif form == 2:
        kernel_name = "k_aggregate_phased<ROUND, MOMENTUM>: a1-a7, gradient reads then x update per round"
    else:
        kernel_name = "k_aggregate<ROUND, FUSED=true, MOMENTUM>: a1-a7 in one tile sweep"
    sat = int(st.sat_count.cpu().numpy().view("uint64").sum())
    alpha_last = float(st.alpha.cpu()[0])

    # Bytes of the fused sweep that the memory-side cache absorbs (the resident part of the
    # state is read and written there, not in DRAM): what is left is the DRAM-only figure.
    dram_only_frac = None
    if kernel_ms and args.mode == "fused" and not args.diana:
        state_bytes = 4 * w.d * state_vectors
        resident = state_bytes if state_bytes <= RESIDENT_BYTES else KEEP_BYTES
        dram_bytes = algo_bytes - 2 * resident
        dram_only_frac = dram_bytes / (avg_kernel_ms * 1e-3) / 1e9 / HBM_PEAK_GBS
    counters = {}
    if args.mode == "fused" and not (args.momentum or args.diana):
        counters = load_counters(w.name, "two_phase" if form == 2 else "tile")

    claim = cfg != 1        # workload 1 is 16 MB of gradients: cache-resident, launch-bound
    roofline = {
        "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": achieved / HBM_PEAK_GBS if kernel_ms else None,
        "traffic": counters.get("bytes_per_launch"),
        "traffic_source": "profiles/traffic.json: committed rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE "
                          "summary of this kernel and workload, not measured in this run",
        "dram_only_frac": dram_only_frac,
        "valu_busy": counters.get("valu_busy"),
        "alu_frac": (counters["valu_insts_per_launch"] * 64 / (avg_kernel_ms * 1e-3) / ALU_PEAK_LANE_OPS
                     if kernel_ms and counters.get("valu_insts_per_launch") else None),
        "alu_note": "vector lane-instructions per second (SQ_INSTS_VALU of the committed profile x 64 "
                    "/ this run's kernel time) against 256 CUs x 64 lanes x 2.4 GHz",
        "kernel": kernel_name,
        "algorithmic_bytes_per_launch": algo_bytes,
        "kernel_ms_avg": avg_kernel_ms, "kernel_ms_min": kernel_ms[0] if kernel_ms else None,
        "kernel_ms_median": median(kernel_ms) if kernel_ms else None,
        "claim": claim,
    }
    if per_set is not None:
        roofline["kernel_ms_per_gradient_set"] = per_set
    result = {
        "metric": "fp32 gradient GB/s per IntSGD step (n workers)",
        "value": grad_bytes / (host_ms[0] * 1e-3) / 1e9,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": args.warmup,
        "ms_per_step": host_ms[0],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": w.name, "d": w.d, "n_workers": w.n, "blocks": w.num_blocks,
            "rounding": "stochastic" if w.rounding else "nearest-even", "wire": "int%d" % w.wire,
            "clip": w.clip, "grad_dist": w.grad_kind,
            "mode": "heuristic-alpha+fused" if args.heuristic else "diana" if args.diana else args.mode + ("+momentum" if args.momentum else ""),
            "gradient_sets": pool,
            "untimed_settling_steps_before_warmup": settle_steps,
            "launch_options": {"tile_coords": args.tile, "max_workgroups": args.grid,
                               "workgroups_per_cu": args.wgs_per_cu, "two_phase": args.two_phase},
            "alpha_last": alpha_last,
            "clipped_last_step": sat,
            "largest_sum_last_step": (int(largest.cpu().numpy().view("uint32").max())
                                      if largest is not None else None),
            "placement": ("allocator's choice" if arena is None else
                          {"rule": "one arena over the free device memory, read as three regions of "
                                   "a third of the HBM each: gradient sets (only read) in one region, "
                                   "written state in another",
                           "check_at_setup": placement_check,
                           "gradient_set_regions": set_regions,
                           "state_regions": {k: v for k, v in state_region.items() if k != "x0"}}),
        },
        "timing": {
            "regions": len(loop_ev), "steps_per_region": steps,
            "clock": "HIP events on the launch stream around each region; ms per step",
            "ms_per_step_median": median(event_ms), "ms_per_step_min": min(event_ms),
            "ms_per_step_host_clock_first_region": host_ms[0],
        },
        "roofline": roofline,
    }
    if cpu_legs:
        one = cpu_baseline(w, sets[0][1], alpha0, x0, threads=1,
                           coords_per_thread=cpu_legs["one_core_wc"] // w.n)
        result["cpu_baseline"] = one
        if cpu_legs.get("all_cores_wc_per_thread"):
            th = args.cpu_threads or host_threads()
            result["cpu_baseline_all_cores"] = cpu_baseline(
                w, sets[0][1], alpha0, x0, threads=th,
                coords_per_thread=cpu_legs["all_cores_wc_per_thread"] // w.n)
    entry = {
        "workload": w.name, "d": w.d, "n_workers": w.n,
        "rounding": "stochastic" if w.rounding else "nearest-even",
        "steps_per_region": steps, "regions": len(loop_ev),
        "ms_per_step_median": median(event_ms), "ms_per_step_min": min(event_ms),
        "gradient_gbs": grad_bytes / (median(event_ms) * 1e-3) / 1e9,
        "kernel": kernel_name.split(":")[0], "kernel_ms": avg_kernel_ms,
        "algorithmic_bytes": algo_bytes,
        "frac": roofline["frac"] if claim else None,
        "dram_only_frac": dram_only_frac if claim else None,
        "valu_busy": counters.get("valu_busy"),
        "alu_frac": roofline["alu_frac"] if claim else None,
        "note": None if claim else "no roofline claim: 16 MB of gradients, cache-resident and launch-bound",
    }
    if "cpu_baseline" in result:
        entry["cpu_baseline_gbs_1_core"] = result["cpu_baseline"]["value"]
    del sets, x, st, state
    torch.cuda.empty_cache()
    return result, entry


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (the n workers are "
              "n gradient buffers in one HBM); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.copy_probe:
        copy_probe(args.copy_probe)
        return
    torch.zeros(1, device="cuda:0")          # loads the HIP runtime before HipEvents looks for it
    hip = HipEvents()
    widened = args.heuristic or args.diana or args.momentum
    cpu = not args.no_cpu_baseline and not widened
    # CPU legs: about 10 s of single-core oracle work; the all-cores leg gives every thread a quarter of it
    big_legs = {"one_core_wc": 1 << 29, "all_cores_wc_per_thread": 1 << 27}
    import paper_2102_08374_amd as P
    arena = None if args.no_placement else P.Arena("cuda:0", keep_free=8 << 30)
    if args.config:
        result, _ = run_workload(args, hip, args.config, cpu_legs=big_legs if cpu else None, arena=arena)
        result["device"] = device_state()
        print(json.dumps(result))
        return
    result, head_entry = run_workload(args, hip, HEADLINE_CONFIG, cpu_legs=big_legs if cpu else None,
                                      arena=arena)
    per_config = []
    for cfg in (1, 2, 3, 4):
        _, entry = run_workload(args, hip, cfg, cpu_legs={"one_core_wc": 1 << 26} if cpu else None,
                                arena=arena)
        per_config.append(entry)
    per_config.append(head_entry)
    result["per_config"] = per_config
    result["device"] = device_state()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
