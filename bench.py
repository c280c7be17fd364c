#!/usr/bin/env python3
"""Benchmark of the IntSGD compression hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic gradients:
scale + round + clip + aggregate + decode + update + norm (one fused sweep kernel)
and the fixed-order final sums + next alpha (one small kernel behind it), through
a single library call.  Gradients, parameters and all state are resident in HBM
before the timed region; nothing is copied to the host inside it.  Prints ONE JSON
line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--mode fused]
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


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2, help="workload 1..5 (2 = headline)")
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
    ap.add_argument("--cpu-threads", type=int, default=1,
                    help="threads for the oracle baseline (each runs the unchanged oracle on a slice)")
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
    return ap.parse_args()


def cpu_baseline(w, rows, alpha_host, x_host, max_wc=420_000_000, steps=6, threads=1):
    """The oracle as it stands on a bounded sample of the same workload: `steps`
    consecutive steps on the leading slice of at most max_wc worker-coordinates (the whole
    vector when it is small enough); reported in the metric's unit.  One thread by default;
    with threads > 1 the coordinate range is cut into that many slices and each thread
    calls the unchanged oracle on its slice (coordinates are independent, norms add)."""
    from concurrent.futures import ThreadPoolExecutor

    import numpy as np

    import oracle
    ln = min(w.d, max(4096, max_wc // w.n))
    off = None
    if w.block_offsets is not None:
        off = np.array(w.block_offsets, np.uint64)
    g = [r[:ln].cpu().numpy() for r in rows]
    x = x_host[:ln].copy()
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
            "sample": "%d steps on the first %d of %d coordinates x %d workers (%.1f s)" % (
                steps, ln, w.d, w.n, dt)}


class HipEvents:
    """Raw HIP events from the runtime this process already has loaded (the library's
    profiling taps take hipEvent_t handles)."""

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
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.hip.hipEventDestroy.argtypes = [C.c_void_p]

    def create(self):
        ev = self.C.c_void_p()
        assert self.hip.hipEventCreate(self.C.byref(ev)) == 0
        return ev.value

    def elapsed_ms(self, a, b):
        ms = self.C.c_float()
        rc = self.hip.hipEventElapsedTime(self.C.byref(ms), a, b)
        assert rc == 0, "hipEventElapsedTime -> %d" % rc
        return float(ms.value)

    def destroy(self, ev):
        self.hip.hipEventDestroy(ev)


def load_traffic(name, form):
    """HBM bytes per launch of the dominant kernel (fused step, `form` = "tile" or
    "two_phase") from committed rocprofv3 counter summaries (profiles/traffic.json), or None."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as fh:
            table = json.load(fh)
        return table.get("%s/%s" % (name, form), {}).get("bytes_per_launch")
    except (OSError, ValueError):
        return None


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (the n workers are "
              "n gradient buffers in one HBM); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2102_08374_amd as P
    from paper_2102_08374_amd import workloads as W
    from paper_2102_08374_amd.stepper import Stepper

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    rounding = {"config": None, "nearest": 0, "stochastic": 1}[args.rounding]
    w = W.config(args.config, per_bucket=not args.global_alpha, rounding=rounding)
    P.intsgd_set_tuning(args.tile, args.grid, args.wgs_per_cu, args.two_phase)
    tile, grid, wgs_per_cu, two_phase = P.intsgd_get_tuning()

    desc = P.Desc(w.d, w.n, rounding=w.rounding, wire=w.wire, clip=w.clip, seed=w.philox_seed,
                  block_offsets=w.block_offsets)
    st = Stepper(desc, eta=w.eta, beta=w.beta, eps=w.eps, device=dev)
    x = W.make_params(w, dev)

    grad_bytes = 4 * w.n * w.d
    free, _ = torch.cuda.mem_get_info()
    pool = args.pool or max(1, min(args.steps + args.warmup, 16, int(0.6 * free // grad_bytes)))
    sets = []
    for s in range(pool):
        buf, rows = W.make_gradients(w, s + 1, dev)
        sets.append((buf, rows))
    sum_buf = torch.empty(w.d, dtype=torch.int32, device=dev) if args.mode != "fused" else None
    q_bufs = x_old_buf = None
    if args.mode == "unfused":
        qdt = torch.int8 if w.wire == 8 else torch.int32
        qbuf = torch.empty((w.n, W.row_stride(w.d)), dtype=qdt, device=dev)
        q_bufs = [qbuf[i, :w.d] for i in range(w.n)]
        x_old_buf = torch.empty_like(x)
    mom = torch.zeros_like(x) if args.momentum else None
    if args.diana:
        hbuf = torch.zeros((w.n, W.row_stride(w.d)), dtype=torch.float32, device=dev)
        h_local = [hbuf[i, :w.d] for i in range(w.n)]
        h_global = torch.zeros_like(x)
    torch.cuda.synchronize()

    def one_step(k, tap=None):
        rows = sets[(k - 1) % pool][1]
        if args.heuristic:
            nb = 7 if w.wire == 8 else 31
            P.intsgd_heuristic_alpha(desc, rows, nb, st.alpha, st.workspace)   # extra sweep
        if tap is not None:
            P.intsgd_tap_next_launch(tap[0], tap[1])     # events right around the next sweep
        if args.heuristic:
            st.step_fused(rows, x, k, chain_alpha=False)
        elif args.diana:
            desc.step = k
            P.intsgd_diana_step(desc, rows, h_local, st.alpha, st.eta, x, h_global, st.r, st.beta,
                                st.eps, st.norm_sq, st.sat_count, st.workspace)
        elif args.momentum:
            st.step_momentum(rows, x, mom, k, 0.9, 1e-4)  # a1-a8 with the momentum update
        elif args.mode == "fused":
            st.step_fused(rows, x, k)                    # a1-a8, one call
        elif args.mode == "two_pass":
            st.step_two_pass(rows, x, k, sum_buf)        # F1, F2, a8
        else:
            st.step_unfused(rows, x, k, q_bufs, sum_buf, x_old_buf)   # five calls + a copy of x

    st.start(w.first_normsq)
    alpha0 = st.alpha.cpu().numpy().copy()
    x0 = None if args.no_cpu_baseline else x.cpu().numpy().copy()

    for k in range(1, args.warmup + 1):
        one_step(k)
    torch.cuda.synchronize()

    # timed region: exactly K steps.  In every step the library records a pair of HIP
    # events right around the sweep kernel, on the stream it launches it on.
    hip = HipEvents()
    ev = [(hip.create(), hip.create()) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        one_step(args.warmup + 1 + i, None if args.no_taps else ev[i])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    kernel_ms = sorted(hip.elapsed_ms(a, b) for a, b in ev) if not args.no_taps else None
    for a, b in ev:
        hip.destroy(a)
        hip.destroy(b)
    avg_kernel_ms = sum(kernel_ms) / len(kernel_ms) if kernel_ms else None
    per_coord = (4 * w.n + 8) if args.mode == "fused" else (4 * w.n + 4)
    if args.mode == "unfused":
        per_coord = (4 + w.wire // 8) * w.n
    if args.momentum:
        per_coord = 4 * w.n + 16
    if args.diana:
        per_coord = 12 * w.n + 16
    algo_bytes = per_coord * w.d
    achieved = algo_bytes / (avg_kernel_ms * 1e-3) / 1e9 if kernel_ms else None
    if args.diana:
        kernel_name = "k_diana<ROUND>: Algorithm 3 in one sweep"
    elif args.mode == "unfused":
        kernel_name = "k_compress<ROUND, WIRE>: a1-a3 for all n workers (first of the five calls)"
    elif args.mode != "fused":
        kernel_name = ("k_aggregate_phased<ROUND, sum only>" if P.intsgd_fused_step_form(desc) == 2
                       else "k_aggregate<ROUND, FUSED=false>") + ": a1-a4 (first of the two sweeps)"
    elif P.intsgd_fused_step_form(desc) == 2:
        kernel_name = "k_aggregate_phased<ROUND, MOMENTUM>: a1-a7, gradient reads then x update per round"
    else:
        kernel_name = "k_aggregate<ROUND, FUSED=true, MOMENTUM>: a1-a7 in one tile sweep"
    sat = int(st.sat_count.cpu().numpy().view("uint64").sum())
    alpha_last = float(st.alpha.cpu()[0])

    result = {
        "metric": "fp32 gradient GB/s per IntSGD step (n workers)",
        "value": grad_bytes * args.steps / dt / 1e9,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": dt * 1e3 / args.steps,
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
            "tuning_overrides": {"tile_coords": tile, "max_workgroups": grid,
                                 "workgroups_per_cu": wgs_per_cu, "two_phase": two_phase},
            "alpha_last": alpha_last,
            "clipped_last_step": sat,
        },
        "roofline": {
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS if kernel_ms else None,
            "traffic": None if (args.momentum or args.diana or args.mode != "fused")
                       else load_traffic(w.name, "two_phase" if P.intsgd_fused_step_form(desc) == 2 else "tile"),
            "kernel": kernel_name,
            "algorithmic_bytes_per_launch": algo_bytes,
            "kernel_ms_avg": avg_kernel_ms, "kernel_ms_min": kernel_ms[0] if kernel_ms else None,
            "kernel_ms_median": kernel_ms[len(kernel_ms) // 2] if kernel_ms else None,
        },
    }
    if not args.no_cpu_baseline and not args.momentum and not args.diana:
        result["cpu_baseline"] = cpu_baseline(w, sets[0][1], alpha0, x0, threads=args.cpu_threads)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
